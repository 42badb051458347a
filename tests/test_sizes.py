"""Width / footprint arithmetic against the values printed in the paper (no GPU needed)."""
from fractions import Fraction
from pathlib import Path

import numpy as np
import pytest

from paper_2410_01799_amd import workloads as W

GOLD = Path(__file__).parent / "golden"


def table2():
    rows = []
    for line in (GOLD / "table2_widths.txt").read_text().splitlines():
        if line.startswith("#") or not line.strip():
            continue
        rows.append([int(x) for x in line.split()])
    return rows


def scalars():
    out = {}
    for line in (GOLD / "printed_values.txt").read_text().splitlines():
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = float(line[1])
    return out


def test_table2_widths():
    rates = [Fraction(8, 16), Fraction(7, 16), Fraction(6, 16), Fraction(5, 16), Fraction(4, 16)]
    for m, n, _count, *ws in table2():
        assert [W.width_for_compression(m, n, p) for p in rates] == ws
        for p, w in zip(rates, ws):
            assert W.compression_rate(w, m, n) <= float(p) < W.compression_rate(w + 1, m, n)


def test_total_terms_at_half():
    total = sum(count * ws[0] for _m, _n, count, *ws in table2())
    assert total == int(scalars()["total_terms_at_half"])
    man = W.config5_manifest()
    assert len(man) == 226
    assert sum(e["widths"]["1/2"] for e in man) == total


def test_fig3_sizes():
    g = scalars()
    dims = (4000, 3000, 3)
    assert 4000 * 3000 * 3 / 2 ** 20 == pytest.approx(g["fig3_raw_mib"], abs=0.005)
    # the printed sizes correspond to shared s,t plus three f32 scalars per term, widths 8..256/2
    per_term_bits = 4000 + 3000 + 3 * 32
    assert 8 * per_term_bits / 8 / 1024 == pytest.approx(g["fig3_smallest_kib"], abs=0.005)
    assert 128 * per_term_bits / 8 / 1024 == pytest.approx(g["fig3_largest_kib"], abs=0.005)
    # the all-signs variant at width 129 (one f32 per term) has about the same footprint
    assert W.packed_bits(129, dims) / 8 / 1024 == pytest.approx(110.8, abs=0.05)


def test_config_widths():
    assert W.compression_rate(8192, 4096, 4096) == pytest.approx(0.251, abs=1e-3)
    names = [(n, w) for n, _a, w, _s in ((n, None, W.width_for_compression(m, k, Fraction(1, 2)), 0)
                                         for n, m, k in W.LAYER_SHAPES)]
    assert dict(names) == dict(q_proj=16320, k_proj=6512, v_proj=6512, o_proj=16320, gate_proj=25442,
                               up_proj=25442, down_proj=25442)


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.005859375, 1.01171875, -3.140625, 0.0], dtype=np.float32)
    r = W.round_to_bf16(x)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-9 rounds up
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == np.float32(1.0078125)
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)
    # against the library's cast on random values
    import torch

    y = np.random.default_rng(3).standard_normal(10000).astype(np.float32)
    np.testing.assert_array_equal(W.round_to_bf16(y), torch.from_numpy(y).to(torch.bfloat16).to(torch.float32).numpy())


def test_weight_like_recipe():
    A = W.weight_like_matrix(256, 512, 300)
    assert A.dtype == np.float32 and A.shape == (256, 512)
    assert np.all((A.view(np.uint32) & 0xFFFF) == 0)          # bf16-representable
    col = np.sqrt((A.astype(np.float64) ** 2).mean(axis=0))
    assert (col > 4 * np.median(col)).sum() == 5              # 1 % of 512 columns scaled x8
    body = A.astype(np.float64)[:, col <= 4 * np.median(col)]
    # noise carries 0.9 of the energy, the rank-16 part 0.1: mean square = sigma^2 / 0.9
    assert (body ** 2).mean() == pytest.approx(0.02 ** 2 / 0.9, rel=0.05)
    sv = np.linalg.svd(body, compute_uv=False)
    noise_top = 0.02 * (np.sqrt(256) + np.sqrt(507))
    assert sv[0] > 1.2 * noise_top and sv[40] < 1.05 * noise_top   # a low-rank part stands out
