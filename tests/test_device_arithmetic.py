"""Host-side models of two pieces of integer / lane arithmetic the sparse engine relies on (no GPU needed).

They restate what the kernels do in numpy and check it exhaustively, so that a change of a constant
(items per thread, words per slot, the number of sums joined at once) that breaks the arithmetic fails here.
"""
import numpy as np


def test_item_to_member_by_float_product_is_exact():
    # the exchange maps item -> (member, word) with floor((item + 0.5) * (1 / per)) in f32 instead of an
    # integer division: exact for every slot width the engine can have (1..18 words) and every item a thread
    # can own (6 items x 512 threads)
    for per in range(1, 19):
        r = np.float32(1.0) / np.float32(per)
        idx = np.arange(0, 6 * 512, dtype=np.int32)
        mem = ((idx.astype(np.float32) + np.float32(0.5)) * r).astype(np.int32)
        assert np.array_equal(mem, idx // per), per


def test_halving_butterfly_leaves_sum_i_in_lane_pair_i():
    # 32 sums over the 64 lanes of a wave: at distance 32, 16, 8, 4, 2 a lane keeps one half of its values
    # and adds the partner's copy of that half; after the last step lanes 2i and 2i+1 together hold sum i
    rng = np.random.default_rng(0)
    vals = rng.integers(-1000, 1000, size=(64, 32)).astype(np.float64)  # [lane][value]
    vv = vals.copy()
    h = 16
    while h >= 1:
        d = 2 * h
        new = vv.copy()
        for lane in range(64):
            upper = (lane & d) != 0
            partner = lane ^ d
            for i in range(h):
                sent = vv[partner][i] if (partner & d) else vv[partner][i + h]
                keep = vv[lane][i + h] if upper else vv[lane][i]
                new[lane][i] = keep + sent
        vv = new
        h //= 2
    total = vals.sum(axis=0)
    for lane in range(64):
        assert vv[lane][0] + vv[lane ^ 1][0] == total[lane >> 1]


def test_stream_engine_geometry_stays_inside_what_the_kernel_assumes():
    """Host model of the persistent streaming kernel's index arithmetic: for every shape the engine accepts, each
    workgroup owns at least one row, the slices of the first exchange cover all columns in whole bytes of sign
    bits (whole rows of the contracted array for order 3), slots and LDS hold what is indexed, and a thread never
    has more words to gather than its registers are declared for."""
    import torch

    from paper_2410_01799_amd import scd

    scd.lib()
    threads, max_slice, slot2, max_items2, max_lds = 512, 256, 16, 6, 160 * 1024 - 512
    shapes = [(256, 256), (100, 76), (8, 8), (77, 1024), (1000, 4096), (2052, 516), (1030, 520), (130, 8200), (16, 64),
              (8, 4), (4096, 4096), (700, 16384), (512, 512), (14336, 4096), (4096, 14336), (32000, 4096), (1, 4), (3, 64),
              (65, 130), (300, 8192), (2048, 2048), (4000, 3000, 3), (40, 30, 3), (130, 64, 4), (300, 200, 3), (50, 40, 2),
              (64, 33, 1), (9, 8, 7), (20, 30, 5)]
    seen = 0
    for dtype, es, ve in ((torch.float32, 4, 4), (torch.float64, 8, 2)):
        for dims in shapes:
            for limit in (256, 85, 64, 16):
                geo = scd.scd_stream_geometry(dtype, dims, limit)
                m = dims[0]
                n = dims[1] if len(dims) == 2 else dims[1] * dims[2]
                n3 = dims[2] if len(dims) == 3 else 0
                if geo is None:
                    continue
                seen += 1
                G, rpw, cs, lds_rows = geo["grid"], geo["rpw"], geo["cs"], geo["lds_rows"]
                assert 1 <= G <= min(limit, 256) and rpw >= 1
                assert (G - 1) * rpw < m <= G * rpw, (dims, limit)         # the last workgroup has a row, all rows are owned
                assert n % ve == 0 and (n // ve + threads - 1) // threads <= 8   # chunks per thread the kernel is built for
                assert cs % 8 == 0 and 8 <= cs <= max_slice and G * cs >= n      # slices cover the columns
                assert threads // cs >= 1
                unit = n3 if n3 else 1
                assert n3 <= 4 and cs % (8 * unit) == 0                          # whole bytes of sign bits per slice
                tw = (cs // unit + 31) // 32
                per = tw + (2 * n3 if n3 else 2) + 2
                assert per <= slot2 and (G * per + threads - 1) // threads <= max_items2
                nw, w2 = (n + 63) // 64, ((dims[1] + 63) // 64 if n3 else 0)
                bits = dims[1] if n3 else n
                assert G * (cs // unit // 8) >= (bits + 7) // 8            # the slices' sign bytes cover the whole vector
                assert 0 <= lds_rows <= rpw
                need = -(-lds_rows * n * es // 16) * 16 + -(-n * es // 16) * 16 + 2 * nw * 8 + w2 * 8 + 2 * (-(-rpw // 16) * 16)
                assert need < geo["lds_bytes"] <= max_lds + 64, (dims, limit)
                assert geo["xp_bytes"] == 2 * G * n * (1 if es == 4 else 2) * 8 and geo["xq_bytes"] == 2 * G * slot2 * 8
    assert seen > 60
    # shapes it must refuse: rows that are no multiple of 16 bytes or longer than 64 KB, too few workgroups for the
    # slices, orders above 3, a last mode above 4
    for dims in [(100, 77), (64, 16388), (64, 20000), (3, 4096), (9, 8, 7, 6), (20, 30, 5)]:
        assert scd.scd_stream_geometry(torch.float32, dims, 256) is None, dims


def test_column_signs_of_a_tensor_built_32_bits_per_thread():
    # Host model of ps_kron_bits (scd_stream.hip): the sign of column q of the n_1 x (n_2 n_3) view is
    # s2[q / n3] xor s3[q % n3]; a thread forms 32 consecutive bits from a 64-bit window of s2 that starts at row
    # q0 / n3, with the division by a float32 product.  Checked against the definition for all last modes, ragged
    # lengths and the padding; the float division exhaustively on the whole range the engine admits.
    f32 = np.float32
    M64 = (1 << 64) - 1
    for n3 in (1, 2, 3, 4):
        q = np.arange(0, (1 << 20) + 64, dtype=np.int64)
        j = ((q.astype(f32) + f32(0.5)) * (f32(1.0) / f32(n3))).astype(np.int64)
        assert np.array_equal(j, q // n3)
    rs = np.random.default_rng(5)
    for n3 in (1, 2, 3, 4):
        for n2 in (1, 5, 63, 64, 65, 700, 3000):
            n = n2 * n3
            s2 = rs.integers(0, 2, n2).astype(np.uint8)
            s3 = rs.integers(0, 2, n3).astype(np.uint8)
            w2 = (n2 + 63) // 64
            words = [0] * w2                                              # packed, LSB first, padding zero
            for i in np.nonzero(s2)[0]:
                words[i >> 6] |= 1 << (int(i) & 63)
            s3w = int(sum(int(b) << i for i, b in enumerate(s3)))
            nw = (n + 63) // 64
            out = []
            for h in range(2 * nw):
                q0 = 32 * h
                jx = int((f32(q0) + f32(0.5)) * (f32(1.0) / f32(n3)))
                cc, jj, wi, sh = q0 - jx * n3, 0, jx >> 6, jx & 63
                lo, hi = words[min(wi, w2 - 1)], words[min(wi + 1, w2 - 1)]
                x = ((lo >> sh) | (hi << (64 - sh))) & M64 if sh else lo
                o = 0
                for b in range(32):
                    o |= (((x >> jj) ^ (s3w >> cc)) & 1) << b
                    cc += 1
                    if cc == n3:
                        cc, jj = 0, jj + 1
                assert jj <= 33
                valid = n - q0
                out.append(o if valid >= 32 else (o & ((1 << valid) - 1) if valid > 0 else 0))
            bits = np.array([(out[q >> 5] >> (q & 31)) & 1 for q in range(64 * nw)], dtype=np.uint8)
            want = np.bitwise_xor.outer(s2, s3).reshape(-1)               # q = j * n3 + c
            assert np.array_equal(bits[:n], want), (n3, n2)
            assert not bits[n:].any()
