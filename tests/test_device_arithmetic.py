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
