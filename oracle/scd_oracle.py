"""ctypes front end of the plain f64 CPU oracle (``scd_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the benchmark's
CPU-baseline leg.  The GPU package never imports this module.

Every function takes and returns numpy arrays; sign vectors are ``uint64`` bitsets in which a
1 bit stands for -1 (Section 3.1 of the paper), element ``64p+q`` in bit ``q`` of word ``p``.
"""
from __future__ import annotations

import ctypes as C
import math
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "scd_oracle.c"
_LIB = _HERE / "libscd_oracle.so"
_lib = None

_f64p = np.ctypeslib.ndpointer(dtype=np.float64, flags="C_CONTIGUOUS")
_u64p = np.ctypeslib.ndpointer(dtype=np.uint64, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(dtype=np.int32, flags="C_CONTIGUOUS")
_i64p = np.ctypeslib.ndpointer(dtype=np.int64, flags="C_CONTIGUOUS")


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (-O2, OpenMP).  Rebuilds when the source is newer."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        cmd = ["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-std=c11", "-shared",
               "-fPIC", "-o", str(_LIB), str(_SRC), "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    L = C.CDLL(str(_LIB))
    vp = C.c_void_p
    L.scdo_set_threads.argtypes = [C.c_int]
    L.scdo_get_threads.restype = C.c_int
    L.scdo_rng_word.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint64]
    L.scdo_rng_word.restype = C.c_uint64
    L.scdo_rng_signs.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_int64, _u64p]
    L.scdo_pack.argtypes = [_f64p, C.c_int64, _u64p]
    L.scdo_unpack.argtypes = [_u64p, C.c_int64, _f64p]
    L.scdo_row_signed_sum.argtypes = [_f64p, C.c_int64, C.c_int64, _u64p, _f64p]
    L.scdo_col_signed_sum.argtypes = [_f64p, C.c_int64, C.c_int64, _u64p, _f64p]
    L.scdo_fro2.argtypes = [_f64p, C.c_int64, C.c_int64]
    L.scdo_fro2.restype = C.c_double
    L.scdo_rank1_update.argtypes = [_f64p, C.c_int64, C.c_int64, C.c_double, _u64p, _u64p]
    L.scdo_greedy_signed_cut.argtypes = [_f64p, C.c_int64, C.c_int64, _u64p, _u64p,
                                         C.POINTER(C.c_double), C.c_int32, C.POINTER(C.c_int32), vp, vp]
    L.scdo_greedy_signed_cut.restype = C.c_int
    L.scdo_decompose.argtypes = [_f64p, C.c_int64, C.c_int64, C.c_int64, C.c_uint64, C.c_int32,
                                 _u64p, _u64p, _f64p, _f64p, vp, vp, vp]
    L.scdo_decompose.restype = C.c_int
    L.scdo_mode_signed_sum.argtypes = [_f64p, C.c_int, _i64p, C.POINTER(vp), C.c_int, _f64p]
    L.scdo_tensor_inner.argtypes = [_f64p, C.c_int, _i64p, C.POINTER(vp)]
    L.scdo_tensor_inner.restype = C.c_double
    L.scdo_tensor_update.argtypes = [_f64p, C.c_int, _i64p, C.c_double, C.POINTER(vp)]
    L.scdo_axial_greedy_cut.argtypes = [_f64p, C.c_int, _i64p, C.POINTER(vp), C.POINTER(C.c_double),
                                        C.c_int32, C.POINTER(C.c_int32), vp, vp]
    L.scdo_axial_greedy_cut.restype = C.c_int
    L.scdo_tensor_decompose.argtypes = [_f64p, C.c_int, _i64p, C.c_int64, C.c_uint64, C.c_int32,
                                        C.POINTER(vp), _f64p, _f64p, vp, vp, vp]
    L.scdo_tensor_decompose.restype = C.c_int
    L.scdo_expand.argtypes = [C.c_int, _i64p, C.c_int64, C.POINTER(vp), _f64p, _f64p]
    L.scdo_lsq_coefficients.argtypes = [_f64p, C.c_int64, C.c_int64, C.c_int64, _u64p, _u64p, _f64p]
    L.scdo_lsq_coefficients.restype = C.c_int
    L.scdo_lsq_decompose.argtypes = [_f64p, C.c_int64, C.c_int64, C.c_int64, C.c_uint64, C.c_int32, _u64p, _u64p,
                                     _f64p, _f64p, C.c_void_p, C.c_void_p]
    L.scdo_lsq_decompose.restype = C.c_int
    L.scdo_tensor_lsq_coefficients.argtypes = [_f64p, C.c_int, _i64p, C.c_int64, C.POINTER(vp), _f64p]
    L.scdo_tensor_lsq_coefficients.restype = C.c_int
    L.scdo_tensor_lsq_decompose.argtypes = [_f64p, C.c_int, _i64p, C.c_int64, C.c_uint64, C.c_int32, C.POINTER(vp), _f64p,
                                            _f64p, C.c_void_p, C.c_void_p]
    L.scdo_tensor_lsq_decompose.restype = C.c_int
    L.scdo_scalars_decompose.argtypes = [_f64p, C.c_int, _i64p, C.c_int64, C.c_uint64, C.c_int32, C.POINTER(vp), _f64p, _f64p,
                                         C.c_void_p, C.c_void_p]
    L.scdo_scalars_decompose.restype = C.c_int
    L.scdo_apply.argtypes = [C.c_int64, C.c_int64, C.c_int64, _u64p, _u64p, _f64p, C.c_int, _f64p, _f64p]
    L.scdo_bruteforce_signed_cut_norm.argtypes = [_f64p, C.c_int64, C.c_int64, C.POINTER(C.c_uint64)]
    L.scdo_bruteforce_signed_cut_norm.restype = C.c_double
    _lib = L
    return L


DEFAULT_MAX_ITERS = 4096


def words(n: int) -> int:
    return (int(n) + 63) // 64


def set_threads(n: int) -> None:
    _load().scdo_set_threads(int(n))


def get_threads() -> int:
    return int(_load().scdo_get_threads())


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _u64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.uint64)


def _ptrs(arrs):
    arr = (C.c_void_p * len(arrs))()
    for i, a in enumerate(arrs):
        arr[i] = a.ctypes.data
    return arr


def _opt(a):
    return None if a is None else a.ctypes.data


def rng_word(seed: int, term: int, mode: int, word: int) -> int:
    return int(_load().scdo_rng_word(seed, term, mode, word))


def rng_signs(seed: int, term: int, mode: int, n: int) -> np.ndarray:
    """Uniform random sign bitset of length n for (seed, term, mode); padding bits are 0."""
    out = np.zeros(words(n), dtype=np.uint64)
    _load().scdo_rng_signs(seed, term, mode, n, out)
    return out


def pack(x) -> np.ndarray:
    x = _f64(x).ravel()
    out = np.zeros(words(x.size), dtype=np.uint64)
    _load().scdo_pack(x, x.size, out)
    return out


def unpack(bits, n: int) -> np.ndarray:
    out = np.empty(int(n), dtype=np.float64)
    _load().scdo_unpack(_u64(bits), int(n), out)
    return out


def row_signed_sum(R, tbits) -> np.ndarray:
    """u = R t."""
    R = _f64(R)
    m, n = R.shape
    u = np.empty(m, dtype=np.float64)
    _load().scdo_row_signed_sum(R, m, n, _u64(tbits), u)
    return u


def col_signed_sum(R, sbits) -> np.ndarray:
    """v = R^T s."""
    R = _f64(R)
    m, n = R.shape
    v = np.empty(n, dtype=np.float64)
    _load().scdo_col_signed_sum(R, m, n, _u64(sbits), v)
    return v


def fro2(R) -> float:
    R = _f64(R)
    R2 = R.reshape(R.shape[0], -1) if R.ndim > 1 else R.reshape(1, -1)
    return float(_load().scdo_fro2(R2, R2.shape[0], R2.shape[1]))


def rank1_update(R, ck: float, sbits, tbits) -> None:
    """In place R <- R - ck s t^T; R must be a C-contiguous float64 array."""
    assert R.dtype == np.float64 and R.flags.c_contiguous
    m, n = R.shape
    _load().scdo_rank1_update(R, m, n, float(ck), _u64(sbits), _u64(tbits))


def greedy_signed_cut(R, t0bits, max_iters: int = DEFAULT_MAX_ITERS):
    """Algorithm 4.  Returns dict(c=<s,Rt> unnormalised, s, t, iters, c_hist, margin, capped)."""
    R = _f64(R)
    m, n = R.shape
    t = _u64(t0bits).copy()
    s = np.zeros(words(m), dtype=np.uint64)
    c = C.c_double()
    it = C.c_int32()
    hist = np.zeros(max_iters, dtype=np.float64)
    margin = np.zeros(2, dtype=np.float64)
    capped = _load().scdo_greedy_signed_cut(R, m, n, t, s, C.byref(c), max_iters, C.byref(it),
                                            hist.ctypes.data, margin.ctypes.data)
    return dict(c=c.value, s=s, t=t, iters=it.value, c_hist=hist[: it.value].copy(), margin=margin,
                capped=bool(capped))


def greedy_signed_cut_near_ties(R, t0bits, tol: float, tol_c: float = 0.0, accept=None,
                                max_iters: int = DEFAULT_MAX_ITERS, max_runs: int = 64):
    """Every outcome of Algorithm 4 that differs from the literal one only at decisions that are near ties.

    Algorithm 4 takes two kinds of decisions: a sign, s_i = sgn((R t)_i) or t_l = sgn((R^T s)_l) (lines 5-6),
    and the stop test c_j <= c_{j-1} (line 8).  An implementation that sums in another order or precision may
    take a sign decision the other way where |value| < tol * max|value| of its vector, and the stop decision
    the other way where 0 < |c_j - c_{j-1}| <= tol_c * |c_j|; everything after such a decision follows
    Algorithm 4 again from the changed state.  This walks the tree of those alternatives, smallest margin
    first: the literal run is outcome 0; with tol = tol_c = 0 it is the only one.

    Steps are the oracle's own (row_signed_sum, col_signed_sum, pack), in the order of Algorithm 4.
    accept: optional predicate on an outcome; the search stops at the first outcome it accepts.
    Returns dict(outcomes=[dict(c, s, t, iters, flips)], accepted=index or None, truncated=bool) where
    `flips` counts the decisions taken against the literal rule on the way to that outcome.
    """
    import heapq

    R = _f64(R)
    m, n = R.shape
    outcomes = []
    accepted = [None]
    counter = [0]
    heap = []

    def push(prio, state):
        counter[0] += 1
        heapq.heappush(heap, (prio, counter[0], state))

    def emit(c, s, t, j, nflips):
        outcomes.append(dict(c=float(c), s=s.copy(), t=t.copy(), iters=int(j), flips=int(nflips)))
        if accept is not None and accepted[0] is None and accept(outcomes[-1]):
            accepted[0] = len(outcomes) - 1

    def decide(x, flip_idx):
        """sgn of a vector with the entries `flip_idx` taken the other way; also the near-tie entries."""
        bits = pack(x)
        ax = np.abs(x)
        mx = ax.max() if ax.size else 0.0
        near = np.nonzero(ax < tol * mx)[0] if tol > 0.0 and mx > 0.0 else np.zeros(0, dtype=np.int64)
        for i in flip_idx:
            bits[i >> 6] ^= np.uint64(1) << np.uint64(i & 63)
        return bits, near, (ax / mx if mx > 0.0 else ax)

    def run(state):
        """Follow Algorithm 4 from a saved decision point to its end, queueing the alternatives met on the way."""
        j, phase, x, s, c_prev, flips_here, nflips = (state[k] for k in ("j", "phase", "x", "s", "c_prev", "flips", "nflips"))
        first = True
        while True:
            if phase == 0:
                # line 5: s_j = sgn(R t_{j-1}), x = R t_{j-1}
                fl = flips_here if first else ()
                s, near, rel = decide(x, fl)
                lo = max(fl) if fl else -1
                for i in near[near > lo]:
                    push(rel[i] / tol, dict(j=j, phase=0, x=x, s=s, c_prev=c_prev, flips=tuple(fl) + (int(i),),
                                            nflips=nflips + 1))
                first = False
                x = col_signed_sum(R, s)
                phase = 1
            # line 6: t_j = sgn(R^T s_j), x = R^T s_j
            fl = flips_here if first else ()
            t, near, rel = decide(x, fl)
            lo = max(fl) if fl else -1
            for i in near[near > lo]:
                push(rel[i] / tol, dict(j=j, phase=1, x=x, s=s, c_prev=c_prev, flips=tuple(fl) + (int(i),),
                                        nflips=nflips + 1))
            first = False
            u = row_signed_sum(R, t)
            c = float(np.cumsum(unpack(s, m) * u)[-1])  # line 7, added in the order i = 0..m-1
            stop = c <= c_prev
            close = tol_c > 0.0 and c != c_prev and abs(c - c_prev) <= tol_c * abs(c)
            if stop or j >= max_iters:
                emit(c, s, t, j, nflips)
                if close and j < max_iters:
                    # the other implementation saw an increase: it goes on from here
                    push(abs(c - c_prev) / (tol_c * abs(c)), dict(j=j + 1, phase=0, x=u, s=s, c_prev=c, flips=(),
                                                                   nflips=nflips + 1))
                return
            if close:
                # the other implementation saw no increase: it stops here with the current triple (line 9)
                emit(c, s, t, j, nflips + 1)
            c_prev = c
            j += 1
            phase = 0
            x = u

    push(0.0, dict(j=1, phase=0, x=row_signed_sum(R, _u64(t0bits)), s=None, c_prev=-np.inf, flips=(), nflips=0))
    runs = 0
    while heap and accepted[0] is None and runs < max_runs:
        _, _, state = heapq.heappop(heap)
        run(state)
        runs += 1
    return dict(outcomes=outcomes, accepted=accepted[0], truncated=bool(heap) and accepted[0] is None)


def decompose(A, w: int, seed: int, max_iters: int = DEFAULT_MAX_ITERS, want_remainder: bool = False):
    """Algorithm 5.  Returns dict(S, T, c, trace, iters, margins, capped[, R])."""
    A = _f64(A)
    m, n = A.shape
    S = np.zeros((w, words(m)), dtype=np.uint64)
    T = np.zeros((w, words(n)), dtype=np.uint64)
    c = np.zeros(w, dtype=np.float64)
    trace = np.zeros(w + 1, dtype=np.float64)
    iters = np.zeros(w, dtype=np.int32)
    margins = np.zeros((w, 2), dtype=np.float64)
    R = np.empty_like(A) if want_remainder else None
    capped = _load().scdo_decompose(A, m, n, w, seed, max_iters, S, T, c, trace, iters.ctypes.data,
                                    margins.ctypes.data, _opt(R))
    out = dict(S=S, T=T, c=c, trace=trace, iters=iters, margins=margins, capped=int(capped))
    if want_remainder:
        out["R"] = R
    return out


def lsq_coefficients(A, S, T) -> np.ndarray:
    """argmin_c ||A - sum_j c_j s_j t_j^T||_F for given sign vectors (Algorithm 6 line 9, Section 3.3)."""
    A = _f64(A)
    m, n = A.shape
    S, T = _u64(S).reshape(-1, words(m)), _u64(T).reshape(-1, words(n))
    k = S.shape[0]
    c = np.zeros(k, dtype=np.float64)
    if _load().scdo_lsq_coefficients(A, m, n, k, S, T, c):
        raise np.linalg.LinAlgError("normal equations singular")
    return c


def lsq_decompose(A, w: int, seed: int, max_iters: int = DEFAULT_MAX_ITERS):
    """Algorithm 6.  Returns dict(S, T, c (final, all terms), trace, iters, margins, capped)."""
    A = _f64(A)
    m, n = A.shape
    S = np.zeros((w, words(m)), dtype=np.uint64)
    T = np.zeros((w, words(n)), dtype=np.uint64)
    c = np.zeros(w, dtype=np.float64)
    trace = np.zeros(w + 1, dtype=np.float64)
    iters = np.zeros(w, dtype=np.int32)
    margins = np.zeros((w, 2), dtype=np.float64)
    capped = _load().scdo_lsq_decompose(A, m, n, w, seed, max_iters, S, T, c, trace, iters.ctypes.data,
                                        margins.ctypes.data)
    if capped < 0:
        raise np.linalg.LinAlgError("normal equations singular")
    return dict(S=S, T=T, c=c, trace=trace, iters=iters, margins=margins, capped=int(capped))


def mode_signed_sum(a, signs, mode: int) -> np.ndarray:
    a = _f64(a)
    dims = np.asarray(a.shape, dtype=np.int64)
    sg = [_u64(s) for s in signs]
    u = np.empty(a.shape[mode], dtype=np.float64)
    _load().scdo_mode_signed_sum(a.reshape(-1), a.ndim, dims, _ptrs(sg), mode, u)
    return u


def tensor_inner(a, signs) -> float:
    a = _f64(a)
    dims = np.asarray(a.shape, dtype=np.int64)
    sg = [_u64(s) for s in signs]
    return float(_load().scdo_tensor_inner(a.reshape(-1), a.ndim, dims, _ptrs(sg)))


def tensor_update(r, ck: float, signs) -> None:
    assert r.dtype == np.float64 and r.flags.c_contiguous
    dims = np.asarray(r.shape, dtype=np.int64)
    sg = [_u64(s) for s in signs]
    _load().scdo_tensor_update(r.reshape(-1), r.ndim, dims, float(ck), _ptrs(sg))


def axial_greedy_cut(a, signs0, max_iters: int = DEFAULT_MAX_ITERS):
    """Algorithm 12.  signs0: one bitset per mode (mode 0's is never read)."""
    a = _f64(a)
    dims = np.asarray(a.shape, dtype=np.int64)
    sg = [_u64(s).copy() for s in signs0]
    c = C.c_double()
    it = C.c_int32()
    hist = np.zeros(max_iters, dtype=np.float64)
    margin = np.zeros(a.ndim, dtype=np.float64)
    capped = _load().scdo_axial_greedy_cut(a.reshape(-1), a.ndim, dims, _ptrs(sg), C.byref(c), max_iters,
                                           C.byref(it), hist.ctypes.data, margin.ctypes.data)
    return dict(c=c.value, signs=sg, iters=it.value, c_hist=hist[: it.value].copy(), margin=margin,
                capped=bool(capped))


def axial_greedy_cut_near_ties(a, signs0, tol: float, tol_c: float = 0.0, accept=None,
                               max_iters: int = DEFAULT_MAX_ITERS, max_runs: int = 64):
    """Algorithm 12 with its near-tie decisions left open, as greedy_signed_cut_near_ties does for Algorithm 4:
    a sign of mode i may go the other way where |value| < tol * max|value| of that mode's sums, the stop test
    (line 11) where 0 < |c_j - c_{j-1}| <= tol_c |c_j|.  Steps: mode_signed_sum, pack, tensor_inner, in the
    order of Algorithm 12.  Returns dict(outcomes=[dict(c, signs, iters, flips)], accepted, truncated)."""
    import heapq

    a = _f64(a)
    order = a.ndim
    outcomes, accepted, counter, heap = [], [None], [0], []

    def push(prio, state):
        counter[0] += 1
        heapq.heappush(heap, (prio, counter[0], state))

    def emit(c, sg, j, nflips):
        outcomes.append(dict(c=float(c), signs=[s.copy() for s in sg], iters=int(j), flips=int(nflips)))
        if accept is not None and accepted[0] is None and accept(outcomes[-1]):
            accepted[0] = len(outcomes) - 1

    def run(state):
        j, i0, sg, c_prev, flips_here, nflips = (state[k] for k in ("j", "mode", "signs", "c_prev", "flips", "nflips"))
        sg = [s.copy() for s in sg]
        first = True
        while True:
            for i in range(i0, order):
                x = mode_signed_sum(a, sg, i)          # lines 5-8: modes before i new, after i old
                fl = flips_here if first else ()
                first = False
                bits = pack(x)
                ax = np.abs(x)
                mx = ax.max()
                if tol > 0.0 and mx > 0.0:
                    lo = max(fl) if fl else -1
                    for q in np.nonzero(ax < tol * mx)[0]:
                        if q > lo:
                            push(ax[q] / mx / tol, dict(j=j, mode=i, signs=[s.copy() for s in sg], c_prev=c_prev,
                                                        flips=tuple(fl) + (int(q),), nflips=nflips + 1))
                for q in fl:
                    bits[q >> 6] ^= np.uint64(1) << np.uint64(q & 63)
                sg[i] = bits
            i0 = 0
            c = tensor_inner(a, sg)                    # line 10
            stop = c <= c_prev
            close = tol_c > 0.0 and c != c_prev and abs(c - c_prev) <= tol_c * abs(c)
            if stop or j >= max_iters:
                emit(c, sg, j, nflips)
                if close and j < max_iters:
                    push(abs(c - c_prev) / (tol_c * abs(c)), dict(j=j + 1, mode=0, signs=[s.copy() for s in sg], c_prev=c,
                                                                   flips=(), nflips=nflips + 1))
                return
            if close:
                emit(c, sg, j, nflips + 1)
            c_prev = c
            j += 1

    push(0.0, dict(j=1, mode=0, signs=[_u64(s).copy() for s in signs0], c_prev=-np.inf, flips=(), nflips=0))
    runs = 0
    while heap and accepted[0] is None and runs < max_runs:
        run(heapq.heappop(heap)[2])
        runs += 1
    return dict(outcomes=outcomes, accepted=accepted[0], truncated=bool(heap) and accepted[0] is None)


def tensor_decompose(a, w: int, seed: int, max_iters: int = DEFAULT_MAX_ITERS, want_remainder: bool = False):
    """Algorithm 13.  Returns dict(signs=[per-mode (w, words) arrays], c, trace, iters, margins[, r])."""
    a = _f64(a)
    dims = np.asarray(a.shape, dtype=np.int64)
    sg = [np.zeros((w, words(d)), dtype=np.uint64) for d in a.shape]
    c = np.zeros(w, dtype=np.float64)
    trace = np.zeros(w + 1, dtype=np.float64)
    iters = np.zeros(w, dtype=np.int32)
    margins = np.zeros((w, a.ndim), dtype=np.float64)
    r = np.empty_like(a) if want_remainder else None
    capped = _load().scdo_tensor_decompose(a.reshape(-1), a.ndim, dims, w, seed, max_iters, _ptrs(sg), c,
                                           trace, iters.ctypes.data, margins.ctypes.data, _opt(r))
    out = dict(signs=sg, c=c, trace=trace, iters=iters, margins=margins, capped=int(capped))
    if want_remainder:
        out["r"] = r
    return out


def tensor_lsq_coefficients(a, signs) -> np.ndarray:
    """argmin_c ||a - sum_j c_j (tensor product of term j's sign vectors)||_2 (Algorithm 14 line 8)."""
    a = _f64(a)
    dims = np.asarray(a.shape, dtype=np.int64)
    sg = [_u64(s).reshape(-1, words(d)) for s, d in zip(signs, a.shape)]
    k = sg[0].shape[0]
    c = np.zeros(k, dtype=np.float64)
    if _load().scdo_tensor_lsq_coefficients(a.reshape(-1), a.ndim, dims, k, _ptrs(sg), c):
        raise np.linalg.LinAlgError("normal equations singular")
    return c


def tensor_lsq_decompose(a, w: int, seed: int, max_iters: int = DEFAULT_MAX_ITERS):
    """Algorithm 14.  Returns dict(signs, c (final, all terms), trace, iters, margins, capped)."""
    a = _f64(a)
    dims = np.asarray(a.shape, dtype=np.int64)
    sg = [np.zeros((w, words(d)), dtype=np.uint64) for d in a.shape]
    c = np.zeros(w, dtype=np.float64)
    trace = np.zeros(w + 1, dtype=np.float64)
    iters = np.zeros(w, dtype=np.int32)
    margins = np.zeros((w, a.ndim), dtype=np.float64)
    capped = _load().scdo_tensor_lsq_decompose(a.reshape(-1), a.ndim, dims, w, seed, max_iters, _ptrs(sg), c, trace,
                                               iters.ctypes.data, margins.ctypes.data)
    if capped < 0:
        raise np.linalg.LinAlgError("normal equations singular")
    return dict(signs=sg, c=c, trace=trace, iters=iters, margins=margins, capped=int(capped))


def scalars_decompose(a, w: int, seed: int, max_iters: int = DEFAULT_MAX_ITERS):
    """"RGB scalars" (Section 5): sign vectors for all modes but the last, a real vector over the last mode per
    term.  Returns dict(signs (all modes, the last one being the cut's), c (w, n_last), trace, iters, margins)."""
    a = _f64(a)
    dims = np.asarray(a.shape, dtype=np.int64)
    sg = [np.zeros((w, words(d)), dtype=np.uint64) for d in a.shape]
    c = np.zeros((w, a.shape[-1]), dtype=np.float64)
    trace = np.zeros(w + 1, dtype=np.float64)
    iters = np.zeros(w, dtype=np.int32)
    margins = np.zeros((w, a.ndim), dtype=np.float64)
    capped = _load().scdo_scalars_decompose(a.reshape(-1), a.ndim, dims, w, seed, max_iters, _ptrs(sg), c.reshape(-1), trace,
                                            iters.ctypes.data, margins.ctypes.data)
    return dict(signs=sg, c=c, trace=trace, iters=iters, margins=margins, capped=int(capped))


def expand(signs, c, dims) -> np.ndarray:
    """sum_j c[j] * (tensor product of term j's sign vectors), f64, terms added in order."""
    dims = np.asarray(dims, dtype=np.int64)
    sg = [_u64(s) for s in signs]
    c = _f64(c).ravel()
    out = np.empty(int(np.prod(dims)), dtype=np.float64)
    _load().scdo_expand(len(dims), dims, c.size, _ptrs(sg), c, out)
    return out.reshape(tuple(int(d) for d in dims))


def apply(S, T, c, m: int, n: int, x, transpose: bool = False) -> np.ndarray:
    """(sum_j c_j s_j t_j^T) x, or the transposed matrix times x, from the packed factors (Section 6.1)."""
    S, T, c, x = _u64(S), _u64(T), _f64(c).ravel(), _f64(x).ravel()
    assert x.size == (m if transpose else n)
    y = np.empty(n if transpose else m, dtype=np.float64)
    _load().scdo_apply(m, n, c.size, S, T, c, 1 if transpose else 0, x, y)
    return y


def relative_error(approx, exact) -> float:
    """r = ||approx - exact||_F / ||exact||_F in f64: the error measure of Section 4.1 (Figure 7's r_k with
    approx = A - R_k), written out entry by entry."""
    a, e = _f64(approx).ravel(), _f64(exact).ravel()
    assert a.size == e.size
    num = math.fsum((x - y) * (x - y) for x, y in zip(a.tolist(), e.tolist())) if a.size <= 4096 else float(np.sum((a - e) ** 2))
    den = math.fsum(y * y for y in e.tolist()) if a.size <= 4096 else float(np.sum(e ** 2))
    return math.sqrt(num / den)


def bruteforce_signed_cut_norm(A):
    """max_s ||A^T s||_1 by enumeration (m <= 24).  Returns (norm, s bitmask as int)."""
    A = _f64(A)
    m, n = A.shape
    arg = C.c_uint64()
    val = _load().scdo_bruteforce_signed_cut_norm(A, m, n, C.byref(arg))
    return float(val), int(arg.value)
