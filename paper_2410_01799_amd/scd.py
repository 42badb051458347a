"""Thin ctypes binding of ``libscd.so`` (see ``include/scd.h``): argument marshalling only.

PyTorch provides device memory and streams; every step of the method runs in the library's HIP
kernels.  There is no CPU fallback: if the library is missing, importing succeeds but the first
call raises.
"""
from __future__ import annotations

import ctypes as C
from pathlib import Path
from typing import List, Optional, Sequence

import torch

_PKG = Path(__file__).resolve().parent
LIB_PATH = _PKG / "libscd.so"
_lib = None

F32, F64 = 0, 1
OK, WMAXITER = 0, 1
EINVAL, ENOMEM, EHIP, EFULL, ENONFINITE, ENODEVICE, ETIMEOUT, ESINGULAR, ETOOBIG = -1, -2, -3, -4, -5, -6, -7, -8, -9
NOALLOC_SCRATCH_BYTES = 24 << 20

EXPORTS = [
    "scd_decompose", "scd_create", "scd_destroy", "scd_set_max_iters", "scd_step", "scd_run", "scd_step_from",
    "scd_width", "scd_results", "scd_remainder", "scd_set_remainder", "scd_row_signed_sum", "scd_col_signed_sum",
    "scd_expand", "scd_pack", "scd_unpack", "scd_rng_signs", "scd_strerror", "scd_last_hip_error", "scd_traffic",
    "scd_probe_stream", "scd_profile_sweeps", "scd_probe_exchange", "scd_engine", "scd_set_workgroups",
    "scd_apply", "scd_apply_workspace_bytes", "scd_lsq_decompose", "scd_lsq_decompose_tensor", "scd_decompose_scalars", "scd_sparse_flips",
    "scd_col_signed_sum_noalloc", "scd_set_option", "scd_get_option", "scd_stream_geometry",
]

# scd_option of include/scd.h
OPTIONS = {"resident": 0, "sparse": 1, "sparse_min_mib": 2, "sparse_delay_width": 3, "rowpass_kernel": 4,
           "poll_delay": 5, "max_spin": 6, "sweep_batch": 7, "verbose": 8, "persistent_stream": 9}


class ScdError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().scd_strerror(code).decode()
        if code == EHIP:
            msg += f" (hipError {lib().scd_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{code}]")


def lib() -> C.CDLL:
    """Load libscd.so (built in-tree by ``paper_2410_01799_amd.build``); raises if it is absent."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2410_01799_amd.build` "
                               "(or __graft_entry__.build()) first; there is no fallback path")
        L = C.CDLL(str(LIB_PATH))
        vp, i64, u64, i32 = C.c_void_p, C.c_int64, C.c_uint64, C.c_int32
        pvp = C.POINTER(C.c_void_p)
        pi64 = C.POINTER(C.c_int64)
        L.scd_decompose.argtypes = [vp, C.c_int, C.c_int, pi64, i64, u64, vp, pvp, vp, vp, vp]
        L.scd_create.argtypes = [pvp, vp, C.c_int, C.c_int, pi64, i64, u64, vp]
        L.scd_destroy.argtypes = [vp]
        L.scd_destroy.restype = None
        L.scd_set_max_iters.argtypes = [vp, i32]
        L.scd_set_workgroups.argtypes = [vp, C.c_int]
        L.scd_stream_geometry.argtypes = [C.c_int, C.c_int, pi64, C.c_int, pi64]
        L.scd_set_option.argtypes = [vp, C.c_int, i64]
        L.scd_get_option.argtypes = [vp, C.c_int, pi64]
        L.scd_sparse_flips.argtypes = [vp, pi64, pi64]
        L.scd_lsq_decompose.argtypes = [vp, C.c_int, i64, i64, i64, C.c_uint64, i32, vp, vp, vp, vp, vp, vp]
        L.scd_lsq_decompose_tensor.argtypes = [vp, C.c_int, C.c_int, pi64, i64, C.c_uint64, i32, vp, pvp, vp, vp, vp]
        L.scd_decompose_scalars.argtypes = [vp, C.c_int, C.c_int, pi64, i64, C.c_uint64, i32, vp, pvp, vp, vp, vp]
        L.scd_apply_workspace_bytes.argtypes = [i64, i64, i64]
        L.scd_apply_workspace_bytes.restype = C.c_size_t
        L.scd_apply.argtypes = [vp, vp, vp, C.c_int, i64, i64, i64, C.c_int, vp, i64, vp, vp, C.c_size_t, vp]
        L.scd_step.argtypes = [vp]
        L.scd_run.argtypes = [vp, i64]
        L.scd_step_from.argtypes = [vp, pvp]
        L.scd_width.argtypes = [vp, pi64]
        L.scd_results.argtypes = [vp, pvp, vp, vp, vp]
        L.scd_remainder.argtypes = [vp, vp]
        L.scd_set_remainder.argtypes = [vp, vp]
        L.scd_row_signed_sum.argtypes = [vp, C.c_int, i64, i64, vp, vp, vp, vp]
        L.scd_col_signed_sum.argtypes = [vp, C.c_int, i64, i64, vp, vp, vp, vp, vp]
        L.scd_col_signed_sum_noalloc.argtypes = [vp, C.c_int, i64, i64, vp, vp, vp, vp, vp]
        L.scd_expand.argtypes = [pvp, vp, C.c_int, C.c_int, pi64, i64, vp, vp]
        L.scd_pack.argtypes = [vp, C.c_int, i64, vp, vp]
        L.scd_unpack.argtypes = [vp, i64, C.c_int, vp, vp]
        L.scd_rng_signs.argtypes = [u64, u64, C.c_uint32, i64, vp, vp]
        L.scd_strerror.argtypes = [C.c_int]
        L.scd_strerror.restype = C.c_char_p
        L.scd_last_hip_error.argtypes = []
        L.scd_traffic.argtypes = [vp, C.POINTER(C.c_double), pi64, pi64]
        L.scd_profile_sweeps.argtypes = [vp, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.scd_engine.argtypes = [vp, C.POINTER(C.c_int), C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.scd_probe_exchange.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, vp, C.POINTER(C.c_double)]
        L.scd_probe_stream.argtypes = [vp, vp, i64, C.c_int, C.c_int, vp, C.POINTER(C.c_double)]
        _lib = L
    return _lib


# --------------------------------------------------------------------------- marshalling helpers


def words(n: int) -> int:
    return (int(n) + 63) // 64


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.float64:
        return F64
    raise TypeError(f"dtype {t.dtype} not supported (float32 or float64)")


def _dev(t: torch.Tensor, name: str) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _dims(shape: Sequence[int]):
    return (C.c_int64 * len(shape))(*[int(d) for d in shape])


def _ptr_array(ts: Sequence[Optional[torch.Tensor]]):
    arr = (C.c_void_p * len(ts))()
    for i, t in enumerate(ts):
        arr[i] = None if t is None else t.data_ptr()
    return arr


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _bits(n_words: int, device, rows: Optional[int] = None) -> torch.Tensor:
    shape = (n_words,) if rows is None else (rows, n_words)
    return torch.zeros(shape, dtype=torch.int64, device=device)   # uint64 words carried as int64 storage


def _check(code: int, where: str) -> int:
    if code < 0:
        raise ScdError(code, where)
    return code


# --------------------------------------------------------------------------- one-shot calls


def scd_decompose(A: torch.Tensor, w: int, seed: int, want_iters: bool = True, options: Optional[dict] = None):
    """Greedy signed cut decomposition of A to width w.  Returns dict(signs=[per-mode (w, words)
    int64 tensors holding uint64 bitsets], c, trace (float64, w+1), iters, status).  With `options` (names of
    OPTIONS) the same steps go through the stateful calls, which is where options can be set."""
    A = _dev(A, "A")
    if options:
        with ScdContext(A, w, seed, options=options) as ctx:
            st = ctx.run(w)
            res = ctx.results()
        res["status"] = st
        return res
    dev = A.device
    signs = [_bits(words(d), dev, rows=w) for d in A.shape]
    c = torch.zeros(w, dtype=A.dtype, device=dev)
    trace = torch.zeros(w + 1, dtype=torch.float64, device=dev)
    iters = torch.zeros(w, dtype=torch.int32, device=dev) if want_iters else None
    st = lib().scd_decompose(_ptr(A), _dt(A), A.dim(), _dims(A.shape), int(w), int(seed), _stream(),
                             _ptr_array(signs), _ptr(c), _ptr(trace), _ptr(iters))
    _check(st, "scd_decompose")
    return dict(signs=signs, c=c, trace=trace, iters=iters, status=st)


def scd_expand(signs: Sequence[torch.Tensor], c: torch.Tensor, dims: Sequence[int]) -> torch.Tensor:
    """sum_j c_j * (tensor product of term j's sign vectors), dtype of c."""
    c = _dev(c, "c")
    w = int(c.numel())
    for s in signs:
        _dev(s, "signs")
    out = torch.empty(tuple(int(d) for d in dims), dtype=c.dtype, device=c.device)
    st = lib().scd_expand(_ptr_array(list(signs)), _ptr(c), _dt(c), len(dims), _dims(dims), w, _stream(), _ptr(out))
    _check(st, "scd_expand")
    return out


def scd_lsq_decompose(A: torch.Tensor, w: int, seed: int, max_iters: int = 4096) -> dict:
    """Algorithms 6 (matrices) and 14 (tensors): greedy cuts with all coefficients refitted by least squares
    after every term.  Returns dict(signs=[per-mode bitsets], c (final coefficients), trace, iters, status)."""
    A = _dev(A, "A")
    if A.dim() < 2:
        raise ValueError("order >= 2")
    w = int(w)
    signs = [_bits(w * words(int(d)), A.device).reshape(w, words(int(d))) for d in A.shape]
    c = torch.empty(w, dtype=A.dtype, device=A.device)
    trace = torch.empty(w + 1, dtype=torch.float64, device=A.device)
    iters = torch.empty(w, dtype=torch.int32, device=A.device)
    if A.dim() == 2:
        st = lib().scd_lsq_decompose(_ptr(A), _dt(A), int(A.shape[0]), int(A.shape[1]), w, int(seed), int(max_iters),
                                     _stream(), _ptr(signs[0]), _ptr(signs[1]), _ptr(c), _ptr(trace), _ptr(iters))
    else:
        st = lib().scd_lsq_decompose_tensor(_ptr(A), _dt(A), A.dim(), _dims(A.shape), w, int(seed), int(max_iters),
                                            _stream(), _ptr_array(signs), _ptr(c), _ptr(trace), _ptr(iters))
    st = _check(st, "scd_lsq_decompose")
    return dict(signs=signs, c=c, trace=trace, iters=iters, status=st)


def scd_decompose_scalars(A: torch.Tensor, w: int, seed: int, max_iters: int = 4096) -> dict:
    """"RGB scalars" (Section 5): sign vectors for every mode but the last, a real vector over the last mode per
    term.  Returns dict(signs=[bitsets of modes 1..k-1], c (w, n_last), trace, iters, status)."""
    A = _dev(A, "A")
    if A.dim() < 2:
        raise ValueError("order >= 2")
    w = int(w)
    signs = [_bits(w * words(int(d)), A.device).reshape(w, words(int(d))) for d in A.shape[:-1]]
    c = torch.empty((w, int(A.shape[-1])), dtype=A.dtype, device=A.device)
    trace = torch.empty(w + 1, dtype=torch.float64, device=A.device)
    iters = torch.empty(w, dtype=torch.int32, device=A.device)
    st = lib().scd_decompose_scalars(_ptr(A), _dt(A), A.dim(), _dims(A.shape), w, int(seed), int(max_iters), _stream(),
                                     _ptr_array(signs), _ptr(c), _ptr(trace), _ptr(iters))
    st = _check(st, "scd_decompose_scalars")
    return dict(signs=signs, c=c, trace=trace, iters=iters, status=st)


def scd_apply(S: torch.Tensor, T: torch.Tensor, c: torch.Tensor, m: int, n: int, x: torch.Tensor,
              transpose: bool = False, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """(sum_j c_j s_j t_j^T) x, or the transposed matrix times x, from the packed factors; x may hold
    several vectors as rows.  dtype of c."""
    c = _dev(c, "c")
    S, T = _dev(S, "S"), _dev(T, "T")
    x = _dev(x, "x")
    if x.dtype != c.dtype:
        raise TypeError("x and c must have the same dtype")
    w = int(c.numel())
    nin, nout = (m, n) if transpose else (n, m)
    single = x.dim() == 1
    x2 = x.reshape(1, -1) if single else x
    if x2.dim() != 2 or x2.shape[1] != nin:
        raise ValueError(f"x must have {nin} entries per vector")
    nvec = int(x2.shape[0])
    need = int(lib().scd_apply_workspace_bytes(int(m), int(n), w))
    if workspace is None:
        workspace = torch.empty((need + 7) // 8, dtype=torch.float64, device=c.device)
    y = torch.empty((nvec, nout), dtype=c.dtype, device=c.device)
    st = lib().scd_apply(_ptr(S), _ptr(T), _ptr(c), _dt(c), int(m), int(n), w, 1 if transpose else 0, _ptr(x2), nvec,
                         _ptr(y), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream())
    _check(st, "scd_apply")
    return y[0] if single else y


def scd_pack(values: torch.Tensor) -> torch.Tensor:
    values = _dev(values, "values").reshape(-1)
    bits = _bits(words(values.numel()), values.device)
    _check(lib().scd_pack(_ptr(values), _dt(values), values.numel(), _stream(), _ptr(bits)), "scd_pack")
    return bits


def scd_unpack(bits: torch.Tensor, n: int, dtype=torch.float32) -> torch.Tensor:
    bits = _dev(bits, "bits")
    out = torch.empty(int(n), dtype=dtype, device=bits.device)
    _check(lib().scd_unpack(_ptr(bits), int(n), _dt(out), _stream(), _ptr(out)), "scd_unpack")
    return out


def scd_rng_signs(seed: int, term: int, mode: int, n: int, device="cuda") -> torch.Tensor:
    bits = _bits(words(n), device)
    _check(lib().scd_rng_signs(int(seed), int(term), int(mode), int(n), _stream(), _ptr(bits)), "scd_rng_signs")
    return bits


def scd_row_signed_sum(R: torch.Tensor, tbits: torch.Tensor):
    """u = R t (float64) and s = sgn(u) packed."""
    R = _dev(R, "R")
    m, n = R.shape
    u = torch.empty(m, dtype=torch.float64, device=R.device)
    s = _bits(words(m), R.device)
    st = lib().scd_row_signed_sum(_ptr(R), _dt(R), m, n, _ptr(_dev(tbits, "tbits")), _stream(), _ptr(u), _ptr(s))
    _check(st, "scd_row_signed_sum")
    return u, s


def scd_col_signed_sum(R: torch.Tensor, sbits: torch.Tensor):
    """v = R^T s (float64), t = sgn(v) packed, c = sum |v| (float64 scalar tensor)."""
    R = _dev(R, "R")
    m, n = R.shape
    v = torch.empty(n, dtype=torch.float64, device=R.device)
    t = _bits(words(n), R.device)
    c = torch.zeros(1, dtype=torch.float64, device=R.device)
    st = lib().scd_col_signed_sum(_ptr(R), _dt(R), m, n, _ptr(_dev(sbits, "sbits")), _stream(), _ptr(v), _ptr(t), _ptr(c))
    _check(st, "scd_col_signed_sum")
    return v, t, c


def scd_col_signed_sum_noalloc(R: torch.Tensor, sbits: torch.Tensor, v: torch.Tensor, t: torch.Tensor, c: torch.Tensor):
    """The column half step into caller-provided outputs, without any device allocation inside the library;
    enqueued on the current stream, not waited for."""
    R = _dev(R, "R")
    m, n = R.shape
    st = lib().scd_col_signed_sum_noalloc(_ptr(R), _dt(R), m, n, _ptr(_dev(sbits, "sbits")), _stream(), _ptr(v), _ptr(t),
                                          _ptr(c))
    _check(st, "scd_col_signed_sum_noalloc")


def scd_stream_geometry(dtype, dims: Sequence[int], limit: int = 256) -> Optional[dict]:
    """Launch geometry of the persistent streaming engine for this dtype and shape (host arithmetic only), or None
    when the engine does not take the shape."""
    out = (C.c_int64 * 8)()
    dt = F32 if dtype == torch.float32 else F64
    _check(lib().scd_stream_geometry(dt, len(dims), _dims(dims), int(limit), out), "scd_stream_geometry")
    if not out[0]:
        return None
    return dict(grid=out[1], rpw=out[2], cs=out[3], lds_rows=out[4], lds_bytes=out[5], xp_bytes=out[6], xq_bytes=out[7])


def scd_probe_stream(src: torch.Tensor, dst: Optional[torch.Tensor] = None, grid: int = 2048, reps: int = 20) -> float:
    """Seconds per launch of the plain streaming read (dst None) or copy kernel over src's bytes."""
    src = _dev(src, "src")
    nbytes = src.numel() * src.element_size()
    sec = C.c_double()
    st = lib().scd_probe_stream(_ptr(src), _ptr(dst), nbytes, int(grid), int(reps), _stream(), C.byref(sec))
    _check(st, "scd_probe_stream")
    return sec.value


def scd_probe_exchange(which: int, grid: int = 256, group: int = 16, rounds: int = 1000) -> float:
    """Seconds per round of the in-kernel exchange probe (0: tagged data, 1: counter barrier)."""
    sec = C.c_double()
    _check(lib().scd_probe_exchange(int(which), int(grid), int(group), int(rounds), _stream(), C.byref(sec)),
           "scd_probe_exchange")
    return sec.value


# --------------------------------------------------------------------------- stateful context


class ScdContext:
    """Owns an ``scd_ctx``: the remainder, the position in the random stream, the terms so far."""

    def __init__(self, A: torch.Tensor, w_capacity: int, seed: int, options: Optional[dict] = None):
        A = _dev(A, "A")
        self.shape = tuple(int(d) for d in A.shape)
        self.dtype = A.dtype
        self.device = A.device
        self.w_capacity = int(w_capacity)
        self._h = C.c_void_p()
        st = lib().scd_create(C.byref(self._h), _ptr(A), _dt(A), A.dim(), _dims(A.shape), int(w_capacity), int(seed),
                              _stream())
        _check(st, "scd_create")
        for name, value in (options or {}).items():
            self.set_option(name, value)

    def set_option(self, name: str, value: int):
        _check(lib().scd_set_option(self._h, OPTIONS[name], int(value)), f"scd_set_option({name})")

    def get_option(self, name: str) -> int:
        v = C.c_int64()
        _check(lib().scd_get_option(self._h, OPTIONS[name], C.byref(v)), f"scd_get_option({name})")
        return int(v.value)

    def close(self):
        if getattr(self, "_h", None) and self._h.value:
            lib().scd_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def set_max_iters(self, n: int):
        _check(lib().scd_set_max_iters(self._h, int(n)), "scd_set_max_iters")

    def sparse_flips(self) -> dict:
        """Row and column signs that changed after the first alternation of their term (sparse engine)."""
        r, cl = C.c_int64(), C.c_int64()
        _check(lib().scd_sparse_flips(self._h, C.byref(r), C.byref(cl)), "scd_sparse_flips")
        return dict(rows=int(r.value), cols=int(cl.value))

    def set_workgroups(self, n: int):
        """Share of the device (workgroups of the persistent launches; 0 = all): lets several contexts,
        each on its own stream and host thread, run side by side."""
        _check(lib().scd_set_workgroups(self._h, int(n)), "scd_set_workgroups")

    def step(self) -> int:
        return _check(lib().scd_step(self._h), "scd_step")

    def run(self, n: int) -> int:
        return _check(lib().scd_run(self._h, int(n)), "scd_run")

    def step_from(self, init_signs: Sequence[Optional[torch.Tensor]]) -> int:
        return _check(lib().scd_step_from(self._h, _ptr_array(list(init_signs))), "scd_step_from")

    @property
    def width(self) -> int:
        k = C.c_int64()
        _check(lib().scd_width(self._h, C.byref(k)), "scd_width")
        return int(k.value)

    def results(self):
        k = self.width
        signs = [_bits(words(d), self.device, rows=k) for d in self.shape]
        c = torch.zeros(k, dtype=self.dtype, device=self.device)
        trace = torch.zeros(k + 1, dtype=torch.float64, device=self.device)
        iters = torch.zeros(k, dtype=torch.int32, device=self.device)
        st = lib().scd_results(self._h, _ptr_array(signs), _ptr(c), _ptr(trace), _ptr(iters))
        _check(st, "scd_results")
        return dict(signs=signs, c=c, trace=trace, iters=iters)

    def remainder(self) -> torch.Tensor:
        R = torch.empty(self.shape, dtype=self.dtype, device=self.device)
        _check(lib().scd_remainder(self._h, _ptr(R)), "scd_remainder")
        return R

    def set_remainder(self, R: torch.Tensor):
        R = _dev(R, "R")
        if tuple(R.shape) != self.shape or R.dtype != self.dtype:
            raise ValueError("remainder must have the shape and dtype of the input")
        _check(lib().scd_set_remainder(self._h, _ptr(R)), "scd_set_remainder")

    def profile_sweeps(self, n: int):
        """Average seconds of the row-pass launch and of the reduce launch over n further sweeps."""
        a, b = C.c_double(), C.c_double()
        _check(lib().scd_profile_sweeps(self._h, int(n), C.byref(a), C.byref(b)), "scd_profile_sweeps")
        return a.value, b.value

    def engine(self):
        """dict(engine=0 launch stream | 1 register-resident, last_launch_seconds, last_launch_bytes)."""
        e, s_, b = C.c_int(), C.c_double(), C.c_double()
        _check(lib().scd_engine(self._h, C.byref(e), C.byref(s_), C.byref(b)), "scd_engine")
        return dict(engine=int(e.value), last_launch_seconds=s_.value, last_launch_bytes=b.value)

    def traffic(self):
        b = C.c_double()
        p = C.c_int64()
        s = C.c_int64()
        _check(lib().scd_traffic(self._h, C.byref(b), C.byref(p), C.byref(s)), "scd_traffic")
        return dict(bytes=b.value, passes=int(p.value), sweeps=int(s.value))
