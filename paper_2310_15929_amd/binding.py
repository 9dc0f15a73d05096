"""ctypes binding of libesparse.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; torch is used for device memory and
for the current stream.  There is no fallback: if the shared library is missing, loading fails.
Names follow include/esparse.h.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

F16, BF16 = 0, 1
USE_ENTROPY, USE_NORM, USE_GNS, USE_LBS, USE_ALL = 1, 2, 4, 8, 15

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libesparse.so")
_lib = None


class EsparseError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"esparse error {code}: {message}")
        self.code = code


class _Opts(C.Structure):
    _fields_ = [("n_keep", C.c_int), ("m_group", C.c_int), ("block", C.c_int), ("bins", C.c_int),
                ("alpha", C.c_double), ("flags", C.c_uint), ("max_swaps", C.c_longlong)]


def load_library():
    """Load libesparse.so (built by __graft_entry__.build()).  Raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python __graft_entry__.py` (there is no fallback path)")
    lib = C.CDLL(_LIB_PATH)
    vp, ll, i32, sz = C.c_void_p, C.c_longlong, C.c_int, C.c_size_t
    P = C.POINTER
    sig = {
        "esparse_create": (i32, [P(vp), i32, vp]),
        "esparse_destroy": (None, [vp]),
        "esparse_set_stream": (i32, [vp, vp]),
        "esparse_last_error": (C.c_char_p, [vp]),
        "esparse_version": (C.c_char_p, []),
        "esparse_channel_stats": (i32, [vp, vp, ll, ll, i32, i32, vp, vp]),
        "esparse_prune": (i32, [vp, vp, ll, vp, ll, ll, i32, P(_Opts), vp, vp, vp, vp, vp]),
        "esparse_prune_with_scores": (i32, [vp, vp, vp, ll, ll, i32, P(_Opts), vp, vp, vp, vp]),
        "esparse_output_error": (i32, [vp, vp, vp, ll, ll, i32, vp, vp]),
        "esparse_matrix_rate": (i32, [vp, i32, i32, i32, i32, P(C.c_double)]),
        "esparse_read_rate": (i32, [vp, sz, P(C.c_double)]),
        "esparse_spmm_group_workspace": (i32, [i32, ll, ll, ll, P(sz)]),
        "esparse_spmm_group": (i32, [vp, i32, P(vp), ll, P(vp), P(vp), ll, ll, i32, i32, i32, P(vp), vp, sz, i32]),
        "esparse_dense_gemm_group": (i32, [vp, i32, P(vp), ll, P(vp), ll, ll, i32, P(vp), vp, sz, i32]),
        "esparse_stage_activations_group": (i32, [vp, i32, P(vp), ll, P(vp), ll, ll, i32, i32, i32, vp, sz, i32]),
        "esparse_spmm_group_staged": (i32, [vp, i32, ll, P(vp), ll, ll, i32, i32, i32, P(vp), vp, sz, i32]),
        "esparse_compressed_size": (i32, [ll, ll, i32, i32, i32, P(sz), P(sz), P(sz)]),
        "esparse_compress": (i32, [vp, vp, vp, vp, ll, ll, i32, i32, i32, vp, vp, vp]),
        "esparse_spmm_workspace": (i32, [ll, ll, ll, i32, P(sz)]),
        "esparse_spmm": (i32, [vp, vp, ll, vp, vp, ll, ll, i32, i32, i32, vp, vp, sz, i32]),
        "esparse_spmm_static": (i32, [vp, vp, ll, vp, vp, ll, ll, i32, i32, i32, vp, i32]),
        "esparse_stage_activations": (i32, [vp, vp, ll, vp, ll, ll, i32, vp, sz]),
        "esparse_spmm_staged": (i32, [vp, ll, vp, ll, ll, i32, i32, i32, vp, vp, sz, i32]),
        "esparse_dense_gemm_staged": (i32, [vp, ll, vp, ll, ll, i32, vp, vp, sz, i32]),
        "esparse_spmm_num_variants": (i32, []),
        "esparse_spmm_variant_name": (C.c_char_p, [i32]),
        "esparse_dense_packed_size": (i32, [ll, ll, P(sz)]),
        "esparse_dense_pack": (i32, [vp, vp, ll, ll, i32, vp]),
        "esparse_dense_gemm": (i32, [vp, vp, ll, vp, ll, ll, i32, vp, vp, sz, i32]),
        "esparse_tune": (i32, [vp, ll, ll, ll, i32, i32, P(i32), P(C.c_float)]),
        "esparse_tune_group": (i32, [vp, i32, ll, ll, ll, i32, i32, P(i32), P(C.c_float)]),
        "esparse_tune_save": (i32, [vp, C.c_char_p]),
        "esparse_tune_load": (i32, [vp, C.c_char_p]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


EXPORTED = ["esparse_create", "esparse_destroy", "esparse_set_stream", "esparse_last_error",
            "esparse_version", "esparse_channel_stats", "esparse_prune", "esparse_prune_with_scores", "esparse_output_error",
            "esparse_matrix_rate", "esparse_read_rate",
            "esparse_spmm_group_workspace", "esparse_spmm_group", "esparse_dense_gemm_group",
            "esparse_stage_activations_group", "esparse_spmm_group_staged",
            "esparse_compressed_size", "esparse_compress", "esparse_spmm_workspace", "esparse_spmm", "esparse_spmm_static",
            "esparse_stage_activations", "esparse_spmm_staged", "esparse_dense_gemm_staged",
            "esparse_spmm_num_variants", "esparse_spmm_variant_name", "esparse_dense_packed_size",
            "esparse_dense_pack", "esparse_dense_gemm", "esparse_tune", "esparse_tune_group", "esparse_tune_save",
            "esparse_tune_load"]


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float16:
        return F16
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def compressed_size(N: int, K: int, n: int, m: int, dtype: int = F16):
    lib = load_library()
    a, b, c = C.c_size_t(), C.c_size_t(), C.c_size_t()
    rc = lib.esparse_compressed_size(N, K, n, m, dtype, C.byref(a), C.byref(b), C.byref(c))
    if rc:
        raise EsparseError(rc, "esparse_compressed_size")
    return a.value, b.value, c.value


def spmm_workspace(M: int, N: int, K: int, variant: int = -1) -> int:
    lib = load_library()
    a = C.c_size_t()
    rc = lib.esparse_spmm_workspace(M, N, K, variant, C.byref(a))
    if rc:
        raise EsparseError(rc, "esparse_spmm_workspace")
    return a.value


def dense_packed_size(N: int, K: int) -> int:
    lib = load_library()
    a = C.c_size_t()
    rc = lib.esparse_dense_packed_size(N, K, C.byref(a))
    if rc:
        raise EsparseError(rc, "esparse_dense_packed_size")
    return a.value


def num_variants() -> int:
    return load_library().esparse_spmm_num_variants()


def variant_name(v: int) -> str:
    return load_library().esparse_spmm_variant_name(v).decode()


@dataclass
class PruneOpts:
    n_keep: int = 2
    m_group: int = 4
    block: int = 64
    bins: int = 100
    alpha: float = 1.0
    flags: int = USE_ALL
    max_swaps: int = 0

    def _c(self) -> _Opts:
        return _Opts(self.n_keep, self.m_group, self.block, self.bins, float(self.alpha), self.flags,
                     self.max_swaps)


@dataclass
class PruneResult:
    perm: torch.Tensor          # int32 [K] device
    mask: torch.Tensor          # uint8 [N, K] device, re-ordered channel order
    score: Optional[np.ndarray]  # float64 [K] host
    swaps: Optional[np.ndarray]  # int64 [K / block] host
    retained: Optional[float]


@dataclass
class Compressed:
    values: Optional[torch.Tensor]
    meta: Optional[torch.Tensor]
    native: Optional[torch.Tensor]  # uint8 [native_bytes]
    N: int
    K: int
    n_keep: int
    m_group: int
    dtype: int


class Context:
    """One library context bound to a device and (per call) to torch's current stream."""

    def __init__(self, device: int = 0):
        self._lib = load_library()
        self._h = C.c_void_p()
        rc = self._lib.esparse_create(C.byref(self._h), device, None)
        if rc:
            raise EsparseError(rc, "esparse_create")
        self.device = device
        self._ws = None

    def close(self):
        if self._h:
            self._lib.esparse_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- helpers ------------------------------------------------------------------------------
    def _check(self, rc: int):
        if rc:
            raise EsparseError(rc, self._lib.esparse_last_error(self._h).decode())

    def _sync_stream(self):
        if torch.cuda.is_available():
            s = torch.cuda.current_stream(self.device).cuda_stream
            self._lib.esparse_set_stream(self._h, C.c_void_p(s))

    def workspace(self, nbytes: int) -> torch.Tensor:
        if self._ws is None or self._ws.numel() < nbytes:
            self._ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=f"cuda:{self.device}")
        off = (-self._ws.data_ptr()) % 256
        return self._ws[off:off + nbytes]

    # -- Section 3.2 --------------------------------------------------------------------------
    def channel_stats(self, calib: torch.Tensor, bins: int = 100):
        T, K = calib.shape
        ir = np.empty(K, dtype=np.float64)
        am = np.empty(K, dtype=np.float64)
        self._sync_stream()
        self._check(self._lib.esparse_channel_stats(self._h, _ptr(calib), T, K, _dtype_code(calib), bins,
                                                    ir.ctypes.data_as(C.c_void_p), am.ctypes.data_as(C.c_void_p)))
        return ir, am

    # -- Section 3.2 eq. 3 + Section 3.3 ------------------------------------------------------
    def prune(self, calib: Optional[torch.Tensor], W: torch.Tensor, opts: PruneOpts, *,
              score: Optional[np.ndarray] = None, want_retained: bool = False) -> PruneResult:
        N, K = W.shape
        dev = W.device
        perm = torch.empty(K, dtype=torch.int32, device=dev)
        mask = torch.empty((N, K), dtype=torch.uint8, device=dev)
        nblk = K // opts.block if (opts.block > 0 and K % opts.block == 0) else 0
        swaps = np.zeros(max(nblk, 1), dtype=np.int64)
        retained = C.c_double(0.0)
        co = opts._c()
        self._sync_stream()
        if score is None:
            T = calib.shape[0]
            assert calib.shape[1] == K and calib.dtype == W.dtype
            s_out = np.empty(K, dtype=np.float64)
            self._check(self._lib.esparse_prune(
                self._h, _ptr(calib), T, _ptr(W), N, K, _dtype_code(W), C.byref(co), _ptr(perm), _ptr(mask),
                s_out.ctypes.data_as(C.c_void_p), swaps.ctypes.data_as(C.c_void_p),
                C.cast(C.byref(retained), C.c_void_p) if want_retained else None))
        else:
            s_out = np.ascontiguousarray(score, dtype=np.float64)
            self._check(self._lib.esparse_prune_with_scores(
                self._h, s_out.ctypes.data_as(C.c_void_p), _ptr(W), N, K, _dtype_code(W), C.byref(co), _ptr(perm),
                _ptr(mask), swaps.ctypes.data_as(C.c_void_p),
                C.cast(C.byref(retained), C.c_void_p) if want_retained else None))
        return PruneResult(perm, mask, s_out, swaps[:nblk], retained.value if want_retained else None)

    # -- Section 4, step 1 --------------------------------------------------------------------
    def compress(self, W: torch.Tensor, mask: Optional[torch.Tensor], perm: Optional[torch.Tensor],
                 n_keep: int = 2, m_group: int = 4, *, canonical: bool = True, native: bool = True) -> Compressed:
        N, K = W.shape
        dt = _dtype_code(W)
        vb, mb, nb = compressed_size(N, K, n_keep, m_group, dt)
        dev = W.device
        values = torch.empty((N, K * n_keep // m_group), dtype=W.dtype, device=dev) if canonical else None
        meta = torch.empty(mb, dtype=torch.uint8, device=dev) if canonical else None
        nat = torch.empty(nb, dtype=torch.uint8, device=dev) if native else None
        self._sync_stream()
        self._check(self._lib.esparse_compress(self._h, _ptr(W), _ptr(mask), _ptr(perm), N, K, dt, n_keep, m_group,
                                               _ptr(values), _ptr(meta), _ptr(nat)))
        return Compressed(values, meta, nat, N, K, n_keep, m_group, dt)

    # -- Section 4: products ------------------------------------------------------------------
    def spmm(self, X: torch.Tensor, comp: Compressed, perm: Optional[torch.Tensor], *, variant: int = -1,
             out: Optional[torch.Tensor] = None) -> torch.Tensor:
        M, K = X.shape
        assert K == comp.K and _dtype_code(X) == comp.dtype
        Y = out if out is not None else torch.empty((M, comp.N), dtype=X.dtype, device=X.device)
        nbytes = spmm_workspace(M, comp.N, K)
        ws = self.workspace(nbytes)
        self._sync_stream()
        self._check(self._lib.esparse_spmm(self._h, _ptr(X), M, _ptr(comp.native), _ptr(perm), comp.N, K, comp.dtype,
                                           comp.n_keep, comp.m_group, _ptr(Y), _ptr(ws), nbytes, variant))
        return Y

    def spmm_static(self, X: torch.Tensor, comp: Compressed, perm: Optional[torch.Tensor], *, variant: int = -1,
                    out: torch.Tensor) -> torch.Tensor:
        """esparse_spmm_static: the product with the library's own fixed scratch; nothing is allocated (the caller
        brings the output)."""
        M, K = X.shape
        assert K == comp.K and _dtype_code(X) == comp.dtype and tuple(out.shape) == (M, comp.N)
        self._sync_stream()
        self._check(self._lib.esparse_spmm_static(self._h, _ptr(X), M, _ptr(comp.native), _ptr(perm), comp.N, K, comp.dtype,
                                                  comp.n_keep, comp.m_group, _ptr(out), variant))
        return out

    def spmm_group(self, Xs, comps, perms, *, variant: int = -1, outs=None):
        """Products of one shape (same M, N, K, dtype, n:m) through one staging and one multiply launch
        where a decode kernel serves the shape; returns the list of outputs."""
        count = len(comps)
        assert len(Xs) == count and (perms is None or len(perms) == count)
        M, K = Xs[0].shape
        c0 = comps[0]
        for X, c in zip(Xs, comps):
            assert tuple(X.shape) == (M, K) and (c.N, c.K, c.dtype, c.n_keep, c.m_group) == (c0.N, K, c0.dtype, c0.n_keep, c0.m_group)
            assert _dtype_code(X) == c0.dtype
        if outs is None:
            outs = [torch.empty((M, c0.N), dtype=Xs[0].dtype, device=Xs[0].device) for _ in range(count)]
        nbytes = C.c_size_t(0)
        rc = self._lib.esparse_spmm_group_workspace(count, M, c0.N, K, C.byref(nbytes))
        if rc:
            raise EsparseError(rc, "esparse_spmm_group_workspace: bad arguments")
        ws = self.workspace(nbytes.value)
        arr = C.c_void_p * count
        xs = arr(*[_ptr(x) for x in Xs])
        wsn = arr(*[_ptr(c.native) for c in comps])
        ps = arr(*[_ptr(p) for p in perms]) if perms is not None else None
        ys = arr(*[_ptr(y) for y in outs])
        self._sync_stream()
        self._check(self._lib.esparse_spmm_group(self._h, count, xs, M, wsn, ps, c0.N, K, c0.dtype, c0.n_keep, c0.m_group, ys,
                                                 _ptr(ws), nbytes.value, variant))
        return outs

    def stage_activations_group(self, Xs, perms, comp0: Compressed, ws: torch.Tensor, *, variant: int = -1):
        count = len(Xs)
        M, K = Xs[0].shape
        arr = C.c_void_p * count
        ps = arr(*[_ptr(p) for p in perms]) if perms is not None else None
        self._sync_stream()
        self._check(self._lib.esparse_stage_activations_group(self._h, count, arr(*[_ptr(x) for x in Xs]), M, ps, comp0.N, K,
                                                              comp0.dtype, comp0.n_keep, comp0.m_group, _ptr(ws), ws.numel(), variant))

    def spmm_group_staged(self, M: int, comps, ws: torch.Tensor, outs, *, variant: int = -1):
        count = len(comps)
        c0 = comps[0]
        arr = C.c_void_p * count
        self._sync_stream()
        self._check(self._lib.esparse_spmm_group_staged(self._h, count, M, arr(*[_ptr(c.native) for c in comps]), c0.N, c0.K,
                                                        c0.dtype, c0.n_keep, c0.m_group, arr(*[_ptr(y) for y in outs]), _ptr(ws),
                                                        ws.numel(), variant))
        return outs

    def dense_gemm_group(self, Xs, packed, N: int, *, variant: int = -1, outs=None):
        count = len(packed)
        M, K = Xs[0].shape
        if outs is None:
            outs = [torch.empty((M, N), dtype=Xs[0].dtype, device=Xs[0].device) for _ in range(count)]
        nbytes = C.c_size_t(0)
        rc = self._lib.esparse_spmm_group_workspace(count, M, N, K, C.byref(nbytes))
        if rc:
            raise EsparseError(rc, "esparse_spmm_group_workspace: bad arguments")
        ws = self.workspace(nbytes.value)
        arr = C.c_void_p * count
        self._sync_stream()
        self._check(self._lib.esparse_dense_gemm_group(self._h, count, arr(*[_ptr(x) for x in Xs]), M, arr(*[_ptr(w) for w in packed]),
                                                       N, K, _dtype_code(Xs[0]), arr(*[_ptr(y) for y in outs]), _ptr(ws), nbytes.value,
                                                       variant))
        return outs

    def stage_activations(self, X: torch.Tensor, perm: Optional[torch.Tensor], N: int,
                          ws: Optional[torch.Tensor] = None) -> torch.Tensor:
        M, K = X.shape
        nbytes = spmm_workspace(M, N, K)
        if ws is None:
            ws = self.workspace(nbytes)
        self._sync_stream()
        self._check(self._lib.esparse_stage_activations(self._h, _ptr(X), M, _ptr(perm), N, K, _dtype_code(X),
                                                        _ptr(ws), ws.numel()))
        return ws

    def spmm_staged(self, M: int, comp: Compressed, ws: torch.Tensor, Y: torch.Tensor, *, variant: int = -1):
        self._sync_stream()
        self._check(self._lib.esparse_spmm_staged(self._h, M, _ptr(comp.native), comp.N, comp.K, comp.dtype,
                                                  comp.n_keep, comp.m_group, _ptr(Y), _ptr(ws), ws.numel(), variant))
        return Y

    def dense_gemm_staged(self, M: int, packed: torch.Tensor, N: int, K: int, ws: torch.Tensor, Y: torch.Tensor, *,
                          variant: int = -1):
        self._sync_stream()
        self._check(self._lib.esparse_dense_gemm_staged(self._h, M, _ptr(packed), N, K, _dtype_code(Y), _ptr(Y),
                                                        _ptr(ws), ws.numel(), variant))
        return Y

    def dense_pack(self, W: torch.Tensor) -> torch.Tensor:
        N, K = W.shape
        packed = torch.empty(dense_packed_size(N, K), dtype=torch.uint8, device=W.device)
        self._sync_stream()
        self._check(self._lib.esparse_dense_pack(self._h, _ptr(W), N, K, _dtype_code(W), _ptr(packed)))
        return packed

    def dense_gemm(self, X: torch.Tensor, packed: torch.Tensor, N: int, *, variant: int = -1,
                   out: Optional[torch.Tensor] = None) -> torch.Tensor:
        M, K = X.shape
        Y = out if out is not None else torch.empty((M, N), dtype=X.dtype, device=X.device)
        nbytes = spmm_workspace(M, N, K)
        ws = self.workspace(nbytes)
        self._sync_stream()
        self._check(self._lib.esparse_dense_gemm(self._h, _ptr(X), M, _ptr(packed), N, K, _dtype_code(X), _ptr(Y),
                                                 _ptr(ws), nbytes, variant))
        return Y

    # -- Section 4, step 2 --------------------------------------------------------------------
    # -- Section 3.3 eq. 4 --------------------------------------------------------------------
    def output_error(self, Yref: torch.Tensor, Y: torch.Tensor):
        """(|| Yref - Y ||_F^2, || Yref ||_F^2) of two outputs of the same shape."""
        assert Yref.shape == Y.shape and Yref.dtype == Y.dtype and Yref.is_contiguous() and Y.is_contiguous()
        M, N = Yref.shape
        num, den = C.c_double(0.0), C.c_double(0.0)
        self._sync_stream()
        self._check(self._lib.esparse_output_error(self._h, _ptr(Yref), _ptr(Y), M, N, _dtype_code(Y),
                                                   C.cast(C.byref(num), C.c_void_p), C.cast(C.byref(den), C.c_void_p)))
        return num.value, den.value

    # -- measurement aid ------------------------------------------------------------------------
    def matrix_rate(self, sparse: bool = True, dtype: int = F16, random_operands: bool = True, mix: int = 0) -> float:
        """Effective TFLOP/s the matrix pipes sustain: mix 0 = operands held in registers, 1 = + a prefill stage's operand
        reads out of LDS, 2 = + its DMA, counted wait and barrier (L2-resident source)."""
        t = C.c_double(0.0)
        self._sync_stream()
        self._check(self._lib.esparse_matrix_rate(self._h, int(bool(sparse)), dtype, int(bool(random_operands)), mix, C.byref(t)))
        return t.value

    def read_rate(self, nbytes: int) -> float:
        """GB/s of a plain streaming read of nbytes per launch, cold (the launches walk through more than the caches hold)."""
        t = C.c_double(0.0)
        self._sync_stream()
        self._check(self._lib.esparse_read_rate(self._h, int(nbytes), C.byref(t)))
        return t.value

    def tune(self, M: int, N: int, K: int, dtype: int = F16, sparse=True):
        """sparse: False / 0 = dense, True / 1 = 2:4, 2 = 4:8."""
        best, ms = C.c_int(-1), C.c_float(0.0)
        self._sync_stream()
        self._check(self._lib.esparse_tune(self._h, M, N, K, dtype, int(sparse), C.byref(best), C.byref(ms)))
        return best.value, ms.value

    def tune_group(self, count: int, M: int, N: int, K: int, dtype: int = F16, sparse=True):
        """The same search for launches of `count` products of one shape (spmm_group, dense_gemm_group)."""
        best, ms = C.c_int(-1), C.c_float(0.0)
        self._sync_stream()
        self._check(self._lib.esparse_tune_group(self._h, count, M, N, K, dtype, int(sparse), C.byref(best), C.byref(ms)))
        return best.value, ms.value

    def tune_save(self, path: str):
        self._check(self._lib.esparse_tune_save(self._h, path.encode()))

    def tune_load(self, path: str):
        self._check(self._lib.esparse_tune_load(self._h, path.encode()))
