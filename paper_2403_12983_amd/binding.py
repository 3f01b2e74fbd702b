"""ctypes binding of include/osscar.h.  Argument marshalling only: every step of the path runs in the
HIP library.  PyTorch supplies device memory (tensors) and the stream; nothing here computes."""
from __future__ import annotations

import ctypes as C
import os
from typing import Tuple, Optional, Sequence

import numpy as np
import torch

OSSCAR_F32, OSSCAR_BF16 = 0, 1
OSSCAR_INIT_MAGNITUDE, OSSCAR_INIT_GIVEN = 0, 1
OSSCAR_SEARCH_ALWAYS_ACCEPT = 1
OSSCAR_SEARCH_EAGER = 2
OSSCAR_SEARCH_NO_LOOKAHEAD = 4
OSSCAR_SEARCH_EXACT_IN = 8
T_H, T_G, T_P, T_B, T_V, T_R, T_REM, T_ADD, T_KEPT, T_CAND = range(10)
_STATUS = {0: "OK", 1: "EINVAL", 2: "ENOMEM", 3: "ENOTPD", 4: "EHIP", 5: "ESTATE"}

EXPORTED_SYMBOLS = ["osscar_workspace_bytes", "osscar_create", "osscar_destroy", "osscar_gram", "osscar_gram_target", "osscar_gram_conv",
                    "osscar_set_quadratic",
                    "osscar_init_support", "osscar_init_greedy", "osscar_local_search", "osscar_block_search", "osscar_apply_swap", "osscar_backsolve",
                    "osscar_get_tensor", "osscar_get_scalars", "osscar_get_timers", "osscar_get_counters", "osscar_debug_tile_schedule",
                    "osscar_debug_gemm_log", "osscar_debug_gemm_log_read", "osscar_debug_int_products", "osscar_debug_refined_inverse", "osscar_debug_side_stream",
                    "osscar_gram_static", "osscar_last_error"]


class OsscarError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"osscar status {_STATUS.get(status, status)}: {message}")
        self.status = status


class _Desc(C.Structure):
    _fields_ = [("d1", C.c_int64), ("m", C.c_int64), ("p", C.c_int32), ("q", C.c_int32), ("k", C.c_int32),
                ("max_swaps", C.c_int32), ("x_dtype", C.c_int32), ("w_dtype", C.c_int32), ("from_dense", C.c_int32),
                ("target_output", C.c_int32)]


class _SearchResult(C.Structure):
    _fields_ = [("iters", C.c_int32), ("accepted", C.c_int32), ("obj_initial", C.c_double), ("obj_final", C.c_double)]


def lib_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libosscar.so")


_LIB = None


def load_library():
    """Loads libosscar.so; raises if it has not been built (there is no fallback path)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: build it with `python -m paper_2403_12983_amd.build` "
                                "(or __graft_entry__.build()); this package has no CPU fallback")
    lib = C.CDLL(path)
    vp, i64, i32, dbl = C.c_void_p, C.c_int64, C.c_int32, C.c_double
    lib.osscar_workspace_bytes.restype = C.c_size_t
    lib.osscar_workspace_bytes.argtypes = [C.POINTER(_Desc)]
    lib.osscar_create.argtypes = [C.POINTER(vp), C.POINTER(_Desc), vp, C.c_size_t, vp]
    lib.osscar_destroy.argtypes = [vp]
    lib.osscar_gram.argtypes = [vp, vp, i64, i64, C.c_int, vp, i64, dbl, dbl]
    lib.osscar_gram_conv.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, C.c_int, vp, i64, dbl, dbl]
    lib.osscar_gram_target.argtypes = [vp, vp, vp, i64, i64, i64, C.c_int, vp, i64, dbl, dbl]
    lib.osscar_set_quadratic.argtypes = [vp, vp, vp, dbl, C.POINTER(dbl)]
    lib.osscar_init_support.argtypes = [vp, C.c_int, C.POINTER(i32), C.POINTER(dbl)]
    lib.osscar_init_greedy.argtypes = [vp, i32, i32, C.c_uint32, C.POINTER(i32), C.POINTER(C.c_float), C.POINTER(dbl)]
    lib.osscar_local_search.argtypes = [vp, i32, dbl, C.c_uint32, i32, C.POINTER(_SearchResult), C.POINTER(i32),
                                        C.POINTER(i32), C.POINTER(C.c_float), C.POINTER(dbl)]
    lib.osscar_block_search.argtypes = [vp, i32, i32, dbl, C.c_uint32, C.POINTER(_SearchResult), C.POINTER(i32), C.POINTER(i32),
                                        C.POINTER(C.c_float), C.POINTER(dbl)]
    lib.osscar_apply_swap.argtypes = [vp, i32, i32]
    lib.osscar_backsolve.argtypes = [vp, vp, i64, i32, C.POINTER(i32), C.POINTER(dbl)]
    lib.osscar_get_tensor.argtypes = [vp, C.c_int, vp, C.c_size_t]
    lib.osscar_get_scalars.argtypes = [vp, C.POINTER(dbl), C.POINTER(dbl)]
    lib.osscar_get_timers.argtypes = [vp, C.POINTER(dbl)]
    lib.osscar_get_counters.argtypes = [vp, C.POINTER(i64)]
    lib.osscar_debug_gemm_log.argtypes = [i32]
    lib.osscar_debug_int_products.argtypes = [i32]
    lib.osscar_debug_refined_inverse.argtypes = [i32]
    lib.osscar_debug_side_stream.argtypes = [i32]
    lib.osscar_debug_gemm_log_read.restype = C.c_int32
    lib.osscar_debug_gemm_log_read.argtypes = [C.POINTER(dbl), i32]
    lib.osscar_gram_static.argtypes = [vp, i64, i64, i32, vp, i64, i32, i64, i64, dbl, dbl, vp, vp, vp, vp]
    lib.osscar_debug_tile_schedule.restype = C.c_int32
    lib.osscar_debug_tile_schedule.argtypes = [i64, C.POINTER(i32), i32]
    lib.osscar_last_error.restype = C.c_char_p
    lib.osscar_last_error.argtypes = [vp]
    for name in EXPORTED_SYMBOLS:
        if name not in ("osscar_workspace_bytes", "osscar_last_error", "osscar_debug_tile_schedule", "osscar_debug_gemm_log_read"):
            getattr(lib, name).restype = C.c_int
    _LIB = lib
    return lib


def _dtype_code(t: torch.dtype) -> int:
    if t == torch.float32:
        return OSSCAR_F32
    if t == torch.bfloat16:
        return OSSCAR_BF16
    raise TypeError(f"unsupported dtype {t}")


class Solver:
    """One layer's context: owns the workspace tensor and forwards every call to the C library."""

    def __init__(self, d1: int, m: int, p: int, q: int, k: int, max_swaps: int, x_dtype=torch.bfloat16,
                 w_dtype=torch.bfloat16, device="cuda:0", stream: Optional[torch.cuda.Stream] = None,
                 from_dense: bool = False, target_output: bool = False):
        self.lib = load_library()
        self.device = torch.device(device)
        self.d1, self.m, self.p, self.q, self.k = d1, m, p, q, k
        self.kr, self.cr = k * q, d1 - k * q
        self.max_swaps = max_swaps
        self.desc = _Desc(d1, m, p, q, k, max_swaps, _dtype_code(x_dtype), _dtype_code(w_dtype), int(from_dense), int(target_output))
        nbytes = self.lib.osscar_workspace_bytes(C.byref(self.desc))
        if nbytes == 0:
            raise OsscarError(1, "invalid problem description")
        self.workspace_bytes = nbytes
        with torch.cuda.device(self.device):
            self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
            self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        base = self.workspace.data_ptr()
        self._ws_ptr = (base + 255) // 256 * 256
        self.ctx = C.c_void_p()
        st = self.lib.osscar_create(C.byref(self.ctx), C.byref(self.desc), C.c_void_p(self._ws_ptr), C.c_size_t(nbytes),
                                    C.c_void_p(self.stream.cuda_stream))
        if st != 0:
            self.ctx = None
            raise OsscarError(st, "osscar_create failed")

    # -- helpers
    def _check(self, st: int):
        if st != 0:
            raise OsscarError(st, self.lib.osscar_last_error(self.ctx).decode())

    def close(self):
        if getattr(self, "ctx", None):
            self.lib.osscar_destroy(self.ctx)
            self.ctx = None
        self.workspace = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the calls of include/osscar.h
    def osscar_gram(self, Xc: Optional[torch.Tensor], finalize: bool = False, W: Optional[torch.Tensor] = None,
                    lambda_abs: float = 0.0, lambda_rel: float = 0.0):
        xp, n_c, ldx = None, 0, self.d1
        if Xc is not None and Xc.shape[0] > 0:
            assert Xc.is_cuda and Xc.dim() == 2 and Xc.shape[1] == self.d1 and Xc.stride(1) == 1
            assert _dtype_code(Xc.dtype) == self.desc.x_dtype
            xp, n_c, ldx = Xc.data_ptr(), Xc.shape[0], Xc.stride(0)
        wp, ldw = None, self.m
        if finalize:
            assert W is not None and W.is_cuda and W.shape == (self.d1, self.m) and W.stride(1) == 1
            assert _dtype_code(W.dtype) == self.desc.w_dtype
            wp, ldw = W.data_ptr(), W.stride(0)
        self._check(self.lib.osscar_gram(self.ctx, xp, n_c, ldx, int(finalize), wp, ldw, lambda_abs, lambda_rel))

    def osscar_gram_conv(self, F: Optional[torch.Tensor], kh: int, kw: int, stride: int = 1, pad: int = 0, finalize: bool = False,
                         W: Optional[torch.Tensor] = None, lambda_abs: float = 0.0, lambda_rel: float = 0.0,
                         shape: Optional[Tuple[int, int, int]] = None):
        """F: (batch, channels, h_in, w_in) contiguous, or None with shape = (channels, h_in, w_in) for an empty finalize."""
        fp, batch = None, 0
        if F is not None:
            assert F.is_cuda and F.dim() == 4 and F.is_contiguous() and _dtype_code(F.dtype) == self.desc.x_dtype
            batch, ch, h_in, w_in = F.shape
            fp = F.data_ptr() if batch > 0 else None
        else:
            ch, h_in, w_in = shape
        wp, ldw = None, self.m
        if finalize:
            assert W is not None and W.is_cuda and W.shape == (self.d1, self.m) and W.stride(1) == 1
            assert _dtype_code(W.dtype) == self.desc.w_dtype
            wp, ldw = W.data_ptr(), W.stride(0)
        self._check(self.lib.osscar_gram_conv(self.ctx, fp, batch, ch, h_in, w_in, kh, kw, stride, pad, int(finalize), wp, ldw,
                                              lambda_abs, lambda_rel))

    def osscar_gram_target(self, Xc: Optional[torch.Tensor], Yc: Optional[torch.Tensor], finalize: bool = False,
                           W: Optional[torch.Tensor] = None, lambda_abs: float = 0.0, lambda_rel: float = 0.0):
        xp, yp, n_c, ldx, ldy = None, None, 0, self.d1, self.m
        if Xc is not None and Xc.shape[0] > 0:
            assert Xc.is_cuda and Xc.dim() == 2 and Xc.shape[1] == self.d1 and Xc.stride(1) == 1
            assert Yc is not None and Yc.is_cuda and Yc.shape == (Xc.shape[0], self.m) and Yc.stride(1) == 1
            assert _dtype_code(Xc.dtype) == self.desc.x_dtype and Yc.dtype == Xc.dtype
            xp, yp, n_c, ldx, ldy = Xc.data_ptr(), Yc.data_ptr(), Xc.shape[0], Xc.stride(0), Yc.stride(0)
        wp, ldw = None, self.m
        if finalize:
            assert W is not None and W.is_cuda and W.shape == (self.d1, self.m) and W.stride(1) == 1
            assert _dtype_code(W.dtype) == self.desc.w_dtype
            wp, ldw = W.data_ptr(), W.stride(0)
        self._check(self.lib.osscar_gram_target(self.ctx, xp, yp, n_c, ldx, ldy, int(finalize), wp, ldw, lambda_abs, lambda_rel))

    def osscar_set_quadratic(self, H: torch.Tensor, G: torch.Tensor, c0: float, group_norms: Sequence[float]):
        assert H.is_cuda and H.dtype == torch.float32 and H.is_contiguous() and H.shape == (self.d1, self.d1)
        assert G.is_cuda and G.dtype == torch.float32 and G.is_contiguous() and G.shape == (self.d1, self.m)
        norms = (C.c_double * self.p)(*[float(v) for v in group_norms])
        self._check(self.lib.osscar_set_quadratic(self.ctx, H.data_ptr(), G.data_ptr(), float(c0), norms))

    def osscar_init_support(self, mode: int = OSSCAR_INIT_MAGNITUDE, groups: Optional[Sequence[int]] = None) -> float:
        obj = C.c_double()
        arr = None
        if groups is not None:
            arr = (C.c_int32 * len(groups))(*[int(g) for g in groups])
            assert len(groups) == self.k
        self._check(self.lib.osscar_init_support(self.ctx, mode, arr, C.byref(obj)))
        return obj.value

    def osscar_init_greedy(self, t_hat: int, refresh_every: int = 0, flags: int = 0):
        """Returns (objective, per-iteration lists of removed groups, per-iteration gaps)."""
        obj = C.c_double()
        nrem = self.p - self.k
        iters = (nrem + t_hat - 1) // t_hat if t_hat > 0 else 0
        removed = np.full(max(nrem, 1), -1, dtype=np.int32)
        gaps = np.zeros(max(iters, 1), dtype=np.float32)
        self._check(self.lib.osscar_init_greedy(self.ctx, t_hat, refresh_every, flags, removed.ctypes.data_as(C.POINTER(C.c_int32)),
                                                gaps.ctypes.data_as(C.POINTER(C.c_float)), C.byref(obj)))
        steps = [removed[i * t_hat:min((i + 1) * t_hat, nrem)].tolist() for i in range(iters)]
        return obj.value, steps, gaps[:iters].copy()

    def osscar_local_search(self, max_swaps: int, rel_tol: float = 0.0, flags: int = 0, refresh_every: int = 0):
        res = _SearchResult()
        n = max(max_swaps, 1)
        t_out = np.full(n, -1, dtype=np.int32)
        t_in = np.full(n, -1, dtype=np.int32)
        t_gap = np.zeros(2 * n, dtype=np.float32)
        t_obj = np.zeros(n, dtype=np.float64)
        self._check(self.lib.osscar_local_search(
            self.ctx, max_swaps, rel_tol, flags, refresh_every, C.byref(res),
            t_out.ctypes.data_as(C.POINTER(C.c_int32)), t_in.ctypes.data_as(C.POINTER(C.c_int32)),
            t_gap.ctypes.data_as(C.POINTER(C.c_float)), t_obj.ctypes.data_as(C.POINTER(C.c_double))))
        it = res.iters
        return dict(iters=it, accepted=res.accepted, obj_initial=res.obj_initial, obj_final=res.obj_final,
                    trace_out=t_out[:it].copy(), trace_in=t_in[:it].copy(), trace_gap=t_gap[:2 * it].reshape(-1, 2).copy(),
                    trace_obj=t_obj[:it].copy())

    def osscar_block_search(self, max_iters: int, block: int, rel_tol: float = 0.0, flags: int = 0):
        res = _SearchResult()
        n = max(max_iters, 1)
        t_out = np.full(n * block, -1, dtype=np.int32)
        t_in = np.full(n * block, -1, dtype=np.int32)
        t_gap = np.zeros(2 * n, dtype=np.float32)
        t_obj = np.zeros(n, dtype=np.float64)
        self._check(self.lib.osscar_block_search(
            self.ctx, max_iters, block, rel_tol, flags, C.byref(res),
            t_out.ctypes.data_as(C.POINTER(C.c_int32)), t_in.ctypes.data_as(C.POINTER(C.c_int32)),
            t_gap.ctypes.data_as(C.POINTER(C.c_float)), t_obj.ctypes.data_as(C.POINTER(C.c_double))))
        it = res.iters
        moves = [([g for g in t_out[i * block:(i + 1) * block].tolist() if g >= 0],
                  [g for g in t_in[i * block:(i + 1) * block].tolist() if g >= 0]) for i in range(it)]
        return dict(iters=it, accepted=res.accepted, obj_initial=res.obj_initial, obj_final=res.obj_final, moves=moves,
                    trace_gap=t_gap[:2 * it].reshape(it, 2).copy(), trace_obj=t_obj[:it].copy())

    def osscar_apply_swap(self, g_out: int, g_in: int):
        self._check(self.lib.osscar_apply_swap(self.ctx, int(g_out), int(g_in)))

    def osscar_backsolve(self, out_dtype=torch.float32):
        What = torch.empty(self.d1, self.m, dtype=out_dtype, device=self.device)
        support = np.zeros(self.k, dtype=np.int32)
        obj = C.c_double()
        self._check(self.lib.osscar_backsolve(self.ctx, What.data_ptr(), self.m, _dtype_code(out_dtype),
                                              support.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(obj)))
        return What, support, obj.value

    def osscar_get_tensor(self, which: int) -> torch.Tensor:
        kr, cr, d1, m, p = self.kr, self.cr, self.d1, self.m, self.p
        shape, dt = {T_H: ((d1, d1), torch.float32), T_G: ((d1, m), torch.float32), T_P: ((kr, kr), torch.float32),
                     T_B: ((kr, m), torch.float32), T_V: ((kr, cr), torch.float32), T_R: ((cr, m), torch.float32),
                     T_REM: ((p,), torch.float64), T_ADD: ((p,), torch.float64), T_KEPT: ((self.k,), torch.int32),
                     T_CAND: ((p - self.k,), torch.int32)}[which]
        out = torch.empty(shape, dtype=dt, device=self.device)
        self._check(self.lib.osscar_get_tensor(self.ctx, which, out.data_ptr(), out.numel() * out.element_size()))
        return out

    def osscar_get_scalars(self):
        lam, c0 = C.c_double(), C.c_double()
        self._check(self.lib.osscar_get_scalars(self.ctx, C.byref(lam), C.byref(c0)))
        return lam.value, c0.value

    def osscar_get_timers(self):
        arr = (C.c_double * 16)()
        self._check(self.lib.osscar_get_timers(self.ctx, arr))
        return list(arr)

    def osscar_get_counters(self):
        arr = (C.c_int64 * 8)()
        self._check(self.lib.osscar_get_counters(self.ctx, arr))
        return dict(flushes=arr[0], pauses=arr[1], lookahead_misses=arr[2], iters=arr[3])


def gemm_log(enable: bool):
    """Switches the library's log of its matrix-product launches on (cleared first) or off."""
    load_library().osscar_debug_gemm_log(1 if enable else 0)


def i8_products(enable: bool):
    """Large float64-accurate products on the int8 matrix cores (default) or on the float64-accumulating kernel."""
    load_library().osscar_debug_int_products(1 if enable else 0)


def refined_inverse(enable: bool):
    """The inverse by the float32 sweep + Newton-Schulz (True) instead of the float64-storage sweep (False, the default)."""
    load_library().osscar_debug_refined_inverse(1 if enable else 0)


def side_stream(enable: bool):
    """The library's second stream (overlap inside the inverse and the flush; the default) on or off."""
    load_library().osscar_debug_side_stream(1 if enable else 0)


def gemm_log_read(capacity: int = 16384) -> np.ndarray:
    """Rows of (M, N, K, kind, ms) for every matrix-product launch since the log was switched on."""
    buf = np.zeros((capacity, 5), dtype=np.float64)
    n = load_library().osscar_debug_gemm_log_read(buf.ctypes.data_as(C.POINTER(C.c_double)), capacity)
    return buf[:max(n, 0)].copy()


def osscar_gram_static(X: torch.Tensor, W: torch.Tensor, H: torch.Tensor, G: torch.Tensor, scalars: torch.Tensor,
                       lambda_abs: float = 0.0, lambda_rel: float = 0.0, stream: Optional[torch.cuda.Stream] = None):
    """The allocation-free Gram of one small layer: X (n x d1), W (d1 x m) in; H (d1 x d1 float32), G (d1 x m float32) and
    scalars (2 float64: lambda, c0) out, all device tensors the caller made.  Enqueues on `stream` and does not wait."""
    lib = load_library()
    assert X.is_cuda and W.is_cuda and X.dim() == 2 and W.dim() == 2 and X.stride(1) == 1 and W.stride(1) == 1
    d1, m = W.shape
    assert X.shape[1] == d1
    assert H.is_cuda and H.dtype == torch.float32 and H.is_contiguous() and tuple(H.shape) == (d1, d1)
    assert G.is_cuda and G.dtype == torch.float32 and G.is_contiguous() and tuple(G.shape) == (d1, m)
    assert scalars.is_cuda and scalars.dtype == torch.float64 and scalars.is_contiguous() and scalars.numel() >= 2
    st = stream if stream is not None else torch.cuda.current_stream(X.device)
    n = X.shape[0]
    with torch.cuda.device(X.device):
        rc = lib.osscar_gram_static(X.data_ptr() if n > 0 else None, n, X.stride(0) if n > 0 else d1, _dtype_code(X.dtype), W.data_ptr(),
                                    W.stride(0), _dtype_code(W.dtype), d1, m, float(lambda_abs), float(lambda_rel), H.data_ptr(),
                                    G.data_ptr(), scalars.data_ptr(), C.c_void_p(st.cuda_stream))
    if rc != 0:
        raise OsscarError(rc, lib.osscar_last_error(None).decode())
