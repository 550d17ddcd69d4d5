"""ctypes binding of libslim.so: one Python method per C entry point, same names, argument
marshalling only.  PyTorch supplies device memory and the HIP stream; every step of the pass runs
in the library's kernels.  There is no fallback: if the library is missing, `load()` raises."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libslim.so")

SLIM_OK = 0
ERR_INVALID_ARG, ERR_NOT_PD, ERR_ALLOC, ERR_HIP, ERR_UNSUPPORTED = -1, -2, -3, -4, -5
F16, BF16, F32, F64 = 0, 1, 2, 3
WEIGHT_MASK_MEAN, WEIGHT_UNIFORM, WEIGHT_ELEMENT = 0, 1, 2
Q1_SIGN, Q1_AFFINE = 0, 1
SCOPE_BLOCK, SCOPE_ROW = 0, 1
SAL_HINV_DIAG, SAL_CHOL_DIAG = 0, 1
OBJ_KL, OBJ_MSE = 0, 1

_DT = {torch.float16: F16, torch.bfloat16: BF16, torch.float32: F32, torch.float64: F64}

# every symbol include/slim.h declares
EXPORTS = [
    "slim_default_params", "slim_default_tau", "slim_create", "slim_destroy", "slim_last_error",
    "slim_workspace_bytes", "slim_workspace_query", "slim_hessian_accumulate", "slim_hessian_inverse", "slim_salience",
    "slim_sba_allocate", "slim_sba_prepare", "slim_sqc_calibrate", "slim_gptq_quantize", "slim_pack", "slim_dequant_matmul",
    "slim_dequant_matmul_noalloc", "slim_dequant_matmul_zp", "slim_pack_zeros", "slim_unpack_zeros", "slim_lwc_quantize",
    "slim_profile_enable", "slim_profile_collect", "slim_profile_entry", "slim_profile_reset",
]


class SlimParams(ctypes.Structure):
    _fields_ = [("sqc_weight_mode", ctypes.c_int), ("mask_scope", ctypes.c_int),
                ("q1_mode", ctypes.c_int), ("sal_mode", ctypes.c_int)]


class SlimShape(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int), ("m", ctypes.c_int), ("beta", ctypes.c_int), ("t_c", ctypes.c_int64),
                ("t_s", ctypes.c_int64), ("t_x", ctypes.c_int), ("lwc_steps", ctypes.c_int)]


def workspace_query(n: int, m: int, beta: int, t_c: int = 0, t_s: int = 0, t_x: int = 0, num_cus: int = 0,
                    lwc_steps: int = 0) -> int:
    """Bytes of workspace the entry points need for a layer of this shape (host only, no GPU needed)."""
    return int(load().slim_workspace_query(ctypes.byref(SlimShape(n, m, beta, t_c, t_s, t_x, lwc_steps)), num_cus))


def zero_bits_for(N: int) -> int:
    """Width of a packed zero point (the stored value is 2 z) for a layer of target width N (App. B.2)."""
    return int(N) + 2


def bit_base_for(N: int) -> int:
    """The width that the 2-bit group value 0 of the stored form stands for, for a layer of target width N (App. B.2):
    1 for the targets 2 and 3, N - 2 above them, so that N - 1, N, N + 1 always fit the four values."""
    return max(1, int(N) - 2)


class SlimError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("libslim status %d: %s" % (status, message))
        self.status = status


_lib = None


def load() -> ctypes.CDLL:
    """Loads the built library; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s is missing: build it with `python -m paper_2405_14917_amd.build`" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    c_void_p, c_int, c_i64, c_double = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_double
    P = ctypes.POINTER
    lib.slim_default_params.argtypes = [P(SlimParams)]
    lib.slim_default_params.restype = None
    lib.slim_default_tau.argtypes = [P(c_double), c_int]
    lib.slim_default_tau.restype = c_int
    lib.slim_create.argtypes = [P(c_void_p), c_void_p, c_void_p, ctypes.c_size_t]
    lib.slim_workspace_query.argtypes = [P(SlimShape), c_int]
    lib.slim_workspace_query.restype = ctypes.c_size_t
    lib.slim_destroy.argtypes = [c_void_p]
    lib.slim_last_error.argtypes = [c_void_p]
    lib.slim_last_error.restype = ctypes.c_char_p
    lib.slim_workspace_bytes.argtypes = [c_void_p]
    lib.slim_workspace_bytes.restype = ctypes.c_size_t
    lib.slim_hessian_accumulate.argtypes = [c_void_p, c_void_p, c_int, c_int, c_i64, c_i64, c_void_p, c_i64, P(c_i64)]
    lib.slim_hessian_inverse.argtypes = [c_void_p, c_void_p, c_i64, c_int, c_i64, c_double, c_void_p, c_i64,
                                         c_void_p, P(c_int)]
    lib.slim_salience.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_i64, c_void_p, c_i64, c_void_p, c_int,
                                  c_int, c_void_p, c_void_p, c_void_p]
    lib.slim_sba_allocate.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_i64, c_void_p, c_int, c_int, c_int,
                                      c_void_p, c_int, c_i64, c_i64, P(SlimParams), c_void_p, P(c_int), P(c_double)]
    lib.slim_sba_prepare.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_i64, c_int, c_int, c_int, c_void_p,
                                     c_int, c_i64, c_i64, P(SlimParams)]
    lib.slim_sqc_calibrate.argtypes = [c_void_p, c_void_p, c_i64, c_int, c_int, c_int, c_void_p, c_void_p,
                                       P(SlimParams), c_void_p, c_int, c_void_p, c_void_p, c_void_p]
    lib.slim_gptq_quantize.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_i64, c_void_p, c_i64, c_void_p,
                                       c_int, c_int, P(SlimParams), c_void_p, c_void_p, c_int, c_void_p, c_void_p,
                                       c_void_p, c_void_p, c_int, c_void_p]
    lib.slim_dequant_matmul.argtypes = [c_void_p, c_void_p, c_i64, c_void_p, c_void_p, c_void_p, c_void_p, c_int,
                                        c_int, c_int, c_int, c_void_p, c_int, c_int, c_i64, c_void_p, c_i64]
    lib.slim_dequant_matmul_noalloc.argtypes = lib.slim_dequant_matmul.argtypes
    lib.slim_dequant_matmul_zp.argtypes = [c_void_p, c_void_p, c_i64, c_void_p, c_void_p, c_void_p, c_void_p, c_i64, c_int,
                                           c_int, c_int, c_int, c_int, c_void_p, c_int, c_int, c_i64, c_void_p, c_i64]
    lib.slim_pack.argtypes = [c_void_p, c_void_p, c_int, c_int, c_i64, c_void_p, c_int, c_int, c_void_p, c_i64,
                              c_void_p, c_void_p, P(c_int)]
    lib.slim_pack_zeros.argtypes = [c_void_p, c_void_p, c_int, c_int, c_i64, c_int, c_void_p, c_i64, P(c_int)]
    lib.slim_unpack_zeros.argtypes = [c_void_p, c_void_p, c_i64, c_int, c_int, c_int, c_void_p, c_i64]
    lib.slim_lwc_quantize.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_i64, c_void_p, c_i64, c_i64, c_void_p,
                                      c_int, c_int, c_double, c_double, c_double, c_double, c_double, c_void_p, c_void_p,
                                      c_void_p, c_void_p, c_int, P(c_double)]
    lib.slim_profile_enable.argtypes = [c_void_p, c_int]
    lib.slim_profile_collect.argtypes = [c_void_p]
    lib.slim_profile_collect.restype = c_int
    lib.slim_profile_entry.argtypes = [c_void_p, c_int, P(ctypes.c_char_p), P(c_double), P(c_int)]
    lib.slim_profile_reset.argtypes = [c_void_p]
    for name in EXPORTS:
        fn = getattr(lib, name)
        if name not in ("slim_default_params", "slim_default_tau", "slim_last_error", "slim_workspace_bytes",
                        "slim_workspace_query", "slim_profile_collect"):
            fn.restype = c_int
    _lib = lib
    return lib


def default_tau() -> np.ndarray:
    lib = load()
    n = lib.slim_default_tau(None, 0)
    buf = (ctypes.c_double * n)()
    lib.slim_default_tau(buf, n)
    return np.frombuffer(buf, dtype=np.float64).copy()


def make_params(sqc_weight_mode: int = 0, mask_scope: int = 0, q1_mode: int = 0, sal_mode: int = 0) -> SlimParams:
    return SlimParams(sqc_weight_mode, mask_scope, q1_mode, sal_mode)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _need_cuda(*tensors):
    for t in tensors:
        if t is None:
            continue
        if not t.is_cuda:
            raise ValueError("libslim takes device tensors")
        if t.dim() >= 1 and t.stride(-1) != 1:
            raise ValueError("libslim takes row-major tensors (last dimension contiguous)")


class Slim:
    """A library context bound to the current torch stream of `device`."""

    def __init__(self, device: str = "cuda:0", workspace_bytes: int = 0):
        """workspace_bytes > 0: the context works in a buffer of that size allocated here, once (see
        workspace_query), and no entry point allocates device memory; 0: the library grows its own on demand."""
        self.lib = load()
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.stream = torch.cuda.current_stream(self.device)
        self.workspace = (torch.empty(workspace_bytes + 256, dtype=torch.uint8, device=self.device)
                          if workspace_bytes > 0 else None)
        ws_ptr = None
        if self.workspace is not None:
            ws_ptr = ctypes.c_void_p((self.workspace.data_ptr() + 255) // 256 * 256)
        handle = ctypes.c_void_p()
        st = self.lib.slim_create(ctypes.byref(handle), ctypes.c_void_p(self.stream.cuda_stream), ws_ptr,
                                  workspace_bytes)
        if st != SLIM_OK:
            raise SlimError(st, "slim_create failed")
        self.ctx = handle

    def close(self):
        if getattr(self, "ctx", None):
            self.lib.slim_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != SLIM_OK:
            raise SlimError(st, self.lib.slim_last_error(self.ctx).decode())

    def workspace_bytes(self) -> int:
        return int(self.lib.slim_workspace_bytes(self.ctx))

    # ---- a1
    def hessian_accumulate(self, X: torch.Tensor, G: torch.Tensor, n_tokens: int = 0) -> int:
        """G (m x m float32) += X X^T for X of shape (m, t_c) float16 / bfloat16; returns the new token count."""
        _need_cuda(X, G)
        m, t_c = X.shape
        assert X.stride(1) == 1 and G.stride(1) == 1 and G.dtype == torch.float32
        nt = ctypes.c_int64(n_tokens)
        self._check(self.lib.slim_hessian_accumulate(self.ctx, _ptr(X), _DT[X.dtype], m, t_c, X.stride(0), _ptr(G),
                                                     G.stride(0), ctypes.byref(nt)))
        return int(nt.value)

    # ---- a2
    def hessian_inverse(self, G: torch.Tensor, n_tokens: int, percdamp: float = 0.01,
                        U: Optional[torch.Tensor] = None, hinv_diag: Optional[torch.Tensor] = None):
        """Returns (U float64 (m, m) upper, hinv_diag float64 (m,)); raises SlimError(ERR_NOT_PD) otherwise."""
        _need_cuda(G)
        m = G.shape[0]
        U = torch.empty((m, m), dtype=torch.float64, device=G.device) if U is None else U
        hinv_diag = torch.empty(m, dtype=torch.float64, device=G.device) if hinv_diag is None else hinv_diag
        info = ctypes.c_int(0)
        st = self.lib.slim_hessian_inverse(self.ctx, _ptr(G), G.stride(0), m, n_tokens, percdamp, _ptr(U), U.stride(0),
                                           _ptr(hinv_diag), ctypes.byref(info))
        self.last_info = int(info.value)
        self._check(st)
        return U, hinv_diag

    # ---- a3
    def salience(self, W: torch.Tensor, hinv_diag: Optional[torch.Tensor], beta: int, U: Optional[torch.Tensor] = None,
                 sal_mode: int = SAL_HINV_DIAG, want_elem: bool = False):
        _need_cuda(W, hinv_diag, U)
        n, m = W.shape
        col = torch.empty(m, dtype=torch.float64, device=W.device)
        grp = torch.empty(max(m // max(beta, 1), 1), dtype=torch.float64, device=W.device)
        elem = torch.empty((n, m), dtype=torch.float64, device=W.device) if want_elem else None
        self._check(self.lib.slim_salience(self.ctx, _ptr(W), _DT[W.dtype], n, m, W.stride(0), _ptr(U),
                                           0 if U is None else U.stride(0), _ptr(hinv_diag), sal_mode, beta, _ptr(col),
                                           _ptr(grp), _ptr(elem)))
        return col, grp, elem

    # ---- a4
    def sba_prepare(self, W: torch.Tensor, beta: int, N: int, Xs: torch.Tensor, params: Optional[SlimParams] = None,
                    objective: int = OBJ_KL) -> None:
        """Enqueues the part of sba_allocate that needs no salience; the next call on this context must be
        sba_allocate with the same W, Xs, beta, N, params and objective."""
        _need_cuda(W, Xs)
        n, m = W.shape
        self._check(self.lib.slim_sba_prepare(self.ctx, _ptr(W), _DT[W.dtype], n, m, W.stride(0), beta, N, objective,
                                              _ptr(Xs), _DT[Xs.dtype], Xs.shape[1], Xs.stride(0),
                                              ctypes.byref(params) if params is not None else None))

    def sba_allocate(self, W: torch.Tensor, group_sal: torch.Tensor, beta: int, N: int, Xs: torch.Tensor,
                     params: Optional[SlimParams] = None, objective: int = OBJ_KL, host_outputs: bool = True):
        """Returns (bits uint8 device tensor (k,), p_star, obj_curve numpy (k//2+1,)); with host_outputs=False the
        call does not wait for the stream and the last two are None."""
        _need_cuda(W, group_sal, Xs)
        n, m = W.shape
        k = m // beta
        t_s = Xs.shape[1]
        bits = torch.empty(k, dtype=torch.uint8, device=W.device)
        p_star = ctypes.c_int(-1)
        curve = (ctypes.c_double * (k // 2 + 1))()
        self._check(self.lib.slim_sba_allocate(self.ctx, _ptr(W), _DT[W.dtype], n, m, W.stride(0), _ptr(group_sal), beta,
                                               N, objective, _ptr(Xs), _DT[Xs.dtype], t_s, Xs.stride(0),
                                               ctypes.byref(params) if params is not None else None, _ptr(bits),
                                               ctypes.byref(p_star) if host_outputs else None,
                                               curve if host_outputs else None))
        if not host_outputs:
            return bits, None, None
        return bits, int(p_star.value), np.frombuffer(curve, dtype=np.float64).copy()

    # ---- a5 + a6
    def sqc_calibrate(self, Wblk: torch.Tensor, bits: int, params: Optional[SlimParams] = None,
                      omega: Optional[torch.Tensor] = None, hinv_diag_blk: Optional[torch.Tensor] = None,
                      tau: Optional[torch.Tensor] = None):
        """Wblk float64 (n, beta).  Returns (scale, zero float64 (n,), cand_idx int32 (n,))."""
        _need_cuda(Wblk, omega, hinv_diag_blk, tau)
        n, beta = Wblk.shape
        scale = torch.empty(n, dtype=torch.float64, device=Wblk.device)
        zero = torch.empty(n, dtype=torch.float64, device=Wblk.device)
        idx = torch.empty(n, dtype=torch.int32, device=Wblk.device)
        self._check(self.lib.slim_sqc_calibrate(self.ctx, _ptr(Wblk), Wblk.stride(0), n, beta, bits, _ptr(omega),
                                                _ptr(hinv_diag_blk),
                                                ctypes.byref(params) if params is not None else None, _ptr(tau),
                                                0 if tau is None else tau.numel(), _ptr(scale), _ptr(zero), _ptr(idx)))
        return scale, zero, idx

    # ---- a5 - a8
    def gptq_quantize(self, W: torch.Tensor, U: torch.Tensor, bits: torch.Tensor, beta: int,
                      params: Optional[SlimParams] = None, hinv_diag: Optional[torch.Tensor] = None,
                      tau: Optional[torch.Tensor] = None, want_what: Optional[torch.dtype] = None,
                      want_sum_e2: bool = False, gptq_block: Optional[int] = None):
        """Returns dict(codes uint8 (n, m), scale, zero float64 (n, k), What or None, sum_e2 or None)."""
        _need_cuda(W, U, bits, hinv_diag, tau)
        n, m = W.shape
        k = m // beta
        codes = torch.empty((n, m), dtype=torch.uint8, device=W.device)
        scale = torch.empty((n, k), dtype=torch.float64, device=W.device)
        zero = torch.empty((n, k), dtype=torch.float64, device=W.device)
        what = torch.empty((n, m), dtype=want_what, device=W.device) if want_what is not None else None
        se2 = torch.zeros(1, dtype=torch.float64, device=W.device) if want_sum_e2 else None
        self._check(self.lib.slim_gptq_quantize(self.ctx, _ptr(W), _DT[W.dtype], n, m, W.stride(0), _ptr(U), U.stride(0),
                                                _ptr(bits), beta, beta if gptq_block is None else gptq_block,
                                                ctypes.byref(params) if params is not None else None, _ptr(hinv_diag),
                                                _ptr(tau), 0 if tau is None else tau.numel(), _ptr(codes), _ptr(scale),
                                                _ptr(zero), _ptr(what), F32 if what is None else _DT[what.dtype],
                                                _ptr(se2)))
        return dict(codes=codes, scale=scale, zero=zero, What=what, sum_e2=se2)

    # ---- a9
    def pack(self, codes: torch.Tensor, bits: torch.Tensor, beta: int, packed_rows: Optional[int] = None,
             host_outputs: bool = True, bit_base: int = 1):
        """Returns (packed uint32-as-int32 (m_star, n), gbits (ceil(k/16),), row_off int32 (k+1,), m_star); with
        host_outputs=False the call does not wait for the stream: packed then has all rows of its capacity (zero
        from row m_star = row_off[k] on) and m_star is None.  bit_base is the width that the 2-bit group value 0
        stands for (bit_base_for(N) of the layer's target width)."""
        _need_cuda(codes, bits)
        n, m = codes.shape
        k = m // beta
        cap = m * (bit_base + 3) // 32 if packed_rows is None else packed_rows     # the widest width the base allows
        packed = torch.zeros((max(cap, 1), n), dtype=torch.int32, device=codes.device)
        gbits = torch.zeros((k + 15) // 16, dtype=torch.int32, device=codes.device)
        row_off = torch.zeros(k + 1, dtype=torch.int32, device=codes.device)
        m_star = ctypes.c_int(0)
        self._check(self.lib.slim_pack(self.ctx, _ptr(codes), n, m, codes.stride(0), _ptr(bits), beta, bit_base, _ptr(packed), cap,
                                       _ptr(gbits), _ptr(row_off), ctypes.byref(m_star) if host_outputs else None))
        if not host_outputs:
            return packed, gbits, row_off, None
        return packed[: m_star.value], gbits, row_off, int(m_star.value)

    def pack_zeros(self, zero: torch.Tensor, zbits: int, host_outputs: bool = True):
        """zero float64 (n, k) -> (zpacked uint32-as-int32 (k, ceil(n zbits / 32)), number of zeros that did not fit
        or None with host_outputs=False)."""
        _need_cuda(zero)
        n, k = zero.shape
        zp = torch.empty((k, (n * zbits + 31) // 32), dtype=torch.int32, device=zero.device)
        bad = ctypes.c_int(0)
        self._check(self.lib.slim_pack_zeros(self.ctx, _ptr(zero), n, k, zero.stride(0), zbits, _ptr(zp), zp.stride(0),
                                             ctypes.byref(bad) if host_outputs else None))
        return zp, (int(bad.value) if host_outputs else None)

    def unpack_zeros(self, zp: torch.Tensor, n: int, zbits: int):
        _need_cuda(zp)
        k = zp.shape[0]
        zero = torch.empty((n, k), dtype=torch.float64, device=zp.device)
        self._check(self.lib.slim_unpack_zeros(self.ctx, _ptr(zp), zp.stride(0), n, k, zbits, _ptr(zero), zero.stride(0)))
        return zero

    # ---- n4
    def lwc_quantize(self, W: torch.Tensor, G: torch.Tensor, n_tokens: int, bits: torch.Tensor, beta: int, steps: int = 20,
                     lr: float = 1e-2, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8, init: float = 4.0,
                     want_what: Optional[torch.dtype] = None, host_outputs: bool = True):
        """SliM-LLM+ on one layer.  Returns dict(codes uint8 (n, m), scale, zero float64 (n, k), What or None,
        loss_curve numpy (steps + 1,) or None with host_outputs=False)."""
        _need_cuda(W, G, bits)
        n, m = W.shape
        k = m // beta
        codes = torch.empty((n, m), dtype=torch.uint8, device=W.device)
        scale = torch.empty((n, k), dtype=torch.float64, device=W.device)
        zero = torch.empty((n, k), dtype=torch.float64, device=W.device)
        what = torch.empty((n, m), dtype=want_what, device=W.device) if want_what is not None else None
        curve = (ctypes.c_double * (steps + 1))()
        self._check(self.lib.slim_lwc_quantize(self.ctx, _ptr(W), _DT[W.dtype], n, m, W.stride(0), _ptr(G), G.stride(0),
                                               n_tokens, _ptr(bits), beta, steps, lr, beta1, beta2, eps, init, _ptr(codes),
                                               _ptr(scale), _ptr(zero), _ptr(what),
                                               F32 if what is None else _DT[what.dtype], curve if host_outputs else None))
        return dict(codes=codes, scale=scale, zero=zero, What=what,
                    loss_curve=np.frombuffer(curve, dtype=np.float64).copy() if host_outputs else None)

    # ---- n1
    def dequant_matmul(self, packed: torch.Tensor, gbits: torch.Tensor, row_off: torch.Tensor, scale: torch.Tensor,
                       zero: torch.Tensor, beta: int, X: torch.Tensor, Y: Optional[torch.Tensor] = None,
                       bit_base: int = 1, noalloc: bool = False):
        """Y (t_x, n) float32 = X (t_x, m) float16 / bfloat16 times the dequantised weights, from the stored form.
        noalloc=True calls slim_dequant_matmul_noalloc (Y must then be passed in, so that nothing is allocated)."""
        _need_cuda(packed, gbits, row_off, scale, zero, X)
        n = packed.shape[1]
        t_x, m = X.shape
        assert scale.dtype == torch.float64 and zero.dtype == torch.float64 and scale.stride(0) == m // beta
        Y = torch.empty((t_x, n), dtype=torch.float32, device=X.device) if Y is None else Y
        fn = self.lib.slim_dequant_matmul_noalloc if noalloc else self.lib.slim_dequant_matmul
        self._check(fn(self.ctx, _ptr(packed), packed.stride(0), _ptr(gbits), _ptr(row_off),
                                                 _ptr(scale), _ptr(zero), n, m, beta, bit_base, _ptr(X), _DT[X.dtype], t_x,
                                                 X.stride(0), _ptr(Y), Y.stride(0)))
        return Y

    def dequant_matmul_zp(self, packed: torch.Tensor, gbits: torch.Tensor, row_off: torch.Tensor, scale: torch.Tensor,
                          zpacked: torch.Tensor, zbits: int, beta: int, X: torch.Tensor, bit_base: int = 1):
        """The linear layer on the stored form with packed zero points (from pack_zeros)."""
        _need_cuda(packed, gbits, row_off, scale, zpacked, X)
        n = packed.shape[1]
        t_x, m = X.shape
        Y = torch.empty((t_x, n), dtype=torch.float32, device=X.device)
        self._check(self.lib.slim_dequant_matmul_zp(self.ctx, _ptr(packed), packed.stride(0), _ptr(gbits), _ptr(row_off),
                                                    _ptr(scale), _ptr(zpacked), zpacked.stride(0), zbits, n, m, beta,
                                                    bit_base, _ptr(X), _DT[X.dtype], t_x, X.stride(0), _ptr(Y), Y.stride(0)))
        return Y

    # ---- measurement aid
    def profile_enable(self, on: bool = True):
        self._check(self.lib.slim_profile_enable(self.ctx, 1 if on else 0))

    def profile_reset(self):
        self._check(self.lib.slim_profile_reset(self.ctx))

    def profile_collect(self):
        """Returns {kernel name: (total_ms, launches)} accumulated since the last reset."""
        n = self.lib.slim_profile_collect(self.ctx)
        out = {}
        for i in range(n):
            name = ctypes.c_char_p()
            ms = ctypes.c_double()
            cnt = ctypes.c_int()
            self._check(self.lib.slim_profile_entry(self.ctx, i, ctypes.byref(name), ctypes.byref(ms), ctypes.byref(cnt)))
            out[name.value.decode()] = (ms.value, cnt.value)
        return out
