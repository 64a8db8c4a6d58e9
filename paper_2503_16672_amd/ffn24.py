"""ctypes binding over libffn24.so: the same names as include/ffn24.h, argument marshalling only.

Tensors are torch CUDA tensors (torch is used for device memory and streams, nothing else); every
call enqueues on torch's current stream.  Loading fails loudly if the library has not been built:
there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libffn24.so")

FFN24_BF16 = 0
FFN24_FP8_E4M3 = 1
FFN24_TRAINING = 1
FFN24_DENSE = 2
FFN24_DEBUG_DUMP_H = 4
FFN24_SPLIT = 8
FFN24_ROWWISE = 16
FFN24_PERMUTE = 32
FFN24_TELEMETRY = 64

EXPORTS = (
    "ffn24_ctx_create", "ffn24_ctx_destroy", "ffn24_set_scales", "ffn24_set_bwd_scales", "ffn24_set_row_scales", "ffn24_set_token_permutation", "ffn24_set_split", "sparsify24", "sparsify24_quantise", "quantise_e4m3", "sparsify24_featurewise", "spmm24", "ffn24_fwd", "ffn24_bwd", "ffn24_bwd_rowwise", "ffn_bwd_rowwise",
    "ffn_fwd", "ffn_bwd", "ffn24_prepare_weights", "ffn24_get_telemetry", "ffn24_policy_use_sparse", "ffn24_saved_bytes", "ffn24_copy_saved", "ffn24_set_profiling", "ffn24_kernel_ms", "ffn24_strerror",
    "ffn24_static_scratch_needed", "ffn24_fwd_static", "ffn24_kernel_mhz", "ffn24_probe_mfma_rate", "ffn24_probe_gemm", "ffn24_probe_copy",
)

KERNEL_NAMES = ("up_prune24", "down_sp", "dh_gather", "dx_sp", "featurewise24", "dw2_sp", "dw1_sp",
                "dense_up", "dense_down", "dense_dh", "dense_dx", "dense_dw2", "dense_dw1", "transpose_weights", "transpose_acts",
                "split_partition", "transpose_dw1", "quantise_rows", "quantise_dz_rows", "quantise_transposed", "panelise_bwd_weights", "panelise_x")



class RowwiseBwdOperands(ctypes.Structure):
    """ffn24_rowwise_bwd_operands of the header: five (codes, scales) pointer pairs."""
    _fields_ = [(n, ctypes.c_void_p) for n in ("dY8r", "sdy_t", "dY8c", "sdy_d", "X8c", "sx_d", "W2_8r", "sw2_f", "W1_8c", "sw1_d")]


_lib = None


class Ffn24Error(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: ffn24 error {code}: {strerror(code)}")
        self.code = code


def lib() -> ctypes.CDLL:
    """Load libffn24.so (once).  Raises if it is missing: build it with `python -m paper_2503_16672_amd.build`."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is not built; run `python -m paper_2503_16672_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        L.ffn24_ctx_create.argtypes = [ctypes.POINTER(vp), i64, i64, i64, ci, ci]
        L.ffn24_ctx_destroy.argtypes = [vp]
        L.ffn24_set_scales.argtypes = [vp, ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_float]
        L.ffn24_set_bwd_scales.argtypes = [vp, ctypes.c_float, ctypes.c_float]
        L.ffn24_set_split.argtypes = [vp, i64]
        L.ffn24_set_token_permutation.argtypes = [vp, vp]
        L.ffn24_set_row_scales.argtypes = [vp, vp, vp, vp]
        L.ffn24_bwd_rowwise.argtypes = [vp, ctypes.POINTER(RowwiseBwdOperands), vp, vp, vp, vp]
        L.ffn_bwd_rowwise.argtypes = [vp, ctypes.POINTER(RowwiseBwdOperands), vp, vp, vp, vp]
        L.sparsify24.argtypes = [vp, i64, i64, ci, vp, vp, vp]
        L.sparsify24_quantise.argtypes = [vp, i64, i64, ctypes.c_float, vp, vp, vp]
        L.quantise_e4m3.argtypes = [vp, i64, i64, ci, vp, vp, vp]
        L.sparsify24_featurewise.argtypes = [vp, vp, vp, i64, i64, vp, vp, vp, vp]
        L.spmm24.argtypes = [vp, vp, vp, i64, i64, i64, vp, vp]
        L.ffn24_fwd.argtypes = [vp, vp, vp, vp, vp, vp, vp]
        L.ffn24_bwd.argtypes = [vp, vp, vp, vp, vp, vp]
        L.ffn_fwd.argtypes = [vp, vp, vp, vp, vp, vp, vp]
        L.ffn_bwd.argtypes = [vp, vp, vp, vp, vp, vp]
        L.ffn24_prepare_weights.argtypes = [vp, vp, vp, vp]
        L.ffn24_get_telemetry.argtypes = [vp, ctypes.POINTER(i64), ci]
        L.ffn24_policy_use_sparse.argtypes = [vp, ctypes.c_double, ctypes.POINTER(ci)]
        L.ffn24_saved_bytes.argtypes = [vp, ci, ctypes.POINTER(i64)]
        L.ffn24_copy_saved.argtypes = [vp, ci, vp, i64, vp]
        L.ffn24_set_profiling.argtypes = [vp, ci]
        L.ffn24_kernel_ms.argtypes = [vp, ci, ctypes.POINTER(ctypes.c_float)]
        L.ffn24_strerror.argtypes = [ci]
        L.ffn24_strerror.restype = ctypes.c_char_p
        dp = ctypes.POINTER(ctypes.c_double)
        L.ffn24_kernel_mhz.argtypes = [vp, ci, ctypes.POINTER(ctypes.c_float)]
        L.ffn24_probe_mfma_rate.argtypes = [ci, ci, dp, dp, dp]
        L.ffn24_probe_gemm.argtypes = [ci, ci, i64, i64, i64, ci, dp, dp]
        L.ffn24_probe_copy.argtypes = [i64, ci, dp]
        L.ffn24_static_scratch_needed.argtypes = [i64, i64, i64]
        L.ffn24_fwd_static.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, vp]
        for name in EXPORTS:
            if name != "ffn24_strerror":
                getattr(L, name).restype = ci
        L.ffn24_static_scratch_needed.restype = i64
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().ffn24_strerror(code).decode()


def _check(code: int, what: str) -> None:
    if code != 0:
        raise Ffn24Error(code, what)


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("ffn24 takes contiguous CUDA tensors")
    return t.data_ptr()


def _expect(t, shape, dtypes, name: str):
    """The C ABI takes bare pointers, so shapes and element types are checked here, before anything is launched."""
    if t is None:
        return
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {tuple(t.shape)}, expected {tuple(shape)}")
    if t.dtype not in dtypes:
        raise ValueError(f"{name}: dtype {t.dtype}, expected one of {dtypes}")


_BF16 = (torch.bfloat16,)
_BYTE = (torch.uint8, torch.float8_e4m3fn)
_F32 = (torch.float32,)


def _stream():
    return torch.cuda.current_stream().cuda_stream


def sparsify24(H: torch.Tensor, values: torch.Tensor | None = None, meta: torch.Tensor | None = None):
    """H [rows, cols] bf16 (or e4m3 bytes) -> (values [rows, cols/2] of the same type, meta [rows, cols/8] uint8);
    outputs may be handed in."""
    rows, cols = H.shape
    f8 = H.dtype in _BYTE
    el = _BYTE if f8 else _BF16
    _expect(H, (rows, cols), el, "H")
    _expect(values, (rows, cols // 2), el, "values")
    _expect(meta, (rows, cols // 8), (torch.uint8,), "meta")
    values = torch.empty((rows, cols // 2), dtype=H.dtype, device=H.device) if values is None else values
    meta = torch.empty((rows, cols // 8), dtype=torch.uint8, device=H.device) if meta is None else meta
    _check(lib().sparsify24(_ptr(H), rows, cols, FFN24_FP8_E4M3 if f8 else FFN24_BF16, _ptr(values), _ptr(meta), _stream()), "sparsify24")
    return values, meta


def sparsify24_quantise(H: torch.Tensor, scale: float, values8: torch.Tensor | None = None, meta: torch.Tensor | None = None):
    """H [rows, cols] bf16 -> (e4m3 codes of the kept values / scale [rows, cols/2] uint8, meta [rows, cols/8] uint8)."""
    rows, cols = H.shape
    _expect(H, (rows, cols), _BF16, "H")
    _expect(values8, (rows, cols // 2), _BYTE, "values8")
    _expect(meta, (rows, cols // 8), (torch.uint8,), "meta")
    values8 = torch.empty((rows, cols // 2), dtype=torch.uint8, device=H.device) if values8 is None else values8
    meta = torch.empty((rows, cols // 8), dtype=torch.uint8, device=H.device) if meta is None else meta
    _check(lib().sparsify24_quantise(_ptr(H), rows, cols, scale, _ptr(values8), _ptr(meta), _stream()), "sparsify24_quantise")
    return values8, meta


def sparsify24_featurewise(Hc: torch.Tensor, meta: torch.Tensor, dZc: torch.Tensor | None = None):
    """Token-wise compressed (Hc [T,F/2], meta [T,F/8]) -> (Hc_t [F,T/2], meta_t [F,T/8], dZc_t [F,T/2] or None)."""
    T, F = Hc.shape[0], Hc.shape[1] * 2
    _expect(Hc, (T, F // 2), _BF16, "Hc")
    _expect(meta, (T, F // 8), (torch.uint8,), "meta")
    _expect(dZc, (T, F // 2), _BF16, "dZc")
    Hc_t = torch.empty((F, T // 2), dtype=torch.bfloat16, device=Hc.device)
    meta_t = torch.empty((F, T // 8), dtype=torch.uint8, device=Hc.device)
    dZc_t = torch.empty((F, T // 2), dtype=torch.bfloat16, device=Hc.device) if dZc is not None else None
    _check(lib().sparsify24_featurewise(_ptr(Hc), _ptr(meta), _ptr(dZc), T, F, _ptr(Hc_t), _ptr(meta_t), _ptr(dZc_t), _stream()),
           "sparsify24_featurewise")
    return Hc_t, meta_t, dZc_t


def spmm24(values: torch.Tensor, meta: torch.Tensor, Bt: torch.Tensor) -> torch.Tensor:
    """C [M,N] = A24 . B with A24 given as (values [M,K/2], meta [M,K/8]) and B given transposed, Bt [N,K]."""
    M, K = values.shape[0], values.shape[1] * 2
    N = Bt.shape[0]
    _expect(values, (M, K // 2), _BF16, "values")
    _expect(meta, (M, K // 8), (torch.uint8,), "meta")
    _expect(Bt, (N, K), _BF16, "Bt")
    C = torch.empty((M, N), dtype=torch.bfloat16, device=values.device)
    _check(lib().spmm24(_ptr(values), _ptr(meta), _ptr(Bt), M, N, K, _ptr(C), _stream()), "spmm24")
    return C


MFMA_KINDS = ("dense bf16 32x32x16", "sparse bf16 32x32x32", "dense fp8 32x32x64", "sparse fp8 32x32x64")
GEMM_PROBE_VARIANTS = {"all": 0, "no_dma": 1, "no_fragment_reads": 4, "dma_only": 6, "mfma_only": 5, "all_l2_hits": 8, "dma_only_l2_hits": 14,
                       "all_dma_issue_unpaced": 256, "all_quarter_less_fill": 512,
                       "all_persistent_workgroups": 1024}


def quantise_e4m3(X, axis: int, codes=None, scales=None):
    """e4m3 codes and one scale per row (axis 1) or per column (axis 0) of a bf16 CUDA matrix (see quantise_e4m3 in the header)."""
    R, C = X.shape
    _expect(X, (R, C), _BF16, "X")
    codes = torch.empty((R, C), dtype=torch.uint8, device=X.device) if codes is None else codes
    scales = torch.empty((R if axis == 1 else C,), dtype=torch.float32, device=X.device) if scales is None else scales
    _expect(codes, (R, C), _BYTE, "codes")
    _expect(scales, (R if axis == 1 else C,), _F32, "scales")
    _check(lib().quantise_e4m3(_ptr(X), R, C, axis, _ptr(codes), _ptr(scales), _stream()), "quantise_e4m3")
    return codes, scales


def probe_mfma_rate(kind: int, iters: int = 20000) -> dict:
    """Register-resident matrix-op loop (see ffn24_probe_mfma_rate in the header)."""
    c, m, t = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    _check(lib().ffn24_probe_mfma_rate(kind, iters, ctypes.byref(c), ctypes.byref(m), ctypes.byref(t)), "ffn24_probe_mfma_rate")
    return {"cycles_per_op": c.value, "mhz": m.value, "tflops_dense_equivalent": t.value}


def probe_gemm(sparse: bool, variant: int, M: int, N: int, K: int, reps: int = 20) -> dict:
    """The GEMM core with ingredients of its main loop taken out (see ffn24_probe_gemm in the header)."""
    ms, m = ctypes.c_double(), ctypes.c_double()
    _check(lib().ffn24_probe_gemm(int(sparse), variant, M, N, K, reps, ctypes.byref(ms), ctypes.byref(m)), "ffn24_probe_gemm")
    return {"ms": ms.value, "mhz": m.value}


def probe_copy(nbytes: int, reps: int = 20) -> float:
    """Median milliseconds of a plain device copy kernel of nbytes bytes (see ffn24_probe_copy in the header)."""
    ms = ctypes.c_double()
    _check(lib().ffn24_probe_copy(nbytes, reps, ctypes.byref(ms)), "ffn24_probe_copy")
    return ms.value


GEMM_PROBE_WALKS = {"grid 4x2 of 8x4 patches (product)": 0, "bands of 8 tile-rows per XCD": 16, "8 patches side by side along M": 32,
                    "4x8 patches": 64, "16x2 patches": 128}
STATIC_SCRATCH_BYTES = 64 << 20


def static_scratch_needed(T: int, D: int, F: int) -> int:
    return int(lib().ffn24_static_scratch_needed(T, D, F))


def ffn24_fwd_static(X, W1, b1, W2, Y):
    """The context-free forward that allocates nothing (see ffn24_fwd_static in the header); Y is handed in."""
    T, D = X.shape
    F = W1.shape[1]
    _expect(X, (T, D), _BF16, "X")
    _expect(W1, (D, F), _BF16, "W1")
    _expect(W2, (F, D), _BF16, "W2")
    _expect(b1, (F,), _F32, "b1")
    _expect(Y, (T, D), _BF16, "Y")
    _check(lib().ffn24_fwd_static(_ptr(X), _ptr(W1), _ptr(b1), _ptr(W2), _ptr(Y), T, D, F, _stream()), "ffn24_fwd_static")
    return Y


class Context:
    """Owns an ffn24_ctx (the device workspace for one (T, D, F) problem)."""

    def __init__(self, T: int, D: int, F: int, flags: int = 0, dtype: int = FFN24_BF16):
        self.T, self.D, self.F, self.flags, self.dtype = T, D, F, flags, dtype
        h = ctypes.c_void_p()
        _check(lib().ffn24_ctx_create(ctypes.byref(h), T, D, F, dtype, flags), "ffn24_ctx_create")
        self._h = h

    def close(self):
        if self._h:
            torch.cuda.synchronize()
            _check(lib().ffn24_ctx_destroy(self._h), "ffn24_ctx_destroy")
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_scales(self, sx: float, sw1: float, sh: float, sw2: float):
        """Per-tensor scales of an fp8 context (see ffn24_set_scales in the header)."""
        _check(lib().ffn24_set_scales(self._h, sx, sw1, sh, sw2), "ffn24_set_scales")

    def set_bwd_scales(self, sdy: float, sdz: float):
        """Scales of the incoming gradient and of the stored dZ of an fp8 training context (see ffn24_set_bwd_scales)."""
        _check(lib().ffn24_set_bwd_scales(self._h, sdy, sdz), "ffn24_set_bwd_scales")

    def set_row_scales(self, sx, sw1, sw2):
        """Row-wise scales of an FFN24_ROWWISE fp8 context: fp32 CUDA tensors [T], [F], [D]; the context keeps them alive."""
        _expect(sx, (self.T,), _F32, "sx")
        _expect(sw1, (self.F,), _F32, "sw1")
        _expect(sw2, (self.D,), _F32, "sw2")
        self._row_scales = (sx, sw1, sw2)
        _check(lib().ffn24_set_row_scales(self._h, _ptr(sx), _ptr(sw1), _ptr(sw2)), "ffn24_set_row_scales")

    def set_token_permutation(self, perm):
        """perm: int32 numpy array [T] on the host (position p inside the FFN holds token perm[p]), or None to switch it off."""
        if perm is None:
            _check(lib().ffn24_set_token_permutation(self._h, None), "ffn24_set_token_permutation")
            return
        import numpy as np
        perm = np.ascontiguousarray(perm, dtype=np.int32)
        if perm.shape != (self.T,):
            raise ValueError("perm must have one entry per token")
        _check(lib().ffn24_set_token_permutation(self._h, perm.ctypes.data), "ffn24_set_token_permutation")

    def set_split(self, n_dense: int):
        """Keep the n_dense least sparse features out of the feature-wise 2:4 (see ffn24_set_split in the header)."""
        _check(lib().ffn24_set_split(self._h, n_dense), "ffn24_set_split")

    def _check_fwd_args(self, X, W1, b1, W2, Y):
        el = _BYTE if self.dtype == FFN24_FP8_E4M3 else _BF16
        _expect(X, (self.T, self.D), el, "X")
        _expect(W1, (self.D, self.F), el, "W1")
        _expect(W2, (self.F, self.D), el, "W2")
        _expect(b1, (self.F,), _F32, "b1")
        _expect(Y, (self.T, self.D), _BF16, "Y")

    def prepare_weights(self, W1, W2):
        """Run the weight pass once; afterwards ffn24_fwd / ffn_fwd take W1 = W2 = None (see ffn24_prepare_weights)."""
        el = _BYTE if self.dtype == FFN24_FP8_E4M3 else _BF16
        _expect(W1, (self.D, self.F), el, "W1")
        _expect(W2, (self.F, self.D), el, "W2")
        self._prepared = (W1, W2)      # keeps them alive
        _check(lib().ffn24_prepare_weights(self._h, _ptr(W1), _ptr(W2), _stream()), "ffn24_prepare_weights")

    def ffn24_fwd(self, X, W1, b1, W2, Y=None):
        Y = torch.empty((self.T, self.D), dtype=torch.bfloat16, device=X.device) if Y is None else Y
        self._check_fwd_args(X, W1, b1, W2, Y)
        _check(lib().ffn24_fwd(self._h, _ptr(X), _ptr(W1), _ptr(b1), _ptr(W2), _ptr(Y), _stream()), "ffn24_fwd")
        return Y

    def ffn_fwd(self, X, W1, b1, W2, Y=None):
        Y = torch.empty((self.T, self.D), dtype=torch.bfloat16, device=X.device) if Y is None else Y
        self._check_fwd_args(X, W1, b1, W2, Y)
        _check(lib().ffn_fwd(self._h, _ptr(X), _ptr(W1), _ptr(b1), _ptr(W2), _ptr(Y), _stream()), "ffn_fwd")
        return Y

    def _bwd(self, fn, name, dY, out):
        dev = dY.device
        if out is None:
            out = (torch.empty((self.T, self.D), dtype=torch.bfloat16, device=dev),
                   torch.empty((self.D, self.F), dtype=torch.bfloat16, device=dev),
                   torch.empty((self.F, self.D), dtype=torch.bfloat16, device=dev))
        dX, dW1, dW2 = out
        _expect(dY, (self.T, self.D), _BYTE if self.dtype == FFN24_FP8_E4M3 else _BF16, "dY")
        _expect(dX, (self.T, self.D), _BF16, "dX")
        _expect(dW1, (self.D, self.F), _BF16, "dW1")
        _expect(dW2, (self.F, self.D), _BF16, "dW2")
        _check(fn(self._h, _ptr(dY), _ptr(dX), _ptr(dW1), _ptr(dW2), _stream()), name)
        return dX, dW1, dW2

    def ffn24_bwd(self, dY, out=None):
        return self._bwd(lib().ffn24_bwd, "ffn24_bwd", dY, out)

    def ffn_bwd(self, dY, out=None):
        return self._bwd(lib().ffn_bwd, "ffn_bwd", dY, out)

    def ffn_bwd_rowwise(self, *operands, out=None):
        """Dense baseline of ffn24_bwd_rowwise (see ffn_bwd_rowwise in the header); same operands."""
        return self.ffn24_bwd_rowwise(*operands, out=out, _fn="ffn_bwd_rowwise")

    def ffn24_bwd_rowwise(self, dY8r, sdy_t, dY8c, sdy_d, X8c, sx_d, W2_8r, sw2_f, W1_8c, sw1_d, out=None, _fn="ffn24_bwd_rowwise"):
        """Backward of a row-wise-scaled forward (see ffn24_bwd_rowwise in the header): e4m3 codes (uint8) and fp32 scale vectors."""
        dev = dY8r.device
        if out is None:
            out = (torch.empty((self.T, self.D), dtype=torch.bfloat16, device=dev),
                   torch.empty((self.D, self.F), dtype=torch.bfloat16, device=dev),
                   torch.empty((self.F, self.D), dtype=torch.bfloat16, device=dev))
        dX, dW1, dW2 = out
        for t, shape, el, nm in ((dY8r, (self.T, self.D), _BYTE, "dY8r"), (sdy_t, (self.T,), _F32, "sdy_t"), (dY8c, (self.T, self.D), _BYTE, "dY8c"),
                                 (sdy_d, (self.D,), _F32, "sdy_d"), (X8c, (self.T, self.D), _BYTE, "X8c"), (sx_d, (self.D,), _F32, "sx_d"),
                                 (W2_8r, (self.F, self.D), _BYTE, "W2_8r"), (sw2_f, (self.F,), _F32, "sw2_f"), (W1_8c, (self.D, self.F), _BYTE, "W1_8c"),
                                 (sw1_d, (self.D,), _F32, "sw1_d"), (dX, (self.T, self.D), _BF16, "dX"), (dW1, (self.D, self.F), _BF16, "dW1"),
                                 (dW2, (self.F, self.D), _BF16, "dW2")):
            _expect(t, shape, el, nm)
        ops = RowwiseBwdOperands(*(_ptr(t) for t in (dY8r, sdy_t, dY8c, sdy_d, X8c, sx_d, W2_8r, sw2_f, W1_8c, sw1_d)))
        _check(getattr(lib(), _fn)(self._h, ctypes.byref(ops), _ptr(dX), _ptr(dW1), _ptr(dW2), _stream()), _fn)
        return dX, dW1, dW2

    _SAVED = {"Hc": (0, torch.bfloat16, lambda T, F: (T, F // 2)), "meta": (1, torch.uint8, lambda T, F: (T, F // 8)),
              "dZc": (2, torch.bfloat16, lambda T, F: (T, F // 2)), "Hc_t": (3, torch.bfloat16, lambda T, F: (F, T // 2)),
              "meta_t": (4, torch.uint8, lambda T, F: (F, T // 8)), "dZc_t": (5, torch.bfloat16, lambda T, F: (F, T // 2)),
              "H_dump": (6, torch.bfloat16, lambda T, F: (T, F)), "H_dense": (7, torch.bfloat16, lambda T, F: (T, F)),
              "dZ_dense": (8, torch.bfloat16, lambda T, F: (T, F)),
              "nnz": (9, torch.int32, lambda T, F: (F,)), "feat_of_row": (10, torch.int32, lambda T, F: (F,)),
              "sh": (11, torch.float32, lambda T, F: (T,)), "Hc16": (12, torch.bfloat16, lambda T, F: (T, F // 2)),
              "sdz_t": (13, torch.float32, lambda T, F: (T,)), "sh_f": (14, torch.float32, lambda T, F: (F,)),
              "sdz_f": (15, torch.float32, lambda T, F: (F,)), "dZc16": (16, torch.bfloat16, lambda T, F: (T, F // 2)),
              "dZ16_dense": (17, torch.bfloat16, lambda T, F: (T, F)), "H_dense_t": (18, torch.uint8, lambda T, F: (F, T)),
              "dZ_dense_t": (19, torch.uint8, lambda T, F: (F, T)),
              "Hdn_t": (20, torch.bfloat16, lambda T, F: (F // 4, T)), "dZdn_t": (21, torch.bfloat16, lambda T, F: (F // 4, T))}

    def saved(self, name: str) -> torch.Tensor:
        """Row-major copy of a saved tensor of the context (enqueued on the current stream)."""
        which, dtype, shape_fn = self._SAVED[name]
        if self.dtype == FFN24_FP8_E4M3 and dtype == torch.bfloat16 and name not in ("H_dump", "Hc16", "dZc16", "dZ16_dense"):
            dtype = torch.uint8      # e4m3 codes
        n = ctypes.c_int64()
        _check(lib().ffn24_saved_bytes(self._h, which, ctypes.byref(n)), "ffn24_saved_bytes")
        out = torch.empty(shape_fn(self.T, self.F), dtype=dtype, device="cuda")
        assert out.numel() * out.element_size() == n.value
        _check(lib().ffn24_copy_saved(self._h, which, _ptr(out), n.value, _stream()), f"ffn24_copy_saved({name})")
        return out

    def telemetry(self, wait: bool = True) -> dict:
        """The newest sparsity snapshot of an FFN24_TELEMETRY context (see ffn24_get_telemetry in the header)."""
        n = (ctypes.c_int64 * 5)()
        _check(lib().ffn24_get_telemetry(self._h, n, int(wait)), "ffn24_get_telemetry")
        sparse = bool(n[4])
        return {"elements": n[0], "nonzero": n[1], "kept_tokenwise": n[2] if sparse else None,
                "kept_featurewise": n[3] if sparse and n[3] else None, "path": "2:4" if sparse else "dense"}

    def policy_use_sparse(self, min_sparsity: float) -> bool:
        """Whether the newest landed snapshot is sparse enough for the 2:4 path (see ffn24_policy_use_sparse)."""
        use = ctypes.c_int()
        _check(lib().ffn24_policy_use_sparse(self._h, min_sparsity, ctypes.byref(use)), "ffn24_policy_use_sparse")
        return bool(use.value)

    def set_profiling(self, on: bool):
        _check(lib().ffn24_set_profiling(self._h, int(on)), "ffn24_set_profiling")

    def kernel_mhz(self, kernel: int) -> float | None:
        """Shader clock (MHz) a GEMM kernel of the last profiled call ran at; None for kernels that take no sample."""
        mhz = ctypes.c_float()
        rc = lib().ffn24_kernel_mhz(self._h, kernel, ctypes.byref(mhz))
        if rc == -5:
            return None
        _check(rc, "ffn24_kernel_mhz")
        return float(mhz.value)

    def kernel_ms(self, kernel: int) -> float:
        ms = ctypes.c_float()
        _check(lib().ffn24_kernel_ms(self._h, kernel, ctypes.byref(ms)), "ffn24_kernel_ms")
        return float(ms.value)
