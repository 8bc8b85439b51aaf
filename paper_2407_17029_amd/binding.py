"""Thin ctypes binding over the C-ABI library (include/qblora.h), same entry-point names.

Argument marshalling only: PyTorch allocates device buffers and supplies the stream; every step
of the method runs inside libqblora.so.  There is no CPU fallback: if the library has not been
built (python -m paper_2407_17029_amd.build) loading raises, and every call checks the returned
status code and raises on error.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_DIR, "libqblora.so")

OK = 0
QUANT_ABSMAX_CODEBOOK, QUANT_MINMAX_INT4 = 0, 1
SCALES_FP32, SCALES_E4M3_GROUPED = 0, 1
MERGE_BETA_SHIFT, MERGE_REQUANT_MINMAX = 0, 1
OP_AVGPOOL_REPEAT, OP_TRUNCATE_PAD0, OP_SAMPLE_ZEROFILL = 0, 1, 2

EXPORTS = ["qblora_quantize_blockwise", "qblora_dequantize_bf16", "qblora_linear_fwd_workspace_bytes",
           "qblora_linear_bwd_workspace_bytes", "qblora_linear_fwd", "qblora_linear_bwd",
           "qblora_tile_product_workspace_bytes", "qblora_tile_product", "qablora_merge_quantize",
           "qablora_merge_quantize_batch",
           "qblora_strerror", "qblora_profile_events", "qblora_codes_tiled_bytes", "qblora_prepack_codes",
           "qblora_saved_bytes", "qblora_linear_fwd_save", "qblora_linear_bwd_saved",
           "qablora_linear_fwd_workspace_bytes", "qablora_linear_bwd_workspace_bytes", "qablora_linear_fwd",
           "qablora_linear_bwd", "qblora_merge_bf16",
           "qblora_linear_decode_workspace_bytes", "qblora_linear_decode_tokens_workspace_bytes", "qblora_linear_decode",
           "qblora_decode_pack_bytes", "qblora_decode_pack",
           "qblora_noalloc_scratch_bytes", "qblora_linear_fwd_noalloc", "qblora_dense_min_tokens"]

PROFILE_FWD_GEMM, PROFILE_BWD_GEMM, PROFILE_MERGE, PROFILE_QUANTIZE = 0, 1, 2, 3
PROFILE_ADAPTER_FWD, PROFILE_ADAPTER_BWD, PROFILE_ADAPTER_GRADS, PROFILE_GRAD_REDUCE = 4, 5, 6, 7
PROFILE_PREP, PROFILE_TILE_PRODUCT, PROFILE_DEQUANT = 8, 9, 10


class CQWeight(C.Structure):
    _fields_ = [("d_out", C.c_int32), ("d_in", C.c_int32), ("block", C.c_int32), ("scale_mode", C.c_int32),
                ("scale_group", C.c_int32), ("codebook", C.c_float * 16), ("codes", C.c_void_p),
                ("scales", C.c_void_p), ("beta", C.c_void_p), ("scale_codes", C.c_void_p),
                ("scale_step", C.c_void_p), ("scale_mid", C.c_void_p), ("codes_tiled", C.c_void_p),
                ("block_rows", C.c_int32)]


class CAdapter(C.Structure):
    _fields_ = [("lambda1", C.c_int32), ("lambda2", C.c_int32), ("R", C.c_int32), ("s", C.c_float),
                ("A", C.c_void_p), ("B", C.c_void_p), ("scale_op", C.c_int32)]


class QBLoRAError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} (code {code})")


_lib = None


def lib():
    """Load libqblora.so (raises if it was not built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2407_17029_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.qblora_strerror.restype = C.c_char_p
        L.qblora_strerror.argtypes = [C.c_int]
        for name in ("qblora_linear_fwd_workspace_bytes", "qblora_linear_bwd_workspace_bytes",
                     "qblora_tile_product_workspace_bytes"):
            getattr(L, name).restype = C.c_size_t
        L.qblora_linear_fwd_workspace_bytes.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
        L.qblora_linear_bwd_workspace_bytes.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
        L.qblora_tile_product_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
        L.qblora_quantize_blockwise.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                                C.c_int32, C.c_void_p, C.c_void_p]
        L.qblora_dequantize_bf16.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.qblora_linear_fwd.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                        C.c_size_t, C.c_void_p]
        L.qblora_linear_bwd.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                                        C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.qblora_tile_product.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t,
                                          C.c_void_p]
        L.qablora_merge_quantize.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_int32,
                                             C.c_void_p, C.c_void_p]
        L.qablora_merge_quantize_batch.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_float,
                                                   C.c_int32, C.c_void_p, C.c_void_p]
        L.qblora_profile_events.argtypes = [C.c_int32, C.c_void_p, C.c_void_p]
        L.qblora_codes_tiled_bytes.restype = C.c_size_t
        L.qblora_codes_tiled_bytes.argtypes = [C.c_int32, C.c_int32]
        L.qblora_prepack_codes.argtypes = [C.c_void_p, C.c_void_p]
        for name in ("qablora_linear_fwd_workspace_bytes", "qablora_linear_bwd_workspace_bytes"):
            getattr(L, name).restype = C.c_size_t
            getattr(L, name).argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int64]
        L.qablora_linear_fwd.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_int64,
                                         C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.qablora_linear_bwd.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_void_p,
                                         C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.qblora_merge_bf16.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_void_p]
        L.qblora_linear_decode_workspace_bytes.restype = C.c_size_t
        L.qblora_linear_decode_workspace_bytes.argtypes = [C.c_void_p]
        L.qblora_linear_decode_tokens_workspace_bytes.restype = C.c_size_t
        L.qblora_linear_decode_tokens_workspace_bytes.argtypes = [C.c_void_p, C.c_int32]
        L.qblora_linear_decode.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t,
                                           C.c_void_p]
        L.qblora_decode_pack_bytes.restype = C.c_size_t
        L.qblora_decode_pack_bytes.argtypes = [C.c_void_p]
        L.qblora_decode_pack.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.qblora_saved_bytes.restype = C.c_size_t
        L.qblora_saved_bytes.argtypes = [C.c_void_p, C.c_int64]
        L.qblora_linear_fwd_save.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                             C.c_void_p, C.c_size_t, C.c_void_p]
        L.qblora_linear_bwd_saved.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.qblora_dense_min_tokens.restype = C.c_int64
        L.qblora_dense_min_tokens.argtypes = []
        L.qblora_noalloc_scratch_bytes.restype = C.c_size_t
        L.qblora_noalloc_scratch_bytes.argtypes = []
        L.qblora_linear_fwd_noalloc.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


_hip = None


def _hip_runtime():
    """The HIP runtime the process already uses (torch has loaded it)."""
    global _hip
    if _hip is None:
        _hip = C.CDLL("libamdhip64.so")
        _hip.hipEventCreateWithFlags.argtypes = [C.POINTER(C.c_void_p), C.c_uint]
        _hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        _hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        _hip.hipEventDestroy.argtypes = [C.c_void_p]
    return _hip


class TimingEvent:
    """A HIP event that only measures time: created with hipEventDisableSystemFence, i.e. without the
    system-scope cache write-back and invalidation an ordinary event record performs (which costs stream time
    and slows the kernel behind it).  Read it only after the stream has been synchronized by other means."""
    DISABLE_SYSTEM_FENCE = 0x20000000

    def __init__(self):
        h = C.c_void_p()
        if _hip_runtime().hipEventCreateWithFlags(C.byref(h), self.DISABLE_SYSTEM_FENCE) != 0:
            raise RuntimeError("hipEventCreateWithFlags failed")
        self.cuda_event = h.value

    def record(self, stream=None):
        if _hip_runtime().hipEventRecord(self.cuda_event, _stream() if stream is None else stream) != 0:
            raise RuntimeError("hipEventRecord failed")

    def elapsed_time(self, stop: "TimingEvent") -> float:
        ms = C.c_float()
        if _hip_runtime().hipEventElapsedTime(C.byref(ms), self.cuda_event, stop.cuda_event) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return float(ms.value)

    def __del__(self):
        try:
            _hip_runtime().hipEventDestroy(self.cuda_event)
        except Exception:
            pass


def qblora_profile_events(which: int, start=None, stop=None) -> None:
    """Register (or with None, unregister) a pair of timing events recorded around one kernel.

    `start` / `stop`: TimingEvent, or torch.cuda.Event created with enable_timing=True and recorded once
    already so that its native handle exists.
    """
    a = None if start is None else C.c_void_p(start.cuda_event)
    b = None if stop is None else C.c_void_p(stop.cuda_event)
    _check(lib().qblora_profile_events(which, a, b), "qblora_profile_events")


def strerror(code: int) -> str:
    return lib().qblora_strerror(code).decode()


def _check(code: int, where: str) -> None:
    if code != OK:
        raise QBLoRAError(code, where)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class QWeight:
    """The triplet (codes, alpha, beta) of Eq. 1 on the device, plus the host-side C struct."""

    def __init__(self, d_out, d_in, block, codebook, codes, scales, beta=None, scale_mode=SCALES_FP32,
                 scale_codes=None, scale_step=None, scale_mid=None, scale_group=256, codes_tiled=None, block_rows=1):
        self.d_out, self.d_in, self.block = d_out, d_in, block
        self.block_rows = int(block_rows)       # 1: blocks of 64 inputs in a row; 8: blocks of 8 rows x 8 inputs
        self.codebook = np.asarray(codebook, np.float32)
        self.codes, self.scales, self.beta = codes, scales, beta
        self.scale_mode, self.scale_group = scale_mode, scale_group
        self.scale_codes, self.scale_step, self.scale_mid = scale_codes, scale_step, scale_mid
        self.codes_tiled = codes_tiled          # optional tile-ordered copy of the codes (forward fast path)

    def c_struct(self) -> CQWeight:
        s = CQWeight()
        s.d_out, s.d_in, s.block = self.d_out, self.d_in, self.block
        s.scale_mode, s.scale_group = self.scale_mode, self.scale_group
        s.block_rows = self.block_rows
        for j in range(16):
            s.codebook[j] = float(self.codebook[j])
        for name in ("codes", "scales", "beta", "scale_codes", "scale_step", "scale_mid", "codes_tiled"):
            t = getattr(self, name)
            setattr(s, name, None if t is None else t.data_ptr())
        return s

    def absorb(self, s: CQWeight) -> None:
        """Take back the scalar fields the library filled in."""
        self.d_out, self.d_in, self.block = s.d_out, s.d_in, s.block
        self.scale_mode, self.scale_group = s.scale_mode, s.scale_group
        self.codebook = np.array([s.codebook[j] for j in range(16)], np.float32)
        if not s.beta:
            self.beta = None


class Adapter:
    """Balanced adapter of Sec. 3.2: A bf16 [d_in/lambda1, R], B bf16 [R, d_out/lambda2], scaling s."""

    def __init__(self, A, B, lambda1, lambda2, s, scale_op=0):
        self.A, self.B, self.lambda1, self.lambda2, self.s = A, B, int(lambda1), int(lambda2), float(s)
        self.R = 0 if A is None else int(A.shape[1])
        self.scale_op = int(scale_op)        # OP_*: the scale operators of the ablation (Sec. 4.3)

    def c_struct(self) -> CAdapter:
        a = CAdapter()
        a.lambda1, a.lambda2, a.R, a.s = self.lambda1, self.lambda2, self.R, self.s
        a.scale_op = self.scale_op
        a.A = None if self.A is None else self.A.data_ptr()
        a.B = None if self.B is None else self.B.data_ptr()
        return a


def _adapter_ref(ad):
    if ad is None:
        return None, None
    s = ad.c_struct()
    return s, C.byref(s)


def qblora_codes_tiled_bytes(d_out: int, d_in: int) -> int:
    return int(lib().qblora_codes_tiled_bytes(d_out, d_in))


def qblora_prepack_codes(qw: QWeight) -> QWeight:
    """Fill (allocating if needed) the tile-ordered copy of the codes from the reference layout."""
    if qw.codes_tiled is None:
        qw.codes_tiled = torch.empty(qblora_codes_tiled_bytes(qw.d_out, qw.d_in), dtype=torch.uint8,
                                     device=qw.codes.device)
    s = qw.c_struct()
    _check(lib().qblora_prepack_codes(C.byref(s), _stream()), "qblora_prepack_codes")
    return qw


def qblora_quantize_blockwise(W: torch.Tensor, block: int = 64, quantizer: int = QUANT_ABSMAX_CODEBOOK,
                              codebook=None, scale_mode: int = SCALES_FP32, out: QWeight = None,
                              tiled: bool = True, block_rows: int = 1) -> QWeight:
    assert W.is_cuda and W.dtype == torch.float32 and W.is_contiguous() and W.dim() == 2
    d_out, d_in = W.shape
    dev = W.device
    if out is not None:                      # reuse the caller's buffers
        cb = np.zeros(16, np.float32) if codebook is None else np.ascontiguousarray(codebook, np.float32)
        s = out.c_struct()
        cb_ptr = None if codebook is None else cb.ctypes.data_as(C.c_void_p)
        rc = lib().qblora_quantize_blockwise(_ptr(W), d_out, d_in, block, quantizer, cb_ptr, scale_mode,
                                             C.byref(s), _stream())
        _check(rc, "qblora_quantize_blockwise")
        out.absorb(s)
        return out
    nblk = d_out * (d_in // max(block, 1))
    codes = torch.empty((d_out, d_in // 2), dtype=torch.uint8, device=dev)
    if block_rows == 8:                      # blocks of 8 rows x (block / 8) inputs: 8 x 8, or 8 x 4 with block = 32
        scales = torch.empty((d_out // 8, d_in // (block // 8)), dtype=torch.float32, device=dev)
    else:
        scales = torch.empty((d_out, d_in // max(block, 1)), dtype=torch.float32, device=dev)
    beta = torch.empty_like(scales) if quantizer == QUANT_MINMAX_INT4 else None
    sc = st = mid = None
    if scale_mode == SCALES_E4M3_GROUPED:
        ng = (nblk + 255) // 256
        sc = torch.empty(nblk, dtype=torch.uint8, device=dev)
        st = torch.empty(ng, dtype=torch.float32, device=dev)
        mid = torch.empty(ng, dtype=torch.float32, device=dev)
    cb = np.zeros(16, np.float32) if codebook is None else np.ascontiguousarray(codebook, np.float32)
    ct = None
    if tiled and block == 64 and d_in % 64 == 0:
        ct = torch.empty(qblora_codes_tiled_bytes(d_out, d_in), dtype=torch.uint8, device=dev)
    qw = QWeight(d_out, d_in, block, cb, codes, scales, beta, scale_mode, sc, st, mid, codes_tiled=ct,
                 block_rows=block_rows)
    s = qw.c_struct()
    cb_ptr = None if codebook is None else cb.ctypes.data_as(C.c_void_p)
    rc = lib().qblora_quantize_blockwise(_ptr(W), d_out, d_in, block, quantizer, cb_ptr, scale_mode, C.byref(s),
                                         _stream())
    _check(rc, "qblora_quantize_blockwise")
    qw.absorb(s)
    return qw


def qblora_dequantize_bf16(qw: QWeight) -> torch.Tensor:
    Wt = torch.empty((qw.d_out, qw.d_in), dtype=torch.bfloat16, device=qw.codes.device)
    s = qw.c_struct()
    _check(lib().qblora_dequantize_bf16(C.byref(s), _ptr(Wt), _stream()), "qblora_dequantize_bf16")
    return Wt


def qblora_linear_fwd_workspace_bytes(qw: QWeight, ad, T: int) -> int:
    s = qw.c_struct()
    a, aref = _adapter_ref(ad)
    return int(lib().qblora_linear_fwd_workspace_bytes(C.byref(s), aref, T))


def qblora_linear_bwd_workspace_bytes(qw: QWeight, ad, T: int) -> int:
    s = qw.c_struct()
    a, aref = _adapter_ref(ad)
    return int(lib().qblora_linear_bwd_workspace_bytes(C.byref(s), aref, T))


def _workspace(nbytes: int, device, workspace):
    if workspace is not None:
        return workspace
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def qblora_saved_bytes(ad, T: int) -> int:
    a, aref = _adapter_ref(ad)
    return int(lib().qblora_saved_bytes(aref, T))


def qblora_linear_fwd(qw: QWeight, ad, X: torch.Tensor, Y: torch.Tensor = None, workspace: torch.Tensor = None,
                      saved: torch.Tensor = None):
    """`saved` (uint8 tensor of qblora_saved_bytes()) selects qblora_linear_fwd_save."""
    assert X.is_cuda and X.dtype == torch.bfloat16 and X.is_contiguous() and X.shape[1] == qw.d_in
    T = X.shape[0]
    if Y is None:
        Y = torch.empty((T, qw.d_out), dtype=torch.bfloat16, device=X.device)
    ws = _workspace(qblora_linear_fwd_workspace_bytes(qw, ad, T), X.device, workspace)
    s = qw.c_struct()
    a, aref = _adapter_ref(ad)
    if saved is None:
        rc = lib().qblora_linear_fwd(C.byref(s), aref, _ptr(X), T, _ptr(Y), _ptr(ws), ws.numel(), _stream())
        _check(rc, "qblora_linear_fwd")
    else:
        assert saved.is_cuda and saved.numel() * saved.element_size() >= qblora_saved_bytes(ad, T)
        rc = lib().qblora_linear_fwd_save(C.byref(s), aref, _ptr(X), T, _ptr(Y), _ptr(saved), _ptr(ws), ws.numel(),
                                          _stream())
        _check(rc, "qblora_linear_fwd_save")
    return Y


def qblora_dense_min_tokens() -> int:
    return int(lib().qblora_dense_min_tokens())


def qblora_noalloc_scratch_bytes() -> int:
    return int(lib().qblora_noalloc_scratch_bytes())


def qblora_linear_fwd_noalloc(qw: QWeight, ad, X: torch.Tensor, Y: torch.Tensor):
    """qblora_linear_fwd on the library's own scratch array: the caller passes inputs and the output only."""
    assert X.is_cuda and X.dtype == torch.bfloat16 and X.is_contiguous() and X.shape[1] == qw.d_in
    assert Y.is_cuda and Y.dtype == torch.bfloat16 and Y.is_contiguous() and tuple(Y.shape) == (X.shape[0], qw.d_out)
    s = qw.c_struct()
    a, aref = _adapter_ref(ad)
    _check(lib().qblora_linear_fwd_noalloc(C.byref(s), aref, _ptr(X), X.shape[0], _ptr(Y), _stream()),
           "qblora_linear_fwd_noalloc")
    return Y


def qblora_linear_bwd(qw: QWeight, ad, X: torch.Tensor, dY: torch.Tensor, need_dx: bool = True,
                      need_grads: bool = True, dX=None, dA=None, dB=None, workspace: torch.Tensor = None,
                      saved: torch.Tensor = None):
    """`saved` (the buffer a forward call filled) selects qblora_linear_bwd_saved."""
    assert dY.is_cuda and dY.dtype == torch.bfloat16 and dY.is_contiguous() and dY.shape[1] == qw.d_out
    T = dY.shape[0]
    dev = dY.device
    if need_dx and dX is None:
        dX = torch.empty((T, qw.d_in), dtype=torch.bfloat16, device=dev)
    if need_grads and ad is not None and ad.R > 0:
        if dA is None:
            dA = torch.empty((qw.d_in // ad.lambda1, ad.R), dtype=torch.float32, device=dev)
        if dB is None:
            dB = torch.empty((ad.R, qw.d_out // ad.lambda2), dtype=torch.float32, device=dev)
    ws = _workspace(qblora_linear_bwd_workspace_bytes(qw, ad, T), dev, workspace)
    s = qw.c_struct()
    a, aref = _adapter_ref(ad)
    if saved is None:
        rc = lib().qblora_linear_bwd(C.byref(s), aref, _ptr(X), _ptr(dY), T, _ptr(dX), _ptr(dA), _ptr(dB), _ptr(ws),
                                     ws.numel(), _stream())
        _check(rc, "qblora_linear_bwd")
    else:
        rc = lib().qblora_linear_bwd_saved(C.byref(s), aref, _ptr(X), _ptr(dY), T, _ptr(saved), _ptr(dX), _ptr(dA),
                                           _ptr(dB), _ptr(ws), ws.numel(), _stream())
        _check(rc, "qblora_linear_bwd_saved")
    return dX, dA, dB


def qablora_linear_fwd(qw: QWeight, H: torch.Tensor, lambda1: int, lambda2: int, s: float, X: torch.Tensor,
                       Y: torch.Tensor = None, workspace: torch.Tensor = None):
    """Single-matrix adapter forward; H is bf16 [d_in/lambda1, d_out/lambda2]."""
    assert X.is_cuda and X.dtype == torch.bfloat16 and X.is_contiguous() and X.shape[1] == qw.d_in
    assert H.is_cuda and H.dtype == torch.bfloat16 and H.is_contiguous()
    assert tuple(H.shape) == (qw.d_in // lambda1, qw.d_out // lambda2)
    T = X.shape[0]
    if Y is None:
        Y = torch.empty((T, qw.d_out), dtype=torch.bfloat16, device=X.device)
    q = qw.c_struct()
    ws = _workspace(int(lib().qablora_linear_fwd_workspace_bytes(C.byref(q), lambda1, lambda2, T)), X.device, workspace)
    rc = lib().qablora_linear_fwd(C.byref(q), _ptr(H), lambda1, lambda2, s, _ptr(X), T, _ptr(Y), _ptr(ws), ws.numel(),
                                  _stream())
    _check(rc, "qablora_linear_fwd")
    return Y


def qablora_linear_bwd(qw: QWeight, H: torch.Tensor, lambda1: int, lambda2: int, s: float, X: torch.Tensor,
                       dY: torch.Tensor, need_dx: bool = True, need_dh: bool = True, dX=None, dH=None,
                       workspace: torch.Tensor = None):
    assert dY.is_cuda and dY.dtype == torch.bfloat16 and dY.is_contiguous() and dY.shape[1] == qw.d_out
    assert H.is_cuda and H.dtype == torch.bfloat16 and H.is_contiguous()
    T = dY.shape[0]
    dev = dY.device
    if need_dx and dX is None:
        dX = torch.empty((T, qw.d_in), dtype=torch.bfloat16, device=dev)
    if need_dh and dH is None:
        dH = torch.empty((qw.d_in // lambda1, qw.d_out // lambda2), dtype=torch.float32, device=dev)
    q = qw.c_struct()
    ws = _workspace(int(lib().qablora_linear_bwd_workspace_bytes(C.byref(q), lambda1, lambda2, T)), dev, workspace)
    rc = lib().qablora_linear_bwd(C.byref(q), _ptr(H), lambda1, lambda2, s, _ptr(X), _ptr(dY), T,
                                  _ptr(dX if need_dx else None), _ptr(dH if need_dh else None), _ptr(ws), ws.numel(),
                                  _stream())
    _check(rc, "qablora_linear_bwd")
    return (dX if need_dx else None), (dH if need_dh else None)


def qblora_tile_product(ad: Adapter, d_in: int, d_out: int, H: torch.Tensor = None, workspace=None):
    dev = ad.A.device
    if H is None:
        H = torch.empty((d_in // ad.lambda1, d_out // ad.lambda2), dtype=torch.float32, device=dev)
    a = ad.c_struct()
    need = int(lib().qblora_tile_product_workspace_bytes(C.byref(a), d_in, d_out))
    ws = _workspace(need, dev, workspace)
    rc = lib().qblora_tile_product(C.byref(a), d_in, d_out, _ptr(H), _ptr(ws), ws.numel(), _stream())
    _check(rc, "qblora_tile_product")
    return H


def qablora_merge_quantize(base: QWeight, H: torch.Tensor, lambda1: int, lambda2: int, s: float, mode: int,
                           out: QWeight = None) -> QWeight:
    assert H.is_cuda and H.dtype == torch.float32 and H.is_contiguous()
    dev = H.device
    if out is None:
        out = QWeight(base.d_out, base.d_in, base.block, base.codebook,
                      torch.empty_like(base.codes),
                      torch.empty(tuple(base.scales.shape), dtype=torch.float32, device=dev),
                      torch.empty(tuple(base.scales.shape), dtype=torch.float32, device=dev),
                      block_rows=base.block_rows)
    b = base.c_struct()
    o = out.c_struct()
    rc = lib().qablora_merge_quantize(C.byref(b), _ptr(H), lambda1, lambda2, s, mode, C.byref(o), _stream())
    _check(rc, "qablora_merge_quantize")
    beta_keep = out.beta
    out.absorb(o)
    out.beta = beta_keep
    out.scale_codes = out.scale_step = out.scale_mid = None
    out.codes_tiled = None
    return out


def qablora_merge_quantize_batch(bases, Hs, lambda1: int, lambda2: int, s: float, mode: int, outs=None):
    """qablora_merge_quantize for a list of weights (one launch per 8 where the kernels allow it)."""
    n = len(bases)
    assert len(Hs) == n and all(H.is_cuda and H.dtype == torch.float32 and H.is_contiguous() for H in Hs)
    if outs is None:
        outs = [QWeight(b.d_out, b.d_in, b.block, b.codebook, torch.empty_like(b.codes),
                        torch.empty(tuple(b.scales.shape), dtype=torch.float32, device=b.codes.device),
                        torch.empty(tuple(b.scales.shape), dtype=torch.float32, device=b.codes.device),
                        block_rows=b.block_rows) for b in bases]
    bs = [b.c_struct() for b in bases]
    os_ = [o.c_struct() for o in outs]
    Pq = C.POINTER(CQWeight)
    barr = (Pq * n)(*[C.pointer(x) for x in bs])
    oarr = (Pq * n)(*[C.pointer(x) for x in os_])
    harr = (C.c_void_p * n)(*[_ptr(H) for H in Hs])
    rc = lib().qablora_merge_quantize_batch(n, barr, harr, lambda1, lambda2, C.c_float(s), mode, oarr, _stream())
    _check(rc, "qablora_merge_quantize_batch")
    for o, oc in zip(outs, os_):
        beta_keep = o.beta
        o.absorb(oc)
        o.beta = beta_keep
        o.scale_codes = o.scale_step = o.scale_mid = None
        o.codes_tiled = None
    return outs


def qblora_merge_bf16(base: QWeight, H: torch.Tensor, lambda1: int, lambda2: int, s: float,
                      W16: torch.Tensor = None) -> torch.Tensor:
    """16-bit merge: bf16 [d_out, d_in] = w~ + s*dW."""
    assert H.is_cuda and H.dtype == torch.float32 and H.is_contiguous()
    if W16 is None:
        W16 = torch.empty((base.d_out, base.d_in), dtype=torch.bfloat16, device=H.device)
    b = base.c_struct()
    rc = lib().qblora_merge_bf16(C.byref(b), _ptr(H), lambda1, lambda2, s, _ptr(W16), _stream())
    _check(rc, "qblora_merge_bf16")
    return W16


def qblora_decode_pack(qw: QWeight) -> torch.Tensor:
    """One-off tile-ordered copy of codes / scales / offsets for qblora_linear_decode."""
    q = qw.c_struct()
    pack = torch.empty(int(lib().qblora_decode_pack_bytes(C.byref(q))), dtype=torch.uint8, device=qw.codes.device)
    _check(lib().qblora_decode_pack(C.byref(q), _ptr(pack), _stream()), "qblora_decode_pack")
    return pack


def qblora_linear_decode(qw: QWeight, X: torch.Tensor, Y: torch.Tensor = None, workspace: torch.Tensor = None,
                         pack: torch.Tensor = None):
    """Small- and mid-batch (T <= 256) forward of a quantized layer without adapter."""
    assert X.is_cuda and X.dtype == torch.bfloat16 and X.is_contiguous() and X.shape[1] == qw.d_in
    T = X.shape[0]
    if Y is None:
        Y = torch.empty((T, qw.d_out), dtype=torch.bfloat16, device=X.device)
    q = qw.c_struct()
    ws = _workspace(int(lib().qblora_linear_decode_tokens_workspace_bytes(C.byref(q), T)), X.device, workspace)
    rc = lib().qblora_linear_decode(C.byref(q), _ptr(pack), _ptr(X), T, _ptr(Y), _ptr(ws), ws.numel(), _stream())
    _check(rc, "qblora_linear_decode")
    return Y
