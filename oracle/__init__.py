"""ctypes front end of the CPU oracle (oracle/qblora_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The product package never imports this module and
this module never imports the product's binding.  All arrays are numpy; bf16
tensors are uint16 bit patterns; forward/backward results are fp64.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "qblora_oracle.cpp")
# ORACLE_SANITIZE=1 selects a build of its own under AddressSanitizer + UndefinedBehaviorSanitizer (host code
# only; run the CPU tests with the sanitizer runtimes preloaded, see README)
_SANITIZE = os.environ.get("ORACLE_SANITIZE", "") not in ("", "0")
_LIB = os.path.join(_DIR, "libqblora_oracle_san.so" if _SANITIZE else "libqblora_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with g++ (plain -O2, no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-pthread", "-ffp-contract=off",
               "-fno-fast-math", "-o", _LIB, _SRC]
        if _SANITIZE:
            cmd[1:2] = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = C.CDLL(_LIB)
        _lib.oracle_e4m3_decode.restype = C.c_float
        _lib.oracle_e4m3_decode.argtypes = [C.c_uint8]
        _lib.oracle_e4m3_encode.restype = C.c_uint8
        _lib.oracle_e4m3_encode.argtypes = [C.c_float]
        _lib.oracle_get_threads.restype = C.c_int
        _lib.oracle_merge_beta_shift.restype = C.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


i64 = C.c_int64


def set_threads(n: int) -> None:
    lib().oracle_set_threads(C.c_int(n))


def get_threads() -> int:
    return int(lib().oracle_get_threads())


def quantize_codebook(W, block, codebook):
    W = _c(W, np.float32); cb = _c(codebook, np.float32)
    d_out, d_in = W.shape
    assert d_in % block == 0 and d_in % 2 == 0
    codes = np.zeros((d_out, d_in // 2), np.uint8)
    absmax = np.zeros((d_out, d_in // block), np.float32)
    lib().oracle_quantize_codebook(_p(W), i64(d_out), i64(d_in), C.c_int(block), _p(cb), _p(codes), _p(absmax))
    return codes, absmax


def quantize_minmax(W, block):
    W = _c(W, np.float32)
    d_out, d_in = W.shape
    assert d_in % block == 0 and d_in % 2 == 0
    codes = np.zeros((d_out, d_in // 2), np.uint8)
    alpha = np.zeros((d_out, d_in // block), np.float32)
    beta = np.zeros((d_out, d_in // block), np.float32)
    lib().oracle_quantize_minmax(_p(W), i64(d_out), i64(d_in), C.c_int(block), _p(codes), _p(alpha), _p(beta))
    return codes, alpha, beta


def e4m3_decode(code: int) -> float:
    return float(lib().oracle_e4m3_decode(C.c_uint8(code)))


def e4m3_encode(x: float) -> int:
    return int(lib().oracle_e4m3_encode(C.c_float(x)))


def scales_double_quantize(scales, group=256):
    s = _c(scales, np.float32).reshape(-1)
    n = s.size
    ng = (n + group - 1) // group
    sc = np.zeros(n, np.uint8); step = np.zeros(ng, np.float32); mid = np.zeros(ng, np.float32)
    lib().oracle_scales_double_quantize(_p(s), i64(n), C.c_int(group), _p(sc), _p(step), _p(mid))
    return sc, step, mid


def scales_double_dequantize(scale_codes, step, mid, group=256):
    sc = _c(scale_codes, np.uint8).reshape(-1)
    step = _c(step, np.float32); mid = _c(mid, np.float32)
    out = np.zeros(sc.size, np.float32)
    lib().oracle_scales_double_dequantize(_p(sc), i64(sc.size), C.c_int(group), _p(step), _p(mid), _p(out))
    return out


def dequantize(codes, alpha, beta, codebook, block, mode):
    """mode 0: exact fp64 formula; 1: fp32 arithmetic; 2: fp32 then rounded to bf16."""
    codes = _c(codes, np.uint8); alpha = _c(alpha, np.float32); cb = _c(codebook, np.float32)
    beta = None if beta is None else _c(beta, np.float32)
    d_out, d_in = codes.shape[0], codes.shape[1] * 2
    Wt = np.zeros((d_out, d_in), np.float64)
    lib().oracle_dequantize(_p(codes), _p(alpha), _p(beta), _p(cb), i64(d_out), i64(d_in), C.c_int(block),
                            C.c_int(mode), _p(Wt))
    return Wt


def forward(Wt, X, A, B, lam1, lam2, s, want_intermediates=False):
    Wt = _c(Wt, np.float64); X = _c(X, np.uint16)
    d_out, d_in = Wt.shape
    T = X.shape[0]
    assert X.shape[1] == d_in
    Y = np.zeros((T, d_out), np.float64)
    if A is None:
        lib().oracle_forward(_p(Wt), i64(d_out), i64(d_in), _p(X), i64(T), None, None, i64(0), C.c_int(1),
                             C.c_int(1), C.c_double(0.0), _p(Y), None, None, None)
        return (Y, None, None, None) if want_intermediates else Y
    A = _c(A, np.uint16); B = _c(B, np.uint16)
    R = A.shape[1]
    assert d_in % lam1 == 0 and d_out % lam2 == 0
    assert A.shape == (d_in // lam1, R) and B.shape == (R, d_out // lam2)
    P = U = V = None
    if want_intermediates:
        P = np.zeros((T, d_in // lam1)); U = np.zeros((T, R)); V = np.zeros((T, d_out // lam2))
    lib().oracle_forward(_p(Wt), i64(d_out), i64(d_in), _p(X), i64(T), _p(A), _p(B), i64(R), C.c_int(lam1),
                         C.c_int(lam2), C.c_double(s), _p(Y), _p(P), _p(U), _p(V))
    return (Y, P, U, V) if want_intermediates else Y


def backward(Wt, X, dY, A, B, lam1, lam2, s, compute_dx=True, compute_dab=True, d_out=None, d_in=None):
    """Wt may be None (with d_out, d_in given) when compute_dx is False: dA, dB do not involve the base weight."""
    X = _c(X, np.uint16); dY = _c(dY, np.uint16)
    if Wt is None:
        assert not compute_dx and d_out is not None and d_in is not None
    else:
        Wt = _c(Wt, np.float64)
        d_out, d_in = Wt.shape
    T = X.shape[0]
    assert X.shape == (T, d_in) and dY.shape == (T, d_out)
    dX = np.zeros((T, d_in), np.float64) if compute_dx else None
    if A is None:
        lib().oracle_backward(_p(Wt), i64(d_out), i64(d_in), _p(X), _p(dY), i64(T), None, None, i64(0),
                              C.c_int(1), C.c_int(1), C.c_double(0.0), C.c_int(int(compute_dx)), _p(dX), None, None)
        return dX, None, None
    A = _c(A, np.uint16); B = _c(B, np.uint16)
    R = A.shape[1]
    assert A.shape == (d_in // lam1, R) and B.shape == (R, d_out // lam2)
    dA = np.zeros(A.shape, np.float64) if compute_dab else None
    dB = np.zeros(B.shape, np.float64) if compute_dab else None
    lib().oracle_backward(_p(Wt), i64(d_out), i64(d_in), _p(X), _p(dY), i64(T), _p(A), _p(B), i64(R),
                          C.c_int(lam1), C.c_int(lam2), C.c_double(s), C.c_int(int(compute_dx)),
                          _p(dX), _p(dA), _p(dB))
    return dX, dA, dB


OP_AVGPOOL_REPEAT, OP_TRUNCATE_PAD0, OP_SAMPLE_ZEROFILL = 0, 1, 2


def forward_op(Wt, X, A, B, lam1, lam2, s, op):
    """Adapted forward with one of the scale-operator pairs of the ablation (op 0 is the default pair)."""
    Wt = _c(Wt, np.float64); X = _c(X, np.uint16); A = _c(A, np.uint16); B = _c(B, np.uint16)
    d_out, d_in = Wt.shape
    T, R = X.shape[0], A.shape[1]
    assert X.shape[1] == d_in and d_in % lam1 == 0 and d_out % lam2 == 0 and op in (0, 1, 2)
    assert A.shape == (d_in // lam1, R) and B.shape == (R, d_out // lam2)
    Y = np.zeros((T, d_out), np.float64)
    lib().oracle_forward_op(_p(Wt), i64(d_out), i64(d_in), _p(X), i64(T), _p(A), _p(B), i64(R), C.c_int(lam1),
                            C.c_int(lam2), C.c_int(op), C.c_double(s), _p(Y))
    return Y


def backward_op(Wt, X, dY, A, B, lam1, lam2, s, op, compute_dx=True, compute_dab=True, d_out=None, d_in=None):
    X = _c(X, np.uint16); dY = _c(dY, np.uint16); A = _c(A, np.uint16); B = _c(B, np.uint16)
    if Wt is None:
        assert not compute_dx and d_out is not None and d_in is not None
    else:
        Wt = _c(Wt, np.float64)
        d_out, d_in = Wt.shape
    T, R = X.shape[0], A.shape[1]
    assert X.shape == (T, d_in) and dY.shape == (T, d_out) and op in (0, 1, 2)
    assert A.shape == (d_in // lam1, R) and B.shape == (R, d_out // lam2)
    dX = np.zeros((T, d_in), np.float64) if compute_dx else None
    dA = np.zeros(A.shape, np.float64) if compute_dab else None
    dB = np.zeros(B.shape, np.float64) if compute_dab else None
    lib().oracle_backward_op(_p(Wt), i64(d_out), i64(d_in), _p(X), _p(dY), i64(T), _p(A), _p(B), i64(R),
                             C.c_int(lam1), C.c_int(lam2), C.c_int(op), C.c_double(s), C.c_int(int(compute_dx)),
                             _p(dX), _p(dA), _p(dB))
    return dX, dA, dB


def qa_forward(Wt, X, H, lam1, lam2, s):
    """Single-matrix adapter (QA-BLoRA): H is bf16 bits [d_in/lam1, d_out/lam2]."""
    Wt = _c(Wt, np.float64); X = _c(X, np.uint16); H = _c(H, np.uint16)
    d_out, d_in = Wt.shape
    T = X.shape[0]
    assert X.shape == (T, d_in) and H.shape == (d_in // lam1, d_out // lam2)
    Y = np.zeros((T, d_out), np.float64)
    lib().oracle_qa_forward(_p(Wt), i64(d_out), i64(d_in), _p(X), i64(T), _p(H), C.c_int(lam1), C.c_int(lam2),
                            C.c_double(s), _p(Y))
    return Y


def qa_backward(Wt, X, dY, H, lam1, lam2, s, compute_dx=True, compute_dh=True, d_out=None, d_in=None):
    """Wt may be None (with d_out, d_in given) when compute_dx is False."""
    X = _c(X, np.uint16); dY = _c(dY, np.uint16); H = _c(H, np.uint16)
    if Wt is None:
        assert not compute_dx and d_out is not None and d_in is not None
    else:
        Wt = _c(Wt, np.float64)
        d_out, d_in = Wt.shape
    T = X.shape[0]
    assert X.shape == (T, d_in) and dY.shape == (T, d_out) and H.shape == (d_in // lam1, d_out // lam2)
    dX = np.zeros((T, d_in), np.float64) if compute_dx else None
    dH = np.zeros(H.shape, np.float64) if compute_dh else None
    lib().oracle_qa_backward(_p(Wt), i64(d_out), i64(d_in), _p(X), _p(dY), i64(T), _p(H), C.c_int(lam1),
                             C.c_int(lam2), C.c_double(s), C.c_int(int(compute_dx)), _p(dX), _p(dH))
    return dX, dH


def tile_product(A, B):
    A = _c(A, np.uint16); B = _c(B, np.uint16)
    rows, R = A.shape
    cols = B.shape[1]
    assert B.shape[0] == R
    H = np.zeros((rows, cols), np.float64)
    lib().oracle_tile_product(_p(A), _p(B), i64(rows), i64(R), i64(cols), _p(H))
    return H


def delta_weight(H, lam1, lam2):
    """Full-size delta weight in the paper's [d_in, d_out] layout."""
    H = _c(H, np.float64)
    d_in, d_out = H.shape[0] * lam1, H.shape[1] * lam2
    dW = np.zeros((d_in, d_out), np.float64)
    lib().oracle_delta_weight(_p(H), i64(d_in), i64(d_out), C.c_int(lam1), C.c_int(lam2), _p(dW))
    return dW


def merge_beta_shift(beta, H, d_out, d_in, block, lam1, lam2, s):
    H = _c(H, np.float32)
    assert H.shape == (d_in // lam1, d_out // lam2)
    beta = None if beta is None else _c(beta, np.float32)
    out = np.zeros((d_out, d_in // block), np.float32)
    rc = lib().oracle_merge_beta_shift(_p(beta), _p(H), i64(d_out), i64(d_in), C.c_int(block), C.c_int(lam1),
                                       C.c_int(lam2), C.c_float(s), _p(out))
    if rc != 0:
        raise ValueError("beta-shift merge needs every quantization block inside one (lam1 x lam2) tile")
    return out


def quantize_codebook_tile(W, br, bc, codebook):
    """Codebook quantizer on blocks of br output rows x bc inputs; absmax is [d_out/br, d_in/bc]."""
    W = _c(W, np.float32); cb = _c(codebook, np.float32)
    d_out, d_in = W.shape
    assert d_out % br == 0 and d_in % bc == 0 and d_in % 2 == 0
    codes = np.zeros((d_out, d_in // 2), np.uint8)
    absmax = np.zeros((d_out // br, d_in // bc), np.float32)
    lib().oracle_quantize_codebook_tile(_p(W), i64(d_out), i64(d_in), C.c_int(br), C.c_int(bc), _p(cb), _p(codes),
                                        _p(absmax))
    return codes, absmax


def quantize_minmax_tile(W, br, bc):
    W = _c(W, np.float32)
    d_out, d_in = W.shape
    assert d_out % br == 0 and d_in % bc == 0 and d_in % 2 == 0
    codes = np.zeros((d_out, d_in // 2), np.uint8)
    alpha = np.zeros((d_out // br, d_in // bc), np.float32)
    beta = np.zeros((d_out // br, d_in // bc), np.float32)
    lib().oracle_quantize_minmax_tile(_p(W), i64(d_out), i64(d_in), C.c_int(br), C.c_int(bc), _p(codes), _p(alpha),
                                      _p(beta))
    return codes, alpha, beta


def dequantize_tile(codes, alpha, beta, codebook, br, bc, mode):
    codes = _c(codes, np.uint8); alpha = _c(alpha, np.float32); cb = _c(codebook, np.float32)
    beta = None if beta is None else _c(beta, np.float32)
    d_out, d_in = codes.shape[0], codes.shape[1] * 2
    assert alpha.size == (d_out // br) * (d_in // bc)
    Wt = np.zeros((d_out, d_in), np.float64)
    lib().oracle_dequantize_tile(_p(codes), _p(alpha), _p(beta), _p(cb), i64(d_out), i64(d_in), C.c_int(br),
                                 C.c_int(bc), C.c_int(mode), _p(Wt))
    return Wt


def merge_beta_shift_tile(beta, H, d_out, d_in, br, bc, lam1, lam2, s):
    H = _c(H, np.float32)
    assert H.shape == (d_in // lam1, d_out // lam2)
    beta = None if beta is None else _c(beta, np.float32)
    out = np.zeros((d_out // br, d_in // bc), np.float32)
    lib().oracle_merge_beta_shift_tile.restype = C.c_int
    rc = lib().oracle_merge_beta_shift_tile(_p(beta), _p(H), i64(d_out), i64(d_in), C.c_int(br), C.c_int(bc),
                                            C.c_int(lam1), C.c_int(lam2), C.c_float(s), _p(out))
    if rc != 0:
        raise ValueError("offset-shift merge needs every quantization block inside one (lam1 x lam2) tile")
    return out


def merge_requant(codes, alpha, beta, codebook, H, block, lam1, lam2, s):
    codes = _c(codes, np.uint8); alpha = _c(alpha, np.float32); cb = _c(codebook, np.float32)
    beta = None if beta is None else _c(beta, np.float32)
    H = _c(H, np.float32)
    d_out, d_in = codes.shape[0], codes.shape[1] * 2
    assert H.shape == (d_in // lam1, d_out // lam2)
    co = np.zeros_like(codes); ao = np.zeros_like(alpha); bo = np.zeros_like(alpha)
    lib().oracle_merge_requant(_p(codes), _p(alpha), _p(beta), _p(cb), _p(H), i64(d_out), i64(d_in),
                               C.c_int(block), C.c_int(lam1), C.c_int(lam2), C.c_float(s), _p(co), _p(ao), _p(bo))
    return co, ao, bo


def merge_bf16(codes, alpha, beta, codebook, H, block, lam1, lam2, s):
    """16-bit merge: bf16 bit patterns of w~ + s*dW, [d_out, d_in]."""
    codes = _c(codes, np.uint8); alpha = _c(alpha, np.float32); cb = _c(codebook, np.float32)
    beta = None if beta is None else _c(beta, np.float32)
    H = _c(H, np.float32)
    d_out, d_in = codes.shape[0], codes.shape[1] * 2
    assert H.shape == (d_in // lam1, d_out // lam2)
    W16 = np.zeros((d_out, d_in), np.uint16)
    lib().oracle_merge_bf16(_p(codes), _p(alpha), _p(beta), _p(cb), _p(H), i64(d_out), i64(d_in), C.c_int(block),
                            C.c_int(lam1), C.c_int(lam2), C.c_float(s), _p(W16))
    return W16


def merge_requant_tile(codes, alpha, beta, codebook, H, br, bc, lam1, lam2, s):
    """Requantizing merge on br x bc blocks: alpha / beta are [d_out/br, d_in/bc]."""
    codes = _c(codes, np.uint8); alpha = _c(alpha, np.float32); cb = _c(codebook, np.float32)
    beta = None if beta is None else _c(beta, np.float32)
    H = _c(H, np.float32)
    d_out, d_in = codes.shape[0], codes.shape[1] * 2
    assert H.shape == (d_in // lam1, d_out // lam2) and alpha.size == (d_out // br) * (d_in // bc)
    co = np.zeros_like(codes); ao = np.zeros_like(alpha); bo = np.zeros_like(alpha)
    lib().oracle_merge_requant_tile(_p(codes), _p(alpha), _p(beta), _p(cb), _p(H), i64(d_out), i64(d_in), C.c_int(br),
                                    C.c_int(bc), C.c_int(lam1), C.c_int(lam2), C.c_float(s), _p(co), _p(ao), _p(bo))
    return co, ao, bo


def merge_bf16_tile(codes, alpha, beta, codebook, H, br, bc, lam1, lam2, s):
    """16-bit merge on br x bc blocks: bf16 bit patterns [d_out, d_in]."""
    codes = _c(codes, np.uint8); alpha = _c(alpha, np.float32); cb = _c(codebook, np.float32)
    beta = None if beta is None else _c(beta, np.float32)
    H = _c(H, np.float32)
    d_out, d_in = codes.shape[0], codes.shape[1] * 2
    assert H.shape == (d_in // lam1, d_out // lam2) and alpha.size == (d_out // br) * (d_in // bc)
    W16 = np.zeros((d_out, d_in), np.uint16)
    lib().oracle_merge_bf16_tile(_p(codes), _p(alpha), _p(beta), _p(cb), _p(H), i64(d_out), i64(d_in), C.c_int(br),
                                 C.c_int(bc), C.c_int(lam1), C.c_int(lam2), C.c_float(s), _p(W16))
    return W16
