#!/usr/bin/env python3
"""Per-kernel timings of the library beyond the benchmark step: the streaming kernels on the large layer
shapes (where launch overhead no longer dominates) and the rows built next to the hot path.

    python -m paper_2407_17029_amd.kernel_bench [merge] [quantize] [decode] [qablora] [tile8]

Each measurement is one JSON line: 10 warm-up launches, then 50 back-to-back launches between two HIP events on
the current stream, algorithmic bytes or flops as defined in the design notes, and the fraction of the MI355X
peak (HBM 8000 GB/s, bf16 MFMA 2500 TFLOP/s).  `us` is with warm caches (the 256 MB last-level cache holds the
operands of the smaller shapes between launches); `cold_us` (streaming kernels) rotates the launches over
enough operand sets to exceed that cache, so every launch reads from HBM.  The one-off re-layouts
(`prepack`, `decode_pack`) are lines of their own.  The
short kernels are launched through the C ABI with arguments marshalled once, so that the host keeps ahead
of the GPU (the Python wrappers cost ~25 us a call).
"""
from __future__ import annotations

import ctypes as C
import json
import sys

import numpy as np
import torch

from . import binding as qb
from . import synth

HBM_GBS, MFMA_TFLOPS = 8000.0, 2500.0
SHAPES = [(4096, 4096), (11008, 4096), (22016, 8192)]          # 7B attention, 7B MLP up, 65B MLP up
DEV = "cuda:0"


def timed(fn, iters=50, warm=10):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(iters):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / iters * 1e-3                      # seconds per launch


def timed_rotating(fns, iters=50, warm=10):
    """Like timed(), the launches cycling through `fns` (one per operand set)."""
    n = len(fns)
    for i in range(warm):
        fns[i % n]()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for i in range(iters):
        fns[i % n]()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / iters * 1e-3


def n_sets(bytes_per_set, cache_bytes=256 * 2**20):
    """Operand sets needed so that a set has left the last-level cache when its turn comes again."""
    return max(2, int(np.ceil(2 * cache_bytes / max(bytes_per_set, 1))) + 1)


def emit(**kw):
    print(json.dumps(kw), flush=True)


def bench_quantize():
    cb = synth.codebook_nf4_style()
    for d_out, d_in in SHAPES:
        W = torch.randn(d_out, d_in, device=DEV) * 0.02
        qw = qb.qblora_quantize_blockwise(W, 64, qb.QUANT_ABSMAX_CODEBOOK, cb, tiled=False)
        q, cbp = qw.c_struct(), np.ascontiguousarray(cb, np.float32)
        args = (qb._ptr(W), d_out, d_in, 64, qb.QUANT_ABSMAX_CODEBOOK, cbp.ctypes.data_as(C.c_void_p), qb.SCALES_FP32,
                C.byref(q), qb._stream())
        s = timed(lambda: qb.lib().qblora_quantize_blockwise(*args))
        nbytes = d_out * d_in * (4 + 0.5 + 4 / 64)
        # cold: every launch reads another copy of W
        Ws = [W] + [W.clone() for _ in range(n_sets(4 * d_out * d_in) - 1)]
        fns = []
        for Wi in Ws:
            ai = (qb._ptr(Wi),) + args[1:]
            fns.append(lambda ai=ai: qb.lib().qblora_quantize_blockwise(*ai))
        sc = timed_rotating(fns)
        emit(kernel="quantize_codebook", shape=[d_out, d_in], us=round(s * 1e6, 1), GBps=round(nbytes / s / 1e9, 1),
             frac_hbm=round(nbytes / s / 1e9 / HBM_GBS, 3), cold_us=round(sc * 1e6, 1), cold_sets=len(Ws),
             cold_frac_hbm=round(nbytes / sc / 1e9 / HBM_GBS, 3))
        del W, qw, Ws, fns


def bench_merge():
    cb = synth.codebook_nf4_style()
    for d_out, d_in in SHAPES:
        for lam in (2, 8):
            W = torch.randn(d_out, d_in, device=DEV) * 0.02
            qw = qb.qblora_quantize_blockwise(W, 64, qb.QUANT_ABSMAX_CODEBOOK, cb, tiled=False)
            H = torch.randn(d_in // lam, d_out // lam, device=DEV) * 0.01
            out = qb.qablora_merge_quantize(qw, H, lam, lam, 1.0, qb.MERGE_REQUANT_MINMAX)
            b, o = qw.c_struct(), out.c_struct()
            args = (C.byref(b), qb._ptr(H), lam, lam, C.c_float(1.0), qb.MERGE_REQUANT_MINMAX, C.byref(o), qb._stream())
            s = timed(lambda: qb.lib().qablora_merge_quantize(*args))
            nbytes = d_out * d_in * (0.5 + 4 / 64 + 4.0 / (lam * lam) + 0.5 + 8 / 64)
            # cold: every launch works on another copy of the weight, of H and of the output
            keep, fns = [], []
            for _ in range(n_sets(nbytes) - 1):
                qi = qb.qblora_quantize_blockwise(W, 64, qb.QUANT_ABSMAX_CODEBOOK, cb, tiled=False)
                Hi = H.clone()
                oi = qb.qablora_merge_quantize(qi, Hi, lam, lam, 1.0, qb.MERGE_REQUANT_MINMAX)
                bi, ooi = qi.c_struct(), oi.c_struct()
                ai = (C.byref(bi), qb._ptr(Hi), lam, lam, C.c_float(1.0), qb.MERGE_REQUANT_MINMAX, C.byref(ooi), qb._stream())
                keep.append((qi, Hi, oi, bi, ooi))
                fns.append(lambda ai=ai: qb.lib().qablora_merge_quantize(*ai))
            fns.append(lambda: qb.lib().qablora_merge_quantize(*args))
            sc = timed_rotating(fns)
            emit(kernel="merge_requant", shape=[d_out, d_in], lam=lam, us=round(s * 1e6, 1),
                 GBps=round(nbytes / s / 1e9, 1), frac_hbm=round(nbytes / s / 1e9 / HBM_GBS, 3),
                 cold_us=round(sc * 1e6, 1), cold_sets=len(fns), cold_frac_hbm=round(nbytes / sc / 1e9 / HBM_GBS, 3))
            del W, qw, H, out, keep, fns


def bench_decode():
    for d_out, d_in in SHAPES:
        W = torch.randn(d_out, d_in, device=DEV) * 0.02
        qw = qb.qblora_quantize_blockwise(W, 64, qb.QUANT_MINMAX_INT4, tiled=False)
        pack = qb.qblora_decode_pack(qw)
        qp = qw.c_struct()
        sp = timed(lambda: qb.lib().qblora_decode_pack(C.byref(qp), qb._ptr(pack), qb._stream()), iters=10, warm=2)
        emit(kernel="decode_pack (one-off)", shape=[d_out, d_in], us=round(sp * 1e6, 1))
        for T in (1, 4, 16):
            X = torch.randn(T, d_in, device=DEV).to(torch.bfloat16)
            Y = torch.empty(T, d_out, dtype=torch.bfloat16, device=DEV)
            q = qw.c_struct()
            for name, pk in (("packed", pack), ("row-major", None)):
                args = (C.byref(q), qb._ptr(pk), qb._ptr(X), T, qb._ptr(Y), None, 0, qb._stream())
                s = timed(lambda: qb.lib().qblora_linear_decode(*args), iters=50)
                nbytes = d_out * d_in * (0.5 + 8 / 64) + 2 * T * (d_in + d_out)
                emit(kernel="w4_decode", layout=name, shape=[d_out, d_in], T=T, us=round(s * 1e6, 1),
                     GBps=round(nbytes / s / 1e9, 1), frac_hbm=round(nbytes / s / 1e9 / HBM_GBS, 3))
        del W, qw, pack


def bench_qablora():
    cb = synth.codebook_nf4_style()
    T, d_out, d_in = 8192, 4096, 4096
    W = torch.randn(d_out, d_in, device=DEV) * 0.02
    qw = qb.qblora_quantize_blockwise(W, 64, qb.QUANT_ABSMAX_CODEBOOK, cb)
    X = torch.randn(T, d_in, device=DEV).to(torch.bfloat16)
    dY = torch.randn(T, d_out, device=DEV).to(torch.bfloat16)
    Y = torch.empty_like(dY)
    dX = torch.empty_like(X)
    for l1, l2 in ((8, 8), (4, 8), (2, 2)):
        H = (torch.randn(d_in // l1, d_out // l2, device=DEV) * 0.02).to(torch.bfloat16)
        dH = torch.empty(d_in // l1, d_out // l2, device=DEV)
        f = timed(lambda: qb.qablora_linear_fwd(qw, H, l1, l2, 1.0, X, Y), iters=10)
        b = timed(lambda: qb.qablora_linear_bwd(qw, H, l1, l2, 1.0, X, dY, True, True, dX, dH), iters=10)
        flops = 4.0 * T * d_in * d_out + 6.0 * T * (d_in // l1) * (d_out // l2)
        emit(kernel="qablora_fwd+bwd", shape=[d_out, d_in], T=T, lam=[l1, l2], fwd_us=round(f * 1e6, 1),
             bwd_us=round(b * 1e6, 1), TFLOPs=round(flops / (f + b) / 1e12, 1),
             frac_mfma=round(flops / (f + b) / 1e12 / MFMA_TFLOPS, 3))


def bench_tile8():
    """The quantization-aware loop on 8 x 8 quantization blocks (block 64 with lambda1 = lambda2 = 8): min-max INT4
    quantizer, single-matrix forward / backward, the exact offset-shift merge, small-batch inference."""
    T, d_out, d_in, l1, l2 = 8192, 4096, 4096, 8, 8
    W = torch.randn(d_out, d_in, device=DEV) * 0.02
    qw = qb.qblora_quantize_blockwise(W, 64, qb.QUANT_MINMAX_INT4, block_rows=8, tiled=True)
    q = qw.c_struct()
    args = (qb._ptr(W), d_out, d_in, 64, qb.QUANT_MINMAX_INT4, None, qb.SCALES_FP32, C.byref(q), qb._stream())
    s = timed(lambda: qb.lib().qblora_quantize_blockwise(*args))
    nbytes = d_out * d_in * (4 + 0.5 + 8 / 64)
    emit(kernel="quantize_minmax 8x8 blocks (+ tile-ordered code copy)", shape=[d_out, d_in], us=round(s * 1e6, 1),
         GBps=round(nbytes / s / 1e9, 1), frac_hbm=round(nbytes / s / 1e9 / HBM_GBS, 3))
    X = torch.randn(T, d_in, device=DEV).to(torch.bfloat16)
    dY = torch.randn(T, d_out, device=DEV).to(torch.bfloat16)
    Y = torch.empty_like(dY)
    dX = torch.empty_like(X)
    H = (torch.randn(d_in // l1, d_out // l2, device=DEV) * 0.02).to(torch.bfloat16)
    dH = torch.empty(d_in // l1, d_out // l2, device=DEV)
    f = timed(lambda: qb.qablora_linear_fwd(qw, H, l1, l2, 1.0, X, Y), iters=10)
    b = timed(lambda: qb.qablora_linear_bwd(qw, H, l1, l2, 1.0, X, dY, True, True, dX, dH), iters=10)
    flops = 4.0 * T * d_in * d_out + 6.0 * T * (d_in // l1) * (d_out // l2)
    emit(kernel="qablora_fwd+bwd 8x8 blocks", shape=[d_out, d_in], T=T, lam=[l1, l2], fwd_us=round(f * 1e6, 1),
         bwd_us=round(b * 1e6, 1), TFLOPs=round(flops / (f + b) / 1e12, 1),
         frac_mfma=round(flops / (f + b) / 1e12 / MFMA_TFLOPS, 3))
    Hf = H.float().contiguous()
    merged = qb.qablora_merge_quantize(qw, Hf, l1, l2, 1.0, qb.MERGE_BETA_SHIFT)
    bq, o = qw.c_struct(), merged.c_struct()
    margs = (C.byref(bq), qb._ptr(Hf), l1, l2, C.c_float(1.0), qb.MERGE_BETA_SHIFT, C.byref(o), qb._stream())
    s = timed(lambda: qb.lib().qablora_merge_quantize(*margs))
    nb = d_out * d_in // 64
    nbytes = d_out * d_in * 0.5 * 2 + nb * 4 * 4 + Hf.numel() * 4           # codes and alpha copied, beta shifted
    emit(kernel="merge_beta_shift 8x8 blocks (codes + alpha copied)", shape=[d_out, d_in], us=round(s * 1e6, 1),
         GBps=round(nbytes / s / 1e9, 1), frac_hbm=round(nbytes / s / 1e9 / HBM_GBS, 3))
    for d_out2, d_in2 in ((4096, 4096), (22016, 8192)):
        W2 = torch.randn(d_out2, d_in2, device=DEV) * 0.02
        q2 = qb.qblora_quantize_blockwise(W2, 64, qb.QUANT_MINMAX_INT4, block_rows=8, tiled=False)
        pack = qb.qblora_decode_pack(q2)
        for Tn in (1, 16):
            Xs = torch.randn(Tn, d_in2, device=DEV).to(torch.bfloat16)
            Ys = torch.empty(Tn, d_out2, dtype=torch.bfloat16, device=DEV)
            qs = q2.c_struct()
            dargs = (C.byref(qs), qb._ptr(pack), qb._ptr(Xs), Tn, qb._ptr(Ys), None, 0, qb._stream())
            s = timed(lambda: qb.lib().qblora_linear_decode(*dargs), iters=50)
            nbytes = d_out2 * d_in2 * (0.5 + 8 / 64) + 2 * Tn * (d_in2 + d_out2)
            emit(kernel="w4_decode 8x8 blocks", layout="packed", shape=[d_out2, d_in2], T=Tn, us=round(s * 1e6, 1),
                 GBps=round(nbytes / s / 1e9, 1), frac_hbm=round(nbytes / s / 1e9 / HBM_GBS, 3))
        del W2, q2, pack


def main(argv):
    qb.lib()
    torch.cuda.set_device(0)
    what = argv or ["quantize", "merge", "decode", "qablora", "tile8"]
    for w in what:
        {"quantize": bench_quantize, "merge": bench_merge, "decode": bench_decode, "qablora": bench_qablora,
         "tile8": bench_tile8}[w]()
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
