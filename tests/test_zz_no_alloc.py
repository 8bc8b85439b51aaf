"""The forward entry point that allocates nothing (qblora_linear_fwd_noalloc): same bits as qblora_linear_fwd.

The library's own scratch array replaces the caller's workspace; it keeps the previous call's contents, so the
check runs two calls in a row, the second on a smaller problem, and a third on the first problem again.
"""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2407_17029_amd import synth

pytestmark = pytest.mark.gpu


def _case(qb, codebook, seed, T, d_out, d_in, R, lam, s, grouped):
    from gpu_util import f32_to_dev, bf16_to_dev, adapter_to_dev
    L = synth.make_layer(seed, T, d_out, d_in, R, lam, lam, b_std=0.5)
    qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook,
                                      qb.SCALES_E4M3_GROUPED if grouped else qb.SCALES_FP32)
    return L, qw, adapter_to_dev(L, lam, lam, s), bf16_to_dev(L.X)


def test_no_alloc_forward_matches_the_workspace_forward(oracle, codebook):
    from paper_2407_17029_amd import binding as qb
    from gpu_util import assert_close_bf16, OracleWeight
    qb.lib()
    limit = qb.qblora_noalloc_scratch_bytes()
    assert limit == 16 << 20
    big = _case(qb, codebook, 8100, 1500, 1024, 1536, 128, 2, 0.5, False)     # several tiles, ragged tokens
    small = _case(qb, codebook, 8101, 77, 320, 192, 16, 2, 2.0, True)         # smaller, grouped scales
    outs = []
    for name, (L, qw, ad, X) in (("first", big), ("second, smaller", small), ("first again", big)):
        print(f"no-alloc forward, {name}: T={X.shape[0]} {qw.d_out}x{qw.d_in} R={ad.R}", flush=True)
        assert qb.qblora_linear_fwd_workspace_bytes(qw, ad, X.shape[0]) <= limit
        Y = torch.full((X.shape[0], qw.d_out), float("nan"), dtype=torch.bfloat16, device=X.device)
        qb.qblora_linear_fwd_noalloc(qw, ad, X, Y)
        torch.cuda.synchronize()
        ref = qb.qblora_linear_fwd(qw, ad, X)
        torch.cuda.synchronize()
        assert torch.equal(Y.view(torch.int16), ref.view(torch.int16)), name
        outs.append(Y)
    assert torch.equal(outs[0].view(torch.int16), outs[2].view(torch.int16))
    # and against the oracle, like the workspace forward itself
    L, qw, ad, X = big
    Wt = OracleWeight(oracle, L.W, codebook).assert_same(qw).dequantize(oracle, 2)
    assert_close_bf16(outs[0], oracle.forward(Wt, L.X, L.A, L.B, 2, 2, 0.5), "Y (no-alloc forward)")
    # the base layer alone (no adapter) goes through the same array
    Y0 = torch.empty_like(outs[0])
    qb.qblora_linear_fwd_noalloc(qw, None, X, Y0)
    torch.cuda.synchronize()
    assert torch.equal(Y0.view(torch.int16), qb.qblora_linear_fwd(qw, None, X).view(torch.int16))


def test_no_alloc_forward_rejects_what_does_not_fit():
    from paper_2407_17029_amd import binding as qb
    L = qb.lib()
    qw = qb.CQWeight()
    qw.d_out, qw.d_in, qw.block = 8192, 8192, 64
    qw.codes = qw.scales = 0x1000
    dummy = C.c_void_p(0x1000)           # never dereferenced: rejected on the host
    ad = qb.CAdapter()
    ad.lambda1, ad.lambda2, ad.R, ad.s, ad.A, ad.B = 2, 2, 256, 1.0, 0x1000, 0x1000
    assert L.qblora_linear_fwd_workspace_bytes(C.byref(qw), C.byref(ad), 65536) > qb.qblora_noalloc_scratch_bytes()
    assert L.qblora_linear_fwd_noalloc(C.byref(qw), C.byref(ad), dummy, 65536, dummy, None) == -4
    assert L.qblora_linear_fwd_noalloc(C.byref(qw), C.byref(ad), None, 16, dummy, None) == -1
    assert L.qblora_linear_fwd_noalloc(C.byref(qw), C.byref(ad), dummy, 0, dummy, None) == 0
