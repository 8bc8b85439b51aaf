"""GPU parity: adapted forward / backward against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2407_17029_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qb():
    from paper_2407_17029_amd import binding
    binding.lib()
    return binding


def _setup(qb, oracle, codebook, seed, T, d_out, d_in, R, lam1, lam2, s, minmax=False, grouped=False,
           channel_outliers=False):
    from gpu_util import f32_to_dev, bf16_to_dev, adapter_to_dev, OracleWeight
    L = synth.make_layer(seed, T, d_out, d_in, max(R, 8), lam1, lam2, channel_outliers=channel_outliers)
    if minmax:
        qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 64, qb.QUANT_MINMAX_INT4)
    else:
        qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook,
                                          qb.SCALES_E4M3_GROUPED if grouped else qb.SCALES_FP32)
    torch.cuda.synchronize()
    ow = OracleWeight(oracle, L.W, codebook, minmax, grouped).assert_same(qw)
    Wt = ow.dequantize(oracle, 2)                                         # the bf16 compute weight
    ad = adapter_to_dev(L, lam1, lam2, s) if R > 0 else None
    return L, qw, Wt, ad, bf16_to_dev(L.X), bf16_to_dev(L.dY)


CASES = [
    # T, d_out, d_in, R, lam1, lam2, s
    (256, 512, 512, 32, 2, 2, 1.0),          # the tiny configuration: rank 16, lambda 2
    (300, 320, 192, 16, 2, 2, 0.25),         # ragged token count, partial tiles in every dimension
    (77, 576, 832, 64, 4, 8, 2.0),           # lambda1 != lambda2 (the block-32 recommendation 4, 8)
    (513, 512, 1024, 128, 8, 8, 1.0),        # lambda 8, inner rank 128 (two K-extension steps)
    (130, 256, 256, 8, 1, 1, 1.0),           # lambda 1: plain LoRA, inner rank smaller than a K step
    (333, 384, 640, 128, 2, 2, 0.5),         # lambda 2 with inner rank 128: the narrow GEMMs read A^T / B unexpanded; ragged T
    (200, 512, 512, 96, 2, 2, 1.0),          # the same with a rank that leaves a partial column tile
    (8200, 256, 384, 224, 2, 2, 0.75),       # enough token tiles for the narrow GEMMs' 128-column form: ragged T, partial second column tile
]


@pytest.mark.parametrize("T,d_out,d_in,R,lam1,lam2,s", CASES)
def test_forward_parity(qb, oracle, codebook, T, d_out, d_in, R, lam1, lam2, s):
    from gpu_util import assert_close_bf16
    print(f"case fwd T={T} {d_out}x{d_in} R={R} lam=({lam1},{lam2})", flush=True)
    L, qw, Wt, ad, X, dY = _setup(qb, oracle, codebook, 500 + T, T, d_out, d_in, R, lam1, lam2, s)
    Y = qb.qblora_linear_fwd(qw, ad, X)
    torch.cuda.synchronize()
    ref = oracle.forward(Wt, L.X, L.A, L.B, lam1, lam2, s)
    assert_close_bf16(Y, ref, "Y")


@pytest.mark.parametrize("T,d_out,d_in,R,lam1,lam2,s", CASES)
def test_backward_parity(qb, oracle, codebook, T, d_out, d_in, R, lam1, lam2, s):
    from gpu_util import assert_close_bf16, assert_close_f32
    print(f"case bwd T={T} {d_out}x{d_in} R={R} lam=({lam1},{lam2})", flush=True)
    L, qw, Wt, ad, X, dY = _setup(qb, oracle, codebook, 600 + T, T, d_out, d_in, R, lam1, lam2, s)
    dX, dA, dB = qb.qblora_linear_bwd(qw, ad, X, dY)
    torch.cuda.synchronize()
    rX, rA, rB = oracle.backward(Wt, L.X, L.dY, L.A, L.B, lam1, lam2, s)
    assert_close_bf16(dX, rX, "dX")
    assert_close_f32(dA, rA, "dA")
    assert_close_f32(dB, rB, "dB")


def test_base_layer_without_adapter_and_b_zero(qb, oracle, codebook):
    from gpu_util import assert_close_bf16, bf16_to_dev
    T, d_out, d_in = 200, 320, 448
    L, qw, Wt, ad, X, dY = _setup(qb, oracle, codebook, 700, T, d_out, d_in, 16, 2, 2, 3.0)
    Y0 = qb.qblora_linear_fwd(qw, None, X)
    dX0, _, _ = qb.qblora_linear_bwd(qw, None, X, dY, need_grads=False)
    torch.cuda.synchronize()
    assert_close_bf16(Y0, oracle.forward(Wt, L.X, None, None, 1, 1, 0.0), "Y base")
    assert_close_bf16(dX0, oracle.backward(Wt, L.X, L.dY, None, None, 1, 1, 0.0)[0], "dX base")
    # B = 0: the adapter term vanishes and the scaling must not touch the base output
    ad0 = qb.Adapter(ad.A, torch.zeros_like(ad.B), 2, 2, 3.0)
    Yb = qb.qblora_linear_fwd(qw, ad0, X)
    torch.cuda.synchronize()
    assert torch.equal(Yb.view(torch.int16), Y0.view(torch.int16))


def test_forward_same_bits_with_and_without_tiled_codes(qb, oracle, codebook):
    T, d_out, d_in, R = 300, 576, 448, 32
    L, qw, Wt, ad, X, dY = _setup(qb, oracle, codebook, 740, T, d_out, d_in, R, 2, 2, 1.0)
    assert qw.codes_tiled is not None
    Y_tiled = qb.qblora_linear_fwd(qw, ad, X)
    tiled, qw.codes_tiled = qw.codes_tiled, None
    Y_ref = qb.qblora_linear_fwd(qw, ad, X)
    qw.codes_tiled = tiled
    torch.cuda.synchronize()
    assert torch.equal(Y_tiled.view(torch.int16), Y_ref.view(torch.int16))


@pytest.mark.parametrize("T,d_out,d_in,R,lam1,lam2,s", [CASES[1], CASES[3]])
def test_saved_activation_calls_match_the_plain_calls(qb, oracle, codebook, T, d_out, d_in, R, lam1, lam2, s):
    """Forward that keeps s*U + backward that reuses it: same bits as the recomputing calls, and
    parity with the oracle."""
    from gpu_util import assert_close_bf16, assert_close_f32
    print(f"case saved T={T} {d_out}x{d_in} R={R} lam=({lam1},{lam2})", flush=True)
    L, qw, Wt, ad, X, dY = _setup(qb, oracle, codebook, 900 + T, T, d_out, d_in, R, lam1, lam2, s)
    assert qb.qblora_saved_bytes(ad, T) == 2 * T * R * 2
    saved = torch.empty(qb.qblora_saved_bytes(ad, T), dtype=torch.uint8, device=X.device)
    Y_s = qb.qblora_linear_fwd(qw, ad, X, saved=saved)
    dX_s, dA_s, dB_s = qb.qblora_linear_bwd(qw, ad, X, dY, saved=saved)
    Y = qb.qblora_linear_fwd(qw, ad, X)
    dX, dA, dB = qb.qblora_linear_bwd(qw, ad, X, dY)
    torch.cuda.synchronize()
    assert torch.equal(Y_s.view(torch.int16), Y.view(torch.int16))
    assert torch.equal(dX_s.view(torch.int16), dX.view(torch.int16))
    assert torch.equal(dA_s, dA) and torch.equal(dB_s, dB)
    rX, rA, rB = oracle.backward(Wt, L.X, L.dY, L.A, L.B, lam1, lam2, s)
    assert_close_bf16(Y_s, oracle.forward(Wt, L.X, L.A, L.B, lam1, lam2, s), "Y")
    assert_close_bf16(dX_s, rX, "dX")
    assert_close_f32(dA_s, rA, "dA")
    assert_close_f32(dB_s, rB, "dB")
    # without an adapter the buffer is ignored; with one it is required
    assert qb.qblora_saved_bytes(None, T) == 0
    Y0 = qb.qblora_linear_fwd(qw, None, X, saved=saved)
    torch.cuda.synchronize()
    assert torch.equal(Y0.view(torch.int16), qb.qblora_linear_fwd(qw, None, X).view(torch.int16))


def test_minmax_base_with_beta(qb, oracle, codebook):
    from gpu_util import assert_close_bf16, assert_close_f32
    T, d_out, d_in, R = 150, 256, 384, 32
    L, qw, Wt, ad, X, dY = _setup(qb, oracle, codebook, 710, T, d_out, d_in, R, 2, 2, 1.0, minmax=True)
    Y = qb.qblora_linear_fwd(qw, ad, X)
    dX, dA, dB = qb.qblora_linear_bwd(qw, ad, X, dY)
    torch.cuda.synchronize()
    assert_close_bf16(Y, oracle.forward(Wt, L.X, L.A, L.B, 2, 2, 1.0), "Y")
    rX, rA, rB = oracle.backward(Wt, L.X, L.dY, L.A, L.B, 2, 2, 1.0)
    assert_close_bf16(dX, rX, "dX"); assert_close_f32(dA, rA, "dA"); assert_close_f32(dB, rB, "dB")


def test_grouped_scales_and_channel_outliers(qb, oracle, codebook):
    from gpu_util import assert_close_bf16, assert_close_f32
    T, d_out, d_in, R = 160, 512, 512, 64
    L, qw, Wt, ad, X, dY = _setup(qb, oracle, codebook, 720, T, d_out, d_in, R, 2, 2, 1.0, grouped=True,
                                  channel_outliers=True)
    Y = qb.qblora_linear_fwd(qw, ad, X)
    dX, dA, dB = qb.qblora_linear_bwd(qw, ad, X, dY)
    torch.cuda.synchronize()
    assert_close_bf16(Y, oracle.forward(Wt, L.X, L.A, L.B, 2, 2, 1.0), "Y")
    rX, rA, rB = oracle.backward(Wt, L.X, L.dY, L.A, L.B, 2, 2, 1.0)
    assert_close_bf16(dX, rX, "dX"); assert_close_f32(dA, rA, "dA"); assert_close_f32(dB, rB, "dB")


def test_empty_batch_and_errors(qb, oracle, codebook):
    from gpu_util import f32_to_dev, bf16_to_dev, DEV
    L, qw, Wt, ad, X, dY = _setup(qb, oracle, codebook, 730, 8, 128, 128, 16, 2, 2, 1.0)
    Y = qb.qblora_linear_fwd(qw, ad, X[:0].contiguous())
    assert Y.shape == (0, 128)
    dX, dA, dB = qb.qblora_linear_bwd(qw, ad, X[:0].contiguous(), dY[:0].contiguous())
    torch.cuda.synchronize()
    assert float(dA.abs().max()) == 0.0 and float(dB.abs().max()) == 0.0
    bad = qb.Adapter(ad.A, ad.B, 3, 2, 1.0)                      # 128 % 3 != 0
    with pytest.raises(qb.QBLoRAError) as e:
        qb.qblora_linear_fwd(qw, bad, X)
    assert e.value.code == -2
    with pytest.raises(qb.QBLoRAError) as e:
        qb.qblora_linear_fwd(qw, ad, X, workspace=torch.empty(16, dtype=torch.uint8, device=DEV))
    assert e.value.code == -4


# ---- the adapter term on its own scale --------------------------------------------------------------
# With the workloads' B ~ N(0, 0.01^2) the adapter is a few per cent of Y and dX, so the 1e-2 * rms bar of
# the cases above would let a sizeable error in it pass.  Here the adapter dominates: either the base weight
# is all zero (absmax 0 => w~ = 0, the output IS s * expand(pool(X) A B), and dX IS expand(dU A^T) / lambda1),
# or B ~ N(0, 0.5^2) on the usual base.  The bar then resolves the K-extension of both GEMM kernels: the scale
# s, the 1/lambda1 factor, the n / lambda2 and k / lambda1 row maps under partial tiles.
ADAPTER_CASES = CASES + [
    (300, 320, 448, 24, 4, 8, 0.5),          # lambda1 != lambda2 = 8, partial feature tile (320 = 256 + 64), ragged T
    (520, 832, 320, 40, 8, 4, 1.5),          # lambda1 = 8 > lambda2, partial tiles on both sides of the backward
    (257, 576, 576, 136, 2, 2, 1.0),         # inner rank 136: a partial third K-extension step
]


@pytest.mark.parametrize("zero_base", [True, False])
@pytest.mark.parametrize("T,d_out,d_in,R,lam1,lam2,s", ADAPTER_CASES)
def test_adapter_dominant_parity(qb, oracle, codebook, T, d_out, d_in, R, lam1, lam2, s, zero_base):
    from gpu_util import f32_to_dev, bf16_to_dev, assert_close_bf16, assert_close_f32, OracleWeight
    print(f"case adapter-dominant T={T} {d_out}x{d_in} R={R} lam=({lam1},{lam2}) zero_base={zero_base}", flush=True)
    L = synth.make_layer(1300 + T + R, T, d_out, d_in, R, lam1, lam2, b_std=0.5)
    W = np.zeros_like(L.W) if zero_base else L.W
    qw = qb.qblora_quantize_blockwise(f32_to_dev(W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook)
    torch.cuda.synchronize()
    Wt = OracleWeight(oracle, W, codebook).assert_same(qw).dequantize(oracle, 2)
    if zero_base:
        assert not Wt.any()
    ad = qb.Adapter(bf16_to_dev(L.A), bf16_to_dev(L.B), lam1, lam2, s)
    X, dY = bf16_to_dev(L.X), bf16_to_dev(L.dY)
    Y = qb.qblora_linear_fwd(qw, ad, X)
    dX, dA, dB = qb.qblora_linear_bwd(qw, ad, X, dY)
    torch.cuda.synchronize()
    ref = oracle.forward(Wt, L.X, L.A, L.B, lam1, lam2, s)
    rX, rA, rB = oracle.backward(Wt, L.X, L.dY, L.A, L.B, lam1, lam2, s)
    if not zero_base:
        # the adapter term is a large part of the output (a quarter to nine tenths of its energy, by s and R)
        base = oracle.forward(Wt, L.X, None, None, 1, 1, 0.0)
        assert np.mean((ref - base) ** 2) > 0.2 * np.mean(ref ** 2)
    assert_close_bf16(Y, ref, "Y (adapter-dominant)")
    assert_close_bf16(dX, rX, "dX (adapter-dominant)")
    assert_close_f32(dA, rA, "dA")
    assert_close_f32(dB, rB, "dB")


# ---- many tokens: the weight is dequantized once per call ---------------------------------------------
# From qblora_dense_min_tokens() tokens on, the forward / backward calls first write the bf16 compute weight
# (transposed for the backward) into their workspace and contract that.  Small widths with ragged token counts
# keep the oracle fast while the path sees partial tiles, every block geometry and scale format.
DENSE_CASES = [
    # extra tokens, d_out, d_in, R, lam1, lam2, s, minmax, grouped, block_rows
    (52, 320, 192, 16, 2, 2, 0.25, False, False, 1),       # ragged tokens, partial tiles in every dimension
    (256, 576, 832, 64, 4, 8, 2.0, False, True, 1),        # lambda1 != lambda2, double-quantized scales
    (1, 256, 384, 40, 2, 2, 1.0, True, False, 1),          # min-max base with offsets, one token beyond a tile
    (130, 320, 448, 24, 8, 8, 0.5, True, False, 8),        # 8 x 8 blocks with offsets
    (77, 512, 256, 0, 1, 1, 1.0, False, False, 8),         # 8 x 8 blocks, codebook base, no adapter
]


@pytest.mark.parametrize("extra,d_out,d_in,R,lam1,lam2,s,minmax,grouped,block_rows", DENSE_CASES)
def test_many_token_calls_dequantize_once(qb, oracle, codebook, extra, d_out, d_in, R, lam1, lam2, s, minmax, grouped,
                                          block_rows):
    from gpu_util import f32_to_dev, bf16_to_dev, assert_close_bf16, assert_close_f32, OracleWeight
    T = qb.qblora_dense_min_tokens() + extra
    print(f"case many tokens T={T} {d_out}x{d_in} R={R} lam=({lam1},{lam2}) minmax={minmax} grouped={grouped} "
          f"block_rows={block_rows}", flush=True)
    L = synth.make_layer(1500 + extra + d_out, T, d_out, d_in, max(R, 8), lam1, lam2, b_std=0.2)
    Wd = f32_to_dev(L.W)
    if minmax:
        qw = qb.qblora_quantize_blockwise(Wd, 64, qb.QUANT_MINMAX_INT4, block_rows=block_rows)
    else:
        qw = qb.qblora_quantize_blockwise(Wd, 64, qb.QUANT_ABSMAX_CODEBOOK, codebook,
                                          qb.SCALES_E4M3_GROUPED if grouped else qb.SCALES_FP32, block_rows=block_rows)
    torch.cuda.synchronize()
    Wt = OracleWeight(oracle, L.W, codebook, minmax, grouped, block_rows).assert_same(qw).dequantize(oracle, 2)
    ad = qb.Adapter(bf16_to_dev(L.A), bf16_to_dev(L.B), lam1, lam2, s) if R > 0 else None
    A, B = (L.A, L.B) if R > 0 else (None, None)
    X, dY = bf16_to_dev(L.X), bf16_to_dev(L.dY)
    assert qb.qblora_linear_fwd_workspace_bytes(qw, ad, T) >= 2 * d_out * d_in
    Y = qb.qblora_linear_fwd(qw, ad, X)
    dX, dA, dB = qb.qblora_linear_bwd(qw, ad, X, dY, need_grads=R > 0)
    torch.cuda.synchronize()
    assert_close_bf16(Y, oracle.forward(Wt, L.X, A, B, lam1, lam2, s if R > 0 else 0.0), "Y")
    rX, rA, rB = oracle.backward(Wt, L.X, L.dY, A, B, lam1, lam2, s if R > 0 else 0.0)
    assert_close_bf16(dX, rX, "dX")
    if R > 0:
        assert_close_f32(dA, rA, "dA")
        assert_close_f32(dB, rB, "dB")
    # the same bf16 weight either way: the form that rebuilds tiles in LDS (which the no-allocation entry point
    # always takes) gives the same bits
    Y2 = torch.empty_like(Y)
    qb.qblora_linear_fwd_noalloc(qw, ad, X, Y2)
    torch.cuda.synchronize()
    assert torch.equal(Y.view(torch.int16), Y2.view(torch.int16))
