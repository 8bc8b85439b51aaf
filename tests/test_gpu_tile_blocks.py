"""GPU parity for 8 x 8 quantization blocks (Sec. 3.3 / ablation "The balancing factor of QA-BLoRA": block 64
with lambda1 = lambda2 = 8): quantizers, standalone dequantize and the exact offset-shift merge, bit for bit."""
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


SHAPES = [(64, 64), (256, 512), (320, 832), (72, 1088), (1024, 4096)]


@pytest.mark.parametrize("d_out,d_in", SHAPES)
def test_quantizers_bit_exact(qb, oracle, codebook, d_out, d_in):
    from gpu_util import f32_to_dev, to_np
    print(f"case 8x8 quantize {d_out}x{d_in}", flush=True)
    W = synth.make_layer(1200 + d_out, 2, d_out, d_in, 8, 1, 1, channel_outliers=True).W
    qw = qb.qblora_quantize_blockwise(f32_to_dev(W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook, block_rows=8)
    qm = qb.qblora_quantize_blockwise(f32_to_dev(W), 64, qb.QUANT_MINMAX_INT4, block_rows=8)
    torch.cuda.synchronize()
    codes, absmax = oracle.quantize_codebook_tile(W, 8, 8, codebook)
    assert np.array_equal(to_np(qw.codes), codes)
    assert np.array_equal(to_np(qw.scales).view(np.uint32), absmax.view(np.uint32))
    cm, am, bm = oracle.quantize_minmax_tile(W, 8, 8)
    assert np.array_equal(to_np(qm.codes), cm)
    assert np.array_equal(to_np(qm.scales).view(np.uint32), am.view(np.uint32))
    assert np.array_equal(to_np(qm.beta).view(np.uint32), bm.view(np.uint32))
    # the tile-ordered copy of the codes has the same bytes as the re-layout of the reference copy
    ref = qb.QWeight(d_out, d_in, 64, qw.codebook, qw.codes, qw.scales, block_rows=8)
    qb.qblora_prepack_codes(ref)
    torch.cuda.synchronize()
    t1, t2 = to_np(qw.codes_tiled), to_np(ref.codes_tiled)
    full = (d_out // 256) * 256 * (d_in // 64) * 32          # whole row tiles (rows past d_out are unspecified)
    assert np.array_equal(t1[:full], t2[:full])
    # standalone dequantize (bf16 compute weight), against the oracle's own triplets (equal to the device's, above)
    for q, c_o, a_o, b_o, cb in ((qw, codes, absmax, None, codebook), (qm, cm, am, bm, synth.codebook_int4())):
        Wt = qb.qblora_dequantize_bf16(q)
        torch.cuda.synchronize()
        want = oracle.dequantize_tile(c_o, a_o, b_o, cb, 8, 8, 2)
        assert np.array_equal(Wt.float().cpu().numpy().astype(np.float64), want)


@pytest.mark.parametrize("lam1,lam2", [(8, 8), (16, 8), (8, 32)])
def test_offset_shift_merge_bit_exact(qb, oracle, lam1, lam2):
    from gpu_util import f32_to_dev, to_np
    d_out, d_in, s = 256, 512, 0.75
    W = synth.make_layer(1300 + lam1, 2, d_out, d_in, 8, 1, 1).W
    H = (np.random.default_rng(1300 + lam2).standard_normal((d_in // lam1, d_out // lam2)) * 0.02).astype(np.float32)
    for quantizer in (qb.QUANT_MINMAX_INT4, qb.QUANT_ABSMAX_CODEBOOK):
        cb = synth.codebook_nf4_style()
        base = qb.qblora_quantize_blockwise(f32_to_dev(W), 64, quantizer, cb, block_rows=8)
        merged = qb.qablora_merge_quantize(base, f32_to_dev(H), lam1, lam2, s, qb.MERGE_BETA_SHIFT)
        torch.cuda.synchronize()
        from gpu_util import OracleWeight
        ow = OracleWeight(oracle, W, cb, quantizer == qb.QUANT_MINMAX_INT4, block_rows=8).assert_same(base)
        want = oracle.merge_beta_shift_tile(ow.beta, H, d_out, d_in, 8, 8, lam1, lam2, s)
        assert np.array_equal(to_np(merged.beta).view(np.uint32), want.view(np.uint32))
        assert np.array_equal(to_np(merged.codes), to_np(base.codes))
        assert np.array_equal(to_np(merged.scales).view(np.uint32), to_np(base.scales).view(np.uint32))
        assert merged.block_rows == 8


def test_errors(qb, oracle, codebook):
    from gpu_util import f32_to_dev
    W = f32_to_dev(synth.make_layer(1400, 2, 64, 128, 8, 1, 1).W)
    base = qb.qblora_quantize_blockwise(W, 64, qb.QUANT_MINMAX_INT4, block_rows=8)
    H = torch.zeros((128 // 4, 64 // 8), dtype=torch.float32, device=W.device)
    with pytest.raises(qb.QBLoRAError):                      # lambda1 = 4 splits an 8-wide block
        qb.qablora_merge_quantize(base, H, 4, 8, 1.0, qb.MERGE_BETA_SHIFT)
    qb.qablora_merge_quantize(base, H, 4, 8, 1.0, qb.MERGE_REQUANT_MINMAX)      # ... which the requantizing merge takes
    with pytest.raises(qb.QBLoRAError):                      # d_out must be a multiple of 8
        qb.qblora_quantize_blockwise(W[:60].contiguous(), 64, qb.QUANT_MINMAX_INT4, block_rows=8)
    with pytest.raises(qb.QBLoRAError):
        qb.qblora_quantize_blockwise(W, 64, qb.QUANT_ABSMAX_CODEBOOK, codebook, qb.SCALES_E4M3_GROUPED, block_rows=8)


def _layer(qb, oracle, codebook, seed, T, d_out, d_in, R, lam1, lam2, minmax):
    from gpu_util import f32_to_dev, bf16_to_dev, OracleWeight
    L = synth.make_layer(seed, T, d_out, d_in, max(R, 8), lam1, lam2)
    if minmax:
        qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 64, qb.QUANT_MINMAX_INT4, block_rows=8)
    else:
        qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook, block_rows=8)
    torch.cuda.synchronize()
    ow = OracleWeight(oracle, L.W, codebook, minmax, block_rows=8).assert_same(qw)
    qw.oracle_weight = ow                                   # the oracle's triplets, for the tests that go on from them
    Wt = ow.dequantize(oracle, 2)                           # the bf16 compute weight
    return L, qw, Wt, bf16_to_dev(L.X), bf16_to_dev(L.dY)


LAYER_CASES = [
    # T, d_out, d_in, R, lam1, lam2, s, minmax
    (256, 512, 512, 32, 2, 2, 1.0, False),
    (300, 320, 192, 16, 2, 2, 0.25, True),          # ragged token count, partial tiles in every dimension
    (77, 576, 832, 64, 4, 8, 2.0, False),
    (513, 512, 1024, 128, 8, 8, 1.0, True),
]


@pytest.mark.parametrize("T,d_out,d_in,R,lam1,lam2,s,minmax", LAYER_CASES)
def test_two_matrix_layer_on_8x8_blocks(qb, oracle, codebook, T, d_out, d_in, R, lam1, lam2, s, minmax):
    from gpu_util import assert_close_bf16, assert_close_f32, adapter_to_dev
    print(f"case 8x8 layer T={T} {d_out}x{d_in} R={R} lam=({lam1},{lam2}) minmax={minmax}", flush=True)
    L, qw, Wt, X, dY = _layer(qb, oracle, codebook, 1500 + T, T, d_out, d_in, R, lam1, lam2, minmax)
    ad = adapter_to_dev(L, lam1, lam2, s)
    Y = qb.qblora_linear_fwd(qw, ad, X)
    dX, dA, dB = qb.qblora_linear_bwd(qw, ad, X, dY)
    Y0 = qb.qblora_linear_fwd(qw, None, X)
    torch.cuda.synchronize()
    assert_close_bf16(Y, oracle.forward(Wt, L.X, L.A, L.B, lam1, lam2, s), "Y")
    assert_close_bf16(Y0, oracle.forward(Wt, L.X, None, None, 1, 1, 0.0), "Y base")
    rX, rA, rB = oracle.backward(Wt, L.X, L.dY, L.A, L.B, lam1, lam2, s)
    assert_close_bf16(dX, rX, "dX")
    assert_close_f32(dA, rA, "dA")
    assert_close_f32(dB, rB, "dB")


@pytest.mark.parametrize("T,d_out,d_in,lam1,lam2", [(200, 512, 512, 8, 8), (77, 320, 896, 16, 8)])
def test_quantization_aware_loop_on_8x8_blocks(qb, oracle, T, d_out, d_in, lam1, lam2):
    """Sec. 3.3 end to end: single-matrix adapter on an INT4 base with 8 x 8 blocks (forward and backward
    against the oracle), offset-shift merge, and the merged INT4 layer reproduces the adapted layer."""
    from gpu_util import bf16_to_dev, f32_to_dev, to_np, assert_close_bf16, assert_close_f32, bf16_to_f64
    s = 0.75
    L, qw, Wt, X, dY = _layer(qb, oracle, None, 1600 + T, T, d_out, d_in, 8, lam1, lam2, True)
    Hb = synth.f32_to_bf16_bits((np.random.default_rng(1600 + T).standard_normal((d_in // lam1, d_out // lam2)) * 0.02)
                                .astype(np.float32))
    H = bf16_to_dev(Hb)
    Y = qb.qablora_linear_fwd(qw, H, lam1, lam2, s, X)
    dX, dH = qb.qablora_linear_bwd(qw, H, lam1, lam2, s, X, dY)
    torch.cuda.synchronize()
    assert_close_bf16(Y, oracle.qa_forward(Wt, L.X, Hb, lam1, lam2, s), "Y")
    rX, rH = oracle.qa_backward(Wt, L.X, L.dY, Hb, lam1, lam2, s)
    assert_close_bf16(dX, rX, "dX")
    assert_close_f32(dH, rH, "dH")
    # merge: beta' = beta + s*H/lambda1, codes and alpha untouched; then plain INT4 forward
    merged = qb.qablora_merge_quantize(qw, H.float().contiguous(), lam1, lam2, s, qb.MERGE_BETA_SHIFT)
    Ym = qb.qblora_linear_fwd(merged, None, X)
    torch.cuda.synchronize()
    from helpers import bf16_exact
    ow = qw.oracle_weight
    beta2 = oracle.merge_beta_shift_tile(ow.beta, bf16_exact(Hb).astype(np.float32), d_out, d_in, 8, 8, lam1, lam2, s)
    assert np.array_equal(to_np(merged.beta).view(np.uint32), beta2.view(np.uint32))
    assert np.array_equal(to_np(merged.codes), ow.codes)
    Wm = oracle.dequantize_tile(ow.codes, ow.scales, beta2, synth.codebook_int4(), 8, 8, 2)
    assert_close_bf16(Ym, oracle.forward(Wm, L.X, None, None, 1, 1, 0.0), "Y merged")
    # the merged layer against the adapted layer: they differ by the bf16 rounding of the merged weight only
    ref = oracle.qa_forward(ow.dequantize(oracle, 0), L.X, Hb, lam1, lam2, s)
    err = np.abs(bf16_to_f64(Ym) - ref)
    rms = np.sqrt((ref ** 2).mean())
    assert np.sqrt((err ** 2).mean()) <= 5e-3 * rms and err.max() <= 4e-2 * rms


@pytest.mark.parametrize("T", [1, 5, 16, 40, 130])       # above 16: the mid-batch form of the same call
# (the tall case: more than 512 row groups, where few tokens of an INT4 model take the form with all of X in LDS)
@pytest.mark.parametrize("d_out,d_in,minmax", [(512, 1024, True), (328, 832, True), (256, 512, False), (8264, 192, True),
                                               (16456, 128, True)])
def test_small_batch_inference_on_8x8_blocks(qb, oracle, codebook, T, d_out, d_in, minmax):
    """Merged-model inference (Sec. 3.3) on 8 x 8 blocks: the small-batch kernel contracts the bf16 compute
    weight bf16(fma(c, alpha, beta)), like the training forward; with and without the tile-ordered code copy."""
    from gpu_util import assert_close_bf16, to_np
    print(f"case 8x8 decode T={T} {d_out}x{d_in} minmax={minmax}", flush=True)
    L, qw, Wt, X, dY = _layer(qb, oracle, codebook, 1700 + T + d_out, T, d_out, d_in, 8, 1, 1, minmax)
    Y = qb.qblora_linear_decode(qw, X)
    pack = qb.qblora_decode_pack(qw)
    Yp = qb.qblora_linear_decode(qw, X, pack=pack)
    torch.cuda.synchronize()
    ref = oracle.forward(Wt, L.X, None, None, 1, 1, 0.0)
    assert_close_bf16(Y, ref, "Y")
    assert torch.equal(Y, Yp)


@pytest.mark.parametrize("minmax", [True, False])
@pytest.mark.parametrize("d_out,d_in,lam1,lam2,s", [(512, 512, 2, 2, 1.0), (328, 832, 4, 2, 0.5), (96, 192, 3, 2, 1.5),
                                                     (256, 1024, 8, 8, 0.75), (64, 64, 1, 1, 1.0)])
def test_requantizing_and_16bit_merge_on_8x8_blocks(qb, oracle, codebook, d_out, d_in, lam1, lam2, s, minmax):
    """Sec. 3.3 with lambdas that do not cover whole 8 x 8 blocks: the merge requantizes every block (or writes the
    16-bit weight); codes, scales, offsets and bf16 bits against the oracle, bit for bit."""
    from gpu_util import f32_to_dev, to_np, bf16_to_f64
    print(f"case 8x8 merge {d_out}x{d_in} lam=({lam1},{lam2}) minmax={minmax}", flush=True)
    L, qw, Wt, X, dY = _layer(qb, oracle, codebook, 1800 + d_out + lam1, 4, d_out, d_in, 8, 1, 1, minmax)
    ow = qw.oracle_weight
    H = synth.normal_f32(1801, 1, (d_in // lam1, d_out // lam2), 0.01)
    out = qb.qablora_merge_quantize(qw, f32_to_dev(H), lam1, lam2, s, qb.MERGE_REQUANT_MINMAX)
    W16 = qb.qblora_merge_bf16(qw, f32_to_dev(H), lam1, lam2, s)
    torch.cuda.synchronize()
    co, ao, bo = oracle.merge_requant_tile(ow.codes, ow.scales, ow.beta, ow.cb, H, 8, 8, lam1, lam2, s)
    bits = lambda a: np.ascontiguousarray(a).view(np.uint32).reshape(-1)
    assert out.block_rows == 8
    assert np.array_equal(to_np(out.codes), co)
    assert np.array_equal(bits(to_np(out.scales)), bits(ao)) and np.array_equal(bits(to_np(out.beta)), bits(bo))
    assert np.array_equal(out.codebook, np.arange(16, dtype=np.float32))
    ref16 = oracle.merge_bf16_tile(ow.codes, ow.scales, ow.beta, ow.cb, H, 8, 8, lam1, lam2, s)
    assert np.array_equal(to_np(W16.view(torch.int16)).view(np.uint16), ref16)
    # the merged INT4 model runs through the small-batch call like any other 8 x 8 weight
    Ym = qb.qblora_linear_decode(out, X)
    torch.cuda.synchronize()
    from gpu_util import assert_close_bf16
    Wm = oracle.dequantize_tile(co, ao, bo, synth.codebook_int4(), 8, 8, 2)
    assert_close_bf16(Ym, oracle.forward(Wm, L.X, None, None, 1, 1, 0.0), "Y (merged, 8x8)")


# ---- blocks of 8 output rows x 4 inputs (block size 32; the other block shape of Sec. 3.3) ------------------------

def _layer84(qb, oracle, codebook, seed, T, d_out, d_in, R, lam1, lam2, minmax):
    from gpu_util import f32_to_dev, bf16_to_dev, OracleWeight
    L = synth.make_layer(seed, T, d_out, d_in, max(R, 8), lam1, lam2)
    if minmax:
        qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 32, qb.QUANT_MINMAX_INT4, block_rows=8)
    else:
        qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 32, qb.QUANT_ABSMAX_CODEBOOK, codebook, block_rows=8)
    torch.cuda.synchronize()
    ow = OracleWeight(oracle, L.W, codebook, minmax, block_rows=8, block_cols=4).assert_same(qw)    # quantizers: bit for bit
    qw.oracle_weight = ow
    return L, qw, ow.dequantize(oracle, 2), bf16_to_dev(L.X), bf16_to_dev(L.dY)


@pytest.mark.parametrize("minmax", [True, False])
@pytest.mark.parametrize("d_out,d_in", [(64, 64), (328, 832), (512, 1088)])
def test_quantize_and_dequantize_on_8x4_blocks(qb, oracle, codebook, d_out, d_in, minmax):
    from gpu_util import to_np
    print(f"case 8x4 quantize {d_out}x{d_in} minmax={minmax}", flush=True)
    L, qw, Wt, X, dY = _layer84(qb, oracle, codebook, 1900 + d_out, 4, d_out, d_in, 8, 1, 1, minmax)
    assert qw.block == 32 and tuple(qw.scales.shape) == (d_out // 8, d_in // 4)
    W16 = qb.qblora_dequantize_bf16(qw)
    torch.cuda.synchronize()
    from helpers import bf16_exact
    assert np.array_equal(bf16_exact(to_np(W16.view(torch.int16)).view(np.uint16)), Wt)      # Eq. 1, one rounding


@pytest.mark.parametrize("T,d_out,d_in,R,lam1,lam2,s,minmax", [(77, 320, 192, 16, 2, 2, 0.25, True),
                                                            (300, 576, 832, 64, 4, 8, 2.0, False),
                                                            (2100, 512, 1024, 32, 4, 8, 1.0, True)])
def test_two_matrix_layer_on_8x4_blocks(qb, oracle, codebook, T, d_out, d_in, R, lam1, lam2, s, minmax):
    """Forward and backward: at any token count the call dequantizes the weight once (there is no in-kernel form for
    this block shape) and contracts that."""
    from gpu_util import assert_close_bf16, assert_close_f32, adapter_to_dev
    print(f"case 8x4 layer T={T} {d_out}x{d_in} R={R} lam=({lam1},{lam2}) minmax={minmax}", flush=True)
    L, qw, Wt, X, dY = _layer84(qb, oracle, codebook, 1950 + T, T, d_out, d_in, R, lam1, lam2, minmax)
    ad = adapter_to_dev(L, lam1, lam2, s)
    Y = qb.qblora_linear_fwd(qw, ad, X)
    dX, dA, dB = qb.qblora_linear_bwd(qw, ad, X, dY)
    torch.cuda.synchronize()
    assert_close_bf16(Y, oracle.forward(Wt, L.X, L.A, L.B, lam1, lam2, s), "Y")
    rX, rA, rB = oracle.backward(Wt, L.X, L.dY, L.A, L.B, lam1, lam2, s)
    assert_close_bf16(dX, rX, "dX"); assert_close_f32(dA, rA, "dA"); assert_close_f32(dB, rB, "dB")


def test_quantization_aware_loop_on_8x4_blocks(qb, oracle, codebook):
    """Sec. 3.3 at (lambda1, lambda2) = (4, 8): single-matrix training calls, then the offset-shift merge, exact because
    every 8 x 4 block lies in one adapter tile; the requantizing and 16-bit merges for lambdas that split blocks."""
    from gpu_util import f32_to_dev, to_np, bf16_to_dev, assert_close_bf16, assert_close_f32
    from helpers import bf16_exact
    T, d_out, d_in, lam1, lam2, s = 200, 256, 512, 4, 8, 0.75
    L, qw, Wt, X, dY = _layer84(qb, oracle, codebook, 1990, T, d_out, d_in, 8, lam1, lam2, True)
    ow = qw.oracle_weight
    Hb = synth.f32_to_bf16_bits((np.random.default_rng(1991).standard_normal((d_in // lam1, d_out // lam2)) * 0.05)
                                .astype(np.float32))
    H = bf16_to_dev(Hb)
    Y = qb.qablora_linear_fwd(qw, H, lam1, lam2, s, X)
    dX, dH = qb.qablora_linear_bwd(qw, H, lam1, lam2, s, X, dY)
    torch.cuda.synchronize()
    assert_close_bf16(Y, oracle.qa_forward(Wt, L.X, Hb, lam1, lam2, s), "Y")
    rX, rH = oracle.qa_backward(Wt, L.X, L.dY, Hb, lam1, lam2, s)
    assert_close_bf16(dX, rX, "dX"); assert_close_f32(dH, rH, "dH")
    Hf = bf16_exact(Hb).astype(np.float32)
    merged = qb.qablora_merge_quantize(qw, f32_to_dev(Hf), lam1, lam2, s, qb.MERGE_BETA_SHIFT)
    torch.cuda.synchronize()
    want = oracle.merge_beta_shift_tile(ow.beta, Hf, d_out, d_in, 8, 4, lam1, lam2, s)
    assert np.array_equal(to_np(merged.beta).view(np.uint32), want.view(np.uint32))
    assert np.array_equal(to_np(merged.codes), ow.codes) and merged.block == 32 and merged.block_rows == 8
    with pytest.raises(qb.QBLoRAError):                      # lambda1 = 2 splits a 4-wide block
        qb.qablora_merge_quantize(qw, torch.zeros((d_in // 2, d_out // 8), device=X.device), 2, 8, s, qb.MERGE_BETA_SHIFT)
    H2 = synth.normal_f32(1992, 1, (d_in // 2, d_out // 2), 0.01)
    out = qb.qablora_merge_quantize(qw, f32_to_dev(H2), 2, 2, s, qb.MERGE_REQUANT_MINMAX)
    W16 = qb.qblora_merge_bf16(qw, f32_to_dev(H2), 2, 2, s)
    torch.cuda.synchronize()
    co, ao, bo = oracle.merge_requant_tile(ow.codes, ow.scales, ow.beta, ow.cb, H2, 8, 4, 2, 2, s)
    bits = lambda a: np.ascontiguousarray(a).view(np.uint32).reshape(-1)
    assert np.array_equal(to_np(out.codes), co)
    assert np.array_equal(bits(to_np(out.scales)), bits(ao)) and np.array_equal(bits(to_np(out.beta)), bits(bo))
    assert np.array_equal(to_np(W16.view(torch.int16)).view(np.uint16),
                          oracle.merge_bf16_tile(ow.codes, ow.scales, ow.beta, ow.cb, H2, 8, 4, 2, 2, s))
    # inference on the merged model (and on the base): the mid-batch kernel at every token count, with and without
    # the tile-ordered code copy
    for weight, codes_o, a_o, b_o in ((merged, ow.codes, ow.scales, want), (out, co, ao, bo)):
        Wm = oracle.dequantize_tile(codes_o, a_o, b_o, synth.codebook_int4(), 8, 4, 2)
        pack = qb.qblora_decode_pack(weight)
        for Tn in (1, 16, 40, 200):
            Yd = qb.qblora_linear_decode(weight, X[:Tn].contiguous())
            Yp = qb.qblora_linear_decode(weight, X[:Tn].contiguous(), pack=pack)
            torch.cuda.synchronize()
            assert_close_bf16(Yd, oracle.forward(Wm, L.X[:Tn], None, None, 1, 1, 0.0), f"Y (8x4 inference, T={Tn})")
            assert torch.equal(Yd, Yp)
    with pytest.raises(qb.QBLoRAError):                      # the forward on the library's own scratch does not take the shape
        qb.qblora_linear_fwd_noalloc(qw, None, X, torch.empty((T, d_out), dtype=torch.bfloat16, device=X.device))
