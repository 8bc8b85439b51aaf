"""GPU parity: small-batch forward of a quantized layer (merged-model inference) against the fp64 oracle."""
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


@pytest.mark.parametrize("base", ["codebook", "minmax", "grouped"])
# (the last two: long rows, where the activations of a few tokens no longer fit the workgroup's LDS copy)
@pytest.mark.parametrize("T,d_out,d_in", [(1, 512, 512), (3, 320, 192), (8, 1000, 1088), (16, 256, 2048), (5, 40, 64),
                                         (8, 96, 4096), (4, 80, 8192), (2, 16448, 128), (7, 16440, 192), (12, 16448, 128)])   # (the last three: tall layers, two row groups per workgroup)
def test_decode_parity(qb, oracle, codebook, T, d_out, d_in, base):
    from gpu_util import f32_to_dev, bf16_to_dev, assert_close_bf16, OracleWeight
    print(f"case decode T={T} {d_out}x{d_in} base={base}", flush=True)
    L = synth.make_layer(2000 + T, T, d_out, d_in, 8, 1, 1)
    if base == "minmax":
        qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 64, qb.QUANT_MINMAX_INT4)
        cb = synth.codebook_int4()
    else:
        qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook,
                                          qb.SCALES_E4M3_GROUPED if base == "grouped" else qb.SCALES_FP32)
        cb = codebook
    X = bf16_to_dev(L.X)
    Y = qb.qblora_linear_decode(qw, X)
    Yp = qb.qblora_linear_decode(qw, X, pack=qb.qblora_decode_pack(qw))
    torch.cuda.synchronize()
    if base != "minmax":
        assert torch.equal(Y.view(torch.int16), Yp.view(torch.int16))   # tile-ordered pack: same sums, same bits
    ow = OracleWeight(oracle, L.W, codebook, base == "minmax", base == "grouped").assert_same(qw)
    Wt = ow.dequantize(oracle, 3)                                        # the inference weight: alpha*bf16(c)+beta
    ref = oracle.forward(Wt, L.X, None, None, 1, 1, 0.0)
    assert_close_bf16(Y, ref, "Y")
    # the pack of an INT4 model with offsets is contracted without the code table (operand 128 + c, the 128
    # taken off through the block's activation sum): other roundings, same result within the bar
    assert_close_bf16(Yp, ref, "Y (packed)")


@pytest.mark.parametrize("base", ["codebook", "grouped"])
@pytest.mark.parametrize("T,d_out,d_in", [(4, 1024, 2048), (16, 512, 4096), (1, 768, 11008)])
def test_decode_against_the_exact_weight(qb, oracle, codebook, T, d_out, d_in, base):
    """Eq. 1 as written (fp64 alpha * codebook[c], nothing rounded) against the small-batch kernel on a base with a
    non-integer codebook: the kernel's bf16 rounding of the table entries (and of nothing else before the fp32
    sums) must stay inside the same bar as every other output, so the bar does not rest on the rounded-table
    weight the other decode tests compare with."""
    from gpu_util import f32_to_dev, bf16_to_dev, assert_close_bf16, OracleWeight
    print(f"case decode vs exact Eq. 1 T={T} {d_out}x{d_in} base={base}", flush=True)
    L = synth.make_layer(2300 + T, T, d_out, d_in, 8, 1, 1)
    qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook,
                                      qb.SCALES_E4M3_GROUPED if base == "grouped" else qb.SCALES_FP32)
    X = bf16_to_dev(L.X)
    Y = qb.qblora_linear_decode(qw, X)
    Yp = qb.qblora_linear_decode(qw, X, pack=qb.qblora_decode_pack(qw))
    torch.cuda.synchronize()
    ow = OracleWeight(oracle, L.W, codebook, False, base == "grouped").assert_same(qw)
    ref = oracle.forward(ow.dequantize(oracle, 0), L.X, None, None, 1, 1, 0.0)
    assert_close_bf16(Y, ref, "Y vs exact Eq. 1")
    assert_close_bf16(Yp, ref, "Y (packed) vs exact Eq. 1")


def test_decode_of_the_merged_int4_model(qb, oracle, codebook):
    """Sec. 3.3 deployment path: train-time layer with aligned tiles -> beta-shift merge -> 4-bit inference."""
    from gpu_util import f32_to_dev, to_np, bf16_to_dev, assert_close_bf16, OracleWeight
    T, d_out, d_in, lam1, lam2, s = 4, 512, 1024, 64, 8, 0.75
    L = synth.make_layer(2100, T, d_out, d_in, 8, lam1, lam2)
    Hb = synth.f32_to_bf16_bits((np.random.default_rng(2101).standard_normal((d_in // lam1, d_out // lam2)) * 0.05)
                                .astype(np.float32))
    qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 64, qb.QUANT_MINMAX_INT4)
    H = bf16_to_dev(Hb)
    merged = qb.qablora_merge_quantize(qw, H.float(), lam1, lam2, s, qb.MERGE_BETA_SHIFT)
    X = bf16_to_dev(L.X)
    Y = qb.qblora_linear_decode(merged, X, pack=qb.qblora_decode_pack(merged))
    torch.cuda.synchronize()
    # the merged model itself: beta' from the oracle's merge, the bf16 compute weight, a plain forward
    from helpers import bf16_exact
    from gpu_util import bf16_to_f64
    cb = synth.codebook_int4()
    ow = OracleWeight(oracle, L.W, None, minmax=True).assert_same(qw)
    beta2 = oracle.merge_beta_shift(ow.beta, bf16_exact(Hb).astype(np.float32), d_out, d_in, 64, lam1, lam2, s)
    assert np.array_equal(to_np(merged.beta).view(np.uint32), beta2.view(np.uint32))
    assert np.array_equal(to_np(merged.codes), ow.codes)
    Wm = oracle.dequantize(ow.codes, ow.scales, beta2, cb, 64, 3)
    assert_close_bf16(Y, oracle.forward(Wm, L.X, None, None, 1, 1, 0.0), "Y (merged INT4, decode)")
    # ... and the train-time layer it replaces (whose base weight is rounded to bf16)
    Wt = ow.dequantize(oracle, 2)
    ref = oracle.qa_forward(Wt, L.X, Hb, lam1, lam2, s)
    err = bf16_to_f64(Y) - ref
    rms = np.sqrt(np.mean(ref ** 2))
    assert np.sqrt(np.mean(err ** 2)) <= 5e-3 * rms and np.abs(err).max() <= 4e-2 * rms


MID_CASES = [
    # T, d_out, d_in: token tiles of 32 / 64 / 128, two chunks above 128, ragged rows, one to many steps
    (17, 512, 512), (32, 320, 192), (33, 1000, 1088), (64, 256, 2048), (100, 40, 64), (128, 1024, 1024),
    (129, 384, 320), (200, 648, 704), (256, 512, 4096),
]


@pytest.mark.parametrize("base", ["codebook", "minmax", "grouped"])
@pytest.mark.parametrize("T,d_out,d_in", MID_CASES)
def test_mid_batch_parity(qb, oracle, codebook, T, d_out, d_in, base):
    """16 < T <= 256: the entry point contracts the bf16 compute weight (Eq. 1 rounded once, as the training
    forward does) on token tiles of 32 / 64 / 128; from the row-major arrays and from the pack (INT4 models: codes
    regrouped, converted without the table)."""
    from gpu_util import f32_to_dev, bf16_to_dev, assert_close_bf16, OracleWeight
    print(f"case mid batch T={T} {d_out}x{d_in} base={base}", flush=True)
    L = synth.make_layer(2400 + T, T, d_out, d_in, 8, 1, 1)
    if base == "minmax":
        qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 64, qb.QUANT_MINMAX_INT4)
    else:
        qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook,
                                          qb.SCALES_E4M3_GROUPED if base == "grouped" else qb.SCALES_FP32)
    X = bf16_to_dev(L.X)
    Y = qb.qblora_linear_decode(qw, X)
    Yp = qb.qblora_linear_decode(qw, X, pack=qb.qblora_decode_pack(qw))
    torch.cuda.synchronize()
    ow = OracleWeight(oracle, L.W, codebook, base == "minmax", base == "grouped").assert_same(qw)
    ref = oracle.forward(ow.dequantize(oracle, 2), L.X, None, None, 1, 1, 0.0)
    assert_close_bf16(Y, ref, "Y")
    assert_close_bf16(Yp, ref, "Y (packed)")
    # same weights, same order of the sums: the layout of the codes changes nothing
    assert torch.equal(Y.view(torch.int16), Yp.view(torch.int16))
    # a second call gives the same bits (fixed order of the split sums)
    Y2 = qb.qblora_linear_decode(qw, X)
    torch.cuda.synchronize()
    assert torch.equal(Y.view(torch.int16), Y2.view(torch.int16))


def test_mid_batch_matches_the_training_forward(qb, oracle, codebook):
    """Without adapter qblora_linear_fwd and the mid-batch call contract the same bf16 weight: they agree to
    fp32 summation order."""
    from gpu_util import f32_to_dev, bf16_to_dev, bf16_to_f64
    T, d_out, d_in = 96, 768, 1536
    L = synth.make_layer(2500, T, d_out, d_in, 8, 1, 1)
    qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook)
    X = bf16_to_dev(L.X)
    Ym = qb.qblora_linear_decode(qw, X)
    Yf = qb.qblora_linear_fwd(qw, None, X)
    torch.cuda.synchronize()
    a, b = bf16_to_f64(Ym), bf16_to_f64(Yf)
    rms = np.sqrt(np.mean(b ** 2))
    assert np.all(np.abs(a - b) <= 2.0 ** -7 * np.abs(b) + 1e-5 * rms)          # one bf16 step at most


def test_decode_errors(qb, oracle, codebook):
    from gpu_util import f32_to_dev
    W = synth.base_weight(2200, 0, 128, 128)
    qw = qb.qblora_quantize_blockwise(f32_to_dev(W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook)
    X = torch.zeros((257, 128), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(RuntimeError):
        qb.qblora_linear_decode(qw, X)                                   # more than 256 tokens
    assert qb.qblora_linear_decode(qw, X[:0]).shape == (0, 128)
