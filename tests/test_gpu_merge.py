"""GPU parity (bit-exact given H): tile product and the QA-BLoRA merge in both forms."""
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


def _bits(a):
    return a.view(np.uint32)


@pytest.mark.parametrize("d_out,d_in,R,lam1,lam2", [(512, 512, 32, 2, 2), (320, 192, 16, 4, 8), (256, 1024, 64, 1, 1),
                                                    (1024, 512, 256, 2, 2), (512, 256, 144, 4, 2), (768, 384, 128, 2, 3)])
def test_tile_product(qb, oracle, d_out, d_in, R, lam1, lam2):
    from gpu_util import adapter_to_dev, assert_close_f32
    L = synth.make_layer(800, 1, d_out, d_in, R, lam1, lam2)
    ad = adapter_to_dev(L, lam1, lam2, 1.0)
    H = qb.qblora_tile_product(ad, d_in, d_out)
    torch.cuda.synchronize()
    assert_close_f32(H, oracle.tile_product(L.A, L.B), "H")


@pytest.mark.parametrize("grouped", [False, True])
@pytest.mark.parametrize("d_out,d_in,lam1,lam2,s", [(512, 512, 2, 2, 1.0), (192, 320, 4, 8, 0.25),
                                                     (128, 1088, 8, 8, 1.0), (100, 192, 1, 1, 1.5),
                                                     (64, 768, 64, 2, 1.0), (96, 192, 3, 2, 1.0)])
def test_merge_requant_bit_exact(qb, oracle, codebook, d_out, d_in, lam1, lam2, s, grouped):
    from gpu_util import f32_to_dev, to_np, OracleWeight
    print(f"case requant {d_out}x{d_in} lam=({lam1},{lam2}) grouped={grouped}", flush=True)
    if d_in % lam1 or d_out % lam2:
        pytest.skip("shape not divisible")
    W = synth.base_weight(810 + d_in, 0, d_out, d_in)
    H = synth.normal_f32(811, 1, (d_in // lam1, d_out // lam2), 0.01)
    qw = qb.qblora_quantize_blockwise(f32_to_dev(W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook,
                                      qb.SCALES_E4M3_GROUPED if grouped else qb.SCALES_FP32)
    out = qb.qablora_merge_quantize(qw, f32_to_dev(H), lam1, lam2, s, qb.MERGE_REQUANT_MINMAX)
    torch.cuda.synchronize()
    ow = OracleWeight(oracle, W, codebook, grouped=grouped).assert_same(qw)
    co, ao, bo = oracle.merge_requant(ow.codes, ow.scales, None, codebook, H, 64, lam1, lam2, s)
    assert np.array_equal(_bits(to_np(out.scales)), _bits(ao))
    assert np.array_equal(_bits(to_np(out.beta)), _bits(bo))
    assert np.array_equal(to_np(out.codes), co)
    assert np.array_equal(out.codebook, np.arange(16, dtype=np.float32))


def test_merge_requant_of_minmax_base(qb, oracle):
    from gpu_util import f32_to_dev, to_np, OracleWeight
    W = synth.base_weight(820, 0, 128, 256)
    H = synth.normal_f32(821, 1, (128, 64), 0.01)
    qw = qb.qblora_quantize_blockwise(f32_to_dev(W), 64, qb.QUANT_MINMAX_INT4)
    out = qb.qablora_merge_quantize(qw, f32_to_dev(H), 2, 2, 1.0, qb.MERGE_REQUANT_MINMAX)
    torch.cuda.synchronize()
    ow = OracleWeight(oracle, W, None, minmax=True).assert_same(qw)
    co, ao, bo = oracle.merge_requant(ow.codes, ow.scales, ow.beta, synth.codebook_int4(), H, 64, 2, 2, 1.0)
    assert np.array_equal(to_np(out.codes), co)
    assert np.array_equal(_bits(to_np(out.scales)), _bits(ao)) and np.array_equal(_bits(to_np(out.beta)), _bits(bo))


@pytest.mark.parametrize("minmax", [False, True])
@pytest.mark.parametrize("lam1,lam2", [(64, 1), (64, 8), (128, 2)])
def test_merge_beta_shift_bit_exact(qb, oracle, codebook, lam1, lam2, minmax):
    from gpu_util import f32_to_dev, to_np, OracleWeight
    d_out, d_in, s = 192, 512, 0.75
    W = synth.base_weight(830, 0, d_out, d_in)
    H = synth.normal_f32(831, 1, (d_in // lam1, d_out // lam2), 0.01)
    if minmax:
        qw = qb.qblora_quantize_blockwise(f32_to_dev(W), 64, qb.QUANT_MINMAX_INT4)
    else:
        qw = qb.qblora_quantize_blockwise(f32_to_dev(W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook)
    out = qb.qablora_merge_quantize(qw, f32_to_dev(H), lam1, lam2, s, qb.MERGE_BETA_SHIFT)
    torch.cuda.synchronize()
    ow = OracleWeight(oracle, W, codebook, minmax=minmax).assert_same(qw)
    want = oracle.merge_beta_shift(ow.beta, H, d_out, d_in, 64, lam1, lam2, s)
    assert np.array_equal(_bits(to_np(out.beta)), _bits(want))
    assert torch.equal(out.codes, qw.codes) and torch.equal(out.scales, qw.scales)     # codes, alpha untouched
    assert np.array_equal(out.codebook, qw.codebook)


def test_merge_beta_shift_rejects_misaligned(qb, codebook):
    from gpu_util import f32_to_dev
    W = synth.base_weight(840, 0, 64, 128)
    qw = qb.qblora_quantize_blockwise(f32_to_dev(W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook)
    H = f32_to_dev(np.zeros((64, 32), np.float32))
    with pytest.raises(qb.QBLoRAError) as e:
        qb.qablora_merge_quantize(qw, H, 2, 2, 1.0, qb.MERGE_BETA_SHIFT)
    assert e.value.code == -5


@pytest.mark.parametrize("base", ["codebook", "grouped", "minmax"])
@pytest.mark.parametrize("d_out,d_in,lam1,lam2,s", [(512, 512, 2, 2, 1.0), (192, 320, 4, 8, 0.25),
                                                     (128, 1088, 8, 8, 1.0), (100, 192, 1, 1, 1.5),
                                                     (64, 768, 64, 2, 1.0), (96, 192, 3, 2, 1.0)])
def test_merge_bf16_bit_exact(qb, oracle, codebook, d_out, d_in, lam1, lam2, s, base):
    """16-bit merge: the bf16 weight w~ + s*dW, bit for bit."""
    from gpu_util import f32_to_dev, OracleWeight
    print(f"case merge16 {d_out}x{d_in} lam=({lam1},{lam2}) base={base}", flush=True)
    W = synth.base_weight(830 + d_in, 0, d_out, d_in)
    H = synth.normal_f32(831, 1, (d_in // lam1, d_out // lam2), 0.01)
    if base == "minmax":
        qw = qb.qblora_quantize_blockwise(f32_to_dev(W), 64, qb.QUANT_MINMAX_INT4)
        cb = synth.codebook_int4()
    else:
        qw = qb.qblora_quantize_blockwise(f32_to_dev(W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook,
                                          qb.SCALES_E4M3_GROUPED if base == "grouped" else qb.SCALES_FP32)
        cb = codebook
    W16 = qb.qblora_merge_bf16(qw, f32_to_dev(H), lam1, lam2, s)
    torch.cuda.synchronize()
    ow = OracleWeight(oracle, W, codebook, base == "minmax", base == "grouped").assert_same(qw)
    ref = oracle.merge_bf16(ow.codes, ow.scales, ow.beta, cb, H, 64, lam1, lam2, s)
    assert np.array_equal(W16.view(torch.int16).cpu().numpy().view(np.uint16), ref)


def test_merged_bf16_layer_reproduces_the_adapted_layer(qb, oracle, codebook):
    """X * W16^T (a plain bf16 matmul) against the adapted forward of this library and the oracle."""
    from gpu_util import f32_to_dev, bf16_to_dev, adapter_to_dev, to_np, assert_close_bf16, assert_close_f32, OracleWeight
    T, d_out, d_in, R, lam, s = 256, 512, 768, 32, 2, 1.0
    L = synth.make_layer(840, T, d_out, d_in, R, lam, lam)
    qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook)
    ad = adapter_to_dev(L, lam, lam, s)
    X = bf16_to_dev(L.X)
    H = qb.qblora_tile_product(ad, d_in, d_out)
    W16 = qb.qblora_merge_bf16(qw, H, lam, lam, s)
    Y16 = torch.matmul(X.float(), W16.float().t()).to(torch.bfloat16)
    torch.cuda.synchronize()
    # the merged dense layer itself, from the oracle's own tile matrix and merged weight (the device's tile
    # matrix differs from the oracle's in the last fp32 bits, which moves an occasional bf16 rounding)
    ow = OracleWeight(oracle, L.W, codebook).assert_same(qw)
    H32 = oracle.tile_product(L.A, L.B).astype(np.float32)
    assert_close_f32(H, H32.astype(np.float64), "H")
    W16_ref = oracle.merge_bf16(ow.codes, ow.scales, None, codebook, H32, 64, lam, lam, s)
    from helpers import bf16_exact
    assert_close_bf16(Y16, oracle.forward(bf16_exact(W16_ref), L.X, None, None, 1, 1, 0.0), "Y (16-bit merged)")
    # ... and the adapted layer it replaces: every merged weight carries one more bf16 rounding (2^-9
    # relative), which shows as ~3e-3 rms and a few 1e-2 at the worst of 131072 outputs
    from gpu_util import bf16_to_f64
    Wt = ow.dequantize(oracle, 2)
    ref = oracle.forward(Wt, L.X, L.A, L.B, lam, lam, s)
    err = bf16_to_f64(Y16) - ref
    rms = np.sqrt(np.mean(ref ** 2))
    assert np.sqrt(np.mean(err ** 2)) <= 5e-3 * rms and np.abs(err).max() <= 4e-2 * rms


@pytest.mark.parametrize("grouped", [False, True])
def test_batched_merge_equals_single_merges(qb, oracle, codebook, grouped):
    """The projections of a layer merged in one call: same bits as one call per weight (and so as the oracle);
    mixed shapes, more weights than one launch takes, and a mode that goes one by one."""
    from gpu_util import f32_to_dev, to_np
    shapes = [(128, 256), (192, 512), (64, 1024), (128, 256), (256, 192), (64, 64), (320, 256), (128, 128), (64, 320)]
    lam1, lam2, s = 2, 2, 0.75
    bases, Hs = [], []
    for i, (d_out, d_in) in enumerate(shapes):
        W = synth.base_weight(860 + i, 0, d_out, d_in)
        bases.append(qb.qblora_quantize_blockwise(f32_to_dev(W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook,
                                                  qb.SCALES_E4M3_GROUPED if grouped else qb.SCALES_FP32))
        Hs.append(f32_to_dev(synth.normal_f32(870 + i, 1, (d_in // lam1, d_out // lam2), 0.01)))
    outs = qb.qablora_merge_quantize_batch(bases, Hs, lam1, lam2, s, qb.MERGE_REQUANT_MINMAX)
    torch.cuda.synchronize()
    for b, H, o in zip(bases, Hs, outs):
        single = qb.qablora_merge_quantize(b, H, lam1, lam2, s, qb.MERGE_REQUANT_MINMAX)
        torch.cuda.synchronize()
        assert torch.equal(o.codes, single.codes)
        assert torch.equal(o.scales.view(torch.int32), single.scales.view(torch.int32))
        assert torch.equal(o.beta.view(torch.int32), single.beta.view(torch.int32))
        assert np.array_equal(o.codebook, np.arange(16, dtype=np.float32)) and o.scale_mode == qb.SCALES_FP32
    # against the oracle directly, for one of them
    from gpu_util import OracleWeight
    W3 = synth.base_weight(863, 0, *shapes[3])
    ow = OracleWeight(oracle, W3, codebook, grouped=grouped).assert_same(bases[3])
    co, ao, bo = oracle.merge_requant(ow.codes, ow.scales, None, codebook, to_np(Hs[3]), 64, lam1, lam2, s)
    assert np.array_equal(to_np(outs[3].codes), co) and np.array_equal(_bits(to_np(outs[3].scales)), _bits(ao))


def test_batched_merge_offset_shift_and_errors(qb, oracle, codebook):
    from gpu_util import f32_to_dev
    lam1, lam2, s = 64, 2, 0.5
    bases = [qb.qblora_quantize_blockwise(f32_to_dev(synth.base_weight(880 + i, 0, 128, 256)), 64, qb.QUANT_MINMAX_INT4)
             for i in range(3)]
    Hs = [f32_to_dev(synth.normal_f32(885 + i, 1, (256 // lam1, 128 // lam2), 0.01)) for i in range(3)]
    outs = qb.qablora_merge_quantize_batch(bases, Hs, lam1, lam2, s, qb.MERGE_BETA_SHIFT)
    torch.cuda.synchronize()
    for b, H, o in zip(bases, Hs, outs):
        single = qb.qablora_merge_quantize(b, H, lam1, lam2, s, qb.MERGE_BETA_SHIFT)
        torch.cuda.synchronize()
        assert torch.equal(o.codes, single.codes) and torch.equal(o.beta.view(torch.int32), single.beta.view(torch.int32))
    assert qb.qablora_merge_quantize_batch([], [], 2, 2, 1.0, qb.MERGE_REQUANT_MINMAX) == []
    with pytest.raises(qb.QBLoRAError):                      # one misaligned weight rejects the whole call
        qb.qablora_merge_quantize_batch(bases, Hs, 2, 2, s, qb.MERGE_BETA_SHIFT)
