"""GPU parity (bit-exact): block-wise quantizers, scale double quantization, standalone dequantize."""
import numpy as np
import pytest
import torch

from paper_2407_17029_amd import synth

pytestmark = pytest.mark.gpu

SHAPES = [(512, 512), (192, 320), (64, 64), (1000, 1088)]


@pytest.fixture(scope="module")
def qb():
    from paper_2407_17029_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("d_out,d_in", SHAPES)
def test_codebook_quantize_bit_exact(qb, oracle, codebook, d_out, d_in):
    from gpu_util import f32_to_dev, to_np
    print(f"case codebook quantize {d_out}x{d_in}", flush=True)
    W = synth.base_weight(100 + d_out, 0, d_out, d_in)
    W[3, :64] = 0.0                                         # a degenerate all-zero block
    qw = qb.qblora_quantize_blockwise(f32_to_dev(W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook)
    torch.cuda.synchronize()
    codes, absmax = oracle.quantize_codebook(W, 64, codebook)
    assert qw.beta is None
    assert np.array_equal(to_np(qw.scales).view(np.uint32), absmax.view(np.uint32))
    assert np.array_equal(to_np(qw.codes), codes)


@pytest.mark.parametrize("d_out,d_in", SHAPES)
def test_minmax_quantize_bit_exact(qb, oracle, d_out, d_in):
    from gpu_util import f32_to_dev, to_np
    print(f"case minmax quantize {d_out}x{d_in}", flush=True)
    W = synth.base_weight(200 + d_out, 0, d_out, d_in)
    W[5, 64:128] = 0.25                                     # a constant block (alpha = 0)
    qw = qb.qblora_quantize_blockwise(f32_to_dev(W), 64, qb.QUANT_MINMAX_INT4)
    torch.cuda.synchronize()
    codes, alpha, beta = oracle.quantize_minmax(W, 64)
    assert np.array_equal(to_np(qw.scales).view(np.uint32), alpha.view(np.uint32))
    assert np.array_equal(to_np(qw.beta).view(np.uint32), beta.view(np.uint32))
    assert np.array_equal(to_np(qw.codes), codes)
    assert np.array_equal(qw.codebook, np.arange(16, dtype=np.float32))


@pytest.mark.parametrize("d_out,d_in", [(512, 512), (100, 192), (256, 1024)])
def test_double_quantized_scales_bit_exact(qb, oracle, codebook, d_out, d_in):
    from gpu_util import f32_to_dev, to_np
    print(f"case double quant {d_out}x{d_in}", flush=True)
    W = synth.base_weight(300 + d_out, 0, d_out, d_in)
    rows_const = 256 // (d_in // 64)                        # the first 256 blocks get equal scales: a group with step 0
    W[:rows_const, :] = 0.5
    qw = qb.qblora_quantize_blockwise(f32_to_dev(W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook,
                                      qb.SCALES_E4M3_GROUPED)
    torch.cuda.synchronize()
    codes, absmax = oracle.quantize_codebook(W, 64, codebook)
    sc, step, mid = oracle.scales_double_quantize(absmax.reshape(-1), 256)
    assert np.array_equal(to_np(qw.codes), codes)
    assert np.array_equal(to_np(qw.scale_codes), sc)
    assert np.array_equal(to_np(qw.scale_step).view(np.uint32), step.view(np.uint32))
    assert np.array_equal(to_np(qw.scale_mid).view(np.uint32), mid.view(np.uint32))


def test_dequantize_bf16_bit_exact(qb, oracle, codebook):
    from gpu_util import f32_to_dev, bf16_to_f64, OracleWeight
    W = synth.base_weight(400, 0, 192, 320)
    qw = qb.qblora_quantize_blockwise(f32_to_dev(W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook)
    Wt = qb.qblora_dequantize_bf16(qw)
    torch.cuda.synchronize()
    want = OracleWeight(oracle, W, codebook).assert_same(qw).dequantize(oracle, 2)
    assert np.array_equal(bf16_to_f64(Wt), want)
    qm = qb.qblora_quantize_blockwise(f32_to_dev(W), 64, qb.QUANT_MINMAX_INT4)
    Wm = qb.qblora_dequantize_bf16(qm)
    torch.cuda.synchronize()
    want = OracleWeight(oracle, W, None, minmax=True).assert_same(qm).dequantize(oracle, 2)
    assert np.array_equal(bf16_to_f64(Wm), want)


@pytest.mark.parametrize("d_out,d_in", [(512, 512), (320, 192), (256, 1088)])
def test_tiled_code_copy(qb, oracle, codebook, d_out, d_in):
    """The tile-ordered copy holds the same code bytes as the reference layout, from either producer."""
    from gpu_util import f32_to_dev, to_np
    W = synth.base_weight(900 + d_in, 0, d_out, d_in)
    qw = qb.qblora_quantize_blockwise(f32_to_dev(W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook)
    assert qw.codes_tiled is not None and qw.codes_tiled.numel() == qb.qblora_codes_tiled_bytes(d_out, d_in)
    from_quantizer = to_np(qw.codes_tiled).copy()
    qw.codes_tiled = None
    qb.qblora_prepack_codes(qw)
    torch.cuda.synchronize()
    from_prepack = to_np(qw.codes_tiled)
    codes = to_np(qw.codes)                                   # [d_out, d_in/2]
    bpr = d_in // 64
    tiles = (d_out + 255) // 256
    want = np.zeros((tiles, bpr, 256, 32), np.uint8)          # rows past d_out stay zero
    for n in range(d_out):
        want[n // 256, :, n % 256, :] = codes[n].reshape(bpr, 32)
    got_p = from_prepack.reshape(tiles, bpr, 256, 32)
    got_q = from_quantizer.reshape(tiles, bpr, 256, 32)
    assert np.array_equal(got_p, want)
    valid = np.zeros((tiles, 1, 256, 1), bool)
    for n in range(d_out):
        valid[n // 256, 0, n % 256, 0] = True
    assert np.array_equal(np.where(valid, got_q, 0), want)
