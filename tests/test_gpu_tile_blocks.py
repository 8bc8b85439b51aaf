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
    # standalone dequantize (bf16 compute weight)
    for q, beta, cb in ((qw, None, codebook), (qm, bm, synth.codebook_int4())):
        Wt = qb.qblora_dequantize_bf16(q)
        torch.cuda.synchronize()
        want = oracle.dequantize_tile(to_np(q.codes), to_np(q.scales), beta, cb, 8, 8, 2)
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
        beta = None if base.beta is None else to_np(base.beta)
        want = oracle.merge_beta_shift_tile(beta, H, d_out, d_in, 8, 8, lam1, lam2, s)
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
    with pytest.raises(qb.QBLoRAError):                      # the requantizing merge is for row-segment blocks
        qb.qablora_merge_quantize(base, H, 4, 8, 1.0, qb.MERGE_REQUANT_MINMAX)
    with pytest.raises(qb.QBLoRAError):                      # d_out must be a multiple of 8
        qb.qblora_quantize_blockwise(W[:60].contiguous(), 64, qb.QUANT_MINMAX_INT4, block_rows=8)
    with pytest.raises(qb.QBLoRAError):
        qb.qblora_quantize_blockwise(W, 64, qb.QUANT_ABSMAX_CODEBOOK, codebook, qb.SCALES_E4M3_GROUPED, block_rows=8)
