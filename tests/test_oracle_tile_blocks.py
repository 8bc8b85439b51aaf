"""Pins for the oracle's two-dimensional quantization blocks (the 4 x 8 and 8 x 8 shapes of Sec. 3.3) and the
exact offset-shift merge they allow at lambda1 = lambda2 = 8 (Alg. 2 get_new_beta; ablation "The balancing
factor of QA-BLoRA").  A block of lambda1 inputs x lambda2 outputs is br = lambda2 rows x bc = lambda1 columns
of the stored [d_out, d_in] weight: block size 32 with (lambda1, lambda2) = (4, 8) is br = 8, bc = 4."""
import numpy as np
import pytest

from paper_2407_17029_amd import synth
from helpers import unpack_codes, bf16_exact


def _blocks(W, br, bc):
    """[d_out, d_in] -> [d_out/br, d_in/bc, br*bc], elements of a block row by row (numpy reshapes only)."""
    d_out, d_in = W.shape
    return W.reshape(d_out // br, br, d_in // bc, bc).transpose(0, 2, 1, 3).reshape(d_out // br, d_in // bc, br * bc)


def test_one_row_blocks_are_the_row_segment_functions(oracle, codebook):
    W = synth.make_layer(71, 2, 24, 256, 4, 1, 1).W
    c0, a0 = oracle.quantize_codebook(W, 64, codebook)
    c1, a1 = oracle.quantize_codebook_tile(W, 1, 64, codebook)
    assert np.array_equal(c0, c1) and np.array_equal(a0.view(np.uint32), a1.view(np.uint32))
    m0 = oracle.quantize_minmax(W, 64); m1 = oracle.quantize_minmax_tile(W, 1, 64)
    for x, y in zip(m0, m1):
        assert np.array_equal(x.view(np.uint8), y.view(np.uint8))
    for mode in (0, 1, 2, 3):
        assert np.array_equal(oracle.dequantize(m0[0], m0[1], m0[2], synth.codebook_int4(), 64, mode),
                              oracle.dequantize_tile(m0[0], m0[1], m0[2], synth.codebook_int4(), 1, 64, mode))


@pytest.mark.parametrize("br,bc", [(8, 8), (4, 8), (8, 4)])
def test_tile_quantizers_against_numpy_on_gathered_blocks(oracle, codebook, br, bc):
    """Scales are the per-block reductions; codes are the brute-force nearest entry (codebook) and the Eq. 1
    rounding (min-max) evaluated on the gathered block with its own scale."""
    rng = np.random.default_rng(72)
    d_out, d_in = 32, 48
    W = (rng.standard_normal((d_out, d_in)) * 0.05).astype(np.float32)
    codes, absmax = oracle.quantize_codebook_tile(W, br, bc, codebook)
    Wb = _blocks(W, br, bc)
    assert np.array_equal(absmax, np.abs(Wb).max(-1))
    cb = np.asarray(codebook, np.float64)
    cbk = _blocks(unpack_codes(codes), br, bc)
    # nearest codebook entry of w / absmax (away from ties, which have measure zero for random data)
    want = np.abs(Wb.astype(np.float64)[..., None] / absmax[..., None, None] - cb).argmin(-1)
    assert (cbk == want).mean() > 0.999 and np.abs(cbk.astype(int) - want).max() <= 1
    codes, alpha, beta = oracle.quantize_minmax_tile(W, br, bc)
    lo, hi = Wb.min(-1), Wb.max(-1)
    assert np.array_equal(beta, lo)
    assert np.allclose(alpha, (hi.astype(np.float64) - lo) / 15, rtol=1e-6)
    q = _blocks(unpack_codes(codes), br, bc)
    ideal = (Wb.astype(np.float64) - lo[..., None]) * (15.0 / (hi.astype(np.float64) - lo)[..., None])
    assert np.abs(q - ideal).max() <= 0.5 + 1e-4          # Eq. 1: round to the nearest level
    # reconstruction error bound alpha/2 per element
    Wd = oracle.dequantize_tile(codes, alpha, beta, synth.codebook_int4(), br, bc, 0)
    assert np.all(np.abs(_blocks(Wd, br, bc) - Wb) <= alpha[..., None] * 0.5 * (1 + 1e-5) + 1e-9)


def test_tile_dequantize_closed_form(oracle):
    br, bc, d_out, d_in = 8, 8, 16, 32
    rng = np.random.default_rng(73)
    codes = rng.integers(0, 256, (d_out, d_in // 2), dtype=np.uint8)
    alpha = rng.uniform(0.01, 0.1, (d_out // br, d_in // bc)).astype(np.float32)
    beta = rng.uniform(-0.5, 0.5, (d_out // br, d_in // bc)).astype(np.float32)
    Wd = oracle.dequantize_tile(codes, alpha, beta, synth.codebook_int4(), br, bc, 0)
    a_full = np.repeat(np.repeat(alpha.astype(np.float64), br, 0), bc, 1)
    b_full = np.repeat(np.repeat(beta.astype(np.float64), br, 0), bc, 1)
    assert np.array_equal(Wd, a_full * unpack_codes(codes) + b_full)
    W1 = oracle.dequantize_tile(codes, alpha, beta, synth.codebook_int4(), br, bc, 1)
    assert np.array_equal(W1, (np.float32(1) * unpack_codes(codes).astype(np.float32) * np.repeat(np.repeat(alpha, br, 0), bc, 1)
                               + np.repeat(np.repeat(beta, br, 0), bc, 1)).astype(np.float64)) or \
        np.abs(W1 - Wd).max() <= 1e-7                      # fused multiply-add: within one fp32 rounding


@pytest.mark.parametrize("lam1,lam2,br,bc", [(8, 8, 8, 8), (8, 8, 4, 8), (16, 8, 8, 8), (4, 8, 8, 4)])
def test_offset_shift_merge_is_exact_on_aligned_tiles(oracle, lam1, lam2, br, bc):
    """get_new_beta: every block sits in one adapter tile, so the merged INT4 weight is w~ + s*dW exactly (up
    to the fp32 rounding of beta + delta), with the codes and alpha untouched."""
    d_out, d_in, s = 32, 64, 0.75
    L = synth.make_layer(74, 5, d_out, d_in, 8, lam1, lam2, b_std=0.05)
    codes, alpha, beta = oracle.quantize_minmax_tile(L.W, br, bc)
    cb = synth.codebook_int4()
    Hb = synth.f32_to_bf16_bits((np.random.default_rng(74).standard_normal((d_in // lam1, d_out // lam2)) * 0.05)
                                .astype(np.float32))
    H = bf16_exact(Hb).astype(np.float32)
    beta2 = oracle.merge_beta_shift_tile(beta, H, d_out, d_in, br, bc, lam1, lam2, s)
    delta = (s * np.repeat(np.repeat(H.astype(np.float64), lam1, 0), lam2, 1).T) / lam1        # [d_out, d_in]
    Wt = oracle.dequantize_tile(codes, alpha, beta, cb, br, bc, 0)
    Wm = oracle.dequantize_tile(codes, alpha, beta2, cb, br, bc, 0)
    assert np.abs(Wm - (Wt + delta)).max() <= 2.0 ** -23 * np.abs(Wt + delta).max()
    # the single-matrix adapted layer (Alg. 2 qablora_forward) is the merged INT4 layer
    Y_adapted = oracle.qa_forward(Wt, L.X, Hb, lam1, lam2, s)
    Y_merged = oracle.forward(Wm, L.X, None, None, 1, 1, 0.0)
    assert np.allclose(Y_merged, Y_adapted, rtol=0, atol=1e-5 * np.abs(Y_adapted).max())


def test_offset_shift_merge_rejects_straddling_blocks_and_handles_missing_beta(oracle):
    d_out, d_in = 16, 32
    H = np.ones((d_in // 4, d_out // 8), np.float32)
    with pytest.raises(ValueError):
        oracle.merge_beta_shift_tile(None, H, d_out, d_in, 8, 8, 4, 8, 1.0)      # lambda1 = 4 splits an 8-wide block
    H = np.full((d_in // 8, d_out // 8), 0.5, np.float32)
    out = oracle.merge_beta_shift_tile(None, H, d_out, d_in, 8, 8, 8, 8, 2.0)
    assert np.array_equal(out, np.full((2, 4), 0.125, np.float32))              # (2 * 0.5) / 8


def test_tile_merges_with_one_row_blocks_are_the_row_segment_merges(oracle, codebook):
    """br = 1, bc = 64 is the block of Sec. 3.1: both merges must reproduce the row-segment functions bit for bit."""
    d_out, d_in, lam1, lam2, s = 16, 128, 2, 4, 0.5
    L = synth.make_layer(81, 2, d_out, d_in, 8, lam1, lam2)
    H = (np.random.default_rng(81).standard_normal((d_in // lam1, d_out // lam2)) * 0.05).astype(np.float32)
    for minmax in (False, True):
        if minmax:
            codes, alpha, beta = oracle.quantize_minmax(L.W, 64); cb = synth.codebook_int4()
        else:
            (codes, alpha), beta, cb = oracle.quantize_codebook(L.W, 64, codebook), None, codebook
        a = oracle.merge_requant(codes, alpha, beta, cb, H, 64, lam1, lam2, s)
        b = oracle.merge_requant_tile(codes, alpha, beta, cb, H, 1, 64, lam1, lam2, s)
        for x, y in zip(a, b):
            assert np.array_equal(x.view(np.uint8), y.view(np.uint8))
        assert np.array_equal(oracle.merge_bf16(codes, alpha, beta, cb, H, 64, lam1, lam2, s),
                              oracle.merge_bf16_tile(codes, alpha, beta, cb, H, 1, 64, lam1, lam2, s))


@pytest.mark.parametrize("br,bc", [(8, 8), (4, 8)])
@pytest.mark.parametrize("lam1,lam2", [(2, 2), (4, 2), (8, 8), (3, 5)])
def test_tile_merges_against_numpy_on_gathered_blocks(oracle, br, bc, lam1, lam2):
    """The merged weight written out: w' = fl(fl(fma(c, alpha, beta)) + fl(fl(s h) / lambda1)) per element, then per
    block alpha' = (max - min) / 15, beta' = min, codes rint((w' - min) * (15 / (max - min))); the 16-bit merge
    rounds w' once.  Built with numpy float32 operations on blocks gathered by reshapes."""
    d_out, d_in, s = 120, 120, np.float32(0.75)          # divisible by 8, 4 and the lambdas 2, 3, 4, 5, 8
    L = synth.make_layer(82 + lam1, 2, d_out, d_in, 8, 1, 1)
    codes, alpha, beta = oracle.quantize_minmax_tile(L.W, br, bc)
    cb = synth.codebook_int4()
    H = (np.random.default_rng(83).standard_normal((d_in // lam1, d_out // lam2)) * 0.05).astype(np.float32)
    c = unpack_codes(codes).astype(np.float32)                                   # [d_out, d_in] code values 0..15
    A = np.repeat(np.repeat(alpha, br, 0), bc, 1); Bt = np.repeat(np.repeat(beta, br, 0), bc, 1)
    wt = (c.astype(np.float64) * A.astype(np.float64) + Bt.astype(np.float64)).astype(np.float32)   # one rounding = fma
    delta = ((s * np.repeat(np.repeat(H, lam1, 0), lam2, 1).T).astype(np.float32) / np.float32(lam1)).astype(np.float32)
    w = (wt + delta).astype(np.float32)
    # 16-bit merge
    W16 = oracle.merge_bf16_tile(codes, alpha, beta, cb, H, br, bc, lam1, lam2, float(s))
    assert np.array_equal(W16, synth.f32_to_bf16_bits(w))
    # requantizing merge
    co, ao, bo = oracle.merge_requant_tile(codes, alpha, beta, cb, H, br, bc, lam1, lam2, float(s))
    wb = _blocks(w, br, bc)
    lo, hi = wb.min(-1), wb.max(-1)
    rng_ = (hi - lo).astype(np.float32)
    assert np.array_equal(bo, lo) and np.array_equal(ao, (rng_ / np.float32(15)).astype(np.float32))
    inv = (np.float32(15) / rng_).astype(np.float32)
    q = np.rint(((wb - lo[..., None]).astype(np.float32) * inv[..., None]).astype(np.float32)).astype(np.uint8)
    assert np.array_equal(_blocks(unpack_codes(co), br, bc), q)
    # and the merged INT4 model is the shifted weight to within half a quantization step
    Wm = oracle.dequantize_tile(co, ao, bo, cb, br, bc, 0)
    step = np.repeat(np.repeat(ao, br, 0), bc, 1).astype(np.float64)
    assert np.all(np.abs(Wm - w.astype(np.float64)) <= 0.5 * step * (1 + 1e-5) + 1e-9)


def test_tile_16bit_merge_without_shift_is_the_compute_weight(oracle, codebook):
    """H = 0: the 16-bit merge is the bf16 compute weight of the forward pass (dequantize mode 2)."""
    d_out, d_in = 24, 64
    W = synth.make_layer(84, 2, d_out, d_in, 8, 1, 1).W
    codes, absmax = oracle.quantize_codebook_tile(W, 8, 8, codebook)
    H = np.zeros((d_in // 2, d_out // 2), np.float32)
    W16 = oracle.merge_bf16_tile(codes, absmax, None, codebook, H, 8, 8, 2, 2, 1.0)
    ref = oracle.dequantize_tile(codes, absmax, None, codebook, 8, 8, 2)
    assert np.array_equal(bf16_exact(W16), ref)
