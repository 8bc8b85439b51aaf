"""Pins for the oracle's quantizers and dequantizer (Eq. 1, Sec. 3.1).

Every expected value here comes from something other than the oracle: a
brute-force search, a closed form or error bound of Eq. 1, a hand-written
fixture under tests/golden/, or a library routine (numpy / torch dtype casts).
"""
import os

import numpy as np
import pytest
import torch

from paper_2407_17029_amd import synth
from helpers import unpack_codes

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _weights(seed, d_out=8, d_in=256):
    return synth.base_weight(seed, 0, d_out, d_in)


# ------------------------------------------------------------------ codebook quantizer
def test_codebook_shape_and_properties(codebook):
    assert codebook.dtype == np.float32 and codebook.shape == (16,)
    assert codebook[0] == -1.0 and codebook[15] == 1.0 and codebook[7] == 0.0
    assert np.all(np.diff(codebook) > 0)
    assert (codebook < 0).sum() == 7 and (codebook > 0).sum() == 8


def test_codebook_quantize_is_nearest_entry(oracle, codebook):
    W = _weights(11, 16, 512)
    codes, absmax = oracle.quantize_codebook(W, 64, codebook)
    blocks = W.reshape(16, 8, 64).astype(np.float64)
    a = np.abs(blocks).max(-1)
    assert np.array_equal(absmax, a.astype(np.float32))             # absmax scale is exact
    ratio = blocks / a[..., None]
    dist = np.abs(ratio[..., None] - codebook.astype(np.float64))   # brute force over 16 entries
    nearest = dist.argmin(-1)
    srt = np.sort(dist, -1)
    clear = (srt[..., 1] - srt[..., 0]) > 1e-5                      # skip inputs that sit on a threshold
    got = unpack_codes(codes).reshape(16, 8, 64)
    assert clear.mean() > 0.99
    assert np.array_equal(got[clear], nearest[clear])


def test_codebook_quantize_monotone_and_extremes(oracle, codebook):
    W = _weights(12, 4, 128)
    codes, absmax = oracle.quantize_codebook(W, 64, codebook)
    got = unpack_codes(codes).reshape(4, 2, 64)
    blocks = W.reshape(4, 2, 64)
    for n in range(4):
        for b in range(2):
            order = np.argsort(blocks[n, b], kind="stable")
            assert np.all(np.diff(got[n, b][order]) >= 0)            # w1 <= w2  =>  code1 <= code2
            i = np.abs(blocks[n, b]).argmax()
            assert got[n, b, i] == (15 if blocks[n, b, i] > 0 else 0)  # +-absmax hits the end entries


def test_codebook_fixed_point_bit_exact(oracle, codebook):
    """dequantize(quantize(c_j * a)) == c_j * a exactly when the block contains +-a."""
    rng = np.random.default_rng(5)
    d_out, d_in = 6, 128
    scale = rng.uniform(0.01, 3.0, size=(d_out, d_in // 64)).astype(np.float32)
    idx = rng.integers(0, 16, size=(d_out, d_in))
    idx[:, 0::64] = 15                                              # block holds +a
    idx[:, 1::64] = 0                                               # ... and -a
    W = (codebook[idx] * np.repeat(scale, 64, axis=1)).astype(np.float32)   # one fp32 multiply
    codes, absmax = oracle.quantize_codebook(W, 64, codebook)
    assert np.array_equal(absmax, scale)
    assert np.array_equal(unpack_codes(codes), idx)
    Wt = oracle.dequantize(codes, absmax, None, codebook, 64, mode=1)
    assert np.array_equal(Wt.astype(np.float32).view(np.uint32), W.view(np.uint32))


def test_codebook_tie_takes_lower_index_and_zero_block(oracle, codebook):
    # a = 1 (block holds +1): the threshold between entries 9 and 10 is exactly their fp32 midpoint
    mid = np.float32((codebook[9] + codebook[10]) * np.float32(0.5))
    W = np.zeros((2, 64), np.float32)
    W[0, 0] = 1.0
    W[0, 1] = mid
    W[0, 2] = np.nextafter(mid, np.float32(2.0))
    codes, absmax = oracle.quantize_codebook(W, 64, codebook)
    c = unpack_codes(codes)
    assert c[0, 0] == 15 and c[0, 1] == 9 and c[0, 2] == 10
    assert c[0, 3] == 7                                              # 0.0 maps to the zero entry
    # an all-zero block: scale 0, every comparison w > 0 fails -> code 0, value c_0 * 0 = -0.0
    assert absmax[1, 0] == 0.0 and np.all(c[1] == 0)
    assert np.all(oracle.dequantize(codes, absmax, None, codebook, 64, mode=1)[1] == 0.0)


def test_nibble_packing_layout(oracle, codebook):
    W = np.zeros((1, 64), np.float32)
    W[0, 0] = 1.0      # k=0 -> code 15 in the low nibble of byte 0
    W[0, 1] = -1.0     # k=1 -> code 0 in the high nibble of byte 0
    W[0, 3] = 1.0      # k=3 -> code 15 in the high nibble of byte 1
    codes, _ = oracle.quantize_codebook(W, 64, codebook)
    assert codes[0, 0] == 0x0F
    assert codes[0, 1] == 0xF7      # k=2 is 0.0 -> entry 7 (low nibble), k=3 -> 15 (high nibble)


# ------------------------------------------------------------------ min-max quantizer
def test_minmax_golden_ramp(oracle):
    """Hand-worked block: w_i = i mod 16 gives lo=0, hi=15, alpha=1, codes = i mod 16."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "minmax_ramp.txt")) if not l.startswith("#")]
    w = np.array([float(r[0]) for r in rows], np.float32).reshape(1, 64)
    want = np.array([int(r[1]) for r in rows])
    codes, alpha, beta = oracle.quantize_minmax(w, 64)
    assert alpha[0, 0] == 1.0 and beta[0, 0] == 0.0
    assert np.array_equal(unpack_codes(codes)[0], want)


@pytest.mark.parametrize("block", [32, 64])
def test_minmax_error_bound_and_endpoints(oracle, block):
    W = _weights(21, 16, 256)
    codes, alpha, beta = oracle.quantize_minmax(W, block)
    c = unpack_codes(codes).reshape(16, 256 // block, block)
    blocks = W.reshape(16, 256 // block, block)
    assert np.array_equal(beta, blocks.min(-1))                      # beta = w_min
    want_alpha = ((blocks.max(-1).astype(np.float64) - blocks.min(-1)) / 15.0)
    assert np.allclose(alpha, want_alpha, rtol=3e-7, atol=0)         # alpha = (max-min)/(2^4-1)
    assert np.all(c[np.arange(16)[:, None], np.arange(256 // block)[None], blocks.argmin(-1)] == 0)
    assert np.all(c[np.arange(16)[:, None], np.arange(256 // block)[None], blocks.argmax(-1)] == 15)
    deq = alpha[..., None].astype(np.float64) * c + beta[..., None]
    assert np.all(np.abs(deq - blocks) <= alpha[..., None] * 0.5 * (1 + 1e-5))   # |w~ - w| <= alpha/2
    assert c.min() >= 0 and c.max() <= 15


def test_minmax_rounds_half_to_even(oracle):
    # lo = 0, hi = 15 -> inv = 1, q = w; halves go to the even neighbour
    w = np.zeros((1, 64), np.float32)
    w[0, :6] = [0.0, 15.0, 0.5, 1.5, 2.5, 13.5]
    codes, alpha, beta = oracle.quantize_minmax(w, 64)
    assert list(unpack_codes(codes)[0, :6]) == [0, 15, 0, 2, 2, 14]


def test_minmax_constant_block(oracle):
    w = np.full((1, 64), np.float32(0.375))
    codes, alpha, beta = oracle.quantize_minmax(w, 64)
    assert alpha[0, 0] == 0.0 and beta[0, 0] == np.float32(0.375) and np.all(codes == 0)
    Wt = oracle.dequantize(codes, alpha, beta, synth.codebook_int4(), 64, mode=1)
    assert np.all(Wt == 0.375)


# ------------------------------------------------------------------ dequantize
def test_dequantize_modes(oracle, codebook):
    W = _weights(31, 8, 128)
    codes, absmax = oracle.quantize_codebook(W, 64, codebook)
    c = unpack_codes(codes)
    a = np.repeat(absmax, 64, axis=1)
    want_real = a.astype(np.float64) * codebook[c].astype(np.float64)            # Eq. 1 with beta = 0
    assert np.array_equal(oracle.dequantize(codes, absmax, None, codebook, 64, 0), want_real)
    want_f32 = codebook[c] * a                                                   # numpy fp32 multiply
    assert np.array_equal(oracle.dequantize(codes, absmax, None, codebook, 64, 1), want_f32.astype(np.float64))
    want_bf16 = torch.from_numpy(want_f32).to(torch.bfloat16).to(torch.float64).numpy()   # library RNE cast
    assert np.array_equal(oracle.dequantize(codes, absmax, None, codebook, 64, 2), want_bf16)


def test_dequantize_with_beta(oracle):
    W = _weights(32, 4, 128)
    codes, alpha, beta = oracle.quantize_minmax(W, 64)
    c = unpack_codes(codes).astype(np.float64)
    want = np.repeat(alpha, 64, 1).astype(np.float64) * c + np.repeat(beta, 64, 1)
    assert np.array_equal(oracle.dequantize(codes, alpha, beta, synth.codebook_int4(), 64, 0), want)
    got1 = oracle.dequantize(codes, alpha, beta, synth.codebook_int4(), 64, 1)
    assert np.array_equal(got1, want.astype(np.float32).astype(np.float64))      # fma = one rounding of the exact value


# ------------------------------------------------------------------ E4M3 / double quantization
def test_e4m3_decode_matches_format(oracle):
    codes = torch.arange(256, dtype=torch.uint8)
    want = codes.view(torch.float8_e4m3fn).to(torch.float32).numpy()             # library decode
    got = np.array([oracle.e4m3_decode(int(c)) for c in range(256)], np.float32)
    nan = np.isnan(want)
    assert nan.sum() == 2 and np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert got[0x7E] == 448.0 and got[0x01] == 2.0 ** -9 and got[0x08] == 2.0 ** -6


def test_e4m3_encode_round_trip_and_nearest(oracle):
    for c in range(256):
        if (c & 0x7F) == 0x7F:
            continue
        assert oracle.e4m3_encode(oracle.e4m3_decode(c)) == c
    rng = np.random.default_rng(3)
    xs = np.concatenate([rng.uniform(-448, 448, 3000), rng.normal(0, 1, 3000), rng.normal(0, 0.01, 2000)])
    xs = xs.astype(np.float32)
    want = torch.from_numpy(xs).to(torch.float8_e4m3fn).view(torch.uint8).numpy()  # library RNE cast
    got = np.array([oracle.e4m3_encode(float(x)) for x in xs], np.uint8)
    assert np.array_equal(got & 0x7F, want & 0x7F)
    nz = (got & 0x7F) != 0
    assert np.array_equal(got[nz], want[nz])
    # ties go to the even code; saturation at 448
    assert oracle.e4m3_encode(1.0625) == 0x38          # halfway between 1.0 (0x38) and 1.125 (0x39)
    assert oracle.e4m3_encode(1.1875) == 0x3A          # halfway between 1.125 (0x39) and 1.25 (0x3a)
    assert oracle.e4m3_encode(1e6) == 0x7E and oracle.e4m3_encode(-1e6) == 0xFE


def test_double_quant_scales(oracle, codebook):
    W = synth.base_weight(41, 0, 64, 1024)
    _, absmax = oracle.quantize_codebook(W, 64, codebook)
    s = absmax.reshape(-1)                                         # 1024 scales -> 4 groups of 256
    sc, step, mid = oracle.scales_double_quantize(s, 256)
    g = s.reshape(4, 256)
    assert np.array_equal(mid, ((g.min(1) + g.max(1)) * np.float32(0.5)).astype(np.float32))
    dmax = np.abs(g - mid[:, None]).max(1)
    assert np.allclose(step, dmax / 448.0, rtol=3e-7)
    rec = oracle.scales_double_dequantize(sc, step, mid, 256).reshape(4, 256)
    # E4M3 keeps 4 significant bits: relative half-ulp 2^-4 of |d|, absolute floor half the smallest subnormal
    d = (g - mid[:, None]).astype(np.float64)
    bound = np.maximum(np.abs(d) * 2.0 ** -4, step[:, None] * 2.0 ** -10) + np.abs(g) * 2.0 ** -22
    assert np.all(np.abs(rec - g) <= bound)
    # the group's extreme deviation is reproduced with code magnitude 448
    assert np.all(((sc.reshape(4, 256) & 0x7F) == 0x7E).any(1))


def test_double_quant_equal_scales_and_ragged_group(oracle):
    s = np.full(300, np.float32(0.7))
    sc, step, mid = oracle.scales_double_quantize(s, 256)
    assert sc.shape == (300,) and step.shape == (2,)
    assert np.all(sc == 0) and np.all(step == 0) and np.all(mid == np.float32(0.7))
    assert np.array_equal(oracle.scales_double_dequantize(sc, step, mid, 256), s)


def test_dequantize_inference_mode_is_scale_times_bf16_code_plus_offset(oracle, codebook):
    """Mode 3 (small-batch inference weight): alpha * bf16(c) + beta without further rounding; for the integer
    codebook of INT4 models it is the real-number formula of Eq. 1 itself."""
    from helpers import unpack_codes, bf16_exact
    W = synth.base_weight(77, 0, 8, 128)
    codes, alpha, beta = oracle.quantize_minmax(W, 64)
    cb = synth.codebook_int4()
    assert np.array_equal(oracle.dequantize(codes, alpha, beta, cb, 64, 3), oracle.dequantize(codes, alpha, beta, cb, 64, 0))
    codes, alpha = oracle.quantize_codebook(W, 64, codebook)
    cbr = bf16_exact(synth.f32_to_bf16_bits(np.asarray(codebook, np.float32)))
    want = np.repeat(alpha.astype(np.float64), 64, axis=1) * cbr[unpack_codes(codes)]
    assert np.array_equal(oracle.dequantize(codes, alpha, None, codebook, 64, 3), want)
