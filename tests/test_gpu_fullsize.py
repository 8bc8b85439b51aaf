"""GPU parity at the full layer shapes of the workloads, in the launch configuration bench.py times.

The benchmark workload (LLaMA-7B attention projection, T = 8192, 4096 x 4096, rank 64, lambda 2) is
checked end to end: integer outputs bit for bit in full, forward / backward-dX on a seeded sample of
token rows (each output row depends on its own input row only, so the oracle evaluates exactly those
rows), the parameter gradients in full (they need every token).  The larger layer shapes (7B MLP,
65B with double-quantized scales) run with the real weight shape and a reduced token count so that
the fp64 oracle stays within seconds; they cover the non-power-of-two widths 11008 and 22016.
"""
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


def _run_layer(qb, oracle, codebook, seed, T, d_out, d_in, rank, lam, s, grouped, sample, full_grads,
               use_saved=False):
    from gpu_util import (f32_to_dev, to_np, bf16_to_dev, adapter_to_dev, assert_close_bf16, assert_close_f32,
                          bf16_to_f64)
    R = lam * rank
    print(f"full-size case T={T} {d_out}x{d_in} R={R} grouped={grouped}", flush=True)
    L = synth.make_layer(seed, T, d_out, d_in, R, lam, lam)
    qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook,
                                      qb.SCALES_E4M3_GROUPED if grouped else qb.SCALES_FP32)
    ad = adapter_to_dev(L, lam, lam, s)
    X, dY = bf16_to_dev(L.X), bf16_to_dev(L.dY)
    saved = torch.empty(qb.qblora_saved_bytes(ad, T), dtype=torch.uint8, device=X.device) if use_saved else None
    Y = qb.qblora_linear_fwd(qw, ad, X, saved=saved)                 # as bench.py calls them
    dX, dA, dB = qb.qblora_linear_bwd(qw, ad, X, dY, saved=saved)
    H = qb.qblora_tile_product(ad, d_in, d_out)
    merged = qb.qablora_merge_quantize(qw, H, lam, lam, s, qb.MERGE_REQUANT_MINMAX)      # the chain bench.py times
    Ho = oracle.tile_product(L.A, L.B).astype(np.float32)
    merged_o = qb.qablora_merge_quantize(qw, f32_to_dev(Ho), lam, lam, s, qb.MERGE_REQUANT_MINMAX)
    torch.cuda.synchronize()

    # integer paths, in full (everything the oracle is fed below is the oracle's own or the seeded input)
    codes, absmax = oracle.quantize_codebook(L.W, 64, codebook)
    assert np.array_equal(to_np(qw.codes), codes)
    assert np.array_equal(to_np(qw.scales).view(np.uint32), absmax.view(np.uint32))
    scales = absmax
    if grouped:
        sc, stp, mid = oracle.scales_double_quantize(absmax.reshape(-1), 256)
        assert np.array_equal(to_np(qw.scale_codes), sc)
        assert np.array_equal(to_np(qw.scale_step).view(np.uint32), stp.view(np.uint32))
        assert np.array_equal(to_np(qw.scale_mid).view(np.uint32), mid.view(np.uint32))
        scales = oracle.scales_double_dequantize(sc, stp, mid, 256).reshape(absmax.shape)
    # the merge, bit for bit, on the oracle's tile matrix; the device's own tile matrix differs from it in the
    # last fp32 bits (summation order), so the chained result is compared by how many codes may move
    co, ao, bo = oracle.merge_requant(codes, scales, None, codebook, Ho, 64, lam, lam, s)
    assert np.array_equal(to_np(merged_o.codes), co)
    assert np.array_equal(to_np(merged_o.scales).view(np.uint32), ao.view(np.uint32))
    assert np.array_equal(to_np(merged_o.beta).view(np.uint32), bo.view(np.uint32))
    assert_close_f32(H, oracle.tile_product(L.A, L.B), "H")
    assert np.mean(to_np(merged.codes) != co) < 1e-3
    assert np.allclose(to_np(merged.scales), ao, rtol=1e-5, atol=0) and np.allclose(to_np(merged.beta), bo, rtol=1e-4, atol=1e-7)

    # forward / backward-dX on sampled token rows
    Wt = oracle.dequantize(codes, scales, None, codebook, 64, 2)
    rows = synth.sample_rows(T, sample, seed)
    Xs, dYs = np.ascontiguousarray(L.X[rows]), np.ascontiguousarray(L.dY[rows])
    ridx = torch.from_numpy(rows).to(Y.device)
    assert_close_bf16(Y[ridx], oracle.forward(Wt, Xs, L.A, L.B, lam, lam, s), "Y (sampled rows)")
    rX, _, _ = oracle.backward(Wt, Xs, dYs, L.A, L.B, lam, lam, s, compute_dx=True, compute_dab=False)
    assert_close_bf16(dX[ridx], rX, "dX (sampled rows)")
    del Wt

    # parameter gradients need every token
    if full_grads:
        _, rA, rB = oracle.backward(None, L.X, L.dY, L.A, L.B, lam, lam, s, compute_dx=False, compute_dab=True,
                                    d_out=d_out, d_in=d_in)
        assert_close_f32(dA, rA, "dA")
        assert_close_f32(dB, rB, "dB")


def test_benchmark_workload_llama7b_attn(qb, oracle, codebook):
    wl = synth.WORKLOADS["llama7b_attn"]
    p = wl.projections[0]
    _run_layer(qb, oracle, codebook, wl.seed, wl.tokens, p.d_out, p.d_in, wl.rank, wl.lam, wl.s, False, 160, True, use_saved=True)


def test_llama7b_mlp_shapes_reduced_tokens(qb, oracle, codebook):
    wl = synth.WORKLOADS["llama7b_mlp"]
    for i, p in enumerate((wl.projections[0], wl.projections[2])):      # up [11008x4096] and down [4096x11008]
        _run_layer(qb, oracle, codebook, wl.seed + 1 + i, 768, p.d_out, p.d_in, wl.rank, wl.lam, wl.s, False, 96, True)


def test_llama13b_shapes_reduced_tokens(qb, oracle, codebook):
    wl = synth.WORKLOADS["llama13b_layer"]
    for i, p in enumerate((wl.projections[0], wl.projections[4])):      # attention [5120x5120] and up [13824x5120]
        _run_layer(qb, oracle, codebook, wl.seed + 1 + i, 512, p.d_out, p.d_in, wl.rank, wl.lam, wl.s, False, 64, True)


def test_llama65b_down_proj_grouped_scales_reduced_tokens(qb, oracle, codebook):
    wl = synth.WORKLOADS["llama65b_layer"]
    p = wl.projections[6]                                                # down_proj [8192 x 22016]
    _run_layer(qb, oracle, codebook, wl.seed + 7, 320, p.d_out, p.d_in, wl.rank, wl.lam, wl.s, True, 64, True)


def test_single_matrix_adapter_benchmark_shape(qb, oracle, codebook):
    """QA-BLoRA at the benchmark layer shape with the block-64 recommendation lambda = (8, 8)."""
    from gpu_util import f32_to_dev, to_np, bf16_to_dev, assert_close_bf16, assert_close_f32
    wl = synth.WORKLOADS["llama7b_attn"]
    p = wl.projections[0]
    T, d_out, d_in, lam1, lam2, s = wl.tokens, p.d_out, p.d_in, 8, 8, 1.0
    print(f"full-size single-matrix case T={T} {d_out}x{d_in} lam=({lam1},{lam2})", flush=True)
    L = synth.make_layer(wl.seed + 20, T, d_out, d_in, 8, lam1, lam2)
    Hb = synth.f32_to_bf16_bits((np.random.default_rng(wl.seed + 21).standard_normal((d_in // lam1, d_out // lam2)) * 0.02)
                                .astype(np.float32))
    qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook)
    H, X, dY = bf16_to_dev(Hb), bf16_to_dev(L.X), bf16_to_dev(L.dY)
    Y = qb.qablora_linear_fwd(qw, H, lam1, lam2, s, X)
    dX, dH = qb.qablora_linear_bwd(qw, H, lam1, lam2, s, X, dY)
    torch.cuda.synchronize()
    from gpu_util import OracleWeight
    Wt = OracleWeight(oracle, L.W, codebook).assert_same(qw).dequantize(oracle, 2)
    rows = synth.sample_rows(T, 128, wl.seed + 22)
    Xs, dYs = np.ascontiguousarray(L.X[rows]), np.ascontiguousarray(L.dY[rows])
    ridx = torch.from_numpy(rows).to(Y.device)
    assert_close_bf16(Y[ridx], oracle.qa_forward(Wt, Xs, Hb, lam1, lam2, s), "Y (sampled rows)")
    rX, _ = oracle.qa_backward(Wt, Xs, dYs, Hb, lam1, lam2, s, compute_dh=False)
    assert_close_bf16(dX[ridx], rX, "dX (sampled rows)")
    del Wt
    _, rH = oracle.qa_backward(None, L.X, L.dY, Hb, lam1, lam2, s, compute_dx=False, d_out=d_out, d_in=d_in)
    assert_close_f32(dH, rH, "dH")


@pytest.mark.parametrize("op", [1, 2])
def test_scale_operators_benchmark_shape(qb, oracle, codebook, op):
    """The ablation's alternative scale operators at the benchmark layer shape, as bench.py calls them."""
    from gpu_util import f32_to_dev, to_np, bf16_to_dev, assert_close_bf16, assert_close_f32
    wl = synth.WORKLOADS["llama7b_attn"]
    p = wl.projections[0]
    T, d_out, d_in, lam, s = wl.tokens, p.d_out, p.d_in, wl.lam, wl.s
    R = lam * wl.rank
    print(f"full-size scale-operator case op={op} T={T} {d_out}x{d_in} R={R}", flush=True)
    L = synth.make_layer(wl.seed + 30 + op, T, d_out, d_in, R, lam, lam)
    qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook)
    ad = qb.Adapter(bf16_to_dev(L.A), bf16_to_dev(L.B), lam, lam, s, scale_op=op)
    X, dY = bf16_to_dev(L.X), bf16_to_dev(L.dY)
    saved = torch.empty(qb.qblora_saved_bytes(ad, T), dtype=torch.uint8, device=X.device)
    Y = qb.qblora_linear_fwd(qw, ad, X, saved=saved)
    dX, dA, dB = qb.qblora_linear_bwd(qw, ad, X, dY, saved=saved)
    torch.cuda.synchronize()
    from gpu_util import OracleWeight
    Wt = OracleWeight(oracle, L.W, codebook).assert_same(qw).dequantize(oracle, 2)
    rows = synth.sample_rows(T, 128, wl.seed + 40 + op)
    Xs, dYs = np.ascontiguousarray(L.X[rows]), np.ascontiguousarray(L.dY[rows])
    ridx = torch.from_numpy(rows).to(Y.device)
    assert_close_bf16(Y[ridx], oracle.forward_op(Wt, Xs, L.A, L.B, lam, lam, s, op), "Y (sampled rows)")
    rX, _, _ = oracle.backward_op(Wt, Xs, dYs, L.A, L.B, lam, lam, s, op, compute_dab=False)
    assert_close_bf16(dX[ridx], rX, "dX (sampled rows)")
    del Wt
    _, rA, rB = oracle.backward_op(None, L.X, L.dY, L.A, L.B, lam, lam, s, op, compute_dx=False, d_out=d_out, d_in=d_in)
    assert_close_f32(dA, rA, "dA")
    assert_close_f32(dB, rB, "dB")


def _inference_on_sampled_rows(qb, oracle, d_out, d_in, tokens, seed):
    """Sampled output features of qblora_linear_decode on a packed INT4 model against the oracle (a feature needs its own
    weight row only), with 64-blocks and with 8 x 8 blocks."""
    from gpu_util import f32_to_dev, bf16_to_dev, bf16_to_f64, bf16_half_ulp
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((d_out, d_in), dtype=np.float32) * np.float32(0.02))
    rows = np.sort(rng.choice(d_out, 192, replace=False))
    cb = synth.codebook_int4()
    for block_rows in (1, 8):
        print(f"full-size decode case {d_out}x{d_in} block_rows={block_rows}", flush=True)
        qw = qb.qblora_quantize_blockwise(f32_to_dev(W), 64, qb.QUANT_MINMAX_INT4, tiled=False, block_rows=block_rows)
        pack = qb.qblora_decode_pack(qw)
        # the oracle's weight for the sampled rows: whole 8-row groups so that 8 x 8 blocks stay whole
        grp = np.unique(rows // 8)
        sel = (grp[:, None] * 8 + np.arange(8)[None, :]).reshape(-1)
        Wsel = np.ascontiguousarray(W[sel])
        if block_rows == 8:
            c, a, b = oracle.quantize_minmax_tile(Wsel, 8, 8)
            Wt = oracle.dequantize_tile(c, a, b, cb, 8, 8, 2)             # bf16 compute weight (8 x 8 inference arithmetic)
        else:
            c, a, b = oracle.quantize_minmax(Wsel, 64)
            Wt = oracle.dequantize(c, a, b, cb, 64, 3)                    # alpha * bf16(c) + beta
            Wt_mid = oracle.dequantize(c, a, b, cb, 64, 2)                # above 16 tokens: the bf16 compute weight
        sel_t = torch.from_numpy(sel).to(qw.codes.device)
        assert np.array_equal(qw.codes[sel_t].cpu().numpy(), c)          # the device weight holds the oracle's bits there
        for T in tokens:
            Xb = synth.f32_to_bf16_bits(rng.standard_normal((T, d_in), dtype=np.float32))
            Y = qb.qblora_linear_decode(qw, bf16_to_dev(Xb), pack=pack)
            torch.cuda.synchronize()
            ref = oracle.forward(Wt if (T <= 16 or block_rows == 8) else Wt_mid, Xb, None, None, 1, 1, 0.0)   # [T, len(sel)]
            got = bf16_to_f64(Y[:, sel_t])
            rms = np.sqrt(np.mean(ref ** 2))
            excess = np.abs(got - ref) - bf16_half_ulp(ref)
            assert excess.max() <= 1e-2 * rms, (block_rows, T, excess.max() / rms)
        del qw, pack


def test_small_batch_inference_at_the_measured_shape(qb, oracle):
    """The decode kernel on the 65B up-projection shape bench.py times among its side measurements (22016 x 8192, INT4 with
    offsets, tile-ordered pack): one token (all of X in LDS, two row groups per workgroup), 2 .. 16 (activations staged per
    wave, two row groups), and the mid-batch form at 32, 128 and 200 tokens."""
    _inference_on_sampled_rows(qb, oracle, 22016, 8192, (1, 2, 3, 7, 16, 32, 128, 200), 4242)


@pytest.mark.parametrize("d_out,d_in", [(8192, 22016), (8192, 8192)])
def test_small_batch_inference_short_layers(qb, oracle, d_out, d_in):
    """The 65B down and attention projections: at most two workgroups per CU, so the forms with eight waves per workgroup
    (one token; up to three at 8192 inputs) and the staged form with one row group."""
    _inference_on_sampled_rows(qb, oracle, d_out, d_in, (1, 2, 3, 4, 9, 16), 4243)


def test_8x8_blocks_mlp_shapes_reduced_tokens(qb, oracle, codebook):
    """The layer on 8 x 8 quantization blocks at the 7B MLP shapes (non-power-of-two widths), single-matrix adapter
    with lambda = (8, 8), forward / backward on sampled rows, dH in full, and the exact merge."""
    from gpu_util import f32_to_dev, to_np, bf16_to_dev, assert_close_bf16, assert_close_f32, OracleWeight
    from helpers import bf16_exact
    wl = synth.WORKLOADS["llama7b_mlp"]
    for i, p in enumerate((wl.projections[0], wl.projections[2])):
        T, d_out, d_in, lam1, lam2, s = 512, p.d_out, p.d_in, 8, 8, 1.0
        print(f"full-size 8x8 case T={T} {d_out}x{d_in}", flush=True)
        L = synth.make_layer(wl.seed + 50 + i, T, d_out, d_in, 8, lam1, lam2)
        Hb = synth.f32_to_bf16_bits((np.random.default_rng(wl.seed + 60 + i).standard_normal((d_in // lam1, d_out // lam2)) * 0.02)
                                    .astype(np.float32))
        qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 64, qb.QUANT_MINMAX_INT4, block_rows=8)
        H, X, dY = bf16_to_dev(Hb), bf16_to_dev(L.X), bf16_to_dev(L.dY)
        Y = qb.qablora_linear_fwd(qw, H, lam1, lam2, s, X)
        dX, dH = qb.qablora_linear_bwd(qw, H, lam1, lam2, s, X, dY)
        merged = qb.qablora_merge_quantize(qw, H.float().contiguous(), lam1, lam2, s, qb.MERGE_BETA_SHIFT)
        torch.cuda.synchronize()
        ow = OracleWeight(oracle, L.W, None, minmax=True, block_rows=8).assert_same(qw)
        Wt = ow.dequantize(oracle, 2)
        rows = synth.sample_rows(T, 64, wl.seed + 70 + i)
        Xs, dYs = np.ascontiguousarray(L.X[rows]), np.ascontiguousarray(L.dY[rows])
        ridx = torch.from_numpy(rows).to(Y.device)
        assert_close_bf16(Y[ridx], oracle.qa_forward(Wt, Xs, Hb, lam1, lam2, s), "Y (sampled rows)")
        rX, _ = oracle.qa_backward(Wt, Xs, dYs, Hb, lam1, lam2, s, compute_dh=False)
        assert_close_bf16(dX[ridx], rX, "dX (sampled rows)")
        del Wt
        _, rH = oracle.qa_backward(None, L.X, L.dY, Hb, lam1, lam2, s, compute_dx=False, d_out=d_out, d_in=d_in)
        assert_close_f32(dH, rH, "dH")
        want = oracle.merge_beta_shift_tile(ow.beta, bf16_exact(Hb).astype(np.float32), d_out, d_in, 8, 8, lam1, lam2, s)
        assert np.array_equal(to_np(merged.beta).view(np.uint32), want.view(np.uint32))


def test_token_count_beyond_2_31_elements(qb, oracle, codebook):
    """Maximum sizes: T * d exceeds 2^31 elements, so every row offset in the kernels must be 64-bit.

    The activations are a seeded block of 1024 token rows repeated down the token axis (513 times, ragged by 44
    rows): forward / backward-dX are checked on rows on both sides of element offset 2^31 and at the end, the
    parameter gradients in full -- the sum over tokens of a periodic input is the block's gradient times the
    number of repetitions plus the gradient of the ragged rest, both from the oracle.
    """
    from gpu_util import f32_to_dev, bf16_to_dev, adapter_to_dev, assert_close_bf16, assert_close_f32
    d_out, d_in, rank, lam, s, P = 4096, 4096, 16, 2, 0.5, 1024
    T = (2**31) // d_in + 300                                        # 524588 rows: 2.149e9 elements per tensor
    q, rem = divmod(T, P)
    print(f"large case T={T} {d_out}x{d_in} (period {P}, {q} repetitions + {rem})", flush=True)
    R = lam * rank
    L = synth.make_layer(4100, P, d_out, d_in, R, lam, lam)
    qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook)
    ad = adapter_to_dev(L, lam, lam, s)
    Xb, dYb = bf16_to_dev(L.X), bf16_to_dev(L.dY)
    X = torch.cat([Xb.repeat(q, 1), Xb[:rem]]).contiguous()
    dY = torch.cat([dYb.repeat(q, 1), dYb[:rem]]).contiguous()
    assert X.numel() > 2**31 and X.shape[0] == T
    Y = qb.qblora_linear_fwd(qw, ad, X)
    dX, dA, dB = qb.qblora_linear_bwd(qw, ad, X, dY)
    torch.cuda.synchronize()

    codes, absmax = oracle.quantize_codebook(L.W, 64, codebook)
    Wt = oracle.dequantize(codes, absmax, None, codebook, 64, 2)
    edge = (2**31) // d_in                                            # first row whose elements lie beyond 2^31
    rows = np.array([0, 1, P - 1, P, edge - 2, edge - 1, edge, edge + 1, edge + 255, T - 2, T - 1], dtype=np.int64)
    Xs, dYs = np.ascontiguousarray(L.X[rows % P]), np.ascontiguousarray(L.dY[rows % P])
    ridx = torch.from_numpy(rows).to(Y.device)
    assert_close_bf16(Y[ridx], oracle.forward(Wt, Xs, L.A, L.B, lam, lam, s), "Y (rows around 2^31)")
    rX, _, _ = oracle.backward(Wt, Xs, dYs, L.A, L.B, lam, lam, s, compute_dx=True, compute_dab=False)
    assert_close_bf16(dX[ridx], rX, "dX (rows around 2^31)")
    _, rA, rB = oracle.backward(None, L.X, L.dY, L.A, L.B, lam, lam, s, compute_dx=False, compute_dab=True,
                                d_out=d_out, d_in=d_in)
    _, rA2, rB2 = oracle.backward(None, np.ascontiguousarray(L.X[:rem]), np.ascontiguousarray(L.dY[:rem]), L.A, L.B,
                                  lam, lam, s, compute_dx=False, compute_dab=True, d_out=d_out, d_in=d_in)
    assert_close_f32(dA, q * rA + rA2, "dA")
    assert_close_f32(dB, q * rB + rB2, "dB")


def test_weight_beyond_2_31_elements(qb, oracle, codebook):
    """Maximum sizes on the weight side: d_out * d_in exceeds 2^31 elements (quantizers, tile-ordered copy,
    standalone dequantize, offset-shift merge).  The weight is a seeded block of 256 rows repeated down the row
    axis, so the oracle's result for the block is the expected value of every repetition; rows on both sides of
    element offset 2^31 and the last rows are compared bit for bit."""
    from gpu_util import f32_to_dev, to_np
    d_in, P = 32768, 256
    d_out = (2**31) // d_in + 2 * P                                  # 66048 rows: 2.164e9 elements
    Wb = synth.base_weight(4200, 0, P, d_in)
    print(f"large weight {d_out}x{d_in} (period {P})", flush=True)
    W = f32_to_dev(Wb).repeat(d_out // P, 1).contiguous()
    assert W.numel() > 2**31 and W.shape[0] == d_out
    edge = (2**31) // d_in
    spans = [(0, P), (edge - P, edge + P), (d_out - P, d_out)]        # whole periods: row r holds block row r % P

    codes_b, absmax_b = oracle.quantize_codebook(Wb, 64, codebook)
    qw = qb.qblora_quantize_blockwise(W, 64, qb.QUANT_ABSMAX_CODEBOOK, codebook)
    qm = qb.qblora_quantize_blockwise(W, 64, qb.QUANT_MINMAX_INT4, tiled=False)
    cm_b, am_b, bm_b = oracle.quantize_minmax(Wb, 64)
    Wd = qb.qblora_dequantize_bf16(qm)
    # offset-shift merge with lambda = (64, 8): one element of H per block, H periodic with the weight rows
    lam1, lam2, s = 64, 8, 0.75
    Hb = (np.random.default_rng(4201).standard_normal((d_in // lam1, P // lam2)) * 0.05).astype(np.float32)
    H = f32_to_dev(Hb).repeat(1, d_out // P).contiguous()
    merged = qb.qablora_merge_quantize(qm, H, lam1, lam2, s, qb.MERGE_BETA_SHIFT)
    torch.cuda.synchronize()
    beta_b = oracle.merge_beta_shift(bm_b, Hb, P, d_in, 64, lam1, lam2, s)
    Wd_b = oracle.dequantize(cm_b, am_b, bm_b, synth.codebook_int4(), 64, 2)
    from gpu_util import bf16_to_f64
    for lo, hi in spans:
        reps = (hi - lo) // P
        tile = lambda a: np.tile(a, (reps, 1))
        assert np.array_equal(to_np(qw.codes[lo:hi]), tile(codes_b))
        assert np.array_equal(to_np(qw.scales[lo:hi]).view(np.uint32), tile(absmax_b).view(np.uint32))
        assert np.array_equal(to_np(qm.codes[lo:hi]), tile(cm_b))
        assert np.array_equal(to_np(qm.scales[lo:hi]).view(np.uint32), tile(am_b).view(np.uint32))
        assert np.array_equal(to_np(qm.beta[lo:hi]).view(np.uint32), tile(bm_b).view(np.uint32))
        assert np.array_equal(to_np(merged.beta[lo:hi]).view(np.uint32), tile(beta_b).view(np.uint32))
        assert np.array_equal(bf16_to_f64(Wd[lo:hi]), tile(Wd_b))
    # the tile-ordered copy of the codes is the canonical one, re-ordered (both written by the quantizer)
    tiled_again = torch.empty_like(qw.codes_tiled)
    keep = qw.codes_tiled
    qw.codes_tiled = tiled_again
    qb.qblora_prepack_codes(qw)
    torch.cuda.synchronize()
    assert torch.equal(keep, tiled_again)
