"""GPU parity of the alternative scale operators (ablation "The scale operators", Table 6): truncation with
zero padding and interval sampling with zero fill, forward and backward, against the fp64 oracle."""
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


def _setup(qb, oracle, codebook, seed, T, d_out, d_in, R, lam1, lam2, s, op):
    from gpu_util import f32_to_dev, bf16_to_dev, OracleWeight
    L = synth.make_layer(seed, T, d_out, d_in, R, lam1, lam2)
    qw = qb.qblora_quantize_blockwise(f32_to_dev(L.W), 64, qb.QUANT_ABSMAX_CODEBOOK, codebook)
    torch.cuda.synchronize()
    Wt = OracleWeight(oracle, L.W, codebook).assert_same(qw).dequantize(oracle, 2)
    ad = qb.Adapter(bf16_to_dev(L.A), bf16_to_dev(L.B), lam1, lam2, s, scale_op=op)
    return L, qw, Wt, ad, bf16_to_dev(L.X), bf16_to_dev(L.dY)


CASES = [
    # T, d_out, d_in, R, lam1, lam2, s
    (256, 512, 512, 32, 2, 2, 1.0),
    (300, 320, 192, 16, 2, 2, 0.25),         # ragged token count, partial tiles in every dimension
    (77, 576, 832, 64, 4, 8, 2.0),           # lambda1 != lambda2
    (513, 512, 1024, 128, 8, 8, 1.0),
]


@pytest.mark.parametrize("op", [1, 2])
@pytest.mark.parametrize("T,d_out,d_in,R,lam1,lam2,s", CASES)
def test_forward_backward_parity(qb, oracle, codebook, T, d_out, d_in, R, lam1, lam2, s, op):
    from gpu_util import assert_close_bf16, assert_close_f32
    print(f"case op={op} T={T} {d_out}x{d_in} R={R} lam=({lam1},{lam2})", flush=True)
    L, qw, Wt, ad, X, dY = _setup(qb, oracle, codebook, 900 + T + op, T, d_out, d_in, R, lam1, lam2, s, op)
    Y = qb.qblora_linear_fwd(qw, ad, X)
    dX, dA, dB = qb.qblora_linear_bwd(qw, ad, X, dY)
    torch.cuda.synchronize()
    assert_close_bf16(Y, oracle.forward_op(Wt, L.X, L.A, L.B, lam1, lam2, s, op), "Y")
    rX, rA, rB = oracle.backward_op(Wt, L.X, L.dY, L.A, L.B, lam1, lam2, s, op)
    assert_close_bf16(dX, rX, "dX")
    assert_close_f32(dA, rA, "dA")
    assert_close_f32(dB, rB, "dB")


@pytest.mark.parametrize("op", [1, 2])
def test_saved_activation_and_partial_outputs(qb, oracle, codebook, op):
    """The forms that keep s*U between the passes, and dX-only / gradients-only calls, give the same bits."""
    from gpu_util import to_np
    T, d_out, d_in, R, lam1, lam2, s = 200, 256, 384, 16, 2, 4, 0.5
    L, qw, Wt, ad, X, dY = _setup(qb, oracle, codebook, 950 + op, T, d_out, d_in, R, lam1, lam2, s, op)
    Y = qb.qblora_linear_fwd(qw, ad, X)
    dX, dA, dB = qb.qblora_linear_bwd(qw, ad, X, dY)
    saved = torch.empty(qb.qblora_saved_bytes(ad, T), dtype=torch.uint8, device=X.device)
    Y2 = qb.qblora_linear_fwd(qw, ad, X, saved=saved)
    dX2, dA2, dB2 = qb.qblora_linear_bwd(qw, ad, X, dY, saved=saved)
    dX3, _, _ = qb.qblora_linear_bwd(qw, ad, X, dY, True, False)
    _, dA4, dB4 = qb.qblora_linear_bwd(qw, ad, X, dY, False, True)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y2) and torch.equal(dX, dX2) and torch.equal(dX, dX3)
    assert np.array_equal(to_np(dA), to_np(dA2)) and np.array_equal(to_np(dB), to_np(dB2))
    assert np.array_equal(to_np(dA), to_np(dA4)) and np.array_equal(to_np(dB), to_np(dB4))


def test_operators_coincide_at_lambda_one_and_errors(qb, oracle, codebook):
    from gpu_util import bf16_to_dev
    T, d_out, d_in, R = 130, 256, 256, 8
    L, qw, Wt, ad0, X, dY = _setup(qb, oracle, codebook, 960, T, d_out, d_in, R, 1, 1, 1.0, 0)
    Y0 = qb.qblora_linear_fwd(qw, ad0, X)
    for op in (1, 2):
        ad = qb.Adapter(ad0.A, ad0.B, 1, 1, 1.0, scale_op=op)
        Y = qb.qblora_linear_fwd(qw, ad, X)
        torch.cuda.synchronize()
        assert torch.equal(Y, Y0)                      # identical operands reach the same kernels
    bad = qb.Adapter(ad0.A, ad0.B, 1, 1, 1.0, scale_op=7)
    with pytest.raises(qb.QBLoRAError):
        qb.qblora_linear_fwd(qw, bad, X)
    alt = qb.Adapter(ad0.A, ad0.B, 1, 1, 1.0, scale_op=1)
    with pytest.raises(qb.QBLoRAError):
        qb.qblora_tile_product(alt, d_in, d_out)       # no tile-constant delta weight to merge
