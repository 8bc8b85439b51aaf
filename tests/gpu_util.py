"""Plumbing for the GPU parity tests: numpy <-> device tensors and the tolerance rule."""
import numpy as np
import torch

from paper_2407_17029_amd import binding as qb
from paper_2407_17029_amd import synth

DEV = "cuda:0"


def bf16_to_dev(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(DEV)


def bf16_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def f32_to_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy()


def adapter_to_dev(L, lam1, lam2, s):
    return qb.Adapter(bf16_to_dev(L.A), bf16_to_dev(L.B), lam1, lam2, s)


def qweight_from_oracle(codes, alpha, beta, codebook, block=64):
    return qb.QWeight(codes.shape[0], codes.shape[1] * 2, block, codebook,
                      torch.from_numpy(codes).to(DEV), f32_to_dev(alpha),
                      None if beta is None else f32_to_dev(beta))


class OracleWeight:
    """The quantized frozen weight as the oracle produces it from the seeded fp32 matrix: everything the
    oracle is later fed comes from here, never from a device buffer."""

    def __init__(self, oracle, W, codebook, minmax=False, grouped=False, block_rows=1):
        self.block_rows = block_rows
        self.sc = self.step = self.mid = None
        if minmax:
            self.cb = synth.codebook_int4()
            if block_rows == 8:
                self.codes, self.alpha, self.beta = oracle.quantize_minmax_tile(W, 8, 8)
            else:
                self.codes, self.alpha, self.beta = oracle.quantize_minmax(W, 64)
        else:
            self.cb = np.asarray(codebook, np.float32)
            self.beta = None
            if block_rows == 8:
                self.codes, self.alpha = oracle.quantize_codebook_tile(W, 8, 8, codebook)
            else:
                self.codes, self.alpha = oracle.quantize_codebook(W, 64, codebook)
        self.scales = self.alpha                     # what consumers read
        if grouped:
            self.sc, self.step, self.mid = oracle.scales_double_quantize(self.alpha.reshape(-1), 256)
            self.scales = oracle.scales_double_dequantize(self.sc, self.step, self.mid, 256).reshape(self.alpha.shape)

    def dequantize(self, oracle, mode):
        if self.block_rows == 8:
            return oracle.dequantize_tile(self.codes, self.scales, self.beta, self.cb, 8, 8, mode)
        return oracle.dequantize(self.codes, self.scales, self.beta, self.cb, 64, mode)

    def assert_same(self, qw):
        """The device weight holds the oracle's bits (codes, scales, offsets, second-level scale codes)."""
        bits = lambda a: np.ascontiguousarray(a).view(np.uint32)
        assert np.array_equal(to_np(qw.codes), self.codes), "codes"
        assert np.array_equal(bits(to_np(qw.scales)).reshape(-1), bits(self.alpha).reshape(-1)), "scales"
        if self.beta is None:
            assert qw.beta is None
        else:
            assert np.array_equal(bits(to_np(qw.beta)).reshape(-1), bits(self.beta).reshape(-1)), "offsets"
        if self.sc is not None:
            assert np.array_equal(to_np(qw.scale_codes), self.sc), "scale codes"
            assert np.array_equal(bits(to_np(qw.scale_step)), bits(self.step)), "scale steps"
            assert np.array_equal(bits(to_np(qw.scale_mid)), bits(self.mid)), "scale mids"
        return self


REL_TOL = 1e-2            # max |gpu - oracle| / rms(oracle), the bar for bf16 outputs and gradients


def assert_close_bf16(got_bf16: torch.Tensor, ref: np.ndarray, what: str):
    """bf16 output vs fp64 oracle.

    A bf16 value carries 8 significant bits, so even the correctly rounded oracle value sits up to
    2^-9 * |ref| (half an ulp, at most 2^-8 relative to the power of two below it) away from the
    oracle; that representation term is allowed on top of the 1e-2 * rms bar and reported apart.
    """
    got = bf16_to_f64(got_bf16)
    rms = float(np.sqrt(np.mean(ref * ref)))
    err = np.abs(got - ref)
    excess = err - np.abs(ref) * 2.0 ** -8
    worst = float(excess.max()) / max(rms, 1e-300)
    raw = float(err.max()) / max(rms, 1e-300)
    rms_err = float(np.sqrt(np.mean(err * err))) / max(rms, 1e-300)
    assert worst <= REL_TOL, f"{what}: max excess err/rms {worst:.3e} (raw {raw:.3e}, rms err {rms_err:.3e})"
    assert rms_err <= REL_TOL, f"{what}: rms err/rms {rms_err:.3e}"
    return raw, rms_err


def assert_close_f32(got: torch.Tensor, ref: np.ndarray, what: str):
    g = to_np(got).astype(np.float64)
    rms = float(np.sqrt(np.mean(ref * ref)))
    worst = float(np.abs(g - ref).max()) / max(rms, 1e-300)
    assert worst <= REL_TOL, f"{what}: max err/rms {worst:.3e}"
    return worst
