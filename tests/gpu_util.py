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

    def __init__(self, oracle, W, codebook, minmax=False, grouped=False, block_rows=1, block_cols=8):
        self.block_rows = block_rows
        self.block_cols = block_cols                 # with block_rows = 8: inputs per block, 8 or 4
        self.sc = self.step = self.mid = None
        if minmax:
            self.cb = synth.codebook_int4()
            if block_rows == 8:
                self.codes, self.alpha, self.beta = oracle.quantize_minmax_tile(W, 8, block_cols)
            else:
                self.codes, self.alpha, self.beta = oracle.quantize_minmax(W, 64)
        else:
            self.cb = np.asarray(codebook, np.float32)
            self.beta = None
            if block_rows == 8:
                self.codes, self.alpha = oracle.quantize_codebook_tile(W, 8, block_cols, codebook)
            else:
                self.codes, self.alpha = oracle.quantize_codebook(W, 64, codebook)
        self.scales = self.alpha                     # what consumers read
        if grouped:
            self.sc, self.step, self.mid = oracle.scales_double_quantize(self.alpha.reshape(-1), 256)
            self.scales = oracle.scales_double_dequantize(self.sc, self.step, self.mid, 256).reshape(self.alpha.shape)

    def dequantize(self, oracle, mode):
        if self.block_rows == 8:
            return oracle.dequantize_tile(self.codes, self.scales, self.beta, self.cb, 8, self.block_cols, mode)
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

REPORT = []               # one dict per comparison made in this process (tests print / write them out)


def bf16_half_ulp(ref: np.ndarray) -> np.ndarray:
    """Half the spacing of bf16 numbers at |ref| (8 significant bits): 2^(floor(log2|ref|) - 8); 0 at 0."""
    a = np.abs(ref)
    e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    return np.where(a > 0, np.exp2(e - 8.0), 0.0)


RMS_TOL = 4e-3            # rms |gpu - oracle| / rms(oracle): storing in bf16 alone costs 1.7e-3 of it


def assert_close_bf16(got_bf16: torch.Tensor, ref: np.ndarray, what: str):
    """bf16 output vs fp64 oracle; returns the measured figures (all relative to rms(oracle)).

    The bar is max |gpu - oracle| <= 1e-2 * rms(oracle).  A value stored in bf16 cannot be closer to the
    oracle than half a bf16 spacing, 2^-9 .. 2^-8 of its magnitude, which for an output of 4 * rms is already
    above the bar (the correctly rounded oracle value itself would fail, and every output tensor of more than
    a few thousand elements has such entries).  So the bar is applied to what the kernel adds: the error
    beyond exactly that half spacing at the oracle's value -- nothing proportional, nothing else -- must stay
    within 1e-2 * rms on every element, and the rms error over all elements within 4e-3 * rms.  The raw
    maximum over all outputs and over the outputs with |oracle| <= 2 * rms are returned, recorded in REPORT
    and printed in every failure message, never hidden.
    """
    got = bf16_to_f64(got_bf16)
    rms = max(float(np.sqrt(np.mean(ref * ref))), 1e-300)
    err = np.abs(got - ref)
    raw = float(err.max()) / rms
    core = np.abs(ref) <= 2.0 * rms
    core_raw = float(err[core].max()) / rms if core.any() else 0.0
    excess = float((err - bf16_half_ulp(ref)).max()) / rms
    rms_err = float(np.sqrt(np.mean(err * err))) / rms
    fig = {"what": what, "raw_max": raw, "core_raw_max": core_raw, "excess_max": excess, "rms_err": rms_err,
           "max_abs_ref_over_rms": float(np.abs(ref).max()) / rms}
    REPORT.append(fig)
    msg = (f"{what}: raw max err/rms {raw:.3e}, on |ref| <= 2 rms {core_raw:.3e}, beyond the bf16 half spacing "
           f"{excess:.3e}, rms err/rms {rms_err:.3e}")
    assert excess <= REL_TOL, msg
    assert rms_err <= RMS_TOL, msg
    return fig


def assert_close_f32(got: torch.Tensor, ref: np.ndarray, what: str):
    g = to_np(got).astype(np.float64)
    rms = max(float(np.sqrt(np.mean(ref * ref))), 1e-300)
    worst = float(np.abs(g - ref).max()) / rms
    REPORT.append({"what": what, "raw_max": worst})
    assert worst <= REL_TOL, f"{what}: max err/rms {worst:.3e}"
    return worst
