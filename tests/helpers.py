"""Small numpy helpers for the tests (format plumbing only)."""
import numpy as np


def unpack_codes(codes: np.ndarray) -> np.ndarray:
    """[d_out, d_in/2] packed bytes -> [d_out, d_in] code values; even k is the low nibble."""
    lo = codes & 0xF
    hi = codes >> 4
    return np.stack([lo, hi], axis=-1).reshape(codes.shape[0], -1).astype(np.int64)


def bf16_exact(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> float64 values (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def rel_to_rms(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / rms(ref)."""
    rms = float(np.sqrt(np.mean(np.square(ref, dtype=np.float64))))
    return float(np.max(np.abs(got.astype(np.float64) - ref))) / max(rms, 1e-300)
