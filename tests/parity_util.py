"""Helpers for the GPU parity tests: device buffers from bf16 bit patterns, tolerance checks."""
import numpy as np

# Float tolerance of the path (projection, norm, RoPE) against the fp64 oracle:
# max |g - o| <= ABS_TOL and max |g - o| / max(|o|, 1) <= REL_TOL, where g is the GPU's bf16
# output widened exactly.  One bf16 rounding of a value below 8 in magnitude is at most 2^-6 = 0.0156.
ABS_TOL = 2e-2
REL_TOL = 1e-2


def to_dev(bits: np.ndarray):
    """uint16 bit patterns (or int32/float32 arrays) -> torch tensor on cuda:0 (bf16 bits travel as int16)."""
    import torch
    a = np.ascontiguousarray(bits)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).to("cuda:0")


def dev_empty(shape, dtype="bits"):
    import torch
    dt = {"bits": torch.int16, "i32": torch.int32, "u8": torch.uint8, "f32": torch.float32}[dtype]
    return torch.empty(shape, dtype=dt, device="cuda:0")


def to_host_bits(t) -> np.ndarray:
    return t.cpu().numpy().view(np.uint16)


def widen_bits(bits: np.ndarray) -> np.ndarray:
    """bf16 bits -> float64 (test-side helper, independent of the library)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    with np.errstate(invalid="ignore"):
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def float_errors(gpu_bits: np.ndarray, oracle_f64: np.ndarray):
    g = widen_bits(gpu_bits)
    err = np.abs(g - oracle_f64)
    return float(err.max()), float((err / np.maximum(np.abs(oracle_f64), 1.0)).max())


def assert_float_parity(gpu_bits: np.ndarray, oracle_f64: np.ndarray, what: str = ""):
    assert gpu_bits.shape == oracle_f64.shape, (gpu_bits.shape, oracle_f64.shape)
    abs_err, rel_err = float_errors(gpu_bits, oracle_f64)
    assert abs_err <= ABS_TOL and rel_err <= REL_TOL, f"{what}: max abs {abs_err:.4g}, max rel {rel_err:.4g}"
    return abs_err, rel_err
