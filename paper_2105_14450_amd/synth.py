"""Seeded synthetic inputs for the 3-D linear layer's hot path.

This module only draws numbers and stores them in the dtype a kernel reads
(fp32, bf16 bit patterns, fp8-e4m3 codes with a per-tensor scale).  It holds
none of the method's arithmetic: no products, no block slicing, no collectives.
Both the GPU path and the CPU oracle receive the very same stored bytes; each
side decodes them with its own code.

The paper's experiments run Transformer linears at hidden sizes 2048 and 8192
with sequence length 512 (Table 1) on unspecified training batches, so the
inputs here are synthetic with the usual statistics of such layers:
activations and output gradients ~ N(0, 1), weights ~ N(0, sigma = 0.02); plus
uniform[-1, 1] for the small fp32 case and small integers in [-4, 4] for the
bit-exact cases (every product and partial sum is then exact in fp32).
"""
import numpy as np

DTYPES = ("f32", "bf16", "fp8_e4m3")

# tensor ids: one independent Philox stream per (seed, tensor)
TID_X, TID_W, TID_DY = 1, 2, 3


def stream(seed: int, tensor_id: int) -> np.random.Generator:
    """Counter-based generator keyed by (seed, tensor id)."""
    return np.random.Generator(np.random.Philox(key=[int(seed), int(tensor_id)]))


def draw(shape, dist: str, seed: int, tensor_id: int, sigma: float = 1.0) -> np.ndarray:
    """fp32 draws. dist: 'uniform' on [-1,1), 'normal' N(0, sigma), 'int' on {-4..4}."""
    g = stream(seed, tensor_id)
    if dist == "uniform":
        return g.uniform(-1.0, 1.0, size=shape).astype(np.float32)
    if dist == "normal":
        return (g.standard_normal(size=shape, dtype=np.float32) * np.float32(sigma))
    if dist == "int":
        return g.integers(-4, 5, size=shape).astype(np.float32)
    raise ValueError(dist)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the uint16 patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def _e4m3_magnitudes() -> np.ndarray:
    mags = []
    for code in range(0x7F):                # 0x7F is NaN in the "fn" encoding
        e, m = code >> 3, code & 7
        mags.append((m / 8.0) * 2.0 ** -6 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7))
    return np.array(mags, dtype=np.float64)


_MAGS = _e4m3_magnitudes()
E4M3_MAX = 448.0


def f32_to_e4m3(x: np.ndarray, scale: float) -> np.ndarray:
    """Quantise x/scale to fp8 e4m3 (nearest, ties to even code, saturating)."""
    y = np.asarray(x, dtype=np.float64) / float(scale)
    mag = np.minimum(np.abs(y), E4M3_MAX)
    hi = np.clip(np.searchsorted(_MAGS, mag, side="left"), 1, len(_MAGS) - 1)
    lo = hi - 1
    d_lo = mag - _MAGS[lo]
    d_hi = _MAGS[hi] - mag
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    return np.where(np.signbit(y), code | np.uint8(0x80), code).astype(np.uint8)


def store(x_f32: np.ndarray, dtype: str, integer_valued: bool = False):
    """Encode fp32 draws in `dtype`. Returns (raw array, scale)."""
    if dtype == "f32":
        return np.ascontiguousarray(x_f32, dtype=np.float32), 1.0
    if dtype == "bf16":
        return f32_to_bf16_bits(x_f32), 1.0
    if dtype == "fp8_e4m3":
        if integer_valued:
            scale = 1.0
        else:
            amax = float(np.max(np.abs(x_f32))) if x_f32.size else 0.0
            scale = amax / E4M3_MAX if amax > 0 else 1.0
            scale = float(np.float32(scale))
        return f32_to_e4m3(x_f32, scale), scale
    raise ValueError(dtype)


def linear_inputs(M: int, K: int, N: int, dtype: str, dist: str, seed: int):
    """Stored X [M,K], W [K,N], dY [M,N] for one linear layer.

    dist 'uniform' / 'int' apply to all three tensors; 'normal' means
    X, dY ~ N(0,1) and W ~ N(0, 0.02).
    Returns a dict: name -> (raw array, scale).
    """
    integer = dist == "int"
    sig_w = 0.02 if dist == "normal" else 1.0
    out = {}
    out["X"] = store(draw((M, K), dist, seed, TID_X), dtype, integer)
    out["W"] = store(draw((K, N), dist, seed, TID_W, sig_w), dtype, integer)
    out["dY"] = store(draw((M, N), dist, seed, TID_DY), dtype, integer)
    return out


NUMPY_STORAGE = {"f32": np.float32, "bf16": np.uint16, "fp8_e4m3": np.uint8}
