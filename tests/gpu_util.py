"""Helpers for the GPU parity tests: move stored bytes to the device and back.

No arithmetic of the method lives here.  Device tensors are plain byte
containers (torch is only the allocator); decoding of results is done by the
oracle's number-format module.
"""
import numpy as np
import torch

import paper_2105_14450_amd as c3
from oracle import numfmt

TORCH_STORAGE = {"f32": torch.float32, "bf16": torch.int16, "fp8_e4m3": torch.uint8}
NP_STORAGE = {"f32": np.float32, "bf16": np.uint16, "fp8_e4m3": np.uint8}
CODE = c3.binding.DTYPE_CODES


def to_device(raw: np.ndarray) -> torch.Tensor:
    raw = np.ascontiguousarray(raw)
    if raw.dtype == np.uint16:
        raw = raw.view(np.int16)
    return torch.from_numpy(raw).cuda()


def empty(shape, dtype: str) -> torch.Tensor:
    # poison the buffer so that an element the kernel never writes is caught
    t = torch.empty(shape, dtype=TORCH_STORAGE[dtype], device="cuda")
    t.view(torch.uint8).fill_(0xFF if dtype != "fp8_e4m3" else 0x7F)
    return t


def to_host(t: torch.Tensor, dtype: str) -> np.ndarray:
    """Device result -> fp64 values."""
    a = t.cpu().numpy()
    if dtype == "bf16":
        return numfmt.decode_bf16(a.view(np.uint16))
    return a.astype(np.float64)


def raw_host(t: torch.Tensor) -> np.ndarray:
    a = t.cpu().numpy()
    return a.view(np.uint16) if a.dtype == np.int16 else a


def scaled_max_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / max |ref| (the error measure of the stated tolerances)."""
    denom = float(np.max(np.abs(ref))) if ref.size else 1.0
    if denom == 0.0:
        denom = 1.0
    return float(np.max(np.abs(got - ref))) / denom if ref.size else 0.0


# Stated tolerances of the scale-normalised error, per dtype (the benchmark's target sentence).
TOL = {"f32": 1e-5, "bf16": 2e-2, "fp8_e4m3": 2e-2}

# What the arithmetic allows, per dtype the compared values were last rounded to.  Both sides
# read the same stored inputs, so the only differences are the accumulation and each bf16
# rounding on the way (<= 2^-8 of the rounded value).  Accumulation: fp32 inputs go through
# fp32 multiply-adds (relative ~ sqrt(Kc) * 2^-24 of the sum of |terms|, far below 2e-5 of the
# largest entry).  bf16 and fp8 inputs go through the matrix cores' multi-term adds, which align
# the exact products of one instruction to the largest of them and drop what falls below its
# last fp32 bit: up to ~ Kc * 2^-24 * max|term|, measured 3e-5 of the largest entry at Kc = 45
# and below 1e-4 up to Kc = 8192 on N(0,1) data.
#   scaled: bound on max|got - ref| / max|ref|
#   rel, floor: per-element bound |got - ref| <= rel * |ref| + floor * max|ref|
TIGHT = {"f32": {"scaled": 2e-5, "rel": 0.0, "floor": 2e-5},
         "f32acc": {"scaled": 1e-4, "rel": 0.0, "floor": 1e-4},
         "bf16": {"scaled": 4e-3, "rel": 2.0 ** -8, "floor": 1e-4},
         # a sum of q bf16-rounded partial products (rounded to bf16 again or kept in fp32)
         "bf16x2": {"scaled": 1e-2, "rel": 2.0 ** -8, "floor": 8e-3}}


def check_close(got: np.ndarray, ref: np.ndarray, kind: str, what: str):
    """Element-by-element comparison within TIGHT[kind]."""
    t = TIGHT[kind]
    scale = float(np.max(np.abs(ref))) if ref.size else 1.0
    scale = scale or 1.0
    diff = np.abs(got - ref)
    err = float(np.max(diff)) / scale if ref.size else 0.0
    assert err <= t["scaled"], "%s: scaled max error %g > %g" % (what, err, t["scaled"])
    bound = t["rel"] * np.abs(ref) + t["floor"] * scale
    bad = diff > bound
    assert not bad.any(), "%s: %d elements outside |err| <= %g |ref| + %g max|ref| (worst excess %g)" % (
        what, int(bad.sum()), t["rel"], t["floor"], float(np.max(diff - bound)))


def workspace(desc, op, batched):
    n = c3.cube3d_workspace_bytes(desc, op, batched)
    return torch.empty(max(n, 16), dtype=torch.uint8, device="cuda") if n else None
