"""bfloat16 rounding emulation for the oracle (round to nearest, ties to even).

The paper is silent on precision.  For the bf16-input workloads the reading
taken is: a value is first held in fp32 and then narrowed to bf16, so the
emulation rounds fp64 -> fp32 -> bf16 and returns the result as fp64.
"""
from __future__ import annotations

import numpy as np


def round_bf16(x) -> np.ndarray:
    """Nearest bf16 value (ties to even) of each element, returned as float64."""
    f32 = np.asarray(x, dtype=np.float64).astype(np.float32)
    bits = f32.view(np.uint32).astype(np.uint64)
    keep = bits >> np.uint64(16)
    rem = bits & np.uint64(0xFFFF)
    up = (rem > np.uint64(0x8000)) | ((rem == np.uint64(0x8000)) & ((keep & np.uint64(1)) == 1))
    keep = keep + up.astype(np.uint64)
    out = (keep << np.uint64(16)).astype(np.uint32).view(np.float32)
    nan = np.isnan(f32)
    if nan.any():
        out = np.where(nan, np.float32(np.nan), out)
    return out.astype(np.float64)


def bits_to_f64(payload_u16) -> np.ndarray:
    """uint16 bf16 payload -> float64 values."""
    b = np.asarray(payload_u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)
