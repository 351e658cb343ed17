"""bfloat16 storage <-> fp64 (oracle's own copy; the HIP path has its own)."""
import numpy as np


def decode(bits):
    """uint16 bf16 bit patterns -> float64 (exact)."""
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def encode(x64):
    """float64 -> bf16 bits.  Two roundings (fp64->fp32->bf16, both to nearest even),
    matching a kernel that accumulates in fp32 and stores bf16."""
    f = np.asarray(x64, dtype=np.float64).astype(np.float32)
    u = np.ascontiguousarray(f).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)
