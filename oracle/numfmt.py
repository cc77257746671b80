"""bfloat16 emulation for the oracle (test infrastructure only).

bfloat16 is the upper 16 bits of an IEEE-754 binary32; conversion from
binary32 is round-to-nearest, ties-to-even on the discarded 16 bits.
"""
import numpy as np


def round_bf16(x):
    """Round every element to the nearest bfloat16 value (ties to even).

    Input of any float dtype is first rounded to binary32 (what the GPU holds
    before it converts), then to bfloat16.  The result keeps the input dtype.
    Finite inputs only (NaN/Inf are not part of any workload here).
    """
    x = np.asarray(x)
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    r = u.astype(np.uint32).view(np.float32).reshape(f.shape)
    return r.astype(x.dtype if x.dtype.kind == "f" else np.float32)
