"""bfloat16 storage helpers: numpy has no bf16, so tensors travel as uint16 bit patterns."""
import numpy as np


def f32_to_bf16_bits(x):
    """Round-to-nearest-even float32 -> bf16 bit pattern (uint16). Finite inputs only."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits):
    """Exact widening of bf16 bit patterns to float32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
