"""The packed code layout of include/hif4.h, restated for the tests: within each group of
8 elements (4 bytes), byte t holds element t in its low nibble and element t + 4 in its
high nibble."""
import numpy as np


def nibbles_to_codes(n):
    """[..., K] nibbles -> [..., K/2] bytes."""
    n = np.asarray(n, dtype=np.uint8)
    g = n.reshape(n.shape[:-1] + (n.shape[-1] // 8, 2, 4))
    return (g[..., 0, :] | (g[..., 1, :] << 4)).reshape(n.shape[:-1] + (n.shape[-1] // 2,)).astype(np.uint8)


def codes_to_nibbles(c):
    """[..., K/2] bytes -> [..., K] nibbles."""
    c = np.asarray(c, dtype=np.uint8)
    g = c.reshape(c.shape[:-1] + (c.shape[-1] // 4, 4))
    out = np.stack([g & 0xF, g >> 4], axis=-2)
    return out.reshape(c.shape[:-1] + (c.shape[-1] * 2,)).astype(np.uint8)
