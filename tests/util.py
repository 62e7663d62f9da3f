"""Shared test helpers: code conversion with library routines (numpy / torch), never the oracle's own."""
import numpy as np
import torch

F16, BF16 = 0, 1


def codes_from_floats(x, dtype_code):
    """Round an array of floats to the 16-bit format and return (codes uint16, rounded values fp64)."""
    x = np.array(x, dtype=np.float64)
    if dtype_code == F16:
        h = x.astype(np.float16)
        return h.view(np.uint16).copy(), h.astype(np.float64)
    t = torch.from_numpy(x).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy(), t.to(torch.float64).numpy()


def floats_from_codes(c, dtype_code):
    c = np.ascontiguousarray(c, dtype=np.uint16)
    if dtype_code == F16:
        return c.view(np.float16).astype(np.float64)
    return (c.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
