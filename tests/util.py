"""Helpers shared by the tests (no method arithmetic: array plumbing only)."""
import numpy as np


def unpack_codes(packed, M, bits):
    """Logical packed layout -> one byte per subspace [n][M]."""
    packed = np.asarray(packed, np.uint8)
    if bits == 8:
        return packed[:, :M].copy()
    out = np.empty((packed.shape[0], M), np.uint8)
    out[:, 0::2] = packed[:, : (M + 1) // 2] & 15
    out[:, 1::2] = (packed[:, : M // 2] >> 4) & 15
    return out


def unit_rows(rng, n, d):
    x = rng.standard_normal((n, d)).astype(np.float32)
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    return x.astype(np.float32)
