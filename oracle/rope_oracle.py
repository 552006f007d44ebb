"""TEST INFRASTRUCTURE ONLY - plain fp64 reference for rotary position embedding on a packed
buffer with the position reset at every sequence start.  Packing requires that "positional
embeddings ... be adjusted" so that a sequence inside a buffer sees the positions it would see
alone (arXiv 2412.07894, Sec. 2.1, the packing paragraph); the paper names no embedding, its models
are LLaMA 2 (Sec. 8.1), which use rotary embeddings (Su et al., RoFormer, Eq. 34).  The reading
taken here, stated because the paper is silent:

    position of packed row t of sequence s:   m = t - cu_seqlens[s]            (local, from 0)
    pair i of a head's d elements:            (x[i], x[i + d/2]),  i in [0, d/2)   ("rotate-half")
    angle:                                    m * base^(-2 i / d),  base = 10000 unless given
    forward:   y[i]       = x[i] cos - x[i + d/2] sin
               y[i + d/2] = x[i + d/2] cos + x[i] sin
    inverse (the transpose; it carries gradients back through the rotation): angle negated.

Dense numpy, one row at a time.  Only tests/ may import this module.
"""
import numpy as np


def positions(cu, total):
    """Local position of every packed row."""
    pos = np.zeros(total, dtype=np.int64)
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        pos[a:b] = np.arange(b - a)
    return pos


def rope_packed(x, cu, base=10000.0, inverse=False):
    """x [T, H, d] -> rotated copy (fp64)."""
    x = np.asarray(x, dtype=np.float64)
    T, H, d = x.shape
    half = d // 2
    out = np.empty_like(x)
    pos = positions(cu, T)
    inv_freq = np.array([base ** (-2.0 * i / d) for i in range(half)])
    for t in range(T):
        ang = pos[t] * inv_freq
        if inverse:
            ang = -ang
        c, s = np.cos(ang), np.sin(ang)
        lo, hi = x[t, :, :half], x[t, :, half:]
        out[t, :, :half] = lo * c - hi * s
        out[t, :, half:] = hi * c + lo * s
    return out
