"""Rotary position shift in float64 (oracle side).

The paper leaves the positional embedding out of its figure (Fig. 7 caption) and
only says that a stored cache lacks position information (Sec. 2.3).  The build
target fixes the reading: a cached key computed at chunk-local position t is moved
to global position off + t by rotating it by the angle of `off`.  Pairing is the
rotate-half convention of the LLaMA-family decoders inside LLaVA (Sec. 5.1):
coordinate i pairs with i + D/2 and turns by delta * theta**(-2i/D); the
interleaved convention pairs (2i, 2i+1) with the same frequencies.
"""
import numpy as np


def rotate(x, delta, theta, interleaved=False):
    """Rotate head vectors x[..., D] (float64) by position shift `delta`.

    `delta` is a scalar or an array broadcastable against x[..., 0].
    """
    x = np.asarray(x, dtype=np.float64)
    D = x.shape[-1]
    half = D // 2
    i = np.arange(half, dtype=np.float64)
    inv_freq = theta ** (-2.0 * i / D)
    phi = np.asarray(delta, dtype=np.float64)[..., None] * inv_freq
    c, s = np.cos(phi), np.sin(phi)
    y = np.empty_like(x)
    if interleaved:
        a, b = x[..., 0::2], x[..., 1::2]
        y[..., 0::2] = a * c - b * s
        y[..., 1::2] = a * s + b * c
    else:
        a, b = x[..., :half], x[..., half:]
        y[..., :half] = a * c - b * s
        y[..., half:] = a * s + b * c
    return y
