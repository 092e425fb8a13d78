"""Token ranking by K distance in float64 (oracle side).

Sec. 4.2 (the experiment behind the first-k rule): two KV caches of the same image are
computed at different positions; the K distance of a token is the L1 distance between its
two K tensors; per layer the tokens are sorted by that distance and the figure counts, for
every token, the layers in which it is among the 50 most distant ones.
"""
import numpy as np


def k_distance(k_a, k_b):
    """k_a, k_b [L][Hkv][D]: two stored key caches of one chunk.  Returns [L] float64:
    sum over heads and coordinates of |k_a - k_b| for every token."""
    a = np.asarray(k_a, dtype=np.float64)
    b = np.asarray(k_b, dtype=np.float64)
    return np.abs(a - b).sum(axis=(1, 2))


def top_tokens(dist, n_top):
    """Indices of the n_top tokens of largest distance, in ascending index order; of two
    tokens with the same distance the one with the lower index ranks higher."""
    dist = np.asarray(dist, dtype=np.float64)
    order = sorted(range(len(dist)), key=lambda t: (-dist[t], t))
    return np.asarray(sorted(order[:max(0, min(n_top, len(dist)))]), dtype=np.int32)


def top_counts(dist_per_layer, n_top):
    """dist_per_layer [layers][L].  For every token the number of layers in which it is among
    the n_top most distant tokens (the quantity plotted in the figure of Sec. 4.2)."""
    dist_per_layer = np.asarray(dist_per_layer, dtype=np.float64)
    counts = np.zeros(dist_per_layer.shape[1], dtype=np.int32)
    for layer in dist_per_layer:
        counts[top_tokens(layer, n_top)] += 1
    return counts
