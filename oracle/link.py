"""Linking of stored chunk caches and fresh rows into one context (oracle side).

Fig. 7 step 2 and Sec. 4.1: the K (and V) rows of the selected tokens are replaced
by the freshly generated ones; every other row comes from the stored cache of its
image.  Stored keys are moved from chunk-local to global positions with
rope.rotate; values carry no position and are copied.

Fresh rows may be handed over straight from the projections, before any positional
embedding (the step Fig. 7 leaves out): position_fresh then turns every fresh row by
the position id of its token inside the request, the same rotation full prefill would
apply.  Queries and keys take it; values never do.
"""
import numpy as np
from .rope import rotate


def position_fresh(x, plan, theta, interleaved=False):
    """x [Nq][H][D], one row per token of the recompute set, not yet rotated.  Returns the
    rows rotated to their position ids plan["q_pos"] (float64)."""
    x = np.asarray(x, dtype=np.float64)
    pos = np.asarray(plan["q_pos"], dtype=np.float64)
    return rotate(x, pos[:, None], theta, interleaved)


def link_kv(plan, chunk_k, chunk_v, fresh_k, fresh_v, theta, interleaved=False, fresh_pre_rope=False):
    """chunk_k / chunk_v: mapping source id -> float64 array [L][Hkv][D];
    fresh_k / fresh_v: float64 [Nq][Hkv][D].  Returns (K, V) in logical order
    [N][Hkv][D] (requests one after the other), float64.  With fresh_pre_rope the
    fresh keys are rotated to their positions first (see position_fresh)."""
    n = int(plan["ctx_off"][-1])
    fresh_k = np.asarray(fresh_k, dtype=np.float64)
    if fresh_pre_rope:
        fresh_k = position_fresh(fresh_k, plan, theta, interleaved)
    fresh_v = np.asarray(fresh_v, dtype=np.float64)
    K = np.empty((n,) + fresh_k.shape[1:], dtype=np.float64)
    V = np.empty_like(K)
    for g in range(n):
        inst, row = int(plan["src_inst"][g]), int(plan["src_row"][g])
        if inst < 0:
            K[g] = fresh_k[row]
            V[g] = fresh_v[row]
        else:
            src = int(plan["inst_src"][inst])
            shift = float(plan["inst_delta"][inst])
            K[g] = rotate(np.asarray(chunk_k[src][row], dtype=np.float64), shift, theta, interleaved)
            V[g] = np.asarray(chunk_v[src][row], dtype=np.float64)
    return K, V


def link_kv_unshifted(plan, chunk_k, chunk_v, fresh_k, fresh_v, theta, interleaved=False, fresh_pre_rope=False):
    """The linked context with the stored keys left as they are stored (Sec. 4.1: the linker
    only joins caches; Fig. 7 step 2 replaces rows and touches nothing else).  Returns
    (K, V, shift): K and V as link_kv but stored keys unrotated, and shift [N] = the position
    shift each key still lacks (its chunk's offset; 0 for fresh rows, which carry their
    global position).  attend.attend_unshifted consumes the triple."""
    n = int(plan["ctx_off"][-1])
    fresh_k = np.asarray(fresh_k, dtype=np.float64)
    if fresh_pre_rope:
        fresh_k = position_fresh(fresh_k, plan, theta, interleaved)
    fresh_v = np.asarray(fresh_v, dtype=np.float64)
    K = np.empty((n,) + fresh_k.shape[1:], dtype=np.float64)
    V = np.empty_like(K)
    shift = np.zeros(n, dtype=np.int64)
    for pos in range(n):
        i, r = int(plan["src_inst"][pos]), int(plan["src_row"][pos])
        if i < 0:
            K[pos], V[pos] = fresh_k[r], fresh_v[r]
        else:
            cache = int(plan["inst_src"][i])
            K[pos], V[pos] = chunk_k[cache][r], chunk_v[cache][r]
            shift[pos] = int(plan["inst_delta"][i])
    return K, V, shift


def to_slots(x_logical, dst_slot, n_slots, fill=np.nan):
    """Place logical rows at their physical slots (paged layout); unused slots = fill."""
    out = np.full((n_slots,) + x_logical.shape[1:], fill, dtype=x_logical.dtype)
    out[np.asarray(dst_slot, dtype=np.int64)] = x_logical
    return out
