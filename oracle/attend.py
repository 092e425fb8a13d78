"""Selective attention in float64 (oracle side).

App. A: a_ij = exp(q_i.k_j / sqrt(d)) / sum_{t<=i} exp(q_i.k_t / sqrt(d)),
o_i = sum_{j<=i} a_ij v_j.  Sec. 4.1 / Fig. 7 step 3: only the selected tokens are
queries and each of them is multiplied with the whole linked K cache; "j <= i" is
taken by position inside the linked context, the token itself included.
Query head h reads key/value head h // (Hq/Hkv).
"""
import numpy as np


def attend(q, k_ctx, v_ctx, plan, scale, rows=None):
    """q [Nq][Hq][D]; k_ctx, v_ctx [N][Hkv][D] in logical order (see link.link_kv).
    Returns O [Nq][Hq][D] and LSE [Nq][Hq] (natural log of the softmax denominator),
    float64.  `rows` limits the computation to some fresh rows (others stay NaN)."""
    q = np.asarray(q, dtype=np.float64)
    k_ctx = np.asarray(k_ctx, dtype=np.float64)
    v_ctx = np.asarray(v_ctx, dtype=np.float64)
    nq, hq, d = q.shape
    group = hq // k_ctx.shape[1]
    out = np.full((nq, hq, d), np.nan)
    lse = np.full((nq, hq), np.nan)
    todo = np.arange(nq) if rows is None else np.asarray(rows, dtype=np.int64)
    req = np.asarray(plan["q_req"])[todo]
    for b in np.unique(req):
        sel = todo[req == b]                       # fresh rows of request b
        base = int(plan["ctx_off"][b])
        pos = np.asarray(plan["q_pos"], dtype=np.int64)[sel]
        n_keys = int(pos.max()) + 1
        hidden = np.arange(n_keys)[None, :] > pos[:, None]   # key j is seen iff j <= position
        for h in range(hq):
            g = h // group
            s = scale * (q[sel, h, :] @ k_ctx[base:base + n_keys, g, :].T)
            s[hidden] = -np.inf
            m = s.max(axis=1, keepdims=True)
            w = np.exp(s - m)
            z = w.sum(axis=1, keepdims=True)
            out[sel, h, :] = (w @ v_ctx[base:base + n_keys, g, :]) / z
            lse[sel, h] = (m + np.log(z))[:, 0]
    return out, lse


def attend_unshifted(q, k_ctx, v_ctx, shift, plan, theta, scale, interleaved=False, rows=None):
    """Selective attention over a context whose stored keys were linked without their position
    shift (link.link_kv_unshifted).  The rotation is orthogonal, so the logit of query q and a
    key that still lacks the shift D is <q, Rot(D) k> = <Rot(-D) q, k>: the query is turned
    back by the shift of the key's chunk instead of the key being turned forward.  Same
    softmax and same sums as attend (App. A); written key by key."""
    from .rope import rotate
    q = np.asarray(q, dtype=np.float64)
    k_ctx = np.asarray(k_ctx, dtype=np.float64)
    v_ctx = np.asarray(v_ctx, dtype=np.float64)
    nq, hq, d = q.shape
    group = hq // k_ctx.shape[1]
    out = np.full((nq, hq, d), np.nan)
    lse = np.full((nq, hq), np.nan)
    todo = np.arange(nq) if rows is None else np.asarray(rows, dtype=np.int64)
    for r in todo:
        b = int(plan["q_req"][r])
        base = int(plan["ctx_off"][b])
        n_keys = int(plan["q_pos"][r]) + 1
        sh = np.asarray(shift[base:base + n_keys])
        s = np.empty((hq, n_keys))
        for dlt in np.unique(sh):                      # one turned-back query per distinct shift
            qt = rotate(q[r], -float(dlt), theta, interleaved)      # [Hq][D]
            at = np.nonzero(sh == dlt)[0]
            for h in range(hq):
                s[h, at] = scale * (k_ctx[base + at, h // group, :] @ qt[h])
        for h in range(hq):
            m = s[h].max()
            w = np.exp(s[h] - m)
            z = w.sum()
            out[r, h] = (w @ v_ctx[base:base + n_keys, h // group, :]) / z
            lse[r, h] = m + np.log(z)
    return out, lse


def attend_loops(q, k_ctx, v_ctx, plan, scale):
    """The same definition with every sum written as a Python loop (tiny inputs)."""
    import math
    nq, hq, d = len(q), len(q[0]), len(q[0][0])
    group = hq // len(k_ctx[0])
    out = [[[0.0] * d for _ in range(hq)] for _ in range(nq)]
    for r in range(nq):
        base = int(plan["ctx_off"][int(plan["q_req"][r])])
        i = int(plan["q_pos"][r])
        for h in range(hq):
            g = h // group
            e = []
            for j in range(i + 1):
                dot = 0.0
                for c in range(d):
                    dot += float(q[r][h][c]) * float(k_ctx[base + j][g][c])
                e.append(math.exp(dot * scale))
            den = 0.0
            for t in range(i + 1):
                den += e[t]
            for j in range(i + 1):
                a = e[j] / den
                for c in range(d):
                    out[r][h][c] += a * float(v_ctx[base + j][g][c])
    return np.asarray(out, dtype=np.float64)
