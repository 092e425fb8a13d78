"""Decode-step attention over a linked context in float64 (oracle side).

App. A, autoregressive generation: after the prefill the model produces one token at
a time; the key and value of the new token are appended to the KV cache and its query
attends to every cached position and to itself (the attention definition of App. A,
a_ij over t <= i, with i the new position).  Here the cache is the linked context of
one request (Fig. 7 step 2) and the new token sits at position N, right after it.
Query head h reads key/value head h // (Hq/Hkv).
"""
import numpy as np


def decode_attend(q, k_ctx, v_ctx, plan, scale, new_k=None, new_v=None):
    """q [B][Hq][D]: query of the next token of every request; k_ctx, v_ctx [N][Hkv][D]
    in logical order (see link.link_kv); new_k, new_v [B][Hkv][D]: key and value of
    that token itself, or None to attend to the linked context only.
    Returns O [B][Hq][D] and LSE [B][Hq] (natural log of the softmax denominator),
    float64.  A request with no key at all gets O = 0 and LSE = -inf."""
    q = np.asarray(q, dtype=np.float64)
    k_ctx = np.asarray(k_ctx, dtype=np.float64)
    v_ctx = np.asarray(v_ctx, dtype=np.float64)
    n_req, hq, d = q.shape
    group = hq // k_ctx.shape[1]
    out = np.zeros((n_req, hq, d))
    lse = np.full((n_req, hq), -np.inf)
    for b in range(n_req):
        lo, hi = int(plan["ctx_off"][b]), int(plan["ctx_off"][b + 1])
        for h in range(hq):
            g = h // group
            keys, vals = k_ctx[lo:hi, g, :], v_ctx[lo:hi, g, :]
            if new_k is not None:
                keys = np.concatenate([keys, np.asarray(new_k, dtype=np.float64)[b, g][None, :]])
                vals = np.concatenate([vals, np.asarray(new_v, dtype=np.float64)[b, g][None, :]])
            if len(keys) == 0:
                continue
            s = scale * (keys @ q[b, h])
            m = s.max()
            w = np.exp(s - m)
            z = w.sum()
            out[b, h] = (w @ vals) / z
            lse[b, h] = m + np.log(z)
    return out, lse
