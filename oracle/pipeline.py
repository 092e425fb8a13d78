"""Prefill of every layer of a batch from the library of stored caches (oracle side).

Sec. 3.2 and Fig. 6: at the start of a request the caches of its n images are looked
up; m of them are missing (expired, or their load fails) and are computed like text
while the other n - m are fetched, and the two proceed side by side.  What that
computes does not depend on the overlap, so the oracle is sequential: look up, treat a
missing image as a span in which every token is recomputed, then link and attend
layer after layer (Sec. 4.1, Fig. 7) with the layer's slice of every stored cache.
"""
import numpy as np

from .attend import attend
from .link import link_kv, position_fresh
from .plan import build_plan
from .store import MISSING


def plan_with_lookup(requests, ids, default_k, store, page_size=0, page_tables=None, failed=()):
    """requests as in plan.build_plan; ids[s] = library id of chunk source s.  A chunk whose
    cache is missing, or whose id is in `failed` (a load that went wrong), is planned with
    k = its length: all of its tokens join the recompute set (Sec. 3.2, the fall-back to
    inference without the stored cache)."""
    place, _ = store.lookup(ids)
    out = []
    for segs in requests:
        row = []
        for seg in segs:
            if seg[0] == "chunk" and (place[seg[1]] == MISSING or ids[seg[1]] in failed):
                seg = ("chunk", seg[1], seg[2], seg[2])
            row.append(seg)
        out.append(row)
    return build_plan(out, default_k, page_size, page_tables), out


def prefill_layers(plan, ids, store, n_layers, fresh, theta, scale, interleaved=False, fresh_pre_rope=False,
                   rows=None, layers=None):
    """fresh(layer) -> (q, k, v) float64 arrays [Nq][H][D] for the plan's recompute set.
    Returns per layer (K, V, O, LSE) in logical order, float64; `rows` limits the attention
    to some fresh rows, `layers` the work to some layers (the others give None)."""
    result = []
    used = sorted(set(int(s) for i, s in enumerate(plan["inst_src"])
                      if int(plan["inst_k"][i]) < int(plan["inst_len"][i])))
    for layer in range(n_layers):
        if layers is not None and layer not in layers:
            result.append(None)
            continue
        ck, cv = {}, {}
        for s in used:
            k_l, v_l = store.layer(ids[s], layer)
            ck[s] = np.asarray(k_l, dtype=np.float64)
            cv[s] = np.asarray(v_l, dtype=np.float64)
        # fully recomputed chunks never read their source: any row count will do
        for s in set(int(x) for x in plan["inst_src"]) - set(used):
            ck[s] = cv[s] = None
        q, fk, fv = fresh(layer)
        K, V = link_kv(plan, ck, cv, fk, fv, theta, interleaved, fresh_pre_rope)
        if fresh_pre_rope:
            q = position_fresh(q, plan, theta, interleaved)
        O, lse = attend(q, K, V, plan, scale, rows=rows)
        result.append((K, V, O, lse))
    return result
