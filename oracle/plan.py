"""Integer plan of a batch of requests (oracle side, plain Python loops).

Selection rule (Sec. 4.2, last paragraph): the recompute set holds every text
token and the first k tokens of every image chunk.  Text tokens are always in the
set because their cache is only a placeholder (Sec. 4.1, the "dummy cache").
A chunk may instead name the tokens to recompute one by one (any selection policy,
e.g. the tokens of largest deviation that Sec. 5.1 attributes to CacheBlend-r, or
the ranking by K distance of Sec. 4.2); the rest of the plan does not care how the
set was chosen.
Linking (Sec. 3.1 item 5; Fig. 7 step 2): every context position has exactly one
source, either a stored chunk row or a freshly computed row that replaces it.
"""
import numpy as np


def build_plan(requests, default_k, page_size=0, page_tables=None):
    """requests: list (batch) of segment lists; a segment is ("text", L) or
    ("chunk", src_id, L, k) with k None -> default_k; k may also be a sequence of
    chunk-local token indices (0 <= index < L), the explicit recompute set of the chunk.

    Returns a dict of int32 arrays.  Positions are request-local ("global" in the
    paper's sense: offset inside the linked context); rows of the fresh tensors and
    context positions of the batch are numbered request after request.
      ctx_off[B+1], q_off[B+1]   prefix sums of context length / recompute-set size
      q_pos[Nq]                  position id of each fresh row
      q_req[Nq]                  request of each fresh row
      src_inst[N]                chunk instance feeding the position, -1 = fresh row
      src_row[N]                 row inside that chunk, or fresh-row index
      dst_slot[N]                physical slot of the position in the context buffer
      slot_map[Nq]               physical slot of each fresh row
      inst_src/inst_delta/inst_len/inst_k/inst_req[n_inst]
                                 per chunk instance: caller's source id, position
                                 shift (= offset of its first token), length,
                                 effective k (explicit set: length of its leading
                                 run 0, 1, 2, ...), owning request
      runs[n_runs][4]            (request, first fresh row, length, first position)
                                 maximal runs of consecutive positions in the set
    """
    ctx_off, q_off = [0], [0]
    q_pos, q_req, src_inst, src_row, dst_slot, slot_map = [], [], [], [], [], []
    inst_src, inst_delta, inst_len, inst_k, inst_req = [], [], [], [], []
    runs = []
    for b, segs in enumerate(requests):
        # 1. offsets and the recompute set, as a set of positions
        off = 0
        selected = set()
        owner = {}            # position -> (instance, local row) for chunk tokens
        for seg in segs:
            if seg[0] == "text":
                L = seg[1]
                for t in range(L):
                    selected.add(off + t)
            elif seg[0] == "chunk":
                _, src, L, k = seg
                if k is None or isinstance(k, (int, np.integer)):
                    k = default_k if k is None or k < 0 else k
                    chosen = set(range(min(k, L)))
                else:
                    chosen = set(int(t) for t in k)
                    if any(t < 0 or t >= L for t in chosen):
                        raise ValueError("selected token outside its chunk")
                k_eff = 0
                while k_eff in chosen:
                    k_eff += 1
                inst = len(inst_src)
                inst_src.append(src); inst_delta.append(off); inst_len.append(L)
                inst_k.append(k_eff); inst_req.append(b)
                for t in range(L):
                    owner[off + t] = (inst, t)
                    if t in chosen:
                        selected.add(off + t)
            else:
                raise ValueError(seg[0])
            off += L
        n_ctx = off
        order = sorted(selected)
        row_of = {p: q_off[-1] + i for i, p in enumerate(order)}
        # 2. per-position source and destination
        for p in range(n_ctx):
            if page_size:
                slot = int(page_tables[b][p // page_size]) * page_size + p % page_size
            else:
                slot = ctx_off[-1] + p
            dst_slot.append(slot)
            if p in row_of:
                src_inst.append(-1); src_row.append(row_of[p])
            else:
                src_inst.append(owner[p][0]); src_row.append(owner[p][1])
        # 3. fresh rows and their runs
        for i, p in enumerate(order):
            r = q_off[-1] + i
            q_pos.append(p); q_req.append(b); slot_map.append(dst_slot[ctx_off[-1] + p])
            if i > 0 and order[i - 1] == p - 1:
                runs[-1][2] += 1
            else:
                runs.append([b, r, 1, p])
        ctx_off.append(ctx_off[-1] + n_ctx)
        q_off.append(q_off[-1] + len(order))
    i32 = lambda a, shape=None: np.asarray(a, dtype=np.int32).reshape(shape if shape else (-1,))
    return dict(ctx_off=i32(ctx_off), q_off=i32(q_off), q_pos=i32(q_pos), q_req=i32(q_req),
                src_inst=i32(src_inst), src_row=i32(src_row), dst_slot=i32(dst_slot),
                slot_map=i32(slot_map), inst_src=i32(inst_src), inst_delta=i32(inst_delta),
                inst_len=i32(inst_len), inst_k=i32(inst_k), inst_req=i32(inst_req),
                runs=i32(runs, (-1, 4)))
