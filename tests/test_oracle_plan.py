"""Pins of oracle.plan.build_plan (CPU only).

The selection rule is Sec. 4.2 (all text tokens + first k tokens of each chunk);
"replace" semantics of linking is Fig. 7 step 2.  The pins are a hand-derived
layout, closed-form counts and an independent set-based construction.
"""
import os

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import workloads
from oracle import build_plan

GOLD = os.path.join(os.path.dirname(__file__), "golden", "config_sizes.txt")


def test_tiny_config_by_hand():
    reqs, _, _ = workloads.layout(1)
    p = build_plan(reqs, 8)
    # T16 A64 T8 B64 T8: text [0,16) [80,88) [152,160), chunk heads [16,24) [88,96)
    want = list(range(0, 24)) + list(range(80, 96)) + list(range(152, 160))
    assert p["q_pos"].tolist() == want
    assert p["inst_delta"].tolist() == [16, 88]
    assert p["inst_k"].tolist() == [8, 8]
    assert p["runs"].tolist() == [[0, 0, 24, 0], [0, 24, 16, 80], [0, 40, 8, 152]]
    assert p["ctx_off"].tolist() == [0, 160] and p["q_off"].tolist() == [0, 48]
    # position 24 is row 8 of chunk instance 0, position 96 is row 8 of instance 1
    assert (p["src_inst"][24], p["src_row"][24]) == (0, 8)
    assert (p["src_inst"][96], p["src_row"][96]) == (1, 8)
    assert (p["src_inst"][79], p["src_row"][79]) == (0, 63)
    assert (p["src_inst"][80], p["src_row"][80]) == (-1, 24)
    assert p["dst_slot"].tolist() == list(range(160))


def _golden_rows():
    rows = []
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        rows.append(tuple(int(x) for x in line.split()))
    return rows


@pytest.mark.parametrize("cfg,k,n,nq,sum_p1", _golden_rows())
def test_closed_form_counts(cfg, k, n, nq, sum_p1):
    reqs, _, _ = workloads.layout(cfg, batch=1)
    p = build_plan(reqs, k)
    assert int(p["ctx_off"][-1]) == n
    assert len(p["q_pos"]) == nq
    assert int((p["q_pos"].astype(np.int64) + 1).sum()) == sum_p1


@st.composite
def _chunk(draw):
    L = draw(st.integers(1, 12))
    k = draw(st.one_of(st.none(), st.integers(0, 14),
                       st.lists(st.integers(0, L - 1), max_size=L).map(tuple)))   # explicit token set
    return ("chunk", draw(st.integers(0, 3)), L, k)


segment = st.one_of(st.tuples(st.just("text"), st.integers(0, 9)), _chunk())


def _chosen(seg, default_k):
    """Chunk-local tokens a chunk segment asks to recompute, from its k or its explicit set."""
    k = seg[3]
    if k is None or isinstance(k, int):
        return set(range(min(default_k if k is None else k, seg[2])))
    return set(k)


def _check_invariants(reqs, default_k, p, page_size=0, tables=None):
    B = len(reqs)
    # chunk instances are numbered in prompt order over the batch; their shift is the offset of
    # their first token and their effective k the length of the leading run 0, 1, 2, ... of their set
    inst = 0
    for b in range(B):
        off = 0
        for s in reqs[b]:
            if s[0] == "chunk":
                pick = _chosen(s, default_k)
                lead = next(t for t in range(s[2] + 1) if t not in pick)
                assert (p["inst_src"][inst], p["inst_delta"][inst], p["inst_len"][inst], p["inst_k"][inst],
                        p["inst_req"][inst]) == (s[1], off, s[2], lead, b)
                inst += 1
            off += s[1] if s[0] == "text" else s[2]
    assert inst == len(p["inst_src"])
    for b in range(B):
        segs = reqs[b]
        # independent construction: label every position, then filter
        label = []
        for s in segs:
            if s[0] == "text":
                label += [("t", None)] * s[1]
            else:
                pick = _chosen(s, default_k)
                label += [("c", t in pick) for t in range(s[2])]
        c0, c1 = int(p["ctx_off"][b]), int(p["ctx_off"][b + 1])
        q0, q1 = int(p["q_off"][b]), int(p["q_off"][b + 1])
        assert c1 - c0 == len(label)
        want = [i for i, (kind, first) in enumerate(label) if kind == "t" or first]
        assert p["q_pos"][q0:q1].tolist() == want
        n_text = sum(s[1] for s in segs if s[0] == "text")
        n_head = sum(len(_chosen(s, default_k)) for s in segs if s[0] == "chunk")
        assert q1 - q0 == n_text + n_head
        # every position has one source; fresh rows and positions are mutual inverses
        for i, r in enumerate(range(q0, q1)):
            g = c0 + int(p["q_pos"][r])
            assert p["src_inst"][g] == -1 and p["src_row"][g] == r
            assert p["slot_map"][r] == p["dst_slot"][g]
            assert p["q_req"][r] == b
        fresh = [g for g in range(c0, c1) if p["src_inst"][g] < 0]
        assert len(fresh) == q1 - q0
        for g in range(c0, c1):
            inst = int(p["src_inst"][g])
            if inst >= 0:
                assert p["inst_req"][inst] == b
                t = int(p["src_row"][g])
                assert 0 <= t < p["inst_len"][inst] and t >= p["inst_k"][inst]
                assert g - c0 == p["inst_delta"][inst] + t
    # runs partition the fresh rows into maximal runs of consecutive positions
    covered = 0
    for (b, r0, ln, p0) in p["runs"].tolist():
        assert r0 == covered and ln > 0
        assert p["q_pos"][r0:r0 + ln].tolist() == list(range(p0, p0 + ln))
        assert all(x == b for x in p["q_req"][r0:r0 + ln])
        if r0 > int(p["q_off"][b]):
            assert p["q_pos"][r0 - 1] != p0 - 1
        covered += ln
    assert covered == len(p["q_pos"])
    # physical slots are unique
    assert len(set(p["dst_slot"].tolist())) == len(p["dst_slot"])
    if page_size:
        for b in range(B):
            c0, c1 = int(p["ctx_off"][b]), int(p["ctx_off"][b + 1])
            for pos in range(c1 - c0):
                assert p["dst_slot"][c0 + pos] == tables[b][pos // page_size] * page_size + pos % page_size


@settings(max_examples=150, deadline=None)
@given(st.lists(st.lists(segment, min_size=0, max_size=6), min_size=1, max_size=3),
       st.integers(0, 6))
def test_random_layouts(reqs, default_k):
    p = build_plan(reqs, default_k)
    _check_invariants(reqs, default_k, p)


@settings(max_examples=60, deadline=None)
@given(st.lists(st.lists(segment, min_size=1, max_size=5), min_size=1, max_size=3),
       st.integers(0, 5), st.sampled_from([1, 4, 16]), st.randoms(use_true_random=False))
def test_random_layouts_paged(reqs, default_k, ps, rnd):
    lens = [workloads.request_len(s) for s in reqs]
    need = [(n + ps - 1) // ps for n in lens]
    pool = list(range(sum(need) + 3))
    rnd.shuffle(pool)
    tables, at = [], 0
    for n in need:
        tables.append(pool[at:at + n]); at += n
    p = build_plan(reqs, default_k, page_size=ps, page_tables=tables)
    _check_invariants(reqs, default_k, p, ps, tables)


def test_explicit_token_sets_by_hand():
    """A chunk that names its recompute tokens one by one: T2 C6{1,4,5} T1 C4{0,1,3}.
    Positions: text 0,1; chunk tokens 2..7 of which 3,6,7; text 8; chunk 9..12 of which 9,10,12."""
    reqs = [[("text", 2), ("chunk", 0, 6, (4, 1, 5, 1)), ("text", 1), ("chunk", 1, 4, [0, 1, 3])]]
    p = build_plan(reqs, 99)
    assert p["q_pos"].tolist() == [0, 1, 3, 6, 7, 8, 9, 10, 12]
    assert p["runs"].tolist() == [[0, 0, 2, 0], [0, 2, 1, 3], [0, 3, 5, 6], [0, 8, 1, 12]]
    assert p["inst_k"].tolist() == [0, 2]               # leading runs of the two sets
    assert p["src_inst"].tolist() == [-1, -1, 0, -1, 0, 0, -1, -1, -1, -1, -1, 1, -1]
    assert p["src_row"].tolist() == [0, 1, 0, 2, 2, 3, 3, 4, 5, 6, 7, 2, 8]
    # an explicit prefix set is the first-k rule
    a = build_plan([[("text", 3), ("chunk", 0, 9, (0, 1, 2, 3))]], 0)
    b = build_plan([[("text", 3), ("chunk", 0, 9, 4)]], 0)
    assert all(np.array_equal(a[f], b[f]) for f in a)
    with pytest.raises(ValueError):
        build_plan([[("chunk", 0, 4, (4,))]], 0)


def test_missing_chunk_equals_text():
    """A chunk whose cache cannot be loaded is recomputed in full (Sec. 3.2, fallback):
    with k >= L it selects exactly what a text segment of the same length selects."""
    a = [[("text", 5), ("chunk", 0, 7, 7), ("text", 2), ("chunk", 1, 6, None)]]
    b = [[("text", 5), ("text", 7), ("text", 2), ("chunk", 1, 6, None)]]
    pa, pb = build_plan(a, 2), build_plan(b, 2)
    assert pa["q_pos"].tolist() == pb["q_pos"].tolist()
    assert pa["runs"].tolist() == pb["runs"].tolist()
    big = build_plan([[("text", 5), ("chunk", 0, 7, 100), ("text", 2), ("chunk", 1, 6, None)]], 2)
    assert big["q_pos"].tolist() == pa["q_pos"].tolist()
    # the effective k of a chunk is clipped to its length: min(k, L) tokens are recomputed
    assert pa["inst_k"].tolist() == [7, 2] and big["inst_k"].tolist() == [7, 2]


def test_k_zero_and_no_text_gives_empty_set():
    p = build_plan([[("chunk", 0, 4, None), ("chunk", 1, 3, None)]], 0)
    assert len(p["q_pos"]) == 0 and p["runs"].shape == (0, 4)
    assert p["src_inst"].tolist() == [0, 0, 0, 0, 1, 1, 1]
