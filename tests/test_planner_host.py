"""Host logic of libmpic without a GPU: the C++ planner against the oracle plan (bit
exact), the rotary tables against float64, argument checking, exported symbols."""
import ctypes
import os
import re

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import workloads
import paper_2502_01960_amd as mpic
from oracle import build_plan

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INT_FIELDS = [f for f in mpic.PLAN_FIELDS
              if f not in ("attn_tiles", "launch_estimate") and not f.startswith(("key_block", "lazy_tiles"))]


def _ctx(hq=4, hkv=2, d=128, dtype=mpic.MPIC_BF16, theta=1e4, page_size=0):
    return mpic.Context(hq, hkv, d, dtype, theta, 0, page_size)


def test_header_is_plain_c():
    """include/mpic.h compiles as C99 (no C++-isms) and the C program links against the library."""
    import subprocess, tempfile
    src = os.path.join(ROOT, "tests", "native", "header_is_c.c")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "header_is_c")
        cmd = ["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-Wno-pedantic", "-I", os.path.join(ROOT, "include"),
               src, "-o", exe, mpic.lib_path(), "-Wl,-rpath," + os.path.dirname(mpic.lib_path())]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
    # the header alone, strictly
    r = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c",
                        os.path.join(ROOT, "include", "mpic.h")], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    header = open(os.path.join(ROOT, "include", "mpic.h")).read()
    names = set(re.findall(r"\b(mpic_[a-z_]+)\s*\(", header))
    used = set(re.findall(r"\(void\*\)(mpic_[a-z_]+)", open(src).read()))
    assert names == used, names ^ used


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "mpic.h")).read()
    names = sorted(set(re.findall(r"\b(mpic_[a-z_]+)\s*\(", header)))
    assert {"mpic_assemble_kv", "mpic_selective_attn", "mpic_plan_create", "mpic_create"} <= set(names)
    lib = ctypes.CDLL(mpic.lib_path())
    for n in names:
        assert hasattr(lib, n), f"{n} declared in mpic.h but not exported"


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_plan_matches_oracle_on_benchmark_layouts(cfg):
    sh = workloads.shape(cfg)
    reqs, _, _ = workloads.layout(cfg)
    tables, pool = (None, 0)
    if sh.page_size:
        tables, pool = workloads.gen_page_tables(sh, [workloads.request_len(r) for r in reqs])
    ks = [0, 16, 64, 1024] if cfg == 4 else [sh.default_k]
    ctx = _ctx(sh.n_q_heads, sh.n_kv_heads, sh.head_dim,
               mpic.MPIC_F32 if sh.dtype == "f32" else mpic.MPIC_BF16, sh.rope_theta, sh.page_size)
    for k in ks:
        want = build_plan(reqs, k, sh.page_size, tables)
        got = mpic.Plan(ctx, reqs, k, tables, pool)
        for f in INT_FIELDS:
            assert np.array_equal(got.get(f), want[f]), (cfg, k, f)
        _check_tiles(got, want, sh.n_q_heads // sh.n_kv_heads, sh.n_kv_heads)


def _check_tiles(plan, want, group, n_kv):
    """Tiles cover every (fresh row, query head, visible key) exactly once: row ranges stay
    inside one request; a tile cut along the keys comes as pieces whose key ranges are
    64-aligned, contiguous from 0 to the key count of its last row, with distinct partial
    slots; an uncut tile writes the output itself."""
    tiles = plan.get("attn_tiles")
    nq = len(want["q_pos"])
    seen = np.zeros((nq, n_kv * group), dtype=np.int32)
    pieces = {}
    for (b, g, row0, n_rows, key_end, key0, part, _pad) in tiles.tolist():
        if n_rows == 0:
            continue
        assert 0 < n_rows <= 256
        pieces.setdefault((b, g, row0, n_rows), []).append((key0, key_end, part))
    slots = []
    for (b, g, row0, n_rows), parts in pieces.items():
        flat = np.arange(row0, row0 + n_rows)
        fresh = int(want["q_off"][b]) + flat // group
        assert fresh.max() < want["q_off"][b + 1]
        n_keys = int(want["q_pos"][fresh].max()) + 1
        parts.sort()
        assert parts[0][0] == 0 and parts[-1][1] == n_keys
        for (k0, k1, part), nxt in zip(parts, parts[1:] + [None]):
            assert k0 % 64 == 0 and k0 < k1
            if nxt is not None:
                assert k1 == nxt[0]
            assert (part == -1) == (len(parts) == 1)
            if part >= 0:
                slots.append(part)
        seen[fresh, g * group + flat % group] += 1
    assert (seen == 1).all()
    assert sorted(slots) == list(range(len(slots)))


@st.composite
def _chunk(draw):
    L = draw(st.integers(1, 70))
    k = draw(st.one_of(st.none(), st.integers(0, 80),
                       st.lists(st.integers(0, L - 1), max_size=L).map(tuple)))   # tokens named one by one
    return ("chunk", draw(st.integers(0, 5)), L, k)


segment = st.one_of(st.tuples(st.just("text"), st.integers(0, 40)), _chunk())


@settings(max_examples=120, deadline=None)
@given(st.lists(st.lists(segment, min_size=0, max_size=6), min_size=1, max_size=4),
       st.integers(0, 20), st.sampled_from([(4, 4), (8, 2), (7, 1), (28, 4)]))
def test_plan_matches_oracle_on_random_layouts(reqs, default_k, heads):
    ctx = _ctx(heads[0], heads[1])
    want = build_plan(reqs, default_k)
    got = mpic.Plan(ctx, reqs, default_k)
    for f in INT_FIELDS:
        assert np.array_equal(got.get(f), want[f]), f
    _check_tiles(got, want, heads[0] // heads[1], heads[1])


@settings(max_examples=60, deadline=None)
@given(st.lists(st.lists(segment, min_size=1, max_size=5), min_size=1, max_size=3),
       st.integers(0, 9), st.sampled_from([1, 16, 5]), st.randoms(use_true_random=False))
def test_paged_plan_matches_oracle(reqs, default_k, ps, rnd):
    need = [(workloads.request_len(r) + ps - 1) // ps for r in reqs]
    pool = list(range(sum(need) + 2))
    rnd.shuffle(pool)
    tables, at = [], 0
    for n in need:
        tables.append(np.asarray(pool[at:at + n], dtype=np.int32)); at += n
    ctx = _ctx(page_size=ps)
    want = build_plan(reqs, default_k, ps, tables)
    got = mpic.Plan(ctx, reqs, default_k, tables, len(pool))
    for f in INT_FIELDS:
        assert np.array_equal(got.get(f), want[f]), f


def _check_key_blocks(plan, want, group):
    """lazy_rope plans: for every block size the blocks list the keys of every request, each position
    exactly once: first the blocks of fresh rows, then the blocks of stored rows, each part in position
    order; a block never straddles a change of source (one chunk instance, or fresh rows) and its stored
    rows are consecutive rows of the cache; a piece of a tile that was cut along the keys owns whole
    blocks; the two block ranges of a tile hold exactly the blocks that start inside its key range."""
    ctx_off = want["ctx_off"]
    tiles = plan.get("attn_tiles")
    for bn in (32, 64, 96):
        blocks = plan.get(f"key_blocks_{bn}")
        parts = plan.get(f"key_block_parts_{bn}")
        assert len(parts) == len(ctx_off) - 1
        at_end = 0
        for b, (lo, mid, hi) in enumerate(parts.tolist()):
            assert lo == at_end and lo <= mid <= hi
            at_end = hi
            n = ctx_off[b + 1] - ctx_off[b]
            covered = np.zeros(n, dtype=np.int32)
            for part, (x, y) in (("fresh", (lo, mid)), ("stored", (mid, hi))):
                last = -1
                for (pos0, n_valid, inst, req) in blocks[x:y].tolist():
                    assert req == b and 1 <= n_valid <= bn
                    assert (inst < 0) == (part == "fresh")
                    assert pos0 > last, "each part lists its blocks in position order"
                    last = pos0
                    covered[pos0:pos0 + n_valid] += 1
                    src = want["src_inst"][ctx_off[b] + pos0: ctx_off[b] + pos0 + n_valid]
                    assert (src == inst).all(), "a block holds keys of one source only"
                    if inst >= 0:
                        rows = want["src_row"][ctx_off[b] + pos0: ctx_off[b] + pos0 + n_valid]
                        assert (np.diff(rows) == 1).all()
            assert (covered == 1).all(), "every position of the request in exactly one block"
        assert at_end == len(blocks)
        if bn == 32:
            continue
        ranges = plan.get(f"lazy_tiles_{bn}")
        assert len(ranges) == len(tiles)
        for t, (f0, f1, s0, s1) in zip(tiles.tolist(), ranges.tolist()):
            if t[3] == 0:
                continue
            b, key_end, key0 = t[0], t[4], t[5]
            lo, mid, hi = parts[b].tolist()
            mine = np.concatenate([blocks[lo + f0:lo + f1], blocks[mid + s0:mid + s1]])
            rest = np.concatenate([blocks[lo:lo + f0], blocks[lo + f1:mid], blocks[mid:mid + s0], blocks[mid + s1:hi]])
            assert len(mine) >= 1
            assert ((mine[:, 0] >= key0) & (mine[:, 0] < key_end)).all(), "the tile's blocks start inside its key range"
            assert not ((rest[:, 0] >= key0) & (rest[:, 0] < key_end)).any(), "no other block starts there"
            assert mine[:, 0].min() == key0, "a tile (or piece) starts at a block start"
            # no earlier block reaches into the range (a piece owns whole blocks)
            before = rest[rest[:, 0] < key0]
            assert (before[:, 0] + before[:, 1] <= key0).all()


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_key_blocks_of_lazy_plans_on_benchmark_layouts(cfg):
    sh = workloads.shape(cfg)
    reqs, _, _ = workloads.layout(cfg)
    tables, pool = (None, 0)
    if sh.page_size:
        tables, pool = workloads.gen_page_tables(sh, [workloads.request_len(r) for r in reqs])
    ctx = mpic.Context(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, mpic.MPIC_BF16, sh.rope_theta, 0, sh.page_size, 0, 1)
    for k in ([0, 16, 1024] if cfg == 4 else [sh.default_k]):
        want = build_plan(reqs, k, sh.page_size, tables)
        got = mpic.Plan(ctx, reqs, k, tables, pool)
        for f in INT_FIELDS:
            assert np.array_equal(got.get(f), want[f]), (cfg, k, f)
        _check_key_blocks(got, want, sh.n_q_heads // sh.n_kv_heads)
    # a context without lazy_rope has no such lists
    plain = mpic.Plan(_ctx(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, mpic.MPIC_BF16, sh.rope_theta, sh.page_size), reqs,
                      sh.default_k, tables, pool)
    assert len(plain.get("key_blocks_64")) == 0 and len(plain.get("lazy_tiles_96")) == 0


@settings(max_examples=80, deadline=None)
@given(st.lists(st.lists(segment, min_size=0, max_size=6), min_size=1, max_size=4),
       st.integers(0, 40), st.sampled_from([(4, 4), (8, 2), (28, 4), (7, 1)]))
def test_key_blocks_of_lazy_plans_on_random_layouts(reqs, default_k, heads):
    hq, hkv = heads
    ctx = mpic.Context(hq, hkv, 128, mpic.MPIC_BF16, 1e4, 0, 0, 0, 1)
    want = build_plan(reqs, default_k)
    got = mpic.Plan(ctx, reqs, default_k)
    _check_key_blocks(got, want, hq // hkv)


def test_rope_tables_are_float64_accurate():
    theta, d = 1e6, 128
    reqs = [[("text", 64), ("chunk", 0, 2304, None)] * 32 + [("text", 64)]]
    plan = mpic.Plan(_ctx(64, 8, d, theta=theta), reqs, 32)
    cos, sin = plan.rope()
    delta = plan.get("inst_delta").astype(np.float64)
    assert delta[-1] == 31 * 2368 + 64
    phi = delta[:, None] * theta ** (-2.0 * np.arange(d // 2) / d)
    assert cos.shape == (32 * 64,)
    np.testing.assert_allclose(cos.reshape(32, 64), np.cos(phi), rtol=0, atol=6e-8)
    np.testing.assert_allclose(sin.reshape(32, 64), np.sin(phi), rtol=0, atol=6e-8)


def test_fresh_row_rotary_tables_are_float64_accurate():
    """fresh_pre_rope contexts: one table row per distinct position id of the batch, every
    fresh row pointing at the row of its own position id; values against float64 cos / sin."""
    theta, d = 1e6, 128
    reqs = [[("text", 64), ("chunk", 0, 2304, None)] * 32 + [("text", 64)],
            [("chunk", 0, 2304, 7), ("text", 300)]]
    ctx = mpic.Context(64, 8, d, mpic.MPIC_BF16, theta, 0, 0, 1)
    plan = mpic.Plan(ctx, reqs, 32)
    row, cos, sin = plan.fresh_rope()
    q_pos = plan.get("q_pos")
    assert len(row) == len(q_pos) and cos.shape == sin.shape == (len(np.unique(q_pos)), d // 2)
    assert row.min() == 0 and row.max() == len(cos) - 1
    phi = q_pos.astype(np.float64)[:, None] * theta ** (-2.0 * np.arange(d // 2) / d)
    assert q_pos.max() == 75839
    np.testing.assert_allclose(cos[row], np.cos(phi), rtol=0, atol=6e-8)
    np.testing.assert_allclose(sin[row], np.sin(phi), rtol=0, atol=6e-8)
    # almost always the correctly rounded float (the two evaluations differ by ~1e-11)
    assert (cos[row] != np.cos(phi).astype(np.float32)).mean() < 1e-3
    # a context without the flag carries no such table
    r0, c0, s0 = mpic.Plan(_ctx(64, 8, d, theta=theta), reqs, 32).fresh_rope()
    assert len(r0) == 0 and len(c0) == 0
    with pytest.raises(mpic.MpicError):
        mpic.Context(4, 4, 64, mpic.MPIC_F32, 1e4, 0, 0, 2)


def test_listed_recompute_sets():
    reqs = [[("text", 2), ("chunk", 0, 6, (4, 1, 5, 1)), ("text", 1), ("chunk", 1, 4, [0, 1, 3])],
            [("chunk", 1, 4, ()), ("chunk", 0, 6, None)]]
    want = build_plan(reqs, 3)
    got = mpic.Plan(_ctx(), reqs, 3)
    for f in INT_FIELDS:
        assert np.array_equal(got.get(f), want[f]), f
    assert got.get("q_pos").tolist() == [0, 1, 3, 6, 7, 8, 9, 10, 12, 4, 5, 6]
    with pytest.raises(mpic.MpicError):
        mpic.Plan(_ctx(), [[("chunk", 0, 4, (4,))]], 0)          # token outside its chunk
    with pytest.raises(mpic.MpicError):
        mpic.Plan(_ctx(), [[("chunk", 0, 4, mpic.MPIC_K_LISTED)]], 0)   # listed, but no list given


def test_token_ranking_matches_oracle():
    from oracle import top_tokens
    rng = np.random.default_rng(9)
    for n in (1, 7, 50, 2304):
        dist = rng.integers(0, 12, size=n).astype(np.float32)        # many ties
        for n_top in (0, 1, 5, 50, n, n + 3):
            assert mpic.mpic_rank_tokens(dist, n_top).tolist() == top_tokens(dist, n_top).tolist()
    dist = rng.standard_normal(500).astype(np.float32)
    assert mpic.mpic_rank_tokens(dist, 50).tolist() == top_tokens(dist, 50).tolist()
    dist[[3, 77]] = np.nan                                            # never among the chosen unless forced
    got = mpic.mpic_rank_tokens(dist, 498).tolist()
    assert 3 not in got and 77 not in got and len(got) == 498
    assert mpic.mpic_rank_tokens(np.zeros(0, np.float32), 5).tolist() == []


def test_rejected_arguments():
    with pytest.raises(mpic.MpicError):
        _ctx(hq=6, hkv=4)                      # heads do not group
    with pytest.raises(mpic.MpicError):
        _ctx(d=96)                             # unsupported head_dim
    with pytest.raises(mpic.MpicError):
        mpic.Context(4, 4, 128, mpic.MPIC_BF16, -1.0)
    ctx = _ctx()
    with pytest.raises(mpic.MpicError):
        mpic.Plan(ctx, [[("text", -1)]], 4)
    with pytest.raises(mpic.MpicError):
        mpic.Plan(ctx, [[("chunk", -2, 4, None)]], 4)
    with pytest.raises(mpic.MpicError):
        mpic.Plan(ctx, [[("text", 3)]], -1)
    paged = _ctx(page_size=16)
    with pytest.raises(mpic.MpicError):
        mpic.Plan(paged, [[("text", 40)]], 0, [np.array([0, 1], np.int32)], 8)       # table too short
    with pytest.raises(mpic.MpicError):
        mpic.Plan(paged, [[("text", 40)]], 0, [np.array([0, 1, 1], np.int32)], 8)    # page used twice
    with pytest.raises(mpic.MpicError):
        mpic.Plan(paged, [[("text", 40)]], 0, [np.array([0, 1, 9], np.int32)], 8)    # id out of range
    with pytest.raises(mpic.MpicError):
        mpic.Plan(paged, [[("text", 20)], [("text", 20)]], 0,
                  [np.array([0, 1], np.int32), np.array([1, 2], np.int32)], 8)        # shared between requests
    assert "page" in mpic.mpic_last_error(paged.handle)
    assert mpic.mpic_strerror(-2) == "unsupported configuration"


def test_empty_recompute_set_and_empty_request():
    ctx = _ctx()
    p = mpic.Plan(ctx, [[("chunk", 0, 5, None)], []], 0)
    assert len(p.get("q_pos")) == 0 and p.get("attn_tiles").shape == (0, 8)
    assert p.get("ctx_off").tolist() == [0, 5, 5]


def test_launch_estimate_is_the_list_scheduling_of_the_tile_order():
    """MPIC_PLAN_LAUNCH_ESTIMATE against a replay of the launch order in Python: workgroup i goes to
    L2 domain i % 8, each domain hands its tiles in order to the first free of its 32 compute units."""
    import heapq
    want_fits = {2: 1, 3: 1, 4: 0, 5: 1}      # where the next layer's linking rides in the attention launch
    for cfg in (2, 3, 4, 5):
        sh = workloads.shape(cfg)
        reqs, n_src, src_len = workloads.layout(cfg)
        lens = [workloads.request_len(r) for r in reqs]
        tables, pool = workloads.gen_page_tables(sh, lens) if sh.page_size else (None, 0)
        ctx = _ctx(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, mpic.MPIC_BF16, sh.rope_theta, sh.page_size)
        plan = mpic.Plan(ctx, reqs, sh.default_k, tables, pool)
        tiles = plan.get("attn_tiles")
        makespan, busy = 0, 0
        for x in range(8):
            cus = [0] * 32
            heapq.heapify(cus)
            for t in tiles[x::8]:
                if t[3] <= 0:
                    continue
                cost = (t[4] - t[5] + 63) // 64 + 2 + (3 if t[6] >= 0 else 0)
                heapq.heappush(cus, heapq.heappop(cus) + cost)
                busy += cost
            makespan = max(makespan, max(cus))
        est = plan.get("launch_estimate")
        assert est[0] == makespan and est[1] == makespan * 256 - busy, (cfg, est, makespan, busy)
        assert est[2] == 1 and est[3] == want_fits[cfg], (cfg, est)
    # fp32 contexts have no fused launch
    sh = workloads.shape(1)
    reqs, _, _ = workloads.layout(1)
    plan = mpic.Plan(_ctx(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, mpic.MPIC_F32, sh.rope_theta, 0), reqs, sh.default_k)
    assert plan.get("launch_estimate")[2] == 0 and plan.get("launch_estimate")[3] == 0
