"""Parity of the HIP library against the float64 oracle (needs an MI355X).

Every test feeds the same seeded inputs to both sides through the C ABI binding and
compares element by element: integer maps bit-exact, copied rows bit-exact, rotated
keys and attention outputs within the stated floating-point gates."""
import numpy as np
import pytest
import torch

import workloads
import paper_2502_01960_amd as mpic
from helpers import Problem, assert_bf16_close, assert_f32_close, err_stats

pytestmark = pytest.mark.gpu

INT_FIELDS = [f for f in mpic.PLAN_FIELDS
              if f not in ("attn_tiles", "launch_estimate") and not f.startswith(("key_block", "lazy_tiles"))]


def _check_plan(p):
    for f in INT_FIELDS:
        assert np.array_equal(p.plan.get(f), p.oplan[f]), f


def _check_link(p, K_ref, V_ref, bf16):
    Kg, Vg = p.gpu_logical_kv()
    fresh = p.oplan["src_inst"] < 0
    # values and replaced rows are copies: bit-exact
    assert np.array_equal(Vg, V_ref), "V context must be a bit-exact copy"
    if not p.pre_rope:
        assert np.array_equal(Kg[fresh], K_ref[fresh]), "fresh K rows must be bit-exact copies"
    if bf16:
        assert_bf16_close(Kg, K_ref, "K context")
    else:
        assert_f32_close(Kg, K_ref, "K context")
    # slots that belong to no position stay untouched (NaN canary)
    used = np.zeros(p.n_slots, dtype=bool)
    used[p.oplan["dst_slot"]] = True
    if (~used).any():
        idle = torch.from_numpy(np.nonzero(~used)[0]).to(p.k_ctx.device)
        assert torch.isnan(p.k_ctx[idle].float()).all() and torch.isnan(p.v_ctx[idle].float()).all()
    return Kg, Vg


def _run_full(p, host_sourced=None):
    """assemble + attend on the GPU, oracle on the CPU, compare everything."""
    bf16 = p.sh.dtype == "bf16"
    p.gpu_setup(host_sourced)
    _check_plan(p)
    p.gpu_assemble()
    p.gpu_attend()
    torch.cuda.synchronize()
    K_ref, V_ref = p.oracle_link()
    Kg, Vg = _check_link(p, K_ref, V_ref, bf16)
    O_ref, L_ref = p.oracle_attend(K_ref, V_ref)
    O = p.out.to(torch.float64).cpu().numpy()
    L = p.lse.to(torch.float64).cpu().numpy()
    if len(O_ref) == 0:
        return
    if bf16:
        assert_bf16_close(O, O_ref, "attention output (end to end)")
        # isolated attention: oracle fed with the GPU-assembled context
        O_iso, _ = p.oracle_attend(Kg, Vg)
        assert_bf16_close(O, O_iso, "attention output (isolated)")
        assert np.abs(L - L_ref).max() < 2e-2
    else:
        assert_f32_close(O, O_ref, "attention output")
        assert np.abs(L - L_ref).max() <= 1e-5 * max(1.0, np.abs(L_ref).max())


def test_config1_tiny_fp32():
    _run_full(Problem(1))


def test_config2_llava15_like_full():
    _run_full(Problem(2))


def test_config3_reduced_ragged_device_and_host_sources():
    # three ragged chunks per request, two requests: several tiles and ragged tails
    _run_full(Problem(3, n_chunks=3, chunk_len=301, text_len=37, batch=2), host_sourced=False)
    _run_full(Problem(3, n_chunks=3, chunk_len=301, text_len=37, batch=2), host_sourced=True)


def test_config4_reduced_k_sweep():
    for k in (0, 16, 64, 200):      # 200 >= chunk length: everything recomputed
        _run_full(Problem(4, k=k, n_chunks=4, chunk_len=160, text_len=70, batch=3))


def test_config5_reduced_paged():
    _run_full(Problem(5, n_chunks=5, chunk_len=203, text_len=21), host_sourced=False)   # N % 16 != 0
    _run_full(Problem(5, n_chunks=5, chunk_len=203, text_len=21), host_sourced=True)


@pytest.mark.parametrize("block_keys", [64, 96])
def test_both_shapes_of_the_attention_kernel(block_keys):
    """The bf16 kernel exists with 64 and with 96 keys per LDS block: full config 2 (tiles cut along
    the keys, pieces that end inside a block), ragged GQA batch, paged layout with N % 16 != 0,
    listed recompute sets."""
    for p in (Problem(2), Problem(3, n_chunks=3, chunk_len=301, text_len=37, batch=2),
              Problem(5, n_chunks=5, chunk_len=203, text_len=21), Problem(4, k=16, n_chunks=4, chunk_len=160, text_len=70, batch=3)):
        p.block_keys = block_keys
        _run_full(p, host_sourced=False)
    with pytest.raises(mpic.MpicError):
        p.ctx.set_option(mpic.MPIC_OPT_ATTN_BLOCK_KEYS, 80)
    with pytest.raises(mpic.MpicError):
        p.ctx.set_option(99, 1)


@pytest.mark.parametrize("block_keys", [64, 96])
def test_logits_that_grow_fall_and_jump_along_the_keys(block_keys):
    """The reference point of the lazily rescaled softmax: logits that rise by many powers of two
    from block to block (a new reference point in every block), that fall (never a new one, late
    keys underflow), and that jump at random; rows whose first keys are their largest."""
    n = 1500
    base = _custom([[("text", n)], [("text", 40)]], 0, [], 0)
    hq, hkv, d = base.sh.n_q_heads, base.sh.n_kv_heads, base.sh.head_dim
    u = torch.zeros(d)
    u[:64] = 0.5                                             # |u|^2 = 16
    j = torch.arange(n + 40, dtype=torch.float32)
    rng = np.random.default_rng(77)
    walk = torch.from_numpy(np.cumsum(rng.choice([-30.0, 0.0, 0.0, 25.0], size=n + 40)).astype(np.float32))
    for name, level in (("rising", 0.106 * j), ("falling", 0.106 * (n + 40 - j)), ("jumping", 0.05 * walk)):
        p = _custom([[("text", n)], [("text", 40)]], 0, [], 0)
        p.block_keys = block_keys
        p.q = u.expand(n + 40, hq, d).clone().to(torch.bfloat16)
        p.fresh_k = (level[:, None, None] * u[None, None, :]).expand(n + 40, hkv, d).clone().to(torch.bfloat16)
        print(name, "logit range", float((level * 16 / np.sqrt(128)).min()), float((level * 16 / np.sqrt(128)).max()), flush=True)
        _run_full(p, host_sourced=False)


def test_paged_and_contiguous_agree_bitwise():
    a = Problem(5, n_chunks=4, chunk_len=128, text_len=32, paged=16)
    b = Problem(5, n_chunks=4, chunk_len=128, text_len=32, paged=0)
    outs = []
    for p in (a, b):
        p.gpu_setup(False); p.gpu_assemble(); p.gpu_attend(); torch.cuda.synchronize()
        outs.append(p.out.cpu())
    assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16))


def _sampled_rows(p, per_run=6, seed=0):
    rng = np.random.default_rng(seed)
    rows = []
    for (b, r0, ln, p0) in p.oplan["runs"].tolist():
        pick = {r0, r0 + ln - 1} | set((r0 + rng.integers(0, ln, size=per_run)).tolist())
        rows += sorted(pick)
    return np.asarray(rows, dtype=np.int64)


def _run_sampled(p, host_sourced, per_run=6):
    """Full-size configuration: link checked in full, attention on sampled rows (first
    and last row of every run plus random ones), all heads."""
    p.gpu_setup(host_sourced)
    _check_plan(p)
    p.gpu_assemble()
    p.gpu_attend()
    torch.cuda.synchronize()
    K_ref, V_ref = p.oracle_link()
    _check_link(p, K_ref, V_ref, True)
    rows = _sampled_rows(p, per_run)
    O_ref, L_ref = p.oracle_attend(K_ref, V_ref, rows=rows)
    O = p.out.to(torch.float64).cpu().numpy()
    assert np.isfinite(O).all()
    assert_bf16_close(O[rows], O_ref[rows], "attention output (sampled rows)")
    assert np.abs(p.lse.cpu().numpy()[rows] - L_ref[rows]).max() < 2e-2
    # the decode step over the same full-size context (every request, every head)
    _check_decode(p, True, (K_ref, V_ref))


def test_config3_full_size_sampled():
    _run_sampled(Problem(3), host_sourced=False, per_run=3)


def test_config3_full_size_host_sourced_link():
    p = Problem(3, batch=2)
    p.gpu_setup(True)
    p.gpu_assemble()
    K_ref, V_ref = p.oracle_link()
    _check_link(p, K_ref, V_ref, True)
    # a second layer reuses plan, context and staging
    p.gpu_assemble()
    _check_link(p, K_ref, V_ref, True)


def test_config4_full_size_one_layer_sampled():
    _run_sampled(Problem(4, k=16, batch=2), host_sourced=False, per_run=2)


def test_config5_full_size_paged_sampled():
    _run_sampled(Problem(5), host_sourced=True, per_run=1)


# ------------------------------------------------------------------ edge cases
def _custom(requests, n_src, src_len, k, sh_id=3, paged=0):
    p = Problem.__new__(Problem)
    p.sh = workloads.shape(sh_id)
    p.layer, p.k = 0, k
    p.requests, p.n_src, p.src_len = requests, n_src, src_len
    p.page_size = paged
    lens = [workloads.request_len(r) for r in requests]
    if paged:
        p.page_tables, p.n_pool_pages = workloads.gen_page_tables(p.sh, lens, paged)
        p.n_slots = p.n_pool_pages * paged
    else:
        p.page_tables, p.n_pool_pages, p.n_slots = None, 0, max(1, sum(lens))
    from oracle import build_plan
    p.oplan = build_plan(requests, k, paged, p.page_tables)
    p.chunks = {s: workloads.gen_chunk(p.sh, 0, s, src_len[s]) for s in sorted(set(p.oplan["inst_src"].tolist()))}
    q_off = p.oplan["q_off"]
    fresh = [workloads.gen_fresh(p.sh, 0, b, int(q_off[b + 1] - q_off[b])) for b in range(len(requests))]
    p.q = torch.cat([f[0] for f in fresh]); p.fresh_k = torch.cat([f[1] for f in fresh]); p.fresh_v = torch.cat([f[2] for f in fresh])
    return p


def test_edge_layouts():
    # chunk first (zero shift = bit-exact copy), same chunk twice, single-token and empty
    # text segments, k = 0 next to k >= L, request with no fresh row at all
    reqs = [[("chunk", 0, 70, None), ("text", 1), ("chunk", 0, 70, 0), ("text", 0), ("chunk", 1, 33, 99), ("text", 1)],
            [("chunk", 1, 33, 0)],
            [("text", 5)]]
    p = _custom(reqs, 2, [70, 33], 3)
    _run_full(p, host_sourced=False)
    Kg, _ = p.gpu_logical_kv()
    first = p.chunks[0][0].to(torch.float64).numpy()
    assert np.array_equal(Kg[3:70], first[3:70]), "zero shift must copy keys bit-exactly"
    _run_full(_custom(reqs, 2, [70, 33], 3, paged=16), host_sourced=True)


def test_empty_recompute_set_is_a_noop():
    p = _custom([[("chunk", 0, 40, None), ("chunk", 1, 24, None)]], 2, [40, 24], 0)
    _run_full(p, host_sourced=False)
    assert torch.isnan(p.out.float()).all() or p.out.numel() == 0


def test_rejected_gpu_calls_enqueue_nothing():
    p = Problem(1)
    p.gpu_setup()
    small = p.k_ctx[:100]
    with pytest.raises(mpic.MpicError):
        mpic.mpic_assemble_kv(p.ctx.handle, p.plan.handle, p.srcs, p.d_fk, p.d_fv, small, small)
    with pytest.raises(mpic.MpicError):
        mpic.mpic_assemble_kv(p.ctx.handle, p.plan.handle, p.srcs, p.d_fk[:10], p.d_fv[:10], p.k_ctx, p.v_ctx)
    with pytest.raises(mpic.MpicError):
        mpic.mpic_assemble_kv(p.ctx.handle, p.plan.handle, p.srcs[:1], p.d_fk, p.d_fv, p.k_ctx, p.v_ctx)
    with pytest.raises(mpic.MpicError):
        mpic.mpic_selective_attn(p.ctx.handle, p.plan.handle, p.d_q, p.k_ctx, p.v_ctx, float("nan"), p.out)
    torch.cuda.synchronize()
    assert torch.isnan(p.k_ctx).all() and torch.isnan(p.out).all()
    other = mpic.Context(4, 4, 64, mpic.MPIC_F32, 1e4)
    with pytest.raises(mpic.MpicError):
        mpic.mpic_assemble_kv(other.handle, p.plan.handle, p.srcs, p.d_fk, p.d_fv, p.k_ctx, p.v_ctx)


def test_interleaved_rotary_pairs():
    from oracle import link_kv
    for cfg in (1, 3):
        p = Problem(cfg, n_chunks=2, chunk_len=64, text_len=9, batch=1) if cfg == 3 else Problem(1)
        p.gpu_setup(False)
        sh = p.sh
        dt = mpic.MPIC_F32 if sh.dtype == "f32" else mpic.MPIC_BF16
        p.ctx = mpic.Context(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, dt, sh.rope_theta, 1, 0)
        p.plan = mpic.Plan(p.ctx, p.requests, p.k)
        p.gpu_assemble()
        f64 = lambda t: t.to(torch.float64).numpy()
        K_ref, V_ref = link_kv(p.oplan, {s: f64(kv[0]) for s, kv in p.chunks.items()},
                               {s: f64(kv[1]) for s, kv in p.chunks.items()},
                               f64(p.fresh_k), f64(p.fresh_v), sh.rope_theta, interleaved=True)
        _check_link(p, K_ref, V_ref, sh.dtype == "bf16")


def test_fresh_rows_before_positional_embedding():
    """Contexts created with fresh_pre_rope: the library rotates fresh keys while linking and
    fresh queries while attending, by their position ids; fp32 and bf16, both pairings,
    contiguous and paged, several requests (position ids restart per request)."""
    _run_full(Problem(1, pre_rope=True))
    _run_full(Problem(1, pre_rope=True, interleaved=True))
    _run_full(Problem(3, n_chunks=3, chunk_len=301, text_len=37, batch=2, pre_rope=True), host_sourced=False)
    _run_full(Problem(3, n_chunks=3, chunk_len=301, text_len=37, batch=2, pre_rope=True, interleaved=True),
              host_sourced=True)
    _run_full(Problem(5, n_chunks=5, chunk_len=203, text_len=21, pre_rope=True), host_sourced=False)
    _run_full(Problem(4, k=200, n_chunks=4, chunk_len=160, text_len=70, batch=3, pre_rope=True))
    # the fresh part alone takes the same route
    p = Problem(3, n_chunks=2, chunk_len=130, text_len=11, batch=2, pre_rope=True)
    p.gpu_setup(False)
    p.gpu_assemble(); torch.cuda.synchronize()
    k_ref = p.k_ctx.clone()
    p.k_ctx.fill_(float("nan")); p.v_ctx.fill_(float("nan"))
    mpic.mpic_assemble_kv_parts(p.ctx.handle, p.plan.handle, p.srcs, None, None, p.k_ctx, p.v_ctx, mpic.MPIC_PART_CACHED)
    mpic.mpic_assemble_kv_parts(p.ctx.handle, p.plan.handle, None, p.d_fk, p.d_fv, p.k_ctx, p.v_ctx, mpic.MPIC_PART_FRESH)
    torch.cuda.synchronize()
    assert torch.equal(p.k_ctx.view(torch.int16), k_ref.view(torch.int16))


def test_random_layouts_and_head_groupings():
    """Seeded random layouts (ragged chunks, empty text, k from 0 to beyond the chunk) with
    several head groupings, including a group size of 7 and tiles that straddle runs and
    end in a partial wavefront."""
    import dataclasses
    rng = np.random.default_rng(20250201)
    groupings = [(4, 4), (8, 2), (28, 4), (7, 1), (64, 8)]
    for case in range(10):
        hq, hkv = groupings[case % len(groupings)]
        n_src = int(rng.integers(1, 4))
        src_len = [int(rng.integers(1, 200)) for _ in range(n_src)]
        reqs = []
        for _ in range(int(rng.integers(1, 4))):
            segs = []
            for _ in range(int(rng.integers(1, 6))):
                if rng.random() < 0.45:
                    segs.append(("text", int(rng.integers(0, 50))))
                else:
                    s = int(rng.integers(0, n_src))
                    k = [None, 0, 1, 17, 500][int(rng.integers(0, 5))]
                    segs.append(("chunk", s, src_len[s], k))
            reqs.append(segs)
        paged = 16 if case % 3 == 2 else 0
        p = _custom(reqs, n_src, src_len, int(rng.integers(0, 40)), paged=paged)
        p.sh = dataclasses.replace(p.sh, n_q_heads=hq, n_kv_heads=hkv)
        p.pre_rope, p.interleaved = case % 3 == 1, case % 4 == 3
        # regenerate the tensors for the new head counts
        p.chunks = {s: workloads.gen_chunk(p.sh, case, s, src_len[s]) for s in p.chunks}
        q_off = p.oplan["q_off"]
        fresh = [workloads.gen_fresh(p.sh, case, b, int(q_off[b + 1] - q_off[b])) for b in range(len(reqs))]
        p.q = torch.cat([f[0] for f in fresh]); p.fresh_k = torch.cat([f[1] for f in fresh]); p.fresh_v = torch.cat([f[2] for f in fresh])
        _run_full(p, host_sourced=bool(case % 2))


def test_linking_in_two_parts_equals_one_call():
    """Cached rows first (they need no model output), fresh rows later, on two streams:
    bit-identical to the single call; either part alone leaves the other rows untouched."""
    for host in (False, True):
        p = Problem(3, n_chunks=3, chunk_len=301, text_len=37, batch=2)
        p.gpu_setup(host)
        p.gpu_assemble()
        torch.cuda.synchronize()
        k_ref, v_ref = p.k_ctx.clone(), p.v_ctx.clone()
        fresh = torch.from_numpy(p.oplan["dst_slot"][p.oplan["src_inst"] < 0].astype(np.int64)).to(p.k_ctx.device)
        p.k_ctx.fill_(float("nan")); p.v_ctx.fill_(float("nan"))
        side = torch.cuda.Stream()
        torch.cuda.synchronize()
        mpic.mpic_assemble_kv_parts(p.ctx.handle, p.plan.handle, p.srcs, None, None, p.k_ctx, p.v_ctx,
                                    mpic.MPIC_PART_CACHED | (mpic.MPIC_PART_BACKGROUND if host else 0), side)
        side.synchronize()
        assert torch.isnan(p.k_ctx[fresh].float()).all(), "the cached part must not touch fresh rows"
        mpic.mpic_assemble_kv_parts(p.ctx.handle, p.plan.handle, None, p.d_fk, p.d_fv, p.k_ctx, p.v_ctx,
                                    mpic.MPIC_PART_FRESH)
        torch.cuda.synchronize()
        assert torch.equal(p.k_ctx.view(torch.int16), k_ref.view(torch.int16))
        assert torch.equal(p.v_ctx.view(torch.int16), v_ref.view(torch.int16))
    # the background hint changes the launch shape only
    p = Problem(3, n_chunks=3, chunk_len=301, text_len=37, batch=2)
    p.gpu_setup(False)
    p.gpu_assemble(); torch.cuda.synchronize()
    k_ref = p.k_ctx.clone()
    p.k_ctx.fill_(float("nan"))
    mpic.mpic_assemble_kv_parts(p.ctx.handle, p.plan.handle, p.srcs, p.d_fk, p.d_fv, p.k_ctx, p.v_ctx,
                                mpic.MPIC_PART_CACHED | mpic.MPIC_PART_FRESH | mpic.MPIC_PART_BACKGROUND)
    torch.cuda.synchronize()
    assert torch.equal(p.k_ctx.view(torch.int16), k_ref.view(torch.int16))
    for bad in (0, mpic.MPIC_PART_BACKGROUND, 8):
        with pytest.raises(mpic.MpicError):
            mpic.mpic_assemble_kv_parts(p.ctx.handle, p.plan.handle, p.srcs, p.d_fk, p.d_fv, p.k_ctx, p.v_ctx, bad)


def _check_decode(p, with_self=True, linked=None):
    """Decode step over the context that p has linked on the GPU: oracle fed the oracle's
    own linked context (end to end)."""
    bf16 = p.sh.dtype == "bf16"
    K_ref, V_ref = linked if linked is not None else p.oracle_link()
    q, nk, nv = p.decode_inputs()
    if not with_self:
        nk = nv = None
    O, L = p.gpu_decode(q, nk, nv)
    O_ref, L_ref = p.oracle_decode(K_ref, V_ref, q, nk, nv)
    empty = np.isneginf(L_ref)
    assert np.array_equal(np.isneginf(L), empty)
    if bf16:
        assert_bf16_close(O, O_ref, "decode output")
        assert np.abs(L[~empty] - L_ref[~empty]).max(initial=0.0) < 2e-2
    else:
        assert_f32_close(O, O_ref, "decode output")
        assert np.abs(L[~empty] - L_ref[~empty]).max(initial=0.0) <= 1e-5 * max(1.0, np.abs(L_ref[~empty]).max(initial=0.0))


def test_recompute_sets_named_token_by_token():
    """Recompute sets from another policy than first-k (scattered tokens, many short runs):
    a seeded 12 % of every chunk plus its first token, contiguous and paged, device and
    host sources; and a set that is everything / nothing."""
    rng = np.random.default_rng(77)
    for paged, host in ((0, False), (16, True)):
        reqs = []
        for b in range(3):
            segs = [("text", 9 + b)]
            for c in range(3):
                L = 257
                pick = sorted(set([0] + rng.choice(L, size=L // 8, replace=False).tolist()))
                segs += [("chunk", c, L, pick), ("text", 5)]
            reqs.append(segs)
        reqs.append([("chunk", 0, 257, list(range(257))), ("chunk", 1, 257, []), ("text", 2)])
        p = _custom(reqs, 3, [257, 257, 257], 4, paged=paged)
        assert len(p.oplan["runs"]) > 200
        _run_full(p, host_sourced=host)


def test_k_distance_and_ranked_recompute_set():
    """K distance of Sec. 4.2 on the GPU against the oracle (fp32 and bf16), then the whole
    chain: rank the tokens of each chunk by it, recompute the top 10 %, link and attend."""
    from oracle import k_distance, top_tokens
    dev = torch.device("cuda:0")
    for cfg in (1, 5):
        sh = workloads.shape(cfg)
        dt = mpic.MPIC_F32 if sh.dtype == "f32" else mpic.MPIC_BF16
        ctx = mpic.Context(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, dt, sh.rope_theta)
        L = 1153
        a, b = workloads.gen_chunk(sh, 0, 0, L)[0], workloads.gen_chunk(sh, 1, 0, L)[0]
        b[5] = a[5]                                  # an identical token: distance exactly 0
        dist = torch.full((L,), float("nan"), dtype=torch.float32, device=dev)
        mpic.mpic_k_distance(ctx.handle, a.to(dev), b.to(dev), dist)
        torch.cuda.synchronize()
        want = k_distance(a.to(torch.float64).numpy(), b.to(torch.float64).numpy())
        got = dist.cpu().numpy().astype(np.float64)
        assert got[5] == 0.0
        assert np.abs(got - want).max() <= 1e-5 * want.max()
        assert mpic.mpic_rank_tokens(dist.cpu().numpy(), 50).tolist() == top_tokens(dist.cpu().numpy(), 50).tolist()
    # the chain on a reduced config 3: sets chosen by rank instead of by position
    sh = workloads.shape(3)
    ctx = mpic.Context(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, mpic.MPIC_BF16, sh.rope_theta)
    L, picks = 301, []
    for c in range(3):
        a, b = workloads.gen_chunk(sh, 0, c, L)[0].to(dev), workloads.gen_chunk(sh, 7, c, L)[0].to(dev)
        dist = torch.empty((L,), dtype=torch.float32, device=dev)
        mpic.mpic_k_distance(ctx.handle, a, b, dist)
        picks.append(mpic.mpic_rank_tokens(dist.cpu().numpy(), L // 10).tolist())
    reqs = [[("text", 20)] + [seg for c in range(3) for seg in (("chunk", c, L, picks[c]), ("text", 11))]]
    _run_full(_custom(reqs, 3, [L, L, L], 0), host_sourced=False)


def test_host_chunks_read_in_place_by_the_kernel():
    """MPIC_SRC_HOST_MAPPED: pinned host chunks are read over the bus by the linking kernel
    itself (no staging copies).  Same gates as the other routes, bit-identical context, also
    when only the cached part is linked, and mixed with device-resident chunks."""
    for make in (lambda: Problem(3, n_chunks=3, chunk_len=301, text_len=37, batch=2),
                 lambda: Problem(5, n_chunks=5, chunk_len=203, text_len=21)):
        ref = make(); ref.gpu_setup(False); ref.gpu_assemble(); torch.cuda.synchronize()
        p = make()
        p.host_mode = mpic.MPIC_SRC_HOST_MAPPED
        _run_full(p, host_sourced=True)
        assert torch.equal(p.k_ctx[~torch.isnan(p.k_ctx.float())].view(torch.int16),
                           ref.k_ctx[~torch.isnan(ref.k_ctx.float())].view(torch.int16))
        # one chunk from the device, the others from the host, cached part on a second stream
        p.srcs[0] = tuple(t.to(p.k_ctx.device) for t in p.chunks[0])
        p.k_ctx.fill_(float("nan")); p.v_ctx.fill_(float("nan"))
        side = torch.cuda.Stream()
        torch.cuda.synchronize()
        mpic.mpic_assemble_kv_parts(p.ctx.handle, p.plan.handle, p.srcs, None, None, p.k_ctx, p.v_ctx,
                                    mpic.MPIC_PART_CACHED, side, mpic.MPIC_SRC_HOST_MAPPED)
        mpic.mpic_assemble_kv_parts(p.ctx.handle, p.plan.handle, None, p.d_fk, p.d_fv, p.k_ctx, p.v_ctx,
                                    mpic.MPIC_PART_FRESH)
        torch.cuda.synchronize()
        same = ~torch.isnan(ref.k_ctx.float())
        assert torch.equal(p.k_ctx[same].view(torch.int16), ref.k_ctx[same].view(torch.int16))
        assert torch.equal(p.v_ctx[same].view(torch.int16), ref.v_ctx[same].view(torch.int16))
    with pytest.raises(mpic.MpicError):
        mpic.mpic_assemble_kv(p.ctx.handle, p.plan.handle, p.srcs, p.d_fk, p.d_fv, p.k_ctx, p.v_ctx, None, 3)


def test_decode_step_after_prefill():
    """One query per request over the linked context (contiguous and paged, fp32 and bf16,
    ragged lengths that end inside a 32-key block and inside a split), with and without
    the new token's own key and value."""
    cases = [Problem(1),
             Problem(2, n_chunks=2, chunk_len=150, text_len=13),
             Problem(3, n_chunks=3, chunk_len=301, text_len=37, batch=2),
             Problem(4, k=16, n_chunks=4, chunk_len=160, text_len=70, batch=3),
             Problem(5, n_chunks=5, chunk_len=203, text_len=21)]
    for p in cases:
        p.gpu_setup(False)
        p.gpu_assemble()
        _check_decode(p, True)
        _check_decode(p, False)


def test_decode_step_edge_cases():
    # requests of very different lengths in one batch, one of them empty, one a single token
    reqs = [[("text", 1)], [], [("chunk", 0, 700, None), ("text", 3)], [("chunk", 1, 33, 0)]]
    for paged in (0, 16):
        p = _custom(reqs, 2, [700, 33], 5, paged=paged)
        p.gpu_setup(False)
        p.gpu_assemble()
        _check_decode(p, True)
        _check_decode(p, False)     # the empty request has no key at all: zeros, lse = -inf
    # head groupings: multi-head (1 column in use), a group of 7, a group wider than one tile
    import dataclasses
    for hq, hkv in [(4, 4), (7, 1), (80, 2)]:
        p = _custom([[("text", 40), ("chunk", 0, 300, None), ("text", 9)], [("chunk", 0, 300, 2)]], 1, [300], 4)
        p.sh = dataclasses.replace(p.sh, n_q_heads=hq, n_kv_heads=hkv)
        p.chunks = {s: workloads.gen_chunk(p.sh, 0, s, 300) for s in p.chunks}
        q_off = p.oplan["q_off"]
        fresh = [workloads.gen_fresh(p.sh, 0, b, int(q_off[b + 1] - q_off[b])) for b in range(2)]
        p.q = torch.cat([f[0] for f in fresh]); p.fresh_k = torch.cat([f[1] for f in fresh]); p.fresh_v = torch.cat([f[2] for f in fresh])
        p.gpu_setup(False)
        p.gpu_assemble()
        _check_decode(p, True)
    with pytest.raises(mpic.MpicError):
        mpic.mpic_decode_attn(p.ctx.handle, p.plan.handle, p.d_q[:2], p.d_fk[:2], None, p.k_ctx, p.v_ctx, 1.0, p.out[:2])


def test_rows_staged_past_a_request_end_are_linked_rows():
    """Paged layout whose page 0 is in no table and holds NaN: the last key block of a request
    is staged past the request's end, and what is staged there must never be an untouched
    slot (zero weight times NaN would poison the output)."""
    reqs = [[("text", 5), ("chunk", 0, 90, None), ("text", 6)]]      # 101 tokens: ends inside a page and a block
    p = _custom(reqs, 1, [90], 4, paged=16)
    tables = [np.asarray(t).copy() for t in p.page_tables]
    used = set(np.concatenate(tables).tolist())
    spare = next(i for i in range(1, p.n_pool_pages) if i not in used)
    for t in tables:
        t[t == 0] = spare
    p.page_tables = tables
    from oracle import build_plan
    p.oplan = build_plan(reqs, 4, 16, tables)
    assert 0 not in set(np.concatenate(tables).tolist())
    _run_full(p, host_sourced=False)
    assert torch.isnan(p.k_ctx[:16].float()).all()
    _check_decode(p, True)


def test_calls_can_be_captured_in_a_graph():
    """After one eager call (which uploads the plan and sizes the workspaces) linking, attention
    and the decode step are plain kernel launches on the caller's stream, so a launch-bound
    loop can be captured in a HIP graph: three replays with new inputs in the same buffers,
    eager work between the replays, every replay bit-identical to the eager result."""
    p = Problem(2, n_chunks=2, chunk_len=150, text_len=13)     # small: tiles cut along the keys, merge kernel
    p.gpu_setup(False)
    dq, dk, dv = (t.to(p.k_ctx.device) for t in p.decode_inputs())
    dec_out = torch.empty_like(dq)

    nk, nv = torch.full_like(p.k_ctx, float("nan")), torch.full_like(p.v_ctx, float("nan"))   # the next layer's context

    def run():
        p.gpu_assemble()
        # attention with the next layer's stored rows linked by the same launch
        mpic.mpic_selective_attn_link_next(p.ctx.handle, p.plan.handle, p.d_q, p.k_ctx, p.v_ctx, p.sh.softmax_scale,
                                           p.out, p.srcs, nk, nv, p.lse)
        mpic.mpic_decode_attn(p.ctx.handle, p.plan.handle, dq, dk, dv, p.k_ctx, p.v_ctx, p.sh.softmax_scale, dec_out)

    run()                                                       # eager warm-up: uploads, workspaces
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    gen = torch.Generator(device="cpu").manual_seed(5)
    for rep in range(3):
        for t in (p.d_q, p.d_fk, p.d_fv, dq, dk, dv):
            t.copy_(torch.randn(t.shape, generator=gen).to(t.dtype))
        run()                                                   # eager reference on the new inputs
        torch.cuda.synchronize()
        want = [x.clone() for x in (p.k_ctx, p.v_ctx, p.out, p.lse, dec_out, nk, nv)]
        for x in (p.k_ctx, p.v_ctx, p.out, dec_out, nk, nv):
            x.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((p.k_ctx, p.v_ctx, p.out, p.lse, dec_out, nk, nv), want):
            assert torch.equal(got.view(torch.int16 if got.dtype == torch.bfloat16 else torch.int32),
                               ref.view(torch.int16 if ref.dtype == torch.bfloat16 else torch.int32))


def test_random_feature_combinations():
    """Seeded random mixes of everything the library takes: batch sizes, head groupings from
    multi-head to a group of 32, first-k and listed recompute sets, contiguous and paged with
    several page sizes, both rotary pairings, fresh rows handed over rotated or not, chunks on the
    device, staged from the host or read in place; link, attention and the decode step against
    the oracle for every mix."""
    import dataclasses
    rng = np.random.default_rng(424242)
    groupings = [(32, 1), (16, 1), (32, 32), (28, 4), (8, 8), (12, 3)]
    for case in range(12):
        hq, hkv = groupings[case % len(groupings)]
        n_src = int(rng.integers(1, 5))
        src_len = [int(rng.integers(1, 400)) for _ in range(n_src)]
        reqs = []
        for _ in range(int(rng.integers(1, 7))):
            segs = []
            for _ in range(int(rng.integers(1, 7))):
                if rng.random() < 0.4:
                    segs.append(("text", int(rng.integers(0, 80))))
                else:
                    s_ = int(rng.integers(0, n_src))
                    pick = rng.random()
                    if pick < 0.35:
                        k = sorted(set(rng.integers(0, src_len[s_], size=int(rng.integers(0, 1 + src_len[s_] // 3))).tolist()))
                    else:
                        k = [None, 0, 1, 33, 1000][int(rng.integers(0, 5))]
                    segs.append(("chunk", s_, src_len[s_], k))
            reqs.append(segs)
        paged = [0, 16, 32, 1][case % 4]
        p = _custom(reqs, n_src, src_len, int(rng.integers(0, 70)), paged=paged)
        p.sh = dataclasses.replace(p.sh, n_q_heads=hq, n_kv_heads=hkv)
        p.pre_rope, p.interleaved = bool(case % 2), bool((case // 2) % 2)
        p.host_mode = mpic.MPIC_SRC_HOST_MAPPED if case % 3 == 0 else mpic.MPIC_SRC_HOST_STAGED
        p.block_keys = [0, 64, 96][(case // 2) % 3]
        p.chunks = {s_: workloads.gen_chunk(p.sh, 100 + case, s_, src_len[s_]) for s_ in p.chunks}
        q_off = p.oplan["q_off"]
        fresh = [workloads.gen_fresh(p.sh, 100 + case, b, int(q_off[b + 1] - q_off[b])) for b in range(len(reqs))]
        p.q = torch.cat([f[0] for f in fresh]); p.fresh_k = torch.cat([f[1] for f in fresh]); p.fresh_v = torch.cat([f[2] for f in fresh])
        _run_full(p, host_sourced=case % 3 != 1)
        if p.pre_rope:
            continue      # the decode step takes rotated inputs; its oracle check links with rotated fresh keys
        _check_decode(p, bool(case % 2 == 0))
