"""Contexts with lazy_rope (needs an MI355X): stored keys are never rewritten.  Linking copies
them as stored, or does not touch them at all (caches linked by reference), and the attention
and decode kernels turn the query back by the shift of each chunk instance.

Expected values: the oracle's linked-and-shifted context and its attention (link_kv + attend),
at the gates of the other parity tests -- the lazy route must give the same outputs.  What the
context holds is compared bit for bit with oracle.link_kv_unshifted (stored keys as stored)."""
import dataclasses

import numpy as np
import pytest
import torch

import workloads
import paper_2502_01960_amd as mpic
from helpers import Problem, assert_bf16_close, assert_f32_close
from test_gpu_parity import _custom, _sampled_rows

pytestmark = pytest.mark.gpu


def _bits(t):
    return t.view(torch.int16 if t.element_size() == 2 else torch.int32)


def _close(p):
    return assert_f32_close if p.sh.dtype == "f32" else assert_bf16_close


def _check_outputs(p, O_ref, L_ref, rows=None, what="attention output"):
    O = p.out.to(torch.float64).cpu().numpy()
    L = p.lse.to(torch.float64).cpu().numpy()
    if O_ref.size == 0:
        return
    sel = slice(None) if rows is None else rows
    assert np.isfinite(O).all()
    _close(p)(O[sel], O_ref[sel], what)
    tol = 1e-5 * max(1.0, np.abs(L_ref[sel]).max()) if p.sh.dtype == "f32" else 2e-2
    assert np.abs(L[sel] - L_ref[sel]).max() <= tol


def _run_lazy(p, rows=None, decode=True):
    """Both lazy routes on problem p: (a) stored rows copied unrotated into the context, (b) caches
    linked by reference (only fresh rows reach the context).  Returns the oracle's linked context."""
    p.lazy = True
    p.gpu_setup(False)
    for f in ("q_pos", "slot_map", "src_inst", "src_row", "dst_slot"):
        assert np.array_equal(p.plan.get(f), p.oplan[f]), f
    K_ref, V_ref = p.oracle_link()
    O_ref, L_ref = p.oracle_attend(K_ref, V_ref, rows=rows)
    K0, V0, shift = p.oracle_link_unshifted()
    # (a) the context holds every row; stored keys exactly as stored
    p.gpu_assemble()
    p.gpu_attend()
    torch.cuda.synchronize()
    Kg, Vg = p.gpu_logical_kv()
    assert np.array_equal(Vg, V0), "V context must be a bit-exact copy"
    stored = p.oplan["src_inst"] >= 0
    assert np.array_equal(Kg[stored], K0[stored]), "stored keys must be copied as stored"
    if p.pre_rope:
        _close(p)(Kg[~stored], K0[~stored], "fresh K rows (rotated by the library)")
    else:
        assert np.array_equal(Kg[~stored], K0[~stored]), "fresh K rows must be bit-exact copies"
    _check_outputs(p, O_ref, L_ref, rows, "attention output (stored keys copied unrotated)")
    out_copy = p.out.clone()
    dec = None
    if decode and not p.pre_rope:
        q, nk, nv = p.decode_inputs()
        Od_ref, Ld_ref = p.oracle_decode(K_ref, V_ref, q, nk, nv)
        Od, Ld = p.gpu_decode(q, nk, nv)
        _close(p)(Od, Od_ref, "decode output (stored keys copied unrotated)")
        dec = (q, nk, nv, Od_ref, Od)
    # (b) by reference: the context receives the fresh rows only, the rest stays untouched
    p.k_ctx.fill_(float("nan")); p.v_ctx.fill_(float("nan")); p.out.fill_(float("nan")); p.lse.fill_(float("nan"))
    p.gpu_link_fresh_only()
    p.gpu_attend_in_place()
    torch.cuda.synchronize()
    Kg, Vg = p.gpu_logical_kv()
    assert np.isnan(Kg[stored]).all() and np.isnan(Vg[stored]).all(), "stored rows must not reach the context"
    assert not np.isnan(Kg[~stored]).any()
    _check_outputs(p, O_ref, L_ref, rows, "attention output (caches linked by reference)")
    # the two routes stage the same values and do the same arithmetic
    if len(O_ref):
        assert torch.equal(_bits(p.out), _bits(out_copy)), "by reference and by copy must agree bit for bit"
    if dec is not None:
        q, nk, nv, Od_ref, Od = dec
        Od2, _ = p.gpu_decode_in_place(q, nk, nv)
        _close(p)(Od2, Od_ref, "decode output (caches linked by reference)")
        assert np.array_equal(Od2, Od)
    return K_ref, V_ref


@pytest.mark.parametrize("block_keys", [64, 96])
def test_lazy_routes_on_reduced_configurations(block_keys):
    """Reduced configs 2-5 (ragged chunks, several requests, paged with N % 16 != 0, the k sweep with
    k = 0 and k beyond the chunk), both shapes of the attention kernel."""
    cases = [Problem(2, n_chunks=2, chunk_len=150, text_len=13),
             Problem(3, n_chunks=3, chunk_len=301, text_len=37, batch=2),
             Problem(5, n_chunks=5, chunk_len=203, text_len=21)]
    cases += [Problem(4, k=k, n_chunks=4, chunk_len=160, text_len=70, batch=3) for k in (0, 16, 64, 200)]
    for p in cases:
        p.block_keys = block_keys
        _run_lazy(p)


def test_lazy_fp32_configuration():
    _run_lazy(Problem(1))
    _run_lazy(Problem(1, interleaved=True))


def test_lazy_config2_full_with_tiles_cut_along_the_keys():
    """Full config 2: a small problem whose tiles are cut along the keys, so pieces must own whole
    key blocks and the partial results are merged."""
    for bk in (64, 96):
        p = Problem(2)
        p.block_keys = bk
        _run_lazy(p)
        assert (p.plan.get("attn_tiles")[:, 6] >= 0).any()


def test_lazy_with_other_pairing_and_unpositioned_fresh_rows():
    _run_lazy(Problem(3, n_chunks=3, chunk_len=301, text_len=37, batch=2, interleaved=True))
    _run_lazy(Problem(3, n_chunks=3, chunk_len=301, text_len=37, batch=2, pre_rope=True))
    _run_lazy(Problem(5, n_chunks=4, chunk_len=203, text_len=21, pre_rope=True, interleaved=True))
    _run_lazy(Problem(1, pre_rope=True))


def test_lazy_edge_layouts_and_listed_recompute_sets():
    # chunk first (no shift at all), same chunk twice, single-token and empty text, k = 0 next to
    # k >= L, a request with no fresh row, a request of text only
    reqs = [[("chunk", 0, 70, None), ("text", 1), ("chunk", 0, 70, 0), ("text", 0), ("chunk", 1, 33, 99), ("text", 1)],
            [("chunk", 1, 33, 0)],
            [("text", 5)]]
    _run_lazy(_custom(reqs, 2, [70, 33], 3))
    _run_lazy(_custom(reqs, 2, [70, 33], 3, paged=16))
    # recompute sets named token by token: many short stored and fresh runs, i.e. many short key blocks
    rng = np.random.default_rng(5)
    pick = lambda L, n: tuple(sorted(rng.choice(L, size=n, replace=False).tolist()))
    reqs = [[("text", 7), ("chunk", 0, 300, pick(300, 40)), ("chunk", 1, 211, pick(211, 5)), ("text", 3)],
            [("chunk", 1, 211, pick(211, 60)), ("text", 2), ("chunk", 0, 300, ())]]
    _run_lazy(_custom(reqs, 2, [300, 211], 0))


def test_lazy_random_layouts_and_head_groupings():
    rng = np.random.default_rng(20260101)
    groupings = [(4, 4), (8, 2), (28, 4), (7, 1), (64, 8)]
    for case in range(6):
        hq, hkv = groupings[case % len(groupings)]
        n_src = int(rng.integers(1, 4))
        src_len = [int(rng.integers(1, 400)) for _ in range(n_src)]
        reqs = []
        for _ in range(int(rng.integers(1, 4))):
            segs = []
            for _ in range(int(rng.integers(1, 6))):
                if rng.random() < 0.4:
                    segs.append(("text", int(rng.integers(0, 50))))
                else:
                    s = int(rng.integers(0, n_src))
                    segs.append(("chunk", s, src_len[s], [None, 0, 5, 1000][int(rng.integers(0, 4))]))
            reqs.append(segs)
        p = _custom(reqs, n_src, src_len, int(rng.integers(0, 40)), paged=[0, 16][case % 2])
        p.sh = dataclasses.replace(p.sh, n_q_heads=hq, n_kv_heads=hkv)
        p.chunks = {s: workloads.gen_chunk(p.sh, 200 + case, s, src_len[s]) for s in p.chunks}
        q_off = p.oplan["q_off"]
        fresh = [workloads.gen_fresh(p.sh, 200 + case, b, int(q_off[b + 1] - q_off[b])) for b in range(len(reqs))]
        p.q = torch.cat([f[0] for f in fresh]); p.fresh_k = torch.cat([f[1] for f in fresh]); p.fresh_v = torch.cat([f[2] for f in fresh])
        p.block_keys = [0, 64, 96][case % 3]
        print("lazy random case", case, (hq, hkv), [len(r) for r in reqs], flush=True)
        _run_lazy(p)


def test_lazy_config5_full_size_in_place_sampled():
    """The long paged request at full size (75 840 tokens, 32 chunks): linked by reference, sampled rows."""
    p = Problem(5)
    rows = _sampled_rows(p, per_run=1)
    _run_lazy(p, rows=rows)


def test_lazy_config3_full_size_in_place_sampled():
    p = Problem(3)
    rows = _sampled_rows(p, per_run=2)
    _run_lazy(p, rows=rows)


def test_lazy_rejections():
    p = Problem(3, n_chunks=2, chunk_len=100, text_len=9, batch=1)
    p.gpu_setup(False)                      # a context without lazy_rope
    with pytest.raises(mpic.MpicError):
        p.gpu_attend_in_place()
    q = Problem(3, n_chunks=2, chunk_len=100, text_len=9, batch=1)
    q.lazy = True
    q.gpu_setup(True)                       # caches in pinned host memory cannot be read in place
    q.gpu_link_fresh_only()
    with pytest.raises(mpic.MpicError):
        q.gpu_attend_in_place()
    with pytest.raises(mpic.MpicError):
        mpic.mpic_selective_attn_in_place(q.ctx.handle, q.plan.handle, q.d_q, q.srcs[:1], q.k_ctx, q.v_ctx,
                                          q.sh.softmax_scale, q.out)
    torch.cuda.synchronize()
    assert torch.isnan(q.out.float()).all()
    # ... but the copying route takes them (staged over the side stream, copied unrotated)
    q.gpu_assemble()
    q.gpu_attend()
    torch.cuda.synchronize()
    K_ref, V_ref = q.oracle_link()
    O_ref, L_ref = q.oracle_attend(K_ref, V_ref)
    _check_outputs(q, O_ref, L_ref)


def test_lazy_layers_through_the_pipeline(tmp_path):
    """mpic_prefill_layers on a lazy_rope context.  Caches in the HBM tier are linked by reference:
    the context receives the fresh rows only.  Caches in the host and disk tiers are linked as
    stored (read over the bus, copied unrotated).  Outputs at the gates of the oracle either way."""
    from helpers import LayeredProblem
    HBM, HOST, DISK = mpic.MPIC_TIER_HBM, mpic.MPIC_TIER_HOST, mpic.MPIC_TIER_DISK
    small = dict(n_chunks=3, chunk_len=300, text_len=24, batch=2)
    for tiers in ((HBM,), (HOST, DISK), (HBM, HOST)):
        p = LayeredProblem(3, 3, tiers, tmp_path if DISK in tiers else None, lazy=True, **small)
        p.plan_for()
        assert p.gpu_run() is None
        ref = p.oracle_run()
        p.check(ref, kv_layers=[])                      # outputs and log-sum-exp of every layer
        slots = torch.from_numpy(p.oplan["dst_slot"].astype(np.int64)).to(p.k_ctx[0].device)
        stored = torch.from_numpy(p.oplan["src_inst"] >= 0).to(slots.device)
        for l in range(p.n_layers):
            K, V, _, _ = ref[l]
            k_log, v_log = p.k_ctx[l][slots], p.v_ctx[l][slots]
            assert np.array_equal(v_log[~stored].to(torch.float64).cpu().numpy(), V[~stored.cpu().numpy()])
            assert np.array_equal(k_log[~stored].to(torch.float64).cpu().numpy(), K[~stored.cpu().numpy()])
            if tiers == (HBM,):
                assert torch.isnan(k_log[stored].float()).all() and torch.isnan(v_log[stored].float()).all(), \
                    "caches in GPU memory are linked by reference: their rows must not be copied"
            else:
                assert np.array_equal(v_log[stored].to(torch.float64).cpu().numpy(), V[stored.cpu().numpy()])
                # stored keys as stored: row t of its cache, layer l
                inst = p.oplan["src_inst"]
                for g in np.nonzero(inst >= 0)[0][::17]:
                    s_ = int(p.oplan["inst_src"][inst[g]])
                    want = p.raw[s_][0][l][int(p.oplan["src_row"][g])]
                    assert torch.equal(k_log[g].cpu().view(torch.int16), want.view(torch.int16))
        p.close()
