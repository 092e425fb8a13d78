"""Pins of oracle.rope / oracle.link / oracle.attend (CPU only).

Each test checks the oracle against something other than itself: the complex-number
statement of rotary embedding, group laws, closed forms, a loop transcription of
the attention definition of App. A, and a library SDPA for the case in which every
token is recomputed (which is ordinary causal prefill, Sec. 2.2).
"""
import numpy as np
import pytest
import torch

import workloads
from oracle import (attend, attend_loops, attend_unshifted, build_plan, decode_attend, link_kv, link_kv_unshifted,
                    position_fresh, rotate, to_slots)

RNG = np.random.default_rng(1234)


# ----------------------------------------------------------------- rotation
def _rope_complex(x, pos, theta, interleaved):
    """Textbook RoPE: each coordinate pair is a complex number times exp(i*pos*w)."""
    D = x.shape[-1]
    w = theta ** (-np.arange(0, D, 2, dtype=np.float64) / D)
    if interleaved:
        z = x[..., 0::2] + 1j * x[..., 1::2]
    else:
        z = x[..., : D // 2] + 1j * x[..., D // 2:]
    z = z * np.exp(1j * pos * w)
    y = np.empty_like(x)
    if interleaved:
        y[..., 0::2], y[..., 1::2] = z.real, z.imag
    else:
        y[..., : D // 2], y[..., D // 2:] = z.real, z.imag
    return y


@pytest.mark.parametrize("interleaved", [False, True])
@pytest.mark.parametrize("theta,D", [(1e4, 64), (1e6, 128)])
def test_rotate_matches_complex_form(theta, D, interleaved):
    x = RNG.standard_normal((5, 3, D))
    for pos in (0, 1, 17, 2432, 75839):
        np.testing.assert_allclose(rotate(x, pos, theta, interleaved),
                                   _rope_complex(x, pos, theta, interleaved), rtol=0, atol=1e-11)


@pytest.mark.parametrize("interleaved", [False, True])
def test_rotate_group_laws(interleaved):
    theta, D = 1e4, 64
    x = RNG.standard_normal((4, 2, D))
    assert np.array_equal(rotate(x, 0, theta, interleaved), x)            # zero shift = identity
    ab = rotate(rotate(x, 88, theta, interleaved), 16, theta, interleaved)
    np.testing.assert_allclose(ab, rotate(x, 104, theta, interleaved), atol=1e-12)
    np.testing.assert_allclose(rotate(rotate(x, 7, theta, interleaved), -7, theta, interleaved), x, atol=1e-12)
    y = rotate(x, 1234, theta, interleaved)
    np.testing.assert_allclose((y ** 2).sum(-1), (x ** 2).sum(-1), rtol=1e-12)


def test_rotate_relative_position_law():
    theta, D = 1e6, 128
    q0, k0 = RNG.standard_normal(D), RNG.standard_normal(D)
    ref = rotate(q0, 40, theta) @ rotate(k0, 10, theta)
    for shift in (1, 2304, 70000):
        got = rotate(q0, 40 + shift, theta) @ rotate(k0, 10 + shift, theta)
        assert abs(got - ref) < 1e-9
    # a different relative distance gives a different logit
    assert abs(rotate(q0, 41, theta) @ rotate(k0, 10, theta) - ref) > 1e-6


def test_rotate_per_row_shifts_and_sign():
    theta, D = 1e4, 8
    # e_0 turned by a quarter of the slowest..fastest pair: the fastest pair (i=0) has w=1
    x = np.zeros(D); x[0] = 1.0
    y = rotate(x, np.pi / 2, theta)
    np.testing.assert_allclose(y[[0, D // 2]], [0.0, 1.0], atol=1e-12)   # counter-clockwise
    xs = RNG.standard_normal((3, D))
    ys = rotate(xs, np.array([0.0, 5.0, 9.0]), theta)
    for i, d in enumerate((0.0, 5.0, 9.0)):
        np.testing.assert_allclose(ys[i], rotate(xs[i], d, theta), atol=1e-13)


# ----------------------------------------------------------------- attention
def _tiny_problem(seed=0, hq=4, hkv=2, d=8):
    reqs = [[("text", 3), ("chunk", 0, 6, None), ("text", 2), ("chunk", 1, 5, 3), ("text", 1)],
            [("chunk", 1, 5, None), ("text", 4)]]
    plan = build_plan(reqs, 2)
    rng = np.random.default_rng(seed)
    n, nq = int(plan["ctx_off"][-1]), len(plan["q_pos"])
    q = rng.standard_normal((nq, hq, d))
    k = rng.standard_normal((n, hkv, d))
    v = rng.standard_normal((n, hkv, d))
    return reqs, plan, q, k, v


def test_attend_matches_loop_transcription():
    _, plan, q, k, v = _tiny_problem()
    o, lse = attend(q, k, v, plan, 0.37)
    np.testing.assert_allclose(o, attend_loops(q, k, v, plan, 0.37), rtol=1e-12, atol=1e-13)


def test_attend_tiny_config_matches_loops():
    sh = workloads.shape(1)
    reqs, _, _ = workloads.layout(1)
    plan = build_plan(reqs, sh.default_k)
    rng = np.random.default_rng(5)
    q = rng.standard_normal((48, 4, 64)); k = rng.standard_normal((160, 4, 64)); v = rng.standard_normal((160, 4, 64))
    rows = [0, 23, 24, 39, 47]
    o, _ = attend(q, k, v, plan, sh.softmax_scale, rows=rows)
    ref = attend_loops(q, k, v, plan, sh.softmax_scale)
    np.testing.assert_allclose(o[rows], ref[rows], rtol=1e-12, atol=1e-13)
    assert np.isnan(o[1]).all()


def test_softmax_rows_sum_to_one_and_lse():
    _, plan, q, k, v = _tiny_problem(1)
    ones = np.ones_like(v)
    o, lse = attend(q, k, ones, plan, 0.5)
    np.testing.assert_allclose(o, 1.0, rtol=0, atol=1e-14)
    # LSE against its definition, row by row
    for r in (0, 5, len(q) - 1):
        base = int(plan["ctx_off"][plan["q_req"][r]]); p = int(plan["q_pos"][r])
        s = 0.5 * k[base:base + p + 1, 1] @ q[r, 3]
        assert abs(lse[r, 3] - np.log(np.exp(s).sum())) < 1e-12


def test_weights_exposed_by_one_hot_values_are_causal_by_position():
    reqs, plan, q, k, _ = _tiny_problem(2, hq=2, hkv=2, d=17)
    n = int(plan["ctx_off"][-1])
    # request 0 has 17 positions: value row j = e_j, so the output IS the weight vector
    v = np.zeros((n, 2, 17))
    for j in range(17):
        v[j, :, j] = 1.0
    o, _ = attend(q, k, v, plan, 1.0)
    for r in range(int(plan["q_off"][1])):
        p = int(plan["q_pos"][r])
        w = o[r, 0]
        assert abs(w.sum() - 1.0) < 1e-13 and (w[: p + 1] > 0).all() and (w[p + 1:] == 0).all()
        s = k[: p + 1, 0] @ q[r, 0]
        np.testing.assert_allclose(w[: p + 1], np.exp(s) / np.exp(s).sum(), rtol=1e-12)


def test_zero_queries_give_prefix_means():
    _, plan, q, k, v = _tiny_problem(3)
    o, lse = attend(np.zeros_like(q), k, v, plan, 1.0)
    for r in range(len(q)):
        base = int(plan["ctx_off"][plan["q_req"][r]]); p = int(plan["q_pos"][r])
        np.testing.assert_allclose(o[r, 2], v[base:base + p + 1, 1].mean(0), atol=1e-13)
        assert abs(lse[r, 2] - np.log(p + 1)) < 1e-13


def test_gqa_equals_mha_with_repeated_heads_and_batch_equals_alone():
    reqs, plan, q, k, v = _tiny_problem(4)
    o, lse = attend(q, k, v, plan, 0.3)
    o2, lse2 = attend(q, np.repeat(k, 2, axis=1), np.repeat(v, 2, axis=1), plan, 0.3)
    np.testing.assert_allclose(o, o2, atol=1e-14); np.testing.assert_allclose(lse, lse2, atol=1e-14)
    # second request alone
    p1 = build_plan(reqs[1:], 2)
    c0, q0 = int(plan["ctx_off"][1]), int(plan["q_off"][1])
    o1, _ = attend(q[q0:], k[c0:], v[c0:], p1, 0.3)
    np.testing.assert_allclose(o1, o[q0:], atol=1e-14)


def _sdpa(q, k, v, scale, group):
    """Library causal attention on [n][h][d] tensors, float64."""
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.repeat(k, group, axis=1)).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.repeat(v, group, axis=1)).permute(1, 0, 2)[None]
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
    return o[0].permute(1, 0, 2).numpy()


def test_recompute_everything_is_plain_causal_prefill():
    """k >= L for every chunk: the linked cache is the fresh K/V and the result is
    ordinary causal attention (the arithmetic of prefix caching, Sec. 2.2)."""
    reqs = [[("text", 5), ("chunk", 0, 9, None), ("text", 3), ("chunk", 1, 7, None)]]
    plan = build_plan(reqs, 1000)
    n, hq, hkv, d = 24, 6, 2, 16
    assert len(plan["q_pos"]) == n
    rng = np.random.default_rng(6)
    q, fk, fv = rng.standard_normal((n, hq, d)), rng.standard_normal((n, hkv, d)), rng.standard_normal((n, hkv, d))
    junk = {0: rng.standard_normal((9, hkv, d)), 1: rng.standard_normal((7, hkv, d))}
    K, V = link_kv(plan, junk, junk, fk, fv, 1e4)
    assert np.array_equal(K, fk) and np.array_equal(V, fv)
    o, _ = attend(q, K, V, plan, 0.25)
    np.testing.assert_allclose(o, _sdpa(q, fk, fv, 0.25, hq // hkv), rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("interleaved", [False, True])
@pytest.mark.parametrize("k", [0, 2, 5])
def test_consistent_cache_reproduces_full_prefill(k, interleaved):
    """If the stored chunks and the fresh rows come from the same position-free base
    K0/V0 (stored = rotated at local positions, fresh = rotated at global positions),
    linking rebuilds the full-prefill K/V exactly, so the selected rows of selective
    attention equal the same rows of full causal prefill -- for any k."""
    theta, hq, hkv, d = 1e4, 4, 2, 16
    reqs = [[("text", 4), ("chunk", 0, 8, None), ("text", 3), ("chunk", 1, 6, None), ("text", 2)]]
    plan = build_plan(reqs, k)
    n = int(plan["ctx_off"][-1])
    rng = np.random.default_rng(7)
    k0, v0, q0 = rng.standard_normal((n, hkv, d)), rng.standard_normal((n, hkv, d)), rng.standard_normal((n, hq, d))
    pos = np.arange(n, dtype=np.float64)[:, None]
    k_full = rotate(k0, pos, theta, interleaved)
    q_full = rotate(q0, pos, theta, interleaved)
    chunk_k, chunk_v = {}, {}
    for inst in range(len(plan["inst_src"])):
        off, L, src = int(plan["inst_delta"][inst]), int(plan["inst_len"][inst]), int(plan["inst_src"][inst])
        local = np.arange(L, dtype=np.float64)[:, None]
        chunk_k[src] = rotate(k0[off:off + L], local, theta, interleaved)
        chunk_v[src] = v0[off:off + L]
    sel = plan["q_pos"]
    K, V = link_kv(plan, chunk_k, chunk_v, k_full[sel], v0[sel], theta, interleaved)
    np.testing.assert_allclose(K, k_full, atol=1e-12)
    assert np.array_equal(V, v0)
    o, _ = attend(q_full[sel], K, V, plan, 0.25)
    full = _sdpa(q_full, k_full, v0, 0.25, hq // hkv)
    np.testing.assert_allclose(o, full[sel], rtol=1e-10, atol=1e-11)


@pytest.mark.parametrize("interleaved", [False, True])
def test_pre_rope_fresh_rows_take_their_position_inside_the_request(interleaved):
    """Fresh rows handed over before positional embedding: linking must give every context
    row the rotation of its own position id, counted from the start of *its* request, which
    is what full prefill applies -- checked against the complex-number form of RoPE, row by
    row, on a batch of two requests (so a batch-flattened index or a fresh-row index used as
    the position would show)."""
    theta, hq, hkv, d = 1e4, 4, 2, 16
    reqs = [[("text", 4), ("chunk", 0, 8, None), ("text", 3), ("chunk", 1, 6, None), ("text", 2)],
            [("chunk", 1, 6, None), ("text", 5), ("chunk", 0, 8, 3)]]
    plan = build_plan(reqs, 2)
    n = int(plan["ctx_off"][-1])
    rng = np.random.default_rng(17)
    k0, v0, q0 = rng.standard_normal((n, hkv, d)), rng.standard_normal((n, hkv, d)), rng.standard_normal((n, hq, d))
    # the two requests share their stored chunks, so the position-free base rows of a chunk
    # must agree wherever it appears
    first = {}
    for inst in range(len(plan["inst_src"])):
        src, L = int(plan["inst_src"][inst]), int(plan["inst_len"][inst])
        g0 = int(plan["ctx_off"][plan["inst_req"][inst]]) + int(plan["inst_delta"][inst])
        if src in first:
            k0[g0:g0 + L], v0[g0:g0 + L] = k0[first[src]:first[src] + L], v0[first[src]:first[src] + L]
        else:
            first[src] = g0
    pos = np.concatenate([np.arange(plan["ctx_off"][b + 1] - plan["ctx_off"][b]) for b in range(2)])
    k_full = np.stack([_rope_complex(k0[g], float(pos[g]), theta, interleaved) for g in range(n)])
    q_full = np.stack([_rope_complex(q0[g], float(pos[g]), theta, interleaved) for g in range(n)])
    chunk_k, chunk_v = {}, {}
    for src, g0 in first.items():
        L = 8 if src == 0 else 6
        chunk_k[src] = np.stack([_rope_complex(k0[g0 + t], float(t), theta, interleaved) for t in range(L)])
        chunk_v[src] = v0[g0:g0 + L]
    sel = plan["ctx_off"][plan["q_req"]] + plan["q_pos"]          # batch-flattened rows of the recompute set
    K, V = link_kv(plan, chunk_k, chunk_v, k0[sel], v0[sel], theta, interleaved, fresh_pre_rope=True)
    np.testing.assert_allclose(K, k_full, atol=1e-12)
    assert np.array_equal(V, v0)
    q_rot = position_fresh(q0[sel], plan, theta, interleaved)
    np.testing.assert_allclose(q_rot, q_full[sel], atol=1e-12)
    o, _ = attend(q_rot, K, V, plan, 0.25)
    for b in range(2):
        lo, hi = int(plan["ctx_off"][b]), int(plan["ctx_off"][b + 1])
        full = _sdpa(q_full[lo:hi], k_full[lo:hi], v0[lo:hi], 0.25, hq // hkv)
        rows = np.flatnonzero(plan["q_req"] == b)
        np.testing.assert_allclose(o[rows], full[plan["q_pos"][rows]], rtol=1e-10, atol=1e-11)


def test_pre_rope_logits_depend_on_relative_position_only():
    """<Rot(p) q, Rot(j) k> = <q, Rot(j - p) k>: the logit of a positioned fresh query against a
    positioned fresh key equals the unpositioned query against the key turned by the signed
    distance (a rotation of the query in the wrong direction would fail this)."""
    theta, d = 1e6, 32
    reqs = [[("text", 3), ("chunk", 0, 40, None), ("text", 2)]]
    plan = build_plan(reqs, 4)
    rng = np.random.default_rng(18)
    nq = len(plan["q_pos"])
    q0, k0 = rng.standard_normal((nq, 1, d)), rng.standard_normal((nq, 1, d))
    q, k = position_fresh(q0, plan, theta), position_fresh(k0, plan, theta)
    for r in range(nq):
        for j in range(nq):
            dist = float(plan["q_pos"][j] - plan["q_pos"][r])
            want = q0[r, 0] @ _rope_complex(k0[j, 0], dist, theta, False)
            assert abs(q[r, 0] @ k[j, 0] - want) < 1e-10


def test_link_replaces_rows_and_shifts_by_chunk_offset():
    reqs = [[("text", 2), ("chunk", 3, 4, None), ("chunk", 3, 4, None)]]   # same chunk twice
    plan = build_plan(reqs, 1)
    rng = np.random.default_rng(8)
    ck = {3: rng.standard_normal((4, 1, 8))}; cv = {3: rng.standard_normal((4, 1, 8))}
    fk, fv = rng.standard_normal((4, 1, 8)), rng.standard_normal((4, 1, 8))
    K, V = link_kv(plan, ck, cv, fk, fv, 1e4)
    assert plan["q_pos"].tolist() == [0, 1, 2, 6]
    assert np.array_equal(K[[0, 1, 2, 6]], fk) and np.array_equal(V[[0, 1, 2, 6]], fv)
    np.testing.assert_allclose(K[3:6], rotate(ck[3][1:4], 2, 1e4), atol=0)
    np.testing.assert_allclose(K[7:10], rotate(ck[3][1:4], 6, 1e4), atol=0)
    assert np.array_equal(V[3:6], cv[3][1:4]) and np.array_equal(V[7:10], cv[3][1:4])


def test_to_slots_places_rows():
    x = np.arange(12, dtype=np.float64).reshape(6, 2)
    out = to_slots(x, [4, 5, 0, 1, 8, 9], 12)
    assert np.array_equal(out[[4, 5, 0, 1, 8, 9]], x) and np.isnan(out[[2, 3, 6, 7, 10, 11]]).all()


# ----------------------------------------------------------------- decode step
def test_decode_step_is_the_last_row_of_causal_prefill():
    """Context of N tokens plus the new token = causal prefill of N + 1 tokens, last row
    (library SDPA, float64), for two requests of different length, GQA 3:1."""
    reqs = [[("text", 3), ("chunk", 0, 6, None), ("text", 2)], [("chunk", 1, 5, None), ("text", 4)]]
    plan = build_plan(reqs, 2)
    hq, hkv, d = 6, 2, 8
    rng = np.random.default_rng(21)
    n = int(plan["ctx_off"][-1])
    K, V = rng.standard_normal((n, hkv, d)), rng.standard_normal((n, hkv, d))
    q, nk, nv = rng.standard_normal((2, hq, d)), rng.standard_normal((2, hkv, d)), rng.standard_normal((2, hkv, d))
    o, lse = decode_attend(q, K, V, plan, 0.3, nk, nv)
    for b in range(2):
        lo, hi = int(plan["ctx_off"][b]), int(plan["ctx_off"][b + 1])
        kk, vv = np.concatenate([K[lo:hi], nk[b][None]]), np.concatenate([V[lo:hi], nv[b][None]])
        qq = np.concatenate([rng.standard_normal((hi - lo, hq, d)), q[b][None]])   # earlier rows are irrelevant
        np.testing.assert_allclose(o[b], _sdpa(qq, kk, vv, 0.3, hq // hkv)[-1], rtol=1e-11, atol=1e-12)


def test_decode_step_without_self_equals_attend_row_of_a_final_text_token():
    """A request that ends in a text token: that token is in the recompute set, sees every
    position up to itself, so its row of selective attention equals a decode step over the
    whole context with the same query and no appended token."""
    _, plan, q, k, v = _tiny_problem(seed=3)
    o, lse = attend(q, k, v, plan, 0.37)
    last = [int(plan["q_off"][b + 1]) - 1 for b in range(2)]
    for b in range(2):
        assert plan["q_pos"][last[b]] == plan["ctx_off"][b + 1] - plan["ctx_off"][b] - 1
    od, ld = decode_attend(q[last], k, v, plan, 0.37)
    np.testing.assert_allclose(od, o[last], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(ld, lse[last], rtol=1e-12, atol=1e-13)


def test_decode_step_closed_forms():
    reqs = [[("chunk", 0, 7, None)], [("text", 0)], [("text", 2), ("chunk", 1, 3, None)]]
    plan = build_plan(reqs, 1)
    hq, hkv, d = 4, 4, 8
    rng = np.random.default_rng(22)
    n = int(plan["ctx_off"][-1])
    K, V = rng.standard_normal((n, hkv, d)), rng.standard_normal((n, hkv, d))
    zero_q = np.zeros((3, hq, d))
    o, lse = decode_attend(zero_q, K, V, plan, 1.0)
    np.testing.assert_allclose(o[0], V[:7].mean(axis=0), atol=1e-13)       # uniform weights
    np.testing.assert_allclose(lse[0], np.log(7.0), atol=1e-13)
    assert np.array_equal(o[1], np.zeros((hq, d))) and np.isneginf(lse[1]).all()   # no key at all
    nk, nv = rng.standard_normal((3, hkv, d)), rng.standard_normal((3, hkv, d))
    o2, lse2 = decode_attend(zero_q, K, V, plan, 1.0, nk, nv)
    np.testing.assert_allclose(o2[1], nv[1], atol=1e-13)                   # the token sees only itself
    np.testing.assert_allclose(lse2[:, 0], np.log([8.0, 1.0, 6.0]), atol=1e-13)
    # a key aligned with the query and scaled up takes all the weight
    q = rng.standard_normal((3, hq, d))
    big = K.copy(); big[9] = 50.0 * q[2] / np.linalg.norm(q[2], axis=-1, keepdims=True)
    o3, _ = decode_attend(q, big, V, plan, 1.0)
    np.testing.assert_allclose(o3[2], V[9], atol=1e-6)


# ----------------------------------------------------------------- keys linked without their shift
@pytest.mark.parametrize("interleaved", [False, True])
def test_turning_the_query_back_equals_turning_the_key_forward(interleaved):
    """<Rot(-D) q, k> = <q, Rot(D) k>, per head, for the shifts of real layouts; the left side
    also against the complex-number form of RoPE (conjugate phase on the query)."""
    theta, D = 1e6, 128
    q = RNG.standard_normal((6, D))
    k = RNG.standard_normal((6, D))
    for delta in (0, 1, 128, 2560, 19584, 75776):
        lhs = np.einsum("id,id->i", rotate(q, -delta, theta, interleaved), k)
        rhs = np.einsum("id,id->i", q, rotate(k, delta, theta, interleaved))
        assert np.abs(lhs - rhs).max() < 1e-10
        ref = np.einsum("id,id->i", _rope_complex(q, -delta, theta, interleaved), k)
        assert np.abs(lhs - ref).max() < 1e-10
    # the sign matters: turning the query forward instead is a different number
    wrong = np.einsum("id,id->i", rotate(q, 2560, theta, interleaved), k)
    assert np.abs(wrong - np.einsum("id,id->i", q, rotate(k, 2560, theta, interleaved))).max() > 1e-3


@pytest.mark.parametrize("interleaved,pre_rope", [(False, False), (True, False), (False, True)])
def test_unshifted_link_and_attend_equal_shifted_link_and_attend(interleaved, pre_rope):
    """Leaving stored keys as stored and turning each query back per chunk instance gives the
    outputs of the linked-and-shifted context: same chunk twice, adjacent chunks, k = 0 and
    k beyond the chunk, two requests."""
    theta, hq, hkv, d = 5e5, 4, 2, 16
    reqs = [[("text", 3), ("chunk", 0, 9, None), ("chunk", 1, 5, 0), ("text", 2), ("chunk", 0, 9, 4), ("text", 1)],
            [("chunk", 1, 5, 9), ("chunk", 0, 9, None), ("text", 4)]]
    plan = build_plan(reqs, 2)
    ck = {0: RNG.standard_normal((9, hkv, d)), 1: RNG.standard_normal((5, hkv, d))}
    cv = {0: RNG.standard_normal((9, hkv, d)), 1: RNG.standard_normal((5, hkv, d))}
    nq = int(plan["q_off"][-1])
    q, fk, fv = (RNG.standard_normal((nq, h, d)) for h in (hq, hkv, hkv))
    K, V = link_kv(plan, ck, cv, fk, fv, theta, interleaved, pre_rope)
    qq = position_fresh(q, plan, theta, interleaved) if pre_rope else q
    O, L = attend(qq, K, V, plan, 0.25)
    K0, V0, shift = link_kv_unshifted(plan, ck, cv, fk, fv, theta, interleaved, pre_rope)
    assert np.array_equal(V0, V)
    stored = plan["src_inst"] >= 0
    assert np.array_equal(K0[~stored], K[~stored])                       # fresh rows are the same rows
    assert np.array_equal(shift[stored], plan["inst_delta"][plan["src_inst"][stored]]) and not shift[~stored].any()
    for g in np.nonzero(stored)[0]:                                      # stored rows: exactly as stored
        i = int(plan["src_inst"][g])
        assert np.array_equal(K0[g], ck[int(plan["inst_src"][i])][int(plan["src_row"][g])])
    O0, L0 = attend_unshifted(qq, K0, V0, shift, plan, theta, 0.25, interleaved)
    assert np.abs(O0 - O).max() < 1e-11 and np.abs(L0 - L).max() < 1e-11
