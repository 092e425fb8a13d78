"""Are the parity gates tight enough?  (CPU only.)

The GPU tests compare the library with the float64 oracle through assert_bf16_close (max-abs
2e-2, mean-abs 2e-3 per tensor) on problems like the one below.  Here the place of the library is
taken by the oracle itself with its results rounded to bf16 -- which must pass the gates, as a
correct kernel does -- and then by copies of the oracle with one planted mistake each, which must
not: a gate that lets a wrong causal boundary or a missing rotation through would prove nothing.
Mistakes are planted in copies of the oracle's modules, on the CPU; the oracle is not changed.
"""
import numpy as np
import pytest
import torch

import oracle.link
from helpers import Problem, assert_bf16_close
from test_pins_catch_planted_mistakes import ATTEND, ATTEND_MISTAKES, LINK_MISTAKES, ROPE_MISTAKES, _mutant


def _bf16(x):
    """Round to bf16 (nearest even) and back, as a kernel that stores bf16 does."""
    return torch.from_numpy(np.asarray(x)).to(torch.bfloat16).to(torch.float64).numpy()


@pytest.fixture(scope="module")
def problem():
    # ragged chunks, two requests, grouped heads: the shape of a GPU parity case
    p = Problem(3, n_chunks=3, chunk_len=301, text_len=37, batch=2)
    K, V = p.oracle_link()
    O, L = p.oracle_attend(K, V)
    return p, K, V, O, L


def test_a_correct_result_rounded_to_bf16_passes(problem):
    p, K, V, O, L = problem
    assert_bf16_close(_bf16(K), K, "K context")
    assert np.array_equal(_bf16(V), V)                     # values are copies of bf16 inputs: exact
    assert_bf16_close(_bf16(O), O, "attention output")


def _link_with(p, module):
    f64 = lambda t: t.to(torch.float64).numpy()
    ck = {s: f64(kv[0]) for s, kv in p.chunks.items()}
    cv = {s: f64(kv[1]) for s, kv in p.chunks.items()}
    return module.link_kv(p.oplan, ck, cv, f64(p.fresh_k), f64(p.fresh_v), p.sh.rope_theta, p.interleaved, p.pre_rope)


ROTARY = [m for m in ROPE_MISTAKES if m[0] not in ("pairings swapped", "same sign in both rows")]   # (those two: interleaved pairing only)


@pytest.mark.parametrize("what,old,new", ROTARY, ids=[m[0] for m in ROTARY])
def test_gate_of_the_linked_keys_sees_a_wrong_rotation(problem, monkeypatch, what, old, new):
    p, K, V, O, L = problem
    import oracle.rope
    monkeypatch.setattr(oracle.link, "rotate", _mutant(oracle.rope, old, new).rotate)
    K_bad, _ = _link_with(p, oracle.link)
    with pytest.raises(AssertionError):
        assert_bf16_close(_bf16(K_bad), K, "K context")


LINKING = [m for m in LINK_MISTAKES if m[0] != "fresh rows positioned by their row number"]   # (pre-rope mode only)


@pytest.mark.parametrize("what,old,new", LINKING, ids=[m[0] for m in LINKING])
def test_gates_of_the_linked_context_see_a_wrong_link(problem, what, old, new):
    p, K, V, O, L = problem
    K_bad, V_bad = _link_with(p, _mutant(oracle.link, old, new))
    ok = True
    try:
        assert_bf16_close(_bf16(K_bad), K, "K context")
        assert np.array_equal(_bf16(V_bad), V), "V context"
    except AssertionError:
        ok = False
    assert not ok, what


@pytest.mark.filterwarnings("ignore::RuntimeWarning")
@pytest.mark.parametrize("what,old,new", ATTEND_MISTAKES, ids=[m[0] for m in ATTEND_MISTAKES])
def test_gates_of_the_attention_output_see_a_wrong_attention(problem, what, old, new):
    p, K, V, O, L = problem
    q = p.q.to(torch.float64).numpy()
    O_bad, L_bad = _mutant(ATTEND, old, new).attend(q, K, V, p.oplan, p.sh.softmax_scale)
    ok = True
    try:
        assert_bf16_close(_bf16(O_bad), O, "attention output")
        assert np.abs(L_bad.astype(np.float32).astype(np.float64) - L).max() < 2e-2, "log-sum-exp"
    except AssertionError:
        ok = False
    assert not ok, what
