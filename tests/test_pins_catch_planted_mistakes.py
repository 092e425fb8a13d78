"""Do the pins of the oracle bite?  (CPU only.)

Every case below plants one plausible mistake in a *copy* of an oracle module (a wrong sign, a
dropped term, a wrong index, an operand taken from the wrong tensor, an off-by-one at the causal
boundary ...), lets the pin tests of that module run against the copy and expects at least one of
them to fail.  The oracle itself is never changed: the copy is compiled from the module's source
text with one line replaced and is bound into the pin tests' namespace for the duration of the case.
"""
import inspect
import types

import pytest

import importlib

import oracle.decode
import oracle.link
import oracle.plan
import oracle.rope
import oracle.select
import oracle.store
import test_oracle_math as M
import test_oracle_plan as P
import test_oracle_select as S
import test_oracle_store as T


ATTEND = importlib.import_module("oracle.attend")   # (the package binds the name `attend` to the function)


def _mutant(module, old, new):
    src = inspect.getsource(module)
    assert src.count(old) == 1, f"{module.__name__}: pattern must occur exactly once: {old!r}"
    ns = types.ModuleType(module.__name__ + "_with_mistake")
    ns.__package__ = module.__package__
    ns.__file__ = module.__file__
    exec(compile(src.replace(old, new), module.__file__, "exec"), ns.__dict__)
    return ns


def _golden(cfg):
    return next(r for r in P._golden_rows() if r[0] == cfg)


# pin tests per oracle module, as argument-free callables
ROPE_PINS = [lambda: M.test_rotate_matches_complex_form(1e4, 64, False),
             lambda: M.test_rotate_matches_complex_form(1e6, 128, True),
             lambda: M.test_rotate_group_laws(False), lambda: M.test_rotate_group_laws(True),
             M.test_rotate_relative_position_law, M.test_rotate_per_row_shifts_and_sign]
LINK_PINS = [lambda: M.test_consistent_cache_reproduces_full_prefill(8, False),
             lambda: M.test_consistent_cache_reproduces_full_prefill(0, True),
             lambda: M.test_pre_rope_fresh_rows_take_their_position_inside_the_request(False),
             M.test_pre_rope_logits_depend_on_relative_position_only,
             M.test_link_replaces_rows_and_shifts_by_chunk_offset, M.test_to_slots_places_rows]
ATTEND_PINS = [M.test_attend_matches_loop_transcription, M.test_attend_tiny_config_matches_loops,
               M.test_softmax_rows_sum_to_one_and_lse, M.test_weights_exposed_by_one_hot_values_are_causal_by_position,
               M.test_zero_queries_give_prefix_means, M.test_gqa_equals_mha_with_repeated_heads_and_batch_equals_alone,
               M.test_recompute_everything_is_plain_causal_prefill]
DECODE_PINS = [M.test_decode_step_is_the_last_row_of_causal_prefill,
               M.test_decode_step_without_self_equals_attend_row_of_a_final_text_token,
               M.test_decode_step_closed_forms]
PLAN_PINS = [P.test_tiny_config_by_hand, lambda: P.test_closed_form_counts(*_golden(2)),
             lambda: P.test_closed_form_counts(*_golden(3)), P.test_explicit_token_sets_by_hand,
             P.test_missing_chunk_equals_text, P.test_k_zero_and_no_text_gives_empty_set]
SELECT_PINS = [S.test_k_distance_matches_loops_and_closed_forms, S.test_ranking_by_hand]


def _bites(pins):
    """Number of pins that fail (an assertion, or an exception the mistake provokes)."""
    failed = 0
    for pin in pins:
        try:
            pin()
        except (Exception, pytest.fail.Exception):      # noqa: BLE001 -- any failure of a pin counts
            failed += 1
    return failed


ROPE_MISTAKES = [
    ("turns the wrong way", "y[..., :half] = a * c - b * s\n        y[..., half:] = a * s + b * c",
     "y[..., :half] = a * c + b * s\n        y[..., half:] = -a * s + b * c"),
    ("half the frequency exponent", "theta ** (-2.0 * i / D)", "theta ** (-1.0 * i / D)"),
    ("dropped term", "y[..., half:] = a * s + b * c", "y[..., half:] = b * c"),
    ("same sign in both rows", "y[..., 0::2] = a * c - b * s", "y[..., 0::2] = a * c + b * s"),
    ("pairings swapped", "if interleaved:\n        a, b = x[..., 0::2], x[..., 1::2]", "if not interleaved:\n        a, b = x[..., 0::2], x[..., 1::2]"),
    ("cosine and sine swapped", "c, s = np.cos(phi), np.sin(phi)", "s, c = np.cos(phi), np.sin(phi)"),
]


@pytest.mark.parametrize("what,old,new", ROPE_MISTAKES, ids=[m[0] for m in ROPE_MISTAKES])
def test_rotation_pins(monkeypatch, what, old, new):
    bad = _mutant(oracle.rope, old, new)
    monkeypatch.setattr(M, "rotate", bad.rotate)
    monkeypatch.setattr(oracle.link, "rotate", bad.rotate)
    assert _bites(ROPE_PINS) >= 1, what


LINK_MISTAKES = [
    ("stored keys not shifted", "shift = float(plan[\"inst_delta\"][inst])", "shift = 0.0"),
    ("shift by the chunk's index instead of its offset", "shift = float(plan[\"inst_delta\"][inst])", "shift = float(inst)"),
    ("shift off by one", "shift = float(plan[\"inst_delta\"][inst])", "shift = float(plan[\"inst_delta\"][inst]) + 1.0"),
    ("shift with the wrong sign", "shift = float(plan[\"inst_delta\"][inst])", "shift = -float(plan[\"inst_delta\"][inst])"),
    ("values shifted too", "V[g] = np.asarray(chunk_v[src][row], dtype=np.float64)",
     "V[g] = rotate(np.asarray(chunk_v[src][row], dtype=np.float64), shift, theta, interleaved)"),
    ("value taken from the key cache", "V[g] = np.asarray(chunk_v[src][row], dtype=np.float64)",
     "V[g] = np.asarray(chunk_k[src][row], dtype=np.float64)"),
    ("fresh row index taken as a position", "K[g] = fresh_k[row]", "K[g] = fresh_k[min(g, len(fresh_k) - 1)]"),
    ("fresh rows positioned by their row number", "pos = np.asarray(plan[\"q_pos\"], dtype=np.float64)",
     "pos = np.arange(len(plan[\"q_pos\"]), dtype=np.float64)"),
]


@pytest.mark.parametrize("what,old,new", LINK_MISTAKES, ids=[m[0] for m in LINK_MISTAKES])
def test_linking_pins(monkeypatch, what, old, new):
    bad = _mutant(oracle.link, old, new)
    monkeypatch.setattr(M, "link_kv", bad.link_kv)
    monkeypatch.setattr(M, "position_fresh", bad.position_fresh)
    monkeypatch.setattr(M, "to_slots", bad.to_slots)
    assert _bites(LINK_PINS) >= 1, what


UNSHIFTED_PINS = [lambda: M.test_unshifted_link_and_attend_equal_shifted_link_and_attend(False, False),
                  lambda: M.test_unshifted_link_and_attend_equal_shifted_link_and_attend(True, False),
                  lambda: M.test_unshifted_link_and_attend_equal_shifted_link_and_attend(False, True)]
UNSHIFTED_LINK_MISTAKES = [
    ("the shift a key lacks is its chunk's index", "shift[pos] = int(plan[\"inst_delta\"][i])", "shift[pos] = i"),
    ("fresh rows marked as lacking a shift", "shift = np.zeros(n, dtype=np.int64)", "shift = np.full(n, 5, dtype=np.int64)"),
    ("stored value taken from the key cache", "K[pos], V[pos] = chunk_k[cache][r], chunk_v[cache][r]",
     "K[pos], V[pos] = chunk_k[cache][r], chunk_k[cache][r]"),
]
UNSHIFTED_ATTEND_MISTAKES = [
    ("query turned forward instead of back", "qt = rotate(q[r], -float(dlt), theta, interleaved)", "qt = rotate(q[r], float(dlt), theta, interleaved)"),
    ("query never turned", "qt = rotate(q[r], -float(dlt), theta, interleaved)", "qt = q[r]"),
    ("one key too few", "n_keys = int(plan[\"q_pos\"][r]) + 1", "n_keys = max(1, int(plan[\"q_pos\"][r]))"),
    ("kv head by remainder", "k_ctx[base + at, h // group, :] @ qt[h]", "k_ctx[base + at, h % k_ctx.shape[1], :] @ qt[h]"),
    ("scale dropped", "s[h, at] = scale * (", "s[h, at] = 1.0 * ("),
]


@pytest.mark.parametrize("what,old,new", UNSHIFTED_LINK_MISTAKES, ids=[m[0] for m in UNSHIFTED_LINK_MISTAKES])
def test_unshifted_linking_pins(monkeypatch, what, old, new):
    bad = _mutant(oracle.link, old, new)
    monkeypatch.setattr(M, "link_kv_unshifted", bad.link_kv_unshifted)
    assert _bites(UNSHIFTED_PINS) >= 1, what


@pytest.mark.parametrize("what,old,new", UNSHIFTED_ATTEND_MISTAKES, ids=[m[0] for m in UNSHIFTED_ATTEND_MISTAKES])
def test_unshifted_attention_pins(monkeypatch, what, old, new):
    bad = _mutant(ATTEND, old, new)
    monkeypatch.setattr(M, "attend_unshifted", bad.attend_unshifted)
    assert _bites(UNSHIFTED_PINS) >= 1, what


ATTEND_MISTAKES = [
    ("a token does not see itself", "> pos[:, None]", ">= pos[:, None]"),
    ("a token sees one key too many", "np.arange(n_keys)[None, :] > pos[:, None]", "np.arange(n_keys)[None, :] > pos[:, None] + 1"),
    ("kv head by remainder", "g = h // group\n            s = scale", "g = h % k_ctx.shape[1]\n            s = scale"),
    ("scale dropped", "s = scale * (q[sel, h, :] @", "s = 1.0 * (q[sel, h, :] @"),
    ("weights applied to the keys", "(w @ v_ctx[base:base + n_keys, g, :]) / z", "(w @ k_ctx[base:base + n_keys, g, :]) / z"),
    ("not normalised", "(w @ v_ctx[base:base + n_keys, g, :]) / z", "(w @ v_ctx[base:base + n_keys, g, :])"),
    ("log-sum-exp without the maximum", "lse[sel, h] = (m + np.log(z))[:, 0]", "lse[sel, h] = (np.log(z))[:, 0]"),
    ("positions of another request", "base = int(plan[\"ctx_off\"][b])\n        pos", "base = 0\n        pos"),
]


@pytest.mark.filterwarnings("ignore::RuntimeWarning")
@pytest.mark.parametrize("what,old,new", ATTEND_MISTAKES, ids=[m[0] for m in ATTEND_MISTAKES])
def test_attention_pins(monkeypatch, what, old, new):
    bad = _mutant(ATTEND, old, new)
    monkeypatch.setattr(M, "attend", bad.attend)
    assert _bites(ATTEND_PINS) >= 1, what


DECODE_MISTAKES = [
    ("scale dropped", "s = scale * (keys @ q[b, h])", "s = keys @ q[b, h]"),
    ("kv head by remainder", "g = h // group", "g = h % k_ctx.shape[1]"),
    ("own value left out", "vals = np.concatenate([vals, np.asarray(new_v, dtype=np.float64)[b, g][None, :]])",
     "vals = np.concatenate([vals, np.zeros((1, d))])"),
    ("context of the first request for all", "lo, hi = int(plan[\"ctx_off\"][b]), int(plan[\"ctx_off\"][b + 1])",
     "lo, hi = int(plan[\"ctx_off\"][0]), int(plan[\"ctx_off\"][1])"),
    ("last context row not read", "keys, vals = k_ctx[lo:hi, g, :], v_ctx[lo:hi, g, :]", "keys, vals = k_ctx[lo:hi - 1, g, :], v_ctx[lo:hi - 1, g, :]"),
    ("log-sum-exp without the maximum", "lse[b, h] = m + np.log(z)", "lse[b, h] = np.log(z)"),
]


@pytest.mark.parametrize("what,old,new", DECODE_MISTAKES, ids=[m[0] for m in DECODE_MISTAKES])
def test_decode_pins(monkeypatch, what, old, new):
    bad = _mutant(oracle.decode, old, new)
    monkeypatch.setattr(M, "decode_attend", bad.decode_attend)
    assert _bites(DECODE_PINS) >= 1, what


PLAN_MISTAKES = [
    ("one token too many per chunk", "chosen = set(range(min(k, L)))", "chosen = set(range(min(k + 1, L)))"),
    ("k not clipped to the chunk", "chosen = set(range(min(k, L)))", "chosen = set(range(k))"),
    ("text tokens not selected", "for t in range(L):\n                    selected.add(off + t)", "for t in range(0):\n                    selected.add(off + t)"),
    ("shift counts chunks, not tokens", "inst_delta.append(off)", "inst_delta.append(len(inst_src) - 1)"),
    ("stored row by position, not by chunk-local index", "owner[off + t] = (inst, t)", "owner[off + t] = (inst, off + t)"),
    ("runs never merged", "if i > 0 and order[i - 1] == p - 1:", "if False:"),
    ("fresh rows numbered per request", "row_of = {p: q_off[-1] + i for i, p in enumerate(order)}", "row_of = {p: i for i, p in enumerate(order)}"),
    ("page offset dropped", "* page_size + p % page_size", "* page_size"),
    ("page table of the first request for all", "int(page_tables[b][p // page_size])", "int(page_tables[0][p // page_size])"),
    ("effective k counts the set, not its leading run", "k_eff = 0\n                while k_eff in chosen:\n                    k_eff += 1",
     "k_eff = len(chosen)"),
    ("slot of a fresh row taken from the first request", "slot_map.append(dst_slot[ctx_off[-1] + p])", "slot_map.append(dst_slot[p])"),
]
BATCH_OR_PAGED = {"fresh rows numbered per request", "page offset dropped", "page table of the first request for all",
                  "effective k counts the set, not its leading run", "slot of a fresh row taken from the first request"}


@pytest.mark.parametrize("what,old,new", PLAN_MISTAKES, ids=[m[0] for m in PLAN_MISTAKES])
def test_plan_pins(monkeypatch, what, old, new):
    bad = _mutant(oracle.plan, old, new)
    monkeypatch.setattr(P, "build_plan", bad.build_plan)
    pins = list(PLAN_PINS)
    if what in BATCH_OR_PAGED:   # needs a batch, pages or an explicit token set: the brute-force construction on random layouts
        pins += [P.test_random_layouts, P.test_random_layouts_paged]
    assert _bites(pins) >= 1, what


SELECT_MISTAKES = [
    ("squared distance", "np.abs(a - b).sum(axis=(1, 2))", "((a - b) ** 2).sum(axis=(1, 2))"),
    ("heads not summed", "np.abs(a - b).sum(axis=(1, 2))", "np.abs(a - b).sum(axis=2)[:, 0]"),
    ("signed difference", "np.abs(a - b).sum(axis=(1, 2))", "np.abs((a - b).sum(axis=(1, 2)))"),
    ("smallest distance first", "key=lambda t: (-dist[t], t)", "key=lambda t: (dist[t], t)"),
    ("ties to the higher index", "key=lambda t: (-dist[t], t)", "key=lambda t: (-dist[t], -t)"),
    ("one token too many", "order[:max(0, min(n_top, len(dist)))]", "order[:max(0, min(n_top + 1, len(dist)))]"),
]


@pytest.mark.parametrize("what,old,new", SELECT_MISTAKES, ids=[m[0] for m in SELECT_MISTAKES])
def test_selection_pins(monkeypatch, what, old, new):
    bad = _mutant(oracle.select, old, new)
    for name in ("k_distance", "top_tokens", "top_counts"):
        monkeypatch.setattr(S, name, getattr(bad, name))
    assert _bites(SELECT_PINS) >= 1, what


STORE_MISTAKES = [
    ("powers start at P^0", "powers = np.multiply.accumulate(np.full(w.size, P, dtype=np.uint64))",
     "powers = np.multiply.accumulate(np.full(w.size, P, dtype=np.uint64)) * pow(P, -1, 1 << 64)"),
    ("word count left out", "return (int(total) + w.size) & MASK", "return int(total) & MASK"),
    ("plain sum of the words", "total = np.add.reduce(w.astype(np.uint64) * powers, dtype=np.uint64)",
     "total = np.add.reduce(w.astype(np.uint64), dtype=np.uint64)"),
    ("sums of K and V swapped in the table", "struct.pack(\"<QQ\", checksum(k[layer].tobytes()), checksum(v[layer].tobytes()))",
     "struct.pack(\"<QQ\", checksum(v[layer].tobytes()), checksum(k[layer].tobytes()))"),
    ("header sum not checked", "if struct.unpack(\"<Q\", raw[56:64])[0] != checksum(raw[:56]):", "if False:"),
    ("block sums not checked", "if checksum(kb) != want_k or checksum(vb) != want_v:", "if False:"),
    ("file size not checked", "or len(raw) != payload_off + 2 * n_layers * block:", ":"),
    ("expiry time itself survives", "if 0 <= e[\"expires_at\"] <= now)", "if 0 <= e[\"expires_at\"] < now)"),
    ("caches kept for ever expire", "if 0 <= e[\"expires_at\"] <= now)", "if e[\"expires_at\"] <= now)"),
    ("length of a layer, not of the cache", "self.entries[i][\"k\"].shape[1] if i in self.entries else 0",
     "self.entries[i][\"k\"].shape[0] if i in self.entries else 0"),
]


@pytest.mark.parametrize("what,old,new", STORE_MISTAKES, ids=[m[0] for m in STORE_MISTAKES])
def test_store_pins(monkeypatch, tmp_path, what, old, new):
    bad = _mutant(oracle.store, old, new)
    for name in ("checksum", "write_chunk_file", "read_chunk_file", "ChunkStore"):
        monkeypatch.setattr(T, name, getattr(bad, name))
    dirs = iter(tmp_path / f"d{i}" for i in range(8))

    def fresh_dir():
        d = next(dirs)
        d.mkdir()
        return d
    pins = [T.test_checksum_against_exact_integers, T.test_checksum_sees_every_single_byte_change_and_word_swaps,
            lambda: T.test_file_layout_by_hand(fresh_dir()), lambda: T.test_every_corruption_of_a_small_file_is_refused(fresh_dir()),
            T.test_library_returns_what_it_was_given_until_expiry]
    assert _bites(pins) >= 1, what


PIPELINE_MISTAKES = [
    ("a missing cache is still read", "if seg[0] == \"chunk\" and (place[seg[1]] == MISSING or ids[seg[1]] in failed):",
     "if seg[0] == \"chunk\" and ids[seg[1]] in failed:"),
    ("a failed load is still read", "if seg[0] == \"chunk\" and (place[seg[1]] == MISSING or ids[seg[1]] in failed):",
     "if seg[0] == \"chunk\" and place[seg[1]] == MISSING:"),
    ("every layer reads layer 0", "k_l, v_l = store.layer(ids[s], layer)", "k_l, v_l = store.layer(ids[s], 0)"),
    ("fresh rows of layer 0 for every layer", "q, fk, fv = fresh(layer)", "q, fk, fv = fresh(0)"),
    ("a missing chunk recomputes one token too few", "seg = (\"chunk\", seg[1], seg[2], seg[2])", "seg = (\"chunk\", seg[1], seg[2], seg[2] - 1)"),
]


@pytest.mark.parametrize("what,old,new", PIPELINE_MISTAKES, ids=[m[0] for m in PIPELINE_MISTAKES])
def test_pipeline_pins(monkeypatch, what, old, new):
    import oracle.pipeline
    bad = _mutant(oracle.pipeline, old, new)
    monkeypatch.setattr(T, "plan_with_lookup", bad.plan_with_lookup)
    monkeypatch.setattr(T, "prefill_layers", bad.prefill_layers)
    pins = [T.test_missing_cache_is_planned_like_text, T.test_all_caches_missing_is_full_causal_prefill_of_every_layer,
            T.test_layers_use_their_own_slice_of_every_cache]
    assert _bites(pins) >= 1, what
