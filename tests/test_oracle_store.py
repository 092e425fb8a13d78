"""Pins of oracle.store and oracle.pipeline (CPU only): the checksum and file layout against
exact integer arithmetic and exhaustive corruption of a small file, the library's expiry
rule, and the layer loop against full causal prefill and the text-segment equivalence."""
import struct

import numpy as np
import pytest
import torch

from oracle import build_plan
from oracle.pipeline import plan_with_lookup, prefill_layers
from oracle.store import (DISK, HBM, HOST, MISSING, P, ChunkStore, checksum, file_name, read_chunk_file,
                          write_chunk_file)


def test_checksum_against_exact_integers():
    rng = np.random.default_rng(3)
    words = rng.integers(0, 2**63, size=37, dtype=np.uint64) * 2 + rng.integers(0, 2, size=37, dtype=np.uint64)
    exact = len(words)
    for i, w in enumerate(words.tolist()):
        exact += w * pow(P, i + 1)                 # unbounded Python integers, reduced once at the end
    assert checksum(words.tobytes()) == exact % 2**64
    assert checksum(b"") == 0
    assert checksum(bytes(8)) == 1 and checksum(bytes(16)) == 2      # zero words: only the count is left
    assert checksum(struct.pack("<Q", 1)) == (1 + P) % 2**64


def test_checksum_sees_every_single_byte_change_and_word_swaps():
    rng = np.random.default_rng(4)
    data = bytearray(rng.integers(0, 256, size=96, dtype=np.uint8).tobytes())
    ref = checksum(bytes(data))
    for at in range(len(data)):
        for flip in (1, 0x80, 0xFF):
            data[at] ^= flip
            assert checksum(bytes(data)) != ref, at
            data[at] ^= flip
    w = np.frombuffer(bytes(data), dtype="<u8").copy()
    for i in range(len(w) - 1):
        s = w.copy()
        s[i], s[i + 1] = s[i + 1], s[i]
        assert checksum(s.tobytes()) != ref
    assert checksum(bytes(data) + bytes(8)) != ref                  # appended zeros are seen


def _tiny_cache(seed, n_layers=2, length=3, n_kv=2, d=4, dtype=np.uint16):
    rng = np.random.default_rng(seed)
    hi = 2**16 if dtype == np.uint16 else 2**32
    shape = (n_layers, length, n_kv, d)
    return rng.integers(0, hi, size=shape).astype(dtype), rng.integers(0, hi, size=shape).astype(dtype)


def test_file_layout_by_hand(tmp_path):
    k, v = _tiny_cache(1)
    path = tmp_path / file_name(0xABC)
    assert path.name == "0000000000000abc.mpickv"
    write_chunk_file(path, 0xABC, k, v, 1)
    raw = path.read_bytes()
    block = 3 * 2 * 4 * 2
    assert raw[:8] == b"MPICKV01"
    assert struct.unpack("<Q", raw[8:16])[0] == 0xABC
    assert struct.unpack("<6i", raw[16:40]) == (3, 2, 2, 4, 1, 0)
    assert struct.unpack("<QQ", raw[40:56]) == (block, 4096)
    assert len(raw) == 4096 + 2 * 2 * block
    assert raw[4096:4096 + block] == k[0].tobytes() and raw[4096 + block:4096 + 2 * block] == v[0].tobytes()
    assert raw[4096 + 2 * block:4096 + 3 * block] == k[1].tobytes()
    assert set(raw[64 + 32:4096]) == {0}
    cid, dt, ks, vs, dims = read_chunk_file(path)
    assert (cid, dt, dims) == (0xABC, 1, (3, 2, 4))
    assert ks == [k[0].tobytes(), k[1].tobytes()] and vs == [v[0].tobytes(), v[1].tobytes()]


def test_every_corruption_of_a_small_file_is_refused(tmp_path):
    k, v = _tiny_cache(2)
    path = tmp_path / "c.mpickv"
    write_chunk_file(path, 7, k, v, 1)
    good = path.read_bytes()
    meaningful = list(range(0, 64 + 32)) + list(range(4096, len(good)))
    for at in meaningful:
        bad = bytearray(good)
        bad[at] ^= 0x10
        path.write_bytes(bytes(bad))
        with pytest.raises(ValueError):
            read_chunk_file(path)
    for cut in (0, 63, 64, 4096, len(good) - 1):
        path.write_bytes(good[:cut])
        with pytest.raises(ValueError):
            read_chunk_file(path)
    path.write_bytes(good + b"\0")
    with pytest.raises(ValueError):
        read_chunk_file(path)
    path.write_bytes(good)
    read_chunk_file(path)


def test_library_returns_what_it_was_given_until_expiry():
    st = ChunkStore()
    k, v = _tiny_cache(3)
    st.put(10, k, v, HBM)                      # kept for ever
    st.put(11, k + 1, v + 1, HOST, expires_at=100)
    st.put(12, k + 2, v + 2, DISK, expires_at=50)
    k[:] = 0                                   # the library holds its own copy
    assert st.lookup([10, 11, 12, 13]) == ([HBM, HOST, DISK, MISSING], [3, 3, 3, 0])
    assert st.expire(49) == []
    assert st.expire(50) == [12]               # the expiry time itself counts as expired
    assert st.lookup([12])[0] == [MISSING]
    st.move(11, DISK)
    assert st.lookup([11])[0] == [DISK]
    assert np.array_equal(st.layer(11, 1)[0], _tiny_cache(3)[0][1] + 1)
    assert st.expire(10**9) == [11] and st.lookup([10])[0] == [HBM]
    st.put(10, v, v, HOST)                     # put replaces
    assert np.array_equal(st.layer(10, 0)[0], v[0]) and st.lookup([10])[0] == [HOST]


def _layered_problem(seed, n_layers=3):
    rng = np.random.default_rng(seed)
    hq, hkv, d = 4, 2, 8
    lens = {0: 6, 1: 5, 2: 7}
    st = ChunkStore()
    ids = [100, 101, 102]
    for s, cid in enumerate(ids):
        st.put(cid, rng.standard_normal((n_layers, lens[s], hkv, d)), rng.standard_normal((n_layers, lens[s], hkv, d)),
               (HBM, HOST, DISK)[s])
    requests = [[("text", 3), ("chunk", 0, 6, None), ("text", 2), ("chunk", 1, 5, None), ("text", 1)],
                [("chunk", 2, 7, None), ("chunk", 0, 6, 1), ("text", 4)]]
    return st, ids, requests, (hq, hkv, d), rng


def _fresh_fn(plan, dims, seed):
    hq, hkv, d = dims
    nq = int(plan["q_off"][-1])

    def fresh(layer):
        r = np.random.default_rng((seed, layer))
        return r.standard_normal((nq, hq, d)), r.standard_normal((nq, hkv, d)), r.standard_normal((nq, hkv, d))
    return fresh


def test_missing_cache_is_planned_like_text():
    st, ids, requests, dims, _ = _layered_problem(5)
    st.drop(101)
    plan, used = plan_with_lookup(requests, ids, 2, st)
    as_text = [[("text", seg[2]) if seg[0] == "chunk" and seg[1] == 1 else seg for seg in r] for r in requests]
    ref = build_plan(as_text, 2)
    for f in ("q_pos", "q_req", "q_off", "ctx_off", "slot_map", "dst_slot", "runs"):
        assert np.array_equal(plan[f], ref[f]), f
    # same thing when the cache is there but its load failed
    st2, ids2, _, _, _ = _layered_problem(5)
    plan2, _ = plan_with_lookup(requests, ids2, 2, st2, failed={101})
    assert np.array_equal(plan2["q_pos"], ref["q_pos"])
    # and the results: chunk 1's stored rows are never read, its fresh rows are
    fresh = _fresh_fn(plan, dims, 9)
    a = prefill_layers(plan, ids, st, 2, fresh, 1e4, 0.3)
    st.put(101, np.full((3, 5, 2, 8), np.nan), np.full((3, 5, 2, 8), np.nan), DISK)
    b = prefill_layers(plan, ids, st, 2, fresh, 1e4, 0.3)
    for (K1, V1, O1, L1), (K2, V2, O2, L2) in zip(a, b):
        assert np.array_equal(O1, O2) and np.array_equal(K1, K2) and not np.isnan(O1).any()


def test_all_caches_missing_is_full_causal_prefill_of_every_layer():
    st, ids, requests, dims, _ = _layered_problem(6)
    empty = ChunkStore()
    plan, _ = plan_with_lookup(requests, ids, 0, empty)
    hq, hkv, d = dims
    assert int(plan["q_off"][-1]) == int(plan["ctx_off"][-1])
    fresh = _fresh_fn(plan, dims, 11)
    scale = 1 / np.sqrt(d)
    res = prefill_layers(plan, ids, empty, 3, fresh, 1e4, scale)
    for layer in range(3):
        q, fk, fv = fresh(layer)
        for b in range(2):
            lo, hi = int(plan["ctx_off"][b]), int(plan["ctx_off"][b + 1])
            tq = torch.from_numpy(q[lo:hi]).permute(1, 0, 2)[None]
            tk = torch.from_numpy(np.repeat(fk[lo:hi], hq // hkv, axis=1)).permute(1, 0, 2)[None]
            tv = torch.from_numpy(np.repeat(fv[lo:hi], hq // hkv, axis=1)).permute(1, 0, 2)[None]
            ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
            np.testing.assert_allclose(res[layer][2][lo:hi], ref[0].permute(1, 0, 2).numpy(), rtol=1e-10, atol=1e-12)


def test_layers_use_their_own_slice_of_every_cache():
    st, ids, requests, dims, rng = _layered_problem(7)
    plan, _ = plan_with_lookup(requests, ids, 2, st)
    fresh = _fresh_fn(plan, dims, 13)
    base = prefill_layers(plan, ids, st, 3, fresh, 1e4, 0.3)
    e = st.entries[100]
    e["k"][1] += 1.0                            # touch layer 1 of one cache only
    again = prefill_layers(plan, ids, st, 3, fresh, 1e4, 0.3)
    assert np.array_equal(base[0][2], again[0][2]) and np.array_equal(base[2][2], again[2][2])
    assert not np.array_equal(base[1][2], again[1][2])
    # a stored value row arrives unchanged at its global position, per layer
    inst = int(np.flatnonzero(plan["inst_src"] == 0)[0])
    g = int(plan["ctx_off"][plan["inst_req"][inst]]) + int(plan["inst_delta"][inst]) + 4
    for layer in range(3):
        assert np.array_equal(again[layer][1][g], st.layer(100, layer)[1][4])
