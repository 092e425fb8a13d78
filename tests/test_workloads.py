"""The seeded input generator: totals of the five layouts, determinism, dtype."""
import numpy as np
import torch

import workloads


def test_layout_totals():
    want = {1: 160, 2: 2624, 3: 19840, 4: 16896, 5: 75840}
    for cfg, n in want.items():
        reqs, n_src, lens = workloads.layout(cfg)
        assert len(reqs) == workloads.shape(cfg).batch
        assert all(workloads.request_len(r) == n for r in reqs)
        assert len(lens) == n_src


def test_mrag_draws_distinct_chunks_from_pool():
    reqs, pool, _ = workloads.layout(4)
    assert pool == 64
    for r in reqs:
        ids = [s[1] for s in r if s[0] == "chunk"]
        assert len(ids) == 16 and len(set(ids)) == 16 and max(ids) < 64
    assert reqs[0] != reqs[1]


def test_generator_is_deterministic_and_rounded_once():
    sh = workloads.shape(3)
    k1, v1 = workloads.gen_chunk(sh, 0, 5, 32)
    k2, _ = workloads.gen_chunk(sh, 0, 5, 32)
    k3, _ = workloads.gen_chunk(sh, 0, 6, 32)
    assert k1.dtype == torch.bfloat16 and k1.shape == (32, 4, 128)
    assert torch.equal(k1, k2) and not torch.equal(k1, k3) and not torch.equal(k1, v1)
    q, fk, fv = workloads.gen_fresh(workloads.shape(2), 0, 0, 16)
    assert q.shape == (16, 32, 128) and fk.shape == (16, 32, 128)
    assert abs(q.float().std().item() - 1 / np.sqrt(128)) < 0.01
    assert abs(fk.float().std().item() - 1.0) < 0.02


def test_page_tables_are_a_partial_permutation():
    sh = workloads.shape(5)
    tables, pool = workloads.gen_page_tables(sh, [75840])
    assert len(tables[0]) == 4740 and pool == 5925
    assert len(set(tables[0].tolist())) == 4740 and tables[0].max() < pool
    assert (np.diff(tables[0]) != 1).any()
