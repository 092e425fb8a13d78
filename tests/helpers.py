"""Shared plumbing of the tests: build one layer's inputs from the seeded generator,
run the HIP library on them, run the float64 oracle on them.  No arithmetic of the
method lives here."""
import numpy as np
import torch

import workloads
import paper_2502_01960_amd as mpic
from oracle import attend, build_plan, decode_attend, link_kv, link_kv_unshifted, position_fresh


class Problem:
    """Inputs of one layer of one batch, as host tensors in the storage dtype."""
    interleaved = False
    pre_rope = False
    block_keys = 0        # shape of the bf16 attention kernel: 0 = the library's choice, 64 or 96
    lazy = False          # context with lazy_rope: stored keys are never rewritten, queries are turned back

    def __init__(self, cfg_id, *, k=None, layer=0, paged=None, interleaved=False, pre_rope=False, **layout_kw):
        self.sh = sh = workloads.shape(cfg_id)
        self.interleaved = interleaved   # rotary pairing (2i, 2i+1) instead of (i, i+D/2)
        self.pre_rope = pre_rope         # fresh Q/K are handed over before positional embedding
        self.layer = layer
        self.k = sh.default_k if k is None else k
        self.requests, self.n_src, self.src_len = workloads.layout(cfg_id, **layout_kw)
        self.page_size = sh.page_size if paged is None else paged
        lens = [workloads.request_len(r) for r in self.requests]
        if self.page_size:
            self.page_tables, self.n_pool_pages = workloads.gen_page_tables(sh, lens, self.page_size)
            self.n_slots = self.n_pool_pages * self.page_size
        else:
            self.page_tables, self.n_pool_pages = None, 0
            self.n_slots = sum(lens)
        self.oplan = build_plan(self.requests, self.k, self.page_size, self.page_tables)
        used = sorted(set(self.oplan["inst_src"].tolist()))
        self.chunks = {s: workloads.gen_chunk(sh, layer, s, self.src_len[s]) for s in used}
        q_off = self.oplan["q_off"]
        fresh = [workloads.gen_fresh(sh, layer, b, int(q_off[b + 1] - q_off[b]))
                 for b in range(len(self.requests))]
        self.q = torch.cat([f[0] for f in fresh])
        self.fresh_k = torch.cat([f[1] for f in fresh])
        self.fresh_v = torch.cat([f[2] for f in fresh])

    # ---- oracle side -------------------------------------------------------
    def oracle_link(self):
        f64 = lambda t: t.to(torch.float64).numpy()
        ck = {s: f64(kv[0]) for s, kv in self.chunks.items()}
        cv = {s: f64(kv[1]) for s, kv in self.chunks.items()}
        return link_kv(self.oplan, ck, cv, f64(self.fresh_k), f64(self.fresh_v), self.sh.rope_theta,
                       self.interleaved, self.pre_rope)

    def oracle_link_unshifted(self):
        """(K, V, shift): the linked context with stored keys left as stored (float64)."""
        f64 = lambda t: t.to(torch.float64).numpy()
        ck = {s: f64(kv[0]) for s, kv in self.chunks.items()}
        cv = {s: f64(kv[1]) for s, kv in self.chunks.items()}
        return link_kv_unshifted(self.oplan, ck, cv, f64(self.fresh_k), f64(self.fresh_v), self.sh.rope_theta,
                                 self.interleaved, self.pre_rope)

    def oracle_attend(self, K, V, rows=None):
        q = self.q.to(torch.float64).numpy()
        if self.pre_rope:
            q = position_fresh(q, self.oplan, self.sh.rope_theta, self.interleaved)
        return attend(q, K, V, self.oplan, self.sh.softmax_scale, rows=rows)

    # ---- HIP side ----------------------------------------------------------
    def gpu_setup(self, host_sourced=None):
        sh = self.sh
        dev = torch.device("cuda:0")
        dt = mpic.MPIC_F32 if sh.dtype == "f32" else mpic.MPIC_BF16
        self.ctx = mpic.Context(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, dt, sh.rope_theta,
                                int(self.interleaved), self.page_size, int(self.pre_rope), int(self.lazy))
        if self.block_keys:
            self.ctx.set_option(mpic.MPIC_OPT_ATTN_BLOCK_KEYS, self.block_keys)
        self.plan = mpic.Plan(self.ctx, self.requests, self.k, self.page_tables, self.n_pool_pages)
        host = sh.host_sourced if host_sourced is None else host_sourced
        self.srcs = []
        for s in range(self.n_src):
            if s not in self.chunks:
                self.srcs.append((None, None))
            elif host:
                self.srcs.append(tuple(t.pin_memory() for t in self.chunks[s]))
            else:
                self.srcs.append(tuple(t.to(dev) for t in self.chunks[s]))
        # sources the plan never touches still need a length: give them empty placeholders
        self.d_q, self.d_fk, self.d_fv = self.q.to(dev), self.fresh_k.to(dev), self.fresh_v.to(dev)
        shape = (self.n_slots, sh.n_kv_heads, sh.head_dim)
        self.k_ctx = torch.full(shape, float("nan"), dtype=sh.torch_dtype, device=dev)
        self.v_ctx = torch.full(shape, float("nan"), dtype=sh.torch_dtype, device=dev)
        self.out = torch.full(tuple(self.q.shape), float("nan"), dtype=sh.torch_dtype, device=dev)
        self.lse = torch.full(tuple(self.q.shape[:2]), float("nan"), dtype=torch.float32, device=dev)

    host_mode = mpic.MPIC_SRC_HOST_STAGED   # how pinned host chunks reach the GPU (staged copies / read in place)

    def gpu_assemble(self):
        mpic.mpic_assemble_kv(self.ctx.handle, self.plan.handle, self.srcs, self.d_fk, self.d_fv,
                              self.k_ctx, self.v_ctx, None, self.host_mode)

    def gpu_attend(self, lse=True):
        mpic.mpic_selective_attn(self.ctx.handle, self.plan.handle, self.d_q, self.k_ctx, self.v_ctx,
                                 self.sh.softmax_scale, self.out, self.lse if lse else None)

    def gpu_link_fresh_only(self):
        """Only the rows of the recompute set reach the context (caches linked by reference)."""
        mpic.mpic_assemble_kv_parts(self.ctx.handle, self.plan.handle, None, self.d_fk, self.d_fv, self.k_ctx, self.v_ctx,
                                    mpic.MPIC_PART_FRESH)

    def gpu_attend_in_place(self, lse=True):
        mpic.mpic_selective_attn_in_place(self.ctx.handle, self.plan.handle, self.d_q, self.srcs, self.k_ctx, self.v_ctx,
                                          self.sh.softmax_scale, self.out, self.lse if lse else None)

    def gpu_decode_in_place(self, q, new_k, new_v):
        dev = self.k_ctx.device
        out = torch.full(tuple(q.shape), float("nan"), dtype=self.sh.torch_dtype, device=dev)
        l = torch.full(tuple(q.shape[:2]), float("nan"), dtype=torch.float32, device=dev)
        mpic.mpic_decode_attn_in_place(self.ctx.handle, self.plan.handle, q.to(dev),
                                       None if new_k is None else new_k.to(dev), None if new_v is None else new_v.to(dev),
                                       self.srcs, self.k_ctx, self.v_ctx, self.sh.softmax_scale, out, l)
        torch.cuda.synchronize()
        return out.to(torch.float64).cpu().numpy(), l.to(torch.float64).cpu().numpy()

    # ---- decode step after the prefill --------------------------------------
    def decode_inputs(self):
        """Seeded query, key and value of the next token of every request (storage dtype)."""
        n_req = len(self.requests)
        rows = [workloads.gen_fresh(self.sh, self.layer + 1000, b, 1) for b in range(n_req)]
        return (torch.cat([r[0] for r in rows]), torch.cat([r[1] for r in rows]), torch.cat([r[2] for r in rows]))

    def gpu_decode(self, q, new_k, new_v, lse=True):
        dev = self.k_ctx.device
        out = torch.full(tuple(q.shape), float("nan"), dtype=self.sh.torch_dtype, device=dev)
        l = torch.full(tuple(q.shape[:2]), float("nan"), dtype=torch.float32, device=dev) if lse else None
        mpic.mpic_decode_attn(self.ctx.handle, self.plan.handle, q.to(dev),
                              None if new_k is None else new_k.to(dev), None if new_v is None else new_v.to(dev),
                              self.k_ctx, self.v_ctx, self.sh.softmax_scale, out, l)
        torch.cuda.synchronize()
        return out.to(torch.float64).cpu().numpy(), (l.to(torch.float64).cpu().numpy() if lse else None)

    def oracle_decode(self, K, V, q, new_k, new_v):
        f64 = lambda t: None if t is None else t.to(torch.float64).numpy()
        return decode_attend(f64(q), K, V, self.oplan, self.sh.softmax_scale, f64(new_k), f64(new_v))

    def gpu_logical_kv(self):
        """Context rows in logical order (request after request), float64 numpy."""
        slots = torch.from_numpy(self.oplan["dst_slot"].astype(np.int64)).to(self.k_ctx.device)
        torch.cuda.synchronize()
        return (self.k_ctx[slots].to(torch.float64).cpu().numpy(),
                self.v_ctx[slots].to(torch.float64).cpu().numpy())


def err_stats(got, ref):
    e = np.abs(np.asarray(got, dtype=np.float64) - ref)
    return float(e.max()), float(e.mean())


def assert_bf16_close(got, ref, what, max_abs=2e-2, mean_abs=2e-3):
    """Gate of the bf16 configurations: max-abs <= 2e-2 and mean-abs <= 2e-3."""
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    mx, mean = err_stats(got, ref)
    assert mx <= max_abs and mean <= mean_abs, f"{what}: max-abs {mx:.3e}, mean-abs {mean:.3e}"
    return mx, mean


def assert_f32_close(got, ref, what, rel=1e-5):
    """Gate of the fp32 configuration: 1e-5 relative, per tensor and per element."""
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    e = np.abs(got - ref)
    scale = np.abs(ref).max()
    rms = np.sqrt((ref ** 2).mean())
    assert e.max() <= rel * scale, f"{what}: max err {e.max():.3e} vs {rel * scale:.3e}"
    assert (e <= rel * np.abs(ref) + rel * rms).all(), f"{what}: element-wise bound violated"


class LayeredProblem:
    """Several layers of one batch, cached chunks kept in a store (library on the GPU side,
    oracle.store.ChunkStore on the oracle side, both filled with the same seeded bytes)."""

    def __init__(self, cfg_id, n_layers, tiers, disk_dir, *, k=None, paged=None, io_threads=0, id_base=1000,
                 custom=None, interleaved=False, pre_rope=False, lazy=False, **layout_kw):
        from oracle.store import ChunkStore
        self.sh = sh = workloads.shape(cfg_id)
        self.n_layers = n_layers
        self.k = sh.default_k if k is None else k
        # custom = (requests, n_src, src_len) replaces the workload's layout
        self.requests, self.n_src, self.src_len = custom or workloads.layout(cfg_id, **layout_kw)
        self.page_size = sh.page_size if paged is None else paged
        lens = [workloads.request_len(r) for r in self.requests]
        if self.page_size:
            self.page_tables, self.n_pool_pages = workloads.gen_page_tables(sh, lens, self.page_size)
            self.n_slots = self.n_pool_pages * self.page_size
        else:
            self.page_tables, self.n_pool_pages = None, 0
            self.n_slots = max(1, sum(lens))
        self.ids = [id_base + s for s in range(self.n_src)]
        dt = mpic.MPIC_F32 if sh.dtype == "f32" else mpic.MPIC_BF16
        self.interleaved, self.pre_rope, self.lazy = interleaved, pre_rope, lazy
        self.ctx = mpic.Context(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, dt, sh.rope_theta, int(interleaved),
                                self.page_size, int(pre_rope), int(lazy))
        self.store = mpic.Store(self.ctx, n_layers, None if disk_dir is None else str(disk_dir), io_threads)
        self.model = ChunkStore()
        self.raw = {}
        for s in range(self.n_src):
            layers = [workloads.gen_chunk(sh, l, s, self.src_len[s]) for l in range(n_layers)]
            kk = torch.stack([x[0] for x in layers]).contiguous()
            vv = torch.stack([x[1] for x in layers]).contiguous()
            tier = tiers[s % len(tiers)]
            self.store.put(self.ids[s], kk, vv, tier)
            self.model.put(self.ids[s], kk.to(torch.float64).numpy(), vv.to(torch.float64).numpy(), tier)
            self.raw[s] = (kk, vv)

    def plan_for(self, missing=()):
        """Library plan and oracle plan with the sources in `missing` recomputed in full."""
        from oracle.pipeline import plan_with_lookup
        failed = {self.ids[s] for s in missing}
        self.oplan, reqs = plan_with_lookup(self.requests, self.ids, self.k, self.model, self.page_size,
                                            self.page_tables, failed=failed)
        self.plan = mpic.Plan(self.ctx, reqs, self.k, self.page_tables, self.n_pool_pages)
        for f in ("q_pos", "slot_map", "src_inst", "src_row", "dst_slot"):
            assert np.array_equal(self.plan.get(f), self.oplan[f]), f
        q_off = self.oplan["q_off"]
        self.fresh = []
        for l in range(self.n_layers):
            rows = [workloads.gen_fresh(self.sh, l, b, int(q_off[b + 1] - q_off[b])) for b in range(len(reqs))]
            self.fresh.append(tuple(torch.cat([r[i] for r in rows]) for i in range(3)))

    def gpu_run(self, shared_buffers=False, lse=True):
        """One mpic_prefill_layers call; returns its list of failed sources (None = all fine)."""
        dev = torch.device("cuda:0")
        sh, L = self.sh, self.n_layers
        shape = (self.n_slots, sh.n_kv_heads, sh.head_dim)
        nan = lambda shp, dt: torch.full(shp, float("nan"), dtype=dt, device=dev)
        n_buf = 1 if shared_buffers else L
        kb = [nan(shape, sh.torch_dtype) for _ in range(n_buf)]
        vb = [nan(shape, sh.torch_dtype) for _ in range(n_buf)]
        self.k_ctx = [kb[l % n_buf] for l in range(L)]
        self.v_ctx = [vb[l % n_buf] for l in range(L)]
        self.d_fresh = [tuple(t.to(dev) for t in f) for f in self.fresh]
        self.out = [nan(tuple(f[0].shape), sh.torch_dtype) for f in self.fresh]
        self.lse = [nan(tuple(f[0].shape[:2]), torch.float32) for f in self.fresh] if lse else None
        failed = mpic.mpic_prefill_layers(self.ctx.handle, self.plan.handle, self.store.handle, self.ids,
                                          [f[0] for f in self.d_fresh], [f[1] for f in self.d_fresh],
                                          [f[2] for f in self.d_fresh], self.k_ctx, self.v_ctx,
                                          sh.softmax_scale, self.out, self.lse)
        torch.cuda.synchronize()
        return failed

    def oracle_run(self, rows=None, layers=None):
        from oracle.pipeline import prefill_layers
        f64 = lambda t: t.to(torch.float64).numpy()
        return prefill_layers(self.oplan, self.ids, self.model, self.n_layers,
                              lambda l: tuple(f64(t) for t in self.fresh[l]), self.sh.rope_theta,
                              self.sh.softmax_scale, self.interleaved, self.pre_rope, rows=rows, layers=layers)

    def check(self, ref, layers=None, kv_layers=None):
        """Outputs of `layers` and linked contexts of `kv_layers` against the oracle's."""
        close = assert_f32_close if self.sh.dtype == "f32" else assert_bf16_close
        slots = torch.from_numpy(self.oplan["dst_slot"].astype(np.int64)).to(self.k_ctx[0].device)
        for l in (range(self.n_layers) if layers is None else layers):
            K, V, O, lse = ref[l]
            if O.size == 0:
                continue
            got = self.out[l].to(torch.float64).cpu().numpy()
            seen = ~np.isnan(O)
            assert not np.isnan(got).any(), "layer %d: output rows left unwritten" % l
            close(got[seen], O[seen], "layer %d attention output" % l)
            if self.lse is not None:
                g = self.lse[l].to(torch.float64).cpu().numpy()
                seen_l = ~np.isnan(lse)
                assert np.abs(g[seen_l] - lse[seen_l]).max() < (1e-4 if self.sh.dtype == "f32" else 2e-2)
        for l in (range(self.n_layers) if kv_layers is None else kv_layers):
            K, V, O, lse = ref[l]
            assert np.array_equal(self.v_ctx[l][slots].to(torch.float64).cpu().numpy(), V), "layer %d V" % l
            close(self.k_ctx[l][slots].to(torch.float64).cpu().numpy(), K, "layer %d K context" % l)

    def close(self):
        self.plan = None
        self.store.close()
        self.ctx.close()
