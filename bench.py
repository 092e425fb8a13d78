#!/usr/bin/env python3
"""Benchmark of the selective-recompute prefill hot path on one MI355X.

One step = one layer of one batch: mpic_assemble_kv (gather of cached chunks, rotary
shift of the keys, scatter of the fresh rows) followed by mpic_selective_attn.  The
integer plan is built once per batch and reused by every step, as the method reuses
it for every layer; its cost is reported separately (plan_ms, first_layer_ms).
Inputs are seeded synthetic tensors resident in HBM before the timed region.  The
steps cycle over several distinct layer input sets so that no step finds its inputs
in the last-level cache left by the previous one.

Prints ONE JSON line (see the keys below).  `value` is the causal-exact attention
work of a step divided by the time of the whole step.
"""
import argparse
import json
import os
import subprocess
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=3, help="workload id (1-5, see workloads/)")
    ap.add_argument("--layers", type=int, default=4, help="distinct layer input sets the steps cycle over")
    ap.add_argument("--fresh-pre-rope", action="store_true",
                    help="hand fresh Q/K over before positional embedding (the library rotates them)")
    ap.add_argument("--k", type=int, default=None, help="recompute the first K tokens of every chunk (default: the workload's)")
    ap.add_argument("--device-data", action="store_true",
                    help="draw the inputs on the GPU (seeded torch generator) instead of the host generator: for sweeps "
                         "over many layer sets, where only the timing matters")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-host-sourced", action="store_true")
    ap.add_argument("--no-device-state", action="store_true", help="skip the clock sample under load (3 s)")
    ap.add_argument("--attn-block-keys", type=int, default=0,
                    help="keys per LDS block of the attention kernel in the main context: 64, 96 or 0 = the library's choice")
    ap.add_argument("--pipeline-layers", type=int, default=8,
                    help="layers of the mpic_prefill_layers leg (caches fetched from the store's HBM, host and disk "
                         "tiers while earlier layers compute); 0 skips it")
    ap.add_argument("--pipeline-tiers", default="disk,host,hbm",
                    help="tiers the mpic_prefill_layers leg is timed from, in this order (hbm alone needs no disk directory)")
    ap.add_argument("--disk-dir", default=None, help="directory of the store's disk tier (default: a temporary one)")
    ap.add_argument("--mfma-ceiling", action="store_true",
                    help="also regenerate the ablation table: the bf16 attention launch of this workload timed with parts of "
                         "its inner loop left out (timing-only kernel variants that only the probe library contains)")
    ap.add_argument("--no-sustained-probe", action="store_true",
                    help="skip the matrix-core probe (sustained bf16 MFMA rate of this GPU with register operands)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch a plain elementwise copy of 512 MiB (reads and writes 512 MiB per "
                         "launch): the reference dispatch for scaling hardware traffic counters")
    return ap.parse_args()


def sample_clocks_under_load(run, seconds=3.0):
    """Run `run()` in a loop for about `seconds`; meanwhile ask rocm-smi (a child process) for
    the clocks and the power cap.  Returns None when the tool is missing or prints nothing usable."""
    import re
    import shutil
    import threading
    tool = shutil.which("rocm-smi") or "/opt/rocm/bin/rocm-smi"
    if not os.path.exists(tool):
        return None
    out = {}

    def ask():
        time.sleep(seconds / 3)
        try:
            r = subprocess.run([tool, "--showclocks", "--showmaxpower"], capture_output=True, text=True, timeout=30)
            out["text"] = r.stdout
        except Exception:
            pass
    th = threading.Thread(target=ask)
    th.start()
    t0 = time.time()
    while time.time() - t0 < seconds or th.is_alive():
        run()
        if time.time() - t0 > 40:
            break
    th.join()
    text = out.get("text", "")
    sclk = re.search(r"sclk clock level: *\d+: *\((\d+)Mhz\)", text)
    mclk = re.search(r"mclk clock level: *\d+: *\((\d+)Mhz\)", text)
    cap = re.search(r"Max Graphics Package Power \(W\): *([0-9.]+)", text)
    if not sclk:
        return None
    return {"sclk_mhz_under_attention": int(sclk.group(1)), "mclk_mhz": int(mclk.group(1)) if mclk else None,
            "power_cap_w": float(cap.group(1)) if cap else None, "sclk_mhz_of_the_peak_figure": 2400,
            "source": "rocm-smi --showclocks --showmaxpower, sampled while the attention kernel ran back to back"}


def probe_lib_path():
    return os.path.join(ROOT, "paper_2502_01960_amd", "libmpic_probe.so")


def sustained_mfma(torch, dev, with_clock):
    """Sustained bf16 matrix-core rate of this GPU: 48 v_mfma_f32_32x32x16_bf16 per wavefront and block on
    register operands (random values), 8 wavefronts per workgroup, one workgroup per compute unit;
    alone, in the kernel's ping-pong schedule, and with the softmax work on the vector ALU beside it."""
    import ctypes as C
    if not os.path.exists(probe_lib_path()):
        return None
    lib = C.CDLL(probe_lib_path())
    lib.mpic_probe_mfma.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_double)]
    lib.mpic_probe_mfma.restype = C.c_int
    gen = torch.Generator(device=dev).manual_seed(0x4D504943)
    seed = torch.randn((64 * 16 * 8,), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    n_wgs = 256 * 4
    sink = torch.empty((n_wgs * 512,), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()
    fl = C.c_double()
    out = {"note": "probe: 48 v_mfma_f32_32x32x16_bf16 per wavefront and block on register operands (random bf16), 8 wavefronts "
                   "per workgroup, one workgroup per compute unit, 4 workgroups per unit in sequence",
           "peak_TFLOPs": PEAK_BF16_TFLOPS}

    zeros = torch.zeros_like(seed)

    def run(flags, n_blocks, operands=seed):
        rc = lib.mpic_probe_mfma(flags, n_wgs, n_blocks, C.c_void_p(operands.data_ptr()), C.c_void_p(sink.data_ptr()),
                                 C.c_void_p(stream.cuda_stream), C.byref(fl))
        assert rc == 0, rc

    # the same instruction stream on operands that are all zero: nothing toggles in the data paths, so
    # what this run gains over "mfma_only" is what the power management takes from random operands
    # (flag 8: the fragments of the matrix instructions are read from LDS the way the kernel reads them; flag 4:
    # the same work divided the other way, one wavefront per SIMD with 64 query columns and the softmax
    # interleaved into its own instruction stream instead of hidden behind a second wavefront)
    for name, flags, ops in (("mfma_only", 0, seed), ("mfma_pingpong", 1, seed), ("mfma_pingpong_softmax", 3, seed),
                             ("mfma_pingpong_softmax_lds_reads", 11, seed), ("one_wave_per_simd_softmax", 4, seed),
                             ("one_wave_per_simd_softmax_lds_reads", 12, seed), ("mfma_only_zero_operands", 0, zeros),
                             ("mfma_pingpong_softmax_lds_reads_zero_operands", 11, zeros)):
        n_blocks = 300
        run(flags, n_blocks, ops)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(10):
            run(flags, n_blocks, ops)
        e1.record(stream)
        e1.synchronize()
        ms = e0.elapsed_time(e1) / 10
        out[name + "_TFLOPs"] = round(fl.value * n_wgs * n_blocks / (ms * 1e-3) / 1e12, 2)
        if with_clock and flags in (0, 3):
            st = sample_clocks_under_load(lambda: run(flags, n_blocks, ops), seconds=2.0)
            if st:
                out[name + "_sclk_mhz"] = st["sclk_mhz_under_attention"]
    return out


def streaming_read_probe(torch, dev, n_bytes, repeats=20):
    """What one launch that only reads n_bytes from HBM takes on this GPU (16-byte loads, four in flight per
    lane; best of a few grid sizes): the floor under a decode step that has to read that many bytes of keys and
    values.  Four buffers are read in turn, so that none is still in the 256 MB Infinity Cache when its turn comes."""
    import ctypes as C
    if not os.path.exists(probe_lib_path()):
        return None
    lib = C.CDLL(probe_lib_path())
    if not hasattr(lib, "mpic_probe_read"):
        return None
    lib.mpic_probe_read.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_void_p]
    lib.mpic_probe_read.restype = C.c_int
    n_bytes = int(n_bytes) // 4096 * 4096
    gen = torch.Generator(device=dev).manual_seed(0x4D504943)
    buf = torch.randint(0, 2 ** 31 - 1, (4, n_bytes // 4), generator=gen, device=dev, dtype=torch.int32)
    stream = torch.cuda.current_stream()
    best = None
    for per_cu in (2, 4, 8, 16):
        n_wgs = 256 * per_cu
        sink = torch.empty((n_wgs + 1,), dtype=torch.float32, device=dev)

        def run(i):
            rc = lib.mpic_probe_read(C.c_void_p(buf[i % 4].data_ptr()), n_bytes, n_wgs, C.c_void_p(sink.data_ptr()),
                                     C.c_void_p(stream.cuda_stream))
            assert rc == 0, rc
        for i in range(4):
            run(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(repeats):
            run(i)
        e1.record(stream)
        e1.synchronize()
        ms = e0.elapsed_time(e1) / repeats
        if best is None or ms < best["ms"]:
            best = {"ms": round(ms, 5), "GBps": round(n_bytes / (ms * 1e-3) / 1e9, 1), "workgroups": n_wgs, "bytes": n_bytes}
    best["pct_hbm_peak"] = round(100 * best["GBps"] / PEAK_HBM_GBS, 2)
    best["note"] = "a launch that does nothing but read this many bytes once (libmpic_probe.so, probe_read_kernel), back to back"
    return best


def ablation_table(args, torch, dev, sh, requests, tables, pool, n_slots, n_q, attn_flops):
    """The bf16 attention launch of this workload timed with parts of its inner loop left out: timing-only
    kernel variants that only the probe library contains.  It is loaded beside the product library through a
    second instance of the binding module (same process: a second process on the GPU would halve both)."""
    import importlib.util
    if not os.path.exists(probe_lib_path()):
        return None
    spec = importlib.util.spec_from_file_location("mpic_probe_binding", os.path.join(ROOT, "paper_2502_01960_amd", "binding.py"))
    pb = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(pb)
    pb.lib_path = probe_lib_path
    ctx = pb.Context(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, pb.MPIC_BF16, sh.rope_theta, 0, sh.page_size)
    ctx.set_option(pb.MPIC_OPT_ATTN_BLOCK_KEYS, args.attn_block_keys or 96)
    plan = pb.Plan(ctx, requests, sh.default_k, tables, pool)
    gen = torch.Generator(device=dev).manual_seed(0x4D504943)
    draw = lambda *shape: torch.randn(shape, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    sets = []
    for _ in range(max(2, args.layers)):
        q = draw(n_q, sh.n_q_heads, sh.head_dim)
        sets.append((q, draw(n_slots, sh.n_kv_heads, sh.head_dim), draw(n_slots, sh.n_kv_heads, sh.head_dim), torch.empty_like(q)))
    stream = torch.cuda.current_stream()

    def run(i):
        q, k, v, o = sets[i % len(sets)]
        pb.mpic_selective_attn(ctx.handle, plan.handle, q, k, v, sh.softmax_scale, o, None, stream)
    run(0)     # uploads the plan
    names = {0: "whole kernel", 1: "without the K/V loads", 2: "without the LDS fragment reads", 4: "without the softmax",
             3: "without loads and LDS reads", 5: "without loads and softmax", 6: "without LDS reads and softmax",
             7: "matrix instructions, barriers and the ping-pong skeleton only",
             8: "all loads issued, but every block staged from the rows of the tile's first block (cache hits)",
             # what the loads cost on top of the skeleton (mask 6 above is skeleton + loads), taken apart
             6 | 8: "skeleton + loads from the rows of the first block (cache hits)",
             6 | 32: "skeleton + loads, no wait for them inside the loop",
             6 | 64: "skeleton + the address arithmetic of the loads, no load issued"}
    # every variant twice: on the random operands, and on operands that are all zero -- there the clock does
    # not give way to the power the data paths draw, so the second column is the instruction stream alone
    zero_sets = [tuple(torch.zeros_like(t) for t in sets[0][:3]) + (sets[0][3],)]
    out = {}
    for mask in (0, 1, 2, 4, 3, 5, 6, 7, 8, 6 | 8, 6 | 32, 6 | 64):
        ctx.set_option(1000, mask)     # kProbeOptionAblate of the probe library
        row = {}
        for column, use in (("", sets), ("_zero_operands", zero_sets)):
            def run_on(i):
                q, k, v, o = use[i % len(use)]
                pb.mpic_selective_attn(ctx.handle, plan.handle, q, k, v, sh.softmax_scale, o, None, stream)
            for i in range(max(args.warmup, 10)):
                run_on(i)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for i in range(args.steps):
                run_on(i)
            e1.record(stream)
            e1.synchronize()
            ms = e0.elapsed_time(e1) / args.steps
            row["ms" + column] = round(ms, 5)
            row["TFLOPs_of_the_whole_kernels_work" + column] = round(attn_flops / (ms * 1e-3) / 1e12, 2)
        out[names[mask]] = row
    out["note"] = ("timing-only variants of attn_bf16_kernel (probe library, same launch; random inputs drawn on the GPU, and "
                   "all-zero inputs); rates are the whole kernel's algorithmic flops over each variant's time")
    plan.close()
    ctx.close()
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2
    import torch
    import workloads
    import paper_2502_01960_amd as mpic

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    mpic.load_library()  # fails loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    sh = workloads.shape(args.config)
    if sh.dtype != "bf16":
        print("bench.py: the timed workloads are the bf16 configurations (2-5)", file=sys.stderr)
        return 2
    requests, n_src, src_len = workloads.layout(args.config)
    lens = [workloads.request_len(r) for r in requests]
    tables, pool = (None, 0)
    if sh.page_size:
        tables, pool = workloads.gen_page_tables(sh, lens)
    n_slots = pool * sh.page_size if sh.page_size else sum(lens)

    if args.k is not None:
        import dataclasses
        sh = dataclasses.replace(sh, default_k=args.k)
    if args.device_data:
        args.no_cpu_baseline = args.no_host_sourced = True   # both legs read the host copies of the inputs
        gen = torch.Generator(device=dev).manual_seed(0x4D504943)

        def draw(*shape):
            return torch.randn(shape, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    ctx = mpic.Context(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, mpic.MPIC_BF16, sh.rope_theta, 0, sh.page_size,
                       int(args.fresh_pre_rope))
    if args.attn_block_keys:
        ctx.set_option(mpic.MPIC_OPT_ATTN_BLOCK_KEYS, args.attn_block_keys)
    t0 = time.perf_counter()
    plan = mpic.Plan(ctx, requests, sh.default_k, tables, pool)
    plan_ms = (time.perf_counter() - t0) * 1e3
    q_off = plan.get("q_off")
    q_pos = plan.get("q_pos").astype(np.int64)
    n_q, n_ctx = int(q_off[-1]), int(sum(lens))
    used_src = sorted(set(plan.get("inst_src").tolist()))

    # ---- inputs: `layers` distinct sets, all resident in HBM -----------------
    L = max(1, args.layers)
    sets = []
    host_chunks0 = None
    host_chunks = []
    for layer in range(L):
        if args.device_data:
            kv_shape = (sh.n_kv_heads, sh.head_dim)
            srcs = [(draw(src_len[s], *kv_shape), draw(src_len[s], *kv_shape)) if s in used_src else (None, None)
                    for s in range(n_src)]
            q = draw(max(n_q, 1), sh.n_q_heads, sh.head_dim)[:n_q]
            fk, fv = draw(max(n_q, 1), *kv_shape)[:n_q], draw(max(n_q, 1), *kv_shape)[:n_q]
        else:
            chunks = {s: workloads.gen_chunk(sh, layer, s, src_len[s]) for s in used_src}
            host_chunks.append(chunks)
            if layer == 0:
                host_chunks0 = chunks
            srcs = [tuple(t.to(dev) for t in chunks[s]) if s in chunks else (None, None) for s in range(n_src)]
            fresh = [workloads.gen_fresh(sh, layer, b, int(q_off[b + 1] - q_off[b])) for b in range(len(requests))]
            q = torch.cat([f[0] for f in fresh]).to(dev)
            fk = torch.cat([f[1] for f in fresh]).to(dev)
            fv = torch.cat([f[2] for f in fresh]).to(dev)
        k_ctx = torch.empty((n_slots, sh.n_kv_heads, sh.head_dim), dtype=torch.bfloat16, device=dev)
        v_ctx = torch.empty_like(k_ctx)
        out = torch.empty_like(q)
        sets.append(dict(index=layer, srcs=srcs, srcs_c=mpic.ChunkSources(srcs), q=q, fk=fk, fv=fv, k_ctx=k_ctx, v_ctx=v_ctx, out=out))
    stream = torch.cuda.current_stream()
    # A context that links in the background switches its attention kernel to the shape that leaves
    # room for the linking waves (64 keys per block instead of 96), so the two-stream and the
    # read-in-place schedules get a context of their own.
    ctx_bg = mpic.Context(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, mpic.MPIC_BF16, sh.rope_theta, 0, sh.page_size,
                          int(args.fresh_pre_rope))
    plan_bg = mpic.Plan(ctx_bg, requests, sh.default_k, tables, pool)

    def assemble(s, srcs=None):
        mpic.mpic_assemble_kv(ctx.handle, plan.handle, srcs or s["srcs_c"], s["fk"], s["fv"], s["k_ctx"], s["v_ctx"], stream)

    def attend(s, c=None, p=None):
        mpic.mpic_selective_attn((c or ctx).handle, (p or plan).handle, s["q"], s["k_ctx"], s["v_ctx"], sh.softmax_scale,
                                 s["out"], None, stream)

    # first layer end to end (plan + upload of the plan + link + attention)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    assemble(sets[0]); attend(sets[0])
    torch.cuda.synchronize()
    first_layer_ms = plan_ms + (time.perf_counter() - t0) * 1e3

    # ---- whole steps -----------------------------------------------------------
    # Every step links one layer's context and attends over it.  The rows that come from
    # stored chunks need no model output, so their linking for step i+1 is issued on a second
    # stream and runs while step i attends (the transfer / compute overlap of Sec. 3.2); the
    # fresh rows are scattered on the main stream right before the attention that reads them.
    side = torch.cuda.Stream()
    ev_cached = [torch.cuda.Event() for _ in range(L)]
    ev_free = [torch.cuda.Event() for _ in range(L)]

    def link_cached(i, srcs=None, mode=mpic.MPIC_SRC_HOST_STAGED):
        s = sets[i % L]
        side.wait_event(ev_free[i % L])   # the attention that last read this context has finished
        mpic.mpic_assemble_kv_parts(ctx_bg.handle, plan_bg.handle, srcs or s["srcs_c"], None, None, s["k_ctx"], s["v_ctx"],
                                    mpic.MPIC_PART_CACHED | mpic.MPIC_PART_BACKGROUND, side, mode)
        ev_cached[i % L].record(side)

    def step(i, n_total, srcs=None, mode=mpic.MPIC_SRC_HOST_STAGED):
        s = sets[i % L]
        if i + 1 < n_total:
            link_cached(i + 1, srcs, mode)
        stream.wait_event(ev_cached[i % L])
        mpic.mpic_assemble_kv_parts(ctx_bg.handle, plan_bg.handle, None, s["fk"], s["fv"], s["k_ctx"], s["v_ctx"],
                                    mpic.MPIC_PART_FRESH, stream)
        attend(s, ctx_bg, plan_bg)
        ev_free[i % L].record(stream)

    def run_steps(n, srcs=None, mode=mpic.MPIC_SRC_HOST_STAGED):
        for e in ev_free:
            e.record(stream)
        link_cached(0, srcs, mode)
        for i in range(n):
            step(i, n, srcs, mode)

    # Chunks resident in HBM need no second stream: the stored rows of step i+1 are linked by
    # the attention launch of step i, in workgroups that run while that attention drains.
    def run_fused(n):
        s0 = sets[0]
        mpic.mpic_assemble_kv_parts(ctx.handle, plan.handle, s0["srcs_c"], None, None, s0["k_ctx"], s0["v_ctx"],
                                    mpic.MPIC_PART_CACHED, stream)
        for i in range(n):
            s, nx = sets[i % L], sets[(i + 1) % L]
            mpic.mpic_assemble_kv_parts(ctx.handle, plan.handle, None, s["fk"], s["fv"], s["k_ctx"], s["v_ctx"],
                                        mpic.MPIC_PART_FRESH, stream)
            if i + 1 < n:
                mpic.mpic_selective_attn_link_next(ctx.handle, plan.handle, s["q"], s["k_ctx"], s["v_ctx"],
                                                   sh.softmax_scale, s["out"], nx["srcs_c"], nx["k_ctx"], nx["v_ctx"],
                                                   None, stream)
            else:
                attend(s)

    # Which of the two schedules is the step: the planner's estimate decides, as it does inside
    # mpic_prefill_layers (is the linking predicted to fit into what the attention launch leaves idle?)
    fuse = bool(plan.get("launch_estimate")[3])
    # (The event-timed kernel loops come first, after an untimed stretch of load: the whole-step timing below
    # should not pay for the clock ramp of a GPU that was idle with its first steps.)
    # ---- per-kernel durations with events on the launch stream -----------------
    def timed(fn, n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(stream)
        for i in range(n):
            fn(sets[i % L])
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_time(e1) / n

    # the attention launch of the schedule that is the step (its kernel shape included)
    attend_of_step = attend if fuse or L < 2 else (lambda s: attend(s, ctx_bg, plan_bg))
    # Untimed load first.  (1) Every context is assembled, so that the attention launches below read real
    # keys and values: on buffers that were never written the kernel runs some 15 % faster, because the power
    # the matrix cores draw -- and with it the clock the part holds -- depends on the operand bits.  (2) After
    # an idle period the clocks need about half a second of load to settle (1.12 -> 1.06 ms per launch over
    # the first 0.5 s measured); every figure below is meant to be the settled one.
    for s_ in sets:
        assemble(s_)
    if not fuse and L >= 2:
        run_steps(2)    # the context that links in the background takes its attention shape with the first such link
        torch.cuda.synchronize()
    t_heat = time.perf_counter()
    i = 0
    while time.perf_counter() - t_heat < 0.6:
        attend_of_step(sets[i % L])
        i += 1
        if i % 50 == 0:
            torch.cuda.synchronize()
    attn_ms = timed(attend_of_step, args.steps)

    def each(fn, n):
        """Durations of n back-to-back launches one by one (an event between neighbours)."""
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        torch.cuda.synchronize()
        evs[0].record(stream)
        for i in range(n):
            fn(sets[i % L])
            evs[i + 1].record(stream)
        evs[-1].synchronize()
        return np.array([evs[i].elapsed_time(evs[i + 1]) for i in range(n)])
    attn_each = each(attend_of_step, max(args.steps, 20))
    asm_ms = timed(assemble, args.steps)
    # the launch the fused step uses: the same attention plus, in trailing workgroups, the stored rows
    # of the next layer set (attn_bf16_kernel<..., LinkNext>)
    fused_launch_ms = None
    if fuse and L >= 2:
        def attend_link(i_s):
            nx = sets[(i_s["index"] + 1) % L]
            mpic.mpic_selective_attn_link_next(ctx.handle, plan.handle, i_s["q"], i_s["k_ctx"], i_s["v_ctx"], sh.softmax_scale,
                                               i_s["out"], nx["srcs_c"], nx["k_ctx"], nx["v_ctx"], None, stream)
        fused_launch_ms = timed(attend_link, args.steps)

    # The same launch on operands that are all zero (queries, keys, values): the instruction stream and the
    # memory traffic are unchanged, only the bits that toggle in the data paths are gone.  What it gains is
    # what the part's power management takes from the launch on real operands (lower clock under higher power).
    zq = torch.zeros_like(sets[0]["q"])
    zk, zv = torch.zeros_like(sets[0]["k_ctx"]), torch.zeros_like(sets[0]["v_ctx"])
    zero_set = dict(q=zq, k_ctx=zk, v_ctx=zv, out=sets[0]["out"])
    zero_ms = timed(lambda s_: attend_of_step(zero_set), args.steps)
    attend_of_step(sets[0])    # (out of set 0 holds real results again)
    del zq, zk, zv, zero_set

    other_ms = None
    if L >= 2:
        both = {}
        for name, fn in (("fused", run_fused), ("two_stream", run_steps)):
            fn(args.warmup)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fn(args.steps)
            torch.cuda.synchronize()
            both[name] = (time.perf_counter() - t0) * 1e3 / args.steps
        ms_per_step = both["fused" if fuse else "two_stream"]
        other_ms = both["two_stream" if fuse else "fused"]
    else:
        for i in range(args.warmup):
            s = sets[i % L]; assemble(s); attend(s)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            s = sets[i % L]; assemble(s); attend(s)
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # a new batch in a warm process: plan + its upload + link + attention of the first layer
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    plan2 = mpic.Plan(ctx, requests, sh.default_k, tables, pool)
    s0 = sets[0]
    mpic.mpic_assemble_kv(ctx.handle, plan2.handle, s0["srcs"], s0["fk"], s0["fv"], s0["k_ctx"], s0["v_ctx"], stream)
    mpic.mpic_selective_attn(ctx.handle, plan2.handle, s0["q"], s0["k_ctx"], s0["v_ctx"], sh.softmax_scale,
                             s0["out"], None, stream)
    torch.cuda.synchronize()
    warm_first_layer_ms = (time.perf_counter() - t0) * 1e3
    plan2.close()

    # ---- caches linked by reference (lazy_rope context): no stored row is copied or rewritten; the step
    # is the scatter of the fresh rows plus the attention launch that reads the caches in place ----
    ctx_lz = mpic.Context(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, mpic.MPIC_BF16, sh.rope_theta, 0, sh.page_size,
                          int(args.fresh_pre_rope), 1)
    if args.attn_block_keys:
        ctx_lz.set_option(mpic.MPIC_OPT_ATTN_BLOCK_KEYS, args.attn_block_keys)
    plan_lz = mpic.Plan(ctx_lz, requests, sh.default_k, tables, pool)

    def attend_in_place(s):
        mpic.mpic_selective_attn_in_place(ctx_lz.handle, plan_lz.handle, s["q"], s["srcs_c"], s["k_ctx"], s["v_ctx"],
                                          sh.softmax_scale, s["out"], None, stream)

    def step_in_place(s):
        mpic.mpic_assemble_kv_parts(ctx_lz.handle, plan_lz.handle, None, s["fk"], s["fv"], s["k_ctx"], s["v_ctx"],
                                    mpic.MPIC_PART_FRESH, stream)
        attend_in_place(s)

    in_place = None
    if len(plan_lz.get("inst_src")) <= 128:
        for i in range(args.warmup):
            step_in_place(sets[i % L])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step_in_place(sets[i % L])
        torch.cuda.synchronize()
        ip_step_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        ip_attn_ms = timed(attend_in_place, args.steps)
        ip_fresh_ms = timed(lambda s: mpic.mpic_assemble_kv_parts(ctx_lz.handle, plan_lz.handle, None, s["fk"], s["fv"], s["k_ctx"],
                                                                  s["v_ctx"], mpic.MPIC_PART_FRESH, stream), args.steps)
        blocks = plan_lz.get("key_blocks_%d" % (args.attn_block_keys or 96))
        in_place = {"ms_per_step": round(ip_step_ms, 5), "attention_ms": round(ip_attn_ms, 5), "fresh_rows_ms": round(ip_fresh_ms, 5),
                    "padding_keys_pct": round(100.0 * (len(blocks) * (args.attn_block_keys or 96) / max(1, n_ctx) - 1.0), 3),
                    "note": "lazy_rope context: fresh rows scattered into the context, stored rows read where their caches are "
                            "stored, queries turned back per chunk instance; same outputs as the linked step within the gates"}

    # ---- clocks while the attention kernel runs back to back (the 2.5 PFLOP/s peak is a 2.4 GHz
    # figure; what the part holds under this load says how much of the gap is clock) ----
    device_state = None
    if not args.no_device_state:
        device_state = sample_clocks_under_load(lambda: timed(attend, 50))

    # ---- one step captured in a HIP graph and replayed: what a launch-bound serving loop would
    # do for small batches (extra figure).  The step as above when it is the fused one: fresh rows,
    # then the attention launch that also links the next layer's stored rows; else link + attention.
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        s0, s1 = sets[0], sets[1 % L]
        if fuse and L >= 2:
            mpic.mpic_assemble_kv_parts(ctx.handle, plan.handle, None, s0["fk"], s0["fv"], s0["k_ctx"], s0["v_ctx"],
                                        mpic.MPIC_PART_FRESH, None)
            mpic.mpic_selective_attn_link_next(ctx.handle, plan.handle, s0["q"], s0["k_ctx"], s0["v_ctx"],
                                               sh.softmax_scale, s0["out"], s1["srcs_c"], s1["k_ctx"], s1["v_ctx"],
                                               None, None)
        else:
            mpic.mpic_assemble_kv(ctx.handle, plan.handle, s0["srcs"], s0["fk"], s0["fv"], s0["k_ctx"], s0["v_ctx"], None)
            mpic.mpic_selective_attn(ctx.handle, plan.handle, s0["q"], s0["k_ctx"], s0["v_ctx"], sh.softmax_scale,
                                     s0["out"], None, None)
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        graph.replay()
    torch.cuda.synchronize()
    graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    del graph

    # ---- decode step right after the prefill (extra figure; HBM-bound) ----------
    for l, s in enumerate(sets):
        s["dec"] = [torch.cat([workloads.gen_fresh(sh, 1000 + l, b, 1)[i] for b in range(len(requests))]).to(dev)
                    for i in range(3)]
    dec_out = torch.empty_like(sets[0]["dec"][0])

    def decode(s):
        dq, dk, dv = s["dec"]
        mpic.mpic_decode_attn(ctx.handle, plan.handle, dq, dk, dv, s["k_ctx"], s["v_ctx"],
                              sh.softmax_scale, dec_out, None, stream)

    decode(sets[0])
    dec_ms = timed(decode, args.steps)

    # ---- K distance of two caches (analysis kernel; every row of both is read once) ----
    kd = None
    if L >= 2:
        dist = torch.empty((n_slots,), dtype=torch.float32, device=dev)

        def kdist(s):
            other = sets[1] if s is sets[0] else sets[0]
            mpic.mpic_k_distance(ctx.handle, s["k_ctx"], other["k_ctx"], dist, stream)

        kdist(sets[0])
        kd_ms = timed(kdist, args.steps)
        kd_bytes = 2.0 * n_slots * sh.n_kv_heads * sh.head_dim * 2
        kd = {"ms": round(kd_ms, 5), "GBps": round(kd_bytes / (kd_ms * 1e-3) / 1e9, 2),
              "pct_hbm_peak": round(100 * kd_bytes / (kd_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 3), "bytes": kd_bytes,
              "note": "per-token L1 distance between two linked K caches of the whole batch"}

    if args.calibrate_copy:
        x = torch.zeros(256 * 1024 * 1024, dtype=torch.bfloat16, device=dev)
        y = torch.empty_like(x)
        for _ in range(5):
            torch.add(x, 1.0, out=y)
        torch.cuda.synchronize()
        del x, y

    # ---- algorithmic work ------------------------------------------------------
    # attention: 2*D flops for q.k and 2*D for p.v per visible (row, head, key)
    pairs = int((q_pos + 1).sum())
    attn_flops = 4.0 * sh.head_dim * sh.n_q_heads * pairs
    # linking: every context row is read once from its source and written once, K and V
    row_bytes = sh.n_kv_heads * sh.head_dim * 2
    asm_bytes = 4.0 * n_ctx * row_bytes
    attn_tflops = attn_flops / (attn_ms * 1e-3) / 1e12
    asm_gbs = asm_bytes / (asm_ms * 1e-3) / 1e9
    value = attn_flops / (ms_per_step * 1e-3) / 1e12
    # decode step: every context row of K and V is read once
    dec_bytes = 2.0 * n_ctx * row_bytes
    dec_gbs = dec_bytes / (dec_ms * 1e-3) / 1e9

    # ---- host-sourced chunks (PCIe inclusive; never `value`) -------------------
    host = None
    if not args.no_host_sourced:
        pinned = [tuple(t.pin_memory() for t in host_chunks0[s]) if s in host_chunks0 else (None, None)
                  for s in range(n_src)]
        n_h = max(3, min(10, args.steps))
        for _ in range(2):
            assemble(sets[0], pinned); attend(sets[0])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_h):
            assemble(sets[0], pinned); attend(sets[0])
        torch.cuda.synchronize()
        h_ms = (time.perf_counter() - t0) * 1e3 / n_h
        inst_src, inst_len, inst_k = plan.get("inst_src"), plan.get("inst_len"), plan.get("inst_k")
        # per distinct source: rows below the smallest effective k of its instances stay on the host
        kmin = {}
        for s_, l_, k_ in zip(inst_src.tolist(), inst_len.tolist(), inst_k.tolist()):
            if k_ < l_:
                kmin[s_] = min(kmin.get(s_, l_), k_)
        copied = sum(2 * (src_len[s_] - k_) * row_bytes for s_, k_ in kmin.items())
        # the same transfers with no attention beside them: what the bus alone allows
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_h):
            assemble(sets[0], pinned)
        torch.cuda.synchronize()
        copy_ms = (time.perf_counter() - t0) * 1e3 / n_h
        host = dict(ms_per_step=round(h_ms, 4), pcie_bytes=int(copied), transfer_alone_ms=round(copy_ms, 4),
                    overlap_efficiency=round(max(copy_ms, ms_per_step) / h_ms, 4),
                    pcie_GBps=round(copied / (h_ms * 1e-3) / 1e9, 2), steps=n_h,
                    note="cached chunks in pinned host memory, reused rows staged over the side stream, overlapped with the previous step; "
                         "overlap_efficiency = max(linking from the host alone, HBM-resident step) / this step")
        if L >= 2:
            # the same chunks read in place by the linking kernel (no staging), cached part of step
            # i+1 on the second stream while step i attends
            run_steps(2, pinned, mpic.MPIC_SRC_HOST_MAPPED)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            run_steps(n_h, pinned, mpic.MPIC_SRC_HOST_MAPPED)
            torch.cuda.synchronize()
            m_ms = (time.perf_counter() - t0) * 1e3 / n_h
            host["mapped"] = dict(ms_per_step=round(m_ms, 4), pcie_GBps=round(copied / (m_ms * 1e-3) / 1e9, 2),
                                  note="chunks read over the bus by the linking kernel itself, on a second stream while the previous step attends")

    # ---- all layers of a batch in one call, caches fetched from the store (Sec. 3.2, Fig. 6) ----
    pipe = None
    if not args.no_host_sourced and args.pipeline_layers > 0:
        import shutil
        import tempfile
        P = args.pipeline_layers
        tiers = [t for t in args.pipeline_tiers.split(",") if t]
        tier_id = {"disk": mpic.MPIC_TIER_DISK, "host": mpic.MPIC_TIER_HOST, "hbm": mpic.MPIC_TIER_HBM}
        need_disk = "disk" in tiers
        tmp = tempfile.mkdtemp(prefix="mpic_store_") if need_disk and not args.disk_dir else None
        store = mpic.Store(ctx, P, (args.disk_dir or tmp) if need_disk else None, 8)
        ids = [5000 + s for s in range(n_src)]
        cache_bytes = 0
        for s in used_src:
            kk = torch.stack([host_chunks[l % L][s][0] for l in range(P)]).contiguous()
            vv = torch.stack([host_chunks[l % L][s][1] for l in range(P)]).contiguous()
            store.put(ids[s], kk, vv, tier_id[tiers[0]])
            cache_bytes += 2 * kk.numel() * 2
            del kk, vv
        lists = [[sets[l % L][f] for l in range(P)] for f in ("q", "fk", "fv", "k_ctx", "v_ctx", "out")]
        pipe = dict(layers=P, stored_bytes_per_layer=cache_bytes // P, reader_threads=8,
                    note="one mpic_prefill_layers call per batch: stored rows of later layers are read from their tier and "
                         "linked (read over the bus in place, or staged copies when caches are shared by requests) while earlier layers attend; ms per layer = call to stream sync / layers")
        reps = max(2, min(4, args.steps))
        for name in tiers:
            for s in used_src:
                store.move(ids[s], tier_id[name])

            def call():
                assert mpic.mpic_prefill_layers(ctx.handle, plan.handle, store.handle, ids, *lists[:5],
                                                sh.softmax_scale, lists[5], None, stream) is None
            call()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                call()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / (reps * P)
            pipe[name] = dict(ms_per_layer=round(ms, 4), TFLOPs=round(4.0 * sh.head_dim * sh.n_q_heads * int((q_pos + 1).sum()) / (ms * 1e-3) / 1e12, 2))
            if name != "hbm":
                pipe[name]["fetch_GBps"] = round(cache_bytes / P / (ms * 1e-3) / 1e9, 2)
        store.close()
        if tmp:
            shutil.rmtree(tmp, ignore_errors=True)

    # ---- the oracle on the host cores (reported baseline, bounded sample) ------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import attend as o_attend, build_plan, link_kv, position_fresh
        n_req = min(3, len(requests))
        sub = requests[:n_req]
        oplan = build_plan(sub, sh.default_k)
        f64 = lambda t: t.to(torch.float64).numpy()
        ck = {s: f64(host_chunks0[s][0]) for s in set(oplan["inst_src"].tolist())}
        cv = {s: f64(host_chunks0[s][1]) for s in set(oplan["inst_src"].tolist())}
        fresh = [workloads.gen_fresh(sh, 0, b, int(oplan["q_off"][b + 1] - oplan["q_off"][b])) for b in range(n_req)]
        fq = np.concatenate([f64(f[0]) for f in fresh])
        fk = np.concatenate([f64(f[1]) for f in fresh])
        fv = np.concatenate([f64(f[2]) for f in fresh])
        # bounded sample: at most about 1.2 TFLOP of attention (every m-th fresh row of the sample)
        opos = oplan["q_pos"].astype(np.int64)
        every = max(1, int(np.ceil(4.0 * sh.head_dim * sh.n_q_heads * int((opos + 1).sum()) / 1.2e12)))
        rows = np.arange(0, len(opos), every)
        t0 = time.perf_counter()
        K, V = link_kv(oplan, ck, cv, fk, fv, sh.rope_theta, False, args.fresh_pre_rope)
        if args.fresh_pre_rope:
            fq = position_fresh(fq, oplan, sh.rope_theta)
        o_attend(fq, K, V, oplan, sh.softmax_scale, rows=None if every == 1 else rows)
        dt = time.perf_counter() - t0
        fl = 4.0 * sh.head_dim * sh.n_q_heads * int((opos[rows] + 1).sum())
        cpu = dict(value=round(fl / dt / 1e12, 6), unit="TFLOP/s", cores=int(torch.get_num_threads()),
                   kind="oracle", seconds=round(dt, 2),
                   sample=f"requests 0..{n_req - 1} of the batch: float64 link of all rows + attention of "
                          f"{'every' if every == 1 else f'every {every}th'} fresh row, all heads")

    # ---- what the matrix cores sustain on this GPU with nothing in their way, and (on request) the
    # attention launch with parts of its inner loop left out ----
    sustained = None if args.no_sustained_probe else sustained_mfma(torch, dev, not args.no_device_state)
    read_floor = None if args.no_sustained_probe else streaming_read_probe(torch, dev, dec_bytes)
    ablation = None
    if args.mfma_ceiling:
        ablation = ablation_table(args, torch, dev, sh, requests, tables, pool, n_slots, n_q, attn_flops)

    traffic = None
    tfile = os.path.join(ROOT, "profiles", "attn_traffic.json")
    if os.path.exists(tfile):
        try:
            traffic = json.load(open(tfile)).get(f"config{args.config}")
        except Exception:
            traffic = None

    rec = {
        "metric": "selective-prefill attention TFLOP/s (link + attention step)",
        "value": round(value, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic (device RNG)" if args.device_data else "synthetic",
        "config": {"workload": f"config{args.config}:{sh.name}", "batch": len(requests), "tokens_per_request": lens[0],
                   "recompute_rows": n_q, "q_heads": sh.n_q_heads, "kv_heads": sh.n_kv_heads, "head_dim": sh.head_dim,
                   "k": sh.default_k, "page_size": sh.page_size, "layer_sets": L,
                   "fresh_rows": "rotated by the library" if args.fresh_pre_rope else "handed over rotated",
                   "chunks": "HBM-resident", "plan": "built once per batch, reused by every step",
                   "overlap": ("stored rows of step i+1 linked by the attention launch of step i (trailing workgroups)" if fuse else
                               "stored rows of step i+1 linked on a second stream while step i attends")},
        "roofline": {"bound": "mfma", "achieved": round(attn_tflops, 3), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(attn_tflops / PEAK_BF16_TFLOPS, 5),
                     # HBM-side bytes per launch (FETCH_SIZE + WRITE_SIZE, scaled by the copy calibration)
                     "traffic": traffic["total_bytes"] if traffic else None, "traffic_detail": traffic,
                     "kernel": "attn_bf16_kernel<%d keys per block, NoLink> (attention alone, event-timed back-to-back launches)"
                               % (64 if not (fuse or L < 2) else args.attn_block_keys or 96),
                     "avg_launch_ms": round(attn_ms, 5),
                     "same_launch_on_zero_operands": {"avg_launch_ms": round(zero_ms, 5),
                                                      "TFLOPs": round(attn_flops / (zero_ms * 1e-3) / 1e12, 3),
                                                      "frac": round(attn_flops / (zero_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 5),
                                                      "note": "not a result: the launch with every bit of Q, K and V zero, i.e. at the "
                                                              "clock the part holds when the data paths draw no switching power"},
                     # the launch of the timed step when it is the fused one: attention + the next layer's stored rows
                     "fused_launch": None if fused_launch_ms is None else {
                         "kernel": "attn_bf16_kernel<%d keys per block, LinkNext>" % (args.attn_block_keys or 96),
                         "avg_launch_ms": round(fused_launch_ms, 5),
                         "TFLOPs": round(attn_flops / (fused_launch_ms * 1e-3) / 1e12, 3),
                         "frac": round(attn_flops / (fused_launch_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 5),
                         "linked_bytes": asm_bytes * (1.0 - n_q / max(1, n_ctx))},
                     # beside frac, never instead of it: the same rate against what this GPU's matrix cores sustain
                     "sustained": sustained,
                     "frac_of_sustained_mfma": None if not sustained else round(attn_tflops / sustained["mfma_only_TFLOPs"], 5),
                     "frac_of_sustained_mfma_with_softmax_and_lds_reads": None if not sustained else round(
                         attn_tflops / sustained["mfma_pingpong_softmax_lds_reads_TFLOPs"], 5),
                     "frac_of_sustained_mfma_with_softmax_mix": None if not sustained else
                     round(attn_tflops / sustained["mfma_pingpong_softmax_TFLOPs"], 5),
                     "ablation": ablation},
        "cpu_baseline": cpu,
        "attention": {"ms": round(attn_ms, 5), "ms_median": round(float(np.median(attn_each)), 5),
                      "ms_min": round(float(attn_each.min()), 5), "TFLOPs": round(attn_tflops, 3),
                      "pct_mfma_peak": round(100 * attn_tflops / PEAK_BF16_TFLOPS, 3), "flops": attn_flops},
        "assembly": {"ms": round(asm_ms, 5), "GBps": round(asm_gbs, 2), "pct_hbm_peak": round(100 * asm_gbs / PEAK_HBM_GBS, 3),
                     "bytes": asm_bytes},
        "decode_step": {"ms": round(dec_ms, 5), "GBps": round(dec_gbs, 2), "pct_hbm_peak": round(100 * dec_gbs / PEAK_HBM_GBS, 3),
                        "bytes": dec_bytes, "note": "one query per request over the linked context plus itself; two launches",
                        # beside pct_hbm_peak, never instead of it: a launch that only reads the same number of bytes
                        "read_only_launch": read_floor,
                        "frac_of_read_only_launch": None if not read_floor else round(read_floor["ms"] / dec_ms, 4)},
        "k_distance": kd,
        "in_place_step": None if in_place is None else dict(
            in_place, TFLOPs=round(attn_flops / (in_place["ms_per_step"] * 1e-3) / 1e12, 3),
            attention_TFLOPs=round(attn_flops / (in_place["attention_ms"] * 1e-3) / 1e12, 3),
            linking_bytes_per_step_linked=asm_bytes, linking_bytes_per_step_in_place=4.0 * n_q * row_bytes),
        "other_schedule_step_ms": None if other_ms is None else round(other_ms, 5),
        "graph_replay_step_ms": round(graph_ms, 5),
        "plan_ms": round(plan_ms, 4),
        "first_layer_ms": round(first_layer_ms, 4),
        "first_layer_ms_warm_process": round(warm_first_layer_ms, 4),
        "host_sourced": host,
        "layer_pipeline": pipe,
        "device_state": device_state,
    }
    print(json.dumps(rec))
    return 0


if __name__ == "__main__":
    sys.exit(main())
