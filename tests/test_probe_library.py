"""The measurement aid libmpic_probe.so (bench.py --mfma-ceiling): the product library contains none
of it, and on a GPU its entry points run and its unablated attention launch is the product's."""
import ctypes
import importlib.util
import os

import numpy as np
import pytest

import paper_2502_01960_amd as mpic

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROBE = os.path.join(ROOT, "paper_2502_01960_amd", "libmpic_probe.so")
PROBE_OPTION_ABLATE = 1000


def test_product_library_has_no_probe_code():
    lib = ctypes.CDLL(mpic.lib_path())
    for name in ("mpic_probe_mfma", "mpic_probe_read"):
        assert not hasattr(lib, name), name
    ctx = mpic.Context(8, 2, 128, mpic.MPIC_BF16, 1e4)
    with pytest.raises(mpic.MpicError):
        ctx.set_option(PROBE_OPTION_ABLATE, 1)      # timing-only kernel variants exist in the probe build only
    ctx.close()


def test_probe_library_exports_what_bench_calls():
    if not os.path.exists(PROBE):
        pytest.skip("probe library not built")
    lib = ctypes.CDLL(PROBE)
    for name in ("mpic_probe_mfma", "mpic_probe_read", "mpic_selective_attn", "mpic_set_option"):
        assert hasattr(lib, name), name


def test_chunk_sources_marshalled_once_are_passed_through():
    from paper_2502_01960_amd import binding
    once = mpic.ChunkSources([(4096, 8192, 7, 0), (0, 0, 0, 0)])
    arr, n = binding._src_array(once, mpic.MPIC_SRC_HOST_STAGED)
    assert n == 2 and arr is once.arr and (arr[0].len, arr[0].on_host) == (7, 0)


@pytest.mark.gpu
def test_probe_entry_points_run_and_mask_zero_is_the_product_kernel():
    import torch
    import workloads
    if not os.path.exists(PROBE):
        pytest.skip("probe library not built")
    dev = torch.device("cuda:0")
    lib = ctypes.CDLL(PROBE)
    lib.mpic_probe_mfma.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                    ctypes.POINTER(ctypes.c_double)]
    lib.mpic_probe_read.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    stream = torch.cuda.current_stream()
    seed = torch.randn((64 * 16 * 8,), device=dev).to(torch.bfloat16)
    sink = torch.full((64 * 512 + 1,), float("nan"), dtype=torch.float32, device=dev)
    fl = ctypes.c_double()
    for flags in (0, 1, 3, 11, 4, 12):
        assert lib.mpic_probe_mfma(flags, 64, 5, seed.data_ptr(), sink.data_ptr(), stream.cuda_stream, ctypes.byref(fl)) == 0
    assert lib.mpic_probe_mfma(2, 64, 5, seed.data_ptr(), sink.data_ptr(), stream.cuda_stream, ctypes.byref(fl)) == -1
    assert lib.mpic_probe_mfma(0, 0, 5, seed.data_ptr(), sink.data_ptr(), stream.cuda_stream, ctypes.byref(fl)) == -1
    assert fl.value == 8.0 * 48.0 * 32768.0          # (= 4 * 96 * 32768 of the one-wavefront division)
    torch.cuda.synchronize()
    assert torch.isfinite(sink[:64 * 512]).all()
    buf = torch.zeros((1 << 20,), dtype=torch.int32, device=dev)
    assert lib.mpic_probe_read(buf.data_ptr(), buf.numel() * 4, 64, sink.data_ptr(), stream.cuda_stream) == 0
    assert lib.mpic_probe_read(buf.data_ptr(), 24, 64, sink.data_ptr(), stream.cuda_stream) == -1       # not a multiple of 16
    assert lib.mpic_probe_read(buf.data_ptr() + 4, 1 << 20, 64, sink.data_ptr(), stream.cuda_stream) == -1  # misaligned
    torch.cuda.synchronize()

    # the probe build's attention launch with nothing left out gives the product's output bit for bit
    spec = importlib.util.spec_from_file_location("mpic_probe_binding", os.path.join(ROOT, "paper_2502_01960_amd", "binding.py"))
    pb = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(pb)
    pb.lib_path = lambda: PROBE
    sh = workloads.shape(3)
    requests = [[("text", 40), ("chunk", 0, 300, None), ("text", 25), ("chunk", 1, 200, None), ("text", 31)]]
    n_ctx, k = 596, 16
    outs = []
    for m in (mpic, pb):
        ctx = m.Context(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, m.MPIC_BF16, sh.rope_theta)
        plan = m.Plan(ctx, requests, k)
        n_q = int(plan.get("q_off")[-1])
        gen = torch.Generator(device=dev).manual_seed(7)
        draw = lambda *s: torch.randn(s, generator=gen, device=dev).to(torch.bfloat16)
        q, kc, vc = draw(n_q, sh.n_q_heads, sh.head_dim), draw(n_ctx, sh.n_kv_heads, sh.head_dim), draw(n_ctx, sh.n_kv_heads, sh.head_dim)
        out = torch.empty_like(q)
        if m is pb:
            ctx.set_option(PROBE_OPTION_ABLATE, 0)
        m.mpic_selective_attn(ctx.handle, plan.handle, q, kc, vc, sh.softmax_scale, out, None, stream)
        torch.cuda.synchronize()
        outs.append(out.view(torch.int16).cpu().numpy())
        plan.close()
        ctx.close()
    assert np.array_equal(outs[0], outs[1])
