"""mpic_decode_attn_static: the decode step for callers that cannot allocate.  Its partial
results live in a file-scope device array of the library; the output must equal that of
mpic_decode_attn (same kernels, same splits), also on a second call with a smaller input that
finds the first call's contents in the array."""
import numpy as np
import pytest
import torch

import paper_2502_01960_amd as mpic
from helpers import Problem, assert_bf16_close, assert_f32_close

pytestmark = pytest.mark.gpu


def _both(p, with_self):
    dev = p.k_ctx.device
    q, nk, nv = (t.to(dev) for t in p.decode_inputs())
    if not with_self:
        nk = nv = None
    outs = []
    for fn in (mpic.mpic_decode_attn, mpic.mpic_decode_attn_static):
        out = torch.full(tuple(q.shape), float("nan"), dtype=p.sh.torch_dtype, device=dev)
        lse = torch.full(tuple(q.shape[:2]), float("nan"), dtype=torch.float32, device=dev)
        fn(p.ctx.handle, p.plan.handle, q, nk, nv, p.k_ctx, p.v_ctx, p.sh.softmax_scale, out, lse)
        torch.cuda.synchronize()
        outs.append((out, lse))
    (o0, l0), (o1, l1) = outs
    assert not torch.isnan(o1.float()).any()
    # same kernels, same split of the keys: identical bits
    assert torch.equal(o0.view(torch.int16 if o0.element_size() == 2 else torch.int32),
                       o1.view(torch.int16 if o1.element_size() == 2 else torch.int32))
    assert torch.equal(l0, l1)
    return q, nk, nv, o1


def test_static_scratch_decode_equals_the_allocating_one():
    big = Problem(3, n_chunks=3, chunk_len=301, text_len=37, batch=2)       # several splits per request
    small = Problem(4, k=16, n_chunks=2, chunk_len=160, text_len=70, batch=1)
    tiny = Problem(1)                                                       # fp32 kernels, same array
    for p in (big, small, tiny):
        p.gpu_setup(False)
    # a plan that no call has brought to the GPU is refused (the entry point may not upload it)
    with pytest.raises(mpic.MpicError):
        q0 = big.decode_inputs()[0].to("cuda:0")
        mpic.mpic_decode_attn_static(big.ctx.handle, big.plan.handle, q0, None, None, big.k_ctx, big.v_ctx,
                                     big.sh.softmax_scale, torch.empty_like(q0))
    for p in (big, small, tiny):
        p.gpu_assemble()
    # two calls in a row, the second with a smaller input, then fp32, then the first again
    for p in (big, small, tiny, big):
        for with_self in (True, False):
            q, nk, nv, out = _both(p, with_self)
        # and against the oracle, at the gates of the decode tests
        K, V = p.oracle_link()
        ref, _ = p.oracle_decode(K, V, q.cpu(), None, None)
        close = assert_f32_close if p.sh.dtype == "f32" else assert_bf16_close
        close(out.to(torch.float64).cpu().numpy(), ref, "decode output (static scratch)")


def test_static_scratch_rejects_what_does_not_fit():
    """Partial results beyond the array's 8 MiB are refused before anything is enqueued."""
    import dataclasses
    import workloads
    from test_gpu_parity import _custom
    # one short request per batch element, many heads: B * Hq * (D + 1) * 4 bytes > 8 MiB
    n_req = 140
    p = _custom([[("text", 3)] for _ in range(n_req)], 0, [], 0, sh_id=4)
    p.sh = dataclasses.replace(p.sh, n_q_heads=128, n_kv_heads=8)
    q_off = p.oplan["q_off"]
    fresh = [workloads.gen_fresh(p.sh, 0, b, int(q_off[b + 1] - q_off[b])) for b in range(n_req)]
    p.q = torch.cat([f[0] for f in fresh]); p.fresh_k = torch.cat([f[1] for f in fresh]); p.fresh_v = torch.cat([f[2] for f in fresh])
    p.gpu_setup(False)
    p.gpu_assemble()
    dev = p.k_ctx.device
    q, nk, nv = (t.to(dev) for t in p.decode_inputs())
    out = torch.full(tuple(q.shape), float("nan"), dtype=p.sh.torch_dtype, device=dev)
    with pytest.raises(mpic.MpicError) as e:
        mpic.mpic_decode_attn_static(p.ctx.handle, p.plan.handle, q, nk, nv, p.k_ctx, p.v_ctx, p.sh.softmax_scale, out)
    assert e.value.status == -2
    torch.cuda.synchronize()
    assert torch.isnan(out.float()).all()
    # the allocating entry point takes the same batch
    mpic.mpic_decode_attn(p.ctx.handle, p.plan.handle, q, nk, nv, p.k_ctx, p.v_ctx, p.sh.softmax_scale, out)
    torch.cuda.synchronize()
    assert not torch.isnan(out.float()).any()
