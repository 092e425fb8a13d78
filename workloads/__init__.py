"""Seeded synthetic inputs for the selective-recompute prefill path.

This module only *describes and draws inputs*: request layouts (ordered text
and cached-chunk segments), model shapes, page tables and N(0,1) tensors from
a counter-based generator.  It contains none of the method's arithmetic (no
selection rule, no rotation, no attention) so that the float64 oracle and the
HIP library can both be fed from it without sharing any computation.

Layouts stand in for the paper's workloads: 576- and 2304-token images of the
LLaVA-1.5 / LLaVA-1.6 families (Sec. 1), sentence- and word-level interleaving
of images and text (Sec. 5.1), one to ten images per conversation (App. C) and
retrieved references for MRAG (Sec. 3.1).  The datasets themselves are not
used; every value is i.i.d. N(0,1).

A segment is a tuple:
    ("text", L)                      L text tokens (always recomputed)
    ("chunk", src_id, L, k)          cached image chunk `src_id` of L tokens;
                                     k = None means "use the request default"
"""
from __future__ import annotations

import dataclasses
import numpy as np
import torch

SEED_BASE = 0x4D504943  # "MPIC"

# tensor tags for the generator key
TAG_CHUNK_K, TAG_CHUNK_V, TAG_Q, TAG_FRESH_K, TAG_FRESH_V, TAG_PAGES, TAG_DRAW = range(7)


@dataclasses.dataclass(frozen=True)
class Shape:
    """Model-side shape of one workload."""
    cfg_id: int
    name: str
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str            # "f32" or "bf16": storage type of every tensor
    rope_theta: float
    default_k: int
    page_size: int        # 0 = contiguous context
    host_sourced: bool    # cached chunks live in pinned host memory
    batch: int
    layers: int
    q_prescale: float     # factor folded into Q by the generator
    softmax_scale: float  # scale handed to the attention call

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


def shape(cfg_id: int) -> Shape:
    d128 = 1.0 / np.sqrt(128.0)
    if cfg_id == 1:
        return Shape(1, "tiny-f32", 4, 4, 64, "f32", 1.0e4, 8, 0, False, 1, 1, 1.0, 1.0 / 8.0)
    if cfg_id == 2:
        # Q is pre-multiplied by 1/sqrt(128) and the call uses scale 1.
        return Shape(2, "llava15-like", 32, 32, 128, "bf16", 1.0e4, 32, 0, False, 1, 1, d128, 1.0)
    if cfg_id == 3:
        return Shape(3, "llava16-like-18k", 28, 4, 128, "bf16", 1.0e6, 64, 0, True, 4, 1, 1.0, d128)
    if cfg_id == 4:
        return Shape(4, "mrag", 32, 8, 128, "bf16", 5.0e5, 64, 0, False, 8, 32, 1.0, d128)
    if cfg_id == 5:
        return Shape(5, "long-paged", 64, 8, 128, "bf16", 1.0e6, 32, 16, True, 1, 1, 1.0, d128)
    raise ValueError(f"unknown config {cfg_id}")


def _interleaved(n_chunks, chunk_len, text_len, first_src, tail=()):
    segs = []
    for c in range(n_chunks):
        segs.append(("text", text_len))
        segs.append(("chunk", first_src + c, chunk_len, None))
    segs.append(("text", text_len))
    for t in tail:
        segs.append(("text", t))
    return segs


def _rng(cfg_id, layer, tag, ident):
    key = np.array([(SEED_BASE << 32) | (cfg_id & 0xFFFFFFFF),
                    ((layer & 0xFFFF) << 48) | ((tag & 0xFF) << 40) | (ident & 0xFFFFFFFFFF)],
                   dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def layout(cfg_id: int, *, n_chunks=None, chunk_len=None, text_len=None, batch=None):
    """Per-request segment lists and the number of distinct chunk sources.

    Keyword overrides shrink a configuration for tests while keeping its
    structure.  Returns (requests, n_sources, source_lengths).
    """
    sh = shape(cfg_id)
    B = sh.batch if batch is None else batch
    if cfg_id == 1:
        reqs = [[("text", 16), ("chunk", 0, 64, None), ("text", 8),
                 ("chunk", 1, 64, None), ("text", 8)]]
        return reqs, 2, [64, 64]
    if cfg_id == 2:
        n = 4 if n_chunks is None else n_chunks
        L = 576 if chunk_len is None else chunk_len
        T = 64 if text_len is None else text_len
        return [_interleaved(n, L, T, 0)], n, [L] * n
    if cfg_id == 3:
        n = 8 if n_chunks is None else n_chunks
        L = 2304 if chunk_len is None else chunk_len
        T = 128 if text_len is None else text_len
        reqs = [_interleaved(n, L, T, b * n, tail=(2 * T,)) for b in range(B)]
        return reqs, n * B, [L] * (n * B)
    if cfg_id == 4:
        n = 16 if n_chunks is None else n_chunks
        L = 1024 if chunk_len is None else chunk_len
        T = 512 if text_len is None else text_len
        pool = 4 * n
        reqs = []
        for b in range(B):
            draw = _rng(cfg_id, 0, TAG_DRAW, b).permutation(pool)[:n]
            segs = [("chunk", int(c), L, None) for c in draw]
            segs.append(("text", T))
            reqs.append(segs)
        return reqs, pool, [L] * pool
    if cfg_id == 5:
        n = 32 if n_chunks is None else n_chunks
        L = 2304 if chunk_len is None else chunk_len
        T = 64 if text_len is None else text_len
        reqs = [_interleaved(n, L, T, b * n) for b in range(B)]
        return reqs, n * B, [L] * (n * B)
    raise ValueError(f"unknown config {cfg_id}")


def request_len(segs) -> int:
    return sum(s[1] if s[0] == "text" else s[2] for s in segs)


def _normal(cfg_id, layer, tag, ident, shape_, dtype, scale=1.0):
    x = _rng(cfg_id, layer, tag, ident).standard_normal(shape_, dtype=np.float32)
    if scale != 1.0:
        x *= np.float32(scale)
    return torch.from_numpy(x).to(dtype)  # bf16: one round-to-nearest-even


def gen_chunk(sh: Shape, layer: int, src_id: int, length: int):
    """Cached K and V of one chunk: [length][n_kv_heads][head_dim] each."""
    dims = (length, sh.n_kv_heads, sh.head_dim)
    k = _normal(sh.cfg_id, layer, TAG_CHUNK_K, src_id, dims, sh.torch_dtype)
    v = _normal(sh.cfg_id, layer, TAG_CHUNK_V, src_id, dims, sh.torch_dtype)
    return k, v


def gen_fresh(sh: Shape, layer: int, request: int, n_q: int):
    """Fresh Q [n_q][Hq][D], K and V [n_q][Hkv][D] of one request's recompute set."""
    q = _normal(sh.cfg_id, layer, TAG_Q, request, (n_q, sh.n_q_heads, sh.head_dim),
                sh.torch_dtype, sh.q_prescale)
    k = _normal(sh.cfg_id, layer, TAG_FRESH_K, request, (n_q, sh.n_kv_heads, sh.head_dim),
                sh.torch_dtype)
    v = _normal(sh.cfg_id, layer, TAG_FRESH_V, request, (n_q, sh.n_kv_heads, sh.head_dim),
                sh.torch_dtype)
    return q, k, v


def gen_page_tables(sh: Shape, request_lens, page_size=None, slack=1.25):
    """One shared pool of physical pages, handed out to the requests of a batch in a
    seeded random order (non-contiguous, non-monotone).  Returns (tables, n_pool_pages).
    """
    ps = sh.page_size if page_size is None else page_size
    need = [(n + ps - 1) // ps for n in request_lens]
    pool = max(1, int(np.ceil(slack * sum(need))))
    perm = _rng(sh.cfg_id, 0, TAG_PAGES, len(request_lens)).permutation(pool).astype(np.int32)
    tables, at = [], 0
    for n in need:
        tables.append(np.ascontiguousarray(perm[at:at + n]))
        at += n
    return tables, pool
