"""ctypes binding of libmpic.so.  The functions carry the names of the C entry points
declared in include/mpic.h and only marshal arguments; Context / Plan are thin
owners of the opaque handles.  There is no fallback: a missing library raises."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
MPIC_F32, MPIC_BF16 = 0, 1

PLAN_FIELDS = dict(ctx_off=0, q_off=1, q_pos=2, q_req=3, slot_map=4, src_inst=5, src_row=6,
                   dst_slot=7, inst_src=8, inst_delta=9, inst_len=10, inst_k=11, inst_req=12,
                   runs=13, attn_tiles=14, launch_estimate=15, key_blocks_32=16, key_blocks_64=17,
                   key_blocks_96=18, lazy_tiles_64=19, lazy_tiles_96=20, key_block_parts_32=21,
                   key_block_parts_64=22, key_block_parts_96=23)


class MpicError(RuntimeError):
    def __init__(self, status, detail=""):
        self.status = status
        super().__init__(f"libmpic status {status} ({mpic_strerror(status)}): {detail}")


class _Config(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("dtype", C.c_int32), ("rope_theta", C.c_double), ("rope_interleaved", C.c_int32),
                ("page_size", C.c_int32), ("fresh_pre_rope", C.c_int32), ("lazy_rope", C.c_int32)]


class _Segment(C.Structure):
    _fields_ = [("kind", C.c_int32), ("len", C.c_int32), ("chunk", C.c_int32), ("k", C.c_int32)]


class _ChunkSrc(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("len", C.c_int32), ("on_host", C.c_int32)]


def lib_path():
    return os.path.join(_HERE, "libmpic.so")


_lib = None


def load_library():
    """Load libmpic.so (built by paper_2502_01960_amd/build.py).  Raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} not found: build it with `python paper_2502_01960_amd/build.py`")
    lib = C.CDLL(path)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.mpic_create.argtypes = [C.POINTER(vp), C.POINTER(_Config)]
    lib.mpic_create.restype = C.c_int
    lib.mpic_set_option.argtypes = [vp, i32, i64]
    lib.mpic_set_option.restype = C.c_int
    lib.mpic_destroy.argtypes = [vp]
    lib.mpic_destroy.restype = None
    lib.mpic_plan_create.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(_Segment), i32,
                                     C.POINTER(i32), C.POINTER(i32), i64, C.POINTER(vp)]
    lib.mpic_plan_create.restype = C.c_int
    lib.mpic_plan_create_selected.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(_Segment), i32,
                                              C.POINTER(i32), C.POINTER(i32),
                                              C.POINTER(i32), C.POINTER(i32), i64, C.POINTER(vp)]
    lib.mpic_plan_create_selected.restype = C.c_int
    lib.mpic_plan_get.argtypes = [vp, i32, C.POINTER(C.POINTER(i32)), C.POINTER(C.c_size_t)]
    lib.mpic_plan_get.restype = C.c_int
    lib.mpic_plan_get_rope.argtypes = [vp, C.POINTER(C.POINTER(C.c_float)),
                                       C.POINTER(C.POINTER(C.c_float)), C.POINTER(C.c_size_t)]
    lib.mpic_plan_get_rope.restype = C.c_int
    lib.mpic_plan_get_fresh_rope.argtypes = [vp, C.POINTER(C.POINTER(i32)), C.POINTER(C.POINTER(C.c_float)),
                                             C.POINTER(C.POINTER(C.c_float)), C.POINTER(C.c_size_t)]
    lib.mpic_plan_get_fresh_rope.restype = C.c_int
    lib.mpic_plan_destroy.argtypes = [vp]
    lib.mpic_plan_destroy.restype = None
    lib.mpic_assemble_kv.argtypes = [vp, vp, C.POINTER(_ChunkSrc), i32, vp, vp, i64, vp, vp, i64, vp]
    lib.mpic_assemble_kv.restype = C.c_int
    lib.mpic_assemble_kv_parts.argtypes = [vp, vp, C.POINTER(_ChunkSrc), i32, vp, vp, i64, vp, vp, i64, C.c_uint32, vp]
    lib.mpic_assemble_kv_parts.restype = C.c_int
    lib.mpic_selective_attn.argtypes = [vp, vp, vp, i64, vp, vp, i64, C.c_double, vp, vp, vp]
    lib.mpic_selective_attn.restype = C.c_int
    lib.mpic_selective_attn_link_next.argtypes = [vp, vp, vp, i64, vp, vp, i64, C.c_double, vp, vp,
                                                  C.POINTER(_ChunkSrc), i32, vp, vp, vp]
    lib.mpic_selective_attn_link_next.restype = C.c_int
    lib.mpic_decode_attn.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, C.c_double, vp, vp, vp]
    lib.mpic_decode_attn.restype = C.c_int
    lib.mpic_selective_attn_in_place.argtypes = [vp, vp, vp, i64, C.POINTER(_ChunkSrc), i32, vp, vp, i64, C.c_double,
                                                 vp, vp, vp]
    lib.mpic_selective_attn_in_place.restype = C.c_int
    lib.mpic_decode_attn_in_place.argtypes = [vp, vp, vp, vp, vp, C.POINTER(_ChunkSrc), i32, vp, vp, i64, C.c_double,
                                              vp, vp, vp]
    lib.mpic_decode_attn_in_place.restype = C.c_int
    lib.mpic_decode_attn_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, C.c_double, vp, vp, vp]
    lib.mpic_decode_attn_static.restype = C.c_int
    lib.mpic_k_distance.argtypes = [vp, vp, vp, i64, vp, vp]
    lib.mpic_k_distance.restype = C.c_int
    lib.mpic_rank_tokens.argtypes = [C.POINTER(C.c_float), i64, i64, C.POINTER(i32)]
    lib.mpic_rank_tokens.restype = C.c_int
    u64 = C.c_uint64
    lib.mpic_store_create.argtypes = [vp, i32, C.c_char_p, i32, C.POINTER(vp)]
    lib.mpic_store_create.restype = C.c_int
    lib.mpic_store_destroy.argtypes = [vp]
    lib.mpic_store_destroy.restype = None
    lib.mpic_store_put.argtypes = [vp, u64, i32, vp, vp, i32, i64]
    lib.mpic_store_put.restype = C.c_int
    lib.mpic_store_move.argtypes = [vp, u64, i32]
    lib.mpic_store_move.restype = C.c_int
    lib.mpic_store_expire.argtypes = [vp, i64, C.POINTER(i32)]
    lib.mpic_store_expire.restype = C.c_int
    lib.mpic_store_drop.argtypes = [vp, u64]
    lib.mpic_store_drop.restype = C.c_int
    lib.mpic_store_lookup.argtypes = [vp, C.POINTER(u64), i32, C.POINTER(i32), C.POINTER(i32)]
    lib.mpic_store_lookup.restype = C.c_int
    lib.mpic_store_layer.argtypes = [vp, u64, i32, C.POINTER(_ChunkSrc)]
    lib.mpic_store_layer.restype = C.c_int
    lib.mpic_prefill_layers.argtypes = [vp, vp, vp, C.POINTER(u64), i32, i32, C.POINTER(vp), C.POINTER(vp),
                                        C.POINTER(vp), i64, C.POINTER(vp), C.POINTER(vp), i64, C.c_double,
                                        C.POINTER(vp), C.POINTER(vp), vp, C.POINTER(i32)]
    lib.mpic_prefill_layers.restype = C.c_int
    lib.mpic_strerror.argtypes = [C.c_int]
    lib.mpic_strerror.restype = C.c_char_p
    lib.mpic_last_error.argtypes = [vp]
    lib.mpic_last_error.restype = C.c_char_p
    _lib = lib
    return lib


# ---------------------------------------------------------------- C entry points
def mpic_strerror(status):
    return load_library().mpic_strerror(int(status)).decode()


def mpic_last_error(ctx):
    return load_library().mpic_last_error(ctx).decode()


def _check(rc, ctx=None):
    if rc != 0:
        raise MpicError(rc, mpic_last_error(ctx) if ctx else "")


def mpic_create(n_q_heads, n_kv_heads, head_dim, dtype, rope_theta, rope_interleaved=0, page_size=0,
                fresh_pre_rope=0, lazy_rope=0):
    cfg = _Config(n_q_heads, n_kv_heads, head_dim, dtype, rope_theta, rope_interleaved, page_size,
                  fresh_pre_rope, lazy_rope)
    h = C.c_void_p()
    _check(load_library().mpic_create(C.byref(h), C.byref(cfg)))
    return h


def mpic_destroy(ctx):
    load_library().mpic_destroy(ctx)


MPIC_OPT_ATTN_BLOCK_KEYS = 1


def mpic_set_option(ctx, option, value):
    _check(load_library().mpic_set_option(ctx, int(option), int(value)), ctx)


def _i32_array(values):
    arr = np.ascontiguousarray(values, dtype=np.int32)
    return arr, arr.ctypes.data_as(C.POINTER(C.c_int32))


MPIC_K_LISTED = -2


def mpic_plan_create(ctx, requests, default_k, page_tables=None, n_pool_pages=0):
    """requests: list of segment lists, ("text", L) / ("chunk", src, L, k or None); k may be a
    sequence of chunk-local token indices, in which case mpic_plan_create_selected is called."""
    seg_off, flat = [0], []
    sel_off, sel_idx, listed = [0], [], False
    for segs in requests:
        for s in segs:
            if s[0] == "text":
                flat.append(_Segment(0, s[1], 0, -1))
            elif s[0] == "chunk":
                k = s[3]
                if k is None or isinstance(k, (int, np.integer)):
                    flat.append(_Segment(1, s[2], s[1], -1 if k is None else int(k)))
                else:
                    flat.append(_Segment(1, s[2], s[1], MPIC_K_LISTED))
                    sel_idx.extend(int(t) for t in k)
                    listed = True
            else:
                raise ValueError(f"unknown segment kind {s[0]!r}")
            sel_off.append(len(sel_idx))
        seg_off.append(len(flat))
    segs_c = (_Segment * max(1, len(flat)))(*flat)
    off_keep, off_p = _i32_array(seg_off)
    if page_tables is not None:
        pt_off = np.cumsum([0] + [len(t) for t in page_tables])
        pt_keep, pt_p = _i32_array(np.concatenate([np.asarray(t, dtype=np.int32) for t in page_tables])
                                   if len(page_tables) else [])
        pto_keep, pto_p = _i32_array(pt_off)
    else:
        pt_p = pto_p = None
    h = C.c_void_p()
    if listed:
        so_keep, so_p = _i32_array(sel_off)
        si_keep, si_p = _i32_array(sel_idx)
        rc = load_library().mpic_plan_create_selected(ctx, len(requests), off_p, segs_c, default_k, so_p, si_p,
                                                      pt_p, pto_p, n_pool_pages, C.byref(h))
    else:
        rc = load_library().mpic_plan_create(ctx, len(requests), off_p, segs_c, default_k, pt_p, pto_p,
                                             n_pool_pages, C.byref(h))
    _check(rc, ctx)
    return h


def mpic_plan_get(plan, what):
    """Copy of one int32 array of the plan (runs -> [n][4], attn_tiles -> [n][8])."""
    code = PLAN_FIELDS[what] if isinstance(what, str) else int(what)
    p = C.POINTER(C.c_int32)()
    n = C.c_size_t()
    _check(load_library().mpic_plan_get(plan, code, C.byref(p), C.byref(n)))
    out = np.ctypeslib.as_array(p, shape=(n.value,)).copy() if n.value else np.zeros(0, np.int32)
    if code == PLAN_FIELDS["runs"]:
        out = out.reshape(-1, 4)
    elif code == PLAN_FIELDS["attn_tiles"]:
        out = out.reshape(-1, 8)
    elif code in (PLAN_FIELDS["key_blocks_32"], PLAN_FIELDS["key_blocks_64"], PLAN_FIELDS["key_blocks_96"],
                  PLAN_FIELDS["lazy_tiles_64"], PLAN_FIELDS["lazy_tiles_96"]):
        out = out.reshape(-1, 4)
    elif code in (PLAN_FIELDS["key_block_parts_32"], PLAN_FIELDS["key_block_parts_64"], PLAN_FIELDS["key_block_parts_96"]):
        out = out.reshape(-1, 3)
    return out


def mpic_plan_get_rope(plan):
    c, s, n = C.POINTER(C.c_float)(), C.POINTER(C.c_float)(), C.c_size_t()
    _check(load_library().mpic_plan_get_rope(plan, C.byref(c), C.byref(s), C.byref(n)))
    if not n.value:
        return np.zeros(0, np.float32), np.zeros(0, np.float32)
    return (np.ctypeslib.as_array(c, shape=(n.value,)).copy(),
            np.ctypeslib.as_array(s, shape=(n.value,)).copy())


def mpic_plan_get_fresh_rope(plan, n_fresh_rows, half_dim):
    """(table_row [Nq], cos [n_rows][D/2], sin [n_rows][D/2]) of a fresh_pre_rope context."""
    idx, c, s, n = C.POINTER(C.c_int32)(), C.POINTER(C.c_float)(), C.POINTER(C.c_float)(), C.c_size_t()
    _check(load_library().mpic_plan_get_fresh_rope(plan, C.byref(idx), C.byref(c), C.byref(s), C.byref(n)))
    if not n.value:
        return np.zeros(0, np.int32), np.zeros((0, half_dim), np.float32), np.zeros((0, half_dim), np.float32)
    return (np.ctypeslib.as_array(idx, shape=(n_fresh_rows,)).copy(),
            np.ctypeslib.as_array(c, shape=(n.value, half_dim)).copy(),
            np.ctypeslib.as_array(s, shape=(n.value, half_dim)).copy())


def mpic_plan_destroy(plan):
    load_library().mpic_plan_destroy(plan)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    return C.c_void_p(getattr(stream, "cuda_stream", stream))


MPIC_PART_CACHED, MPIC_PART_FRESH, MPIC_PART_BACKGROUND = 1, 2, 4
MPIC_SRC_DEVICE, MPIC_SRC_HOST_STAGED, MPIC_SRC_HOST_MAPPED = 0, 1, 2


def mpic_assemble_kv(ctx, plan, srcs, fresh_k, fresh_v, k_ctx, v_ctx, stream=None, host_mode=MPIC_SRC_HOST_STAGED):
    """srcs: list of (k_tensor, v_tensor) per source id; a device tensor is read in place, a
    pinned CPU tensor is staged by the library (host_mode = MPIC_SRC_HOST_STAGED) or read in
    place by the kernel (MPIC_SRC_HOST_MAPPED).  Tensors are torch tensors.  An entry may also
    be the 4-tuple (k address, v address, len, on_host) that mpic_store_layer returns."""
    mpic_assemble_kv_parts(ctx, plan, srcs, fresh_k, fresh_v, k_ctx, v_ctx,
                           MPIC_PART_CACHED | MPIC_PART_FRESH, stream, host_mode)


class ChunkSources:
    """Chunk sources marshalled once (the mpic_chunk_src array of a list as mpic_assemble_kv takes
    it), for callers that hand the same list to many calls: pass the object wherever a list of
    sources is accepted.  It keeps the tensors alive."""

    def __init__(self, srcs, host_mode=MPIC_SRC_HOST_STAGED):
        self.arr, self.n = _src_array(list(srcs or []), host_mode)
        self.keep = srcs


def _src_array(srcs, host_mode):
    if isinstance(srcs, ChunkSources):
        return srcs.arr, srcs.n
    srcs = srcs or []
    arr = (_ChunkSrc * max(1, len(srcs)))()
    for i, src in enumerate(srcs):
        if len(src) == 4:      # (k address, v address, len, on_host) as mpic_store_layer returns them
            arr[i] = _ChunkSrc(*src)
            continue
        k, v = src
        if k is None:
            arr[i] = _ChunkSrc(None, None, 0, 0)
            continue
        on_host = MPIC_SRC_DEVICE if k.is_cuda else int(host_mode)
        if on_host and not (k.is_pinned() and v.is_pinned()):
            raise ValueError("host chunk sources must be pinned")
        arr[i] = _ChunkSrc(k.data_ptr(), v.data_ptr(), k.shape[0], on_host)
    return arr, len(srcs)


def mpic_assemble_kv_parts(ctx, plan, srcs, fresh_k, fresh_v, k_ctx, v_ctx, parts, stream=None,
                           host_mode=MPIC_SRC_HOST_STAGED):
    arr, n_srcs = _src_array(srcs, host_mode)
    n_fresh = 0 if fresh_k is None else fresh_k.shape[0]
    rc = load_library().mpic_assemble_kv_parts(ctx, plan, arr, n_srcs, _ptr(fresh_k), _ptr(fresh_v), n_fresh,
                                               _ptr(k_ctx), _ptr(v_ctx), k_ctx.shape[0], int(parts),
                                               _stream(stream))
    _check(rc, ctx)


def mpic_selective_attn(ctx, plan, fresh_q, k_ctx, v_ctx, softmax_scale, out, lse=None, stream=None):
    n_fresh = 0 if fresh_q is None else fresh_q.shape[0]
    rc = load_library().mpic_selective_attn(ctx, plan, _ptr(fresh_q), n_fresh, _ptr(k_ctx), _ptr(v_ctx),
                                            k_ctx.shape[0], float(softmax_scale), _ptr(out), _ptr(lse),
                                            _stream(stream))
    _check(rc, ctx)


def mpic_selective_attn_in_place(ctx, plan, fresh_q, srcs, k_ctx, v_ctx, softmax_scale, out, lse=None, stream=None):
    """Attention over caches linked by reference (lazy_rope contexts): stored rows are read in `srcs`."""
    arr, n_srcs = _src_array(srcs, MPIC_SRC_HOST_STAGED)
    n_fresh = 0 if fresh_q is None else fresh_q.shape[0]
    rc = load_library().mpic_selective_attn_in_place(ctx, plan, _ptr(fresh_q), n_fresh, arr, n_srcs, _ptr(k_ctx),
                                                     _ptr(v_ctx), k_ctx.shape[0], float(softmax_scale), _ptr(out),
                                                     _ptr(lse), _stream(stream))
    _check(rc, ctx)


def mpic_decode_attn_in_place(ctx, plan, q, new_k, new_v, srcs, k_ctx, v_ctx, softmax_scale, out, lse=None, stream=None):
    arr, n_srcs = _src_array(srcs, MPIC_SRC_HOST_STAGED)
    rc = load_library().mpic_decode_attn_in_place(ctx, plan, _ptr(q), _ptr(new_k), _ptr(new_v), arr, n_srcs,
                                                  _ptr(k_ctx), _ptr(v_ctx), 0 if k_ctx is None else k_ctx.shape[0],
                                                  float(softmax_scale), _ptr(out), _ptr(lse), _stream(stream))
    _check(rc, ctx)


def mpic_selective_attn_link_next(ctx, plan, fresh_q, k_ctx, v_ctx, softmax_scale, out, next_srcs, next_k_ctx,
                                  next_v_ctx, lse=None, stream=None, host_mode=MPIC_SRC_HOST_STAGED):
    """Attention of one layer plus the stored rows of the next layer's context in one launch."""
    arr, n_srcs = _src_array(next_srcs, host_mode)
    n_fresh = 0 if fresh_q is None else fresh_q.shape[0]
    rc = load_library().mpic_selective_attn_link_next(ctx, plan, _ptr(fresh_q), n_fresh, _ptr(k_ctx), _ptr(v_ctx),
                                                      k_ctx.shape[0], float(softmax_scale), _ptr(out), _ptr(lse),
                                                      arr, n_srcs, _ptr(next_k_ctx), _ptr(next_v_ctx),
                                                      _stream(stream))
    _check(rc, ctx)


def mpic_decode_attn(ctx, plan, q, new_k, new_v, k_ctx, v_ctx, softmax_scale, out, lse=None, stream=None):
    rc = load_library().mpic_decode_attn(ctx, plan, _ptr(q), _ptr(new_k), _ptr(new_v), _ptr(k_ctx), _ptr(v_ctx),
                                         0 if k_ctx is None else k_ctx.shape[0], float(softmax_scale),
                                         _ptr(out), _ptr(lse), _stream(stream))
    _check(rc, ctx)


def mpic_decode_attn_static(ctx, plan, q, new_k, new_v, k_ctx, v_ctx, softmax_scale, out, lse=None, stream=None):
    """mpic_decode_attn with its partial results in the library's static device array (no allocation)."""
    rc = load_library().mpic_decode_attn_static(ctx, plan, _ptr(q), _ptr(new_k), _ptr(new_v), _ptr(k_ctx),
                                                _ptr(v_ctx), 0 if k_ctx is None else k_ctx.shape[0],
                                                float(softmax_scale), _ptr(out), _ptr(lse), _stream(stream))
    _check(rc, ctx)


def mpic_k_distance(ctx, k_a, k_b, dist, stream=None):
    rc = load_library().mpic_k_distance(ctx, _ptr(k_a), _ptr(k_b), k_a.shape[0], _ptr(dist), _stream(stream))
    _check(rc, ctx)


def mpic_rank_tokens(dist, n_top):
    """dist: host float32 array; returns the ascending indices of the n_top largest entries."""
    d = np.ascontiguousarray(dist, dtype=np.float32)
    out = np.zeros(max(0, min(int(n_top), len(d))), dtype=np.int32)
    rc = load_library().mpic_rank_tokens(d.ctypes.data_as(C.POINTER(C.c_float)), len(d), int(n_top),
                                         out.ctypes.data_as(C.POINTER(C.c_int32)))
    _check(rc)
    return out


MPIC_TIER_MISSING, MPIC_TIER_HBM, MPIC_TIER_HOST, MPIC_TIER_DISK = 0, 1, 2, 3
MPIC_ERR_IO, MPIC_ERR_CACHE_MISS = -5, -6


def mpic_store_create(ctx, n_layers, disk_dir=None, io_threads=0):
    h = C.c_void_p()
    d = None if disk_dir is None else str(disk_dir).encode()
    _check(load_library().mpic_store_create(ctx, int(n_layers), d, int(io_threads), C.byref(h)), ctx)
    return h


def mpic_store_destroy(store):
    load_library().mpic_store_destroy(store)


def mpic_store_put(ctx, store, chunk_id, k, v, tier, expires_at=-1):
    """k, v: contiguous host arrays or CPU tensors [n_layers][len][Hkv][D] of the storage type."""
    def addr(x):
        return x.data_ptr() if hasattr(x, "data_ptr") else x.ctypes.data

    def contiguous(x):
        return x.is_contiguous() if hasattr(x, "is_contiguous") else x.flags["C_CONTIGUOUS"]
    if tuple(k.shape) != tuple(v.shape) or len(k.shape) != 4 or not (contiguous(k) and contiguous(v)):
        raise ValueError("k and v must be contiguous [n_layers][len][Hkv][D] arrays of one shape")
    if getattr(k, "is_cuda", False) or getattr(v, "is_cuda", False):
        raise ValueError("mpic_store_put takes host memory")
    _check(load_library().mpic_store_put(store, int(chunk_id), int(k.shape[1]), C.c_void_p(addr(k)),
                                         C.c_void_p(addr(v)), int(tier), int(expires_at)), ctx)


def mpic_store_move(ctx, store, chunk_id, tier):
    _check(load_library().mpic_store_move(store, int(chunk_id), int(tier)), ctx)


def mpic_store_expire(ctx, store, now):
    n = C.c_int32()
    _check(load_library().mpic_store_expire(store, int(now), C.byref(n)), ctx)
    return n.value


def mpic_store_drop(ctx, store, chunk_id):
    _check(load_library().mpic_store_drop(store, int(chunk_id)), ctx)


def mpic_store_lookup(ctx, store, ids):
    """Returns (tiers, lens) as lists."""
    n = len(ids)
    a = (C.c_uint64 * max(1, n))(*[int(i) for i in ids])
    tier, length = (C.c_int32 * max(1, n))(), (C.c_int32 * max(1, n))()
    _check(load_library().mpic_store_lookup(store, a, n, tier, length), ctx)
    return list(tier[:n]), list(length[:n])


def mpic_store_layer(ctx, store, chunk_id, layer):
    """Returns (k address, v address, len, on_host) of one layer of a cache held in memory."""
    src = _ChunkSrc()
    _check(load_library().mpic_store_layer(store, int(chunk_id), int(layer), C.byref(src)), ctx)
    return src.k, src.v, src.len, src.on_host


def mpic_prefill_layers(ctx, plan, store, ids, fresh_q, fresh_k, fresh_v, k_ctx, v_ctx, softmax_scale, out,
                        lse=None, stream=None):
    """Per-layer lists of torch device tensors.  Returns None, or on a cache miss the list of
    source indices whose cache is missing or failed to load (MPIC_ERR_CACHE_MISS)."""
    n_layers = len(fresh_q)
    vp = C.c_void_p

    def ptrs(ts):
        return (vp * max(1, n_layers))(*[None if t is None else t.data_ptr() for t in ts])
    n_srcs = len(ids)
    a = (C.c_uint64 * max(1, n_srcs))(*[int(i) for i in ids])
    failed = (C.c_int32 * max(1, n_srcs))()
    n_fresh = fresh_q[0].shape[0] if n_layers else 0
    n_slots = k_ctx[0].shape[0] if n_layers else 0
    rc = load_library().mpic_prefill_layers(ctx, plan, store, a, n_srcs, n_layers, ptrs(fresh_q), ptrs(fresh_k),
                                            ptrs(fresh_v), n_fresh, ptrs(k_ctx), ptrs(v_ctx), n_slots,
                                            float(softmax_scale), ptrs(out), None if lse is None else ptrs(lse),
                                            _stream(stream), failed)
    if rc == MPIC_ERR_CACHE_MISS:
        return [s for s in range(n_srcs) if failed[s]]
    _check(rc, ctx)
    return None


# ---------------------------------------------------------------- handle owners
class Context:
    def __init__(self, n_q_heads, n_kv_heads, head_dim, dtype, rope_theta, rope_interleaved=0, page_size=0,
                 fresh_pre_rope=0, lazy_rope=0):
        self.handle = mpic_create(n_q_heads, n_kv_heads, head_dim, dtype, rope_theta, rope_interleaved, page_size,
                                  fresh_pre_rope, lazy_rope)
        self.n_q_heads, self.n_kv_heads, self.head_dim = n_q_heads, n_kv_heads, head_dim
        self.dtype, self.page_size = dtype, page_size

    def set_option(self, option, value):
        mpic_set_option(self.handle, option, value)

    def close(self):
        if self.handle is not None:
            mpic_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Plan:
    def __init__(self, ctx: Context, requests, default_k, page_tables=None, n_pool_pages=0):
        self.ctx = ctx  # keeps the context alive
        self.handle = mpic_plan_create(ctx.handle, requests, default_k, page_tables, n_pool_pages)

    def get(self, what):
        return mpic_plan_get(self.handle, what)

    def rope(self):
        return mpic_plan_get_rope(self.handle)

    def fresh_rope(self):
        return mpic_plan_get_fresh_rope(self.handle, len(self.get("q_pos")), self.ctx.head_dim // 2)

    def as_dict(self):
        return {k: self.get(k) for k in PLAN_FIELDS}

    def close(self):
        if self.handle is not None:
            mpic_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Store:
    """Owner of an mpic_store handle (destroy it before its Context)."""

    def __init__(self, ctx: Context, n_layers, disk_dir=None, io_threads=0):
        self.ctx = ctx
        self.n_layers = int(n_layers)
        self.handle = mpic_store_create(ctx.handle, n_layers, disk_dir, io_threads)

    def put(self, chunk_id, k, v, tier, expires_at=-1):
        if k.shape[0] != self.n_layers or tuple(k.shape[2:]) != (self.ctx.n_kv_heads, self.ctx.head_dim):
            raise ValueError("cache shape must be [n_layers][len][Hkv][D] of this store")
        mpic_store_put(self.ctx.handle, self.handle, chunk_id, k, v, tier, expires_at)

    def move(self, chunk_id, tier):
        mpic_store_move(self.ctx.handle, self.handle, chunk_id, tier)

    def expire(self, now):
        return mpic_store_expire(self.ctx.handle, self.handle, now)

    def drop(self, chunk_id):
        mpic_store_drop(self.ctx.handle, self.handle, chunk_id)

    def lookup(self, ids):
        return mpic_store_lookup(self.ctx.handle, self.handle, ids)

    def layer(self, chunk_id, layer):
        return mpic_store_layer(self.ctx.handle, self.handle, chunk_id, layer)

    def close(self):
        if self.handle is not None:
            mpic_store_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
