// Linking of one work item, shared by the linking kernel and by the attention kernel's
// trailing workgroups (which link the stored rows of the next layer while the attention of
// this one drains).
//
// Fig. 7 step 2 / Sec. 4.1: rows of the recompute set are replaced by the fresh K/V, every
// other context row is taken from the stored cache of its image chunk; stored keys are moved
// from chunk-local to global positions by a rotary shift of the chunk's offset, values are
// copied.  A work item is a pair of 16-byte units of one context row (a low/high pair of a key
// head and two value units): all four loads are issued before the first store and consecutive
// lanes touch consecutive 16-byte units of a row.
#pragma once

#include "common.h"

namespace mpic {
namespace link {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <typename T>
struct Unit;  // 16 bytes of storage type T and its fp32 image

template <>
struct Unit<float> {
  static constexpr int kElems = 4;
  using Raw = f32x4;
  using Wide = f32x4;
  __device__ static Wide widen(Raw r) { return r; }
  __device__ static Raw narrow(Wide w) { return w; }
};

template <>
struct Unit<__bf16> {
  static constexpr int kElems = 8;
  using Raw = bf16x8;
  using Wide = f32x8;
  __device__ static Wide widen(Raw r) { return __builtin_convertvector(r, Wide); }
  __device__ static Raw narrow(Wide w) { return __builtin_convertvector(w, Raw); }  // round to nearest even
};

// Geometry of a launch: how a flat item index maps to (context row, unit pair).
struct Shape {
  int D, half, units_per_half, pairs_per_row;
  int64_t row_elems;
};
template <typename T>
__device__ inline Shape shape_of(const AssembleArgs& a) {
  Shape s;
  s.D = a.head_dim;
  s.half = s.D / 2;
  s.units_per_half = s.half / Unit<T>::kElems;
  s.pairs_per_row = a.n_kv_heads * s.units_per_half;
  s.row_elems = static_cast<int64_t>(a.n_kv_heads) * s.D;
  return s;
}

// A work item after its loads have been issued: the four units on their way, where they go and
// how the key units are turned.
template <typename T>
struct Loaded {
  typename Unit<T>::Raw k0, k1, w0, w1;
  const float* ct;  // rotary table row of this context row (null: the key is copied)
  const float* st;
  T* kdst;          // null: nothing to do for this item
  T* vdst;
  int e0, e1, c0, v0, v1;
};

// First half of a work item of the launch described by a -- unit pair u (0 <= u < pairs_per_row)
// of entry `item` (pos_begin <= item < pos_end) of its range: find source and destination,
// issue the loads.
template <typename T, bool kInterleaved>
__device__ inline Loaded<T> load_item_at(const AssembleArgs& a, const AssembleSrcTable& tab, const Shape& sh,
                                         int64_t item, int u) {
  using U = Unit<T>;
  using Raw = typename U::Raw;
  constexpr int E = U::kElems;
  const int D = sh.D, half = sh.half, units_per_half = sh.units_per_half, pairs_per_row = sh.pairs_per_row;
  const int64_t row_elems = sh.row_elems;
  Loaded<T> r;
  r.kdst = nullptr;
  const int64_t pos = a.pos_list ? a.pos_list[item] : item;

  const int inst = a.src_inst[pos];
  const int64_t srow = a.src_row[pos];
  const int64_t slot = a.dst_slot[pos];

  const T* ksrc;
  const T* vsrc;
  const float* ct = nullptr;  // rotary table row of this context row (null: the key is copied)
  const float* st = nullptr;
  if (inst < 0) {
    if (a.skip_fresh) return r;
    ksrc = static_cast<const T*>(a.fresh_k) + srow * row_elems;
    vsrc = static_cast<const T*>(a.fresh_v) + srow * row_elems;
    if (a.fresh_rot) {  // fresh keys arrive without positions: turn them by their position id
      const int64_t u = a.fresh_rot[srow];
      ct = a.fresh_cos + u * half;
      st = a.fresh_sin + u * half;
    }
  } else {
    const T* kt = static_cast<const T*>(tab.k[inst - a.inst_base]);
    const T* vt = static_cast<const T*>(tab.v[inst - a.inst_base]);
    if (kt == nullptr) return r;  // source still in flight: a later launch links this row
    ksrc = kt + srow * row_elems;
    vsrc = vt + srow * row_elems;
    if (a.rope_cos) {  // (null: stored keys are copied as stored)
      ct = a.rope_cos + static_cast<int64_t>(inst) * half;
      st = a.rope_sin + static_cast<int64_t>(inst) * half;
    }
  }
  T* kdst = static_cast<T*>(a.k_ctx) + slot * row_elems;
  T* vdst = static_cast<T*>(a.v_ctx) + slot * row_elems;

  // element offsets of this thread's two units inside the row
  int e0, e1;   // key units
  int c0;       // first rotary pair index of unit e0 (pair index inside a head)
  if (kInterleaved) {
    e0 = u * E;
    e1 = (u + pairs_per_row) * E;
    c0 = (e0 % D) / 2;
  } else {
    const int head = u / units_per_half;
    c0 = (u % units_per_half) * E;
    e0 = head * D + c0;
    e1 = e0 + half;
  }
  const int v0 = u * E, v1 = (u + pairs_per_row) * E;

  // sources are read exactly once: streaming (non-temporal) loads keep them out of the way
  // of the context rows, which the attention kernel reads next
  r.k0 = __builtin_nontemporal_load(reinterpret_cast<const Raw*>(ksrc + e0));
  r.k1 = __builtin_nontemporal_load(reinterpret_cast<const Raw*>(ksrc + e1));
  r.w0 = __builtin_nontemporal_load(reinterpret_cast<const Raw*>(vsrc + v0));
  r.w1 = __builtin_nontemporal_load(reinterpret_cast<const Raw*>(vsrc + v1));
  r.ct = ct;
  r.st = st;
  r.kdst = kdst;
  r.vdst = vdst;
  r.e0 = e0;
  r.e1 = e1;
  r.c0 = c0;
  r.v0 = v0;
  r.v1 = v1;
  return r;
}

// Second half: turn the key units, store all four.
template <typename T, bool kInterleaved>
__device__ inline void finish_item(const Loaded<T>& r, const Shape& sh) {
  using U = Unit<T>;
  using Raw = typename U::Raw;
  using Wide = typename U::Wide;
  constexpr int E = U::kElems;
  if (r.kdst == nullptr) return;
  const int D = sh.D;
  const float* ct = r.ct;
  const float* st = r.st;
  const int e0 = r.e0, e1 = r.e1, c0 = r.c0, v0 = r.v0, v1 = r.v1;
  T* kdst = r.kdst;
  T* vdst = r.vdst;
  const Raw k0 = r.k0, k1 = r.k1, w0 = r.w0, w1 = r.w1;
  (void)D;

  Raw o0 = k0, o1 = k1;
  if (ct) {
    const Wide x0 = U::widen(k0), x1 = U::widen(k1);
    Wide y0, y1;
    if (kInterleaved) {
      const int c1 = (e1 % D) / 2;
#pragma unroll
      for (int i = 0; i < E / 2; ++i) {
        const float ca = ct[c0 + i], sa = st[c0 + i];
        const float cb = ct[c1 + i], sb = st[c1 + i];
        y0[2 * i] = x0[2 * i] * ca - x0[2 * i + 1] * sa;
        y0[2 * i + 1] = x0[2 * i] * sa + x0[2 * i + 1] * ca;
        y1[2 * i] = x1[2 * i] * cb - x1[2 * i + 1] * sb;
        y1[2 * i + 1] = x1[2 * i] * sb + x1[2 * i + 1] * cb;
      }
    } else {
#pragma unroll
      for (int i = 0; i < E; ++i) {
        const float c = ct[c0 + i], s = st[c0 + i];
        y0[i] = x0[i] * c - x1[i] * s;
        y1[i] = x0[i] * s + x1[i] * c;
      }
    }
    o0 = U::narrow(y0);
    o1 = U::narrow(y1);
  }
  // streaming stores as well: the rows are next read by another kernel, from HBM or the
  // memory-side cache either way, and bypassing the L2 write path is worth 5 %
  __builtin_nontemporal_store(o0, reinterpret_cast<Raw*>(kdst + e0));
  __builtin_nontemporal_store(o1, reinterpret_cast<Raw*>(kdst + e1));
  __builtin_nontemporal_store(w0, reinterpret_cast<Raw*>(vdst + v0));
  __builtin_nontemporal_store(w1, reinterpret_cast<Raw*>(vdst + v1));
}

// Item w of the launch, 0 <= w < (pos_end - pos_begin) * pairs_per_row, in one go.
template <typename T, bool kInterleaved>
__device__ inline void link_item(const AssembleArgs& a, const AssembleSrcTable& tab, const Shape& sh, int64_t w) {
  finish_item<T, kInterleaved>(
      load_item_at<T, kInterleaved>(a, tab, sh, a.pos_begin + w / sh.pairs_per_row, static_cast<int>(w % sh.pairs_per_row)), sh);
}

}  // namespace link
}  // namespace mpic
