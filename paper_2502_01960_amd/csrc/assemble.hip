// KV linking kernel of libmpic (gfx950).
//
// Fig. 7 step 2 / Sec. 4.1: rows of the recompute set are replaced by the fresh
// K/V, every other context row is taken from the stored cache of its image chunk
// (Sec. 3.1 item 5).  Stored keys are moved from chunk-local to global positions by
// a rotary shift of the chunk's offset; values are copied.  One launch covers a
// range of batch-flattened context positions: gather, rotation and scatter are fused
// and every destination row has exactly one source, so there is no ordering hazard.
//
// The kernel is bandwidth bound (3 flops per key element): each thread moves four
// 16-byte units (a low/high pair of a key head and two value units), all loads are
// issued before the first store, and consecutive lanes touch consecutive 16-byte
// units of a row.
#include <algorithm>

#include "common.h"

namespace mpic {
namespace {

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

template <typename T, bool kInterleaved>
__global__ __launch_bounds__(256) void assemble_kernel(AssembleArgs a, AssembleSrcTable tab) {
  using U = Unit<T>;
  using Raw = typename U::Raw;
  using Wide = typename U::Wide;
  constexpr int E = U::kElems;
  const int D = a.head_dim;
  const int half = D / 2;
  const int units_per_half = half / E;                     // 16-byte units in half a head
  const int pairs_per_row = a.n_kv_heads * units_per_half;  // threads per context row
  const int64_t row_elems = static_cast<int64_t>(a.n_kv_heads) * D;

  // one work item (a pair of 16-byte units of one context row) per thread; launches that
  // are held to a small grid (sources read over the bus, see launch_assemble) stride on
  const int64_t n_items = (a.pos_end - a.pos_begin) * pairs_per_row;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
  for (int64_t w = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; w < n_items; w += stride) {
    const int64_t item = a.pos_begin + w / pairs_per_row;
    const int64_t pos = a.pos_list ? a.pos_list[item] : item;
    const int u = static_cast<int>(w % pairs_per_row);

    const int inst = a.src_inst[pos];
    const int64_t srow = a.src_row[pos];
    const int64_t slot = a.dst_slot[pos];

    const T* ksrc;
    const T* vsrc;
    const float* ct = nullptr;  // rotary table row of this context row (null: the key is copied)
    const float* st = nullptr;
    if (inst < 0) {
      if (a.skip_fresh) continue;
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
      if (kt == nullptr) continue;  // source still in flight: a later launch links this row
      ksrc = kt + srow * row_elems;
      vsrc = vt + srow * row_elems;
      ct = a.rope_cos + static_cast<int64_t>(inst) * half;
      st = a.rope_sin + static_cast<int64_t>(inst) * half;
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
    const Raw k0 = __builtin_nontemporal_load(reinterpret_cast<const Raw*>(ksrc + e0));
    const Raw k1 = __builtin_nontemporal_load(reinterpret_cast<const Raw*>(ksrc + e1));
    const Raw w0 = __builtin_nontemporal_load(reinterpret_cast<const Raw*>(vsrc + v0));
    const Raw w1 = __builtin_nontemporal_load(reinterpret_cast<const Raw*>(vsrc + v1));

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
}

}  // namespace

hipError_t launch_assemble(int dtype, const AssembleArgs& a, const AssembleSrcTable& t,
                           hipStream_t stream) {
  const int64_t n_pos = a.pos_end - a.pos_begin;
  if (n_pos <= 0) return hipSuccess;
  const int elems = dtype == MPIC_F32 ? 4 : 8;
  const int64_t pairs_per_row = static_cast<int64_t>(a.n_kv_heads) * (a.head_dim / 2 / elems);
  const int64_t threads = n_pos * pairs_per_row;
  const dim3 block(256);
  // Sources in mapped host memory: the launch lasts as long as the transfer over the bus.  A
  // grid of one item per thread would fill every wave slot of the chip for that long and keep
  // a concurrent kernel (the attention of the previous layer) from being scheduled; a few
  // waves per compute unit are plenty to keep the bus busy, so those launches stride.
  int64_t blocks = (threads + 255) / 256;
  if (a.grid_limit > 0) blocks = std::min<int64_t>(blocks, a.grid_limit);
  const dim3 grid(static_cast<unsigned>(blocks));
  if (dtype == MPIC_F32) {
    if (a.interleaved)
      hipLaunchKernelGGL((assemble_kernel<float, true>), grid, block, 0, stream, a, t);
    else
      hipLaunchKernelGGL((assemble_kernel<float, false>), grid, block, 0, stream, a, t);
  } else {
    if (a.interleaved)
      hipLaunchKernelGGL((assemble_kernel<__bf16, true>), grid, block, 0, stream, a, t);
    else
      hipLaunchKernelGGL((assemble_kernel<__bf16, false>), grid, block, 0, stream, a, t);
  }
  return hipGetLastError();
}

}  // namespace mpic
