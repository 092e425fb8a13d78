// Host-only exercise of the cache library and the layer pipeline (store.cpp) under
// ThreadSanitizer or AddressSanitizer (built by tests/test_host_sanitizers.py with g++).
// The HIP runtime is replaced by the plain-memory stand-ins below and linking by a CPU copy
// of the stored value rows, so the reader threads, the ring of pinned buffers, the checks of
// the files and the fall-back paths run for real while no GPU is touched.
#include <sys/stat.h>
#include <unistd.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <string>
#include <vector>

#include "common.h"

// ---- stand-ins for the HIP runtime: memory is host memory, streams and events are inert ----
extern "C" {
hipError_t hipMalloc(void** p, size_t n) { *p = std::malloc(n ? n : 1); return *p ? hipSuccess : hipErrorOutOfMemory; }
hipError_t hipHostMalloc(void** p, size_t n, unsigned int) { *p = std::malloc(n ? n : 1); return *p ? hipSuccess : hipErrorOutOfMemory; }
hipError_t hipFree(void* p) { std::free(p); return hipSuccess; }
hipError_t hipHostFree(void* p) { std::free(p); return hipSuccess; }
hipError_t hipMemcpy(void* d, const void* s, size_t n, hipMemcpyKind) { std::memcpy(d, s, n); return hipSuccess; }
hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned) { *e = reinterpret_cast<hipEvent_t>(new int(0)); return hipSuccess; }
hipError_t hipEventDestroy(hipEvent_t e) { delete reinterpret_cast<int*>(e); return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipStreamCreateWithFlags(hipStream_t* s, unsigned) { *s = reinterpret_cast<hipStream_t>(new int(0)); return hipSuccess; }
hipError_t hipStreamDestroy(hipStream_t s) { delete reinterpret_cast<int*>(s); return hipSuccess; }
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t, unsigned int) { return hipSuccess; }
hipError_t hipDeviceSynchronize(void) { return hipSuccess; }
hipError_t hipSetDevice(int) { return hipSuccess; }
hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
hipError_t hipGetLastError(void) { return hipSuccess; }
const char* hipGetErrorString(hipError_t) { return "stub"; }
}

namespace mpic {
int bind_device(mpic_ctx* ctx) {
  ctx->device = 0;
  return MPIC_OK;
}
// CPU stand-in for the linking launch: stored value and key rows are copied (keys unrotated)
// to their context rows, fresh rows likewise; contiguous layout only.
int assemble_parts(mpic_ctx* ctx, mpic_plan* plan, const mpic_chunk_src* srcs, int32_t, const void* fresh_k,
                   const void* fresh_v, int64_t, void* k_ctx, void* v_ctx, int64_t, uint32_t parts, void*) {
  const size_t row = static_cast<size_t>(ctx->cfg.n_kv_heads) * ctx->cfg.head_dim * 2;
  for (int64_t g = 0; g < plan->n_ctx; ++g) {
    const int32_t inst = plan->src_inst[g], r = plan->src_row[g];
    const char *ks, *vs;
    if (inst < 0) {
      if (!(parts & MPIC_PART_FRESH)) continue;
      ks = static_cast<const char*>(fresh_k) + r * row;
      vs = static_cast<const char*>(fresh_v) + r * row;
    } else {
      if (!(parts & MPIC_PART_CACHED)) continue;
      const mpic_chunk_src& s = srcs[plan->inst_src[inst]];
      ks = static_cast<const char*>(s.k) + r * row;
      vs = static_cast<const char*>(s.v) + r * row;
    }
    std::memcpy(static_cast<char*>(k_ctx) + plan->dst_slot[g] * row, ks, row);
    std::memcpy(static_cast<char*>(v_ctx) + plan->dst_slot[g] * row, vs, row);
  }
  return MPIC_OK;
}
int attend(mpic_ctx* ctx, mpic_plan* plan, const void*, int64_t, const void*, const void*, int64_t n_ctx_slots, double,
           void*, float*, void* stream, const NextLink* next, int32_t, const SrcRefs*) {
  if (next)
    return assemble_parts(ctx, plan, next->srcs, next->n_srcs, nullptr, nullptr, 0, next->k_ctx, next->v_ctx, n_ctx_slots,
                          MPIC_PART_CACHED, stream);
  return MPIC_OK;
}
}  // namespace mpic

// The two destructors of the GPU-facing translation unit, for objects that never reached a GPU.
extern "C" void mpic_plan_destroy(mpic_plan* plan) { delete plan; }
extern "C" void mpic_destroy(mpic_ctx* ctx) {
  if (!ctx) return;
  if (ctx->link_stream) (void)hipStreamDestroy(ctx->link_stream);
  for (hipEvent_t ev : ctx->ev_layer) (void)hipEventDestroy(ev);
  delete ctx;
}

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

namespace {
constexpr int kLayers = 5, kHkv = 2, kD = 128;
constexpr size_t kRow = kHkv * kD * 2;

// value of byte `at` of row `t`, tensor `kv`, layer `l` of cache `id`
unsigned char byte_of(uint64_t id, int l, int kv, int t, size_t at) {
  return static_cast<unsigned char>((id * 131 + l * 31 + kv * 17 + t * 7 + at * 3) & 0xFF);
}
std::vector<char> make_cache(uint64_t id, int len, int kv) {
  std::vector<char> x(static_cast<size_t>(kLayers) * len * kRow);
  for (int l = 0; l < kLayers; ++l)
    for (int t = 0; t < len; ++t)
      for (size_t at = 0; at < kRow; ++at) x[(static_cast<size_t>(l) * len + t) * kRow + at] = static_cast<char>(byte_of(id, l, kv, t, at));
  return x;
}
}  // namespace

int main(int argc, char** argv) {
  CHECK(argc == 2);
  const std::string dir = argv[1];
  mpic_config cfg{};
  cfg.n_q_heads = 4;
  cfg.n_kv_heads = kHkv;
  cfg.head_dim = kD;
  cfg.dtype = MPIC_BF16;
  cfg.rope_theta = 1e4;
  mpic_ctx* ctx = nullptr;
  CHECK(mpic_create(&ctx, &cfg) == MPIC_OK);
  std::mt19937 rng(99);
  for (int round = 0; round < 6; ++round) {
    mpic_store* st = nullptr;
    CHECK(mpic_store_create(ctx, kLayers, dir.c_str(), 1 + round % 4, &st) == MPIC_OK);
    // caches: ids 10.., lengths differ, tiers rotate
    const int n_src = 5;
    std::vector<uint64_t> ids;
    std::vector<int> lens;
    for (int s = 0; s < n_src; ++s) {
      ids.push_back(10 + s + 100 * round);
      lens.push_back(20 + 13 * s);
      auto k = make_cache(ids[s], lens[s], 0), v = make_cache(ids[s], lens[s], 1);
      const int tier = round == 0 ? MPIC_TIER_DISK : 1 + (s + round) % 3;
      CHECK(mpic_store_put(st, ids[s], lens[s], k.data(), v.data(), tier, s == 4 ? 50 : -1) == MPIC_OK);
    }
    // one request: text, then every chunk with a few leading tokens recomputed
    std::vector<mpic_segment> segs;
    auto text = [&](int len) { mpic_segment g{}; g.kind = 0; g.len = len; segs.push_back(g); };
    auto chunk = [&](int s, int k) { mpic_segment g{}; g.kind = 1; g.len = lens[s]; g.chunk = s; g.k = k; segs.push_back(g); };
    text(3);
    for (int s = 0; s < n_src; ++s) { chunk(s, static_cast<int>(rng() % 6)); text(static_cast<int>(rng() % 4)); }
    chunk(1, 2);  // one cache twice
    auto plan_now = [&](mpic_plan** out) {
      const int32_t seg_off[2] = {0, static_cast<int32_t>(segs.size())};
      return mpic_plan_create(ctx, 1, seg_off, segs.data(), 4, nullptr, nullptr, 0, out);
    };
    mpic_plan* plan = nullptr;
    CHECK(plan_now(&plan) == MPIC_OK);
    const int64_t n_ctx = plan->n_ctx, n_q = plan->n_q;
    std::vector<std::vector<char>> kc(kLayers, std::vector<char>(n_ctx * kRow)), vc = kc;
    std::vector<char> fresh(static_cast<size_t>(n_q > 0 ? n_q : 1) * kRow * 2, 0x5A), out(static_cast<size_t>(n_q > 0 ? n_q : 1) * 4 * kD * 2);
    std::vector<const void*> fq(kLayers, out.data()), fk(kLayers, fresh.data()), fv(kLayers, fresh.data());
    std::vector<void*> kp, vp, op(kLayers, out.data());
    for (int l = 0; l < kLayers; ++l) { kp.push_back(kc[l].data()); vp.push_back(vc[l].data()); }
    std::vector<int32_t> failed(n_src, -1);
    auto run = [&](mpic_plan* p, int64_t rows) {
      return mpic_prefill_layers(ctx, p, st, ids.data(), n_src, kLayers, fq.data(), fk.data(), fv.data(), rows, kp.data(),
                                 vp.data(), n_ctx, 0.1, op.data(), nullptr, nullptr, failed.data());
    };
    auto verify = [&](mpic_plan* p) {
      for (int l = 0; l < kLayers; ++l)
        for (int64_t g = 0; g < p->n_ctx; ++g) {
          const int32_t inst = p->src_inst[g];
          if (inst < 0) continue;
          const int s = p->inst_src[inst], t = p->src_row[g];
          for (size_t at = 0; at < kRow; at += 61) {
            if (static_cast<unsigned char>(vc[l][g * kRow + at]) != byte_of(ids[s], l, 1, t, at)) return false;
            if (static_cast<unsigned char>(kc[l][g * kRow + at]) != byte_of(ids[s], l, 0, t, at)) return false;
          }
        }
      return true;
    };
    CHECK(run(plan, n_q) == MPIC_OK);
    CHECK(verify(plan));
    CHECK(run(plan, n_q) == MPIC_OK);  // the ring and the readers are reused
    CHECK(verify(plan));
    // expiry: the cache disappears, the call names it, the request falls back to recomputing it
    int32_t gone = -1;
    CHECK(mpic_store_expire(st, 50, &gone) == MPIC_OK && gone == 1);
    CHECK(run(plan, n_q) == MPIC_ERR_CACHE_MISS);
    for (int s = 0; s < n_src; ++s) CHECK(failed[s] == (s == 4));
    for (mpic_segment& g : segs)
      if (g.kind == 1 && g.chunk == 4) g.k = g.len;
    mpic_plan* plan2 = nullptr;
    CHECK(plan_now(&plan2) == MPIC_OK);
    fresh.assign(static_cast<size_t>(plan2->n_q) * kRow * 2, 0x5A);
    out.assign(static_cast<size_t>(plan2->n_q) * 4 * kD * 2, 0);
    for (int l = 0; l < kLayers; ++l) { fq[l] = out.data(); fk[l] = fv[l] = fresh.data(); op[l] = out.data(); }
    CHECK(run(plan2, plan2->n_q) == MPIC_OK);
    CHECK(verify(plan2));
    // damage: one byte in layer 3 of a cache that is (moved) on disk
    CHECK(mpic_store_move(st, ids[2], MPIC_TIER_DISK) == MPIC_OK);
    char name[64];
    std::snprintf(name, sizeof name, "/%016llx.mpickv", static_cast<unsigned long long>(ids[2]));
    const std::string path = dir + name;
    FILE* f = std::fopen(path.c_str(), "r+b");
    CHECK(f);
    const long at = 4096 + (2 * 3 + 1) * static_cast<long>(lens[2] * kRow) + 77;
    CHECK(std::fseek(f, at, SEEK_SET) == 0);
    int c = std::fgetc(f);
    CHECK(std::fseek(f, at, SEEK_SET) == 0);
    std::fputc(c ^ 0x20, f);
    std::fclose(f);
    CHECK(run(plan2, plan2->n_q) == MPIC_ERR_CACHE_MISS);
    for (int s = 0; s < n_src; ++s) CHECK(failed[s] == (s == 2));
    int32_t tier = -1;
    CHECK(mpic_store_lookup(st, &ids[2], 1, &tier, nullptr) == MPIC_OK && tier == MPIC_TIER_MISSING);
    struct stat sb;
    CHECK(stat(path.c_str(), &sb) != 0);  // the damaged file is gone
    // a moved cache keeps its bytes: disk -> HBM -> host -> disk
    for (int t : {MPIC_TIER_HBM, MPIC_TIER_HOST, MPIC_TIER_DISK, MPIC_TIER_HOST}) CHECK(mpic_store_move(st, ids[0], t) == MPIC_OK);
    mpic_chunk_src src{};
    CHECK(mpic_store_layer(st, ids[0], 4, &src) == MPIC_OK && src.len == lens[0]);
    CHECK(static_cast<unsigned char>(static_cast<const char*>(src.v)[5 * kRow + 9]) == byte_of(ids[0], 4, 1, 5, 9));
    mpic_plan_destroy(plan);
    mpic_plan_destroy(plan2);
    mpic_store_destroy(st);
  }
  // a new store finds what the earlier ones left on disk
  mpic_store* st = nullptr;
  CHECK(mpic_store_create(ctx, kLayers, dir.c_str(), 2, &st) == MPIC_OK);
  const uint64_t id = 10 + 100 * 5;
  int32_t tier = -1, len = -1;
  CHECK(mpic_store_lookup(st, &id, 1, &tier, &len) == MPIC_OK && tier == MPIC_TIER_DISK && len == 20);
  mpic_store_destroy(st);
  mpic_destroy(ctx);
  std::printf("sanitized store run ok\n");
  return 0;
}
