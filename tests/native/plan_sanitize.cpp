// Host-only exercise of the planner and the argument checks of libmpic under
// AddressSanitizer / UBSan (built by tests/test_host_sanitizers.py with g++; the kernel
// launchers are stubbed out, no GPU call is reached).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "common.h"

namespace mpic {
hipError_t launch_assemble(int, const AssembleArgs&, const AssembleSrcTable&, hipStream_t) { return hipSuccess; }
hipError_t launch_attn_bf16(const AttnArgs&, const AssembleArgs*, const AssembleSrcTable*, const LazyRefs*, hipStream_t) { return hipSuccess; }
hipError_t launch_attn_f32(const AttnArgs&, int64_t, const LazyRefs*, hipStream_t) { return hipSuccess; }
hipError_t launch_decode(int, const DecodeArgs&, const LazyRefs*, hipStream_t) { return hipSuccess; }
hipError_t decode_static_scratch(float**, size_t*) { return hipErrorInvalidDevice; }
}  // namespace mpic

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

int main() {
  std::mt19937 rng(12345);
  auto rnd = [&](int lo, int hi) { return lo + static_cast<int>(rng() % static_cast<unsigned>(hi - lo + 1)); };
  const int heads[][2] = {{4, 4}, {8, 2}, {28, 4}, {7, 1}, {64, 8}};
  for (int iter = 0; iter < 400; ++iter) {
    mpic_config cfg{};
    cfg.n_q_heads = heads[iter % 5][0];
    cfg.n_kv_heads = heads[iter % 5][1];
    cfg.head_dim = 128;
    cfg.dtype = MPIC_BF16;
    cfg.rope_theta = 1e4 + iter;
    cfg.page_size = (iter % 3 == 0) ? 16 : 0;
    cfg.fresh_pre_rope = iter % 2;
    cfg.lazy_rope = (iter / 2) % 2;  // lazy plans build their key-block lists too
    mpic_ctx* ctx = nullptr;
    CHECK(mpic_create(&ctx, &cfg) == MPIC_OK);
    const int B = rnd(1, 4);
    std::vector<int32_t> seg_off(1, 0);
    std::vector<mpic_segment> segs;
    std::vector<int64_t> lens;
    for (int b = 0; b < B; ++b) {
      int64_t n = 0;
      const int ns = rnd(0, 7);
      for (int s = 0; s < ns; ++s) {
        mpic_segment g{};
        g.kind = rnd(0, 1);
        g.len = g.kind ? rnd(1, 300) : rnd(0, 90);
        g.chunk = rnd(0, 5);
        g.k = rnd(-1, 320);
        n += g.len;
        segs.push_back(g);
      }
      seg_off.push_back(static_cast<int32_t>(segs.size()));
      lens.push_back(n);
    }
    std::vector<int32_t> table, table_off(1, 0);
    int64_t pool = 0;
    if (cfg.page_size) {
      for (int64_t n : lens) pool += (n + 15) / 16;
      pool += 3;
      std::vector<int32_t> perm(pool);
      for (int64_t i = 0; i < pool; ++i) perm[i] = static_cast<int32_t>(i);
      for (int64_t i = pool - 1; i > 0; --i) std::swap(perm[i], perm[rng() % (i + 1)]);
      int64_t at = 0;
      for (int64_t n : lens) {
        for (int64_t pg = 0; pg < (n + 15) / 16; ++pg) table.push_back(perm[at++]);
        table_off.push_back(static_cast<int32_t>(table.size()));
      }
    }
    // every fourth batch names the recompute tokens of some chunks one by one
    std::vector<int32_t> sel_off(1, 0), sel_idx;
    const bool listed = iter % 4 == 1;
    for (mpic_segment& g : segs) {
      if (listed && g.kind == 1 && rnd(0, 1)) {
        g.k = MPIC_K_LISTED;
        const int cnt = rnd(0, g.len + 3);
        for (int i = 0; i < cnt; ++i) sel_idx.push_back(rnd(0, g.len - 1));
      }
      sel_off.push_back(static_cast<int32_t>(sel_idx.size()));
    }
    mpic_plan* plan = nullptr;
    const int rc = mpic_plan_create_selected(ctx, B, seg_off.data(), segs.data(), rnd(0, 40),
                                             listed ? sel_off.data() : nullptr, listed ? sel_idx.data() : nullptr,
                                             cfg.page_size ? table.data() : nullptr,
                                             cfg.page_size ? table_off.data() : nullptr, pool, &plan);
    CHECK(rc == MPIC_OK);
    // every array is readable end to end and consistent in size
    const int32_t* p = nullptr;
    size_t n = 0, n_ctx = 0, n_q = 0;
    CHECK(mpic_plan_get(plan, MPIC_PLAN_CTX_OFF, &p, &n) == MPIC_OK && n == static_cast<size_t>(B + 1));
    n_ctx = p[B];
    CHECK(mpic_plan_get(plan, MPIC_PLAN_Q_OFF, &p, &n) == MPIC_OK);
    n_q = p[B];
    long long sum = 0;
    for (int what = 0; what <= MPIC_PLAN_ATTN_TILES; ++what) {
      CHECK(mpic_plan_get(plan, what, &p, &n) == MPIC_OK);
      for (size_t i = 0; i < n; ++i) sum += p[i];
      if (what == MPIC_PLAN_SRC_INST || what == MPIC_PLAN_DST_SLOT) CHECK(n == n_ctx);
      if (what == MPIC_PLAN_Q_POS || what == MPIC_PLAN_SLOT_MAP) CHECK(n == n_q);
    }
    const float *c = nullptr, *s = nullptr;
    CHECK(mpic_plan_get_rope(plan, &c, &s, &n) == MPIC_OK);
    for (size_t i = 0; i < n; ++i) sum += static_cast<long long>(c[i] * 4 + s[i] * 4);
    const int32_t* fr = nullptr;
    CHECK(mpic_plan_get_fresh_rope(plan, &fr, &c, &s, &n) == MPIC_OK);
    CHECK(cfg.fresh_pre_rope ? (n_q == 0 || n > 0) : n == 0);
    if (n > 0) {
      for (size_t r = 0; r < n_q; ++r) {
        CHECK(fr[r] >= 0 && static_cast<size_t>(fr[r]) < n);
        sum += static_cast<long long>(c[fr[r] * 64 + 63] * 4 + s[fr[r] * 64] * 4);
      }
    }
    // argument checks that fail before any GPU call
    CHECK(mpic_assemble_kv(ctx, plan, nullptr, 0, nullptr, nullptr, static_cast<int64_t>(n_q) + 1, nullptr, nullptr, 0, nullptr) == MPIC_ERR_INVALID);
    CHECK(mpic_selective_attn(ctx, plan, nullptr, static_cast<int64_t>(n_q) + 1, nullptr, nullptr, 0, 1.0, nullptr, nullptr, nullptr) == MPIC_ERR_INVALID);
    CHECK(mpic_decode_attn(ctx, plan, nullptr, nullptr, nullptr, nullptr, nullptr, 0, 1.0, nullptr, nullptr, nullptr) == MPIC_ERR_INVALID);
    CHECK(mpic_plan_get(plan, 99, &p, &n) == MPIC_ERR_INVALID);
    if (sum == 42) std::puts("");
    mpic_plan_destroy(plan);
    mpic_destroy(ctx);
  }
  // rejected plans leave nothing behind
  mpic_config cfg{4, 4, 128, MPIC_BF16, 1e4, 0, 16};
  mpic_ctx* ctx = nullptr;
  CHECK(mpic_create(&ctx, &cfg) == MPIC_OK);
  const int32_t off[2] = {0, 1};
  const mpic_segment seg{0, 40, 0, -1};
  const int32_t tab[3] = {0, 1, 1}, tab_off[2] = {0, 3};
  mpic_plan* plan = nullptr;
  CHECK(mpic_plan_create(ctx, 1, off, &seg, 0, tab, tab_off, 8, &plan) == MPIC_ERR_INVALID && plan == nullptr);
  mpic_destroy(ctx);
  std::puts("sanitized planner run ok");
  return 0;
}
