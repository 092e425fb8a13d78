// Library of stored chunk caches in three tiers (GPU memory, pinned CPU memory, files) and
// the layer pipeline that fetches from it while earlier layers compute.
//
// Sec. 3.1 items 2-3 and the serving workflow: caches of uploaded items are kept for
// serving, copied to disk and deleted when they expire.  Sec. 3.2 / Fig. 6: at the start of
// a request the caches are looked up; those in CPU memory or on disk are transferred while
// the computation runs, those that are missing or fail to load are recomputed.
//
// This file contains no kernel; it uses the HIP runtime for memory, copies, streams, events.
#include <dirent.h>
#include <fcntl.h>
#include <sys/stat.h>
#include <unistd.h>

#include <algorithm>
#include <cerrno>
#include <cinttypes>
#include <cmath>
#include <condition_variable>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <system_error>
#include <thread>
#include <unordered_map>

#include "common.h"

namespace {

constexpr uint64_t kP = 0x9E3779B97F4A7C15ull;
constexpr char kMagic[8] = {'M', 'P', 'I', 'C', 'K', 'V', '0', '1'};
constexpr size_t kHeaderBytes = 64;
constexpr size_t kRingLimit = size_t(4) << 30;  // pinned bytes the disk ring may take

// (n + sum_i w_i * P^(i+1)) mod 2^64 over the 8-byte little-endian words of the buffer.
// Four interleaved accumulators: word i goes to lane i % 4, whose power advances by P^4.
uint64_t checksum(const void* data, size_t bytes) {
  const size_t n = bytes / 8;
  const unsigned char* p = static_cast<const unsigned char*>(data);
  const uint64_t p2 = kP * kP, p4 = p2 * p2;
  uint64_t pw[4] = {kP, p2, p2 * kP, p4};
  uint64_t acc[4] = {0, 0, 0, 0};
  size_t i = 0;
  for (; i + 4 <= n; i += 4) {
    uint64_t w[4];
    std::memcpy(w, p + 8 * i, 32);
    for (int a = 0; a < 4; ++a) {
      acc[a] += w[a] * pw[a];
      pw[a] *= p4;
    }
  }
  for (int a = 0; i < n; ++i, ++a) {
    uint64_t w;
    std::memcpy(&w, p + 8 * i, 8);
    acc[a] += w * pw[a];
  }
  return n + acc[0] + acc[1] + acc[2] + acc[3];
}

struct FileHeader {
  char magic[8];
  uint64_t id;
  int32_t len, n_layers, n_kv_heads, head_dim, dtype, zero;
  uint64_t block_bytes, payload_off, header_sum;
};
static_assert(sizeof(FileHeader) == kHeaderBytes, "file header layout");

struct Entry {
  int32_t len = 0;
  int32_t tier = MPIC_TIER_MISSING;
  int64_t expires_at = -1;
  bool has_file = false;
  void* mem = nullptr;  // HBM: device memory; HOST: pinned memory; layout = file payload
};

bool read_fully(int fd, void* dst, size_t bytes, off_t off) {
  char* p = static_cast<char*>(dst);
  while (bytes > 0) {
    const ssize_t got = pread(fd, p, bytes, off);
    if (got < 0 && errno == EINTR) continue;
    if (got <= 0) return false;
    p += got;
    off += got;
    bytes -= static_cast<size_t>(got);
  }
  return true;
}

bool write_fully(int fd, const void* src, size_t bytes) {
  const char* p = static_cast<const char*>(src);
  while (bytes > 0) {
    const ssize_t put = write(fd, p, bytes);
    if (put < 0 && errno == EINTR) continue;
    if (put <= 0) return false;
    p += put;
    bytes -= static_cast<size_t>(put);
  }
  return true;
}

// One read of the disk tier: both blocks of one layer of one cache into a ring slot.
struct IoJob {
  int fd = -1;
  off_t off = 0;
  size_t block = 0;
  char* dst = nullptr;
  uint64_t want_k = 0, want_v = 0;
  int32_t layer = 0, src = 0;
  bool ok = false;
};

// All reads of one mpic_prefill_layers call, in layer order.
struct IoBatch {
  std::vector<IoJob> jobs;
  size_t next = 0;               // first job no reader has taken yet
  int depth = 1;                 // ring sets: layer l uses set l % depth
  int layers_enqueued = 0;       // layers whose linking out of the ring has been enqueued
  bool cancel = false;
  int active = 0;                // readers inside a job
  std::vector<int> done;         // finished jobs per layer
  hipEvent_t ev_release[2] = {nullptr, nullptr};  // recorded after the kernels that read a ring set
  int device = -1;
};

}  // namespace

struct mpic_store {
  mpic_ctx* ctx = nullptr;
  int32_t n_layers = 0;
  std::string dir;  // empty: no disk tier
  size_t row_bytes = 0;
  std::unordered_map<uint64_t, Entry> map;
  // disk readers
  int n_threads = 4;
  std::vector<std::thread> readers;
  std::mutex mu;
  std::condition_variable cv;
  IoBatch* batch = nullptr;
  bool quit = false;
  // ring of pinned buffers the readers fill
  void* ring = nullptr;
  size_t ring_bytes = 0;
  hipEvent_t ev_release[2] = {nullptr, nullptr};

  size_t block_bytes(int32_t len) const { return static_cast<size_t>(len) * row_bytes; }
  size_t cache_bytes(int32_t len) const { return 2 * block_bytes(len) * static_cast<size_t>(n_layers); }
  size_t table_end() const { return kHeaderBytes + 16 * static_cast<size_t>(n_layers); }
  size_t payload_off() const { return (table_end() + 4095) / 4096 * 4096; }
  std::string path_of(uint64_t id) const {
    char name[40];
    std::snprintf(name, sizeof name, "/%016" PRIx64 ".mpickv", id);
    return dir + name;
  }
};

namespace {

using mpic::fail;

void reader_main(mpic_store* st) {
  std::unique_lock<std::mutex> lock(st->mu);
  for (;;) {
    st->cv.wait(lock, [&] { return st->quit || (st->batch && st->batch->next < st->batch->jobs.size()); });
    if (st->quit) return;
    IoBatch* b = st->batch;
    IoJob& job = b->jobs[b->next++];
    ++b->active;
    // the ring set of this layer is free once the linking of the layer that used it before
    // has been enqueued (host side) and has completed (device side)
    st->cv.wait(lock, [&] { return b->cancel || b->layers_enqueued >= job.layer - b->depth + 1; });
    bool ok = !b->cancel;
    lock.unlock();
    if (ok && job.layer >= b->depth) {
      ok = hipSetDevice(b->device) == hipSuccess &&
           hipEventSynchronize(b->ev_release[job.layer % b->depth]) == hipSuccess;
    }
    if (ok) ok = read_fully(job.fd, job.dst, 2 * job.block, job.off);
    if (ok) ok = checksum(job.dst, job.block) == job.want_k && checksum(job.dst + job.block, job.block) == job.want_v;
    lock.lock();
    job.ok = ok;
    --b->active;
    ++b->done[job.layer];
    st->cv.notify_all();
  }
}

void free_memory(Entry& e) {
  if (e.mem) {
    if (e.tier == MPIC_TIER_HBM) (void)hipFree(e.mem);
    if (e.tier == MPIC_TIER_HOST) (void)hipHostFree(e.mem);
    e.mem = nullptr;
  }
}

void drop(mpic_store* st, uint64_t id) {
  auto it = st->map.find(id);
  if (it == st->map.end()) return;
  if (it->second.mem) (void)hipDeviceSynchronize();
  free_memory(it->second);
  if (it->second.has_file) (void)unlink(st->path_of(id).c_str());
  st->map.erase(it);
}

// Open the file of a cache and check everything but the blocks themselves.
// On success the per-layer sums are returned and the descriptor stays open.
int open_checked(const mpic_store* st, uint64_t id, int32_t len, std::vector<uint64_t>* sums) {
  const int fd = open(st->path_of(id).c_str(), O_RDONLY | O_CLOEXEC);
  if (fd < 0) return -1;
  FileHeader h;
  struct stat sb;
  const mpic_config& c = st->ctx->cfg;
  bool ok = read_fully(fd, &h, sizeof h, 0) && std::memcmp(h.magic, kMagic, 8) == 0 &&
            h.header_sum == checksum(&h, 56) && h.id == id && h.n_layers == st->n_layers &&
            h.n_kv_heads == c.n_kv_heads && h.head_dim == c.head_dim && h.dtype == c.dtype && h.zero == 0 &&
            h.len > 0 && (len < 0 || h.len == len) && h.block_bytes == st->block_bytes(h.len) &&
            h.payload_off == st->payload_off() && fstat(fd, &sb) == 0 &&
            static_cast<uint64_t>(sb.st_size) == h.payload_off + st->cache_bytes(h.len);
  if (ok && sums) {
    sums->resize(2 * static_cast<size_t>(st->n_layers));
    ok = read_fully(fd, sums->data(), 16 * static_cast<size_t>(st->n_layers), kHeaderBytes);
  }
  if (!ok) {
    close(fd);
    return -1;
  }
  if (sums) sums->push_back(static_cast<uint64_t>(h.len));  // last element: token count
  return fd;
}

// Write the file of a cache under a temporary name and rename it into place.
bool write_file(const mpic_store* st, uint64_t id, int32_t len, const char* k, const char* v) {
  const size_t block = st->block_bytes(len);
  const mpic_config& c = st->ctx->cfg;
  std::vector<unsigned char> head(st->payload_off(), 0);
  FileHeader h{};
  std::memcpy(h.magic, kMagic, 8);
  h.id = id;
  h.len = len;
  h.n_layers = st->n_layers;
  h.n_kv_heads = c.n_kv_heads;
  h.head_dim = c.head_dim;
  h.dtype = c.dtype;
  h.block_bytes = block;
  h.payload_off = st->payload_off();
  h.header_sum = checksum(&h, 56);
  std::memcpy(head.data(), &h, sizeof h);
  for (int32_t l = 0; l < st->n_layers; ++l) {
    const uint64_t sums[2] = {checksum(k + l * block, block), checksum(v + l * block, block)};
    std::memcpy(head.data() + kHeaderBytes + 16 * static_cast<size_t>(l), sums, 16);
  }
  const std::string path = st->path_of(id), tmp = path + ".tmp";
  const int fd = open(tmp.c_str(), O_WRONLY | O_CREAT | O_TRUNC | O_CLOEXEC, 0644);
  if (fd < 0) return false;
  bool ok = write_fully(fd, head.data(), head.size());
  for (int32_t l = 0; ok && l < st->n_layers; ++l)
    ok = write_fully(fd, k + l * block, block) && write_fully(fd, v + l * block, block);
  ok = (close(fd) == 0) && ok;
  if (ok) ok = rename(tmp.c_str(), path.c_str()) == 0;
  if (!ok) (void)unlink(tmp.c_str());
  return ok;
}

// Read and verify a whole cache from its file into `dst` (payload layout).
bool read_file(const mpic_store* st, uint64_t id, int32_t len, char* dst) {
  std::vector<uint64_t> sums;
  const int fd = open_checked(st, id, len, &sums);
  if (fd < 0) return false;
  const size_t block = st->block_bytes(len);
  bool ok = read_fully(fd, dst, st->cache_bytes(len), static_cast<off_t>(st->payload_off()));
  close(fd);
  for (int32_t l = 0; ok && l < st->n_layers; ++l)
    ok = checksum(dst + 2 * l * block, block) == sums[2 * l] && checksum(dst + (2 * l + 1) * block, block) == sums[2 * l + 1];
  return ok;
}

// Allocate the memory of a tier and fill it from a host image in payload layout.
int fill_tier(mpic_store* st, Entry& e, int32_t tier, const char* image) {
  mpic_ctx* ctx = st->ctx;
  const size_t bytes = st->cache_bytes(e.len);
  void* mem = nullptr;
  if (tier == MPIC_TIER_HBM) {
    if (hipMalloc(&mem, bytes) != hipSuccess) {
      (void)hipGetLastError();
      return fail(ctx, MPIC_ERR_OOM, "store: device allocation failed");
    }
    const hipError_t err = hipMemcpy(mem, image, bytes, hipMemcpyHostToDevice);
    if (err != hipSuccess) {
      (void)hipFree(mem);
      return mpic::fail_hip(ctx, err, "store: copy to device");
    }
  } else {
    if (hipHostMalloc(&mem, bytes, hipHostMallocDefault) != hipSuccess) {
      (void)hipGetLastError();
      return fail(ctx, MPIC_ERR_OOM, "store: pinned allocation failed");
    }
    std::memcpy(mem, image, bytes);
  }
  e.mem = mem;
  e.tier = tier;
  return MPIC_OK;
}

int store_put(mpic_store* st, uint64_t id, int32_t len, const void* k_, const void* v_, int32_t tier,
              int64_t expires_at) {
  if (!st) return MPIC_ERR_INVALID;
  mpic_ctx* ctx = st->ctx;
  if (!k_ || !v_ || len < 1) return fail(ctx, MPIC_ERR_INVALID, "store_put: need k, v and len >= 1");
  if (tier < MPIC_TIER_HBM || tier > MPIC_TIER_DISK) return fail(ctx, MPIC_ERR_INVALID, "store_put: unknown tier");
  if (tier == MPIC_TIER_DISK && st->dir.empty()) return fail(ctx, MPIC_ERR_INVALID, "store_put: the store has no disk tier");
  const char* k = static_cast<const char*>(k_);
  const char* v = static_cast<const char*>(v_);
  const size_t block = st->block_bytes(len);
  Entry e;
  e.len = len;
  e.expires_at = expires_at;
  if (tier != MPIC_TIER_DISK) {
    const int rc = mpic::bind_device(ctx);
    if (rc != MPIC_OK) return rc;
    // payload layout: K block, V block of layer 0, K block, V block of layer 1, ...
    std::vector<char> image(st->cache_bytes(len));
    for (int32_t l = 0; l < st->n_layers; ++l) {
      std::memcpy(image.data() + 2 * l * block, k + l * block, block);
      std::memcpy(image.data() + (2 * l + 1) * block, v + l * block, block);
    }
    const int rc2 = fill_tier(st, e, tier, image.data());
    if (rc2 != MPIC_OK) return rc2;
  } else {
    e.tier = MPIC_TIER_DISK;
  }
  if (!st->dir.empty()) {
    if (!write_file(st, id, len, k, v)) {
      free_memory(e);
      return fail(ctx, MPIC_ERR_IO, "store_put: could not write " + st->path_of(id));
    }
    e.has_file = true;
  }
  auto old = st->map.find(id);
  if (old != st->map.end()) {
    if (old->second.mem) (void)hipDeviceSynchronize();
    free_memory(old->second);
  }
  st->map[id] = e;
  return MPIC_OK;
}

int store_move(mpic_store* st, uint64_t id, int32_t tier) {
  if (!st) return MPIC_ERR_INVALID;
  mpic_ctx* ctx = st->ctx;
  auto it = st->map.find(id);
  if (it == st->map.end()) return fail(ctx, MPIC_ERR_INVALID, "store_move: unknown id");
  if (tier < MPIC_TIER_HBM || tier > MPIC_TIER_DISK) return fail(ctx, MPIC_ERR_INVALID, "store_move: unknown tier");
  Entry& e = it->second;
  if (e.tier == tier) return MPIC_OK;
  if (tier == MPIC_TIER_DISK) {
    if (!e.has_file) return fail(ctx, MPIC_ERR_INVALID, "store_move: the cache has no file to fall back on");
    (void)hipDeviceSynchronize();
    free_memory(e);
    e.tier = MPIC_TIER_DISK;
    return MPIC_OK;
  }
  const int rc = mpic::bind_device(ctx);
  if (rc != MPIC_OK) return rc;
  const size_t bytes = st->cache_bytes(e.len);
  std::vector<char> image(bytes);
  if (e.tier == MPIC_TIER_DISK) {
    if (!read_file(st, id, e.len, image.data())) {
      drop(st, id);
      return fail(ctx, MPIC_ERR_CACHE_MISS, "store_move: the file of the cache is gone or damaged");
    }
  } else if (e.tier == MPIC_TIER_HBM) {
    MPIC_HIP(ctx, hipMemcpy(image.data(), e.mem, bytes, hipMemcpyDeviceToHost));
  } else {
    (void)hipDeviceSynchronize();
    std::memcpy(image.data(), e.mem, bytes);
  }
  Entry moved = e;
  moved.mem = nullptr;
  const int rc2 = fill_tier(st, moved, tier, image.data());
  if (rc2 != MPIC_OK) return rc2;
  (void)hipDeviceSynchronize();
  free_memory(e);
  e = moved;
  return MPIC_OK;
}

int store_lookup(mpic_store* st, const uint64_t* ids, int32_t n, int32_t* tier, int32_t* len) {
  if (!st) return MPIC_ERR_INVALID;
  if (n < 0 || (n > 0 && (!ids || !tier))) return fail(st->ctx, MPIC_ERR_INVALID, "store_lookup: null argument");
  for (int32_t i = 0; i < n; ++i) {
    auto it = st->map.find(ids[i]);
    if (it != st->map.end() && it->second.tier == MPIC_TIER_DISK) {
      struct stat sb;
      if (stat(st->path_of(ids[i]).c_str(), &sb) != 0 ||
          static_cast<uint64_t>(sb.st_size) != st->payload_off() + st->cache_bytes(it->second.len)) {
        drop(st, ids[i]);
        it = st->map.end();
      }
    }
    tier[i] = it == st->map.end() ? MPIC_TIER_MISSING : it->second.tier;
    if (len) len[i] = it == st->map.end() ? 0 : it->second.len;
  }
  return MPIC_OK;
}

// Register the cache files already present in the directory.
void scan_directory(mpic_store* st) {
  DIR* d = opendir(st->dir.c_str());
  if (!d) return;
  while (dirent* ent = readdir(d)) {
    const char* name = ent->d_name;
    if (std::strlen(name) != 16 + 7 || std::strcmp(name + 16, ".mpickv") != 0) continue;
    char* end = nullptr;
    const uint64_t id = std::strtoull(name, &end, 16);
    if (end != name + 16) continue;
    std::vector<uint64_t> sums;
    const int fd = open_checked(st, id, -1, &sums);
    if (fd < 0) continue;
    close(fd);
    Entry e;
    e.len = static_cast<int32_t>(sums.back());
    e.tier = MPIC_TIER_DISK;
    e.has_file = true;
    st->map[id] = e;
  }
  closedir(d);
}

struct FdGuard {
  std::vector<int> fds;
  ~FdGuard() {
    for (int fd : fds)
      if (fd >= 0) close(fd);
  }
};

// Stop the readers of a batch and wait until none is inside a job.
void end_batch(mpic_store* st, IoBatch* b) {
  std::unique_lock<std::mutex> lock(st->mu);
  b->cancel = true;
  b->next = b->jobs.size();
  st->cv.notify_all();
  st->cv.wait(lock, [&] { return b->active == 0; });
  st->batch = nullptr;
}

int prefill_layers(mpic_ctx* ctx, mpic_plan* plan, mpic_store* st, const uint64_t* ids, int32_t n_srcs,
                   int32_t n_layers, const void* const* fresh_q, const void* const* fresh_k,
                   const void* const* fresh_v, int64_t n_fresh_rows, void* const* k_ctx, void* const* v_ctx,
                   int64_t n_ctx_slots, double softmax_scale, void* const* out, float* const* lse,
                   void* stream_, int32_t* failed) {
  if (!ctx) return MPIC_ERR_INVALID;
  if (!plan || plan->ctx != ctx) return fail(ctx, MPIC_ERR_INVALID, "prefill_layers: plan does not belong to this context");
  if (!st || st->ctx != ctx) return fail(ctx, MPIC_ERR_INVALID, "prefill_layers: store does not belong to this context");
  if (n_layers < 0 || n_layers > st->n_layers) return fail(ctx, MPIC_ERR_INVALID, "prefill_layers: n_layers beyond the store's");
  if (n_fresh_rows != plan->n_q) return fail(ctx, MPIC_ERR_INVALID, "prefill_layers: n_fresh_rows differs from the plan's recompute set");
  if (!(softmax_scale > 0.0) || !std::isfinite(softmax_scale)) return fail(ctx, MPIC_ERR_INVALID, "prefill_layers: softmax_scale must be finite and positive");
  if (n_ctx_slots <= plan->max_slot) return fail(ctx, MPIC_ERR_INVALID, "prefill_layers: context buffers smaller than the plan's largest slot");
  const size_t n_inst = plan->inst_src.size();
  if (n_inst > 0 && (!ids || n_srcs <= plan->max_src)) return fail(ctx, MPIC_ERR_INVALID, "prefill_layers: ids does not cover every chunk index of the plan");
  if (n_layers > 0 && (!fresh_q || !fresh_k || !fresh_v || !k_ctx || !v_ctx || !out)) return fail(ctx, MPIC_ERR_INVALID, "prefill_layers: null pointer array");
  auto aligned16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
  for (int32_t l = 0; l < n_layers; ++l) {
    if (plan->n_ctx > 0 && (!k_ctx[l] || !v_ctx[l] || !aligned16(k_ctx[l]) || !aligned16(v_ctx[l])))
      return fail(ctx, MPIC_ERR_INVALID, "prefill_layers: context buffer of a layer missing or not 16-byte aligned");
    if (plan->n_q > 0 && (!fresh_q[l] || !fresh_k[l] || !fresh_v[l] || !out[l] || !aligned16(fresh_q[l]) ||
                          !aligned16(fresh_k[l]) || !aligned16(fresh_v[l]) || !aligned16(out[l])))
      return fail(ctx, MPIC_ERR_INVALID, "prefill_layers: fresh tensor or output of a layer missing or not 16-byte aligned");
  }
  if (failed) std::fill(failed, failed + std::max(n_srcs, 0), 0);
  if (n_layers == 0 || plan->n_ctx == 0) return MPIC_OK;

  // ---- the lookup: where is every cache the plan reads? ----
  std::vector<char> read_by_plan(std::max(n_srcs, 0), 0);
  for (size_t i = 0; i < n_inst; ++i)
    if (plan->inst_cached[i] > 0) read_by_plan[plan->inst_src[i]] = 1;
  std::vector<const Entry*> entry(std::max(n_srcs, 0), nullptr);
  std::vector<int32_t> disk_srcs;
  std::vector<std::vector<uint64_t>> sums(std::max(n_srcs, 0));
  FdGuard guard;
  guard.fds.assign(std::max(n_srcs, 0), -1);
  bool miss = false;
  for (int32_t s = 0; s < n_srcs; ++s) {
    if (!read_by_plan[s]) continue;
    auto it = st->map.find(ids[s]);
    bool ok = it != st->map.end();
    if (ok) {
      for (size_t i = 0; i < n_inst; ++i)
        if (plan->inst_src[i] == s && plan->inst_len[i] != it->second.len)
          return fail(ctx, MPIC_ERR_INVALID, "prefill_layers: stored cache and segment differ in length");
      if (it->second.tier == MPIC_TIER_DISK) {
        guard.fds[s] = open_checked(st, ids[s], it->second.len, &sums[s]);
        ok = guard.fds[s] >= 0;
        if (!ok) drop(st, ids[s]);
        else disk_srcs.push_back(s);
      }
    }
    if (!ok) {
      miss = true;
      if (failed) failed[s] = 1;
    } else {
      entry[s] = &it->second;
    }
  }
  if (miss) return fail(ctx, MPIC_ERR_CACHE_MISS, "prefill_layers: a stored cache the plan reads is missing or unreadable");

  int rc = mpic::bind_device(ctx);
  if (rc != MPIC_OK) return rc;
  if (!ctx->link_stream) MPIC_HIP(ctx, hipStreamCreateWithFlags(&ctx->link_stream, hipStreamNonBlocking));
  while (ctx->ev_layer.size() < 2 * static_cast<size_t>(n_layers) + 1) {
    hipEvent_t ev;
    MPIC_HIP(ctx, hipEventCreateWithFlags(&ev, hipEventDisableTiming));
    ctx->ev_layer.push_back(ev);
  }
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  // whatever the caller enqueued before this call may still read the context buffers
  MPIC_HIP(ctx, hipEventRecord(ctx->ev_layer[2 * n_layers], stream));
  MPIC_HIP(ctx, hipStreamWaitEvent(ctx->link_stream, ctx->ev_layer[2 * n_layers], 0));

  // ---- disk tier: ring of pinned buffers and the read jobs ----
  IoBatch batch;
  const size_t n_disk = disk_srcs.size();
  std::vector<size_t> slot_off(std::max(n_srcs, 0), 0);
  if (n_disk > 0) {
    size_t set_bytes = 0;
    for (int32_t s : disk_srcs) {
      slot_off[s] = set_bytes;
      set_bytes += (2 * st->block_bytes(entry[s]->len) + 4095) / 4096 * 4096;
    }
    batch.depth = 2 * set_bytes <= kRingLimit ? 2 : 1;
    const size_t need = batch.depth * set_bytes;
    if (need > st->ring_bytes) {
      MPIC_HIP(ctx, hipDeviceSynchronize());
      if (st->ring) MPIC_HIP(ctx, hipHostFree(st->ring));
      st->ring = nullptr;
      st->ring_bytes = 0;
      if (hipHostMalloc(&st->ring, need, hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        return fail(ctx, MPIC_ERR_OOM, "prefill_layers: pinned ring allocation failed");
      }
      st->ring_bytes = need;
    }
    for (hipEvent_t& ev : st->ev_release)
      if (!ev) MPIC_HIP(ctx, hipEventCreateWithFlags(&ev, hipEventDisableTiming));
    batch.ev_release[0] = st->ev_release[0];
    batch.ev_release[1] = st->ev_release[1];
    batch.device = ctx->device;
    batch.done.assign(n_layers, 0);
    batch.jobs.reserve(n_disk * n_layers);
    for (int32_t l = 0; l < n_layers; ++l) {
      for (int32_t s : disk_srcs) {
        IoJob j;
        j.fd = guard.fds[s];
        j.block = st->block_bytes(entry[s]->len);
        j.off = static_cast<off_t>(st->payload_off() + 2 * static_cast<size_t>(l) * j.block);
        j.dst = static_cast<char*>(st->ring) + (l % batch.depth) * set_bytes + slot_off[s];
        j.want_k = sums[s][2 * l];
        j.want_v = sums[s][2 * l + 1];
        j.layer = l;
        j.src = s;
        batch.jobs.push_back(j);
      }
    }
    // the ring may still be read by the linking kernels or the copies of an earlier call
    MPIC_HIP(ctx, hipStreamSynchronize(ctx->link_stream));
    MPIC_HIP(ctx, hipStreamSynchronize(ctx->side_stream));
    if (st->readers.empty())
      for (int t = 0; t < st->n_threads; ++t) st->readers.emplace_back(reader_main, st);
    {
      std::lock_guard<std::mutex> lock(st->mu);
      st->batch = &batch;
    }
    st->cv.notify_all();
  }
  struct BatchEnd {
    mpic_store* st;
    IoBatch* b;
    bool on;
    ~BatchEnd() {
      if (on) end_batch(st, b);
    }
  } batch_end{st, &batch, n_disk > 0};

  // ---- layer loop ----
  // Pinned memory of both slower tiers comes from hipHostMalloc, so the linking kernel can read
  // it in place over the bus (held to a few workgroups on the library's stream, beside the
  // attention of the layer before).  Measured against staged copies, per layer: 18K-token
  // batch of 4, 2.79 ms against 3.88 ms from the host tier and 2.91 against 3.63 from disk;
  // 75K-token paged request, 6.28 against 7.22 and 6.41 against 6.57.  A kernel that reads in
  // place fetches a cache once per *use*, staged copies fetch it once per call: when the batch
  // uses its caches more than once on average (retrieval batches that draw from a common pool:
  // 9.1 ms against 5.9 ms per layer for 8 requests x 16 chunks out of 64), copies win.
  int64_t rows_used = 0, rows_stored = 0;
  {
    std::vector<int32_t> first_row(std::max(n_srcs, 0), INT32_MAX);
    for (size_t i = 0; i < n_inst; ++i) {
      const int32_t s = plan->inst_src[i];
      if (plan->inst_cached[i] > 0 && entry[s] && entry[s]->tier != MPIC_TIER_HBM) {
        rows_used += plan->inst_cached[i];
        first_row[s] = std::min(first_row[s], plan->inst_k[i]);
      }
    }
    for (int32_t s = 0; s < n_srcs; ++s)
      if (first_row[s] != INT32_MAX) rows_stored += entry[s]->len - first_row[s];
  }
  const int host_route = 4 * rows_used > 5 * rows_stored ? MPIC_SRC_HOST_STAGED : MPIC_SRC_HOST_MAPPED;
  hipStream_t ring_reader = host_route == MPIC_SRC_HOST_MAPPED ? ctx->link_stream : ctx->side_stream;
  std::vector<mpic_chunk_src> srcs(std::max(n_srcs, 0));
  auto fill_srcs = [&](int32_t l, std::vector<mpic_chunk_src>& out) {
    for (int32_t s = 0; s < n_srcs; ++s) {
      mpic_chunk_src& c = out[s];
      c = mpic_chunk_src{};
      if (!entry[s]) {
        // not read by the plan: only its length is looked at
        for (size_t i = 0; i < n_inst; ++i)
          if (plan->inst_src[i] == s) c.len = plan->inst_len[i];
        continue;
      }
      const size_t block = st->block_bytes(entry[s]->len);
      c.len = entry[s]->len;
      if (entry[s]->tier == MPIC_TIER_DISK) {
        const char* base = batch.jobs[l * n_disk].dst - slot_off[disk_srcs[0]] + slot_off[s];
        c.k = base;
        c.v = base + block;
        c.on_host = host_route;
      } else {
        const char* base = static_cast<const char*>(entry[s]->mem) + 2 * static_cast<size_t>(l) * block;
        c.k = base;
        c.v = base + block;
        c.on_host = entry[s]->tier == MPIC_TIER_HBM ? MPIC_SRC_DEVICE : host_route;
      }
    }
  };

  // Every cache the plan reads is in GPU memory: nothing to fetch ahead.  When the planner's
  // simulation of the attention launch leaves enough idle time at its end, the stored rows of
  // layer l+1 are linked by the attention launch of layer l itself, in workgroups that run as
  // that attention drains: one stream, no events.  A batch whose tiles fill the chip evenly has
  // no such room, and the two-stream schedule below is the faster one there: 2.17 ms against
  // 2.22 ms per layer for 8 requests x 16 chunks, while a 75K-token request gains from the fused
  // launch, 3.56 ms against 3.60 ms.  A context buffer shared by consecutive layers cannot be
  // written while it is read: those layers are linked by a launch of their own.
  // lazy_rope context with every cache in GPU memory: the caches are linked by reference.  No
  // stored row is copied; each layer is the scatter of its fresh rows and an attention launch
  // that reads the caches where the store keeps them.
  if (ctx->cfg.lazy_rope && rows_stored == 0 && n_inst <= static_cast<size_t>(mpic::kMaxInstPerLaunch)) {
    for (int32_t l = 0; l < n_layers; ++l) {
      fill_srcs(l, srcs);
      rc = mpic::assemble_parts(ctx, plan, nullptr, 0, fresh_k[l], fresh_v[l], n_fresh_rows, k_ctx[l], v_ctx[l],
                                n_ctx_slots, MPIC_PART_FRESH, stream);
      if (rc != MPIC_OK) return rc;
      const mpic::SrcRefs refs{srcs.data(), n_srcs};
      rc = mpic::attend(ctx, plan, fresh_q[l], n_fresh_rows, k_ctx[l], v_ctx[l], n_ctx_slots, softmax_scale, out[l],
                        lse ? lse[l] : nullptr, stream, nullptr, 0, &refs);
      if (rc != MPIC_OK) return rc;
    }
    return MPIC_OK;
  }
  if (rows_stored == 0 && mpic::can_link_in_attention(ctx, plan) && mpic::link_fits_attention_tail(ctx, plan)) {
    std::vector<mpic_chunk_src> next_srcs(std::max(n_srcs, 0));
    const size_t ctx_bytes = static_cast<size_t>(n_ctx_slots) * st->row_bytes;
    auto overlap = [&](const void* x, const void* y) {
      const char* a0 = static_cast<const char*>(x);
      const char* b0 = static_cast<const char*>(y);
      return a0 < b0 + ctx_bytes && b0 < a0 + ctx_bytes;
    };
    bool linked = false;  // stored rows of the current layer are already in place
    for (int32_t l = 0; l < n_layers; ++l) {
      if (!linked) {
        fill_srcs(l, srcs);
        rc = mpic::assemble_parts(ctx, plan, srcs.data(), n_srcs, nullptr, nullptr, 0, k_ctx[l], v_ctx[l], n_ctx_slots,
                                  MPIC_PART_CACHED, stream);
        if (rc != MPIC_OK) return rc;
      }
      rc = mpic::assemble_parts(ctx, plan, nullptr, 0, fresh_k[l], fresh_v[l], n_fresh_rows, k_ctx[l], v_ctx[l],
                                n_ctx_slots, MPIC_PART_FRESH, stream);
      if (rc != MPIC_OK) return rc;
      linked = l + 1 < n_layers && !overlap(k_ctx[l + 1], k_ctx[l]) && !overlap(k_ctx[l + 1], v_ctx[l]) &&
               !overlap(v_ctx[l + 1], k_ctx[l]) && !overlap(v_ctx[l + 1], v_ctx[l]);
      mpic::NextLink next{next_srcs.data(), n_srcs, nullptr, nullptr};
      if (linked) {
        fill_srcs(l + 1, next_srcs);
        next.k_ctx = k_ctx[l + 1];
        next.v_ctx = v_ctx[l + 1];
      }
      rc = mpic::attend(ctx, plan, fresh_q[l], n_fresh_rows, k_ctx[l], v_ctx[l], n_ctx_slots, softmax_scale, out[l],
                        lse ? lse[l] : nullptr, stream, linked ? &next : nullptr, ctx->attn_block_keys ? 0 : 96);
      if (rc != MPIC_OK) return rc;
    }
    return MPIC_OK;
  }
  std::unordered_map<const void*, int32_t> last_reader;  // context buffer -> layer whose attention read it last
  for (int32_t l = 0; l < n_layers; ++l) {
    if (n_disk > 0) {
      std::unique_lock<std::mutex> lock(st->mu);
      st->cv.wait(lock, [&] { return batch.done[l] == static_cast<int>(n_disk); });
      lock.unlock();
      bool bad = false;
      for (size_t j = l * n_disk; j < (l + 1) * n_disk; ++j) {
        if (!batch.jobs[j].ok) {
          bad = true;
          if (failed) failed[batch.jobs[j].src] = 1;
        }
      }
      if (bad) {
        end_batch(st, &batch);
        batch_end.on = false;
        for (size_t j = l * n_disk; j < (l + 1) * n_disk; ++j)
          if (!batch.jobs[j].ok) drop(st, ids[batch.jobs[j].src]);
        return fail(ctx, MPIC_ERR_CACHE_MISS, "prefill_layers: a block of a stored cache failed its check while loading");
      }
    }
    fill_srcs(l, srcs);
    // stored rows: on the library's stream, after whatever last read these buffers
    for (const void* buf : {static_cast<const void*>(k_ctx[l]), static_cast<const void*>(v_ctx[l])}) {
      auto it = last_reader.find(buf);
      if (it != last_reader.end())
        MPIC_HIP(ctx, hipStreamWaitEvent(ctx->link_stream, ctx->ev_layer[2 * it->second + 1], 0));
    }
    rc = mpic::assemble_parts(ctx, plan, srcs.data(), n_srcs, nullptr, nullptr, 0, k_ctx[l], v_ctx[l], n_ctx_slots,
                              MPIC_PART_CACHED | MPIC_PART_BACKGROUND, ctx->link_stream);
    if (rc != MPIC_OK) return rc;
    MPIC_HIP(ctx, hipEventRecord(ctx->ev_layer[2 * l], ctx->link_stream));
    if (n_disk > 0) {
      MPIC_HIP(ctx, hipEventRecord(batch.ev_release[l % batch.depth], ring_reader));
      std::lock_guard<std::mutex> lock(st->mu);
      batch.layers_enqueued = l + 1;
      st->cv.notify_all();
    }
    // fresh rows and attention: on the caller's stream
    rc = mpic::assemble_parts(ctx, plan, nullptr, 0, fresh_k[l], fresh_v[l], n_fresh_rows, k_ctx[l], v_ctx[l],
                              n_ctx_slots, MPIC_PART_FRESH, stream);
    if (rc != MPIC_OK) return rc;
    MPIC_HIP(ctx, hipStreamWaitEvent(stream, ctx->ev_layer[2 * l], 0));
    rc = mpic::attend(ctx, plan, fresh_q[l], n_fresh_rows, k_ctx[l], v_ctx[l], n_ctx_slots, softmax_scale, out[l],
                      lse ? lse[l] : nullptr, stream, nullptr, ctx->attn_block_keys ? 0 : 64);
    if (rc != MPIC_OK) return rc;
    MPIC_HIP(ctx, hipEventRecord(ctx->ev_layer[2 * l + 1], stream));
    last_reader[k_ctx[l]] = l;
    last_reader[v_ctx[l]] = l;
  }
  return MPIC_OK;
}

}  // namespace

#define MPIC_STORE_GUARDED(ctx, call)                     \
  try {                                                   \
    return call;                                          \
  } catch (const std::bad_alloc&) {                       \
    return fail(ctx, MPIC_ERR_OOM, "out of host memory"); \
  } catch (const std::system_error&) {                    \
    return fail(ctx, MPIC_ERR_OOM, "could not start a reader thread"); \
  }

extern "C" int mpic_store_create(mpic_ctx* ctx, int32_t n_layers, const char* disk_dir, int32_t io_threads,
                                 mpic_store** out) {
  if (!ctx) return MPIC_ERR_INVALID;
  if (!out) return fail(ctx, MPIC_ERR_INVALID, "store_create: out is NULL");
  *out = nullptr;
  if (n_layers < 1) return fail(ctx, MPIC_ERR_INVALID, "store_create: n_layers must be >= 1");
  try {
    mpic_store* st = new mpic_store;
    st->ctx = ctx;
    st->n_layers = n_layers;
    st->n_threads = io_threads > 0 ? std::min(io_threads, 64) : 4;
    const mpic_config& c = ctx->cfg;
    st->row_bytes = static_cast<size_t>(c.n_kv_heads) * c.head_dim * (c.dtype == MPIC_F32 ? 4 : 2);
    if (st->row_bytes % 8 != 0) {  // the checksum runs over 8-byte words
      delete st;
      return fail(ctx, MPIC_ERR_UNSUPPORTED, "store_create: a cache row must be a multiple of 8 bytes");
    }
    if (disk_dir) {
      struct stat sb;
      if (stat(disk_dir, &sb) != 0 || !S_ISDIR(sb.st_mode)) {
        delete st;
        return fail(ctx, MPIC_ERR_INVALID, "store_create: disk_dir is not a directory");
      }
      st->dir = disk_dir;
      while (st->dir.size() > 1 && st->dir.back() == '/') st->dir.pop_back();
      scan_directory(st);
    }
    *out = st;
    return MPIC_OK;
  } catch (const std::bad_alloc&) {
    return fail(ctx, MPIC_ERR_OOM, "out of host memory");
  }
}

extern "C" void mpic_store_destroy(mpic_store* st) {
  if (!st) return;
  {
    std::lock_guard<std::mutex> lock(st->mu);
    st->quit = true;
  }
  st->cv.notify_all();
  for (std::thread& t : st->readers) t.join();
  bool gpu = st->ring != nullptr;
  for (auto& kv : st->map) gpu = gpu || kv.second.mem != nullptr;
  if (gpu) {
    int cur = -1;
    (void)hipGetDevice(&cur);
    (void)hipSetDevice(st->ctx->device);
    (void)hipDeviceSynchronize();
    for (auto& kv : st->map) free_memory(kv.second);
    if (st->ring) (void)hipHostFree(st->ring);
    for (hipEvent_t ev : st->ev_release)
      if (ev) (void)hipEventDestroy(ev);
    if (cur >= 0) (void)hipSetDevice(cur);
  }
  delete st;
}

extern "C" int mpic_store_put(mpic_store* st, uint64_t id, int32_t len, const void* k, const void* v,
                              int32_t tier, int64_t expires_at) {
  MPIC_STORE_GUARDED(st ? st->ctx : nullptr, store_put(st, id, len, k, v, tier, expires_at))
}

extern "C" int mpic_store_move(mpic_store* st, uint64_t id, int32_t tier) {
  MPIC_STORE_GUARDED(st ? st->ctx : nullptr, store_move(st, id, tier))
}

extern "C" int mpic_store_expire(mpic_store* st, int64_t now, int32_t* n_removed) {
  if (!st) return MPIC_ERR_INVALID;
  try {
    std::vector<uint64_t> gone;
    for (auto& kv : st->map)
      if (kv.second.expires_at >= 0 && kv.second.expires_at <= now) gone.push_back(kv.first);
    for (uint64_t id : gone) drop(st, id);
    if (n_removed) *n_removed = static_cast<int32_t>(gone.size());
    return MPIC_OK;
  } catch (const std::bad_alloc&) {
    return fail(st->ctx, MPIC_ERR_OOM, "out of host memory");
  }
}

extern "C" int mpic_store_drop(mpic_store* st, uint64_t id) {
  if (!st) return MPIC_ERR_INVALID;
  drop(st, id);
  return MPIC_OK;
}

extern "C" int mpic_store_lookup(mpic_store* st, const uint64_t* ids, int32_t n, int32_t* tier, int32_t* len) {
  MPIC_STORE_GUARDED(st ? st->ctx : nullptr, store_lookup(st, ids, n, tier, len))
}

extern "C" int mpic_store_layer(mpic_store* st, uint64_t id, int32_t layer, mpic_chunk_src* out) {
  if (!st) return MPIC_ERR_INVALID;
  if (!out) return fail(st->ctx, MPIC_ERR_INVALID, "store_layer: out is NULL");
  auto it = st->map.find(id);
  if (it == st->map.end()) return fail(st->ctx, MPIC_ERR_INVALID, "store_layer: unknown id");
  if (layer < 0 || layer >= st->n_layers) return fail(st->ctx, MPIC_ERR_INVALID, "store_layer: layer out of range");
  const Entry& e = it->second;
  if (!e.mem) return fail(st->ctx, MPIC_ERR_INVALID, "store_layer: the cache is in the disk tier; move it first");
  const size_t block = st->block_bytes(e.len);
  const char* base = static_cast<const char*>(e.mem) + 2 * static_cast<size_t>(layer) * block;
  out->k = base;
  out->v = base + block;
  out->len = e.len;
  out->on_host = e.tier == MPIC_TIER_HBM ? MPIC_SRC_DEVICE : MPIC_SRC_HOST_STAGED;
  return MPIC_OK;
}

extern "C" int mpic_prefill_layers(mpic_ctx* ctx, mpic_plan* plan, mpic_store* store, const uint64_t* ids,
                                   int32_t n_srcs, int32_t n_layers, const void* const* fresh_q,
                                   const void* const* fresh_k, const void* const* fresh_v, int64_t n_fresh_rows,
                                   void* const* k_ctx, void* const* v_ctx, int64_t n_ctx_slots,
                                   double softmax_scale, void* const* out, float* const* lse, void* stream,
                                   int32_t* failed) {
  MPIC_STORE_GUARDED(ctx, prefill_layers(ctx, plan, store, ids, n_srcs, n_layers, fresh_q, fresh_k, fresh_v,
                                         n_fresh_rows, k_ctx, v_ctx, n_ctx_slots, softmax_scale, out, lse, stream,
                                         failed))
}
