// C-ABI layer: argument checks, host bookkeeping, workspaces, kernel launches.
// Declarations and their semantics are in include/racer_pool.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <new>
#include <string>
#include <vector>

#include "../../include/racer_pool.h"  // also fixes RACER_NOALLOC_MAX_*
#include "kernels.h"
#include "pool_host.h"
#include "alpha_ctl.h"

namespace {

thread_local std::string g_last_error;

int32_t hip_fail(hipError_t e, const char* what) {
  g_last_error = std::string(what) + ": " + hipGetErrorString(e);
  return RACER_EHIP;
}

#define HIP_TRY(expr)                                   \
  do {                                                  \
    hipError_t _e = (expr);                             \
    if (_e != hipSuccess) return hip_fail(_e, #expr);   \
  } while (0)

bool is_pow2(uint64_t x) { return x && !(x & (x - 1)); }

// Tests of the error paths name the call that is to fail once in the environment (RACER_FAULT_INJECT=split); the
// variable is cleared by the call that honours it.  Nothing on the GPU is made to fail: the call returns before it
// queues its device work.
bool fault_injected(const char* what) {
  const char* v = std::getenv("RACER_FAULT_INJECT");
  if (!v || std::strcmp(v, what) != 0) return false;
  unsetenv("RACER_FAULT_INJECT");
  return true;
}

// Device memory for metadata and workspaces.  With `zero` the memory is cleared by a fill kernel on `stream`,
// the stream whose later kernels use it (a clear on the null stream is not ordered with a non-blocking stream).
template <typename T>
int32_t dev_alloc(T** p, uint64_t count, bool zero, hipStream_t stream) {
  *p = nullptr;
  if (count == 0) count = 1;
  const uint64_t bytes = (count * sizeof(T) + 3) & ~3ull;  // cleared in 32-bit words
  HIP_TRY(hipMalloc(reinterpret_cast<void**>(p), bytes));
  if (zero) HIP_TRY(racer::launch_fill_u32(reinterpret_cast<uint32_t*>(*p), bytes / 4, 0u, stream));
  return RACER_OK;
}

// Pinned staging that is written by the host and copied to the device asynchronously;
// two buffers alternate so a call only ever waits for the copy issued two calls earlier.
struct Staging {
  uint8_t* buf[2] = {nullptr, nullptr};
  hipEvent_t done[2] = {nullptr, nullptr};
  uint64_t cap[2] = {0, 0};
  bool pending[2] = {false, false};
  int next = 0;
  uint64_t allocs = 0;  // pinned (re)allocations so far

  // both buffers at least `bytes` large, so that no later acquire of up to that size allocates
  int32_t reserve(uint64_t bytes) {
    for (int k = 0; k < 2; ++k) {
      if (!done[k]) HIP_TRY(hipEventCreateWithFlags(&done[k], hipEventDisableTiming));
      if (cap[k] >= bytes) continue;
      if (pending[k]) {
        HIP_TRY(hipEventSynchronize(done[k]));
        pending[k] = false;
      }
      if (buf[k]) HIP_TRY(hipHostFree(buf[k]));
      buf[k] = nullptr;
      cap[k] = 0;
      HIP_TRY(hipHostMalloc(reinterpret_cast<void**>(&buf[k]), bytes, hipHostMallocDefault));
      cap[k] = bytes;
      ++allocs;
    }
    return RACER_OK;
  }

  int32_t acquire(uint64_t bytes, uint8_t** out, int* which) {
    const int k = next;
    next ^= 1;
    if (pending[k]) {
      HIP_TRY(hipEventSynchronize(done[k]));
      pending[k] = false;
    }
    if (cap[k] < bytes) {
      if (buf[k]) HIP_TRY(hipHostFree(buf[k]));
      buf[k] = nullptr;
      cap[k] = 0;
      const uint64_t want = std::max<uint64_t>(bytes * 2, 1 << 16);
      HIP_TRY(hipHostMalloc(reinterpret_cast<void**>(&buf[k]), want, hipHostMallocDefault));
      cap[k] = want;
      ++allocs;
    }
    if (!done[k]) HIP_TRY(hipEventCreateWithFlags(&done[k], hipEventDisableTiming));
    *out = buf[k];
    *which = k;
    return RACER_OK;
  }
  int32_t mark(int which, hipStream_t s) {
    HIP_TRY(hipEventRecord(done[which], s));
    pending[which] = true;
    return RACER_OK;
  }
  void release() {
    for (int k = 0; k < 2; ++k) {
      if (pending[k]) (void)hipEventSynchronize(done[k]);
      if (buf[k]) (void)hipHostFree(buf[k]);
      if (done[k]) (void)hipEventDestroy(done[k]);
      buf[k] = nullptr;
      done[k] = nullptr;
      pending[k] = false;
      cap[k] = 0;
    }
  }
};

// ---- work space of emb_lookup_noalloc -----------------------------------------------------------------------
// One array per GPU, part of the library's code object, alive until the process ends.  It holds the miss path's
// lists for up to kNoallocMaxLookups lookups whose rows add up to at most kNoallocStagingBytes.  In host code the
// array's name is only a handle for hipGetSymbolAddress: the address that kernels and fills take is the one
// that call returns for the current device, kept in g_scratch_ptr.
constexpr uint64_t kNoallocMaxLookups = RACER_NOALLOC_MAX_LOOKUPS;
constexpr uint64_t kNoallocStagingBytes = RACER_NOALLOC_MAX_ROW_BYTES_TOTAL;
constexpr uint64_t kNoallocHash = 2 * kNoallocMaxLookups;  // slots of the dedupe table and of the set-chain heads
constexpr uint64_t align256(uint64_t x) { return (x + 255) & ~255ull; }
constexpr uint64_t kOffCtr = 0;                                                   // 8 x u32
constexpr uint64_t kOffMissList = 256;                                            // u32 [lookups]
constexpr uint64_t kOffDefList = kOffMissList + align256(4 * kNoallocMaxLookups);  // u32 [lookups]
constexpr uint64_t kOffLoc = kOffDefList + align256(4 * kNoallocMaxLookups);       // i64 [lookups]
constexpr uint64_t kOffHkeys = kOffLoc + align256(8 * kNoallocMaxLookups);         // u64 [hash]
constexpr uint64_t kOffHvals = kOffHkeys + align256(8 * kNoallocHash);             // u64 [hash]
constexpr uint64_t kOffHeads = kOffHvals + align256(8 * kNoallocHash);             // u64 [hash]
constexpr uint64_t kOffHslot = kOffHeads + align256(8 * kNoallocHash);             // u32 [hash]
constexpr uint64_t kOffUi = kOffHslot + align256(4 * kNoallocHash);                // five u32 / i32 [lookups]
constexpr uint64_t kOffStaging = kOffUi + 5 * align256(4 * kNoallocMaxLookups);
constexpr uint64_t kScratchBytes = kOffStaging + kNoallocStagingBytes;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
uint8_t* g_scratch_ptr[kMaxDevices] = {};

// address of the current device's copy of `scratch` (looked up once per device)
int32_t scratch_address(uint8_t** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return RACER_EINVAL;
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return RACER_EHIP;
    g_scratch_ptr[dev] = static_cast<uint8_t*>(ptr);
  }
  *out = g_scratch_ptr[dev];
  return RACER_OK;
}

}  // namespace

struct racer_pool {
  racer::HostPool host;
  racer_pool_cfg cfg;
  uint8_t* base = nullptr;
  uint64_t bytes = 0, page_size = 0;
  bool device = false;
  uint32_t* d_tags = nullptr;
  uint32_t* d_stamps = nullptr;
  int32_t* d_emb_pages = nullptr;
  unsigned long long* d_counters = nullptr;
  const uint8_t* d_table = nullptr;
  // every table behind the pool (the first is pool_create's); the device copy exists once a second one was added
  std::vector<racer::TableDesc> tables;
  racer::TableDesc* d_tables = nullptr;
  int64_t* gid_buf = nullptr;  // global ids of a multi-table lookup
  uint64_t gid_cap = 0;
  Staging stage;
  uint32_t batch = 0;
  uint64_t ws_allocs = 0;  // device work-space (re)allocations so far (pool_reserve keeps later calls from adding any)
  uint64_t launches = 0;  // emb_lookup calls that reached the device (selects the list-counter parity)
  hipStream_t last_stream = nullptr;
  // miss-path workspace, grown on demand
  uint64_t ws_cap = 0;
  uint32_t* ws_ctr = nullptr;
  racer::MissWs ws{};
  // hstu workspace
  uint64_t hw_slot = 0;  // bytes of each of the six activation matrices of a step
  uint8_t* hw_buf = nullptr;
  uint64_t hl_cap = 0;
  uint8_t* hl_dev = nullptr;
  uint64_t hp_cap = 0;  // fp32 partial outputs of split attention items
  uint8_t* hp_dev = nullptr;
  Staging hstage;
  // further streams of a step that runs as several pipelines (default priority), with the fork and join events
  hipStream_t aux_stream[3] = {nullptr, nullptr, nullptr};
  hipEvent_t ev_fork = nullptr, ev_join[3] = {nullptr, nullptr, nullptr};
  // optional per-kernel-class timing with events on the caller's stream
  struct ProfMark { hipEvent_t a, b; int kind; };
  bool prof_on = false;
  std::vector<ProfMark> prof;
  std::vector<hipEvent_t> prof_spare;

  racer_pool(uint64_t n_pages, const racer_pool_cfg& c, uint32_t spp) : host(n_pages, c.page_tokens, spp, c.w_max), cfg(c) {}

  racer::EmbView view() const {
    racer::EmbView v{};
    v.base = base;
    v.page_size = page_size;
    v.row_bytes = cfg.row_bytes;
    v.spp = host.spp();
    v.w_max = cfg.w_max;
    v.elem = cfg.elem;
    v.sets = static_cast<uint32_t>(host.sets());
    v.layer_pages = static_cast<uint32_t>(host.layer_pages());
    v.full_ways = static_cast<uint32_t>(host.n_emb() / host.layer_pages());
    v.part_sets = static_cast<uint32_t>((host.n_emb() % host.layer_pages()) * host.spp());
    v.tags = d_tags;
    v.stamps = d_stamps;
    v.emb_pages = d_emb_pages;
    v.table = d_table;
    v.rows = tables.empty() ? cfg.rows : tables.back().base + tables.back().rows;
    v.tables = tables.size() > 1 ? d_tables : nullptr;
    v.n_tables = static_cast<uint32_t>(tables.size());
    v.counters = d_counters;
    return v;
  }
};

struct racer_hstu {
  racer_hstu_cfg cfg;
  racer_hstu_weights w;
  void* w1t = nullptr;  // bf16 models: [L][4d][d], the MFMA kernels want output-major weights; half precision copies
  void* w2t = nullptr;  // [L][d][d]
  float* pos_s = nullptr;   // bf16 models: pos and time tables times log2(e), as the attention kernel wants them
  float* time_s = nullptr;
};

namespace {

// Bracket one launch (or a fixed group of launches) with events when timing is enabled.
struct ProfScope {
  racer_pool* p;
  hipStream_t s;
  bool live = false;
  ProfScope(racer_pool* pool, int kind, hipStream_t stream) : p(pool), s(stream) {
    if (!p->prof_on) return;
    hipEvent_t ev[2] = {nullptr, nullptr};
    for (hipEvent_t& e : ev) {
      if (!p->prof_spare.empty()) {
        e = p->prof_spare.back();
        p->prof_spare.pop_back();
      } else if (hipEventCreate(&e) != hipSuccess) {
        return;
      }
    }
    if (hipEventRecord(ev[0], s) != hipSuccess) return;
    p->prof.push_back({ev[0], ev[1], kind});
    live = true;
  }
  ~ProfScope() {
    if (live) (void)hipEventRecord(p->prof.back().b, s);
  }
};

void free_miss_ws(racer_pool* p) {
  racer::MissWs& w = p->ws;
  (void)hipFree(p->ws_ctr);
  (void)hipFree(w.miss_list); (void)hipFree(w.def_list); (void)hipFree(w.loc); (void)hipFree(w.hkeys); (void)hipFree(w.hvals);
  (void)hipFree(w.hslot_u); (void)hipFree(w.heads); (void)hipFree(w.u_i); (void)hipFree(w.u_id); (void)hipFree(w.u_set);
  (void)hipFree(w.u_next); (void)hipFree(w.u_way); (void)hipFree(w.staging);
  p->ws = racer::MissWs{};
  p->ws_ctr = nullptr;
  p->ws_cap = 0;
}

int32_t ensure_miss_ws(racer_pool* p, uint64_t n, hipStream_t stream) {
  if (n <= p->ws_cap) return RACER_OK;
  if (p->ws_cap) {
    HIP_TRY(hipStreamSynchronize(p->last_stream));
    free_miss_ws(p);
  }
  const uint64_t cap = std::max<uint64_t>(n, 1024);
  uint64_t hsize = 2048;
  while (hsize < 2 * cap) hsize <<= 1;
  p->ws_allocs += 1;
  racer::MissWs& w = p->ws;
  int32_t rc;
  if ((rc = dev_alloc(&p->ws_ctr, 8, true, stream))) return rc;
  if ((rc = dev_alloc(&w.miss_list, cap, false, stream))) return rc;
  if ((rc = dev_alloc(&w.def_list, cap, false, stream))) return rc;
  if ((rc = dev_alloc(&w.loc, cap, false, stream))) return rc;
  if ((rc = dev_alloc(&w.hkeys, hsize, true, stream))) return rc;
  if ((rc = dev_alloc(&w.hvals, hsize, true, stream))) return rc;
  if ((rc = dev_alloc(&w.hslot_u, hsize, false, stream))) return rc;
  if ((rc = dev_alloc(&w.heads, hsize, true, stream))) return rc;
  if ((rc = dev_alloc(&w.u_i, cap, false, stream))) return rc;
  if ((rc = dev_alloc(&w.u_id, cap, false, stream))) return rc;
  if ((rc = dev_alloc(&w.u_set, cap, false, stream))) return rc;
  if ((rc = dev_alloc(&w.u_next, cap, false, stream))) return rc;
  if ((rc = dev_alloc(&w.u_way, cap, false, stream))) return rc;
  if ((rc = dev_alloc(&w.staging, cap * p->cfg.row_bytes, false, stream))) return rc;
  w.hmask = static_cast<uint32_t>(hsize - 1);
  w.headmask = static_cast<uint32_t>(hsize - 1);
  p->ws_cap = cap;
  return RACER_OK;
}


// The remaining work spaces grow on demand (a growth waits for the streams that may still use the old buffer);
// pool_reserve sizes them all ahead of time.
int32_t ensure_gid(racer_pool* p, uint64_t n) {  // global ids of a multi-table lookup
  if (n <= p->gid_cap) return RACER_OK;
  HIP_TRY(hipStreamSynchronize(p->last_stream));
  if (p->gid_buf) HIP_TRY(hipFree(p->gid_buf));
  p->gid_buf = nullptr;
  p->gid_cap = 0;
  const uint64_t cap = std::max<uint64_t>(n, 1024);
  HIP_TRY(hipMalloc(reinterpret_cast<void**>(&p->gid_buf), cap * sizeof(int64_t)));
  p->gid_cap = cap;
  p->ws_allocs += 1;
  return RACER_OK;
}

int32_t ensure_partials(racer_pool* p, uint64_t bytes, hipStream_t stream) {  // fp32 partials of split attention items
  if (bytes <= p->hp_cap) return RACER_OK;
  HIP_TRY(hipStreamSynchronize(p->last_stream));
  HIP_TRY(hipStreamSynchronize(stream));
  if (p->hp_dev) HIP_TRY(hipFree(p->hp_dev));
  p->hp_dev = nullptr;
  p->hp_cap = 0;
  HIP_TRY(hipMalloc(reinterpret_cast<void**>(&p->hp_dev), bytes));
  p->hp_cap = bytes;
  p->ws_allocs += 1;
  return RACER_OK;
}

int32_t ensure_lists(racer_pool* p, uint64_t need, uint64_t want) {  // device copy of a step's host-built lists
  if (need <= p->hl_cap) return RACER_OK;
  HIP_TRY(hipStreamSynchronize(p->last_stream));
  if (p->hl_dev) HIP_TRY(hipFree(p->hl_dev));
  p->hl_dev = nullptr;
  p->hl_cap = 0;
  HIP_TRY(hipMalloc(reinterpret_cast<void**>(&p->hl_dev), want));
  p->hl_cap = want;
  p->ws_allocs += 1;
  return RACER_OK;
}

// Activation work space of a step: six matrices (xn, u, q, o and two layer buffers) of `slot` bytes each.
int32_t ensure_hstu_ws(racer_pool* p, uint64_t slot, hipStream_t stream) {
  if (slot <= p->hw_slot) return RACER_OK;
  HIP_TRY(hipStreamSynchronize(stream));
  HIP_TRY(hipStreamSynchronize(p->last_stream));
  if (p->hw_buf) HIP_TRY(hipFree(p->hw_buf));
  p->hw_buf = nullptr;
  p->hw_slot = 0;
  HIP_TRY(hipMalloc(reinterpret_cast<void**>(&p->hw_buf), slot * 6));
  p->hw_slot = slot;
  p->ws_allocs += 1;
  return RACER_OK;
}

// The step's further streams and its fork / join events.
int32_t ensure_step_streams(racer_pool* p, uint32_t n_aux) {
  if (!p->ev_fork) HIP_TRY(hipEventCreateWithFlags(&p->ev_fork, hipEventDisableTiming));
  for (uint32_t k = 0; k < n_aux; ++k) {
    if (p->aux_stream[k]) continue;
    HIP_TRY(hipStreamCreateWithFlags(&p->aux_stream[k], hipStreamNonBlocking));
    HIP_TRY(hipEventCreateWithFlags(&p->ev_join[k], hipEventDisableTiming));
  }
  return RACER_OK;
}

}  // namespace

extern "C" {

const char* racer_last_error(void) { return g_last_error.c_str(); }

int32_t pool_create(void* dev_base, uint64_t bytes, uint64_t page_size, const racer_pool_cfg* cfg, racer_pool_t** out) {
  if (!cfg || !out) return RACER_EINVAL;
  *out = nullptr;
  if (cfg->row_bytes == 0 || cfg->row_bytes % 16 != 0) return RACER_EINVAL;
  if (cfg->elem != RACER_ELEM_F32 && cfg->elem != RACER_ELEM_BF16) return RACER_EINVAL;
  if (cfg->page_tokens == 0 || !is_pow2(cfg->w_max) || cfg->w_max > 32) return RACER_EINVAL;
  if (page_size == 0 || bytes == 0 || bytes % page_size != 0 || page_size % cfg->row_bytes != 0) return RACER_EINVAL;
  const uint64_t n_pages = bytes / page_size;
  if (n_pages % cfg->w_max != 0 || n_pages >= (1ull << 31)) return RACER_EINVAL;
  if (cfg->rows >= 0xFFFFFFFFull) return RACER_EINVAL;
  if (!(cfg->emb_frac0 >= 0.0 && cfg->emb_frac0 <= 1.0)) return RACER_EINVAL;
  const uint64_t spp = page_size / cfg->row_bytes;
  const uint64_t sets = n_pages / cfg->w_max * spp;
  if (spp >= (1ull << 31) || sets >= (1ull << 32)) return RACER_EINVAL;
  if (dev_base && (reinterpret_cast<uintptr_t>(dev_base) & 255)) return RACER_EINVAL;

  racer_pool* p = new (std::nothrow) racer_pool(n_pages, *cfg, static_cast<uint32_t>(spp));
  if (!p) return RACER_ENOMEM;
  p->base = static_cast<uint8_t*>(dev_base);
  p->bytes = bytes;
  p->page_size = page_size;
  p->device = dev_base != nullptr;
  p->host.seed_emb(static_cast<uint64_t>(std::llround(cfg->emb_frac0 * static_cast<double>(n_pages))));
  if (p->device) {
    int32_t rc = RACER_OK;
    const uint64_t n_tags = sets * cfg->w_max;
    if ((rc = dev_alloc(&p->d_tags, n_tags, false, nullptr)) || (rc = dev_alloc(&p->d_stamps, n_tags, true, nullptr)) ||
        (rc = dev_alloc(&p->d_emb_pages, n_pages, true, nullptr)) ||
        (rc = dev_alloc(&p->d_counters, racer::kCtrCount * racer::kCtrShards, true, nullptr))) {
      pool_destroy(p);
      return rc;
    }
    hipError_t e = racer::launch_fill_u32(p->d_tags, n_tags, RACER_TAG_EMPTY, nullptr);
    if (e == hipSuccess && p->host.n_emb())
      e = hipMemcpy(p->d_emb_pages, p->host.emb_pages().data(), p->host.n_emb() * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e == hipSuccess && cfg->host_table) {
      void* dp = nullptr;
      e = hipHostGetDevicePointer(&dp, const_cast<void*>(cfg->host_table), 0);
      p->d_table = static_cast<const uint8_t*>(dp);
      if (e == hipSuccess) p->tables.push_back(racer::TableDesc{0, cfg->rows, p->d_table, cfg->row_bytes, 0});
    }
    if (e != hipSuccess) {
      pool_destroy(p);
      return hip_fail(e, "pool_create device setup");
    }
  }
  *out = p;
  return RACER_OK;
}

int32_t pool_destroy(racer_pool_t* p) {
  if (!p) return RACER_EINVAL;
  if (p->device) {
    (void)hipStreamSynchronize(p->last_stream);
    free_miss_ws(p);
    p->stage.release();
    p->hstage.release();
    for (const racer_pool::ProfMark& m : p->prof) {
      (void)hipEventDestroy(m.a);
      (void)hipEventDestroy(m.b);
    }
    for (hipEvent_t e : p->prof_spare) (void)hipEventDestroy(e);
    for (int k = 0; k < 3; ++k)
      if (p->aux_stream[k]) {
        (void)hipStreamSynchronize(p->aux_stream[k]);
        (void)hipStreamDestroy(p->aux_stream[k]);
        (void)hipEventDestroy(p->ev_join[k]);
      }
    if (p->ev_fork) (void)hipEventDestroy(p->ev_fork);
    (void)hipFree(p->d_tables);
    (void)hipFree(p->gid_buf);
    (void)hipFree(p->d_tags);
    (void)hipFree(p->d_stamps);
    (void)hipFree(p->d_emb_pages);
    (void)hipFree(p->d_counters);
    (void)hipFree(p->hw_buf);
    (void)hipFree(p->hl_dev);
    (void)hipFree(p->hp_dev);
  }
  delete p;
  return RACER_OK;
}

int32_t pool_set_split(racer_pool_t* p, double emb_frac, void* stream_v, double* achieved) {
  if (!p) return RACER_EINVAL;
  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  const uint64_t G = p->host.layer_pages();
  // The host bookkeeping changes first (the device half needs its result); a copy of it is kept until the device
  // half has been queued, and put back if that fails, so that host and device never disagree about the EMB pages.
  std::unique_ptr<racer::HostPool> undo;
  if (p->device) undo.reset(new (std::nothrow) racer::HostPool(p->host));
  if (p->device && !undo) return RACER_ENOMEM;
  const racer::SplitPlan plan = p->host.set_split(emb_frac);
  if (plan.rc < 0) return plan.rc;
  int32_t rc = RACER_OK;
  if (p->device && plan.new_emb != plan.old_emb) {
    rc = [&]() -> int32_t {
      if (fault_injected("split")) return hip_fail(hipErrorUnknown, "pool_set_split (injected fault)");
      if (plan.new_emb > plan.old_emb) {
        // newly mapped logical pages: ship their physical ids; the new ways are already empty
        const uint64_t count = plan.new_emb - plan.old_emb;
        uint8_t* buf;
        int which;
        int32_t r = p->stage.acquire(count * sizeof(int32_t), &buf, &which);
        if (r) return r;
        std::memcpy(buf, p->host.emb_pages().data() + plan.old_emb, count * sizeof(int32_t));
        HIP_TRY(hipMemcpyAsync(p->d_emb_pages + plan.old_emb, buf, count * sizeof(int32_t), hipMemcpyHostToDevice, stream));
        return p->stage.mark(which, stream);
      }
      const uint32_t old_full = static_cast<uint32_t>(plan.old_emb / G);
      const uint32_t old_part = static_cast<uint32_t>((plan.old_emb % G) * p->host.spp());
      HIP_TRY(racer::launch_emb_shrink(p->view(), old_full, old_part, stream));
      return RACER_OK;
    }();
    if (rc) {
      p->host = std::move(*undo);  // nothing has changed: the device still holds the old split's state
      if (achieved) *achieved = static_cast<double>(p->host.n_emb()) / static_cast<double>(p->host.n_pages());
      return rc;
    }
    p->last_stream = stream;
  }
  if (achieved) *achieved = static_cast<double>(p->host.n_emb()) / static_cast<double>(p->host.n_pages());
  return plan.rc;
}

int32_t pool_stats(racer_pool_t* p, racer_pool_stats* out) {
  if (!p || !out) return RACER_EINVAL;
  std::memset(out, 0, sizeof(*out));
  if (p->device) {
    HIP_TRY(hipStreamSynchronize(p->last_stream));
    unsigned long long shards[racer::kCtrShards][racer::kCtrCount];
    HIP_TRY(hipMemcpy(shards, p->d_counters, sizeof(shards), hipMemcpyDeviceToHost));
    unsigned long long c[racer::kCtrCount] = {};
    for (int sh = 0; sh < racer::kCtrShards; ++sh)
      for (int k = 0; k < racer::kCtrCount; ++k) c[k] += shards[sh][k];
    out->lookups = c[racer::kCtrLookups];
    out->hits = c[racer::kCtrHits];
    out->misses = c[racer::kCtrMisses];
    out->unique_misses = c[racer::kCtrUnique];
    out->inserted = c[racer::kCtrInserted];
    out->evicted = c[racer::kCtrEvicted];
    out->bypassed = c[racer::kCtrBypassed];
    out->invalid_ids = c[racer::kCtrInvalid];
    out->shrink_evicted = c[racer::kCtrShrinkEvicted];
    out->shrink_moved = c[racer::kCtrShrinkMoved];
    out->bad_pages = c[racer::kCtrBadPages];
    out->unordered_ts = c[racer::kCtrUnorderedTs];
  }
  out->ws_allocs = p->ws_allocs + p->stage.allocs + p->hstage.allocs;
  out->pages_total = p->host.n_pages();
  out->pages_emb = p->host.n_emb();
  out->pages_kv_free = p->host.free_count();
  out->pages_kv_used = p->host.n_pages() - p->host.n_emb() - p->host.free_count();
  out->seqs_resident = p->host.seqs_resident();
  out->seqs_evicted = p->host.seqs_evicted();
  out->batch = p->batch;
  return RACER_OK;
}

int32_t pool_dump(racer_pool_t* p, int64_t* emb_pages, uint8_t* owner) {
  if (!p) return RACER_EINVAL;
  if (emb_pages)
    for (uint64_t k = 0; k < p->host.n_emb(); ++k) emb_pages[k] = p->host.emb_pages()[k];
  if (owner) std::memcpy(owner, p->host.owner().data(), p->host.n_pages());
  return RACER_OK;
}

int32_t emb_cache_dump(racer_pool_t* p, uint32_t* tags, uint32_t* stamps) {
  if (!p || !p->device) return RACER_EINVAL;
  HIP_TRY(hipStreamSynchronize(p->last_stream));
  const uint64_t bytes = p->host.sets() * p->cfg.w_max * sizeof(uint32_t);
  if (tags) HIP_TRY(hipMemcpy(tags, p->d_tags, bytes, hipMemcpyDeviceToHost));
  if (stamps) HIP_TRY(hipMemcpy(stamps, p->d_stamps, bytes, hipMemcpyDeviceToHost));
  return RACER_OK;
}

uint64_t pool_num_sets(const racer_pool_t* p) { return p ? p->host.sets() : 0; }

int64_t pool_slot_of(const racer_pool_t* p, uint64_t set, uint32_t way) { return p ? p->host.slot_of(set, way) : -1; }

int32_t kv_seq_reserve(racer_pool_t* p, uint64_t key, uint32_t tokens, int32_t* pages_out, uint32_t cap, uint32_t* n_out) {
  return p ? p->host.reserve(key, tokens, pages_out, cap, n_out) : RACER_EINVAL;
}
int32_t kv_seq_lookup(const racer_pool_t* p, uint64_t key, uint32_t* tokens, int32_t* pages_out, uint32_t cap, uint32_t* n_out) {
  return p ? p->host.lookup(key, tokens, pages_out, cap, n_out) : RACER_EINVAL;
}
int32_t kv_seq_pin(racer_pool_t* p, uint64_t key) { return p ? p->host.pin(key) : RACER_EINVAL; }
int32_t kv_seq_unpin(racer_pool_t* p, uint64_t key) { return p ? p->host.unpin(key) : RACER_EINVAL; }
int32_t kv_seq_release(racer_pool_t* p, uint64_t key) { return p ? p->host.release(key) : RACER_EINVAL; }

int32_t emb_lookup(racer_pool_t* p, const int64_t* ids, uint64_t n, uint32_t bag, void* out, uint8_t* hit_flags, void* stream_v) {
  if (!p || !p->device || !p->d_table) return RACER_EINVAL;
  if (bag == 0 || bag > 64 || n % bag != 0 || n >= 0xFFFFFFFFull) return RACER_EINVAL;
  if (n && (!ids || !out)) return RACER_EINVAL;
  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  p->batch += 1;  // one call = one LRU batch, empty or not
  if (n == 0) return RACER_OK;
  int32_t rc = ensure_miss_ws(p, n, stream);
  if (rc) return rc;
  racer::MissWs ws = p->ws;
  ws.ctr = p->ws_ctr + 4 * (p->launches & 1);
  ws.ctr_next = p->ws_ctr + 4 * ((p->launches + 1) & 1);
  p->launches += 1;
  p->last_stream = stream;
  {
    ProfScope t(p, RACER_PROF_EMB_GATHER, stream);
    HIP_TRY(racer::launch_emb_probe(p->view(), ws, ids, static_cast<uint32_t>(n), bag, static_cast<uint8_t*>(out),
                                    hit_flags, p->batch, stream));
  }
  {
    ProfScope t(p, RACER_PROF_EMB_MISS, stream);
    HIP_TRY(racer::launch_emb_miss_path(p->view(), ws, ids, static_cast<uint32_t>(n), bag, static_cast<uint8_t*>(out),
                                        p->batch, stream));
  }
  return RACER_OK;
}

int32_t emb_lookup_noalloc(racer_pool_t* p, const int64_t* ids, uint64_t n, uint32_t bag, void* out, uint8_t* hit_flags,
                           void* stream_v) {
  if (!p || !p->device || !p->d_table) return RACER_EINVAL;
  if (bag == 0 || bag > 64 || n % bag != 0) return RACER_EINVAL;
  if (n && (!ids || !out)) return RACER_EINVAL;
  if (n > kNoallocMaxLookups || n * p->cfg.row_bytes > kNoallocStagingBytes) {
    g_last_error = "emb_lookup_noalloc: batch beyond the fixed work space (RACER_NOALLOC_MAX_LOOKUPS lookups, "
                   "RACER_NOALLOC_MAX_ROW_BYTES_TOTAL bytes of rows)";
    return RACER_ERANGE;
  }
  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  uint8_t* base = nullptr;
  int32_t rc = scratch_address(&base);
  if (rc) return rc;
  p->batch += 1;  // one call = one LRU batch, empty or not
  if (n == 0) return RACER_OK;
  uint64_t hsize = 2048;
  while (hsize < 2 * n) hsize <<= 1;  // <= kNoallocHash
  racer::MissWs ws{};
  ws.ctr = reinterpret_cast<uint32_t*>(base + kOffCtr);
  ws.ctr_next = ws.ctr + 4;
  ws.miss_list = reinterpret_cast<uint32_t*>(base + kOffMissList);
  ws.def_list = reinterpret_cast<uint32_t*>(base + kOffDefList);
  ws.loc = reinterpret_cast<int64_t*>(base + kOffLoc);
  ws.hkeys = reinterpret_cast<unsigned long long*>(base + kOffHkeys);
  ws.hvals = reinterpret_cast<unsigned long long*>(base + kOffHvals);
  ws.heads = reinterpret_cast<unsigned long long*>(base + kOffHeads);
  ws.hslot_u = reinterpret_cast<uint32_t*>(base + kOffHslot);
  ws.hmask = ws.headmask = static_cast<uint32_t>(hsize - 1);
  const uint64_t list = align256(4 * kNoallocMaxLookups);
  ws.u_i = reinterpret_cast<uint32_t*>(base + kOffUi);
  ws.u_id = reinterpret_cast<uint32_t*>(base + kOffUi + list);
  ws.u_set = reinterpret_cast<uint32_t*>(base + kOffUi + 2 * list);
  ws.u_next = reinterpret_cast<int32_t*>(base + kOffUi + 3 * list);
  ws.u_way = reinterpret_cast<int32_t*>(base + kOffUi + 4 * list);
  ws.staging = base + kOffStaging;
  // The array keeps the last call's contents, whichever pool made it: the list counters and the three tables
  // whose entries are told apart by the batch number must start at zero.  Fill kernels, so that the call can
  // be captured into a graph.
  HIP_TRY(racer::launch_fill_u32(ws.ctr, 8, 0u, stream));
  HIP_TRY(racer::launch_fill_u32(reinterpret_cast<uint32_t*>(ws.hkeys), 2 * hsize, 0u, stream));
  HIP_TRY(racer::launch_fill_u32(reinterpret_cast<uint32_t*>(ws.hvals), 2 * hsize, 0u, stream));
  HIP_TRY(racer::launch_fill_u32(reinterpret_cast<uint32_t*>(ws.heads), 2 * hsize, 0u, stream));
  p->last_stream = stream;
  HIP_TRY(racer::launch_emb_probe(p->view(), ws, ids, static_cast<uint32_t>(n), bag, static_cast<uint8_t*>(out), hit_flags,
                                  p->batch, stream));
  HIP_TRY(racer::launch_emb_miss_path(p->view(), ws, ids, static_cast<uint32_t>(n), bag, static_cast<uint8_t*>(out), p->batch,
                                      stream));
  return RACER_OK;
}

int32_t pool_add_table(racer_pool_t* p, const void* host_table, uint64_t rows, uint32_t row_bytes, uint32_t* table_out) {
  if (!p || !p->device || !p->d_table || p->tables.empty() || !host_table) return RACER_EINVAL;
  if (rows == 0 || row_bytes == 0 || row_bytes % 16 != 0 || row_bytes > p->cfg.row_bytes) return RACER_EINVAL;
  if (p->tables.size() >= racer::kMaxTables) return RACER_EINVAL;
  const uint64_t base = p->tables.back().base + p->tables.back().rows;
  if (base + rows >= 0xFFFFFFFFull) return RACER_EINVAL;  // global ids are the 32-bit cache tags
  void* dp = nullptr;
  HIP_TRY(hipHostGetDevicePointer(&dp, const_cast<void*>(host_table), 0));
  // lookups in flight read the old descriptor array: wait for them, then replace it
  HIP_TRY(hipStreamSynchronize(p->last_stream));
  std::vector<racer::TableDesc> next = p->tables;
  next.push_back(racer::TableDesc{base, rows, static_cast<const uint8_t*>(dp), row_bytes, 0});
  racer::TableDesc* d_next = nullptr;
  HIP_TRY(hipMalloc(reinterpret_cast<void**>(&d_next), sizeof(racer::TableDesc) * next.size()));
  hipError_t e = hipMemcpy(d_next, next.data(), sizeof(racer::TableDesc) * next.size(), hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    (void)hipFree(d_next);
    return hip_fail(e, "pool_add_table");
  }
  if (p->d_tables) (void)hipFree(p->d_tables);
  p->d_tables = d_next;
  p->tables.swap(next);
  if (table_out) *table_out = static_cast<uint32_t>(p->tables.size() - 1);
  return RACER_OK;
}

int32_t emb_lookup_tables(racer_pool_t* p, const uint32_t* table_of, const int64_t* ids, uint64_t n, uint32_t bag,
                          void* out, uint8_t* hit_flags, void* stream_v) {
  if (!p || !p->device || !p->d_table) return RACER_EINVAL;
  if (n >= 0xFFFFFFFFull || (n && (!table_of || !ids))) return RACER_EINVAL;
  if (p->tables.size() < 2) return RACER_EINVAL;  // one table: emb_lookup
  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  int32_t rc_g = ensure_gid(p, n);
  if (rc_g) return rc_g;
  HIP_TRY(racer::launch_emb_global_ids(p->view(), table_of, ids, static_cast<uint32_t>(n), p->gid_buf, stream));
  return emb_lookup(p, p->gid_buf, n, bag, out, hit_flags, stream_v);
}

int32_t emb_refill(racer_pool_t* p, const int64_t* ids, uint64_t n, void* stream_v) {
  if (!p || !p->device || !p->d_table) return RACER_EINVAL;
  if (n >= 0xFFFFFFFFull || (n && !ids)) return RACER_EINVAL;
  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  p->batch += 1;  // a batch of its own in LRU time (and a fresh key for the dedupe table)
  if (n == 0) return RACER_OK;
  int32_t rc = ensure_miss_ws(p, n, stream);
  if (rc) return rc;
  racer::MissWs ws = p->ws;
  ws.ctr = p->ws_ctr + 4 * (p->launches & 1);
  ws.ctr_next = p->ws_ctr + 4 * ((p->launches + 1) & 1);
  p->launches += 1;
  p->last_stream = stream;
  ProfScope t(p, RACER_PROF_EMB_MISS, stream);
  HIP_TRY(racer::launch_emb_refill(p->view(), ws, ids, static_cast<uint32_t>(n), p->batch, stream));
  return RACER_OK;
}

// ---- HSTU ---------------------------------------------------------------------------------

int32_t hstu_model_create(const racer_hstu_cfg* cfg, const racer_hstu_weights* w, racer_hstu_t** out) {
  if (!cfg || !w || !out) return RACER_EINVAL;
  *out = nullptr;
  if (cfg->L == 0 || cfg->H == 0 || cfg->d == 0 || cfg->d % cfg->H != 0) return RACER_EINVAL;
  if (cfg->page_tokens == 0 || cfg->n_pos == 0 || cfg->n_time == 0 || cfg->n_time > 64) return RACER_EINVAL;
  if (!(cfg->n_scale > 0.0f) || !(cfg->eps > 0.0f) || cfg->d > 1024) return RACER_EINVAL;
  const uint32_t dh = cfg->d / cfg->H;
  if (cfg->elem == RACER_ELEM_BF16) {
    if (dh != 64 || cfg->d % 64 != 0 || cfg->page_tokens % 8 != 0) return RACER_EINVAL;
  } else if (cfg->elem == RACER_ELEM_F32) {
    if (dh > 64 || cfg->d % 16 != 0) return RACER_EINVAL;
  } else {
    return RACER_EINVAL;
  }
  const void* ptrs[] = {w->ln1_g, w->ln1_b, w->w1, w->b1, w->ln2_g, w->ln2_b, w->w2, w->b2, w->pos, w->time};
  for (const void* q : ptrs)
    if (!q) return RACER_EINVAL;
  racer_hstu* m = new (std::nothrow) racer_hstu();
  if (!m) return RACER_ENOMEM;
  m->cfg = *cfg;
  m->w = *w;
  if (cfg->elem == RACER_ELEM_BF16) {
    const uint64_t d = cfg->d;
    hipError_t e = hipMalloc(&m->w1t, cfg->L * d * 4 * d * 2);
    if (e == hipSuccess) e = hipMalloc(&m->w2t, cfg->L * d * d * 2);
    for (uint32_t l = 0; l < cfg->L && e == hipSuccess; ++l) {
      e = racer::launch_transpose_weights(static_cast<const uint16_t*>(w->w1) + l * d * 4 * d,
                                          static_cast<uint16_t*>(m->w1t) + l * d * 4 * d, cfg->d, 4 * cfg->d, 1, nullptr);
      if (e == hipSuccess)
        e = racer::launch_transpose_weights(static_cast<const uint16_t*>(w->w2) + l * d * d,
                                            static_cast<uint16_t*>(m->w2t) + l * d * d, cfg->d, cfg->d, 1, nullptr);
    }
    const uint64_t n_pos_all = static_cast<uint64_t>(cfg->L) * cfg->H * cfg->n_pos;
    const uint64_t n_time_all = static_cast<uint64_t>(cfg->L) * cfg->H * cfg->n_time;
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&m->pos_s), n_pos_all * sizeof(float));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&m->time_s), n_time_all * sizeof(float));
    if (e == hipSuccess) e = racer::launch_scale_bias(static_cast<const float*>(w->pos), m->pos_s, n_pos_all, nullptr);
    if (e == hipSuccess) e = racer::launch_scale_bias(static_cast<const float*>(w->time), m->time_s, n_time_all, nullptr);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
      hstu_model_destroy(m);
      return hip_fail(e, "hstu_model_create weight preparation");
    }
  }
  *out = m;
  return RACER_OK;
}

int32_t hstu_model_destroy(racer_hstu_t* m) {
  if (!m) return RACER_EINVAL;
  (void)hipFree(m->w1t);
  (void)hipFree(m->w2t);
  (void)hipFree(m->pos_s);
  (void)hipFree(m->time_s);
  delete m;
  return RACER_OK;
}

}  // extern "C"

namespace {

// a step with fewer new tokens than this runs as one pipeline (its kernels do not fill the chip twice over)
#ifndef RACER_SPLIT_MIN_TOKENS
#define RACER_SPLIT_MIN_TOKENS 32768
#endif
constexpr uint64_t kSplitMinTokens = RACER_SPLIT_MIN_TOKENS;
// ... or with fewer (query, key) pairs than this (a few new tokens against long cached prefixes are a large step too)
#ifndef RACER_SPLIT_MIN_PAIRS
#define RACER_SPLIT_MIN_PAIRS (64ull << 20)
#endif
constexpr uint64_t kSplitMinPairs = RACER_SPLIT_MIN_PAIRS;
#ifndef RACER_STEP_RUNS
#define RACER_STEP_RUNS 3
#endif
constexpr uint32_t kMaxRuns = 4;
constexpr uint32_t kStepRuns = RACER_STEP_RUNS;  // pipelines of a large step
static_assert(kStepRuns >= 2 && kStepRuns <= kMaxRuns, "pipelines per step");

// Upper bounds of a step's list bytes and partial-output bytes for up to B requests, N new tokens and sequences of up
// to max_seq tokens (pool_reserve sizes the work spaces with them; prepare_step's own sizes never exceed them).
// Q query tiles (128 new tokens of one request), V visits of 64-key tiles; a query tile is cut into at most
// n_kt / chunk + 1 items, and the chunk is at least V * H / 2048 tiles unless the item's page-table slice caps it.
struct StepBounds { uint64_t list_bytes, partial_bytes; };
StepBounds step_bounds(uint64_t B, uint64_t N, uint64_t max_seq, uint32_t H, uint32_t page_tokens) {
  const uint64_t Q = N / 128 + B;
  const uint64_t V = Q * (max_seq / 64 + 1);
  const uint64_t chunk_cap = std::max<uint64_t>(1, (static_cast<uint64_t>(racer::kAttnMaxItemPages) - 2) * page_tokens / 64 * 4 / 5);
  const uint64_t items = Q + std::max<uint64_t>(2048 / H + 1, V / chunk_cap + 1);
  StepBounds b;
  b.list_bytes = sizeof(racer::ReqDev) * (B + 1) + 4 * (N + 1) + sizeof(racer::AttnItem) * items +
                 (sizeof(racer::AttnGroup) + sizeof(racer::RowTile)) * (Q + 1) +
                 sizeof(racer::AttnWork) * racer::kXcds * items * H + 6 * 256;
  b.partial_bytes = items * H * 128 * 64 * sizeof(float);
  b.partial_bytes += b.partial_bytes / 4;
  return b;
}

struct StepCtx {
  racer::HstuDims hd;
  racer::KvView kv;
  racer::StepLists sl;       // the whole batch
  racer::StepLists run[kMaxRuns];  // with a split: consecutive runs of requests, each with lists of its own
  uint32_t run_row0[kMaxRuns] = {}, run_rows[kMaxRuns] = {};  // a run's new-token rows
  uint32_t n_runs = 1;             // 1: no split
  uint64_t esize;
};

// Validate the requests, build the row->request map and the attention work lists, ship them
// to the device on `stream`.  With `want_split` the batch is also cut into kStepRuns runs of requests with about
// equal attention work, each with its own work list, groups and row tiles (pipelines that touch disjoint rows,
// pages and partial slots), if it has at least as many requests as pipelines.
int32_t prepare_step(racer_pool* p, racer_hstu* m, const racer_hstu_req* reqs, uint32_t B, uint64_t n_page_entries,
                     const int64_t* ts, hipStream_t stream, StepCtx* ctx, bool want_split = false) {
  const racer_hstu_cfg& c = m->cfg;
  if (!p->device || c.page_tokens != p->cfg.page_tokens || c.elem != p->cfg.elem) return RACER_EINVAL;
  const uint64_t esize = c.elem == RACER_ELEM_BF16 ? 2 : 4;
  if (static_cast<uint64_t>(c.page_tokens) * 2 * c.L * c.d * esize != p->page_size) return RACER_EINVAL;
  uint64_t N = 0;
  for (uint32_t r = 0; r < B; ++r) {
    const racer_hstu_req& q = reqs[r];
    const uint64_t S = static_cast<uint64_t>(q.prefix_len) + q.new_len;
    const uint64_t need = (S + c.page_tokens - 1) / c.page_tokens;
    if (q.page_table_off + need > n_page_entries) return RACER_EINVAL;
    if (q.x_off != N) return RACER_EINVAL;  // rows are packed request after request
    if (q.page_table_off >= (1ull << 32) || q.ts_off >= (1ull << 32) || S >= (1ull << 31)) return RACER_EINVAL;
    N += q.new_len;
  }
  if (N >= (1ull << 31) || B >= (1u << 24)) return RACER_EINVAL;

  // Attention work items.  The score matrix of a request is a staircase: late query tiles see
  // many more key tiles than early ones, and one long request would otherwise set the
  // kernel's duration.  Key ranges are therefore cut at multiples of `chunk` tiles (sized so
  // that about two items per resident block slot exist; a short tail joins the chunk before
  // it), which also makes the items of different query tiles with the same chunk index read
  // exactly the same keys.
  const uint32_t q_block = 128;
  struct QTile { uint32_t req, qt, n_kt, n_ch, slot0; };
  std::vector<QTile> qtiles;
  uint64_t visits = 0;
  for (uint32_t r = 0; r < B; ++r) {
    const uint32_t T = reqs[r].new_len;
    for (uint32_t qt = 0; qt * q_block < T; ++qt) {
      const uint64_t last = static_cast<uint64_t>(reqs[r].prefix_len) + std::min<uint64_t>(qt * q_block + q_block - 1, T - 1);
      qtiles.push_back({r, qt, static_cast<uint32_t>(last / 64 + 1), 0, 0});
      visits += last / 64 + 1;
    }
  }
  // run_begin[k] = first request of run k; a cut is placed where the visits so far come closest to k / n_runs of all
  uint32_t n_runs = 1, run_begin[kMaxRuns + 1] = {0, B, B, B, B};
  if (want_split && B >= kStepRuns) {
    n_runs = kStepRuns;
    uint64_t acc = 0;
    size_t qi = 0;
    uint32_t k = 1;
    for (uint32_t r = 0; r < B && k < n_runs; ++r) {
      const uint64_t before = acc;
      while (qi < qtiles.size() && qtiles[qi].req == r) acc += qtiles[qi++].n_kt;
      const uint64_t target = visits * k / n_runs;
      if (acc >= target) {  // the cut goes before or after request r, whichever is closer; runs stay non-empty
        uint32_t cut = (acc - target <= target - before) ? r + 1 : r;
        cut = std::max(cut, run_begin[k - 1] + 1);
        cut = std::min(cut, B - (n_runs - k));
        run_begin[k++] = cut;
      }
    }
    while (k < n_runs) { run_begin[k] = std::max(run_begin[k - 1] + 1, B - (n_runs - k)); ++k; }
    run_begin[n_runs] = B;
  }
  auto run_of = [&](uint32_t req) {
    uint32_t k = 0;
    while (k + 1 < n_runs && req >= run_begin[k + 1]) ++k;
    return k;
  };
  const uint64_t block_slots = 1024;  // about 256 CUs x resident blocks
  uint32_t chunk = static_cast<uint32_t>(std::max<uint64_t>(8, (visits * c.H + 2 * block_slots - 1) / (2 * block_slots)));
  // an item's slice of the page table (a chunk and a quarter at most) must fit the kernel's LDS copy
  const uint32_t chunk_cap = static_cast<uint32_t>((static_cast<uint64_t>(racer::kAttnMaxItemPages) - 2) * c.page_tokens / 64 * 4 / 5);
  chunk = std::min(chunk, std::max<uint32_t>(1, chunk_cap));
  std::vector<racer::AttnGroup> groups;
  uint32_t n_slots = 0;
  for (QTile& t : qtiles) {
    t.n_ch = t.n_kt / chunk;
    if (t.n_ch == 0 || t.n_kt % chunk > chunk / 4) ++t.n_ch;
    if (t.n_ch > 1) {
      t.slot0 = n_slots;
      groups.push_back({t.req, t.qt, n_slots, t.n_ch});
      n_slots += t.n_ch;
    }
  }
  // units: the items of one request with the same chunk index, for one head
  struct Unit { uint32_t item0, n_items, req; uint64_t weight; };
  std::vector<racer::AttnItem> items;
  std::vector<Unit> units;
  for (size_t q0 = 0; q0 < qtiles.size();) {
    size_t q1 = q0;
    uint32_t max_ch = 0;
    while (q1 < qtiles.size() && qtiles[q1].req == qtiles[q0].req) max_ch = std::max(max_ch, qtiles[q1++].n_ch);
    for (uint32_t k = 0; k < max_ch; ++k) {
      Unit u{static_cast<uint32_t>(items.size()), 0, qtiles[q0].req, 0};
      for (size_t q = q0; q < q1; ++q) {
        const QTile& t = qtiles[q];
        if (k >= t.n_ch) continue;
        const uint32_t b = k * chunk, e = k + 1 == t.n_ch ? t.n_kt : b + chunk;
        items.push_back({t.req, t.qt, b, e, t.n_ch > 1 ? t.slot0 + k : racer::kDirect, 0});
        u.weight += e - b;
      }
      u.n_items = static_cast<uint32_t>(items.size()) - u.item0;
      units.push_back(u);
    }
    q0 = q1;
  }
  // heaviest unit first onto the least loaded die; a die's list keeps that order, so its last
  // workgroups are the short ones
  std::vector<uint32_t> order(units.size());
  for (uint32_t i = 0; i < order.size(); ++i) order[i] = i;
  std::stable_sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) { return units[a].weight > units[b].weight; });
  // (with a split: one set of die lists per run of requests, laid out one after the other)
  std::vector<racer::AttnWork> die_list[kMaxRuns][racer::kXcds];
  uint64_t die_load[kMaxRuns][racer::kXcds] = {};
  for (uint32_t ui : order) {
    const uint32_t run = run_of(units[ui].req);
    for (uint32_t h = 0; h < c.H; ++h) {
      uint32_t best = 0;
      for (uint32_t x = 1; x < racer::kXcds; ++x)
        if (die_load[run][x] < die_load[run][best]) best = x;
      die_load[run][best] += units[ui].weight;
      for (uint32_t i = 0; i < units[ui].n_items; ++i) die_list[run][best].push_back({units[ui].item0 + i, h});
    }
  }
  std::vector<racer::AttnWork> work;
  size_t work_begin[kMaxRuns + 1] = {};
  for (uint32_t run = 0; run < n_runs; ++run) {
    size_t die_len = 0;
    for (uint32_t x = 0; x < racer::kXcds; ++x) die_len = std::max(die_len, die_list[run][x].size());
    work_begin[run] = work.size();
    work.resize(work.size() + die_len * racer::kXcds, racer::AttnWork{racer::kNoWork, 0});
    for (uint32_t x = 0; x < racer::kXcds; ++x)
      for (size_t i = 0; i < die_list[run][x].size(); ++i) work[work_begin[run] + i * racer::kXcds + x] = die_list[run][x][i];
  }
  work_begin[n_runs] = work.size();
  const uint64_t partial_bytes = static_cast<uint64_t>(n_slots) * c.H * q_block * 64 * sizeof(float);
  {
    int32_t rc_p = ensure_partials(p, partial_bytes + partial_bytes / 4, stream);
    if (rc_p) return rc_p;
  }

  const uint64_t bytes_reqs = sizeof(racer::ReqDev) * std::max<uint32_t>(B, 1);
  const uint64_t bytes_rows = sizeof(uint32_t) * std::max<uint64_t>(N, 1);
  const uint64_t bytes_items = sizeof(racer::AttnItem) * std::max<size_t>(items.size(), 1);
  const uint64_t bytes_groups = sizeof(racer::AttnGroup) * std::max<size_t>(groups.size(), 1);
  std::vector<racer::RowTile> row_tiles;
  for (uint32_t r = 0; r < B; ++r)
    for (uint32_t t0 = 0; t0 < reqs[r].new_len; t0 += 128)
      row_tiles.push_back({static_cast<uint32_t>(reqs[r].x_off) + t0, std::min<uint32_t>(128, reqs[r].new_len - t0), r, 0});
  const uint64_t bytes_row_tiles = sizeof(racer::RowTile) * std::max<size_t>(row_tiles.size(), 1);
  const uint64_t bytes_work = sizeof(racer::AttnWork) * std::max<size_t>(work.size(), 1);
  const uint64_t off_rows = (bytes_reqs + 255) & ~255ull, off_items = (off_rows + bytes_rows + 255) & ~255ull;
  const uint64_t off_groups = (off_items + bytes_items + 255) & ~255ull;
  const uint64_t off_row_tiles = (off_groups + bytes_groups + 255) & ~255ull;
  const uint64_t off_work = (off_row_tiles + bytes_row_tiles + 255) & ~255ull;
  const uint64_t total = off_work + bytes_work;
  {
    int32_t rc_l = ensure_lists(p, total, total * 2);
    if (rc_l) return rc_l;
  }
  uint8_t* hbuf;
  int which;
  int32_t rc = p->hstage.acquire(total, &hbuf, &which);
  if (rc) return rc;
  racer::ReqDev* hr = reinterpret_cast<racer::ReqDev*>(hbuf);
  uint32_t* hrow = reinterpret_cast<uint32_t*>(hbuf + off_rows);
  for (uint32_t r = 0; r < B; ++r) {
    hr[r] = racer::ReqDev{reqs[r].prefix_len, reqs[r].new_len, static_cast<uint32_t>(reqs[r].page_table_off),
                          static_cast<uint32_t>(reqs[r].ts_off), static_cast<uint32_t>(reqs[r].x_off), (ts && N) ? 1u : 0u /* cleared by the check */};
    for (uint32_t i = 0; i < reqs[r].new_len; ++i) hrow[reqs[r].x_off + i] = r;
  }
  if (!items.empty()) std::memcpy(hbuf + off_items, items.data(), sizeof(racer::AttnItem) * items.size());
  if (!groups.empty()) std::memcpy(hbuf + off_groups, groups.data(), sizeof(racer::AttnGroup) * groups.size());
  if (!row_tiles.empty()) std::memcpy(hbuf + off_row_tiles, row_tiles.data(), sizeof(racer::RowTile) * row_tiles.size());
  if (!work.empty()) std::memcpy(hbuf + off_work, work.data(), sizeof(racer::AttnWork) * work.size());
  HIP_TRY(hipMemcpyAsync(p->hl_dev, hbuf, total, hipMemcpyHostToDevice, stream));
  if ((rc = p->hstage.mark(which, stream))) return rc;
  // which requests' timestamps never decrease (the attention kernels' 32-bit time paths rely on it)
  if (ts && N) {
    uint32_t longest = 0;
    for (uint32_t r = 0; r < B; ++r) longest = std::max(longest, reqs[r].prefix_len + reqs[r].new_len);
    HIP_TRY(racer::launch_check_timestamps(reinterpret_cast<racer::ReqDev*>(p->hl_dev), B, longest, ts, p->d_counters, stream));
  }

  ctx->esize = esize;
  uint32_t pt_shift = 32;
  for (uint32_t b = 0; b < 32; ++b)
    if ((1u << b) == c.page_tokens) pt_shift = b;
  ctx->hd = racer::HstuDims{c.L, c.d, c.H, c.d / c.H, c.elem, c.page_tokens, c.n_pos, c.n_time, 1.0f / c.n_scale, c.eps, pt_shift};
  ctx->kv = racer::KvView{p->base, p->page_size, static_cast<uint32_t>(p->host.n_pages()), p->d_counters};
  ctx->sl.reqs = reinterpret_cast<const racer::ReqDev*>(p->hl_dev);
  ctx->sl.row_req = reinterpret_cast<const uint32_t*>(p->hl_dev + off_rows);
  ctx->sl.items = reinterpret_cast<const racer::AttnItem*>(p->hl_dev + off_items);
  ctx->sl.groups = reinterpret_cast<const racer::AttnGroup*>(p->hl_dev + off_groups);
  ctx->sl.partials = reinterpret_cast<float*>(p->hp_dev);
  ctx->sl.n_items = static_cast<uint32_t>(items.size());
  ctx->sl.work = reinterpret_cast<const racer::AttnWork*>(p->hl_dev + off_work);
  ctx->sl.n_work = static_cast<uint32_t>(work.size());
  ctx->sl.n_groups = static_cast<uint32_t>(groups.size());
  ctx->sl.q_block = q_block;
  ctx->sl.row_tiles = reinterpret_cast<const racer::RowTile*>(p->hl_dev + off_row_tiles);
  ctx->sl.n_row_tiles = static_cast<uint32_t>(row_tiles.size());
  ctx->sl.B = B;
  ctx->sl.N = static_cast<uint32_t>(N);
  ctx->n_runs = n_runs;
  if (n_runs > 1) {
    // groups and row tiles were built request after request: a run's are a contiguous piece of each array
    size_t g = 0, t = 0;
    for (uint32_t run = 0; run < n_runs; ++run) {
      racer::StepLists& h = ctx->run[run];
      h = ctx->sl;
      h.work = ctx->sl.work + work_begin[run];
      h.n_work = static_cast<uint32_t>(work_begin[run + 1] - work_begin[run]);
      const size_t g0 = g, t0 = t;
      while (g < groups.size() && groups[g].req < run_begin[run + 1]) ++g;
      while (t < row_tiles.size() && row_tiles[t].req < run_begin[run + 1]) ++t;
      h.groups = ctx->sl.groups + g0;
      h.n_groups = static_cast<uint32_t>(g - g0);
      h.row_tiles = ctx->sl.row_tiles + t0;
      h.n_row_tiles = static_cast<uint32_t>(t - t0);
      ctx->run_row0[run] = run_begin[run] < B ? static_cast<uint32_t>(reqs[run_begin[run]].x_off) : static_cast<uint32_t>(N);
      const uint64_t row_end = run_begin[run + 1] < B ? reqs[run_begin[run + 1]].x_off : N;
      ctx->run_rows[run] = static_cast<uint32_t>(row_end - ctx->run_row0[run]);
    }
  }
  return RACER_OK;
}

}  // namespace

extern "C" {

int32_t pool_reserve(racer_pool_t* p, const racer_hstu_t* m, const racer_reserve* r, void* stream_v) {
  if (!p || !r || !p->device) return RACER_EINVAL;
  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  int32_t rc;
  if ((rc = p->stage.reserve(p->host.n_pages() * sizeof(int32_t)))) return rc;  // the largest growth a split change can ship
  if (r->max_lookups) {
    if (r->max_lookups >= 0xFFFFFFFFull) return RACER_EINVAL;
    if ((rc = ensure_miss_ws(p, r->max_lookups, stream))) return rc;
    if ((rc = ensure_gid(p, r->max_lookups))) return rc;
  }
  if (m && r->max_requests) {
    const racer_hstu_cfg& c = m->cfg;
    if (r->max_new_tokens >= (1ull << 31) || r->max_seq_tokens == 0) return RACER_EINVAL;
    const uint64_t esize = c.elem == RACER_ELEM_BF16 ? 2 : 4;
    const StepBounds b = step_bounds(r->max_requests, r->max_new_tokens, r->max_seq_tokens, c.H, c.page_tokens);
    if ((rc = ensure_lists(p, b.list_bytes, b.list_bytes))) return rc;
    if ((rc = p->hstage.reserve(b.list_bytes))) return rc;
    if (c.elem == RACER_ELEM_BF16 && (rc = ensure_partials(p, b.partial_bytes, stream))) return rc;
    if ((rc = ensure_hstu_ws(p, (r->max_new_tokens * c.d * esize + 255) & ~255ull, stream))) return rc;
    if ((rc = ensure_step_streams(p, kStepRuns - 1))) return rc;
  }
  return RACER_OK;
}

int32_t hstu_step(racer_pool_t* p, racer_hstu_t* m, const racer_hstu_req* reqs, uint32_t B, const int32_t* page_tables,
                  uint64_t n_page_entries, const void* x_in, const int64_t* ts, void* out, void* stream_v) {
  if (!p || !m || (B && !reqs)) return RACER_EINVAL;
  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  const racer_hstu_cfg& c = m->cfg;
  // A large bf16 batch runs as several pipelines, one per run of requests, all but the first on streams of the
  // pool's own: requests share nothing inside a step, and the workgroups of one pipeline's kernel fill the slots
  // that another's leaves idle towards its end.  Not while kernels are being timed (their durations would overlap).
  const bool fused = c.elem == RACER_ELEM_BF16 && (c.d == 128 || c.d == 256);
  uint64_t n_tokens = 0, n_pairs = 0;
  for (uint32_t r = 0; r < B; ++r) {
    n_tokens += reqs[r].new_len;
    n_pairs += static_cast<uint64_t>(reqs[r].new_len) * (reqs[r].prefix_len + reqs[r].new_len / 2);
  }
  const bool want_split = c.elem == RACER_ELEM_BF16 && !p->prof_on && B >= 2 &&
                          (n_tokens >= kSplitMinTokens || n_pairs >= kSplitMinPairs);
  StepCtx ctx;
  int32_t rc = prepare_step(p, m, reqs, B, n_page_entries, ts, stream, &ctx, want_split);
  if (rc) return rc;
  p->last_stream = stream;
  const uint32_t N = ctx.sl.N;
  if (N == 0) return RACER_OK;
  if (!page_tables || !x_in || !ts || !out) return RACER_EINVAL;
  const uint64_t d = c.d;
  if ((rc = ensure_hstu_ws(p, (static_cast<uint64_t>(N) * d * ctx.esize + 255) & ~255ull, stream))) return rc;
  const uint64_t stride = p->hw_slot;
  uint8_t* xn = p->hw_buf;
  uint8_t* u = xn + stride;
  uint8_t* q = u + stride;
  uint8_t* o = q + stride;
  uint8_t* xb[2] = {o + stride, o + 2 * stride};
  const bool bf16 = c.elem == RACER_ELEM_BF16;
  const uint64_t w1_layer = d * 4 * d * ctx.esize, w2_layer = d * d * ctx.esize;
  const uint32_t n_runs = ctx.n_runs;
  bool split = n_runs > 1;
  for (uint32_t run = 0; split && run < n_runs; ++run)
    if (ctx.run[run].n_row_tiles == 0 || ctx.run[run].n_work == 0) split = false;  // a run without new tokens
  if (split) {  // the other pipelines start behind everything the caller's stream holds so far (lists included)
    if ((rc = ensure_step_streams(p, n_runs - 1))) return rc;
    HIP_TRY(hipEventRecord(p->ev_fork, stream));
    for (uint32_t k = 0; k + 1 < n_runs; ++k) HIP_TRY(hipStreamWaitEvent(p->aux_stream[k], p->ev_fork, 0));
  }
  // one layer of one pipeline: rows, pages and partial slots of `sl` only
  auto layer_of = [&](const racer::StepLists& sl, uint32_t row0, uint32_t rows, hipStream_t st, uint32_t l,
                      const void* x_cur, void* x_next) -> int32_t {
    // the separate LayerNorm and output GEMM work on rows [row0, row0 + rows) of every matrix
    const uint64_t off = static_cast<uint64_t>(row0) * d * ctx.esize;
    auto at = [&](const void* base) { return static_cast<const uint8_t*>(base) + off; };
    auto at_w = [&](void* base) { return static_cast<uint8_t*>(base) + off; };
    const float* ln1_g = static_cast<const float*>(m->w.ln1_g) + l * d;
    const float* ln1_b = static_cast<const float*>(m->w.ln1_b) + l * d;
    const float* ln2_g = static_cast<const float*>(m->w.ln2_g) + l * d;
    const float* ln2_b = static_cast<const float*>(m->w.ln2_b) + l * d;
    const float* b1 = static_cast<const float*>(m->w.b1) + l * 4 * d;
    const float* b2 = static_cast<const float*>(m->w.b2) + l * d;
    const uint8_t* w1 = static_cast<const uint8_t*>(bf16 ? m->w1t : m->w.w1) + l * w1_layer;
    const uint8_t* w2 = static_cast<const uint8_t*>(bf16 ? m->w2t : m->w.w2) + l * w2_layer;
    if (fused) {
      ProfScope t(p, RACER_PROF_GEMM_FRONT, st);
      HIP_TRY(racer::launch_layer_front_fused(ctx.hd, l, x_cur, ln1_g, ln1_b, w1, b1, u, q, ctx.kv, sl, page_tables, st));
    } else {
      {
        ProfScope t(p, RACER_PROF_LAYERNORM, st);
        HIP_TRY(racer::launch_layernorm(ctx.hd, at(x_cur), ln1_g, ln1_b, nullptr, at_w(xn), rows, st));
      }
      ProfScope t(p, RACER_PROF_GEMM_FRONT, st);
      HIP_TRY(racer::launch_gemm_front(ctx.hd, l, xn, w1, b1, u, q, ctx.kv, sl, page_tables, st));
    }
    {
      ProfScope t(p, RACER_PROF_ATTENTION, st);
      HIP_TRY(racer::launch_attention(ctx.hd, l, q, bf16 ? m->pos_s : static_cast<const float*>(m->w.pos),
                                      bf16 ? m->time_s : static_cast<const float*>(m->w.time), ctx.kv, sl,
                                      page_tables, ts, o, /*o_half=*/bf16, st));
    }
    if (sl.n_groups) {
      ProfScope t(p, RACER_PROF_ATTN_REDUCE, st);
      HIP_TRY(racer::launch_attention_reduce(ctx.hd, sl, o, /*o_half=*/bf16, st));
    }
    if (fused) {
      ProfScope t(p, RACER_PROF_GEMM_BACK, st);
      HIP_TRY(racer::launch_layer_back_fused(ctx.hd, o, u, ln2_g, ln2_b, w2, b2, x_cur, x_next, sl, st));
    } else {
      {
        ProfScope t(p, RACER_PROF_LAYERNORM, st);
        HIP_TRY(racer::launch_layernorm(ctx.hd, at(o), ln2_g, ln2_b, at(u), at_w(xn), rows, st));
      }
      ProfScope t(p, RACER_PROF_GEMM_BACK, st);
      HIP_TRY(racer::launch_gemm_back(ctx.hd, at(xn), w2, b2, at(x_cur), at_w(x_next), rows, st));
    }
    return RACER_OK;
  };
  const void* x_cur = x_in;
  for (uint32_t l = 0; l < c.L; ++l) {
    void* x_next = (l + 1 == c.L) ? out : static_cast<void*>(xb[l & 1]);
    if (split) {
      for (uint32_t run = 0; run < n_runs; ++run)
        if ((rc = layer_of(ctx.run[run], ctx.run_row0[run], ctx.run_rows[run], run ? p->aux_stream[run - 1] : stream, l,
                           x_cur, x_next)))
          return rc;
    } else {
      if ((rc = layer_of(ctx.sl, 0, N, stream, l, x_cur, x_next))) return rc;
    }
    x_cur = x_next;
  }
  if (split) {  // the caller's stream goes on when every pipeline is through
    for (uint32_t k = 0; k + 1 < n_runs; ++k) {
      HIP_TRY(hipEventRecord(p->ev_join[k], p->aux_stream[k]));
      HIP_TRY(hipStreamWaitEvent(stream, p->ev_join[k], 0));
    }
  }
  return RACER_OK;
}

int32_t hstu_attn_paged(racer_pool_t* p, racer_hstu_t* m, uint32_t layer, const racer_hstu_req* reqs, uint32_t B,
                        const int32_t* page_tables, uint64_t n_page_entries, const void* q, const int64_t* ts, void* o,
                        void* stream_v) {
  if (!p || !m || (B && !reqs) || layer >= m->cfg.L) return RACER_EINVAL;
  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  StepCtx ctx;
  int32_t rc = prepare_step(p, m, reqs, B, n_page_entries, ts, stream, &ctx);
  if (rc) return rc;
  p->last_stream = stream;
  if (ctx.sl.N == 0) return RACER_OK;
  if (!page_tables || !q || !ts || !o) return RACER_EINVAL;
  if (m->cfg.elem == RACER_ELEM_BF16) {
    // the MFMA kernel takes q * log2(e); hstu_step's projection writes it that way, here it is a pre-pass
    if ((rc = ensure_hstu_ws(p, (static_cast<uint64_t>(ctx.sl.N) * m->cfg.d * ctx.esize + 255) & ~255ull, stream))) return rc;
    const uint64_t stride = p->hw_slot;
    void* qs = p->hw_buf + 2 * stride;
    HIP_TRY(racer::launch_scale_q(q, qs, static_cast<uint64_t>(ctx.sl.N) * m->cfg.d, stream));
    q = qs;
  }
  {
    ProfScope t(p, RACER_PROF_ATTENTION, stream);
    const bool bf16 = m->cfg.elem == RACER_ELEM_BF16;
    HIP_TRY(racer::launch_attention(ctx.hd, layer, q, bf16 ? m->pos_s : static_cast<const float*>(m->w.pos),
                                    bf16 ? m->time_s : static_cast<const float*>(m->w.time), ctx.kv, ctx.sl,
                                    page_tables, ts, o, /*o_half=*/false, stream));
  }
  if (ctx.sl.n_groups) {
    ProfScope t(p, RACER_PROF_ATTN_REDUCE, stream);
    HIP_TRY(racer::launch_attention_reduce(ctx.hd, ctx.sl, o, /*o_half=*/false, stream));
  }
  return RACER_OK;
}

// ---- split controller (host only) --------------------------------------------------------------------------

int32_t alpha_ctl_create(double slo_ms, racer_alpha_ctl_t** out) {
  if (!out) return RACER_EINVAL;
  *out = nullptr;
  if (!(slo_ms > 0.0)) return RACER_EINVAL;
  racer::AlphaController* c = new (std::nothrow) racer::AlphaController(slo_ms);
  if (!c) return RACER_ENOMEM;
  *out = reinterpret_cast<racer_alpha_ctl_t*>(c);
  return RACER_OK;
}

int32_t alpha_ctl_destroy(racer_alpha_ctl_t* ctl) {
  if (!ctl) return RACER_EINVAL;
  delete reinterpret_cast<racer::AlphaController*>(ctl);
  return RACER_OK;
}

int32_t alpha_ctl_decide(racer_alpha_ctl_t* ctl, const racer_alpha_state* s, double* step, double* alpha_next, int32_t* burst) {
  if (!ctl || !s || !alpha_next) return RACER_EINVAL;
  if (!(s->alpha >= 0.0 && s->alpha <= 1.0) || !(s->p99_latency_ms >= 0.0)) return RACER_EINVAL;
  const racer::AlphaState st{s->hot_user_ratio, s->kv_hit_rate, s->emb_hit_rate, s->mean_seq_len, s->slo_violation,
                             s->alpha, s->p99_latency_ms};
  *alpha_next = reinterpret_cast<racer::AlphaController*>(ctl)->decide(st, step, burst);
  return RACER_OK;
}

double alpha_ctl_reward(double slo_satisfaction, double p99_latency_ms, double slo_ms) {
  return racer::alpha_reward(slo_satisfaction, p99_latency_ms, slo_ms);
}

int32_t racer_hbm_probe(const void* dev_base, uint64_t bytes, uint32_t row_bytes, uint64_t n_reads, void* dev_out,
                        uint64_t seed, void* stream_v) {
  if (!dev_base || n_reads == 0 || (row_bytes != 128 && row_bytes != 256 && row_bytes != 512 && row_bytes != 1024)) return RACER_EINVAL;
  if (bytes < row_bytes || (reinterpret_cast<uintptr_t>(dev_base) & 15) || (reinterpret_cast<uintptr_t>(dev_out) & 15)) return RACER_EINVAL;
  HIP_TRY(racer::launch_random_row_reads(dev_base, bytes / row_bytes, row_bytes, n_reads, dev_out, seed,
                                         static_cast<hipStream_t>(stream_v)));
  return RACER_OK;
}

int32_t racer_prof_enable(racer_pool_t* p, int32_t on) {
  if (!p || !p->device) return RACER_EINVAL;
  p->prof_on = on != 0;
  return RACER_OK;
}

int32_t racer_prof_read(racer_pool_t* p, racer_prof* out) {
  if (!p || !p->device || !out) return RACER_EINVAL;
  std::memset(out, 0, sizeof(*out));
  HIP_TRY(hipStreamSynchronize(p->last_stream));
  for (const racer_pool::ProfMark& m : p->prof) {
    float ms = 0.0f;
    HIP_TRY(hipEventElapsedTime(&ms, m.a, m.b));
    out->ms[m.kind] += ms;
    out->launches[m.kind] += 1;
    p->prof_spare.push_back(m.a);
    p->prof_spare.push_back(m.b);
  }
  p->prof.clear();
  return RACER_OK;
}

}  // extern "C"
