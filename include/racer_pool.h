/*
 * C-ABI of the MI355X hot path of one HSTU serving step over a single shared
 * HBM page pool (embedding hot cache + paged KV cache behind one movable
 * EMB:KV boundary).
 *
 * Conventions
 *   - plain C, opaque handles, every call returns int32_t:
 *       0 = OK, > 0 = OK with a condition (RACER_DEFERRED, RACER_NOT_FOUND),
 *       < 0 = error (negated errno-style codes below); nothing is thrown.
 *   - "dev" pointers are device addresses, "host" pointers are host addresses.
 *     All data buffers (the pool's backing store, ids, outputs, page tables,
 *     weights) are owned by the caller; the library allocates only its own
 *     metadata and workspaces and frees them in the destroy calls.  It never
 *     frees or reallocates caller memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Work
 *     is enqueued on it and the call returns without waiting unless stated.
 *     All calls on one pool must be issued from one host thread at a time and
 *     on streams the caller keeps ordered with one another; two calls that
 *     overlap on one pool race.
 *   - Counters live on the device; pool_stats() waits for the pool's last
 *     stream before reading them.
 */
#ifndef RACER_POOL_H
#define RACER_POOL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RACER_OK 0
#define RACER_DEFERRED 1  /* EMB expansion only partly served (paper Sec. IV-B: "throttled/deferred") */
#define RACER_NOT_FOUND 2 /* kv_seq_*: no such resident sequence */
#define RACER_EINVAL (-22)
#define RACER_ENOMEM (-12)
#define RACER_ERANGE (-34)
#define RACER_EBUSY (-16)
#define RACER_EHIP (-5) /* a HIP runtime call failed; see racer_last_error() */

#define RACER_ELEM_F32 0
#define RACER_ELEM_BF16 1
#define RACER_TAG_EMPTY 0xFFFFFFFFu

typedef struct racer_pool racer_pool_t;
typedef struct racer_hstu racer_hstu_t;

typedef struct {
  uint32_t row_bytes;     /* R: bytes of one embedding row = d * elem size; multiple of 16 */
  uint32_t elem;          /* RACER_ELEM_F32 or RACER_ELEM_BF16 */
  uint32_t page_tokens;   /* KV tokens per page */
  uint32_t w_max;         /* ways per set when the whole pool is EMB: power of two <= 32 */
  const void* host_table; /* host: pinned, device-mapped table [rows][row_bytes]; may be NULL if emb_lookup is unused */
  uint64_t rows;          /* rows of host_table, < 2^32 - 1 */
  double emb_frac0;       /* initial EMB fraction in [0, 1] */
} racer_pool_cfg;

typedef struct {
  uint64_t lookups, hits, misses, unique_misses, inserted, evicted, bypassed, invalid_ids;
  uint64_t shrink_evicted, shrink_moved;
  uint64_t pages_total, pages_emb, pages_kv_used, pages_kv_free;
  uint64_t seqs_resident, seqs_evicted;
  uint64_t batch;        /* number of emb_lookup calls so far (the LRU clock) */
  uint64_t bad_pages;    /* page-table entries outside the pool seen by hstu kernels (skipped) */
  uint64_t unordered_ts; /* requests of hstu calls whose timestamps decreased somewhere (served by the general time path) */
  uint64_t ws_allocs;    /* (re)allocations of the library's work spaces so far; constant once pool_reserve covers the load */
} racer_pool_stats;

/* ---- pool (paper Sec. IV-B: one shared paged HBM space, movable logical EMB:KV boundary;
 *      Sec. IV-A: M_emb = alpha * M, M_kv = (1 - alpha) * M) -------------------------------
 *
 * pool_create: dev_base (dev, caller-owned, 256-byte aligned) backs bytes/page_size pages.
 * Requirements: bytes % page_size == 0, page_size % row_bytes == 0, pages % w_max == 0,
 * pages < 2^31.  Page p occupies [dev_base + p*page_size, +page_size).  On the KV side a
 * page holds page_tokens tokens of all layers as [layer][K|V][head] blocks of
 * page_tokens*d_h elements: a K block is [token][d_h], a V block is stored transposed,
 * [d_h][token] (the attention kernel contracts over tokens and reads them contiguously);
 * KV bytes per token are 2*L*d*elem (paper Sec. V-E: 60-184 MB per user at 8K-15K tokens).
 * On the EMB side a page holds page_size/row_bytes embedding slots.  round-half-away(emb_frac0 * pages)
 * lowest-numbered pages start on the EMB side, the rest on the KV free list.
 * dev_base == NULL creates a metadata-only pool (host bookkeeping works, device calls
 * return RACER_EINVAL): this is what CPU-only hosts can exercise.
 * Errors: RACER_EINVAL (geometry), RACER_ENOMEM / RACER_EHIP (metadata allocation). */
int32_t pool_create(void* dev_base, uint64_t bytes, uint64_t page_size, const racer_pool_cfg* cfg,
                    racer_pool_t** out);
int32_t pool_destroy(racer_pool_t* pool);

/* pool_set_split (paper Sec. IV-B "Embedding-only boundary adjustment", Eq. 6 for the
 * domain): move the boundary to round(emb_frac * pages).  emb_frac outside [0.1, 0.9] ->
 * RACER_EINVAL.  Growing EMB: free KV pages are taken lowest id first; if too few are
 * free, cold unpinned sequences are dropped in LRU order (metadata only); if still short
 * the pages that exist are taken and RACER_DEFERRED is returned with *achieved < emb_frac.
 * Shrinking EMB: per cache set the least recently used entries leave, survivors from the
 * removed ways move into vacated lower ways (device-to-device, enqueued on `stream`), the
 * tail pages return to the KV free list.  Resident KV pages never move and no host<->device
 * data copy is made.  Host metadata is final on return; `achieved` (host, may be NULL)
 * receives pages_emb / pages.  If the device half cannot be queued (RACER_EHIP, RACER_ENOMEM)
 * the host metadata is put back as it was: the split, the page owners and the resident
 * sequences are those from before the call. */
int32_t pool_set_split(racer_pool_t* pool, double emb_frac, void* stream, double* achieved);

/* pool_reserve: size the library's work spaces once.  The miss path's lists, the step's activation matrices,
 * work lists, partial outputs, pinned staging buffers and the step's streams otherwise grow on demand, and a
 * growth (hipFree + hipMalloc, after waiting for the streams that use the old buffer) stalls the device in the
 * middle of serving.  After pool_reserve, no call whose sizes stay within *r allocates (pool_stats.ws_allocs
 * stays constant).  model (may be NULL: EMB calls only) fixes width, heads, element type and page tokens of the
 * steps to come.  A later call beyond the reserved sizes still works and grows what it needs.
 * Errors: RACER_EINVAL (metadata-only pool, sizes out of range), RACER_EHIP / RACER_ENOMEM. */
typedef struct {
  uint64_t max_lookups;    /* ids per emb_lookup / emb_lookup_tables / emb_refill call; 0: none */
  uint32_t max_requests;   /* requests per hstu_step / hstu_attn_paged call; 0: none */
  uint64_t max_new_tokens; /* sum of new_len over the requests of one call */
  uint32_t max_seq_tokens; /* largest prefix_len + new_len of a request */
} racer_reserve;
int32_t pool_reserve(racer_pool_t* pool, const racer_hstu_t* model, const racer_reserve* r, void* stream);

/* pool_stats: waits for the pool's last stream, then fills *out (host). */
int32_t pool_stats(racer_pool_t* pool, racer_pool_stats* out);

/* pool_dump / emb_cache_dump: parity helpers. Host output arrays, NULL = skip.
 * emb_pages[pages_emb] logical->physical, owner[pages] (0 free, 1 EMB, 2 KV);
 * tags, stamps: [sets][w_max] copied from the device after a stream wait. */
int32_t pool_dump(racer_pool_t* pool, int64_t* emb_pages, uint8_t* owner);
int32_t emb_cache_dump(racer_pool_t* pool, uint32_t* tags, uint32_t* stamps);
uint64_t pool_num_sets(const racer_pool_t* pool);
/* physical slot (page * slots_per_page + offset) of way `way` of set `set`, -1 if absent */
int64_t pool_slot_of(const racer_pool_t* pool, uint64_t set, uint32_t way);

/* ---- KV sequences (paper Sec. IV-B: paged block pool with free list and page tables,
 *      indexed per user; LRU reclaim of cold blocks is metadata-only; in-flight blocks
 *      are pinned).  Host-only calls, no device work. --------------------------------------
 * kv_seq_reserve: make sequence `key` cover at least `tokens` tokens (never shrinks).  New
 * pages are the lowest-numbered free ones; when none are free, other unpinned sequences
 * are dropped least-recently-used first.  If free + reclaimable pages do not suffice:
 * RACER_ENOMEM and no state change.  Touches the sequence's LRU stamp.  pages_out (host,
 * may be NULL) receives all pages of the sequence if cap suffices, else RACER_EINVAL. */
int32_t kv_seq_reserve(racer_pool_t* pool, uint64_t key, uint32_t tokens, int32_t* pages_out,
                       uint32_t cap, uint32_t* n_pages_out);
int32_t kv_seq_lookup(const racer_pool_t* pool, uint64_t key, uint32_t* tokens, int32_t* pages_out,
                      uint32_t cap, uint32_t* n_pages_out);
int32_t kv_seq_pin(racer_pool_t* pool, uint64_t key);   /* also touches the LRU stamp */
int32_t kv_seq_unpin(racer_pool_t* pool, uint64_t key);
int32_t kv_seq_release(racer_pool_t* pool, uint64_t key); /* RACER_EBUSY while pinned */

/* ---- emb_lookup (paper Sec. II-B stage "EMB lookup": probe the node's HBM embedding
 *      cache, fetch absent rows from the CPU-resident table; Sec. IV-B: LRU-managed slab
 *      with page-granular allocation) -------------------------------------------------------
 * ids (dev) int64[n]; bag = lookups summed per output row (n % bag == 0); out (dev)
 * [n/bag][row_bytes] in the pool's element type; hit_flags (dev, may be NULL) u8[n].
 * One call is one LRU batch: hit = resident when the call starts; every hit way is stamped
 * with the batch number; each distinct missing id is inserted once, in order of first
 * occurrence (empty way, else least recently used way not touched in this batch, else the
 * id bypasses the cache).  out rows always equal the host table's rows; bags are summed in
 * fp32 left to right and rounded once.  ids outside [0, rows) count as invalid_ids and
 * contribute zeros.  Errors: RACER_EINVAL (bag, NULL pool data), RACER_EHIP. */
int32_t emb_lookup(racer_pool_t* pool, const int64_t* ids, uint64_t n, uint32_t bag, void* out,
                   uint8_t* hit_flags, void* stream);

/* ---- emb_lookup_noalloc: emb_lookup for callers that cannot allocate device memory: code under HIP graph
 *      capture, tight serving loops, harnesses that forbid allocation.  Same arguments, results and LRU
 *      semantics as emb_lookup; the miss path's work space is a fixed array inside the library (one per GPU,
 *      about 10 MB, held until the process ends), and the call makes no hipMalloc / hipFree or other
 *      allocating call and creates no events (racer_prof does not see it).  Limits: n <=
 *      RACER_NOALLOC_MAX_LOOKUPS and n * row_bytes <= RACER_NOALLOC_MAX_ROW_BYTES_TOTAL, else RACER_ERANGE
 *      and nothing is done.  Every call on a GPU, whatever its pool, shares that GPU's array: calls that
 *      overlap on one GPU (two streams, two threads) race; calls ordered on one stream, or by the caller's own
 *      events, do not.  Must be called with the pool's GPU current. */
#define RACER_NOALLOC_MAX_LOOKUPS 16384ull
#define RACER_NOALLOC_MAX_ROW_BYTES_TOTAL (8ull << 20)
int32_t emb_lookup_noalloc(racer_pool_t* pool, const int64_t* ids, uint64_t n, uint32_t bag, void* out,
                           uint8_t* hit_flags, void* stream);

/* ---- several tables in one pool (paper Sec. II-B / III: a model looks up 10-25 embedding
 *      tables per request, and the lookup cost grows linearly with their number) -----------
 * pool_add_table: another pinned, device-mapped host table [rows][row_bytes] of the pool's
 * element type behind the same hot cache; row_bytes a multiple of 16, at most the pool's
 * (a narrower row occupies a whole slot, zero-padded).  Tables are numbered in the order
 * they were added, pool_create's being table 0; *table_out (host, may be NULL) receives the
 * number.  A row's global id is the sum of the rows of the tables before its own plus its
 * row number: global ids are what the cache tags hold and what emb_lookup / emb_refill
 * take once there is more than one table; all tables together must stay below 2^32 - 1
 * rows, and there are at most 32.  Waits for the pool's stream.
 * emb_lookup_tables: emb_lookup for (table, row) pairs: table_of (dev) u32[n], ids (dev)
 * int64[n] row numbers inside their tables; all tables are probed in one launch.  out (dev)
 * [n/bag][pool row_bytes]: a narrower table's row comes zero-padded.  A pair whose table or
 * row does not exist counts as an invalid id.  Equal to emb_lookup on the concatenation of
 * the zero-padded tables.  Errors: RACER_EINVAL (fewer than two tables, geometry), RACER_EHIP. */
int32_t pool_add_table(racer_pool_t* pool, const void* host_table, uint64_t rows, uint32_t row_bytes,
                       uint32_t* table_out);
int32_t emb_lookup_tables(racer_pool_t* pool, const uint32_t* table_of, const int64_t* ids, uint64_t n,
                          uint32_t bag, void* out, uint8_t* hit_flags, void* stream);

/* ---- emb_refill (paper Sec. IV-B, last paragraph: after the EMB side has grown, its new
 *      capacity is filled with hot rows in the background, throttled against the live
 *      misses' host-to-device traffic) ------------------------------------------------------
 * ids (dev) int64[n], hottest first (the caller's ranking).  One call is one LRU batch of its
 * own: every valid id that is not resident when the call starts is fetched from the host
 * table, once, into the lowest empty way of its set (the k-th such id of a set, by first
 * occurrence, takes the set's k-th empty way) and stamped with the batch; an id whose set
 * has no empty way left is skipped.  A refill never evicts, never re-stamps a resident row,
 * writes no output and counts only in pool_stats.inserted.  It moves at most n * row_bytes
 * over PCIe: the caller throttles by the size and pacing of its calls (calls on one pool
 * must not overlap each other or a lookup: they share the pool's work space).
 * Errors: RACER_EINVAL (NULL pool data, n >= 2^32 - 1), RACER_EHIP. */
int32_t emb_refill(racer_pool_t* pool, const int64_t* ids, uint64_t n, void* stream);

/* ---- HSTU (paper Sec. II-A/II-B stage "Compute": stacked HSTU blocks that reuse resident
 *      KV state; equations are the published HSTU layer) ------------------------------------ */
typedef struct {
  uint32_t L, d, H;
  uint32_t elem;        /* storage type of activations, W1/W2 and KV: RACER_ELEM_* */
  uint32_t page_tokens; /* must equal the pool's */
  uint32_t n_pos;       /* rows of the positional bias table; distance is clamped to n_pos-1 */
  uint32_t n_time;      /* log2 time-gap buckets, clamped to n_time-1 */
  float n_scale;        /* attention output is divided by this */
  float eps;            /* LayerNorm epsilon */
} racer_hstu_cfg;

/* device pointers, all layers concatenated; w1 [L][d][4d] and w2 [L][d][d] in the model's
 * element type (row-major, input-major: y = x W), everything else fp32:
 * ln1_g, ln1_b [L][d]; b1 [L][4d]; ln2_g, ln2_b [L][d]; b2 [L][d]; pos [L][H][n_pos];
 * time [L][H][n_time].  Columns of W1 are ordered U | V | Q | K, head h owning columns
 * h*d/H .. (h+1)*d/H - 1 of each block.  The arrays must stay valid while the model lives. */
typedef struct {
  const void *ln1_g, *ln1_b, *w1, *b1, *ln2_g, *ln2_b, *w2, *b2, *pos, *time;
} racer_hstu_weights;

typedef struct {
  uint32_t prefix_len;     /* tokens whose K,V already sit in the request's pages */
  uint32_t new_len;        /* tokens processed by this step */
  uint64_t page_table_off; /* first entry of this request in kv_page_tables */
  uint64_t ts_off;         /* first of prefix_len + new_len timestamps in ts */
  uint64_t x_off;          /* first of new_len rows in x_in / out */
} racer_hstu_req;

/* Supported shapes: elem bf16 with d/H == 64 (MFMA path) or elem fp32 with d/H <= 64;
 * d % 64 == 0 for bf16, d % 16 == 0 for fp32; otherwise RACER_EINVAL. */
int32_t hstu_model_create(const racer_hstu_cfg* cfg, const racer_hstu_weights* weights,
                          racer_hstu_t** out);
int32_t hstu_model_destroy(racer_hstu_t* model);

/* hstu_step: all L layers for B requests.  reqs (host) [B]; kv_page_tables (dev) int32,
 * n_page_entries long, request r using ceil((prefix+new)/page_tokens) entries from its
 * offset; x_in (dev) [N][d] new-token inputs (N = sum new_len); ts (dev) int64 seconds,
 * normally non-decreasing per request (a request whose timestamps decrease somewhere is
 * served all the same, by a slower path in which a negative gap falls into bucket 0, and
 * counted in pool_stats.unordered_ts); out (dev) [N][d].  For every layer the new tokens' K,V are
 * written into the request's pages at positions prefix_len.., then every new token attends
 * to positions 0..its own through the page table.  Page ids outside the pool are skipped
 * and counted in bad_pages.  The work is ordered on `stream` as usual: what the caller
 * queues behind the call sees the finished outputs.  Inside, a bf16 batch of 32 768 or more
 * new tokens, or 2^26 or more (query, key) pairs, runs as three pipelines over three runs of requests, two of
 * them on streams of the pool's own (default priority) that fork from `stream` at the start
 * and join it at the end; results do not depend on it.  While racer_prof_enable is on,
 * the step runs as one pipeline so that kernel durations do not overlap.
 * Errors: RACER_EINVAL (shape mismatch with the pool, offsets beyond n_page_entries),
 * RACER_ENOMEM/RACER_EHIP (workspace). */
int32_t hstu_step(racer_pool_t* pool, racer_hstu_t* model, const racer_hstu_req* reqs, uint32_t B,
                  const int32_t* kv_page_tables, uint64_t n_page_entries, const void* x_in,
                  const int64_t* ts, void* out, void* stream);

/* hstu_attn_paged: the attention of one layer alone (for kernel-level measurement and
 * parity): q (dev) [N][d] in the element type, K,V read from the pages as they are,
 * o (dev) [N][d] = (1/n) sum_{j<=p} SiLU(q.k_j + rab(p, j)) v_j per head. */
int32_t hstu_attn_paged(racer_pool_t* pool, racer_hstu_t* model, uint32_t layer,
                        const racer_hstu_req* reqs, uint32_t B, const int32_t* kv_page_tables,
                        uint64_t n_page_entries, const void* q, const int64_t* ts, void* o,
                        void* stream);

/* ---- split controller (paper Sec. IV-A "Adaptive EMB-KV Memory Allocation") -------------------------------
 * Host only.  Once per decision epoch the caller hands over the state vector of Table I (what it measured
 * over the last window: rates in [0, 1], lengths in tokens, latency in ms, alpha = the fraction that was in
 * force) and receives a step out of the action set of Eq. 3, {+-0.06, +-0.04, +-0.02, 0}, and the next
 * fraction clip(alpha + step, 0.1, 0.9) (Eq. 4, Eq. 6), which it applies with pool_set_split.  The paper's
 * policy networks (PPO base policy, Online Adapter) were trained on traces that are not published; the
 * policy here is a stand-in, a hill climb on the measured P99 latency (the objective of Eq. 1): it keeps
 * its direction and step while the latency falls, turns back with the next smaller step when it rises,
 * shrinks the step when nothing changes, holds when the step has reached 0, and probes again with 0.02 after
 * six epochs or when the latency drifts up by more than 10 %.  The Recovery Controller is the paper's rule:
 * an epoch whose latency exceeds the mean of the last ten epochs by more than three standard deviations
 * (floored at 5 % of that mean, so that the controller's own probes on a quiet system are no bursts) is a
 * burst (*burst = 1); the step is then -0.06 (memory towards the KV cache) if the hot-user ratio exceeds
 * 0.2, else 0, and the climb starts over afterwards.  slo_ms = tau_SLO.  No parity claim against the
 * paper's controller is possible.
 * alpha_ctl_reward: the reward of Eq. 5, slo_satisfaction - max(0, p99 - slo) / slo. */
typedef struct racer_alpha_ctl racer_alpha_ctl_t;
typedef struct {
  double hot_user_ratio;  /* h_t: share of the window's requests that came from hot users */
  double kv_hit_rate;     /* k_t */
  double emb_hit_rate;    /* e_t */
  double mean_seq_len;    /* L_t */
  double slo_violation;   /* v_t */
  double alpha;           /* alpha_t */
  double p99_latency_ms;  /* l_t */
} racer_alpha_state;
int32_t alpha_ctl_create(double slo_ms, racer_alpha_ctl_t** out);
int32_t alpha_ctl_destroy(racer_alpha_ctl_t* ctl);
int32_t alpha_ctl_decide(racer_alpha_ctl_t* ctl, const racer_alpha_state* s, double* step /* may be NULL */,
                         double* alpha_next, int32_t* burst /* may be NULL */);
double alpha_ctl_reward(double slo_satisfaction, double p99_latency_ms, double slo_ms);

/* ---- per-kernel-class timing for benchmarks: when enabled, every launch (the miss path as
 *      one group) is bracketed by HIP events on the caller's stream.  racer_prof_read waits
 *      for the pool's last stream, adds up the intervals recorded since the previous read and
 *      clears them. */
#define RACER_PROF_EMB_GATHER 0 /* probe + hit gather kernel */
#define RACER_PROF_EMB_MISS 1   /* the miss-path kernels of one emb_lookup, as a group */
#define RACER_PROF_LAYERNORM 2
#define RACER_PROF_GEMM_FRONT 3
#define RACER_PROF_ATTENTION 4
#define RACER_PROF_GEMM_BACK 5
#define RACER_PROF_ATTN_REDUCE 6 /* sum of the partial outputs of split attention items */
#define RACER_PROF_KINDS 7
typedef struct {
  double ms[RACER_PROF_KINDS];
  uint64_t launches[RACER_PROF_KINDS];
} racer_prof;
int32_t racer_prof_enable(racer_pool_t* pool, int32_t on);
int32_t racer_prof_read(racer_pool_t* pool, racer_prof* out);

/* ---- racer_hbm_probe: a measurement aid, not part of the serving path.  It reads n_reads rows of row_bytes
 *      (128, 256, 512 or 1024) bytes, picked by a counter-based hash of (seed, index), out of the bytes at dev_base
 *      (dev, 16-byte aligned), four rows in flight per lane group, and writes them back to back to dev_out (dev,
 *      n_reads * row_bytes bytes; NULL: read only).  Timed by the caller, it gives the rate that the memory
 *      system grants a gather of rows of that size out of a region that no cache holds: the practical ceiling
 *      against which the embedding gather is read (bench.py --config hbmceiling).  RACER_EINVAL on bad arguments. */
int32_t racer_hbm_probe(const void* dev_base, uint64_t bytes, uint32_t row_bytes, uint64_t n_reads, void* dev_out,
                        uint64_t seed, void* stream);

/* text of the last HIP error seen by this library on the calling thread ("" if none) */
const char* racer_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
