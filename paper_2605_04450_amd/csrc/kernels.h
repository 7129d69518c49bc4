// Launch interfaces between the C-ABI layer and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <cstdint>

namespace racer {

// Device counters (unsigned long long each)
enum Counter : int {
  kCtrLookups = 0, kCtrHits, kCtrMisses, kCtrUnique, kCtrInserted, kCtrEvicted, kCtrBypassed,
  kCtrInvalid, kCtrShrinkEvicted, kCtrShrinkMoved, kCtrBadPages, kCtrUnorderedTs, kCtrCount
};

// The counters exist in kCtrShards copies; a block adds to the copy chosen by its index so that
// thousands of blocks do not serialise on one address.  pool_stats adds the copies up.
constexpr int kCtrShards = 64;
#if defined(__HIPCC__)
__device__ __forceinline__ int ctr_index(int counter) { return static_cast<int>(blockIdx.x & (kCtrShards - 1)) * kCtrCount + counter; }
#endif

// One embedding table behind the pool.  With several tables a row is known by its global id, base + row; rows
// narrower than the pool's slots are kept zero-padded.
struct TableDesc {
  uint64_t base, rows;
  const uint8_t* ptr;  // device-visible address of the pinned host rows
  uint32_t row_bytes, pad;
};
constexpr uint32_t kMaxTables = 32;

// Everything a kernel needs to find a cache set, its ways and its rows.
// Way layer w of the cache = slot w of every set = `layer_pages` consecutive logical EMB
// pages; slot (w, s) lives in logical page w*layer_pages + s/spp at offset s%spp.
struct EmbView {
  uint8_t* base;            // pool backing store
  uint64_t page_size;
  uint32_t row_bytes;
  uint32_t spp;             // slots per page
  uint32_t w_max;
  uint32_t elem;            // 0 fp32, 1 bf16
  uint32_t sets;
  uint32_t layer_pages;
  uint32_t full_ways;       // n_emb / layer_pages
  uint32_t part_sets;       // (n_emb % layer_pages) * spp: these sets have one more way
  uint32_t* tags;           // [sets][w_max]
  uint32_t* stamps;         // [sets][w_max]
  const int32_t* emb_pages; // logical -> physical page
  const uint8_t* table;     // device-visible address of the pinned host table
  uint64_t rows;            // rows of all tables together
  const TableDesc* tables;  // more than one table: their descriptors, bases ascending (else nullptr)
  uint32_t n_tables;
  unsigned long long* counters;
};

// Per-call scratch of the miss path.  ctr points at three zeroed words:
// [0] misses listed, [1] deferred output rows, [2] unique misses.
struct MissWs {
  uint32_t* ctr;
  uint32_t* ctr_next;       // the other parity's words, zeroed by the probe kernel
  uint32_t* miss_list;      // lookup indices that missed
  uint32_t* def_list;       // output rows that wait for a miss
  int64_t* loc;             // per lookup of a deferred row: >=0 pool byte offset, -1 zero row, <=-3 staging row -(v+3)
  unsigned long long* hkeys;  // id dedupe table: (batch << 32) | id
  unsigned long long* hvals;  // (batch << 32) | (0xFFFFFFFF - first lookup index)
  uint32_t* hslot_u;          // unique-miss number of the table slot
  uint32_t hmask;
  unsigned long long* heads;  // per-set chains of unique misses: (batch << 32) | unique number
  uint32_t headmask;
  uint32_t* u_i;
  uint32_t* u_id;
  uint32_t* u_set;
  int32_t* u_next;
  int32_t* u_way;
  uint8_t* staging;         // [unique][row_bytes] rows fetched from the host table
};

hipError_t launch_emb_probe(const EmbView& v, const MissWs& ws, const int64_t* ids, uint32_t n, uint32_t bag,
                            uint8_t* out, uint8_t* hit_flags, uint32_t batch, hipStream_t stream);
hipError_t launch_emb_miss_path(const EmbView& v, const MissWs& ws, const int64_t* ids, uint32_t n, uint32_t bag,
                                uint8_t* out, uint32_t batch, hipStream_t stream);

// refill of empty ways with `ids` (hottest first): probe, then the miss path restricted to empty ways
hipError_t launch_emb_refill(const EmbView& v, const MissWs& ws, const int64_t* ids, uint32_t n, uint32_t batch,
                             hipStream_t stream);

hipError_t launch_emb_shrink(const EmbView& v, uint32_t old_full, uint32_t old_part_sets,
                             hipStream_t stream);

hipError_t launch_fill_u32(uint32_t* p, uint64_t n, uint32_t value, hipStream_t stream);

// measurement aid: n_reads reads of random rows (128, 256, 512 or 1024 bytes) out of n_rows rows at `base`,
// written out back to back at `out` unless that is null
hipError_t launch_random_row_reads(const void* base, uint64_t n_rows, uint32_t row_bytes, uint64_t n_reads, void* out,
                                   uint64_t seed, hipStream_t stream);

// (table, row) pairs -> global ids (-1 for a table or row that does not exist)
hipError_t launch_emb_global_ids(const EmbView& v, const uint32_t* table_of, const int64_t* ids, uint32_t n, int64_t* gids,
                                 hipStream_t stream);

// ---- HSTU -----------------------------------------------------------------------------
struct HstuDims {
  uint32_t L, d, H, dh, elem, pt, n_pos, n_time;
  float inv_n, eps;
  uint32_t pt_shift;  // log2(pt) when pt is a power of two, else 32
};

struct ReqDev {  // device copy of one request
  uint32_t prefix_len, new_len;
  uint32_t page_table_off, ts_off, x_off;
  uint32_t ts_ordered;  // 1 from the host, cleared by the timestamp check if the request's timestamps decrease somewhere
};

struct KvView {
  uint8_t* base;
  uint64_t page_size;
  uint32_t n_pages;
  unsigned long long* counters;
};

constexpr uint32_t kAttnQueries = 256;
constexpr uint32_t kAttnMaxItemPages = 1024;  // page-table entries one attention item may span

// One attention work item: q_block (128) queries of one request against the key tiles [kt_begin, kt_end)
// (64 keys each).  A query tile whose key range was cut into several items accumulates
// through fp32 partial slots (slot .. slot + chunks - 1) that a reduction pass adds up in
// order; an item that covers its whole key range writes the output directly (slot = kDirect).
struct AttnItem {
  uint32_t req, qt, kt_begin, kt_end, slot, pad;
};
struct AttnGroup {
  uint32_t req, qt, slot0, chunks;
};
constexpr uint32_t kDirect = 0xFFFFFFFFu;

// What one attention workgroup does: an item for one head.  Workgroup ids go round-robin over
// the chip's kXcds dies, each with an L2 of its own, so entry i of the work list runs on die
// i % kXcds: the host lays the list out so that the items of all query tiles that read the
// same keys of the same head sit on one die, next to each other, and share those keys through
// its L2 instead of each fetching them from memory.  Entries with item = kNoWork pad the list.
struct AttnWork {
  uint32_t item, head;
};
constexpr uint32_t kXcds = 8;
constexpr uint32_t kNoWork = 0xFFFFFFFFu;

// Up to 128 consecutive new-token rows of one request (projection GEMM tile)
struct RowTile {
  uint32_t row0, rows, req, pad;
};

// row -> request map and work lists built on the host for one step
struct StepLists {
  const ReqDev* reqs;        // [B]
  const uint32_t* row_req;   // [N] request of each new-token row
  const AttnItem* items;     // grouped by (request, key chunk)
  const AttnWork* work;      // [n_work] workgroup -> (item, head), die-interleaved
  uint32_t n_work;
  const AttnGroup* groups;   // query tiles that were split
  const RowTile* row_tiles;  // projection tiles, none crosses a request
  uint32_t n_row_tiles;
  float* partials;           // [slot][head][q_block][64]
  uint32_t n_items, n_groups;
  uint32_t q_block;          // queries per item
  uint32_t B, N;
};

// One pass over every request's timestamps (max_seq: the longest request's prefix + new tokens): ts_ordered, which
// the host has set to 1, is cleared for each request whose timestamps decrease somewhere, and the number of such
// requests is added to the kCtrUnorderedTs counter.  The attention kernels take their 32-bit
// relative-time paths only for ordered requests (an unordered one gets the general 64-bit gaps, where a negative gap
// falls into bucket 0).
hipError_t launch_check_timestamps(ReqDev* reqs, uint32_t B, uint32_t max_seq, const int64_t* ts,
                                   unsigned long long* counters, hipStream_t stream);

hipError_t launch_layernorm(const HstuDims& hd, const void* x, const float* g, const float* b,
                            const void* gate /*nullable: multiply by gate rows*/, void* y, uint32_t N,
                            hipStream_t stream);
hipError_t launch_gemm_front(const HstuDims& hd, uint32_t layer, const void* xn, const void* w1t,
                             const float* b1, void* u, void* q, const KvView& kv, const StepLists& sl,
                             const int32_t* page_tables, hipStream_t stream);
hipError_t launch_gemm_back(const HstuDims& hd, const void* g, const void* w2t, const float* b2,
                            const void* x, void* y, uint32_t N, hipStream_t stream);
// bf16 models with d = 128 or 256: LayerNorm, projection and epilogue of a layer half in one kernel
// (front: X -> U, Q*log2(e), K/V pages; back: O, U, X -> Y); weights transposed as for the GEMMs.
// In bf16 models U, O, the normalised matrices and the transposed weights (launch_transpose_weights) are half precision.
bool layer_halves_fused(const HstuDims& hd);
hipError_t launch_layer_front_fused(const HstuDims& hd, uint32_t layer, const void* x, const float* ln_g,
                                    const float* ln_b, const void* w1t, const float* b1, void* u, void* q,
                                    const KvView& kv, const StepLists& sl, const int32_t* page_tables,
                                    hipStream_t stream);
hipError_t launch_layer_back_fused(const HstuDims& hd, const void* o, const void* u, const float* ln_g,
                                   const float* ln_b, const void* w2t, const float* b2, const void* x, void* y,
                                   const StepLists& sl, hipStream_t stream);
// o_half (bf16 models): the output is written in half precision (the step's own matrix between the attention and the
// second LayerNorm) instead of bf16 (what a caller of the attention alone gets)
hipError_t launch_attention(const HstuDims& hd, uint32_t layer, const void* q, const float* pos,
                            const float* time, const KvView& kv, const StepLists& sl,
                            const int32_t* page_tables, const int64_t* ts, void* o, bool o_half, hipStream_t stream);
// adds up the fp32 partials of split attention items (no-op when nothing was split)
hipError_t launch_attention_reduce(const HstuDims& hd, const StepLists& sl, void* o, bool o_half, hipStream_t stream);
// bf16 models: pos and time must be the tables multiplied by log2(e) (launch_scale_bias), and
// q must already be multiplied by log2(e) (launch_gemm_front stores it that way)
hipError_t launch_scale_bias(const float* in, float* out, uint64_t n, hipStream_t stream);
hipError_t launch_scale_q(const void* in, void* out, uint64_t n, hipStream_t stream);
hipError_t launch_transpose_weights(const void* w, void* wt, uint32_t rows, uint32_t cols, uint32_t elem,
                                    hipStream_t stream);

}  // namespace racer
