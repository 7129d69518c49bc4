// Embedding hot-cache kernels for gfx950: wavefront-parallel set probe fused with the
// row gather, and the miss path (LDS-staged compaction, dedupe by first occurrence,
// ordered per-set victim choice, zero-copy fetch from the pinned host table).
//
// The policy these kernels realise (paper Sec. IV-B: an LRU-managed EMB slab with
// page-granular allocation; the batch rules are this build's reading):
//   hit = resident when the batch starts; hit ways are stamped with the batch number;
//   each distinct missing id is inserted once, in first-occurrence order, into the
//   lowest empty way of its set, else into the way with the least (stamp, way) whose
//   stamp is older than this batch, else it bypasses the cache.
// Because a set's victim candidates are fixed once the probe has stamped the hits, the
// k-th unique miss of a set (by first occurrence) simply takes the k-th candidate, so
// the insertion order needs no serial loop: each unique miss computes its own rank.
#include "kernels.h"

namespace racer {
namespace {

constexpr uint32_t kEmpty = 0xFFFFFFFFu;
constexpr int kWave = 64;

__device__ __forceinline__ uint32_t set_of(const EmbView& v, int64_t id) {
  const unsigned long long h = static_cast<unsigned long long>(id) * 0x9E3779B97F4A7C15ull;
  return static_cast<uint32_t>(h >> 32) % v.sets;
}

__device__ __forceinline__ uint32_t ways_of(const EmbView& v, uint32_t set) {
  return v.full_ways + (set < v.part_sets ? 1u : 0u);
}

__device__ __forceinline__ int64_t slot_offset(const EmbView& v, uint32_t set, uint32_t way) {
  const uint32_t logical = way * v.layer_pages + set / v.spp;
  return static_cast<int64_t>(v.emb_pages[logical]) * static_cast<int64_t>(v.page_size) +
         static_cast<int64_t>(set % v.spp) * v.row_bytes;
}

__device__ __forceinline__ int64_t shfl64(int64_t x, int src) {
  int lo = __shfl(static_cast<int>(x & 0xFFFFFFFFll), src, kWave);
  int hi = __shfl(static_cast<int>(x >> 32), src, kWave);
  return (static_cast<int64_t>(hi) << 32) | static_cast<uint32_t>(lo);
}

__device__ __forceinline__ uint32_t lanes_per_row(uint32_t chunks) {
  uint32_t l = 1;
  while (l < 32 && l < chunks) l <<= 1;
  return l;
}

__device__ __forceinline__ float bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

__device__ __forceinline__ uint32_t f32_to_bf16(float f) {  // round to nearest even; finite or inf in
  const uint32_t u = __float_as_uint(f);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// acc (8 fp32 lanes of one 16-byte chunk; fp32 rows use the first 4) <- chunk or acc + chunk
__device__ __forceinline__ void accumulate_chunk(float acc[8], const uint4& c, bool bf16, bool first) {
  float v[8];
  if (bf16) {
    const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      v[2 * k] = bf16_to_f32(w[k] & 0xFFFFu);
      v[2 * k + 1] = bf16_to_f32(w[k] >> 16);
    }
  } else {
    v[0] = __uint_as_float(c.x); v[1] = __uint_as_float(c.y);
    v[2] = __uint_as_float(c.z); v[3] = __uint_as_float(c.w);
    v[4] = v[5] = v[6] = v[7] = 0.0f;
  }
#pragma unroll
  for (int k = 0; k < 8; ++k) acc[k] = first ? v[k] : acc[k] + v[k];
}

__device__ __forceinline__ uint4 pack_chunk(const float acc[8], bool bf16) {
  uint4 r;
  if (bf16) {
    r.x = f32_to_bf16(acc[0]) | (f32_to_bf16(acc[1]) << 16);
    r.y = f32_to_bf16(acc[2]) | (f32_to_bf16(acc[3]) << 16);
    r.z = f32_to_bf16(acc[4]) | (f32_to_bf16(acc[5]) << 16);
    r.w = f32_to_bf16(acc[6]) | (f32_to_bf16(acc[7]) << 16);
  } else {
    r.x = __float_as_uint(acc[0]); r.y = __float_as_uint(acc[1]);
    r.z = __float_as_uint(acc[2]); r.w = __float_as_uint(acc[3]);
  }
  return r;
}

// Resolve a `loc` code to a row address (nullptr = all-zero row).
__device__ __forceinline__ const uint8_t* row_address(const EmbView& v, const MissWs& ws, int64_t loc) {
  if (loc >= 0) return v.base + loc;
  if (loc <= -3) return ws.staging + static_cast<uint64_t>(-(loc + 3)) * v.row_bytes;
  return nullptr;
}

// One output row handled by `lpr` lanes (`sub` = this lane's number in the group): bag == 1
// is a raw copy, bag > 1 the fp32 left-to-right sum rounded once.
template <typename LocFn>
__device__ __forceinline__ void emit_row(const EmbView& v, const MissWs& ws, uint32_t bag, uint32_t lpr,
                                         uint32_t sub, uint8_t* dst, LocFn loc_of) {
  const uint32_t chunks = v.row_bytes / 16;
  const bool bf16 = v.elem == 1;
  for (uint32_t c = sub; c < chunks; c += lpr) {
    uint4 outv;
    if (bag == 1) {
      const uint8_t* src = row_address(v, ws, loc_of(0));
      outv = src ? *reinterpret_cast<const uint4*>(src + 16 * c) : make_uint4(0, 0, 0, 0);
    } else {
      float acc[8];
      for (uint32_t f = 0; f < bag; ++f) {
        const uint8_t* src = row_address(v, ws, loc_of(f));
        const uint4 cv = src ? *reinterpret_cast<const uint4*>(src + 16 * c) : make_uint4(0, 0, 0, 0);
        accumulate_chunk(acc, cv, bf16, f == 0);
      }
      outv = pack_chunk(acc, bf16);
    }
    *reinterpret_cast<uint4*>(dst + 16 * c) = outv;
  }
}

// ---------------------------------------------------------------------------------------
// Probe + hit gather.  One wavefront takes `lb` consecutive lookups (a whole number of
// bags, at most 64): lane i owns lookup i, two lookups are probed per step with 32 lanes
// reading one set's tag line each (128 B, coalesced), then rows are copied with
// 16-byte lanes.  Misses and the output rows that must wait for them are staged in LDS
// and appended to the global lists with one atomic per block.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void emb_probe_gather(EmbView v, MissWs ws, const int64_t* __restrict__ ids,
                                                        uint32_t n, uint32_t bag, uint32_t lb,
                                                        uint8_t* __restrict__ out,
                                                        uint8_t* __restrict__ hit_flags, uint32_t batch) {
  __shared__ uint32_t s_miss[256];
  __shared__ uint32_t s_def[256];
  __shared__ uint32_t s_n[2], s_base[2];
  __shared__ uint32_t s_cnt[3];
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid < 2) s_n[tid] = 0;
  if (tid < 3) s_cnt[tid] = 0;
  if (blockIdx.x == 0 && tid < 3) ws.ctr_next[tid] = 0;  // the next call's list counters
  __syncthreads();

  const uint64_t i0 = (static_cast<uint64_t>(blockIdx.x) * 4 + wave) * lb;
  const uint64_t i = i0 + lane;
  const bool active = lane < lb && i < n;
  const int64_t id = active ? ids[i] : -1;
  const bool valid = active && id >= 0 && static_cast<uint64_t>(id) < v.rows;
  const uint32_t id32 = static_cast<uint32_t>(id);
  const uint32_t set = valid ? set_of(v, id) : 0;
  const uint32_t nw = valid ? ways_of(v, set) : 0;

  int my_way = -1;
  if (i0 < n) {
    const uint32_t l32 = lane & 31, half = lane >> 5;
#pragma unroll 4
    for (uint32_t it = 0; it < 32; ++it) {
      const uint32_t a = 2 * it + half;
      const uint32_t id_a = __shfl(id32, a, kWave);
      const uint32_t set_a = __shfl(set, a, kWave);
      const uint32_t nw_a = __shfl(nw, a, kWave);
      bool match = false;
      if (l32 < nw_a) match = v.tags[static_cast<uint64_t>(set_a) * v.w_max + l32] == id_a;
      const unsigned long long m = __ballot(match);
      const uint32_t lo = static_cast<uint32_t>(m), hi = static_cast<uint32_t>(m >> 32);
      if (lane == 2 * it) my_way = lo ? __ffs(lo) - 1 : -1;
      if (lane == 2 * it + 1) my_way = hi ? __ffs(hi) - 1 : -1;
    }
  }
  const bool hit = valid && my_way >= 0;
  const bool miss = valid && !hit;
  int64_t loc = -1;  // zero row (invalid id or padding lane)
  if (hit) {
    loc = slot_offset(v, set, static_cast<uint32_t>(my_way));
    v.stamps[static_cast<uint64_t>(set) * v.w_max + my_way] = batch;
  } else if (miss) {
    loc = -2;  // replaced by the staging row once the miss is resolved
  }
  if (hit_flags && active) hit_flags[i] = hit ? 1 : 0;

  const unsigned long long hit_m = __ballot(hit), valid_m = __ballot(valid), miss_m = __ballot(miss);
  const unsigned long long inval_m = __ballot(active && !valid);
  if (lane == 0) {
    if (hit_m) atomicAdd(&s_cnt[0], __popcll(hit_m));
    if (valid_m) atomicAdd(&s_cnt[1], __popcll(valid_m));
    if (inval_m) atomicAdd(&s_cnt[2], __popcll(inval_m));
  }
  const unsigned long long lt_mask = (1ull << lane) - 1ull;
  if (miss_m) {
    uint32_t base = 0;
    if (lane == 0) base = atomicAdd(&s_n[0], __popcll(miss_m));
    base = __shfl(base, 0, kWave);
    if (miss) s_miss[base + __popcll(miss_m & lt_mask)] = static_cast<uint32_t>(i);
  }
  // an output row waits if any lookup of its bag missed
  const uint32_t b = lane / bag;  // bag of this lane inside the wave's batch
  const unsigned long long bag_mask = (bag >= 64 ? ~0ull : ((1ull << bag) - 1ull)) << (b * bag);
  const bool deferred = active && (miss_m & bag_mask) != 0;
  const bool def_leader = deferred && (lane % bag) == 0;
  const unsigned long long def_m = __ballot(def_leader);
  if (deferred) ws.loc[i] = loc;
  if (def_m) {
    uint32_t base = 0;
    if (lane == 0) base = atomicAdd(&s_n[1], __popcll(def_m));
    base = __shfl(base, 0, kWave);
    if (def_leader) s_def[base + __popcll(def_m & lt_mask)] = static_cast<uint32_t>(i / bag);
  }

  // gather the rows that are complete
  if (i0 < n) {
    const uint32_t chunks = v.row_bytes / 16;
    const uint32_t lpr = lanes_per_row(chunks);
    const uint32_t rows_per_pass = kWave / lpr;
    const uint32_t n_out = lb / bag;  // output rows of this wave's batch
    const uint32_t sub = lane % lpr;
    for (uint32_t r0 = 0; r0 < n_out; r0 += rows_per_pass) {
      const uint32_t r = r0 + lane / lpr;                 // output row inside the batch
      const uint32_t first = (r < n_out ? r : 0) * bag;   // its first lookup lane
      const bool row_active = r < n_out && (i0 + first) < n;
      const bool row_deferred = (__shfl(deferred ? 1 : 0, first, kWave) != 0);
      // all lanes take part in the shuffles; only complete rows are written
      const uint64_t o = (i0 + first) / bag;
      if (bag == 1) {
        const int64_t l0 = shfl64(loc, first);
        if (row_active && !row_deferred)
          emit_row(v, ws, 1, lpr, sub, out + o * v.row_bytes, [&](uint32_t) { return l0; });
      } else {
        // the shuffles inside the lambda are executed by every lane of the wave
        const uint32_t chunks_pad = ((chunks + lpr - 1) / lpr) * lpr;
        for (uint32_t c = sub; c < chunks_pad; c += lpr) {
          float acc[8];
          for (uint32_t f = 0; f < bag; ++f) {
            const int64_t lf = shfl64(loc, first + f);
            if (row_active && !row_deferred && c < chunks) {
              const uint8_t* src = row_address(v, ws, lf);
              const uint4 cv = src ? *reinterpret_cast<const uint4*>(src + 16 * c) : make_uint4(0, 0, 0, 0);
              accumulate_chunk(acc, cv, v.elem == 1, f == 0);
            }
          }
          if (row_active && !row_deferred && c < chunks)
            *reinterpret_cast<uint4*>(out + o * v.row_bytes + 16 * c) = pack_chunk(acc, v.elem == 1);
        }
      }
    }
  }

  __syncthreads();
  if (tid == 0) {
    s_base[0] = s_n[0] ? atomicAdd(&ws.ctr[0], s_n[0]) : 0;
    s_base[1] = s_n[1] ? atomicAdd(&ws.ctr[1], s_n[1]) : 0;
    if (s_cnt[1]) atomicAdd(&v.counters[ctr_index(kCtrLookups)], static_cast<unsigned long long>(s_cnt[1]));
    if (s_cnt[0]) atomicAdd(&v.counters[ctr_index(kCtrHits)], static_cast<unsigned long long>(s_cnt[0]));
    if (s_cnt[1] - s_cnt[0]) atomicAdd(&v.counters[ctr_index(kCtrMisses)], static_cast<unsigned long long>(s_cnt[1] - s_cnt[0]));
    if (s_cnt[2]) atomicAdd(&v.counters[ctr_index(kCtrInvalid)], static_cast<unsigned long long>(s_cnt[2]));
  }
  __syncthreads();
  for (uint32_t k = tid; k < s_n[0]; k += 256) ws.miss_list[s_base[0] + k] = s_miss[k];
  for (uint32_t k = tid; k < s_n[1]; k += 256) ws.def_list[s_base[1] + k] = s_def[k];
}

// ---------------------------------------------------------------------------------------
// Probe + hit gather, fast path for 32-way sets, one lookup per output row and rows that are
// a multiple of 128 bytes.  Eight lanes serve one lookup: they read the set's 128-byte tag
// line as eight 16-byte words, agree on the way with three cross-lane steps, and copy the
// row with 16-byte lanes, so a wavefront keeps eight independent lookups in flight per
// instruction and nothing is serialised over the lookups of a batch.
// ---------------------------------------------------------------------------------------
constexpr uint32_t kW32Rounds = 2;  // lookups per group of eight lanes (more leaves too few blocks for a Mid-sized batch)
template <int PASSES>  // row_bytes / 128
__global__ __launch_bounds__(256) void emb_probe_gather_w32(EmbView v, MissWs ws, const int64_t* __restrict__ ids,
                                                            uint32_t n, uint8_t* __restrict__ out,
                                                            uint8_t* __restrict__ hit_flags, uint32_t batch) {
  constexpr uint32_t kRounds = kW32Rounds;
  constexpr uint32_t kPerBlock = 32 * kRounds;  // lookups per block: 4 waves x 8 groups x rounds
  __shared__ uint32_t s_miss[kPerBlock];
  __shared__ uint32_t s_n, s_base_m, s_base_d;
  __shared__ uint32_t s_cnt[3];
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, grp = lane >> 3, j = lane & 7;
  if (tid == 0) s_n = 0;
  if (tid < 3) s_cnt[tid] = 0;
  if (blockIdx.x == 0 && tid < 3) ws.ctr_next[tid] = 0;  // the next call's list counters
  __syncthreads();
  const uint4* tags4 = reinterpret_cast<const uint4*>(v.tags);
  // The dependent memory steps (ids -> tag lines -> rows -> output) are each taken for all rounds at once:
  // a wavefront has 8 * kRounds independent lookups in flight per step.
  uint64_t idx[kRounds];
  bool active[kRounds], valid[kRounds];
  int64_t id[kRounds];
  uint32_t set[kRounds], nw[kRounds];
  uint4 tag[kRounds];
#pragma unroll
  for (uint32_t r = 0; r < kRounds; ++r) {
    idx[r] = static_cast<uint64_t>(blockIdx.x) * kPerBlock + (r * 4 + wave) * 8 + grp;
    active[r] = idx[r] < n;
    id[r] = active[r] ? ids[idx[r]] : -1;
  }
#pragma unroll
  for (uint32_t r = 0; r < kRounds; ++r) {
    valid[r] = active[r] && id[r] >= 0 && static_cast<uint64_t>(id[r]) < v.rows;
    set[r] = valid[r] ? set_of(v, id[r]) : 0;
    nw[r] = valid[r] ? ways_of(v, set[r]) : 0;
    tag[r] = make_uint4(0, 0, 0, 0);
    if (4 * j < nw[r]) tag[r] = tags4[static_cast<uint64_t>(set[r]) * 8 + j];
  }
  uint32_t n_hit = 0, n_valid = 0, n_invalid = 0;  // counted by lane 0 of each group
  bool hit[kRounds];
  uint4 row[kRounds][PASSES];
#pragma unroll
  for (uint32_t r = 0; r < kRounds; ++r) {
    const uint32_t id32 = static_cast<uint32_t>(id[r]);
    uint32_t cand = 255;  // lowest matching way seen by this lane
    if (4 * j < nw[r]) {
      const uint4 t = tag[r];
      if (4 * j + 3 < nw[r] && t.w == id32) cand = 4 * j + 3;
      if (4 * j + 2 < nw[r] && t.z == id32) cand = 4 * j + 2;
      if (4 * j + 1 < nw[r] && t.y == id32) cand = 4 * j + 1;
      if (t.x == id32) cand = 4 * j;
    }
#pragma unroll
    for (int o = 4; o > 0; o >>= 1) {
      const uint32_t other = __shfl_xor(cand, o, kWave);
      cand = other < cand ? other : cand;
    }
    hit[r] = valid[r] && cand != 255;
#pragma unroll
    for (int c = 0; c < PASSES; ++c) row[r][c] = make_uint4(0, 0, 0, 0);
    if (hit[r]) {
      const uint8_t* src = v.base + slot_offset(v, set[r], cand);
#pragma unroll
      for (int c = 0; c < PASSES; ++c) row[r][c] = *reinterpret_cast<const uint4*>(src + 16 * (j + 8 * c));
    }
    set[r] = set[r] * 32 + (hit[r] ? cand : 0);  // from here on: the stamp index
  }
#pragma unroll
  for (uint32_t r = 0; r < kRounds; ++r) {
    const bool miss = valid[r] && !hit[r];
    if (j == 0) {
      n_hit += hit[r];
      n_valid += valid[r];
      n_invalid += active[r] && !valid[r];
      if (hit_flags && active[r]) hit_flags[idx[r]] = hit[r] ? 1 : 0;
      if (hit[r]) v.stamps[set[r]] = batch;
    }
    uint8_t* dst = out + idx[r] * v.row_bytes;
    if (hit[r] || (active[r] && !valid[r])) {  // the row, or zeros for an id outside the table
#pragma unroll
      for (int c = 0; c < PASSES; ++c) *reinterpret_cast<uint4*>(dst + 16 * (j + 8 * c)) = row[r][c];
    } else if (miss && j == 0) {
      ws.loc[idx[r]] = -2;  // replaced by the staging row once the miss is resolved
      s_miss[atomicAdd(&s_n, 1u)] = static_cast<uint32_t>(idx[r]);
    }
  }
  if (j == 0) {
    if (n_hit) atomicAdd(&s_cnt[0], n_hit);
    if (n_valid) atomicAdd(&s_cnt[1], n_valid);
    if (n_invalid) atomicAdd(&s_cnt[2], n_invalid);
  }
  __syncthreads();
  if (tid == 0) {
    // with one lookup per row the missing lookups are also the output rows that wait
    s_base_m = s_n ? atomicAdd(&ws.ctr[0], s_n) : 0;
    s_base_d = s_n ? atomicAdd(&ws.ctr[1], s_n) : 0;
    if (s_cnt[1]) atomicAdd(&v.counters[ctr_index(kCtrLookups)], static_cast<unsigned long long>(s_cnt[1]));
    if (s_cnt[0]) atomicAdd(&v.counters[ctr_index(kCtrHits)], static_cast<unsigned long long>(s_cnt[0]));
    if (s_cnt[1] - s_cnt[0]) atomicAdd(&v.counters[ctr_index(kCtrMisses)], static_cast<unsigned long long>(s_cnt[1] - s_cnt[0]));
    if (s_cnt[2]) atomicAdd(&v.counters[ctr_index(kCtrInvalid)], static_cast<unsigned long long>(s_cnt[2]));
  }
  __syncthreads();
  for (uint32_t k = tid; k < s_n; k += 256) {
    ws.miss_list[s_base_m + k] = s_miss[k];
    ws.def_list[s_base_d + k] = s_miss[k];
  }
}

// ---------------------------------------------------------------------------------------
// The same probe for pooled lookups (bag = 2, 4 or 8 consecutive lookups summed into one output
// row): a wavefront's eight lookups are 8 / bag whole bags.  The rows of the hits pass
// through a wave-private LDS tile, from which every lane sums its 4-byte word of an output
// row over the bag's members in order, in fp32, and rounds once (the definition of the pooled
// row).  A bag with a missing member is left to the miss path, as in the generic kernel.
// ---------------------------------------------------------------------------------------
template <int PASSES>  // row_bytes / 128
__global__ __launch_bounds__(256) void emb_probe_gather_w32_bag(EmbView v, MissWs ws, const int64_t* __restrict__ ids,
                                                                uint32_t n, uint32_t bag, uint8_t* __restrict__ out,
                                                                uint8_t* __restrict__ hit_flags, uint32_t batch) {
  constexpr uint32_t kRounds = 4;
  constexpr uint32_t kPerBlock = 32 * kRounds;  // lookups per block: 4 waves x 8 groups x rounds
  constexpr uint32_t kRowWords = PASSES * 32;   // 4-byte words per row
  __shared__ uint32_t s_miss[kPerBlock], s_def[kPerBlock];
  __shared__ uint32_t s_n[2], s_base[2];
  __shared__ uint32_t s_cnt[3];
  __shared__ __attribute__((aligned(16))) uint32_t s_rows[4][8][kRowWords];
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, grp = lane >> 3, j = lane & 7;
  if (tid < 2) s_n[tid] = 0;
  if (tid < 3) s_cnt[tid] = 0;
  if (blockIdx.x == 0 && tid < 3) ws.ctr_next[tid] = 0;  // the next call's list counters
  __syncthreads();
  const uint4* tags4 = reinterpret_cast<const uint4*>(v.tags);
  const bool bf16 = v.elem == 1;
  // The three dependent memory steps (ids -> tag lines -> rows) are taken for all rounds at once, so that a
  // wavefront has 32 independent lookups in flight per step instead of eight.
  uint64_t i0[kRounds];
  bool active[kRounds], valid[kRounds];
  uint32_t id32[kRounds], set[kRounds], nw[kRounds];
  uint4 tag[kRounds];
#pragma unroll
  for (uint32_t r = 0; r < kRounds; ++r) {
    i0[r] = static_cast<uint64_t>(blockIdx.x) * kPerBlock + (r * 4 + wave) * 8;  // n % bag == 0, 8 % bag == 0
    active[r] = i0[r] + grp < n;
  }
  int64_t id[kRounds];
#pragma unroll
  for (uint32_t r = 0; r < kRounds; ++r) id[r] = active[r] ? ids[i0[r] + grp] : -1;
#pragma unroll
  for (uint32_t r = 0; r < kRounds; ++r) {
    valid[r] = active[r] && id[r] >= 0 && static_cast<uint64_t>(id[r]) < v.rows;
    id32[r] = static_cast<uint32_t>(id[r]);
    set[r] = valid[r] ? set_of(v, id[r]) : 0;
    nw[r] = valid[r] ? ways_of(v, set[r]) : 0;
    tag[r] = make_uint4(0, 0, 0, 0);
    if (4 * j < nw[r]) tag[r] = tags4[static_cast<uint64_t>(set[r]) * 8 + j];
  }
  uint32_t n_hit = 0, n_valid = 0, n_invalid = 0;  // counted by lane 0 of each group
  bool hit[kRounds], miss[kRounds];
  int64_t loc[kRounds];
  uint4 row[kRounds][PASSES];
#pragma unroll
  for (uint32_t r = 0; r < kRounds; ++r) {
    uint32_t cand = 255;  // lowest matching way seen by this lane
    if (4 * j < nw[r]) {
      const uint4 t = tag[r];
      if (4 * j + 3 < nw[r] && t.w == id32[r]) cand = 4 * j + 3;
      if (4 * j + 2 < nw[r] && t.z == id32[r]) cand = 4 * j + 2;
      if (4 * j + 1 < nw[r] && t.y == id32[r]) cand = 4 * j + 1;
      if (t.x == id32[r]) cand = 4 * j;
    }
#pragma unroll
    for (int o = 4; o > 0; o >>= 1) {
      const uint32_t other = __shfl_xor(cand, o, kWave);
      cand = other < cand ? other : cand;
    }
    hit[r] = valid[r] && cand != 255;
    miss[r] = valid[r] && !hit[r];
    // the member's row (zeros for an invalid id or a miss)
    loc[r] = miss[r] ? -2 : -1;  // -2: replaced by the staging row once the miss is resolved
#pragma unroll
    for (int c = 0; c < PASSES; ++c) row[r][c] = make_uint4(0, 0, 0, 0);
    if (hit[r]) {
      loc[r] = slot_offset(v, set[r], cand);
      const uint8_t* src = v.base + loc[r];
#pragma unroll
      for (int c = 0; c < PASSES; ++c) row[r][c] = *reinterpret_cast<const uint4*>(src + 16 * (j + 8 * c));
    }
    if (j == 0) {
      n_hit += hit[r];
      n_valid += valid[r];
      n_invalid += active[r] && !valid[r];
    }
    const uint32_t way = hit[r] ? cand : 0;
    set[r] = set[r] * 32 + way;  // from here on: the stamp index
  }
#pragma unroll
  for (uint32_t r = 0; r < kRounds; ++r) {
    const uint64_t i = i0[r] + grp;
    if (j == 0) {
      if (hit[r]) v.stamps[set[r]] = batch;
      if (hit_flags && active[r]) hit_flags[i] = hit[r] ? 1 : 0;
    }
#pragma unroll
    for (int c = 0; c < PASSES; ++c) *reinterpret_cast<uint4*>(&s_rows[wave][grp][4 * (j + 8 * c)]) = row[r][c];
    // a bag with a missing member waits for the miss path, which needs every member's location
    const unsigned long long miss_m = __ballot(miss[r]);  // eight equal bits per group
    const uint32_t bag_first = (grp / bag) * bag;
    const unsigned long long bag_mask = bag == 8 ? ~0ull : (1ull << (8 * bag)) - 1ull;
    const bool deferred = active[r] && ((miss_m >> (8 * bag_first)) & bag_mask) != 0;
    if (j == 0) {
      if (deferred) ws.loc[i] = loc[r];
      if (miss[r]) s_miss[atomicAdd(&s_n[0], 1u)] = static_cast<uint32_t>(i);
      if (deferred && grp == bag_first) s_def[atomicAdd(&s_n[1], 1u)] = static_cast<uint32_t>(i / bag);
    }
    // ordered sums: word w of the wavefront's output rows
    const uint32_t out_words = kRowWords * (8 / bag);
    for (uint32_t w = lane; w < out_words; w += 64) {
      const uint32_t orow = w / kRowWords, word = w % kRowWords, first = orow * bag;
      if (i0[r] + first >= n || ((miss_m >> (8 * first)) & bag_mask) != 0) continue;
      uint32_t res;
      if (bf16) {
        float a0 = 0.0f, a1 = 0.0f;
        for (uint32_t f = 0; f < bag; ++f) {
          const uint32_t x = s_rows[wave][first + f][word];
          const float v0 = bf16_to_f32(x & 0xFFFFu), v1 = bf16_to_f32(x >> 16);
          a0 = f == 0 ? v0 : a0 + v0;
          a1 = f == 0 ? v1 : a1 + v1;
        }
        res = f32_to_bf16(a0) | (f32_to_bf16(a1) << 16);
      } else {
        float a0 = 0.0f;
        for (uint32_t f = 0; f < bag; ++f) {
          const float v0 = __uint_as_float(s_rows[wave][first + f][word]);
          a0 = f == 0 ? v0 : a0 + v0;
        }
        res = __float_as_uint(a0);
      }
      reinterpret_cast<uint32_t*>(out + ((i0[r] + first) / bag) * v.row_bytes)[word] = res;
    }
  }
  if (j == 0) {
    if (n_hit) atomicAdd(&s_cnt[0], n_hit);
    if (n_valid) atomicAdd(&s_cnt[1], n_valid);
    if (n_invalid) atomicAdd(&s_cnt[2], n_invalid);
  }
  __syncthreads();
  if (tid == 0) {
    s_base[0] = s_n[0] ? atomicAdd(&ws.ctr[0], s_n[0]) : 0;
    s_base[1] = s_n[1] ? atomicAdd(&ws.ctr[1], s_n[1]) : 0;
    if (s_cnt[1]) atomicAdd(&v.counters[ctr_index(kCtrLookups)], static_cast<unsigned long long>(s_cnt[1]));
    if (s_cnt[0]) atomicAdd(&v.counters[ctr_index(kCtrHits)], static_cast<unsigned long long>(s_cnt[0]));
    if (s_cnt[1] - s_cnt[0]) atomicAdd(&v.counters[ctr_index(kCtrMisses)], static_cast<unsigned long long>(s_cnt[1] - s_cnt[0]));
    if (s_cnt[2]) atomicAdd(&v.counters[ctr_index(kCtrInvalid)], static_cast<unsigned long long>(s_cnt[2]));
  }
  __syncthreads();
  for (uint32_t k = tid; k < s_n[0]; k += 256) ws.miss_list[s_base[0] + k] = s_miss[k];
  for (uint32_t k = tid; k < s_n[1]; k += 256) ws.def_list[s_base[1] + k] = s_def[k];
}

// ---------------------------------------------------------------------------------------
// Miss path.  All kernels read the list lengths from device memory and return at once
// when the batch had no miss.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t mix32(uint32_t x) {
  x ^= x >> 16; x *= 0x7FEB352Du; x ^= x >> 15; x *= 0x846CA68Bu; x ^= x >> 16;
  return x;
}

// slot of (batch, id) in the dedupe table; inserts when `insert`
__device__ __forceinline__ uint32_t dedupe_slot(const MissWs& ws, uint32_t batch, uint32_t id32, bool insert) {
  const unsigned long long key = (static_cast<unsigned long long>(batch) << 32) | id32;
  uint32_t h = mix32(id32) & ws.hmask;
  for (;;) {
    const unsigned long long k = __atomic_load_n(&ws.hkeys[h], __ATOMIC_RELAXED);
    if (k == key) return h;
    if ((k >> 32) != batch) {  // older batch or never used: free for this batch
      if (!insert) return h;   // cannot happen for ids that were inserted
      const unsigned long long prev = atomicCAS(&ws.hkeys[h], k, key);
      if (prev == k || prev == key) return h;
      continue;  // someone else took the slot: look at it again
    }
    h = (h + 1) & ws.hmask;
  }
}

__global__ __launch_bounds__(256) void miss_dedupe(MissWs ws, const int64_t* __restrict__ ids, uint32_t batch) {
  const uint32_t n_miss = ws.ctr[0];
  for (uint32_t m = blockIdx.x * 256 + threadIdx.x; m < n_miss; m += gridDim.x * 256) {
    const uint32_t i = ws.miss_list[m];
    const uint32_t id32 = static_cast<uint32_t>(ids[i]);
    const uint32_t h = dedupe_slot(ws, batch, id32, true);
    atomicMax(&ws.hvals[h], (static_cast<unsigned long long>(batch) << 32) | (0xFFFFFFFFu - i));
  }
}

__global__ __launch_bounds__(256) void miss_link(EmbView v, MissWs ws, const int64_t* __restrict__ ids,
                                                 uint32_t batch) {
  const uint32_t n_miss = ws.ctr[0];
  for (uint32_t m = blockIdx.x * 256 + threadIdx.x; m < n_miss; m += gridDim.x * 256) {
    const uint32_t i = ws.miss_list[m];
    const int64_t id = ids[i];
    const uint32_t id32 = static_cast<uint32_t>(id);
    const uint32_t h = dedupe_slot(ws, batch, id32, false);
    const uint32_t first_i = 0xFFFFFFFFu - static_cast<uint32_t>(ws.hvals[h]);
    if (first_i != i) continue;  // a later duplicate of this id
    const uint32_t u = atomicAdd(&ws.ctr[2], 1u);
    const uint32_t set = set_of(v, id);
    ws.u_i[u] = i;
    ws.u_id[u] = id32;
    ws.u_set[u] = set;
    ws.hslot_u[h] = u;
    const unsigned long long prev =
        atomicExch(&ws.heads[mix32(set) & ws.headmask], (static_cast<unsigned long long>(batch) << 32) | u);
    ws.u_next[u] = (prev >> 32) == batch ? static_cast<int32_t>(static_cast<uint32_t>(prev)) : -1;
  }
}

// Half a wavefront per unique miss: lane = way.  rank = number of unique misses of the same
// set that occur earlier in the batch; the miss takes the rank-th victim candidate of the
// set in (empty ways by index, then (stamp, way) ascending among stamps older than the batch).
// With `refill` only empty ways are candidates (a refill never evicts) and only insertions are counted.
__global__ __launch_bounds__(256) void miss_decide(EmbView v, MissWs ws, uint32_t batch, bool refill) {
  const uint32_t n_unique = ws.ctr[2];
  const uint32_t lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
  const uint32_t wave = (blockIdx.x * 256 + threadIdx.x) >> 6, n_waves = (gridDim.x * 256) >> 6;
  for (uint32_t u0 = wave * 2; u0 < n_unique; u0 += n_waves * 2) {
    const uint32_t u = u0 + half;
    const bool act = u < n_unique;
    uint32_t set = 0, my_i = 0, rank = 0, nw = 0;
    if (act) {
      set = ws.u_set[u];
      my_i = ws.u_i[u];
      nw = ways_of(v, set);
      const unsigned long long hv = ws.heads[mix32(set) & ws.headmask];
      int32_t cur = (hv >> 32) == batch ? static_cast<int32_t>(static_cast<uint32_t>(hv)) : -1;
      while (cur >= 0) {
        if (ws.u_set[cur] == set && ws.u_i[cur] < my_i) ++rank;
        cur = ws.u_next[cur];
      }
    }
    uint32_t tg = kEmpty, sp = 0;
    const bool way_ok = act && l32 < nw;
    if (way_ok) {
      tg = v.tags[static_cast<uint64_t>(set) * v.w_max + l32];
      sp = v.stamps[static_cast<uint64_t>(set) * v.w_max + l32];
    }
    const bool cand = way_ok && (tg == kEmpty || (!refill && sp < batch));
    const unsigned long long key =
        !cand ? ~0ull : (tg == kEmpty ? l32 : ((1ull << 40) | (static_cast<unsigned long long>(sp) << 5) | l32));
    uint32_t pos = 0;
    for (uint32_t j = 0; j < 32; ++j) {
      const unsigned long long kj = static_cast<unsigned long long>(shfl64(static_cast<int64_t>(key), half * 32 + j));
      pos += (kj < key) ? 1u : 0u;
    }
    const unsigned long long vm = __ballot(cand && pos == rank);
    const uint32_t mine = half ? static_cast<uint32_t>(vm >> 32) : static_cast<uint32_t>(vm);
    const int32_t way = mine ? __ffs(mine) - 1 : -1;
    const uint32_t victim_tag = __shfl(tg, half * 32 + (way >= 0 ? way : 0), kWave);
    if (act && l32 == 0 && refill) {
      ws.u_way[u] = way;
      if (way >= 0) atomicAdd(&v.counters[ctr_index(kCtrInserted)], 1ull);
    } else if (act && l32 == 0) {
      ws.u_way[u] = way;
      atomicAdd(&v.counters[ctr_index(kCtrUnique)], 1ull);
      if (way >= 0) {
        atomicAdd(&v.counters[ctr_index(kCtrInserted)], 1ull);
        if (victim_tag != kEmpty) atomicAdd(&v.counters[ctr_index(kCtrEvicted)], 1ull);
      } else {
        atomicAdd(&v.counters[ctr_index(kCtrBypassed)], 1ull);
      }
    }
  }
}

// every missing lookup, duplicates included, learns the staging row of its id
__global__ __launch_bounds__(256) void miss_resolve(MissWs ws, const int64_t* __restrict__ ids, uint32_t batch) {
  const uint32_t n_miss = ws.ctr[0];
  for (uint32_t m = blockIdx.x * 256 + threadIdx.x; m < n_miss; m += gridDim.x * 256) {
    const uint32_t i = ws.miss_list[m];
    const uint32_t h = dedupe_slot(ws, batch, static_cast<uint32_t>(ids[i]), false);
    ws.loc[i] = -(static_cast<int64_t>(ws.hslot_u[h]) + 3);
  }
}

// Apply the decisions: new tag and stamp, then one read of the row from the pinned host
// table (zero-copy over PCIe) into the staging row and, if inserted, into the pool slot.
// With `refill` nobody waits for the row: it is fetched only if it enters the cache, and not staged.
__global__ __launch_bounds__(256) void miss_apply_fetch(EmbView v, MissWs ws, uint32_t batch, bool refill) {
  const uint32_t n_unique = ws.ctr[2];
  const uint32_t lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
  const uint32_t wave = (blockIdx.x * 256 + threadIdx.x) >> 6, n_waves = (gridDim.x * 256) >> 6;
  const uint32_t chunks = v.row_bytes / 16;
  for (uint32_t u0 = wave * 2; u0 < n_unique; u0 += n_waves * 2) {
    const uint32_t u = u0 + half;
    if (u >= n_unique) continue;
    const uint32_t id32 = ws.u_id[u], set = ws.u_set[u];
    const int32_t way = ws.u_way[u];
    if (refill && way < 0) continue;
    uint8_t* dst = nullptr;
    if (way >= 0) {
      dst = v.base + slot_offset(v, set, static_cast<uint32_t>(way));
      if (l32 == 0) {
        v.tags[static_cast<uint64_t>(set) * v.w_max + way] = id32;
        v.stamps[static_cast<uint64_t>(set) * v.w_max + way] = batch;
      }
    }
    const uint8_t* src = v.table + static_cast<uint64_t>(id32) * v.row_bytes;
    uint32_t src_chunks = chunks;
    if (v.n_tables > 1) {  // the table whose range holds the id; its row may be narrower than a slot
      uint32_t t = 0;
      while (t + 1 < v.n_tables && v.tables[t + 1].base <= id32) ++t;
      src = v.tables[t].ptr + (id32 - v.tables[t].base) * v.tables[t].row_bytes;
      src_chunks = v.tables[t].row_bytes / 16;
    }
    uint8_t* stg = ws.staging + static_cast<uint64_t>(u) * v.row_bytes;
    for (uint32_t c = l32; c < chunks; c += 32) {
      const uint4 val = c < src_chunks ? *reinterpret_cast<const uint4*>(src + 16 * c) : make_uint4(0, 0, 0, 0);
      if (!refill) *reinterpret_cast<uint4*>(stg + 16 * c) = val;
      if (dst) *reinterpret_cast<uint4*>(dst + 16 * c) = val;
    }
  }
}

// Output rows that waited for a miss.
__global__ __launch_bounds__(256) void emb_deferred_gather(EmbView v, MissWs ws, uint32_t bag,
                                                           uint8_t* __restrict__ out) {
  const uint32_t n_def = ws.ctr[1];
  const uint32_t chunks = v.row_bytes / 16;
  const uint32_t lpr = lanes_per_row(chunks);
  const uint32_t gid = blockIdx.x * 256 + threadIdx.x;
  const uint32_t sub = gid % lpr;
  const uint32_t groups = gridDim.x * 256 / lpr;
  for (uint32_t k = gid / lpr; k < n_def; k += groups) {
    const uint64_t o = ws.def_list[k];
    emit_row(v, ws, bag, lpr, sub, out + o * v.row_bytes,
             [&](uint32_t f) { return ws.loc[o * bag + f]; });
  }
}

// ---------------------------------------------------------------------------------------
// Refill of empty ways (paper Sec. IV-B: new EMB capacity is filled with hot rows in the
// background).  The probe only finds out which ids are not resident: half a wavefront per id,
// lane = way, one coalesced read of the set's tag line; nothing is stamped and nothing is
// written out.  The ids that are not resident then take the miss path with `refill` set.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void emb_refill_probe(EmbView v, MissWs ws, const int64_t* __restrict__ ids, uint32_t n) {
  const uint32_t lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
  const uint32_t wave = (blockIdx.x * 256 + threadIdx.x) >> 6, n_waves = (gridDim.x * 256) >> 6;
  if (blockIdx.x == 0 && threadIdx.x < 3) ws.ctr_next[threadIdx.x] = 0;  // the next call's list counters
  for (uint32_t i0 = wave * 2; i0 < n; i0 += n_waves * 2) {
    const uint32_t i = i0 + half;
    const int64_t id = i < n ? ids[i] : -1;
    const bool valid = id >= 0 && static_cast<uint64_t>(id) < v.rows;
    bool match = false;
    if (valid) {
      const uint32_t set = set_of(v, id);
      if (l32 < ways_of(v, set)) match = v.tags[static_cast<uint64_t>(set) * v.w_max + l32] == static_cast<uint32_t>(id);
    }
    const unsigned long long m = __ballot(match);
    const bool resident = (half ? static_cast<uint32_t>(m >> 32) : static_cast<uint32_t>(m)) != 0;
    if (l32 == 0 && valid && !resident) ws.miss_list[atomicAdd(&ws.ctr[0], 1u)] = i;
  }
}

// ---------------------------------------------------------------------------------------
// Split shrink: per set, evict down to the new way count (empties first, then least
// (stamp, way)), move survivors of the removed ways into the vacated lower ways.
// Half a wavefront per set, lane = way.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void emb_shrink_sets(EmbView v, uint32_t old_full, uint32_t old_part_sets) {
  const uint32_t lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
  const uint32_t wave = (blockIdx.x * 256 + threadIdx.x) >> 6, n_waves = (gridDim.x * 256) >> 6;
  const uint32_t chunks = v.row_bytes / 16;
  for (uint32_t s0 = wave * 2; s0 < v.sets; s0 += n_waves * 2) {
    const uint32_t s = s0 + half;
    const bool act = s < v.sets;
    const uint32_t a = act ? old_full + (s < old_part_sets ? 1u : 0u) : 0;
    const uint32_t b = act ? ways_of(v, s) : 0;
    const bool shrinks = b < a;
    // A set whose removed ways hold nothing keeps all its entries where they are: most sets of a cache that is
    // not full.  Only the removed ways' tags are read to find that out (a few bytes of the set's tag line).
    uint32_t tg = kEmpty, sp = 0;
    if (shrinks && l32 >= b && l32 < a) tg = v.tags[static_cast<uint64_t>(s) * v.w_max + l32];
    if (__ballot(tg != kEmpty) == 0) continue;
    if (shrinks && l32 < a) {
      if (l32 < b) tg = v.tags[static_cast<uint64_t>(s) * v.w_max + l32];
      sp = v.stamps[static_cast<uint64_t>(s) * v.w_max + l32];
    }
    const bool live = tg != kEmpty;
    const unsigned long long live_all = __ballot(live);
    const uint32_t live_m = half ? static_cast<uint32_t>(live_all >> 32) : static_cast<uint32_t>(live_all);
    const uint32_t n_live = __popc(live_m);
    const uint32_t n_evict = n_live > b ? n_live - b : 0;
    // rank among live entries by (stamp, way) ascending
    const unsigned long long key = live ? ((static_cast<unsigned long long>(sp) << 5) | l32) : ~0ull;
    uint32_t rank = 0;
    for (uint32_t j = 0; j < 32; ++j) {
      const unsigned long long kj = static_cast<unsigned long long>(shfl64(static_cast<int64_t>(key), half * 32 + j));
      rank += (kj < key) ? 1u : 0u;
    }
    const bool evicted = live && rank < n_evict;
    const bool survivor = live && !evicted;
    const bool mover = survivor && l32 >= b;
    const bool hole = shrinks && l32 < b && !survivor;
    const unsigned long long mover_all = __ballot(mover), hole_all = __ballot(hole);
    const uint32_t mover_m = half ? static_cast<uint32_t>(mover_all >> 32) : static_cast<uint32_t>(mover_all);
    const uint32_t hole_m = half ? static_cast<uint32_t>(hole_all >> 32) : static_cast<uint32_t>(hole_all);
    const uint32_t lt = (1u << l32) - 1u;
    // the k-th hole receives the k-th mover
    int src_way = -1;
    if (hole) {
      const uint32_t k = __popc(hole_m & lt);
      uint32_t mm = mover_m;
      for (uint32_t q = 0; q < k && mm; ++q) mm &= mm - 1;
      if (mm) src_way = __ffs(mm) - 1;
    }
    const uint32_t in_tag = __shfl(tg, half * 32 + (src_way >= 0 ? src_way : 0), kWave);
    const uint32_t in_stamp = __shfl(sp, half * 32 + (src_way >= 0 ? src_way : 0), kWave);
    if (shrinks && l32 < a) {
      uint32_t new_tag = kEmpty, new_stamp = 0;
      if (l32 < b) {
        if (survivor) { new_tag = tg; new_stamp = sp; }
        else if (src_way >= 0) { new_tag = in_tag; new_stamp = in_stamp; }
      }
      if (new_tag != tg || new_stamp != sp) {
        v.tags[static_cast<uint64_t>(s) * v.w_max + l32] = new_tag;
        v.stamps[static_cast<uint64_t>(s) * v.w_max + l32] = new_stamp;
      }
    }
    const unsigned long long ev_all = __ballot(evicted);
    const uint32_t ev_m = half ? static_cast<uint32_t>(ev_all >> 32) : static_cast<uint32_t>(ev_all);
    if (act && l32 == 0) {
      if (ev_m) atomicAdd(&v.counters[ctr_index(kCtrShrinkEvicted)], static_cast<unsigned long long>(__popc(ev_m)));
      if (mover_m) atomicAdd(&v.counters[ctr_index(kCtrShrinkMoved)], static_cast<unsigned long long>(__popc(mover_m)));
    }
    // row moves: destination ways are below every source way, and a destination is never
    // a later mover's source, so moving in ascending order is safe
    uint32_t mm = mover_m, hm = hole_m;
    while (mm) {
      const uint32_t from = __ffs(mm) - 1, to = __ffs(hm) - 1;
      mm &= mm - 1;
      hm &= hm - 1;
      // old geometry for the source: the page of a removed way is still mapped in emb_pages
      const uint8_t* src = v.base + slot_offset(v, s, from);
      uint8_t* dst = v.base + slot_offset(v, s, to);
      for (uint32_t c = l32; c < chunks; c += 32)
        *reinterpret_cast<uint4*>(dst + 16 * c) = *reinterpret_cast<const uint4*>(src + 16 * c);
    }
  }
}

// (table, row) pairs -> global ids of the rows; -1 where the table or the row does not exist
__global__ void emb_global_ids(EmbView v, const uint32_t* __restrict__ table_of, const int64_t* __restrict__ ids,
                               uint32_t n, int64_t* __restrict__ gids) {
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
    const uint32_t t = table_of[i];
    const int64_t id = ids[i];
    int64_t gid = -1;
    if (t < v.n_tables && id >= 0 && static_cast<uint64_t>(id) < v.tables[t].rows)
      gid = static_cast<int64_t>(v.tables[t].base) + id;
    gids[i] = gid;
  }
}

// Measurement aid: what the memory system gives a gather.  Groups of LPR lanes read rows of LPR * 16 bytes picked by
// a counter-based hash out of [base, base + n_rows rows), ROUNDS rows in flight per group, and (optionally) write
// them out back to back.  No cache helps when the region is much larger than the caches.
__device__ __forceinline__ uint64_t splitmix(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
template <int LPR, int ROUNDS>
__global__ __launch_bounds__(256) void random_row_reads(const uint4* __restrict__ base, uint64_t n_rows, uint64_t n_reads,
                                                        uint4* __restrict__ out, uint64_t seed) {
  const uint64_t gid = (blockIdx.x * 256ull + threadIdx.x) / LPR, sub = threadIdx.x % LPR;
  const uint64_t n_groups = gridDim.x * 256ull / LPR;
  uint4 acc = make_uint4(0, 0, 0, 0);
  for (uint64_t i = gid * ROUNDS; i + ROUNDS <= n_reads; i += n_groups * ROUNDS) {
    uint4 v[ROUNDS];
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) v[r] = base[(splitmix(seed + i + r) % n_rows) * LPR + sub];
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
      if (out) out[(i + r) * LPR + sub] = v[r];
      acc.x ^= v[r].x; acc.y ^= v[r].y; acc.z ^= v[r].z; acc.w ^= v[r].w;
    }
  }
  if (!out && acc.x == 0x12345678u && acc.y == 0x9ABCDEF0u && acc.z == 1u) const_cast<uint4*>(base)[0] = acc;  // keeps the loads alive
}

__global__ void fill_u32_kernel(uint32_t* p, uint64_t n, uint32_t value) {
  for (uint64_t k = blockIdx.x * static_cast<uint64_t>(blockDim.x) + threadIdx.x; k < n;
       k += static_cast<uint64_t>(gridDim.x) * blockDim.x)
    p[k] = value;
}

}  // namespace

hipError_t launch_random_row_reads(const void* base, uint64_t n_rows, uint32_t row_bytes, uint64_t n_reads, void* out,
                                   uint64_t seed, hipStream_t stream) {
  const dim3 grid(256 * 8), block(256);
  const uint4* b = static_cast<const uint4*>(base);
  uint4* o = static_cast<uint4*>(out);
  switch (row_bytes) {
    case 128: hipLaunchKernelGGL((random_row_reads<8, 4>), grid, block, 0, stream, b, n_rows, n_reads, o, seed); break;
    case 256: hipLaunchKernelGGL((random_row_reads<16, 4>), grid, block, 0, stream, b, n_rows, n_reads, o, seed); break;
    case 512: hipLaunchKernelGGL((random_row_reads<32, 4>), grid, block, 0, stream, b, n_rows, n_reads, o, seed); break;
    case 1024: hipLaunchKernelGGL((random_row_reads<64, 2>), grid, block, 0, stream, b, n_rows, n_reads, o, seed); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_fill_u32(uint32_t* p, uint64_t n, uint32_t value, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  const uint32_t blocks = static_cast<uint32_t>(n / 256 + 1 < 4096 ? n / 256 + 1 : 4096);
  hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks), dim3(256), 0, stream, p, n, value);
  return hipGetLastError();
}

hipError_t launch_emb_probe(const EmbView& v, const MissWs& ws, const int64_t* ids, uint32_t n, uint32_t bag,
                            uint8_t* out, uint8_t* hit_flags, uint32_t batch, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  if (bag == 1 && v.w_max == 32 && v.row_bytes % 128 == 0 && v.row_bytes <= 1024) {
    const uint32_t per_block = 32 * kW32Rounds;
    const dim3 grid((n + per_block - 1) / per_block), block(256);
    switch (v.row_bytes / 128) {
#define RACER_W32_CASE(P) \
  case P: hipLaunchKernelGGL(emb_probe_gather_w32<P>, grid, block, 0, stream, v, ws, ids, n, out, hit_flags, batch); break;
      RACER_W32_CASE(1) RACER_W32_CASE(2) RACER_W32_CASE(3) RACER_W32_CASE(4)
      RACER_W32_CASE(5) RACER_W32_CASE(6) RACER_W32_CASE(7) RACER_W32_CASE(8)
#undef RACER_W32_CASE
    }
    return hipGetLastError();
  }
  if ((bag == 2 || bag == 4 || bag == 8) && v.w_max == 32 && v.row_bytes % 128 == 0 && v.row_bytes <= 512) {
    const dim3 grid((n + 127) / 128), block(256);  // 128 lookups per block
    switch (v.row_bytes / 128) {
#define RACER_W32_BAG_CASE(P) \
  case P: hipLaunchKernelGGL(emb_probe_gather_w32_bag<P>, grid, block, 0, stream, v, ws, ids, n, bag, out, hit_flags, batch); break;
      RACER_W32_BAG_CASE(1) RACER_W32_BAG_CASE(2) RACER_W32_BAG_CASE(3) RACER_W32_BAG_CASE(4)
#undef RACER_W32_BAG_CASE
    }
    return hipGetLastError();
  }
  const uint32_t lb = (64 / bag) * bag;
  const uint32_t per_block = 4 * lb;
  const uint32_t blocks = (n + per_block - 1) / per_block;
  hipLaunchKernelGGL(emb_probe_gather, dim3(blocks), dim3(256), 0, stream, v, ws, ids, n, bag, lb, out, hit_flags, batch);
  return hipGetLastError();
}

hipError_t launch_emb_miss_path(const EmbView& v, const MissWs& ws, const int64_t* ids, uint32_t n, uint32_t bag,
                                uint8_t* out, uint32_t batch, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  // the miss kernels size themselves from device counters; a modest grid keeps the
  // no-miss case cheap and still saturates PCIe when a cold batch arrives
  const uint32_t mblocks = n / 256 + 1 < 1024 ? n / 256 + 1 : 1024;
  hipLaunchKernelGGL(miss_dedupe, dim3(mblocks), dim3(256), 0, stream, ws, ids, batch);
  hipLaunchKernelGGL(miss_link, dim3(mblocks), dim3(256), 0, stream, v, ws, ids, batch);
  hipLaunchKernelGGL(miss_decide, dim3(mblocks), dim3(256), 0, stream, v, ws, batch, false);
  hipLaunchKernelGGL(miss_resolve, dim3(mblocks), dim3(256), 0, stream, ws, ids, batch);
  hipLaunchKernelGGL(miss_apply_fetch, dim3(mblocks), dim3(256), 0, stream, v, ws, batch, false);
  hipLaunchKernelGGL(emb_deferred_gather, dim3(mblocks), dim3(256), 0, stream, v, ws, bag, out);
  return hipGetLastError();
}

hipError_t launch_emb_global_ids(const EmbView& v, const uint32_t* table_of, const int64_t* ids, uint32_t n, int64_t* gids,
                                 hipStream_t stream) {
  if (n == 0) return hipSuccess;
  const uint32_t blocks = n / 256 + 1 < 2048 ? n / 256 + 1 : 2048;
  hipLaunchKernelGGL(emb_global_ids, dim3(blocks), dim3(256), 0, stream, v, table_of, ids, n, gids);
  return hipGetLastError();
}

hipError_t launch_emb_refill(const EmbView& v, const MissWs& ws, const int64_t* ids, uint32_t n, uint32_t batch,
                             hipStream_t stream) {
  if (n == 0) return hipSuccess;
  const uint32_t pblocks = n / 8 + 1 < 2048 ? n / 8 + 1 : 2048;  // two ids per wavefront and pass
  const uint32_t mblocks = n / 256 + 1 < 1024 ? n / 256 + 1 : 1024;
  hipLaunchKernelGGL(emb_refill_probe, dim3(pblocks), dim3(256), 0, stream, v, ws, ids, n);
  hipLaunchKernelGGL(miss_dedupe, dim3(mblocks), dim3(256), 0, stream, ws, ids, batch);
  hipLaunchKernelGGL(miss_link, dim3(mblocks), dim3(256), 0, stream, v, ws, ids, batch);
  hipLaunchKernelGGL(miss_decide, dim3(mblocks), dim3(256), 0, stream, v, ws, batch, true);
  hipLaunchKernelGGL(miss_apply_fetch, dim3(mblocks), dim3(256), 0, stream, v, ws, batch, true);
  return hipGetLastError();
}

hipError_t launch_emb_shrink(const EmbView& v, uint32_t old_full, uint32_t old_part_sets, hipStream_t stream) {
  // one pass over the sets with as many blocks as that takes: each set costs one dependent round trip to
  // memory, so the latency is hidden by the number of wavefronts in flight, not by a loop
  const uint32_t waves_needed = (v.sets + 1) / 2;
  uint32_t blocks = (waves_needed + 3) / 4;
  if (blocks > (1u << 20)) blocks = 1u << 20;
  if (blocks == 0) blocks = 1;
  hipLaunchKernelGGL(emb_shrink_sets, dim3(blocks), dim3(256), 0, stream, v, old_full, old_part_sets);
  return hipGetLastError();
}

}  // namespace racer
