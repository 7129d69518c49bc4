// HSTU layer kernels for gfx950 (paper Sec. II-A/II-B "Compute" stage; the layer equations
// are the published HSTU form):
//   Xn = LayerNorm(X);  [U|V|Q|K] = SiLU(Xn W1 + b1);  K,V of the new tokens -> KV pages
//   O_i = (1/n) sum_{j<=p_i} SiLU(q_i.k_j + pos[min(p_i-j, n_pos-1)] + time[bucket(ts_p-ts_j)]) v_j
//   Y = X + (LayerNorm(O) * U) W2 + b2
// bf16 models run on MFMA with fp32 accumulation; the small fp32 configuration uses plain FMA kernels.
// What a bf16 model stores where a caller can see it (inputs, weights, K and V in the pages, outputs) is bf16.
// The library's own intermediate matrices (the normalised activations, U, the attention output O, the gated
// activations) and its transposed copies of the weights are IEEE half precision: eleven significant bits
// instead of eight at the same size and the same MFMA rate (v_mfma_f32_32x32x16_f16), which halves the
// distance to the fp64 oracle; a bf16 weight converts exactly.  Values of these matrices must stay below
// 65504 in magnitude, which LayerNorm and the 1/n scaling ensure for any sane model.  The two attention
// products take bf16 operands (Q, and K, V as the pages hold them).
//
// KV page layout (one page = page_tokens tokens of every layer):
//   [layer][K|V][head] blocks of page_tokens*d_h elements;
//   a K block is [token][d_h]; a V block is stored transposed, [d_h][token], so that the
//   second product's matrix operand (contraction over keys) is read key-contiguous.
#include "kernels.h"

namespace racer {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct bf16_t { uint16_t bits; };
struct half_t { uint16_t bits; };  // IEEE binary16 (the library's own intermediates)
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf2f(uint16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }
__device__ __forceinline__ uint16_t f2bf(float f) {
  const uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return static_cast<uint16_t>((u >> 16) | 0x40);
  return static_cast<uint16_t>((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ uint16_t f2h(float f) { return __builtin_bit_cast(uint16_t, static_cast<_Float16>(f)); }  // nearest even
__device__ __forceinline__ float load_elem(const float* p, uint64_t i) { return p[i]; }
__device__ __forceinline__ float load_elem(const bf16_t* p, uint64_t i) { return bf2f(p[i].bits); }
__device__ __forceinline__ void store_elem(float* p, uint64_t i, float v) { p[i] = v; }
__device__ __forceinline__ void store_elem(bf16_t* p, uint64_t i, float v) { p[i].bits = f2bf(v); }

__device__ __forceinline__ float silu(float x) { return x / (1.0f + __expf(-x)); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__device__ __forceinline__ uint32_t time_bucket(long long dt, uint32_t n_time) {
  const unsigned long long v = dt > 1 ? static_cast<unsigned long long>(dt) : 1ull;
  const uint32_t b = 63u - static_cast<uint32_t>(__clzll(static_cast<long long>(v)));
  return b < n_time - 1 ? b : n_time - 1;
}

// byte offset of the K (kv = 0) or V (kv = 1) block of (layer, head) inside a page
__device__ __forceinline__ uint64_t kv_block_offset(const HstuDims& hd, uint32_t layer, uint32_t kv, uint32_t head,
                                                    uint32_t esize) {
  return ((static_cast<uint64_t>(layer) * 2 + kv) * hd.H + head) * hd.pt * hd.dh * esize;
}

// page index and offset inside the page of token j (page_tokens is usually a power of two)
__device__ __forceinline__ void split_token(const HstuDims& hd, uint32_t j, uint32_t* page_idx, uint32_t* in_page) {
  if (hd.pt_shift < 32) {
    *page_idx = j >> hd.pt_shift;
    *in_page = j & (hd.pt - 1);
  } else {
    *page_idx = j / hd.pt;
    *in_page = j % hd.pt;
  }
}

// ---------------------------------------------------------------------------------------
// LayerNorm over d (optionally times a gate row), two-pass in fp32.  A row is owned by LPR
// consecutive lanes of a wavefront (64 / LPR rows per wavefront, LPR chosen so that every
// lane has work); a lane holds KC chunks of 8 consecutive elements (16-byte accesses for
// bf16), d <= 1024.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void load8(const float* p, float v[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16_t* p, float v[8]) {
  const uint4 a = *reinterpret_cast<const uint4*>(p);
  const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    v[2 * k] = __uint_as_float(w[k] << 16);
    v[2 * k + 1] = __uint_as_float(w[k] & 0xFFFF0000u);
  }
}
__device__ __forceinline__ void load8(const half_t* p, float v[8]) {
  const uint4 a = *reinterpret_cast<const uint4*>(p);
  const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const f16x2 h = __builtin_bit_cast(f16x2, w[k]);
    v[2 * k] = static_cast<float>(h[0]);
    v[2 * k + 1] = static_cast<float>(h[1]);
  }
}
__device__ __forceinline__ uint32_t pack2_f16(float lo, float hi) {
  typedef float v2f __attribute__((ext_vector_type(2)));
  const v2f v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
}
__device__ __forceinline__ void store8(half_t* p, const float v[8]) {
  *reinterpret_cast<uint4*>(p) = make_uint4(pack2_f16(v[0], v[1]), pack2_f16(v[2], v[3]), pack2_f16(v[4], v[5]), pack2_f16(v[6], v[7]));
}
__device__ __forceinline__ void store8(float* p, const float v[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
template <int LPR>
__device__ __forceinline__ float group_sum(float v) {  // sum over the LPR lanes that share a row
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

template <typename TX, typename TY, int LPR, int KC>  // TX: input rows; TY: gate rows and output rows
__global__ __launch_bounds__(256) void layernorm_rows(const TX* __restrict__ x, const float* __restrict__ g,
                                                      const float* __restrict__ b, const TY* __restrict__ gate,
                                                      TY* __restrict__ y, uint32_t N, uint32_t d, float eps) {
  const uint32_t sub = threadIdx.x % LPR;
  const uint32_t row = blockIdx.x * (256 / LPR) + threadIdx.x / LPR;
  const bool row_ok = row < N;  // lanes of a missing row still take part in the shuffles
  const uint32_t chunks = d / 8;
  const uint64_t base = static_cast<uint64_t>(row_ok ? row : 0) * d;
  float v[KC][8], gt[KC][8];
#pragma unroll
  for (int k = 0; k < KC; ++k) {
    const uint32_t c = sub + LPR * k;
    const bool on = row_ok && c < chunks;
    if (on) load8(x + base + 8 * c, v[k]);
    if (on && gate) load8(gate + base + 8 * c, gt[k]);
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (!on) v[k][e] = 0.0f;
  }
  float s = 0.0f;
#pragma unroll
  for (int k = 0; k < KC; ++k)
#pragma unroll
    for (int e = 0; e < 8; ++e) s += v[k][e];
  const float mean = group_sum<LPR>(s) / d;
  float q = 0.0f;
#pragma unroll
  for (int k = 0; k < KC; ++k)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float dv = (sub + LPR * k < chunks) ? v[k][e] - mean : 0.0f;
      q += dv * dv;
    }
  const float rstd = 1.0f / sqrtf(group_sum<LPR>(q) / d + eps);
#pragma unroll
  for (int k = 0; k < KC; ++k) {
    const uint32_t c = sub + LPR * k;
    if (!row_ok || c >= chunks) continue;
    float gg[8], bb[8], o[8];
    load8(g + 8 * c, gg);
    load8(b + 8 * c, bb);
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (v[k][e] - mean) * rstd * gg[e] + bb[e];
    if (gate) {
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] *= gt[k][e];
    }
    store8(y + base + 8 * c, o);
  }
}

// ---------------------------------------------------------------------------------------
// Epilogues
// ---------------------------------------------------------------------------------------
template <typename T>
struct FrontEpilogue {  // SiLU(acc + b1), split U | V | Q | K, K and V into the pages
  HstuDims hd;
  uint32_t layer;
  const float* b1;
  T* u;
  T* q;
  KvView kv;
  const ReqDev* reqs;
  const uint32_t* row_req;
  const int32_t* page_tables;

  __device__ __forceinline__ void operator()(uint32_t row, uint32_t col, float acc) const {
    const float z = silu(acc + b1[col]);
    const uint32_t which = col / hd.d, c = col % hd.d;
    if (which == 0) { store_elem(u, static_cast<uint64_t>(row) * hd.d + c, z); return; }
    if (which == 2) {  // bf16 models: the attention kernel wants q * log2(e) (one rounding, here)
      store_elem(q, static_cast<uint64_t>(row) * hd.d + c, sizeof(T) == 2 ? z * 1.4426950408889634f : z);
      return;
    }
    const ReqDev rq = reqs[row_req[row]];
    const uint32_t pos = rq.prefix_len + (row - rq.x_off);
    const int32_t page = page_tables[rq.page_table_off + pos / hd.pt];
    if (page < 0 || static_cast<uint32_t>(page) >= kv.n_pages) {
      atomicAdd(&kv.counters[ctr_index(kCtrBadPages)], 1ull);
      return;
    }
    const uint32_t head = c / hd.dh, cc = c % hd.dh, tok = pos % hd.pt;
    T* blk = reinterpret_cast<T*>(kv.base + static_cast<uint64_t>(page) * kv.page_size +
                                  kv_block_offset(hd, layer, which == 1 ? 1 : 0, head, sizeof(T)));
    if (which == 3) store_elem(blk, static_cast<uint64_t>(tok) * hd.dh + cc, z);   // K: [token][d_h]
    else store_elem(blk, static_cast<uint64_t>(cc) * hd.pt + tok, z);              // V: [d_h][token]
  }
};

template <typename T>
struct BackEpilogue {  // y = x + acc + b2
  uint32_t d;
  const float* b2;
  const T* x;
  T* y;
  __device__ __forceinline__ void operator()(uint32_t row, uint32_t col, float acc) const {
    const uint64_t i = static_cast<uint64_t>(row) * d + col;
    store_elem(y, i, load_elem(x, i) + acc + b2[col]);
  }
};

// ---------------------------------------------------------------------------------------
// Half-precision GEMM on MFMA (both operands are the library's own: a normalised activation matrix and a
// transposed weight copy): C[M][Nout] = A[M][K] * Bt[Nout][K]^T, block tile 128 x 64, four
// wavefronts of 32 rows x 64 columns each, K staged through LDS 64 at a time.
// Operand layout of v_mfma_f32_32x32x16_f16 / _bf16: lane (g = lane/32, i = lane%32) supplies row
// (A) or column (B) i with eight consecutive k of its half g; the result lane holds column
// i and rows 8*(r/4) + 4*g + r%4 for r = 0..15.
// ---------------------------------------------------------------------------------------
constexpr int kLdsPad = 8;

template <typename Epi>
__global__ __launch_bounds__(256) void gemm_bf16_mfma(const uint16_t* __restrict__ A, const uint16_t* __restrict__ Bt,
                                                      uint32_t M, uint32_t K, Epi epi) {
  __shared__ __attribute__((aligned(16))) uint16_t As[128][64 + kLdsPad];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[64][64 + kLdsPad];
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, li = lane & 31;
  const uint32_t m0 = blockIdx.x * 128, n0 = blockIdx.y * 64;
  f32x16 acc[2];
#pragma unroll
  for (int cb = 0; cb < 2; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[cb][r] = 0.0f;

  for (uint32_t k0 = 0; k0 < K; k0 += 64) {
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const uint32_t c = tid + 256 * it, row = c >> 3, part = c & 7;
      uint4 val = make_uint4(0, 0, 0, 0);
      if (m0 + row < M) val = *reinterpret_cast<const uint4*>(A + static_cast<uint64_t>(m0 + row) * K + k0 + part * 8);
      *reinterpret_cast<uint4*>(&As[row][part * 8]) = val;
    }
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const uint32_t c = tid + 256 * it, row = c >> 3, part = c & 7;
      *reinterpret_cast<uint4*>(&Bs[row][part * 8]) =
          *reinterpret_cast<const uint4*>(Bt + static_cast<uint64_t>(n0 + row) * K + k0 + part * 8);
    }
    __syncthreads();
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      const f16x8 a = __builtin_bit_cast(f16x8, *reinterpret_cast<const uint4*>(&As[32 * wave + li][16 * st + 8 * g]));
#pragma unroll
      for (int cb = 0; cb < 2; ++cb) {
        const f16x8 b = __builtin_bit_cast(f16x8, *reinterpret_cast<const uint4*>(&Bs[32 * cb + li][16 * st + 8 * g]));
        acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[cb], 0, 0, 0);
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int cb = 0; cb < 2; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const uint32_t row = m0 + 32 * wave + 8 * (r / 4) + 4 * g + (r % 4);
      if (row < M) epi(row, n0 + 32 * cb + li, acc[cb][r]);
    }
}

// ---------------------------------------------------------------------------------------
// Pointwise projection of bf16 models: [U|V|Q|K] = SiLU(Xn W1 + b1) on MFMA, one block per
// (row tile, 64 output columns).  Row tiles never cross a request (host-built list), and 64
// columns are exactly one head's slice of U, V, Q or K, so a block has one destination:
// the results go through LDS and leave as 16-byte stores - rows of U/Q, token rows of the K
// block, and key-contiguous runs of the transposed V block.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gemm_front_bf16(HstuDims hd, uint32_t layer, const uint16_t* __restrict__ A,
                                                       const uint16_t* __restrict__ Bt, const float* __restrict__ b1,
                                                       uint16_t* __restrict__ u, uint16_t* __restrict__ q, KvView kv,
                                                       const ReqDev* __restrict__ reqs,
                                                       const RowTile* __restrict__ row_tiles,
                                                       const int32_t* __restrict__ page_tables) {
  __shared__ __attribute__((aligned(16))) uint16_t As[128][64 + kLdsPad];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[64][64 + kLdsPad];
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, li = lane & 31;
  const RowTile rt = row_tiles[blockIdx.x];
  const uint32_t m0 = rt.row0, rows = rt.rows, n0 = blockIdx.y * 64, K = hd.d;
  f32x16 acc[2];
#pragma unroll
  for (int cb = 0; cb < 2; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[cb][r] = 0.0f;
  for (uint32_t k0 = 0; k0 < K; k0 += 64) {
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const uint32_t c = tid + 256 * it, row = c >> 3, part = c & 7;
      uint4 val = make_uint4(0, 0, 0, 0);
      if (row < rows) val = *reinterpret_cast<const uint4*>(A + static_cast<uint64_t>(m0 + row) * K + k0 + part * 8);
      *reinterpret_cast<uint4*>(&As[row][part * 8]) = val;
    }
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const uint32_t c = tid + 256 * it, row = c >> 3, part = c & 7;
      *reinterpret_cast<uint4*>(&Bs[row][part * 8]) =
          *reinterpret_cast<const uint4*>(Bt + static_cast<uint64_t>(n0 + row) * K + k0 + part * 8);
    }
    __syncthreads();
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      const f16x8 a = __builtin_bit_cast(f16x8, *reinterpret_cast<const uint4*>(&As[32 * wave + li][16 * st + 8 * g]));
#pragma unroll
      for (int cb = 0; cb < 2; ++cb) {
        const f16x8 b = __builtin_bit_cast(f16x8, *reinterpret_cast<const uint4*>(&Bs[32 * cb + li][16 * st + 8 * g]));
        acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[cb], 0, 0, 0);
      }
    }
    __syncthreads();
  }
  // ---- epilogue: bias + SiLU (+ log2 e for Q) -> bf16 tile in LDS (reusing As) ----
  const uint32_t which = n0 / hd.d, head = (n0 % hd.d) / 64;  // 0 U, 1 V, 2 Q, 3 K
  const float qscale = which == 2 ? 1.4426950408889634f : 1.0f;
#pragma unroll
  for (int cb = 0; cb < 2; ++cb) {
    const float bias = b1[n0 + 32 * cb + li];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const uint32_t row = 32 * wave + 8 * (r / 4) + 4 * g + (r % 4);
      const float z = silu(acc[cb][r] + bias) * qscale;
      As[row][32 * cb + li] = which == 0 ? f2h(z) : f2bf(z);  // U is the library's own (half precision); Q, K, V are bf16
    }
  }
  __syncthreads();
  if (which == 0 || which == 2) {
    uint16_t* dst = which == 0 ? u : q;
    for (uint32_t idx = tid; idx < 128 * 8; idx += 256) {
      const uint32_t row = idx >> 3, part = idx & 7;
      if (row < rows)
        *reinterpret_cast<uint4*>(dst + static_cast<uint64_t>(m0 + row) * hd.d + head * 64 + part * 8) =
            *reinterpret_cast<const uint4*>(&As[row][part * 8]);
    }
    return;
  }
  const ReqDev rq = reqs[rt.req];
  const uint32_t pos0 = rq.prefix_len + (m0 - rq.x_off);  // sequence position of the tile's first row
  if (which == 3) {  // K block: [token][d_h], one 128-byte row per token
    const uint64_t koff = kv_block_offset(hd, layer, 0, head, 2);
    for (uint32_t idx = tid; idx < 128 * 8; idx += 256) {
      const uint32_t row = idx >> 3, part = idx & 7;
      if (row >= rows) continue;
      uint32_t pi, ip;
      split_token(hd, pos0 + row, &pi, &ip);
      const int32_t page = page_tables[rq.page_table_off + pi];
      if (page < 0 || static_cast<uint32_t>(page) >= kv.n_pages) {
        if (part == 0) atomicAdd(&kv.counters[ctr_index(kCtrBadPages)], 1ull);
        continue;
      }
      *reinterpret_cast<uint4*>(kv.base + static_cast<uint64_t>(page) * kv.page_size + koff + (static_cast<uint64_t>(ip) * 64 + part * 8) * 2) =
          *reinterpret_cast<const uint4*>(&As[row][part * 8]);
    }
    return;
  }
  // V block, stored transposed [d_h][token]: a thread takes one d_h row and 8 consecutive tokens
  const uint64_t voff = kv_block_offset(hd, layer, 1, head, 2);
  for (uint32_t idx = tid; idx < 64 * 16; idx += 256) {
    const uint32_t dh = idx >> 4, t0 = (idx & 15) * 8;
    if (t0 >= rows) continue;
    uint32_t pi, ip;
    split_token(hd, pos0 + t0, &pi, &ip);
    const bool whole = t0 + 8 <= rows && (ip & 7) == 0;  // the 8 tokens are one aligned run inside a page
    if (whole) {
      const int32_t page = page_tables[rq.page_table_off + pi];
      if (page < 0 || static_cast<uint32_t>(page) >= kv.n_pages) {
        if (dh == 0) atomicAdd(&kv.counters[ctr_index(kCtrBadPages)], 1ull);
        continue;
      }
      uint32_t w[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) w[e] = As[t0 + 2 * e][dh] | (static_cast<uint32_t>(As[t0 + 2 * e + 1][dh]) << 16);
      *reinterpret_cast<uint4*>(kv.base + static_cast<uint64_t>(page) * kv.page_size + voff + (static_cast<uint64_t>(dh) * hd.pt + ip) * 2) =
          make_uint4(w[0], w[1], w[2], w[3]);
    } else {
      for (uint32_t e = 0; e < 8 && t0 + e < rows; ++e) {
        split_token(hd, pos0 + t0 + e, &pi, &ip);
        const int32_t page = page_tables[rq.page_table_off + pi];
        if (page < 0 || static_cast<uint32_t>(page) >= kv.n_pages) {
          if (dh == 0) atomicAdd(&kv.counters[ctr_index(kCtrBadPages)], 1ull);
          continue;
        }
        *reinterpret_cast<uint16_t*>(kv.base + static_cast<uint64_t>(page) * kv.page_size + voff + (static_cast<uint64_t>(dh) * hd.pt + ip) * 2) =
            As[t0 + e][dh];
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// Fused layer halves for bf16 models with d = KD <= 256 (one kernel each, no normalised copy
// of the activations in memory):
//   FRONT: [U|V|Q|K] = SiLU(LN1(X) W1 + b1), U and Q*log2(e) to row-major buffers, K and V into
//          the pages;
//   BACK:  Y = X + (LN2(O) * U) W2 + b2.
// (X, Q, K, V, Y are bf16; O, U, the normalised operand and the weight copies are half precision.)
// A wavefront owns 32 token rows.  Their activations are loaded once (whole-line loads, dealt
// out to the lanes through LDS), normalised in registers (a row is split over the two lanes
// (g = 0, 1) that share the token: two cross-lane sums) and kept as the token-side MFMA operand
// for the whole sweep over the output columns, KD/16 fragments of 8 elements.  The weights (stored transposed, [out][KD]) pass through LDS in
// tiles of 32 output columns, double buffered with one barrier per tile; chunk c of tile row R
// sits at chunk position c ^ (R & 7) so that the operand reads of eight neighbouring lanes
// (eight rows, same c) hit different banks.  The product is taken as (W tile) x (X^T), so a
// lane ends up with one token and 16 output features (four runs of four); row-major outputs and
// K rows pass through a wave-private LDS tile and leave as 16-byte stores, V^T leaves as
// lane-coalesced 2-byte stores.
// WPB = wavefronts per block (a block covers 32 * WPB rows of a row tile of up to 128 rows).
// ---------------------------------------------------------------------------------------
struct LayerHalfArgs {
  HstuDims hd;
  uint32_t layer;
  const uint16_t* a_in;    // FRONT: X   BACK: O       [N][KD]
  const uint16_t* gate;    // BACK: U
  const float* ln_g;
  const float* ln_b;
  const uint16_t* wt;      // [n_out][KD] of this layer
  const float* bias;       // [n_out]
  uint16_t* u;             // FRONT outputs
  uint16_t* q;
  KvView kv;
  const ReqDev* reqs;
  const int32_t* page_tables;
  const uint16_t* resid;   // BACK: X
  uint16_t* y;             // BACK output
  const RowTile* row_tiles;
  uint32_t col_blocks_per_split;  // 32-column tiles one block sweeps
};

__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {
  typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
  typedef float v2f __attribute__((ext_vector_type(2)));
  const v2f v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, v2bf));
}
__device__ __forceinline__ void unpack8(const uint4& a, float v[8]) {  // eight bf16
  const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    v[2 * k] = __uint_as_float(w[k] << 16);
    v[2 * k + 1] = __uint_as_float(w[k] & 0xFFFF0000u);
  }
}
__device__ __forceinline__ void unpack8h(const uint4& a, float v[8]) {  // eight half-precision values
  const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const f16x2 h = __builtin_bit_cast(f16x2, w[k]);
    v[2 * k] = static_cast<float>(h[0]);
    v[2 * k + 1] = static_cast<float>(h[1]);
  }
}
// the rows a layer half normalises: the bf16 residual stream (front) or the half-precision attention output (back)
template <bool FRONT>
__device__ __forceinline__ void unpack_in(const uint4& a, float v[8]) {
  if (FRONT) unpack8(a, v);
  else unpack8h(a, v);
}

// Tells the compiler nothing about the value it returns: the unpacked fp32 copy of a row that an
// earlier pass over the registers made cannot be kept alive for a later pass (it would double
// the registers the row takes).
__device__ __forceinline__ void forget(uint4& a) { asm volatile("" : "+v"(a.x), "+v"(a.y), "+v"(a.z), "+v"(a.w)); }

template <int KD, bool FRONT, int WPB>
__global__ __attribute__((amdgpu_flat_work_group_size(64 * WPB, 64 * WPB), amdgpu_waves_per_eu(3, 3))) void layer_half_fused(LayerHalfArgs a) {
  constexpr int kSt = KD / 16;                 // MFMA steps over the contraction
  constexpr int kTileChunks = 32 * KD / 8;     // 16-byte chunks of a weight tile
  constexpr int kPerThread = kTileChunks / (64 * WPB);
  constexpr int kRowChunks = KD / 8;
  static_assert(kTileChunks % (64 * WPB) == 0, "weight tile must split evenly over the block");
  __shared__ __attribute__((aligned(16))) uint16_t wtile[2][32 * KD];
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, li = lane & 31;
  const RowTile rt = a.row_tiles[blockIdx.x / (4 / WPB)];
  const uint32_t sub = blockIdx.x % (4 / WPB);
  if (32 * WPB * sub >= rt.rows) return;  // this part of the row tile is empty
  const uint32_t rloc = 32 * (WPB * sub + wave) + li;  // row inside the tile
  const bool row_ok = rloc < rt.rows;
  const uint64_t row = rt.row0 + (row_ok ? rloc : 0);
  const HstuDims& hd = a.hd;

  // ---- activation rows: issue the loads ---------------------------------------------------------
  // A wavefront's 32 rows come in with whole-line loads (a load instruction covers the same half of 64 / (KD/16)
  // rows, 16 bytes per lane) and are dealt out to the operand layout (lane = token, 8 of every 16 elements)
  // through LDS: half a row of each of the 32 rows at a time, in the wavefront's quarter of the weight tile
  // buffers, which nothing uses before the first barrier below.  Chunk c of row r sits at c ^ (r mod chunks).
  // Rows past the tile's end read its first row; their results are never stored.
  constexpr int kHalfChunks = KD / 16;            // 16-byte chunks in half a row
  constexpr int kRowsPerLoad = 64 / kHalfChunks;  // rows one wave-wide load covers
  constexpr int kLoads = 32 / kRowsPerLoad;       // loads per half
  static_assert(kSt % 2 == 0 && 64 % kHalfChunks == 0 && 32 % kRowsPerLoad == 0, "row staging layout");
  const uint32_t stage_lr = lane / kHalfChunks, stage_lc = lane % kHalfChunks;
  auto issue_rows = [&](const uint16_t* src, int h, uint4 (&v)[kLoads]) {
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
      const uint32_t rl = 32 * (WPB * sub + wave) + kRowsPerLoad * i + stage_lr;
      v[i] = *reinterpret_cast<const uint4*>(src + (rt.row0 + (rl < rt.rows ? rl : 0)) * KD + 8 * (kHalfChunks * h + stage_lc));
    }
  };
  auto deal_rows = [&](const uint4 (&v)[kLoads], int h, uint4 (&dst)[kSt]) {
    uint16_t* stage = &wtile[0][0] + wave * (32 * KD / 2);
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
      const uint32_t r = kRowsPerLoad * i + stage_lr;
      *reinterpret_cast<uint4*>(stage + r * (KD / 2) + 8 * (stage_lc ^ (r & (kHalfChunks - 1)))) = v[i];
    }
#pragma unroll
    for (int s2 = 0; s2 < kSt / 2; ++s2)
      dst[kSt / 2 * h + s2] =
          *reinterpret_cast<const uint4*>(stage + li * (KD / 2) + 8 * ((2 * s2 + g) ^ (li & (kHalfChunks - 1))));
  };
  uint4 va[kLoads], vb[kLoads];
  issue_rows(a.a_in, 0, va);
  issue_rows(a.a_in, 1, vb);
  uint4 xr[kSt];  // this lane's half of its token's row: raw, then normalised (and gated) bf16
  deal_rows(va, 0, xr);
  if constexpr (!FRONT) issue_rows(a.gate, 0, va);
  deal_rows(vb, 1, xr);
  if constexpr (!FRONT) issue_rows(a.gate, 1, vb);

  // ---- where this lane's token goes (these dependent loads fly during the LayerNorm) ----------------
  const uint8_t* page_ptr = nullptr;  // FRONT: start of the token's page (nullptr: bad page id)
  uint32_t tok = 0;
  if (FRONT) {
    const ReqDev rq = a.reqs[rt.req];
    const uint32_t pos = rq.prefix_len + static_cast<uint32_t>(row - rq.x_off);
    uint32_t pi;
    split_token(hd, pos, &pi, &tok);
    if (row_ok) {
      const int32_t page = a.page_tables[rq.page_table_off + pi];
      if (page < 0 || static_cast<uint32_t>(page) >= a.kv.n_pages) {
        if (blockIdx.y == 0 && g == 0) atomicAdd(&a.kv.counters[ctr_index(kCtrBadPages)], 1ull);
      } else {
        page_ptr = a.kv.base + static_cast<uint64_t>(page) * a.kv.page_size;
      }
    }
  }

  // Row-major outputs leave through a wave-private LDS tile that turns "one token, four runs of four
  // features per lane" into 16-byte pieces: lane l then stores features 8 (l % 4) .. + 8 of the tokens
  // l / 4 and l / 4 + 16 of its wavefront, so four lanes cover 64 contiguous bytes of a row.
  const bool wave_has_rows = 32 * (WPB * sub + wave) < rt.rows;
  bool ok2[2];
  uint64_t row2[2];
  uint8_t* kdst2[2] = {nullptr, nullptr};  // FRONT: K row of the token inside its page, before the head offset
#pragma unroll
  for (int h2 = 0; h2 < 2; ++h2) {
    const uint32_t rl = 32 * (WPB * sub + wave) + (lane >> 2) + 16 * h2;
    ok2[h2] = rl < rt.rows;
    row2[h2] = rt.row0 + (ok2[h2] ? rl : 0);
    if (FRONT && ok2[h2]) {
      const ReqDev rq = a.reqs[rt.req];
      const uint32_t pos = rq.prefix_len + static_cast<uint32_t>(row2[h2] - rq.x_off);
      uint32_t pi, tk;
      split_token(hd, pos, &pi, &tk);
      const int32_t page = a.page_tables[rq.page_table_off + pi];
      if (page >= 0 && static_cast<uint32_t>(page) < a.kv.n_pages)
        kdst2[h2] = a.kv.base + static_cast<uint64_t>(page) * a.kv.page_size + static_cast<uint64_t>(tk) * 128;
    }
  }
  // ---- activations: load, normalise, keep as MFMA operand ----------------------------------
  __shared__ __attribute__((aligned(16))) float lnp[4][KD];  // LayerNorm scale and shift in the first two rows
  for (uint32_t i = tid; i < KD; i += 64 * WPB) {
    lnp[0][i] = a.ln_g[i];
    lnp[1][i] = a.ln_b[i];
  }
  {
    uint4 gr[FRONT ? 1 : kSt];  // BACK: the gate row
    if constexpr (!FRONT) {
      deal_rows(va, 0, gr);
      deal_rows(vb, 1, gr);
    }
    float s = 0.0f;
#pragma unroll
    for (int st = 0; st < kSt; ++st) {
      float v[8];
      unpack_in<FRONT>(xr[st], v);
#pragma unroll
      for (int e = 0; e < 8; ++e) s += v[e];
    }
    s += __shfl_xor(s, 32, 64);
    const float mean = s / KD;
    float qq = 0.0f;
#pragma unroll
    for (int st = 0; st < kSt; ++st) forget(xr[st]);
#pragma unroll
    for (int st = 0; st < kSt; ++st) {
      float v[8];
      unpack_in<FRONT>(xr[st], v);
#pragma unroll
      for (int e = 0; e < 8; ++e) qq += (v[e] - mean) * (v[e] - mean);
    }
    qq += __shfl_xor(qq, 32, 64);
    const float rstd = 1.0f / sqrtf(qq / KD + hd.eps);
    __syncthreads();  // lnp is visible
#pragma unroll
    for (int st = 0; st < kSt; ++st) forget(xr[st]);
#pragma unroll
    for (int st = 0; st < kSt; ++st) {
      float v[8], gg[8], bb[8];
      unpack_in<FRONT>(xr[st], v);
      load8(&lnp[0][16 * st + 8 * g], gg);
      load8(&lnp[1][16 * st + 8 * g], bb);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = (v[e] - mean) * rstd * gg[e] + bb[e];
      if (!FRONT) {
        float uv[8];
        unpack8h(gr[st], uv);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] *= uv[e];
      }
      xr[st] = make_uint4(pack2_f16(v[0], v[1]), pack2_f16(v[2], v[3]), pack2_f16(v[4], v[5]), pack2_f16(v[6], v[7]));
      // the result is pinned down here and memory operations may not pass: the LDS reads of later
      // steps stay behind this step's arithmetic instead of piling up in registers
      forget(xr[st]);
      asm volatile("" ::: "memory");

    }
  }
  // The LayerNorm parameters are done with; their LDS space takes this block's slice of the bias (at most
  // 4 KD columns per block).  Nothing inside the sweep below may read global memory for immediate use: the
  // wait for such a load also waits for every store and every weight prefetch issued before it.
  const uint32_t cb0 = blockIdx.y * a.col_blocks_per_split, n_cb = a.col_blocks_per_split;
  float* bias_s = &lnp[0][0];
  __syncthreads();
  for (uint32_t i = tid; i < n_cb * 32; i += 64 * WPB) bias_s[i] = a.bias[cb0 * 32 + i];

  constexpr int kOutStride = FRONT ? 40 : 72;  // 16-bit units per token row of the tile: 32 bf16 or 32 fp32, padded
  __shared__ __attribute__((aligned(16))) uint16_t otile[WPB][32 * kOutStride];
  uint16_t* ot = otile[wave];

  // ---- sweep over the output columns ----------------------------------------------------------
  // weight tiles travel global -> registers -> LDS, two tiles ahead of their use (two register sets;
  // named members and spelled-out steps, so that they are registers whatever the optimiser's unrolling order)
  struct WSet { uint4 c0, c1, c2, c3; };
  static_assert(kPerThread == 2 || kPerThread == 4, "a thread stages two or four chunks of a weight tile");
  const uint4 zero4 = make_uint4(0, 0, 0, 0);
  WSet wregA{zero4, zero4, zero4, zero4}, wregB{zero4, zero4, zero4, zero4};
  auto fetch_w = [&](WSet& wr, uint32_t cb) {
    const uint4* src = reinterpret_cast<const uint4*>(a.wt + static_cast<uint64_t>(cb) * 32 * KD) + tid;
    wr.c0 = src[0];
    wr.c1 = src[64 * WPB];
    if (kPerThread == 4) {
      wr.c2 = src[2 * 64 * WPB];
      wr.c3 = src[3 * 64 * WPB];
    }
  };
  auto put_w = [&](const uint4& v, uint32_t it, uint16_t* dst) {
    const uint32_t c = tid + 64 * WPB * it, R = c / kRowChunks, ch = c % kRowChunks;
    *reinterpret_cast<uint4*>(dst + R * KD + 8 * (ch ^ (R & 7))) = v;
  };
  auto commit_w = [&](const WSet& wr, uint16_t* dst) {
    put_w(wr.c0, 0, dst);
    put_w(wr.c1, 1, dst);
    if (kPerThread == 4) {
      put_w(wr.c2, 2, dst);
      put_w(wr.c3, 3, dst);
    }
  };
  uint32_t swz[4];  // element offset of chunk 2 j + g (j < 4) inside this lane's tile row
#pragma unroll
  for (uint32_t j = 0; j < 4; ++j) swz[j] = li * KD + 8 * ((2 * j + g) ^ (li & 7));

  // BACK: the residual pieces a lane adds at its two stores, fetched one tile ahead (the wait for them then
  // covers the stores of the tile before, not those just issued)
  struct RSet { uint4 r0, r1; };
  // (row2 of a lane without a row points at the tile's first row, so the loads need no condition)
  auto fetch_resid = [&](RSet& rs, uint32_t cb) {
    if (FRONT) return;
    rs.r0 = *reinterpret_cast<const uint4*>(a.resid + row2[0] * KD + cb * 32 + 8 * (lane & 3));
    rs.r1 = *reinterpret_cast<const uint4*>(a.resid + row2[1] * KD + cb * 32 + 8 * (lane & 3));
  };

  // Prefetches are issued unconditionally (past the end they fetch the last tile again): the compiler sizes
  // each wait by the memory operations that every path issues after the awaited one, and a prefetch under a
  // condition would make it wait for the stores just issued as well.
  const uint32_t cb_last = cb0 + n_cb - 1;
  // one 32-column tile: product, epilogue, stores
  auto compute = [&](const uint16_t* wb, uint32_t cb, const RSet& res, RSet& res_next) {
    const uint32_t n0 = cb * 32;
    fetch_resid(res_next, cb < cb_last ? cb + 1 : cb_last);
    f32x16 acc;
    // acc[e]: feature n0 + 8*(e/4) + 4*g + e%4 of this lane's token; the bias is the starting value
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      const float4 b = *reinterpret_cast<const float4*>(bias_s + (cb - cb0) * 32 + 8 * r4 + 4 * g);
      acc[4 * r4] = b.x; acc[4 * r4 + 1] = b.y; acc[4 * r4 + 2] = b.z; acc[4 * r4 + 3] = b.w;
    }
#pragma unroll
    for (int st = 0; st < kSt; ++st) {
      const f16x8 wf = __builtin_bit_cast(f16x8, *reinterpret_cast<const uint4*>(wb + swz[st & 3] + 64 * (st >> 2)));
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf, __builtin_bit_cast(f16x8, xr[st]), acc, 0, 0, 0);
    }
    if (!wave_has_rows) return;
    if (FRONT) {
      const uint32_t which = n0 / KD, c0 = n0 % KD;  // 0: U, 1: V, 2: Q, 3: K
      float z[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) z[e] = acc[e] * __builtin_amdgcn_rcpf(1.0f + __expf(-acc[e]));
      if (which == 1) {
        // V block [64][page_tokens]: the 32 lanes of a half-wave write 32 consecutive tokens of one feature
        if (page_ptr) {
          const uint32_t head = c0 / 64, cc = c0 % 64 + 4 * g;
          uint16_t* dst = reinterpret_cast<uint16_t*>(const_cast<uint8_t*>(page_ptr) + kv_block_offset(hd, a.layer, 1, head, 2)) + tok;
#pragma unroll
          for (int e = 0; e < 16; ++e)
            dst[static_cast<uint64_t>(cc + 8 * (e / 4) + e % 4) * hd.pt] = static_cast<uint16_t>(pack2_bf16(z[e], 0.0f));
        }
        return;
      }
      const float sc = which == 2 ? 1.4426950408889634f : 1.0f;  // the attention kernel wants q * log2(e)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4)
        *reinterpret_cast<uint2*>(ot + li * kOutStride + 8 * r4 + 4 * g) =
            which == 0  // U is the library's own (half precision); Q and K are bf16
                ? make_uint2(pack2_f16(z[4 * r4], z[4 * r4 + 1]), pack2_f16(z[4 * r4 + 2], z[4 * r4 + 3]))
                : make_uint2(pack2_bf16(z[4 * r4] * sc, z[4 * r4 + 1] * sc), pack2_bf16(z[4 * r4 + 2] * sc, z[4 * r4 + 3] * sc));
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        const uint4 v = *reinterpret_cast<const uint4*>(ot + ((lane >> 2) + 16 * h2) * kOutStride + 8 * (lane & 3));
        if (which == 3) {  // K block [token][64]
          if (kdst2[h2])
            *reinterpret_cast<uint4*>(kdst2[h2] + kv_block_offset(hd, a.layer, 0, c0 / 64, 2) + (c0 % 64 + 8 * (lane & 3)) * 2) = v;
        } else if (ok2[h2]) {
          *reinterpret_cast<uint4*>((which == 0 ? a.u : a.q) + row2[h2] * KD + c0 + 8 * (lane & 3)) = v;
        }
      }
    } else {
      float* otf = reinterpret_cast<float*>(ot);
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4)
        *reinterpret_cast<float4*>(otf + li * (kOutStride / 2) + 8 * r4 + 4 * g) =
            make_float4(acc[4 * r4], acc[4 * r4 + 1], acc[4 * r4 + 2], acc[4 * r4 + 3]);
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        const float* src = otf + ((lane >> 2) + 16 * h2) * (kOutStride / 2) + 8 * (lane & 3);
        const float4 p0 = *reinterpret_cast<const float4*>(src), p1 = *reinterpret_cast<const float4*>(src + 4);
        if (!ok2[h2]) continue;
        const uint64_t at = row2[h2] * KD + n0 + 8 * (lane & 3);
        float xv[8];
        unpack8(h2 == 0 ? res.r0 : res.r1, xv);
        *reinterpret_cast<uint4*>(a.y + at) = make_uint4(pack2_bf16(xv[0] + p0.x, xv[1] + p0.y), pack2_bf16(xv[2] + p0.z, xv[3] + p0.w),
                                                        pack2_bf16(xv[4] + p1.x, xv[5] + p1.y), pack2_bf16(xv[6] + p1.z, xv[7] + p1.w));
      }
    }
  };

  RSet resA{zero4, zero4}, resB{zero4, zero4};
  auto tile_at = [&](uint32_t k) { return cb0 + k < cb_last ? cb0 + k : cb_last; };
  fetch_resid(resA, cb0);
  fetch_w(wregA, cb0);
  fetch_w(wregB, tile_at(1));
  asm volatile("" ::: "memory");  // keeps the issue order: the waits inside the loop are sized by it
  commit_w(wregA, wtile[0]);
  asm volatile("" ::: "memory");
  fetch_w(wregA, tile_at(2));
  asm volatile("" ::: "memory");
  for (uint32_t k = 0; k < n_cb; k += 2) {  // n_cb is even (the launchers check it)
    // tile k is visible, and every wave is done with tile k-1, whose buffer takes tile k+1
    __syncthreads();
    commit_w(wregB, wtile[1]);
    fetch_w(wregB, tile_at(k + 3));
    compute(wtile[0], cb0 + k, resA, resB);
    __syncthreads();
    commit_w(wregA, wtile[0]);  // after the last pair: a copy of the last tile that nobody reads
    fetch_w(wregA, tile_at(k + 4));
    compute(wtile[1], cb0 + k + 1, resB, resA);
  }
}

// fp32 GEMM for the small configuration: one thread per output, W is [K][Nout]
template <typename Epi>
__global__ __launch_bounds__(256) void gemm_f32_simple(const float* __restrict__ A, const float* __restrict__ W,
                                                       uint32_t M, uint32_t K, uint32_t Nout, Epi epi) {
  const uint64_t idx = static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= static_cast<uint64_t>(M) * Nout) return;
  const uint32_t row = static_cast<uint32_t>(idx / Nout), col = static_cast<uint32_t>(idx % Nout);
  float acc = 0.0f;
  for (uint32_t k = 0; k < K; ++k) acc = fmaf(A[static_cast<uint64_t>(row) * K + k], W[static_cast<uint64_t>(k) * Nout + col], acc);
  epi(row, col, acc);
}

// ---------------------------------------------------------------------------------------
// fp32 attention: one wavefront per (query row, head); lanes stride over the keys
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void attention_f32(HstuDims hd, uint32_t layer, const float* __restrict__ q,
                                                     const float* __restrict__ pos, const float* __restrict__ time,
                                                     KvView kv, const ReqDev* __restrict__ reqs,
                                                     const uint32_t* __restrict__ row_req, uint32_t N,
                                                     const int32_t* __restrict__ page_tables,
                                                     const long long* __restrict__ ts, float* __restrict__ o) {
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t item = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= N * hd.H) return;
  const uint32_t row = item / hd.H, h = item % hd.H;
  const ReqDev rq = reqs[row_req[row]];
  const uint32_t p = rq.prefix_len + (row - rq.x_off);
  const long long ts_p = ts[rq.ts_off + p];
  float qv[64], acc[64];
#pragma unroll
  for (int c = 0; c < 64; ++c) {
    qv[c] = c < static_cast<int>(hd.dh) ? q[static_cast<uint64_t>(row) * hd.d + h * hd.dh + c] : 0.0f;
    acc[c] = 0.0f;
  }
  const float* pos_h = pos + (static_cast<uint64_t>(layer) * hd.H + h) * hd.n_pos;
  const float* time_h = time + (static_cast<uint64_t>(layer) * hd.H + h) * hd.n_time;
  const uint64_t koff = kv_block_offset(hd, layer, 0, h, 4), voff = kv_block_offset(hd, layer, 1, h, 4);
  for (uint32_t j = lane; j <= p; j += 64) {
    const int32_t page = page_tables[rq.page_table_off + j / hd.pt];
    if (page < 0 || static_cast<uint32_t>(page) >= kv.n_pages) {
      atomicAdd(&kv.counters[ctr_index(kCtrBadPages)], 1ull);
      continue;
    }
    const uint8_t* pb = kv.base + static_cast<uint64_t>(page) * kv.page_size;
    const float* kr = reinterpret_cast<const float*>(pb + koff) + static_cast<uint64_t>(j % hd.pt) * hd.dh;
    const float* vt = reinterpret_cast<const float*>(pb + voff) + (j % hd.pt);
    float s = 0.0f;
#pragma unroll
    for (int c = 0; c < 64; ++c)
      if (c < static_cast<int>(hd.dh)) s = fmaf(qv[c], kr[c], s);
    const uint32_t rel = p - j < hd.n_pos - 1 ? p - j : hd.n_pos - 1;
    s += pos_h[rel] + time_h[time_bucket(ts_p - ts[rq.ts_off + j], hd.n_time)];
    const float a = s / (1.0f + expf(-s));
#pragma unroll
    for (int c = 0; c < 64; ++c)
      if (c < static_cast<int>(hd.dh)) acc[c] = fmaf(a, vt[static_cast<uint64_t>(c) * hd.pt], acc[c]);
  }
#pragma unroll
  for (int c = 0; c < 64; ++c) {
    if (c < static_cast<int>(hd.dh)) {
      const float t = wave_sum(acc[c]);
      if (lane == 0) o[static_cast<uint64_t>(row) * hd.d + h * hd.dh + c] = t * hd.inv_n;
    }
  }
}

// ---------------------------------------------------------------------------------------
// bf16 paged attention on MFMA, d_h = 64.  A block of four wavefronts owns 128 * NQB consecutive
// queries of one request and one head (32 * NQB per wavefront, as NQB 32-query groups) and walks
// a range of key tiles (64 keys), staging K [key][d_h] and V^T [d_h][key] of the tile in
// LDS through the page table (tile k+1 is fetched into registers while tile k is used).
// Each wavefront computes S^T = K Q^T (keys x queries, so a lane ends up holding one query
// and 16 keys), applies bias, SiLU and the causal mask in registers, and feeds the bf16
// result straight back as the second operand of O^T += V^T P^T: the accumulator layout of
// the first product is the operand layout of the second, so the scores never leave
// registers.  K rows are kept in LDS in a permuted order (bits 2 and 3 of the key
// index swapped) so that the 8 keys a lane holds per contraction step are consecutive
// and the matching V^T operand is one 16-byte LDS read.
//
// The epilogue is the binding unit (16 scores per lane against 8 MFMAs), so it is pared
// down to the minimum:
//   - Q arrives multiplied by log2(e) and both bias tables are scaled likewise, so that
//     y = x*log2(e) comes out of the matrix product and SiLU(x) = ln2 * y / (1 + 2^-y);
//     ln2 and 1/n are applied once to the output accumulators;
//   - the positional bias is Toeplitz: the window of the (reversed, scaled) table that a key
//     tile needs sits in LDS, in four copies shifted by one element each so that every lane
//     can read its 8 consecutive entries as aligned 16-byte words, and initialises the score
//     accumulators, so adding it costs no arithmetic;
//   - time gaps are taken from 32-bit timestamps relative to the request's first one; for a
//     32x32 block whose smallest and largest gap fall into the same log2 bucket (most blocks
//     away from the diagonal) the time bias is one scalar; if they fall into adjacent
//     buckets it is a compare-and-select per score; other blocks take the bucket per score;
//     requests spanning >= 2^31 s (or models with more than 32 buckets) use 64-bit gaps;
//   - the causal select is applied only in blocks that touch the diagonal.
// ---------------------------------------------------------------------------------------
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr uint32_t kPosWinMax = 320;  // 256 queries + 64 keys - 1 distances per tile, padded

struct AttnTile {  // one staged key tile
  uint16_t Ks[64][64 + kLdsPad];
  uint16_t Vs[64][64 + kLdsPad];
  uint32_t tk[64];             // key timestamps relative to the request's first one
  // copy s holds window entry x at [s][4 + x - s]; a copy is 32 bytes (mod 128) long, which spreads the
  // 16-byte reads of eight neighbouring lanes (two per copy) over all LDS banks
  float pos[4][kPosWinMax + 8];
};

struct AttnShared {
  AttnTile tile[2];  // tile k is consumed from one half while tile k+1 is written into the other
  float time[64];
  float rtime[32];   // rtime[c] = time bias of a gap with c leading zero bits (32-bit gaps, n_time <= 32)
  int32_t pages[kAttnMaxItemPages];  // page ids of the item's key range (-1: outside the pool)
};

__device__ __forceinline__ uint32_t bucket_u32(uint32_t dt, uint32_t n_time) {
  const uint32_t b = dt > 1 ? 31u - static_cast<uint32_t>(__clz(static_cast<int>(dt))) : 0u;
  return b < n_time - 1 ? b : n_time - 1;
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// y * sigmoid(y / log2 e) without the ln2 factor: y / (1 + 2^-y)
__device__ __forceinline__ float silu_log2(float y) {
  return y * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-y));
}

// NQB = 32-query groups per wavefront (1: 128 queries per block, three resident blocks per CU).
// OHALF: the output goes out in half precision (the step's own matrix between the attention and the second
// LayerNorm) instead of bf16 (what a caller of the attention alone gets).
template <int NQB, bool OHALF>
__global__ __launch_bounds__(256, NQB == 1 ? 3 : 2) void attention_bf16_mfma(HstuDims hd, uint32_t layer, const uint16_t* __restrict__ q,
                                                              const float* __restrict__ pos,
                                                              const float* __restrict__ time, KvView kv,
                                                              const ReqDev* __restrict__ reqs,
                                                              const AttnItem* __restrict__ items,
                                                              const AttnWork* __restrict__ work,
                                                              float* __restrict__ partials,
                                                              const int32_t* __restrict__ page_tables,
                                                              const long long* __restrict__ ts,
                                                              uint16_t* __restrict__ o) {
  constexpr uint32_t kQ = 128 * NQB;     // queries per block
  constexpr uint32_t kPosWin = kQ + 64;  // distances a tile can need (kQ + 63), padded
  __shared__ __attribute__((aligned(16))) AttnShared sm;
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, li = lane & 31;
  const AttnWork wk = work[blockIdx.x];
  if (wk.item == kNoWork) return;  // padding of a die's list
  const AttnItem item = items[wk.item];
  const uint32_t r = item.req, qt = item.qt, h = wk.head;
  const ReqDev rq = reqs[r];
  const uint32_t P = rq.prefix_len, T = rq.new_len, S = P + T;
  const uint32_t q0 = qt * kQ;  // first query (index among the new tokens) of the block
  const long long* tsr = ts + rq.ts_off;
  const long long ts_base = tsr[0];
  const long long span = tsr[S - 1] - ts_base;
  // 32-bit times relative to the request's first: only for requests whose timestamps never decrease
  const bool fast = hd.n_time <= 32 && rq.ts_ordered != 0 && span >= 0 && span < (1ll << 31);
  if (tid < 64) sm.time[tid] = tid < hd.n_time ? time[(static_cast<uint64_t>(layer) * hd.H + h) * hd.n_time + tid] : 0.0f;
  if (tid >= 64 && tid < 96) {
    const uint32_t bkt = 95 - tid;  // floor(log2(gap)) of a gap with tid - 64 leading zeros
    sm.rtime[tid - 64] = time[(static_cast<uint64_t>(layer) * hd.H + h) * hd.n_time + (bkt < hd.n_time - 1 ? bkt : hd.n_time - 1)];
  }
  const float* pos_h = pos + (static_cast<uint64_t>(layer) * hd.H + h) * hd.n_pos;

  // per 32-query group qb of this wavefront
  uint32_t ql[NQB], p[NQB], grp_first[NQB], grp_last[NQB], tq[NQB], tq_first[NQB], tq_last[NQB];
  bool q_ok[NQB], grp_active[NQB];
  long long ts_q[NQB];
  bf16x8 qf[NQB][4];  // Q^T operand: lane (g, li) holds query li, d_h elements 16*st + 8*g .. +8
  f32x16 oacc[NQB][2];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    ql[qb] = 32 * NQB * wave + 32 * qb + li;  // query index inside the block
    const uint32_t qi = q0 + ql[qb];
    q_ok[qb] = qi < T;
    p[qb] = P + qi;
    const uint32_t first = q0 + 32 * NQB * wave + 32 * qb;
    grp_active[qb] = first < T;
    grp_first[qb] = P + first;
    grp_last[qb] = P + (first + 31 < T - 1 ? first + 31 : T - 1);
    ts_q[qb] = q_ok[qb] ? tsr[p[qb]] : ts_base;
    tq[qb] = static_cast<uint32_t>(ts_q[qb] - ts_base);
    uint32_t a = 0, b = 0;
    if (grp_active[qb]) {
      a = static_cast<uint32_t>(tsr[grp_first[qb]] - ts_base);
      b = static_cast<uint32_t>(tsr[grp_last[qb]] - ts_base);
    }
    tq_first[qb] = __builtin_amdgcn_readfirstlane(a);
    tq_last[qb] = __builtin_amdgcn_readfirstlane(b);
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      uint4 val = make_uint4(0, 0, 0, 0);
      if (q_ok[qb]) val = *reinterpret_cast<const uint4*>(q + static_cast<uint64_t>(rq.x_off + qi) * hd.d + h * 64 + 16 * st + 8 * g);
      qf[qb][st] = __builtin_bit_cast(bf16x8, val);
    }
#pragma unroll
    for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[qb][b2][e] = 0.0f;
  }

  const uint64_t koff = kv_block_offset(hd, layer, 0, h, 2), voff = kv_block_offset(hd, layer, 1, h, 2);
  const uint32_t kt_begin = item.kt_begin, kt_end = item.kt_end;
  // the item's slice of the page table goes to LDS once, so that a tile fetch is a single
  // global round trip instead of two dependent ones
  uint32_t page0, unused_ip;
  split_token(hd, kt_begin * 64, &page0, &unused_ip);
  {
    const uint32_t last_key = (kt_end * 64 < S ? kt_end * 64 : S) - 1;
    uint32_t page_last;
    split_token(hd, last_key, &page_last, &unused_ip);
    for (uint32_t i = tid; i <= page_last - page0 && i < kAttnMaxItemPages; i += 256) {
      int32_t pg = page_tables[rq.page_table_off + page0 + i];
      if (pg < 0 || static_cast<uint32_t>(pg) >= kv.n_pages) {
        atomicAdd(&kv.counters[ctr_index(kCtrBadPages)], 1ull);
        pg = -1;
      }
      sm.pages[i] = pg;
    }
  }
  __syncthreads();

  // registers that carry the next tile from global memory to LDS
  uint4 kreg[2], vreg[2];
  uint32_t treg = 0;
  float preg[2] = {0.0f, 0.0f};
  // thread-constant byte offsets of its two K and two V^T chunks inside a tile that lies in one page
  const bool one_page_tiles = hd.pt_shift < 32 && hd.pt >= 64;
  uint32_t kconst[2], vconst[2];
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const uint32_t c = tid + 256 * it, row = c >> 3, part = c & 7;
    kconst[it] = row * 128 + part * 16;
    vconst[it] = (row * hd.pt + part * 8) * 2;
  }
  const int32_t pos_top = static_cast<int32_t>(P + q0 + kQ - 1);  // window entry m of tile j0 is pos[pos_top - j0 - m]
  auto fetch = [&](uint32_t kt) {
    const uint32_t j0 = kt * 64;
    bool done = false;
    if (one_page_tiles && j0 + 64 <= S) {
      // the whole tile sits in one page and inside the sequence: one scalar base, no per-thread arithmetic
      const int32_t page = __builtin_amdgcn_readfirstlane(sm.pages[(j0 >> hd.pt_shift) - page0]);
      if (page >= 0) {
        const uint32_t tb = j0 & (hd.pt - 1);
        const uint8_t* pb = kv.base + static_cast<uint64_t>(page) * kv.page_size;
        const uint8_t* kbase = pb + koff + static_cast<uint64_t>(tb) * 128;
        const uint8_t* vbase = pb + voff + static_cast<uint64_t>(tb) * 2;
#pragma unroll
        for (int it = 0; it < 2; ++it) {
          kreg[it] = *reinterpret_cast<const uint4*>(kbase + kconst[it]);
          vreg[it] = *reinterpret_cast<const uint4*>(vbase + vconst[it]);
        }
        done = true;
      }
    }
    if (!done) {
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        const uint32_t c = tid + 256 * it, row = c >> 3, part = c & 7;
        // K: row = key, part = 8 d_h elements
        kreg[it] = make_uint4(0, 0, 0, 0);
        const uint32_t j = j0 + row;
        if (j < S) {
          uint32_t pi, ip;
          split_token(hd, j, &pi, &ip);
          const int32_t page = sm.pages[pi - page0];
          if (page >= 0)
            kreg[it] = *reinterpret_cast<const uint4*>(kv.base + static_cast<uint64_t>(page) * kv.page_size + koff +
                                                       (static_cast<uint64_t>(ip) * 64 + part * 8) * 2);
        }
        // V^T: row = d_h element, part = 8 consecutive keys (inside one page: page_tokens % 8 == 0)
        vreg[it] = make_uint4(0, 0, 0, 0);
        const uint32_t jv = j0 + part * 8;
        if (jv < S) {
          uint32_t pi, ip;
          split_token(hd, jv, &pi, &ip);
          const int32_t page = sm.pages[pi - page0];
          if (page >= 0) {
            uint4 vval = *reinterpret_cast<const uint4*>(kv.base + static_cast<uint64_t>(page) * kv.page_size + voff +
                                                         (static_cast<uint64_t>(row) * hd.pt + ip) * 2);
            if (jv + 8 > S) {  // keys past the end of the sequence hold whatever the page held before
              uint32_t w[4] = {vval.x, vval.y, vval.z, vval.w};
#pragma unroll
              for (int e = 0; e < 8; ++e)
                if (jv + e >= S) w[e >> 1] &= (e & 1) ? 0x0000FFFFu : 0xFFFF0000u;
              vval = make_uint4(w[0], w[1], w[2], w[3]);
            }
            vreg[it] = vval;
          }
        }
      }
    }
    // window of the reversed positional table (already scaled by log2 e); entries with a negative
    // distance belong to keys after the query, which the causal select removes
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const uint32_t m = tid + 256 * it;
      if (m < kPosWin) {
        int32_t i = pos_top - static_cast<int32_t>(j0) - static_cast<int32_t>(m);
        i = i < 0 ? 0 : (i > static_cast<int32_t>(hd.n_pos) - 1 ? static_cast<int32_t>(hd.n_pos) - 1 : i);
        preg[it] = pos_h[i];
      }
    }
    if (tid < 64) treg = (j0 + tid < S) ? static_cast<uint32_t>(tsr[j0 + tid] - ts_base) : 0u;
  };
  auto commit = [&](AttnTile& t) {
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const uint32_t c = tid + 256 * it, row = c >> 3, part = c & 7;
      // key row r is stored at row perm(r) (bits 2 and 3 swapped): the first product then reads
      // consecutive LDS rows, which the row padding keeps free of bank conflicts
      *reinterpret_cast<uint4*>(&t.Ks[(row & 0x33) | ((row & 8) >> 1) | ((row & 4) << 1)][part * 8]) = kreg[it];
      *reinterpret_cast<uint4*>(&t.Vs[row][part * 8]) = vreg[it];
      if (c < kPosWin) {
#pragma unroll
        for (uint32_t s = 0; s < 4; ++s) t.pos[s][4 + c - s] = preg[it];  // copy s = window shifted by s
      }
    }
    if (tid < 64) t.tk[tid] = treg;
  };

  // first and last key timestamp of the two 32-key halves of a tile, through the scalar unit
  // (read-only), one tile ahead; indices are clamped to the sequence
  auto tile_times = [&](uint32_t kt, uint32_t out[4]) {
    const uint32_t j0 = kt * 64;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint32_t j = j0 + 32 * (k >> 1) + 31 * (k & 1);
      out[k] = static_cast<uint32_t>(tsr[j < S ? j : S - 1] - ts_base);
    }
  };
  uint32_t tkb[4], tkb_next[4] = {0, 0, 0, 0};
  fetch(kt_begin);
  tile_times(kt_begin, tkb);
  commit(sm.tile[0]);
  if (kt_begin + 1 < kt_end) fetch(kt_begin + 1);
  uint32_t cur = 0;
  for (uint32_t kt = kt_begin; kt < kt_end; ++kt, cur ^= 1) {
    const uint32_t j0 = kt * 64;
    AttnTile& tl = sm.tile[cur];
    // one barrier per tile: tile kt is visible, and every wave is done with tile kt-1, whose
    // half now takes tile kt+1 (in registers since the previous iteration)
    __syncthreads();
    if (kt != kt_begin) {
#pragma unroll
      for (int k = 0; k < 4; ++k) tkb[k] = tkb_next[k];
    }
    if (kt + 1 < kt_end) {
      commit(sm.tile[cur ^ 1]);
      tile_times(kt + 1, tkb_next);
      if (kt + 2 < kt_end) fetch(kt + 2);  // its global loads fly while this tile is consumed
    }

    {
      // operands are read from LDS right where they are consumed: holding all of them across
      // the epilogue would push the kernel past 256 registers
      auto k_frag = [&](int sb, int st) {
        return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&tl.Ks[32 * sb + li][16 * st + 8 * g]));
      };
      auto v_frag = [&](int sb, int s2, int db) {
        return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&tl.Vs[32 * db + li][32 * sb + 16 * s2 + 8 * g]));
      };
      // S^T = K Q^T on top of the positional bias: lane's window entries m0 .. m0+7 and m0+16 .. m0+23
      auto scores_begin = [&](int qb, int sb) {
        const uint32_t m0 = (kQ - 1) - ql[qb] + 32 * sb + 8 * g;
        const float* pw = &tl.pos[m0 & 3][4 + (m0 & ~3u)];
        const float4 w0 = *reinterpret_cast<const float4*>(pw), w1 = *reinterpret_cast<const float4*>(pw + 4);
        const float4 w2 = *reinterpret_cast<const float4*>(pw + 16), w3 = *reinterpret_cast<const float4*>(pw + 20);
        f32x16 sacc;
        sacc[0] = w0.x; sacc[1] = w0.y; sacc[2] = w0.z; sacc[3] = w0.w;
        sacc[4] = w1.x; sacc[5] = w1.y; sacc[6] = w1.z; sacc[7] = w1.w;
        sacc[8] = w2.x; sacc[9] = w2.y; sacc[10] = w2.z; sacc[11] = w2.w;
        sacc[12] = w3.x; sacc[13] = w3.y; sacc[14] = w3.z; sacc[15] = w3.w;
        return sacc;
      };
      // bias, SiLU, mask -> bf16 pairs.  sacc[e]: key kb + 16*(e/8) + 8*g + e%8, query li of group qb;
      // y = (q.k + pos) * log2 e
      auto epilogue = [&](int qb, int sb, const f32x16& sacc, uint32_t pk[8]) {
        const uint32_t kb = j0 + 32 * sb;
        const bool diag = kb + 31 > grp_first[qb];
        int mode = 2;  // 0: one time bias for the block, 1: two adjacent buckets, 2: bucket per score (+ mask)
        float c_lo = 0.0f, c_hi = 0.0f;
        uint32_t thr = 0;
        if (fast && !diag) {
          const uint32_t tk_first = tkb[2 * sb], tk_last = tkb[2 * sb + 1];
          const uint32_t bmin = bucket_u32(tq_first[qb] - tk_last, hd.n_time);
          const uint32_t bmax = bucket_u32(tq_last[qb] - tk_first, hd.n_time);
          c_lo = sm.time[bmin];
          if (bmin == bmax) {
            mode = 0;
          } else if (bmax == bmin + 1) {
            mode = 1;
            c_hi = sm.time[bmax];
            thr = 2u << bmin;  // gaps >= 2^(bmin+1) belong to the upper bucket
          }
        }
        if (mode == 0) {
#pragma unroll
          for (int e = 0; e < 16; e += 2)
            pk[e >> 1] = pack_bf16x2(silu_log2(sacc[e] + c_lo), silu_log2(sacc[e + 1] + c_lo));
          return;
        }
        if (fast) {
          // eight scores at a time: the lane's key timestamps (all below 2^31) come as two 16-byte reads
          const uint4* tkp = reinterpret_cast<const uint4*>(&tl.tk[32 * sb + 8 * g]);
          const int32_t lim_t = tq[qb] >= thr ? static_cast<int32_t>(tq[qb] - thr) : -1;
          const int lim = static_cast<int>(p[qb]) - static_cast<int>(kb) - 8 * static_cast<int>(g);  // visible: key offset <= lim
#pragma unroll
          for (int hf = 0; hf < 2; ++hf) {
            const uint4 t0 = tkp[4 * hf], t1 = tkp[4 * hf + 1];
            const uint32_t tkl[8] = {t0.x, t0.y, t0.z, t0.w, t1.x, t1.y, t1.z, t1.w};
            float a[8];
            if (mode == 1) {
              // gap >= thr  <=>  key time <= query time - thr (never, if that is negative)
#pragma unroll
              for (int e = 0; e < 8; ++e)
                a[e] = silu_log2(sacc[8 * hf + e] + (static_cast<int32_t>(tkl[e]) <= lim_t ? c_hi : c_lo));
            } else {
              // bucket per score through the table indexed by the gap's leading zero count; a key after
              // the query gives a wrapped gap, whose (valid) table entry the causal select discards
#pragma unroll
              for (int e = 0; e < 8; ++e) {
                const uint32_t gap = tq[qb] - tkl[e];
                a[e] = silu_log2(sacc[8 * hf + e] + sm.rtime[__clz(static_cast<int>(gap > 1 ? gap : 1))]);
              }
              if (diag) {
#pragma unroll
                for (int e = 0; e < 8; ++e) a[e] = 16 * hf + e <= lim ? a[e] : 0.0f;
              }
            }
#pragma unroll
            for (int e = 0; e < 8; e += 2) pk[4 * hf + (e >> 1)] = pack_bf16x2(a[e], a[e + 1]);
          }
          return;
        }
        float a[16];
        {
          // 64-bit gaps (requests spanning 2^31 s or more, or more than 32 buckets)
          const int lim = static_cast<int>(p[qb]) - static_cast<int>(kb) - 8 * static_cast<int>(g);
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int off = 16 * (e / 8) + (e % 8);
            const uint32_t jl = 32 * sb + off + 8 * g;
            const uint32_t bkt = time_bucket(ts_q[qb] - (j0 + jl < S ? tsr[j0 + jl] : ts_base), hd.n_time);
            const float v = silu_log2(sacc[e] + sm.time[bkt]);
            a[e] = off <= lim ? v : 0.0f;
          }
        }
#pragma unroll
        for (int e = 0; e < 16; e += 2) pk[e >> 1] = pack_bf16x2(a[e], a[e + 1]);
      };
      // O^T += V^T P^T; the P^T operand of step s2 = elements 8*s2 .. 8*s2+7: keys kb + 16*s2 + 8*g + 0..7
      auto accumulate = [&](int qb, int sb, const uint32_t pk[8]) {
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const bf16x8 pf = __builtin_bit_cast(bf16x8, make_uint4(pk[4 * s2], pk[4 * s2 + 1], pk[4 * s2 + 2], pk[4 * s2 + 3]));
#pragma unroll
          for (int db = 0; db < 2; ++db)
            oacc[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_frag(sb, s2, db), pf, oacc[qb][db], 0, 0, 0);
        }
      };
      // which (query group, sub-block) pairs hold at least one visible (query, key) pair
      auto visible = [&](int qb, int sb) { return grp_active[qb] && j0 + 32 * sb <= grp_last[qb]; };
      if (NQB == 1 && visible(0, 1)) {
        // both sub-blocks are visible: the two score chains are issued interleaved, and each
        // sub-block's second product runs while the other's epilogue executes
        f32x16 s0 = scores_begin(0, 0), s1 = scores_begin(0, 1);
#pragma unroll
        for (int st = 0; st < 4; ++st) {
          s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_frag(0, st), qf[0][st], s0, 0, 0, 0);
          s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_frag(1, st), qf[0][st], s1, 0, 0, 0);
        }
        uint32_t pk0[8], pk1[8];
        epilogue(0, 0, s0, pk0);
        accumulate(0, 0, pk0);
        epilogue(0, 1, s1, pk1);
        accumulate(0, 1, pk1);
      } else {
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
          if (NQB == 2 && visible(0, sb) && visible(NQB - 1, sb) && j0 + 32 * sb <= grp_last[0]) {
            // both query groups see the sub-block: same interleaving over the groups
            f32x16 s0 = scores_begin(0, sb), s1 = scores_begin(NQB - 1, sb);
#pragma unroll
            for (int st = 0; st < 4; ++st) {
              const bf16x8 kf = k_frag(sb, st);
              s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[0][st], s0, 0, 0, 0);
              s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[NQB - 1][st], s1, 0, 0, 0);
            }
            uint32_t pk0[8], pk1[8];
            epilogue(0, sb, s0, pk0);
            accumulate(0, sb, pk0);
            epilogue(NQB - 1, sb, s1, pk1);
            accumulate(NQB - 1, sb, pk1);
          } else {
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb) {
              if (!visible(qb, sb)) continue;
              f32x16 s0 = scores_begin(qb, sb);
#pragma unroll
              for (int st = 0; st < 4; ++st) s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_frag(sb, st), qf[qb][st], s0, 0, 0, 0);
              uint32_t pk0[8];
              epilogue(qb, sb, s0, pk0);
              accumulate(qb, sb, pk0);
            }
          }
        }
      }
    }
  }
  // oacc[qb][db][e]: d_h element 32*db + 8*(e/4) + 4*g + e%4 of the lane's query; undo the log2 e scaling, apply 1/n
  const float sc = hd.inv_n * kLn2;
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    if (item.slot != kDirect) {
      // part of a split query tile: fp32 partial [slot][head][query][d_h], summed by attention_reduce
      float* prow = partials + ((static_cast<uint64_t>(item.slot) * hd.H + h) * kQ + ql[qb]) * 64;
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4)
          *reinterpret_cast<float4*>(prow + 32 * db + 8 * e4 + 4 * g) =
              make_float4(oacc[qb][db][4 * e4] * sc, oacc[qb][db][4 * e4 + 1] * sc, oacc[qb][db][4 * e4 + 2] * sc,
                          oacc[qb][db][4 * e4 + 3] * sc);
    } else if (q_ok[qb]) {
      uint16_t* orow = o + static_cast<uint64_t>(rq.x_off + q0 + ql[qb]) * hd.d + h * 64;
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          uint2 w;
          if (OHALF) {
            w.x = pack2_f16(oacc[qb][db][4 * e4] * sc, oacc[qb][db][4 * e4 + 1] * sc);
            w.y = pack2_f16(oacc[qb][db][4 * e4 + 2] * sc, oacc[qb][db][4 * e4 + 3] * sc);
          } else {
            w.x = pack_bf16x2(oacc[qb][db][4 * e4] * sc, oacc[qb][db][4 * e4 + 1] * sc);
            w.y = pack_bf16x2(oacc[qb][db][4 * e4 + 2] * sc, oacc[qb][db][4 * e4 + 3] * sc);
          }
          *reinterpret_cast<uint2*>(orow + 32 * db + 8 * e4 + 4 * g) = w;
        }
    }
  }
}

// Sum the fp32 partials of a split query tile in chunk order and write the bf16 output.
__global__ __launch_bounds__(256) void attention_reduce(HstuDims hd, uint32_t q_block, const ReqDev* __restrict__ reqs,
                                                        const AttnGroup* __restrict__ groups,
                                                        const float* __restrict__ partials, uint16_t* __restrict__ o,
                                                        uint32_t o_half) {
  // blockIdx.x = (group, head); blockIdx.y = which 16 of the tile's query rows: a thread owns one 16-byte piece of
  // one row, so that the chunks' loads of a whole tile are in flight at once
  const AttnGroup gr = groups[blockIdx.x / hd.H];
  const uint32_t h = blockIdx.x % hd.H;
  const ReqDev rq = reqs[gr.req];
  const uint32_t idx = blockIdx.y * 256 + threadIdx.x;
  const uint32_t row = idx >> 4, c4 = idx & 15;
  const uint32_t qi = gr.qt * q_block + row;
  if (row >= q_block || qi >= rq.new_len) return;
  const float* src = partials + ((static_cast<uint64_t>(gr.slot0) * hd.H + h) * q_block + row) * 64 + 4 * c4;
  const uint64_t step = static_cast<uint64_t>(hd.H) * q_block * 64;  // from one chunk's partial to the next
  float4 acc = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  uint32_t k = 0;
  for (; k + 4 <= gr.chunks; k += 4) {  // four loads in flight; the sum keeps the chunk order
    const float4 v0 = *reinterpret_cast<const float4*>(src + (k + 0) * step);
    const float4 v1 = *reinterpret_cast<const float4*>(src + (k + 1) * step);
    const float4 v2 = *reinterpret_cast<const float4*>(src + (k + 2) * step);
    const float4 v3 = *reinterpret_cast<const float4*>(src + (k + 3) * step);
    acc.x += v0.x; acc.y += v0.y; acc.z += v0.z; acc.w += v0.w;
    acc.x += v1.x; acc.y += v1.y; acc.z += v1.z; acc.w += v1.w;
    acc.x += v2.x; acc.y += v2.y; acc.z += v2.z; acc.w += v2.w;
    acc.x += v3.x; acc.y += v3.y; acc.z += v3.z; acc.w += v3.w;
  }
  for (; k < gr.chunks; ++k) {
    const float4 v = *reinterpret_cast<const float4*>(src + k * step);
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  uint2 w;
  if (o_half) {
    w.x = pack2_f16(acc.x, acc.y);
    w.y = pack2_f16(acc.z, acc.w);
  } else {
    w.x = pack_bf16x2(acc.x, acc.y);
    w.y = pack_bf16x2(acc.z, acc.w);
  }
  *reinterpret_cast<uint2*>(o + static_cast<uint64_t>(rq.x_off + qi) * hd.d + h * 64 + 4 * c4) = w;
}

// Are a request's timestamps non-decreasing?  Block (c, r) looks at tokens 2048 c + 1 .. 2048 (c + 1) of request r
// (eight per thread, all loads independent).  The host sets ts_ordered to 1; the first block that finds a decrease
// clears it and counts the request.
constexpr uint32_t kTsChunk = 2048;
__global__ __launch_bounds__(256) void check_timestamps(ReqDev* __restrict__ reqs, uint32_t B,
                                                        const long long* __restrict__ ts,
                                                        unsigned long long* __restrict__ counters) {
  for (uint32_t r = blockIdx.y; r < B; r += gridDim.y) {  // (the grid's second dimension stops at 65 535)
    const uint32_t S = reqs[r].prefix_len + reqs[r].new_len;
    const uint32_t j0 = blockIdx.x * kTsChunk + 1;
    if (j0 >= S) continue;  // uniform over the block
    const long long* t = ts + reqs[r].ts_off;
    bool bad = false;
#pragma unroll
    for (uint32_t k = 0; k < kTsChunk / 256; ++k) {
      const uint32_t j = j0 + k * 256 + threadIdx.x;
      if (j < S) bad |= t[j] < t[j - 1];
    }
    if (__syncthreads_or(bad) && threadIdx.x == 0) {
      if (atomicExch(&reqs[r].ts_ordered, 0u) == 1u) atomicAdd(&counters[ctr_index(kCtrUnorderedTs)], 1ull);
    }
  }
}

__global__ void scale_f32(const float* __restrict__ in, float* __restrict__ out, uint64_t n, float s) {
  for (uint64_t k = blockIdx.x * static_cast<uint64_t>(blockDim.x) + threadIdx.x; k < n;
       k += static_cast<uint64_t>(gridDim.x) * blockDim.x)
    out[k] = in[k] * s;
}

// q * log2(e) for callers that hand the attention kernel an unscaled query matrix
__global__ void scale_bf16(const uint16_t* __restrict__ in, uint16_t* __restrict__ out, uint64_t n, float s) {
  for (uint64_t k = blockIdx.x * static_cast<uint64_t>(blockDim.x) + threadIdx.x; k < n;
       k += static_cast<uint64_t>(gridDim.x) * blockDim.x)
    out[k] = f2bf(bf2f(in[k]) * s);
}

template <typename T>
__global__ void transpose_kernel(const T* __restrict__ w, T* __restrict__ wt, uint32_t rows, uint32_t cols) {
  __shared__ T tile[32][33];
  const uint32_t bx = blockIdx.x * 32, by = blockIdx.y * 32;
  for (uint32_t yy = threadIdx.y; yy < 32; yy += 8)
    if (by + yy < rows && bx + threadIdx.x < cols) tile[yy][threadIdx.x] = w[static_cast<uint64_t>(by + yy) * cols + bx + threadIdx.x];
  __syncthreads();
  for (uint32_t yy = threadIdx.y; yy < 32; yy += 8)
    if (bx + yy < cols && by + threadIdx.x < rows) wt[static_cast<uint64_t>(bx + yy) * rows + by + threadIdx.x] = tile[threadIdx.x][yy];
}

// transposed copy of a bf16 weight matrix in half precision (exact unless a weight is below 2^-14 in magnitude)
__global__ void transpose_bf16_to_f16(const uint16_t* __restrict__ w, uint16_t* __restrict__ wt, uint32_t rows, uint32_t cols) {
  __shared__ uint16_t tile[32][33];
  const uint32_t bx = blockIdx.x * 32, by = blockIdx.y * 32;
  for (uint32_t yy = threadIdx.y; yy < 32; yy += 8)
    if (by + yy < rows && bx + threadIdx.x < cols) tile[yy][threadIdx.x] = f2h(bf2f(w[static_cast<uint64_t>(by + yy) * cols + bx + threadIdx.x]));
  __syncthreads();
  for (uint32_t yy = threadIdx.y; yy < 32; yy += 8)
    if (bx + yy < cols && by + threadIdx.x < rows) wt[static_cast<uint64_t>(bx + yy) * rows + by + threadIdx.x] = tile[threadIdx.x][yy];
}

}  // namespace

template <typename TX, typename TY>
static void layernorm_dispatch(const HstuDims& hd, const void* x, const float* g, const float* b, const void* gate,
                               void* y, uint32_t N, hipStream_t stream) {
  const TX* xs = static_cast<const TX*>(x);
  const TY* gs = static_cast<const TY*>(gate);
  TY* ys = static_cast<TY*>(y);
  const uint32_t chunks = hd.d / 8;
  const dim3 block(256);
#define RACER_LN(LPR, KC)                                                                                        \
  hipLaunchKernelGGL((layernorm_rows<TX, TY, LPR, KC>), dim3((N + 256 / LPR - 1) / (256 / LPR)), block, 0, stream, \
                     xs, g, b, gs, ys, N, hd.d, hd.eps)
  if (chunks <= 8) RACER_LN(8, 1);
  else if (chunks <= 16) RACER_LN(16, 1);
  else if (chunks <= 32) RACER_LN(32, 1);
  else if (chunks <= 64) RACER_LN(64, 1);
  else RACER_LN(64, 2);
#undef RACER_LN
}

// bf16 models: the first LayerNorm of a layer reads the bf16 residual stream, the second one the half-precision
// attention output and gate; both write half precision (the next product's operand)
hipError_t launch_layernorm(const HstuDims& hd, const void* x, const float* g, const float* b, const void* gate,
                            void* y, uint32_t N, hipStream_t stream) {
  if (N == 0) return hipSuccess;
  if (hd.elem != 1) layernorm_dispatch<float, float>(hd, x, g, b, gate, y, N, stream);
  else if (gate) layernorm_dispatch<half_t, half_t>(hd, x, g, b, gate, y, N, stream);
  else layernorm_dispatch<bf16_t, half_t>(hd, x, g, b, gate, y, N, stream);
  return hipGetLastError();
}

bool layer_halves_fused(const HstuDims& hd) { return hd.elem == 1 && (hd.d == 128 || hd.d == 256); }

hipError_t launch_layer_front_fused(const HstuDims& hd, uint32_t layer, const void* x, const float* ln_g,
                                    const float* ln_b, const void* w1t, const float* b1, void* u, void* q,
                                    const KvView& kv, const StepLists& sl, const int32_t* page_tables,
                                    hipStream_t stream) {
  if (sl.N == 0) return hipSuccess;
  if (!layer_halves_fused(hd)) return hipErrorInvalidValue;
  LayerHalfArgs a{};
  a.hd = hd;
  a.layer = layer;
  a.a_in = static_cast<const uint16_t*>(x);
  a.ln_g = ln_g;
  a.ln_b = ln_b;
  a.wt = static_cast<const uint16_t*>(w1t);
  a.bias = b1;
  a.u = static_cast<uint16_t*>(u);
  a.q = static_cast<uint16_t*>(q);
  a.kv = kv;
  a.reqs = sl.reqs;
  a.page_tables = page_tables;
  a.row_tiles = sl.row_tiles;
  // A block sweeps all 4 d output columns of its rows, so that the rows are read and normalised once; only a launch
  // with too few row tiles to fill a third of the chip's block slots is cut into the column halves U|V and Q|K.
  const uint32_t kSplit = sl.n_row_tiles >= 256 ? 1 : 2;
  a.col_blocks_per_split = 4 * hd.d / 32 / kSplit;
  if (a.col_blocks_per_split % 2 != 0) return hipErrorInvalidValue;  // the sweep takes column tiles in pairs
  const dim3 grid(sl.n_row_tiles, kSplit), block(256);
  if (hd.d == 256) hipLaunchKernelGGL((layer_half_fused<256, true, 4>), grid, block, 0, stream, a);
  else hipLaunchKernelGGL((layer_half_fused<128, true, 4>), grid, block, 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_layer_back_fused(const HstuDims& hd, const void* o, const void* u, const float* ln_g,
                                   const float* ln_b, const void* w2t, const float* b2, const void* x, void* y,
                                   const StepLists& sl, hipStream_t stream) {
  if (sl.N == 0) return hipSuccess;
  if (!layer_halves_fused(hd)) return hipErrorInvalidValue;
  LayerHalfArgs a{};
  a.hd = hd;
  a.a_in = static_cast<const uint16_t*>(o);
  a.gate = static_cast<const uint16_t*>(u);
  a.ln_g = ln_g;
  a.ln_b = ln_b;
  a.wt = static_cast<const uint16_t*>(w2t);
  a.bias = b2;
  a.resid = static_cast<const uint16_t*>(x);
  a.y = static_cast<uint16_t*>(y);
  a.row_tiles = sl.row_tiles;
  a.col_blocks_per_split = hd.d / 32;
  if (a.col_blocks_per_split % 2 != 0) return hipErrorInvalidValue;  // the sweep takes column tiles in pairs
  const dim3 grid(sl.n_row_tiles, 1), block(256);
  if (hd.d == 256) hipLaunchKernelGGL((layer_half_fused<256, false, 4>), grid, block, 0, stream, a);
  else hipLaunchKernelGGL((layer_half_fused<128, false, 4>), grid, block, 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_gemm_front(const HstuDims& hd, uint32_t layer, const void* xn, const void* w1, const float* b1,
                             void* u, void* q, const KvView& kv, const StepLists& sl, const int32_t* page_tables,
                             hipStream_t stream) {
  if (sl.N == 0) return hipSuccess;
  if (hd.elem == 1) {
    hipLaunchKernelGGL(gemm_front_bf16, dim3(sl.n_row_tiles, 4 * hd.d / 64), dim3(256), 0, stream, hd, layer,
                       static_cast<const uint16_t*>(xn), static_cast<const uint16_t*>(w1), b1, static_cast<uint16_t*>(u),
                       static_cast<uint16_t*>(q), kv, sl.reqs, sl.row_tiles, page_tables);
  } else {
    FrontEpilogue<float> epi{hd, layer, b1, static_cast<float*>(u), static_cast<float*>(q), kv, sl.reqs, sl.row_req, page_tables};
    const uint64_t total = static_cast<uint64_t>(sl.N) * 4 * hd.d;
    hipLaunchKernelGGL(gemm_f32_simple<FrontEpilogue<float>>, dim3(static_cast<uint32_t>((total + 255) / 256)), dim3(256),
                       0, stream, static_cast<const float*>(xn), static_cast<const float*>(w1), sl.N, hd.d, 4 * hd.d, epi);
  }
  return hipGetLastError();
}

hipError_t launch_gemm_back(const HstuDims& hd, const void* g, const void* w2, const float* b2, const void* x,
                            void* y, uint32_t N, hipStream_t stream) {
  if (N == 0) return hipSuccess;
  if (hd.elem == 1) {
    BackEpilogue<bf16_t> epi{hd.d, b2, static_cast<const bf16_t*>(x), static_cast<bf16_t*>(y)};
    hipLaunchKernelGGL(gemm_bf16_mfma<BackEpilogue<bf16_t>>, dim3((N + 127) / 128, hd.d / 64), dim3(256), 0, stream,
                       static_cast<const uint16_t*>(g), static_cast<const uint16_t*>(w2), N, hd.d, epi);
  } else {
    BackEpilogue<float> epi{hd.d, b2, static_cast<const float*>(x), static_cast<float*>(y)};
    const uint64_t total = static_cast<uint64_t>(N) * hd.d;
    hipLaunchKernelGGL(gemm_f32_simple<BackEpilogue<float>>, dim3(static_cast<uint32_t>((total + 255) / 256)), dim3(256), 0,
                       stream, static_cast<const float*>(g), static_cast<const float*>(w2), N, hd.d, hd.d, epi);
  }
  return hipGetLastError();
}

hipError_t launch_attention(const HstuDims& hd, uint32_t layer, const void* q, const float* pos, const float* time,
                            const KvView& kv, const StepLists& sl, const int32_t* page_tables, const int64_t* ts,
                            void* o, bool o_half, hipStream_t stream) {
  if (sl.N == 0) return hipSuccess;
  if (hd.elem == 1) {
    if (sl.q_block != 128) return hipErrorInvalidValue;  // the work items are cut for 128-query blocks
    if (o_half)
      hipLaunchKernelGGL((attention_bf16_mfma<1, true>), dim3(sl.n_work), dim3(256), 0, stream, hd, layer,
                         static_cast<const uint16_t*>(q), pos, time, kv, sl.reqs, sl.items, sl.work, sl.partials, page_tables,
                         reinterpret_cast<const long long*>(ts), static_cast<uint16_t*>(o));
    else
      hipLaunchKernelGGL((attention_bf16_mfma<1, false>), dim3(sl.n_work), dim3(256), 0, stream, hd, layer,
                         static_cast<const uint16_t*>(q), pos, time, kv, sl.reqs, sl.items, sl.work, sl.partials, page_tables,
                         reinterpret_cast<const long long*>(ts), static_cast<uint16_t*>(o));
  } else {
    const uint32_t items = sl.N * hd.H;
    hipLaunchKernelGGL(attention_f32, dim3((items + 3) / 4), dim3(256), 0, stream, hd, layer,
                       static_cast<const float*>(q), pos, time, kv, sl.reqs, sl.row_req, sl.N, page_tables,
                       reinterpret_cast<const long long*>(ts), static_cast<float*>(o));
  }
  return hipGetLastError();
}

hipError_t launch_attention_reduce(const HstuDims& hd, const StepLists& sl, void* o, bool o_half, hipStream_t stream) {
  if (hd.elem != 1 || sl.n_groups == 0) return hipSuccess;
  hipLaunchKernelGGL(attention_reduce, dim3(sl.n_groups * hd.H, (sl.q_block * 16 + 255) / 256), dim3(256), 0, stream, hd,
                     sl.q_block, sl.reqs, sl.groups, sl.partials, static_cast<uint16_t*>(o), o_half ? 1u : 0u);
  return hipGetLastError();
}

hipError_t launch_check_timestamps(ReqDev* reqs, uint32_t B, uint32_t max_seq, const int64_t* ts,
                                   unsigned long long* counters, hipStream_t stream) {
  if (B == 0 || max_seq < 2) return hipSuccess;
  hipLaunchKernelGGL(check_timestamps, dim3((max_seq - 1 + kTsChunk - 1) / kTsChunk, B < 65535 ? B : 65535), dim3(256), 0,
                     stream, reqs, B, reinterpret_cast<const long long*>(ts), counters);
  return hipGetLastError();
}

hipError_t launch_scale_bias(const float* in, float* out, uint64_t n, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  const uint32_t blocks = static_cast<uint32_t>((n + 255) / 256 < 8192 ? (n + 255) / 256 : 8192);
  hipLaunchKernelGGL(scale_f32, dim3(blocks), dim3(256), 0, stream, in, out, n, kLog2e);
  return hipGetLastError();
}

hipError_t launch_scale_q(const void* in, void* out, uint64_t n, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  const uint32_t blocks = static_cast<uint32_t>((n + 255) / 256 < 8192 ? (n + 255) / 256 : 8192);
  hipLaunchKernelGGL(scale_bf16, dim3(blocks), dim3(256), 0, stream, static_cast<const uint16_t*>(in),
                     static_cast<uint16_t*>(out), n, kLog2e);
  return hipGetLastError();
}

hipError_t launch_transpose_weights(const void* w, void* wt, uint32_t rows, uint32_t cols, uint32_t elem,
                                    hipStream_t stream) {
  const dim3 grid((cols + 31) / 32, (rows + 31) / 32), block(32, 8);
  if (elem == 1)  // bf16 in, half precision out
    hipLaunchKernelGGL(transpose_bf16_to_f16, grid, block, 0, stream, static_cast<const uint16_t*>(w),
                       static_cast<uint16_t*>(wt), rows, cols);
  else
    hipLaunchKernelGGL(transpose_kernel<float>, grid, block, 0, stream, static_cast<const float*>(w),
                       static_cast<float*>(wt), rows, cols);
  return hipGetLastError();
}

}  // namespace racer
