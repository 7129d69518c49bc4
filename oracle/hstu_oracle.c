/*
 * Oracle, part 2: naive HSTU layer stack over a paged KV store, fp64
 * arithmetic.  Test infrastructure only (see racer_oracle.h).
 *
 * The paper (Sec. II-A, Sec. II-B "Request serving") says what the stage is:
 * stacked self-attention blocks over a user's history that reuse resident KV
 * state; it prints no equations.  The layer below is the published HSTU form:
 *   Xn = LayerNorm(X)
 *   [U | V | Q | K] = SiLU(Xn W1 + b1)               (pointwise projection)
 *   O_i = (1/n) sum_{j<=p_i} SiLU(<q_i,k_j> + rab(p_i, j)) v_j   (per head)
 *   Y = X + (LayerNorm(O) * U) W2 + b2               (gated transformation)
 * with rab(p, j) = pos[min(p-j, n_pos-1)] + time[bucket(ts_p - ts_j)] and
 * bucket(D) = min(floor(log2(max(D,1))), n_time-1) taken in integers.
 * KV bytes per token are 2*L*d*elem, which reproduces the paper's 60-184 MB
 * per user at 5K-15K tokens (Sec. V-E, hardware generalisability).
 * One page holds page_tokens tokens of every layer:
 * [layer][K|V][head][token][d_h].  K and V are rounded to the storage type
 * when stored, because later steps read them back from the cache; nothing
 * else is rounded.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#include "racer_oracle.h"

static int omp_in_parallel_(void) {
#ifdef _OPENMP
  return omp_in_parallel();
#else
  return 1;
#endif
}

uint16_t orc_f32_to_bf16_bits(float x) {
  uint32_t u;
  memcpy(&u, &x, 4);
  if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) return (uint16_t)((u >> 16) | 0x40);
  /* round to nearest, ties to even, on the 16 dropped bits */
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7FFFu + lsb;
  return (uint16_t)(u >> 16);
}

float orc_bf16_bits_to_f32(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

float orc_round_bf16(float x) { return orc_bf16_bits_to_f32(orc_f32_to_bf16_bits(x)); }

double orc_silu(double x) { return x / (1.0 + exp(-x)); }

uint32_t orc_time_bucket(int64_t dt, uint32_t n_time) {
  uint32_t b = 0;
  while (dt > 1) { /* floor(log2(dt)) by halving; dt <= 1 gives bucket 0 */
    dt >>= 1;
    b++;
  }
  return b < n_time - 1 ? b : n_time - 1;
}

void orc_layernorm(const double* x, const float* g, const float* b, uint32_t d, double eps,
                   double* y) {
  double mean = 0.0;
  for (uint32_t c = 0; c < d; ++c) mean += x[c];
  mean /= d;
  double var = 0.0;
  for (uint32_t c = 0; c < d; ++c) var += (x[c] - mean) * (x[c] - mean);
  var /= d; /* population variance */
  double r = 1.0 / sqrt(var + eps);
  for (uint32_t c = 0; c < d; ++c) y[c] = (x[c] - mean) * r * (double)g[c] + (double)b[c];
}

uint64_t orc_kv_elems_per_page(const orc_hstu_cfg* cfg) {
  return (uint64_t)cfg->page_tokens * 2 * cfg->L * cfg->d;
}

uint64_t orc_kv_offset(const orc_hstu_cfg* cfg, uint64_t page, uint32_t layer, uint32_t kv,
                       uint32_t head, uint32_t tok) {
  uint32_t dh = cfg->d / cfg->H;
  uint64_t in_page = ((((uint64_t)layer * 2 + kv) * cfg->H + head) * cfg->page_tokens + tok) * dh;
  return page * orc_kv_elems_per_page(cfg) + in_page;
}

void orc_attn_paged(const orc_hstu_cfg* cfg, uint32_t layer, const float* pos, const float* time,
                    uint32_t P, uint32_t T, const int32_t* pages, const int64_t* ts,
                    const float* kv_mem, const double* q, double* o) {
  const uint32_t d = cfg->d, H = cfg->H, dh = d / H, pt = cfg->page_tokens;
  /* (head, query) pairs are independent of one another; a caller that is not itself inside a
   * parallel region (one request at a time) spreads them over the threads */
#pragma omp parallel for collapse(2) schedule(dynamic, 8) if (!omp_in_parallel_())
  for (uint32_t h = 0; h < H; ++h) {
    for (uint32_t i = 0; i < T; ++i) {
      const uint32_t p = P + i;
      double* orow = o + (uint64_t)i * d + h * dh;
      for (uint32_t c = 0; c < dh; ++c) orow[c] = 0.0;
      for (uint32_t j = 0; j <= p; ++j) { /* keys after p contribute nothing */
        const float* k = kv_mem + orc_kv_offset(cfg, (uint64_t)pages[j / pt], layer, 0, h, j % pt);
        const float* v = kv_mem + orc_kv_offset(cfg, (uint64_t)pages[j / pt], layer, 1, h, j % pt);
        double s = 0.0;
        for (uint32_t c = 0; c < dh; ++c) s += q[(uint64_t)i * d + h * dh + c] * (double)k[c];
        uint32_t rel = p - j;
        if (rel > cfg->n_pos - 1) rel = cfg->n_pos - 1;
        s += (double)pos[(uint64_t)h * cfg->n_pos + rel];
        s += (double)time[(uint64_t)h * cfg->n_time + orc_time_bucket(ts[p] - ts[j], cfg->n_time)];
        double a = orc_silu(s) / cfg->n_scale;
        for (uint32_t c = 0; c < dh; ++c) orow[c] += a * (double)v[c];
      }
    }
  }
}

static void step_one_request(const orc_hstu_cfg* cfg, const orc_hstu_weights* w,
                             const orc_hstu_req* rq, const int32_t* page_tables, float* kv_mem,
                             const float* x_in, const int64_t* ts_all, double* out) {
  const uint32_t d = cfg->d, H = cfg->H, dh = d / H, pt = cfg->page_tokens, L = cfg->L;
  const uint32_t P = rq->prefix_len, T = rq->new_len;
  if (T == 0) return;
  const int32_t* pages = page_tables + rq->page_table_off;
  const int64_t* ts = ts_all + rq->ts_off;
  double* X = (double*)malloc(sizeof(double) * T * d);
  double* U = (double*)malloc(sizeof(double) * T * d);
  double* Q = (double*)malloc(sizeof(double) * T * d);
  double* O = (double*)malloc(sizeof(double) * T * d);
  for (uint64_t e = 0; e < (uint64_t)T * d; ++e) X[e] = (double)x_in[rq->x_off * d + e];

  for (uint32_t l = 0; l < L; ++l) {
    const float* w1 = w->w1 + (uint64_t)l * d * 4 * d;
    const float* b1 = w->b1 + (uint64_t)l * 4 * d;
    const float* w2 = w->w2 + (uint64_t)l * d * d;
    const float* b2 = w->b2 + (uint64_t)l * d;
    /* pointwise projection, then K,V of the new tokens go into the pages (tokens are independent
     * here: each has scratch of its own) */
#pragma omp parallel for schedule(static) if (!omp_in_parallel_())
    for (uint32_t i = 0; i < T; ++i) {
      double Xn[d], Z[4 * d];
      orc_layernorm(X + (uint64_t)i * d, w->ln1_g + (uint64_t)l * d, w->ln1_b + (uint64_t)l * d, d,
                    cfg->eps, Xn);
      for (uint32_t c = 0; c < 4 * d; ++c) {
        double acc = 0.0;
        for (uint32_t k = 0; k < d; ++k) acc += Xn[k] * (double)w1[(uint64_t)k * 4 * d + c];
        Z[c] = orc_silu(acc + (double)b1[c]);
      }
      const uint32_t pos = P + i;
      for (uint32_t c = 0; c < d; ++c) {
        U[(uint64_t)i * d + c] = Z[c];
        Q[(uint64_t)i * d + c] = Z[2 * d + c];
        float vv = (float)Z[d + c], kk = (float)Z[3 * d + c];
        if (cfg->store_bf16) {
          vv = orc_round_bf16(vv);
          kk = orc_round_bf16(kk);
        }
        uint32_t h = c / dh, e = c % dh;
        kv_mem[orc_kv_offset(cfg, (uint64_t)pages[pos / pt], l, 0, h, pos % pt) + e] = kk;
        kv_mem[orc_kv_offset(cfg, (uint64_t)pages[pos / pt], l, 1, h, pos % pt) + e] = vv;
      }
    }
    orc_attn_paged(cfg, l, w->pos + (uint64_t)l * H * cfg->n_pos,
                   w->time + (uint64_t)l * H * cfg->n_time, P, T, pages, ts, kv_mem, Q, O);
    /* gated transformation with residual */
#pragma omp parallel for schedule(static) if (!omp_in_parallel_())
    for (uint32_t i = 0; i < T; ++i) {
      double G[d], Xn[d];
      orc_layernorm(O + (uint64_t)i * d, w->ln2_g + (uint64_t)l * d, w->ln2_b + (uint64_t)l * d, d,
                    cfg->eps, G);
      for (uint32_t c = 0; c < d; ++c) G[c] *= U[(uint64_t)i * d + c];
      for (uint32_t c = 0; c < d; ++c) {
        double acc = 0.0;
        for (uint32_t k = 0; k < d; ++k) acc += G[k] * (double)w2[(uint64_t)k * d + c];
        Xn[c] = X[(uint64_t)i * d + c] + acc + (double)b2[c];
      }
      memcpy(X + (uint64_t)i * d, Xn, sizeof(double) * d);
    }
  }
  memcpy(out + rq->x_off * d, X, sizeof(double) * T * d);
  free(O);
  free(Q);
  free(U);
  free(X);
}

int orc_hstu_step(const orc_hstu_cfg* cfg, const orc_hstu_weights* w, const orc_hstu_req* reqs,
                  uint32_t B, const int32_t* page_tables, float* kv_mem, uint64_t kv_pages,
                  const float* x_in, const int64_t* ts, double* out, int threads) {
  if (cfg->H == 0 || cfg->d % cfg->H != 0 || cfg->page_tokens == 0) return ORC_EINVAL;
  if (cfg->n_pos == 0 || cfg->n_time == 0) return ORC_EINVAL;
  for (uint32_t r = 0; r < B; ++r) { /* every request's table must cover prefix + new tokens */
    uint32_t np = (reqs[r].prefix_len + reqs[r].new_len + cfg->page_tokens - 1) / cfg->page_tokens;
    for (uint32_t k = 0; k < np; ++k) {
      int32_t pg = page_tables[reqs[r].page_table_off + k];
      if (pg < 0 || (uint64_t)pg >= kv_pages) return ORC_ERANGE;
    }
  }
  /* requests own disjoint pages, so they are independent of one another */
#ifdef _OPENMP
  if (threads > 0) omp_set_num_threads(threads);
#else
  (void)threads;
#endif
  /* (a single request is served by the threads inside it instead) */
#pragma omp parallel for schedule(dynamic, 1) if (B > 1)
  for (int r = 0; r < (int)B; ++r)
    step_one_request(cfg, w, &reqs[r], page_tables, kv_mem, x_in, ts, out);
  return ORC_OK;
}

int orc_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
