/*
 * CPU oracle for the RACER hot path (test infrastructure, not product code).
 *
 * Plain, slow, single-purpose C: an exact simulator of the shared EMB/KV page
 * pool with its set-associative LRU embedding cache, and a naive HSTU layer
 * stack evaluated in fp64.  Only tests, the smoke check and the cpu_baseline
 * leg of the benchmark may call it; the GPU library shares no code with it.
 *
 * What each part follows:
 *   pool / KV side  - paper Sec. IV-B ("Non-Disruptive Memory Allocation
 *                     Adjustment"): one paged space, movable EMB:KV boundary,
 *                     KV blocks immobile, LRU reclaim of cold unpinned user
 *                     blocks, deferral when reclaimable pages run out,
 *                     alpha in [0.1, 0.9] (Sec. IV-A, Eq. 6).
 *   EMB cache       - Sec. IV-B "contiguous LRU-managed slab backed by
 *                     page-granularity allocation"; set/way geometry, hash,
 *                     batch semantics and shrink rule are this build's
 *                     readings (the paper gives none).
 *   HSTU layer      - Sec. II-A names the model only; the layer equations are
 *                     the published HSTU form (pointwise projection, pointwise
 *                     SiLU attention with relative bias, gated output).
 *
 * Parity pins: every function below is pinned by tests/test_oracle_*.py
 * (brute force, textbook LRU, closed forms, invariants).  End-to-end output
 * values have no printed example in the paper: "parity unpinned" by the paper,
 * pinned only by those properties.
 */
#ifndef RACER_ORACLE_H
#define RACER_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ORC_OK 0
#define ORC_DEFERRED 1
#define ORC_NOT_FOUND 2
#define ORC_EINVAL (-22)
#define ORC_ENOMEM (-12)
#define ORC_ERANGE (-34)
#define ORC_EBUSY (-16)

#define ORC_TAG_EMPTY 0xFFFFFFFFu

typedef struct orc_pool orc_pool;

typedef struct {
  uint64_t lookups, hits, misses, unique_misses, inserted, evicted, bypassed, invalid_ids;
  uint64_t shrink_evicted, shrink_moved;
  uint64_t pages_total, pages_emb, pages_kv_used, pages_kv_free;
  uint64_t seqs_resident, seqs_evicted;
  uint64_t batch;
} orc_stats;

/* ---- pool + KV side ---------------------------------------------------- */
orc_pool* orc_pool_create(uint64_t n_pages, uint32_t page_tokens, uint32_t slots_per_page,
                          uint32_t w_max, double emb_frac0);
void orc_pool_destroy(orc_pool* p);
int orc_pool_set_split(orc_pool* p, double emb_frac, double* achieved);
int orc_pool_stats(const orc_pool* p, orc_stats* out);
uint64_t orc_pool_num_sets(const orc_pool* p);
uint32_t orc_pool_ways(const orc_pool* p, uint64_t set);
/* copies: emb_pages[n_emb] (logical -> physical), page owner bytes [n_pages]
 * (0 free, 1 EMB, 2 KV), tags/stamps [S][w_max]. NULL pointers are skipped. */
int orc_pool_dump(const orc_pool* p, int64_t* emb_pages, uint8_t* owner, uint32_t* tags,
                  uint32_t* stamps);
/* physical slot index (page * slots_per_page + offset) of way w of set s */
int64_t orc_pool_slot_of(const orc_pool* p, uint64_t set, uint32_t way);

int orc_kv_seq_reserve(orc_pool* p, uint64_t key, uint32_t tokens, int32_t* pages_out,
                       uint32_t cap, uint32_t* n_pages_out);
int orc_kv_seq_lookup(const orc_pool* p, uint64_t key, uint32_t* tokens, int32_t* pages_out,
                      uint32_t cap, uint32_t* n_pages_out);
int orc_kv_seq_pin(orc_pool* p, uint64_t key);
int orc_kv_seq_unpin(orc_pool* p, uint64_t key);
int orc_kv_seq_release(orc_pool* p, uint64_t key);

/* ---- EMB cache ----------------------------------------------------------
 * table: host rows [rows][d], elem 0 = fp32, 1 = bf16 (uint16 bit patterns).
 * out: [n/bag][d] in the same element type. hit may be NULL. */
uint64_t orc_emb_set_of(const orc_pool* p, int64_t id);
int orc_emb_lookup(orc_pool* p, const int64_t* ids, uint64_t n, uint32_t bag, const void* table,
                   uint64_t rows, uint32_t d, int elem, void* out, uint8_t* hit);
/* refill of empty ways with the given ids (hottest first); never evicts; *inserted may be NULL */
int orc_emb_refill(orc_pool* p, const int64_t* ids, uint64_t n, uint64_t rows, uint64_t* inserted);

/* ---- HSTU ---------------------------------------------------------------
 * All tensors are passed as fp32 arrays whose values are already representable
 * in the storage type; arithmetic is fp64. */
typedef struct {
  uint32_t L, d, H;
  uint32_t page_tokens;
  uint32_t n_pos, n_time;
  double n_scale; /* the "n" of the 1/n attention scaling */
  double eps;
  int store_bf16; /* K,V rows are rounded to bf16 (1) or fp32 (0) when stored */
} orc_hstu_cfg;

typedef struct {
  uint32_t prefix_len, new_len;
  uint64_t page_table_off; /* into page_tables[] */
  uint64_t ts_off;         /* into ts[], prefix_len+new_len entries */
  uint64_t x_off;          /* row offset into x_in / out */
} orc_hstu_req;

/* per-layer weights, all layers concatenated:
 * ln1_g[L][d] ln1_b[L][d] w1[L][d][4d] b1[L][4d] ln2_g[L][d] ln2_b[L][d]
 * w2[L][d][d] b2[L][d] pos[L][H][n_pos] time[L][H][n_time] */
typedef struct {
  const float *ln1_g, *ln1_b, *w1, *b1, *ln2_g, *ln2_b, *w2, *b2, *pos, *time;
} orc_hstu_weights;

float orc_round_bf16(float x);
uint16_t orc_f32_to_bf16_bits(float x);
float orc_bf16_bits_to_f32(uint16_t b);
double orc_silu(double x);
uint32_t orc_time_bucket(int64_t dt, uint32_t n_time);
void orc_layernorm(const double* x, const float* g, const float* b, uint32_t d, double eps,
                   double* y);

/* attention of one layer for one request, Q given ([T][d] fp64, head-major columns),
 * K,V read from kv_mem through the page table. o: [T][d]. */
void orc_attn_paged(const orc_hstu_cfg* cfg, uint32_t layer, const float* pos, const float* time,
                    uint32_t P, uint32_t T, const int32_t* pages, const int64_t* ts,
                    const float* kv_mem, const double* q, double* o);

/* whole step: all layers, all requests. kv_mem is read (prefix) and written
 * (new tokens). out: [N][d] fp64. threads: OpenMP threads over requests
 * (0 = library default). */
int orc_hstu_step(const orc_hstu_cfg* cfg, const orc_hstu_weights* w, const orc_hstu_req* reqs,
                  uint32_t B, const int32_t* page_tables, float* kv_mem, uint64_t kv_pages,
                  const float* x_in, const int64_t* ts, double* out, int threads);

uint64_t orc_kv_elems_per_page(const orc_hstu_cfg* cfg);
/* element offset inside kv_mem of (page, layer, kv(0=K,1=V), head, token-in-page, 0) */
uint64_t orc_kv_offset(const orc_hstu_cfg* cfg, uint64_t page, uint32_t layer, uint32_t kv,
                       uint32_t head, uint32_t tok);

int orc_max_threads(void);

#ifdef __cplusplus
}
#endif
#endif
