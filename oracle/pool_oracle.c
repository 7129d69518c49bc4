/*
 * Oracle, part 1: the shared page pool, the KV sequence table and the EMB
 * set-associative LRU cache, simulated exactly on the host.  Test
 * infrastructure only (see racer_oracle.h).
 *
 * Paper Sec. IV-B fixes: one paged space of N pages; M_emb = alpha*M,
 * M_kv = (1-alpha)*M (Sec. IV-A problem formulation); KV = paged block pool
 * with a free list and page tables, user-granularity LRU reclaim that is
 * metadata-only, pinned in-flight blocks, deferral of an EMB expansion that
 * cannot be served; EMB = LRU slab with page-granular allocation; alpha kept
 * in [0.1, 0.9] (Eq. 6).
 *
 * Readings where the paper is silent (all deterministic):
 *   - page allocation order: lowest-numbered free page first;
 *   - target page count: llround(alpha * N) (round half away from zero);
 *   - cache geometry: w_max ways, S = N*slots_per_page/w_max sets; way layer
 *     w = slot w of every set = G = N/w_max consecutive logical EMB pages, so
 *     slot (w, s) sits in logical page w*G + s/slots_per_page at offset
 *     s % slots_per_page; with n_emb logical pages a set has n_emb/G ways,
 *     plus one if s < (n_emb % G)*slots_per_page.  Set index never changes
 *     with the split;
 *   - hash: set = ((uint64)id * 0x9E3779B97F4A7C15 >> 32) % S;
 *   - batch semantics: hit = resident at batch start; every lookup of a
 *     missing id is a miss; unique misses are inserted in first-occurrence
 *     order, victim = lowest empty way, else least (stamp, way) among ways not
 *     touched in this batch, else the id bypasses the cache;
 *   - shrink: per set evict empties first, then least (stamp, way); surviving
 *     entries in removed ways move, in way order, into the vacated lower ways
 *     in ascending order; entries already below the new way count stay.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include "racer_oracle.h"

typedef struct {
  uint64_t key;
  uint32_t tokens;
  uint32_t n_pages;
  uint32_t cap_pages;
  int32_t* pages;
  uint64_t stamp;
  uint32_t pins;
  int live;
} orc_seq;

struct orc_pool {
  uint64_t n_pages;
  uint32_t page_tokens, spp, w_max;
  uint64_t S, G;
  uint8_t* owner; /* 0 free, 1 EMB, 2 KV */
  uint64_t free_count;
  uint64_t free_hint; /* no free page has an id below this */
  int64_t* emb_pages;
  uint64_t n_emb;
  uint32_t* tag;
  uint32_t* stamp;
  uint32_t t;
  orc_seq* seqs;
  uint64_t n_seqs, cap_seqs;
  uint64_t kv_clock;
  orc_stats st;
};

static int is_pow2(uint32_t x) { return x && !(x & (x - 1)); }

orc_pool* orc_pool_create(uint64_t n_pages, uint32_t page_tokens, uint32_t slots_per_page,
                          uint32_t w_max, double emb_frac0) {
  if (n_pages == 0 || page_tokens == 0 || slots_per_page == 0) return NULL;
  if (!is_pow2(w_max) || w_max > 32) return NULL;
  if (n_pages % w_max != 0) return NULL;
  if (!(emb_frac0 >= 0.0 && emb_frac0 <= 1.0)) return NULL;
  if (n_pages > 0x7FFFFFFFull) return NULL;
  orc_pool* p = (orc_pool*)calloc(1, sizeof(orc_pool));
  p->n_pages = n_pages;
  p->page_tokens = page_tokens;
  p->spp = slots_per_page;
  p->w_max = w_max;
  p->G = n_pages / w_max;
  p->S = p->G * slots_per_page;
  p->owner = (uint8_t*)calloc(n_pages, 1);
  p->emb_pages = (int64_t*)malloc(sizeof(int64_t) * n_pages);
  p->tag = (uint32_t*)malloc(sizeof(uint32_t) * p->S * w_max);
  p->stamp = (uint32_t*)calloc(p->S * w_max, sizeof(uint32_t));
  for (uint64_t i = 0; i < p->S * w_max; ++i) p->tag[i] = ORC_TAG_EMPTY;
  p->free_count = n_pages;
  p->free_hint = 0;
  uint64_t n0 = (uint64_t)llround(emb_frac0 * (double)n_pages);
  for (uint64_t i = 0; i < n0; ++i) { /* lowest-numbered pages first */
    p->owner[i] = 1;
    p->emb_pages[i] = (int64_t)i;
  }
  p->n_emb = n0;
  p->free_count -= n0;
  p->free_hint = n0;
  return p;
}

void orc_pool_destroy(orc_pool* p) {
  if (!p) return;
  for (uint64_t i = 0; i < p->n_seqs; ++i) free(p->seqs[i].pages);
  free(p->seqs);
  free(p->owner);
  free(p->emb_pages);
  free(p->tag);
  free(p->stamp);
  free(p);
}

uint64_t orc_pool_num_sets(const orc_pool* p) { return p->S; }

static uint32_t ways_at(const orc_pool* p, uint64_t n_emb, uint64_t s) {
  uint64_t full = n_emb / p->G;
  uint64_t rem = n_emb % p->G;
  return (uint32_t)(full + (s < rem * p->spp ? 1 : 0));
}

uint32_t orc_pool_ways(const orc_pool* p, uint64_t set) { return ways_at(p, p->n_emb, set); }

int64_t orc_pool_slot_of(const orc_pool* p, uint64_t set, uint32_t way) {
  if (set >= p->S || way >= ways_at(p, p->n_emb, set)) return -1;
  uint64_t logical = (uint64_t)way * p->G + set / p->spp;
  return p->emb_pages[logical] * (int64_t)p->spp + (int64_t)(set % p->spp);
}

/* lowest-numbered free page, or -1 */
static int64_t take_free_page(orc_pool* p, uint8_t new_owner) {
  for (uint64_t i = p->free_hint; i < p->n_pages; ++i) {
    if (p->owner[i] == 0) {
      p->owner[i] = new_owner;
      p->free_count--;
      p->free_hint = i + 1;
      return (int64_t)i;
    }
  }
  return -1;
}

static void give_back_page(orc_pool* p, int64_t page) {
  p->owner[page] = 0;
  p->free_count++;
  if ((uint64_t)page < p->free_hint) p->free_hint = (uint64_t)page;
}

static orc_seq* find_seq(const orc_pool* p, uint64_t key) {
  for (uint64_t i = 0; i < p->n_seqs; ++i)
    if (p->seqs[i].live && p->seqs[i].key == key) return &p->seqs[i];
  return NULL;
}

/* the unpinned live sequence with the least (stamp, key), skipping `except` */
static orc_seq* coldest_unpinned(const orc_pool* p, const orc_seq* except) {
  orc_seq* best = NULL;
  for (uint64_t i = 0; i < p->n_seqs; ++i) {
    orc_seq* s = &p->seqs[i];
    if (!s->live || s->pins > 0 || s == except) continue;
    if (!best || s->stamp < best->stamp || (s->stamp == best->stamp && s->key < best->key))
      best = s;
  }
  return best;
}

static void drop_seq(orc_pool* p, orc_seq* s) {
  for (uint32_t i = 0; i < s->n_pages; ++i) give_back_page(p, s->pages[i]);
  s->n_pages = 0;
  s->tokens = 0;
  s->live = 0;
}

/* EMB shrink of one set from a ways to b ways (a > b) */
static void shrink_set(orc_pool* p, uint64_t s, uint32_t a, uint32_t b) {
  uint32_t* tg = p->tag + s * p->w_max;
  uint32_t* sp = p->stamp + s * p->w_max;
  uint32_t live = 0;
  for (uint32_t w = 0; w < a; ++w)
    if (tg[w] != ORC_TAG_EMPTY) live++;
  /* evict least (stamp, way) until at most b entries remain */
  while (live > b) {
    int victim = -1;
    for (uint32_t w = 0; w < a; ++w) {
      if (tg[w] == ORC_TAG_EMPTY) continue;
      if (victim < 0 || sp[w] < sp[victim]) victim = (int)w; /* ties: lowest way wins */
    }
    tg[victim] = ORC_TAG_EMPTY;
    sp[victim] = 0;
    live--;
    p->st.shrink_evicted++;
  }
  /* survivors in ways >= b move, in way order, into the empty ways < b */
  uint32_t hole = 0;
  for (uint32_t w = b; w < a; ++w) {
    if (tg[w] == ORC_TAG_EMPTY) continue;
    while (tg[hole] != ORC_TAG_EMPTY) hole++;
    tg[hole] = tg[w];
    sp[hole] = sp[w];
    tg[w] = ORC_TAG_EMPTY;
    sp[w] = 0;
    p->st.shrink_moved++;
  }
}

int orc_pool_set_split(orc_pool* p, double emb_frac, double* achieved) {
  if (!(emb_frac >= 0.1 && emb_frac <= 0.9)) return ORC_EINVAL;
  uint64_t target = (uint64_t)llround(emb_frac * (double)p->n_pages);
  int rc = ORC_OK;
  if (target > p->n_emb) {
    uint64_t need = target - p->n_emb;
    while (p->free_count < need) {
      orc_seq* cold = coldest_unpinned(p, NULL);
      if (!cold) break;
      drop_seq(p, cold);
      p->st.seqs_evicted++;
    }
    if (p->free_count < need) {
      need = p->free_count;
      rc = ORC_DEFERRED;
    }
    for (uint64_t k = 0; k < need; ++k) p->emb_pages[p->n_emb++] = take_free_page(p, 1);
  } else if (target < p->n_emb) {
    for (uint64_t s = 0; s < p->S; ++s) {
      uint32_t a = ways_at(p, p->n_emb, s), b = ways_at(p, target, s);
      if (b < a) shrink_set(p, s, a, b);
    }
    while (p->n_emb > target) give_back_page(p, p->emb_pages[--p->n_emb]);
  }
  if (achieved) *achieved = (double)p->n_emb / (double)p->n_pages;
  return rc;
}

int orc_pool_stats(const orc_pool* p, orc_stats* out) {
  *out = p->st;
  out->pages_total = p->n_pages;
  out->pages_emb = p->n_emb;
  out->pages_kv_free = p->free_count;
  out->pages_kv_used = p->n_pages - p->n_emb - p->free_count;
  uint64_t r = 0;
  for (uint64_t i = 0; i < p->n_seqs; ++i) r += p->seqs[i].live ? 1 : 0;
  out->seqs_resident = r;
  out->batch = p->t;
  return ORC_OK;
}

int orc_pool_dump(const orc_pool* p, int64_t* emb_pages, uint8_t* owner, uint32_t* tags,
                  uint32_t* stamps) {
  if (emb_pages) memcpy(emb_pages, p->emb_pages, sizeof(int64_t) * p->n_emb);
  if (owner) memcpy(owner, p->owner, p->n_pages);
  if (tags) memcpy(tags, p->tag, sizeof(uint32_t) * p->S * p->w_max);
  if (stamps) memcpy(stamps, p->stamp, sizeof(uint32_t) * p->S * p->w_max);
  return ORC_OK;
}

/* ---- KV sequences -------------------------------------------------------- */

static int copy_pages(const orc_seq* s, int32_t* pages_out, uint32_t cap, uint32_t* n_out) {
  if (n_out) *n_out = s->n_pages;
  if (pages_out) {
    if (cap < s->n_pages) return ORC_EINVAL;
    memcpy(pages_out, s->pages, sizeof(int32_t) * s->n_pages);
  }
  return ORC_OK;
}

int orc_kv_seq_reserve(orc_pool* p, uint64_t key, uint32_t tokens, int32_t* pages_out,
                       uint32_t cap, uint32_t* n_pages_out) {
  orc_seq* s = find_seq(p, key);
  uint32_t have = s ? s->n_pages : 0;
  uint32_t want_tokens = (s && s->tokens > tokens) ? s->tokens : tokens;
  uint32_t want = (want_tokens + p->page_tokens - 1) / p->page_tokens;
  uint64_t need = want > have ? want - have : 0;
  if (pages_out && cap < want) return ORC_EINVAL;
  /* reclaimable = free + pages of every other unpinned sequence */
  uint64_t reclaimable = p->free_count;
  for (uint64_t i = 0; i < p->n_seqs; ++i) {
    orc_seq* o = &p->seqs[i];
    if (o->live && o->pins == 0 && o != s) reclaimable += o->n_pages;
  }
  if (need > reclaimable) return ORC_ENOMEM;
  while (p->free_count < need) {
    orc_seq* cold = coldest_unpinned(p, s);
    drop_seq(p, cold);
    p->st.seqs_evicted++;
  }
  if (!s) {
    for (uint64_t i = 0; i < p->n_seqs && !s; ++i)
      if (!p->seqs[i].live) s = &p->seqs[i];
    if (!s) {
      if (p->n_seqs == p->cap_seqs) {
        p->cap_seqs = p->cap_seqs ? p->cap_seqs * 2 : 64;
        p->seqs = (orc_seq*)realloc(p->seqs, sizeof(orc_seq) * p->cap_seqs);
        memset(p->seqs + p->n_seqs, 0, sizeof(orc_seq) * (p->cap_seqs - p->n_seqs));
      }
      s = &p->seqs[p->n_seqs++];
    }
    s->key = key;
    s->tokens = 0;
    s->n_pages = 0;
    s->pins = 0;
    s->live = 1;
  }
  if (want > s->cap_pages) {
    s->pages = (int32_t*)realloc(s->pages, sizeof(int32_t) * want);
    s->cap_pages = want;
  }
  for (uint64_t k = 0; k < need; ++k) s->pages[s->n_pages++] = (int32_t)take_free_page(p, 2);
  s->tokens = want_tokens;
  s->stamp = ++p->kv_clock;
  return copy_pages(s, pages_out, cap, n_pages_out);
}

int orc_kv_seq_lookup(const orc_pool* p, uint64_t key, uint32_t* tokens, int32_t* pages_out,
                      uint32_t cap, uint32_t* n_pages_out) {
  const orc_seq* s = find_seq(p, key);
  if (!s) {
    if (tokens) *tokens = 0;
    if (n_pages_out) *n_pages_out = 0;
    return ORC_NOT_FOUND;
  }
  if (tokens) *tokens = s->tokens;
  return copy_pages(s, pages_out, cap, n_pages_out);
}

int orc_kv_seq_pin(orc_pool* p, uint64_t key) {
  orc_seq* s = find_seq(p, key);
  if (!s) return ORC_NOT_FOUND;
  s->pins++;
  s->stamp = ++p->kv_clock;
  return ORC_OK;
}

int orc_kv_seq_unpin(orc_pool* p, uint64_t key) {
  orc_seq* s = find_seq(p, key);
  if (!s) return ORC_NOT_FOUND;
  if (s->pins == 0) return ORC_EINVAL;
  s->pins--;
  return ORC_OK;
}

int orc_kv_seq_release(orc_pool* p, uint64_t key) {
  orc_seq* s = find_seq(p, key);
  if (!s) return ORC_NOT_FOUND;
  if (s->pins > 0) return ORC_EBUSY;
  drop_seq(p, s);
  return ORC_OK;
}

/* ---- EMB cache ----------------------------------------------------------- */

uint64_t orc_emb_set_of(const orc_pool* p, int64_t id) {
  uint64_t h = (uint64_t)id * 0x9E3779B97F4A7C15ull;
  return (h >> 32) % p->S;
}

typedef struct {
  int64_t id;
  uint64_t idx;
} miss_rec;

static int cmp_miss(const void* a, const void* b) {
  const miss_rec* x = (const miss_rec*)a;
  const miss_rec* y = (const miss_rec*)b;
  if (x->id != y->id) return x->id < y->id ? -1 : 1;
  if (x->idx != y->idx) return x->idx < y->idx ? -1 : 1;
  return 0;
}

int orc_emb_lookup(orc_pool* p, const int64_t* ids, uint64_t n, uint32_t bag, const void* table,
                   uint64_t rows, uint32_t d, int elem, void* out, uint8_t* hit) {
  if (bag == 0 || n % bag != 0) return ORC_EINVAL;
  if (rows >= 0xFFFFFFFFull) return ORC_EINVAL;
  p->t += 1;
  const uint32_t t = p->t;
  uint8_t* is_hit = (uint8_t*)calloc(n ? n : 1, 1);
  uint8_t* valid = (uint8_t*)calloc(n ? n : 1, 1);
  int32_t* way_of = (int32_t*)malloc(sizeof(int32_t) * (n ? n : 1));

  /* 1. hit = resident at batch start (tags are not modified in this pass) */
  for (uint64_t i = 0; i < n; ++i) {
    way_of[i] = -1;
    if (ids[i] < 0 || (uint64_t)ids[i] >= rows) {
      p->st.invalid_ids++;
      continue;
    }
    valid[i] = 1;
    uint64_t s = orc_emb_set_of(p, ids[i]);
    uint32_t nw = ways_at(p, p->n_emb, s);
    for (uint32_t w = 0; w < nw; ++w)
      if (p->tag[s * p->w_max + w] == (uint32_t)ids[i]) {
        is_hit[i] = 1;
        way_of[i] = (int32_t)w;
      }
    p->st.lookups++;
    if (is_hit[i]) p->st.hits++;
    else p->st.misses++;
  }
  /* 2. every way hit in this batch is stamped with the batch counter */
  for (uint64_t i = 0; i < n; ++i)
    if (is_hit[i]) p->stamp[orc_emb_set_of(p, ids[i]) * p->w_max + (uint32_t)way_of[i]] = t;
  if (hit) memcpy(hit, is_hit, n);

  /* 3. output rows always equal the host table's rows; bags are summed in
   *    fp32, features left to right, one round-to-nearest-even at the end */
  if (out) {
    for (uint64_t o = 0; o < n / bag; ++o) {
      for (uint32_t c = 0; c < d; ++c) {
        float acc = 0.0f;
        int any = 0;
        for (uint32_t f = 0; f < bag; ++f) {
          uint64_t i = o * bag + f;
          float v = 0.0f;
          if (valid[i]) {
            if (elem == 0) v = ((const float*)table)[(uint64_t)ids[i] * d + c];
            else v = orc_bf16_bits_to_f32(((const uint16_t*)table)[(uint64_t)ids[i] * d + c]);
          }
          if (bag == 1) acc = v;
          else if (!any) acc = v; /* first term starts the sum: 0 + v would turn -0 into +0 */
          else acc = acc + v;
          any = 1;
        }
        if (elem == 0) ((float*)out)[o * d + c] = acc;
        else ((uint16_t*)out)[o * d + c] = orc_f32_to_bf16_bits(acc);
      }
    }
  }

  /* 4. unique misses in first-occurrence order */
  uint64_t n_miss = 0;
  miss_rec* mr = (miss_rec*)malloc(sizeof(miss_rec) * (n ? n : 1));
  for (uint64_t i = 0; i < n; ++i)
    if (valid[i] && !is_hit[i]) {
      mr[n_miss].id = ids[i];
      mr[n_miss].idx = i;
      n_miss++;
    }
  qsort(mr, n_miss, sizeof(miss_rec), cmp_miss);
  uint8_t* first = (uint8_t*)calloc(n ? n : 1, 1);
  for (uint64_t k = 0; k < n_miss; ++k)
    if (k == 0 || mr[k].id != mr[k - 1].id) first[mr[k].idx] = 1;
  for (uint64_t i = 0; i < n; ++i) {
    if (!first[i]) continue;
    p->st.unique_misses++;
    uint64_t s = orc_emb_set_of(p, ids[i]);
    uint32_t nw = ways_at(p, p->n_emb, s);
    uint32_t* tg = p->tag + s * p->w_max;
    uint32_t* sp = p->stamp + s * p->w_max;
    int victim = -1;
    for (uint32_t w = 0; w < nw && victim < 0; ++w)
      if (tg[w] == ORC_TAG_EMPTY) victim = (int)w;
    if (victim < 0) {
      for (uint32_t w = 0; w < nw; ++w) {
        if (sp[w] >= t) continue; /* touched in this batch: not evictable */
        if (victim < 0 || sp[w] < sp[victim]) victim = (int)w;
      }
      if (victim >= 0) p->st.evicted++;
    }
    if (victim < 0) {
      p->st.bypassed++;
      continue;
    }
    tg[victim] = (uint32_t)ids[i];
    sp[victim] = t;
    p->st.inserted++;
  }
  free(first);
  free(mr);
  free(way_of);
  free(valid);
  free(is_hit);
  return ORC_OK;
}

/* Background refill of empty capacity (paper Sec. IV-B: after the EMB side has grown, the new
 * space is filled with hot rows in the background).  `ids` comes in order of decreasing
 * hotness.  The call is one batch of its own in LRU time.  A valid id that is not resident is
 * put, once, into the lowest empty way of its set and stamped with the batch; a refill never
 * evicts (an id whose set has no empty way is skipped), never touches the stamp of a resident
 * row, and counts only in `inserted`.  Taken one id after the other, which is the same as "the
 * k-th new id of a set takes its k-th empty way". */
int orc_emb_refill(orc_pool* p, const int64_t* ids, uint64_t n, uint64_t rows, uint64_t* inserted) {
  if (rows >= 0xFFFFFFFFull) return ORC_EINVAL;
  p->t += 1;
  const uint32_t t = p->t;
  uint64_t ins = 0;
  for (uint64_t i = 0; i < n; ++i) {
    if (ids[i] < 0 || (uint64_t)ids[i] >= rows) continue;
    uint64_t s = orc_emb_set_of(p, ids[i]);
    uint32_t nw = ways_at(p, p->n_emb, s);
    uint32_t* tg = p->tag + s * p->w_max;
    int resident = 0, empty = -1;
    for (uint32_t w = 0; w < nw; ++w) {
      if (tg[w] == (uint32_t)ids[i]) resident = 1;
      if (tg[w] == ORC_TAG_EMPTY && empty < 0) empty = (int)w;
    }
    if (resident || empty < 0) continue;
    tg[empty] = (uint32_t)ids[i];
    p->stamp[s * p->w_max + (uint32_t)empty] = t;
    p->st.inserted++;
    ins++;
  }
  if (inserted) *inserted = ins;
  return ORC_OK;
}
