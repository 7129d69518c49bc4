// Sanitizer run of the host-side code (test infrastructure; built and run by tests/test_host_sanitizers.py with
// -fsanitize=address,undefined): the library's host bookkeeping (csrc/pool_host.h) and split controller
// (csrc/alpha_ctl.h), which contain no device calls, and the C oracle.  The program replays random traces of KV
// and split operations on the host bookkeeping and on the oracle's pool simulator, compares their states after
// every operation, and drives the oracle's cache and HSTU routines over small inputs with empty, ragged and
// out-of-range cases.  Any difference, and any report of a sanitizer, ends it with a non-zero status.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "../../oracle/racer_oracle.h"
#include "../../paper_2605_04450_amd/csrc/alpha_ctl.h"
#include "../../paper_2605_04450_amd/csrc/pool_host.h"

#define CHECK(cond)                                                          \
  do {                                                                       \
    if (!(cond)) {                                                           \
      std::fprintf(stderr, "replay.cpp:%d: check failed: %s\n", __LINE__, #cond); \
      std::exit(1);                                                          \
    }                                                                        \
  } while (0)

static void same_state(const racer::HostPool& h, const orc_pool* o) {
  orc_stats so;
  orc_pool_stats(o, &so);
  CHECK(h.n_pages() == so.pages_total && h.n_emb() == so.pages_emb && h.free_count() == so.pages_kv_free);
  CHECK(h.seqs_resident() == so.seqs_resident && h.seqs_evicted() == so.seqs_evicted);
  std::vector<int64_t> emb(so.pages_emb + 1);
  std::vector<uint8_t> owner(so.pages_total);
  orc_pool_dump(o, emb.data(), owner.data(), nullptr, nullptr);
  for (uint64_t k = 0; k < so.pages_emb; ++k) CHECK(emb[k] == h.emb_pages()[k]);
  CHECK(std::memcmp(owner.data(), h.owner().data(), so.pages_total) == 0);
}

static void replay_traces(uint32_t seed) {
  std::mt19937_64 rng(seed);
  const uint64_t n_pages = 96;
  const uint32_t pt = 4, spp = 8, w_max = 32;
  racer::HostPool h(n_pages, pt, spp, w_max);
  h.seed_emb(static_cast<uint64_t>(std::llround(0.3 * n_pages)));
  orc_pool* o = orc_pool_create(n_pages, pt, spp, w_max, 0.3);
  CHECK(o && h.sets() == orc_pool_num_sets(o));
  for (int step = 0; step < 800; ++step) {
    const int op = static_cast<int>(rng() % 10);
    const uint64_t key = rng() % 12;
    int32_t pg_h[64], pg_o[64];
    uint32_t n_h = 0, n_o = 0, tok_h = 0, tok_o = 0;
    if (op <= 3) {
      const uint32_t tokens = 1 + static_cast<uint32_t>(rng() % 60);
      const int rc_h = h.reserve(key, tokens, pg_h, 64, &n_h), rc_o = orc_kv_seq_reserve(o, key, tokens, pg_o, 64, &n_o);
      CHECK(rc_h == rc_o);
      if (rc_h == 0) CHECK(n_h == n_o && std::memcmp(pg_h, pg_o, n_h * sizeof(int32_t)) == 0);
    } else if (op == 4) {
      CHECK(h.pin(key) == orc_kv_seq_pin(o, key));
    } else if (op == 5) {
      CHECK(h.unpin(key) == orc_kv_seq_unpin(o, key));
    } else if (op == 6) {
      CHECK(h.release(key) == orc_kv_seq_release(o, key));
    } else if (op == 7) {
      const int rc_h = h.lookup(key, &tok_h, pg_h, 64, &n_h), rc_o = orc_kv_seq_lookup(o, key, &tok_o, pg_o, 64, &n_o);
      CHECK(rc_h == rc_o && tok_h == tok_o && n_h == n_o);
      if (rc_h == 0) CHECK(std::memcmp(pg_h, pg_o, n_h * sizeof(int32_t)) == 0);
    } else {
      const double frac = 0.08 + 0.02 * static_cast<double>(rng() % 44);  // also values outside [0.1, 0.9]
      double ach = -1.0;
      const racer::SplitPlan plan = h.set_split(frac);
      const int rc_o = orc_pool_set_split(o, frac, &ach);
      CHECK(plan.rc == rc_o);
      if (rc_o >= 0) CHECK(ach == static_cast<double>(h.n_emb()) / static_cast<double>(n_pages));
    }
    same_state(h, o);
    for (uint64_t s = 0; s < h.sets(); s += 7)
      for (uint32_t w : {0u, 3u, 9u, 31u}) CHECK(h.slot_of(s, w) == orc_pool_slot_of(o, s, w));
  }
  // a copy of the bookkeeping (what pool_set_split keeps to undo a move) is independent of the original
  racer::HostPool copy(h);
  (void)h.set_split(0.9);
  (void)copy.set_split(0.1);
  CHECK(copy.n_emb() <= h.n_emb());
  orc_pool_destroy(o);
}

static void oracle_cache_and_layers(uint32_t seed) {
  std::mt19937_64 rng(seed);
  std::normal_distribution<float> normal(0.0f, 1.0f);
  // cache: small pool under pressure, pooled lookups, ids outside the table, an empty batch, refills, split moves
  const uint64_t rows = 500;
  const uint32_t d = 16;
  std::vector<float> table(rows * d);
  for (float& v : table) v = normal(rng);
  orc_pool* o = orc_pool_create(64, 4, 8, 32, 0.5);
  CHECK(o);
  for (int b = 0; b < 30; ++b) {
    const uint32_t bag = b % 3 == 0 ? 4 : 1;
    const uint64_t n = b == 7 ? 0 : bag * (1 + rng() % 200);
    std::vector<int64_t> ids(n + 1);
    for (uint64_t i = 0; i < n; ++i) ids[i] = static_cast<int64_t>(rng() % (rows + 20)) - 5;  // some negative, some too large
    std::vector<float> out((n / bag + 1) * d);
    std::vector<uint8_t> hit(n + 1);
    CHECK(orc_emb_lookup(o, ids.data(), n, bag, table.data(), rows, d, 0, out.data(), hit.data()) == ORC_OK);
    uint64_t ins = 0;
    if (b % 5 == 4) CHECK(orc_emb_refill(o, ids.data(), n, rows, &ins) == ORC_OK);
    if (b % 4 == 3) (void)orc_pool_set_split(o, 0.1 + 0.1 * static_cast<double>(rng() % 9), nullptr);
    orc_stats st;
    orc_pool_stats(o, &st);
    CHECK(st.hits + st.misses == st.lookups);
  }
  CHECK(orc_emb_lookup(o, nullptr, 0, 0, table.data(), rows, d, 0, nullptr, nullptr) == ORC_EINVAL);
  orc_pool_destroy(o);
  // layers: ragged requests, one with a cached prefix, one empty, shuffled pages; then a bad page id
  orc_hstu_cfg cfg{2, 16, 2, 4, 24, 6, 40.0, 1e-6, 1};
  const uint32_t L = cfg.L, dd = cfg.d, H = cfg.H;
  auto filled = [&](size_t n, float scale) {
    std::vector<float> v(n);
    for (float& x : v) x = orc_round_bf16(scale * normal(rng));
    return v;
  };
  std::vector<float> ln1g = filled(L * dd, 1.0f), ln1b = filled(L * dd, 0.1f), w1 = filled(L * dd * 4 * dd, 0.25f),
                     b1 = filled(L * 4 * dd, 0.1f), ln2g = filled(L * dd, 1.0f), ln2b = filled(L * dd, 0.1f),
                     w2 = filled(L * dd * dd, 0.25f), b2 = filled(L * dd, 0.1f), pos = filled(L * H * cfg.n_pos, 0.1f),
                     tim = filled(L * H * cfg.n_time, 0.1f);
  orc_hstu_weights w{ln1g.data(), ln1b.data(), w1.data(), b1.data(), ln2g.data(), ln2b.data(), w2.data(), b2.data(),
                     pos.data(), tim.data()};
  const uint32_t prefix[4] = {0, 9, 0, 0}, fresh[4] = {13, 6, 0, 1};
  std::vector<orc_hstu_req> reqs;
  std::vector<int32_t> pages;
  std::vector<int64_t> ts;
  uint64_t rows_x = 0;
  int32_t next_page = 11;
  for (int r = 0; r < 4; ++r) {
    reqs.push_back({prefix[r], fresh[r], pages.size(), ts.size(), rows_x});
    const uint32_t S = prefix[r] + fresh[r];
    for (uint32_t k = 0; k < (S + cfg.page_tokens - 1) / cfg.page_tokens; ++k) {
      pages.push_back(next_page);
      next_page = (next_page * 7 + 3) % 31;  // a permutation walk through the 31 pages below
    }
    int64_t t = 1600000000;
    for (uint32_t j = 0; j < S; ++j) ts.push_back(t += static_cast<int64_t>(rng() % 5000));
    rows_x += fresh[r];
  }
  const uint64_t n_kv_pages = 31;
  std::vector<float> kv = filled(n_kv_pages * orc_kv_elems_per_page(&cfg), 0.5f);
  std::vector<float> x = filled(rows_x * dd, 1.0f);
  std::vector<double> out(rows_x * dd);
  CHECK(orc_hstu_step(&cfg, &w, reqs.data(), 4, pages.data(), kv.data(), n_kv_pages, x.data(), ts.data(), out.data(), 2) == ORC_OK);
  CHECK(orc_hstu_step(&cfg, &w, reqs.data(), 1, pages.data(), kv.data(), n_kv_pages, x.data(), ts.data(), out.data(), 2) == ORC_OK);
  for (double v : out) CHECK(v == v);
  pages[1] = 31;  // one past the last page
  CHECK(orc_hstu_step(&cfg, &w, reqs.data(), 4, pages.data(), kv.data(), n_kv_pages, x.data(), ts.data(), out.data(), 1) == ORC_ERANGE);
}

static void controller_epochs() {
  racer::AlphaController ctl(30.0);
  double alpha = 0.5;
  std::mt19937_64 rng(3);
  for (int t = 0; t < 500; ++t) {
    const double lat = 5.0 + static_cast<double>(rng() % 1000) / 10.0;
    double step = 0.0;
    int32_t burst = 0;
    const racer::AlphaState s{static_cast<double>(rng() % 100) / 100.0, 0.5, static_cast<double>(rng() % 100) / 100.0, 2000.0, 0.0, alpha, lat};
    alpha = ctl.decide(s, &step, &burst);
    CHECK(alpha >= racer::kAlphaMin && alpha <= racer::kAlphaMax);
  }
}

int main() {
  for (uint32_t seed = 0; seed < 4; ++seed) replay_traces(seed);
  for (uint32_t seed = 0; seed < 3; ++seed) oracle_cache_and_layers(seed);
  controller_epochs();
  std::puts("host sanitizer replay: ok");
  return 0;
}
