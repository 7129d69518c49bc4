// Host-side bookkeeping of the shared page pool: which physical page belongs to the
// EMB side, which to a KV sequence, which is free; the KV sequence table with LRU
// stamps and pins.  Pure C++, no device calls (paper Sec. IV-B: boundary updates are
// metadata-only; KV reclaim is metadata-only LRU at user-block granularity; pinned
// blocks are never evicted; an EMB expansion that cannot be served is deferred).
#pragma once

#include <cstdint>
#include <cmath>
#include <set>
#include <unordered_map>
#include <utility>
#include <vector>

namespace racer {

enum : uint8_t { kFree = 0, kEmb = 1, kKv = 2 };

struct SplitPlan {
  int32_t rc = 0;
  uint64_t old_emb = 0, new_emb = 0;
};

class HostPool {
 public:
  HostPool(uint64_t n_pages, uint32_t page_tokens, uint32_t slots_per_page, uint32_t w_max)
      : n_pages_(n_pages), pt_(page_tokens), spp_(slots_per_page), w_max_(w_max),
        layer_pages_(n_pages / w_max), sets_(layer_pages_ * slots_per_page),
        owner_(n_pages, kFree), free_bits_((n_pages + 63) / 64, 0), free_count_(n_pages) {
    for (uint64_t p = 0; p < n_pages; ++p) free_bits_[p >> 6] |= 1ull << (p & 63);
    emb_pages_.reserve(n_pages);
  }

  uint64_t n_pages() const { return n_pages_; }
  uint64_t sets() const { return sets_; }
  uint64_t layer_pages() const { return layer_pages_; }
  uint32_t spp() const { return spp_; }
  uint32_t w_max() const { return w_max_; }
  uint32_t page_tokens() const { return pt_; }
  uint64_t n_emb() const { return emb_pages_.size(); }
  uint64_t free_count() const { return free_count_; }
  uint64_t seqs_resident() const { return seqs_.size(); }
  uint64_t seqs_evicted() const { return seqs_evicted_; }
  const std::vector<int32_t>& emb_pages() const { return emb_pages_; }
  const std::vector<uint8_t>& owner() const { return owner_; }

  static uint32_t ways_for(uint64_t n_emb, uint64_t layer_pages, uint32_t spp, uint64_t set) {
    const uint64_t full = n_emb / layer_pages, part = n_emb % layer_pages;
    return static_cast<uint32_t>(full + (set < part * spp ? 1 : 0));
  }
  uint32_t ways(uint64_t set) const { return ways_for(n_emb(), layer_pages_, spp_, set); }

  int64_t slot_of(uint64_t set, uint32_t way) const {
    if (set >= sets_ || way >= ways(set)) return -1;
    const uint64_t logical = static_cast<uint64_t>(way) * layer_pages_ + set / spp_;
    return static_cast<int64_t>(emb_pages_[logical]) * spp_ + static_cast<int64_t>(set % spp_);
  }

  // Take `count` lowest-numbered free pages onto the EMB side (used at creation).
  void seed_emb(uint64_t count) {
    for (uint64_t k = 0; k < count; ++k) emb_pages_.push_back(take_lowest(kEmb));
  }

  // Host half of a split change.  Growth appends pages to emb_pages(); shrink pops the
  // tail (the caller runs the device-side set compaction against old_emb/new_emb first
  // in stream order; popped pages are only handed to KV writes enqueued later).
  SplitPlan set_split(double emb_frac) {
    SplitPlan plan;
    plan.old_emb = plan.new_emb = n_emb();
    if (!(emb_frac >= 0.1 && emb_frac <= 0.9)) {
      plan.rc = -22;
      return plan;
    }
    const uint64_t target = static_cast<uint64_t>(std::llround(emb_frac * static_cast<double>(n_pages_)));
    if (target > n_emb()) {
      uint64_t need = target - n_emb();
      while (free_count_ < need && !cold_.empty()) evict(cold_.begin()->second);
      if (free_count_ < need) {
        need = free_count_;
        plan.rc = 1;
      }
      for (uint64_t k = 0; k < need; ++k) emb_pages_.push_back(take_lowest(kEmb));
    } else {
      while (n_emb() > target) {
        give_back(emb_pages_.back());
        emb_pages_.pop_back();
      }
    }
    plan.new_emb = n_emb();
    return plan;
  }

  int32_t reserve(uint64_t key, uint32_t tokens, int32_t* pages_out, uint32_t cap, uint32_t* n_out) {
    auto it = seqs_.find(key);
    const uint32_t have_tokens = it == seqs_.end() ? 0 : it->second.tokens;
    const uint32_t want_tokens = tokens > have_tokens ? tokens : have_tokens;
    const uint64_t want_pages = (static_cast<uint64_t>(want_tokens) + pt_ - 1) / pt_;
    const uint64_t have_pages = it == seqs_.end() ? 0 : it->second.pages.size();
    const uint64_t need = want_pages > have_pages ? want_pages - have_pages : 0;
    if (pages_out && cap < want_pages) return -22;
    uint64_t reclaimable = free_count_;
    for (const auto& c : cold_)
      if (c.second != key) reclaimable += seqs_.at(c.second).pages.size();
    if (need > reclaimable) return -12;
    while (free_count_ < need) {
      auto c = cold_.begin();
      if (c->second == key) ++c;
      evict(c->second);
    }
    if (it == seqs_.end()) it = seqs_.emplace(key, Seq{}).first;
    else if (it->second.pins == 0) cold_.erase({it->second.stamp, key});
    Seq& s = it->second;
    for (uint64_t k = 0; k < need; ++k) s.pages.push_back(take_lowest(kKv));
    s.tokens = want_tokens;
    s.stamp = ++clock_;
    if (s.pins == 0) cold_.insert({s.stamp, key});
    return copy_out(s, pages_out, cap, n_out);
  }

  int32_t lookup(uint64_t key, uint32_t* tokens, int32_t* pages_out, uint32_t cap, uint32_t* n_out) const {
    auto it = seqs_.find(key);
    if (it == seqs_.end()) {
      if (tokens) *tokens = 0;
      if (n_out) *n_out = 0;
      return 2;
    }
    if (tokens) *tokens = it->second.tokens;
    return copy_out(it->second, pages_out, cap, n_out);
  }

  int32_t pin(uint64_t key) {
    auto it = seqs_.find(key);
    if (it == seqs_.end()) return 2;
    Seq& s = it->second;
    if (s.pins == 0) cold_.erase({s.stamp, key});
    s.pins++;
    s.stamp = ++clock_;
    return 0;
  }

  int32_t unpin(uint64_t key) {
    auto it = seqs_.find(key);
    if (it == seqs_.end()) return 2;
    Seq& s = it->second;
    if (s.pins == 0) return -22;
    if (--s.pins == 0) cold_.insert({s.stamp, key});
    return 0;
  }

  int32_t release(uint64_t key) {
    auto it = seqs_.find(key);
    if (it == seqs_.end()) return 2;
    if (it->second.pins > 0) return -16;
    drop(it);
    return 0;
  }

 private:
  struct Seq {
    std::vector<int32_t> pages;
    uint32_t tokens = 0;
    uint32_t pins = 0;
    uint64_t stamp = 0;
  };

  static int32_t copy_out(const Seq& s, int32_t* pages_out, uint32_t cap, uint32_t* n_out) {
    if (n_out) *n_out = static_cast<uint32_t>(s.pages.size());
    if (pages_out) {
      if (cap < s.pages.size()) return -22;
      for (size_t k = 0; k < s.pages.size(); ++k) pages_out[k] = s.pages[k];
    }
    return 0;
  }

  int32_t take_lowest(uint8_t new_owner) {
    while (first_word_ < free_bits_.size() && free_bits_[first_word_] == 0) ++first_word_;
    const uint64_t w = free_bits_[first_word_];
    const int bit = __builtin_ctzll(w);
    free_bits_[first_word_] = w & (w - 1);
    const int32_t page = static_cast<int32_t>(first_word_ * 64 + bit);
    owner_[page] = new_owner;
    --free_count_;
    return page;
  }

  void give_back(int32_t page) {
    free_bits_[page >> 6] |= 1ull << (page & 63);
    owner_[page] = kFree;
    ++free_count_;
    if (static_cast<size_t>(page >> 6) < first_word_) first_word_ = page >> 6;
  }

  void drop(std::unordered_map<uint64_t, Seq>::iterator it) {
    if (it->second.pins == 0) cold_.erase({it->second.stamp, it->first});
    for (int32_t p : it->second.pages) give_back(p);
    seqs_.erase(it);
  }

  void evict(uint64_t key) {
    drop(seqs_.find(key));
    ++seqs_evicted_;
  }

  uint64_t n_pages_;
  uint32_t pt_, spp_, w_max_;
  uint64_t layer_pages_, sets_;
  std::vector<uint8_t> owner_;
  std::vector<uint64_t> free_bits_;  // bit set = page is on the KV free list
  size_t first_word_ = 0;            // no free page lives in a word below this one
  uint64_t free_count_;
  std::vector<int32_t> emb_pages_;   // logical EMB page -> physical page
  std::unordered_map<uint64_t, Seq> seqs_;
  std::set<std::pair<uint64_t, uint64_t>> cold_;  // (stamp, key) of unpinned sequences, LRU first
  uint64_t clock_ = 0;
  uint64_t seqs_evicted_ = 0;
};

}  // namespace racer
