// Host-memory parameter cache of the MEM-PS (paper: Appendix D "MEM-PS Implementation", cache
// policy; Algorithm 1: pull the working parameters of a batch, collect the updates of the HBM
// tier, update the local cache, hand the evicted parameters to the SSD tier).  Host code only.
//
// Policy (Appendix D): a visited parameter goes to the most-recently-used end of an LRU list;
// what the LRU list evicts enters an LFU cache; what the LFU cache evicts is collected for the
// tier below; parameters visited by a batch that is not completed yet are pinned.  Where the
// appendix is silent: capacities count parameters; evictions happen when a batch completes;
// the LRU list gives up its least recently visited unpinned parameter; a parameter's frequency
// counts its visits since it entered the memory and travels with it between the two caches;
// LFU ties go to the parameter that entered the LFU cache first; a visit moves a parameter of
// the LFU cache back to the LRU list; a batch pins a parameter once however often it visits it.
#pragma once

#include <cstdint>
#include <cstring>
#include <set>
#include <tuple>
#include <unordered_map>
#include <unordered_set>
#include <vector>

namespace hps {

class MemTier {
 public:
  MemTier(uint32_t dim, uint32_t acc_len, uint64_t lru_capacity, uint64_t lfu_capacity)
      : dim_(dim), acc_len_(acc_len), lru_cap_(lru_capacity), lfu_cap_(lfu_capacity) {}

  uint32_t dim() const { return dim_; }
  uint32_t acc_len() const { return acc_len_; }

  // Visits the keys the memory holds on behalf of `batch` and copies their rows out.
  void fetch(const uint64_t* keys, uint64_t n, uint64_t batch, float* w, float* acc, uint8_t* found) {
    for (uint64_t i = 0; i < n; ++i) {
      auto it = index_.find(keys[i]);
      if (it == index_.end()) {
        found[i] = 0;
        ++misses_;
        continue;
      }
      visit(it->second, batch);
      const float* row = row_of(it->second);
      std::memcpy(w + i * dim_, row, dim_ * sizeof(float));
      std::memcpy(acc + i * acc_len_, row + dim_, acc_len_ * sizeof(float));
      found[i] = 1;
      ++hits_;
    }
  }

  // Puts rows into the memory.  visit: they come from the tier below (a miss being filled);
  // otherwise they are new values of parameters the memory holds (the collect step), and a
  // key it does not hold is taken in as a visit.
  void store(const uint64_t* keys, uint64_t n, const float* w, const float* acc, uint64_t batch,
             bool visit_them) {
    for (uint64_t i = 0; i < n; ++i) {
      auto it = index_.find(keys[i]);
      const bool present = it != index_.end();
      const uint32_t e = present ? it->second : new_entry(keys[i]);
      float* row = row_of(e);
      std::memcpy(row, w + i * dim_, dim_ * sizeof(float));
      std::memcpy(row + dim_, acc + i * acc_len_, acc_len_ * sizeof(float));
      if (visit_them || !present) visit(e, batch);
    }
  }

  // The batch's parameters are no longer pinned; both caches go back to their capacities.
  void complete_batch(uint64_t batch) {
    auto b = batches_.find(batch);
    if (b != batches_.end()) {
      for (uint64_t key : b->second) --entries_[index_.at(key)].pins;
      batches_.erase(b);
    }
    // the LRU list's least recently visited unpinned parameters, oldest first
    uint32_t e = lru_tail_;
    while (lru_size_ > lru_cap_ && e != kNone) {
      const uint32_t newer = entries_[e].prev;
      if (entries_[e].pins == 0) {
        unlink(e);
        entries_[e].in_lfu = true;
        entries_[e].lfu_seq = ++lfu_clock_;
        lfu_.insert(std::make_tuple(entries_[e].freq, entries_[e].lfu_seq, e));
      }
      e = newer;
    }
    while (lfu_.size() > lfu_cap_) {
      const uint32_t victim = std::get<2>(*lfu_.begin());
      lfu_.erase(lfu_.begin());
      const float* row = row_of(victim);
      evicted_keys_.push_back(entries_[victim].key);
      evicted_rows_.insert(evicted_rows_.end(), row, row + dim_ + acc_len_);
      index_.erase(entries_[victim].key);
      free_.push_back(victim);
    }
  }

  uint64_t evicted_waiting() const { return evicted_keys_.size(); }

  // Hands over up to max_rows collected parameters, oldest first; returns how many.
  uint64_t take_evicted(uint64_t* keys, float* w, float* acc, uint64_t max_rows) {
    const uint64_t n = evicted_keys_.size() < max_rows ? evicted_keys_.size() : max_rows;
    const size_t stride = dim_ + acc_len_;
    for (uint64_t i = 0; i < n; ++i) {
      keys[i] = evicted_keys_[i];
      std::memcpy(w + i * dim_, &evicted_rows_[i * stride], dim_ * sizeof(float));
      std::memcpy(acc + i * acc_len_, &evicted_rows_[i * stride + dim_], acc_len_ * sizeof(float));
    }
    evicted_keys_.erase(evicted_keys_.begin(), evicted_keys_.begin() + n);
    evicted_rows_.erase(evicted_rows_.begin(), evicted_rows_.begin() + n * stride);
    return n;
  }

  // Keys of the LRU list, most recently visited first (which = 0), or of the LFU cache in the
  // order they entered it (which = 1).  Returns the number of keys there; writes at most max.
  uint64_t list(int which, uint64_t* keys, uint64_t max) const {
    uint64_t n = 0;
    if (which == 0) {
      for (uint32_t e = lru_head_; e != kNone; e = entries_[e].next, ++n)
        if (n < max) keys[n] = entries_[e].key;
    } else {
      std::vector<std::pair<uint64_t, uint64_t>> by_seq;
      for (const auto& t : lfu_) by_seq.emplace_back(std::get<1>(t), entries_[std::get<2>(t)].key);
      std::sort(by_seq.begin(), by_seq.end());
      for (const auto& p : by_seq) { if (n < max) keys[n] = p.second; ++n; }
    }
    return n;
  }

  uint64_t lru_size() const { return lru_size_; }
  uint64_t lfu_size() const { return lfu_.size(); }
  uint64_t hits() const { return hits_; }
  uint64_t misses() const { return misses_; }
  uint64_t pinned() const {
    uint64_t n = 0;
    for (uint32_t e = lru_head_; e != kNone; e = entries_[e].next) n += entries_[e].pins ? 1 : 0;
    return n;
  }

 private:
  static constexpr uint32_t kNone = ~0u;
  struct Entry {
    uint64_t key;
    uint64_t freq;       // visits since it entered the memory
    uint64_t lfu_seq;    // when it entered the LFU cache
    uint32_t prev, next; // LRU list: prev is more recent
    uint32_t pins;       // uncompleted batches that visited it
    bool in_lfu;
  };

  float* row_of(uint32_t e) { return &rows_[(size_t)e * (dim_ + acc_len_)]; }

  uint32_t new_entry(uint64_t key) {
    uint32_t e;
    if (!free_.empty()) {
      e = free_.back();
      free_.pop_back();
    } else {
      e = (uint32_t)entries_.size();
      entries_.push_back(Entry());
      rows_.resize(rows_.size() + dim_ + acc_len_);
    }
    entries_[e] = Entry{key, 0, 0, kNone, kNone, 0, false};
    linked_.resize(entries_.size(), false);
    linked_[e] = false;
    index_[key] = e;
    return e;
  }

  void unlink(uint32_t e) {
    Entry& x = entries_[e];
    if (x.prev != kNone) entries_[x.prev].next = x.next; else lru_head_ = x.next;
    if (x.next != kNone) entries_[x.next].prev = x.prev; else lru_tail_ = x.prev;
    x.prev = x.next = kNone;
    linked_[e] = false;
    --lru_size_;
  }

  void visit(uint32_t e, uint64_t batch) {
    Entry& x = entries_[e];
    if (x.in_lfu) {
      lfu_.erase(std::make_tuple(x.freq, x.lfu_seq, e));
      x.in_lfu = false;
    } else if (linked_[e]) {
      unlink(e);
    }
    x.prev = kNone;
    x.next = lru_head_;
    if (lru_head_ != kNone) entries_[lru_head_].prev = e; else lru_tail_ = e;
    lru_head_ = e;
    linked_[e] = true;
    ++lru_size_;
    ++x.freq;
    if (batches_[batch].insert(x.key).second) ++x.pins;
  }

  uint32_t dim_, acc_len_;
  uint64_t lru_cap_, lfu_cap_;
  std::vector<Entry> entries_;
  std::vector<bool> linked_;          // entry is on the LRU list
  std::vector<float> rows_;           // entry e: weights then accumulators
  std::vector<uint32_t> free_;
  std::unordered_map<uint64_t, uint32_t> index_;
  uint32_t lru_head_ = kNone, lru_tail_ = kNone;
  uint64_t lru_size_ = 0;
  std::set<std::tuple<uint64_t, uint64_t, uint32_t>> lfu_;   // (frequency, entered, entry)
  uint64_t lfu_clock_ = 0;
  std::unordered_map<uint64_t, std::unordered_set<uint64_t>> batches_;
  std::vector<uint64_t> evicted_keys_;
  std::vector<float> evicted_rows_;
  uint64_t hits_ = 0, misses_ = 0;
};

}  // namespace hps
