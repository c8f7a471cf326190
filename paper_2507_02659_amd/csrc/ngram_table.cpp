// See ngram_table.h.  Plain C++17, no GPU call.
#include "ngram_table.h"

#include <algorithm>
#include <cstring>
#include <string>

namespace otv {

void NgramTable::init(int32_t capacity, int32_t policy, int32_t max_len) {
  uint32_t slots = 16;
  while (slots < 2u * (uint32_t)capacity) slots <<= 1;
  capacity_ = capacity; policy_ = policy; max_len_ = max_len; stride_ = 2 + max_len; mask_ = slots - 1;
  n_entries_ = 0; clock_ = 0; next_seq_ = 0;
  table_.assign((size_t)slots * stride_, 0);
  seq_.assign(slots, 0);
  uses_.assign(slots, 0);
  last_.assign(slots, 0);
  is_dirty_.assign(slots, 0);
  dirty_.clear();
  order_.clear();
  slot_of_seq_.clear();
}

int64_t NgramTable::total_key_ids() const {
  int64_t ids = 0;
  for (uint32_t s = 0; s <= mask_; ++s) ids += slot(s)[0];
  return ids;
}

uint32_t NgramTable::find(const int32_t* ids, int len, bool* found) const {
  uint32_t h = hash_ngram(ids, len) & mask_;
  for (;;) {
    const int32_t* s = slot(h);
    if (s[0] == 0) { *found = false; return h; }
    if (s[0] == len && std::memcmp(s + 2, ids, sizeof(int32_t) * len) == 0) { *found = true; return h; }
    h = (h + 1) & mask_;
  }
}

int64_t NgramTable::lookup(const int32_t* ids, int len) const {
  bool found;
  const uint32_t s = find(ids, len, &found);
  return found ? (int64_t)s : -1;
}

void NgramTable::touch(uint32_t s) {
  if (!is_dirty_[s]) { is_dirty_[s] = 1; dirty_.push_back(s); }
}

void NgramTable::order_add(uint32_t s) {
  if (policy_ == kPolicyNone) return;
  order_.insert(rank_of(s));
  slot_of_seq_[seq_[s]] = s;
}

void NgramTable::order_remove(uint32_t s) {
  if (policy_ == kPolicyNone) return;
  order_.erase(rank_of(s));
  slot_of_seq_.erase(seq_[s]);
}

int64_t NgramTable::count_fresh(int32_t n, const int32_t* key_off, const int32_t* key_ids) const {
  std::set<std::vector<int32_t>> seen;
  int64_t fresh = 0;
  bool found;
  for (int32_t e = 0; e < n; ++e) {
    const int32_t* ids = key_ids + key_off[e];
    const int len = key_off[e + 1] - key_off[e];
    find(ids, len, &found);
    if (!found && seen.insert(std::vector<int32_t>(ids, ids + len)).second) ++fresh;
  }
  return fresh;
}

bool NgramTable::record_use(uint32_t s, uint32_t clock) {
  if (s > mask_ || slot(s)[0] == 0) return false;
  order_remove(s);
  uses_[s] += 1;
  last_[s] = clock;
  order_add(s);
  return true;
}

void NgramTable::replace_statistics(const uint32_t* uses, const uint32_t* last) {
  order_.clear();
  slot_of_seq_.clear();
  for (uint32_t s = 0; s <= mask_; ++s) {
    const bool live = slot(s)[0] != 0;
    uses_[s] = live ? uses[s] : 0;
    last_[s] = live ? last[s] : 0;
    if (live) order_add(s);
  }
}

// Removes the entry in slot i and closes the gap (backward-shift deletion for linear probing).
void NgramTable::erase(uint32_t i) {
  order_remove(i);
  uint32_t j = i;
  for (;;) {
    slot_mut(i)[0] = 0;
    touch(i);
    for (;;) {
      j = (j + 1) & mask_;
      const int32_t* sj = slot(j);
      if (sj[0] == 0) {                      // the gap stays at i: an empty slot carries no statistics
        std::fill(slot_mut(i), slot_mut(i) + stride_, 0);
        uses_[i] = 0; last_[i] = 0; seq_[i] = 0;
        return;
      }
      const uint32_t home = hash_ngram(sj + 2, sj[0]) & mask_;
      // the entry at j may stay if its home slot lies cyclically in (i, j]
      const bool stays = (i <= j) ? (i < home && home <= j) : (i < home || home <= j);
      if (!stays) break;
    }
    std::memcpy(slot_mut(i), slot(j), sizeof(int32_t) * stride_);
    uses_[i] = uses_[j]; last_[i] = last_[j]; seq_[i] = seq_[j];
    if (policy_ != kPolicyNone) slot_of_seq_[seq_[i]] = i;     // same rank, new place
    i = j;
  }
}

int32_t NgramTable::insert(int32_t n, const int32_t* key_off, const int32_t* key_ids, const int32_t* target_ids) {
  if (n <= 0) return 0;
  clock_ += 1;
  int32_t evicted = 0;
  bool found;
  for (int32_t e = 0; e < n; ++e) {
    const int32_t* ids = key_ids + key_off[e];
    const int len = key_off[e + 1] - key_off[e];
    uint32_t s = find(ids, len, &found);
    if (found) {
      order_remove(s);
    } else {
      if (n_entries_ >= capacity_) {                           // full: the lowest-ranked entry makes room
        const uint32_t victim = slot_of_seq_.at(std::get<2>(*order_.begin()));
        erase(victim);
        n_entries_ -= 1;
        ++evicted;
        s = find(ids, len, &found);                            // the shift may have moved the insertion point
      }
      int32_t* sl = slot_mut(s);
      sl[0] = len;
      std::memcpy(sl + 2, ids, sizeof(int32_t) * len);
      std::fill(sl + 2 + len, sl + stride_, 0);
      seq_[s] = next_seq_++;
      uses_[s] = 0;
      n_entries_ += 1;
    }
    slot_mut(s)[1] = target_ids[e];                            // equal key: the later pair wins
    last_[s] = clock_;
    order_add(s);
    touch(s);
  }
  return evicted;
}

void NgramTable::import_entries(int32_t n, const int32_t* key_off, const int32_t* key_ids, const int32_t* target_ids,
                                const int64_t* uses, const int64_t* last_used) {
  bool found;
  for (int32_t e = 0; e < n; ++e) {
    const int32_t* ids = key_ids + key_off[e];
    const int len = key_off[e + 1] - key_off[e];
    const uint32_t s = find(ids, len, &found);
    if (found) {
      order_remove(s);
    } else {
      int32_t* sl = slot_mut(s);
      sl[0] = len;
      std::memcpy(sl + 2, ids, sizeof(int32_t) * len);
      std::fill(sl + 2 + len, sl + stride_, 0);
      seq_[s] = next_seq_++;
      n_entries_ += 1;
    }
    slot_mut(s)[1] = target_ids[e];
    uses_[s] = (uint32_t)uses[e];
    last_[s] = (uint32_t)last_used[e];
    clock_ = std::max(clock_, last_[s]);
    order_add(s);
    touch(s);
  }
}

void NgramTable::export_entries(int32_t* key_off, int32_t* key_ids, int32_t* target_ids, int64_t* uses,
                                int64_t* last_used) const {
  // entries leave in insertion order, so that bringing an export back reproduces the tie-breaking of the original
  std::vector<uint32_t> order;
  for (uint32_t s = 0; s <= mask_; ++s) if (slot(s)[0] != 0) order.push_back(s);
  std::sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) { return seq_[a] < seq_[b]; });
  int64_t at = 0;
  int32_t e = 0;
  key_off[0] = 0;
  for (uint32_t s : order) {
    const int32_t* sl = slot(s);
    std::memcpy(key_ids + at, sl + 2, sizeof(int32_t) * sl[0]);
    at += sl[0];
    target_ids[e] = sl[1];
    if (uses) uses[e] = uses_[s];
    if (last_used) last_used[e] = last_[s];
    key_off[++e] = (int32_t)at;
  }
}

std::vector<uint32_t> NgramTable::take_dirty() {
  std::vector<uint32_t> out;
  out.swap(dirty_);
  for (uint32_t s : out) is_dirty_[s] = 0;
  return out;
}

std::string NgramTable::check() const {
  int32_t live = 0;
  for (uint32_t s = 0; s <= mask_; ++s) {
    const int32_t* sl = slot(s);
    if (sl[0] == 0) {
      if (uses_[s] != 0 || last_[s] != 0) return "an empty slot carries statistics";
      continue;
    }
    ++live;
    if (sl[0] < 2 || sl[0] > max_len_) return "a slot holds a key of a length out of range";
    // the probe for this key must reach this slot without meeting an empty one
    uint32_t h = hash_ngram(sl + 2, sl[0]) & mask_;
    while (h != s) {
      if (slot(h)[0] == 0) return "a probe chain is broken";
      h = (h + 1) & mask_;
    }
    if (policy_ != kPolicyNone) {
      if (!order_.count(rank_of(s))) return "an entry is missing from the eviction order";
      auto it = slot_of_seq_.find(seq_[s]);
      if (it == slot_of_seq_.end() || it->second != s) return "the insertion-number index points elsewhere";
    }
  }
  if (live != n_entries_) return "the entry count is off";
  if (live > capacity_) return "more entries than the capacity";
  if (policy_ != kPolicyNone && ((int32_t)order_.size() != live || (int32_t)slot_of_seq_.size() != live))
    return "the eviction order holds stale entries";
  return std::string();
}

int check_row_offsets(int32_t B, const int32_t* row_off_host, int32_t max_k, const char** what) {
  if (row_off_host[0] != 0) { *what = "row_off[0] must be 0"; return 1; }
  for (int32_t b = 0; b < B; ++b) {
    const int64_t rows = (int64_t)row_off_host[b + 1] - row_off_host[b];
    if (rows < 1) { *what = "every sequence owns k_b + 1 >= 1 rows"; return b + 1; }
    if (rows - 1 > max_k) { *what = "a sequence drafted more than max_k tokens"; return b + 1; }
  }
  return 0;
}

int check_entries(int32_t n, const int32_t* key_off, const int32_t* key_ids, const int32_t* target_ids, int32_t max_len,
                  int32_t V_d, int32_t V_t, const char** what) {
  for (int32_t e = 0; e < n; ++e) {
    const int64_t len = (int64_t)key_off[e + 1] - key_off[e];
    if (key_off[e] < 0 || len < 2 || len > max_len) { *what = "key length outside 2..max_ngram_len"; return e + 1; }
    for (int64_t i = key_off[e]; i < key_off[e + 1]; ++i)
      if (key_ids[i] < 0 || key_ids[i] >= V_d) { *what = "draft id outside [0, V_d)"; return e + 1; }
    if (target_ids[e] < 0 || target_ids[e] >= V_t) { *what = "target id outside [0, V_t)"; return e + 1; }
  }
  return 0;
}

}  // namespace otv
