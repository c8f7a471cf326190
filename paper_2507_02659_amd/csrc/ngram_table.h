// Host side of the n-gram cache C = {(t_i, [d_j])} (Section "Cross-vocabulary N-gram Cache") in plain C++: the
// open-addressing table that the device copy mirrors, the use statistics of every entry and the eviction order
// (Appendix "N-gram Cache Scalability": least recently used / least frequently used).  No GPU call in here, so the
// whole life cycle (insert, evict, use, export, import) can be driven and sanitised on a CPU.
//
// Table: linear probing, slot = { len, target, ids[max_len] } as int32, len == 0 marks an empty slot, never more than
// half full.  Deletion is backward-shift deletion, so there are no tombstones and a probe ends at the first empty
// slot.  Every slot the host changes is recorded in `dirty` for the caller to copy to the device.
#pragma once

#include <cstddef>
#include <cstdint>
#include <set>
#include <string>
#include <tuple>
#include <unordered_map>
#include <vector>

namespace otv {

constexpr int kPolicyNone = 0, kPolicyLru = 1, kPolicyLfu = 2;   // values of OT_EVICT_*

// Same mixing on host and device (the device probes what the host placed).
#if defined(__HIPCC__)
__host__ __device__
#endif
inline uint32_t hash_ngram(const int32_t* ids, int len) {
  uint32_t h = 0x9E3779B9u ^ (uint32_t)len;
  for (int i = 0; i < len; ++i) {
    h ^= (uint32_t)ids[i] + 0x7F4A7C15u + (h << 6) + (h >> 2);
    h *= 0x85EBCA6Bu;
    h ^= h >> 13;
  }
  h *= 0xC2B2AE35u;
  h ^= h >> 16;
  return h;
}

class NgramTable {
 public:
  // capacity >= 0 entries, policy kPolicy*, keys of 2..max_len ids.  Throws std::bad_alloc.
  void init(int32_t capacity, int32_t policy, int32_t max_len);

  int32_t capacity() const { return capacity_; }
  int32_t policy() const { return policy_; }
  int32_t size() const { return n_entries_; }
  int32_t stride() const { return stride_; }
  int32_t max_len() const { return max_len_; }
  uint32_t mask() const { return mask_; }
  uint32_t slots() const { return mask_ + 1; }
  uint32_t clock() const { return clock_; }
  void tick() { clock_ += 1; }                       // one verification step was handed the cache
  const int32_t* slot(uint32_t s) const { return &table_[(size_t)s * stride_]; }
  uint32_t uses(uint32_t s) const { return uses_[s]; }
  uint32_t last_used(uint32_t s) const { return last_[s]; }
  const std::vector<int32_t>& table() const { return table_; }
  const std::vector<uint32_t>& all_uses() const { return uses_; }
  const std::vector<uint32_t>& all_last_used() const { return last_; }
  int64_t total_key_ids() const;

  // Slot that holds the key, or -1.
  int64_t lookup(const int32_t* ids, int len) const;
  // Number of distinct keys among the given ones that the table does not hold yet.
  int64_t count_fresh(int32_t n, const int32_t* key_off, const int32_t* key_ids) const;

  // The translation used the entry in `slot` at logical time `clock`: one more use, last used then.
  // Returns false (and changes nothing) if the slot is empty or out of range.
  bool record_use(uint32_t slot, uint32_t clock);
  // Replaces all use statistics by the given per-slot arrays (slots() values each) and rebuilds the eviction order.
  void replace_statistics(const uint32_t* uses, const uint32_t* last);

  // Online update: one tick of the clock, then the pairs in order.  A known key gets the new target and the call's
  // time stamp and keeps its count; a new key that finds the table full first evicts the smallest
  // (last use, insertion number) [LRU] or (uses, last use, insertion number) [LFU].  The caller has checked that the
  // keys are valid and that they fit if there is no policy.  n == 0 changes nothing (no tick).  Returns evictions.
  int32_t insert(int32_t n, const int32_t* key_off, const int32_t* key_ids, const int32_t* target_ids);

  // Like insert for keys the table does not hold, but each entry arrives with its statistics (a saved cache coming
  // back); nothing is evicted, the caller has checked that everything fits.  The clock becomes at least the largest
  // last_used.
  void import_entries(int32_t n, const int32_t* key_off, const int32_t* key_ids, const int32_t* target_ids,
                      const int64_t* uses, const int64_t* last_used);

  // Entries in insertion order.  Arrays sized by size() / total_key_ids(); uses / last_used may be nullptr.
  void export_entries(int32_t* key_off, int32_t* key_ids, int32_t* target_ids, int64_t* uses, int64_t* last_used) const;

  // Slots changed by the host since the last call (each once), for the device copy.
  std::vector<uint32_t> take_dirty();

  // Checks every structural invariant (probe chains unbroken, order and index consistent with the slots); used by
  // tests.  Returns an empty string or a description of the first violation.
  std::string check() const;

 private:
  typedef std::tuple<uint32_t, uint32_t, uint64_t> Rank;   // (uses or 0, last use, insertion number)
  Rank rank_of(uint32_t s) const { return Rank(policy_ == kPolicyLfu ? uses_[s] : 0u, last_[s], seq_[s]); }
  int32_t* slot_mut(uint32_t s) { return &table_[(size_t)s * stride_]; }
  uint32_t find(const int32_t* ids, int len, bool* found) const;
  void erase(uint32_t s);
  void touch(uint32_t s);
  void order_add(uint32_t s);
  void order_remove(uint32_t s);

  int32_t capacity_ = 0, policy_ = kPolicyNone, n_entries_ = 0, stride_ = 0, max_len_ = 0;
  uint32_t mask_ = 0, clock_ = 0;
  uint64_t next_seq_ = 0;
  std::vector<int32_t> table_;
  std::vector<uint64_t> seq_;                   // insertion number of the entry in each slot
  std::vector<uint32_t> uses_, last_;
  std::set<Rank> order_;                        // entries by eviction rank (kept only with a policy)
  std::unordered_map<uint64_t, uint32_t> slot_of_seq_;
  std::vector<uint32_t> dirty_;
  std::vector<uint8_t> is_dirty_;
};

// Argument checks shared by the entry points (plain integers only).  Return 0 or the index+1 of the first offending
// item; *what receives a static description.
int check_row_offsets(int32_t B, const int32_t* row_off_host, int32_t max_k, const char** what);
int check_entries(int32_t n, const int32_t* key_off, const int32_t* key_ids, const int32_t* target_ids, int32_t max_len,
                  int32_t V_d, int32_t V_t, const char** what);

}  // namespace otv
