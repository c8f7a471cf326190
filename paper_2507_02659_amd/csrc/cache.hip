// Host side of the n-gram cache C = {(t_i, [d_j])} (Section "Cross-vocabulary N-gram Cache"): bulk build, online
// insertion (Algorithm 1, "Add to n-gram cache if there exists unseen n-gram instance"), eviction at a maximum size
// (Appendix "N-gram Cache Scalability": least recently used / least frequently used) and export.
//
// The table is open addressing with linear probing, mirrored on the host; the device copy is what the translation
// kernel probes, and the kernel keeps two counters per slot (uses, last use).  All maintenance happens between
// steps: every call here first synchronises the context's stream.  Deletion is backward-shift deletion, so the
// table never holds tombstones and a probe still ends at the first empty slot.
#include <algorithm>
#include <cstring>
#include <new>
#include <set>

#include "otv_host.h"

using namespace otv;

namespace {

constexpr int32_t kMaxCapacity = 1 << 26;    // slot indices must fit in 28 bits next to the key length

inline int32_t* slot_of(ot_ngram_cache* c, uint32_t s) { return &c->table[(size_t)s * c->stride]; }

// Slot that holds `ids`, or the empty slot where it would go.
uint32_t find_slot(ot_ngram_cache* c, const int32_t* ids, int len, bool* found) {
  uint32_t h = hash_ngram(ids, len) & c->mask;
  for (;;) {
    const int32_t* s = slot_of(c, h);
    if (s[0] == 0) { *found = false; return h; }
    if (s[0] == len && std::memcmp(s + 2, ids, sizeof(int32_t) * len) == 0) { *found = true; return h; }
    h = (h + 1) & c->mask;
  }
}

struct Counters {                 // host copies of the device counters, fetched only when a call needs them
  std::vector<uint32_t> uses, last;
  bool loaded = false;
};

int load_counters(ot_ngram_cache* c, Counters* k) {
  if (k->loaded) return OT_OK;
  const size_t n = (size_t)c->mask + 1;
  try { k->uses.resize(n); k->last.resize(n); } catch (const std::bad_alloc&) { return ot_fail(OT_ERR_NOMEM, "n-gram cache: host allocation failed"); }
  hipError_t e = hipMemcpy(k->uses.data(), c->d_uses, n * sizeof(uint32_t), hipMemcpyDeviceToHost);
  if (e == hipSuccess) e = hipMemcpy(k->last.data(), c->d_last, n * sizeof(uint32_t), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return ot_fail_hip(e, "n-gram cache: reading the use counters");
  k->loaded = true;
  return OT_OK;
}

// Removes the entry in slot i and closes the gap (backward-shift deletion for linear probing).
void erase_slot(ot_ngram_cache* c, Counters* k, uint32_t i) {
  const uint32_t mask = c->mask;
  uint32_t j = i;
  for (;;) {
    slot_of(c, i)[0] = 0;
    for (;;) {
      j = (j + 1) & mask;
      int32_t* sj = slot_of(c, j);
      if (sj[0] == 0) {                      // the gap stays at i: an empty slot carries no statistics
        k->uses[i] = 0; k->last[i] = 0; c->seq[i] = 0;
        return;
      }
      const uint32_t home = hash_ngram(sj + 2, sj[0]) & mask;
      // the entry at j may stay if its home slot lies cyclically in (i, j]
      const bool stays = (i <= j) ? (i < home && home <= j) : (i < home || home <= j);
      if (!stays) break;
    }
    std::memcpy(slot_of(c, i), slot_of(c, j), sizeof(int32_t) * c->stride);
    k->uses[i] = k->uses[j]; k->last[i] = k->last[j]; c->seq[i] = c->seq[j];
    i = j;
  }
}

uint32_t pick_victim(ot_ngram_cache* c, const Counters& k) {
  uint32_t best = 0;
  bool have = false;
  for (uint32_t s = 0; s <= c->mask; ++s) {
    if (slot_of(c, s)[0] == 0) continue;
    bool better;
    if (!have) better = true;
    else if (c->policy == OT_EVICT_LRU)
      better = k.last[s] != k.last[best] ? k.last[s] < k.last[best] : c->seq[s] < c->seq[best];
    else
      better = k.uses[s] != k.uses[best] ? k.uses[s] < k.uses[best]
             : k.last[s] != k.last[best] ? k.last[s] < k.last[best] : c->seq[s] < c->seq[best];
    if (better) { best = s; have = true; }
  }
  return best;
}

int validate_entries(ot_ctx* ctx, const char* who, int32_t n, const int32_t* key_off, const int32_t* key_ids,
                     const int32_t* target_ids) {
  if (n < 0) return ot_fail(OT_ERR_SHAPE, "%s: n_entries < 0", who);
  if (n > 0 && (!key_off || !key_ids || !target_ids)) return ot_fail(OT_ERR_NULL, "%s: NULL entry arrays", who);
  for (int32_t e = 0; e < n; ++e) {
    const int64_t len = (int64_t)key_off[e + 1] - key_off[e];
    if (key_off[e] < 0 || len < 2 || len > ctx->max_ngram_len)
      return ot_fail(OT_ERR_NGRAM, "%s: entry %d has length %lld, allowed 2..%d", who, e, (long long)len, ctx->max_ngram_len);
    for (int64_t i = key_off[e]; i < key_off[e + 1]; ++i)
      if (key_ids[i] < 0 || key_ids[i] >= ctx->V_d)
        return ot_fail(OT_ERR_NGRAM, "%s: entry %d holds draft id %d outside [0, V_d)", who, e, key_ids[i]);
    if (target_ids[e] < 0 || target_ids[e] >= ctx->V_t)
      return ot_fail(OT_ERR_NGRAM, "%s: entry %d maps to target id %d outside [0, V_t)", who, e, target_ids[e]);
  }
  return OT_OK;
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

int ot_ngram_cache_create(ot_ctx* ctx, int32_t capacity, int32_t policy, ot_ngram_cache** out) {
  if (out) *out = nullptr;
  if (!ctx || !out) return ot_fail(OT_ERR_NULL, "ot_ngram_cache_create: ctx and out must not be NULL");
  if (capacity < 0 || capacity > kMaxCapacity) return ot_fail(OT_ERR_SHAPE, "ot_ngram_cache_create: capacity must be in 0..%d", kMaxCapacity);
  if (policy != OT_EVICT_NONE && policy != OT_EVICT_LRU && policy != OT_EVICT_LFU)
    return ot_fail(OT_ERR_SHAPE, "ot_ngram_cache_create: unknown eviction policy %d", policy);
  ot_ngram_cache* c = new (std::nothrow) ot_ngram_cache();
  if (!c) return ot_fail(OT_ERR_NOMEM, "ot_ngram_cache_create: host allocation failed");
  uint32_t slots = 16;
  while (slots < 2u * (uint32_t)capacity) slots <<= 1;
  c->owner = ctx; c->capacity = capacity; c->policy = policy; c->stride = 2 + ctx->max_ngram_len;
  c->max_len = ctx->max_ngram_len; c->mask = slots - 1;
  try {
    c->table.assign((size_t)slots * c->stride, 0);
    c->seq.assign(slots, 0);
  } catch (const std::bad_alloc&) {
    delete c;
    return ot_fail(OT_ERR_NOMEM, "ot_ngram_cache_create: host allocation failed");
  }
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&c->d_slots), c->table.size() * sizeof(int32_t));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->d_uses), slots * sizeof(uint32_t));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->d_last), slots * sizeof(uint32_t));
  if (e != hipSuccess) {
    (void)hipGetLastError();
    ot_ngram_cache_destroy(c);
    return ot_fail(OT_ERR_NOMEM, "ot_ngram_cache_create: device allocation failed");
  }
  e = hipMemset(c->d_slots, 0, c->table.size() * sizeof(int32_t));
  if (e == hipSuccess) e = hipMemset(c->d_uses, 0, slots * sizeof(uint32_t));
  if (e == hipSuccess) e = hipMemset(c->d_last, 0, slots * sizeof(uint32_t));
  if (e != hipSuccess) { ot_ngram_cache_destroy(c); return ot_fail_hip(e, "ot_ngram_cache_create: clearing the table"); }
  *out = c;
  return OT_OK;
}

int ot_ngram_cache_insert(ot_ngram_cache* c, int32_t n_entries, const int32_t* key_off, const int32_t* key_ids,
                          const int32_t* target_ids, int32_t* n_evicted) {
  if (n_evicted) *n_evicted = 0;
  if (!c) return ot_fail(OT_ERR_NULL, "ot_ngram_cache_insert: cache is NULL");
  int rc = validate_entries(c->owner, "ot_ngram_cache_insert", n_entries, key_off, key_ids, target_ids);
  if (rc != OT_OK) return rc;
  if (n_entries == 0) return OT_OK;

  // how many places do the new keys of this call need?
  bool found;
  int64_t fresh = 0;
  {
    std::set<std::vector<int32_t>> seen;
    for (int32_t e = 0; e < n_entries; ++e) {
      const int32_t* ids = key_ids + key_off[e];
      const int len = key_off[e + 1] - key_off[e];
      find_slot(c, ids, len, &found);
      if (!found && seen.insert(std::vector<int32_t>(ids, ids + len)).second) ++fresh;
    }
  }
  const bool overflow = (int64_t)c->n_entries + fresh > c->capacity;
  if (overflow && (c->policy == OT_EVICT_NONE || c->capacity == 0))
    return ot_fail(OT_ERR_SHAPE, "ot_ngram_cache_insert: %lld new keys do not fit into %d free places and the cache has no "
                   "eviction policy", (long long)fresh, c->capacity - c->n_entries);

  hipError_t he = hipStreamSynchronize(c->owner->stream);      // no step may be probing the table while it changes
  if (he != hipSuccess) return ot_fail_hip(he, "ot_ngram_cache_insert: synchronize");

  Counters k;
  const bool bulk = overflow || n_entries > 32;                // bulk: work on full host copies, upload everything
  if (bulk && (rc = load_counters(c, &k)) != OT_OK) return rc;
  c->clock += 1;
  std::vector<uint32_t> touched;
  int32_t evicted = 0;
  for (int32_t e = 0; e < n_entries; ++e) {
    const int32_t* ids = key_ids + key_off[e];
    const int len = key_off[e + 1] - key_off[e];
    uint32_t s = find_slot(c, ids, len, &found);
    if (!found) {
      if (c->n_entries >= c->capacity) {                       // full: make room (only reachable in bulk mode)
        erase_slot(c, &k, pick_victim(c, k));
        c->n_entries -= 1;
        ++evicted;
        s = find_slot(c, ids, len, &found);                    // the shift may have moved the insertion point
      }
      int32_t* slot = slot_of(c, s);
      slot[0] = len;
      std::memcpy(slot + 2, ids, sizeof(int32_t) * len);
      std::fill(slot + 2 + len, slot + c->stride, 0);
      c->seq[s] = c->next_seq++;
      c->n_entries += 1;
      if (bulk) k.uses[s] = 0;
    }
    slot_of(c, s)[1] = target_ids[e];                          // equal key: the later pair wins
    if (bulk) k.last[s] = c->clock;
    else touched.push_back(s);
  }
  if (bulk) {
    const size_t n = (size_t)c->mask + 1;
    he = hipMemcpy(c->d_slots, c->table.data(), c->table.size() * sizeof(int32_t), hipMemcpyHostToDevice);
    if (he == hipSuccess) he = hipMemcpy(c->d_uses, k.uses.data(), n * sizeof(uint32_t), hipMemcpyHostToDevice);
    if (he == hipSuccess) he = hipMemcpy(c->d_last, k.last.data(), n * sizeof(uint32_t), hipMemcpyHostToDevice);
  } else {
    // a few slots changed and nothing moved: patch them in place (a fresh slot's use counter is still 0 on the device)
    for (uint32_t s : touched) {
      if (he == hipSuccess)
        he = hipMemcpy(c->d_slots + (size_t)s * c->stride, slot_of(c, s), sizeof(int32_t) * c->stride, hipMemcpyHostToDevice);
      if (he == hipSuccess) he = hipMemcpy(c->d_last + s, &c->clock, sizeof(uint32_t), hipMemcpyHostToDevice);
    }
  }
  if (he != hipSuccess) return ot_fail_hip(he, "ot_ngram_cache_insert: upload");
  if (n_evicted) *n_evicted = evicted;
  return OT_OK;
}

int ot_ngram_cache_build(ot_ctx* ctx, int32_t n_entries, const int32_t* key_off, const int32_t* key_ids,
                         const int32_t* target_ids, ot_ngram_cache** out) {
  if (out) *out = nullptr;
  if (!ctx || !out) return ot_fail(OT_ERR_NULL, "ot_ngram_cache_build: ctx and out must not be NULL");
  int rc = validate_entries(ctx, "ot_ngram_cache_build", n_entries, key_off, key_ids, target_ids);
  if (rc != OT_OK) return rc;
  if (n_entries > kMaxCapacity) return ot_fail(OT_ERR_SHAPE, "ot_ngram_cache_build: too many entries");
  ot_ngram_cache* c = nullptr;
  rc = ot_ngram_cache_create(ctx, n_entries, OT_EVICT_NONE, &c);
  if (rc != OT_OK) return rc;
  rc = ot_ngram_cache_insert(c, n_entries, key_off, key_ids, target_ids, nullptr);
  if (rc != OT_OK) { ot_ngram_cache_destroy(c); return rc; }
  *out = c;
  return OT_OK;
}

int ot_ngram_cache_size(const ot_ngram_cache* c, int32_t* n_entries, int32_t* n_key_ids) {
  if (!c || !n_entries) return ot_fail(OT_ERR_NULL, "ot_ngram_cache_size: NULL argument");
  *n_entries = c->n_entries;
  if (n_key_ids) {
    int64_t ids = 0;
    for (uint32_t s = 0; s <= c->mask; ++s) ids += c->table[(size_t)s * c->stride];
    *n_key_ids = (int32_t)ids;
  }
  return OT_OK;
}

int ot_ngram_cache_export(ot_ngram_cache* c, int32_t max_entries, int32_t max_key_ids, int32_t* key_off,
                          int32_t* key_ids, int32_t* target_ids, int64_t* uses, int64_t* last_used) {
  if (!c || !key_off || !key_ids || !target_ids) return ot_fail(OT_ERR_NULL, "ot_ngram_cache_export: NULL argument");
  hipError_t he = hipStreamSynchronize(c->owner->stream);
  if (he != hipSuccess) return ot_fail_hip(he, "ot_ngram_cache_export: synchronize");
  Counters k;
  int rc = load_counters(c, &k);
  if (rc != OT_OK) return rc;
  if (max_entries < c->n_entries) return ot_fail(OT_ERR_SHAPE, "ot_ngram_cache_export: room for %d entries, cache holds %d", max_entries, c->n_entries);
  // entries leave in insertion order, so that re-inserting an export reproduces the tie-breaking of the original
  std::vector<uint32_t> order;
  for (uint32_t s = 0; s <= c->mask; ++s) if (slot_of(c, s)[0] != 0) order.push_back(s);
  std::sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) { return c->seq[a] < c->seq[b]; });
  int64_t at = 0;
  int32_t e = 0;
  key_off[0] = 0;
  for (uint32_t s : order) {
    const int32_t* slot = slot_of(c, s);
    if (at + slot[0] > max_key_ids) return ot_fail(OT_ERR_SHAPE, "ot_ngram_cache_export: room for %d key ids is not enough", max_key_ids);
    std::memcpy(key_ids + at, slot + 2, sizeof(int32_t) * slot[0]);
    at += slot[0];
    target_ids[e] = slot[1];
    if (uses) uses[e] = k.uses[s];
    if (last_used) last_used[e] = k.last[s];
    key_off[++e] = (int32_t)at;
  }
  return OT_OK;
}

void ot_ngram_cache_destroy(ot_ngram_cache* cache) {
  if (!cache) return;
  if (cache->owner) (void)hipStreamSynchronize(cache->owner->stream);
  if (cache->d_slots) (void)hipFree(cache->d_slots);
  if (cache->d_uses) (void)hipFree(cache->d_uses);
  if (cache->d_last) (void)hipFree(cache->d_last);
  delete cache;
}

}  // extern "C"
#pragma GCC visibility pop
