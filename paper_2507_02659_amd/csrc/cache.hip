// Device side of the n-gram cache C = {(t_i, [d_j])} (Section "Cross-vocabulary N-gram Cache") and the entry points
// that maintain it: bulk build, online insertion (the cache-update step at the end of Algorithm 1), eviction at a
// maximum size (Appendix "N-gram Cache Scalability": least recently used / least frequently used), export and import.
//
// The table itself, its use statistics and the eviction order live on the host in plain C++ (ngram_table.h); the
// device holds a copy that the translation kernel probes.  The two are kept in step incrementally:
//   device -> host  the translation kernel appends (slot, clock) for every entry it uses to a small log in pinned host
//                   memory, which it writes directly; a maintenance call reads the log in place (no copy) and replays it
//                   on the host table.  A log that overflowed is replaced by a read-back of the per-slot counters.
//   host -> device  the host records the slots it changed; they travel as one packed patch in pinned host memory that
//                   one small kernel reads in place and scatters (it also clears the log's count).  Only a change of
//                   more than kPatchCap slots (a bulk build) uploads the arrays whole.
// All maintenance happens between steps: every call here first makes sure that the context's stream is idle (a query
// when it already is, a wait otherwise).  Measured: an insert that evicts one entry of a full 100 000-entry cache
// costs about 20 us inside the library.
#include <algorithm>
#include <cstring>
#include <new>

#include "otv_host.h"

using namespace otv;

namespace {

constexpr int32_t kMaxCapacity = 1 << 26;    // slot indices must fit in 28 bits next to the key length

// Scatters a packed patch into the device table.  Record r = { slot, uses, last_used, slot words[stride] }.
__global__ __launch_bounds__(256) void cache_patch_kernel(const uint32_t* __restrict__ patch, int n, int stride,
                                                          int32_t* __restrict__ slots, uint32_t* __restrict__ uses,
                                                          uint32_t* __restrict__ last, uint32_t* __restrict__ log_count) {
  const int words = 3 + stride;
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i == 0) log_count[0] = 0;              // the log has been read: start it over
  if (i >= n * words) return;
  const int r = i / words, w = i % words;
  const uint32_t* rec = patch + (size_t)r * words;
  const uint32_t s = rec[0];
  if (w == 1) uses[s] = rec[1];
  else if (w == 2) last[s] = rec[2];
  else if (w >= 3) slots[(size_t)s * stride + (w - 3)] = (int32_t)rec[w];
}

// Replays what the device did since the last maintenance call on the host table.  The stream is idle.  The log lives in
// pinned host memory that the device wrote directly, so it is read in place: entries are filled from the front and an
// entry that is still 0 ends them.  Only when every entry is taken is the device's own count fetched, to tell a full
// log from one that overflowed.
int pull_use_log(ot_ngram_cache* c) {
  const uint2* log = c->h_log;
  uint32_t count = c->log_replayed;
  while (count < (uint32_t)kCacheLogCap && log[count].x != 0) ++count;
  c->log_pending = count != 0;
  if (count == (uint32_t)kCacheLogCap) {
    uint32_t logged = 0;
    hipError_t e = hipMemcpy(&logged, c->d_log_count, sizeof(uint32_t), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return ot_fail_hip(e, "n-gram cache: reading the use count");
    if (logged > (uint32_t)kCacheLogCap) {
      // more uses than the log holds: take the per-slot counters instead
      const size_t n = c->tab.slots();
      std::vector<uint32_t> uses, last;
      try { uses.resize(n); last.resize(n); } catch (const std::bad_alloc&) { return ot_fail(OT_ERR_NOMEM, "n-gram cache: host allocation failed"); }
      e = hipMemcpy(uses.data(), c->d_uses, n * sizeof(uint32_t), hipMemcpyDeviceToHost);
      if (e == hipSuccess) e = hipMemcpy(last.data(), c->d_last, n * sizeof(uint32_t), hipMemcpyDeviceToHost);
      if (e != hipSuccess) return ot_fail_hip(e, "n-gram cache: reading the use counters");
      c->tab.replace_statistics(uses.data(), last.data());
      return OT_OK;
    }
  }
  for (uint32_t i = c->log_replayed; i < count; ++i) {
    if (!c->tab.record_use(log[i].x - 1u, log[i].y)) return ot_fail(OT_ERR_HIP, "n-gram cache: the use log names an empty slot");
  }
  c->log_replayed = count;
  return OT_OK;
}

// Sends the slots the host changed to the device (a kernel on the context's stream that reads the packed patch out of
// pinned host memory) and clears the log: the entries here, the device's count in that kernel.  The patch memory is
// not written again before the next maintenance call, which starts by waiting for the stream.
int push_changes(ot_ngram_cache* c) {
  std::vector<uint32_t> dirty = c->tab.take_dirty();
  hipStream_t st = c->owner->stream;
  const int stride = c->tab.stride();
  hipError_t e = hipSuccess;
  if ((int64_t)dirty.size() > kCachePatchCap) {
    const size_t n = c->tab.slots();
    e = hipMemcpy(c->d_slots, c->tab.table().data(), c->tab.table().size() * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(c->d_uses, c->tab.all_uses().data(), n * sizeof(uint32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(c->d_last, c->tab.all_last_used().data(), n * sizeof(uint32_t), hipMemcpyHostToDevice);
    if (e != hipSuccess) return ot_fail_hip(e, "n-gram cache: upload");
    dirty.clear();
  }
  if (dirty.empty() && !c->log_pending) return OT_OK;
  const int words = 3 + stride;
  uint32_t* h = c->h_stage;
  for (size_t r = 0; r < dirty.size(); ++r) {
    const uint32_t s = dirty[r];
    uint32_t* rec = h + r * words;
    rec[0] = s; rec[1] = c->tab.uses(s); rec[2] = c->tab.last_used(s);
    std::memcpy(rec + 3, c->tab.slot(s), sizeof(int32_t) * stride);
  }
  const int n = (int)dirty.size();
  hipLaunchKernelGGL(cache_patch_kernel, dim3(std::max(1, ceil_div((int64_t)n * words, 256))), dim3(256), 0, st, c->d_stage, n,
                     stride, c->d_slots, c->d_uses, c->d_last, c->d_log_count);
  e = hipGetLastError();
  if (e != hipSuccess) return ot_fail_hip(e, "n-gram cache: patch launch");
  // the stream has been idle since this call began and the kernel above does not touch the entries
  uint32_t used = c->log_replayed;
  while (used < (uint32_t)kCacheLogCap && c->h_log[used].x != 0) ++used;
  std::memset(c->h_log, 0, sizeof(uint2) * used);
  c->log_pending = false;
  c->log_replayed = 0;
  return OT_OK;
}

int validate_entries(ot_ctx* ctx, const char* who, int32_t n, const int32_t* key_off, const int32_t* key_ids,
                     const int32_t* target_ids) {
  if (n < 0) return ot_fail(OT_ERR_SHAPE, "%s: n_entries < 0", who);
  if (n > 0 && (!key_off || !key_ids || !target_ids)) return ot_fail(OT_ERR_NULL, "%s: NULL entry arrays", who);
  const char* what = "";
  const int bad = check_entries(n, key_off, key_ids, target_ids, ctx->max_ngram_len, ctx->V_d, ctx->V_t, &what);
  if (bad) return ot_fail(OT_ERR_NGRAM, "%s: entry %d: %s (V_d = %d, V_t = %d, max_ngram_len = %d)", who, bad - 1, what, ctx->V_d,
                          ctx->V_t, ctx->max_ngram_len);
  return OT_OK;
}

// Start of every maintenance call: no step may be probing the table while it changes, and the host table first
// catches up with what the device did.
int begin_maintenance(ot_ngram_cache* c, const char* who) {
  hipError_t he = hipStreamQuery(c->owner->stream);                 // cheap when the stream is idle already
  if (he == hipErrorNotReady) he = hipStreamSynchronize(c->owner->stream);
  if (he != hipSuccess) return ot_fail_hip(he, who);
  return pull_use_log(c);
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
  c->owner = ctx;
  try {
    c->tab.init(capacity, policy, ctx->max_ngram_len);
  } catch (const std::bad_alloc&) {
    delete c;
    return ot_fail(OT_ERR_NOMEM, "ot_ngram_cache_create: host allocation failed");
  }
  const size_t slots = c->tab.slots(), words = c->tab.table().size();
  const size_t stage_words = (size_t)kCachePatchCap * (3 + c->tab.stride());
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&c->d_slots), words * sizeof(int32_t));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->d_uses), slots * sizeof(uint32_t));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->d_last), slots * sizeof(uint32_t));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->d_log_count), sizeof(uint32_t));
  // pinned host memory that the device reads (patch) and writes (use log) in place
  if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void**>(&c->h_stage), stage_words * sizeof(uint32_t), hipHostMallocMapped);
  if (e == hipSuccess) e = hipHostGetDevicePointer(reinterpret_cast<void**>(&c->d_stage), c->h_stage, 0);
  if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void**>(&c->h_log), (size_t)kCacheLogCap * sizeof(uint2), hipHostMallocMapped);
  if (e == hipSuccess) e = hipHostGetDevicePointer(reinterpret_cast<void**>(&c->d_log), c->h_log, 0);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    ot_ngram_cache_destroy(c);
    return ot_fail(OT_ERR_NOMEM, "ot_ngram_cache_create: allocation failed");
  }
  e = hipMemset(c->d_slots, 0, words * sizeof(int32_t));
  if (e == hipSuccess) e = hipMemset(c->d_uses, 0, slots * sizeof(uint32_t));
  if (e == hipSuccess) e = hipMemset(c->d_last, 0, slots * sizeof(uint32_t));
  if (e == hipSuccess) e = hipMemset(c->d_log_count, 0, sizeof(uint32_t));
  if (e == hipSuccess) std::memset(c->h_log, 0, (size_t)kCacheLogCap * sizeof(uint2));
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
  if (n_entries == 0) return OT_OK;                            // nothing to add: not even a tick of the clock

  const int64_t fresh = c->tab.count_fresh(n_entries, key_off, key_ids);
  const bool overflow = (int64_t)c->tab.size() + fresh > c->tab.capacity();
  if (overflow && (c->tab.policy() == OT_EVICT_NONE || c->tab.capacity() == 0))
    return ot_fail(OT_ERR_SHAPE, "ot_ngram_cache_insert: %lld new keys do not fit into %d free places and the cache has no "
                   "eviction policy", (long long)fresh, c->tab.capacity() - c->tab.size());
  if ((rc = begin_maintenance(c, "ot_ngram_cache_insert: synchronize")) != OT_OK) return rc;
  int32_t evicted = 0;
  try {
    evicted = c->tab.insert(n_entries, key_off, key_ids, target_ids);
  } catch (const std::bad_alloc&) {
    return ot_fail(OT_ERR_NOMEM, "ot_ngram_cache_insert: host allocation failed");
  }
  if ((rc = push_changes(c)) != OT_OK) return rc;
  if (n_evicted) *n_evicted = evicted;
  return OT_OK;
}

int ot_ngram_cache_import(ot_ngram_cache* c, int32_t n_entries, const int32_t* key_off, const int32_t* key_ids,
                          const int32_t* target_ids, const int64_t* uses, const int64_t* last_used) {
  if (!c) return ot_fail(OT_ERR_NULL, "ot_ngram_cache_import: cache is NULL");
  int rc = validate_entries(c->owner, "ot_ngram_cache_import", n_entries, key_off, key_ids, target_ids);
  if (rc != OT_OK) return rc;
  if (n_entries == 0) return OT_OK;
  if (!uses || !last_used) return ot_fail(OT_ERR_NULL, "ot_ngram_cache_import: uses and last_used must not be NULL");
  for (int32_t e = 0; e < n_entries; ++e)
    if (uses[e] < 0 || uses[e] > 0xFFFFFFFFll || last_used[e] < 0 || last_used[e] > 0xFFFFFFFFll)
      return ot_fail(OT_ERR_SHAPE, "ot_ngram_cache_import: entry %d carries statistics outside 0..2^32-1", e);
  const int64_t fresh = c->tab.count_fresh(n_entries, key_off, key_ids);
  if ((int64_t)c->tab.size() + fresh > c->tab.capacity())
    return ot_fail(OT_ERR_SHAPE, "ot_ngram_cache_import: %lld new keys do not fit into %d free places (an import evicts nothing)",
                   (long long)fresh, c->tab.capacity() - c->tab.size());
  if ((rc = begin_maintenance(c, "ot_ngram_cache_import: synchronize")) != OT_OK) return rc;
  try {
    c->tab.import_entries(n_entries, key_off, key_ids, target_ids, uses, last_used);
  } catch (const std::bad_alloc&) {
    return ot_fail(OT_ERR_NOMEM, "ot_ngram_cache_import: host allocation failed");
  }
  return push_changes(c);
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
  *n_entries = c->tab.size();
  if (n_key_ids) *n_key_ids = (int32_t)c->tab.total_key_ids();
  return OT_OK;
}

int ot_ngram_cache_export(ot_ngram_cache* c, int32_t max_entries, int32_t max_key_ids, int32_t* key_off,
                          int32_t* key_ids, int32_t* target_ids, int64_t* uses, int64_t* last_used) {
  if (!c || !key_off || !key_ids || !target_ids) return ot_fail(OT_ERR_NULL, "ot_ngram_cache_export: NULL argument");
  int rc = begin_maintenance(c, "ot_ngram_cache_export: synchronize");
  if (rc != OT_OK) return rc;
  if (max_entries < c->tab.size()) return ot_fail(OT_ERR_SHAPE, "ot_ngram_cache_export: room for %d entries, cache holds %d", max_entries, c->tab.size());
  if (max_key_ids < c->tab.total_key_ids()) return ot_fail(OT_ERR_SHAPE, "ot_ngram_cache_export: room for %d key ids is not enough", max_key_ids);
  c->tab.export_entries(key_off, key_ids, target_ids, uses, last_used);
  return push_changes(c);        // nothing changed on the host; clears the device log that was just replayed
}

void ot_ngram_cache_destroy(ot_ngram_cache* cache) {
  if (!cache) return;
  if (cache->owner) (void)hipStreamSynchronize(cache->owner->stream);
  if (cache->d_slots) (void)hipFree(cache->d_slots);
  if (cache->d_uses) (void)hipFree(cache->d_uses);
  if (cache->d_last) (void)hipFree(cache->d_last);
  if (cache->d_log_count) (void)hipFree(cache->d_log_count);
  if (cache->h_log) (void)hipHostFree(cache->h_log);
  if (cache->h_stage) (void)hipHostFree(cache->h_stage);
  delete cache;
}

}  // extern "C"
#pragma GCC visibility pop
