// Host-side structures shared by the translation units that implement the C ABI (api.hip, cache.hip, loss.hip, adapt.hip).
#pragma once

#include <vector>

#include "ngram_table.h"
#include "otv_internal.h"

// Records the message ot_last_error() returns on this thread and hands back `code`.
int ot_fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
int ot_fail_hip(hipError_t e, const char* what);
// Looks up, for the current device, the address of the static scratch array of ot_adaptive_drafting_static.
int ot_static_scratch_prepare();

struct ot_ctx {
  int32_t d = 0, V_t = 0, V_d = 0, max_batch = 0, max_k = 0, dtype = 0, max_ngram_len = 0, draft_side = 0;
  int32_t max_rows = 0, max_K = 0, Kp = 0, Vp = 0, ncht = 0, nchd = 0, ntiles = 0;
  hipStream_t stream = nullptr;
  int device = 0;
  std::vector<void*> allocs;
  uint16_t* Wp = nullptr;
  uint16_t* zeros = nullptr;          // 64 zero bytes: source of the K tail in the LM-head's hidden slices
  float* Wf = nullptr;
  int32_t *dmap = nullptr, *tmap = nullptr;
  float* Z = nullptr;
  float *tpart_max = nullptr, *dpart_max = nullptr, *row_max = nullptr, *drow_max = nullptr;
  double *tpart_sum = nullptr, *dpart_sum = nullptr, *row_sum = nullptr, *drow_sum = nullptr;
  int32_t *tpart_arg = nullptr, *dpart_arg = nullptr, *row_arg = nullptr, *drow_arg = nullptr;
  otv::Partial* fpart = nullptr;      // [max_rows, Vp/256] softmax partials from the LM-head epilogue (bf16)
  int n_cu = 0;                       // compute units of the device
  otv::DraftPiece* dpiece = nullptr;  // [max_K, kDraftPieces] pieces of the draft rows' statistics, as the probe records
  otv::ProbeRecord* probe = nullptr;  // [max_batch] lookups of the drafted ids, between the LM-head launch and the next
  double *tile_r = nullptr, *tile_p = nullptr;
  int32_t* resid_count = nullptr;     // [max_batch] arrival counters of the residual launch, zero between launches
  otv::FinalInfo* fin = nullptr;
  void* loss_rows = nullptr;          // [max_rows] records of kLossRowBytes: per-token constants of the loss kernels
  double* loss_tiles = nullptr;       // [max_rows, ntiles] KL tile sums
  double* adapt_part = nullptr;       // [max_batch, 2] per-sequence partials of the acceptance head's loss
  // profiling
  bool profiling = false;
  std::vector<hipEvent_t> events;   // OT_N_STAGES + 1 per pending step
  int pending = 0;
};

// One n-gram cache: the host table with its statistics and eviction order (plain C++), and the device copy that the
// translation kernel probes.
struct ot_ngram_cache {
  ot_ctx* owner = nullptr;
  otv::NgramTable tab;
  int32_t* d_slots = nullptr;         // device copy of the slots
  uint32_t* d_uses = nullptr;         // [slots] times the translation used the entry
  uint32_t* d_last = nullptr;         // [slots] clock of the last use or (re-)insertion
  uint32_t* d_log_count = nullptr;    // device word: number of uses the device logged since the log was cleared
  uint2* h_log = nullptr;             // [kCacheLogCap] pinned host memory: (slot + 1, clock) of every such use, written by the device
  uint2* d_log = nullptr;             // the same memory as the device addresses it
  uint32_t* h_stage = nullptr;        // pinned host memory that holds a packed patch; the patch kernel reads it in place
  uint32_t* d_stage = nullptr;        // the same memory as the device addresses it
  bool log_pending = false;           // the device log holds entries that have been replayed but not cleared yet
  uint32_t log_replayed = 0;          // how many of them: a call that fails before the log is cleared leaves them
                                      // there, and the next call must not count those uses a second time
};
