// Internal declarations shared by the host API and the kernel translation units of libotverify.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ngram_table.h"
#include "otverify.h"

namespace otv {

// ------------------------------------------------------------------------------------------------ geometry
constexpr int kStatThreads = 256;
constexpr int kStatChunk = 8192;     // logits per workgroup of the softmax-statistics kernel (measured: 4096 and 16384 are slower)
constexpr int kResidTile = 1024;     // vocabulary entries per workgroup of the residual kernel
constexpr int kGemmColsPerWave = 64; // LM-head columns owned by one wavefront
constexpr int kGemmKPad = 128;       // packed K extent is a multiple of this
// Gap, in 16-byte units, between the packed weights of consecutive 64-column tiles.  Without it the tiles of a
// d = 4096 head are exactly 512 KB apart and the hundreds of weight streams that run side by side, all at the same
// depth, differ only in high address bits; measured LM-head time at 144 rows: no gap 205 us, 4 KB 243 us (worst),
// 16 KB 201 us, 16.1 KB 197.5 us, 48.1 KB 199 us (d = 3584 heads: no measurable difference).
constexpr int kGemmTileGapUnits = 1032;
// 16-byte units from one 64-column tile of the packed weights to the next (nks 32-deep steps of 4 fragments each)
constexpr int64_t packed_tile_units(int nks) { return (int64_t)nks * 256 + kGemmTileGapUnits; }
constexpr int kLossRowBytes = 128;   // size of the per-token record of the distillation-loss kernels

inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

// ------------------------------------------------------------------------------------------------ n-gram table
// Open addressing, linear probing.  Slot = { len, target, ids[max_len] } as int32; len == 0 marks an empty slot.
struct CacheTable {
  const int32_t* slots;
  uint32_t mask;       // slots - 1, slots a power of two >= 2 * capacity
  int32_t stride;      // int32 words per slot = 2 + max_len
  int32_t max_len;
  uint32_t* uses;      // [slots] incremented for every use of the entry by the translation scan
  uint32_t* last_used; // [slots] set to `clock` on use
  uint32_t clock;      // logical time of this step
  uint32_t* log_count; // device word: uses logged since the log was last cleared (a use beyond the capacity is only counted)
  uint2* log;          // [kCacheLogCap] (slot + 1, clock) of those uses, in pinned HOST memory that the device writes
                       // directly: the maintenance calls read it without a copy; 0 marks an entry not written yet
};
constexpr int kCacheLogCap = 4096;    // uses the device can log between two maintenance calls of a cache
constexpr int kCachePatchCap = 1024;  // slots that travel as a packed patch; more than that uploads the arrays whole

// ------------------------------------------------------------------------------------------------ per-step view
// What the final-token kernels need to know about sequence b; written by the translate-and-accept kernel.
struct FinalInfo {
  int32_t mode;          // 0: nothing to draw (greedy, or bad id), 2: draw from p (free token), 3: draw from the residual
  int32_t row;           // global row of the final token (row_off[b] + n_b)
  int32_t drow;          // global draft row whose distribution fills Eq. 2's "otherwise" branch
  int32_t t_ng;          // target id of the n-gram matched at the rejected position, or -1
  int32_t t_pre;         // direct image of that n-gram's first sub-token, or -1
  int32_t argq;          // argmax of the draft row (used when the draft temperature is 0)
  int32_t greedy_draft;  // draft temperature is 0: q is one-hot at argq
  int32_t pad;
  double pi;             // product of the n-gram's sub-token probabilities
  double q_pre;          // q(d_1) - pi
  double u2;             // uniform of the draw
  // p(v) = exp((z_v - mx) * invT) * invS at the final row; q_s(d) = exp((zq_d - mxq) * invTd) * invSq at draft row drow
  double mx, invT, invS, mxq, invTd, invSq;
};

// One mapped position of a translated proposal, parked in memory between the kernel that translates (it needs only the
// drafter's side of the step) and the kernel that tests acceptance (it needs the target's logits).  Entry
// row_off[b] + j belongs to mapped position j of sequence b; j == n_mapped is filled when the proposal was cut by an
// untranslatable id (its `start` is that id's draft position).
struct RowProposal {
  int32_t t;             // target id t_j, or -1 beyond the proposal
  int32_t start, len;    // draft positions covered
  int32_t t_pre;         // direct image of the draft id at `start` (Eq. 2, prefix case), or -1
  int32_t argq;          // argmax of the draft row at `start`
  float mxq;             // maximum of that row
  double lq;             // log q'(t_j): sum of the sub-tokens' log-probabilities (Eq. 1)
  double lq_first;       // log q(d) of the draft id at `start`
  double Sq;             // sum of exponentials of that row
  int32_t pad[4];
};
static_assert(sizeof(RowProposal) == 64, "one record per 64 bytes");

// Softmax partial of one row over one column tile: maximum, its lowest column, sum of exp((z - mx) / T).
struct alignas(16) Partial {
  float mx;
  int32_t arg;
  double sum;
};
static_assert(sizeof(Partial) == 16, "stored and loaded as one 16-byte vector");

// Softmax partials emitted by the LM-head epilogue (one per row and column tile of the kernel), so that the logits
// need not be read again for their row statistics.  part == nullptr: not wanted.
constexpr int kFusedMaxB = 255;      // sequences whose row offsets and temperatures the LM-head kernel stages in LDS
struct FusedStats {
  const int32_t* row_off;            // [B + 1]
  const float* temperature;          // [B]
  int32_t B;
  int32_t nfine;                     // partials per row (row stride of `part`)
  Partial* part;                     // [M, nfine]
};

struct StepArgs {
  // problem
  int32_t B, M, K, d, V_t, V_d, dtype, max_ngram_len;
  uint32_t step;
  uint64_t seed;
  // inputs (device)
  const int32_t* row_off;
  const void* hidden;
  const void* draft_logits;
  const int32_t* draft_ids;
  const float* temperature;
  const float* draft_temperature;
  const uint64_t* seq_id;
  const int32_t* dmap;   // [V_d]
  const int32_t* tmap;   // [V_t]
  CacheTable cache;      // slots == nullptr: no cache
  // workspace (device)
  const float* Z;        // [M, ldz]
  int64_t ldz;
  int32_t ncht, nchd;    // statistic chunks per target / draft row
  float* tpart_max; double* tpart_sum; int32_t* tpart_arg;   // [M, ncht]
  FusedStats fused;      // fused.nfine > 0: the LM head left fine partials; the statistics kernel merges them per row
  float* dpart_max; double* dpart_sum; int32_t* dpart_arg;   // [K, nchd]
  float* row_max; double* row_sum; int32_t* row_arg;         // [M]
  float* drow_max; double* drow_sum; int32_t* drow_arg;      // [K]
  RowProposal* proposal; // [M] written by the draft side when it runs apart from the acceptance test
  int32_t pre_translated; // the draft side has already run (inside the LM-head launch): `proposal`, drow_* and the
                         // translation outputs are final; the acceptance kernel only merges the LM head's partials
  FinalInfo* fin;        // [B]
  int32_t ntiles;        // residual tiles per row
  double* tile_r; double* tile_p;                            // [B, ntiles]
  int32_t* resid_count;  // [B] tile workgroups of the residual launch that have delivered their mass; 0 between launches
  // outputs (device)
  ot_step_out out;
};

// ------------------------------------------------------------------------------------------------ launchers
// Each returns the hipError_t of its launch.  All work goes to `stream`.
hipError_t launch_pack_w_bf16(const uint16_t* W, int d, int V_t, uint16_t* Wp, int Kp, int Vp, hipStream_t stream);
// Partials per row that launch_lmhead_bf16 emits for M rows of a Vp-column (padded) head; 0: that shape runs a
// kernel without the fused statistics.
int lmhead_bf16_fused_partials(int M, int Vp);
// Whether a step of this shape lets the LM-head launch host the draft side and emit the partials (else the step runs
// the statistics and the translation as launches of their own).
bool lmhead_bf16_hosts_draft_side(int M, int d, int Vp, int B, int K, int V_d);
// `fused` may be nullptr or have part == nullptr (no statistics); otherwise fused->nfine must be
// lmhead_bf16_fused_partials(M, Vp) > 0 and fused->B <= kFusedMaxB.  With fused statistics and `draft_side` not
// nullptr, extra workgroups of the same launch run the draft side of the step (draft row statistics, translation,
// parked proposals: everything of *draft_side that does not need the logits), hidden behind the weight stream.
hipError_t launch_lmhead_bf16(const uint16_t* H, int M, int d, const uint16_t* Wp, int Kp, int Vp, float* Z, int V_t,
                              int64_t ldz, const uint16_t* zeros, const FusedStats* fused, const StepArgs* draft_side,
                              hipStream_t stream);
hipError_t launch_lmhead_f32(const float* H, int M, int d, const float* W, float* Z, int V_t, int64_t ldz,
                             hipStream_t stream);
hipError_t launch_softmax_stats(const StepArgs& a, hipStream_t stream);
hipError_t launch_translate_accept(const StepArgs& a, hipStream_t stream);
// acceptance test (when the draft side ran inside the LM-head launch) and the draw of the final tokens
hipError_t launch_final_draw(const StepArgs& a, const int32_t* row_off_host, hipStream_t stream);

}  // namespace otv
