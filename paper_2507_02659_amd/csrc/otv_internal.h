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

// What the drafted ids of one sequence look up, none of which needs the target's logits: per draft position the longest
// n-gram cache hit that starts there, the drafted id's own logit and its direct image.  Written by a workgroup of the
// LM-head launch, read by the launch that follows it (which walks the window, Eq. 1, and tests acceptance).
struct ProbeRecord {
  unsigned long long hit[64];   // (length << 60) | (slot << 32) | target, 0 = no hit
  float zq[64];                 // draft logit of the drafted id
  int32_t dm[64];               // direct image of the drafted id, or -1
  int32_t bad;                  // a drafted id was outside [0, V_d)
  int32_t pad[3];
};

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

// Softmax statistics of one piece of a draft row: (maximum, lowest index of it within the row, sum of
// exp((x - maximum) / T_d)).  The LM-head launch shares the K draft rows out over `workers` of its workgroups, one job
// each: the first `more` rows are cut into `base + 1` equal pieces (whole 16-byte vectors), the others into `base`
// (at most kDraftPieces), and the launch that follows merges a row's pieces in ascending order.  With fewer workers
// than rows a job takes whole rows, every `workers`-th.
constexpr int kDraftPieces = 3;
struct DraftPiece { float mx; int32_t arg; double sum; };
static_assert(sizeof(DraftPiece) == 16, "one 16-byte record");
struct PiecePlan {
  int32_t workers, base, more;
  __host__ __device__ int pieces(int q) const { return q < more ? base + 1 : base; }
  __host__ __device__ int jobs(int K) const {
    const int64_t all = (int64_t)more * (base + 1) + (int64_t)(K - more) * base;
    return (int)(all < workers ? all : workers);
  }
  // job -> (row, piece index); rows q + workers, q + 2 workers, ... follow when workers < K (then base == 1, more == 0)
  __host__ __device__ void locate(int job, int* q, int* i) const {
    const int split = more * (base + 1);
    if (job < split) { *q = job / (base + 1); *i = job % (base + 1); }
    else { *q = more + (job - split) / base; *i = (job - split) % base; }
  }
  // elements [e0, e0 + n) of a V-element row that piece i of P covers (n <= 0: nothing)
  __host__ __device__ static void span(int V, int P, int i, int* e0, int* n) {
    const int len = ((V + P - 1) / P + 7) / 8 * 8;
    *e0 = i * len;
    *n = (V - *e0 < len ? V - *e0 : len);
  }
};
inline PiecePlan make_piece_plan(int workers, int K) {
  PiecePlan p{workers, 1, 0};
  if (workers >= K && K > 0) {
    p.base = workers / K < kDraftPieces ? workers / K : kDraftPieces;
    p.more = p.base < kDraftPieces ? (workers - p.base * K < K ? workers - p.base * K : K) : 0;
  }
  return p;
}

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
  DraftPiece* dpiece;    // [K, kDraftPieces] statistics of the pieces of the draft rows, left by the LM-head launch
  PiecePlan plan;        // how the LM-head launch shared out the draft rows
  ProbeRecord* probe;    // [B] what the drafted ids of each sequence look up (see ProbeRecord), left by the LM-head launch
  int32_t hosted;        // the LM-head launch left the target rows' softmax partials (`fused`), the draft rows' pieces
                         // and the probe records: one launch follows it, which translates, tests and draws
  int32_t chunked;       // the statistics launch left chunk partials (tpart_*, dpart_*) and the probe records: the same
                         // one launch follows it (at most kFusedMaxB sequences)
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
// (n_cu = compute units of the device: the column width of a workgroup is chosen so that the launch takes few rounds.)
int lmhead_bf16_fused_partials(int M, int Vp, int n_cu);
// Whether a step of this shape lets the LM-head launch host the draft side and emit the partials (else the step runs
// the statistics and the translation as launches of their own).
bool lmhead_bf16_hosts_draft_side(int M, int d, int Vp, int B, int K, int V_d, int n_cu);
// workgroups of launch_lmhead_bf16 that share the draft rows (0: that shape leaves no partials and hosts nothing)
int lmhead_bf16_draft_workers(int M, int Vp, int B, int K, int n_cu);
// `fused` may be nullptr or have part == nullptr (no statistics); otherwise fused->nfine must be
// lmhead_bf16_fused_partials(M, Vp, n_cu) > 0 and fused->B <= kFusedMaxB.  With fused statistics and `draft_side` not
// nullptr, the workgroups of the launch also compute the softmax statistics of the draft rows of *draft_side (one row
// each, before their main loop) into its drow_* arrays.
hipError_t launch_lmhead_bf16(const uint16_t* H, int M, int d, const uint16_t* Wp, int Kp, int Vp, float* Z, int V_t,
                              int64_t ldz, const uint16_t* zeros, const FusedStats* fused, const StepArgs* draft_side,
                              int n_cu, hipStream_t stream);
hipError_t launch_lmhead_f32(const float* H, int M, int d, const float* W, float* Z, int V_t, int64_t ldz,
                             hipStream_t stream);
hipError_t launch_softmax_stats(const StepArgs& a, hipStream_t stream);
hipError_t launch_translate_accept(const StepArgs& a, hipStream_t stream);
// translation and acceptance test (when the LM-head launch hosted the draft side) and the draw of the final tokens
hipError_t launch_final_draw(const StepArgs& a, const int32_t* row_off_host, hipStream_t stream);

}  // namespace otv
