// The launches that draw the final token of every sequence (Algorithm 1: correction token from the residual of Eq. 2,
// or free token from p), grid = (groups of 8 tiles of kResidTile target ids) x (sequences).
//   final_draw_kernel   the outcome records of the acceptance test are in memory (written by the launch before).
//   accept_draw_kernel  follows an LM-head launch that hosted the draft side: every workgroup first repeats the
//                       translation and the acceptance test of its sequence (one wavefront merges the pieces of the
//                       draft rows' statistics and walks the window from the probe record while the others merge the
//                       LM head's softmax partials, one wavefront per target row; then that wavefront runs the test:
//                       a few microseconds of work on data that sits in L2, cheaper than a launch of its own), then
//                       takes part in the draw.  The workgroups of a sequence reach the same outcome; only group 0
//                       writes the outputs of the translation and the test, the draft rows' merged statistics and
//                       the cache's use statistics.
#include "accept.h"
#include "resid.h"

namespace otv {
namespace {

__global__ __launch_bounds__(kDrawThreads) void final_draw_kernel(StepArgs a) {
  const int b = blockIdx.y, grp = blockIdx.x, tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  extern __shared__ double s_tiles[];       // [2][ntiles]: residual masses, then p masses
  __shared__ DrawLds s_draw;
  int dv[kPerLane];
  load_tmap<kPerLane>(a.tmap, a.V_t, draw_first_id(grp, wave, lane), 64, dv);   // overlaps the next load
  const FinalInfo f = a.fin[b];
  if (f.mode == 0) return;                  // greedy or flagged sequence: nothing to draw
  draw_final_token(a, b, grp, f, dv, &s_draw, s_tiles);
}

// Row offsets of the sequences as a kernel argument (the host has them): the workgroup knows its rows without a
// dependent load in front of everything else.
struct RowOffsets { int32_t v[kFusedMaxB + 1]; };
constexpr int64_t kRepeatedMergeBytes = 32 << 20;

// kDraw = false: grid = (1) x (sequences); the workgroup only runs the test and leaves the outcome record in memory for
// a final_draw_kernel launch (used when repeating the test in every tile group would cost more than a launch).
// kChunks: the partials come from the statistics launch (chunk partials in three arrays per side) instead of the
// LM head's epilogue and draft-row pieces.
template <bool kDraw, bool kChunks>
__global__ __launch_bounds__(kDrawThreads) void accept_draw_kernel(StepArgs a, RowOffsets ro) {
  const int b = blockIdx.y, grp = blockIdx.x, tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  extern __shared__ double s_tiles[];
  __shared__ DrawLds s_draw;
  __shared__ DraftLds s_d;
  __shared__ FinalInfo s_fin;
  __shared__ float s_pmx[64];
  __shared__ double s_pS[64];
  __shared__ int s_parg[64];
  int dv[kPerLane];

  const int r0 = ro.v[b];
  const int k = ro.v[b + 1] - r0 - 1;
  const float T = a.temperature[b];
  const float Td = a.draft_temperature ? a.draft_temperature[b] : T;
  const uint64_t sid = a.seq_id[b];
  const double invT = T > 0.f ? 1.0 / (double)T : 1.0;
  const double invTd = Td > 0.f ? 1.0 / (double)Td : 1.0;
  const bool lead = grp == 0;               // the group that writes the test's outputs and the row statistics
  if (!(T > 0.f) && !lead) return;          // a greedy sequence draws nothing: its other groups have nothing to do

  // The LM-head launch left what the drafted ids look up (ProbeRecord) and the draft rows' statistics.  The last
  // wavefront fetches them (one load of each array per lane), walks the window (Eq. 1) and asks for the logits of the
  // proposed tokens, all on its own, while the other wavefronts merge the softmax partials of the target rows; the
  // translation is thus repeated by every tile group of the sequence, and the lead group writes its outputs and the
  // cache's use statistics.
  const int q0 = r0 - b;
  constexpr int kTestWave = kDrawWaves - 1;   // runs the walk and the test
  LaneProposal P;
  P.t = -1; P.start = -1; P.L = 0; P.lq = 0.0; P.t_pre = -1; P.argq = -1; P.mxq = 0.f; P.Sq = 1.0; P.lq_first = 0.0;
  P.m = 0; P.flags = 0;
  float z_tok = 0.f;
  if (wave == kTestWave) {
    const ProbeRecord* rec = a.probe + b;
    s_d.hit[lane] = rec->hit[lane]; s_d.zq[lane] = rec->zq[lane]; s_d.dm[lane] = rec->dm[lane];
    if (lane < k) {
      float mxq; double Sq; int argq;
      if (kChunks) merge_draft_chunks(a, q0 + lane, Td, &mxq, &Sq, &argq);
      else merge_draft_pieces(a, q0 + lane, Td, &mxq, &Sq, &argq);
      s_d.qmx[lane] = mxq; s_d.qS[lane] = Sq; s_d.qarg[lane] = argq;
      if (lead) { a.drow_max[q0 + lane] = mxq; a.drow_sum[q0 + lane] = Sq; a.drow_arg[q0 + lane] = argq; }
    }
    const int bad = rec->bad;               // wavefront-uniform
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    if (bad) {
      if (lead) translate_bad_sequence(a, b, r0, k, lane);
      P.flags = OT_FLAG_BAD_ID;
    } else {
      translate_walk(a, b, r0, k, q0, Td, invTd, lane, &s_d, &P, lead);
    }
    if (!(P.flags & OT_FLAG_BAD_ID) && lane < P.m && T > 0.f) z_tok = a.Z[(int64_t)(r0 + lane) * a.ldz + P.t];
  }
  for (int row = wave; row <= k; row += kDrawWaves) {
    if (kChunks)
      merge_chunk_row(a.tpart_max, a.tpart_sum, a.tpart_arg, a.ncht, r0 + row, invT, lane, s_pmx, s_pS, s_parg, row, lead,
                      a.row_max, a.row_sum, a.row_arg);
    else
      merge_fused_row(a.fused.part, a.fused.nfine, r0 + row, invT, lane, s_pmx, s_pS, s_parg, row, lead, a.row_max,
                      a.row_sum, a.row_arg);
  }
  // The inverse map of this wavefront's ids is needed last (by the tile masses) and asked for here, behind the loads
  // that the test waits for: loads return in issue order, and asked for first it held those back by its own latency.
  if (kDraw) load_tmap<kPerLane>(a.tmap, a.V_t, draw_first_id(grp, wave, lane), 64, dv);
  __syncthreads();
  if (wave == kTestWave) {
    const FinalInfo fin = accept_wave(a, b, r0, k, q0, T, Td, invT, invTd, sid, P, true, z_tok, s_pmx, s_pS, s_parg, lane, lead);
    if (lane == 0) s_fin = fin;
  }
  if (!kDraw) {
    if (tid == kTestWave * 64) a.fin[b] = s_fin;
    return;
  }
  __syncthreads();
  const FinalInfo f = s_fin;
  if (f.mode == 0) return;
  draw_final_token(a, b, grp, f, dv, &s_draw, s_tiles);
}

}  // namespace

// hosted: the LM-head launch left its softmax partials, the draft rows' pieces and the probe records; chunked: the
// statistics launch left its chunk partials and the probe records (in both cases B <= kFusedMaxB and row_off_host holds
// the B + 1 row offsets); otherwise a.fin is filled.
hipError_t launch_final_draw(const StepArgs& a, const int32_t* row_off_host, hipStream_t stream) {
  if (a.B == 0) return hipSuccess;
  const dim3 grid(ceil_div(a.ntiles, kGroupTiles), a.B), block(kDrawThreads);
  const size_t lds = 2 * (size_t)a.ntiles * sizeof(double);
  if (a.chunked) {
    if (a.B > kFusedMaxB || a.hosted) return hipErrorInvalidValue;
    RowOffsets ro;
    for (int b = 0; b <= kFusedMaxB; ++b) ro.v[b] = row_off_host[b <= a.B ? b : a.B];
    hipLaunchKernelGGL((accept_draw_kernel<true, true>), grid, block, lds, stream, a, ro);   // a few chunks per row: always one launch
    return hipGetLastError();
  }
  if (a.hosted) {
    if (a.B > kFusedMaxB) return hipErrorInvalidValue;
    RowOffsets ro;
    for (int b = 0; b <= kFusedMaxB; ++b) ro.v[b] = row_off_host[b <= a.B ? b : a.B];
    // Every tile group of a sequence repeats the merge of its rows' partials: M x nfine x 16 bytes per group.  Up to
    // about the traffic that costs as much as a launch this is one launch; beyond it the test gets a launch of its own.
    const int64_t repeated = (int64_t)a.M * a.fused.nfine * (int64_t)sizeof(Partial) * grid.x;
    if (repeated <= kRepeatedMergeBytes) {
      hipLaunchKernelGGL((accept_draw_kernel<true, false>), grid, block, lds, stream, a, ro);
      return hipGetLastError();
    }
    hipLaunchKernelGGL((accept_draw_kernel<false, false>), dim3(1, a.B), block, 0, stream, a, ro);
  }
  hipLaunchKernelGGL(final_draw_kernel, grid, block, lds, stream, a);
  return hipGetLastError();
}

}  // namespace otv
