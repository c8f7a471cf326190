// Translation and acceptance test in one launch, for steps whose draft side has not run inside the LM-head launch:
// one workgroup of 768 threads per sequence.  The three jobs that do not depend on each other run in different
// wavefronts of the workgroup at the same time: threads 0-255 merge the target rows' chunk partials, threads 256-511
// the draft rows' partials, threads 512-767 fetch the drafted ids, their logits and direct images and probe the n-gram
// table (Section "Cross-vocabulary N-gram Cache", Eq. 1); one barrier later the walk and the acceptance test
// (Algorithm 1, rejection-sampling step) need only LDS and one gather of z[t_j].  The outcome record of every sequence
// goes to memory for the launch that draws the final token.
#include "accept.h"

namespace otv {
namespace {

__global__ __launch_bounds__(768) void translate_accept_kernel(StepArgs a) {
  const int b = blockIdx.x, tid = threadIdx.x;
  const int role = tid >> 8, g = tid & 255;          // role 0: target rows, 1: draft rows, 2: ids and table probes
  const int lane = tid & 63;
  const int r0 = a.row_off[b];
  const int k = a.row_off[b + 1] - r0 - 1;
  const int q0 = r0 - b;
  __shared__ DraftLds s_d;
  __shared__ float s_pmx[64];
  __shared__ double s_pS[64];
  __shared__ int s_parg[64];

  const float T = a.temperature[b];
  const float Td = a.draft_temperature ? a.draft_temperature[b] : T;
  const uint64_t sid = a.seq_id[b];
  const double invT = T > 0.f ? 1.0 / (double)T : 1.0;
  const double invTd = Td > 0.f ? 1.0 / (double)Td : 1.0;

  draft_lds_reset(&s_d, tid);
  __syncthreads();
  if (role == 0) {
    merge_partials(a.tpart_max, a.tpart_sum, a.tpart_arg, a.ncht, r0, k + 1, invT, s_pmx, s_pS, s_parg, a.row_max,
                   a.row_sum, a.row_arg, g);
  } else if (role == 1) {
    merge_partials(a.dpart_max, a.dpart_sum, a.dpart_arg, a.nchd, q0, k, invTd, s_d.qmx, s_d.qS, s_d.qarg, a.drow_max,
                   a.drow_sum, a.drow_arg, g);
  } else {
    fetch_ids_and_probe(a, q0, k, g, 256, &s_d);
  }
  __syncthreads();
  if (tid >= 64) return;          // the rest is one wavefront's work
  LaneProposal P;
  P.t = -1; P.start = -1; P.L = 0; P.lq = 0.0; P.t_pre = -1; P.argq = -1; P.mxq = 0.f; P.Sq = 1.0; P.lq_first = 0.0;
  P.m = 0; P.flags = 0;
  if (s_d.bad) {
    translate_bad_sequence(a, b, r0, k, lane);
    P.flags = OT_FLAG_BAD_ID;
  } else {
    translate_walk(a, b, r0, k, q0, Td, invTd, lane, &s_d, &P);
  }
  const FinalInfo fin = accept_wave(a, b, r0, k, q0, T, Td, invT, invTd, sid, P, false, 0.f, s_pmx, s_pS, s_parg, lane, true);
  if (lane == 0) a.fin[b] = fin;
}

}  // namespace

hipError_t launch_translate_accept(const StepArgs& a, hipStream_t stream) {
  if (a.B == 0) return hipSuccess;
  hipLaunchKernelGGL(translate_accept_kernel, dim3(a.B), dim3(768), 0, stream, a);
  return hipGetLastError();
}

}  // namespace otv
