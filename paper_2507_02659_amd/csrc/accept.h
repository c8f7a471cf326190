// Acceptance test of a translated proposal (Algorithm 1, rejection-sampling step) as device functions: the merge of
// softmax partials into row statistics, and the test itself, which one wavefront runs for a whole sequence.
//
// Lane j owns mapped position j: it forms p_j(t_j), the ratio min(1, p/q') and its Philox uniform; acceptance tests at
// different positions are independent given (u_j, p_j(t_j), q'_j), so "stop at the first rejection" is a ballot and a
// find-first-set, not a loop.  The outcome is the FinalInfo record of the sequence: where and from what the final token
// is drawn.
#pragma once

#include "translate.h"

namespace otv {

// Merges the chunk partials of up to 64 rows starting at row `first`: 4 threads per row, every 4th chunk each,
// combined in a fixed order.  Thread 4*r publishes row r's (max, sum, argmax) to LDS and to the workspace.
__device__ inline void merge_partials(const float* __restrict__ pmax, const double* __restrict__ psum,
                                      const int32_t* __restrict__ parg, int nch, int first, int n_rows, double invT,
                                      float* s_mx, double* s_S, int* s_arg, float* g_mx, double* g_S, int32_t* g_arg,
                                      int local_tid) {
  const int row = local_tid >> 2, part = local_tid & 3;
  const bool live = row < n_rows;
  const int64_t o = (int64_t)(first + (live ? row : 0)) * nch;
  float mx = -INFINITY;
  int arg = 0x7FFFFFFF;
  if (live) {
    for (int c = part; c < nch; c += 4) {
      const float m = pmax[o + c];
      const int ai = parg[o + c];
      if (m > mx || (m == mx && ai < arg)) { mx = m; arg = ai; }
    }
  }
#pragma unroll
  for (int off = 1; off <= 2; off <<= 1) {
    const float om = __shfl_xor(mx, off);
    const int oa = __shfl_xor(arg, off);
    if (om > mx || (om == mx && oa < arg)) { mx = om; arg = oa; }
  }
  double S = 0.0;
  if (live) {
    for (int c = part; c < nch; c += 4) S += psum[o + c] * exp(((double)pmax[o + c] - (double)mx) * invT);
  }
  const double s1 = __shfl_xor(S, 1);
  const double lo = (part & 1) ? s1 + S : S + s1;          // (part0 + part1) or (part2 + part3), same order in both lanes
  const double s2 = __shfl_xor(lo, 2);
  const double total = (part & 2) ? s2 + lo : lo + s2;     // (p0 + p1) + (p2 + p3)
  if (live && part == 0) {
    s_mx[row] = mx; s_S[row] = total; s_arg[row] = arg;
    g_mx[first + row] = mx; g_S[first + row] = total; g_arg[first + row] = arg;
  }
}

// Lanes of a wavefront hold running statistics r of parts of one row (exponent scale sc): merges them by shuffles in a
// fixed order; lane 0 publishes the row's (max, sum, argmax) to LDS slot `at` and, if asked, to the workspace.
__device__ inline void wave_publish_row(const RunStat& r, float sc, int row, int lane, float* s_mx, double* s_S,
                                        int* s_arg, int at, bool to_workspace, float* g_mx, double* g_S, int32_t* g_arg) {
  float mx = r.mx;
  int arg = r.arg;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float om = __shfl_xor(mx, off);
    const int oa = __shfl_xor(arg, off);
    if (om > mx || (om == mx && oa < arg)) { mx = om; arg = oa; }
  }
  double S = r.mx == -INFINITY ? 0.0 : r.sum * (double)__builtin_amdgcn_exp2f((r.mx - mx) * sc);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) S += __shfl_xor(S, off);
  if (lane == 0) {
    s_mx[at] = mx; s_S[at] = S; s_arg[at] = arg;
    if (to_workspace) { g_mx[row] = mx; g_S[row] = S; g_arg[row] = arg; }
  }
}

// Merges the LM head's partials of one target row (nfine of them, one per column tile): called by a whole wavefront.
// A lane requests eight 16-byte partials at a time before it looks at any of them (one round trip to memory for up
// to 512 tiles) and keeps a running maximum with the sum rescaled to it; the lanes are then merged by shuffles.  Sums
// are rescaled and added in binary64, in a fixed order.  Lane 0 publishes the row's (max, sum, argmax) to LDS and to
// the workspace.
__device__ inline void merge_fused_row(const Partial* __restrict__ part, int nfine, int row, double invT, int lane,
                                       float* s_mx, double* s_S, int* s_arg, int at, bool to_workspace, float* g_mx,
                                       double* g_S, int32_t* g_arg) {
  const uint4* p = reinterpret_cast<const uint4*>(part + (int64_t)row * nfine);
  const float sc = (float)invT * kLog2eF;
  RunStat r;
  for (int c0 = 0; c0 < nfine; c0 += 512) {
    uint4 raw[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int c = c0 + j * 64 + lane;
      raw[j] = c < nfine ? p[c] : make_uint4(0xFF800000u, 0x7FFFFFFFu, 0u, 0u);     // (-inf, no column, 0.0)
    }
    float bm = -INFINITY;
    int bi = 0x7FFFFFFF;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float m = __uint_as_float(raw[j].x);
      const int ai = (int)raw[j].y;
      if (m > bm || (m == bm && ai < bi)) { bm = m; bi = ai; }
    }
    if (bm > r.mx || (bm == r.mx && bi < r.arg)) {
      r.sum *= (double)__builtin_amdgcn_exp2f((r.mx - bm) * sc);
      r.mx = bm; r.arg = bi;
    }
    if (r.mx != -INFINITY) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float m = __uint_as_float(raw[j].x);
        const double sum = __hiloint2double((int)raw[j].w, (int)raw[j].z);
        r.sum += sum * (double)__builtin_amdgcn_exp2f((m - r.mx) * sc);              // empty: 0 * exp2(-inf) = 0
      }
    }
  }
  wave_publish_row(r, sc, row, lane, s_mx, s_S, s_arg, at, to_workspace, g_mx, g_S, g_arg);
}

// The same for the chunk partials of the statistics launch (three arrays, nch entries per row): lane c takes chunks
// c, c + 64, ...
__device__ inline void merge_chunk_row(const float* __restrict__ pmax, const double* __restrict__ psum,
                                       const int32_t* __restrict__ parg, int nch, int row, double invT, int lane,
                                       float* s_mx, double* s_S, int* s_arg, int at, bool to_workspace, float* g_mx,
                                       double* g_S, int32_t* g_arg) {
  const int64_t o = (int64_t)row * nch;
  const float sc = (float)invT * kLog2eF;
  RunStat r;
  for (int c = lane; c < nch; c += 64) {
    const float m = pmax[o + c];
    const int ai = parg[o + c];
    const double sum = psum[o + c];
    if (m > r.mx || (m == r.mx && ai < r.arg)) {
      r.sum *= (double)__builtin_amdgcn_exp2f((r.mx - m) * sc);        // r.mx = -inf: the sum is 0 and stays 0
      r.mx = m; r.arg = ai;
    }
    if (m != -INFINITY) r.sum += sum * (double)__builtin_amdgcn_exp2f((m - r.mx) * sc);
  }
  wave_publish_row(r, sc, row, lane, s_mx, s_S, s_arg, at, to_workspace, g_mx, g_S, g_arg);
}

// Statistics of draft row q from the chunk partials of the statistics launch (ascending chunks): lane-local.
__device__ inline void merge_draft_chunks(const StepArgs& a, int q, float Td, float* out_mx, double* out_S, int* out_arg) {
  const int64_t o = (int64_t)q * a.nchd;
  const float sc = Td > 0.f ? kLog2eF / Td : kLog2eF;
  float bm = -INFINITY;
  int ba = 0x7FFFFFFF;
  for (int c = 0; c < a.nchd; ++c) {
    const float m = a.dpart_max[o + c];
    if (m > bm) { bm = m; ba = a.dpart_arg[o + c]; }       // ascending chunks: a later equal maximum does not replace
  }
  double total = 0.0;
  for (int c = 0; c < a.nchd; ++c) {
    const float m = a.dpart_max[o + c];
    if (m != -INFINITY) total += a.dpart_sum[o + c] * (double)__builtin_amdgcn_exp2f((m - bm) * sc);
  }
  *out_mx = bm; *out_S = total; *out_arg = ba;
}

// The acceptance test of sequence b by one wavefront (lane = mapped position).  P is the lane's proposal (P.m, P.flags
// wavefront-uniform), s_pmx / s_pS / s_parg the statistics of the sequence's target rows; z_tok, if `have_z`, is
// z[row lane, t_lane] fetched by the caller.  With write_out the per-row and per-sequence outputs of the test are
// written.  Returns the outcome record (valid in lane 0).
__device__ inline FinalInfo accept_wave(const StepArgs& a, int b, int r0, int k, int q0, float T, float Td, double invT,
                                        double invTd, uint64_t sid, const LaneProposal& P, bool have_z, float z_tok,
                                        const float* s_pmx, const double* s_pS, const int* s_parg, int lane,
                                        bool write_out) {
  FinalInfo fin;
  fin.mode = 0; fin.row = r0; fin.drow = 0; fin.t_ng = -1; fin.t_pre = -1; fin.argq = -1; fin.greedy_draft = 0;
  fin.pad = 0; fin.pi = 0.0; fin.q_pre = 0.0; fin.u2 = 0.0;
  fin.mx = 0.0; fin.invT = 1.0; fin.invS = 1.0; fin.mxq = 0.0; fin.invTd = 1.0; fin.invSq = 1.0;
  if (P.flags & OT_FLAG_BAD_ID) {   // a drafted id outside [0, V_d): the sequence emits nothing
    if (write_out) {
      if (lane <= k) {
        a.out.out_tokens[r0 + lane] = -1;
        a.out.p_tok[r0 + lane] = 0.f; a.out.ratio[r0 + lane] = 0.f;
      }
      if (lane == 0) { a.out.n_accept[b] = 0; a.out.n_accept_draft[b] = 0; a.out.n_emit[b] = 0; a.out.hits_accepted[b] = 0; }
    }
    return fin;
  }
  const int m = P.m, flags = P.flags;
  const int t_j = P.t, L_j = P.L;
  const uint32_t k0 = (uint32_t)a.seed, k1 = (uint32_t)(a.seed >> 32);
  const float mx = lane <= k ? s_pmx[lane] : 0.f;
  const double S = lane <= k ? s_pS[lane] : 1.0;
  const int arg = lane <= k ? s_parg[lane] : 0;
  bool ok = true;               // lanes >= m do not veto
  double pt = 0.0, qp = 0.0, ratio = 0.0;
  uint32_t w[4] = {0, 0, 0, 0};  // the uniforms of row `lane`: word 0 tests mapped position `lane`, word 1 draws its final token
  if (T > 0.f && lane <= k) philox4x32_10((uint32_t)lane, a.step, (uint32_t)sid, (uint32_t)(sid >> 32), k0, k1, w);
  if (lane < m) {
    qp = exp(P.lq);
    if (T > 0.f) {
      const double z = (double)(have_z ? z_tok : a.Z[(int64_t)(r0 + lane) * a.ldz + t_j]);
      pt = exp((z - (double)mx) * invT) / S;
      if (qp > 0.0) ratio = fmin(1.0, pt / qp);
      else ratio = pt > 0.0 ? 1.0 : 0.0;
      ok = u24(w[0]) < ratio;
    } else {
      ok = (t_j == arg);
      pt = ok ? 1.0 : 0.0;
      ratio = pt;
    }
  }
  const unsigned long long rejected = __ballot(!ok);
  const int n = rejected ? (int)__ffsll((long long)rejected) - 1 : m;     // first rejection, or m
  if (write_out && lane <= k) {
    a.out.p_tok[r0 + lane] = (float)pt;
    a.out.ratio[r0 + lane] = (float)ratio;
    // accepted tokens; a greedy sequence's final token is the argmax of row n, which lane n holds; otherwise entry n
    // belongs to the draw (which may run before or after this store)
    if (lane != n || !(T > 0.f)) a.out.out_tokens[r0 + lane] = (lane < n) ? t_j : (lane == n ? arg : -1);
  }
  int len_acc = (lane < n) ? L_j : 0;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) len_acc += __shfl_xor(len_acc, off);
  const int hits_acc = __popcll(__ballot(lane < n && L_j > 1));

  // ---- final token at row n: its values live in lane n
  const int fin_start = __shfl(P.start, n);
  const int fin_L = __shfl(L_j, n);
  const int fin_t = __shfl(t_j, n);
  const double fin_qp = __shfl(qp, n);
  const float fin_mx = __shfl(mx, n);
  const double fin_S = __shfl(S, n);
  const int fin_t_pre = __shfl(P.t_pre, n);
  const int fin_argq = __shfl(P.argq, n);
  const float fin_mxq = __shfl(P.mxq, n);
  const double fin_Sq = __shfl(P.Sq, n);
  const double fin_lq_first = __shfl(P.lq_first, n);
  const uint32_t fin_w1 = __shfl(w[1], n);
  if (lane == 0) {
    if (write_out) {
      a.out.n_accept[b] = n;
      a.out.n_accept_draft[b] = len_acc;
      a.out.hits_accepted[b] = hits_acc;
      a.out.n_emit[b] = n + 1;
    }
    fin.row = r0 + n;
    if (T > 0.f) {
      fin.u2 = u24(fin_w1);
      fin.mx = (double)fin_mx; fin.invT = invT; fin.invS = 1.0 / fin_S;
      const bool unmappable = (flags & OT_FLAG_UNMAPPABLE) != 0;
      if (n == m && !unmappable) {
        fin.mode = 2;                                   // everything accepted: free token ~ p
      } else {
        fin.mode = 3;                                   // correction token ~ norm(max(0, p - q'))
        fin.drow = q0 + fin_start;                      // the rejected span's first draft row, or the untranslatable id's
        fin.greedy_draft = !(Td > 0.f);
        fin.invTd = invTd;
        fin.mxq = (double)fin_mxq;
        fin.invSq = 1.0 / fin_Sq;
        fin.argq = fin_argq;
        if (n < m && fin_L > 1) {                       // Eq. 2 overrides for the n-gram matched at this position
          fin.t_ng = fin_t;
          fin.pi = fin_qp;
          fin.t_pre = fin_t_pre;
          fin.q_pre = exp(fin_lq_first) - fin_qp;
        }
      }
    }
  }
  return fin;
}

}  // namespace otv
