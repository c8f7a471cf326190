// Acceptance test, residual mass and final-token draw (Algorithm 1, rejection sampling and free-token steps;
// residual norm(max(0, p - q')) of the Notation paragraph with q' extended over the target vocabulary by Eq. 2).
//
//   accept_kernel      one wavefront per sequence.  Lane j merges the softmax partials of row j, forms
//                      p_j(t_j), the ratio min(1, p/q') and its Philox uniform; acceptance tests at different
//                      positions are independent given (u_j, p_j(t_j), q'_j), so the sequential "stop at the
//                      first rejection" is a ballot + find-first-set, not a loop.
//   resid_sums_kernel  for the one row per sequence where the final token is drawn: mass of max(0, p - q')
//                      (and of p, the fallback) per tile of kResidTile target ids, in binary64.
//   resid_pick_kernel  walks the tile masses in ascending order to the tile that holds u * total, re-forms
//                      that tile and finds the first id whose running sum exceeds the target.
//
// Everything that decides an integer (acceptance, the CDF crossing) is evaluated in binary64 from the fp32
// logits, so that differences to a float64 reference stem only from the logits and the row sums.
#include "otv_internal.h"

namespace otv {
namespace {

__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies and key-mixed xors.
__device__ inline void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1,
                                     uint32_t out[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

__device__ inline double u24(uint32_t w) { return (double)(w >> 8) * (1.0 / 16777216.0); }

__global__ __launch_bounds__(64) void accept_kernel(StepArgs a) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const int r0 = a.row_off[b];
  const int k = a.row_off[b + 1] - r0 - 1;
  const int q0 = r0 - b;
  const float T = a.temperature[b];
  const double invT = T > 0.f ? 1.0 / (double)T : 1.0;
  const int flags = a.out.flags[b];
  const int m = a.out.n_mapped[b];

  // ---- row statistics (all k+1 rows, also for bad-id sequences: they are part of the diagnostics view)
  float mx = 0.f;
  double S = 1.0;
  int arg = 0;
  if (lane <= k) {
    const int64_t o = (int64_t)(r0 + lane) * a.ncht;
    mx = a.tpart_max[o];
    arg = a.tpart_arg[o];
    for (int c = 1; c < a.ncht; ++c) {
      if (a.tpart_max[o + c] > mx) { mx = a.tpart_max[o + c]; arg = a.tpart_arg[o + c]; }
    }
    S = 0.0;
    for (int c = 0; c < a.ncht; ++c) S += a.tpart_sum[o + c] * exp(((double)a.tpart_max[o + c] - (double)mx) * invT);
    a.row_max[r0 + lane] = mx;
    a.row_sum[r0 + lane] = S;
    a.row_arg[r0 + lane] = arg;
  }

  FinalInfo fin;
  fin.mode = 0; fin.row = r0; fin.drow = 0; fin.t_ng = -1; fin.t_pre = -1; fin.pad = 0;
  fin.pi = 0.0; fin.q_pre = 0.0; fin.u2 = 0.0;

  if (flags & OT_FLAG_BAD_ID) {
    if (lane <= k) {
      a.out.out_tokens[r0 + lane] = -1;
      a.out.p_tok[r0 + lane] = 0.f; a.out.q_tok[r0 + lane] = 0.f; a.out.ratio[r0 + lane] = 0.f;
    }
    if (lane == 0) {
      a.out.n_accept[b] = 0; a.out.n_accept_draft[b] = 0; a.out.n_emit[b] = 0; a.out.hits_accepted[b] = 0;
      a.fin[b] = fin;
    }
    return;
  }

  // ---- acceptance test of mapped position `lane`
  const uint32_t k0 = (uint32_t)a.seed, k1 = (uint32_t)(a.seed >> 32);
  const uint64_t sid = a.seq_id[b];
  bool ok = true;               // lanes >= m do not veto
  int t_j = -1, L_j = 0;
  double pt = 0.0, qp = 0.0, ratio = 0.0;
  if (lane < m) {
    t_j = a.out.mapped_ids[r0 + lane];
    L_j = a.out.span_len[r0 + lane];
    const double lq = a.logq_map[r0 + lane];
    qp = exp(lq);
    if (T > 0.f) {
      const double z = (double)a.Z[(int64_t)(r0 + lane) * a.ldz + t_j];
      pt = exp((z - (double)mx) * invT) / S;
      if (qp > 0.0) ratio = fmin(1.0, pt / qp);
      else ratio = pt > 0.0 ? 1.0 : 0.0;
      uint32_t w[4];
      philox4x32_10((uint32_t)lane, a.step, (uint32_t)sid, (uint32_t)(sid >> 32), k0, k1, w);
      ok = u24(w[0]) < ratio;
    } else {
      ok = (t_j == arg);
      pt = ok ? 1.0 : 0.0;
      ratio = pt;
    }
  }
  if (lane <= k) {
    a.out.p_tok[r0 + lane] = (float)pt;
    a.out.q_tok[r0 + lane] = (float)qp;
    a.out.ratio[r0 + lane] = (float)ratio;
  }
  const unsigned long long rejected = __ballot(!ok);
  const int n = rejected ? (int)__ffsll((long long)rejected) - 1 : m;     // first rejection, or m

  // ---- accepted tokens, counts
  // (a greedy sequence's final token is the argmax of row n, which lane n holds)
  if (lane <= k) a.out.out_tokens[r0 + lane] = (lane < n) ? t_j : ((lane == n && !(T > 0.f)) ? arg : -1);
  const unsigned long long acc_mask = n >= 64 ? ~0ull : ((1ull << n) - 1ull);
  int len_acc = (lane < n) ? L_j : 0;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) len_acc += __shfl_xor(len_acc, off);
  const int hits_acc = __popcll(__ballot(lane < n && L_j > 1) & acc_mask);

  // ---- final token at row n: values live in lane n
  const int fin_span_s = __shfl((lane < m) ? a.out.span_start[r0 + lane] : 0, n);
  const int fin_L = __shfl(L_j, n);
  const int fin_t = __shfl(t_j, n);
  const double fin_qp = __shfl(qp, n);
  if (lane == 0) {
    a.out.n_accept[b] = n;
    a.out.n_accept_draft[b] = len_acc;
    a.out.hits_accepted[b] = hits_acc;
    a.out.n_emit[b] = n + 1;
    fin.row = r0 + n;
    if (T > 0.f) {
      uint32_t w[4];
      philox4x32_10((uint32_t)n, a.step, (uint32_t)sid, (uint32_t)(sid >> 32), k0, k1, w);
      fin.u2 = u24(w[1]);
      const bool unmappable = (flags & OT_FLAG_UNMAPPABLE) != 0;
      if (n == m && !unmappable) {
        fin.mode = 2;
      } else {
        fin.mode = 3;
        const int s = (n < m) ? fin_span_s : a.s_end[b];
        fin.drow = q0 + s;
        if (n < m && fin_L > 1) {
          const int d1 = a.draft_ids[q0 + s];
          fin.t_ng = fin_t;
          fin.pi = fin_qp;
          fin.t_pre = a.dmap[d1];
          fin.q_pre = exp(a.logq_tok[q0 + s]) - fin_qp;
        }
      }
    }
    a.fin[b] = fin;
  }
}

// p(v) and q'(v) of Eq. 2 at the final row of one sequence.
struct FinalRow {
  const float* z;
  double mx, invT, invS;
  const void* zq;
  int dtype;
  double mxq, invTd, invSq;
  int argq;
  bool greedy_draft;
  const int32_t* tmap;
  int t_ng, t_pre;
  double pi, q_pre;
  bool residual;

  __device__ inline double p(int v) const { return exp(((double)z[v] - mx) * invT) * invS; }
  __device__ inline double qprime(int v) const {
    double q = 0.0;
    const int dv = tmap[v];
    if (dv >= 0) {
      if (greedy_draft) {
        q = (dv == argq) ? 1.0 : 0.0;
      } else {
        const float x = dtype == OT_BF16 ? bf16_to_f32(static_cast<const uint16_t*>(zq)[dv])
                                         : static_cast<const float*>(zq)[dv];
        q = exp(((double)x - mxq) * invTd) * invSq;
      }
    }
    if (v == t_pre) q = q_pre;
    if (v == t_ng) q = pi;       // the n-gram case of Eq. 2 wins when both name the same id
    return q;
  }
  __device__ inline double r(int v, double pv) const { return residual ? fmax(0.0, pv - qprime(v)) : pv; }
};

__device__ inline FinalRow make_final_row(const StepArgs& a, int b, const FinalInfo& f) {
  FinalRow R;
  const float T = a.temperature[b];
  R.z = a.Z + (int64_t)f.row * a.ldz;
  R.mx = (double)a.row_max[f.row];
  R.invT = 1.0 / (double)T;
  R.invS = 1.0 / a.row_sum[f.row];
  R.residual = f.mode == 3;
  R.dtype = a.dtype;
  R.tmap = a.tmap;
  R.t_ng = f.t_ng; R.t_pre = f.t_pre; R.pi = f.pi; R.q_pre = f.q_pre;
  R.zq = nullptr; R.mxq = 0.0; R.invTd = 1.0; R.invSq = 1.0; R.argq = -1; R.greedy_draft = false;
  if (R.residual) {
    const float Td = a.draft_temperature ? a.draft_temperature[b] : T;
    const size_t esz = a.dtype == OT_BF16 ? 2 : 4;
    R.zq = static_cast<const char*>(a.draft_logits) + (size_t)f.drow * a.V_d * esz;
    R.mxq = (double)a.drow_max[f.drow];
    R.greedy_draft = !(Td > 0.f);
    R.invTd = R.greedy_draft ? 1.0 : 1.0 / (double)Td;
    R.invSq = 1.0 / a.drow_sum[f.drow];
    R.argq = a.drow_arg[f.drow];
  }
  return R;
}

__device__ inline double block_sum_256(double x, double* s_tmp) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
  const int wave = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) s_tmp[wave] = x;
  __syncthreads();
  return s_tmp[0] + s_tmp[1] + s_tmp[2] + s_tmp[3];
}

__global__ __launch_bounds__(256) void resid_sums_kernel(StepArgs a) {
  const int b = blockIdx.y, tile = blockIdx.x;
  const FinalInfo f = a.fin[b];
  if (f.mode == 0) return;
  const FinalRow R = make_final_row(a, b, f);
  const int v0 = tile * kResidTile;
  const int v1 = min(a.V_t, v0 + kResidTile);
  double sr = 0.0, sp = 0.0;
  for (int v = v0 + threadIdx.x; v < v1; v += 256) {
    const double pv = R.p(v);
    sp += pv;
    sr += R.r(v, pv);
  }
  __shared__ double s_tmp[4];
  sr = block_sum_256(sr, s_tmp);
  sp = block_sum_256(sp, s_tmp);
  if (threadIdx.x == 0) {
    a.tile_r[(int64_t)b * a.ntiles + tile] = sr;
    a.tile_p[(int64_t)b * a.ntiles + tile] = sp;
  }
}

__global__ __launch_bounds__(256) void resid_pick_kernel(StepArgs a) {
  const int b = blockIdx.x, tid = threadIdx.x;
  const FinalInfo f = a.fin[b];
  if (f.mode == 0) return;
  FinalRow R = make_final_row(a, b, f);
  __shared__ int s_tile;
  __shared__ int s_fallback;
  __shared__ double s_base, s_target;
  __shared__ double s_part[256];
  __shared__ int s_first, s_last;
  if (tid == 0) {
    const double* tr = a.tile_r + (int64_t)b * a.ntiles;
    double total = 0.0;
    for (int t = 0; t < a.ntiles; ++t) total += tr[t];
    int fallback = 0;
    if (!(total > 0.0)) {                 // residual of zero mass: draw from p
      fallback = 1;
      tr = a.tile_p + (int64_t)b * a.ntiles;
      total = 0.0;
      for (int t = 0; t < a.ntiles; ++t) total += tr[t];
      a.out.flags[b] |= OT_FLAG_RESID_ZERO;
    }
    const double target = f.u2 * total;
    double cum = 0.0;
    int pick = -1, last_nonzero = 0;
    for (int t = 0; t < a.ntiles; ++t) {
      if (tr[t] > 0.0) last_nonzero = t;
      if (cum + tr[t] > target) { pick = t; break; }
      cum += tr[t];
    }
    if (pick < 0) {                       // rounding pushed the target past the last tile
      pick = last_nonzero;
      cum = 0.0;
      for (int t = 0; t < pick; ++t) cum += tr[t];
    }
    s_tile = pick; s_base = cum; s_target = target; s_fallback = fallback;
    s_first = 0x7FFFFFFF; s_last = -1;
  }
  __syncthreads();
  if (s_fallback) R.residual = false;
  const double target = s_target;
  // thread t owns 16 consecutive ids of the tile, so the running sum is formed in ascending id order
  constexpr int kPer = kResidTile / 256;
  const int v0 = s_tile * kResidTile + tid * kPer;
  double rv[kPer];
  double local = 0.0;
#pragma unroll
  for (int e = 0; e < kPer; ++e) {
    const int v = v0 + e;
    rv[e] = v < a.V_t ? R.r(v, R.p(v)) : 0.0;
    local += rv[e];
  }
  s_part[tid] = local;
  __syncthreads();
  if (tid == 0) {                          // exclusive scan of the 256 thread masses, in order
    double run = s_base;
    for (int t = 0; t < 256; ++t) { const double x = s_part[t]; s_part[t] = run; run += x; }
  }
  __syncthreads();
  double c = s_part[tid];
  int first = 0x7FFFFFFF, last = -1;
#pragma unroll
  for (int e = 0; e < kPer; ++e) {
    c += rv[e];
    if (rv[e] > 0.0) {
      last = v0 + e;
      if (first == 0x7FFFFFFF && c > target) first = v0 + e;
    }
  }
  if (first != 0x7FFFFFFF) atomicMin(&s_first, first);
  if (last >= 0) atomicMax(&s_last, last);
  __syncthreads();
  if (tid == 0) a.out.out_tokens[f.row] = (s_first != 0x7FFFFFFF) ? s_first : s_last;
}

}  // namespace

hipError_t launch_accept(const StepArgs& a, hipStream_t stream) {
  if (a.B == 0) return hipSuccess;
  hipLaunchKernelGGL(accept_kernel, dim3(a.B), dim3(64), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_resid_sums(const StepArgs& a, hipStream_t stream) {
  if (a.B == 0) return hipSuccess;
  hipLaunchKernelGGL(resid_sums_kernel, dim3(a.ntiles, a.B), dim3(256), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_resid_pick(const StepArgs& a, hipStream_t stream) {
  if (a.B == 0) return hipSuccess;
  hipLaunchKernelGGL(resid_pick_kernel, dim3(a.B), dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace otv
