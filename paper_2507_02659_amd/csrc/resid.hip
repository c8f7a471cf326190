// Final token of every sequence (Algorithm 1: correction token from the residual, or free token from p).
//
// At the first rejected row the token is drawn from norm(max(0, p - q')) (Notation paragraph), with q' extended over
// the whole target vocabulary by Eq. 2: q'(v) = q_s(tmap[v]) through the inverse direct map (0 where v has no
// pre-image), except that the n-gram matched at this position gets the product pi of its sub-token probabilities
// and the direct image of its first sub-token gets q_s(d_1) - pi.  When everything was accepted the draw is from p.
//
// Only the ONE row per sequence where the draw happens is touched.
//   resid_sums_kernel  grid = (tiles of kResidTile target ids) x (sequences): the mass of max(0, p - q') of each
//                      tile in binary64 (and the mass of p, the fallback when the residual is empty).
//   resid_pick_kernel  one workgroup per sequence: a wavefront scan walks the tile masses in ascending order to
//                      the tile that holds u * total; the tile is re-formed with each thread owning 4 consecutive
//                      ids, the running sum is scanned in ascending id order and the first id whose running sum
//                      exceeds the target is emitted (inverse CDF).
#include "device_math.h"
#include "otv_internal.h"

namespace otv {
namespace {

constexpr int kThreads = 256;
constexpr int kPer = kResidTile / kThreads;   // 4 ids per thread
static_assert(kPer == 4, "the fixed summation trees below are written for 4 ids per thread");

// p(v) and q'(v) of Eq. 2 at the final row of one sequence.
struct FinalRow {
  const float* z;
  float mx, sc_hi, sc_lo;        // row maximum; log2(e) / T split into two floats
  double invS;
  const void* zq;
  int dtype;
  float mxq, scq_hi, scq_lo;     // the same for the draft row
  double invSq;
  int argq;
  bool greedy_draft;
  bool residual;
  const int32_t* tmap;
  int t_ng, t_pre;
  double pi, q_pre;

  // exp((x - max) / T) / S for x <= max.  The exponent goes through the hardware 2^x in binary32: the difference to the
  // row maximum is formed in binary32 (its rounding is random, not a bias), the scale is applied as a two-float
  // product so that its own rounding does not tilt the whole row, and the normaliser is applied in binary64.  Relative
  // error about 2e-7 per value, unbiased; the running sums over the vocabulary are binary64.
  __device__ static inline double softmax_term(float x, float mx, float sc_hi, float sc_lo, double invS) {
    const float d = x - mx;
    return (double)__builtin_amdgcn_exp2f(fmaf(d, sc_hi, d * sc_lo)) * invS;
  }
  __device__ inline double p_of(float zv) const { return softmax_term(zv, mx, sc_hi, sc_lo, invS); }
  __device__ inline float draft_logit(int dv) const {
    return dtype == OT_BF16 ? bf16_to_f32(static_cast<const uint16_t*>(zq)[dv]) : static_cast<const float*>(zq)[dv];
  }
  // q'(v) given the draft id dv = tmap[v] (or -1) and, when dv >= 0 and the draft is not greedy, its logit
  __device__ inline double qprime(int v, int dv, float xq) const {
    double q = 0.0;
    if (dv >= 0) q = greedy_draft ? ((dv == argq) ? 1.0 : 0.0) : softmax_term(xq, mxq, scq_hi, scq_lo, invSq);
    if (v == t_pre) q = q_pre;
    if (v == t_ng) q = pi;       // the n-gram case of Eq. 2 wins when both name the same id
    return q;
  }
};

__device__ inline FinalRow make_final_row(const StepArgs& a, const FinalInfo& f) {
  FinalRow R;
  R.z = a.Z + (int64_t)f.row * a.ldz;
  const double sc = f.invT * 1.4426950408889634, scq = f.invTd * 1.4426950408889634;
  R.mx = (float)f.mx; R.sc_hi = (float)sc; R.sc_lo = (float)(sc - (double)R.sc_hi); R.invS = f.invS;
  R.residual = f.mode == 3;
  R.dtype = a.dtype;
  R.tmap = a.tmap;
  R.t_ng = f.t_ng; R.t_pre = f.t_pre; R.pi = f.pi; R.q_pre = f.q_pre;
  R.zq = static_cast<const char*>(a.draft_logits) + (size_t)f.drow * a.V_d * (a.dtype == OT_BF16 ? 2 : 4);
  R.mxq = (float)f.mxq; R.scq_hi = (float)scq; R.scq_lo = (float)(scq - (double)R.scq_hi); R.invSq = f.invSq; R.argq = f.argq; R.greedy_draft = f.greedy_draft != 0;
  return R;
}

// Inverse direct map of kPer ids v = first + e * stride (independent of which row is drawn from: issued early).
__device__ inline void load_tmap(const int32_t* __restrict__ tmap, int V_t, int first, int stride, int* dv) {
#pragma unroll
  for (int e = 0; e < kPer; ++e) {
    const int v = first + e * stride;
    dv[e] = v < V_t ? tmap[v] : -1;
  }
}

// Residual mass r(v) and p(v) for kPer ids v = first + e * stride.  All loads are issued before any arithmetic.
__device__ inline void tile_values(const FinalRow& R, int V_t, int first, int stride, const int* dv, double* r,
                                   double* p) {
  float zv[kPer];
  float xq[kPer];
#pragma unroll
  for (int e = 0; e < kPer; ++e) {
    const int v = first + e * stride;
    zv[e] = v < V_t ? R.z[v] : -INFINITY;
    xq[e] = (R.residual && dv[e] >= 0 && !R.greedy_draft) ? R.draft_logit(dv[e]) : 0.f;
  }
#pragma unroll
  for (int e = 0; e < kPer; ++e) {
    const int v = first + e * stride;
    p[e] = v < V_t ? R.p_of(zv[e]) : 0.0;
    r[e] = (R.residual && v < V_t) ? fmax(0.0, p[e] - R.qprime(v, dv[e], xq[e])) : p[e];
  }
}

__global__ __launch_bounds__(kThreads) void resid_sums_kernel(StepArgs a) {
  const int b = blockIdx.y, tile = blockIdx.x, tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  int dv[kPer];
  load_tmap(a.tmap, a.V_t, tile * kResidTile + tid, kThreads, dv);     // does not depend on the row: overlaps the next load
  const FinalInfo f = a.fin[b];
  if (f.mode == 0) return;                  // greedy or flagged sequence: nothing to draw
  const FinalRow R = make_final_row(a, f);
  __shared__ double s_w[2][kThreads / 64];

  // ---- mass of this tile (coalesced: consecutive threads on consecutive ids)
  {
    double r[kPer], p[kPer];
    tile_values(R, a.V_t, tile * kResidTile + tid, kThreads, dv, r, p);
    double sr = (r[0] + r[1]) + (r[2] + r[3]);
    double sp = (p[0] + p[1]) + (p[2] + p[3]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) { sr += __shfl_xor(sr, off); sp += __shfl_xor(sp, off); }
    if (lane == 0) { s_w[0][wave] = sr; s_w[1][wave] = sp; }
    __syncthreads();
    if (tid == 0) {
      a.tile_r[(int64_t)b * a.ntiles + tile] = (s_w[0][0] + s_w[0][1]) + (s_w[0][2] + s_w[0][3]);
      a.tile_p[(int64_t)b * a.ntiles + tile] = (s_w[1][0] + s_w[1][1]) + (s_w[1][2] + s_w[1][3]);
    }
  }
}

__global__ __launch_bounds__(kThreads) void resid_pick_kernel(StepArgs a) {
  const int b = blockIdx.x, tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  __shared__ double s_w[2][kThreads / 64];
  extern __shared__ double s_tiles[];       // [2][ntiles]: residual masses, then p masses
  __shared__ int s_pick, s_fallback, s_first, s_lastnz;
  __shared__ double s_base, s_target;
  // the tile masses do not depend on the outcome record: both loads are in flight together
  for (int t = tid; t < a.ntiles; t += kThreads) {
    s_tiles[t] = a.tile_r[(int64_t)b * a.ntiles + t];
    s_tiles[a.ntiles + t] = a.tile_p[(int64_t)b * a.ntiles + t];
  }
  const FinalInfo f = a.fin[b];
  if (f.mode == 0) return;
  FinalRow R = make_final_row(a, f);
  __syncthreads();
  if (wave == 0) {
    // Running mass over the tiles in ascending order, in place: wavefront scan of 64 tiles at a time plus a carry.
    // The total and the crossing both come from these same sums.
    auto prefix = [&](double* m) -> double {
      double carry = 0.0;
      for (int t0 = 0; t0 < a.ntiles; t0 += 64) {
        const int t = t0 + lane;
        double incl = t < a.ntiles ? m[t] : 0.0;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
          const double up = __shfl_up(incl, off);
          if (lane >= off) incl += up;
        }
        incl += carry;
        if (t < a.ntiles) m[t] = incl;
        carry = __shfl(incl, 63);
      }
      return carry;
    };
    double* m = s_tiles;
    double total = prefix(m);
    const int fallback = !(total > 0.0);    // residual of zero mass: draw from p
    if (fallback) {
      m = s_tiles + a.ntiles;
      total = prefix(m);
    }
    const double target = f.u2 * total;
    int pick = -1;
    for (int t0 = 0; t0 < a.ntiles && pick < 0; t0 += 64) {
      const int t = t0 + lane;
      const unsigned long long hit = __ballot(t < a.ntiles && m[t] > target);
      if (hit) pick = t0 + (int)__ffsll((long long)hit) - 1;
    }
    if (pick < 0) {                          // rounding pushed the target past the end: take the last tile that adds mass
      pick = 0;
      for (int t = 1; t < a.ntiles; ++t) if (m[t] > m[t - 1]) pick = t;
    }
    const double base = pick > 0 ? m[pick - 1] : 0.0;
    if (lane == 0) {
      if (fallback) a.out.flags[b] |= OT_FLAG_RESID_ZERO;
      s_pick = pick; s_base = base; s_target = target; s_fallback = fallback;
      s_first = 0x7FFFFFFF; s_lastnz = -1;
    }
  }
  __syncthreads();
  if (s_fallback) R.residual = false;
  const double target = s_target;
  const int v0 = s_pick * kResidTile + tid * kPer;       // thread owns kPer consecutive ids: ascending running sum
  double r[kPer], p[kPer];
  int dv[kPer];
  load_tmap(a.tmap, a.V_t, v0, 1, dv);
  tile_values(R, a.V_t, v0, 1, dv, r, p);
  const double local = ((r[0] + r[1]) + r[2]) + r[3];
  double incl = local;                                   // inclusive scan over the wavefront, fixed order
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const double up = __shfl_up(incl, off);
    if (lane >= off) incl += up;
  }
  double excl = __shfl_up(incl, 1);
  if (lane == 0) excl = 0.0;
  if (lane == 63) s_w[0][wave] = incl;
  __syncthreads();
  double before = s_base;
  for (int w = 0; w < wave; ++w) before += s_w[0][w];
  double c = before + excl;
  int first = 0x7FFFFFFF, last = -1;
#pragma unroll
  for (int e = 0; e < kPer; ++e) {
    c += r[e];
    if (r[e] > 0.0) {
      last = v0 + e;
      if (first == 0x7FFFFFFF && c > target) first = v0 + e;
    }
  }
  if (first != 0x7FFFFFFF) atomicMin(&s_first, first);
  if (last >= 0) atomicMax(&s_lastnz, last);
  __syncthreads();
  if (tid == 0) a.out.out_tokens[f.row] = (s_first != 0x7FFFFFFF) ? s_first : s_lastnz;
}

}  // namespace

hipError_t launch_resid_sums(const StepArgs& a, hipStream_t stream) {
  if (a.B == 0) return hipSuccess;
  hipLaunchKernelGGL(resid_sums_kernel, dim3(a.ntiles, a.B), dim3(kThreads), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_resid_pick(const StepArgs& a, hipStream_t stream) {
  if (a.B == 0) return hipSuccess;
  hipLaunchKernelGGL(resid_pick_kernel, dim3(a.B), dim3(kThreads), 2 * a.ntiles * sizeof(double), stream, a);
  return hipGetLastError();
}

}  // namespace otv
