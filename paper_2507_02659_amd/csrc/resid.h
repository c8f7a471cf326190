// Final token of every sequence (Algorithm 1: correction token from the residual, or free token from p), as device
// functions for the kernels that host the draw.
//
// At the first rejected row the token is drawn from norm(max(0, p - q')) (Notation paragraph), with q' extended over
// the whole target vocabulary by Eq. 2: q'(v) = q_s(tmap[v]) through the inverse direct map (0 where v has no
// pre-image), except that the n-gram matched at this position gets the product pi of its sub-token probabilities
// and the direct image of its first sub-token gets q_s(d_1) - pi.  When everything was accepted the draw is from p.
//
// Only the ONE row per sequence where the draw happens is touched.  A workgroup of 16 wavefronts takes 8 consecutive
// tiles of kResidTile target ids of one sequence, two wavefronts per tile:
//   every workgroup  forms the masses of max(0, p - q') of its tiles in binary64 (and the masses of p, the fallback
//                    when the residual is empty), publishes them and counts itself in;
//   the workgroup that arrives last for its sequence  walks the tile masses in ascending order with a wavefront scan
//                    to the tile that holds u * total, re-forms that tile with each thread owning 4 consecutive ids,
//                    scans the running sum in ascending id order and emits the first id whose running sum exceeds the
//                    target (inverse CDF).  Which workgroup that is varies from run to run; what it computes does not.
// Nothing waits: a workgroup that is not last simply ends.
#pragma once

#include "device_math.h"
#include "otv_internal.h"

namespace otv {

constexpr int kDrawWaves = 16;                       // wavefronts per workgroup
constexpr int kDrawThreads = kDrawWaves * 64;
constexpr int kGroupTiles = kDrawWaves / 2;          // tiles per workgroup: two wavefronts share one
constexpr int kPerLane = kResidTile / 128;           // ids per lane while two wavefronts sum one tile
constexpr int kPickThreads = 256;
constexpr int kPer = kResidTile / kPickThreads;      // consecutive ids per thread while the chosen tile is scanned
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
  R.mxq = (float)f.mxq; R.scq_hi = (float)scq; R.scq_lo = (float)(scq - (double)R.scq_hi); R.invSq = f.invSq; R.argq = f.argq;
  R.greedy_draft = f.greedy_draft != 0;
  return R;
}

// Inverse direct map of N ids v = first + e * stride (independent of which row is drawn from: issued early).
template <int N>
__device__ inline void load_tmap(const int32_t* __restrict__ tmap, int V_t, int first, int stride, int* dv) {
#pragma unroll
  for (int e = 0; e < N; ++e) {
    const int v = first + e * stride;
    dv[e] = v < V_t ? tmap[v] : -1;
  }
}

// Stand-in logit of an id that does not exist or has no pre-image: finite, so that the two-float scaling below never
// meets inf * 0, and so far below any maximum that its exponential is exactly 0.
constexpr float kFarBelow = -1e30f;

// Residual mass r(v) and p(v) for N ids v = first + e * stride.  All loads are issued before any arithmetic.  The
// common case (every id below V_t, a sampling drafter, no id of Eq. 2's two overrides among them) runs without any
// per-element test other than "has a pre-image".
template <int N>
__device__ inline void tile_values(const FinalRow& R, int V_t, int first, int stride, const int* dv, double* r,
                                   double* p) {
  float zv[N];
  float xq[N];
  const int last = first + (N - 1) * stride;
  const bool gather = R.residual && !R.greedy_draft;
  if (last < V_t) {
#pragma unroll
    for (int e = 0; e < N; ++e) zv[e] = R.z[first + e * stride];
  } else {
#pragma unroll
    for (int e = 0; e < N; ++e) zv[e] = first + e * stride < V_t ? R.z[first + e * stride] : kFarBelow;
  }
#pragma unroll
  for (int e = 0; e < N; ++e) xq[e] = (gather && dv[e] >= 0) ? R.draft_logit(dv[e]) : kFarBelow;
#pragma unroll
  for (int e = 0; e < N; ++e) p[e] = R.p_of(zv[e]);             // beyond V_t: 2^(-huge) = 0
  if (!R.residual) {
#pragma unroll
    for (int e = 0; e < N; ++e) r[e] = p[e];
    return;
  }
  // wavefront-uniform: does any lane hold an id that Eq. 2 overrides, or is the drafter greedy?
  bool special = R.greedy_draft;
#pragma unroll
  for (int e = 0; e < N; ++e) special = special || first + e * stride == R.t_pre || first + e * stride == R.t_ng;
  if (!__any(special)) {
#pragma unroll
    for (int e = 0; e < N; ++e)                                   // no pre-image: 2^(-huge) = 0
      r[e] = fmax(0.0, p[e] - FinalRow::softmax_term(xq[e], R.mxq, R.scq_hi, R.scq_lo, R.invSq));
  } else {
#pragma unroll
    for (int e = 0; e < N; ++e) {
      const int v = first + e * stride;
      r[e] = v < V_t ? fmax(0.0, p[e] - R.qprime(v, dv[e], xq[e])) : 0.0;
    }
  }
}

// Agent-scope accesses to the tile masses and the arrival counter.  Workgroups of one launch run on different XCDs,
// each with its own L2, and exchange these few words through memory: the stores are write-through, the loads bypass
// the local L2 and the counter lives in memory, so no whole-cache write-back or invalidate is needed.
__device__ inline void publish(double* p, double v) {
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), (unsigned long long)__double_as_longlong(v), __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline double observe(double* p) {
  return __longlong_as_double((long long)__hip_atomic_load(reinterpret_cast<unsigned long long*>(p), __ATOMIC_RELAXED,
                                                           __HIP_MEMORY_SCOPE_AGENT));
}

// first id a lane sums in workgroup `grp`
__device__ inline int draw_first_id(int grp, int wave, int lane) {
  return (grp * kGroupTiles + (wave >> 1)) * kResidTile + (wave & 1) * (kResidTile / 2) + lane;
}

struct DrawLds {
  double half[2][kGroupTiles];   // masses of the second halves of the tiles
  double w[kPickThreads / 64];
  double base, target;
  int pick, fallback, first, lastnz, last;
};

// Workgroup `grp` of sequence b (all kDrawThreads threads call this; f is the sequence's outcome record with
// f.mode != 0; dv holds tmap of the ids draw_first_id(grp, wave, lane) + e * 64, e < kPerLane, of this wavefront's
// half tile).  s_tiles is
// dynamic LDS of 2 * ntiles doubles.
__device__ inline void draw_final_token(const StepArgs& a, int b, int grp, const FinalInfo& f, const int* dv, DrawLds* L,
                                        double* s_tiles) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  FinalRow R = make_final_row(a, f);
  const int n_groups = (a.ntiles + kGroupTiles - 1) / kGroupTiles;

  // ---- masses of this workgroup's tiles: wavefronts 2i and 2i+1 take the two halves of tile i (coalesced:
  // consecutive lanes on consecutive ids), wavefront 2i adds the halves and publishes
  const int tile = grp * kGroupTiles + (wave >> 1);
  double sr = 0.0, sp = 0.0;
  if (tile < a.ntiles) {
    double r[kPerLane], p[kPerLane];
    tile_values<kPerLane>(R, a.V_t, tile * kResidTile + (wave & 1) * (kResidTile / 2) + lane, 64, dv, r, p);
#pragma unroll
    for (int e = 0; e < kPerLane; e += 4) {
      sr += (r[e] + r[e + 1]) + (r[e + 2] + r[e + 3]);
      sp += (p[e] + p[e + 1]) + (p[e + 2] + p[e + 3]);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) { sr += __shfl_xor(sr, off); sp += __shfl_xor(sp, off); }
    if (lane == 0 && (wave & 1)) { L->half[0][wave >> 1] = sr; L->half[1][wave >> 1] = sp; }
  }
  __syncthreads();
  if (tile < a.ntiles && lane == 0 && !(wave & 1)) {
    publish(&a.tile_r[(int64_t)b * a.ntiles + tile], sr + L->half[0][wave >> 1]);
    publish(&a.tile_p[(int64_t)b * a.ntiles + tile], sp + L->half[1][wave >> 1]);
    // the two stores have reached memory before this workgroup is counted
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): vector-memory stores count there as well
    asm volatile("" ::: "memory");
  }
  __syncthreads();
  if (tid == 0) {
    const int arrived = __hip_atomic_fetch_add(&a.resid_count[b], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    L->last = arrived == n_groups - 1;
    if (L->last) __hip_atomic_store(&a.resid_count[b], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next launch
  }
  __syncthreads();
  if (!L->last) return;

  // ---- the last workgroup of the sequence: inverse CDF over the tile masses, then inside the tile that holds the draw
  for (int t = tid; t < a.ntiles; t += kDrawThreads) {
    s_tiles[t] = observe(&a.tile_r[(int64_t)b * a.ntiles + t]);
    s_tiles[a.ntiles + t] = observe(&a.tile_p[(int64_t)b * a.ntiles + t]);
  }
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
      L->pick = pick; L->base = base; L->target = target; L->fallback = fallback;
      L->first = 0x7FFFFFFF; L->lastnz = -1;
    }
  }
  __syncthreads();
  if (L->fallback) R.residual = false;
  const double target = L->target;
  const bool picker = tid < kPickThreads;
  const int v0 = L->pick * kResidTile + tid * kPer;      // a picking thread owns kPer consecutive ids: ascending running sum
  double r[kPer] = {0.0, 0.0, 0.0, 0.0}, p[kPer];
  double excl = 0.0;
  if (picker) {
    int dvp[kPer];
    load_tmap<kPer>(a.tmap, a.V_t, v0, 1, dvp);
    tile_values<kPer>(R, a.V_t, v0, 1, dvp, r, p);
    const double local = ((r[0] + r[1]) + r[2]) + r[3];
    double incl = local;                                 // inclusive scan over the wavefront, fixed order
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const double up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    excl = __shfl_up(incl, 1);
    if (lane == 0) excl = 0.0;
    if (lane == 63) L->w[wave] = incl;
  }
  __syncthreads();
  if (picker) {
    double before = L->base;
    for (int w = 0; w < wave; ++w) before += L->w[w];
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
    if (first != 0x7FFFFFFF) atomicMin(&L->first, first);
    if (last >= 0) atomicMax(&L->lastnz, last);
  }
  __syncthreads();
  if (tid == 0) a.out.out_tokens[f.row] = (L->first != 0x7FFFFFFF) ? L->first : L->lastnz;
}

}  // namespace otv
