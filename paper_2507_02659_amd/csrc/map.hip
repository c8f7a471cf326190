// Translation of a drafted window into the target vocabulary (Section "Cross-vocabulary N-gram Cache", Eq. 1).
//
// One wavefront per sequence.  Lane i owns draft position i: it merges that draft row's softmax partials,
// forms log q_i(d_i), and probes the n-gram table for every window (i, L), longest first.  Lane 0 then walks
// the window left to right: a cache hit of length L at position s yields one target token whose log q' is the
// sum of the L sub-token log-probabilities (the product of Eq. 1, kept in log space so that five or six
// factors of 1e-6 do not underflow); otherwise the direct image of d_s; a draft id with neither ends the
// proposal.  The kernel touches a few KB and is latency bound.
#include "otv_internal.h"

namespace otv {
namespace {

__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

__device__ inline int cache_lookup(const CacheTable& C, const int32_t* ids, int L) {
  uint32_t h = hash_ngram(ids, L) & C.mask;
  for (uint32_t probe = 0; probe <= C.mask; ++probe) {     // bounded: the table is never more than half full
    const int32_t* slot = C.slots + (size_t)h * C.stride;
    const int sl = slot[0];
    if (sl == 0) return -1;
    if (sl == L) {
      bool same = true;
      for (int i = 0; i < L; ++i) same = same && (slot[2 + i] == ids[i]);
      if (same) return slot[1];
    }
    h = (h + 1) & C.mask;
  }
  return -1;
}

__global__ __launch_bounds__(64) void map_kernel(StepArgs a) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const int r0 = a.row_off[b];
  const int k = a.row_off[b + 1] - r0 - 1;
  const int q0 = r0 - b;
  __shared__ int32_t s_d[64];
  __shared__ double s_logq[64];
  __shared__ int32_t s_hit_len[64];
  __shared__ int32_t s_hit_tok[64];

  // rows of this sequence start out unmapped
  if (lane <= k) {
    a.out.mapped_ids[r0 + lane] = -1;
    a.out.span_start[r0 + lane] = -1;
    a.out.span_len[r0 + lane] = 0;
    a.logq_map[r0 + lane] = 0.0;
  }
  int d = 0;
  bool bad = false;
  if (lane < k) {
    d = a.draft_ids[q0 + lane];
    bad = d < 0 || d >= a.V_d;
  }
  s_d[lane] = d;
  if (__any(bad)) {
    if (lane == 0) {
      a.out.n_mapped[b] = 0;
      a.out.hits_proposed[b] = 0;
      a.out.flags[b] = OT_FLAG_BAD_ID;
      a.s_end[b] = 0;
    }
    return;
  }
  const float Td = a.draft_temperature ? a.draft_temperature[b] : a.temperature[b];

  // ---- draft-row statistics and log q_i(d_i)
  if (lane < k) {
    const int64_t o = (int64_t)(q0 + lane) * a.nchd;
    float mx = a.dpart_max[o];
    int arg = a.dpart_arg[o];
    for (int c = 1; c < a.nchd; ++c) {
      if (a.dpart_max[o + c] > mx) { mx = a.dpart_max[o + c]; arg = a.dpart_arg[o + c]; }
    }
    const double invT = Td > 0.f ? 1.0 / (double)Td : 1.0;
    double S = 0.0;
    for (int c = 0; c < a.nchd; ++c) S += a.dpart_sum[o + c] * exp(((double)a.dpart_max[o + c] - (double)mx) * invT);
    a.drow_max[q0 + lane] = mx;
    a.drow_sum[q0 + lane] = S;
    a.drow_arg[q0 + lane] = arg;
    double lq;
    if (Td > 0.f) {
      const int64_t at = (int64_t)(q0 + lane) * a.V_d + d;
      const float zq = a.dtype == OT_BF16 ? bf16_to_f32(static_cast<const uint16_t*>(a.draft_logits)[at])
                                          : static_cast<const float*>(a.draft_logits)[at];
      lq = ((double)zq - (double)mx) * invT - log(S);
    } else {
      lq = (d == arg) ? 0.0 : -INFINITY;
    }
    s_logq[lane] = lq;
    a.logq_tok[q0 + lane] = lq;
  }
  __syncthreads();

  // ---- longest cache hit starting at each position
  int hit_len = 0, hit_tok = -1;
  if (lane < k && a.cache.slots != nullptr) {
    int Lmax = min(a.cache.max_len, k - lane);
    for (int L = Lmax; L >= 2; --L) {
      const int t = cache_lookup(a.cache, &s_d[lane], L);
      if (t >= 0) { hit_len = L; hit_tok = t; break; }
    }
  }
  s_hit_len[lane] = hit_len;
  s_hit_tok[lane] = hit_tok;
  __syncthreads();

  // ---- greedy left-to-right walk
  if (lane == 0) {
    int s = 0, j = 0, hits = 0, flags = 0;
    while (s < k) {
      int L, t;
      if (s_hit_len[s] > 0) {
        L = s_hit_len[s]; t = s_hit_tok[s]; ++hits;
      } else {
        t = a.dmap[s_d[s]];
        L = 1;
        if (t < 0) { flags |= OT_FLAG_UNMAPPABLE; break; }
      }
      double lq = 0.0;
      for (int l = 0; l < L; ++l) lq += s_logq[s + l];
      a.out.mapped_ids[r0 + j] = t;
      a.out.span_start[r0 + j] = s;
      a.out.span_len[r0 + j] = L;
      a.logq_map[r0 + j] = lq;
      s += L;
      ++j;
    }
    a.out.n_mapped[b] = j;
    a.out.hits_proposed[b] = hits;
    a.out.flags[b] = flags;
    a.s_end[b] = s;
  }
}

}  // namespace

hipError_t launch_map(const StepArgs& a, hipStream_t stream) {
  if (a.B == 0) return hipSuccess;
  hipLaunchKernelGGL(map_kernel, dim3(a.B), dim3(64), 0, stream, a);
  return hipGetLastError();
}

}  // namespace otv
