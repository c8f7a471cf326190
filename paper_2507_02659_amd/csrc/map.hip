// Translation of a drafted window into the target vocabulary (Section "Cross-vocabulary N-gram Cache", Eq. 1).
//
// One workgroup of 256 threads per sequence.  The draft rows' softmax partials are merged by 4 threads per row,
// thread i then forms log q_i(d_i); every window (start s, length L) of the drafted ids is probed in the n-gram
// table by its own thread; thread 0 walks the window left to right over LDS only: the longest cache hit at s
// yields one target token whose log q' is the sum of the L sub-token log-probabilities (the product of Eq. 1,
// kept in log space so that five or six factors of 1e-6 do not underflow), otherwise the direct image of d_s, and
// a draft id with neither ends the proposal.  The kernel touches a few KB and is latency bound, so every
// dependent global access (ids -> logits / direct map / table slots) is issued by many threads at once.
#include "device_math.h"
#include "otv_internal.h"

namespace otv {
namespace {

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

__global__ __launch_bounds__(256) void map_kernel(StepArgs a) {
  const int b = blockIdx.x, tid = threadIdx.x;
  const int r0 = a.row_off[b];
  const int k = a.row_off[b + 1] - r0 - 1;
  const int q0 = r0 - b;
  __shared__ int32_t s_d[64], s_dm[64];
  __shared__ unsigned long long s_hit[64];   // (length << 32) | target of the longest cache hit starting here, 0 = none
  __shared__ int32_t s_tok[64], s_start[64], s_len[64];
  __shared__ double s_logq[64], s_lq[64];
  __shared__ int s_bad;

  if (tid == 0) s_bad = 0;
  if (tid < 64) { s_hit[tid] = 0ull; s_tok[tid] = -1; s_start[tid] = -1; s_len[tid] = 0; s_lq[tid] = 0.0; }
  __syncthreads();
  int d = 0;
  if (tid < k) {
    d = a.draft_ids[q0 + tid];
    if (d < 0 || d >= a.V_d) { s_bad = 1; d = 0; }
    s_d[tid] = d;
  }
  __syncthreads();
  if (s_bad) {
    if (tid <= k) {
      a.out.mapped_ids[r0 + tid] = -1; a.out.span_start[r0 + tid] = -1; a.out.span_len[r0 + tid] = 0;
      a.logq_map[r0 + tid] = 0.0;
    }
    if (tid == 0) {
      a.out.n_mapped[b] = 0; a.out.hits_proposed[b] = 0; a.out.flags[b] = OT_FLAG_BAD_ID; a.s_end[b] = 0;
    }
    return;
  }
  const float Td = a.draft_temperature ? a.draft_temperature[b] : a.temperature[b];
  const double invT = Td > 0.f ? 1.0 / (double)Td : 1.0;

  // ---- loads that depend only on the ids: the drafted logit and the direct image
  float zq = 0.f;
  if (tid < k) {
    s_dm[tid] = a.dmap[d];
    const int64_t at = (int64_t)(q0 + tid) * a.V_d + d;
    zq = a.dtype == OT_BF16 ? bf16_to_f32(static_cast<const uint16_t*>(a.draft_logits)[at])
                            : static_cast<const float*>(a.draft_logits)[at];
  }

  // ---- draft-row statistics: 4 threads per row, every 4th chunk each, fixed combination order
  {
    const int row = tid >> 2, part = tid & 3;
    const bool live = row < k;
    const int64_t o = (int64_t)(q0 + (live ? row : 0)) * a.nchd;
    float mx = -INFINITY;
    int arg = 0x7FFFFFFF;
    if (live) {
      for (int c = part; c < a.nchd; c += 4) {
        const float m = a.dpart_max[o + c];
        const int ai = a.dpart_arg[o + c];
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
      for (int c = part; c < a.nchd; c += 4)
        S += a.dpart_sum[o + c] * exp(((double)a.dpart_max[o + c] - (double)mx) * invT);
    }
    const double s1 = __shfl_xor(S, 1);
    const double lo = (part & 1) ? s1 + S : S + s1;
    const double s2 = __shfl_xor(lo, 2);
    const double total = (part & 2) ? s2 + lo : lo + s2;
    // hand the row's statistics to the thread that owns draft position `row`
    __shared__ float s_mx[64];
    __shared__ double s_S[64];
    __shared__ int s_arg[64];
    if (live && part == 0) {
      s_mx[row] = mx; s_S[row] = total; s_arg[row] = arg;
      a.drow_max[q0 + row] = mx; a.drow_sum[q0 + row] = total; a.drow_arg[q0 + row] = arg;
    }
    __syncthreads();
    if (tid < k) {
      double lq;
      if (Td > 0.f) lq = ((double)zq - (double)s_mx[tid]) * invT - log(s_S[tid]);
      else lq = (d == s_arg[tid]) ? 0.0 : -INFINITY;
      s_logq[tid] = lq;
      a.logq_tok[q0 + tid] = lq;
    }
  }

  // ---- probe every window (s, L), L = 2 .. max_len; the longest hit per start wins
  if (a.cache.slots != nullptr) {
    const int nL = a.cache.max_len - 1;
    for (int w = tid; w < k * nL; w += 256) {
      const int s = w / nL, L = 2 + w % nL;
      if (s + L <= k) {
        const int t = cache_lookup(a.cache, &s_d[s], L);
        if (t >= 0) atomicMax(&s_hit[s], ((unsigned long long)L << 32) | (unsigned int)t);
      }
    }
  }
  __syncthreads();

  // ---- greedy left-to-right walk over LDS
  if (tid == 0) {
    int s = 0, j = 0, hits = 0, flags = 0;
    while (s < k) {
      int L, t;
      if (s_hit[s] != 0ull) {
        L = (int)(s_hit[s] >> 32); t = (int)(s_hit[s] & 0xFFFFFFFFull); ++hits;
      } else {
        t = s_dm[s];
        L = 1;
        if (t < 0) { flags |= OT_FLAG_UNMAPPABLE; break; }
      }
      double lq = 0.0;
      for (int l = 0; l < L; ++l) lq += s_logq[s + l];
      s_tok[j] = t; s_start[j] = s; s_len[j] = L; s_lq[j] = lq;
      s += L;
      ++j;
    }
    a.out.n_mapped[b] = j;
    a.out.hits_proposed[b] = hits;
    a.out.flags[b] = flags;
    a.s_end[b] = s;
  }
  __syncthreads();
  if (tid <= k) {
    a.out.mapped_ids[r0 + tid] = s_tok[tid];
    a.out.span_start[r0 + tid] = s_start[tid];
    a.out.span_len[r0 + tid] = s_len[tid];
    a.logq_map[r0 + tid] = s_lq[tid];
  }
}

}  // namespace

hipError_t launch_map(const StepArgs& a, hipStream_t stream) {
  if (a.B == 0) return hipSuccess;
  hipLaunchKernelGGL(map_kernel, dim3(a.B), dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace otv
