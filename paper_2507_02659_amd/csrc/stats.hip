// Softmax statistics of logit rows, and the acceptance test that consumes them (two kernels).
//
// Statistics: per row the maximum, its lowest index, and sum_v exp((z_v - max)/T).  These three numbers are all
// the step needs of p = softmax(z/T) (Notation paragraph): p(v) is re-formed on demand as
// exp((z_v - max)/T) / sum, so no probability row is ever written to memory.  One workgroup reduces one chunk of
// kStatChunk logits of one row: the chunk is read once into registers (16-byte loads, consecutive lanes on
// consecutive vectors), reduced to its maximum through wavefront shuffles and LDS, and only then exponentiated,
// so every logit is read from HBM exactly once.
//
// Acceptance (Algorithm 1, rejection-sampling step): one workgroup per sequence merges the sequence's chunk
// partials in a fixed order (4 threads per row) and runs the test.  Lane j of its first wavefront owns mapped
// position j: it forms p_j(t_j), the ratio min(1, p/q') and its Philox uniform; acceptance tests at different
// positions are independent given (u_j, p_j(t_j), q'_j), so "stop at the first rejection" is a ballot and a
// find-first-set, not a loop.  It also prepares what the final-token kernels need (FinalInfo).
// (Electing the last statistics workgroup of a sequence to run the test inside the same launch was measured and
// dropped: the agent-scope release fence it needs writes back the L2, which still holds the freshly written logits,
// in every one of the thousands of workgroups.)
#include "device_math.h"
#include "otv_internal.h"

namespace otv {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kPerThread = kStatChunk / kStatThreads;   // 16 logits per thread

// Sequence that owns `row`: rows of sequence b start at off[b] - shift*b (shift = 0 target rows, 1 draft rows).
__device__ inline int find_sequence(const int32_t* off, int B, int row, int shift) {
  int lo = 0, hi = B - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (off[mid] - shift * mid <= row) lo = mid; else hi = mid - 1;
  }
  return lo;
}

template <typename T> struct Loader;
template <> struct Loader<float> {
  static constexpr int kVec = 4;
  __device__ static void load(const float* p, float* v) {
    float4 x = *reinterpret_cast<const float4*>(p);
    v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
  }
  __device__ static float one(const float* p) { return *p; }
};
template <> struct Loader<uint16_t> {
  static constexpr int kVec = 8;
  __device__ static void load(const uint16_t* p, float* v) {
    uint4 x = *reinterpret_cast<const uint4*>(p);
    uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(w[i] << 16);
      v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
  }
  __device__ static float one(const uint16_t* p) { return bf16_to_f32(*p); }
};

// Reduces chunk c of one row; thread 0 writes (max, sum, argmax) to the partial arrays.
template <typename T, bool kAligned>
__device__ inline void chunk_stats(const T* __restrict__ x_row, int V, int c, float scale, float* __restrict__ pmax,
                                   double* __restrict__ psum, int32_t* __restrict__ parg, int64_t slot) {
  constexpr int kVec = Loader<T>::kVec;
  constexpr int kLoads = kPerThread / kVec;
  const int tid = threadIdx.x;
  const int base = c * kStatChunk;
  const int n = min(kStatChunk, V - base);
  const T* x = x_row + base;

  float v[kPerThread];
  float best = -INFINITY;
  int best_i = 0x7FFFFFFF;
#pragma unroll
  for (int i = 0; i < kLoads; ++i) {
    const int at = (i * kStatThreads + tid) * kVec;
    if (kAligned && at + kVec <= n) {
      Loader<T>::load(x + at, &v[i * kVec]);
    } else {
#pragma unroll
      for (int e = 0; e < kVec; ++e) v[i * kVec + e] = (at + e < n) ? Loader<T>::one(x + at + e) : -INFINITY;
    }
  }
#pragma unroll
  for (int i = 0; i < kLoads; ++i) {
    const int at = (i * kStatThreads + tid) * kVec;
#pragma unroll
    for (int e = 0; e < kVec; ++e) {
      if (v[i * kVec + e] > best) { best = v[i * kVec + e]; best_i = at + e; }   // ascending index: first maximum kept
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    float ob = __shfl_xor(best, off);
    int oi = __shfl_xor(best_i, off);
    if (ob > best || (ob == best && oi < best_i)) { best = ob; best_i = oi; }
  }
  __shared__ float s_max[kStatThreads / 64];
  __shared__ int s_idx[kStatThreads / 64];
  __shared__ double s_sum[kStatThreads / 64];
  const int wave = tid >> 6, lane = tid & 63;
  if (lane == 0) { s_max[wave] = best; s_idx[wave] = best_i; }
  __syncthreads();
  best = s_max[0]; best_i = s_idx[0];
#pragma unroll
  for (int w = 1; w < kStatThreads / 64; ++w) {
    if (s_max[w] > best || (s_max[w] == best && s_idx[w] < best_i)) { best = s_max[w]; best_i = s_idx[w]; }
  }
  // exponentials relative to the chunk maximum; masked slots hold -inf and contribute exp2(-inf) = 0
  float acc = 0.f;
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) acc += __builtin_amdgcn_exp2f((v[i] - best) * scale);
  double sum = (double)acc;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
  if (lane == 0) s_sum[wave] = sum;
  __syncthreads();
  if (tid == 0) {
    double total = s_sum[0];
#pragma unroll
    for (int w = 1; w < kStatThreads / 64; ++w) total += s_sum[w];
    pmax[slot] = best;
    psum[slot] = total;
    parg[slot] = base + best_i;
  }
}

template <typename T, bool kAligned>
__global__ __launch_bounds__(kStatThreads) void draft_stats_kernel(StepArgs a) {
  const int row = blockIdx.y, c = blockIdx.x;
  const int b = find_sequence(a.row_off, a.B, row, 1);
  const float T_b = a.draft_temperature ? a.draft_temperature[b] : a.temperature[b];
  const float scale = T_b > 0.f ? kLog2e / T_b : kLog2e;
  const T* x = static_cast<const T*>(a.draft_logits) + (int64_t)row * a.V_d;
  chunk_stats<T, kAligned>(x, a.V_d, c, scale, a.dpart_max, a.dpart_sum, a.dpart_arg, (int64_t)row * a.nchd + c);
}

// ------------------------------------------------------------------------------------------------ acceptance
__global__ __launch_bounds__(256) void accept_kernel(StepArgs a) {
  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const int r0 = a.row_off[b];
  const int k = a.row_off[b + 1] - r0 - 1;
  const int q0 = r0 - b;
  const float T = a.temperature[b];
  const double invT = T > 0.f ? 1.0 / (double)T : 1.0;
  __shared__ float s_mx[64];
  __shared__ double s_S[64];
  __shared__ int s_arg[64];

  // ---- merge the chunk partials: 4 threads per row, each takes every 4th chunk; fixed combination order
  {
    const int row = tid >> 2, part = tid & 3;
    const bool live = row <= k;
    const int64_t o = (int64_t)(r0 + (live ? row : 0)) * a.ncht;
    float mx = -INFINITY;
    int arg = 0x7FFFFFFF;
    if (live) {
      for (int c = part; c < a.ncht; c += 4) {
        const float m = a.tpart_max[o + c];
        const int ai = a.tpart_arg[o + c];
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
      for (int c = part; c < a.ncht; c += 4)
        S += a.tpart_sum[o + c] * exp(((double)a.tpart_max[o + c] - (double)mx) * invT);
    }
    const double s1 = __shfl_xor(S, 1);
    const double lo = (part & 1) ? s1 + S : S + s1;          // (part0 + part1) or (part2 + part3), same order in both lanes
    const double s2 = __shfl_xor(lo, 2);
    const double total = (part & 2) ? s2 + lo : lo + s2;     // (p0 + p1) + (p2 + p3)
    if (live && part == 0) {
      s_mx[row] = mx; s_S[row] = total; s_arg[row] = arg;
      a.row_max[r0 + row] = mx;
      a.row_sum[r0 + row] = total;
      a.row_arg[r0 + row] = arg;
    }
  }
  __syncthreads();
  if (tid >= 64) return;
  const int lane = tid;
  const int flags = a.out.flags[b];
  const int m = a.out.n_mapped[b];
  const float mx = lane <= k ? s_mx[lane] : 0.f;
  const double S = lane <= k ? s_S[lane] : 1.0;
  const int arg = lane <= k ? s_arg[lane] : 0;

  FinalInfo fin;
  fin.mode = 0; fin.row = r0; fin.drow = 0; fin.t_ng = -1; fin.t_pre = -1; fin.argq = -1; fin.greedy_draft = 0;
  fin.pad = 0; fin.pi = 0.0; fin.q_pre = 0.0; fin.u2 = 0.0;
  fin.mx = 0.0; fin.invT = 1.0; fin.invS = 1.0; fin.mxq = 0.0; fin.invTd = 1.0; fin.invSq = 1.0;

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
  int t_j = -1, L_j = 0, start_j = 0;
  double pt = 0.0, qp = 0.0, ratio = 0.0;
  if (lane < m) {
    t_j = a.out.mapped_ids[r0 + lane];
    L_j = a.out.span_len[r0 + lane];
    start_j = a.out.span_start[r0 + lane];
    qp = exp(a.logq_map[r0 + lane]);
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

  // ---- accepted tokens and counts (a greedy sequence's final token is the argmax of row n, which lane n holds)
  if (lane <= k) a.out.out_tokens[r0 + lane] = (lane < n) ? t_j : ((lane == n && !(T > 0.f)) ? arg : -1);
  int len_acc = (lane < n) ? L_j : 0;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) len_acc += __shfl_xor(len_acc, off);
  const int hits_acc = __popcll(__ballot(lane < n && L_j > 1));

  // ---- final token at row n: its values live in lane n
  const int fin_span_s = __shfl(start_j, n);
  const int fin_L = __shfl(L_j, n);
  const int fin_t = __shfl(t_j, n);
  const double fin_qp = __shfl(qp, n);
  const float fin_mx = __shfl(mx, n);
  const double fin_S = __shfl(S, n);
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
      fin.mx = (double)fin_mx; fin.invT = invT; fin.invS = 1.0 / fin_S;
      const bool unmappable = (flags & OT_FLAG_UNMAPPABLE) != 0;
      if (n == m && !unmappable) {
        fin.mode = 2;
      } else {
        fin.mode = 3;
        const int s = (n < m) ? fin_span_s : a.s_end[b];
        fin.drow = q0 + s;
        const float Td = a.draft_temperature ? a.draft_temperature[b] : T;
        fin.greedy_draft = !(Td > 0.f);
        fin.invTd = fin.greedy_draft ? 1.0 : 1.0 / (double)Td;
        fin.mxq = (double)a.drow_max[q0 + s];
        fin.invSq = 1.0 / a.drow_sum[q0 + s];
        fin.argq = a.drow_arg[q0 + s];
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

template <bool kAligned>
__global__ __launch_bounds__(kStatThreads) void target_stats_kernel(StepArgs a) {
  const int row = blockIdx.y, c = blockIdx.x;
  const int b = find_sequence(a.row_off, a.B, row, 0);
  const float T_b = a.temperature[b];
  const float scale = T_b > 0.f ? kLog2e / T_b : kLog2e;
  chunk_stats<float, kAligned>(a.Z + (int64_t)row * a.ldz, a.V_t, c, scale, a.tpart_max, a.tpart_sum, a.tpart_arg,
                               (int64_t)row * a.ncht + c);
}

}  // namespace

hipError_t launch_draft_stats(const StepArgs& a, hipStream_t stream) {
  if (a.K == 0) return hipSuccess;
  dim3 grid(a.nchd, a.K), block(kStatThreads);
  const bool base16 = (reinterpret_cast<uintptr_t>(a.draft_logits) % 16) == 0;
  if (a.dtype == OT_BF16) {
    if (base16 && a.V_d % 8 == 0) hipLaunchKernelGGL((draft_stats_kernel<uint16_t, true>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((draft_stats_kernel<uint16_t, false>), grid, block, 0, stream, a);
  } else {
    if (base16 && a.V_d % 4 == 0) hipLaunchKernelGGL((draft_stats_kernel<float, true>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((draft_stats_kernel<float, false>), grid, block, 0, stream, a);
  }
  return hipGetLastError();
}

hipError_t launch_target_stats(const StepArgs& a, hipStream_t stream) {
  if (a.M == 0) return hipSuccess;
  dim3 grid(a.ncht, a.M), block(kStatThreads);
  const bool aligned = (a.ldz % 4) == 0 && (reinterpret_cast<uintptr_t>(a.Z) % 16) == 0;
  if (aligned) hipLaunchKernelGGL((target_stats_kernel<true>), grid, block, 0, stream, a);
  else hipLaunchKernelGGL((target_stats_kernel<false>), grid, block, 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_accept(const StepArgs& a, hipStream_t stream) {
  if (a.B == 0) return hipSuccess;
  hipLaunchKernelGGL(accept_kernel, dim3(a.B), dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace otv
