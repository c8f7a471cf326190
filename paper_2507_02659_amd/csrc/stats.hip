// Softmax statistics of logit rows: per row the maximum, its lowest index, and sum_v exp((z_v - max)/T).
// These three numbers are all the step needs of p = softmax(z/T) (Notation paragraph): p(v) is re-formed
// on demand as exp((z_v - max)/T) / sum, so no probability row is ever written to memory.
//
// One workgroup reduces one chunk of kStatChunk logits of one row: the chunk is read once into registers
// (16-byte loads, consecutive lanes on consecutive vectors), reduced to its maximum through wavefront
// shuffles and LDS, and only then exponentiated, so the kernel reads each logit from HBM exactly once.
// The per-chunk partials are merged by the consumer (map / accept kernels) in a fixed order.
#include "otv_internal.h"

namespace otv {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kPerThread = kStatChunk / kStatThreads;   // 16 logits per thread

__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

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

template <typename T, bool kAligned>
__global__ __launch_bounds__(kStatThreads) void softmax_stats_kernel(
    const T* __restrict__ X, int64_t ld, int V, const int32_t* __restrict__ row_off, int B, int shift,
    const float* __restrict__ temperature, float* __restrict__ pmax, double* __restrict__ psum,
    int32_t* __restrict__ parg, int nch) {
  constexpr int kVec = Loader<T>::kVec;
  constexpr int kLoads = kPerThread / kVec;
  const int row = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
  const int b = find_sequence(row_off, B, row, shift);
  const float T_b = temperature[b];
  const float scale = T_b > 0.f ? kLog2e / T_b : kLog2e;
  const int base = c * kStatChunk;
  const int n = min(kStatChunk, V - base);
  const T* x = X + (int64_t)row * ld + base;

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
#pragma unroll
    for (int e = 0; e < kVec; ++e) {
      if (v[i * kVec + e] > best) { best = v[i * kVec + e]; best_i = at + e; }   // ascending index: first maximum kept
    }
  }
  // wavefront reduction of (max, lowest index)
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
    const int64_t o = (int64_t)row * nch + c;
    pmax[o] = best;
    psum[o] = total;
    parg[o] = base + best_i;
  }
}

}  // namespace

hipError_t launch_stats(const StepArgs& a, bool draft, hipStream_t stream) {
  const int rows = draft ? a.K : a.M;
  if (rows == 0) return hipSuccess;
  const int V = draft ? a.V_d : a.V_t;
  const int nch = draft ? a.nchd : a.ncht;
  const float* temp = (draft && a.draft_temperature) ? a.draft_temperature : a.temperature;
  dim3 grid(nch, rows), block(kStatThreads);
  if (draft) {
    if (a.dtype == OT_BF16) {
      const bool aligned = (a.V_d % 8) == 0 && (reinterpret_cast<uintptr_t>(a.draft_logits) % 16) == 0;
      auto* X = static_cast<const uint16_t*>(a.draft_logits);
      if (aligned)
        hipLaunchKernelGGL((softmax_stats_kernel<uint16_t, true>), grid, block, 0, stream, X, (int64_t)a.V_d, V,
                           a.row_off, a.B, 1, temp, a.dpart_max, a.dpart_sum, a.dpart_arg, nch);
      else
        hipLaunchKernelGGL((softmax_stats_kernel<uint16_t, false>), grid, block, 0, stream, X, (int64_t)a.V_d, V,
                           a.row_off, a.B, 1, temp, a.dpart_max, a.dpart_sum, a.dpart_arg, nch);
    } else {
      const bool aligned = (a.V_d % 4) == 0 && (reinterpret_cast<uintptr_t>(a.draft_logits) % 16) == 0;
      auto* X = static_cast<const float*>(a.draft_logits);
      if (aligned)
        hipLaunchKernelGGL((softmax_stats_kernel<float, true>), grid, block, 0, stream, X, (int64_t)a.V_d, V,
                           a.row_off, a.B, 1, temp, a.dpart_max, a.dpart_sum, a.dpart_arg, nch);
      else
        hipLaunchKernelGGL((softmax_stats_kernel<float, false>), grid, block, 0, stream, X, (int64_t)a.V_d, V,
                           a.row_off, a.B, 1, temp, a.dpart_max, a.dpart_sum, a.dpart_arg, nch);
    }
  } else {
    const bool aligned = (a.ldz % 4) == 0 && (reinterpret_cast<uintptr_t>(a.Z) % 16) == 0;
    if (aligned)
      hipLaunchKernelGGL((softmax_stats_kernel<float, true>), grid, block, 0, stream, a.Z, a.ldz, V, a.row_off, a.B,
                         0, a.temperature, a.tpart_max, a.tpart_sum, a.tpart_arg, nch);
    else
      hipLaunchKernelGGL((softmax_stats_kernel<float, false>), grid, block, 0, stream, a.Z, a.ldz, V, a.row_off, a.B,
                         0, a.temperature, a.tpart_max, a.tpart_sum, a.tpart_arg, nch);
  }
  return hipGetLastError();
}

}  // namespace otv
