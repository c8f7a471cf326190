// Softmax statistics of logit rows: per row the maximum, its lowest index, and sum_v exp((z_v - max)/T).
//
// These three numbers are all the step needs of p = softmax(z/T) and q = softmax(zq/T_d) (Notation paragraph):
// a probability is re-formed on demand as exp((z_v - max)/T) / sum, so no probability row is ever written to
// memory.  One launch covers the M target rows (fp32 logits from the LM head) and the K draft rows (storage
// dtype): one workgroup reduces one chunk of kStatChunk logits of one row.  The chunk is read once into registers
// (16-byte loads, consecutive lanes on consecutive vectors), reduced to its maximum through wavefront shuffles and
// LDS, and only then exponentiated, so every logit is read from HBM exactly once.  The per-chunk partials are
// merged in a fixed order by the consumer (the translate-and-accept kernel).
#include "device_math.h"
#include "otv_internal.h"

namespace otv {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kPerThread = kStatChunk / kStatThreads;   // 32 logits per thread

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
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const f32x4 x = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));   // a pass over rows far larger than L2
    v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
  }
  __device__ static float one(const float* p) { return *p; }
};
template <> struct Loader<uint16_t> {
  static constexpr int kVec = 8;
  __device__ static void load(const uint16_t* p, float* v) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 x = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
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

// Rows 0..M-1 are target rows, rows M..M+K-1 draft rows.  TD is the draft logits' storage type.
template <typename TD, bool kAlignedT, bool kAlignedD>
__global__ __launch_bounds__(kStatThreads) void softmax_stats_kernel(StepArgs a) {
  const int n_target = a.M * a.ncht;                 // workgroups 0 .. n_target-1 take target chunks, the rest draft chunks
  if ((int)blockIdx.x < n_target) {
    const int row = blockIdx.x / a.ncht, c = blockIdx.x % a.ncht;
    const int b = find_sequence(a.row_off, a.B, row, 0);
    const float T_b = a.temperature[b];
    const float scale = T_b > 0.f ? kLog2e / T_b : kLog2e;
    chunk_stats<float, kAlignedT>(a.Z + (int64_t)row * a.ldz, a.V_t, c, scale, a.tpart_max, a.tpart_sum, a.tpart_arg,
                                  (int64_t)row * a.ncht + c);
  } else {
    const int id = blockIdx.x - n_target;
    const int drow = id / a.nchd, c = id % a.nchd;
    const int b = find_sequence(a.row_off, a.B, drow, 1);
    const float T_b = a.draft_temperature ? a.draft_temperature[b] : a.temperature[b];
    const float scale = T_b > 0.f ? kLog2e / T_b : kLog2e;
    const TD* x = static_cast<const TD*>(a.draft_logits) + (int64_t)drow * a.V_d;
    chunk_stats<TD, kAlignedD>(x, a.V_d, c, scale, a.dpart_max, a.dpart_sum, a.dpart_arg, (int64_t)drow * a.nchd + c);
  }
}

template <typename TD>
hipError_t launch_typed(const StepArgs& a, bool at, bool ad, hipStream_t stream) {
  dim3 grid(a.M * a.ncht + a.K * a.nchd), block(kStatThreads);
  if (at && ad) hipLaunchKernelGGL((softmax_stats_kernel<TD, true, true>), grid, block, 0, stream, a);
  else if (at) hipLaunchKernelGGL((softmax_stats_kernel<TD, true, false>), grid, block, 0, stream, a);
  else if (ad) hipLaunchKernelGGL((softmax_stats_kernel<TD, false, true>), grid, block, 0, stream, a);
  else hipLaunchKernelGGL((softmax_stats_kernel<TD, false, false>), grid, block, 0, stream, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_softmax_stats(const StepArgs& a, hipStream_t stream) {
  if (a.M + a.K == 0) return hipSuccess;
  const bool at = (a.ldz % 4) == 0 && (reinterpret_cast<uintptr_t>(a.Z) % 16) == 0;
  const bool base16 = (reinterpret_cast<uintptr_t>(a.draft_logits) % 16) == 0;
  if (a.dtype == OT_BF16) return launch_typed<uint16_t>(a, at, base16 && a.V_d % 8 == 0, stream);
  return launch_typed<float>(a, at, base16 && a.V_d % 4 == 0, stream);
}

}  // namespace otv
