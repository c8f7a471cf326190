// Softmax statistics of logit rows: per row the maximum, its lowest index, and sum_v exp((z_v - max)/T).
//
// These three numbers are all the step needs of p = softmax(z/T) and q = softmax(zq/T_d) (Notation paragraph):
// a probability is re-formed on demand as exp((z_v - max)/T) / sum, so no probability row is ever written to
// memory.  One launch covers the M target rows (fp32 logits from the LM head) and the K draft rows (storage
// dtype): one workgroup reduces one chunk of kStatChunk logits of one row.  The chunk is read once into registers
// (16-byte loads, consecutive lanes on consecutive vectors), reduced to its maximum through wavefront shuffles and
// LDS, and only then exponentiated, so every logit is read from HBM exactly once.  The per-chunk partials are
// merged in a fixed order by the consumer.  With a.chunked the launch also carries one workgroup per sequence that
// looks up what its drafted ids need (drafted logit, direct image, n-gram table probes: Eq. 1) and leaves a
// ProbeRecord, so that a single launch can follow (walk, acceptance test, final draw).
#include "device_math.h"
#include "otv_internal.h"
#include "translate.h"

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

// The same for up to 256 sequences without a chain of dependent loads: every lane of the wavefront holds the first
// row of sequences lane, lane + 64, ... (four independent loads, issued together), the predicate "starts at or before
// `row`" is monotone in b, and the owner is the number of sequences it holds for, less one.  A workgroup's first loads
// of logits then leave one round trip after its start, not five.
constexpr int kBallotSequences = 256;
struct SequenceStarts { int first_row[kBallotSequences / 64]; float temp[kBallotSequences / 64]; };
__device__ inline SequenceStarts load_sequence_starts(const int32_t* off, const float* temperature, int B, int shift,
                                                      int lane) {
  SequenceStarts s;
#pragma unroll
  for (int j = 0; j < kBallotSequences / 64; ++j) {
    const int b = min(64 * j + lane, B - 1);
    s.first_row[j] = off[b] - shift * b;
    s.temp[j] = temperature[b];
  }
  return s;
}
// temperature of the sequence that owns `row`
__device__ inline float owner_temperature(const SequenceStarts& s, int B, int row, int lane) {
  int owner = -1;
#pragma unroll
  for (int j = 0; j < kBallotSequences / 64; ++j)
    owner += __popcll(__ballot(64 * j + lane < B && s.first_row[j] <= row));
  float T = 1.f;
#pragma unroll
  for (int j = 0; j < kBallotSequences / 64; ++j) {
    const float t = __shfl(s.temp[j], owner & 63);
    if ((owner >> 6) == j) T = t;
  }
  return T;
}

template <typename T> struct Loader;
template <> struct Loader<float> {
  static constexpr int kVec = 4;
  typedef float Raw __attribute__((ext_vector_type(4)));
  __device__ static Raw load(const float* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const Raw*>(p));   // a pass over rows far larger than L2
  }
  __device__ static void unpack(const Raw& x, float* v) { v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w; }
  __device__ static float one(const float* p) { return *p; }
};
template <> struct Loader<uint16_t> {
  static constexpr int kVec = 8;
  typedef uint32_t Raw __attribute__((ext_vector_type(4)));
  __device__ static Raw load(const uint16_t* p) { return __builtin_nontemporal_load(reinterpret_cast<const Raw*>(p)); }
  __device__ static void unpack(const Raw& x, float* v) {
    uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(w[i] << 16);
      v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
  }
  __device__ static float one(const uint16_t* p) { return bf16_to_f32(*p); }
};

// Reduces chunk c of one row; thread 0 writes (max, sum, argmax) to the partial arrays.  All vector loads of the chunk
// are issued before anything waits; scale_of() (the row's sequence and its temperature: it waits for loads issued before
// the call, and issues one more) is called behind them, so that a workgroup's logits are on their way one instruction
// after its start.
template <typename T, bool kAligned, typename ScaleFn>
__device__ __forceinline__ void chunk_stats(const T* __restrict__ x_row, int V, int c, ScaleFn scale_of,
                                            float* __restrict__ pmax, double* __restrict__ psum,
                                            int32_t* __restrict__ parg, int64_t slot) {
  constexpr int kVec = Loader<T>::kVec;
  constexpr int kLoads = kPerThread / kVec;
  const int tid = threadIdx.x;
  const int base = c * kStatChunk;
  const int n = min(kStatChunk, V - base);
  const T* x = x_row + base;

  float v[kPerThread];
  float best = -INFINITY;
  int best_i = 0x7FFFFFFF;
  typename Loader<T>::Raw raw[kLoads];
#pragma unroll
  for (int i = 0; i < kLoads; ++i) {
    const int at = (i * kStatThreads + tid) * kVec;
    if (kAligned && at + kVec <= n) raw[i] = Loader<T>::load(x + at);
  }
  const float scale = scale_of();
#pragma unroll
  for (int i = 0; i < kLoads; ++i) {
    const int at = (i * kStatThreads + tid) * kVec;
    if (kAligned && at + kVec <= n) {
      Loader<T>::unpack(raw[i], &v[i * kVec]);
    } else {                                 // the ragged end of a row, or a row that is not 16-byte aligned
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
  // With a.chunked the first B workgroups look up one sequence's drafted ids each: chains of dependent loads, started
  // first so that they run underneath the stream of the others.  Then n_target workgroups take target chunks, the rest
  // draft chunks.
  const int n_lookup = a.chunked ? a.B : 0;
  const int wg = (int)blockIdx.x - n_lookup;
  const int n_target = a.M * a.ncht;
  const int lane = threadIdx.x & 63;
  const bool by_ballot = a.B <= kBallotSequences;
  if (wg < 0) {
    __shared__ DraftLds s_d;
    const int b = blockIdx.x, tid = threadIdx.x;
    const int r0 = a.row_off[b], k = a.row_off[b + 1] - r0 - 1;
    draft_lds_reset(&s_d, tid);
    __syncthreads();
    fetch_ids_and_probe(a, r0 - b, k, tid, kStatThreads, &s_d);
    __syncthreads();
    ProbeRecord* rec = a.probe + b;
    if (tid < 64) { rec->hit[tid] = s_d.hit[tid]; rec->zq[tid] = s_d.zq[tid]; rec->dm[tid] = s_d.dm[tid]; }
    if (tid == 0) rec->bad = s_d.bad;
    return;
  }
  if (wg < n_target) {
    const int row = wg / a.ncht, c = wg % a.ncht;
    SequenceStarts starts;
    if (by_ballot) starts = load_sequence_starts(a.row_off, a.temperature, a.B, 0, lane);
    auto scale_of = [&]() {
      const float T_b = by_ballot ? owner_temperature(starts, a.B, row, lane)
                                  : a.temperature[find_sequence(a.row_off, a.B, row, 0)];
      return T_b > 0.f ? kLog2e / T_b : kLog2e;
    };
    chunk_stats<float, kAlignedT>(a.Z + (int64_t)row * a.ldz, a.V_t, c, scale_of, a.tpart_max, a.tpart_sum, a.tpart_arg,
                                  (int64_t)row * a.ncht + c);
  } else {
    const int id = wg - n_target;
    const int drow = id / a.nchd, c = id % a.nchd;
    SequenceStarts starts;
    const float* temps = a.draft_temperature ? a.draft_temperature : a.temperature;
    if (by_ballot) starts = load_sequence_starts(a.row_off, temps, a.B, 1, lane);
    auto scale_of = [&]() {
      const float T_b = by_ballot ? owner_temperature(starts, a.B, drow, lane)
                                  : temps[find_sequence(a.row_off, a.B, drow, 1)];
      return T_b > 0.f ? kLog2e / T_b : kLog2e;
    };
    const TD* x = static_cast<const TD*>(a.draft_logits) + (int64_t)drow * a.V_d;
    chunk_stats<TD, kAlignedD>(x, a.V_d, c, scale_of, a.dpart_max, a.dpart_sum, a.dpart_arg, (int64_t)drow * a.nchd + c);
  }
}

template <typename TD>
hipError_t launch_typed(const StepArgs& a, bool at, bool ad, hipStream_t stream) {
  dim3 grid(a.M * a.ncht + a.K * a.nchd + (a.chunked ? a.B : 0)), block(kStatThreads);
  if (at && ad) hipLaunchKernelGGL((softmax_stats_kernel<TD, true, true>), grid, block, 0, stream, a);
  else if (at) hipLaunchKernelGGL((softmax_stats_kernel<TD, true, false>), grid, block, 0, stream, a);
  else if (ad) hipLaunchKernelGGL((softmax_stats_kernel<TD, false, true>), grid, block, 0, stream, a);
  else hipLaunchKernelGGL((softmax_stats_kernel<TD, false, false>), grid, block, 0, stream, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_softmax_stats(const StepArgs& a, hipStream_t stream) {
  if (a.M + a.K + (a.chunked ? a.B : 0) == 0) return hipSuccess;
  const bool at = (a.ldz % 4) == 0 && (reinterpret_cast<uintptr_t>(a.Z) % 16) == 0;
  const bool base16 = (reinterpret_cast<uintptr_t>(a.draft_logits) % 16) == 0;
  if (a.dtype == OT_BF16) return launch_typed<uint16_t>(a, at, base16 && a.V_d % 8 == 0, stream);
  return launch_typed<float>(a, at, base16 && a.V_d % 4 == 0, stream);
}

}  // namespace otv
