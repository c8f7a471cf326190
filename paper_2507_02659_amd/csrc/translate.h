// Draft side of a verification step, as device functions shared by the kernels that host it: everything that needs
// the drafter's logits and ids but nothing of the target's logits.
//   * softmax statistics of the draft rows (Notation paragraph: q = softmax(zq / T_d)): one wavefront per row, or one
//     workgroup per piece of a row with the pieces merged where they are used;
//   * translation of the drafted window into the target vocabulary (Section "Cross-vocabulary N-gram Cache", Eq. 1):
//     every window (start s, length L) of the drafted ids is probed in the n-gram table by its own thread; lane s of
//     one wavefront prepares the segment that would start at s, and the window is then walked left to right as a chase
//     through start + length: the longest cache hit at s yields one target token whose log q' is the sum of the L
//     sub-token log-probabilities (the product of Eq. 1, kept in log space so that five or six factors of 1e-6 do not
//     underflow), otherwise the direct image of d_s, and a draft id with neither ends the proposal.
// The lookups of a sequence (drafted logits, direct images, table probes) need memory and can run early, next to the
// LM head, which leaves them in a ProbeRecord; the walk itself is a few microseconds of one wavefront and runs where
// the acceptance test does.  Its outcome is one LaneProposal per mapped position, held by lane j of that wavefront.
#pragma once

#include "device_math.h"
#include "otv_internal.h"

namespace otv {

constexpr float kLog2eF = 1.4426950408889634f;

// LDS scratch of one sequence's translation (k <= 63 drafted positions).
struct DraftLds {
  unsigned long long hit[64];   // (length << 60) | (slot << 32) | target of the longest cache hit starting here, 0 = none
  double logq[64];              // log q_i(d_i)
  double qS[64];                // draft row statistics
  float qmx[64];
  float zq[64];                 // draft logit of the drafted id
  int32_t qarg[64];
  int32_t dm[64];               // direct image of the drafted id, or -1
  int32_t bad;                  // a drafted id was outside [0, V_d)
};

// What lane j of the walking wavefront knows about mapped position j after the translation.
struct LaneProposal {
  int t, start, L;              // target id (-1 beyond the proposal), first draft position, draft tokens covered
  double lq;                    // log q'(t_j)
  // the draft row a final draw at this position would use (Eq. 2): the row of the span's first sub-token, or for
  // lane m the row of the draft id that could not be translated
  int t_pre, argq;              // direct image of that row's drafted id (-1: none); argmax of the row
  float mxq;                    // its maximum
  double Sq;                    // its sum of exponentials
  double lq_first;              // log q(d) of its drafted id
  // wavefront-uniform
  int m, flags;
};

// Probe of one key held in registers (fully unrolled so that `ids` never has to live in scratch memory).
// Returns the slot index of the entry, or -1.
__device__ __forceinline__ int cache_lookup(const CacheTable& C, const int32_t (&ids)[OT_MAX_NGRAM_LEN], int L) {
  uint32_t h = 0x9E3779B9u ^ (uint32_t)L;                  // same mixing as hash_ngram()
#pragma unroll
  for (int i = 0; i < OT_MAX_NGRAM_LEN; ++i) {
    if (i < L) {
      h ^= (uint32_t)ids[i] + 0x7F4A7C15u + (h << 6) + (h >> 2);
      h *= 0x85EBCA6Bu;
      h ^= h >> 13;
    }
  }
  h *= 0xC2B2AE35u;
  h ^= h >> 16;
  h &= C.mask;
  for (uint32_t probe = 0; probe <= C.mask; ++probe) {     // bounded: the table is never more than half full
    const int32_t* slot = C.slots + (size_t)h * C.stride;
    const int sl = slot[0];
    if (sl == 0) return -1;
    if (sl == L) {
      bool same = true;
#pragma unroll
      for (int i = 0; i < OT_MAX_NGRAM_LEN; ++i)
        if (i < L) same = same && (slot[2 + i] == ids[i]);
      if (same) return (int)h;
    }
    h = (h + 1) & C.mask;
  }
  return -1;
}

__device__ __forceinline__ void draft_lds_reset(DraftLds* L, int g) {
  if (g == 0) L->bad = 0;
  if (g < 64) { L->hit[g] = 0ull; L->dm[g] = -1; }
}

// Thread g of n: range check, drafted logit and direct image of the drafted positions; every window (s, len) of the
// drafted ids against the n-gram table, the longest hit per start wins.  draft_lds_reset and a barrier come before,
// a barrier after.
__device__ __forceinline__ void fetch_ids_and_probe(const StepArgs& a, int q0, int k, int g, int n, DraftLds* L) {
  for (int i = g; i < k; i += n) {
    const int d = a.draft_ids[q0 + i];
    if (d < 0 || d >= a.V_d) {
      L->bad = 1;
    } else {
      const int64_t at = (int64_t)(q0 + i) * a.V_d + d;
      L->zq[i] = a.dtype == OT_BF16 ? bf16_to_f32(static_cast<const uint16_t*>(a.draft_logits)[at])
                                    : static_cast<const float*>(a.draft_logits)[at];
      L->dm[i] = a.dmap[d];
    }
  }
  if (a.cache.slots != nullptr) {
    const int nL = a.cache.max_len - 1;
    for (int w = g; w < k * nL; w += n) {
      const int s = w / nL, len = 2 + w % nL;
      if (s + len <= k) {
        int32_t ids[OT_MAX_NGRAM_LEN];
        bool in_range = true;
#pragma unroll
        for (int i = 0; i < OT_MAX_NGRAM_LEN; ++i) {
          ids[i] = i < len ? a.draft_ids[q0 + s + i] : 0;
          in_range = in_range && ids[i] >= 0 && ids[i] < a.V_d;
        }
        if (in_range) {
          const int slot = cache_lookup(a.cache, ids, len);
          if (slot >= 0) {
            const unsigned int t = (unsigned int)a.cache.slots[(size_t)slot * a.cache.stride + 1];
            atomicMax(&L->hit[s], ((unsigned long long)len << 60) | ((unsigned long long)slot << 32) | t);
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------- draft row statistics
// 16-byte vectors of a logit row, kept as loaded until they are used (a bf16 vector unpacks to 8 floats).
template <typename T> struct RowVec;
template <> struct RowVec<float> {
  static constexpr int kVec = 4;
  typedef float4 Raw;
  __device__ static Raw load(const float* p) { return *reinterpret_cast<const float4*>(p); }
  __device__ static Raw lowest() { return make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY); }
  __device__ static void unpack(const Raw& r, float* v) { v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w; }
  __device__ static float one(const float* p) { return *p; }
};
template <> struct RowVec<uint16_t> {
  static constexpr int kVec = 8;
  typedef uint4 Raw;
  __device__ static Raw load(const uint16_t* p) { return *reinterpret_cast<const uint4*>(p); }
  __device__ static Raw lowest() { return make_uint4(0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u); }   // -inf
  __device__ static void unpack(const Raw& r, float* v) {
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(w[i] << 16);
      v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
  }
  __device__ static float one(const uint16_t* p) { return bf16_to_f32(*p); }
};

// Running (maximum, lowest index of it, sum of exponentials relative to it) of one lane.
struct RunStat {
  float mx = -INFINITY;
  int arg = 0x7FFFFFFF;
  double sum = 0.0;
  // raises the maximum to (bm, bi) if that is larger; the sum is rescaled to the new maximum
  __device__ inline void raise(float bm, int bi, float scale) {
    if (bm > mx) {
      sum *= (double)__builtin_amdgcn_exp2f((mx - bm) * scale);   // mx = -inf: the sum is 0 and stays 0
      mx = bm;
      arg = bi;
    }
  }
};

// One wavefront reduces one whole logit row to (maximum, its lowest index, sum of exp((x - max) * scale / log2 e)).
// Every lane requests kBatch 16-byte vectors at a time before it touches any of them: the draft side runs next to a
// kernel that saturates the memory system, where a load takes several microseconds to return, so the bytes in flight
// decide how long a row takes.  A lane keeps a running maximum and a running sum relative to it (rescaled when the
// maximum moves); the 64 lanes are merged at the end by shuffles in a fixed order.  Sums of one vector are formed in
// binary32, everything above that in binary64.  Rows that do not start on a 16-byte boundary, and the last V % kVec
// elements of the others, are read element by element.  All lanes return the row's statistics.
// kFirst: the first batch was requested earlier (row_first_batch_load with the same x and V) and is taken from `first`.
template <typename T, int kBatch> struct RowFirstBatch { typename RowVec<T>::Raw raw[kBatch]; };

template <typename T, int kBatch>
__device__ __forceinline__ void row_first_batch_load(const T* __restrict__ x, int V, int lane,
                                                     RowFirstBatch<T, kBatch>& first) {
  constexpr int kVec = RowVec<T>::kVec;
  const bool aligned = (reinterpret_cast<uintptr_t>(x) % 16) == 0;
  const int n_vec = aligned && V > 0 ? V / kVec : 0;
#pragma unroll
  for (int j = 0; j < kBatch; ++j) {
    const int at = j * 64 + lane;
    first.raw[j] = at < n_vec ? RowVec<T>::load(x + (int64_t)at * kVec) : RowVec<T>::lowest();
  }
}

template <typename T, int kBatch, bool kFirst = false>
__device__ __forceinline__ void wave_row_stats(const T* __restrict__ x, int V, float scale, int lane, float* out_max,
                                               int* out_arg, double* out_sum,
                                               const RowFirstBatch<T, kBatch>* first = nullptr) {
  constexpr int kVec = RowVec<T>::kVec;
  typedef typename RowVec<T>::Raw Raw;
  const bool aligned = (reinterpret_cast<uintptr_t>(x) % 16) == 0;
  const int n_vec = aligned ? V / kVec : 0;       // whole vectors read as such
  RunStat r;
  for (int base = 0; base < n_vec; base += 64 * kBatch) {
    Raw raw[kBatch];
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      const int at = base + j * 64 + lane;
      if (kFirst && base == 0) raw[j] = first->raw[j];
      else raw[j] = at < n_vec ? RowVec<T>::load(x + (int64_t)at * kVec) : RowVec<T>::lowest();
    }
    float bm = -INFINITY;
    int bi = 0x7FFFFFFF;
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      if (base + j * 64 >= n_vec) break;        // wavefront-uniform: the remaining vectors of the batch are empty
      float v[kVec];
      RowVec<T>::unpack(raw[j], v);
#pragma unroll
      for (int e = 0; e < kVec; ++e)
        if (v[e] > bm) { bm = v[e]; bi = (base + j * 64 + lane) * kVec + e; }   // ascending index: first maximum kept
    }
    r.raise(bm, bi, scale);
    if (r.mx != -INFINITY) {
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        if (base + j * 64 >= n_vec) break;
        // the vector is unpacked again rather than kept unpacked since the first pass (8 registers instead of 4 each)
        asm volatile("" : "+v"(raw[j].x), "+v"(raw[j].y), "+v"(raw[j].z), "+v"(raw[j].w));
        float v[kVec];
        RowVec<T>::unpack(raw[j], v);
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < kVec; ++e) s += __builtin_amdgcn_exp2f((v[e] - r.mx) * scale);   // masked: exp2(-inf) = 0
        r.sum += (double)s;
      }
    }
  }
  for (int at = n_vec * kVec + lane; at < V; at += 64) {
    const float v = RowVec<T>::one(x + at);
    r.raise(v, at, scale);
    r.sum += (double)__builtin_amdgcn_exp2f((v - r.mx) * scale);
  }
  float mx = r.mx;
  int arg = r.arg;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float om = __shfl_xor(mx, off);
    const int oa = __shfl_xor(arg, off);
    if (om > mx || (om == mx && oa < arg)) { mx = om; arg = oa; }
  }
  double s = r.mx == -INFINITY ? 0.0 : r.sum * (double)__builtin_amdgcn_exp2f((r.mx - mx) * scale);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
  *out_max = mx; *out_arg = arg; *out_sum = s;
}

// ---------------------------------------------------------------------------------------------- the walk
// One wavefront (lane = threadIdx within it), after the barrier that publishes L: forms log q_i(d_i), walks the window
// and returns mapped position `lane` in P.  With `lead` it also writes the translation's outputs (n_mapped,
// hits_proposed, flags; mapped_ids, span_start, span_len, q_tok of the sequence's rows) and the use statistics of the
// cache entries; where several workgroups walk the same sequence exactly one of them leads.
__device__ inline void translate_walk(const StepArgs& a, int b, int r0, int k, int q0, float Td, double invTd, int lane,
                                      DraftLds* L, LaneProposal* P, bool lead = true) {
  if (lane < k) {
    double lq;
    if (Td > 0.f) lq = ((double)L->zq[lane] - (double)L->qmx[lane]) * invTd - log(L->qS[lane]);
    else lq = (a.draft_ids[q0 + lane] == L->qarg[lane]) ? 0.0 : -INFINITY;
    L->logq[lane] = lq;
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");

  // Lane s first prepares the segment that would start at draft position s (the longest cache hit there, else the
  // direct image; log q' = sum of its sub-tokens' log-probabilities); the walk itself is then a chase through
  // "start + length" with wavefront-uniform lane reads, a few cycles per token.
  int seg_t = -1, seg_L = 1, seg_slot = -1;
  double seg_lq = 0.0;
  if (lane < k) {
    const unsigned long long h = L->hit[lane];
    if (h != 0ull) {
      seg_L = (int)(h >> 60); seg_t = (int)(h & 0xFFFFFFFFull); seg_slot = (int)((h >> 32) & 0x0FFFFFFFull);
    } else {
      seg_t = L->dm[lane];
    }
    for (int l = 0; l < seg_L; ++l) seg_lq += L->logq[lane + l];
  }
  int m = 0, s_end = 0, flags = 0, start_j = -1;
  while (s_end < k) {
    const int at = __builtin_amdgcn_readfirstlane(s_end);
    if (__builtin_amdgcn_readlane(seg_t, at) < 0) { flags |= OT_FLAG_UNMAPPABLE; break; }   // neither a hit nor a direct image
    if (lane == m) start_j = at;
    s_end = at + __builtin_amdgcn_readlane(seg_L, at);
    ++m;
  }
  // lane j < m takes over the segment that starts at start_j
  // (all lanes take part in the shuffles: a lane outside the active set would not supply its value)
  const int src = start_j >= 0 ? start_j : 0;
  const int got_t = __shfl(seg_t, src), got_L = __shfl(seg_L, src);
  const double lq_j = __shfl(seg_lq, src);
  const int slot_j = __shfl(seg_slot, src);
  P->t = lane < m ? got_t : -1;
  P->L = lane < m ? got_L : 0;
  P->start = start_j;
  P->lq = lane < m ? lq_j : 0.0;
  P->m = m; P->flags = flags;
  const int hits = __popcll(__ballot(lane < m && P->L > 1));
  if (lead && lane < m && P->L > 1) {
    // use statistics of the entry (Appendix, cache eviction): one more use, last used now
    atomicAdd(&a.cache.uses[slot_j], 1u);
    a.cache.last_used[slot_j] = a.cache.clock;
    const uint32_t at = atomicAdd(a.cache.log_count, 1u);        // and the host hears of it through the log
    if (at < (uint32_t)kCacheLogCap) a.cache.log[at] = make_uint2((uint32_t)slot_j + 1u, a.cache.clock);
  }
  // the draft row a final draw at this position would read
  const int s_fin = lane < m ? start_j : ((lane == m && s_end < k) ? s_end : -1);
  P->t_pre = -1; P->argq = -1; P->mxq = 0.f; P->Sq = 1.0; P->lq_first = 0.0;
  if (s_fin >= 0) {
    P->t_pre = L->dm[s_fin]; P->argq = L->qarg[s_fin]; P->mxq = L->qmx[s_fin]; P->Sq = L->qS[s_fin];
    P->lq_first = L->logq[s_fin];
    if (lane == m) P->start = s_fin;
  }
  if (lead && lane == 0) {
    a.out.n_mapped[b] = m;
    a.out.hits_proposed[b] = hits;
    a.out.flags[b] = flags;
  }
  if (lead && lane <= k) {
    a.out.mapped_ids[r0 + lane] = P->t;
    a.out.span_start[r0 + lane] = lane < m ? start_j : -1;
    a.out.span_len[r0 + lane] = P->L;
    a.out.q_tok[r0 + lane] = lane < m ? (float)exp(P->lq) : 0.f;
  }
}

// Translation outputs of a sequence with a drafted id outside [0, V_d): it proposes nothing.
__device__ inline void translate_bad_sequence(const StepArgs& a, int b, int r0, int k, int lane) {
  if (lane <= k) {
    a.out.mapped_ids[r0 + lane] = -1; a.out.span_start[r0 + lane] = -1; a.out.span_len[r0 + lane] = 0;
    a.out.q_tok[r0 + lane] = 0.f;
  }
  if (lane == 0) { a.out.n_mapped[b] = 0; a.out.hits_proposed[b] = 0; a.out.flags[b] = OT_FLAG_BAD_ID; }
}

// Softmax statistics of elements [e0, e0 + n) of draft row q by one workgroup of kWaves wavefronts (all threads call it;
// it contains workgroup barriers): every wavefront takes a contiguous slice, the slices are merged through LDS in
// ascending order (of equal maxima the lowest index is kept, the sums are added in one fixed order), thread 0 writes the
// record.  s_mx / s_arg / s_S: kWaves LDS words each.
constexpr int kPieceBatch = 8;
// the slice of elements [e0, e0 + n) of draft row q that wavefront `wave` of kWaves takes: whole 16-byte vectors
template <typename TD, int kWaves>
__device__ __forceinline__ const TD* piece_wave_slice(const StepArgs& a, int q, int e0, int n, int wave, int* lo, int* n_own) {
  constexpr int kVec = RowVec<TD>::kVec;
  const int slice = ((n + kWaves - 1) / kWaves + kVec - 1) / kVec * kVec;
  *lo = wave * slice;
  *n_own = min(slice, n - *lo);
  return static_cast<const TD*>(a.draft_logits) + (int64_t)q * a.V_d + e0 + *lo;
}

// requests the first batch of this wavefront's slice, for a later workgroup_draft_piece<.., true> of the same piece
template <typename TD, int kWaves>
__device__ __forceinline__ void workgroup_draft_piece_request(const StepArgs& a, int q, int e0, int n, int tid,
                                                              RowFirstBatch<TD, kPieceBatch>& first) {
  int lo, n_own;
  const TD* x = piece_wave_slice<TD, kWaves>(a, q, e0, n, tid >> 6, &lo, &n_own);
  row_first_batch_load<TD, kPieceBatch>(x, n_own, tid & 63, first);
}

template <typename TD, int kWaves, bool kFirst = false>
__device__ __forceinline__ void workgroup_draft_piece(const StepArgs& a, int q, int e0, int n, float Td, int tid,
                                                      float* s_mx, int32_t* s_arg, double* s_S, DraftPiece* out,
                                                      const RowFirstBatch<TD, kPieceBatch>* first = nullptr) {
  const int wave = tid >> 6, lane = tid & 63;
  int lo, n_own;
  const TD* x = piece_wave_slice<TD, kWaves>(a, q, e0, n, wave, &lo, &n_own);
  const float scale = Td > 0.f ? kLog2eF / Td : kLog2eF;
  float mx = -INFINITY;
  int arg = 0x7FFFFFFF;
  double S = 0.0;
  if (n_own > 0) {
    wave_row_stats<TD, kPieceBatch, kFirst>(x, n_own, scale, lane, &mx, &arg, &S, first);
    arg += e0 + lo;
  }
  // The two barriers order LDS accesses only (all LDS operations of this wavefront done, then meet): the fence of
  // __syncthreads() would also wait for the record's store to be acknowledged, microseconds next to a saturating stream.
  auto lds_barrier = []() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0), vmcnt and expcnt unconstrained
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };
  if (lane == 0) { s_mx[wave] = mx; s_arg[wave] = arg; s_S[wave] = S; }
  lds_barrier();
  if (tid == 0) {
    float bm = -INFINITY;
    int ba = 0x7FFFFFFF;
    for (int w = 0; w < kWaves; ++w)
      if (s_mx[w] > bm) { bm = s_mx[w]; ba = s_arg[w]; }     // ascending slices: a later equal maximum does not replace
    double total = 0.0;
    for (int w = 0; w < kWaves; ++w)
      if (s_mx[w] != -INFINITY) total += s_S[w] * (double)__builtin_amdgcn_exp2f((s_mx[w] - bm) * scale);
    DraftPiece r; r.mx = bm; r.arg = ba; r.sum = total;
    *out = r;
  }
  lds_barrier();
}

// Statistics of draft row q from its pieces (ascending order, the merge rule of the slices above): lane-local.
__device__ __forceinline__ void merge_draft_pieces(const StepArgs& a, int q, float Td, float* out_mx, double* out_S,
                                                   int* out_arg) {
  const int j0 = 0, j1 = a.plan.pieces(q) - 1;
  const DraftPiece* rec = a.dpiece + (int64_t)q * kDraftPieces;
  DraftPiece pc[kDraftPieces];
#pragma unroll
  for (int j = 0; j < kDraftPieces; ++j) pc[j] = rec[min(j, j1 - j0)];     // all loads before any use
  const float scale = Td > 0.f ? kLog2eF / Td : kLog2eF;
  float bm = -INFINITY;
  int ba = 0x7FFFFFFF;
#pragma unroll
  for (int j = 0; j < kDraftPieces; ++j)
    if (j <= j1 - j0 && pc[j].mx > bm) { bm = pc[j].mx; ba = pc[j].arg; }
  double total = 0.0;
#pragma unroll
  for (int j = 0; j < kDraftPieces; ++j)
    if (j <= j1 - j0 && pc[j].mx != -INFINITY) total += pc[j].sum * (double)__builtin_amdgcn_exp2f((pc[j].mx - bm) * scale);
  *out_mx = bm; *out_S = total; *out_arg = ba;
}

}  // namespace otv
