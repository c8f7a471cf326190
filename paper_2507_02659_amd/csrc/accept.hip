// Translation of the drafted window into the target vocabulary (Section "Cross-vocabulary N-gram Cache", Eq. 1)
// followed by the acceptance test (Algorithm 1, rejection-sampling step), one workgroup of 768 threads per sequence.
//
// Translation.  The draft rows' softmax partials are merged by 4 threads per row, thread i then forms
// log q_i(d_i); every window (start s, length L) of the drafted ids is probed in the n-gram table by its own thread;
// lane s prepares the segment that would start at s and the window is then walked left to right as a chase
// through start + length: the longest cache hit at s yields one target token whose log q' is the sum of the L
// sub-token log-probabilities (the product of Eq. 1, kept in log space so that five or six factors of 1e-6 do not
// underflow), otherwise the direct image of d_s, and a draft id with neither ends the proposal.
//
// Acceptance.  The target rows' partials are merged the same way.  Lane j of the first wavefront owns mapped
// position j: it forms p_j(t_j), the ratio min(1, p/q') and its Philox uniform; acceptance tests at different
// positions are independent given (u_j, p_j(t_j), q'_j), so "stop at the first rejection" is a ballot and a
// find-first-set, not a loop.  It also writes what the final-token kernels need (FinalInfo).
//
// The kernel touches a few KB and is latency bound, so the three jobs that do not depend on each other run in
// different wavefronts of the workgroup at the same time: threads 0-255 merge the target rows' partials, threads
// 256-511 the draft rows' partials, threads 512-767 fetch the drafted ids, their logits and direct images and probe
// the table.  One barrier later the walk and the acceptance test need only LDS and one gather of z[t_j].
#include "device_math.h"
#include "otv_internal.h"

namespace otv {
namespace {

// Probe of one key held in registers (fully unrolled so that `ids` never has to live in scratch memory).
// Returns the slot index of the entry, or -1.
__device__ inline int cache_lookup(const CacheTable& C, const int32_t (&ids)[OT_MAX_NGRAM_LEN], int L) {
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

// Merges the chunk partials of up to 64 rows starting at row `first`: 4 threads per row, every 4th chunk each,
// combined in a fixed order.  Thread 4*r publishes row r's (max, sum, argmax) to LDS and to the workspace.
__device__ inline void merge_partials(const float* __restrict__ pmax, const double* __restrict__ psum,
                                      const int32_t* __restrict__ parg, int nch, int first, int n_rows, double invT,
                                      float* s_mx, double* s_S, int* s_arg, float* g_mx, double* g_S, int32_t* g_arg,
                                      int local_tid) {
  const int row = local_tid >> 2, part = local_tid & 3;
  const bool live = row < n_rows;
  const int64_t o = (int64_t)(first + (live ? row : 0)) * nch;
  float mx = -INFINITY;
  int arg = 0x7FFFFFFF;
  if (live) {
    for (int c = part; c < nch; c += 4) {
      const float m = pmax[o + c];
      const int ai = parg[o + c];
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
    for (int c = part; c < nch; c += 4) S += psum[o + c] * exp(((double)pmax[o + c] - (double)mx) * invT);
  }
  const double s1 = __shfl_xor(S, 1);
  const double lo = (part & 1) ? s1 + S : S + s1;          // (part0 + part1) or (part2 + part3), same order in both lanes
  const double s2 = __shfl_xor(lo, 2);
  const double total = (part & 2) ? s2 + lo : lo + s2;     // (p0 + p1) + (p2 + p3)
  if (live && part == 0) {
    s_mx[row] = mx; s_S[row] = total; s_arg[row] = arg;
    g_mx[first + row] = mx; g_S[first + row] = total; g_arg[first + row] = arg;
  }
}

__global__ __launch_bounds__(768) void translate_accept_kernel(StepArgs a) {
  const int b = blockIdx.x, tid = threadIdx.x;
  const int role = tid >> 8, g = tid & 255;          // role 0: target rows, 1: draft rows, 2: ids and table probes
  const int r0 = a.row_off[b];
  const int k = a.row_off[b + 1] - r0 - 1;
  const int q0 = r0 - b;
  __shared__ int32_t s_dm[64];
  __shared__ unsigned long long s_hit[64];   // (length << 60) | (slot << 32) | target of the longest cache hit starting here, 0 = none
  __shared__ double s_logq[64];
  __shared__ float s_zq[64];
  __shared__ float s_qmx[64], s_pmx[64];
  __shared__ double s_qS[64], s_pS[64];
  __shared__ int s_qarg[64], s_parg[64];
  __shared__ int s_bad;

  // ---- loads that depend on nothing but b
  const float T = a.temperature[b];
  const float Td = a.draft_temperature ? a.draft_temperature[b] : T;
  const uint64_t sid = a.seq_id[b];
  const double invT = T > 0.f ? 1.0 / (double)T : 1.0;
  const double invTd = Td > 0.f ? 1.0 / (double)Td : 1.0;

  if (tid == 0) s_bad = 0;
  if (tid < 64) { s_hit[tid] = 0ull; s_dm[tid] = -1; }
  __syncthreads();
  if (role == 0) {
    merge_partials(a.tpart_max, a.tpart_sum, a.tpart_arg, a.ncht, r0, k + 1, invT, s_pmx, s_pS, s_parg, a.row_max,
                   a.row_sum, a.row_arg, g);
  } else if (role == 1) {
    merge_partials(a.dpart_max, a.dpart_sum, a.dpart_arg, a.nchd, q0, k, invTd, s_qmx, s_qS, s_qarg, a.drow_max,
                   a.drow_sum, a.drow_arg, g);
  } else {
    if (g < k) {                                // owner of draft position g: range check, drafted logit, direct image
      const int d = a.draft_ids[q0 + g];
      if (d < 0 || d >= a.V_d) {
        s_bad = 1;
      } else {
        const int64_t at = (int64_t)(q0 + g) * a.V_d + d;
        s_zq[g] = a.dtype == OT_BF16 ? bf16_to_f32(static_cast<const uint16_t*>(a.draft_logits)[at])
                                     : static_cast<const float*>(a.draft_logits)[at];
        s_dm[g] = a.dmap[d];
      }
    }
    if (a.cache.slots != nullptr) {            // every window (s, L), L = 2 .. max_len; the longest hit per start wins
      const int nL = a.cache.max_len - 1;
      for (int w = g; w < k * nL; w += 256) {
        const int s = w / nL, L = 2 + w % nL;
        if (s + L <= k) {
          int32_t ids[OT_MAX_NGRAM_LEN];
          bool in_range = true;
#pragma unroll
          for (int i = 0; i < OT_MAX_NGRAM_LEN; ++i) {
            ids[i] = i < L ? a.draft_ids[q0 + s + i] : 0;
            in_range = in_range && ids[i] >= 0 && ids[i] < a.V_d;
          }
          if (in_range) {
            const int slot = cache_lookup(a.cache, ids, L);
            if (slot >= 0) {
              const unsigned int t = (unsigned int)a.cache.slots[(size_t)slot * a.cache.stride + 1];
              atomicMax(&s_hit[s], ((unsigned long long)L << 60) | ((unsigned long long)slot << 32) | t);
            }
          }
        }
      }
    }
  }
  __syncthreads();

  FinalInfo fin;
  fin.mode = 0; fin.row = r0; fin.drow = 0; fin.t_ng = -1; fin.t_pre = -1; fin.argq = -1; fin.greedy_draft = 0;
  fin.pad = 0; fin.pi = 0.0; fin.q_pre = 0.0; fin.u2 = 0.0;
  fin.mx = 0.0; fin.invT = 1.0; fin.invS = 1.0; fin.mxq = 0.0; fin.invTd = 1.0; fin.invSq = 1.0;

  if (s_bad) {                   // a drafted id outside [0, V_d): the sequence emits nothing
    if (tid <= k) {
      a.out.mapped_ids[r0 + tid] = -1; a.out.span_start[r0 + tid] = -1; a.out.span_len[r0 + tid] = 0;
      a.out.out_tokens[r0 + tid] = -1;
      a.out.p_tok[r0 + tid] = 0.f; a.out.q_tok[r0 + tid] = 0.f; a.out.ratio[r0 + tid] = 0.f;
    }
    if (tid == 0) {
      a.out.n_mapped[b] = 0; a.out.hits_proposed[b] = 0; a.out.flags[b] = OT_FLAG_BAD_ID;
      a.out.n_accept[b] = 0; a.out.n_accept_draft[b] = 0; a.out.n_emit[b] = 0; a.out.hits_accepted[b] = 0;
      a.fin[b] = fin;
    }
    return;
  }
  if (tid >= 64) return;          // the rest is one wavefront's work

  // ---- log q_i(d_i)
  if (tid < k) {
    double lq;
    if (Td > 0.f) lq = ((double)s_zq[tid] - (double)s_qmx[tid]) * invTd - log(s_qS[tid]);
    else lq = (a.draft_ids[q0 + tid] == s_qarg[tid]) ? 0.0 : -INFINITY;
    s_logq[tid] = lq;
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");

  // ---- greedy left-to-right walk.  Lane s first prepares the segment that would start at draft position s (the
  // longest cache hit there, else the direct image; log q' = sum of its sub-tokens' log-probabilities); the walk
  // itself is then a chase through "start + length" with wavefront-uniform lane reads, a few cycles per token.
  const int lane = tid;
  int seg_t = -1, seg_L = 1, seg_slot = -1;
  double seg_lq = 0.0;
  if (lane < k) {
    const unsigned long long h = s_hit[lane];
    if (h != 0ull) {
      seg_L = (int)(h >> 60); seg_t = (int)(h & 0xFFFFFFFFull); seg_slot = (int)((h >> 32) & 0x0FFFFFFFull);
    } else {
      seg_t = s_dm[lane];
    }
    for (int l = 0; l < seg_L; ++l) seg_lq += s_logq[lane + l];
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
  const int t_j = lane < m ? got_t : -1;
  const int L_j = lane < m ? got_L : 0;
  const int hits = __popcll(__ballot(lane < m && L_j > 1));
  if (lane < m && L_j > 1) {
    // use statistics of the entry (Appendix, cache eviction): one more use, last used now
    atomicAdd(&a.cache.uses[slot_j], 1u);
    a.cache.last_used[slot_j] = a.cache.clock;
  }
  if (lane == 0) {
    a.out.n_mapped[b] = m;
    a.out.hits_proposed[b] = hits;
    a.out.flags[b] = flags;
  }

  // ---- acceptance test of mapped position `lane` (first wavefront only)
  const uint32_t k0 = (uint32_t)a.seed, k1 = (uint32_t)(a.seed >> 32);
  const float mx = lane <= k ? s_pmx[lane] : 0.f;
  const double S = lane <= k ? s_pS[lane] : 1.0;
  const int arg = lane <= k ? s_parg[lane] : 0;
  bool ok = true;               // lanes >= m do not veto
  double pt = 0.0, qp = 0.0, ratio = 0.0;
  if (lane < m) {
    qp = exp(lq_j);
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
  const unsigned long long rejected = __ballot(!ok);
  const int n = rejected ? (int)__ffsll((long long)rejected) - 1 : m;     // first rejection, or m
  if (lane <= k) {
    a.out.mapped_ids[r0 + lane] = t_j;
    a.out.span_start[r0 + lane] = start_j;
    a.out.span_len[r0 + lane] = L_j;
    a.out.p_tok[r0 + lane] = (float)pt;
    a.out.q_tok[r0 + lane] = (float)qp;
    a.out.ratio[r0 + lane] = (float)ratio;
    // accepted tokens; a greedy sequence's final token is the argmax of row n, which lane n holds
    a.out.out_tokens[r0 + lane] = (lane < n) ? t_j : ((lane == n && !(T > 0.f)) ? arg : -1);
  }
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
        fin.mode = 2;                                   // everything accepted: free token ~ p
      } else {
        fin.mode = 3;                                   // correction token ~ norm(max(0, p - q'))
        const int s = (n < m) ? fin_span_s : s_end;
        fin.drow = q0 + s;
        fin.greedy_draft = !(Td > 0.f);
        fin.invTd = invTd;
        fin.mxq = (double)s_qmx[s];
        fin.invSq = 1.0 / s_qS[s];
        fin.argq = s_qarg[s];
        if (n < m && fin_L > 1) {                       // Eq. 2 overrides for the n-gram matched at this position
          fin.t_ng = fin_t;
          fin.pi = fin_qp;
          fin.t_pre = s_dm[s];
          fin.q_pre = exp(s_logq[s]) - fin_qp;
        }
      }
    }
    a.fin[b] = fin;
  }
}

}  // namespace

hipError_t launch_translate_accept(const StepArgs& a, hipStream_t stream) {
  if (a.B == 0) return hipSuccess;
  hipLaunchKernelGGL(translate_accept_kernel, dim3(a.B), dim3(768), 0, stream, a);
  return hipGetLastError();
}

}  // namespace otv
