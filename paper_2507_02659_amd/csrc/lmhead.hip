// LM-head projection z = h . W for the k+1 verified rows of every sequence (Algorithm 1, the target pass that
// yields p(t_t) .. p(t_{t+m}) in parallel): Z[M, V_t] (fp32) = H[M, d] (bf16) x W[d, V_t] (bf16), fp32 accumulate.
//
// At verification time M = sum_b (k_b + 1) is a few rows to a few hundred, so the product is bound by streaming
// the d x V_t weights from HBM exactly once, not by the matrix cores.  The design follows from that:
//   * W is re-tiled once at init into the register layout of v_mfma_f32_16x16x32_bf16 operands: the fragment for
//     16 vocabulary columns x 32 hidden indices is 64 lanes x 16 bytes, stored contiguously, and the four
//     fragments of 64 adjacent columns per 32-deep step are adjacent.  A wavefront streams the fragments of its
//     columns with fully coalesced 1 KB loads: no transpose anywhere.
//   * Every weight is used by exactly one wavefront, which keeps accumulators for ALL rows of the M-block
//     (up to 11 x 16 rows while the product is bound by HBM), so W is read from HBM once.  More than 176 rows run as
//     several M-blocks of up to 18 x 16 rows per column tile, scheduled so that they share W in one L2.
//   * From 17 rows on, both operands travel by direct global->LDS loads.  The hidden rows, shared by the wavefronts
//     of a workgroup, go through double-buffered slices 128 (or, for the tall M-blocks, 64) columns deep (swizzled
//     rows: conflict-free 16-byte reads); each hidden fragment read from LDS feeds NW MFMAs.  The weight fragments
//     go through a wavefront-private ring four (two) steps deep, so that the one barrier per slice never waits on
//     HBM latency.
//   * The epilogue also reduces each row's logits over the workgroup's columns to softmax partials (maximum, its
//     column, sum of exponentials at the row's temperature), so that no later pass has to read the logits for them.
//   * A workgroup owns 256 columns, or 512 where that lets the launch fit into fewer rounds of one workgroup per
//     compute unit (what a workgroup does outside its main loop is time its compute unit does not stream).
//   * The launch can host the draft side of the step, the work that needs no target logits (see draft-side jobs in
//     the kernel): with one M-block inside the multiplying workgroups, behind their first loads; with several in a
//     few workgroups at the front of the launch.
//   * All waits on the load counter are written by hand, by number (loads complete in issue order), and workgroup
//     barriers carry no fence: with direct-to-LDS loads in flight every wait the compiler adds itself is a full
//     drain of the counter, which would empty the weight pipeline at every slice.
// Operand roles: the weight fragment is MFMA operand A and the hidden fragment operand B, so a lane ends up with
// four consecutive vocabulary columns of one row and stores them as one float4.
#include <algorithm>
#include <cmath>

#include "translate.h"

namespace otv {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));


// Packed layout (16-byte units): unit(wt * packed_tile_units(nks) + (ks * 4 + sub) * 64 + lane) holds
//   W[ks*32 + 8*(lane/16) + e][wt*64 + sub*16 + lane%16], e = 0..7; zero outside [d, V_t].  The gap between tiles is
//   never read.
__global__ __launch_bounds__(256) void pack_w_kernel(const uint16_t* __restrict__ W, int d, int V_t,
                                                     uint4* __restrict__ Wp, int nks, int64_t n_units) {
  const int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (u >= n_units) return;
  const int lane = (int)(u & 63);
  const int sub = (int)((u >> 6) & 3);
  const int64_t rest = u >> 8;
  const int ks = (int)(rest % nks);
  const int wt = (int)(rest / nks);
  const int n = wt * 64 + sub * 16 + (lane & 15);
  const int kb = ks * 32 + 8 * (lane >> 4);
  uint32_t w[4] = {0, 0, 0, 0};
  if (n < V_t) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int kk = kb + e;
      const uint32_t x = kk < d ? (uint32_t)W[(int64_t)kk * V_t + n] : 0u;
      w[e >> 1] |= x << (16 * (e & 1));
    }
  }
  Wp[(int64_t)wt * packed_tile_units(nks) + ((int64_t)ks * 4 + sub) * 64 + lane] = make_uint4(w[0], w[1], w[2], w[3]);
}

// ---------------------------------------------------------------------------------------------------------------
// Wide kernel: M-blocks of up to MT*16 rows.  WPG wavefronts per workgroup, each owning NW*16 columns over the whole
// hidden dimension.  The hidden slice (KC columns of all rows of the M-block) is double-buffered in LDS and filled
// by direct global->LDS loads (no staging registers): the next slice is requested before the current one feeds the
// MFMAs, and one barrier per slice hands the buffers over.  LDS rows are unpadded; the 16-byte chunks of a row are
// XOR-swizzled with the row index (applied on the global side of the copy, since a direct load writes consecutive
// lanes to consecutive LDS addresses) so that the 16 rows a fragment read touches fall into 16 distinct bank groups.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;

// s_waitcnt immediate (gfx9 encoding) that waits until at most N vector-memory loads are outstanding and nothing else
constexpr int vmcnt_imm(int n) { return (n & 0xF) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

// Workgroup barrier without the memory fence of __syncthreads().  The fence makes the compiler drain every
// outstanding vector-memory load (it cannot tell a direct-to-LDS load that must be visible from a register prefetch
// that need not be), which would empty the prefetch pipelines at every hand-over.  The kernels below wait by count for
// exactly the loads that have to be visible (s_waitcnt above) and then meet here; LDS reads of the buffer that is
// handed back have been consumed by MFMAs before a wavefront arrives.
// The empty asm statements keep the compiler from moving memory accesses across the barrier.
__device__ inline void wg_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Barrier that publishes this wavefront's LDS writes (all LDS operations done) without touching the load counter.
__device__ inline void lds_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0), vmcnt and expcnt unconstrained
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

constexpr int gcd_c(int a, int b) { return b == 0 ? a : gcd_c(b, a % b); }
// largest divisor of n that is at most `limit` (limit >= 1)
constexpr int largest_divisor_c(int n, int limit) { return n % limit == 0 ? limit : largest_divisor_c(n, limit - 1); }

template <int MT, int PF, int WPG, int KC, int NW, bool W_ONCE>
__global__ __launch_bounds__(WPG * 64) void lmhead_bf16_wide_kernel(const uint16_t* __restrict__ H, int M, int d,
                                                                    const uint4* __restrict__ Wp, int nks,
                                                                    int n_wtiles, float* __restrict__ Z, int V_t,
                                                                    int64_t ldz, int vec_store,
                                                                    const uint16_t* __restrict__ zeros, int m_blocks,
                                                                    FusedStats fs, int n_front, int n_piece_jobs,
                                                                    int helpers_look_up, StepArgs ds) {
  constexpr int kKSteps = KC / 32;                 // MFMA steps per slice
  constexpr int kCPR = KC / 8;                     // 16-byte chunks per slice row
  constexpr int kSliceChunks = MT * 16 * kCPR;
  constexpr int kDma = (kSliceChunks + WPG * 64 - 1) / (WPG * 64);
  static_assert(kSliceChunks % 64 == 0 && kSliceChunks >= 64, "a slice is a whole number of wavefront-wide loads");
  constexpr int kPatchRow = NW * 16 + 4;           // floats per padded row of the epilogue patch
  // steps per trip of the main loop: whole pairs of slices (buffers A, B) and whole turns of the weight ring, so
  // that both the buffer and the ring array of every step are known at compile time
  constexpr int kUnroll = 2 * kKSteps * PF / gcd_c(2 * kKSteps, PF);
  static_assert(PF % kKSteps == 0 && PF <= 6, "a weight fetch is used a whole number of slices later");
  static_assert(kGemmKPad % KC == 0 && (kCPR == 8 || kCPR == 16), "slice geometry");
  static_assert((PF - 1) * NW + (PF / kKSteps) * kDma + NW < 64, "the load counter has 6 bits");
  static_assert(NW == 1 || NW == 2 || NW == 4, "a wavefront owns 16, 32 or 64 columns");
  __shared__ __attribute__((aligned(16))) uint16_t sA[MT * 16 * KC];
  __shared__ __attribute__((aligned(16))) uint16_t sB[MT * 16 * KC];
  __shared__ __attribute__((aligned(16))) float sPatch[WPG][16 * kPatchRow];   // epilogue: one 16-row tile per wavefront
  // The weight fragments travel by direct global->LDS loads as well, into a ring of PF steps: one array per step (so
  // that the compiler can tell them apart), each wavefront using its own NW KB of every array.  A register prefetch
  // next to direct-to-LDS loads would make the compiler drain the load counter at each first use of a register.
  // (Measured: fetching the weights into registers eight steps ahead instead, which doubles the bytes in flight per CU
  // and keeps them out of LDS, is no faster at 144 rows: 222 against 218 us per step.)
  constexpr int kRing = WPG * NW * 64;
  __shared__ uint4 sW0[kRing], sW1[kRing], sW2[PF > 2 ? kRing : 1], sW3[PF > 3 ? kRing : 1], sW4[PF > 4 ? kRing : 1],
      sW5[PF > 5 ? kRing : 1];
  // fused row statistics: row offsets and temperatures of the sequences (staged by direct loads in the prologue),
  // and the exponent scale log2(e)/T of each row of the M-block
  __shared__ int32_t sRowOff[kFusedMaxB + 1];
  __shared__ float sTemp[kFusedMaxB + 1];
  __shared__ float sTempDraft[kFusedMaxB + 1];       // the drafter's temperatures, staged only when they are given apart
  __shared__ float sScale[MT * 16];
  static_assert(WPG * 64 >= kFusedMaxB + 1, "one thread per sequence stages its row offset and temperature");
  static_assert((WPG & (WPG - 1)) == 0, "the mask below tells the compiler the range of the wavefront index");
  const int tid = threadIdx.x, wave = (tid >> 6) & (WPG - 1), lane = tid & 63;
  // The first n_front workgroups of the launch (a multiple of 8) multiply nothing: they run the draft side (see below).
  const int wg = (int)blockIdx.x - n_front;
  // Workgroup id -> (column tile, M-block).  Consecutive ids go round-robin to the 8 XCDs, each with its own L2; the
  // M-blocks of one column tile get ids that land on the same XCD back to back, so that when M needs several
  // blocks their weight streams coincide in that XCD's L2 and HBM is still read once.
  const int xcd = wg & 7, slot = wg >> 3;
  const int col_tile = (slot / m_blocks) * 8 + xcd, m_block = slot % m_blocks;
  const int n_col_tiles = (n_wtiles * 4 + WPG * NW - 1) / (WPG * NW);
  const bool hosts = n_piece_jobs > 0;               // this launch runs the draft side of the step (see below)
  // stages the sequences' row offsets and temperatures in LDS (4-byte direct loads: lane i of a wavefront fills entry
  // 64*wave + i); a wait for the loads and a barrier follow
  auto stage_sequences = [&]() {
    if (fs.part && wave * 64 <= fs.B) {
      __builtin_amdgcn_global_load_lds((glb_ptr_t)(fs.row_off + min(tid, fs.B)), (lds_ptr_t)(sRowOff + wave * 64), 4, 0,
                                       0);
      __builtin_amdgcn_global_load_lds((glb_ptr_t)(fs.temperature + min(tid, fs.B - 1)), (lds_ptr_t)(sTemp + wave * 64),
                                       4, 0, 0);
      if (hosts && ds.draft_temperature)
        __builtin_amdgcn_global_load_lds((glb_ptr_t)(ds.draft_temperature + min(tid, fs.B - 1)),
                                         (lds_ptr_t)(sTempDraft + wave * 64), 4, 0, 0);
    }
  };
  // The draft side of the step, the part that needs none of the logits, comes in two kinds of jobs.
  // Piece job j: the softmax statistics (a3) of one piece of a draft row (see PiecePlan); at most one per multiplying
  // workgroup, which asks for it in front of its first loads and reduces it while those land.  Lookup job b: what the
  // drafted ids of sequence b look up (the drafted logit, the direct image, the n-gram table probes of every window),
  // left as a ProbeRecord for the next launch, which walks the windows.
  // All threads call a job (workgroup barriers inside).
  // Every lane holds the row offsets and the drafter's temperatures of sequences lane, lane + 64, ...: the owner of a
  // draft row (the last b with row_off[b] - b <= q, a monotone predicate) is then a count over ballots and its
  // temperature one lane read, with no chain of dependent loads.  piece_request asks for these and for the first
  // batch of the job's first row piece; piece_job (later, so that the loads overlap whatever is issued in between)
  // reduces it and goes through the rest of the chunk.
  constexpr int kSeqRegs = (kFusedMaxB + 64) / 64;
  int seq_before[kSeqRegs];
  float seq_temp[kSeqRegs];
  RowFirstBatch<uint16_t, kPieceBatch> first_batch;
  auto piece_request = [&](int job) {
    const float* temps = ds.draft_temperature ? ds.draft_temperature : fs.temperature;
#pragma unroll
    for (int j = 0; j < kSeqRegs; ++j) {
      const int b = min(64 * j + lane, fs.B - 1);
      seq_before[j] = fs.row_off[b] - b;
      seq_temp[j] = temps[b];
    }
    int q, i, e0, n;
    ds.plan.locate(job, &q, &i);
    PiecePlan::span(ds.V_d, ds.plan.pieces(q), i, &e0, &n);
    workgroup_draft_piece_request<uint16_t, WPG>(ds, q, e0, n, tid, first_batch);
  };
  auto piece_job = [&](int job) {
    float* st_mx = reinterpret_cast<float*>(&sPatch[0][0]);
    int32_t* st_arg = reinterpret_cast<int32_t*>(st_mx + WPG);
    double* st_S = reinterpret_cast<double*>(st_mx + 2 * WPG);
    int q, i, e0, n;
    ds.plan.locate(job, &q, &i);
    bool first = true;
    for (; q < ds.K; q += ds.plan.workers) {
      PiecePlan::span(ds.V_d, ds.plan.pieces(q), i, &e0, &n);
      int owner = -1;
      float Td = 1.f;
#pragma unroll
      for (int j = 0; j < kSeqRegs; ++j) {
        const bool before = 64 * j + lane < fs.B && seq_before[j] <= q;
        owner += __popcll(__ballot(before));
      }
#pragma unroll
      for (int j = 0; j < kSeqRegs; ++j) {
        const float t = __shfl(seq_temp[j], owner & 63);
        if ((owner >> 6) == j) Td = t;
      }
      DraftPiece* out = ds.dpiece + (int64_t)q * kDraftPieces + i;
      if (first) workgroup_draft_piece<uint16_t, WPG, true>(ds, q, e0, n, Td, tid, st_mx, st_arg, st_S, out, &first_batch);
      else workgroup_draft_piece<uint16_t, WPG>(ds, q, e0, n, Td, tid, st_mx, st_arg, st_S, out);
      first = false;
    }
  };
  // The same for one wavefront on its own (front workgroups: every wavefront is a worker of the plan): no workgroup
  // barriers, and 16 sixteen-byte loads in flight per lane, because a workgroup that only reads next to the other
  // workgroups' streams gets the bytes it keeps in flight once per several microseconds.
  auto wave_piece_jobs = [&](int job) {
    const float* temps = ds.draft_temperature ? ds.draft_temperature : fs.temperature;
#pragma unroll
    for (int j = 0; j < kSeqRegs; ++j) {
      const int b = min(64 * j + lane, fs.B - 1);
      seq_before[j] = fs.row_off[b] - b;
      seq_temp[j] = temps[b];
    }
    int q, i, e0, n;
    ds.plan.locate(job, &q, &i);
    for (; q < ds.K; q += ds.plan.workers) {
      PiecePlan::span(ds.V_d, ds.plan.pieces(q), i, &e0, &n);
      int owner = -1;
      float Td = 1.f;
#pragma unroll
      for (int j = 0; j < kSeqRegs; ++j) {
        const bool before = 64 * j + lane < fs.B && seq_before[j] <= q;
        owner += __popcll(__ballot(before));
      }
#pragma unroll
      for (int j = 0; j < kSeqRegs; ++j) {
        const float t = __shfl(seq_temp[j], owner & 63);
        if ((owner >> 6) == j) Td = t;
      }
      DraftPiece r; r.mx = -INFINITY; r.arg = 0x7FFFFFFF; r.sum = 0.0;
      if (n > 0) {
        wave_row_stats<uint16_t, 16>(static_cast<const uint16_t*>(ds.draft_logits) + (int64_t)q * ds.V_d + e0, n,
                                     Td > 0.f ? kLog2eF / Td : kLog2eF, lane, &r.mx, &r.arg, &r.sum);
        r.arg += e0;
      }
      if (lane == 0) ds.dpiece[(int64_t)q * kDraftPieces + i] = r;
    }
  };
  auto lookup_job = [&](int b) {               // the sequences are staged in LDS
    DraftLds* probe_lds = reinterpret_cast<DraftLds*>(&sPatch[0][0]);
    static_assert(sizeof(DraftLds) <= sizeof(sPatch), "the lookups' scratch fits into the epilogue patch");
    const int r0 = sRowOff[b], k = sRowOff[b + 1] - r0 - 1;
    draft_lds_reset(probe_lds, tid);
    __syncthreads();
    fetch_ids_and_probe(ds, r0 - b, k, tid, WPG * 64, probe_lds);
    __syncthreads();
    ProbeRecord* rec = ds.probe + b;
    if (tid < 64) { rec->hit[tid] = probe_lds->hit[tid]; rec->zq[tid] = probe_lds->zq[tid]; rec->dm[tid] = probe_lds->dm[tid]; }
    if (tid == 0) rec->bad = probe_lds->bad;
    __syncthreads();
  };
  // A workgroup with nothing to multiply takes the lookups of every n_helpers-th group of four sequences, 128 threads
  // each: next to the other workgroups' weight streams every dependent load of a lookup takes several microseconds, and
  // so the chains of loads of four sequences run side by side.  The sequences are staged first.
  auto helper_lookups = [&](int helper, int n_helpers) {
    stage_sequences();
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    wg_barrier();
    constexpr int kAtOnce = WPG * 64 / 128;
    static_assert(sizeof(DraftLds) * kAtOnce <= sizeof(sPatch), "the lookups' scratch fits into the epilogue patch");
    const int slot = tid >> 7, g = tid & 127;
    DraftLds* L = reinterpret_cast<DraftLds*>(&sPatch[0][0]) + slot;
    for (int b0 = helper; b0 < fs.B; b0 += kAtOnce * n_helpers) {
      const int b = b0 + slot * n_helpers;
      const bool valid = b < fs.B;
      const int r0 = valid ? sRowOff[b] : 0, k = valid ? sRowOff[b + 1] - r0 - 1 : 0;
      if (valid) draft_lds_reset(L, g);
      __syncthreads();
      if (valid) fetch_ids_and_probe(ds, r0 - b, k, g, 128, L);
      __syncthreads();
      if (valid && g < 64) {
        ProbeRecord* rec = ds.probe + b;
        rec->hit[g] = L->hit[g]; rec->zq[g] = L->zq[g]; rec->dm[g] = L->dm[g];
        if (g == 0) rec->bad = L->bad;
      }
      __syncthreads();
    }
  };
  if (wg < 0) {
    // Front workgroups: the whole draft side of a launch that is bound by the matrix cores (several M-blocks), where a
    // piece in front of every multiplying workgroup's loop would add its time to each of them.  They start first and
    // are done long before the launch ends; every wavefront of them is a worker of the plan, and front workgroup h takes
    // its share of the lookups.
    // The lookups come first: their chains of dependent loads are short while the launch has not yet filled the
    // memory system, and several times as long afterwards.
    const int h = (int)blockIdx.x;
    helper_lookups(h, n_front);
    if (h * WPG + wave < n_piece_jobs) wave_piece_jobs(h * WPG + wave);
    return;
  }
  if (col_tile >= n_col_tiles) {
    // Padding of the id space: a workgroup with nothing to multiply.  Where the launch has such workgroups and they can
    // finish in time (the host decides), they take the sequences' lookups, on compute units that the multiplying
    // workgroups leave idle.  (The draft rows stay with the multiplying workgroups: next to their saturating streams a
    // workgroup that only reads was measured at about 10 GB/s however many loads it keeps in flight, so five of them
    // cannot get through 8 MB of draft logits in time.)
    if (helpers_look_up && hosts) {
      const int n_pad_tiles = (n_col_tiles + 7) / 8 * 8 - n_col_tiles;
      helper_lookups((col_tile - n_col_tiles) * m_blocks + m_block, n_pad_tiles * m_blocks);
    }
    return;
  }
  const int t16_own = (col_tile * WPG + wave) * NW;   // first 16-column tile of this wavefront
  const bool active = t16_own < n_wtiles * 4;
  // A wavefront past the last tile (only in the last workgroup) multiplies the last tile again and stores nothing:
  // the main loop then has no wavefront-dependent branch and every wavefront issues the same loads in the same order.
  const int t16 = active ? t16_own : n_wtiles * 4 - NW;
  const int row0 = m_block * (MT * 16);
  // fragment (16-column tile t, step ks) sits at 16-byte unit (t/4) * packed_tile_units(nks) + (ks * 4 + t%4) * 64 + lane
  const uint4* wp = Wp + (int64_t)(t16 / 4) * packed_tile_units(nks) + (t16 % 4) * 64 + lane;

  // Swizzle key of a row: the 16-byte chunks of a row are XORed with the low bits of the row index (measured: with
  // 128-byte rows, folding bit 3 of the row into the key as well stalls 46 % of the LDS cycles on bank conflicts,
  // the plain low bits 2 %).
  auto row_key = [](int row) { return row & (kCPR - 1); };
  // request slice kc (in 32-column steps) into buffer s: chunk q of the buffer holds logical chunk (q%kCPR)^key(row).
  // A request past the end of K re-reads the last slice, so that every slice issues the same number of loads and
  // the in-order load counter can be waited on by number.
  auto request = [&](int kc_want, uint16_t* s) {
    const int kc = min(kc_want, nks - kKSteps);
#pragma unroll
    for (int j = 0; j < kDma; ++j) {
      // wave-uniform.  A wavefront whose turn falls past the end loads the last 64 chunks once more (the same bytes to
      // the same place as their owner): every wavefront then issues exactly kDma loads per slice, the loop has no
      // branch, and the load counter can be waited on by number.
      const int q0 = min((j * WPG + wave) * 64, kSliceChunks - 64);
      {
        const int q = q0 + lane;
        const int row = q / kCPR, pc = q % kCPR;
        const int lc = pc ^ row_key(row);
        const int gr = min(row0 + row, M - 1);     // rows past M are never stored: any valid row will do
        const int gk = kc * 32 + lc * 8;
        const uint16_t* src = gk < d ? H + (int64_t)gr * d + gk : zeros;   // the padded tail of K must read as zero
        __builtin_amdgcn_global_load_lds((glb_ptr_t)src, (lds_ptr_t)(s + q0 * 8), 16, 0, 0);
      }
    }
  };
  auto ring = [&](int s) -> uint4* {
    return (s == 0 ? sW0 : s == 1 ? sW1 : s == 2 ? sW2 : s == 3 ? sW3 : s == 4 ? sW4 : sW5) + wave * (NW * 64);
  };
  // fetch the fragments of step kf into this wavefront's part of ring array s
  // With a single M-block every weight is read exactly once by the whole launch: those loads are marked nontemporal
  // (cache-policy bit 1 of the load), which a plain streaming read of the same bytes was measured to gain 12 % from
  // (7.05 against 6.3 TB/s).  With several M-blocks the later ones find the weights in L2 and the mark would not help.
  constexpr int kWeightPolicy = W_ONCE ? 2 : 0;
  auto fetch_w = [&](int kf, int s) {
#pragma unroll
    for (int nw = 0; nw < NW; ++nw)
      __builtin_amdgcn_global_load_lds((glb_ptr_t)(wp + ((int64_t)kf * 4 + nw) * 64), (lds_ptr_t)(ring(s) + nw * 64), 16,
                                       0, kWeightPolicy);
  };

  // This workgroup's piece of the draft rows is asked for first: it is reduced while the first weight fragments and the
  // hidden slice, asked for right behind it, land.  2 to 3 us that the launch which follows no longer has to wait for.
  const int own_job = col_tile * m_blocks + m_block;
  // (only a launch with a single M-block gives its multiplying workgroups pieces: W_ONCE says so at compile time, which
  // keeps the piece's registers out of the kernels whose accumulators leave none to spare)
  const bool has_job = W_ONCE && n_front == 0 && own_job < n_piece_jobs;
  if (has_job) piece_request(own_job);
  request(0, sA);
#pragma unroll
  for (int s = 0; s < PF; ++s) fetch_w(min(s, nks - 1), s);
  stage_sequences();
  if (has_job) piece_job(own_job);
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
  wg_barrier();
  // Without idle workgroups to take them, the lookups go to the multiplying workgroups as well, from the last one down.
  if (hosts && !helpers_look_up && n_front == 0)
    for (int b = n_col_tiles * m_blocks - 1 - own_job; b < fs.B; b += n_col_tiles * m_blocks) lookup_job(b);

  f32x4 acc[MT][NW];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nw = 0; nw < NW; ++nw) acc[mt][nw] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int a_row = lane & 15, a_grp = lane >> 4;
  // one slice out of buffer hs; kc = its first step, s0 = ring array of that step (compile-time after unrolling)
  auto compute = [&](const uint16_t* hs, int kc, int s0) {
#pragma unroll
    for (int ks = 0; ks < kKSteps; ++ks) {
      const int kk = kc + ks;
      const int rs = (s0 + ks) % PF;
      // This step's weight fragments were requested PF steps ago; since then PF-1 refills and PF/kKSteps hidden slices
      // were requested, so they have landed once no more loads than that are outstanding.  Waiting by number here
      // (with an instruction between the wait and the read) also spares the compiler from inserting its own wait,
      // which with direct-to-LDS loads in flight is always a full drain.
      __builtin_amdgcn_s_waitcnt(vmcnt_imm((PF - 1) * NW + (PF / kKSteps) * kDma));
      asm volatile("s_nop 0");
      __builtin_amdgcn_sched_barrier(0);
      uint4 bw[NW];
#pragma unroll
      for (int nw = 0; nw < NW; ++nw) bw[nw] = ring(rs)[nw * 64 + lane];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int pc = (ks * 4 + a_grp) ^ row_key(a_row);
        const uint4 hv = *reinterpret_cast<const uint4*>(&hs[(mt * 16 + a_row) * KC + pc * 8]);
        const bf16x8 hf = __builtin_bit_cast(bf16x8, hv);
#pragma unroll
        for (int nw = 0; nw < NW; ++nw) {
          acc[mt][nw] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, bw[nw]), hf, acc[mt][nw],
                                                                0, 0, 0);
        }
      }
      // the ring array is free again: refill it with the fragments PF steps ahead (past the end: the last ones again)
      fetch_w(min(kk + PF, nks - 1), rs);
      __builtin_amdgcn_sched_barrier(0);   // keep the next step's LDS reads from being hoisted (register budget)
    }
  };
  // Loads complete in issue order, so once at most kKSteps*NW loads (the weight fragments requested during the slice)
  // are outstanding, this wavefront's part of the next hidden slice has landed in LDS.
  auto hand_over = [&]() {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(kKSteps * NW));
    wg_barrier();
  };

  // Whole trips run without a branch inside (the compiler's bookkeeping of the load counter degrades to full drains at
  // the first use of a loaded register behind any control-flow merge that a shorter path could reach); the slices that
  // are left after the last whole trip follow as straight-line code behind forward branches.
  auto one_slice = [&](int kc, int p) {
    request(kc + kKSteps, (p & 1) ? sA : sB);
    __builtin_amdgcn_sched_barrier(0);
    compute((p & 1) ? sB : sA, kc, (p * kKSteps) % PF);
    hand_over();
  };
  int base = 0;
  for (; base + kUnroll <= nks; base += kUnroll) {
#pragma unroll
    for (int p = 0; p < kUnroll / kKSteps; ++p) one_slice(base + p * kKSteps, p);
  }
#pragma unroll
  for (int p = 0; p < kUnroll / kKSteps - 1; ++p)
    if (base + p * kKSteps < nks) one_slice(base + p * kKSteps, p);
  if (fs.part) {
    // Row statistics of this workgroup's column tile, from the accumulators: per row the maximum, its lowest column
    // and sum exp((z - max)/T), first per wavefront (NW*16 columns), then merged over the wavefronts; one partial per
    // row and column tile goes to memory.  All LDS buffers of the main loop are free: every wavefront has passed the
    // barrier that followed its last slice (the weight ring may still receive the surplus refills; it is not used).
    // The statistics scratch (3 x 4 bytes per lane and row tile) reuses LDS of the main loop: either both hidden
    // buffers (maxima and sums in the first, columns in the second), or, where that holds fewer row tiles at once, one
    // hidden buffer each for the maxima and the sums and the first weight-ring array for the columns (the ring is
    // drained first: the surplus refills past the end of K still land there).  Not the epilogue patch: a wavefront that
    // is done here goes on to turn its logits through its part of the patch while the merging threads still read.
    // When even that is too small for all row tiles at once the row tiles are taken in groups of kStatMT.
    constexpr int kFitHidden = MT * KC / (16 * WPG), kFitSpread = MT * KC / (8 * WPG) < 4 * NW ? MT * KC / (8 * WPG) : 4 * NW;
    // row tiles per group: the largest divisor of MT that fits, in whichever layout allows the larger one
    constexpr int kGroupHidden = largest_divisor_c(MT, kFitHidden < MT ? kFitHidden : MT);
    constexpr int kGroupSpread = largest_divisor_c(MT, kFitSpread < MT ? kFitSpread : MT);
    constexpr bool kSpread = kGroupSpread > kGroupHidden;
    constexpr int kStatMT = kSpread ? kGroupSpread : kGroupHidden;
    static_assert(kStatMT >= 1 && MT % kStatMT == 0, "row tiles split evenly into statistics groups");
    static_assert(sizeof(float) * WPG * kStatMT * 64 * (kSpread ? 1 : 2) <= sizeof(sA) &&
                  sizeof(float) * WPG * kStatMT * 64 <= (kSpread ? sizeof(sW0) : sizeof(sB)), "the scratch fits");
    float* st_max = reinterpret_cast<float*>(sA);
    float* st_sum = kSpread ? reinterpret_cast<float*>(sB) : st_max + WPG * kStatMT * 64;
    int32_t* st_arg = kSpread ? reinterpret_cast<int32_t*>(sW0) : reinterpret_cast<int32_t*>(sB);
    if (kSpread) __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));   // before the barrier below
    for (int r = tid; r < MT * 16; r += WPG * 64) {
      const int row = min(row0 + r, M - 1);
      int lo = 0, hi = fs.B - 1;                    // sequence that owns the row: last b with row_off[b] <= row
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (sRowOff[mid] <= row) lo = mid; else hi = mid - 1;
      }
      const float T_b = sTemp[lo];
      sScale[r] = T_b > 0.f ? 1.4426950408889634f / T_b : 1.4426950408889634f;
    }
    lds_barrier();
    // every lane reduces its own NW*4 values of a row (no cross-lane traffic) and parks the partial in LDS; only a
    // wavefront that reaches past column V_t (or repeats the last tile) has to mask
    const int n_valid = active ? V_t - (t16 * 16 + 4 * (lane >> 4)) : 0;   // this lane's columns n0 + 16*nw + e < V_t
    const bool all_valid = __builtin_amdgcn_readfirstlane(active && (t16 + NW) * 16 <= V_t);
#pragma unroll
    for (int h = 0; h < MT; h += kStatMT) {
#pragma unroll
      for (int ml = 0; ml < kStatMT; ++ml) {
        const int mt = h + ml;
        const float sc = sScale[mt * 16 + (lane & 15)];
        float v[NW * 4];
#pragma unroll
        for (int nw = 0; nw < NW; ++nw)
#pragma unroll
          for (int e = 0; e < 4; ++e)
            v[nw * 4 + e] = (all_valid || nw * 16 + e < n_valid) ? acc[mt][nw][e] : -INFINITY;
        float best = v[0];
        int bi = 0;
#pragma unroll
        for (int i = 1; i < NW * 4; ++i)            // ascending columns: the first maximum is kept
          if (v[i] > best) { best = v[i]; bi = i; }
        const int barg = best == -INFINITY ? 0x7FFFFFFF : t16 * 16 + 4 * (lane >> 4) + (bi >> 2) * 16 + (bi & 3);
        const float nb = best == -INFINITY ? 0.f : -best * sc;
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < NW * 4; ++i) sum += __builtin_amdgcn_exp2f(fmaf(v[i], sc, nb));   // masked: exp2(-inf) = 0
        const int at = (wave * (kStatMT * 16) + ml * 16 + (lane & 15)) * 4 + (lane >> 4);
        st_max[at] = best; st_sum[at] = sum; st_arg[at] = barg;
      }
      lds_barrier();
      // one thread per row merges the WPG x 4 partials in a fixed order and writes the tile's partial
      if (tid < kStatMT * 16 && row0 + h * 16 + tid < M) {
        const float sc = sScale[h * 16 + tid];
        float best = -INFINITY;
        int barg = 0x7FFFFFFF;
#pragma unroll
        for (int w = 0; w < WPG; ++w) {
          const f32x4 m4 = *reinterpret_cast<const f32x4*>(&st_max[(w * (kStatMT * 16) + tid) * 4]);
          const int4 a4 = *reinterpret_cast<const int4*>(&st_arg[(w * (kStatMT * 16) + tid) * 4]);
          const int a[4] = {a4.x, a4.y, a4.z, a4.w};
#pragma unroll
          for (int g = 0; g < 4; ++g)
            if (m4[g] > best || (m4[g] == best && a[g] < barg)) { best = m4[g]; barg = a[g]; }
        }
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < WPG; ++w) {
          const f32x4 m4 = *reinterpret_cast<const f32x4*>(&st_max[(w * (kStatMT * 16) + tid) * 4]);
          const f32x4 s4 = *reinterpret_cast<const f32x4*>(&st_sum[(w * (kStatMT * 16) + tid) * 4]);
#pragma unroll
          for (int g = 0; g < 4; ++g)
            if (m4[g] != -INFINITY) sum += s4[g] * __builtin_amdgcn_exp2f((m4[g] - best) * sc);
        }
        Partial out;
        out.mx = best; out.arg = barg; out.sum = (double)sum;
        fs.part[(int64_t)(row0 + h * 16 + tid) * fs.nfine + col_tile] = out;
      }
      if (h + kStatMT < MT) lds_barrier();         // the next group overwrites the scratch
    }
  }
  if (!active) return;
  // Epilogue.  After the MFMAs a lane holds Z[row0 + mt*16 + lane%16][(t16 + nw)*16 + 4*(lane/16) + 0..3]: 64-byte
  // pieces of 16 rows per store.  Each 16-row tile is turned through a wave-private LDS patch (padded rows) so that a
  // store instruction writes whole rows of the wavefront's columns contiguously.  With several M-blocks the logits are
  // written with nontemporal stores: they are not re-read by this kernel and should not evict the weights that the
  // other M-blocks of the column tile are about to find in L2 (measured at 160 rows: 242 against 253 us per step).  With
  // one M-block nothing in L2 is worth keeping, and plain stores were measured 1 % faster (144 rows: 205 against 207 us).
  float* patch = sPatch[wave];
  constexpr int kVecPerRow = NW * 4;                   // float4 per patch row
  constexpr int kIters = 16 * kVecPerRow / 64;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
    for (int nw = 0; nw < NW; ++nw)
      *reinterpret_cast<f32x4*>(&patch[(lane & 15) * kPatchRow + nw * 16 + 4 * (lane >> 4)]) = acc[mt][nw];
#pragma unroll
    for (int i = 0; i < kIters; ++i) {
      const int idx = i * 64 + lane;
      const int r = idx / kVecPerRow, c4 = idx % kVecPerRow;
      const f32x4 v = *reinterpret_cast<const f32x4*>(&patch[r * kPatchRow + 4 * c4]);
      const int m = row0 + mt * 16 + r;
      const int n = t16 * 16 + 4 * c4;
      if (m < M) {
        float* dst = Z + (int64_t)m * ldz + n;
        if (vec_store && n + 3 < V_t) {
          if (W_ONCE) *reinterpret_cast<f32x4*>(dst) = v;
          else __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(dst));
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (n + e < V_t) dst[e] = v[e];
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------------------------
// Skinny kernel: M <= 16 rows (one MFMA row tile).  A workgroup owns 64 columns and splits the hidden dimension
// over its 8 wavefronts, so that even a 32000-column head yields thousands of wavefronts streaming W; the hidden
// fragments are tiny and read straight from global memory (L2 resident).  The 8 partial tiles are summed through
// LDS in a fixed order.
template <int PF>
__global__ __launch_bounds__(512) void lmhead_bf16_skinny_kernel(const uint16_t* __restrict__ H, int M, int d,
                                                                 const uint4* __restrict__ Wp, int nks,
                                                                 float* __restrict__ Z, int V_t, int64_t ldz) {
  constexpr int kWaves = 8;
  __shared__ __attribute__((aligned(16))) float sRed[kWaves][4][64][4];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wt = blockIdx.x;
  const int ks0 = (int)(((int64_t)nks * wave) / kWaves), ks1 = (int)(((int64_t)nks * (wave + 1)) / kWaves);
  const uint4* wp = Wp + (int64_t)wt * packed_tile_units(nks) + lane;
  const int h_row = lane & 15, h_col = 8 * (lane >> 4);
  const bool h_ok = h_row < M;
  const uint16_t* hp = H + (int64_t)(h_ok ? h_row : 0) * d + h_col;

  f32x4 acc[4];
#pragma unroll
  for (int nw = 0; nw < 4; ++nw) acc[nw] = f32x4{0.f, 0.f, 0.f, 0.f};
  uint4 bq[PF][4], hq[PF];
  auto fetch = [&](int slot, int ks) {
#pragma unroll
    for (int nw = 0; nw < 4; ++nw) {               // read once by the whole launch: nontemporal (see the wide kernel)
      const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(wp + ((int64_t)ks * 4 + nw) * 64));
      bq[slot][nw] = make_uint4(v.x, v.y, v.z, v.w);
    }
    hq[slot] = make_uint4(0, 0, 0, 0);
    if (h_ok && ks * 32 + h_col < d) hq[slot] = *reinterpret_cast<const uint4*>(hp + ks * 32);
  };
#pragma unroll
  for (int s = 0; s < PF; ++s) {
    if (ks0 + s < ks1) fetch(s, ks0 + s);
  }
  for (int base = ks0; base < ks1; base += PF) {
#pragma unroll
    for (int s = 0; s < PF; ++s) {
      const int ks = base + s;
      if (ks < ks1) {
        uint4 bw[4];
#pragma unroll
        for (int nw = 0; nw < 4; ++nw) bw[nw] = bq[s][nw];
        const bf16x8 hf = __builtin_bit_cast(bf16x8, hq[s]);
        if (ks + PF < ks1) fetch(s, ks + PF);
#pragma unroll
        for (int nw = 0; nw < 4; ++nw)
          acc[nw] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, bw[nw]), hf, acc[nw], 0, 0, 0);
      }
    }
  }
#pragma unroll
  for (int nw = 0; nw < 4; ++nw)
    *reinterpret_cast<float4*>(&sRed[wave][nw][lane][0]) = make_float4(acc[nw][0], acc[nw][1], acc[nw][2], acc[nw][3]);
  __syncthreads();
  if (tid < 256) {
    const int nw = tid >> 6, l = tid & 63;
    float4 sum = *reinterpret_cast<const float4*>(&sRed[0][nw][l][0]);
#pragma unroll
    for (int w = 1; w < kWaves; ++w) {
      const float4 x = *reinterpret_cast<const float4*>(&sRed[w][nw][l][0]);
      sum.x += x.x; sum.y += x.y; sum.z += x.z; sum.w += x.w;
    }
    const int m = l & 15;
    const int n = wt * 64 + nw * 16 + 4 * (l >> 4);
    if (m < M) {
      float* dst = Z + (int64_t)m * ldz + n;
      const float v[4] = {sum.x, sum.y, sum.z, sum.w};
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (n + e < V_t) dst[e] = v[e];
    }
  }
}

// fp32 path (meant for small fp32 problems; no matrix cores): a thread owns one vocabulary column for kF32Rows rows, so
// a weight is read once per kF32Rows rows, coalesced over the vocabulary, and the hidden values are wave-uniform
// (scalar loads).  Each logit is one chain of fused multiply-adds in ascending hidden index.
constexpr int kF32Rows = 8;
__global__ __launch_bounds__(256) void lmhead_f32_kernel(const float* __restrict__ H, int M, int d,
                                                         const float* __restrict__ W, float* __restrict__ Z, int V_t,
                                                         int64_t ldz) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  const int m0 = blockIdx.y * kF32Rows;
  if (n >= V_t) return;
  const int rows = min(kF32Rows, M - m0);
  float acc[kF32Rows];
#pragma unroll
  for (int i = 0; i < kF32Rows; ++i) acc[i] = 0.f;
  for (int kk = 0; kk < d; ++kk) {
    const float w = W[(int64_t)kk * V_t + n];
#pragma unroll
    for (int i = 0; i < kF32Rows; ++i)
      if (i < rows) acc[i] = fmaf(H[(int64_t)(m0 + i) * d + kk], w, acc[i]);
  }
#pragma unroll
  for (int i = 0; i < kF32Rows; ++i)
    if (i < rows) Z[(int64_t)(m0 + i) * ldz + n] = acc[i];
}

// Rows above which an M-block is split: up to 11 row tiles run as one block that streams every weight once (9 with
// either wavefront width, 10 and 11 only with 64 columns per wavefront, whose accumulators just fit).  Measured at 160 /
// 176 rows: 217 / 225 us per step as one block against 244 / 246 us as two.
constexpr int kSingleBlockRows = 176;

// Rough duration of an LM-head launch: the weights stream at 6 TB/s or the product runs at 1 PFLOP/s, whichever is longer.
double lmhead_launch_us(int M, int d, int Vp) { return std::max(2.0 * d * (double)Vp / 6.0e6, 2.0 * M * d * (double)Vp / 1.0e9); }

// How more than 176 rows run: as several M-blocks per column tile (their weight streams meet in one L2), of `tiles` row
// tiles each, by the kernel whose wavefronts own 32 columns or by the one whose wavefronts own 64 (`wide`).  That regime
// is bound by the L2 -> LDS traffic and by LDS reads, and the time of an M-block was measured to grow almost in
// proportion to its height (about 1.3 row tiles of fixed cost per block: 144, 256, 288 rows take 150, 251, 284 us at
// d = 4096, V_t = 128256), so the plan that minimises blocks x (1.3 + row tiles) is taken: mostly the height that pads
// least.  With 64 columns per wavefront a hidden fragment read from LDS feeds four MFMAs instead of two and the same
// cost comes out about 7 % lower, but the accumulators leave room for 11 row tiles at most.  Measured, us per step,
// best 32-column plan against the 64-column one: 176 rows 264 / 244, 320 rows 417 / 386, 352 rows 461 / 408,
// 425 rows 538 / 507, 432 rows 517 / 493, 576 rows 677 / 663, 1024 rows 1118 / 1076; 384 rows 468 / 519 (stays).
struct TallPlan { int tiles; bool wide; };
TallPlan tall_plan(int M) {
  TallPlan best{9, false};
  int best_cost = 100 * ceil_div(M, 144) * (13 + 10 * 9);
  for (int mt : {10, 12, 14, 16, 18}) {
    const int cost = 100 * ceil_div(M, 16 * mt) * (13 + 10 * mt);
    if (cost <= best_cost) { best_cost = cost; best = TallPlan{mt, false}; }
  }
  for (int mt : {9, 10, 11}) {
    const int cost = 93 * ceil_div(M, 16 * mt) * (13 + 10 * mt);
    if (cost < best_cost) { best_cost = cost; best = TallPlan{mt, true}; }
  }
  return best;
}

// Front workgroups of a launch that hosts the draft side with several M-blocks: one per four sequences (the lookups go
// four sequences at a time), a multiple of 8 (the XCD mapping of the multiplying workgroups holds), 8 to 64.  A
// workgroup that only reads, next to the multiplying ones, draws 5 to 10 GB/s however much it keeps in flight (measured:
// 8 of them need about 230 us for the 9.2 MB of 144 draft rows, 64 of them 35 us for 23 MB), so the compute-unit time
// the draft rows cost is given by their bytes; few front workgroups keep that time inside the slack of the last round
// of multiplying workgroups, many push some of those into a round of their own (160 rows, 501 multiplying workgroups in
// two rounds on 256 CUs: 64 front workgroups 257 us per step, separate launches 243).  0: one M-block, where the
// multiplying workgroups take the draft side themselves.
constexpr double kFrontBytesPerUs = 5e3;     // one front workgroup, next to the multiplying ones
int lmhead_bf16_front_workgroups(int M, int B) {
  if (M <= kSingleBlockRows) return 0;
  return std::min(64, std::max(8, ceil_div(ceil_div(B, 4), 8) * 8));
}
constexpr int kWideWaves = 8;      // wavefronts per workgroup of every wide kernel: each one of a front workgroup is a worker

template <int MT, int PF, int WPG, int KC, int NW, bool W_ONCE = false>
hipError_t launch_wide(const uint16_t* H, int M, int d, const uint16_t* Wp, int Kp, int Vp, float* Z, int V_t,
                       int64_t ldz, const uint16_t* zeros, const FusedStats& fs, const StepArgs* draft_side, int n_cu,
                       hipStream_t stream) {
  const int nks = Kp / 32, n_wtiles = Vp / kGemmColsPerWave;
  const int m_blocks = ceil_div(M, MT * 16);
  const int col_tiles = ceil_div(n_wtiles * 4, WPG * NW);
  StepArgs ds{};
  int n_front = 0, n_piece_jobs = 0, helpers_look_up = 0;
  const int padded_tiles = ceil_div(col_tiles, 8) * 8;
  if (draft_side && fs.part) {
    ds = *draft_side;
    const PiecePlan& plan = ds.plan;
    static_assert(WPG == kWideWaves, "the plan of the front workgroups counts on this many wavefronts each");
    n_front = lmhead_bf16_front_workgroups(M, ds.B);
    const int workers = n_front > 0 ? n_front * WPG : col_tiles * m_blocks;
    if (ds.K < 1 || plan.workers < 1 || plan.workers > workers || plan.base < 1 ||
        plan.base + (plan.more > 0) > kDraftPieces || plan.more < 0 || plan.more > ds.K ||
        (plan.workers < ds.K && (plan.base != 1 || plan.more != 0)))
      return hipErrorInvalidValue;
    n_piece_jobs = plan.jobs(ds.K);
    // the workgroups that pad the id space take the sequences' lookups if they finish well inside the launch: about
    // 60 us per four sequences (a chain of about six dependent loads next to the saturating weight streams) against
    // the time the weights take to stream or the product to be formed
    const int helpers = (padded_tiles - col_tiles) * m_blocks;
    if (n_front == 0 && helpers > 0 && ceil_div(ds.B, 4 * helpers) * 60.0 <= 0.5 * lmhead_launch_us(M, d, Vp))
      helpers_look_up = 1;
  }
  dim3 grid(n_front + padded_tiles * m_blocks), block(WPG * 64);
  const int vec_store = (ldz % 4 == 0) && (reinterpret_cast<uintptr_t>(Z) % 16 == 0);
  if (W_ONCE && m_blocks != 1) return hipErrorInvalidValue;
  hipLaunchKernelGGL((lmhead_bf16_wide_kernel<MT, PF, WPG, KC, NW, W_ONCE>), grid, block, 0, stream, H, M, d,
                     reinterpret_cast<const uint4*>(Wp), nks, n_wtiles, Z, V_t, ldz, vec_store, zeros, m_blocks, fs,
                     n_front, n_piece_jobs, helpers_look_up, ds);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_pack_w_bf16(const uint16_t* W, int d, int V_t, uint16_t* Wp, int Kp, int Vp, hipStream_t stream) {
  const int nks = Kp / 32;
  const int64_t n_units = (int64_t)(Vp / 64) * nks * 256;
  hipLaunchKernelGGL(pack_w_kernel, dim3((unsigned)((n_units + 255) / 256)), dim3(256), 0, stream, W, d, V_t,
                     reinterpret_cast<uint4*>(Wp), nks, n_units);
  return hipGetLastError();
}

// Columns per workgroup of the wide kernels.  A single M-block streams every weight once, bound by HBM, and what a
// workgroup does outside its main loop (first loads, row statistics, stores: about 12 us) is time its CU does not
// stream; with one workgroup per CU the launch runs in rounds, and a round costs its stream time whether or not all CUs
// take part.  512 columns per workgroup halve the rounds where that lets the launch fit into fewer, e.g. one round of
// 251 workgroups instead of two of 256-column ones on 256 CUs for a 128256-column head (measured: 175 against 196 us).
int lmhead_bf16_tile_cols(int M, int Vp, int n_cu) {
  if (M > kSingleBlockRows) return tall_plan(M).wide ? 512 : 256;
  if (M > 144) return 512;             // 10 or 11 row tiles in one block: only the 64-column wavefronts hold them
  if (M <= 16 || n_cu < 1) return 256;
  const int tiles256 = Vp / 256, tiles512 = ceil_div(Vp, 512);
  constexpr int kOutsideLoop = 40;                    // per round, in units of columns streamed
  const int cost256 = ceil_div(tiles256, n_cu) * (256 + kOutsideLoop);
  const int cost512 = ceil_div(tiles512, n_cu) * (512 + kOutsideLoop);
  return cost512 < cost256 ? 512 : 256;
}

int lmhead_bf16_fused_partials(int M, int Vp, int n_cu) {
  if (M <= 16) return 0;             // the skinny kernel does not fuse
  return ceil_div(Vp, lmhead_bf16_tile_cols(M, Vp, n_cu));
}

// Workgroups of launch_lmhead_bf16 that share the draft rows when the launch hosts the draft side: the multiplying
// ones with a single M-block (their number: one per tile of columns), the front ones otherwise.  0: the shape leaves no
// partials and hosts nothing.
int lmhead_bf16_draft_workers(int M, int Vp, int B, int K, int n_cu) {
  const int nfine = lmhead_bf16_fused_partials(M, Vp, n_cu);
  if (nfine == 0) return 0;
  return M > kSingleBlockRows ? lmhead_bf16_front_workgroups(M, B) * kWideWaves : nfine;
}

// Whether the LM-head launch should host the draft side (the draft rows' statistics, the drafted ids' lookups, and the
// target rows' softmax partials from its epilogue).  With a single M-block the launch is bound by the weight stream
// and a multiplying workgroup's piece of a draft row costs it about the 3 us that it would otherwise wait for its first
// loads: hosted when a workgroup gets at most two rows.  With several M-blocks front workgroups take the draft side:
// hosted when they are done within three quarters of the launch (their bytes at the rate above, 15 us per round of
// lookups).
bool lmhead_bf16_hosts_draft_side(int M, int d, int Vp, int B, int K, int V_d, int n_cu) {
  if (B < 1 || B > kFusedMaxB || K < 1) return false;
  const int workers = lmhead_bf16_draft_workers(M, Vp, B, K, n_cu);
  if (workers == 0) return false;
  if (M <= kSingleBlockRows) return K <= 2 * workers;
  const int n_front = workers / kWideWaves;
  const double front_us = 2.0 * K * (double)V_d / (n_front * kFrontBytesPerUs) + ceil_div(B, 4 * n_front) * 15.0;
  return front_us <= 0.75 * lmhead_launch_us(M, d, Vp);
}

hipError_t launch_lmhead_bf16(const uint16_t* H, int M, int d, const uint16_t* Wp, int Kp, int Vp, float* Z, int V_t,
                              int64_t ldz, const uint16_t* zeros, const FusedStats* fused, const StepArgs* draft_side,
                              int n_cu, hipStream_t stream) {
  if (M == 0) return hipSuccess;
  const int tiles = ceil_div(M, 16);
  FusedStats fs{};
  if (fused && fused->part) {
    if (fused->nfine != lmhead_bf16_fused_partials(M, Vp, n_cu) || fused->nfine == 0 || fused->B < 1 || fused->B > kFusedMaxB)
      return hipErrorInvalidValue;
    fs = *fused;
  }
  if (tiles <= 1) {
    const int nks = Kp / 32, n_wtiles = Vp / kGemmColsPerWave;
    hipLaunchKernelGGL((lmhead_bf16_skinny_kernel<4>), dim3(n_wtiles), dim3(512), 0, stream, H, M, d,
                       reinterpret_cast<const uint4*>(Wp), nks, Z, V_t, ldz);
    return hipGetLastError();
  }
  if (tiles == 10) return launch_wide<10, 2, 8, 64, 4, true>(H, M, d, Wp, Kp, Vp, Z, V_t, ldz, zeros, fs, draft_side, n_cu, stream);
  if (tiles == 11) return launch_wide<11, 2, 8, 64, 4, true>(H, M, d, Wp, Kp, Vp, Z, V_t, ldz, zeros, fs, draft_side, n_cu, stream);
  if (tiles <= 9 && lmhead_bf16_tile_cols(M, Vp, n_cu) == 512) {
    // wavefronts of 64 columns, hidden slices of 64 columns and a ring two (twice as long) steps deep: the same bytes
    // in flight per CU as the 256-column shape
    if (tiles <= 4) return launch_wide<4, 2, 8, 64, 4, true>(H, M, d, Wp, Kp, Vp, Z, V_t, ldz, zeros, fs, draft_side, n_cu, stream);
    if (tiles <= 6) return launch_wide<6, 2, 8, 64, 4, true>(H, M, d, Wp, Kp, Vp, Z, V_t, ldz, zeros, fs, draft_side, n_cu, stream);
    return launch_wide<9, 2, 8, 64, 4, true>(H, M, d, Wp, Kp, Vp, Z, V_t, ldz, zeros, fs, draft_side, n_cu, stream);
  }
  if (tiles <= 2) return launch_wide<2, 4, 8, 128, 2, true>(H, M, d, Wp, Kp, Vp, Z, V_t, ldz, zeros, fs, draft_side, n_cu, stream);
  if (tiles <= 4) return launch_wide<4, 4, 8, 128, 2, true>(H, M, d, Wp, Kp, Vp, Z, V_t, ldz, zeros, fs, draft_side, n_cu, stream);
  if (tiles <= 6) return launch_wide<6, 4, 8, 128, 2, true>(H, M, d, Wp, Kp, Vp, Z, V_t, ldz, zeros, fs, draft_side, n_cu, stream);
  if (tiles <= 9) return launch_wide<9, 4, 8, 128, 2, true>(H, M, d, Wp, Kp, Vp, Z, V_t, ldz, zeros, fs, draft_side, n_cu, stream);
  // More than 176 rows run as several M-blocks per column tile (tall_plan).  Heights above 144 rows use hidden
  // slices of 64 columns and a weight ring two steps deep to fit in LDS.
  const TallPlan plan = tall_plan(M);
  if (plan.wide) {
    switch (plan.tiles) {
      case 10: return launch_wide<10, 2, 8, 64, 4>(H, M, d, Wp, Kp, Vp, Z, V_t, ldz, zeros, fs, draft_side, n_cu, stream);
      case 11: return launch_wide<11, 2, 8, 64, 4>(H, M, d, Wp, Kp, Vp, Z, V_t, ldz, zeros, fs, draft_side, n_cu, stream);
      default: return launch_wide<9, 2, 8, 64, 4>(H, M, d, Wp, Kp, Vp, Z, V_t, ldz, zeros, fs, draft_side, n_cu, stream);
    }
  }
  const int best_mt = plan.tiles;
  switch (best_mt) {
    case 10: return launch_wide<10, 2, 8, 64, 2>(H, M, d, Wp, Kp, Vp, Z, V_t, ldz, zeros, fs, draft_side, n_cu, stream);
    case 12: return launch_wide<12, 2, 8, 64, 2>(H, M, d, Wp, Kp, Vp, Z, V_t, ldz, zeros, fs, draft_side, n_cu, stream);
    case 14: return launch_wide<14, 2, 8, 64, 2>(H, M, d, Wp, Kp, Vp, Z, V_t, ldz, zeros, fs, draft_side, n_cu, stream);
    case 16: return launch_wide<16, 2, 8, 64, 2>(H, M, d, Wp, Kp, Vp, Z, V_t, ldz, zeros, fs, draft_side, n_cu, stream);
    case 18: return launch_wide<18, 2, 8, 64, 2>(H, M, d, Wp, Kp, Vp, Z, V_t, ldz, zeros, fs, draft_side, n_cu, stream);
    default: return launch_wide<9, 4, 8, 128, 2>(H, M, d, Wp, Kp, Vp, Z, V_t, ldz, zeros, fs, draft_side, n_cu, stream);
  }
}

hipError_t launch_lmhead_f32(const float* H, int M, int d, const float* W, float* Z, int V_t, int64_t ldz,
                             hipStream_t stream) {
  if (M == 0) return hipSuccess;
  hipLaunchKernelGGL(lmhead_f32_kernel, dim3(ceil_div(V_t, 256), ceil_div(M, kF32Rows)), dim3(256), 0, stream, H, M, d, W, Z, V_t, ldz);
  return hipGetLastError();
}

}  // namespace otv
