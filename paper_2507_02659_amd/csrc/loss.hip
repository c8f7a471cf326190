// Forward values of the hybrid cross-vocabulary distillation loss (Section "Cross-vocabulary Distillation", the
// loss equation): reverse KL D_KL(q' || p) on drafted tokens that translate through the direct map, and on the
// sub-tokens of n-gram tokens either the negative log-likelihood -log q(d_i) or the approximate KL with Eq. 2's two
// overrides, weighted by lambda (a constant, or the verified target probability p(t_i)).
//
// The call follows a verification step on the same inputs and reuses what that step left behind: the translation
// (mapped ids and spans in the step's output buffers), the logits and the softmax statistics of every target and
// draft row in the workspace.  With those, ln p(v) = (z_v - max)/T - ln S costs one fused multiply-add per id and
// q'(v) one exponential; no probability row is materialised unless the caller asks for the q' rows.
//
//   loss_prepare_kernel   one workgroup per sequence, one lane per mapped token: kind, NLL, lambda and the
//                         constants of p and q' at that position (LossRow).
//   loss_kl_tiles_kernel  grid = (tiles of 1024 target ids) x (rows): sum over the tile of q' (ln q' - ln p) in
//                         binary64 for the rows that carry a KL term (HBM bound: one logit row, the inverse map and
//                         a gather of the draft row per position); optionally writes q' (Eq. 2) as fp32.
//   loss_row_kernel       one workgroup per row: the row's tile sums in a fixed order.
//   loss_total_kernel     one workgroup: sums over rows in a fixed order and the mean over the drafted tokens.
#include "device_math.h"
#include "otv_host.h"

namespace otv {
namespace {

constexpr int kThreads = 256;
constexpr int kPer = kResidTile / kThreads;   // 4 ids per thread
static_assert(kPer == 4, "the fixed summation trees below are written for 4 ids per thread");

struct LossRow {
  int32_t need_tiles;    // the tile kernel visits this row (it carries a KL term, or q' rows are exported)
  int32_t need_kl;
  int32_t drow;          // draft row of the token's first sub-token
  int32_t t_ng, t_pre;   // Eq. 2 overrides: target id of the n-gram / direct image of its first sub-token, or -1
  int32_t pad;
  double pi, q_pre, ln_pi, ln_q_pre;
  // ln p(v) = (z_v - mx) * invT - lnS at the token's target row; ln q(d) = (zq_d - mxq) * invTd - lnSq at draft row drow
  double mx, invT, lnS, mxq, invTd, lnSq;
};

static_assert(sizeof(LossRow) <= kLossRowBytes, "the context allocates kLossRowBytes per row");

struct LossArgs {
  int32_t B, M, V_t, V_d, dtype, ntiles;
  const int32_t* row_off;
  const float* temperature;
  const float* draft_temperature;
  const void* draft_logits;
  const int32_t* draft_ids;
  const int32_t* dmap;
  const int32_t* tmap;
  const float* Z;
  int64_t ldz;
  const float* row_max; const double* row_sum;
  const float* drow_max; const double* drow_sum;
  // translation and outcome of the verification step
  const int32_t* n_mapped; const int32_t* n_accept; const int32_t* mapped_ids; const int32_t* span_start;
  const int32_t* span_len; const float* p_tok;
  // options
  float lambda; int32_t lambda_mode, ngram_term, accepted_only;
  // workspace
  LossRow* rows;         // [M]
  double* tile_kl;       // [M, ntiles]
  // outputs
  ot_loss_out out;
};

__device__ inline float draft_logit(const LossArgs& a, int drow, int dv) {
  const int64_t at = (int64_t)drow * a.V_d + dv;
  return a.dtype == OT_BF16 ? bf16_to_f32(static_cast<const uint16_t*>(a.draft_logits)[at])
                            : static_cast<const float*>(a.draft_logits)[at];
}

__global__ __launch_bounds__(64) void loss_prepare_kernel(LossArgs a) {
  const int b = blockIdx.x, j = threadIdx.x;
  const int r0 = a.row_off[b], k = a.row_off[b + 1] - r0 - 1, q0 = r0 - b;
  if (j > k) return;
  const int row = r0 + j;
  const float T = a.temperature[b];
  const float Td = a.draft_temperature ? a.draft_temperature[b] : T;
  LossRow R;
  R.need_tiles = 0; R.need_kl = 0; R.drow = 0; R.t_ng = -1; R.t_pre = -1; R.pad = 0;
  R.pi = 0.0; R.q_pre = 0.0; R.ln_pi = 0.0; R.ln_q_pre = 0.0;
  R.mx = 0.0; R.invT = 0.0; R.lnS = 0.0; R.mxq = 0.0; R.invTd = 0.0; R.lnSq = 0.0;
  int kind = 0;
  double nll = 0.0, weight = 0.0;
  if (j < a.n_mapped[b] && T > 0.f && Td > 0.f) {
    const int s = a.span_start[row], L = a.span_len[row], t = a.mapped_ids[row];
    R.drow = q0 + s;
    R.mx = (double)a.row_max[row]; R.invT = 1.0 / (double)T; R.lnS = log(a.row_sum[row]);
    R.mxq = (double)a.drow_max[R.drow]; R.invTd = 1.0 / (double)Td; R.lnSq = log(a.drow_sum[R.drow]);
    if (L == 1) {
      kind = 1;
      R.need_kl = 1;
    } else if (!a.accepted_only || j < a.n_accept[b]) {
      kind = 2;
      double lq_first = 0.0, lq_sum = 0.0;
      for (int l = 0; l < L; ++l) {
        const int dr = q0 + s + l;
        const double lq = ((double)draft_logit(a, dr, a.draft_ids[dr]) - (double)a.drow_max[dr]) * R.invTd - log(a.drow_sum[dr]);
        if (l == 0) lq_first = lq;
        lq_sum += lq;
      }
      nll = -lq_sum;
      weight = a.lambda_mode == OT_LAMBDA_TARGET_PROB ? (double)a.p_tok[row] : (double)a.lambda;
      // Eq. 2's overrides for this n-gram
      R.t_ng = t;
      R.pi = exp(lq_sum); R.ln_pi = lq_sum;
      const int d1 = a.draft_ids[q0 + s];
      R.t_pre = a.dmap[d1];
      R.q_pre = exp(lq_first) - R.pi;
      R.ln_q_pre = R.q_pre > 0.0 ? log(R.q_pre) : 0.0;
      R.need_kl = a.ngram_term == OT_NGRAM_TERM_APPROX_KL;
    }
    R.need_tiles = (kind != 0) && (R.need_kl || a.out.qprime != nullptr);
  }
  a.rows[row] = R;
  a.out.kind[row] = kind;
  a.out.nll[row] = nll;
  a.out.weight[row] = weight;
}

__global__ __launch_bounds__(kThreads) void loss_kl_tiles_kernel(LossArgs a) {
  const int row = blockIdx.y, tile = blockIdx.x, tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int first = tile * kResidTile + tid;
  const LossRow R = a.rows[row];
  if (!R.need_tiles) {                                   // most rows of a batch: checked before anything is fetched
    if (a.out.qprime) {                                  // rows without a token export zeros
#pragma unroll
      for (int e = 0; e < kPer; ++e) {
        const int v = first + e * kThreads;
        if (v < a.V_t) a.out.qprime[(int64_t)row * a.V_t + v] = 0.f;
      }
    }
    return;
  }
  const float* z = a.Z + (int64_t)row * a.ldz;
  int dv[kPer];
  float zv[kPer], xq[kPer];
#pragma unroll
  for (int e = 0; e < kPer; ++e) {
    const int v = first + e * kThreads;
    dv[e] = v < a.V_t ? a.tmap[v] : -1;
    zv[e] = v < a.V_t ? z[v] : 0.f;
  }
#pragma unroll
  for (int e = 0; e < kPer; ++e) xq[e] = dv[e] >= 0 ? draft_logit(a, R.drow, dv[e]) : 0.f;
  double term[kPer];
#pragma unroll
  for (int e = 0; e < kPer; ++e) {
    const int v = first + e * kThreads;
    double q = 0.0, lq = 0.0;
    if (dv[e] >= 0) {
      lq = ((double)xq[e] - R.mxq) * R.invTd - R.lnSq;
      q = exp_neg_fast(lq);
    }
    if (v == R.t_pre) { q = R.q_pre; lq = R.ln_q_pre; }
    if (v == R.t_ng) { q = R.pi; lq = R.ln_pi; }         // the n-gram case of Eq. 2 wins when both name the same id
    const double lp = ((double)zv[e] - R.mx) * R.invT - R.lnS;
    term[e] = (v < a.V_t && q > 0.0) ? q * (lq - lp) : 0.0;
    if (a.out.qprime && v < a.V_t) a.out.qprime[(int64_t)row * a.V_t + v] = (float)q;
  }
  if (!R.need_kl) return;
  double sum = (term[0] + term[1]) + (term[2] + term[3]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
  __shared__ double s_w[kThreads / 64];
  if (lane == 0) s_w[wave] = sum;
  __syncthreads();
  if (tid == 0) a.tile_kl[(int64_t)row * a.ntiles + tile] = (s_w[0] + s_w[1]) + (s_w[2] + s_w[3]);
}

// Sum of n doubles x[i * stride] by one workgroup in a fixed order; the result is valid in thread 0.
__device__ inline double block_sum(const double* x, int n, double* s_w) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  double sum = 0.0;
  for (int i = tid; i < n; i += kThreads) sum += x[i];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
  if (lane == 0) s_w[wave] = sum;
  __syncthreads();
  return (s_w[0] + s_w[1]) + (s_w[2] + s_w[3]);
}

__global__ __launch_bounds__(kThreads) void loss_row_kernel(LossArgs a) {
  const int row = blockIdx.x;
  __shared__ double s_w[kThreads / 64];
  const bool need = a.rows[row].need_kl != 0;
  const double total = need ? block_sum(a.tile_kl + (int64_t)row * a.ntiles, a.ntiles, s_w) : 0.0;
  if (threadIdx.x == 0) a.out.kl[row] = total;
}

__global__ __launch_bounds__(kThreads) void loss_total_kernel(LossArgs a) {
  __shared__ double s_term[4][kThreads / 64];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  double dm = 0.0, ng = 0.0, n_dm = 0.0, n_ng = 0.0;
  for (int row = tid; row < a.M; row += kThreads) {
    const int kind = a.out.kind[row];
    if (kind == 1) {
      dm += a.out.kl[row];
      n_dm += 1.0;
    } else if (kind == 2) {
      const double term = a.ngram_term == OT_NGRAM_TERM_APPROX_KL ? a.out.kl[row] : a.out.nll[row];
      ng += a.out.weight[row] * term;
      n_ng += (double)a.span_len[row];
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    dm += __shfl_xor(dm, off); ng += __shfl_xor(ng, off); n_dm += __shfl_xor(n_dm, off); n_ng += __shfl_xor(n_ng, off);
  }
  if (lane == 0) { s_term[0][wave] = dm; s_term[1][wave] = ng; s_term[2][wave] = n_dm; s_term[3][wave] = n_ng; }
  __syncthreads();
  if (tid == 0) {
    double t[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) t[i] = (s_term[i][0] + s_term[i][1]) + (s_term[i][2] + s_term[i][3]);
    a.out.totals[0] = t[0];
    a.out.totals[1] = t[1];
    a.out.totals[2] = t[2];
    a.out.totals[3] = t[3];
    a.out.totals[4] = (t[0] + t[1]) / fmax(1.0, t[2] + t[3]);
  }
}

}  // namespace
}  // namespace otv

using namespace otv;

#pragma GCC visibility push(default)
extern "C" {

int ot_distill_loss(ot_ctx* ctx, const ot_step_in* in, const ot_step_out* step, const float* target_logits,
                    const ot_loss_config* cfg, ot_loss_out* out) {
  if (!ctx || !in || !step || !cfg || !out) return ot_fail(OT_ERR_NULL, "ot_distill_loss: ctx, in, step_out, cfg and out must not be NULL");
  if (cfg->lambda_mode != OT_LAMBDA_FIXED && cfg->lambda_mode != OT_LAMBDA_TARGET_PROB)
    return ot_fail(OT_ERR_SHAPE, "ot_distill_loss: unknown lambda_mode %d", cfg->lambda_mode);
  if (cfg->ngram_term != OT_NGRAM_TERM_NLL && cfg->ngram_term != OT_NGRAM_TERM_APPROX_KL)
    return ot_fail(OT_ERR_SHAPE, "ot_distill_loss: unknown ngram_term %d", cfg->ngram_term);
  if (in->B < 0 || in->B > ctx->max_batch) return ot_fail(OT_ERR_SHAPE, "ot_distill_loss: B = %d exceeds max_batch = %d", in->B, ctx->max_batch);
  if (!out->kind || !out->kl || !out->nll || !out->weight || !out->totals)
    return ot_fail(OT_ERR_NULL, "ot_distill_loss: kind, kl, nll, weight and totals are required");
  if (in->B > 0) {
    if (!in->row_off || !in->row_off_host || !in->temperature)
      return ot_fail(OT_ERR_NULL, "ot_distill_loss: row_off, row_off_host and temperature must not be NULL");
    if (!step->n_mapped || !step->n_accept || !step->mapped_ids || !step->span_start || !step->span_len || !step->p_tok)
      return ot_fail(OT_ERR_NULL, "ot_distill_loss: the step's n_mapped, n_accept, mapped_ids, span_start, span_len and p_tok are required");
    if (in->row_off_host[0] != 0) return ot_fail(OT_ERR_SHAPE, "ot_distill_loss: row_off[0] must be 0");
    for (int b = 0; b < in->B; ++b) {
      const int64_t rows = (int64_t)in->row_off_host[b + 1] - in->row_off_host[b];
      if (rows < 1 || rows - 1 > ctx->max_k) return ot_fail(OT_ERR_SHAPE, "ot_distill_loss: sequence %d owns %lld rows", b, (long long)rows);
    }
  }
  const int M = in->B > 0 ? in->row_off_host[in->B] : 0;
  if (M - in->B > 0 && (!in->draft_logits || !in->draft_ids)) return ot_fail(OT_ERR_NULL, "ot_distill_loss: draft_logits and draft_ids must not be NULL");

  LossArgs a{};
  a.B = in->B; a.M = M; a.V_t = ctx->V_t; a.V_d = ctx->V_d; a.dtype = ctx->dtype; a.ntiles = ctx->ntiles;
  a.row_off = in->row_off; a.temperature = in->temperature; a.draft_temperature = in->draft_temperature;
  a.draft_logits = in->draft_logits; a.draft_ids = in->draft_ids; a.dmap = ctx->dmap; a.tmap = ctx->tmap;
  a.Z = target_logits ? target_logits : ctx->Z; a.ldz = ctx->V_t;
  a.row_max = ctx->row_max; a.row_sum = ctx->row_sum; a.drow_max = ctx->drow_max; a.drow_sum = ctx->drow_sum;
  a.n_mapped = step->n_mapped; a.n_accept = step->n_accept; a.mapped_ids = step->mapped_ids;
  a.span_start = step->span_start; a.span_len = step->span_len; a.p_tok = step->p_tok;
  a.lambda = cfg->lambda; a.lambda_mode = cfg->lambda_mode; a.ngram_term = cfg->ngram_term; a.accepted_only = cfg->accepted_only != 0;
  a.rows = static_cast<LossRow*>(ctx->loss_rows); a.tile_kl = ctx->loss_tiles;
  a.out = *out;

  hipStream_t st = ctx->stream;
  if (M > 0) {
    hipLaunchKernelGGL(loss_prepare_kernel, dim3(in->B), dim3(64), 0, st, a);
    hipLaunchKernelGGL(loss_kl_tiles_kernel, dim3(a.ntiles, M), dim3(kThreads), 0, st, a);
    hipLaunchKernelGGL(loss_row_kernel, dim3(M), dim3(kThreads), 0, st, a);
  }
  hipLaunchKernelGGL(loss_total_kernel, dim3(1), dim3(kThreads), 0, st, a);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return ot_fail_hip(e, "ot_distill_loss: launch");
  return OT_OK;
}

}  // extern "C"
#pragma GCC visibility pop
