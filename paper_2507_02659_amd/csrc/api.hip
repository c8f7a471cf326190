// Host side of libotverify: argument validation, context / workspace / n-gram table management, and the launch
// order of one verification step.  Exports the C ABI declared in otverify.h; nothing here does arithmetic of
// the method itself.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "otv_host.h"

using namespace otv;

namespace {

thread_local char g_err[512] = "";
constexpr int kProfileCapacity = 1024;   // steps whose events can be pending between two profile reads
constexpr int kEventsPerStep = OT_N_STAGES + 1;

}  // namespace

int ot_fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int ot_fail_hip(hipError_t e, const char* what) { return ot_fail(OT_ERR_HIP, "%s: %s", what, hipGetErrorString(e)); }

#define fail ot_fail
#define fail_hip ot_fail_hip

namespace {

template <typename T>
bool dev_alloc(ot_ctx* c, T** p, size_t count) {
  void* q = nullptr;
  if (hipMalloc(&q, (count ? count : 1) * sizeof(T)) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  c->allocs.push_back(q);
  *p = static_cast<T*>(q);
  return true;
}

void free_ctx(ot_ctx* c) {
  for (void* p : c->allocs) (void)hipFree(p);
  for (hipEvent_t e : c->events) (void)hipEventDestroy(e);
  delete c;
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

const char* ot_last_error(void) { return g_err; }
const char* ot_version(void) { return "otverify 0.1 (gfx950)"; }

int ot_verify_init(const ot_verify_config* cfg, ot_ctx** out) {
  if (out) *out = nullptr;
  if (!cfg || !out) return fail(OT_ERR_NULL, "ot_verify_init: cfg and out must not be NULL");
  if (!cfg->W || !cfg->direct_map) return fail(OT_ERR_NULL, "ot_verify_init: W and direct_map must not be NULL");
  if (cfg->dtype != OT_BF16 && cfg->dtype != OT_F32) return fail(OT_ERR_DTYPE, "ot_verify_init: unknown dtype %d", cfg->dtype);
  if (cfg->d <= 0 || cfg->V_t <= 0 || cfg->V_d <= 0) return fail(OT_ERR_SHAPE, "ot_verify_init: d, V_t, V_d must be positive");
  if (cfg->dtype == OT_BF16 && cfg->d % 8 != 0) return fail(OT_ERR_SHAPE, "ot_verify_init: bf16 needs d %% 8 == 0 (d = %d)", cfg->d);
  if (cfg->max_batch < 1 || cfg->max_k < 0 || cfg->max_k > OT_MAX_K)
    return fail(OT_ERR_SHAPE, "ot_verify_init: need max_batch >= 1 and 0 <= max_k <= %d", OT_MAX_K);
  if (cfg->max_ngram_len < 2 || cfg->max_ngram_len > OT_MAX_NGRAM_LEN)
    return fail(OT_ERR_SHAPE, "ot_verify_init: max_ngram_len must be in 2..%d", OT_MAX_NGRAM_LEN);
  if (cfg->draft_side < OT_DRAFT_SIDE_AUTO || cfg->draft_side > OT_DRAFT_SIDE_SEPARATE)
    return fail(OT_ERR_SHAPE, "ot_verify_init: draft_side must be one of OT_DRAFT_SIDE_*");
  if ((int64_t)cfg->max_batch * (cfg->max_k + 1) > (1 << 20)) return fail(OT_ERR_SHAPE, "ot_verify_init: more than 2^20 rows");

  // direct map: in range and one-to-one on its mapped part
  std::vector<int32_t> tmap_h;
  try {
    tmap_h.assign((size_t)cfg->V_t, -1);
  } catch (const std::bad_alloc&) {
    return fail(OT_ERR_NOMEM, "ot_verify_init: host allocation failed");
  }
  for (int32_t dd = 0; dd < cfg->V_d; ++dd) {
    const int32_t t = cfg->direct_map[dd];
    if (t == -1) continue;
    if (t < 0 || t >= cfg->V_t) return fail(OT_ERR_MAP, "ot_verify_init: direct_map[%d] = %d is outside [0, V_t)", dd, t);
    if (tmap_h[t] != -1) return fail(OT_ERR_MAP, "ot_verify_init: draft ids %d and %d both map to target id %d", tmap_h[t], dd, t);
    tmap_h[t] = dd;
  }

  ot_ctx* c = new (std::nothrow) ot_ctx();
  if (!c) return fail(OT_ERR_NOMEM, "ot_verify_init: host allocation failed");
  c->d = cfg->d; c->V_t = cfg->V_t; c->V_d = cfg->V_d; c->max_batch = cfg->max_batch; c->max_k = cfg->max_k;
  c->dtype = cfg->dtype; c->max_ngram_len = cfg->max_ngram_len; c->draft_side = cfg->draft_side;
  c->stream = static_cast<hipStream_t>(cfg->stream);
  c->max_rows = cfg->max_batch * (cfg->max_k + 1);
  c->max_K = cfg->max_batch * cfg->max_k;
  c->Kp = ceil_div(cfg->d, kGemmKPad) * kGemmKPad;
  c->Vp = ceil_div(cfg->V_t, 256) * 256;
  c->ncht = ceil_div(cfg->V_t, kStatChunk);
  c->nchd = ceil_div(cfg->V_d, kStatChunk);
  c->ntiles = ceil_div(cfg->V_t, kResidTile);
  hipError_t e = hipGetDevice(&c->device);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&c->n_cu, hipDeviceAttributeMultiprocessorCount, c->device);
  if (e != hipSuccess) { free_ctx(c); return fail_hip(e, "hipGetDevice"); }
  if (ot_static_scratch_prepare() != OT_OK) { free_ctx(c); return OT_ERR_HIP; }

  const size_t R = (size_t)c->max_rows, KQ = (size_t)c->max_K, Bm = (size_t)c->max_batch;
  bool ok = true;
  if (c->dtype == OT_BF16) ok = ok && dev_alloc(c, &c->Wp, (size_t)(c->Vp / 64) * (size_t)packed_tile_units(c->Kp / 32) * 8) && dev_alloc(c, &c->zeros, 32);
  else ok = ok && dev_alloc(c, &c->Wf, (size_t)c->d * c->V_t);
  ok = ok && dev_alloc(c, &c->dmap, (size_t)c->V_d) && dev_alloc(c, &c->tmap, (size_t)c->V_t);
  ok = ok && dev_alloc(c, &c->Z, R * (size_t)c->V_t);
  ok = ok && dev_alloc(c, &c->tpart_max, R * c->ncht) && dev_alloc(c, &c->tpart_sum, R * c->ncht) && dev_alloc(c, &c->tpart_arg, R * c->ncht);
  if (c->dtype == OT_BF16) {
    const size_t nf = (size_t)(c->Vp / 256);
    ok = ok && dev_alloc(c, &c->fpart, R * nf);
  }
  ok = ok && dev_alloc(c, &c->dpart_max, KQ * c->nchd) && dev_alloc(c, &c->dpart_sum, KQ * c->nchd) && dev_alloc(c, &c->dpart_arg, KQ * c->nchd);
  ok = ok && dev_alloc(c, &c->row_max, R) && dev_alloc(c, &c->row_sum, R) && dev_alloc(c, &c->row_arg, R);
  ok = ok && dev_alloc(c, &c->drow_max, KQ) && dev_alloc(c, &c->drow_sum, KQ) && dev_alloc(c, &c->drow_arg, KQ);
  ok = ok && dev_alloc(c, &c->fin, Bm) && dev_alloc(c, &c->probe, Bm) &&
       dev_alloc(c, &c->dpiece, KQ * otv::kDraftPieces);
  {
    char* rows = nullptr;
    ok = ok && dev_alloc(c, &rows, R * kLossRowBytes) && dev_alloc(c, &c->loss_tiles, R * c->ntiles);
    c->loss_rows = rows;
  }
  ok = ok && dev_alloc(c, &c->adapt_part, 2 * Bm);
  ok = ok && dev_alloc(c, &c->tile_r, Bm * c->ntiles) && dev_alloc(c, &c->tile_p, Bm * c->ntiles);
  ok = ok && dev_alloc(c, &c->resid_count, Bm);
  if (!ok) { free_ctx(c); return fail(OT_ERR_NOMEM, "ot_verify_init: device allocation failed"); }

  if (c->zeros) e = hipMemsetAsync(c->zeros, 0, 64, c->stream);
  if (e == hipSuccess) e = hipMemsetAsync(c->resid_count, 0, sizeof(int32_t) * Bm, c->stream);
  if (e == hipSuccess) e = hipMemcpyAsync(c->dmap, cfg->direct_map, sizeof(int32_t) * c->V_d, hipMemcpyHostToDevice, c->stream);
  if (e == hipSuccess) e = hipMemcpyAsync(c->tmap, tmap_h.data(), sizeof(int32_t) * c->V_t, hipMemcpyHostToDevice, c->stream);
  if (e == hipSuccess) {
    if (c->dtype == OT_BF16)
      e = launch_pack_w_bf16(static_cast<const uint16_t*>(cfg->W), c->d, c->V_t, c->Wp, c->Kp, c->Vp, c->stream);
    else
      e = hipMemcpyAsync(c->Wf, cfg->W, sizeof(float) * (size_t)c->d * c->V_t, hipMemcpyDeviceToDevice, c->stream);
  }
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);    // tmap_h and the caller's W are released here
  if (e != hipSuccess) { free_ctx(c); return fail_hip(e, "ot_verify_init"); }
  *out = c;
  return OT_OK;
}

void ot_verify_destroy(ot_ctx* ctx) {
  if (!ctx) return;
  (void)hipStreamSynchronize(ctx->stream);
  free_ctx(ctx);
}

static int step_impl(ot_ctx* ctx, ot_ngram_cache* cache, const ot_step_in* in, const float* ext_logits,
                     bool from_logits, ot_step_out* o) {
  if (!ctx || !in || !o) return fail(OT_ERR_NULL, "ot_verify_step: ctx, in and out must not be NULL");
  if (in->B < 0 || in->B > ctx->max_batch) return fail(OT_ERR_SHAPE, "ot_verify_step: B = %d exceeds max_batch = %d", in->B, ctx->max_batch);
  if (cache && cache->owner != ctx) return fail(OT_ERR_CTX_MISMATCH, "ot_verify_step: the n-gram cache was built for another context");
  if (in->B == 0) return OT_OK;
  if (!in->row_off || !in->row_off_host || !in->temperature || !in->seq_id)
    return fail(OT_ERR_NULL, "ot_verify_step: row_off, row_off_host, temperature and seq_id must not be NULL");
  {
    const char* what = "";
    const int bad = check_row_offsets(in->B, in->row_off_host, ctx->max_k, &what);
    if (bad) return fail(OT_ERR_SHAPE, "ot_verify_step: sequence %d: %s (max_k = %d)", bad - 1, what, ctx->max_k);
  }
  const int M = in->row_off_host[in->B], K = M - in->B;
  if (from_logits ? !ext_logits : !in->hidden) return fail(OT_ERR_NULL, "ot_verify_step: %s must not be NULL", from_logits ? "target_logits" : "hidden");
  if (K > 0 && (!in->draft_logits || !in->draft_ids)) return fail(OT_ERR_NULL, "ot_verify_step: draft_logits and draft_ids must not be NULL");
  if (!o->n_mapped || !o->n_accept || !o->n_accept_draft || !o->n_emit || !o->hits_proposed || !o->hits_accepted ||
      !o->flags || !o->out_tokens || !o->mapped_ids || !o->span_start || !o->span_len || !o->p_tok || !o->q_tok || !o->ratio)
    return fail(OT_ERR_NULL, "ot_verify_step: every output buffer is required");

  StepArgs a;
  std::memset(&a, 0, sizeof(a));
  a.B = in->B; a.M = M; a.K = K; a.d = ctx->d; a.V_t = ctx->V_t; a.V_d = ctx->V_d; a.dtype = ctx->dtype;
  a.max_ngram_len = ctx->max_ngram_len; a.step = in->step; a.seed = in->seed;
  a.row_off = in->row_off; a.hidden = in->hidden; a.draft_logits = in->draft_logits; a.draft_ids = in->draft_ids;
  a.temperature = in->temperature; a.draft_temperature = in->draft_temperature; a.seq_id = in->seq_id;
  a.dmap = ctx->dmap; a.tmap = ctx->tmap;
  if (cache) cache->tab.tick();             // one tick of the cache's logical time per step that is given the cache
  if (cache && cache->tab.size() > 0) {
    a.cache.slots = cache->d_slots; a.cache.mask = cache->tab.mask(); a.cache.stride = cache->tab.stride();
    a.cache.max_len = cache->tab.max_len(); a.cache.uses = cache->d_uses; a.cache.last_used = cache->d_last;
    a.cache.clock = cache->tab.clock(); a.cache.log_count = cache->d_log_count; a.cache.log = cache->d_log;
  }
  a.Z = from_logits ? ext_logits : ctx->Z;
  a.ldz = ctx->V_t;
  a.ncht = ctx->ncht; a.nchd = ctx->nchd; a.ntiles = ctx->ntiles;
  a.tpart_max = ctx->tpart_max; a.tpart_sum = ctx->tpart_sum; a.tpart_arg = ctx->tpart_arg;
  a.dpart_max = ctx->dpart_max; a.dpart_sum = ctx->dpart_sum; a.dpart_arg = ctx->dpart_arg;
  a.row_max = ctx->row_max; a.row_sum = ctx->row_sum; a.row_arg = ctx->row_arg;
  a.drow_max = ctx->drow_max; a.drow_sum = ctx->drow_sum; a.drow_arg = ctx->drow_arg;
  a.fin = ctx->fin;
  a.probe = ctx->probe;
  a.dpiece = ctx->dpiece;
  a.tile_r = ctx->tile_r; a.tile_p = ctx->tile_p; a.resid_count = ctx->resid_count;
  a.out = *o;

  hipStream_t st = ctx->stream;
  hipEvent_t* ev = nullptr;
  if (ctx->profiling && ctx->pending < kProfileCapacity) {
    const size_t need = (size_t)(ctx->pending + 1) * kEventsPerStep;
    while (ctx->events.size() < need) {
      hipEvent_t x;
      hipError_t e = hipEventCreate(&x);
      if (e != hipSuccess) return fail_hip(e, "hipEventCreate");
      ctx->events.push_back(x);
    }
    ev = &ctx->events[(size_t)ctx->pending * kEventsPerStep];
  }
  hipError_t e = hipSuccess;
#define OT_MARK(i) do { if (ev && e == hipSuccess) e = hipEventRecord(ev[i], st); } while (0)
  OT_MARK(0);
  if (e == hipSuccess && !from_logits) {
    if (ctx->dtype == OT_BF16) {
      // Where its kernel supports it, the LM-head launch leaves per-tile softmax partials of the target rows (no second
      // pass over the logits) and hosts the draft side of the step (the draft rows' statistics in pieces, the drafted
      // ids' lookups): what follows it is then one launch that merges both, walks the windows, tests and draws.
      const bool supported = lmhead_bf16_draft_workers(M, ctx->Vp, in->B, K, ctx->n_cu) > 0 && K >= 1 && in->B <= kFusedMaxB;
      const bool host_it = supported && (ctx->draft_side == OT_DRAFT_SIDE_IN_LM_HEAD ||
                                         (ctx->draft_side == OT_DRAFT_SIDE_AUTO &&
                                          lmhead_bf16_hosts_draft_side(M, ctx->d, ctx->Vp, in->B, K, ctx->V_d, ctx->n_cu)));
      const int nfine = host_it ? lmhead_bf16_fused_partials(M, ctx->Vp, ctx->n_cu) : 0;
      if (nfine > 0) {
        a.fused.row_off = in->row_off; a.fused.temperature = in->temperature; a.fused.B = in->B; a.fused.nfine = nfine;
        a.fused.part = ctx->fpart;
        a.hosted = 1;
        a.plan = make_piece_plan(lmhead_bf16_draft_workers(M, ctx->Vp, in->B, K, ctx->n_cu), K);
      }
      e = launch_lmhead_bf16(static_cast<const uint16_t*>(in->hidden), M, ctx->d, ctx->Wp, ctx->Kp, ctx->Vp, ctx->Z,
                             ctx->V_t, a.ldz, ctx->zeros, &a.fused, a.hosted ? &a : nullptr, ctx->n_cu, st);
    }
    else
      e = launch_lmhead_f32(static_cast<const float*>(in->hidden), M, ctx->d, ctx->Wf, ctx->Z, ctx->V_t, a.ldz, st);
  }
  OT_MARK(1);
  // Without the LM head's help the statistics get a launch of their own; with at most kFusedMaxB sequences it also does
  // the lookups, and one launch follows it as above; with more, the translation and the test get a launch of their own.
  if (!a.hosted && in->B <= kFusedMaxB) a.chunked = 1;
  if (e == hipSuccess && !a.hosted) e = launch_softmax_stats(a, st);
  OT_MARK(2);
  if (e == hipSuccess && !a.hosted && !a.chunked) e = launch_translate_accept(a, st);
  OT_MARK(3);
  if (e == hipSuccess) e = launch_final_draw(a, in->row_off_host, st);
  OT_MARK(4);
#undef OT_MARK
  if (e != hipSuccess) return fail_hip(e, "ot_verify_step: launch");
  if (ev) ctx->pending += 1;
  return OT_OK;
}

int ot_verify_step(ot_ctx* ctx, ot_ngram_cache* cache, const ot_step_in* in, ot_step_out* out) {
  return step_impl(ctx, cache, in, nullptr, false, out);
}

int ot_verify_step_from_logits(ot_ctx* ctx, ot_ngram_cache* cache, const ot_step_in* in,
                               const float* target_logits, ot_step_out* out) {
  return step_impl(ctx, cache, in, target_logits, true, out);
}

int ot_verify_workspace(ot_ctx* ctx, ot_workspace_view* v) {
  if (!ctx || !v) return fail(OT_ERR_NULL, "ot_verify_workspace: NULL argument");
  v->logits = ctx->Z; v->ld_logits = ctx->V_t;
  v->row_max = ctx->row_max; v->row_sumexp = ctx->row_sum; v->row_argmax = ctx->row_arg;
  v->draft_row_max = ctx->drow_max; v->draft_row_sumexp = ctx->drow_sum; v->draft_row_argmax = ctx->drow_arg;
  return OT_OK;
}

int ot_verify_profile(ot_ctx* ctx, int32_t enable) {
  if (!ctx) return fail(OT_ERR_NULL, "ot_verify_profile: ctx is NULL");
  ctx->profiling = enable != 0;
  return OT_OK;
}

int ot_verify_profile_read(ot_ctx* ctx, float* ms, int32_t* n_steps) {
  if (!ctx || !ms || !n_steps) return fail(OT_ERR_NULL, "ot_verify_profile_read: NULL argument");
  hipError_t e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return fail_hip(e, "ot_verify_profile_read: synchronize");
  for (int s = 0; s < OT_N_STAGES; ++s) ms[s] = 0.f;
  for (int p = 0; p < ctx->pending; ++p) {
    hipEvent_t* ev = &ctx->events[(size_t)p * kEventsPerStep];
    for (int s = 0; s < OT_N_STAGES; ++s) {
      float t = 0.f;
      e = hipEventElapsedTime(&t, ev[s], ev[s + 1]);
      if (e != hipSuccess) return fail_hip(e, "hipEventElapsedTime");
      ms[s] += t;
    }
  }
  *n_steps = ctx->pending;
  ctx->pending = 0;
  return OT_OK;
}

}  // extern "C"
#pragma GCC visibility pop
