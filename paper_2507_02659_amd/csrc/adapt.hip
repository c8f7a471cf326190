// Adaptive drafting (Section "Online Adaptive Drafting"): the stop rule 1 - prod sigmoid(f_phi(e_i)) > gamma over the
// proposed tokens of every sequence, and the value of the weighted binary cross-entropy that trains the head
// against the acceptance ratios min(1, p/q).  The head's logits are an input.
//
//   adapt_rule_kernel   one workgroup (one wavefront) per sequence: lane i forms sigmoid(a_i) and its two
//                       log-probabilities in binary64; lane 0 walks the running product left to right (at most 63
//                       factors) so that the product has one fixed order; per-sequence loss partials go to the
//                       workspace.
//   adapt_total_kernel  one workgroup adds the partials in a fixed order.
#include <mutex>

#include "otv_host.h"

namespace otv {
namespace {

struct AdaptArgs {
  ot_adapt_in in;
  ot_adapt_out out;
  double* part;      // [B, 2] loss sum and token count of each sequence
};

__global__ __launch_bounds__(64) void adapt_rule_kernel(AdaptArgs a) {
  const int b = blockIdx.x, i = threadIdx.x;
  const int r0 = a.in.row_off[b], k = a.in.row_off[b + 1] - r0 - 1;
  const int n = a.in.n_valid ? min(k, max(a.in.n_valid[b], 0)) : k;
  __shared__ double s_sig[64];
  __shared__ double s_cost[64];
  double sig = 0.0, cost = 0.0;
  if (i < n) {
    const double x = (double)a.in.head_logits[r0 + i];
    sig = 1.0 / (1.0 + exp(-x));
    if (a.out.bce) {
      // ln sigmoid(x) = -(ln(1 + e^-|x|) + max(-x, 0)),  ln(1 - sigmoid(x)) = -(ln(1 + e^-|x|) + max(x, 0))
      const double t = log1p(exp(-fabs(x)));
      const double l = (double)a.in.labels[r0 + i];
      cost = (double)a.in.w_accept * l * (t + fmax(-x, 0.0)) + (double)a.in.w_reject * (1.0 - l) * (t + fmax(x, 0.0));
    }
  }
  s_sig[i] = sig;
  s_cost[i] = cost;
  if (i <= k) a.out.p_accept[r0 + i] = (float)sig;       // the sequence's unused entries read 0
  __syncthreads();
  if (i == 0) {
    const double gamma = (double)a.in.gamma;
    double alive = 1.0, total = 0.0;
    int keep = n;
    for (int j = 0; j <= k; ++j) {
      double rej = 0.0;
      if (j < n) {
        alive *= s_sig[j];
        rej = 1.0 - alive;
        total += s_cost[j];
        if (keep == n && rej > gamma) keep = j + 1;
      }
      a.out.p_any_reject[r0 + j] = (float)rej;
    }
    a.out.n_keep[b] = keep;
    a.part[2 * b] = total;
    a.part[2 * b + 1] = (double)n;
  }
}

__global__ __launch_bounds__(256) void adapt_total_kernel(AdaptArgs a) {
  __shared__ double s_w[2][4];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  double total = 0.0, count = 0.0;
  for (int b = tid; b < a.in.B; b += 256) { total += a.part[2 * b]; count += a.part[2 * b + 1]; }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) { total += __shfl_xor(total, off); count += __shfl_xor(count, off); }
  if (lane == 0) { s_w[0][wave] = total; s_w[1][wave] = count; }
  __syncthreads();
  if (tid == 0) {
    const double t = (s_w[0][0] + s_w[0][1]) + (s_w[0][2] + s_w[0][3]);
    const double c = (s_w[1][0] + s_w[1][1]) + (s_w[1][2] + s_w[1][3]);
    a.out.bce[0] = t;
    a.out.bce[1] = c;
    a.out.bce[2] = t / fmax(1.0, c);
  }
}

}  // namespace
}  // namespace otv

using namespace otv;

namespace {

// Scratch of ot_adaptive_drafting_static: the per-sequence loss partials, in an array that is part of the library's
// code object instead of an allocation.  Every GPU the library runs on holds its own copy at its own address; that
// address is looked up once per device (the array's name is only a host-side handle, never a device pointer).
static __device__ __align__(256) double scratch[2 * OT_STATIC_MAX_BATCH];

constexpr int kMaxDevices = 64;
double* g_scratch_ptr[kMaxDevices];        // device address of `scratch` on each device, nullptr until looked up
std::mutex g_scratch_mutex;

// Address of `scratch` on the current device (looked up on the first call per device), or nullptr with the error set.
double* static_scratch() {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { (void)ot_fail_hip(e, "hipGetDevice"); return nullptr; }
  if (dev < 0 || dev >= kMaxDevices) { (void)ot_fail(OT_ERR_SHAPE, "device index %d is not supported", dev); return nullptr; }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) { (void)ot_fail_hip(e, "hipGetSymbolAddress(scratch)"); return nullptr; }
    g_scratch_ptr[dev] = static_cast<double*>(p);
  }
  return g_scratch_ptr[dev];
}

// Validates the arguments shared by the two entry points and launches on `stream` with the loss partials in `part`.
int adaptive_drafting(const char* who, const ot_adapt_in* in, ot_adapt_out* out, int max_batch, int max_k, double* part,
                      hipStream_t stream) {
  if (in->reserved != 0) return ot_fail(OT_ERR_SHAPE, "%s: reserved must be 0", who);
  if (in->B < 0 || in->B > max_batch) return ot_fail(OT_ERR_SHAPE, "%s: B = %d exceeds the limit of %d sequences", who, in->B, max_batch);
  if (!(in->gamma >= 0.f && in->gamma <= 1.f)) return ot_fail(OT_ERR_SHAPE, "%s: gamma must be in [0, 1]", who);
  if (out->bce && !in->labels) return ot_fail(OT_ERR_NULL, "%s: the loss value needs labels", who);
  if (out->bce && !(in->w_accept >= 0.f && in->w_reject >= 0.f)) return ot_fail(OT_ERR_SHAPE, "%s: weights must be non-negative", who);
  AdaptArgs a{};
  a.in = *in; a.out = *out; a.part = part;
  if (in->B > 0) {
    if (!in->row_off || !in->row_off_host || !in->head_logits) return ot_fail(OT_ERR_NULL, "%s: row_off, row_off_host and head_logits must not be NULL", who);
    if (!out->p_accept || !out->p_any_reject || !out->n_keep) return ot_fail(OT_ERR_NULL, "%s: p_accept, p_any_reject and n_keep are required", who);
    if (in->row_off_host[0] != 0) return ot_fail(OT_ERR_SHAPE, "%s: row_off[0] must be 0", who);
    for (int b = 0; b < in->B; ++b) {
      const int64_t rows = (int64_t)in->row_off_host[b + 1] - in->row_off_host[b];
      if (rows < 1 || rows - 1 > max_k) return ot_fail(OT_ERR_SHAPE, "%s: sequence %d owns %lld rows", who, b, (long long)rows);
    }
    hipLaunchKernelGGL(adapt_rule_kernel, dim3(in->B), dim3(64), 0, stream, a);
  }
  if (out->bce) hipLaunchKernelGGL(adapt_total_kernel, dim3(1), dim3(256), 0, stream, a);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return ot_fail_hip(e, who);
  return OT_OK;
}

}  // namespace

// Looks up the static scratch of the current device ahead of the first ot_adaptive_drafting_static call (from
// ot_verify_init, so that a caller who must not trigger any set-up later has it done).
int ot_static_scratch_prepare() { return static_scratch() ? OT_OK : OT_ERR_HIP; }

#pragma GCC visibility push(default)
extern "C" {

int ot_adaptive_drafting(ot_ctx* ctx, const ot_adapt_in* in, ot_adapt_out* out) {
  if (!ctx || !in || !out) return ot_fail(OT_ERR_NULL, "ot_adaptive_drafting: ctx, in and out must not be NULL");
  return adaptive_drafting("ot_adaptive_drafting", in, out, ctx->max_batch, ctx->max_k, ctx->adapt_part, ctx->stream);
}

int ot_adaptive_drafting_static(const ot_adapt_in* in, ot_adapt_out* out, void* stream) {
  if (!in || !out) return ot_fail(OT_ERR_NULL, "ot_adaptive_drafting_static: in and out must not be NULL");
  if (in->B > OT_STATIC_MAX_BATCH)
    return ot_fail(OT_ERR_SHAPE, "ot_adaptive_drafting_static: B = %d exceeds OT_STATIC_MAX_BATCH = %d, the size of the static "
                   "scratch; use ot_adaptive_drafting", in->B, OT_STATIC_MAX_BATCH);
  double* part = static_scratch();
  if (!part) return OT_ERR_HIP;
  return adaptive_drafting("ot_adaptive_drafting_static", in, out, OT_STATIC_MAX_BATCH, OT_MAX_K, part, static_cast<hipStream_t>(stream));
}

}  // extern "C"
#pragma GCC visibility pop
