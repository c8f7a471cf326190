// Small device helpers shared by the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace otv {

__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// exp(x) for x <= 0 in binary64 with a relative error of about one binary32 ulp (1e-7), at a dozen instructions
// instead of a full binary64 exponential: the range reduction x*log2(e) = n + f, |f| <= 1/2, is done in binary64, the
// fraction goes through the hardware 2^f, and the result is scaled by 2^n.  Used where millions of terms are summed
// (residual masses); single decisive values (p(t_j), q') use the full-precision exp().
__device__ inline double exp_neg_fast(double x) {
  const double t = fmax(x, -1000.0) * 1.4426950408889634;
  const double n = rint(t);
  const float e = __builtin_amdgcn_exp2f((float)(t - n));
  return ldexp((double)e, (int)n);
}

// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies and key-mixed xors.
__device__ inline void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1,
                                     uint32_t out[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Uniform in [0, 1): the top 24 bits of a word, exactly representable in binary32 and binary64.
__device__ inline double u24(uint32_t w) { return (double)(w >> 8) * (1.0 / 16777216.0); }

}  // namespace otv
