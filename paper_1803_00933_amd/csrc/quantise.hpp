// Priority -> integer sampling mass:  Q(p) = clamp(floor((|p| + eps)^alpha * 2^F), 1, QMAX).
//
// The paper draws a transition with probability p^alpha / sum_k p_k^alpha (Appendix
// "Implementation", "Sampling Data") and leaves the arithmetic open.  Here the mass is an
// integer so that tree sums are exact and order independent, and the power is a fixed chain of
// IEEE fp32 operations (no fast-math intrinsics, no contraction: this file must be compiled
// with -ffp-contract=off) so that the integer does not depend on the machine:
//   x = m * 2^e, m in (sqrt(1/2), sqrt(2)];  log2 m = f * P10(f), f = m - 1;
//   alpha * (e + log2 m) kept as hi + zl with hi = fl(e * alpha), zl = fma(alpha, log2 m, e*alpha - hi);
//   n = rint(hi + zl), r = (hi - n) + zl, 2^r = P7(r);  result = P7(r) * 2^n.
// Relative error against the exact power is below 2e-7 for x in [2^-100, 2^100], |alpha| <= 1.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace apex {

__device__ __forceinline__ float pow_fixed_sequence(float x, float alpha)
{
  // coefficients of log2(1+f)/f, f in [sqrt(1/2)-1, sqrt(2)-1], lowest order first
  constexpr float kLog2[11] = {0x1.715476p+0f, -0x1.715476p-1f, 0x1.ec707ep-2f, -0x1.71548cp-2f,
                               0x1.2780bap-2f, -0x1.ec7be2p-3f, 0x1.a3e68ap-3f, -0x1.6e459ap-3f,
                               0x1.60767ep-3f, -0x1.5b108p-3f, 0x1.8efecp-4f};
  // coefficients of 2^r, r in [-0.53, 0.53]
  constexpr float kExp2[8] = {0x1.0p+0f, 0x1.62e43p-1f, 0x1.ebfbep-3f, 0x1.c6b08ep-5f,
                              0x1.3b299ep-7f, 0x1.5d8716p-10f, 0x1.449884p-13f, 0x1.00faccp-16f};
  const uint32_t bits = __float_as_uint(x);
  int e = (int)((bits >> 23) & 0xffu) - 127;
  float m = __uint_as_float((bits & 0x007fffffu) | 0x3f800000u);
  if (m > 0x1.6a09e6p+0f) {
    m = m * 0.5f;
    e += 1;
  }
  const float f = m - 1.0f;
  float pl = kLog2[10];
#pragma unroll
  for (int i = 9; i >= 0; --i) pl = __builtin_fmaf(pl, f, kLog2[i]);
  const float log2m = f * pl;

  const float ef = (float)e;
  const float hi = ef * alpha;
  const float lo = __builtin_fmaf(ef, alpha, -hi);
  const float zl = __builtin_fmaf(alpha, log2m, lo);
  const float t = hi + zl;
  const float n = __builtin_rintf(t);
  const float r = (hi - n) + zl;

  float pe = kExp2[7];
#pragma unroll
  for (int i = 6; i >= 0; --i) pe = __builtin_fmaf(pe, r, kExp2[i]);
  const float two_n = __uint_as_float((uint32_t)((int)n + 127) << 23);
  return pe * two_n;
}

struct QuantParams {
  float alpha;
  float eps;
  uint32_t frac_bits;
  uint64_t qmax;
};

// Returns the mass; *clamped is set when the value had to be forced into [1, qmax].
__device__ __forceinline__ uint64_t quantise_priority(float p, const QuantParams &qp, bool *clamped)
{
  float x = __builtin_fabsf(p) + qp.eps;
  if (!(x >= 0x1p-100f)) x = 0x1p-100f;  // also catches NaN
  if (x > 0x1p+100f) x = 0x1p+100f;
  const float y = pow_fixed_sequence(x, qp.alpha);
  const float s = y * __uint_as_float((qp.frac_bits + 127u) << 23);
  uint64_t q = (s >= 0x1p+62f) ? (1ull << 62) : (uint64_t)s;  // conversion truncates
  bool c = false;
  if (q < 1) {
    q = 1;
    c = true;
  }
  if (q > qp.qmax) {
    q = qp.qmax;
    c = true;
  }
  *clamped = c;
  return q;
}

}  // namespace apex
