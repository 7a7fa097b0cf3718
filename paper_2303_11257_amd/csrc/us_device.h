// Device-side helpers shared by the gfx950 kernels: vector types, FP8/FP16 conversion, GELU math.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/us.h"

namespace us {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef short v4s __attribute__((ext_vector_type(4)));

// Unit-scaling factors of gelu(x) = x*Phi(x) for x ~ N(0,1) (Table A.2 prints 1.701 / 1.481):
// alpha = 1/std(gelu), beta = 1/rms(gelu'), closed forms
//   E[gelu^2] = 1/3 + 1/(2 pi sqrt3), E[gelu] = 1/(2 sqrt pi), E[gelu'^2] = 1/3 + 2/(3 pi sqrt3).
constexpr float kGeluAlpha = 1.7009261846542358f;
constexpr float kGeluBeta = 1.481114387512207f;

// ---- FP32 -> FP16 ------------------------------------------------------------------------------------
// Round-to-nearest-even conversion that keeps the sign of a zero product: the compiler likes to fuse
// "multiply, then convert" into v_fma_mixlo_f16(a, b, +0), and (-0) + (+0) is +0.  The empty asm makes
// the product a value of its own, so the conversion stays a plain v_cvt.
__device__ __forceinline__ _Float16 to_half(float x) {
  asm volatile("" : "+v"(x));
  return (_Float16)x;
}

// ---- write-through global stores ------------------------------------------------------------------------------
// A plain (or non-temporal) store leaves its line dirty in the XCD's L2 until it is evicted or until the write-back
// that ends the kernel; with tens of MB written per launch every launch then ends with a burst of up to 32 MB that
// nothing overlaps (measured with an idle kernel that only writes: 1.2 us between launches without writes, 4.0 us with
// 32 MB or more of plain or non-temporal stores, 1.2 us again with the stores below).  sc0 sc1 sends the data on to
// memory at once, where the next launch finds it (its own L2 starts empty either way).  8 or 16 bytes per lane; the
// s_nop covers the store-data hazard that the compiler cannot see through the asm statement.
template <class V>
__device__ __forceinline__ void wt_store(V* p, V v) {
  static_assert(sizeof(V) == 16 || sizeof(V) == 8, "");
  if constexpr (sizeof(V) == 16) {
    v4i w;
    __builtin_memcpy(&w, &v, 16);
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" ::"v"(p), "v"(w) : "memory");
  } else {
    v2i w;
    __builtin_memcpy(&w, &v, 8);
    asm volatile("global_store_dwordx2 %0, %1, off sc0 sc1\n\ts_nop 1" ::"v"(p), "v"(w) : "memory");
  }
}

// ---- FP32 x FP16 -> FP16 with one rounding ---------------------------------------------------------------
// fp16(t * y) for an FP32 factor t and the FP16 value in half SRC_HI of the pair `ypair`, written into half DST_HI of
// `dst` (the other half of dst is kept): one v_fma_mix instruction, which rounds the exact product once.  Its addend
// is -0, so that a zero product keeps its sign ((-0) + (-0) = -0, (+0) + (-0) = +0) and every other product is unchanged.
template <int SRC_HI, int DST_HI>
__device__ __forceinline__ void mul_to_half(uint32_t& dst, float t, uint32_t ypair) {
  const float neg_zero = -0.0f;
  if constexpr (DST_HI == 0) {
    if constexpr (SRC_HI == 0)
      asm volatile("v_fma_mixlo_f16 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[0,1,0]" : "+v"(dst) : "v"(t), "v"(ypair), "v"(neg_zero));
    else
      asm volatile("v_fma_mixlo_f16 %0, %1, %2, %3 op_sel:[0,1,0] op_sel_hi:[0,1,0]" : "+v"(dst) : "v"(t), "v"(ypair), "v"(neg_zero));
  } else {
    if constexpr (SRC_HI == 0)
      asm volatile("v_fma_mixhi_f16 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[0,1,0]" : "+v"(dst) : "v"(t), "v"(ypair), "v"(neg_zero));
    else
      asm volatile("v_fma_mixhi_f16 %0, %1, %2, %3 op_sel:[0,1,0] op_sel_hi:[0,1,0]" : "+v"(dst) : "v"(t), "v"(ypair), "v"(neg_zero));
  }
}
// the same for one value
__device__ __forceinline__ _Float16 mul_to_half(float t, _Float16 y) {
  unsigned short yb;
  __builtin_memcpy(&yb, &y, 2);
  uint32_t d = 0;
  mul_to_half<0, 0>(d, t, (uint32_t)yb);
  const unsigned short r = (unsigned short)d;
  _Float16 h;
  __builtin_memcpy(&h, &r, 2);
  return h;
}

// ---- FP32 -> FP8 (E4M3: max 448, one NaN, no inf; E5M2: max 57344) -------------------------------
// The hardware converter rounds to nearest-even and handles subnormals; it turns overflow into
// NaN/inf, so the value is first clipped to the finite range (that also maps +-inf to +-max).
// v_med3 drops a NaN operand, so NaN inputs get their NaN code put back afterwards.
// Returns code(a) | code(b) << 8.
template <int FMT>
__device__ __forceinline__ uint32_t cvt_pk_fp8(float a, float b) {
  constexpr float kMax = (FMT == US_E4M3) ? 448.0f : 57344.0f;
  float ca = __builtin_amdgcn_fmed3f(a, -kMax, kMax);
  float cb = __builtin_amdgcn_fmed3f(b, -kMax, kMax);
  uint32_t r = (FMT == US_E4M3) ? (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(ca, cb, 0, false)
                                : (uint32_t)__builtin_amdgcn_cvt_pk_bf8_f32(ca, cb, 0, false);
  r &= 0xffffu;
  if (a != a) r |= 0x007fu;
  if (b != b) r |= 0x7f00u;
  return r;
}

template <int FMT>
__device__ __forceinline__ uint32_t cvt4_fp8(float a, float b, float c, float d) {
  return cvt_pk_fp8<FMT>(a, b) | (cvt_pk_fp8<FMT>(c, d) << 16);
}

// ---- FP16 -> FP8, two values per instruction ----------------------------------------------------------
// For values that already are FP16 (the epilogues' stored results): clip with the NaN-propagating
// packed minimum/maximum, then the packed FP16->FP8 converter with unit scale.  Checked on the
// device against cvt_pk_fp8 above for all 65536 FP16 inputs (identical codes, NaN stays NaN).
// Returns code(h[0]) | code(h[1]) << 8.
template <int FMT>
__device__ __forceinline__ uint32_t cvt_pk_fp8_from_half(v2h h) {
  typedef short v2s __attribute__((ext_vector_type(2)));
  const _Float16 mx = (FMT == US_E4M3) ? (_Float16)448.0f : (_Float16)57344.0f;
  const v2h hi = {mx, mx}, lo = {-mx, -mx};
  const v2h c = __builtin_elementwise_minimum(__builtin_elementwise_maximum(h, lo), hi);
  const v2s old = {0, 0};
  const v2s r = (FMT == US_E4M3) ? __builtin_amdgcn_cvt_scalef32_pk_fp8_f16(old, c, 1.0f, false)
                                 : __builtin_amdgcn_cvt_scalef32_pk_bf8_f16(old, c, 1.0f, false);
  return (uint32_t)(uint16_t)r.x;
}

// ---- Gaussian tail for GELU -------------------------------------------------------------------------
// Q(x) = P(N(0,1) > x) for x >= 0 is evaluated as exp(-x^2/2) * t*(c0 + c1 t + ... + c5 t^5) with
// t = 1/(1 + p x): a fit of the scaled complementary error function erfcx(x/sqrt2)/2 whose relative
// error stays below 4e-6 on [0, 14], so Phi keeps relative accuracy in the negative tail too
// (coefficients from fit_gauss_tail.py beside this header: reweighted least squares against a double-precision erfcx).
struct GaussTerms {
  float Phi;  // standard normal CDF at z
  float pdf;  // standard normal density at z
};

__device__ __forceinline__ GaussTerms gauss_terms(float z) {
  constexpr float p = 0.308158117f;
  constexpr float c0 = 0.12318376f, c1 = 0.11897348f, c2 = 0.136421f, c3 = 0.00767712f,
                  c4 = 0.18914684f, c5 = -0.07540414f;
  float az = __builtin_fabsf(z);
  float t = __builtin_amdgcn_rcpf(__builtin_fmaf(p, az, 1.0f));
  float e = __builtin_amdgcn_exp2f(-0.7213475204444817f * (z * z));  // exp(-z^2/2) = 2^(-z^2 * log2(e)/2)
  float poly = __builtin_fmaf(c5, t, c4);
  poly = __builtin_fmaf(poly, t, c3);
  poly = __builtin_fmaf(poly, t, c2);
  poly = __builtin_fmaf(poly, t, c1);
  poly = __builtin_fmaf(poly, t, c0);
  const float pt = poly * t;
  GaussTerms g;
  g.Phi = (z < 0.0f) ? pt * e : __builtin_fmaf(-pt, e, 1.0f);
  g.pdf = 0.3989422804014327f * e;
  return g;
}

// h = alpha_g * z * Phi(z)
__device__ __forceinline__ float gelu_scaled(float z, float alpha_g) {
  GaussTerms g = gauss_terms(z);
  return alpha_g * (z * g.Phi);
}
// beta_g * gelu'(|z|),  gelu'(x) = Phi(x) + x*phi(x)
__device__ __forceinline__ float gelu_slope_abs(float az, float beta_g) {
  GaussTerms g = gauss_terms(az);
  return beta_g * __builtin_fmaf(az, g.pdf, g.Phi);
}
// beta_g * gelu'(z).  Negative arguments use gelu'(-x) = 1 - gelu'(x), so that the function of |z| can also be
// tabulated (see the table-driven GEMM epilogue); +-inf and NaN give NaN.
__device__ __forceinline__ float gelu_slope_scaled(float z, float beta_g) {
  const float t = gelu_slope_abs(__builtin_fabsf(z), beta_g);
  return (__builtin_signbit(z)) ? beta_g - t : t;
}
// beta_g * gelu'(z) * gh in FP32
__device__ __forceinline__ float gelu_grad_scaled(float z, float gh, float beta_g) { return gelu_slope_scaled(z, beta_g) * gh; }
// fp16(beta_g * gelu'(z) * gh) for FP16 z and gh: the FP32 slope times gh, rounded once (what the table-driven epilogue
// computes from its table of slopes)
__device__ __forceinline__ _Float16 gelu_grad_half(_Float16 z, _Float16 gh, float beta_g) {
  return mul_to_half(gelu_slope_scaled((float)z, beta_g), gh);
}

// ---- the other activations of Table A.2 ---------------------------------------------------------------
// kind: 0 gelu, 1 relu, 2 tanh, 3 sigmoid (us_activation).  Unit-scaling factors by the rule of Sec. 5.2
// (alpha = 1/std f(z), beta = 1/rms f'(z), z ~ N(0,1)): relu in closed form (App. E.1), tanh and sigmoid
// by quadrature (Table A.2 prints 1.593 / 1.467 and 4.802 / 4.722).
constexpr float kActAlpha[4] = {kGeluAlpha, 1.7128585577011108f, 1.5925374031066895f, 4.801313400268555f};
constexpr float kActBeta[4] = {kGeluBeta, 1.4142135381698608f, 1.4674135446548462f, 4.722646236419678f};

// exp(-a) for a >= 0
__device__ __forceinline__ float exp_neg(float a) { return __builtin_amdgcn_exp2f(-1.4426950408889634f * a); }

__device__ __forceinline__ float tanh_f32(float x) {
  const float ax = __builtin_fabsf(x);
  float t;
  if (ax < 0.25f) {
    // odd Taylor polynomial: (1 - u)/(1 + u) below would cancel for small arguments
    const float x2 = ax * ax;
    float p = __builtin_fmaf(x2, 62.0f / 2835.0f, -17.0f / 315.0f);
    p = __builtin_fmaf(p, x2, 2.0f / 15.0f);
    p = __builtin_fmaf(p, x2, -1.0f / 3.0f);
    t = __builtin_fmaf(p * x2, ax, ax);
  } else {
    const float u = exp_neg(2.0f * ax);
    t = (1.0f - u) * __builtin_amdgcn_rcpf(1.0f + u);
  }
  return __builtin_copysignf(t, x);
}

// scale * f(x)
__device__ __forceinline__ float act_scaled(int kind, float x, float scale) {
  if (kind == 1) return scale * (x > 0.0f ? x : 0.0f);
  if (kind == 2) return scale * tanh_f32(x);
  if (kind == 3) {
    const float u = exp_neg(__builtin_fabsf(x));
    const float r = __builtin_amdgcn_rcpf(1.0f + u);
    return scale * (x >= 0.0f ? r : u * r);
  }
  return gelu_scaled(x, scale);
}
// scale * f'(z)   (relu'(0) = 0)
__device__ __forceinline__ float act_slope_scaled(int kind, float z, float scale) {
  if (kind == 1) return z > 0.0f ? scale : 0.0f;
  if (kind == 2) {                                    // sech^2 = 4u / (1 + u)^2, u = exp(-2|z|)
    const float u = exp_neg(2.0f * __builtin_fabsf(z));
    const float r = __builtin_amdgcn_rcpf(1.0f + u);
    return scale * (4.0f * u * r * r);
  }
  if (kind == 3) {                                    // s (1 - s) = u / (1 + u)^2, u = exp(-|z|)
    const float u = exp_neg(__builtin_fabsf(z));
    const float r = __builtin_amdgcn_rcpf(1.0f + u);
    return scale * (u * r * r);
  }
  return gelu_slope_scaled(z, scale);
}
// scale * f'(z) * gh in FP32, and rounded once to FP16 for an FP16 gh (the form every FP16 backward path uses)
__device__ __forceinline__ float act_grad_scaled(int kind, float z, float gh, float scale) { return act_slope_scaled(kind, z, scale) * gh; }
__device__ __forceinline__ _Float16 act_grad_half(int kind, float z, _Float16 gh, float scale) {
  return mul_to_half(act_slope_scaled(kind, z, scale), gh);
}

// ---- tables over the FP16 pre-activation (65536 possible inputs) ----------------------------------------
// Forward: the E4M3 code of fp16(alpha_g * gelu(z)) for every bit pattern of z.
// Backward: beta_g * gelu'(|z|) in FP32 for |z| <= 8 (bit patterns 0 .. 0x4800; the slope is exactly
// 1 in FP32 beyond that).  Both are filled by the same device functions the arithmetic epilogues use,
// so the table-driven epilogues give identical results.
constexpr int kGeluTableBytes = 65536;
constexpr int kGeluSlopeLast = 0x4800;                                   // FP16 bits of 8.0
constexpr int kGeluSlopeTableBytes = 73 * 1024;                          // (0x4801 entries * 4 B) rounded up to whole KB
constexpr int kTableAreaBytes = US_TABLE_AREA_BYTES;                     // head of a workspace reserved for tables
// Forward with FP16 activation output: fp16(alpha_g * gelu(z)) for |z| <= 6 (bit patterns 0 .. 0x4600), the
// non-negative inputs first, then the negative ones.  Beyond 6 the FP32 Phi is exactly 1 (result
// alpha_g * z) resp. small enough that the product rounds to -0.
constexpr int kGeluHalfLast = 0x4600;                                    // FP16 bits of 6.0
constexpr int kGeluHalfTableBytes = 72 * 1024;                           // (2 * 0x4601 entries * 2 B) rounded up to whole KB
// places of the three tables in the table area
constexpr int kGeluTableOffset = 0;
constexpr int kGeluSlopeTableOffset = kGeluTableOffset + kGeluTableBytes;
constexpr int kGeluHalfTableOffset = kGeluSlopeTableOffset + kGeluSlopeTableBytes;
static_assert(kGeluHalfTableOffset + kGeluHalfTableBytes <= kTableAreaBytes, "the tables fit their area");

__device__ __forceinline__ _Float16 half_from_bits(uint32_t b) {
  const unsigned short u = (unsigned short)b;
  _Float16 h;
  __builtin_memcpy(&h, &u, 2);
  return h;
}
__device__ __forceinline__ uint32_t half_bits(_Float16 h) {
  unsigned short u;
  __builtin_memcpy(&u, &h, 2);
  return u;
}

}  // namespace us
