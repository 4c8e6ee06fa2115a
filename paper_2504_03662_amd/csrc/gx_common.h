// Internal helpers shared by the HIP translation units of the library (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gx {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((address_space(3))) void* lds_void_ptr;

#define GX_DEVINL __device__ __forceinline__

GX_DEVINL float to_f32(float v) { return v; }
GX_DEVINL float to_f32(bf16 v) { return (float)v; }
template <typename T> GX_DEVINL T from_f32(float v);
template <> GX_DEVINL float from_f32<float>(float v) { return v; }
template <> GX_DEVINL bf16 from_f32<bf16>(float v) { return (bf16)v; }   // round to nearest even

// exact (erf) GELU and its derivative, fp32
GX_DEVINL float gelu_f(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752440f)); }
GX_DEVINL float gelu_grad_f(float z) {
  float cdf = 0.5f * (1.0f + erff(z * 0.70710678118654752440f));
  float pdf = 0.39894228040143267794f * __expf(-0.5f * z * z);
  return cdf + z * pdf;
}

// erf by Abramowitz & Stegun 7.1.26 (|error| <= 1.5e-7): one reciprocal, one exponential and a
// degree-5 polynomial; returns erf(|x|) and exp(-x^2) so that the GELU derivative can share them.
GX_DEVINL float erf_abs_as(float ax, float& e) {
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  e = __expf(-ax * ax);
  return fmaf(-p * t, e, 1.0f);
}
// GELU and its derivative on that erf; accurate to ~2e-7 absolute, for bf16 outputs
GX_DEVINL float gelu_fast(float z) {
  float e;
  const float r = erf_abs_as(fabsf(z) * 0.70710678118654752440f, e);
  return 0.5f * z * (1.0f + copysignf(r, z));
}
GX_DEVINL float gelu_grad_fast(float z) {
  float e;
  const float r = erf_abs_as(fabsf(z) * 0.70710678118654752440f, e);
  return fmaf(z * 0.39894228040143267794f, e, 0.5f * (1.0f + copysignf(r, z)));
}

// The tanh form of GELU, z * sigmoid(2u) with u = sqrt(2/pi) (z + 0.044715 z^3), and its derivative
// s + 2 z s (1 - s) u'(z), s = sigmoid(2u); full-precision exponential and division for fp32
// outputs, hardware exponential and reciprocal for bf16 outputs.
GX_DEVINL float gelu_tanh_f(float z) {
  const float u = 0.7978845608028654f * fmaf(0.044715f * z * z, z, z);
  return z / (1.0f + expf(-2.0f * u));
}
GX_DEVINL float gelu_tanh_grad_f(float z) {
  const float z2 = z * z;
  const float u = 0.7978845608028654f * fmaf(0.044715f * z2, z, z);
  const float s = 1.0f / (1.0f + expf(-2.0f * u));
  return fmaf(2.0f * z * s * (1.0f - s), 0.7978845608028654f * fmaf(0.134145f, z2, 1.0f), s);
}
GX_DEVINL float gelu_tanh_fast(float z) {
  const float u = 0.7978845608028654f * fmaf(0.044715f * z * z, z, z);
  return z * __builtin_amdgcn_rcpf(1.0f + __expf(-2.0f * u));
}
GX_DEVINL float gelu_tanh_grad_fast(float z) {
  const float z2 = z * z;
  const float u = 0.7978845608028654f * fmaf(0.044715f * z2, z, z);
  const float s = __builtin_amdgcn_rcpf(1.0f + __expf(-2.0f * u));
  return fmaf(2.0f * z * s * (1.0f - s), 0.7978845608028654f * fmaf(0.134145f, z2, 1.0f), s);
}

GX_DEVINL float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
GX_DEVINL float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Transposing LDS read (ds_read_b64_tr_b16) issued through inline assembly.  The compiler cannot
// tell that such a read does not touch the LDS region a direct-to-LDS load is still filling, and
// makes the builtin form wait for every load in flight (vmcnt(0)), which serialises the global
// prefetch with the matrix work.  The kernels already order tiles with explicit waits and
// barriers, so the read is issued untracked here; its result may only be used after
// lds_wait_all() and lds_pin() on the destination registers.
typedef __attribute__((address_space(3))) const char* lds_cptr;
GX_DEVINL unsigned lds_addr(const char* p) { return (unsigned)(unsigned long)(lds_cptr)p; }
template <int OFF>
GX_DEVINL bf16x4 lds_read_tr_issue(unsigned addr) {
  bf16x4 r;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF) : "memory");
  return r;
}
GX_DEVINL void lds_wait_all() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
// wait until at most N LDS operations of this wavefront are outstanding (they complete in order)
template <int N>
GX_DEVINL void lds_wait_le() { asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory"); }
GX_DEVINL void lds_pin(bf16x4& v) { asm volatile("" : "+v"(v)); }

inline int cdiv(long a, long b) { return (int)((a + b - 1) / b); }

}  // namespace gx
