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

// GELU and its derivative are evaluated together (they share the erf, or the sigmoid, and the
// exponential): the FC1 epilogue stores gelu(z) for the next product and gelu'(z) for the backward
// pass.  Exact (erf) form  gelu(z) = z Phi(z),  gelu'(z) = Phi(z) + z phi(z):
// fp32 outputs use erff; bf16 outputs use erf by Abramowitz & Stegun 7.1.26 (|error| <= 1.5e-7:
// one reciprocal, one exponential and a degree-5 polynomial).
GX_DEVINL void gelu_both_f(float z, float& y, float& dy) {
  const float cdf = 0.5f * (1.0f + erff(z * 0.70710678118654752440f));
  y = z * cdf;
  dy = fmaf(z * 0.39894228040143267794f, __expf(-0.5f * z * z), cdf);
}
GX_DEVINL void gelu_both_fast(float z, float& y, float& dy) {
  const float ax = fabsf(z) * 0.70710678118654752440f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  const float e = __expf(-ax * ax);                    // exp(-z^2 / 2)
  const float cdf = 0.5f * (1.0f + copysignf(fmaf(-p * t, e, 1.0f), z));
  y = z * cdf;
  dy = fmaf(z * 0.39894228040143267794f, e, cdf);
}

// The tanh form, gelu(z) = z s with s = sigmoid(2u), u = sqrt(2/pi) (z + 0.044715 z^3), and
// gelu'(z) = s + 2 z s (1 - s) u'(z): full-precision exponential and division for fp32 outputs,
// hardware exponential and reciprocal for bf16 outputs.
GX_DEVINL void gelu_tanh_both_f(float z, float& y, float& dy) {
  const float z2 = z * z;
  const float u = 0.7978845608028654f * fmaf(0.044715f * z2, z, z);
  const float s = 1.0f / (1.0f + expf(-2.0f * u));
  y = z * s;
  dy = fmaf(2.0f * y * (1.0f - s), 0.7978845608028654f * fmaf(0.134145f, z2, 1.0f), s);
}
GX_DEVINL void gelu_tanh_both_fast(float z, float& y, float& dy) {
  const float z2 = z * z;
  const float u = 0.7978845608028654f * fmaf(0.044715f * z2, z, z);
  const float s = __builtin_amdgcn_rcpf(1.0f + __expf(-2.0f * u));
  y = z * s;
  dy = fmaf(2.0f * y * (1.0f - s), 0.7978845608028654f * fmaf(0.134145f, z2, 1.0f), s);
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
// maximum of a value over lanes l and l ^ 32 (the two halves of a wavefront), in every lane, by one
// v_permlane32_swap instead of a round trip through the LDS crossbar: the swap of two copies of x
// leaves (low half, low half) in one register and (high half, high half) in the other
GX_DEVINL float max_across_halves(float x) {
  const unsigned u = __builtin_bit_cast(unsigned, x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__builtin_bit_cast(float, r[0]), __builtin_bit_cast(float, r[1]));
}
GX_DEVINL void lds_wait_all() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
// wait until at most N LDS operations of this wavefront are outstanding (they complete in order)
template <int N>
GX_DEVINL void lds_wait_le() { asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory"); }
GX_DEVINL void lds_pin(bf16x4& v) { asm volatile("" : "+v"(v)); }

inline int cdiv(long a, long b) { return (int)((a + b - 1) / b); }

}  // namespace gx
