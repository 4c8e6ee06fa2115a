// fp32 GEMM for the full-precision configuration: a plain LDS-tiled kernel (64x64x32 tile, 4x4
// outputs per thread, fp32 FMAs only, next tile prefetched into registers) with the same layouts
// and epilogues as the bf16 family.  That configuration is a few GFLOP with at most 64 tiles per
// product, so this kernel is written for exactness (no reduced-precision shortcut anywhere), not
// for the matrix cores.
#include "gx_kernels.h"

namespace gx {
namespace {

constexpr int TM = 64, TN = 64, TK = 32;
constexpr int PER = TM * TK / 256;       // elements of each operand tile per thread

template <int LAY, int EPI>
__global__ void __launch_bounds__(256) gemm_f32_kernel(GemmArgs g) {
  __shared__ float sa[TK][TM + 4];
  __shared__ float sb[TK][TN + 4];
  const float* A = static_cast<const float*>(g.A);
  const float* B = static_cast<const float*>(g.B);
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++) acc[i][j] = 0.f;

  // each thread brings PER elements of each tile, walking the operand's contiguous index fastest;
  // the next tile's elements are fetched into registers while the current tile is multiplied
  auto a_pos = [&](int i, int& m, int& k) {
    const int e = tid + 256 * i;
    if (LAY == LAY_TN) { m = e & (TM - 1); k = e / TM; } else { k = e & (TK - 1); m = e / TK; }
  };
  auto b_pos = [&](int i, int& n, int& k) {
    const int e = tid + 256 * i;
    if (LAY == LAY_NT) { k = e & (TK - 1); n = e / TK; } else { n = e & (TN - 1); k = e / TN; }
  };
  float ra[PER], rb[PER];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < PER; i++) {
      int m, k, n, kb;
      a_pos(i, m, k);
      b_pos(i, n, kb);
      ra[i] = 0.f;
      if (m0 + m < g.M && k0 + k < g.K)
        ra[i] = (LAY == LAY_TN) ? A[(size_t)(k0 + k) * g.lda + m0 + m] : A[(size_t)(m0 + m) * g.lda + k0 + k];
      rb[i] = 0.f;
      if (n0 + n < g.N && k0 + kb < g.K)
        rb[i] = (LAY == LAY_NT) ? B[(size_t)(n0 + n) * g.ldb + k0 + kb] : B[(size_t)(k0 + kb) * g.ldb + n0 + n];
    }
  };
  fetch(0);
  for (int k0 = 0; k0 < g.K; k0 += TK) {
#pragma unroll
    for (int i = 0; i < PER; i++) {
      int m, k, n, kb;
      a_pos(i, m, k);
      b_pos(i, n, kb);
      sa[k][m] = ra[i];
      sb[kb][n] = rb[i];
    }
    __syncthreads();
    if (k0 + TK < g.K) fetch(k0 + TK);
#pragma unroll
    for (int k = 0; k < TK; k++) {
      float av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; i++) av[i] = sa[k][ty + 16 * i];
#pragma unroll
      for (int j = 0; j < 4; j++) bv[j] = sb[k][tx + 16 * j];
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
    __syncthreads();
  }

  const float* bias = static_cast<const float*>(g.bias);
  const float* resid = static_cast<const float*>(g.resid);
  const float* zin = static_cast<const float*>(g.z);
  float* aux = static_cast<float*>(g.aux);
  float* C = static_cast<float*>(g.C);
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int row = m0 + ty + 16 * i;
    if (row >= g.M) continue;
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const int col = n0 + tx + 16 * j;
      if (col >= g.N) continue;
      const size_t idx = (size_t)row * g.ldc + col;
      float x = acc[i][j];
      const float bv = ((EPI == EPI_BIAS || EPI == EPI_RESID || EPI == EPI_GELU) && bias) ? bias[col] : 0.f;
      if (EPI == EPI_STORE || EPI == EPI_F32) {
        C[idx] = x;
      } else if (EPI == EPI_BIAS) {
        C[idx] = x + bv;
      } else if (EPI == EPI_RESID) {
        x += bv;
        if (aux) aux[idx] = x;
        C[idx] = x + resid[idx];
      } else if (EPI == EPI_GELU) {
        x += bv;
        float y, dy;
        if (g.gelu_tanh) gelu_tanh_both_f(x, y, dy);
        else gelu_both_f(x, y, dy);
        C[idx] = dy;
        aux[idx] = y;
      } else if (EPI == EPI_DGELU) {
        C[idx] = x * zin[idx];
      } else {
        C[idx] += x;
      }
    }
  }
}

template <int LAY, int EPI>
hipError_t launch(const GemmArgs& g, hipStream_t s) {
  hipLaunchKernelGGL((gemm_f32_kernel<LAY, EPI>), dim3(cdiv(g.N, TN), cdiv(g.M, TM)), dim3(256), 0, s, g);
  return hipGetLastError();
}

template <int LAY>
hipError_t dispatch_epi(Epilogue epi, const GemmArgs& g, hipStream_t s) {
  switch (epi) {
    case EPI_STORE: return launch<LAY, EPI_STORE>(g, s);
    case EPI_BIAS: return launch<LAY, EPI_BIAS>(g, s);
    case EPI_RESID: return launch<LAY, EPI_RESID>(g, s);
    case EPI_GELU: return launch<LAY, EPI_GELU>(g, s);
    case EPI_DGELU: return launch<LAY, EPI_DGELU>(g, s);
    case EPI_F32: return launch<LAY, EPI_F32>(g, s);
    case EPI_F32_ACC: return launch<LAY, EPI_F32_ACC>(g, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t gemm_f32(Layout lay, Epilogue epi, const GemmArgs& g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipErrorInvalidValue;
  switch (lay) {
    case LAY_NN: return dispatch_epi<LAY_NN>(epi, g, s);
    case LAY_NT: return dispatch_epi<LAY_NT>(epi, g, s);
    case LAY_TN: return dispatch_epi<LAY_TN>(epi, g, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace gx
