// Bandwidth-bound kernels of the block: LayerNorm forward / backward and fixed-order column sums
// (bias and LayerNorm parameter gradients).  All loads and stores are 16 B per lane and
// contiguous across a wavefront; reductions use wavefront shuffles and a two-stage, fixed-order
// scheme (no atomics), so results are bitwise reproducible.
#include "gx_kernels.h"

namespace gx {
namespace {

template <typename T> struct Vec;
template <> struct Vec<float> { static constexpr int N = 4; typedef f32x4 type; };
template <> struct Vec<bf16> { static constexpr int N = 8; typedef bf16x8 type; };

template <typename T> GX_DEVINL void load_vec(const T* p, float (&out)[Vec<T>::N]) {
  typename Vec<T>::type v = *reinterpret_cast<const typename Vec<T>::type*>(p);
#pragma unroll
  for (int i = 0; i < Vec<T>::N; i++) out[i] = to_f32(v[i]);
}
template <typename T> GX_DEVINL void store_vec(T* p, const float (&in)[Vec<T>::N]) {
  typename Vec<T>::type v;
#pragma unroll
  for (int i = 0; i < Vec<T>::N; i++) v[i] = from_f32<T>(in[i]);
  *reinterpret_cast<typename Vec<T>::type*>(p) = v;
}

constexpr int LN_MAXC = 16;   // 16 B chunks a lane keeps in registers (one wavefront per row)

// One wavefront per row, the row held in registers: mean, then centred variance, then output.
template <typename T>
__global__ void __launch_bounds__(256) ln_fwd_kernel(const T* __restrict__ x, const T* __restrict__ g,
                                                     const T* __restrict__ b, T* __restrict__ y,
                                                     float* __restrict__ mean, float* __restrict__ rstd, int rows,
                                                     int cols, float eps) {
  constexpr int V = Vec<T>::N;
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int nchunk = cols / V;
  const T* xr = x + (size_t)row * cols;
  float vals[LN_MAXC][V];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < LN_MAXC; i++) {
    const int c = lane + 64 * i;
    if (c < nchunk) {
      load_vec<T>(xr + c * V, vals[i]);
#pragma unroll
      for (int e = 0; e < V; e++) s += vals[i][e];
    }
  }
  const float mu = wave_sum(s) / (float)cols;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < LN_MAXC; i++) {
    if (lane + 64 * i < nchunk) {
#pragma unroll
      for (int e = 0; e < V; e++) { const float d = vals[i][e] - mu; q += d * d; }
    }
  }
  const float rs = rsqrtf(wave_sum(q) / (float)cols + eps);
  if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
  T* yr = y + (size_t)row * cols;
#pragma unroll
  for (int i = 0; i < LN_MAXC; i++) {
    const int c = lane + 64 * i;
    if (c < nchunk) {
      float gv[V], bv[V], o[V];
      load_vec<T>(g + c * V, gv);
      load_vec<T>(b + c * V, bv);
#pragma unroll
      for (int e = 0; e < V; e++) o[e] = gv[e] * ((vals[i][e] - mu) * rs) + bv[e];
      store_vec<T>(yr + c * V, o);
    }
  }
}

constexpr int LNB_MAXC = 4;   // chunks per thread in the backward kernel (256 threads per row)

// A workgroup walks a block of rows with a fixed thread -> column mapping, so the column sums
// for dg / db stay in registers; the two per-row means go through a wavefront + LDS reduction.
template <typename T>
__global__ void __launch_bounds__(256) ln_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                     const T* __restrict__ g, const float* __restrict__ mean,
                                                     const float* __restrict__ rstd, const T* __restrict__ resid,
                                                     T* __restrict__ dx, float* __restrict__ part, int rows, int cols,
                                                     int rows_per_block) {
  constexpr int V = Vec<T>::N;
  __shared__ float red[2][4][2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nchunk = cols / V;
  float gv[LNB_MAXC][V], dg[LNB_MAXC][V], db[LNB_MAXC][V];
#pragma unroll
  for (int i = 0; i < LNB_MAXC; i++) {
    const int c = tid + 256 * i;
#pragma unroll
    for (int e = 0; e < V; e++) { dg[i][e] = 0.f; db[i][e] = 0.f; gv[i][e] = 0.f; }
    if (c < nchunk) load_vec<T>(g + c * V, gv[i]);
  }
  const int r0 = blockIdx.x * rows_per_block;
  const int r1 = min(rows, r0 + rows_per_block);
  for (int row = r0; row < r1; row++) {
    const float mu = mean[row], rs = rstd[row];
    const size_t off = (size_t)row * cols;
    float dyv[LNB_MAXC][V], xh[LNB_MAXC][V];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < LNB_MAXC; i++) {
      const int c = tid + 256 * i;
      if (c < nchunk) {
        load_vec<T>(dy + off + c * V, dyv[i]);
        load_vec<T>(x + off + c * V, xh[i]);
#pragma unroll
        for (int e = 0; e < V; e++) {
          xh[i][e] = (xh[i][e] - mu) * rs;
          const float t = dyv[i][e] * gv[i][e];
          s1 += t;
          s2 += t * xh[i][e];
          dg[i][e] += dyv[i][e] * xh[i][e];
          db[i][e] += dyv[i][e];
        }
      }
    }
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    const int slot = row & 1;
    if (lane == 0) { red[slot][wave][0] = s1; red[slot][wave][1] = s2; }
    __syncthreads();
    const float c1 = (red[slot][0][0] + red[slot][1][0] + red[slot][2][0] + red[slot][3][0]) / (float)cols;
    const float c2 = (red[slot][0][1] + red[slot][1][1] + red[slot][2][1] + red[slot][3][1]) / (float)cols;
#pragma unroll
    for (int i = 0; i < LNB_MAXC; i++) {
      const int c = tid + 256 * i;
      if (c < nchunk) {
        float o[V];
#pragma unroll
        for (int e = 0; e < V; e++) o[e] = rs * (dyv[i][e] * gv[i][e] - c1 - xh[i][e] * c2);
        if (resid) {
          float rv[V];
          load_vec<T>(resid + off + c * V, rv);
#pragma unroll
          for (int e = 0; e < V; e++) o[e] += rv[e];
        }
        store_vec<T>(dx + off + c * V, o);
      }
    }
  }
  float* pg = part + (size_t)blockIdx.x * cols;
  float* pb = part + ((size_t)gridDim.x + blockIdx.x) * cols;
#pragma unroll
  for (int i = 0; i < LNB_MAXC; i++) {
    const int c = tid + 256 * i;
    if (c < nchunk) {
#pragma unroll
      for (int e = 0; e < V; e++) { pg[c * V + e] = dg[i][e]; pb[c * V + e] = db[i][e]; }
    }
  }
}

// stage 1 of a column sum: block (bx, by) adds rows [by*rpb, (by+1)*rpb) of 16 B column chunks
template <typename T>
__global__ void __launch_bounds__(256) colsum_kernel(const T* __restrict__ a, int rows, int cols, int ld,
                                                     int rows_per_block, float* __restrict__ part) {
  constexpr int V = Vec<T>::N;
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c * V >= cols) return;
  const int r0 = blockIdx.y * rows_per_block, r1 = min(rows, r0 + rows_per_block);
  float acc[V];
#pragma unroll
  for (int e = 0; e < V; e++) acc[e] = 0.f;
  for (int r = r0; r < r1; r++) {
    float v[V];
    load_vec<T>(a + (size_t)r * ld + c * V, v);
#pragma unroll
    for (int e = 0; e < V; e++) acc[e] += v[e];
  }
  float* p = part + (size_t)blockIdx.y * cols + c * V;
#pragma unroll
  for (int e = 0; e < V; e++) p[e] = acc[e];
}

// stage 2: out[c] (=|+=) sum over blocks, in block order
__global__ void __launch_bounds__(256) colsum_finish_kernel(const float* __restrict__ part, int nblk, int cols,
                                                            float* __restrict__ out, int accumulate) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= cols) return;
  float s = 0.f;
  for (int b = 0; b < nblk; b++) s += part[(size_t)b * cols + c];
  out[c] = accumulate ? out[c] + s : s;
}

}  // namespace

int ln_bwd_blocks(int rows) { return rows < 1024 ? cdiv(rows, 4) : 256; }
int colsum_blocks(int rows) { return rows < 512 ? cdiv(rows, 8) : 64; }

hipError_t ln_fwd(bool is_bf16, const void* x, const void* g, const void* b, void* y, float* mean, float* rstd,
                  int rows, int cols, float eps, hipStream_t s) {
  const int vec = is_bf16 ? 8 : 4;
  if (rows <= 0 || cols <= 0 || cols % vec || cols / vec > 64 * LN_MAXC) return hipErrorInvalidValue;
  dim3 grid(cdiv(rows, 4)), block(256);
  if (is_bf16)
    hipLaunchKernelGGL(ln_fwd_kernel<bf16>, grid, block, 0, s, (const bf16*)x, (const bf16*)g, (const bf16*)b,
                       (bf16*)y, mean, rstd, rows, cols, eps);
  else
    hipLaunchKernelGGL(ln_fwd_kernel<float>, grid, block, 0, s, (const float*)x, (const float*)g, (const float*)b,
                       (float*)y, mean, rstd, rows, cols, eps);
  return hipGetLastError();
}

hipError_t ln_bwd(bool is_bf16, const void* dy, const void* x, const void* g, const float* mean, const float* rstd,
                  const void* resid, void* dx, float* part, int rows, int cols, hipStream_t s) {
  const int vec = is_bf16 ? 8 : 4;
  if (rows <= 0 || cols <= 0 || cols % vec || cols / vec > 256 * LNB_MAXC) return hipErrorInvalidValue;
  const int nblk = ln_bwd_blocks(rows);
  const int rpb = cdiv(rows, nblk);
  dim3 grid(nblk), block(256);
  if (is_bf16)
    hipLaunchKernelGGL(ln_bwd_kernel<bf16>, grid, block, 0, s, (const bf16*)dy, (const bf16*)x, (const bf16*)g, mean,
                       rstd, (const bf16*)resid, (bf16*)dx, part, rows, cols, rpb);
  else
    hipLaunchKernelGGL(ln_bwd_kernel<float>, grid, block, 0, s, (const float*)dy, (const float*)x, (const float*)g,
                       mean, rstd, (const float*)resid, (float*)dx, part, rows, cols, rpb);
  return hipGetLastError();
}

hipError_t colsum_finish(const float* part, int nblk, int cols, float* out, bool accumulate, hipStream_t s) {
  hipLaunchKernelGGL(colsum_finish_kernel, dim3(cdiv(cols, 256)), dim3(256), 0, s, part, nblk, cols, out,
                     accumulate ? 1 : 0);
  return hipGetLastError();
}

hipError_t colsum(bool is_bf16, const void* a, int rows, int cols, int ld, float* part, float* out, bool accumulate,
                  hipStream_t s) {
  const int vec = is_bf16 ? 8 : 4;
  if (rows <= 0 || cols <= 0 || cols % vec || ld % vec) return hipErrorInvalidValue;
  const int nblk = colsum_blocks(rows);
  const int rpb = cdiv(rows, nblk);
  dim3 grid(cdiv(cols / vec, 256), nblk), block(256);
  if (is_bf16)
    hipLaunchKernelGGL(colsum_kernel<bf16>, grid, block, 0, s, (const bf16*)a, rows, cols, ld, rpb, part);
  else
    hipLaunchKernelGGL(colsum_kernel<float>, grid, block, 0, s, (const float*)a, rows, cols, ld, rpb, part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return colsum_finish(part, nblk, cols, out, accumulate, s);
}

}  // namespace gx
