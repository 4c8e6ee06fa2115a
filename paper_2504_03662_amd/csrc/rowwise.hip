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

constexpr int LN_MAXC = 16;   // most 16 B chunks a lane keeps in registers (one wavefront per row)

// One wavefront per row, the row held in registers (up to MAXC chunks per lane): mean, then
// centred variance, then output.
template <typename T, int MAXC>
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
  float vals[MAXC][V];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < MAXC; i++) {
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
  for (int i = 0; i < MAXC; i++) {
    if (lane + 64 * i < nchunk) {
#pragma unroll
      for (int e = 0; e < V; e++) { const float d = vals[i][e] - mu; q += d * d; }
    }
  }
  const float rs = rsqrtf(wave_sum(q) / (float)cols + eps);
  if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
  T* yr = y + (size_t)row * cols;
#pragma unroll
  for (int i = 0; i < MAXC; i++) {
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

// LayerNorm backward, input gradient: one wavefront per row, the row of dy and x-hat held in
// registers; dx = rstd * (dy g - mean(dy g) - xhat mean(dy g xhat)) (+ residual gradient).
template <typename T, int MAXC>
__global__ void __launch_bounds__(256) ln_bwd_dx_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                        const T* __restrict__ g, const float* __restrict__ mean,
                                                        const float* __restrict__ rstd, const T* __restrict__ resid,
                                                        T* __restrict__ dx, int rows, int cols) {
  constexpr int V = Vec<T>::N;
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int nchunk = cols / V;
  const size_t off = (size_t)row * cols;
  const float mu = mean[row], rs = rstd[row];
  float t[MAXC][V], xh[MAXC][V];
  typename Vec<T>::type rraw[MAXC];          // residual gradient, fetched with the first wave of loads
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int i = 0; i < MAXC; i++) {
    const int c = lane + 64 * i;
    if (c < nchunk) {
      float gv[V];
      load_vec<T>(dy + off + c * V, t[i]);
      load_vec<T>(x + off + c * V, xh[i]);
      if (resid) rraw[i] = *reinterpret_cast<const typename Vec<T>::type*>(resid + off + c * V);
      load_vec<T>(g + c * V, gv);
#pragma unroll
      for (int e = 0; e < V; e++) {
        xh[i][e] = (xh[i][e] - mu) * rs;
        t[i][e] *= gv[e];
        s1 += t[i][e];
        s2 += t[i][e] * xh[i][e];
      }
    }
  }
  const float c1 = wave_sum(s1) / (float)cols, c2 = wave_sum(s2) / (float)cols;
#pragma unroll
  for (int i = 0; i < MAXC; i++) {
    const int c = lane + 64 * i;
    if (c < nchunk) {
      float o[V];
#pragma unroll
      for (int e = 0; e < V; e++) o[e] = rs * (t[i][e] - c1 - xh[i][e] * c2);
      if (resid) {
#pragma unroll
        for (int e = 0; e < V; e++) o[e] += to_f32(rraw[i][e]);
      }
      store_vec<T>(dx + off + c * V, o);
    }
  }
}

// LayerNorm backward, parameter gradients, stage 1: workgroup (bx, by) adds dy * xhat and dy over
// rows [by*rpb, (by+1)*rpb) for 64 column chunks of 16 B.  Its 4 wavefronts take every 4th row and
// combine through LDS in wavefront order; partials go to part[0][by][col], part[1][by][col].
template <typename T>
__global__ void __launch_bounds__(256) ln_bwd_param_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                           const float* __restrict__ mean,
                                                           const float* __restrict__ rstd, int rows, int cols,
                                                           int rows_per_block, float* __restrict__ part) {
  constexpr int V = Vec<T>::N;
  __shared__ float red[2][3][64][V + 1];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane;
  const bool live = c * V < cols;
  const int r0 = blockIdx.y * rows_per_block, r1 = min(rows, r0 + rows_per_block);
  float dg[V], db[V];
#pragma unroll
  for (int e = 0; e < V; e++) { dg[e] = 0.f; db[e] = 0.f; }
  if (live) {
#pragma unroll 4
    for (int r = r0 + w; r < r1; r += 4) {
      float dv[V], xv[V];
      load_vec<T>(dy + (size_t)r * cols + c * V, dv);
      load_vec<T>(x + (size_t)r * cols + c * V, xv);
      const float mu = mean[r], rs = rstd[r];
#pragma unroll
      for (int e = 0; e < V; e++) {
        dg[e] += dv[e] * ((xv[e] - mu) * rs);
        db[e] += dv[e];
      }
    }
  }
  if (w) {
#pragma unroll
    for (int e = 0; e < V; e++) { red[0][w - 1][lane][e] = dg[e]; red[1][w - 1][lane][e] = db[e]; }
  }
  __syncthreads();
  if (w == 0 && live) {
    float* pg = part + (size_t)blockIdx.y * cols + c * V;
    float* pb = part + ((size_t)gridDim.y + blockIdx.y) * cols + c * V;
#pragma unroll
    for (int e = 0; e < V; e++) {
      pg[e] = (dg[e] + red[0][0][lane][e]) + (red[0][1][lane][e] + red[0][2][lane][e]);
      pb[e] = (db[e] + red[1][0][lane][e]) + (red[1][1][lane][e] + red[1][2][lane][e]);
    }
  }
}

// stage 1 of a column sum: workgroup (bx, by) adds rows [by*rpb, (by+1)*rpb) of 64 column chunks of
// 16 B; its 4 wavefronts take every 4th row and combine through LDS in wavefront order.
template <typename T>
__global__ void __launch_bounds__(256) colsum_kernel(const T* __restrict__ a, int rows, int cols, int ld,
                                                     int rows_per_block, float* __restrict__ part) {
  constexpr int V = Vec<T>::N;
  __shared__ float red[3][64][V + 1];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane;
  const bool live = c * V < cols;
  const int r0 = blockIdx.y * rows_per_block, r1 = min(rows, r0 + rows_per_block);
  float acc[V];
#pragma unroll
  for (int e = 0; e < V; e++) acc[e] = 0.f;
  if (live) {
#pragma unroll 8
    for (int r = r0 + w; r < r1; r += 4) {
      float v[V];
      load_vec<T>(a + (size_t)r * ld + c * V, v);
#pragma unroll
      for (int e = 0; e < V; e++) acc[e] += v[e];
    }
  }
  if (w) {
#pragma unroll
    for (int e = 0; e < V; e++) red[w - 1][lane][e] = acc[e];
  }
  __syncthreads();
  if (w == 0 && live) {
    float* p = part + (size_t)blockIdx.y * cols + c * V;
#pragma unroll
    for (int e = 0; e < V; e++) p[e] = (acc[e] + red[0][lane][e]) + (red[1][lane][e] + red[2][lane][e]);
  }
}

// stage 2: out[c] (=|+=) sum over blocks.  A workgroup owns 64 columns; its 4 wavefronts take
// every 4th partial row, then combine through LDS in wavefront order (a fixed summation tree).
__global__ void __launch_bounds__(256) colsum_finish_kernel(const float* __restrict__ part, int nblk, int cols,
                                                            float* __restrict__ out, int accumulate) {
  __shared__ float red[4][64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane;
  float s = 0.f;
  if (c < cols) {
#pragma unroll 8
    for (int b = w; b < nblk; b += 4) s += part[(size_t)b * cols + c];
  }
  red[w][lane] = s;
  __syncthreads();
  if (w == 0 && c < cols) {
    const float t = (red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane]);
    out[c] = accumulate ? out[c] + t : t;
  }
}

}  // namespace

int ln_bwd_blocks(int rows) { return rows < 2048 ? cdiv(rows, 16) : 128; }
int colsum_blocks(int rows) { return rows < 2048 ? cdiv(rows, 16) : 128; }

hipError_t ln_fwd(bool is_bf16, const void* x, const void* g, const void* b, void* y, float* mean, float* rstd,
                  int rows, int cols, float eps, hipStream_t s) {
  const int vec = is_bf16 ? 8 : 4;
  if (rows <= 0 || cols <= 0 || cols % vec || cols / vec > 64 * LN_MAXC) return hipErrorInvalidValue;
  dim3 grid(cdiv(rows, 4)), block(256);
  const int per_lane = cdiv(cols / vec, 64);
#define GX_LN_FWD(T, C)                                                                                          \
  hipLaunchKernelGGL((ln_fwd_kernel<T, C>), grid, block, 0, s, (const T*)x, (const T*)g, (const T*)b, (T*)y, mean, \
                     rstd, rows, cols, eps)
  if (is_bf16) {
    if (per_lane <= 4) GX_LN_FWD(bf16, 4); else if (per_lane <= 8) GX_LN_FWD(bf16, 8); else GX_LN_FWD(bf16, 16);
  } else {
    if (per_lane <= 4) GX_LN_FWD(float, 4); else if (per_lane <= 8) GX_LN_FWD(float, 8); else GX_LN_FWD(float, 16);
  }
#undef GX_LN_FWD
  return hipGetLastError();
}

hipError_t ln_bwd_dx(bool is_bf16, const void* dy, const void* x, const void* g, const float* mean,
                     const float* rstd, const void* resid, void* dx, int rows, int cols, hipStream_t s) {
  const int vec = is_bf16 ? 8 : 4;
  if (rows <= 0 || cols <= 0 || cols % vec || cols / vec > 64 * LN_MAXC) return hipErrorInvalidValue;
  dim3 gdx(cdiv(rows, 4)), block(256);
  const int per_lane = cdiv(cols / vec, 64);
#define GX_LN_DX(T, C)                                                                                            \
  hipLaunchKernelGGL((ln_bwd_dx_kernel<T, C>), gdx, block, 0, s, (const T*)dy, (const T*)x, (const T*)g, mean, rstd, \
                     (const T*)resid, (T*)dx, rows, cols)
  if (is_bf16) {
    if (per_lane <= 4) GX_LN_DX(bf16, 4); else if (per_lane <= 8) GX_LN_DX(bf16, 8); else GX_LN_DX(bf16, 16);
  } else {
    if (per_lane <= 4) GX_LN_DX(float, 4); else if (per_lane <= 8) GX_LN_DX(float, 8); else GX_LN_DX(float, 16);
  }
#undef GX_LN_DX
  return hipGetLastError();
}

hipError_t ln_bwd_params(bool is_bf16, const void* dy, const void* x, const float* mean, const float* rstd,
                         float* part, int rows, int cols, float* dg, float* db, bool accumulate, hipStream_t s) {
  const int vec = is_bf16 ? 8 : 4;
  if (rows <= 0 || cols <= 0 || cols % vec) return hipErrorInvalidValue;
  const int nblk = ln_bwd_blocks(rows);
  const int rpb = cdiv(rows, nblk);
  dim3 gpar(cdiv(cols / vec, 64), nblk), block(256);
  if (is_bf16)
    hipLaunchKernelGGL(ln_bwd_param_kernel<bf16>, gpar, block, 0, s, (const bf16*)dy, (const bf16*)x, mean, rstd, rows,
                       cols, rpb, part);
  else
    hipLaunchKernelGGL(ln_bwd_param_kernel<float>, gpar, block, 0, s, (const float*)dy, (const float*)x, mean, rstd,
                       rows, cols, rpb, part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  e = colsum_finish(part, nblk, cols, dg, accumulate, s);
  if (e != hipSuccess) return e;
  return colsum_finish(part + (size_t)nblk * cols, nblk, cols, db, accumulate, s);
}

hipError_t colsum_finish(const float* part, int nblk, int cols, float* out, bool accumulate, hipStream_t s) {
  hipLaunchKernelGGL(colsum_finish_kernel, dim3(cdiv(cols, 64)), dim3(256), 0, s, part, nblk, cols, out,
                     accumulate ? 1 : 0);
  return hipGetLastError();
}

hipError_t colsum(bool is_bf16, const void* a, int rows, int cols, int ld, float* part, float* out, bool accumulate,
                  hipStream_t s) {
  const int vec = is_bf16 ? 8 : 4;
  if (rows <= 0 || cols <= 0 || cols % vec || ld % vec) return hipErrorInvalidValue;
  const int nblk = colsum_blocks(rows);
  const int rpb = cdiv(rows, nblk);
  dim3 grid(cdiv(cols / vec, 64), nblk), block(256);
  if (is_bf16)
    hipLaunchKernelGGL(colsum_kernel<bf16>, grid, block, 0, s, (const bf16*)a, rows, cols, ld, rpb, part);
  else
    hipLaunchKernelGGL(colsum_kernel<float>, grid, block, 0, s, (const float*)a, rows, cols, ld, rpb, part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return colsum_finish(part, nblk, cols, out, accumulate, s);
}

}  // namespace gx
