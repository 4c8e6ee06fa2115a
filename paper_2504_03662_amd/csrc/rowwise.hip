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

// LayerNorm backward in one pass over dy and x: input gradient
//   dx = rstd * (dy g - mean(dy g) - xhat mean(dy g xhat)) (+ residual gradient)
// and, from the same registers, the per-workgroup partial column sums that the parameter and bias
// gradients need: sum dy * xhat (gain), sum dy (bias) and, with NSUM = 4, sum resid and sum dx (the
// bias gradients of the row-parallel products on either side of the LayerNorm, whose upstream
// gradients are exactly these two tensors).
// A workgroup of 8 wavefronts; a row is shared by G of them (CPT chunks of 16 B per lane), the
// 8 / G row groups each take R rows per step; the next step's rows are fetched before this step's
// are worked on, so loads, arithmetic and stores overlap.  Row sums cross the G wavefronts through
// LDS (one barrier per step, double-buffered by step parity).
// Every row group keeps its own column accumulators and writes its own partial row:
// part[a][blockIdx.x * (8 / G) + group][cols] for a < NSUM.  Fixed order throughout.
template <typename T, int G, int CPT, int NSUM>
__global__ void __launch_bounds__(512) ln_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                     const T* __restrict__ g, const float* __restrict__ mean,
                                                     const float* __restrict__ rstd, const T* __restrict__ resid,
                                                     T* __restrict__ dx, int rows, int cols, float* __restrict__ part) {
  constexpr int V = Vec<T>::N;
  constexpr int NG = 8 / G, R = 4 / CPT;
  typedef typename Vec<T>::type Raw;
  __shared__ float red[2][NG][R][G][2];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int grp = wave / G, wg = wave % G;
  const int nchunk = cols / V;
  const bool has_resid = (NSUM == 4) || resid != nullptr;
  bool live[CPT];
  int col[CPT];
  float gv[CPT][V];
#pragma unroll
  for (int i = 0; i < CPT; i++) {
    const int c = wg * 64 + lane + 64 * G * i;
    live[i] = c < nchunk;
    col[i] = c * V;
#pragma unroll
    for (int e = 0; e < V; e++) gv[i][e] = 0.f;
    if (live[i]) load_vec<T>(g + col[i], gv[i]);
  }
  float acc[NSUM][CPT][V];
#pragma unroll
  for (int a = 0; a < NSUM; a++)
#pragma unroll
    for (int i = 0; i < CPT; i++)
#pragma unroll
      for (int e = 0; e < V; e++) acc[a][i][e] = 0.f;
  const float inv_cols = 1.0f / (float)cols;

  // one step's rows of this row group, as they come from memory
  struct Step {
    Raw dyr[R][CPT], xr[R][CPT], rr[R][CPT];
    float mu[R], rs[R];
  };
  auto fetch = [&](Step& st, int base) {
    const int r0 = base + grp * R;
#pragma unroll
    for (int j = 0; j < R; j++) {
      const int row = r0 + j;
      const bool ok = row < rows;
      st.mu[j] = ok ? mean[row] : 0.f;
      st.rs[j] = ok ? rstd[row] : 0.f;
#pragma unroll
      for (int i = 0; i < CPT; i++) {
        Raw z;
#pragma unroll
        for (int e = 0; e < V; e++) z[e] = from_f32<T>(0.f);
        st.dyr[j][i] = z;
        st.xr[j][i] = z;
        st.rr[j][i] = z;
        if (ok && live[i]) {
          const size_t off = (size_t)row * cols + col[i];
          st.dyr[j][i] = *reinterpret_cast<const Raw*>(dy + off);
          st.xr[j][i] = *reinterpret_cast<const Raw*>(x + off);
          if (has_resid) st.rr[j][i] = *reinterpret_cast<const Raw*>(resid + off);
        }
      }
    }
  };
  auto process = [&](Step& st, int base, int par) {
    const int r0 = base + grp * R;
    // row sums of dy g and of dy g xhat
#pragma unroll
    for (int j = 0; j < R; j++) {
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int i = 0; i < CPT; i++)
#pragma unroll
        for (int e = 0; e < V; e++) {
          const float t = to_f32(st.dyr[j][i][e]) * gv[i][e];
          s1 += t;
          s2 += t * ((to_f32(st.xr[j][i][e]) - st.mu[j]) * st.rs[j]);
        }
      s1 = wave_sum(s1);
      s2 = wave_sum(s2);
      if (lane == 0) {
        red[par][grp][j][wg][0] = s1;
        red[par][grp][j][wg][1] = s2;
      }
    }
    __syncthreads();
    // the second walk starts again from the rows as loaded: keeping the first walk's products
    // alive across the barrier instead would cost more registers than the two steps in flight
#pragma unroll
    for (int j = 0; j < R; j++)
#pragma unroll
      for (int i = 0; i < CPT; i++) {
        asm volatile("" : "+v"(st.dyr[j][i]));
        asm volatile("" : "+v"(st.xr[j][i]));
      }
#pragma unroll
    for (int j = 0; j < R; j++) {
      const int row = r0 + j;
      if (row >= rows) continue;
      float c1 = 0.f, c2 = 0.f;
#pragma unroll
      for (int w = 0; w < G; w++) {
        c1 += red[par][grp][j][w][0];
        c2 += red[par][grp][j][w][1];
      }
      c1 *= inv_cols;
      c2 *= inv_cols;
#pragma unroll
      for (int i = 0; i < CPT; i++) {
        if (!live[i]) continue;
        Raw o;
#pragma unroll
        for (int e = 0; e < V; e++) {
          const float d = to_f32(st.dyr[j][i][e]);
          const float xh = (to_f32(st.xr[j][i][e]) - st.mu[j]) * st.rs[j];
          float v = st.rs[j] * (d * gv[i][e] - c1 - xh * c2);
          acc[0][i][e] += d * xh;
          acc[1][i][e] += d;
          if (has_resid) v += to_f32(st.rr[j][i][e]);
          o[e] = from_f32<T>(v);
          if (NSUM == 4) {
            acc[2][i][e] += to_f32(st.rr[j][i][e]);
            acc[3][i][e] += to_f32(o[e]);          // the value the consumers of dx read
          }
        }
        *reinterpret_cast<Raw*>(dx + (size_t)row * cols + col[i]) = o;
      }
    }
  };
  // two steps in registers: the next step's rows travel while this step's are worked on.  The LDS
  // exchange alternates with the step parity, so one barrier per step suffices: a wavefront can
  // only reach the write of step k + 2 after every wavefront has passed the barrier of step k + 1,
  // i.e. has finished reading step k's sums.
  const int stride = gridDim.x * NG * R;
  Step s0, s1;
  int base = blockIdx.x * NG * R;
  if (base < rows) fetch(s0, base);
  while (base < rows) {
    if (base + stride < rows) fetch(s1, base + stride);
    process(s0, base, 0);
    base += stride;
    if (base >= rows) break;
    if (base + stride < rows) fetch(s0, base + stride);
    process(s1, base, 1);
    base += stride;
  }
  const size_t nblk = (size_t)gridDim.x * NG, blk = (size_t)blockIdx.x * NG + grp;
#pragma unroll
  for (int a = 0; a < NSUM; a++)
#pragma unroll
    for (int i = 0; i < CPT; i++) {
      if (!live[i]) continue;
      float* p = part + (a * nblk + blk) * cols + col[i];
#pragma unroll
      for (int e = 0; e < V; e += 4)
        *reinterpret_cast<f32x4*>(p + e) = f32x4{acc[a][i][e], acc[a][i][e + 1], acc[a][i][e + 2], acc[a][i][e + 3]};
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

// stage 2 of every column reduction of a pass, in one launch: segment s sums nblk partial rows of
// `cols` floats into out (=|+=).  A workgroup of 16 wavefronts owns 256 columns of one segment
// (16 B per lane); its wavefronts take every 16th partial row, then combine through LDS in
// wavefront order (a fixed summation tree).
__global__ void __launch_bounds__(1024) colsum_finish_kernel(FinishArgs a) {
  __shared__ f32x4 red[16][64];
  int si = 0;
  while (si + 1 < a.nseg && (int)blockIdx.x >= a.seg[si + 1].wg0) si++;
  const FinishSeg sg = a.seg[si];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = (((int)blockIdx.x - sg.wg0) * 64 + lane) * 4;
  f32x4 s = {0.f, 0.f, 0.f, 0.f};
  if (c < sg.cols) {
#pragma unroll 4
    for (int b = w; b < sg.nblk; b += 16) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(sg.part + (size_t)b * sg.cols + c);
      s = f32x4{s[0] + v[0], s[1] + v[1], s[2] + v[2], s[3] + v[3]};
    }
  }
  red[w][lane] = s;
  __syncthreads();
  if (w == 0 && c < sg.cols) {
    f32x4 t = red[0][lane];
#pragma unroll
    for (int k = 1; k < 16; k++) {
      const f32x4 v = red[k][lane];
      t = f32x4{t[0] + v[0], t[1] + v[1], t[2] + v[2], t[3] + v[3]};
    }
    f32x4* o = reinterpret_cast<f32x4*>(sg.out + c);
    if (sg.accumulate) {
      const f32x4 old = *o;
      t = f32x4{t[0] + old[0], t[1] + old[1], t[2] + old[2], t[3] + old[3]};
    }
    *o = t;
  }
}

// shape of the fused LayerNorm-backward launch for a row length: wavefronts per row, chunks per lane
void ln_bwd_shape(int nchunk, int& G, int& CPT) {
  G = nchunk >= 512 ? 8 : nchunk >= 256 ? 4 : nchunk >= 128 ? 2 : 1;
  CPT = cdiv(nchunk, 64 * G);
}

}  // namespace

int colsum_blocks(int rows) { return rows < 2048 ? cdiv(rows, 16) : 128; }

int ln_bwd_blocks(bool is_bf16, int rows, int cols) {
  int G, CPT;
  ln_bwd_shape(cols / (is_bf16 ? 8 : 4), G, CPT);
  const int per_step = (8 / G) * (4 / CPT);            // rows a workgroup takes per step
  // one workgroup per compute unit, but at least four steps each: every row group leaves a partial
  // row of `cols` sums, which should stay a small fraction of the rows read
  const int want = cdiv(rows, 4 * per_step);
  const int wgs = want < 256 ? want : 256;
  return wgs * (8 / G);
}

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

hipError_t ln_bwd(bool is_bf16, const void* dy, const void* x, const void* g, const float* mean, const float* rstd,
                  const void* resid, void* dx, int rows, int cols, int nsum, float* part, hipStream_t s) {
  const int vec = is_bf16 ? 8 : 4;
  if (rows <= 0 || cols <= 0 || cols % vec || cols / vec > 64 * LN_MAXC) return hipErrorInvalidValue;
  if ((nsum != 2 && nsum != 4) || (nsum == 4 && !resid)) return hipErrorInvalidValue;
  int G, CPT;
  ln_bwd_shape(cols / vec, G, CPT);
  if (CPT > 2) return hipErrorInvalidValue;
  const int wgs = ln_bwd_blocks(is_bf16, rows, cols) / (8 / G);
#define GX_LN_BWD(T, GG, CC, NN)                                                                                  \
  hipLaunchKernelGGL((ln_bwd_kernel<T, GG, CC, NN>), dim3(wgs), dim3(512), 0, s, (const T*)dy, (const T*)x,        \
                     (const T*)g, mean, rstd, (const T*)resid, (T*)dx, rows, cols, part)
#define GX_LN_BWD_N(T, GG, CC)              \
  do {                                      \
    if (nsum == 4) GX_LN_BWD(T, GG, CC, 4); \
    else GX_LN_BWD(T, GG, CC, 2);           \
  } while (0)
#define GX_LN_BWD_C(T, GG)            \
  do {                                \
    if (CPT == 1) GX_LN_BWD_N(T, GG, 1); \
    else GX_LN_BWD_N(T, GG, 2);       \
  } while (0)
#define GX_LN_BWD_G(T)                  \
  do {                                  \
    if (G == 8) GX_LN_BWD_C(T, 8);      \
    else if (G == 4) GX_LN_BWD_C(T, 4); \
    else if (G == 2) GX_LN_BWD_C(T, 2); \
    else GX_LN_BWD_C(T, 1);             \
  } while (0)
  if (is_bf16) GX_LN_BWD_G(bf16);
  else GX_LN_BWD_G(float);
#undef GX_LN_BWD_G
#undef GX_LN_BWD_C
#undef GX_LN_BWD_N
#undef GX_LN_BWD
  return hipGetLastError();
}

hipError_t colsum_finish(const FinishSeg* segs, int nseg, hipStream_t s) {
  if (nseg <= 0) return hipSuccess;
  if (nseg > FINISH_MAX) return hipErrorInvalidValue;
  FinishArgs a;
  int wg = 0;
  for (int i = 0; i < nseg; i++) {
    if (segs[i].nblk <= 0 || segs[i].cols <= 0 || (segs[i].cols & 3)) return hipErrorInvalidValue;
    a.seg[i] = segs[i];
    a.seg[i].wg0 = wg;
    wg += cdiv(segs[i].cols, 256);
  }
  a.nseg = nseg;
  hipLaunchKernelGGL(colsum_finish_kernel, dim3(wg), dim3(1024), 0, s, a);
  return hipGetLastError();
}

hipError_t colsum_partial(bool is_bf16, const void* a, int rows, int cols, int ld, float* part, hipStream_t s) {
  const int vec = is_bf16 ? 8 : 4;
  if (rows <= 0 || cols <= 0 || cols % vec || ld % vec) return hipErrorInvalidValue;
  const int nblk = colsum_blocks(rows);
  const int rpb = cdiv(rows, nblk);
  dim3 grid(cdiv(cols / vec, 64), nblk), block(256);
  if (is_bf16)
    hipLaunchKernelGGL(colsum_kernel<bf16>, grid, block, 0, s, (const bf16*)a, rows, cols, ld, rpb, part);
  else
    hipLaunchKernelGGL(colsum_kernel<float>, grid, block, 0, s, (const float*)a, rows, cols, ld, rpb, part);
  return hipGetLastError();
}

}  // namespace gx
