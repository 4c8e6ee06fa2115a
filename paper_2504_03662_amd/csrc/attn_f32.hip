// fp32 causal attention for the full-precision configuration: one wavefront per query row
// (forward, dQ) or per key row (dK / dV), scores kept in LDS, every sum in fp32 and in a fixed
// order.  Small and exact rather than fast: that configuration is launch-bound.
#include "gx_kernels.h"

namespace gx {
namespace {

// qkv row stride is 3*Hl; head h's Q, K, V start at columns h*dh, Hl + h*dh, 2*Hl + h*dh.
struct HeadView {
  const float* q; const float* k; const float* v;
  int ld;
};
GX_DEVINL HeadView head_view(const float* qkv, int b, int h, int S, int nl, int dh) {
  const int Hl = nl * dh;
  const float* base = qkv + (size_t)b * S * 3 * Hl + h * dh;
  return HeadView{base, base + Hl, base + 2 * Hl, 3 * Hl};
}

// Dropout of the probabilities: keep bits of (sample, head) pair bh, row-major (bit j % 32 of word
// j / 32 of query row i); a null array keeps everything.
struct KeepBits {
  const unsigned* row;   // this pair's [S][wpr] words, or null
  int wpr;
  float scale;           // multiplier of a kept probability
  GX_DEVINL float factor(int i, int j) const {
    if (!row) return 1.0f;
    return ((row[(size_t)i * wpr + (j >> 5)] >> (j & 31)) & 1u) ? scale : 0.0f;
  }
};
GX_DEVINL KeepBits keep_view(const unsigned* rowbits, int wpr, float scale, int b, int h, int S, int nl) {
  return KeepBits{rowbits ? rowbits + ((size_t)b * nl + h) * S * wpr : nullptr, wpr, scale};
}

__global__ void __launch_bounds__(64) attn_fwd_f32_kernel(const float* __restrict__ qkv, float* __restrict__ ctx,
                                                          float* __restrict__ lse, int S, int nl, int dh,
                                                          const unsigned* __restrict__ rowbits, int wpr,
                                                          float keep_scale) {
  extern __shared__ float sc[];          // [S] scores of this row, then probabilities
  const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
  const HeadView hv = head_view(qkv, b, h, S, nl, dh);
  const KeepBits kb = keep_view(rowbits, wpr, keep_scale, b, h, S, nl);
  const float scale = rsqrtf((float)dh);
  const float* qi = hv.q + (size_t)i * hv.ld;
  float mx = -INFINITY;
  for (int j = lane; j <= i; j += 64) {
    const float* kj = hv.k + (size_t)j * hv.ld;
    float s = 0.f;
    for (int d = 0; d < dh; d++) s = fmaf(qi[d], kj[d], s);
    s *= scale;
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  mx = wave_max(mx);
  float sum = 0.f;
  for (int j = lane; j <= i; j += 64) {
    const float p = expf(sc[j] - mx);
    sc[j] = p * kb.factor(i, j);         // the normaliser below is the sum of the undropped values
    sum += p;
  }
  sum = wave_sum(sum);
  __syncthreads();
  const float inv = 1.0f / sum;
  for (int d = lane; d < dh; d += 64) {
    float o = 0.f;
    for (int j = 0; j <= i; j++) o = fmaf(sc[j], hv.v[(size_t)j * hv.ld + d], o);
    ctx[((size_t)b * S + i) * (nl * dh) + h * dh + d] = o * inv;
  }
  if (lane == 0) lse[((size_t)b * nl + h) * S + i] = mx + logf(sum);
}

// per query row: D_i = dO_i . O_i, dS_ij = P_ij (dO_i . V_j - D_i), dQ_i = scale * sum_j dS_ij K_j
__global__ void __launch_bounds__(64) attn_bwd_dq_f32_kernel(const float* __restrict__ qkv,
                                                             const float* __restrict__ ctx,
                                                             const float* __restrict__ dctx,
                                                             const float* __restrict__ lse, float* __restrict__ dsum,
                                                             float* __restrict__ dqkv, int S, int nl, int dh,
                                                             const unsigned* __restrict__ rowbits, int wpr,
                                                             float keep_scale) {
  extern __shared__ float ds[];          // [S]
  const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
  const HeadView hv = head_view(qkv, b, h, S, nl, dh);
  const KeepBits kb = keep_view(rowbits, wpr, keep_scale, b, h, S, nl);
  const int Hl = nl * dh;
  const float scale = rsqrtf((float)dh);
  const float* qi = hv.q + (size_t)i * hv.ld;
  const float* doi = dctx + ((size_t)b * S + i) * Hl + h * dh;
  const float* oi = ctx + ((size_t)b * S + i) * Hl + h * dh;
  float dd = 0.f;
  for (int d = lane; d < dh; d += 64) dd = fmaf(doi[d], oi[d], dd);
  dd = wave_sum(dd);
  const float l = lse[((size_t)b * nl + h) * S + i];
  if (lane == 0) dsum[((size_t)b * nl + h) * S + i] = dd;
  for (int j = lane; j <= i; j += 64) {
    const float* kj = hv.k + (size_t)j * hv.ld;
    const float* vj = hv.v + (size_t)j * hv.ld;
    float s = 0.f, dp = 0.f;
    for (int d = 0; d < dh; d++) { s = fmaf(qi[d], kj[d], s); dp = fmaf(doi[d], vj[d], dp); }
    ds[j] = expf(s * scale - l) * (dp * kb.factor(i, j) - dd);
  }
  __syncthreads();
  float* dq = dqkv + ((size_t)b * S + i) * 3 * Hl + h * dh;
  for (int d = lane; d < dh; d += 64) {
    float a = 0.f;
    for (int j = 0; j <= i; j++) a = fmaf(ds[j], hv.k[(size_t)j * hv.ld + d], a);
    dq[d] = a * scale;
  }
}

// per key row j: dV_j = sum_{i>=j} P_ij dO_i, dK_j = scale * sum_{i>=j} dS_ij Q_i
__global__ void __launch_bounds__(64) attn_bwd_dkv_f32_kernel(const float* __restrict__ qkv,
                                                              const float* __restrict__ dctx,
                                                              const float* __restrict__ lse,
                                                              const float* __restrict__ dsum,
                                                              float* __restrict__ dqkv, int S, int nl, int dh,
                                                              const unsigned* __restrict__ rowbits, int wpr,
                                                              float keep_scale) {
  extern __shared__ float sm[];          // p[S] (as it multiplies V: dropped and rescaled) | ds[S]
  float* pp = sm;
  float* ds = sm + S;
  const int j = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
  const HeadView hv = head_view(qkv, b, h, S, nl, dh);
  const int Hl = nl * dh;
  const float scale = rsqrtf((float)dh);
  const float* kj = hv.k + (size_t)j * hv.ld;
  const float* vj = hv.v + (size_t)j * hv.ld;
  const float* lrow = lse + ((size_t)b * nl + h) * S;
  const float* drow = dsum + ((size_t)b * nl + h) * S;
  const KeepBits kb = keep_view(rowbits, wpr, keep_scale, b, h, S, nl);
  for (int i = j + lane; i < S; i += 64) {
    const float* qi = hv.q + (size_t)i * hv.ld;
    const float* doi = dctx + ((size_t)b * S + i) * Hl + h * dh;
    float s = 0.f, dp = 0.f;
    for (int d = 0; d < dh; d++) { s = fmaf(qi[d], kj[d], s); dp = fmaf(doi[d], vj[d], dp); }
    const float p = expf(s * scale - lrow[i]);
    const float keep = kb.factor(i, j);
    pp[i] = p * keep;
    ds[i] = p * (dp * keep - drow[i]);
  }
  __syncthreads();
  float* dk = dqkv + ((size_t)b * S + j) * 3 * Hl + Hl + h * dh;
  float* dv = dk + Hl;
  for (int d = lane; d < dh; d += 64) {
    float ak = 0.f, av = 0.f;
    for (int i = j; i < S; i++) {
      ak = fmaf(ds[i], hv.q[(size_t)i * hv.ld + d], ak);
      av = fmaf(pp[i], dctx[((size_t)b * S + i) * Hl + h * dh + d], av);
    }
    dk[d] = ak * scale;
    dv[d] = av;
  }
}

}  // namespace

hipError_t attn_fwd_f32(const AttnArgs& a, hipStream_t s) {
  if (a.S > 8192) return hipErrorInvalidValue;
  dim3 grid(a.S, a.nl, a.B);
  hipLaunchKernelGGL(attn_fwd_f32_kernel, grid, dim3(64), a.S * sizeof(float), s, (const float*)a.qkv,
                     (float*)a.ctx, a.lse, a.S, a.nl, a.dh, a.rowbits, a.wpr, a.keep_scale);
  return hipGetLastError();
}

hipError_t attn_bwd_f32(const AttnArgs& a, hipStream_t s) {
  if (a.S > 8192) return hipErrorInvalidValue;
  dim3 grid(a.S, a.nl, a.B);
  hipLaunchKernelGGL(attn_bwd_dq_f32_kernel, grid, dim3(64), a.S * sizeof(float), s, (const float*)a.qkv,
                     (const float*)a.ctx, (const float*)a.dctx, a.lse, a.dsum, (float*)a.dqkv, a.S, a.nl, a.dh, a.rowbits,
                     a.wpr, a.keep_scale);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attn_bwd_dkv_f32_kernel, grid, dim3(64), 2 * a.S * sizeof(float), s, (const float*)a.qkv,
                     (const float*)a.dctx, a.lse, a.dsum, (float*)a.dqkv, a.S, a.nl, a.dh, a.rowbits, a.wpr, a.keep_scale);
  return hipGetLastError();
}

}  // namespace gx
