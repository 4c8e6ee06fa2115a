// Dropout masks for the dropout variant of the block: a counter-based generator (Philox4x32 with
// 10 rounds, Salmon et al., SC 2011) turned into keep bits.
//
// Attention probabilities: the masks are materialised once per pass as bit arrays, because the
// attention kernels hold the score tile in MFMA accumulator layouts (a lane of the forward and dQ
// kernels owns 16 keys of one query, a lane of the dK/dV kernel 16 queries of one key) and
// regenerating 16-byte counters in those layouts would cost several generator calls per element.
// One wavefront covers 64 queries and 128 keys; per group of 16 keys every lane makes one
// generator call for its query, keeps the 16 bits for the row-major array and contributes them to
// 16 wavefront ballots, each of which is the column-major word pair "64 queries of one key".
//   rowbits[(bh * S + i) * wpr + j / 32]  bit j % 32  = keep(i, j)        (forward, dQ)
//   colbits[(bh * S + j) * wpr + i / 32]  bit i % 32  = keep(i, j)        (dK / dV)
// wpr = 2 * ceil(S / 64) words per row.  Only words that a causal kernel can touch are written:
// keys below 64 * (i / 64 + 1).
//
// Outputs of the two halves: one pass, out = residual + keep * scale * in (forward) or
// out = keep * scale * in (backward), one generator call per 16 consecutive columns.
#include "gx_kernels.h"

namespace gx {
namespace {

struct Philox {
  unsigned x[4];
};

GX_DEVINL Philox philox4x32_10(unsigned c0, unsigned c1, unsigned c2, unsigned c3, unsigned k0, unsigned k1) {
  constexpr unsigned M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; r++) {
    const unsigned hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
    const unsigned hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
    k0 += W0;
    k1 += W1;
  }
  return Philox{{c0, c1, c2, c3}};
}

// bit e of the result = (byte e of the 16 random bytes >= t), i.e. element e is kept
GX_DEVINL unsigned keep_bits16(const Philox& r, unsigned t) {
  unsigned bits = 0;
#pragma unroll
  for (int w = 0; w < 4; w++)
#pragma unroll
    for (int b = 0; b < 4; b++) bits |= (((r.x[w] >> (8 * b)) & 0xFFu) >= t ? 1u : 0u) << (4 * w + b);
  return bits;
}

// One wavefront: 64 queries x MASK_GROUPS groups of 16 keys.
constexpr int MASK_GROUPS = 8;

__global__ void __launch_bounds__(64) attn_mask_kernel(unsigned* __restrict__ rowbits, unsigned* __restrict__ colbits,
                                                       int S, int wpr, int nchunk, int heads, int head0, unsigned k0,
                                                       unsigned k1, unsigned t) {
  const int lane = threadIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int blk = blockIdx.x / nchunk, chunk = blockIdx.x % nchunk;
  const int nl = gridDim.y;
  const int groups = min(4 * (blk + 1), 2 * wpr);      // 16-key groups up to the end of the diagonal tile
  const int jg0 = chunk * MASK_GROUPS;
  if (jg0 >= groups) return;                           // wavefront-uniform
  const int jg1 = min(jg0 + MASK_GROUPS, groups);      // jg0, jg1 and groups are even
  const int i = 64 * blk + lane;
  const size_t bh = (size_t)b * nl + h;
  const unsigned c2 = (unsigned)(b * heads + head0 + h);
  unsigned word = 0;
  for (int jg = jg0; jg < jg1; jg++) {
    const unsigned kb = keep_bits16(philox4x32_10((unsigned)i, (unsigned)jg, c2, 1u, k0, k1), t);
    word |= kb << (16 * (jg & 1));
    if (jg & 1) {
      if (i < S) rowbits[(bh * S + i) * wpr + (jg >> 1)] = word;
      word = 0;
    }
    if (colbits) {
      unsigned long long mine = 0;
#pragma unroll
      for (int k = 0; k < 16; k++) {
        const unsigned long long col = __builtin_amdgcn_ballot_w64((kb >> k) & 1u);
        if (lane == k) mine = col;
      }
      const int j = 16 * jg + lane;
      if (lane < 16 && j < S)
        *reinterpret_cast<unsigned long long*>(colbits + (bh * S + j) * wpr + 2 * blk) = mine;
    }
  }
}

template <typename T>
struct Vec16B;                       // 16 bytes of T
template <>
struct Vec16B<float> {
  using type = f32x4;
  static constexpr int N = 4;
};
template <>
struct Vec16B<bf16> {
  using type = bf16x8;
  static constexpr int N = 8;
};

// one lane: the 16 consecutive columns of one generator call, moved as 16-byte vectors
template <typename T>
__global__ void __launch_bounds__(256) dropout_rows_kernel(const T* __restrict__ in, const T* __restrict__ resid,
                                                           T* __restrict__ out, int rows, int cols, int groups,
                                                           unsigned stream, unsigned k0, unsigned k1, unsigned t,
                                                           float scale) {
  using V = typename Vec16B<T>::type;
  constexpr int N = Vec16B<T>::N;
  const long id = (long)blockIdx.x * 256 + threadIdx.x;
  if (id >= (long)rows * groups) return;
  const int r = (int)(id / groups), cg = (int)(id % groups);
  const unsigned kb = keep_bits16(philox4x32_10((unsigned)r, (unsigned)cg, 0u, stream, k0, k1), t);
#pragma unroll
  for (int q = 0; q < 16 / N; q++) {
    const int c = 16 * cg + N * q;
    if (c >= cols) break;                                // cols is a multiple of N
    const size_t idx = (size_t)r * cols + c;
    const V v = *reinterpret_cast<const V*>(in + idx);
    V o;
    if (resid) o = *reinterpret_cast<const V*>(resid + idx);
#pragma unroll
    for (int e = 0; e < N; e++) {
      const float x = ((kb >> (N * q + e)) & 1u) ? (float)v[e] * scale : 0.f;
      o[e] = (T)(resid ? (float)o[e] + x : x);
    }
    *reinterpret_cast<V*>(out + idx) = o;
  }
}

}  // namespace

int attn_mask_wpr(int S) { return 2 * cdiv(S, 64); }

hipError_t attn_mask(unsigned* rowbits, unsigned* colbits, int B, int nl, int S, int heads, int head0, unsigned k0,
                     unsigned k1, int t, hipStream_t s) {
  if (!rowbits || S <= 0 || t < 0 || t > 255) return hipErrorInvalidValue;
  const int wpr = attn_mask_wpr(S), nchunk = cdiv(2 * wpr, MASK_GROUPS);
  hipLaunchKernelGGL(attn_mask_kernel, dim3(cdiv(S, 64) * nchunk, nl, B), dim3(64), 0, s, rowbits, colbits, S, wpr,
                     nchunk, heads, head0, k0, k1, (unsigned)t);
  return hipGetLastError();
}

hipError_t dropout_rows(bool bf, const void* in, const void* resid, void* out, int rows, int cols, unsigned stream,
                        unsigned k0, unsigned k1, int t, hipStream_t s) {
  if (t < 0 || t > 255 || (cols & (bf ? 7 : 3))) return hipErrorInvalidValue;
  const int groups = cdiv(cols, 16);
  const long n = (long)rows * groups;
  const float scale = 256.0f / (256.0f - (float)t);
  const dim3 grid((unsigned)cdiv(n, 256L));
  if (bf)
    hipLaunchKernelGGL(dropout_rows_kernel<bf16>, grid, dim3(256), 0, s, static_cast<const bf16*>(in),
                       static_cast<const bf16*>(resid), static_cast<bf16*>(out), rows, cols, groups, stream, k0, k1,
                       (unsigned)t, scale);
  else
    hipLaunchKernelGGL(dropout_rows_kernel<float>, grid, dim3(256), 0, s, static_cast<const float*>(in),
                       static_cast<const float*>(resid), static_cast<float*>(out), rows, cols, groups, stream, k0,
                       k1, (unsigned)t, scale);
  return hipGetLastError();
}

}  // namespace gx
