// Internal launcher interface between the layer driver and the kernel translation units.
#pragma once
#include "gx_common.h"

namespace gx {

// true when the current device is the architecture this library is built for (cached per process)
bool device_is_gfx950();

// C[M,N] = op(A) * op(B), all matrices row-major with leading dimensions in elements.
//   NN: A is [M,K], B is [K,N]      (forward: activations times "in x out" weights)
//   NT: A is [M,K], B is [N,K]      (input gradient: dY times W^T, reduction over W's columns)
//   TN: A is [K,M], B is [K,N]      (weight gradient: X^T times dY, reduction over tokens)
enum Layout { LAY_NN = 0, LAY_NT = 1, LAY_TN = 2 };

enum Epilogue {
  EPI_STORE = 0,   // C = acc                                   (storage type)
  EPI_BIAS,        // C = acc + bias[n]            (bias may be null)
  EPI_RESID,       // p = acc + bias[n]; aux = p if aux; C = resid + p
  EPI_GELU,        // z = acc + bias[n]; C = gelu'(z); aux = gelu(z)  (erf form, or tanh form if gelu_tanh)
  EPI_DGELU,       // C = acc * z[m,n], z holding what EPI_GELU left in C
  EPI_F32,         // C (fp32) = acc
  EPI_F32_ACC      // C (fp32) += acc
};

struct GemmArgs {
  const void* A;
  const void* B;
  void* C;
  int M, N, K;
  int lda, ldb, ldc;
  const void* bias;    // [N], storage type
  const void* resid;   // [M, ldc], storage type
  void* aux;           // [M, ldc], storage type
  const void* z;       // [M, ldc], storage type: EPI_DGELU's multiplier
  int gelu_tanh;       // EPI_GELU: tanh form of GELU instead of the erf form
  float* colpart;      // bf16 EPI_DGELU only, optional: partial column sums of the stored C over blocks of 64
                       // rows, [ceil(M / 64)][N] fp32 (stage 1 of the bias gradient; finished by colsum_finish)
  // set by the bf16 launcher only (callers leave them 0): a launch that covers the super-tiles
  // (2 x 2 kernel tiles) numbered tile_first onwards in the tile walk, four workgroups each
  int tail, tile_first;
};

hipError_t gemm_bf16(Layout lay, Epilogue epi, const GemmArgs& g, hipStream_t s);
hipError_t gemm_f32(Layout lay, Epilogue epi, const GemmArgs& g, hipStream_t s);

// Causal attention over the local heads.  qkv is [T, 3*Hl] with column blocks [Q | K | V], each
// head's dh columns contiguous; ctx / dctx are [T, Hl]; lse and dsum are [B, nl, S] fp32.
struct AttnArgs {
  const void* qkv;
  void* ctx;          // fwd out / bwd in
  float* lse;         // fwd out / bwd in: log-sum-exp of the scaled, masked scores per row
  const void* dctx;   // bwd in
  void* dqkv;         // bwd out, same layout as qkv
  float* dsum;        // bwd scratch: rowsum(dctx * ctx)
  int B, S, nl, dh;
  // dropout of the probabilities (rowbits == nullptr: none): keep bits from attn_mask, row-major for
  // the forward and dQ kernels, column-major for dK / dV (bf16 path; the fp32 path reads rowbits
  // throughout), wpr words per row, kept probabilities multiplied by keep_scale
  const unsigned* rowbits;
  const unsigned* colbits;
  int wpr;
  float keep_scale;
};
hipError_t attn_fwd_bf16(const AttnArgs& a, hipStream_t s);
// s_dq may equal s (everything in order on one stream); otherwise the dQ kernel runs on s_dq between
// the two caller-owned events: fork (recorded on s after D is known) and join (s waits for it).
hipError_t attn_bwd_bf16(const AttnArgs& a, hipStream_t s, hipStream_t s_dq, hipEvent_t fork, hipEvent_t join);
hipError_t attn_fwd_f32(const AttnArgs& a, hipStream_t s);
hipError_t attn_bwd_f32(const AttnArgs& a, hipStream_t s);

// Dropout (Philox4x32-10 bytes; an element is dropped iff its byte < t, t in 0..255).
// Keep bits of the attention probabilities of B x nl (sample, local head) pairs, heads `head0`..
// of a model with `heads` heads: rowbits / colbits are [B * nl * S * attn_mask_wpr(S)] words
// (colbits may be null).  Counter (i, j / 16, b * heads + head0 + h, 1), byte j % 16.
int attn_mask_wpr(int S);
hipError_t attn_mask(unsigned* rowbits, unsigned* colbits, int B, int nl, int S, int heads, int head0, unsigned k0,
                     unsigned k1, int t, hipStream_t s);
// out = (resid ? resid : 0) + keep * 256 / (256 - t) * in over [rows, cols]; counter
// (row, column / 16, 0, stream), byte column % 16.  out may alias in.  The fourth counter word
// separates the masks: 1 attention probabilities (attn_mask), 2 and 3 the two halves' outputs.
constexpr unsigned DROP_STREAM_ATTN_OUT = 2, DROP_STREAM_MLP_OUT = 3;
hipError_t dropout_rows(bool bf16, const void* in, const void* resid, void* out, int rows, int cols,
                        unsigned stream, unsigned k0, unsigned k1, int t, hipStream_t s);

// Row-wise and column-sum kernels, templated on storage type through the `bf16` switch.
// LayerNorm forward: y = g * (x - mean) * rstd + b; writes mean/rstd per row.
hipError_t ln_fwd(bool bf16, const void* x, const void* g, const void* b, void* y, float* mean, float* rstd,
                  int rows, int cols, float eps, hipStream_t s);
// Column reductions are two-stage and fixed-order: a producer leaves per-block partial rows
// part[nblk][cols] (fp32), and ONE launch at the end of a pass finishes all of them.
struct FinishSeg {
  const float* part;   // [nblk][cols]
  float* out;          // [cols], written or, with accumulate, added to
  int nblk, cols, accumulate;
  int wg0;             // set by colsum_finish
};
constexpr int FINISH_MAX = 10;
struct FinishArgs {
  FinishSeg seg[FINISH_MAX];
  int nseg;
};
hipError_t colsum_finish(const FinishSeg* segs, int nseg, hipStream_t s);
// LayerNorm backward in one pass: dx = (resid ? resid : 0) + LNbwd(dy), and partial column sums
// part[a][ln_bwd_blocks(..)][cols]: a = 0 sum dy * xhat (gain gradient), 1 sum dy (bias gradient) and,
// with nsum = 4 (resid required), 2 sum resid, 3 sum dx.
hipError_t ln_bwd(bool bf16, const void* dy, const void* x, const void* g, const float* mean, const float* rstd,
                  const void* resid, void* dx, int rows, int cols, int nsum, float* part, hipStream_t s);
int ln_bwd_blocks(bool bf16, int rows, int cols);
// Stage 1 of the column sums of a [rows, cols] matrix: part[colsum_blocks(rows)][cols].
hipError_t colsum_partial(bool bf16, const void* a, int rows, int cols, int ld, float* part, hipStream_t s);
int colsum_blocks(int rows);

}  // namespace gx
