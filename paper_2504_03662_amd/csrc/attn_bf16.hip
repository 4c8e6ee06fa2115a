// Flash-style causal attention for gfx950, bf16 in / fp32 accumulate, head dim 128 or 64 (the
// kernels live in attn_bf16_impl.h, compiled once per head dimension).
//
// Forward: a workgroup owns a block of query rows of one (sample, head); K and V tiles of 64 rows
// stream through a double-buffered LDS stage (direct-to-LDS buffer loads).  Each wavefront keeps
// 32 query rows and works on the transposed problem S^T = K Q^T, so that a lane owns one query
// column of every v_mfma_f32_32x32x16_bf16 accumulator: the online-softmax row statistics are
// lane-local (plus one cross-half shuffle), and the probabilities, once rounded to bf16, are
// already laid out as the B operand of O^T = V^T P^T.  V^T (and every other operand whose
// reduction index is strided in memory) is read with the transposing ds_read_b64_tr_b16.
//
// Backward: D = rowsum(dO * O); then two kernels so that every output has exactly one writer
// and sums run in a fixed order (no atomics): one owns key/value rows and produces dK, dV, the
// other owns query rows and produces dQ.  Probabilities are recomputed from the saved
// log-sum-exp.
#include "gx_kernels.h"
#include <type_traits>

namespace gx {
namespace {

constexpr unsigned OOB = 0x80000000u;
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
typedef __attribute__((address_space(3))) bf16x4* lds_bf16x4_ptr;
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16((a), (b), (c), 0, 0, 0)
#define WAIT_VM0() __builtin_amdgcn_s_waitcnt(0x0F70)

namespace dh128 {
#define GX_ATTN_DH 128
#include "attn_bf16_impl.h"
#undef GX_ATTN_DH
}  // namespace dh128
namespace dh64 {
#define GX_ATTN_DH 64
#include "attn_bf16_impl.h"
#undef GX_ATTN_DH
}  // namespace dh64

}  // namespace

hipError_t attn_fwd_bf16(const AttnArgs& a, hipStream_t s) {
  return a.dh == 128 ? dh128::fwd(a, s) : a.dh == 64 ? dh64::fwd(a, s) : hipErrorInvalidValue;
}

hipError_t attn_bwd_bf16(const AttnArgs& a, hipStream_t s, hipStream_t s_dq, hipEvent_t fork, hipEvent_t join) {
  return a.dh == 128 ? dh128::bwd(a, s, s_dq, fork, join)
                     : a.dh == 64 ? dh64::bwd(a, s, s_dq, fork, join) : hipErrorInvalidValue;
}

}  // namespace gx
