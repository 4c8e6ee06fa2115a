// Neighbours of the layer step, both bound by HBM bandwidth: the AdamW update on fp32 master
// weights and the strided copies that cut a tensor-parallel shard out of whole parameters or put
// it back.  16 bytes per lane per access, several accesses in flight per lane.
#include "../../include/gx.h"
#include "gx_kernels.h"

#include <math.h>

namespace {

using namespace gx;

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; }

// ------------------------------------------------------------------------------- AdamW
struct AdamArgs {
  float lr, beta1, beta2, eps, wd, gscale, c1, c2;   // c1 = 1 / (1 - beta1^t), c2 = 1 / (1 - beta2^t)
};

GX_DEVINL float adam_one(float& w, float& m, float& v, float g, const AdamArgs& a) {
  const float gs = g * a.gscale;
  m = a.beta1 * m + (1.f - a.beta1) * gs;
  v = a.beta2 * v + (1.f - a.beta2) * (gs * gs);
  const float upd = (m * a.c1) / (sqrtf(v * a.c2) + a.eps) + a.wd * w;
  w = w - a.lr * upd;
  return w;
}

// OUT: 0 none, 1 bf16, 2 fp32.  One 16-byte group of four elements per lane per pass; the last
// partial group (n % 4 elements) is done element by element by one lane.
template <int OUT>
__global__ void __launch_bounds__(256) adamw_kernel(float* __restrict__ w, float* __restrict__ m,
                                                    float* __restrict__ v, const float* __restrict__ g,
                                                    void* __restrict__ out, size_t n, AdamArgs a) {
  const size_t groups = n >> 2;
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < groups; i += stride) {
    f32x4 w4 = reinterpret_cast<const f32x4*>(w)[i];
    f32x4 m4 = reinterpret_cast<const f32x4*>(m)[i];
    f32x4 v4 = reinterpret_cast<const f32x4*>(v)[i];
    const f32x4 g4 = reinterpret_cast<const f32x4*>(g)[i];
#pragma unroll
    for (int e = 0; e < 4; e++) {
      float we = w4[e], me = m4[e], ve = v4[e];
      adam_one(we, me, ve, g4[e], a);
      w4[e] = we; m4[e] = me; v4[e] = ve;
    }
    reinterpret_cast<f32x4*>(w)[i] = w4;
    reinterpret_cast<f32x4*>(m)[i] = m4;
    reinterpret_cast<f32x4*>(v)[i] = v4;
    if (OUT == 1) {
      bf16x4 o;
#pragma unroll
      for (int e = 0; e < 4; e++) o[e] = (bf16)w4[e];
      reinterpret_cast<bf16x4*>(out)[i] = o;
    } else if (OUT == 2) {
      reinterpret_cast<f32x4*>(out)[i] = w4;
    }
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    for (size_t i = groups << 2; i < n; i++) {
      float we = w[i], me = m[i], ve = v[i];
      adam_one(we, me, ve, g[i], a);
      w[i] = we; m[i] = me; v[i] = ve;
      if (OUT == 1) static_cast<bf16*>(out)[i] = (bf16)we;
      else if (OUT == 2) static_cast<float*>(out)[i] = we;
    }
  }
}

// ------------------------------------------------------------------------------- shard copies
// A transition is a short list of 2-D block copies: `rows` rows of `chunks` 16-byte pieces, with
// independent row strides on the two sides.  One launch serves the whole list: workgroup b looks
// up the segment that contains it in a table of cumulative workgroup counts.
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
constexpr int MAX_SEG = 16;
constexpr int PIECES = 4;                       // 16-byte pieces per lane: 16 KB per workgroup measured fastest
constexpr int CHUNKS_PER_WG = 256 * PIECES;
struct Segments {
  const char* src[MAX_SEG];
  char* dst[MAX_SEG];
  long src_stride[MAX_SEG], dst_stride[MAX_SEG];   // bytes between rows
  long chunks[MAX_SEG];                             // 16-byte pieces per row
  long total[MAX_SEG];                              // rows * chunks
  int first_wg[MAX_SEG + 1];
  int n;
};

__global__ void __launch_bounds__(256) segment_copy_kernel(Segments s) {
  int k = 0;
  while (k + 1 < s.n && (int)blockIdx.x >= s.first_wg[k + 1]) k++;
  const long base = (long)(blockIdx.x - s.first_wg[k]) * CHUNKS_PER_WG + threadIdx.x;
  const long cpr = s.chunks[k], total = s.total[k];
  const char* src = s.src[k];
  char* dst = s.dst[k];
  const long ss = s.src_stride[k], ds = s.dst_stride[k];
  // (row, piece) of this lane's first piece by one division; the next ones are 256 pieces further
  // on, which moves (row, piece) by the segment-wide constants (256 / cpr, 256 % cpr)
  long r = base / cpr, c = base - r * cpr;
  const long dr = 256 / cpr, dc = 256 - dr * cpr;
  u32x4 val[PIECES];
  long doff[PIECES];
#pragma unroll
  for (int u = 0; u < PIECES; u++) {
    if (base + u * 256 < total) {
      val[u] = *reinterpret_cast<const u32x4*>(src + r * ss + c * 16);
      doff[u] = r * ds + c * 16;
    }
    r += dr;
    c += dc;
    if (c >= cpr) { c -= cpr; r++; }
  }
#pragma unroll
  for (int u = 0; u < PIECES; u++)
    if (base + u * 256 < total) *reinterpret_cast<u32x4*>(dst + doff[u]) = val[u];
}

struct SegBuilder {
  Segments s;
  gx_status err = GX_OK;
  SegBuilder() { s.n = 0; s.first_wg[0] = 0; }
  // rows x row_bytes block; a contiguous tensor is one row
  void add(const void* src, void* dst, long rows, long row_bytes, long src_stride, long dst_stride) {
    if (err != GX_OK) return;
    if (!src || !dst) { err = GX_ERR_NULL; return; }
    if (misaligned(src) || misaligned(dst)) { err = GX_ERR_ALIGN; return; }
    if ((row_bytes & 15) || (src_stride & 15) || (dst_stride & 15)) { err = GX_ERR_DIVIS; return; }
    if (s.n >= MAX_SEG) { err = GX_ERR_SHAPE; return; }
    const int k = s.n++;
    s.src[k] = static_cast<const char*>(src);
    s.dst[k] = static_cast<char*>(dst);
    s.src_stride[k] = src_stride;
    s.dst_stride[k] = dst_stride;
    s.chunks[k] = row_bytes / 16;
    s.total[k] = rows * s.chunks[k];
    s.first_wg[k + 1] = s.first_wg[k] + cdiv(s.total[k], CHUNKS_PER_WG);
  }
  void whole(const void* src, void* dst, long bytes) { add(src, dst, 1, bytes, bytes, bytes); }
};

static_assert(sizeof(gx_params) == 12 * sizeof(void*) && sizeof(gx_params_out) == 12 * sizeof(void*),
              "the transition code indexes both parameter structs as arrays of 12 pointers");

// slice: src = whole, dst = shard; merge: the other way round.  W() picks the whole-side pointer
// and S() the shard-side pointer of a tensor, whichever struct they live in.
gx_status transition(const gx_layer_cfg* c, const void* const* whole, const void* const* shard, bool to_shard,
                     hipStream_t st) {
  if (!c || !whole || !shard) return GX_ERR_NULL;
  if (c->dtype != GX_F32 && c->dtype != GX_BF16) return GX_ERR_DTYPE;
  if (c->hidden <= 0 || c->heads <= 0 || c->ffn <= 0 || c->tp_attn <= 0 || c->tp_ffn <= 0 || c->tp_rank < 0)
    return GX_ERR_SHAPE;
  if (c->hidden % c->heads || c->heads % c->tp_attn || c->ffn % c->tp_ffn) return GX_ERR_DIVIS;
  const bool attn = c->flags & GX_PHASE_ATTN, mlp = c->flags & GX_PHASE_MLP;
  if (!attn && !mlp) return GX_ERR_FLAGS;
  const long e = c->dtype == GX_BF16 ? 2 : 4;
  const long H = c->hidden, F = c->ffn, Hl = H / c->tp_attn, Fl = F / c->tp_ffn;
  const long ra = c->tp_rank % c->tp_attn, rf = c->tp_rank % c->tp_ffn;
  if ((H * e) & 15 || (Hl * e) & 15 || (Fl * e) & 15) return GX_ERR_DIVIS;
  // indices into gx_params / gx_params_out (both are 12 pointers in the same order)
  enum { LN1G, LN1B, WQKV, BQKV, WO, BO, LN2G, LN2B, WFC1, BFC1, WFC2, BFC2 };
  SegBuilder b;
  auto blockcopy = [&](int t, long rows, long row_bytes, long whole_off, long whole_stride, long shard_off,
                       long shard_stride) {
    const char* w = static_cast<const char*>(whole[t]);
    const char* s = static_cast<const char*>(shard[t]);
    if (!w || !s) { b.err = GX_ERR_NULL; return; }
    if (to_shard) b.add(w + whole_off, const_cast<char*>(s) + shard_off, rows, row_bytes, whole_stride, shard_stride);
    else          b.add(s + shard_off, const_cast<char*>(w) + whole_off, rows, row_bytes, shard_stride, whole_stride);
  };
  auto replicated = [&](int t, long bytes) { blockcopy(t, 1, bytes, 0, bytes, 0, bytes); };
  if (attn) {
    replicated(LN1G, H * e);
    replicated(LN1B, H * e);
    for (int part = 0; part < 3; part++) {
      blockcopy(WQKV, H, Hl * e, (part * H + ra * Hl) * e, 3 * H * e, part * Hl * e, 3 * Hl * e);
      blockcopy(BQKV, 1, Hl * e, (part * H + ra * Hl) * e, Hl * e, part * Hl * e, Hl * e);
    }
    blockcopy(WO, 1, Hl * H * e, ra * Hl * H * e, Hl * H * e, 0, Hl * H * e);     // contiguous rows
    replicated(BO, H * e);
  }
  if (mlp) {
    replicated(LN2G, H * e);
    replicated(LN2B, H * e);
    blockcopy(WFC1, H, Fl * e, rf * Fl * e, F * e, 0, Fl * e);
    blockcopy(BFC1, 1, Fl * e, rf * Fl * e, Fl * e, 0, Fl * e);
    blockcopy(WFC2, 1, Fl * H * e, rf * Fl * H * e, Fl * H * e, 0, Fl * H * e);
    replicated(BFC2, H * e);
  }
  if (b.err != GX_OK) return b.err;
  if (!device_is_gfx950()) return GX_ERR_ARCH;
  const int nwg = b.s.first_wg[b.s.n];
  if (nwg > 0) {
    hipLaunchKernelGGL(segment_copy_kernel, dim3(nwg), dim3(256), 0, st, b.s);
    if (hipGetLastError() != hipSuccess) return GX_ERR_LAUNCH;
  }
  return GX_OK;
}

}  // namespace

extern "C" {

gx_status gx_adamw_step(const gx_adamw_cfg* cfg, size_t n, float* master, float* m, float* v, const float* grad,
                        void* param_out, int param_dtype, void* hip_stream) {
  if (!cfg) return GX_ERR_NULL;
  if (cfg->step < 1 || !(cfg->beta1 >= 0.f && cfg->beta1 < 1.f) || !(cfg->beta2 >= 0.f && cfg->beta2 < 1.f) ||
      n >= ((size_t)1 << 40))
    return GX_ERR_SHAPE;
  if (param_out && param_dtype != GX_F32 && param_dtype != GX_BF16) return GX_ERR_DTYPE;
  if (n == 0) return GX_OK;
  if (!master || !m || !v || !grad) return GX_ERR_NULL;
  if (misaligned(master) || misaligned(m) || misaligned(v) || misaligned(grad) || misaligned(param_out))
    return GX_ERR_ALIGN;
  if (!device_is_gfx950()) return GX_ERR_ARCH;
  AdamArgs a;
  a.lr = cfg->lr; a.beta1 = cfg->beta1; a.beta2 = cfg->beta2; a.eps = cfg->eps; a.wd = cfg->weight_decay;
  a.gscale = cfg->grad_scale;
  a.c1 = (float)(1.0 / (1.0 - pow((double)cfg->beta1, (double)cfg->step)));
  a.c2 = (float)(1.0 / (1.0 - pow((double)cfg->beta2, (double)cfg->step)));
  // enough workgroups to keep every CU's memory pipeline full, each lane walking a few groups
  const size_t groups = n >> 2;
  size_t wgs = (groups + 256 * 4 - 1) / (256 * 4);
  if (wgs < 1) wgs = 1;
  if (wgs > 65536) wgs = 65536;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int out = !param_out ? 0 : (param_dtype == GX_BF16 ? 1 : 2);
  if (out == 0) hipLaunchKernelGGL(adamw_kernel<0>, dim3((unsigned)wgs), dim3(256), 0, st, master, m, v, grad, param_out, n, a);
  else if (out == 1) hipLaunchKernelGGL(adamw_kernel<1>, dim3((unsigned)wgs), dim3(256), 0, st, master, m, v, grad, param_out, n, a);
  else hipLaunchKernelGGL(adamw_kernel<2>, dim3((unsigned)wgs), dim3(256), 0, st, master, m, v, grad, param_out, n, a);
  return hipGetLastError() == hipSuccess ? GX_OK : GX_ERR_LAUNCH;
}

gx_status gx_params_slice(const gx_layer_cfg* cfg, const gx_params* whole, const gx_params_out* shard,
                          void* hip_stream) {
  return transition(cfg, reinterpret_cast<const void* const*>(whole), reinterpret_cast<const void* const*>(shard),
                    true, static_cast<hipStream_t>(hip_stream));
}

gx_status gx_params_merge(const gx_layer_cfg* cfg, const gx_params* shard, const gx_params_out* whole,
                          void* hip_stream) {
  return transition(cfg, reinterpret_cast<const void* const*>(whole), reinterpret_cast<const void* const*>(shard),
                    false, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
