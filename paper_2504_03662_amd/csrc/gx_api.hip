// C-ABI entry points of libgx: validation, buffer planning and the kernel sequences of one
// rank's block forward and backward pass.  Everything here is host code that only enqueues
// kernels on the caller's stream.
#include "../../include/gx.h"
#include "gx_kernels.h"

#include <string.h>

namespace gx {
bool device_is_gfx950() {
  static int cached = -1;     // per process; the library targets a single architecture
  if (cached < 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return false;
    cached = (strncmp(prop.gcnArchName, "gfx950", 6) == 0) ? 1 : 0;
  }
  return cached == 1;
}
}  // namespace gx

// Backward workspace of gx_layer_bwd_static: one array per GPU, in the library's device image,
// held until the process ends.  The compiler exports a file-local device variable that host code
// refers to, which is what the runtime's lookup by name needs; marking it `used` would keep the
// symbol local to the code object and the lookup would fail.
static __device__ __align__(256) unsigned char scratch[GX_STATIC_SCRATCH_BYTES];

namespace {

using namespace gx;

static_assert(sizeof(gx_layer_cfg) == 15 * 4, "gx_layer_cfg is 15 packed 32-bit fields");

constexpr int ALL_FLAGS = GX_PHASE_ATTN | GX_PHASE_MLP | GX_ROW_BIAS_ATTN | GX_ROW_BIAS_MLP | GX_ACCUM_WGRAD |
                          GX_RECOMPUTE | GX_GELU_TANH | GX_WGRAD_BF16 | GX_DROPOUT | GX_FWD_SAVED_ONLY;

struct Dims {
  long T, H, Hl, Fl, S, B, nl, dh;
  size_t e;        // bytes per activation element
  bool bf;
};

Dims dims_of(const gx_layer_cfg& c) {
  Dims d;
  d.H = c.hidden;
  d.dh = c.hidden / c.heads;
  d.nl = c.heads / c.tp_attn;
  d.Hl = d.nl * d.dh;
  d.Fl = c.ffn / c.tp_ffn;
  d.S = c.seq;
  d.B = c.micro_batch;
  d.T = d.S * d.B;
  d.bf = (c.dtype == GX_BF16);
  d.e = d.bf ? 2 : 4;
  return d;
}

size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

// Bump allocator over an opaque block; with base == nullptr it only measures.
struct Arena {
  char* base;
  size_t off = 0;
  explicit Arena(void* b) : base(static_cast<char*>(b)) {}
  void* take(size_t bytes) {
    void* p = base ? base + off : nullptr;
    off += align_up(bytes);
    return p;
  }
};

// Activations the forward pass keeps for the backward pass.
struct Saved {
  float *mean1, *rstd1, *lse, *mean2, *rstd2;
  void *y1, *qkv, *ctx, *h1, *y2, *gelu_grad, *act;   // gelu_grad: gelu'(z) of the FC1 pre-activation z
};

Saved plan_saved(const gx_layer_cfg& c, Arena& a) {
  const Dims d = dims_of(c);
  Saved s;
  memset(&s, 0, sizeof(s));
  if (c.flags & GX_PHASE_ATTN) {
    s.mean1 = static_cast<float*>(a.take(d.T * 4));
    s.rstd1 = static_cast<float*>(a.take(d.T * 4));
    s.y1 = a.take(d.T * d.H * d.e);
    s.qkv = a.take(d.T * 3 * d.Hl * d.e);
    s.ctx = a.take(d.T * d.Hl * d.e);
    s.lse = static_cast<float*>(a.take(d.B * d.nl * d.S * 4));
  }
  if ((c.flags & GX_PHASE_ATTN) && (c.flags & GX_PHASE_MLP)) s.h1 = a.take(d.T * d.H * d.e);
  if (c.flags & GX_PHASE_MLP) {
    s.mean2 = static_cast<float*>(a.take(d.T * 4));
    s.rstd2 = static_cast<float*>(a.take(d.T * 4));
    s.y2 = a.take(d.T * d.H * d.e);
    s.gelu_grad = a.take(d.T * d.Fl * d.e);
    s.act = a.take(d.T * d.Fl * d.e);
  }
  return s;
}

// Backward scratch.
struct Work {
  void *dz, *dy2, *dy1, *dh1, *dctx, *dqkv;
  float* dsum;
  // stage-1 partial sums of the column reductions, one buffer per producer (all are finished by one
  // launch at the end of the pass): the two LayerNorm-backward kernels (up to 4 sums each), the FC1
  // bias gradient (blocks of 64 rows of dz), and the plain column sums of dqkv, dp_mlp and dp_attn
  float *part_ln2, *part_ln1, *part_fc1, *part_qkv, *part_fc2, *part_o;
  void* recomputed;     // a Saved block when GX_RECOMPUTE is set
};

Work plan_work(const gx_layer_cfg& c, Arena& a) {
  const Dims d = dims_of(c);
  Work w;
  memset(&w, 0, sizeof(w));
  if (c.flags & GX_PHASE_MLP) {
    w.dz = a.take(d.T * d.Fl * d.e);
    w.dy2 = a.take(d.T * d.H * d.e);
  }
  if (c.flags & GX_PHASE_ATTN) w.dy1 = a.take(d.T * d.H * d.e);
  if ((c.flags & GX_PHASE_ATTN) && (c.flags & GX_PHASE_MLP)) w.dh1 = a.take(d.T * d.H * d.e);
  if (c.flags & GX_PHASE_ATTN) {
    w.dctx = a.take(d.T * d.Hl * d.e);
    w.dqkv = a.take(d.T * 3 * d.Hl * d.e);
    w.dsum = static_cast<float*>(a.take(d.B * d.nl * d.S * 4));
  }
  const size_t lnb = (size_t)ln_bwd_blocks(d.bf, (int)d.T, (int)d.H), csb = (size_t)colsum_blocks((int)d.T);
  const size_t fcb = (size_t)cdiv(d.T, 64) > csb ? (size_t)cdiv(d.T, 64) : csb;
  if (c.flags & GX_PHASE_MLP) {
    w.part_ln2 = static_cast<float*>(a.take(4 * lnb * d.H * 4));
    w.part_fc1 = static_cast<float*>(a.take(fcb * d.Fl * 4));
    w.part_fc2 = static_cast<float*>(a.take(csb * d.H * 4));
  }
  if (c.flags & GX_PHASE_ATTN) {
    w.part_ln1 = static_cast<float*>(a.take(2 * lnb * d.H * 4));
    w.part_qkv = static_cast<float*>(a.take(csb * 3 * d.Hl * 4));
    w.part_o = static_cast<float*>(a.take(csb * d.H * 4));
  }
  if (c.flags & GX_RECOMPUTE) {
    Arena probe(nullptr);
    plan_saved(c, probe);
    w.recomputed = a.take(probe.off);
  }
  return w;
}

// Dropout variant: what the configuration asks for and the scratch it needs.
struct Drop {
  bool attn = false, hidden = false;   // probabilities; the two halves' outputs (two-phase calls only)
  int t_attn = 0, t_hidden = 0;        // drop probabilities in 1/256ths
  unsigned k0 = 0, k1 = 0;             // generator key
  int head0 = 0;                       // global index of this rank's first head
};

Drop drop_of(const gx_layer_cfg& c) {
  Drop d;
  if (!(c.flags & GX_DROPOUT)) return d;
  const bool attn = c.flags & GX_PHASE_ATTN, mlp = c.flags & GX_PHASE_MLP;
  d.t_attn = c.drop_attn;
  d.t_hidden = c.drop_hidden;
  d.k0 = c.drop_seed_lo;
  d.k1 = c.drop_seed_hi;
  d.attn = attn && c.drop_attn > 0;
  d.hidden = attn && mlp && c.drop_hidden > 0;
  d.head0 = (c.tp_rank % c.tp_attn) * (c.heads / c.tp_attn);
  return d;
}

struct DropBufs {
  unsigned *rowbits, *colbits;   // keep bits of the attention probabilities
  void* partial;                 // a half's output before dropout, when the caller does not ask for it
  void *dym, *dh1m;              // upstream gradients after the output masks
};

DropBufs plan_drop(const gx_layer_cfg& c, Arena& a, bool bwd) {
  DropBufs b;
  memset(&b, 0, sizeof(b));
  const Drop dr = drop_of(c);
  const Dims d = dims_of(c);
  if (dr.attn) {
    const size_t bytes = (size_t)d.B * d.nl * d.S * attn_mask_wpr((int)d.S) * 4;
    b.rowbits = static_cast<unsigned*>(a.take(bytes));
    if (bwd) b.colbits = static_cast<unsigned*>(a.take(bytes));
  }
  if (dr.hidden) {
    if (!bwd || (c.flags & GX_RECOMPUTE)) b.partial = a.take(d.T * d.H * d.e);
    if (bwd) {
      b.dym = a.take(d.T * d.H * d.e);
      b.dh1m = a.take(d.T * d.H * d.e);
    }
  }
  return b;
}

gx_status validate(const gx_layer_cfg* c) {
  if (!c) return GX_ERR_NULL;
  if (c->dtype != GX_F32 && c->dtype != GX_BF16) return GX_ERR_DTYPE;
  if (c->hidden <= 0 || c->heads <= 0 || c->ffn <= 0 || c->tp_attn <= 0 || c->tp_ffn <= 0 || c->seq <= 0 ||
      c->micro_batch <= 0 || !(c->ln_eps >= 0.f))
    return GX_ERR_SHAPE;
  if ((c->flags & ~ALL_FLAGS) || !(c->flags & (GX_PHASE_ATTN | GX_PHASE_MLP))) return GX_ERR_FLAGS;
  if ((c->flags & GX_WGRAD_BF16) && c->dtype != GX_BF16) return GX_ERR_DTYPE;
  if ((c->flags & GX_DROPOUT) && (c->drop_attn < 0 || c->drop_attn > 255 || c->drop_hidden < 0 || c->drop_hidden > 255))
    return GX_ERR_SHAPE;
  if (c->hidden % c->heads || c->heads % c->tp_attn || c->ffn % c->tp_ffn) return GX_ERR_DIVIS;
  const int tpmax = c->tp_attn > c->tp_ffn ? c->tp_attn : c->tp_ffn;
  if (c->tp_rank < 0 || c->tp_rank >= tpmax) return GX_ERR_SHAPE;
  const Dims d = dims_of(*c);
  const int vec = d.bf ? 8 : 4;
  if (d.H % vec || d.Fl % vec || d.Hl % vec) return GX_ERR_DIVIS;
  if (d.bf) {
    if ((d.dh != 128 && d.dh != 64) || d.H > 8192) return GX_ERR_SHAPE;
  } else {
    if (d.dh > 128 || d.H > 4096 || d.S > 8192) return GX_ERR_SHAPE;
  }
  long widest = d.H;
  if (3 * d.Hl > widest) widest = 3 * d.Hl;
  if (d.Fl > widest) widest = d.Fl;
  if ((size_t)d.T * widest * d.e >= (1ul << 31)) return GX_ERR_SHAPE;
  // weight shards are also addressed with 31-bit byte offsets
  if ((size_t)d.H * 3 * d.Hl * d.e >= (1ul << 31) || (size_t)d.H * d.Fl * d.e >= (1ul << 31)) return GX_ERR_SHAPE;
  return GX_OK;
}

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; }

gx_status check_arch() { return device_is_gfx950() ? GX_OK : GX_ERR_ARCH; }

#define GX_TRY(expr)                              \
  do {                                            \
    if ((expr) != hipSuccess) return GX_ERR_LAUNCH; \
  } while (0)

// Optional per-kernel-class timing: when enabled, every launch site is bracketed by a pair of
// HIP events on the caller's stream.  Process-global, not thread-safe, off by default.
constexpr int PROF_MAX = 8192;
struct Prof {
  bool on = false;
  int n = 0;
  hipEvent_t* ev = nullptr;      // 2 * PROF_MAX events, created on first enable
  int cls[PROF_MAX];
} g_prof;

struct ProfScope {
  hipStream_t st;
  int slot;
  ProfScope(int cls, hipStream_t s) : st(s), slot(-1) {
    if (g_prof.on && g_prof.n < PROF_MAX) {
      slot = g_prof.n++;
      g_prof.cls[slot] = cls;
      (void)hipEventRecord(g_prof.ev[2 * slot], st);
    }
  }
  ~ProfScope() {
    if (slot >= 0) (void)hipEventRecord(g_prof.ev[2 * slot + 1], st);
  }
};

int gemm_class(Layout lay, Epilogue epi) { return GX_KC_GEMM + 10 * (int)lay + (int)epi; }

hipError_t gemm(const Dims& d, Layout lay, Epilogue epi, const GemmArgs& g, hipStream_t s) {
  ProfScope ps(gemm_class(lay, epi), s);
  return d.bf ? gemm_bf16(lay, epi, g, s) : gemm_f32(lay, epi, g, s);
}

// stage 1 of a column sum on stream s; its finish is queued in `fin`
struct Finisher {
  FinishSeg seg[FINISH_MAX];
  int n = 0;
  void add(const float* part, int nblk, long cols, float* out, bool acc) {
    if (n < FINISH_MAX) seg[n++] = FinishSeg{part, out, nblk, (int)cols, acc ? 1 : 0, 0};
  }
};

hipError_t colsum_p(bool bf, const void* a, long rows, long cols, float* part, float* out, bool acc, Finisher& fin,
                    hipStream_t s) {
  ProfScope ps(GX_KC_COLSUM, s);
  fin.add(part, colsum_blocks((int)rows), cols, out, acc);
  return colsum_partial(bf, a, (int)rows, (int)cols, (int)cols, part, s);
}

// The backward pass has work whose inputs are ready long before anything consumes its results:
// the bandwidth-bound column reductions (bias and LayerNorm parameter gradients) and every
// weight-gradient product.  It runs on a second, library-owned stream beside the dependent chain
// (input gradients, LayerNorm input gradients, attention) on the caller's stream, and a third
// stream takes the dQ kernel beside the dK/dV kernel: fork with an event after the producer, join
// once at the end of the call.  Created on first use, default priority, shared by all calls of the
// process (calls from several host threads must not overlap).
struct SideStream {
  bool tried = false, ok = false;
  hipStream_t s = nullptr;
  hipEvent_t fork[8];
  hipEvent_t join;
};
constexpr int MAX_DEVICES = 64;
// one per host thread and device, created on first use and kept: calls from different host threads
// never share a side stream or an event
thread_local SideStream t_side[MAX_DEVICES];

bool g_overlap = true;     // gx_set_overlap

SideStream* side_ready() {
  if (!g_overlap) return nullptr;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
  SideStream& sd = t_side[dev];
  if (!sd.tried) {
    sd.tried = true;
    bool ok = hipStreamCreateWithFlags(&sd.s, hipStreamNonBlocking) == hipSuccess;
    for (int i = 0; ok && i < 8; i++) ok = hipEventCreateWithFlags(&sd.fork[i], hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&sd.join, hipEventDisableTiming) == hipSuccess;
    sd.ok = ok;
  }
  return sd.ok ? &sd : nullptr;
}

// Work queued on the side stream after everything queued so far on the caller's stream.
struct Fork {
  hipStream_t main, side;
  SideStream* ss;
  int n = 0;
  bool used = false;
  Fork(hipStream_t m, bool allow_side) : main(m), side(m), ss(allow_side ? side_ready() : nullptr) {
    if (ss) side = ss->s;
  }
  hipError_t err = hipSuccess;     // first failure of an event call; reported by join()
  // stream for a task that depends on what `main` holds now
  hipStream_t branch() {
    if (side != main && n < 8 && err == hipSuccess) {
      err = hipEventRecord(ss->fork[n], main);
      if (err == hipSuccess) err = hipStreamWaitEvent(side, ss->fork[n], 0);
      if (err != hipSuccess) return main;       // not ordered after the producer: stay on its stream
      n++;
      used = true;
      return side;
    }
    return main;
  }
  hipError_t join() {
    if (err != hipSuccess) return err;
    if (!used) return hipSuccess;
    hipError_t e = hipEventRecord(ss->join, side);
    if (e != hipSuccess) return e;
    return hipStreamWaitEvent(main, ss->join, 0);
  }
};

GemmArgs gargs(const void* A, const void* B, void* C, long M, long N, long K, long lda, long ldb, long ldc) {
  GemmArgs g;
  memset(&g, 0, sizeof(g));
  g.A = A; g.B = B; g.C = C;
  g.M = (int)M; g.N = (int)N; g.K = (int)K;
  g.lda = (int)lda; g.ldb = (int)ldb; g.ldc = (int)ldc;
  return g;
}

__global__ void fill_zero_kernel(float* p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

hipError_t dropout_p(const Dims& d, const Drop& dr, const void* in, const void* resid, void* out, unsigned stream,
                     hipStream_t s) {
  ProfScope ps(GX_KC_DROPOUT, s);
  return dropout_rows(d.bf, in, resid, out, (int)d.T, (int)d.H, stream, dr.k0, dr.k1, dr.t_hidden, s);
}

// Keep bits of the attention probabilities for this call (both layouts for a backward pass).
gx_status make_attn_mask(const gx_layer_cfg& c, const DropBufs& db, hipStream_t st) {
  const Drop dr = drop_of(c);
  if (!dr.attn) return GX_OK;
  const Dims d = dims_of(c);
  ProfScope ps(GX_KC_DROPOUT, st);
  GX_TRY(attn_mask(db.rowbits, db.colbits, (int)d.B, (int)d.nl, (int)d.S, c.heads, dr.head0, dr.k0, dr.k1, dr.t_attn,
                   st));
  return GX_OK;
}

void set_attn_drop(AttnArgs& a, const Dims& d, const Drop& dr, const DropBufs& db) {
  if (!dr.attn) return;
  a.rowbits = db.rowbits;
  a.colbits = db.colbits;
  a.wpr = attn_mask_wpr((int)d.S);
  a.keep_scale = 256.0f / (256.0f - (float)dr.t_attn);
}

// Forward kernel sequence.  `for_backward_only` skips the products whose results the backward
// pass does not need (used when recomputing activations).
gx_status run_fwd(const gx_layer_cfg& c, const gx_params& p, const void* x, void* y, void* p_attn, void* p_mlp,
                  const Saved& sv, const DropBufs& db, bool for_backward_only, hipStream_t st) {
  const Dims d = dims_of(c);
  const Drop dr = drop_of(c);
  const bool attn = c.flags & GX_PHASE_ATTN, mlp = c.flags & GX_PHASE_MLP;
  const void* h1 = x;
  if (attn) {
    { ProfScope ps(GX_KC_LN_FWD, st);
    GX_TRY(ln_fwd(d.bf, x, p.ln1_g, p.ln1_b, sv.y1, sv.mean1, sv.rstd1, (int)d.T, (int)d.H, c.ln_eps, st)); }
    GemmArgs g = gargs(sv.y1, p.w_qkv, sv.qkv, d.T, 3 * d.Hl, d.H, d.H, 3 * d.Hl, 3 * d.Hl);
    g.bias = p.b_qkv;
    GX_TRY(gemm(d, LAY_NN, EPI_BIAS, g, st));
    AttnArgs a;
    memset(&a, 0, sizeof(a));
    a.qkv = sv.qkv; a.ctx = sv.ctx; a.lse = sv.lse;
    a.B = (int)d.B; a.S = (int)d.S; a.nl = (int)d.nl; a.dh = (int)d.dh;
    set_attn_drop(a, d, dr, db);
    { ProfScope ps(GX_KC_ATTN_FWD, st);
    GX_TRY(d.bf ? attn_fwd_bf16(a, st) : attn_fwd_f32(a, st)); }
    if (mlp && dr.hidden) {
      // the half's output goes to memory undropped, then one pass drops it and adds the residual
      void* pa = p_attn ? p_attn : db.partial;
      GemmArgs o = gargs(sv.ctx, p.w_o, pa, d.T, d.H, d.Hl, d.Hl, d.H, d.H);
      o.bias = (c.flags & GX_ROW_BIAS_ATTN) ? p.b_o : nullptr;
      GX_TRY(gemm(d, LAY_NN, EPI_BIAS, o, st));
      GX_TRY(dropout_p(d, dr, pa, x, sv.h1, DROP_STREAM_ATTN_OUT, st));
      h1 = sv.h1;
    } else if (mlp) {
      GemmArgs o = gargs(sv.ctx, p.w_o, sv.h1, d.T, d.H, d.Hl, d.Hl, d.H, d.H);
      o.bias = (c.flags & GX_ROW_BIAS_ATTN) ? p.b_o : nullptr;
      o.resid = x;
      o.aux = p_attn;
      GX_TRY(gemm(d, LAY_NN, EPI_RESID, o, st));
      h1 = sv.h1;
    } else if (!for_backward_only) {
      GemmArgs o = gargs(sv.ctx, p.w_o, p_attn, d.T, d.H, d.Hl, d.Hl, d.H, d.H);
      o.bias = (c.flags & GX_ROW_BIAS_ATTN) ? p.b_o : nullptr;
      GX_TRY(gemm(d, LAY_NN, EPI_BIAS, o, st));
    }
  }
  if (mlp) {
    { ProfScope ps(GX_KC_LN_FWD, st);
    GX_TRY(ln_fwd(d.bf, h1, p.ln2_g, p.ln2_b, sv.y2, sv.mean2, sv.rstd2, (int)d.T, (int)d.H, c.ln_eps, st)); }
    GemmArgs f1 = gargs(sv.y2, p.w_fc1, sv.gelu_grad, d.T, d.Fl, d.H, d.H, d.Fl, d.Fl);
    f1.bias = p.b_fc1;
    f1.aux = sv.act;
    f1.gelu_tanh = (c.flags & GX_GELU_TANH) ? 1 : 0;
    GX_TRY(gemm(d, LAY_NN, EPI_GELU, f1, st));
    if (!for_backward_only) {
      void* pm = p_mlp ? p_mlp : db.partial;
      GemmArgs f2 = gargs(sv.act, p.w_fc2, dr.hidden ? pm : attn ? y : p_mlp, d.T, d.H, d.Fl, d.Fl, d.H, d.H);
      f2.bias = (c.flags & GX_ROW_BIAS_MLP) ? p.b_fc2 : nullptr;
      if (dr.hidden) {
        GX_TRY(gemm(d, LAY_NN, EPI_BIAS, f2, st));
        GX_TRY(dropout_p(d, dr, pm, h1, y, DROP_STREAM_MLP_OUT, st));
      } else if (attn) {
        f2.resid = h1;
        f2.aux = p_mlp;
        GX_TRY(gemm(d, LAY_NN, EPI_RESID, f2, st));
      } else {
        GX_TRY(gemm(d, LAY_NN, EPI_BIAS, f2, st));
      }
    }
  }
  return GX_OK;
}

gx_status zero_grad(bool acc, float* out, long cols, hipStream_t st) {
  if (!acc) {
    hipLaunchKernelGGL(fill_zero_kernel, dim3(cdiv(cols, 256)), dim3(256), 0, st, out, (int)cols);
    GX_TRY(hipGetLastError());
  }
  return GX_OK;
}

gx_status run_bwd(const gx_layer_cfg& c, const gx_params& p, const void* x, const void* dy, void* dx,
                  const gx_grads& gr, const Saved& sv, const Work& w, const DropBufs& db, hipStream_t st,
                  bool allow_side) {
  const Dims d = dims_of(c);
  const Drop dr = drop_of(c);
  const bool attn = c.flags & GX_PHASE_ATTN, mlp = c.flags & GX_PHASE_MLP;
  const bool acc = c.flags & GX_ACCUM_WGRAD;
  // weight gradient A^T B into fp32 (store or add) or, on request, into bf16: a plain rounding
  // store, or the residual epilogue reading the old value from the output itself (every lane
  // reads exactly the four elements it then writes, so in place is safe)
  auto wgrad = [&](GemmArgs g, hipStream_t s) -> hipError_t {
    if (!(c.flags & GX_WGRAD_BF16)) return gemm(d, LAY_TN, acc ? EPI_F32_ACC : EPI_F32, g, s);
    if (!acc) return gemm(d, LAY_TN, EPI_STORE, g, s);
    g.resid = g.C;
    return gemm(d, LAY_TN, EPI_RESID, g, s);
  };
  Fork fk(st, allow_side);
  Finisher fin;
  gx_status s;
  // The weight-gradient products only consume finished tensors, so they are handed to the side
  // stream, beside the dependent chain on the caller's stream.  When they are handed over matters
  // little (the large products simply share the chip with whatever runs beside them) but measurably:
  // FC2's, FC1's and the output projection's after LayerNorm 2, QKV's after the attention kernels
  // measured best at the benchmark's shard shape (about 1 % over handing each over as soon as its
  // operands exist, 1 - 3 % over handing them over later), and needs two fork points instead of four.
  // Points: 0 start, 1 after dz, 2 after dy2, 3 after LayerNorm 2, 4 after dctx, 5 after attention,
  // 6 after dy1; one character per product (dW2, dW1, dWo, dWqkv).
  const char sched[5] = "3335";
  const bool ln2_sums_biases = attn && mlp && !dr.hidden;
  const int lnb = ln_bwd_blocks(d.bf, (int)d.T, (int)d.H);
  const void* dp_mlp = dy;
  const void* dp_attn = nullptr;
  auto task = [&](int t, hipStream_t sd) -> gx_status {
    if (t == 0) {        // dW2 (+ b_fc2)
      if (!(c.flags & GX_ROW_BIAS_MLP)) { if ((s = zero_grad(acc, gr.b_fc2, d.H, sd)) != GX_OK) return s; }
      else if (!ln2_sums_biases) GX_TRY(colsum_p(d.bf, dp_mlp, d.T, d.H, w.part_fc2, gr.b_fc2, acc, fin, sd));
      GemmArgs w2 = gargs(sv.act, dp_mlp, gr.w_fc2, d.Fl, d.H, d.T, d.Fl, d.H, d.H);
      GX_TRY(wgrad(w2, sd));
    } else if (t == 1) { // dW1
      if (!d.bf) GX_TRY(colsum_p(d.bf, w.dz, d.T, d.Fl, w.part_fc1, gr.b_fc1, acc, fin, sd));
      GemmArgs w1 = gargs(sv.y2, w.dz, gr.w_fc1, d.H, d.Fl, d.T, d.H, d.Fl, d.Fl);
      GX_TRY(wgrad(w1, sd));
    } else if (t == 2) { // dWo (+ b_o)
      if (!(c.flags & GX_ROW_BIAS_ATTN)) { if ((s = zero_grad(acc, gr.b_o, d.H, sd)) != GX_OK) return s; }
      else if (!ln2_sums_biases) GX_TRY(colsum_p(d.bf, dp_attn, d.T, d.H, w.part_o, gr.b_o, acc, fin, sd));
      GemmArgs wo = gargs(sv.ctx, dp_attn, gr.w_o, d.Hl, d.H, d.T, d.Hl, d.H, d.H);
      GX_TRY(wgrad(wo, sd));
    } else {             // dWqkv (+ b_qkv)
      GX_TRY(colsum_p(d.bf, w.dqkv, d.T, 3 * d.Hl, w.part_qkv, gr.b_qkv, acc, fin, sd));
      GemmArgs wq = gargs(sv.y1, w.dqkv, gr.w_qkv, d.H, 3 * d.Hl, d.T, d.H, 3 * d.Hl, 3 * d.Hl);
      GX_TRY(wgrad(wq, sd));
    }
    return GX_OK;
  };
  auto point = [&](int k) -> gx_status {
    hipStream_t sd = nullptr;
    for (int t = 0; t < 4; t++) {
      if (sched[t] - '0' != k) continue;
      if ((t < 2 && !mlp) || (t >= 2 && !attn)) continue;
      if (!sd) sd = fk.branch();
      if ((s = task(t, sd)) != GX_OK) return s;
    }
    return GX_OK;
  };
  const void* dcur = dy;
  if (mlp) {
    const void* h1 = attn ? sv.h1 : x;
    if (dr.hidden) {
      GX_TRY(dropout_p(d, dr, dy, nullptr, db.dym, DROP_STREAM_MLP_OUT, st));
      dp_mlp = db.dym;
    }
    if ((s = point(0)) != GX_OK) return s;
    GemmArgs dz = gargs(dp_mlp, p.w_fc2, w.dz, d.T, d.Fl, d.H, d.H, d.H, d.Fl);
    dz.z = sv.gelu_grad;
    if (d.bf) {
      dz.colpart = w.part_fc1;
      fin.add(w.part_fc1, cdiv(d.T, 64), d.Fl, gr.b_fc1, acc);
    }
    GX_TRY(gemm(d, LAY_NT, EPI_DGELU, dz, st));
    if ((s = point(1)) != GX_OK) return s;
    GemmArgs dy2 = gargs(w.dz, p.w_fc1, w.dy2, d.T, d.H, d.Fl, d.Fl, d.Fl, d.H);
    GX_TRY(gemm(d, LAY_NT, EPI_STORE, dy2, st));
    if ((s = point(2)) != GX_OK) return s;
    void* out = attn ? w.dh1 : dx;
    {
      ProfScope ps(GX_KC_LN_BWD, st);
      GX_TRY(ln_bwd(d.bf, w.dy2, h1, p.ln2_g, sv.mean2, sv.rstd2, attn ? dy : nullptr, out, (int)d.T, (int)d.H,
                    ln2_sums_biases ? 4 : 2, w.part_ln2, st));
    }
    const size_t stride = (size_t)lnb * d.H;
    fin.add(w.part_ln2, lnb, d.H, gr.ln2_g, acc);
    fin.add(w.part_ln2 + stride, lnb, d.H, gr.ln2_b, acc);
    if (ln2_sums_biases) {
      if (c.flags & GX_ROW_BIAS_MLP) fin.add(w.part_ln2 + 2 * stride, lnb, d.H, gr.b_fc2, acc);
      if (c.flags & GX_ROW_BIAS_ATTN) fin.add(w.part_ln2 + 3 * stride, lnb, d.H, gr.b_o, acc);
    }
    dcur = w.dh1;
    if (!attn)                       // a lone feed-forward half: no later point will come
      for (int k = 3; k <= 6; k++)
        if ((s = point(k)) != GX_OK) return s;
  }
  if (attn) {
    dp_attn = dcur;
    if (dr.hidden) {
      GX_TRY(dropout_p(d, dr, dcur, nullptr, db.dh1m, DROP_STREAM_ATTN_OUT, st));
      dp_attn = db.dh1m;
    }
    if ((s = point(3)) != GX_OK) return s;
    GemmArgs dc = gargs(dp_attn, p.w_o, w.dctx, d.T, d.Hl, d.H, d.H, d.H, d.Hl);
    GX_TRY(gemm(d, LAY_NT, EPI_STORE, dc, st));
    if ((s = point(4)) != GX_OK) return s;
    AttnArgs a;
    memset(&a, 0, sizeof(a));
    a.qkv = sv.qkv; a.ctx = sv.ctx; a.lse = sv.lse; a.dctx = w.dctx; a.dqkv = w.dqkv; a.dsum = w.dsum;
    a.B = (int)d.B; a.S = (int)d.S; a.nl = (int)d.nl; a.dh = (int)d.dh;
    set_attn_drop(a, d, dr, db);
    { ProfScope ps(GX_KC_ATTN_BWD, st);
    // the dQ kernel follows the dK / dV kernel on the caller's stream: a stream of its own for it
    // measured slightly slower (its workgroups cannot share a compute unit with the other kernel's)
    GX_TRY(d.bf ? attn_bwd_bf16(a, st, st, nullptr, nullptr) : attn_bwd_f32(a, st));
    }
    if ((s = point(5)) != GX_OK) return s;
    GemmArgs dy1 = gargs(w.dqkv, p.w_qkv, w.dy1, d.T, d.H, 3 * d.Hl, 3 * d.Hl, 3 * d.Hl, d.H);
    GX_TRY(gemm(d, LAY_NT, EPI_STORE, dy1, st));
    if ((s = point(6)) != GX_OK) return s;
    {
      ProfScope ps(GX_KC_LN_BWD, st);
      GX_TRY(ln_bwd(d.bf, w.dy1, x, p.ln1_g, sv.mean1, sv.rstd1, mlp ? dcur : nullptr, dx, (int)d.T, (int)d.H, 2,
                    w.part_ln1, st));
    }
    fin.add(w.part_ln1, lnb, d.H, gr.ln1_g, acc);
    fin.add(w.part_ln1 + (size_t)lnb * d.H, lnb, d.H, gr.ln1_b, acc);
  }
  GX_TRY(fk.join());
  {
    ProfScope ps(GX_KC_COLSUM, st);
    GX_TRY(colsum_finish(fin.seg, fin.n, st));
  }
  return GX_OK;
}

gx_status check_params(const gx_layer_cfg& c, const gx_params& p) {
  const void* a[] = {p.ln1_g, p.ln1_b, p.w_qkv, p.b_qkv, p.w_o, p.b_o};
  const void* m[] = {p.ln2_g, p.ln2_b, p.w_fc1, p.b_fc1, p.w_fc2, p.b_fc2};
  if (c.flags & GX_PHASE_ATTN)
    for (const void* q : a) {
      if (!q) return GX_ERR_NULL;
      if (misaligned(q)) return GX_ERR_ALIGN;
    }
  if (c.flags & GX_PHASE_MLP)
    for (const void* q : m) {
      if (!q) return GX_ERR_NULL;
      if (misaligned(q)) return GX_ERR_ALIGN;
    }
  return GX_OK;
}

gx_status check_grads(const gx_layer_cfg& c, const gx_grads& g) {
  const float* a[] = {g.ln1_g, g.ln1_b, g.w_qkv, g.b_qkv, g.w_o, g.b_o};
  const float* m[] = {g.ln2_g, g.ln2_b, g.w_fc1, g.b_fc1, g.w_fc2, g.b_fc2};
  if (c.flags & GX_PHASE_ATTN)
    for (const float* q : a) {
      if (!q) return GX_ERR_NULL;
      if (misaligned(q)) return GX_ERR_ALIGN;
    }
  if (c.flags & GX_PHASE_MLP)
    for (const float* q : m) {
      if (!q) return GX_ERR_NULL;
      if (misaligned(q)) return GX_ERR_ALIGN;
    }
  return GX_OK;
}

gx_status layer_bwd(const gx_layer_cfg* cfg, const gx_params* params, const void* x, const void* dy, void* dx,
                    const gx_grads* grads, const void* saved, void* workspace, void* hip_stream, bool allow_side) {
  gx_status s = validate(cfg);
  if (s != GX_OK) return s;
  const bool recompute = cfg->flags & GX_RECOMPUTE;
  if (!params || !x || !dy || !dx || !grads || !workspace || (!recompute && !saved)) return GX_ERR_NULL;
  if (misaligned(x) || misaligned(dy) || misaligned(dx) || misaligned(workspace) || (!recompute && misaligned(saved)))
    return GX_ERR_ALIGN;
  if ((s = check_params(*cfg, *params)) != GX_OK) return s;
  if ((s = check_grads(*cfg, *grads)) != GX_OK) return s;
  if ((s = check_arch()) != GX_OK) return s;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  Arena wa(workspace);
  const Work w = plan_work(*cfg, wa);
  const DropBufs db = plan_drop(*cfg, wa, true);
  Arena sa(recompute ? w.recomputed : const_cast<void*>(saved));
  const Saved sv = plan_saved(*cfg, sa);
  if ((s = make_attn_mask(*cfg, db, st)) != GX_OK) return s;
  if (recompute) {
    s = run_fwd(*cfg, *params, x, nullptr, nullptr, nullptr, sv, db, true, st);
    if (s != GX_OK) return s;
  }
  return run_bwd(*cfg, *params, x, dy, dx, *grads, sv, w, db, st, allow_side);
}

// The device address of `scratch` (the name itself is only a handle for the runtime's symbol
// lookup in host code, never an address): asked for once per device, with that device current.
void* g_scratch_ptr[MAX_DEVICES];

void* static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

}  // namespace

extern "C" {

gx_status gx_layer_validate(const gx_layer_cfg* cfg) { return validate(cfg); }

size_t gx_layer_saved_bytes(const gx_layer_cfg* cfg) {
  if (validate(cfg) != GX_OK) return 0;
  Arena a(nullptr);
  plan_saved(*cfg, a);
  return a.off;
}

size_t gx_layer_workspace_bytes(const gx_layer_cfg* cfg, int is_backward) {
  if (validate(cfg) != GX_OK) return 0;
  Arena a(nullptr);
  if (is_backward) plan_work(*cfg, a);
  plan_drop(*cfg, a, is_backward != 0);
  return a.off;
}

gx_status gx_layer_fwd(const gx_layer_cfg* cfg, const gx_params* params, const void* x, void* y, void* p_attn,
                       void* p_mlp, void* saved, void* workspace, void* hip_stream) {
  gx_status s = validate(cfg);
  if (s != GX_OK) return s;
  if (!params || !x || !saved) return GX_ERR_NULL;
  if (!workspace && gx_layer_workspace_bytes(cfg, 0) != 0) return GX_ERR_NULL;
  if (misaligned(workspace)) return GX_ERR_ALIGN;
  const bool attn = cfg->flags & GX_PHASE_ATTN, mlp = cfg->flags & GX_PHASE_MLP;
  const bool saved_only = cfg->flags & GX_FWD_SAVED_ONLY;
  if (!saved_only) {
    if (attn && mlp && !y) return GX_ERR_NULL;
    if (attn && !mlp && !p_attn) return GX_ERR_NULL;
    if (!attn && mlp && !p_mlp) return GX_ERR_NULL;
  }
  if (misaligned(x) || misaligned(y) || misaligned(p_attn) || misaligned(p_mlp) || misaligned(saved))
    return GX_ERR_ALIGN;
  if ((s = check_params(*cfg, *params)) != GX_OK) return s;
  if ((s = check_arch()) != GX_OK) return s;
  Arena a(saved);
  const Saved sv = plan_saved(*cfg, a);
  Arena wa(workspace);
  const DropBufs db = plan_drop(*cfg, wa, false);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if ((s = make_attn_mask(*cfg, db, st)) != GX_OK) return s;
  if (saved_only) return run_fwd(*cfg, *params, x, nullptr, nullptr, nullptr, sv, db, true, st);
  return run_fwd(*cfg, *params, x, y, p_attn, p_mlp, sv, db, false, st);
}

gx_status gx_layer_bwd(const gx_layer_cfg* cfg, const gx_params* params, const void* x, const void* dy, void* dx,
                       const gx_grads* grads, const void* saved, void* workspace, void* hip_stream) {
  return layer_bwd(cfg, params, x, dy, dx, grads, saved, workspace, hip_stream, true);
}

gx_status gx_layer_bwd_static(const gx_layer_cfg* cfg, const gx_params* params, const void* x, const void* dy,
                              void* dx, const gx_grads* grads, const void* saved, void* hip_stream) {
  const gx_status s = validate(cfg);
  if (s != GX_OK) return s;
  if (gx_layer_workspace_bytes(cfg, 1) > GX_STATIC_SCRATCH_BYTES) return GX_ERR_SHAPE;
  void* ws = static_scratch();
  if (!ws) return GX_ERR_LAUNCH;
  // everything on the caller's stream: the side streams and their events are created on first use,
  // which a caller that may not allocate cannot be asked to tolerate
  return layer_bwd(cfg, params, x, dy, dx, grads, saved, ws, hip_stream, false);
}

const char* gx_status_str(gx_status s) {
  switch (s) {
    case GX_OK: return "ok";
    case GX_ERR_NULL: return "a required pointer is NULL";
    case GX_ERR_SHAPE: return "a size is non-positive or outside the supported range";
    case GX_ERR_DIVIS: return "sizes are not divisible as the sharding or vector width requires";
    case GX_ERR_DTYPE: return "unknown dtype";
    case GX_ERR_ALIGN: return "a pointer is not 16-byte aligned";
    case GX_ERR_FLAGS: return "no phase selected or unknown flag bits";
    case GX_ERR_ARCH: return "the current device is not gfx950";
    case GX_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
    case GX_ERR_INFEASIBLE: return "no assignment fits the memory budget";
  }
  return "unknown status";
}

const char* gx_version(void) { return "gx 0.1 (gfx950)"; }

gx_status gx_set_overlap(int on) {
  g_overlap = on != 0;
  return GX_OK;
}

gx_status gx_prof_enable(int on) {
  if (on && !g_prof.ev) {
    g_prof.ev = new hipEvent_t[2 * PROF_MAX];
    for (int i = 0; i < 2 * PROF_MAX; i++)
      if (hipEventCreate(&g_prof.ev[i]) != hipSuccess) return GX_ERR_LAUNCH;
  }
  g_prof.on = on != 0;
  g_prof.n = 0;
  return GX_OK;
}

int gx_prof_collect(int* kernel_class, float* ms, int capacity) {
  const int n = g_prof.n < capacity ? g_prof.n : capacity;
  for (int i = 0; i < n; i++) {
    if (hipEventSynchronize(g_prof.ev[2 * i + 1]) != hipSuccess) return -1;
    float t = 0.f;
    if (hipEventElapsedTime(&t, g_prof.ev[2 * i], g_prof.ev[2 * i + 1]) != hipSuccess) return -1;
    kernel_class[i] = g_prof.cls[i];
    ms[i] = t;
  }
  g_prof.n = 0;
  return n;
}

}  // extern "C"
