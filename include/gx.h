/* gx.h - C ABI of libgx: one GPU's share of a pre-LayerNorm transformer block's training step
 * (forward and backward) on AMD MI355X (gfx950), at the sharded shapes a hybrid
 * data/tensor/pipeline-parallel strategy assigns to one rank.
 *
 * Background (Galvatron paper, arXiv 2504.03662): section 2 "Layer-Specific Parallelism
 * Optimization" and section 3 "NVIDIA Megatron-LM" describe tensor parallelism as splitting a
 * layer's matrix products across GPUs, possibly with different degrees for the attention and the
 * feed-forward halves of a layer; section 2 "Training Phase Adaptation" and section 3
 * "ParallelismManager" describe micro-batches flowing through a pipeline stage; section 4's
 * ParallelismConfig record (strategy type, pipeline size, tensor degree, micro-batch size) is the
 * model for gx_layer_cfg.  The paper prints no layer equations; the block computed here is the
 * textbook pre-LN GPT block:
 *
 *   attention half : y1 = LN(x; ln1_g, ln1_b);  [Q|K|V] = y1 * w_qkv + b_qkv   (column-parallel)
 *                    causal softmax(Q K^T / sqrt(dh)) V per sample and local head -> ctx
 *                    p_attn = ctx * w_o (+ b_o)                                 (row-parallel)
 *   feed-forward   : y2 = LN(h1; ln2_g, ln2_b); z = y2 * w_fc1 + b_fc1; act = gelu_erf(z)
 *                    p_mlp = act * w_fc2 (+ b_fc2)                              (row-parallel)
 *   both phases    : h1 = x + p_attn;  y = h1 + p_mlp
 *
 * Row-parallel outputs are this rank's PARTIAL sums: the library runs no collective.  With both
 * phases selected the rank's own partial stands in for the reduced sum (exact when the degree is
 * 1); with a single phase selected the call returns the pure partial, so that a caller can put a
 * reduction between the two halves.
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless stated otherwise, owned by the caller, 16-byte
 *     aligned, and must stay valid until the work queued on `hip_stream` has completed.
 *   - All matrices are row-major and dense.  T = micro_batch * seq tokens, token t = b * seq + s.
 *     H = hidden, dh = H / heads, Hl = (heads / tp_attn) * dh, Fl = ffn / tp_ffn.
 *       x, y, dy, dx, p_attn, p_mlp : [T, H]
 *       w_qkv [H, 3*Hl]  columns ordered [Q heads | K heads | V heads], dh columns per head
 *       b_qkv [3*Hl]     w_o [Hl, H]   b_o [H]   w_fc1 [H, Fl]   b_fc1 [Fl]   w_fc2 [Fl, H]   b_fc2 [H]
 *       ln1_g, ln1_b, ln2_g, ln2_b : [H]
 *     ("in x out": y = x * W).  Weights are passed ALREADY SHARDED: rank r's column shard is
 *     columns [r*Hl, (r+1)*Hl) of each of Wq, Wk, Wv (resp. [r*Fl, (r+1)*Fl) of W1); its row shard
 *     is the same index range of the rows of Wo / W2.
 *   - Activations and parameters have the element type cfg->dtype (fp32, or bf16 with fp32
 *     accumulation); parameter gradients are fp32 (GX_WGRAD_BF16: the weight matrices' in bf16).
 *   - Variants selected by flags: tanh-form GELU (GX_GELU_TANH), dropout of the attention
 *     probabilities and of each half's output (GX_DROPOUT), recomputation of the activations in
 *     the backward call (GX_RECOMPUTE), gradient accumulation (GX_ACCUM_WGRAD).  Since the calls
 *     only enqueue kernels and event operations, a caller may capture them into a HIP graph after
 *     one ordinary call has created the library's streams and events.
 *   - Calls only enqueue work (a hipStream_t, or NULL for the default stream); they never allocate
 *     device memory, free or synchronise the host, and results are bitwise reproducible run to
 *     run.  gx_layer_bwd forks part of its work (the weight-gradient products and the stage-1 sums
 *     of a bias gradient) onto a stream that the library creates on first use (default priority,
 *     non-blocking; one per host thread and device, with its events) and joins it back with events
 *     before returning: to the caller everything is ordered on `hip_stream` as if it had run there
 *     (gx_set_overlap(0) really runs it there).  Calls from different host threads may overlap;
 *     two calls that share a `workspace` or `saved` block may not.  The gx_set_overlap switch and
 *     the optional timing record of gx_prof_* are process-global.
 *   - Errors are returned as gx_status; nothing is thrown across the boundary.  Configuration and
 *     pointer checks happen before anything is enqueued.
 */
#ifndef GX_H_
#define GX_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GX_OK = 0,
  GX_ERR_NULL = 1,      /* a required pointer is NULL */
  GX_ERR_SHAPE = 2,     /* a size is non-positive or outside what the kernels support */
  GX_ERR_DIVIS = 3,     /* hidden % heads, heads % tp_attn, ffn % tp_ffn or a vector width fails */
  GX_ERR_DTYPE = 4,     /* dtype is not GX_F32 / GX_BF16 */
  GX_ERR_ALIGN = 5,     /* a pointer is not 16-byte aligned */
  GX_ERR_FLAGS = 6,     /* no phase selected, or unknown flag bits */
  GX_ERR_ARCH = 7,      /* the current device is not gfx950 */
  GX_ERR_LAUNCH = 8,    /* the HIP runtime refused a launch; see hipGetLastError */
  GX_ERR_INFEASIBLE = 9 /* gx_plan_search: no assignment fits the memory budget */
} gx_status;

typedef enum { GX_F32 = 0, GX_BF16 = 1 } gx_dtype;

enum {
  GX_PHASE_ATTN = 1,      /* run the attention half */
  GX_PHASE_MLP = 2,       /* run the feed-forward half (both bits: the whole block) */
  GX_ROW_BIAS_ATTN = 4,   /* this rank adds b_o to p_attn (exactly one rank of a group should) */
  GX_ROW_BIAS_MLP = 8,    /* this rank adds b_fc2 to p_mlp */
  GX_ACCUM_WGRAD = 16,    /* backward: add into the parameter gradients instead of overwriting */
  GX_RECOMPUTE = 32,      /* backward: recompute the forward activations from x; `saved` unused */
  GX_GELU_TANH = 64,      /* feed-forward activation 0.5 z (1 + tanh(sqrt(2/pi) (z + 0.044715 z^3))) instead of
                             the erf form; pass the same flag to the forward and the backward call */
  GX_WGRAD_BF16 = 128,    /* backward, bf16 configurations only: the four weight-matrix gradients (w_qkv, w_o,
                             w_fc1, w_fc2 of gx_grads) point to bf16 buffers; each element is the fp32
                             accumulator rounded once (with GX_ACCUM_WGRAD: old bf16 value + accumulator, added
                             in fp32 and rounded once).  Bias and LayerNorm gradients stay fp32. */
  GX_FWD_SAVED_ONLY = 512,/* forward: compute only what gx_layer_bwd needs, into `saved` (no FC2 product, no output
                             projection of a lone attention phase); y, p_attn and p_mlp are not written and may
                             be NULL.  For callers that recompute activations themselves, e.g. on another
                             stream ahead of the backward pass; gx_layer_bwd ignores the flag. */
  GX_DROPOUT = 256        /* dropout variant: cfg->drop_attn, drop_hidden and drop_seed_* are read (without
                             the flag they are ignored).  Pass the same values to the forward and the backward
                             call.  Both passes then need a workspace (gx_layer_workspace_bytes). */
};

/* One rank's share of one block.  tp_rank is informational (which shard the caller passed). */
typedef struct {
  int32_t hidden, heads, ffn;
  int32_t tp_attn, tp_ffn, tp_rank;
  int32_t seq, micro_batch;
  int32_t dtype;            /* gx_dtype */
  int32_t flags;            /* GX_PHASE_* | GX_ROW_BIAS_* | GX_ACCUM_WGRAD | GX_RECOMPUTE | GX_GELU_TANH | GX_WGRAD_BF16 |
                               GX_DROPOUT | GX_FWD_SAVED_ONLY */
  float ln_eps;             /* LayerNorm epsilon (inside the square root; biased variance) */
  /* Dropout (only with GX_DROPOUT).  Probabilities are given in 1/256ths, 0..255.  Random bytes come
   * from Philox4x32-10 keyed by the 64-bit seed (drop_seed_lo, drop_seed_hi); the 16 bytes of one
   * counter (output words in order, least-significant byte first) serve 16 consecutive elements;
   * an element is dropped iff its byte < the probability, and kept elements are multiplied by
   * 256 / (256 - probability).
   *   drop_attn  : attention probabilities P[b, head, i, j] after the softmax; counter
   *                (i, j / 16, b * heads + global head, 1), byte j % 16, where the global head is
   *                (tp_rank % tp_attn) * (heads / tp_attn) + local head, so that the ranks of a group
   *                draw the masks of the unsharded layer.
   *   drop_hidden: with both phases in one call, p_attn and p_mlp (bias included) before they are added
   *                to the residual stream; counter (token, column / 16, 0, 2 for p_attn or 3 for p_mlp),
   *                byte column % 16.  A single-phase call returns its partial sum undropped; the p_attn /
   *                p_mlp extra outputs of a two-phase call are the undropped values too. */
  int32_t drop_attn, drop_hidden;
  uint32_t drop_seed_lo, drop_seed_hi;
} gx_layer_cfg;

/* Parameter shards, element type cfg->dtype.  Pointers of a phase that is not selected may be NULL. */
typedef struct {
  const void *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_o, *b_o;
  const void *ln2_g, *ln2_b, *w_fc1, *b_fc1, *w_fc2, *b_fc2;
} gx_params;

/* Parameter gradients, same shapes as the parameters: fp32, except that with GX_WGRAD_BF16 the four
 * weight-matrix pointers are reinterpreted as bf16 buffers. */
typedef struct {
  float *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_o, *b_o;
  float *ln2_g, *ln2_b, *w_fc1, *b_fc1, *w_fc2, *b_fc2;
} gx_grads;

/* Host-only check of a configuration (no GPU needed): sizes positive, hidden % heads == 0,
 * heads % tp_attn == 0, ffn % tp_ffn == 0, 0 <= tp_rank < max(tp_attn, tp_ffn), at least one phase,
 * no unknown flag, GX_WGRAD_BF16 only with dtype bf16 (else GX_ERR_DTYPE), with GX_DROPOUT both
 * probabilities in 0..255 (else GX_ERR_SHAPE), and the kernels' limits: bf16 needs head dim 64 or 128, hidden and Fl multiples of 8,
 * hidden <= 8192; fp32 needs head dim <= 128 and hidden, Fl multiples of 4, hidden <= 4096,
 * seq <= 8192; every activation tensor must stay below 2 GiB. */
gx_status gx_layer_validate(const gx_layer_cfg* cfg);

/* Bytes of the opaque `saved` block (activations the forward pass keeps for the backward pass)
 * and of the opaque `workspace` block (scratch; is_backward selects the pass, and with
 * GX_RECOMPUTE the backward workspace includes room for the recomputed activations).  Both depend
 * on cfg's sizes, dtype and flags; 0 is returned for an invalid cfg. */
size_t gx_layer_saved_bytes(const gx_layer_cfg* cfg);
size_t gx_layer_workspace_bytes(const gx_layer_cfg* cfg, int is_backward);

/* Forward pass (attention and feed-forward halves as defined at the top of this file).
 *   both phases : x [T,H] in, y [T,H] out; p_attn / p_mlp optional extra outputs (NULL to skip).
 *   ATTN only   : x in, p_attn out (required); y, p_mlp ignored.
 *   MLP only    : x holds h1, p_mlp out (required); y, p_attn ignored.
 * `saved` (gx_layer_saved_bytes) receives the activations gx_layer_bwd needs; `workspace` may be
 * NULL when gx_layer_workspace_bytes(cfg, 0) is 0. */
gx_status gx_layer_fwd(const gx_layer_cfg* cfg, const gx_params* params, const void* x, void* y, void* p_attn,
                       void* p_mlp, void* saved, void* workspace, void* hip_stream);

/* Backward pass: the exact gradient of what gx_layer_fwd computes for the same cfg.
 *   both phases : dy = dL/dy in, dx = dL/dx out.
 *   ATTN only   : dy = dL/dp_attn in, dx = the gradient reaching x through LayerNorm 1 only.
 *   MLP only    : x holds h1, dy = dL/dp_mlp in, dx = the gradient reaching h1 through LayerNorm 2.
 * Gradients of the selected phases' parameters are written (or, with GX_ACCUM_WGRAD, added) to
 * `grads`; a row-parallel bias whose GX_ROW_BIAS_* flag is off gets a zero gradient.  `saved` must
 * come from gx_layer_fwd with the same cfg, params and x (ignored with GX_RECOMPUTE).  dx may not
 * alias x or dy. */
gx_status gx_layer_bwd(const gx_layer_cfg* cfg, const gx_params* params, const void* x, const void* dy, void* dx,
                       const gx_grads* grads, const void* saved, void* workspace, void* hip_stream);

/* gx_layer_bwd for callers that cannot allocate device memory or let a library do so (code under
 * HIP graph capture, tight serving or training loops, harnesses that forbid it): the same backward
 * pass with the same arguments except `workspace`, which is replaced by an array of
 * GX_STATIC_SCRATCH_BYTES that lives in the library's device image (one per GPU, held until the
 * process ends).  The call allocates and frees nothing, creates no stream or event, and queues
 * every kernel on `hip_stream` in order (as gx_layer_bwd does after gx_set_overlap(0)); results are
 * bit-identical to gx_layer_bwd's.  A configuration whose gx_layer_workspace_bytes(cfg, 1) exceeds
 * GX_STATIC_SCRATCH_BYTES is refused with GX_ERR_SHAPE before anything is queued; GX_ERR_LAUNCH
 * also reports a failed lookup of the array's device address (done once per device, on the first
 * call there).  Every call on a GPU uses that GPU's one array: the array keeps the previous call's
 * contents (nothing in it needs clearing, each part is written before it is read), and two calls
 * whose work overlaps on one GPU (different streams, or host threads) race on it. */
#define GX_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
gx_status gx_layer_bwd_static(const gx_layer_cfg* cfg, const gx_params* params, const void* x, const void* dy,
                              void* dx, const gx_grads* grads, const void* saved, void* hip_stream);

/* Optional per-launch timing, for benchmarks and cost tables (the paper's section 3 "Profilers"
 * feed per-layer costs to the strategy selector; this is the per-kernel source of such costs).
 * While enabled, every kernel launch site inside gx_layer_fwd / gx_layer_bwd is bracketed by a
 * pair of HIP events on the call's stream and tagged with a kernel class:
 *   GX_KC_LN_FWD, GX_KC_LN_BWD (input gradient and partial parameter sums in one kernel),
 *   GX_KC_ATTN_FWD, GX_KC_ATTN_BWD (its three kernels together), GX_KC_COLSUM (a stage-1 pass of
 *   a bias gradient, or the one launch that finishes every column sum of the backward pass),
 *   GX_KC_DROPOUT (mask generation and the
 *   dropout passes over a half's output or its gradient), and GX_KC_GEMM + 10 * layout + epilogue
 *   with layout 0 = A[M,K] B[K,N], 1 = A[M,K] B[N,K], 2 = A[K,M] B[K,N] and epilogue 0 = store,
 *   1 = +bias, 2 = +bias +residual, 3 = +bias then GELU, 4 = times GELU', 5 = fp32 store,
 *   6 = fp32 accumulate.
 * gx_prof_enable(1) creates the events on first use (the only allocation the library ever makes)
 * and clears the record; gx_prof_enable(0) stops recording.  gx_prof_collect waits for the
 * recorded events, writes up to `capacity` (class, milliseconds) pairs to HOST arrays in launch
 * order, clears the record and returns the count (-1 on a HIP error).  At most 8192 launches are
 * recorded between collects; later ones are silently not timed.  Process-global state, not
 * thread-safe; leave it off in production loops (the event records perturb timing slightly). */
/* gx_set_overlap(0) makes gx_layer_bwd queue everything on the caller's stream, in order, instead
 * of forking part of it onto the library's side streams (the default, 1).  Results are identical
 * either way; the serial form is for timing kernels one at a time (with gx_prof_* or a profiler),
 * since kernels that overlap share the chip and their individual durations stretch. */
gx_status gx_set_overlap(int on);

enum { GX_KC_LN_FWD = 1, GX_KC_LN_BWD = 2, GX_KC_ATTN_FWD = 3, GX_KC_ATTN_BWD = 4, GX_KC_COLSUM = 5,
       GX_KC_DROPOUT = 6,
       GX_KC_GEMM = 100 };
gx_status gx_prof_enable(int on);
int gx_prof_collect(int* kernel_class, float* ms, int capacity);

/* Measured ceilings of the chip, to hold the layer's kernels against (benchmarks only; both calls
 * create two HIP events, queue their work on `hip_stream`, wait for it and destroy the events):
 *   gx_peak_mfma : `launches` launches of a register-only v_mfma_f32_32x32x16_bf16 loop (1024
 *                       workgroups of 4 wavefronts, 4 independent accumulators each, no memory
 *                       traffic); *tflops receives the sustained rate.  `scratch`: at least 64
 *                       bytes of device memory (never written in practice).
 *   gx_peak_copy      : `launches` copies of `bytes` (a multiple of 16) from src to dst, 16 bytes per
 *                       lane, grid-stride; *gbytes_per_s receives read + write bytes per second.
 * Errors: GX_ERR_NULL, GX_ERR_SHAPE (launches outside 1..1000, bytes), GX_ERR_ALIGN, GX_ERR_ARCH,
 * GX_ERR_LAUNCH. */
gx_status gx_peak_mfma(void* scratch, int launches, double* tflops, void* hip_stream);
gx_status gx_peak_copy(const void* src, void* dst, size_t bytes, int launches, double* gbytes_per_s,
                       void* hip_stream);

/* ------------------------------------------------------------------------------------------
 * Neighbours of the layer step: the optimizer update and the re-partitioning of a block's
 * parameters between tensor-parallel degrees.  Both are memory-bound passes over device arrays.
 * ------------------------------------------------------------------------------------------ */

/* AdamW on a flat range of n elements (the paper's section 3 "Microsoft DeepSpeed" and section 5.2
 * place partitioned fp32 optimizer states next to the layer compute; a rank passes the range it
 * owns).  Per element, with g' = grad_scale * grad and t = step >= 1:
 *     m = beta1 m + (1 - beta1) g';   v = beta2 v + (1 - beta2) g'^2
 *     w = w - lr * ( (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps) + weight_decay * w )
 * master, m, v : fp32 [n], updated in place;  grad : fp32 [n], read only;
 * param_out    : optional copy of the new w in param_dtype (GX_BF16: round to nearest even;
 *                GX_F32), [n]; NULL to skip.  Arithmetic is fp32.
 * n = 0 is a no-op.  Errors: GX_ERR_NULL (cfg or a required array), GX_ERR_SHAPE (step < 1, a beta
 * outside [0, 1), n >= 2^40), GX_ERR_DTYPE, GX_ERR_ALIGN (16 bytes), GX_ERR_ARCH, GX_ERR_LAUNCH. */
typedef struct {
  float lr, beta1, beta2, eps, weight_decay, grad_scale;
  int32_t step;
} gx_adamw_cfg;
gx_status gx_adamw_step(const gx_adamw_cfg* cfg, size_t n, float* master, float* m, float* v, const float* grad,
                        void* param_out, int param_dtype, void* hip_stream);

/* Shard transitions (the paper's section 4, "Handling Transitions": going to model parallelism
 * cuts a rank's shard out of whole weights, going back puts shards side by side again).
 * `whole` holds the unsharded block (w_qkv [H, 3H] with column blocks [Q | K | V], w_o [H, H],
 * w_fc1 [H, F], b_fc1 [F], w_fc2 [F, H]); `shard` holds one rank's tensors at cfg's degrees,
 * laid out as gx_layer_fwd takes them.  The rank is tp_rank % tp_attn for the attention half and
 * tp_rank % tp_ffn for the feed-forward half.
 *   gx_params_slice : shard <- the rank's part of whole   (whole is read, shard written)
 *   gx_params_merge : whole <- shard, in the rank's place (shard is read; other ranks' parts of
 *                     whole are left untouched)
 * LayerNorm parameters and the row-parallel biases b_o, b_fc2 are whole on every rank and are
 * copied as they are.  cfg->flags selects the halves (GX_PHASE_*); cfg->dtype is the element type
 * of every tensor, so the same calls move fp32 master weights, moments or gradients.  Only
 * hidden, heads, ffn, tp_*, dtype and the phase bits of cfg are used (seq and micro_batch are
 * ignored, and the layer kernels' size limits do not apply), but H/tp_attn and F/tp_ffn must be
 * multiples of 16 bytes' worth of elements.  Source and destination must not overlap.
 * Errors: GX_ERR_NULL, GX_ERR_SHAPE, GX_ERR_DIVIS, GX_ERR_DTYPE, GX_ERR_ALIGN, GX_ERR_FLAGS,
 * GX_ERR_ARCH, GX_ERR_LAUNCH; checks happen before anything is enqueued. */
typedef struct {
  void *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_o, *b_o;
  void *ln2_g, *ln2_b, *w_fc1, *b_fc1, *w_fc2, *b_fc2;
} gx_params_out;
gx_status gx_params_slice(const gx_layer_cfg* cfg, const gx_params* whole, const gx_params_out* shard,
                          void* hip_stream);
gx_status gx_params_merge(const gx_layer_cfg* cfg, const gx_params* shard, const gx_params_out* whole,
                          void* hip_stream);

/* ------------------------------------------------------------------------------------------
 * Layer-wise strategy plan (host only, no GPU involved).  The paper's strategy selector, in its
 * discovery phase (section 3, "Dynamic Strategy Selector"; section 2, "Layer-Specific Parallelism
 * Optimization"), prunes the candidate strategies with a decision tree and then runs a dynamic
 * program over the layers, driven by a cost model; neither the model nor the recurrence is
 * printed, so the problem solved here is the plainest one of that shape:
 *     choose one of `strategies` per layer so that the layers' memories (each first rounded up
 *     to a multiple of mem_quantum_bytes when that is > 0) sum to at most mem_budget_bytes,
 *     minimising  sum_l time_ms[l][c_l] + sum_{l>0} switch_ms[c_{l-1}][c_l].
 * Rounding rule: with q = mem_quantum_bytes > 0 a memory x becomes k * q for the least whole
 * number k whose product k * q, formed in double precision, is not below x.  A memory that is
 * such a product already stays as it is; one that exceeds it by a single unit in the last place
 * moves up to (k + 1) * q; no tolerance is applied.
 * The cost table is what a sweep of gx_layer_fwd / gx_layer_bwd over shard shapes measures.
 * Pruning: strategies that cannot fit beside the other layers' least memories; without switching
 * costs also strategies that another one beats or equals in both time and memory.  Search: exact
 * dynamic program whose state is the last layer's strategy with a Pareto frontier of (memory,
 * time); ties in total time go to less memory.
 * All pointers are HOST pointers owned by the caller; `choice` receives `layers` strategy indices.
 * Errors: GX_ERR_NULL, GX_ERR_SHAPE (sizes <= 0 or > 4096 layers / 1024 strategies, negative or
 * non-finite costs, or a frontier beyond 4 M points: use a coarser quantum), GX_ERR_INFEASIBLE. */
typedef struct {
  int32_t layers, strategies;
  const double* time_ms;     /* [layers][strategies] */
  const double* mem_bytes;   /* [layers][strategies] */
  const double* switch_ms;   /* [strategies][strategies], diagonal ignored; NULL: switching is free */
  double mem_budget_bytes;
  double mem_quantum_bytes;  /* 0: memories are used as given */
} gx_plan_problem;
typedef struct {
  double total_ms, total_mem_bytes;   /* of the returned plan (memory after rounding) */
  int64_t pruned;                      /* (layer, strategy) pairs removed before the search */
  int64_t frontier_peak;               /* largest Pareto frontier met */
} gx_plan_result;
gx_status gx_plan_search(const gx_plan_problem* problem, int32_t* choice, gx_plan_result* result);

/* Cost model of one layer under one strategy (host only): the part of the cost table that is
 * computed rather than measured.  The paper's model profiler (section 3, "Model Profiler") records
 * parameter counts and per-layer memory, and its selector weighs communication overhead (section 3,
 * "Dynamic Strategy Selector"); it prints no formula, so the model is the textbook one:
 *   - a strategy is (tp_attn, tp_ffn) on a group of `gpus` devices, the rest of the group data
 *     parallel: a half of degree d runs micro-batches of global_batch * d / gpus samples
 *     (GX_ERR_DIVIS when that is not a whole number, or when a degree does not divide the group,
 *     the heads or the FFN width);
 *   - attn_elems / ffn_elems: elements of one rank's parameter shards of each half (LayerNorm gain
 *     and bias [H] each, the column-parallel matrix and its bias, the row-parallel matrix, the
 *     row-parallel bias [H]);  state_bytes = (attn_elems + ffn_elems) * (e + 16) with e the bytes
 *     of the storage type: the parameter itself, its fp32 gradient, fp32 master copy and two fp32
 *     optimizer moments;
 *   - ring all-reduce of n bytes over p ranks: every rank sends and receives 2 (p - 1) / p * n
 *     bytes, taken at link_gbps * 1e9 bytes per second; 0 for p = 1.
 *     tp_comm_ms: per half two all-reduces of its [micro_batch * seq, hidden] activations (one in
 *     the forward pass after the row-parallel product, one in the backward pass after the
 *     column-parallel input gradient) over its tensor-parallel group;
 *     dp_comm_ms: one all-reduce of each half's fp32 gradients (4 bytes per element) over its
 *     data-parallel group of gpus / degree ranks;
 *   - switch_ms: handing activations to a next layer whose attention degree differs from this
 *     layer's feed-forward degree: every GPU moves its 1/gpus share of the step's
 *     [global_batch * seq, hidden] activations once forward and once backward;
 *   - flops_attn / flops_ffn: model FLOPs per GPU of each half, forward + backward (backward twice
 *     the forward), causal attention counted on the seq (seq + 1) / 2 unmasked pairs.
 * Errors: GX_ERR_NULL, GX_ERR_DTYPE, GX_ERR_SHAPE (a non-positive size or bandwidth), GX_ERR_DIVIS. */
typedef struct {
  int32_t hidden, heads, ffn, seq;
  int32_t dtype;                 /* gx_dtype of parameters and activations */
  int32_t gpus, global_batch;
  int32_t tp_attn, tp_ffn;
  double link_gbps;
} gx_strategy_query;
typedef struct {
  int64_t micro_batch_attn, micro_batch_ffn;
  int64_t attn_elems, ffn_elems;
  double state_bytes;
  double tp_comm_ms, dp_comm_ms, switch_ms;
  double flops_attn, flops_ffn;
} gx_strategy_costs;
gx_status gx_strategy_cost(const gx_strategy_query* query, gx_strategy_costs* costs);

/* ---- Pipeline regrouping (host only) ------------------------------------------------------------
 * Paper section 4 "Handling Transitions": a pipeline-parallel transition changes how layers are
 * grouped; the groups are formed anew and every process is told which layers to hold.  The paper
 * gives no rule for the grouping.  This library's reading: a stage holds consecutive layers, every
 * stage at least one, and the grouping makes the slowest stage (the pipeline's bottleneck) as fast
 * as possible given a time per layer, e.g. a column of the cost table.  Among the groupings that
 * reach the smallest bottleneck the one returned has every stage, from the first on, as short as it
 * can be.  Exact search (dynamic program over (stage, first layer)); host memory only.
 *
 * gx_stage_partition
 *   layers, stages : 1 <= stages <= layers <= 65536, stages <= 4096
 *   layer_ms       : host, `layers` positive finite times, or NULL for equal times
 *   first          : host, out, stages + 1 entries; stage s holds layers first[s] .. first[s+1]-1,
 *                    first[0] = 0, first[stages] = layers
 *   bottleneck_ms  : host, out, the largest stage time (sum of its layers' times); may be NULL
 * gx_stage_moves: what a change of grouping moves.
 *   old_first, new_first : host, groupings of the same `layers` layers in the format above
 *   new_stage_of         : host, out, `layers` entries: the stage that holds each layer afterwards
 *   moved                : host, out, number of layers whose stage index changes
 * Errors: GX_ERR_NULL, GX_ERR_SHAPE (sizes out of range, a non-positive or non-finite time, a
 * grouping that is not increasing from 0 to layers). */
gx_status gx_stage_partition(int32_t layers, int32_t stages, const double* layer_ms, int32_t* first,
                             double* bottleneck_ms);
gx_status gx_stage_moves(int32_t layers, int32_t old_stages, const int32_t* old_first, int32_t new_stages,
                         const int32_t* new_first, int32_t* new_stage_of, int32_t* moved);

/* Static strings; never NULL. */
const char* gx_status_str(gx_status s);
const char* gx_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GX_H_ */
