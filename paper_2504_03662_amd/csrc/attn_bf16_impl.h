// Body of the bf16 attention kernels for one head dimension.  Included by attn_bf16.hip once per
// supported head dimension, inside a namespace of its own, with GX_ATTN_DH defined.
constexpr int DH = GX_ATTN_DH;         // head dimension of this instantiation (128 or 64)
constexpr int ROWB = DH * 2;           // bytes per tile row
constexpr int CPR = DH / 8;            // 16 B chunks per tile row
static_assert(DH == 128 || DH == 64, "tile swizzles are worked out for these two row lengths");

// 16 B chunk c of tile row r lives at chunk c ^ swz(r), chosen so that both access patterns of a
// tile are free of bank conflicts: ds_read_b128 of 16 consecutive rows at one logical chunk, and
// the transposing read of 4 consecutive rows x 64 B.
//   256 B rows: the low row bits move whole 64 B groups (the 4 rows of a transposing read fall in
//   distinct banks); the next two bits permute inside a group.
//   128 B rows: two rows share a 256 B bank window, so the swizzle depends on r / 2: its low bit
//   flips the 64 B group (rows r and r + 2 of a transposing read), the rest permutes inside it;
//   it is a bijection of (r / 2) % 8 onto the 8 chunks, which keeps 16 consecutive rows distinct.
GX_DEVINL int swz(int r) {
  if (DH == 128) return ((r & 3) << 2) | ((r >> 2) & 3);
  const int x = (r >> 1) & 7;
  return ((x & 1) << 2) | (x >> 1);
}

// direct-to-LDS load of ROWS x DH starting at global row `row0` of one (sample, head, q|k|v)
// column block; rows at or beyond `nrows` are zero-filled.  elem0 = element offset of (row 0,
// first column) from the tensor start; ld = row stride in elements.
template <int ROWS, int NW>
GX_DEVINL void tile_load(__amdgpu_buffer_rsrc_t rsrc, unsigned elem0, int ld, int row0, int nrows, char* dst,
                         int wave, int lane) {
  constexpr int RPI = 64 / CPR;                        // rows per 64-lane instruction
  constexpr int PER_WAVE = ROWS / RPI / NW;
  static_assert(PER_WAVE >= 1, "tile too small for the workgroup");
#pragma unroll
  for (int i = 0; i < PER_WAVE; i++) {
    const int q = wave * PER_WAVE + i;
    const int r = RPI * q + lane / CPR;
    const int c = (lane % CPR) ^ swz(r);
    const unsigned off = (row0 + r < nrows) ? (elem0 + (unsigned)((row0 + r) * ld + c * 8)) * 2u : OOB;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_ptr)(dst + q * 1024), 16, off, 0, 0, 0);
  }
}

// The same load for a kernel that brings in many tiles of one column block: the lane's byte offsets
// within a tile are worked out once, and a tile that lies wholly inside the rows puts its first
// row into the instruction's scalar offset (which takes no part in the range check, hence the
// condition), so that a load costs no vector arithmetic; a ragged last tile takes tile_load().
template <int ROWS, int NW>
struct TileStream {
  static constexpr int RPI = 64 / CPR, PER_WAVE = ROWS / RPI / NW;
  static_assert(PER_WAVE >= 1, "tile too small for the workgroup");
  unsigned voff[PER_WAVE];
  GX_DEVINL void init(unsigned elem0, int ld, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < PER_WAVE; i++) {
      const int r = RPI * (wave * PER_WAVE + i) + lane / CPR;
      const int c = (lane % CPR) ^ swz(r);
      voff[i] = (elem0 + (unsigned)(r * ld + c * 8)) * 2u;
    }
  }
  GX_DEVINL void load(__amdgpu_buffer_rsrc_t rsrc, unsigned elem0, int ld, int row0, int nrows, char* dst, int wave,
                      int lane) const {
    if (row0 + ROWS <= nrows) {
      const unsigned so = (unsigned)(row0 * ld) * 2u;
#pragma unroll
      for (int i = 0; i < PER_WAVE; i++) {
        unsigned off = voff[i];
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_ptr)(dst + (wave * PER_WAVE + i) * 1024), 16, off,
                                                 so, 0, 0);
      }
    } else {
      tile_load<ROWS, NW>(rsrc, elem0, ld, row0, nrows, dst, wave, lane);
    }
  }
};

// MFMA operand whose 32 rows are tile rows r0..r0+31 and whose reduction index is the head
// dimension (step s covers d = 16 s .. 16 s + 15)
GX_DEVINL bf16x8 frag_rows(const char* tile, int r, int s, int g) {
  const int c = (2 * s + g) ^ swz(r);
  return *reinterpret_cast<const bf16x8*>(tile + r * ROWB + (c << 4));
}
// MFMA operands whose 32 rows are head-dim columns 32 dt .. 32 dt + 31 and whose reduction index
// runs over 16 tile rows starting at a multiple of 16, in the slot order of an accumulator column
// (slot (g, e) <-> row 8 (e / 4) + 4 g + e % 4 of the group), come from transposing reads issued
// as untracked asm (see lds_read_tr_issue): the four
// head-dim blocks of the 16 tile rows starting at 16 * GI, from per-lane addresses prepared by
// cols_lane_offsets() plus the tile's LDS address.  The caller waits (lds_wait_le) and pins.
GX_DEVINL void cols_lane_offsets(int lane, unsigned (&off)[2][DH / 32]) {
  const int g = lane >> 5, s = lane & 15, hb = (lane >> 4) & 1;
#pragma unroll
  for (int half = 0; half < 2; half++) {
    const int r = 4 * g + (s >> 2) + 8 * half;       // swz(16 k + r) == swz(r)
#pragma unroll
    for (int dt = 0; dt < DH / 32; dt++) {
      const int d0 = 32 * dt + 16 * hb + 4 * (s & 3);
      off[half][dt] = (unsigned)(r * ROWB + (((d0 >> 3) ^ swz(r)) << 4) + (d0 & 7) * 2);
    }
  }
}
struct ColFrags {
  bf16x4 lo[DH / 32], hi[DH / 32];
};
template <int GI>
GX_DEVINL void cols_issue(unsigned tile, const unsigned (&off)[2][DH / 32], ColFrags& f) {
#pragma unroll
  for (int dt = 0; dt < DH / 32; dt++) {
    f.lo[dt] = lds_read_tr_issue<GI * 16 * ROWB>(tile + off[0][dt]);
    f.hi[dt] = lds_read_tr_issue<GI * 16 * ROWB>(tile + off[1][dt]);
  }
}
GX_DEVINL bf16x8 cols_get(ColFrags& f, int dt) {
  lds_pin(f.lo[dt]);
  lds_pin(f.hi[dt]);
  return __builtin_shufflevector(f.lo[dt], f.hi[dt], 0, 1, 2, 3, 4, 5, 6, 7);
}

// registers v = 8 h .. 8 h + 7 of an accumulator, rounded to bf16, as an MFMA operand
GX_DEVINL bf16x8 pack_half(const f32x16& a, int h) {
  bf16x8 o;
#pragma unroll
  for (int e = 0; e < 8; e++) o[e] = (bf16)a[8 * h + e];
  return o;
}

GX_DEVINL f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int v = 0; v < 16; v++) z[v] = 0.f;
  return z;
}

// this lane's 8 steps of a 32-row operand read straight from global memory (row clamped)
GX_DEVINL void load_row_frags(const bf16* base, int ld, int row, int nrows, int g, bf16x8 (&out)[DH / 16]) {
  const bf16* p = base + (size_t)min(row, nrows - 1) * ld + 8 * g;
#pragma unroll
  for (int s = 0; s < DH / 16; s++) out[s] = *reinterpret_cast<const bf16x8*>(p + 16 * s);
}


// acc[dt] += product of the transposed fragments of a tile of 16 * NG16 rows (groups of 16 rows at
// LDS address `ct`) with xf[group]; COLS_A puts the transposed fragment first (rows of the result =
// head-dim columns).  Groups 0 and 1 must have been issued into cf[0], cf[1] by the caller (as
// early as it likes, to cover LDS latency with its own work); with four groups, groups 2 and 3
// are issued here, so that two groups are always in flight.
template <bool COLS_A, int NG16>
GX_DEVINL void tr_product(f32x16 (&acc)[DH / 32], unsigned ct, const unsigned (&coff)[2][DH / 32],
                          ColFrags (&cf)[2], const bf16x8 (&xf)[NG16]) {
  static_assert(NG16 == 2 || NG16 == 4, "tiles of 32 or 64 rows");
#define GX_TR_GROUP(U, BUF)                                                                              \
  _Pragma("unroll") for (int dt = 0; dt < DH / 32; dt++)                                                 \
      acc[dt] = COLS_A ? MFMA(cols_get(cf[BUF], dt), xf[U], acc[dt]) : MFMA(xf[U], cols_get(cf[BUF], dt), acc[dt])
  lds_wait_le<2 * (DH / 32)>();
  GX_TR_GROUP(0, 0);
  if (NG16 == 4) {
    cols_issue<2>(ct, coff, cf[0]);
    lds_wait_le<2 * (DH / 32)>();
    GX_TR_GROUP(1, 1);
    cols_issue<3>(ct, coff, cf[1]);
    lds_wait_le<2 * (DH / 32)>();
    GX_TR_GROUP(NG16 - 2, 0);
    lds_wait_all();
    GX_TR_GROUP(NG16 - 1, 1);
  } else {
    lds_wait_all();
    GX_TR_GROUP(1, 1);
  }
#undef GX_TR_GROUP
}
template <bool COLS_A>
GX_DEVINL void tr_product4(f32x16 (&acc)[DH / 32], unsigned ct, const unsigned (&coff)[2][DH / 32],
                           ColFrags (&cf)[2], const bf16x8 (&xf)[4]) {
  tr_product<COLS_A, 4>(acc, ct, coff, cf, xf);
}

// ------------------------------------------------------------------------------- forward
// A workgroup owns 32 NQ query rows of one (sample, head); its NQ * SPLIT wavefronts are NQ blocks
// of 32 rows times SPLIT shares of the keys: every step brings SPLIT tiles of BKV keys (K and V)
// into LDS and wavefront (q, part) works on tile `part`; the SPLIT partial softmax states
// (max, sum, O) of a row block are merged through LDS at the end, in the order of `part`.
//   many (sample, head) pairs : NQ 4, SPLIT 1, BKV 64 (4 wavefronts, two workgroups per compute unit)
//   few pairs                 : NQ 2, SPLIT 2, BKV 32 (4 wavefronts, two workgroups per compute unit;
//     the forward pass in the kernel after this one): the causal triangle gives query blocks
//     between 1 and S / 32 NQ units of work, so with few pairs the chip is filled by short blocks
//     cut fine, each with its keys spread over two wavefronts.  Two independent workgroups per
//     unit matter more than wavefronts per workgroup: the wavefronts of one workgroup pass every
//     step's barrier together and are then all in the matrix pipe or all in the vector units at
//     once, while two workgroups drift apart and fill each other's gaps.
// Workgroups are numbered longest query block first over the whole launch (all pairs' last blocks,
// then all pairs' next-to-last blocks, ...): the hardware hands them out in that order.
// Dropout of the probabilities: keep bits (1 = kept) of the whole launch, `wpr` 32-bit words per
// row; row-major (a query's keys) for the forward and dQ kernels, column-major (a key's queries)
// for the dK / dV kernel.  Kept probabilities are multiplied by `scale`.
struct KeepArgs {
  const unsigned* bits;
  int wpr;
  float scale;
};
// The keep bits of a lane's NJT 32 x 32 accumulator tiles: zero the values whose bit is clear.
// Accumulator register v of tile jt sits at bit 32 jt + 8 (v / 4) + 4 g + v % 4.
template <int NJT>
GX_DEVINL void drop_unkept(f32x16 (&a)[NJT], unsigned long long kw, int g) {
#pragma unroll
  for (int jt = 0; jt < NJT; jt++) {
    const unsigned w = (unsigned)(kw >> (32 * jt)) >> (4 * g);
#pragma unroll
    for (int v = 0; v < 16; v++)
      if (!((w >> (8 * (v >> 2) + (v & 3))) & 1u)) a[jt][v] = 0.f;
  }
}
// this lane's keep bits of the BKV keys starting at key j0 of one query row (bits: the row's words)
template <int NJT>
GX_DEVINL unsigned long long keep_bits_of_step(const unsigned* row_words, int j0) {
  if (NJT == 2) return *reinterpret_cast<const unsigned long long*>(row_words + (j0 >> 5));
  return row_words[j0 >> 5];
}

// End of a forward workgroup: merge the SPLIT partial softmax states of each row block through LDS
// (the tiles are no longer needed), then normalise and store the block's rows of ctx and lse.
template <int NQ, int SPLIT, bool DROP>
GX_DEVINL void fwd_merge_store(char* smem, f32x16 (&o)[DH / 32], float m, float lsum, int part, int qs, int lane,
                               int iw, int b, int h, int S, int nl, bf16* __restrict__ ctx,
                               float* __restrict__ lse, const KeepArgs& keep) {
  const int g = lane >> 5, l32 = lane & 31;
  const int Hl = nl * DH;
  if (SPLIT > 1) {
    // merge the parts' partial softmax states; the tiles are no longer needed, so parts 1.. park
    // (m, l, O) in LDS as [part - 1][row block][2 + DH / 2 values][64 lanes] and part 0 folds them
    // in, in order.  A part that saw no key has m = -inf, l = 0, O = 0 and folds in as nothing
    // (part 0 always saw key 0, so the merged maximum is finite).
    constexpr int REGION = (2 + DH / 2) * 64;
    if (part > 0) {
      float* park = reinterpret_cast<float*>(smem) + ((part - 1) * NQ + qs) * REGION + lane;
      park[0] = m;
      park[64] = lsum;
#pragma unroll
      for (int dt = 0; dt < DH / 32; dt++)
#pragma unroll
        for (int v = 0; v < 16; v++) park[(2 + 16 * dt + v) * 64] = o[dt][v];
    }
    __syncthreads();
    if (part > 0) return;
#pragma unroll
    for (int pp = 1; pp < SPLIT; pp++) {
      const float* park = reinterpret_cast<const float*>(smem) + ((pp - 1) * NQ + qs) * REGION + lane;
      const float m1 = park[0], l1 = park[64];
      const float mm = fmaxf(m, m1);
      const float a0 = __builtin_amdgcn_exp2f(m - mm), a1 = __builtin_amdgcn_exp2f(m1 - mm);
      lsum = lsum * a0 + l1 * a1;
      m = mm;
#pragma unroll
      for (int dt = 0; dt < DH / 32; dt++)
#pragma unroll
        for (int v = 0; v < 16; v++) o[dt][v] = o[dt][v] * a0 + park[(2 + 16 * dt + v) * 64] * a1;
    }
  }
  lsum += __shfl_xor(lsum, 32, 64);
  const int i = iw + l32;
  if (i < S) {
    const float inv = (DROP ? keep.scale : 1.0f) / lsum;
    bf16* orow = ctx + ((size_t)b * S + i) * Hl + h * DH;
#pragma unroll
    for (int dt = 0; dt < DH / 32; dt++)
#pragma unroll
      for (int q4 = 0; q4 < 4; q4++) {
        bf16x4 pk;
#pragma unroll
        for (int e = 0; e < 4; e++) pk[e] = (bf16)(o[dt][4 * q4 + e] * inv);
        *reinterpret_cast<bf16x4*>(orow + 32 * dt + 8 * q4 + 4 * g) = pk;
      }
    if (g == 0) lse[((size_t)b * nl + h) * S + i] = (m + __builtin_amdgcn_logf(lsum)) * LN2;
  }
}

template <int NQ, int SPLIT, int BKV, bool DROP>
__global__ void __launch_bounds__(64 * NQ * SPLIT, NQ * SPLIT == 4 ? 2 : 1)
    attn_fwd_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ ctx, float* __restrict__ lse, int S, int nl,
                    int npair, unsigned qkv_bytes, KeepArgs keep) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  constexpr int NW = NQ * SPLIT, BQ = 32 * NQ, ROWS = BKV * SPLIT, STAGE = 2 * ROWS * ROWB;   // K rows | V rows
  constexpr int NJT = BKV / 32;
  static_assert((NQ & (NQ - 1)) == 0 && (BKV == 32 || BKV == 64), "shape of the step");
  static_assert((SPLIT - 1) * NQ * (2 + DH / 2) * 256 <= 2 * STAGE, "merge area fits the tile buffers");
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int qs = wave % NQ, part = wave / NQ;
  const int g = lane >> 5, l32 = lane & 31;
  const int nq = (S + BQ - 1) / BQ;
  const int pair = blockIdx.x % npair;
  const int qt = nq - 1 - blockIdx.x / npair;         // longest rows first
  const int h = pair % nl, b = pair / nl;
  const int Hl = nl * DH, ld = 3 * Hl;
  const int i0 = qt * BQ, iw = i0 + qs * 32;          // this wave's first query row
  const unsigned eq = (unsigned)((size_t)b * S * ld + h * DH);
  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16*>(qkv), 0, qkv_bytes,
                                                                        0x00020000);
  bf16x8 qf[DH / 16];
  load_row_frags(qkv + eq, ld, iw + l32, S, g, qf);

  f32x16 o[DH / 32];
#pragma unroll
  for (int dt = 0; dt < DH / 32; dt++) o[dt] = zero16();
  float m = -INFINITY, lsum = 0.f;
  const float c2 = rsqrtf((float)DH) * LOG2E;
  unsigned coff[2][DH / 32];
  cols_lane_offsets(lane, coff);

  const int jend = min(S, i0 + BQ);                   // keys 0 .. jend-1 can be visible
  const int nt = (jend + ROWS - 1) / ROWS;
  tile_load<ROWS, NW>(rsrc, eq + Hl, ld, 0, S, smem, wave, lane);
  tile_load<ROWS, NW>(rsrc, eq + 2 * Hl, ld, 0, S, smem + ROWS * ROWB, wave, lane);
  WAIT_VM0();
  __syncthreads();
  for (int t = 0; t < nt; t++) {
    if (t + 1 < nt) {
      char* nxt = smem + ((t + 1) & 1) * STAGE;
      tile_load<ROWS, NW>(rsrc, eq + Hl, ld, (t + 1) * ROWS, S, nxt, wave, lane);
      tile_load<ROWS, NW>(rsrc, eq + 2 * Hl, ld, (t + 1) * ROWS, S, nxt + ROWS * ROWB, wave, lane);
    }
    const int j0 = t * ROWS + part * BKV;              // this wave's keys of the step
    // wave-uniform; j0 and iw are multiples of 32, so when it holds every row of the wave sees key j0
    if (j0 <= iw + 31) {
      const char* kt = smem + (t & 1) * STAGE + part * BKV * ROWB;
      const char* vt = kt + ROWS * ROWB;
      unsigned long long kw = ~0ull;                    // keep bits of this query's keys of the step
      if (DROP && iw + l32 < S)
        kw = keep_bits_of_step<NJT>(keep.bits + (((size_t)b * nl + h) * S + iw + l32) * keep.wpr, j0);
      f32x16 sacc[NJT];
#pragma unroll
      for (int jt = 0; jt < NJT; jt++) {
        sacc[jt] = zero16();
#pragma unroll
        for (int s = 0; s < DH / 16; s++) sacc[jt] = MFMA(frag_rows(kt, 32 * jt + l32, s, g), qf[s], sacc[jt]);
      }
      // transposed V fragments of the first 32 keys travel while the softmax runs
      const unsigned ct = lds_addr(vt);
      ColFrags cf[2];
      cols_issue<0>(ct, coff, cf[0]);
      cols_issue<1>(ct, coff, cf[1]);
      // online softmax for query column i = iw + l32 (base-2 exponentials, scale folded into the
      // exponent's multiply-add)
      const int i = iw + l32;
      if (j0 + BKV - 1 > iw) {                         // the tile touches the diagonal
#pragma unroll
        for (int jt = 0; jt < NJT; jt++)
#pragma unroll
          for (int v = 0; v < 16; v++)
            if (j0 + 32 * jt + 8 * (v >> 2) + 4 * g + (v & 3) > i) sacc[jt][v] = -INFINITY;
      }
      float mloc = sacc[0][0];
#pragma unroll
      for (int jt = 0; jt < NJT; jt++)
#pragma unroll
        for (int v = 0; v < 16; v++) mloc = fmaxf(mloc, sacc[jt][v]);
      mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64)) * c2;
      const float mnew = fmaxf(m, mloc);
      if (__builtin_amdgcn_ballot_w64(mnew > m)) {     // wave-uniform: some row's running max moved
        const float alpha = __builtin_amdgcn_exp2f(m - mnew);
        m = mnew;
        lsum *= alpha;
#pragma unroll
        for (int dt = 0; dt < DH / 32; dt++)
#pragma unroll
          for (int v = 0; v < 16; v++) o[dt][v] *= alpha;
      }
      float psum = 0.f;
#pragma unroll
      for (int jt = 0; jt < NJT; jt++)
#pragma unroll
        for (int v = 0; v < 16; v++) {
          const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[jt][v], c2, -m));
          sacc[jt][v] = p;
          psum += p;
        }
      lsum += psum;
      if (DROP) drop_unkept<NJT>(sacc, kw, g);         // the row sum above is the undropped one
      // O^T += V^T P^T, 16 keys per group
      bf16x8 pf[2 * NJT];
#pragma unroll
      for (int u = 0; u < 2 * NJT; u++) pf[u] = pack_half(sacc[u >> 1], u & 1);
      tr_product<true, 2 * NJT>(o, ct, coff, cf, pf);
    }
    WAIT_VM0();
    __syncthreads();
  }
  fwd_merge_store<NQ, SPLIT, DROP>(smem, o, m, lsum, part, qs, lane, iw, b, h, S, nl, ctx, lse, keep);
}

// The split-key shape of the forward pass with the scores one step ahead: while the softmax of step
// t runs on the vector units, the same wavefront's matrix instructions already compute the scores
// of step t + 1 (one matrix instruction, then a share of the softmax, kept in that order by
// scheduling barriers).  The two wavefronts of a SIMD pass the workgroup barrier together and so
// are in the same phase of a step at the same time; without the interleave inside a wavefront the
// matrix pipe idles through both softmaxes and the vector units through both score products.
// K and V have separate double buffers because K runs a step ahead of V: at the top of step t,
// K(t + 2) goes into the buffer of K(t) (its scores were taken during step t - 1) and V(t + 1)
// into the buffer of V(t - 1).
template <int NQ, int SPLIT, bool DROP>
__global__ void __launch_bounds__(64 * NQ * SPLIT, NQ * SPLIT == 4 ? 2 : 1)
    attn_fwd_ahead_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ ctx, float* __restrict__ lse, int S,
                          int nl, int npair, unsigned qkv_bytes, KeepArgs keep) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  constexpr int NW = NQ * SPLIT, BQ = 32 * NQ, BKV = 32, ROWS = BKV * SPLIT, TILE = ROWS * ROWB, NS = DH / 16;
  static_assert((NQ & (NQ - 1)) == 0 && SPLIT > 1, "shape of the step");
  static_assert((SPLIT - 1) * NQ * (2 + DH / 2) * 256 <= 4 * TILE, "merge area fits the tile buffers");
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int qs = wave % NQ, part = wave / NQ;
  const int g = lane >> 5, l32 = lane & 31;
  const int nq = (S + BQ - 1) / BQ;
  const int pair = blockIdx.x % npair;
  // First half of the launch: longest blocks first; second half: shortest first.  With two
  // workgroups per compute unit and a launch of twice the number of units, workgroups x and
  // x + gridDim.x / 2 tend to share a unit, and their causal work then adds up to the same total.
  const int rq = blockIdx.x / npair, hq = (nq + 1) / 2;
  const int qt = rq < hq ? nq - 1 - rq : rq - hq;
  const int h = pair % nl, b = pair / nl;
  const int Hl = nl * DH, ld = 3 * Hl;
  const int i0 = qt * BQ, iw = i0 + qs * 32;          // this wave's first query row
  const unsigned eq = (unsigned)((size_t)b * S * ld + h * DH);
  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16*>(qkv), 0, qkv_bytes,
                                                                        0x00020000);
  bf16x8 qf[NS];
  load_row_frags(qkv + eq, ld, iw + l32, S, g, qf);

  f32x16 o[DH / 32];
#pragma unroll
  for (int dt = 0; dt < DH / 32; dt++) o[dt] = zero16();
  float m = -INFINITY, lsum = 0.f;
  const float c2 = rsqrtf((float)DH) * LOG2E;
  constexpr float MAX_SLACK = 8.0f;
  unsigned coff[2][DH / 32];
  cols_lane_offsets(lane, coff);

  char* const kst = smem;                             // K(t) at kst + (t & 1) * TILE
  char* const vst = smem + 2 * TILE;                  // V(t) at vst + (t & 1) * TILE
  const int jend = min(S, i0 + BQ);                   // keys 0 .. jend-1 can be visible
  const int nt = (jend + ROWS - 1) / ROWS;
  TileStream<ROWS, NW> ksrc, vsrc;
  ksrc.init(eq + Hl, ld, wave, lane);
  vsrc.init(eq + 2 * Hl, ld, wave, lane);
  ksrc.load(rsrc, eq + Hl, ld, 0, S, kst, wave, lane);
  vsrc.load(rsrc, eq + 2 * Hl, ld, 0, S, vst, wave, lane);
  if (nt > 1) ksrc.load(rsrc, eq + Hl, ld, ROWS, S, kst + TILE, wave, lane);
  WAIT_VM0();
  __syncthreads();
  // scores of step 0; a wavefront's keys of a step are visible when the step's first key is at or
  // before the wavefront's last row (wave-uniform; both are multiples of 32 up to the 31)
  f32x16 s_even = zero16(), s_odd;
  if (part * BKV <= iw + 31) {
    const char* k0 = kst + part * BKV * ROWB;
#pragma unroll
    for (int s = 0; s < NS; s++) s_even = MFMA(frag_rows(k0, l32, s, g), qf[s], s_even);
  }
  // one step: `sacc` holds the scores of step t on entry, `snxt` those of step t + 1 on exit
  auto step = [&](int t, f32x16& sacc, f32x16& snxt) __attribute__((always_inline)) {
    if (t + 2 < nt) ksrc.load(rsrc, eq + Hl, ld, (t + 2) * ROWS, S, kst + (t & 1) * TILE, wave, lane);
    if (t + 1 < nt) vsrc.load(rsrc, eq + 2 * Hl, ld, (t + 1) * ROWS, S, vst + ((t + 1) & 1) * TILE, wave, lane);
    const int j0 = t * ROWS + part * BKV;              // this wave's keys of the step
    if (j0 <= iw + 31) {
      // Scores of the next step are always taken, also when that step does not exist or is not
      // visible to this wavefront: the buffer then holds an older tile (or nothing yet), the
      // products are never looked at, and the loop body stays free of a second code path.
      const char* kn = kst + ((t + 1) & 1) * TILE + part * BKV * ROWB;
      const char* vt = vst + (t & 1) * TILE + part * BKV * ROWB;
      unsigned long long kw = ~0ull;                    // keep bits of this query's keys of the step
      if (DROP && iw + l32 < S)
        kw = keep_bits_of_step<1>(keep.bits + (((size_t)b * nl + h) * S + iw + l32) * keep.wpr, j0);
      bf16x8 kf[NS];
#pragma unroll
      for (int s = 0; s < NS; s++) kf[s] = frag_rows(kn, l32, s, g);
      snxt = zero16();
      const int i = iw + l32;
      float psum = 0.f;
      // the softmax of step t for query column i (base-2 exponentials, scale folded into the
      // exponent's multiply-add), cut into pieces
      auto piece = [&](int k) __attribute__((always_inline)) {
        if (k == 0) {
          if (j0 + BKV - 1 > iw) {                     // the tile touches the diagonal
#pragma unroll
            for (int v = 0; v < 16; v++)
              if (j0 + 8 * (v >> 2) + 4 * g + (v & 3) > i) sacc[v] = -INFINITY;
          }
        } else if (k == 1) {
          float mloc = sacc[0];
#pragma unroll
          for (int v = 1; v < 16; v++) mloc = fmaxf(mloc, sacc[v]);
          mloc = max_across_halves(mloc) * c2;
          // The reference maximum m follows the true one lazily: it moves only when some row's new
          // maximum exceeds it by more than MAX_SLACK (wave-uniform), so exponentials stay below
          // 2^MAX_SLACK and the rescaling of O, four multiplies per score, becomes rare.  Any
          // reference gives the same softmax up to rounding; lse = m + log2(l) is exact for any m.
          if (__builtin_amdgcn_ballot_w64(mloc > m + MAX_SLACK)) {
            const float mnew = fmaxf(m, mloc);
            const float alpha = __builtin_amdgcn_exp2f(m - mnew);
            m = mnew;
            lsum *= alpha;
#pragma unroll
            for (int dt = 0; dt < DH / 32; dt++)
#pragma unroll
              for (int v = 0; v < 16; v++) o[dt][v] *= alpha;
          }
        } else if (k >= 2 && k < 6) {
#pragma unroll
          for (int v = 4 * (k - 2); v < 4 * (k - 2) + 4; v++) {
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[v], c2, -m));
            sacc[v] = p;
            psum += p;
          }
        }
      };
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int s = 0; s < NS; s++) {
        snxt = MFMA(kf[s], qf[s], snxt);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < 8; k++)
          if (k * NS / 8 == s) piece(k);
        __builtin_amdgcn_sched_barrier(0);
      }
      // transposed V fragments travel while the probabilities are rounded
      const unsigned ct = lds_addr(vt);
      ColFrags cf[2];
      cols_issue<0>(ct, coff, cf[0]);
      cols_issue<1>(ct, coff, cf[1]);
      lsum += psum;
      f32x16 pacc[1] = {sacc};
      if (DROP) drop_unkept<1>(pacc, kw, g);           // the row sum above is the undropped one
      // O^T += V^T P^T, 16 keys per group
      bf16x8 pf[2];
#pragma unroll
      for (int u = 0; u < 2; u++) pf[u] = pack_half(pacc[0], u);
      tr_product<true, 2>(o, ct, coff, cf, pf);
    }
    WAIT_VM0();
    __syncthreads();
  };
  for (int t = 0; t < nt; t += 2) {
    step(t, s_even, s_odd);
    if (t + 1 < nt) step(t + 1, s_odd, s_even);
  }
  fwd_merge_store<NQ, SPLIT, DROP>(smem, o, m, lsum, part, qs, lane, iw, b, h, S, nl, ctx, lse, keep);
}

// ------------------------------------------------------------------------------- backward: D
// D[b, h, s] = sum_d dO * O; DH / 8 lanes per (token, head), 8 elements each
__global__ void __launch_bounds__(256) attn_dsum_kernel(const bf16* __restrict__ ctx, const bf16* __restrict__ dctx,
                                                        float* __restrict__ dsum, int B, int S, int nl) {
  const long gid = (long)blockIdx.x * 256 + threadIdx.x;
  const long pair = gid / CPR;                // (token, head) index
  const int sub = (int)(gid % CPR);
  const long npair = (long)B * S * nl;
  float acc = 0.f;
  if (pair < npair) {
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(ctx + pair * DH + sub * 8);
    const bf16x8 d = *reinterpret_cast<const bf16x8*>(dctx + pair * DH + sub * 8);
#pragma unroll
    for (int e = 0; e < 8; e++) acc += (float)a[e] * (float)d[e];
  }
#pragma unroll
  for (int o = CPR / 2; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
  if (pair < npair && sub == 0) {
    const long tok = pair / nl;
    const int h = (int)(pair % nl);
    const long b = tok / S, s = tok % S;
    dsum[(b * nl + h) * S + s] = acc;
  }
}

// ------------------------------------------------------------------------------- backward: dK, dV
// A workgroup owns 128 key rows as 4 blocks of 32; each block belongs to a PAIR of wavefronts on
// the same SIMD that split the work by output: wavefront `pair` (role V) forms S = Q K^T, the
// probabilities P and dV += P^T dO; wavefront `pair + 4` (role K) forms dP = dO V^T, then
// dS = P (dP - D) and dK += dS^T Q.  P crosses from one to the other through LDS as bf16, in the
// accumulator's own lane layout (16 B per lane per half sub-tile, conflict-free).  Each wavefront
// thus keeps one operand (K or V) and one 32 x 128 accumulator in registers, which leaves room
// for two wavefronts per SIMD.
//
// The roles are skewed so that the exponentials of one run under the matrix work of the other and
// one barrier per query tile suffices.  In phase n
//   role V: S(n), P(n) -> LDS, dV += P(n)^T dO(n)
//   role K: dS(n-1) from P(n-1) and the dP(n-1) it kept in registers, dK += dS(n-1)^T Q(n-1), then dP(n)
// Tiles n+1 and n+2 are in flight meanwhile (a tile has two phases to arrive from HBM).
constexpr int KV_PAIRS = 4, KV_NW = 2 * KV_PAIRS, KV_BJ = 32 * KV_PAIRS, KV_BI = 64;
// LDS: Q tiles (+ their D rows) in a ring of 4 (tiles n-1 .. n+2), dO tiles (+ lse rows) in a ring
// of 3 (tiles n .. n+2), two P exchange buffers, and a 256 B sink (see stage_load).
constexpr int KV_NQ = 4, KV_NDO = 3;
constexpr int KV_TILE = KV_BI * ROWB + KV_BI * 4;            // 64 rows of Q or dO | 64 floats
constexpr int KV_PX = KV_PAIRS * 4 * 1024;                   // P exchange: [pair][sub-tile, half][lane] x 16 B
constexpr int KV_OFF_DO = KV_NQ * KV_TILE, KV_OFF_PX = KV_OFF_DO + KV_NDO * KV_TILE;
constexpr int KV_OFF_SINK = KV_OFF_PX + 2 * KV_PX, KV_SMEM = KV_OFF_SINK + 256;
// direct-to-LDS loads per wavefront per tile: its share of the Q rows, of the dO rows (tile_load's
// PER_WAVE each, which depends on the row length) and one lse / D / sink load
constexpr int KV_TILE_LOADS = KV_BI / (64 / CPR) / KV_NW;
static_assert(KV_TILE_LOADS >= 1 && KV_TILE_LOADS * (64 / CPR) * KV_NW == KV_BI, "tile_load<KV_BI, KV_NW> split");
constexpr int KV_LOADS = 2 * KV_TILE_LOADS + 1;

template <bool DROP>
__global__ void __launch_bounds__(64 * KV_NW) attn_bwd_dkv_kernel(const bf16* __restrict__ qkv,
                                                                  const bf16* __restrict__ dctx,
                                                                  const float* __restrict__ lse,
                                                                  const float* __restrict__ dsum,
                                                                  bf16* __restrict__ dqkv, int S, int nl,
                                                                  unsigned qkv_bytes, unsigned dctx_bytes,
                                                                  KeepArgs keep) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const bool role_v = wave < KV_PAIRS;
  const int pair = wave & (KV_PAIRS - 1);
  const int g = lane >> 5, l32 = lane & 31;
  const int h = blockIdx.y, b = blockIdx.z;
  const int Hl = nl * DH, ld = 3 * Hl;
  const int j0 = blockIdx.x * KV_BJ, jw = j0 + pair * 32;
  const unsigned eq = (unsigned)((size_t)b * S * ld + h * DH);
  const unsigned edo = (unsigned)((size_t)b * S * Hl + h * DH);
  const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16*>(qkv), 0, qkv_bytes,
                                                                      0x00020000);
  const __amdgpu_buffer_rsrc_t rdo = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16*>(dctx), 0, dctx_bytes,
                                                                       0x00020000);
  bf16x8 kvf[DH / 16];                      // role V: this block's K rows; role K: its V rows
  load_row_frags(qkv + eq + (role_v ? Hl : 2 * Hl), ld, jw + l32, S, g, kvf);
  f32x16 acc[DH / 32];                      // role V: dV; role K: dK
#pragma unroll
  for (int dt = 0; dt < DH / 32; dt++) acc[dt] = zero16();
  const float scale = rsqrtf((float)DH), c2 = scale * LOG2E;
  const float* lrow = lse + ((size_t)b * nl + h) * S;
  const float* drow = dsum + ((size_t)b * nl + h) * S;
  char* px = smem + KV_OFF_PX + pair * 4096 + lane * 16;
  unsigned coff[2][DH / 32];
  cols_lane_offsets(lane, coff);

  const int t0 = j0 / KV_BI, nt = (S + KV_BI - 1) / KV_BI;     // query tiles t0 .. nt-1 see these keys
  // lse and D rows of a query tile go to LDS by the same direct path, 4 B per lane (wavefront 0:
  // lse, wavefront 1: D; the others send an out-of-range load to a sink so that every wavefront
  // has the same number of loads in flight per tile).  Rows beyond the sequence read as 0
  // everywhere (Q, dO, lse, D): their probabilities are 1 but their contributions to dV and dK
  // are exactly 0, and whole tiles beyond the sequence may be requested harmlessly.
  const __amdgpu_buffer_rsrc_t raux = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<float*>(wave == 0 ? lrow : drow), 0, (unsigned)S * 4u, 0x00020000);
  auto stage_load = [&](int t, int qslot, int dslot) {
    char* qs = smem + qslot * KV_TILE;
    char* ds = smem + KV_OFF_DO + dslot * KV_TILE;
    tile_load<KV_BI, KV_NW>(rq, eq, ld, t * KV_BI, S, qs, wave, lane);
    tile_load<KV_BI, KV_NW>(rdo, edo, Hl, t * KV_BI, S, ds, wave, lane);
    const int i = t * KV_BI + lane;
    char* ad = (wave == 0) ? ds + KV_BI * ROWB : (wave == 1) ? qs + KV_BI * ROWB : smem + KV_OFF_SINK;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(raux, (lds_void_ptr)ad, 4, (wave < 2 && i < S) ? (unsigned)i * 4u : OOB,
                                             0, 0, 0);
  };
  // first product of a role over both 32-row query sub-tiles: [query i][key j]
  f32x16 sp[2];
  auto first_product = [&](const char* rows_of) {
    bf16x8 fr[2][DH / 16];
#pragma unroll
    for (int s = 0; s < DH / 16; s++) fr[0][s] = frag_rows(rows_of, l32, s, g);
#pragma unroll
    for (int sub = 0; sub < 2; sub++) {
      sp[sub] = zero16();
#pragma unroll
      for (int s = 0; s < DH / 16; s++) {
        if (sub == 0) fr[1][s] = frag_rows(rows_of, 32 + l32, s, g);
        sp[sub] = MFMA(fr[sub][s], kvf[s], sp[sub]);
      }
    }
  };
  stage_load(t0, 0, 0);
  stage_load(t0 + 1, 1, 1);
  __builtin_amdgcn_s_waitcnt(0x0F70 | KV_LOADS);                  // tile t0 has landed, t0 + 1 may be in flight
  __syncthreads();
  const int j = jw + l32;
  // dropout: this key's column of keep bits, one 64-bit word per query tile (both roles read it;
  // a word is fetched one phase before its use, ahead of that phase's tile requests, so that
  // waiting for it never waits for a tile)
  const unsigned* kcol = DROP ? keep.bits + (((size_t)b * nl + h) * S + min(j, S - 1)) * keep.wpr : nullptr;
  auto keep_word = [&](int t) -> unsigned long long {
    return (t >= t0 && t < nt) ? *reinterpret_cast<const unsigned long long*>(kcol + 2 * t) : 0ull;
  };
  // One loop per role (the branch is wavefront-uniform and both loops pass the same number of
  // barriers), so that neither role carries the other's addresses and fragments in registers.
  auto run = [&](auto role_tag) {
    constexpr bool ROLE_V = decltype(role_tag)::value;
    int qslot = 0, dslot = 0;                                     // ring positions of tile n
    unsigned long long kw = 0, kw_next = 0;                       // role V: tile n; role K: tile n - 1
    if (DROP && ROLE_V) kw_next = keep_word(t0);
#pragma unroll 1
    for (int n = t0; n <= nt; n++) {
      if (DROP) {
        kw = kw_next;
        kw_next = keep_word(ROLE_V ? n + 1 : n);
      }
      stage_load(n + 2, (qslot + 2) & (KV_NQ - 1), dslot == 0 ? 2 : dslot - 1);
      const char* qt = smem + qslot * KV_TILE;                    // Q rows of tile n, then their D
      const char* dot = smem + KV_OFF_DO + dslot * KV_TILE;       // dO rows of tile n, then their lse
      bf16x8 xf[4];                                               // P or dS, 16 query rows per entry
      ColFrags cf[2];
      if (ROLE_V) {
        if (n < nt && n * KV_BI + KV_BI - 1 >= jw) {              // pair-uniform: some query of tile n sees a key
          const float* aux = reinterpret_cast<const float*>(dot + KV_BI * ROWB);
          first_product(qt);                                      // S = Q K^T
          const unsigned ct = lds_addr(dot);
          cols_issue<0>(ct, coff, cf[0]);
          cols_issue<1>(ct, coff, cf[1]);
#pragma unroll
          for (int sub = 0; sub < 2; sub++) {
#pragma unroll
            for (int q4 = 0; q4 < 4; q4++) {
              const f32x4 l4 = *reinterpret_cast<const f32x4*>(aux + 32 * sub + 8 * q4 + 4 * g);
#pragma unroll
              for (int e = 0; e < 4; e++)
                sp[sub][4 * q4 + e] = __builtin_amdgcn_exp2f(__builtin_fmaf(sp[sub][4 * q4 + e], c2, -LOG2E * l4[e]));
            }
            const int it0 = n * KV_BI + 32 * sub;
            if (it0 < jw + 31) {                                  // the sub-tile touches the diagonal
#pragma unroll
              for (int v = 0; v < 16; v++)
                if (j > it0 + 8 * (v >> 2) + 4 * g + (v & 3)) sp[sub][v] = 0.f;
            }
#pragma unroll
            for (int u = 0; u < 2; u++) {
              xf[2 * sub + u] = pack_half(sp[sub], u);
              *reinterpret_cast<bf16x8*>(px + (n & 1) * KV_PX + (2 * sub + u) * 1024) = xf[2 * sub + u];
            }
          }
          if (DROP) {                                             // dV takes the dropped probabilities
            drop_unkept(sp, kw, g);
#pragma unroll
            for (int u = 0; u < 4; u++) xf[u] = pack_half(sp[u >> 1], u & 1);
          }
          tr_product4<false>(acc, ct, coff, cf, xf);              // dV[j][d] += P^T dO
        }
      } else {
        const int m = n - 1;                                      // tile whose dP this wavefront holds
        if (m >= t0 && m * KV_BI + KV_BI - 1 >= jw) {
          const char* qp = smem + ((qslot + KV_NQ - 1) & (KV_NQ - 1)) * KV_TILE;
          const float* dp = reinterpret_cast<const float*>(qp + KV_BI * ROWB);
          const unsigned ct = lds_addr(qp);
          cols_issue<0>(ct, coff, cf[0]);
          cols_issue<1>(ct, coff, cf[1]);
          if (DROP) {                                             // gradient w.r.t. the undropped probabilities
            drop_unkept(sp, kw, g);
#pragma unroll
            for (int sub = 0; sub < 2; sub++)
#pragma unroll
              for (int v = 0; v < 16; v++) sp[sub][v] *= keep.scale;
          }
#pragma unroll
          for (int sub = 0; sub < 2; sub++) {
            bf16x8 pb[2];
#pragma unroll
            for (int u = 0; u < 2; u++)
              pb[u] = *reinterpret_cast<const bf16x8*>(px + (m & 1) * KV_PX + (2 * sub + u) * 1024);
#pragma unroll
            for (int q4 = 0; q4 < 4; q4++) {
              const f32x4 d4 = *reinterpret_cast<const f32x4*>(dp + 32 * sub + 8 * q4 + 4 * g);
#pragma unroll
              for (int e = 0; e < 4; e++) {
                const int v = 4 * q4 + e;
                sp[sub][v] = (float)pb[v >> 3][v & 7] * (sp[sub][v] - d4[e]);
              }
            }
#pragma unroll
            for (int u = 0; u < 2; u++) xf[2 * sub + u] = pack_half(sp[sub], u);
          }
          tr_product4<false>(acc, ct, coff, cf, xf);              // dK[j][d] += dS^T Q
        }
        if (n < nt && n * KV_BI + KV_BI - 1 >= jw) first_product(dot);   // dP = dO V^T, used in the next phase
      }
      // tile n+1 has landed (n+2 may still be in flight) and this wavefront's LDS traffic is
      // complete; then the workgroup meets
      asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(KV_LOADS) : "memory");
      qslot = (qslot + 1) & (KV_NQ - 1);
      dslot = (dslot == KV_NDO - 1) ? 0 : dslot + 1;
    }
  };
  if (role_v) run(std::true_type{});
  else run(std::false_type{});
  WAIT_VM0();   // requests for tiles beyond the last one (zero fill) must not outlive the workgroup's LDS
  // accumulator register v of lane l is row 8 (v/4) + 4 g + v%4, column l%32 of its 32x32 tile
  const float oscale = role_v ? (DROP ? keep.scale : 1.f) : scale;
  bf16* obase = dqkv + (size_t)b * S * ld + h * DH + (role_v ? 2 * Hl : Hl);
#pragma unroll
  for (int dt = 0; dt < DH / 32; dt++)
#pragma unroll
    for (int v = 0; v < 16; v++) {
      const int jr = jw + 8 * (v >> 2) + 4 * g + (v & 3);
      if (jr < S) obase[(size_t)jr * ld + 32 * dt + l32] = (bf16)(acc[dt][v] * oscale);
    }
}

// ------------------------------------------------------------------------------- backward: dQ
// Shapes and workgroup order as in the forward kernel; the parts' dQ partial sums are added
// through LDS in the order of `part`.
template <int NQ, int SPLIT, int BKV, bool DROP>
__global__ void __launch_bounds__(64 * NQ * SPLIT, NQ * SPLIT == 4 ? 2 : 1)
    attn_bwd_dq_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ dctx, const float* __restrict__ lse,
                       const float* __restrict__ dsum, bf16* __restrict__ dqkv, int S, int nl, int npair,
                       unsigned qkv_bytes, KeepArgs keep) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  constexpr int NW = NQ * SPLIT, BQ = 32 * NQ, ROWS = BKV * SPLIT, STAGE = 2 * ROWS * ROWB;
  constexpr int NJT = BKV / 32;
  static_assert((SPLIT - 1) * NQ * (DH / 2) * 256 <= 2 * STAGE, "merge area fits the tile buffers");
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int qs = wave % NQ, part = wave / NQ;
  const int g = lane >> 5, l32 = lane & 31;
  const int nq = (S + BQ - 1) / BQ;
  const int pair = blockIdx.x % npair;
  // longest blocks first; with two workgroups per compute unit (4 wavefronts each), the second
  // half of the launch runs shortest first, as in the forward kernel
  const int rq = blockIdx.x / npair, hq = (nq + 1) / 2;
  const int qt = (NW == 4 && rq >= hq) ? rq - hq : nq - 1 - rq;
  const int h = pair % nl, b = pair / nl;
  const int Hl = nl * DH, ld = 3 * Hl;
  const int i0 = qt * BQ, iw = i0 + qs * 32;
  const unsigned eq = (unsigned)((size_t)b * S * ld + h * DH);
  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16*>(qkv), 0, qkv_bytes,
                                                                        0x00020000);
  bf16x8 qf[DH / 16], dof[DH / 16];
  load_row_frags(qkv + eq, ld, iw + l32, S, g, qf);
  load_row_frags(dctx + (size_t)b * S * Hl + h * DH, Hl, iw + l32, S, g, dof);
  const int i = iw + l32;
  const int ic = min(i, S - 1);
  const float scale = rsqrtf((float)DH), c2 = scale * LOG2E;
  const float lse2 = lse[((size_t)b * nl + h) * S + ic] * LOG2E;
  const float dd = dsum[((size_t)b * nl + h) * S + ic];
  unsigned coff[2][DH / 32];
  cols_lane_offsets(lane, coff);
  f32x16 dq[DH / 32];
#pragma unroll
  for (int dt = 0; dt < DH / 32; dt++) dq[dt] = zero16();

  const int jend = min(S, i0 + BQ);
  const int nt = (jend + ROWS - 1) / ROWS;
  tile_load<ROWS, NW>(rsrc, eq + Hl, ld, 0, S, smem, wave, lane);
  tile_load<ROWS, NW>(rsrc, eq + 2 * Hl, ld, 0, S, smem + ROWS * ROWB, wave, lane);
  WAIT_VM0();
  __syncthreads();
  for (int t = 0; t < nt; t++) {
    if (t + 1 < nt) {
      char* nxt = smem + ((t + 1) & 1) * STAGE;
      tile_load<ROWS, NW>(rsrc, eq + Hl, ld, (t + 1) * ROWS, S, nxt, wave, lane);
      tile_load<ROWS, NW>(rsrc, eq + 2 * Hl, ld, (t + 1) * ROWS, S, nxt + ROWS * ROWB, wave, lane);
    }
    const int j0 = t * ROWS + part * BKV;
    if (j0 <= iw + 31) {
      const char* kt = smem + (t & 1) * STAGE + part * BKV * ROWB;
      const char* vt = kt + ROWS * ROWB;
      unsigned long long kw = ~0ull;                    // keep bits of this query's keys of the step
      if (DROP && i < S)
        kw = keep_bits_of_step<NJT>(keep.bits + (((size_t)b * nl + h) * S + i) * keep.wpr, j0);
      f32x16 sacc[NJT], pacc[NJT];
#pragma unroll
      for (int jt = 0; jt < NJT; jt++) {
        sacc[jt] = zero16();
        pacc[jt] = zero16();
#pragma unroll
        for (int s = 0; s < DH / 16; s++) {
          sacc[jt] = MFMA(frag_rows(kt, 32 * jt + l32, s, g), qf[s], sacc[jt]);    // S^T[j][i]
          pacc[jt] = MFMA(frag_rows(vt, 32 * jt + l32, s, g), dof[s], pacc[jt]);   // dP^T[j][i]
        }
      }
      if (DROP) {                                      // gradient w.r.t. the undropped probabilities
        drop_unkept<NJT>(pacc, kw, g);
#pragma unroll
        for (int jt = 0; jt < NJT; jt++)
#pragma unroll
          for (int v = 0; v < 16; v++) pacc[jt][v] *= keep.scale;
      }
#pragma unroll
      for (int jt = 0; jt < NJT; jt++)
#pragma unroll
        for (int v = 0; v < 16; v++) {
          const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[jt][v], c2, -lse2));
          pacc[jt][v] = p * (pacc[jt][v] - dd);                                    // dS^T
        }
      // the scores are dead: their registers take the first transposed K fragments
      const unsigned ct = lds_addr(kt);
      ColFrags cf[2];
      cols_issue<0>(ct, coff, cf[0]);
      cols_issue<1>(ct, coff, cf[1]);
      if (j0 + BKV - 1 > iw) {                         // the tile touches the diagonal
#pragma unroll
        for (int jt = 0; jt < NJT; jt++)
#pragma unroll
          for (int v = 0; v < 16; v++)
            if (j0 + 32 * jt + 8 * (v >> 2) + 4 * g + (v & 3) > i) pacc[jt][v] = 0.f;
      }
      bf16x8 dsf[2 * NJT];
#pragma unroll
      for (int u = 0; u < 2 * NJT; u++) dsf[u] = pack_half(pacc[u >> 1], u & 1);
      tr_product<true, 2 * NJT>(dq, ct, coff, cf, dsf);       // dQ^T[d][i] += K^T dS^T
    }
    WAIT_VM0();
    __syncthreads();
  }
  if (SPLIT > 1) {
    constexpr int REGION = (DH / 2) * 64;
    if (part > 0) {
      float* park = reinterpret_cast<float*>(smem) + ((part - 1) * NQ + qs) * REGION + lane;
#pragma unroll
      for (int dt = 0; dt < DH / 32; dt++)
#pragma unroll
        for (int v = 0; v < 16; v++) park[(16 * dt + v) * 64] = dq[dt][v];
    }
    __syncthreads();
    if (part > 0) return;
#pragma unroll
    for (int pp = 1; pp < SPLIT; pp++) {
      const float* park = reinterpret_cast<const float*>(smem) + ((pp - 1) * NQ + qs) * REGION + lane;
#pragma unroll
      for (int dt = 0; dt < DH / 32; dt++)
#pragma unroll
        for (int v = 0; v < 16; v++) dq[dt][v] += park[(16 * dt + v) * 64];
    }
  }
  if (i < S) {
    bf16* row = dqkv + ((size_t)b * S + i) * ld + h * DH;
#pragma unroll
    for (int dt = 0; dt < DH / 32; dt++)
#pragma unroll
      for (int q4 = 0; q4 < 4; q4++) {
        bf16x4 pk;
#pragma unroll
        for (int e = 0; e < 4; e++) pk[e] = (bf16)(dq[dt][4 * q4 + e] * scale);
        *reinterpret_cast<bf16x4*>(row + 32 * dt + 8 * q4 + 4 * g) = pk;
      }
  }
}

template <typename K>
hipError_t set_smem(K kernel, int bytes) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             bytes);
}

bool attn_shape_ok(const AttnArgs& a) {
  if (a.dh != DH || a.B <= 0 || a.S <= 0 || a.nl <= 0) return false;
  const size_t bytes = (size_t)a.B * a.S * 3 * a.nl * DH * 2;
  return bytes < (1ul << 31);
}

// With few (sample, head) pairs the chip is filled by cutting the query blocks fine and spreading
// each block's keys over two wavefronts (see the forward kernel).
bool few_pairs(const AttnArgs& a) { return (long)a.B * a.nl * cdiv(a.S, 128) <= 384; }

// row-block kernels (forward, dQ) in their two shapes, <4, 1, 64> and <2, 2, 32>: both 4 wavefronts
// and two stages of 64 rows of K and of V
constexpr int SMEM_MANY = 2 * 2 * 64 * ROWB, SMEM_FEW = 2 * 2 * 64 * ROWB;

hipError_t fwd(const AttnArgs& a, hipStream_t s) {
  if (!attn_shape_ok(a)) return hipErrorInvalidValue;
  static bool configured = false;
  if (!configured) {
    hipError_t e = set_smem(attn_fwd_kernel<4, 1, 64, false>, SMEM_MANY);
    if (e == hipSuccess) e = set_smem(attn_fwd_ahead_kernel<2, 2, false>, SMEM_FEW);
    if (e == hipSuccess) e = set_smem(attn_fwd_kernel<4, 1, 64, true>, SMEM_MANY);
    if (e == hipSuccess) e = set_smem(attn_fwd_ahead_kernel<2, 2, true>, SMEM_FEW);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const unsigned qkv_bytes = (unsigned)((size_t)a.B * a.S * 3 * a.nl * DH * 2);
  const KeepArgs keep{a.rowbits, a.wpr, a.keep_scale};
  const bool drop = a.rowbits != nullptr;
  if (drop && a.wpr != 2 * cdiv(a.S, 64)) return hipErrorInvalidValue;
  const int npair = a.nl * a.B;
  auto go = [&](auto kernel, int bq, int threads, int smem) {
    hipLaunchKernelGGL(kernel, dim3(cdiv(a.S, bq) * npair), dim3(threads), smem, s, (const bf16*)a.qkv, (bf16*)a.ctx,
                       a.lse, a.S, a.nl, npair, qkv_bytes, keep);
  };
  if (few_pairs(a)) {
    if (drop) go(attn_fwd_ahead_kernel<2, 2, true>, 64, 256, SMEM_FEW);
    else go(attn_fwd_ahead_kernel<2, 2, false>, 64, 256, SMEM_FEW);
  } else {
    if (drop) go(attn_fwd_kernel<4, 1, 64, true>, 128, 256, SMEM_MANY);
    else go(attn_fwd_kernel<4, 1, 64, false>, 128, 256, SMEM_MANY);
  }
  return hipGetLastError();
}

// dK/dV and dQ are independent once D is known, and the dK/dV kernel is short of workgroups near
// the end of the causal triangle (heavy key blocks come first): with a second stream the dQ
// kernel runs beside it and fills the compute units it leaves idle.  `fork` / `join` are events
// owned by the caller of this function.
hipError_t bwd(const AttnArgs& a, hipStream_t s, hipStream_t s_dq, hipEvent_t fork, hipEvent_t join) {
  if (!attn_shape_ok(a)) return hipErrorInvalidValue;
  static bool configured = false;
  if (!configured) {
    hipError_t e = set_smem(attn_bwd_dkv_kernel<false>, KV_SMEM);
    if (e == hipSuccess) e = set_smem(attn_bwd_dkv_kernel<true>, KV_SMEM);
    if (e == hipSuccess) e = set_smem(attn_bwd_dq_kernel<4, 1, 64, false>, SMEM_MANY);
    if (e == hipSuccess) e = set_smem(attn_bwd_dq_kernel<2, 2, 32, false>, SMEM_FEW);
    if (e == hipSuccess) e = set_smem(attn_bwd_dq_kernel<4, 1, 64, true>, SMEM_MANY);
    if (e == hipSuccess) e = set_smem(attn_bwd_dq_kernel<2, 2, 32, true>, SMEM_FEW);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const bool drop = a.rowbits != nullptr;
  if (drop && (!a.colbits || a.wpr != 2 * cdiv(a.S, 64))) return hipErrorInvalidValue;
  const KeepArgs keep_rows{a.rowbits, a.wpr, a.keep_scale}, keep_cols{a.colbits, a.wpr, a.keep_scale};
  const unsigned qkv_bytes = (unsigned)((size_t)a.B * a.S * 3 * a.nl * DH * 2);
  const unsigned dctx_bytes = qkv_bytes / 3;
  const long npairs = (long)a.B * a.S * a.nl;
  hipLaunchKernelGGL(attn_dsum_kernel, dim3(cdiv(npairs * CPR, 256)), dim3(256), 0, s, (const bf16*)a.ctx,
                     (const bf16*)a.dctx, a.dsum, a.B, a.S, a.nl);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const bool two = (s_dq != s);
  if (two) {
    if ((e = hipEventRecord(fork, s)) != hipSuccess) return e;
    if ((e = hipStreamWaitEvent(s_dq, fork, 0)) != hipSuccess) return e;
  }
  auto go_dkv = [&](auto kernel) {
    hipLaunchKernelGGL(kernel, dim3(cdiv(a.S, KV_BJ), a.nl, a.B), dim3(64 * KV_NW), KV_SMEM, s, (const bf16*)a.qkv,
                       (const bf16*)a.dctx, a.lse, a.dsum, (bf16*)a.dqkv, a.S, a.nl, qkv_bytes, dctx_bytes,
                       keep_cols);
  };
  if (drop) go_dkv(attn_bwd_dkv_kernel<true>);
  else go_dkv(attn_bwd_dkv_kernel<false>);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  const int npair = a.nl * a.B;
  auto go_dq = [&](auto kernel, int bq, int threads, int smem) {
    hipLaunchKernelGGL(kernel, dim3(cdiv(a.S, bq) * npair), dim3(threads), smem, s_dq, (const bf16*)a.qkv,
                       (const bf16*)a.dctx, a.lse, a.dsum, (bf16*)a.dqkv, a.S, a.nl, npair, qkv_bytes, keep_rows);
  };
  if (few_pairs(a)) {
    if (drop) go_dq(attn_bwd_dq_kernel<2, 2, 32, true>, 64, 256, SMEM_FEW);
    else go_dq(attn_bwd_dq_kernel<2, 2, 32, false>, 64, 256, SMEM_FEW);
  } else {
    if (drop) go_dq(attn_bwd_dq_kernel<4, 1, 64, true>, 128, 256, SMEM_MANY);
    else go_dq(attn_bwd_dq_kernel<4, 1, 64, false>, 128, 256, SMEM_MANY);
  }
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (two) {
    if ((e = hipEventRecord(join, s_dq)) != hipSuccess) return e;
    if ((e = hipStreamWaitEvent(s, join, 0)) != hipSuccess) return e;
  }
  return hipSuccess;
}

