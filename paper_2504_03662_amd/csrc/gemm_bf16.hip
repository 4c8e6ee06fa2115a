// bf16 MFMA GEMM family for gfx950: the dense contractions of one rank's transformer-block share
// (column-parallel QKV / FC1, row-parallel out-proj / FC2, their input and weight gradients).
//
// One workgroup of 8 wavefronts computes a 256x256 tile of C with a K step of 64 through a double
// buffer, or a 128x128 tile with a K step of 32 through a ring of four stages (products with few
// tiles keep only one small workgroup per compute unit, which needs the deeper prefetch).  Operand
// tiles go from HBM straight into LDS (buffer_load ... lds, 16 B per lane, no register staging); fragments for v_mfma_f32_32x32x16_bf16 are read with ds_read_b128 when the
// reduction index is contiguous in memory ("K-major" tiles) and with the transposing
// ds_read_b64_tr_b16 when it is strided ("MN-major" tiles), so no operand is ever transposed in
// HBM.  LDS positions are XOR-swizzled on the global-address side because a direct-to-LDS load
// fixes each lane's LDS slot.
#include "gx_kernels.h"

namespace gx {
namespace {

constexpr int NTHREADS = 512;
constexpr int NWAVES = NTHREADS / 64;
constexpr unsigned OOB = 0x80000000u;           // beyond num_records: the load writes zeros

// K-major tile: [R rows][BK k], 2 BK bytes per row, 16 B chunk c of row r stored at c ^ swz_k(r):
// the 16 rows that one ds_read_b128 pass covers at a fixed chunk then fall in distinct banks.
template <int BK>
GX_DEVINL int swz_k(int r) { return BK == 64 ? ((r >> 1) & 7) : ((r >> 2) & 3); }
// MN-major tile: [BK k-rows][R cols], 2R B per k-row, 16 B chunk c of k-row kr stored at
// c ^ swz_mn(kr) (moves whole 64 B groups so that 4 consecutive k-rows fall in distinct banks).
GX_DEVINL int swz_mn(int kr) { return (kr & 3) << 2; }

GX_DEVINL __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}

// This wave's share of the direct-to-LDS loads of one operand tile (R = 256 or 128 rows/columns
// by BK reduction steps): R * BK / 4096 instructions of 64 lanes x 16 B each.
template <bool KMAJOR, int R, int BK>
struct TileLoader {
  static constexpr int PER = R * BK / (512 * NWAVES);
  unsigned base[PER];   // k-invariant part of the lane's element offset, or OOB
  int kc[PER];          // K-major: k offset of the chunk; MN-major: k-row of the chunk
  unsigned voff[PER];   // the same as a byte offset (or OOB): the vector offset of the cheap form
  __amdgpu_buffer_rsrc_t rsrc;
  int ld, K;

  GX_DEVINL void init(const bf16* ptr, unsigned bytes, int ld_, int K_, int origin, int extent, int wave,
                      int lane) {
    rsrc = make_rsrc(ptr, bytes);
    ld = ld_;
    K = K_;
#pragma unroll
    for (int i = 0; i < PER; i++) {
      const int q = wave * PER + i;
      if (KMAJOR) {
        constexpr int CPR = BK / 8;                // 16 B chunks per row
        constexpr int RPI = 64 / CPR;              // rows per instruction
        const int r = RPI * q + lane / CPR;
        const int c = (lane % CPR) ^ swz_k<BK>(r);
        kc[i] = c * 8;
        base[i] = (origin + r < extent) ? (unsigned)((origin + r) * ld + c * 8) : OOB;
        voff[i] = (base[i] != OOB) ? base[i] * 2u : OOB;
      } else {
        constexpr int CPR = R / 8;                 // 16 B chunks per k-row
        constexpr int KPI = 64 / CPR;              // k-rows per instruction
        const int kr = KPI * q + lane / CPR;
        const int c = (lane % CPR) ^ swz_mn(kr);
        kc[i] = kr;
        base[i] = (origin + c * 8 < extent) ? (unsigned)(kr * ld + origin + c * 8) : OOB;
        voff[i] = (base[i] != OOB) ? base[i] * 2u : OOB;
      }
    }
  }
  // instruction i of this wave's share of the tile that starts at reduction index k0, into LDS at
  // `dst`; lanes beyond the operand or beyond K get zeros
  GX_DEVINL void issue_one(char* dst, int k0, int wave, int i) const {
    unsigned off;
    if (KMAJOR) off = (base[i] != OOB && k0 + kc[i] < K) ? (base[i] + (unsigned)k0) * 2u : OOB;
    else        off = (base[i] != OOB && k0 + kc[i] < K) ? (base[i] + (unsigned)(k0 * ld)) * 2u : OOB;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_ptr)(dst + (wave * PER + i) * 1024), 16, off, 0, 0,
                                             0);
  }
  GX_DEVINL void issue(char* dst, int k0, int wave) const {
#pragma unroll
    for (int i = 0; i < PER; i++) issue_one(dst, k0, wave, i);
  }
  // The cheap form, for a tile that lies wholly inside K: the tile's reduction index goes into the
  // instruction's scalar offset (which takes no part in the range check, hence the condition) and
  // the lane's vector offset never changes, so a load costs no vector arithmetic at all.
  GX_DEVINL unsigned tile_offset(int k0) const { return KMAJOR ? (unsigned)k0 * 2u : (unsigned)(k0 * ld) * 2u; }
  GX_DEVINL void issue_inside(char* dst, unsigned tile_off, int wave, int i) const {
    unsigned off = voff[i];
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_ptr)(dst + (wave * PER + i) * 1024), 16, off,
                                             tile_off, 0, 0);
  }
};

// fragment of a 32-row block for k sub-step ks (16 k), K-major tile
template <int BK>
GX_DEVINL bf16x8 frag_k(const char* tile, int row, int ks, int g) {
  const int c = (2 * ks + g) ^ swz_k<BK>(row);
  return *reinterpret_cast<const bf16x8*>(tile + row * (2 * BK) + (c << 4));
}
// A fragment being fetched: either complete (K-major tile, one ds_read_b128 the compiler tracks)
// or two untracked transposing reads of an MN-major tile that lds_wait_all() must cover.
struct Frag {
  bf16x8 full;
  bf16x4 lo, hi;
};
// fragment of a 32-column block for k sub-step ks, MN-major tile of R columns: issue only
template <int R>
GX_DEVINL void frag_mn_issue(const char* tile, int col0, int ks, int lane, Frag& f) {
  const int g = lane >> 5, s = lane & 15;
  const int kr = 16 * ks + 8 * g + (s >> 2);
  const int ne = col0 + 16 * ((lane >> 4) & 1) + 4 * (s & 3);
  const int c = (ne >> 3) ^ swz_mn(kr);
  const unsigned addr = lds_addr(tile + kr * (2 * R) + (c << 4) + (ne & 7) * 2);
  f.lo = lds_read_tr_issue<0>(addr);
  f.hi = lds_read_tr_issue<4 * (2 * R)>(addr);
}
GX_DEVINL bf16x8 frag_mn_finish(Frag& f) {
  lds_pin(f.lo);
  lds_pin(f.hi);
  return __builtin_shufflevector(f.lo, f.hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// BM x BN output tile (256 x 256, or 128 x 128 for products with too few large tiles to fill the
// chip); 8 wavefronts as 2 x 4, each owning (BM/2) x (BN/4).  K step BK through STAGES LDS stages.
template <int LAY, int EPI, int BM, int BN, int BK>
__global__ void __launch_bounds__(NTHREADS) gemm_kernel(GemmArgs g) {
  constexpr int STAGES = (BK == 64) ? 2 : 4;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  constexpr bool A_K = (LAY != LAY_TN);
  constexpr bool B_K = (LAY == LAY_NT);
  constexpr int TM = BM / 64, TN = BN / 128;          // 32x32 accumulators per wave
  constexpr int WM = BM / 2, WN = BN / 4;             // wave tile
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
  constexpr int KS = BK / 16;
  static_assert(KS % 2 == 0, "fragment double buffer assumes an even number of sub-steps");
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave >> 2, wn = wave & 3;
  const int grp = lane >> 5, l32 = lane & 31;

  // tile index: spread consecutive tiles over the 8 XCDs' round-robin dispatch so that each XCD
  // (own L2) works on a compact block of tiles, then walk tiles in groups of 8 tile-rows.
  int pid = blockIdx.x;
  const int nwg = gridDim.x;
  if ((nwg & 7) == 0) pid = (pid & 7) * (nwg >> 3) + (pid >> 3);
  // tail launch: the walk runs over super-tiles of 2BM x 2BN (the tiles of the large-tile launch
  // that took the whole rounds), starting at g.tile_first; four consecutive workgroups share one
  const int sub = g.tail ? (pid & 3) : 0;
  const int SB = g.tail ? 2 : 1;
  if (g.tail) pid = g.tile_first + (pid >> 2);
  const int tm = (g.M + SB * BM - 1) / (SB * BM), tn = (g.N + SB * BN - 1) / (SB * BN);
  constexpr int GROUP = 8;
  const int in_group = GROUP * tn;
  const int first_m = (pid / in_group) * GROUP;
  const int gsize = min(tm - first_m, GROUP);
  const int pm = first_m + (pid % in_group) % gsize;
  const int pn = (pid % in_group) / gsize;
  const int m0 = (SB * pm + (sub >> 1)) * BM, n0 = (SB * pn + (sub & 1)) * BN;
  if (m0 >= g.M || n0 >= g.N) return;      // quarter of a ragged super-tile that lies outside C

  const bf16* A = static_cast<const bf16*>(g.A);
  const bf16* B = static_cast<const bf16*>(g.B);
  TileLoader<A_K, BM, BK> la;
  TileLoader<B_K, BN, BK> lb;
  la.init(A, (unsigned)((size_t)(A_K ? g.M : g.K) * g.lda * 2), g.lda, g.K, m0, g.M, wave, lane);
  lb.init(B, (unsigned)((size_t)(B_K ? g.N : g.K) * g.ldb * 2), g.ldb, g.K, n0, g.N, wave, lane);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;

  // Epilogue set-up; it sits ahead of the K loop because the first block of what the epilogue
  // reads is requested two tiles before the loop ends.
  const bf16* bias = static_cast<const bf16*>(g.bias);
  const bf16* resid = static_cast<const bf16*>(g.resid);
  const bf16* zin = static_cast<const bf16*>(g.z);
  bf16* aux = static_cast<bf16*>(g.aux);
  constexpr int EPAD = WN + 4;
  constexpr int LPR = WN / 4;                          // lanes per row when reading back
  constexpr int RPI = 64 / LPR;                        // rows per read instruction
  float* stage = reinterpret_cast<float*>(smem + wave * (32 * EPAD * 4));
  const int ecol = n0 + wn * WN + 4 * (lane % LPR);
  float bv[4] = {0.f, 0.f, 0.f, 0.f};
  if ((EPI == EPI_BIAS || EPI == EPI_RESID || EPI == EPI_GELU) && bias && ecol < g.N) {
    const bf16x4 b4 = *reinterpret_cast<const bf16x4*>(bias + ecol);
#pragma unroll
    for (int e = 0; e < 4; e++) bv[e] = (float)b4[e];
  }
  // EPI_DGELU may also leave partial column sums of what it stores (stage 1 of the bias gradient of
  // the product that made z): a wavefront's rows split into blocks of 64 (two 32-row passes), each
  // lane adds its rows of a block, lanes that share columns combine by shuffles, and the block's
  // sums go to colpart[(m0 + wave row) / 64 + block][column].  Every (block, column) has exactly
  // one writer.
  static_assert(WM % 64 == 0, "column-sum blocks of 64 rows");
  float cs[4] = {0.f, 0.f, 0.f, 0.f};
  // What an epilogue reads besides the accumulators (the residual, gelu'(z), the weight gradient
  // being added to) is fetched one 32-row block ahead, all of a block's loads together.  Written
  // as load - use - store per row, every load sits behind the previous row's store (the compiler
  // cannot know that the two tensors do not overlap) and the epilogue pays a memory latency per
  // row: 52 k cycles instead of 11 k for the residual form.
  constexpr bool SIDE16 = (EPI == EPI_RESID || EPI == EPI_DGELU), SIDE32 = (EPI == EPI_F32_ACC);
  constexpr int NJ = 32 / RPI;
  const bf16* side16 = (EPI == EPI_RESID) ? resid : zin;
  bf16x4 s16[2][SIDE16 ? NJ : 1];
  f32x4 s32[2][SIDE32 ? NJ : 1];
  auto fetch = [&](int mi, int buf) {
#pragma unroll
    for (int j = 0; j < NJ; j++) {
      const int row = m0 + wm * WM + mi * 32 + RPI * j + lane / LPR;
      if (row >= g.M || ecol >= g.N) continue;
      const size_t idx = (size_t)row * g.ldc + ecol;
      if (SIDE16) s16[buf][j] = *reinterpret_cast<const bf16x4*>(side16 + idx);
      if (SIDE32) s32[buf][j] = *reinterpret_cast<const f32x4*>(static_cast<const float*>(g.C) + idx);
    }
  };
  char* sa = smem;                       // A[STAGES]
  char* sb = smem + STAGES * A_BYTES;    // B[STAGES]
  const int nk = (g.K + BK - 1) / BK;
  // Fragments of sub-step ks+1 are requested before the products of sub-step ks are issued, also
  // across tiles: the wait for the next tile's DMA and the workgroup barrier sit before the LAST
  // sub-step's products, whose operands are already in registers, so the first fragments of the
  // next tile are in flight while those products run and no wavefront starts a tile by waiting
  // for LDS.  The stage the barrier has just retired receives the next tile to be fetched.
  Frag fa[2][TM], fb[2][TN];
  auto request = [&](const char* ta, const char* tb, int ks, int buf) {
#pragma unroll
    for (int mi = 0; mi < TM; mi++) {
      if (A_K) fa[buf][mi].full = frag_k<BK>(ta, wm * WM + mi * 32 + l32, ks, grp);
      else     frag_mn_issue<BM>(ta, wm * WM + mi * 32, ks, lane, fa[buf][mi]);
    }
#pragma unroll
    for (int ni = 0; ni < TN; ni++) {
      if (B_K) fb[buf][ni].full = frag_k<BK>(tb, wn * WN + ni * 32 + l32, ks, grp);
      else     frag_mn_issue<BN>(tb, wn * WN + ni * 32, ks, lane, fb[buf][ni]);
    }
  };
  // one sub-step: finish this sub-step's fragments, let `between` request the next ones (and do
  // the tile hand-over on the last sub-step), then issue the products
  auto substep = [&](int ks, auto between) {
    const int buf = ks & 1;
    bf16x8 af[TM], bfr[TN];
    if (!A_K || !B_K || ks == KS - 1) lds_wait_all();
#pragma unroll
    for (int mi = 0; mi < TM; mi++) af[mi] = A_K ? fa[buf][mi].full : frag_mn_finish(fa[buf][mi]);
#pragma unroll
    for (int ni = 0; ni < TN; ni++) bfr[ni] = B_K ? fb[buf][ni].full : frag_mn_finish(fb[buf][ni]);
    between(buf);
#pragma unroll
    for (int mi = 0; mi < TM; mi++)
#pragma unroll
      for (int ni = 0; ni < TN; ni++)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ni], af[mi], acc[mi][ni], 0, 0, 0);
    // ask the scheduler to place one LDS read after each matrix instruction instead of a block of
    // reads ahead of a block of products (measured: 0.5 - 1.5 % on the NN and GELU' products, none
    // slower; raising the wavefront's priority around the products or the compiler's canned
    // matrix-loop schedules were 1 - 2 % slower)
#pragma unroll
    for (int i = 0; i < TM * TN; i++) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
  };

  if constexpr (STAGES == 2) {
    // Double buffer, written as a fixed sequence of slots: every matrix instruction is followed by
    // at most one fragment read and one tile load, and a scheduling barrier on either side keeps
    // the compiler from regrouping them.  Left to itself it gathers a tile's loads and their address
    // arithmetic into one block behind the workgroup barrier, during which both wavefronts of a
    // SIMD leave the matrix pipe idle at the same moment (measured: 2 - 8 % per product).
    //   sub-steps 0 .. KS-2: products of sub-step ks, fragments of sub-step ks + 1 requested
    //   sub-step KS-1:       wait for tile kt + 1, workgroup barrier, then the products, the first
    //                        fragments of tile kt + 1, and tile kt + 2 into the stage just retired
    constexpr int SL = TM * TN, NF = TM + TN;
    constexpr int PER = TileLoader<A_K, BM, BK>::PER;
    static_assert(TileLoader<B_K, BN, BK>::PER == PER && 2 * PER <= SL && NF <= SL, "slots of a sub-step");
    auto request_one = [&](const char* ta, const char* tb, int ks, int buf, int j) {
      if (j < TM) {
        if (A_K) fa[buf][j].full = frag_k<BK>(ta, wm * WM + j * 32 + l32, ks, grp);
        else     frag_mn_issue<BM>(ta, wm * WM + j * 32, ks, lane, fa[buf][j]);
      } else {
        const int ni = j - TM;
        if (B_K) fb[buf][ni].full = frag_k<BK>(tb, wn * WN + ni * 32 + l32, ks, grp);
        else     frag_mn_issue<BN>(tb, wn * WN + ni * 32, ks, lane, fb[buf][ni]);
      }
    };
    auto tile = [&](int kt, const bool inside) __attribute__((always_inline)) {
      const int cur = kt & 1;
      const char* ta = sa + cur * A_BYTES;
      const char* tb = sb + cur * B_BYTES;
      const char* na = sa + (cur ^ 1) * A_BYTES;
      const char* nb = sb + (cur ^ 1) * B_BYTES;
      const unsigned offa = la.tile_offset((kt + 2) * BK), offb = lb.tile_offset((kt + 2) * BK);
#pragma unroll
      for (int ks = 0; ks < KS; ks++) {
        const int buf = ks & 1;
        bf16x8 af[TM], bfr[TN];
        if (!A_K || !B_K || ks == KS - 1) lds_wait_all();
#pragma unroll
        for (int mi = 0; mi < TM; mi++) af[mi] = A_K ? fa[buf][mi].full : frag_mn_finish(fa[buf][mi]);
#pragma unroll
        for (int ni = 0; ni < TN; ni++) bfr[ni] = B_K ? fb[buf][ni].full : frag_mn_finish(fb[buf][ni]);
        if (ks == KS - 1) {
          // every LDS read of tile kt by this wavefront has completed (lds_wait_all)
          __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's share of tile kt + 1 has landed
          __syncthreads();
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int sl = 0; sl < SL; sl++) {
          const int mi = sl / TN, ni = sl % TN;
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ni], af[mi], acc[mi][ni], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          if (sl < NF) {
            // past the last tile this reads a stage that holds zeros or a stale tile; never used
            if (ks + 1 < KS) request_one(ta, tb, ks + 1, buf ^ 1, sl);
            else request_one(na, nb, 0, buf ^ 1, sl);
          }
          if (ks == KS - 1 && sl >= SL - 2 * PER) {
            const int i = sl - (SL - 2 * PER);
            if (inside) {
              if (i < PER) la.issue_inside(sa + cur * A_BYTES, offa, wave, i);
              else lb.issue_inside(sb + cur * B_BYTES, offb, wave, i - PER);
            } else {
              // a ragged last tile, or nothing at all beyond K (every lane out of range: zeros, no
              // memory traffic)
              if (i < PER) la.issue_one(sa + cur * A_BYTES, (kt + 2) * BK, wave, i);
              else lb.issue_one(sb + cur * B_BYTES, (kt + 2) * BK, wave, i - PER);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    };
    la.issue(sa, 0, wave);
    lb.issue(sb, 0, wave);
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's LDS-DMA has landed
    __syncthreads();
    la.issue(sa + A_BYTES, BK, wave);
    lb.issue(sb + B_BYTES, BK, wave);
    request(sa, sb, 0, 0);
    const int ninside = max(0, g.K / BK - 2);   // tiles kt whose prefetch target kt + 2 lies wholly inside K
    for (int kt = 0; kt < ninside; kt++) tile(kt, true);
    if (SIDE16 || SIDE32) fetch(0, 0);
    for (int kt = ninside; kt < nk; kt++) tile(kt, false);
    // the zero-fill requests of the last two tiles must have landed before the staging below reuses LDS
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
  } else {
    // ring of STAGES tiles, STAGES - 1 in flight.  Loads in flight are counted per wavefront, LPT
    // per tile; tiles beyond K are requested like any other (every lane out of range: zeros, no
    // memory traffic), so that the count at each wait is the same in every step.
    constexpr int LPT = TileLoader<A_K, BM, BK>::PER + TileLoader<B_K, BN, BK>::PER;
    static_assert((STAGES - 1) * LPT < 16, "vmcnt immediate");
#pragma unroll
    for (int t = 0; t < STAGES; t++) {
      la.issue(sa + t * A_BYTES, t * BK, wave);
      lb.issue(sb + t * B_BYTES, t * BK, wave);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70 | ((STAGES - 1) * LPT));   // vmcnt: tile 0 has landed
    __syncthreads();
    request(sa, sb, 0, 0);
    for (int kt = 0; kt < nk; kt++) {
      const int cur = kt & (STAGES - 1), nxt = (kt + 1) & (STAGES - 1);
      const char* ta = sa + cur * A_BYTES;
      const char* tb = sb + cur * B_BYTES;
#pragma unroll
      for (int ks = 0; ks < KS; ks++) {
        substep(ks, [&](int buf) {
          if (ks + 1 < KS) {
            request(ta, tb, ks + 1, buf ^ 1);
          } else {
            // tile kt+1 has landed once at most STAGES-2 younger tiles are still in flight
            __builtin_amdgcn_s_waitcnt(0x0F70 | ((STAGES - 2) * LPT));
            __syncthreads();
            la.issue(sa + cur * A_BYTES, (kt + STAGES) * BK, wave);
            lb.issue(sb + cur * B_BYTES, (kt + STAGES) * BK, wave);
            if (kt + 1 < nk) request(sa + nxt * A_BYTES, sb + nxt * B_BYTES, 0, buf ^ 1);
          }
        });
      }
    }
    if (SIDE16 || SIDE32) fetch(0, 0);
    // the zero-fill requests of the tail must have landed before the staging below reuses LDS
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
  }
  // every wavefront passed the last barrier with all its LDS reads complete, so the tile buffers
  // are free to serve as staging space below

  // epilogue.  The MFMAs were issued with the B fragment as the row operand, so accumulator
  // register v of lane l holds C[m = tile row l%32][n = 8*(v/4) + 4*(l/32) + v%4]: runs of 4
  // consecutive columns.  Each wavefront passes its block through a private LDS region, 32 rows at
  // a time (row stride WN + 4 floats keeps the 16 B writes conflict-free), and reads it back so
  // that WN/4 lanes cover one row: every global access of the epilogue (C, residual,
  // pre-activation, second output) is a 16 B or 8 B vector in fully used lines.
#pragma unroll
  for (int mi = 0; mi < TM; mi++) {
    if ((SIDE16 || SIDE32) && mi + 1 < TM) fetch(mi + 1, (mi + 1) & 1);
#pragma unroll
    for (int ni = 0; ni < TN; ni++)
#pragma unroll
      for (int q4 = 0; q4 < 4; q4++) {
        const f32x16& a = acc[mi][ni];
        *reinterpret_cast<f32x4*>(stage + l32 * EPAD + ni * 32 + 8 * q4 + 4 * grp) =
            f32x4{a[4 * q4], a[4 * q4 + 1], a[4 * q4 + 2], a[4 * q4 + 3]};
      }
#pragma unroll
    for (int j = 0; j < 32 / RPI; j++) {
      const int r = RPI * j + lane / LPR;
      const f32x4 xv = *reinterpret_cast<const f32x4*>(stage + r * EPAD + 4 * (lane % LPR));
      const int row = m0 + wm * WM + mi * 32 + r;
      if (row >= g.M || ecol >= g.N) continue;            // N is a multiple of 4: whole run in or out
      const size_t idx = (size_t)row * g.ldc + ecol;
      float x[4] = {xv[0] + bv[0], xv[1] + bv[1], xv[2] + bv[2], xv[3] + bv[3]};
      if (EPI == EPI_F32) {
        *reinterpret_cast<f32x4*>(static_cast<float*>(g.C) + idx) = f32x4{x[0], x[1], x[2], x[3]};
      } else if (EPI == EPI_F32_ACC) {
        f32x4* cp = reinterpret_cast<f32x4*>(static_cast<float*>(g.C) + idx);
        const f32x4 old = s32[mi & 1][j];
        *cp = f32x4{old[0] + x[0], old[1] + x[1], old[2] + x[2], old[3] + x[3]};
      } else {
        bf16x4 o;
        if (EPI == EPI_RESID) {
          if (aux) {
#pragma unroll
            for (int e = 0; e < 4; e++) o[e] = (bf16)x[e];
            *reinterpret_cast<bf16x4*>(aux + idx) = o;
          }
          const bf16x4 rv = s16[mi & 1][j];
#pragma unroll
          for (int e = 0; e < 4; e++) x[e] += (float)rv[e];
        } else if (EPI == EPI_GELU) {
          bf16x4 ga;
#pragma unroll
          for (int e = 0; e < 4; e++) {
            float y, dy;
            if (g.gelu_tanh) gelu_tanh_both_fast(x[e], y, dy);
            else gelu_both_fast(x[e], y, dy);
            ga[e] = (bf16)y;
            x[e] = dy;                                     // C receives gelu'(z)
          }
          *reinterpret_cast<bf16x4*>(aux + idx) = ga;
        } else if (EPI == EPI_DGELU) {
          const bf16x4 zv = s16[mi & 1][j];
#pragma unroll
          for (int e = 0; e < 4; e++) x[e] *= (float)zv[e];
        }
#pragma unroll
        for (int e = 0; e < 4; e++) o[e] = (bf16)x[e];
        *reinterpret_cast<bf16x4*>(static_cast<bf16*>(g.C) + idx) = o;
        if (EPI == EPI_DGELU) {
#pragma unroll
          for (int e = 0; e < 4; e++) cs[e] += (float)o[e];
        }
      }
    }
    if (EPI == EPI_DGELU && (mi & 1) && g.colpart) {
#pragma unroll
      for (int e = 0; e < 4; e++) {
#pragma unroll
        for (int o = LPR; o < 64; o <<= 1) cs[e] += __shfl_xor(cs[e], o, 64);
      }
      const int row0 = m0 + wm * WM + (mi - 1) * 32;         // first row of this block of 64
      if (lane < LPR && row0 < g.M && ecol < g.N)
        *reinterpret_cast<f32x4*>(g.colpart + (size_t)(row0 >> 6) * g.N + ecol) = f32x4{cs[0], cs[1], cs[2], cs[3]};
#pragma unroll
      for (int e = 0; e < 4; e++) cs[e] = 0.f;
    }
  }
}

template <int LAY, int EPI, int BM, int BN, int BK>
hipError_t launch_tile(const GemmArgs& g, hipStream_t s, int grid) {
  constexpr int SMEM = ((BK == 64) ? 2 : 4) * (BM + BN) * BK * 2;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<LAY, EPI, BM, BN, BK>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
    if (e != hipSuccess) return e;
    configured = true;
  }
  hipLaunchKernelGGL((gemm_kernel<LAY, EPI, BM, BN, BK>), dim3(grid), dim3(NTHREADS), SMEM, s, g);
  return hipGetLastError();
}

// 256 compute units, one large workgroup each.  Measured on this chip:
//  - up to 144 large tiles the 128 x 128 tile is faster (128 large tiles: by 22 %; 160: large tile
//    4-23 % faster);
//  - beyond one round of 256 large tiles, a remainder of up to TAIL_MAX large tiles would hold the
//    chip for a whole extra round at a fraction of its width: the whole rounds go to the large
//    tile and the remainder region is cut into 128 x 128 tiles in a second launch.
constexpr long ROUND = 256, TAIL_MAX = 128;
template <int LAY, int EPI>
hipError_t launch(const GemmArgs& g, hipStream_t s) {
  const long big = (long)cdiv(g.M, 256) * cdiv(g.N, 256);
  if (big <= 144) return launch_tile<LAY, EPI, 128, 128, 32>(g, s, cdiv(g.M, 128) * cdiv(g.N, 128));
  const long rem = big % ROUND;
  if (big < ROUND || rem == 0 || rem > TAIL_MAX) return launch_tile<LAY, EPI, 256, 256, 64>(g, s, (int)big);
  hipError_t e = launch_tile<LAY, EPI, 256, 256, 64>(g, s, (int)(big - rem));
  if (e != hipSuccess) return e;
  GemmArgs t = g;
  t.tail = 1;
  t.tile_first = (int)(big - rem);
  return launch_tile<LAY, EPI, 128, 128, 32>(t, s, (int)(4 * rem));
}

template <int LAY>
hipError_t dispatch_epi(Epilogue epi, const GemmArgs& g, hipStream_t s) {
  switch (epi) {
    case EPI_STORE: return launch<LAY, EPI_STORE>(g, s);
    case EPI_BIAS: return launch<LAY, EPI_BIAS>(g, s);
    case EPI_RESID: return launch<LAY, EPI_RESID>(g, s);
    case EPI_GELU: return launch<LAY, EPI_GELU>(g, s);
    case EPI_DGELU: return launch<LAY, EPI_DGELU>(g, s);
    case EPI_F32: return launch<LAY, EPI_F32>(g, s);
    case EPI_F32_ACC: return launch<LAY, EPI_F32_ACC>(g, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t gemm_bf16(Layout lay, Epilogue epi, const GemmArgs& args, hipStream_t s) {
  GemmArgs g = args;
  g.tail = g.tile_first = 0;                 // the launcher's own fields
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipErrorInvalidValue;
  // 16-byte chunks along each operand's contiguous index; 31-bit byte offsets in buffer loads
  const long a_rows = (lay == LAY_TN) ? g.K : g.M, b_rows = (lay == LAY_NT) ? g.N : g.K;
  if ((g.lda & 7) || (g.ldb & 7)) return hipErrorInvalidValue;
  if (lay != LAY_TN && (g.K & 7)) return hipErrorInvalidValue;
  if (lay == LAY_TN && (g.M & 7)) return hipErrorInvalidValue;
  if (lay != LAY_NT && (g.N & 7)) return hipErrorInvalidValue;
  // the epilogue moves runs of 4 columns as one vector
  if ((g.N & 3) || (g.ldc & 3) || (reinterpret_cast<uintptr_t>(g.C) & 15)) return hipErrorInvalidValue;
  if (a_rows * g.lda * 2 >= (1L << 31) || b_rows * g.ldb * 2 >= (1L << 31)) return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(g.A) | reinterpret_cast<uintptr_t>(g.B)) & 15) return hipErrorInvalidValue;
  switch (lay) {
    case LAY_NN: return dispatch_epi<LAY_NN>(epi, g, s);
    case LAY_NT: return dispatch_epi<LAY_NT>(epi, g, s);
    case LAY_TN: return dispatch_epi<LAY_TN>(epi, g, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace gx
