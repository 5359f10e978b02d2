// Base GEMM on the bf16 matrix cores with the LoRA expand fused in:
//
//   out[tok(m), :] = Aop[tok(m), :] * Bop  +  u(m) * L_t          (m in the segment of adapter t)
//
// m runs over tokens grouped by adapter (tok = perm), Bop is the shared frozen
// base weight (paper Sec. 1 principle (1)), u = s_t * (x A_t) is the fp32 result
// of the shrink, and L_t is the adapter's output-side factor (B_t in forward,
// A_t in backward).
//
// gemm_bf16_kernel (large batches): the expand enters as extra contraction
// steps [u_hi | u_lo] * [L_t ; L_t] (u split into two bf16 terms); rows of a
// tile that belong to another adapter are fed zeros for these steps, so a tile
// may straddle any number of segments.  Tile: 256 x 256 per workgroup of 4 waves
// (2 x 2), each wave 128 x 128 as 8 x 8 MFMA 16x16x32 accumulators (the same
// loop with 32x32x16 MFMAs measured 3 to 6 % slower on the large configurations).  The
// contraction runs in k-tiles of 64 that go from global memory straight into LDS
// (16 bytes per lane, no register staging; every row segment is one whole
// 128-byte line) through two 64 KB slots.  The parts of a k-tile are requested
// while the previous one is multiplied, at least three MFMA phases before they
// are needed; the single barrier per k-tile sits before the last phase, so the
// first fragment reads of the next tile overlap MFMAs.  16-byte units are
// XOR-swizzled so that DMA writes and fragment reads are bank-conflict free.
//
// gemm_skinny_kernel + splitk_finish_kernel (small batches, decode): 128 x 128
// tiles with the contraction split over workgroups, fp32 partial sums, and the
// shrink computed by the same kernel as 32 extended columns per column tile;
// the finish kernel adds the splits, applies the expand in fp32 and scatters
// the rows.  transpose_bf16_kernel: per-call transposed copy of a weight that
// is stored output-contiguous, for large batches.
#include "gemm_args.h"

#include <atomic>
#include <cstring>

namespace marlaas {

static constexpr int BM = 256, BN = 256, BK = 64;
static constexpr int WAVES_M = 2, WAVES_N = 2;             // wave grid inside the tile
static constexpr int NWAVES = WAVES_M * WAVES_N;
static constexpr int GEMM_THREADS = 64 * NWAVES;
static constexpr int MT = BM / WAVES_M / 16, NT = BN / WAVES_N / 16;   // 16x16 MFMA tiles per wave (8 x 8)
static constexpr int DPW = 32 / NWAVES;                    // DMA instructions per wave, operand and k-tile
static constexpr int LROWS = GEMM_THREADS / 8;             // rows per pass of the register-staged loaders
static constexpr int LPASS = BM / LROWS;
static constexpr int LKROWS = GEMM_THREADS / 32;           // k-rows per pass (k-n tiles)
static constexpr int LKPASS = BK / LKROWS;
static constexpr int STAGE_BYTES = BM * BK * 2;            // 32 KB: one operand tile
static constexpr int SLOT_BYTES = 2 * STAGE_BYTES;         // 64 KB: A part then B part
static constexpr int SLOT_B_OFF = STAGE_BYTES;
static constexpr int RING_SLOTS = 2;
static constexpr int LT_LDS = 16 * (4 * 4 + 8);             // the tile's extra contraction tiles: first row, end row, first k, rank; factor
static constexpr int GEMM_LDS = RING_SLOTS * SLOT_BYTES + BM * 4 + LT_LDS;  // ring + token ids + LoRA tile list

// LDS byte offset of 16-byte unit `unit` (of 32) of k-row `k` in a [64][256] bf16 tile.
__device__ __forceinline__ int kn_swz(int k) { return ((k & 3) << 2) | (((k >> 3) & 1) << 1); }
__device__ __forceinline__ int swz_kn(int k, int unit) {
  return k * 512 + ((unit ^ kn_swz(k)) << 4);
}

__device__ __forceinline__ uint4 pack8(const bf16_t* o) {
  uint4 pk;
  pk.x = o[0] | ((uint32_t)o[1] << 16); pk.y = o[2] | ((uint32_t)o[3] << 16);
  pk.z = o[4] | ((uint32_t)o[5] << 16); pk.w = o[6] | ((uint32_t)o[7] << 16);
  return pk;
}

// One 32-wide contraction step of the wave's block from a 64-wide LDS tile pair (as, bs).
template <int FORM>
__device__ __forceinline__ void mma_kstep(const char* as, const char* bs, int ks, int a_off_row,
                                          int a_swz, int fg, int b_off_row, int b_swz,
                                          const int (&btr)[NT], f32x4 (&acc)[MT][NT]) {
  bf16x8 af[MT], bfr[NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
    af[mt] = *(const bf16x8*)(as + a_off_row + mt * (16 * 128) + (((ks * 4 + fg) ^ a_swz) << 4));
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    if (FORM == FORM_NT) {
      bfr[nt] = *(const bf16x8*)(bs + b_off_row + nt * (16 * 128) + (((ks * 4 + fg) ^ b_swz) << 4));
    } else {
      // btr[nt]: byte offset of this lane's (k = kb, column) element for ks = 0; a k-step moves
      // 32 rows down (the swizzle depends on k & 3 and k & 8 only)
      const char* p = bs + btr[nt] + ks * (32 * 512);
      bfr[nt] = lds_read_frag_tr(p, p + 4 * 512);
    }
  }
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
      acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[nt], af[mt], acc[mt][nt], 0, 0, 0);
}

// The MFMAs of this kernel take the weight fragment as their first operand, so a block of the
// accumulators is the transpose of the output block: in a 16 x 16 block lane l holds output
// row (token) l % 16 and the four consecutive output columns 4 (l / 16) .. + 3.  Four consecutive
// columns of one row are contiguous in memory, so the results leave in 8- or 16-byte pieces.
// FORM: storage of the weight operand; LFORM: storage of the adapters' expand factors (they
// differ when the weight was transposed into scratch for this call).
template <int FORM, bool OUT_F32, int LFORM = FORM>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_bf16_kernel(GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  int32_t* tok_s = (int32_t*)(smem + RING_SLOTS * SLOT_BYTES);
  uint64_t* ltL_s = (uint64_t*)(tok_s + BM);     // per extra contraction tile: factor of its adapter,
  int32_t* ltlo_s = (int32_t*)(ltL_s + 16);      // first and end row of its segment inside the tile,
  int32_t* lthi_s = ltlo_s + 16;
  int32_t* ltkc_s = lthi_s + 16;                 // first contraction index, rank
  int32_t* ltr_s = ltkc_s + 16;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: LDS DMA targets stay scalar
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  // ---- block -> tile: each XCD (blocks b = x mod 8) walks a compact run of
  // tiles; inside a run, groups of 8 row tiles share their column tiles.
  int tm, tn, ks_idx;
  {
    const int G = a.tiles_m * a.tiles_n * a.ksplit;
    const int b = blockIdx.x;
    const int xcd = b & 7, idx = b >> 3;
    const int q = G >> 3, rem = G & 7;
    const int start = xcd * q + (xcd < rem ? xcd : rem);
    const int bbs = start + idx;
    const int bb = bbs / a.ksplit;          // the splits of one tile stay on one XCD (one L2)
    ks_idx = bbs - bb * a.ksplit;
    const int GM = 8;
    const int per_group = GM * a.tiles_n;
    const int gid = bb / per_group;
    const int first_m = gid * GM;
    const int gsz = (a.tiles_m - first_m) < GM ? (a.tiles_m - first_m) : GM;
    const int in_g = bb - gid * per_group;
    tm = first_m + in_g % gsz;
    tn = in_g / gsz;
  }
  const int64_t m0 = (int64_t)tm * BM;
  const int64_t n0 = (int64_t)tn * BN;

  for (int i = tid; i < BM; i += GEMM_THREADS) {
    int64_t m = m0 + i;
    int32_t tok = -1;
    if (m < a.T) tok = a.perm ? a.perm[m] : (int32_t)m;
    tok_s[i] = tok;
  }
  // LoRA expand by DMA: this row tile's list of extra contraction tiles (they run after the main loop)
  int lt_cnt = -1;
  if (a.lora_dma && a.ksplit == 1 && a.n_adapters > 0) {
    const int32_t* lt = a.lora_tiles + (int64_t)tm * LT_STRIDE;
    lt_cnt = lt[0];
    if (tid < lt_cnt) {
      const int t = lt[1 + 4 * tid];
      const AdapterEntry e = a.table[t];
      ltL_s[tid] = (uint64_t)(uintptr_t)(a.which ? e.B : e.A);
      ltlo_s[tid] = lt[2 + 4 * tid]; lthi_s[tid] = lt[3 + 4 * tid]; ltkc_s[tid] = lt[4 + 4 * tid]; ltr_s[tid] = e.rank;
    }
  }
  __syncthreads();

  const int64_t kbeg = (int64_t)ks_idx * a.kchunk;
  const int64_t kend = (kbeg + a.kchunk) < a.Kc ? (kbeg + a.kchunk) : a.Kc;

  // ---- DMA geometry.  One wave instruction moves 64 x 16 B = 1 KB into consecutive LDS
  // bytes.  Row-k tiles ([256][64] bf16, 128 B per row): 8 rows per instruction, lane l writes
  // unit (l & 7) of row (l >> 3) and so fetches the global unit (l & 7) ^ swizzle(row); every
  // row segment is one whole 128-byte cache line.  k-n tiles ([64][256], 512 B per row): 2
  // k-rows per instruction.  Each wave issues DPW = 8 instructions per operand per k-tile.
  // The weight operand's addresses are one wave-uniform base, advanced per k-tile with scalar
  // arithmetic, plus a constant 32-bit byte offset per lane and instruction (a tile of the weight
  // spans less than 4 GB: the launcher rejects leading dimensions above 2^22 elements); gathered
  // rows of the first operand need full 64-bit addresses.
  const bf16_t* a_src[DPW];
  const char* b_base;      // wave-uniform
  uint32_t b_off[DPW];     // bytes
  int64_t b_step;          // bytes to advance b_base per k-tile
#pragma unroll
  for (int j = 0; j < DPW; ++j) {
    const int row = (wave * DPW + j) * 8 + (lane >> 3);
    const int unit = (lane & 7) ^ ((row >> 1) & 7);
    const int32_t tok = tok_s[row];
    a_src[j] = a.Aop + (int64_t)(tok < 0 ? tok_s[0] : tok) * a.lda + kbeg + unit * 8;
  }
  if (FORM == FORM_NT) {
#pragma unroll
    for (int j = 0; j < DPW; ++j) {
      const int row = (wave * DPW + j) * 8 + (lane >> 3);
      const int unit = (lane & 7) ^ ((row >> 1) & 7);
      int64_t n = n0 + row;
      if (n >= a.Nout) n = a.Nout - 1;           // clamped columns are never stored
      b_off[j] = (uint32_t)(((n - n0) * a.ldb + unit * 8) * 2);
    }
    b_base = (const char*)(a.Bop + n0 * a.ldb + kbeg);
    b_step = BK * 2;
  } else {
#pragma unroll
    for (int j = 0; j < DPW; ++j) {
      const int k = (wave * DPW + j) * 2 + (lane >> 5);
      const int unit = (lane & 31) ^ kn_swz(k);
      int64_t n = n0 + unit * 8;
      if (n >= a.Nout) n = a.Nout - 8;
      b_off[j] = (uint32_t)((k * a.ldb + (n - n0)) * 2);
    }
    b_base = (const char*)(a.Bop + kbeg * a.ldb + n0);
    b_step = (int64_t)BK * a.ldb * 2;
  }
  const int dma_off = wave * DPW * 1024;   // this wave's first KB inside an operand part of a slot

  // ---- fragment geometry (all tiles are 64 wide): 16 rows x 32 contraction values per MFMA
  // operand, lane l supplies row l % 16, values 8 (l / 16) .. + 7
  const int frow = lane & 15;          // row inside a 16-row MFMA tile
  const int fg = lane >> 4;            // which 8-wide quarter of the 32-wide k step
  const int a_row = wm * (MT * 16) + frow;
  const int b_row = wn * (NT * 16) + frow;
  const int a_off_row = a_row * 128;
  const int a_swz = (a_row >> 1) & 7;  // rows 16 apart share the swizzle
  const int b_off_row = b_row * 128;
  const int b_swz = (b_row >> 1) & 7;
  int btr[NT];
  {
    // transposing reads of a [k][n] tile: the 16 lanes of group fg fetch the 4 x 16 block of rows
    // 8 fg .. + 3 (lane i: row i / 4, columns 4 (i % 4) .. + 3) and each receives its own column
    const int kb = fg * 8 + (frow >> 2);
    for (int nt = 0; nt < NT; ++nt) {
      const int ncol = wn * (NT * 16) + nt * 16 + 4 * (frow & 3);
      btr[nt] = swz_kn(kb, ncol >> 3) + (ncol & 7) * 2;
    }
  }

  f32x4 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;

  const int64_t ntile = (kend - kbeg) / BK;

  static_assert(MT == 8 && NT == 8 && DPW == 8, "the interleaved schedule below is written for 8 x 8 MFMA tiles per wave");

// raw barrier: LDS traffic of this wave is complete, DMA traffic is tracked by hand with vmcnt
#define RING_BARRIER() asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory")

// one DMA instruction: part j (0..7) of operand `isb_` (0 = A, 1 = B) of the k-tile going to `slot_`
#define RING_DMA1(slot_, isb_, j_)                                                                        \
  do {                                                                                                    \
    char* _sb = smem + (slot_) * SLOT_BYTES + dma_off + (j_) * 1024;                                      \
    if (isb_) {                                                                                           \
      /* scalar base + 32-bit lane offset: the builtin only emits the 64-bit-address form, which */       \
      /* costs a 64-bit vector add per request (m0 = LDS byte address of lane 0's 16 bytes)       */       \
      const uint32_t _lds = (uint32_t)(uintptr_t)(lptr_t)(_sb + SLOT_B_OFF);                               \
      asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"                        \
                   :: "v"(b_off[j_]), "s"(b_base), "s"(_lds) : "memory", "m0");                            \
      if ((j_) == DPW - 1) b_base += b_step;                                                              \
    } else {                                                                                              \
      __builtin_amdgcn_global_load_lds((gptr_t)a_src[j_], (lptr_t)(_sb), 16, 0, 0);       \
      a_src[j_] += BK;                                                                    \
    }                                                                                                     \
  } while (0)

#define RING_DMA(slot_, isb_)                                                                             \
  do {                                                                                                    \
    _Pragma("unroll") for (int _j = 0; _j < DPW; ++_j) RING_DMA1(slot_, isb_, _j);                        \
  } while (0)

// x fragment (row block mt_) / weight fragment (column block nt_) of k-step ks_ (0, 1) of the
// k-tile in `slot_`
#define RING_READ_X(slot_, ks_, mt_, dst_)                                                                \
  do {                                                                                                    \
    const char* _as = smem + (slot_) * SLOT_BYTES;                                                        \
    dst_ = *(const bf16x8*)(_as + a_off_row + (mt_) * (16 * 128) + ((((ks_) * 4 + fg) ^ a_swz) << 4));    \
  } while (0)
#define RING_READ_W(slot_, ks_, nt_, dst_)                                                                \
  do {                                                                                                    \
    const char* _bs = smem + (slot_) * SLOT_BYTES + SLOT_B_OFF;                                           \
    if (FORM == FORM_NT) {                                                                                \
      dst_ = *(const bf16x8*)(_bs + b_off_row + (nt_) * (16 * 128) + ((((ks_) * 4 + fg) ^ b_swz) << 4));  \
    } else {                                                                                              \
      const char* _p = _bs + btr[nt_] + (ks_) * (32 * 512);                                               \
      dst_ = lds_read_frag_tr(_p, _p + 4 * 512);                                                          \
    }                                                                                                     \
  } while (0)

// One phase: the 32 MFMAs of row blocks 4 h_ .. 4 h_ + 3 (x fragments ux_) against all eight
// column blocks (weight fragments uw_).  In their shadow, after every other MFMA (after every
// MFMA when there are twelve, so that they are back before the next phase starts): up to 4 x fragment
// reads (row blocks 4 lxh_ .., k-step lxks_ of slot lxslot_, into lx_) and nw_ weight fragment
// reads (column blocks lwn0_ .., k-step lwks_ of slot lwslot_, into lw_), and the 8 DMA
// instructions of one operand part at every fourth MFMA.  sched_barrier pins the order (one wave
// per SIMD: nothing else hides the issue latency of LDS and DMA instructions).
#define RING_PHASE(h_, ux_, uw_, nx_, lxslot_, lxks_, lxh_, lx_, nw_, lwslot_, lwks_, lwn0_, lw_,          \
                   do_dma_, dma_slot_, dma_isb_)                                                          \
  do {                                                                                                    \
    _Pragma("unroll") for (int _i = 0; _i < 32; ++_i) {                                                   \
      acc[4 * (h_) + (_i >> 3)][_i & 7] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(                        \
          uw_[_i & 7], ux_[_i >> 3], acc[4 * (h_) + (_i >> 3)][_i & 7], 0, 0, 0);                         \
      __builtin_amdgcn_sched_barrier(0);   /* the MFMA first: a read hoisted above it would be waited for at once */ \
      if ((nx_) + (nw_) > 8 || (_i & 1) == 0) {     /* 12 reads: one per MFMA, else every other */          \
        const int _r = (nx_) + (nw_) > 8 ? _i : _i >> 1;                                                  \
        if (_r < (nx_)) RING_READ_X(lxslot_, lxks_, 4 * (lxh_) + _r, lx_[_r]);                            \
        else if (_r - (nx_) < (nw_)) RING_READ_W(lwslot_, lwks_, (lwn0_) + _r - (nx_), lw_[(lwn0_) + _r - (nx_)]); \
      }                                                                                                   \
      if ((do_dma_) && (_i & 3) == 1) RING_DMA1(dma_slot_, dma_isb_, _i >> 2);                            \
      __builtin_amdgcn_sched_barrier(0);                                                                  \
    }                                                                                                     \
  } while (0)

// One k-tile kt (slot kt & 1): two 32-wide k-steps, each in two phases (row blocks 0-3, 4-7).
// x fragments alternate between two sets of four, weight fragments between two sets of eight.
// Phase 0 also requests the B part of tile kt + 1 (its A part was requested one tile earlier).
// Before phase 3 every wave waits for its own DMA (all of tile kt + 1) and meets the others: tile
// kt + 1 is then complete, and no wave still reads tile kt from LDS (its last fragments are in
// registers), so phase 3 reads the first fragments of tile kt + 1 and requests the A part of tile
// kt + 2 into the slot of tile kt.
#define RING_TILE(kt_, dma_b_, dma_a_, has_next_)                                                         \
  do {                                                                                                    \
    const int _slot = (int)((kt_) & 1), _nslot = _slot ^ 1;                                               \
    RING_PHASE(0, xa0, wb0, 4, _slot, 0, 1, xa1, 4, _slot, 1, 0, wb1, dma_b_, _nslot, 1);                 \
    RING_PHASE(1, xa1, wb0, 4, _slot, 1, 0, xa0, 4, _slot, 1, 4, wb1, 0, 0, 0);                           \
    RING_PHASE(0, xa0, wb1, 4, _slot, 1, 1, xa1, 0, 0, 0, 0, wb0, 0, 0, 0);                               \
    if (has_next_) {                                                                                      \
      __builtin_amdgcn_s_waitcnt(VMCNT(0));                                                               \
      RING_BARRIER();                                                                                     \
    }                                                                                                     \
    RING_PHASE(1, xa1, wb1, (has_next_) ? 4 : 0, _nslot, 0, 0, xa0, (has_next_) ? 8 : 0, _nslot, 0, 0, wb0, \
               dma_a_, _slot, 0);                                                                         \
  } while (0)

  // loader geometry of the register-staged tiles (k tail and LoRA steps)
  const int lc = tid & 7;        // 16-byte unit along k (row-k tiles)
  const int lr = tid >> 3;       // 0..LROWS-1
  const int ncu = tid & 31;      // 16-byte unit along n (k-n tiles)
  const int nkr = tid >> 5;      // 0..LKROWS-1
  const uint4 zero4 = make_uint4(0, 0, 0, 0);


  // ---- request the first k-tile, then (while it is in flight) do the LoRA expand
  if (ntile > 0) { RING_DMA(0, 0); RING_DMA(0, 1); }

  // LoRA expand as extra contraction steps, one adapter segment at a time, staged through slot 1.
  // All global loads of a chunk are issued before any of them is used.
  if (a.ksplit == 1 && a.n_adapters > 0 && a.U != nullptr && lt_cnt < 0) {
    char* La = smem + SLOT_BYTES;
    char* Lb = La + STAGE_BYTES;
    const int64_t T_lora = a.seg_off[a.n_adapters];
    const int64_t m_end = (m0 + BM) < T_lora ? (m0 + BM) : T_lora;
    if (m0 < m_end) {
      int t = segment_of(a.seg_off, a.n_adapters, (int)m0);
      while (t < a.n_adapters && (int64_t)a.seg_off[t] < m_end) {
        const int64_t lo = a.seg_off[t] > m0 ? (int64_t)a.seg_off[t] : m0;
        const int64_t hi = (int64_t)a.seg_off[t + 1] < m_end ? (int64_t)a.seg_off[t + 1] : m_end;
        if (hi > lo) {
          const AdapterEntry e = a.table[t];
          const bf16_t* L = (const bf16_t*)(a.which ? e.B : e.A);
          const int r = e.rank;
          const int r_pad = (r + 15) & ~15;
          const int kext = 2 * r_pad;
          for (int kc = 0; kc < kext; kc += BK) {
            const int kk0 = kc + lc * 8;
            const bool second = kk0 >= r_pad;
            const int q0 = kk0 - (second ? r_pad : 0);
            float4 uf[LPASS][2];
            uint4 lw[LPASS];
            // A side: u of the rows of this segment, zeros elsewhere
#pragma unroll
            for (int i = 0; i < LPASS; ++i) {
              const int64_t m = m0 + lr + LROWS * i;
              uf[i][0] = uf[i][1] = make_float4(0.f, 0.f, 0.f, 0.f);
              if (kk0 < kext && m >= lo && m < hi) {
                const float4* up = (const float4*)(a.U + m * a.r_stride + q0);
                uf[i][0] = up[0]; uf[i][1] = up[1];
              }
            }
            // B side: L_t stacked twice along the contraction
            if (LFORM == FORM_NT) {
#pragma unroll
              for (int i = 0; i < LPASS; ++i) {
                const int64_t n = n0 + lr + LROWS * i;
                lw[i] = zero4;
                if (kk0 < kext && n < a.Nout && q0 < r) {
                  const bf16_t* lp = L + n * r + q0;
                  if ((r & 7) == 0) {
                    lw[i] = *(const uint4*)lp;
                  } else {
                    bf16_t o[8];
                    for (int j = 0; j < 8; ++j) o[j] = (q0 + j < r) ? lp[j] : (bf16_t)0;
                    lw[i] = pack8(o);
                  }
                }
              }
            } else {
#pragma unroll
              for (int i = 0; i < LKPASS; ++i) {
                const int kk = kc + nkr + LKROWS * i;
                const int q = kk - (kk >= r_pad ? r_pad : 0);
                lw[i] = zero4;
                if (kk < kext && q < r && (n0 + ncu * 8) < a.Nout)
                  lw[i] = *(const uint4*)(L + (int64_t)q * a.Nout + n0 + ncu * 8);
              }
            }
            // two-term bf16 split of u: [u_hi | u_lo]
#pragma unroll
            for (int i = 0; i < LPASS; ++i) {
              const float f[8] = {uf[i][0].x, uf[i][0].y, uf[i][0].z, uf[i][0].w,
                                  uf[i][1].x, uf[i][1].y, uf[i][1].z, uf[i][1].w};
              bf16_t o[8];
              for (int j = 0; j < 8; ++j) {
                const bf16_t h = float_to_bf16_bits(f[j]);
                o[j] = second ? float_to_bf16_bits(f[j] - bf16_bits_to_float(h)) : h;
              }
              *(uint4*)(La + swz_rowk(lr + LROWS * i, lc)) = pack8(o);
            }
            if (LFORM == FORM_NT) {
#pragma unroll
              for (int i = 0; i < LPASS; ++i) *(uint4*)(Lb + swz_rowk(lr + LROWS * i, lc)) = lw[i];
            } else {
#pragma unroll
              for (int i = 0; i < LKPASS; ++i) *(uint4*)(Lb + swz_kn(nkr + LKROWS * i, ncu)) = lw[i];
            }
            __syncthreads();
            const int left = kext - kc;
            const int ksteps = left >= BK ? 2 : 1;       // kext is a multiple of 32
            for (int ks = 0; ks < ksteps; ++ks)
              mma_kstep<LFORM>(La, Lb, ks, a_off_row, a_swz, fg, b_off_row, b_swz, btr, acc);
            __syncthreads();
          }
        }
        ++t;
      }
    }
  }

  // One extra contraction tile of the LoRA expand (entry i_ of the row tile's list) into ring slot
  // slot_: 8 + 8 DMA instructions per wave, every lane's source picked on its own.
#define LORA_DMA(i_, slot_)                                                                               \
    do {                                                                                                  \
      const int _lo = ltlo_s[i_], _hi = lthi_s[i_], _kc = ltkc_s[i_], _r = ltr_s[i_];                      \
      const int _rp = (_r + 15) & ~15, _kext = 2 * _rp;                                                   \
      const bf16_t* _L = (const bf16_t*)(uintptr_t)ltL_s[i_];                                             \
      _Pragma("unroll") for (int _j = 0; _j < DPW; ++_j) {                                                \
        char* _sb = smem + (slot_) * SLOT_BYTES + dma_off + _j * 1024;                                    \
        const int _row = (wave * DPW + _j) * 8 + (lane >> 3);                                             \
        const int _kk = _kc + (((lane & 7) ^ ((_row >> 1) & 7)) << 3);                                    \
        const int64_t _m = m0 + _row;                                                                     \
        const bf16_t* _src = a.zero_line;                                                                 \
        if (_m >= _lo && _m < _hi && _kk < _kext) _src = a.U2 + _m * (2 * a.r_stride) + _kk;              \
        __builtin_amdgcn_global_load_lds((gptr_t)_src, (lptr_t)_sb, 16, 0, 0);                            \
      }                                                                                                   \
      _Pragma("unroll") for (int _j = 0; _j < DPW; ++_j) {                                                \
        char* _sb = smem + (slot_) * SLOT_BYTES + SLOT_B_OFF + dma_off + _j * 1024;                       \
        const bf16_t* _src = a.zero_line;                                                                 \
        if (LFORM == FORM_NT) {          /* L_t[n * r + q]: row-k tile, 8 rows of 128 bytes per instruction */ \
          const int _row = (wave * DPW + _j) * 8 + (lane >> 3);                                           \
          const int _kk = _kc + (((lane & 7) ^ ((_row >> 1) & 7)) << 3);                                  \
          const int _q = _kk >= _rp ? _kk - _rp : _kk;                                                    \
          const int64_t _n = n0 + _row;                                                                   \
          if (_kk < _kext && _q < _r && _n < a.Nout) _src = _L + _n * _r + _q;                            \
        } else {                         /* L_t[q * Nout + n]: k-n tile, 2 k-rows of 512 bytes per instruction */ \
          const int _k = (wave * DPW + _j) * 2 + (lane >> 5);                                             \
          const int _kk = _kc + _k;                                                                       \
          const int _q = _kk >= _rp ? _kk - _rp : _kk;                                                    \
          const int64_t _n = n0 + (((lane & 31) ^ kn_swz(_k)) << 3);                                      \
          if (_kk < _kext && _q < _r && _n < a.Nout) _src = _L + (int64_t)_q * a.Nout + _n;               \
        }                                                                                                 \
        __builtin_amdgcn_global_load_lds((gptr_t)_src, (lptr_t)_sb, 16, 0, 0);                            \
      }                                                                                                   \
    } while (0)
  int lslot0 = 0;                  // ring slot of the first extra contraction tile
  bool lora_requested = false;

  // ---- main loop over full k-tiles
  if (ntile > 0) {
    bf16x8 xa0[4], xa1[4], wb0[NT], wb1[NT];
    if (ntile > 1) {
      RING_DMA(1, 0);
      __builtin_amdgcn_s_waitcnt(VMCNT(DPW));     // tile 0 landed, the A part of tile 1 in flight
    } else {
      __builtin_amdgcn_s_waitcnt(VMCNT(0));
    }
    RING_BARRIER();
#pragma unroll
    for (int i = 0; i < 4; ++i) RING_READ_X(0, 0, i, xa0[i]);
#pragma unroll
    for (int i = 0; i < NT; ++i) RING_READ_W(0, 0, i, wb0[i]);
    int64_t kt = 0;
    for (; kt + 2 < ntile; ++kt) RING_TILE(kt, 1, 1, 1);
    if (kt + 1 < ntile) { RING_TILE(kt, 1, 0, 1); ++kt; }
    if (lt_cnt > 0) {
      // the slot the last k-tile does not use is free: the first extra tile travels while the last
      // k-tile is multiplied
      lslot0 = (int)((kt + 1) & 1);
      LORA_DMA(0, lslot0);
      lora_requested = true;
    }
    RING_TILE(kt, 0, 0, 0);
  }
  __syncthreads();   // all reads of the last k-tile are done; slot 0 is reused below

  // ---- LoRA expand by DMA: per adapter segment of the tile's rows, 64-wide contraction tiles of
  // [u_hi | u_lo] x [L_t ; L_t], fetched like the main loop's tiles: the x side from the bf16 split
  // of u the shrink wrote (rows outside the segment fetch zeros), the weight side from the
  // adapter's factor (the two halves of the contraction read the same ranks).  Tile i + 1 is in
  // flight while tile i is multiplied.
  if (lt_cnt > 0) {
    if (!lora_requested) LORA_DMA(0, lslot0);
    for (int i = 0; i < lt_cnt; ++i) {
      __builtin_amdgcn_s_waitcnt(VMCNT(0));
      __syncthreads();               // tile i has landed everywhere, nobody still reads tile i - 1
      if (i + 1 < lt_cnt) LORA_DMA(i + 1, (lslot0 + i + 1) & 1);
      const char* Ls = smem + ((lslot0 + i) & 1) * SLOT_BYTES;
      const int rp = (ltr_s[i] + 15) & ~15;
      const int ksteps = (2 * rp - ltkc_s[i]) >= BK ? 2 : 1;     // 2 r_pad is a multiple of 32
      for (int ks = 0; ks < ksteps; ++ks)
        mma_kstep<LFORM>(Ls, Ls + SLOT_B_OFF, ks, a_off_row, a_swz, fg, b_off_row, b_swz, btr, acc);
    }
    __syncthreads();                 // the slots are reused below
  }
#undef LORA_DMA
  char* As = smem;                 // one 64-wide A tile
  char* Bs = smem + STAGE_BYTES;   // one 64-wide B tile

  // ---- k tail (Kc not a multiple of 64): one masked tile through registers
  if (kbeg + ntile * BK < kend) {
    const int64_t k0 = kbeg + ntile * BK;
    const bool ka = (k0 + lc * 8) < kend;
    for (int i = 0; i < LPASS; ++i) {
      const int row = lr + LROWS * i;
      const int32_t tok = tok_s[row];
      uint4 v = zero4;
      if (ka && tok >= 0) v = *(const uint4*)(a.Aop + (int64_t)tok * a.lda + k0 + lc * 8);
      *(uint4*)(As + swz_rowk(row, lc)) = v;
    }
    if (FORM == FORM_NT) {
      for (int i = 0; i < LPASS; ++i) {
        const int row = lr + LROWS * i;
        uint4 v = zero4;
        if (ka && (n0 + row) < a.Nout) v = *(const uint4*)(a.Bop + (n0 + row) * a.ldb + k0 + lc * 8);
        *(uint4*)(Bs + swz_rowk(row, lc)) = v;
      }
    } else {
      for (int i = 0; i < LKPASS; ++i) {
        const int k = nkr + LKROWS * i;
        uint4 v = zero4;
        if ((k0 + k) < kend && (n0 + ncu * 8) < a.Nout)
          v = *(const uint4*)(a.Bop + (k0 + k) * a.ldb + n0 + ncu * 8);
        *(uint4*)(Bs + swz_kn(k, ncu)) = v;
      }
    }
    __syncthreads();
    const int ksteps = (int)((kend - k0 + 31) / 32);
    for (int ks = 0; ks < ksteps; ++ks)
      mma_kstep<FORM>(As, Bs, ks, a_off_row, a_swz, fg, b_off_row, b_swz, btr, acc);
    __syncthreads();
  }

  if (a.ksplit > 1) {
    // partial sums as plain fp32 rows: [ks][pm][ldp]
    const int64_t ldp = a.ldp;
    float* part = a.partials + ((int64_t)ks_idx * a.pm + m0 + wm * (MT * 16) + (lane & 15)) * ldp + n0 +
                  wn * (NT * 16) + 4 * (lane >> 4);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        *(float4*)(part + (int64_t)(mt * 16) * ldp + nt * 16) =
            make_float4(acc[mt][nt][0], acc[mt][nt][1], acc[mt][nt][2], acc[mt][nt][3]);
    return;
  }

  // ---- epilogue: a lane holds pieces of four consecutive columns of a row; storing those
  // directly would write every cache line in 8-byte pieces, so each wave regroups 32 rows at a
  // time through a private LDS strip and every lane stores 16 contiguous bytes: a row segment of
  // the wave (128 columns) leaves as whole cache lines.  Rows are scattered back to token order.
  // LDS traffic of one wave is ordered, so no workgroup barrier is needed.
  {
    constexpr int ESZ = OUT_F32 ? 4 : 2;
    constexpr int EPITCH = 128 * ESZ + 16;
    constexpr int ECHUNKS = 128 * ESZ / 16;             // 16-byte chunks per row segment
    constexpr int EITERS = 32 * ECHUNKS / 64;
    char* ep = smem + wave * (32 * (128 * 4 + 16));
    char* ew = ep + (lane & 15) * EPITCH + 4 * (lane >> 4) * ESZ;
#pragma unroll
    for (int mp = 0; mp < MT / 2; ++mp) {            // 32 rows (two row blocks) per pass
#pragma unroll
      for (int mh = 0; mh < 2; ++mh)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          const f32x4 c = acc[2 * mp + mh][nt];
          char* dst = ew + mh * (16 * EPITCH) + (nt * 16) * ESZ;
          if (OUT_F32) {
            *(float4*)dst = make_float4(c[0], c[1], c[2], c[3]);
          } else {
            uint2 o;
            o.x = float_to_bf16_bits(c[0]) | ((uint32_t)float_to_bf16_bits(c[1]) << 16);
            o.y = float_to_bf16_bits(c[2]) | ((uint32_t)float_to_bf16_bits(c[3]) << 16);
            *(uint2*)dst = o;
          }
        }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int it = 0; it < EITERS; ++it) {
        const int c = it * 64 + lane;
        const int row_l = c / ECHUNKS, ch = c % ECHUNKS;
        const uint4 val = *(const uint4*)(ep + row_l * EPITCH + ch * 16);
        const int32_t tok = tok_s[wm * (MT * 16) + mp * 32 + row_l];
        const int64_t col = n0 + wn * (NT * 16) + ch * (16 / ESZ);
        if (tok >= 0 && col < a.Nout) {
          if (OUT_F32) *(uint4*)((float*)a.out + (int64_t)tok * a.ldo + col) = val;
          else *(uint4*)((bf16_t*)a.out + (int64_t)tok * a.ldo + col) = val;
        }
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
  }
}


// ---------------------------------------------------------------------------------------------
// Small batches (decode): the weight is streamed once from HBM and is the dominant traffic.  With
// few rows the 256 x 256 tile needs many contraction splits to fill the chip, and the fp32
// partial sums then cost more traffic than the weight.  Here the tile is 128 x 128 (a quarter of
// the splits for the same number of workgroups) and the DMA ring is four k-tiles deep, three of
// them in flight (48 KB of weight per compute unit), which is what covers the HBM latency.  Each
// wave owns 64 x 64.  The result always goes to fp32 partial rows; splitk_finish_kernel adds the
// splits, the LoRA expand and the rounding.
static constexpr int SK_A_BYTES = SK_BM * BK * 2;         // 16 KB
static constexpr int SK_B_BYTES = SK_BN * BK * 2;         // 16 KB
static constexpr int SK_X_BYTES = SK_BX * BK * 2;         // 4 KB: extended (shrink) columns
static constexpr int SK_SLOT = SK_A_BYTES + SK_B_BYTES + SK_X_BYTES;   // 36 KB
static constexpr int SK_SLOTS = 4;
static constexpr int SK_LDS = SK_SLOTS * SK_SLOT + SK_BM * 4;
#define SK_NI (8 + (EXT ? 1 : 0))   // DMA instructions per wave per k-tile

template <int FORM, bool EXT>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  int32_t* tok_s = (int32_t*)(smem + SK_SLOTS * SK_SLOT);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  int tm, tn, ks_idx;
  {
    // consecutive workgroups of one XCD: the row tiles of one column tile (they share the weight
    // tile through that XCD's L2), then its contraction splits, then the next column tile
    const int G = a.tiles_m * a.tiles_n * a.ksplit;
    const int b = blockIdx.x;
    const int xcd = b & 7, idx = b >> 3;
    const int q = G >> 3, rem = G & 7;
    const int bbs = xcd * q + (xcd < rem ? xcd : rem) + idx;
    tm = bbs % a.tiles_m;
    const int rest = bbs / a.tiles_m;
    ks_idx = rest % a.ksplit;
    tn = rest / a.ksplit;
  }
  const int64_t m0 = (int64_t)tm * SK_BM;
  const int64_t pn0 = (int64_t)tn * SK_BN;       // column of this tile in the partial sums
  // the projection this column tile belongs to (wave-uniform)
  const bf16_t* Bop = a.Bop;
  int64_t ldb = a.ldb, Nout = a.Nout, n0 = pn0;
  if (a.n_proj > 1) {
    int p = 0;
    for (int q = 1; q < a.n_proj; ++q) if (tn >= a.proj[q].tile0) p = q;
    const ProjEntry pe = a.proj[p];
    Bop = (const bf16_t*)pe.W; ldb = pe.ldw; Nout = pe.Nout;
    n0 = (int64_t)(tn - pe.tile0) * SK_BN;
  }
  const int64_t kbeg = (int64_t)ks_idx * a.kchunk;
  const int64_t kend = (kbeg + a.kchunk) < a.Kc ? (kbeg + a.kchunk) : a.Kc;
  const int64_t ntile = (kend - kbeg) / BK;
  // (two dependent table loads: requested first, needed last)
  // extended columns: one DMA instruction per wave per k-tile
  const bf16_t* x_src = nullptr;
  int64_t x_step = 0;
  if (EXT) {
    if (FORM == FORM_NT) {           // tile [32 e][64 k]: row = extended column, factor stored [r][Kc]
      const int row = wave * 8 + (lane >> 3);
      const int unit = (lane & 7) ^ ((row >> 1) & 7);
      int e = tn * SK_BX + row;
      if (e >= a.n_ext) e = a.n_ext - 1;
      const ExtCol c = a.ext_cols[e];
      x_src = (const bf16_t*)(a.which ? c.A : c.B) + (int64_t)c.q * a.Kc + kbeg + unit * 8;
      x_step = BK;
    } else {                         // tile [64 k][32 e], 64-byte rows: factor stored [Kc][r], r % 8 == 0
      const int k = wave * 16 + (lane >> 2);
      int e = tn * SK_BX + (lane & 3) * 8;
      if (e >= a.n_ext) e = a.n_ext - 8;
      const ExtCol c = a.ext_cols[e];
      const AdapterEntry en = a.table[c.t - a.ext_t0];     // (this storage form needs the rank)
      x_src = (const bf16_t*)(a.which ? en.A : en.B) + (kbeg + k) * en.rank + c.q;
      x_step = (int64_t)BK * en.rank;
    }
  }

  // DMA sources: 4 instructions (1 KB each) per wave per operand per k-tile.  The weight requests
  // do not depend on the token indices, so the first three k-tiles of the weight go out before
  // the indices are even loaded (three k-tiles stay in flight throughout).
  const bf16_t* a_src[4];
  const bf16_t* b_src[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (FORM == FORM_NT) {           // B tile [128 n][64 k], 128-byte rows
      const int row = (wave * 4 + j) * 8 + (lane >> 3);
      const int unit = (lane & 7) ^ ((row >> 1) & 7);
      int64_t n = n0 + row;
      if (n >= Nout) n = Nout - 1;
      b_src[j] = Bop + n * ldb + kbeg + unit * 8;
    } else {                         // B tile [64 k][128 n], 256-byte rows
      const int k = (wave * 4 + j) * 4 + (lane >> 4);
      int64_t n = n0 + (((lane & 15) ^ ((k & 3) << 2)) << 3);
      if (n >= Nout) n = Nout - 8;
      b_src[j] = Bop + (kbeg + k) * ldb + n;
    }
  }
  const int64_t b_step = FORM == FORM_NT ? (int64_t)BK : (int64_t)BK * ldb;
#pragma unroll
  for (int s3 = 0; s3 < 3; ++s3)
    if (s3 < ntile) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        __builtin_amdgcn_global_load_lds((gptr_t)b_src[j], (lptr_t)(smem + s3 * SK_SLOT + SK_A_BYTES + wave * 4096 + j * 1024), 16, 0, 0);
        b_src[j] += b_step;
      }
    }

  if (tid < SK_BM) {
    const int64_t m = m0 + tid;
    tok_s[tid] = m < a.T ? (a.perm ? a.perm[m] : (int32_t)m) : -1;
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int row = (wave * 4 + j) * 8 + (lane >> 3);
    const int unit = (lane & 7) ^ ((row >> 1) & 7);
    const int32_t tok = tok_s[row];
    a_src[j] = a.Aop + (int64_t)(tok < 0 ? tok_s[0] : tok) * a.lda + kbeg + unit * 8;
  }
#pragma unroll
  for (int s3 = 0; s3 < 3; ++s3)
    if (s3 < ntile) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        __builtin_amdgcn_global_load_lds((gptr_t)a_src[j], (lptr_t)(smem + s3 * SK_SLOT + wave * 4096 + j * 1024), 16, 0, 0);
        a_src[j] += BK;
      }
    }
  const int frow = lane & 31, fk = lane >> 5;
  const int a_row = wm * 64 + frow, b_row = wn * 64 + frow;
  const int a_off = a_row * 128, a_swz = (a_row >> 1) & 7;
  const int b_off = b_row * 128, b_swz = (b_row >> 1) & 7;
  int btr[2];
  {
    const int g16 = lane >> 4, i16 = lane & 15;
    const int kb = (g16 >> 1) * 8 + (i16 >> 2);
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      const int ncol = wn * 64 + nt * 32 + (g16 & 1) * 16 + 4 * (i16 & 3);
      btr[nt] = kb * 256 + (((ncol >> 3) ^ ((kb & 3) << 2)) << 4) + (ncol & 7) * 2;
    }
  }

  const int x_off = frow * 128, x_swz = (frow >> 1) & 7;        // NT fragment of the extended tile
  int xtr = 0;                                                   // NN: transposing read offset
  {
    const int g16 = lane >> 4, i16 = lane & 15;
    const int kb = (g16 >> 1) * 8 + (i16 >> 2);
    xtr = kb * 64 + ((g16 & 1) * 16 + 4 * (i16 & 3)) * 2;
  }
  f32x16 acc_x;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc_x[v] = 0.f;
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

#define SK_DMA_X(slot_)                                                                                   \
  do {                                                                                                    \
    if (EXT) {                                                                                            \
      __builtin_amdgcn_global_load_lds((gptr_t)x_src,                                                     \
          (lptr_t)(smem + (slot_) * SK_SLOT + SK_A_BYTES + SK_B_BYTES + wave * 1024), 16, 0, 0);           \
      x_src += x_step;                                                                                    \
    }                                                                                                     \
  } while (0)

  auto kstep = [&](const char* as, const char* bs, int ks) {
    bf16x8 af[2], bfr[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
      af[mt] = *(const bf16x8*)(as + a_off + mt * (32 * 128) + (((ks * 2 + fk) ^ a_swz) << 4));
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      if (FORM == FORM_NT) {
        bfr[nt] = *(const bf16x8*)(bs + b_off + nt * (32 * 128) + (((ks * 2 + fk) ^ b_swz) << 4));
      } else {
        const char* p = bs + btr[nt] + ks * (16 * 256);   // k & 3 is unchanged by steps of 4
        bfr[nt] = lds_read_frag_tr(p, p + 4 * 256);
      }
    }
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mt], bfr[nt], acc[mt][nt], 0, 0, 0);
    if (EXT) {
      const char* xs = bs + SK_B_BYTES;
      bf16x8 xf;
      if (FORM == FORM_NT) {
        xf = *(const bf16x8*)(xs + x_off + (((ks * 2 + fk) ^ x_swz) << 4));
      } else {
        const char* px = xs + xtr + ks * (16 * 64);
        xf = lds_read_frag_tr(px, px + 4 * 64);
      }
      acc_x = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wn ? af[1] : af[0], xf, acc_x, 0, 0, 0);
    }
  };

  // One wave per SIMD: nothing but the instruction order hides LDS and DMA latency, so the loop
  // is software-pipelined by hand (sched_barrier pins the order).  Fragments of k-step s + 1 are
  // read while the MFMAs of k-step s run; the wait + barrier for the next k-tile sits before the
  // last k-step, whose MFMAs cover the first fragment reads of the next tile and the DMA issue.
#define SK_READ(base_, ks_, af_, bf_)                                                                     \
  do {                                                                                                    \
    const char* _as = (base_);                                                                            \
    const char* _bs = _as + SK_A_BYTES;                                                                   \
    af_[0] = *(const bf16x8*)(_as + a_off + ((((ks_) * 2 + fk) ^ a_swz) << 4));                           \
    af_[1] = *(const bf16x8*)(_as + a_off + 32 * 128 + ((((ks_) * 2 + fk) ^ a_swz) << 4));                \
    if (FORM == FORM_NT) {                                                                                \
      bf_[0] = *(const bf16x8*)(_bs + b_off + ((((ks_) * 2 + fk) ^ b_swz) << 4));                         \
      bf_[1] = *(const bf16x8*)(_bs + b_off + 32 * 128 + ((((ks_) * 2 + fk) ^ b_swz) << 4));              \
    } else {                                                                                              \
      const char* _p0 = _bs + btr[0] + (ks_) * (16 * 256);                                                \
      const char* _p1 = _bs + btr[1] + (ks_) * (16 * 256);                                                \
      bf_[0] = lds_read_frag_tr(_p0, _p0 + 4 * 256);                                                      \
      bf_[1] = lds_read_frag_tr(_p1, _p1 + 4 * 256);                                                      \
    }                                                                                                     \
    if (EXT) {                                                                                            \
      const char* _xs = _bs + SK_B_BYTES;                                                                 \
      if (FORM == FORM_NT) {                                                                              \
        bf_[2] = *(const bf16x8*)(_xs + x_off + ((((ks_) * 2 + fk) ^ x_swz) << 4));                       \
      } else {                                                                                            \
        const char* _px = _xs + xtr + (ks_) * (16 * 64);                                                  \
        bf_[2] = lds_read_frag_tr(_px, _px + 4 * 64);                                                     \
      }                                                                                                   \
    }                                                                                                     \
    __builtin_amdgcn_sched_barrier(0);                                                                    \
  } while (0)
#define SK_MMAX(af_, bf_)                                                                                 \
  do {                                                                                                    \
    if (EXT) {                                                                                            \
      acc_x = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wn ? af_[1] : af_[0], bf_[2], acc_x, 0, 0, 0);                   \
      __builtin_amdgcn_sched_barrier(0);                                                                  \
    }                                                                                                     \
  } while (0)
#define SK_MMA1(af_, bf_, mt_, nt_)                                                                       \
  do {                                                                                                    \
    acc[mt_][nt_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af_[mt_], bf_[nt_], acc[mt_][nt_], 0, 0, 0);  \
    __builtin_amdgcn_sched_barrier(0);                                                                    \
  } while (0)
#define SK_DMA_B(sb_, j_)                                                                                 \
  do {                                                                                                    \
    __builtin_amdgcn_global_load_lds((gptr_t)b_src[j_], (lptr_t)((sb_) + SK_A_BYTES + (j_) * 1024), 16, 0, 0); \
    b_src[j_] += b_step;                                                                                \
  } while (0)
#define SK_DMA_A(sb_, j_)                                                                                 \
  do {                                                                                                    \
    __builtin_amdgcn_global_load_lds((gptr_t)a_src[j_], (lptr_t)((sb_) + (j_) * 1024), 16, 0, 0);         \
    a_src[j_] += BK;                                                                                      \
  } while (0)

  // (three k-tiles of A and B are in flight already;) the extended columns' source addresses
  // arrive last (two dependent table loads), so their requests go last
  if (ntile > 0) SK_DMA_X(0);
  if (ntile > 1) SK_DMA_X(1);
  if (ntile > 2) SK_DMA_X(2);
  if constexpr (FORM == FORM_NT) {
    // The compiler drains the whole LDS queue before the first use of any LDS result, which with
    // one wave per SIMD exposes the LDS latency at every k-step.  Here the fragment reads are
    // inline assembly (the compiler does not see them as pending), issued two k-steps ahead into
    // four fragment sets, and the waits are written by hand: LDS results return in order, so
    // "at most 2 x NR reads outstanding" means the set issued two steps ago is complete.
    constexpr int NR = EXT ? 5 : 4;                 // reads per k-step
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)smem;
    uint32_t ra[4], rb[4], rx[4];                   // this lane's fragment addresses in slot 0, per k-step
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      ra[ks] = lds0 + a_off + (((ks * 2 + fk) ^ a_swz) << 4);
      rb[ks] = lds0 + SK_A_BYTES + b_off + (((ks * 2 + fk) ^ b_swz) << 4);
      rx[ks] = lds0 + SK_A_BYTES + SK_B_BYTES + x_off + (((ks * 2 + fk) ^ x_swz) << 4);
    }
    bf16x8 f0[5], f1[5], f2[5], f3[5];              // a0 a1 b0 b1 x
#define SKP_READ(so_, ks_, f_)                                                                            \
  do {                                                                                                    \
    const uint32_t _a = ra[ks_] + (so_), _b = rb[ks_] + (so_);                                            \
    asm volatile("ds_read_b128 %0, %1" : "=v"(f_[0]) : "v"(_a));                                          \
    asm volatile("ds_read_b128 %0, %1 offset:4096" : "=v"(f_[1]) : "v"(_a));                              \
    asm volatile("ds_read_b128 %0, %1" : "=v"(f_[2]) : "v"(_b));                                          \
    asm volatile("ds_read_b128 %0, %1 offset:4096" : "=v"(f_[3]) : "v"(_b));                              \
    if (EXT) { const uint32_t _x = rx[ks_] + (so_); asm volatile("ds_read_b128 %0, %1" : "=v"(f_[4]) : "v"(_x)); } \
    __builtin_amdgcn_sched_barrier(0);                                                                    \
  } while (0)
#define SKP_WAIT(n_) do { asm volatile("s_waitcnt lgkmcnt(%0)" :: "n"(n_) : "memory"); __builtin_amdgcn_sched_barrier(0); } while (0)
#define SKP_MMA1(f_, mt_, nt_)                                                                            \
  do {                                                                                                    \
    acc[mt_][nt_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f_[mt_], f_[2 + nt_], acc[mt_][nt_], 0, 0, 0); \
    __builtin_amdgcn_sched_barrier(0);                                                                    \
  } while (0)
#define SKP_MMAX(f_)                                                                                      \
  do {                                                                                                    \
    if (EXT) {                                                                                            \
      acc_x = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wn ? f_[1] : f_[0], f_[4], acc_x, 0, 0, 0);          \
      __builtin_amdgcn_sched_barrier(0);                                                                  \
    }                                                                                                     \
  } while (0)
#define SKP_MMA(f_) do { SKP_MMA1(f_, 0, 0); SKP_MMA1(f_, 0, 1); SKP_MMA1(f_, 1, 1); SKP_MMA1(f_, 1, 0); SKP_MMAX(f_); } while (0)
    if (ntile > 0) {
      // (all three tiles: the per-tile counting of the loop needs each tile's requests adjacent)
      __builtin_amdgcn_s_waitcnt(VMCNT(0));
      asm volatile("s_barrier" ::: "memory");
      __builtin_amdgcn_sched_barrier(0);
      SKP_READ(0u, 0, f0);
      SKP_READ(0u, 1, f1);
    }
    int64_t kt = 0;
    // steady state: tile kt + 3 is requested during tile kt
    for (; kt + 3 < ntile; ++kt) {
      const uint32_t so = (uint32_t)(kt & (SK_SLOTS - 1)) * SK_SLOT;
      const uint32_t sn = (uint32_t)((kt + 1) & (SK_SLOTS - 1)) * SK_SLOT;
      SKP_READ(so, 2, f2); SKP_WAIT(2 * NR); SKP_MMA(f0);
      SKP_READ(so, 3, f3); SKP_WAIT(2 * NR); SKP_MMA(f1);
      // this wave's part of tile kt + 1 has landed (tile kt + 2 may still be in flight); after the
      // barrier everyone's has, and nobody still reads tile kt - 1, whose slot is filled next
      // (every read of it was waited for before its MFMAs, a tile ago)
      __builtin_amdgcn_s_waitcnt(VMCNT(SK_NI));
      asm volatile("s_barrier" ::: "memory");
      __builtin_amdgcn_sched_barrier(0);
      SKP_READ(sn, 0, f0); SKP_WAIT(2 * NR);
      char* sb = smem + (int)((kt + 3) & (SK_SLOTS - 1)) * SK_SLOT + wave * 4096;
      SKP_MMA1(f2, 0, 0);
      SK_DMA_B(sb, 0); SK_DMA_B(sb, 1); SK_DMA_B(sb, 2);
      SKP_MMA1(f2, 0, 1);
      SK_DMA_B(sb, 3); SK_DMA_A(sb, 0); SK_DMA_A(sb, 1);
      SKP_MMA1(f2, 1, 1);
      SK_DMA_A(sb, 2); SK_DMA_A(sb, 3);
      SK_DMA_X((int)((kt + 3) & (SK_SLOTS - 1)));
      SKP_MMA1(f2, 1, 0);
      SKP_MMAX(f2);
      SKP_READ(sn, 1, f1); SKP_WAIT(2 * NR); SKP_MMA(f3);
    }
    // the last three tiles are already requested
    for (; kt + 1 < ntile; ++kt) {
      const uint32_t so = (uint32_t)(kt & (SK_SLOTS - 1)) * SK_SLOT;
      const uint32_t sn = (uint32_t)((kt + 1) & (SK_SLOTS - 1)) * SK_SLOT;
      SKP_READ(so, 2, f2); SKP_WAIT(2 * NR); SKP_MMA(f0);
      SKP_READ(so, 3, f3); SKP_WAIT(2 * NR); SKP_MMA(f1);
      __builtin_amdgcn_s_waitcnt(VMCNT(0));
      asm volatile("s_barrier" ::: "memory");
      __builtin_amdgcn_sched_barrier(0);
      SKP_READ(sn, 0, f0); SKP_WAIT(2 * NR); SKP_MMA(f2);
      SKP_READ(sn, 1, f1); SKP_WAIT(2 * NR); SKP_MMA(f3);
    }
    // last tile: nothing follows
    if (kt < ntile) {
      const uint32_t so = (uint32_t)(kt & (SK_SLOTS - 1)) * SK_SLOT;
      SKP_READ(so, 2, f2); SKP_WAIT(2 * NR); SKP_MMA(f0);
      SKP_READ(so, 3, f3); SKP_WAIT(2 * NR); SKP_MMA(f1);
      SKP_WAIT(0);
      SKP_MMA(f2);
      SKP_MMA(f3);
    }
  } else {
    bf16x8 fa0[2], fb0[3], fa1[2], fb1[3];
    if (ntile > 0) {
      // (all three: the per-tile counting of the loop needs each tile's requests to be adjacent)
      __builtin_amdgcn_s_waitcnt(VMCNT(0));
      asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
      SK_READ(smem, 0, fa0, fb0);
    }
    // One k-step: the first MFMA (the compiler's wait for this step's fragments sits before it and
    // drains the LDS queue, so no younger read may be outstanding here), then the reads of the next
    // step into the other fragment set, then the remaining three MFMAs.
#define SK_STEP(ua_, ub_, base_, ks_, la_, lb_)                                                           \
    do {                                                                                                    \
      SK_MMA1(ua_, ub_, 0, 0);                                                                              \
      SK_READ(base_, ks_, la_, lb_);                                                                        \
      SK_MMA1(ua_, ub_, 0, 1); SK_MMA1(ua_, ub_, 1, 1); SK_MMA1(ua_, ub_, 1, 0); SK_MMAX(ua_, ub_);         \
    } while (0)
    // steady state: tile kt + 3 is requested during tile kt
    int64_t kt = 0;
    for (; kt + 3 < ntile; ++kt) {
      const char* cur = smem + (int)(kt & (SK_SLOTS - 1)) * SK_SLOT;
      SK_STEP(fa0, fb0, cur, 1, fa1, fb1);
      SK_STEP(fa1, fb1, cur, 2, fa0, fb0);
      SK_STEP(fa0, fb0, cur, 3, fa1, fb1);
      // this wave's part of tile kt + 1 has landed (tile kt + 2 may still be in flight) ...
      __builtin_amdgcn_s_waitcnt(VMCNT(SK_NI));
      // ... everyone's has, and nobody still reads tile kt - 1, whose slot is filled next
      asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
      __builtin_amdgcn_sched_barrier(0);
      char* sb = smem + (int)((kt + 3) & (SK_SLOTS - 1)) * SK_SLOT + wave * 4096;
      SK_MMA1(fa1, fb1, 0, 0);
      SK_READ(smem + (int)((kt + 1) & (SK_SLOTS - 1)) * SK_SLOT, 0, fa0, fb0);
      SK_DMA_B(sb, 0); SK_DMA_B(sb, 1); SK_DMA_B(sb, 2);
      SK_MMA1(fa1, fb1, 0, 1);
      SK_DMA_B(sb, 3);
      SK_DMA_A(sb, 0); SK_DMA_A(sb, 1);
      SK_MMA1(fa1, fb1, 1, 1);
      SK_DMA_A(sb, 2); SK_DMA_A(sb, 3);
      SK_MMA1(fa1, fb1, 1, 0);
      SK_DMA_X((int)((kt + 3) & (SK_SLOTS - 1)));
      SK_MMAX(fa1, fb1);
    }
    // drain: the last three tiles are already requested
    for (; kt < ntile; ++kt) {
      const char* cur = smem + (int)(kt & (SK_SLOTS - 1)) * SK_SLOT;
      SK_STEP(fa0, fb0, cur, 1, fa1, fb1);
      SK_STEP(fa1, fb1, cur, 2, fa0, fb0);
      SK_STEP(fa0, fb0, cur, 3, fa1, fb1);
      __builtin_amdgcn_s_waitcnt(VMCNT(0));
      asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
      __builtin_amdgcn_sched_barrier(0);
      // (after the last tile this reads a stale slot; those fragments are not used)
      SK_STEP(fa1, fb1, smem + (int)((kt + 1) & (SK_SLOTS - 1)) * SK_SLOT, 0, fa0, fb0);
    }
  }
  __syncthreads();
  // k tail of the last split: one masked tile through registers into slot 0
  if (kbeg + ntile * BK < kend) {
    const int64_t k0 = kbeg + ntile * BK;
    const uint4 zero4 = make_uint4(0, 0, 0, 0);
    char* as = smem;
    char* bs = smem + SK_A_BYTES;
    {
      const int lc = tid & 7, lr = tid >> 3;
      const bool ka = (k0 + lc * 8) < kend;
      for (int i = 0; i < 4; ++i) {
        const int row = lr + 32 * i;
        const int32_t tok = tok_s[row];
        uint4 v = zero4;
        if (ka && tok >= 0) v = *(const uint4*)(a.Aop + (int64_t)tok * a.lda + k0 + lc * 8);
        *(uint4*)(as + swz_rowk(row, lc)) = v;
        if (FORM == FORM_NT) {
          uint4 w = zero4;
          if (ka && (n0 + row) < Nout) w = *(const uint4*)(Bop + (n0 + row) * ldb + k0 + lc * 8);
          *(uint4*)(bs + swz_rowk(row, lc)) = w;
        }
      }
    }
    if (FORM == FORM_NN) {
      const int lc = tid & 15, lr = tid >> 4;
      for (int i = 0; i < 4; ++i) {
        const int k = lr + 16 * i;
        uint4 w = zero4;
        if ((k0 + k) < kend && (n0 + lc * 8) < Nout) w = *(const uint4*)(Bop + (k0 + k) * ldb + n0 + lc * 8);
        *(uint4*)(bs + k * 256 + ((lc ^ ((k & 3) << 2)) << 4)) = w;
      }
    }
    if (EXT) {
      char* xs = bs + SK_B_BYTES;
      if (FORM == FORM_NT) {
        const int lc = tid & 7, row = tid >> 3;             // 32 rows x 8 units
        int e = tn * SK_BX + row;
        if (e >= a.n_ext) e = a.n_ext - 1;
        const ExtCol c = a.ext_cols[e];
        uint4 w = zero4;
        if ((k0 + lc * 8) < kend) w = *(const uint4*)((const bf16_t*)(a.which ? c.A : c.B) + (int64_t)c.q * a.Kc + k0 + lc * 8);
        *(uint4*)(xs + swz_rowk(row, lc)) = w;
      } else {
        const int lc = tid & 3, k = tid >> 2;               // 64 k-rows x 4 units
        int e = tn * SK_BX + lc * 8;
        if (e >= a.n_ext) e = a.n_ext - 8;
        const ExtCol c = a.ext_cols[e];
        uint4 w = zero4;
        const AdapterEntry en = a.table[c.t - a.ext_t0];
        if ((k0 + k) < kend) w = *(const uint4*)((const bf16_t*)(a.which ? en.A : en.B) + (k0 + k) * en.rank + c.q);
        *(uint4*)(xs + k * 64 + lc * 16) = w;
      }
    }
    __syncthreads();
    const int ksteps = (int)((kend - k0 + 15) / 16);
    for (int ks = 0; ks < ksteps; ++ks) kstep(as, bs, ks);
  }
  float* part = a.partials + ((int64_t)ks_idx * a.pm + m0 + wm * 64) * a.ldp + pn0 + wn * 64 + (lane & 31);
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = mt * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) part[(int64_t)row * a.ldp + nt * 32] = acc[mt][nt][v];
    }
  if (EXT) {
    // this wave's 32 rows (row block 2 wm + wn of the tile) x the tile's 32 extended columns
    float* up = a.u_part + ((int64_t)ks_idx * a.pm + m0 + wm * 64 + wn * 32) * a.ldu + tn * SK_BX + (lane & 31);
#pragma unroll
    for (int v = 0; v < 16; ++v) up[(int64_t)(8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)) * a.ldu] = acc_x[v];
  }
}

// Second step of the split-K path: add the partial sums in split order, add the LoRA expand in
// fp32 (u is fp32, so no two-term split is needed here) and scatter the rows.  A block owns one
// row chunk (up to 8 consecutive grouped rows of one adapter) x 512 columns, 2 per thread, so the
// adapter's factor is read once per chunk and every load of a block is issued up front.  With a
// column-chunk count that is a multiple of 8, column chunk c of every row chunk runs on XCD
// c mod 8, whose L2 then holds that slice of each factor.
static constexpr int FIN_THREADS = 256;
static constexpr int FIN_COLS = 2 * FIN_THREADS;

template <int FORM, bool OUT_F32>
__global__ __launch_bounds__(FIN_THREADS) void splitk_finish_kernel(GemmArgs a) {
  constexpr int R = ROW_CHUNK;
  constexpr int UPT = R * 128 / FIN_THREADS;        // u values staged per thread
  __shared__ float u_s[R][128];
  const int tid = threadIdx.x;
  const int ncol = a.fin_cols;
  int col = blockIdx.x % ncol;
  const RowChunk ch = a.chunks[blockIdx.x / ncol];
  // the projection this column chunk belongs to (block-uniform)
  int64_t Nout = a.Nout, ldo = a.ldo, pcol0 = 0;
  void* outp = a.out;
  int tab0 = 0;
  if (a.n_proj > 1) {
    int p = 0;
    for (int q = 1; q < a.n_proj; ++q) if (col >= a.proj[q].fin0) p = q;
    const ProjEntry pe = a.proj[p];
    Nout = pe.Nout; ldo = pe.ldo; outp = pe.out; tab0 = pe.tab0;
    pcol0 = (int64_t)pe.tile0 * SK_BN;
    col -= pe.fin0;
  }
  const int64_t n = (int64_t)col * FIN_COLS + 2 * tid;
  const bool active = n < Nout;                     // Nout is a multiple of 8
  const int64_t kstride = a.pm * a.ldp;
  const bool lora_on = ch.t >= 0 && (a.U != nullptr || a.n_ext > 0);
  // A block's run time is a few dependent memory round trips plus the partial-sum traffic, so
  // the loads are requested in the order of their dependence depth: adapter entry, then u and
  // the factor (ranks up to 32 are prefetched into registers), then the partial sums.
  AdapterEntry e;
  e.A = nullptr; e.B = nullptr; e.rank = 0; e.scale = 0.f;
  float ureg[UPT];
  uint4 wa[4], wb[4];          // FORM_NT prefetch: rows n and n + 1 of the factor, 8 ranks per entry
  uint32_t wn[32];             // FORM_NN prefetch: columns n, n + 1 of factor row q
  const bf16_t* L = nullptr;
  bool pref = false;
  if (lora_on) {
    e = a.table[tab0 + ch.t];
    L = (const bf16_t*)(a.which ? e.B : e.A);
    const int r = e.rank;
    if (a.n_ext > 0) {
      // fused shrink: u = scale * (sum over the splits of this adapter's extended columns)
      const int roff = a.ext_roff[tab0 + ch.t] - a.ext_base;
      const int64_t ustride = a.pm * a.ldu;
#pragma unroll
      for (int i = 0; i < UPT; ++i) {
        const int j = (tid >> 7) + i * (FIN_THREADS >> 7), q = tid & 127;
        float sum = 0.f;
        if (j < ch.nrows && q < r) {
          const float* up = a.u_part + (int64_t)(ch.row0 + j) * a.ldu + roff + q;
          for (int ks0 = 0; ks0 < a.ksplit; ks0 += 4) {
            float pu[4];
#pragma unroll
            for (int ii = 0; ii < 4; ++ii) pu[ii] = up[(ks0 + ii < a.ksplit ? ks0 + ii : a.ksplit - 1) * ustride];
#pragma unroll
            for (int ii = 0; ii < 4; ++ii) if (ks0 + ii < a.ksplit) sum += pu[ii];
          }
          sum *= e.scale;
        }
        // (ranks r .. r_stride - 1 are padding of the row: zeros, as the shrink kernels write them)
        if (col == 0 && a.u_out && j < ch.nrows && q < a.r_stride) a.u_out[(int64_t)(ch.row0 + j) * a.r_stride + q] = sum;
        ureg[i] = sum;
      }
    } else {
#pragma unroll
      for (int i = 0; i < UPT; ++i) {
        const int j = (tid >> 7) + i * (FIN_THREADS >> 7), q = tid & 127;
        ureg[i] = (j < ch.nrows && q < r) ? a.U[(int64_t)(ch.row0 + j) * a.r_stride + q] : 0.f;
      }
    }
    pref = r <= 32 && (FORM == FORM_NN || (r & 7) == 0);
    if (pref && active) {
      if (FORM == FORM_NT) {               // L[n * r + q]
#pragma unroll
        for (int qt = 0; qt < 4; ++qt)
          if (qt * 8 < r) {
            wa[qt] = *(const uint4*)(L + n * r + qt * 8);
            wb[qt] = *(const uint4*)(L + (n + 1) * r + qt * 8);
          }
      } else {                             // L[q * Nout + n]
#pragma unroll
        for (int q = 0; q < 32; ++q)
          if (q < r) wn[q] = *(const uint32_t*)(L + (int64_t)q * Nout + n);
      }
    }
  }
  // partial sums of every row of the chunk, in split order; four splits (32 loads) at a time
  float y0[R], y1[R];
  {
    const float* part = a.partials + (int64_t)ch.row0 * a.ldp + pcol0 + (active ? n : 0);
#pragma unroll
    for (int j = 0; j < R; ++j) { y0[j] = 0.f; y1[j] = 0.f; }
    for (int ks0 = 0; ks0 < a.ksplit; ks0 += 4) {
      float2 p[4][R];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int ks = ks0 + i < a.ksplit ? ks0 + i : a.ksplit - 1;
        const float* pk = part + ks * kstride;
#pragma unroll
        for (int j = 0; j < R; ++j) p[i][j] = *(const float2*)(pk + (j < ch.nrows ? j : 0) * a.ldp);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool on = ks0 + i < a.ksplit;
#pragma unroll
        for (int j = 0; j < R; ++j) {
          if (on && j < ch.nrows) { y0[j] += p[i][j].x; y1[j] += p[i][j].y; }
        }
      }
    }
  }
  if (lora_on) {
    const int r = e.rank;
#pragma unroll
    for (int i = 0; i < UPT; ++i) u_s[(tid >> 7) + i * (FIN_THREADS >> 7)][tid & 127] = ureg[i];
    __syncthreads();
    if (active) {
      if (pref && FORM == FORM_NT) {
#pragma unroll
        for (int qt = 0; qt < 4; ++qt)
          if (qt * 8 < r) {
            const uint32_t aw[4] = {wa[qt].x, wa[qt].y, wa[qt].z, wa[qt].w}, bw[4] = {wb[qt].x, wb[qt].y, wb[qt].z, wb[qt].w};
            float fa[8], fb[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
              fa[i] = __uint_as_float((aw[i >> 1] >> ((i & 1) * 16)) << 16);
              fb[i] = __uint_as_float((bw[i >> 1] >> ((i & 1) * 16)) << 16);
            }
#pragma unroll
            for (int j = 0; j < R; ++j) {
              float sa = 0.f, sb = 0.f;
#pragma unroll
              for (int i = 0; i < 8; ++i) {
                const float uq = u_s[j][qt * 8 + i];
                sa = fmaf(uq, fa[i], sa); sb = fmaf(uq, fb[i], sb);
              }
              y0[j] += sa; y1[j] += sb;
            }
          }
      } else if (pref) {
#pragma unroll
        for (int q = 0; q < 32; ++q)
          if (q < r) {
            const float fa = __uint_as_float(wn[q] << 16), fb = __uint_as_float(wn[q] & 0xffff0000u);
#pragma unroll
            for (int j = 0; j < R; ++j) { y0[j] = fmaf(u_s[j][q], fa, y0[j]); y1[j] = fmaf(u_s[j][q], fb, y1[j]); }
          }
      } else if (FORM == FORM_NT) {        // any rank: stream the factor
        for (int q = 0; q < r; ++q) {
          const float fa = bf16_bits_to_float(L[n * r + q]), fb = bf16_bits_to_float(L[(n + 1) * r + q]);
#pragma unroll
          for (int j = 0; j < R; ++j) { y0[j] = fmaf(u_s[j][q], fa, y0[j]); y1[j] = fmaf(u_s[j][q], fb, y1[j]); }
        }
      } else {
        for (int q = 0; q < r; ++q) {
          const uint32_t w = *(const uint32_t*)(L + (int64_t)q * Nout + n);
          const float fa = __uint_as_float(w << 16), fb = __uint_as_float(w & 0xffff0000u);
#pragma unroll
          for (int j = 0; j < R; ++j) { y0[j] = fmaf(u_s[j][q], fa, y0[j]); y1[j] = fmaf(u_s[j][q], fb, y1[j]); }
        }
      }
    }
  }
  if (!active) return;
#pragma unroll
  for (int j = 0; j < R; ++j) {
    if (j < ch.nrows) {
      const int64_t m = ch.row0 + j;
      const int64_t tok = a.perm ? a.perm[m] : m;
      if (OUT_F32) *(float2*)((float*)outp + tok * ldo + n) = make_float2(y0[j], y1[j]);
      else *(uint32_t*)((bf16_t*)outp + tok * ldo + n) = float_to_bf16_bits(y0[j]) | ((uint32_t)float_to_bf16_bits(y1[j]) << 16);
    }
  }
}

// dst[c][r] = src[r][c] for a bf16 matrix of R rows and C columns (both multiples of 8), 64 x 64
// tiles.  Used to give a large-batch GEMM whose weight is stored output-contiguous the
// contraction-contiguous form, whose LDS fragment reads are plain 16-byte reads.
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const bf16_t* __restrict__ src, int64_t lds_,
                                                             bf16_t* __restrict__ dst, int64_t ldd, int64_t R, int64_t C) {
  __shared__ __attribute__((aligned(16))) bf16_t s[64][72];   // s[c][r]
  const int tid = threadIdx.x, tx = tid & 7, ty = tid >> 3;
  const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int r = ty + 32 * i;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (r0 + r < R && c0 + tx * 8 < C) v = *(const uint4*)(src + (r0 + r) * lds_ + c0 + tx * 8);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 8; ++j) s[tx * 8 + j][r] = (bf16_t)(w[j >> 1] >> ((j & 1) * 16));
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int c = ty + 32 * i;
    if (c0 + c < C && r0 + tx * 8 < R) *(uint4*)(dst + (c0 + c) * ldd + r0 + tx * 8) = *(const uint4*)&s[c][tx * 8];
  }
}

hipError_t launch_transpose_bf16(const bf16_t* src, int64_t lds, bf16_t* dst, int64_t ldd, int64_t R, int64_t C, hipStream_t stream) {
  if (R <= 0 || C <= 0) return hipSuccess;
  hipLaunchKernelGGL(transpose_bf16_kernel, dim3((unsigned)((C + 63) / 64), (unsigned)((R + 63) / 64)), dim3(256), 0, stream, src, lds, dst,
                     ldd, R, C);
  return hipGetLastError();
}

// rows of a batch from which transposing the weight into scratch pays for itself
static constexpr int64_t WT_MIN_ROWS = 4096;

// Raise a kernel's dynamic LDS limit once per device (done: bit i set = device i has it).
static hipError_t allow_lds(const void* kernel, int bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = 1ull << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
  return e;
}

// One thread per 256-row tile: the adapter segments that intersect the tile's rows, each cut into
// 64-wide pieces of its 2 r_pad extra contraction values (the rows are grouped by adapter, so the
// segments of a tile are consecutive adapters).
__global__ __launch_bounds__(64) void lora_tile_list_kernel(const int32_t* __restrict__ seg_off, int n_adapters,
                                                            const AdapterEntry* __restrict__ table, int tiles_m,
                                                            int32_t* __restrict__ out) {
  const int tm = blockIdx.x * 64 + threadIdx.x;
  if (tm >= tiles_m) return;
  int32_t* o = out + (int64_t)tm * LT_STRIDE;
  const int64_t m0 = (int64_t)tm * BM;
  const int64_t T_lora = seg_off[n_adapters];
  const int64_t m_end = (m0 + BM) < T_lora ? (m0 + BM) : T_lora;
  int cnt = 0;
  if (m0 < m_end) {
    int t = segment_of(seg_off, n_adapters, (int)m0);
    while (cnt >= 0 && t < n_adapters && (int64_t)seg_off[t] < m_end) {
      const int64_t lo = seg_off[t] > m0 ? (int64_t)seg_off[t] : m0;
      const int64_t hi = (int64_t)seg_off[t + 1] < m_end ? (int64_t)seg_off[t + 1] : m_end;
      if (hi > lo) {
        const int kext = 2 * ((table[t].rank + 15) & ~15);
        for (int kc = 0; kc < kext; kc += BK) {
          if (cnt == LT_MAX) { cnt = -1; break; }
          o[1 + 4 * cnt] = t; o[2 + 4 * cnt] = (int32_t)lo; o[3 + 4 * cnt] = (int32_t)hi; o[4 + 4 * cnt] = kc;
          ++cnt;
        }
      }
      ++t;
    }
  }
  o[0] = cnt;
}

template <int FORM, bool OUT_F32, int LFORM = FORM>
static hipError_t launch_wide(const GemmArgs& a, hipStream_t stream) {
  static std::atomic<uint64_t> done{0};
  if (a.lora_dma) {
    hipLaunchKernelGGL(lora_tile_list_kernel, dim3((a.tiles_m + 63) / 64), dim3(64), 0, stream, a.seg_off, a.n_adapters, a.table,
                       a.tiles_m, (int32_t*)a.lora_tiles);
    hipError_t el = hipGetLastError();
    if (el != hipSuccess) return el;
  }
  hipError_t e0 = allow_lds((const void*)gemm_bf16_kernel<FORM, OUT_F32, LFORM>, GEMM_LDS, done);
  if (e0 != hipSuccess) return e0;
  hipLaunchKernelGGL((gemm_bf16_kernel<FORM, OUT_F32, LFORM>), dim3(a.tiles_m * a.tiles_n * a.ksplit), dim3(GEMM_THREADS),
                     GEMM_LDS, stream, a);
  return hipGetLastError();
}

template <int FORM, bool OUT_F32>
static hipError_t launch_one(const GemmArgs& a, int mode, bool packed, hipStream_t stream) {
  static std::atomic<uint64_t> done_wide{0}, done_sk{0}, done_skx{0};
  hipError_t e0 = allow_lds((const void*)gemm_bf16_kernel<FORM, OUT_F32>, GEMM_LDS, done_wide);
  if (e0 == hipSuccess) e0 = allow_lds((const void*)gemm_skinny_kernel<FORM, false>, SK_LDS, done_sk);
  if (e0 == hipSuccess) e0 = allow_lds((const void*)gemm_skinny_kernel<FORM, true>, SK_LDS, done_skx);
  if (e0 != hipSuccess) return e0;
  const int G = a.tiles_m * a.tiles_n;
  if (mode == 2 && packed) {
    // packed weight: its fragments go straight into registers (gemm_decode.hip)
    hipError_t ed = launch_gemm_decode(a, stream);
    if (ed != hipSuccess) return ed;
  } else if (mode == 2 && a.n_ext > 0)
    hipLaunchKernelGGL((gemm_skinny_kernel<FORM, true>), dim3(G * a.ksplit), dim3(256), SK_LDS, stream, a);
  else if (mode == 2)
    hipLaunchKernelGGL((gemm_skinny_kernel<FORM, false>), dim3(G * a.ksplit), dim3(256), SK_LDS, stream, a);
  else {
    hipError_t ew = launch_wide<FORM, OUT_F32, FORM>(a, stream);
    if (ew != hipSuccess) return ew;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || mode == 0 || (packed && a.fin_in_kernel)) return e;
  const int64_t fin_blocks = (int64_t)a.fin_cols * a.n_chunks;
  hipLaunchKernelGGL((splitk_finish_kernel<FORM, OUT_F32>), dim3((unsigned)fin_blocks), dim3(FIN_THREADS), 0, stream, a);
  return hipGetLastError();
}

// How a call is tiled.  mode 0: one 256 x 256 workgroup per tile; mode 1: 256 x 256 tiles with
// the contraction split; mode 2: 128 x 128 tiles with the contraction split (small batches),
// which can also carry the shrink as 32 extended columns per column tile.
struct GemmPlan { int mode, tiles_m, tiles_n, ksplit; int64_t kchunk, ldp, pm, ldu; size_t bytes, u_bytes; };

static constexpr int CUS = 256;        // compute units; every GEMM kernel here runs one workgroup on each

// The plan for a given mode and (requested) number of contraction splits.
static GemmPlan plan_for(int mode, int64_t s, int64_t T, int64_t Kc, int64_t Nout, int n_ext) {
  GemmPlan p;
  const int64_t tile_h = mode == 2 ? SK_BM : BM, tile_w = mode == 2 ? SK_BN : BN;
  p.mode = mode;
  p.tiles_m = (int)((T + tile_h - 1) / tile_h);
  p.tiles_n = (int)((Nout + tile_w - 1) / tile_w);
  p.ksplit = 1; p.kchunk = Kc; p.ldp = 0; p.pm = 0; p.bytes = 0; p.ldu = 0; p.u_bytes = 0;
  if (mode == 0) return p;
  int64_t kc = (Kc + s - 1) / s;
  kc = (kc + BK - 1) / BK * BK;
  p.kchunk = kc;
  p.ksplit = (int)((Kc + kc - 1) / kc);
  p.ldp = (int64_t)p.tiles_n * tile_w;
  p.pm = (int64_t)p.tiles_m * tile_h;
  p.bytes = (size_t)p.ksplit * p.pm * p.ldp * sizeof(float);
  if (mode == 2 && n_ext > 0 && n_ext <= SK_BX * p.tiles_n) {
    p.ldu = (int64_t)p.tiles_n * SK_BX;
    p.u_bytes = (size_t)p.ksplit * p.pm * p.ldu * sizeof(float);
  }
  return p;
}

// Estimated run time of a plan in microseconds, from rates measured with one workgroup per
// compute unit: time per 64-deep k-tile (128 x 128 tiles are bound by the LDS fill rate, less so
// when fewer than 256 workgroups share it), a fixed cost per round of workgroups, a separate
// shrink launch where the GEMM does not carry it, and the partial sums written once and read
// once at about 5 TB/s.  Only the ordering of the candidates matters.
static double plan_cost(const GemmPlan& p, int n_ext) {
  const int64_t wgs = (int64_t)p.tiles_m * p.tiles_n * p.ksplit;
  const int64_t rounds = (wgs + CUS - 1) / CUS;
  const int64_t ktiles = (p.kchunk + BK - 1) / BK;
  double us;
  if (p.mode == 2) {
    const double share = 0.75 + 0.25 * (wgs < CUS ? (double)wgs / CUS : 1.0);
    us = (double)rounds * (ktiles * 0.9 * share + 4.5);
  } else {
    us = (double)rounds * (ktiles * (p.mode == 1 ? 1.6 : 2.0) + 16.0);
  }
  if (n_ext > 0 && p.u_bytes == 0) us += 7.0;
  if (p.mode != 0) us += 3.5 + 2.0 * (double)(p.bytes + p.u_bytes) / 5.0e6;
  return us;
}

// small_only: only the 128 x 128 kernels are candidates (the several-projections pass exists for
// them alone); the unsplit large-batch plan is returned when none of them qualifies.
static GemmPlan gemm_plan(int64_t T, int64_t Kc, int64_t Nout, int n_ext, bool small_only = false) {
  GemmPlan best = plan_for(0, 1, T, Kc, Nout, n_ext);
  const int64_t G = (int64_t)best.tiles_m * best.tiles_n;
  if (G <= 0 || G > CUS / 2) return best;          // at least half a round of 256 x 256 tiles: no split
  double best_us = small_only ? 1e30 : plan_cost(best, n_ext);
  for (int mode = small_only ? 2 : 1; mode <= 2; ++mode) {
    const int64_t min_k = mode == 2 ? 256 : 128;    // contraction values per split, at least
    int64_t max_s = Kc / min_k;
    if (max_s > 32) max_s = 32;
    int last = 0;
    for (int64_t s = 1; s <= max_s; ++s) {
      const GemmPlan p = plan_for(mode, s, T, Kc, Nout, n_ext);
      if (p.ksplit == last) continue;               // rounding the chunk to whole k-tiles gave the same split
      last = p.ksplit;
      if ((int64_t)p.tiles_m * p.tiles_n * p.ksplit > 4 * CUS) break;
      const double us = plan_cost(p, n_ext);
      if (us < best_us) { best_us = us; best = p; }
    }
  }
  return best;
}

size_t gemm_splitk_bytes(int64_t T, int64_t Kc, int64_t Nout, int n_ext) {
  if (T <= 0 || Nout <= 0) return 0;
  const GemmPlan p = gemm_plan(T, Kc, Nout, n_ext);
  return p.bytes + p.u_bytes;
}

size_t gemm_wt_bytes(int form, int64_t T, int64_t Kc, int64_t Nout) {
  if (form != FORM_NN || T < WT_MIN_ROWS || Kc <= 0 || Nout <= 0 || Kc > 65535 * 64) return 0;
  if (gemm_plan(T, Kc, Nout, 0).mode != 0) return 0;
  return (size_t)Kc * Nout * sizeof(bf16_t);
}

bool gemm_can_fuse_shrink(int form, int64_t T, int64_t Kc, int64_t Nout, int n_ext, bool ranks_mult8,
                          size_t partial_bytes) {
  if (T <= 0 || Nout <= 0 || n_ext <= 0) return false;
  if (form == FORM_NN && !ranks_mult8) return false;     // 16-byte DMA units must not straddle adapters
  const GemmPlan p = gemm_plan(T, Kc, Nout, n_ext);
  return p.mode == 2 && p.u_bytes > 0 && partial_bytes >= p.bytes + p.u_bytes;
}

size_t lora_tiles_bytes(int64_t T) {
  return T > 0 ? (size_t)((T + BM - 1) / BM) * LT_STRIDE * sizeof(int32_t) : 0;
}

// Way the decode kernel's call is finished: the one asked for where its conditions hold, else the
// next best.  Both ways other than the generic finish kernel need the splits to divide a tile's
// 32 units and u of a tile's rows to fit in LDS.  The in-kernel way also needs its counters; with
// several splits it is only taken when every workgroup of the launch fits on the chip at once, so
// that the splits of a tile normally run at the same time (a split that does not see the others
// in time leaves its share to the last one: correct either way).  DECODE_FINISH_AUTO: in the
// kernel when there is one split (the sums never leave the registers; only u crosses workgroups,
// and the column tiles that carry it are the first to be scheduled), a launch of its own otherwise
// (measured: the counters' round trips cost more than the second launch once 16 MB of partial
// sums have to cross anyway).
static int decode_finish_mode(const DecodeSync* sync, int n_adapters, int r_stride, int tiles_m, int tiles_n, int ksplit) {
  if (!sync || sync->mode == DECODE_FINISH_GENERIC || (n_adapters > 0 && !sync->grp_ids)) return DECODE_FINISH_GENERIC;
  if (n_adapters > 0 && r_stride > 128) return DECODE_FINISH_GENERIC;
  if (ksplit != 1 && ksplit != 2 && ksplit != 4 && ksplit != 8) return DECODE_FINISH_GENERIC;
  int want = sync->mode;
  if (want == DECODE_FINISH_AUTO) want = ksplit == 1 ? DECODE_FINISH_IN_KERNEL : DECODE_FINISH_LAUNCH;
  if (want == DECODE_FINISH_LAUNCH) return DECODE_FINISH_LAUNCH;
  const int64_t tiles = (int64_t)tiles_m * tiles_n;
  if (sync->counters && 2 * tiles + 2 * tiles_m <= DECODE_SYNC_INTS && (ksplit == 1 || tiles * ksplit <= sync->cu_count))
    return DECODE_FINISH_IN_KERNEL;
  return DECODE_FINISH_LAUNCH;
}

hipError_t launch_gemm_bf16(const bf16_t* Aop, int64_t lda, const bf16_t* Bop, int64_t ldb,
                            int form, int64_t T, int64_t Kc, int64_t Nout, const int32_t* perm,
                            const int32_t* seg_off, int n_adapters, const AdapterEntry* table,
                            int which, const float* U, int r_stride, void* out, int64_t ldo,
                            int out_is_f32, float* partials, size_t partial_bytes, const RowChunk* chunks,
                            int n_chunks, const GemmFuse* fuse, bf16_t* wt_scratch, size_t wt_bytes, const bf16_t* Bt_kept, const LoraDma* dma,
                            const bf16_t* Bpacked, const DecodeSync* sync, hipStream_t stream) {
  if (T <= 0 || Nout <= 0) return hipSuccess;
  if (ldb > (1 << 22)) return hipErrorInvalidValue;      // 32-bit byte offsets inside a weight tile
  GemmArgs a;
  a.Aop = Aop; a.lda = lda; a.Bop = Bop; a.ldb = ldb; a.T = T; a.Kc = Kc; a.Nout = Nout;
  a.perm = perm; a.seg_off = seg_off; a.n_adapters = n_adapters; a.table = table; a.which = which;
  a.U = U; a.r_stride = r_stride; a.out = out; a.ldo = ldo;
  GemmPlan p = gemm_plan(T, Kc, Nout, fuse ? fuse->n_ext : 0);
  a.ext_cols = nullptr; a.ext_roff = nullptr; a.n_ext = 0; a.u_part = nullptr; a.ldu = 0; a.u_out = nullptr;
  a.ext_t0 = 0; a.ext_base = 0;
  memset(a.proj, 0, sizeof a.proj);
  a.n_proj = 1; a.fin_cols = (int)((Nout + FIN_COLS - 1) / FIN_COLS);
  a.fin_in_kernel = 0; a.out_is_f32 = out_is_f32; a.lform = form; a.spin_limit = 0;
  a.sync = nullptr; a.grp_ids = nullptr;
  if (fuse) {
    // the caller skipped the shrink: the conditions of gemm_can_fuse_shrink() must hold
    if (!gemm_can_fuse_shrink(form, T, Kc, Nout, fuse->n_ext, fuse->ranks_mult8, partials ? partial_bytes : 0) || chunks == nullptr)
      return hipErrorInvalidValue;
    a.ext_cols = fuse->cols; a.ext_roff = fuse->roff; a.n_ext = fuse->n_ext;
    a.ext_t0 = fuse->t0; a.ext_base = fuse->ext_base;
    a.u_part = partials + p.bytes / sizeof(float); a.ldu = p.ldu; a.u_out = fuse->u_out;
    a.U = nullptr;
  }
  if (p.mode != 0 && (partials == nullptr || partial_bytes < p.bytes || chunks == nullptr)) {
    // no scratch for partial sums: one 256 x 256 workgroup per tile
    p.mode = 0; p.ksplit = 1; p.kchunk = Kc; p.ldp = 0; p.pm = 0;
    p.tiles_m = (int)((T + BM - 1) / BM);
    p.tiles_n = (int)((Nout + BN - 1) / BN);
  }
  a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n; a.ksplit = p.ksplit; a.kchunk = p.kchunk;
  a.ldp = p.ldp; a.pm = p.pm; a.partials = partials; a.chunks = chunks; a.n_chunks = n_chunks;
  // large batch, unsplit: the expand's operands by DMA when the shrink left u as a bf16 split, the
  // row tiles' lists have room, and every 16-byte piece of a factor row stays inside the row
  a.U2 = nullptr; a.lora_tiles = nullptr; a.zero_line = nullptr; a.lora_dma = 0;
  if (dma && dma->u2 && dma->tiles && dma->zero_line && p.mode == 0 && p.ksplit == 1 && n_adapters > 0 && U != nullptr &&
      (form == FORM_NN || dma->ranks_mult8) && dma->tiles_bytes >= (size_t)p.tiles_m * LT_STRIDE * sizeof(int32_t)) {
    a.U2 = dma->u2; a.lora_tiles = dma->tiles; a.zero_line = dma->zero_line; a.lora_dma = 1;
  }
  // small batch with a packed copy of the weight (and, when the shrink is fused, factors stored
  // contraction-contiguous): the decode kernel reads the packed copy instead of Bop
  const bool packed = Bpacked != nullptr && p.mode == 2 && (fuse == nullptr || form == FORM_NT);
  if (packed) {
    a.Bop = Bpacked; a.ldb = packed_weight_ksteps(Kc);
    a.fin_in_kernel = decode_finish_mode(sync, n_adapters, r_stride, p.tiles_m, p.tiles_n, p.ksplit);
    if (a.fin_in_kernel) { a.sync = sync->counters; a.grp_ids = sync->grp_ids; a.spin_limit = sync->spin_limit; }
  }
  if (form == FORM_NT)
    return out_is_f32 ? launch_one<FORM_NT, true>(a, p.mode, packed, stream) : launch_one<FORM_NT, false>(a, p.mode, packed, stream);
  if (p.mode == 0 && Bt_kept != nullptr) {
    // large batch, weight stored [Kc][Nout], and the caller keeps a transposed copy of it
    a.Bop = Bt_kept; a.ldb = Kc;
    return out_is_f32 ? launch_wide<FORM_NT, true, FORM_NN>(a, stream) : launch_wide<FORM_NT, false, FORM_NN>(a, stream);
  }
  if (p.mode == 0 && wt_scratch != nullptr && wt_bytes >= gemm_wt_bytes(form, T, Kc, Nout) && gemm_wt_bytes(form, T, Kc, Nout) > 0) {
    // large batch, weight stored [Kc][Nout]: transpose it into scratch ([Nout][Kc]) and run the
    // contraction-contiguous kernel; the adapters' factors keep their storage
    hipLaunchKernelGGL(transpose_bf16_kernel, dim3((unsigned)((Nout + 63) / 64), (unsigned)((Kc + 63) / 64)), dim3(256), 0,
                       stream, Bop, ldb, wt_scratch, Kc, Kc, Nout);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    a.Bop = wt_scratch; a.ldb = Kc;
    return out_is_f32 ? launch_wide<FORM_NT, true, FORM_NN>(a, stream) : launch_wide<FORM_NT, false, FORM_NN>(a, stream);
  }
  return out_is_f32 ? launch_one<FORM_NN, true>(a, p.mode, packed, stream) : launch_one<FORM_NN, false>(a, p.mode, packed, stream);
}

// ---- several projections in one pass
static int64_t multi_tiles(const ProjEntry* proj, int n_proj) {
  int64_t tiles = 0;
  for (int p = 0; p < n_proj; ++p) tiles += (proj[p].Nout + SK_BN - 1) / SK_BN;
  return tiles;
}

size_t gemm_multi_bytes(int64_t T, int64_t Kc, const ProjEntry* proj_host, int n_proj, int n_ext) {
  if (T <= 0 || n_proj <= 0) return 0;
  const GemmPlan p = gemm_plan(T, Kc, multi_tiles(proj_host, n_proj) * SK_BN, n_ext, true);
  return p.mode == 2 ? p.bytes + p.u_bytes : 0;
}

bool gemm_multi_ok(int form, int64_t T, int64_t Kc, const ProjEntry* proj_host, int n_proj, int n_ext,
                   bool ranks_mult8, size_t partial_bytes) {
  if (T <= 0 || n_proj < 2 || n_ext < 0) return false;
  if (n_ext > 0 && form == FORM_NN && !ranks_mult8) return false;
  const int64_t tiles = multi_tiles(proj_host, n_proj);
  if (tiles * SK_BN > (1 << 24)) return false;
  const GemmPlan p = gemm_plan(T, Kc, tiles * SK_BN, n_ext, true);
  if (p.mode != 2 || (n_ext > 0 && p.u_bytes == 0)) return false;
  return partial_bytes >= p.bytes + p.u_bytes;
}

hipError_t launch_gemm_bf16_multi(const bf16_t* Aop, int64_t lda, int form, int64_t T, int64_t Kc,
                                  const int32_t* perm, const int32_t* seg_off, int n_adapters,
                                  const AdapterEntry* table, const ProjEntry* proj_host,
                                  int n_proj, int out_is_f32, float* partials,
                                  size_t partial_bytes, const RowChunk* chunks, int n_chunks,
                                  const GemmFuse* fuse, int packed, const DecodeSync* sync, int r_stride,
                                  hipStream_t stream) {
  const int n_ext = fuse ? fuse->n_ext : 0;
  if (!gemm_multi_ok(form, T, Kc, proj_host, n_proj, n_ext, fuse ? fuse->ranks_mult8 : true,
                     partials ? partial_bytes : 0) || chunks == nullptr || n_proj > MAX_PROJ)
    return hipErrorInvalidValue;
  const int64_t tiles = multi_tiles(proj_host, n_proj);
  const GemmPlan p = gemm_plan(T, Kc, tiles * SK_BN, n_ext, true);
  GemmArgs a;
  a.Aop = Aop; a.lda = lda; a.Bop = (const bf16_t*)proj_host[0].W; a.ldb = proj_host[0].ldw;
  a.T = T; a.Kc = Kc; a.Nout = proj_host[0].Nout;
  a.perm = perm; a.seg_off = seg_off; a.n_adapters = n_adapters; a.table = table; a.which = 1;
  a.U = nullptr; a.r_stride = 0; a.out = proj_host[0].out; a.ldo = proj_host[0].ldo;
  a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n; a.ksplit = p.ksplit; a.kchunk = p.kchunk;
  a.partials = partials; a.ldp = p.ldp; a.pm = p.pm; a.chunks = chunks; a.n_chunks = n_chunks;
  a.ext_cols = nullptr; a.ext_roff = nullptr; a.n_ext = 0; a.u_part = nullptr; a.ldu = 0; a.u_out = nullptr;
  a.ext_t0 = 0; a.ext_base = 0;
  if (fuse) {
    a.ext_cols = fuse->cols; a.ext_roff = fuse->roff; a.n_ext = n_ext;
    a.ext_t0 = fuse->t0; a.ext_base = fuse->ext_base;
    a.u_part = partials + p.bytes / sizeof(float); a.ldu = p.ldu;
  }
  memset(a.proj, 0, sizeof a.proj);
  for (int q = 0; q < n_proj; ++q) a.proj[q] = proj_host[q];
  a.n_proj = n_proj;
  int fin_cols = 0;
  for (int q = 0; q < n_proj; ++q) fin_cols += (int)((proj_host[q].Nout + FIN_COLS - 1) / FIN_COLS);
  a.fin_cols = fin_cols;
  // (packed: every ProjEntry::W is a packed copy and ProjEntry::ldw its k-steps per column block)
  const bool pk = packed != 0 && (fuse == nullptr || form == FORM_NT);
  if (packed != 0 && !pk) return hipErrorInvalidValue;
  a.fin_in_kernel = 0; a.out_is_f32 = out_is_f32; a.lform = form; a.spin_limit = 0;
  a.sync = nullptr; a.grp_ids = nullptr;
  a.U2 = nullptr; a.lora_tiles = nullptr; a.zero_line = nullptr; a.lora_dma = 0;
  if (pk) a.fin_in_kernel = decode_finish_mode(sync, n_adapters, r_stride, p.tiles_m, p.tiles_n, p.ksplit);
  if (a.fin_in_kernel) {
    a.sync = sync->counters; a.grp_ids = sync->grp_ids; a.spin_limit = sync->spin_limit;
    a.r_stride = r_stride;
  }
  if (form == FORM_NT)
    return out_is_f32 ? launch_one<FORM_NT, true>(a, 2, pk, stream) : launch_one<FORM_NT, false>(a, 2, pk, stream);
  return out_is_f32 ? launch_one<FORM_NN, true>(a, 2, pk, stream) : launch_one<FORM_NN, false>(a, 2, pk, stream);
}

}  // namespace marlaas
