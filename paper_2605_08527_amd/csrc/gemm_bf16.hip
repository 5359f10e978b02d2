// Base GEMM on the bf16 matrix cores with the LoRA expand fused in as extra
// contraction steps:
//
//   out[tok(m), :] = Aop[tok(m), :] * Bop  +  [u_hi(m) | u_lo(m)] * [L_t ; L_t]
//
// m runs over tokens grouped by adapter (tok = perm), Bop is the shared frozen
// base weight (paper Sec. 1 principle (1)), u = s_t * (x A_t) comes from the
// shrink kernel in fp32 and is split here into two bf16 terms, and L_t is the
// adapter's output-side factor (B_t in forward, A_t in backward).  Rows of a
// tile that belong to another adapter are fed zeros for the extra steps, so a
// tile may straddle any number of segments.
//
// Tile: 256 x 256 per workgroup of 4 waves (2 x 2), each wave 128 x 128 as
// 4 x 4 MFMA 32x32x16 accumulators (a large wave tile keeps LDS read traffic,
// which competes with the DMA writes for LDS bandwidth, under the MFMA rate).
// The contraction runs in k-tiles of 64 that go from global memory straight
// into LDS (16 bytes per lane, no register staging; every row segment is one
// whole 128-byte line, which halves the L2 requests of a 32-wide tile) through
// two 64 KB slots.  The parts of a k-tile are requested while the previous one
// is multiplied, at least two MFMA phases before they are needed; the single
// barrier per k-tile sits before the last phase, so the first fragment reads of
// the next tile overlap MFMAs.  16-byte units are XOR-swizzled so that DMA
// writes and fragment reads are bank-conflict free.
#include "common.h"

namespace marlaas {

static constexpr int BM = 256, BN = 256, BK = 64;
static constexpr int WAVES_M = 2, WAVES_N = 2;             // wave grid inside the tile
static constexpr int NWAVES = WAVES_M * WAVES_N;
static constexpr int GEMM_THREADS = 64 * NWAVES;
static constexpr int MT = BM / WAVES_M / 32, NT = BN / WAVES_N / 32;   // 32x32 MFMA tiles per wave
static constexpr int DPW = 32 / NWAVES;                    // DMA instructions per wave, operand and k-tile
static constexpr int LROWS = GEMM_THREADS / 8;             // rows per pass of the register-staged loaders
static constexpr int LPASS = BM / LROWS;
static constexpr int LKROWS = GEMM_THREADS / 32;           // k-rows per pass (k-n tiles)
static constexpr int LKPASS = BK / LKROWS;
static constexpr int STAGE_BYTES = BM * BK * 2;            // 32 KB: one operand tile
static constexpr int SLOT_BYTES = 2 * STAGE_BYTES;         // 64 KB: A part then B part
static constexpr int SLOT_B_OFF = STAGE_BYTES;
static constexpr int RING_SLOTS = 2;
static constexpr int GEMM_LDS = RING_SLOTS * SLOT_BYTES + BM * 4;  // ring + token ids

struct GemmArgs {
  const bf16_t* Aop; int64_t lda;
  const bf16_t* Bop; int64_t ldb;
  int64_t T, Kc, Nout;
  const int32_t* perm;
  const int32_t* seg_off;
  int n_adapters;
  const AdapterEntry* table;
  int which;               // 0: L_t = entry.A, 1: L_t = entry.B
  const float* U; int r_stride;
  void* out; int64_t ldo;
  int tiles_m, tiles_n;
  // split-K (few row tiles, e.g. decode): workgroup (tile, ks) handles contraction values
  // [ks * kchunk, (ks + 1) * kchunk) and leaves its fp32 sums in `partials`
  // ([ks][tiles_m * 256][tiles_n * 256], grouped row order); splitk_finish_kernel adds them up.
  int ksplit; int64_t kchunk; float* partials;
};

#ifndef EXP_NODMA
#define EXP_NODMA 0
#endif
#ifndef EXP_NOADV
#define EXP_NOADV 0
#endif
#ifdef EXP_TIMING
__device__ unsigned long long g_tim[8];
#define TSTAMP(i) do { if (tid == 0) { const long long _t = clock64(); atomicAdd(&g_tim[i], (unsigned long long)(_t - t_prev)); t_prev = _t; } } while (0)
#define TWAIT_BEGIN() long long _tw0 = 0, _tw1 = 0; do { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); _tw0 = clock64(); } while (0)
#define TWAIT_MID() do { _tw1 = clock64(); } while (0)
#define TWAIT_END() do { const long long _tw2 = clock64(); tw_vm += _tw1 - _tw0; tw_bar += _tw2 - _tw1; } while (0)
#else
#define TSTAMP(i) do {} while (0)
#define TWAIT_BEGIN() do {} while (0)
#define TWAIT_MID() do {} while (0)
#define TWAIT_END() do {} while (0)
#endif
typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// LDS byte offset of 16-byte unit `unit` of row `row` in a [rows][64] bf16 tile.
__device__ __forceinline__ int swz_rowk(int row, int unit) {
  return row * 128 + ((unit ^ ((row >> 1) & 7)) << 4);
}
// LDS byte offset of 16-byte unit `unit` (of 32) of k-row `k` in a [64][256] bf16 tile.
__device__ __forceinline__ int swz_kn(int k, int unit) {
  return k * 512 + ((unit ^ ((k & 3) << 2)) << 4);
}

// 8 consecutive contraction values of one column from a [k][n] tile: two
// transposing 64-bit reads (each returns 4 consecutive k for this lane's column).
__device__ __forceinline__ bf16x8 lds_read_frag_tr(const char* p0, const char* p1) {
  typedef short4v __attribute__((address_space(3))) * lds_s4;
  short4v a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)p0);
  short4v b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)p1);
  union { short s[8]; bf16x8 v; } r;
  r.s[0] = a[0]; r.s[1] = a[1]; r.s[2] = a[2]; r.s[3] = a[3];
  r.s[4] = b[0]; r.s[5] = b[1]; r.s[6] = b[2]; r.s[7] = b[3];
  return r.v;
}

__device__ __forceinline__ uint4 pack8(const bf16_t* o) {
  uint4 pk;
  pk.x = o[0] | ((uint32_t)o[1] << 16); pk.y = o[2] | ((uint32_t)o[3] << 16);
  pk.z = o[4] | ((uint32_t)o[5] << 16); pk.w = o[6] | ((uint32_t)o[7] << 16);
  return pk;
}

// One 16-wide contraction step of the wave's block from a 64-wide LDS tile pair (as, bs).
template <int FORM>
__device__ __forceinline__ void mma_kstep(const char* as, const char* bs, int ks, int a_off_row,
                                          int a_swz, int fk, int b_off_row, int b_swz,
                                          const int (&btr)[NT], f32x16 (&acc)[MT][NT]) {
  bf16x8 af[MT], bfr[NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
    af[mt] = *(const bf16x8*)(as + a_off_row + mt * (32 * 128) + (((ks * 2 + fk) ^ a_swz) << 4));
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    if (FORM == FORM_NT) {
      bfr[nt] = *(const bf16x8*)(bs + b_off_row + nt * (32 * 128) + (((ks * 2 + fk) ^ b_swz) << 4));
    } else {
      // btr[nt]: byte offset of this lane's (k = kb, column) element for ks = 0; a k-step moves
      // 16 rows down (the swizzle only depends on k & 3, unchanged by steps of 4)
      const char* p = bs + btr[nt] + ks * (16 * 512);
      bfr[nt] = lds_read_frag_tr(p, p + 4 * 512);
    }
  }
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
      acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mt], bfr[nt], acc[mt][nt], 0, 0, 0);
}

template <int FORM, bool OUT_F32>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_bf16_kernel(GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  int32_t* tok_s = (int32_t*)(smem + RING_SLOTS * SLOT_BYTES);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: LDS DMA targets stay scalar
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
#ifdef EXP_TIMING
  long long t_prev = clock64();
  long long tw_vm = 0, tw_bar = 0;
#endif

  // ---- block -> tile: each XCD (blocks b = x mod 8) walks a compact run of
  // tiles; inside a run, groups of 8 row tiles share their column tiles.
  int tm, tn, ks_idx, tile_lin;
  {
    const int G = a.tiles_m * a.tiles_n * a.ksplit;
    const int b = blockIdx.x;
    const int xcd = b & 7, idx = b >> 3;
    const int q = G >> 3, rem = G & 7;
    const int start = xcd * q + (xcd < rem ? xcd : rem);
    const int bbs = start + idx;
    const int bb = bbs / a.ksplit;          // the splits of one tile stay on one XCD (one L2)
    ks_idx = bbs - bb * a.ksplit;
    tile_lin = bb;
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
  __syncthreads();

  const int64_t kbeg = (int64_t)ks_idx * a.kchunk;
  const int64_t kend = (kbeg + a.kchunk) < a.Kc ? (kbeg + a.kchunk) : a.Kc;

  // ---- DMA geometry.  One wave instruction moves 64 x 16 B = 1 KB into consecutive LDS
  // bytes.  Row-k tiles ([256][64] bf16, 128 B per row): 8 rows per instruction, lane l writes
  // unit (l & 7) of row (l >> 3) and so fetches the global unit (l & 7) ^ swizzle(row); every
  // row segment is one whole 128-byte cache line.  k-n tiles ([64][256], 512 B per row): 2
  // k-rows per instruction.  Each wave issues DPW = 8 instructions per operand per k-tile.
  const bf16_t* a_src[DPW];
  const bf16_t* b_src[DPW];
  int64_t b_step;          // elements to advance b_src per k-tile
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
      b_src[j] = a.Bop + n * a.ldb + kbeg + unit * 8;
    }
    b_step = BK;
  } else {
#pragma unroll
    for (int j = 0; j < DPW; ++j) {
      const int k = (wave * DPW + j) * 2 + (lane >> 5);
      const int unit = (lane & 31) ^ ((k & 3) << 2);
      int64_t n = n0 + unit * 8;
      if (n >= a.Nout) n = a.Nout - 8;
      b_src[j] = a.Bop + (kbeg + k) * a.ldb + n;
    }
    b_step = (int64_t)BK * a.ldb;
  }
  const int dma_off = wave * DPW * 1024;   // this wave's first KB inside an operand part of a slot

  // ---- fragment geometry (all tiles are 64 wide)
  const int frow = lane & 31;          // row inside a 32-row MFMA tile
  const int fk = lane >> 5;            // which 8-wide half of the 16-wide k step
  const int a_row = wm * (MT * 32) + frow;
  const int b_row = wn * (NT * 32) + frow;
  const int a_off_row = a_row * 128;
  const int a_swz = (a_row >> 1) & 7;  // rows 32 apart share the swizzle
  const int b_off_row = b_row * 128;
  const int b_swz = (b_row >> 1) & 7;
  int btr[NT];
  {
    const int g16 = lane >> 4, i16 = lane & 15;
    const int kb = (g16 >> 1) * 8 + (i16 >> 2);
    for (int nt = 0; nt < NT; ++nt) {
      const int ncol = wn * (NT * 32) + nt * 32 + (g16 & 1) * 16 + 4 * (i16 & 3);
      btr[nt] = swz_kn(kb, ncol >> 3) + (ncol & 7) * 2;
    }
  }

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int64_t ntile = (kend - kbeg) / BK;

  static_assert(MT == 4 && NT == 4 && DPW == 8, "the interleaved schedule below is written for 4 x 4 MFMA tiles per wave");

// s_waitcnt immediate that waits only for the vector-memory counter (6 bits, split 3:0 / 15:14)
#define VMCNT(n) (0x0F70 | ((n) & 15) | ((((n) >> 4) & 3) << 14))
// raw barrier: LDS traffic of this wave is complete, DMA traffic is tracked by hand with vmcnt
#ifndef EXP_NOBAR
#define EXP_NOBAR 0
#endif
#if EXP_NOBAR
#define RING_BARRIER() asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory")
#else
#define RING_BARRIER() asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory")
#endif

// one DMA instruction: part j (0..7) of operand `isb_` (0 = A, 1 = B) of the k-tile going to `slot_`
#define RING_DMA1(slot_, isb_, j_)                                                                        \
  do {                                                                                                    \
    char* _sb = smem + (slot_) * SLOT_BYTES + dma_off + (j_) * 1024;                                      \
    if (isb_) {                                                                                           \
      if (!EXP_NODMA) __builtin_amdgcn_global_load_lds((gptr_t)b_src[j_], (lptr_t)(_sb + SLOT_B_OFF), 16, 0, 0); \
      if (!EXP_NOADV) b_src[j_] += b_step;                                                                \
    } else {                                                                                              \
      if (!EXP_NODMA) __builtin_amdgcn_global_load_lds((gptr_t)a_src[j_], (lptr_t)(_sb), 16, 0, 0);       \
      if (!EXP_NOADV) a_src[j_] += BK;                                                                    \
    }                                                                                                     \
  } while (0)

#define RING_DMA(slot_, isb_)                                                                             \
  do {                                                                                                    \
    _Pragma("unroll") for (int _j = 0; _j < DPW; ++_j) RING_DMA1(slot_, isb_, _j);                        \
  } while (0)

// fragment i (0..3 = A rows, 4..7 = B columns) of k-step ks_ of the k-tile in `slot_`
#define RING_READ1(slot_, ks_, i_, af_, bf_)                                                              \
  do {                                                                                                    \
    const char* _as = smem + (slot_) * SLOT_BYTES;                                                        \
    const char* _bs = _as + SLOT_B_OFF;                                                                   \
    if ((i_) < 4) {                                                                                       \
      af_[(i_) & 3] = *(const bf16x8*)(_as + a_off_row + ((i_) & 3) * (32 * 128) +                        \
                                       ((((ks_) * 2 + fk) ^ a_swz) << 4));                                \
    } else if (FORM == FORM_NT) {                                                                         \
      bf_[(i_) & 3] = *(const bf16x8*)(_bs + b_off_row + ((i_) & 3) * (32 * 128) +                        \
                                       ((((ks_) * 2 + fk) ^ b_swz) << 4));                                \
    } else {                                                                                              \
      const char* _p = _bs + btr[(i_) & 3] + (ks_) * (16 * 512);                                          \
      bf_[(i_) & 3] = lds_read_frag_tr(_p, _p + 4 * 512);                                                 \
    }                                                                                                     \
  } while (0)

// 16 MFMAs on (ua_, ub_) with, in their shadow, the 8 fragment reads of (ld_slot_, ld_ks_) into
// (la_, lb_) and 8 DMA instructions; sched_barrier pins this order (one wave per SIMD: nothing
// else hides the issue latency of LDS and DMA instructions).
#define RING_PHASE(ua_, ub_, do_ld_, ld_slot_, ld_ks_, la_, lb_, do_dma_, dma_slot_, dma_isb_)            \
  do {                                                                                                    \
    _Pragma("unroll") for (int _i = 0; _i < 16; ++_i) {                                                   \
      acc[_i >> 2][_i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ua_[_i >> 2], ub_[_i & 3],           \
                                                                     acc[_i >> 2][_i & 3], 0, 0, 0);      \
      if ((do_ld_) && _i < 8) RING_READ1(ld_slot_, ld_ks_, _i, la_, lb_);                                 \
      if ((do_dma_) && _i >= 8) RING_DMA1(dma_slot_, dma_isb_, _i - 8);                                   \
      __builtin_amdgcn_sched_barrier(0);                                                                  \
    }                                                                                                     \
  } while (0)

// One k-tile kt (slot kt & 1), four phases of 16 MFMAs.  Phase 0 also requests the B part of
// tile kt + 1 (its A part was requested one tile earlier).  Before phase 3 every wave waits for
// its own DMA (all of tile kt + 1) and meets the others: tile kt + 1 is then complete, and no
// wave still reads tile kt from LDS (its last fragments are in registers), so phase 3 reads the
// first fragments of tile kt + 1 and requests the A part of tile kt + 2 into the slot of tile kt.
#define RING_TILE(kt_, dma_b_, dma_a_, has_next_)                                                         \
  do {                                                                                                    \
    const int _slot = (int)((kt_) & 1), _nslot = _slot ^ 1;                                               \
    RING_PHASE(fa0, fb0, 1, _slot, 1, fa1, fb1, dma_b_, _nslot, 1);                                       \
    RING_PHASE(fa1, fb1, 1, _slot, 2, fa0, fb0, 0, 0, 0);                                                 \
    RING_PHASE(fa0, fb0, 1, _slot, 3, fa1, fb1, 0, 0, 0);                                                 \
    if (has_next_) {                                                                                      \
      TWAIT_BEGIN();                                                                                      \
      __builtin_amdgcn_s_waitcnt(VMCNT(0));                                                               \
      TWAIT_MID();                                                                                        \
      RING_BARRIER();                                                                                     \
      TWAIT_END();                                                                                        \
    }                                                                                                     \
    RING_PHASE(fa1, fb1, has_next_, _nslot, 0, fa0, fb0, dma_a_, _slot, 0);                               \
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
  if (a.ksplit == 1 && a.n_adapters > 0 && a.U != nullptr) {
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
            if (FORM == FORM_NT) {
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
            if (FORM == FORM_NT) {
#pragma unroll
              for (int i = 0; i < LPASS; ++i) *(uint4*)(Lb + swz_rowk(lr + LROWS * i, lc)) = lw[i];
            } else {
#pragma unroll
              for (int i = 0; i < LKPASS; ++i) *(uint4*)(Lb + swz_kn(nkr + LKROWS * i, ncu)) = lw[i];
            }
            __syncthreads();
            const int left = kext - kc;
            const int ksteps = left >= BK ? 4 : left / 16;
            for (int ks = 0; ks < ksteps; ++ks)
              mma_kstep<FORM>(La, Lb, ks, a_off_row, a_swz, fk, b_off_row, b_swz, btr, acc);
            __syncthreads();
          }
        }
        ++t;
      }
    }
  }

  // ---- main loop over full k-tiles
  if (ntile > 0) {
    bf16x8 fa0[MT], fb0[NT], fa1[MT], fb1[NT];
    if (ntile > 1) {
      RING_DMA(1, 0);
      __builtin_amdgcn_s_waitcnt(VMCNT(DPW));     // tile 0 landed, the A part of tile 1 in flight
    } else {
      __builtin_amdgcn_s_waitcnt(VMCNT(0));
    }
    RING_BARRIER();
    TSTAMP(0);
#pragma unroll
    for (int i = 0; i < 8; ++i) RING_READ1(0, 0, i, fa0, fb0);
    int64_t kt = 0;
    for (; kt + 2 < ntile; ++kt) RING_TILE(kt, 1, 1, 1);
    if (kt + 1 < ntile) { RING_TILE(kt, 1, 0, 1); ++kt; }
    RING_TILE(kt, 0, 0, 0);
  }
  TSTAMP(1);
#ifdef EXP_TIMING
  if (tid == 0) { atomicAdd(&g_tim[4], (unsigned long long)tw_vm); atomicAdd(&g_tim[5], (unsigned long long)tw_bar); }
#endif
  __syncthreads();   // all reads of the last k-tile are done; slot 0 is reused below
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
    const int ksteps = (int)((kend - k0 + 15) / 16);
    for (int ks = 0; ks < ksteps; ++ks)
      mma_kstep<FORM>(As, Bs, ks, a_off_row, a_swz, fk, b_off_row, b_swz, btr, acc);
    __syncthreads();
  }

  if (a.ksplit > 1) {
    // partial sums as plain fp32 rows: [ks][tiles_m * 256][tiles_n * 256]
    const int64_t ldp = (int64_t)a.tiles_n * BN;
    float* part = a.partials + ((int64_t)ks_idx * a.tiles_m * BM + m0) * ldp + n0;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = wm * (MT * 32) + mt * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          part[(int64_t)row * ldp + wn * (NT * 32) + nt * 32 + (lane & 31)] = acc[mt][nt][v];
      }
    return;
  }

#ifdef EXP_NOEPI
  {  // timing experiment only: one store per lane keeps the accumulators alive
    float sum = 0.f;
    for (int mt = 0; mt < MT; ++mt) for (int nt = 0; nt < NT; ++nt) for (int v = 0; v < 16; ++v) sum += acc[mt][nt][v];
    const int32_t tok = tok_s[lane];
    if (tok >= 0) ((bf16_t*)a.out)[(int64_t)tok * a.ldo + n0 + wave] = float_to_bf16_bits(sum);
    return;
  }
#endif
  TSTAMP(2);
#ifdef EXP_OLDEPI
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = wm * (MT * 32) + mt * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      const int32_t tok = tok_s[row];
      if (tok < 0) continue;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const int64_t col = n0 + wn * (NT * 32) + nt * 32 + (lane & 31);
        if (col < a.Nout) {
          if (OUT_F32) ((float*)a.out)[(int64_t)tok * a.ldo + col] = acc[mt][nt][v];
          else ((bf16_t*)a.out)[(int64_t)tok * a.ldo + col] = float_to_bf16_bits(acc[mt][nt][v]);
        }
      }
    }
  }
  return;
#endif
  // ---- epilogue: each wave turns its accumulators (one column per lane) into rows through a
  // private LDS strip, 32 rows at a time, so that every lane stores 16 contiguous bytes and a
  // row segment of the wave (128 columns) leaves as whole cache lines; rows are scattered back
  // to token order.  LDS traffic of one wave is ordered, so no workgroup barrier is needed.
  {
    constexpr int EPITCH = OUT_F32 ? (128 * 4 + 16) : (128 * 2 + 16);
    constexpr int ECHUNKS = OUT_F32 ? 32 : 16;          // 16-byte chunks per row segment
    constexpr int EITERS = 32 * ECHUNKS / 64;
    char* ep = smem + wave * (32 * (128 * 4 + 16));
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row_l = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
          const int col_l = nt * 32 + (lane & 31);
          if (OUT_F32) *(float*)(ep + row_l * EPITCH + col_l * 4) = acc[mt][nt][v];
          else *(bf16_t*)(ep + row_l * EPITCH + col_l * 2) = float_to_bf16_bits(acc[mt][nt][v]);
        }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int it = 0; it < EITERS; ++it) {
        const int c = it * 64 + lane;
        const int row_l = c / ECHUNKS, ch = c % ECHUNKS;
        const uint4 val = *(const uint4*)(ep + row_l * EPITCH + ch * 16);
        const int32_t tok = tok_s[wm * (MT * 32) + mt * 32 + row_l];
        const int64_t col = n0 + wn * (NT * 32) + ch * (OUT_F32 ? 4 : 8);
        if (tok >= 0 && col < a.Nout) {
          if (OUT_F32) *(uint4*)((float*)a.out + (int64_t)tok * a.ldo + col) = val;
          else *(uint4*)((bf16_t*)a.out + (int64_t)tok * a.ldo + col) = val;
        }
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
  }
  TSTAMP(3);
}

#ifdef EXP_TIMING
extern "C" int marlaas_debug_timing(unsigned long long* out8, int reset) {
  if (hipMemcpyFromSymbol(out8, HIP_SYMBOL(g_tim), sizeof(g_tim)) != hipSuccess) return -1;
  if (reset) { unsigned long long z[8] = {0}; if (hipMemcpyToSymbol(HIP_SYMBOL(g_tim), z, sizeof z) != hipSuccess) return -1; }
  return 0;
}
#endif

// Second step of the split-K path: add the partial sums in split order, add the LoRA expand in
// fp32 (u is fp32, so no two-term split is needed here) and scatter the rows.  One thread per
// 4 consecutive output columns of one grouped row.
template <int FORM, bool OUT_F32>
__global__ __launch_bounds__(256) void splitk_finish_kernel(GemmArgs a) {
  const int64_t ldp = (int64_t)a.tiles_n * BN;
  const int64_t n4 = a.Nout / 4;                    // Nout is a multiple of 8
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= a.T * n4) return;
  const int64_t m = idx / n4;
  const int64_t n = (idx - m * n4) * 4;
  const float* part = a.partials + m * ldp + n;
  const int64_t kstride = (int64_t)a.tiles_m * BM * ldp;
  float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
  int ks = 0;
  for (; ks + 4 <= a.ksplit; ks += 4) {
    const float4 p0 = *(const float4*)(part + (ks + 0) * kstride);
    const float4 p1 = *(const float4*)(part + (ks + 1) * kstride);
    const float4 p2 = *(const float4*)(part + (ks + 2) * kstride);
    const float4 p3 = *(const float4*)(part + (ks + 3) * kstride);
    sum.x = ((sum.x + p0.x) + p1.x) + p2.x + p3.x; sum.y = ((sum.y + p0.y) + p1.y) + p2.y + p3.y;
    sum.z = ((sum.z + p0.z) + p1.z) + p2.z + p3.z; sum.w = ((sum.w + p0.w) + p1.w) + p2.w + p3.w;
  }
  for (; ks < a.ksplit; ++ks) {
    const float4 p0 = *(const float4*)(part + ks * kstride);
    sum.x += p0.x; sum.y += p0.y; sum.z += p0.z; sum.w += p0.w;
  }
  float y[4] = {sum.x, sum.y, sum.z, sum.w};
  if (a.n_adapters > 0 && a.U != nullptr && m < (int64_t)a.seg_off[a.n_adapters]) {
    const int t = segment_of(a.seg_off, a.n_adapters, (int)m);
    const AdapterEntry e = a.table[t];
    const bf16_t* L = (const bf16_t*)(a.which ? e.B : e.A);
    const float* u = a.U + m * a.r_stride;
    const int r = e.rank;
    float lora[4] = {0.f, 0.f, 0.f, 0.f};
    if (FORM == FORM_NT) {               // L[n * r + q]
      if ((r & 7) == 0) {
        for (int q0 = 0; q0 < r; q0 += 8) {
          const float4 u0 = *(const float4*)(u + q0), u1 = *(const float4*)(u + q0 + 4);
          const float uu[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const uint4 w = *(const uint4*)(L + (n + j) * r + q0);
            const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int i = 0; i < 8; ++i)
              lora[j] = fmaf(uu[i], __uint_as_float((ww[i >> 1] >> ((i & 1) * 16)) << 16), lora[j]);
          }
        }
      } else {
        for (int q = 0; q < r; ++q)
          for (int j = 0; j < 4; ++j) lora[j] = fmaf(u[q], bf16_bits_to_float(L[(n + j) * r + q]), lora[j]);
      }
    } else {                             // L[q * Nout + n]
      for (int q = 0; q < r; ++q) {
        const uint2 w = *(const uint2*)(L + (int64_t)q * a.Nout + n);
        const float uq = u[q];
        lora[0] = fmaf(uq, __uint_as_float(w.x << 16), lora[0]);
        lora[1] = fmaf(uq, __uint_as_float(w.x & 0xffff0000u), lora[1]);
        lora[2] = fmaf(uq, __uint_as_float(w.y << 16), lora[2]);
        lora[3] = fmaf(uq, __uint_as_float(w.y & 0xffff0000u), lora[3]);
      }
    }
    for (int j = 0; j < 4; ++j) y[j] += lora[j];
  }
  const int64_t tok = a.perm ? a.perm[m] : m;
  if (OUT_F32) {
    *(float4*)((float*)a.out + tok * a.ldo + n) = make_float4(y[0], y[1], y[2], y[3]);
  } else {
    uint2 o;
    o.x = float_to_bf16_bits(y[0]) | ((uint32_t)float_to_bf16_bits(y[1]) << 16);
    o.y = float_to_bf16_bits(y[2]) | ((uint32_t)float_to_bf16_bits(y[3]) << 16);
    *(uint2*)((bf16_t*)a.out + tok * a.ldo + n) = o;
  }
}

template <int FORM, bool OUT_F32>
static hipError_t launch_one(const GemmArgs& a, hipStream_t stream) {
  static bool attr_set = false;
  auto kern = gemm_bf16_kernel<FORM, OUT_F32>;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, GEMM_LDS);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int G = a.tiles_m * a.tiles_n;
  hipLaunchKernelGGL(kern, dim3(G * a.ksplit), dim3(GEMM_THREADS), GEMM_LDS, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || a.ksplit == 1) return e;
  const int64_t work = a.T * (a.Nout / 4);
  hipLaunchKernelGGL((splitk_finish_kernel<FORM, OUT_F32>), dim3((unsigned)((work + 255) / 256)), dim3(256), 0, stream, a);
  return hipGetLastError();
}

size_t gemm_splitk_bytes(int64_t T, int64_t Kc, int64_t Nout) {
  int ksplit; int64_t kchunk;
  gemm_splitk_plan(T, Kc, Nout, &ksplit, &kchunk);
  if (ksplit <= 1) return 0;
  const int64_t G = ((T + BM - 1) / BM) * ((Nout + BN - 1) / BN);
  return (size_t)G * ksplit * BM * BN * sizeof(float);
}

// Split the contraction when the tiles alone cannot fill the 256 compute units.
void gemm_splitk_plan(int64_t T, int64_t Kc, int64_t Nout, int* ksplit, int64_t* kchunk) {
  const int64_t G = ((T + BM - 1) / BM) * ((Nout + BN - 1) / BN);
  int s = 1;
  if (G > 0 && G <= 128) {
    s = (int)(256 / G);
    const int64_t max_s = Kc / 128 > 0 ? Kc / 128 : 1;      // at least 128 contraction values per split
    if (s > max_s) s = (int)max_s;
    if (s > 32) s = 32;
    if (s < 1) s = 1;
  }
  int64_t kc = (Kc + s - 1) / s;
  kc = (kc + BK - 1) / BK * BK;
  *kchunk = kc;
  *ksplit = (int)((Kc + kc - 1) / kc);
}

hipError_t launch_gemm_bf16(const bf16_t* Aop, int64_t lda, const bf16_t* Bop, int64_t ldb,
                            int form, int64_t T, int64_t Kc, int64_t Nout, const int32_t* perm,
                            const int32_t* seg_off, int n_adapters, const AdapterEntry* table,
                            int which, const float* U, int r_stride, void* out, int64_t ldo,
                            int out_is_f32, float* partials, size_t partial_bytes, hipStream_t stream) {
  if (T <= 0 || Nout <= 0) return hipSuccess;
  GemmArgs a;
  a.Aop = Aop; a.lda = lda; a.Bop = Bop; a.ldb = ldb; a.T = T; a.Kc = Kc; a.Nout = Nout;
  a.perm = perm; a.seg_off = seg_off; a.n_adapters = n_adapters; a.table = table; a.which = which;
  a.U = U; a.r_stride = r_stride; a.out = out; a.ldo = ldo;
  a.tiles_m = (int)((T + BM - 1) / BM);
  a.tiles_n = (int)((Nout + BN - 1) / BN);
  gemm_splitk_plan(T, Kc, Nout, &a.ksplit, &a.kchunk);
  a.partials = partials;
  if (a.ksplit > 1 && (partials == nullptr || partial_bytes < gemm_splitk_bytes(T, Kc, Nout))) {
    a.ksplit = 1; a.kchunk = Kc;    // no scratch for partial sums: one workgroup per tile
  }
  if (form == FORM_NT) return out_is_f32 ? launch_one<FORM_NT, true>(a, stream) : launch_one<FORM_NT, false>(a, stream);
  return out_is_f32 ? launch_one<FORM_NN, true>(a, stream) : launch_one<FORM_NN, false>(a, stream);
}

}  // namespace marlaas
