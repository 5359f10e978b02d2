// Decode-shaped base product (few hundred rows against the whole weight) on a packed copy of the
// frozen weight, with the shrink carried along as extended columns:
//
//   partial[ks][m, n]  = sum over the k-chunk of split ks of  x[tok(m), k] * W(k, n)
//   u_part [ks][m, e]  = the same with the stacked shrink factors of all adapters in place of W
//
// (rollout decode is the phase that dominates the paper's run time, Sec. 1 and Sec. 3; the weight is
// read once and is the dominant traffic).  Same 128 x 128 tiles, same contraction splits, same
// partial-sum layout as gemm_skinny_kernel, so splitk_finish_kernel completes either.
//
// What differs from gemm_skinny_kernel is who moves what.  That kernel stages both operands in LDS.
// Here a weight fragment goes from global memory straight into the registers of the one wave that
// multiplies it, and no other wave needs those values.  Read from a row-major weight, such a
// fragment is 64 separate 16-byte pieces (the 16 lanes next to each other hold 16 different rows),
// and the vector cache then spends one tag lookup per lane: measured, 1680 lookups per k-tile and
// compute unit, which is the whole time of the loop.  The base weight is frozen (paper Sec. 1
// principle (1)), so it is packed once, by pack_weight_kernel, in fragment order:
//
//   packed[nb][ks][lane][8]:  element e of lane (lg = lane / 16, li = lane % 16) is
//                             W(k = 32 ks + 8 lg + e, n = 16 nb + li), zero beyond the matrix
//
// and a fragment is one contiguous kilobyte.  Only x (which every wave of the workgroup needs) and
// the 32 extended columns go through LDS, by DMA, in a ring of four k-tiles.  Eight waves: waves
// 0-3 take the first 32-deep k-step of every 64-deep k-tile, waves 4-7 the second, each for all
// 128 rows x 32 columns; the two halves are added through LDS once, at the end.  Two waves per
// SIMD, one from each half, so one wave's LDS and memory latency is covered by the other's MFMAs.
#include "gemm_args.h"

#include <atomic>

namespace marlaas {

static constexpr int DK = 64;                          // k-tile
static constexpr int D_THREADS = 512;
static constexpr int D_X_BYTES = SK_BM * DK * 2;       // 16 KB: [128 rows][64 k], 16-byte units XOR-swizzled
static constexpr int D_E_BYTES = SK_BX * DK * 2;       // 4 KB: [32 extended columns][64 k]
static constexpr int D_NS = 4;                         // ring depth = k-tiles requested ahead
static constexpr int D_E_BASE = D_NS * D_X_BYTES;      // the ring's x parts first, then its extended-column parts
static constexpr int D_RED_BYTES = 8 * 8 * 64 * 16 + 4 * 4 * 64 * 16;   // exchange of the two k-halves: 64 KB + 16 KB
static constexpr int D_RING_BYTES = D_NS * (D_X_BYTES + D_E_BYTES) > D_RED_BYTES ? D_NS * (D_X_BYTES + D_E_BYTES) : D_RED_BYTES;
static constexpr int D_LDS = D_RING_BYTES + SK_BM * 4;

// Tuning aid, compiled in only with -DMARLAAS_DECODE_STAMPS: wave 0 of every workgroup records the
// constant-rate clock at a few points of the kernel; marlaas_debug_decode_stamps copies the record out.
#ifdef MARLAAS_DECODE_STAMPS
__device__ unsigned long long d_stamps[1024][8];
#define D_STAMP(i_) do { if (tid == 0 && blockIdx.x < 1024) d_stamps[blockIdx.x][i_] = wall_clock64(); } while (0)
extern "C" int marlaas_debug_decode_stamps(unsigned long long* host) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(d_stamps), sizeof(d_stamps));
}
#else
#define D_STAMP(i_) do { } while (0)
#endif

// Waits on the vector-memory counter.  The weight fragments and the token indices are loaded by
// inline assembly, invisible to the compiler's own wait insertion (which, across the loop's
// branches, would wait for every outstanding request before the first MFMA), so every wait on them
// is written here: requests complete in order, and "at most n outstanding" means everything but
// the n youngest has arrived.
template <int N>
__device__ __forceinline__ void wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }
// n known at run time (wave-uniform); above 15 it waits as for 15, which is more than asked
__device__ __forceinline__ void wait_vm_dyn(int n) {
  switch (n) {
    case 0: wait_vm<0>(); break;
    case 1: wait_vm<1>(); break;
    case 2: wait_vm<2>(); break;
    case 3: wait_vm<3>(); break;
    case 4: wait_vm<4>(); break;
    case 5: wait_vm<5>(); break;
    case 6: wait_vm<6>(); break;
    case 7: wait_vm<7>(); break;
    case 8: wait_vm<8>(); break;
    case 9: wait_vm<9>(); break;
    case 10: wait_vm<10>(); break;
    case 11: wait_vm<11>(); break;
    case 12: wait_vm<12>(); break;
    case 13: wait_vm<13>(); break;
    case 14: wait_vm<14>(); break;
    default: wait_vm<15>(); break;
  }
}

template <bool EXT>
__global__ __launch_bounds__(D_THREADS) void gemm_decode_kernel(GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  int32_t* tok_s = (int32_t*)(smem + D_RING_BYTES);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = wave >> 2, wn = wave & 3;        // k-step of the wave, its 32-column group
  const int li = lane & 15, lg = lane >> 4;      // MFMA operand: row / column li, k values 8 lg .. + 7
  int tm, tn, ks_idx;
  {
    // Workgroup b runs on XCD b mod 8, and every XCD has its own L2.  Where the sizes allow it, an
    // XCD works on ONE contraction split (and on every 8 / ksplit-th column tile): it then pulls
    // only its own K-range of x (and of the shrink factors) through the fabric, instead of all of
    // x once per XCD.  The row tiles of a column tile stay neighbours on one XCD and share the
    // weight tile through its L2.  Otherwise: a compact run of (column tile, split, row tile).
    const int G = a.tiles_m * a.tiles_n * a.ksplit;
    const int b = blockIdx.x;
    const int xcd = b & 7, idx = b >> 3;
    const int ng = 8 / a.ksplit;                 // XCDs that share a split
    if (a.ksplit <= 8 && ng * a.ksplit == 8 && a.tiles_n % ng == 0) {
      ks_idx = xcd % a.ksplit;
      tm = idx % a.tiles_m;
      tn = (idx / a.tiles_m) * ng + xcd / a.ksplit;
    } else {
      const int q = G >> 3, rem = G & 7;
      const int bbs = xcd * q + (xcd < rem ? xcd : rem) + idx;
      tm = bbs % a.tiles_m;
      const int rest = bbs / a.tiles_m;
      ks_idx = rest % a.ksplit;
      tn = rest / a.ksplit;
    }
  }
  const int64_t m0 = (int64_t)tm * SK_BM;
  const int64_t pn0 = (int64_t)tn * SK_BN;       // column of this tile in the partial sums
  const bf16_t* Bop = a.Bop;                     // packed weight; ldb = its k-steps per column block
  int64_t ldb = a.ldb, Nout = a.Nout, n0 = pn0;
  if (a.n_proj > 1) {                            // the projection this column tile belongs to (wave-uniform)
    int p = 0;
    for (int q = 1; q < a.n_proj; ++q) if (tn >= a.proj[q].tile0) p = q;
    Bop = (const bf16_t*)a.proj[p].W; ldb = a.proj[p].ldw; Nout = a.proj[p].Nout;
    n0 = (int64_t)(tn - a.proj[p].tile0) * SK_BN;
  }
  const int64_t kbeg = (int64_t)ks_idx * a.kchunk;
  const int64_t kend = (kbeg + a.kchunk) < a.Kc ? (kbeg + a.kchunk) : a.Kc;
  const int ntile = (int)((kend - kbeg) / DK);
  D_STAMP(0);

  // ---- the loads everything else waits for go first: the token indices of the x rows this lane
  // requests by DMA (rows past the end repeat the last row: their results are never used) and the
  // source row of its share of the extended columns.  (index, pointer and rank index: 3 requests)
  int32_t tok_r[2] = {0, 0};
  int arow[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    arow[j] = (wave * 2 + j) * 8 + (lane >> 3);
    int64_t m = m0 + arow[j];
    if (m >= a.T) m = a.T - 1;
    tok_r[j] = (int32_t)m;
    if (a.perm) asm volatile("global_load_dword %0, %1, off" : "=v"(tok_r[j]) : "v"(a.perm + m) : "memory");
  }
  const int erow = wave * 4 + ((lane & 31) >> 3);            // extended columns: 4 rows per wave (lanes 0-31)
  uint64_t e_ptr = 0;
  int32_t e_q = 0;
  if (EXT) {
    int e = tn * SK_BX + erow;
    if (e >= a.n_ext) e = a.n_ext - 1;
    const char* ce = (const char*)(a.ext_cols + e);
    asm volatile("global_load_dwordx2 %0, %1, off" : "=v"(e_ptr) : "v"(ce + (a.which ? 0 : 8)) : "memory");
    asm volatile("global_load_dword %0, %1, off" : "=v"(e_q) : "v"(ce + 20) : "memory");
  }
  const int n_first = (a.perm ? 2 : 0) + (EXT ? 2 : 0);      // requests so far

  // ---- weight fragments: straight from the packed weight, one contiguous kilobyte per wave and
  // instruction.  Column block cb of this wave is block n0 / 16 + 2 wn + cb of the packed copy
  // (blocks past the last one repeat it: those columns are never stored); its k-step for k-tile kt
  // is (kbeg + 64 kt) / 32 + g, and consecutive k-tiles are 2 KB apart.
  const bf16_t* wp[2];
  {
    const int64_t nblocks = (Nout + 15) >> 4;
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
      int64_t nb = (n0 >> 4) + wn * 2 + cb;
      if (nb >= nblocks) nb = nblocks - 1;
      wp[cb] = Bop + ((nb * ldb + (kbeg >> 5) + g) << 9) + lane * 8;
    }
  }
  bf16x8 wreg[D_NS][2];
#define D_WLOAD(t_, s_)                                                                                   \
  do {                                                                                                    \
    _Pragma("unroll") for (int cb = 0; cb < 2; ++cb)                                                      \
      asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(wreg[s_][cb]) : "v"(wp[cb] + (int64_t)(t_) * 1024) : "memory"); \
  } while (0)
  // the weight requests do not depend on the token indices: the first tiles go out at once
  int issued = 0;
#pragma unroll
  for (int s = 0; s < D_NS; ++s)
    if (s < ntile) { D_WLOAD(s, s); issued += 2; }
  wait_vm_dyn(issued);                           // the indices and the extended-column entry have arrived
  (void)n_first;
  asm volatile("" : "+v"(tok_r[0]), "+v"(tok_r[1]), "+v"(e_ptr), "+v"(e_q));
  D_STAMP(1);

  // ---- DMA sources.  x tile: 16 instructions of 1 KB (8 rows of 128 bytes), two per wave; the
  // extended columns: 32 rows of 128 bytes, half an instruction (lanes 0-31: 4 rows) per wave.
  const bf16_t* a_src[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int unit = (lane & 7) ^ ((arow[j] >> 1) & 7);
    a_src[j] = a.Aop + (int64_t)tok_r[j] * a.lda + kbeg + unit * 8;
  }
  const bf16_t* e_src = nullptr;
  if (EXT) {
    const int unit = (lane & 7) ^ ((erow >> 1) & 7);
    e_src = (const bf16_t*)e_ptr + (int64_t)e_q * a.Kc + kbeg + unit * 8;
  }
  constexpr int NV = 2 + 2 + (EXT ? 1 : 0);      // vector-memory instructions per wave per k-tile
  // One k-tile's DMA requests of this wave into ring slot s_.
#define D_DMA(t_, s_)                                                                                     \
  do {                                                                                                    \
    _Pragma("unroll") for (int j = 0; j < 2; ++j)                                                         \
      __builtin_amdgcn_global_load_lds((gptr_t)(a_src[j] + (int64_t)(t_) * DK),                           \
                                       (lptr_t)(smem + (s_) * D_X_BYTES + (wave * 2 + j) * 1024), 16, 0, 0); \
    if (EXT) {                                                                                            \
      if (lane < 32)                                                                                      \
        __builtin_amdgcn_global_load_lds((gptr_t)(e_src + (int64_t)(t_) * DK),                            \
                                         (lptr_t)(smem + D_E_BASE + (s_) * D_E_BYTES + wave * 512), 16, 0, 0); \
    }                                                                                                     \
  } while (0)

  // ---- fragment reads from LDS, k-step g; rows 16 apart share the swizzle.  Every wave walks the
  // eight 16-row blocks in its own rotation: its index i is row block (i + 2 wn) mod 8, so that
  // the two row blocks it multiplies with the extended columns are always its indices 0 and 1.
  const int f_off = li * 128;
  const int f_unit = ((g * 4 + lg) ^ ((li >> 1) & 7)) << 4;
  // The reads are inline assembly with hand-written waits: left to the compiler, every other
  // k-tile waits for fragment reads it has only just issued.
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)smem;
  int xoff[8];                                     // byte offsets in slot 0 (the k tail reads them in C)
  uint32_t xaddr[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) { xoff[i] = f_off + f_unit + ((i + 2 * wn) & 7) * 2048; xaddr[i] = lds0 + xoff[i]; }
  const int eoff = D_E_BASE + f_off + f_unit;
  const uint32_t eaddr = lds0 + eoff;
  bf16x8 xf[2][8], ef[2][2];
#define D_READ(s_, b_)                                                                                    \
  do {                                                                                                    \
    _Pragma("unroll") for (int i = 0; i < 8; ++i)                                                         \
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(xf[b_][i]) : "v"(xaddr[i]), "n"((s_) * D_X_BYTES)); \
    if (EXT) {                                                                                            \
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(ef[b_][0]) : "v"(eaddr), "n"((s_) * D_E_BYTES)); \
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(ef[b_][1]) : "v"(eaddr), "n"((s_) * D_E_BYTES + 2048)); \
    }                                                                                                     \
    __builtin_amdgcn_sched_barrier(0);                                                                    \
  } while (0)
// after a wait that covers the reads into fragment set b_: uses of the set stay below this point
#define D_PIN(b_)                                                                                         \
  do {                                                                                                    \
    asm volatile("" : "+v"(xf[b_][0]), "+v"(xf[b_][1]), "+v"(xf[b_][2]), "+v"(xf[b_][3]),                 \
                      "+v"(xf[b_][4]), "+v"(xf[b_][5]), "+v"(xf[b_][6]), "+v"(xf[b_][7]));                \
    if (EXT) asm volatile("" : "+v"(ef[b_][0]), "+v"(ef[b_][1]));                                         \
  } while (0)

  // accumulators: the weight fragment is the first MFMA operand, so in a 16 x 16 block lane l holds
  // token li and the four consecutive output columns 4 lg .. + 3
  f32x4 acc[8][2], eacc[2][2];
#pragma unroll
  for (int rb = 0; rb < 8; ++rb)
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) acc[rb][cb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int xb = 0; xb < 2; ++xb) eacc[j][xb] = f32x4{0.f, 0.f, 0.f, 0.f};
#define D_MMA(b_, s_)                                                                                     \
  do {                                                                                                    \
    _Pragma("unroll") for (int rb = 0; rb < 8; ++rb)                                                      \
      _Pragma("unroll") for (int cb = 0; cb < 2; ++cb)                                                    \
        acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wreg[s_][cb], xf[b_][rb], acc[rb][cb], 0, 0, 0); \
    if (EXT) {                                                                                            \
      /* this wave's share of the extended columns: its indices 0, 1 = row blocks 2 wn, 2 wn + 1 */       \
      _Pragma("unroll") for (int j = 0; j < 2; ++j)                                                       \
        _Pragma("unroll") for (int xb = 0; xb < 2; ++xb)                                                  \
          eacc[j][xb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ef[b_][xb], xf[b_][j], eacc[j][xb], 0, 0, 0); \
    }                                                                                                     \
  } while (0)

  // ---- main loop.  `issued` counts this wave's vector-memory instructions since the weight
  // requests above, dma_end[s] its value right after the DMA requests of the tile in slot s: the
  // tile has landed once at most issued - dma_end[s] younger instructions are outstanding.  Per
  // k-tile a wave issues its DMA requests right after the barrier and the weight fragments of the
  // same tile after the MFMAs that used the registers they replace; so when the DMA of tile kt + 1
  // has landed, so have the (older) weight fragments of tile kt.
  int dma_end[D_NS];
#pragma unroll
  for (int s = 0; s < D_NS; ++s) dma_end[s] = 0;
#pragma unroll
  for (int s = 0; s < D_NS; ++s)
    if (s < ntile) { D_DMA(s, s); issued += NV - 2; dma_end[s] = issued; }
  if (ntile > 0) {
    wait_vm_dyn(issued - dma_end[0]);
    __syncthreads();
    D_READ(0, 0);
  }
  D_STAMP(2);
  constexpr int STEADY = 2 + (D_NS - 2) * NV;    // younger requests than a tile's DMA, D_NS - 1 iterations later
  // iteration kt = kt0 + s_ works on ring slot s_ (kt0 is a multiple of the ring depth)
#define D_ITER(s_)                                                                                        \
  do {                                                                                                    \
    const int kt = kt0 + (s_);                                                                            \
    if (kt < ntile) {                                                                                     \
      constexpr int sn = ((s_) + 1) % D_NS;                                                               \
      /* this wave's part of tile kt + 1 has landed (last tile: its weight fragments have) */             \
      const int younger = kt + 1 < ntile ? issued - dma_end[sn] : 0;                                      \
      if (younger == STEADY) wait_vm<STEADY>(); else wait_vm_dyn(younger);                                \
      /* everyone's has, and nobody still reads tile kt from LDS (its fragments are in registers) */      \
      asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");                                     \
      asm volatile("" : "+v"(wreg[s_][0]), "+v"(wreg[s_][1]));   /* uses of these stay below the wait */  \
      D_PIN((s_) & 1);                                                                                    \
      if (kt + D_NS < ntile) D_DMA(kt + D_NS, s_);                                                        \
      /* fragments of tile kt + 1, in the shadow of the MFMAs below (after the last tile this reads a */  \
      /* stale slot, and those fragments are not used) */                                                \
      D_READ(sn, ((s_) + 1) & 1);                                                                         \
      D_MMA((s_) & 1, s_);                                                                                \
      if (kt + D_NS < ntile) {                                                                            \
        D_WLOAD(kt + D_NS, s_);                                                                           \
        issued += NV;                                                                                     \
        dma_end[s_] = issued - 2;                                                                         \
      }                                                                                                   \
    }                                                                                                     \
  } while (0)
  static_assert(D_NS == 4, "the loop body is written out for a ring of four");
  for (int kt0 = 0; kt0 < ntile; kt0 += D_NS) {
    D_ITER(0); D_ITER(1); D_ITER(2); D_ITER(3);
    if (kt0 == 0) D_STAMP(3);
  }
  D_STAMP(4);
#undef D_ITER
#undef D_WLOAD
#undef D_DMA
#undef D_READ
#undef D_PIN
#undef D_MMA
  // token indices of the tile's rows, for the k tail
  if (tid < SK_BM) {
    const int64_t m = m0 + tid;
    tok_s[tid] = m < a.T ? (a.perm ? a.perm[m] : (int32_t)m) : -1;
  }
  __syncthreads();     // the ring is free

  // ---- k tail (the last split when Kc is not a multiple of 64): one masked tile, staged through
  // registers into slot 0; every wave handles its own k-step, values beyond kend are zeros
  if (kbeg + (int64_t)ntile * DK < kend) {
    const int64_t k0 = kbeg + (int64_t)ntile * DK;
    const uint4 zero4 = make_uint4(0, 0, 0, 0);
    {
      const int lc = tid & 7, lr = tid >> 3;       // 64 rows per pass
      const bool ka = (k0 + lc * 8) < kend;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int row = lr + 64 * i;
        const int32_t tok = tok_s[row];
        uint4 v = zero4;
        if (ka && tok >= 0) v = *(const uint4*)(a.Aop + (int64_t)tok * a.lda + k0 + lc * 8);
        *(uint4*)(smem + swz_rowk(row, lc)) = v;
      }
      if (EXT && tid < 256) {
        const int row = tid >> 3;                  // 32 rows x 8 units
        int e = tn * SK_BX + row;
        if (e >= a.n_ext) e = a.n_ext - 1;
        const ExtCol c = a.ext_cols[e];
        uint4 w = zero4;
        if (ka) w = *(const uint4*)((const bf16_t*)(a.which ? c.A : c.B) + (int64_t)c.q * a.Kc + k0 + lc * 8);
        *(uint4*)(smem + D_E_BASE + swz_rowk(row, lc)) = w;
      }
    }
    // (the packed weight is zero beyond the matrix; a k-step that starts beyond it does not exist)
    bf16x8 wt[2];
    const bool kw = (k0 + g * 32) < kend;
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
      union { uint4 u; bf16x8 v; } w; w.u = zero4;
      if (kw) w.u = *(const uint4*)(wp[cb] + (int64_t)ntile * 1024);
      wt[cb] = w.v;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const bf16x8 xr = *(const bf16x8*)(smem + xoff[i]);
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
        acc[i][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wt[cb], xr, acc[i][cb], 0, 0, 0);
      if (EXT && i < 2) {
#pragma unroll
        for (int xb = 0; xb < 2; ++xb) {
          const bf16x8 er = *(const bf16x8*)(smem + eoff + xb * 2048);
          eacc[i][xb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(er, xr, eacc[i][xb], 0, 0, 0);
        }
      }
    }
    __syncthreads();
  }

  // ---- add the two k-halves through LDS: wave (g, wn) keeps its indices 4 g .. 4 g + 3 and hands
  // the other four to wave (1 - g, wn), which walks the row blocks in the same rotation; the
  // extended columns all go to the g = 0 wave
  {
    f32x4* red = (f32x4*)smem;
    const int partner = (1 - g) * 4 + wn;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
        red[((partner * 8) + i * 2 + cb) * 64 + lane] = g == 0 ? acc[4 + i][cb] : acc[i][cb];
    f32x4* ered = (f32x4*)(smem + 8 * 8 * 64 * 16);
    if (EXT && g == 1) {
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int xb = 0; xb < 2; ++xb) ered[((wn * 4) + j * 2 + xb) * 64 + lane] = eacc[j][xb];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int cb = 0; cb < 2; ++cb) {
        const f32x4 o = red[((wave * 8) + i * 2 + cb) * 64 + lane];
        // (k-step 0 first, then k-step 1: the same order in both halves of the tile)
        if (g == 0) { acc[i][cb][0] += o[0]; acc[i][cb][1] += o[1]; acc[i][cb][2] += o[2]; acc[i][cb][3] += o[3]; }
        else { acc[i][cb][0] = o[0] + acc[4 + i][cb][0]; acc[i][cb][1] = o[1] + acc[4 + i][cb][1];
               acc[i][cb][2] = o[2] + acc[4 + i][cb][2]; acc[i][cb][3] = o[3] + acc[4 + i][cb][3]; }
      }
    if (EXT && g == 0) {
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int xb = 0; xb < 2; ++xb) {
          const f32x4 o = ered[((wn * 4) + j * 2 + xb) * 64 + lane];
          eacc[j][xb][0] += o[0]; eacc[j][xb][1] += o[1]; eacc[j][xb][2] += o[2]; eacc[j][xb][3] += o[3];
        }
    }
  }
  D_STAMP(5);
  // acc[i][cb], i < 4, now holds row block (4 g + i + 2 wn) mod 8 (row li of it), columns
  // 32 wn + 16 cb + 4 lg .. + 3 of this split

  // ---- partial sums as plain fp32 rows: [ks][pm][ldp]
  {
    float* part = a.partials + ((int64_t)ks_idx * a.pm + m0 + li) * a.ldp + pn0 + wn * 32 + 4 * lg;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int rb = (4 * g + i + 2 * wn) & 7;
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
        *(float4*)(part + (int64_t)(rb * 16) * a.ldp + cb * 16) =
            make_float4(acc[i][cb][0], acc[i][cb][1], acc[i][cb][2], acc[i][cb][3]);
    }
  }
  if (EXT && g == 0) {
    // rows 16 (2 wn + j) + li of the tile, extended columns 16 xb + 4 lg .. + 3
    float* up = a.u_part + ((int64_t)ks_idx * a.pm + m0 + 32 * wn + li) * a.ldu + tn * SK_BX + 4 * lg;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int xb = 0; xb < 2; ++xb)
        *(float4*)(up + (int64_t)(j * 16) * a.ldu + xb * 16) =
            make_float4(eacc[j][xb][0], eacc[j][xb][1], eacc[j][xb][2], eacc[j][xb][3]);
  }
  D_STAMP(6);
}

// One 16-column x 32-deep fragment per wave: lane (lg, li) gathers its 8 values and stores 16 bytes.
// Element (c, o) of the [contraction, output] operand is at src[c * sc + o * so].
__global__ __launch_bounds__(256) void pack_weight_kernel(const bf16_t* __restrict__ src, int64_t sc, int64_t so,
                                                          int64_t C, int64_t O, int64_t ksteps, int64_t nfrag,
                                                          bf16_t* __restrict__ dst) {
  const int64_t frag = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (frag >= nfrag) return;
  const int lane = threadIdx.x & 63, li = lane & 15, lg = lane >> 4;
  const int64_t nb = frag / ksteps, ks = frag - nb * ksteps;
  const int64_t o = nb * 16 + li, c0 = ks * 32 + lg * 8;
  bf16_t v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = (o < O && c0 + e < C) ? src[(c0 + e) * sc + o * so] : (bf16_t)0;
  uint4 pk;
  pk.x = v[0] | ((uint32_t)v[1] << 16); pk.y = v[2] | ((uint32_t)v[3] << 16);
  pk.z = v[4] | ((uint32_t)v[5] << 16); pk.w = v[6] | ((uint32_t)v[7] << 16);
  *(uint4*)(dst + (frag << 9) + lane * 8) = pk;
}

size_t packed_weight_bytes(int64_t C, int64_t O) {
  if (C <= 0 || O <= 0) return 0;
  return (size_t)((O + 15) / 16) * (size_t)((C + 31) / 32) * 1024;
}

int64_t packed_weight_ksteps(int64_t C) { return (C + 31) / 32; }

hipError_t launch_pack_weight(const bf16_t* src, int64_t sc, int64_t so, int64_t C, int64_t O, bf16_t* dst,
                              hipStream_t stream) {
  const int64_t ksteps = (C + 31) / 32, nfrag = ((O + 15) / 16) * ksteps;
  if (nfrag <= 0) return hipSuccess;
  if ((nfrag + 3) / 4 > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((nfrag + 3) / 4)), dim3(256), 0, stream, src, sc, so, C, O,
                     ksteps, nfrag, dst);
  return hipGetLastError();
}

// Raise a kernel's dynamic LDS limit once per device (done: bit i set = device i has it).
static hipError_t allow_lds_once(const void* kernel, int bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = 1ull << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
  return e;
}

hipError_t launch_gemm_decode(const GemmArgs& a, hipStream_t stream) {
  static std::atomic<uint64_t> done0{0}, done1{0};
  const int G = a.tiles_m * a.tiles_n * a.ksplit;
  if (a.n_ext > 0) {
    hipError_t e = allow_lds_once((const void*)gemm_decode_kernel<true>, D_LDS, done1);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((gemm_decode_kernel<true>), dim3(G), dim3(D_THREADS), D_LDS, stream, a);
  } else {
    hipError_t e = allow_lds_once((const void*)gemm_decode_kernel<false>, D_LDS, done0);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((gemm_decode_kernel<false>), dim3(G), dim3(D_THREADS), D_LDS, stream, a);
  }
  return hipGetLastError();
}

}  // namespace marlaas
