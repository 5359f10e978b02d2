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
//
// Who finishes the call (adds the splits, adds the expand, rounds, scatters the rows):
//   fin_in_kernel = 0 (default): splitk_finish_kernel, a second launch; partial sums as fp32 rows.
//   fin_in_kernel = 1: this kernel.  The splits of a tile share out its 32 units (16 rows x 32
//     columns) and meet through counters in device memory; the column tiles that carry extended
//     columns publish their partial u the same way.  Everything that crosses workgroups is
//     written and read with the agent-scope policy on the instruction itself.  There is one
//     bounded wait; a split that does not see the others in time leaves its share to whichever
//     split is through with the tile last, and u that does not show up in time is recomputed, so
//     no workgroup ever depends on another one being scheduled.  On MI355X every fabric round
//     trip in that tail costs 1 - 1.5 us and the whole comes out slower than the second launch,
//     which is why it is not the default.
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
static constexpr int D_MAXOCT = 32;                    // octets (8 ranks of one adapter) per 16-row block on the MFMA expand
// after the ring: per row of the tile the expand factor (8 B), token, adapter, rank, rank offset, scale;
// flags; per 16-row block the octet count and per octet its factor address (8 B), adapter, first rank, rank
static constexpr int D_TAB_BYTES = SK_BM * (8 + 4 * 5) + 16 + 8 * 4 + 8 * D_MAXOCT * (8 + 4 + 4 + 4);
static constexpr int D_LDS = D_RING_BYTES + D_TAB_BYTES;

// Tuning aid, compiled in only with -DMARLAAS_DECODE_STAMPS: wave 0 of every workgroup records the
// constant-rate clock at a few points of the kernel; marlaas_debug_decode_stamps copies the record out.
#ifdef MARLAAS_DECODE_STAMPS
__device__ unsigned long long d_stamps[1024][12];
#define D_STAMP(i_) do { if (tid == 0 && blockIdx.x < 1024) d_stamps[blockIdx.x][i_] = wall_clock64(); } while (0)
#define D_STAMP_CLEAR() do { if (tid == 0 && blockIdx.x < 1024) for (int z_ = 7; z_ < 12; ++z_) d_stamps[blockIdx.x][z_] = 0; } while (0)
extern "C" int marlaas_debug_decode_stamps(unsigned long long* host) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(d_stamps), sizeof(d_stamps));
}
#else
#define D_STAMP(i_) do { } while (0)
#define D_STAMP_CLEAR() do { } while (0)
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

// Memory shared between workgroups inside one launch (partial sums, u, counters) is accessed with
// the agent-scope cache policy on the individual instruction (sc1: the access is performed at the
// level all XCDs share), the way relaxed agent-scope atomics are: no write-back or invalidation of
// a whole L2 is needed, which with 256 workgroups costs tens of microseconds.  A store is performed
// once the vector-memory counter has counted it down.
__device__ __forceinline__ void store4_agent(float* p, f32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1" :: "v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void load4_agent(f32x4& v, const float* p) {     // complete after wait_vm<..>()
  asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v) : "v"(p) : "memory");
}

// src of the lane N places down in the 16-lane DPP row; `old` where the row has no such lane
template <int N>
__device__ __forceinline__ int row_shr(int old, int src) {
  return __builtin_amdgcn_update_dpp(old, src, 0x110 + N, 0xf, 0xf, false);
}

// PHASE 0: the products (and, with fin_in_kernel = 1, the finish); PHASE 1: only the finish, as a
// launch of its own after a PHASE 0 launch with fin_in_kernel = 2 on the same arguments.
template <bool EXT, int PHASE>
__global__ __launch_bounds__(D_THREADS) void gemm_decode_kernel(GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  uint64_t* rL_s = (uint64_t*)(smem + D_RING_BYTES);       // per row of the tile: expand factor of its adapter,
  uint64_t* oct_L_s = rL_s + SK_BM;                        // (per octet: address of its 8 ranks in row 0 of the factor)
  int32_t* tok_s = (int32_t*)(oct_L_s + 8 * D_MAXOCT);     // token (-1: past the end),
  int32_t* radp_s = tok_s + SK_BM;                         // adapter (-1: none),
  int32_t* rrank_s = radp_s + SK_BM;                       // rank,
  int32_t* rroff_s = rrank_s + SK_BM;                      // first extended column of the adapter,
  float* rscale_s = (float*)(rroff_s + SK_BM);             // scale
  int32_t* flag_s = rroff_s + 2 * SK_BM;
  int32_t* oct_cnt_s = flag_s + 4;                         // per 16-row block: octets (-1: expand without MFMA)
  int32_t* oct_t_s = oct_cnt_s + 8;
  int32_t* oct_q_s = oct_t_s + 8 * D_MAXOCT;
  int32_t* oct_r_s = oct_q_s + 8 * D_MAXOCT;
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
  int64_t ldb = a.ldb, Nout = a.Nout, n0 = pn0, ldo = a.ldo;
  void* outp = a.out;
  int p_idx = 0, tab0 = 0;
  if (a.n_proj > 1) {                            // the projection this column tile belongs to (wave-uniform)
    for (int q = 1; q < a.n_proj; ++q) if (tn >= a.proj[q].tile0) p_idx = q;
    Bop = (const bf16_t*)a.proj[p_idx].W; ldb = a.proj[p_idx].ldw; Nout = a.proj[p_idx].Nout;
    n0 = (int64_t)(tn - a.proj[p_idx].tile0) * SK_BN;
    outp = a.proj[p_idx].out; ldo = a.proj[p_idx].ldo; tab0 = a.proj[p_idx].tab0;
  }
  const int64_t kbeg = (int64_t)ks_idx * a.kchunk;
  const int64_t kend = (kbeg + a.kchunk) < a.Kc ? (kbeg + a.kchunk) : a.Kc;
  const int ntile = PHASE == 0 ? (int)((kend - kbeg) / DK) : 0;
  D_STAMP(0);
  D_STAMP_CLEAR();

  // ---- the loads everything else waits for go first: the token indices of the x rows this lane
  // requests by DMA (rows past the end repeat the last row: their results are never used) and the
  // source row of its share of the extended columns.  (index, pointer and rank index: 3 requests)
  int32_t tok_r[2] = {0, 0}, adp_r[2] = {-1, -1};
  int arow[2];
  bool row_in[2];
  const bool lora_on = a.n_adapters > 0 && a.table != nullptr && (EXT || a.U != nullptr);
  const bool has_grp = lora_on && a.grp_ids != nullptr;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    arow[j] = (wave * 2 + j) * 8 + (lane >> 3);
    int64_t m = m0 + arow[j];
    if (m >= a.T) m = a.T - 1;
    tok_r[j] = (int32_t)m;
    if (a.perm) asm volatile("global_load_dword %0, %1, off" : "=v"(tok_r[j]) : "v"(a.perm + m) : "memory");
    row_in[j] = m0 + arow[j] < a.T;
    if (has_grp) asm volatile("global_load_dword %0, %1, off" : "=v"(adp_r[j]) : "v"(a.grp_ids + m) : "memory");
  }
  const int erow = wave * 4 + ((lane & 31) >> 3);            // extended columns: 4 rows per wave (lanes 0-31)
  uint64_t e_ptr = 0;
  int32_t e_q = 0;
  if (EXT && PHASE == 0) {
    int e = tn * SK_BX + erow;
    if (e >= a.n_ext) e = a.n_ext - 1;
    const char* ce = (const char*)(a.ext_cols + e);
    asm volatile("global_load_dwordx2 %0, %1, off" : "=v"(e_ptr) : "v"(ce + (a.which ? 0 : 8)) : "memory");
    asm volatile("global_load_dword %0, %1, off" : "=v"(e_q) : "v"(ce + 20) : "memory");
  }
  const int n_first = (a.perm ? 2 : 0) + (has_grp ? 2 : 0) + (EXT && PHASE == 0 ? 2 : 0);      // requests so far

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
  asm volatile("" : "+v"(tok_r[0]), "+v"(tok_r[1]), "+v"(adp_r[0]), "+v"(adp_r[1]), "+v"(e_ptr), "+v"(e_q));
  D_STAMP(1);
  // the rows' adapter entries (expand factor, rank and scale, rank offset): requested before the
  // first DMA, so they have arrived when the first tile has
  uint64_t ent_L[2] = {0, 0}, ent_rs[2] = {0, 0};
  int32_t ent_off[2] = {0, 0};
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    if (!row_in[j]) adp_r[j] = -1;
    if (adp_r[j] >= 0) {
      const char* en = (const char*)(a.table + tab0 + adp_r[j]);
      asm volatile("global_load_dwordx2 %0, %1, off" : "=v"(ent_L[j]) : "v"(en + (a.which ? 8 : 0)) : "memory");
      asm volatile("global_load_dwordx2 %0, %1, off" : "=v"(ent_rs[j]) : "v"(en + 16) : "memory");
      if (EXT) asm volatile("global_load_dword %0, %1, off" : "=v"(ent_off[j]) : "v"(a.ext_roff + tab0 + adp_r[j]) : "memory");
    }
  }

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
  wait_vm_dyn(ntile > 0 ? issued - dma_end[0] : 0);
  asm volatile("" : "+v"(ent_L[0]), "+v"(ent_L[1]), "+v"(ent_rs[0]), "+v"(ent_rs[1]), "+v"(ent_off[0]), "+v"(ent_off[1]));
  if ((lane & 7) == 0) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int r = arow[j];
      const bool on = adp_r[j] >= 0;
      tok_s[r] = row_in[j] ? tok_r[j] : -1;
      radp_s[r] = adp_r[j];
      rL_s[r] = on ? ent_L[j] : 0;
      rrank_s[r] = on ? (int32_t)(ent_rs[j] & 0xffffffffu) : 0;
      rscale_s[r] = on ? __uint_as_float((uint32_t)(ent_rs[j] >> 32)) : 0.f;
      rroff_s[r] = ent_off[j] - a.ext_base;
    }
  }
  if (ntile > 0) {
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
  __syncthreads();     // the ring is free (and the per-row tables are complete)

  // ---- k tail (the last split when Kc is not a multiple of 64): one masked tile, staged through
  // registers into slot 0; every wave handles its own k-step, values beyond kend are zeros
  if (PHASE == 0 && kbeg + (int64_t)ntile * DK < kend) {
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
  if (PHASE == 0) {
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

  const int64_t ustride = a.pm * a.ldu;
  float* up0 = EXT ? a.u_part + (m0 + 32 * wn + li) * a.ldu + tn * SK_BX + 4 * lg : nullptr;   // rows 16 (2 wn + j) + li, ext columns 16 xb + 4 lg ..
  if (PHASE == 0 && !a.fin_in_kernel) {
    // ---- partial sums as plain fp32 rows, [ks][pm][ldp]: splitk_finish_kernel completes the call
    float* part = a.partials + ks_idx * a.pm * a.ldp + (m0 + li) * a.ldp + pn0 + wn * 32 + 4 * lg;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int rb = (4 * g + i + 2 * wn) & 7;
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
        *(f32x4*)(part + (int64_t)(rb * 16) * a.ldp + cb * 16) = acc[i][cb];
    }
    if (EXT && g == 0) {
      float* up = up0 + ks_idx * ustride;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int xb = 0; xb < 2; ++xb) *(f32x4*)(up + (int64_t)(j * 16) * a.ldu + xb * 16) = eacc[j][xb];
    }
    D_STAMP(6);
    return;
  }

  // ---- the call is finished here.  A tile's 32 units (16-row block rb x 32-column group: unit
  // 4 rb + column group) are shared out evenly to its splits: split s adds up, expands and stores
  // units [s * 32 / ksplit, (s + 1) * 32 / ksplit), one or more per wave.  Partial sums travel in
  // accumulator order, [split][tile][unit][column block][lane] x 4 floats: one contiguous kilobyte
  // per wave and instruction on both sides.
  const int ntiles_all = a.tiles_m * a.tiles_n;
  const int tile_id = tm * a.tiles_n + tn;
  const int64_t fstride = (int64_t)ntiles_all * (SK_BM * SK_BN);          // floats between splits
  float* pf0 = a.partials + (int64_t)tile_id * (SK_BM * SK_BN) + lane * 4; // split 0, unit 0, column block 0
  const bool carries = EXT && tn * SK_BX < a.n_ext;
  if (PHASE == 0 && (a.ksplit > 1 || a.fin_in_kernel == 2)) {
    float* pf = pf0 + ks_idx * fstride;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int unit = ((4 * g + i + 2 * wn) & 7) * 4 + wn;
#pragma unroll
      for (int cb = 0; cb < 2; ++cb) store4_agent(pf + (unit * 2 + cb) * 256, acc[i][cb]);
    }
  }
  if (PHASE == 0 && carries && g == 0) {
    float* up = up0 + ks_idx * ustride;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int xb = 0; xb < 2; ++xb) store4_agent(up + (int64_t)(j * 16) * a.ldu + xb * 16, eacc[j][xb]);
  }
  if (PHASE == 0 && a.fin_in_kernel == 2) return;          // the PHASE 1 launch finishes the call
  // while the stores travel: per 16-row block, the octets (8 consecutive ranks of one adapter's
  // factor) its rows' adapters have.  The MFMA expand needs factors stored [column][rank] with
  // ranks that are multiples of 8; other blocks (count -1) take the plain fp32 expand.  One lane
  // per row, a 16-lane DPP row per block: the first row of every adapter in the block appends the
  // adapter's octets at the running count of the rows before it.
  if (tid < SK_BM) {
    const int t = radp_s[tid], rank = rrank_s[tid];
    const bool has = lora_on && t >= 0 && rank > 0;
    const int key = has ? t : -1;
    bool first = has;
    first &= row_shr<1>(-1, key) != key;   first &= row_shr<2>(-1, key) != key;
    first &= row_shr<3>(-1, key) != key;   first &= row_shr<4>(-1, key) != key;
    first &= row_shr<5>(-1, key) != key;   first &= row_shr<6>(-1, key) != key;
    first &= row_shr<7>(-1, key) != key;   first &= row_shr<8>(-1, key) != key;
    first &= row_shr<9>(-1, key) != key;   first &= row_shr<10>(-1, key) != key;
    first &= row_shr<11>(-1, key) != key;  first &= row_shr<12>(-1, key) != key;
    first &= row_shr<13>(-1, key) != key;  first &= row_shr<14>(-1, key) != key;
    first &= row_shr<15>(-1, key) != key;
    const int n_oct = first ? rank >> 3 : 0;
    int inc = n_oct, bad = (has && (rank & 7)) ? 1 : 0;      // inclusive scans along the row
    inc += row_shr<1>(0, inc); bad |= row_shr<1>(0, bad);
    inc += row_shr<2>(0, inc); bad |= row_shr<2>(0, bad);
    inc += row_shr<4>(0, inc); bad |= row_shr<4>(0, bad);
    inc += row_shr<8>(0, inc); bad |= row_shr<8>(0, bad);
    const int rb = tid >> 4, start = inc - n_oct;
    if (first && (rank & 7) == 0 && inc <= D_MAXOCT) {
      for (int q0 = 0, o = rb * D_MAXOCT + start; q0 < rank; q0 += 8, ++o) {
        oct_t_s[o] = t;
        oct_q_s[o] = q0;
        oct_r_s[o] = rank;
        oct_L_s[o] = rL_s[tid] + (uint64_t)q0 * sizeof(bf16_t);
      }
    }
    if ((tid & 15) == 15) {
      const bool ok = a.lform == FORM_NT && (a.r_stride & 3) == 0 && bad == 0 && inc <= D_MAXOCT;
      oct_cnt_s[rb] = !lora_on ? 0 : ok ? inc : -1;
    }
  }
  D_STAMP(6);

  // ---- counters (all zero between launches).  Per tile: `arrive` counts the splits whose partial
  // sums are performed, `done` the splits that are through with the tile (bits 8.. : splits that
  // gave up waiting, whose units the last split through then finishes: nobody ever has to wait).
  // Per row tile: `u_ready` counts the workgroups (every split of every column tile that carries
  // extended columns) whose partial u is performed, `u_done` those that will not read it again.
  int32_t* arrive = a.sync + tile_id;
  int32_t* done = a.sync + ntiles_all + tile_id;
  int32_t* u_ready = a.sync + 2 * ntiles_all + tm;
  int32_t* u_done = u_ready + a.tiles_m;
  const int n_sig = (a.n_ext + SK_BX - 1) / SK_BX < a.tiles_n ? (a.n_ext + SK_BX - 1) / SK_BX : a.tiles_n;
  const int u_need = n_sig * a.ksplit;
  const bool wants_u = EXT && lora_on;
  bool gave_up = false, u_ok = true;
  if (PHASE == 0) {
    wait_vm<0>();                        // this thread's partial sums are performed
    __syncthreads();                     // every thread's are
    D_STAMP(9);
    if (tid == 0) {
      if (a.ksplit > 1) __hip_atomic_fetch_add(arrive, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (carries) __hip_atomic_fetch_add(u_ready, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      // one bounded wait for the other splits of the tile and for u
      int ok_p = a.ksplit == 1, ok_u = !wants_u;
      for (int it = 0; it < a.spin_limit && !(ok_p && ok_u); ++it) {
        // (both counters are read in one round trip)
        const int va = __hip_atomic_load(arrive, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int vu = __hip_atomic_load(u_ready, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ok_p = ok_p || va >= a.ksplit;
        ok_u = ok_u || vu >= u_need;
        if (!(ok_p && ok_u)) __builtin_amdgcn_s_sleep(2);
      }
      flag_s[0] = ok_p; flag_s[1] = ok_u;
    }
    __syncthreads();
    D_STAMP(7);
    gave_up = flag_s[0] == 0;
    u_ok = flag_s[1] != 0;
  } else {
    __syncthreads();                     // the octet lists are complete
  }
  const int rs = a.r_stride;
  float* u_s = (float*)smem;             // [128][rs], rows of the tile (the ring is free)
  const int per = 32 / a.ksplit;         // units of a share (the host allows ksplit 1, 2, 4, 8 here)

  // One unit: sums s[cb] of row block rb (row li), columns n0 + 32 wnu + 16 cb + 4 lg .. + 3.
  auto finish_unit = [&](int rb, int wnu, f32x4 (&s)[2], const uint4 (&pre)[2]) {
    const int row = rb * 16 + li;
    const int32_t tok = tok_s[row];
    const int cnt = oct_cnt_s[rb];
    const int64_t nb = n0 + wnu * 32;
    if (cnt > 0) {
      // expand on the MFMAs: first operand 16 columns x 4 octets of the factors, second the rows'
      // u in two bf16 terms (zeros where the octet is another adapter's)
      for (int k0 = 0; k0 < cnt; k0 += 4) {
        const int o = k0 + lg;
        const bool valid = o < cnt;
        const int oi = rb * D_MAXOCT + (valid ? o : 0);
        const int r = oct_r_s[oi];
        union { uint4 u; bf16x8 v; } fa[2];
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
          fa[cb].u = make_uint4(0, 0, 0, 0);
          const int64_t n = nb + cb * 16 + li;
          if (k0 == 0) fa[cb].u = pre[cb];
          else if (valid && n < Nout) fa[cb].u = *(const uint4*)((const bf16_t*)(uintptr_t)oct_L_s[oi] + n * r);
        }
        float uv[8];
        const bool mine = valid && radp_s[row] == oct_t_s[oi];
        {
          const float* ur = u_s + row * rs + oct_q_s[oi];
          const float4 ua = *(const float4*)ur, ub = *(const float4*)(ur + 4);
          uv[0] = ua.x; uv[1] = ua.y; uv[2] = ua.z; uv[3] = ua.w; uv[4] = ub.x; uv[5] = ub.y; uv[6] = ub.z; uv[7] = ub.w;
        }
        union { uint32_t w[4]; bf16x8 v; } hi, lo;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float u0 = mine ? uv[2 * e] : 0.f, u1 = mine ? uv[2 * e + 1] : 0.f;
          const uint32_t h0 = float_to_bf16_bits(u0), h1 = float_to_bf16_bits(u1);
          const uint32_t l0 = float_to_bf16_bits(u0 - __uint_as_float(h0 << 16)), l1 = float_to_bf16_bits(u1 - __uint_as_float(h1 << 16));
          hi.w[e] = h0 | (h1 << 16);
          lo.w[e] = l0 | (l1 << 16);
        }
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
          s[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[cb].v, lo.v, s[cb], 0, 0, 0);
          s[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[cb].v, hi.v, s[cb], 0, 0, 0);
        }
      }
    } else if (cnt < 0 && tok >= 0 && rrank_s[row] > 0) {
      // plain fp32 expand of this lane's row
      const int rank = rrank_s[row];
      const bf16_t* L = (const bf16_t*)(uintptr_t)rL_s[row];
      const float* ur = u_s + row * rs;
#pragma unroll
      for (int cb = 0; cb < 2; ++cb) {
        const int64_t n = nb + cb * 16 + 4 * lg;
        if (n >= Nout) continue;
        float y4[4] = {0.f, 0.f, 0.f, 0.f};
        if (a.lform == FORM_NT) {                  // L[n * rank + q]
          for (int q = 0; q < rank; ++q) {
            const float uq = ur[q];
#pragma unroll
            for (int v = 0; v < 4; ++v) y4[v] = fmaf(uq, bf16_bits_to_float(L[(n + v) * rank + q]), y4[v]);
          }
        } else {                                   // L[q * Nout + n]
          for (int q = 0; q < rank; ++q) {
            const uint2 w = *(const uint2*)(L + (int64_t)q * Nout + n);
            const float uq = ur[q];
            y4[0] = fmaf(uq, __uint_as_float(w.x << 16), y4[0]); y4[1] = fmaf(uq, __uint_as_float(w.x & 0xffff0000u), y4[1]);
            y4[2] = fmaf(uq, __uint_as_float(w.y << 16), y4[2]); y4[3] = fmaf(uq, __uint_as_float(w.y & 0xffff0000u), y4[3]);
          }
        }
        s[cb][0] += y4[0]; s[cb][1] += y4[1]; s[cb][2] += y4[2]; s[cb][3] += y4[3];
      }
    }
    if (tok < 0) return;
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
      const int64_t n = nb + cb * 16 + 4 * lg;
      if (n >= Nout) continue;                     // (Nout is a multiple of 8: four columns are in or out together)
      if (a.out_is_f32) {
        *(float4*)((float*)outp + (int64_t)tok * ldo + n) = make_float4(s[cb][0], s[cb][1], s[cb][2], s[cb][3]);
      } else {
        uint2 o;
        o.x = float_to_bf16_bits(s[cb][0]) | ((uint32_t)float_to_bf16_bits(s[cb][1]) << 16);
        o.y = float_to_bf16_bits(s[cb][2]) | ((uint32_t)float_to_bf16_bits(s[cb][3]) << 16);
        *(uint2*)((bf16_t*)outp + (int64_t)tok * ldo + n) = o;
      }
    }
  };
  // the first k-step's factor fragments of a unit: they depend on nothing that travels
  auto prefetch_unit = [&](int rb, int wnu, uint4 (&pre)[2]) {
    const int cnt = oct_cnt_s[rb];
    const int oi = rb * D_MAXOCT + (lg < cnt ? lg : 0);
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
      pre[cb] = make_uint4(0, 0, 0, 0);
      const int64_t n = n0 + wnu * 32 + cb * 16 + li;
      if (lg < cnt && n < Nout) pre[cb] = *(const uint4*)((const bf16_t*)(uintptr_t)oct_L_s[oi] + n * oct_r_s[oi]);
    }
  };
  // One share (the units of split `share`): u of its rows into LDS, then its units, wave by wave.
  auto finish_share = [&](int share) {
    const int u0 = share * per;
    const int r0 = (u0 >> 2) * 16, nrows = per >= 4 ? per * 4 : 16;
    const bool from_regs = PHASE == 0 && a.ksplit == 1;   // the only split: the sums are this wave's accumulators
    const int rounds = from_regs ? 4 : (per + 7) >> 3;
#pragma unroll 1
    for (int it = 0; it < rounds; ++it) {
      const int uu = wave + 8 * it;
      const bool active = from_regs || uu < per;
      const int unit = from_regs ? ((4 * g + it + 2 * wn) & 7) * 4 + wn : u0 + uu;
      uint4 pre[2];
      f32x4 pv[8][2];                    // the unit's partial sums, all splits: complete after wait_vm<0>()
      if (active) {
        if (!from_regs) {
#pragma unroll
          for (int ks = 0; ks < 8; ++ks)
            if (ks < a.ksplit) {
#pragma unroll
              for (int cb = 0; cb < 2; ++cb) load4_agent(pv[ks][cb], pf0 + ks * fstride + (unit * 2 + cb) * 256);
            }
        }
        prefetch_unit(unit >> 2, unit & 3, pre);
      }
      if (it == 0) {
        if (lora_on) {
#pragma unroll 1
          for (int idx = tid; idx < nrows * rs; idx += D_THREADS) {
            const int row = r0 + idx / rs, q = idx % rs;
            float sum = 0.f;
            const int t = radp_s[row];
            if (t >= 0 && q < rrank_s[row]) {
              if (!EXT) {
                sum = a.U[(m0 + row) * rs + q];
              } else if (u_ok) {
                // this adapter's extended columns, the splits in order, scaled
                const float* up = a.u_part + (m0 + row) * a.ldu + rroff_s[row] + q;
                float pu[8];
#pragma unroll
                for (int ks = 0; ks < 8; ++ks)
                  pu[ks] = ks < a.ksplit ? __hip_atomic_load(up + ks * ustride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.f;
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) if (ks < a.ksplit) sum += pu[ks];
                sum *= rscale_s[row];
              } else {
                // (not reached in practice) the others' partial u did not show up in time: the
                // shrink of this row again, in plain fp32 arithmetic; factors are stored [rank][Kc]
                const AdapterEntry en = a.table[tab0 + t];
                const bf16_t* lin = (const bf16_t*)(a.which ? en.A : en.B) + (int64_t)q * a.Kc;
                const bf16_t* xr = a.Aop + (int64_t)tok_s[row] * a.lda;
                for (int64_t k = 0; k < a.Kc; ++k) sum = fmaf(bf16_bits_to_float(xr[k]), bf16_bits_to_float(lin[k]), sum);
                sum *= rscale_s[row];
              }
            }
            u_s[row * rs + q] = sum;
            // (ranks beyond the adapter's are padding of the saved row: zeros, as the shrink kernels write them)
            if (EXT && a.u_out != nullptr && tn == 0 && tok_s[row] >= 0) a.u_out[(m0 + row) * rs + q] = sum;
          }
        }
        __syncthreads();
      }
      if (active) {
        f32x4 s[2];
        if (from_regs) {
#pragma unroll
          for (int cb = 0; cb < 2; ++cb) {
            // (selected as values: the accumulators stay in registers)
            f32x4 c0 = acc[0][cb], c1 = acc[1][cb], c2 = acc[2][cb], c3 = acc[3][cb];
            asm volatile("" : "+v"(c0), "+v"(c1), "+v"(c2), "+v"(c3));
            s[cb] = it == 0 ? c0 : it == 1 ? c1 : it == 2 ? c2 : c3;
          }
        } else {
          wait_vm<0>();
          s[0] = f32x4{0.f, 0.f, 0.f, 0.f}; s[1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < 8; ++ks)
            if (ks < a.ksplit) {
#pragma unroll
              for (int cb = 0; cb < 2; ++cb) {
                asm volatile("" : "+v"(pv[ks][cb]));
                s[cb][0] += pv[ks][cb][0]; s[cb][1] += pv[ks][cb][1]; s[cb][2] += pv[ks][cb][2]; s[cb][3] += pv[ks][cb][3];
              }
            }
        }
        finish_unit(unit >> 2, unit & 3, s, pre);
      }
    }
    __syncthreads();                     // u_s may be overwritten by the next share
  };

  // first this split's own share; then, for the last split through with the tile, what the
  // others gave up on
  int u_old = -1;                        // tid 0: what u_done held before this workgroup's count (-1: not counted yet)
#pragma unroll 1
  for (int pass = 0; pass < 2; ++pass) {
    int todo = gave_up ? 0 : 1 << ks_idx;
    if (pass == 1) {
      if (PHASE == 1 || a.ksplit == 1) break;
      if (tid == 0) {
        const int old = __hip_atomic_fetch_add(done, 1 + (gave_up ? 256 << ks_idx : 0), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // a split that did its share and is not asked to do more is through with u as well: both
        // counters in one round trip
        if (EXT && !gave_up) u_old = __hip_atomic_fetch_add(u_done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int left = 0;
        if ((old & 255) == a.ksplit - 1) {
          // everyone is through with the tile: its counters are ready for the next launch
          // (launches on a stream are ordered)
          left = (old >> 8) | (gave_up ? 1 << ks_idx : 0);
          __hip_atomic_store(arrive, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_store(done, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        flag_s[2] = left;
      }
      __syncthreads();
      todo = flag_s[2];
    }
#pragma unroll 1
    for (int share = 0; share < a.ksplit; ++share)
      if ((todo >> share) & 1) finish_share(share);
    if (pass == 0) D_STAMP(8);
  }
  if (EXT && PHASE == 0) {
    // the last workgroup of the row tile through with u clears its two counters
    if (tid == 0) {
      const int old = u_old >= 0 ? u_old : __hip_atomic_fetch_add(u_done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (old == a.tiles_n * a.ksplit - 1) {
        __hip_atomic_store(u_ready, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(u_done, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
  D_STAMP(11);
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

template <bool EXT, int PHASE>
static hipError_t launch_phase(const GemmArgs& a, hipStream_t stream) {
  static std::atomic<uint64_t> done{0};
  hipError_t e = allow_lds_once((const void*)gemm_decode_kernel<EXT, PHASE>, D_LDS, done);
  if (e != hipSuccess) return e;
  const int G = a.tiles_m * a.tiles_n * a.ksplit;
  hipLaunchKernelGGL((gemm_decode_kernel<EXT, PHASE>), dim3(G), dim3(D_THREADS), D_LDS, stream, a);
  return hipGetLastError();
}

hipError_t launch_gemm_decode(const GemmArgs& a, hipStream_t stream) {
  hipError_t e = a.n_ext > 0 ? launch_phase<true, 0>(a, stream) : launch_phase<false, 0>(a, stream);
  if (e != hipSuccess || a.fin_in_kernel != 2) return e;
  return a.n_ext > 0 ? launch_phase<true, 1>(a, stream) : launch_phase<false, 1>(a, stream);
}

}  // namespace marlaas
