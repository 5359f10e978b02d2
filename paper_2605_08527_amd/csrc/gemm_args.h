// Kernel arguments and LDS layout helpers shared by the GEMM kernels (large-batch, small-batch and
// decode) and the split-contraction finish kernel.
#pragma once
#include "common.h"

namespace marlaas {

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
  // ([ks][tiles_m * 256][ldp], grouped row order); splitk_finish_kernel adds them up.
  int ksplit; int64_t kchunk; float* partials;
  int64_t ldp;             // row stride of the partial sums (tiles_n * tile width)
  int64_t pm;              // rows of one split's partial sums (tiles_m * tile height)
  const RowChunk* chunks; int n_chunks;   // row chunks of the grouped order (finish kernel)
  // Fused shrink of the small-batch path: every column tile also computes 32 columns of
  // X * [all adapters' shrink factors] (extended column e = rank offset of adapter t + q); the
  // finish kernel picks each row's own adapter, scales and writes u_out.
  const ExtCol* ext_cols; const int32_t* ext_roff; int n_ext;   // n_ext = sum of the ranks; 0: not fused
  // ExtCol::t counts entries of the whole adapter bank, `table` may start inside it: entry index
  // of table[0]; ext_roff[] are offsets in the bank's column space, ext_base the call's first one
  int ext_t0, ext_base;
  float* u_part; int64_t ldu;   // [ks][pm][ldu] fp32 partial sums of the extended columns
  float* u_out;                 // [T][r_stride] (may be null)
  // Several projections in one pass (small-batch kernels only; n_proj <= 1: the fields above
  // describe the only projection).  Column tile tn belongs to the last projection whose tile0 <=
  // tn; `table`, `ext_roff` and ExtCol::t then index [projection][adapter].
  int n_proj;
  int fin_cols;                 // column chunks of the finish kernel's grid, all projections
  // Decode kernel that finishes the call itself (fin_in_kernel = 1: no finish kernel runs; the
  // partial sums are then in accumulator order, [split][tile][unit][column block][lane] x 4).
  //   sync    : device counters, all zero between launches: per tile the splits whose partial
  //             sums are performed, then per tile the splits that are through with it; then per
  //             row tile the workgroups whose partial u is performed and those through with u
  //   grp_ids : adapter of every grouped row (-1: none)
  //   spin_limit: polls of the kernel's one bounded wait
  int fin_in_kernel, out_is_f32, lform, spin_limit;
  int32_t* sync;
  const int32_t* grp_ids;
  // Large-batch kernel, LoRA expand by DMA (lora_dma = 1): U2 is u as a two-term bf16 split
  // ([T][2 r_stride], row m = [u_hi (r_pad) | u_lo (r_pad)] of its adapter), lora_tiles the list
  // of 64-wide extra contraction tiles of every 256-row tile (lora_tile_list_kernel), zero_line
  // 16 readable zero bytes that masked DMA lanes fetch.
  const bf16_t* U2; const int32_t* lora_tiles; const bf16_t* zero_line; int lora_dma;
  ProjEntry proj[MAX_PROJ];     // by value: read with wave-uniform loads from the kernel arguments
};

// List of one 256-row tile's extra contraction tiles: int32 [LT_STRIDE]: count (-1: more than
// LT_MAX, the kernel then stages the expand through registers), then {adapter, first row, end row,
// first contraction index} per tile.
static constexpr int LT_MAX = 15, LT_STRIDE = 64;

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// LDS byte offset of 16-byte unit `unit` of row `row` in a [rows][64] bf16 tile.
__device__ __forceinline__ int swz_rowk(int row, int unit) {
  return row * 128 + ((unit ^ ((row >> 1) & 7)) << 4);
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

// s_waitcnt immediate that waits only for the vector-memory counter (6 bits, split 3:0 / 15:14)
#define VMCNT(n) (0x0F70 | ((n) & 15) | ((((n) >> 4) & 3) << 14))

// Small-batch kernels: tile of the partial sums and of the finish kernel's grid.
static constexpr int SK_BM = 128, SK_BN = 128, SK_BX = 32;

// Decode kernel on a packed copy of the weight (gemm_decode.hip): same tiles, same partial-sum
// layout and same finish kernel as gemm_skinny_kernel.  Bop (and every ProjEntry::W) is the packed
// copy, ldb (ProjEntry::ldw) its k-steps per column block; the adapters' factors must be stored
// contraction-contiguous when the shrink is fused (n_ext > 0).
hipError_t launch_gemm_decode(const GemmArgs& a, hipStream_t stream);

}  // namespace marlaas
