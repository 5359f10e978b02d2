// The low-rank side of the layer on bf16 data: the segmented shrink
// u = s_t (x A_t)  /  v = s_t (dY B_t^T), and the per-adapter weight-gradient
// reductions dA_t = sum x_i^T v_i, dB_t = sum u_i^T dY_i.  Only the per-task
// LoRA parameters are trained (paper Sec. 4.2), so these are the only weight
// gradients of the layer.  Both kernels read their big operand (x or dY) once
// and are bound by HBM; the small operand stays in LDS.
#include "gemm_args.h"

#include <atomic>

namespace marlaas {

// Raise a kernel's dynamic LDS limit to the hardware maximum, once per (kernel, device): `slot`
// names the kernel instantiation, bit i of its word = device i has it.
static hipError_t allow_big_lds(const void* kernel, int slot) {
  static std::atomic<uint64_t> done[32];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = 1ull << (dev & 63);
  if (done[slot].load(std::memory_order_acquire) & bit) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (e == hipSuccess) done[slot].fetch_or(bit, std::memory_order_release);
  return e;
}

// ============================================================== shrink
static constexpr int SH_THREADS = 256;
static constexpr int SH_ROWS = 64;     // rows per block (16 per wave)
static constexpr int SH_KSTG = 256;    // contraction values staged per step
static constexpr int SH_PITCH = SH_KSTG * 2 + 16;  // bytes per staged L row

struct ShrinkArgs {
  const bf16_t* X; int64_t ldx; int64_t C;
  const int32_t* perm; const int32_t* seg_off;
  const AdapterEntry* table; int which;
  float* u; int r_stride;
  int ksplit; int kchunk;   // kchunk is a multiple of SH_KSTG
  // ksplit > 1: split ks leaves its unscaled sums in partials[ks][T_lora][r_stride] and
  // shrink_finalize_kernel adds them in split order (the result does not depend on timing)
  float* partials; int64_t T_lora;
  // optional second output for the large-batch GEMM's DMA: row m holds [u_hi (r_pad) | u_lo (r_pad)]
  // of its adapter in bf16, u_hi = bf16(u), u_lo = bf16(u - u_hi); row stride 2 * r_stride
  bf16_t* u2;
  const bf16_t* zero_line;  // 16 readable zero bytes (what masked DMA lanes of shrink_ring_kernel fetch)
};

// u (scaled, fp32) and its two-term bf16 split for row m, rank index q of an adapter with padded rank r_pad
__device__ __forceinline__ void shrink_store(const ShrinkArgs& a, int64_t m, int q, int r_pad, float val) {
  a.u[m * a.r_stride + q] = val;
  if (a.u2) {
    const bf16_t h = float_to_bf16_bits(val);
    bf16_t* row = a.u2 + m * (2 * a.r_stride);
    row[q] = h;
    row[r_pad + q] = float_to_bf16_bits(val - bf16_bits_to_float(h));
  }
}

// grid: x = row blocks of the largest segment * ksplit, y = adapter
// NQT: 16-wide output tiles held per wave (covers the largest padded rank of the call)
// The kernel is bound by the one pass over X, so the loop is software-pipelined through
// registers: the x fragments and the factor tile of step s + 1 are requested before the MFMAs
// of step s; only the hand-over of the factor tile to LDS sits between two barriers.
template <int LFORM, int NQT>
__global__ __launch_bounds__(SH_THREADS, (NQT >= 8 ? 1 : 2)) void shrink_bf16_kernel(ShrinkArgs a) {
  extern __shared__ __attribute__((aligned(16))) char Ls[];   // [r_pad][SH_PITCH]
  const int t = blockIdx.y;
  const int lo = a.seg_off[t], hi = a.seg_off[t + 1];
  const int rb = blockIdx.x / a.ksplit, ks = blockIdx.x - rb * a.ksplit;
  const int row0 = lo + rb * SH_ROWS;
  if (row0 >= hi) return;
  const AdapterEntry e = a.table[t];
  const bf16_t* L = (const bf16_t*)(a.which ? e.B : e.A);
  const int r = e.rank;
  const int r_pad = (r + 15) & ~15;
  const int nqt = r_pad >> 4;
  const int64_t kbeg = (int64_t)ks * a.kchunk;
  const int64_t kend = (kbeg + a.kchunk) < a.C ? (kbeg + a.kchunk) : a.C;
  if (kbeg >= kend) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4, li = lane & 15;
  int m = row0 + wave * 16 + li;
  if (m >= hi) m = hi - 1;                   // clamped rows are never stored
  const int64_t tok = a.perm ? a.perm[m] : m;
  const bf16_t* xrow = a.X + tok * a.ldx;

  f32x4 acc[NQT];
  for (int q = 0; q < NQT; ++q) acc[q] = f32x4{0.f, 0.f, 0.f, 0.f};
  const uint4 zero4 = make_uint4(0, 0, 0, 0);
  constexpr int LREG = 2 * NQT;               // 16-byte pieces of the factor tile per thread
  const bool vec_nn = (r & 7) == 0;           // FORM_NN: a k-row of the factor is whole 16-byte pieces

  uint4 xn[2][4];                             // next step's x fragments
  uint4 ln[LREG];                             // next step's part of the factor tile
  // (a macro, not a lambda: the register arrays must not have their address taken)
#define SH_REQUEST(k0_)                                                                                   \
  do {                                                                                                    \
    const int64_t _k0 = (k0_);                                                                            \
    /* instruction (ms, j) covers 32 consecutive k, 8 per lane group: the four lanes of a row fetch */    \
    /* 64 contiguous bytes */                                                                             \
    _Pragma("unroll") for (int ms = 0; ms < 2; ++ms)                                                      \
      _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                     \
        const int64_t k = _k0 + ms * 128 + j * 32 + g * 8;                                                \
        xn[ms][j] = zero4;                                                                                \
        if (k < kend) xn[ms][j] = *(const uint4*)(xrow + k);                                              \
      }                                                                                                   \
    if (LFORM == FORM_NT) {          /* L_t[q * C + c]: thread (q = tid / 32 + 8 i, unit = tid % 32) */   \
      const int64_t k = _k0 + (tid & 31) * 8;                                                             \
      _Pragma("unroll") for (int i = 0; i < LREG; ++i) {                                                  \
        const int q = (tid >> 5) + 8 * i;                                                                 \
        ln[i] = zero4;                                                                                    \
        if (q < r && k < kend) ln[i] = *(const uint4*)(L + (int64_t)q * a.C + k);                         \
      }                                                                                                   \
    } else if (vec_nn) {             /* L_t[c * r + q]: thread = one k, pieces of 8 ranks */              \
      const int64_t k = _k0 + tid;                                                                        \
      _Pragma("unroll") for (int i = 0; i < LREG; ++i) {                                                  \
        ln[i] = zero4;                                                                                    \
        if (k < kend && i * 8 < r) ln[i] = *(const uint4*)(L + k * r + i * 8);                            \
      }                                                                                                   \
    }                                                                                                     \
  } while (0)
  SH_REQUEST(kbeg);
  for (int64_t k0 = kbeg; k0 < kend; k0 += SH_KSTG) {
    uint4 xf[2][4];
#pragma unroll
    for (int ms = 0; ms < 2; ++ms)
#pragma unroll
      for (int j = 0; j < 4; ++j) xf[ms][j] = xn[ms][j];
    __syncthreads();   // previous step's reads of Ls are done
    if (LFORM == FORM_NT) {
#pragma unroll
      for (int i = 0; i < LREG; ++i) {
        const int q = (tid >> 5) + 8 * i;
        if (q < r_pad) *(uint4*)(Ls + q * SH_PITCH + (tid & 31) * 16) = ln[i];
      }
    } else if (vec_nn) {
#pragma unroll
      for (int i = 0; i < LREG; ++i)
        if (i * 8 < r_pad) {
          const uint32_t w[4] = {ln[i].x, ln[i].y, ln[i].z, ln[i].w};
#pragma unroll
          for (int j = 0; j < 8; ++j)
            *(bf16_t*)(Ls + (i * 8 + j) * SH_PITCH + tid * 2) = (bf16_t)(w[j >> 1] >> ((j & 1) * 16));
        }
    } else {                          // odd ranks: element-wise, not pipelined
      const int64_t k = k0 + tid;
      const bool ok = k < kend;
      const bf16_t* lp = L + k * r;
      for (int q = 0; q < r_pad; ++q)
        *(bf16_t*)(Ls + q * SH_PITCH + tid * 2) = (ok && q < r) ? lp[q] : (bf16_t)0;
    }
    __syncthreads();
    if (k0 + SH_KSTG < kend) SH_REQUEST(k0 + SH_KSTG);
#pragma unroll
    for (int ms = 0; ms < 2; ++ms)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        union { uint4 u; bf16x8 v; } xa; xa.u = xf[ms][j];
        const int koff = (ms * 128 + j * 32 + g * 8) * 2;
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt)
          if (qt < nqt) {
            bf16x8 b = *(const bf16x8*)(Ls + (qt * 16 + li) * SH_PITCH + koff);
            acc[qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa.v, b, acc[qt], 0, 0, 0);
          }
      }
  }
  // D layout: row = 4 * (lane / 16) + v, column = lane % 16
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt)
    if (qt < nqt)
      for (int v = 0; v < 4; ++v) {
        const int mr = row0 + wave * 16 + 4 * g + v;
        if (mr < hi) {
          if (a.ksplit > 1) a.partials[((int64_t)ks * a.T_lora + mr) * a.r_stride + qt * 16 + li] = acc[qt][v];
          else shrink_store(a, mr, qt * 16 + li, r_pad, e.scale * acc[qt][v]);
        }
      }
}

// The same shrink with both operands moved global -> LDS by DMA through a ring of four 64-wide
// k-tiles: every request of a wave covers whole 128-byte row segments (the register-staged kernel
// above fetches 64-byte pieces and its factor tile through VGPRs) and three k-tiles are in flight
// per block.  A block takes 128 rows of one adapter where the segments are long (half the factor
// traffic of 64-row blocks) and 64 where they are short.  Measured on MI355X against the
// register-staged kernel: 10 - 15 % faster for factors stored rank-major, 3 - 10 % for
// contraction-major ones.  x part of a slot: [128 rows][64 k], 16-byte units
// XOR-swizzled like the GEMM's tiles; factor part: [r_pad][64 k] for factors stored [rank][C]
// (LFORM NT), [64 k][r_pad] read with transposing LDS reads for factors stored [C][rank] (LFORM
// NN, ranks multiples of 8).  Rows past the end of the segment repeat its last row (never stored),
// rank rows past r and contraction units past the end fetch zeros.
static constexpr int SR_NS = 4;

__device__ __forceinline__ void sr_wait(int n) {      // at most n vector-memory requests outstanding (n <= 16)
  switch (n) {
    case 0: __builtin_amdgcn_s_waitcnt(VMCNT(0)); break;
    case 1: __builtin_amdgcn_s_waitcnt(VMCNT(1)); break;
    case 2: __builtin_amdgcn_s_waitcnt(VMCNT(2)); break;
    case 3: __builtin_amdgcn_s_waitcnt(VMCNT(3)); break;
    case 4: __builtin_amdgcn_s_waitcnt(VMCNT(4)); break;
    case 5: __builtin_amdgcn_s_waitcnt(VMCNT(5)); break;
    case 6: __builtin_amdgcn_s_waitcnt(VMCNT(6)); break;
    case 7: __builtin_amdgcn_s_waitcnt(VMCNT(7)); break;
    case 8: __builtin_amdgcn_s_waitcnt(VMCNT(8)); break;
    case 9: __builtin_amdgcn_s_waitcnt(VMCNT(9)); break;
    case 10: __builtin_amdgcn_s_waitcnt(VMCNT(10)); break;
    case 11: __builtin_amdgcn_s_waitcnt(VMCNT(11)); break;
    case 12: __builtin_amdgcn_s_waitcnt(VMCNT(12)); break;
    case 13: __builtin_amdgcn_s_waitcnt(VMCNT(13)); break;
    case 14: __builtin_amdgcn_s_waitcnt(VMCNT(14)); break;
    case 15: __builtin_amdgcn_s_waitcnt(VMCNT(15)); break;
    case 16: __builtin_amdgcn_s_waitcnt(VMCNT(16)); break;
    default: __builtin_amdgcn_s_waitcnt(VMCNT(0)); break;
  }
}

// RT: 16-row tiles per wave (block = 64 RT rows)
template <int LFORM, int NQT, int RT>
__global__ __launch_bounds__(256) void shrink_ring_kernel(ShrinkArgs a) {
  constexpr int SR_ROWS = 64 * RT, SR_X_BYTES = SR_ROWS * 64 * 2, XI = 2 * RT;   // rows, x part of a slot, x instructions per wave and k-tile
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int t = blockIdx.y;
  const int lo = a.seg_off[t], hi = a.seg_off[t + 1];
  const int rb = blockIdx.x / a.ksplit, ks = blockIdx.x - rb * a.ksplit;
  const int row0 = lo + rb * SR_ROWS;
  if (row0 >= hi) return;
  const AdapterEntry e = a.table[t];
  const bf16_t* L = (const bf16_t*)(a.which ? e.B : e.A);
  const int r = e.rank;
  const int r_pad = (r + 15) & ~15;
  const int nqt = r_pad >> 4;
  const int64_t kbeg = (int64_t)ks * a.kchunk;
  const int64_t kend = (kbeg + a.kchunk) < a.C ? (kbeg + a.kchunk) : a.C;
  if (kbeg >= kend) return;
  const int ntile = (int)((kend - kbeg + 63) >> 6);
  const int l_bytes = NQT * 16 * 128;                  // factor part of a slot (room for the template's largest r_pad)
  const int slot_bytes = SR_X_BYTES + l_bytes;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, li = lane & 15;

  // ---- DMA sources.  x: instructions of 8 rows, XI per wave and k-tile.
  const bf16_t* xsrc[XI];
  int xk[XI];                                           // first contraction index of the lane's unit inside a k-tile
#pragma unroll
  for (int j = 0; j < XI; ++j) {
    const int row = (wave * XI + j) * 8 + (lane >> 3);
    const int unit = (lane & 7) ^ ((row >> 1) & 7);
    int m = row0 + row;
    if (m >= hi) m = hi - 1;
    const int64_t tok = a.perm ? a.perm[m] : m;
    xk[j] = unit * 8;
    xsrc[j] = a.X + tok * a.ldx + kbeg + unit * 8;
  }
  // factor: n_li instructions per k-tile, instruction i = wave + 4 jj
  constexpr int LPW = (2 * NQT + 3) / 4;
  // (contraction-major factors: a k-row of the tile holds 16 lq ranks, lq = the adapter's own count
  // of 16-rank blocks when that is a power of two (a whole number of k-rows per instruction), else
  // the template's; low-rank adapters then move a fraction of the tile)
  const int lq = (nqt & (nqt - 1)) == 0 ? nqt : NQT;
  const int n_li = LFORM == FORM_NT ? 2 * nqt : 2 * lq;
  const bf16_t* lsrc[LPW];
  int lk[LPW];                                         // contraction index (inside the k-tile) the lane's piece starts at
  bool lon[LPW];                                       // the piece exists (rank row / ranks inside r)
  int my_l = 0;
#pragma unroll
  for (int jj = 0; jj < LPW; ++jj) {
    const int i = wave + 4 * jj;
    lsrc[jj] = a.zero_line; lk[jj] = 0; lon[jj] = false;
    if (i < n_li) {
      ++my_l;
      if (LFORM == FORM_NT) {            // L[q * C + k]: 8 rank rows of 128 bytes per instruction
        const int q = i * 8 + (lane >> 3);
        const int unit = (lane & 7) ^ ((q >> 1) & 7);
        lk[jj] = unit * 8;
        lon[jj] = q < r;
        lsrc[jj] = L + (int64_t)q * a.C + kbeg + unit * 8;
      } else {                           // L[k * r + q]: k-rows of 16 NQT values (pieces past r are zeros), 2 NQT lanes per row
        const int lpr = 2 * lq;          // lanes (16-byte pieces) per k-row
        const int krow = i * (64 / lpr) + lane / lpr;
        const int q0 = (lane % lpr) * 8;
        lk[jj] = krow;
        lon[jj] = q0 < r;
        lsrc[jj] = L + (kbeg + krow) * r + q0;
      }
    }
  }
  const int per_tile = XI + my_l;
#define SR_DMA(kt_)                                                                                       \
  do {                                                                                                    \
    char* _sb = smem + ((kt_) % SR_NS) * slot_bytes;                                                      \
    const int64_t _k0 = kbeg + (int64_t)(kt_) * 64;                                                       \
    _Pragma("unroll") for (int _j = 0; _j < XI; ++_j) {                                                   \
      const bf16_t* _src = (_k0 + xk[_j]) < kend ? xsrc[_j] + (int64_t)(kt_) * 64 : a.zero_line;          \
      __builtin_amdgcn_global_load_lds((gptr_t)_src, (lptr_t)(_sb + (wave * XI + _j) * 1024), 16, 0, 0);  \
    }                                                                                                     \
    _Pragma("unroll") for (int _jj = 0; _jj < LPW; ++_jj)                                                 \
      if (wave + 4 * _jj < n_li) {                                                                        \
        const bf16_t* _src = a.zero_line;                                                                 \
        if (lon[_jj] && (_k0 + lk[_jj]) < kend)                                                           \
          _src = lsrc[_jj] + (LFORM == FORM_NT ? (int64_t)(kt_) * 64 : (int64_t)(kt_) * 64 * r);          \
        __builtin_amdgcn_global_load_lds((gptr_t)_src, (lptr_t)(_sb + SR_X_BYTES + (wave + 4 * _jj) * 1024), 16, 0, 0); \
      }                                                                                                   \
  } while (0)

  f32x4 acc[RT][NQT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int q = 0; q < NQT; ++q) acc[rt][q] = f32x4{0.f, 0.f, 0.f, 0.f};

#pragma unroll
  for (int s0 = 0; s0 < SR_NS - 1; ++s0)
    if (s0 < ntile) SR_DMA(s0);
  const int l_pitch = 32 * lq;                         // bytes per k-row of an NN factor tile
  for (int kt = 0; kt < ntile; ++kt) {
    // tile kt has landed (everything but the younger tiles' requests), everywhere; nobody reads tile kt - 1 any more
    const int last_issued = (kt + SR_NS - 2) < (ntile - 1) ? (kt + SR_NS - 2) : (ntile - 1);
    sr_wait((last_issued - kt) * per_tile);
    __syncthreads();
    if (kt + SR_NS - 1 < ntile) SR_DMA(kt + SR_NS - 1);
    const char* sb = smem + (kt % SR_NS) * slot_bytes;
#pragma unroll
    for (int k2 = 0; k2 < 2; ++k2) {
      bf16x8 xa[RT];
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
        xa[rt] = *(const bf16x8*)(sb + swz_rowk(wave * (16 * RT) + rt * 16 + li, k2 * 4 + g));
#pragma unroll
      for (int qt = 0; qt < NQT; ++qt)
        if (qt < nqt) {
          bf16x8 b;
          if (LFORM == FORM_NT) {
            b = *(const bf16x8*)(sb + SR_X_BYTES + swz_rowk(qt * 16 + li, k2 * 4 + g));
          } else {
            const char* p = sb + SR_X_BYTES + (k2 * 32 + g * 8 + (li >> 2)) * l_pitch + (qt * 16 + 4 * (li & 3)) * 2;
            b = lds_read_frag_tr(p, p + 4 * l_pitch);
          }
#pragma unroll
          for (int rt = 0; rt < RT; ++rt)
            acc[rt][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa[rt], b, acc[rt][qt], 0, 0, 0);
        }
    }
  }
#undef SR_DMA
  // D layout: row = 4 * (lane / 16) + v, column = lane % 16
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt)
      if (qt < nqt)
        for (int v = 0; v < 4; ++v) {
          const int mr = row0 + wave * (16 * RT) + rt * 16 + 4 * g + v;
          if (mr < hi) {
            if (a.ksplit > 1) a.partials[((int64_t)ks * a.T_lora + mr) * a.r_stride + qt * 16 + li] = acc[rt][qt][v];
            else shrink_store(a, mr, qt * 16 + li, r_pad, e.scale * acc[rt][qt][v]);
          }
        }
}

// Small batches (decode): one block per (adapter, 16 grouped rows); its 8 waves split the
// contraction, take both operands straight from global memory (L_t stored [r_t, C], so a lane's 8
// contraction values are one 16-byte load) and add their partial tiles through LDS in wave order,
// so the result does not depend on timing.
static constexpr int SS_WAVES = 8;
template <int DUMMY>
__global__ __launch_bounds__(64 * SS_WAVES) void shrink_small_nt_kernel(ShrinkArgs a) {
  extern __shared__ __attribute__((aligned(16))) char red[];   // [SS_WAVES][nqt][64] f32x4
  const int t = blockIdx.y;
  const int lo = a.seg_off[t], hi = a.seg_off[t + 1];
  const int row0 = lo + blockIdx.x * 16;
  if (row0 >= hi) return;
  const AdapterEntry e = a.table[t];
  const bf16_t* L = (const bf16_t*)(a.which ? e.B : e.A);
  const int r = e.rank, r_pad = (r + 15) & ~15, nqt = r_pad >> 4;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4, li = lane & 15;
  int m = row0 + li;
  if (m >= hi) m = hi - 1;
  const int64_t tok = a.perm ? a.perm[m] : m;
  const bf16_t* xrow = a.X + tok * a.ldx;
  const int64_t kw = ((a.C + SS_WAVES * 128 - 1) / (SS_WAVES * 128)) * 128;   // per wave, multiple of 128
  const int64_t kbeg = wave * kw;
  const int64_t kend = (kbeg + kw) < a.C ? (kbeg + kw) : a.C;
  f32x4 acc[8];
  for (int q = 0; q < 8; ++q) acc[q] = f32x4{0.f, 0.f, 0.f, 0.f};
  const uint4 zero4 = make_uint4(0, 0, 0, 0);
  for (int64_t k0 = kbeg; k0 < kend; k0 += 128) {
    uint4 xf[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t k = k0 + g * 32 + j * 8;
      xf[j] = zero4;
      if (k < kend) xf[j] = *(const uint4*)(xrow + k);
    }
#pragma unroll
    for (int qt = 0; qt < 8; ++qt)
      if (qt < nqt) {
        const int q = qt * 16 + li;
        uint4 lf[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int64_t k = k0 + g * 32 + j * 8;
          lf[j] = zero4;
          if (q < r && k < kend) lf[j] = *(const uint4*)(L + (int64_t)q * a.C + k);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          union { uint4 u; bf16x8 v; } xa, lb; xa.u = xf[j]; lb.u = lf[j];
          acc[qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa.v, lb.v, acc[qt], 0, 0, 0);
        }
      }
  }
  f32x4* rp = (f32x4*)red;
#pragma unroll
  for (int qt = 0; qt < 8; ++qt)
    if (qt < nqt) rp[(wave * nqt + qt) * 64 + lane] = acc[qt];
  __syncthreads();
  // wave w finishes q-tiles w, w + 8, ...
  for (int qt = wave; qt < nqt; qt += SS_WAVES) {
    f32x4 sum = rp[(0 * nqt + qt) * 64 + lane];
    for (int w = 1; w < SS_WAVES; ++w) {
      const f32x4 p = rp[(w * nqt + qt) * 64 + lane];
      sum[0] += p[0]; sum[1] += p[1]; sum[2] += p[2]; sum[3] += p[3];
    }
    for (int v = 0; v < 4; ++v) {
      const int mr = row0 + 4 * g + v;
      if (mr < hi) a.u[(int64_t)mr * a.r_stride + qt * 16 + li] = e.scale * sum[v];
    }
  }
}

// Second step of a shrink with a split contraction: block = (adapter, 16 grouped rows), thread =
// (row, 16 rank indices apart); the splits are added in split order, then scaled.
__global__ __launch_bounds__(256) void shrink_finalize_kernel(ShrinkArgs a) {
  const int t = blockIdx.y;
  const int lo = a.seg_off[t], hi = a.seg_off[t + 1];
  const int64_t m = lo + (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
  if (m >= hi) return;
  const AdapterEntry e = a.table[t];
  const int r_pad = (e.rank + 15) & ~15;
  for (int q = threadIdx.x & 15; q < r_pad; q += 16) {
    float sum = 0.f;
    for (int ks = 0; ks < a.ksplit; ++ks) sum += a.partials[((int64_t)ks * a.T_lora + m) * a.r_stride + q];
    shrink_store(a, m, q, r_pad, e.scale * sum);
  }
}

// Splits of the shrink's contraction: enough blocks to fill the chip when the rows alone do not.
static int shrink_splits(int64_t C, int64_t T_lora, int n_adapters, int rows = SH_ROWS) {
  const int64_t real_blocks = (T_lora + rows - 1) / rows + n_adapters;
  const int kst = (int)((C + SH_KSTG - 1) / SH_KSTG);
  int ksplit = 1;
  if (real_blocks < 512) {
    ksplit = (int)((1024 + real_blocks - 1) / real_blocks);
    if (ksplit > kst) ksplit = kst;
  }
  return ksplit;
}

size_t shrink_partial_bytes(int64_t C, int64_t T_lora, int n_adapters, int r_stride) {
  if (T_lora <= 0 || n_adapters <= 0) return 0;
  const int ks = shrink_splits(C, T_lora, n_adapters, SH_ROWS), kr = shrink_splits(C, T_lora, n_adapters, 128);
  const int k = ks > kr ? ks : kr;
  return k > 1 ? (size_t)k * T_lora * r_stride * sizeof(float) : 0;
}

hipError_t launch_shrink_bf16(const bf16_t* X, int64_t ldx, int64_t C, const int32_t* perm,
                              const int32_t* seg_off, int n_adapters, int max_seg,
                              const AdapterEntry* table, int which, int lora_form, float* u,
                              int r_stride, int64_t T_lora, float* partials, size_t partial_bytes,
                              bf16_t* u2, bool* wrote_u2, const bf16_t* zero_line, bool ranks_mult8, hipStream_t stream) {
  if (wrote_u2) *wrote_u2 = false;
  if (n_adapters <= 0 || max_seg <= 0 || T_lora <= 0) return hipSuccess;
  ShrinkArgs a;
  a.X = X; a.ldx = ldx; a.C = C; a.perm = perm; a.seg_off = seg_off; a.table = table;
  a.which = which; a.u = u; a.r_stride = r_stride;
  a.partials = nullptr; a.T_lora = T_lora; a.u2 = nullptr; a.zero_line = zero_line;
  const int64_t real_blocks = (T_lora + SH_ROWS - 1) / SH_ROWS + n_adapters;
  if (lora_form == FORM_NT && real_blocks <= 96) {
    a.ksplit = 1; a.kchunk = 0;
    const size_t lds = (size_t)SS_WAVES * (r_stride / 16) * 64 * sizeof(f32x4);
    hipLaunchKernelGGL(shrink_small_nt_kernel<0>, dim3((max_seg + 15) / 16, n_adapters), dim3(64 * SS_WAVES), lds,
                       stream, a);
    return hipGetLastError();
  }
  // both operands by DMA where every piece of a factor row stays inside the row; 128 rows per
  // block where the segments are long, 64 where they are short
  const bool ring = zero_line != nullptr && (lora_form == FORM_NT || ranks_mult8);
  const bool long_seg = T_lora >= (int64_t)512 * n_adapters;
  const int rows = ring ? (long_seg ? 128 : 64) : SH_ROWS;
  const int rb_max = (max_seg + rows - 1) / rows;
  const int kst = (int)((C + SH_KSTG - 1) / SH_KSTG);
  int ksplit = shrink_splits(C, T_lora, n_adapters, rows);
  // (no room for the splits' sums: fewer splits)
  const size_t per_split = (size_t)T_lora * r_stride * sizeof(float);
  if (ksplit > 1 && (partials == nullptr || partial_bytes < (size_t)ksplit * per_split))
    ksplit = partials ? (int)(partial_bytes / per_split) : 1;
  if (ksplit < 1) ksplit = 1;
  a.kchunk = ((kst + ksplit - 1) / ksplit) * SH_KSTG;
  ksplit = (int)((C + a.kchunk - 1) / a.kchunk);
  a.ksplit = ksplit;
  a.partials = partials;
  a.u2 = u2;
  if (wrote_u2) *wrote_u2 = u2 != nullptr;
  size_t lds = (size_t)r_stride * SH_PITCH;   // r_stride >= every r_pad
  typedef void (*kern_t)(ShrinkArgs);
  const int nq = r_stride / 16;
  kern_t kern;
  if (ring) {
    const int nqt_max = nq <= 1 ? 1 : nq <= 2 ? 2 : nq <= 4 ? 4 : 8;
    lds = (size_t)SR_NS * (rows * 128 + nqt_max * 16 * 128);
#define SR_PICK(F_, R_) (nq <= 1 ? shrink_ring_kernel<F_, 1, R_> : nq <= 2 ? shrink_ring_kernel<F_, 2, R_> \
                         : nq <= 4 ? shrink_ring_kernel<F_, 4, R_> : shrink_ring_kernel<F_, 8, R_>)
    if (lora_form == FORM_NT) kern = long_seg ? SR_PICK(FORM_NT, 2) : SR_PICK(FORM_NT, 1);
    else kern = long_seg ? SR_PICK(FORM_NN, 2) : SR_PICK(FORM_NN, 1);
#undef SR_PICK
    hipError_t e = allow_big_lds((const void*)kern, 16 + (long_seg ? 0 : 8) + (lora_form == FORM_NT ? 0 : 4) + (nq <= 1 ? 0 : nq <= 2 ? 1 : nq <= 4 ? 2 : 3));
    if (e != hipSuccess) return e;
  } else if (lora_form == FORM_NT)
    kern = nq <= 1 ? shrink_bf16_kernel<FORM_NT, 1> : nq <= 2 ? shrink_bf16_kernel<FORM_NT, 2>
         : nq <= 4 ? shrink_bf16_kernel<FORM_NT, 4> : shrink_bf16_kernel<FORM_NT, 8>;
  else
    kern = nq <= 1 ? shrink_bf16_kernel<FORM_NN, 1> : nq <= 2 ? shrink_bf16_kernel<FORM_NN, 2>
         : nq <= 4 ? shrink_bf16_kernel<FORM_NN, 4> : shrink_bf16_kernel<FORM_NN, 8>;
  if (!ring && lds > 64 * 1024) {
    hipError_t e = allow_big_lds((const void*)kern, (lora_form == FORM_NT ? 0 : 4) + (nq <= 1 ? 0 : nq <= 2 ? 1 : nq <= 4 ? 2 : 3));
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kern, dim3(rb_max * ksplit, n_adapters), dim3(SH_THREADS), lds, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || ksplit == 1) return e;
  hipLaunchKernelGGL(shrink_finalize_kernel, dim3((max_seg + 15) / 16, n_adapters), dim3(256), 0, stream, a);
  return hipGetLastError();
}

// ============================================================== reduce
static constexpr int RD_THREADS = 256;
static constexpr int RD_COLS = 256;    // columns of X per block (64 per wave)
static constexpr int RD_TOK = 64;      // tokens staged per step

struct ReduceArgs {
  const bf16_t* X; int64_t ldx; int64_t C;
  const int32_t* perm; const int32_t* seg_off;
  const AdapterEntry* table; const GradEntry* grads; int which;   // 0: write dA, 1: write dB
  const float* V; int r_stride;
  int accumulate;
  int slabs; int tchunk; int chunks_max;   // tchunk multiple of RD_TOK
  const int32_t* order;                    // blockIdx.y -> adapter (longest segment first), or null
  // ragged = 1: only segments longer than tchunk are cut; adapter t's pieces use partial-sum slots
  // chunk_base[t] .. ([slot][C][r_stride]), every other adapter's block writes its result itself
  int ragged; const int32_t* chunk_base;
  float* partials;                         // [adapter][chunk][C][r_stride] when to_partials
  int to_partials;                         // 1: the chunks' sums go to `partials`, reduce_finalize_kernel completes
  ReduceOpt opt;                           // (finalize) optimizer step on every completed gradient element
};

// LDS byte offset of 16-byte unit `unit` (of 32) of token row `tk` in the [64][256] X tile.
__device__ __forceinline__ int swz_tokc(int tk, int unit) {
  const int f = (tk & 3) | (((tk >> 3) & 1) << 2);
  return tk * 512 + ((unit ^ (f << 1)) << 4);
}

// grid: x = slabs * chunks_max, y = adapter.  The kernel is bound by the one pass over X, so the
// loop is software-pipelined through registers: while a 64-token step is multiplied out of LDS,
// the X rows and V rows of the next step are already requested (and the gather indices of the
// step after that), and only the LDS hand-over sits between two barriers.
template <int OFORM, int NQT>
__global__ __launch_bounds__(RD_THREADS, NQT >= 8 ? 1 : 2) void reduce_bf16_kernel(ReduceArgs a) {
  extern __shared__ __attribute__((aligned(16))) char rsm[];
  char* Xs = rsm;                               // [RD_TOK][RD_COLS] bf16, swizzled
  char* Vh = rsm + RD_TOK * RD_COLS * 2;        // [RD_TOK][r_pad] bf16: leading halves of V
  const int t = a.order ? a.order[blockIdx.y] : blockIdx.y;
  const int slab = blockIdx.x % a.slabs, ch = blockIdx.x / a.slabs;
  const int lo = a.seg_off[t], hi = a.seg_off[t + 1];
  const int beg = lo + ch * a.tchunk;
  const bool empty = beg >= hi;
  const int nch_t = (hi - lo + a.tchunk - 1) / a.tchunk;                    // token chunks of this adapter
  if (empty && !(ch == 0 && (a.chunks_max == 1 || a.ragged) && !a.accumulate)) return;  // empty adapter: write zeros
  const int end = (beg + a.tchunk) < hi ? (beg + a.tchunk) : hi;
  const AdapterEntry e = a.table[t];
  const int r = e.rank, r_pad = (r + 15) & ~15, nqt = r_pad >> 4;
  const int vpitch = r_pad * 2 + 16;            // bytes per token row of a V tile
  char* Vl = Vh + RD_TOK * vpitch;              // trailing halves (v - bf16(v))
  const int64_t c0 = (int64_t)slab * RD_COLS;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4, li = lane & 15;
  f32x4 acc[4][NQT];
  for (int i = 0; i < 4; ++i)
    for (int q = 0; q < NQT; ++q) acc[i][q] = f32x4{0.f, 0.f, 0.f, 0.f};
  const uint4 zero4 = make_uint4(0, 0, 0, 0);
  const int xu = tid & 31, xr = tid >> 5;     // X loader: unit along c, token row (+8 per pass)
  const bool col_ok = (c0 + xu * 8) < a.C;
  const int vper = r_pad >> 2;                // float4 per V row (first r_pad ranks only)

  int tokn[8];                                // gather indices of the step after the requested one
  uint4 xv[8];
  float4 vv[NQT];
  auto load_tok = [&](int s) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int m = s + xr + 8 * i;
      tokn[i] = m < end ? (a.perm ? a.perm[m] : m) : -1;
    }
  };
  auto load_step = [&](int s) {               // uses tokn (already arrived)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      xv[i] = zero4;
      if (tokn[i] >= 0 && col_ok) xv[i] = *(const uint4*)(a.X + (int64_t)tokn[i] * a.ldx + c0 + xu * 8);
    }
#pragma unroll
    for (int i = 0; i < NQT; ++i) {
      vv[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (i < nqt) {
        const int f = tid + RD_THREADS * i;   // 64 * vper = 256 * nqt of them
        const int row = f / vper, c4 = f - row * vper;
        if (s + row < end) vv[i] = *(const float4*)(a.V + (int64_t)(s + row) * a.r_stride + c4 * 4);
      }
    }
  };
  if (!empty) {
    load_tok(beg);
    load_step(beg);
    load_tok(beg + RD_TOK);
  }
  for (int s = beg; s < end; s += RD_TOK) {
    __syncthreads();                          // the previous step's fragments have been read
#pragma unroll
    for (int i = 0; i < 8; ++i) *(uint4*)(Xs + swz_tokc(xr + 8 * i, xu)) = xv[i];
#pragma unroll
    for (int i = 0; i < NQT; ++i)
      if (i < nqt) {
        const int f = tid + RD_THREADS * i;
        const int row = f / vper, c4 = f - row * vper;
        const float fv[4] = {vv[i].x, vv[i].y, vv[i].z, vv[i].w};
        bf16_t h[4], l[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float x = (c4 * 4 + j) < r ? fv[j] : 0.f;     // ranks beyond r are padding of the row
          h[j] = float_to_bf16_bits(x);
          l[j] = float_to_bf16_bits(x - bf16_bits_to_float(h[j]));
        }
        *(uint2*)(Vh + row * vpitch + c4 * 8) = make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
        *(uint2*)(Vl + row * vpitch + c4 * 8) = make_uint2(l[0] | ((uint32_t)l[1] << 16), l[2] | ((uint32_t)l[3] << 16));
      }
    __syncthreads();
    if (s + RD_TOK < end) {                   // next step's rows, and the indices of the one after
      load_step(s + RD_TOK);
      load_tok(s + 2 * RD_TOK);
    }
#pragma unroll
    for (int kstep = 0; kstep < 2; ++kstep) {
      typedef short4v __attribute__((address_space(3))) * lds_s4;
      // a 16-lane group g needs tokens kstep*32 + g*8 + 0..7; within it lane li addresses 4
      // consecutive columns of token row (li >> 2) and receives 4 consecutive tokens of one column
      const int tk = kstep * 32 + g * 8 + (li >> 2);
      bf16x8 xa[4];
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) {
        const int col = wave * 64 + ct * 16 + 4 * (li & 3);
        short4v p0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(Xs + swz_tokc(tk, col >> 3) + (col & 7) * 2));
        short4v p1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(Xs + swz_tokc(tk + 4, col >> 3) + (col & 7) * 2));
        union { short s[8]; bf16x8 v; } u;
        u.s[0] = p0[0]; u.s[1] = p0[1]; u.s[2] = p0[2]; u.s[3] = p0[3];
        u.s[4] = p1[0]; u.s[5] = p1[1]; u.s[6] = p1[2]; u.s[7] = p1[3];
        xa[ct] = u.v;
      }
#pragma unroll
      for (int qt = 0; qt < NQT; ++qt)
        if (qt < nqt) {
          const int voff = tk * vpitch + (qt * 16 + 4 * (li & 3)) * 2;
          bf16x8 vh, vl;
          {
            short4v p0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(Vh + voff));
            short4v p1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(Vh + voff + 4 * vpitch));
            union { short s[8]; bf16x8 v; } u;
            u.s[0] = p0[0]; u.s[1] = p0[1]; u.s[2] = p0[2]; u.s[3] = p0[3];
            u.s[4] = p1[0]; u.s[5] = p1[1]; u.s[6] = p1[2]; u.s[7] = p1[3];
            vh = u.v;
          }
          {
            short4v p0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(Vl + voff));
            short4v p1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(Vl + voff + 4 * vpitch));
            union { short s[8]; bf16x8 v; } u;
            u.s[0] = p0[0]; u.s[1] = p0[1]; u.s[2] = p0[2]; u.s[3] = p0[3];
            u.s[4] = p1[0]; u.s[5] = p1[1]; u.s[6] = p1[2]; u.s[7] = p1[3];
            vl = u.v;
          }
#pragma unroll
          for (int ct = 0; ct < 4; ++ct) {
            acc[ct][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa[ct], vh, acc[ct][qt], 0, 0, 0);
            acc[ct][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa[ct], vl, acc[ct][qt], 0, 0, 0);
          }
        }
    }
  }
  // D layout: row (column c of X) = 4 * (lane / 16) + v, column (q) = lane % 16
  const bool via_part = a.ragged ? nch_t > 1 : a.to_partials != 0;
  float* outp = via_part ? nullptr : (a.which ? a.grads[t].dB : a.grads[t].dA);
  float* part = !via_part ? nullptr
                : a.partials + (a.ragged ? (int64_t)a.chunk_base[t] + ch : (int64_t)t * a.chunks_max + ch) * a.C * a.r_stride;
#pragma unroll
  for (int ct = 0; ct < 4; ++ct)
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt)
      if (qt < nqt)
        for (int v = 0; v < 4; ++v) {
          const int64_t c = c0 + wave * 64 + ct * 16 + 4 * g + v;
          const int q = qt * 16 + li;
          if (c < a.C && q < r) {
            if (part) {
              part[c * a.r_stride + q] = acc[ct][qt][v];
            } else {
              float* o = outp + (OFORM == FORM_NN ? c * r + q : (int64_t)q * a.C + c);
              *o = a.accumulate ? *o + acc[ct][qt][v] : acc[ct][qt][v];
            }
          }
        }
}

// out_t (+)= sum over the chunks of adapter t, in chunk order.  With an optimizer step attached
// (a.opt.on) the completed gradient element is consumed on the spot instead: one AdamW update
// (Adam with decoupled weight decay; the policy update of the task being trained, paper Sec. 4.2
// and Alg. 1, whose optimizer state is kept per task) of the fp32 master value and its two
// moments, and the bf16 value of the next version of the factor.  Adapters without tokens in the
// batch are not trained by it and are left alone.
template <int OFORM>
__global__ __launch_bounds__(256) void reduce_finalize_kernel(ReduceArgs a) {
  // block = 32 columns x 32 rank indices of one adapter.  The chunks' sums are read with the rank
  // index fastest (their storage order) and handed over through LDS, so that the gradient and the
  // optimizer state are touched in THEIR storage order: rank fastest for [C, r] outputs, column
  // fastest for [r, C] outputs.
  __shared__ float tile[32][33];
  // (ragged: the grid covers the adapters that are cut, the longest ones, first in `order`)
  const int t = a.ragged ? a.order[blockIdx.y] : blockIdx.y;
  const AdapterEntry e = a.table[t];
  const int r = e.rank;
  const int qtiles = (a.r_stride + 31) / 32;
  const int64_t c0 = (int64_t)(blockIdx.x / qtiles) * 32;
  const int q0 = (int)(blockIdx.x % qtiles) * 32;
  if (q0 >= r) return;
  const int len = a.seg_off[t + 1] - a.seg_off[t];
  if (a.opt.on && len == 0) return;
  const int nch = (len + a.tchunk - 1) / a.tchunk;
  if (a.ragged && nch <= 1) return;      // (written by its one block)
  const int64_t slot0 = a.ragged ? (int64_t)a.chunk_base[t] : (int64_t)t * a.chunks_max;
  for (int i = threadIdx.x; i < 1024; i += 256) {
    const int cc = i >> 5, qq = i & 31;
    const int64_t c = c0 + cc;
    const int q = q0 + qq;
    float sum = 0.f;
    if (c < a.C && q < r)
      for (int ch = 0; ch < nch; ++ch)
        sum += a.partials[((slot0 + ch) * a.C + c) * a.r_stride + q];
    tile[cc][qq] = sum;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 1024; i += 256) {
    const int cc = OFORM == FORM_NN ? i >> 5 : i & 31, qq = OFORM == FORM_NN ? i & 31 : i >> 5;
    const int64_t c = c0 + cc;
    const int q = q0 + qq;
    if (c >= a.C || q >= r) continue;
    const float sum = tile[cc][qq];
    const int64_t off = OFORM == FORM_NN ? c * r + q : (int64_t)q * a.C + c;
    if (a.opt.on) {
      const OptFactor f = a.opt.f[t];
      float p = f.master[off];
      p -= a.opt.lr * a.opt.wd * p;
      const float m = a.opt.beta1 * f.m[off] + (1.f - a.opt.beta1) * sum;
      const float v = a.opt.beta2 * f.v[off] + (1.f - a.opt.beta2) * sum * sum;
      p -= a.opt.lr * (m * a.opt.inv_c1) / (sqrtf(v * a.opt.inv_c2) + a.opt.eps);
      f.master[off] = p; f.m[off] = m; f.v[off] = v;
      f.out[off] = float_to_bf16_bits(p);
    } else {
      float* o = (a.which ? a.grads[t].dB : a.grads[t].dA) + off;
      *o = a.accumulate ? *o + sum : sum;
    }
  }
}

static void reduce_plan(int64_t C, int n_adapters, int max_seg, int* tchunk, int* chunks_max) {
  const int slabs = (int)((C + RD_COLS - 1) / RD_COLS);
  const int64_t base = (int64_t)slabs * n_adapters;
  *tchunk = ((max_seg + RD_TOK - 1) / RD_TOK) * RD_TOK;
  *chunks_max = 1;
  if (*tchunk < RD_TOK) *tchunk = RD_TOK;
  if (base < 256 && max_seg > 1024) {
    int want = (int)((512 + base - 1) / base);
    int tc = (max_seg + want - 1) / want;
    if (tc < 512) tc = 512;
    tc = ((tc + RD_TOK - 1) / RD_TOK) * RD_TOK;
    *tchunk = tc;
    *chunks_max = (max_seg + tc - 1) / tc;
  }
}

// Very unequal segments with enough blocks in all: cut only the long ones (see reduce_ragged_chunk).
static bool reduce_ragged(int64_t C, int n_adapters, int max_seg, int ragged_chunk, int ragged_slots) {
  const int slabs = (int)((C + RD_COLS - 1) / RD_COLS);
  return (int64_t)slabs * n_adapters >= 256 && ragged_slots > 0 && ragged_chunk > 0 && max_seg > 2 * ragged_chunk;
}

size_t reduce_partial_bytes(int64_t C, int n_adapters, int max_seg, int r_stride, bool always, int ragged_chunk,
                            int ragged_slots) {
  int tc, cm;
  reduce_plan(C, n_adapters, max_seg, &tc, &cm);
  size_t need = (cm <= 1 && !always) ? 0 : (size_t)n_adapters * cm * C * r_stride * sizeof(float);
  if (reduce_ragged(C, n_adapters, max_seg, ragged_chunk, ragged_slots)) {
    const size_t rg = (size_t)ragged_slots * C * r_stride * sizeof(float);
    if (rg > need) need = rg;
  }
  return need;
}

hipError_t launch_reduce_bf16(const bf16_t* X, int64_t ldx, int64_t C, const int32_t* perm,
                              const int32_t* seg_off, int n_adapters, int max_seg,
                              const AdapterEntry* table, const GradEntry* grads, int which,
                              int out_form, const float* V, int r_stride, int accumulate,
                              float* partials, size_t partial_bytes, const ReduceOpt* opt, const int32_t* order,
                              const int32_t* chunk_base, int ragged_chunk, int ragged_slots, int ragged_adapters,
                              hipStream_t stream) {
  if (n_adapters <= 0) return hipSuccess;
  ReduceArgs a;
  a.order = order;
  a.ragged = 0; a.chunk_base = nullptr;
  a.X = X; a.ldx = ldx; a.C = C; a.perm = perm; a.seg_off = seg_off; a.table = table;
  a.grads = grads; a.which = which; a.V = V; a.r_stride = r_stride; a.accumulate = accumulate;
  a.slabs = (int)((C + RD_COLS - 1) / RD_COLS);
  reduce_plan(C, n_adapters, max_seg, &a.tchunk, &a.chunks_max);
  if (a.chunks_max > 1 &&
      (partials == nullptr || partial_bytes < (size_t)n_adapters * a.chunks_max * C * r_stride * sizeof(float))) {
    a.chunks_max = 1;   // no room for partial sums: one block walks the whole segment
    a.tchunk = ((max_seg + RD_TOK - 1) / RD_TOK) * RD_TOK;
    if (a.tchunk < RD_TOK) a.tchunk = RD_TOK;
  }
  a.partials = partials;
  a.to_partials = a.chunks_max > 1;
  if (!(opt && opt->on) && a.chunks_max == 1 && chunk_base != nullptr && order != nullptr && partials != nullptr &&
      ragged_adapters > 0 && ragged_adapters <= n_adapters &&
      reduce_ragged(C, n_adapters, max_seg, ragged_chunk, ragged_slots) &&
      partial_bytes >= (size_t)ragged_slots * C * r_stride * sizeof(float)) {
    a.ragged = 1; a.chunk_base = chunk_base;
    a.tchunk = ragged_chunk;
    a.chunks_max = (max_seg + ragged_chunk - 1) / ragged_chunk;
    a.to_partials = 1;               // (the finalize kernel runs; it skips the adapters with one piece)
  }
  a.opt.on = 0;
  if (opt && opt->on) {
    // the optimizer step lives in the finalize kernel: the sums always go through `partials`
    if (n_adapters > OPT_MAX_ADAPTERS || partials == nullptr ||
        partial_bytes < (size_t)n_adapters * a.chunks_max * C * r_stride * sizeof(float))
      return hipErrorInvalidValue;
    a.opt = *opt;
    a.to_partials = 1;
  }
  const size_t lds = (size_t)RD_TOK * RD_COLS * 2 + (size_t)2 * RD_TOK * (r_stride * 2 + 16);   // r_stride >= every r_pad
  typedef void (*rkern_t)(ReduceArgs);
  const int nq = r_stride / 16;
  rkern_t kern;
  if (out_form == FORM_NN)
    kern = nq <= 1 ? reduce_bf16_kernel<FORM_NN, 1> : nq <= 2 ? reduce_bf16_kernel<FORM_NN, 2>
         : nq <= 4 ? reduce_bf16_kernel<FORM_NN, 4> : reduce_bf16_kernel<FORM_NN, 8>;
  else
    kern = nq <= 1 ? reduce_bf16_kernel<FORM_NT, 1> : nq <= 2 ? reduce_bf16_kernel<FORM_NT, 2>
         : nq <= 4 ? reduce_bf16_kernel<FORM_NT, 4> : reduce_bf16_kernel<FORM_NT, 8>;
  if (lds > 64 * 1024) {
    hipError_t e = allow_big_lds((const void*)kern, 8 + (out_form == FORM_NT ? 0 : 4) + (nq <= 1 ? 0 : nq <= 2 ? 1 : nq <= 4 ? 2 : 3));
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kern, dim3(a.slabs * a.chunks_max, n_adapters), dim3(RD_THREADS), lds, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (a.to_partials) {
    auto fin = out_form == FORM_NN ? reduce_finalize_kernel<FORM_NN> : reduce_finalize_kernel<FORM_NT>;
    hipLaunchKernelGGL(fin, dim3((unsigned)(((C + 31) / 32) * ((r_stride + 31) / 32)), a.ragged ? ragged_adapters : n_adapters),
                       dim3(256), 0, stream, a);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace marlaas
