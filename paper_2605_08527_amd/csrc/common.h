// Shared declarations of the HIP library (host + device side).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace marlaas {

typedef uint16_t bf16_t;  // raw bf16 bit pattern

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short short4v;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

// One adapter as the kernels see it.  `lora_in` multiplies the layer input
// (A_t in forward, B_t in backward), `lora_out` produces the layer output
// (B_t in forward, A_t in backward); both are dense, orientation given by the
// kernel's template form.
struct AdapterEntry {
  const void* A;
  const void* B;
  int32_t rank;
  float scale;
};

struct GradEntry {
  float* dA;
  float* dB;
};

// Up to ROW_CHUNK consecutive rows of the grouped token order that belong to one adapter
// (t = -1: rows without an adapter).  The chunks of a segment map cover every row once.
static constexpr int ROW_CHUNK = 8;
struct RowChunk {
  int32_t row0, nrows, t, pad;
};

// Extended column e of the fused shrink: rank q of adapter entry t (e = rank offset of t + q), with
// that entry's factor pointers copied in, so that a kernel finds its source row with one load.
struct ExtCol {
  const void* A;
  const void* B;
  int32_t t, q;
  float scale;      // of entry t
  int32_t pad;
};

// One projection of a fused multi-projection forward (small batches): its weight, its output and
// where it sits in the concatenated column space (each projection padded to whole column tiles).
// The entries of a call travel inside the kernel arguments (no device copy).
struct ProjEntry {
  const void* W; int64_t ldw;     // weight operand, stored in the call's form
  int64_t Nout;                   // output columns of this projection
  void* out; int64_t ldo;
  int32_t tile0;                  // first column tile (128 wide) in the concatenated space
  int32_t fin0;                   // first column chunk (512 wide) of the finish kernel's grid
  int32_t tab0;                   // index of this projection's first adapter in the combined table
  int32_t pad;
};
static constexpr int MAX_PROJ = 8;

// The per-adapter tables of one call as the kernels read them, all in device memory.  They live
// either in an adapter table object (written when an adapter is registered or swapped) or in a
// slice of the caller's workspace (written at the start of the call); the passes only read them.
//   entries[i], grads[i] : i = projection * n_adapters + adapter
//   roff[i]              : sum of the ranks of entries 0 .. i - 1 (P + 1 values, P = entries)
//   cols[e]              : (factor pointers, entry, rank index) of extended column e, for e < min(roff[P], ext_cap)
struct DevTables {
  AdapterEntry* entries = nullptr;
  GradEntry* grads = nullptr;
  int32_t* roff = nullptr;
  ExtCol* cols = nullptr;
  int32_t ext_cap = 0;
};
// Bytes of one DevTables block for P entries and ext_cap extended columns, and its carving.
size_t dev_tables_bytes(int64_t P, int64_t ext_cap);
DevTables dev_tables_carve(void* base, int64_t P, int64_t ext_cap);
// Enqueue: entries[first .. first + count) = host values (by-value kernel arguments, no copy node).
hipError_t enqueue_write_entries(const DevTables& d, int64_t first, int64_t count, const AdapterEntry* host,
                                 hipStream_t stream);
hipError_t enqueue_write_grads(const DevTables& d, int64_t first, int64_t count, const GradEntry* host,
                               hipStream_t stream);
// Enqueue: roff and cols recomputed from entries[0 .. P) (after any change of a rank or a pointer).
hipError_t enqueue_derive(const DevTables& d, int64_t P, hipStream_t stream);

// How a [contraction, output] operand is stored.
//   FORM_NT: element (k, n) at ptr[n * ld + k]   (contraction index contiguous)
//   FORM_NN: element (k, n) at ptr[k * ld + n]   (output index contiguous)
enum { FORM_NT = 0, FORM_NN = 1 };

__device__ __forceinline__ float bf16_bits_to_float(bf16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}
// round to nearest even (the hardware conversion of gfx950)
__device__ __forceinline__ bf16_t float_to_bf16_bits(float f) {
  const __bf16 h = (__bf16)f;
  return __builtin_bit_cast(bf16_t, h);
}

// Segment t of the grouped token order is [seg_off[t], seg_off[t+1]).
// Largest t in [0, n] with seg_off[t] <= m (seg_off has n + 2 entries, last = T).
__device__ __forceinline__ int segment_of(const int32_t* __restrict__ seg_off, int n, int m) {
  int lo = 0, hi = n + 1;  // invariant: seg_off[lo] <= m < seg_off[hi]
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (seg_off[mid] <= m) lo = mid; else hi = mid;
  }
  return lo;
}

// ---- launchers (implemented in the .hip files; all enqueue on `stream`) ----

struct SegmapDev {
  int32_t* perm;      // [T] or nullptr when the grouped order is the identity
  int32_t* seg_off;   // [n + 2]
};

// perm[m] = token of grouped row m, grp_ids[m] = its adapter (-1: none)
hipError_t launch_segmap(const int32_t* ids, int64_t T, int n, int32_t* perm, int32_t* grp_ids, int32_t* seg_off,
                         int32_t* block_hist, int32_t* flags, RowChunk* chunks, int32_t* order, int32_t* chunk_base,
                         hipStream_t stream);
// Token chunk of the weight-gradient reductions for batches whose segments are very unequal: a
// segment longer than this is cut into pieces of this many rows (twice the mean segment, at least
// 512, a multiple of 64), each piece a block of its own; chunk_base[t] (segment map) is the first
// partial-sum slot of adapter t's pieces, counting only adapters with more than one piece.
__host__ __device__ inline int reduce_ragged_chunk(int64_t T_lora, int n) {
  int64_t c = n > 0 ? 2 * T_lora / n : 0;
  if (c < 512) c = 512;
  return (int)((c + 63) / 64 * 64);
}
int segmap_blocks(int64_t T);
// Row chunks of a grouped order with these segment offsets (n + 2 entries): how many there are.
int64_t segmap_chunk_count(const int32_t* seg_off, int n);
// Upper bound of that count for any map of T tokens and n adapters.
int64_t segmap_chunk_bound(int64_t T, int n);

// u[m, 0..r_stride) = scale_t * sum_c X[perm[m], c] * L_t(c, q), grouped order m.
// which = 0 uses AdapterEntry::A as L_t, 1 uses ::B.  lora_form: FORM_NN when
// L_t is stored [C, r_t] (q contiguous), FORM_NT when stored [r_t, C].
hipError_t launch_shrink_bf16(const bf16_t* X, int64_t ldx, int64_t C, const int32_t* perm,
                              const int32_t* seg_off, int n_adapters, int max_seg,
                              const AdapterEntry* table, int which, int lora_form, float* u,
                              int r_stride, int64_t T_lora, float* partials, size_t partial_bytes,
                              bf16_t* u2, bool* wrote_u2, const bf16_t* zero_line, bool ranks_mult8, hipStream_t stream);
// scratch for the sums of a shrink whose contraction is split (0: it is not)
size_t shrink_partial_bytes(int64_t C, int64_t T_lora, int n_adapters, int r_stride);

// How the decode kernel's call gets finished (splits added, expand added, rows rounded and
// scattered), and what the ways other than the generic finish kernel need: the adapter of every
// grouped row; for the in-kernel way also zeroed device counters that stay zero between launches
// and the bounds of its one wait.
enum { DECODE_FINISH_GENERIC = 0,    // splitk_finish_kernel on fp32 rows (any split count)
       DECODE_FINISH_IN_KERNEL = 1,  // the decode kernel itself: one launch
       DECODE_FINISH_LAUNCH = 2,     // a second launch of the decode kernel's own finish
       DECODE_FINISH_AUTO = 3 };     // whichever of the two is faster for the split count
struct DecodeSync {
  int mode = DECODE_FINISH_GENERIC;  // the way asked for; the launcher falls back to the generic one
  int32_t* counters = nullptr;       // at least DECODE_SYNC_INTS
  const int32_t* grp_ids = nullptr;
  int spin_limit = 0;
  int cu_count = 0;
};
static constexpr int DECODE_SYNC_INTS = 4096;

// What lets the large-batch GEMM fetch the expand's operands by DMA: u (or v) as a two-term bf16
// split written by the shrink, scratch for the row tiles' lists of extra contraction tiles
// (lora_tiles_bytes(T) bytes), 16 zero bytes in device memory, and whether every rank is a
// multiple of 8.
struct LoraDma {
  const bf16_t* u2 = nullptr;
  int32_t* tiles = nullptr; size_t tiles_bytes = 0;
  const bf16_t* zero_line = nullptr;
  bool ranks_mult8 = false;
};
size_t lora_tiles_bytes(int64_t T);

struct GemmFuse {
  const ExtCol* cols;      // [n_ext] device
  const int32_t* roff;     // [n_adapters + 1] device: rank offsets
  int n_ext;               // sum of the ranks
  bool ranks_mult8;        // every rank is a multiple of 8
  float* u_out;            // [T][r_stride] device: receives scale_t * (X L_t) per grouped row
  // `cols` and `roff` may point into the tables of a larger adapter bank: ExtCol::t then counts
  // the bank's entries and t0 is the entry index of the call's table[0]; roff values are offsets
  // in the bank's extended-column space and ext_base is the call's first one (roff of table[0]).
  int t0 = 0, ext_base = 0;
};

// out[perm[m], :] = Aop[perm[m], :] * Bop + (m in segment t) U[m, :] * L_t
hipError_t launch_gemm_bf16(const bf16_t* Aop, int64_t lda, const bf16_t* Bop, int64_t ldb,
                            int form, int64_t T, int64_t Kc, int64_t Nout, const int32_t* perm,
                            const int32_t* seg_off, int n_adapters, const AdapterEntry* table,
                            int which, const float* U, int r_stride, void* out, int64_t ldo,
                            int out_is_f32, float* partials, size_t partial_bytes, const RowChunk* chunks,
                            int n_chunks, const GemmFuse* fuse, bf16_t* wt_scratch, size_t wt_bytes, const bf16_t* Bt_kept, const LoraDma* dma,
                            const bf16_t* Bpacked, const DecodeSync* sync, hipStream_t stream);
// (Bpacked: optional packed copy of Bop for this contraction, used by small batches; with it the
// shrink is only fused when the adapters' factors are stored contraction-contiguous, which the
// caller says by passing fuse only then.)
// Several projections of the same input in one pass (small batches only: 128 x 128 tiles with
// the shrink carried as extended columns, or no adapters at all).  `proj_host` holds the n_proj
// entries (host memory); `table` is the combined adapter table ([projection][adapter]), `fuse` (null:
// no adapters) the combined extended-column tables, ExtCol::t indexing the combined table.  The
// projection entries travel in the kernel arguments.
// gemm_multi_ok tells whether the sizes qualify; otherwise the caller runs the projections one by one.
bool gemm_multi_ok(int form, int64_t T, int64_t Kc, const ProjEntry* proj_host, int n_proj, int n_ext,
                   bool ranks_mult8, size_t partial_bytes);
size_t gemm_multi_bytes(int64_t T, int64_t Kc, const ProjEntry* proj_host, int n_proj, int n_ext);
hipError_t launch_gemm_bf16_multi(const bf16_t* Aop, int64_t lda, int form, int64_t T, int64_t Kc,
                                  const int32_t* perm, const int32_t* seg_off, int n_adapters,
                                  const AdapterEntry* table, const ProjEntry* proj_host,
                                  int n_proj, int out_is_f32, float* partials,
                                  size_t partial_bytes, const RowChunk* chunks, int n_chunks,
                                  const GemmFuse* fuse, int packed, const DecodeSync* sync, int r_stride,
                                  hipStream_t stream);
// Packed copy of a [contraction C, output O] operand for the decode kernel, in MFMA fragment order
// (16 output columns x 32 contraction values per kilobyte, zero beyond the matrix).  Element (c, o)
// of the source is at src[c * sc + o * so].
size_t packed_weight_bytes(int64_t C, int64_t O);
int64_t packed_weight_ksteps(int64_t C);
hipError_t launch_pack_weight(const bf16_t* src, int64_t sc, int64_t so, int64_t C, int64_t O, bf16_t* dst,
                              hipStream_t stream);
// Scratch for a transposed copy of the weight: a large batch whose weight is stored
// [contraction][output] runs faster on a [output][contraction] copy made per call (the copy
// costs two passes over the weight, the GEMM gains about a quarter).  0: not used for these sizes.
size_t gemm_wt_bytes(int form, int64_t T, int64_t Kc, int64_t Nout);
// dst[c][r] = src[r][c], bf16, R x C (both multiples of 8)
hipError_t launch_transpose_bf16(const bf16_t* src, int64_t lds, bf16_t* dst, int64_t ldd, int64_t R, int64_t C, hipStream_t stream);
// scratch for partial sums; n_ext = sum of the adapter ranks (0: no adapters)
size_t gemm_splitk_bytes(int64_t T, int64_t Kc, int64_t Nout, int n_ext);
// Small batches: the GEMM can compute the shrink itself (as extra output columns over every
// adapter's factor; the finish kernel keeps each row's own adapter).  When this holds the caller
// skips the shrink launch and passes a GemmFuse; U is then ignored and u_out receives u.
bool gemm_can_fuse_shrink(int form, int64_t T, int64_t Kc, int64_t Nout, int n_ext, bool ranks_mult8,
                          size_t partial_bytes);

// out_t(c, q) (+)= sum_{m in seg t} X[perm[m], c] * V[m, q]
// out_form FORM_NN: out_t[c * r_t + q]; FORM_NT: out_t[q * C + c].
// Optimizer step applied where a gradient element is completed (AdamW; see lora_small.hip):
// per adapter the fp32 master copy, the two moments and the bf16 output of the factor the
// reduction produces the gradient of.  on = 0: gradients are written as usual.
struct OptFactor { float* master; float* m; float* v; bf16_t* out; };
static constexpr int OPT_MAX_ADAPTERS = 8;
struct ReduceOpt {
  int on;
  float lr, beta1, beta2, eps, wd, inv_c1, inv_c2;   // inv_c: 1 / (1 - beta^step)
  OptFactor f[OPT_MAX_ADAPTERS];
};
hipError_t launch_reduce_bf16(const bf16_t* X, int64_t ldx, int64_t C, const int32_t* perm,
                              const int32_t* seg_off, int n_adapters, int max_seg,
                              const AdapterEntry* table, const GradEntry* grads, int which,
                              int out_form, const float* V, int r_stride, int accumulate,
                              float* partials, size_t partial_bytes, const ReduceOpt* opt, const int32_t* order,
                              const int32_t* chunk_base, int ragged_chunk, int ragged_slots, int ragged_adapters,
                              hipStream_t stream);
size_t reduce_partial_bytes(int64_t C, int n_adapters, int max_seg, int max_rank, bool always = false,
                            int ragged_chunk = 0, int ragged_slots = 0);

// fp32 path (plain ALU arithmetic, any shape)
hipError_t launch_shrink_f32(const float* X, int64_t ldx, int64_t C, const int32_t* perm,
                             const int32_t* seg_off, int n_adapters, const AdapterEntry* table,
                             int which, int lora_form, float* u, int r_stride, int64_t T_lora,
                             hipStream_t stream);
hipError_t launch_gemm_f32(const float* Aop, int64_t lda, const float* Bop, int64_t ldb, int form,
                           int64_t T, int64_t Kc, int64_t Nout, const int32_t* perm,
                           const int32_t* seg_off, int n_adapters, const AdapterEntry* table,
                           int which, const float* U, int r_stride, void* out, int64_t ldo,
                           int out_is_f32, hipStream_t stream);
hipError_t launch_reduce_f32(const float* X, int64_t ldx, int64_t C, const int32_t* perm,
                             const int32_t* seg_off, int n_adapters, const AdapterEntry* table,
                             const GradEntry* grads, int which, int out_form, const float* V,
                             int r_stride, int accumulate, hipStream_t stream);

}  // namespace marlaas
