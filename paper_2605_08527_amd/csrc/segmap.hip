// Token grouping by adapter: a stable counting sort in three small kernels.
// The mixed-tenant batch carries one adapter id per token (paper Sec. 4.5,
// cross-task batching of rollouts); every later kernel works on tokens grouped
// by adapter, so this map is built once per batch and reused by all layers.
#include "common.h"

namespace marlaas {

static constexpr int SEG_THREADS = 256;
static constexpr int SEG_CHUNK = 2048;  // tokens per block

int segmap_blocks(int64_t T) { return (int)((T + SEG_CHUNK - 1) / SEG_CHUNK); }

// bucket n collects tokens with id -1; flags[0] |= 1 on an id outside [-1, n),
// flags[1] |= 1 when the ids are not already grouped in bucket order.
__global__ __launch_bounds__(SEG_THREADS) void segmap_hist(const int32_t* __restrict__ ids,
                                                           int64_t T, int n,
                                                           int32_t* __restrict__ block_hist,
                                                           int32_t* __restrict__ flags) {
  extern __shared__ int32_t hist[];
  for (int b = threadIdx.x; b <= n; b += SEG_THREADS) hist[b] = 0;
  __syncthreads();
  int64_t base = (int64_t)blockIdx.x * SEG_CHUNK;
  bool bad = false, unsorted = false;
  for (int j = threadIdx.x; j < SEG_CHUNK; j += SEG_THREADS) {
    int64_t i = base + j;
    if (i >= T) break;
    int id = ids[i];
    if (id < -1 || id >= n) { bad = true; continue; }
    int b = id < 0 ? n : id;
    atomicAdd(&hist[b], 1);
    if (i + 1 < T) {
      int nx = ids[i + 1];
      int bn = nx < 0 ? n : nx;
      if (bn < b) unsorted = true;
    }
  }
  if (bad) atomicOr(&flags[0], 1);
  if (unsorted) atomicOr(&flags[1], 1);
  __syncthreads();
  for (int b = threadIdx.x; b <= n; b += SEG_THREADS)
    block_hist[(int64_t)blockIdx.x * (n + 1) + b] = hist[b];
}

// One block.  seg_off[b] = exclusive prefix of bucket totals (n + 2 entries);
// block_hist[blk][b] is replaced by the first output slot of block blk in bucket b.
__global__ __launch_bounds__(1024) void segmap_scan(int32_t* __restrict__ block_hist, int nblk,
                                                    int n, int32_t* __restrict__ seg_off) {
  extern __shared__ int32_t total[];
  for (int b = threadIdx.x; b <= n; b += blockDim.x) {
    int run = 0;
    for (int k = 0; k < nblk; ++k) {
      int c = block_hist[(int64_t)k * (n + 1) + b];
      block_hist[(int64_t)k * (n + 1) + b] = run;
      run += c;
    }
    total[b] = run;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int b = 0; b <= n; ++b) {
      int c = total[b];
      total[b] = run;
      seg_off[b] = run;
      run += c;
    }
    seg_off[n + 1] = run;
  }
  __syncthreads();
  for (int b = threadIdx.x; b <= n; b += blockDim.x) {
    int off = total[b];
    for (int k = 0; k < nblk; ++k) block_hist[(int64_t)k * (n + 1) + b] += off;
  }
}

// Stable scatter: tokens are taken 256 at a time in index order.  Inside a wave a token's rank
// among the earlier tokens of its bucket comes from ballots (one round per distinct bucket in
// the wave); the four waves of a group then take their slots from the bucket cursors one after
// the other, in wave order, so the order of equal ids is the order of their indices.
__global__ __launch_bounds__(SEG_THREADS) void segmap_scatter(const int32_t* __restrict__ ids,
                                                              int64_t T, int n,
                                                              const int32_t* __restrict__ block_base,
                                                              int32_t* __restrict__ perm,
                                                              int32_t* __restrict__ grp_ids) {
  extern __shared__ int32_t cursor[];  // [n + 1]
  for (int b = threadIdx.x; b <= n; b += SEG_THREADS)
    cursor[b] = block_base[(int64_t)blockIdx.x * (n + 1) + b];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint64_t below = lane == 0 ? 0ull : (~0ull >> (64 - lane));      // lanes before this one
  int64_t base = (int64_t)blockIdx.x * SEG_CHUNK;
  __syncthreads();
  for (int g = 0; g < SEG_CHUNK / SEG_THREADS; ++g) {
    int64_t i = base + (int64_t)g * SEG_THREADS + threadIdx.x;
    int b = -1;
    if (i < T) {
      int id = ids[i];
      if (id >= -1 && id < n) b = id < 0 ? n : id;
    }
    // rank inside the wave, and the number of the wave's tokens in the same bucket
    int rank = 0, cnt = 0;
    uint64_t todo = __ballot(b >= 0);
    while (todo) {
      const int leader = __ffsll((unsigned long long)todo) - 1;
      const int lb = __shfl(b, leader);
      const uint64_t same = __ballot(b == lb);
      if (b == lb) { rank = __popcll(same & below); cnt = __popcll(same); }
      todo &= ~same;
    }
    for (int w = 0; w < SEG_THREADS / 64; ++w) {
      if (wave == w && b >= 0) {
        const int slot = cursor[b] + rank;
        perm[slot] = (int32_t)i;
        grp_ids[slot] = b < n ? b : -1;                  // adapter of that grouped row
        if (rank == cnt - 1) cursor[b] += cnt;           // (the wave's reads of this cursor are behind it)
      }
      __syncthreads();
    }
  }
}

// Row chunks of the grouped order: segment t cut into pieces of ROW_CHUNK rows, the rows without
// an adapter (bucket n) last.  One block; thread b handles bucket b, the first chunk index of a
// bucket is the prefix sum of the buckets' chunk counts (serial over at most n + 1 values).
__global__ __launch_bounds__(1024) void segmap_chunks(const int32_t* __restrict__ seg_off, int n,
                                                      RowChunk* __restrict__ chunks) {
  extern __shared__ int32_t first[];   // [n + 2]
  if (threadIdx.x == 0) {
    int run = 0;
    for (int b = 0; b <= n; ++b) {
      first[b] = run;
      run += (seg_off[b + 1] - seg_off[b] + ROW_CHUNK - 1) / ROW_CHUNK;
    }
  }
  __syncthreads();
  for (int b = threadIdx.x; b <= n; b += blockDim.x) {
    const int32_t end = seg_off[b + 1];
    int c = first[b];
    for (int32_t row0 = seg_off[b]; row0 < end; row0 += ROW_CHUNK, ++c) {
      RowChunk ch;
      ch.row0 = row0; ch.nrows = end - row0 < ROW_CHUNK ? end - row0 : ROW_CHUNK; ch.t = b < n ? b : -1; ch.pad = 0;
      chunks[c] = ch;
    }
  }
}

// Adapters by falling segment length (ties: by index): order[k] = the adapter with the k-th longest
// segment.  Kernels whose blocks own whole segments take their adapter from it, so that the long
// segments start first and the short ones fill the end of the launch.  One block; every thread
// ranks its adapters by counting the ones that come before them (n <= 4096).
__global__ __launch_bounds__(1024) void segmap_order(const int32_t* __restrict__ seg_off, int n, int32_t* __restrict__ order,
                                                     int32_t* __restrict__ chunk_base) {
  extern __shared__ int32_t len[];     // [n]
  for (int t = threadIdx.x; t < n; t += blockDim.x) len[t] = seg_off[t + 1] - seg_off[t];
  __syncthreads();
  if (threadIdx.x == 0 && chunk_base != nullptr) {
    // first partial-sum slot of every adapter whose segment is cut into several token chunks
    const int tc = reduce_ragged_chunk(seg_off[n], n);
    int run = 0;
    for (int t = 0; t < n; ++t) {
      chunk_base[t] = run;
      const int nch = (len[t] + tc - 1) / tc;
      if (nch > 1) run += nch;
    }
    chunk_base[n] = run;
  }
  for (int t = threadIdx.x; t < n; t += blockDim.x) {
    const int mine = len[t];
    int before = 0;
    for (int s = 0; s < n; ++s) before += (len[s] > mine) || (len[s] == mine && s < t);
    order[before] = t;
  }
}

int64_t segmap_chunk_count(const int32_t* seg_off, int n) {
  int64_t c = 0;
  for (int b = 0; b <= n; ++b) c += (seg_off[b + 1] - seg_off[b] + ROW_CHUNK - 1) / ROW_CHUNK;
  return c;
}

int64_t segmap_chunk_bound(int64_t T, int n) { return T / ROW_CHUNK + n + 2; }

// plain fill (a kernel, not a memset node)
__global__ void segmap_clear_flags(int32_t* flags) { flags[threadIdx.x] = 0; }

hipError_t launch_segmap(const int32_t* ids, int64_t T, int n, int32_t* perm, int32_t* grp_ids, int32_t* seg_off,
                         int32_t* block_hist, int32_t* flags, RowChunk* chunks, int32_t* order, int32_t* chunk_base,
                         hipStream_t stream) {
  int nblk = segmap_blocks(T);
  hipLaunchKernelGGL(segmap_clear_flags, dim3(1), dim3(2), 0, stream, flags);
  if (nblk > 0) {
    hipLaunchKernelGGL(segmap_hist, dim3(nblk), dim3(SEG_THREADS), (n + 1) * sizeof(int32_t),
                       stream, ids, T, n, block_hist, flags);
  }
  hipLaunchKernelGGL(segmap_scan, dim3(1), dim3(1024), (n + 1) * sizeof(int32_t), stream,
                     block_hist, nblk, n, seg_off);
  if (nblk > 0) {
    hipLaunchKernelGGL(segmap_scatter, dim3(nblk), dim3(SEG_THREADS),
                       (n + 1) * sizeof(int32_t), stream, ids, T, n, block_hist, perm, grp_ids);
  }
  hipLaunchKernelGGL(segmap_chunks, dim3(1), dim3(1024), (n + 2) * sizeof(int32_t), stream, seg_off, n, chunks);
  if (n > 0 && order != nullptr)
    hipLaunchKernelGGL(segmap_order, dim3(1), dim3(1024), n * sizeof(int32_t), stream, seg_off, n, order, chunk_base);
  return hipGetLastError();
}

}  // namespace marlaas
