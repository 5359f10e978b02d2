// Device copies of the per-adapter tables (factor pointers, ranks, scales, gradient pointers) and
// what is derived from them for the fused shrink (rank offsets, extended columns).  Each task owns
// its LoRA parameters and the manager swaps in a new version after every policy update (paper
// Sec. 4.2, Alg. 1), so the tables are written by tiny kernels whose payload travels in the kernel
// arguments: no allocation, no host-to-device copy node, ordered on the caller's stream, legal
// under stream capture.
#include "common.h"

namespace marlaas {

static constexpr int POKE_WORDS = 384;   // 8-byte words per launch (3 KB of kernel arguments)
struct PokeArgs {
  uint64_t* dst;
  int32_t n;
  int32_t pad;
  uint64_t w[POKE_WORDS];
};

__global__ __launch_bounds__(128) void poke_kernel(PokeArgs a) {
  for (int i = threadIdx.x; i < a.n; i += 128) a.dst[i] = a.w[i];
}

static hipError_t poke(uint64_t* dst, const uint64_t* src, int64_t words, hipStream_t stream) {
  PokeArgs a;
  a.pad = 0;
  while (words > 0) {
    const int n = words < POKE_WORDS ? (int)words : POKE_WORDS;
    a.dst = dst; a.n = n;
    for (int i = 0; i < n; ++i) a.w[i] = src[i];
    hipLaunchKernelGGL(poke_kernel, dim3(1), dim3(128), 0, stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dst += n; src += n; words -= n;
  }
  return hipSuccess;
}

static_assert(sizeof(AdapterEntry) == 24 && sizeof(GradEntry) == 16, "table entries are whole 8-byte words");

hipError_t enqueue_write_entries(const DevTables& d, int64_t first, int64_t count, const AdapterEntry* host,
                                 hipStream_t stream) {
  if (count <= 0) return hipSuccess;
  return poke((uint64_t*)(d.entries + first), (const uint64_t*)host, count * 3, stream);
}

hipError_t enqueue_write_grads(const DevTables& d, int64_t first, int64_t count, const GradEntry* host,
                               hipStream_t stream) {
  if (count <= 0) return hipSuccess;
  return poke((uint64_t*)(d.grads + first), (const uint64_t*)host, count * 2, stream);
}

// One block: exclusive prefix sums of the ranks, then the (entry, rank index) of every extended
// column that fits the capacity.
static constexpr int DERIVE_THREADS = 1024;
__global__ __launch_bounds__(DERIVE_THREADS) void derive_kernel(DevTables d, int P) {
  __shared__ int32_t part[DERIVE_THREADS];
  const int tid = threadIdx.x;
  const int per = (P + DERIVE_THREADS - 1) / DERIVE_THREADS;
  const int lo = tid * per < P ? tid * per : P;
  const int hi = lo + per < P ? lo + per : P;
  int32_t sum = 0;
  for (int i = lo; i < hi; ++i) sum += d.entries[i].rank;
  part[tid] = sum;
  __syncthreads();
  // inclusive scan of the per-thread sums (Hillis-Steele, 10 rounds)
  for (int s = 1; s < DERIVE_THREADS; s <<= 1) {
    const int32_t add = tid >= s ? part[tid - s] : 0;
    __syncthreads();
    part[tid] += add;
    __syncthreads();
  }
  int32_t run = part[tid] - sum;
  for (int i = lo; i < hi; ++i) {
    const AdapterEntry en = d.entries[i];
    const int r = en.rank;
    d.roff[i] = run;
    for (int q = 0; q < r; ++q)
      if (run + q < d.ext_cap) { ExtCol c; c.A = en.A; c.B = en.B; c.t = i; c.q = q; c.scale = en.scale; c.pad = 0; d.cols[run + q] = c; }
    run += r;
  }
  if (tid == DERIVE_THREADS - 1) d.roff[P] = part[tid];
}

hipError_t enqueue_derive(const DevTables& d, int64_t P, hipStream_t stream) {
  if (P <= 0) return hipSuccess;
  hipLaunchKernelGGL(derive_kernel, dim3(1), dim3(DERIVE_THREADS), 0, stream, d, (int)P);
  return hipGetLastError();
}

static size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

size_t dev_tables_bytes(int64_t P, int64_t ext_cap) {
  if (P <= 0) return 0;
  return up256((size_t)P * sizeof(AdapterEntry)) + up256((size_t)P * sizeof(GradEntry)) +
         up256((size_t)(P + 2) * sizeof(int32_t)) + up256((size_t)(ext_cap > 0 ? ext_cap : 1) * sizeof(ExtCol));
}

DevTables dev_tables_carve(void* base, int64_t P, int64_t ext_cap) {
  DevTables d;
  if (P <= 0 || base == nullptr) return d;
  char* p = (char*)base;
  d.entries = (AdapterEntry*)p; p += up256((size_t)P * sizeof(AdapterEntry));
  d.grads = (GradEntry*)p;      p += up256((size_t)P * sizeof(GradEntry));
  d.roff = (int32_t*)p;         p += up256((size_t)(P + 2) * sizeof(int32_t));
  d.cols = (ExtCol*)p;
  d.ext_cap = (int32_t)(ext_cap > 0 ? ext_cap : 0);
  return d;
}

}  // namespace marlaas
