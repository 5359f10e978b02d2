// Host side of the C ABI: contexts, argument checks, the token grouping
// object, the adapter table object, workspace carving and the order in which
// the kernels of a forward / backward pass are enqueued.  Nothing here computes
// on tensors, and the passes (forward, backward, multi-projection forward,
// adapter update) neither allocate nor wait: everything they need on the device
// is either in an object the caller created beforehand or in the workspace.
#include "../../include/marlaas_lora.h"
#include "common.h"

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <cmath>
#include <vector>

using namespace marlaas;

struct marlaas_ctx {
  int device = 0;
  void* ws = nullptr;
  size_t ws_bytes = 0;
  void* static_ws = nullptr;     // device address of this GPU's static scratch array
  int32_t* sync_dev = nullptr;   // counters of the decode kernel (zero between launches)
  int cu_count = 0;
  int spin_limit = 1 << 20;
  void* zero_dev = nullptr;    // 256 zero bytes (what masked DMA lanes fetch)
  int decode_finish = DECODE_FINISH_AUTO;     // how the decode kernel's calls get finished (DECODE_FINISH_*)
  std::string err;
  bool profile = false;
  struct Span { int kernel; hipEvent_t beg, end; };
  std::vector<Span> spans;       // event pairs recorded while profiling is on
};

struct marlaas_segmap {
  int device = 0;
  int64_t T_cap = 0;                // capacity: the device buffers below hold a map of this size
  int32_t n_cap = 0;
  int64_t T = 0;                    // current map (after marlaas_segmap_update)
  int32_t n = 0;
  bool built = false;
  int32_t* perm_dev = nullptr;      // [T_cap] grouped order (always built)
  int32_t* grp_dev = nullptr;       // [T_cap] adapter of every grouped row (-1: none)
  int32_t* seg_off_dev = nullptr;   // [n_cap + 2]
  int32_t* block_hist = nullptr;    // counting-sort scratch
  int32_t* flags_dev = nullptr;     // [2]
  int32_t* readback = nullptr;      // pinned host: seg_off[n_cap + 2], flags[2]
  std::vector<int32_t> seg_off;     // host copy
  bool identity = false;            // ids were already grouped: kernels skip the gather
  int max_seg = 0;                  // largest adapter segment
  int64_t T_lora = 0;               // tokens that have an adapter
  RowChunk* chunks_dev = nullptr;   // row chunks of the grouped order (see RowChunk)
  int32_t* order_dev = nullptr;     // [n_cap] adapters by falling segment length
  int32_t* chunk_base_dev = nullptr; // [n_cap + 1] first partial-sum slot of the adapters cut into several token chunks
  int ragged_chunk = 0, ragged_slots = 0;   // the chunk length of that cut, and how many slots it needs in all
  int ragged_adapters = 0;                  // adapters that are cut (the first ones of order_dev)
  int n_chunks = 0;
};

// Registered adapters of one layer (or of the projections of one block that share an input):
// the device tables the kernels read plus a host mirror used for checks and launch planning.
struct marlaas_adapter_table {
  int device = 0;
  int32_t n = 0, n_proj = 0, max_rank = 0;
  void* dev_block = nullptr;
  DevTables dev;
  std::vector<AdapterEntry> host;        // [n_proj * n]; rank 0 = not registered
  std::vector<GradEntry> hgrads;
  std::vector<int32_t> hranks;           // same ranks, contiguous (what the planners read)
  std::vector<float> hscales;
  std::vector<int64_t> versions;         // per entry: number of updates
  int64_t updates = 0;                   // of the whole table
  int64_t plan_version = 0;              // bumped when an update changes a rank
};

static const size_t WS_ALIGN = 256;
static const int64_t EXT_CAP_MAX = 1 << 16;   // extended columns a table can describe

// Scratch of marlaas_lora_fwd_static: one array per GPU, part of the loaded code object, so no
// call ever allocates it.  Host code must not use the array's name as an address: the device
// address is looked up once per device (in marlaas_create, with that device current) and kept.
static __device__ __align__(256) unsigned char scratch[MARLAAS_STATIC_SCRATCH_BYTES];
static const int MAX_DEVICES = 64;
static void* g_scratch_ptr[MAX_DEVICES];
static std::mutex g_scratch_mutex;

static hipError_t static_scratch_of(int device, void** out) {
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // for the current device
    if (e != hipSuccess) return e;
    g_scratch_ptr[device] = p;
  }
  *out = g_scratch_ptr[device];
  return hipSuccess;
}

static int fail(marlaas_ctx* ctx, int status, const char* fmt, ...) {
  if (ctx) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    ctx->err = buf;
  }
  return status;
}

#define HIP_TRY(ctx, expr)                                                          \
  do {                                                                              \
    hipError_t _e = (expr);                                                         \
    if (_e != hipSuccess)                                                           \
      return fail((ctx), MARLAAS_EHIP, "%s failed: %s", #expr, hipGetErrorString(_e)); \
  } while (0)

// While profiling is on, every kernel launch of a pass is bracketed by a pair of
// events on the caller's stream so that its duration can be read back.
struct ProfSpan {
  marlaas_ctx* ctx; hipStream_t st; hipEvent_t end = nullptr;
  ProfSpan(marlaas_ctx* c, int kernel, hipStream_t s) : ctx(c), st(s) {
    if (!c->profile) return;
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone) return;   // no timing inside a capture
    hipEvent_t b = nullptr;
    if (hipEventCreate(&b) != hipSuccess) return;
    if (hipEventCreate(&end) != hipSuccess) { (void)hipEventDestroy(b); end = nullptr; return; }
    (void)hipEventRecord(b, st);
    c->spans.push_back({kernel, b, end});
  }
  ~ProfSpan() { if (end) (void)hipEventRecord(end, st); }
};
#define PROFILED(ctx, kernel, st, expr) do { ProfSpan _span((ctx), (kernel), (st)); HIP_TRY((ctx), (expr)); } while (0)

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

extern "C" const char* marlaas_strerror(int status) {
  switch (status) {
    case MARLAAS_OK: return "ok";
    case MARLAAS_EINVAL: return "invalid argument";
    case MARLAAS_ESHAPE: return "inconsistent shapes";
    case MARLAAS_EALIGN: return "misaligned pointer, leading dimension or feature size";
    case MARLAAS_ENOMEM: return "workspace missing or too small, or allocation failed";
    case MARLAAS_EHIP: return "HIP runtime error";
    case MARLAAS_EUNSUPPORTED: return "unsupported request";
    default: return "unknown status";
  }
}

extern "C" const char* marlaas_last_error(const marlaas_ctx* ctx) {
  return ctx ? ctx->err.c_str() : "null context";
}

extern "C" int marlaas_create(marlaas_ctx** out, int device) {
  if (!out) return MARLAAS_EINVAL;
  *out = nullptr;
  int count = 0;
  if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count || device >= MAX_DEVICES) return MARLAAS_EHIP;
  if (hipSetDevice(device) != hipSuccess) return MARLAAS_EHIP;
  void* sp = nullptr;
  if (static_scratch_of(device, &sp) != hipSuccess || !sp) return MARLAAS_EHIP;
  marlaas_ctx* ctx = new (std::nothrow) marlaas_ctx();
  if (!ctx) return MARLAAS_ENOMEM;
  ctx->device = device;
  ctx->static_ws = sp;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device) == hipSuccess) ctx->cu_count = prop.multiProcessorCount;
  if (hipMalloc((void**)&ctx->sync_dev, DECODE_SYNC_INTS * sizeof(int32_t)) != hipSuccess ||
      hipMemset(ctx->sync_dev, 0, DECODE_SYNC_INTS * sizeof(int32_t)) != hipSuccess ||
      hipMalloc(&ctx->zero_dev, 256) != hipSuccess || hipMemset(ctx->zero_dev, 0, 256) != hipSuccess) {
    (void)hipFree(ctx->zero_dev);
    (void)hipFree(ctx->sync_dev);
    delete ctx;
    return MARLAAS_ENOMEM;
  }
  // MARLAAS_SPIN_LIMIT: polls of the decode kernel's one bounded wait (0: never wait, always take
  // the slow recomputation; for tests of that path)
  if (const char* sl = getenv("MARLAAS_SPIN_LIMIT")) ctx->spin_limit = atoi(sl) < 0 ? 0 : atoi(sl);
  // MARLAAS_DECODE_FINISH: who finishes the decode kernel's calls.  Unset or 3: the kernel itself
  // when the contraction is not split, a second launch of its own finish when it is; 2: always
  // that second launch; 1: always the kernel itself where its conditions hold; 0: the generic
  // finish kernel
  if (const char* df = getenv("MARLAAS_DECODE_FINISH")) {
    const int v = atoi(df);
    ctx->decode_finish = v == 0 ? DECODE_FINISH_GENERIC : v == 1 ? DECODE_FINISH_IN_KERNEL : v == 2 ? DECODE_FINISH_LAUNCH : DECODE_FINISH_AUTO;
  }
  *out = ctx;
  return MARLAAS_OK;
}

static void drop_spans(marlaas_ctx* ctx) {
  for (auto& sp : ctx->spans) { (void)hipEventDestroy(sp.beg); (void)hipEventDestroy(sp.end); }
  ctx->spans.clear();
}

extern "C" int marlaas_profile_enable(marlaas_ctx* ctx, int on) {
  if (!ctx) return MARLAAS_EINVAL;
  HIP_TRY(ctx, hipSetDevice(ctx->device));
  drop_spans(ctx);
  ctx->profile = on != 0;
  return MARLAAS_OK;
}

extern "C" int marlaas_profile_read(marlaas_ctx* ctx, int kernel, double* total_ms, int64_t* launches) {
  if (!ctx || !total_ms || !launches) return MARLAAS_EINVAL;
  HIP_TRY(ctx, hipSetDevice(ctx->device));
  double sum = 0.0;
  int64_t cnt = 0;
  for (auto& sp : ctx->spans) {
    if (sp.kernel != kernel) continue;
    HIP_TRY(ctx, hipEventSynchronize(sp.end));
    float ms = 0.f;
    HIP_TRY(ctx, hipEventElapsedTime(&ms, sp.beg, sp.end));
    sum += ms;
    ++cnt;
  }
  *total_ms = sum;
  *launches = cnt;
  return MARLAAS_OK;
}

extern "C" void marlaas_destroy(marlaas_ctx* ctx) {
  if (!ctx) return;
  (void)hipSetDevice(ctx->device);
  drop_spans(ctx);
  (void)hipFree(ctx->sync_dev);
  (void)hipFree(ctx->zero_dev);
  delete ctx;
}

// ------------------------------------------------------------------ segmap
extern "C" int marlaas_segmap_create(marlaas_ctx* ctx, int64_t T_max, int32_t n_adapters_max, marlaas_segmap** out) {
  if (!ctx) return MARLAAS_EINVAL;
  if (!out) return fail(ctx, MARLAAS_EINVAL, "segmap_create: out is null");
  *out = nullptr;
  if (T_max < 0 || T_max > 0x7fffffff - 4096) return fail(ctx, MARLAAS_EINVAL, "segmap_create: T_max=%lld out of range", (long long)T_max);
  if (n_adapters_max < 0 || n_adapters_max > MARLAAS_MAX_ADAPTERS)
    return fail(ctx, MARLAAS_EINVAL, "segmap_create: n_adapters_max=%d out of range", n_adapters_max);
  HIP_TRY(ctx, hipSetDevice(ctx->device));
  marlaas_segmap* m = new (std::nothrow) marlaas_segmap();
  if (!m) return fail(ctx, MARLAAS_ENOMEM, "segmap_create: host allocation failed");
  m->device = ctx->device; m->T_cap = T_max; m->n_cap = n_adapters_max;
  const size_t nb = (size_t)(segmap_blocks(T_max) > 0 ? segmap_blocks(T_max) : 1);
  const size_t nn = (size_t)n_adapters_max + 2;
  hipError_t e = hipSuccess;
  do {
    if ((e = hipMalloc((void**)&m->perm_dev, sizeof(int32_t) * (size_t)(T_max > 0 ? T_max : 1))) != hipSuccess) break;
    if ((e = hipMalloc((void**)&m->grp_dev, sizeof(int32_t) * (size_t)(T_max > 0 ? T_max : 1))) != hipSuccess) break;
    if ((e = hipMalloc((void**)&m->seg_off_dev, sizeof(int32_t) * nn)) != hipSuccess) break;
    if ((e = hipMalloc((void**)&m->block_hist, sizeof(int32_t) * nb * nn)) != hipSuccess) break;
    if ((e = hipMalloc((void**)&m->flags_dev, 2 * sizeof(int32_t))) != hipSuccess) break;
    if ((e = hipMalloc((void**)&m->chunks_dev, sizeof(RowChunk) * (size_t)segmap_chunk_bound(T_max, n_adapters_max))) != hipSuccess) break;
    if ((e = hipMalloc((void**)&m->order_dev, sizeof(int32_t) * (size_t)(n_adapters_max > 0 ? n_adapters_max : 1))) != hipSuccess) break;
    if ((e = hipMalloc((void**)&m->chunk_base_dev, sizeof(int32_t) * ((size_t)n_adapters_max + 1))) != hipSuccess) break;
    e = hipHostMalloc((void**)&m->readback, sizeof(int32_t) * (nn + 2), hipHostMallocDefault);
  } while (0);
  if (e != hipSuccess) {
    marlaas_segmap_destroy(m);
    return fail(ctx, MARLAAS_ENOMEM, "segmap_create: %s", hipGetErrorString(e));
  }
  *out = m;
  return MARLAAS_OK;
}

extern "C" int marlaas_segmap_update(marlaas_ctx* ctx, marlaas_segmap* m, const int32_t* token_adapter, int64_t T,
                                     int32_t n_adapters, void* stream) {
  if (!ctx) return MARLAAS_EINVAL;
  if (!m) return fail(ctx, MARLAAS_EINVAL, "segmap_update: map is null");
  if (T < 0 || T > m->T_cap) return fail(ctx, MARLAAS_ESHAPE, "segmap_update: T=%lld exceeds the map's capacity %lld", (long long)T, (long long)m->T_cap);
  if (n_adapters < 0 || n_adapters > m->n_cap)
    return fail(ctx, MARLAAS_ESHAPE, "segmap_update: n_adapters=%d exceeds the map's capacity %d", n_adapters, m->n_cap);
  if (T > 0 && !token_adapter) return fail(ctx, MARLAAS_EINVAL, "segmap_update: token_adapter is null");
  if (m->device != ctx->device) return fail(ctx, MARLAAS_EINVAL, "segmap_update: map belongs to device %d", m->device);
  HIP_TRY(ctx, hipSetDevice(ctx->device));
  hipStream_t st = (hipStream_t)stream;
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(st, &cs) == hipSuccess && cs != hipStreamCaptureStatusNone)
    return fail(ctx, MARLAAS_EUNSUPPORTED, "segmap_update reads the segment sizes back and cannot run inside a stream capture");
  m->built = false;
  const size_t nn = (size_t)n_adapters + 2;
  HIP_TRY(ctx, launch_segmap(token_adapter, T, n_adapters, m->perm_dev, m->grp_dev, m->seg_off_dev, m->block_hist, m->flags_dev,
                             m->chunks_dev, m->order_dev, m->chunk_base_dev, st));
  HIP_TRY(ctx, hipMemcpyAsync(m->readback, m->seg_off_dev, sizeof(int32_t) * nn, hipMemcpyDeviceToHost, st));
  HIP_TRY(ctx, hipMemcpyAsync(m->readback + nn, m->flags_dev, 2 * sizeof(int32_t), hipMemcpyDeviceToHost, st));
  HIP_TRY(ctx, hipStreamSynchronize(st));
  if (m->readback[nn]) return fail(ctx, MARLAAS_EINVAL, "segmap: token id outside [-1, %d)", n_adapters);
  m->T = T; m->n = n_adapters;
  m->seg_off.assign(m->readback, m->readback + nn);
  m->identity = m->readback[nn + 1] == 0;
  m->max_seg = 0;
  for (int t = 0; t < n_adapters; ++t) {
    int len = m->seg_off[t + 1] - m->seg_off[t];
    if (len > m->max_seg) m->max_seg = len;
  }
  m->T_lora = m->seg_off[n_adapters];
  m->ragged_chunk = reduce_ragged_chunk(m->T_lora, n_adapters);
  m->ragged_slots = 0; m->ragged_adapters = 0;
  for (int t = 0; t < n_adapters; ++t) {
    const int nch = (m->seg_off[t + 1] - m->seg_off[t] + m->ragged_chunk - 1) / m->ragged_chunk;
    if (nch > 1) { m->ragged_slots += nch; ++m->ragged_adapters; }
  }
  m->n_chunks = (int)segmap_chunk_count(m->seg_off.data(), n_adapters);
  m->built = true;
  return MARLAAS_OK;
}

extern "C" int marlaas_segmap_build(marlaas_ctx* ctx, const int32_t* token_adapter, int64_t T,
                                    int32_t n_adapters, void* stream, marlaas_segmap** out) {
  if (!ctx) return MARLAAS_EINVAL;
  if (!out) return fail(ctx, MARLAAS_EINVAL, "segmap_build: out is null");
  *out = nullptr;
  if (T > 0 && !token_adapter) return fail(ctx, MARLAAS_EINVAL, "segmap_build: token_adapter is null");
  marlaas_segmap* m = nullptr;
  int rc = marlaas_segmap_create(ctx, T, n_adapters, &m);
  if (rc != MARLAAS_OK) return rc;
  rc = marlaas_segmap_update(ctx, m, token_adapter, T, n_adapters, stream);
  if (rc != MARLAAS_OK) { marlaas_segmap_destroy(m); return rc; }
  *out = m;
  return MARLAAS_OK;
}

extern "C" void marlaas_segmap_destroy(marlaas_segmap* map) {
  if (!map) return;
  (void)hipSetDevice(map->device);
  (void)hipFree(map->perm_dev);
  (void)hipFree(map->grp_dev);
  (void)hipFree(map->seg_off_dev);
  (void)hipFree(map->block_hist);
  (void)hipFree(map->flags_dev);
  (void)hipFree(map->chunks_dev);
  (void)hipFree(map->order_dev);
  (void)hipFree(map->chunk_base_dev);
  if (map->readback) (void)hipHostFree(map->readback);
  delete map;
}

extern "C" int marlaas_segmap_export(const marlaas_segmap* map, int32_t* perm, int32_t* seg_off) {
  if (!map || !map->built) return MARLAAS_EINVAL;
  if (seg_off) memcpy(seg_off, map->seg_off.data(), sizeof(int32_t) * map->seg_off.size());
  if (perm && map->T > 0) {
    if (hipSetDevice(map->device) != hipSuccess) return MARLAAS_EHIP;
    if (hipMemcpy(perm, map->perm_dev, sizeof(int32_t) * (size_t)map->T, hipMemcpyDeviceToHost) != hipSuccess)
      return MARLAAS_EHIP;
  }
  return MARLAAS_OK;
}

// ------------------------------------------------------------------ adapter table
extern "C" int marlaas_adapter_table_create(marlaas_ctx* ctx, int32_t n_adapters, int32_t n_proj, int32_t max_rank,
                                            marlaas_adapter_table** out) {
  if (!ctx) return MARLAAS_EINVAL;
  if (!out) return fail(ctx, MARLAAS_EINVAL, "adapter_table_create: out is null");
  *out = nullptr;
  if (n_adapters < 1 || n_adapters > MARLAAS_MAX_ADAPTERS) return fail(ctx, MARLAAS_EINVAL, "adapter_table_create: n_adapters=%d out of range", n_adapters);
  if (n_proj < 1 || n_proj > MARLAAS_MAX_PROJ) return fail(ctx, MARLAAS_EINVAL, "adapter_table_create: n_proj must be 1..%d", MARLAAS_MAX_PROJ);
  if (max_rank < 1 || max_rank > MARLAAS_MAX_RANK) return fail(ctx, MARLAAS_EINVAL, "adapter_table_create: max_rank must be 1..%d", MARLAAS_MAX_RANK);
  HIP_TRY(ctx, hipSetDevice(ctx->device));
  marlaas_adapter_table* tb = new (std::nothrow) marlaas_adapter_table();
  if (!tb) return fail(ctx, MARLAAS_ENOMEM, "adapter_table_create: host allocation failed");
  tb->device = ctx->device; tb->n = n_adapters; tb->n_proj = n_proj; tb->max_rank = max_rank;
  const int64_t P = (int64_t)n_adapters * n_proj;
  int64_t cap = P * max_rank;
  if (cap > EXT_CAP_MAX) cap = EXT_CAP_MAX;
  const size_t bytes = dev_tables_bytes(P, cap);
  hipError_t e = hipMalloc(&tb->dev_block, bytes);
  if (e == hipSuccess) e = hipMemset(tb->dev_block, 0, bytes);     // creation is not a pass: a plain blocking fill
  if (e != hipSuccess) {
    marlaas_adapter_table_destroy(tb);
    return fail(ctx, MARLAAS_ENOMEM, "adapter_table_create: %s", hipGetErrorString(e));
  }
  tb->dev = dev_tables_carve(tb->dev_block, P, cap);
  AdapterEntry z; z.A = nullptr; z.B = nullptr; z.rank = 0; z.scale = 0.f;
  GradEntry zg; zg.dA = nullptr; zg.dB = nullptr;
  tb->host.assign((size_t)P, z);
  tb->hgrads.assign((size_t)P, zg);
  tb->hranks.assign((size_t)P, 0);
  tb->hscales.assign((size_t)P, 0.f);
  tb->versions.assign((size_t)P, 0);
  *out = tb;
  return MARLAAS_OK;
}

extern "C" void marlaas_adapter_table_destroy(marlaas_adapter_table* tb) {
  if (!tb) return;
  (void)hipSetDevice(tb->device);
  (void)hipFree(tb->dev_block);
  delete tb;
}

extern "C" int marlaas_adapter_table_update(marlaas_ctx* ctx, marlaas_adapter_table* tb, int32_t proj, int32_t t,
                                            const void* A, const void* B, int32_t rank, float scale,
                                            void* dA, void* dB, void* stream) {
  if (!ctx) return MARLAAS_EINVAL;
  if (!tb) return fail(ctx, MARLAAS_EINVAL, "adapter_table_update: table is null");
  if (tb->device != ctx->device) return fail(ctx, MARLAAS_EINVAL, "adapter_table_update: table belongs to device %d", tb->device);
  if (proj < 0 || proj >= tb->n_proj || t < 0 || t >= tb->n)
    return fail(ctx, MARLAAS_EINVAL, "adapter_table_update: (projection %d, adapter %d) outside the table (%d x %d)", proj, t, tb->n_proj, tb->n);
  if (!A || !B) return fail(ctx, MARLAAS_EINVAL, "adapter_table_update: null factor");
  if (!aligned16(A) || !aligned16(B)) return fail(ctx, MARLAAS_EALIGN, "adapter_table_update: factors must be 16-byte aligned");
  if (rank < 1 || rank > tb->max_rank) return fail(ctx, MARLAAS_EINVAL, "adapter_table_update: rank %d, table holds 1..%d", rank, tb->max_rank);
  if ((dA == nullptr) != (dB == nullptr)) return fail(ctx, MARLAAS_EINVAL, "adapter_table_update: dA and dB must both be given or both be null");
  if (dA && (!aligned16(dA) || !aligned16(dB))) return fail(ctx, MARLAAS_EALIGN, "adapter_table_update: gradient buffers must be 16-byte aligned");
  HIP_TRY(ctx, hipSetDevice(ctx->device));
  hipStream_t st = (hipStream_t)stream;
  const int64_t i = (int64_t)proj * tb->n + t;
  AdapterEntry e; e.A = A; e.B = B; e.rank = rank; e.scale = scale;
  GradEntry g; g.dA = (float*)dA; g.dB = (float*)dB;
  const bool rank_changed = tb->hranks[i] != rank;
  HIP_TRY(ctx, enqueue_write_entries(tb->dev, i, 1, &e, st));
  HIP_TRY(ctx, enqueue_write_grads(tb->dev, i, 1, &g, st));
  // (the extended-column list carries copies of the factor pointers: always rebuilt)
  HIP_TRY(ctx, enqueue_derive(tb->dev, (int64_t)tb->n * tb->n_proj, st));
  tb->host[i] = e; tb->hgrads[i] = g; tb->hranks[i] = rank; tb->hscales[i] = scale;
  ++tb->versions[i];
  ++tb->updates;
  if (rank_changed) ++tb->plan_version;
  return MARLAAS_OK;
}

extern "C" int64_t marlaas_adapter_table_version(const marlaas_adapter_table* tb, int32_t proj, int32_t t) {
  if (!tb) return -1;
  if (t < 0) return tb->updates;
  if (proj < 0 || proj >= tb->n_proj || t >= tb->n) return -1;
  return tb->versions[(size_t)proj * tb->n + t];
}

extern "C" int64_t marlaas_adapter_table_plan_version(const marlaas_adapter_table* tb) {
  return tb ? tb->plan_version : -1;
}

// ------------------------------------------------------------------ descriptor checks
// Ranks and scales of a descriptor's adapters (host memory): from its table when it has one.
static const int32_t* ranks_of(const marlaas_lora_desc* d) {
  return d->table ? d->table->hranks.data() + (size_t)d->proj * d->table->n : d->ranks;
}

static int max_rank_of(const marlaas_lora_desc* d) {
  const int32_t* ranks = ranks_of(d);
  int mr = 0;
  for (int t = 0; t < d->n_adapters; ++t) if (ranks[t] > mr) mr = ranks[t];
  return mr;
}

static int sum_ranks_of(const marlaas_lora_desc* d) {
  const int32_t* ranks = ranks_of(d);
  int64_t sum = 0;
  for (int t = 0; t < d->n_adapters; ++t) sum += ranks[t];
  return sum > 0x7fffffff ? 0x7fffffff : (int)sum;
}

static bool ranks_mult8_of(const marlaas_lora_desc* d) {
  const int32_t* ranks = ranks_of(d);
  for (int t = 0; t < d->n_adapters; ++t) if (ranks[t] & 7) return false;
  return true;
}

static int check_sizes(marlaas_ctx* ctx, const marlaas_lora_desc* d) {
  if (!d) return fail(ctx, MARLAAS_EINVAL, "descriptor is null");
  if (d->T < 0 || d->d_in <= 0 || d->d_out <= 0) return fail(ctx, MARLAAS_EINVAL, "negative or zero size");
  if (d->T > 0x7fffffff - 4096 || d->d_in > (1 << 24) || d->d_out > (1 << 24))
    return fail(ctx, MARLAAS_EINVAL, "size too large");
  if (d->n_adapters < 0 || d->n_adapters > MARLAAS_MAX_ADAPTERS) return fail(ctx, MARLAAS_EINVAL, "n_adapters out of range");
  if (d->in_dtype != MARLAAS_BF16 && d->in_dtype != MARLAAS_F32) return fail(ctx, MARLAAS_EINVAL, "bad in_dtype");
  if (d->out_dtype != MARLAAS_BF16 && d->out_dtype != MARLAAS_F32) return fail(ctx, MARLAAS_EINVAL, "bad out_dtype");
  if (d->layout != MARLAAS_LAYOUT_MATH && d->layout != MARLAAS_LAYOUT_TORCH) return fail(ctx, MARLAAS_EINVAL, "bad layout");
  if ((d->d_in & 7) || (d->d_out & 7)) return fail(ctx, MARLAAS_EALIGN, "d_in and d_out must be multiples of 8");
  if (!d->map) return fail(ctx, MARLAAS_EINVAL, "segment map is null");
  if (!d->map->built) return fail(ctx, MARLAAS_EINVAL, "segment map holds no map (marlaas_segmap_update failed or was never called)");
  if (d->map->T != d->T || d->map->n != d->n_adapters)
    return fail(ctx, MARLAAS_ESHAPE, "segment map was built for T=%lld, n=%d", (long long)d->map->T, d->map->n);
  if (d->table) {
    const marlaas_adapter_table* tb = d->table;
    if (tb->n != d->n_adapters) return fail(ctx, MARLAAS_ESHAPE, "adapter table holds %d adapters, descriptor says %d", tb->n, d->n_adapters);
    if (d->proj < 0 || d->proj >= tb->n_proj) return fail(ctx, MARLAAS_EINVAL, "projection %d outside the adapter table (%d)", d->proj, tb->n_proj);
    // an adapter that no token uses may be unregistered (rank 0: the kernels skip it)
    const int32_t* ranks = ranks_of(d);
    for (int t = 0; t < d->n_adapters; ++t)
      if (ranks[t] == 0 && d->map->seg_off[t + 1] > d->map->seg_off[t])
        return fail(ctx, MARLAAS_EINVAL, "adapter %d has tokens but is not registered in the adapter table", t);
  } else if (d->n_adapters > 0) {
    if (!d->ranks || !d->scales) return fail(ctx, MARLAAS_EINVAL, "ranks / scales are null");
    for (int t = 0; t < d->n_adapters; ++t)
      if (d->ranks[t] < 1 || d->ranks[t] > MARLAAS_MAX_RANK)
        return fail(ctx, MARLAAS_EINVAL, "rank of adapter %d is %d, must be 1..%d", t, d->ranks[t], MARLAAS_MAX_RANK);
  }
  return MARLAAS_OK;
}

extern "C" int64_t marlaas_u_stride(const marlaas_lora_desc* d) {
  if (!d || d->n_adapters < 0 || d->n_adapters > MARLAAS_MAX_ADAPTERS) return 0;
  if (d->n_adapters == 0) return 16;
  if (d->table) {
    if (d->table->n != d->n_adapters || d->proj < 0 || d->proj >= d->table->n_proj) return 0;
  } else if (!d->ranks) {
    return 0;
  }
  int mr = max_rank_of(d);
  if (mr < 0 || mr > MARLAAS_MAX_RANK) return 0;
  if (mr == 0) return d->table ? 16 : 0;
  return (mr + 15) & ~15;
}

// Extended columns the workspace copy of a descriptor's tables can describe.
static int64_t ws_ext_cap(int64_t n_ext) { return n_ext < EXT_CAP_MAX ? n_ext : EXT_CAP_MAX; }

struct WsPlan {
  size_t u_off = 0, v_off = 0, part_off = 0, part_bytes = 0, total = 0;   // part: reused by every kernel with partial sums
  size_t u2_off = 0, v2_off = 0, uv2_bytes = 0;   // two-term bf16 splits of u and v, [T][2 r_stride] (bf16 inputs)
  size_t lt_off = 0, lt_bytes = 0;                // the row tiles' lists of extra contraction tiles (large-batch GEMM)
  size_t wt_off = 0, wt_bytes = 0;   // transposed copy of the weight (large batches, output-contiguous storage)
  size_t tab_off = 0, tab_bytes = 0; // per-call copy of the adapter tables (descriptors without a table object)
};

static WsPlan plan_workspace(const marlaas_lora_desc* d, int want_bwd) {
  WsPlan p;
  const size_t rs = (size_t)marlaas_u_stride(d);
  const size_t uv = align_up((size_t)(d->T > 0 ? d->T : 1) * rs * sizeof(float), WS_ALIGN);
  size_t off = 0;
  p.u_off = off; off += uv;
  const bool bf = d->in_dtype == MARLAAS_BF16 && d->n_adapters > 0;
  if (bf) {
    p.uv2_bytes = uv; p.u2_off = off; off += uv;
    p.lt_bytes = align_up(lora_tiles_bytes(d->T), WS_ALIGN); p.lt_off = off; off += p.lt_bytes;
  }
  size_t part = 0;
  const int n_ext = sum_ranks_of(d);
  if (d->in_dtype == MARLAAS_BF16) part = gemm_splitk_bytes(d->T, d->d_in, d->d_out, n_ext);
  if (bf) {
    const size_t ps = shrink_partial_bytes(d->d_in, d->map->T_lora, d->n_adapters, (int)rs);
    if (ps > part) part = ps;
  }
  if (want_bwd) {
    p.v_off = off; off += uv;
    if (bf) { p.v2_off = off; off += uv; }
    if (d->in_dtype == MARLAAS_BF16) {
      const size_t pv = d->n_adapters > 0 ? shrink_partial_bytes(d->d_out, d->map->T_lora, d->n_adapters, (int)rs) : 0;
      if (pv > part) part = pv;
      // (few adapters: room for the reductions' sums even where one chunk covers a segment, so
      // that a backward with the optimizer step attached can always run)
      const bool always = d->n_adapters <= OPT_MAX_ADAPTERS;
      const size_t pa = reduce_partial_bytes(d->d_in, d->n_adapters, d->map->max_seg, (int)rs, always, d->map->ragged_chunk, d->map->ragged_slots);
      const size_t pb = reduce_partial_bytes(d->d_out, d->n_adapters, d->map->max_seg, (int)rs, always, d->map->ragged_chunk, d->map->ragged_slots);
      const size_t pg = gemm_splitk_bytes(d->T, d->d_out, d->d_in, n_ext);
      if (pa > part) part = pa;
      if (pb > part) part = pb;
      if (pg > part) part = pg;
    }
  }
  p.part_bytes = align_up(part, WS_ALIGN);
  p.part_off = off; off += p.part_bytes;
  if (d->in_dtype == MARLAAS_BF16) {
    size_t wt = d->layout == MARLAAS_LAYOUT_MATH ? gemm_wt_bytes(FORM_NN, d->T, d->d_in, d->d_out) : 0;
    if (want_bwd && d->layout == MARLAAS_LAYOUT_TORCH) wt = gemm_wt_bytes(FORM_NN, d->T, d->d_out, d->d_in);
    if (d->W_t) wt = 0;                  // the caller keeps the transposed copy
    p.wt_bytes = align_up(wt, WS_ALIGN);
    p.wt_off = off; off += p.wt_bytes;
  }
  if (!d->table && d->n_adapters > 0) {
    p.tab_bytes = dev_tables_bytes(d->n_adapters, ws_ext_cap(n_ext));
    p.tab_off = off; off += p.tab_bytes;
  }
  p.total = off;
  return p;
}

extern "C" size_t marlaas_workspace_bytes(const marlaas_lora_desc* d, int want_bwd) {
  if (check_sizes(nullptr, d) != MARLAAS_OK) return 0;
  return plan_workspace(d, want_bwd).total;
}

extern "C" int marlaas_set_workspace(marlaas_ctx* ctx, void* dev_ptr, size_t bytes) {
  if (!ctx) return MARLAAS_EINVAL;
  if (dev_ptr && ((uintptr_t)dev_ptr & (WS_ALIGN - 1)))
    return fail(ctx, MARLAAS_EALIGN, "workspace must be %zu-byte aligned", WS_ALIGN);
  ctx->ws = dev_ptr;
  ctx->ws_bytes = dev_ptr ? bytes : 0;
  return MARLAAS_OK;
}

static int check_tensors(marlaas_ctx* ctx, const marlaas_lora_desc* d) {
  const int64_t esz = d->in_dtype == MARLAAS_BF16 ? 2 : 4;
  if (d->T > 0 && !d->x) return fail(ctx, MARLAAS_EINVAL, "x is null");
  if (!d->W) return fail(ctx, MARLAAS_EINVAL, "W is null");
  if (!aligned16(d->x) || !aligned16(d->W)) return fail(ctx, MARLAAS_EALIGN, "x and W must be 16-byte aligned");
  if (!aligned16(d->W_packed_fwd) || !aligned16(d->W_packed_bwd) || !aligned16(d->W_t))
    return fail(ctx, MARLAAS_EALIGN, "packed and transposed weights must be 16-byte aligned");
  if ((d->W_packed_fwd || d->W_packed_bwd || d->W_t) && d->in_dtype != MARLAAS_BF16)
    return fail(ctx, MARLAAS_EINVAL, "packed and transposed weights exist for bf16 only");
  if (d->ldx < d->d_in || (d->ldx * esz) % 16) return fail(ctx, MARLAAS_EALIGN, "ldx=%lld", (long long)d->ldx);
  const int64_t wcols = d->layout == MARLAAS_LAYOUT_MATH ? d->d_out : d->d_in;
  if (d->ldw < wcols || (d->ldw * esz) % 16) return fail(ctx, MARLAAS_EALIGN, "ldw=%lld", (long long)d->ldw);
  if (d->ldw > (1 << 22)) return fail(ctx, MARLAAS_EINVAL, "ldw=%lld is above 4194304", (long long)d->ldw);
  if (d->table) {
    if (d->table->device != ctx->device) return fail(ctx, MARLAAS_EINVAL, "adapter table belongs to device %d", d->table->device);
  } else if (d->n_adapters > 0) {
    if (!d->A || !d->B) return fail(ctx, MARLAAS_EINVAL, "A / B pointer arrays are null");
    for (int t = 0; t < d->n_adapters; ++t) {
      if (!d->A[t] || !d->B[t]) return fail(ctx, MARLAAS_EINVAL, "adapter %d has a null factor", t);
      if (!aligned16(d->A[t]) || !aligned16(d->B[t])) return fail(ctx, MARLAAS_EALIGN, "adapter %d factors must be 16-byte aligned", t);
    }
  }
  return MARLAAS_OK;
}

// Where the kernels of one call find its adapters.
struct Bank {
  const AdapterEntry* entries = nullptr;   // device: this call's adapters, [n_adapters]
  const GradEntry* grads = nullptr;
  DevTables all;                           // the whole bank (a table object's, or the workspace copy)
  int t0 = 0;                              // index of entries[0] in the bank
  int ext_base = 0;                        // first extended column of this call in the bank's column space
  int n_ext = 0;                           // this call's extended columns (sum of its ranks)
  bool mult8 = true;
  bool in_ws = false;                      // tables are a per-call copy in the workspace
};

// Resolve a descriptor's tables.  Without a table object the entries are written into the
// workspace slice `ws_tab` by a small kernel launch on the caller's stream (payload in the kernel
// arguments); with one, nothing is enqueued.
static int resolve_bank(marlaas_ctx* ctx, const marlaas_lora_desc* d, void* ws_tab, size_t ws_tab_bytes,
                        hipStream_t st, Bank* b) {
  *b = Bank();
  if (d->n_adapters == 0) return MARLAAS_OK;
  b->n_ext = sum_ranks_of(d);
  b->mult8 = ranks_mult8_of(d);
  if (d->table) {
    const marlaas_adapter_table* tb = d->table;
    b->all = tb->dev;
    b->t0 = d->proj * tb->n;
    b->entries = tb->dev.entries + b->t0;
    b->grads = tb->dev.grads + b->t0;
    int64_t base = 0;
    for (int i = 0; i < b->t0; ++i) base += tb->hranks[i];
    b->ext_base = (int)base;
    return MARLAAS_OK;
  }
  const size_t need = dev_tables_bytes(d->n_adapters, ws_ext_cap(b->n_ext));
  if (!ws_tab || ws_tab_bytes < need)
    return fail(ctx, MARLAAS_ENOMEM, "a descriptor without an adapter table needs workspace for its tables (%zu bytes)", need);
  b->all = dev_tables_carve(ws_tab, d->n_adapters, ws_ext_cap(b->n_ext));
  b->entries = b->all.entries;
  b->grads = b->all.grads;
  b->in_ws = true;
  std::vector<AdapterEntry> host((size_t)d->n_adapters);
  for (int t = 0; t < d->n_adapters; ++t) {
    host[t].A = d->A[t]; host[t].B = d->B[t]; host[t].rank = d->ranks[t]; host[t].scale = d->scales[t];
  }
  HIP_TRY(ctx, enqueue_write_entries(b->all, 0, d->n_adapters, host.data(), st));
  return MARLAAS_OK;
}

// The fused shrink reads rank offsets and extended columns; a workspace copy derives them now.
static int bank_fuse(marlaas_ctx* ctx, const Bank& b, int n_adapters, hipStream_t st, GemmFuse* f) {
  if (b.in_ws) HIP_TRY(ctx, enqueue_derive(b.all, n_adapters, st));
  f->roff = b.all.roff + b.t0;
  f->cols = b.all.cols + b.ext_base;
  f->n_ext = b.n_ext;
  f->ranks_mult8 = b.mult8;
  f->u_out = nullptr;
  f->t0 = b.t0;
  f->ext_base = b.ext_base;
  return MARLAAS_OK;
}

static bool bank_can_fuse(const Bank& b) {
  return b.n_ext > 0 && (int64_t)b.ext_base + b.n_ext <= b.all.ext_cap;
}

// ------------------------------------------------------------------ packed weight
extern "C" size_t marlaas_packed_weight_bytes(int64_t d_in, int64_t d_out, int32_t direction) {
  if (d_in <= 0 || d_out <= 0 || d_in > (1 << 24) || d_out > (1 << 24) || (direction != 0 && direction != 1)) return 0;
  return direction == 0 ? packed_weight_bytes(d_in, d_out) : packed_weight_bytes(d_out, d_in);
}

extern "C" int marlaas_pack_weight(marlaas_ctx* ctx, const void* W, int64_t ldw, int64_t d_in, int64_t d_out,
                                   int32_t layout, int32_t direction, void* packed, void* stream) {
  if (!ctx) return MARLAAS_EINVAL;
  if (!W || !packed) return fail(ctx, MARLAAS_EINVAL, "pack_weight: null pointer");
  if (d_in <= 0 || d_out <= 0 || d_in > (1 << 24) || d_out > (1 << 24)) return fail(ctx, MARLAAS_EINVAL, "pack_weight: bad sizes");
  if ((d_in & 7) || (d_out & 7)) return fail(ctx, MARLAAS_EALIGN, "d_in and d_out must be multiples of 8");
  if (layout != MARLAAS_LAYOUT_MATH && layout != MARLAAS_LAYOUT_TORCH) return fail(ctx, MARLAAS_EINVAL, "pack_weight: bad layout");
  if (direction != 0 && direction != 1) return fail(ctx, MARLAAS_EINVAL, "pack_weight: direction must be 0 (forward) or 1 (backward)");
  const int64_t wcols = layout == MARLAAS_LAYOUT_MATH ? d_out : d_in;
  if (ldw < wcols) return fail(ctx, MARLAAS_EALIGN, "pack_weight: ldw=%lld", (long long)ldw);
  if (!aligned16(W) || !aligned16(packed)) return fail(ctx, MARLAAS_EALIGN, "pack_weight: pointers must be 16-byte aligned");
  HIP_TRY(ctx, hipSetDevice(ctx->device));
  // element (i, j) of W (i over d_in, j over d_out) is at W[i * si + j * sj]
  const int64_t si = layout == MARLAAS_LAYOUT_MATH ? ldw : 1, sj = layout == MARLAAS_LAYOUT_MATH ? 1 : ldw;
  if (direction == 0)   // forward: contraction over d_in, outputs over d_out
    HIP_TRY(ctx, launch_pack_weight((const bf16_t*)W, si, sj, d_in, d_out, (bf16_t*)packed, (hipStream_t)stream));
  else                  // backward (dX = dY W^T): contraction over d_out, outputs over d_in
    HIP_TRY(ctx, launch_pack_weight((const bf16_t*)W, sj, si, d_out, d_in, (bf16_t*)packed, (hipStream_t)stream));
  return MARLAAS_OK;
}

extern "C" int marlaas_transpose_weight(marlaas_ctx* ctx, const void* W, int64_t ldw, int64_t d_in, int64_t d_out,
                                        int32_t layout, void* out, void* stream) {
  if (!ctx) return MARLAAS_EINVAL;
  if (!W || !out) return fail(ctx, MARLAAS_EINVAL, "transpose_weight: null pointer");
  if (d_in <= 0 || d_out <= 0 || d_in > (1 << 24) || d_out > (1 << 24)) return fail(ctx, MARLAAS_EINVAL, "transpose_weight: bad sizes");
  if ((d_in & 7) || (d_out & 7)) return fail(ctx, MARLAAS_EALIGN, "d_in and d_out must be multiples of 8");
  if (layout != MARLAAS_LAYOUT_MATH && layout != MARLAAS_LAYOUT_TORCH) return fail(ctx, MARLAAS_EINVAL, "transpose_weight: bad layout");
  const int64_t rows = layout == MARLAAS_LAYOUT_MATH ? d_in : d_out, cols = layout == MARLAAS_LAYOUT_MATH ? d_out : d_in;
  if (ldw < cols || (ldw & 7)) return fail(ctx, MARLAAS_EALIGN, "transpose_weight: ldw=%lld", (long long)ldw);
  if (!aligned16(W) || !aligned16(out)) return fail(ctx, MARLAAS_EALIGN, "transpose_weight: pointers must be 16-byte aligned");
  HIP_TRY(ctx, hipSetDevice(ctx->device));
  HIP_TRY(ctx, launch_transpose_bf16((const bf16_t*)W, ldw, (bf16_t*)out, rows, rows, cols, (hipStream_t)stream));
  return MARLAAS_OK;
}

static DecodeSync decode_sync_of(const marlaas_ctx* ctx, const marlaas_segmap* map) {
  DecodeSync s;
  s.mode = ctx->decode_finish; s.counters = ctx->sync_dev; s.grp_ids = map->grp_dev; s.spin_limit = ctx->spin_limit; s.cu_count = ctx->cu_count;
  return s;
}

// ------------------------------------------------------------------ forward
static int fwd_impl(marlaas_ctx* ctx, const marlaas_lora_desc* d, void* y, int64_t ldy, void* u_save, void* stream,
                    void* ws, size_t ws_bytes) {
  int rc = check_sizes(ctx, d);
  if (rc != MARLAAS_OK) return rc;
  if (d->T == 0) return MARLAAS_OK;
  if ((rc = check_tensors(ctx, d)) != MARLAAS_OK) return rc;
  const int64_t osz = d->out_dtype == MARLAAS_BF16 ? 2 : 4;
  if (!y) return fail(ctx, MARLAAS_EINVAL, "y is null");
  if (!aligned16(y) || ldy < d->d_out || (ldy * osz) % 16) return fail(ctx, MARLAAS_EALIGN, "y / ldy");
  if (u_save && !aligned16(u_save)) return fail(ctx, MARLAAS_EALIGN, "u_save must be 16-byte aligned");
  HIP_TRY(ctx, hipSetDevice(ctx->device));
  hipStream_t st = (hipStream_t)stream;
  const marlaas_segmap* map = d->map;
  const int rs = (int)marlaas_u_stride(d);
  float* u = (float*)u_save;
  const bool lora = d->n_adapters > 0 && map->T_lora > 0;
  WsPlan p = plan_workspace(d, 0);
  const bool have_ws = ws && ws_bytes >= p.total;
  if (lora && !u) {
    if (!have_ws)
      return fail(ctx, MARLAAS_ENOMEM, "forward needs %zu workspace bytes, have %zu", p.total, ws_bytes);
    u = (float*)((char*)ws + p.u_off);
  }
  float* part = (have_ws && p.part_bytes) ? (float*)((char*)ws + p.part_off) : nullptr;
  Bank bank;
  if (lora && (rc = resolve_bank(ctx, d, have_ws ? (char*)ws + p.tab_off : nullptr, p.tab_bytes, st, &bank)) != MARLAAS_OK) return rc;
  const AdapterEntry* table = bank.entries;
  const int32_t* perm = map->identity ? nullptr : map->perm_dev;
  // forward contracts over d_in: math W[d_in,d_out] is [contraction, output] (NN), torch is NT;
  // A_t follows W for the shrink, B_t follows W for the expand.
  const int form = d->layout == MARLAAS_LAYOUT_MATH ? FORM_NN : FORM_NT;
  const int out_f32 = d->out_dtype == MARLAAS_F32;
  const DecodeSync dsync = decode_sync_of(ctx, map);
  if (d->in_dtype == MARLAAS_BF16) {
    // small batches: the GEMM computes the shrink itself and no shrink kernel runs
    GemmFuse fuse;
    bool fused = false;
    if (lora && part && bank_can_fuse(bank)) {
      fused = gemm_can_fuse_shrink(form, d->T, d->d_in, d->d_out, bank.n_ext, bank.mult8, p.part_bytes);
      if (fused) {
        if ((rc = bank_fuse(ctx, bank, d->n_adapters, st, &fuse)) != MARLAAS_OK) return rc;
        fuse.u_out = u;
      }
    }
    bool have_u2 = false;
    bf16_t* u2 = (have_ws && p.uv2_bytes) ? (bf16_t*)((char*)ws + p.u2_off) : nullptr;
    if (lora && !fused)
      PROFILED(ctx, MARLAAS_KERNEL_SHRINK, st, launch_shrink_bf16((const bf16_t*)d->x, d->ldx, d->d_in, perm, map->seg_off_dev, d->n_adapters,
                                      map->max_seg, table, 0, form, u, rs, map->T_lora, part, part ? p.part_bytes : 0, u2,
                                      &have_u2, (const bf16_t*)ctx->zero_dev, bank.mult8, st));
    LoraDma dma;
    if (have_u2 && have_ws && p.lt_bytes) {
      dma.u2 = u2; dma.tiles = (int32_t*)((char*)ws + p.lt_off); dma.tiles_bytes = p.lt_bytes;
      dma.zero_line = (const bf16_t*)ctx->zero_dev; dma.ranks_mult8 = bank.mult8;
    }
    PROFILED(ctx, MARLAAS_KERNEL_GEMM, st, launch_gemm_bf16((const bf16_t*)d->x, d->ldx, (const bf16_t*)d->W, d->ldw, form, d->T, d->d_in,
                                  d->d_out, perm, map->seg_off_dev, d->n_adapters, table, 1, lora ? u : nullptr,
                                  rs, y, ldy, out_f32, part, part ? p.part_bytes : 0, map->chunks_dev, map->n_chunks,
                                  fused ? &fuse : nullptr, (have_ws && p.wt_bytes) ? (bf16_t*)((char*)ws + p.wt_off) : nullptr,
                                  p.wt_bytes, d->layout == MARLAAS_LAYOUT_MATH ? (const bf16_t*)d->W_t : nullptr, &dma, (const bf16_t*)d->W_packed_fwd, &dsync, st));
  } else {
    if (lora)
      PROFILED(ctx, MARLAAS_KERNEL_SHRINK, st, launch_shrink_f32((const float*)d->x, d->ldx, d->d_in, perm, map->seg_off_dev, d->n_adapters,
                                     table, 0, form, u, rs, map->T_lora, st));
    PROFILED(ctx, MARLAAS_KERNEL_GEMM, st, launch_gemm_f32((const float*)d->x, d->ldx, (const float*)d->W, d->ldw, form, d->T, d->d_in,
                                 d->d_out, perm, map->seg_off_dev, d->n_adapters, table, 1, lora ? u : nullptr,
                                 rs, y, ldy, out_f32, st));
  }
  return MARLAAS_OK;
}

extern "C" int marlaas_lora_fwd(marlaas_ctx* ctx, const marlaas_lora_desc* d, void* y, int64_t ldy,
                                void* u_save, void* stream) {
  if (!ctx) return MARLAAS_EINVAL;
  return fwd_impl(ctx, d, y, ldy, u_save, stream, ctx->ws, ctx->ws_bytes);
}

extern "C" int marlaas_lora_fwd_static(marlaas_ctx* ctx, const marlaas_lora_desc* d, void* y, int64_t ldy,
                                       void* u_save, void* stream) {
  if (!ctx) return MARLAAS_EINVAL;
  int rc = check_sizes(ctx, d);
  if (rc != MARLAAS_OK) return rc;
  const size_t need = plan_workspace(d, 0).total;
  if (need > (size_t)MARLAAS_STATIC_SCRATCH_BYTES)
    return fail(ctx, MARLAAS_ENOMEM, "this forward needs %zu scratch bytes, the static scratch holds %zu: use marlaas_lora_fwd with a workspace",
                need, (size_t)MARLAAS_STATIC_SCRATCH_BYTES);
  return fwd_impl(ctx, d, y, ldy, u_save, stream, ctx->static_ws, (size_t)MARLAAS_STATIC_SCRATCH_BYTES);
}

// ------------------------------------------------------------------ forward, several projections
// What the projections of one call must share.
static int check_multi(marlaas_ctx* ctx, const marlaas_lora_desc* descs, int32_t n_proj) {
  if (!descs || n_proj < 1 || n_proj > MARLAAS_MAX_PROJ) return fail(ctx, MARLAAS_EINVAL, "n_proj must be 1..%d", MARLAAS_MAX_PROJ);
  for (int p = 0; p < n_proj; ++p) {
    int rc = check_sizes(ctx, &descs[p]);
    if (rc != MARLAAS_OK) return rc;
    const marlaas_lora_desc& a = descs[0];
    const marlaas_lora_desc& b = descs[p];
    if (b.T != a.T || b.d_in != a.d_in || b.x != a.x || b.ldx != a.ldx || b.in_dtype != a.in_dtype ||
        b.out_dtype != a.out_dtype || b.layout != a.layout || b.n_adapters != a.n_adapters || b.map != a.map)
      return fail(ctx, MARLAAS_ESHAPE, "projection %d differs from projection 0 in T, d_in, x, dtypes, layout, n_adapters or map", p);
    if ((b.table == nullptr) != (a.table == nullptr))
      return fail(ctx, MARLAAS_EINVAL, "either every projection or none refers to an adapter table");
  }
  return MARLAAS_OK;
}

// One table object whose projections 0 .. n_proj - 1 are the call's, in order: its combined tables serve the fused pass.
static bool multi_shares_table(const marlaas_lora_desc* descs, int32_t n_proj) {
  if (!descs[0].table || descs[0].table->n_proj != n_proj) return false;
  for (int p = 0; p < n_proj; ++p)
    if (descs[p].table != descs[0].table || descs[p].proj != p) return false;
  return true;
}

static void multi_proj_host(const marlaas_lora_desc* descs, int32_t n_proj, void* const* y, const int64_t* ldy,
                            std::vector<ProjEntry>* out, int* n_ext, bool* mult8) {
  out->assign((size_t)n_proj, ProjEntry());
  memset(out->data(), 0, out->size() * sizeof(ProjEntry));
  int32_t tile0 = 0, fin0 = 0;
  int64_t ext = 0;
  *mult8 = true;
  for (int p = 0; p < n_proj; ++p) {
    ProjEntry& e = (*out)[p];
    e.W = descs[p].W; e.ldw = descs[p].ldw; e.Nout = descs[p].d_out;
    e.out = y ? y[p] : nullptr; e.ldo = ldy ? ldy[p] : 0;
    e.tile0 = tile0; e.fin0 = fin0; e.tab0 = p * descs[p].n_adapters;
    tile0 += (int32_t)((descs[p].d_out + 127) / 128);
    fin0 += (int32_t)((descs[p].d_out + 511) / 512);
    const int32_t* ranks = ranks_of(&descs[p]);
    for (int t = 0; t < descs[p].n_adapters; ++t) { ext += ranks[t]; if (ranks[t] & 7) *mult8 = false; }
  }
  *n_ext = ext > 0x7fffffff ? 0x7fffffff : (int)ext;
}

// Workspace of the fused multi-projection pass: partial sums, then (descriptors without a shared
// table object) the combined tables.
struct MultiPlan { size_t part_bytes = 0, tab_off = 0, tab_bytes = 0, total = 0; int rs = 0; };
static MultiPlan plan_multi(const marlaas_lora_desc* descs, int32_t n_proj, const ProjEntry* proj, int n_ext, bool lora) {
  MultiPlan m;
  m.part_bytes = align_up(gemm_multi_bytes(descs[0].T, descs[0].d_in, proj, n_proj, lora ? n_ext : 0), WS_ALIGN);
  m.tab_off = m.part_bytes;
  if (lora && !multi_shares_table(descs, n_proj))
    m.tab_bytes = dev_tables_bytes((int64_t)n_proj * descs[0].n_adapters, ws_ext_cap(n_ext));
  // the largest rank of any projection: row stride of u where the decode kernel stages it
  for (int p = 0; p < n_proj; ++p) { const int r = (int)marlaas_u_stride(&descs[p]); if (r > m.rs) m.rs = r; }
  m.total = m.tab_off + m.tab_bytes;
  return m;
}

extern "C" size_t marlaas_workspace_bytes_multi(const marlaas_lora_desc* descs, int32_t n_proj) {
  if (check_multi(nullptr, descs, n_proj) != MARLAAS_OK) return 0;
  size_t need = 0;
  for (int p = 0; p < n_proj; ++p) {
    const size_t one = plan_workspace(&descs[p], 0).total;
    if (one > need) need = one;
  }
  if (n_proj > 1 && descs[0].in_dtype == MARLAAS_BF16) {
    std::vector<ProjEntry> proj;
    int n_ext = 0; bool mult8 = true;
    multi_proj_host(descs, n_proj, nullptr, nullptr, &proj, &n_ext, &mult8);
    const bool lora = descs[0].n_adapters > 0 && descs[0].map->T_lora > 0;
    const MultiPlan m = plan_multi(descs, n_proj, proj.data(), n_ext, lora);
    if (m.part_bytes > 0 && m.total > need) need = m.total;
  }
  return need;
}

extern "C" int marlaas_lora_fwd_multi(marlaas_ctx* ctx, const marlaas_lora_desc* descs, int32_t n_proj,
                                      void* const* y, const int64_t* ldy, void* stream) {
  if (!ctx) return MARLAAS_EINVAL;
  int rc = check_multi(ctx, descs, n_proj);
  if (rc != MARLAAS_OK) return rc;
  if (!y || !ldy) return fail(ctx, MARLAAS_EINVAL, "y / ldy arrays are null");
  const marlaas_lora_desc* d0 = &descs[0];
  if (d0->T == 0) return MARLAAS_OK;
  const int64_t osz = d0->out_dtype == MARLAAS_BF16 ? 2 : 4;
  for (int p = 0; p < n_proj; ++p) {
    if ((rc = check_tensors(ctx, &descs[p])) != MARLAAS_OK) return rc;
    if (!y[p]) return fail(ctx, MARLAAS_EINVAL, "y[%d] is null", p);
    if (!aligned16(y[p]) || ldy[p] < descs[p].d_out || (ldy[p] * osz) % 16) return fail(ctx, MARLAAS_EALIGN, "y[%d] / ldy[%d]", p, p);
  }
  const marlaas_segmap* map = d0->map;
  const bool lora = d0->n_adapters > 0 && map->T_lora > 0;
  const int form = d0->layout == MARLAAS_LAYOUT_MATH ? FORM_NN : FORM_NT;
  std::vector<ProjEntry> proj;
  int n_ext = 0; bool mult8 = true;
  multi_proj_host(descs, n_proj, y, ldy, &proj, &n_ext, &mult8);
  if (!lora) n_ext = 0;
  const bool shared = multi_shares_table(descs, n_proj);
  // descriptors that refer to tables, but not to one table in projection order, have no combined tables
  bool fused = n_proj > 1 && d0->in_dtype == MARLAAS_BF16 && ctx->ws != nullptr && (!lora || shared || !d0->table);
  MultiPlan mp;
  if (fused) {
    mp = plan_multi(descs, n_proj, proj.data(), n_ext, lora);
    fused = ctx->ws_bytes >= mp.total && gemm_multi_ok(form, d0->T, d0->d_in, proj.data(), n_proj, n_ext, mult8, mp.part_bytes);
    if (fused && lora && n_ext > (shared ? d0->table->dev.ext_cap : EXT_CAP_MAX)) fused = false;
  }
  if (!fused) {
    // sizes outside the fused path: one projection after the other (same stream, same scratch)
    for (int p = 0; p < n_proj; ++p)
      if ((rc = marlaas_lora_fwd(ctx, &descs[p], y[p], ldy[p], nullptr, stream)) != MARLAAS_OK) return rc;
    return MARLAAS_OK;
  }
  HIP_TRY(ctx, hipSetDevice(ctx->device));
  hipStream_t st = (hipStream_t)stream;
  const int n = d0->n_adapters;
  // combined tables: adapters as [projection][adapter], extended columns over all of them
  const AdapterEntry* table = nullptr;
  GemmFuse fuse;
  if (lora) {
    DevTables all;
    if (shared) {
      all = d0->table->dev;
    } else {
      all = dev_tables_carve((char*)ctx->ws + mp.tab_off, (int64_t)n_proj * n, ws_ext_cap(n_ext));
      std::vector<AdapterEntry> host((size_t)n_proj * n);
      for (int p = 0; p < n_proj; ++p)
        for (int t = 0; t < n; ++t) {
          AdapterEntry& e = host[(size_t)p * n + t];
          e.A = descs[p].A[t]; e.B = descs[p].B[t]; e.rank = descs[p].ranks[t]; e.scale = descs[p].scales[t];
        }
      HIP_TRY(ctx, enqueue_write_entries(all, 0, (int64_t)n_proj * n, host.data(), st));
      HIP_TRY(ctx, enqueue_derive(all, (int64_t)n_proj * n, st));
    }
    table = all.entries;
    fuse.roff = all.roff; fuse.cols = all.cols;
    fuse.n_ext = n_ext; fuse.ranks_mult8 = mult8; fuse.u_out = nullptr; fuse.t0 = 0; fuse.ext_base = 0;
  }
  const int32_t* perm = map->identity ? nullptr : map->perm_dev;
  // packed copies of every projection's weight (and factors stored contraction-contiguous, or no
  // adapters): the decode kernel reads those
  bool packed = !lora || form == FORM_NT;
  for (int p = 0; p < n_proj; ++p) if (!descs[p].W_packed_fwd) packed = false;
  if (packed)
    for (int p = 0; p < n_proj; ++p) { proj[p].W = descs[p].W_packed_fwd; proj[p].ldw = packed_weight_ksteps(d0->d_in); }
  const DecodeSync dsync = decode_sync_of(ctx, map);
  PROFILED(ctx, MARLAAS_KERNEL_GEMM, st, launch_gemm_bf16_multi((const bf16_t*)d0->x, d0->ldx, form, d0->T, d0->d_in, perm,
                                      map->seg_off_dev, n, table, proj.data(), n_proj,
                                      d0->out_dtype == MARLAAS_F32, (float*)ctx->ws, mp.part_bytes, map->chunks_dev,
                                      map->n_chunks, lora ? &fuse : nullptr, packed ? 1 : 0, &dsync, mp.rs, st));
  return MARLAAS_OK;
}

// ------------------------------------------------------------------ backward
// opt: optimizer steps in place of gradient outputs (both reductions then end in the update of the
// factor they differentiate; opt[0] for A, opt[1] for B), or null
static int bwd_impl(marlaas_ctx* ctx, const marlaas_lora_desc* d, const void* dY, int64_t lddy,
                    const void* u_saved, void* dX, int64_t lddx, void* const* dA,
                    void* const* dB, int accumulate, const ReduceOpt* opt, void* stream) {
  if (!ctx) return MARLAAS_EINVAL;
  int rc = check_sizes(ctx, d);
  if (rc != MARLAAS_OK) return rc;
  const bool grads_in_table = dA == MARLAAS_GRADS_IN_TABLE || dB == MARLAAS_GRADS_IN_TABLE;
  if (grads_in_table && (dA != dB || !d->table))
    return fail(ctx, MARLAAS_EINVAL, "MARLAAS_GRADS_IN_TABLE must be passed for both dA and dB, with a descriptor that has an adapter table");
  const bool want_grads = dA != nullptr || dB != nullptr || opt != nullptr;
  if (!opt && want_grads && (!dA || !dB)) return fail(ctx, MARLAAS_EINVAL, "dA and dB must both be given or both be null");
  if (accumulate != 0 && accumulate != 1) return fail(ctx, MARLAAS_EINVAL, "accumulate must be 0 or 1");
  if ((rc = check_tensors(ctx, d)) != MARLAAS_OK) return rc;
  const int64_t esz = d->in_dtype == MARLAAS_BF16 ? 2 : 4;
  const int64_t osz = d->out_dtype == MARLAAS_BF16 ? 2 : 4;
  if (d->T > 0) {
    if (!dY) return fail(ctx, MARLAAS_EINVAL, "dY is null");
    if (!aligned16(dY) || lddy < d->d_out || (lddy * esz) % 16) return fail(ctx, MARLAAS_EALIGN, "dY / lddy");
    if (dX && (!aligned16(dX) || lddx < d->d_in || (lddx * osz) % 16)) return fail(ctx, MARLAAS_EALIGN, "dX / lddx");
    if (u_saved && !aligned16(u_saved)) return fail(ctx, MARLAAS_EALIGN, "u_saved must be 16-byte aligned");
  }
  if (grads_in_table) {
    const marlaas_adapter_table* tb = d->table;
    for (int t = 0; t < d->n_adapters; ++t) {
      const size_t i = (size_t)d->proj * tb->n + t;
      if (tb->hranks[i] > 0 && !tb->hgrads[i].dA)
        return fail(ctx, MARLAAS_EINVAL, "adapter %d was registered without gradient buffers", t);
    }
  } else if (want_grads && !opt) {
    for (int t = 0; t < d->n_adapters; ++t)
      if (!dA[t] || !dB[t] || !aligned16(dA[t]) || !aligned16(dB[t]))
        return fail(ctx, MARLAAS_EINVAL, "gradient buffers of adapter %d are null or misaligned", t);
  }
  if (d->T == 0 && !(want_grads && !accumulate && d->n_adapters > 0)) return MARLAAS_OK;
  HIP_TRY(ctx, hipSetDevice(ctx->device));
  hipStream_t st = (hipStream_t)stream;
  const marlaas_segmap* map = d->map;
  const int rs = (int)marlaas_u_stride(d);
  const bool lora = d->n_adapters > 0 && map->T_lora > 0;
  WsPlan p = plan_workspace(d, 1);
  if (d->n_adapters > 0 && (!ctx->ws || ctx->ws_bytes < p.total))
    return fail(ctx, MARLAAS_ENOMEM, "backward needs %zu workspace bytes, have %zu", p.total, ctx->ws_bytes);
  float* u = (float*)u_saved;
  float* v = d->n_adapters > 0 ? (float*)((char*)ctx->ws + p.v_off) : nullptr;
  const bool need_u = lora && want_grads && !u;
  if (need_u) u = (float*)((char*)ctx->ws + p.u_off);
  Bank bank;
  if (d->n_adapters > 0 && (rc = resolve_bank(ctx, d, (char*)ctx->ws + p.tab_off, p.tab_bytes, st, &bank)) != MARLAAS_OK) return rc;
  const AdapterEntry* table = bank.entries;
  const GradEntry* grads = bank.grads;
  if (want_grads && !opt && !grads_in_table && d->n_adapters > 0) {
    // explicit gradient pointer lists belong to descriptors that carry their own A / B lists; the
    // per-call copy of the tables in the workspace receives them
    if (!bank.in_ws)
      return fail(ctx, MARLAAS_EINVAL, "with an adapter table, register the gradient buffers in the table and pass MARLAAS_GRADS_IN_TABLE");
    std::vector<GradEntry> host((size_t)d->n_adapters);
    for (int t = 0; t < d->n_adapters; ++t) { host[t].dA = (float*)dA[t]; host[t].dB = (float*)dB[t]; }
    HIP_TRY(ctx, enqueue_write_grads(bank.all, 0, d->n_adapters, host.data(), st));
  }
  const int32_t* perm = map->identity ? nullptr : map->perm_dev;
  // forward-side forms (contraction over d_in) and backward-side forms (contraction over d_out)
  const int fform = d->layout == MARLAAS_LAYOUT_MATH ? FORM_NN : FORM_NT;
  const int bform = d->layout == MARLAAS_LAYOUT_MATH ? FORM_NT : FORM_NN;
  // gradients keep the orientation of their factor: math dA[d_in,r] / torch dB[d_out,r] are
  // [wide, r] (NN), math dB[r,d_out] / torch dA[r,d_in] are [r, wide] (NT)
  const int da_form = d->layout == MARLAAS_LAYOUT_MATH ? FORM_NN : FORM_NT;
  const int db_form = d->layout == MARLAAS_LAYOUT_MATH ? FORM_NT : FORM_NN;
  const int out_f32 = d->out_dtype == MARLAAS_F32;
  const bool have_ws = ctx->ws && ctx->ws_bytes >= p.total;
  float* part = (have_ws && p.part_bytes) ? (float*)((char*)ctx->ws + p.part_off) : nullptr;
  const DecodeSync dsync = decode_sync_of(ctx, map);
  if (d->in_dtype == MARLAAS_BF16) {
    const bf16_t* x = (const bf16_t*)d->x;
    const bf16_t* dy = (const bf16_t*)dY;
    if (need_u)
      PROFILED(ctx, MARLAAS_KERNEL_SHRINK, st, launch_shrink_bf16(x, d->ldx, d->d_in, perm, map->seg_off_dev, d->n_adapters, map->max_seg,
                                      table, 0, fform, u, rs, map->T_lora, part, part ? p.part_bytes : 0, nullptr, nullptr, (const bf16_t*)ctx->zero_dev, bank.mult8, st));
    // small batches: the dX GEMM computes v itself (and leaves it in `v` for the dA reduction)
    GemmFuse fuse;
    bool fused = false;
    if (lora && dX && part && bank_can_fuse(bank)) {
      fused = gemm_can_fuse_shrink(bform, d->T, d->d_out, d->d_in, bank.n_ext, bank.mult8, p.part_bytes);
      if (fused) {
        if ((rc = bank_fuse(ctx, bank, d->n_adapters, st, &fuse)) != MARLAAS_OK) return rc;
        fuse.u_out = v;
      }
    }
    bool have_v2 = false;
    bf16_t* v2 = (have_ws && p.uv2_bytes && dX) ? (bf16_t*)((char*)ctx->ws + p.v2_off) : nullptr;
    if (lora && (dX || want_grads) && !fused)
      PROFILED(ctx, MARLAAS_KERNEL_SHRINK, st, launch_shrink_bf16(dy, lddy, d->d_out, perm, map->seg_off_dev, d->n_adapters, map->max_seg,
                                      table, 1, bform, v, rs, map->T_lora, part, part ? p.part_bytes : 0, v2, &have_v2, (const bf16_t*)ctx->zero_dev, bank.mult8, st));
    LoraDma dma;
    if (have_v2 && p.lt_bytes) {
      dma.u2 = v2; dma.tiles = (int32_t*)((char*)ctx->ws + p.lt_off); dma.tiles_bytes = p.lt_bytes;
      dma.zero_line = (const bf16_t*)ctx->zero_dev; dma.ranks_mult8 = bank.mult8;
    }
    if (dX && d->T > 0)
      PROFILED(ctx, MARLAAS_KERNEL_GEMM, st, launch_gemm_bf16(dy, lddy, (const bf16_t*)d->W, d->ldw, bform, d->T, d->d_out, d->d_in, perm,
                                    map->seg_off_dev, d->n_adapters, table, 0, lora ? v : nullptr, rs, dX, lddx,
                                    out_f32, part, part ? p.part_bytes : 0, map->chunks_dev, map->n_chunks,
                                    fused ? &fuse : nullptr, (have_ws && p.wt_bytes) ? (bf16_t*)((char*)ctx->ws + p.wt_off) : nullptr,
                                    p.wt_bytes, d->layout == MARLAAS_LAYOUT_TORCH ? (const bf16_t*)d->W_t : nullptr, &dma, (const bf16_t*)d->W_packed_bwd, &dsync, st));
    if (want_grads && d->n_adapters > 0) {
      PROFILED(ctx, MARLAAS_KERNEL_REDUCE, st, launch_reduce_bf16(dy, lddy, d->d_out, perm, map->seg_off_dev, d->n_adapters, map->max_seg,
                                      table, grads, 1, db_form, u, rs, accumulate, part, part ? p.part_bytes : 0, opt ? &opt[1] : nullptr, map->order_dev, map->chunk_base_dev,
                                      map->ragged_chunk, map->ragged_slots, map->ragged_adapters, st));
      PROFILED(ctx, MARLAAS_KERNEL_REDUCE, st, launch_reduce_bf16(x, d->ldx, d->d_in, perm, map->seg_off_dev, d->n_adapters, map->max_seg,
                                      table, grads, 0, da_form, v, rs, accumulate, part, part ? p.part_bytes : 0, opt ? &opt[0] : nullptr, map->order_dev, map->chunk_base_dev,
                                      map->ragged_chunk, map->ragged_slots, map->ragged_adapters, st));
    }
  } else {
    if (opt) return fail(ctx, MARLAAS_EUNSUPPORTED, "the optimizer step is attached to the bf16 backward only");
    const float* x = (const float*)d->x;
    const float* dy = (const float*)dY;
    if (need_u)
      PROFILED(ctx, MARLAAS_KERNEL_SHRINK, st, launch_shrink_f32(x, d->ldx, d->d_in, perm, map->seg_off_dev, d->n_adapters, table, 0, fform,
                                     u, rs, map->T_lora, st));
    if (lora && (dX || want_grads))
      PROFILED(ctx, MARLAAS_KERNEL_SHRINK, st, launch_shrink_f32(dy, lddy, d->d_out, perm, map->seg_off_dev, d->n_adapters, table, 1, bform,
                                     v, rs, map->T_lora, st));
    if (dX && d->T > 0)
      PROFILED(ctx, MARLAAS_KERNEL_GEMM, st, launch_gemm_f32(dy, lddy, (const float*)d->W, d->ldw, bform, d->T, d->d_out, d->d_in, perm,
                                   map->seg_off_dev, d->n_adapters, table, 0, lora ? v : nullptr, rs, dX, lddx,
                                   out_f32, st));
    if (want_grads && d->n_adapters > 0) {
      PROFILED(ctx, MARLAAS_KERNEL_REDUCE, st, launch_reduce_f32(dy, lddy, d->d_out, perm, map->seg_off_dev, d->n_adapters, table, grads, 1,
                                     db_form, u, rs, accumulate, st));
      PROFILED(ctx, MARLAAS_KERNEL_REDUCE, st, launch_reduce_f32(x, d->ldx, d->d_in, perm, map->seg_off_dev, d->n_adapters, table, grads, 0,
                                     da_form, v, rs, accumulate, st));
    }
  }
  return MARLAAS_OK;
}

extern "C" int marlaas_lora_bwd(marlaas_ctx* ctx, const marlaas_lora_desc* d, const void* dY, int64_t lddy,
                                const void* u_saved, void* dX, int64_t lddx, void* const* dA,
                                void* const* dB, int accumulate, void* stream) {
  return bwd_impl(ctx, d, dY, lddy, u_saved, dX, lddx, dA, dB, accumulate, nullptr, stream);
}

extern "C" int marlaas_lora_bwd_adamw(marlaas_ctx* ctx, const marlaas_lora_desc* d, const void* dY, int64_t lddy,
                                      const void* u_saved, void* dX, int64_t lddx,
                                      const marlaas_adapter_state* states, const marlaas_adamw* hp, void* stream) {
  if (!ctx) return MARLAAS_EINVAL;
  if (!d || !states || !hp) return fail(ctx, MARLAAS_EINVAL, "descriptor, states and hyper-parameters must be given");
  if (d->n_adapters < 1 || d->n_adapters > OPT_MAX_ADAPTERS)
    return fail(ctx, MARLAAS_EUNSUPPORTED, "the fused optimizer step takes 1..%d adapters (one task is trained per update)", OPT_MAX_ADAPTERS);
  if (d->in_dtype != MARLAAS_BF16) return fail(ctx, MARLAAS_EUNSUPPORTED, "the optimizer step is attached to the bf16 backward only");
  if (hp->step < 1 || !(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f) || !(hp->eps >= 0.f))
    return fail(ctx, MARLAAS_EINVAL, "step must be >= 1, beta1 and beta2 in [0, 1), eps >= 0");
  ReduceOpt opt[2];
  for (int w = 0; w < 2; ++w) {
    opt[w].on = 1;
    opt[w].lr = hp->lr; opt[w].beta1 = hp->beta1; opt[w].beta2 = hp->beta2; opt[w].eps = hp->eps; opt[w].wd = hp->weight_decay;
    opt[w].inv_c1 = (float)(1.0 / (1.0 - std::pow((double)hp->beta1, (double)hp->step)));
    opt[w].inv_c2 = (float)(1.0 / (1.0 - std::pow((double)hp->beta2, (double)hp->step)));
    for (int t = 0; t < OPT_MAX_ADAPTERS; ++t) opt[w].f[t] = OptFactor{nullptr, nullptr, nullptr, nullptr};
  }
  for (int t = 0; t < d->n_adapters; ++t) {
    const marlaas_adapter_state& s = states[t];
    if (!s.master_A || !s.master_B || !s.m_A || !s.v_A || !s.m_B || !s.v_B || !s.A_next || !s.B_next)
      return fail(ctx, MARLAAS_EINVAL, "state of adapter %d has a null pointer", t);
    opt[0].f[t] = OptFactor{s.master_A, s.m_A, s.v_A, (bf16_t*)s.A_next};
    opt[1].f[t] = OptFactor{s.master_B, s.m_B, s.v_B, (bf16_t*)s.B_next};
  }
  return bwd_impl(ctx, d, dY, lddy, u_saved, dX, lddx, nullptr, nullptr, 0, opt, stream);
}
