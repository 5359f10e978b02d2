// Host side of the C ABI: contexts, argument checks, the token grouping
// object, cached device copies of the per-adapter pointer tables, workspace
// carving and the order in which the kernels of a forward / backward pass are
// enqueued.  Nothing here computes on tensors.
#include "../../include/marlaas_lora.h"
#include "common.h"

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <list>
#include <new>
#include <string>
#include <vector>

using namespace marlaas;

struct TableSlot {
  std::string key;       // raw bytes of the host-side table
  void* dev = nullptr;
};

struct marlaas_ctx {
  int device = 0;
  void* ws = nullptr;
  size_t ws_bytes = 0;
  std::string err;
  std::list<TableSlot> tables;   // most recently used first
  bool profile = false;
  struct Span { int kernel; hipEvent_t beg, end; };
  std::vector<Span> spans;       // event pairs recorded while profiling is on
};

struct marlaas_segmap {
  int device = 0;
  int64_t T = 0;
  int32_t n = 0;
  int32_t* perm_dev = nullptr;      // [T] grouped order (always built)
  int32_t* seg_off_dev = nullptr;   // [n + 2]
  std::vector<int32_t> seg_off;     // host copy
  bool identity = false;            // ids were already grouped: kernels skip the gather
  int max_seg = 0;                  // largest adapter segment
  int64_t T_lora = 0;               // tokens that have an adapter
  RowChunk* chunks_dev = nullptr;   // row chunks of the grouped order (see RowChunk)
  int n_chunks = 0;
};

static const size_t TABLE_CACHE_SLOTS = 512;
static const size_t WS_ALIGN = 256;

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
  if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return MARLAAS_EHIP;
  marlaas_ctx* ctx = new (std::nothrow) marlaas_ctx();
  if (!ctx) return MARLAAS_ENOMEM;
  ctx->device = device;
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
  for (auto& s : ctx->tables) (void)hipFree(s.dev);
  delete ctx;
}

// Device copy of a small host table, cached by content so that the steady
// state (the same layers called every step) uploads nothing.
static int cached_table(marlaas_ctx* ctx, const void* host, size_t bytes, const void** dev) {
  std::string key((const char*)host, bytes);
  for (auto it = ctx->tables.begin(); it != ctx->tables.end(); ++it) {
    if (it->key == key) {
      ctx->tables.splice(ctx->tables.begin(), ctx->tables, it);
      *dev = ctx->tables.front().dev;
      return MARLAAS_OK;
    }
  }
  if (ctx->tables.size() >= TABLE_CACHE_SLOTS) {
    HIP_TRY(ctx, hipDeviceSynchronize());   // a kernel in flight may still read the victim
    (void)hipFree(ctx->tables.back().dev);
    ctx->tables.pop_back();
  }
  TableSlot s;
  s.key.swap(key);
  HIP_TRY(ctx, hipMalloc(&s.dev, bytes));
  hipError_t e = hipMemcpy(s.dev, host, bytes, hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    (void)hipFree(s.dev);
    return fail(ctx, MARLAAS_EHIP, "table upload failed: %s", hipGetErrorString(e));
  }
  ctx->tables.push_front(std::move(s));
  *dev = ctx->tables.front().dev;
  return MARLAAS_OK;
}

// ------------------------------------------------------------------ segmap
extern "C" int marlaas_segmap_build(marlaas_ctx* ctx, const int32_t* token_adapter, int64_t T,
                                    int32_t n_adapters, void* stream, marlaas_segmap** out) {
  if (!ctx) return MARLAAS_EINVAL;
  if (!out) return fail(ctx, MARLAAS_EINVAL, "segmap_build: out is null");
  *out = nullptr;
  if (T < 0 || T > 0x7fffffff - 4096) return fail(ctx, MARLAAS_EINVAL, "segmap_build: T=%lld out of range", (long long)T);
  if (n_adapters < 0 || n_adapters > MARLAAS_MAX_ADAPTERS)
    return fail(ctx, MARLAAS_EINVAL, "segmap_build: n_adapters=%d out of range", n_adapters);
  if (T > 0 && !token_adapter) return fail(ctx, MARLAAS_EINVAL, "segmap_build: token_adapter is null");
  HIP_TRY(ctx, hipSetDevice(ctx->device));
  hipStream_t st = (hipStream_t)stream;
  marlaas_segmap* m = new (std::nothrow) marlaas_segmap();
  if (!m) return fail(ctx, MARLAAS_ENOMEM, "segmap_build: host allocation failed");
  m->device = ctx->device; m->T = T; m->n = n_adapters;
  const int nblk = segmap_blocks(T);
  int32_t* block_hist = nullptr;
  int32_t* flags = nullptr;
  int status = MARLAAS_OK;
  int32_t hflags[2] = {0, 0};
  m->seg_off.assign((size_t)n_adapters + 2, 0);
  hipError_t e = hipSuccess;
  do {
    if ((e = hipMalloc((void**)&m->perm_dev, sizeof(int32_t) * (size_t)(T > 0 ? T : 1))) != hipSuccess) break;
    if ((e = hipMalloc((void**)&m->seg_off_dev, sizeof(int32_t) * ((size_t)n_adapters + 2))) != hipSuccess) break;
    if ((e = hipMalloc((void**)&block_hist, sizeof(int32_t) * (size_t)(nblk > 0 ? nblk : 1) * ((size_t)n_adapters + 1))) != hipSuccess) break;
    if ((e = hipMalloc((void**)&flags, 2 * sizeof(int32_t))) != hipSuccess) break;
    if ((e = launch_segmap(token_adapter, T, n_adapters, m->perm_dev, m->seg_off_dev, block_hist, flags, st)) != hipSuccess) break;
    if ((e = hipMemcpyAsync(hflags, flags, sizeof hflags, hipMemcpyDeviceToHost, st)) != hipSuccess) break;
    if ((e = hipMemcpyAsync(m->seg_off.data(), m->seg_off_dev, sizeof(int32_t) * m->seg_off.size(), hipMemcpyDeviceToHost, st)) != hipSuccess) break;
    e = hipStreamSynchronize(st);
  } while (0);
  (void)hipFree(block_hist);
  (void)hipFree(flags);
  if (e != hipSuccess) status = fail(ctx, MARLAAS_EHIP, "segmap_build: %s", hipGetErrorString(e));
  else if (hflags[0]) status = fail(ctx, MARLAAS_EINVAL, "segmap_build: token id outside [-1, %d)", n_adapters);
  if (status != MARLAAS_OK) { marlaas_segmap_destroy(m); return status; }
  m->identity = hflags[1] == 0;
  for (int t = 0; t < n_adapters; ++t) {
    int len = m->seg_off[t + 1] - m->seg_off[t];
    if (len > m->max_seg) m->max_seg = len;
  }
  m->T_lora = m->seg_off[n_adapters];
  // row chunks: segment t split into pieces of ROW_CHUNK rows; the rows without an adapter last
  std::vector<RowChunk> chunks;
  for (int t = 0; t <= n_adapters; ++t) {
    const int32_t end = t < n_adapters ? m->seg_off[t + 1] : (int32_t)T;
    for (int32_t row0 = m->seg_off[t]; row0 < end; row0 += ROW_CHUNK) {
      RowChunk c;
      c.row0 = row0; c.nrows = end - row0 < ROW_CHUNK ? end - row0 : ROW_CHUNK; c.t = t < n_adapters ? t : -1; c.pad = 0;
      chunks.push_back(c);
    }
  }
  m->n_chunks = (int)chunks.size();
  if (m->n_chunks > 0) {
    e = hipMalloc((void**)&m->chunks_dev, sizeof(RowChunk) * chunks.size());
    if (e == hipSuccess) e = hipMemcpy(m->chunks_dev, chunks.data(), sizeof(RowChunk) * chunks.size(), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
      status = fail(ctx, MARLAAS_EHIP, "segmap_build: %s", hipGetErrorString(e));
      marlaas_segmap_destroy(m);
      return status;
    }
  }
  *out = m;
  return MARLAAS_OK;
}

extern "C" void marlaas_segmap_destroy(marlaas_segmap* map) {
  if (!map) return;
  (void)hipSetDevice(map->device);
  (void)hipFree(map->perm_dev);
  (void)hipFree(map->seg_off_dev);
  (void)hipFree(map->chunks_dev);
  delete map;
}

extern "C" int marlaas_segmap_export(const marlaas_segmap* map, int32_t* perm, int32_t* seg_off) {
  if (!map) return MARLAAS_EINVAL;
  if (seg_off) memcpy(seg_off, map->seg_off.data(), sizeof(int32_t) * map->seg_off.size());
  if (perm && map->T > 0) {
    if (hipSetDevice(map->device) != hipSuccess) return MARLAAS_EHIP;
    if (hipMemcpy(perm, map->perm_dev, sizeof(int32_t) * (size_t)map->T, hipMemcpyDeviceToHost) != hipSuccess)
      return MARLAAS_EHIP;
  }
  return MARLAAS_OK;
}

// ------------------------------------------------------------------ descriptor checks
static int max_rank_of(const marlaas_lora_desc* d) {
  int mr = 0;
  for (int t = 0; t < d->n_adapters; ++t) if (d->ranks[t] > mr) mr = d->ranks[t];
  return mr;
}

static int sum_ranks_of(const marlaas_lora_desc* d) {
  int64_t sum = 0;
  for (int t = 0; t < d->n_adapters; ++t) sum += d->ranks[t];
  return sum > 0x7fffffff ? 0x7fffffff : (int)sum;
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
  if (d->n_adapters > 0) {
    if (!d->ranks || !d->scales) return fail(ctx, MARLAAS_EINVAL, "ranks / scales are null");
    for (int t = 0; t < d->n_adapters; ++t)
      if (d->ranks[t] < 1 || d->ranks[t] > MARLAAS_MAX_RANK)
        return fail(ctx, MARLAAS_EINVAL, "rank of adapter %d is %d, must be 1..%d", t, d->ranks[t], MARLAAS_MAX_RANK);
  }
  if (!d->map) return fail(ctx, MARLAAS_EINVAL, "segment map is null");
  if (d->map->T != d->T || d->map->n != d->n_adapters)
    return fail(ctx, MARLAAS_ESHAPE, "segment map was built for T=%lld, n=%d", (long long)d->map->T, d->map->n);
  return MARLAAS_OK;
}

extern "C" int64_t marlaas_u_stride(const marlaas_lora_desc* d) {
  if (!d || d->n_adapters < 0 || d->n_adapters > MARLAAS_MAX_ADAPTERS) return 0;
  if (d->n_adapters == 0) return 16;
  if (!d->ranks) return 0;
  int mr = max_rank_of(d);
  if (mr < 1 || mr > MARLAAS_MAX_RANK) return 0;
  return (mr + 15) & ~15;
}

struct WsPlan {
  size_t u_off = 0, v_off = 0, part_off = 0, part_bytes = 0, total = 0;   // part: reused by every kernel with partial sums
  size_t wt_off = 0, wt_bytes = 0;   // transposed copy of the weight (large batches, output-contiguous storage)
};

static WsPlan plan_workspace(const marlaas_lora_desc* d, int want_bwd) {
  WsPlan p;
  const size_t rs = (size_t)marlaas_u_stride(d);
  const size_t uv = align_up((size_t)(d->T > 0 ? d->T : 1) * rs * sizeof(float), WS_ALIGN);
  size_t off = 0;
  p.u_off = off; off += uv;
  size_t part = 0;
  const int n_ext = sum_ranks_of(d);
  if (d->in_dtype == MARLAAS_BF16) part = gemm_splitk_bytes(d->T, d->d_in, d->d_out, n_ext);
  if (want_bwd) {
    p.v_off = off; off += uv;
    if (d->in_dtype == MARLAAS_BF16) {
      const size_t pa = reduce_partial_bytes(d->d_in, d->n_adapters, d->map->max_seg, (int)rs);
      const size_t pb = reduce_partial_bytes(d->d_out, d->n_adapters, d->map->max_seg, (int)rs);
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
    p.wt_bytes = align_up(wt, WS_ALIGN);
    p.wt_off = off; off += p.wt_bytes;
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
  if (d->ldx < d->d_in || (d->ldx * esz) % 16) return fail(ctx, MARLAAS_EALIGN, "ldx=%lld", (long long)d->ldx);
  const int64_t wcols = d->layout == MARLAAS_LAYOUT_MATH ? d->d_out : d->d_in;
  if (d->ldw < wcols || (d->ldw * esz) % 16) return fail(ctx, MARLAAS_EALIGN, "ldw=%lld", (long long)d->ldw);
  if (d->ldw > (1 << 22)) return fail(ctx, MARLAAS_EINVAL, "ldw=%lld is above 4194304", (long long)d->ldw);
  if (d->n_adapters > 0) {
    if (!d->A || !d->B) return fail(ctx, MARLAAS_EINVAL, "A / B pointer arrays are null");
    for (int t = 0; t < d->n_adapters; ++t) {
      if (!d->A[t] || !d->B[t]) return fail(ctx, MARLAAS_EINVAL, "adapter %d has a null factor", t);
      if (!aligned16(d->A[t]) || !aligned16(d->B[t])) return fail(ctx, MARLAAS_EALIGN, "adapter %d factors must be 16-byte aligned", t);
    }
  }
  return MARLAAS_OK;
}

static int adapter_table(marlaas_ctx* ctx, const marlaas_lora_desc* d, const AdapterEntry** dev) {
  *dev = nullptr;
  if (d->n_adapters == 0) return MARLAAS_OK;
  std::vector<AdapterEntry> host((size_t)d->n_adapters);
  memset(host.data(), 0, host.size() * sizeof(AdapterEntry));
  for (int t = 0; t < d->n_adapters; ++t) {
    host[t].A = d->A[t]; host[t].B = d->B[t]; host[t].rank = d->ranks[t]; host[t].scale = d->scales[t];
  }
  return cached_table(ctx, host.data(), host.size() * sizeof(AdapterEntry), (const void**)dev);
}

// Tables of the fused shrink: rank offsets and the (adapter, rank index) of every extended column.
static int fuse_tables(marlaas_ctx* ctx, const marlaas_lora_desc* d, GemmFuse* f) {
  const int n = d->n_adapters;
  std::vector<int32_t> host((size_t)n + 1);
  bool mult8 = true;
  int32_t off = 0;
  for (int t = 0; t < n; ++t) { host[t] = off; off += d->ranks[t]; if (d->ranks[t] & 7) mult8 = false; }
  host[n] = off;
  // offsets padded to an even count, so that the column pairs that follow stay 8-byte aligned
  if (host.size() & 1) host.push_back(0);
  const size_t cols_at = host.size();
  host.resize(cols_at + 2 * (size_t)off);
  for (int t = 0, e = 0; t < n; ++t)
    for (int q = 0; q < d->ranks[t]; ++q, ++e) { host[cols_at + 2 * e] = t; host[cols_at + 2 * e + 1] = q; }
  const void* dev = nullptr;
  int rc = cached_table(ctx, host.data(), host.size() * sizeof(int32_t), &dev);
  if (rc != MARLAAS_OK) return rc;
  f->roff = (const int32_t*)dev;
  f->cols = (const ExtCol*)((const int32_t*)dev + cols_at);
  f->n_ext = off;
  f->ranks_mult8 = mult8;
  f->u_out = nullptr;
  return MARLAAS_OK;
}

// ------------------------------------------------------------------ forward
extern "C" int marlaas_lora_fwd(marlaas_ctx* ctx, const marlaas_lora_desc* d, void* y, int64_t ldy,
                                void* u_save, void* stream) {
  if (!ctx) return MARLAAS_EINVAL;
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
  const bool have_ws = ctx->ws && ctx->ws_bytes >= p.total;
  if (lora && !u) {
    if (!have_ws)
      return fail(ctx, MARLAAS_ENOMEM, "forward needs %zu workspace bytes, have %zu", p.total, ctx->ws_bytes);
    u = (float*)((char*)ctx->ws + p.u_off);
  }
  float* part = (have_ws && p.part_bytes) ? (float*)((char*)ctx->ws + p.part_off) : nullptr;
  const AdapterEntry* table = nullptr;
  if ((rc = adapter_table(ctx, d, &table)) != MARLAAS_OK) return rc;
  const int32_t* perm = map->identity ? nullptr : map->perm_dev;
  // forward contracts over d_in: math W[d_in,d_out] is [contraction, output] (NN), torch is NT;
  // A_t follows W for the shrink, B_t follows W for the expand.
  const int form = d->layout == MARLAAS_LAYOUT_MATH ? FORM_NN : FORM_NT;
  const int out_f32 = d->out_dtype == MARLAAS_F32;
  if (d->in_dtype == MARLAAS_BF16) {
    // small batches: the GEMM computes the shrink itself and no shrink kernel runs
    GemmFuse fuse;
    bool fused = false;
    if (lora && part) {
      const int n_ext = sum_ranks_of(d);
      bool mult8 = true;
      for (int t = 0; t < d->n_adapters; ++t) if (d->ranks[t] & 7) mult8 = false;
      fused = gemm_can_fuse_shrink(form, d->T, d->d_in, d->d_out, n_ext, mult8, p.part_bytes);
      if (fused) {
        if ((rc = fuse_tables(ctx, d, &fuse)) != MARLAAS_OK) return rc;
        fuse.u_out = u;
      }
    }
    if (lora && !fused)
      PROFILED(ctx, MARLAAS_KERNEL_SHRINK, st, launch_shrink_bf16((const bf16_t*)d->x, d->ldx, d->d_in, perm, map->seg_off_dev, d->n_adapters,
                                      map->max_seg, table, 0, form, u, rs, map->T_lora, st));
    PROFILED(ctx, MARLAAS_KERNEL_GEMM, st, launch_gemm_bf16((const bf16_t*)d->x, d->ldx, (const bf16_t*)d->W, d->ldw, form, d->T, d->d_in,
                                  d->d_out, perm, map->seg_off_dev, d->n_adapters, table, 1, lora ? u : nullptr,
                                  rs, y, ldy, out_f32, part, part ? p.part_bytes : 0, map->chunks_dev, map->n_chunks,
                                  fused ? &fuse : nullptr, (have_ws && p.wt_bytes) ? (bf16_t*)((char*)ctx->ws + p.wt_off) : nullptr,
                                  p.wt_bytes, st));
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
  }
  return MARLAAS_OK;
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
    for (int t = 0; t < descs[p].n_adapters; ++t) { ext += descs[p].ranks[t]; if (descs[p].ranks[t] & 7) *mult8 = false; }
  }
  *n_ext = ext > 0x7fffffff ? 0x7fffffff : (int)ext;
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
    const size_t fused = align_up(gemm_multi_bytes(descs[0].T, descs[0].d_in, proj.data(), n_proj, lora ? n_ext : 0), WS_ALIGN);
    if (fused > need) need = fused;
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
  bool fused = n_proj > 1 && d0->in_dtype == MARLAAS_BF16 && ctx->ws != nullptr;
  if (fused) fused = gemm_multi_ok(form, d0->T, d0->d_in, proj.data(), n_proj, n_ext, mult8, ctx->ws_bytes);
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
    std::vector<AdapterEntry> host((size_t)n_proj * n);
    memset(host.data(), 0, host.size() * sizeof(AdapterEntry));
    for (int p = 0; p < n_proj; ++p)
      for (int t = 0; t < n; ++t) {
        AdapterEntry& e = host[(size_t)p * n + t];
        e.A = descs[p].A[t]; e.B = descs[p].B[t]; e.rank = descs[p].ranks[t]; e.scale = descs[p].scales[t];
      }
    if ((rc = cached_table(ctx, host.data(), host.size() * sizeof(AdapterEntry), (const void**)&table)) != MARLAAS_OK) return rc;
    std::vector<int32_t> ft((size_t)n_proj * n + 1);
    int32_t off = 0;
    for (int p = 0; p < n_proj; ++p)
      for (int t = 0; t < n; ++t) { ft[(size_t)p * n + t] = off; off += descs[p].ranks[t]; }
    ft[(size_t)n_proj * n] = off;
    if (ft.size() & 1) ft.push_back(0);
    const size_t cols_at = ft.size();
    ft.resize(cols_at + 2 * (size_t)off);
    size_t e = 0;
    for (int p = 0; p < n_proj; ++p)
      for (int t = 0; t < n; ++t)
        for (int q = 0; q < descs[p].ranks[t]; ++q, ++e) { ft[cols_at + 2 * e] = p * n + t; ft[cols_at + 2 * e + 1] = q; }
    const void* dev = nullptr;
    if ((rc = cached_table(ctx, ft.data(), ft.size() * sizeof(int32_t), &dev)) != MARLAAS_OK) return rc;
    fuse.roff = (const int32_t*)dev;
    fuse.cols = (const ExtCol*)((const int32_t*)dev + cols_at);
    fuse.n_ext = off; fuse.ranks_mult8 = mult8; fuse.u_out = nullptr;
  }
  const ProjEntry* proj_dev = nullptr;
  if ((rc = cached_table(ctx, proj.data(), proj.size() * sizeof(ProjEntry), (const void**)&proj_dev)) != MARLAAS_OK) return rc;
  const int32_t* perm = map->identity ? nullptr : map->perm_dev;
  PROFILED(ctx, MARLAAS_KERNEL_GEMM, st, launch_gemm_bf16_multi((const bf16_t*)d0->x, d0->ldx, form, d0->T, d0->d_in, perm,
                                      map->seg_off_dev, n, table, proj.data(), proj_dev, n_proj,
                                      d0->out_dtype == MARLAAS_F32, (float*)ctx->ws, ctx->ws_bytes, map->chunks_dev,
                                      map->n_chunks, lora ? &fuse : nullptr, st));
  return MARLAAS_OK;
}

// ------------------------------------------------------------------ backward
extern "C" int marlaas_lora_bwd(marlaas_ctx* ctx, const marlaas_lora_desc* d, const void* dY, int64_t lddy,
                                const void* u_saved, void* dX, int64_t lddx, void* const* dA,
                                void* const* dB, int accumulate, void* stream) {
  if (!ctx) return MARLAAS_EINVAL;
  int rc = check_sizes(ctx, d);
  if (rc != MARLAAS_OK) return rc;
  const bool want_grads = dA != nullptr || dB != nullptr;
  if (want_grads && (!dA || !dB)) return fail(ctx, MARLAAS_EINVAL, "dA and dB must both be given or both be null");
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
  if (want_grads)
    for (int t = 0; t < d->n_adapters; ++t)
      if (!dA[t] || !dB[t] || !aligned16(dA[t]) || !aligned16(dB[t]))
        return fail(ctx, MARLAAS_EINVAL, "gradient buffers of adapter %d are null or misaligned", t);
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
  const AdapterEntry* table = nullptr;
  if ((rc = adapter_table(ctx, d, &table)) != MARLAAS_OK) return rc;
  const GradEntry* grads = nullptr;
  if (want_grads && d->n_adapters > 0) {
    std::vector<GradEntry> host((size_t)d->n_adapters);
    for (int t = 0; t < d->n_adapters; ++t) { host[t].dA = (float*)dA[t]; host[t].dB = (float*)dB[t]; }
    if ((rc = cached_table(ctx, host.data(), host.size() * sizeof(GradEntry), (const void**)&grads)) != MARLAAS_OK) return rc;
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
  if (d->in_dtype == MARLAAS_BF16) {
    const bf16_t* x = (const bf16_t*)d->x;
    const bf16_t* dy = (const bf16_t*)dY;
    if (need_u)
      PROFILED(ctx, MARLAAS_KERNEL_SHRINK, st, launch_shrink_bf16(x, d->ldx, d->d_in, perm, map->seg_off_dev, d->n_adapters, map->max_seg,
                                      table, 0, fform, u, rs, map->T_lora, st));
    // small batches: the dX GEMM computes v itself (and leaves it in `v` for the dA reduction)
    GemmFuse fuse;
    bool fused = false;
    if (lora && dX && part) {
      const int n_ext = sum_ranks_of(d);
      bool mult8 = true;
      for (int t = 0; t < d->n_adapters; ++t) if (d->ranks[t] & 7) mult8 = false;
      fused = gemm_can_fuse_shrink(bform, d->T, d->d_out, d->d_in, n_ext, mult8, p.part_bytes);
      if (fused) {
        if ((rc = fuse_tables(ctx, d, &fuse)) != MARLAAS_OK) return rc;
        fuse.u_out = v;
      }
    }
    if (lora && (dX || want_grads) && !fused)
      PROFILED(ctx, MARLAAS_KERNEL_SHRINK, st, launch_shrink_bf16(dy, lddy, d->d_out, perm, map->seg_off_dev, d->n_adapters, map->max_seg,
                                      table, 1, bform, v, rs, map->T_lora, st));
    if (dX && d->T > 0)
      PROFILED(ctx, MARLAAS_KERNEL_GEMM, st, launch_gemm_bf16(dy, lddy, (const bf16_t*)d->W, d->ldw, bform, d->T, d->d_out, d->d_in, perm,
                                    map->seg_off_dev, d->n_adapters, table, 0, lora ? v : nullptr, rs, dX, lddx,
                                    out_f32, part, part ? p.part_bytes : 0, map->chunks_dev, map->n_chunks,
                                    fused ? &fuse : nullptr, (have_ws && p.wt_bytes) ? (bf16_t*)((char*)ctx->ws + p.wt_off) : nullptr,
                                    p.wt_bytes, st));
    if (want_grads && d->n_adapters > 0) {
      PROFILED(ctx, MARLAAS_KERNEL_REDUCE, st, launch_reduce_bf16(dy, lddy, d->d_out, perm, map->seg_off_dev, d->n_adapters, map->max_seg,
                                      table, grads, 1, db_form, u, rs, accumulate, part, part ? p.part_bytes : 0, st));
      PROFILED(ctx, MARLAAS_KERNEL_REDUCE, st, launch_reduce_bf16(x, d->ldx, d->d_in, perm, map->seg_off_dev, d->n_adapters, map->max_seg,
                                      table, grads, 0, da_form, v, rs, accumulate, part, part ? p.part_bytes : 0, st));
    }
  } else {
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
