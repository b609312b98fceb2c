// C ABI of the embedding library (declared in include/persia_emb.h): context, validation,
// workspace, and the sequence of kernel launches of each hot call.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/persia_emb.h"
#include "device_utils.h"
#include "launch.h"

using namespace pemb;

namespace {

enum Stage {
  ST_GATHER_POOL = 0,
  ST_BUILD_KEYS,
  ST_SORT_HIST,
  ST_SORT_SCAN,
  ST_SORT_SCATTER,
  ST_UNIQUE,
  ST_TILE_ORDER,
  ST_REDUCE_UPDATE,
  ST_FIXUP,
  ST_COUNT
};
const char* const kStageNames[ST_COUNT] = {"gather_pool", "build_keys",    "sort_hist",  "sort_scan", "sort_scatter",
                                           "unique",      "tile_order",    "reduce_update", "fixup"};

struct EventRec {
  int stage;
  hipEvent_t e0, e1;
};

thread_local std::string g_create_error;

// Number of the dedup in progress, unique over all contexts of the process (the static workspace is shared): the
// key builder stores it in counters[kBadFlag] when a batch's offsets are inconsistent.  Never 0 (fresh memory).
std::atomic<uint32_t> g_call_seq{0};
constexpr int kBadFlag = 4;
uint32_t next_call() {
  uint32_t c = ++g_call_seq;
  if (c == 0) c = ++g_call_seq;
  return c;
}

// Scratch memory of one emb_backward_update (and of the dedup a cached context runs in its lookups): either the
// buffers a context allocated in emb_create for its max_ids, or the carved-up static array below.
struct Workspace {
  uint64_t cap = 0;  // ids the buffers are sized for
  uint32_t *keys[2] = {nullptr, nullptr}, *bags[2] = {nullptr, nullptr};
  uint32_t *hist = nullptr, *total = nullptr, *blk_heads = nullptr, *blk_multi = nullptr;
  uint32_t *unique_keys = nullptr, *seg_off = nullptr, *multi_list = nullptr, *long_list = nullptr;
  uint32_t *counters = nullptr, *ranges = nullptr;
  double* partials = nullptr;
  uint32_t *tile_key[2] = {nullptr, nullptr}, *tile_val[2] = {nullptr, nullptr};
};

// Scratch of emb_backward_update_static: one array per GPU, part of the loaded code object, so that the call needs
// no allocation of any kind.  Host code never uses this name as an address: g_static_scratch[device] holds what
// hipGetSymbolAddress returned for that device.
constexpr uint64_t kStaticMaxIds = 1ull << 18;
constexpr uint64_t kStaticScratchBytes = 16ull << 20;
constexpr int kMaxDevices = 64;
void* g_static_scratch[kMaxDevices] = {nullptr};

}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

struct emb_ctx {
  int device = 0;
  uint32_t S = 0, width = 0, max_batch = 0;
  uint64_t max_ids = 0;
  int mix = 0, opt = 0;
  float lr = 0, eps = 0;
  int key_bits = 1;
  int sort_max_bits = 8;  // 9-bit digits save a pass at 26 key bits but scatter in shorter runs: measured slower (scatter 0.260 vs 0.225 ms)
  uint32_t payload_width = 0;        // != 0: the sort's payload is the gradient's position in d_pooled / 4, not the bag
  std::vector<uint32_t> slot_col_host;
  uint32_t pstride = 0;
  std::vector<TableView> tables;
  std::vector<uint32_t> key_base_host;
  SlotArrays slots{};
  uint32_t* key_base_dev = nullptr;  // [T]
  uint32_t* zero_row = nullptr;      // kZeroRowBytes of zeros
  uint32_t *bag_beg = nullptr, *bag_end = nullptr;  // [max_batch * S + 1] each: bag bounds of the forward from the index form
  Workspace ws;                      // allocated in emb_create for max_ids
  Workspace last_ws;                 // the workspace that holds the index form of the last dedup
  // tables kept in host memory behind an LRU cache (emb_create_cached); lru[t].C == 0: table t is resident
  std::vector<LruView> lru;
  std::vector<uint64_t*> lru_stats;   // device [4] per cached table
  LruScratch lru_scratch{};
  uint32_t* unique_slots = nullptr;   // unique keys with rows replaced by cache slots
  uint32_t lru_step = 0;              // one step per admission (every lookup and every update is a use)
  bool any_cached = false;
  // calls on a context with cached tables share the cache's admission state: a hot call that arrives on another
  // stream than the one before it first waits for that call (cache_done is recorded at the end of every hot call)
  hipEvent_t cache_done = nullptr;
  hipStream_t cache_stream = nullptr;
  bool cache_busy = false;
  std::vector<void*> host_allocs;
  // last backward
  int sorted_buf = 0;
  uint64_t last_n = 0;
  uint32_t last_call = 0;            // number of the last dedup (see g_call_seq)
  bool have_dedup = false;
  // staging of emb_read_rows / emb_write_rows (allocated at the first use, kept)
  uint64_t* io_rows = nullptr;
  float *io_w = nullptr, *io_acc = nullptr;
  // bookkeeping
  std::vector<void*> allocs;
  uint64_t device_bytes = 0;
  bool profiling = false;
  bool no_events = false;            // set while a call that must not create anything runs
  std::vector<EventRec> recs;
  std::vector<hipEvent_t> free_events;
  float stage_ms[ST_COUNT] = {0};
  uint32_t stage_launches[ST_COUNT] = {0};
  std::string err;
};

namespace {

int fail(emb_ctx* ctx, int code, const std::string& msg) {
  if (ctx) ctx->err = msg;
  else g_create_error = msg;
  return code;
}

int fail_hip(emb_ctx* ctx, const char* what, hipError_t e) {
  return fail(ctx, e == hipErrorOutOfMemory ? EMB_ENOMEM : EMB_EDEVICE,
              std::string(what) + ": " + hipGetErrorString(e));
}

template <typename T>
hipError_t dev_alloc(emb_ctx* ctx, T** p, uint64_t count) {
  void* q = nullptr;
  uint64_t bytes = count * sizeof(T);
  if (bytes == 0) bytes = sizeof(T);
  hipError_t e = hipMalloc(&q, bytes);
  if (e != hipSuccess) return e;
  ctx->allocs.push_back(q);
  ctx->device_bytes += bytes;
  *p = reinterpret_cast<T*>(q);
  return hipSuccess;
}

template <typename T>
hipError_t dev_upload(emb_ctx* ctx, T** p, const std::vector<T>& v) {
  hipError_t e = dev_alloc(ctx, p, v.size());
  if (e != hipSuccess) return e;
  if (!v.empty()) e = hipMemcpy(*p, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice);
  return e;
}

// Pinned host memory the device can address; *dev receives the device-side pointer.
template <typename T>
hipError_t host_alloc(emb_ctx* ctx, T** dev, uint64_t count) {
  void *h = nullptr, *d = nullptr;
  hipError_t e = hipHostMalloc(&h, (count ? count : 1) * sizeof(T), hipHostMallocMapped);
  if (e != hipSuccess) return e;
  ctx->host_allocs.push_back(h);
  e = hipHostGetDevicePointer(&d, h, 0);
  if (e != hipSuccess) return e;
  *dev = reinterpret_cast<T*>(d);
  return hipSuccess;
}

void free_all(emb_ctx* ctx) {
  for (void* p : ctx->allocs) (void)hipFree(p);
  ctx->allocs.clear();
  for (void* p : ctx->host_allocs) (void)hipHostFree(p);
  ctx->host_allocs.clear();
  for (auto& r : ctx->recs) {
    (void)hipEventDestroy(r.e0);
    (void)hipEventDestroy(r.e1);
  }
  ctx->recs.clear();
  for (auto& e : ctx->free_events) (void)hipEventDestroy(e);
  ctx->free_events.clear();
  if (ctx->cache_done) (void)hipEventDestroy(ctx->cache_done);
  ctx->cache_done = nullptr;
}

// Brackets one kernel stage with events when profiling is on.
struct StageTimer {
  emb_ctx* ctx;
  hipStream_t stream;
  EventRec rec{};
  bool on = false;
  StageTimer(emb_ctx* c, int stage, hipStream_t s) : ctx(c), stream(s) {
    if (!ctx->profiling || ctx->no_events) return;
    hipEvent_t ev[2];
    for (int i = 0; i < 2; ++i) {
      if (!ctx->free_events.empty()) {
        ev[i] = ctx->free_events.back();
        ctx->free_events.pop_back();
      } else if (hipEventCreate(&ev[i]) != hipSuccess) {
        if (i == 1) ctx->free_events.push_back(ev[0]);
        return;
      }
    }
    rec.stage = stage;
    rec.e0 = ev[0];
    rec.e1 = ev[1];
    on = true;
    (void)hipEventRecord(rec.e0, stream);
  }
  ~StageTimer() {
    if (!on) return;
    (void)hipEventRecord(rec.e1, stream);
    ctx->recs.push_back(rec);
  }
};

int check_batch(emb_ctx* ctx, const emb_batch* b, uint64_t ids_limit = 0) {  // ids_limit 0: the context's max_ids
  if (!ctx) return fail(nullptr, EMB_EINVAL, "null context");
  if (!b) return fail(ctx, EMB_EINVAL, "null batch");
  if (b->reserved != 0) return fail(ctx, EMB_EINVAL, "batch.reserved must be 0");
  if (b->batch_size > ctx->max_batch) return fail(ctx, EMB_EINVAL, "batch_size exceeds max_batch given to emb_create");
  if (b->num_ids > (ids_limit ? ids_limit : ctx->max_ids))
    return fail(ctx, EMB_EINVAL, ids_limit ? "num_ids exceeds what the workspace is sized for"
                                           : "num_ids exceeds max_ids given to emb_create");
  if (b->batch_size && !b->offsets) return fail(ctx, EMB_EINVAL, "null offsets");
  if (b->num_ids && !b->ids) return fail(ctx, EMB_EINVAL, "null ids");
  if (b->batch_size == 0 && b->num_ids != 0) return fail(ctx, EMB_EINVAL, "ids without samples");
  return EMB_OK;
}

// Every buffer the backward kernels dereference; a null here would be a device-side fault.
bool workspace_complete(const emb_ctx* c, const Workspace& w) {
  const void* ptrs[] = {w.keys[0],  w.keys[1],     w.bags[0], w.bags[1],    w.hist,     w.total,
                        w.blk_heads, w.blk_multi,  w.unique_keys, w.seg_off, w.multi_list, w.long_list, w.counters,
                        w.tile_key[0], w.tile_key[1], w.tile_val[0], w.tile_val[1],
                        w.ranges,    w.partials,   c->key_base_dev, c->slots.salt, c->slots.rows, c->slots.mask,
                        c->slots.key_base, c->slots.col};
  for (const void* p : ptrs)
    if (!p) return false;
  for (const TableView& t : c->tables)
    if (!t.w || !t.acc || !t.slot_list) return false;
  return true;
}

int bit_length(uint64_t v) {
  int b = 0;
  while (v) {
    ++b;
    v >>= 1;
  }
  return b;
}

}  // namespace

extern "C" {

static int emb_create_impl(const emb_config* cfg, const uint64_t* cache_rows, emb_ctx** out) {
  if (!cfg || !out) return fail(nullptr, EMB_EINVAL, "null argument");
  if (cfg->num_tables == 0 || cfg->num_tables > 1023 || !cfg->tables)
    return fail(nullptr, EMB_EINVAL, "num_tables must be in 1..1023");
  if (cfg->num_slots == 0 || !cfg->slots) return fail(nullptr, EMB_EINVAL, "num_slots must be >= 1");
  if (cfg->reserved != 0) return fail(nullptr, EMB_EINVAL, "config.reserved must be 0");
  if (cfg->hash != EMB_HASH_IDENTITY_MOD && cfg->hash != EMB_HASH_MIX_MOD)
    return fail(nullptr, EMB_EINVAL, "unknown hash kind");
  if (cfg->opt != EMB_OPT_SGD && cfg->opt != EMB_OPT_ROWWISE_ADAGRAD)
    return fail(nullptr, EMB_EINVAL, "unknown optimizer kind");
  if (!std::isfinite(cfg->lr) || !std::isfinite(cfg->eps) || !std::isfinite(cfg->acc_init) || cfg->eps < 0 ||
      cfg->acc_init < 0)
    return fail(nullptr, EMB_EINVAL, "lr, eps, acc_init must be finite, eps and acc_init non-negative");
  if (!std::isfinite(cfg->init_lo) || !std::isfinite(cfg->init_hi) || cfg->init_lo > cfg->init_hi)
    return fail(nullptr, EMB_EINVAL, "init range must be finite with lo <= hi");
  if (cfg->max_batch == 0) return fail(nullptr, EMB_EINVAL, "max_batch must be >= 1");
  if ((uint64_t)cfg->max_batch * cfg->num_slots >= (1ull << 31))
    return fail(nullptr, EMB_EINVAL, "max_batch * num_slots must be < 2^31");
  if (cfg->max_ids >= (1ull << 31)) return fail(nullptr, EMB_EINVAL, "max_ids must be < 2^31");
  uint64_t total_rows = 0;
  uint32_t max_dim = 0;
  for (uint32_t t = 0; t < cfg->num_tables; ++t) {
    const emb_table_desc& d = cfg->tables[t];
    if (d.rows == 0) return fail(nullptr, EMB_EINVAL, "table with 0 rows");
    if (d.dim != 8 && d.dim != 16 && d.dim != 32 && d.dim != 64 && d.dim != 128)
      return fail(nullptr, EMB_EINVAL, "table dim must be one of 8, 16, 32, 64, 128");
    if (d.dtype != EMB_F32 && d.dtype != EMB_BF16) return fail(nullptr, EMB_EINVAL, "unknown table dtype");
    total_rows += d.rows;
    if (total_rows >= (1ull << 31)) return fail(nullptr, EMB_EINVAL, "sum of table rows must be < 2^31");
    if (d.dim > max_dim) max_dim = d.dim;
    if (cache_rows && cache_rows[t] != 0 && cache_rows[t] < d.rows) {
      // a batch's rows must all fit at once, whatever was cached before
      const uint64_t need = d.rows < cfg->max_ids ? d.rows : cfg->max_ids;
      if (cache_rows[t] < need) return fail(nullptr, EMB_EINVAL, "cache_rows must be at least min(rows, max_ids)");
    }
  }
  uint64_t pooled_width = 0;
  for (uint32_t s = 0; s < cfg->num_slots; ++s) {
    if (cfg->slots[s].table >= cfg->num_tables) return fail(nullptr, EMB_EINVAL, "slot refers to a missing table");
    if (cfg->slots[s].reserved != 0) return fail(nullptr, EMB_EINVAL, "slot.reserved must be 0");
    pooled_width += cfg->tables[cfg->slots[s].table].dim;
  }
  // with several tables the sort carries the position of a bag's gradient in d_pooled, in units of 4 floats, in 32 bits
  if (cfg->num_tables > 1 && (uint64_t)cfg->max_batch * pooled_width / 4 >= (1ull << 32))
    return fail(nullptr, EMB_EINVAL, "max_batch * pooled width must be < 2^34 floats when there are several tables");
  int ndev = 0;
  hipError_t e = hipGetDeviceCount(&ndev);
  if (e != hipSuccess) return fail_hip(nullptr, "hipGetDeviceCount", e);
  if (cfg->device < 0 || cfg->device >= ndev) return fail(nullptr, EMB_EINVAL, "no such HIP device");
  if ((e = hipSetDevice(cfg->device)) != hipSuccess) return fail_hip(nullptr, "hipSetDevice", e);

  if (cfg->device < kMaxDevices && !g_static_scratch[cfg->device]) {
    // once per device, with that device current: where this GPU's copy of the static scratch array lives
    void* p = nullptr;
    if ((e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) != hipSuccess) return fail_hip(nullptr, "hipGetSymbolAddress(scratch)", e);
    g_static_scratch[cfg->device] = p;
  }

  emb_ctx* ctx = new (std::nothrow) emb_ctx();
  if (!ctx) return fail(nullptr, EMB_ENOMEM, "out of host memory");
  struct Guard {  // frees a half-built context on every early exit, exceptions included
    emb_ctx* c;
    ~Guard() {
      if (c) {
        free_all(c);
        delete c;
      }
    }
  } guard{ctx};
  ctx->device = cfg->device;
  ctx->S = cfg->num_slots;
  ctx->max_batch = cfg->max_batch;
  ctx->max_ids = cfg->max_ids;
  ctx->mix = cfg->hash == EMB_HASH_MIX_MOD;
  ctx->opt = cfg->opt;
  ctx->lr = cfg->lr;
  ctx->eps = cfg->eps;
  ctx->key_bits = bit_length(total_rows - 1);
  if (ctx->key_bits < 1) ctx->key_bits = 1;
  ctx->pstride = max_dim;

#define CK(call, what)                                         \
  do {                                                         \
    hipError_t _e = (call);                                    \
    if (_e != hipSuccess) return fail_hip(nullptr, what, _e);  \
  } while (0)

  // tables + state
  std::vector<uint64_t> s_salt(ctx->S), s_rows(ctx->S), s_mask(ctx->S);
  std::vector<uint32_t> s_kb(ctx->S), s_col(ctx->S);
  ctx->tables.resize(cfg->num_tables);
  ctx->key_base_host.resize(cfg->num_tables);
  ctx->lru.assign(cfg->num_tables, LruView{});
  ctx->lru_stats.assign(cfg->num_tables, nullptr);
  uint32_t kb = 0;
  for (uint32_t t = 0; t < cfg->num_tables; ++t) {
    const emb_table_desc& d = cfg->tables[t];
    TableView& tv = ctx->tables[t];
    tv.rows = d.rows;
    tv.mask = (d.rows & (d.rows - 1)) == 0 ? d.rows - 1 : 0;
    if (d.rows == 1) tv.mask = 0;  // rows == 1: "mod 1" path (mask 0 means "not a power of two" to the kernels)
    tv.dim = d.dim;
    tv.dtype = d.dtype;
    tv.key_base = kb;
    ctx->key_base_host[t] = kb;
    kb += (uint32_t)d.rows;
    const bool cached = cache_rows && cache_rows[t] != 0 && cache_rows[t] < d.rows;
    const uint64_t held = cached ? cache_rows[t] : d.rows;  // rows in device memory
    const uint64_t elems = held * d.dim;
    if (d.dtype == EMB_BF16) {
      bf16_t* p = nullptr;
      CK(dev_alloc(ctx, &p, elems), "hipMalloc(table)");
      tv.w = p;
    } else {
      float* p = nullptr;
      CK(dev_alloc(ctx, &p, elems), "hipMalloc(table)");
      tv.w = p;
    }
    CK(dev_alloc(ctx, &tv.acc, held), "hipMalloc(optimizer state)");
    LruView& lv = ctx->lru[t];
    if (cached) {
      ctx->any_cached = true;
      if (d.dtype == EMB_BF16) {
        bf16_t* p = nullptr;
        CK(host_alloc(ctx, &p, d.rows * d.dim), "hipHostMalloc(table)");
        tv.back_w = p;
      } else {
        float* p = nullptr;
        CK(host_alloc(ctx, &p, d.rows * d.dim), "hipHostMalloc(table)");
        tv.back_w = p;
      }
      CK(host_alloc(ctx, &tv.back_acc, d.rows), "hipHostMalloc(optimizer state)");
      lv.C = (uint32_t)held;
      lv.dim = d.dim;
      lv.dtype = d.dtype;
      lv.key_base = tv.key_base;
      lv.rows = d.rows;
      lv.cache_w = tv.w;
      lv.cache_acc = tv.acc;
      lv.back_w = tv.back_w;
      lv.back_acc = tv.back_acc;
      CK(dev_alloc(ctx, &lv.where, d.rows), "hipMalloc(row -> slot map)");
      CK(dev_alloc(ctx, &lv.slot_row, held), "hipMalloc(slot rows)");
      CK(dev_alloc(ctx, &lv.stamp, held), "hipMalloc(slot stamps)");
      tv.where = lv.where;
      CK(launch_lru_init(lv, nullptr), "lru_init");
      CK(dev_alloc(ctx, &ctx->lru_stats[t], 4), "hipMalloc(cache statistics)");
      CK(hipMemset(ctx->lru_stats[t], 0, 4 * sizeof(uint64_t)), "hipMemset(cache statistics)");
    }
    std::vector<uint32_t> list;
    for (uint32_t s = 0; s < ctx->S; ++s)
      if (cfg->slots[s].table == t) list.push_back(s);
    tv.n_slots = (uint32_t)list.size();
    uint32_t* lp = nullptr;
    CK(dev_upload(ctx, &lp, list), "upload(slot list)");
    tv.slot_list = lp;
    const uint64_t table_key = mix64(cfg->init_seed + (uint64_t)(t + 1) * 0x9E3779B97F4A7C15ull);
    const float scale = (cfg->init_hi - cfg->init_lo) * 5.9604644775390625e-08f;
    const float mid = (cfg->init_hi + cfg->init_lo) * 0.5f;
    if (cached) {  // the whole table is initialised where it lives: in host memory
      TableView whole = tv;
      whole.w = tv.back_w;
      whole.acc = tv.back_acc;
      CK(launch_init_table(whole, table_key, scale, mid, cfg->acc_init, nullptr), "init_table");
    } else {
      CK(launch_init_table(tv, table_key, scale, mid, cfg->acc_init, nullptr), "init_table");
    }
  }
  uint32_t col = 0;
  for (uint32_t s = 0; s < ctx->S; ++s) {
    const TableView& tv = ctx->tables[cfg->slots[s].table];
    s_salt[s] = cfg->slots[s].salt;
    s_rows[s] = tv.rows;
    s_mask[s] = tv.mask;
    s_kb[s] = tv.key_base;
    s_col[s] = col;
    col += tv.dim;
  }
  ctx->width = col;
  ctx->slot_col_host = s_col;
  if (cfg->num_tables > 1) ctx->payload_width = col;  // several tables: the payload carries the gradient's position
  {
    uint64_t *p_salt = nullptr, *p_rows = nullptr, *p_mask = nullptr;
    uint32_t *p_kb = nullptr, *p_col = nullptr;
    CK(dev_upload(ctx, &p_salt, s_salt), "upload(slot salt)");
    CK(dev_upload(ctx, &p_rows, s_rows), "upload(slot rows)");
    CK(dev_upload(ctx, &p_mask, s_mask), "upload(slot mask)");
    CK(dev_upload(ctx, &p_kb, s_kb), "upload(slot key base)");
    CK(dev_upload(ctx, &p_col, s_col), "upload(slot col)");
    ctx->slots.salt = p_salt;
    ctx->slots.rows = p_rows;
    ctx->slots.mask = p_mask;
    ctx->slots.key_base = p_kb;
    ctx->slots.col = p_col;
    CK(dev_upload(ctx, &ctx->key_base_dev, ctx->key_base_host), "upload(table key base)");
    CK(dev_alloc(ctx, &ctx->zero_row, kZeroRowBytes / sizeof(uint32_t)), "hipMalloc(zero row)");
    CK(hipMemset(ctx->zero_row, 0, kZeroRowBytes), "hipMemset(zero row)");
    CK(dev_alloc(ctx, &ctx->bag_beg, (uint64_t)cfg->max_batch * cfg->num_slots + 1), "hipMalloc(bag bounds)");
    CK(dev_alloc(ctx, &ctx->bag_end, (uint64_t)cfg->max_batch * cfg->num_slots + 1), "hipMalloc(bag bounds)");
  }
  // workspace
  const uint64_t cap = ctx->max_ids ? ctx->max_ids : 1;
  const uint64_t ntiles = (cap + kTile - 1) / kTile;
  ctx->ws.cap = cap;
  for (int i = 0; i < 2; ++i) {
    CK(dev_alloc(ctx, &ctx->ws.keys[i], cap), "hipMalloc(sort keys)");
    CK(dev_alloc(ctx, &ctx->ws.bags[i], cap), "hipMalloc(sort payload)");
  }
  for (int i = 0; i < 2; ++i) {  // entries a malformed batch leaves unwritten are then still keys and bags of the context
    CK(hipMemset(ctx->ws.keys[i], 0, cap * sizeof(uint32_t)), "hipMemset(sort keys)");
    CK(hipMemset(ctx->ws.bags[i], 0, cap * sizeof(uint32_t)), "hipMemset(sort payload)");
  }
  CK(dev_alloc(ctx, &ctx->ws.hist, ((uint64_t)1 << kSortMaxBits) * kSortMaxBlocks), "hipMalloc(histograms)");
  CK(dev_alloc(ctx, &ctx->ws.total, (uint64_t)1 << kSortMaxBits), "hipMalloc(digit totals)");
  CK(dev_alloc(ctx, &ctx->ws.blk_heads, (cap + kUniqueTile - 1) / kUniqueTile + 1), "hipMalloc(block heads)");
  CK(dev_alloc(ctx, &ctx->ws.blk_multi, (cap + kUniqueTile - 1) / kUniqueTile + 1), "hipMalloc(block multi-tile counts)");
  CK(dev_alloc(ctx, &ctx->ws.unique_keys, cap), "hipMalloc(unique keys)");
  CK(dev_alloc(ctx, &ctx->ws.seg_off, cap + 1), "hipMalloc(segment offsets)");
  CK(dev_alloc(ctx, &ctx->ws.multi_list, ntiles), "hipMalloc(multi-tile list)");
  CK(dev_alloc(ctx, &ctx->ws.long_list, ntiles), "hipMalloc(long segment list)");
  CK(dev_alloc(ctx, &ctx->ws.counters, 8), "hipMalloc(counters)");
  CK(hipMemset(ctx->ws.counters, 0, 8 * sizeof(uint32_t)), "hipMemset(counters)");
  CK(dev_alloc(ctx, &ctx->ws.ranges, cfg->num_tables + 1), "hipMalloc(table ranges)");
  CK(dev_alloc(ctx, &ctx->ws.partials, 2 * ntiles * ctx->pstride), "hipMalloc(partials)");
  for (int i = 0; i < 2; ++i) {
    CK(dev_alloc(ctx, &ctx->ws.tile_key[i], ntiles), "hipMalloc(tile order keys)");
    CK(dev_alloc(ctx, &ctx->ws.tile_val[i], ntiles), "hipMalloc(tile order)");
  }

  if (ctx->any_cached) {
    CK(hipEventCreateWithFlags(&ctx->cache_done, hipEventDisableTiming), "hipEventCreate(cache order)");
    uint64_t max_c = 0;
    for (const LruView& v : ctx->lru) max_c = v.C > max_c ? v.C : max_c;
    const uint64_t big = max_c > cap ? max_c : cap;
    CK(dev_alloc(ctx, &ctx->lru_scratch.blk_counts, big / 2048 + 2), "hipMalloc(cache scan counts)");
    CK(dev_alloc(ctx, &ctx->lru_scratch.miss_list, cap), "hipMalloc(cache miss list)");
    CK(dev_alloc(ctx, &ctx->lru_scratch.victims, cap), "hipMalloc(cache victim list)");
    CK(dev_alloc(ctx, &ctx->lru_scratch.age_hist, kAgeMax + 1), "hipMalloc(cache age histogram)");
    CK(dev_alloc(ctx, &ctx->lru_scratch.plan, 8), "hipMalloc(cache plan)");
    CK(dev_alloc(ctx, &ctx->lru_scratch.evicted, 1), "hipMalloc(cache eviction counter)");
    CK(hipMemset(ctx->lru_scratch.evicted, 0, sizeof(uint32_t)), "hipMemset(cache eviction counter)");
    CK(dev_alloc(ctx, &ctx->unique_slots, cap), "hipMalloc(unique slots)");
  }
  CK(hipDeviceSynchronize(), "table initialisation");
#undef CK
  guard.c = nullptr;
  *out = ctx;
  return EMB_OK;
}

int emb_destroy(emb_ctx* ctx) {
  if (!ctx) return EMB_OK;
  (void)hipSetDevice(ctx->device);
  (void)hipDeviceSynchronize();
  free_all(ctx);
  delete ctx;
  return EMB_OK;
}

#define CKH(call, what)                                      \
  do {                                                       \
    hipError_t _e = (call);                                  \
    if (_e != hipSuccess) return fail_hip(ctx, what, _e);    \
  } while (0)

// The index form of the batch (section 4.2.3): keys built, sorted (stable LSD radix) and run-length encoded.
// Leaves the sorted pairs in keys/bags[ctx->sorted_buf] and unique_keys / seg_off / counters filled.
static int run_dedup(emb_ctx* ctx, const Workspace& ws, const emb_batch* batch, hipStream_t stream) {
  const uint32_t n = (uint32_t)batch->num_ids;
  ctx->last_n = n;
  ctx->have_dedup = true;
  ctx->last_ws = ws;
  ctx->last_call = next_call();
  ctx->sorted_buf = 0;
  if (n == 0) {  // leave an empty index form behind
    CKH(launch_unique(ws.keys[0], 0, ws.blk_heads, ws.blk_multi, ws.unique_keys, ws.seg_off,
                      ws.multi_list, ws.counters, stream),
        "unique");
    return EMB_OK;
  }
  {
    StageTimer tm(ctx, ST_BUILD_KEYS, stream);
    CKH(launch_build_keys(ctx->slots, batch->ids, batch->offsets, n, batch->batch_size, ctx->S, ctx->mix, 0,
                          ws.keys[0], ws.bags[0], ws.counters + kBadFlag, ctx->last_call, ctx->payload_width, stream),
        "build_keys");
  }
  const SortPlan plan = make_sort_plan(n, ctx->key_bits, ctx->sort_max_bits);
  int src = 0;
  for (int pass = 0; pass < plan.passes; ++pass) {
    const int shift = pass * plan.bits;
    {
      StageTimer tm(ctx, ST_SORT_HIST, stream);
      CKH(launch_radix_hist(plan, shift, ws.keys[src], ws.hist, stream), "radix_hist");
    }
    {
      StageTimer tm(ctx, ST_SORT_SCAN, stream);
      CKH(launch_radix_scan(plan, ws.hist, ws.total, stream), "radix_scan");
    }
    {
      StageTimer tm(ctx, ST_SORT_SCATTER, stream);
      CKH(launch_radix_scatter(plan, shift, ws.keys[src], ws.bags[src], ws.keys[src ^ 1], ws.bags[src ^ 1],
                               ws.hist, ws.total, stream),
          "radix_scatter");
    }
    src ^= 1;
  }
  ctx->sorted_buf = src;
  {
    StageTimer tm(ctx, ST_UNIQUE, stream);
    CKH(launch_unique(ws.keys[src], n, ws.blk_heads, ws.blk_multi, ws.unique_keys, ws.seg_off,
                      ws.multi_list, ws.counters, stream),
        "unique");
  }
  return EMB_OK;
}

// Makes every row of the batch just deduplicated resident in its table's cache (one LRU step per call).
static int admit_batch(emb_ctx* ctx, hipStream_t stream) {
  if (!ctx->any_cached || ctx->last_n == 0) return EMB_OK;
  if (++ctx->lru_step == 0) ctx->lru_step = 1;  // 0 marks a slot that was never used
  for (size_t t = 0; t < ctx->lru.size(); ++t) {
    if (ctx->lru[t].C == 0) continue;
    LruScratch sc = ctx->lru_scratch;
    sc.stats = ctx->lru_stats[t];
    CKH(launch_lru_admit(ctx->lru[t], sc, ctx->ws.unique_keys, ctx->ws.counters, (uint32_t)ctx->last_n, ctx->lru_step, stream),
        "lru_admit");
  }
  return EMB_OK;
}

// Order of the hot calls on a context whose tables sit behind the cache (see emb_ctx::cache_done).
static int cache_enter(emb_ctx* ctx, hipStream_t stream) {
  if (ctx->any_cached && ctx->cache_busy && stream != ctx->cache_stream)
    CKH(hipStreamWaitEvent(stream, ctx->cache_done, 0), "hipStreamWaitEvent(cache order)");
  return EMB_OK;
}
static int cache_leave(emb_ctx* ctx, hipStream_t stream) {
  if (!ctx->any_cached) return EMB_OK;
  CKH(hipEventRecord(ctx->cache_done, stream), "hipEventRecord(cache order)");
  ctx->cache_stream = stream;
  ctx->cache_busy = true;
  return EMB_OK;
}

static int emb_lookup_pool_impl(emb_ctx* ctx, const emb_batch* batch, float* pooled, void* hip_stream) {
  int rc = check_batch(ctx, batch);
  if (rc) return rc;
  if (batch->batch_size == 0) return EMB_OK;
  if (!pooled) return fail(ctx, EMB_EINVAL, "null pooled output");
  hipStream_t stream = (hipStream_t)hip_stream;
  CKH(hipSetDevice(ctx->device), "hipSetDevice");
  if ((rc = cache_enter(ctx, stream)) != EMB_OK) return rc;
  if (ctx->any_cached) {  // the rows must be in the cache before they are gathered
    if (!workspace_complete(ctx, ctx->ws)) return fail(ctx, EMB_ESTATE, "workspace is incomplete (a buffer is null)");
    if ((rc = run_dedup(ctx, ctx->ws, batch, stream)) != EMB_OK) return rc;
    if ((rc = admit_batch(ctx, stream)) != EMB_OK) return rc;
  }
  for (const TableView& tv : ctx->tables) {
    StageTimer tm(ctx, ST_GATHER_POOL, stream);
    CKH(launch_gather_pool(tv, ctx->slots, batch->ids, batch->offsets, (uint32_t)batch->num_ids, batch->batch_size, ctx->S, ctx->width,
                           ctx->mix, ctx->zero_row, pooled, stream),
        "gather_pool");
  }
  return cache_leave(ctx, stream);
}

static int emb_lookup_pool_indexed_impl(emb_ctx* ctx, uint32_t batch_size, uint64_t num_unique, uint64_t num_ids,
                                        const uint64_t* keys, const uint32_t* seg_off, const uint32_t* seg_bags,
                                        float* pooled, void* hip_stream) {
  if (!ctx) return fail(nullptr, EMB_EINVAL, "null context");
  if (batch_size > ctx->max_batch) return fail(ctx, EMB_EINVAL, "batch_size exceeds max_batch");
  if (num_ids > ctx->max_ids || num_unique > num_ids) return fail(ctx, EMB_EINVAL, "num_unique <= num_ids <= max_ids violated");
  if (batch_size == 0) return EMB_OK;
  if (!pooled || (num_ids && (!keys || !seg_off || !seg_bags))) return fail(ctx, EMB_EINVAL, "null buffer");
  if (ctx->any_cached) return fail(ctx, EMB_ESTATE, "not available for tables kept behind a cache");
  const Workspace& ws = ctx->ws;
  if (!workspace_complete(ctx, ws) || !ctx->bag_beg || !ctx->bag_end)
    return fail(ctx, EMB_ESTATE, "workspace is incomplete (a buffer is null)");
  hipStream_t stream = (hipStream_t)hip_stream;
  CKH(hipSetDevice(ctx->device), "hipSetDevice");
  ctx->have_dedup = false;  // the sort buffers that held the last index form are reused below
  const uint32_t n = (uint32_t)num_ids, n_bags = batch_size * ctx->S;
  if (n == 0 || num_unique == 0) {
    CKH(launch_zero_f32(pooled, (uint64_t)batch_size * ctx->width, stream), "zero(pooled)");
    return EMB_OK;
  }
  int src = 0;
  {
    StageTimer tm(ctx, ST_BUILD_KEYS, stream);
    CKH(launch_expand_index(seg_off, seg_bags, (uint32_t)num_unique, n, n_bags, ws.keys[0], ws.bags[0], stream), "expand_index");
  }
  const SortPlan plan = make_sort_plan(n, bit_length(n_bags), ctx->sort_max_bits);  // bag values 0 .. n_bags
  for (int pass = 0; pass < plan.passes; ++pass) {
    const int shift = pass * plan.bits;
    {
      StageTimer tm(ctx, ST_SORT_HIST, stream);
      CKH(launch_radix_hist(plan, shift, ws.keys[src], ws.hist, stream), "radix_hist");
    }
    {
      StageTimer tm(ctx, ST_SORT_SCAN, stream);
      CKH(launch_radix_scan(plan, ws.hist, ws.total, stream), "radix_scan");
    }
    {
      StageTimer tm(ctx, ST_SORT_SCATTER, stream);
      CKH(launch_radix_scatter(plan, shift, ws.keys[src], ws.bags[src], ws.keys[src ^ 1], ws.bags[src ^ 1], ws.hist,
                               ws.total, stream),
          "radix_scatter");
    }
    src ^= 1;
  }
  {
    StageTimer tm(ctx, ST_UNIQUE, stream);
    CKH(launch_zero_u32(ctx->bag_beg, (uint64_t)n_bags + 1, stream), "zero(bag bounds)");
    CKH(launch_zero_u32(ctx->bag_end, (uint64_t)n_bags + 1, stream), "zero(bag bounds)");
    CKH(launch_bag_bounds(ws.keys[src], n, ctx->bag_beg, ctx->bag_end, stream), "bag_bounds");
  }
  for (size_t t = 0; t < ctx->tables.size(); ++t) {
    StageTimer tm(ctx, ST_GATHER_POOL, stream);
    IndexedBags ix{ctx->bag_beg, ctx->bag_end, ws.bags[src], keys, (uint32_t)num_unique, (uint32_t)t};
    CKH(launch_gather_pool(ctx->tables[t], ctx->slots, nullptr, nullptr, n, batch_size, ctx->S, ctx->width, ctx->mix,
                           ctx->zero_row, pooled, stream, &ix),
        "gather_pool(indexed)");
  }
  return EMB_OK;
}

static int emb_hash_rows_impl(emb_ctx* ctx, const emb_batch* batch, uint32_t* rows_out, void* hip_stream) {
  int rc = check_batch(ctx, batch);
  if (rc) return rc;
  if (batch->num_ids == 0) return EMB_OK;
  if (!rows_out) return fail(ctx, EMB_EINVAL, "null rows output");
  hipStream_t stream = (hipStream_t)hip_stream;
  CKH(hipSetDevice(ctx->device), "hipSetDevice");
  CKH(launch_build_keys(ctx->slots, batch->ids, batch->offsets, (uint32_t)batch->num_ids, batch->batch_size, ctx->S,
                        ctx->mix, 1, rows_out, nullptr, nullptr, 0, 0, stream),
      "hash_rows");
  return EMB_OK;
}

static int backward_update_with(emb_ctx* ctx, const Workspace& ws, const emb_batch* batch, const float* d_pooled,
                                void* hip_stream) {
  int rc = check_batch(ctx, batch, ws.cap);
  if (rc) return rc;
  if (!workspace_complete(ctx, ws)) return fail(ctx, EMB_ESTATE, "workspace is incomplete (a buffer is null)");
  if (batch->batch_size && !d_pooled) return fail(ctx, EMB_EINVAL, "null d_pooled");
  hipStream_t stream = (hipStream_t)hip_stream;
  CKH(hipSetDevice(ctx->device), "hipSetDevice");
  const uint32_t n = (uint32_t)batch->num_ids;
  if ((rc = cache_enter(ctx, stream)) != EMB_OK) return rc;
  if ((rc = run_dedup(ctx, ws, batch, stream)) != EMB_OK) return rc;
  if (n == 0) return cache_leave(ctx, stream);  // nothing to update
  const int src = ctx->sorted_buf;
  const bool multi_table = ctx->tables.size() > 1;
  if (multi_table)  // each table's stretch of the sorted list (found before any key is rewritten below)
    CKH(launch_table_ranges(ws.keys[src], n, ctx->key_base_dev, (uint32_t)ctx->tables.size(), ws.ranges, stream),
        "table_ranges");
  const uint32_t* sorted_keys = ws.keys[src];
  const uint32_t* unique_keys = ws.unique_keys;
  if (ctx->any_cached) {
    // rows that were evicted since the lookup come back; then the kernels below address cache slots: they
    // only compare neighbouring keys for equality, and key_base + slot stays inside the table's key range
    if ((rc = admit_batch(ctx, stream)) != EMB_OK) return rc;
    uint32_t* tk = ws.keys[src ^ 1];
    CKH(hipMemcpyAsync(tk, ws.keys[src], (size_t)n * sizeof(uint32_t), hipMemcpyDeviceToDevice, stream), "copy(keys)");
    CKH(hipMemcpyAsync(ctx->unique_slots, ws.unique_keys, (size_t)n * sizeof(uint32_t), hipMemcpyDeviceToDevice, stream),
        "copy(unique keys)");
    for (size_t t = 0; t < ctx->lru.size(); ++t) {
      if (ctx->lru[t].C == 0) continue;
      CKH(launch_lru_translate(ctx->lru[t], tk, multi_table ? ws.ranges + t : nullptr, nullptr, n, stream), "lru_translate");
      CKH(launch_lru_translate(ctx->lru[t], ctx->unique_slots, nullptr, ws.counters, n, stream), "lru_translate");
    }
    sorted_keys = tk;
    unique_keys = ctx->unique_slots;
  }
  BackwardArgs a{};
  a.keys = sorted_keys;
  a.bags = ws.bags[src];
  a.n = n;
  a.d_pooled = d_pooled;
  a.payload_is_position = ctx->payload_width != 0;
  a.partials = ws.partials;
  a.pstride = ctx->pstride;
  a.range = nullptr;
  a.tile_perm = nullptr;
  a.opt = ctx->opt;
  a.lr = ctx->lr;
  a.eps = ctx->eps;
  a.unique_keys = unique_keys;
  a.seg_off = ws.seg_off;
  a.counters = ws.counters;
  a.multi_list = ws.multi_list;
  a.long_list = ws.long_list;
  a.bad_flag = ws.counters + kBadFlag;
  a.call = ctx->last_call;
  {
    StageTimer tm(ctx, ST_TILE_ORDER, stream);
    // shift that leaves 8 bits of the payload (the tile keys use 7: 128 buckets of consecutive bags, sample-major;
    // gradient positions are sample-major too)
    const uint64_t payload_range = ctx->payload_width ? (uint64_t)batch->batch_size * ctx->payload_width / 4
                                                      : (uint64_t)batch->batch_size * ctx->S;
    int shift = bit_length(payload_range - 1) - 8;
    if (shift < 0) shift = 0;
    CKH(launch_tile_order(a.keys, a.bags, n, shift, ctx->key_base_dev, (uint32_t)ctx->tables.size(), ws.tile_key,
                          ws.tile_val, ws.hist, ws.total, &a.tile_perm, stream),
        "tile_order");
  }
  for (size_t t = 0; t < ctx->tables.size(); ++t) {
    StageTimer tm(ctx, ST_REDUCE_UPDATE, stream);
    a.range = multi_table ? ws.ranges + t : nullptr;
    CKH(launch_tile_reduce_update(ctx->tables[t], a, stream), "tile_reduce_update");
  }
  {
    StageTimer tm(ctx, ST_FIXUP, stream);
    CKH(launch_classify_multi(a, ws.counters, ws.long_list, stream), "classify_multi");
  }
  for (size_t t = 0; t < ctx->tables.size(); ++t) {
    StageTimer tm(ctx, ST_FIXUP, stream);
    CKH(launch_fixup(ctx->tables[t], a, stream), "fixup");
  }
  return cache_leave(ctx, stream);
}

static int emb_backward_update_impl(emb_ctx* ctx, const emb_batch* batch, const float* d_pooled, void* hip_stream) {
  if (!ctx) return fail(nullptr, EMB_EINVAL, "null context");
  return backward_update_with(ctx, ctx->ws, batch, d_pooled, hip_stream);
}

// Cuts the static array of the context's device into the buffers of a Workspace for kStaticMaxIds ids.
static int carve_static_workspace(emb_ctx* ctx, Workspace* out) {
  if (ctx->device < 0 || ctx->device >= kMaxDevices || !g_static_scratch[ctx->device])
    return fail(ctx, EMB_ESTATE, "the static scratch of this device was not located at emb_create");
  unsigned char* base = static_cast<unsigned char*>(g_static_scratch[ctx->device]);
  uint64_t off = 0;
  bool fits = true;
  auto take = [&](uint64_t count, uint64_t elem) -> void* {
    void* p = base + off;
    off += (count * elem + 255) / 256 * 256;  // every buffer starts on a 256-byte boundary
    if (off > kStaticScratchBytes) fits = false;
    return p;
  };
  const uint64_t cap = kStaticMaxIds;
  const uint64_t ntiles = (cap + kTile - 1) / kTile;
  const uint64_t sort_blocks = (cap + kSortTile - 1) / kSortTile;  // blocks of a sort pass over at most cap pairs
  Workspace w;
  w.cap = cap;
  for (int i = 0; i < 2; ++i) {
    w.keys[i] = static_cast<uint32_t*>(take(cap, 4));
    w.bags[i] = static_cast<uint32_t*>(take(cap, 4));
  }
  w.hist = static_cast<uint32_t*>(take(((uint64_t)1 << kSortMaxBits) * sort_blocks, 4));
  w.total = static_cast<uint32_t*>(take((uint64_t)1 << kSortMaxBits, 4));
  w.blk_heads = static_cast<uint32_t*>(take((cap + kUniqueTile - 1) / kUniqueTile + 1, 4));
  w.blk_multi = static_cast<uint32_t*>(take((cap + kUniqueTile - 1) / kUniqueTile + 1, 4));
  w.unique_keys = static_cast<uint32_t*>(take(cap, 4));
  w.seg_off = static_cast<uint32_t*>(take(cap + 1, 4));
  w.multi_list = static_cast<uint32_t*>(take(ntiles, 4));
  w.long_list = static_cast<uint32_t*>(take(ntiles, 4));
  w.counters = static_cast<uint32_t*>(take(8, 4));
  w.ranges = static_cast<uint32_t*>(take(ctx->tables.size() + 1, 4));
  w.partials = static_cast<double*>(take(2 * ntiles * ctx->pstride, 8));
  for (int i = 0; i < 2; ++i) {
    w.tile_key[i] = static_cast<uint32_t*>(take(ntiles, 4));
    w.tile_val[i] = static_cast<uint32_t*>(take(ntiles, 4));
  }
  if (!fits) return fail(ctx, EMB_ESTATE, "the static scratch is too small for this context's tables");
  *out = w;
  return EMB_OK;
}

static int emb_backward_update_static_impl(emb_ctx* ctx, const emb_batch* batch, const float* d_pooled, void* hip_stream) {
  if (!ctx) return fail(nullptr, EMB_EINVAL, "null context");
  if (ctx->any_cached) return fail(ctx, EMB_ESTATE, "not available for tables kept behind a cache");
  if (batch && batch->num_ids > kStaticMaxIds)
    return fail(ctx, EMB_EINVAL, "num_ids exceeds the static scratch (262144 ids per call)");
  Workspace w;
  int rc = carve_static_workspace(ctx, &w);
  if (rc) return rc;
  ctx->no_events = true;  // per-stage timing would create events
  rc = backward_update_with(ctx, w, batch, d_pooled, hip_stream);
  ctx->no_events = false;
  return rc;
}

static int emb_dedup_sizes_impl(emb_ctx* ctx, uint64_t* num_unique, uint64_t* num_ids) {
  if (!ctx) return fail(nullptr, EMB_EINVAL, "null context");
  if (!ctx->have_dedup) return fail(ctx, EMB_ESTATE, "no emb_backward_update has run on this context");
  CKH(hipSetDevice(ctx->device), "hipSetDevice");
  CKH(hipDeviceSynchronize(), "hipDeviceSynchronize");
  uint32_t c[kBadFlag + 1] = {0};
  CKH(hipMemcpy(c, ctx->last_ws.counters, sizeof(c), hipMemcpyDeviceToHost), "hipMemcpy(counters)");
  if (c[kBadFlag] == ctx->last_call)
    return fail(ctx, EMB_EINVAL, "the last batch's offsets do not tile [0, num_ids) (non-decreasing, offsets[0] = 0, "
                                 "offsets[B * S] = num_ids): its update was skipped");
  if (num_unique) *num_unique = c[0];
  if (num_ids) *num_ids = ctx->last_n;
  return EMB_OK;
}

static int emb_read_dedup_impl(emb_ctx* ctx, uint64_t* keys, uint32_t* seg_off, uint32_t* seg_bags) {
  uint64_t U = 0, N = 0;
  int rc = emb_dedup_sizes_impl(ctx, &U, &N);
  if (rc) return rc;
  if (keys && U) {
    std::vector<uint32_t> tmp(U);
    CKH(hipMemcpy(tmp.data(), ctx->last_ws.unique_keys, U * sizeof(uint32_t), hipMemcpyDeviceToHost), "hipMemcpy(keys)");
    size_t t = 0;
    const size_t T = ctx->key_base_host.size();
    for (uint64_t u = 0; u < U; ++u) {  // keys ascend, so the table index only moves forward
      while (t + 1 < T && tmp[u] >= ctx->key_base_host[t + 1]) ++t;
      keys[u] = ((uint64_t)t << 32) | (uint64_t)(tmp[u] - ctx->key_base_host[t]);
    }
  }
  if (seg_off) CKH(hipMemcpy(seg_off, ctx->last_ws.seg_off, (U + 1) * sizeof(uint32_t), hipMemcpyDeviceToHost), "hipMemcpy(seg_off)");
  if (seg_bags && N) {
    CKH(hipMemcpy(seg_bags, ctx->last_ws.bags[ctx->sorted_buf], N * sizeof(uint32_t), hipMemcpyDeviceToHost),
        "hipMemcpy(seg_bags)");
    if (ctx->payload_width) {  // gradient positions back to bag indices: sample = p / (W / 4), slot = the one whose columns hold the rest
      const uint32_t w4 = ctx->payload_width / 4;
      const std::vector<uint32_t>& col = ctx->slot_col_host;
      for (uint64_t i = 0; i < N; ++i) {
        const uint32_t b = seg_bags[i] / w4, c = (seg_bags[i] % w4) * 4;
        const uint32_t slot = (uint32_t)(std::upper_bound(col.begin(), col.end(), c) - col.begin()) - 1;
        seg_bags[i] = b * ctx->S + slot;
      }
    }
  }
  return EMB_OK;
}

static int rows_io(emb_ctx* ctx, uint32_t table, const uint64_t* rows, uint64_t n, float* w_out, float* acc_out,
                   const float* w_in, const float* acc_in, bool write) {
  if (!ctx) return fail(nullptr, EMB_EINVAL, "null context");
  if (table >= ctx->tables.size()) return fail(ctx, EMB_EINVAL, "no such table");
  if (n == 0) return EMB_OK;
  if (!rows) return fail(ctx, EMB_EINVAL, "null rows");
  const TableView& tv = ctx->tables[table];
  for (uint64_t i = 0; i < n; ++i)
    if (rows[i] >= tv.rows) return fail(ctx, EMB_EINVAL, "row index out of range");
  CKH(hipSetDevice(ctx->device), "hipSetDevice");
  const uint64_t chunk = 1u << 18;   // rows staged at a time (the staging buffers hold this many rows of the widest table)
  hipError_t e = hipSuccess;
  if (!ctx->io_rows) {
    if ((e = dev_alloc(ctx, &ctx->io_rows, chunk)) == hipSuccess &&
        (e = dev_alloc(ctx, &ctx->io_w, chunk * ctx->pstride)) == hipSuccess)
      e = dev_alloc(ctx, &ctx->io_acc, chunk);
    if (e != hipSuccess) {
      ctx->io_rows = nullptr;  // whatever was allocated stays on the context's list and is freed with it
      return fail_hip(ctx, "hipMalloc(row staging)", e);
    }
  }
  uint64_t* d_rows = ctx->io_rows;
  float *d_w = ctx->io_w, *d_a = ctx->io_acc;
  for (uint64_t i0 = 0; e == hipSuccess && i0 < n; i0 += chunk) {
    const uint64_t c = n - i0 < chunk ? n - i0 : chunk;
    e = hipMemcpy(d_rows, rows + i0, c * sizeof(uint64_t), hipMemcpyHostToDevice);
    if (e != hipSuccess) break;
    if (write) {
      if (w_in) e = hipMemcpy(d_w, w_in + i0 * tv.dim, c * tv.dim * sizeof(float), hipMemcpyHostToDevice);
      if (e == hipSuccess && acc_in) e = hipMemcpy(d_a, acc_in + i0, c * sizeof(float), hipMemcpyHostToDevice);
      if (e == hipSuccess) e = launch_write_rows(tv, d_rows, c, w_in ? d_w : nullptr, acc_in ? d_a : nullptr, nullptr);
      if (e == hipSuccess) e = hipDeviceSynchronize();
    } else {
      e = launch_read_rows(tv, d_rows, c, w_out ? d_w : nullptr, acc_out ? d_a : nullptr, nullptr);
      if (e == hipSuccess) e = hipDeviceSynchronize();
      if (e == hipSuccess && w_out) e = hipMemcpy(w_out + i0 * tv.dim, d_w, c * tv.dim * sizeof(float), hipMemcpyDeviceToHost);
      if (e == hipSuccess && acc_out) e = hipMemcpy(acc_out + i0, d_a, c * sizeof(float), hipMemcpyDeviceToHost);
    }
  }
  if (e != hipSuccess) return fail_hip(ctx, write ? "emb_write_rows" : "emb_read_rows", e);
  return EMB_OK;
}

static int emb_read_rows_impl(emb_ctx* ctx, uint32_t table, const uint64_t* rows, uint64_t n, float* w, float* acc) {
  if (ctx) {
    (void)hipSetDevice(ctx->device);
    (void)hipDeviceSynchronize();
  }
  return rows_io(ctx, table, rows, n, w, acc, nullptr, nullptr, false);
}

static int emb_write_rows_impl(emb_ctx* ctx, uint32_t table, const uint64_t* rows, uint64_t n, const float* w, const float* acc) {
  if (ctx) {
    (void)hipSetDevice(ctx->device);
    (void)hipDeviceSynchronize();
  }
  return rows_io(ctx, table, rows, n, nullptr, nullptr, w, acc, true);
}

int emb_table_ptr(emb_ctx* ctx, uint32_t table, void** w_dev, float** acc_dev) {
  if (!ctx) return fail(nullptr, EMB_EINVAL, "null context");
  if (table >= ctx->tables.size()) return fail(ctx, EMB_EINVAL, "no such table");
  if (ctx->lru[table].C) return fail(ctx, EMB_ESTATE, "the table is kept in host memory behind a cache: no flat device array");
  if (w_dev) *w_dev = ctx->tables[table].w;
  if (acc_dev) *acc_dev = ctx->tables[table].acc;
  return EMB_OK;
}

static int emb_cache_stats_impl(emb_ctx* ctx, uint32_t table, uint64_t* stats) {
  if (!ctx) return fail(nullptr, EMB_EINVAL, "null context");
  if (table >= ctx->tables.size() || !stats) return fail(ctx, EMB_EINVAL, "no such table, or null output");
  if (ctx->lru[table].C == 0) return fail(ctx, EMB_ESTATE, "the table is resident, it has no cache");
  CKH(hipSetDevice(ctx->device), "hipSetDevice");
  CKH(hipDeviceSynchronize(), "hipDeviceSynchronize");
  CKH(hipMemcpy(stats, ctx->lru_stats[table], 4 * sizeof(uint64_t), hipMemcpyDeviceToHost), "hipMemcpy(cache statistics)");
  return EMB_OK;
}

static int emb_cache_where_impl(emb_ctx* ctx, uint32_t table, int32_t* where_host) {
  if (!ctx) return fail(nullptr, EMB_EINVAL, "null context");
  if (table >= ctx->tables.size() || !where_host) return fail(ctx, EMB_EINVAL, "no such table, or null output");
  if (ctx->lru[table].C == 0) return fail(ctx, EMB_ESTATE, "the table is resident, it has no cache");
  CKH(hipSetDevice(ctx->device), "hipSetDevice");
  CKH(hipDeviceSynchronize(), "hipDeviceSynchronize");
  CKH(hipMemcpy(where_host, ctx->lru[table].where, ctx->lru[table].rows * sizeof(int32_t), hipMemcpyDeviceToHost),
      "hipMemcpy(row -> slot map)");
  return EMB_OK;
}

static int emb_cache_flush_impl(emb_ctx* ctx, void* hip_stream) {
  if (!ctx) return fail(nullptr, EMB_EINVAL, "null context");
  CKH(hipSetDevice(ctx->device), "hipSetDevice");
  for (const LruView& v : ctx->lru)
    if (v.C) CKH(launch_lru_flush(v, (hipStream_t)hip_stream), "lru_flush");
  return EMB_OK;
}

int emb_set_profiling(emb_ctx* ctx, int enabled) {
  if (!ctx) return fail(nullptr, EMB_EINVAL, "null context");
  ctx->profiling = enabled != 0;
  return EMB_OK;
}

int emb_stage_count(void) { return ST_COUNT; }
uint32_t emb_tile_entries(void) { return kTile; }

const char* emb_stage_name(int stage) { return (stage >= 0 && stage < ST_COUNT) ? kStageNames[stage] : ""; }

static int drain_events(emb_ctx* ctx) {
  CKH(hipSetDevice(ctx->device), "hipSetDevice");
  CKH(hipDeviceSynchronize(), "hipDeviceSynchronize");
  for (auto& r : ctx->recs) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.e0, r.e1) == hipSuccess) {
      ctx->stage_ms[r.stage] += ms;
      ctx->stage_launches[r.stage] += 1;
    }
    ctx->free_events.push_back(r.e0);
    ctx->free_events.push_back(r.e1);
  }
  ctx->recs.clear();
  return EMB_OK;
}

static int emb_read_stage_ms_impl(emb_ctx* ctx, float* ms, uint32_t* launches) {
  if (!ctx) return fail(nullptr, EMB_EINVAL, "null context");
  int rc = drain_events(ctx);
  if (rc) return rc;
  for (int i = 0; i < ST_COUNT; ++i) {
    if (ms) ms[i] = ctx->stage_ms[i];
    if (launches) launches[i] = ctx->stage_launches[i];
  }
  return EMB_OK;
}

static int emb_reset_stage_ms_impl(emb_ctx* ctx) {
  if (!ctx) return fail(nullptr, EMB_EINVAL, "null context");
  int rc = drain_events(ctx);
  if (rc) return rc;
  for (int i = 0; i < ST_COUNT; ++i) {
    ctx->stage_ms[i] = 0.f;
    ctx->stage_launches[i] = 0;
  }
  return EMB_OK;
}


// ---- exported entry points: no exception leaves the library ----
#define PEMB_GUARDED(ctx_expr, call)                                               \
  try {                                                                            \
    return call;                                                                   \
  } catch (const std::bad_alloc&) {                                                \
    return fail(ctx_expr, EMB_ENOMEM, "out of host memory");                       \
  } catch (...) {                                                                  \
    return fail(ctx_expr, EMB_ESTATE, "unexpected exception inside the library");  \
  }

int emb_create(const emb_config* cfg, emb_ctx** out) { PEMB_GUARDED(nullptr, emb_create_impl(cfg, nullptr, out)) }
int emb_create_cached(const emb_config* cfg, const uint64_t* cache_rows, emb_ctx** out) { PEMB_GUARDED(nullptr, emb_create_impl(cfg, cache_rows, out)) }
int emb_cache_stats(emb_ctx* ctx, uint32_t table, uint64_t* stats) { PEMB_GUARDED(ctx, emb_cache_stats_impl(ctx, table, stats)) }
int emb_cache_where(emb_ctx* ctx, uint32_t table, int32_t* where_host) { PEMB_GUARDED(ctx, emb_cache_where_impl(ctx, table, where_host)) }
int emb_cache_flush(emb_ctx* ctx, void* hip_stream) { PEMB_GUARDED(ctx, emb_cache_flush_impl(ctx, hip_stream)) }
int emb_lookup_pool(emb_ctx* ctx, const emb_batch* batch, float* pooled, void* hip_stream) { PEMB_GUARDED(ctx, emb_lookup_pool_impl(ctx, batch, pooled, hip_stream)) }
int emb_lookup_pool_indexed(emb_ctx* ctx, uint32_t batch_size, uint64_t num_unique, uint64_t num_ids, const uint64_t* keys,
                            const uint32_t* seg_off, const uint32_t* seg_bags, float* pooled, void* hip_stream) {
  PEMB_GUARDED(ctx, emb_lookup_pool_indexed_impl(ctx, batch_size, num_unique, num_ids, keys, seg_off, seg_bags, pooled, hip_stream))
}
int emb_hash_rows(emb_ctx* ctx, const emb_batch* batch, uint32_t* rows_out, void* hip_stream) { PEMB_GUARDED(ctx, emb_hash_rows_impl(ctx, batch, rows_out, hip_stream)) }
int emb_backward_update(emb_ctx* ctx, const emb_batch* batch, const float* d_pooled, void* hip_stream) { PEMB_GUARDED(ctx, emb_backward_update_impl(ctx, batch, d_pooled, hip_stream)) }
int emb_backward_update_static(emb_ctx* ctx, const emb_batch* batch, const float* d_pooled, void* hip_stream) { PEMB_GUARDED(ctx, emb_backward_update_static_impl(ctx, batch, d_pooled, hip_stream)) }
uint64_t emb_static_max_ids(void) { return kStaticMaxIds; }
int emb_dedup_sizes(emb_ctx* ctx, uint64_t* num_unique, uint64_t* num_ids) { PEMB_GUARDED(ctx, emb_dedup_sizes_impl(ctx, num_unique, num_ids)) }
int emb_read_dedup(emb_ctx* ctx, uint64_t* keys, uint32_t* seg_off, uint32_t* seg_bags) { PEMB_GUARDED(ctx, emb_read_dedup_impl(ctx, keys, seg_off, seg_bags)) }
int emb_read_rows(emb_ctx* ctx, uint32_t table, const uint64_t* rows, uint64_t n, float* w, float* acc) { PEMB_GUARDED(ctx, emb_read_rows_impl(ctx, table, rows, n, w, acc)) }
int emb_write_rows(emb_ctx* ctx, uint32_t table, const uint64_t* rows, uint64_t n, const float* w, const float* acc) { PEMB_GUARDED(ctx, emb_write_rows_impl(ctx, table, rows, n, w, acc)) }
int emb_read_stage_ms(emb_ctx* ctx, float* ms, uint32_t* launches) { PEMB_GUARDED(ctx, emb_read_stage_ms_impl(ctx, ms, launches)) }
int emb_reset_stage_ms(emb_ctx* ctx) { PEMB_GUARDED(ctx, emb_reset_stage_ms_impl(ctx)) }
#undef PEMB_GUARDED

static int codec_args_ok(const void* a, const void* b, const void* c, uint64_t n_blocks, uint32_t block_len, float kappa) {
  if (n_blocks == 0) return EMB_OK;
  if (!a || !b || !c) return fail(nullptr, EMB_EINVAL, "codec: null buffer");
  if (block_len == 0 || block_len % 4 != 0) return fail(nullptr, EMB_EINVAL, "codec: block_len must be a positive multiple of 4");
  if (!(kappa > 0.f) || kappa > 65504.f) return fail(nullptr, EMB_EINVAL, "codec: kappa must be in (0, 65504]");
  return EMB_OK;
}

int emb_codec_compress(const float* v, uint64_t n_blocks, uint32_t block_len, float kappa, uint16_t* q, float* norm,
                       void* hip_stream) {
  int rc = codec_args_ok(v, q, norm, n_blocks, block_len, kappa);
  if (rc) return rc;
  hipError_t e = launch_codec_compress(v, n_blocks, block_len, kappa, q, norm, (hipStream_t)hip_stream);
  return e == hipSuccess ? EMB_OK : fail_hip(nullptr, "codec_compress", e);
}

int emb_codec_decompress(const uint16_t* q, const float* norm, uint64_t n_blocks, uint32_t block_len, float kappa,
                         float* out, void* hip_stream) {
  int rc = codec_args_ok(q, norm, out, n_blocks, block_len, kappa);
  if (rc) return rc;
  hipError_t e = launch_codec_decompress(q, norm, n_blocks, block_len, kappa, out, (hipStream_t)hip_stream);
  return e == hipSuccess ? EMB_OK : fail_hip(nullptr, "codec_decompress", e);
}

uint64_t emb_device_bytes(emb_ctx* ctx) { return ctx ? ctx->device_bytes : 0; }
int emb_describe(emb_ctx* ctx, uint32_t* num_slots, uint32_t* pooled_width, uint32_t* max_batch, uint64_t* max_ids,
                 int32_t* device) {
  if (!ctx) return fail(nullptr, EMB_EINVAL, "null context");
  if (num_slots) *num_slots = ctx->S;
  if (pooled_width) *pooled_width = ctx->width;
  if (max_batch) *max_batch = ctx->max_batch;
  if (max_ids) *max_ids = ctx->max_ids;
  if (device) *device = ctx->device;
  return EMB_OK;
}

const char* emb_last_error(emb_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

}  // extern "C"
