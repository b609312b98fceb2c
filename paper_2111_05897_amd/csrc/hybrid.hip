// The hybrid step loop (section 3.2: embedding layer asynchronous, dense network synchronous; section 5: the
// staleness of the embedding parameters is bounded by tau).  Host-side scheduling only: every arithmetic step
// is one of the emb_* / mlp_* entry points.
//
// Batch t is looked up as soon as it is submitted, but trained (dense step, then the embedding put + optimizer)
// only when batch t + tau has been looked up.  The order is fixed by events, so the lookup of batch t sees the
// updates of the batches 0 .. t - tau - 1 and of no others -- the same result as running
//   L(0) .. L(tau);  [train(0), L(tau+1)];  [train(1), L(tau+2)]; ...
// on one stream -- while the lookup of batch t runs beside the dense step of batch t - tau on a second stream.
#include <hip/hip_runtime.h>

#include <string>
#include <vector>

#include "../../include/persia_emb.h"

namespace {
std::string g_hyb_create_error;
constexpr uint64_t kLossRing = 65536;  // losses of the most recent batches stay readable
}  // namespace

struct hyb_ctx {
  emb_ctx* emb = nullptr;
  mlp_ctx* mlp = nullptr;
  uint32_t tau = 0;
  int device = 0;
  uint32_t S = 0, P = 0, Dn = 0, max_batch = 0;
  uint64_t max_ids = 0;
  hipStream_t s_lookup = nullptr, s_train = nullptr;
  struct Slot {  // one in-flight batch: the library's own copy of its inputs, and its pooled activations
    uint64_t* ids = nullptr;
    int32_t* offsets = nullptr;
    float *dense = nullptr, *labels = nullptr, *pooled = nullptr;
    uint32_t B = 0;
    uint64_t N = 0;
    hipEvent_t looked_up = nullptr, updated = nullptr;
    bool used = false;
  };
  std::vector<Slot> ring;  // tau + 1 slots; batch t lives in slot t % (tau + 1)
  float* d_pooled = nullptr;
  float* losses = nullptr;  // [kLossRing], batch k at k % kLossRing
  hipEvent_t copied = nullptr;
  uint64_t submitted = 0, trained = 0;
  std::vector<void*> allocs;
  std::string err;
};

namespace {

int hfail(hyb_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg;
  else g_hyb_create_error = msg;
  return code;
}
int hfail_hip(hyb_ctx* c, const char* what, hipError_t e) {
  return hfail(c, e == hipErrorOutOfMemory ? EMB_ENOMEM : EMB_EDEVICE, std::string(what) + ": " + hipGetErrorString(e));
}

#define HCK(c, call, what)                               \
  do {                                                   \
    hipError_t e_ = (call);                              \
    if (e_ != hipSuccess) return hfail_hip(c, what, e_); \
  } while (0)

template <typename T>
hipError_t hyb_malloc(hyb_ctx* c, T** p, uint64_t count) {
  void* q = nullptr;
  hipError_t e = hipMalloc(&q, (count ? count : 1) * sizeof(T));
  if (e != hipSuccess) return e;
  c->allocs.push_back(q);
  *p = reinterpret_cast<T*>(q);
  return hipSuccess;
}

void hyb_release(hyb_ctx* c) {
  for (auto& s : c->ring) {
    if (s.looked_up) (void)hipEventDestroy(s.looked_up);
    if (s.updated) (void)hipEventDestroy(s.updated);
  }
  if (c->copied) (void)hipEventDestroy(c->copied);
  if (c->s_lookup) (void)hipStreamDestroy(c->s_lookup);
  if (c->s_train) (void)hipStreamDestroy(c->s_train);
  for (void* p : c->allocs) (void)hipFree(p);
  c->allocs.clear();
}

int hyb_create_impl(emb_ctx* emb, mlp_ctx* mlp, uint32_t tau, hyb_ctx** out) {
  if (!emb || !mlp || !out) return hfail(nullptr, EMB_EINVAL, "null argument");
  if (tau > 1024) return hfail(nullptr, EMB_EINVAL, "tau must be at most 1024");
  uint32_t S, W, eB, mP, mD, mB;
  uint64_t eN;
  int32_t edev, mdev;
  if (emb_describe(emb, &S, &W, &eB, &eN, &edev) != EMB_OK || mlp_describe(mlp, &mP, &mD, &mB, &mdev) != EMB_OK)
    return hfail(nullptr, EMB_EINVAL, "cannot describe the contexts");
  if (W != mP) return hfail(nullptr, EMB_EINVAL, "the network's pooled_width differs from the embedding layer's output width");
  if (edev != mdev) return hfail(nullptr, EMB_EINVAL, "the two contexts live on different devices");
  hyb_ctx* c = new hyb_ctx();
  struct Guard {
    hyb_ctx* c;
    ~Guard() {
      if (c) {
        hyb_release(c);
        delete c;
      }
    }
  } guard{c};
  c->emb = emb;
  c->mlp = mlp;
  c->tau = tau;
  c->device = edev;
  c->S = S;
  c->P = W;
  c->Dn = mD;
  c->max_batch = eB < mB ? eB : mB;
  c->max_ids = eN;
  HCK(nullptr, hipSetDevice(c->device), "hipSetDevice");
  // default priority on both streams
  HCK(nullptr, hipStreamCreateWithFlags(&c->s_lookup, hipStreamNonBlocking), "hipStreamCreate");
  HCK(nullptr, hipStreamCreateWithFlags(&c->s_train, hipStreamNonBlocking), "hipStreamCreate");
  HCK(nullptr, hipEventCreateWithFlags(&c->copied, hipEventDisableTiming), "hipEventCreate");
  c->ring.resize((size_t)tau + 1);
  const uint64_t bags = (uint64_t)c->max_batch * S;
  for (auto& s : c->ring) {
    HCK(nullptr, hyb_malloc(c, &s.ids, c->max_ids), "hipMalloc(ids)");
    HCK(nullptr, hyb_malloc(c, &s.offsets, bags + 1), "hipMalloc(offsets)");
    HCK(nullptr, hyb_malloc(c, &s.dense, (uint64_t)c->max_batch * c->Dn), "hipMalloc(dense)");
    HCK(nullptr, hyb_malloc(c, &s.labels, c->max_batch), "hipMalloc(labels)");
    HCK(nullptr, hyb_malloc(c, &s.pooled, (uint64_t)c->max_batch * c->P), "hipMalloc(pooled)");
    HCK(nullptr, hipEventCreateWithFlags(&s.looked_up, hipEventDisableTiming), "hipEventCreate");
    HCK(nullptr, hipEventCreateWithFlags(&s.updated, hipEventDisableTiming), "hipEventCreate");
  }
  HCK(nullptr, hyb_malloc(c, &c->d_pooled, (uint64_t)c->max_batch * c->P), "hipMalloc(d_pooled)");
  HCK(nullptr, hyb_malloc(c, &c->losses, kLossRing), "hipMalloc(losses)");
  guard.c = nullptr;
  *out = c;
  return EMB_OK;
}

emb_batch slot_batch(const hyb_ctx::Slot& s) {
  emb_batch b;
  b.batch_size = s.B;
  b.reserved = 0;
  b.num_ids = s.N;
  b.ids = s.ids;
  b.offsets = s.offsets;
  return b;
}

// Dense step and embedding update of batch k on the training stream.  `after_lookup` (may be null): the
// event of the youngest lookup that must not see this update.
int train_one(hyb_ctx* c, uint64_t k, hipEvent_t after_lookup) {
  hyb_ctx::Slot& s = c->ring[k % c->ring.size()];
  HCK(c, hipStreamWaitEvent(c->s_train, s.looked_up, 0), "hipStreamWaitEvent(pooled)");
  if (mlp_step(c->mlp, s.B, s.pooled, s.dense, s.labels, c->d_pooled, c->losses + k % kLossRing, c->s_train) != EMB_OK)
    return hfail(c, EMB_EDEVICE, std::string("mlp_step: ") + mlp_last_error(c->mlp));
  if (after_lookup) HCK(c, hipStreamWaitEvent(c->s_train, after_lookup, 0), "hipStreamWaitEvent(lookup)");
  const emb_batch b = slot_batch(s);
  if (emb_backward_update(c->emb, &b, c->d_pooled, c->s_train) != EMB_OK)
    return hfail(c, EMB_EDEVICE, std::string("emb_backward_update: ") + emb_last_error(c->emb));
  HCK(c, hipEventRecord(s.updated, c->s_train), "hipEventRecord(updated)");
  c->trained = k + 1;
  return EMB_OK;
}

int hyb_submit_impl(hyb_ctx* c, const emb_batch* batch, const float* dense, const float* labels) {
  if (!c) return hfail(nullptr, EMB_EINVAL, "null context");
  if (!batch || !batch->ids || !batch->offsets || !labels || (c->Dn && !dense)) return hfail(c, EMB_EINVAL, "null buffer");
  if (batch->reserved != 0) return hfail(c, EMB_EINVAL, "batch.reserved must be 0");
  if (batch->batch_size == 0 || batch->batch_size > c->max_batch || batch->batch_size % 64 != 0)
    return hfail(c, EMB_EINVAL, "batch_size must be a multiple of 64 within max_batch");
  if (batch->num_ids > c->max_ids) return hfail(c, EMB_EINVAL, "num_ids exceeds max_ids");
  HCK(c, hipSetDevice(c->device), "hipSetDevice");
  const uint64_t t = c->submitted;
  hyb_ctx::Slot& s = c->ring[t % c->ring.size()];
  // The slot last held batch t - tau - 1: its update is the youngest one this lookup may see, and its inputs
  // may be overwritten once that update has run.
  if (s.used) HCK(c, hipStreamWaitEvent(c->s_lookup, s.updated, 0), "hipStreamWaitEvent(updated)");
  s.B = batch->batch_size;
  s.N = batch->num_ids;
  s.used = true;
  const uint64_t bags = (uint64_t)s.B * c->S;
  if (s.N) HCK(c, hipMemcpyAsync(s.ids, batch->ids, s.N * sizeof(uint64_t), hipMemcpyDeviceToDevice, c->s_lookup), "copy(ids)");
  HCK(c, hipMemcpyAsync(s.offsets, batch->offsets, (bags + 1) * sizeof(int32_t), hipMemcpyDeviceToDevice, c->s_lookup),
      "copy(offsets)");
  if (c->Dn)
    HCK(c, hipMemcpyAsync(s.dense, dense, (uint64_t)s.B * c->Dn * sizeof(float), hipMemcpyDeviceToDevice, c->s_lookup),
        "copy(dense)");
  HCK(c, hipMemcpyAsync(s.labels, labels, (uint64_t)s.B * sizeof(float), hipMemcpyDeviceToDevice, c->s_lookup), "copy(labels)");
  HCK(c, hipEventRecord(c->copied, c->s_lookup), "hipEventRecord(copied)");
  const emb_batch b = slot_batch(s);
  if (emb_lookup_pool(c->emb, &b, s.pooled, c->s_lookup) != EMB_OK)
    return hfail(c, EMB_EDEVICE, std::string("emb_lookup_pool: ") + emb_last_error(c->emb));
  HCK(c, hipEventRecord(s.looked_up, c->s_lookup), "hipEventRecord(looked_up)");
  c->submitted = t + 1;
  if (t >= c->tau) return train_one(c, t - c->tau, s.looked_up);
  return EMB_OK;
}

int hyb_drain_impl(hyb_ctx* c) {
  if (!c) return hfail(nullptr, EMB_EINVAL, "null context");
  HCK(c, hipSetDevice(c->device), "hipSetDevice");
  while (c->trained < c->submitted) {
    const int rc = train_one(c, c->trained, nullptr);
    if (rc != EMB_OK) return rc;
  }
  return EMB_OK;
}

int hyb_sync_impl(hyb_ctx* c) {
  if (!c) return hfail(nullptr, EMB_EINVAL, "null context");
  HCK(c, hipSetDevice(c->device), "hipSetDevice");
  HCK(c, hipStreamSynchronize(c->s_lookup), "hipStreamSynchronize");
  HCK(c, hipStreamSynchronize(c->s_train), "hipStreamSynchronize");
  return EMB_OK;
}

int hyb_read_losses_impl(hyb_ctx* c, uint64_t first, uint64_t count, float* losses) {
  if (!c) return hfail(nullptr, EMB_EINVAL, "null context");
  if (!losses && count) return hfail(c, EMB_EINVAL, "null buffer");
  if (first + count > c->trained) return hfail(c, EMB_EINVAL, "batches not trained yet");
  if (c->trained - first > kLossRing) return hfail(c, EMB_EINVAL, "losses that old are no longer kept");
  const int rc = hyb_sync_impl(c);
  if (rc != EMB_OK) return rc;
  for (uint64_t i = 0; i < count;) {  // the ring may wrap
    const uint64_t at = (first + i) % kLossRing;
    const uint64_t run = (count - i < kLossRing - at) ? count - i : kLossRing - at;
    HCK(c, hipMemcpy(losses + i, c->losses + at, run * sizeof(float), hipMemcpyDeviceToHost), "hipMemcpy(losses)");
    i += run;
  }
  return EMB_OK;
}

}  // namespace

extern "C" {

#define HYB_GUARDED(ctx_expr, call)                                                 \
  try {                                                                             \
    return call;                                                                    \
  } catch (const std::bad_alloc&) {                                                 \
    return hfail(ctx_expr, EMB_ENOMEM, "host allocation failed");                   \
  } catch (const std::exception& e) {                                               \
    return hfail(ctx_expr, EMB_EDEVICE, std::string("unexpected exception: ") + e.what()); \
  } catch (...) {                                                                   \
    return hfail(ctx_expr, EMB_EDEVICE, "unexpected exception");                    \
  }

int hyb_create(emb_ctx* emb, mlp_ctx* mlp, uint32_t tau, hyb_ctx** out) { HYB_GUARDED(nullptr, hyb_create_impl(emb, mlp, tau, out)) }
int hyb_submit(hyb_ctx* ctx, const emb_batch* batch, const float* dense, const float* labels) {
  HYB_GUARDED(ctx, hyb_submit_impl(ctx, batch, dense, labels))
}
int hyb_drain(hyb_ctx* ctx) { HYB_GUARDED(ctx, hyb_drain_impl(ctx)) }
int hyb_sync(hyb_ctx* ctx) { HYB_GUARDED(ctx, hyb_sync_impl(ctx)) }
int hyb_wait_inputs(hyb_ctx* ctx) {
  if (!ctx) return hfail(nullptr, EMB_EINVAL, "null context");
  hipError_t e = hipEventSynchronize(ctx->copied);
  return e == hipSuccess ? EMB_OK : hfail_hip(ctx, "hipEventSynchronize", e);
}
int hyb_counts(hyb_ctx* ctx, uint64_t* submitted, uint64_t* trained) {
  if (!ctx) return hfail(nullptr, EMB_EINVAL, "null context");
  if (submitted) *submitted = ctx->submitted;
  if (trained) *trained = ctx->trained;
  return EMB_OK;
}
int hyb_read_losses(hyb_ctx* ctx, uint64_t first, uint64_t count, float* losses) {
  HYB_GUARDED(ctx, hyb_read_losses_impl(ctx, first, count, losses))
}
int hyb_destroy(hyb_ctx* ctx) {
  if (!ctx) return EMB_OK;
  (void)hipSetDevice(ctx->device);
  (void)hipDeviceSynchronize();
  hyb_release(ctx);
  delete ctx;
  return EMB_OK;
}
const char* hyb_last_error(hyb_ctx* ctx) { return ctx ? ctx->err.c_str() : g_hyb_create_error.c_str(); }

}  // extern "C"
