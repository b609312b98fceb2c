/* persia_emb.h -- C ABI of the MI355X embedding hot path.
 *
 * The library keeps the embedding parameter w^emb of a deep recommender resident in HBM
 * and implements the two operations the paper's training loop performs on it
 * (section 2.1: y = NN_{w_nn}(lookup_{w_emb}(x^ID), x^NID); section 3.1 / Algorithm 1:
 * get(x^ID) in the forward task, put(x^ID, F'^emb) plus the optimizer Omega^emb in the
 * backward task):
 *
 *   emb_lookup_pool      get + the embedding worker's aggregation (section 4.1, step 4):
 *                        hash every ID to a row, gather the rows, sum them per slot.
 *   emb_backward_update  put + update (section 4.1, step 7; Algorithm 1 backward task;
 *                        equation (2)): turn the gradient of the pooled activations into
 *                        one gradient per touched row, via the unique-key index form of
 *                        the batch (section 4.2.3, "Lossless compression"), and apply the
 *                        row's optimizer, whose state is stored beside the row
 *                        (section 4.2.2).
 *
 * Conventions
 *   - Every function returns an emb_status (0 = ok, negative = error) and never throws or
 *     aborts; on error outputs are untouched and emb_last_error() describes the failure.
 *   - "device" pointers are HIP device memory on the context's GPU, owned by the caller
 *     (e.g. torch tensors); "host" pointers are ordinary memory.  The library owns the
 *     tables, the optimizer state and its workspace, all sized in emb_create, so the hot
 *     calls allocate nothing.
 *   - Hot calls (emb_lookup_pool, emb_hash_rows, emb_backward_update) only enqueue work on
 *     the given hipStream_t (passed as void*, NULL = the null stream) and return; caller
 *     buffers must stay valid until the stream has passed the call.  The functions marked
 *     "synchronous" wait for the device.
 *   - A batch is CSR over bags: bag index = b * num_slots + s for sample b and slot s;
 *     ids[offsets[bag] .. offsets[bag+1]) are the bag's 64-bit IDs.  offsets must be
 *     non-decreasing with offsets[0] = 0 and offsets[B*S] = num_ids; this is a caller
 *     contract, checked on the device only (see below), never on the host.
 *   - Pooled activations and their gradient are fp32, row-major [B, W] with
 *     W = sum over slots of the slot's table dim; slot s occupies columns
 *     [col(s), col(s) + dim) where col(s) is the sum of the dims of slots before it.
 *   - A context is not thread-safe; calls on one context must be issued from one thread
 *     (or externally serialised).  An emb_lookup_pool and an emb_backward_update on
 *     different streams may overlap on the device if the caller orders them as it needs
 *     (bounded-staleness training, section 5: a lookup may read rows an earlier update is
 *     still writing).  Two emb_backward_update calls (or emb_lookup_pool_indexed, which
 *     uses the same buffers) must not overlap: the context has one workspace, and inside
 *     a call the id sort and the tile-order sort share its histogram buffers, which is
 *     safe only because a call's kernels run in order on one stream.  On a context with
 *     cached tables (emb_create_cached) every hot call uses that workspace; the library
 *     therefore makes a hot call that arrives on another stream wait for the previous one.
 *   - offsets that do not tile [0, num_ids) are the caller's error, but not a fault: ids
 *     are never read outside [0, num_ids), and emb_backward_update then leaves every row
 *     untouched (emb_dedup_sizes / emb_read_dedup report EMB_EINVAL for that batch).
 */
#ifndef PERSIA_EMB_H
#define PERSIA_EMB_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct emb_ctx emb_ctx; /* opaque */

typedef enum { EMB_OK = 0, EMB_EINVAL = -1, EMB_ENOMEM = -2, EMB_EDEVICE = -3, EMB_ESTATE = -4 } emb_status;
typedef enum { EMB_F32 = 0, EMB_BF16 = 1 } emb_dtype;          /* table storage type */
typedef enum { EMB_OPT_SGD = 0, EMB_OPT_ROWWISE_ADAGRAD = 1 } emb_opt_kind;
typedef enum { EMB_HASH_IDENTITY_MOD = 0, EMB_HASH_MIX_MOD = 1 } emb_hash_kind;

/* One embedding table: `rows` x `dim`, row-major, rows contiguous.
 * dim must be one of 8, 16, 32, 64, 128; sum of rows over all tables must be < 2^31. */
typedef struct {
  uint64_t rows;
  uint32_t dim;
  int32_t dtype; /* emb_dtype */
} emb_table_desc;

/* One ID-type feature group (section 2.1): which table it reads and the salt that makes
 * its IDs a key space of their own. */
typedef struct {
  uint32_t table;
  uint32_t reserved; /* must be 0 */
  uint64_t salt;
} emb_slot_desc;

/* hash:  EMB_HASH_IDENTITY_MOD: row = id mod rows.
 *        EMB_HASH_MIX_MOD:      row = mix64(id + salt) mod rows, with
 *          mix64(z): z ^= z>>31; z *= 0x9FB21C651E98DF25; z ^= z>>29;
 *                    z *= 0xC2B2AE3D27D4EB4F; z ^= z>>32   (arithmetic mod 2^64).
 *        Distinct IDs that hash to one row share it.
 * opt:   EMB_OPT_SGD:             w <- w - lr * G
 *        EMB_OPT_ROWWISE_ADAGRAD: a <- a + mean_d(G_d^2);  w_d <- w_d - lr * G_d / (sqrt(a) + eps)
 *        with G the sum of the upstream gradients of all occurrences of the row in the
 *        batch, a one fp32 accumulator per row (initially acc_init); one application per
 *        unique row per batch.  bf16 tables round the new row to nearest-even.
 * init:  element d of row r of table t starts at lo + (hi-lo) * k / 2^24, k = the top 24 bits of
 *        mix64(mix64(init_seed + (t+1)*0x9E3779B97F4A7C15) + r*dim + d), evaluated as
 *        float(k - 2^23) * ((hi-lo) * 2^-24) + (hi+lo)/2 with separate fp32 multiply and add.
 * max_batch / max_ids bound batch_size and num_ids of every later call (workspace sizing): max_ids < 2^31,
 * max_batch * num_slots < 2^31 and, with more than one table, max_batch * pooled width < 2^34 floats (the sorted index form
 * carries the position of a bag's gradient in d_pooled in 32 bits). */
typedef struct {
  uint32_t num_tables;
  uint32_t num_slots;
  const emb_table_desc* tables; /* host, [num_tables] */
  const emb_slot_desc* slots;   /* host, [num_slots]  */
  int32_t hash;                 /* emb_hash_kind */
  int32_t opt;                  /* emb_opt_kind  */
  float lr, eps, acc_init;
  float init_lo, init_hi;
  int32_t device;               /* HIP device ordinal */
  uint64_t init_seed;
  uint64_t max_ids;
  uint32_t max_batch;
  uint32_t reserved;            /* must be 0 */
} emb_config;

typedef struct {
  uint32_t batch_size;     /* B */
  uint32_t reserved;       /* must be 0 */
  uint64_t num_ids;        /* N = offsets[B * num_slots] */
  const uint64_t* ids;     /* device, [N] */
  const int32_t* offsets;  /* device, [B * num_slots + 1] */
} emb_batch;

/* Allocates and initialises tables, optimizer state and workspace on cfg->device
 * (synchronous).  On failure *out is untouched and emb_last_error(NULL) has the reason. */
int emb_create(const emb_config* cfg, emb_ctx** out);
int emb_destroy(emb_ctx* ctx); /* synchronous; frees everything the context owns */

/* Forward (section 2.1 lookup; Algorithm 1 forward task; section 4.1 step 4):
 * pooled[b, col(s) + d] = sum over ids i of bag (b, s) of W_table(s)[row(i), d], duplicates
 * counted with multiplicity, empty bags give zeros.  pooled: device, fp32 [B, W], written whole. */
int emb_lookup_pool(emb_ctx* ctx, const emb_batch* batch, float* pooled, void* hip_stream);

/* The forward from the index form (section 4.2.3: a batch compressed losslessly as its unique keys, each with
 * the list of places that hold it) -- the same pooled activations as emb_lookup_pool, from what emb_read_dedup
 * describes: keys[u] = (table << 32) | row strictly ascending (device, [num_unique]), seg_off (device,
 * [num_unique + 1], seg_off[0] = 0, seg_off[num_unique] = num_ids), seg_bags (device, [num_ids], bag = sample *
 * num_slots + slot).  The lists are turned back into per-bag lists by a stable sort of (bag, key position) pairs
 * -- no atomics -- and every bag sums its rows in fp64 in ascending key order: reproducible, and equal to
 * emb_lookup_pool up to the order of fp64 additions (i.e. bit for bit except where that order tips an fp32
 * rounding).  Entries that name no bag of the batch or no row of a table contribute nothing.
 * pooled: device fp32 [batch_size, W], written whole.  Uses the context's sort workspace: num_ids <= max_ids, and
 * the index form of an earlier emb_backward_update is gone afterwards (emb_read_dedup then returns EMB_ESTATE).
 * Not available for tables behind a cache.  This is the wire format of the paper put to use; with the table in
 * local HBM emb_lookup_pool is the faster forward, since the sort that undoes the compression costs more than the
 * repeated row reads it saves. */
int emb_lookup_pool_indexed(emb_ctx* ctx, uint32_t batch_size, uint64_t num_unique, uint64_t num_ids, const uint64_t* keys,
                            const uint32_t* seg_off, const uint32_t* seg_bags, float* pooled, void* hip_stream);

/* The hash step alone (section 4.2.2: the global hashing function that locates a parameter):
 * rows_out[i] = row of ids[i] in the table of its slot.  rows_out: device, uint32 [N]. */
int emb_hash_rows(emb_ctx* ctx, const emb_batch* batch, uint32_t* rows_out, void* hip_stream);

/* Backward + update (section 4.1 step 7; Algorithm 1 backward task; equation (2)) for the same
 * batch the forward saw.  d_pooled: device, fp32 [B, W], gradient of the loss w.r.t. pooled.
 * Builds the index form of the batch -- unique (table,row) keys ascending, and for each key
 * the bag indices holding it in batch order -- sums d_pooled over each key's bags, and applies
 * the optimizer once per unique row.  Rows not in the batch are not touched.  The index form
 * stays in the context's workspace until the next call on the context. */
int emb_backward_update(emb_ctx* ctx, const emb_batch* batch, const float* d_pooled, void* hip_stream);

/* emb_backward_update for callers that cannot allocate and cannot rely on a context sized for the batch: code
 * under HIP graph capture, tight serving loops that apply an occasional small update, harnesses that forbid
 * hipMalloc.  Same inputs, same result (bit for bit) and same index form left behind as emb_backward_update, but
 * every scratch buffer of the call (sort keys, histograms, unique keys, segment offsets, partial sums, tile order)
 * lives in one fixed array of 16 MiB that is part of the library's code object -- one copy per GPU, located once per
 * device in emb_create and held until the process ends -- so the call performs no allocation of any kind, whatever
 * max_ids the context was created with.  Limit: batch->num_ids <= emb_static_max_ids() (262144); beyond it the
 * call returns EMB_EINVAL and does nothing.  Not available for tables behind a cache (EMB_ESTATE).  No per-stage
 * timing is recorded for this call.  All contexts of a GPU share that GPU's array: calls to this function that
 * overlap on one GPU (two streams, two contexts, two threads) race, and the index form emb_read_dedup reports
 * after it is only valid until the next such call on that GPU.  Nothing in the array has to start at zero: every
 * buffer is written by the call before it is read. */
int emb_backward_update_static(emb_ctx* ctx, const emb_batch* batch, const float* d_pooled, void* hip_stream);
uint64_t emb_static_max_ids(void);

/* Inspection of the index form left by the last emb_backward_update (synchronous; for tests
 * and benchmarks).  keys[u] = (table << 32) | row, strictly ascending; seg_off[U+1] with
 * seg_off[0] = 0, seg_off[U] = N; seg_bags[N]: bag indices, non-decreasing inside a segment.
 * Host buffers; any of the three may be NULL. */
int emb_dedup_sizes(emb_ctx* ctx, uint64_t* num_unique, uint64_t* num_ids);
int emb_read_dedup(emb_ctx* ctx, uint64_t* keys, uint32_t* seg_off, uint32_t* seg_bags);

/* Copy rows of a table, widened to fp32, and their optimizer accumulators to the host /
 * overwrite them from the host (values rounded to the table's storage type).  Synchronous.
 * rows: host [n]; w: host fp32 [n, dim] or NULL; acc: host fp32 [n] or NULL. */
int emb_read_rows(emb_ctx* ctx, uint32_t table, const uint64_t* rows, uint64_t n, float* w, float* acc);
int emb_write_rows(emb_ctx* ctx, uint32_t table, const uint64_t* rows, uint64_t n, const float* w, const float* acc);

/* Device pointers to a table's storage and accumulators (library-owned; for checksums). */
int emb_table_ptr(emb_ctx* ctx, uint32_t table, void** w_dev, float** acc_dev);

/* Per-stage device timing.  While enabled, every hot call brackets each kernel stage with HIP
 * events on the call's stream; emb_read_stage_ms waits for the device and returns, per stage,
 * the accumulated milliseconds and number of launches since the last emb_reset_stage_ms.
 * Stage names: emb_stage_name(i) for 0 <= i < emb_stage_count(). */
int emb_set_profiling(emb_ctx* ctx, int enabled);
int emb_stage_count(void);
uint32_t emb_tile_entries(void); /* entries of the sorted occurrence list one lane-group reduces (for byte accounting) */
const char* emb_stage_name(int stage);
int emb_read_stage_ms(emb_ctx* ctx, float* ms, uint32_t* launches); /* host arrays [emb_stage_count()] */
int emb_reset_stage_ms(emb_ctx* ctx);

/* Lossy value codec for pooled activations and their gradients (section 4.2.3, "Lossy compression"):
 * every block of block_len consecutive fp32 values v is scaled by kappa / ||v||_inf and converted to
 * fp16 (round to nearest even); the inverse converts back to fp32 and divides by the same factor.
 * The factor is formed in fp32 from the stored norm on both sides.  A block of zeros is stored as zeros.
 * v, out: device fp32 [n_blocks * block_len]; q: device fp16 [n_blocks * block_len]; norm: device fp32
 * [n_blocks] (||v||_inf of each block, written by compress, read by decompress).  block_len must be a
 * multiple of 4, kappa finite and in (0, 65504]; values must be finite.  Enqueue-only; no context needed. */
int emb_codec_compress(const float* v, uint64_t n_blocks, uint32_t block_len, float kappa, uint16_t* q, float* norm,
                       void* hip_stream);
int emb_codec_decompress(const uint16_t* q, const float* norm, uint64_t n_blocks, uint32_t block_len, float kappa,
                         float* out, void* hip_stream);

/* ---- optional dense step: the network NN_{w_nn} of section 2.1, trained as in Algorithm 2 --------------
 * A feed-forward ReLU network with one logit: input [pooled | dense] of width widths[0] = pooled_width +
 * dense_width, hidden widths widths[1..L-1], widths[L] = 1; loss = binary cross-entropy on the logit,
 * averaged over the batch (loss_mean != 0) or summed as Algorithm 2 writes it (loss_mean == 0); Omega^nn =
 * plain SGD with rate lr on fp32 master weights.  Every product takes bf16 operands (inputs, weights,
 * stored activations and back-propagated deltas are rounded to bf16, nearest even) and accumulates in
 * fp32 on the matrix cores.  widths[0..L-1] and the batch must be multiples of 64.
 * mlp_create: weights[l] host fp32 [widths[l], widths[l+1]] row-major, biases[l] host fp32 [widths[l+1]];
 *   copied; synchronous.
 * mlp_step: one forward + backward + update (Algorithm 2) of a batch.  pooled: device fp32 [B, pooled_width]
 *   (what emb_lookup_pool wrote), dense: device fp32 [B, dense_width], labels: device fp32 [B] in {0,1};
 *   d_pooled: device fp32 [B, pooled_width], receives F'^emb, the gradient of the loss w.r.t. pooled, ready for
 *   emb_backward_update; loss: device fp32 [1].  Enqueue-only on the given stream.
 * mlp_read_weights: master weights and bias of a layer to the host (synchronous; either pointer may be NULL). */
typedef struct mlp_ctx mlp_ctx;
typedef struct {
  uint32_t num_layers;      /* L >= 2 */
  uint32_t pooled_width;
  uint32_t dense_width;
  uint32_t max_batch;
  const uint32_t* widths;   /* host, [L + 1] */
  float lr;
  int32_t loss_mean;
  int32_t device;
  uint32_t reserved;        /* must be 0 */
} mlp_config;
int mlp_create(const mlp_config* cfg, const float* const* weights, const float* const* biases, mlp_ctx** out);
int mlp_step(mlp_ctx* ctx, uint32_t batch, const float* pooled, const float* dense, const float* labels, float* d_pooled,
             float* loss, void* hip_stream);
int mlp_read_weights(mlp_ctx* ctx, uint32_t layer, float* w, float* b);
/* A fully asynchronous dense side, for comparison with the hybrid algorithm (section 3.1 describes what
 * asynchrony does to the dense network; Algorithm 2 itself is synchronous): with delay d > 0 the gradients
 * F'^nn of step t are applied at the beginning of step t + d + 1, so every step works with weights that miss
 * the last d updates (d = 0 is the synchronous step).  Set once, before the first mlp_step (EMB_ESTATE
 * otherwise); d <= 256; allocates d more sets of gradient buffers.  The gradients of the last d + 1 steps of a
 * run are never applied. */
int mlp_set_update_delay(mlp_ctx* ctx, uint32_t delay);
/* Inspection of what the last mlp_step left behind (synchronous; for tests): what = 0 stored activation of
 * `layer` (bf16 [B, widths[layer]]; layer 0 is the packed input), 1 back-propagated delta at the input of
 * layer `layer` >= 1 (bf16 [B, widths[layer]]), 2 weight gradient (fp32 [widths[layer], widths[layer+1]]),
 * 3 bias gradient (fp32 [widths[layer+1]]), 4 d loss / d logit (fp32 [B]).  `bytes` must be the exact size. */
int mlp_read_state(mlp_ctx* ctx, int what, uint32_t layer, void* host, uint64_t bytes);
int mlp_destroy(mlp_ctx* ctx);
uint64_t mlp_device_bytes(mlp_ctx* ctx);
/* The contraction the dense step is built from, on its own: C[M,N] = A[M,K] * Bt[N,K]^T with bf16 operands
 * (device, row strides lda / ldb in elements, multiples of 8; K a multiple of 64) and fp32 accumulation.
 * epilogue 0: C bf16 = relu(acc + bias[n]) (bias: device fp32 [N]); 1: C fp32 = acc; 2: C bf16 = acc where
 * the bf16 matrix mask[M,N] (row stride ldm) is positive, else 0.  Enqueue-only. */
int mlp_gemm_nt(int epilogue, const uint16_t* A, uint32_t lda, const uint16_t* Bt, uint32_t ldb, uint32_t M, uint32_t N,
                uint32_t K, void* C, uint32_t ldc, const float* bias, const uint16_t* mask, uint32_t ldm, void* hip_stream);
const char* mlp_last_error(mlp_ctx* ctx); /* ctx == NULL: the last failed mlp_create */

/* ---- hybrid step loop (section 3.2: the embedding layer is trained asynchronously, the dense network
 * synchronously; section 5: the staleness of the embedding parameters is bounded by tau) ------------------
 * hyb_submit hands over batch t = 0, 1, 2, ...: its lookup (Algorithm 1, forward task) is enqueued at once,
 * and batch t - tau -- whose pooled activations have been waiting since its own submission, like a sample in
 * the embedding worker's buffer -- gets its dense step (Algorithm 2) and its embedding put + optimizer
 * (Algorithm 1, backward task).  Events fix the order so that the lookup of batch t sees the updates of the
 * batches 0 .. t - tau - 1 and of no others (tau = 0 is fully synchronous training); the lookup of batch t
 * runs on a second stream beside the dense step of batch t - tau.  The results are those of the same calls
 * made one after the other in the order L(0)..L(tau), train(0), L(tau+1), train(1), ...
 * hyb_create: emb and mlp must live on one device and agree on the pooled width; they stay owned by the
 *   caller, must outlive the loop, and must not be used elsewhere between hyb_submit and hyb_sync.  Allocates
 *   tau + 1 sets of input copies and pooled activations.
 * hyb_submit: batch->ids / offsets, dense [B, dense_width], labels [B]: device buffers, copied by work
 *   enqueued in this call; they may be overwritten after hyb_wait_inputs (or hyb_sync) returns.  Enqueue-only.
 * hyb_drain: trains the batches that have been looked up but not trained (the last tau), in order.
 * hyb_sync: waits for everything enqueued.  hyb_counts: batches submitted / trained (enqueued) so far.
 * hyb_read_losses: losses[i] = loss of batch first + i as mlp_step reported it (synchronous; host array;
 *   the most recent 65536 trained batches are kept). */
typedef struct hyb_ctx hyb_ctx;
int hyb_create(emb_ctx* emb, mlp_ctx* mlp, uint32_t tau, hyb_ctx** out);
int hyb_submit(hyb_ctx* ctx, const emb_batch* batch, const float* dense, const float* labels);
int hyb_drain(hyb_ctx* ctx);
int hyb_sync(hyb_ctx* ctx);
int hyb_wait_inputs(hyb_ctx* ctx);
int hyb_counts(hyb_ctx* ctx, uint64_t* submitted, uint64_t* trained);
int hyb_read_losses(hyb_ctx* ctx, uint64_t first, uint64_t count, float* losses);
int hyb_destroy(hyb_ctx* ctx); /* synchronous; does not destroy emb or mlp */
const char* hyb_last_error(hyb_ctx* ctx); /* ctx == NULL: the last failed hyb_create */

/* ---- tables larger than device memory (section 4.2.2: the parameter server holds the embedding parameters
 * in an LRU cache -- an array list plus a hash map whose links are indices) --------------------------------
 * emb_create_cached is emb_create with cache_rows[t] (host, [num_tables]): 0, or a value >= rows, keeps table
 * t wholly in device memory; otherwise the table (rows and optimizer state) lives in pinned host memory and
 * cache_rows[t] slots of device memory hold the rows in use.  Every emb_lookup_pool and emb_backward_update
 * first brings the batch's rows in; a missing row replaces the least recently used slot (recency = the last
 * call that touched the row; ties, and everything idle for 1022 calls or more, in slot order), whose row is
 * written back to the host table first.  Results are those of a resident table, bit for bit.  Rule:
 * cache_rows[t] >= min(rows, max_ids), so that any batch fits at once.  emb_read_rows / emb_write_rows see a
 * row wherever it currently is.  Calls on such a context must not overlap (the cache is shared state), and in
 * it emb_lookup_pool builds the index form too (so emb_read_dedup then describes the looked-up batch).
 * emb_cache_stats: stats[0] rows requested (unique per call), [1] of those not in the cache, [2] rows written
 *   back, [3] calls that found fewer replaceable slots than missing rows (0 under the rule above); synchronous.
 * emb_cache_where: where_host[r] = slot of row r or -1 (host, [rows]; synchronous; for tests).
 * emb_cache_flush: writes every cached row back to the host table (the cache stays valid); enqueue-only. */
int emb_create_cached(const emb_config* cfg, const uint64_t* cache_rows, emb_ctx** out);
int emb_cache_stats(emb_ctx* ctx, uint32_t table, uint64_t* stats);
int emb_cache_where(emb_ctx* ctx, uint32_t table, int32_t* where_host);
int emb_cache_flush(emb_ctx* ctx, void* hip_stream);

/* Measurement aid (no part of the paper's path): the barest kernel with the path's access pattern.  Reads
 * n_reads rows of row_bytes (a power of two, 16 .. 512) at pseudo-random positions of the array base[rows * row_bytes]
 * (device), 16 bytes per lane, eight rows in flight per lane group, and discards them; hot_of_8 of every 8 reads fall
 * into the first hot_rows rows, the others anywhere (hot_of_8 = 0: all anywhere).  sink16: 16 bytes of device memory
 * that receive one value depending on the rows read.  Enqueue-only; the caller times it.  bench.py runs it on the
 * benchmark's own table and gradient buffer, so that the gather and the segmented reduction are set against what
 * this box delivers to random row reads rather than against a datasheet. */
int emb_probe_random_rows(const void* base, uint64_t rows, uint32_t row_bytes, uint64_t n_reads, uint64_t hot_rows,
                          uint32_t hot_of_8, void* sink16, void* hip_stream);

/* Shapes and limits a context was created with (any pointer may be NULL). */
int emb_describe(emb_ctx* ctx, uint32_t* num_slots, uint32_t* pooled_width, uint32_t* max_batch, uint64_t* max_ids,
                 int32_t* device);
int mlp_describe(mlp_ctx* ctx, uint32_t* pooled_width, uint32_t* dense_width, uint32_t* max_batch, int32_t* device);

/* Bytes of device memory the context holds (tables, state, workspace). */
uint64_t emb_device_bytes(emb_ctx* ctx);

/* Message of the last failed call on ctx (or of the last failed emb_create if ctx is NULL).
 * The pointer stays valid until the next failing call. */
const char* emb_last_error(emb_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* PERSIA_EMB_H */
