// Host-side launchers of the kernels; each only enqueues on `stream` and returns the launch status.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pemb {

// Occurrences per tile of the segmented reduce: one lane-group walks this many sorted occurrences.
constexpr uint32_t kTile = 64;
// Radix sort geometry: a block ranks and scatters tiles of 256 threads x 16 pairs (runs of one digit are
// then long enough to be written as whole cache lines).
constexpr uint32_t kSortTile = 4096;
constexpr uint32_t kSortMaxBlocks = 2048;
constexpr int kSortMaxBits = 9;                 // widest digit a pass may use (512 bins)
constexpr uint32_t kUniqueTile = 2048;

// What a kernel needs to know about one table.
struct TableView {
  void* w;            // [rows, dim] fp32 or bf16
  float* acc;         // [rows]
  uint64_t rows;
  uint64_t mask;      // rows-1 if rows is a power of two, else 0
  uint32_t dim;
  int32_t dtype;      // 0 fp32, 1 bf16
  uint32_t key_base;  // first global row index of the table (sort keys are key_base + row)
  uint32_t n_slots;   // slots reading this table
  const uint32_t* slot_list;  // device, [n_slots] slot indices, ascending
  // A table kept in host memory behind an LRU cache (else all null): w / acc above are then the cache's slot
  // arrays, where[row] is the slot holding a row or -1, back_w / back_acc the whole table in host memory.
  const int32_t* where;
  void* back_w;
  float* back_acc;
};

// ---- lru.hip: least-recently-used cache in HBM over a table in pinned host memory ----
constexpr uint32_t kAgeMax = 1023;            // recency is exact up to kAgeMax - 2 steps back; kAgeMax = an empty slot
constexpr uint32_t kEmptySlot = 0xFFFFFFFFu;  // slot_row value of a slot that holds nothing
struct LruView {
  int32_t* where;       // [rows] slot of a row, or -1
  uint32_t* slot_row;   // [C] row held by a slot, or kEmptySlot
  uint32_t* stamp;      // [C] step number of the slot's last use
  void* cache_w;        // [C, dim]
  float* cache_acc;     // [C]
  void* back_w;         // [rows, dim], host memory mapped into the device
  float* back_acc;      // [rows]
  uint32_t C, dim;
  int32_t dtype;
  uint32_t key_base;
  uint64_t rows;
};
struct LruScratch {       // shared by the cached tables of a context, used by one admission at a time
  uint32_t* blk_counts;   // [max(C, max_unique) / 2048 + 1]
  uint32_t* miss_list;    // [max_unique] rows to bring in, ascending
  uint32_t* victims;      // [max_unique] slots to replace
  uint32_t* age_hist;     // [kAgeMax + 1]
  uint32_t* plan;         // [8]
  uint32_t* evicted;      // [1]
  uint64_t* stats;        // [4] of the table being admitted: rows seen, misses, evictions, overflows
};
hipError_t launch_lru_init(const LruView& v, hipStream_t stream);
// Makes every row of unique_keys[0 .. counters[0]) that belongs to the table resident: hits are stamped with
// `step`, misses replace the least recently used slots (written back to the host table first).
hipError_t launch_lru_admit(const LruView& v, const LruScratch& s, const uint32_t* unique_keys, const uint32_t* counters,
                            uint32_t max_unique, uint32_t step, hipStream_t stream);
// keys[i] = key_base + slot of the row, for the table's elements in [range[0], range[1]) (range null: in
// [0, count[0]) or, with count null too, in [0, n_max)).
hipError_t launch_lru_translate(const LruView& v, uint32_t* keys, const uint32_t* range, const uint32_t* count,
                                uint32_t n_max, hipStream_t stream);
hipError_t launch_lru_flush(const LruView& v, hipStream_t stream);

// Per-slot arrays, device, [S] each.
struct SlotArrays {
  const uint64_t* salt;
  const uint64_t* rows;
  const uint64_t* mask;
  const uint32_t* key_base;
  const uint32_t* col;
};

// ---- table.hip ----
hipError_t launch_init_table(const TableView& t, uint64_t table_key, float scale, float mid, float acc_init,
                             hipStream_t stream);
hipError_t launch_read_rows(const TableView& t, const uint64_t* rows_dev, uint64_t n, float* w_out, float* acc_out,
                            hipStream_t stream);
hipError_t launch_write_rows(const TableView& t, const uint64_t* rows_dev, uint64_t n, const float* w_in,
                             const float* acc_in, hipStream_t stream);

// ---- forward.hip ----
// zeros: kZeroRowBytes of device memory holding zeros (read in place of rows past the end of a bag).
constexpr uint32_t kZeroRowBytes = 512;
// ix (optional): the forward from the index form -- a bag's entries are positions of unique keys instead of ids
// (ids / offsets are then not read): bag g holds entry_key[bag_beg[g] .. bag_end[g]), keys64[u] = (table << 32) | row.
struct IndexedBags {
  const uint32_t* bag_beg;
  const uint32_t* bag_end;
  const uint32_t* entry_key;
  const uint64_t* keys64;
  uint32_t num_unique, table;
};
hipError_t launch_gather_pool(const TableView& t, const SlotArrays& sl, const uint64_t* ids, const int32_t* offsets,
                              uint32_t num_ids, uint32_t B, uint32_t S, uint32_t width, int mix, const void* zeros,
                              float* pooled, hipStream_t stream, const IndexedBags* ix = nullptr);
// Pieces of the forward from the index form: (bag, u) pairs of every entry of the bag lists; first / last position
// of every bag in the pairs once sorted by bag (bag_beg / bag_end zeroed beforehand).
hipError_t launch_zero_f32(float* p, uint64_t n, hipStream_t stream);
hipError_t launch_zero_u32(uint32_t* p, uint64_t n, hipStream_t stream);
hipError_t launch_expand_index(const uint32_t* seg_off, const uint32_t* seg_bags, uint32_t U, uint32_t N, uint32_t n_bags,
                               uint32_t* key_out, uint32_t* val_out, hipStream_t stream);
hipError_t launch_bag_bounds(const uint32_t* sorted_bags, uint32_t N, uint32_t* bag_beg, uint32_t* bag_end,
                             hipStream_t stream);
// keys_out[i] = key_base(slot) + row (or the bare row when bare_rows != 0); bags_out may be null.  bad_flag
// (optional, device): receives `call` if the offsets do not tile [0, num_ids) bag by bag; nothing is written outside
// [0, num_ids) either way.  payload_width != 0: bags_out receives (sample * payload_width + col(slot)) / 4, the
// position of the bag's gradient in d_pooled in units of 4 floats, instead of the bag index.
hipError_t launch_build_keys(const SlotArrays& sl, const uint64_t* ids, const int32_t* offsets, uint32_t num_ids,
                             uint32_t B, uint32_t S, int mix, int bare_rows, uint32_t* keys_out, uint32_t* bags_out,
                             uint32_t* bad_flag, uint32_t call, uint32_t payload_width, hipStream_t stream);

// ---- sort.hip ----
struct SortPlan {
  uint32_t n, chunk, nblk;
  int passes, bits;
};
SortPlan make_sort_plan(uint32_t n, int key_bits, int max_bits);
// One LSD pass: digit = (key >> shift) & (2^bits - 1).  hist: [2^bits * nblk], total: [2^bits].
hipError_t launch_radix_hist(const SortPlan& p, int shift, const uint32_t* keys, uint32_t* hist, hipStream_t stream);
hipError_t launch_radix_scan(const SortPlan& p, uint32_t* hist, uint32_t* total, hipStream_t stream);
hipError_t launch_radix_scatter(const SortPlan& p, int shift, const uint32_t* kin, const uint32_t* pin,
                                uint32_t* kout, uint32_t* pout, const uint32_t* hist, const uint32_t* total,
                                hipStream_t stream);
// Run heads of the sorted keys -> unique_keys[U], seg_off[U+1], and multi_list[M] = indices u (ascending)
// of the runs that cross an edge between tiles of kTile positions; counters[0] = U, counters[1] = M,
// counters[2] = 0.
static_assert(kUniqueTile % kTile == 0, "a unique block must end on a tile edge");
hipError_t launch_unique(const uint32_t* keys, uint32_t n, uint32_t* blk_heads, uint32_t* blk_multi,
                         uint32_t* unique_keys, uint32_t* seg_off, uint32_t* multi_list, uint32_t* counters,
                         hipStream_t stream);

// ---- backward.hip ----
struct BackwardArgs {
  const uint32_t* keys;      // sorted, [n]
  const uint32_t* bags;      // sorted with the keys, [n]: the payload launch_build_keys wrote
  int payload_is_position;   // 1: the payload is (sample * width + col(slot)) / 4, the gradient's position in d_pooled in
                             // units of 4 floats (several tables); 0: it is the bag index and every slot has this
                             // table's dim, so the gradient of bag g starts at g * dim (one table)
  uint32_t n;
  const float* d_pooled;     // [B, width]
  double* partials;          // [2 * ntiles, pstride] fp64 partial sums of segments that cross tile edges
  uint32_t pstride;
  const uint32_t* range;     // device [2]: occurrences [range[0], range[1]) belong to this table; null = all
  const uint32_t* tile_perm; // device [ntiles]: order in which lane-groups take the tiles; null = ascending
  int opt;
  float lr, eps;
  // fix-up only
  const uint32_t* unique_keys;
  const uint32_t* seg_off;
  const uint32_t* counters;  // [0] = U, [1] = number of multi-tile segments, [2] = of those, the long ones
  const uint32_t* bad_flag;  // device word: equal to `call` if the batch's offsets were inconsistent -- then the kernels
  uint32_t call;             // that turn keys and bags into addresses do nothing
  const uint32_t* multi_list;
  const uint32_t* long_list; // multi-tile segments spanning more than 16 tiles (filled by launch_classify_multi)
};
hipError_t launch_table_ranges(const uint32_t* keys, uint32_t n, const uint32_t* key_base_dev, uint32_t num_tables,
                               uint32_t* ranges /*[num_tables+1]*/, hipStream_t stream);
// Processing order of the tiles: ascending by (table of the tile's first key, first bag of the tile >> shift),
// ties in tile order.  Each table's tiles are then contiguous in the order, and within a table
// tiles that read the same stretch of d_pooled run close together in time, so a gradient row
// that several hot keys need is fetched from HBM once and found in the memory-side cache afterwards.
// tile_key / tile_val: two buffers of ntiles entries each; returns the sorted permutation in *perm_out.
hipError_t launch_tile_order(const uint32_t* keys, const uint32_t* bags, uint32_t n, int shift,
                             const uint32_t* key_base_dev, uint32_t num_tables, uint32_t* const tile_key[2],
                             uint32_t* const tile_val[2], uint32_t* hist, uint32_t* total,
                             const uint32_t** perm_out, hipStream_t stream);
hipError_t launch_tile_reduce_update(const TableView& t, const BackwardArgs& a, hipStream_t stream);
hipError_t launch_classify_multi(const BackwardArgs& a, uint32_t* counters, uint32_t* long_list, hipStream_t stream);
hipError_t launch_fixup(const TableView& t, const BackwardArgs& a, hipStream_t stream);

// ---- gemm.hip ----
// C[M,N] = A[M,K] * Bt[N,K]^T, bf16 operands (row strides lda, ldb, multiples of 8), fp32 accumulation, K a
// multiple of 64.  epilogue 0: C bf16 = relu(acc + bias[n]); 1: C fp32 = acc; 2: C bf16 = acc where the bf16
// matrix `mask` (row stride ldm) is positive, else 0.  Ct (optional, bf16 epilogues only) receives C
// transposed, [N, M] with row stride ldct.  split_ws (optional, epilogue 1 only): fp32 scratch of
// split_ws_elems elements; with it a product of few output tiles and long K is cut along K into up to
// gemm_splits(M, N, K) partial products of M*N elements each, summed in a fixed order.
uint32_t gemm_splits(uint32_t M, uint32_t N, uint32_t K);
hipError_t launch_gemm_nt(int epilogue, const void* A, uint32_t lda, const void* Bt, uint32_t ldb, uint32_t M, uint32_t N,
                          uint32_t K, void* C, uint32_t ldc, const float* bias, const void* mask, uint32_t ldm,
                          hipStream_t stream, void* Ct = nullptr, uint32_t ldct = 0, float* split_ws = nullptr,
                          uint64_t split_ws_elems = 0);
hipError_t launch_transpose_bf16(const void* in, uint32_t R, uint32_t Cc, uint32_t ld_in, void* out, uint32_t ld_out,
                                 hipStream_t stream);

// ---- codec.hip ----
hipError_t launch_codec_compress(const float* v, uint64_t n_blocks, uint32_t block_len, float kappa, void* q_fp16,
                                 float* norm, hipStream_t stream);
hipError_t launch_codec_decompress(const void* q_fp16, const float* norm, uint64_t n_blocks, uint32_t block_len,
                                   float kappa, float* out, hipStream_t stream);

}  // namespace pemb
