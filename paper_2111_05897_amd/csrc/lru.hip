// A table larger than device memory: the whole table lives in pinned host memory and the rows in use live in
// a cache of C slots in HBM, replaced least-recently-used first (section 4.2.2: the parameter server keeps the
// embedding parameters in an LRU cache built from an array list and a hash map whose "pointers" are indices).
//
// The same structure on the GPU: the array list is the slot arrays (cache_w, cache_acc, slot_row, stamp), and
// because rows are already dense indices after the hashing trick the hash map is a flat array where[row] ->
// slot (or -1).  Recency is kept per batch: every row a batch touches is stamped with the batch's step number,
// and when M rows are missing the M slots with the oldest stamps (ties, and all ages of kAgeMax - 1 steps or
// more, in slot order; empty slots first) are written back to the host table and refilled.  All lists are made by scans, not atomics, so the
// slot a row lands in is a function of the batch sequence only.
#include "device_utils.h"
#include "launch.h"

namespace pemb {
namespace {

constexpr uint32_t kLruTile = 2048;            // elements per workgroup of a compaction (8 per thread)
constexpr int kLruPer = kLruTile / kBlock;
constexpr int kPlanThreads = 1024;

// plan[] slots (device): filled per admission
enum { PL_MISSES = 0, PL_AGE = 1, PL_OLDER = 2, PL_TAKE = 3, PL_SCRATCH = 4, PL_COUNT = 8 };

// An empty slot (stamp 0; steps start at 1) is older than any row; rows idle for kAgeMax - 1 steps or more are
// equally old.
__device__ __forceinline__ uint32_t age_of(uint32_t stamp, uint32_t step) {
  if (stamp == 0) return kAgeMax;
  const uint32_t a = step - stamp;  // stamps are never in the future
  return a > kAgeMax - 1 ? kAgeMax - 1 : a;
}

// ---- predicates over an index range; each is evaluated twice (count pass, write pass) with the same result ----
struct MissPred {  // u: index into unique_keys; true if the row belongs to the table and is not cached
  const uint32_t* unique_keys;
  const uint32_t* counters;  // [0] = number of unique keys
  LruView v;
  uint32_t step;
  __device__ __forceinline__ uint32_t limit() const { return counters[0]; }
  __device__ __forceinline__ bool operator()(uint32_t u, uint32_t* out) const {
    const uint32_t key = unique_keys[u];
    if (key < v.key_base || (uint64_t)(key - v.key_base) >= v.rows) return false;  // another table's row
    const uint32_t row = key - v.key_base;
    const int32_t slot = v.where[row];
    if (slot >= 0) {
      v.stamp[slot] = step;  // a hit: most recently used (idempotent, so harmless in both passes)
      return false;
    }
    *out = row;
    return true;
  }
};
struct OlderPred {  // slot: true if strictly older than the threshold age
  LruView v;
  uint32_t step;
  const uint32_t* plan;
  __device__ __forceinline__ uint32_t limit() const { return v.C; }
  __device__ __forceinline__ bool operator()(uint32_t slot, uint32_t* out) const {
    const uint32_t st = v.stamp[slot];
    *out = slot;
    return st != step && age_of(st, step) > plan[PL_AGE];
  }
};
struct EqualPred {  // slot: true if exactly at the threshold age
  LruView v;
  uint32_t step;
  const uint32_t* plan;
  __device__ __forceinline__ uint32_t limit() const { return v.C; }
  __device__ __forceinline__ bool operator()(uint32_t slot, uint32_t* out) const {
    const uint32_t st = v.stamp[slot];
    *out = slot;
    return st != step && age_of(st, step) == plan[PL_AGE];
  }
};

template <typename Pred>
__global__ __launch_bounds__(kBlock) void k_compact_count(Pred p, uint32_t* __restrict__ blk_counts) {
  __shared__ uint32_t s_w[kWavesPerBlock];
  const uint32_t lim = p.limit();
  const uint32_t i0 = blockIdx.x * kLruTile + threadIdx.x * kLruPer;
  uint32_t c = 0, dummy;
#pragma unroll
  for (int j = 0; j < kLruPer; ++j)
    if (i0 + j < lim && p(i0 + j, &dummy)) ++c;
  uint32_t tot;
  block_exclusive_scan(c, s_w, &tot);
  if (threadIdx.x == 0) blk_counts[blockIdx.x] = tot;
}

// In-place exclusive scan of blk_counts[0..nb) by one workgroup; the total goes to *total.
__global__ __launch_bounds__(kPlanThreads) void k_scan_counts(uint32_t* __restrict__ blk_counts, uint32_t nb,
                                                              uint32_t* __restrict__ total) {
  constexpr int NW = kPlanThreads / kWave;
  __shared__ uint32_t s_w[NW];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  const uint32_t per = (nb + kPlanThreads - 1) / kPlanThreads;
  const uint32_t b0 = threadIdx.x * per;
  uint32_t sum = 0;
  for (uint32_t j = 0; j < per; ++j)
    if (b0 + j < nb) sum += blk_counts[b0 + j];
  uint32_t incl = sum;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const uint32_t t = __shfl_up(incl, off);
    if (lane >= off) incl += t;
  }
  if (lane == kWave - 1) s_w[wave] = incl;
  __syncthreads();
  uint32_t run = incl - sum, tot = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    if (w < wave) run += s_w[w];
    tot += s_w[w];
  }
  for (uint32_t j = 0; j < per; ++j)
    if (b0 + j < nb) {
      const uint32_t c = blk_counts[b0 + j];
      blk_counts[b0 + j] = run;
      run += c;
    }
  if (threadIdx.x == 0) *total = tot;
}

// Writes the values of the true elements, in index order, to out[out_base[0] + rank]; ranks >= cap[0] are dropped.
template <typename Pred>
__global__ __launch_bounds__(kBlock) void k_compact_write(Pred p, const uint32_t* __restrict__ blk_counts,
                                                          uint32_t* __restrict__ out,
                                                          const uint32_t* __restrict__ out_base,
                                                          const uint32_t* __restrict__ cap) {
  __shared__ uint32_t s_w[kWavesPerBlock];
  const uint32_t lim = p.limit();
  const uint32_t i0 = blockIdx.x * kLruTile + threadIdx.x * kLruPer;
  uint32_t val[kLruPer];
  bool on[kLruPer];
  uint32_t c = 0;
#pragma unroll
  for (int j = 0; j < kLruPer; ++j) {
    val[j] = 0;
    on[j] = i0 + j < lim && p(i0 + j, &val[j]);
    c += on[j] ? 1u : 0u;
  }
  uint32_t rank = blk_counts[blockIdx.x] + block_exclusive_scan(c, s_w, nullptr);
  const uint32_t base = out_base ? out_base[0] : 0u;
  const uint32_t limit = cap ? cap[0] : 0xFFFFFFFFu;
#pragma unroll
  for (int j = 0; j < kLruPer; ++j)
    if (on[j]) {
      if (rank < limit) out[base + rank] = val[j];
      ++rank;
    }
}

__global__ void k_lru_reset(uint32_t* __restrict__ age_hist, uint32_t* __restrict__ plan) {
  for (uint32_t i = threadIdx.x; i <= kAgeMax; i += blockDim.x) age_hist[i] = 0;
  if (threadIdx.x < PL_COUNT) plan[threadIdx.x] = 0;
}

// age_hist[a] = number of slots of age a that this batch does not use.
__global__ __launch_bounds__(kBlock) void k_lru_age_hist(LruView v, uint32_t step, uint32_t* __restrict__ age_hist) {
  __shared__ uint32_t s_h[kAgeMax + 1];
  for (uint32_t i = threadIdx.x; i <= kAgeMax; i += kBlock) s_h[i] = 0;
  __syncthreads();
  for (uint32_t s = blockIdx.x * kBlock + threadIdx.x; s < v.C; s += gridDim.x * kBlock) {
    const uint32_t st = v.stamp[s];
    if (st != step) atomicAdd(&s_h[age_of(st, step)], 1u);
  }
  __syncthreads();
  for (uint32_t i = threadIdx.x; i <= kAgeMax; i += kBlock)
    if (s_h[i]) atomicAdd(&age_hist[i], s_h[i]);
}

// From the number of misses M and the age histogram: the threshold age A (the youngest age that still has to
// give up slots), the number of slots strictly older than A, and how many slots of age exactly A are taken.
__global__ __launch_bounds__(kPlanThreads) void k_lru_plan(const uint32_t* __restrict__ age_hist,
                                                           uint32_t* __restrict__ plan, uint64_t* __restrict__ stats,
                                                           const uint32_t* __restrict__ counters, LruView v) {
  __shared__ uint32_t s_h[kAgeMax + 1];
  for (uint32_t i = threadIdx.x; i <= kAgeMax; i += kPlanThreads) s_h[i] = age_hist[i];
  __syncthreads();
  if (threadIdx.x != 0) return;
  uint32_t M = plan[PL_MISSES];
  uint32_t older = 0, age = kAgeMax, take = 0;
  if (M > 0) {
    uint32_t cum = 0;
    int a = (int)kAgeMax;
    for (; a >= 1; --a) {
      if (cum + s_h[a] >= M) break;
      cum += s_h[a];
    }
    if (a < 1) {  // fewer replaceable slots than misses (the cache size rule of emb_create_cached forbids it)
      a = 1;
      cum -= s_h[1];
      M = cum + s_h[1];
      plan[PL_MISSES] = M;
      stats[3] += 1;
    }
    age = (uint32_t)a;
    older = cum;
    take = M - cum;
  }
  plan[PL_AGE] = age;
  plan[PL_OLDER] = older;
  plan[PL_TAKE] = take;
  // rows of this table in the batch: misses + hits; the probe cannot count hits without atomics, so count here
  stats[1] += M;
  (void)counters;
  (void)v;
}

// A group of G lanes (16 bytes each: G = row bytes / 16) per replaced slot, kSwapRows slots per group at a time: write the
// old row back to the host table, bring the new row in.  The host link is a long pipe of small requests (a row is
// one or a few 64-byte reads), so what matters is how many rows are in flight: 64 / G groups per wave, kSwapRows rows
// per group, and all loads of a round (cache rows and host rows) issued before the first store.
constexpr int kSwapRows = 4;
template <typename T, int G>
__global__ __launch_bounds__(kBlock) void k_lru_swap(LruView v, uint32_t step, const uint32_t* __restrict__ plan,
                                                     const uint32_t* __restrict__ miss_list,
                                                     const uint32_t* __restrict__ victims, uint32_t* __restrict__ evicted) {
  constexpr int VEC = 16 / (int)sizeof(T);
  const int lane = threadIdx.x % G;
  const uint32_t gid = (blockIdx.x * kBlock + threadIdx.x) / G, ngroups = (gridDim.x * kBlock) / G;
  const uint32_t M = plan[PL_MISSES];
  T* cw = reinterpret_cast<T*>(v.cache_w);
  T* bw = reinterpret_cast<T*>(v.back_w);
  constexpr int R = kSwapRows;
  for (uint32_t i0 = gid; i0 < M; i0 += R * ngroups) {
    uint32_t slot[R], row[R], old[R];
    bool on[R], had[R];
    uint4 from_cache[R], from_host[R];
    float acc_cache[R], acc_host[R];
#pragma unroll
    for (int k = 0; k < R; ++k) {
      const uint32_t idx = i0 + k * ngroups;
      on[k] = idx < M;
      acc_cache[k] = acc_host[k] = 0.f;
      slot[k] = on[k] ? victims[idx] : 0u;
      row[k] = on[k] ? miss_list[idx] : 0u;
      old[k] = on[k] ? v.slot_row[slot[k]] : kEmptySlot;
      had[k] = old[k] != kEmptySlot;
    }
#pragma unroll
    for (int k = 0; k < R; ++k) {
      from_cache[k] = had[k] ? *reinterpret_cast<const uint4*>(cw + (size_t)slot[k] * v.dim + lane * VEC) : make_uint4(0, 0, 0, 0);
      from_host[k] = on[k] ? *reinterpret_cast<const uint4*>(bw + (size_t)row[k] * v.dim + lane * VEC) : make_uint4(0, 0, 0, 0);
      if (lane == 0) {
        if (had[k]) acc_cache[k] = v.cache_acc[slot[k]];
        if (on[k]) acc_host[k] = v.back_acc[row[k]];
      }
    }
    // every load above precedes the stores below in program order, so a slot is read before it is refilled
#pragma unroll
    for (int k = 0; k < R; ++k) {
      if (had[k]) {
        *reinterpret_cast<uint4*>(bw + (size_t)old[k] * v.dim + lane * VEC) = from_cache[k];
        if (lane == 0) {
          v.back_acc[old[k]] = acc_cache[k];
          v.where[old[k]] = -1;
          atomicAdd(evicted, 1u);
        }
      }
      if (on[k]) {
        *reinterpret_cast<uint4*>(cw + (size_t)slot[k] * v.dim + lane * VEC) = from_host[k];
        if (lane == 0) {
          v.cache_acc[slot[k]] = acc_host[k];
          v.slot_row[slot[k]] = row[k];
          v.stamp[slot[k]] = step;
          v.where[row[k]] = (int32_t)slot[k];
        }
      }
    }
  }
}

template <typename T>
hipError_t launch_swap_t(const LruView& v, uint32_t step, const uint32_t* plan, const uint32_t* miss_list,
                         const uint32_t* victims, uint32_t* evicted, uint32_t max_unique, hipStream_t stream) {
  const uint32_t G = v.dim * (uint32_t)sizeof(T) / 16u;   // 1 .. 32
  const uint64_t groups = ((uint64_t)max_unique + kSwapRows - 1) / kSwapRows;
  uint64_t blocks = (groups * G + kBlock - 1) / kBlock;
  blocks = blocks < 1 ? 1 : (blocks > 4096 ? 4096 : blocks);
#define PEMB_SWAP(GG)                                                                                                  \
  case GG:                                                                                                             \
    hipLaunchKernelGGL((k_lru_swap<T, GG>), dim3((uint32_t)blocks), dim3(kBlock), 0, stream, v, step, plan, miss_list,  \
                       victims, evicted);                                                                              \
    break;
  switch (G) {
    PEMB_SWAP(1) PEMB_SWAP(2) PEMB_SWAP(4) PEMB_SWAP(8) PEMB_SWAP(16) PEMB_SWAP(32)
    default: return hipErrorInvalidValue;
  }
#undef PEMB_SWAP
  return hipGetLastError();
}

__global__ void k_lru_fold_stats(uint64_t* __restrict__ stats, uint32_t* __restrict__ evicted,
                                 const uint32_t* __restrict__ table_unique) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    stats[2] += evicted[0];
    evicted[0] = 0;
    stats[0] += table_unique[0];  // rows of this table in the batch (hits = stats[0] - stats[1])
  }
}

// Counts the unique keys of the batch that belong to the table (for the statistics).
__global__ __launch_bounds__(kBlock) void k_lru_count_rows(const uint32_t* __restrict__ unique_keys,
                                                           const uint32_t* __restrict__ counters, LruView v,
                                                           uint32_t* __restrict__ table_unique) {
  __shared__ uint32_t s_w[kWavesPerBlock];
  const uint32_t U = counters[0];
  uint32_t c = 0;
  for (uint32_t u = blockIdx.x * kBlock + threadIdx.x; u < U; u += gridDim.x * kBlock) {
    const uint32_t key = unique_keys[u];
    if (key >= v.key_base && (uint64_t)(key - v.key_base) < v.rows) ++c;
  }
  uint32_t tot;
  block_exclusive_scan(c, s_w, &tot);
  if (threadIdx.x == 0 && tot) atomicAdd(table_unique, tot);
}

// keys[i] (a global row index of this table) -> key_base + slot of the row, for i in [range[0], range[1]);
// `range` null: every element whose key falls into the table, for i < count[0].
__global__ __launch_bounds__(kBlock) void k_lru_translate(uint32_t* __restrict__ keys, const uint32_t* __restrict__ range,
                                                          const uint32_t* __restrict__ count, uint32_t n_max, LruView v) {
  const uint32_t lo = range ? range[0] : 0u;
  const uint32_t hi = range ? range[1] : (count ? count[0] : n_max);
  for (uint32_t i = lo + blockIdx.x * kBlock + threadIdx.x; i < hi; i += gridDim.x * kBlock) {
    const uint32_t key = keys[i];
    if (key < v.key_base || (uint64_t)(key - v.key_base) >= v.rows) continue;
    const int32_t slot = v.where[key - v.key_base];
    // every row of the batch was admitted before this runs; a negative slot cannot occur, but must not be
    // turned into an address if it ever did: park it on slot 0's key, which the caller's statistics expose
    keys[i] = v.key_base + (slot >= 0 ? (uint32_t)slot : 0u);
  }
}

__global__ __launch_bounds__(kBlock) void k_lru_init(LruView v) {
  const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  for (uint64_t r = i; r < v.rows; r += stride) v.where[r] = -1;
  for (uint64_t s = i; s < v.C; s += stride) {
    v.slot_row[s] = kEmptySlot;
    v.stamp[s] = 0;
  }
}

// Every cached row back to the host table (the cache stays valid).
template <typename T>
__global__ __launch_bounds__(kBlock) void k_lru_flush(LruView v) {
  const int lane = threadIdx.x & (kWave - 1);
  const uint32_t wave = (blockIdx.x * kBlock + threadIdx.x) >> 6, nwaves = (gridDim.x * kBlock) >> 6;
  constexpr int VEC = 16 / (int)sizeof(T);
  const uint32_t chunks = v.dim / VEC;
  const T* cw = reinterpret_cast<const T*>(v.cache_w);
  T* bw = reinterpret_cast<T*>(v.back_w);
  for (uint32_t s = wave; s < v.C; s += nwaves) {
    const uint32_t row = v.slot_row[s];
    if (row == kEmptySlot) continue;
    if ((uint32_t)lane < chunks)
      *reinterpret_cast<uint4*>(bw + (size_t)row * v.dim + lane * VEC) =
          *reinterpret_cast<const uint4*>(cw + (size_t)s * v.dim + lane * VEC);
    if (lane == 0) v.back_acc[row] = v.cache_acc[s];
  }
}

uint32_t blocks_for(uint64_t n, uint32_t per, uint32_t cap) {
  uint64_t b = (n + per - 1) / per;
  if (b < 1) b = 1;
  return (uint32_t)(b > cap ? cap : b);
}

template <typename Pred>
hipError_t compact(const Pred& p, uint32_t n_max, uint32_t* blk_counts, uint32_t* total, uint32_t* out,
                   const uint32_t* out_base, const uint32_t* cap, hipStream_t stream) {
  const uint32_t nb = (n_max + kLruTile - 1) / kLruTile;
  if (nb == 0) return hipSuccess;
  hipLaunchKernelGGL(k_compact_count<Pred>, dim3(nb), dim3(kBlock), 0, stream, p, blk_counts);
  hipLaunchKernelGGL(k_scan_counts, dim3(1), dim3(kPlanThreads), 0, stream, blk_counts, nb, total);
  hipLaunchKernelGGL(k_compact_write<Pred>, dim3(nb), dim3(kBlock), 0, stream, p, (const uint32_t*)blk_counts, out,
                     out_base, cap);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_lru_init(const LruView& v, hipStream_t stream) {
  const uint64_t n = v.rows > v.C ? v.rows : v.C;
  hipLaunchKernelGGL(k_lru_init, dim3(blocks_for(n, kBlock, 1u << 16)), dim3(kBlock), 0, stream, v);
  return hipGetLastError();
}

hipError_t launch_lru_admit(const LruView& v, const LruScratch& s, const uint32_t* unique_keys, const uint32_t* counters,
                            uint32_t max_unique, uint32_t step, hipStream_t stream) {
  hipLaunchKernelGGL(k_lru_reset, dim3(1), dim3(kBlock), 0, stream, s.age_hist, s.plan);
  hipLaunchKernelGGL(k_lru_count_rows, dim3(blocks_for(max_unique, kBlock * 8, 1024)), dim3(kBlock), 0, stream, unique_keys,
                     counters, v, s.plan + PL_SCRATCH);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // 1. hits are stamped, misses listed (ascending key order)
  MissPred mp{unique_keys, counters, v, step};
  e = compact(mp, max_unique, s.blk_counts, s.plan + PL_MISSES, s.miss_list, nullptr, nullptr, stream);
  if (e != hipSuccess) return e;
  // 2. ages of the slots this batch does not use -> how far down the recency order the replacement reaches
  hipLaunchKernelGGL(k_lru_age_hist, dim3(blocks_for(v.C, kBlock * 8, 2048)), dim3(kBlock), 0, stream, v, step, s.age_hist);
  hipLaunchKernelGGL(k_lru_plan, dim3(1), dim3(kPlanThreads), 0, stream, (const uint32_t*)s.age_hist, s.plan, s.stats,
                     counters, v);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  // 3. victims: every slot older than the threshold, then the first `take` slots at the threshold, in slot order
  OlderPred op{v, step, s.plan};
  e = compact(op, v.C, s.blk_counts, s.plan + PL_SCRATCH + 1, s.victims, nullptr, nullptr, stream);
  if (e != hipSuccess) return e;
  EqualPred ep{v, step, s.plan};
  e = compact(ep, v.C, s.blk_counts, s.plan + PL_SCRATCH + 2, s.victims, s.plan + PL_OLDER, s.plan + PL_TAKE, stream);
  if (e != hipSuccess) return e;
  // 4. write back + refill
  e = v.dtype == 1 ? launch_swap_t<bf16_t>(v, step, s.plan, s.miss_list, s.victims, s.evicted, max_unique, stream)
                   : launch_swap_t<float>(v, step, s.plan, s.miss_list, s.victims, s.evicted, max_unique, stream);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_lru_fold_stats, dim3(1), dim3(64), 0, stream, s.stats, s.evicted, (const uint32_t*)(s.plan + PL_SCRATCH));
  return hipGetLastError();
}

hipError_t launch_lru_translate(const LruView& v, uint32_t* keys, const uint32_t* range, const uint32_t* count,
                                uint32_t n_max, hipStream_t stream) {
  if (n_max == 0) return hipSuccess;
  hipLaunchKernelGGL(k_lru_translate, dim3(blocks_for(n_max, kBlock * 4, 4096)), dim3(kBlock), 0, stream, keys, range, count,
                     n_max, v);
  return hipGetLastError();
}

hipError_t launch_lru_flush(const LruView& v, hipStream_t stream) {
  const uint32_t blocks = blocks_for((uint64_t)v.C * kWave, kBlock, 4096);
  if (v.dtype == 1) hipLaunchKernelGGL(k_lru_flush<bf16_t>, dim3(blocks), dim3(kBlock), 0, stream, v);
  else hipLaunchKernelGGL(k_lru_flush<float>, dim3(blocks), dim3(kBlock), 0, stream, v);
  return hipGetLastError();
}

}  // namespace pemb
