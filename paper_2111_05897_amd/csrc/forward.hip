// Forward: hash + gather + per-slot sum pooling, and the key builder of the backward's dedup.
//
// gather_pool: a group of LANES adjacent lanes owns one bag; each lane owns 16 bytes of the row
// (4 fp32 or 8 bf16 elements), so a row read is one fully coalesced LANES*16-byte access and a
// wave keeps 64/LANES bags in flight.  Per round the group fetches max(LANES, 8) ids with one
// coalesced load, each lane hashes its own id(s), rows are broadcast inside the group, and eight
// row loads are issued before the first add so that every lane keeps several HBM requests in flight.
#include "device_utils.h"
#include "launch.h"

namespace pemb {
namespace {

struct GatherArgs {
  const uint64_t* ids;
  const int32_t* offsets;
  const void* w;
  const void* zeros;           // 512 bytes of zeros (the widest row): what a load past the end of a bag reads
  const int32_t* where;        // null, or row -> cache slot for a table kept behind the LRU cache
  uint64_t rows, mask;
  const uint32_t* slot_list;   // slots reading this table
  const uint64_t* slot_salt;   // indexed by slot
  const uint32_t* slot_col;    // indexed by slot
  uint32_t n_slots_t, S, width;
  uint32_t n_local_bags;       // B * n_slots_t
  uint32_t num_ids;            // offsets are clamped to [0, num_ids]: a malformed batch cannot read outside ids
  int mix;
  int stream_out;              // 1: the table serves every slot, so a launch writes whole rows of `pooled`
  float* pooled;
  // forward from the index form (INDEXED kernels): bag `g` holds entries [bag_beg[g], bag_end[g]) of entry_key,
  // entry_key[i] = position u of a unique key, keys64[u] = (table << 32) | row
  const uint32_t* bag_beg;
  const uint32_t* bag_end;
  const uint32_t* entry_key;
  const uint64_t* keys64;
  uint32_t num_unique, table;
};

// 16 bytes of a row as loaded, widened only when it is added.
template <typename T>
struct Raw16 {
  uint4 v;
  static constexpr int VEC = 16 / (int)sizeof(T);
  __device__ __forceinline__ void load(const T* p) { v = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void zero() { v = make_uint4(0u, 0u, 0u, 0u); }
  template <typename A>  // A = double for the per-bag sums, float where a single row is widened
  __device__ __forceinline__ void add_to(A (&s)[VEC]) const {
    if constexpr (sizeof(T) == 4) {
      s[0] += (A)__uint_as_float(v.x); s[1] += (A)__uint_as_float(v.y);
      s[2] += (A)__uint_as_float(v.z); s[3] += (A)__uint_as_float(v.w);
    } else {
      s[0] += (A)__uint_as_float(v.x << 16); s[1] += (A)__uint_as_float(v.x & 0xFFFF0000u);
      s[2] += (A)__uint_as_float(v.y << 16); s[3] += (A)__uint_as_float(v.y & 0xFFFF0000u);
      s[4] += (A)__uint_as_float(v.z << 16); s[5] += (A)__uint_as_float(v.z & 0xFFFF0000u);
      s[6] += (A)__uint_as_float(v.w << 16); s[7] += (A)__uint_as_float(v.w & 0xFFFF0000u);
    }
  }
};

// Value of `v` held by lane `src` of this lane's group of LANES adjacent lanes.
template <int LANES>
__device__ __forceinline__ uint32_t group_bcast(uint32_t v, int src) {
  if constexpr (LANES == 1) return v;
  else return (uint32_t)__shfl((int)v, src, LANES);
}

constexpr uint32_t kNoRow = 0xFFFFFFFFu;  // INDEXED: an entry that names no row of this table (malformed input) adds zeros

template <typename T, int D, bool INDEXED>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(sizeof(T) == 4 && D <= 64 ? 8 : 1, 8))) void k_gather_pool(GatherArgs a) {
  constexpr int VEC = 16 / (int)sizeof(T);
  constexpr int LANES = D / VEC;            // lanes that cover one row with 16 bytes each
  constexpr int GPB = kBlock / LANES;       // bags per workgroup
  constexpr int CH = LANES > 8 ? LANES : 8; // ids the group fetches and hashes per round, one or more per lane
  constexpr int IPL = CH / LANES;           // ids per lane per round
  constexpr int RIF = 8;                    // row loads in flight per lane (four: 0.418 -> 0.438 ms at config 2)
  static_assert(LANES >= 1 && LANES <= 64 && (LANES & (LANES - 1)) == 0, "row must map onto a power-of-two lane group");
  static_assert(CH % RIF == 0 && CH % LANES == 0, "round geometry");
  const uint32_t lb = blockIdx.x * GPB + threadIdx.x / LANES;
  const int lane = threadIdx.x % LANES;
  // What belongs to a bag -- its stretch of the ids, its slot's salt, where its pooled vector goes -- is fetched by one
  // thread per bag and handed to the bag's lanes through LDS: fetched by every lane, these five loads were a third of
  // the vector-memory instructions a wave issues for a bag of 8 rows.  (One lane per bag: nothing to share.)
  constexpr bool kStage = LANES >= 4;
  __shared__ int s_beg[kStage ? GPB : 1], s_end[kStage ? GPB : 1];
  __shared__ uint64_t s_salt[kStage ? GPB : 1], s_out[kStage ? GPB : 1];
  int beg = 0, end = 0;
  uint64_t salt = 0, out_at = 0;
  auto fetch_bag = [&](uint32_t l) {  // bag number l of this launch
    if (l >= a.n_local_bags) return;  // beg = end: nothing to read
    const uint32_t b = l / a.n_slots_t;
    const uint32_t slot = a.slot_list[l - b * a.n_slots_t];
    const size_t bag = (size_t)b * a.S + slot;
    beg = INDEXED ? (int)a.bag_beg[bag] : a.offsets[bag];
    end = INDEXED ? (int)a.bag_end[bag] : a.offsets[bag + 1];
    beg = beg < 0 ? 0 : beg;
    end = end > (int)a.num_ids ? (int)a.num_ids : end;  // beg >= end: an empty bag
    salt = a.slot_salt[slot];
    out_at = (uint64_t)b * a.width + a.slot_col[slot];
  };
  if constexpr (kStage) {
    if (threadIdx.x < GPB) {
      fetch_bag(blockIdx.x * GPB + threadIdx.x);
      s_beg[threadIdx.x] = beg;
      s_end[threadIdx.x] = end;
      s_salt[threadIdx.x] = salt;
      s_out[threadIdx.x] = out_at;
    }
    __syncthreads();
    const int g = threadIdx.x / LANES;
    beg = s_beg[g];
    end = s_end[g];
    salt = s_salt[g];
    out_at = s_out[g];
  } else {
    fetch_bag(lb);
  }
  if (lb >= a.n_local_bags) return;         // whole groups leave together
  const T* __restrict__ base = reinterpret_cast<const T*>(a.w) + lane * VEC;
  const T* __restrict__ zero_row = reinterpret_cast<const T*>(a.zeros) + lane * VEC;
  const uint64_t* __restrict__ ids = a.ids;

  // Rows are summed in batch order in fp64 and the sum is rounded once to fp32: the definition of the pooled
  // vector to within fp64 rounding, whatever the bag length or the cancellation between its rows.
  double acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = 0.0;

  for (int cbase = beg; cbase < end; cbase += CH) {
    const int cnt = end - cbase < CH ? end - cbase : CH;
    // each id of the round is loaded and hashed by exactly one lane of the group
    uint32_t myrow[IPL];
#pragma unroll
    for (int q = 0; q < IPL; ++q) {
      const int idx = cbase + q * LANES + lane;
      // ids are read once and pooled rows written once: with one table they are streamed past the caches, which
      // are kept for table rows (with several tables the launches share cache lines of both arrays)
      uint32_t r = 0u;
      if constexpr (INDEXED) {
        if (idx < end) {
          const uint32_t u = a.entry_key[idx];
          const uint64_t key = u < a.num_unique ? a.keys64[u] : ~0ull;
          r = ((uint32_t)(key >> 32) == a.table && (key & 0xFFFFFFFFull) < a.rows) ? (uint32_t)key : kNoRow;
        }
      } else {
        const uint64_t id = idx < end ? (a.stream_out ? __builtin_nontemporal_load(ids + idx) : ids[idx]) : 0ull;
        r = idx < end ? hash_row(id, salt, a.rows, a.mask, a.mix) : 0u;
      }
      if (a.where && r != kNoRow) {  // table behind the LRU cache: the row's slot (every row of the batch was admitted)
        const int32_t slot = idx < end ? a.where[r] : 0;
        r = slot >= 0 ? (uint32_t)slot : 0u;
      }
      myrow[q] = r;
    }
#pragma unroll
    for (int j0 = 0; j0 < CH; j0 += RIF) {
      if (j0 < cnt) {  // same for all lanes of the group
        // Every one of the RIF loads is issued, without a branch: past the bag's end it reads a row of zeros (one
        // cached line).  Straight-line code keeps all RIF requests in flight and the widening to fp64 behind them;
        // with a branch per row -- or one scalar branch around the second half of the loads, for waves none of whose
        // bags reaches it -- the compiler widens between the loads and waits for them in turn.
        Raw16<T> r[RIF];
#pragma unroll
        for (int jj = 0; jj < RIF; ++jj) {
          const int j = j0 + jj;  // compile-time: id j of the round sits in lane j % LANES, register j / LANES
          const uint32_t row = group_bcast<LANES>(myrow[j / LANES], j % LANES);
          r[jj].load((j < cnt && !(INDEXED && row == kNoRow)) ? base + (size_t)row * D : zero_row);
        }
#pragma unroll
        for (int jj = 0; jj < RIF; ++jj) r[jj].add_to(acc);
      }
    }
  }

  float* out = a.pooled + out_at + lane * VEC;
#pragma unroll
  for (int e = 0; e < VEC; e += 4)
    if (a.stream_out) {  // this launch writes whole pooled rows: streamed, nothing re-reads them here
      typedef float f32x4 __attribute__((ext_vector_type(4)));
      const f32x4 v = {(float)acc[e], (float)acc[e + 1], (float)acc[e + 2], (float)acc[e + 3]};
      __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(out + e));
    } else {  // several tables share the pooled rows: their pieces of a cache line must meet in the cache
      *reinterpret_cast<float4*>(out + e) =
          make_float4((float)acc[e], (float)acc[e + 1], (float)acc[e + 2], (float)acc[e + 3]);
    }
}

// A workgroup takes kKeyBags consecutive bags and walks their ids, one thread per id.  Everything that belongs to a
// bag -- its offset, its slot's hash parameters and key base, its payload -- is fetched once per bag into LDS; a
// thread finds the bag of id i by binary search over the staged offsets (the last bag whose offset is <= i: empty
// bags share their offset with the next one).  Per 64 ids the kernel then issues one coalesced load and two
// coalesced stores; with a group of lanes per bag it issued about eleven vector-memory instructions per 64 ids,
// most of them for bag metadata, and ran at the rate its texture-address unit takes instructions (0.092 ms at
// config 2 against what its 216 MB need at the copy rate: 0.042 ms).
// The offsets are checked on the way: 0 <= offsets[bag] <= n, non-decreasing, the first 0 and the last n -- together:
// the bags tile [0, n) exactly, so every key and payload slot below n is written.  A violation is recorded as
// bad_flag[0] = call (the number of this call); ids are only ever read, and keys written, inside [0, n), and the
// kernels that turn keys into addresses look at the flag first.
// The payload stored beside a key is the bag index, or -- payload_width != 0, contexts with several tables -- the
// position of the bag's gradient in d_pooled in units of 4 floats, (sample * payload_width + col(slot)) / 4: the
// segmented reduction then forms the gradient's address with one multiply.
constexpr int kKeyBags = 256;
static_assert(kKeyBags == kBlock, "one thread per bag while the bags' metadata is staged");
__global__ __launch_bounds__(kBlock) void k_build_keys(SlotArrays sl, const uint64_t* __restrict__ ids,
                                                       const int32_t* __restrict__ offsets, uint32_t n_bags,
                                                       uint32_t S, int mix, int bare_rows, uint32_t n,
                                                       uint32_t* __restrict__ keys_out,
                                                       uint32_t* __restrict__ bags_out, uint32_t* __restrict__ bad_flag,
                                                       uint32_t call, uint32_t payload_width) {
  __shared__ uint32_t s_off[kKeyBags + 1];
  __shared__ uint32_t s_pay[kKeyBags], s_kb[kKeyBags];
  __shared__ uint64_t s_salt[kKeyBags], s_rows[kKeyBags], s_mask[kKeyBags];
  const uint32_t bag0 = blockIdx.x * kKeyBags;
  const uint32_t nb = n_bags - bag0 < (uint32_t)kKeyBags ? n_bags - bag0 : (uint32_t)kKeyBags;  // bag0 < n_bags
  const uint32_t j = threadIdx.x;
  bool bad = false;
  for (uint32_t q = j; q <= nb; q += kBlock) {  // nb + 1 offsets: thread 0 also takes the last one
    const int32_t raw = offsets[bag0 + q];
    bad |= raw < 0 || (uint32_t)raw > n || (bag0 + q == 0 && raw != 0) || (bag0 + q == n_bags && (uint32_t)raw != n);
    s_off[q] = raw < 0 ? 0u : ((uint32_t)raw > n ? n : (uint32_t)raw);
  }
  if (j < nb) {
    const uint32_t bag = bag0 + j, slot = bag % S;
    s_salt[j] = sl.salt[slot];
    s_rows[j] = sl.rows[slot];
    s_mask[j] = sl.mask[slot];
    s_kb[j] = bare_rows ? 0u : sl.key_base[slot];
    s_pay[j] = payload_width ? (uint32_t)(((uint64_t)(bag / S) * payload_width + sl.col[slot]) >> 2) : bag;
  }
  __syncthreads();
  if (j < nb) bad |= s_off[j + 1] < s_off[j];
  if (bad && bad_flag) *bad_flag = call;  // every writer stores the same value
  const uint32_t lo = s_off[0], hi = s_off[nb];  // both inside [0, n]; lo > hi (inconsistent offsets): nothing to do
  for (uint32_t i = lo + j; i < hi; i += kBlock) {
    const uint64_t id = ids[i];
    uint32_t pos = 0;  // the last bag in [0, nb) whose offset is <= i
#pragma unroll
    for (uint32_t step = kKeyBags / 2; step >= 1; step >>= 1)
      if (pos + step < nb && s_off[pos + step] <= i) pos += step;
    keys_out[i] = s_kb[pos] + hash_row(id, s_salt[pos], s_rows[pos], s_mask[pos], mix);
    if (bags_out) bags_out[i] = s_pay[pos];
  }
}

template <typename T, int D>
hipError_t launch_gp(const GatherArgs& a, hipStream_t stream) {
  constexpr int LANES = D / (16 / (int)sizeof(T));
  constexpr int GPB = kBlock / LANES;
  const uint32_t grid = (a.n_local_bags + GPB - 1) / GPB;
  if (a.entry_key)
    hipLaunchKernelGGL((k_gather_pool<T, D, true>), dim3(grid), dim3(kBlock), 0, stream, a);
  else
    hipLaunchKernelGGL((k_gather_pool<T, D, false>), dim3(grid), dim3(kBlock), 0, stream, a);
  return hipGetLastError();
}

template <typename T>
hipError_t dispatch_dim(uint32_t dim, const GatherArgs& a, hipStream_t stream) {
  switch (dim) {
    case 8: return launch_gp<T, 8>(a, stream);
    case 16: return launch_gp<T, 16>(a, stream);
    case 32: return launch_gp<T, 32>(a, stream);
    case 64: return launch_gp<T, 64>(a, stream);
    case 128: return launch_gp<T, 128>(a, stream);
    default: return hipErrorInvalidValue;
  }
}

// ---- forward from the index form (section 4.2.3: the batch arrives as unique keys, each with the list of
// bags that hold it) ----
// The list is turned back into per-bag lists without atomics: every entry p of seg_bags becomes the pair
// (bag, u) with u the unique key whose segment holds p (k_expand_index), the pairs are sorted by bag with the
// stable radix sort of the dedup (a bag's entries then stand in ascending key order, whatever the launch), the
// first and last position of every bag are recorded (k_bag_bounds), and the gather kernel above runs with the
// bag's entries naming unique keys instead of ids.  The sums are fp64 in a fixed order: reproducible, and equal to
// emb_lookup_pool up to the order of fp64 additions.
struct ExpandArgs {
  const uint32_t* seg_off;   // [U + 1]
  const uint32_t* seg_bags;  // [N]
  uint32_t U, N, n_bags;
  uint32_t* key_out;         // [N] bag of the entry (n_bags for an entry that names no bag)
  uint32_t* val_out;         // [N] u of the entry
};

__global__ __launch_bounds__(kBlock) void k_expand_index(ExpandArgs a) {
  __shared__ uint32_t s_first;
  const uint32_t p0 = blockIdx.x * kBlock;
  if (threadIdx.x == 0) {  // the unique key entry p0 belongs to: the last u with seg_off[u] <= p0
    uint32_t lo = 0, hi = a.U;
    while (hi - lo > 1) {
      const uint32_t mid = lo + (hi - lo) / 2;
      if (a.seg_off[mid] <= p0) lo = mid;
      else hi = mid;
    }
    s_first = lo;
  }
  __syncthreads();
  const uint32_t p = p0 + threadIdx.x;
  if (p >= a.N) return;
  // entries of one block span at most kBlock segment starts: search that window only
  uint32_t lo = s_first, hi = s_first + kBlock + 1 < a.U ? s_first + kBlock + 1 : a.U;
  while (hi - lo > 1) {
    const uint32_t mid = lo + (hi - lo) / 2;
    if (a.seg_off[mid] <= p) lo = mid;
    else hi = mid;
  }
  if (hi < a.U && a.seg_off[hi] <= p) {  // only with empty segments in the input: search the rest of the list
    lo = hi;
    hi = a.U;
    while (hi - lo > 1) {
      const uint32_t mid = lo + (hi - lo) / 2;
      if (a.seg_off[mid] <= p) lo = mid;
      else hi = mid;
    }
  }
  const uint32_t bag = a.seg_bags[p];
  a.key_out[p] = bag < a.n_bags ? bag : a.n_bags;
  a.val_out[p] = lo;
}

// bag_beg / bag_end (zeroed first) from the pairs sorted by bag: position i starts the run of sorted[i] and ends
// the run of sorted[i - 1] when the two differ.  The sentinel bag n_bags is recorded like any other and never read.
__global__ __launch_bounds__(kBlock) void k_bag_bounds(const uint32_t* __restrict__ sorted, uint32_t n,
                                                       uint32_t* __restrict__ bag_beg, uint32_t* __restrict__ bag_end) {
  const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
  if (i >= n) return;
  const uint32_t k = sorted[i];
  if (i == 0 || sorted[i - 1] != k) {
    bag_beg[k] = i;
    if (i) bag_end[sorted[i - 1]] = i;
  }
  if (i == n - 1) bag_end[k] = n;
}

__global__ __launch_bounds__(kBlock) void k_zero_u32(uint32_t* __restrict__ p, uint64_t n) {
  for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (uint64_t)gridDim.x * kBlock) p[i] = 0u;
}

__global__ __launch_bounds__(kBlock) void k_zero_f32(float4* __restrict__ p, uint64_t n4) {
  for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < n4; i += (uint64_t)gridDim.x * kBlock)
    p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

}  // namespace

hipError_t launch_zero_f32(float* p, uint64_t n, hipStream_t stream) {  // n a multiple of 4, p 16-byte aligned
  if (n == 0) return hipSuccess;
  const uint64_t n4 = n / 4;
  const uint64_t blocks = (n4 + kBlock - 1) / kBlock;
  hipLaunchKernelGGL(k_zero_f32, dim3((uint32_t)(blocks > 16384 ? 16384 : blocks)), dim3(kBlock), 0, stream,
                     reinterpret_cast<float4*>(p), n4);
  return hipGetLastError();
}

hipError_t launch_zero_u32(uint32_t* p, uint64_t n, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  const uint64_t blocks = (n + kBlock - 1) / kBlock;
  hipLaunchKernelGGL(k_zero_u32, dim3((uint32_t)(blocks > 16384 ? 16384 : blocks)), dim3(kBlock), 0, stream, p, n);
  return hipGetLastError();
}

hipError_t launch_expand_index(const uint32_t* seg_off, const uint32_t* seg_bags, uint32_t U, uint32_t N, uint32_t n_bags,
                               uint32_t* key_out, uint32_t* val_out, hipStream_t stream) {
  if (N == 0 || U == 0) return hipSuccess;
  ExpandArgs a{seg_off, seg_bags, U, N, n_bags, key_out, val_out};
  hipLaunchKernelGGL(k_expand_index, dim3((N + kBlock - 1) / kBlock), dim3(kBlock), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_bag_bounds(const uint32_t* sorted_bags, uint32_t N, uint32_t* bag_beg, uint32_t* bag_end,
                             hipStream_t stream) {
  if (N == 0) return hipSuccess;
  hipLaunchKernelGGL(k_bag_bounds, dim3((N + kBlock - 1) / kBlock), dim3(kBlock), 0, stream, sorted_bags, N, bag_beg,
                     bag_end);
  return hipGetLastError();
}

hipError_t launch_gather_pool(const TableView& t, const SlotArrays& sl, const uint64_t* ids, const int32_t* offsets,
                              uint32_t num_ids, uint32_t B, uint32_t S, uint32_t width, int mix, const void* zeros,
                              float* pooled, hipStream_t stream, const IndexedBags* ix) {
  if (B == 0 || t.n_slots == 0) return hipSuccess;
  if (!zeros) return hipErrorInvalidValue;
  GatherArgs a;
  a.ids = ids;
  a.offsets = offsets;
  a.w = t.w;
  a.zeros = zeros;
  a.where = t.where;
  a.rows = t.rows;
  a.mask = t.mask;
  a.slot_list = t.slot_list;
  a.slot_salt = sl.salt;
  a.slot_col = sl.col;
  a.n_slots_t = t.n_slots;
  a.S = S;
  a.width = width;
  a.n_local_bags = B * t.n_slots;
  a.num_ids = num_ids;
  a.mix = mix;
  a.stream_out = t.n_slots == S ? 1 : 0;
  a.pooled = pooled;
  a.bag_beg = ix ? ix->bag_beg : nullptr;
  a.bag_end = ix ? ix->bag_end : nullptr;
  a.entry_key = ix ? ix->entry_key : nullptr;
  a.keys64 = ix ? ix->keys64 : nullptr;
  a.num_unique = ix ? ix->num_unique : 0u;
  a.table = ix ? ix->table : 0u;
  if (ix && (!ix->bag_beg || !ix->bag_end || !ix->entry_key || !ix->keys64)) return hipErrorInvalidValue;
  return t.dtype == 1 ? dispatch_dim<bf16_t>(t.dim, a, stream) : dispatch_dim<float>(t.dim, a, stream);
}

hipError_t launch_build_keys(const SlotArrays& sl, const uint64_t* ids, const int32_t* offsets, uint32_t num_ids,
                             uint32_t B, uint32_t S, int mix, int bare_rows, uint32_t* keys_out, uint32_t* bags_out,
                             uint32_t* bad_flag, uint32_t call, uint32_t payload_width, hipStream_t stream) {
  const uint32_t n_bags = B * S;
  if (n_bags == 0) return hipSuccess;
  const uint32_t grid = (n_bags + kKeyBags - 1) / kKeyBags;
  hipLaunchKernelGGL(k_build_keys, dim3(grid), dim3(kBlock), 0, stream, sl, ids, offsets, n_bags, S, mix, bare_rows,
                     num_ids, keys_out, bags_out, bad_flag, call, payload_width);
  return hipGetLastError();
}

}  // namespace pemb
