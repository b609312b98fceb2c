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
  int mix;
  int stream_out;              // 1: the table serves every slot, so a launch writes whole rows of `pooled`
  float* pooled;
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

template <typename T, int D>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(sizeof(T) == 4 && D <= 64 ? 8 : 1, 8))) void k_gather_pool(GatherArgs a) {
  constexpr int VEC = 16 / (int)sizeof(T);
  constexpr int LANES = D / VEC;            // lanes that cover one row with 16 bytes each
  constexpr int GPB = kBlock / LANES;       // bags per workgroup
  constexpr int CH = LANES > 8 ? LANES : 8; // ids the group fetches and hashes per round, one or more per lane
  constexpr int IPL = CH / LANES;           // ids per lane per round
  constexpr int RIF = 8;                    // row loads in flight per lane
  static_assert(LANES >= 1 && LANES <= 64 && (LANES & (LANES - 1)) == 0, "row must map onto a power-of-two lane group");
  static_assert(CH % RIF == 0 && CH % LANES == 0, "round geometry");
  const uint32_t lb = blockIdx.x * GPB + threadIdx.x / LANES;
  const int lane = threadIdx.x % LANES;
  if (lb >= a.n_local_bags) return;         // whole groups leave together
  const uint32_t b = lb / a.n_slots_t;
  const uint32_t slot = a.slot_list[lb - b * a.n_slots_t];
  const size_t bag = (size_t)b * a.S + slot;
  const int beg = a.offsets[bag], end = a.offsets[bag + 1];
  const uint64_t salt = a.slot_salt[slot];
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
      const uint64_t id = idx < end ? (a.stream_out ? __builtin_nontemporal_load(ids + idx) : ids[idx]) : 0ull;
      uint32_t r = idx < end ? hash_row(id, salt, a.rows, a.mask, a.mix) : 0u;
      if (a.where) {  // table behind the LRU cache: the row's slot (every row of the batch was admitted)
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
        // with a branch per row the compiler widens inside the branch and waits for every load in turn.
        Raw16<T> r[RIF];
#pragma unroll
        for (int jj = 0; jj < RIF; ++jj) {
          const int j = j0 + jj;  // compile-time: id j of the round sits in lane j % LANES, register j / LANES
          const uint32_t row = group_bcast<LANES>(myrow[j / LANES], j % LANES);
          r[jj].load(j < cnt ? base + (size_t)row * D : zero_row);
        }
#pragma unroll
        for (int jj = 0; jj < RIF; ++jj) r[jj].add_to(acc);
      }
    }
  }

  float* out = a.pooled + (size_t)b * a.width + a.slot_col[slot] + lane * VEC;
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

// 8 lanes per bag; lane j takes ids beg+j, beg+j+8, ...
__global__ __launch_bounds__(kBlock) void k_build_keys(SlotArrays sl, const uint64_t* __restrict__ ids,
                                                       const int32_t* __restrict__ offsets, uint32_t n_bags,
                                                       uint32_t S, int mix, int bare_rows,
                                                       uint32_t* __restrict__ keys_out,
                                                       uint32_t* __restrict__ bags_out) {
  const uint32_t bag = blockIdx.x * (kBlock / 8) + threadIdx.x / 8;
  const int lane = threadIdx.x % 8;
  if (bag >= n_bags) return;
  const uint32_t slot = bag % S;
  const int beg = offsets[bag], end = offsets[bag + 1];
  const uint64_t salt = sl.salt[slot], rows = sl.rows[slot], mask = sl.mask[slot];
  const uint32_t kb = bare_rows ? 0u : sl.key_base[slot];
  for (int i = beg + lane; i < end; i += 8) {
    keys_out[i] = kb + hash_row(ids[i], salt, rows, mask, mix);
    if (bags_out) bags_out[i] = bag;
  }
}

template <typename T, int D>
hipError_t launch_gp(const GatherArgs& a, hipStream_t stream) {
  constexpr int LANES = D / (16 / (int)sizeof(T));
  constexpr int GPB = kBlock / LANES;
  const uint32_t grid = (a.n_local_bags + GPB - 1) / GPB;
  hipLaunchKernelGGL((k_gather_pool<T, D>), dim3(grid), dim3(kBlock), 0, stream, a);
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
// A group of LANES lanes walks a tile of kTile entries of the bag list.  The table row of the unique key the
// entries belong to is read once per (tile, key) and added into the pooled rows of the listed bags with
// hardware fp32 atomics: a bag's sum then forms in no fixed order (fp32 rounding may differ from run to run,
// inside the forward's tolerance), which is the price of reading each row once.  pooled must start at zero.
struct IndexedArgs {
  const uint64_t* keys;      // [U] (table << 32) | row, ascending
  const uint32_t* seg_off;   // [U + 1]
  const uint32_t* seg_bags;  // [N]
  uint32_t U, N;
  const void* w;
  const int32_t* where;
  uint32_t table;
  uint64_t rows;
  const uint32_t* slot_col;
  uint32_t S, width, n_bags;
  float* pooled;
};

template <typename T, int D>
__global__ __launch_bounds__(kBlock) void k_indexed_pool(IndexedArgs a) {
  constexpr int VEC = 16 / (int)sizeof(T);
  constexpr int LANES = D / VEC;
  constexpr int GPB = kBlock / LANES;
  const uint32_t tile = blockIdx.x * GPB + threadIdx.x / LANES;
  const int lane = threadIdx.x % LANES;
  const uint64_t p0 = (uint64_t)tile * kTile;
  if (p0 >= a.N) return;
  const uint32_t p1 = (a.N - p0 < kTile) ? a.N : (uint32_t)p0 + kTile;
  // the unique key entry p0 belongs to: the last u with seg_off[u] <= p0 (seg_off[U] = N > p0)
  uint32_t lo = 0, hi = a.U;
  while (hi - lo > 1) {
    const uint32_t mid = lo + (hi - lo) / 2;
    if (a.seg_off[mid] <= p0) lo = mid;
    else hi = mid;
  }
  uint32_t u = lo, u_end = a.seg_off[u + 1];
  const T* __restrict__ base = reinterpret_cast<const T*>(a.w) + lane * VEC;
  bool mine = false, loaded = false;
  float r[VEC];
  for (uint32_t p = (uint32_t)p0; p < p1; ++p) {
    while (p >= u_end) {  // next key (empty segments are skipped)
      if (u + 1 >= a.U) return;  // seg_off does not reach N: a malformed index form must not run off the arrays
      ++u;
      u_end = a.seg_off[u + 1];
      loaded = false;
    }
    if (!loaded) {
      const uint64_t key = a.keys[u];
      mine = (uint32_t)(key >> 32) == a.table && (key & 0xFFFFFFFFull) < a.rows;
      if (mine) {
        uint32_t row = (uint32_t)key;
        if (a.where) {
          const int32_t slot = a.where[row];
          row = slot >= 0 ? (uint32_t)slot : 0u;
        }
        Raw16<T> raw;
        raw.load(base + (size_t)row * D);
#pragma unroll
        for (int e = 0; e < VEC; ++e) r[e] = 0.f;
        raw.add_to(r);
      }
      loaded = true;
    }
    if (mine) {
      const uint32_t bag = a.seg_bags[p];
      if (bag >= a.n_bags) continue;  // malformed input: no such bag
      const uint32_t b = bag / a.S, s = bag - b * a.S;
      float* out = a.pooled + (size_t)b * a.width + a.slot_col[s] + lane * VEC;
#pragma unroll
      for (int e = 0; e < VEC; ++e) unsafeAtomicAdd(out + e, r[e]);
    }
  }
}

template <typename T, int D>
hipError_t launch_ip(const IndexedArgs& a, hipStream_t stream) {
  constexpr int LANES = D / (16 / (int)sizeof(T));
  constexpr int GPB = kBlock / LANES;
  const uint64_t tiles = ((uint64_t)a.N + kTile - 1) / kTile;
  hipLaunchKernelGGL((k_indexed_pool<T, D>), dim3((uint32_t)((tiles + GPB - 1) / GPB)), dim3(kBlock), 0, stream, a);
  return hipGetLastError();
}
template <typename T>
hipError_t dispatch_ip(uint32_t dim, const IndexedArgs& a, hipStream_t stream) {
  switch (dim) {
    case 8: return launch_ip<T, 8>(a, stream);
    case 16: return launch_ip<T, 16>(a, stream);
    case 32: return launch_ip<T, 32>(a, stream);
    case 64: return launch_ip<T, 64>(a, stream);
    case 128: return launch_ip<T, 128>(a, stream);
    default: return hipErrorInvalidValue;
  }
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

hipError_t launch_indexed_pool(const TableView& t, uint32_t table, const SlotArrays& sl, const uint64_t* keys,
                               const uint32_t* seg_off, const uint32_t* seg_bags, uint32_t U, uint32_t N, uint32_t B,
                               uint32_t S, uint32_t width, float* pooled, hipStream_t stream) {
  if (N == 0 || U == 0 || t.n_slots == 0) return hipSuccess;
  IndexedArgs a;
  a.keys = keys;
  a.seg_off = seg_off;
  a.seg_bags = seg_bags;
  a.U = U;
  a.N = N;
  a.w = t.w;
  a.where = t.where;
  a.table = table;
  a.rows = t.rows;
  a.slot_col = sl.col;
  a.S = S;
  a.width = width;
  a.n_bags = B * S;
  a.pooled = pooled;
  return t.dtype == 1 ? dispatch_ip<bf16_t>(t.dim, a, stream) : dispatch_ip<float>(t.dim, a, stream);
}

hipError_t launch_gather_pool(const TableView& t, const SlotArrays& sl, const uint64_t* ids, const int32_t* offsets,
                              uint32_t B, uint32_t S, uint32_t width, int mix, const void* zeros, float* pooled,
                              hipStream_t stream) {
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
  a.mix = mix;
  a.stream_out = t.n_slots == S ? 1 : 0;
  a.pooled = pooled;
  return t.dtype == 1 ? dispatch_dim<bf16_t>(t.dim, a, stream) : dispatch_dim<float>(t.dim, a, stream);
}

hipError_t launch_build_keys(const SlotArrays& sl, const uint64_t* ids, const int32_t* offsets, uint32_t B,
                             uint32_t S, int mix, int bare_rows, uint32_t* keys_out, uint32_t* bags_out,
                             hipStream_t stream) {
  const uint32_t n_bags = B * S;
  if (n_bags == 0) return hipSuccess;
  const uint32_t grid = (n_bags + kBlock / 8 - 1) / (kBlock / 8);
  hipLaunchKernelGGL(k_build_keys, dim3(grid), dim3(kBlock), 0, stream, sl, ids, offsets, n_bags, S, mix, bare_rows,
                     keys_out, bags_out);
  return hipGetLastError();
}

}  // namespace pemb
