// Backward after the dedup: segmented reduction of the upstream gradient over the sorted
// occurrences, fused with the row-wise optimizer update.
//
// The sorted occurrence list is cut into fixed tiles of kTile entries, one lane-group per tile
// (each lane owns 4 of the row's D elements), so work per group is constant however skewed the
// key frequencies are.  A group walks its tile in order, summing d_pooled rows of the bags it
// meets; when the key changes, the finished run is a whole segment unless it touches a tile edge:
//   - a run that began before the tile is stored as a partial in slot first[tile];
//   - otherwise a run that continues past the tile is stored in slot last[tile];
//   - every other run is a complete segment and the optimizer is applied to its row at once.
// Segments that span tiles are listed by the unique kernels and finished by the fix-up kernels, which add
// last[t0], first[t0+1], ..., first[t1] in a fixed order and then apply the optimizer.  No float
// atomics: the summation order is a function of the batch alone, so results are reproducible.
//
// Arithmetic: the gradient sums, the partial sums and the optimizer are fp64, and every stored quantity (row
// element, accumulator) is rounded once from the fp64 result -- the definition of the update evaluated to
// within fp64 rounding, whatever the length of a segment or the cancellation inside it.  These kernels move
// bytes; fp64 adds run at the rate of fp32 adds here and the conversions are hidden behind the loads.
#include "device_utils.h"
#include "launch.h"

namespace pemb {
namespace {

// Row update by a group of LG lanes; lane owns elements [4*lane, 4*lane+4) and G holds its part of
// the row's gradient; v = the lane's part of the row, a_old = the row's accumulator (both may have
// been fetched long before).  OPT 0: SGD.  OPT 1: row-wise Adagrad (mean of G^2 over the row feeds
// one accumulator; eps outside the square root).
// A table row is touched once per update.  When a row fills whole cache lines (>= 128 bytes) it is read and
// written with the streaming hint, so that it does not displace the gradient rows the kernel re-reads; smaller
// rows share their lines with neighbours that other lane-groups touch, and there the hint was measured to cost
// (16..64-byte rows of the mixed-width configuration: 7.7 -> 8.7 ms), so they take the ordinary path.
template <typename T, int D>
struct RowIo {
  static constexpr bool kStream = D * sizeof(T) >= 128;
  static __device__ __forceinline__ float4 load(const T* p) {
    if constexpr (kStream) return load_frag4_stream(p);
    else return load_frag4(p);
  }
  static __device__ __forceinline__ void store(T* p, const d4& v) {  // fp64 results, rounded once to T
    if constexpr (kStream) store_round4_stream(p, v);
    else store_round4(p, v);
  }
  static __device__ __forceinline__ float load_acc(const float* p) {
    if constexpr (kStream) return __builtin_nontemporal_load(p);
    else return *p;
  }
  static __device__ __forceinline__ void store_acc(float* p, float a) {
    if constexpr (kStream) __builtin_nontemporal_store(a, p);
    else *p = a;
  }
};

template <typename T, int D, int OPT>
__device__ __forceinline__ void finish_update(T* __restrict__ w, float* __restrict__ accs, uint32_t row, const d4& G,
                                              float4 v, float a_old, int lane, float lr, float eps) {
  constexpr int LG = D / 4;
  T* p = w + (size_t)row * D + lane * 4;
  double step;
  if constexpr (OPT == 0) {
    step = (double)lr;
  } else {
    double sq = G.x * G.x + G.y * G.y + G.z * G.z + G.w * G.w;
#pragma unroll
    for (int m = LG / 2; m >= 1; m >>= 1) sq += __shfl_xor(sq, m);
    const double a = (double)a_old + sq * (1.0 / D);
    step = (double)lr / (sqrt(a) + (double)eps);
    if (lane == 0) RowIo<T, D>::store_acc(accs + row, (float)a);
  }
  d4 o;
  o.x = fma(-step, G.x, (double)v.x);
  o.y = fma(-step, G.y, (double)v.y);
  o.z = fma(-step, G.z, (double)v.z);
  o.w = fma(-step, G.w, (double)v.w);
  RowIo<T, D>::store(p, o);
}

template <typename T, int D, int OPT>
__device__ __forceinline__ void apply_update(T* __restrict__ w, float* __restrict__ accs, uint32_t row, const d4& G,
                                             int lane, float lr, float eps) {
  const float4 v = RowIo<T, D>::load(w + (size_t)row * D + lane * 4);
  const float a_old = OPT == 0 ? 0.f : RowIo<T, D>::load_acc(accs + row);
  finish_update<T, D, OPT>(w, accs, row, G, v, a_old, lane, lr, eps);
}

struct TileArgs {
  const uint32_t* keys;
  const uint32_t* bags;
  uint32_t n;
  const float* d_pooled;
  int position;           // 1: the payload is the gradient's position in d_pooled in units of 4 floats (several
                          // tables); 0: it is the bag index, and the gradient of bag g is at g * D (one table)
  double* partials;
  uint32_t pstride;
  const uint32_t* range;
  const uint32_t* tile_perm;
  void* w;
  float* accs;
  uint32_t key_base;
  float lr, eps;
  const uint32_t* bad_flag;  // see BackwardArgs
  uint32_t call;
};

template <int D>
__device__ __forceinline__ const float* grad_ptr(const TileArgs& a, uint32_t payload, int lane) {
  return a.d_pooled + (size_t)payload * (a.position ? 4 : D) + lane * 4;
}

template <typename T, int D, int OPT>
__global__ __launch_bounds__(kBlock) void k_tile_reduce_update(TileArgs a) {
  constexpr int LG = D / 4;          // lanes per tile
  constexpr int GPB = kBlock / LG;   // tiles per workgroup
  // entries fetched together: SC gradient rows + the table rows of the runs they start.  More keep more requests in
  // flight per wave, fewer leave registers for more waves per SIMD.  Measured (reduce + update, ms): fp32 D = 64
  // (config 2) 0.717 with four against 0.725 with two; bf16 D = 64 (config 4) 1.034 with four, 0.965 with two, 1.012
  // with one; the bf16 tables of config 3 per launch (us) with 1 / 2 / 4 / 8 entries: D = 128: 2537 / 2586 / 2747 / -,
  // D = 64: 1494 / 1536 / 1633 / -, D = 32: - / 969 / 978 / -, D = 16: - / 799 / 776 / -, D = 8 (whose LDS tiles allow
  // two waves per SIMD whatever the register count): - / 877 / 820 / 828.
  constexpr int SC = sizeof(T) == 4 ? 4 : (D <= 16 ? 4 : D == 128 ? 1 : 2);
  static_assert(kTile % SC == 0, "sub-chunk geometry");
  if (*a.bad_flag == a.call) return;  // inconsistent offsets: keys and bags cannot be trusted as addresses (uniform exit)
  __shared__ uint32_t s_key[GPB][kTile];
  __shared__ uint32_t s_bag[GPB][kTile];
  const int grp = threadIdx.x / LG, lane = threadIdx.x % LG;
  const uint32_t slot_idx = blockIdx.x * GPB + grp;  // position in the processing order
  const uint32_t n_tiles = (a.n + kTile - 1) / kTile;
  const uint32_t tile = slot_idx < n_tiles ? (a.tile_perm ? a.tile_perm[slot_idx] : slot_idx) : n_tiles;
  const uint64_t p0_64 = (uint64_t)tile * kTile;
  bool in_list = p0_64 < a.n;
  uint32_t p0 = in_list ? (uint32_t)p0_64 : 0u;
  uint32_t p1 = in_list ? ((a.n - p0 < kTile) ? a.n : p0 + kTile) : 0u;
  uint32_t q0 = p0, q1 = p1;
  if (a.range) {  // several tables: only this table's stretch of the sorted list
    const uint32_t rb = a.range[0], re = a.range[1];
    q0 = q0 > rb ? q0 : rb;
    q1 = q1 < re ? q1 : re;
    if (q0 >= q1) in_list = false, p0 = p1 = 0u;  // nothing of this table in the tile: stage nothing
  }
  const uint32_t* __restrict__ keys = a.keys;
  const uint32_t* __restrict__ bags = a.bags;

  // stage the tile's (key, bag) pairs in LDS with coalesced loads
  for (uint32_t e = lane; e < kTile; e += LG) {
    const bool ok = p0 + e < p1;
    s_key[grp][e] = ok ? keys[p0 + e] : 0u;
    s_bag[grp][e] = ok ? bags[p0 + e] : 0u;
  }
  __syncthreads();
  if (!in_list) return;
  T* w = reinterpret_cast<T*>(a.w);
  const uint32_t* sk = s_key[grp];
  const uint32_t* sb = s_bag[grp];

  const bool cont_in = (q0 == p0) && p0 > 0 && keys[p0 - 1] == sk[0];
  const bool cont_out = (q1 == p1) && p1 < a.n && keys[p1] == sk[p1 - 1 - p0];
  const uint32_t last_key = sk[q1 - 1 - p0];

  // the run being summed: its key, sum, and (fetched when the run started) its table row + accumulator
  uint32_t cur = sk[q0 - p0];
  uint32_t prev = cont_in ? cur : ~cur;   // key before entry q0: equal = the first run came in from the left
  d4 acc = d4_zero();
  float4 cur_row = make_float4(0.f, 0.f, 0.f, 0.f);
  float cur_a = 0.f;
  bool first = true, have_run = cont_in;

  for (uint32_t i = q0; i < q1; i += SC) {
    uint32_t k[SC];
    float4 g[SC], wr[SC];
    float av[SC];
    bool start[SC];
#pragma unroll
    for (int j = 0; j < SC; ++j) {
      const bool ok = i + j < q1;
      k[j] = ok ? sk[i + j - p0] : prev;
      const uint32_t bag = ok ? sb[i + j - p0] : 0u;
      start[j] = ok && k[j] != (j == 0 ? prev : k[j - 1]);
      g[j] = ok ? load_frag4(grad_ptr<D>(a, bag, lane)) : make_float4(0.f, 0.f, 0.f, 0.f);
      // a run that starts here and ends inside the tile is updated by this group: fetch its row now
      const bool need_row = start[j] && !(cont_out && k[j] == last_key);
      const uint32_t row = k[j] - a.key_base;
      wr[j] = need_row ? RowIo<T, D>::load(w + (size_t)row * D + lane * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
      av[j] = (need_row && OPT != 0) ? RowIo<T, D>::load_acc(a.accs + row) : 0.f;
    }
    prev = k[SC - 1];
#pragma unroll
    for (int j = 0; j < SC; ++j) {
      if (i + j < q1) {
        if (start[j]) {
          if (have_run) {  // the run of `cur` ended inside the tile
            if (first && cont_in)
              store_d4(a.partials + (size_t)(2 * tile) * a.pstride + lane * 4, acc);
            else
              finish_update<T, D, OPT>(w, a.accs, cur - a.key_base, acc, cur_row, cur_a, lane, a.lr, a.eps);
            first = false;
          }
          have_run = true;
          cur = k[j];
          cur_row = wr[j];
          cur_a = av[j];
          acc = d4_zero();
        }
        d4_add(acc, g[j]);
      }
    }
  }
  if (first && cont_in)
    store_d4(a.partials + (size_t)(2 * tile) * a.pstride + lane * 4, acc);
  else if (cont_out)
    store_d4(a.partials + (size_t)(2 * tile + 1) * a.pstride + lane * 4, acc);
  else
    finish_update<T, D, OPT>(w, a.accs, cur - a.key_base, acc, cur_row, cur_a, lane, a.lr, a.eps);
}

struct FixupArgs {
  const uint32_t* unique_keys;
  const uint32_t* seg_off;
  const uint32_t* counters;   // [1] = entries of multi_list, [2] = entries of long_list
  const uint32_t* multi_list;
  const uint32_t* long_list;
  const double* partials;
  uint32_t pstride;
  void* w;
  float* accs;
  uint32_t key_base;
  uint64_t rows;
  float lr, eps;
  const uint32_t* bad_flag;
  uint32_t call;
};

// Segments that span at most kShortSpan tiles: one lane-group per listed segment (grid-stride), the
// partials added in tile order.
constexpr uint32_t kShortSpan = 16;

template <typename T, int D, int OPT>
__global__ __launch_bounds__(kBlock) void k_fixup_short(FixupArgs a) {
  constexpr int LG = D / 4;
  constexpr int GPB = kBlock / LG;
  const int lane = threadIdx.x % LG;
  if (*a.bad_flag == a.call) return;
  const uint32_t count = a.counters[1];
  T* w = reinterpret_cast<T*>(a.w);
  for (uint32_t e = blockIdx.x * GPB + threadIdx.x / LG; e < count; e += gridDim.x * GPB) {
    const uint32_t u = a.multi_list[e];
    const uint32_t key = a.unique_keys[u];
    if (key < a.key_base || (uint64_t)(key - a.key_base) >= a.rows) continue;  // another table's row
    const uint32_t s = a.seg_off[u], end = a.seg_off[u + 1];
    const uint32_t t0 = s / kTile, t1 = (end - 1) / kTile;
    const uint32_t np = t1 - t0 + 1;
    if (np > kShortSpan) continue;  // left to k_fixup_long
    const uint32_t row = key - a.key_base;
    const float4 v = RowIo<T, D>::load(w + (size_t)row * D + lane * 4);  // in flight together with the partials
    const float a_old = OPT == 0 ? 0.f : RowIo<T, D>::load_acc(a.accs + row);
    d4 acc = d4_zero();
    for (uint32_t k0 = 0; k0 < np; k0 += 4) {
      d4 pv[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t k = k0 + j;
        const size_t slot = (k == 0) ? (size_t)2 * t0 + 1 : (size_t)2 * (t0 + k);
        pv[j] = k < np ? load_d4(a.partials + slot * a.pstride + lane * 4) : d4_zero();
      }
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (k0 + j < np) d4_add(acc, pv[j]);
    }
    finish_update<T, D, OPT>(w, a.accs, row, acc, v, a_old, lane, a.lr, a.eps);
  }
}

// Thread per multi-tile segment: those spanning more than kShortSpan tiles go to long_list (one
// atomic per wave; the list's order varies from run to run, what is computed per entry does not).
__global__ __launch_bounds__(kBlock) void k_classify_multi(const uint32_t* __restrict__ seg_off,
                                                           const uint32_t* __restrict__ multi_list,
                                                           uint32_t* __restrict__ counters,
                                                           uint32_t* __restrict__ long_list) {
  const uint32_t count = counters[1];
  const int lane = threadIdx.x & (kWave - 1);
  // grid-stride; every wave runs the same number of rounds for all its lanes (the ballot needs them all)
  for (uint32_t e0 = blockIdx.x * kBlock; e0 < count; e0 += gridDim.x * kBlock) {
    const uint32_t e = e0 + threadIdx.x;
    bool is_long = false;
    uint32_t u = 0;
    if (e < count) {
      u = multi_list[e];
      const uint32_t s = seg_off[u], end = seg_off[u + 1];
      is_long = (end - 1) / kTile - s / kTile + 1 > kShortSpan;
    }
    const uint64_t m = __ballot(is_long);
    if (m != 0) {
      const int leader = __ffsll((unsigned long long)m) - 1;
      uint32_t base = 0;
      if (lane == leader) base = atomicAdd(&counters[2], (uint32_t)__popcll(m));
      base = __shfl(base, leader);
      if (is_long) long_list[base + (uint32_t)__popcll(m & ((1ull << lane) - 1ull))] = u;
    }
  }
}

// Longer segments (hot keys): one workgroup per entry of long_list (grid-stride).  Group g adds partials
// g, g+NG, ... of the segment in order; the NG group sums are then added in group order and the row is updated.
template <typename T, int D, int OPT>
__global__ __launch_bounds__(kBlock) void k_fixup_long(FixupArgs a) {
  constexpr int LG = D / 4;
  constexpr int NG = kBlock / LG;
  __shared__ double s_part[NG][D];
  const int g = threadIdx.x / LG, lane = threadIdx.x % LG;
  if (*a.bad_flag == a.call) return;
  const uint32_t count = a.counters[2];
  T* w = reinterpret_cast<T*>(a.w);
  for (uint32_t e = blockIdx.x; e < count; e += gridDim.x) {  // every branch below is uniform over the workgroup
    const uint32_t u = a.long_list[e];
    const uint32_t key = a.unique_keys[u];
    if (key < a.key_base || (uint64_t)(key - a.key_base) >= a.rows) continue;  // another table's row
    const uint32_t s = a.seg_off[u], end = a.seg_off[u + 1];
    const uint32_t t0 = s / kTile, t1 = (end - 1) / kTile;
    const uint32_t np = t1 - t0 + 1;
    d4 acc = d4_zero();
    for (uint32_t k0 = g; k0 < np; k0 += 4 * NG) {  // four loads in flight per lane
      d4 v[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t k = k0 + j * NG;
        const size_t slot = (k == 0) ? (size_t)2 * t0 + 1 : (size_t)2 * (t0 + k);
        v[j] = k < np ? load_d4(a.partials + slot * a.pstride + lane * 4) : d4_zero();
      }
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (k0 + j * NG < np) d4_add(acc, v[j]);
    }
    store_d4(&s_part[g][lane * 4], acc);
    __syncthreads();
    if (g == 0) {
      d4 tot = d4_zero();
      const int ng = np < (uint32_t)NG ? (int)np : NG;
      for (int gg = 0; gg < ng; ++gg) d4_add(tot, load_d4(&s_part[gg][lane * 4]));
      apply_update<T, D, OPT>(w, a.accs, key - a.key_base, tot, lane, a.lr, a.eps);
    }
    __syncthreads();
  }
}

// tile_key[t] = (table of the tile's first key) << 8 | bucket << 1 | mixed, tile_val[t] = t.  A tile that lies
// inside one key's segment (first key = last key) is put in bucket (first bag of the tile) >> (shift + 1), at
// most 127; a tile with several keys ("mixed": runs end inside it, the optimizer is applied many times) has no
// bag order to follow and is put in bucket t * 128 / n_tiles.  In every bucket the single-key tiles run first,
// then the mixed ones: the four tiles a wave holds are then mostly of one kind (the waves of single-key tiles
// never execute the optimizer's instructions), while over time the launch keeps its blend of gradient reads
// (single-key tiles) and table-row traffic (mixed tiles).
__global__ __launch_bounds__(kBlock) void k_tile_keys(const uint32_t* __restrict__ keys,
                                                      const uint32_t* __restrict__ bags, uint32_t n, uint32_t n_tiles,
                                                      int shift, const uint32_t* __restrict__ key_base,
                                                      uint32_t num_tables, uint32_t* __restrict__ tile_key,
                                                      uint32_t* __restrict__ tile_val) {
  const uint32_t t = blockIdx.x * kBlock + threadIdx.x;
  if (t >= n_tiles) return;
  const size_t p0 = (size_t)t * kTile;
  const size_t p1 = p0 + kTile < n ? p0 + kTile : n;
  const uint32_t k = keys[p0];
  uint32_t table = 0;
  if (num_tables > 1)
    while (table + 1 < num_tables && k >= key_base[table + 1]) ++table;
  const bool mixed = keys[p1 - 1] != k;
  uint32_t bucket = mixed ? (uint32_t)(((uint64_t)t * 128u) / n_tiles) : bags[p0] >> (shift + 1);
  if (bucket > 127u) bucket = 127u;
  tile_key[t] = (table << 8) | (bucket << 1) | (mixed ? 1u : 0u);
  tile_val[t] = t;
}

// Thread t <= num_tables: ranges[t] = first position whose key >= key_base[t] (ranges[num_tables] = n).
__global__ void k_table_ranges(const uint32_t* __restrict__ keys, uint32_t n, const uint32_t* __restrict__ key_base,
                               uint32_t num_tables, uint32_t* __restrict__ ranges) {
  const uint32_t t = threadIdx.x;
  if (t > num_tables) return;
  if (t == num_tables) {
    ranges[t] = n;
    return;
  }
  const uint32_t kb = key_base[t];
  uint32_t lo = 0, hi = n;
  while (lo < hi) {
    const uint32_t mid = lo + (hi - lo) / 2;
    if (keys[mid] < kb) lo = mid + 1;
    else hi = mid;
  }
  ranges[t] = lo;
}

template <typename T, int D>
hipError_t launch_tile_td(const TileArgs& a, int opt, hipStream_t stream) {
  constexpr int GPB = kBlock / (D / 4);
  const uint32_t tiles = (a.n + kTile - 1) / kTile;
  const uint32_t grid = (tiles + GPB - 1) / GPB;
  if (opt == 0)
    hipLaunchKernelGGL((k_tile_reduce_update<T, D, 0>), dim3(grid), dim3(kBlock), 0, stream, a);
  else
    hipLaunchKernelGGL((k_tile_reduce_update<T, D, 1>), dim3(grid), dim3(kBlock), 0, stream, a);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_fixup_td(const FixupArgs& a, int opt, uint32_t tiles, hipStream_t stream) {
  constexpr int GPB = kBlock / (D / 4);
  // multi-tile segments <= tiles; both kernels stride over the list, so the grids only need to fill the chip
  const uint32_t want_s = (tiles + GPB - 1) / GPB;
  const uint32_t grid_s = want_s < 4096u ? want_s : 4096u;
  const uint32_t grid_l = tiles < 2048u ? tiles : 2048u;
  if (opt == 0) {
    hipLaunchKernelGGL((k_fixup_short<T, D, 0>), dim3(grid_s), dim3(kBlock), 0, stream, a);
    hipLaunchKernelGGL((k_fixup_long<T, D, 0>), dim3(grid_l), dim3(kBlock), 0, stream, a);
  } else {
    hipLaunchKernelGGL((k_fixup_short<T, D, 1>), dim3(grid_s), dim3(kBlock), 0, stream, a);
    hipLaunchKernelGGL((k_fixup_long<T, D, 1>), dim3(grid_l), dim3(kBlock), 0, stream, a);
  }
  return hipGetLastError();
}

#define PEMB_DIM_SWITCH(T, dim, FN, ...)             \
  switch (dim) {                                     \
    case 8: return FN<T, 8>(__VA_ARGS__);            \
    case 16: return FN<T, 16>(__VA_ARGS__);          \
    case 32: return FN<T, 32>(__VA_ARGS__);          \
    case 64: return FN<T, 64>(__VA_ARGS__);          \
    case 128: return FN<T, 128>(__VA_ARGS__);        \
    default: return hipErrorInvalidValue;            \
  }

}  // namespace

hipError_t launch_table_ranges(const uint32_t* keys, uint32_t n, const uint32_t* key_base_dev, uint32_t num_tables,
                               uint32_t* ranges, hipStream_t stream) {
  if (num_tables + 1 > 1024) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_table_ranges, dim3(1), dim3(num_tables + 1), 0, stream, keys, n, key_base_dev, num_tables,
                     ranges);
  return hipGetLastError();
}

hipError_t launch_tile_order(const uint32_t* keys, const uint32_t* bags, uint32_t n, int shift,
                             const uint32_t* key_base_dev, uint32_t num_tables, uint32_t* const tile_key[2],
                             uint32_t* const tile_val[2], uint32_t* hist, uint32_t* total,
                             const uint32_t** perm_out, hipStream_t stream) {
  const uint32_t n_tiles = (n + kTile - 1) / kTile;
  *perm_out = nullptr;
  if (n_tiles < 2) return hipSuccess;  // nothing to order
  hipLaunchKernelGGL(k_tile_keys, dim3((n_tiles + kBlock - 1) / kBlock), dim3(kBlock), 0, stream, keys, bags, n, n_tiles,
                     shift, key_base_dev, num_tables, tile_key[0], tile_val[0]);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  int table_bits = 0;
  while ((1u << table_bits) < num_tables) ++table_bits;
  const SortPlan plan = make_sort_plan(n_tiles, 8 + table_bits, 8);  // one pass for a single table
  int src = 0;
  for (int pass = 0; pass < plan.passes; ++pass) {
    const int sh = pass * plan.bits;
    if ((e = launch_radix_hist(plan, sh, tile_key[src], hist, stream)) != hipSuccess) return e;
    if ((e = launch_radix_scan(plan, hist, total, stream)) != hipSuccess) return e;
    if ((e = launch_radix_scatter(plan, sh, tile_key[src], tile_val[src], tile_key[src ^ 1], tile_val[src ^ 1], hist,
                                  total, stream)) != hipSuccess)
      return e;
    src ^= 1;
  }
  *perm_out = tile_val[src];
  return hipSuccess;
}

hipError_t launch_tile_reduce_update(const TableView& t, const BackwardArgs& b, hipStream_t stream) {
  if (b.n == 0) return hipSuccess;
  TileArgs a;
  a.keys = b.keys;
  a.bags = b.bags;
  a.n = b.n;
  a.d_pooled = b.d_pooled;
  a.position = b.payload_is_position;
  a.partials = b.partials;
  a.pstride = b.pstride;
  a.range = b.range;
  a.tile_perm = b.tile_perm;
  a.w = t.w;
  a.accs = t.acc;
  a.key_base = t.key_base;
  a.lr = b.lr;
  a.eps = b.eps;
  a.bad_flag = b.bad_flag;
  a.call = b.call;
  if (!a.bad_flag) return hipErrorInvalidValue;
  if (t.dtype == 1) {
    PEMB_DIM_SWITCH(bf16_t, t.dim, launch_tile_td, a, b.opt, stream)
  } else {
    PEMB_DIM_SWITCH(float, t.dim, launch_tile_td, a, b.opt, stream)
  }
}

hipError_t launch_classify_multi(const BackwardArgs& b, uint32_t* counters, uint32_t* long_list, hipStream_t stream) {
  if (b.n == 0) return hipSuccess;
  const uint32_t tiles = (b.n + kTile - 1) / kTile;  // multi-tile segments <= tiles; the kernel strides over the list
  const uint32_t want = (tiles + kBlock - 1) / kBlock;
  hipLaunchKernelGGL(k_classify_multi, dim3(want < 512u ? want : 512u), dim3(kBlock), 0, stream, b.seg_off,
                     b.multi_list, counters, long_list);
  return hipGetLastError();
}

hipError_t launch_fixup(const TableView& t, const BackwardArgs& b, hipStream_t stream) {
  if (b.n == 0) return hipSuccess;
  FixupArgs a;
  a.unique_keys = b.unique_keys;
  a.seg_off = b.seg_off;
  a.counters = b.counters;
  a.multi_list = b.multi_list;
  a.long_list = b.long_list;
  a.partials = b.partials;
  a.pstride = b.pstride;
  a.w = t.w;
  a.accs = t.acc;
  a.key_base = t.key_base;
  a.rows = t.rows;
  a.lr = b.lr;
  a.eps = b.eps;
  a.bad_flag = b.bad_flag;
  a.call = b.call;
  if (!a.bad_flag) return hipErrorInvalidValue;
  const uint32_t tiles = (b.n + kTile - 1) / kTile;
  if (t.dtype == 1) {
    PEMB_DIM_SWITCH(bf16_t, t.dim, launch_fixup_td, a, b.opt, tiles, stream)
  } else {
    PEMB_DIM_SWITCH(float, t.dim, launch_fixup_td, a, b.opt, tiles, stream)
  }
}

}  // namespace pemb
