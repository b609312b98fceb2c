// Dedup of the batch: stable LSD radix sort of (key, bag) pairs and run-length "unique".
//
// One radix pass = three kernels.  hist: every block counts the digits of its contiguous chunk.
// scan: one block per digit turns that digit's per-block counts into exclusive prefixes and
// emits the digit total.  scatter: every block walks its chunk in tiles of kSortTile pairs; inside a
// tile each wave ranks its keys with ballot-based digit matching (stable: rank = number of
// earlier pairs of the tile with the same digit), the tile is reordered digit-major through LDS,
// and written out so that consecutive lanes store to consecutive addresses of a digit's region.
// Only the significant key bits are sorted, in passes of equal width of at most kSortMaxBits bits.
#include "device_utils.h"
#include "launch.h"

namespace pemb {
namespace {

constexpr int kItems = 8;  // keys per thread of a unique-kernel tile
static_assert(kUniqueTile == kBlock * kItems, "tile geometry");
constexpr int kSortItems = kSortTile / kBlock;  // pairs per thread of a scatter tile
static_assert(kSortTile == kBlock * kSortItems, "tile geometry");

constexpr int kHistThreads = 1024;  // the histogram is latency-bound: more waves per chunk than the scatter uses

// Counts the digits of four consecutive keys.  After the first passes the many occurrences of a hot key
// sit next to each other, and 64 lanes adding to one LDS counter serialise; so equal digits are merged
// first: inside the lane's four keys, and -- when every lane of the wave holds four keys of one and the
// same digit -- across the wave, where a single lane adds 256.
template <int BITS>
__device__ __forceinline__ void count4(uint32_t* h, uint4 a, int shift, int lane) {
  constexpr uint32_t M = (1u << BITS) - 1u;
  const uint32_t d0 = (a.x >> shift) & M, d1 = (a.y >> shift) & M, d2 = (a.z >> shift) & M, d3 = (a.w >> shift) & M;
  const bool same4 = d0 == d1 && d1 == d2 && d2 == d3;
  const uint32_t first = __builtin_amdgcn_readfirstlane(d0);
  if (__all(same4 && d0 == first)) {  // whole wave, one digit (partial waves never get here with inactive lanes)
    if (lane == 0) atomicAdd(&h[first], 4u * kWave);
    return;
  }
  if (same4) {
    atomicAdd(&h[d0], 4u);
    return;
  }
  uint32_t c = 1;  // run-length merge of the four digits
  if (d1 == d0) ++c; else { atomicAdd(&h[d0], c); c = 1; }
  if (d2 == d1) ++c; else { atomicAdd(&h[d1], c); c = 1; }
  if (d3 == d2) ++c; else { atomicAdd(&h[d2], c); c = 1; }
  atomicAdd(&h[d3], c);
}

template <int BITS>
__global__ __launch_bounds__(kHistThreads) void k_radix_hist(const uint32_t* __restrict__ keys, uint32_t n,
                                                             uint32_t chunk, int shift, uint32_t nblk,
                                                             uint32_t* __restrict__ hist) {
  constexpr int NB = 1 << BITS;
  constexpr uint32_t TH = kHistThreads;
  __shared__ uint32_t h[NB];
  const int lane = threadIdx.x & (kWave - 1);
  for (int i = threadIdx.x; i < NB; i += TH) h[i] = 0;
  __syncthreads();
  const uint32_t beg = blockIdx.x * chunk;
  const uint32_t end = (n - beg < chunk) ? n : beg + chunk;  // beg < n by construction of the plan
  // beg is a multiple of the tile size and the buffer is 256-byte aligned: 16-byte loads.
  const uint32_t nvec = (end - beg) / 4;
  const uint32_t nvec_full = nvec / kWave * kWave;  // vectors that whole waves take (count4 needs all 64 lanes)
  const uint4* __restrict__ kv = reinterpret_cast<const uint4*>(keys + beg);
  uint32_t v = threadIdx.x;
  for (; v + TH < nvec_full; v += 2 * TH) {  // both loads in flight before the counting
    const uint4 a = kv[v], b = kv[v + TH];
    count4<BITS>(h, a, shift, lane);
    count4<BITS>(h, b, shift, lane);
  }
  for (; v < nvec_full; v += TH) count4<BITS>(h, kv[v], shift, lane);
  // ragged rest: fewer than 64 vectors, then fewer than 4 keys
  for (uint32_t i = beg + nvec_full * 4 + threadIdx.x; i < end; i += TH)
    atomicAdd(&h[(keys[i] >> shift) & (NB - 1)], 1u);
  __syncthreads();
  for (int d = threadIdx.x; d < NB; d += TH) hist[(size_t)d * nblk + blockIdx.x] = h[d];
}

// Block d: exclusive scan of hist[d*nblk .. (d+1)*nblk) in place, total[d] = sum.
__global__ __launch_bounds__(kBlock) void k_radix_scan(uint32_t* __restrict__ hist, uint32_t nblk,
                                                       uint32_t* __restrict__ total) {
  __shared__ uint32_t s_w[kWavesPerBlock];
  uint32_t* row = hist + (size_t)blockIdx.x * nblk;
  const uint32_t per = (nblk + kBlock - 1) / kBlock;
  const uint32_t b0 = threadIdx.x * per;
  uint32_t sum = 0;
  for (uint32_t j = 0; j < per; ++j)
    if (b0 + j < nblk) sum += row[b0 + j];
  uint32_t tot;
  uint32_t run = block_exclusive_scan(sum, s_w, &tot);
  for (uint32_t j = 0; j < per; ++j)
    if (b0 + j < nblk) {
      uint32_t v = row[b0 + j];
      row[b0 + j] = run;
      run += v;
    }
  if (threadIdx.x == 0) total[blockIdx.x] = tot;
}

template <int BITS, bool STREAM>
__global__ __launch_bounds__(kBlock) void k_radix_scatter(const uint32_t* __restrict__ kin,
                                                          const uint32_t* __restrict__ pin,
                                                          uint32_t* __restrict__ kout, uint32_t* __restrict__ pout,
                                                          uint32_t n, uint32_t chunk, int shift, uint32_t nblk,
                                                          const uint32_t* __restrict__ hist,
                                                          const uint32_t* __restrict__ total) {
  constexpr int NB = 1 << BITS;
  constexpr int DPT = NB > kBlock ? NB / kBlock : 1;  // digits owned by a thread: tid*DPT .. tid*DPT + DPT-1
  static_assert(NB <= kBlock || NB % kBlock == 0, "digit ownership");
  __shared__ uint32_t s_key[kSortTile];
  __shared__ uint32_t s_pay[kSortTile];
  __shared__ uint32_t s_cnt[kWavesPerBlock][NB];
  __shared__ uint32_t s_gofs[NB];
  __shared__ uint32_t s_w[kWavesPerBlock];

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const bool owner = tid * DPT < NB;

  // Where this block's first pair of each owned digit goes: pairs of smaller digits anywhere, plus
  // pairs of the same digit in earlier blocks.
  uint32_t running[DPT];
  {
    uint32_t v[DPT], sum = 0;
#pragma unroll
    for (int q = 0; q < DPT; ++q) {
      v[q] = owner ? total[tid * DPT + q] : 0u;
      sum += v[q];
    }
    uint32_t ex = block_exclusive_scan(sum, s_w, nullptr);
#pragma unroll
    for (int q = 0; q < DPT; ++q) {
      running[q] = owner ? ex + hist[(size_t)(tid * DPT + q) * nblk + blockIdx.x] : 0u;
      ex += v[q];
    }
  }

  const uint32_t beg = blockIdx.x * chunk;
  const uint32_t end = (n - beg < chunk) ? n : beg + chunk;

  for (uint32_t tile_base = beg; tile_base < end; tile_base += kSortTile) {
    const uint32_t tile_cnt = (end - tile_base < kSortTile) ? end - tile_base : kSortTile;
    for (int i = tid; i < kWavesPerBlock * NB; i += kBlock) (&s_cnt[0][0])[i] = 0;
    __syncthreads();

    uint32_t key[kSortItems], pay[kSortItems], lrank[kSortItems];
#pragma unroll
    for (int k = 0; k < kSortItems; ++k) {
      const uint32_t off = wave * (kWave * kSortItems) + k * kWave + lane;  // position inside the tile
      const bool valid = off < tile_cnt;
      if constexpr (STREAM) {  // pairs that do not fit the memory-side cache anyway: do not displace anything for them
        key[k] = valid ? __builtin_nontemporal_load(kin + tile_base + off) : 0xFFFFFFFFu;
        pay[k] = valid ? __builtin_nontemporal_load(pin + tile_base + off) : 0u;
      } else {
        key[k] = valid ? kin[tile_base + off] : 0xFFFFFFFFu;
        pay[k] = valid ? pin[tile_base + off] : 0u;
      }
    }
#pragma unroll
    for (int k = 0; k < kSortItems; ++k) {
      const uint32_t off = wave * (kWave * kSortItems) + k * kWave + lane;
      const bool valid = off < tile_cnt;
      const uint32_t d = (key[k] >> shift) & (NB - 1);
      // peers: the valid lanes of this wave whose key has the same digit (includes this lane), kept as two 32-bit
      // halves.  Per bit: all-ones or zero from the lane's own bit, one ballot, and peers &= ~(ballot ^ own), which
      // is the ballot where the own bit is set and its complement where it is not.
      const uint64_t vmask = __ballot(valid);
      uint32_t plo = (uint32_t)vmask, phi = (uint32_t)(vmask >> 32);
#pragma unroll
      for (int b = 0; b < BITS; ++b) {
        const uint32_t own = 0u - ((d >> b) & 1u);
        const uint64_t bt = __ballot(own != 0u);
        plo &= ~((uint32_t)bt ^ own);
        phi &= ~((uint32_t)(bt >> 32) ^ own);
      }
      lrank[k] = 0;
      if (valid) {
        const int leader = plo ? __ffs((int)plo) - 1 : 32 + __ffs((int)phi) - 1;
        uint32_t old = 0;
        if (lane == leader) old = atomicAdd(&s_cnt[wave][d], (uint32_t)(__popc(plo) + __popc(phi)));
        old = __shfl(old, leader);
        // peers below this lane: mbcnt counts the bits of a mask that belong to lower lanes
        lrank[k] = old + __builtin_amdgcn_mbcnt_hi(phi, __builtin_amdgcn_mbcnt_lo(plo, 0u));
      }
    }
    __syncthreads();

    // Digit-major layout of the tile: digit start, then waves in order.
    uint32_t c[DPT][kWavesPerBlock], tot[DPT], sum = 0;
#pragma unroll
    for (int q = 0; q < DPT; ++q) {
      tot[q] = 0;
#pragma unroll
      for (int w = 0; w < kWavesPerBlock; ++w) {
        c[q][w] = owner ? s_cnt[w][tid * DPT + q] : 0u;
        tot[q] += c[q][w];
      }
      sum += tot[q];
    }
    uint32_t ex = block_exclusive_scan(sum, s_w, nullptr);
    if (owner) {
#pragma unroll
      for (int q = 0; q < DPT; ++q) {
        uint32_t run = ex;
#pragma unroll
        for (int w = 0; w < kWavesPerBlock; ++w) {
          s_cnt[w][tid * DPT + q] = run;
          run += c[q][w];
        }
        s_gofs[tid * DPT + q] = running[q] - ex;  // global index = s_gofs[digit] + position in the reordered tile
        running[q] += tot[q];
        ex += tot[q];
      }
    }
    __syncthreads();

#pragma unroll
    for (int k = 0; k < kSortItems; ++k) {
      const uint32_t off = wave * (kWave * kSortItems) + k * kWave + lane;
      if (off < tile_cnt) {
        const uint32_t d = (key[k] >> shift) & (NB - 1);
        const uint32_t pos = s_cnt[wave][d] + lrank[k];
        s_key[pos] = key[k];
        s_pay[pos] = pay[k];
      }
    }
    __syncthreads();

    for (uint32_t j = tid; j < tile_cnt; j += kBlock) {
      const uint32_t kk = s_key[j];
      const uint32_t g = s_gofs[(kk >> shift) & (NB - 1)] + j;
      kout[g] = kk;
      pout[g] = s_pay[j];
    }
    __syncthreads();
  }
}

// ---- unique: heads of runs in the sorted keys, and the list of runs that cross a tile edge ----
// Thread t of a block owns the 8 consecutive positions base + 8t .. base + 8t + 7.
__device__ __forceinline__ uint32_t head_flags(const uint32_t* __restrict__ keys, uint32_t n, uint32_t i0,
                                               uint32_t (&k)[kItems]) {
  uint32_t flags = 0;
  if (i0 >= n) return 0;
  uint32_t prev = i0 ? keys[i0 - 1] : 0u;
  if (i0 + kItems <= n) {
    const uint4 a = *reinterpret_cast<const uint4*>(keys + i0);
    const uint4 b = *reinterpret_cast<const uint4*>(keys + i0 + 4);
    k[0] = a.x; k[1] = a.y; k[2] = a.z; k[3] = a.w; k[4] = b.x; k[5] = b.y; k[6] = b.z; k[7] = b.w;
  } else {
#pragma unroll
    for (int j = 0; j < kItems; ++j) k[j] = (i0 + j < n) ? keys[i0 + j] : 0u;
  }
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    if (i0 + j < n && (i0 + j == 0 || k[j] != prev)) flags |= 1u << j;
    prev = k[j];
  }
  return flags;
}

// End to assume for the last run of a block's stretch [.., blk_end): if the run goes on in the next
// block it crosses the tile edge at blk_end (the stretch ends on one), which "blk_end + 1" expresses;
// otherwise it ends where the stretch (or the list) ends.
__device__ __forceinline__ uint32_t stretch_limit(const uint32_t* __restrict__ keys, uint32_t n, uint32_t blk_end) {
  if (blk_end >= n) return n;
  return keys[blk_end] == keys[blk_end - 1] ? blk_end + 1 : blk_end;
}

// Shared by the count and the write kernel.  Returns, for this thread's heads, a bit mask of the
// ones whose run crosses an edge between tiles of kTile positions.  first_local = index, among the
// block's heads, of this thread's first head; n_heads = heads in the block; limit = stretch_limit().
__device__ __forceinline__ uint32_t multi_flags(uint32_t flags, uint32_t i0, uint32_t first_local, uint32_t n_heads,
                                                uint32_t limit, uint32_t* s_heads) {
  uint32_t h = first_local;
#pragma unroll
  for (int j = 0; j < kItems; ++j)
    if (flags & (1u << j)) s_heads[h++] = i0 + j;
  __syncthreads();
  uint32_t multi = 0;
  h = first_local;
#pragma unroll
  for (int j = 0; j < kItems; ++j)
    if (flags & (1u << j)) {
      const uint32_t s = i0 + j;
      const uint32_t e = (h + 1 < n_heads) ? s_heads[h + 1] : limit;  // end of the run, or a lower bound past an edge
      if (s / kTile != (e - 1) / kTile) multi |= 1u << j;
      ++h;
    }
  return multi;
}

__global__ __launch_bounds__(kBlock) void k_unique_count(const uint32_t* __restrict__ keys, uint32_t n,
                                                         uint32_t* __restrict__ blk_heads,
                                                         uint32_t* __restrict__ blk_multi) {
  __shared__ uint32_t s_w[kWavesPerBlock];
  __shared__ uint32_t s_heads[kUniqueTile];
  uint32_t k[kItems];
  const uint32_t i0 = blockIdx.x * kUniqueTile + threadIdx.x * kItems;
  const uint32_t blk_end = (blockIdx.x + 1) * kUniqueTile;
  const uint32_t limit = stretch_limit(keys, n, blk_end);
  const uint32_t flags = head_flags(keys, n, i0, k);
  uint32_t n_heads;
  const uint32_t first_local = block_exclusive_scan(__popc(flags), s_w, &n_heads);
  const uint32_t multi = multi_flags(flags, i0, first_local, n_heads, limit, s_heads);
  uint32_t n_multi;
  block_exclusive_scan(__popc(multi), s_w, &n_multi);
  if (threadIdx.x == 0) {
    blk_heads[blockIdx.x] = n_heads;
    blk_multi[blockIdx.x] = n_multi;
  }
}

// Single block of 1024 threads: exclusive scans of blk_heads[nb] and blk_multi[nb] in place;
// counters[0] = U, counters[1] = number of multi-tile runs, counters[2] = 0; seg_off[U] = n.
// The arrays are walked in chunks of 4096 entries, four consecutive entries per thread (one 16-byte access, so a
// wave reads whole cache lines); per chunk one block-wide scan of the threads' sums, carried into the next chunk.
constexpr int kScanThreads = 1024;

__global__ __launch_bounds__(kScanThreads) void k_unique_scan(uint32_t* __restrict__ blk_heads,
                                                              uint32_t* __restrict__ blk_multi, uint32_t nb,
                                                              uint32_t n, uint32_t* __restrict__ counters,
                                                              uint32_t* __restrict__ seg_off) {
  constexpr int NW = kScanThreads / kWave;
  __shared__ uint32_t s_h[NW], s_m[NW];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  uint32_t carry_h = 0, carry_m = 0;
  for (uint32_t base = 0; base < nb; base += 4 * kScanThreads) {  // the loop bounds are the same for every thread
    const uint32_t i0 = base + 4 * threadIdx.x;
    uint32_t h[4] = {0, 0, 0, 0}, m[4] = {0, 0, 0, 0};
    if (i0 + 4 <= nb) {
      const uint4 a = *reinterpret_cast<const uint4*>(blk_heads + i0), c = *reinterpret_cast<const uint4*>(blk_multi + i0);
      h[0] = a.x; h[1] = a.y; h[2] = a.z; h[3] = a.w;
      m[0] = c.x; m[1] = c.y; m[2] = c.z; m[3] = c.w;
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (i0 + j < nb) {
          h[j] = blk_heads[i0 + j];
          m[j] = blk_multi[i0 + j];
        }
    }
    const uint32_t sum_h = h[0] + h[1] + h[2] + h[3], sum_m = m[0] + m[1] + m[2] + m[3];
    uint32_t inc_h = sum_h, inc_m = sum_m;  // inclusive scans inside the wave
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const uint32_t th = __shfl_up(inc_h, off), tm = __shfl_up(inc_m, off);
      if (lane >= off) {
        inc_h += th;
        inc_m += tm;
      }
    }
    if (lane == kWave - 1) {
      s_h[wave] = inc_h;
      s_m[wave] = inc_m;
    }
    __syncthreads();
    uint32_t run_h = carry_h + inc_h - sum_h, run_m = carry_m + inc_m - sum_m, tot_h = 0, tot_m = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const uint32_t xh = s_h[w], xm = s_m[w];
      if (w < wave) {
        run_h += xh;
        run_m += xm;
      }
      tot_h += xh;
      tot_m += xm;
    }
    __syncthreads();  // s_h / s_m are rewritten by the next chunk
    carry_h += tot_h;
    carry_m += tot_m;
    uint32_t oh[4], om[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      oh[j] = run_h;
      om[j] = run_m;
      run_h += h[j];
      run_m += m[j];
    }
    if (i0 + 4 <= nb) {
      *reinterpret_cast<uint4*>(blk_heads + i0) = make_uint4(oh[0], oh[1], oh[2], oh[3]);
      *reinterpret_cast<uint4*>(blk_multi + i0) = make_uint4(om[0], om[1], om[2], om[3]);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (i0 + j < nb) {
          blk_heads[i0 + j] = oh[j];
          blk_multi[i0 + j] = om[j];
        }
    }
  }
  if (threadIdx.x == 0) {
    counters[0] = carry_h;
    counters[1] = carry_m;
    counters[2] = 0;
    seg_off[carry_h] = n;
  }
}

__global__ __launch_bounds__(kBlock) void k_unique_write(const uint32_t* __restrict__ keys, uint32_t n,
                                                         const uint32_t* __restrict__ blk_heads,
                                                         const uint32_t* __restrict__ blk_multi,
                                                         uint32_t* __restrict__ unique_keys,
                                                         uint32_t* __restrict__ seg_off,
                                                         uint32_t* __restrict__ multi_list) {
  __shared__ uint32_t s_w[kWavesPerBlock];
  __shared__ uint32_t s_heads[kUniqueTile];
  uint32_t k[kItems];
  const uint32_t i0 = blockIdx.x * kUniqueTile + threadIdx.x * kItems;
  const uint32_t blk_end = (blockIdx.x + 1) * kUniqueTile;
  const uint32_t limit = stretch_limit(keys, n, blk_end);
  const uint32_t flags = head_flags(keys, n, i0, k);
  uint32_t n_heads;
  const uint32_t first_local = block_exclusive_scan(__popc(flags), s_w, &n_heads);
  const uint32_t multi = multi_flags(flags, i0, first_local, n_heads, limit, s_heads);
  uint32_t m = blk_multi[blockIdx.x] + block_exclusive_scan(__popc(multi), s_w, nullptr);
  uint32_t u = blk_heads[blockIdx.x] + first_local;
#pragma unroll
  for (int j = 0; j < kItems; ++j)
    if (flags & (1u << j)) {
      unique_keys[u] = k[j];
      seg_off[u] = i0 + j;
      if (multi & (1u << j)) multi_list[m++] = u;
      ++u;
    }
}

template <int BITS>
hipError_t pass_hist(const SortPlan& p, int shift, const uint32_t* keys, uint32_t* hist, hipStream_t stream) {
  hipLaunchKernelGGL(k_radix_hist<BITS>, dim3(p.nblk), dim3(kHistThreads), 0, stream, keys, p.n, p.chunk, shift,
                     p.nblk, hist);
  return hipGetLastError();
}
template <int BITS>
hipError_t pass_scatter(const SortPlan& p, int shift, const uint32_t* kin, const uint32_t* pin, uint32_t* kout,
                        uint32_t* pout, const uint32_t* hist, const uint32_t* total, hipStream_t stream) {
  // the (key, payload) arrays of one pass: 8 bytes per pair; beyond half the 256 MB memory-side cache the next
  // pass cannot find them there, and streaming loads were measured faster (config 4: 0.596 -> 0.559 ms), below
  // it slower (config 2: 0.256 -> 0.265 ms)
  if ((uint64_t)p.n * 8 > (128ull << 20))
    hipLaunchKernelGGL((k_radix_scatter<BITS, true>), dim3(p.nblk), dim3(kBlock), 0, stream, kin, pin, kout, pout, p.n,
                       p.chunk, shift, p.nblk, hist, total);
  else
    hipLaunchKernelGGL((k_radix_scatter<BITS, false>), dim3(p.nblk), dim3(kBlock), 0, stream, kin, pin, kout, pout, p.n,
                       p.chunk, shift, p.nblk, hist, total);
  return hipGetLastError();
}

}  // namespace

SortPlan make_sort_plan(uint32_t n, int key_bits, int max_bits) {
  SortPlan p;
  p.n = n;
  if (key_bits < 1) key_bits = 1;
  if (max_bits < 4) max_bits = 4;
  if (max_bits > kSortMaxBits) max_bits = kSortMaxBits;
  p.passes = (key_bits + max_bits - 1) / max_bits;
  p.bits = (key_bits + p.passes - 1) / p.passes;
  uint32_t tiles = (n + kSortTile - 1) / kSortTile;
  if (tiles == 0) tiles = 1;
  uint32_t target = tiles < kSortMaxBlocks ? tiles : kSortMaxBlocks;
  uint32_t tiles_per_blk = (tiles + target - 1) / target;
  p.chunk = tiles_per_blk * kSortTile;
  p.nblk = (tiles + tiles_per_blk - 1) / tiles_per_blk;  // every block starts below n
  return p;
}

#define PEMB_BITS_SWITCH(bits, CALL) \
  switch (bits) {                    \
    case 1: return CALL(1);          \
    case 2: return CALL(2);          \
    case 3: return CALL(3);          \
    case 4: return CALL(4);          \
    case 5: return CALL(5);          \
    case 6: return CALL(6);          \
    case 7: return CALL(7);          \
    case 8: return CALL(8);          \
    case 9: return CALL(9);          \
    default: return hipErrorInvalidValue; \
  }

hipError_t launch_radix_hist(const SortPlan& p, int shift, const uint32_t* keys, uint32_t* hist, hipStream_t stream) {
#define CALL(B) pass_hist<B>(p, shift, keys, hist, stream)
  PEMB_BITS_SWITCH(p.bits, CALL)
#undef CALL
}

hipError_t launch_radix_scan(const SortPlan& p, uint32_t* hist, uint32_t* total, hipStream_t stream) {
  hipLaunchKernelGGL(k_radix_scan, dim3(1u << p.bits), dim3(kBlock), 0, stream, hist, p.nblk, total);
  return hipGetLastError();
}

hipError_t launch_radix_scatter(const SortPlan& p, int shift, const uint32_t* kin, const uint32_t* pin,
                                uint32_t* kout, uint32_t* pout, const uint32_t* hist, const uint32_t* total,
                                hipStream_t stream) {
#define CALL(B) pass_scatter<B>(p, shift, kin, pin, kout, pout, hist, total, stream)
  PEMB_BITS_SWITCH(p.bits, CALL)
#undef CALL
}

hipError_t launch_unique(const uint32_t* keys, uint32_t n, uint32_t* blk_heads, uint32_t* blk_multi,
                         uint32_t* unique_keys, uint32_t* seg_off, uint32_t* multi_list, uint32_t* counters,
                         hipStream_t stream) {
  const uint32_t nb = (n + kUniqueTile - 1) / kUniqueTile;  // 0 when n == 0
  if (nb) {
    hipLaunchKernelGGL(k_unique_count, dim3(nb), dim3(kBlock), 0, stream, keys, n, blk_heads, blk_multi);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(k_unique_scan, dim3(1), dim3(kScanThreads), 0, stream, blk_heads, blk_multi, nb, n, counters,
                     seg_off);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (nb) {
    hipLaunchKernelGGL(k_unique_write, dim3(nb), dim3(kBlock), 0, stream, keys, n, blk_heads, blk_multi, unique_keys,
                       seg_off, multi_list);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace pemb
