// Measurement aid, not part of the path: what the memory system of this GPU delivers to the barest possible
// kernel with the path's access pattern -- random reads of whole rows -- so that the gather and the segmented
// reduction can be judged against something measured on the same box instead of a datasheet figure.
#include <hip/hip_runtime.h>

#include "../../include/persia_emb.h"
#include "device_utils.h"

using namespace pemb;

namespace {

// A group of LANES lanes (16 bytes each) reads `reads_per_group` rows, UNROLL of them in flight; row numbers come
// from the bijective mixer of the hash applied to a counter.  hot_of_8 of every 8 reads fall into the first
// hot_rows rows (a stand-in for the frequent keys of a skewed batch), the others anywhere in [0, rows).
template <int LANES>
__global__ __launch_bounds__(kBlock) void k_probe_rows(const char* __restrict__ base, uint64_t rows, uint64_t hot_rows,
                                                       uint32_t hot_of_8, uint32_t reads_per_group, uint64_t n_groups,
                                                       uint4* __restrict__ sink) {
  constexpr int UNROLL = 8;
  const uint64_t gid = ((uint64_t)blockIdx.x * kBlock + threadIdx.x) / LANES;
  const int lane = threadIdx.x % LANES;
  if (gid >= n_groups) return;
  uint4 acc = make_uint4(0u, 0u, 0u, 0u);
  const uint64_t ctr = gid * 0x9E3779B97F4A7C15ull;
  for (uint32_t it = 0; it < reads_per_group; it += UNROLL) {
    uint4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const uint64_t h = mix64(ctr + it + u);
      const uint64_t r = ((uint32_t)u < hot_of_8) ? h % hot_rows : h % rows;
      v[u] = *reinterpret_cast<const uint4*>(base + r * (uint64_t)(LANES * 16) + lane * 16);
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      acc.x ^= v[u].x;
      acc.y ^= v[u].y;
      acc.z ^= v[u].z;
      acc.w ^= v[u].w;
    }
  }
  // the rows are only read; one value that depends on all of them is kept so that the loads cannot be dropped
  if (gid == 0 && lane == 0) *sink = acc;
}

}  // namespace

extern "C" int emb_probe_random_rows(const void* base, uint64_t rows, uint32_t row_bytes, uint64_t n_reads, uint64_t hot_rows,
                                     uint32_t hot_of_8, void* sink16, void* hip_stream) {
  if (!base || !sink16 || rows == 0 || hot_of_8 > 8 || (hot_of_8 && (hot_rows == 0 || hot_rows > rows))) return EMB_EINVAL;
  if (row_bytes < 16 || row_bytes > 512 || (row_bytes & (row_bytes - 1))) return EMB_EINVAL;
  if (n_reads == 0) return EMB_OK;
  const uint32_t lanes = row_bytes / 16;
  const uint32_t reads_per_group = 64;                       // a multiple of the 8 reads in flight
  const uint64_t n_groups = (n_reads + reads_per_group - 1) / reads_per_group;
  const uint64_t blocks = (n_groups * lanes + kBlock - 1) / kBlock;
  if (blocks > 0x7FFFFFFFull) return EMB_EINVAL;
  hipStream_t stream = (hipStream_t)hip_stream;
  const char* b = static_cast<const char*>(base);
  uint4* s = static_cast<uint4*>(sink16);
  if (hot_rows == 0) hot_rows = 1;
#define PEMB_PROBE(L)                                                                                            \
  case L:                                                                                                        \
    hipLaunchKernelGGL(k_probe_rows<L>, dim3((uint32_t)blocks), dim3(kBlock), 0, stream, b, rows, hot_rows, hot_of_8, \
                       reads_per_group, n_groups, s);                                                            \
    break;
  switch (lanes) {
    PEMB_PROBE(1) PEMB_PROBE(2) PEMB_PROBE(4) PEMB_PROBE(8) PEMB_PROBE(16) PEMB_PROBE(32)
    default: return EMB_EINVAL;
  }
#undef PEMB_PROBE
  return hipGetLastError() == hipSuccess ? EMB_OK : EMB_EDEVICE;
}
