// Lossy value codec for pooled activations and their gradients: per block of `block_len` fp32
// values, scale by kappa / ||v||_inf and store as fp16; the inverse converts back and divides by
// the same factor.  Pure bandwidth kernels: 4 bytes in, 2 bytes out per value (and back).
#include <hip/hip_fp16.h>

#include "device_utils.h"
#include "launch.h"

namespace pemb {
namespace {

// A group of `lpb` adjacent lanes (a power of two, <= 64) owns one block; a lane owns every lpb-th
// 16-byte quad of it.  The first four quads of a lane stay in registers between the norm pass and
// the conversion pass; longer blocks are read a second time (from cache).
__global__ __launch_bounds__(kBlock) void k_codec_compress(const float* __restrict__ v, uint64_t n_blocks,
                                                           uint32_t block_len, int lpb, float kappa,
                                                           __half* __restrict__ q, float* __restrict__ norm) {
  const uint32_t groups_per_wg = kBlock / lpb;
  const uint64_t blk = (uint64_t)blockIdx.x * groups_per_wg + threadIdx.x / lpb;
  const int lane = threadIdx.x % lpb;
  if (blk >= n_blocks) return;  // whole groups leave together
  const uint32_t quads = block_len / 4;
  const float4* __restrict__ src = reinterpret_cast<const float4*>(v + blk * block_len);
  float4 keep[4];
  float m = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint32_t i = lane + j * lpb;
    keep[j] = i < quads ? src[i] : make_float4(0.f, 0.f, 0.f, 0.f);
    m = fmaxf(m, fmaxf(fmaxf(fabsf(keep[j].x), fabsf(keep[j].y)), fmaxf(fabsf(keep[j].z), fabsf(keep[j].w))));
  }
  for (uint32_t i = lane + 4 * lpb; i < quads; i += lpb) {
    const float4 t = src[i];
    m = fmaxf(m, fmaxf(fmaxf(fabsf(t.x), fabsf(t.y)), fmaxf(fabsf(t.z), fabsf(t.w))));
  }
  for (int s = lpb / 2; s >= 1; s >>= 1) m = fmaxf(m, __shfl_xor(m, s));
  const float factor = m > 0.f ? kappa / m : 0.f;
  if (lane == 0) norm[blk] = m;
  uint2* __restrict__ dst = reinterpret_cast<uint2*>(q + blk * block_len);
  auto pack = [factor](float4 t) {
    const __half2 lo = __floats2half2_rn(t.x * factor, t.y * factor);
    const __half2 hi = __floats2half2_rn(t.z * factor, t.w * factor);
    uint2 o;
    o.x = *reinterpret_cast<const uint32_t*>(&lo);
    o.y = *reinterpret_cast<const uint32_t*>(&hi);
    return o;
  };
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint32_t i = lane + j * lpb;
    if (i < quads) dst[i] = pack(keep[j]);
  }
  for (uint32_t i = lane + 4 * lpb; i < quads; i += lpb) dst[i] = pack(src[i]);
}

// Thread per quad of values.
__global__ __launch_bounds__(kBlock) void k_codec_decompress(const __half* __restrict__ q,
                                                             const float* __restrict__ norm, uint64_t n_quads,
                                                             uint32_t quads_per_block, float kappa,
                                                             float* __restrict__ out) {
  const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= n_quads) return;
  const float m = norm[i / quads_per_block];
  const uint2 raw = reinterpret_cast<const uint2*>(q)[i];
  float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
  if (m > 0.f) {
    const float factor = kappa / m;
    const float2 lo = __half22float2(*reinterpret_cast<const __half2*>(&raw.x));
    const float2 hi = __half22float2(*reinterpret_cast<const __half2*>(&raw.y));
    r = make_float4(lo.x / factor, lo.y / factor, hi.x / factor, hi.y / factor);
  }
  reinterpret_cast<float4*>(out)[i] = r;
}

}  // namespace

hipError_t launch_codec_compress(const float* v, uint64_t n_blocks, uint32_t block_len, float kappa, void* q_fp16,
                                 float* norm, hipStream_t stream) {
  if (n_blocks == 0) return hipSuccess;
  int lpb = 1;
  while (lpb < 64 && (uint32_t)lpb * 4u < block_len) lpb <<= 1;
  const uint32_t groups_per_wg = kBlock / lpb;
  const uint64_t grid = (n_blocks + groups_per_wg - 1) / groups_per_wg;
  if (grid > 0x7FFFFFFFull) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_codec_compress, dim3((uint32_t)grid), dim3(kBlock), 0, stream, v, n_blocks, block_len, lpb, kappa,
                     reinterpret_cast<__half*>(q_fp16), norm);
  return hipGetLastError();
}

hipError_t launch_codec_decompress(const void* q_fp16, const float* norm, uint64_t n_blocks, uint32_t block_len,
                                   float kappa, float* out, hipStream_t stream) {
  if (n_blocks == 0) return hipSuccess;
  const uint64_t n_quads = n_blocks * (block_len / 4);
  const uint64_t grid = (n_quads + kBlock - 1) / kBlock;
  if (grid > 0x7FFFFFFFull) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_codec_decompress, dim3((uint32_t)grid), dim3(kBlock), 0, stream,
                     reinterpret_cast<const __half*>(q_fp16), norm, n_quads, block_len / 4, kappa, out);
  return hipGetLastError();
}

}  // namespace pemb
