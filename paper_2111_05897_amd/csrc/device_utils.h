// Device-side helpers shared by the kernels of the embedding library (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pemb {

constexpr int kWave = 64;
constexpr int kBlock = 256;                 // every kernel here runs 256-thread workgroups (4 waves)
constexpr int kWavesPerBlock = kBlock / kWave;

typedef uint16_t bf16_t;                    // raw bf16 storage

// 64-bit bijective mixer of the hash (definition in include/persia_emb.h).
__host__ __device__ __forceinline__ uint64_t mix64(uint64_t z) {
  z ^= z >> 31;
  z *= 0x9FB21C651E98DF25ull;
  z ^= z >> 29;
  z *= 0xC2B2AE3D27D4EB4Full;
  z ^= z >> 32;
  return z;
}

// ID -> row.  mask = rows-1 when rows is a power of two (then mod is an AND), else 0.
__device__ __forceinline__ uint32_t hash_row(uint64_t id, uint64_t salt, uint64_t rows, uint64_t mask, int mix) {
  uint64_t z = mix ? mix64(id + salt) : id;
  return (uint32_t)(mask ? (z & mask) : (z % rows));
}

__device__ __forceinline__ float bf16_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// fp32 -> bf16, round to nearest even; NaN stays a quiet NaN.
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x0040u;
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

// Initial value of one table element (definition in include/persia_emb.h): separate multiply and add.
__device__ __forceinline__ float init_value(uint64_t table_key, uint64_t elem, float scale, float mid) {
#pragma clang fp contract(off)  // two roundings: the product must not fuse into the add
  uint64_t h = mix64(table_key + elem);
  int k = (int)(h >> 40) - (1 << 23);
  float prod = (float)k * scale;
  return prod + mid;
}

// Compensated add: sum += x with the rounding error of every add carried in comp.
__device__ __forceinline__ void kahan_add(float& sum, float& comp, float x) {
#pragma clang fp contract(off)
  const float y = x - comp;
  const float t = sum + y;
  comp = (t - sum) - y;
  sum = t;
}

// ---- fp64 results -> storage.  Sums and the optimizer are evaluated in fp64 and every stored quantity is
// rounded once: to fp32 by the conversion instruction, to bf16 through "round to odd" -- the fp64 value is
// truncated to fp32 and the last fp32 bit is set when anything was cut off; that sticky bit sits 16 places below the
// bf16 rounding point, so the nearest-even rounding of the fp32 pattern to bf16 sees exactly on which side of a tie
// the fp64 value lay, and the result is the one a direct fp64 -> bf16 rounding gives.
__device__ __forceinline__ uint32_t f64_to_bf16(double v) {
  const float f = __double2float_rz(v);
  uint32_t u = __float_as_uint(f);
  if ((double)f != v) u |= 1u;  // inexact (also true of a NaN, which stays a NaN)
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x0040u;
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

// 4 consecutive row elements in fp64: what one lane of the backward kernels accumulates.
struct d4 {
  double x, y, z, w;
};
__device__ __forceinline__ d4 d4_zero() { return d4{0.0, 0.0, 0.0, 0.0}; }
__device__ __forceinline__ void d4_add(d4& a, float4 g) {
  a.x += (double)g.x;
  a.y += (double)g.y;
  a.z += (double)g.z;
  a.w += (double)g.w;
}
__device__ __forceinline__ void d4_add(d4& a, const d4& b) {
  a.x += b.x;
  a.y += b.y;
  a.z += b.z;
  a.w += b.w;
}
__device__ __forceinline__ d4 load_d4(const double* p) {
  const double2 a = *reinterpret_cast<const double2*>(p), b = *reinterpret_cast<const double2*>(p + 2);
  return d4{a.x, a.y, b.x, b.y};
}
__device__ __forceinline__ void store_d4(double* p, const d4& v) {
  *reinterpret_cast<double2*>(p) = make_double2(v.x, v.y);
  *reinterpret_cast<double2*>(p + 2) = make_double2(v.z, v.w);
}

// ---- 4-element row fragments (what one lane owns of a row in the backward kernels) ----
__device__ __forceinline__ float4 load_frag4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ float4 load_frag4(const bf16_t* p) {
  uint2 v = *reinterpret_cast<const uint2*>(p);
  return make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xFFFF0000u), __uint_as_float(v.y << 16),
                     __uint_as_float(v.y & 0xFFFF0000u));
}
__device__ __forceinline__ void store_frag4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
__device__ __forceinline__ void store_frag4(bf16_t* p, float4 v) {
  uint2 o;
  o.x = f32_to_bf16(v.x) | (f32_to_bf16(v.y) << 16);
  o.y = f32_to_bf16(v.z) | (f32_to_bf16(v.w) << 16);
  *reinterpret_cast<uint2*>(p) = o;
}
// fp64 results, each rounded once to the storage type
__device__ __forceinline__ void store_round4(float* p, const d4& v) {
  *reinterpret_cast<float4*>(p) = make_float4((float)v.x, (float)v.y, (float)v.z, (float)v.w);
}
__device__ __forceinline__ void store_round4(bf16_t* p, const d4& v) {
  uint2 o;
  o.x = f64_to_bf16(v.x) | (f64_to_bf16(v.y) << 16);
  o.y = f64_to_bf16(v.z) | (f64_to_bf16(v.w) << 16);
  *reinterpret_cast<uint2*>(p) = o;
}

// The same with the streaming hint: for data a kernel touches once (a table row being updated), so that it
// does not displace what the kernel re-reads (gradient rows) from the caches.
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float4 load_frag4_stream(const float* p) {
  const f32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p));
  return make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ float4 load_frag4_stream(const bf16_t* p) {
  const u32x2_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t*>(p));
  return make_float4(__uint_as_float(v[0] << 16), __uint_as_float(v[0] & 0xFFFF0000u), __uint_as_float(v[1] << 16),
                     __uint_as_float(v[1] & 0xFFFF0000u));
}
__device__ __forceinline__ void store_round4_stream(float* p, const d4& v) {
  const f32x4_t o = {(float)v.x, (float)v.y, (float)v.z, (float)v.w};
  __builtin_nontemporal_store(o, reinterpret_cast<f32x4_t*>(p));
}
__device__ __forceinline__ void store_round4_stream(bf16_t* p, const d4& v) {
  const u32x2_t o = {f64_to_bf16(v.x) | (f64_to_bf16(v.y) << 16), f64_to_bf16(v.z) | (f64_to_bf16(v.w) << 16)};
  __builtin_nontemporal_store(o, reinterpret_cast<u32x2_t*>(p));
}

// ---- block-wide exclusive scan over kBlock threads; s_w: shared uint32_t[kWavesPerBlock] ----
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* s_w, uint32_t* total) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  uint32_t incl = v;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    uint32_t t = __shfl_up(incl, off);
    if (lane >= off) incl += t;
  }
  if (lane == kWave - 1) s_w[wave] = incl;
  __syncthreads();
  uint32_t woff = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kWavesPerBlock; ++w) {
    uint32_t x = s_w[w];
    if (w < wave) woff += x;
    tot += x;
  }
  __syncthreads();  // s_w may be reused by the caller right away
  if (total) *total = tot;
  return woff + incl - v;
}

}  // namespace pemb
