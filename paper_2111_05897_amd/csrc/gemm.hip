// Dense contractions of the MLP step on the matrix cores: C[M,N] = A[M,K] * Bt[N,K]^T with bf16
// operands (both K-contiguous) and fp32 accumulation, plus the bf16 transpose that brings every
// operand of the step into that form.
//
// k_gemm_nt: a 512-thread workgroup computes a 256x256 tile of C; its 8 waves sit 2x4 and own 128x64
// each, i.e. 4x2 MFMA tiles of v_mfma_f32_32x32x16_bf16 (lane l feeds row/column l%32 with the 8
// consecutive k values starting at 8*(l/32)).  K is walked in steps of 64 through two LDS stages that
// global_load_lds_dwordx4 fills directly (no staging registers, whole 128-byte lines per row), one tile
// ahead of the products; rows are unpadded and XOR-swizzled against bank conflicts.  The loop over K is rotated: its
// one barrier per tile sits in front of the tile's last k-step, whose products cover what follows the barrier (the
// requests for the tile after next and the first fragment reads of the next tile).  Workgroups are numbered so that
// the ones running together on an XCD cover a compact block of tiles and share their A and Bt strips in that XCD's
// L2, and XCDs that run at the same time share strips through the memory-side cache.
#include "device_utils.h"
#include "launch.h"

#include <algorithm>
#include <type_traits>

namespace pemb {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 64;              // K elements per LDS stage
constexpr int kKUnit = 64;          // K must be a multiple of this; splits along K are counted in these units
constexpr int kStages = 2;          // ring of LDS stages: tile i is multiplied while the later ones arrive
// 512-thread workgroups: 8 waves sit 2 (M) x 4 (N); a wave owns WM x WN MFMA tiles of 32x32.
constexpr int kGemmThreads = 512;
constexpr int WM = 4, WN = 2;
constexpr int BM = 2 * 32 * WM, BN = 4 * 32 * WN;  // 256 x 256
constexpr int kRowBytes = BK * 2;                   // a staged row: chunks of 16 bytes, no padding
constexpr int kStageBytes = (BM + BN) * kRowBytes;  // one LDS stage: A tile then Bt tile
constexpr size_t kGemmLdsBytes = (size_t)kStages * kStageBytes;
constexpr uint32_t kXcds = 8;
constexpr uint32_t kBlockM = 8, kBlockN = 4;  // tiles the 32 CUs of an XCD work on together

struct GemmArgs {
  const bf16_t* A;   // [M, K], row stride lda
  const bf16_t* Bt;  // [N, K], row stride ldb
  uint32_t M, N, K, lda, ldb;
  void* C;           // [M, N], row stride ldc (fp32 or bf16 by epilogue)
  uint32_t ldc;
  const float* bias;     // [N]            (epilogue 0)
  const bf16_t* mask;    // [M, N], ldm    (epilogue 2: keep where mask > 0)
  uint32_t ldm;
  uint32_t vec_out;      // 1: C (and mask) rows can be written 16 bytes at a time
  uint32_t k_tiles_per_split;  // blockIdx.y takes this many K tiles and writes the fp32 partial product
  uint64_t part_stride;        // number blockIdx.y, part_stride elements apart (split-K, epilogue 1 only)
  bf16_t* Ct;            // optional second copy of a bf16 C, transposed: [N, M], row stride ldct (needs vec_out)
  uint32_t ldct;
};

template <int EPI>
__global__ __launch_bounds__(kGemmThreads, 2) void k_gemm_nt(GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
  const uint32_t tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  // XCD-aware numbering.  Workgroup b runs on XCD b % 8, and an XCD starts its workgroups in the order of b / 8, 32 at
  // a time (one per CU): those 32 take a block of kBlockM x kBlockN tiles, so that 8 + 4 operand strips serve 32 tiles
  // out of that XCD's L2.  The blocks are numbered along n first, and at any time the 8 XCDs hold 8 consecutive
  // blocks: XCDs that work on the same m-tiles at the same time fetch the same strips of A, and all but the first
  // find them in the memory-side cache instead of HBM (likewise the strips of Bt for XCDs on the same n-tiles).
  // A product with fewer than 8 such blocks (the ones cut along K) instead gives every XCD a contiguous stretch of a
  // raster that runs down kBlockM m-tiles at a time.
  const uint32_t nchunks = (tiles_n + kBlockN - 1) / kBlockN;
  const uint32_t nblocks = ((tiles_m + kBlockM - 1) / kBlockM) * nchunks;
  uint32_t tile_m, tile_n;
  if (nblocks >= kXcds) {
    const uint32_t local = blockIdx.x / kXcds;                     // order of this workgroup on its XCD
    const uint32_t blk = (local / (kBlockM * kBlockN)) * kXcds + blockIdx.x % kXcds;
    const uint32_t within = local % (kBlockM * kBlockN);
    if (blk >= nblocks) return;
    tile_m = (blk / nchunks) * kBlockM + within % kBlockM;
    tile_n = (blk % nchunks) * kBlockN + within / kBlockM;
    if (tile_m >= tiles_m || tile_n >= tiles_n) return;
  } else {
    const uint32_t per_xcd = gridDim.x / kXcds;
    const uint32_t lid = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    if (lid >= tiles_m * tiles_n) return;
    const uint32_t group_sz = kBlockM * tiles_n;
    const uint32_t gidx = lid / group_sz;
    const uint32_t first_m = gidx * kBlockM;
    const uint32_t rows_in_group = (tiles_m - first_m < kBlockM) ? tiles_m - first_m : kBlockM;
    const uint32_t in_group = lid - gidx * group_sz;
    tile_m = first_m + in_group % rows_in_group;
    tile_n = in_group / rows_in_group;
  }
  const uint32_t m0 = tile_m * BM, n0 = tile_n * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  floatx16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // Global -> LDS without passing through registers (global_load_lds_dwordx4): one wave instruction moves 64
  // x 16 bytes to 1 KB of consecutive LDS, i.e. RPI staged rows of CPR chunks; lane l lands on row l / CPR,
  // chunk position l % CPR.  Rows are not padded; instead chunk c of row r is kept at position
  // c ^ ((r >> SWZ_SHIFT) & (CPR - 1)), which makes the fragment reads below (32 rows, one chunk each) hit
  // every bank once.  The lane chooses the global chunk
  // that belongs at its position.  Rows past the end of A or Bt are replaced by the last valid row (their
  // products are never stored), so no load needs a predicate.
  constexpr int CPR = kRowBytes / 16;                               // 16-byte chunks per staged row
  constexpr int RPI = kWave / CPR;                                  // rows one wave instruction stages
  constexpr int SWZ_SHIFT = (256 / kRowBytes) == 4 ? 2 : 1;         // rows per 256 bytes of LDS, as a shift
  static_assert(kRowBytes == 64 || kRowBytes == 128, "swizzle geometry");
  constexpr int kGroupsA = BM / RPI, kGroupsB = BN / RPI;           // row groups per operand tile
  constexpr int kWaves = kGemmThreads / kWave;
  static_assert(kGroupsA % kWaves == 0 && kGroupsB % kWaves == 0, "whole wave instructions per stage");
  constexpr int LA = kGroupsA / kWaves, LB = kGroupsB / kWaves;     // loads per thread and stage
  const uint32_t kt0 = blockIdx.y * g.k_tiles_per_split;            // first K unit of this split
  const int uwave = __builtin_amdgcn_readfirstlane(wave);
  // position lane % CPR of row lane / CPR holds chunk pos ^ swz(row); the row groups start at multiples of RPI,
  // which only matter to swz through (g * RPI) >> SWZ_SHIFT
  auto chunk_of = [&](uint32_t row_in_tile) {
    return (uint32_t)(lane % CPR) ^ ((row_in_tile >> SWZ_SHIFT) & (uint32_t)(CPR - 1));
  };
  const char* srcA[LA];
  const char* srcB[LB];
#pragma unroll
  for (int j = 0; j < LA; ++j) {
    const uint32_t rt = (uint32_t)((j * kWaves + wave) * RPI + lane / CPR);
    const uint32_t r = min(rt, g.M - 1 - m0);
    srcA[j] = reinterpret_cast<const char*>(g.A + (size_t)(m0 + r) * g.lda + (size_t)kt0 * kKUnit + chunk_of(rt) * 8);
  }
#pragma unroll
  for (int j = 0; j < LB; ++j) {
    const uint32_t rt = (uint32_t)((j * kWaves + wave) * RPI + lane / CPR);
    const uint32_t r = min(rt, g.N - 1 - n0);
    srcB[j] = reinterpret_cast<const char*>(g.Bt + (size_t)(n0 + r) * g.ldb + (size_t)kt0 * kKUnit + chunk_of(rt) * 8);
  }
  char* lds_bytes = reinterpret_cast<char*>(lds);
  // one wave instruction of a tile's requests: numbers 0 .. LA-1 are A's, LA .. LA+LB-1 are Bt's
  auto request_one = [&](uint32_t tile, int stage, int j) {  // tile: index of the BK-wide K tile inside this split
    char* dst = lds_bytes + stage * kStageBytes;
    if (j < LA)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(srcA[j] + (size_t)tile * kRowBytes),
                                       (__attribute__((address_space(3))) void*)(dst + (j * kWaves + uwave) * 1024), 16, 0, 0);
    else
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(srcB[j - LA] + (size_t)tile * kRowBytes),
                                       (__attribute__((address_space(3))) void*)(dst + BM * kRowBytes + ((j - LA) * kWaves + uwave) * 1024), 16, 0, 0);
  };
  auto request = [&](uint32_t tile, int stage) {
#pragma unroll
    for (int j = 0; j < LA + LB; ++j) request_one(tile, stage, j);
  };
  // fragment rows are base + lane % 32 with base a multiple of 32, so swz(row) depends on the lane only
  const uint32_t swz = (uint32_t)(((lane & 31) >> SWZ_SHIFT) & (CPR - 1));
  static_assert(LA + LB <= 15, "the wait in the K loop encodes its count in four bits");
  // The K loop is rotated so that its one barrier per tile has work behind it.  Fragments are read one k-step ahead of
  // the products (two register sets).  When the products of the last-but-one k-step of tile i have been issued, the
  // stage of tile i has been read for the last time (the reads of its last k-step went out in front of those
  // products), and the wave waits for its part of tile i + 1 and meets the others at the barrier.  Behind the barrier:
  // the requests for tile i + 2 into the stage just vacated, the fragment reads of the first k-step of tile i + 1,
  // and the products of the last k-step of tile i, which cover the latency of those reads.  (With the barrier at the
  // top of a tile, all eight waves stand behind it with empty hands until the first fragments arrive from the LDS.)
  constexpr int KSTEPS = BK / 16;
  static_assert(LA + LB <= WM * WN, "one request behind every product of a k-step");
  static_assert(KSTEPS == 4 && kStages == 2, "the rotation below is written out for four k-steps and two stages");
  bf16x8 af[2][WM], bfr[2][WN];
  auto read_frags = [&](int stage, int kk, int set) {
    const char* As = lds_bytes + stage * kStageBytes;
    const char* Bs = As + BM * kRowBytes;
    const uint32_t pos = ((uint32_t)(kk * 2 + (lane >> 5)) ^ swz) * 16;
#pragma unroll
    for (int i = 0; i < WM; ++i)
      af[set][i] = *reinterpret_cast<const bf16x8*>(As + (wm * 32 * WM + i * 32 + (lane & 31)) * kRowBytes + pos);
#pragma unroll
    for (int j = 0; j < WN; ++j)
      bfr[set][j] = *reinterpret_cast<const bf16x8*>(Bs + (wn * 32 * WN + j * 32 + (lane & 31)) * kRowBytes + pos);
  };
  // products of one k-step from register set `set`; behind the first of them (whose operands are then the only LDS
  // reads outstanding, so that the wait in front of it is exact) goes `between`, the next k-step's fragment reads
  auto products = [&](int set, auto between) {
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
      for (int j = 0; j < WN; ++j) {
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[set][i], bfr[set][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        between(i * WN + j);
        __builtin_amdgcn_sched_barrier(0);
      }
  };

  // K tiles of BK inside this split
  const uint32_t nk = min(g.K / kKUnit - kt0, g.k_tiles_per_split) * (kKUnit / BK);
  // Tile 0 is awaited up front.  Past the end the last tile is requested (and its first fragments read) again, into a
  // stage nobody multiplies from any more, so that every iteration is the same.
  request(0, 0);
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
  request(min(1u, nk - 1), 1);
  read_frags(0, 0, 0);
  for (uint32_t i = 0; i < nk; ++i) {
    const int stage = (int)(i % kStages);
    products(0, [&](int m) { if (m == 0) read_frags(stage, 1, 1); });
    products(1, [&](int m) { if (m == 0) read_frags(stage, 2, 0); });
    products(0, [&](int m) { if (m == 0) read_frags(stage, 3, 1); });
    // this wave's part of tile i + 1 has landed and its reads of tile i are complete; the barrier makes both true of
    // everybody.  A bare barrier: __syncthreads() would add a fence of its own.
    __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) and lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    const uint32_t refill = min(i + 2, nk - 1);
    products(1, [&](int m) {  // the next tile's first fragments early, the requests one behind each product
      if (m == 0) read_frags(stage ^ 1, 0, 0);
      if (m < LA + LB) request_one(refill, stage, m);
    });
  }
  __syncthreads();  // the epilogue reuses the stages
  __builtin_amdgcn_s_waitcnt(0x0F70);  // the surplus requests of the last iterations must not land on the epilogue's patch
  __syncthreads();

  // epilogue: accumulator element e of lane l is C[8*(e/4) + 4*(l/32) + e%4][l%32] of its 32x32 tile
  if (g.vec_out) {
    // Each wave passes its 32-row strips (32*WN columns wide) through a private LDS patch and writes whole
    // rows, 16 bytes per lane; the K loop ended with a barrier, so the stages are free.  A wave's LDS
    // accesses complete in order, so the patch needs no workgroup barrier.
    using out_t = typename std::conditional<EPI == 1, float, bf16_t>::type;
    constexpr int PW = 32 * WN;                       // patch width in elements
    constexpr int VEC = 16 / (int)sizeof(out_t);      // elements per lane on the way out
    constexpr int PS = PW + VEC;                      // padded patch stride
    constexpr int LPR = PW / VEC, RPP = kWave / LPR;  // lanes per row, rows per pass
    out_t* patch = reinterpret_cast<out_t*>(lds) + wave * 32 * PS;
    const uint32_t cbase = n0 + wn * PW;
#pragma unroll
    for (int i = 0; i < WM; ++i) {
#pragma unroll
      for (int j = 0; j < WN; ++j) {
        const int cl = j * 32 + (lane & 31);
        float bias = 0.f;
        if constexpr (EPI == 0) bias = (cbase + cl < g.N) ? g.bias[cbase + cl] : 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int r = 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
          float v = acc[i][j][e];
          if constexpr (EPI == 0) v = fmaxf(v + bias, 0.f);
          if constexpr (EPI == 1) patch[r * PS + cl] = v;
          else patch[r * PS + cl] = (bf16_t)f32_to_bf16(v);
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int pass = 0; pass < 32 / RPP; ++pass) {
        const int r = pass * RPP + lane / LPR, c = (lane % LPR) * VEC;
        const uint32_t row = m0 + wm * 32 * WM + i * 32 + r, col = cbase + c;
        uint4 v = *reinterpret_cast<const uint4*>(&patch[r * PS + c]);
        if (row < g.M && col < g.N) {  // N is a multiple of VEC here, so the whole vector is inside
          if constexpr (EPI == 2) {    // keep where the stored activation is positive
            const uint4 mv = *reinterpret_cast<const uint4*>(g.mask + (size_t)row * g.ldm + col);
            auto keep = [](uint32_t val, uint32_t m) {
              const uint32_t lo = m & 0xFFFFu, hi = m >> 16;
              const uint32_t klo = ((lo & 0x7FFFu) != 0 && !(lo & 0x8000u)) ? 0x0000FFFFu : 0u;
              const uint32_t khi = ((hi & 0x7FFFu) != 0 && !(hi & 0x8000u)) ? 0xFFFF0000u : 0u;
              return val & (klo | khi);
            };
            v.x = keep(v.x, mv.x); v.y = keep(v.y, mv.y); v.z = keep(v.z, mv.z); v.w = keep(v.w, mv.w);
          }
          *reinterpret_cast<uint4*>(reinterpret_cast<out_t*>(g.C) + (size_t)row * g.ldc + col) = v;
        }
        if constexpr (EPI == 2) {  // the transposed copy below wants the masked values
          if (g.Ct) *reinterpret_cast<uint4*>(&patch[r * PS + c]) = v;
        }
      }
      if constexpr (EPI != 1) {
        if (g.Ct) {
          static_assert(EPI == 1 || PW == kWave, "one patch column per lane");
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
          __builtin_amdgcn_wave_barrier();
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
          const uint32_t col = cbase + lane;
#pragma unroll
          for (int p8 = 0; p8 < 4; ++p8) {  // 8 consecutive rows of column `lane` -> 16 bytes of Ct's row
            uint32_t w4[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const uint32_t lo = patch[(p8 * 8 + 2 * q) * PS + lane], hi = patch[(p8 * 8 + 2 * q + 1) * PS + lane];
              w4[q] = lo | (hi << 16);
            }
            const uint32_t row0 = m0 + wm * 32 * WM + i * 32 + p8 * 8;
            if (col < g.N && row0 < g.M)  // M is a multiple of 8 here
              *reinterpret_cast<uint4*>(g.Ct + (size_t)col * g.ldct + row0) = make_uint4(w4[0], w4[1], w4[2], w4[3]);
          }
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j) {
      const uint32_t col = n0 + wn * 32 * WN + j * 32 + (lane & 31);
      if (col >= g.N) continue;
      float bias = 0.f;
      if constexpr (EPI == 0) bias = g.bias[col];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const uint32_t row = m0 + wm * 32 * WM + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        if (row >= g.M) continue;
        float v = acc[i][j][e];
        if constexpr (EPI == 0) {  // bias + ReLU -> bf16
          v = fmaxf(v + bias, 0.f);
          reinterpret_cast<bf16_t*>(g.C)[(size_t)row * g.ldc + col] = (bf16_t)f32_to_bf16(v);
        } else if constexpr (EPI == 1) {  // fp32
          reinterpret_cast<float*>(g.C)[blockIdx.y * g.part_stride + (size_t)row * g.ldc + col] = v;
        } else {  // keep where the stored activation is positive -> bf16
          const bf16_t mv = g.mask[(size_t)row * g.ldm + col];
          const bool on = (mv & 0x7FFFu) != 0 && !(mv & 0x8000u);
          reinterpret_cast<bf16_t*>(g.C)[(size_t)row * g.ldc + col] = (bf16_t)f32_to_bf16(on ? v : 0.f);
        }
      }
    }
}

// out[c][r] = in[r][c] for bf16 matrices, 64x64 tiles through LDS.
__global__ __launch_bounds__(kBlock) void k_transpose_bf16(const bf16_t* __restrict__ in, uint32_t R, uint32_t Cc,
                                                           uint32_t ld_in, bf16_t* __restrict__ out, uint32_t ld_out) {
  __shared__ bf16_t t[64][66];
  const uint32_t r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  for (int i = threadIdx.x; i < 64 * 64; i += kBlock) {
    const uint32_t r = i / 64, c = i % 64;
    t[r][c] = (r0 + r < R && c0 + c < Cc) ? in[(size_t)(r0 + r) * ld_in + c0 + c] : (bf16_t)0;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 64 * 64; i += kBlock) {
    const uint32_t c = i / 64, r = i % 64;
    if (r0 + r < R && c0 + c < Cc) out[(size_t)(c0 + c) * ld_out + r0 + r] = t[r][c];
  }
}

template <int EPI>
hipError_t launch_epi(const GemmArgs& g, hipStream_t stream) {
  // the ring of LDS stages needs more than the 64 KB a kernel gets by default; the attribute belongs to the
  // current device, so it is set (a host-side call) before every launch rather than once per process
  const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_nt<EPI>),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)kGemmLdsBytes);
  if (attr != hipSuccess) return attr;
  const uint32_t tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  const uint32_t nblocks = ((tiles_m + kBlockM - 1) / kBlockM) * ((tiles_n + kBlockN - 1) / kBlockN);
  const uint32_t grid = nblocks >= kXcds ? (nblocks + kXcds - 1) / kXcds * kXcds * kBlockM * kBlockN  // whole blocks on every XCD
                                         : (tiles_m * tiles_n + kXcds - 1) / kXcds * kXcds;
  const uint32_t splits = (g.K / kKUnit + g.k_tiles_per_split - 1) / g.k_tiles_per_split;
  hipLaunchKernelGGL(k_gemm_nt<EPI>, dim3(grid, splits), dim3(kGemmThreads), kGemmLdsBytes, stream, g);
  return hipGetLastError();
}

// C[r][c] = sum over s of parts[s][r][c], in the order of s.
__global__ __launch_bounds__(kBlock) void k_sum_splits(const float* __restrict__ parts, uint32_t splits, uint32_t M,
                                                       uint32_t N, float* __restrict__ C, uint32_t ldc) {
  const uint64_t n = (uint64_t)M * N;
  for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (uint64_t)gridDim.x * kBlock) {
    float acc = parts[i];
    for (uint32_t sp = 1; sp < splits; ++sp) acc += parts[sp * n + i];
    C[(i / N) * ldc + i % N] = acc;
  }
}

}  // namespace

// A product with few output tiles and a long K leaves most compute units idle: such a product is cut along K
// into this many partial products (1 = no split), summed afterwards in a fixed order.
uint32_t gemm_splits(uint32_t M, uint32_t N, uint32_t K) {
  const uint32_t tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  const uint32_t nk = K / kKUnit;
  if (tiles == 0 || tiles * 2 > 256) return 1;
  uint32_t s = 256 / tiles;
  if (s > nk / 4) s = nk / 4;  // at least four K tiles per split
  if (s > 16) s = 16;
  return s < 2 ? 1 : s;
}

hipError_t launch_gemm_nt(int epilogue, const void* A, uint32_t lda, const void* Bt, uint32_t ldb, uint32_t M, uint32_t N,
                          uint32_t K, void* C, uint32_t ldc, const float* bias, const void* mask, uint32_t ldm,
                          hipStream_t stream, void* Ct, uint32_t ldct, float* split_ws, uint64_t split_ws_elems) {
  if (M == 0 || N == 0) return hipSuccess;
  if (K == 0 || K % kKUnit != 0 || lda % 8 != 0 || ldb % 8 != 0) return hipErrorInvalidValue;  // 16-byte operand loads
  if (!A || !Bt || !C || (epilogue == 0 && !bias) || (epilogue == 2 && !mask)) return hipErrorInvalidValue;
  GemmArgs g;
  g.A = reinterpret_cast<const bf16_t*>(A);
  g.Bt = reinterpret_cast<const bf16_t*>(Bt);
  g.M = M;
  g.N = N;
  g.K = K;
  g.lda = lda;
  g.ldb = ldb;
  g.C = C;
  g.ldc = ldc;
  g.bias = bias;
  g.mask = reinterpret_cast<const bf16_t*>(mask);
  g.ldm = ldm;
  auto vec16 = [](const void* p, uint32_t ld) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0 && ld % 8 == 0; };
  // fp32 output already writes 128 contiguous bytes per row from the accumulator layout
  g.vec_out = (epilogue != 1 && N % 8 == 0 && vec16(C, ldc) && (epilogue != 2 || vec16(mask, ldm))) ? 1u : 0u;
  if (Ct && epilogue == 1) return hipErrorInvalidValue;  // the transposed copy is bf16
  g.k_tiles_per_split = K / kKUnit;
  g.part_stride = 0;
  uint32_t splits = 1;
  if (epilogue == 1 && split_ws) {
    splits = gemm_splits(M, N, K);
    const uint64_t fit = split_ws_elems / ((uint64_t)M * N);
    if (splits > fit) splits = (uint32_t)fit;
    if (splits >= 2) {
      g.k_tiles_per_split = (K / kKUnit + splits - 1) / splits;
      splits = (K / kKUnit + g.k_tiles_per_split - 1) / g.k_tiles_per_split;  // no empty split
      g.C = split_ws;
      g.ldc = N;
      g.part_stride = (uint64_t)M * N;
    }
  }
  const bool fused_t = Ct && g.vec_out && M % 8 == 0 && vec16(Ct, ldct);
  g.Ct = fused_t ? reinterpret_cast<bf16_t*>(Ct) : nullptr;
  g.ldct = ldct;
  hipError_t e;
  switch (epilogue) {
    case 0: e = launch_epi<0>(g, stream); break;
    case 1: e = launch_epi<1>(g, stream); break;
    case 2: e = launch_epi<2>(g, stream); break;
    default: return hipErrorInvalidValue;
  }
  if (e == hipSuccess && splits >= 2) {
    const uint64_t n = (uint64_t)M * N;
    const uint32_t blocks = (uint32_t)std::min<uint64_t>((n + kBlock - 1) / kBlock, 4096);
    hipLaunchKernelGGL(k_sum_splits, dim3(blocks), dim3(kBlock), 0, stream, split_ws, splits, M, N,
                       reinterpret_cast<float*>(C), ldc);
    e = hipGetLastError();
  }
  if (e == hipSuccess && Ct && !fused_t) e = launch_transpose_bf16(C, M, N, ldc, Ct, ldct, stream);
  return e;
}

hipError_t launch_transpose_bf16(const void* in, uint32_t R, uint32_t Cc, uint32_t ld_in, void* out, uint32_t ld_out,
                                 hipStream_t stream) {
  if (R == 0 || Cc == 0) return hipSuccess;
  hipLaunchKernelGGL(k_transpose_bf16, dim3((Cc + 63) / 64, (R + 63) / 64), dim3(kBlock), 0, stream,
                     reinterpret_cast<const bf16_t*>(in), R, Cc, ld_in, reinterpret_cast<bf16_t*>(out), ld_out);
  return hipGetLastError();
}

}  // namespace pemb
