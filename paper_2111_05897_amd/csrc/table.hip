// Table storage kernels: counter-based initialisation and row read/write for inspection.
#include "device_utils.h"
#include "launch.h"

namespace pemb {
namespace {

// One thread initialises 4 consecutive elements (fp32: one 16-byte store; bf16: one 8-byte store).
template <typename T>
__global__ __launch_bounds__(kBlock) void k_init_table(T* __restrict__ w, uint64_t n_elems, uint64_t table_key,
                                                       float scale, float mid) {
  uint64_t q = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  for (; q * 4 < n_elems; q += stride) {
    uint64_t e = q * 4;
    float4 v = make_float4(init_value(table_key, e, scale, mid), init_value(table_key, e + 1, scale, mid),
                           init_value(table_key, e + 2, scale, mid), init_value(table_key, e + 3, scale, mid));
    store_frag4(w + e, v);  // bf16 tables round the fp32 value to storage here
  }
}

__global__ __launch_bounds__(kBlock) void k_fill_f32(float* __restrict__ p, uint64_t n, float v) {
  uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  for (; i < n; i += stride) p[i] = v;
}

// For a table behind the LRU cache (`where` not null) a row is in its cache slot if it has one, else in the
// host table.
template <typename T>
__global__ __launch_bounds__(kBlock) void k_read_rows(const T* __restrict__ w, const float* __restrict__ acc,
                                                      uint32_t dim, const uint64_t* __restrict__ rows, uint64_t n,
                                                      float* __restrict__ w_out, float* __restrict__ acc_out,
                                                      const int32_t* __restrict__ where, const T* __restrict__ back_w,
                                                      const float* __restrict__ back_acc) {
  uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= n * dim) return;
  uint64_t r = i / dim;
  uint32_t d = (uint32_t)(i - r * dim);
  uint64_t row = rows[r];
  if (where) {
    const int32_t slot = where[row];
    if (slot >= 0) row = (uint64_t)slot;
    else w = back_w, acc = back_acc;
  }
  if (w_out) {
    if constexpr (sizeof(T) == 2) w_out[i] = bf16_to_f32(w[row * dim + d]);
    else w_out[i] = w[row * dim + d];
  }
  if (acc_out && d == 0) acc_out[r] = acc[row];
}

template <typename T>
__global__ __launch_bounds__(kBlock) void k_write_rows(T* __restrict__ w, float* __restrict__ acc, uint32_t dim,
                                                       const uint64_t* __restrict__ rows, uint64_t n,
                                                       const float* __restrict__ w_in,
                                                       const float* __restrict__ acc_in,
                                                       const int32_t* __restrict__ where, T* __restrict__ back_w,
                                                       float* __restrict__ back_acc) {
  uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= n * dim) return;
  uint64_t r = i / dim;
  uint32_t d = (uint32_t)(i - r * dim);
  uint64_t row = rows[r];
  if (where) {
    const int32_t slot = where[row];
    if (slot >= 0) row = (uint64_t)slot;
    else w = back_w, acc = back_acc;
  }
  if (w_in) {
    if constexpr (sizeof(T) == 2) w[row * dim + d] = (bf16_t)f32_to_bf16(w_in[i]);
    else w[row * dim + d] = w_in[i];
  }
  if (acc_in && d == 0) acc[row] = acc_in[r];
}

uint32_t capped_grid(uint64_t work_items, uint32_t cap) {
  uint64_t b = (work_items + kBlock - 1) / kBlock;
  if (b < 1) b = 1;
  return (uint32_t)(b < cap ? b : cap);
}

}  // namespace

hipError_t launch_init_table(const TableView& t, uint64_t table_key, float scale, float mid, float acc_init,
                             hipStream_t stream) {
  const uint64_t n_elems = t.rows * t.dim;  // dim is a multiple of 8, so n_elems % 4 == 0
  const uint32_t grid = capped_grid(n_elems / 4, 1u << 16);
  if (t.dtype == 1)
    hipLaunchKernelGGL(k_init_table<bf16_t>, dim3(grid), dim3(kBlock), 0, stream, (bf16_t*)t.w, n_elems, table_key,
                       scale, mid);
  else
    hipLaunchKernelGGL(k_init_table<float>, dim3(grid), dim3(kBlock), 0, stream, (float*)t.w, n_elems, table_key,
                       scale, mid);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_fill_f32, dim3(capped_grid(t.rows, 1u << 14)), dim3(kBlock), 0, stream, t.acc, t.rows,
                     acc_init);
  return hipGetLastError();
}

hipError_t launch_read_rows(const TableView& t, const uint64_t* rows_dev, uint64_t n, float* w_out, float* acc_out,
                            hipStream_t stream) {
  if (n == 0) return hipSuccess;
  const uint32_t grid = (uint32_t)((n * t.dim + kBlock - 1) / kBlock);
  if (t.dtype == 1)
    hipLaunchKernelGGL(k_read_rows<bf16_t>, dim3(grid), dim3(kBlock), 0, stream, (const bf16_t*)t.w, (const float*)t.acc,
                       t.dim, rows_dev, n, w_out, acc_out, t.where, (const bf16_t*)t.back_w, (const float*)t.back_acc);
  else
    hipLaunchKernelGGL(k_read_rows<float>, dim3(grid), dim3(kBlock), 0, stream, (const float*)t.w, (const float*)t.acc,
                       t.dim, rows_dev, n, w_out, acc_out, t.where, (const float*)t.back_w, (const float*)t.back_acc);
  return hipGetLastError();
}

hipError_t launch_write_rows(const TableView& t, const uint64_t* rows_dev, uint64_t n, const float* w_in,
                             const float* acc_in, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  const uint32_t grid = (uint32_t)((n * t.dim + kBlock - 1) / kBlock);
  if (t.dtype == 1)
    hipLaunchKernelGGL(k_write_rows<bf16_t>, dim3(grid), dim3(kBlock), 0, stream, (bf16_t*)t.w, t.acc, t.dim,
                       rows_dev, n, w_in, acc_in, t.where, (bf16_t*)t.back_w, t.back_acc);
  else
    hipLaunchKernelGGL(k_write_rows<float>, dim3(grid), dim3(kBlock), 0, stream, (float*)t.w, t.acc, t.dim, rows_dev,
                       n, w_in, acc_in, t.where, (float*)t.back_w, t.back_acc);
  return hipGetLastError();
}

}  // namespace pemb
