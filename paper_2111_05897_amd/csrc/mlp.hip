// Dense step of the hybrid model: feed-forward ReLU net with one logit, BCE loss, SGD -- forward,
// backward (gradients of the weights and of the pooled embedding activations) and update, bf16
// operands on the matrix cores with fp32 accumulation and fp32 master weights.  C ABI in
// include/persia_emb.h (mlp_*).
#include <hip/hip_runtime.h>

#include <cmath>
#include <new>
#include <string>
#include <vector>

#include "../../include/persia_emb.h"
#include "device_utils.h"
#include "launch.h"

using namespace pemb;

namespace {

thread_local std::string g_mlp_create_error;

// x[b, :] = bf16([pooled[b, :] | dense[b, :]]) and xt = x transposed ([P + Dn, B]); 64x64 tiles through LDS.
__global__ __launch_bounds__(kBlock) void k_pack_input(const float* __restrict__ pooled, uint32_t P,
                                                       const float* __restrict__ dense, uint32_t Dn, uint32_t B,
                                                       bf16_t* __restrict__ x, bf16_t* __restrict__ xt) {
  __shared__ bf16_t t[64][66];
  const uint32_t K0 = P + Dn;
  const uint32_t b0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  for (int i = threadIdx.x; i < 64 * 64; i += kBlock) {
    const uint32_t r = i / 64, cc = i % 64;
    const uint32_t b = b0 + r, c = c0 + cc;
    bf16_t v = 0;
    if (b < B && c < K0) {
      v = (bf16_t)f32_to_bf16(c < P ? pooled[(size_t)b * P + c] : dense[(size_t)b * Dn + (c - P)]);
      x[(size_t)b * K0 + c] = v;
    }
    t[r][cc] = v;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 64 * 64; i += kBlock) {
    const uint32_t cc = i / 64, r = i % 64;
    if (b0 + r < B && c0 + cc < K0) xt[(size_t)(c0 + cc) * B + b0 + r] = t[r][cc];
  }
}

// One wave per sample: z = h[b, :] . w + bias; dz = scale * (sigmoid(z) - y); loss term;
// delta[b, k] = bf16(dz * w[k] * [h[b, k] > 0]).  Per-workgroup loss sums go to loss_parts.
__global__ __launch_bounds__(kBlock) void k_logit_loss(const bf16_t* __restrict__ h, uint32_t H, uint32_t B,
                                                       const bf16_t* __restrict__ w, const float* __restrict__ bias,
                                                       const float* __restrict__ labels, float scale,
                                                       float* __restrict__ dz_out, bf16_t* __restrict__ delta,
                                                       float* __restrict__ loss_parts) {
  __shared__ float s_loss[kWavesPerBlock];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t b = blockIdx.x * kWavesPerBlock + wave;
  float term = 0.f;
  if (b < B) {
    float acc = 0.f;
    for (uint32_t k = lane; k < H; k += kWave) acc += bf16_to_f32(h[(size_t)b * H + k]) * bf16_to_f32(w[k]);
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) acc += __shfl_xor(acc, m);
    const float z = acc + bias[0];
    const float y = labels[b];
    // softplus(z) - y z, computed without overflow
    term = scale * (fmaxf(z, 0.f) + log1pf(expf(-fabsf(z))) - y * z);
    const float dz = scale * (1.f / (1.f + expf(-z)) - y);
    if (lane == 0) dz_out[b] = dz;
    for (uint32_t k = lane; k < H; k += kWave) {
      const bf16_t hv = h[(size_t)b * H + k];
      const bool on = (hv & 0x7FFFu) != 0 && !(hv & 0x8000u);
      delta[(size_t)b * H + k] = (bf16_t)f32_to_bf16(on ? dz * bf16_to_f32(w[k]) : 0.f);
    }
  }
  if (lane == 0) s_loss[wave] = term;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = 0.f;
    for (int i = 0; i < kWavesPerBlock; ++i) t += s_loss[i];
    loss_parts[blockIdx.x] = t;
  }
}

// Single block: out[0] = sum of parts[n], compensated, fixed order per thread then a fixed tree.
__global__ __launch_bounds__(kBlock) void k_sum_parts(const float* __restrict__ parts, uint32_t n,
                                                      float* __restrict__ out) {
  __shared__ float s[kBlock];
  float acc = 0.f, comp = 0.f;
  for (uint32_t i = threadIdx.x; i < n; i += kBlock) kahan_add(acc, comp, parts[i]);
  s[threadIdx.x] = acc;
  __syncthreads();
  for (int w = kBlock / 2; w >= 1; w >>= 1) {
    if ((int)threadIdx.x < w) s[threadIdx.x] += s[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = s[0];
}

// parts[chunk][c] = sum over the chunk's rows r of in[r][c] * (weight ? weight[r] : 1).
constexpr uint32_t kColChunks = 64;
__global__ __launch_bounds__(kBlock) void k_colsum_partial(const bf16_t* __restrict__ in, uint32_t R, uint32_t Cc,
                                                           const float* __restrict__ weight,
                                                           float* __restrict__ parts) {
  __shared__ float s[4][64];
  const int cx = threadIdx.x & 63, ry = threadIdx.x >> 6;
  const uint32_t c = blockIdx.x * 64 + cx;
  const uint32_t rows_per = (R + kColChunks - 1) / kColChunks;
  const uint32_t r0 = blockIdx.y * rows_per;
  const uint32_t r1 = (R - r0 < rows_per) ? R : r0 + rows_per;
  float acc = 0.f;
  if (c < Cc && r0 < R)
    for (uint32_t r = r0 + ry; r < r1; r += 4) acc += bf16_to_f32(in[(size_t)r * Cc + c]) * (weight ? weight[r] : 1.f);
  s[ry][cx] = acc;
  __syncthreads();
  if (ry == 0 && c < Cc) parts[(size_t)blockIdx.y * Cc + c] = (s[0][cx] + s[1][cx]) + (s[2][cx] + s[3][cx]);
}

__global__ __launch_bounds__(kBlock) void k_colsum_final(const float* __restrict__ parts, uint32_t Cc,
                                                         float* __restrict__ out) {
  const uint32_t c = blockIdx.x * kBlock + threadIdx.x;
  if (c >= Cc) return;
  float acc = 0.f;
  for (uint32_t j = 0; j < kColChunks; ++j) acc += parts[(size_t)j * Cc + c];
  out[c] = acc;
}

// SGD on the fp32 master weights [in, out] and refresh of both bf16 copies: W [in, out] and Wt [out, in].
__global__ __launch_bounds__(kBlock) void k_sgd_weights(float* __restrict__ master, const float* __restrict__ grad,
                                                        uint32_t n_in, uint32_t n_out, float lr,
                                                        bf16_t* __restrict__ w, bf16_t* __restrict__ wt) {
  __shared__ bf16_t t[64][66];
  const uint32_t r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  for (int i = threadIdx.x; i < 64 * 64; i += kBlock) {
    const uint32_t r = r0 + i / 64, c = c0 + i % 64;
    bf16_t v = 0;
    if (r < n_in && c < n_out) {
      const size_t idx = (size_t)r * n_out + c;
      const float nv = grad ? fmaf(-lr, grad[idx], master[idx]) : master[idx];
      master[idx] = nv;
      v = (bf16_t)f32_to_bf16(nv);
      w[idx] = v;
    }
    t[i / 64][i % 64] = v;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 64 * 64; i += kBlock) {
    const uint32_t c = c0 + i / 64, r = r0 + i % 64;
    if (r < n_in && c < n_out) wt[(size_t)c * n_in + r] = t[i % 64][i / 64];
  }
}

__global__ __launch_bounds__(kBlock) void k_sgd_vector(float* __restrict__ p, const float* __restrict__ grad,
                                                       uint32_t n, float lr) {
  const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
  if (i < n) p[i] = fmaf(-lr, grad[i], p[i]);
}

}  // namespace

struct mlp_ctx {
  int device = 0;
  uint32_t L = 0, P = 0, Dn = 0, max_batch = 0;
  std::vector<uint32_t> widths;  // [L+1]
  float lr = 0;
  int loss_mean = 1;
  // parameters
  std::vector<float*> Wm, bias, dW, db;   // fp32 master weights, biases and their gradients
  std::vector<bf16_t*> W, Wt;             // bf16 copies: [in, out] and [out, in]
  // activations for max_batch
  std::vector<bf16_t*> h, ht, delta, deltat;  // h[l]: [B, widths[l]] (h[0] = packed input), ht: transposed; delta[l] for l = 1..L-1
  float *dz = nullptr, *loss_parts = nullptr, *col_parts = nullptr;
  float* split_ws = nullptr;  // partial weight-gradient products (split along the batch dimension)
  uint64_t split_ws_elems = 0;
  uint32_t last_batch = 0;
  // delayed application of the gradients (a fully asynchronous dense side, for comparison): step t works with
  // weights that miss the last `delay` gradients; those of step t wait in ring_*[t % (delay + 1)] and are
  // applied at the beginning of step t + delay + 1
  uint32_t delay = 0;
  uint64_t steps_done = 0;
  std::vector<std::vector<float*>> ring_dW, ring_db;
  std::vector<void*> allocs;
  uint64_t device_bytes = 0;
  std::string err;
};

namespace {

int mfail(mlp_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg;
  else g_mlp_create_error = msg;
  return code;
}
int mfail_hip(mlp_ctx* c, const char* what, hipError_t e) {
  return mfail(c, e == hipErrorOutOfMemory ? EMB_ENOMEM : EMB_EDEVICE, std::string(what) + ": " + hipGetErrorString(e));
}

template <typename T>
hipError_t malloc_dev(mlp_ctx* c, T** p, uint64_t count) {
  void* q = nullptr;
  const uint64_t bytes = (count ? count : 1) * sizeof(T);
  hipError_t e = hipMalloc(&q, bytes);
  if (e != hipSuccess) return e;
  c->allocs.push_back(q);
  c->device_bytes += bytes;
  *p = reinterpret_cast<T*>(q);
  return hipSuccess;
}

void mlp_free(mlp_ctx* c) {
  for (void* p : c->allocs) (void)hipFree(p);
  c->allocs.clear();
}

int mlp_create_impl(const mlp_config* cfg, const float* const* weights, const float* const* biases, mlp_ctx** out) {
  if (!cfg || !weights || !biases || !out) return mfail(nullptr, EMB_EINVAL, "null argument");
  if (cfg->num_layers < 2 || cfg->num_layers > 16 || !cfg->widths) return mfail(nullptr, EMB_EINVAL, "num_layers must be in 2..16");
  if (cfg->reserved != 0) return mfail(nullptr, EMB_EINVAL, "config.reserved must be 0");
  const uint32_t L = cfg->num_layers;
  if (cfg->widths[0] != cfg->pooled_width + cfg->dense_width || cfg->pooled_width == 0)
    return mfail(nullptr, EMB_EINVAL, "widths[0] must equal pooled_width + dense_width");
  if (cfg->widths[L] != 1) return mfail(nullptr, EMB_EINVAL, "the last layer must have one output (the logit)");
  for (uint32_t l = 0; l < L; ++l)
    if (cfg->widths[l] == 0 || cfg->widths[l] % 64 != 0)
      return mfail(nullptr, EMB_EINVAL, "input and hidden widths must be positive multiples of 64");
  if (cfg->max_batch == 0 || cfg->max_batch % 64 != 0) return mfail(nullptr, EMB_EINVAL, "max_batch must be a positive multiple of 64");
  if (!std::isfinite(cfg->lr)) return mfail(nullptr, EMB_EINVAL, "lr must be finite");
  for (uint32_t l = 0; l < L; ++l)
    if (!weights[l] || !biases[l]) return mfail(nullptr, EMB_EINVAL, "null weight or bias array");
  int ndev = 0;
  hipError_t e = hipGetDeviceCount(&ndev);
  if (e != hipSuccess) return mfail_hip(nullptr, "hipGetDeviceCount", e);
  if (cfg->device < 0 || cfg->device >= ndev) return mfail(nullptr, EMB_EINVAL, "no such HIP device");
  if ((e = hipSetDevice(cfg->device)) != hipSuccess) return mfail_hip(nullptr, "hipSetDevice", e);

  mlp_ctx* c = new (std::nothrow) mlp_ctx();
  if (!c) return mfail(nullptr, EMB_ENOMEM, "out of host memory");
  struct Guard {
    mlp_ctx* c;
    ~Guard() {
      if (c) {
        mlp_free(c);
        delete c;
      }
    }
  } guard{c};
  c->device = cfg->device;
  c->L = L;
  c->P = cfg->pooled_width;
  c->Dn = cfg->dense_width;
  c->max_batch = cfg->max_batch;
  c->lr = cfg->lr;
  c->loss_mean = cfg->loss_mean;
  c->widths.assign(cfg->widths, cfg->widths + L + 1);
  c->Wm.resize(L); c->bias.resize(L); c->dW.resize(L); c->db.resize(L); c->W.resize(L); c->Wt.resize(L);
  c->h.resize(L); c->ht.resize(L); c->delta.resize(L); c->deltat.resize(L);
#define CK(call, what)                                        \
  do {                                                        \
    hipError_t _e = (call);                                   \
    if (_e != hipSuccess) return mfail_hip(nullptr, what, _e); \
  } while (0)
  const uint64_t B = c->max_batch;
  uint32_t max_w = 0;
  for (uint32_t l = 0; l < L; ++l) {
    const uint64_t n_in = c->widths[l], n_out = c->widths[l + 1];
    CK(malloc_dev(c, &c->Wm[l], n_in * n_out), "hipMalloc(weights)");
    CK(malloc_dev(c, &c->dW[l], n_in * n_out), "hipMalloc(weight gradient)");
    CK(malloc_dev(c, &c->W[l], n_in * n_out), "hipMalloc(bf16 weights)");
    CK(malloc_dev(c, &c->Wt[l], n_in * n_out), "hipMalloc(bf16 transposed weights)");
    CK(malloc_dev(c, &c->bias[l], n_out), "hipMalloc(bias)");
    CK(malloc_dev(c, &c->db[l], n_out), "hipMalloc(bias gradient)");
    CK(hipMemcpy(c->Wm[l], weights[l], n_in * n_out * sizeof(float), hipMemcpyHostToDevice), "upload(weights)");
    CK(hipMemcpy(c->bias[l], biases[l], n_out * sizeof(float), hipMemcpyHostToDevice), "upload(bias)");
    hipLaunchKernelGGL(k_sgd_weights, dim3((n_out + 63) / 64, (n_in + 63) / 64), dim3(kBlock), 0, nullptr, c->Wm[l],
                       (const float*)nullptr, (uint32_t)n_in, (uint32_t)n_out, 0.f, c->W[l], c->Wt[l]);
    CK(hipGetLastError(), "bf16 weight copies");
    CK(malloc_dev(c, &c->h[l], B * n_in), "hipMalloc(activations)");
    CK(malloc_dev(c, &c->ht[l], B * n_in), "hipMalloc(transposed activations)");
    if (l >= 1) {
      CK(malloc_dev(c, &c->delta[l], B * n_in), "hipMalloc(deltas)");
      CK(malloc_dev(c, &c->deltat[l], B * n_in), "hipMalloc(transposed deltas)");
    }
    if (n_in > max_w) max_w = (uint32_t)n_in;
  }
  // scratch for the weight-gradient products that are cut along the batch dimension
  c->split_ws_elems = 0;
  for (uint32_t l = 0; l + 1 < L; ++l) {
    const uint64_t need = (uint64_t)gemm_splits(c->widths[l], c->widths[l + 1], (uint32_t)B) * c->widths[l] * c->widths[l + 1];
    if (gemm_splits(c->widths[l], c->widths[l + 1], (uint32_t)B) >= 2 && need > c->split_ws_elems) c->split_ws_elems = need;
  }
  if (c->split_ws_elems) CK(malloc_dev(c, &c->split_ws, c->split_ws_elems), "hipMalloc(split-K scratch)");
  CK(malloc_dev(c, &c->dz, B), "hipMalloc(dz)");
  CK(malloc_dev(c, &c->loss_parts, (B + kWavesPerBlock - 1) / kWavesPerBlock), "hipMalloc(loss parts)");
  CK(malloc_dev(c, &c->col_parts, (uint64_t)kColChunks * max_w), "hipMalloc(column sums)");
  CK(hipDeviceSynchronize(), "mlp initialisation");
#undef CK
  guard.c = nullptr;
  *out = c;
  return EMB_OK;
}

#define CKM(call, what)                                     \
  do {                                                      \
    hipError_t _e = (call);                                 \
    if (_e != hipSuccess) return mfail_hip(c, what, _e);    \
  } while (0)

hipError_t colsum(mlp_ctx* c, const bf16_t* in, uint32_t R, uint32_t Cc, const float* weight, float* out,
                  hipStream_t s) {
  hipLaunchKernelGGL(k_colsum_partial, dim3((Cc + 63) / 64, kColChunks), dim3(kBlock), 0, s, in, R, Cc, weight,
                     c->col_parts);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_colsum_final, dim3((Cc + kBlock - 1) / kBlock), dim3(kBlock), 0, s, c->col_parts, Cc, out);
  return hipGetLastError();
}

// w -= lr * (the gradients c->dW / c->db point at), on the fp32 masters; refreshes the bf16 copies.
int apply_sgd(mlp_ctx* c, hipStream_t s) {
  const std::vector<uint32_t>& w = c->widths;
  for (uint32_t l = 0; l < c->L; ++l) {
    const uint32_t n_in = w[l], n_out = w[l + 1];
    hipLaunchKernelGGL(k_sgd_weights, dim3((n_out + 63) / 64, (n_in + 63) / 64), dim3(kBlock), 0, s, c->Wm[l],
                       (const float*)c->dW[l], n_in, n_out, c->lr, c->W[l], c->Wt[l]);
    CKM(hipGetLastError(), "sgd(weights)");
    hipLaunchKernelGGL(k_sgd_vector, dim3((n_out + kBlock - 1) / kBlock), dim3(kBlock), 0, s, c->bias[l],
                       (const float*)c->db[l], n_out, c->lr);
    CKM(hipGetLastError(), "sgd(bias)");
  }
  return EMB_OK;
}

int mlp_set_update_delay_impl(mlp_ctx* c, uint32_t delay) {
  if (!c) return mfail(nullptr, EMB_EINVAL, "null context");
  if (c->steps_done != 0 || c->delay != 0) return mfail(c, EMB_ESTATE, "the delay can be set once, before the first step");
  if (delay > 256) return mfail(c, EMB_EINVAL, "delay must be at most 256");
  if (delay == 0) return EMB_OK;
  CKM(hipSetDevice(c->device), "hipSetDevice");
  c->ring_dW.assign((size_t)delay + 1, std::vector<float*>(c->L, nullptr));
  c->ring_db.assign((size_t)delay + 1, std::vector<float*>(c->L, nullptr));
  c->ring_dW[0] = c->dW;  // the set the context was created with is the first of the ring
  c->ring_db[0] = c->db;
  for (uint32_t d = 1; d <= delay; ++d)
    for (uint32_t l = 0; l < c->L; ++l) {
      CKM(malloc_dev(c, &c->ring_dW[d][l], (uint64_t)c->widths[l] * c->widths[l + 1]), "hipMalloc(delayed weight gradient)");
      CKM(malloc_dev(c, &c->ring_db[d][l], c->widths[l + 1]), "hipMalloc(delayed bias gradient)");
    }
  c->delay = delay;
  return EMB_OK;
}

int mlp_step_impl(mlp_ctx* c, uint32_t B, const float* pooled, const float* dense, const float* labels,
                  float* d_pooled, float* loss, void* hip_stream) {
  if (!c) return mfail(nullptr, EMB_EINVAL, "null context");
  if (B == 0 || B > c->max_batch || B % 64 != 0) return mfail(c, EMB_EINVAL, "batch must be a multiple of 64 within max_batch");
  if (!pooled || (c->Dn && !dense) || !labels || !d_pooled || !loss) return mfail(c, EMB_EINVAL, "null buffer");
  hipStream_t s = (hipStream_t)hip_stream;
  CKM(hipSetDevice(c->device), "hipSetDevice");
  const uint32_t L = c->L;
  const std::vector<uint32_t>& w = c->widths;
  c->last_batch = B;
  if (c->delay) {  // the gradients computed delay + 1 steps ago are due now; this step's go into their place
    const size_t slot = (size_t)(c->steps_done % ((uint64_t)c->delay + 1));
    c->dW = c->ring_dW[slot];
    c->db = c->ring_db[slot];
    if (c->steps_done >= (uint64_t)c->delay + 1) {
      const int rc = apply_sgd(c, s);
      if (rc != EMB_OK) return rc;
    }
  }
  // forward
  {
    hipLaunchKernelGGL(k_pack_input, dim3((w[0] + 63) / 64, (B + 63) / 64), dim3(kBlock), 0, s, pooled, c->P, dense,
                       c->Dn, B, c->h[0], c->ht[0]);
    CKM(hipGetLastError(), "pack_input");
  }
  // h[l+1] = relu(h[l] W[l] + b[l]); the weight gradients below want h[1..L-2] transposed as well
  for (uint32_t l = 0; l + 1 < L; ++l)
    CKM(launch_gemm_nt(0, c->h[l], w[l], c->Wt[l], w[l], B, w[l + 1], w[l], c->h[l + 1], w[l + 1], c->bias[l], nullptr, 0, s,
                       l + 2 < L ? c->ht[l + 1] : nullptr, B),
        "gemm(forward)");
  const uint32_t H = w[L - 1];
  const float scale = c->loss_mean ? 1.0f / (float)B : 1.0f;
  const uint32_t loss_blocks = (B + kWavesPerBlock - 1) / kWavesPerBlock;
  hipLaunchKernelGGL(k_logit_loss, dim3(loss_blocks), dim3(kBlock), 0, s, c->h[L - 1], H, B, c->W[L - 1], c->bias[L - 1],
                     labels, scale, c->dz, c->delta[L - 1], c->loss_parts);
  CKM(hipGetLastError(), "logit_loss");
  hipLaunchKernelGGL(k_sum_parts, dim3(1), dim3(kBlock), 0, s, c->loss_parts, loss_blocks, loss);
  CKM(hipGetLastError(), "loss_sum");
  // backward: last layer (a vector): dW = h^T dz, db = sum dz
  CKM(colsum(c, c->h[L - 1], B, H, c->dz, c->dW[L - 1], s), "dW(last)");
  hipLaunchKernelGGL(k_sum_parts, dim3(1), dim3(kBlock), 0, s, c->dz, B, c->db[L - 1]);
  CKM(hipGetLastError(), "db(last)");
  for (uint32_t l = L - 1; l >= 1; --l) {
    // delta[l]: [B, w[l]] is the gradient w.r.t. the pre-activation of h[l]; it feeds layer l-1's weights
    CKM(colsum(c, c->delta[l], B, w[l], nullptr, c->db[l - 1], s), "db");
    // ht[l-1] came with the forward pass and deltat[l] with the GEMM that made delta[l]; the last layer's
    // delta comes from the loss kernel
    if (l == L - 1) CKM(launch_transpose_bf16(c->delta[l], B, w[l], w[l], c->deltat[l], B, s), "transpose(delta)");
    // dW[l-1] [w[l-1], w[l]] = h[l-1]^T delta[l]
    CKM(launch_gemm_nt(1, c->ht[l - 1], B, c->deltat[l], B, w[l - 1], w[l], B, c->dW[l - 1], w[l], nullptr, nullptr, 0, s,
                       nullptr, 0, c->split_ws, c->split_ws_elems),
        "gemm(dW)");
    if (l >= 2) {  // delta[l-1] = (delta[l] W[l-1]^T) masked by h[l-1] > 0
      CKM(launch_gemm_nt(2, c->delta[l], w[l], c->W[l - 1], w[l], B, w[l - 1], w[l], c->delta[l - 1], w[l - 1], nullptr,
                         c->h[l - 1], w[l - 1], s, c->deltat[l - 1], B),
          "gemm(delta)");
    } else {  // gradient of the pooled embedding activations: the first P input columns, fp32
      CKM(launch_gemm_nt(1, c->delta[1], w[1], c->W[0], w[1], B, c->P, w[1], d_pooled, c->P, nullptr, nullptr, 0, s),
          "gemm(d_pooled)");
    }
  }
  if (c->delay == 0) {
    const int rc = apply_sgd(c, s);
    if (rc != EMB_OK) return rc;
  }
  ++c->steps_done;
  return EMB_OK;
}

int mlp_read_weights_impl(mlp_ctx* c, uint32_t layer, float* w_host, float* b_host) {
  if (!c) return mfail(nullptr, EMB_EINVAL, "null context");
  if (layer >= c->L) return mfail(c, EMB_EINVAL, "no such layer");
  CKM(hipSetDevice(c->device), "hipSetDevice");
  CKM(hipDeviceSynchronize(), "hipDeviceSynchronize");
  const uint64_t n = (uint64_t)c->widths[layer] * c->widths[layer + 1];
  if (w_host) CKM(hipMemcpy(w_host, c->Wm[layer], n * sizeof(float), hipMemcpyDeviceToHost), "hipMemcpy(weights)");
  if (b_host)
    CKM(hipMemcpy(b_host, c->bias[layer], c->widths[layer + 1] * sizeof(float), hipMemcpyDeviceToHost), "hipMemcpy(bias)");
  return EMB_OK;
}

int mlp_read_state_impl(mlp_ctx* c, int what, uint32_t layer, void* host, uint64_t bytes) {
  if (!c) return mfail(nullptr, EMB_EINVAL, "null context");
  if (!host) return mfail(c, EMB_EINVAL, "null buffer");
  if (c->last_batch == 0) return mfail(c, EMB_ESTATE, "no mlp_step has run on this context");
  const uint64_t B = c->last_batch;
  const void* src = nullptr;
  uint64_t need = 0;
  switch (what) {
    case 0:  // activation h[layer], bf16 [B, widths[layer]]
      if (layer >= c->L) return mfail(c, EMB_EINVAL, "no such layer");
      src = c->h[layer];
      need = B * c->widths[layer] * 2;
      break;
    case 1:  // delta[layer], bf16 [B, widths[layer]], layer in 1..L-1
      if (layer < 1 || layer >= c->L) return mfail(c, EMB_EINVAL, "no such layer");
      src = c->delta[layer];
      need = B * c->widths[layer] * 2;
      break;
    case 2:  // weight gradient of layer, fp32 [widths[layer], widths[layer+1]]
      if (layer >= c->L) return mfail(c, EMB_EINVAL, "no such layer");
      src = c->dW[layer];
      need = (uint64_t)c->widths[layer] * c->widths[layer + 1] * 4;
      break;
    case 3:  // bias gradient of layer, fp32 [widths[layer+1]]
      if (layer >= c->L) return mfail(c, EMB_EINVAL, "no such layer");
      src = c->db[layer];
      need = (uint64_t)c->widths[layer + 1] * 4;
      break;
    case 4:  // d loss / d logit, fp32 [B]
      src = c->dz;
      need = B * 4;
      break;
    default: return mfail(c, EMB_EINVAL, "unknown state kind");
  }
  if (bytes != need) return mfail(c, EMB_EINVAL, "buffer size does not match the state's size");
  CKM(hipSetDevice(c->device), "hipSetDevice");
  CKM(hipDeviceSynchronize(), "hipDeviceSynchronize");
  CKM(hipMemcpy(host, src, need, hipMemcpyDeviceToHost), "hipMemcpy(state)");
  return EMB_OK;
}

}  // namespace

extern "C" {

#define MLP_GUARDED(ctx_expr, call)                                                 \
  try {                                                                             \
    return call;                                                                    \
  } catch (const std::bad_alloc&) {                                                 \
    return mfail(ctx_expr, EMB_ENOMEM, "out of host memory");                       \
  } catch (...) {                                                                   \
    return mfail(ctx_expr, EMB_ESTATE, "unexpected exception inside the library");  \
  }

int mlp_create(const mlp_config* cfg, const float* const* weights, const float* const* biases, mlp_ctx** out) {
  MLP_GUARDED(nullptr, mlp_create_impl(cfg, weights, biases, out))
}
int mlp_step(mlp_ctx* ctx, uint32_t batch, const float* pooled, const float* dense, const float* labels, float* d_pooled,
             float* loss, void* hip_stream) {
  MLP_GUARDED(ctx, mlp_step_impl(ctx, batch, pooled, dense, labels, d_pooled, loss, hip_stream))
}
int mlp_read_weights(mlp_ctx* ctx, uint32_t layer, float* w, float* b) {
  MLP_GUARDED(ctx, mlp_read_weights_impl(ctx, layer, w, b))
}
int mlp_read_state(mlp_ctx* ctx, int what, uint32_t layer, void* host, uint64_t bytes) {
  MLP_GUARDED(ctx, mlp_read_state_impl(ctx, what, layer, host, bytes))
}
int mlp_destroy(mlp_ctx* ctx) {
  if (!ctx) return EMB_OK;
  (void)hipSetDevice(ctx->device);
  (void)hipDeviceSynchronize();
  mlp_free(ctx);
  delete ctx;
  return EMB_OK;
}
uint64_t mlp_device_bytes(mlp_ctx* ctx) { return ctx ? ctx->device_bytes : 0; }
int mlp_set_update_delay(mlp_ctx* ctx, uint32_t delay) { MLP_GUARDED(ctx, mlp_set_update_delay_impl(ctx, delay)) }
int mlp_describe(mlp_ctx* ctx, uint32_t* pooled_width, uint32_t* dense_width, uint32_t* max_batch, int32_t* device) {
  if (!ctx) return mfail(nullptr, EMB_EINVAL, "null context");
  if (pooled_width) *pooled_width = ctx->P;
  if (dense_width) *dense_width = ctx->Dn;
  if (max_batch) *max_batch = ctx->max_batch;
  if (device) *device = ctx->device;
  return EMB_OK;
}
int mlp_gemm_nt(int epilogue, const uint16_t* A, uint32_t lda, const uint16_t* Bt, uint32_t ldb, uint32_t M, uint32_t N,
                uint32_t K, void* C, uint32_t ldc, const float* bias, const uint16_t* mask, uint32_t ldm, void* hip_stream) {
  hipError_t e = launch_gemm_nt(epilogue, A, lda, Bt, ldb, M, N, K, C, ldc, bias, mask, ldm, (hipStream_t)hip_stream);
  if (e == hipErrorInvalidValue) return mfail(nullptr, EMB_EINVAL, "gemm_nt: bad shape, stride, epilogue or null operand");
  return e == hipSuccess ? EMB_OK : mfail_hip(nullptr, "gemm_nt", e);
}
const char* mlp_last_error(mlp_ctx* ctx) { return ctx ? ctx->err.c_str() : g_mlp_create_error.c_str(); }

}  // extern "C"
