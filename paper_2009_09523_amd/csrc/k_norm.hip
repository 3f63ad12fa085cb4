// Per-virtual-node BatchNorm (+ReLU) forward and backward, and column sums.
// The statistics are taken over exactly the R rows passed in -- the rows of the virtual node
// being processed (Section 4.1: such state is computed by each pass on its own; Section 3.2:
// each node is a separate forward and backward pass).  All reductions in fp32.
#include "vf_device.h"

namespace vf {
namespace {

constexpr int CB = 32;    // columns per workgroup (128-byte fp32 row segments)
constexpr int RL = 8;     // row lanes per column; 256 threads = CB x RL

// Sum over the RL row lanes of one column (threads with equal tx); result to all lanes.
__device__ __forceinline__ float col_reduce(float v, float (*red)[CB + 1], int tx, int ty) {
  red[ty][tx] = v;
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < RL; ++i) s += red[i][tx];
  __syncthreads();
  return s;
}

template <typename T>
__global__ __launch_bounds__(256) void bn_relu_fwd_kernel(const float* __restrict__ z, int64_t ldz,
                                                          int R, int C, const float* __restrict__ gamma,
                                                          const float* __restrict__ beta,
                                                          int round_params, float eps,
                                                          T* __restrict__ a, int64_t lda,
                                                          float* __restrict__ mean_out,
                                                          float* __restrict__ rstd_out) {
  __shared__ float red[RL][CB + 1];
  const int tx = threadIdx.x % CB, ty = threadIdx.x / CB;
  const int c = blockIdx.x * CB + tx;
  const bool live = c < C;
  if (gamma == nullptr) {                 // plain ReLU
    if (live)
      for (int r = ty; r < R; r += RL) store_f(&a[(int64_t)r * lda + c], fmaxf(z[(int64_t)r * ldz + c], 0.f));
    return;
  }
  float s = 0.f;
  if (live)
    for (int r = ty; r < R; r += RL) s += z[(int64_t)r * ldz + c];
  const float mean = col_reduce(s, red, tx, ty) / (float)R;
  float q = 0.f;
  if (live)
    for (int r = ty; r < R; r += RL) {
      float d = z[(int64_t)r * ldz + c] - mean;
      q = fmaf(d, d, q);
    }
  const float var = col_reduce(q, red, tx, ty) / (float)R;
  const float rstd = 1.0f / sqrtf(var + eps);
  if (!live) return;
  float g = gamma[c], b = beta[c];
  if (round_params) { g = round_bf16(g); b = round_bf16(b); }
  for (int r = ty; r < R; r += RL) {
    float xhat = (z[(int64_t)r * ldz + c] - mean) * rstd;
    store_f(&a[(int64_t)r * lda + c], fmaxf(fmaf(g, xhat, b), 0.f));
  }
  if (ty == 0) { mean_out[c] = mean; rstd_out[c] = rstd; }
}

template <typename T>
__global__ __launch_bounds__(256) void bn_relu_bwd_kernel(const float* __restrict__ da, int64_t ldda,
                                                          const float* __restrict__ z, int64_t ldz,
                                                          int R, int C, const float* __restrict__ gamma,
                                                          const float* __restrict__ beta,
                                                          int round_params,
                                                          const float* __restrict__ mean_in,
                                                          const float* __restrict__ rstd_in,
                                                          T* __restrict__ dz, int64_t lddz,
                                                          GradOut gout_g, GradOut gout_b) {
  __shared__ float red[RL][CB + 1];
  const int tx = threadIdx.x % CB, ty = threadIdx.x / CB;
  const int c = blockIdx.x * CB + tx;
  const bool live = c < C;
  if (gamma == nullptr) {                 // ReLU backward + bias gradient
    float sb = 0.f;
    if (live)
      for (int r = ty; r < R; r += RL) {
        float d = z[(int64_t)r * ldz + c] > 0.f ? da[(int64_t)r * ldda + c] : 0.f;
        store_f(&dz[(int64_t)r * lddz + c], d);
        sb += d;
      }
    sb = col_reduce(sb, red, tx, ty);
    if (live && ty == 0 && gout_b.dst) grad_store(gout_b, c, sb);
    return;
  }
  float g = 0.f, b = 0.f, mean = 0.f, rstd = 0.f;
  if (live) {
    g = gamma[c]; b = beta[c];
    if (round_params) { g = round_bf16(g); b = round_bf16(b); }
    mean = mean_in[c]; rstd = rstd_in[c];
  }
  float sg = 0.f, sb = 0.f;               // sum dout*xhat, sum dout
  if (live)
    for (int r = ty; r < R; r += RL) {
      float xhat = (z[(int64_t)r * ldz + c] - mean) * rstd;
      float dout = fmaf(g, xhat, b) > 0.f ? da[(int64_t)r * ldda + c] : 0.f;
      sg = fmaf(dout, xhat, sg);
      sb += dout;
    }
  sg = col_reduce(sg, red, tx, ty);
  sb = col_reduce(sb, red, tx, ty);
  if (!live) return;
  const float invR = 1.0f / (float)R;
  const float k = g * rstd;
  for (int r = ty; r < R; r += RL) {
    float xhat = (z[(int64_t)r * ldz + c] - mean) * rstd;
    float dout = fmaf(g, xhat, b) > 0.f ? da[(int64_t)r * ldda + c] : 0.f;
    store_f(&dz[(int64_t)r * lddz + c], k * (dout - sb * invR - xhat * sg * invR));
  }
  if (ty == 0) { grad_store(gout_g, c, sg); grad_store(gout_b, c, sb); }
}

template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(const T* __restrict__ x, int64_t ld, int R, int C,
                                                     GradOut out) {
  __shared__ float red[RL][CB + 1];
  const int tx = threadIdx.x % CB, ty = threadIdx.x / CB;
  const int c = blockIdx.x * CB + tx;
  float s = 0.f;
  if (c < C)
    for (int r = ty; r < R; r += RL) s += load_f(&x[(int64_t)r * ld + c]);
  s = col_reduce(s, red, tx, ty);
  if (c < C && ty == 0) grad_store(out, c, s);
}

}  // namespace

int launch_bn_relu_fwd(const float* z, int64_t ldz, int R, int C, const float* gamma,
                       const float* beta, int round_params, float eps, void* a, int64_t lda,
                       int a_is_bf16, float* mean, float* rstd, hipStream_t s) {
  if (R <= 0 || C <= 0) return VF_EINVAL;
  int grid = (C + CB - 1) / CB;
  if (a_is_bf16)
    bn_relu_fwd_kernel<bf16_t><<<grid, 256, 0, s>>>(z, ldz, R, C, gamma, beta, round_params, eps,
                                                    static_cast<bf16_t*>(a), lda, mean, rstd);
  else
    bn_relu_fwd_kernel<float><<<grid, 256, 0, s>>>(z, ldz, R, C, gamma, beta, round_params, eps,
                                                   static_cast<float*>(a), lda, mean, rstd);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_bn_relu_bwd(const float* da, int64_t ldda, const float* z, int64_t ldz, int R, int C,
                       const float* gamma, const float* beta, int round_params,
                       const float* mean, const float* rstd, void* dz, int64_t lddz,
                       int dz_is_bf16, GradOut gout_g, GradOut gout_b, hipStream_t s) {
  if (R <= 0 || C <= 0) return VF_EINVAL;
  int grid = (C + CB - 1) / CB;
  if (dz_is_bf16)
    bn_relu_bwd_kernel<bf16_t><<<grid, 256, 0, s>>>(da, ldda, z, ldz, R, C, gamma, beta, round_params,
                                                    mean, rstd, static_cast<bf16_t*>(dz), lddz,
                                                    gout_g, gout_b);
  else
    bn_relu_bwd_kernel<float><<<grid, 256, 0, s>>>(da, ldda, z, ldz, R, C, gamma, beta, round_params,
                                                   mean, rstd, static_cast<float*>(dz), lddz,
                                                   gout_g, gout_b);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_colsum(const void* x, int64_t ld, int x_is_bf16, int R, int C, GradOut out,
                  hipStream_t s) {
  if (R <= 0 || C <= 0) return VF_EINVAL;
  int grid = (C + CB - 1) / CB;
  if (x_is_bf16) colsum_kernel<bf16_t><<<grid, 256, 0, s>>>(static_cast<const bf16_t*>(x), ld, R, C, out);
  else           colsum_kernel<float><<<grid, 256, 0, s>>>(static_cast<const float*>(x), ld, R, C, out);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

}  // namespace vf
