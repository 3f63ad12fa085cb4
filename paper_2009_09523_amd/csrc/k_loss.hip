// Fused softmax cross-entropy: per row logsumexp, loss, and the gradient of the node's mean
// loss w.r.t. the logits in one kernel; then the node loss and the running weighted loss.
#include "vf_device.h"

namespace vf {
namespace {

__device__ __forceinline__ float block_reduce(float v, bool is_max, float* red) {
  v = is_max ? wave_max(v) : wave_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int i = 1; i < 4; ++i) r = is_max ? fmaxf(r, red[i]) : r + red[i];
  __syncthreads();
  return r;
}

// One workgroup per row.
template <typename T>
__global__ __launch_bounds__(256) void softmax_xent_kernel(const float* zp, int nsplit,
                                                           int64_t slab, int64_t ldzp,
                                                           float* z, int64_t ldz,
                                                           const int32_t* __restrict__ labels, int R,
                                                           int C, float* __restrict__ rowloss,
                                                           T* __restrict__ dz, int64_t lddz) {
  __shared__ float red[4];
  const int r = blockIdx.x;
  float* zr = z + (int64_t)r * ldz;
  int label = labels[r];
  label = label < 0 ? 0 : (label >= C ? C - 1 : label);
  float mx = -INFINITY;
  for (int c = threadIdx.x; c < C; c += 256) {      // add the partial slabs in order
    const int64_t idx = (int64_t)r * ldzp + c;
    float v = zp[idx];
    for (int s = 1; s < nsplit; ++s) v += zp[(int64_t)s * slab + idx];
    zr[c] = v;
    mx = fmaxf(mx, v);
  }
  mx = block_reduce(mx, true, red);
  float sum = 0.f;
  for (int c = threadIdx.x; c < C; c += 256) sum += expf(zr[c] - mx);
  sum = block_reduce(sum, false, red);
  const float inv = 1.0f / sum;
  const float invR = 1.0f / (float)R;
  T* dr = dz + (int64_t)r * lddz;
  for (int c = threadIdx.x; c < C; c += 256) {
    float p = expf(zr[c] - mx) * inv;
    store_f(&dr[c], (p - (c == label ? 1.f : 0.f)) * invR);
  }
  __syncthreads();   // zr[label] was written by another thread of this workgroup
  if (threadIdx.x == 0) rowloss[r] = logf(sum) + mx - zr[label];
}

__global__ __launch_bounds__(256) void loss_reduce_kernel(const float* __restrict__ rowloss, int R,
                                                          float w, int node,
                                                          float* __restrict__ node_loss,
                                                          float* __restrict__ total) {
  __shared__ float red[4];
  float s = 0.f;
  for (int r = threadIdx.x; r < R; r += 256) s += rowloss[r];
  s = block_reduce(s, false, red);
  if (threadIdx.x == 0) {
    float L = s / (float)R;
    node_loss[node] = L;
    float old = node == 0 ? 0.f : *total;
    *total = fmaf(w, L, old);
  }
}

}  // namespace

int launch_softmax_xent(const float* zp, int nsplit, int64_t slab, int64_t ldzp, float* z, int64_t ldz,
                        const int32_t* labels, int R, int C, float* rowloss, void* dz, int64_t lddz,
                        int dz_is_bf16, hipStream_t s) {
  if (R <= 0 || C <= 0 || nsplit < 1) return VF_EINVAL;
  if (dz_is_bf16)
    softmax_xent_kernel<bf16_t><<<R, 256, 0, s>>>(zp, nsplit, slab, ldzp, z, ldz, labels, R, C, rowloss,
                                                  static_cast<bf16_t*>(dz), lddz);
  else
    softmax_xent_kernel<float><<<R, 256, 0, s>>>(zp, nsplit, slab, ldzp, z, ldz, labels, R, C, rowloss,
                                                 static_cast<float*>(dz), lddz);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_loss_reduce(const float* rowloss, int R, float w, int node, float* node_loss,
                       float* total, hipStream_t s) {
  loss_reduce_kernel<<<1, 256, 0, s>>>(rowloss, R, w, node, node_loss, total);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

}  // namespace vf
