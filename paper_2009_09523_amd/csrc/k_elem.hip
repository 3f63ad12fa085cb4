// Layout kernels: bf16 transposes and the fp32 -> bf16 weight copies the GEMMs read.
#include "vf_device.h"

namespace vf {
namespace {

constexpr int TS = 32;   // tile side; 256 threads = 32 x 8

// out[c*ldo + r] = in[r*ldi + c]
template <typename TIN>
__global__ __launch_bounds__(256) void transpose_kernel(const TIN* __restrict__ in, int64_t ldi,
                                                        bf16_t* __restrict__ out, int64_t ldo,
                                                        bf16_t* __restrict__ nat, int64_t ldn,
                                                        int R, int C) {
  __shared__ bf16_t tile[TS][TS + 2];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int r0 = blockIdx.y * TS, c0 = blockIdx.x * TS;
#pragma unroll
  for (int i = 0; i < TS; i += 8) {
    int r = r0 + ty + i, c = c0 + tx;
    if (r < R && c < C) {
      bf16_t v;
      if constexpr (sizeof(TIN) == 4) v = f32_to_bf16(in[(int64_t)r * ldi + c]);
      else v = in[(int64_t)r * ldi + c];
      tile[ty + i][tx] = v;
      if (nat) nat[(int64_t)r * ldn + c] = v;
    }
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < TS; i += 8) {
    int c = c0 + ty + i, r = r0 + tx;
    if (r < R && c < C) out[(int64_t)c * ldo + r] = tile[tx][ty + i];
  }
}

__global__ __launch_bounds__(256) void cast_kernel(const float* __restrict__ in, int64_t ldi,
                                                   bf16_t* __restrict__ out, int64_t ldo, int R, int C) {
  int c = blockIdx.x * 256 + threadIdx.x;
  int r = blockIdx.y;
  if (c < C) out[(int64_t)r * ldo + c] = f32_to_bf16(in[(int64_t)r * ldi + c]);
}

}  // namespace

int launch_transpose_bf16(const bf16_t* in, int64_t ldi, bf16_t* out, int64_t ldo, int R, int C,
                          hipStream_t s) {
  if (R <= 0 || C <= 0) return VF_OK;
  dim3 grid((C + TS - 1) / TS, (R + TS - 1) / TS);
  transpose_kernel<bf16_t><<<grid, 256, 0, s>>>(in, ldi, out, ldo, nullptr, 0, R, C);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_cast_weight(const float* w, int R, int C, bf16_t* nat, int64_t ldn, bf16_t* tr,
                       int64_t ldt, hipStream_t s) {
  if (R <= 0 || C <= 0) return VF_OK;
  dim3 grid((C + TS - 1) / TS, (R + TS - 1) / TS);
  transpose_kernel<float><<<grid, 256, 0, s>>>(w, C, tr, ldt, nat, ldn, R, C);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_cast_bf16(const float* in, int64_t ldi, bf16_t* out, int64_t ldo, int R, int C,
                     hipStream_t s) {
  if (R <= 0 || C <= 0) return VF_OK;
  dim3 grid((C + 255) / 256, R);
  cast_kernel<<<grid, 256, 0, s>>>(in, ldi, out, ldo, R, C);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

}  // namespace vf
