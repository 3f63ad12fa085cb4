// fp32 GEMM with arbitrary operand strides, LDS-tiled, for the fp32 workloads (the small
// parity configuration).  acc[m,n] = sum_k A[m*sam + k*sak] * B[n*sbn + k*sbk].
#include "vf_device.h"

namespace vf {
namespace {

constexpr int TM = 64, TN = 64, TK = 16, NT = 256;

// Loads a [ROWS x TK] tile (row index r in [0,ROWS), k in [0,TK)) into dst[k][r].
// When the k stride is 1 consecutive threads walk k, otherwise they walk rows, so that
// the unit-stride index is always the fastest across a wavefront.
__device__ __forceinline__ void load_tile(const float* __restrict__ base, int64_t srow, int64_t sk,
                                          int row0, int nrows, int k0, int K,
                                          float (*dst)[TM + 4], int tid) {
  if (sk == 1) {
#pragma unroll
    for (int i = 0; i < (TM * TK) / NT; ++i) {
      int e = tid + i * NT;
      int k = e % TK, r = e / TK;
      int gr = row0 + r, gk = k0 + k;
      float v = 0.f;
      if (gr < nrows && gk < K) v = base[(int64_t)gr * srow + gk];
      dst[k][r] = v;
    }
  } else {
#pragma unroll
    for (int i = 0; i < (TM * TK) / NT; ++i) {
      int e = tid + i * NT;
      int r = e % TM, k = e / TM;
      int gr = row0 + r, gk = k0 + k;
      float v = 0.f;
      if (gr < nrows && gk < K) v = base[(int64_t)gr * srow + (int64_t)gk * sk];
      dst[k][r] = v;
    }
  }
}

// blockIdx.z selects the contraction slice [z*kchunk, (z+1)*kchunk); slice z writes its partial
// product to slab z of C (the consumer adds the slabs in order), the bias goes to slab 0.
__global__ __launch_bounds__(NT) void gemm_f32_kernel(const float* __restrict__ A, int64_t sam,
                                                      int64_t sak, const float* __restrict__ B,
                                                      int64_t sbn, int64_t sbk, int M, int N, int K,
                                                      int kchunk, int64_t slab_stride, Epilogue ep) {
  __shared__ float As[TK][TM + 4];
  __shared__ float Bs[TK][TN + 4];
  const int tid = threadIdx.x;
  const int tx = tid % 16, ty = tid / 16;
  const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
  float acc[4][4] = {};
  const int kbeg = blockIdx.z * kchunk;
  const int kend = min(K, kbeg + kchunk);
  for (int k0 = kbeg; k0 < kend; k0 += TK) {
    load_tile(A, sam, sak, m0, M, k0, kend, As, tid);
    load_tile(B, sbn, sbk, n0, N, k0, kend, Bs, tid);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < TK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  float* C = static_cast<float*>(ep.C) + (int64_t)blockIdx.z * slab_stride;
  const bool first_slice = blockIdx.z == 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      float addend = (ep.bias && first_slice) ? ep.bias[n] : 0.f;
      if (ep.R) addend = fmaf(ep.beta, ep.R[(int64_t)m * ep.ldr + n], addend);
      float v = fmaf(ep.alpha, acc[i][j], addend);
      C[(int64_t)m * ep.ldc + n] = v;
    }
  }
}

}  // namespace

int gemm_f32_pick_split(int M, int N, int K) {
  // small fp32 products are latency bound: spread the contraction until about 128 workgroups
  // exist, slices no shorter than four 16-wide stages
  int64_t tiles = (int64_t)((M + TM - 1) / TM) * ((N + TN - 1) / TN);
  int split = 1;
  while (tiles * split < 128 && K / (split * 2) >= 4 * TK && split < 32) split *= 2;
  return split;
}

int launch_gemm_f32(const float* A, int64_t sam, int64_t sak, const float* B, int64_t sbn,
                    int64_t sbk, int M, int N, int K, int nsplit, int64_t slab_stride,
                    const Epilogue& ep, hipStream_t s) {
  if (M <= 0 || N <= 0 || K < 0 || !A || !B || !ep.C || ep.c_is_bf16 || nsplit < 1) return VF_EINVAL;
  if (nsplit > 1 && ep.R) return VF_EINVAL;
  const int kchunk = ((K + nsplit - 1) / nsplit + TK - 1) / TK * TK;
  dim3 grid((N + TN - 1) / TN, (M + TM - 1) / TM, nsplit);
  gemm_f32_kernel<<<grid, NT, 0, s>>>(A, sam, sak, B, sbn, sbk, M, N, K, kchunk > 0 ? kchunk : TK,
                                      slab_stride, ep);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

}  // namespace vf
