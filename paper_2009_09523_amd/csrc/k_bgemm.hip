// Batched small GEMM with arbitrary strides and mixed operand types, fp32 accumulation on
// the vector ALUs.  Used for the per-(sequence, head) contractions of self-attention
// (scores, probabilities x values, and their backward products), where every matrix is a
// strided window of a larger activation tensor.
//   C[b][m,n] = alpha * sum_k A[b][m,k] * B[b][n,k]
// with X[b][i,k] at X + (b / inner) * x.outer + (b % inner) * x.inner + i * x.rs + k * x.cs.
#include "vf_device.h"

namespace vf {
namespace {

constexpr int TM = 64, TN = 64, TK = 16, NT = 256;

__device__ __forceinline__ float load_any(const BMat& x, int64_t idx) {
  if (x.is_bf16) return bf16_to_f32(static_cast<const bf16_t*>(x.p)[idx]);
  float v = static_cast<const float*>(x.p)[idx];
  return x.round_bf16 ? round_bf16(v) : v;
}

__device__ __forceinline__ void load_tile(const BMat& x, int64_t base, int row0, int nrows, int k0, int K,
                                          float (*dst)[TM + 4], int tid) {
  if (x.cs == 1) {
#pragma unroll
    for (int i = 0; i < (TM * TK) / NT; ++i) {
      int e = tid + i * NT;
      int k = e % TK, r = e / TK;
      int gr = row0 + r, gk = k0 + k;
      dst[k][r] = (gr < nrows && gk < K) ? load_any(x, base + (int64_t)gr * x.rs + gk) : 0.f;
    }
  } else {
#pragma unroll
    for (int i = 0; i < (TM * TK) / NT; ++i) {
      int e = tid + i * NT;
      int r = e % TM, k = e / TM;
      int gr = row0 + r, gk = k0 + k;
      dst[k][r] = (gr < nrows && gk < K)
                      ? load_any(x, base + (int64_t)gr * x.rs + (int64_t)gk * x.cs) : 0.f;
    }
  }
}

__global__ __launch_bounds__(NT) void bgemm_kernel(BMat A, BMat B, BMat C, int M, int N, int K, int inner,
                                                   float alpha) {
  __shared__ float As[TK][TM + 4];
  __shared__ float Bs[TK][TN + 4];
  const int tid = threadIdx.x;
  const int tx = tid % 16, ty = tid / 16;
  const int batch = blockIdx.z;
  const int bo = batch / inner, bi = batch % inner;
  const int64_t abase = (int64_t)bo * A.outer + (int64_t)bi * A.inner;
  const int64_t bbase = (int64_t)bo * B.outer + (int64_t)bi * B.inner;
  const int64_t cbase = (int64_t)bo * C.outer + (int64_t)bi * C.inner;
  const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += TK) {
    load_tile(A, abase, m0, M, k0, K, As, tid);
    load_tile(B, bbase, n0, N, k0, K, Bs, tid);
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
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      float v = alpha * acc[i][j];
      int64_t idx = cbase + (int64_t)m * C.rs + (int64_t)n * C.cs;
      if (C.is_bf16) static_cast<bf16_t*>(const_cast<void*>(C.p))[idx] = f32_to_bf16(v);
      else           static_cast<float*>(const_cast<void*>(C.p))[idx] = v;
    }
  }
}

}  // namespace

int launch_bgemm(const BMat& A, const BMat& B, const BMat& C, int M, int N, int K, int batch, int inner,
                 float alpha, hipStream_t s) {
  if (M <= 0 || N <= 0 || K <= 0 || batch <= 0 || inner <= 0 || !A.p || !B.p || !C.p) return VF_EINVAL;
  if (batch > 65535) return VF_EINVAL;
  dim3 grid((N + TN - 1) / TN, (M + TM - 1) / TM, batch);
  bgemm_kernel<<<grid, NT, 0, s>>>(A, B, C, M, N, K, inner, alpha);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

}  // namespace vf
