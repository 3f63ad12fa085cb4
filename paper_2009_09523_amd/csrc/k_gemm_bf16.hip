// bf16 GEMM on the matrix cores of gfx950:  acc[m,n] = sum_k A[m*lda+k] * B[n*ldb+k]
// (both operands contiguous along the contraction), fp32 accumulation with
// v_mfma_f32_32x32x16_bf16, tiles staged through LDS.  Used for the forward, input-gradient
// and weight-gradient contractions of every Linear layer.
#include "vf_device.h"

namespace vf {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int NT = 256;          // 4 wavefronts
constexpr int BK = 64;           // contraction elements per LDS stage
constexpr int LDS_LD = BK + 8;   // padded row (144 bytes) keeps 16-byte reads conflict-free

// 16-byte global load of 8 consecutive bf16 of row `row` at contraction offset k, zero
// beyond the matrix (rows >= nrows, k >= K); a vector straddling K is masked by element.
__device__ __forceinline__ u32x4 load_vec(const bf16_t* __restrict__ base, int64_t ld, int row,
                                          int nrows, int k, int K) {
  u32x4 v = {0u, 0u, 0u, 0u};
  if (row < nrows && k < K) {
    v = *reinterpret_cast<const u32x4*>(base + (int64_t)row * ld + k);
    int valid = K - k;                 // >= 1
    if (valid < 8) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int e = 2 * j;                 // elements e, e+1 live in dword j
        uint32_t keep = (e + 1 < valid) ? 0xffffffffu : (e < valid ? 0x0000ffffu : 0u);
        v[j] &= keep;
      }
    }
  }
  return v;
}

// Workgroup tile BM x BN, waves arranged WGM x WGN, each wave owns (BM/WGM) x (BN/WGN)
// made of 32x32 MFMA tiles.
template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(NT) void gemm_bf16_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                       const bf16_t* __restrict__ B, int64_t ldb,
                                                       int M, int N, int K, Epilogue ep) {
  static_assert(WGM * WGN == 4, "four waves");
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  static_assert(TM >= 1 && TN >= 1 && WTM % 32 == 0 && WTN % 32 == 0, "wave tile");
  constexpr int A_VECS = BM * (BK / 8) / NT;   // 16-byte vectors per thread per stage
  constexpr int B_VECS = BN * (BK / 8) / NT;
  static_assert(A_VECS >= 1 && B_VECS >= 1, "tile too small for 256 threads");

  __shared__ __attribute__((aligned(16))) bf16_t As[BM * LDS_LD];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[BN * LDS_LD];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int vcol = (tid & 7) * 8;    // contraction offset of this thread's vector in a stage
  const int vrow = tid >> 3;         // 0..31

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  u32x4 ra[A_VECS], rb[B_VECS];
  auto load_stage = [&](int k0) {
#pragma unroll
    for (int i = 0; i < A_VECS; ++i) ra[i] = load_vec(A, lda, m0 + vrow + 32 * i, M, k0 + vcol, K);
#pragma unroll
    for (int i = 0; i < B_VECS; ++i) rb[i] = load_vec(B, ldb, n0 + vrow + 32 * i, N, k0 + vcol, K);
  };
  auto store_stage = [&]() {
#pragma unroll
    for (int i = 0; i < A_VECS; ++i)
      *reinterpret_cast<u32x4*>(&As[(vrow + 32 * i) * LDS_LD + vcol]) = ra[i];
#pragma unroll
    for (int i = 0; i < B_VECS; ++i)
      *reinterpret_cast<u32x4*>(&Bs[(vrow + 32 * i) * LDS_LD + vcol]) = rb[i];
  };

  load_stage(0);
  for (int k0 = 0; k0 < K; k0 += BK) {
    store_stage();
    __syncthreads();
    if (k0 + BK < K) load_stage(k0 + BK);    // next stage in flight while this one is used
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      bf16x8 a[TM], b[TN];
      const int koff = kk + (lane >> 5) * 8;
#pragma unroll
      for (int i = 0; i < TM; ++i)
        a[i] = *reinterpret_cast<const bf16x8*>(&As[(wm * WTM + i * 32 + (lane & 31)) * LDS_LD + koff]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        b[j] = *reinterpret_cast<const bf16x8*>(&Bs[(wn * WTN + j * 32 + (lane & 31)) * LDS_LD + koff]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }

  // Epilogue.  Accumulator register r of a lane holds row 8*(r/4) + 4*(lane/32) + r%4 and
  // column lane%32 of its 32x32 tile.
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + wn * WTN + j * 32 + (lane & 31);
      if (n >= N) continue;
      float bias = 0.f;
      if (ep.bias) {
        bias = ep.bias[n];
        if (ep.bias_round_bf16) bias = round_bf16(bias);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * WTM + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (m >= M) continue;
        float addend = bias;
        if (ep.R) addend = fmaf(ep.beta, ep.R[(int64_t)m * ep.ldr + n], bias);
        float v = fmaf(ep.alpha, acc[i][j][r], addend);
        if (ep.c_is_bf16) static_cast<bf16_t*>(ep.C)[(int64_t)m * ep.ldc + n] = f32_to_bf16(v);
        else              static_cast<float*>(ep.C)[(int64_t)m * ep.ldc + n] = v;
      }
    }
  }
}

template <int BM, int BN, int WGM, int WGN>
int launch_cfg(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, int M, int N, int K,
               const Epilogue& ep, hipStream_t s) {
  dim3 grid((N + BN - 1) / BN, (M + BM - 1) / BM);
  gemm_bf16_kernel<BM, BN, WGM, WGN><<<grid, NT, 0, s>>>(A, lda, B, ldb, M, N, K, ep);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

}  // namespace

int launch_gemm_bf16(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, int M, int N,
                     int K, const Epilogue& ep, hipStream_t s) {
  if (M <= 0 || N <= 0 || K <= 0 || !A || !B || !ep.C) return VF_EINVAL;
  if ((lda & 7) || (ldb & 7) || (reinterpret_cast<uintptr_t>(A) & 15) ||
      (reinterpret_cast<uintptr_t>(B) & 15))
    return VF_EINVAL;
  // Tile choice: big tiles when both extents are large; otherwise shrink the tile along
  // the small extent so that the grid still covers the chip.
  if (M <= 32) return launch_cfg<32, 128, 1, 4>(A, lda, B, ldb, M, N, K, ep, s);
  if (M <= 64) return launch_cfg<64, 64, 2, 2>(A, lda, B, ldb, M, N, K, ep, s);
  if (N <= 32) return launch_cfg<128, 32, 4, 1>(A, lda, B, ldb, M, N, K, ep, s);
  int64_t big_tiles = (int64_t)((M + 127) / 128) * ((N + 127) / 128);
  if (big_tiles >= 256) return launch_cfg<128, 128, 2, 2>(A, lda, B, ldb, M, N, K, ep, s);
  return launch_cfg<64, 64, 2, 2>(A, lda, B, ldb, M, N, K, ep, s);
}

}  // namespace vf
