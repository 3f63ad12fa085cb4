// bf16 GEMM on the matrix cores of gfx950:  acc[m,n] = sum_k A[m*lda+k] * B[n*ldb+k]
// (both operands contiguous along the contraction), fp32 accumulation with
// v_mfma_f32_32x32x16_bf16, tiles staged through LDS.  Used for the forward, input-gradient
// and weight-gradient contractions of every Linear layer.
//
// A virtual node has few rows (16..128), so the forward and input-gradient products are
// skinny: one or two row tiles, a long contraction.  To fill 256 compute units the
// contraction is cut into `nsplit` slices (blockIdx.z); slice s writes its partial product
// to slab s of the output ([nsplit][M][ldc]) and the consumer kernel adds the slabs in a
// fixed order, so results do not depend on scheduling.
#include <cstdlib>
#include <cstring>

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
// beyond the matrix (rows >= nrows, k >= kend); a vector straddling kend is masked by element.
__device__ __forceinline__ u32x4 load_vec(const bf16_t* __restrict__ base, int64_t ld, int row,
                                          int nrows, int k, int kend) {
  u32x4 v = {0u, 0u, 0u, 0u};
  if (row < nrows && k < kend) {
    v = *reinterpret_cast<const u32x4*>(base + (int64_t)row * ld + k);
    int valid = kend - k;              // >= 1
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
// made of 32x32 MFMA tiles.  blockIdx.z selects the contraction slice [z*kchunk, (z+1)*kchunk).
template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(NT) void gemm_bf16_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                       const bf16_t* __restrict__ B, int64_t ldb,
                                                       int M, int N, int K, int kchunk,
                                                       int64_t slab_stride, Epilogue ep) {
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
  const int kbeg = blockIdx.z * kchunk;
  const int kend = min(K, kbeg + kchunk);
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
    for (int i = 0; i < A_VECS; ++i) ra[i] = load_vec(A, lda, m0 + vrow + 32 * i, M, k0 + vcol, kend);
#pragma unroll
    for (int i = 0; i < B_VECS; ++i) rb[i] = load_vec(B, ldb, n0 + vrow + 32 * i, N, k0 + vcol, kend);
  };
  auto store_stage = [&]() {
#pragma unroll
    for (int i = 0; i < A_VECS; ++i)
      *reinterpret_cast<u32x4*>(&As[(vrow + 32 * i) * LDS_LD + vcol]) = ra[i];
#pragma unroll
    for (int i = 0; i < B_VECS; ++i)
      *reinterpret_cast<u32x4*>(&Bs[(vrow + 32 * i) * LDS_LD + vcol]) = rb[i];
  };

  load_stage(kbeg);
  for (int k0 = kbeg; k0 < kend; k0 += BK) {
    store_stage();
    __syncthreads();
    if (k0 + BK < kend) load_stage(k0 + BK);    // next stage in flight while this one is used
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
  const bool first_slice = blockIdx.z == 0;
  char* cbase = static_cast<char*>(ep.C) +
                (int64_t)blockIdx.z * slab_stride * (ep.c_is_bf16 ? 2 : 4);
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + wn * WTN + j * 32 + (lane & 31);
      if (n >= N) continue;
      float bias = 0.f;
      if (ep.bias && first_slice) {
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
        if (ep.c_is_bf16) reinterpret_cast<bf16_t*>(cbase)[(int64_t)m * ep.ldc + n] = f32_to_bf16(v);
        else              reinterpret_cast<float*>(cbase)[(int64_t)m * ep.ldc + n] = v;
      }
    }
  }
}

// Short contraction (K <= 2*BK = 128: the weight gradient of a node of up to 128 rows).  The
// cost of such a product is one trip to memory for the operands and the write (or
// read-modify-write) of the output, so everything is issued at once: both stages of operand
// loads and, when the epilogue adds into C (fused fold into the gradient buffer), the old C
// values as well; then one LDS barrier, the MFMAs, and the stores.
template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(NT) void gemm_bf16_shortk_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                              const bf16_t* __restrict__ B, int64_t ldb,
                                                              int M, int N, int K, Epilogue ep) {
  static_assert(WGM * WGN == 4, "four waves");
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int KT = 2 * BK;                  // 128
  constexpr int LD2 = KT + 8;                 // padded LDS row
  constexpr int A_VECS = BM * (KT / 8) / NT;  // 16-byte vectors per thread
  constexpr int B_VECS = BN * (KT / 8) / NT;

  __shared__ __attribute__((aligned(16))) bf16_t As[BM * LD2];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[BN * LD2];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int vcol = (tid & 15) * 8;   // 16 vectors per 128-wide row
  const int vrow = tid >> 4;         // 0..15

  u32x4 ra[A_VECS], rb[B_VECS];
#pragma unroll
  for (int i = 0; i < A_VECS; ++i) ra[i] = load_vec(A, lda, m0 + vrow + 16 * i, M, vcol, K);
#pragma unroll
  for (int i = 0; i < B_VECS; ++i) rb[i] = load_vec(B, ldb, n0 + vrow + 16 * i, N, vcol, K);

  // old C values for a read-modify-write epilogue, requested before anything waits
  float oldc[TM][TN][16];
  if (ep.R) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn * WTN + j * 32 + (lane & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = m0 + wm * WTM + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          oldc[i][j][r] = (m < M && n < N) ? ep.R[(int64_t)m * ep.ldr + n] : 0.f;
        }
      }
  }

#pragma unroll
  for (int i = 0; i < A_VECS; ++i) *reinterpret_cast<u32x4*>(&As[(vrow + 16 * i) * LD2 + vcol]) = ra[i];
#pragma unroll
  for (int i = 0; i < B_VECS; ++i) *reinterpret_cast<u32x4*>(&Bs[(vrow + 16 * i) * LD2 + vcol]) = rb[i];
  __syncthreads();

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  const int ksteps = (K + 15) / 16;            // 16-wide MFMA steps that hold any data
#pragma unroll
  for (int ks = 0; ks < KT / 16; ++ks) {
    if (ks < ksteps) {
      bf16x8 a[TM], b[TN];
      const int koff = ks * 16 + (lane >> 5) * 8;
#pragma unroll
      for (int i = 0; i < TM; ++i)
        a[i] = *reinterpret_cast<const bf16x8*>(&As[(wm * WTM + i * 32 + (lane & 31)) * LD2 + koff]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        b[j] = *reinterpret_cast<const bf16x8*>(&Bs[(wn * WTN + j * 32 + (lane & 31)) * LD2 + koff]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  }

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
        if (ep.R) addend = fmaf(ep.beta, oldc[i][j][r], bias);
        float v = fmaf(ep.alpha, acc[i][j][r], addend);
        if (ep.c_is_bf16) static_cast<bf16_t*>(ep.C)[(int64_t)m * ep.ldc + n] = f32_to_bf16(v);
        else              static_cast<float*>(ep.C)[(int64_t)m * ep.ldc + n] = v;
      }
    }
  }
}

struct Shape {
  const bf16_t* A; int64_t lda; const bf16_t* B; int64_t ldb; int M, N, K, nsplit; int64_t slab;
};

template <int BM, int BN, int WGM, int WGN>
int launch_cfg(const Shape& g, const Epilogue& ep, hipStream_t s) {
  int kchunk = ((g.K + g.nsplit - 1) / g.nsplit + BK - 1) / BK * BK;
  dim3 grid((g.N + BN - 1) / BN, (g.M + BM - 1) / BM, g.nsplit);
  gemm_bf16_kernel<BM, BN, WGM, WGN><<<grid, NT, 0, s>>>(g.A, g.lda, g.B, g.ldb, g.M, g.N, g.K, kchunk,
                                                         g.slab, ep);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

// Tuning aid: VF_GEMM_TILE=<BM>x<BN> forces a tile for every launch that it fits.
int forced_tile() {
  static int cached = -1;
  if (cached < 0) {
    cached = 0;
    const char* e = std::getenv("VF_GEMM_TILE");
    if (e) {
      if (!std::strcmp(e, "128x128")) cached = 1;
      else if (!std::strcmp(e, "128x64")) cached = 2;
      else if (!std::strcmp(e, "64x128")) cached = 3;
      else if (!std::strcmp(e, "64x64")) cached = 4;
      else if (!std::strcmp(e, "32x128")) cached = 5;
      else if (!std::strcmp(e, "128x32")) cached = 6;
    }
  }
  return cached;
}

}  // namespace

// Compute-bound shapes take the big tile; everything else (few rows, or a short contraction
// whose cost is writing the output) does better with many small workgroups in flight.
static bool use_big_tile(int M, int N, int K) { return M >= 1024 && N >= 1024 && K >= 512; }

int gemm_bf16_pick_split(int M, int N, int K) {
  // Measured on the node-sized products (128 x 4096 x 4096 and relatives): about four
  // 64x64 workgroups per compute unit, slices no shorter than 3 LDS stages.
  if (use_big_tile(M, N, K)) return 1;
  int bm = M <= 32 ? 32 : 64;
  int bn = M <= 32 ? 128 : 64;
  int64_t tiles = (int64_t)((M + bm - 1) / bm) * ((N + bn - 1) / bn);
  int split = 1;
  while (tiles * split < 1024 && K / (split * 2) >= 3 * BK && split < 32) split *= 2;
  return split;
}

int launch_gemm_bf16(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, int M, int N,
                     int K, int nsplit, int64_t slab_stride, const Epilogue& ep, hipStream_t s) {
  if (M <= 0 || N <= 0 || K <= 0 || !A || !B || !ep.C || nsplit < 1) return VF_EINVAL;
  if (nsplit > 1 && ep.R) return VF_EINVAL;   // slabs are partial sums: nothing may be added in
  if ((lda & 7) || (ldb & 7) || (reinterpret_cast<uintptr_t>(A) & 15) ||
      (reinterpret_cast<uintptr_t>(B) & 15))
    return VF_EINVAL;
  Shape g{A, lda, B, ldb, M, N, K, nsplit, slab_stride};
  switch (forced_tile()) {
    case 1: return launch_cfg<128, 128, 2, 2>(g, ep, s);
    case 2: return launch_cfg<128, 64, 2, 2>(g, ep, s);
    case 3: return launch_cfg<64, 128, 2, 2>(g, ep, s);
    case 4: return launch_cfg<64, 64, 2, 2>(g, ep, s);
    case 5: return launch_cfg<32, 128, 1, 4>(g, ep, s);
    case 6: return launch_cfg<128, 32, 4, 1>(g, ep, s);
    default: break;
  }
  // short contraction with a read-modify-write epilogue: single-trip kernel (measured faster
  // there; the plain-store case does better with the smaller LDS footprint of the general one)
  if (K <= 2 * BK && nsplit == 1 && ep.R && M > 32 && N > 32) {
    dim3 grid((N + 63) / 64, (M + 63) / 64);
    gemm_bf16_shortk_kernel<64, 64, 2, 2><<<grid, NT, 0, s>>>(A, lda, B, ldb, M, N, K, ep);
    VF_LAUNCH_CHECK();
    return VF_OK;
  }
  if (use_big_tile(M, N, K)) return launch_cfg<128, 128, 2, 2>(g, ep, s);
  if (M <= 32) return launch_cfg<32, 128, 1, 4>(g, ep, s);
  if (N <= 32) return launch_cfg<128, 32, 4, 1>(g, ep, s);
  return launch_cfg<64, 64, 2, 2>(g, ep, s);
}

}  // namespace vf
