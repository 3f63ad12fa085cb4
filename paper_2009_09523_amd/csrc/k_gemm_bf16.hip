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
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <type_traits>

#include "vf_device.h"

namespace vf {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int NT = 256;          // 4 wavefronts
constexpr int BK = 64;           // contraction elements per LDS stage
constexpr int LDS_LD = BK + 8;   // padded row (144 bytes) keeps 16-byte reads conflict-free

// 16-byte global load of 8 consecutive bf16 of row `row` at contraction offset k (a multiple of
// 8), zero beyond the matrix (rows >= nrows, k >= kend); a vector straddling kend is masked by
// element.  The load itself is unconditional, at an address clamped into the matrix (one that an
// in-range call would read), and the selection comes after it: a caller that issues several of
// these before using any has them all in flight.  Requires nrows >= 1, kend >= 1.
__device__ __forceinline__ u32x4 load_vec(const bf16_t* __restrict__ base, int64_t ld, int row,
                                          int nrows, int k, int kend) {
  const int rc = min(row, nrows - 1);
  const int kc = min(k, ((kend - 1) >> 3) << 3);
  u32x4 v = *reinterpret_cast<const u32x4*>(base + (int64_t)rc * ld + kc);
  const int valid = (row < nrows && k < kend) ? kend - k : 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int e = 2 * j;                 // elements e, e+1 live in dword j
    const uint32_t keep = (e + 1 < valid) ? 0xffffffffu : (e < valid ? 0x0000ffffu : 0u);
    v[j] &= keep;
  }
  return v;
}

// Workgroup tile BM x BN, waves arranged WGM x WGN, each wave owns (BM/WGM) x (BN/WGN)
// made of 32x32 MFMA tiles.  blockIdx.z selects the contraction slice [z*kchunk, (z+1)*kchunk).
// Epilogue shared by the kernels that keep the product in MFMA layout: a wavefront's TM x TN
// tiles of 32 x 32 (accumulator register r of a lane holds row 8*(r/4) + 4*(lane/32) + r%4 and
// column lane%32 of its tile), top-left corner (mbase, nbase):
//     C = alpha * acc + (beta * R + bias)
// A wavefront whose tiles lie wholly inside the matrix takes a path without per-element
// branches, so that all its reads of R are in flight together (a weight gradient that adds
// into the gradient buffer would otherwise pay one trip to memory per element).
template <int TM, int TN, bool STREAM = false>
__device__ __forceinline__ void store_tiles(const f32x16 (&acc)[TM][TN], const Epilogue& ep, char* cbase,
                                            bool first_slice, int mbase, int nbase, int M, int N, int lane) {
  const int rowoff = 4 * (lane >> 5);
  const int col = lane & 31;
  if (mbase + TM * 32 <= M && nbase + TN * 32 <= N) {
    float bias[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      bias[j] = 0.f;
      if (ep.bias && first_slice) {
        bias[j] = ep.bias[nbase + j * 32 + col];
        if (ep.bias_round_bf16) bias[j] = round_bf16(bias[j]);
      }
    }
    float add[TM][TN][16];
    if (ep.R) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int m = mbase + i * 32 + 8 * (r >> 2) + rowoff + (r & 3);
            add[i][j][r] = ep.R[(int64_t)m * ep.ldr + nbase + j * 32 + col];
          }
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = mbase + i * 32 + 8 * (r >> 2) + rowoff + (r & 3);
          const int n = nbase + j * 32 + col;
          const float addend = ep.R ? fmaf(ep.beta, add[i][j][r], bias[j]) : bias[j];
          const float v = fmaf(ep.alpha, acc[i][j][r], addend);
          if (ep.c_is_bf16) reinterpret_cast<bf16_t*>(cbase)[(int64_t)m * ep.ldc + n] = f32_to_bf16(v);
          else if (STREAM) __builtin_nontemporal_store(v, &reinterpret_cast<float*>(cbase)[(int64_t)m * ep.ldc + n]);
          else              reinterpret_cast<float*>(cbase)[(int64_t)m * ep.ldc + n] = v;
        }
    return;
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = nbase + j * 32 + col;
      if (n >= N) continue;
      float bias = 0.f;
      if (ep.bias && first_slice) {
        bias = ep.bias[n];
        if (ep.bias_round_bf16) bias = round_bf16(bias);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mbase + i * 32 + 8 * (r >> 2) + rowoff + (r & 3);
        if (m >= M) continue;
        float addend = bias;
        if (ep.R) addend = fmaf(ep.beta, ep.R[(int64_t)m * ep.ldr + n], bias);
        const float v = fmaf(ep.alpha, acc[i][j][r], addend);
        if (ep.c_is_bf16) reinterpret_cast<bf16_t*>(cbase)[(int64_t)m * ep.ldc + n] = f32_to_bf16(v);
        else              reinterpret_cast<float*>(cbase)[(int64_t)m * ep.ldc + n] = v;
      }
    }
  }
}

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
  store_tiles<TM, TN>(acc, ep, cbase, first_slice, m0 + wm * WTM, n0 + wn * WTN, M, N, lane);
}

// ---- software-pipelined variant ---------------------------------------------------------------
// Same tiling as gemm_bf16_kernel, but NS stages of global loads are kept in flight in
// registers.  A virtual node's products are short and memory-latency bound, so the depth of
// this ring is what fills the memory system.  The loads are issued with inline assembly and
// waited for with explicit s_waitcnt vmcnt(n): loads complete in order, so "all but the newest
// n" is exactly "the stage about to be written to LDS has landed".  (The compiler's own wait
// insertion falls back to vmcnt(0) across the loop's control flow, which serialises the ring.)
// Every load uses an in-bounds address (row and contraction offset clamped); what lies outside
// the matrix is zeroed when the stage is written to LDS.  LDS is double buffered: one barrier
// per stage.
__device__ __forceinline__ u32x4 load_vec_async(const bf16_t* p) {
  u32x4 v;
  asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(v) : "v"(p) : "memory");
  return v;
}
template <int N>
__device__ __forceinline__ void wait_loads_but() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// The same wait for loads whose destinations are registers (load_vec_async).  The compiler takes
// the output of the load statement as defined at once, and a statement that only clobbers
// memory orders memory accesses, not register arithmetic: a v_and of the edge masking below was
// scheduled ahead of the bare wait and read its register before the data had landed (rare wrong
// products whenever the contraction length was no multiple of 8 and the operand was not yet in
// a near cache).  So the wait takes the stage's registers as read-write operands: everything
// derived from them depends on the wait itself.
template <int N>
__device__ __forceinline__ void wait_loads_into(u32x4 (&r)[1]) {
  asm volatile("s_waitcnt vmcnt(%1)" : "+v"(r[0]) : "n"(N) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_loads_into(u32x4 (&r)[2]) {
  asm volatile("s_waitcnt vmcnt(%2)" : "+v"(r[0]), "+v"(r[1]) : "n"(N) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_loads_into(u32x4 (&r)[4]) {
  asm volatile("s_waitcnt vmcnt(%4)" : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]) : "n"(N) : "memory");
}

__device__ __forceinline__ u32x4 mask_vec(u32x4 v, bool row_ok, int k, int kend) {
  const int valid = row_ok ? kend - k : 0;
  if (valid >= 8) return v;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int e = 2 * j;
    const uint32_t keep = (e + 1 < valid) ? 0xffffffffu : (e < valid ? 0x0000ffffu : 0u);
    v[j] &= keep;
  }
  return v;
}

template <int BM, int BN, int WGM, int WGN, int NS>
__global__ __launch_bounds__(NT) void gemm_bf16_pipe_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                            const bf16_t* __restrict__ B, int64_t ldb,
                                                            int M, int N, int K, int kchunk,
                                                            int64_t slab_stride, Epilogue ep) {
  static_assert(WGM * WGN == 4, "four waves");
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int A_VECS = BM * (BK / 8) / NT;
  constexpr int B_VECS = BN * (BK / 8) / NT;
  constexpr int VPS = A_VECS + B_VECS;           // loads per thread per stage
  static_assert(NS >= 2 && NS <= 4 && (NS - 1) * VPS < 60, "ring depth");

  __shared__ __attribute__((aligned(16))) bf16_t As[2][BM * LDS_LD];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[2][BN * LDS_LD];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int kbeg = blockIdx.z * kchunk;
  const int kend = min(K, kbeg + kchunk);
  const int nstage = kend > kbeg ? (kend - kbeg + BK - 1) / BK : 0;
  const int vcol = (tid & 7) * 8;
  const int vrow = tid >> 3;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // row base pointers, clamped into the matrix
  const bf16_t* arow[A_VECS];
  const bf16_t* brow[B_VECS];
  bool aok[A_VECS], bok[B_VECS];
#pragma unroll
  for (int i = 0; i < A_VECS; ++i) {
    const int r = m0 + vrow + 32 * i;
    aok[i] = r < M;
    arow[i] = A + (int64_t)min(r, M - 1) * lda;
  }
#pragma unroll
  for (int i = 0; i < B_VECS; ++i) {
    const int r = n0 + vrow + 32 * i;
    bok[i] = r < N;
    brow[i] = B + (int64_t)min(r, N - 1) * ldb;
  }
  const int klast = ((K - 1) / 8) * 8;           // last 16-byte vector that starts inside a row

  u32x4 ra[NS][A_VECS], rb[NS][B_VECS];
  auto issue = [&](int slot, int stage) {
    const int k = min(kbeg + stage * BK + vcol, klast);
#pragma unroll
    for (int i = 0; i < A_VECS; ++i) ra[slot][i] = load_vec_async(arow[i] + k);
#pragma unroll
    for (int i = 0; i < B_VECS; ++i) rb[slot][i] = load_vec_async(brow[i] + k);
  };
  auto to_lds = [&](int slot, int stage, int buf) {
    const int k = kbeg + stage * BK + vcol;
#pragma unroll
    for (int i = 0; i < A_VECS; ++i)
      *reinterpret_cast<u32x4*>(&As[buf][(vrow + 32 * i) * LDS_LD + vcol]) = mask_vec(ra[slot][i], aok[i], k, kend);
#pragma unroll
    for (int i = 0; i < B_VECS; ++i)
      *reinterpret_cast<u32x4*>(&Bs[buf][(vrow + 32 * i) * LDS_LD + vcol]) = mask_vec(rb[slot][i], bok[i], k, kend);
  };
  auto compute = [&](int buf) {
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      bf16x8 a[TM], b[TN];
      const int koff = kk + (lane >> 5) * 8;
#pragma unroll
      for (int i = 0; i < TM; ++i)
        a[i] = *reinterpret_cast<const bf16x8*>(&As[buf][(wm * WTM + i * 32 + (lane & 31)) * LDS_LD + koff]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        b[j] = *reinterpret_cast<const bf16x8*>(&Bs[buf][(wn * WTN + j * 32 + (lane & 31)) * LDS_LD + koff]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  };

  if (nstage > 0) {
    // prologue: the first NS stages (stage indices past the end repeat the last address: their
    // data is never used, they only keep the count of outstanding loads uniform)
#pragma unroll
    for (int s = 0; s < NS; ++s) issue(s, min(s, nstage - 1));
    // outstanding on entry to a stage: stages it .. it+NS-1 (NS of them); stage `it` is the oldest
    auto stage = [&](auto slot_c, int it) {
      constexpr int s = decltype(slot_c)::value;
      wait_loads_into<(NS - 1) * VPS>(ra[s]);
      wait_loads_into<(NS - 1) * VPS>(rb[s]);
      to_lds(s, it, it & 1);
      // refill the slot; past the end this re-reads the last stage's lines (cache hits)
      issue(s, min(it + NS, nstage - 1));
      __syncthreads();
      compute(it & 1);
    };
    // whole rounds of NS stages without a branch inside, then the last stages one inside the
    // other: every path through the ring in the compiled code is one that can be taken
    int base = 0;
    for (; base + NS <= nstage; base += NS) {
      stage(std::integral_constant<int, 0>{}, base);
      stage(std::integral_constant<int, 1>{}, base + 1);
      if constexpr (NS > 2) stage(std::integral_constant<int, 2>{}, base + 2);
      if constexpr (NS > 3) stage(std::integral_constant<int, 3>{}, base + 3);
    }
    if (base < nstage) {
      stage(std::integral_constant<int, 0>{}, base);
      if (base + 1 < nstage) {
        stage(std::integral_constant<int, 1>{}, base + 1);
        if constexpr (NS > 3) {
          if (base + 2 < nstage) stage(std::integral_constant<int, 2>{}, base + 2);
        }
      }
    }
    wait_loads_but<0>();   // drain the padding loads before the registers are reused
    // the destination registers of loads that were still in flight stay allocated up to here
#pragma unroll
    for (int s = 0; s < NS; ++s) {
#pragma unroll
      for (int i = 0; i < A_VECS; ++i) asm volatile("" ::"v"(ra[s][i]));
#pragma unroll
      for (int i = 0; i < B_VECS; ++i) asm volatile("" ::"v"(rb[s][i]));
    }
  }

  const bool first_slice = blockIdx.z == 0;
  char* cbase = static_cast<char*>(ep.C) +
                (int64_t)blockIdx.z * slab_stride * (ep.c_is_bf16 ? 2 : 4);
  store_tiles<TM, TN>(acc, ep, cbase, first_slice, m0 + wm * WTM, n0 + wn * WTN, M, N, lane);
}

// ---- LDS-direct variant -----------------------------------------------------------------------
// Same 64 x 64 tiling, but the operand tiles go from global memory straight into LDS
// (global_load_lds_dwordx4: lane l of a wavefront deposits its 16 bytes at LDS base + 16 l), so a
// stage in flight costs no registers and no LDS-store instructions: a ring of NS stages of
// 16 KB keeps NS-1 stages (48 KB per workgroup at NS = 4) on their way, which is what a
// latency-bound node-sized product needs.  A wavefront instruction fills 8 rows of 128 bytes;
// rows cannot be padded, so the eight 16-byte chunks of a row are stored permuted
// (chunk c of row r at position c ^ f(r), f(r) = (r & 7) ^ ((r >> 3) & 1)): the 16-byte reads of
// the MFMA operands (32 rows, one chunk index) then spread over all banks.  The permutation is
// applied on the global side: a lane fetches the chunk that belongs at its position.
// Requires a contraction that is a whole number of 64-element stages per slice (operand rows
// are clamped into the matrix, their products never stored; nothing is masked).
__device__ __forceinline__ int dl_swizzle(int r) { return (r & 7) ^ ((r >> 3) & 1); }

//
// CONV: the first operand is not stored as a matrix.  Row r = (n*H + h)*W + w of it is the 3x3
// neighbourhood of position (h, w) of a channels-last image stack A[rows, Cin] (Cin a multiple
// of 64): element (r, tap*Cin + c) = A[r + (kh-1)*W + (kw-1), c] for tap = 3 kh + kw inside the
// image, 0 outside.  A 64-element stage lies within one tap, so a lane's 16 bytes of a stage come
// from the shifted row or, outside the image, from a block of zeros (`zeros`, 128 bytes): the
// convolution (stride 1, zero padding 1) as a product without a patch matrix.
struct ConvOperand { int H, W, Cin; const bf16_t* zeros; };

template <int NS, bool CONV = false>
__global__ __launch_bounds__(NT) void gemm_bf16_dl_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                          const bf16_t* __restrict__ B, int64_t ldb,
                                                          int M, int N, int K, int kchunk,
                                                          int64_t slab_stride, Epilogue ep,
                                                          ConvOperand cv = ConvOperand{0, 0, 0, nullptr}) {
  constexpr int TILE = 64 * BK;                 // elements of one operand tile (8 KB)
  constexpr int STAGE = 2 * TILE;
  constexpr int LPS = 4;                        // loads per lane and stage (2 for A, 2 for B)
  static_assert(NS >= 3 && NS <= 6, "ring depth");
  __shared__ __attribute__((aligned(1024))) bf16_t lds[NS * STAGE];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int kbeg = blockIdx.z * kchunk;
  const int kend = min(K, kbeg + kchunk);
  const int nstage = kend > kbeg ? (kend - kbeg) / BK : 0;

  // this lane's source of each of its loads: row (8 rows per wavefront instruction), permuted chunk
  const bf16_t* ga[2];
  const bf16_t* gb[2];
  int ah[2], aw[2];                             // CONV: image position of this lane's rows
  const bf16_t* az[2];                          // CONV: this lane's 16 bytes of the block of zeros
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int row = (wave * 2 + q) * 8 + (lane >> 3);
    const int chunk = (lane & 7) ^ dl_swizzle(row);
    const int r = min(m0 + row, M - 1);
    if (CONV) {
      ga[q] = A + (int64_t)r * cv.Cin + chunk * 8;
      aw[q] = r % cv.W;
      ah[q] = (r / cv.W) % cv.H;
      az[q] = cv.zeros + chunk * 8;
    } else {
      ga[q] = A + (int64_t)r * lda + kbeg + chunk * 8;
      ah[q] = aw[q] = 0; az[q] = nullptr;
    }
    gb[q] = B + (int64_t)min(n0 + row, N - 1) * ldb + kbeg + chunk * 8;
  }
  const int per_tap = CONV ? cv.Cin / BK : 1;   // stages per tap
  auto issue = [&](int stage, int slot) {
    const int k = stage * BK;
    const bf16_t* src[2];
    if (CONV) {
      const int gs = kbeg / BK + stage;         // stage index within the whole contraction
      const int tap = gs / per_tap, c0 = (gs - tap * per_tap) * BK;
      const int kh = tap / 3, kw = tap - 3 * kh;
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int hh = ah[q] + kh - 1, ww = aw[q] + kw - 1;
        const bool inside = hh >= 0 && hh < cv.H && ww >= 0 && ww < cv.W;
        // an inside tap of row r is row r + (kh-1)*W + (kw-1) of the same image
        src[q] = inside ? ga[q] + ((int64_t)(kh - 1) * cv.W + (kw - 1)) * cv.Cin + c0 : az[q];
      }
    } else {
      src[0] = ga[0] + k; src[1] = ga[1] + k;
    }
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(src[q]),
                                       (void __attribute__((address_space(3)))*)&lds[slot * STAGE + (wave * 2 + q) * 512],
                                       16, 0, 0);
      __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(gb[q] + k),
                                       (void __attribute__((address_space(3)))*)&lds[slot * STAGE + TILE + (wave * 2 + q) * 512],
                                       16, 0, 0);
    }
  };

  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  const int arow = wm * 32 + (lane & 31), brow = wn * 32 + (lane & 31);
  const int asw = dl_swizzle(arow), bsw = dl_swizzle(brow);

  if (nstage > 0) {
    // NS-1 stages in flight (indices past the end repeat the last stage into a free slot: never
    // read, they only keep the count of outstanding loads uniform)
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) issue(min(s, nstage - 1), s);
    for (int it = 0; it < nstage; ++it) {
      // loads complete in order: stage `it` has landed when at most NS-2 stages are outstanding
      wait_loads_but<(NS - 2) * LPS>();
      // every wave's part of stage `it` is in LDS, and every wave is done reading stage it-1,
      // whose slot the next loads overwrite.  (A bare barrier: the loop issues no LDS stores, and
      // __syncthreads would wait for ALL outstanding loads.)
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      issue(min(it + NS - 1, nstage - 1), (it + NS - 1) % NS);
      const bf16_t* as = &lds[(it % NS) * STAGE];
      const bf16_t* bs = as + TILE;
#pragma unroll
      for (int kk = 0; kk < BK / 16; ++kk) {
        const int cidx = 2 * kk + (lane >> 5);
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(&as[arow * BK + ((cidx ^ asw) * 8)]);
        const bf16x8 b = *reinterpret_cast<const bf16x8*>(&bs[brow * BK + ((cidx ^ bsw) * 8)]);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
      }
    }
    wait_loads_but<0>();
  }

  char* cbase = static_cast<char*>(ep.C) + (int64_t)blockIdx.z * slab_stride * (ep.c_is_bf16 ? 2 : 4);
  f32x16 tiles[1][1];
  tiles[0][0] = acc;
  store_tiles<1, 1>(tiles, ep, cbase, blockIdx.z == 0, m0 + wm * 32, n0 + wn * 32, M, N, lane);
}

// ---- wide LDS-direct variant: 256 x BN tiles, eight wavefronts ---------------------------------
// For products with at least a few hundred rows (two or more virtual nodes taken as one product,
// the weight gradients of a fold window, the token products of the encoder).  What bounds a
// product here is the volume a compute unit has to pull through its vector memory path per flop,
// (1/BM + 1/BN) operand elements per multiply-add, so the tile is as large as LDS allows:
// 256 x 128 or 256 x 256, one workgroup per compute unit, eight wavefronts as 4 x 2, each owning
// 64 x BN/2 (two per SIMD: one wavefront's LDS reads run beside the other's MFMAs; within a
// wavefront the fragments of MFMA step k+1 are read while the MFMAs of step k run).
// Operand tiles go from global memory straight into LDS in stages of KS contraction elements
// (KS = 64: rows of 128 bytes, eight 16-byte chunks; KS = 32: rows of 64 bytes, four chunks), the
// chunks of a row permuted so that the 16-byte operand reads of 32 consecutive rows spread over
// all banks.  A ring of NS stages: NS-1 stages are on their way while one is consumed, and a
// stage's loads are not issued in one burst but spread over the MFMA steps of the stage before
// (a wavefront never sits on a full memory queue with its matrix work waiting behind it).  What
// matters is how long before its use a stage is requested: 256 x 256 tiles take three stages of 32
// (32 KB each), 256 x 128 tiles three stages of 64 (48 KB each).
// Workgroup numbering: XCD x (workgroup index modulo 8) takes a contiguous run of the tile order
// "eight row tiles down, then one column right", so the 32 tiles that run side by side on one
// XCD form an 8 x 4 block sharing 8 + 4 operand panels on that XCD's L2.
// Requires whole stages in every contraction slice; operand rows are clamped into the matrix
// (their products never stored).
// One LDS-direct load of 16 bytes per lane: global address = scalar base + 32-bit lane offset, LDS
// address (wavefront-uniform; lane l lands 16 l bytes behind it) through M0.  No destination
// register: the data is in LDS when the wavefront's vmcnt says so.
__device__ __forceinline__ void lds_load16(const char* base, uint32_t off, bf16_t* dst) {
  const uint32_t l = (uint32_t)(uintptr_t)(void __attribute__((address_space(3)))*)dst;
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(l), "v"(off), "s"(base) : "memory", "m0");
}

template <int KS>
__device__ __forceinline__ int wide_swizzle(int r) {
  return KS == 64 ? ((r & 7) ^ ((r >> 3) & 1)) : ((r >> 2) & 3);
}

template <int BN, int KS, int NS>
__global__ __launch_bounds__(512) void gemm_bf16_wide_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                             const bf16_t* __restrict__ B, int64_t ldb,
                                                             int M, int N, int K, int kchunk,
                                                             int64_t slab_stride, Epilogue ep, int tiles_m,
                                                             int tiles_n) {
  static_assert(BN == 128 || BN == 256, "tile width");
  static_assert(KS == 64 || KS == 32, "stage depth");
  constexpr int BM = 256;
  constexpr int CPR = KS / 8;                            // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;                          // rows one load instruction of a wavefront fills
  constexpr int ATILE = BM * KS, BTILE = BN * KS;        // elements
  constexpr int STAGE = ATILE + BTILE;
  constexpr int AL = BM / (8 * RPI), BL = BN / (8 * RPI);   // load instructions per lane and stage (8 waves)
  constexpr int LPS = AL + BL;
  constexpr int STEPS = KS / 16;                         // MFMA steps per stage
  constexpr int TN = BN / 64;                            // 32-column MFMA tiles per wavefront (2 row tiles)
  static_assert(NS * STAGE * 2 <= 160 * 1024 && NS >= 2, "LDS");
  extern __shared__ __attribute__((aligned(1024))) bf16_t lds_wide[];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // (in a scalar register)
  const int wm = wave >> 1, wn = wave & 1;
  // this workgroup's tile
  const int ntile = tiles_m * tiles_n;
  const int per = (ntile + 7) >> 3;
  const int local = blockIdx.x >> 3;
  if (local >= per) return;
  const int t = (blockIdx.x & 7) * per + local;
  if (t >= ntile) return;
  const int panel = t / (8 * tiles_n);
  const int in_panel = t - panel * 8 * tiles_n;
  const int prow = min(8, tiles_m - panel * 8);
  const int m0 = (panel * 8 + in_panel % prow) * BM, n0 = (in_panel / prow) * BN;
  const int kbeg = blockIdx.z * kchunk;
  const int kend = min(K, kbeg + kchunk);
  const int nstage = kend > kbeg ? (kend - kbeg) / KS : 0;

  // Addresses are a scalar base (matrix, contraction offset) plus a 32-bit byte offset per lane (row
  // and chunk), and the LDS address of a load goes through M0 from scalar registers: the loop then
  // has no vector arithmetic for its loads.  (The host checks that both operands span less than 2 GiB.)
  uint32_t oa[AL], ob[BL];
#pragma unroll
  for (int q = 0; q < AL; ++q) {
    const int row = (wave + 8 * q) * RPI + lane / CPR;
    oa[q] = (uint32_t)(((int64_t)min(m0 + row, M - 1) * lda + (((lane % CPR) ^ wide_swizzle<KS>(row)) * 8)) * 2);
  }
#pragma unroll
  for (int q = 0; q < BL; ++q) {
    const int row = (wave + 8 * q) * RPI + lane / CPR;
    ob[q] = (uint32_t)(((int64_t)min(n0 + row, N - 1) * ldb + (((lane % CPR) ^ wide_swizzle<KS>(row)) * 8)) * 2);
  }
  const char* Ab = reinterpret_cast<const char*>(A + kbeg);
  const char* Bb = reinterpret_cast<const char*>(B + kbeg);
  // load number j (0 .. LPS-1) of a stage: first the A rows, then the B rows
  auto issue_one = [&](int j, int stage, int slot) {
    const size_t k = (size_t)stage * (KS * 2);
    bf16_t* base = &lds_wide[slot * STAGE];
    if (j < AL) lds_load16(Ab + k, oa[j], base + (wave + 8 * j) * 512);
    else lds_load16(Bb + k, ob[j - AL], base + ATILE + (wave + 8 * (j - AL)) * 512);
  };

  f32x16 acc[2][TN];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  int arow[2], asw[2], brow[TN], bsw[TN];
#pragma unroll
  for (int i = 0; i < 2; ++i) { arow[i] = wm * 64 + i * 32 + (lane & 31); asw[i] = wide_swizzle<KS>(arow[i]); }
#pragma unroll
  for (int j = 0; j < TN; ++j) { brow[j] = wn * (BN / 2) + j * 32 + (lane & 31); bsw[j] = wide_swizzle<KS>(brow[j]); }

  if (nstage > 0) {
    // Schedule.  A step's MFMAs are issued with the step's other instructions between them, one at a
    // time: the two wavefronts of a SIMD run in step (every barrier puts them side by side again), so
    // what a wavefront issues in a block of its own leaves the matrix core idle, while an instruction
    // issued behind an MFMA runs in that MFMA's shadow.  Behind the first MFMAs of a step come the
    // reads of the next step's fragments (in the order that step uses them); the loads of the stage
    // NS-1 ahead follow, half of them in the stage's last step -- there the wavefront first waits
    // for the next stage's loads and meets the others at the barrier, after which every wavefront has
    // read all of the current stage, so that its slot is free -- and the rest over the steps before.
    constexpr int H0 = LPS / 2;                        // loads issued behind the barrier
    constexpr int NM = 2 * TN;                         // MFMAs of a step
    constexpr int NR = 2 + TN;                         // fragment reads of a step
    static_assert(H0 <= NM && (LPS - H0 + STEPS - 2) / (STEPS - 1) <= NM, "a load behind every MFMA at most");
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
#pragma unroll
      for (int j = 0; j < LPS; ++j) issue_one(j, min(s, nstage - 1), s);
    bf16x8 a[2][2], b[2][TN];
    // fragment number r of step kk of a stage, in the order a step uses them: A tile 0, the B tiles, A tile 1
    auto read_one = [&](int stage, int kk, int buf, int r) {
      const bf16_t* as = &lds_wide[(stage % NS) * STAGE];
      const bf16_t* bs = as + ATILE;
      const int cidx = 2 * kk + (lane >> 5);
      if (r == 0 || r == NR - 1) {
        const int i = r ? 1 : 0;
        a[buf][i] = *reinterpret_cast<const bf16x8*>(&as[arow[i] * KS + ((cidx ^ asw[i]) * 8)]);
      } else {
        const int j = r - 1;
        b[buf][j] = *reinterpret_cast<const bf16x8*>(&bs[brow[j] * KS + ((cidx ^ bsw[j]) * 8)]);
      }
    };
    // stage 0 has landed when at most NS-2 stages are outstanding (loads complete in order)
    wait_loads_but<(NS - 2) * LPS>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int r = 0; r < NR; ++r) read_one(0, 0, 0, r);
    // the last ring slot is still empty: stage NS-1 goes there (first half now, second half in the first steps)
#pragma unroll
    for (int j = 0; j < H0; ++j) issue_one(j, min(NS - 1, nstage - 1), NS - 1);
    for (int it = 0; it < nstage; ++it) {
      // the stage whose loads are being issued while stage `it` is consumed, and its slot
      const int cur_ld = min(it + NS - 1, nstage - 1), cur_slot = (it + NS - 1) % NS;
      const int nxt_ld = min(it + NS, nstage - 1), nxt_slot = it % NS;
      const bool more = it + 1 < nstage;
#pragma unroll
      for (int kk = 0; kk < STEPS; ++kk) {
        const int buf = kk & 1;
        const bool last = kk + 1 == STEPS;
        __builtin_amdgcn_sched_barrier(0);
        if (last && more) {
          // this wavefront's own reads of stage `it` have returned (the slot is overwritten behind the
          // barrier), and everything of stage it+1 has landed: outstanding may be the stages it+2 .. it+NS-1
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          wait_loads_but<(NS - 2) * LPS>();
          __builtin_amdgcn_s_barrier();
          asm volatile("" ::: "memory");
        }
        // the loads of this step: [lo, hi) of stage cur_ld, or (last step) the first H0 of stage nxt_ld
        const int lo = last ? 0 : H0 + kk * (LPS - H0) / (STEPS - 1);
        const int hi = last ? H0 : H0 + (kk + 1) * (LPS - H0) / (STEPS - 1);
#pragma unroll
        for (int m = 0; m < NM; ++m) {
          const int i = m / TN, j = m % TN;
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[buf][i], b[buf][j], acc[i][j], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          if (m < NR && (!last || more)) read_one(last ? it + 1 : it, last ? 0 : kk + 1, buf ^ 1, m);
          // loads behind the last MFMAs of the step
          const int l = lo + m - (NM - (hi - lo));
          if (l >= lo && l < hi && (!last || more)) issue_one(l, last ? nxt_ld : cur_ld, last ? nxt_slot : cur_slot);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    wait_loads_but<0>();
  }

  char* cbase = static_cast<char*>(ep.C) + (int64_t)blockIdx.z * slab_stride * (ep.c_is_bf16 ? 2 : 4);
  // one row of 32 x 32 tiles at a time (the addend of a whole wavefront tile would not fit in registers)
  auto store_row = [&](auto ic) {
    constexpr int i = decltype(ic)::value;
    f32x16 row[1][TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) row[0][j] = acc[i][j];
    if (ep.stream_c) store_tiles<1, TN, true>(row, ep, cbase, blockIdx.z == 0, m0 + wm * 64 + i * 32, n0 + wn * (BN / 2), M, N, lane);
    else store_tiles<1, TN>(row, ep, cbase, blockIdx.z == 0, m0 + wm * 64 + i * 32, n0 + wn * (BN / 2), M, N, lane);
  };
  store_row(std::integral_constant<int, 0>{});
  store_row(std::integral_constant<int, 1>{});
}

// ---- the same tile with whole lines in flight for longer ------------------------------------------
// What the ring above cannot give a 256 x 256 tile is time: a load takes about 1.3 us from issue to
// arrival here (the workgroups of an XCD walk along their shared operand panels in step, so almost
// every load instruction holds a line that nobody has fetched yet and waits for HBM), and three
// stages of 32 elements keep 64 KB in flight per compute unit -- 12.5 TB/s over the chip by
// Little's law, which is what the loads of that kernel reach with everything else switched off;
// deeper rings of half lines then meet the L2-to-L1 limit, because every 128-byte line crosses
// twice.  Here a stage is 64 elements (whole lines), and LDS, all 160 KB of it, is cut so that
// every load is issued one and a half to two stages before its first use:
//   A: three slots of 256 rows (32 KB); stage s+2 is requested while stage s is consumed;
//   B: a wavefront works through its four column tiles in two halves (tiles 0, 1 over all four
//      steps of the stage, then tiles 2, 3, its A fragments staying in registers), so the rows of
//      the first half (BF, 128 rows, 16 KB) are free in the middle of the stage and those of the
//      second (BS) are not needed before: two slots each, BF of stage s+2 requested at the middle
//      of stage s, BS of stage s+1 at its start.
// Two barriers per stage (start: A and BF of the stage have landed, A and BS of the one before are
// read; middle: BS has landed, BF is read), loads complete in order, and per wavefront four load
// instructions follow each barrier (two at once, two a phase later), so the waits are fixed counts:
// at most 8 outstanding at the start of a stage, at most 10 at its middle.
__device__ __forceinline__ int line_swizzle(int r) { return (r & 7) ^ ((r >> 3) & 1); }

__global__ __launch_bounds__(512) void gemm_bf16_wide_line_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                                  const bf16_t* __restrict__ B, int64_t ldb,
                                                                  int M, int N, int K, int kchunk,
                                                                  int64_t slab_stride, Epilogue ep, int tiles_m,
                                                                  int tiles_n) {
  constexpr int BM = 256, BN = 256, KS = 64;
  constexpr int AUNIT = BM * KS, BUNIT = (BN / 2) * KS;      // elements: 32 KB, 16 KB
  constexpr int A0 = 0, BF0 = 3 * AUNIT, BS0 = BF0 + 2 * BUNIT;
  static_assert((BS0 + 2 * BUNIT) * 2 == 160 * 1024, "LDS");
  extern __shared__ __attribute__((aligned(1024))) bf16_t lds_wide[];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // (in a scalar register)
  const int wm = wave >> 1, wn = wave & 1;
  const int ntile = tiles_m * tiles_n;
  const int per = (ntile + 7) >> 3;
  const int local = blockIdx.x >> 3;
  if (local >= per) return;
  const int t = (blockIdx.x & 7) * per + local;
  if (t >= ntile) return;
  const int panel = t / (8 * tiles_n);
  const int in_panel = t - panel * 8 * tiles_n;
  const int prow = min(8, tiles_m - panel * 8);
  const int m0 = (panel * 8 + in_panel % prow) * BM, n0 = (in_panel / prow) * BN;
  const int kbeg = blockIdx.z * kchunk;
  const int kend = min(K, kbeg + kchunk);
  const int nstage = kend > kbeg ? (kend - kbeg) / KS : 0;

  // One load instruction of a wavefront: 8 rows of 128 bytes (lane / 8 the row, lane % 8 the chunk).
  // Addresses are a scalar base (matrix, contraction offset) plus a 32-bit byte offset per lane (row
  // and chunk): the stage to stage arithmetic is scalar, and a load reads one address register per
  // lane.  (The host checks that both operands span less than 2 GiB.)
  uint32_t oa[4], obf[2], obs[2];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int row = (wave + 8 * q) * 8 + (lane >> 3);
    oa[q] = (uint32_t)(((int64_t)min(m0 + row, M - 1) * lda + (((lane & 7) ^ line_swizzle(row)) * 8)) * 2);
  }
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int lr = (wave + 8 * q) * 8 + (lane >> 3);          // row within the half unit: 64 rows per column half
    const int trow = (lr >> 6) * (BN / 2) + (lr & 63);
    const int chunk = ((lane & 7) ^ line_swizzle(lr)) * 8;
    obf[q] = (uint32_t)(((int64_t)min(n0 + trow, N - 1) * ldb + chunk) * 2);
    obs[q] = (uint32_t)(((int64_t)min(n0 + trow + 64, N - 1) * ldb + chunk) * 2);
  }
  const char* Ab = reinterpret_cast<const char*>(A + kbeg);
  const char* Bb = reinterpret_cast<const char*>(B + kbeg);
  auto load16 = [&](const char* base, uint32_t off, bf16_t* dst) { lds_load16(base, off, dst); };
  // (a stage past the end repeats the last one: it lands in a free slot and is never read)
  auto issue_a = [&](int q, int stage, int slot) {
    load16(Ab + (size_t)min(stage, nstage - 1) * (KS * 2), oa[q], &lds_wide[A0 + slot * AUNIT + (wave + 8 * q) * 512]);
  };
  auto issue_bf = [&](int q, int stage, int slot) {
    load16(Bb + (size_t)min(stage, nstage - 1) * (KS * 2), obf[q], &lds_wide[BF0 + slot * BUNIT + (wave + 8 * q) * 512]);
  };
  auto issue_bs = [&](int q, int stage, int slot) {
    load16(Bb + (size_t)min(stage, nstage - 1) * (KS * 2), obs[q], &lds_wide[BS0 + slot * BUNIT + (wave + 8 * q) * 512]);
  };

  f32x16 acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  int arow[2], asw[2], brow[2], bsw[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) { arow[i] = wm * 64 + i * 32 + (lane & 31); asw[i] = line_swizzle(arow[i]); }
#pragma unroll
  for (int j = 0; j < 2; ++j) { brow[j] = wn * 64 + j * 32 + (lane & 31); bsw[j] = line_swizzle(brow[j]); }

  if (nstage > 0) {
    // prologue, in the order the steady state would have issued them
#pragma unroll
    for (int q = 0; q < 4; ++q) issue_a(q, 0, 0);
#pragma unroll
    for (int q = 0; q < 2; ++q) issue_bf(q, 0, 0);
#pragma unroll
    for (int q = 0; q < 2; ++q) issue_bs(q, 0, 0);
#pragma unroll
    for (int q = 0; q < 4; ++q) issue_a(q, 1, 1);
#pragma unroll
    for (int q = 0; q < 2; ++q) issue_bf(q, 1, 1);

    bf16x8 a[4][2], b[2][2];
    auto read_a = [&](int slot, int kk) {
      const bf16_t* as = &lds_wide[A0 + slot * AUNIT];
      const int cidx = 2 * kk + (lane >> 5);
#pragma unroll
      for (int i = 0; i < 2; ++i) a[kk][i] = *reinterpret_cast<const bf16x8*>(&as[arow[i] * KS + ((cidx ^ asw[i]) * 8)]);
    };
    auto read_b = [&](const bf16_t* bs, int kk, int buf) {
      const int cidx = 2 * kk + (lane >> 5);
#pragma unroll
      for (int j = 0; j < 2; ++j) b[buf][j] = *reinterpret_cast<const bf16x8*>(&bs[brow[j] * KS + ((cidx ^ bsw[j]) * 8)]);
    };
    wait_loads_but<8>();                   // A and BF of stage 0
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    read_a(0, 0);
    read_b(&lds_wide[BF0], 0, 0);
#pragma unroll
    for (int q = 0; q < 2; ++q) issue_bs(q, 1, 1);

    // One fragment read: A row tile i or B column tile j of MFMA step kk.
    auto rd_a = [&](int slot, int kk, int i) {
      const bf16_t* as = &lds_wide[A0 + slot * AUNIT];
      a[kk][i] = *reinterpret_cast<const bf16x8*>(&as[arow[i] * KS + (((2 * kk + (lane >> 5)) ^ asw[i]) * 8)]);
    };
    auto rd_b = [&](const bf16_t* bs, int kk, int buf, int j) {
      b[buf][j] = *reinterpret_cast<const bf16x8*>(&bs[brow[j] * KS + (((2 * kk + (lane >> 5)) ^ bsw[j]) * 8)]);
    };

    int sa = 0, sb = 0;                    // stage % 3, stage % 2
    for (int s = 0; s < nstage; ++s) {
      const int sa1 = sa == 2 ? 0 : sa + 1, sa2 = sa == 0 ? 2 : sa - 1;    // (s+1) % 3, (s+2) % 3
      const bf16_t* bf = &lds_wide[BF0 + sb * BUNIT];
      const bf16_t* bs = &lds_wide[BS0 + sb * BUNIT];
      const bf16_t* bfn = &lds_wide[BF0 + (sb ^ 1) * BUNIT];
      const bool more = s + 1 < nstage;
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        const int h = p >> 2, kk = p & 3;
        __builtin_amdgcn_sched_barrier(0);
        if (p == 3) {
          // middle of the stage: BS of this stage has landed, and behind the barrier BF is read by all
          // (this wavefront's own reads have returned)
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          wait_loads_but<10>();
          __builtin_amdgcn_s_barrier();
          asm volatile("" ::: "memory");
        } else if (p == 7 && more) {
          // start of the next stage: its A and BF have landed; A and BS of this one are read by all
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          wait_loads_but<8>();
          __builtin_amdgcn_s_barrier();
          asm volatile("" ::: "memory");
        }
        // The phase's four MFMAs with its other instructions between them, one at a time: the two
        // wavefronts of a SIMD run in step (every barrier puts them side by side again), so what a
        // wavefront issues in a block of its own leaves the matrix core idle, while an instruction
        // issued behind an MFMA runs in that MFMA's shadow.
        //   slot 0, 1: fragments of the next phase (A of step kk+1 in the first half; at a barrier:
        //              of the unit that has just landed);  slot 2, 3: its B fragments and the loads
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          const int i = m >> 1, j = m & 1;
          acc[i][2 * h + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk][i], b[p & 1][j], acc[i][2 * h + j], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          // (fragments in the order the next phase uses them: A tile 0, B tile 0, B tile 1, A tile 1)
          if (p == 3) {
            if (m < 2) rd_b(bs, 0, 0, m);
            else issue_bf(m - 2, s + 2, sb);
          } else if (p == 7) {
            if (more) {
              if (m == 0) rd_a(sa1, 0, 0);
              if (m == 1) rd_b(bfn, 0, 0, 0);
              if (m == 2) { rd_b(bfn, 0, 0, 1); issue_bs(0, s + 2, sb); }
              if (m == 3) { rd_a(sa1, 0, 1); issue_bs(1, s + 2, sb); }
            }
          } else {
            if (h == 0) {
              if (m == 0) rd_a(sa, kk + 1, 0);
              if (m == 1) rd_b(bf, kk + 1, (p + 1) & 1, 0);
              if (m == 2) rd_b(bf, kk + 1, (p + 1) & 1, 1);
              if (m == 3) rd_a(sa, kk + 1, 1);
            } else {
              if (m < 2) rd_b(bs, kk + 1, (p + 1) & 1, m);
            }
            if (p == 0 && m >= 2) issue_a(m - 2, s + 2, sa2);
            if (p == 4 && m >= 2) issue_a(m, s + 2, sa2);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      sa = sa1;
      sb ^= 1;
    }
    wait_loads_but<0>();
  }

  char* cbase = static_cast<char*>(ep.C) + (int64_t)blockIdx.z * slab_stride * (ep.c_is_bf16 ? 2 : 4);
  auto store_row = [&](auto ic) {
    constexpr int i = decltype(ic)::value;
    f32x16 row[1][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) row[0][j] = acc[i][j];
    if (ep.stream_c) store_tiles<1, 4, true>(row, ep, cbase, blockIdx.z == 0, m0 + wm * 64 + i * 32, n0 + wn * (BN / 2), M, N, lane);
    else store_tiles<1, 4>(row, ep, cbase, blockIdx.z == 0, m0 + wm * 64 + i * 32, n0 + wn * (BN / 2), M, N, lane);
  };
  store_row(std::integral_constant<int, 0>{});
  store_row(std::integral_constant<int, 1>{});
}

// ---- the whole-line kernel on the 16x16x32 instruction ------------------------------------------
// Same tile, same LDS plan, same loads and waits as gemm_bf16_wide_line_kernel.  The chip lowers
// its clock under these products, and per flop the 16x16x32 MFMA draws less than 32x32x16 (a
// register-only loop on random operands: 2.0 against 1.7 PFLOP/s), so on normally distributed
// operands this form is the faster one.  A wavefront's 64 x 128 tile is 4 x 8 tiles of 16 x 16;
// a stage of 64 elements is two MFMA steps of 32; the halves of B are column tiles 0-3 and 4-7:
// four phases (half, step) of 16 MFMAs per stage, the A fragments of both steps (8) staying in
// registers for the second half.  A fragment of 16 rows x 32 elements is one 16-byte read per lane
// (lane % 16 the row, lane / 16 the 16-byte chunk), and the products are taken as B-tile x A-tile,
// so that a lane ends up with four CONSECUTIVE columns of one row of C (row lane % 16 of the tile,
// columns 4 (lane / 16) ..): the epilogue stores 16 bytes per lane.
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Chunk permutation of this kernel's LDS rows.  A 16-byte fragment read of 16 rows x 4 chunks (lane % 16
// the row, lane / 16 the chunk) takes 4 cycles when no two of the 16 lanes served together meet on a
// bank, and a probe that timed such reads under every linear map from the row's low four bits to the
// chunk position measured: unpermuted 16 cycles, line_swizzle 8 (half of this kernel's LDS cycles were
// bank conflicts by the counters), and 4 for the maps that send bits 0-2 or bits 1-3 of the row to the
// three position bits one to one.  The first of those:
__device__ __forceinline__ int line16_swizzle(int r) { return r & 7; }

// Epilogue of one row of 16 x 16 tiles (tile row i of the wavefront: 16 rows, 8 x 16 columns).
template <bool STREAM>
__device__ __forceinline__ void store_tiles16_row(const f32x4 (&acc)[8], const Epilogue& ep, char* cbase, bool first_slice,
                                                  int mbase, int nbase, int M, int N, int lane) {
  const int m = mbase + (lane & 15);
  const int nq = 4 * (lane >> 4);
  float* C = reinterpret_cast<float*>(cbase);
  const bool vec = !ep.c_is_bf16 && mbase + 16 <= M && nbase + 128 <= N && (ep.ldc & 3) == 0 &&
                   (reinterpret_cast<uintptr_t>(cbase) & 15) == 0 &&
                   (!ep.R || ((ep.ldr & 3) == 0 && (reinterpret_cast<uintptr_t>(ep.R) & 15) == 0)) &&
                   (!ep.bias || (reinterpret_cast<uintptr_t>(ep.bias) & 15) == 0);
  if (vec) {
    f32x4 add[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      f32x4 bias = {0.f, 0.f, 0.f, 0.f};
      if (ep.bias && first_slice) {
        bias = *reinterpret_cast<const f32x4*>(&ep.bias[nbase + 16 * j + nq]);
        if (ep.bias_round_bf16)
#pragma unroll
          for (int e = 0; e < 4; ++e) bias[e] = round_bf16(bias[e]);
      }
      add[j] = bias;
    }
    if (ep.R) {
      f32x4 r[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) r[j] = *reinterpret_cast<const f32x4*>(&ep.R[(int64_t)m * ep.ldr + nbase + 16 * j + nq]);
#pragma unroll
      for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) add[j][e] = fmaf(ep.beta, r[j][e], add[j][e]);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      f32x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = fmaf(ep.alpha, acc[j][e], add[j][e]);
      f32x4* dst = reinterpret_cast<f32x4*>(&C[(int64_t)m * ep.ldc + nbase + 16 * j + nq]);
      if (STREAM) __builtin_nontemporal_store(v, dst);
      else *dst = v;
    }
    return;
  }
  if (m >= M) return;
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int n = nbase + 16 * j + nq + e;
      if (n >= N) continue;
      float addend = 0.f;
      if (ep.bias && first_slice) {
        addend = ep.bias[n];
        if (ep.bias_round_bf16) addend = round_bf16(addend);
      }
      if (ep.R) addend = fmaf(ep.beta, ep.R[(int64_t)m * ep.ldr + n], addend);
      const float v = fmaf(ep.alpha, acc[j][e], addend);
      if (ep.c_is_bf16) reinterpret_cast<bf16_t*>(cbase)[(int64_t)m * ep.ldc + n] = f32_to_bf16(v);
      else C[(int64_t)m * ep.ldc + n] = v;
    }
}

// BatchNorm + ReLU backward of a finished 256 x 256 tile of the incoming gradient, in place of
// storing it (Section 4.1: statistics per virtual node; here a tile's rows are two whole nodes of
// 128, wavefronts wm = 0, 1 on the first and 2, 3 on the second).  With dr = the gradient where the
// layer's output was positive, xhat = (z - mean) rstd:
//   dz = gamma rstd (dr - sum(dr) / 128 - xhat sum(dr xhat) / 128)        (dz = dr without BatchNorm),
// the sums over the node's rows: four rows per lane, 16 lanes by exchange, the node's two wavefronts
// through LDS (the lower rows first), one group of 16 columns at a time.  A lane holds four consecutive columns of a row, so dz leaves in
// 8-byte stores; the transposed copy goes through LDS (per wavefront 128 columns x 64 rows) and
// leaves in 16-byte stores of eight rows.  LDS: the sums at 0 (8 KB), the transposed tiles behind.
// Sum over the 16 lanes of a row (lanes 16 k .. 16 k + 15), to all of them, by data-parallel-primitive
// moves: neighbours, pairs, the quad's mirror image in its half row, the half row's in the row.  Both
// partners of an exchange add the same two values, so every lane ends with the same bits.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_move<0xB1>(v);    // quad_perm [1, 0, 3, 2]
  v += dpp_move<0x4E>(v);    // quad_perm [2, 3, 0, 1]
  v += dpp_move<0x141>(v);   // row_half_mirror
  v += dpp_move<0x140>(v);   // row_mirror
  return v;
}

constexpr int kFuseTPitch = 72;   // bf16 elements per column of a wavefront's transposed tile (64 rows + 8)
__device__ __forceinline__ void bn_bwd_tile(f32x4 (&acc)[4][8], const BnBwdArgs& fa, bf16_t* lds, int m0, int n0, int N,
                                            int wave, int lane) {
  const int wm = wave >> 1, wn = wave & 1;
  const int lq = lane >> 4, lr = lane & 15;
  const int node = (m0 + wm * 64) >> 7;
  const int colw = n0 + wn * 128;                      // the wavefront's first column
  const int row0 = m0 + wm * 64;                       // ... and first row
  const bool bn = fa.gamma != nullptr;
  const bool same = fa.tscale == 1.f;
  const float invR = 1.0f / 128.0f;
  float* part = reinterpret_cast<float*>(lds);         // [wave][2][128]
  bf16_t* tT = lds + 4096 + wave * (128 * kFuseTPitch);

  // every wavefront is done with the operand stages before the sums and tiles overwrite them
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");

  auto params = [&](int c, f32x4& mean, f32x4& rstd, f32x4& g, f32x4& b) {
    mean = f32x4{0.f, 0.f, 0.f, 0.f}; rstd = f32x4{1.f, 1.f, 1.f, 1.f};
    g = f32x4{1.f, 1.f, 1.f, 1.f}; b = f32x4{0.f, 0.f, 0.f, 0.f};
    if (bn) {
      mean = *reinterpret_cast<const f32x4*>(&fa.mean[(int64_t)node * N + c]);
      rstd = *reinterpret_cast<const f32x4*>(&fa.rstd[(int64_t)node * N + c]);
      g = *reinterpret_cast<const f32x4*>(&fa.gamma[c]);
      b = *reinterpret_cast<const f32x4*>(&fa.beta[c]);
      if (fa.round_params)
#pragma unroll
        for (int e = 0; e < 4; ++e) { g[e] = round_bf16(g[e]); b[e] = round_bf16(b[e]); }
    }
  };

  // Column group j (16 columns; 4 per lane) at a time: the layer's pre-activations of group j + 1 are
  // requested before group j is worked on, so that they are read once and a trip to memory is hidden
  // behind the group before; mask by the layer's output, sums of this wavefront's 64 rows, exchange
  // with the node's other wavefront (the lower rows first), dz and the transposed tile.
  const int w0 = (wm & ~1) * 2 + wn, w1 = w0 + 2;
  auto load_z = [&](int j, f32x4 (&zz)[4]) {
    const int c = colw + 16 * j + 4 * lq;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      zz[i] = *reinterpret_cast<const f32x4*>(&fa.z[(int64_t)(row0 + 16 * i + lr) * fa.ldz + c]);   // (half a line: the
  };                                                     // next group asks for the other half, so no streaming hint)
  uint2 held[4][4];
  f32x4 znext[4], mean_n, rstd_n, g_n, b_n;
  load_z(0, znext);
  params(colw + 4 * lq, mean_n, rstd_n, g_n, b_n);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int c = colw + 16 * j + 4 * lq;
    const int pc = 16 * j + 4 * lq;
    f32x4 zz[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) zz[i] = znext[i];
    const f32x4 mean = mean_n, rstd = rstd_n, g = g_n, b = b_n;
    if (j + 1 < 8) {
      load_z(j + 1, znext);
      params(c + 16, mean_n, rstd_n, g_n, b_n);
    }
    f32x4 sg = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float xhat = (zz[i][e] - mean[e]) * rstd[e];
        const float pre = bn ? fmaf(g[e], xhat, b[e]) : zz[i][e];
        const float dr = pre > 0.f ? acc[i][j][e] : 0.f;
        acc[i][j][e] = dr;
        zz[i][e] = xhat;
        sg[e] = fmaf(dr, xhat, sg[e]);
        sb[e] += dr;
      }
#pragma unroll
    for (int e = 0; e < 4; ++e) { sg[e] = row16_sum(sg[e]); sb[e] = row16_sum(sb[e]); }
    if (lr == 0) {
      *reinterpret_cast<f32x4*>(&part[(wave * 2 + 0) * 128 + pc]) = sg;
      *reinterpret_cast<f32x4*>(&part[(wave * 2 + 1) * 128 + pc]) = sb;
    }
    __syncthreads();
    const f32x4 sg0 = *reinterpret_cast<const f32x4*>(&part[(w0 * 2 + 0) * 128 + pc]);
    const f32x4 sg1 = *reinterpret_cast<const f32x4*>(&part[(w1 * 2 + 0) * 128 + pc]);
    const f32x4 sb0 = *reinterpret_cast<const f32x4*>(&part[(w0 * 2 + 1) * 128 + pc]);
    const f32x4 sb1 = *reinterpret_cast<const f32x4*>(&part[(w1 * 2 + 1) * 128 + pc]);
#pragma unroll
    for (int e = 0; e < 4; ++e) { sg[e] = sg0[e] + sg1[e]; sb[e] = sb0[e] + sb1[e]; }
    if (!(wm & 1) && lr == 0) {
      *reinterpret_cast<f32x4*>(&fa.sums[((int64_t)node * 2 + 0) * N + c]) = sg;
      *reinterpret_cast<f32x4*>(&fa.sums[((int64_t)node * 2 + 1) * N + c]) = sb;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float dr = acc[i][j][e];
        if (bn) {
          const float kk = g[e] * rstd[e];
          v[e] = kk * (dr - sb[e] * invR - zz[i][e] * sg[e] * invR);
        } else {
          v[e] = dr;
        }
      }
      uint2 pk;
      pk.x = f32x2_to_bf16x2(v[0], v[1]);
      pk.y = f32x2_to_bf16x2(v[2], v[3]);
      held[j & 3][i] = pk;
      uint2 pt = pk;                      // the transposed copy's values: the same where the scale is 1
      if (!same) { pt.x = f32x2_to_bf16x2(v[0] * fa.tscale, v[1] * fa.tscale); pt.y = f32x2_to_bf16x2(v[2] * fa.tscale, v[3] * fa.tscale); }
      bf16_t* tp = &tT[pc * kFuseTPitch + 16 * i + lr];
      tp[0] = (bf16_t)pt.x; tp[kFuseTPitch] = (bf16_t)(pt.x >> 16);
      tp[2 * kFuseTPitch] = (bf16_t)pt.y; tp[3 * kFuseTPitch] = (bf16_t)(pt.y >> 16);
    }
    // dz leaves four groups at a time, the four 32-byte parts of a row's 128-byte line one behind the
    // other (stored group by group as they are finished, a line's parts reached the memory apart:
    // 1.3 times the bytes written by the counters)
    if ((j & 3) == 3) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
          *reinterpret_cast<uint2*>(&fa.dz[(int64_t)(row0 + 16 * i + lr) * fa.lddz + colw + 16 * (j - 3 + jj) + 4 * lq]) = held[jj][i];
    }
  }
  __syncthreads();
  // the wavefront's transposed tile: 8 columns per instruction, 8 lanes x 8 rows each
#pragma unroll
  for (int it = 0; it < 16; ++it) {
    const int col = it * 8 + (lane >> 3), seg = lane & 7;
    const u32x4 v = *reinterpret_cast<const u32x4*>(&tT[col * kFuseTPitch + seg * 8]);
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(&fa.dzT[(int64_t)(colw + col) * fa.ldt + row0 + seg * 8]));
  }
}

// BatchNorm + ReLU forward of a finished 256 x 256 tile of pre-activations (two whole nodes of 128
// rows, as in bn_bwd_tile): per group of 16 columns the node's mean (sum over its rows), then the
// sum of squared deviations from it, each exchanged between the node's two wavefronts through LDS
// (slots 0 and 1 of the sums), then a = max(gamma (z - mean) rstd + beta, 0) -- without BatchNorm
// a = max(z, 0), z including the layer's bias.  z is stored two groups at a time (a row's 128-byte
// line), a four groups at a time, the transposed copy through LDS.
__device__ __forceinline__ void bn_fwd_tile(f32x4 (&acc)[4][8], const BnFwdArgs& fa, bf16_t* lds, int m0, int n0, int N,
                                            int wave, int lane) {
  const int wm = wave >> 1, wn = wave & 1;
  const int lq = lane >> 4, lr = lane & 15;
  const int node = (m0 + wm * 64) >> 7;
  const int colw = n0 + wn * 128;
  const int row0 = m0 + wm * 64;
  const bool bn = fa.gamma != nullptr;
  const float invR = 1.0f / 128.0f;
  float* part = reinterpret_cast<float*>(lds);         // [wave][2][128]
  bf16_t* tT = lds + 4096 + wave * (128 * kFuseTPitch);
  const int w0 = (wm & ~1) * 2 + wn, w1 = w0 + 2;

  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");

  uint2 held[4][4];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int c = colw + 16 * j + 4 * lq;
    const int pc = 16 * j + 4 * lq;
    f32x4 g = {1.f, 1.f, 1.f, 1.f}, b = {0.f, 0.f, 0.f, 0.f};
    if (bn) {
      g = *reinterpret_cast<const f32x4*>(&fa.gamma[c]);
      b = *reinterpret_cast<const f32x4*>(&fa.beta[c]);
      if (fa.round_params)
#pragma unroll
        for (int e = 0; e < 4; ++e) { g[e] = round_bf16(g[e]); b[e] = round_bf16(b[e]); }
    } else if (fa.bias) {
      f32x4 bias = *reinterpret_cast<const f32x4*>(&fa.bias[c]);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float bb = fa.round_params ? round_bf16(bias[e]) : bias[e];
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i][j][e] = fmaf(1.f, acc[i][j][e], bb);   // (the product epilogue's own form)
      }
    }
    f32x4 mean = {0.f, 0.f, 0.f, 0.f}, rstd = {1.f, 1.f, 1.f, 1.f};
    if (bn) {
      f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) s[e] += acc[i][j][e];
#pragma unroll
      for (int e = 0; e < 4; ++e) s[e] = row16_sum(s[e]);
      if (lr == 0) *reinterpret_cast<f32x4*>(&part[(wave * 2 + 0) * 128 + pc]) = s;
      __syncthreads();
      {
        const f32x4 s0 = *reinterpret_cast<const f32x4*>(&part[(w0 * 2 + 0) * 128 + pc]);
        const f32x4 s1 = *reinterpret_cast<const f32x4*>(&part[(w1 * 2 + 0) * 128 + pc]);
#pragma unroll
        for (int e = 0; e < 4; ++e) mean[e] = (s0[e] + s1[e]) * invR;
      }
      f32x4 q = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float d = acc[i][j][e] - mean[e];
          q[e] = fmaf(d, d, q[e]);
        }
#pragma unroll
      for (int e = 0; e < 4; ++e) q[e] = row16_sum(q[e]);
      if (lr == 0) *reinterpret_cast<f32x4*>(&part[(wave * 2 + 1) * 128 + pc]) = q;
      __syncthreads();
      f32x4 var;
      {
        const f32x4 q0 = *reinterpret_cast<const f32x4*>(&part[(w0 * 2 + 1) * 128 + pc]);
        const f32x4 q1 = *reinterpret_cast<const f32x4*>(&part[(w1 * 2 + 1) * 128 + pc]);
#pragma unroll
        for (int e = 0; e < 4; ++e) { var[e] = (q0[e] + q1[e]) * invR; rstd[e] = 1.0f / sqrtf(var[e] + fa.eps); }
      }
      if (!(wm & 1) && lr == 0) {
        *reinterpret_cast<f32x4*>(&fa.mean[(int64_t)node * N + c]) = mean;
        *reinterpret_cast<f32x4*>(&fa.rstd[(int64_t)node * N + c]) = rstd;
        *reinterpret_cast<f32x4*>(&fa.var[(int64_t)node * N + c]) = var;
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float zz = acc[i][j][e];
        v[e] = bn ? fmaxf(fmaf(g[e], (zz - mean[e]) * rstd[e], b[e]), 0.f) : fmaxf(zz, 0.f);
      }
      uint2 pk;
      pk.x = f32x2_to_bf16x2(v[0], v[1]);
      pk.y = f32x2_to_bf16x2(v[2], v[3]);
      held[j & 3][i] = pk;
      bf16_t* tp = &tT[pc * kFuseTPitch + 16 * i + lr];
      tp[0] = (bf16_t)pk.x; tp[kFuseTPitch] = (bf16_t)(pk.x >> 16);
      tp[2 * kFuseTPitch] = (bf16_t)pk.y; tp[3 * kFuseTPitch] = (bf16_t)(pk.y >> 16);
    }
    if (j & 1) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
          *reinterpret_cast<f32x4*>(&fa.z[(int64_t)(row0 + 16 * i + lr) * fa.ldz + colw + 16 * (j - 1 + jj) + 4 * lq]) = acc[i][j - 1 + jj];
    }
    if ((j & 3) == 3) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
          *reinterpret_cast<uint2*>(&fa.a[(int64_t)(row0 + 16 * i + lr) * fa.lda + colw + 16 * (j - 3 + jj) + 4 * lq]) = held[jj][i];
    }
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < 16; ++it) {
    const int col = it * 8 + (lane >> 3), seg = lane & 7;
    const u32x4 v = *reinterpret_cast<const u32x4*>(&tT[col * kFuseTPitch + seg * 8]);
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(&fa.aT[(int64_t)(colw + col) * fa.ldt + row0 + seg * 8]));
  }
}

// FUSE = 1: the tile is finished by bn_bwd_tile instead of being stored, FUSE = 2: by bn_fwd_tile (whole tiles only: M and N are
// multiples of 256, one slice).
template <int FUSE>
__global__ __launch_bounds__(512) void gemm_bf16_wide_line16_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                                    const bf16_t* __restrict__ B, int64_t ldb,
                                                                    int M, int N, int K, int kchunk,
                                                                    int64_t slab_stride, Epilogue ep, int tiles_m,
                                                                    int tiles_n, BnBwdArgs fa, BnFwdArgs ff) {
  constexpr int BM = 256, BN = 256, KS = 64;
  constexpr int AUNIT = BM * KS, BUNIT = (BN / 2) * KS;      // elements: 32 KB, 16 KB
  constexpr int A0 = 0, BF0 = 3 * AUNIT, BS0 = BF0 + 2 * BUNIT;
  static_assert((BS0 + 2 * BUNIT) * 2 == 160 * 1024, "LDS");
  extern __shared__ __attribute__((aligned(1024))) bf16_t lds_wide[];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // (in a scalar register)
  const int wm = wave >> 1, wn = wave & 1;
  const int ntile = tiles_m * tiles_n;
  const int per = (ntile + 7) >> 3;
  const int local = blockIdx.x >> 3;
  if (local >= per) return;
  const int t = (blockIdx.x & 7) * per + local;
  if (t >= ntile) return;
  const int panel = t / (8 * tiles_n);
  const int in_panel = t - panel * 8 * tiles_n;
  const int prow = min(8, tiles_m - panel * 8);
  const int m0 = (panel * 8 + in_panel % prow) * BM, n0 = (in_panel / prow) * BN;
  const int kbeg = blockIdx.z * kchunk;
  const int kend = min(K, kbeg + kchunk);
  const int nstage = kend > kbeg ? (kend - kbeg) / KS : 0;

  // loads: exactly those of gemm_bf16_wide_line_kernel
  uint32_t oa[4], obf[2], obs[2];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int row = (wave + 8 * q) * 8 + (lane >> 3);
    oa[q] = (uint32_t)(((int64_t)min(m0 + row, M - 1) * lda + (((lane & 7) ^ line16_swizzle(row)) * 8)) * 2);
  }
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int lr = (wave + 8 * q) * 8 + (lane >> 3);
    const int trow = (lr >> 6) * (BN / 2) + (lr & 63);
    const int chunk = ((lane & 7) ^ line16_swizzle(lr)) * 8;
    obf[q] = (uint32_t)(((int64_t)min(n0 + trow, N - 1) * ldb + chunk) * 2);
    obs[q] = (uint32_t)(((int64_t)min(n0 + trow + 64, N - 1) * ldb + chunk) * 2);
  }
  const char* Ab = reinterpret_cast<const char*>(A + kbeg);
  const char* Bb = reinterpret_cast<const char*>(B + kbeg);
  auto issue_a = [&](int q, int stage, int slot) {
    lds_load16(Ab + (size_t)min(stage, nstage - 1) * (KS * 2), oa[q], &lds_wide[A0 + slot * AUNIT + (wave + 8 * q) * 512]);
  };
  auto issue_bf = [&](int q, int stage, int slot) {
    lds_load16(Bb + (size_t)min(stage, nstage - 1) * (KS * 2), obf[q], &lds_wide[BF0 + slot * BUNIT + (wave + 8 * q) * 512]);
  };
  auto issue_bs = [&](int q, int stage, int slot) {
    lds_load16(Bb + (size_t)min(stage, nstage - 1) * (KS * 2), obs[q], &lds_wide[BS0 + slot * BUNIT + (wave + 8 * q) * 512]);
  };

  f32x4 acc[4][8];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // fragment rows of tile 0 (tile i is 16 rows = 2 KB further: the chunk permutation repeats every 16 rows)
  const int ar = wm * 64 + (lane & 15), br = wn * 64 + (lane & 15);
  const int asw = line16_swizzle(ar), bsw = line16_swizzle(br);

  if (nstage > 0) {
#pragma unroll
    for (int q = 0; q < 4; ++q) issue_a(q, 0, 0);
#pragma unroll
    for (int q = 0; q < 2; ++q) issue_bf(q, 0, 0);
#pragma unroll
    for (int q = 0; q < 2; ++q) issue_bs(q, 0, 0);
#pragma unroll
    for (int q = 0; q < 4; ++q) issue_a(q, 1, 1);
#pragma unroll
    for (int q = 0; q < 2; ++q) issue_bf(q, 1, 1);

    bf16x8 a[2][4], b[2][4];
    auto rd_a = [&](int slot, int ks, int i) {
      const bf16_t* as = &lds_wide[A0 + slot * AUNIT];
      a[ks][i] = *reinterpret_cast<const bf16x8*>(&as[(ar + 16 * i) * KS + (((4 * ks + (lane >> 4)) ^ asw) * 8)]);
    };
    auto rd_b = [&](const bf16_t* bs, int ks, int buf, int j) {
      b[buf][j] = *reinterpret_cast<const bf16x8*>(&bs[(br + 16 * j) * KS + (((4 * ks + (lane >> 4)) ^ bsw) * 8)]);
    };

    wait_loads_but<8>();                   // A and BF of stage 0
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int i = 0; i < 4; ++i) rd_a(0, 0, i);
#pragma unroll
    for (int j = 0; j < 4; ++j) rd_b(&lds_wide[BF0], 0, 0, j);
#pragma unroll
    for (int q = 0; q < 2; ++q) issue_bs(q, 1, 1);

    int sa = 0, sb = 0;                    // stage % 3, stage % 2
    for (int s = 0; s < nstage; ++s) {
      const int sa1 = sa == 2 ? 0 : sa + 1, sa2 = sa == 0 ? 2 : sa - 1;    // (s+1) % 3, (s+2) % 3
      const bf16_t* bf = &lds_wide[BF0 + sb * BUNIT];
      const bf16_t* bs = &lds_wide[BS0 + sb * BUNIT];
      const bf16_t* bfn = &lds_wide[BF0 + (sb ^ 1) * BUNIT];
      const bool more = s + 1 < nstage;
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const int h = p >> 1, ks = p & 1;
        __builtin_amdgcn_sched_barrier(0);
        if (p == 1) {
          // middle of the stage: BS of this stage has landed, and behind the barrier BF is read by all
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          wait_loads_but<10>();
          __builtin_amdgcn_s_barrier();
          asm volatile("" ::: "memory");
        } else if (p == 3 && more) {
          // start of the next stage: its A and BF have landed; A and BS of this one are read by all
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          wait_loads_but<8>();
          __builtin_amdgcn_s_barrier();
          asm volatile("" ::: "memory");
        }
        // 16 MFMAs, one other instruction behind each of the first ten at most (see
        // gemm_bf16_wide_line_kernel): the next phase's fragments, then this phase's two loads
#pragma unroll
        for (int m = 0; m < 16; ++m) {
          const int i = m >> 2, j = m & 3;
          acc[i][4 * h + j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[p & 1][j], a[ks][i], acc[i][4 * h + j], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          if (p == 0) {          // next: (half 0, step 1): its A fragments, B from BF
            if (m < 4) rd_a(sa, 1, m);
            else if (m < 8) rd_b(bf, 1, 1, m - 4);
            else if (m < 10) issue_a(m - 8, s + 2, sa2);
          } else if (p == 1) {   // next: (half 1, step 0): B from BS (A of step 0 is in registers)
            if (m < 4) rd_b(bs, 0, 0, m);
            else if (m < 6) issue_bf(m - 4, s + 2, sb);
          } else if (p == 2) {   // next: (half 1, step 1)
            if (m < 4) rd_b(bs, 1, 1, m);
            else if (m < 6) issue_a(m - 2, s + 2, sa2);
          } else if (more) {     // next: (half 0, step 0) of stage s+1
            if (m < 4) rd_a(sa1, 0, m);
            else if (m < 8) rd_b(bfn, 0, 0, m - 4);
            else if (m < 10) issue_bs(m - 8, s + 2, sb);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      sa = sa1;
      sb ^= 1;
    }
    wait_loads_but<0>();
  }

  if constexpr (FUSE == 1) {
    bn_bwd_tile(acc, fa, lds_wide, m0, n0, N, wave, lane);
    return;
  }
  if constexpr (FUSE == 2) {
    bn_fwd_tile(acc, ff, lds_wide, m0, n0, N, wave, lane);
    return;
  }
  char* cbase = static_cast<char*>(ep.C) + (int64_t)blockIdx.z * slab_stride * (ep.c_is_bf16 ? 2 : 4);
  auto store_row = [&](auto ic) {
    constexpr int i = decltype(ic)::value;
    f32x4 row[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) row[j] = acc[i][j];
    if (ep.stream_c) store_tiles16_row<true>(row, ep, cbase, blockIdx.z == 0, m0 + wm * 64 + 16 * i, n0 + wn * (BN / 2), M, N, lane);
    else store_tiles16_row<false>(row, ep, cbase, blockIdx.z == 0, m0 + wm * 64 + 16 * i, n0 + wn * (BN / 2), M, N, lane);
  };
  store_row(std::integral_constant<int, 0>{});
  store_row(std::integral_constant<int, 1>{});
  store_row(std::integral_constant<int, 2>{});
  store_row(std::integral_constant<int, 3>{});
}

// ---- 3x3 convolution with the filters resident in LDS -------------------------------------------
// 64 input channels (one 128-byte row per position), 64 output channels per workgroup, image width
// W a power of two from 8 to 64.  The workgroup keeps its 64 x 576 filters in LDS (nine 64 x 64 tiles,
// one per tap) and walks over stages of 64 consecutive positions (64 / W image rows).  A stage's
// input is staged once: the image rows from one above to one below the stage, each with one empty
// position before and after it; rows outside the image come from a block of zeros and the empty
// positions are cleared once, so the nine shifted reads of a position find their value or 0 at
// fixed offsets.  Per stage a workgroup then fetches 64 + 2 W positions instead of nine times 64
// (and no filters): a ninth of what the patch-free product kernel pulls through the L2s.
// Rows are stored with the same 16-byte chunk permutation as the other LDS-direct kernels
// (by stored position for the input, by output channel for the filters).
// Requires H % (64 / W) == 0 (a stage lies within one image) and rows % 64 == 0.
// With `stats` (plain epilogue only: what is stored is the product itself) the workgroup also
// leaves, per output channel, the mean of the values it stored and their sum of squared
// deviations from it -- stats[(blockIdx.y * 2 + 0) * N + n] and [.. + 1 ..] -- for a per-channel
// normalisation over all positions: every lane keeps shifted sums over its own values (shift =
// its first value), and the four lanes that share a channel are joined in a fixed order.
template <int W>
__global__ __launch_bounds__(NT) void conv3x3_lds_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ Wk,
                                                         int64_t ldb, int H, const bf16_t* __restrict__ zeros,
                                                         int nstages, int stages_per_wg, int N, Epilogue ep,
                                                         float* __restrict__ stats) {
  static_assert(W == 8 || W == 16 || W == 32 || W == 64, "image width");
  constexpr int IR = 64 / W;                     // image rows per stage
  constexpr int PW = W + 2;                      // stored positions per image row
  constexpr int XR = (IR + 2) * PW;              // stored positions per stage
  constexpr int XB = XR * 64;                    // elements of one input buffer
  constexpr int FE = 9 * 64 * 64;                // elements of the filters
  constexpr int NI = (IR + 2) * (W / 8);         // load instructions per stage (8 positions each)
  extern __shared__ __attribute__((aligned(1024))) bf16_t lds_dyn[];
  bf16_t* F = lds_dyn;
  bf16_t* X = lds_dyn + FE;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1, hi = lane >> 5, m = lane & 31;
  const int n0 = blockIdx.x * 64;
  const int sbeg = blockIdx.y * stages_per_wg, send = min(nstages, sbeg + stages_per_wg);

  // filters: tile t = tap, 64 rows (output channels) of 64 channels, 8 rows per instruction
  for (int i = wave; i < 72; i += 4) {
    const int t = i >> 3, row = (i & 7) * 8 + (lane >> 3);
    const int chunk = (lane & 7) ^ dl_swizzle(row);
    const bf16_t* src = Wk + (int64_t)min(n0 + row, N - 1) * ldb + t * 64 + chunk * 8;
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)src,
                                     (void __attribute__((address_space(3)))*)&F[i * 512], 16, 0, 0);
  }
  // the empty positions before and after every stored image row, both buffers (32 dwords each)
  for (int k = tid; k < 2 * (IR + 2) * 2 * 32; k += NT) {
    const int dword = k & 31, which = k >> 5;
    const int side = which & 1, irow = (which >> 1) % (IR + 2), buf = (which >> 1) / (IR + 2);
    const int pos = irow * PW + (side ? PW - 1 : 0);
    reinterpret_cast<uint32_t*>(X + buf * XB + pos * 64)[dword] = 0u;
  }

  auto issue = [&](int stage, int buf) {
    for (int idx = wave; idx < NI; idx += 4) {
      const int ir = idx / (W / 8) - 1, sub = idx % (W / 8);
      const int p = (ir + 1) * PW + 1 + sub * 8 + (lane >> 3);      // stored position of this lane's row
      const int chunk = (lane & 7) ^ dl_swizzle(p);
      const int g = stage * IR + ir;                                // image row among all images' rows
      const int hh = (stage * IR) % H + ir;
      const bf16_t* src = (hh >= 0 && hh < H) ? x + ((int64_t)g * W + sub * 8 + (lane >> 3)) * 64 + chunk * 8
                                              : zeros + chunk * 8;
      __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)src,
                                       (void __attribute__((address_space(3)))*)&X[buf * XB + ((ir + 1) * PW + 1 + sub * 8) * 64],
                                       16, 0, 0);
    }
  };

  // this lane's operand rows: stage position e under tap t sits at stored position
  // (e / W + kh) * PW + e % W + kw; its filter row is output channel wn * 32 + m of tile t
  const int e = wm * 32 + m;
  int pa[9], fa[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) {
    const int p = (e / W + t / 3) * PW + e % W + t % 3;
    pa[t] = p * 64;
    fa[t] = dl_swizzle(p);
  }
  const int brow = (wn * 32 + m) * 64, fb = dl_swizzle(wn * 32 + m);

  float shift = 0.f, sd = 0.f, sq = 0.f;           // stats: this lane's values v as sums of (v - shift) and (v - shift)^2
  if (sbeg < send) issue(sbeg, 0);
  for (int st = sbeg; st < send; ++st) {
    const int buf = (st - sbeg) & 1;
    wait_loads_but<0>();
    __syncthreads();                               // stage st (and the filters) are in LDS; everybody is done with the other buffer
    if (st + 1 < send) issue(st + 1, buf ^ 1);
    const bf16_t* xs = X + buf * XB;
    f32x16 acc0, acc1;
#pragma unroll
    for (int r = 0; r < 16; ++r) { acc0[r] = 0.f; acc1[r] = 0.f; }
    // 36 MFMAs (9 taps x 4 contraction steps); the operand reads of step i + AHEAD are issued
    // before the MFMA of step i (one wave per SIMD: nobody else covers the LDS latency)
    constexpr int AHEAD = 3, SLOTS = AHEAD + 1;
    bf16x8 fa_[SLOTS], fb_[SLOTS];
    auto read_step = [&](int i, int slot) {
      const int t = i >> 2, ci = 2 * (i & 3) + hi;
      fa_[slot] = *reinterpret_cast<const bf16x8*>(&xs[pa[t] + ((ci ^ fa[t]) * 8)]);
      fb_[slot] = *reinterpret_cast<const bf16x8*>(&F[t * 4096 + brow + ((ci ^ fb) * 8)]);
    };
#pragma unroll
    for (int i = 0; i < AHEAD; ++i) read_step(i, i);
#pragma unroll
    for (int i = 0; i < 36; ++i) {
      if (i + AHEAD < 36) read_step(i + AHEAD, (i + AHEAD) % SLOTS);
      __builtin_amdgcn_sched_barrier(0);
      if (i & 1) acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa_[i % SLOTS], fb_[i % SLOTS], acc1, 0, 0, 0);
      else       acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa_[i % SLOTS], fb_[i % SLOTS], acc0, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    f32x16 tiles[1][1];
#pragma unroll
    for (int r = 0; r < 16; ++r) tiles[0][0][r] = acc0[r] + acc1[r];
    store_tiles<1, 1>(tiles, ep, static_cast<char*>(ep.C), true, st * 64 + wm * 32, n0 + wn * 32, nstages * 64, N, lane);
    if (stats) {
      if (st == sbeg) shift = tiles[0][0][0];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float d = tiles[0][0][r] - shift;
        sd += d;
        sq = fmaf(d, d, sq);
      }
    }
  }
  wait_loads_but<0>();
  if (stats && sbeg < send) {
    __shared__ float st_m[4][64], st_q[4][64];
    const float cnt = 16.f * (float)(send - sbeg);           // values per lane
    const float dm = sd / cnt;
    st_m[wm * 2 + hi][wn * 32 + m] = shift + dm;
    st_q[wm * 2 + hi][wn * 32 + m] = sq - sd * dm;
    __syncthreads();
    if (tid < 64 && n0 + tid < N) {
      // the two-group update of a mean and a sum of squared deviations, groups of equal size joined in order
      float mean = st_m[0][tid], m2 = st_q[0][tid], have = cnt;
#pragma unroll
      for (int g = 1; g < 4; ++g) {
        const float tot = have + cnt, delta = st_m[g][tid] - mean;
        mean = fmaf(delta, cnt / tot, mean);
        m2 = m2 + st_q[g][tid] + delta * delta * (have * cnt / tot);
        have = tot;
      }
      stats[((int64_t)blockIdx.y * 2 + 0) * N + n0 + tid] = mean;
      stats[((int64_t)blockIdx.y * 2 + 1) * N + n0 + tid] = m2;
    }
  }
}

// Short contraction (K <= 2*BK = 128: the weight gradient of a node of up to 128 rows).  The
// cost of such a product is one trip to memory for the operands and the write (or
// read-modify-write) of the fp32 output, so everything is issued at once: both stages of
// operand loads and, when the epilogue adds into C (fused fold into the gradient buffer), the
// old C values as well; then one LDS barrier and the MFMAs.  The accumulators are then passed
// through LDS so that every lane reads/writes 16 contiguous bytes of C: a wavefront touches
// four full 256-byte row segments per instruction instead of two 128-byte ones.
// Requires fp32 C, 16-byte aligned, ldc (and ldr) multiples of 4, N a multiple of 4.
template <int BM, int BN>
__global__ __launch_bounds__(NT) void gemm_bf16_shortk_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                              const bf16_t* __restrict__ B, int64_t ldb,
                                                              int M, int N, int K, Epilogue ep) {
  static_assert(BM == 64 && BN == 64, "2x2 waves of 32x32");
  constexpr int KT = 2 * BK;                  // 128
  constexpr int LD2 = KT + 8;                 // padded LDS row of the operands
  constexpr int LDC = BN + 4;                 // padded fp32 row of the staged output tile
  constexpr int A_VECS = BM * (KT / 8) / NT;  // 16-byte vectors per thread
  constexpr int B_VECS = BN * (KT / 8) / NT;
  constexpr int C_VECS = BM * (BN / 4) / NT;  // float4 per thread of the output tile

  __shared__ __attribute__((aligned(16))) char smem[(BM + BN) * LD2 * 2];
  bf16_t* As = reinterpret_cast<bf16_t*>(smem);
  bf16_t* Bs = As + BM * LD2;
  float* Ct = reinterpret_cast<float*>(smem);   // reused after the MFMAs
  static_assert(BM * LDC * 4 <= (BM + BN) * LD2 * 2, "output tile fits in the operand buffers");

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int vcol = (tid & 15) * 8;   // 16 vectors per 128-wide row
  const int vrow = tid >> 4;         // 0..15

  u32x4 ra[A_VECS], rb[B_VECS];
#pragma unroll
  for (int i = 0; i < A_VECS; ++i) ra[i] = load_vec(A, lda, m0 + vrow + 16 * i, M, vcol, K);
#pragma unroll
  for (int i = 0; i < B_VECS; ++i) rb[i] = load_vec(B, ldb, n0 + vrow + 16 * i, N, vcol, K);

  // this thread's float4 pieces of the output tile: row crow + 16*i, columns ccol..ccol+3
  const int ccol = (tid & 15) * 4;
  const int crow = tid >> 4;
  const bool col_ok = n0 + ccol < N;           // N % 4 == 0: a float4 is all in or all out
  float4 oldc[C_VECS];
  if (ep.R) {
#pragma unroll
    for (int i = 0; i < C_VECS; ++i) {
      const int m = m0 + crow + 16 * i;
      oldc[i] = (col_ok && m < M) ? *reinterpret_cast<const float4*>(&ep.R[(int64_t)m * ep.ldr + n0 + ccol])
                                  : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }

#pragma unroll
  for (int i = 0; i < A_VECS; ++i) *reinterpret_cast<u32x4*>(&As[(vrow + 16 * i) * LD2 + vcol]) = ra[i];
#pragma unroll
  for (int i = 0; i < B_VECS; ++i) *reinterpret_cast<u32x4*>(&Bs[(vrow + 16 * i) * LD2 + vcol]) = rb[i];
  __syncthreads();

  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  const int ksteps = (K + 15) / 16;            // 16-wide MFMA steps that hold any data
#pragma unroll
  for (int ks = 0; ks < KT / 16; ++ks) {
    if (ks < ksteps) {
      const int koff = ks * 16 + (lane >> 5) * 8;
      bf16x8 a = *reinterpret_cast<const bf16x8*>(&As[(wm * 32 + (lane & 31)) * LD2 + koff]);
      bf16x8 b = *reinterpret_cast<const bf16x8*>(&Bs[(wn * 32 + (lane & 31)) * LD2 + koff]);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
    }
  }
  __syncthreads();                             // operands no longer needed: reuse LDS for the tile
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int row = wm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
    Ct[row * LDC + wn * 32 + (lane & 31)] = acc[r];
  }
  __syncthreads();

  float4 bias4 = make_float4(0.f, 0.f, 0.f, 0.f);
  if (ep.bias && col_ok) {
    bias4 = *reinterpret_cast<const float4*>(&ep.bias[n0 + ccol]);
    if (ep.bias_round_bf16) {
      bias4.x = round_bf16(bias4.x); bias4.y = round_bf16(bias4.y);
      bias4.z = round_bf16(bias4.z); bias4.w = round_bf16(bias4.w);
    }
  }
  float* C = static_cast<float*>(ep.C);
#pragma unroll
  for (int i = 0; i < C_VECS; ++i) {
    const int row = crow + 16 * i;
    const int m = m0 + row;
    if (!col_ok || m >= M) continue;
    const float4 a4 = *reinterpret_cast<const float4*>(&Ct[row * LDC + ccol]);
    float4 add = bias4;
    if (ep.R) {
      add.x = fmaf(ep.beta, oldc[i].x, bias4.x); add.y = fmaf(ep.beta, oldc[i].y, bias4.y);
      add.z = fmaf(ep.beta, oldc[i].z, bias4.z); add.w = fmaf(ep.beta, oldc[i].w, bias4.w);
    }
    float4 v;
    v.x = fmaf(ep.alpha, a4.x, add.x); v.y = fmaf(ep.alpha, a4.y, add.y);
    v.z = fmaf(ep.alpha, a4.z, add.z); v.w = fmaf(ep.alpha, a4.w, add.w);
    *reinterpret_cast<float4*>(&C[(int64_t)m * ep.ldc + n0 + ccol]) = v;
  }
}

// Weight gradients of up to kFoldMax consecutive virtual nodes folded into the gradient buffer
// in ONE pass over it (Section 3.2 step 3 with the weights of Section 5.2):
//     C[m, n] <- fma(w_{c-1}, P_{c-1}[m, n], ... fma(w_1, P_1[m, n], fma(w_0, P_0[m, n], C[m, n])))
// with P_j = A_j B_j^T the product over node j's rows (at most 128, contiguous in the transposed
// operand copies) -- exactly the chain of fused multiply-adds that one launch per node produces,
// so the result is bitwise the same, but C is read and written once per window instead of once
// per node.  With `overwrite` the chain starts from zero (first window of a step).
// 128 x 128 tile, four waves of 64 x 64; node j+1's operands are in flight while node j's
// products are computed; each product passes through LDS so that a lane owns 16 contiguous
// bytes of C.  Requires fp32 C, 16-byte aligned, ldc % 4 == 0, N % 4 == 0.
__global__ __launch_bounds__(NT) void gemm_bf16_fold_kernel(FoldArgs fa, int64_t ld, int M, int N,
                                                            float* __restrict__ C, int64_t ldc) {
  constexpr int BM = 128, BN = 128;
  constexpr int KT = 2 * BK;                  // 128: the longest node
  constexpr int LD2 = KT + 8;
  constexpr int LDC = BN + 4;
  constexpr int A_VECS = BM * (KT / 8) / NT;  // 8
  constexpr int B_VECS = BN * (KT / 8) / NT;  // 8
  constexpr int C_VECS = BM * (BN / 4) / NT;  // 16

  __shared__ __attribute__((aligned(16))) char smem[(BM + BN) * LD2 * 2];
  bf16_t* As = reinterpret_cast<bf16_t*>(smem);
  bf16_t* Bs = As + BM * LD2;
  float* Ct = reinterpret_cast<float*>(smem);   // reused between the MFMAs of consecutive nodes
  static_assert(BM * LDC * 4 <= (BM + BN) * LD2 * 2, "output tile fits in the operand buffers");

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int vcol = (tid & 15) * 8;
  const int vrow = tid >> 4;         // 0..15
  const int ccol = (tid & 31) * 4;
  const int crow = tid >> 5;         // 0..7
  const bool col_ok = n0 + ccol < N;

  u32x4 ra[A_VECS], rb[B_VECS];
  auto load_node = [&](int j) {
    const bf16_t* A = fa.A[j];
    const bf16_t* B = fa.B[j];
    const int K = fa.K[j];
#pragma unroll
    for (int i = 0; i < A_VECS; ++i) ra[i] = load_vec(A, ld, m0 + vrow + 16 * i, M, vcol, K);
#pragma unroll
    for (int i = 0; i < B_VECS; ++i) rb[i] = load_vec(B, ld, n0 + vrow + 16 * i, N, vcol, K);
  };
  load_node(0);

  float4 c[C_VECS];
#pragma unroll
  for (int i = 0; i < C_VECS; ++i) {
    const int m = m0 + crow + 8 * i;
    c[i] = (!fa.overwrite && col_ok && m < M) ? *reinterpret_cast<const float4*>(&C[(int64_t)m * ldc + n0 + ccol])
                                              : make_float4(0.f, 0.f, 0.f, 0.f);
  }

  for (int j = 0; j < fa.count; ++j) {
    if (j) __syncthreads();                    // every lane has read node j-1's tile
#pragma unroll
    for (int i = 0; i < A_VECS; ++i) *reinterpret_cast<u32x4*>(&As[(vrow + 16 * i) * LD2 + vcol]) = ra[i];
#pragma unroll
    for (int i = 0; i < B_VECS; ++i) *reinterpret_cast<u32x4*>(&Bs[(vrow + 16 * i) * LD2 + vcol]) = rb[i];
    __syncthreads();
    if (j + 1 < fa.count) load_node(j + 1);    // in flight during this node's MFMAs

    f32x16 acc[2][2];
#pragma unroll
    for (int ti = 0; ti < 2; ++ti)
#pragma unroll
      for (int tj = 0; tj < 2; ++tj)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[ti][tj][r] = 0.f;
    const int ksteps = (fa.K[j] + 15) / 16;
#pragma unroll
    for (int ks = 0; ks < KT / 16; ++ks) {
      if (ks < ksteps) {
        const int koff = ks * 16 + (lane >> 5) * 8;
        bf16x8 a[2], b[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          a[t] = *reinterpret_cast<const bf16x8*>(&As[(wm * 64 + t * 32 + (lane & 31)) * LD2 + koff]);
          b[t] = *reinterpret_cast<const bf16x8*>(&Bs[(wn * 64 + t * 32 + (lane & 31)) * LD2 + koff]);
        }
#pragma unroll
        for (int ti = 0; ti < 2; ++ti)
#pragma unroll
          for (int tj = 0; tj < 2; ++tj)
            acc[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ti], b[tj], acc[ti][tj], 0, 0, 0);
      }
    }
    __syncthreads();                           // operands consumed: the tile may overwrite them
#pragma unroll
    for (int ti = 0; ti < 2; ++ti)
#pragma unroll
      for (int tj = 0; tj < 2; ++tj)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = wm * 64 + ti * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          Ct[row * LDC + wn * 64 + tj * 32 + (lane & 31)] = acc[ti][tj][r];
        }
    __syncthreads();
    const float w = fa.w[j];
#pragma unroll
    for (int i = 0; i < C_VECS; ++i) {
      const float4 p = *reinterpret_cast<const float4*>(&Ct[(crow + 8 * i) * LDC + ccol]);
      c[i].x = fmaf(w, p.x, c[i].x); c[i].y = fmaf(w, p.y, c[i].y);
      c[i].z = fmaf(w, p.z, c[i].z); c[i].w = fmaf(w, p.w, c[i].w);
    }
  }
#pragma unroll
  for (int i = 0; i < C_VECS; ++i) {
    const int m = m0 + crow + 8 * i;
    if (col_ok && m < M) *reinterpret_cast<float4*>(&C[(int64_t)m * ldc + n0 + ccol]) = c[i];
  }
}

struct Shape {
  const bf16_t* A; int64_t lda; const bf16_t* B; int64_t ldb; int M, N, K, nsplit; int64_t slab;
};

bool shortk_enabled();
int dl_depth();
int pipe_depth();   // 0 = plain kernel, 2..4 = ring depth of the pipelined kernel

template <int BM, int BN, int WGM, int WGN>
int launch_cfg(const Shape& g, const Epilogue& ep, hipStream_t s) {
  int kchunk = ((g.K + g.nsplit - 1) / g.nsplit + BK - 1) / BK * BK;
  dim3 grid((g.N + BN - 1) / BN, (g.M + BM - 1) / BM, g.nsplit);
  constexpr int VPS = (BM + BN) * (BK / 8) / NT;
  const int depth = pipe_depth();
#define VF_PIPE(NS)                                                                               \
  gemm_bf16_pipe_kernel<BM, BN, WGM, WGN, NS><<<grid, NT, 0, s>>>(g.A, g.lda, g.B, g.ldb, g.M, g.N, \
                                                                  g.K, kchunk, g.slab, ep)
  if (depth >= 4 && 3 * VPS < 60 && VPS <= 8) VF_PIPE(4);
  else if (depth >= 3 && VPS <= 8) VF_PIPE(3);
  else if (depth >= 2) VF_PIPE(2);
  else
    gemm_bf16_kernel<BM, BN, WGM, WGN><<<grid, NT, 0, s>>>(g.A, g.lda, g.B, g.ldb, g.M, g.N, g.K, kchunk,
                                                           g.slab, ep);
#undef VF_PIPE
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

bool shortk_enabled() {   // tuning aid: VF_GEMM_SHORTK=0 sends weight gradients to the general kernel
  static int cached = -1;
  if (cached < 0) {
    const char* e = std::getenv("VF_GEMM_SHORTK");
    cached = (e && e[0] == '0') ? 0 : 1;
  }
  return cached != 0;
}

int dl_depth() {   // tuning aid: VF_GEMM_DL=0 disables the LDS-direct kernel, 3..5 sets its ring depth
  static int cached = -1;
  if (cached < 0) {
    const char* e = std::getenv("VF_GEMM_DL");
    cached = e ? std::atoi(e) : 4;
    if (cached != 0 && (cached < 3 || cached > 5)) cached = 4;
  }
  return cached;
}

int pipe_depth() {
  static int cached = -1;
  if (cached < 0) {
    const char* e = std::getenv("VF_GEMM_PIPE");   // tuning aid; 3 measured best on the node shapes
    cached = e ? std::atoi(e) : 3;
    if (cached < 0 || cached > 4) cached = 0;
  }
  return cached;
}

int launch_wide(const Shape& g, const Epilogue& ep, hipStream_t s);

}  // namespace
static int launch_gemm_bf16_ep(const Shape& g, const Epilogue& ep, hipStream_t s);

// Compute-bound shapes take the big tile; everything else (few rows, or a short contraction
// whose cost is writing the output) does better with many small workgroups in flight.
static bool use_big_tile(int M, int N, int K) { return M >= 1024 && N >= 1024 && K >= 512; }

// The wide kernel takes products of more than 128 rows whose contraction slices are whole stages.
// Tuning aid: VF_GEMM_WIDE=0 switches it off, 128 / 256 forces the tile width.
static int wide_mode() {
  static int cached = -1;
  if (cached < 0) {
    const char* e = std::getenv("VF_GEMM_WIDE");
    cached = e ? std::atoi(e) : 1;
  }
  return cached;
}
static int wide_tile_n(int M, int N) {
  const int mode = wide_mode();
  if (mode == 128 || mode == 256) return mode;
  const int64_t tm = (M + 255) / 256;
  // 256 x 256 once that still gives every compute unit a tile; narrow matrices keep 128
  const int64_t t256 = tm * ((N + 255) / 256), t128 = tm * ((N + 127) / 128);
  if (N < 256 || t256 < 256) return 128;
  // Every compute unit takes one tile at a time, so a grid runs in rounds of 256 tiles and the last
  // round costs as much as a full one.  A 256-wide tile takes about 1.85 times as long as a
  // 128-wide one (twice the work, somewhat better fed): take whichever needs less time in rounds.
  const int64_t r256 = (t256 + 255) / 256, r128 = (t128 + 255) / 256;
  return (r256 * 185 <= r128 * 100) ? 256 : 128;
}
static bool wide_fits(int M, int N, int K, int nsplit) {
  if (!wide_mode() || M <= 128 || N < 128 || (K % BK)) return false;
  // (the 256-row kernels address their operands with 32-bit byte offsets: launch_gemm_bf16 checks the spans)
  const int kchunk = ((K + nsplit - 1) / nsplit + BK - 1) / BK * BK;
  return (K % kchunk) == 0 || nsplit == 1;
}

int gemm_bf16_pick_split(int M, int N, int K) {
  if (wide_fits(M, N, K, 1)) {
    // one workgroup per compute unit: slices until about 256 workgroups, each at least 8 stages long
    const int bn = wide_tile_n(M, N);
    const int64_t tiles = (int64_t)((M + 255) / 256) * ((N + bn - 1) / bn);
    int split = 1;
    while (tiles * split * 2 <= 256 && K / (split * 2) >= 8 * BK && (K / BK) % (split * 2) == 0 && split < 32) split *= 2;
    return split;
  }
  // Measured on the node-sized products (128 x 4096 x 4096 and relatives) with the
  // pipelined kernel: about two 64x64 workgroups per compute unit, slices no shorter than
  // 3 LDS stages.
  if (use_big_tile(M, N, K)) return 1;
  int bm = M <= 32 ? 32 : 64;
  int bn = M <= 32 ? 128 : 64;
  int64_t tiles = (int64_t)((M + bm - 1) / bm) * ((N + bn - 1) / bn);
  static const int target = std::getenv("VF_GEMM_SPLIT_TARGET") ? std::atoi(std::getenv("VF_GEMM_SPLIT_TARGET")) : 256;
  int split = 1;
  while (tiles * split < target && K / (split * 2) >= 3 * BK && split < 32) split *= 2;
  return split;
}

namespace {
template <int BN, int KS, int NS>
int launch_wide_cfg(const Shape& g, const Epilogue& ep, hipStream_t s) {
  constexpr int bytes = NS * (256 + BN) * KS * 2;
  static bool ready = false;
  if (!ready) {
    VF_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_wide_kernel<BN, KS, NS>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    ready = true;
  }
  const int kchunk = ((g.K + g.nsplit - 1) / g.nsplit + BK - 1) / BK * BK;
  const int tiles_m = (g.M + 255) / 256, tiles_n = (g.N + BN - 1) / BN;
  const int ntile = tiles_m * tiles_n;
  dim3 grid(((ntile + 7) / 8) * 8, 1, g.nsplit);
  gemm_bf16_wide_kernel<BN, KS, NS><<<grid, 512, bytes, s>>>(g.A, g.lda, g.B, g.ldb, g.M, g.N, g.K, kchunk, g.slab, ep,
                                                             tiles_m, tiles_n);
  VF_LAUNCH_CHECK();
  return VF_OK;
}
int wide_variant();
int launch_wide_line(const Shape& g, const Epilogue& ep, hipStream_t s) {
  constexpr int bytes = 160 * 1024;
  static bool ready = false;
  if (!ready) {
    VF_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_wide_line_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    VF_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_wide_line16_kernel<0>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    VF_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_wide_line16_kernel<1>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    ready = true;
  }
  const int kchunk = ((g.K + g.nsplit - 1) / g.nsplit + BK - 1) / BK * BK;
  const int tiles_m = (g.M + 255) / 256, tiles_n = (g.N + 255) / 256;
  const int ntile = tiles_m * tiles_n;
  dim3 grid(((ntile + 7) / 8) * 8, 1, g.nsplit);
  // Several rounds of tiles: an fp32 result is stored with the non-temporal hint (see launch_gemm_bf16),
  // which is worth 9 % there (8192^3: 690 -> 630 us on operands of zeros); one round gains nothing.
  Epilogue epx = ep;
  if (ntile >= 512 && !ep.c_is_bf16 && !ep.R) epx.stream_c = 1;
  if (wide_variant() == 2)
    gemm_bf16_wide_line_kernel<<<grid, 512, bytes, s>>>(g.A, g.lda, g.B, g.ldb, g.M, g.N, g.K, kchunk, g.slab, epx, tiles_m,
                                                        tiles_n);
  else
    gemm_bf16_wide_line16_kernel<0><<<grid, 512, bytes, s>>>(g.A, g.lda, g.B, g.ldb, g.M, g.N, g.K, kchunk, g.slab, epx,
                                                                 tiles_m, tiles_n, BnBwdArgs{}, BnFwdArgs{});
  VF_LAUNCH_CHECK();
  return VF_OK;
}
int wide_variant() {   // tuning aid: VF_GEMM_WIDE_V=1 runs 256-wide tiles on the ring of three half-line stages, 2 on the whole-line kernel with 32x32x16 MFMAs
  static int cached = -1;
  if (cached < 0) {
    const char* e = std::getenv("VF_GEMM_WIDE_V");
    cached = e ? std::atoi(e) : 0;
  }
  return cached;
}
int launch_wide(const Shape& g, const Epilogue& ep, hipStream_t s) {
  if (wide_tile_n(g.M, g.N) == 256)
    return wide_variant() == 1 ? launch_wide_cfg<256, 32, 3>(g, ep, s) : launch_wide_line(g, ep, s);
  return launch_wide_cfg<128, 64, 3>(g, ep, s);
}
}  // namespace

// The product with the BatchNorm backward pass in its epilogue (see bn_bwd_tile): shapes that the
// 256 x 256 kernel on the 16x16x32 MFMA takes in whole tiles.  VF_BN_FUSE = 0 switches it off.
bool gemm_bf16_bn_fwd_takes(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, int M, int N, int K,
                            const BnFwdArgs& fa) {
  static const bool enabled = !(std::getenv("VF_BN_FUSE_FWD") && std::atoi(std::getenv("VF_BN_FUSE_FWD")) == 0);
  if (!enabled || M <= 0 || N <= 0 || K <= 0 || !A || !B || !fa.z || !fa.a || !fa.aT) return false;
  if ((fa.gamma == nullptr) != (fa.beta == nullptr) || (fa.gamma && (!fa.mean || !fa.rstd || !fa.var || fa.bias))) return false;
  auto al = [](const void* p, uintptr_t n) { return (reinterpret_cast<uintptr_t>(p) & (n - 1)) == 0; };
  const bool spans32 = (int64_t)M * lda * 2 < ((int64_t)1 << 31) && (int64_t)N * ldb * 2 < ((int64_t)1 << 31);
  return (M % 256) == 0 && (N % 256) == 0 && (K % 64) == 0 && spans32 && wide_fits(M, N, K, 1) &&
         wide_tile_n(M, N) == 256 && wide_variant() == 0 && !(lda & 7) && !(ldb & 7) && al(A, 16) && al(B, 16) &&
         !(fa.ldz & 3) && !(fa.lda & 3) && !(fa.ldt & 7) && al(fa.z, 16) && al(fa.a, 8) && al(fa.aT, 16) &&
         al(fa.mean, 16) && al(fa.rstd, 16) && al(fa.var, 16) && al(fa.gamma, 16) && al(fa.beta, 16) && al(fa.bias, 16);
}

int launch_gemm_bf16_bn_fwd(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, int M, int N, int K,
                            const BnFwdArgs& fa, hipStream_t s) {
  if (!gemm_bf16_bn_fwd_takes(A, lda, B, ldb, M, N, K, fa)) return VF_EINVAL;
  constexpr int bytes = 160 * 1024;
  static bool ready = false;
  if (!ready) {
    VF_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_wide_line16_kernel<2>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    ready = true;
  }
  const int tiles_m = M / 256, tiles_n = N / 256;
  const int ntile = tiles_m * tiles_n;
  dim3 grid(((ntile + 7) / 8) * 8, 1, 1);
  gemm_bf16_wide_line16_kernel<2><<<grid, 512, bytes, s>>>(A, lda, B, ldb, M, N, K, K, 0, Epilogue{}, tiles_m, tiles_n,
                                                           BnBwdArgs{}, fa);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

bool gemm_bf16_bn_bwd_takes(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, int M, int N, int K,
                            const BnBwdArgs& fa) {
  static const bool enabled = !(std::getenv("VF_BN_FUSE") && std::atoi(std::getenv("VF_BN_FUSE")) == 0);
  if (!enabled || M <= 0 || N <= 0 || K <= 0 || !A || !B || !fa.z || !fa.dz || !fa.dzT || !fa.sums) return false;
  if ((fa.gamma == nullptr) != (fa.beta == nullptr) || (fa.gamma && (!fa.mean || !fa.rstd))) return false;
  auto al = [](const void* p, uintptr_t n) { return (reinterpret_cast<uintptr_t>(p) & (n - 1)) == 0; };
  const bool spans32 = (int64_t)M * lda * 2 < ((int64_t)1 << 31) && (int64_t)N * ldb * 2 < ((int64_t)1 << 31);
  return (M % 256) == 0 && (N % 256) == 0 && (K % 64) == 0 && spans32 && wide_fits(M, N, K, 1) &&
         wide_tile_n(M, N) == 256 && wide_variant() == 0 && !(lda & 7) && !(ldb & 7) && al(A, 16) && al(B, 16) &&
         !(fa.ldz & 3) && !(fa.lddz & 3) && !(fa.ldt & 7) && al(fa.z, 16) && al(fa.dz, 8) && al(fa.dzT, 16) &&
         al(fa.sums, 16) && al(fa.mean, 16) && al(fa.rstd, 16) && al(fa.gamma, 16) && al(fa.beta, 16);
}

int launch_gemm_bf16_bn_bwd(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, int M, int N, int K,
                            const BnBwdArgs& fa, hipStream_t s) {
  if (!gemm_bf16_bn_bwd_takes(A, lda, B, ldb, M, N, K, fa)) return VF_EINVAL;
  constexpr int bytes = 160 * 1024;
  static bool ready = false;
  if (!ready) {
    VF_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_wide_line16_kernel<1>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    ready = true;
  }
  const int tiles_m = M / 256, tiles_n = N / 256;
  const int ntile = tiles_m * tiles_n;
  dim3 grid(((ntile + 7) / 8) * 8, 1, 1);
  gemm_bf16_wide_line16_kernel<1><<<grid, 512, bytes, s>>>(A, lda, B, ldb, M, N, K, K, 0, Epilogue{}, tiles_m, tiles_n, fa, BnFwdArgs{});
  VF_LAUNCH_CHECK();
  return VF_OK;
}


int launch_gemm_bf16(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, int M, int N,
                     int K, int nsplit, int64_t slab_stride, const Epilogue& ep, hipStream_t s) {
  if (M <= 0 || N <= 0 || K <= 0 || !A || !B || !ep.C || nsplit < 1) return VF_EINVAL;
  if (nsplit > 1 && ep.R) return VF_EINVAL;   // slabs are partial sums: nothing may be added in
  if ((lda & 7) || (ldb & 7) || (reinterpret_cast<uintptr_t>(A) & 15) ||
      (reinterpret_cast<uintptr_t>(B) & 15))
    return VF_EINVAL;
  Shape g{A, lda, B, ldb, M, N, K, nsplit, slab_stride};
  // Epilogue::stream_c stores an fp32 result with the non-temporal hint.  Stored the ordinary way,
  // the tiles that the workgroups of an XCD finish together (8 MB) pass through its 4 MB L2 and push
  // out the operand panels the next tiles share: the operand traffic of an 8192^3 product alone
  // takes 330 us, with the result stored the ordinary way 590 us, with the hint 370 us.  Inside the
  // product that is worth 3 % on long contractions (8192^3: 939 -> 906 us) and costs on short ones
  // (8192 x 8192 x 1024: 151 -> 166 us), and the kernel that reads the result next finds less of it
  // in the caches (BatchNorm forward of a 2048-row unit: 48 -> 54 us), so no caller sets it;
  // VF_GEMM_NT=1 sets it for every product (tuning aid).
  static const int force_nt = std::getenv("VF_GEMM_NT") ? std::atoi(std::getenv("VF_GEMM_NT")) : 0;
  Epilogue epx = ep;
  if (force_nt && !ep.c_is_bf16) epx.stream_c = 1;
  return launch_gemm_bf16_ep(g, epx, s);
}

static int launch_gemm_bf16_ep(const Shape& g, const Epilogue& ep, hipStream_t s) {
  const bf16_t* A = g.A; const bf16_t* B = g.B;
  const int64_t lda = g.lda, ldb = g.ldb;
  const int M = g.M, N = g.N, K = g.K, nsplit = g.nsplit;
  const int64_t slab_stride = g.slab;
  switch (forced_tile()) {
    case 1: return launch_cfg<128, 128, 2, 2>(g, ep, s);
    case 2: return launch_cfg<128, 64, 2, 2>(g, ep, s);
    case 3: return launch_cfg<64, 128, 2, 2>(g, ep, s);
    case 4: return launch_cfg<64, 64, 2, 2>(g, ep, s);
    case 5: return launch_cfg<32, 128, 1, 4>(g, ep, s);
    case 6: return launch_cfg<128, 32, 4, 1>(g, ep, s);
    default: break;
  }
  // short contraction into an fp32 matrix (weight gradients): single-trip kernel
  const bool vec_ok = !ep.c_is_bf16 && (N & 3) == 0 && (ep.ldc & 3) == 0 &&
                      (reinterpret_cast<uintptr_t>(ep.C) & 15) == 0 &&
                      (!ep.R || ((ep.ldr & 3) == 0 && (reinterpret_cast<uintptr_t>(ep.R) & 15) == 0)) &&
                      (!ep.bias || (reinterpret_cast<uintptr_t>(ep.bias) & 15) == 0);
  if (K <= 2 * BK && nsplit == 1 && vec_ok && M > 32 && N > 32 && shortk_enabled()) {
    dim3 grid((N + 63) / 64, (M + 63) / 64);
    gemm_bf16_shortk_kernel<64, 64><<<grid, NT, 0, s>>>(A, lda, B, ldb, M, N, K, ep);
    VF_LAUNCH_CHECK();
    return VF_OK;
  }
  // (the 256-row kernels address their operands with 32-bit byte offsets)
  const bool spans32 = (int64_t)M * lda * 2 < ((int64_t)1 << 31) && (int64_t)N * ldb * 2 < ((int64_t)1 << 31);
  if (spans32 && wide_fits(M, N, K, nsplit)) return launch_wide(g, ep, s);
  if (use_big_tile(M, N, K)) return launch_cfg<128, 128, 2, 2>(g, ep, s);
  if (M <= 32) return launch_cfg<32, 128, 1, 4>(g, ep, s);
  if (N <= 32) return launch_cfg<128, 32, 4, 1>(g, ep, s);
  // whole 64-element stages in every slice: operand tiles straight into LDS
  const int kchunk = ((K + nsplit - 1) / nsplit + BK - 1) / BK * BK;
  const int depth = dl_depth();
  if (depth && (K % BK) == 0 && (K % kchunk) == 0) {
    dim3 grid((N + 63) / 64, (M + 63) / 64, nsplit);
    switch (depth) {
      case 3: gemm_bf16_dl_kernel<3><<<grid, NT, 0, s>>>(A, lda, B, ldb, M, N, K, kchunk, slab_stride, ep); break;
      case 5: gemm_bf16_dl_kernel<5><<<grid, NT, 0, s>>>(A, lda, B, ldb, M, N, K, kchunk, slab_stride, ep); break;
      default: gemm_bf16_dl_kernel<4><<<grid, NT, 0, s>>>(A, lda, B, ldb, M, N, K, kchunk, slab_stride, ep); break;
    }
    VF_LAUNCH_CHECK();
    return VF_OK;
  }
  return launch_cfg<64, 64, 2, 2>(g, ep, s);
}

// C[r, n] = sum over the 3x3 neighbourhood and the channels of x (rows = images * H * W
// positions, channels last, Cin a multiple of 64) times Wk[n, (kh, kw, c)] (row pitch ldb):
// a 3x3 convolution, stride 1, zero padding 1, without a patch matrix.  `zeros`: 128 bytes of 0.
int launch_conv3x3_bf16(const bf16_t* x, int64_t rows, int H, int W, int Cin, const bf16_t* Wk, int64_t ldb, int N,
                        const Epilogue& ep, const bf16_t* zeros, hipStream_t s, float* stats, int* stats_chunks,
                        int* stats_rows) {
  if (stats_chunks) *stats_chunks = 0;
  if (!x || !Wk || !ep.C || !zeros || rows <= 0 || rows > 0x7fffffff || H <= 0 || W <= 0 || N <= 0) return VF_EINVAL;
  if ((Cin % BK) || rows % ((int64_t)H * W) || (ldb & 7) || ldb < 9 * Cin) return VF_EINVAL;
  if ((reinterpret_cast<uintptr_t>(x) & 15) || (reinterpret_cast<uintptr_t>(Wk) & 15) ||
      (reinterpret_cast<uintptr_t>(zeros) & 15))
    return VF_EINVAL;
  const int K = 9 * Cin;
  // filters resident in LDS, the input staged once per 64 positions
  static const bool lds_path = !(std::getenv("VF_CONV_LDS") && std::getenv("VF_CONV_LDS")[0] == '0');
  if (lds_path && Cin == 64 && (W == 8 || W == 16 || W == 32 || W == 64) && H % (64 / W) == 0 && rows % 64 == 0) {
    const int nstages = (int)(rows / 64), otiles = (N + 63) / 64;
    const int spw = std::max(1, (int)(((int64_t)nstages * otiles + 255) / 256));
    dim3 grid(otiles, (nstages + spw - 1) / spw);
    // per-channel statistics of what is stored, if asked for and if that is the product itself
    float* st = (stats && stats_chunks && stats_rows && ep.alpha == 1.f && !ep.R && !ep.bias && !ep.c_is_bf16 &&
                 (int)grid.y <= kConvStatsChunks)
                    ? stats : nullptr;
    if (st) { *stats_chunks = (int)grid.y; *stats_rows = spw * 64; }
#define VF_CONV_LDS(WW)                                                                                   \
  case WW: {                                                                                              \
    constexpr int bytes = (9 * 64 * 64 + 2 * (64 / WW + 2) * (WW + 2) * 64) * 2;                          \
    static bool ready = false;                                                                            \
    if (!ready) {                                                                                         \
      VF_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&conv3x3_lds_kernel<WW>),                  \
                                 hipFuncAttributeMaxDynamicSharedMemorySize, bytes));                     \
      ready = true;                                                                                       \
    }                                                                                                     \
    conv3x3_lds_kernel<WW><<<grid, NT, bytes, s>>>(x, Wk, ldb, H, zeros, nstages, spw, N, ep, st);            \
  } break;
    switch (W) { VF_CONV_LDS(8) VF_CONV_LDS(16) VF_CONV_LDS(32) default: VF_CONV_LDS(64) }
#undef VF_CONV_LDS
    VF_LAUNCH_CHECK();
    return VF_OK;
  }
  dim3 grid((N + 63) / 64, (unsigned)((rows + 63) / 64), 1);
  ConvOperand cv{H, W, Cin, zeros};
  gemm_bf16_dl_kernel<4, true><<<grid, NT, 0, s>>>(x, Cin, Wk, ldb, (int)rows, N, K, K, 0, ep, cv);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_gemm_bf16_fold(const FoldArgs& fa, int64_t ld, int M, int N, float* C, int64_t ldc, hipStream_t s) {
  if (fa.count < 1 || fa.count > kFoldMax || M <= 0 || N <= 0 || !C) return VF_EINVAL;
  if ((N & 3) || (ldc & 3) || (ld & 7) || (reinterpret_cast<uintptr_t>(C) & 15)) return VF_EINVAL;
  for (int j = 0; j < fa.count; ++j) {
    if (!fa.A[j] || !fa.B[j] || fa.K[j] < 1 || fa.K[j] > 2 * BK || fa.K[j] > ld) return VF_EINVAL;
    if ((reinterpret_cast<uintptr_t>(fa.A[j]) & 15) || (reinterpret_cast<uintptr_t>(fa.B[j]) & 15)) return VF_EINVAL;
  }
  dim3 grid((N + 127) / 128, (M + 127) / 128);
  gemm_bf16_fold_kernel<<<grid, NT, 0, s>>>(fa, ld, M, N, C, ldc);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

}  // namespace vf
