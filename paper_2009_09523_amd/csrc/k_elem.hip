// Layout kernels: bf16 transposes and the fp32 -> bf16 weight copies the GEMMs read.
#include "vf_device.h"

namespace vf {
namespace {

constexpr int TS = 32;   // tile side; 256 threads = 32 x 8
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

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

// out[c*ldo + r] = in[r*ldi + c] for bf16, 64x64 tiles, 16 bytes per lane on both sides (eight
// lanes cover 128 contiguous bytes of an input row, and of an output row).  Loads go to clamped,
// always valid addresses and come first, so both of a thread's loads are in flight together.
// Requires C % 8 == 0, ldi % 8 == 0, ldo % 8 == 0, 16-byte aligned bases, and output rows that
// may be written up to R rounded to 8 (the rows past R receive copies of row R-1).
__device__ __forceinline__ void transpose64_body(const bf16_t* __restrict__ in, int64_t ldi,
                                                 bf16_t* __restrict__ out, int64_t ldo, int R, int C, int bx, int by) {
  __shared__ __attribute__((aligned(16))) bf16_t tile[64][64 + 8];
  const int r0 = by * 64, c0 = bx * 64;
  const int v = threadIdx.x & 7, row = threadIdx.x >> 3;     // 8 vectors per row, 32 rows per pass
  u32x4 x[2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
    x[i] = *reinterpret_cast<const u32x4*>(&in[(int64_t)min(r0 + row + 32 * i, R - 1) * ldi + min(c0 + 8 * v, C - 8)]);
#pragma unroll
  for (int i = 0; i < 2; ++i) *reinterpret_cast<u32x4*>(&tile[row + 32 * i][8 * v]) = x[i];
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int col = (threadIdx.x >> 3) + 32 * i;             // output row = input column
    const int rb = 8 * (threadIdx.x & 7);                    // eight input rows -> one 16-byte vector
    u32x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      o[e] = (uint32_t)tile[rb + 2 * e][col] | ((uint32_t)tile[rb + 2 * e + 1][col] << 16);
    if (c0 + col < C && r0 + rb < R)
      *reinterpret_cast<u32x4*>(&out[(int64_t)(c0 + col) * ldo + r0 + rb]) = o;
  }
}

__global__ __launch_bounds__(256) void transpose64_kernel(const bf16_t* __restrict__ in, int64_t ldi,
                                                          bf16_t* __restrict__ out, int64_t ldo, int R, int C) {
  transpose64_body(in, ldi, out, ldo, R, C, blockIdx.x, blockIdx.y);
}
// Several matrices of R rows in one launch: blockIdx.x runs over the column tiles of all of them.
__global__ __launch_bounds__(256) void transpose64_jobs_kernel(TransposeJobs tj) {
  int j = 0, first = 0;
  while (j < tj.count - 1 && (int)blockIdx.x >= first + (tj.C[j] + 63) / 64) { first += (tj.C[j] + 63) / 64; ++j; }
  transpose64_body(tj.in[j], tj.ldi[j], tj.out[j], tj.ldo, tj.R, tj.C[j], blockIdx.x - first, blockIdx.y);
}

// fp32 [R, C] -> bf16 natural copy [R, ldn] and transposed copy [C, ldt], 64x64 tiles.
// Every thread reads 16 bytes and writes 8 bytes at a time in both orientations.
// Requires C % 4 == 0, ldi % 4 == 0, ldn % 4 == 0, ldt % 4 == 0 and 16-byte aligned bases.
__global__ __launch_bounds__(256) void cast_weight_kernel(const float* __restrict__ in, int64_t ldi,
                                                          bf16_t* __restrict__ nat, int64_t ldn,
                                                          bf16_t* __restrict__ tr, int64_t ldt, int R, int C) {
  __shared__ bf16_t tile[64][64 + 2];
  const int q = threadIdx.x & 15, g = threadIdx.x >> 4;      // 16 quads per row, 16 row groups
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  // loads at clamped (always valid) positions first, all four in flight together (C % 4 == 0,
  // so C - 4 starts a whole quad)
  float4 vin[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    vin[i] = load4_stream(&in[(int64_t)min(r0 + g + 16 * i, R - 1) * ldi + min(c0 + 4 * q, C - 4)]);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int rl = g + 16 * i, r = r0 + rl, c = c0 + 4 * q;
    bf16_t h[4] = {0, 0, 0, 0};
    if (r < R && c < C) {
      const float4 v = vin[i];
      h[0] = f32_to_bf16(v.x); h[1] = f32_to_bf16(v.y); h[2] = f32_to_bf16(v.z); h[3] = f32_to_bf16(v.w);
      uint2 pk;
      pk.x = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
      pk.y = (uint32_t)h[2] | ((uint32_t)h[3] << 16);
      *reinterpret_cast<uint2*>(&nat[(int64_t)r * ldn + c]) = pk;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) tile[rl][4 * q + u] = h[u];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int cl = g + 16 * i, c = c0 + cl, r = r0 + 4 * q;
    if (c < C && r < R) {      // R % 4 == 0 is not required: rows past R inside the quad are padding of ldt
      uint2 pk;
      pk.x = (uint32_t)tile[4 * q][cl] | ((uint32_t)tile[4 * q + 1][cl] << 16);
      pk.y = (uint32_t)tile[4 * q + 2][cl] | ((uint32_t)tile[4 * q + 3][cl] << 16);
      *reinterpret_cast<uint2*>(&tr[(int64_t)c * ldt + r]) = pk;
    }
  }
}

// The same transpose for every node of a fold window (blockIdx.z = node).
__global__ __launch_bounds__(256) void transpose_nodes_kernel(NodeList nl, int64_t ldi, int64_t ldo, int C) {
  __shared__ bf16_t tile[TS][TS + 2];
  const int j = blockIdx.z;
  const int R = nl.rows[j];
  const int r0 = blockIdx.y * TS, c0 = blockIdx.x * TS;
  if (r0 >= R) return;
  const bf16_t* __restrict__ in = nl.src[j];
  bf16_t* __restrict__ out = nl.dst[j];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
#pragma unroll
  for (int i = 0; i < TS; i += 8) {
    const int r = r0 + ty + i, c = c0 + tx;
    if (r < R && c < C) tile[ty + i][tx] = in[(int64_t)r * ldi + c];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < TS; i += 8) {
    const int c = c0 + ty + i, r = r0 + tx;
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
  const bool wide = (C & 7) == 0 && (ldi & 7) == 0 && (ldo & 7) == 0 && ldo >= ((R + 7) & ~7) &&
                    (reinterpret_cast<uintptr_t>(in) & 15) == 0 && (reinterpret_cast<uintptr_t>(out) & 15) == 0;
  if (wide) {
    dim3 grid64((C + 63) / 64, (R + 63) / 64);
    transpose64_kernel<<<grid64, 256, 0, s>>>(in, ldi, out, ldo, R, C);
    VF_LAUNCH_CHECK();
    return VF_OK;
  }
  dim3 grid((C + TS - 1) / TS, (R + TS - 1) / TS);
  transpose_kernel<bf16_t><<<grid, 256, 0, s>>>(in, ldi, out, ldo, nullptr, 0, R, C);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_transpose_bf16_jobs(const TransposeJobs& tj, hipStream_t s) {
  if (tj.count < 1 || tj.count > kTransposeJobs || tj.R <= 0 || (tj.ldo & 7) || tj.ldo < ((tj.R + 7) & ~7)) return VF_EINVAL;
  int tiles = 0;
  for (int j = 0; j < tj.count; ++j) {
    if (!tj.in[j] || !tj.out[j] || tj.C[j] <= 0 || (tj.C[j] & 7) || (tj.ldi[j] & 7) || tj.ldi[j] < tj.C[j] ||
        (reinterpret_cast<uintptr_t>(tj.in[j]) & 15) || (reinterpret_cast<uintptr_t>(tj.out[j]) & 15))
      return VF_EINVAL;
    tiles += (tj.C[j] + 63) / 64;
  }
  dim3 grid(tiles, (tj.R + 63) / 64);
  transpose64_jobs_kernel<<<grid, 256, 0, s>>>(tj);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_transpose_nodes(const NodeList& nl, int64_t ldi, int64_t ldo, int C, hipStream_t s) {
  if (nl.count < 1 || nl.count > kFoldMax || C <= 0) return VF_EINVAL;
  int max_rows = 0;
  for (int j = 0; j < nl.count; ++j) {
    if (!nl.src[j] || !nl.dst[j] || nl.rows[j] < 1 || nl.rows[j] > ldo || C > ldi) return VF_EINVAL;
    max_rows = nl.rows[j] > max_rows ? nl.rows[j] : max_rows;
  }
  dim3 grid((C + TS - 1) / TS, (max_rows + TS - 1) / TS, nl.count);
  transpose_nodes_kernel<<<grid, 256, 0, s>>>(nl, ldi, ldo, C);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_cast_weight(const float* w, int R, int C, bf16_t* nat, int64_t ldn, bf16_t* tr,
                       int64_t ldt, hipStream_t s) {
  if (R <= 0 || C <= 0) return VF_OK;
  const bool vec = (C & 3) == 0 && (ldn & 3) == 0 && (ldt & 3) == 0 &&
                   (reinterpret_cast<uintptr_t>(w) & 15) == 0 && (reinterpret_cast<uintptr_t>(nat) & 7) == 0 &&
                   (reinterpret_cast<uintptr_t>(tr) & 7) == 0;
  if (vec) {
    dim3 grid((C + 63) / 64, (R + 63) / 64);
    cast_weight_kernel<<<grid, 256, 0, s>>>(w, C, nat, ldn, tr, ldt, R, C);
  } else {
    dim3 grid((C + TS - 1) / TS, (R + TS - 1) / TS);
    transpose_kernel<float><<<grid, 256, 0, s>>>(w, C, tr, ldt, nat, ldn, R, C);
  }
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
