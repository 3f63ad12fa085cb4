// Self-attention of one virtual node on the matrix cores: one workgroup per (sequence, head)
// keeps q, k, v of that head in LDS and runs all contractions with v_mfma_f32_32x32x16_bf16.
//   forward :  S = q k^T / sqrt(64);  P = softmax_rows(S) (fp32);  O = P v
//   backward:  dV = P^T dO;  dP = dO v^T;  dS = P (dP - rowsum(dP P));  dQ = dS k / 8;  dK = dS^T q / 8
// Head size 64, sequence length TS in {32, 64, 128} (TS/32 wavefronts, each owning 32 query
// rows); other shapes use the generic batched kernel.  Every operand that the MFMA reads along
// a non-contiguous axis is transposed while it is staged into LDS.
#include "vf_device.h"

namespace vf {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int DH = 64;            // head size
constexpr int LDE = DH + 8;       // LDS row of a [t][e] tile
// rows of a 32x32 accumulator tile held by register r of a lane
__device__ __forceinline__ int acc_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

__device__ __forceinline__ bf16x8 frag(const bf16_t* base, int ld, int row, int k) {
  return *reinterpret_cast<const bf16x8*>(&base[row * ld + k]);
}

// max / sum over the 32 lanes that share a row of an accumulator tile (one half of the wave)
__device__ __forceinline__ float half_max(float v) {
#pragma unroll
  for (int o = 16; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float half_sum(float v) {
#pragma unroll
  for (int o = 16; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Stage a [TS][64] bf16 window (row stride `rs` elements) into LDS as [t][e] (ld LDE).
template <int TS>
__device__ __forceinline__ void stage_rows(const bf16_t* __restrict__ g, int64_t rs, bf16_t* lds) {
  for (int v = threadIdx.x; v < TS * (DH / 8); v += blockDim.x) {
    const int t = v >> 3, e8 = (v & 7) * 8;
    *reinterpret_cast<u32x4*>(&lds[t * LDE + e8]) = *reinterpret_cast<const u32x4*>(&g[(int64_t)t * rs + e8]);
  }
}
// Stage the same window transposed: lds[e][t] (ld TS+8).  A thread takes two neighbouring rows
// t, t+1 and eight columns, and writes the pairs (e, t), (e, t+1) as one 32-bit word each; the
// threads of a wavefront run along t, so the words of one store instruction are neighbours in
// LDS (one bank each) -- single 16-bit stores 272 bytes apart had put sixteen lanes on two banks.
__device__ __forceinline__ uint32_t pick16(const u32x4& x, int u) { return (x[u >> 1] >> ((u & 1) * 16)) & 0xffffu; }
template <int TS>
__device__ __forceinline__ void stage_cols(const bf16_t* __restrict__ g, int64_t rs, bf16_t* lds) {
  constexpr int LDT = TS + 8;
  for (int v = threadIdx.x; v < (TS / 2) * (DH / 8); v += blockDim.x) {
    const int t = 2 * (v % (TS / 2)), e8 = (v / (TS / 2)) * 8;
    const u32x4 x0 = *reinterpret_cast<const u32x4*>(&g[(int64_t)t * rs + e8]);
    const u32x4 x1 = *reinterpret_cast<const u32x4*>(&g[(int64_t)(t + 1) * rs + e8]);
#pragma unroll
    for (int u = 0; u < 8; ++u)
      *reinterpret_cast<uint32_t*>(&lds[(e8 + u) * LDT + t]) = pick16(x0, u) | (pick16(x1, u) << 16);
  }
}

template <int TS>
__global__ __launch_bounds__(2 * TS) void attn_fwd_kernel(const bf16_t* __restrict__ qkv, int d, int n_heads,
                                                          bf16_t* __restrict__ prob, bf16_t* __restrict__ om,
                                                          float scale) {
  constexpr int LDT = TS + 8;
  constexpr int JT = TS / 32;                       // 32-wide tiles along the keys
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  bf16_t* Qs = smem;                                // [TS][LDE]
  bf16_t* Ks = Qs + TS * LDE;                       // [TS][LDE]
  bf16_t* Vt = Ks + TS * LDE;                       // [DH][LDT]
  bf16_t* Ps = smem;                                // [TS][LDT], overlays Qs/Ks after the scores
  static_assert(TS * LDT <= 2 * TS * LDE, "P fits over q and k");

  const int bh = blockIdx.x, seq = bh / n_heads, head = bh % n_heads;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int64_t rs = 3 * (int64_t)d;
  const bf16_t* qg = qkv + (int64_t)seq * TS * rs + head * DH;
  stage_rows<TS>(qg, rs, Qs);
  stage_rows<TS>(qg + d, rs, Ks);
  stage_cols<TS>(qg + 2 * d, rs, Vt);
  __syncthreads();

  // scores of this wave's 32 query rows against all keys
  f32x16 s[JT];
#pragma unroll
  for (int jt = 0; jt < JT; ++jt) {
#pragma unroll
    for (int r = 0; r < 16; ++r) s[jt][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < DH / 16; ++ks) {
      const int k = ks * 16 + (lane >> 5) * 8;
      s[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(Qs, LDE, 32 * w + (lane & 31), k),
                                                      frag(Ks, LDE, 32 * jt + (lane & 31), k), s[jt], 0, 0, 0);
    }
  }
  // row softmax in fp32: register r of every tile belongs to row acc_row(r, lane)
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    float m = -INFINITY;
#pragma unroll
    for (int jt = 0; jt < JT; ++jt) m = fmaxf(m, s[jt][r] * scale);
    m = half_max(m);
    float sum = 0.f;
#pragma unroll
    for (int jt = 0; jt < JT; ++jt) {
      s[jt][r] = expf(s[jt][r] * scale - m);
      sum += s[jt][r];
    }
    const float inv = 1.0f / half_sum(sum);
#pragma unroll
    for (int jt = 0; jt < JT; ++jt) s[jt][r] *= inv;
  }
  __syncthreads();                                  // every wave is done with Qs / Ks
  bf16_t* pg = prob + (int64_t)bh * TS * TS;
#pragma unroll
  for (int jt = 0; jt < JT; ++jt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = 32 * w + acc_row(r, lane), col = 32 * jt + (lane & 31);
      const bf16_t p = f32_to_bf16(s[jt][r]);
      Ps[row * LDT + col] = p;
      pg[row * TS + col] = p;
    }
  __syncthreads();

  // O = P V for this wave's rows
#pragma unroll
  for (int et = 0; et < DH / 32; ++et) {
    f32x16 o;
#pragma unroll
    for (int r = 0; r < 16; ++r) o[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < TS / 16; ++ks) {
      const int k = ks * 16 + (lane >> 5) * 8;
      o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(Ps, LDT, 32 * w + (lane & 31), k),
                                                  frag(Vt, LDT, 32 * et + (lane & 31), k), o, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = 32 * w + acc_row(r, lane);
      om[((int64_t)seq * TS + row) * d + head * DH + 32 * et + (lane & 31)] = f32_to_bf16(o[r]);
    }
  }
}

template <int TS>
__global__ __launch_bounds__(2 * TS) void attn_bwd_kernel(const float* __restrict__ dO,
                                                          const bf16_t* __restrict__ qkv,
                                                          const bf16_t* __restrict__ prob, int d, int n_heads,
                                                          bf16_t* __restrict__ dqkv, float scale) {
  constexpr int LDT = TS + 8;
  constexpr int JT = TS / 32;
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  bf16_t* Kt = smem;                                // [DH][LDT]   k transposed
  bf16_t* Qt = Kt + DH * LDT;                       // [DH][LDT]   q transposed
  bf16_t* Vs = Qt + DH * LDT;                       // [TS][LDE]   v
  bf16_t* Pt = Vs + TS * LDE;                       // [TS][LDT]   P transposed; later dS transposed, in place
  bf16_t* dOt = Pt + TS * LDT;                      // [DH][LDT]   dO transposed
  bf16_t* dOs = dOt + DH * LDT;                     // [TS][LDE]   dO
  bf16_t* dSs = dOt;                                // [TS][LDT]   dS, overlays dOt + dOs
  static_assert(TS * LDT <= DH * LDT + TS * LDE, "dS fits over the two dO tiles");

  const int bh = blockIdx.x, seq = bh / n_heads, head = bh % n_heads;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int64_t rs = 3 * (int64_t)d;
  const bf16_t* qg = qkv + (int64_t)seq * TS * rs + head * DH;
  stage_cols<TS>(qg, rs, Qt);
  stage_cols<TS>(qg + d, rs, Kt);
  stage_rows<TS>(qg + 2 * d, rs, Vs);
  // dO: fp32 [t][e] -> bf16, both orientations: rows as they are (16-byte stores), and transposed
  // with the pair-of-rows mapping of stage_cols
  const float* dog = dO + (int64_t)seq * TS * d + head * DH;
  for (int v = threadIdx.x; v < TS * (DH / 8); v += blockDim.x) {
    const int t = v >> 3, e8 = (v & 7) * 8;
    const float4 a = *reinterpret_cast<const float4*>(&dog[(int64_t)t * d + e8]);
    const float4 b = *reinterpret_cast<const float4*>(&dog[(int64_t)t * d + e8 + 4]);
    u32x4 h;
    h[0] = (uint32_t)f32_to_bf16(a.x) | ((uint32_t)f32_to_bf16(a.y) << 16);
    h[1] = (uint32_t)f32_to_bf16(a.z) | ((uint32_t)f32_to_bf16(a.w) << 16);
    h[2] = (uint32_t)f32_to_bf16(b.x) | ((uint32_t)f32_to_bf16(b.y) << 16);
    h[3] = (uint32_t)f32_to_bf16(b.z) | ((uint32_t)f32_to_bf16(b.w) << 16);
    *reinterpret_cast<u32x4*>(&dOs[t * LDE + e8]) = h;
  }
  for (int v = threadIdx.x; v < (TS / 2) * (DH / 8); v += blockDim.x) {
    const int t = 2 * (v % (TS / 2)), e8 = (v / (TS / 2)) * 8;
    const float4 a0 = *reinterpret_cast<const float4*>(&dog[(int64_t)t * d + e8]);
    const float4 b0 = *reinterpret_cast<const float4*>(&dog[(int64_t)t * d + e8 + 4]);
    const float4 a1 = *reinterpret_cast<const float4*>(&dog[(int64_t)(t + 1) * d + e8]);
    const float4 b1 = *reinterpret_cast<const float4*>(&dog[(int64_t)(t + 1) * d + e8 + 4]);
    const float f0[8] = {a0.x, a0.y, a0.z, a0.w, b0.x, b0.y, b0.z, b0.w};
    const float f1[8] = {a1.x, a1.y, a1.z, a1.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
    for (int u = 0; u < 8; ++u)
      *reinterpret_cast<uint32_t*>(&dOt[(e8 + u) * LDT + t]) =
          (uint32_t)f32_to_bf16(f0[u]) | ((uint32_t)f32_to_bf16(f1[u]) << 16);
  }
  // P: [q][j] in memory -> Pt[j][q], two query rows per thread, words along q
  const bf16_t* pg = prob + (int64_t)bh * TS * TS;
  for (int v = threadIdx.x; v < (TS / 2) * (TS / 8); v += blockDim.x) {
    const int q = 2 * (v % (TS / 2)), j8 = (v / (TS / 2)) * 8;
    const u32x4 x0 = *reinterpret_cast<const u32x4*>(&pg[q * TS + j8]);
    const u32x4 x1 = *reinterpret_cast<const u32x4*>(&pg[(q + 1) * TS + j8]);
#pragma unroll
    for (int u = 0; u < 8; ++u)
      *reinterpret_cast<uint32_t*>(&Pt[(j8 + u) * LDT + q]) = pick16(x0, u) | (pick16(x1, u) << 16);
  }
  __syncthreads();

  const int64_t orow = (int64_t)seq * TS;
  // dV[j, e] = sum_q P[q, j] dO[q, e]: this wave's 32 key rows
#pragma unroll
  for (int et = 0; et < DH / 32; ++et) {
    f32x16 a;
#pragma unroll
    for (int r = 0; r < 16; ++r) a[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < TS / 16; ++ks) {
      const int k = ks * 16 + (lane >> 5) * 8;
      a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(Pt, LDT, 32 * w + (lane & 31), k),
                                                  frag(dOt, LDT, 32 * et + (lane & 31), k), a, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r)
      dqkv[(orow + 32 * w + acc_row(r, lane)) * rs + 2 * d + head * DH + 32 * et + (lane & 31)] = f32_to_bf16(a[r]);
  }
  // dP[q, j] = sum_e dO[q, e] v[j, e]: this wave's 32 query rows
  f32x16 dp[JT];
#pragma unroll
  for (int jt = 0; jt < JT; ++jt) {
#pragma unroll
    for (int r = 0; r < 16; ++r) dp[jt][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < DH / 16; ++ks) {
      const int k = ks * 16 + (lane >> 5) * 8;
      dp[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(dOs, LDE, 32 * w + (lane & 31), k),
                                                       frag(Vs, LDE, 32 * jt + (lane & 31), k), dp[jt], 0, 0, 0);
    }
  }
  // dS = P (dP - sum_j dP P), row by row; P(q, j) is read back from Pt[j][q]
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int q = 32 * w + acc_row(r, lane);
    float p[JT];
    float dot = 0.f;
#pragma unroll
    for (int jt = 0; jt < JT; ++jt) {
      p[jt] = bf16_to_f32(Pt[(32 * jt + (lane & 31)) * LDT + q]);
      dot = fmaf(dp[jt][r], p[jt], dot);
    }
    dot = half_sum(dot);
#pragma unroll
    for (int jt = 0; jt < JT; ++jt) dp[jt][r] = p[jt] * (dp[jt][r] - dot);
  }
  __syncthreads();                                  // all waves are done with Pt, dOt, dOs
#pragma unroll
  for (int jt = 0; jt < JT; ++jt)
#pragma unroll
    for (int r = 0; r < 16; r += 2) {               // registers r, r+1: query rows q, q+1 (q even)
      const int q = 32 * w + acc_row(r, lane), j = 32 * jt + (lane & 31);
      const bf16_t h0 = f32_to_bf16(dp[jt][r]), h1 = f32_to_bf16(dp[jt][r + 1]);
      dSs[q * LDT + j] = h0;
      dSs[(q + 1) * LDT + j] = h1;
      *reinterpret_cast<uint32_t*>(&Pt[j * LDT + q]) = (uint32_t)h0 | ((uint32_t)h1 << 16);   // dS transposed, over P transposed
    }
  __syncthreads();
  // dQ[q, e] = scale sum_j dS[q, j] k[j, e];  dK[j, e] = scale sum_q dS[q, j] q[q, e]
#pragma unroll
  for (int et = 0; et < DH / 32; ++et) {
    f32x16 aq, ak;
#pragma unroll
    for (int r = 0; r < 16; ++r) { aq[r] = 0.f; ak[r] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < TS / 16; ++ks) {
      const int k = ks * 16 + (lane >> 5) * 8;
      aq = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(dSs, LDT, 32 * w + (lane & 31), k),
                                                   frag(Kt, LDT, 32 * et + (lane & 31), k), aq, 0, 0, 0);
      ak = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(Pt, LDT, 32 * w + (lane & 31), k),
                                                   frag(Qt, LDT, 32 * et + (lane & 31), k), ak, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int64_t row = (orow + 32 * w + acc_row(r, lane)) * rs + head * DH + 32 * et + (lane & 31);
      dqkv[row] = f32_to_bf16(aq[r] * scale);
      dqkv[row + d] = f32_to_bf16(ak[r] * scale);
    }
  }
}

template <int TS>
size_t fwd_lds() { return (size_t)(2 * TS * LDE + DH * (TS + 8)) * sizeof(bf16_t); }
template <int TS>
size_t bwd_lds() {
  return (size_t)(2 * DH * (TS + 8) + TS * LDE + TS * (TS + 8) + DH * (TS + 8) + TS * LDE) * sizeof(bf16_t);
}

template <int TS>
int set_lds_limits() {
  static bool done = false;      // per process; the attribute is per function
  if (done) return VF_OK;
  VF_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_fwd_kernel<TS>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)fwd_lds<TS>()));
  VF_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bwd_kernel<TS>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)bwd_lds<TS>()));
  done = true;
  return VF_OK;
}

}  // namespace

bool attn_mfma_supported(int seq_len, int d_head) {
  return d_head == DH && (seq_len == 32 || seq_len == 64 || seq_len == 128);
}

int launch_attn_fwd(const bf16_t* qkv, int n_seq, int seq_len, int d, int n_heads, bf16_t* prob, bf16_t* om,
                    float scale, hipStream_t s) {
  if (!attn_mfma_supported(seq_len, d / n_heads) || n_seq <= 0 || (d & 7)) return VF_EINVAL;
  const int grid = n_seq * n_heads;
#define VF_AF(TS)                                                                                  \
  case TS:                                                                                         \
    VF_TRY(set_lds_limits<TS>());                                                                  \
    attn_fwd_kernel<TS><<<grid, 2 * TS, fwd_lds<TS>(), s>>>(qkv, d, n_heads, prob, om, scale);      \
    break;
  switch (seq_len) { VF_AF(32) VF_AF(64) VF_AF(128) default: return VF_EINVAL; }
#undef VF_AF
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_attn_bwd(const float* dO, const bf16_t* qkv, const bf16_t* prob, int n_seq, int seq_len, int d,
                    int n_heads, bf16_t* dqkv, float scale, hipStream_t s) {
  if (!attn_mfma_supported(seq_len, d / n_heads) || n_seq <= 0 || (d & 7)) return VF_EINVAL;
  const int grid = n_seq * n_heads;
#define VF_AB(TS)                                                                                  \
  case TS:                                                                                         \
    VF_TRY(set_lds_limits<TS>());                                                                  \
    attn_bwd_kernel<TS><<<grid, 2 * TS, bwd_lds<TS>(), s>>>(dO, qkv, prob, d, n_heads, dqkv, scale); \
    break;
  switch (seq_len) { VF_AB(32) VF_AB(64) VF_AB(128) default: return VF_EINVAL; }
#undef VF_AB
  VF_LAUNCH_CHECK();
  return VF_OK;
}

}  // namespace vf
