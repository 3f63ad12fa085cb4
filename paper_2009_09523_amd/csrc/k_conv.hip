// Kernels of the convolutional workload family (a residual network of 3x3 convolutions, stride 1,
// zero padding 1, NHWC): the convolution itself is a product (k_gemm_bf16.hip) over patch rows
// written by im2col; here are im2col, the filter copies, BatchNorm over the positions of one
// virtual node (Section 4.1: statistics of the pass that is running, i.e. of the node's n*H*W
// rows), the mean over positions, and the folding of contraction slabs into a gradient.
//
// Tall-matrix reductions ([rows, C] with rows = n*H*W in the 10^5 and C <= 256) go in two steps:
// per-chunk partial results, then one small kernel that combines the chunks in chunk order, so
// results do not depend on scheduling.  Loads go to clamped, always valid addresses ahead of any
// selection, so that all of a thread's loads are in flight together.
#include <algorithm>

#include "vf_device.h"

namespace vf {
namespace {

constexpr int NT = 256;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ---- im2col ---------------------------------------------------------------------------------
// cols[r, (kh*3+kw)*C + c] = x[n, h+kh-1, w+kw-1, c] (0 outside the image), r = (n*H + h)*W + w;
// columns 9C .. Kp-1 (padding of the row to a multiple of 8) are written as 0.
// Vector form: C % 8 == 0, one 16-byte piece per thread.
__global__ __launch_bounds__(NT) void im2col8_kernel(const bf16_t* __restrict__ x, int64_t rows, int H, int W, int C,
                                                     bf16_t* __restrict__ cols, int64_t Kp) {
  const int c8n = C >> 3;
  const int64_t per_row = 9 * c8n;
  const int64_t idx = (int64_t)blockIdx.x * NT + threadIdx.x;
  if (idx >= rows * per_row) return;
  const int64_t r = idx / per_row;
  const int rem = (int)(idx - r * per_row);
  const int tap = rem / c8n, c8 = rem - tap * c8n;
  const int kh = tap / 3, kw = tap - 3 * kh;
  const int w = (int)(r % W);
  const int h = (int)((r / W) % H);
  const int hh = h + kh - 1, ww = w + kw - 1;
  const bool in = hh >= 0 && hh < H && ww >= 0 && ww < W;
  // the source row of an inside tap is r + (kh-1)*W + (kw-1): same image, since hh and ww are inside
  const int64_t src = in ? r + (int64_t)(kh - 1) * W + (kw - 1) : r;
  u32x4 v = *reinterpret_cast<const u32x4*>(&x[src * C + 8 * c8]);
  if (!in) v = u32x4{0u, 0u, 0u, 0u};
  *reinterpret_cast<u32x4*>(&cols[r * Kp + (int64_t)tap * C + 8 * c8]) = v;
}

// Scalar form (any C; the first layer with 3 input channels): one thread per (row, column < Kp).
__global__ __launch_bounds__(NT) void im2col1_kernel(const bf16_t* __restrict__ x, int64_t rows, int H, int W, int C,
                                                     bf16_t* __restrict__ cols, int Kp) {
  const int64_t idx = (int64_t)blockIdx.x * NT + threadIdx.x;
  if (idx >= rows * Kp) return;
  const int64_t r = idx / Kp;
  const int k = (int)(idx - r * Kp);
  bf16_t v = 0;
  if (k < 9 * C) {
    const int tap = k / C, c = k - tap * C;
    const int kh = tap / 3, kw = tap - 3 * kh;
    const int w = (int)(r % W);
    const int h = (int)((r / W) % H);
    const int hh = h + kh - 1, ww = w + kw - 1;
    if (hh >= 0 && hh < H && ww >= 0 && ww < W) v = x[(r + (int64_t)(kh - 1) * W + (kw - 1)) * C + c];
  }
  cols[idx] = v;
}

// The transposed patch matrix straight from the transposed activation xT [C, ldx] (row c holds
// channel c of all positions): colsT[(tap*C + c), r] = xT[c, r + (kh-1)*W + (kw-1)] inside the
// image, 0 outside and for r >= rows (the padding of a row up to ldo).  Row (tap, c) is row c
// shifted by the tap's offset, so reads and writes both run along the row; one thread writes 8
// consecutive positions (16 bytes).  ldo % 8 == 0.
__global__ __launch_bounds__(NT) void im2colT_kernel(const bf16_t* __restrict__ xT, int64_t ldx, int64_t rows, int H, int W,
                                                     int C, bf16_t* __restrict__ colsT, int64_t ldo) {
  const int64_t nvec = (rows + 7) >> 3;
  const int64_t idx = (int64_t)blockIdx.x * NT + threadIdx.x;
  if (idx >= (int64_t)9 * C * nvec) return;
  const int k = (int)(idx / nvec);
  const int64_t r0 = (idx - (int64_t)k * nvec) << 3;
  const int tap = k / C, c = k - tap * C;
  const int kh = tap / 3, kw = tap - 3 * kh;
  const int64_t shift = (int64_t)(kh - 1) * W + (kw - 1);
  const bf16_t* src = xT + (int64_t)c * ldx;
  int w = (int)(r0 % W);
  int h = (int)((r0 / W) % H);
  uint32_t out[4] = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int64_t r = r0 + e;
    const int hh = h + kh - 1, ww = w + kw - 1;
    const bool in = r < rows && hh >= 0 && hh < H && ww >= 0 && ww < W;
    // an inside tap of position r is position r + shift of the same image; otherwise read r0 (valid) and drop it
    const bf16_t v = src[in ? r + shift : r0];
    out[e >> 1] |= in ? ((uint32_t)v << (16 * (e & 1))) : 0u;
    if (++w == W) { w = 0; if (++h == H) h = 0; }
  }
  *reinterpret_cast<u32x4*>(&colsT[(int64_t)k * ldo + r0]) = u32x4{out[0], out[1], out[2], out[3]};
}

// ---- filter copies ----------------------------------------------------------------------------
// nat[o, k] = bf16(Wf[o, k]) for k < 9*Cin (row pitch Kp; the padding stays as it is: zero);
// flip[c, (2-kh)*3*Cout + (2-kw)*Cout + o] = bf16(Wf[o, kh, kw, c]): the filters of the input
// gradient, which is the 3x3 convolution of the output gradient with the filters turned by 180
// degrees and input/output channels exchanged (row pitch Kpf).
__global__ __launch_bounds__(NT) void conv_weight_copies_kernel(const float* __restrict__ Wf, int Cout, int Cin,
                                                                bf16_t* __restrict__ nat, int Kp,
                                                                bf16_t* __restrict__ flip, int Kpf) {
  const int K = 9 * Cin;
  const int idx = blockIdx.x * NT + threadIdx.x;
  if (idx >= Cout * K) return;
  const int o = idx / K, k = idx - o * K;
  const bf16_t v = f32_to_bf16(Wf[idx]);
  nat[(int64_t)o * Kp + k] = v;
  if (flip) {
    const int tap = k / Cin, c = k - tap * Cin;
    const int kh = tap / 3, kw = tap - 3 * kh;
    flip[(int64_t)c * Kpf + ((2 - kh) * 3 + (2 - kw)) * Cout + o] = v;
  }
}

// ---- tall column reductions --------------------------------------------------------------------
// A workgroup owns CHUNK consecutive rows; a thread owns 4 consecutive columns (float4) of every
// RL-th row: NT threads = C/4 column groups x RL row lanes (C in {8, 16, 32, 64, 128, 256} uses
// all 256 threads; other C leave the last few idle).  C % 4 == 0, C <= 256.
constexpr int CHUNK = 256;       // rows per workgroup

struct Tall {
  int cg;        // column groups of 4 (C / 4)
  int rl;        // row lanes = NT / cg (at least 1)
  int passes;    // ceil(CHUNK / rl)
};
__device__ __forceinline__ Tall tall_shape(int C) {
  Tall t;
  t.cg = C >> 2;
  t.rl = NT / t.cg;
  if (t.rl < 1) t.rl = 1;
  t.passes = (CHUNK + t.rl - 1) / t.rl;
  return t;
}

// Combines the row lanes of one column group in lane order; result valid in row lane 0.
// (Threads past the last row lane take part in the barriers only.)
__device__ __forceinline__ float4 lanes_sum(float4 v, float4* red, int g, int lane, const Tall& t) {
  if (lane < t.rl) red[lane * t.cg + g] = v;
  __syncthreads();
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (lane == 0)
    for (int l = 0; l < t.rl; ++l) {
      const float4 a = red[l * t.cg + g];
      s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
    }
  __syncthreads();
  return s;
}

// Rows of a chunk are read PB per thread at a time, at clamped (always valid) row indices and
// ahead of the selection, so that PB loads per operand are in flight per thread.
constexpr int PB = 8;

// The two-group update of a mean and a sum of squared deviations: group B (nb rows, mean mb,
// deviations qb) joins group A (cnt, mean, m2).
__device__ __forceinline__ void join_stats(float& cnt, float& mean, float& m2, float nb, float mb, float qb) {
  if (nb <= 0.f) return;
  const float tot = cnt + nb;
  const float delta = mb - mean;
  mean = fmaf(delta, nb / tot, mean);
  m2 = m2 + qb + delta * delta * (cnt * nb / tot);
  cnt = tot;
}

// Per chunk and column: the mean of the chunk's rows and the sum of squared deviations from it.
// partial[(chunk*2 + 0)*C + c] = mean, partial[(chunk*2 + 1)*C + c] = M2.
__global__ __launch_bounds__(NT) void bn2d_stats_partial_kernel(const float* __restrict__ y, int64_t rows, int C,
                                                                float* __restrict__ partial) {
  extern __shared__ float4 red[];
  __shared__ float4 mean_s[64];
  const Tall t = tall_shape(C);
  const int g = threadIdx.x % t.cg, lane = threadIdx.x / t.cg;
  const bool active = lane < t.rl;
  const int64_t r0 = (int64_t)blockIdx.x * CHUNK;
  const int n = (int)min((int64_t)CHUNK, rows - r0);
  const float* yb = y + r0 * C + 4 * g;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int p0 = 0; p0 < t.passes; p0 += PB) {
    float4 v[PB];
#pragma unroll
    for (int u = 0; u < PB; ++u)
      v[u] = *reinterpret_cast<const float4*>(&yb[(int64_t)min(lane + (p0 + u) * t.rl, n - 1) * C]);
#pragma unroll
    for (int u = 0; u < PB; ++u)
      if (active && p0 + u < t.passes && lane + (p0 + u) * t.rl < n) {
        s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w;
      }
  }
  const float4 tot = lanes_sum(s, red, g, lane, t);
  if (lane == 0) {
    const float inv = 1.f / (float)n;
    mean_s[g] = make_float4(tot.x * inv, tot.y * inv, tot.z * inv, tot.w * inv);
  }
  __syncthreads();
  const float4 m = mean_s[g];
  float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int p0 = 0; p0 < t.passes; p0 += PB) {            // second read of the chunk: from the caches
    float4 v[PB];
#pragma unroll
    for (int u = 0; u < PB; ++u)
      v[u] = *reinterpret_cast<const float4*>(&yb[(int64_t)min(lane + (p0 + u) * t.rl, n - 1) * C]);
#pragma unroll
    for (int u = 0; u < PB; ++u)
      if (active && p0 + u < t.passes && lane + (p0 + u) * t.rl < n) {
        const float dx = v[u].x - m.x, dy = v[u].y - m.y, dz = v[u].z - m.z, dw = v[u].w - m.w;
        q.x = fmaf(dx, dx, q.x); q.y = fmaf(dy, dy, q.y); q.z = fmaf(dz, dz, q.z); q.w = fmaf(dw, dw, q.w);
      }
  }
  const float4 m2 = lanes_sum(q, red, g, lane, t);
  if (lane == 0) {
    *reinterpret_cast<float4*>(&partial[((int64_t)blockIdx.x * 2 + 0) * C + 4 * g]) = m;
    *reinterpret_cast<float4*>(&partial[((int64_t)blockIdx.x * 2 + 1) * C + 4 * g]) = m2;
  }
}

// Chunks combined in a fixed order: one workgroup of NTF threads, thread = (column, lane); a lane
// joins a contiguous run of chunks in chunk order (eight chunks' values in flight), then the lanes
// are joined in lane order.  Mean and
// biased variance over all rows; rstd; moving statistics of this device blended once per pass
// (Section 4.1).  C <= 256.
constexpr int NTF = 1024;
__global__ __launch_bounds__(NTF) void bn2d_stats_finish_kernel(const float* __restrict__ partial, int nchunk,
                                                               int rpc, int64_t rows, int C, float eps,
                                                               float* __restrict__ mean_out, float* __restrict__ rstd_out,
                                                               float* __restrict__ run_mean, float* __restrict__ run_var,
                                                               float run_mix) {
  __shared__ float sm[3][NTF];
  const int nl = NTF / C;                      // lanes per column
  const int c = threadIdx.x % C, lane = threadIdx.x / C;
  const bool active = lane < nl;
  const int per = (nchunk + nl - 1) / nl;
  const int k0 = lane * per, k1 = min(nchunk, k0 + per);
  float mean = 0.f, m2 = 0.f, cnt = 0.f;
  if (active) {
    int k = k0;
    for (; k + 7 < k1; k += 8) {               // eight chunks' values in flight, joined in order
      float mb[8], qb[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        mb[u] = partial[((int64_t)(k + u) * 2 + 0) * C + c];
        qb[u] = partial[((int64_t)(k + u) * 2 + 1) * C + c];
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
        join_stats(cnt, mean, m2, (float)min((int64_t)rpc, rows - (int64_t)(k + u) * rpc), mb[u], qb[u]);
    }
    for (; k < k1; ++k)
      join_stats(cnt, mean, m2, (float)min((int64_t)rpc, rows - (int64_t)k * rpc),
                 partial[((int64_t)k * 2 + 0) * C + c], partial[((int64_t)k * 2 + 1) * C + c]);
  }
  sm[0][threadIdx.x] = cnt; sm[1][threadIdx.x] = mean; sm[2][threadIdx.x] = m2;
  __syncthreads();
  if (lane != 0) return;
  for (int l = 1; l < nl; ++l) join_stats(cnt, mean, m2, sm[0][l * C + c], sm[1][l * C + c], sm[2][l * C + c]);
  const float var = m2 / cnt;
  mean_out[c] = mean;
  rstd_out[c] = 1.0f / sqrtf(var + eps);
  if (run_mean) {
    run_mean[c] = fmaf(run_mix, mean - run_mean[c], run_mean[c]);
    run_var[c] = fmaf(run_mix, var - run_var[c], run_var[c]);
  }
}

__device__ __forceinline__ float4 unpack4(uint2 p) {
  return make_float4(bf16_to_f32((bf16_t)(p.x & 0xffffu)), bf16_to_f32((bf16_t)(p.x >> 16)),
                     bf16_to_f32((bf16_t)(p.y & 0xffffu)), bf16_to_f32((bf16_t)(p.y >> 16)));
}
__device__ __forceinline__ uint2 pack4(float4 v) {
  uint2 p;
  p.x = (uint32_t)f32_to_bf16(v.x) | ((uint32_t)f32_to_bf16(v.y) << 16);
  p.y = (uint32_t)f32_to_bf16(v.z) | ((uint32_t)f32_to_bf16(v.w) << 16);
  return p;
}

// a = relu(gamma * (y - mean) * rstd + beta (+ skip)), stored bf16; one float4 of y per thread.
__global__ __launch_bounds__(NT) void bn2d_apply_fwd_kernel(const float* __restrict__ y, int64_t n4, int C,
                                                            const float* __restrict__ gamma, const float* __restrict__ beta,
                                                            int round_params, const float* __restrict__ mean,
                                                            const float* __restrict__ rstd, const bf16_t* __restrict__ skip,
                                                            bf16_t* __restrict__ a) {
  const int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x;
  if (i >= n4) return;
  const int c = (int)((i * 4) % C);
  const float4 v = reinterpret_cast<const float4*>(y)[i];
  float4 g = *reinterpret_cast<const float4*>(&gamma[c]);
  float4 b = *reinterpret_cast<const float4*>(&beta[c]);
  const float4 m = *reinterpret_cast<const float4*>(&mean[c]);
  const float4 r = *reinterpret_cast<const float4*>(&rstd[c]);
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (skip) s = unpack4(reinterpret_cast<const uint2*>(skip)[i]);
  if (round_params) {
    g.x = round_bf16(g.x); g.y = round_bf16(g.y); g.z = round_bf16(g.z); g.w = round_bf16(g.w);
    b.x = round_bf16(b.x); b.y = round_bf16(b.y); b.z = round_bf16(b.z); b.w = round_bf16(b.w);
  }
  float4 o;
  o.x = fmaxf(fmaf(g.x, (v.x - m.x) * r.x, b.x) + s.x, 0.f);
  o.y = fmaxf(fmaf(g.y, (v.y - m.y) * r.y, b.y) + s.y, 0.f);
  o.z = fmaxf(fmaf(g.z, (v.z - m.z) * r.z, b.z) + s.z, 0.f);
  o.w = fmaxf(fmaf(g.w, (v.w - m.w) * r.w, b.w) + s.w, 0.f);
  reinterpret_cast<uint2*>(a)[i] = pack4(o);
}

// Backward, step 1: per chunk and column, the sums over the chunk's rows of dpre and of
// dpre * xhat, with dpre = da where the ReLU was open (its stored output a > 0) and
// xhat = (y - mean) * rstd.  partial[(chunk*2 + 0)*C + c] = sum dpre, [.. + 1 ..] = sum dpre*xhat.
__global__ __launch_bounds__(NT) void bn2d_bwd_partial_kernel(const float* __restrict__ da, const bf16_t* __restrict__ a,
                                                              const float* __restrict__ y, int64_t rows, int C,
                                                              const float* __restrict__ mean, const float* __restrict__ rstd,
                                                              float* __restrict__ partial) {
  extern __shared__ float4 red[];
  const Tall t = tall_shape(C);
  const int g = threadIdx.x % t.cg, lane = threadIdx.x / t.cg;
  const bool active = lane < t.rl;
  const int64_t r0 = (int64_t)blockIdx.x * CHUNK;
  const int n = (int)min((int64_t)CHUNK, rows - r0);
  const int64_t base = r0 * C + 4 * g;
  const float4 m = *reinterpret_cast<const float4*>(&mean[4 * g]);
  const float4 rs = *reinterpret_cast<const float4*>(&rstd[4 * g]);
  float4 sb = make_float4(0.f, 0.f, 0.f, 0.f), sg = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int p0 = 0; p0 < t.passes; p0 += PB) {
    float4 d[PB], v[PB];
    uint2 o2[PB];
#pragma unroll
    for (int u = 0; u < PB; ++u) {
      const int64_t at = base + (int64_t)min(lane + (p0 + u) * t.rl, n - 1) * C;
      d[u] = *reinterpret_cast<const float4*>(&da[at]);
      v[u] = *reinterpret_cast<const float4*>(&y[at]);
      o2[u] = *reinterpret_cast<const uint2*>(&a[at]);
    }
#pragma unroll
    for (int u = 0; u < PB; ++u)
      if (active && p0 + u < t.passes && lane + (p0 + u) * t.rl < n) {
        const float4 o = unpack4(o2[u]);
        const float dx = o.x > 0.f ? d[u].x : 0.f, dy = o.y > 0.f ? d[u].y : 0.f;
        const float dz = o.z > 0.f ? d[u].z : 0.f, dw = o.w > 0.f ? d[u].w : 0.f;
        sb.x += dx; sb.y += dy; sb.z += dz; sb.w += dw;
        sg.x = fmaf(dx, (v[u].x - m.x) * rs.x, sg.x); sg.y = fmaf(dy, (v[u].y - m.y) * rs.y, sg.y);
        sg.z = fmaf(dz, (v[u].z - m.z) * rs.z, sg.z); sg.w = fmaf(dw, (v[u].w - m.w) * rs.w, sg.w);
      }
  }
  const float4 tb = lanes_sum(sb, red, g, lane, t);
  const float4 tg = lanes_sum(sg, red, g, lane, t);
  if (lane == 0) {
    *reinterpret_cast<float4*>(&partial[((int64_t)blockIdx.x * 2 + 0) * C + 4 * g]) = tb;
    *reinterpret_cast<float4*>(&partial[((int64_t)blockIdx.x * 2 + 1) * C + 4 * g]) = tg;
  }
}

// Step 2: one workgroup, thread = (column, lane); a lane adds a contiguous run of chunks in chunk
// order, the lanes are added in lane order.  The sums go to sums[0][c] (dbeta) and sums[1][c]
// (dgamma) for the apply kernel, and, weighted, into the gradient (Section 3.2 step 3,
// Section 5.2).  C <= 256.
__global__ __launch_bounds__(NTF) void bn2d_bwd_finish_kernel(const float* __restrict__ partial, int nchunk, int C,
                                                             float* __restrict__ sums, GradOut gout_g, GradOut gout_b) {
  __shared__ float sm[2][NTF];
  const int nl = NTF / C;
  const int c = threadIdx.x % C, lane = threadIdx.x / C;
  const int per = (nchunk + nl - 1) / nl;
  const int k0 = lane * per, k1 = min(nchunk, k0 + per);
  float sb = 0.f, sg = 0.f;
  if (lane < nl) {
    int k = k0;
    for (; k + 7 < k1; k += 8) {
      float b8[8], g8[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        b8[u] = partial[((int64_t)(k + u) * 2 + 0) * C + c];
        g8[u] = partial[((int64_t)(k + u) * 2 + 1) * C + c];
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) { sb += b8[u]; sg += g8[u]; }
    }
    for (; k < k1; ++k) {
      sb += partial[((int64_t)k * 2 + 0) * C + c];
      sg += partial[((int64_t)k * 2 + 1) * C + c];
    }
  }
  sm[0][threadIdx.x] = sb; sm[1][threadIdx.x] = sg;
  __syncthreads();
  if (lane != 0) return;
  for (int l = 1; l < nl; ++l) { sb += sm[0][l * C + c]; sg += sm[1][l * C + c]; }
  sums[c] = sb;
  sums[C + c] = sg;
  grad_store(gout_b, c, sb);
  grad_store(gout_g, c, sg);
}

// Step 3: dy = gamma * rstd * (dpre - sum_b/R - xhat * sum_g/R), stored bf16 (operand of the
// backward products); with keep_dpre the masked gradient dpre replaces da (it also flows through
// the skip connection).
__global__ __launch_bounds__(NT) void bn2d_bwd_apply_kernel(float* __restrict__ da, const bf16_t* __restrict__ a,
                                                            const float* __restrict__ y, int64_t n4, int C, float inv_rows,
                                                            const float* __restrict__ gamma, int round_params,
                                                            const float* __restrict__ mean, const float* __restrict__ rstd,
                                                            const float* __restrict__ sums, int keep_dpre,
                                                            bf16_t* __restrict__ dy) {
  const int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x;
  if (i >= n4) return;
  const int c = (int)((i * 4) % C);
  const float4 d = reinterpret_cast<const float4*>(da)[i];
  const float4 v = reinterpret_cast<const float4*>(y)[i];
  const float4 o = unpack4(reinterpret_cast<const uint2*>(a)[i]);
  float4 g = *reinterpret_cast<const float4*>(&gamma[c]);
  const float4 m = *reinterpret_cast<const float4*>(&mean[c]);
  const float4 r = *reinterpret_cast<const float4*>(&rstd[c]);
  const float4 sb = *reinterpret_cast<const float4*>(&sums[c]);
  const float4 sg = *reinterpret_cast<const float4*>(&sums[C + c]);
  if (round_params) { g.x = round_bf16(g.x); g.y = round_bf16(g.y); g.z = round_bf16(g.z); g.w = round_bf16(g.w); }
  float4 dp;
  dp.x = o.x > 0.f ? d.x : 0.f; dp.y = o.y > 0.f ? d.y : 0.f;
  dp.z = o.z > 0.f ? d.z : 0.f; dp.w = o.w > 0.f ? d.w : 0.f;
  float4 out;
  out.x = g.x * r.x * (dp.x - sb.x * inv_rows - (v.x - m.x) * r.x * sg.x * inv_rows);
  out.y = g.y * r.y * (dp.y - sb.y * inv_rows - (v.y - m.y) * r.y * sg.y * inv_rows);
  out.z = g.z * r.z * (dp.z - sb.z * inv_rows - (v.z - m.z) * r.z * sg.z * inv_rows);
  out.w = g.w * r.w * (dp.w - sb.w * inv_rows - (v.w - m.w) * r.w * sg.w * inv_rows);
  reinterpret_cast<uint2*>(dy)[i] = pack4(out);
  if (keep_dpre) reinterpret_cast<float4*>(da)[i] = dp;
}

// ---- mean over the positions of an image -------------------------------------------------------
// pooled[n, c] = (1/HW) sum_p a[n, p, c], stored bf16 (operand of the classifier's product).
// One workgroup per image: threads = C/4 column groups x row lanes, lanes combined in order.
__global__ __launch_bounds__(NT) void avgpool_fwd_kernel(const bf16_t* __restrict__ a, int HW, int C,
                                                         bf16_t* __restrict__ pooled, int64_t ldp) {
  extern __shared__ float4 red[];
  Tall t = tall_shape(C);
  const int g = threadIdx.x % t.cg, lane = threadIdx.x / t.cg;
  const bool active = lane < t.rl;
  const int64_t base = (int64_t)blockIdx.x * HW * C;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (active)
    for (int p = lane; p < HW; p += t.rl) {
      const float4 v = unpack4(*reinterpret_cast<const uint2*>(&a[base + (int64_t)p * C + 4 * g]));
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
  const float4 tot = lanes_sum(s, red, g, lane, t);
  if (lane == 0) {
    const float inv = 1.f / (float)HW;
    *reinterpret_cast<uint2*>(&pooled[(int64_t)blockIdx.x * ldp + 4 * g]) =
        pack4(make_float4(tot.x * inv, tot.y * inv, tot.z * inv, tot.w * inv));
  }
}

// da[n, p, c] = dpooled[n, c] / HW.
__global__ __launch_bounds__(NT) void avgpool_bwd_kernel(const float* __restrict__ dpooled, int64_t ldd, int HW, int C,
                                                         int64_t n4, float* __restrict__ da) {
  const int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x;
  if (i >= n4) return;
  const int64_t e = i * 4;
  const int c = (int)(e % C);
  const int64_t img = e / ((int64_t)HW * C);
  const float inv = 1.f / (float)HW;
  const float4 d = *reinterpret_cast<const float4*>(&dpooled[img * ldd + c]);
  reinterpret_cast<float4*>(da)[i] = make_float4(d.x * inv, d.y * inv, d.z * inv, d.w * inv);
}

// ---- contraction slabs folded into a gradient ----------------------------------------------------
// out[p] (+)= alpha * (slab_0[p] + slab_1[p] + ...), slabs in order.
__global__ __launch_bounds__(NT) void fold_slabs_kernel(const float* __restrict__ slabs, int nsplit, int64_t stride,
                                                        int64_t n, GradOut out) {
  const int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x;
  if (i >= n) return;
  float v = slabs[i];
  for (int s = 1; s < nsplit; ++s) v += slabs[(int64_t)s * stride + i];
  grad_store(out, i, v);
}

// The same for many slabs: eight lanes per group of four elements, lane g adding slabs
// g * per .. (g + 1) * per - 1 in order (eight 16-byte loads in flight), the eight sums then added in
// lane order.  Requires n % 4 == 0, stride % 4 == 0, 16-byte aligned slabs.
__global__ __launch_bounds__(NT) void fold_slabs_wide_kernel(const float* __restrict__ slabs, int nsplit, int64_t stride,
                                                             int64_t n4, GradOut out) {
  __shared__ float4 part[8][32];
  const int q = threadIdx.x & 31, g = threadIdx.x >> 5;
  const int64_t i4 = (int64_t)blockIdx.x * 32 + q;
  const int per = (nsplit + 7) / 8;
  const int sbeg = g * per, send = min(nsplit, sbeg + per);
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (i4 < n4) {
    const float4* base = reinterpret_cast<const float4*>(slabs) + i4;
    const int64_t st4 = stride / 4;
    int sl = sbeg;
    for (; sl + 8 <= send; sl += 8) {
      float4 t[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) t[u] = base[(int64_t)(sl + u) * st4];
#pragma unroll
      for (int u = 0; u < 8; ++u) { v.x += t[u].x; v.y += t[u].y; v.z += t[u].z; v.w += t[u].w; }
    }
    for (; sl < send; ++sl) {
      const float4 t = base[(int64_t)sl * st4];
      v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
    }
  }
  part[g][q] = v;
  __syncthreads();
  if (g == 0 && i4 < n4) {
    float4 a = part[0][q];
#pragma unroll
    for (int k = 1; k < 8; ++k) { const float4 b = part[k][q]; a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w; }
    grad_store(out, 4 * i4, a.x); grad_store(out, 4 * i4 + 1, a.y);
    grad_store(out, 4 * i4 + 2, a.z); grad_store(out, 4 * i4 + 3, a.w);
  }
}

inline int64_t blocks(int64_t n) { return (n + NT - 1) / NT; }
inline bool tall_ok(int C) { return C >= 8 && C <= 256 && (C & 3) == 0; }
inline size_t tall_lds(int C) {
  const int cg = C >> 2;
  const int rl = NT / cg < 1 ? 1 : NT / cg;
  return (size_t)cg * rl * sizeof(float4);
}


// ---- weight gradient of a 3x3 convolution straight from the stored tensors -------------------
//   dW[o, tap, c] = sum over positions r of dy[r, o] * x[r + (kh-1) W + (kw-1), c]   (tap = 3 kh + kw;
//   terms whose source lies outside r's image are 0)
// for one 64 x 64 block of (o, c), all nine taps, and a slice of the positions.  The contraction
// runs over positions, which both tensors store as ROWS (channels are contiguous), so neither is
// in the orientation the matrix cores read (eight consecutive contraction elements per lane).
// Instead of transposing both through memory and writing a transposed patch matrix, a stage of
// 64 positions (64 / W image rows, W a power of two from 8 to 64) is staged in LDS as it is: the
// 64 rows of dy, and the image rows of x from one above to one below the stage, each image row
// with one empty position before and after it.  Image rows outside the image are fetched from a
// block of zeros and the empty positions are cleared once, so every shifted read finds either
// its value or 0 at a fixed offset: no masks.  The operands come out of LDS through the
// transposing read (wg_read8: two reads give a lane its eight consecutive contraction elements
// -- positions -- of one channel); the dy operand of a contraction step serves all nine taps.
// Workgroup (block, slice z) writes slab z of [Cout, 9 Cin]; the slabs are added in order
// afterwards.  Requires Cout % 64 == 0, Cin % 64 == 0, H % (64 / W) == 0 (a stage lies within
// one image), rows % 64 == 0.
typedef __bf16 wg_bf16x8 __attribute__((ext_vector_type(8)));
typedef float wg_f32x16 __attribute__((ext_vector_type(16)));

// Transposing LDS read (ds_read_b64_tr_b16): within each group of 16 lanes, lane 4a + b receives
// element b of the four 64-bit words that lanes a, a + 4, a + 8, a + 12 point at.  With source lane
// s pointing at position s / 4 (of four consecutive positions), channels 4 (s % 4) .. + 3, lane i
// of the group receives channel i at those four positions: four consecutive contraction
// elements of one operand row, which is what the matrix cores read.
typedef short wg_s16x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ wg_bf16x8 wg_read8(const bf16_t* first4, const bf16_t* next4) {
  const wg_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((wg_s16x4 __attribute__((address_space(3)))*)first4);
  const wg_s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((wg_s16x4 __attribute__((address_space(3)))*)next4);
  wg_bf16x8 r;
  __builtin_memcpy(&r, &lo, 8);
  __builtin_memcpy(reinterpret_cast<char*>(&r) + 8, &hi, 8);
  return r;
}

// One stage of 64 positions for taps T0 .. T0+NTAP-1.  A: this lane's source address in the dy rows
// for contraction step 0, first half; B[kk][r]: its source address in the stored x positions for
// step kk, half r, tap (0, 0).
template <int W, int T0, int NTAP>
__device__ __forceinline__ void wgrad_stage(const bf16_t* A, const bf16_t* const (&B)[4][2], wg_f32x16 (&acc)[5]) {
  constexpr int PW = W + 2;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    const wg_bf16x8 a = wg_read8(A + (16 * kk) * 64, A + (16 * kk + 4) * 64);
#pragma unroll
    for (int tt = 0; tt < NTAP; ++tt) {
      const int kh = (T0 + tt) / 3, kw = (T0 + tt) % 3;
      const int shift = (kh * PW + kw) * 64;
      const wg_bf16x8 b = wg_read8(B[kk][0] + shift, B[kk][1] + shift);
      acc[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[tt], 0, 0, 0);
    }
  }
}

constexpr int WG_NT = 512;       // eight waves: 2 x 2 over the 64 x 64 block, times two groups of taps
template <int W>
__global__ __launch_bounds__(WG_NT) void conv_wgrad_kernel(const bf16_t* __restrict__ dy, int Cout,
                                                        const bf16_t* __restrict__ x, int Cin, int H,
                                                        const bf16_t* __restrict__ zeros, int nstages,
                                                        int stages_per_wg, float* __restrict__ slabs,
                                                        int64_t slab_stride) {
  static_assert(W == 8 || W == 16 || W == 32 || W == 64, "image width");
  constexpr int IR = 64 / W;                               // image rows per stage
  constexpr int PW = W + 2;                                // positions of a stored image row
  constexpr int XR = (IR + 2) * PW;                        // stored positions of x per stage
  constexpr int BUF = (64 + XR) * 64;                      // elements of one stage buffer
  constexpr int NI = 8 + (IR + 2) * (W / 8);               // load instructions per stage (8 rows of 128 bytes each)
  extern __shared__ __attribute__((aligned(1024))) bf16_t wg_lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave >> 1) & 1, wn = wave & 1, khalf = lane >> 5, lc = lane & 31;
  const int tgroup = wave >> 2;                            // taps 0..4 or 5..8
  const int ctiles = Cin / 64;
  const int o0 = (blockIdx.x / ctiles) * 64, c0 = (blockIdx.x % ctiles) * 64;
  const int sbeg = blockIdx.y * stages_per_wg, send = min(nstages, sbeg + stages_per_wg);

  // the empty positions before and after every stored image row, both buffers (32 dwords each)
  for (int k = tid; k < 2 * (IR + 2) * 2 * 32; k += WG_NT) {
    const int dword = k & 31, which = k >> 5;              // which = ((buf * (IR + 2)) + image row) * 2 + side
    const int side = which & 1, irow = (which >> 1) % (IR + 2), buf = (which >> 1) / (IR + 2);
    const int pos = irow * PW + (side ? PW - 1 : 0);
    reinterpret_cast<uint32_t*>(wg_lds + buf * BUF + (64 + pos) * 64)[dword] = 0u;
  }

  auto issue = [&](int stage, int buf) {
    for (int idx = wave; idx < NI; idx += 8) {
      const bf16_t* src;
      int dst;                                             // element offset in the buffer of this instruction's first row
      if (idx < 8) {
        src = dy + ((int64_t)stage * 64 + idx * 8 + (lane >> 3)) * Cout + o0 + (lane & 7) * 8;
        dst = idx * 512;
      } else {
        const int k = idx - 8, ir = k / (W / 8) - 1, sub = k % (W / 8);
        const int g = stage * IR + ir;                     // image row among all images' rows; the stage starts at row h0
        const int hh = (stage * IR) % H + ir;
        src = (hh >= 0 && hh < H) ? x + ((int64_t)g * W + sub * 8 + (lane >> 3)) * Cin + c0 + (lane & 7) * 8
                                  : zeros + (lane & 7) * 8;
        dst = (64 + (ir + 1) * PW + 1 + sub * 8) * 64;
      }
      __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)src,
                                       (void __attribute__((address_space(3)))*)&wg_lds[buf * BUF + dst],
                                       16, 0, 0);
    }
  };

  wg_f32x16 acc[5];
#pragma unroll
  for (int t = 0; t < 5; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

  // this lane as a SOURCE of the transposing reads (see wg_read8): position j of four, channels 4 a .. 4 a + 3
  // of the 16-channel half its group of 16 lanes serves; element offsets inside a stage buffer
  // (one position = 64 elements).  Stage position e is stored at (e / W + kh) * PW + e % W + kw under tap (kh, kw).
  const int srcj = (lane & 15) >> 2, srca = lane & 3, half16 = (lane >> 4) & 1;
  const int a_off = (8 * khalf + srcj) * 64 + wm * 32 + 16 * half16 + 4 * srca;
  int b_off[4][2];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int e = 16 * kk + 8 * khalf + 4 * r + srcj;
      b_off[kk][r] = (64 + (e / W) * PW + e % W) * 64 + wn * 32 + 16 * half16 + 4 * srca;
    }

  if (sbeg < send) issue(sbeg, 0);
  for (int st = sbeg; st < send; ++st) {
    const int buf = (st - sbeg) & 1;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                                       // stage st is in LDS; everybody is done with the other buffer
    if (st + 1 < send) issue(st + 1, buf ^ 1);
    const bf16_t* A = wg_lds + buf * BUF + a_off;
    const bf16_t* B[4][2];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) { B[kk][0] = wg_lds + buf * BUF + b_off[kk][0]; B[kk][1] = wg_lds + buf * BUF + b_off[kk][1]; }
    if (tgroup == 0) wgrad_stage<W, 0, 5>(A, B, acc);
    else             wgrad_stage<W, 5, 4>(A, B, acc);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  // accumulator register q of a lane: row 8 (q/4) + 4 (lane/32) + q%4 (an output channel o), column lane%32 (c)
  float* out = slabs + (int64_t)blockIdx.y * slab_stride;
  const int64_t Kc = 9 * (int64_t)Cin;
#pragma unroll
  for (int tt = 0; tt < 5; ++tt) {
    const int t = tgroup * 5 + tt;
    if (t < 9) {
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int o = o0 + wm * 32 + 8 * (q >> 2) + 4 * khalf + (q & 3);
        out[(int64_t)o * Kc + (int64_t)t * Cin + c0 + wn * 32 + lc] = acc[tt][q];
      }
    }
  }
}

}  // namespace

int conv_chunks(int64_t rows) { return (int)((rows + CHUNK - 1) / CHUNK); }

int launch_im2col3x3(const bf16_t* x, int64_t rows, int H, int W, int C, bf16_t* cols, int64_t Kp, hipStream_t s) {
  if (rows <= 0 || H <= 0 || W <= 0 || C <= 0 || Kp < 9 * C || (Kp & 7) || rows % ((int64_t)H * W)) return VF_EINVAL;
  if ((C & 7) == 0 && Kp == 9 * C && (reinterpret_cast<uintptr_t>(x) & 15) == 0 && (reinterpret_cast<uintptr_t>(cols) & 15) == 0) {
    im2col8_kernel<<<(unsigned)blocks(rows * 9 * (C >> 3)), NT, 0, s>>>(x, rows, H, W, C, cols, Kp);
  } else {
    im2col1_kernel<<<(unsigned)blocks(rows * Kp), NT, 0, s>>>(x, rows, H, W, C, cols, (int)Kp);
  }
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_im2col3x3_transposed(const bf16_t* xT, int64_t ldx, int64_t rows, int H, int W, int C, bf16_t* colsT,
                                int64_t ldo, hipStream_t s) {
  if (rows <= 0 || H <= 0 || W <= 0 || C <= 0 || rows % ((int64_t)H * W) || ldx < rows || (ldo & 7) ||
      ldo < ((rows + 7) & ~int64_t(7)) || (reinterpret_cast<uintptr_t>(colsT) & 15))
    return VF_EINVAL;
  im2colT_kernel<<<(unsigned)blocks((int64_t)9 * C * ((rows + 7) >> 3)), NT, 0, s>>>(xT, ldx, rows, H, W, C, colsT, ldo);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_conv_weight_copies(const float* Wf, int Cout, int Cin, bf16_t* nat, int Kp, bf16_t* flip, int Kpf,
                              hipStream_t s) {
  if (Cout <= 0 || Cin <= 0 || Kp < 9 * Cin || (flip && Kpf < 9 * Cout)) return VF_EINVAL;
  conv_weight_copies_kernel<<<(unsigned)blocks((int64_t)Cout * 9 * Cin), NT, 0, s>>>(Wf, Cout, Cin, nat, Kp, flip, Kpf);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_bn2d_stats(const float* y, int64_t rows, int C, float eps, float* partial, float* mean, float* rstd,
                      float* run_mean, float* run_var, float run_mix, hipStream_t s) {
  if (rows <= 0 || !tall_ok(C) || !partial) return VF_EINVAL;
  if ((run_mean == nullptr) != (run_var == nullptr)) return VF_EINVAL;
  const int nchunk = conv_chunks(rows);
  bn2d_stats_partial_kernel<<<nchunk, NT, tall_lds(C), s>>>(y, rows, C, partial);
  VF_LAUNCH_CHECK();
  bn2d_stats_finish_kernel<<<1, NTF, 0, s>>>(partial, nchunk, CHUNK, rows, C, eps, mean, rstd, run_mean, run_var, run_mix);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_bn2d_stats_finish(const float* partial, int nchunk, int rows_per_chunk, int64_t rows, int C, float eps,
                             float* mean, float* rstd, float* run_mean, float* run_var, float run_mix, hipStream_t s) {
  if (rows <= 0 || !tall_ok(C) || !partial || nchunk < 1 || rows_per_chunk < 1) return VF_EINVAL;
  if ((int64_t)nchunk * rows_per_chunk < rows || (int64_t)(nchunk - 1) * rows_per_chunk >= rows) return VF_EINVAL;
  if ((run_mean == nullptr) != (run_var == nullptr)) return VF_EINVAL;
  bn2d_stats_finish_kernel<<<1, NTF, 0, s>>>(partial, nchunk, rows_per_chunk, rows, C, eps, mean, rstd, run_mean, run_var,
                                             run_mix);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_bn2d_apply_fwd(const float* y, int64_t rows, int C, const float* gamma, const float* beta, int round_params,
                          const float* mean, const float* rstd, const bf16_t* skip, bf16_t* a, hipStream_t s) {
  if (rows <= 0 || !tall_ok(C)) return VF_EINVAL;
  const int64_t n4 = rows * C / 4;
  bn2d_apply_fwd_kernel<<<(unsigned)blocks(n4), NT, 0, s>>>(y, n4, C, gamma, beta, round_params, mean, rstd, skip, a);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_bn2d_bwd(float* da, const bf16_t* a, const float* y, int64_t rows, int C, const float* gamma,
                    int round_params, const float* mean, const float* rstd, float* partial, float* sums,
                    int keep_dpre, bf16_t* dy, GradOut gout_g, GradOut gout_b, hipStream_t s) {
  if (rows <= 0 || !tall_ok(C) || !partial || !sums) return VF_EINVAL;
  const int nchunk = conv_chunks(rows);
  bn2d_bwd_partial_kernel<<<nchunk, NT, tall_lds(C), s>>>(da, a, y, rows, C, mean, rstd, partial);
  VF_LAUNCH_CHECK();
  bn2d_bwd_finish_kernel<<<1, NTF, 0, s>>>(partial, nchunk, C, sums, gout_g, gout_b);
  VF_LAUNCH_CHECK();
  const int64_t n4 = rows * C / 4;
  bn2d_bwd_apply_kernel<<<(unsigned)blocks(n4), NT, 0, s>>>(da, a, y, n4, C, 1.0f / (float)rows, gamma, round_params,
                                                            mean, rstd, sums, keep_dpre, dy);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_avgpool_fwd(const bf16_t* a, int n_img, int HW, int C, bf16_t* pooled, int64_t ldp, hipStream_t s) {
  if (n_img <= 0 || HW <= 0 || !tall_ok(C) || ldp < C || (ldp & 3)) return VF_EINVAL;
  avgpool_fwd_kernel<<<n_img, NT, tall_lds(C), s>>>(a, HW, C, pooled, ldp);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_avgpool_bwd(const float* dpooled, int64_t ldd, int n_img, int HW, int C, float* da, hipStream_t s) {
  if (n_img <= 0 || HW <= 0 || !tall_ok(C) || ldd < C || (ldd & 3)) return VF_EINVAL;
  const int64_t n4 = (int64_t)n_img * HW * C / 4;
  avgpool_bwd_kernel<<<(unsigned)blocks(n4), NT, 0, s>>>(dpooled, ldd, HW, C, n4, da);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

// Weight gradient of a 3x3 convolution (stride 1, zero padding 1) from dy [rows, Cout] and the
// layer's input x [rows, Cin] (bf16, channels last): slabs [nsplit][Cout, 9 Cin] of partial sums
// over slices of the positions, to be added in order.  *nsplit_out = the number of slabs written.
bool conv_wgrad_direct_fits(int Cout, int Cin, int H, int W, int64_t rows) {
  if (Cout % 64 || Cin % 64 || rows % 64) return false;
  if (W != 8 && W != 16 && W != 32 && W != 64) return false;
  return H >= 64 / W && H % (64 / W) == 0;
}

template <int W>
int launch_conv_wgrad_w(const bf16_t* dy, int Cout, const bf16_t* x, int Cin, int H, const bf16_t* zeros, int nstages,
                        int spw, int nsplit, float* slabs, int64_t slab_stride, hipStream_t s) {
  constexpr int bytes = 2 * (64 + (64 / W + 2) * (W + 2)) * 128;
  static bool ready = false;
  if (!ready) {
    VF_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_wgrad_kernel<W>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    ready = true;
  }
  dim3 grid((Cout / 64) * (Cin / 64), nsplit);
  conv_wgrad_kernel<W><<<grid, WG_NT, bytes, s>>>(dy, Cout, x, Cin, H, zeros, nstages, spw, slabs, slab_stride);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_conv_wgrad_direct(const bf16_t* dy, int Cout, const bf16_t* x, int Cin, int64_t rows, int H, int W,
                             const bf16_t* zeros, float* slabs, int64_t slab_stride, int max_split, int* nsplit_out,
                             hipStream_t s) {
  if (!dy || !x || !zeros || !slabs || !nsplit_out || rows <= 0 || rows > 0x7fffffff || max_split < 1) return VF_EINVAL;
  if (!conv_wgrad_direct_fits(Cout, Cin, H, W, rows) || rows % ((int64_t)H * W) ||
      slab_stride < (int64_t)Cout * 9 * Cin)
    return VF_EINVAL;
  if ((reinterpret_cast<uintptr_t>(dy) & 15) || (reinterpret_cast<uintptr_t>(x) & 15) ||
      (reinterpret_cast<uintptr_t>(zeros) & 15))
    return VF_EINVAL;
  const int nstages = (int)(rows / 64);
  const int tiles = (Cout / 64) * (Cin / 64);
  // about 256 workgroups, at least 4 stages each
  const int want = std::max(1, std::min(max_split, std::min((nstages + 3) / 4, (256 + tiles - 1) / tiles)));
  const int spw = (nstages + want - 1) / want;
  const int nsplit = (nstages + spw - 1) / spw;
  int rc;
  switch (W) {
    case 8: rc = launch_conv_wgrad_w<8>(dy, Cout, x, Cin, H, zeros, nstages, spw, nsplit, slabs, slab_stride, s); break;
    case 16: rc = launch_conv_wgrad_w<16>(dy, Cout, x, Cin, H, zeros, nstages, spw, nsplit, slabs, slab_stride, s); break;
    case 32: rc = launch_conv_wgrad_w<32>(dy, Cout, x, Cin, H, zeros, nstages, spw, nsplit, slabs, slab_stride, s); break;
    default: rc = launch_conv_wgrad_w<64>(dy, Cout, x, Cin, H, zeros, nstages, spw, nsplit, slabs, slab_stride, s); break;
  }
  if (rc == VF_OK) *nsplit_out = nsplit;
  return rc;
}

int launch_fold_slabs(const float* slabs, int nsplit, int64_t stride, int64_t n, GradOut out, hipStream_t s) {
  if (n <= 0 || nsplit < 1 || !slabs || !out.dst) return VF_EINVAL;
  if (nsplit >= 64 && (n & 3) == 0 && (stride & 3) == 0 && (reinterpret_cast<uintptr_t>(slabs) & 15) == 0)
    fold_slabs_wide_kernel<<<(unsigned)((n / 4 + 31) / 32), NT, 0, s>>>(slabs, nsplit, stride, n / 4, out);
  else
    fold_slabs_kernel<<<(unsigned)blocks(n), NT, 0, s>>>(slabs, nsplit, stride, n, out);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

}  // namespace vf
