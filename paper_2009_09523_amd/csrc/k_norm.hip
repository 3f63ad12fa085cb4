// Per-virtual-node BatchNorm (+ReLU) forward and backward, and column sums.
// The statistics are taken over exactly the R rows passed in -- the rows of the virtual node
// being processed (Section 4.1: such state is computed by each pass on its own; Section 3.2:
// each node is a separate forward and backward pass).  All reductions in fp32.
//
// Inputs that come from a GEMM arrive as NS partial slabs (see k_gemm_bf16.hip) and are summed
// here in slab order.  Outputs that feed a weight-gradient GEMM are also written transposed
// ([C, ldt], rows of the node contiguous), staged through LDS so that both copies are written
// with wide stores.
//
// Shape: a workgroup owns CB = 16 columns and all rows; 256 threads = 16 columns x 16 row
// lanes, so a 4096-wide layer gives 256 workgroups (one per compute unit).  For nodes of up
// to RPT*16 = 128 rows every thread keeps its rows in registers and global memory is read
// exactly once; larger nodes re-read the reduced values.
#include <algorithm>
#include <cstdlib>

#include "vf_device.h"

namespace vf {
namespace {

constexpr int CB = 16;    // columns per workgroup
constexpr int RL = 16;    // row lanes per column; 256 threads = CB x RL
constexpr int RPT = 8;    // rows per thread held in registers (nodes up to RL*RPT rows)
constexpr int RCH = RL * RPT;  // 128: rows per transposed-store chunk

// Sum over the RL row lanes of one column (threads with equal tx); result to all lanes.
__device__ __forceinline__ float col_reduce(float v, float (*red)[CB + 1], int tx, int ty) {
  red[ty][tx] = v;
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < RL; ++i) s += red[i][tx];
  __syncthreads();
  return s;
}

// Sum of the NS slabs at one element, in slab order; all loads are issued before the adds.
template <int NS>
__device__ __forceinline__ float sum_slabs(const float* __restrict__ p, int64_t stride, int64_t idx) {
  float v[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) v[s] = p[(int64_t)s * stride + idx];
  float t = v[0];
#pragma unroll
  for (int s = 1; s < NS; ++s) t += v[s];
  return t;
}

// Writes the bf16 tile held in LDS ([CB][RCH+8]: column c, rows r0..r0+RCH) to
// outT[c*ldt + r] with 16-byte stores; rows beyond R are padding inside the buffer's row.
__device__ __forceinline__ void store_transposed(const bf16_t (*tile)[RCH + 8], bf16_t* __restrict__ outT,
                                                 int64_t ldt, int c0, int C, int r0, int R) {
  const int col = threadIdx.x >> 4, seg = threadIdx.x & 15;    // 16 columns x 16 segments of 8 rows
  const int c = c0 + col;
  const int rl = seg * 8;
  if (c < C && r0 + rl < R)   // the vector holds at least one live row; ldt is a multiple of 8
    *reinterpret_cast<uint4*>(&outT[(int64_t)c * ldt + r0 + rl]) =
        *reinterpret_cast<const uint4*>(&tile[col][rl]);
}

// Which block of CB columns workgroup b takes.  A block of 16 columns is half a 128-byte line of
// an fp32 row and a quarter of a line of a bf16 row, and workgroups are dealt to the eight XCDs
// (each with an L2 of its own) in turn, so with the identity mapping the parts of one line are
// fetched into, and written back from, several L2s: the hardware counters showed twice the
// algorithmic bytes fetched.  Within every whole group of 32 blocks, the four workgroups that one
// XCD receives in a row (b, b+8, b+16, b+24) take four neighbouring blocks instead.
__device__ __forceinline__ int xcd_column_block(int b, int nblocks) {
  if (b >= (nblocks & ~31)) return b;
  const int q = b >> 3, x = b & 7;
  return (q >> 2) * 32 + x * 4 + (q & 3);
}

// SMALL: R <= RCH, rows live in registers.
// G > 1 (SMALL only): the rows are G virtual nodes of R rows each, one after the other (a group of
// equal-sized nodes whose products were taken as one): statistics, normalisation and the moving
// statistics' blend are per node, in node order, exactly as G launches would do them; the rows of
// node n+1 are requested before node n is worked on.  mean_out / rstd_out hold G
// vectors of C, the transposed copy node g's rows at columns g*R .. g*R + R-1.
template <typename T, int NS, bool SMALL, int G>
__global__ __launch_bounds__(256) void bn_relu_fwd_kernel(const float* zp, int64_t slab,
                                                          int64_t ldzp, int R, int C,
                                                          const float* __restrict__ gamma,
                                                          const float* __restrict__ beta,
                                                          int round_params, float eps,
                                                          float* z, int64_t ldz,
                                                          T* __restrict__ a, int64_t lda,
                                                          bf16_t* __restrict__ aT, int64_t ldt,
                                                          float* __restrict__ mean_out,
                                                          float* __restrict__ rstd_out,
                                                          float* __restrict__ run_mean,
                                                          float* __restrict__ run_var, float run_mix) {
  static_assert(G == 1 || SMALL, "groups of nodes only on the register-resident path");
  __shared__ float redg[1][RL][CB + 1];
  __shared__ __attribute__((aligned(16))) bf16_t tileg[1][CB][RCH + 8];
  float (*red)[CB + 1] = redg[0];
  bf16_t (*tile)[RCH + 8] = tileg[0];
  const int tx = threadIdx.x % CB, ty = threadIdx.x / CB;
  const int c0 = xcd_column_block(blockIdx.x, gridDim.x) * CB;
  const int c = c0 + tx;
  const bool live = c < C;
  const bool bn = gamma != nullptr;
  float g = 1.f, b = 0.f;
  float rm = 0.f, rv = 0.f;
  if (bn && live) {   // issued with the first row loads, needed only after the reductions
    g = gamma[c]; b = beta[c];
    if (run_mean && ty == 0) { rm = run_mean[c]; rv = run_var[c]; }
  }
  float zr[1][RPT];
  if (SMALL) {
    // Loads at clamped (always valid) addresses, selection afterwards: no load sits behind a
    // branch, so all of a thread's loads are in flight together.
    const int cc = min(c, C - 1);
#pragma unroll
    for (int k = 0; k < RPT; ++k) {             // (a group's further nodes are requested one node ahead, below)
      const int r = ty + RL * k;
      zr[0][k] = sum_slabs<NS>(zp, slab, (int64_t)min(r, R - 1) * ldzp + cc);
    }
  }
  if (bn && live && round_params) { g = round_bf16(g); b = round_bf16(b); }
  static_assert(G == 1, "groups of nodes have kernels of their own");
  constexpr int ONE = 1;
#pragma unroll
  for (int n = 0; n < ONE; ++n) {
    const int rb = n * R;                       // first row of this node
    float mean = 0.f, rstd = 1.f;
    // pass 1: reduce the slabs into z, column sums
    float s = 0.f;
    if (SMALL) {
#pragma unroll
      for (int k = 0; k < RPT; ++k) {
        const int r = ty + RL * k;
        zr[n][k] = (live && r < R) ? zr[n][k] : 0.f;
        s += zr[n][k];
      }
#pragma unroll
      for (int k = 0; k < RPT; ++k) {
        const int r = ty + RL * k;
        if ((NS > 1 || zp != z) && live && r < R) z[(int64_t)(rb + r) * ldz + c] = zr[n][k];
      }
    } else if (live) {
      for (int r = ty; r < R; r += RL) {
        float v = sum_slabs<NS>(zp, slab, (int64_t)r * ldzp + c);
        if (NS > 1 || zp != z) z[(int64_t)r * ldz + c] = v;
        s += v;
      }
    }
    if (bn) {
      mean = col_reduce(s, red, tx, ty) / (float)R;
      float q = 0.f;
      if (SMALL) {
#pragma unroll
        for (int k = 0; k < RPT; ++k) {
          const int r = ty + RL * k;
          float d = (live && r < R) ? zr[n][k] - mean : 0.f;
          q = fmaf(d, d, q);
        }
      } else if (live) {
        for (int r = ty; r < R; r += RL) {
          float d = z[(int64_t)r * ldz + c] - mean;
          q = fmaf(d, d, q);
        }
      }
      const float var = col_reduce(q, red, tx, ty) / (float)R;
      rstd = 1.0f / sqrtf(var + eps);
      if (live && ty == 0) {
        mean_out[(int64_t)n * C + c] = mean; rstd_out[(int64_t)n * C + c] = rstd;
        if (run_mean) {   // moving statistics of this device: one blend per pass (Section 4.1)
          rm = fmaf(run_mix, mean - rm, rm);
          rv = fmaf(run_mix, var - rv, rv);
        }
      }
    }
    // pass 2: activation, in chunks of RCH rows so the transposed copy can go through LDS
    for (int r0 = 0; r0 < R; r0 += RCH) {
#pragma unroll
      for (int k = 0; k < RPT; ++k) {
        const int rl = ty + RL * k;
        const int r = r0 + rl;
        float v = 0.f;
        if (live && r < R) {
          float zz = SMALL ? zr[n][k] : z[(int64_t)r * ldz + c];
          v = bn ? fmaxf(fmaf(g, (zz - mean) * rstd, b), 0.f) : fmaxf(zz, 0.f);
          store_f(&a[(int64_t)(rb + r) * lda + c], v);
        }
        if (aT) tile[tx][rl] = f32_to_bf16(v);
      }
      if (aT) {
        __syncthreads();
        store_transposed(tile, aT + rb, ldt, c0, C, r0, R);
        __syncthreads();
      }
    }
  }
  if (bn && live && ty == 0 && run_mean) { run_mean[c] = rm; run_var[c] = rv; }
}

template <typename T, int NS, bool SMALL, int G>
__global__ __launch_bounds__(256) void bn_relu_bwd_kernel(float* __restrict__ dap, int64_t slab,
                                                          int64_t ldda, const float* __restrict__ z,
                                                          int64_t ldz, int R, int C,
                                                          const float* __restrict__ gamma,
                                                          const float* __restrict__ beta,
                                                          int round_params,
                                                          const float* __restrict__ mean_in,
                                                          const float* __restrict__ rstd_in,
                                                          T* __restrict__ dz, int64_t lddz,
                                                          bf16_t* __restrict__ dzT, int64_t ldt,
                                                          GradOut gout_g, GradOut gout_b, float tscale) {
  static_assert(G == 1 || SMALL, "groups of nodes only on the register-resident path");
  __shared__ float redg[1][RL][CB + 1];
  __shared__ __attribute__((aligned(16))) bf16_t tileg[1][CB][RCH + 8];
  float (*red)[CB + 1] = redg[0];
  bf16_t (*tile)[RCH + 8] = tileg[0];
  const int tx = threadIdx.x % CB, ty = threadIdx.x / CB;
  const int c0 = xcd_column_block(blockIdx.x, gridDim.x) * CB;
  const int c = c0 + tx;
  const bool live = c < C;
  const bool bn = gamma != nullptr;
  float g = 1.f, b = 0.f, mean[G], rstd[G];
#pragma unroll
  for (int n = 0; n < G; ++n) { mean[n] = 0.f; rstd[n] = 1.f; }
  if (live && bn) {
    g = gamma[c]; b = beta[c];
    if (round_params) { g = round_bf16(g); b = round_bf16(b); }
#pragma unroll
    for (int n = 0; n < G; ++n) { mean[n] = mean_in[(int64_t)n * C + c]; rstd[n] = rstd_in[(int64_t)n * C + c]; }
  }
  float xr[1][RPT], dr[1][RPT];
  if (SMALL) {
    // loads at clamped (always valid) addresses first, all in flight together; selection after
    // (a group's further nodes are requested one node ahead, below)
    const int cc = min(c, C - 1);
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
      const int rc = min(ty + RL * k, R - 1);
      xr[0][k] = z[(int64_t)rc * ldz + cc];
      dr[0][k] = sum_slabs<NS>(dap, slab, (int64_t)rc * ldda + cc);
    }
  }
  // the nodes of a group have one weight: their small-vector gradients are added up in node order
  // and folded in once (what the staged path does with its staging vector, bit for bit)
  float tg = 0.f, tb = 0.f;
  static_assert(G == 1, "groups of nodes have kernels of their own");
  constexpr int ONE = 1;
#pragma unroll
  for (int n = 0; n < ONE; ++n) {
    const int rb = n * R;
    // pass 1: sum dout*xhat, sum dout  (dout = da where the ReLU was open)
    float sg = 0.f, sb = 0.f;
    if (SMALL) {
#pragma unroll
      for (int k = 0; k < RPT; ++k) {
        const int r = ty + RL * k;
        const float zz = xr[n][k];
        const float xhat = (zz - mean[n]) * rstd[n];
        const float pre = bn ? fmaf(g, xhat, b) : zz;
        const bool on = live && r < R;
        xr[n][k] = on ? xhat : 0.f;
        dr[n][k] = (on && pre > 0.f) ? dr[n][k] : 0.f;
        sg = fmaf(dr[n][k], xr[n][k], sg);
        sb += dr[n][k];
      }
    } else if (live) {
      for (int r = ty; r < R; r += RL) {
        float zz = z[(int64_t)r * ldz + c];
        float xhat = (zz - mean[n]) * rstd[n];
        float pre = bn ? fmaf(g, xhat, b) : zz;
        float d = sum_slabs<NS>(dap, slab, (int64_t)r * ldda + c);
        float dout = pre > 0.f ? d : 0.f;
        dap[(int64_t)r * ldda + c] = dout;   // keep the reduced, masked value in slab 0
        sg = fmaf(dout, xhat, sg);
        sb += dout;
      }
    }
    sg = col_reduce(sg, red, tx, ty);
    sb = col_reduce(sb, red, tx, ty);
    tg = n ? tg + sg : sg;
    tb = n ? tb + sb : sb;
    if (n == G - 1 && live && ty == 0) {
      if (bn) grad_store(gout_g, c, tg);
      if (gout_b.dst) grad_store(gout_b, c, tb);
    }
    const float invR = 1.0f / (float)R;
    const float kk = g * rstd[n];
    // pass 2: dz (and its transposed copy)
    for (int r0 = 0; r0 < R; r0 += RCH) {
#pragma unroll
      for (int k = 0; k < RPT; ++k) {
        const int rl = ty + RL * k;
        const int r = r0 + rl;
        float v = 0.f;
        if (live && r < R) {
          float xhat, dout;
          if (SMALL) {
            xhat = xr[n][k]; dout = dr[n][k];
          } else {
            xhat = (z[(int64_t)r * ldz + c] - mean[n]) * rstd[n];
            dout = dap[(int64_t)r * ldda + c];           // written by this thread in pass 1
          }
          v = bn ? kk * (dout - sb * invR - xhat * sg * invR) : dout;
          store_f(&dz[(int64_t)(rb + r) * lddz + c], v);
        }
        if (dzT) tile[tx][rl] = f32_to_bf16(v * tscale);
      }
      if (dzT) {
        __syncthreads();
        store_transposed(tile, dzT + rb, ldt, c0, C, r0, R);
        __syncthreads();
      }
    }
  }
}

// ---- groups of nodes ------------------------------------------------------------------------------
// The rows are G virtual nodes of R <= 128 rows each, one after the other (a group of equal-sized
// nodes whose products were taken as one).  Statistics, normalisation, the blend of the moving
// statistics and the small-vector gradients are per node, in node order, exactly as G launches of
// the kernels above would do them (same sums, same order).  A workgroup owns CB columns as
// above but has up to four sub-groups of 256 threads, each working on a node of its own at the
// same time (G = 8: two rounds); what couples the nodes -- the moving statistics, blended node
// after node, and the gamma / beta gradients, added up in node order and folded in once -- goes
// through LDS and is finished by one thread per column.  mean_out / rstd_out hold G vectors of C,
// the transposed copy node n's rows at columns n*R .. n*R + R-1.
// Row ranges of the nodes of a unit: node n has rows[n] <= 128 rows starting at row base[n] of the
// unit (a multiple of 8 when transposed copies are written); entries beyond the unit's nodes are 0.
constexpr int kBnGroup = 8;   // nodes per launch of the group kernels
constexpr int kBnGroupPair = 16;   // nodes per launch of the forward two-column kernel
struct GroupRows { int base[16]; int rows[16]; };

template <int G, int SG_> struct GroupShape {
  static constexpr int SG = SG_ < G ? SG_ : G;   // sub-groups side by side
  static constexpr int RND = G / SG;             // rounds
  static constexpr int THREADS = 256 * SG;
};

__device__ __forceinline__ void store_transposed_sub(const bf16_t (*tile)[RCH + 8], bf16_t* __restrict__ outT,
                                                     int64_t ldt, int c0, int C, int R, int t) {
  const int col = t >> 4, seg = t & 15;          // 16 columns x 16 segments of 8 rows
  const int c = c0 + col;
  const int rl = seg * 8;
  if (c < C && rl < R)
    *reinterpret_cast<uint4*>(&outT[(int64_t)c * ldt + rl]) = *reinterpret_cast<const uint4*>(&tile[col][rl]);
}

template <int NS, int G, int SGP>
__global__ __launch_bounds__((GroupShape<G, SGP>::THREADS)) void bn_relu_fwd_group_kernel(
    const float* zp, int64_t slab, int64_t ldzp, GroupRows gr, int count, int C, const float* __restrict__ gamma,
    const float* __restrict__ beta, int round_params, float eps, float* z, int64_t ldz,
    bf16_t* __restrict__ a, int64_t lda, bf16_t* __restrict__ aT, int64_t ldt, float* __restrict__ mean_out,
    float* __restrict__ rstd_out, float* __restrict__ run_mean, float* __restrict__ run_var, float run_mix) {
  constexpr int SG = GroupShape<G, SGP>::SG, RND = GroupShape<G, SGP>::RND;
  __shared__ float red[SG][RL][CB + 1];
  __shared__ __attribute__((aligned(16))) bf16_t tile[SG][CB][RCH + 8];
  __shared__ float stat[G][2][CB];
  const int sub = threadIdx.x >> 8, t = threadIdx.x & 255;
  const int tx = t % CB, ty = t / CB;
  const int c0 = xcd_column_block(blockIdx.x, gridDim.x) * CB;
  const int c = c0 + tx;
  const bool live = c < C;
  const bool bn = gamma != nullptr;
  const int cc = min(c, C - 1);
  float g = 1.f, b = 0.f;
  if (bn && live) { g = gamma[c]; b = beta[c]; }
  // all rows of this sub-group's nodes, at clamped (always valid) addresses
  float zr[RND][RPT];
#pragma unroll
  for (int q = 0; q < RND; ++q)
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
      const int r = ty + RL * k;
      const int n = q * SG + sub;
      zr[q][k] = sum_slabs<NS>(zp, slab, (int64_t)(gr.base[n] + max(min(r, gr.rows[n] - 1), 0)) * ldzp + cc);
    }
  if (bn && live && round_params) { g = round_bf16(g); b = round_bf16(b); }
#pragma unroll
  for (int q = 0; q < RND; ++q) {
    const int n = q * SG + sub;
    const int R = gr.rows[n], rb = gr.base[n];    // (R = 0 behind the unit's last node: nothing is stored)
    float mean = 0.f, rstd = 1.f;
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
      const int r = ty + RL * k;
      zr[q][k] = (live && r < R) ? zr[q][k] : 0.f;
      s += zr[q][k];
    }
    if (NS > 1 || zp != z) {
#pragma unroll
      for (int k = 0; k < RPT; ++k) {
        const int r = ty + RL * k;
        if (live && r < R) z[(int64_t)(rb + r) * ldz + c] = zr[q][k];
      }
    }
    if (bn) {
      mean = col_reduce(s, red[sub], tx, ty) / (float)R;
      float qq = 0.f;
#pragma unroll
      for (int k = 0; k < RPT; ++k) {
        const int r = ty + RL * k;
        float d = (live && r < R) ? zr[q][k] - mean : 0.f;
        qq = fmaf(d, d, qq);
      }
      const float var = col_reduce(qq, red[sub], tx, ty) / (float)R;
      rstd = 1.0f / sqrtf(var + eps);
      if (ty == 0) {
        stat[n][0][tx] = mean; stat[n][1][tx] = var;
        if (live && n < count) { mean_out[(int64_t)n * C + c] = mean; rstd_out[(int64_t)n * C + c] = rstd; }
      }
    } else if (q > 0 && aT) {
      __syncthreads();                            // the tile of the round before has been read
    }
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
      const int r = ty + RL * k;
      float v = 0.f;
      if (live && r < R) {
        v = bn ? fmaxf(fmaf(g, (zr[q][k] - mean) * rstd, b), 0.f) : fmaxf(zr[q][k], 0.f);
        a[(int64_t)(rb + r) * lda + c] = f32_to_bf16(v);
      }
      if (aT) tile[sub][tx][r] = f32_to_bf16(v);
    }
    if (aT) {
      __syncthreads();
      store_transposed_sub(tile[sub], aT + rb, ldt, c0, C, R, t);
    }
  }
  // moving statistics of this device: one blend per pass, node after node (Section 4.1)
  if (bn && run_mean) {
    __syncthreads();
    if (sub == 0 && ty == 0 && live) {
      float rm = run_mean[c], rv = run_var[c];
#pragma unroll
      for (int n = 0; n < G; ++n) {
        if (n < count) {
          rm = fmaf(run_mix, stat[n][0][tx] - rm, rm);
          rv = fmaf(run_mix, stat[n][1][tx] - rv, rv);
        }
      }
      run_mean[c] = rm; run_var[c] = rv;
    }
  }
}

template <int NS, int G, int SGP>
__global__ __launch_bounds__((GroupShape<G, SGP>::THREADS)) void bn_relu_bwd_group_kernel(
    float* __restrict__ dap, int64_t slab, int64_t ldda, const float* __restrict__ z, int64_t ldz, GroupRows gr,
    int count, int C,
    const float* __restrict__ gamma, const float* __restrict__ beta, int round_params,
    const float* __restrict__ mean_in, const float* __restrict__ rstd_in, bf16_t* __restrict__ dz, int64_t lddz,
    bf16_t* __restrict__ dzT, int64_t ldt, GradOut gout_g, GradOut gout_b, float tscale) {
  constexpr int SG = GroupShape<G, SGP>::SG, RND = GroupShape<G, SGP>::RND;
  __shared__ float red[SG][RL][CB + 1];
  __shared__ __attribute__((aligned(16))) bf16_t tile[SG][CB][RCH + 8];
  __shared__ float sums[G][2][CB];
  const int sub = threadIdx.x >> 8, t = threadIdx.x & 255;
  const int tx = t % CB, ty = t / CB;
  const int c0 = xcd_column_block(blockIdx.x, gridDim.x) * CB;
  const int c = c0 + tx;
  const bool live = c < C;
  const bool bn = gamma != nullptr;
  const int cc = min(c, C - 1);
  float g = 1.f, b = 0.f, mean[RND], rstd[RND];
#pragma unroll
  for (int q = 0; q < RND; ++q) { mean[q] = 0.f; rstd[q] = 1.f; }
  if (live && bn) {
    g = gamma[c]; b = beta[c];
    if (round_params) { g = round_bf16(g); b = round_bf16(b); }
#pragma unroll
    for (int q = 0; q < RND; ++q) {
      mean[q] = mean_in[(int64_t)(q * SG + sub) * C + c]; rstd[q] = rstd_in[(int64_t)(q * SG + sub) * C + c];
    }
  }
  float xr[RND][RPT], dr[RND][RPT];
#pragma unroll
  for (int q = 0; q < RND; ++q)
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
      const int rc = gr.base[q * SG + sub] + max(min(ty + RL * k, gr.rows[q * SG + sub] - 1), 0);
      xr[q][k] = z[(int64_t)rc * ldz + cc];
      dr[q][k] = sum_slabs<NS>(dap, slab, (int64_t)rc * ldda + cc);
    }
#pragma unroll
  for (int q = 0; q < RND; ++q) {
    const int n = q * SG + sub;
    const int R = gr.rows[n], rb = gr.base[n];    // (R = 0 behind the unit's last node: nothing is stored)
    const float invR = 1.0f / (float)R;
    float sg = 0.f, sb = 0.f;
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
      const int r = ty + RL * k;
      const float zz = xr[q][k];
      const float xhat = (zz - mean[q]) * rstd[q];
      const float pre = bn ? fmaf(g, xhat, b) : zz;
      const bool on = live && r < R;
      xr[q][k] = on ? xhat : 0.f;
      dr[q][k] = (on && pre > 0.f) ? dr[q][k] : 0.f;
      sg = fmaf(dr[q][k], xr[q][k], sg);
      sb += dr[q][k];
    }
    sg = col_reduce(sg, red[sub], tx, ty);
    sb = col_reduce(sb, red[sub], tx, ty);
    if (ty == 0) { sums[n][0][tx] = sg; sums[n][1][tx] = sb; }
    const float kk = g * rstd[q];
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
      const int r = ty + RL * k;
      float v = 0.f;
      if (live && r < R) {
        v = bn ? kk * (dr[q][k] - sb * invR - xr[q][k] * sg * invR) : dr[q][k];
        dz[(int64_t)(rb + r) * lddz + c] = f32_to_bf16(v);
      }
      if (dzT) tile[sub][tx][r] = f32_to_bf16(v * tscale);
    }
    if (dzT) {
      __syncthreads();                            // (the next round writes the tile behind its reductions' barriers)
      store_transposed_sub(tile[sub], dzT + rb, ldt, c0, C, R, t);
    }
  }
  // the nodes of a group have one weight: their small-vector gradients are added up in node order
  // and folded in once (what the staged path does with its staging vector, bit for bit)
  __syncthreads();
  if (sub == 0 && ty == 0 && live) {
    float tg = 0.f, tb = 0.f;
#pragma unroll
    for (int n = 0; n < G; ++n) {
      if (n < count) {
        tg = n ? tg + sums[n][0][tx] : sums[n][0][tx];
        tb = n ? tb + sums[n][1][tx] : sums[n][1][tx];
      }
    }
    if (bn) grad_store(gout_g, c, tg);
    if (gout_b.dst) grad_store(gout_b, c, tb);
  }
}


// ---- two columns per thread -----------------------------------------------------------------------
// The group kernels above with a workgroup on 2 CB = 32 columns, every thread on two neighbouring
// ones: a row of a workgroup's block is a whole 128-byte line of the fp32 tensors (8 bytes per lane)
// and half a line of the bf16 ones, and the four workgroups that an XCD receives in a row cover 512
// contiguous bytes of every row.  (A probe of the bare access pattern over 2048 x 8192: 16 columns
// per workgroup 5.0 TB/s, 32 columns 6.1, and 7.0 with sixteen nodes per launch; 64 columns leave
// too few workgroups.)  For wide layers whose input is unsliced and lies where it is kept.  Per
// column the arithmetic is that of the kernels above, operation for operation.
constexpr int CB2 = 2 * CB;

__device__ __forceinline__ float2 col_reduce2(float2 v, float (*red)[RL][CB + 1], int tx, int ty) {
  red[0][ty][tx] = v.x;
  red[1][ty][tx] = v.y;
  __syncthreads();
  float2 s = {0.f, 0.f};
#pragma unroll
  for (int i = 0; i < RL; ++i) { s.x += red[0][i][tx]; s.y += red[1][i][tx]; }
  __syncthreads();
  return s;
}

__device__ __forceinline__ void store_transposed_pair(const bf16_t (*tile)[RCH + 8], bf16_t* __restrict__ outT,
                                                      int64_t ldt, int c0, int C, int R, int t) {
  const int seg = t & 15, rl = seg * 8;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int col = (t >> 4) + 16 * h;          // 2 x 16 columns x 16 segments of 8 rows
    const int c = c0 + col;
    if (c < C && rl < R)
      store16_stream(&outT[(int64_t)c * ldt + rl], *reinterpret_cast<const uint4*>(&tile[col][rl]));
  }
}

template <int G, int SGP>
__global__ __launch_bounds__((GroupShape<G, SGP>::THREADS)) void bn_relu_fwd_pair_kernel(
    const float* __restrict__ z, int64_t ldz, GroupRows gr, int count, int C, const float* __restrict__ gamma,
    const float* __restrict__ beta, int round_params, float eps, bf16_t* __restrict__ a, int64_t lda,
    bf16_t* __restrict__ aT, int64_t ldt, float* __restrict__ mean_out, float* __restrict__ rstd_out,
    float* __restrict__ run_mean, float* __restrict__ run_var, float run_mix) {
  constexpr int SG = GroupShape<G, SGP>::SG, RND = GroupShape<G, SGP>::RND;
  __shared__ float red[SG][2][RL][CB + 1];
  __shared__ __attribute__((aligned(16))) bf16_t tile[SG][CB2][RCH + 8];
  __shared__ float stat[G][2][CB2];
  const int sub = threadIdx.x >> 8, t = threadIdx.x & 255;
  const int tx = t % CB, ty = t / CB;
  const int c0 = xcd_column_block(blockIdx.x, gridDim.x) * CB2;
  const int c = c0 + 2 * tx;                      // C is even: c and c + 1 are live together
  const bool live = c < C;
  const bool bn = gamma != nullptr;
  const int cc = min(c, C - 2);
  float2 g = {1.f, 1.f}, b = {0.f, 0.f};
  if (bn && live) { g = *reinterpret_cast<const float2*>(&gamma[c]); b = *reinterpret_cast<const float2*>(&beta[c]); }
  float2 zr[RND][RPT];
#pragma unroll
  for (int q = 0; q < RND; ++q)
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
      const int r = ty + RL * k;
      const int n = q * SG + sub;
      zr[q][k] = load2_stream(&z[(int64_t)(gr.base[n] + max(min(r, gr.rows[n] - 1), 0)) * ldz + cc]);
    }
  if (bn && live && round_params) { g.x = round_bf16(g.x); g.y = round_bf16(g.y); b.x = round_bf16(b.x); b.y = round_bf16(b.y); }
#pragma unroll
  for (int q = 0; q < RND; ++q) {
    const int n = q * SG + sub;
    const int R = gr.rows[n], rb = gr.base[n];    // (R = 0 behind the unit's last node: nothing is stored)
    float2 mean = {0.f, 0.f}, rstd = {1.f, 1.f};
    float2 s = {0.f, 0.f};
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
      const int r = ty + RL * k;
      if (!(live && r < R)) zr[q][k] = float2{0.f, 0.f};
      s.x += zr[q][k].x; s.y += zr[q][k].y;
    }
    if (bn) {
      const float2 sm = col_reduce2(s, red[sub], tx, ty);
      mean.x = sm.x / (float)R; mean.y = sm.y / (float)R;
      float2 qq = {0.f, 0.f};
#pragma unroll
      for (int k = 0; k < RPT; ++k) {
        const int r = ty + RL * k;
        const bool on = live && r < R;
        const float dx = on ? zr[q][k].x - mean.x : 0.f, dy = on ? zr[q][k].y - mean.y : 0.f;
        qq.x = fmaf(dx, dx, qq.x); qq.y = fmaf(dy, dy, qq.y);
      }
      const float2 sq = col_reduce2(qq, red[sub], tx, ty);
      const float2 var = {sq.x / (float)R, sq.y / (float)R};
      rstd.x = 1.0f / sqrtf(var.x + eps); rstd.y = 1.0f / sqrtf(var.y + eps);
      if (ty == 0) {
        stat[n][0][2 * tx] = mean.x; stat[n][0][2 * tx + 1] = mean.y;
        stat[n][1][2 * tx] = var.x;  stat[n][1][2 * tx + 1] = var.y;
        if (live && n < count) {
          *reinterpret_cast<float2*>(&mean_out[(int64_t)n * C + c]) = mean;
          *reinterpret_cast<float2*>(&rstd_out[(int64_t)n * C + c]) = rstd;
        }
      }
    } else if (q > 0 && aT) {
      __syncthreads();                            // the tile of the round before has been read
    }
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
      const int r = ty + RL * k;
      float vx = 0.f, vy = 0.f;
      if (live && r < R) {
        vx = bn ? fmaxf(fmaf(g.x, (zr[q][k].x - mean.x) * rstd.x, b.x), 0.f) : fmaxf(zr[q][k].x, 0.f);
        vy = bn ? fmaxf(fmaf(g.y, (zr[q][k].y - mean.y) * rstd.y, b.y), 0.f) : fmaxf(zr[q][k].y, 0.f);
        *reinterpret_cast<uint32_t*>(&a[(int64_t)(rb + r) * lda + c]) = (uint32_t)f32_to_bf16(vx) | ((uint32_t)f32_to_bf16(vy) << 16);
      }
      if (aT) { tile[sub][2 * tx][r] = f32_to_bf16(vx); tile[sub][2 * tx + 1][r] = f32_to_bf16(vy); }
    }
    if (aT) {
      __syncthreads();
      store_transposed_pair(tile[sub], aT + rb, ldt, c0, C, R, t);
    }
  }
  // moving statistics of this device: one blend per pass, node after node (Section 4.1)
  if (bn && run_mean) {
    __syncthreads();
    if (sub == 0 && ty == 0 && live) {
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        float rm = run_mean[c + e], rv = run_var[c + e];
#pragma unroll
        for (int n = 0; n < G; ++n) {
          if (n < count) {
            rm = fmaf(run_mix, stat[n][0][2 * tx + e] - rm, rm);
            rv = fmaf(run_mix, stat[n][1][2 * tx + e] - rv, rv);
          }
        }
        run_mean[c + e] = rm; run_var[c + e] = rv;
      }
    }
  }
}

template <int G, int SGP>
__global__ __launch_bounds__((GroupShape<G, SGP>::THREADS)) void bn_relu_bwd_pair_kernel(
    const float* __restrict__ da, int64_t ldda, const float* __restrict__ z, int64_t ldz, GroupRows gr, int count, int C,
    const float* __restrict__ gamma, const float* __restrict__ beta, int round_params,
    const float* __restrict__ mean_in, const float* __restrict__ rstd_in, bf16_t* __restrict__ dz, int64_t lddz,
    bf16_t* __restrict__ dzT, int64_t ldt, GradOut gout_g, GradOut gout_b, float tscale) {
  constexpr int SG = GroupShape<G, SGP>::SG, RND = GroupShape<G, SGP>::RND;
  __shared__ float red[SG][2][RL][CB + 1];
  __shared__ __attribute__((aligned(16))) bf16_t tile[SG][CB2][RCH + 8];
  __shared__ float sums[G][2][CB2];
  const int sub = threadIdx.x >> 8, t = threadIdx.x & 255;
  const int tx = t % CB, ty = t / CB;
  const int c0 = xcd_column_block(blockIdx.x, gridDim.x) * CB2;
  const int c = c0 + 2 * tx;
  const bool live = c < C;
  const bool bn = gamma != nullptr;
  const int cc = min(c, C - 2);
  float2 g = {1.f, 1.f}, b = {0.f, 0.f}, mean[RND], rstd[RND];
#pragma unroll
  for (int q = 0; q < RND; ++q) { mean[q] = float2{0.f, 0.f}; rstd[q] = float2{1.f, 1.f}; }
  if (live && bn) {
    g = *reinterpret_cast<const float2*>(&gamma[c]); b = *reinterpret_cast<const float2*>(&beta[c]);
    if (round_params) { g.x = round_bf16(g.x); g.y = round_bf16(g.y); b.x = round_bf16(b.x); b.y = round_bf16(b.y); }
#pragma unroll
    for (int q = 0; q < RND; ++q) {
      const int nn = min(q * SG + sub, count - 1);
      mean[q] = *reinterpret_cast<const float2*>(&mean_in[(int64_t)nn * C + c]);
      rstd[q] = *reinterpret_cast<const float2*>(&rstd_in[(int64_t)nn * C + c]);
    }
  }
  float2 xr[RND][RPT], dr[RND][RPT];
#pragma unroll
  for (int q = 0; q < RND; ++q)
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
      const int rc = gr.base[q * SG + sub] + max(min(ty + RL * k, gr.rows[q * SG + sub] - 1), 0);
      xr[q][k] = load2_stream(&z[(int64_t)rc * ldz + cc]);
      dr[q][k] = load2_stream(&da[(int64_t)rc * ldda + cc]);
    }
#pragma unroll
  for (int q = 0; q < RND; ++q) {
    const int n = q * SG + sub;
    const int R = gr.rows[n], rb = gr.base[n];    // (R = 0 behind the unit's last node: nothing is stored)
    const float invR = 1.0f / (float)R;
    float2 sg = {0.f, 0.f}, sb = {0.f, 0.f};
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
      const int r = ty + RL * k;
      const bool on = live && r < R;
      {
        const float zz = xr[q][k].x;
        const float xhat = (zz - mean[q].x) * rstd[q].x;
        const float pre = bn ? fmaf(g.x, xhat, b.x) : zz;
        xr[q][k].x = on ? xhat : 0.f;
        dr[q][k].x = (on && pre > 0.f) ? dr[q][k].x : 0.f;
        sg.x = fmaf(dr[q][k].x, xr[q][k].x, sg.x);
        sb.x += dr[q][k].x;
      }
      {
        const float zz = xr[q][k].y;
        const float xhat = (zz - mean[q].y) * rstd[q].y;
        const float pre = bn ? fmaf(g.y, xhat, b.y) : zz;
        xr[q][k].y = on ? xhat : 0.f;
        dr[q][k].y = (on && pre > 0.f) ? dr[q][k].y : 0.f;
        sg.y = fmaf(dr[q][k].y, xr[q][k].y, sg.y);
        sb.y += dr[q][k].y;
      }
    }
    sg = col_reduce2(sg, red[sub], tx, ty);
    sb = col_reduce2(sb, red[sub], tx, ty);
    if (ty == 0) {
      sums[n][0][2 * tx] = sg.x; sums[n][0][2 * tx + 1] = sg.y;
      sums[n][1][2 * tx] = sb.x; sums[n][1][2 * tx + 1] = sb.y;
    }
    const float2 kk = {g.x * rstd[q].x, g.y * rstd[q].y};
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
      const int r = ty + RL * k;
      float vx = 0.f, vy = 0.f;
      if (live && r < R) {
        vx = bn ? kk.x * (dr[q][k].x - sb.x * invR - xr[q][k].x * sg.x * invR) : dr[q][k].x;
        vy = bn ? kk.y * (dr[q][k].y - sb.y * invR - xr[q][k].y * sg.y * invR) : dr[q][k].y;
        *reinterpret_cast<uint32_t*>(&dz[(int64_t)(rb + r) * lddz + c]) = (uint32_t)f32_to_bf16(vx) | ((uint32_t)f32_to_bf16(vy) << 16);
      }
      if (dzT) { tile[sub][2 * tx][r] = f32_to_bf16(vx * tscale); tile[sub][2 * tx + 1][r] = f32_to_bf16(vy * tscale); }
    }
    if (dzT) {
      __syncthreads();                            // (the next round writes the tile behind its reductions' barriers)
      store_transposed_pair(tile[sub], dzT + rb, ldt, c0, C, R, t);
    }
  }
  // small-vector gradients: added up in node order and folded in once, as in the kernels above
  __syncthreads();
  if (sub == 0 && ty == 0 && live) {
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      float tg = 0.f, tb = 0.f;
#pragma unroll
      for (int n = 0; n < G; ++n) {
        if (n < count) {
          tg = n ? tg + sums[n][0][2 * tx + e] : sums[n][0][2 * tx + e];
          tb = n ? tb + sums[n][1][2 * tx + e] : sums[n][1][2 * tx + e];
        }
      }
      if (bn) grad_store(gout_g, c + e, tg);
      if (gout_b.dst) grad_store(gout_b, c + e, tb);
    }
  }
}

// Scale / shift (or bias) gradients from per-node column sums [nodes][2][C] (left by a product whose
// epilogue took the BatchNorm backward pass): added up in node order and folded in once, as the
// group kernels do.
__global__ __launch_bounds__(256) void bn_sums_finish_kernel(const float* __restrict__ sums, int nodes, int C,
                                                             GradOut gout_g, GradOut gout_b) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= C) return;
  float tg = 0.f, tb = 0.f;
  for (int n0 = 0; n0 < nodes; n0 += 16) {         // sixteen nodes' loads in flight together
    float sg[16], sb[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const int n = min(n0 + k, nodes - 1);
      sg[k] = sums[((int64_t)n * 2 + 0) * C + c];
      sb[k] = sums[((int64_t)n * 2 + 1) * C + c];
    }
#pragma unroll
    for (int k = 0; k < 16; ++k)
      if (n0 + k < nodes) {
        tg = (n0 + k) ? tg + sg[k] : sg[k];
        tb = (n0 + k) ? tb + sb[k] : sb[k];
      }
  }
  if (gout_g.dst) grad_store(gout_g, c, tg);
  if (gout_b.dst) grad_store(gout_b, c, tb);
}

// Moving statistics from per-node batch statistics [nodes][C] (left by a product whose epilogue took
// the BatchNorm forward pass): one blend per node, node after node (Section 4.1), as the kernels above.
__global__ __launch_bounds__(256) void bn_stats_finish_kernel(const float* __restrict__ mean, const float* __restrict__ var,
                                                              int nodes, int C, float* __restrict__ run_mean,
                                                              float* __restrict__ run_var, float run_mix) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= C) return;
  float rm = run_mean[c], rv = run_var[c];
  for (int n0 = 0; n0 < nodes; n0 += 16) {
    float m[16], v[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const int n = min(n0 + k, nodes - 1);
      m[k] = mean[(int64_t)n * C + c];
      v[k] = var[(int64_t)n * C + c];
    }
#pragma unroll
    for (int k = 0; k < 16; ++k)
      if (n0 + k < nodes) {
        rm = fmaf(run_mix, m[k] - rm, rm);
        rv = fmaf(run_mix, v[k] - rv, rv);
      }
  }
  run_mean[c] = rm; run_var[c] = rv;
}

constexpr int SCB = 32, SRL = 8;
template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(const T* __restrict__ x, int64_t ld, int R, int C,
                                                     GradOut out) {
  __shared__ float red[SRL][SCB + 1];
  const int tx = threadIdx.x % SCB, ty = threadIdx.x / SCB;
  const int c = blockIdx.x * SCB + tx;
  float s = 0.f;
  if (c < C)
    for (int r = ty; r < R; r += SRL) s += load_f(&x[(int64_t)r * ld + c]);
  red[ty][tx] = s;
  __syncthreads();
  if (ty == 0 && c < C) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < SRL; ++i) t += red[i][tx];
    grad_store(out, c, t);
  }
}

// out[r] = sum_c x[r*ld + c]: one wavefront per row (bias gradient from a transposed gradient)
__global__ __launch_bounds__(256) void rowsum_kernel(const bf16_t* __restrict__ x, int64_t ld, int R, int C,
                                                     GradOut out) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= R) return;
  float s = 0.f;
  for (int c = lane; c < C; c += 64) s += bf16_to_f32(x[(int64_t)r * ld + c]);
  s = wave_sum(s);
  if (lane == 0) grad_store(out, r, s);
}

// Bias gradients of a fold window: one wavefront per row, the nodes one after another.
__global__ __launch_bounds__(256) void rowsum_nodes_kernel(NodeList nl, int64_t ld, int R, float* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= R) return;
  float c = nl.overwrite ? 0.f : out[r];
  for (int j = 0; j < nl.count; ++j) {
    const bf16_t* __restrict__ x = nl.src[j];
    float s = 0.f;
    for (int k = lane; k < nl.rows[j]; k += 64) s += bf16_to_f32(x[(int64_t)r * ld + k]);
    s = wave_sum(s);
    c = fmaf(nl.w[j], s, c);
  }
  if (lane == 0) out[r] = c;
}

}  // namespace

// Sub-groups of 256 threads per workgroup of the group kernels: four while that is what it takes to
// give every compute unit enough threads, two for wide layers (whose column blocks alone do).
// VF_BN_SUBGROUPS = 2 | 4 overrides (tuning aid).
// Whether the two-column kernels take a layer of C columns: even, and wide enough that blocks of 32
// columns still give every compute unit a workgroup.  VF_BN_PAIR = 0 switches them off, 1 takes
// them for every even width (tuning and testing aid).
bool pair_width(int C) {
  static const int mode = std::getenv("VF_BN_PAIR") ? std::atoi(std::getenv("VF_BN_PAIR")) : -1;
  if (mode == 0 || (C & 1)) return false;
  return mode == 1 || (C + CB2 - 1) / CB2 >= 192;
}
bool aligned_to(const void* p, uintptr_t n) { return (reinterpret_cast<uintptr_t>(p) & (n - 1)) == 0; }

int group_subgroups(int grid) {
  static const int forced = std::getenv("VF_BN_SUBGROUPS") ? std::atoi(std::getenv("VF_BN_SUBGROUPS")) : 0;
  if (forced == 2 || forced == 4) return forced;
  return grid <= 256 ? 4 : 2;
}

// The row ranges of a unit's nodes for the group kernels: `group` nodes of R rows each, or of
// node_rows[n] rows when given.  Every node at most 128 rows; ranges start on multiples of 8 when
// transposed copies are written.
int group_rows(int group, int R, const int* node_rows, bool transposed, GroupRows* gr) {
  if (group < 2 || group > kBnGroupPair) return VF_EINVAL;
  int at = 0;
  for (int n = 0; n < kBnGroupPair; ++n) {
    const int rows = n < group ? (node_rows ? node_rows[n] : R) : 0;
    if (n < group && (rows < 1 || rows > RCH || (transposed && (rows & 7)))) return VF_EINVAL;
    gr->base[n] = n < group ? at : 0;
    gr->rows[n] = rows;
    at += rows;
  }
  return VF_OK;
}

int launch_bn_relu_fwd(const float* zp, int nsplit, int64_t slab, int64_t ldzp, int R, int C,
                       const float* gamma, const float* beta, int round_params, float eps, float* z,
                       int64_t ldz, void* a, int64_t lda, int a_is_bf16, bf16_t* aT, int64_t ldt,
                       float* mean, float* rstd, float* run_mean, float* run_var, float run_mix,
                       hipStream_t s, int group, const int* node_rows) {
  if (R <= 0 || C <= 0 || nsplit < 1) return VF_EINVAL;
  const bool pair = group >= 2 && nsplit == 1 && zp == z && a_is_bf16 && pair_width(C) && !(ldz & 1) && !(lda & 1) &&
                    aligned_to(z, 8) && aligned_to(a, 4) && aligned_to(gamma, 8) && aligned_to(beta, 8) &&
                    aligned_to(mean, 8) && aligned_to(rstd, 8);
  const int per = pair ? kBnGroupPair : kBnGroup;
  if (group > per) {
    // a unit of more nodes than a launch takes: one launch per `per` nodes, in node order (the moving
    // statistics are blended node after node by launches that follow each other on the stream)
    if (!a_is_bf16) return VF_EINVAL;
    int64_t row = 0;
    for (int n0 = 0; n0 < group; n0 += per) {
      const int cnt = std::min(per, group - n0);
      int64_t rows = 0;
      for (int n = 0; n < cnt; ++n) rows += node_rows ? node_rows[n0 + n] : R;
      VF_TRY(launch_bn_relu_fwd(zp + row * ldzp, nsplit, slab, ldzp, node_rows ? node_rows[n0] : R, C, gamma, beta,
                                round_params, eps, z + row * ldz, ldz, static_cast<bf16_t*>(a) + row * lda, lda, 1,
                                aT ? aT + row : nullptr, ldt, mean + (int64_t)n0 * C, rstd + (int64_t)n0 * C, run_mean,
                                run_var, run_mix, s, cnt, node_rows ? node_rows + n0 : nullptr));
      row += rows;
    }
    return VF_OK;
  }
  if ((run_mean == nullptr) != (run_var == nullptr)) return VF_EINVAL;
  if (aT && ((ldt & 7) || !a_is_bf16)) return VF_EINVAL;
  const int grid = (C + CB - 1) / CB;
  const int subgroups = group_subgroups(grid);
  const bool small = R <= RCH;
  GroupRows gr{};
  if (group != 1) {
    if (!a_is_bf16) return VF_EINVAL;
    VF_TRY(group_rows(group, R, node_rows, aT != nullptr, &gr));
  }
  if (pair) {
    const int pgrid = (C + CB2 - 1) / CB2;
#define VF_FWDP(GG, SS)                                                                              \
  bn_relu_fwd_pair_kernel<GG, SS><<<pgrid, GroupShape<GG, SS>::THREADS, 0, s>>>(z, ldz, gr, group, C, gamma, beta, \
      round_params, eps, static_cast<bf16_t*>(a), lda, aT, ldt, mean, rstd, run_mean, run_var, run_mix)
    if (group > 8) VF_FWDP(16, 4);
    else if (group > 4) VF_FWDP(8, 4);
    else if (group > 2) VF_FWDP(4, 4);
    else VF_FWDP(2, 2);
#undef VF_FWDP
    VF_LAUNCH_CHECK();
    return VF_OK;
  }
#define VF_FWD2(TT, NS, SM, GG)                                                                    \
  bn_relu_fwd_kernel<TT, NS, SM, GG><<<grid, 256, 0, s>>>(zp, slab, ldzp, R, C, gamma, beta, round_params, \
      eps, z, ldz, static_cast<TT*>(a), lda, aT, ldt, mean, rstd, run_mean, run_var, run_mix)
#define VF_FWDG1(NS, GG, SS)                                                                        \
  bn_relu_fwd_group_kernel<NS, GG, SS><<<grid, GroupShape<GG, SS>::THREADS, 0, s>>>(zp, slab, ldzp, gr, group, C, gamma, beta, \
      round_params, eps, z, ldz, static_cast<bf16_t*>(a), lda, aT, ldt, mean, rstd, run_mean, run_var, run_mix)
#define VF_FWDG(NS, GG)                                                                            \
  do { if (subgroups == 4) VF_FWDG1(NS, GG, 4); else VF_FWDG1(NS, GG, 2); } while (0)
#define VF_FWD(NS)                                                                                 \
  case NS:                                                                                         \
    if (group == 2) VF_FWDG(NS, 2);                                                                \
    else if (group > 2 && group <= 4) VF_FWDG(NS, 4);                                              \
    else if (group > 4) VF_FWDG(NS, 8);                                                            \
    else if (a_is_bf16) { if (small) VF_FWD2(bf16_t, NS, true, 1); else VF_FWD2(bf16_t, NS, false, 1); } \
    else           { if (small) VF_FWD2(float, NS, true, 1);  else VF_FWD2(float, NS, false, 1); } \
    break;
  switch (nsplit) {
    VF_FWD(1) VF_FWD(2) VF_FWD(4) VF_FWD(8) VF_FWD(16) VF_FWD(32)
    default: return VF_EINVAL;
  }
#undef VF_FWD
#undef VF_FWDG
#undef VF_FWDG1
#undef VF_FWD2
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_bn_relu_bwd(float* dap, int nsplit, int64_t slab, int64_t ldda, const float* z,
                       int64_t ldz, int R, int C, const float* gamma, const float* beta,
                       int round_params, const float* mean, const float* rstd, void* dz, int64_t lddz,
                       int dz_is_bf16, bf16_t* dzT, int64_t ldt, GradOut gout_g, GradOut gout_b,
                       hipStream_t s, float tscale, int group, const int* node_rows) {
  if (R <= 0 || C <= 0 || nsplit < 1) return VF_EINVAL;
  const bool pair = group >= 2 && nsplit == 1 && dz_is_bf16 && pair_width(C) && !(ldz & 1) && !(ldda & 1) && !(lddz & 1) &&
                    aligned_to(z, 8) && aligned_to(dap, 8) && aligned_to(dz, 4) && aligned_to(gamma, 8) &&
                    aligned_to(beta, 8) && aligned_to(mean, 8) && aligned_to(rstd, 8);
  if (group > kBnGroup) {
    // a unit of more than kBnGroup nodes: one launch per kBnGroup nodes; the small-vector gradients
    // of the later launches are added to what the first one left
    if (!dz_is_bf16) return VF_EINVAL;
    int64_t row = 0;
    for (int n0 = 0; n0 < group; n0 += kBnGroup) {
      const int cnt = std::min(kBnGroup, group - n0);
      int64_t rows = 0;
      for (int n = 0; n < cnt; ++n) rows += node_rows ? node_rows[n0 + n] : R;
      GradOut gg = gout_g, gb = gout_b;
      if (n0) { gg.accumulate = 1; gb.accumulate = 1; }
      VF_TRY(launch_bn_relu_bwd(dap + row * ldda, nsplit, slab, ldda, z + row * ldz, ldz, node_rows ? node_rows[n0] : R, C,
                                gamma, beta, round_params, mean + (int64_t)n0 * C, rstd + (int64_t)n0 * C,
                                static_cast<bf16_t*>(dz) + row * lddz, lddz, 1, dzT ? dzT + row : nullptr, ldt, gg, gb, s,
                                tscale, cnt, node_rows ? node_rows + n0 : nullptr));
      row += rows;
    }
    return VF_OK;
  }
  if (dzT && ((ldt & 7) || !dz_is_bf16)) return VF_EINVAL;
  const int grid = (C + CB - 1) / CB;
  const int subgroups = group_subgroups(grid);
  const bool small = R <= RCH;
  GroupRows gr{};
  if (group != 1) {
    if (!dz_is_bf16) return VF_EINVAL;
    VF_TRY(group_rows(group, R, node_rows, dzT != nullptr, &gr));
  }
  if (pair) {
    const int pgrid = (C + CB2 - 1) / CB2;
#define VF_BWDP(GG, SS)                                                                              \
  bn_relu_bwd_pair_kernel<GG, SS><<<pgrid, GroupShape<GG, SS>::THREADS, 0, s>>>(dap, ldda, z, ldz, gr, group, C, gamma, \
      beta, round_params, mean, rstd, static_cast<bf16_t*>(dz), lddz, dzT, ldt, gout_g, gout_b, tscale)
    if (group > 4) VF_BWDP(8, 4);
    else if (group > 2) VF_BWDP(4, 4);
    else VF_BWDP(2, 2);
#undef VF_BWDP
    VF_LAUNCH_CHECK();
    return VF_OK;
  }
#define VF_BWD2(TT, NS, SM, GG)                                                                    \
  bn_relu_bwd_kernel<TT, NS, SM, GG><<<grid, 256, 0, s>>>(dap, slab, ldda, z, ldz, R, C, gamma, beta,  \
      round_params, mean, rstd, static_cast<TT*>(dz), lddz, dzT, ldt, gout_g, gout_b, tscale)
#define VF_BWDG1(NS, GG, SS)                                                                        \
  bn_relu_bwd_group_kernel<NS, GG, SS><<<grid, GroupShape<GG, SS>::THREADS, 0, s>>>(dap, slab, ldda, z, ldz, gr, group, C, gamma, \
      beta, round_params, mean, rstd, static_cast<bf16_t*>(dz), lddz, dzT, ldt, gout_g, gout_b, tscale)
#define VF_BWDG(NS, GG)                                                                            \
  do { if (subgroups == 4) VF_BWDG1(NS, GG, 4); else VF_BWDG1(NS, GG, 2); } while (0)
#define VF_BWD(NS)                                                                                 \
  case NS:                                                                                         \
    if (group == 2) VF_BWDG(NS, 2);                                                                \
    else if (group > 2 && group <= 4) VF_BWDG(NS, 4);                                              \
    else if (group > 4) VF_BWDG(NS, 8);                                                            \
    else if (dz_is_bf16) { if (small) VF_BWD2(bf16_t, NS, true, 1); else VF_BWD2(bf16_t, NS, false, 1); } \
    else            { if (small) VF_BWD2(float, NS, true, 1);  else VF_BWD2(float, NS, false, 1); } \
    break;
  switch (nsplit) {
    VF_BWD(1) VF_BWD(2) VF_BWD(4) VF_BWD(8) VF_BWD(16) VF_BWD(32)
    default: return VF_EINVAL;
  }
#undef VF_BWD
#undef VF_BWDG
#undef VF_BWDG1
#undef VF_BWD2
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_bn_stats_finish(const float* mean, const float* var, int nodes, int C, float* run_mean, float* run_var,
                           float run_mix, hipStream_t s) {
  if (!mean || !var || !run_mean || !run_var || nodes < 1 || C <= 0) return VF_EINVAL;
  bn_stats_finish_kernel<<<(C + 255) / 256, 256, 0, s>>>(mean, var, nodes, C, run_mean, run_var, run_mix);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_bn_sums_finish(const float* sums, int nodes, int C, GradOut gout_g, GradOut gout_b, hipStream_t s) {
  if (!sums || nodes < 1 || C <= 0) return VF_EINVAL;
  bn_sums_finish_kernel<<<(C + 255) / 256, 256, 0, s>>>(sums, nodes, C, gout_g, gout_b);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_colsum(const void* x, int64_t ld, int x_is_bf16, int R, int C, GradOut out,
                  hipStream_t s) {
  if (R <= 0 || C <= 0) return VF_EINVAL;
  int grid = (C + SCB - 1) / SCB;
  if (x_is_bf16) colsum_kernel<bf16_t><<<grid, 256, 0, s>>>(static_cast<const bf16_t*>(x), ld, R, C, out);
  else           colsum_kernel<float><<<grid, 256, 0, s>>>(static_cast<const float*>(x), ld, R, C, out);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_rowsum_nodes(const NodeList& nl, int64_t ld, int R, float* out, hipStream_t s) {
  if (nl.count < 1 || nl.count > kFoldMax || R <= 0 || !out) return VF_EINVAL;
  for (int j = 0; j < nl.count; ++j)
    if (!nl.src[j] || nl.rows[j] < 1 || nl.rows[j] > ld) return VF_EINVAL;
  rowsum_nodes_kernel<<<(R + 3) / 4, 256, 0, s>>>(nl, ld, R, out);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_rowsum_bf16(const bf16_t* x, int64_t ld, int R, int C, GradOut out, hipStream_t s) {
  if (R <= 0 || C <= 0) return VF_EINVAL;
  rowsum_kernel<<<(R + 3) / 4, 256, 0, s>>>(x, ld, R, C, out);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

}  // namespace vf
