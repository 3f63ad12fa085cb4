// Row-wise and element-wise kernels of the pre-LayerNorm encoder: embedding gather and its
// deterministic scatter-add backward, LayerNorm forward/backward, exact GELU, row softmax.
// All statistics and reductions in fp32; one wavefront per row where a row is reduced.
#include <algorithm>

#include <cstdlib>

#include "vf_device.h"

namespace vf {
namespace {

constexpr int NT = 256;
constexpr int WAVES = NT / 64;

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

__global__ __launch_bounds__(NT) void embed_fwd_kernel(const int32_t* __restrict__ ids,
                                                       const float* __restrict__ tok,
                                                       const float* __restrict__ pos, int R, int T, int d,
                                                       int vocab, int round_params, float* __restrict__ h) {
  const int r = blockIdx.x;
  const int id = clampi(ids[r], 0, vocab - 1);
  const int t = r % T;
  for (int c = threadIdx.x; c < d; c += NT) {
    float a = tok[(int64_t)id * d + c], b = pos[(int64_t)t * d + c];
    if (round_params) { a = round_bf16(a); b = round_bf16(b); }
    h[(int64_t)r * d + c] = a + b;
  }
}

__global__ __launch_bounds__(NT) void embed_pos_bwd_kernel(const float* __restrict__ dh, int nseq, int T,
                                                           int d, GradOut out) {
  const int t = blockIdx.x;
  for (int c = threadIdx.x; c < d; c += NT) {
    float s = 0.f;
    int q = 0;
    for (; q + 8 <= nseq; q += 8) {              // eight sequences' values in flight, added in sequence order
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = dh[((int64_t)(q + u) * T + t) * d + c];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; q < nseq; ++q) s += dh[((int64_t)q * T + t) * d + c];
    grad_store(out, (int64_t)t * d + c, s);
  }
}

// One workgroup per token r.  The first token that carries a given id (the "leader") adds up
// the rows of all tokens with that id in increasing token order and writes the table row;
// the other workgroups exit.  No atomics: the sum order is fixed.  The workgroup first marks
// the matching tokens in an LDS bitmap (one coalesced scan of the ids), then every thread
// walks the set bits for its columns.
constexpr int MAX_TOK_WORDS = 2048;     // bitmap capacity: 65536 tokens per node
__global__ __launch_bounds__(NT) void embed_tok_bwd_kernel(const int32_t* __restrict__ ids,
                                                           const float* __restrict__ dh, int R, int d,
                                                           int vocab, GradOut out) {
  __shared__ uint32_t match[MAX_TOK_WORDS];
  __shared__ int list[256];      // matching tokens of the current batch, in increasing order
  __shared__ int nlist, next_word;
  __shared__ int earlier;
  const int r = blockIdx.x;
  const int id = clampi(ids[r], 0, vocab - 1);
  const int nwords = (R + 31) / 32;
  if (threadIdx.x == 0) earlier = 0;
  for (int wd = threadIdx.x; wd < nwords; wd += NT) match[wd] = 0u;
  __syncthreads();
  for (int q0 = 0; q0 < R; q0 += 8 * NT) {          // eight loads of ids in flight per thread
    int other[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) other[u] = ids[min(q0 + u * NT + (int)threadIdx.x, R - 1)];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int q = q0 + u * NT + threadIdx.x;
      const bool hit = q < R && clampi(other[u], 0, vocab - 1) == id;
      if (hit) {
        if (q < r) earlier = 1;                       // benign race: every writer stores 1
        else atomicOr(&match[q >> 5], 1u << (q & 31));  // LDS bit set; order does not matter
      }
    }
  }
  __syncthreads();
  if (earlier) return;
  // Walk the bitmap in batches of up to 256 matches: thread 0 lists them in increasing order,
  // then every thread adds its columns of those rows, 8 independent loads at a time.
  constexpr int CPT = 4;                            // columns per thread: d <= 1024
  float acc[CPT] = {0.f, 0.f, 0.f, 0.f};
  if (threadIdx.x == 0) next_word = r >> 5;
  __syncthreads();
  while (true) {
    if (threadIdx.x == 0) {
      int n = 0, wd = next_word;
      for (; wd < nwords && n <= 256 - 32; ++wd) {
        uint32_t bits = match[wd];
        while (bits) {
          list[n++] = (wd << 5) + __ffs(bits) - 1;
          bits &= bits - 1;
        }
      }
      nlist = n;
      next_word = wd;
    }
    __syncthreads();
    const int n = nlist;
    const bool last = next_word >= nwords;
    for (int k0 = 0; k0 < n; k0 += 8) {
#pragma unroll
      for (int j = 0; j < CPT; ++j) {
        const int c = threadIdx.x + NT * j;
        if (c < d) {
          float v[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) v[u] = (k0 + u < n) ? dh[(int64_t)list[k0 + u] * d + c] : 0.f;
#pragma unroll
          for (int u = 0; u < 8; ++u) acc[j] += v[u];   // increasing token order; padding adds +0
        }
      }
    }
    __syncthreads();
    if (last) break;
  }
#pragma unroll
  for (int j = 0; j < CPT; ++j) {
    const int c = threadIdx.x + NT * j;
    if (c < d) grad_store(out, (int64_t)id * d + c, acc[j]);
  }
}

// The same with 16-byte accesses (d a multiple of 4, d <= 1024) and the matching rows dealt out
// to the four wavefronts: wavefront w adds the matches k = w, w + 4, w + 8, .. of the increasing
// list, eight rows in flight per lane (read at clamped list positions, selected afterwards, so no
// load waits behind a branch), and the four partial sums are joined in wavefront order.  An id
// that many tokens share (the id that stands in for masked positions: 15 % of a node's tokens)
// is the launch's critical path: 32 rows in flight for it instead of 8.  The order of the
// additions is fixed, so the result is the same on every run.
__global__ __launch_bounds__(NT) void embed_tok_bwd4_kernel(const int32_t* __restrict__ ids,
                                                            const float* __restrict__ dh, int R, int d,
                                                            int vocab, GradOut out) {
  __shared__ uint32_t match[MAX_TOK_WORDS];
  __shared__ int list[256];
  __shared__ int scan[NT];
  __shared__ int earlier;
  __shared__ __attribute__((aligned(16))) float part[3 * 1024];
  const int r = blockIdx.x;
  const int id = clampi(ids[r], 0, vocab - 1);
  const int nwords = (R + 31) / 32;
  if (threadIdx.x == 0) earlier = 0;
  for (int wd = threadIdx.x; wd < nwords; wd += NT) match[wd] = 0u;
  __syncthreads();
  for (int q0 = 0; q0 < R; q0 += 8 * NT) {
    int other[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) other[u] = ids[min(q0 + u * NT + (int)threadIdx.x, R - 1)];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int q = q0 + u * NT + threadIdx.x;
      const bool hit = q < R && clampi(other[u], 0, vocab - 1) == id;
      if (hit) {
        if (q < r) earlier = 1;
        else atomicOr(&match[q >> 5], 1u << (q & 31));
      }
    }
  }
  __syncthreads();
  if (earlier) return;
  constexpr int CPL = 4;                            // 16-byte columns per lane: d <= 1024
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float4 acc[CPL];
#pragma unroll
  for (int j = 0; j < CPL; ++j) acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
  // The matching tokens in increasing order, 256 at a time.  Every thread owns eight words of the
  // bitmap: it counts their bits, a scan over the threads gives each word the position of its
  // first match in the whole list, and for each window of 256 positions a thread writes the
  // matches of its words that fall into it (one thread walking the whole bitmap bit by bit was
  // the critical path of the launch for an id that many tokens share).
  constexpr int WPT = MAX_TOK_WORDS / NT;
  int cnt[WPT], mine = 0;
#pragma unroll
  for (int i = 0; i < WPT; ++i) {
    const int wd = threadIdx.x * WPT + i;
    cnt[i] = wd < nwords ? __popc(match[wd]) : 0;
    mine += cnt[i];
  }
  scan[threadIdx.x] = mine;
  __syncthreads();
  for (int off = 1; off < NT; off <<= 1) {
    const int add = (int)threadIdx.x >= off ? scan[threadIdx.x - off] : 0;
    __syncthreads();
    scan[threadIdx.x] += add;
    __syncthreads();
  }
  const int first = scan[threadIdx.x] - mine;       // list position of this thread's first match
  const int total = scan[NT - 1];
  for (int base = 0; base < total; base += 256) {
    int o = first;
#pragma unroll
    for (int i = 0; i < WPT; ++i) {
      if (cnt[i] && o < base + 256 && o + cnt[i] > base) {
        const int wd = threadIdx.x * WPT + i;
        uint32_t bits = match[wd];
        int at = o;
        while (bits) {
          if (at >= base && at < base + 256) list[at - base] = (wd << 5) + __ffs(bits) - 1;
          ++at;
          bits &= bits - 1;
        }
      }
      o += cnt[i];
    }
    __syncthreads();
    const int n = min(256, total - base);
    for (int k0 = 0; k0 < n; k0 += 32) {
      int row[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) row[u] = list[min(k0 + 4 * u + wave, n - 1)];
      // the loads of all column groups before the first addition (one trip to memory per 32
      // rows, not one per column group); a column group beyond the row is skipped by everybody
      float4 v[CPL][8];
#pragma unroll
      for (int j = 0; j < CPL; ++j) {
        if (256 * j < d) {
          const int c = min(4 * lane + 256 * j, d - 4);
#pragma unroll
          for (int u = 0; u < 8; ++u) v[j][u] = *reinterpret_cast<const float4*>(&dh[(int64_t)row[u] * d + c]);
        }
      }
#pragma unroll
      for (int j = 0; j < CPL; ++j) {
        if (256 * j < d) {
#pragma unroll
          for (int u = 0; u < 8; ++u) {             // padding adds +0
            const bool live = k0 + 4 * u + wave < n;
            acc[j].x += live ? v[j][u].x : 0.f;
            acc[j].y += live ? v[j][u].y : 0.f;
            acc[j].z += live ? v[j][u].z : 0.f;
            acc[j].w += live ? v[j][u].w : 0.f;
          }
        }
      }
    }
    __syncthreads();
  }
  // join the wavefronts' sums in wavefront order; wavefront 0 writes the table row
  if (wave > 0) {
#pragma unroll
    for (int j = 0; j < CPL; ++j) {
      const int c = 4 * lane + 256 * j;
      if (c < d) *reinterpret_cast<float4*>(&part[(wave - 1) * 1024 + c]) = acc[j];
    }
  }
  __syncthreads();
  if (wave > 0) return;
  float4 old[CPL];
#pragma unroll
  for (int j = 0; j < CPL; ++j) {
    const int c = min(4 * lane + 256 * j, d - 4);
    old[j] = *reinterpret_cast<const float4*>(&out.dst[(int64_t)id * d + c]);
  }
#pragma unroll
  for (int j = 0; j < CPL; ++j) {
    const int c = 4 * lane + 256 * j;
    if (c < d) {
      float4 t = acc[j];
#pragma unroll
      for (int w = 0; w < 3; ++w) {
        const float4 p = *reinterpret_cast<const float4*>(&part[w * 1024 + c]);
        t.x += p.x; t.y += p.y; t.z += p.z; t.w += p.w;
      }
      const float4 o = out.accumulate ? old[j] : make_float4(0.f, 0.f, 0.f, 0.f);
      *reinterpret_cast<float4*>(&out.dst[(int64_t)id * d + c]) =
          make_float4(fmaf(out.alpha, t.x, o.x), fmaf(out.alpha, t.y, o.y), fmaf(out.alpha, t.z, o.z),
                      fmaf(out.alpha, t.w, o.w));
    }
  }
}

__global__ __launch_bounds__(NT) void extract_masked_kernel(const int32_t* __restrict__ y, int nseq, int m,
                                                            int T, int vocab, int32_t* __restrict__ rowidx,
                                                            int32_t* __restrict__ labels) {
  const int i = blockIdx.x * NT + threadIdx.x;
  if (i >= nseq * m) return;
  const int sq = i / m, j = i % m;
  const int p = clampi(y[(int64_t)sq * 2 * m + j], 0, T - 1);
  rowidx[i] = sq * T + p;
  labels[i] = clampi(y[(int64_t)sq * 2 * m + m + j], 0, vocab - 1);
}

// ---- LayerNorm: one wavefront per row ------------------------------------------------------
constexpr int LN_JMAX = 16;     // columns per lane held in registers: d <= 64*LN_JMAX
template <typename T>
__global__ __launch_bounds__(NT) void layernorm_fwd_kernel(const float* __restrict__ x, int64_t ldx,
                                                           const int32_t* __restrict__ row_map, int R,
                                                           int d, const float* __restrict__ gamma,
                                                           const float* __restrict__ beta,
                                                           int round_params, float eps, T* __restrict__ y,
                                                           int64_t ldy, float* __restrict__ mean_out,
                                                           float* __restrict__ rstd_out) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * WAVES + (threadIdx.x >> 6);
  if (r >= R) return;
  const float* xr = x + (int64_t)(row_map ? row_map[r] : r) * ldx;
  if (d <= 64 * LN_JMAX) {
    // The row lives in registers.  Loads go to clamped (always valid) columns and come before
    // any selection, so all of a lane's loads are in flight together; sums in column order.
    float v[LN_JMAX], g[LN_JMAX], b[LN_JMAX];
#pragma unroll
    for (int j = 0; j < LN_JMAX; ++j) {
      const int c = min(lane + 64 * j, d - 1);
      v[j] = xr[c]; g[j] = gamma[c]; b[j] = beta[c];
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < LN_JMAX; ++j) s += (lane + 64 * j < d) ? v[j] : 0.f;
    const float mean = wave_sum(s) / (float)d;
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < LN_JMAX; ++j) {
      const float t = (lane + 64 * j < d) ? v[j] - mean : 0.f;
      q = fmaf(t, t, q);
    }
    const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)d + eps);
#pragma unroll
    for (int j = 0; j < LN_JMAX; ++j) {
      const int c = lane + 64 * j;
      if (round_params) { g[j] = round_bf16(g[j]); b[j] = round_bf16(b[j]); }
      if (c < d) store_f(&y[(int64_t)r * ldy + c], fmaf(g[j], (v[j] - mean) * rstd, b[j]));
    }
    if (lane == 0) { mean_out[r] = mean; rstd_out[r] = rstd; }
    return;
  }
  float s = 0.f;
  for (int c = lane; c < d; c += 64) s += xr[c];
  const float mean = wave_sum(s) / (float)d;
  float q = 0.f;
  for (int c = lane; c < d; c += 64) {
    float v = xr[c] - mean;
    q = fmaf(v, v, q);
  }
  const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)d + eps);
  for (int c = lane; c < d; c += 64) {
    float g = gamma[c], b = beta[c];
    if (round_params) { g = round_bf16(g); b = round_bf16(b); }
    store_f(&y[(int64_t)r * ldy + c], fmaf(g, (xr[c] - mean) * rstd, b));
  }
  if (lane == 0) { mean_out[r] = mean; rstd_out[r] = rstd; }
}

// Backward of LayerNorm for `rows_per_wg` consecutive rows per workgroup (one wavefront per
// row at a time).  Besides dx it produces this row chunk's contribution to dgamma and dbeta
// (partial[0][chunk][c], partial[1][chunk][c]) so that no second pass over dy and x is needed;
// layernorm_param_finish adds the chunks in order.
__global__ __launch_bounds__(NT) void layernorm_bwd_kernel(const float* __restrict__ dyp, int nsplit,
                                                           int64_t slab, int64_t lddy,
                                                           const float* __restrict__ x, int64_t ldx,
                                                           const int32_t* __restrict__ row_map, int R,
                                                           int d, const float* __restrict__ gamma,
                                                           int round_params,
                                                           const float* __restrict__ mean_in,
                                                           const float* __restrict__ rstd_in,
                                                           const float* __restrict__ dres,
                                                           float* __restrict__ dx, int64_t lddx,
                                                           int rows_per_wg, float* __restrict__ partial,
                                                           int64_t pstride) {
  extern __shared__ __attribute__((aligned(16))) float wsum[];   // [2][WAVES][d]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int chunk = blockIdx.x;
  const int rbeg = chunk * rows_per_wg;
  const int rend = min(R, rbeg + rows_per_wg);
  float pg[LN_JMAX], pb[LN_JMAX];
#pragma unroll
  for (int j = 0; j < LN_JMAX; ++j) { pg[j] = 0.f; pb[j] = 0.f; }
  for (int r = rbeg + wave; r < rend; r += WAVES) {
    const int64_t orow = row_map ? row_map[r] : r;
    const float* xr = x + orow * ldx;
    const float mean = mean_in[r], rstd = rstd_in[r];
    float dyv[LN_JMAX], xhv[LN_JMAX], resv[LN_JMAX], gv[LN_JMAX];
    float s1 = 0.f, s2 = 0.f;
    // All loads first, at clamped (always valid) columns, so that they are in flight together;
    // the selection of the live columns follows.
#pragma unroll
    for (int j = 0; j < LN_JMAX; ++j) {
      const int c = min(lane + 64 * j, d - 1);
      resv[j] = dres ? dres[orow * lddx + c] : 0.f;
      dyv[j] = dyp[(int64_t)r * lddy + c];
      xhv[j] = xr[c];
      gv[j] = gamma[c];
    }
    for (int s = 1; s < nsplit; ++s) {            // the slabs in order
#pragma unroll
      for (int j = 0; j < LN_JMAX; ++j)
        dyv[j] += dyp[(int64_t)s * slab + (int64_t)r * lddy + min(lane + 64 * j, d - 1)];
    }
#pragma unroll
    for (int j = 0; j < LN_JMAX; ++j) {
      const bool on = lane + 64 * j < d;
      if (round_params) gv[j] = round_bf16(gv[j]);
      const float dy = on ? dyv[j] : 0.f;
      const float xh = on ? (xhv[j] - mean) * rstd : 0.f;
      dyv[j] = dy; xhv[j] = xh;
      if (on) {
        const float dxh = dy * gv[j];
        s1 += dxh;
        s2 = fmaf(dxh, xh, s2);
        pg[j] = fmaf(dy, xh, pg[j]);
        pb[j] += dy;
      }
    }
    s1 = wave_sum(s1) / (float)d;
    s2 = wave_sum(s2) / (float)d;
#pragma unroll
    for (int j = 0; j < LN_JMAX; ++j) {
      const int c = lane + 64 * j;
      if (c < d) {
        float v = (dyv[j] * gv[j] - s1 - xhv[j] * s2) * rstd;
        dx[orow * lddx + c] = v + resv[j];
      }
    }
  }
  if (!partial) return;
#pragma unroll
  for (int j = 0; j < LN_JMAX; ++j) {
    const int c = lane + 64 * j;
    if (c < d) { wsum[(0 * WAVES + wave) * d + c] = pg[j]; wsum[(1 * WAVES + wave) * d + c] = pb[j]; }
  }
  __syncthreads();
  for (int c = threadIdx.x; c < d; c += NT) {
    float a = 0.f, b = 0.f;
#pragma unroll
    for (int wv = 0; wv < WAVES; ++wv) { a += wsum[(0 * WAVES + wv) * d + c]; b += wsum[(1 * WAVES + wv) * d + c]; }
    partial[(int64_t)chunk * d + c] = a;
    partial[pstride + (int64_t)chunk * d + c] = b;
  }
}

// The same with 16-byte accesses: a lane owns columns 4 lane + 256 j .. + 3 (j < 4: d <= 1024).
// Requires d % 4 == 0, leading dimensions multiples of 4, 16-byte aligned bases.
__global__ __launch_bounds__(NT) void layernorm_bwd4_kernel(const float* __restrict__ dyp, int nsplit,
                                                            int64_t slab, int64_t lddy,
                                                            const float* __restrict__ x, int64_t ldx,
                                                            const int32_t* __restrict__ row_map, int R,
                                                            int d, const float* __restrict__ gamma,
                                                            int round_params,
                                                            const float* __restrict__ mean_in,
                                                            const float* __restrict__ rstd_in,
                                                            const float* __restrict__ dres,
                                                            float* __restrict__ dx, int64_t lddx,
                                                            int rows_per_wg, float* __restrict__ partial,
                                                            int64_t pstride) {
  extern __shared__ __attribute__((aligned(16))) float wsum[];   // [2][WAVES][d]
  constexpr int JQ = 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int chunk = blockIdx.x;
  const int rbeg = chunk * rows_per_wg;
  const int rend = min(R, rbeg + rows_per_wg);
  float4 pg[JQ], pb[JQ], gv[JQ];
#pragma unroll
  for (int j = 0; j < JQ; ++j) {
    pg[j] = make_float4(0.f, 0.f, 0.f, 0.f); pb[j] = pg[j];
    const int c = min(4 * lane + 256 * j, d - 4);
    gv[j] = *reinterpret_cast<const float4*>(&gamma[c]);
    if (round_params) { gv[j].x = round_bf16(gv[j].x); gv[j].y = round_bf16(gv[j].y); gv[j].z = round_bf16(gv[j].z); gv[j].w = round_bf16(gv[j].w); }
  }
  for (int r = rbeg + wave; r < rend; r += WAVES) {
    const int64_t orow = row_map ? row_map[r] : r;
    const float* xr = x + orow * ldx;
    const float mean = mean_in[r], rstd = rstd_in[r];
    float4 dyv[JQ], xhv[JQ], resv[JQ];
    // all loads first, at clamped (always valid) columns, so that they are in flight together
#pragma unroll
    for (int j = 0; j < JQ; ++j) {
      const int c = min(4 * lane + 256 * j, d - 4);
      resv[j] = dres ? *reinterpret_cast<const float4*>(&dres[orow * lddx + c]) : make_float4(0.f, 0.f, 0.f, 0.f);
      dyv[j] = *reinterpret_cast<const float4*>(&dyp[(int64_t)r * lddy + c]);
      xhv[j] = *reinterpret_cast<const float4*>(&xr[c]);
    }
    for (int s = 1; s < nsplit; ++s) {            // the slabs in order
#pragma unroll
      for (int j = 0; j < JQ; ++j) {
        const float4 t = *reinterpret_cast<const float4*>(&dyp[(int64_t)s * slab + (int64_t)r * lddy + min(4 * lane + 256 * j, d - 4)]);
        dyv[j].x += t.x; dyv[j].y += t.y; dyv[j].z += t.z; dyv[j].w += t.w;
      }
    }
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int j = 0; j < JQ; ++j) {
      const bool on = 4 * lane + 256 * j < d;
      float* dyp4 = reinterpret_cast<float*>(&dyv[j]);
      float* xh4 = reinterpret_cast<float*>(&xhv[j]);
      const float* g4 = reinterpret_cast<const float*>(&gv[j]);
      float* pg4 = reinterpret_cast<float*>(&pg[j]);
      float* pb4 = reinterpret_cast<float*>(&pb[j]);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float dy = on ? dyp4[e] : 0.f;
        const float xh = on ? (xh4[e] - mean) * rstd : 0.f;
        dyp4[e] = dy; xh4[e] = xh;
        const float dxh = dy * g4[e];
        s1 += dxh;
        s2 = fmaf(dxh, xh, s2);
        pg4[e] = fmaf(dy, xh, pg4[e]);
        pb4[e] += dy;
      }
    }
    s1 = wave_sum(s1) / (float)d;
    s2 = wave_sum(s2) / (float)d;
#pragma unroll
    for (int j = 0; j < JQ; ++j) {
      const int c = 4 * lane + 256 * j;
      if (c < d) {
        float4 o;
        o.x = (dyv[j].x * gv[j].x - s1 - xhv[j].x * s2) * rstd + resv[j].x;
        o.y = (dyv[j].y * gv[j].y - s1 - xhv[j].y * s2) * rstd + resv[j].y;
        o.z = (dyv[j].z * gv[j].z - s1 - xhv[j].z * s2) * rstd + resv[j].z;
        o.w = (dyv[j].w * gv[j].w - s1 - xhv[j].w * s2) * rstd + resv[j].w;
        *reinterpret_cast<float4*>(&dx[orow * lddx + c]) = o;
      }
    }
  }
  if (!partial) return;
#pragma unroll
  for (int j = 0; j < JQ; ++j) {
    const int c = 4 * lane + 256 * j;
    if (c < d) {
      *reinterpret_cast<float4*>(&wsum[(0 * WAVES + wave) * d + c]) = pg[j];
      *reinterpret_cast<float4*>(&wsum[(1 * WAVES + wave) * d + c]) = pb[j];
    }
  }
  __syncthreads();
  for (int c = threadIdx.x; c < d; c += NT) {
    float a = 0.f, b = 0.f;
#pragma unroll
    for (int wv = 0; wv < WAVES; ++wv) { a += wsum[(0 * WAVES + wv) * d + c]; b += wsum[(1 * WAVES + wv) * d + c]; }
    partial[(int64_t)chunk * d + c] = a;
    partial[pstride + (int64_t)chunk * d + c] = b;
  }
}

// out_g[c] = sum over chunks of partial[0][chunk][c]; out_b likewise from partial[1].
// 16 columns per workgroup, 16 chunk lanes (lane q adds chunks q, q+16, ...), combined in lane order.
__device__ __forceinline__ void layernorm_param_finish_body(const float* __restrict__ partial, int64_t pstride,
                                                            int nchunk, int d, GradOut gout_g, GradOut gout_b,
                                                            int wg) {
  __shared__ float red[2][16][17];
  const int tx = threadIdx.x & 15, q = threadIdx.x >> 4;
  const int c = wg * 16 + tx;
  float a = 0.f, b = 0.f;
  if (c < d)
    for (int k = q; k < nchunk; k += 16) { a += partial[(int64_t)k * d + c]; b += partial[pstride + (int64_t)k * d + c]; }
  red[0][q][tx] = a;
  red[1][q][tx] = b;
  __syncthreads();
  if (q == 0 && c < d) {
    float sa = 0.f, sb = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) { sa += red[0][i][tx]; sb += red[1][i][tx]; }
    grad_store(gout_g, c, sa);
    grad_store(gout_b, c, sb);
  }
}

__global__ __launch_bounds__(NT) void layernorm_param_finish_kernel(const float* __restrict__ partial,
                                                                    int64_t pstride, int nchunk, int d,
                                                                    GradOut gout_g, GradOut gout_b) {
  layernorm_param_finish_body(partial, pstride, nchunk, d, gout_g, gout_b, blockIdx.x);
}

// Column sums over many rows in two steps: partial sums per row chunk, then the chunks in order.
template <typename T>
__global__ __launch_bounds__(NT) void colsum_partial_kernel(const T* __restrict__ xin, int64_t ld, int R, int C,
                                                            int rows_per_chunk, float* __restrict__ partial) {
  __shared__ float red[8][33];
  const int tx = threadIdx.x % 32, ty = threadIdx.x / 32;
  const int c = blockIdx.x * 32 + tx;
  const int rbeg = blockIdx.y * rows_per_chunk, rend = min(R, rbeg + rows_per_chunk);
  float s = 0.f;
  if (c < C) {
    int r = rbeg + ty;
    for (; r + 24 < rend; r += 32) {            // four loads in flight, added in row order
      const float v0 = load_f(&xin[(int64_t)r * ld + c]);
      const float v1 = load_f(&xin[(int64_t)(r + 8) * ld + c]);
      const float v2 = load_f(&xin[(int64_t)(r + 16) * ld + c]);
      const float v3 = load_f(&xin[(int64_t)(r + 24) * ld + c]);
      s += v0; s += v1; s += v2; s += v3;
    }
    for (; r < rend; r += 8) s += load_f(&xin[(int64_t)r * ld + c]);
  }
  red[ty][tx] = s;
  __syncthreads();
  if (ty == 0 && c < C) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) t += red[i][tx];
    partial[(int64_t)blockIdx.y * C + c] = t;
  }
}

// 64 columns per workgroup, 4 chunk lanes (lane q adds chunks q, q+4, ...), combined in lane order.
__device__ __forceinline__ void colsum_finish_body(const float* __restrict__ partial, int nchunk, int C,
                                                   GradOut out, int wg) {
  __shared__ float red[4][64];
  const int tx = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int c = wg * 64 + tx;
  float a = 0.f;
  if (c < C)
    for (int k = q; k < nchunk; k += 4) a += partial[(int64_t)k * C + c];
  red[q][tx] = a;
  __syncthreads();
  if (q == 0 && c < C) grad_store(out, c, (red[0][tx] + red[1][tx]) + (red[2][tx] + red[3][tx]));
}
__global__ __launch_bounds__(NT) void colsum_finish_kernel(const float* __restrict__ partial, int nchunk, int C,
                                                           GradOut out) {
  colsum_finish_body(partial, nchunk, C, out, blockIdx.x);
}

// Several finish steps in one launch: workgroup w belongs to the job whose range of workgroups
// holds it (wg_end = running totals) and does what that job's own kernel would do.
struct FinishArgs {
  FinishJob job[kFinishJobs];
  int wg_end[kFinishJobs];
  int count;
};
__global__ __launch_bounds__(NT) void finish_jobs_kernel(FinishArgs fa) {
  int j = 0;
  while (j < fa.count - 1 && (int)blockIdx.x >= fa.wg_end[j]) ++j;
  const int wg = blockIdx.x - (j ? fa.wg_end[j - 1] : 0);
  const FinishJob& J = fa.job[j];
  if (J.kind == 0) colsum_finish_body(J.partial, J.nchunk, J.C, J.a, wg);
  else layernorm_param_finish_body(J.partial, J.pstride, J.nchunk, J.C, J.a, J.b, wg);
}

// One pass over a gradient matrix dy [R, C] that feeds a Linear layer's backward pass, 64 x 64
// tiles: the transposed bf16 copy the weight-gradient product reads, (fp32 input) the bf16 copy
// in place the input-gradient product reads, and per-tile column sums of the values as read
// (partial[tile row][c]), which colsum_finish_kernel adds in tile order: the bias gradient.
// Loads come first, at clamped positions; rows at or past R add nothing.
// fp32 input: C % 4 == 0, ld % 4 == 0.  Every thread reads 16 bytes, writes 8 in both orientations.
__global__ __launch_bounds__(NT) void dy_f32_prepare_kernel(const float* __restrict__ in, int64_t ldi,
                                                            bf16_t* __restrict__ nat, int64_t ldn,
                                                            bf16_t* __restrict__ tr, int64_t ldt,
                                                            float* __restrict__ partial, int R, int C) {
  __shared__ bf16_t tile[64][64 + 2];
  __shared__ float red[16][64];
  const int q = threadIdx.x & 15, g = threadIdx.x >> 4;      // 16 quads per row, 16 row groups
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  float4 vin[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    vin[i] = *reinterpret_cast<const float4*>(&in[(int64_t)min(r0 + g + 16 * i, R - 1) * ldi + min(c0 + 4 * q, C - 4)]);
  float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int rl = g + 16 * i, r = r0 + rl, c = c0 + 4 * q;
    bf16_t h[4] = {0, 0, 0, 0};
    if (r < R && c < C) {
      const float4 v = vin[i];
      sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
      h[0] = f32_to_bf16(v.x); h[1] = f32_to_bf16(v.y); h[2] = f32_to_bf16(v.z); h[3] = f32_to_bf16(v.w);
      uint2 pk;
      pk.x = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
      pk.y = (uint32_t)h[2] | ((uint32_t)h[3] << 16);
      *reinterpret_cast<uint2*>(&nat[(int64_t)r * ldn + c]) = pk;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) tile[rl][4 * q + u] = h[u];
  }
  red[g][4 * q] = sum.x; red[g][4 * q + 1] = sum.y; red[g][4 * q + 2] = sum.z; red[g][4 * q + 3] = sum.w;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int cl = g + 16 * i, c = c0 + cl, r = r0 + 4 * q;
    if (c < C && r < R) {      // rows past R inside the quad are padding of ldt
      uint2 pk;
      pk.x = (uint32_t)tile[4 * q][cl] | ((uint32_t)tile[4 * q + 1][cl] << 16);
      pk.y = (uint32_t)tile[4 * q + 2][cl] | ((uint32_t)tile[4 * q + 3][cl] << 16);
      *reinterpret_cast<uint2*>(&tr[(int64_t)c * ldt + r]) = pk;
    }
  }
  if (threadIdx.x < 64 && c0 + threadIdx.x < C) {
    float t = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) t += red[k][threadIdx.x];
    partial[(int64_t)blockIdx.y * C + c0 + threadIdx.x] = t;
  }
}

// bf16 input: C % 8 == 0, ldi % 8 == 0, ldt % 8 == 0 and ldt >= R rounded up to 8 (the transposed
// rows are written in whole 16-byte vectors; the columns past R receive copies of row R-1).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(NT) void dy_bf16_prepare_kernel(const bf16_t* __restrict__ in, int64_t ldi,
                                                             bf16_t* __restrict__ tr, int64_t ldt,
                                                             float* __restrict__ partial, int R, int C) {
  __shared__ __attribute__((aligned(16))) bf16_t tile[64][64 + 8];
  __shared__ float red[4][64];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int v = threadIdx.x & 7, row = threadIdx.x >> 3;     // 8 vectors per row, 32 rows per pass
  u32x4 x[2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
    x[i] = *reinterpret_cast<const u32x4*>(&in[(int64_t)min(r0 + row + 32 * i, R - 1) * ldi + min(c0 + 8 * v, C - 8)]);
#pragma unroll
  for (int i = 0; i < 2; ++i) *reinterpret_cast<u32x4*>(&tile[row + 32 * i][8 * v]) = x[i];
  __syncthreads();
  {
    const int col = threadIdx.x & 63, part = threadIdx.x >> 6;   // 16 rows of one column, in row order
    float t = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const int rl = part * 16 + k;
      const float val = bf16_to_f32(tile[rl][col]);
      t += (r0 + rl < R) ? val : 0.f;
    }
    red[part][col] = t;
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int col = (threadIdx.x >> 3) + 32 * i;             // output row = input column
    const int rb = 8 * (threadIdx.x & 7);                    // eight input rows -> one 16-byte vector
    u32x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      o[e] = (uint32_t)tile[rb + 2 * e][col] | ((uint32_t)tile[rb + 2 * e + 1][col] << 16);
    if (c0 + col < C && r0 + rb < R)
      *reinterpret_cast<u32x4*>(&tr[(int64_t)(c0 + col) * ldt + r0 + rb]) = o;
  }
  __syncthreads();
  if (threadIdx.x < 64 && c0 + threadIdx.x < C)
    partial[(int64_t)blockIdx.y * C + c0 + threadIdx.x] =
        (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
}

// ---- GELU (exact) ---------------------------------------------------------------------------
// The pre-activation u is what a Linear layer put out: fp32 in every workload (only operands of
// contractions are bf16).  T is the type of the GELU output (the next Linear layer's operand) and
// of the gradient du handed to the backward products.
__device__ __forceinline__ float gelu_f(float v) { return 0.5f * v * (1.0f + erff(v * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_df(float v) {
  const float cdf = 0.5f * (1.0f + erff(v * 0.70710678118654752f));
  const float pdf = 0.3989422804014327f * expf(-0.5f * v * v);
  return cdf + v * pdf;
}
template <typename T>
__global__ __launch_bounds__(NT) void gelu_fwd_kernel(const float* __restrict__ u, T* __restrict__ g, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * NT;
  for (; i < n; i += stride) store_f(&g[i], gelu_f(u[i]));
}

// Eight elements per lane and trip (16-byte accesses, bf16 out); n % 8 == 0, 16-byte aligned.
__global__ __launch_bounds__(NT) void gelu_fwd8_kernel(const float4* __restrict__ u, uint4* __restrict__ g, int64_t nvec) {
  int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * NT;
  for (; i < nvec; i += stride) {
    const float4 u0 = u[2 * i], u1 = u[2 * i + 1];
    const float v[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
    uint32_t o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
      o[e] = (uint32_t)f32_to_bf16(gelu_f(v[2 * e])) | ((uint32_t)f32_to_bf16(gelu_f(v[2 * e + 1])) << 16);
    g[i] = make_uint4(o[0], o[1], o[2], o[3]);
  }
}
__global__ __launch_bounds__(NT) void gelu_bwd8_kernel(const float4* __restrict__ dg, const float4* __restrict__ u,
                                                       uint4* __restrict__ du, int64_t nvec) {
  int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * NT;
  for (; i < nvec; i += stride) {
    const float4 u0 = u[2 * i], u1 = u[2 * i + 1];
    const float4 d0 = dg[2 * i], d1 = dg[2 * i + 1];
    const float v[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
    const float d[8] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
    uint32_t o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
      o[e] = (uint32_t)f32_to_bf16(d[2 * e] * gelu_df(v[2 * e])) |
             ((uint32_t)f32_to_bf16(d[2 * e + 1] * gelu_df(v[2 * e + 1])) << 16);
    du[i] = make_uint4(o[0], o[1], o[2], o[3]);
  }
}

template <typename T>
__global__ __launch_bounds__(NT) void gelu_bwd_kernel(const float* __restrict__ dg, const float* __restrict__ u,
                                                      T* __restrict__ du, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * NT;
  for (; i < n; i += stride) store_f(&du[i], dg[i] * gelu_df(u[i]));
}

// ---- row softmax: one wavefront per row --------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(NT) void softmax_rows_kernel(const float* __restrict__ S, T* __restrict__ P,
                                                          int64_t rows, int n) {
  const int lane = threadIdx.x & 63;
  const int64_t r = (int64_t)blockIdx.x * WAVES + (threadIdx.x >> 6);
  if (r >= rows) return;
  const float* sr = S + r * n;
  float mx = -INFINITY;
  for (int c = lane; c < n; c += 64) mx = fmaxf(mx, sr[c]);
  mx = wave_max(mx);
  float sum = 0.f;
  for (int c = lane; c < n; c += 64) sum += expf(sr[c] - mx);
  const float inv = 1.0f / wave_sum(sum);
  for (int c = lane; c < n; c += 64) store_f(&P[r * n + c], expf(sr[c] - mx) * inv);
}

template <typename T>
__global__ __launch_bounds__(NT) void softmax_rows_bwd_kernel(float* __restrict__ dP, const T* __restrict__ P,
                                                              int64_t rows, int n) {
  const int lane = threadIdx.x & 63;
  const int64_t r = (int64_t)blockIdx.x * WAVES + (threadIdx.x >> 6);
  if (r >= rows) return;
  float dot = 0.f;
  for (int c = lane; c < n; c += 64) dot = fmaf(dP[r * n + c], load_f(&P[r * n + c]), dot);
  dot = wave_sum(dot);
  for (int c = lane; c < n; c += 64) {
    float p = load_f(&P[r * n + c]);
    dP[r * n + c] = p * (dP[r * n + c] - dot);
  }
}

__global__ __launch_bounds__(NT) void reduce_slabs_kernel(const float* __restrict__ in, int nsplit,
                                                          int64_t slab, int64_t n, float* __restrict__ out) {
  int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * NT;
  for (; i < n; i += stride) {
    float v = in[i];
    for (int s = 1; s < nsplit; ++s) v += in[(int64_t)s * slab + i];
    out[i] = v;
  }
}

inline int blocks_for(int64_t n) {
  int64_t b = (n + NT - 1) / NT;
  return (int)(b > 8192 ? 8192 : (b < 1 ? 1 : b));
}

}  // namespace

int launch_embed_fwd(const int32_t* ids, const float* tok, const float* pos, int R, int T, int d,
                     int vocab, int round_params, float* h, hipStream_t s) {
  if (R <= 0) return VF_EINVAL;
  embed_fwd_kernel<<<R, NT, 0, s>>>(ids, tok, pos, R, T, d, vocab, round_params, h);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_embed_pos_bwd(const float* dh, int nseq, int T, int d, GradOut out, hipStream_t s) {
  embed_pos_bwd_kernel<<<T, NT, 0, s>>>(dh, nseq, T, d, out);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_embed_tok_bwd(const int32_t* ids, const float* dh, int R, int d, int vocab, GradOut out,
                         hipStream_t s) {
  if (R <= 0 || d <= 0 || d > 1024 || (int64_t)R > 32 * (int64_t)MAX_TOK_WORDS) return VF_EINVAL;
  const bool vec4 = (d & 3) == 0 && ((reinterpret_cast<uintptr_t>(dh) | reinterpret_cast<uintptr_t>(out.dst)) & 15) == 0;
  if (vec4) embed_tok_bwd4_kernel<<<R, NT, 0, s>>>(ids, dh, R, d, vocab, out);
  else embed_tok_bwd_kernel<<<R, NT, 0, s>>>(ids, dh, R, d, vocab, out);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_extract_masked(const int32_t* y, int nseq, int m, int T, int vocab, int32_t* rowidx,
                          int32_t* labels, hipStream_t s) {
  extract_masked_kernel<<<(nseq * m + NT - 1) / NT, NT, 0, s>>>(y, nseq, m, T, vocab, rowidx, labels);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_layernorm_fwd(const float* x, int64_t ldx, const int32_t* row_map, int R, int d,
                         const float* gamma, const float* beta, int round_params, float eps, void* y,
                         int64_t ldy, int y_is_bf16, float* mean, float* rstd, hipStream_t s) {
  if (R <= 0 || d <= 0) return VF_EINVAL;
  int grid = (R + WAVES - 1) / WAVES;
  if (y_is_bf16)
    layernorm_fwd_kernel<bf16_t><<<grid, NT, 0, s>>>(x, ldx, row_map, R, d, gamma, beta, round_params, eps,
                                                     static_cast<bf16_t*>(y), ldy, mean, rstd);
  else
    layernorm_fwd_kernel<float><<<grid, NT, 0, s>>>(x, ldx, row_map, R, d, gamma, beta, round_params, eps,
                                                    static_cast<float*>(y), ldy, mean, rstd);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_layernorm_bwd(const float* dyp, int nsplit, int64_t slab, int64_t lddy, const float* x,
                         int64_t ldx, const int32_t* row_map, int R, int d, const float* gamma,
                         int round_params, const float* mean, const float* rstd, const float* dres,
                         float* dx, int64_t lddx, float* scratch, GradOut gout_g, GradOut gout_b,
                         hipStream_t s, FinishList* defer) {
  if (R <= 0 || d <= 0 || nsplit < 1 || d > 64 * LN_JMAX || !scratch) return VF_EINVAL;
  // about one workgroup per compute unit: fewer row chunks for the finish kernel to add up
  static const int ln_wgs = std::getenv("VF_LN_WGS") ? std::atoi(std::getenv("VF_LN_WGS")) : 256;
  const int rows_per_wg = std::max(std::max(WAVES, (R + kLnChunks - 1) / kLnChunks), (R + ln_wgs - 1) / ln_wgs);
  const int nchunk = (R + rows_per_wg - 1) / rows_per_wg;
  int64_t pstride = (int64_t)kLnChunks * d;
  float* later = defer ? defer->take((size_t)2 * nchunk * d) : nullptr;
  if (later) {
    scratch = later;
    pstride = (int64_t)nchunk * d;
  }
  const size_t lds = (size_t)2 * WAVES * d * sizeof(float);
  const bool vec4 = (d & 3) == 0 && (lddy & 3) == 0 && (ldx & 3) == 0 && (lddx & 3) == 0 && (slab & 3) == 0 &&
                    ((reinterpret_cast<uintptr_t>(dyp) | reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(dx) |
                      reinterpret_cast<uintptr_t>(gamma) | reinterpret_cast<uintptr_t>(dres)) & 15) == 0;
  if (vec4)
    layernorm_bwd4_kernel<<<nchunk, NT, lds, s>>>(dyp, nsplit, slab, lddy, x, ldx, row_map, R, d, gamma,
                                                  round_params, mean, rstd, dres, dx, lddx, rows_per_wg,
                                                  scratch, pstride);
  else
    layernorm_bwd_kernel<<<nchunk, NT, lds, s>>>(dyp, nsplit, slab, lddy, x, ldx, row_map, R, d, gamma,
                                                 round_params, mean, rstd, dres, dx, lddx, rows_per_wg,
                                                 scratch, pstride);
  VF_LAUNCH_CHECK();
  if (later) {
    defer->job[defer->count++] = FinishJob{scratch, pstride, nchunk, d, 1, gout_g, gout_b};
    return VF_OK;
  }
  layernorm_param_finish_kernel<<<(d + 15) / 16, NT, 0, s>>>(scratch, pstride, nchunk, d, gout_g, gout_b);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_finish_jobs(FinishList& list, hipStream_t s) {
  if (list.count == 0) return VF_OK;
  FinishArgs fa;
  int total = 0;
  for (int j = 0; j < list.count; ++j) {
    fa.job[j] = list.job[j];
    total += list.job[j].kind == 0 ? (list.job[j].C + 63) / 64 : (list.job[j].C + 15) / 16;
    fa.wg_end[j] = total;
  }
  for (int j = list.count; j < kFinishJobs; ++j) { fa.job[j] = list.job[0]; fa.wg_end[j] = total; }
  fa.count = list.count;
  list.count = 0;
  list.used = 0;       // launches that follow on this stream may take the slices again
  finish_jobs_kernel<<<total, NT, 0, s>>>(fa);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_colsum_rows(const void* x, int64_t ld, int x_is_bf16, int R, int C, float* scratch, GradOut out,
                       hipStream_t s, FinishList* defer) {
  if (R <= 0 || C <= 0 || !scratch) return VF_EINVAL;
  const int rows_per_chunk = std::max(32, (R + kReduceChunks - 1) / kReduceChunks);
  const int nchunk = (R + rows_per_chunk - 1) / rows_per_chunk;
  float* later = defer ? defer->take((size_t)nchunk * C) : nullptr;
  if (later) scratch = later;
  dim3 grid((C + 31) / 32, nchunk);
  if (x_is_bf16)
    colsum_partial_kernel<bf16_t><<<grid, NT, 0, s>>>(static_cast<const bf16_t*>(x), ld, R, C, rows_per_chunk, scratch);
  else
    colsum_partial_kernel<float><<<grid, NT, 0, s>>>(static_cast<const float*>(x), ld, R, C, rows_per_chunk, scratch);
  VF_LAUNCH_CHECK();
  if (later) {
    defer->job[defer->count++] = FinishJob{scratch, 0, nchunk, C, 0, out, out};
    return VF_OK;
  }
  colsum_finish_kernel<<<(C + 63) / 64, NT, 0, s>>>(scratch, nchunk, C, out);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

bool dy_prepare_fits(int is_f32, int64_t ldi, int64_t ldn, int64_t ldt, int R, int C) {
  if (R <= 0 || C <= 0 || (R + 63) / 64 > kReduceChunks) return false;
  if (is_f32) return (C & 3) == 0 && (ldi & 3) == 0 && (ldn & 3) == 0 && (ldt & 3) == 0 && ldt >= ((R + 3) & ~3);
  return (C & 7) == 0 && (ldi & 7) == 0 && (ldt & 7) == 0 && ldt >= ((R + 7) & ~7);
}

int launch_dy_prepare(const void* dy, int dy_is_f32, int64_t ldi, int R, int C, bf16_t* nat, int64_t ldn,
                      bf16_t* tr, int64_t ldt, float* scratch, GradOut out, hipStream_t s, FinishList* defer) {
  if (!dy || !tr || !scratch || (dy_is_f32 && !nat)) return VF_EINVAL;
  if (!dy_prepare_fits(dy_is_f32, ldi, ldn, ldt, R, C)) return VF_EINVAL;
  const uintptr_t bits = reinterpret_cast<uintptr_t>(dy) | reinterpret_cast<uintptr_t>(tr) |
                         (dy_is_f32 ? reinterpret_cast<uintptr_t>(nat) : 0);
  if (bits & 15) return VF_EINVAL;
  dim3 grid((C + 63) / 64, (R + 63) / 64);
  float* later = defer ? defer->take((size_t)grid.y * C) : nullptr;
  if (later) scratch = later;
  if (dy_is_f32)
    dy_f32_prepare_kernel<<<grid, NT, 0, s>>>(static_cast<const float*>(dy), ldi, nat, ldn, tr, ldt, scratch, R, C);
  else
    dy_bf16_prepare_kernel<<<grid, NT, 0, s>>>(static_cast<const bf16_t*>(dy), ldi, tr, ldt, scratch, R, C);
  VF_LAUNCH_CHECK();
  if (later) {
    defer->job[defer->count++] = FinishJob{scratch, 0, (int)grid.y, C, 0, out, out};
    return VF_OK;
  }
  colsum_finish_kernel<<<(C + 63) / 64, NT, 0, s>>>(scratch, (int)grid.y, C, out);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_gelu_fwd(const float* u, void* g, int g_is_bf16, int64_t n, hipStream_t s) {
  if (n <= 0) return VF_OK;
  if (g_is_bf16 && (n & 7) == 0 && ((reinterpret_cast<uintptr_t>(u) | reinterpret_cast<uintptr_t>(g)) & 15) == 0) {
    gelu_fwd8_kernel<<<blocks_for(n / 8), NT, 0, s>>>(reinterpret_cast<const float4*>(u), static_cast<uint4*>(g), n / 8);
    VF_LAUNCH_CHECK();
    return VF_OK;
  }
  if (g_is_bf16) gelu_fwd_kernel<bf16_t><<<blocks_for(n), NT, 0, s>>>(u, static_cast<bf16_t*>(g), n);
  else           gelu_fwd_kernel<float><<<blocks_for(n), NT, 0, s>>>(u, static_cast<float*>(g), n);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_gelu_bwd(const float* dg, const float* u, void* du, int du_is_bf16, int64_t n, hipStream_t s) {
  if (n <= 0) return VF_OK;
  if (du_is_bf16 && (n & 7) == 0 &&
      ((reinterpret_cast<uintptr_t>(u) | reinterpret_cast<uintptr_t>(du) | reinterpret_cast<uintptr_t>(dg)) & 15) == 0) {
    gelu_bwd8_kernel<<<blocks_for(n / 8), NT, 0, s>>>(reinterpret_cast<const float4*>(dg), reinterpret_cast<const float4*>(u),
                                                      static_cast<uint4*>(du), n / 8);
    VF_LAUNCH_CHECK();
    return VF_OK;
  }
  if (du_is_bf16) gelu_bwd_kernel<bf16_t><<<blocks_for(n), NT, 0, s>>>(dg, u, static_cast<bf16_t*>(du), n);
  else            gelu_bwd_kernel<float><<<blocks_for(n), NT, 0, s>>>(dg, u, static_cast<float*>(du), n);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_softmax_rows(const float* S, void* P, int p_is_bf16, int64_t rows, int n, hipStream_t s) {
  if (rows <= 0 || n <= 0) return VF_EINVAL;
  int grid = (int)((rows + WAVES - 1) / WAVES);
  if (p_is_bf16) softmax_rows_kernel<bf16_t><<<grid, NT, 0, s>>>(S, static_cast<bf16_t*>(P), rows, n);
  else           softmax_rows_kernel<float><<<grid, NT, 0, s>>>(S, static_cast<float*>(P), rows, n);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_softmax_rows_bwd(float* dP, const void* P, int p_is_bf16, int64_t rows, int n, hipStream_t s) {
  if (rows <= 0 || n <= 0) return VF_EINVAL;
  int grid = (int)((rows + WAVES - 1) / WAVES);
  if (p_is_bf16) softmax_rows_bwd_kernel<bf16_t><<<grid, NT, 0, s>>>(dP, static_cast<const bf16_t*>(P), rows, n);
  else           softmax_rows_bwd_kernel<float><<<grid, NT, 0, s>>>(dP, static_cast<const float*>(P), rows, n);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_reduce_slabs(const float* in, int nsplit, int64_t slab, int64_t n, float* out, hipStream_t s) {
  if (n <= 0) return VF_OK;
  reduce_slabs_kernel<<<blocks_for(n), NT, 0, s>>>(in, nsplit, slab, n, out);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

}  // namespace vf
