// Fused softmax cross-entropy: per row logsumexp, loss, and the gradient of the node's mean
// loss w.r.t. the logits in one kernel; then the node loss and the running weighted loss.
#include "vf_device.h"

namespace vf {
namespace {

__device__ __forceinline__ float block_reduce(float v, bool is_max, float* red) {
  v = is_max ? wave_max(v) : wave_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int i = 1; i < 4; ++i) r = is_max ? fmaxf(r, red[i]) : r + red[i];
  __syncthreads();
  return r;
}

// One workgroup per row.  SMALL: the row (C <= 256*CPT classes) lives in registers and global
// memory is read once; otherwise the reduced logits are re-read from z.
constexpr int CPT = 4;

template <int NS>
__device__ __forceinline__ float slab_sum(const float* zp, int nsplit, int64_t slab, int64_t idx) {
  if (NS > 0) {
    float v[NS > 0 ? NS : 1];
#pragma unroll
    for (int s = 0; s < NS; ++s) v[s] = zp[(int64_t)s * slab + idx];
    float t = v[0];
#pragma unroll
    for (int s = 1; s < NS; ++s) t += v[s];
    return t;
  }
  float t = zp[idx];
  for (int s = 1; s < nsplit; ++s) t += zp[(int64_t)s * slab + idx];
  return t;
}

template <typename T, bool SMALL, int NS>
__global__ __launch_bounds__(256) void softmax_xent_kernel(const float* zp, int nsplit,
                                                           int64_t slab, int64_t ldzp,
                                                           float* z, int64_t ldz,
                                                           const int32_t* __restrict__ labels, int R,
                                                           int C, float* __restrict__ rowloss,
                                                           T* __restrict__ dz, int64_t lddz,
                                                           bf16_t* __restrict__ dzT, int64_t ldt, float tscale) {
  __shared__ float red[4];
  __shared__ float zlabel;
  const int r = blockIdx.x;
  float* zr = z + (int64_t)r * ldz;
  int label = labels[r];
  label = label < 0 ? 0 : (label >= C ? C - 1 : label);
  float v[CPT];
  float mx = -INFINITY;
  if (SMALL) {
    // loads at clamped (always valid) columns first, all in flight together; selection after
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int c = min(threadIdx.x + 256 * k, C - 1);
      v[k] = slab_sum<NS>(zp, nsplit, slab, (int64_t)r * ldzp + c);   // slabs in order
    }
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int c = threadIdx.x + 256 * k;
      if (c < C) {
        zr[c] = v[k];
        if (c == label) zlabel = v[k];
      } else {
        v[k] = -INFINITY;
      }
      mx = fmaxf(mx, v[k]);
    }
  } else {
    // Long rows: four columns per trip, their loads issued together, handled in column order.
    // When the logits are reduced in place (one slab that is z itself) nothing is written back.
    const bool in_place = nsplit == 1 && zp + (int64_t)r * ldzp == zr;
    int c = threadIdx.x;
    for (; c + 768 < C; c += 1024) {
      float t[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) t[k] = slab_sum<NS>(zp, nsplit, slab, (int64_t)r * ldzp + c + 256 * k);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (!in_place) zr[c + 256 * k] = t[k];
        if (c + 256 * k == label) zlabel = t[k];
        mx = fmaxf(mx, t[k]);
      }
    }
    for (; c < C; c += 256) {
      const float t = slab_sum<NS>(zp, nsplit, slab, (int64_t)r * ldzp + c);
      if (!in_place) zr[c] = t;
      if (c == label) zlabel = t;
      mx = fmaxf(mx, t);
    }
  }
  mx = block_reduce(mx, true, red);
  float sum = 0.f;
  if (SMALL) {
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      v[k] = expf(v[k] - mx);          // exp(-inf) = 0 for the padding
      sum += v[k];
    }
  } else {
    int c = threadIdx.x;
    for (; c + 768 < C; c += 1024) {
      float t[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) t[k] = zr[c + 256 * k];
#pragma unroll
      for (int k = 0; k < 4; ++k) sum += expf(t[k] - mx);
    }
    for (; c < C; c += 256) sum += expf(zr[c] - mx);
  }
  sum = block_reduce(sum, false, red);
  const float inv = 1.0f / sum;
  const float invR = 1.0f / (float)R;
  T* dr = dz + (int64_t)r * lddz;
  if (SMALL) {
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int c = threadIdx.x + 256 * k;
      if (c < C) {
        float d = (v[k] * inv - (c == label ? 1.f : 0.f)) * invR;
        store_f(&dr[c], d);
        if (dzT) dzT[(int64_t)c * ldt + r] = f32_to_bf16(d * tscale);
      }
    }
  } else {
    int c = threadIdx.x;
    for (; c + 768 < C; c += 1024) {
      float t[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) t[k] = zr[c + 256 * k];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int cc = c + 256 * k;
        const float d = (expf(t[k] - mx) * inv - (cc == label ? 1.f : 0.f)) * invR;
        store_f(&dr[cc], d);
        if (dzT) dzT[(int64_t)cc * ldt + r] = f32_to_bf16(d * tscale);
      }
    }
    for (; c < C; c += 256) {
      float d = (expf(zr[c] - mx) * inv - (c == label ? 1.f : 0.f)) * invR;
      store_f(&dr[c], d);
      if (dzT) dzT[(int64_t)c * ldt + r] = f32_to_bf16(d * tscale);
    }
  }
  if (threadIdx.x == 0) rowloss[r] = logf(sum) + mx - zlabel;   // zlabel: visible after the reductions' barriers
}

// Long rows held in registers: 512 threads, thread t owns the column pairs 2t + 1024k, k < TRIPS
// (C <= 1024 TRIPS), so global memory is read once -- every load of the row is in flight before
// the first reduction -- where the kernel above makes three trips of dependent loads.  One slab,
// even leading dimensions (8-byte loads of logits, 4- or 8-byte stores of the gradient).
// No branch depends on the column: a pair beyond the row is redirected to the row's last pair,
// left out of the reductions by selection, and stores there what that pair's owner stores (the
// same bits to the same address).  With an odd C the last pair's second element is the row's
// first padding element (ldzp, ldz, lddz >= C + 1): read but never used, written as 0.
constexpr int ROW_NT = 512;

__device__ __forceinline__ float block_reduce8(float v, bool is_max, float* red) {
  v = is_max ? wave_max(v) : wave_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int i = 1; i < ROW_NT / 64; ++i) r = is_max ? fmaxf(r, red[i]) : r + red[i];
  __syncthreads();
  return r;
}

template <typename T, int TRIPS>
__global__ __launch_bounds__(ROW_NT) void softmax_xent_row_kernel(const float* __restrict__ zp, int64_t ldzp,
                                                                  float* z, int64_t ldz,
                                                                  const int32_t* __restrict__ labels, int R,
                                                                  int C, float* __restrict__ rowloss,
                                                                  T* __restrict__ dz, int64_t lddz) {
  __shared__ float red[ROW_NT / 64];
  __shared__ float zlabel;
  const int r = blockIdx.x;
  const float* src = zp + (int64_t)r * ldzp;
  float* zr = z + (int64_t)r * ldz;
  int label = labels[r];
  label = label < 0 ? 0 : (label >= C ? C - 1 : label);
  const int clast = (C - 1) & ~1;
  const int c0 = 2 * (int)threadIdx.x;
  float2 v[TRIPS];
#pragma unroll
  for (int k = 0; k < TRIPS; ++k)
    v[k] = *reinterpret_cast<const float2*>(src + min(c0 + 2 * ROW_NT * k, clast));
  float mx = -INFINITY, zl = 0.f;
#pragma unroll
  for (int k = 0; k < TRIPS; ++k) {
    const int c = c0 + 2 * ROW_NT * k;
    const bool own = c <= clast;                 // this thread's own pair, not a redirected one
    const bool second = own && c + 1 < C;
    zl = c == label ? v[k].x : zl;
    zl = (second && c + 1 == label) ? v[k].y : zl;
    mx = fmaxf(mx, fmaxf(own ? v[k].x : -INFINITY, second ? v[k].y : -INFINITY));
  }
  if (src != zr) {   // the logits as the later passes read them
#pragma unroll
    for (int k = 0; k < TRIPS; ++k) {
      const int cc = min(c0 + 2 * ROW_NT * k, clast);
      *reinterpret_cast<float2*>(zr + cc) = make_float2(v[k].x, cc + 1 < C ? v[k].y : 0.f);
    }
  }
  if (((label >> 1) & (ROW_NT - 1)) == (int)threadIdx.x) zlabel = zl;   // the one thread that owns the label's pair
  mx = block_reduce8(mx, true, red);
  float sum = 0.f;
#pragma unroll
  for (int k = 0; k < TRIPS; ++k) {
    const int c = c0 + 2 * ROW_NT * k;
    const bool own = c <= clast;
    const bool second = own && c + 1 < C;
    v[k].x = expf(v[k].x - mx);
    v[k].y = expf(v[k].y - mx);
    sum += own ? v[k].x : 0.f;
    sum += second ? v[k].y : 0.f;
  }
  sum = block_reduce8(sum, false, red);
  const float inv = 1.0f / sum;
  const float invR = 1.0f / (float)R;
  T* dr = dz + (int64_t)r * lddz;
#pragma unroll
  for (int k = 0; k < TRIPS; ++k) {
    const int cc = min(c0 + 2 * ROW_NT * k, clast);
    const float d0 = (v[k].x * inv - (cc == label ? 1.f : 0.f)) * invR;
    const float d1 = (v[k].y * inv - (cc + 1 == label ? 1.f : 0.f)) * invR;
    store_f2(&dr[cc], d0, cc + 1 < C ? d1 : 0.f);
  }
  if (threadIdx.x == 0) rowloss[r] = logf(sum) + mx - zlabel;   // zlabel: visible after the reductions' barriers
}

__global__ __launch_bounds__(256) void loss_reduce_kernel(const float* __restrict__ rowloss, int R,
                                                          float w, int node,
                                                          float* __restrict__ node_loss,
                                                          float* __restrict__ total) {
  __shared__ float red[4];
  float s = 0.f;
  for (int r = threadIdx.x; r < R; r += 256) s += rowloss[r];
  s = block_reduce(s, false, red);
  if (threadIdx.x == 0) {
    float L = s / (float)R;
    node_loss[node] = L;
    float old = node == 0 ? 0.f : *total;
    *total = fmaf(w, L, old);
  }
}

// The same bookkeeping for a run of nodes in one launch: node j's rows start at off[j] of
// `rowloss`; sums and the chain over the nodes are those of one launch per node, node by node.
__global__ __launch_bounds__(256) void loss_reduce_nodes_kernel(const float* __restrict__ rowloss, LossNodes ln,
                                                                float* __restrict__ node_loss,
                                                                float* __restrict__ total) {
  __shared__ float red[4];
  float acc = ln.first == 0 ? 0.f : *total;
  for (int j = 0; j < ln.count; ++j) {
    const int R = ln.rows[j];
    const float* __restrict__ p = rowloss + ln.off[j];
    float s = 0.f;
    for (int r = threadIdx.x; r < R; r += 256) s += p[r];
    s = block_reduce(s, false, red);
    const float L = s / (float)R;
    if (threadIdx.x == 0) node_loss[ln.first + j] = L;
    acc = fmaf(ln.w[j], L, acc);
  }
  if (threadIdx.x == 0) *total = acc;
}

}  // namespace

int launch_loss_reduce_nodes(const float* rowloss, const LossNodes& ln, float* node_loss, float* total,
                             hipStream_t s) {
  if (ln.count < 1 || ln.count > kLossNodes || ln.first < 0 || !rowloss || !node_loss || !total) return VF_EINVAL;
  for (int j = 0; j < ln.count; ++j)
    if (ln.rows[j] < 1 || ln.off[j] < 0) return VF_EINVAL;
  loss_reduce_nodes_kernel<<<1, 256, 0, s>>>(rowloss, ln, node_loss, total);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_softmax_xent(const float* zp, int nsplit, int64_t slab, int64_t ldzp, float* z, int64_t ldz,
                        const int32_t* labels, int R, int C, float* rowloss, void* dz, int64_t lddz,
                        int dz_is_bf16, bf16_t* dzT, int64_t ldt, float w, int node, float* node_loss,
                        float* total, hipStream_t s, float tscale) {
  if (R <= 0 || C <= 0 || nsplit < 1) return VF_EINVAL;
  if (dzT && !dz_is_bf16) return VF_EINVAL;
  if (node_loss && !total) return VF_EINVAL;
  const bool small = C <= 256 * CPT;
  // rows of up to 32768 classes that one workgroup can keep in registers
  const bool even = !(ldzp & 1) && !(ldz & 1) && !(lddz & 1) && !(reinterpret_cast<uintptr_t>(zp) & 7) &&
                    !(reinterpret_cast<uintptr_t>(z) & 7) && !(reinterpret_cast<uintptr_t>(dz) & 7);
  if (!small && nsplit == 1 && !dzT && even && C <= 2 * ROW_NT * 32 &&
      ldzp >= ((C + 1) & ~1) && ldz >= ((C + 1) & ~1) && lddz >= ((C + 1) & ~1)) {
    const int trips = (C + 2 * ROW_NT - 1) / (2 * ROW_NT);
#define VF_SXR(TT, TR)                                                                             \
  softmax_xent_row_kernel<TT, TR><<<R, ROW_NT, 0, s>>>(zp, ldzp, z, ldz, labels, R, C, rowloss,    \
                                                       static_cast<TT*>(dz), lddz)
#define VF_SXR2(TT)                                                                                \
  switch ((trips + 3) / 4) {                                                                       \
    case 1: VF_SXR(TT, 4); break;                                                                  \
    case 2: VF_SXR(TT, 8); break;                                                                  \
    case 3: VF_SXR(TT, 12); break;                                                                 \
    case 4: VF_SXR(TT, 16); break;                                                                 \
    case 5: VF_SXR(TT, 20); break;                                                                 \
    case 6: VF_SXR(TT, 24); break;                                                                 \
    case 7: VF_SXR(TT, 28); break;                                                                 \
    default: VF_SXR(TT, 32); break;                                                                \
  }
    if (dz_is_bf16) { VF_SXR2(bf16_t); } else { VF_SXR2(float); }
#undef VF_SXR2
#undef VF_SXR
    VF_LAUNCH_CHECK();
    if (node_loss) return launch_loss_reduce(rowloss, R, w, node, node_loss, total, s);
    return VF_OK;
  }
#define VF_SX3(TT, SM, NS)                                                                         \
  softmax_xent_kernel<TT, SM, NS><<<R, 256, 0, s>>>(zp, nsplit, slab, ldzp, z, ldz, labels, R, C,  \
                                                    rowloss, static_cast<TT*>(dz), lddz, dzT, ldt, tscale)
#define VF_SX2(TT, SM)                                                                             \
  switch (nsplit) {                                                                                \
    case 1: VF_SX3(TT, SM, 1); break;                                                              \
    case 2: VF_SX3(TT, SM, 2); break;                                                              \
    case 4: VF_SX3(TT, SM, 4); break;                                                              \
    case 8: VF_SX3(TT, SM, 8); break;                                                              \
    case 16: VF_SX3(TT, SM, 16); break;                                                            \
    default: VF_SX3(TT, SM, 0); break;                                                             \
  }
  if (dz_is_bf16) { if (small) { VF_SX2(bf16_t, true) } else { VF_SX2(bf16_t, false) } }
  else            { if (small) { VF_SX2(float, true) }  else { VF_SX2(float, false) } }
#undef VF_SX2
#undef VF_SX3
  VF_LAUNCH_CHECK();
  // the node's loss bookkeeping: a second, tiny launch (folding it into the last workgroup to
  // finish costs a device-scope fence per workgroup, which is slower than the launch)
  if (node_loss) return launch_loss_reduce(rowloss, R, w, node, node_loss, total, s);
  return VF_OK;
}

int launch_loss_reduce(const float* rowloss, int R, float w, int node, float* node_loss,
                       float* total, hipStream_t s) {
  loss_reduce_kernel<<<1, 256, 0, s>>>(rowloss, R, w, node, node_loss, total);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

}  // namespace vf
