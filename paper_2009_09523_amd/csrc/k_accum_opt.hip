// Bandwidth-bound kernels over flat fp32 vectors: the size-weighted fold of one virtual
// node's gradient into the shared gradient buffer (Section 3.2 step 3 with the weight
// b_i/B of Section 5.2) and the single optimizer update of a step (Section 3.2 step 5).
#include "vf_device.h"

namespace vf {

namespace {

constexpr int kThreads = 256;
constexpr int kVecPerThread = 4;   // float4 loads in flight per thread and operand

inline int grid_for(int64_t nvec) {
  int64_t per_block = (int64_t)kThreads * kVecPerThread;
  int64_t blocks = (nvec + per_block - 1) / per_block;
  if (blocks < 1) blocks = 1;
  return (int)blocks;
}

// Each block owns a contiguous chunk of kThreads*kVecPerThread float4 elements; a thread
// issues all its loads before the first arithmetic so kVecPerThread 16-byte requests per
// operand are in flight.
template <bool FIRST>
__global__ __launch_bounds__(kThreads) void accumulate_kernel(float* __restrict__ buf,
                                                              const float* __restrict__ g, float w,
                                                              int64_t n) {
  const int64_t nvec = n >> 2;
  const int64_t base = (int64_t)blockIdx.x * (kThreads * kVecPerThread) + threadIdx.x;
  if (nvec > 0) {   // (fewer than four elements: only the scalar tail below)
    // loads at clamped (always valid) positions, so that none sits behind a branch and all of a
    // thread's requests are in flight together; the stores below are guarded (n >= 4 here)
    float4 gv[kVecPerThread], bv[kVecPerThread];
#pragma unroll
    for (int i = 0; i < kVecPerThread; ++i) {
      const int64_t v = min(base + (int64_t)i * kThreads, nvec - 1);
      gv[i] = reinterpret_cast<const float4*>(g)[v];
      if (!FIRST) bv[i] = reinterpret_cast<const float4*>(buf)[v];
    }
#pragma unroll
    for (int i = 0; i < kVecPerThread; ++i) {
      int64_t v = base + (int64_t)i * kThreads;
      if (v < nvec) {
        float4 o;
        if (FIRST) {
          o.x = fmaf(w, gv[i].x, 0.f); o.y = fmaf(w, gv[i].y, 0.f);
          o.z = fmaf(w, gv[i].z, 0.f); o.w = fmaf(w, gv[i].w, 0.f);
        } else {
          o.x = fmaf(w, gv[i].x, bv[i].x); o.y = fmaf(w, gv[i].y, bv[i].y);
          o.z = fmaf(w, gv[i].z, bv[i].z); o.w = fmaf(w, gv[i].w, bv[i].w);
        }
        reinterpret_cast<float4*>(buf)[v] = o;
      }
    }
  }
  // scalar tail (n not a multiple of 4): handled by the last block's first threads
  if (blockIdx.x == gridDim.x - 1) {
    int64_t t = (nvec << 2) + threadIdx.x;
    if (t < n) buf[t] = FIRST ? fmaf(w, g[t], 0.f) : fmaf(w, g[t], buf[t]);
  }
}

__global__ __launch_bounds__(kThreads) void sgdm_kernel(float* __restrict__ theta,
                                                        float* __restrict__ vel,
                                                        const float* __restrict__ G, float lr,
                                                        float mu, int64_t n) {
  const int64_t nvec = n >> 2;
  const int64_t base = (int64_t)blockIdx.x * (kThreads * kVecPerThread) + threadIdx.x;
  if (nvec > 0) {   // (fewer than four elements: only the scalar tail below)
    float4 gv[kVecPerThread], tv[kVecPerThread], vv[kVecPerThread];
#pragma unroll
    for (int i = 0; i < kVecPerThread; ++i) {       // clamped positions: no load behind a branch
      const int64_t v = min(base + (int64_t)i * kThreads, nvec - 1);
      gv[i] = reinterpret_cast<const float4*>(G)[v];
      tv[i] = reinterpret_cast<const float4*>(theta)[v];
      vv[i] = reinterpret_cast<const float4*>(vel)[v];
    }
#pragma unroll
    for (int i = 0; i < kVecPerThread; ++i) {
      int64_t v = base + (int64_t)i * kThreads;
      if (v < nvec) {
        float4 nv, nt;
        nv.x = fmaf(mu, vv[i].x, gv[i].x); nv.y = fmaf(mu, vv[i].y, gv[i].y);
        nv.z = fmaf(mu, vv[i].z, gv[i].z); nv.w = fmaf(mu, vv[i].w, gv[i].w);
        nt.x = fmaf(-lr, nv.x, tv[i].x); nt.y = fmaf(-lr, nv.y, tv[i].y);
        nt.z = fmaf(-lr, nv.z, tv[i].z); nt.w = fmaf(-lr, nv.w, tv[i].w);
        reinterpret_cast<float4*>(vel)[v] = nv;
        reinterpret_cast<float4*>(theta)[v] = nt;
      }
    }
  }
  if (blockIdx.x == gridDim.x - 1) {
    int64_t t = (nvec << 2) + threadIdx.x;
    if (t < n) {
      float nv = fmaf(mu, vel[t], G[t]);
      vel[t] = nv;
      theta[t] = fmaf(-lr, nv, theta[t]);
    }
  }
}

__device__ __forceinline__ void adam_one(float g, float& th, float& m, float& u, float lr, float b1,
                                         float b2, float eps, float inv_c1, float inv_c2) {
  m = fmaf(b1, m, (1.f - b1) * g);
  u = fmaf(b2, u, (1.f - b2) * g * g);
  float mh = m * inv_c1;
  float uh = u * inv_c2;
  th = th - lr * mh / (sqrtf(uh) + eps);
}

__global__ __launch_bounds__(kThreads) void adam_kernel(float* __restrict__ theta,
                                                        float* __restrict__ m1,
                                                        float* __restrict__ m2,
                                                        const float* __restrict__ G, float lr,
                                                        float b1, float b2, float eps, float inv_c1,
                                                        float inv_c2, int64_t n) {
  const int64_t nvec = n >> 2;
  const int64_t base = (int64_t)blockIdx.x * (kThreads * kVecPerThread) + threadIdx.x;
  if (nvec > 0) {   // (fewer than four elements: only the scalar tail below)
    float4 gv[kVecPerThread], tv[kVecPerThread], mv[kVecPerThread], uv[kVecPerThread];
#pragma unroll
    for (int i = 0; i < kVecPerThread; ++i) {       // clamped positions: no load behind a branch
      const int64_t v = min(base + (int64_t)i * kThreads, nvec - 1);
      gv[i] = reinterpret_cast<const float4*>(G)[v];
      tv[i] = reinterpret_cast<const float4*>(theta)[v];
      mv[i] = reinterpret_cast<const float4*>(m1)[v];
      uv[i] = reinterpret_cast<const float4*>(m2)[v];
    }
#pragma unroll
    for (int i = 0; i < kVecPerThread; ++i) {
      int64_t v = base + (int64_t)i * kThreads;
      if (v < nvec) {
        adam_one(gv[i].x, tv[i].x, mv[i].x, uv[i].x, lr, b1, b2, eps, inv_c1, inv_c2);
        adam_one(gv[i].y, tv[i].y, mv[i].y, uv[i].y, lr, b1, b2, eps, inv_c1, inv_c2);
        adam_one(gv[i].z, tv[i].z, mv[i].z, uv[i].z, lr, b1, b2, eps, inv_c1, inv_c2);
        adam_one(gv[i].w, tv[i].w, mv[i].w, uv[i].w, lr, b1, b2, eps, inv_c1, inv_c2);
        reinterpret_cast<float4*>(m1)[v] = mv[i];
        reinterpret_cast<float4*>(m2)[v] = uv[i];
        reinterpret_cast<float4*>(theta)[v] = tv[i];
      }
    }
  }
  if (blockIdx.x == gridDim.x - 1) {
    int64_t t = (nvec << 2) + threadIdx.x;
    if (t < n) {
      float th = theta[t], m = m1[t], u = m2[t];
      adam_one(G[t], th, m, u, lr, b1, b2, eps, inv_c1, inv_c2);
      theta[t] = th; m1[t] = m; m2[t] = u;
    }
  }
}

__global__ __launch_bounds__(kThreads) void fill_kernel(float* __restrict__ p, float value, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  int64_t stride = (int64_t)gridDim.x * kThreads;
  for (; i < n; i += stride) p[i] = value;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

int launch_accumulate(float* buf, const float* g, float w, int64_t n, int first, hipStream_t s) {
  if (n == 0) return VF_OK;
  if (n < 0 || !buf || !g) return VF_EINVAL;
  if (!aligned16(buf) || !aligned16(g)) return VF_EINVAL;
  int grid = grid_for(n >> 2);
  if (first) accumulate_kernel<true><<<grid, kThreads, 0, s>>>(buf, g, w, n);
  else       accumulate_kernel<false><<<grid, kThreads, 0, s>>>(buf, g, w, n);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_sgdm(float* theta, float* v, const float* G, float lr, float mu, int64_t n, hipStream_t s) {
  if (n == 0) return VF_OK;
  if (n < 0 || !theta || !v || !G) return VF_EINVAL;
  if (!aligned16(theta) || !aligned16(v) || !aligned16(G)) return VF_EINVAL;
  sgdm_kernel<<<grid_for(n >> 2), kThreads, 0, s>>>(theta, v, G, lr, mu, n);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_adam(float* theta, float* m, float* u, const float* G, float lr, float b1, float b2,
                float eps, float inv_c1, float inv_c2, int64_t n, hipStream_t s) {
  if (n == 0) return VF_OK;
  if (n < 0 || !theta || !m || !u || !G) return VF_EINVAL;
  if (!aligned16(theta) || !aligned16(m) || !aligned16(u) || !aligned16(G)) return VF_EINVAL;
  adam_kernel<<<grid_for(n >> 2), kThreads, 0, s>>>(theta, m, u, G, lr, b1, b2, eps, inv_c1, inv_c2, n);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_fill_f32(float* p, float value, int64_t n, hipStream_t s) {
  if (n <= 0) return VF_OK;
  int64_t blocks = (n + kThreads - 1) / kThreads;
  if (blocks > 4096) blocks = 4096;
  fill_kernel<<<(int)blocks, kThreads, 0, s>>>(p, value, n);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

}  // namespace vf
