// Bandwidth-bound kernels over flat fp32 vectors: the size-weighted fold of one virtual
// node's gradient into the shared gradient buffer (Section 3.2 step 3 with the weight
// b_i/B of Section 5.2) and the single optimizer update of a step (Section 3.2 step 5).
#include <cstdlib>

#include "vf_device.h"

namespace vf {

namespace {

constexpr int kThreads = 256;
constexpr int kVecPerThread = 4;   // float4 loads in flight per thread and operand

// 16-byte accesses with or without the non-temporal hint.  These kernels read and write every byte
// once; on vectors that do not fit the memory-side cache anyway (a probe of the accumulate pattern
// on 1.44 GB vectors: 5.48 TB/s plain, 5.51 with the hint on the stores alone, 6.18 with it on loads
// and stores), the hint keeps them from displacing one another's lines on the way.
typedef float f32x4v __attribute__((ext_vector_type(4)));
template <bool NT>
__device__ __forceinline__ float4 ld4(const float* p, int64_t v) {
  const f32x4v* q = reinterpret_cast<const f32x4v*>(p) + v;
  const f32x4v r = NT ? __builtin_nontemporal_load(q) : *q;
  return float4{r[0], r[1], r[2], r[3]};
}
template <bool NT>
__device__ __forceinline__ void st4(float* p, int64_t v, float4 x) {
  f32x4v* q = reinterpret_cast<f32x4v*>(p) + v;
  const f32x4v r = {x.x, x.y, x.z, x.w};
  if (NT) __builtin_nontemporal_store(r, q); else *q = r;
}

inline int grid_for(int64_t nvec) {
  int64_t per_block = (int64_t)kThreads * kVecPerThread;
  int64_t blocks = (nvec + per_block - 1) / per_block;
  if (blocks < 1) blocks = 1;
  return (int)blocks;
}

// Each block owns a contiguous chunk of kThreads*kVecPerThread float4 elements; a thread
// issues all its loads before the first arithmetic so kVecPerThread 16-byte requests per
// operand are in flight.
template <bool FIRST, bool NT = false>
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
      gv[i] = ld4<NT>(g, v);
      if (!FIRST) bv[i] = ld4<NT>(buf, v);
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
        st4<NT>(buf, v, o);
      }
    }
  }
  // scalar tail (n not a multiple of 4): handled by the last block's first threads
  if (blockIdx.x == gridDim.x - 1) {
    int64_t t = (nvec << 2) + threadIdx.x;
    if (t < n) buf[t] = FIRST ? fmaf(w, g[t], 0.f) : fmaf(w, g[t], buf[t]);
  }
}

template <bool NT>
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
      gv[i] = ld4<NT>(G, v);
      tv[i] = ld4<NT>(theta, v);
      vv[i] = ld4<NT>(vel, v);
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
        st4<NT>(vel, v, nv);
        st4<NT>(theta, v, nt);
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

template <bool NT>
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
      gv[i] = ld4<NT>(G, v);
      tv[i] = ld4<NT>(theta, v);
      mv[i] = ld4<NT>(m1, v);
      uv[i] = ld4<NT>(m2, v);
    }
#pragma unroll
    for (int i = 0; i < kVecPerThread; ++i) {
      int64_t v = base + (int64_t)i * kThreads;
      if (v < nvec) {
        adam_one(gv[i].x, tv[i].x, mv[i].x, uv[i].x, lr, b1, b2, eps, inv_c1, inv_c2);
        adam_one(gv[i].y, tv[i].y, mv[i].y, uv[i].y, lr, b1, b2, eps, inv_c1, inv_c2);
        adam_one(gv[i].z, tv[i].z, mv[i].z, uv[i].z, lr, b1, b2, eps, inv_c1, inv_c2);
        adam_one(gv[i].w, tv[i].w, mv[i].w, uv[i].w, lr, b1, b2, eps, inv_c1, inv_c2);
        st4<NT>(m1, v, mv[i]);
        st4<NT>(m2, v, uv[i]);
        st4<NT>(theta, v, tv[i]);
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

// The hint for vectors of 64 MB and more.  (Also where a vector would fit the 256 MB memory-side
// cache: C2's update, 167 MB per vector, 5.87 -> 6.12 TB/s with it.)  VF_FLAT_NT = 0 | 1: never |
// always (tuning aid).
inline bool stream_hint(int64_t n) {
  static const int mode = std::getenv("VF_FLAT_NT") ? std::atoi(std::getenv("VF_FLAT_NT")) : -1;
  return mode < 0 ? n >= (int64_t(16) << 20) : mode != 0;
}

}  // namespace

int launch_accumulate(float* buf, const float* g, float w, int64_t n, int first, hipStream_t s) {
  if (n == 0) return VF_OK;
  if (n < 0 || !buf || !g) return VF_EINVAL;
  if (!aligned16(buf) || !aligned16(g)) return VF_EINVAL;
  int grid = grid_for(n >> 2);
  if (stream_hint(n)) {
    if (first) accumulate_kernel<true, true><<<grid, kThreads, 0, s>>>(buf, g, w, n);
    else       accumulate_kernel<false, true><<<grid, kThreads, 0, s>>>(buf, g, w, n);
  } else {
    if (first) accumulate_kernel<true><<<grid, kThreads, 0, s>>>(buf, g, w, n);
    else       accumulate_kernel<false><<<grid, kThreads, 0, s>>>(buf, g, w, n);
  }
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_sgdm(float* theta, float* v, const float* G, float lr, float mu, int64_t n, hipStream_t s) {
  if (n == 0) return VF_OK;
  if (n < 0 || !theta || !v || !G) return VF_EINVAL;
  if (!aligned16(theta) || !aligned16(v) || !aligned16(G)) return VF_EINVAL;
  if (stream_hint(n)) sgdm_kernel<true><<<grid_for(n >> 2), kThreads, 0, s>>>(theta, v, G, lr, mu, n);
  else                sgdm_kernel<false><<<grid_for(n >> 2), kThreads, 0, s>>>(theta, v, G, lr, mu, n);
  VF_LAUNCH_CHECK();
  return VF_OK;
}

int launch_adam(float* theta, float* m, float* u, const float* G, float lr, float b1, float b2,
                float eps, float inv_c1, float inv_c2, int64_t n, hipStream_t s) {
  if (n == 0) return VF_OK;
  if (n < 0 || !theta || !m || !u || !G) return VF_EINVAL;
  if (!aligned16(theta) || !aligned16(m) || !aligned16(u) || !aligned16(G)) return VF_EINVAL;
  if (stream_hint(n)) adam_kernel<true><<<grid_for(n >> 2), kThreads, 0, s>>>(theta, m, u, G, lr, b1, b2, eps, inv_c1, inv_c2, n);
  else                adam_kernel<false><<<grid_for(n >> 2), kThreads, 0, s>>>(theta, m, u, G, lr, b1, b2, eps, inv_c1, inv_c2, n);
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
