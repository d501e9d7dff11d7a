// Fused sumGradients + applyUpdate kernel (Section 2.1 server steps; n-softsync rule of
// Section 2.2 with the per-gradient learning rate of Section 2.4).
//
// One streaming pass over the parameter vector:
//     s      = sum_{l=0}^{c-1} coef_l * g_l            (arrival order, fp32 FMA chain)
//     v'     = m * v + s + decay * theta_i              decay = (sum_l coef_l) * wd
//     theta' = theta_i - v'
// Reads c gradients, theta_i and v once, writes theta_{i+1} and v once (plus an optional bf16
// copy of theta_{i+1}): 4 (c + 4) bytes per parameter, nothing else touches HBM.  The kernel is
// bandwidth bound; each lane moves 16-byte vectors, gradients are read with non-temporal loads
// because they are never read again.
#include "ctx.hpp"

namespace sasgd {

struct GradTable {
  const float* g[kMaxLearners];
  float coef[kMaxLearners];
};

__device__ __forceinline__ bf16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)0x7fc0;   // NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

__device__ __forceinline__ float4 ldg_nt(const float4* p) {
  float4 r;
  r.x = __builtin_nontemporal_load(&p->x);
  r.y = __builtin_nontemporal_load(&p->y);
  r.z = __builtin_nontemporal_load(&p->z);
  r.w = __builtin_nontemporal_load(&p->w);
  return r;
}

__device__ __forceinline__ void stg_nt(float4* p, float4 v) {
  __builtin_nontemporal_store(v.x, &p->x);
  __builtin_nontemporal_store(v.y, &p->y);
  __builtin_nontemporal_store(v.z, &p->z);
  __builtin_nontemporal_store(v.w, &p->w);
}

// One-shot grid: a workgroup of 256 lanes owns ILP consecutive 4 KiB pieces of every stream, so each
// lane keeps ILP * U 16-byte gradient loads in flight.  Measured on MI355X at P = 60 M this shape
// (ILP 4, U 3, non-temporal loads and stores) gave the highest rate of the shapes tried; grid-stride
// loops with fewer, longer-lived workgroups were 5-10 % slower.
template <int ILP, int U, bool EARLY, bool SHADOW>
__global__ __launch_bounds__(256) void apply_update_kernel(const float4* theta_in, float4* theta_out, float4* v,
                                                           uint2* __restrict__ shadow, int64_t n4, int c,
                                                           GradTable t, float m, float decay) {
  const int64_t base = (int64_t)blockIdx.x * (256 * ILP) + threadIdx.x;
  float4 s[ILP], th[ILP], vv[ILP];
#pragma unroll
  for (int e = 0; e < ILP; e++) s[e] = make_float4(0.f, 0.f, 0.f, 0.f);
  if (EARLY) {
#pragma unroll
    for (int e = 0; e < ILP; e++) {
      const int64_t i = base + e * 256;
      if (i < n4) { th[e] = ldg_nt(theta_in + i); vv[e] = ldg_nt(v + i); }
    }
  }
  int l = 0;
  for (; l + U <= c; l += U) {
    float4 g[U][ILP];
#pragma unroll
    for (int u = 0; u < U; u++)
#pragma unroll
      for (int e = 0; e < ILP; e++) {
        const int64_t i = base + e * 256;
        if (i < n4) g[u][e] = ldg_nt(reinterpret_cast<const float4*>(t.g[l + u]) + i);
      }
#pragma unroll
    for (int u = 0; u < U; u++) {           // arrival order l, l+1, ... within every element
      const float cf = t.coef[l + u];
#pragma unroll
      for (int e = 0; e < ILP; e++) {
        s[e].x = fmaf(cf, g[u][e].x, s[e].x);
        s[e].y = fmaf(cf, g[u][e].y, s[e].y);
        s[e].z = fmaf(cf, g[u][e].z, s[e].z);
        s[e].w = fmaf(cf, g[u][e].w, s[e].w);
      }
    }
  }
  for (; l < c; l++) {
    const float cf = t.coef[l];
#pragma unroll
    for (int e = 0; e < ILP; e++) {
      const int64_t i = base + e * 256;
      if (i < n4) {
        float4 g = ldg_nt(reinterpret_cast<const float4*>(t.g[l]) + i);
        s[e].x = fmaf(cf, g.x, s[e].x);
        s[e].y = fmaf(cf, g.y, s[e].y);
        s[e].z = fmaf(cf, g.z, s[e].z);
        s[e].w = fmaf(cf, g.w, s[e].w);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < ILP; e++) {
    const int64_t i = base + e * 256;
    if (i < n4) {
      if (!EARLY) { th[e] = ldg_nt(theta_in + i); vv[e] = ldg_nt(v + i); }
      float4 a = th[e], b = vv[e];
      b.x = fmaf(m, b.x, s[e].x) + decay * a.x;
      b.y = fmaf(m, b.y, s[e].y) + decay * a.y;
      b.z = fmaf(m, b.z, s[e].z) + decay * a.z;
      b.w = fmaf(m, b.w, s[e].w) + decay * a.w;
      a.x -= b.x;
      a.y -= b.y;
      a.z -= b.z;
      a.w -= b.w;
      stg_nt(v + i, b);
      stg_nt(theta_out + i, a);
      if (SHADOW) {
        uint2 o;
        o.x = (uint32_t)f32_to_bf16_rne(a.x) | ((uint32_t)f32_to_bf16_rne(a.y) << 16);
        o.y = (uint32_t)f32_to_bf16_rne(a.z) | ((uint32_t)f32_to_bf16_rne(a.w) << 16);
        shadow[i] = o;
      }
    }
  }
}

// Scalar tail (P not a multiple of 4): at most 3 elements.
__global__ void apply_update_tail_kernel(const float* theta_in, float* theta_out, float* v, bf16_t* shadow,
                                         int64_t begin, int64_t P, int c, GradTable t, float m, float decay) {
  int64_t i = begin + threadIdx.x;
  if (i >= P) return;
  float s = 0.f;
  for (int l = 0; l < c; l++) s = fmaf(t.coef[l], t.g[l][i], s);
  float vv = fmaf(m, v[i], s) + decay * theta_in[i];
  float th = theta_in[i] - vv;
  v[i] = vv;
  theta_out[i] = th;
  if (shadow) shadow[i] = f32_to_bf16_rne(th);
}

template <int ILP, int U, bool EARLY>
static void launch_shape(const UpdateLaunch& u, const GradTable& t, int64_t n4, hipStream_t stream) {
  const int blocks = (int)((n4 + 256 * ILP - 1) / (256 * ILP));
  const float4* tin = reinterpret_cast<const float4*>(u.theta_in);
  float4* tout = reinterpret_cast<float4*>(u.theta_out);
  float4* vv = reinterpret_cast<float4*>(u.v);
  uint2* sh = reinterpret_cast<uint2*>(u.shadow_out);
  if (u.shadow_out)
    hipLaunchKernelGGL((apply_update_kernel<ILP, U, EARLY, true>), dim3(blocks), dim3(256), 0, stream, tin, tout, vv, sh, n4, u.c, t, u.momentum, u.decay);
  else
    hipLaunchKernelGGL((apply_update_kernel<ILP, U, EARLY, false>), dim3(blocks), dim3(256), 0, stream, tin, tout, vv, sh, n4, u.c, t, u.momentum, u.decay);
}

hipError_t launch_apply_update(const UpdateLaunch& u, hipStream_t stream) {
  if (u.P <= 0) return hipSuccess;
  if (u.P / 4 > (int64_t)0x7fffffff * 256) return hipErrorInvalidValue;
  GradTable t;
  for (int l = 0; l < kMaxLearners; l++) {
    t.g[l] = l < u.c ? u.grads[l] : nullptr;
    t.coef[l] = l < u.c ? u.coef[l] : 0.f;
  }
  const int64_t n4 = u.P / 4;
  if (n4 > 0) {
    if (u.c == 1) launch_shape<4, 1, true>(u, t, n4, stream);
    else if (u.c == 2 || u.c == 4) launch_shape<4, 2, true>(u, t, n4, stream);
    else launch_shape<4, 3, false>(u, t, n4, stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (n4 * 4 < u.P) {
    hipLaunchKernelGGL(apply_update_tail_kernel, dim3(1), dim3(64), 0, stream, u.theta_in, u.theta_out, u.v,
                       u.shadow_out, n4 * 4, u.P, u.c, t, u.momentum, u.decay);
    return hipGetLastError();
  }
  return hipSuccess;
}

__global__ void fp32_to_bf16_kernel(const float* __restrict__ src, bf16_t* __restrict__ dst, int64_t n) {
  int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = f32_to_bf16_rne(src[i]);
}
__global__ void bf16_to_fp32_kernel(const bf16_t* __restrict__ src, float* __restrict__ dst, int64_t n) {
  int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
    dst[i] = __uint_as_float((uint32_t)src[i] << 16);
}

hipError_t launch_fp32_to_bf16(const float* src, bf16_t* dst, int64_t n, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  int64_t want = (n + 255) / 256;
  int blocks = (int)(want < 4096 ? want : 4096);
  hipLaunchKernelGGL(fp32_to_bf16_kernel, dim3(blocks), dim3(256), 0, stream, src, dst, n);
  return hipGetLastError();
}
hipError_t launch_bf16_to_fp32(const bf16_t* src, float* dst, int64_t n, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  int64_t want = (n + 255) / 256;
  int blocks = (int)(want < 4096 ? want : 4096);
  hipLaunchKernelGGL(bf16_to_fp32_kernel, dim3(blocks), dim3(256), 0, stream, src, dst, n);
  return hipGetLastError();
}

}  // namespace sasgd
