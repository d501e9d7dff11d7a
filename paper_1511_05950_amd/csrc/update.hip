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

template <int UNROLL, bool SHADOW>
__global__ __launch_bounds__(256) void apply_update_kernel(const float4* __restrict__ theta_in,
                                                           float4* __restrict__ theta_out,
                                                           float4* __restrict__ v,
                                                           uint2* __restrict__ shadow, int64_t n4, int c,
                                                           GradTable t, float m, float decay) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
    float4 th = theta_in[i];
    float4 vv = v[i];
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    int l = 0;
    for (; l + UNROLL <= c; l += UNROLL) {
      float4 g[UNROLL];
#pragma unroll
      for (int u = 0; u < UNROLL; u++) g[u] = ldg_nt(reinterpret_cast<const float4*>(t.g[l + u]) + i);
#pragma unroll
      for (int u = 0; u < UNROLL; u++) {
        float cf = t.coef[l + u];
        s.x = fmaf(cf, g[u].x, s.x);
        s.y = fmaf(cf, g[u].y, s.y);
        s.z = fmaf(cf, g[u].z, s.z);
        s.w = fmaf(cf, g[u].w, s.w);
      }
    }
    for (; l < c; l++) {
      float4 g = ldg_nt(reinterpret_cast<const float4*>(t.g[l]) + i);
      float cf = t.coef[l];
      s.x = fmaf(cf, g.x, s.x);
      s.y = fmaf(cf, g.y, s.y);
      s.z = fmaf(cf, g.z, s.z);
      s.w = fmaf(cf, g.w, s.w);
    }
    vv.x = fmaf(m, vv.x, s.x) + decay * th.x;
    vv.y = fmaf(m, vv.y, s.y) + decay * th.y;
    vv.z = fmaf(m, vv.z, s.z) + decay * th.z;
    vv.w = fmaf(m, vv.w, s.w) + decay * th.w;
    th.x -= vv.x;
    th.y -= vv.y;
    th.z -= vv.z;
    th.w -= vv.w;
    v[i] = vv;
    theta_out[i] = th;
    if (SHADOW) {
      uint2 o;
      o.x = (uint32_t)f32_to_bf16_rne(th.x) | ((uint32_t)f32_to_bf16_rne(th.y) << 16);
      o.y = (uint32_t)f32_to_bf16_rne(th.z) | ((uint32_t)f32_to_bf16_rne(th.w) << 16);
      shadow[i] = o;
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

static int update_blocks() {
  static int blocks = 0;
  if (blocks == 0) {
    const char* e = getenv("SASGD_UPDATE_BLOCKS");
    blocks = e ? atoi(e) : 0;
    if (blocks <= 0) blocks = 256 * 8;   // 8 workgroups per compute unit
  }
  return blocks;
}

hipError_t launch_apply_update(const UpdateLaunch& u, hipStream_t stream) {
  if (u.P <= 0) return hipSuccess;
  GradTable t;
  for (int l = 0; l < kMaxLearners; l++) {
    t.g[l] = l < u.c ? u.grads[l] : nullptr;
    t.coef[l] = l < u.c ? u.coef[l] : 0.f;
  }
  const int64_t n4 = u.P / 4;
  if (n4 > 0) {
    int64_t want = (n4 + 255) / 256;
    int blocks = (int)(want < update_blocks() ? want : update_blocks());
    const float4* tin = reinterpret_cast<const float4*>(u.theta_in);
    float4* tout = reinterpret_cast<float4*>(u.theta_out);
    float4* vv = reinterpret_cast<float4*>(u.v);
    uint2* sh = reinterpret_cast<uint2*>(u.shadow_out);
    if (u.shadow_out) {
      if (u.c >= 6)
        hipLaunchKernelGGL((apply_update_kernel<6, true>), dim3(blocks), dim3(256), 0, stream, tin, tout, vv, sh, n4, u.c, t, u.momentum, u.decay);
      else
        hipLaunchKernelGGL((apply_update_kernel<1, true>), dim3(blocks), dim3(256), 0, stream, tin, tout, vv, sh, n4, u.c, t, u.momentum, u.decay);
    } else {
      if (u.c >= 6)
        hipLaunchKernelGGL((apply_update_kernel<6, false>), dim3(blocks), dim3(256), 0, stream, tin, tout, vv, sh, n4, u.c, t, u.momentum, u.decay);
      else
        hipLaunchKernelGGL((apply_update_kernel<1, false>), dim3(blocks), dim3(256), 0, stream, tin, tout, vv, sh, n4, u.c, t, u.momentum, u.decay);
    }
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
