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
//
// Long windows (c >= kTwoPassMinC) take the same arithmetic in two launches per stretch of kSumStretch parameters:
// sum_gradients_kernel writes s for the stretch to a small buffer, apply_update_kernel then runs on the stretch with
// that buffer as its one "gradient" of coefficient 1 (fma(1, s, 0) = s: the result is bit-identical).  A pass that
// only reads streams c gradients at the rate of a pure read (7.07 TB/s measured); in the single pass the two written
// streams are interleaved with the 54 read ones all the time and the whole runs at copy speed (5.7 TB/s).  The
// buffer is 8 MiB and is read back right after it was written (it passes the L2s' memory interface both ways, 8 bytes
// per parameter of counted traffic, and fits the memory-side cache many times over).  P = 60 M, c = 54:
// 2.43 -> 2.15 ms; the two forms cross at c of about 24.
#include "ctx.hpp"
#include "dev_common.hpp"

#include <string.h>

#include <algorithm>
#include <mutex>

namespace sasgd {

// Buffer of partial sums for callers that may not allocate (sasgd_applyUpdateNoAlloc): one stretch of the two-pass
// form, 8 MiB per device, held from the library's load until the process ends.  Host code never passes this name to a
// kernel: it is a host-side stand-in, the device address comes from hipGetSymbolAddress (static_sum_buffer below).
static __device__ __align__(256) float scratch[kSumStretch];

constexpr int kMaxDevices = 64;
static float* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

hipError_t static_sum_buffer(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // this device's copy of the array (the current device's)
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

struct GradTable {
  const float* g[kMaxLearners];
  float coef[kMaxLearners];
};

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
// reverse: workgroups take the pieces from the far end first.  A server that applies updates back to back
// alternates the direction, so each pass starts on the theta and v lines the previous pass touched last, which
// the 256 MB last-level cache still holds (P = 60 M, c = 1: 204 -> 175 us per update).  NT bit 0 / bit 1: theta
// and v are read / written with non-temporal hints, which lose that reuse (gradients always are: nobody reads
// them again).
// GPLAIN: the gradients are read with ordinary loads (the second pass of a long window reads the sums just written).
template <int ILP, int U, bool EARLY, bool SHADOW, int NT, bool GPLAIN = false>
__global__ __launch_bounds__(256) void apply_update_kernel(const float4* theta_in, float4* theta_out, float4* v,
                                                           uint2* __restrict__ shadow, int64_t n4, int c,
                                                           GradTable t, float m, float decay, int reverse) {
  const int64_t blk = reverse ? gridDim.x - 1 - blockIdx.x : blockIdx.x;
  const int64_t base = blk * (256 * ILP) + threadIdx.x;
  float4 s[ILP], th[ILP], vv[ILP];
#pragma unroll
  for (int e = 0; e < ILP; e++) s[e] = make_float4(0.f, 0.f, 0.f, 0.f);
  if (EARLY) {
#pragma unroll
    for (int e = 0; e < ILP; e++) {
      const int64_t i = base + e * 256;
      if (i < n4) { if (NT & 1) { th[e] = ldg_nt(theta_in + i); vv[e] = ldg_nt(v + i); } else { th[e] = theta_in[i]; vv[e] = v[i]; } }
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
        if (i < n4) g[u][e] = GPLAIN ? reinterpret_cast<const float4*>(t.g[l + u])[i] : ldg_nt(reinterpret_cast<const float4*>(t.g[l + u]) + i);
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
      if (!EARLY) { if (NT & 1) { th[e] = ldg_nt(theta_in + i); vv[e] = ldg_nt(v + i); } else { th[e] = theta_in[i]; vv[e] = v[i]; } }
      float4 a = th[e], b = vv[e];
      b.x = fmaf(m, b.x, s[e].x) + decay * a.x;
      b.y = fmaf(m, b.y, s[e].y) + decay * a.y;
      b.z = fmaf(m, b.z, s[e].z) + decay * a.z;
      b.w = fmaf(m, b.w, s[e].w) + decay * a.w;
      a.x -= b.x;
      a.y -= b.y;
      a.z -= b.z;
      a.w -= b.w;
      if (NT & 2) { stg_nt(v + i, b); stg_nt(theta_out + i, a); } else { v[i] = b; theta_out[i] = a; }
      if (SHADOW) {
        uint2 o;
        o.x = (uint32_t)f2bf(a.x) | ((uint32_t)f2bf(a.y) << 16);
        o.y = (uint32_t)f2bf(a.z) | ((uint32_t)f2bf(a.w) << 16);
        shadow[i] = o;
      }
    }
  }
}

// First pass of a long window: s = sum_l coef_l g_l for one stretch, the FMA chain of apply_update_kernel, written
// with ordinary stores.
template <int ILP, int U>
__global__ __launch_bounds__(256) void sum_gradients_kernel(float4* __restrict__ out, int64_t n4, int c, GradTable t) {
  const int64_t base = (int64_t)blockIdx.x * (256 * ILP) + threadIdx.x;
  float4 s[ILP];
#pragma unroll
  for (int e = 0; e < ILP; e++) s[e] = make_float4(0.f, 0.f, 0.f, 0.f);
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
    if (i < n4) out[i] = s[e];
  }
}

// Fused steps over a flat stretch (see StepTable): per element the operations of apply_update_kernel, step after step.
template <int ILP>
__global__ __launch_bounds__(256) void apply_updates_fused_kernel(const float4* theta_in, float4* theta_final, float4* v, int64_t n4,
                                                                  GradTable t, StepTable st, float m) {
  const int64_t base = (int64_t)blockIdx.x * (256 * ILP) + threadIdx.x;
  float4 th[ILP], vv[ILP];
#pragma unroll
  for (int e = 0; e < ILP; e++) {
    const int64_t i = base + e * 256;
    if (i < n4) { th[e] = ldg_nt(theta_in + i); vv[e] = ldg_nt(v + i); }
  }
  for (int step = 0; step < st.steps; step++) {
    float4 s[ILP];
#pragma unroll
    for (int e = 0; e < ILP; e++) s[e] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int l = st.first[step]; l < st.first[step + 1]; l++) {   // arrival order
      const float cf = t.coef[l];
      float4 g[ILP];
#pragma unroll
      for (int e = 0; e < ILP; e++) {
        const int64_t i = base + e * 256;
        if (i < n4) g[e] = ldg_nt(reinterpret_cast<const float4*>(t.g[l]) + i);
      }
#pragma unroll
      for (int e = 0; e < ILP; e++) {
        s[e].x = fmaf(cf, g[e].x, s[e].x);
        s[e].y = fmaf(cf, g[e].y, s[e].y);
        s[e].z = fmaf(cf, g[e].z, s[e].z);
        s[e].w = fmaf(cf, g[e].w, s[e].w);
      }
    }
    const float decay = st.decay[step];
    float4* tout = reinterpret_cast<float4*>(st.theta_out[step]);
    uint2* shadow = reinterpret_cast<uint2*>(st.shadow_out[step]);
#pragma unroll
    for (int e = 0; e < ILP; e++) {
      const int64_t i = base + e * 256;
      if (i < n4) {
        float4 a = th[e], b = vv[e];
        b.x = fmaf(m, b.x, s[e].x) + decay * a.x;
        b.y = fmaf(m, b.y, s[e].y) + decay * a.y;
        b.z = fmaf(m, b.z, s[e].z) + decay * a.z;
        b.w = fmaf(m, b.w, s[e].w) + decay * a.w;
        a.x -= b.x;
        a.y -= b.y;
        a.z -= b.z;
        a.w -= b.w;
        th[e] = a;
        vv[e] = b;
        if (tout) stg_nt(tout + i, a);
        if (shadow) {
          uint2 o;
          o.x = (uint32_t)f2bf(a.x) | ((uint32_t)f2bf(a.y) << 16);
          o.y = (uint32_t)f2bf(a.z) | ((uint32_t)f2bf(a.w) << 16);
          shadow[i] = o;
        }
      }
    }
  }
#pragma unroll
  for (int e = 0; e < ILP; e++) {
    const int64_t i = base + e * 256;
    if (i < n4) {
      stg_nt(v + i, vv[e]);
      if (theta_final) stg_nt(theta_final + i, th[e]);
    }
  }
}

// Scalar tail of the fused steps (P not a multiple of 4): at most 3 elements.
__global__ void apply_updates_fused_tail_kernel(const float* theta_in, float* theta_final, float* v, int64_t begin, int64_t P, GradTable t,
                                                StepTable st, float m) {
  const int64_t i = begin + threadIdx.x;
  if (i >= P) return;
  float th = theta_in[i], vv = v[i];
  for (int step = 0; step < st.steps; step++) {
    float s = 0.f;
    for (int l = st.first[step]; l < st.first[step + 1]; l++) s = fmaf(t.coef[l], t.g[l][i], s);
    vv = fmaf(m, vv, s) + st.decay[step] * th;
    th = th - vv;
    if (st.theta_out[step]) st.theta_out[step][i] = th;
    if (st.shadow_out[step]) st.shadow_out[step][i] = f2bf(th);
  }
  v[i] = vv;
  if (theta_final) theta_final[i] = th;
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
  if (shadow) shadow[i] = f2bf(th);
}

template <int ILP, int U, bool EARLY, int NT>
static void launch_shape_nt(const UpdateLaunch& u, const GradTable& t, int64_t n4, hipStream_t stream) {
  const int blocks = (int)((n4 + 256 * ILP - 1) / (256 * ILP));
  const float4* tin = reinterpret_cast<const float4*>(u.theta_in);
  float4* tout = reinterpret_cast<float4*>(u.theta_out);
  float4* vv = reinterpret_cast<float4*>(u.v);
  uint2* sh = reinterpret_cast<uint2*>(u.shadow_out);
  if (u.shadow_out)
    hipLaunchKernelGGL((apply_update_kernel<ILP, U, EARLY, true, NT>), dim3(blocks), dim3(256), 0, stream, tin, tout, vv, sh, n4, u.c, t, u.momentum, u.decay, u.reverse);
  else
    hipLaunchKernelGGL((apply_update_kernel<ILP, U, EARLY, false, NT>), dim3(blocks), dim3(256), 0, stream, tin, tout, vv, sh, n4, u.c, t, u.momentum, u.decay, u.reverse);
}
// theta and v take ordinary loads and stores for windows of up to kKeepMaxC gradients, so that the next update
// finds their tail in the last-level cache; behind longer gradient sweeps nothing of them survives and the
// streaming hints are the faster choice (P = 60 M, c = 54, after other updates: 2.45 against 2.61 ms in one pass).
constexpr int kKeepMaxC = kTwoPassMinC - 1;
template <int ILP, int U, bool EARLY>
static void launch_shape(const UpdateLaunch& u, const GradTable& t, int64_t n4, hipStream_t stream) {
  if (u.c <= kKeepMaxC) launch_shape_nt<ILP, U, EARLY, 0>(u, t, n4, stream);
  else launch_shape_nt<ILP, U, EARLY, 3>(u, t, n4, stream);
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
  if (u.P >= kSumStretch && u.c >= kTwoPassMinC && u.sum_buf) {   // shorter vectors: one launch, nothing to separate
    // stretches of 512 workgroups (two per compute unit; 256-1024 measured within 4 %, other counts slower)
    constexpr int64_t stretch4 = kSumStretch / 4;
    float4* sums = reinterpret_cast<float4*>(u.sum_buf);
    GradTable tb;
    for (int l = 0; l < kMaxLearners; l++) { tb.g[l] = nullptr; tb.coef[l] = 0.f; }
    tb.g[0] = u.sum_buf;
    tb.coef[0] = 1.0f;
    for (int64_t off = 0; off < n4; off += stretch4) {
      const int64_t len = std::min(stretch4, n4 - off);
      const int blocks = (int)((len + 256 * 4 - 1) / (256 * 4));
      GradTable ta = t;
      for (int l = 0; l < u.c; l++) ta.g[l] = t.g[l] + off * 4;
      hipLaunchKernelGGL((sum_gradients_kernel<4, 3>), dim3(blocks), dim3(256), 0, stream, sums, len, u.c, ta);
      const float4* tin = reinterpret_cast<const float4*>(u.theta_in) + off;
      float4* tout = reinterpret_cast<float4*>(u.theta_out) + off;
      float4* vv = reinterpret_cast<float4*>(u.v) + off;
      uint2* sh = u.shadow_out ? reinterpret_cast<uint2*>(u.shadow_out) + off : nullptr;
      if (sh)
        hipLaunchKernelGGL((apply_update_kernel<4, 1, true, true, 3, true>), dim3(blocks), dim3(256), 0, stream, tin, tout, vv, sh, len, 1, tb, u.momentum, u.decay, 0);
      else
        hipLaunchKernelGGL((apply_update_kernel<4, 1, true, false, 3, true>), dim3(blocks), dim3(256), 0, stream, tin, tout, vv, sh, len, 1, tb, u.momentum, u.decay, 0);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  } else if (n4 > 0) {
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

hipError_t launch_apply_updates_fused(const UpdateLaunch& u, const StepTable& st, float* final_theta, hipStream_t stream) {
  if (u.P <= 0) return hipSuccess;
  if (st.steps < 1 || st.steps > kMaxFusedSteps || st.first[0] != 0 || st.first[st.steps] != u.c || u.c > kMaxLearners) return hipErrorInvalidValue;
  if (u.P / 4 > (int64_t)0x7fffffff * 256) return hipErrorInvalidValue;
  GradTable t;
  for (int l = 0; l < kMaxLearners; l++) {
    t.g[l] = l < u.c ? u.grads[l] : nullptr;
    t.coef[l] = l < u.c ? u.coef[l] : 0.f;
  }
  const int64_t n4 = u.P / 4;
  if (n4 > 0) {
    const int blocks = (int)((n4 + 256 * 4 - 1) / (256 * 4));
    hipLaunchKernelGGL((apply_updates_fused_kernel<4>), dim3(blocks), dim3(256), 0, stream, reinterpret_cast<const float4*>(u.theta_in),
                       reinterpret_cast<float4*>(final_theta), reinterpret_cast<float4*>(u.v), n4, t, st, u.momentum);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (n4 * 4 < u.P) {
    hipLaunchKernelGGL(apply_updates_fused_tail_kernel, dim3(1), dim3(64), 0, stream, u.theta_in, final_theta, u.v, n4 * 4, u.P, t, st, u.momentum);
    return hipGetLastError();
  }
  return hipSuccess;
}

// ------------------------------------------------------------------ update of a fully connected layer from factors
// For a fully connected layer with a mini-batch of N images the weight gradient is dW[o][i] = sum_n dy[n][o] x[n][i].
// A learner keeps x [N][in] and dy transposed [out][NP] (bf16) instead of writing dW; this kernel forms the product
// while it streams theta and v: per gradient  p = sum_n dy x  (fp32 FMA in image order, the arithmetic of the
// written-out gradient),  s += coef * p,  then the same update as apply_update_kernel.  HBM traffic per weight drops
// by the 4 bytes of gradient; the N FMAs per weight are far below what the streaming rate leaves room for.
// Gradients without factors (pushed from outside) are read as written-out vectors.  The layer's bias follows its
// weights in the flat vector and is updated by one extra row of workgroups from the written-out bias gradients.
struct FcFactors {
  const bf16_t* x[kMaxLearners];     // [N][in] or nullptr: gradient l is a written-out vector
  const bf16_t* dyT[kMaxLearners];   // [out][NP]
};

constexpr int kFcRows = 4;           // output units per workgroup (2, 8 and 16 measured slower at config 4)

// Steps: see StepTable (one step = the plain update; st.theta_out is not used here, the weights are written once).
template <bool SHADOW>
__global__ __launch_bounds__(256) void apply_update_fc_kernel(const float* theta_in, float* theta_out, float* v, int in, int out, int N,
                                                              int NP, GradTable t, FcFactors f, StepTable st, float m) {
  const int nrb = (out + kFcRows - 1) / kFcRows;
  const int col = (blockIdx.x * 256 + threadIdx.x) * 4;
  if ((int)blockIdx.y == nrb) {       // bias: elements out * in + col .. col + 3
    if (col >= out) return;
    const int64_t e = (int64_t)out * in + col;
    float4 a = *reinterpret_cast<const float4*>(theta_in + e), b = *reinterpret_cast<const float4*>(v + e);
    for (int step = 0; step < st.steps; step++) {
      float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
      for (int l = st.first[step]; l < st.first[step + 1]; l++) {
        const float4 g = *reinterpret_cast<const float4*>(t.g[l] + e);
        s.x = fmaf(t.coef[l], g.x, s.x); s.y = fmaf(t.coef[l], g.y, s.y);
        s.z = fmaf(t.coef[l], g.z, s.z); s.w = fmaf(t.coef[l], g.w, s.w);
      }
      const float decay = st.decay[step];
      b.x = fmaf(m, b.x, s.x) + decay * a.x; b.y = fmaf(m, b.y, s.y) + decay * a.y;
      b.z = fmaf(m, b.z, s.z) + decay * a.z; b.w = fmaf(m, b.w, s.w) + decay * a.w;
      a.x -= b.x; a.y -= b.y; a.z -= b.z; a.w -= b.w;
      if (SHADOW) {
        uint2 o;
        o.x = (uint32_t)f2bf(a.x) | ((uint32_t)f2bf(a.y) << 16);
        o.y = (uint32_t)f2bf(a.z) | ((uint32_t)f2bf(a.w) << 16);
        *reinterpret_cast<uint2*>(st.shadow_out[step] + e) = o;
      }
    }
    *reinterpret_cast<float4*>(v + e) = b;
    *reinterpret_cast<float4*>(theta_out + e) = a;
    return;
  }
  if (col >= in) return;
  const int o0 = blockIdx.y * kFcRows;
  float4 th[kFcRows], vv[kFcRows];
#pragma unroll
  for (int r = 0; r < kFcRows; r++) {
    if (o0 + r < out) {
      const int64_t e = (int64_t)(o0 + r) * in + col;
      th[r] = ldg_nt(reinterpret_cast<const float4*>(theta_in + e));
      vv[r] = ldg_nt(reinterpret_cast<const float4*>(v + e));
    }
  }
  for (int step = 0; step < st.steps; step++) {
    float4 s[kFcRows];
#pragma unroll
    for (int r = 0; r < kFcRows; r++) s[r] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int l = st.first[step]; l < st.first[step + 1]; l++) {
      const float cf = t.coef[l];
      if (f.x[l]) {
        float4 p[kFcRows];
#pragma unroll
        for (int r = 0; r < kFcRows; r++) p[r] = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int n0 = 0; n0 < NP; n0 += 8) {
          uint2 xr[8];
#pragma unroll
          for (int k = 0; k < 8; k++)
            xr[k] = n0 + k < N ? *reinterpret_cast<const uint2*>(f.x[l] + (int64_t)(n0 + k) * in + col) : make_uint2(0u, 0u);
#pragma unroll
          for (int r = 0; r < kFcRows; r++) {
            const int o = min(o0 + r, out - 1);           // rows beyond the layer compute a value nobody stores
            const uint4 d8 = *reinterpret_cast<const uint4*>(f.dyT[l] + (int64_t)o * NP + n0);   // same address for the whole workgroup
            const uint32_t dw[4] = {d8.x, d8.y, d8.z, d8.w};
#pragma unroll
            for (int k = 0; k < 8; k++) {
              const float d = __uint_as_float((k & 1) ? (dw[k >> 1] & 0xffff0000u) : (dw[k >> 1] << 16));
              p[r].x = fmaf(d, __uint_as_float(xr[k].x << 16), p[r].x);
              p[r].y = fmaf(d, __uint_as_float(xr[k].x & 0xffff0000u), p[r].y);
              p[r].z = fmaf(d, __uint_as_float(xr[k].y << 16), p[r].z);
              p[r].w = fmaf(d, __uint_as_float(xr[k].y & 0xffff0000u), p[r].w);
            }
          }
        }
#pragma unroll
        for (int r = 0; r < kFcRows; r++) {
          s[r].x = fmaf(cf, p[r].x, s[r].x); s[r].y = fmaf(cf, p[r].y, s[r].y);
          s[r].z = fmaf(cf, p[r].z, s[r].z); s[r].w = fmaf(cf, p[r].w, s[r].w);
        }
      } else {
#pragma unroll
        for (int r = 0; r < kFcRows; r++) {
          if (o0 + r < out) {
            const float4 g = ldg_nt(reinterpret_cast<const float4*>(t.g[l] + (int64_t)(o0 + r) * in + col));
            s[r].x = fmaf(cf, g.x, s[r].x); s[r].y = fmaf(cf, g.y, s[r].y);
            s[r].z = fmaf(cf, g.z, s[r].z); s[r].w = fmaf(cf, g.w, s[r].w);
          }
        }
      }
    }
    const float decay = st.decay[step];
#pragma unroll
    for (int r = 0; r < kFcRows; r++) {
      if (o0 + r >= out) continue;
      float4 a = th[r], b = vv[r];
      b.x = fmaf(m, b.x, s[r].x) + decay * a.x; b.y = fmaf(m, b.y, s[r].y) + decay * a.y;
      b.z = fmaf(m, b.z, s[r].z) + decay * a.z; b.w = fmaf(m, b.w, s[r].w) + decay * a.w;
      a.x -= b.x; a.y -= b.y; a.z -= b.z; a.w -= b.w;
      th[r] = a;
      vv[r] = b;
      if (SHADOW) {
        uint2 o;
        o.x = (uint32_t)f2bf(a.x) | ((uint32_t)f2bf(a.y) << 16);
        o.y = (uint32_t)f2bf(a.z) | ((uint32_t)f2bf(a.w) << 16);
        *reinterpret_cast<uint2*>(st.shadow_out[step] + (int64_t)(o0 + r) * in + col) = o;
      }
    }
  }
#pragma unroll
  for (int r = 0; r < kFcRows; r++) {
    if (o0 + r >= out) continue;
    const int64_t e = (int64_t)(o0 + r) * in + col;
    stg_nt(reinterpret_cast<float4*>(v + e), vv[r]);
    stg_nt(reinterpret_cast<float4*>(theta_out + e), th[r]);
  }
}

hipError_t launch_apply_update_fc(const FcUpdateLaunch& u, hipStream_t stream, const StepTable* steps) {
  if (u.in < 4 || u.out < 4 || (u.in & 3) || (u.out & 3) || u.c < 1 || u.c > kMaxLearners) return hipErrorInvalidValue;
  GradTable t;
  FcFactors f;
  for (int l = 0; l < kMaxLearners; l++) {
    t.g[l] = l < u.c ? u.grads[l] : nullptr;
    t.coef[l] = l < u.c ? u.coef[l] : 0.f;
    f.x[l] = l < u.c ? u.fx[l] : nullptr;
    f.dyT[l] = l < u.c ? u.fdyT[l] : nullptr;
  }
  StepTable st;
  if (steps) {
    st = *steps;
    if (st.steps < 1 || st.steps > kMaxFusedSteps || st.first[0] != 0 || st.first[st.steps] != u.c) return hipErrorInvalidValue;
  } else {
    memset(&st, 0, sizeof(st));
    st.steps = 1;
    st.first[1] = u.c;
    st.decay[0] = u.decay;
    st.shadow_out[0] = u.shadow_out;
  }
  bool shadow = st.shadow_out[0] != nullptr;
  for (int k = 0; k < st.steps; k++)
    if ((st.shadow_out[k] != nullptr) != shadow) return hipErrorInvalidValue;
  const int widest = u.in > u.out ? u.in : u.out;
  dim3 grid((unsigned)((widest + 1023) / 1024), (unsigned)((u.out + kFcRows - 1) / kFcRows + 1));
  if (shadow)
    hipLaunchKernelGGL((apply_update_fc_kernel<true>), grid, dim3(256), 0, stream, u.theta_in, u.theta_out, u.v, u.in, u.out, u.N, u.NP, t, f,
                       st, u.momentum);
  else
    hipLaunchKernelGGL((apply_update_fc_kernel<false>), grid, dim3(256), 0, stream, u.theta_in, u.theta_out, u.v, u.in, u.out, u.N, u.NP, t, f,
                       st, u.momentum);
  return hipGetLastError();
}

__global__ void fp32_to_bf16_kernel(const float* __restrict__ src, bf16_t* __restrict__ dst, int64_t n) {
  int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = f2bf(src[i]);
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
