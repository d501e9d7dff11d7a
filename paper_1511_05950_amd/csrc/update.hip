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
// For a fully connected layer with a mini-batch of N images the weight gradient is the rank-N product
// dW[o][i] = sum_n dy[n][o] x[n][i].  A learner keeps the two factors transposed, dyT [out][NP] and xT [in][NP] (bf16, NP = N
// rounded up to 8, zero-filled), instead of writing dW, and this kernel forms the product while it streams theta and v:
// one bf16 MFMA (32 x 32 x 16, fp32 accumulation) yields the gradient of a 32 x 32 block of weights from two 1 KiB operand
// reads -- both factors are k-contiguous, so the fragments come straight from memory.  HBM traffic per weight drops by the
// 4 bytes of gradient, and with several steps fused theta and v pass through once for all of them.
// A wavefront owns 32 output units x 32 input units.  theta, v and the running sums live in registers in row-major order
// (8 lanes x 16 bytes cover the 128 contiguous bytes of a row); a product leaves the matrix cores in MFMA order and is
// turned around through the wavefront's own piece of LDS.  Gradients without factors (pushed from outside) are read as
// written-out vectors, in the same order.  Per element: p_l = product (or the written-out value), s = sum_l coef_l p_l in
// arrival order, then the update of apply_update_kernel.  The layer's bias follows its weights in the flat vector and is
// updated by one extra row of workgroups from the written-out bias gradients.
struct FcFactors {
  const bf16_t* base[kMaxLearners];  // the pending gradient's factors, or nullptr: gradient l is a written-out vector
};
// The layers of one launch: workgroups tile0[k] .. tile0[k + 1] - 1 belong to layer k, cols[k] of them per block of 32
// output units (plus one such row for the bias).
struct FcLayerTab {
  int count;
  int in[kMaxFactoredLayers], out[kMaxFactoredLayers], cols[kMaxFactoredLayers];
  int tile0[kMaxFactoredLayers + 1];
  int64_t w_off[kMaxFactoredLayers];
  int64_t fx_off[kMaxFactoredLayers], fdy_off[kMaxFactoredLayers];
};

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16_t;

constexpr int kFcTileRows = 32, kFcTileCols = 32;     // per wavefront
constexpr int kFcCB = kFcTileCols / 32;               // MFMA column blocks per wavefront
constexpr int kFcLPR = kFcTileCols / 4;               // lanes per tile row in row-major order (16 bytes each)
constexpr int kFcRPI = 64 / kFcLPR;                   // tile rows one 64-lane access covers
constexpr int kFcNQ = kFcTileRows / kFcRPI;           // 16-byte pieces per lane and array
constexpr int kFcLds = kFcTileCols + 4;               // LDS row stride in floats

template <bool SHADOW>
__global__ __launch_bounds__(256) void apply_update_fc_kernel(const float* theta_in, float* theta_out, float* v, int NP, GradTable t,
                                                              FcFactors f, FcLayerTab lt, StepTable st, float m) {
  __shared__ __attribute__((aligned(16))) float lds[4 * kFcTileRows * kFcLds];
  int layer = 0;
  for (int k = 1; k < lt.count; k++) layer = (int)blockIdx.x >= lt.tile0[k] ? k : layer;
  const int local = (int)blockIdx.x - lt.tile0[layer];
  const int bx = local % lt.cols[layer], by = local / lt.cols[layer];
  const int in = lt.in[layer], out = lt.out[layer];
  const int64_t woff = lt.w_off[layer];
  theta_in += woff; theta_out += woff; v += woff;
  const int nrb = (out + kFcTileRows - 1) / kFcTileRows;
  if (by == nrb) {       // bias: elements out * in + col .. col + 3
    const int col = (bx * 256 + threadIdx.x) * 4;
    if (col >= out) return;
    const int64_t e = (int64_t)out * in + col;
    float4 a = *reinterpret_cast<const float4*>(theta_in + e), b = *reinterpret_cast<const float4*>(v + e);
    for (int step = 0; step < st.steps; step++) {
      float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
      for (int l = st.first[step]; l < st.first[step + 1]; l++) {
        const float4 g = *reinterpret_cast<const float4*>(t.g[l] + woff + e);
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
        *reinterpret_cast<uint2*>(st.shadow_out[step] + woff + e) = o;
      }
    }
    *reinterpret_cast<float4*>(v + e) = b;
    *reinterpret_cast<float4*>(theta_out + e) = a;
    return;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int o0 = by * kFcTileRows;
  const int w0 = (bx * 4 + wave) * kFcTileCols;
  if (w0 >= in) return;               // whole wavefronts leave: no workgroup barrier below
  float* tile = lds + wave * (kFcTileRows * kFcLds);
  // row-major registers: piece q is row kFcRPI q + lane / kFcLPR, columns 4 (lane % kFcLPR) .. + 3 of the tile
  const int rr = lane / kFcLPR, cc = (lane % kFcLPR) * 4;
  const bool col_ok = w0 + cc < in;   // in is a multiple of 4
  float4 th[kFcNQ], vv[kFcNQ];
#pragma unroll
  for (int q = 0; q < kFcNQ; q++) {
    const int o = o0 + kFcRPI * q + rr;
    if (o < out && col_ok) {
      const int64_t e = (int64_t)o * in + w0 + cc;
      th[q] = ldg_nt(reinterpret_cast<const float4*>(theta_in + e));
      vv[q] = ldg_nt(reinterpret_cast<const float4*>(v + e));
    }
  }
  // MFMA operands: lane (j = lane % 32, h = lane / 32) holds k = 8 h .. 8 h + 7 of row / column j
  const int j = lane & 31, h = lane >> 5;
  const int KB = (NP + 15) >> 4;
  for (int step = 0; step < st.steps; step++) {
    float4 s[kFcNQ];
#pragma unroll
    for (int q = 0; q < kFcNQ; q++) s[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int l = st.first[step]; l < st.first[step + 1]; l++) {
      const float cf = t.coef[l];
      if (f.base[l]) {
        const bf16_t* xT = f.base[l] + lt.fx_off[layer];
        const bf16_t* dyT = f.base[l] + lt.fdy_off[layer];
        floatx16_t p[kFcCB];
#pragma unroll
        for (int b = 0; b < kFcCB; b++)
#pragma unroll
          for (int r = 0; r < 16; r++) p[b][r] = 0.f;
        for (int kb = 0; kb < KB; kb++) {
          const int n0 = 16 * kb + 8 * h;
          union { uint4 u; bf16x8_t x; } fa, fb[kFcCB];
          fa.u = make_uint4(0u, 0u, 0u, 0u);
          if (n0 < NP && o0 + j < out) fa.u = *reinterpret_cast<const uint4*>(dyT + (int64_t)(o0 + j) * NP + n0);
#pragma unroll
          for (int b = 0; b < kFcCB; b++) {
            fb[b].u = make_uint4(0u, 0u, 0u, 0u);
            if (n0 < NP && w0 + 32 * b + j < in) fb[b].u = *reinterpret_cast<const uint4*>(xT + (int64_t)(w0 + 32 * b + j) * NP + n0);
          }
#pragma unroll
          for (int b = 0; b < kFcCB; b++) p[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.x, fb[b].x, p[b], 0, 0, 0);
        }
        // MFMA order (column 32 b + j, rows 8 (r / 4) + 4 h + r % 4) -> row-major, through this wavefront's LDS piece
#pragma unroll
        for (int b = 0; b < kFcCB; b++)
#pragma unroll
          for (int r = 0; r < 16; r++) tile[(8 * (r >> 2) + 4 * h + (r & 3)) * kFcLds + 32 * b + j] = p[b][r];
        __builtin_amdgcn_wave_barrier();
        asm volatile("" ::: "memory");
#pragma unroll
        for (int q = 0; q < kFcNQ; q++) {
          const float4 g = *reinterpret_cast<const float4*>(tile + (kFcRPI * q + rr) * kFcLds + cc);
          s[q].x = fmaf(cf, g.x, s[q].x); s[q].y = fmaf(cf, g.y, s[q].y);
          s[q].z = fmaf(cf, g.z, s[q].z); s[q].w = fmaf(cf, g.w, s[q].w);
        }
        __builtin_amdgcn_wave_barrier();
        asm volatile("" ::: "memory");
      } else {
#pragma unroll
        for (int q = 0; q < kFcNQ; q++) {
          const int o = o0 + kFcRPI * q + rr;
          if (o < out && col_ok) {
            const float4 g = ldg_nt(reinterpret_cast<const float4*>(t.g[l] + woff + (int64_t)o * in + w0 + cc));
            s[q].x = fmaf(cf, g.x, s[q].x); s[q].y = fmaf(cf, g.y, s[q].y);
            s[q].z = fmaf(cf, g.z, s[q].z); s[q].w = fmaf(cf, g.w, s[q].w);
          }
        }
      }
    }
    const float decay = st.decay[step];
#pragma unroll
    for (int q = 0; q < kFcNQ; q++) {
      const int o = o0 + kFcRPI * q + rr;
      if (o >= out || !col_ok) continue;
      float4 a = th[q], b = vv[q];
      b.x = fmaf(m, b.x, s[q].x) + decay * a.x; b.y = fmaf(m, b.y, s[q].y) + decay * a.y;
      b.z = fmaf(m, b.z, s[q].z) + decay * a.z; b.w = fmaf(m, b.w, s[q].w) + decay * a.w;
      a.x -= b.x; a.y -= b.y; a.z -= b.z; a.w -= b.w;
      th[q] = a;
      vv[q] = b;
      if (SHADOW) {
        uint2 w2;
        w2.x = (uint32_t)f2bf(a.x) | ((uint32_t)f2bf(a.y) << 16);
        w2.y = (uint32_t)f2bf(a.z) | ((uint32_t)f2bf(a.w) << 16);
        *reinterpret_cast<uint2*>(st.shadow_out[step] + woff + (int64_t)o * in + w0 + cc) = w2;
      }
    }
  }
#pragma unroll
  for (int q = 0; q < kFcNQ; q++) {
    const int o = o0 + kFcRPI * q + rr;
    if (o >= out || !col_ok) continue;
    const int64_t e = (int64_t)o * in + w0 + cc;
    stg_nt(reinterpret_cast<float4*>(v + e), vv[q]);
    stg_nt(reinterpret_cast<float4*>(theta_out + e), th[q]);
  }
}

hipError_t launch_apply_update_fc(const FcUpdateLaunch& u, hipStream_t stream, const StepTable* steps) {
  if (u.layers < 1 || u.layers > kMaxFactoredLayers || u.c < 1 || u.c > kMaxLearners) return hipErrorInvalidValue;
  if (u.NP < 8 || u.NP > 32 || (u.NP & 7)) return hipErrorInvalidValue;
  GradTable t;
  FcFactors f;
  for (int l = 0; l < kMaxLearners; l++) {
    t.g[l] = l < u.c ? u.grads[l] : nullptr;
    t.coef[l] = l < u.c ? u.coef[l] : 0.f;
    f.base[l] = l < u.c ? u.factors[l] : nullptr;
  }
  FcLayerTab lt;
  memset(&lt, 0, sizeof(lt));
  lt.count = u.layers;
  int64_t tiles = 0;
  for (int k = 0; k < u.layers; k++) {
    if (u.in[k] < 4 || u.out[k] < 4 || (u.in[k] & 3) || (u.out[k] & 3)) return hipErrorInvalidValue;
    lt.in[k] = u.in[k];
    lt.out[k] = u.out[k];
    lt.w_off[k] = u.w_off[k];
    lt.fx_off[k] = (int64_t)u.fx_off[k];
    lt.fdy_off[k] = (int64_t)u.fdy_off[k];
    // 4 kFcTileCols input units per workgroup (four wavefronts side by side), or 1024 bias elements in the extra row
    lt.cols[k] = std::max((u.in[k] + 4 * kFcTileCols - 1) / (4 * kFcTileCols), (u.out[k] + 1023) / 1024);
    lt.tile0[k] = (int)tiles;
    tiles += (int64_t)lt.cols[k] * ((u.out[k] + kFcTileRows - 1) / kFcTileRows + 1);
    if (tiles > 0x7fffffff) return hipErrorInvalidValue;
  }
  lt.tile0[u.layers] = (int)tiles;
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
  const dim3 grid((unsigned)tiles);
  if (shadow)
    hipLaunchKernelGGL((apply_update_fc_kernel<true>), grid, dim3(256), 0, stream, u.theta_in, u.theta_out, u.v, u.NP, t, f, lt, st, u.momentum);
  else
    hipLaunchKernelGGL((apply_update_fc_kernel<false>), grid, dim3(256), 0, stream, u.theta_in, u.theta_out, u.v, u.NP, t, f, lt, st, u.momentum);
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
