// Direct (non-MFMA) convolution / fully-connected kernels: forward, input gradient, weight and bias
// gradient.  Used for fp32 compute, where the products must be exact fp32, and as the general fallback
// for shapes the MFMA kernels do not take.  A fully connected layer is the 1x1 case on a 1x1 image.
// Accumulation is fp32 in a fixed order, so reruns are bit-identical.
//
// Layouts: x [N][H][W][C], y [N][OH][OW][K] of type T; weights in the flat parameter order
// w[K][C][ks][ks], b[K] of type T (fp32 ring or bf16 copy); dW, db fp32 in the same order.
#include "dev_common.hpp"
#include "kernels.hpp"

namespace sasgd {

// ------------------------------------------------------------------ forward
// One lane per output element (image, oh, ow, k), k innermost: the lanes of a wavefront share the input
// pixel (broadcast load) and read weights of consecutive output channels.
template <typename T>
__global__ __launch_bounds__(256) void conv_fwd_simple_kernel(PtrTab ws, CPtrTab wts, size_t x_off, size_t y_off, int64_t w_off,
                                                              int64_t b_off, ConvShape sh, int relu, int out_f32) {
  const T* x = (const T*)ws.p[blockIdx.z] + x_off;
  T* y = (T*)ws.p[blockIdx.z] + y_off;
  const T* w = (const T*)wts.p[blockIdx.z] + w_off;
  const T* b = (const T*)wts.p[blockIdx.z] + b_off;
  const int64_t total = (int64_t)sh.N * sh.OH * sh.OW * sh.K;
  const int kk = sh.ks * sh.ks;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    int k = (int)(i % sh.K);
    int64_t r = i / sh.K;
    int ow = (int)(r % sh.OW);
    r /= sh.OW;
    int oh = (int)(r % sh.OH);
    int n = (int)(r / sh.OH);
    float acc = ldf(b + k);
    const T* wk = w + (int64_t)k * sh.C * kk;
    for (int kh = 0; kh < sh.ks; kh++) {
      int ih = oh * sh.stride + kh - sh.pad;
      if (ih < 0 || ih >= sh.H) continue;
      for (int kw = 0; kw < sh.ks; kw++) {
        int iw = ow * sh.stride + kw - sh.pad;
        if (iw < 0 || iw >= sh.W) continue;
        const T* xp = x + (((int64_t)n * sh.H + ih) * sh.W + iw) * sh.C;
        const T* wp = wk + kh * sh.ks + kw;
        for (int c = 0; c < sh.C; c++) acc = fmaf(ldf(xp + c), ldf(wp + (int64_t)c * kk), acc);
      }
    }
    if (relu) acc = fmaxf(acc, 0.f);
    if (out_f32) reinterpret_cast<float*>(y)[i] = acc;
    else stf(y + i, acc);
  }
}

// Fully connected forward with a long contraction: one wavefront per image and group of kFcKU output units, lanes
// stride over the inputs (both operands contiguous; x is read once for the group), butterfly sums.  Every output is
// the same chain of operations whatever the launch shape.
constexpr int kFcKU = 8;
template <typename T>
__global__ __launch_bounds__(256) void fc_fwd_wave_kernel(PtrTab ws, CPtrTab wts, size_t x_off, size_t y_off, int64_t w_off,
                                                          int64_t b_off, int N, int C, int K, int relu, int out_f32) {
  const T* x = (const T*)ws.p[blockIdx.z] + x_off;
  T* y = (T*)ws.p[blockIdx.z] + y_off;
  const T* w = (const T*)wts.p[blockIdx.z] + w_off;
  const T* b = (const T*)wts.p[blockIdx.z] + b_off;
  const int groups = (K + kFcKU - 1) / kFcKU;
  const int o = blockIdx.x * 4 + (threadIdx.x >> 6);      // (image, group of units)
  const int lane = threadIdx.x & 63;
  if (o >= N * groups) return;
  const int n = o / groups, k0 = (o - n * groups) * kFcKU;
  const T* xp = x + (int64_t)n * C;
  const T* wp[kFcKU];
#pragma unroll
  for (int u = 0; u < kFcKU; u++) wp[u] = w + (int64_t)min(k0 + u, K - 1) * C;   // units beyond K repeat the last one and are not stored
  float acc[kFcKU];
#pragma unroll
  for (int u = 0; u < kFcKU; u++) acc[u] = 0.f;
  for (int c = lane; c < C; c += 64) {
    const float xv = ldf(xp + c);
#pragma unroll
    for (int u = 0; u < kFcKU; u++) acc[u] = fmaf(xv, ldf(wp[u] + c), acc[u]);
  }
#pragma unroll
  for (int u = 0; u < kFcKU; u++) {
    const int k = k0 + u;
    float v = wave_sum(acc[u]);
    if (k >= K) continue;
    v += ldf(b + k);
    if (relu) v = fmaxf(v, 0.f);
    if (lane == 0) {
      if (out_f32) reinterpret_cast<float*>(y)[(int64_t)n * K + k] = v;
      else stf(y + (int64_t)n * K + k, v);
    }
  }
}

// Input gradient of a fully connected layer (1 x 1 window on a 1 x 1 image): dx[n][c] = sum_k dy[n][k] w[k][c], one
// thread per element, neighbouring lanes on neighbouring c; 32-bit index arithmetic.
template <typename T>
__global__ __launch_bounds__(256) void fc_dgrad_simple_kernel(PtrTab ws, CPtrTab wts, size_t dy_off, size_t dx_off, int64_t w_off, int N, int C,
                                                              int K, int use_mask, size_t mask_off) {
  const T* dy = (const T*)ws.p[blockIdx.z] + dy_off;
  T* dx = (T*)ws.p[blockIdx.z] + dx_off;
  const T* mask = (const T*)ws.p[blockIdx.z] + mask_off;
  const T* w = (const T*)wts.p[blockIdx.z] + w_off;
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (i >= (uint32_t)N * (uint32_t)C) return;
  const uint32_t n = i / (uint32_t)C, c = i - n * (uint32_t)C;
  float acc = 0.f;
  if (!use_mask || ldf(mask + i) > 0.f) {
    const T* dp = dy + (size_t)n * K;
#pragma unroll 4
    for (int k = 0; k < K; k++) acc = fmaf(ldf(dp + k), ldf(w + (size_t)k * C + c), acc);
  }
  stf(dx + i, acc);
}

// ------------------------------------------------------------------ input gradient
// dx[n][ih][iw][c] = sum_{kh,kw,k} dy[n][oh][ow][k] * w[k][c][kh][kw],  oh*stride + kh - pad = ih.
template <typename T>
__global__ __launch_bounds__(256) void conv_dgrad_simple_kernel(PtrTab ws, CPtrTab wts, size_t dy_off, size_t dx_off, int64_t w_off,
                                                                ConvShape sh, int use_mask, size_t mask_off) {
  const T* dy = (const T*)ws.p[blockIdx.z] + dy_off;
  T* dx = (T*)ws.p[blockIdx.z] + dx_off;
  const T* mask = (const T*)ws.p[blockIdx.z] + mask_off;
  const T* w = (const T*)wts.p[blockIdx.z] + w_off;
  const int64_t total = (int64_t)sh.N * sh.H * sh.W * sh.C;
  const int kk = sh.ks * sh.ks;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    int c = (int)(i % sh.C);
    int64_t r = i / sh.C;
    int iw = (int)(r % sh.W);
    r /= sh.W;
    int ih = (int)(r % sh.H);
    int n = (int)(r / sh.H);
    float acc = 0.f;
    if (!use_mask || ldf(mask + i) > 0.f) {
      for (int kh = 0; kh < sh.ks; kh++) {
        int th = ih + sh.pad - kh;
        if (th < 0 || th % sh.stride) continue;
        int oh = th / sh.stride;
        if (oh >= sh.OH) continue;
        for (int kw = 0; kw < sh.ks; kw++) {
          int tw = iw + sh.pad - kw;
          if (tw < 0 || tw % sh.stride) continue;
          int ow = tw / sh.stride;
          if (ow >= sh.OW) continue;
          const T* dp = dy + (((int64_t)n * sh.OH + oh) * sh.OW + ow) * sh.K;
          const T* wp = w + (int64_t)c * kk + kh * sh.ks + kw;
          for (int k = 0; k < sh.K; k++) acc = fmaf(ldf(dp + k), ldf(wp + (int64_t)k * sh.C * kk), acc);
        }
      }
    }
    stf(dx + i, acc);
  }
}

// ------------------------------------------------------------------ weight and bias gradient
// One wavefront per weight element (k, c, kh, kw) -- and one per bias element -- reducing over the
// N*OH*OW output positions: lanes take positions m = lane, lane+64, ..., then a butterfly sum.
template <typename T>
__global__ __launch_bounds__(256) void conv_wgrad_simple_kernel(PtrTab ws, PtrTab grads, size_t x_off, size_t dy_off, int64_t w_off,
                                                                int64_t b_off, ConvShape sh) {
  const T* x = (const T*)ws.p[blockIdx.z] + x_off;
  const T* dy = (const T*)ws.p[blockIdx.z] + dy_off;
  float* dw = (float*)grads.p[blockIdx.z] + w_off;
  float* db = (float*)grads.p[blockIdx.z] + b_off;
  const int kk = sh.ks * sh.ks;
  const int64_t nw = (int64_t)sh.K * sh.C * kk;
  const int64_t e = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);   // element index: weights then biases
  const int lane = threadIdx.x & 63;
  if (e >= nw + sh.K) return;
  const int M = sh.N * sh.OH * sh.OW;
  float acc = 0.f;
  if (e < nw) {
    int kw = (int)(e % sh.ks);
    int64_t r = e / sh.ks;
    int kh = (int)(r % sh.ks);
    r /= sh.ks;
    int c = (int)(r % sh.C);
    int k = (int)(r / sh.C);
    for (int m = lane; m < M; m += 64) {
      int ow = m % sh.OW;
      int r2 = m / sh.OW;
      int oh = r2 % sh.OH;
      int n = r2 / sh.OH;
      int ih = oh * sh.stride + kh - sh.pad, iw = ow * sh.stride + kw - sh.pad;
      if (ih < 0 || ih >= sh.H || iw < 0 || iw >= sh.W) continue;
      acc = fmaf(ldf(dy + (int64_t)m * sh.K + k), ldf(x + (((int64_t)n * sh.H + ih) * sh.W + iw) * sh.C + c), acc);
    }
    acc = wave_sum(acc);
    if (lane == 0) dw[e] = acc;
  } else {
    int k = (int)(e - nw);
    for (int m = lane; m < M; m += 64) acc += ldf(dy + (int64_t)m * sh.K + k);
    acc = wave_sum(acc);
    if (lane == 0) db[k] = acc;
  }
}

// Fully connected layer (1 x 1 window on a 1 x 1 input): dW[k][c] = sum_n dy[n][k] x[n][c].  One thread per input
// unit c, one-wavefront workgroups, one workgroup row per kFcWU output units: neighbouring lanes read neighbouring
// x, dy[n][k] is a broadcast.  The thread of c = 0 also accumulates the bias gradients.
constexpr int kFcWU = 4;     // output units per wavefront in fc_wgrad_simple_kernel: x is read once for them
template <typename T>
__global__ __launch_bounds__(64) void fc_wgrad_simple_kernel(PtrTab ws, PtrTab grads, size_t x_off, size_t dy_off, int64_t w_off,
                                                             int64_t b_off, int N, int C, int K) {
  const T* x = (const T*)ws.p[blockIdx.z] + x_off;
  const T* dy = (const T*)ws.p[blockIdx.z] + dy_off;
  float* dw = (float*)grads.p[blockIdx.z] + w_off;
  float* db = (float*)grads.p[blockIdx.z] + b_off;
  const int c = blockIdx.x * 64 + threadIdx.x, k0 = blockIdx.y * kFcWU;
  if (c >= C) return;
  int ku[kFcWU];
#pragma unroll
  for (int u = 0; u < kFcWU; u++) ku[u] = min(k0 + u, K - 1);               // units beyond K repeat the last one and are not stored
  float acc[kFcWU], bsum[kFcWU];
#pragma unroll
  for (int u = 0; u < kFcWU; u++) acc[u] = bsum[u] = 0.f;
#pragma unroll 8
  for (int n = 0; n < N; n++) {                                             // loads of several images in flight; sums stay in image order
    const float xv = ldf(x + (int64_t)n * C + c);
#pragma unroll
    for (int u = 0; u < kFcWU; u++) {
      const float d = ldf(dy + (int64_t)n * K + ku[u]);
      acc[u] = fmaf(d, xv, acc[u]);
      bsum[u] += d;
    }
  }
#pragma unroll
  for (int u = 0; u < kFcWU; u++) {
    if (k0 + u >= K) continue;
    dw[(int64_t)(k0 + u) * C + c] = acc[u];
    if (c == 0) db[k0 + u] = bsum[u];
  }
}

static inline dim3 grid1(int64_t total, int count) {
  int64_t b = (total + 255) / 256;
  if (b > 8192) b = 8192;
  if (b < 1) b = 1;
  return dim3((unsigned)b, 1, (unsigned)count);
}

hipError_t launch_conv_fwd_simple(bool is_bf16, const PtrTab& ws, const CPtrTab& wts, size_t x_off, size_t y_off, int64_t w_off,
                                  int64_t b_off, const ConvShape& sh, bool relu, bool out_f32, int count, hipStream_t s) {
  int r = relu ? 1 : 0, of = out_f32 ? 1 : 0;
  if (sh.ks == 1 && sh.H == 1 && sh.W == 1 && sh.C >= 256 && (int64_t)sh.N * sh.K < (1 << 22)) {
    dim3 gw((unsigned)(((int64_t)sh.N * ((sh.K + kFcKU - 1) / kFcKU) + 3) / 4), 1, (unsigned)count);
    if (is_bf16) hipLaunchKernelGGL(fc_fwd_wave_kernel<bf16_t>, gw, dim3(256), 0, s, ws, wts, x_off, y_off, w_off, b_off, sh.N, sh.C, sh.K, r, of);
    else hipLaunchKernelGGL(fc_fwd_wave_kernel<float>, gw, dim3(256), 0, s, ws, wts, x_off, y_off, w_off, b_off, sh.N, sh.C, sh.K, r, of);
    return hipGetLastError();
  }
  dim3 g = grid1((int64_t)sh.N * sh.OH * sh.OW * sh.K, count);
  if (is_bf16) hipLaunchKernelGGL(conv_fwd_simple_kernel<bf16_t>, g, dim3(256), 0, s, ws, wts, x_off, y_off, w_off, b_off, sh, r, of);
  else hipLaunchKernelGGL(conv_fwd_simple_kernel<float>, g, dim3(256), 0, s, ws, wts, x_off, y_off, w_off, b_off, sh, r, of);
  return hipGetLastError();
}

hipError_t launch_conv_dgrad_simple(bool is_bf16, const PtrTab& ws, const CPtrTab& wts, size_t dy_off, size_t dx_off, int64_t w_off,
                                    const ConvShape& sh, bool use_mask, size_t mask_off, int count, hipStream_t s) {
  int um = use_mask ? 1 : 0;
  if (sh.ks == 1 && sh.H == 1 && sh.W == 1 && sh.OH == 1 && sh.OW == 1 && sh.pad == 0 && sh.stride == 1 && (int64_t)sh.N * sh.C < ((int64_t)1 << 31)) {
    dim3 gf((unsigned)(((int64_t)sh.N * sh.C + 255) / 256), 1, (unsigned)count);
    if (is_bf16) hipLaunchKernelGGL(fc_dgrad_simple_kernel<bf16_t>, gf, dim3(256), 0, s, ws, wts, dy_off, dx_off, w_off, sh.N, sh.C, sh.K, um, mask_off);
    else hipLaunchKernelGGL(fc_dgrad_simple_kernel<float>, gf, dim3(256), 0, s, ws, wts, dy_off, dx_off, w_off, sh.N, sh.C, sh.K, um, mask_off);
    return hipGetLastError();
  }
  dim3 g = grid1((int64_t)sh.N * sh.H * sh.W * sh.C, count);
  if (is_bf16) hipLaunchKernelGGL(conv_dgrad_simple_kernel<bf16_t>, g, dim3(256), 0, s, ws, wts, dy_off, dx_off, w_off, sh, um, mask_off);
  else hipLaunchKernelGGL(conv_dgrad_simple_kernel<float>, g, dim3(256), 0, s, ws, wts, dy_off, dx_off, w_off, sh, um, mask_off);
  return hipGetLastError();
}

hipError_t launch_conv_wgrad_simple(bool is_bf16, const PtrTab& ws, const PtrTab& grads, size_t x_off, size_t dy_off, int64_t w_off,
                                    int64_t b_off, const ConvShape& sh, int count, hipStream_t s) {
  if (sh.ks == 1 && sh.H == 1 && sh.W == 1 && sh.pad == 0 && sh.K <= 65535) {
    dim3 g((unsigned)((sh.C + 63) / 64), (unsigned)((sh.K + kFcWU - 1) / kFcWU), (unsigned)count);
    if (is_bf16) hipLaunchKernelGGL(fc_wgrad_simple_kernel<bf16_t>, g, dim3(64), 0, s, ws, grads, x_off, dy_off, w_off, b_off, sh.N, sh.C, sh.K);
    else hipLaunchKernelGGL(fc_wgrad_simple_kernel<float>, g, dim3(64), 0, s, ws, grads, x_off, dy_off, w_off, b_off, sh.N, sh.C, sh.K);
    return hipGetLastError();
  }
  const int64_t elems = (int64_t)sh.K * sh.C * sh.ks * sh.ks + sh.K;
  const int64_t blocks = (elems + 3) / 4;
  if (blocks > 0x7fffffff) return hipErrorInvalidValue;
  dim3 g((unsigned)blocks, 1, (unsigned)count);
  if (is_bf16) hipLaunchKernelGGL(conv_wgrad_simple_kernel<bf16_t>, g, dim3(256), 0, s, ws, grads, x_off, dy_off, w_off, b_off, sh);
  else hipLaunchKernelGGL(conv_wgrad_simple_kernel<float>, g, dim3(256), 0, s, ws, grads, x_off, dy_off, w_off, b_off, sh);
  return hipGetLastError();
}

}  // namespace sasgd
