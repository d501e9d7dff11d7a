// Element-wise and windowed layers of calcGradient (Section 2.1; layer types of Section 4.1): input
// re-layout, max / average pooling with clipped ceil-mode windows, flattening, softmax cross-entropy.
// All are bandwidth-bound; lanes walk the channel-innermost (NHWC) index so loads and stores coalesce,
// reductions over classes use one wavefront per image.  blockIdx.z selects the learner.
#include "dev_common.hpp"
#include "kernels.hpp"

namespace sasgd {

static inline dim3 grid_for(int64_t total, int count, int cap = 4096) {
  int64_t b = (total + 255) / 256;
  if (b > cap) b = cap;
  if (b < 1) b = 1;
  return dim3((unsigned)b, 1, (unsigned)count);
}

struct bf8 {
  uint4 v;
  __device__ __forceinline__ float get(int i) const {
    uint32_t w = i < 2 ? v.x : (i < 4 ? v.y : (i < 6 ? v.z : v.w));
    return __uint_as_float((i & 1) ? (w & 0xffff0000u) : (w << 16));
  }
};
__device__ __forceinline__ uint4 pack8(const float* f) {
  uint4 o;
  o.x = (uint32_t)f2bf(f[0]) | ((uint32_t)f2bf(f[1]) << 16);
  o.y = (uint32_t)f2bf(f[2]) | ((uint32_t)f2bf(f[3]) << 16);
  o.z = (uint32_t)f2bf(f[4]) | ((uint32_t)f2bf(f[5]) << 16);
  o.w = (uint32_t)f2bf(f[6]) | ((uint32_t)f2bf(f[7]) << 16);
  return o;
}

// ------------------------------------------------------------------ input NCHW fp32 -> NHWC T
template <typename T>
__global__ __launch_bounds__(256) void pack_input_kernel(CPtrTab images, PtrTab ws, size_t out_off, int N, InPack ip,
                                                         const float* __restrict__ mean) {
  const float* in = (const float*)images.p[blockIdx.z];
  T* out = (T*)ws.p[blockIdx.z] + out_off;
  const int64_t total = (int64_t)N * ip.Hp * ip.Wp * ip.Cp;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    int cp = (int)(i % ip.Cp);
    int64_t r = i / ip.Cp;
    int X = (int)(r % ip.Wp);
    r /= ip.Wp;
    int Y = (int)(r % ip.Hp);
    int n = (int)(r / ip.Hp);
    float v = 0.f;
    if (ip.s2d == 1) {
      if (cp < ip.C) {
        const int64_t pix = ((int64_t)cp * ip.H + Y) * ip.W + X;
        v = in[(int64_t)n * ip.C * ip.H * ip.W + pix] - (mean ? mean[pix] : 0.f);
      }
    } else {
      int g = cp / ip.C, c = cp % ip.C;
      int h = ip.s2d * Y + g / ip.s2d, w = ip.s2d * X + g % ip.s2d;
      if (g < ip.s2d * ip.s2d && h < ip.H && w < ip.W) {
        const int64_t pix = ((int64_t)c * ip.H + h) * ip.W + w;
        v = in[(int64_t)n * ip.C * ip.H * ip.W + pix] - (mean ? mean[pix] : 0.f);
      }
    }
    stf(out + i, v);
  }
}

// One lane per destination pixel (bf16, Cp % 8 == 0): the Cp channels are assembled in registers and written as
// 16-byte chunks; neighbouring lanes read neighbouring source columns.
__global__ __launch_bounds__(256) void pack_input_pixel_kernel(CPtrTab images, PtrTab ws, size_t out_off, int N, InPack ip,
                                                               const float* __restrict__ mean) {
  const float* in = (const float*)images.p[blockIdx.z];
  bf16_t* out = (bf16_t*)ws.p[blockIdx.z] + out_off;
  const int64_t total = (int64_t)N * ip.Hp * ip.Wp;
  const int64_t plane = (int64_t)ip.H * ip.W;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    int X = (int)(i % ip.Wp);
    int64_t r = i / ip.Wp;
    int Y = (int)(r % ip.Hp);
    int n = (int)(r / ip.Hp);
    const float* src = in + (int64_t)n * ip.C * plane;
    for (int c0 = 0; c0 < ip.Cp; c0 += 8) {
      float f[8];
#pragma unroll
      for (int e = 0; e < 8; e++) {
        const int cp = c0 + e;
        float v = 0.f;
        if (ip.s2d == 1) {
          if (cp < ip.C) {
            const int64_t pix = cp * plane + (int64_t)Y * ip.W + X;
            v = src[pix] - (mean ? mean[pix] : 0.f);
          }
        } else {
          int g = cp / ip.C, c = cp - g * ip.C;
          int h = ip.s2d * Y + g / ip.s2d, w = ip.s2d * X + g % ip.s2d;
          if (g < ip.s2d * ip.s2d && h < ip.H && w < ip.W) {
            const int64_t pix = c * plane + (int64_t)h * ip.W + w;
            v = src[pix] - (mean ? mean[pix] : 0.f);
          }
        }
        f[e] = v;
      }
      *reinterpret_cast<uint4*>(out + i * ip.Cp + c0) = pack8(f);
    }
  }
}

// Space-to-depth by 4 of a 3-channel image (the 11 x 11 / 4 first layer): one lane per destination pixel reads twelve
// aligned float4 (channel c, row 4Y + dh, columns 4X .. 4X+3) and writes its 48 channels (dh * 4 + dw) * 3 + c as six
// 16-byte chunks.  Needs W % 4 == 0 and 16-byte aligned images (and mean).
__global__ __launch_bounds__(256) void pack_input_s2d4_kernel(CPtrTab images, PtrTab ws, size_t out_off, int N, InPack ip,
                                                              const float* __restrict__ mean) {
  const float* in = (const float*)images.p[blockIdx.z];
  bf16_t* out = (bf16_t*)ws.p[blockIdx.z] + out_off;
  const int64_t total = (int64_t)N * ip.Hp * ip.Wp;
  const int64_t plane = (int64_t)ip.H * ip.W;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    uint32_t r = (uint32_t)i;
    const int X = (int)(r % (uint32_t)ip.Wp);
    r /= (uint32_t)ip.Wp;
    const int Y = (int)(r % (uint32_t)ip.Hp);
    const int n = (int)(r / (uint32_t)ip.Hp);
    const float* src = in + (int64_t)n * 3 * plane;
    float f[48];
#pragma unroll
    for (int dh = 0; dh < 4; dh++) {
      const int h = 4 * Y + dh;
#pragma unroll
      for (int c = 0; c < 3; c++) {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (h < ip.H && 4 * X < ip.W) {
          const int64_t pix = c * plane + (int64_t)h * ip.W + 4 * X;
          v = *reinterpret_cast<const float4*>(src + pix);
          if (mean) {
            const float4 mv = *reinterpret_cast<const float4*>(mean + pix);
            v.x -= mv.x; v.y -= mv.y; v.z -= mv.z; v.w -= mv.w;
          }
        }
        f[(dh * 4 + 0) * 3 + c] = v.x;
        f[(dh * 4 + 1) * 3 + c] = v.y;
        f[(dh * 4 + 2) * 3 + c] = v.z;
        f[(dh * 4 + 3) * 3 + c] = v.w;
      }
    }
#pragma unroll
    for (int c0 = 0; c0 < 48; c0 += 8) *reinterpret_cast<uint4*>(out + i * 48 + c0) = pack8(f + c0);
  }
}

hipError_t launch_pack_input(bool is_bf16, const CPtrTab& images, const PtrTab& ws, size_t out_off, int count, int N,
                             const InPack& ip, const float* mean, hipStream_t s) {
  if (is_bf16 && ip.s2d == 4 && ip.C == 3 && ip.Cp == 48 && ip.W % 4 == 0 && out_off % 8 == 0 && ((uintptr_t)mean & 15) == 0) {
    bool aligned = true;
    for (int k = 0; k < count; k++) aligned = aligned && ((uintptr_t)images.p[k] & 15) == 0;
    if (aligned) {
      dim3 gv = grid_for((int64_t)N * ip.Hp * ip.Wp, count, 16384);
      hipLaunchKernelGGL(pack_input_s2d4_kernel, gv, dim3(256), 0, s, images, ws, out_off, N, ip, mean);
      return hipGetLastError();
    }
  }
  if (is_bf16 && ip.Cp % 8 == 0 && out_off % 8 == 0) {
    dim3 gv = grid_for((int64_t)N * ip.Hp * ip.Wp, count, 16384);
    hipLaunchKernelGGL(pack_input_pixel_kernel, gv, dim3(256), 0, s, images, ws, out_off, N, ip, mean);
    return hipGetLastError();
  }
  dim3 g = grid_for((int64_t)N * ip.Cp * ip.Hp * ip.Wp, count);
  if (is_bf16) hipLaunchKernelGGL(pack_input_kernel<bf16_t>, g, dim3(256), 0, s, images, ws, out_off, N, ip, mean);
  else hipLaunchKernelGGL(pack_input_kernel<float>, g, dim3(256), 0, s, images, ws, out_off, N, ip, mean);
  return hipGetLastError();
}

// ------------------------------------------------------------------ pooling
// Windows start at (oh*stride, ow*stride) and are clipped at the border.  Max: the first maximum in
// row-major window order wins and its position inside the window is kept (one byte) for the backward
// pass.  Average: the divisor is the number of in-bounds elements.
template <typename T, bool MAX>
__global__ __launch_bounds__(256) void pool_fwd_kernel(PtrTab ws, size_t x_off, size_t y_off, size_t arg_byte_off, PoolShape sh,
                                                       int relu) {
  const T* x = (const T*)ws.p[blockIdx.z] + x_off;
  T* y = (T*)ws.p[blockIdx.z] + y_off;
  uint8_t* arg = (uint8_t*)ws.p[blockIdx.z] + arg_byte_off;
  const int64_t total = (int64_t)sh.N * sh.OH * sh.OW * sh.C;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    int c = (int)(i % sh.C);
    int64_t r = i / sh.C;
    int ow = (int)(r % sh.OW);
    r /= sh.OW;
    int oh = (int)(r % sh.OH);
    int n = (int)(r / sh.OH);
    const int h0 = oh * sh.stride, w0 = ow * sh.stride;
    float acc = 0.f;
    int best = 0, cnt = 0;
    for (int kh = 0; kh < sh.ks && h0 + kh < sh.H; kh++)
      for (int kw = 0; kw < sh.ks && w0 + kw < sh.W; kw++) {
        float v = ldf(x + (((int64_t)n * sh.H + h0 + kh) * sh.W + w0 + kw) * sh.C + c);
        if (MAX) {
          if (cnt == 0 || v > acc) { acc = v; best = kh * sh.ks + kw; }
        } else {
          acc += v;
        }
        cnt++;
      }
    if (!MAX) acc /= (float)cnt;
    if (relu) acc = fmaxf(acc, 0.f);
    stf(y + i, acc);
    if (MAX) arg[i] = (uint8_t)best;
  }
}

template <typename T, bool MAX>
__global__ __launch_bounds__(256) void pool_bwd_kernel(PtrTab ws, size_t dy_off, size_t dx_off, size_t arg_byte_off, PoolShape sh,
                                                       int use_mask, size_t mask_off) {
  const T* dy = (const T*)ws.p[blockIdx.z] + dy_off;
  T* dx = (T*)ws.p[blockIdx.z] + dx_off;
  const T* mask = (const T*)ws.p[blockIdx.z] + mask_off;
  const uint8_t* arg = (const uint8_t*)ws.p[blockIdx.z] + arg_byte_off;
  const int64_t total = (int64_t)sh.N * sh.H * sh.W * sh.C;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    int c = (int)(i % sh.C);
    int64_t r = i / sh.C;
    int iw = (int)(r % sh.W);
    r /= sh.W;
    int ih = (int)(r % sh.H);
    int n = (int)(r / sh.H);
    float acc = 0.f;
    if (!use_mask || ldf(mask + i) > 0.f) {
      // windows that contain (ih, iw): oh*stride <= ih < oh*stride + ks
      int oh_lo = ih - sh.ks + 1 > 0 ? (ih - sh.ks + sh.stride) / sh.stride : 0;
      int oh_hi = min(sh.OH - 1, ih / sh.stride);
      int ow_lo = iw - sh.ks + 1 > 0 ? (iw - sh.ks + sh.stride) / sh.stride : 0;
      int ow_hi = min(sh.OW - 1, iw / sh.stride);
      for (int oh = oh_lo; oh <= oh_hi; oh++)
        for (int ow = ow_lo; ow <= ow_hi; ow++) {
          const int64_t o = (((int64_t)n * sh.OH + oh) * sh.OW + ow) * sh.C + c;
          if (MAX) {
            if (arg[o] == (uint8_t)((ih - oh * sh.stride) * sh.ks + (iw - ow * sh.stride))) acc += ldf(dy + o);
          } else {
            int ch = min(oh * sh.stride + sh.ks, sh.H) - oh * sh.stride;
            int cw = min(ow * sh.stride + sh.ks, sh.W) - ow * sh.stride;
            acc += ldf(dy + o) / (float)(ch * cw);
          }
        }
    }
    stf(dx + i, acc);
  }
}

// ------------------------------------------------------------------ pooling, 8 channels per lane (bf16, C % 8 == 0)
// Same arithmetic as the scalar kernels; each lane moves 16-byte channel chunks, so a wavefront reads and
// writes 1 KiB contiguous runs.
template <bool MAX>
__global__ __launch_bounds__(256) void pool_fwd_vec8_kernel(PtrTab ws, size_t x_off, size_t y_off, size_t arg_byte_off, PoolShape sh,
                                                            int relu) {
  const bf16_t* x = (const bf16_t*)ws.p[blockIdx.z] + x_off;
  bf16_t* y = (bf16_t*)ws.p[blockIdx.z] + y_off;
  uint8_t* arg = (uint8_t*)ws.p[blockIdx.z] + arg_byte_off;
  const int C8 = sh.C / 8;
  const int64_t total = (int64_t)sh.N * sh.OH * sh.OW * C8;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    // 32-bit index arithmetic: a tensor of one learner has fewer than 2^31 elements
    uint32_t r = (uint32_t)i;
    const int c8 = (int)(r % (uint32_t)C8);
    r /= (uint32_t)C8;
    const int ow = (int)(r % (uint32_t)sh.OW);
    r /= (uint32_t)sh.OW;
    const int oh = (int)(r % (uint32_t)sh.OH);
    const int n = (int)(r / (uint32_t)sh.OH);
    const int h0 = oh * sh.stride, w0 = ow * sh.stride;
    float acc[8];
    int best[8];
#pragma unroll
    for (int e = 0; e < 8; e++) { acc[e] = 0.f; best[e] = 0; }
    int cnt = 0;
    for (int kh = 0; kh < sh.ks && h0 + kh < sh.H; kh++)
      for (int kw = 0; kw < sh.ks && w0 + kw < sh.W; kw++) {
        bf8 v;
        v.v = *reinterpret_cast<const uint4*>(x + (((int64_t)n * sh.H + h0 + kh) * sh.W + w0 + kw) * sh.C + c8 * 8);
#pragma unroll
        for (int e = 0; e < 8; e++) {
          float f = v.get(e);
          if (MAX) {
            if (cnt == 0 || f > acc[e]) { acc[e] = f; best[e] = kh * sh.ks + kw; }
          } else {
            acc[e] += f;
          }
        }
        cnt++;
      }
#pragma unroll
    for (int e = 0; e < 8; e++) {
      if (!MAX) acc[e] /= (float)cnt;
      if (relu) acc[e] = fmaxf(acc[e], 0.f);
    }
    *reinterpret_cast<uint4*>(y + i * 8) = pack8(acc);
    if (MAX) {
      uint2 a;
      a.x = (uint32_t)best[0] | ((uint32_t)best[1] << 8) | ((uint32_t)best[2] << 16) | ((uint32_t)best[3] << 24);
      a.y = (uint32_t)best[4] | ((uint32_t)best[5] << 8) | ((uint32_t)best[6] << 16) | ((uint32_t)best[7] << 24);
      *reinterpret_cast<uint2*>(arg + i * 8) = a;
    }
  }
}

// 3 x 3 windows (every pooling layer of the two reference networks): the nine 16-byte reads of a window are all
// requested before the first is used (the general kernel above walks the window in a loop whose trip count the
// compiler does not know, one dependent read after the other).  Same arithmetic and the same winner on ties.
template <bool MAX>
__global__ __launch_bounds__(256) void pool_fwd_3x3_kernel(PtrTab ws, size_t x_off, size_t y_off, size_t arg_byte_off, PoolShape sh, int relu) {
  const bf16_t* x = (const bf16_t*)ws.p[blockIdx.z] + x_off;
  bf16_t* y = (bf16_t*)ws.p[blockIdx.z] + y_off;
  uint8_t* arg = (uint8_t*)ws.p[blockIdx.z] + arg_byte_off;
  const int C8 = sh.C / 8;
  const uint32_t total = (uint32_t)sh.N * sh.OH * sh.OW * C8;
  for (uint32_t i = blockIdx.x * 256 + threadIdx.x; i < total; i += gridDim.x * 256) {
    uint32_t r = i;
    const int c8 = (int)(r % (uint32_t)C8);
    r /= (uint32_t)C8;
    const int ow = (int)(r % (uint32_t)sh.OW);
    r /= (uint32_t)sh.OW;
    const int oh = (int)(r % (uint32_t)sh.OH);
    const int n = (int)(r / (uint32_t)sh.OH);
    const int h0 = oh * sh.stride, w0 = ow * sh.stride;
    const int nh = min(3, sh.H - h0), nw = min(3, sh.W - w0);          // rows and columns of the window inside the image
    const bf16_t* base = x + (((int64_t)n * sh.H + h0) * sh.W + w0) * sh.C + c8 * 8;
    bf8 v[9];
#pragma unroll
    for (int kh = 0; kh < 3; kh++)
#pragma unroll
      for (int kw = 0; kw < 3; kw++) {
        const bool in = kh < nh && kw < nw;
        v[kh * 3 + kw].v = *reinterpret_cast<const uint4*>(base + (in ? ((int64_t)kh * sh.W + kw) * sh.C : 0));   // outside: the first element again
      }
    float acc[8];
    int best[8];
#pragma unroll
    for (int e = 0; e < 8; e++) { acc[e] = v[0].get(e); best[e] = 0; }
#pragma unroll
    for (int t = 1; t < 9; t++) {
      const bool in = t / 3 < nh && t % 3 < nw;
#pragma unroll
      for (int e = 0; e < 8; e++) {
        const float f = v[t].get(e);
        if (MAX) {
          if (in && f > acc[e]) { acc[e] = f; best[e] = t; }
        } else {
          if (in) acc[e] += f;
        }
      }
    }
    const float cnt = (float)(nh * nw);
#pragma unroll
    for (int e = 0; e < 8; e++) {
      if (!MAX) acc[e] /= cnt;
      if (relu) acc[e] = fmaxf(acc[e], 0.f);
    }
    *reinterpret_cast<uint4*>(y + (size_t)i * 8) = pack8(acc);
    if (MAX) {
      uint2 a;
      a.x = (uint32_t)best[0] | ((uint32_t)best[1] << 8) | ((uint32_t)best[2] << 16) | ((uint32_t)best[3] << 24);
      a.y = (uint32_t)best[4] | ((uint32_t)best[5] << 8) | ((uint32_t)best[6] << 16) | ((uint32_t)best[7] << 24);
      *reinterpret_cast<uint2*>(arg + (size_t)i * 8) = a;
    }
  }
}

template <bool MAX>
__global__ __launch_bounds__(256) void pool_bwd_vec8_kernel(PtrTab ws, size_t dy_off, size_t dx_off, size_t arg_byte_off, PoolShape sh,
                                                            int use_mask, size_t mask_off) {
  const bf16_t* dy = (const bf16_t*)ws.p[blockIdx.z] + dy_off;
  bf16_t* dx = (bf16_t*)ws.p[blockIdx.z] + dx_off;
  const bf16_t* mask = (const bf16_t*)ws.p[blockIdx.z] + mask_off;
  const uint8_t* arg = (const uint8_t*)ws.p[blockIdx.z] + arg_byte_off;
  const int C8 = sh.C / 8;
  const int64_t total = (int64_t)sh.N * sh.H * sh.W * C8;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    uint32_t r = (uint32_t)i;
    const int c8 = (int)(r % (uint32_t)C8);
    r /= (uint32_t)C8;
    const int iw = (int)(r % (uint32_t)sh.W);
    r /= (uint32_t)sh.W;
    const int ih = (int)(r % (uint32_t)sh.H);
    const int n = (int)(r / (uint32_t)sh.H);
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; e++) acc[e] = 0.f;
    int oh_lo = ih - sh.ks + 1 > 0 ? (ih - sh.ks + sh.stride) / sh.stride : 0;
    int oh_hi = min(sh.OH - 1, ih / sh.stride);
    int ow_lo = iw - sh.ks + 1 > 0 ? (iw - sh.ks + sh.stride) / sh.stride : 0;
    int ow_hi = min(sh.OW - 1, iw / sh.stride);
    for (int oh = oh_lo; oh <= oh_hi; oh++)
      for (int ow = ow_lo; ow <= ow_hi; ow++) {
        const int64_t o = ((((int64_t)n * sh.OH + oh) * sh.OW + ow) * C8 + c8) * 8;
        bf8 d;
        d.v = *reinterpret_cast<const uint4*>(dy + o);
        if (MAX) {
          const uint2 a = *reinterpret_cast<const uint2*>(arg + o);
          const uint32_t pos = (uint32_t)((ih - oh * sh.stride) * sh.ks + (iw - ow * sh.stride));
#pragma unroll
          for (int e = 0; e < 8; e++) {
            uint32_t ae = ((e < 4 ? a.x : a.y) >> (8 * (e & 3))) & 0xffu;
            if (ae == pos) acc[e] += d.get(e);
          }
        } else {
          int ch = min(oh * sh.stride + sh.ks, sh.H) - oh * sh.stride;
          int cw = min(ow * sh.stride + sh.ks, sh.W) - ow * sh.stride;
          const float inv = (float)(ch * cw);
#pragma unroll
          for (int e = 0; e < 8; e++) acc[e] += d.get(e) / inv;
        }
      }
    if (use_mask) {
      bf8 mk;
      mk.v = *reinterpret_cast<const uint4*>(mask + i * 8);
#pragma unroll
      for (int e = 0; e < 8; e++)
        if (!(mk.get(e) > 0.f)) acc[e] = 0.f;
    }
    *reinterpret_cast<uint4*>(dx + i * 8) = pack8(acc);
  }
}

// 3 x 3 windows at stride 2 (every pooling layer of the two reference networks): one lane owns 8 channels of a 2 x 2
// block of the input, rows 2a, 2a+1 and columns 2b, 2b+1.  Only the four windows (a-1 | a, b-1 | b) reach into the
// block, so they are read once for the four results instead of once per covered element (nine reads per block).
template <bool MAX>
__global__ __launch_bounds__(256) void pool_bwd_3x3s2_kernel(PtrTab ws, size_t dy_off, size_t dx_off, size_t arg_byte_off, PoolShape sh,
                                                             int use_mask, size_t mask_off) {
  const bf16_t* dy = (const bf16_t*)ws.p[blockIdx.z] + dy_off;
  bf16_t* dx = (bf16_t*)ws.p[blockIdx.z] + dx_off;
  const bf16_t* mask = (const bf16_t*)ws.p[blockIdx.z] + mask_off;
  const uint8_t* arg = (const uint8_t*)ws.p[blockIdx.z] + arg_byte_off;
  const int C8 = sh.C / 8, HB = (sh.H + 1) / 2, WB = (sh.W + 1) / 2;
  const uint32_t total = (uint32_t)sh.N * HB * WB * C8;
  for (uint32_t i = blockIdx.x * 256 + threadIdx.x; i < total; i += gridDim.x * 256) {
    uint32_t r = i;
    const int c8 = (int)(r % (uint32_t)C8);
    r /= (uint32_t)C8;
    const int b = (int)(r % (uint32_t)WB);
    r /= (uint32_t)WB;
    const int a = (int)(r % (uint32_t)HB);
    const int n = (int)(r / (uint32_t)HB);
    // All reads are requested before the first is used: windows outside the output and block elements outside the
    // input read a clamped (valid) address and are discarded by a predicate instead of a branch around the load.
    bool w_ok[4];
    uint4 dv[4];
    uint2 av[4];
    float inv[4];
#pragma unroll
    for (int wh = 0; wh < 2; wh++)
#pragma unroll
      for (int ww = 0; ww < 2; ww++) {
        const int oh = a - 1 + wh, ow = b - 1 + ww;
        const int q = 2 * wh + ww;
        w_ok[q] = oh >= 0 && oh < sh.OH && ow >= 0 && ow < sh.OW;
        const int ohc = min(max(oh, 0), sh.OH - 1), owc = min(max(ow, 0), sh.OW - 1);
        const int64_t o = ((((int64_t)n * sh.OH + ohc) * sh.OW + owc) * C8 + c8) * 8;
        dv[q] = *reinterpret_cast<const uint4*>(dy + o);
        av[q] = make_uint2(0u, 0u);
        if (MAX) av[q] = *reinterpret_cast<const uint2*>(arg + o);
        inv[q] = 1.f;
        if (!MAX) {
          const int ch = min(ohc * 2 + 3, sh.H) - ohc * 2, cw = min(owc * 2 + 3, sh.W) - owc * 2;
          inv[q] = 1.f / (float)(ch * cw);
        }
      }
    bool x_ok[4];
    int64_t xo[4];
    uint4 mv[4];
#pragma unroll
    for (int dh = 0; dh < 2; dh++)
#pragma unroll
      for (int dw = 0; dw < 2; dw++) {
        const int ih = 2 * a + dh, iw = 2 * b + dw;
        const int q = 2 * dh + dw;
        x_ok[q] = ih < sh.H && iw < sh.W;
        xo[q] = ((((int64_t)n * sh.H + min(ih, sh.H - 1)) * sh.W + min(iw, sh.W - 1)) * C8 + c8) * 8;
        mv[q] = make_uint4(0u, 0u, 0u, 0u);
        if (use_mask) mv[q] = *reinterpret_cast<const uint4*>(mask + xo[q]);
      }
    float acc[4][8];                                    // [2 * dh + dw][channel]
#pragma unroll
    for (int q = 0; q < 4; q++)
#pragma unroll
      for (int e = 0; e < 8; e++) acc[q][e] = 0.f;
#pragma unroll
    for (int wh = 0; wh < 2; wh++)
#pragma unroll
      for (int ww = 0; ww < 2; ww++) {
        const int wq = 2 * wh + ww;
        bf8 d;
        d.v = w_ok[wq] ? dv[wq] : make_uint4(0u, 0u, 0u, 0u);
        const uint2 ar = av[wq];
        // window (oh, ow) = (a - 1 + wh, b - 1 + ww) starts at row 2 oh, column 2 ow: block row dh sits at window row
        // 2 (a - oh) + dh, i.e. 2, 3 for the window above (only 2 is inside), 0, 1 for the own one
#pragma unroll
        for (int dh = 0; dh < 2; dh++) {
          const int wr = 2 * (1 - wh) + dh;
          if (wr > 2) continue;
#pragma unroll
          for (int dw = 0; dw < 2; dw++) {
            const int wc = 2 * (1 - ww) + dw;
            if (wc > 2) continue;
            const uint32_t pos = (uint32_t)(wr * 3 + wc);
#pragma unroll
            for (int e = 0; e < 8; e++) {
              if (MAX) {
                const uint32_t ae = ((e < 4 ? ar.x : ar.y) >> (8 * (e & 3))) & 0xffu;
                if (ae == pos) acc[2 * dh + dw][e] += d.get(e);
              } else {
                acc[2 * dh + dw][e] += d.get(e) * inv[wq];
              }
            }
          }
        }
      }
#pragma unroll
    for (int q = 0; q < 4; q++) {
      if (!x_ok[q]) continue;
      if (use_mask) {
        bf8 mk;
        mk.v = mv[q];
#pragma unroll
        for (int e = 0; e < 8; e++)
          if (!(mk.get(e) > 0.f)) acc[q][e] = 0.f;
      }
      *reinterpret_cast<uint4*>(dx + xo[q]) = pack8(acc[q]);
    }
  }
}

hipError_t launch_pool_fwd(bool is_bf16, bool is_max, const PtrTab& ws, size_t x_off, size_t y_off, size_t arg_byte_off,
                           const PoolShape& sh, bool relu, int count, hipStream_t s) {
  dim3 g = grid_for((int64_t)sh.N * sh.OH * sh.OW * sh.C, count);
  int r = relu ? 1 : 0;
  if (is_bf16 && sh.C % 8 == 0 && x_off % 8 == 0 && y_off % 8 == 0 && arg_byte_off % 8 == 0) {
    dim3 gv = grid_for((int64_t)sh.N * sh.OH * sh.OW * (sh.C / 8), count, 16384);
    if (sh.ks == 3 && (int64_t)sh.N * sh.H * sh.W * sh.C < ((int64_t)1 << 31)) {
      if (is_max) hipLaunchKernelGGL((pool_fwd_3x3_kernel<true>), gv, dim3(256), 0, s, ws, x_off, y_off, arg_byte_off, sh, r);
      else hipLaunchKernelGGL((pool_fwd_3x3_kernel<false>), gv, dim3(256), 0, s, ws, x_off, y_off, arg_byte_off, sh, r);
      return hipGetLastError();
    }
    if (is_max) hipLaunchKernelGGL((pool_fwd_vec8_kernel<true>), gv, dim3(256), 0, s, ws, x_off, y_off, arg_byte_off, sh, r);
    else hipLaunchKernelGGL((pool_fwd_vec8_kernel<false>), gv, dim3(256), 0, s, ws, x_off, y_off, arg_byte_off, sh, r);
    return hipGetLastError();
  }
  if (is_bf16) {
    if (is_max) hipLaunchKernelGGL((pool_fwd_kernel<bf16_t, true>), g, dim3(256), 0, s, ws, x_off, y_off, arg_byte_off, sh, r);
    else hipLaunchKernelGGL((pool_fwd_kernel<bf16_t, false>), g, dim3(256), 0, s, ws, x_off, y_off, arg_byte_off, sh, r);
  } else {
    if (is_max) hipLaunchKernelGGL((pool_fwd_kernel<float, true>), g, dim3(256), 0, s, ws, x_off, y_off, arg_byte_off, sh, r);
    else hipLaunchKernelGGL((pool_fwd_kernel<float, false>), g, dim3(256), 0, s, ws, x_off, y_off, arg_byte_off, sh, r);
  }
  return hipGetLastError();
}

hipError_t launch_pool_bwd(bool is_bf16, bool is_max, const PtrTab& ws, size_t dy_off, size_t dx_off, size_t arg_byte_off,
                           const PoolShape& sh, bool use_mask, size_t mask_off, int count, hipStream_t s) {
  dim3 g = grid_for((int64_t)sh.N * sh.H * sh.W * sh.C, count);
  int um = use_mask ? 1 : 0;
  if (is_bf16 && sh.C % 8 == 0 && dy_off % 8 == 0 && dx_off % 8 == 0 && arg_byte_off % 8 == 0 && mask_off % 8 == 0) {
    if (sh.ks == 3 && sh.stride == 2) {
      dim3 gb = grid_for((int64_t)sh.N * ((sh.H + 1) / 2) * ((sh.W + 1) / 2) * (sh.C / 8), count, 16384);
      if (is_max) hipLaunchKernelGGL((pool_bwd_3x3s2_kernel<true>), gb, dim3(256), 0, s, ws, dy_off, dx_off, arg_byte_off, sh, um, mask_off);
      else hipLaunchKernelGGL((pool_bwd_3x3s2_kernel<false>), gb, dim3(256), 0, s, ws, dy_off, dx_off, arg_byte_off, sh, um, mask_off);
      return hipGetLastError();
    }
    dim3 gv = grid_for((int64_t)sh.N * sh.H * sh.W * (sh.C / 8), count, 16384);
    if (is_max) hipLaunchKernelGGL((pool_bwd_vec8_kernel<true>), gv, dim3(256), 0, s, ws, dy_off, dx_off, arg_byte_off, sh, um, mask_off);
    else hipLaunchKernelGGL((pool_bwd_vec8_kernel<false>), gv, dim3(256), 0, s, ws, dy_off, dx_off, arg_byte_off, sh, um, mask_off);
    return hipGetLastError();
  }
  if (is_bf16) {
    if (is_max) hipLaunchKernelGGL((pool_bwd_kernel<bf16_t, true>), g, dim3(256), 0, s, ws, dy_off, dx_off, arg_byte_off, sh, um, mask_off);
    else hipLaunchKernelGGL((pool_bwd_kernel<bf16_t, false>), g, dim3(256), 0, s, ws, dy_off, dx_off, arg_byte_off, sh, um, mask_off);
  } else {
    if (is_max) hipLaunchKernelGGL((pool_bwd_kernel<float, true>), g, dim3(256), 0, s, ws, dy_off, dx_off, arg_byte_off, sh, um, mask_off);
    else hipLaunchKernelGGL((pool_bwd_kernel<float, false>), g, dim3(256), 0, s, ws, dy_off, dx_off, arg_byte_off, sh, um, mask_off);
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------ flatten (NHWC -> C,H,W order) and back
template <typename T>
__global__ __launch_bounds__(256) void flatten_fwd_kernel(PtrTab ws, size_t x_off, size_t y_off, int N, int C, int H, int W) {
  const T* x = (const T*)ws.p[blockIdx.z] + x_off;
  T* y = (T*)ws.p[blockIdx.z] + y_off;
  const int HW = H * W;
  const int64_t total = (int64_t)N * C * HW;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    int hw = (int)(i % HW);
    int64_t r = i / HW;
    int c = (int)(r % C);
    int n = (int)(r / C);
    y[i] = x[((int64_t)n * HW + hw) * C + c];
  }
}

template <typename T>
__global__ __launch_bounds__(256) void flatten_bwd_kernel(PtrTab ws, size_t dy_off, size_t dx_off, int N, int C, int H, int W,
                                                          int use_mask, size_t mask_off) {
  const T* dy = (const T*)ws.p[blockIdx.z] + dy_off;
  T* dx = (T*)ws.p[blockIdx.z] + dx_off;
  const T* mask = (const T*)ws.p[blockIdx.z] + mask_off;
  const int HW = H * W;
  const int64_t total = (int64_t)N * C * HW;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    int c = (int)(i % C);
    int64_t r = i / C;
    int hw = (int)(r % HW);
    int n = (int)(r / HW);
    float v = ldf(dy + ((int64_t)n * C + c) * HW + hw);
    if (use_mask && !(ldf(mask + i) > 0.f)) v = 0.f;
    stf(dx + i, v);
  }
}

hipError_t launch_flatten_fwd(bool is_bf16, const PtrTab& ws, size_t x_off, size_t y_off, int N, int C, int H, int W, int count,
                              hipStream_t s) {
  dim3 g = grid_for((int64_t)N * C * H * W, count);
  if (is_bf16) hipLaunchKernelGGL(flatten_fwd_kernel<bf16_t>, g, dim3(256), 0, s, ws, x_off, y_off, N, C, H, W);
  else hipLaunchKernelGGL(flatten_fwd_kernel<float>, g, dim3(256), 0, s, ws, x_off, y_off, N, C, H, W);
  return hipGetLastError();
}

hipError_t launch_flatten_bwd(bool is_bf16, const PtrTab& ws, size_t dy_off, size_t dx_off, int N, int C, int H, int W, bool use_mask,
                              size_t mask_off, int count, hipStream_t s) {
  dim3 g = grid_for((int64_t)N * C * H * W, count);
  int um = use_mask ? 1 : 0;
  if (is_bf16) hipLaunchKernelGGL(flatten_bwd_kernel<bf16_t>, g, dim3(256), 0, s, ws, dy_off, dx_off, N, C, H, W, um, mask_off);
  else hipLaunchKernelGGL(flatten_bwd_kernel<float>, g, dim3(256), 0, s, ws, dy_off, dx_off, N, C, H, W, um, mask_off);
  return hipGetLastError();
}

// ------------------------------------------------------------------ softmax cross-entropy
// One workgroup per image: dz = (softmax(z) - onehot(label)) / N, i.e. the gradient of the MEAN loss: this is
// where the division by the mini-batch size enters (Section 2.1).  The per-image losses go to a small array and
// are summed in image order by a second tiny kernel, so the result does not depend on scheduling.
template <typename T, typename Z>
__global__ __launch_bounds__(256) void softmax_ce_kernel(PtrTab ws, CPtrTab labels, size_t z_off, size_t dz_off, size_t loss_byte_off,
                                                         int N, int K) {
  __shared__ float red[4];
  const int l = blockIdx.z, n = blockIdx.x;
  const Z* zn = reinterpret_cast<const Z*>((const T*)ws.p[l] + z_off) + (int64_t)n * K;
  T* dz = (T*)ws.p[l] + dz_off + (int64_t)n * K;
  float* img_loss = reinterpret_cast<float*>((char*)ws.p[l] + loss_byte_off);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float m = -INFINITY;
  for (int j = threadIdx.x; j < K; j += 256) m = fmaxf(m, ldf(zn + j));
  m = wave_max(m);
  if (lane == 0) red[wave] = m;
  __syncthreads();
  m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float sum = 0.f;
  for (int j = threadIdx.x; j < K; j += 256) sum += expf(ldf(zn + j) - m);
  sum = wave_sum(sum);
  if (lane == 0) red[wave] = sum;
  __syncthreads();
  sum = (red[0] + red[1]) + (red[2] + red[3]);
  const int y = ((const int32_t*)labels.p[l])[n];
  const float inv = 1.0f / sum, invN = 1.0f / (float)N;
  for (int j = threadIdx.x; j < K; j += 256) stf(dz + j, (expf(ldf(zn + j) - m) * inv - (j == y ? 1.f : 0.f)) * invN);
  if (threadIdx.x == 0) img_loss[n] = (y >= 0 && y < K) ? -(ldf(zn + y) - m - logf(sum)) : NAN;   // a bad label poisons the loss
}

__global__ void loss_mean_kernel(PtrTab ws, size_t loss_byte_off, int N, float* loss_out) {
  const int l = blockIdx.x;
  if (threadIdx.x != 0) return;
  const float* img_loss = reinterpret_cast<const float*>((const char*)ws.p[l] + loss_byte_off);
  float tot = 0.f;
  for (int n = 0; n < N; n++) tot += img_loss[n];
  loss_out[l] = tot / (float)N;
}

hipError_t launch_softmax_ce(bool is_bf16, bool z_f32, const PtrTab& ws, const CPtrTab& labels, size_t z_off, size_t dz_off,
                             size_t loss_byte_off, int N, int K, float* loss_out, int count, hipStream_t s) {
  dim3 g((unsigned)N, 1, (unsigned)count);
  if (is_bf16 && z_f32) hipLaunchKernelGGL((softmax_ce_kernel<bf16_t, float>), g, dim3(256), 0, s, ws, labels, z_off, dz_off, loss_byte_off, N, K);
  else if (is_bf16) hipLaunchKernelGGL((softmax_ce_kernel<bf16_t, bf16_t>), g, dim3(256), 0, s, ws, labels, z_off, dz_off, loss_byte_off, N, K);
  else hipLaunchKernelGGL((softmax_ce_kernel<float, float>), g, dim3(256), 0, s, ws, labels, z_off, dz_off, loss_byte_off, N, K);
  if (loss_out) hipLaunchKernelGGL(loss_mean_kernel, dim3(count), dim3(64), 0, s, ws, loss_byte_off, N, loss_out);
  return hipGetLastError();
}

// ------------------------------------------------------------------ evaluation: rank of the true class
// rank[n] = number of classes ordered before the label's class when scores are sorted in descending order (equal
// scores: lower class index first).  rank < k  <=>  the label is among the k best: top-1 / top-5 errors (Section 4.3)
// are counts of rank >= 1 / rank >= 5.  A label outside [0, K) gets rank K.  One workgroup per image.
template <typename T, typename Z>
__global__ __launch_bounds__(256) void label_rank_kernel(PtrTab ws, CPtrTab labels, size_t z_off, int N, int K, int32_t* rank_out) {
  __shared__ int red[4];
  const int l = blockIdx.z, n = blockIdx.x;
  const Z* zn = reinterpret_cast<const Z*>((const T*)ws.p[l] + z_off) + (int64_t)n * K;
  const int y = ((const int32_t*)labels.p[l])[n];
  const bool ok = y >= 0 && y < K;
  const float zy = ok ? ldf(zn + y) : 0.f;
  int cnt = 0;
  for (int j = threadIdx.x; j < K; j += 256) {
    const float zj = ldf(zn + j);
    cnt += (zj > zy || (zj == zy && j < y)) ? 1 : 0;
  }
  for (int o = 32; o > 0; o >>= 1) cnt += __shfl_down(cnt, o, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = cnt;
  __syncthreads();
  if (threadIdx.x == 0) rank_out[(int64_t)l * N + n] = ok ? (red[0] + red[1]) + (red[2] + red[3]) : K;
}

hipError_t launch_label_rank(bool is_bf16, bool z_f32, const PtrTab& ws, const CPtrTab& labels, size_t z_off, int N, int K,
                             int32_t* rank_out, int count, hipStream_t s) {
  dim3 g((unsigned)N, 1, (unsigned)count);
  if (is_bf16 && z_f32) hipLaunchKernelGGL((label_rank_kernel<bf16_t, float>), g, dim3(256), 0, s, ws, labels, z_off, N, K, rank_out);
  else if (is_bf16) hipLaunchKernelGGL((label_rank_kernel<bf16_t, bf16_t>), g, dim3(256), 0, s, ws, labels, z_off, N, K, rank_out);
  else hipLaunchKernelGGL((label_rank_kernel<float, float>), g, dim3(256), 0, s, ws, labels, z_off, N, K, rank_out);
  return hipGetLastError();
}

// ------------------------------------------------------------------ stacking the mini-batches of several learners
// Learners that read the same weight version take a fully connected layer as ONE matrix product on their stacked
// mini-batches: member k's rows ([bytes_per_member] at byte offset member_off of its workspace) are copied to / from rows
// k * bytes_per_member of a staging area.  16-byte pieces; blockIdx.z = member.
__global__ __launch_bounds__(256) void stack_rows_kernel(PtrTab members, size_t member_off, char* stage, int64_t bytes_per_member,
                                                         int to_stage) {
  char* own = (char*)members.p[blockIdx.z] + member_off;
  char* stg = stage + (int64_t)blockIdx.z * bytes_per_member;
  const uint4* src = reinterpret_cast<const uint4*>(to_stage ? own : stg);
  uint4* dst = reinterpret_cast<uint4*>(to_stage ? stg : own);
  const int64_t n = bytes_per_member >> 4;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) dst[i] = src[i];
}

hipError_t launch_stack_rows(const PtrTab& members, int count, size_t member_off_bytes, void* stage, int64_t bytes_per_member,
                             bool to_stage, hipStream_t s) {
  if (bytes_per_member <= 0 || (bytes_per_member & 15) || (member_off_bytes & 15)) return hipErrorInvalidValue;
  const int64_t n = bytes_per_member >> 4;
  const unsigned blocks = (unsigned)((n + 255) / 256 < 256 ? (n + 255) / 256 : 256);
  hipLaunchKernelGGL(stack_rows_kernel, dim3(blocks, 1, (unsigned)count), dim3(256), 0, s, members, member_off_bytes, (char*)stage,
                     bytes_per_member, to_stage ? 1 : 0);
  return hipGetLastError();
}

// ------------------------------------------------------------------ fully connected weight gradient as factors
// The weight gradient of a fully connected layer over a mini-batch of N images is the rank-N product
// dW[o][i] = sum_n dy[n][o] x[n][i].  Instead of writing out * in values, keep the factors, both with the images
// innermost: x transposed to [in][NP] and dy transposed to [out][NP] (NP = N rounded up to 8, zero-filled), so that the
// update kernel reads the N values of one unit as contiguous 16-byte pieces (the k-contiguous operands of an MFMA).
// The bias gradient db[o] = sum_n dy[n][o] is written out.
__global__ __launch_bounds__(256) void fc_save_factors_kernel(PtrTab ws, PtrTab grads, size_t x_off, size_t dy_off, size_t fx_off,
                                                              size_t fdy_off, int64_t b_off, int N, int in, int out, int NP) {
  const bf16_t* x = (const bf16_t*)ws.p[blockIdx.z] + x_off;
  const bf16_t* dy = (const bf16_t*)ws.p[blockIdx.z] + dy_off;
  bf16_t* fx = (bf16_t*)ws.p[blockIdx.z] + fx_off;
  bf16_t* fdy = (bf16_t*)ws.p[blockIdx.z] + fdy_off;
  float* db = (float*)grads.p[blockIdx.z] + b_off;
  const int xchunks = in / 8;                 // one thread turns 8 input units x 8 images around at a time
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t < xchunks) {
    for (int n0 = 0; n0 < NP; n0 += 8) {
      union { uint4 q; bf16_t h[8]; } src[8], dst[8];
#pragma unroll
      for (int k = 0; k < 8; k++)
        src[k].q = n0 + k < N ? *reinterpret_cast<const uint4*>(x + (int64_t)(n0 + k) * in + t * 8) : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
      for (int e = 0; e < 8; e++)
#pragma unroll
        for (int k = 0; k < 8; k++) dst[e].h[k] = src[k].h[e];
#pragma unroll
      for (int e = 0; e < 8; e++) *reinterpret_cast<uint4*>(fx + (int64_t)(t * 8 + e) * NP + n0) = dst[e].q;
    }
  } else if (t - xchunks < out) {
    const int o = t - xchunks;
    float sum = 0.f;
    for (int n = 0; n < NP; n++) {
      const bf16_t d = n < N ? dy[(int64_t)n * out + o] : (bf16_t)0;
      fdy[(int64_t)o * NP + n] = d;
      sum += bf2f(d);
    }
    db[o] = sum;
  }
}

// dW[o][i] = sum_n dy[n][o] x[n][i] from the saved factors (fp32 FMA in image order): the written-out gradient for the
// getters.  Four input units per thread.
__global__ __launch_bounds__(256) void fc_expand_factors_kernel(const bf16_t* __restrict__ fx, const bf16_t* __restrict__ fdy,
                                                                float* __restrict__ dw, int N, int in, int out, int NP) {
  const int64_t total4 = (int64_t)out * in / 4;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total4; t += (int64_t)gridDim.x * 256) {
    const int o = (int)(t / (in / 4)), i = (int)(t % (in / 4)) * 4;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    for (int n = 0; n < N; n++) {
      const float d = bf2f(fdy[(int64_t)o * NP + n]);
      a0 = fmaf(d, bf2f(fx[(int64_t)(i + 0) * NP + n]), a0);
      a1 = fmaf(d, bf2f(fx[(int64_t)(i + 1) * NP + n]), a1);
      a2 = fmaf(d, bf2f(fx[(int64_t)(i + 2) * NP + n]), a2);
      a3 = fmaf(d, bf2f(fx[(int64_t)(i + 3) * NP + n]), a3);
    }
    *reinterpret_cast<float4*>(dw + (int64_t)o * in + i) = make_float4(a0, a1, a2, a3);
  }
}

hipError_t launch_fc_save_factors(const PtrTab& ws, const PtrTab& grads, size_t x_off, size_t dy_off, size_t fx_off, size_t fdy_off,
                                  int64_t b_off, int N, int in, int out, int NP, int count, hipStream_t s) {
  const int work = in / 8 + out;
  hipLaunchKernelGGL(fc_save_factors_kernel, dim3((unsigned)((work + 255) / 256), 1, (unsigned)count), dim3(256), 0, s, ws, grads, x_off,
                     dy_off, fx_off, fdy_off, b_off, N, in, out, NP);
  return hipGetLastError();
}

hipError_t launch_fc_expand_factors(const void* fx, const void* fdy, float* dw, int N, int in, int out, int NP, hipStream_t s) {
  const int64_t total4 = (int64_t)out * in / 4;
  const unsigned blocks = (unsigned)((total4 + 255) / 256 < 8192 ? (total4 + 255) / 256 : 8192);
  hipLaunchKernelGGL(fc_expand_factors_kernel, dim3(blocks), dim3(256), 0, s, (const bf16_t*)fx, (const bf16_t*)fdy, dw, N, in, out, NP);
  return hipGetLastError();
}

}  // namespace sasgd
