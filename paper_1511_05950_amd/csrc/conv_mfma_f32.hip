// fp32 MFMA implicit-GEMM kernels (v_mfma_f32_32x32x2_f32: exact fp32 products, fp32 accumulation) for the
// fp32-compute configurations of calcGradient (Section 2.1; layer shapes of Section 4.1).  Same GEMM views as
// the bf16 kernels; everything is simpler because the fp32 matrix rate is 16x lower and neither LDS nor the
// vector cache limits it:
//   * activations NHWC fp32, gathered as 16-byte chunks of 4 channels through hardware-bounds-checked buffer loads;
//   * filters are read straight from the flat parameter vector [K][C][kh][kw] with 4-byte loads (no packed copy),
//     for the forward pass as B[n][(tap, c)] and for the input gradient as B[c][(flipped tap, n)];
//   * wgrad keeps its two tiles as they lie in memory (rows = output positions): one lane needs one scalar per
//     MFMA operand, so no transpose is involved; the bias gradient is an extra im2col column of ones.
// Block tile 128 x 32 (forward / dgrad) and 32 x 128 (wgrad), four wavefronts of one 32 x 32 MFMA block each.
#include <algorithm>

#include "dev_common.hpp"
#include "kernels.hpp"

namespace sasgd {

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef int v4i_t __attribute__((ext_vector_type(4)));
constexpr uint32_t kOOB = 0x80000000u;     // buffer offset beyond any tensor: the load returns zeros
constexpr int FK = 16;                     // contraction elements per step
constexpr int FLD = 20;                    // LDS row stride in floats (80 bytes, 16-byte aligned)

__device__ __forceinline__ uint32_t fdiv(uint32_t n, int d, uint32_t magic) { return d == 1 ? n : __umulhi(n, magic); }

// dgrad == 0: y[m][n] = sum_k im2col(x)[m][k] W(n, k)          (v = the layer itself)
// dgrad == 1: dx[m][c] = sum_k im2col(dy)[m][k] W^T(c, k)      (g describes the gather over dy, v the forward layer)
__global__ __launch_bounds__(256) void igemm_f32_kernel(PtrTab ws, CPtrTab wts, IGemm g, VConv v, Epilogue ep, int64_t w_off,
                                                        int dgrad) {
  __shared__ __attribute__((aligned(16))) float lds[2 * (128 + 32) * FLD];
  const int z = blockIdx.z / g.splits, sp = blockIdx.z % g.splits;
  const float* act = (const float*)ws.p[z] + g.a_off;
  const float* W = (const float*)wts.p[z] + w_off;
  const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc((void*)act, 0, (int)g.a_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void*)W, 0, (int)g.b_bytes, 0x00020000);
  const int m0 = blockIdx.x * 128, n0 = blockIdx.y * 32;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  // A loader: chunk column cc (4 floats) of rows lrow and lrow + 64
  const int cc = tid & 3, lrow = tid >> 2;
  int row_off[2], row_oh[2], row_ow[2];
#pragma unroll
  for (int i = 0; i < 2; i++) {
    const int m = m0 + lrow + 64 * i;
    const bool valid = m < g.M;
    const uint32_t mm = valid ? (uint32_t)m : 0u;
    const uint32_t rest = fdiv(mm, g.OW, g.mg_ow);
    const int ow = (int)(mm - rest * (uint32_t)g.OW);
    const uint32_t n = fdiv(rest, g.OH, g.mg_oh);
    const int oh = (int)(rest - n * (uint32_t)g.OH);
    row_oh[i] = valid ? oh - g.pad : -0x40000000;
    row_ow[i] = ow - g.pad;
    row_off[i] = (int)(((((int64_t)n * g.H + (oh - g.pad)) * g.W + (ow - g.pad)) * g.C) * 4);
  }
  // B loader: row brow (output column n0 + brow), contraction elements bk and bk + 8 of every step
  const int brow = tid >> 3, bk = tid & 7;
  const int kk2 = v.ks * v.ks;

  v4i_t ra[2];
  float rb[2];
  auto load = [&](int ks) {
    const int q = ks * 4 + cc;
    const uint32_t tap = fdiv((uint32_t)q, g.CPT, g.mg_cpt);
    const int c4 = q - (int)tap * g.CPT;
    const int kh = (int)fdiv(tap, g.ks, g.mg_ks), kw = (int)tap - kh * g.ks;
    const int koff = ((kh * g.W + kw) * g.C + c4 * 4) * 4;
    const bool qok = q < g.Kchunks;
#pragma unroll
    for (int i = 0; i < 2; i++) {
      const bool ok = qok && (unsigned)(row_oh[i] + kh) < (unsigned)g.H && (unsigned)(row_ow[i] + kw) < (unsigned)g.W;
      ra[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, ok ? row_off[i] + koff : (int)kOOB, 0, 0);
    }
#pragma unroll
    for (int h = 0; h < 2; h++) {
      const int k = ks * FK + bk + 8 * h;           // im2col column = tap * C + channel
      const int r = n0 + brow;
      int64_t src = -1;
      if (k < g.Kchunks * 4 && r < g.Ncols) {
        const int t = k / g.C, ch = k - t * g.C;
        src = dgrad ? filter_src(v, ch, kk2 - 1 - t, r) : filter_src(v, r, t, ch);
      }
      rb[h] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc_w, src >= 0 ? (int)(src * 4) : (int)kOOB, 0, 0));
    }
  };
  auto store = [&](int buf) {
    float* A = lds + buf * (128 + 32) * FLD;
    float* B = A + 128 * FLD;
#pragma unroll
    for (int i = 0; i < 2; i++) *reinterpret_cast<v4i_t*>(A + (lrow + 64 * i) * FLD + cc * 4) = ra[i];
    B[brow * FLD + bk] = rb[0];
    B[brow * FLD + bk + 8] = rb[1];
  };

  floatx16 acc;
#pragma unroll
  for (int r = 0; r < 16; r++) acc[r] = 0.f;
  const int all_steps = (g.Kchunks + 3) / 4;
  const int per = (all_steps + g.splits - 1) / g.splits;
  const int ks_begin = sp * per, ksteps = min(all_steps, ks_begin + per);
  if (ks_begin < ksteps) {
    load(ks_begin);
    store(0);
  }
  __syncthreads();
  for (int ks = ks_begin; ks < ksteps; ks++) {
    const int buf = (ks - ks_begin) & 1;
    if (ks + 1 < ksteps) load(ks + 1);
    const float* A = lds + buf * (128 + 32) * FLD + (wave * 32 + (lane & 31)) * FLD + 8 * (lane >> 5);
    const float* B = lds + buf * (128 + 32) * FLD + 128 * FLD + (lane & 31) * FLD + 8 * (lane >> 5);
    // contraction element order inside a step: lanes 0-31 take k = 0..7, lanes 32-63 take k = 8..15
#pragma unroll
    for (int kk = 0; kk < 8; kk++) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(A[kk], B[kk], acc, 0, 0, 0);
    if (ks + 1 < ksteps) store(buf ^ 1);
    __syncthreads();
  }

  const int n = n0 + (lane & 31);
  if (n >= g.Ncols) return;
  if (g.splits > 1) {   // raw partial sums [split][m][n]; igemm_finish_f32_kernel adds them in split order
    float* part = reinterpret_cast<float*>((char*)ws.p[z] + g.scratch_off) + (int64_t)sp * g.M * g.Ncols;
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int m = m0 + wave * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      if (m < g.M) part[(int64_t)m * g.Ncols + n] = acc[r];
    }
    return;
  }
  float* out = (float*)ws.p[z] + ep.out_off;
  const float* mask = (const float*)ws.p[z] + ep.mask_off;
  const float* bias = (const float*)wts.p[z] + ep.bias_off;
  const float bv = ep.has_bias ? bias[n] : 0.f;
#pragma unroll
  for (int r = 0; r < 16; r++) {
    const int m = m0 + wave * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
    if (m >= g.M) continue;
    float val = acc[r] + bv;
    if (ep.relu) val = fmaxf(val, 0.f);
    const int64_t o = (int64_t)m * g.Ncols + n;
    if (ep.use_mask && !(mask[o] > 0.f)) val = 0.f;
    out[o] = val;
  }
}

// Sum of the partial tiles of a split contraction, in split order, then bias, ReLU and the ReLU mask of the input
// gradient: the epilogue of igemm_f32_kernel.
__global__ __launch_bounds__(256) void igemm_finish_f32_kernel(PtrTab ws, CPtrTab wts, IGemm g, Epilogue ep) {
  const int z = blockIdx.z;
  const float* part = reinterpret_cast<const float*>((const char*)ws.p[z] + g.scratch_off);
  float* out = (float*)ws.p[z] + ep.out_off;
  const float* mask = (const float*)ws.p[z] + ep.mask_off;
  const float* bias = (const float*)wts.p[z] + ep.bias_off;
  const uint32_t total = (uint32_t)((int64_t)g.M * g.Ncols);
  for (uint32_t o = blockIdx.x * 256 + threadIdx.x; o < total; o += gridDim.x * 256) {
    float val = 0.f;
#pragma unroll 4
    for (int sp = 0; sp < g.splits; sp++) val += part[(size_t)sp * total + o];
    if (ep.has_bias) val += bias[o % (uint32_t)g.Ncols];
    if (ep.relu) val = fmaxf(val, 0.f);
    if (ep.use_mask && !(mask[o] > 0.f)) val = 0.f;
    out[o] = val;
  }
}

// g.splits > 1 divides the contraction among that many workgroups per tile (mini-batches of a few images give a
// handful of tiles, each a serial chain of hundreds of fp32 MFMAs); needs g.scratch_off and M * Ncols < 2^32.
hipError_t launch_igemm_f32(const PtrTab& ws, const CPtrTab& wts, const IGemm& g, const VConv& v, const Epilogue& ep, int64_t w_off,
                            bool dgrad, int count, hipStream_t s) {
  if (g.C % 4 || g.splits < 1 || (int64_t)count * g.splits > 65535) return hipErrorInvalidValue;
  dim3 grid((unsigned)((g.M + 127) / 128), (unsigned)((g.Ncols + 31) / 32), (unsigned)(count * g.splits));
  hipLaunchKernelGGL(igemm_f32_kernel, grid, dim3(256), 0, s, ws, wts, g, v, ep, w_off, dgrad ? 1 : 0);
  if (g.splits > 1) {
    const int64_t total = (int64_t)g.M * g.Ncols;
    const unsigned blocks = (unsigned)std::min<int64_t>((total + 255) / 256, 2048);
    hipLaunchKernelGGL(igemm_finish_f32_kernel, dim3(blocks, 1, (unsigned)count), dim3(256), 0, s, ws, wts, g, ep);
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------ weight + bias gradient
// dW tile [32 output channels][128 im2col columns]; contraction over output positions m in steps of 16.
__global__ __launch_bounds__(256) void igemm_wgrad_f32_kernel(PtrTab ws, PtrTab grads, IGemm g, VConv v, size_t dy_off, int64_t w_off,
                                                              int64_t b_off) {
  constexpr int LA = 32 + 4, LB = 128 + 4;     // row strides (floats) of the dy and im2col tiles, 16-byte aligned
  __shared__ __attribute__((aligned(16))) float lds[2 * FK * (LA + LB)];
  const int z = blockIdx.z / g.splits, sp = blockIdx.z % g.splits;
  const float* x = (const float*)ws.p[z] + g.a_off;
  const float* dy = (const float*)ws.p[z] + dy_off;
  const float* consts = (const float*)ws.p[z] + g.zero_off;
  const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc((void*)x, 0, (int)g.a_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_dy = __builtin_amdgcn_make_buffer_rsrc((void*)dy, 0, (int)((int64_t)g.M * g.Ncols * 4), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_c = __builtin_amdgcn_make_buffer_rsrc((void*)consts, 0, 1024, 0x00020000);
  const int n0 = blockIdx.x * 32, k0 = blockIdx.y * 128;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // dy tile: 16 rows x 8 chunks = 128 chunk loads (threads 0..127); im2col tile: 16 rows x 32 chunks = 512 (2 per thread)
  const int ar = tid >> 3, ac = tid & 7;
  const int br = tid >> 5, bc = tid & 31;      // rows br and br + 8
  v4i_t ra, rb[2];
  auto load = [&](int ms) {
    {
      const int m = ms * FK + ar, n = n0 + ac * 4;
      const bool ok = tid < 128 && m < g.M && n < g.Ncols;
      ra = __builtin_amdgcn_raw_buffer_load_b128(rsrc_dy, ok ? (int)(((int64_t)m * g.Ncols + n) * 4) : (int)kOOB, 0, 0);
    }
    const int q = k0 / 4 + bc;
    const uint32_t tap = fdiv((uint32_t)q, g.CPT, g.mg_cpt);
    const int c4 = q - (int)tap * g.CPT;
    const int kh = (int)fdiv(tap, g.ks, g.mg_ks), kw = (int)tap - kh * g.ks;
#pragma unroll
    for (int h = 0; h < 2; h++) {
      const int m = ms * FK + br + 8 * h;
      const bool valid = m < g.M;
      const uint32_t mm = valid ? (uint32_t)m : 0u;
      const uint32_t rest = fdiv(mm, g.OW, g.mg_ow);
      const int ow = (int)(mm - rest * (uint32_t)g.OW) - g.pad;
      const uint32_t n = fdiv(rest, g.OH, g.mg_oh);
      const int oh = (int)(rest - n * (uint32_t)g.OH) - g.pad;
      const int ih = oh + kh, iw = ow + kw;
      const bool ok = valid && q < g.Kchunks && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W;
      const int off = (int)(((((int64_t)n * g.H + ih) * g.W + iw) * g.C + c4 * 4) * 4);
      if (q == g.Kchunks)   // the bias column: the constant chunk {1, 0, 0, 0} for every real output position
        rb[h] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_c, valid ? 512 : (int)kOOB, 0, 0);
      else
        rb[h] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, ok ? off : (int)kOOB, 0, 0);
    }
  };
  auto store = [&](int buf) {
    float* A = lds + buf * FK * (LA + LB);
    float* B = A + FK * LA;
    if (tid < 128) *reinterpret_cast<v4i_t*>(A + ar * LA + ac * 4) = ra;
#pragma unroll
    for (int h = 0; h < 2; h++) *reinterpret_cast<v4i_t*>(B + (br + 8 * h) * LB + bc * 4) = rb[h];
  };

  floatx16 acc;
#pragma unroll
  for (int r = 0; r < 16; r++) acc[r] = 0.f;
  const int all_steps = (g.M + FK - 1) / FK;
  const int per = (all_steps + g.splits - 1) / g.splits;
  const int ms_begin = sp * per, msteps = min(all_steps, ms_begin + per);
  if (ms_begin < msteps) {
    load(ms_begin);
    store(0);
  }
  __syncthreads();
  for (int ms = ms_begin; ms < msteps; ms++) {
    const int buf = (ms - ms_begin) & 1;
    if (ms + 1 < msteps) load(ms + 1);
    const float* A = lds + buf * FK * (LA + LB) + 8 * (lane >> 5) * LA + (lane & 31);
    const float* B = lds + buf * FK * (LA + LB) + FK * LA + 8 * (lane >> 5) * LB + wave * 32 + (lane & 31);
#pragma unroll
    for (int kk = 0; kk < 8; kk++) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(A[kk * LA], B[kk * LB], acc, 0, 0, 0);
    if (ms + 1 < msteps) store(buf ^ 1);
    __syncthreads();
  }

  const int kcols = g.Kchunks * 4;
  const int k = k0 + wave * 32 + (lane & 31);
  if (k > kcols) return;
  if (g.splits > 1) {   // partial sums [split][n][kcols + 4]; wgrad_finish_f32_kernel adds them and writes the gradient
    const int ldk = kcols + 4;
    float* part = reinterpret_cast<float*>((char*)ws.p[z] + g.scratch_off) + (int64_t)sp * g.Ncols * ldk;
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int n = n0 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      if (n < g.Ncols) part[(int64_t)n * ldk + k] = acc[r];
    }
    return;
  }
  float* dw = (float*)grads.p[z] + w_off;
  float* db = (float*)grads.p[z] + b_off;
  const int tap = k / g.C, cp = k - tap * g.C;
#pragma unroll
  for (int r = 0; r < 16; r++) {
    const int n = n0 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
    if (n >= g.Ncols) continue;
    if (k == kcols) { db[n] = acc[r]; continue; }
    const int64_t dst = filter_src(v, n, tap, cp);
    if (dst >= 0) dw[dst] = acc[r];
  }
}

// Sum of the partial weight gradients in split order; element (n, k) goes to its place in the flat gradient
// (column kcols is the bias gradient).
__global__ __launch_bounds__(256) void wgrad_finish_f32_kernel(PtrTab ws, PtrTab grads, IGemm g, VConv v, int64_t w_off, int64_t b_off) {
  const int z = blockIdx.z;
  const int kcols = g.Kchunks * 4, ldk = kcols + 4;
  const float* part = reinterpret_cast<const float*>((const char*)ws.p[z] + g.scratch_off);
  float* dw = (float*)grads.p[z] + w_off;
  float* db = (float*)grads.p[z] + b_off;
  const int64_t split_stride = (int64_t)g.Ncols * ldk;
  const int total = g.Ncols * (kcols + 1);
  for (int idx = blockIdx.x * 256 + threadIdx.x; idx < total; idx += gridDim.x * 256) {
    const int n = idx / (kcols + 1), k = idx - n * (kcols + 1);
    float val = 0.f;
#pragma unroll 4
    for (int sp = 0; sp < g.splits; sp++) val += part[sp * split_stride + (int64_t)n * ldk + k];
    if (k == kcols) { db[n] = val; continue; }
    const int tap = k / g.C, cp = k - tap * g.C;
    const int64_t dst = filter_src(v, n, tap, cp);
    if (dst >= 0) dw[dst] = val;
  }
}

// g.splits > 1 divides the output positions among that many workgroups per tile (needs g.scratch_off).
hipError_t launch_igemm_wgrad_f32(const PtrTab& ws, const PtrTab& grads, const IGemm& g, const VConv& v, size_t dy_off, int64_t w_off,
                                  int64_t b_off, int count, hipStream_t s) {
  if (g.C % 4 || g.Ncols % 4 || g.splits < 1 || (int64_t)count * g.splits > 65535) return hipErrorInvalidValue;
  const int cols = g.Kchunks * 4 + 1;
  dim3 grid((unsigned)((g.Ncols + 31) / 32), (unsigned)((cols + 127) / 128), (unsigned)(count * g.splits));
  hipLaunchKernelGGL(igemm_wgrad_f32_kernel, grid, dim3(256), 0, s, ws, grads, g, v, dy_off, w_off, b_off);
  if (g.splits > 1) {
    const int total = g.Ncols * cols;
    hipLaunchKernelGGL(wgrad_finish_f32_kernel, dim3((unsigned)std::min((total + 255) / 256, 1024), 1, (unsigned)count), dim3(256), 0, s,
                       ws, grads, g, v, w_off, b_off);
  }
  return hipGetLastError();
}

}  // namespace sasgd
