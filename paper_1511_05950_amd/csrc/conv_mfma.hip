// bf16 MFMA implicit-GEMM kernels for calcGradient's convolutions and fully connected layers
// (Section 2.1 learner step; layer shapes of Section 4.1), written for gfx950 (CDNA4):
// v_mfma_f32_32x32x16_bf16 tiles, fp32 accumulation, LDS-staged im2col tiles, 64-wide wavefronts.
//
// GEMM views (activations NHWC bf16, "chunk" = 8 consecutive channels = 16 bytes):
//   forward  y[m][n]  = sum_k im2col(x)[m][k] * Wp[n][k]      m = (image, oh, ow), k = (kh, kw, c)
//   dgrad    dx[m][c] = sum_k im2col(dy)[m][k] * Wt[c][k]     the same kernel on dy with flipped, transposed
//                                                             filters (stride 1), or, for fully connected
//                                                             layers, with the B operand read transposed
//   wgrad    dW[n][k] = sum_m dy[m][n] * im2col(x)[m][k]      both operands are contraction-major in memory;
//                                                             they are staged as they lie and read with the
//                                                             LDS transpose load (ds_read_b64_tr_b16)
// The im2col matrix is never materialised: a tile loader gathers 16-byte chunks straight from the NHWC
// tensor (zero outside the image).  Only stride-1 windows are handled here; a strided first layer is
// turned into a stride-1 layer by a space-to-depth re-layout of the input (see pack_input).
#include <algorithm>
#include <type_traits>
#include "dev_common.hpp"
#include "kernels.hpp"

namespace sasgd {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short shortx4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

constexpr int BK = 32;           // contraction elements per step (4 chunks)
constexpr int LDA = BK + 8;      // row stride (elements) of k-contiguous LDS tiles: 80 B, conflict-free 16 B reads

// ------------------------------------------------------------------ filter packing (once per weight version)
// Filters are stored in MFMA operand ("fragment") order so that a wavefront fetches the B operand of one
// 32x32x16 MFMA as one contiguous 1 KiB read, straight into registers:
//   frag[(nb * KB16 + kb) * 512 + lane * 8 + t] = B[row 32 nb + lane%32][k = 16 kb + 8 (lane/32) + t]
// fwd: B = Wp[n][tap][cp] (k = tap * C + cp, Kp = padded ks*ks*C);   rows beyond K and k beyond the filter are zero
// bwd: B = Wt[c][tap'][n] (k = tap' * K + n, tap' = flipped tap, Kpt = padded ks*ks*K), stride-1 layers only
// One thread produces one lane's 16-byte chunk (8 consecutive k of one row); index arithmetic is 32-bit.
__global__ __launch_bounds__(256) void pack_filters_kernel(PackVersions pv, PackTable t) {
  const bf16_t* __restrict__ flat = (const bf16_t*)pv.flat[blockIdx.y];      // blockIdx.y = weight version
  bf16_t* __restrict__ packed = (bf16_t*)pv.packed[blockIdx.y];
  const int64_t chunks = t.total >> 3;
  for (int64_t gc = (int64_t)blockIdx.x * 256 + threadIdx.x; gc < chunks; gc += (int64_t)gridDim.x * 256) {
    int li = 0;                                   // layer this chunk belongs to
    while (li + 1 < t.count && gc * 8 >= t.job[li + 1].start) li++;
    const PackJob& jb = t.job[li];
    const VConv& v = jb.v;
    const uint32_t i = (uint32_t)(gc * 8 - jb.start);
    const uint32_t nf = (uint32_t)((v.K + 31) & ~31) * (uint32_t)jb.Kp;
    const bool fwd = i < nf;
    const uint32_t e = fwd ? i : i - nf;
    const uint32_t KB16 = (uint32_t)(fwd ? jb.Kp : jb.Kpt) / 16u;
    const uint32_t lane = (e >> 3) & 63u, blk = e >> 9;
    const uint32_t rb = blk / KB16, kb = blk - rb * KB16;
    const int row = (int)(32u * rb + (lane & 31u));
    const uint32_t k0 = 16u * kb + 8u * (lane >> 5);
    const int taps = v.ks * v.ks;
    union { bf16_t h[8]; uint4 q; } out;
    out.q = make_uint4(0u, 0u, 0u, 0u);
    if (fwd) {
      // k = tap * C + cp; C is a multiple of 8, so the 8 elements share the tap
      const int tap = (int)(k0 / (uint32_t)v.C), cp0 = (int)(k0 - (uint32_t)tap * (uint32_t)v.C);
      if (row < v.K && tap < taps) {
#pragma unroll
        for (int j = 0; j < 8; j++) {
          const int64_t src = filter_src(v, row, tap, cp0 + j);
          if (src >= 0) out.h[j] = flat[jb.w_off + src];
        }
      }
      *reinterpret_cast<uint4*>(packed + jb.fwd_off + e) = out.q;
    } else {
      // k = tap' * K + n; K is a multiple of 8
      const int tap = (int)(k0 / (uint32_t)v.K), n0 = (int)(k0 - (uint32_t)tap * (uint32_t)v.K);
      if (row < v.C && tap < taps) {
#pragma unroll
        for (int j = 0; j < 8; j++) {
          const int64_t src = filter_src(v, n0 + j, taps - 1 - tap, row);   // flipped tap (ks-1-kh, ks-1-kw)
          if (src >= 0) out.h[j] = flat[jb.w_off + src];
        }
      }
      *reinterpret_cast<uint4*>(packed + jb.bwd_off + e) = out.q;
    }
  }
}

// Layers with a multiple of 32 input and 16 output channels and no re-layout of the first layer: the repack is a
// transposition ([n][c][tap] -> [n][tap][c] and [c][tap'][n]), done through LDS so that both the reads of the flat
// filter and the writes of the fragments are contiguous.
//   forward block  (32 output channels, 16 input channels): reads 32 runs of 16 T elements, writes T fragment blocks
//   backward block (32 input channels, 16 output channels): reads 16 runs of 32 T elements, writes T fragment blocks
// Fragment blocks of the zero padding (k beyond the filter) are never written: they keep the zeros the ring was
// created with.
struct PackFastJob {
  int64_t w_off, fwd_off, bwd_off;
  int C, K, T, KB16, KB16t;          // T = taps; fragment k-blocks per row of the two copies
  int first_block, fwd_blocks;       // workgroups [first_block, next job's first_block): forward ones first
};
struct PackFastTable {
  PackFastJob job[kMaxPackJobs];
  int count;
};
constexpr int kPackMaxTaps = 25;

__global__ __launch_bounds__(256) void pack_filters_lds_kernel(PackVersions pv, PackFastTable t) {
  const bf16_t* __restrict__ flat = (const bf16_t*)pv.flat[blockIdx.y];      // blockIdx.y = weight version
  bf16_t* __restrict__ packed = (bf16_t*)pv.packed[blockIdx.y];
  __shared__ __attribute__((aligned(16))) bf16_t tile[32 * 16 * kPackMaxTaps];
  int li = 0;
  while (li + 1 < t.count && (int)blockIdx.x >= t.job[li + 1].first_block) li++;
  const PackFastJob& jb = t.job[li];
  const int b = blockIdx.x - jb.first_block;
  const int T = jb.T, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row = lane & 31, h = lane >> 5;
  const bf16_t* W = flat + jb.w_off;
  if (b < jb.fwd_blocks) {
    const int groups = jb.C / 16, rb = b / groups, cg = b - rb * groups;
    const int run = 16 * T;                                  // contiguous elements of one output channel
    for (int ch = tid; ch < 64 * T; ch += 256) {             // 16-byte pieces: 2 T per run
      const int r = ch / (2 * T), rem = (ch - r * 2 * T) * 8, n = 32 * rb + r;
      uint4 q = make_uint4(0u, 0u, 0u, 0u);
      if (n < jb.K) q = *reinterpret_cast<const uint4*>(W + ((int64_t)n * jb.C + 16 * cg) * T + rem);
      *reinterpret_cast<uint4*>(tile + r * run + rem) = q;
    }
    __syncthreads();
    for (int tap = wave; tap < T; tap += 4) {
      union { bf16_t e[8]; uint4 q; } o;
#pragma unroll
      for (int j = 0; j < 8; j++) o.e[j] = tile[row * run + (8 * h + j) * T + tap];
      const int kb = tap * groups + cg;
      *reinterpret_cast<uint4*>(packed + jb.fwd_off + ((int64_t)rb * jb.KB16 + kb) * 512 + lane * 8) = o.q;
    }
  } else {
    const int bb = b - jb.fwd_blocks;
    const int groups = jb.K / 16, cb = bb / groups, ng = bb - cb * groups;
    const int run = 32 * T;                                  // contiguous elements of 32 input channels of one filter
    for (int ch = tid; ch < 64 * T; ch += 256) {             // 16-byte pieces: 4 T per run (the 32 channels all exist)
      const int nn = ch / (4 * T), rem = (ch - nn * 4 * T) * 8;
      *reinterpret_cast<uint4*>(tile + nn * run + rem) =
          *reinterpret_cast<const uint4*>(W + ((int64_t)(16 * ng + nn) * jb.C + 32 * cb) * T + rem);
    }
    __syncthreads();
    for (int tap = wave; tap < T; tap += 4) {                // tap' of the flipped filter
      union { bf16_t e[8]; uint4 q; } o;
#pragma unroll
      for (int j = 0; j < 8; j++) o.e[j] = tile[(8 * h + j) * run + row * T + (T - 1 - tap)];
      const int kb = tap * groups + ng;
      *reinterpret_cast<uint4*>(packed + jb.bwd_off + ((int64_t)cb * jb.KB16t + kb) * 512 + lane * 8) = o.q;
    }
  }
}

hipError_t launch_pack_filters(const PackVersions& pv, int versions, const PackTable& t, hipStream_t s) {
  if (t.count == 0 || t.total == 0 || versions < 1) return hipSuccess;
  if (versions > kMaxPackVersions) return hipErrorInvalidValue;
  PackTable slow;
  PackFastTable fast;
  slow.count = 0; slow.total = 0;
  fast.count = 0;
  int blocks_fast = 0;
  for (int k = 0; k < t.count; k++) {
    const PackJob& jb = t.job[k];
    const VConv& v = jb.v;
    const int T = v.ks * v.ks;
    if (v.s2d == 1 && v.C == v.Creal && v.ks == v.ksr && v.C % 32 == 0 && v.K % 16 == 0 && T <= kPackMaxTaps && jb.Kpt > 0 && jb.w_off % 8 == 0) {
      PackFastJob& f = fast.job[fast.count++];
      f.w_off = jb.w_off; f.fwd_off = jb.fwd_off; f.bwd_off = jb.bwd_off;
      f.C = v.C; f.K = v.K; f.T = T; f.KB16 = jb.Kp / 16; f.KB16t = jb.Kpt / 16;
      f.first_block = blocks_fast;
      f.fwd_blocks = ((v.K + 31) / 32) * (v.C / 16);
      blocks_fast += f.fwd_blocks + ((v.C + 31) / 32) * (v.K / 16);
    } else {
      PackJob& o = slow.job[slow.count++];
      o = jb;
      o.start = slow.total;
      slow.total += (int64_t)((v.K + 31) & ~31) * jb.Kp + (jb.Kpt > 0 ? (int64_t)((v.C + 31) & ~31) * jb.Kpt : 0);
    }
  }
  if (slow.count > 0) {
    const int64_t chunks = slow.total / 8;
    int blocks = (int)((chunks + 255) / 256 < 8192 ? (chunks + 255) / 256 : 8192);
    hipLaunchKernelGGL(pack_filters_kernel, dim3(blocks, (unsigned)versions), dim3(256), 0, s, pv, slow);
  }
  if (fast.count > 0)
    hipLaunchKernelGGL(pack_filters_lds_kernel, dim3((unsigned)blocks_fast, (unsigned)versions), dim3(256), 0, s, pv, fast);
  return hipGetLastError();
}

// ------------------------------------------------------------------ im2col chunk gather
// Row m of the virtual im2col matrix, chunk q (8 channels of one tap): 16 bytes from the NHWC tensor or zeros.
// All loads are unconditional (an out-of-range chunk is read from a block of zeros kept in the workspace) and all
// index arithmetic is branch-free, so the loops below are straight-line code: nothing touches a loaded value
// before the MFMAs of the current step have been issued, and the compiler can wait on exactly the loads it needs
// instead of draining the whole queue.
__device__ __forceinline__ uint32_t fastdiv(uint32_t n, int d, uint32_t magic) { return d == 1 ? n : __umulhi(n, magic); }

__device__ __forceinline__ uint4 ld16_or_zero(const bf16_t* p, bool ok, const bf16_t* zeros) {
  return *reinterpret_cast<const uint4*>(ok ? p : zeros);
}

struct RowPos {
  const bf16_t* base;   // &t[n][oh - pad][ow - pad][0]  (may point outside; only dereferenced when in range)
  int oh, ow;           // already offset by -pad
  bool valid;
};

__device__ __forceinline__ RowPos row_pos(const bf16_t* t, const IGemm& g, int m) {
  RowPos r;
  r.valid = m < g.M;
  const uint32_t mm = r.valid ? (uint32_t)m : 0u;
  const uint32_t rest = fastdiv(mm, g.OW, g.mg_ow);
  const int ow = (int)(mm - rest * (uint32_t)g.OW);
  const uint32_t n = fastdiv(rest, g.OH, g.mg_oh);
  const int oh = (int)(rest - n * (uint32_t)g.OH);
  r.oh = oh - g.pad;
  r.ow = ow - g.pad;
  r.base = t + (((int64_t)n * g.H + r.oh) * g.W + r.ow) * g.C;
  return r;
}

__device__ __forceinline__ uint4 gather_chunk(const RowPos& r, const IGemm& g, int q, const bf16_t* zeros) {
  const uint32_t tap = fastdiv((uint32_t)q, g.CPT, g.mg_cpt);
  const int c8 = q - (int)tap * g.CPT;
  const int kh = (int)fastdiv(tap, g.ks, g.mg_ks), kw = (int)tap - kh * g.ks;
  const int ih = r.oh + kh, iw = r.ow + kw;
  const bool ok = r.valid && q < g.Kchunks && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W;
  return ld16_or_zero(r.base + ((int64_t)kh * g.W + kw) * g.C + c8 * 8, ok, zeros);
}

// ------------------------------------------------------------------ forward / dgrad kernel
// Block tile BM x BN, four wavefronts each owning a WM x WN sub-tile of 32x32 MFMA blocks.
// BT = false: B rows are output columns, k-contiguous (packed filters): B[n][k], row length ldb.
// BT = true : B is stored contraction-major, B[k][n] with row length ldb (flat fully connected weights
//             used for dgrad); its tile is staged as it lies and read with the transpose load.
template <int BM, int BN, int WM, int WN, bool BT>
__global__ __launch_bounds__(256) void igemm_kernel(PtrTab ws, CPtrTab wts, IGemm g, Epilogue ep) {
  constexpr int WAVES_N = BN / WN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int LDBT = BN + (BN == 128 ? 32 : (BN == 64 ? 32 : 0));   // transposed tile: row stride = 16 (mod 64) words
  constexpr int A_ELEMS = BM * LDA;
  constexpr int B_ELEMS = BT ? BK * LDBT : BN * LDA;
  __shared__ __attribute__((aligned(16))) bf16_t lds[2 * (A_ELEMS + B_ELEMS)];

  const int z = blockIdx.z / g.splits, sp = blockIdx.z % g.splits;
  const bf16_t* act = (const bf16_t*)ws.p[z] + g.a_off;
  const bf16_t* zeros = (const bf16_t*)ws.p[z] + g.zero_off;
  const bf16_t* Bm = (const bf16_t*)wts.p[z] + g.b_off;
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;

  // loader assignment: chunk column cc (0..3) is fixed per thread, rows stride 64
  constexpr int A_LOADS = (BM * 4 + 255) / 256;
  constexpr int B_LOADS = BT ? (BK * (BN / 8) + 255) / 256 : (BN * 4 + 255) / 256;
  const int cc = tid & 3, lrow = tid >> 2;
  RowPos rp[A_LOADS];
#pragma unroll
  for (int i = 0; i < A_LOADS; i++) rp[i] = row_pos(act, g, m0 + lrow + 64 * i);

  uint4 ra[A_LOADS], rb[B_LOADS];
  auto load_regs = [&](int ks) {
#pragma unroll
    for (int i = 0; i < A_LOADS; i++) ra[i] = gather_chunk(rp[i], g, ks * 4 + cc, zeros);
    if (!BT) {
#pragma unroll
      for (int i = 0; i < B_LOADS; i++) {
        const int r = lrow + 64 * i;
        const int n = n0 + r;
        const int q = ks * 4 + cc;
        rb[i] = ld16_or_zero(Bm + (int64_t)n * g.ldb + q * 8, r < BN && n < g.Ncols && q * 8 < g.ldb, zeros);
      }
    } else {
      constexpr int CPR = BN / 8;   // chunks per tile row
#pragma unroll
      for (int i = 0; i < B_LOADS; i++) {
        const int idx = tid + 256 * i;
        const int r = idx / CPR, ch = idx % CPR;
        const int k = ks * BK + r, n = n0 + ch * 8;
        rb[i] = ld16_or_zero(Bm + (int64_t)k * g.ldb + n, r < BK && k < g.Kchunks * 8 && n < g.Ncols, zeros);
      }
    }
  };
  auto store_lds = [&](int buf) {
    bf16_t* A = lds + buf * (A_ELEMS + B_ELEMS);
    bf16_t* B = A + A_ELEMS;
#pragma unroll
    for (int i = 0; i < A_LOADS; i++)
      if (lrow + 64 * i < BM) *reinterpret_cast<uint4*>(A + (lrow + 64 * i) * LDA + cc * 8) = ra[i];
    if (!BT) {
#pragma unroll
      for (int i = 0; i < B_LOADS; i++)
        if (lrow + 64 * i < BN) *reinterpret_cast<uint4*>(B + (lrow + 64 * i) * LDA + cc * 8) = rb[i];
    } else {
      constexpr int CPR = BN / 8;
#pragma unroll
      for (int i = 0; i < B_LOADS; i++) {
        int idx = tid + 256 * i;
        int r = idx / CPR, ch = idx % CPR;
        if (r < BK) *reinterpret_cast<uint4*>(B + r * LDBT + ch * 8) = rb[i];
      }
    }
  };

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

  const int all_steps = (g.Kchunks + 3) / 4;
  const int per = (all_steps + g.splits - 1) / g.splits;
  const int ks_begin = sp * per;
  const int ksteps = min(all_steps, ks_begin + per);
  if (ks_begin < ksteps) {
    load_regs(ks_begin);
    store_lds(ks_begin & 1);
  }
  __syncthreads();
  for (int ks = ks_begin; ks < ksteps; ks++) {
    const int buf = ks & 1;
    if (ks + 1 < ksteps) load_regs(ks + 1);
    const bf16_t* A = lds + buf * (A_ELEMS + B_ELEMS);
    const bf16_t* B = A + A_ELEMS;
#pragma unroll
    for (int kk = 0; kk < 2; kk++) {
      bf16x8 a[TM], b[TN];
#pragma unroll
      for (int i = 0; i < TM; i++)
        a[i] = *reinterpret_cast<const bf16x8*>(A + (wm0 + 32 * i + (lane & 31)) * LDA + 16 * kk + 8 * (lane >> 5));
      if (!BT) {
#pragma unroll
        for (int j = 0; j < TN; j++)
          b[j] = *reinterpret_cast<const bf16x8*>(B + (wn0 + 32 * j + (lane & 31)) * LDA + 16 * kk + 8 * (lane >> 5));
      } else {
        // transpose load: lane j16 of a 16-lane group supplies the row k0 + j16/4, columns 4*(j16%4)..+3 and
        // receives the four k values of column (lane%16) of the group's 16 columns
        const int j16 = lane & 15, half = (lane >> 4) & 1, kb = 16 * kk + 8 * (lane >> 5);
#pragma unroll
        for (int j = 0; j < TN; j++) {
          const bf16_t* p = B + (kb + (j16 >> 2)) * LDBT + wn0 + 32 * j + 16 * half + 4 * (j16 & 3);
          union { bf16x8 v; shortx4 h[2]; } u;
          u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((shortx4 __attribute__((address_space(3)))*)(p));
          u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((shortx4 __attribute__((address_space(3)))*)(p + 4 * LDBT));
          b[j] = u.v;
        }
      }
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (ks + 1 < ksteps) store_lds(buf ^ 1);
    __syncthreads();
  }

  // epilogue: lane holds column n = l%32 and rows 8*(r/4) + 4*(l/32) + r%4 of every 32x32 block
  if (g.splits > 1) {   // raw fp32 partial tile; igemm_finish_kernel adds the splits and applies the epilogue
    float* part = reinterpret_cast<float*>((char*)ws.p[z] + g.scratch_off) + (int64_t)sp * g.M * g.Ncols;
#pragma unroll
    for (int j = 0; j < TN; j++) {
      const int n = n0 + wn0 + 32 * j + (lane & 31);
      if (n >= g.Ncols) continue;
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const int m = m0 + wm0 + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          if (m < g.M) part[(int64_t)m * g.Ncols + n] = acc[i][j][r];
        }
    }
    return;
  }
  bf16_t* out = (bf16_t*)ws.p[z] + ep.out_off;
  const bf16_t* mask = (const bf16_t*)ws.p[z] + ep.mask_off;
  const bf16_t* bias = (const bf16_t*)wts.p[z] + ep.bias_off;
#pragma unroll
  for (int j = 0; j < TN; j++) {
    const int n = n0 + wn0 + 32 * j + (lane & 31);
    if (n >= g.Ncols) continue;
    const float bv = ep.has_bias ? bf2f(bias[n]) : 0.f;
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int m = m0 + wm0 + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (m >= g.M) continue;
        float v = acc[i][j][r] + bv;
        if (ep.relu) v = fmaxf(v, 0.f);
        const int64_t o = (int64_t)m * g.Ncols + n;
        if (ep.use_mask && !(bf2f(mask[o]) > 0.f)) v = 0.f;
        if (ep.out_f32) reinterpret_cast<float*>(out)[o] = v;
        else out[o] = f2bf(v);
      }
  }
}

typedef int v4i_t __attribute__((ext_vector_type(4)));
// Bias, ReLU, ReLU mask of the input gradient, conversion and store of one wavefront's WM x WN accumulator tile whose
// origin is (mw, nw).  `lds` is the workgroup's tile memory, free once every wavefront has passed the barrier inside.
template <int WM, int WN>
__device__ __forceinline__ void frag_epilogue(floatx16 (&acc)[WM / 32][WN / 32], bf16_t* lds, void* ws_base, const void* wt_base,
                                              const IGemm& g, const Epilogue& ep, int mw, int nw, int lane, int wave) {
  constexpr int TM = WM / 32, TN = WN / 32;
  bf16_t* out = (bf16_t*)ws_base + ep.out_off;
  const bf16_t* mask = (const bf16_t*)ws_base + ep.mask_off;
  const bf16_t* bias = (const bf16_t*)wt_base + ep.bias_off;
  if (!ep.out_f32) {
    // bf16 output: a lane holds single elements of 16 different rows, which written straight out are 2-byte stores.
    // Each wavefront turns its 32-row blocks around in its own piece of LDS (the tiles there are no longer needed) and
    // writes 16 bytes per lane, 8 lanes per row; the ReLU mask of the input gradient is read the same way.
    constexpr int LDE = WN + 8;                          // row stride of the staging piece (elements)
    __syncthreads();                                     // every wavefront has finished reading the last tile
    bf16_t* stage = lds + wave * (32 * LDE);
    constexpr int CPRW = WN / 8;                         // 16-byte chunks per row of the wavefront's tile
    constexpr int RPI = 64 / CPRW;                       // rows covered by one 64-lane pass
    const int rrow = lane / CPRW, rchunk = lane % CPRW;
#pragma unroll
    for (int i = 0; i < TM; i++) {
#pragma unroll
      for (int j = 0; j < TN; j++) {
        const int n = nw + 32 * j + (lane & 31);
        const float bv = (ep.has_bias && n < g.Ncols) ? bf2f(bias[n]) : 0.f;
#pragma unroll
        for (int r = 0; r < 16; r++) {
          float v = acc[i][j][r] + bv;
          if (ep.relu) v = fmaxf(v, 0.f);
          stage[(8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) * LDE + 32 * j + (lane & 31)] = f2bf(v);
        }
      }
      // LDS operations of one wavefront complete in order, so its reads below see its writes above; the compiler is
      // told not to move LDS accesses across the two phases
      __builtin_amdgcn_wave_barrier();
      asm volatile("" ::: "memory");
#pragma unroll
      for (int it = 0; it < 32 / RPI; it++) {
        const int row = rrow + RPI * it;
        const int m = mw + 32 * i + row, n = nw + rchunk * 8;
        uint4 q = *reinterpret_cast<const uint4*>(stage + row * LDE + rchunk * 8);
        if (m < g.M && n < g.Ncols) {
          const int64_t o = (int64_t)m * g.Ncols + n;
          if (ep.use_mask) {
            const uint4 mk = *reinterpret_cast<const uint4*>(mask + o);
            const uint32_t mw[4] = {mk.x, mk.y, mk.z, mk.w};
            uint32_t qw[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int w = 0; w < 4; w++) {                // keep a 16-bit half where the forward value is positive
              const uint32_t lo = mw[w] & 0xffffu, hi = mw[w] >> 16;
              const uint32_t keep = (((lo & 0x8000u) == 0 && (lo & 0x7fffu) != 0) ? 0x0000ffffu : 0u) |
                                    (((hi & 0x8000u) == 0 && (hi & 0x7fffu) != 0) ? 0xffff0000u : 0u);
              qw[w] &= keep;
            }
            q = make_uint4(qw[0], qw[1], qw[2], qw[3]);
          }
          *reinterpret_cast<uint4*>(out + o) = q;
        }
      }
      __builtin_amdgcn_wave_barrier();
      asm volatile("" ::: "memory");
    }
    return;
  }
#pragma unroll
  for (int j = 0; j < TN; j++) {
    const int n = nw + 32 * j + (lane & 31);
    if (n >= g.Ncols) continue;
    const float bv = ep.has_bias ? bf2f(bias[n]) : 0.f;
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int m = mw + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (m >= g.M) continue;
        float v = acc[i][j][r] + bv;
        if (ep.relu) v = fmaxf(v, 0.f);
        const int64_t o = (int64_t)m * g.Ncols + n;
        if (ep.use_mask && !(bf2f(mask[o]) > 0.f)) v = 0.f;
        reinterpret_cast<float*>(out)[o] = v;
      }
  }
}

// ------------------------------------------------------------------ convolution forward / dgrad, B from fragments
// Same tiling as igemm_kernel, but only the gathered im2col tile goes through LDS; the filter operand comes
// from the fragment-packed copy, one coalesced 1 KiB read per MFMA operand, prefetched one step ahead.  This
// halves the LDS traffic per MFMA, which is what bounds the LDS-only variant.
constexpr uint32_t kOutOfRange = 0x80000000u;   // buffer offset beyond any tensor: the load returns zeros

// NT = threads per workgroup = 64 x number of wave tiles.
// UNI: every contraction step stays inside one filter tap (channels per tap are a multiple of the step) and the
// window has at most 32 taps.  Then the tap is wavefront-uniform and advances in scalar registers, the per-row
// bounds test is one bit of a mask computed once, and a step costs a handful of vector instructions besides the
// loads and MFMAs.  Otherwise (first layer, large windows) the tap is decoded per lane and step.
template <int BM, int BN, int WM, int WN, int BKT, int NT, bool UNI>
__global__ __launch_bounds__(NT, (WM * WN > 64 * 64 ? 2 : 1)) void igemm_frag_kernel(PtrTab ws, CPtrTab wts, IGemm g, Epilogue ep) {
  constexpr int WAVES_N = BN / WN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int LDF = BKT + 8;                 // 80 or 144 byte rows: conflict-free 16-byte reads
  constexpr int CPS = BKT / 8;                 // chunks per contraction step
  constexpr int KK = BKT / 16;                 // MFMA k-blocks per step
  constexpr int A_ELEMS = BM * LDF;
  __shared__ __attribute__((aligned(16))) bf16_t lds[2 * A_ELEMS];

  const int z = blockIdx.z / g.splits, sp = blockIdx.z % g.splits;
  const bf16_t* act = (const bf16_t*)ws.p[z] + g.a_off;
  const bf16_t* Bf = (const bf16_t*)wts.p[z] + g.b_off;
  // Buffer resources: an offset at or beyond the size reads as zero in hardware, so padding taps, ragged rows
  // and ragged columns need no branch, no select on the data and no 64-bit address arithmetic.
  const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc((void*)act, 0, (int)g.a_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_b = __builtin_amdgcn_make_buffer_rsrc((void*)Bf, 0, (int)g.b_bytes, 0x00020000);
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  const int KB16 = g.ldb / 16;
  const int NB = (g.Ncols + 31) / 32;

  constexpr int A_LOADS = (BM * CPS + NT - 1) / NT;
  constexpr int RPP = NT / CPS;                // tile rows covered per loader pass
  constexpr bool FULL = (BM % RPP) == 0;       // every loader pass lies inside the tile
  const int cc = tid % CPS, lrow = tid / CPS;
  // per tile row handled by this thread: byte offset of its window origin (plus this thread's chunk in UNI mode),
  // and either the origin's coordinates or (UNI) a mask with one bit per tap that falls outside the tensor
  int row_off[A_LOADS], row_oh[A_LOADS], row_ow[A_LOADS];
  uint32_t row_bad[A_LOADS];
#pragma unroll
  for (int i = 0; i < A_LOADS; i++) {
    const RowPos r = row_pos(act, g, m0 + lrow + RPP * i);
    row_off[i] = (int)((r.base - act) * 2) + (UNI ? cc * 16 : 0);
    row_oh[i] = r.valid ? r.oh : -0x40000000;  // an invalid row fails every bounds test below
    row_ow[i] = r.ow;
    if (UNI) {
      uint32_t good = 0;
      if (r.valid) {
        const int kw_lo = max(0, -r.ow), kw_hi = min(g.ks, g.W - r.ow);              // valid kw: [kw_lo, kw_hi)
        const uint32_t kwmask = kw_hi > kw_lo ? (((1u << kw_hi) - 1u) & ~((1u << kw_lo) - 1u)) : 0u;
        for (int kh = 0; kh < g.ks; kh++)
          if ((unsigned)(r.oh + kh) < (unsigned)g.H) good |= kwmask << (kh * g.ks);
      }
      row_bad[i] = ~good;
    }
  }

  const int all_steps = (g.Kchunks + CPS - 1) / CPS;
  const int per = (all_steps + g.splits - 1) / g.splits;
  const int ks_begin = __builtin_amdgcn_readfirstlane(sp * per);
  const int ksteps = __builtin_amdgcn_readfirstlane(min(all_steps, ks_begin + per));

  // UNI: tap state of the step that load_a fetches next, kept in scalar registers
  int u_tap = 0, u_c8 = 0, u_kw = 0, u_koff = 0;
  if (UNI) {
    const uint32_t q0 = (uint32_t)(ks_begin * CPS);
    u_tap = (int)fastdiv(q0, g.CPT, g.mg_cpt);
    u_c8 = (int)q0 - u_tap * g.CPT;
    const int kh = (int)fastdiv((uint32_t)u_tap, g.ks, g.mg_ks);
    u_kw = u_tap - kh * g.ks;
    u_koff = ((kh * g.W + u_kw) * g.C + u_c8 * 8) * 2;
    u_tap = __builtin_amdgcn_readfirstlane(u_tap);
    u_c8 = __builtin_amdgcn_readfirstlane(u_c8);
    u_kw = __builtin_amdgcn_readfirstlane(u_kw);
    u_koff = __builtin_amdgcn_readfirstlane(u_koff);
  }
  const int u_row_step = __builtin_amdgcn_readfirstlane((g.W - g.ks) * g.C * 2);   // extra bytes when kw wraps to the next kh

  v4i_t ra[A_LOADS];
  auto load_a = [&](int ks) {
    if (UNI) {
#pragma unroll
      for (int i = 0; i < A_LOADS; i++) {
        const int bad = __builtin_amdgcn_sbfe((int)row_bad[i], u_tap, 1);            // 0 or -1
        const int off = (row_off[i] + u_koff) | (bad & (int)kOutOfRange);
        ra[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, off, 0, 0);
      }
      // advance to the next step: CPS more chunks of the same tap, or the first chunks of the next tap
      u_c8 += CPS;
      u_koff += CPS * 16;
      const bool next_tap = u_c8 >= g.CPT;
      u_c8 = next_tap ? 0 : u_c8;
      u_tap += next_tap ? 1 : 0;
      u_kw += next_tap ? 1 : 0;
      const bool next_row = u_kw == g.ks;
      u_kw = next_row ? 0 : u_kw;
      u_koff += next_row ? u_row_step : 0;
    } else {
      const int q = ks * CPS + cc;
      const uint32_t tap = fastdiv((uint32_t)q, g.CPT, g.mg_cpt);
      const int c8 = q - (int)tap * g.CPT;
      const int kh = (int)fastdiv(tap, g.ks, g.mg_ks), kw = (int)tap - kh * g.ks;
      const int koff = ((kh * g.W + kw) * g.C + c8 * 8) * 2;
      const bool qok = q < g.Kchunks;
#pragma unroll
      for (int i = 0; i < A_LOADS; i++) {
        const bool ok = qok && (unsigned)(row_oh[i] + kh) < (unsigned)g.H && (unsigned)(row_ow[i] + kw) < (unsigned)g.W;
        ra[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, ok ? (row_off[i] + koff) : (int)kOutOfRange, 0, 0);
      }
    }
  };
  auto store_a = [&](int buf) {
    bf16_t* A = lds + buf * A_ELEMS;
#pragma unroll
    for (int i = 0; i < A_LOADS; i++)
      if (FULL || lrow + RPP * i < BM) *reinterpret_cast<v4i_t*>(A + (lrow + RPP * i) * LDF + cc * 8) = ra[i];
  };
  // B fragments: one fixed byte offset per column block of this wavefront; the step advances a scalar offset
  uint32_t boff[TN];
#pragma unroll
  for (int j = 0; j < TN; j++) {
    const int nb = (n0 + wn0) / 32 + j;
    boff[j] = nb < NB ? (uint32_t)(((int64_t)nb * KB16 * 512 + lane * 8) * 2) : kOutOfRange;
  }
  int b_step = ks_begin * KK * 1024;           // scalar byte offset of the step that load_b fetches next
  auto load_b = [&](bf16x8 (&bt)[KK][TN]) {
#pragma unroll
    for (int kk = 0; kk < KK; kk++)
#pragma unroll
      for (int j = 0; j < TN; j++) {
        union { v4i_t u; bf16x8 v; } f;
        f.u = __builtin_amdgcn_raw_buffer_load_b128(rsrc_b, (int)(boff[j] + kk * 1024), b_step, 0);
        bt[kk][j] = f.v;
      }
    b_step += KK * 1024;
  };

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

  // One contraction step ks on LDS buffer `buf`.  At entry the A fragments of its first k-block (`a0`) are already in
  // registers.  The im2col chunks of step ks+1 (fetched during step ks-1, now in staging registers) go to the other
  // LDS buffer, the chunks of step ks+2 and the filter fragments of step ks+1 (into `bnext`) are requested, the A
  // fragments of the second k-block are read, and the first k-block's MFMAs run.  The single barrier of the step
  // sits in the middle: after it every wavefront has finished reading `buf` and writing the other buffer, so the
  // first A fragments of step ks+1 (`a0n`) are read while the second k-block's MFMAs run, and nothing waits on LDS
  // right after a barrier.  Fragment sets swap roles from step to step: two steps per loop iteration, no copies.
  auto lds_frag = [&](int buf, int i, int kk) {
    return *reinterpret_cast<const bf16x8*>(lds + buf * A_ELEMS + (wm0 + 32 * i + (lane & 31)) * LDF + 16 * kk + 8 * (lane >> 5));
  };
  auto step = [&](bf16x8 (&bcur)[KK][TN], bf16x8 (&bnext)[KK][TN], bf16x8 (&a0)[TM], bf16x8 (&a0n)[TM], int ks, int buf, bool has1,
                  bool has2) {
    static_assert(KK == 2, "two k-blocks per step");
    if (has1) store_a(buf ^ 1);
    if (has2) load_a(ks + 2);
    if (has1) load_b(bnext);
    bf16x8 a1[TM];
#pragma unroll
    for (int i = 0; i < TM; i++) a1[i] = lds_frag(buf, i, 1);
    __builtin_amdgcn_sched_barrier(0);         // requests and LDS traffic first: they need the step to complete
    __builtin_amdgcn_s_setprio(1);             // a wavefront in its MFMA phase keeps the matrix pipe; others issue memory work
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[i], bcur[0][j], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_s_setprio(0);
    __syncthreads();
    if (has1) {
#pragma unroll
      for (int i = 0; i < TM; i++) a0n[i] = lds_frag(buf ^ 1, i, 0);
    }
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[i], bcur[1][j], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_s_setprio(0);
  };

  bf16x8 b0[KK][TN], b1[KK][TN], fa[TM], fb[TM];
  int ks = ks_begin;
  if (ks < ksteps) {
    load_a(ks);
    load_b(b0);
    store_a(0);
    if (ks + 1 < ksteps) load_a(ks + 1);
  }
  __syncthreads();
  if (ks < ksteps) {
#pragma unroll
    for (int i = 0; i < TM; i++) fa[i] = lds_frag(0, i, 0);
  }
  // Inside the loop both steps prefetch unconditionally: a branch around the loads would make the compiler wait
  // for the most pessimistic count of outstanding loads where the paths join.
  for (; ks + 3 < ksteps; ks += 2) {
    step(b0, b1, fa, fb, ks, 0, true, true);
    step(b1, b0, fb, fa, ks + 1, 1, true, true);
  }
  for (; ks + 1 < ksteps; ks += 2) {          // at most once: two or three steps remain
    step(b0, b1, fa, fb, ks, 0, true, ks + 2 < ksteps);
    step(b1, b0, fb, fa, ks + 1, 1, ks + 2 < ksteps, false);
  }
  if (ks < ksteps) step(b0, b1, fa, fb, ks, 0, false, false);

  if (g.splits > 1) {
    float* part = reinterpret_cast<float*>((char*)ws.p[z] + g.scratch_off) + (int64_t)sp * g.M * g.Ncols;
#pragma unroll
    for (int j = 0; j < TN; j++) {
      const int n = n0 + wn0 + 32 * j + (lane & 31);
      if (n >= g.Ncols) continue;
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const int m = m0 + wm0 + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          if (m < g.M) part[(int64_t)m * g.Ncols + n] = acc[i][j][r];
        }
    }
    return;
  }
  static_assert(4 * 32 * (WN + 8) <= 2 * A_ELEMS || NT != 256, "the epilogue's staging piece fits the tile buffers");
  frag_epilogue<WM, WN>(acc, lds, ws.p[z], wts.p[z], g, ep, m0 + wm0, n0 + wn0, lane, wave);
}

// ------------------------------------------------------------------ convolution forward / dgrad, input patch in LDS
// For windows larger than 1 x 1 the im2col tile of one tap is the tile of the neighbouring tap shifted by one
// pixel, so gathering it tap by tap moves every input pixel ks*ks times from the L1 into LDS.  This kernel puts
// the input patch under a tile of BM output positions into LDS once per 32 input channels (zero padding and the
// halo rows included, 80 bytes per pixel) and reads the MFMA A operand of tap (kh, kw) from it at the address of the
// output position's window origin plus a wavefront-uniform offset.  The ks*ks contraction steps of one channel
// chunk run without a barrier; the filter operand comes from the fragment-packed copy as in igemm_frag_kernel
// (k = tap * C + c, so the 32 channels of a chunk are two 16-k blocks at tap * C/16 + 2 * chunk).
//   patch rows: the output rows gr = m / OW of the tile, gr_lo .. gr_hi, may belong to several images; image n owns
//   a band of (its output rows in the tile) + ks - 1 input rows, so the row of (gr, kh) is
//   (gr - gr_lo) + kh + (ks - 1)(n - n_lo);  patch columns: OW + ks - 1 = W + 2 pad.
// The contraction may be split over channel chunks (g.splits <= C / 32).
// Workgroups are handed to the eight XCDs round-robin in launch order, and each XCD has its own L2.  This turns the
// launch-order index around so that every XCD works through one contiguous eighth of the (x, y, z) tile space: tiles
// that share filter fragments and halo rows then share an L2 instead of being spread over all eight.
struct TileIdx { int x, y, z; };
__device__ __forceinline__ TileIdx xcd_tile(int on) {
  uint32_t lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
  const uint32_t per = (gridDim.x * gridDim.y * gridDim.z) >> 3;
  if (on && lin < per * 8u) lin = (lin & 7u) * per + (lin >> 3);   // the last (count mod 8) workgroups keep their place
  TileIdx t;
  const uint32_t q = lin / gridDim.x;
  t.x = (int)(lin - q * gridDim.x);
  t.z = (int)(q / gridDim.y);
  t.y = (int)(q - (uint32_t)t.z * gridDim.y);
  return t;
}

struct HaloArgs {
  int PW;              // patch width in pixels
  uint32_t mg_pw;      // multiplier for division by PW
  int n_px_max;        // pixels the LDS patch has room for
  int xcd;             // 1: XCD-contiguous tile order (see xcd_tile)
  int tab_off;         // bytes from the start of LDS to the pixel table (behind the patch, rounded up to whole refill rounds)
};

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(64 * (BM / WM) * (BN / WN), (WM * WN > 64 * 64 ? 2 : 3)) void conv_halo_kernel(PtrTab ws, CPtrTab wts, IGemm g, Epilogue ep, HaloArgs h) {
  constexpr int NT = 64 * (BM / WM) * (BN / WN);
  constexpr int WAVES_N = BN / WN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int PST = 40;                      // elements per patch pixel: 32 channels + 8 of padding (conflict-free 16-byte reads)
  extern __shared__ __attribute__((aligned(16))) bf16_t halo_lds[];
  bf16_t* lds = halo_lds;
  int* tab = reinterpret_cast<int*>(reinterpret_cast<char*>(lds) + h.tab_off);   // byte offset of every patch pixel in the tensor

  const TileIdx tile = xcd_tile(h.xcd);
  const int z = tile.z / g.splits, sp = tile.z % g.splits;
  const bf16_t* act = (const bf16_t*)ws.p[z] + g.a_off;
  const bf16_t* Bf = (const bf16_t*)wts.p[z] + g.b_off;
  const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc((void*)act, 0, (int)g.a_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_b = __builtin_amdgcn_make_buffer_rsrc((void*)Bf, 0, (int)g.b_bytes, 0x00020000);
  const int m0 = tile.x * BM, n0 = tile.y * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  const int KB16 = g.ldb / 16;
  const int NB = (g.Ncols + 31) / 32;

  const int ks = g.ks, PW = h.PW;
  const int m_last = min(m0 + BM, g.M) - 1;
  const int gr_lo = (int)fastdiv((uint32_t)m0, g.OW, g.mg_ow), gr_hi = (int)fastdiv((uint32_t)m_last, g.OW, g.mg_ow);
  const int n_lo = (int)fastdiv((uint32_t)gr_lo, g.OH, g.mg_oh), n_hi = (int)fastdiv((uint32_t)gr_hi, g.OH, g.mg_oh);
  const int oh_lo = gr_lo - n_lo * g.OH;
  const int NR = gr_hi - gr_lo + 1;
  const int n_px = (NR + (ks - 1) * (n_hi - n_lo + 1)) * PW;   // <= h.n_px_max (checked by the launcher's bound)

  for (int p = tid; p < n_px; p += NT) {
    const int pr = (int)fastdiv((uint32_t)p, PW, h.mg_pw), pc = p - pr * PW;
    int start = 0, rem = NR, n = n_lo, first = oh_lo, ih = -1, nn = -1;
    while (rem > 0) {
      const int rows = min(g.OH - first, rem), len = rows + ks - 1;
      if (pr < start + len) { nn = n; ih = first - g.pad + (pr - start); break; }
      start += len; rem -= rows; n++; first = 0;
    }
    const int iw = pc - g.pad;
    const bool ok = nn >= 0 && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W;
    tab[p] = ok ? ((nn * g.H + ih) * g.W + iw) * g.C * 2 : (int)kOutOfRange;
  }

  // window origin of this lane's rows in the patch (bytes); rows beyond M repeat the last one and are never stored
  int abase[TM];
#pragma unroll
  for (int i = 0; i < TM; i++) {
    const uint32_t m = (uint32_t)min(m0 + wm0 + 32 * i + (lane & 31), g.M - 1);
    const uint32_t gr = fastdiv(m, g.OW, g.mg_ow), ow = m - gr * (uint32_t)g.OW;
    const uint32_t n = fastdiv(gr, g.OH, g.mg_oh);
    const int pr0 = ((int)gr - gr_lo) + (ks - 1) * ((int)n - n_lo);
    abase[i] = ((pr0 * PW + (int)ow) * PST + 8 * (lane >> 5)) * 2;
  }
  __syncthreads();

  // Patch refill: LDS-direct loads, 64 consecutive 16-byte slots per wavefront and instruction.  Slot s holds piece
  // s % 5 of pixel s / 5; the fifth piece of a pixel is its padding and, like the slots beyond the patch, is
  // requested out of range (the hardware writes zeros).
  const int n_slots = n_px * 5;
  const int dma_rounds = (n_slots + NT - 1) / NT;
  const int wave_slot = __builtin_amdgcn_readfirstlane(wave * 64);
  auto refill = [&](int cc) {
#pragma unroll 1
    for (int r = 0; r < dma_rounds; r++) {
      const int sl = r * NT + tid;
      const int px = (int)(__umulhi((uint32_t)sl, 0xCCCCCCCDu) >> 2);   // sl / 5
      const int sub = sl - 5 * px;
      const int voff = (sub < 4 && sl < n_slots) ? tab[min(px, n_px - 1)] + sub * 16 : (int)kOutOfRange;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, (__attribute__((address_space(3))) void*)(reinterpret_cast<char*>(lds) + (r * NT + wave_slot) * 16),
                                               16, voff, cc * 64, 0, 0);
    }
  };

  uint32_t boff[TN];
#pragma unroll
  for (int j = 0; j < TN; j++) {
    const int nb = (n0 + wn0) / 32 + j;
    boff[j] = nb < NB ? (uint32_t)(((int64_t)nb * KB16 * 512 + lane * 8) * 2) : kOutOfRange;
  }
  const int b_tap = __builtin_amdgcn_readfirstlane((g.C / 16) * 1024);   // bytes from one tap's k-blocks to the next tap's
  auto load_b = [&](bf16x8 (&bt)[2][TN], int s_off) {
#pragma unroll
    for (int kk = 0; kk < 2; kk++)
#pragma unroll
      for (int j = 0; j < TN; j++) {
        union { v4i_t u; bf16x8 v; } f;
        f.u = __builtin_amdgcn_raw_buffer_load_b128(rsrc_b, (int)(boff[j] + kk * 1024), s_off, 0);
        bt[kk][j] = f.v;
      }
  };
  auto lds_a = [&](int i, int toff, int kk) {
    return *reinterpret_cast<const bf16x8*>(reinterpret_cast<const char*>(lds) + abase[i] + toff + kk * 32);
  };

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

  const int chunks = g.C >> 5;
  const int per = (chunks + g.splits - 1) / g.splits;
  const int cc_begin = __builtin_amdgcn_readfirstlane(sp * per);
  const int cc_end = __builtin_amdgcn_readfirstlane(min(chunks, cc_begin + per));
  const int T = ks * ks;
  const int a_wrap = (PW - ks) * PST * 2;

  // patch byte offset of the running tap (c_aoff); patch offset, kw and filter byte offset of the tap after it (n_*)
  int c_aoff = 0, n_aoff = 0, n_kw = 0, n_boff = 0;
  auto advance = [&]() {
    c_aoff = n_aoff;
    n_kw++; n_aoff += PST * 2; n_boff += b_tap;
    const bool wrap = n_kw == ks;
    n_kw = wrap ? 0 : n_kw;
    n_aoff += wrap ? a_wrap : 0;
  };
  // One tap.  The filter fragments travel two taps ahead through a ring of three register sets (the L2 round trip is
  // longer than one tap's MFMAs): `bld` receives tap t + 2 while `bcur` (tap t) is consumed.  The second k-block's A
  // fragments are read, the first k-block's MFMAs run, the next tap's first A fragments are read, the second
  // k-block's MFMAs run.
  bf16x8 a0[TM];
  auto step = [&](bf16x8 (&bcur)[2][TN], bf16x8 (&bld)[2][TN], bool ld, bool has_next) {
    if (ld) load_b(bld, n_boff + b_tap);
    bf16x8 a1[TM];
#pragma unroll
    for (int i = 0; i < TM; i++) a1[i] = lds_a(i, c_aoff, 1);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[i], bcur[0][j], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
    if (has_next) {                              // straight into a0: its last readers have been issued
#pragma unroll
      for (int i = 0; i < TM; i++) a0[i] = lds_a(i, n_aoff, 0);
    }
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[i], bcur[1][j], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_s_setprio(0);
    advance();
  };

  bf16x8 bq0[2][TN], bq1[2][TN], bq2[2][TN];
  if (cc_begin < cc_end) {
    refill(cc_begin);
    load_b(bq0, cc_begin * 2048);
    load_b(bq1, cc_begin * 2048 + b_tap);
  }
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  // ks * ks leaves the remainder 0 or 1 when divided by three, so after the full groups of three taps either three
  // or four taps remain.  They are written out straight-line in two copies of the chunk loop: with a joined tail the
  // compiler kept a second set of accumulators.
  auto run = [&](auto four) {
    const int groups = (T - 2) / 3;
#pragma unroll 1
    for (int cc = cc_begin; cc < cc_end; cc++) {
      n_aoff = 0; n_kw = 0; n_boff = cc * 2048;
      advance();                                 // c_aoff = tap 0, n_* = tap 1
#pragma unroll
      for (int i = 0; i < TM; i++) a0[i] = lds_a(i, 0, 0);
#pragma unroll 1
      for (int t = 0; t < groups; t++) {
        step(bq0, bq2, true, true);
        step(bq1, bq0, true, true);
        step(bq2, bq1, true, true);
      }
      if constexpr (decltype(four)::value) {
        step(bq0, bq2, true, true);
        step(bq1, bq0, true, true);
        step(bq2, bq1, false, true);
        step(bq0, bq2, false, false);
      } else {
        step(bq0, bq2, true, true);
        step(bq1, bq0, false, true);
        step(bq2, bq1, false, false);
      }
      const bool more = cc + 1 < cc_end;
      if (more) {
        load_b(bq0, (cc + 1) * 2048);
        load_b(bq1, (cc + 1) * 2048 + b_tap);
      }
      __syncthreads();                           // every wavefront has finished reading the patch
      if (more) refill(cc + 1);
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();
    }
  };
  if (T % 3 == 1) run(std::true_type{});
  else run(std::false_type{});

  if (g.splits > 1) {
    float* part = reinterpret_cast<float*>((char*)ws.p[z] + g.scratch_off) + (int64_t)sp * g.M * g.Ncols;
#pragma unroll
    for (int j = 0; j < TN; j++) {
      const int n = n0 + wn0 + 32 * j + (lane & 31);
      if (n >= g.Ncols) continue;
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const int m = m0 + wm0 + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          if (m < g.M) part[(int64_t)m * g.Ncols + n] = acc[i][j][r];
        }
    }
    return;
  }
  frag_epilogue<WM, WN>(acc, lds, ws.p[z], wts.p[z], g, ep, m0 + wm0, n0 + wn0, lane, wave);
}

// ------------------------------------------------------------------ patch-in-LDS convolution for few input channels
// First layers: 8 channels (3 padded) or a multiple of 16 that is not one of 32 (48 after the space-to-depth
// re-layout).  The whole pixel goes into the patch, loaded once per tile, and the contraction walks the 16-k blocks
// of the packed filters in their own order, k = tap * C + c:
//   C % 16 == 0: block b is channels 16 (b % (C/16)) ... + 15 of tap b / (C/16); the lane halves take its two 8-channel
//                halves, as in conv_halo_kernel, but each of a step's two blocks has a patch offset of its own;
//   C == 8:      block b is taps 2 b (lane half 0) and 2 b + 1 (lane half 1), all 8 channels each.
// Pixels are C * 2 bytes plus 16 bytes of padding (none for C == 8, where consecutive pixels are consecutive
// 16-byte reads).  Blocks behind the last tap exist only as zero padding of the filters; they read the last tap.
// The contraction may be split over steps (two blocks each).
struct HaloSeqArgs {
  int PW;              // patch width in pixels
  uint32_t mg_pw;      // multiplier for division by PW
  int n_px_max;        // pixels the LDS patch has room for
  int tab_off;         // bytes from the start of LDS to the pixel table
  int spp;             // 16-byte slots per pixel in LDS (data + padding)
  uint32_t mg_spp;     // multiplier for division by spp
  int pixb;            // bytes per pixel in LDS = 16 spp
  int C16;             // 16-channel blocks per tap (C % 16 == 0)
  uint32_t mg_c16;     // multiplier for division by C16
};

template <int BM, int BN, int WM, int WN, bool C8>
__global__ __launch_bounds__(64 * (BM / WM) * (BN / WN), (WM * WN > 64 * 64 ? 2 : 3)) void conv_halo_seq_kernel(PtrTab ws, CPtrTab wts, IGemm g, Epilogue ep, HaloSeqArgs h) {
  constexpr int NT = 64 * (BM / WM) * (BN / WN);
  constexpr int WAVES_N = BN / WN;
  constexpr int TM = WM / 32, TN = WN / 32;
  extern __shared__ __attribute__((aligned(16))) bf16_t halo_seq_lds[];
  bf16_t* lds = halo_seq_lds;
  int* tab = reinterpret_cast<int*>(reinterpret_cast<char*>(lds) + h.tab_off);

  const int z = blockIdx.z / g.splits, sp = blockIdx.z % g.splits;
  const bf16_t* act = (const bf16_t*)ws.p[z] + g.a_off;
  const bf16_t* Bf = (const bf16_t*)wts.p[z] + g.b_off;
  const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc((void*)act, 0, (int)g.a_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_b = __builtin_amdgcn_make_buffer_rsrc((void*)Bf, 0, (int)g.b_bytes, 0x00020000);
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  const int KB16 = g.ldb / 16;
  const int NB = (g.Ncols + 31) / 32;

  // patch geometry and pixel table: as in conv_halo_kernel
  const int ks = g.ks, PW = h.PW, pixb = h.pixb;
  const int m_last = min(m0 + BM, g.M) - 1;
  const int gr_lo = (int)fastdiv((uint32_t)m0, g.OW, g.mg_ow), gr_hi = (int)fastdiv((uint32_t)m_last, g.OW, g.mg_ow);
  const int n_lo = (int)fastdiv((uint32_t)gr_lo, g.OH, g.mg_oh), n_hi = (int)fastdiv((uint32_t)gr_hi, g.OH, g.mg_oh);
  const int oh_lo = gr_lo - n_lo * g.OH;
  const int NR = gr_hi - gr_lo + 1;
  const int n_px = (NR + (ks - 1) * (n_hi - n_lo + 1)) * PW;
  for (int p = tid; p < n_px; p += NT) {
    const int pr = (int)fastdiv((uint32_t)p, PW, h.mg_pw), pc = p - pr * PW;
    int start = 0, rem = NR, n = n_lo, first = oh_lo, ih = -1, nn = -1;
    while (rem > 0) {
      const int rows = min(g.OH - first, rem), len = rows + ks - 1;
      if (pr < start + len) { nn = n; ih = first - g.pad + (pr - start); break; }
      start += len; rem -= rows; n++; first = 0;
    }
    const int iw = pc - g.pad;
    const bool ok = nn >= 0 && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W;
    tab[p] = ok ? ((nn * g.H + ih) * g.W + iw) * g.C * 2 : (int)kOutOfRange;
  }
  int abase[TM];
#pragma unroll
  for (int i = 0; i < TM; i++) {
    const uint32_t m = (uint32_t)min(m0 + wm0 + 32 * i + (lane & 31), g.M - 1);
    const uint32_t gr = fastdiv(m, g.OW, g.mg_ow), ow = m - gr * (uint32_t)g.OW;
    const uint32_t n = fastdiv(gr, g.OH, g.mg_oh);
    const int pr0 = ((int)gr - gr_lo) + (ks - 1) * ((int)n - n_lo);
    abase[i] = (pr0 * PW + (int)ow) * pixb + (C8 ? 0 : 16 * (lane >> 5));
  }
  __syncthreads();
  {
    const int dpp = g.C / 8;                               // data slots per pixel
    const int n_slots = n_px * h.spp;
    const int dma_rounds = (n_slots + NT - 1) / NT;
    const int wave_slot = __builtin_amdgcn_readfirstlane(wave * 64);
#pragma unroll 1
    for (int r = 0; r < dma_rounds; r++) {
      const int sl = r * NT + tid;
      const int px = (int)fastdiv((uint32_t)sl, h.spp, h.mg_spp), sub = sl - px * h.spp;
      const int voff = (sub < dpp && sl < n_slots) ? tab[min(px, n_px - 1)] + sub * 16 : (int)kOutOfRange;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, (__attribute__((address_space(3))) void*)(reinterpret_cast<char*>(lds) + (r * NT + wave_slot) * 16),
                                               16, voff, 0, 0, 0);
    }
  }

  uint32_t boff[TN];
#pragma unroll
  for (int j = 0; j < TN; j++) {
    const int nb = (n0 + wn0) / 32 + j;
    boff[j] = nb < NB ? (uint32_t)(((int64_t)nb * KB16 * 512 + lane * 8) * 2) : kOutOfRange;
  }
  auto load_b = [&](bf16x8 (&bt)[2][TN], int step) {
#pragma unroll
    for (int kk = 0; kk < 2; kk++)
#pragma unroll
      for (int j = 0; j < TN; j++) {
        union { v4i_t u; bf16x8 v; } f;
        f.u = __builtin_amdgcn_raw_buffer_load_b128(rsrc_b, (int)(boff[j] + kk * 1024), step * 2048, 0);
        bt[kk][j] = f.v;
      }
  };
  // patch byte offset of tap t (clamped to the last tap)
  const int T = ks * ks;
  auto tap_off = [&](int t) {
    t = min(t, T - 1);
    const int kh = (int)fastdiv((uint32_t)t, ks, g.mg_ks), kw = t - kh * ks;
    return (kh * PW + kw) * pixb;
  };
  // patch byte offset the lanes of k-block b add to their window origin
  const bool upper = lane >= 32;
  auto blk_off = [&](int b) {
    if (C8) {
      const int o0 = tap_off(2 * b), o1 = tap_off(2 * b + 1);
      return upper ? o1 : o0;
    }
    const int t = (int)fastdiv((uint32_t)b, h.C16, h.mg_c16), c16 = b - t * h.C16;
    return tap_off(t) + c16 * 32;
  };
  auto lds_a = [&](int i, int off) { return *reinterpret_cast<const bf16x8*>(reinterpret_cast<const char*>(lds) + abase[i] + off); };

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

  const int all_steps = (KB16 + 1) / 2;
  const int per = (all_steps + g.splits - 1) / g.splits;
  const int s_begin = __builtin_amdgcn_readfirstlane(sp * per);
  const int s_end = __builtin_amdgcn_readfirstlane(min(all_steps, s_begin + per));

  // One step = two k-blocks.  The filter fragments of the next step are requested, the second block's A fragments
  // are read, the first block's MFMAs run, the next step's first A fragments are read, the second block's MFMAs run.
  auto step = [&](bf16x8 (&bcur)[2][TN], bf16x8 (&bnext)[2][TN], bf16x8 (&a0)[TM], bf16x8 (&a0n)[TM], int s, bool has_next) {
    if (has_next) load_b(bnext, s + 1);
    const int o1 = blk_off(2 * s + 1);
    bf16x8 a1[TM];
#pragma unroll
    for (int i = 0; i < TM; i++) a1[i] = lds_a(i, o1);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[i], bcur[0][j], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_s_setprio(0);
    if (has_next) {
      const int o0 = blk_off(2 * s + 2);
#pragma unroll
      for (int i = 0; i < TM; i++) a0n[i] = lds_a(i, o0);
    }
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[i], bcur[1][j], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_s_setprio(0);
  };

  bf16x8 b0[2][TN], b1[2][TN], fa[TM], fb[TM];
  if (s_begin < s_end) load_b(b0, s_begin);
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  if (s_begin < s_end) {
    const int o0 = blk_off(2 * s_begin);
#pragma unroll
    for (int i = 0; i < TM; i++) fa[i] = lds_a(i, o0);
  }
  // two copies for an odd and an even number of steps: the last steps written out straight-line (see conv_halo_kernel)
  auto run = [&](auto odd) {
    int s = s_begin;
    const int pairs = (s_end - s_begin - 1) >> 1;
#pragma unroll 1
    for (int t = 0; t < pairs; t++, s += 2) {
      step(b0, b1, fa, fb, s, true);
      step(b1, b0, fb, fa, s + 1, true);
    }
    if constexpr (decltype(odd)::value) {
      step(b0, b1, fa, fb, s, false);
    } else {
      step(b0, b1, fa, fb, s, true);
      step(b1, b0, fb, fa, s + 1, false);
    }
  };
  if (s_begin < s_end) {
    if ((s_end - s_begin) & 1) run(std::true_type{});
    else run(std::false_type{});
  }

  if (g.splits > 1) {
    float* part = reinterpret_cast<float*>((char*)ws.p[z] + g.scratch_off) + (int64_t)sp * g.M * g.Ncols;
#pragma unroll
    for (int j = 0; j < TN; j++) {
      const int n = n0 + wn0 + 32 * j + (lane & 31);
      if (n >= g.Ncols) continue;
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const int m = m0 + wm0 + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          if (m < g.M) part[(int64_t)m * g.Ncols + n] = acc[i][j][r];
        }
    }
    return;
  }
  frag_epilogue<WM, WN>(acc, lds, ws.p[z], wts.p[z], g, ep, m0 + wm0, n0 + wn0, lane, wave);
}

// Sum of the split partials in split order, then bias / ReLU / mask / conversion.
__global__ __launch_bounds__(256) void igemm_finish_kernel(PtrTab ws, CPtrTab wts, IGemm g, Epilogue ep) {
  const int z = blockIdx.z;
  const float4* part = reinterpret_cast<const float4*>((const char*)ws.p[z] + g.scratch_off);
  bf16_t* out = (bf16_t*)ws.p[z] + ep.out_off;
  const bf16_t* mask = (const bf16_t*)ws.p[z] + ep.mask_off;
  const bf16_t* bias = (const bf16_t*)wts.p[z] + ep.bias_off;
  // four consecutive columns per thread (the column count is a multiple of 8)
  const uint32_t total4 = (uint32_t)(((int64_t)g.M * g.Ncols) >> 2);
  for (uint32_t o4 = blockIdx.x * 256 + threadIdx.x; o4 < total4; o4 += gridDim.x * 256) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
    for (int sp = 0; sp < g.splits; sp++) {   // loads of several splits in flight; the additions keep split order
      const float4 p = part[(size_t)sp * total4 + o4];
      v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
    }
    const int64_t o = (int64_t)o4 * 4;
    float f[4] = {v.x, v.y, v.z, v.w};
    if (ep.has_bias) {
      const int n = (int)((o4 * 4u) % (uint32_t)g.Ncols);
#pragma unroll
      for (int e = 0; e < 4; e++) f[e] += bf2f(bias[n + e]);
    }
    if (ep.relu) {
#pragma unroll
      for (int e = 0; e < 4; e++) f[e] = fmaxf(f[e], 0.f);
    }
    if (ep.use_mask) {
      const uint2 mk = *reinterpret_cast<const uint2*>(mask + o);
      const bf16_t m4[4] = {(bf16_t)(mk.x & 0xffffu), (bf16_t)(mk.x >> 16), (bf16_t)(mk.y & 0xffffu), (bf16_t)(mk.y >> 16)};
#pragma unroll
      for (int e = 0; e < 4; e++)
        if (!(bf2f(m4[e]) > 0.f)) f[e] = 0.f;
    }
    if (ep.out_f32) {
      reinterpret_cast<float4*>(out)[o4] = make_float4(f[0], f[1], f[2], f[3]);
    } else {
      uint2 w;
      w.x = (uint32_t)f2bf(f[0]) | ((uint32_t)f2bf(f[1]) << 16);
      w.y = (uint32_t)f2bf(f[2]) | ((uint32_t)f2bf(f[3]) << 16);
      *reinterpret_cast<uint2*>(out + o) = w;
    }
  }
}

int choose_splits(int64_t tiles, int count, int steps, size_t bytes_per_split, size_t scratch_bytes, int64_t target) {
  // target = workgroups wanted per launch; 600 by default (256..1024 measured, flat between 400 and 768 at 6 and 18 learners)
  int64_t sp = (target + tiles * count - 1) / (tiles * count);
  if (sp > steps / 4) sp = steps / 4;                // keep at least four contraction steps per workgroup
  if (bytes_per_split > 0 && (int64_t)(scratch_bytes / bytes_per_split) < sp) sp = (int64_t)(scratch_bytes / bytes_per_split);
  if (sp > 64) sp = 64;
  return sp < 2 ? 1 : (int)sp;
}

template <int BM, int BN, int WM, int WN, bool BT>
static void launch_igemm_t(const PtrTab& ws, const CPtrTab& wts, const IGemm& g, const Epilogue& ep, int count, hipStream_t s) {
  dim3 grid((unsigned)((g.M + BM - 1) / BM), (unsigned)((g.Ncols + BN - 1) / BN), (unsigned)(count * g.splits));
  hipLaunchKernelGGL((igemm_kernel<BM, BN, WM, WN, BT>), grid, dim3(256), 0, s, ws, wts, g, ep);
  if (g.splits > 1) {
    int64_t total = ((int64_t)g.M * g.Ncols) >> 2;
    unsigned blocks = (unsigned)((total + 255) / 256 < 2048 ? (total + 255) / 256 : 2048);
    hipLaunchKernelGGL(igemm_finish_kernel, dim3(blocks, 1, (unsigned)count), dim3(256), 0, s, ws, wts, g, ep);
  }
}

template <int BM, int BN, int WM, int WN>
static void launch_frag_t(const PtrTab& ws, const CPtrTab& wts, const IGemm& g_in, const Epilogue& ep, int count, hipStream_t s) {
  IGemm g = g_in;
  {
    // a split of up to six ways is not worth its second pass once the tiles alone take a fifth of the resident places
    const int64_t tiles = (int64_t)((g.M + BM - 1) / BM) * ((g.Ncols + BN - 1) / BN) * count;
    const int64_t places = 256 * (WM * WN > 64 * 64 ? 2 : 3);
    if (g.splits <= 6 && tiles * 5 >= places) g.splits = 1;
  }
  dim3 grid((unsigned)((g.M + BM - 1) / BM), (unsigned)((g.Ncols + BN - 1) / BN), (unsigned)(count * g.splits));
  constexpr int NT = 64 * (BM / WM) * (BN / WN);
  const bool uni = g.CPT % 4 == 0 && g.ks * g.ks <= 32 && g.Kchunks % 4 == 0;
  if (uni) hipLaunchKernelGGL((igemm_frag_kernel<BM, BN, WM, WN, 32, NT, true>), grid, dim3(NT), 0, s, ws, wts, g, ep);
  else hipLaunchKernelGGL((igemm_frag_kernel<BM, BN, WM, WN, 32, NT, false>), grid, dim3(NT), 0, s, ws, wts, g, ep);
  if (g.splits > 1) {
    int64_t total = ((int64_t)g.M * g.Ncols) >> 2;
    unsigned blocks = (unsigned)((total + 255) / 256 < 2048 ? (total + 255) / 256 : 2048);
    hipLaunchKernelGGL(igemm_finish_kernel, dim3(blocks, 1, (unsigned)count), dim3(256), 0, s, ws, wts, g, ep);
  }
}

// Convolution forward / input gradient with fragment-packed filters (g.b_off points at the fragment copy).
// The patch-in-LDS kernel applies to windows larger than 1 x 1 over a multiple of 32 channels whose patch (plus the
// pixel table, 84 bytes per pixel) fits 64 KiB of LDS; the contraction is split at most once per channel chunk.
template <int BM, int BN, int WM, int WN>
static bool launch_halo_t(const PtrTab& ws, const CPtrTab& wts, const IGemm& g_in, const Epilogue& ep, int count, bool xcd_order, hipStream_t s) {
  if (g_in.ks < 2 || g_in.C % 32 || g_in.OW + g_in.ks - 1 != g_in.W + 2 * g_in.pad) return false;
  IGemm g = g_in;
  g.splits = std::min(g.splits, g.C / 32);
  {
    // A split of up to six ways is not worth its partials and second pass once the tiles alone take a fifth of the
    // resident places (conv5 forward of the AlexNet shape at 18 learners, 396 tiles on 512 places: 92 us unsplit against
    // 104 + 25 us; conv3 forward at 8 learners, 264 tiles: two-way split 60 + 18 us for the second pass; over a run of
    // config 4 the calcGradient phase takes 0.230 ms per update with this rule against 0.237 ms when only two-way
    // splits of tiles filling 60 % of the places were dropped, and 0.233 ms when nothing is split)
    const int64_t tiles = (int64_t)((g.M + BM - 1) / BM) * ((g.Ncols + BN - 1) / BN) * count;
    const int64_t places = 256 * (WM * WN > 64 * 64 ? 2 : 3);
    if (g.splits <= 6 && tiles * 5 >= places) g.splits = 1;
  }
  HaloArgs h;
  h.PW = g.OW + g.ks - 1;
  h.xcd = xcd_order ? 1 : 0;
  h.mg_pw = magic_u32(h.PW);
  const int rows = (BM + g.OW - 2) / g.OW + 1;               // output rows a tile of BM positions can touch
  const int images = (rows + g.OH - 2) / g.OH + 1;           // and images those rows can belong to
  h.n_px_max = (rows + (g.ks - 1) * images) * h.PW;
  constexpr int NT = 64 * (BM / WM) * (BN / WN);
  const size_t stage = (size_t)(NT / 64) * 32 * (WN + 8) * 2;   // the epilogue's staging pieces
  const size_t slot_round = (size_t)NT * 16;                 // bytes one refill instruction per thread covers
  h.tab_off = (int)(((size_t)h.n_px_max * 80 + slot_round - 1) / slot_round * slot_round);
  const size_t bytes = std::max((size_t)h.tab_off + (size_t)h.n_px_max * 4, stage);
  if (bytes > 64 * 1024) return false;
  dim3 grid((unsigned)((g.M + BM - 1) / BM), (unsigned)((g.Ncols + BN - 1) / BN), (unsigned)(count * g.splits));
  hipLaunchKernelGGL((conv_halo_kernel<BM, BN, WM, WN>), grid, dim3(NT), bytes, s, ws, wts, g, ep, h);
  if (g.splits > 1) {
    int64_t total = ((int64_t)g.M * g.Ncols) >> 2;
    unsigned blocks = (unsigned)((total + 255) / 256 < 2048 ? (total + 255) / 256 : 2048);
    hipLaunchKernelGGL(igemm_finish_kernel, dim3(blocks, 1, (unsigned)count), dim3(256), 0, s, ws, wts, g, ep);
  }
  return true;
}

// Layers over 8 channels, or over a multiple of 16 (not of 32, at most 112) with windows of 4 x 4 and more:
// conv_halo_seq_kernel, if one tile's patch fits 64 KiB of LDS.  CIFAR-shaped conv1 (5 x 5 over 3 -> 8 channels, 18
// learners x 128 images): 63 us against 95 us for the tap-by-tap gather.
template <int BM, int BN, int WM, int WN>
static bool launch_halo_seq_t(const PtrTab& ws, const CPtrTab& wts, const IGemm& g_in, const Epilogue& ep, int count, hipStream_t s) {
  const bool c8 = g_in.C == 8;
  // (with 3 x 3 windows over 48 channels, the first layer of the AlexNet shape after space-to-depth, one fill of the
  // 50 KiB patch per tile costs more than nine-fold reuse saves: 155 us against 140 us for the tap-by-tap gather)
  if (g_in.ks < 2 || !(c8 || (g_in.C % 16 == 0 && g_in.C % 32 != 0 && g_in.C <= 112 && g_in.ks >= 4)) ||
      g_in.OW + g_in.ks - 1 != g_in.W + 2 * g_in.pad)
    return false;
  IGemm g = g_in;
  const int all_steps = (g.ldb / 16 + 1) / 2;
  g.splits = std::min(g.splits, std::max(1, all_steps / 2));
  {
    const int64_t tiles = (int64_t)((g.M + BM - 1) / BM) * ((g.Ncols + BN - 1) / BN) * count;
    const int64_t places = 256 * (WM * WN > 64 * 64 ? 2 : 3);
    if (g.splits <= 6 && tiles * 5 >= places) g.splits = 1;
  }
  HaloSeqArgs h;
  h.PW = g.OW + g.ks - 1;
  h.mg_pw = magic_u32(h.PW);
  h.spp = c8 ? 1 : g.C / 8 + 1;
  h.mg_spp = magic_u32(h.spp);
  h.pixb = 16 * h.spp;
  h.C16 = c8 ? 1 : g.C / 16;
  h.mg_c16 = magic_u32(h.C16);
  const int rows = (BM + g.OW - 2) / g.OW + 1;
  const int images = (rows + g.OH - 2) / g.OH + 1;
  h.n_px_max = (rows + (g.ks - 1) * images) * h.PW;
  constexpr int NT = 64 * (BM / WM) * (BN / WN);
  const size_t stage = (size_t)(NT / 64) * 32 * (WN + 8) * 2;
  const size_t slot_round = (size_t)NT * 16;
  h.tab_off = (int)(((size_t)h.n_px_max * h.pixb + slot_round - 1) / slot_round * slot_round);
  const size_t bytes = std::max((size_t)h.tab_off + (size_t)h.n_px_max * 4, stage);
  if (bytes > 64 * 1024) return false;
  dim3 grid((unsigned)((g.M + BM - 1) / BM), (unsigned)((g.Ncols + BN - 1) / BN), (unsigned)(count * g.splits));
  if (c8) hipLaunchKernelGGL((conv_halo_seq_kernel<BM, BN, WM, WN, true>), grid, dim3(NT), bytes, s, ws, wts, g, ep, h);
  else hipLaunchKernelGGL((conv_halo_seq_kernel<BM, BN, WM, WN, false>), grid, dim3(NT), bytes, s, ws, wts, g, ep, h);
  if (g.splits > 1) {
    int64_t total = ((int64_t)g.M * g.Ncols) >> 2;
    unsigned blocks = (unsigned)((total + 255) / 256 < 2048 ? (total + 255) / 256 : 2048);
    hipLaunchKernelGGL(igemm_finish_kernel, dim3(blocks, 1, (unsigned)count), dim3(256), 0, s, ws, wts, g, ep);
  }
  return true;
}

hipError_t launch_igemm_frag(const PtrTab& ws, const CPtrTab& wts, const IGemm& g, const Epilogue& ep, int count, hipStream_t s) {
  if (g.C % 8 || g.ldb % 32 || g.splits < 1) return hipErrorInvalidValue;
  if (g.C % 32 != 0) {
    bool done;
    if (g.Ncols <= 32) {
      const bool many = (int64_t)((g.M + 255) / 256) * count >= 1024;
      done = many ? launch_halo_seq_t<256, 32, 64, 32>(ws, wts, g, ep, count, s) : launch_halo_seq_t<128, 32, 32, 32>(ws, wts, g, ep, count, s);
    } else if (g.Ncols <= 64) {
      done = launch_halo_seq_t<128, 64, 64, 32>(ws, wts, g, ep, count, s);
    } else {
      done = launch_halo_seq_t<128, 128, 64, 64>(ws, wts, g, ep, count, s);
    }
    if (done) return hipGetLastError();
  }
  // own: most learners of this call read a weight version of their own (lambda-softsync) rather than a shared one
  int same = 0;
  for (int k = 1; k < count; k++) same += wts.p[k] == wts.p[0] ? 1 : 0;
  const bool own = count > 1 && 2 * same < count;
  // Narrow layers: 256-row tiles (64 x 32 per wavefront) once there are enough of them to fill the chip, else 128 rows.
  // Measured on the CIFAR-shaped layers (18 learners x 128 images): 5x5 over 32 channels, 16x16 images, 39 us against
  // 46 us with 128-row tiles and 68 us for the tap-by-tap gather; 8x8 images 27 us against 33 us and 43 us.
  if (g.Ncols <= 32) {
    const bool many = (int64_t)((g.M + 255) / 256) * count >= 1024;
    const bool done = many ? launch_halo_t<256, 32, 64, 32>(ws, wts, g, ep, count, own, s) : launch_halo_t<128, 32, 32, 32>(ws, wts, g, ep, count, own, s);
    if (done) return hipGetLastError();
  } else if (g.Ncols <= 64) {
    if (launch_halo_t<128, 64, 64, 32>(ws, wts, g, ep, count, own, s)) return hipGetLastError();
  }
  if (g.Ncols > 64) {
    // (measured slower for the 128-wide layers: 128 x 64 wave tiles in blocks of two wavefronts, and 256 x 128 blocks)
    // Learners on one weight version share their filter fragments in every L2 and 128-row tiles spread over all XCDs
    // are fastest (conv3 forward, 18 learners: 89 us; 101 us with the XCD-contiguous order, 105 us with 256 rows).  With
    // a version per learner the fragments are the larger part of a workgroup's traffic: 256-row tiles read them half as
    // often and the XCD-contiguous order keeps a learner's tiles on one L2 (101 us against 120 us).  Also measured
    // slower in both cases: 128 x 64 wave tiles in two-wavefront blocks, eight-wavefront 256 x 128 blocks, 256 x 256.
    const bool done = g.Ncols % 256 == 0 ? launch_halo_t<128, 256, 128, 64>(ws, wts, g, ep, count, own, s)
                      : own && g.Ncols > 128 ? launch_halo_t<256, 128, 128, 64>(ws, wts, g, ep, count, own, s)
                                             : launch_halo_t<128, 128, 64, 64>(ws, wts, g, ep, count, own, s);
    if (done) return hipGetLastError();
  }
  // Wave tile 128 x 64 (two wavefronts per SIMD, accumulators in ordinary registers) wins where the columns fill
  // whole 256-wide tiles: each B fragment then serves four MFMAs instead of two.  Measured slower: 256 x 128 blocks,
  // 192-wide tiles of three wavefronts for 384 columns, 96-wide tiles for 96 columns, and taking the filters
  // through LDS as well (tiles 128 x 128 to 256 x 256, staging registers two steps deep): with both operands in
  // LDS its bandwidth becomes the limit instead of the vector L1's.
  if (g.Ncols <= 32) launch_frag_t<128, 32, 32, 32>(ws, wts, g, ep, count, s);
  else if (g.Ncols <= 64) launch_frag_t<128, 64, 64, 32>(ws, wts, g, ep, count, s);
  else if (g.Ncols % 256 == 0) launch_frag_t<128, 256, 128, 64>(ws, wts, g, ep, count, s);
  else launch_frag_t<128, 128, 64, 64>(ws, wts, g, ep, count, s);
  return hipGetLastError();
}

hipError_t launch_igemm(const PtrTab& ws, const CPtrTab& wts, const IGemm& g_in, const Epilogue& ep, bool b_transposed, int count,
                        hipStream_t s) {
  const IGemm& g = g_in;
  if (g.C % 8 || g.ldb % 8 || (b_transposed && g.Ncols % 8) || g.splits < 1) return hipErrorInvalidValue;
  if (g.M <= 32) {
    // input gradient of a wide fully connected layer: 512-byte pieces of the weight rows (236 us against 252 us)
    if (b_transposed && g.Ncols >= 1024) launch_igemm_t<32, 256, 32, 64, true>(ws, wts, g, ep, count, s);
    else if (b_transposed) launch_igemm_t<32, 128, 32, 32, true>(ws, wts, g, ep, count, s);
    else launch_igemm_t<32, 128, 32, 32, false>(ws, wts, g, ep, count, s);
  } else if (g.Ncols <= 32) {
    if (b_transposed) launch_igemm_t<128, 32, 32, 32, true>(ws, wts, g, ep, count, s);
    else launch_igemm_t<128, 32, 32, 32, false>(ws, wts, g, ep, count, s);
  } else if (g.Ncols <= 64) {
    if (b_transposed) launch_igemm_t<128, 64, 64, 32, true>(ws, wts, g, ep, count, s);
    else launch_igemm_t<128, 64, 64, 32, false>(ws, wts, g, ep, count, s);
  } else {
    if (b_transposed) launch_igemm_t<128, 128, 64, 64, true>(ws, wts, g, ep, count, s);
    else launch_igemm_t<128, 128, 64, 64, false>(ws, wts, g, ep, count, s);
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------ weight gradient
// dW tile [BMG output channels][BNG im2col columns], contraction over output positions m in steps of 32.
// dy tile  [32 m][BMG n]  and  im2col tile [32 m][BNG k]  are staged as they lie in memory (rows = m) and
// read with the transpose load.  The result is scattered into the flat fp32 gradient through filter_src().
// INCR: the output position (image, oh, ow) of a thread's tile row advances from step to step by additions and
// two conditional wraps (possible when 32 / OW + 1 <= OH); otherwise it is decoded from the row index every step.
template <int BMG, int BNG, int WMG, int WNG, bool INCR>
__global__ __launch_bounds__(256) void igemm_wgrad_kernel(PtrTab ws, PtrTab grads, IGemm g, VConv v, size_t dy_off, int64_t w_off,
                                                          int64_t b_off, int partial) {
  constexpr int WAVES_NG = BNG / WNG;                  // four wavefronts: (BMG / WMG) x (BNG / WNG)
  constexpr int TM = WMG / 32, TN = WNG / 32;
  constexpr int LDT_A = BMG + 32 - (BMG == 32 ? 32 : 0);
  constexpr int LDT_B = BNG + 32 - (BNG == 32 ? 32 : 0);
  constexpr int A_ELEMS = BK * LDT_A, B_ELEMS = BK * LDT_B;
  __shared__ __attribute__((aligned(16))) bf16_t lds[2 * (A_ELEMS + B_ELEMS)];

  const TileIdx tile = xcd_tile(1);   // a learner's tiles share dy and x: keep them on one XCD's L2 (AlexNet layers 3-9 % faster)
  const int z = tile.z / g.splits, sp = tile.z % g.splits;
  const bf16_t* x = (const bf16_t*)ws.p[z] + g.a_off;
  const bf16_t* dy = (const bf16_t*)ws.p[z] + dy_off;
  const int n0 = tile.x * BMG, k0 = tile.y * BNG;           // output-channel and im2col-column origins
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave / WAVES_NG) * WMG, wn0 = (wave % WAVES_NG) * WNG;

  constexpr int CPR_A = BMG / 8, CPR_B = BNG / 8;
  constexpr int TPR = 256 / BK;                        // threads per tile row of the im2col tile
  constexpr int A_LOADS = (BK * CPR_A + 255) / 256, B_LOADS = CPR_B / TPR;
  static_assert(CPR_B % TPR == 0, "im2col tile: whole chunks per thread");
  const int all_steps = (g.M + BK - 1) / BK;
  const int per = (all_steps + g.splits - 1) / g.splits;
  const int ms_begin = __builtin_amdgcn_readfirstlane(sp * per);
  const int msteps = __builtin_amdgcn_readfirstlane(min(all_steps, ms_begin + per));

  // Hardware-bounds-checked buffer loads (an offset at or beyond the tensor reads as zero): rows beyond M, columns
  // beyond the layer and taps in the zero padding need no branch and no patching of loaded data.
  const __amdgpu_buffer_rsrc_t rsrc_dy = __builtin_amdgcn_make_buffer_rsrc((void*)dy, 0, (int)((int64_t)g.M * g.Ncols * 2), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc((void*)x, 0, (int)g.a_bytes, 0x00020000);
  // dy tile: chunk (row r, 8 channels from n) per thread; its offset advances by a constant every step
  uint32_t a_off[A_LOADS];
  const uint32_t a_step = (uint32_t)(BK * g.Ncols * 2);
#pragma unroll
  for (int i = 0; i < A_LOADS; i++) {
    const int idx = tid + 256 * i;
    const int r = idx / CPR_A, n = n0 + (idx % CPR_A) * 8;
    a_off[i] = (r < BK && n < g.Ncols) ? (uint32_t)((((int64_t)ms_begin * BK + r) * g.Ncols + n) * 2) : kOutOfRange;
  }
  // im2col tile: a thread owns B_LOADS chunks of ONE tile row; their filter taps are fixed, only the row's output
  // position changes from step to step
  const int b_row = tid / TPR;
  int b_dkh[B_LOADS], b_dkw[B_LOADS], b_koff[B_LOADS];
  bool b_ok[B_LOADS], b_ones[B_LOADS];
#pragma unroll
  for (int i = 0; i < B_LOADS; i++) {
    const int q = k0 / 8 + tid % TPR + TPR * i;
    const uint32_t tap = fastdiv((uint32_t)q, g.CPT, g.mg_cpt);
    const int c8 = q - (int)tap * g.CPT;
    const int kh = (int)fastdiv(tap, g.ks, g.mg_ks), kw = (int)tap - kh * g.ks;
    b_dkh[i] = kh - g.pad;
    b_dkw[i] = kw - g.pad;
    b_koff[i] = ((b_dkh[i] * g.W + b_dkw[i]) * g.C + c8 * 8) * 2;
    b_ok[i] = q < g.Kchunks;
    b_ones[i] = q == g.Kchunks;                  // the bias column: im2col value 1 for every real output position
  }
  // position of the row that load_regs fetches next: m, its (oh, ow) and the byte offset of x[image][oh][ow][0]
  int r_m = ms_begin * BK + b_row, r_oh, r_ow, r_off;
  auto decode_row = [&]() {
    const uint32_t mm = r_m < g.M ? (uint32_t)r_m : 0u;
    const uint32_t rest = fastdiv(mm, g.OW, g.mg_ow);
    const uint32_t n = fastdiv(rest, g.OH, g.mg_oh);
    r_ow = (int)(mm - rest * (uint32_t)g.OW);
    r_oh = (int)(rest - n * (uint32_t)g.OH);
    r_off = (int)(((n * (uint32_t)g.H + (uint32_t)r_oh) * (uint32_t)g.W + (uint32_t)r_ow) * (uint32_t)g.C * 2u);
  };
  decode_row();
  const int d_ow = BK / g.OW, m_ow = BK - d_ow * g.OW;          // 32 rows further: d_ow lines down, m_ow positions right
  const int inc0 = (d_ow * g.W + m_ow) * g.C * 2;               // the same in bytes of x
  const int inc_w = (g.W - g.OW) * g.C * 2;                      // extra when ow wraps into the next line
  const int inc_h = (g.H - g.OH) * g.W * g.C * 2;                // extra when oh wraps into the next image

  v4i_t ra[A_LOADS], rb[B_LOADS];
  uint32_t bias_one[B_LOADS];
  auto load_regs = [&]() {
#pragma unroll
    for (int i = 0; i < A_LOADS; i++) {
      ra[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_dy, (int)a_off[i], 0, 0);
      a_off[i] += a_step;
    }
    const bool valid = r_m < g.M;
#pragma unroll
    for (int i = 0; i < B_LOADS; i++) {
      const bool ok = b_ok[i] && valid && (unsigned)(r_oh + b_dkh[i]) < (unsigned)g.H && (unsigned)(r_ow + b_dkw[i]) < (unsigned)g.W;
      rb[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, ok ? r_off + b_koff[i] : (int)kOutOfRange, 0, 0);
      bias_one[i] = (b_ones[i] && valid) ? 0x3F80u : 0u;
    }
    // advance the row by BK output positions
    r_m += BK;
    if (INCR) {
      r_ow += m_ow;
      const bool c1 = r_ow >= g.OW;
      r_ow -= c1 ? g.OW : 0;
      r_oh += d_ow + (c1 ? 1 : 0);
      const bool c2 = r_oh >= g.OH;
      r_oh -= c2 ? g.OH : 0;
      r_off += inc0 + (c1 ? inc_w : 0) + (c2 ? inc_h : 0);
    } else {
      decode_row();
    }
  };
  auto store_lds = [&](int buf) {
    bf16_t* A = lds + buf * (A_ELEMS + B_ELEMS);
    bf16_t* B = A + A_ELEMS;
#pragma unroll
    for (int i = 0; i < A_LOADS; i++) {
      int idx = tid + 256 * i;
      int r = idx / CPR_A, ch = idx % CPR_A;
      if (BK * CPR_A % 256 == 0 || r < BK) *reinterpret_cast<v4i_t*>(A + r * LDT_A + ch * 8) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < B_LOADS; i++) {
      v4i_t val = rb[i];
      val.x |= (int)bias_one[i];                 // the chunk of the bias column loads as zeros; its first element becomes 1.0
      *reinterpret_cast<v4i_t*>(B + b_row * LDT_B + (tid % TPR + TPR * i) * 8) = val;
    }
  };

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

  const int j16 = lane & 15, half = (lane >> 4) & 1;
  // One step: the tiles of step ms+1 (fetched during step ms-1) go to the other LDS buffer, the tiles of step ms+2 are
  // requested, then the MFMAs run on buffer `buf`: a global load has a whole step to arrive.  Two steps per loop
  // iteration make `buf` a constant.
  auto step = [&](int buf, bool has1, bool has2) {
    const bf16_t* A = lds + buf * (A_ELEMS + B_ELEMS);
    const bf16_t* B = A + A_ELEMS;
#pragma unroll
    for (int kk = 0; kk < 2; kk++) {
      const int kb = 16 * kk + 8 * (lane >> 5);
      bf16x8 a[TM], b[TN];
#pragma unroll
      for (int i = 0; i < TM; i++) {
        const bf16_t* p = A + (kb + (j16 >> 2)) * LDT_A + wm0 + 32 * i + 16 * half + 4 * (j16 & 3);
        union { bf16x8 v; shortx4 h[2]; } u;
        u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((shortx4 __attribute__((address_space(3)))*)(p));
        u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((shortx4 __attribute__((address_space(3)))*)(p + 4 * LDT_A));
        a[i] = u.v;
      }
#pragma unroll
      for (int j = 0; j < TN; j++) {
        const bf16_t* p = B + (kb + (j16 >> 2)) * LDT_B + wn0 + 32 * j + 16 * half + 4 * (j16 & 3);
        union { bf16x8 v; shortx4 h[2]; } u;
        u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((shortx4 __attribute__((address_space(3)))*)(p));
        u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((shortx4 __attribute__((address_space(3)))*)(p + 4 * LDT_B));
        b[j] = u.v;
      }
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    // the wait for the next tiles' global loads falls behind this step's MFMAs instead of in front of its LDS reads
    __builtin_amdgcn_sched_barrier(0);
    if (has1) store_lds(buf ^ 1);
    if (has2) load_regs();
    __syncthreads();
  };

  int ms = ms_begin;
  if (ms < msteps) {
    load_regs();
    store_lds(0);
    if (ms + 1 < msteps) load_regs();
  }
  __syncthreads();
  for (; ms + 3 < msteps; ms += 2) {            // no branch around the loads inside the loop
    step(0, true, true);
    step(1, true, true);
  }
  for (; ms + 1 < msteps; ms += 2) {            // at most once: two or three steps remain
    step(0, true, ms + 2 < msteps);
    step(1, ms + 2 < msteps, false);
  }
  if (ms < msteps) step(0, false, false);

  const int kcols = g.Kchunks * 8;
  if (partial) {   // fp32 partial [split][n][kcols + 8]; wgrad_finish_kernel adds and writes the flat gradient in its order
    const int ldk = kcols + 8;
    float* part = reinterpret_cast<float*>((char*)ws.p[z] + g.scratch_off) + (int64_t)sp * g.Ncols * ldk;
#pragma unroll
    for (int j = 0; j < TN; j++) {
      const int k = k0 + wn0 + 32 * j + (lane & 31);
      if (k > kcols) continue;
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const int n = n0 + wm0 + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          if (n < g.Ncols) part[(int64_t)n * ldk + k] = acc[i][j][r];
        }
    }
    return;
  }
  float* dw = (float*)grads.p[z] + w_off;
  float* db = (float*)grads.p[z] + b_off;
  if (v.ks == 1 && v.s2d == 1 && v.C == v.Creal) {
    // fully connected layer: dW[n][k] is the tile itself, row length C; 32 lanes write 128 contiguous bytes
#pragma unroll
    for (int j = 0; j < TN; j++) {
      const int k = k0 + wn0 + 32 * j + (lane & 31);
      if (k > kcols) continue;
#pragma unroll
      for (int i = 0; i < TM; i++) {
        const int nb = n0 + wm0 + 32 * i + 4 * (lane >> 5);
        float* row = dw + (int64_t)nb * v.C + k;
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const int dn = 8 * (r >> 2) + (r & 3);
          if (nb + dn >= g.Ncols) continue;
          if (k == kcols) db[nb + dn] = acc[i][j][r];
          else row[(int64_t)dn * v.C] = acc[i][j][r];
        }
      }
    }
    return;
  }
#pragma unroll
  for (int j = 0; j < TN; j++) {
    const int k = k0 + wn0 + 32 * j + (lane & 31);       // im2col column = tap * C + cp; column kcols = bias
    if (k > kcols) continue;
    const int tap = k / g.C, cp = k - tap * g.C;
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int n = n0 + wm0 + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (n >= g.Ncols) continue;
        if (k == kcols) { db[n] = acc[i][j][r]; continue; }
        const int64_t dst = filter_src(v, n, tap, cp);
        if (dst >= 0) dw[dst] = acc[i][j][r];
      }
  }
}

// One workgroup per output channel n: the row of partial sums is added in split order into LDS (coalesced reads),
// then written to the flat gradient in ITS order (coalesced writes), the im2col column of each filter element
// being looked up on the way.
__global__ __launch_bounds__(256) void wgrad_finish_kernel(PtrTab ws, PtrTab grads, IGemm g, VConv v, int64_t w_off, int64_t b_off,
                                                           int cgroup) {
  extern __shared__ float row[];                 // sums of this workgroup's columns
  const int z = blockIdx.z, n = blockIdx.x;
  const int kcols = g.Kchunks * 8, ldk = kcols + 8;
  const float* part = reinterpret_cast<const float*>((const char*)ws.p[z] + g.scratch_off) + (int64_t)n * ldk;
  const int64_t split_stride = (int64_t)g.Ncols * ldk;
  float* dw = (float*)grads.p[z] + w_off + (int64_t)n * v.Creal * v.ksr * v.ksr;
  if (blockIdx.y == 0 && threadIdx.x == 0) {     // bias gradient: the extra im2col column
    float acc = 0.f;
    for (int sp = 0; sp < g.splits; sp++) acc += part[sp * split_stride + kcols];
    ((float*)grads.p[z] + b_off)[n] = acc;
  }
  if (v.s2d == 1) {
    // channels [c_lo, c_hi) of this filter, all taps: columns tap * C + c are read tap by tap (contiguous runs), the
    // run [c_lo * T, c_hi * T) of the flat gradient is written in its own order
    const int T = v.ks * v.ks;
    const int c_lo = blockIdx.y * cgroup, c_hi = min(v.Creal, c_lo + cgroup), cw = c_hi - c_lo;
    if (cw <= 0) return;
    for (int idx = threadIdx.x; idx < T * cw; idx += 256) {
      const int tap = idx / cw, cc = idx - tap * cw;
      const int k = tap * g.C + c_lo + cc;
      float acc = 0.f;
#pragma unroll 8
      for (int sp = 0; sp < g.splits; sp++) acc += part[sp * split_stride + k];
      row[idx] = acc;
    }
    __syncthreads();
    for (int j = threadIdx.x; j < T * cw; j += 256) {
      const int cc = j / T, tap = j - cc * T;
      dw[(int64_t)c_lo * T + j] = row[tap * cw + cc];
    }
    return;
  }
  // first layer seen through a space-to-depth input (a small filter): one thread per im2col column, blockIdx.y
  // selects a run of 256 columns; the column's place in the flat filter is looked up and written on its own
  const int k = blockIdx.y * 256 + threadIdx.x;
  if (k >= kcols) return;
  const int tap = k / g.C, cp = k - tap * g.C;
  const int64_t dst = filter_src(v, 0, tap, cp);          // position inside one filter, or -1 for padding
  if (dst < 0) return;
  float acc = 0.f;
#pragma unroll 8
  for (int sp = 0; sp < g.splits; sp++) acc += part[sp * split_stride + k];
  dw[dst] = acc;
}

hipError_t launch_igemm_wgrad(const PtrTab& ws, const PtrTab& grads, const IGemm& g, const VConv& v, size_t dy_off, int64_t w_off,
                              int64_t b_off, int count, hipStream_t s) {
  if (g.C % 8 || g.Ncols % 8 || g.splits < 1) return hipErrorInvalidValue;
  const int cols = g.Kchunks * 8 + 1;          // im2col columns plus the bias column
  const bool incr = BK / g.OW + 1 <= g.OH;      // one wrap of oh per step at most
  // A convolution's tile holds one tap of many channels, the flat gradient wants all taps of one channel together:
  // written straight from the tile every 4-byte element lands alone and every cache line is completed by as many
  // workgroups as the window has taps (measured: 65-125 us per AlexNet layer at 18 learners).  So convolutions
  // always go through the partial buffer and the second pass, which reads and writes whole lines (28-51 us).
  const bool conv = v.ks > 1 || v.s2d > 1;
  const int partial = (g.splits > 1 || conv) ? 1 : 0;
#define SASGD_WGRAD(BMG, BNG, WMG, WNG)                                                                                          \
  do {                                                                                                                           \
    if (incr) hipLaunchKernelGGL((igemm_wgrad_kernel<BMG, BNG, WMG, WNG, true>), grid, dim3(256), 0, s, ws, grads, g, v, dy_off, w_off, b_off, partial); \
    else hipLaunchKernelGGL((igemm_wgrad_kernel<BMG, BNG, WMG, WNG, false>), grid, dim3(256), 0, s, ws, grads, g, v, dy_off, w_off, b_off, partial);    \
  } while (0)
  if (g.Ncols <= 32) {
    dim3 grid(1, (unsigned)((cols + 127) / 128), (unsigned)(count * g.splits));
    SASGD_WGRAD(32, 128, 32, 32);
  } else if (g.Ncols <= 64) {
    dim3 grid(1, (unsigned)((cols + 127) / 128), (unsigned)(count * g.splits));
    SASGD_WGRAD(64, 128, 32, 64);
  } else {
    dim3 grid((unsigned)((g.Ncols + 127) / 128), (unsigned)((cols + 127) / 128), (unsigned)(count * g.splits));
    SASGD_WGRAD(128, 128, 64, 64);
  }
#undef SASGD_WGRAD
  if (partial) {
    // enough workgroups to keep the chip busy: the channels of a filter are divided among several of them
    int groups = (cols + 254) / 256, cgroup = v.Creal;   // space-to-depth first layer: runs of 256 columns, no LDS
    size_t lds = 0;
    if (v.s2d == 1) {
      groups = (int)((1536 + (int64_t)g.Ncols * count - 1) / ((int64_t)g.Ncols * count));
      if (groups > v.Creal / 8) groups = v.Creal / 8;
      if (groups < 1) groups = 1;
      cgroup = (v.Creal + groups - 1) / groups;
      const int cap = 15360 / (v.ks * v.ks);       // 60 KiB of sums per workgroup
      if (cgroup > cap) cgroup = cap < 1 ? 1 : cap;
      groups = (v.Creal + cgroup - 1) / cgroup;
      lds = (size_t)cgroup * v.ks * v.ks * sizeof(float);
    }
    hipLaunchKernelGGL(wgrad_finish_kernel, dim3((unsigned)g.Ncols, (unsigned)groups, (unsigned)count), dim3(256), lds, s, ws, grads, g, v,
                       w_off, b_off, cgroup);
  }
  return hipGetLastError();
}

}  // namespace sasgd
