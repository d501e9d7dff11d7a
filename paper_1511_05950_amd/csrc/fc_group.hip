// Fully connected layers of calcGradient (Section 2.1) for small mini-batches, grouped by weight version.
//
// Under n-softsync several learners of one batched call often read the same weight version (Section 2.2: a learner
// pulls whatever version is current when it starts).  With mu <= 32 images per learner a fully connected layer uses
// every weight once per image row block, so the layer runs at the rate its weights stream in from HBM; reading them
// once per VERSION instead of once per learner is what grouping buys.  A group = learners of a call on one version, at
// most 128 image rows (more learners on a version are cut into several equal groups, whose reads of the same weights at
// the same time meet in the last-level cache); a learner alone is a group of one.  All groups of a call run in one launch (blockIdx.z =
// group x split): nothing is copied together, a row's address is looked up through its member's workspace pointer.
//
//   forward   y[m][n]  = sum_k x[m][k] W[n][k] + b[n]        W rows are contraction-major: streamed as they lie
//   dgrad     dx[m][c] = sum_n dy[m][n] W[n][c]              W rows are output-major: staged as they lie, read with the
//                                                            LDS transpose load
// Both walk the weights in 512-byte row pieces, 16 KiB per workgroup and step, and split the contraction over several
// workgroups when the groups alone do not fill the chip (partials in the first member's scratch, added in split order
// by fc_group_finish_kernel, so the result does not depend on scheduling).
#include <algorithm>
#include "dev_common.hpp"
#include "kernels.hpp"

namespace sasgd {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short shortx4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef int v4i_t __attribute__((ext_vector_type(4)));

namespace {

constexpr uint32_t kOutOfRange = 0x80000000u;   // buffer offset beyond any tensor: the load returns zeros
constexpr int FCK = 256;                        // contraction elements per forward step
constexpr int FCLD = FCK + 8;                   // LDS row stride (elements): 528 bytes, conflict-free 16-byte reads

__device__ __forceinline__ uint4 ld16(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }
// Workspace base of member q of the group whose first member is z0 (a per-lane lookup in the by-value pointer table).
__device__ __forceinline__ char* member_base(const PtrTab& ws, int z0, int q) { return (char*)ws.p[z0 + q]; }

}  // namespace

// ------------------------------------------------------------------ forward
// A workgroup owns 32 output units of one group and walks the contraction in steps of 256: 32 lanes fetch 512
// contiguous bytes of one weight row; the tile goes through LDS.  Each of the four wavefronts multiplies one quarter
// of the step (64 k) into R accumulators of 32 units x 32 image rows (R row blocks cover the group's rows), and the
// four are added at the end.  The image rows come straight from the members' workspaces (they stay in L2: every
// workgroup of the group reads the same rows).
template <int R>
__global__ __launch_bounds__(256) void fc_group_fwd_kernel(PtrTab ws, CPtrTab wts, GroupTab gt, IGemm g, Epilogue ep) {
  __shared__ __attribute__((aligned(16))) bf16_t lds[2 * 32 * FCLD];
  const int grp = blockIdx.z / g.splits, sp = blockIdx.z % g.splits;
  const int z0 = gt.first[grp], nm = gt.members[grp];
  const int Mg = nm * g.M;
  char* const lead = (char*)ws.p[z0];                // the first member: zeros and split partials live in its workspace
  const bf16_t* W = (const bf16_t*)wts.p[z0] + g.b_off;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n0 = blockIdx.x * 32;
  const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void*)W, 0, (int)((int64_t)g.Ncols * g.ldb * 2), 0x00020000);
  // loader: pass i fetches rows 8 i + tid / 32, 16 bytes at element 8 (tid % 32) of the step
  const int lrow = tid >> 5, lpiece = tid & 31;
  uint32_t woff[4];
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int n = n0 + 8 * i + lrow;
    woff[i] = n < g.Ncols ? (uint32_t)(((int64_t)n * g.ldb + 8 * lpiece) * 2) : kOutOfRange;
  }
  // image rows of this wavefront's quarter: lane (m, h) of row block rb holds x[32 rb + m][step + 64 wave + 16 j + 8 h ...];
  // rows beyond the group read the workspace's block of zeros and do not advance
  const int m = lane & 31, h = lane >> 5;
  const bf16_t* xrow[R];
  int xstep[R];
#pragma unroll
  for (int rb = 0; rb < R; rb++) {
    const int row = 32 * rb + m;
    const bool ok = row < Mg;
    const int q = ok ? row / g.M : 0;
    xrow[rb] = ok ? (const bf16_t*)member_base(ws, z0, q) + g.a_off + (int64_t)(row - q * g.M) * g.C + 64 * wave + 8 * h
                  : (const bf16_t*)lead + g.zero_off;
    xstep[rb] = ok ? FCK : 0;
  }

  const int steps_all = g.C / FCK;
  const int per = (steps_all + g.splits - 1) / g.splits;
  const int s_begin = __builtin_amdgcn_readfirstlane(sp * per);
  const int s_end = __builtin_amdgcn_readfirstlane(min(steps_all, s_begin + per));

  v4i_t rw[4];
  bf16x8 xb[R][4], xn[R][4];
  auto fetch_w = [&](int st) {
#pragma unroll
    for (int i = 0; i < 4; i++) rw[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, (int)woff[i], st * (FCK * 2), 0);
  };
  auto fetch_x = [&](bf16x8 (&dst)[R][4], int st) {
#pragma unroll
    for (int rb = 0; rb < R; rb++)
#pragma unroll
      for (int j = 0; j < 4; j++) dst[rb][j] = *reinterpret_cast<const bf16x8*>(xrow[rb] + (int64_t)st * xstep[rb] + 16 * j);
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; i++) *reinterpret_cast<v4i_t*>(lds + buf * (32 * FCLD) + (8 * i + lrow) * FCLD + 8 * lpiece) = rw[i];
  };
  floatx16 acc[R];
#pragma unroll
  for (int rb = 0; rb < R; rb++)
#pragma unroll
    for (int e = 0; e < 16; e++) acc[rb][e] = 0.f;

  int st = s_begin;
  if (st < s_end) {
    fetch_w(st);
    fetch_x(xb, st);
    stash(0);
    if (st + 1 < s_end) fetch_w(st + 1);
  }
  __syncthreads();
  for (int buf = 0; st < s_end; st++, buf ^= 1) {
    const bool has1 = st + 1 < s_end;
    if (has1) {
      stash(buf ^ 1);                   // the tile fetched during the previous step
      fetch_x(xn, st + 1);
    }
    if (st + 2 < s_end) fetch_w(st + 2);
    const bf16_t* A = lds + buf * (32 * FCLD) + m * FCLD + 64 * wave + 8 * h;
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(A + 16 * j);
#pragma unroll
      for (int rb = 0; rb < R; rb++) acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, xb[rb][j], acc[rb], 0, 0, 0);
    }
    if (has1) {
#pragma unroll
      for (int rb = 0; rb < R; rb++)
#pragma unroll
        for (int j = 0; j < 4; j++) xb[rb][j] = xn[rb][j];
    }
    __syncthreads();
  }

  // add the four wavefronts' accumulators: D[i][j], i = unit (MFMA row), j = image row (lane & 31)
  float* red = reinterpret_cast<float*>(lds);                   // [wave][16][64]: 16 KiB, the tiles are no longer needed
  const int q4 = wave;                                          // thread (q4, lane): units 8 q4 + 4 h .. + 3 of image row m
  const int n = n0 + 8 * q4 + 4 * h;
#pragma unroll
  for (int rb = 0; rb < R; rb++) {
    if (32 * rb >= Mg) break;                                   // uniform: the group has no rows in this block
#pragma unroll
    for (int e = 0; e < 16; e++) red[(wave * 16 + e) * 64 + lane] = acc[rb][e];
    __syncthreads();
    float f[4];
#pragma unroll
    for (int e = 0; e < 4; e++) {
      float v = 0.f;
#pragma unroll
      for (int w = 0; w < 4; w++) v += red[(w * 16 + 4 * q4 + e) * 64 + lane];
      f[e] = v;
    }
    __syncthreads();
    const int row = 32 * rb + m;
    if (row >= Mg || n >= g.Ncols) continue;
    if (g.splits > 1) {
      float* part = reinterpret_cast<float*>(lead + g.scratch_off) + ((int64_t)sp * Mg + row) * g.Ncols + n;
      *reinterpret_cast<float4*>(part) = make_float4(f[0], f[1], f[2], f[3]);
      continue;
    }
    const int q = row / g.M;
    bf16_t* out = (bf16_t*)member_base(ws, z0, q) + ep.out_off;
    const bf16_t* bias = (const bf16_t*)wts.p[z0] + ep.bias_off;
#pragma unroll
    for (int e = 0; e < 4; e++) {
      if (ep.has_bias) f[e] += bf2f(bias[n + e]);
      if (ep.relu) f[e] = fmaxf(f[e], 0.f);
    }
    const int64_t o = (int64_t)(row - q * g.M) * g.Ncols + n;
    if (ep.out_f32) {
      *reinterpret_cast<float4*>(reinterpret_cast<float*>(out) + o) = make_float4(f[0], f[1], f[2], f[3]);
    } else {
      uint2 w2;
      w2.x = (uint32_t)f2bf(f[0]) | ((uint32_t)f2bf(f[1]) << 16);
      w2.y = (uint32_t)f2bf(f[2]) | ((uint32_t)f2bf(f[3]) << 16);
      *reinterpret_cast<uint2*>(out + o) = w2;
    }
  }
}

// ------------------------------------------------------------------ input gradient
// Tile: BM image rows of one group (all of them) x 256 input units; contraction over the output units in steps of 32.
// The weight tile [32 units][256 inputs] is staged as it lies (512-byte row pieces) and read with the transpose load;
// the dy tile [BM][32] is gathered from the members' workspaces.  Four wavefronts, each BM x 64.
constexpr int GBK = 32;
constexpr int GLDA = GBK + 8;
constexpr int GBN = 256;
template <int BM>
__global__ __launch_bounds__(256) void fc_group_dgrad_kernel(PtrTab ws, CPtrTab wts, GroupTab gt, IGemm g, Epilogue ep) {
  constexpr int TM = BM / 32, TN = 2;
  constexpr int A_ELEMS = BM * GLDA, B_ELEMS = GBK * GBN;
  __shared__ __attribute__((aligned(16))) bf16_t lds[2 * (A_ELEMS + B_ELEMS)];
  const int grp = blockIdx.z / g.splits, sp = blockIdx.z % g.splits;
  const int z0 = gt.first[grp], nm = gt.members[grp];
  const int Mg = nm * g.M;
  char* const lead = (char*)ws.p[z0];                // the first member: zeros and split partials live in its workspace
  const bf16_t* zeros = (const bf16_t*)lead + g.zero_off;
  const bf16_t* Bm = (const bf16_t*)wts.p[z0] + g.b_off;
  const int n0 = blockIdx.x * GBN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wn0 = wave * 64;
  const int K = g.Kchunks * 8;                       // contraction length (the layer's output units)

  // dy loader: chunk column cc (0..3) is fixed per thread, rows stride 64
  constexpr int A_LOADS = (BM * 4 + 255) / 256;
  const int cc = tid & 3, lrow = tid >> 2;
  const bf16_t* arow[A_LOADS];
#pragma unroll
  for (int i = 0; i < A_LOADS; i++) {
    const int row = lrow + 64 * i;
    const bool ok = row < Mg;
    const int q = ok ? row / g.M : 0;
    arow[i] = ok ? (const bf16_t*)member_base(ws, z0, q) + g.a_off + (int64_t)(row - q * g.M) * K + cc * 8 : nullptr;
  }
  uint4 ra[A_LOADS], rb[4];
  auto load_regs = [&](int ks) {
    const bool kin = (ks * 4 + cc) < g.Kchunks;
#pragma unroll
    for (int i = 0; i < A_LOADS; i++)
      ra[i] = ld16(arow[i] != nullptr && kin ? arow[i] + ks * GBK : zeros);
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int idx = tid + 256 * i;
      const int r = idx >> 5, ch = idx & 31;       // 32 chunks of 8 inputs per tile row
      const int k = ks * GBK + r, n = n0 + ch * 8;
      rb[i] = ld16(k < K && n < g.Ncols ? Bm + (int64_t)k * g.ldb + n : zeros);
    }
  };
  auto store_lds = [&](int buf) {
    bf16_t* A = lds + buf * (A_ELEMS + B_ELEMS);
    bf16_t* B = A + A_ELEMS;
#pragma unroll
    for (int i = 0; i < A_LOADS; i++)
      if (lrow + 64 * i < BM) *reinterpret_cast<uint4*>(A + (lrow + 64 * i) * GLDA + cc * 8) = ra[i];
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int idx = tid + 256 * i;
      *reinterpret_cast<uint4*>(B + (idx >> 5) * GBN + (idx & 31) * 8) = rb[i];
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
        a[i] = *reinterpret_cast<const bf16x8*>(A + (32 * i + (lane & 31)) * GLDA + 16 * kk + 8 * (lane >> 5));
      // transpose load: lane j16 of a 16-lane group supplies the row k0 + j16/4, columns 4*(j16%4)..+3 and receives
      // the four k values of column (lane%16) of the group's 16 columns
      const int j16 = lane & 15, half = (lane >> 4) & 1, kb = 16 * kk + 8 * (lane >> 5);
#pragma unroll
      for (int j = 0; j < TN; j++) {
        const bf16_t* p = B + (kb + (j16 >> 2)) * GBN + wn0 + 32 * j + 16 * half + 4 * (j16 & 3);
        union { bf16x8 v; shortx4 h[2]; } u;
        u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((shortx4 __attribute__((address_space(3)))*)(p));
        u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((shortx4 __attribute__((address_space(3)))*)(p + 4 * GBN));
        b[j] = u.v;
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
  if (g.splits > 1) {
    float* part = reinterpret_cast<float*>(lead + g.scratch_off) + (int64_t)sp * Mg * g.Ncols;
#pragma unroll
    for (int j = 0; j < TN; j++) {
      const int n = n0 + wn0 + 32 * j + (lane & 31);
      if (n >= g.Ncols) continue;
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const int row = 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          if (row < Mg) part[(int64_t)row * g.Ncols + n] = acc[i][j][r];
        }
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int row = 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      if (row >= Mg) continue;
      const int q = row / g.M;
      char* base = member_base(ws, z0, q);
      bf16_t* out = (bf16_t*)base + ep.out_off;
      const bf16_t* mask = (const bf16_t*)base + ep.mask_off;
#pragma unroll
      for (int j = 0; j < TN; j++) {
        const int n = n0 + wn0 + 32 * j + (lane & 31);
        if (n >= g.Ncols) continue;
        float v = acc[i][j][r];
        const int64_t o = (int64_t)(row - q * g.M) * g.Ncols + n;
        if (ep.use_mask && !(bf2f(mask[o]) > 0.f)) v = 0.f;
        out[o] = f2bf(v);
      }
    }
}

// Sum of the split partials of every group in split order, then bias / ReLU / mask / conversion; blockIdx.z = group.
__global__ __launch_bounds__(256) void fc_group_finish_kernel(PtrTab ws, CPtrTab wts, GroupTab gt, IGemm g, Epilogue ep) {
  const int z0 = gt.first[blockIdx.z], nm = gt.members[blockIdx.z];
  const int Mg = nm * g.M;
  char* const lead = (char*)ws.p[z0];                // the first member: zeros and split partials live in its workspace
  const float4* part = reinterpret_cast<const float4*>(lead + g.scratch_off);
  const bf16_t* bias = (const bf16_t*)wts.p[z0] + ep.bias_off;
  // four consecutive columns per thread (the column count is a multiple of 8)
  const uint32_t total4 = (uint32_t)(((int64_t)Mg * g.Ncols) >> 2);
  const uint32_t per_member4 = (uint32_t)(((int64_t)g.M * g.Ncols) >> 2);
  for (uint32_t o4 = blockIdx.x * 256 + threadIdx.x; o4 < total4; o4 += gridDim.x * 256) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
    for (int sp = 0; sp < g.splits; sp++) {   // loads of several splits in flight; the additions keep split order
      const float4 p = part[(size_t)sp * total4 + o4];
      v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
    }
    const uint32_t q = o4 / per_member4;
    const uint32_t l4 = o4 - q * per_member4;           // four-column piece inside the member's own tensor
    const int64_t o = (int64_t)l4 * 4;
    char* base = member_base(ws, z0, (int)q);
    bf16_t* out = (bf16_t*)base + ep.out_off;
    const bf16_t* mask = (const bf16_t*)base + ep.mask_off;
    float f[4] = {v.x, v.y, v.z, v.w};
    if (ep.has_bias) {
      const int n = (int)((l4 * 4u) % (uint32_t)g.Ncols);
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
      reinterpret_cast<float4*>(out)[l4] = make_float4(f[0], f[1], f[2], f[3]);
    } else {
      uint2 w;
      w.x = (uint32_t)f2bf(f[0]) | ((uint32_t)f2bf(f[1]) << 16);
      w.y = (uint32_t)f2bf(f[2]) | ((uint32_t)f2bf(f[3]) << 16);
      *reinterpret_cast<uint2*>(out + o) = w;
    }
  }
}

// ------------------------------------------------------------------ host side
bool fc_group_layer_ok(int mu, int in, int out) {
  return mu >= 1 && mu <= 32 && in % FCK == 0 && out % 8 == 0 && (int64_t)out * in * 2 < ((int64_t)1 << 31) &&
         (int64_t)mu * std::max(in, out) * 4 < ((int64_t)1 << 31);
}

static bool group_table_ok(const GroupTab& gt, int groups, int mu, int* max_rows) {
  if (groups < 1 || groups > kMaxLearners) return false;
  int mr = 0;
  for (int k = 0; k < groups; k++) {
    const int nm = gt.members[k];
    if (nm < 1 || nm * mu > kMaxGroupRows || gt.first[k] + nm > kMaxLearners) return false;
    mr = std::max(mr, nm * mu);
  }
  *max_rows = mr;
  return true;
}

// Split of the contraction (`steps` steps of 16 KiB of weights) for `blocks` equal pieces of work.  Both kernels keep four
// workgroups on a compute unit (1 024 places on the chip) and their workgroups all take the same time, so a launch runs in
// rounds: the split with the least (rounds x (steps per workgroup + fixed cost of a workgroup, about three steps)) wins,
// with at least four steps per workgroup and the partials within the scratch area.
static int group_splits(int64_t blocks, int steps, size_t bytes_per_split, size_t scratch_bytes) {
  const int64_t places = 1024;
  int64_t max_sp = std::max(1, steps / 4);
  if (bytes_per_split > 0) max_sp = std::min<int64_t>(max_sp, (int64_t)(scratch_bytes / bytes_per_split));
  max_sp = std::max<int64_t>(1, std::min<int64_t>(max_sp, 64));
  int best = 1;
  double best_cost = 0.0;
  for (int64_t sp = 1; sp <= max_sp; sp++) {
    const int64_t rounds = (blocks * sp + places - 1) / places;
    const double cost = (double)rounds * ((double)((steps + sp - 1) / sp) + 3.0 + (sp > 1 ? 1.0 : 0.0));
    if (sp == 1 || cost < best_cost * 0.97) { best = (int)sp; best_cost = cost; }
  }
  return best;
}

static void launch_group_finish(const PtrTab& ws, const CPtrTab& wts, const GroupTab& gt, int groups, int max_rows, const IGemm& g,
                                const Epilogue& ep, hipStream_t s) {
  const int64_t total = ((int64_t)max_rows * g.Ncols) >> 2;
  const unsigned blocks = (unsigned)((total + 255) / 256 < 2048 ? (total + 255) / 256 : 2048);
  hipLaunchKernelGGL(fc_group_finish_kernel, dim3(blocks, 1, (unsigned)groups), dim3(256), 0, s, ws, wts, gt, g, ep);
}

hipError_t launch_fc_group_fwd(const PtrTab& ws, const CPtrTab& wts, const GroupTab& gt, int groups, const IGemm& g_in, const Epilogue& ep,
                               size_t scratch_off, size_t scratch_bytes, hipStream_t s) {
  IGemm g = g_in;
  int max_rows = 0;
  if (!fc_group_layer_ok(g.M, g.C, g.Ncols) || g.ldb != g.C || ep.use_mask || !group_table_ok(gt, groups, g.M, &max_rows))
    return hipErrorInvalidValue;
  const int64_t blocks = (int64_t)((g.Ncols + 31) / 32) * groups;
  g.splits = group_splits(blocks, g.C / FCK, (size_t)max_rows * g.Ncols * 4, scratch_bytes);
  g.scratch_off = scratch_off;
  const dim3 grid((unsigned)((g.Ncols + 31) / 32), 1, (unsigned)(groups * g.splits));
  if (max_rows <= 32) hipLaunchKernelGGL(fc_group_fwd_kernel<1>, grid, dim3(256), 0, s, ws, wts, gt, g, ep);
  else if (max_rows <= 64) hipLaunchKernelGGL(fc_group_fwd_kernel<2>, grid, dim3(256), 0, s, ws, wts, gt, g, ep);
  else hipLaunchKernelGGL(fc_group_fwd_kernel<4>, grid, dim3(256), 0, s, ws, wts, gt, g, ep);
  if (g.splits > 1) launch_group_finish(ws, wts, gt, groups, max_rows, g, ep, s);
  return hipGetLastError();
}

hipError_t launch_fc_group_dgrad(const PtrTab& ws, const CPtrTab& wts, const GroupTab& gt, int groups, const IGemm& g_in, const Epilogue& ep,
                                 size_t scratch_off, size_t scratch_bytes, hipStream_t s) {
  IGemm g = g_in;
  int max_rows = 0;
  // here g.C is the contraction length (the layer's output units) and g.Ncols the layer's input units
  if (g.M < 1 || g.M > 32 || g.C % 8 || g.Ncols % 8 || g.ldb != g.Ncols || ep.has_bias || ep.out_f32 ||
      (int64_t)g.C * g.ldb * 2 >= ((int64_t)1 << 31) || !group_table_ok(gt, groups, g.M, &max_rows))
    return hipErrorInvalidValue;
  const int64_t tiles = (g.Ncols + GBN - 1) / GBN;
  g.scratch_off = scratch_off;
  g.splits = group_splits(tiles * groups, (g.Kchunks + 3) / 4, (size_t)max_rows * g.Ncols * 4, scratch_bytes);
  const dim3 grid((unsigned)tiles, 1, (unsigned)(groups * g.splits));
  if (max_rows <= 32) hipLaunchKernelGGL(fc_group_dgrad_kernel<32>, grid, dim3(256), 0, s, ws, wts, gt, g, ep);
  else if (max_rows <= 64) hipLaunchKernelGGL(fc_group_dgrad_kernel<64>, grid, dim3(256), 0, s, ws, wts, gt, g, ep);
  else hipLaunchKernelGGL(fc_group_dgrad_kernel<128>, grid, dim3(256), 0, s, ws, wts, gt, g, ep);
  if (g.splits > 1) launch_group_finish(ws, wts, gt, groups, max_rows, g, ep, s);
  return hipGetLastError();
}

}  // namespace sasgd
