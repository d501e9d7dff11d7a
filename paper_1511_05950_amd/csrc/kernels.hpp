// Launch wrappers of the calcGradient kernels (Section 2.1 learner step; layer types of Section 4.1).
// Every launch covers `count` learners at once: blockIdx.z (or .y) selects the learner, and per-learner
// base addresses come from small by-value tables.  Activations are NHWC ([image][h][w][channel]) of type
// T = float (fp32 compute) or bf16 bits (bf16 compute); parameters and parameter gradients use the flat
// order of the C ABI.
#pragma once
#include "ctx.hpp"

namespace sasgd {

struct PtrTab {
  void* p[kMaxLearners];
};
struct CPtrTab {
  const void* p[kMaxLearners];
};

struct ConvShape {
  int N;                 // images per learner (mu)
  int C, H, W;           // input
  int K, OH, OW;         // output channels and size
  int ks, stride, pad;   // square window
};

struct PoolShape {
  int N, C, H, W, OH, OW, ks, stride;
};

// Re-layout of the caller's images.  s2d == 1: NCHW fp32 -> NHWC with channels zero-padded to Cp.
// s2d == s > 1 (space to depth): out[n][Y][X][(dy*s+dx)*C + c] = in[n][c][s*Y+dy][s*X+dx], zero outside the
// image and in the padding channels; a stride-s convolution on the image is a stride-1 one on this tensor.
struct InPack {
  int C, H, W;      // source
  int Cp, Hp, Wp;   // destination
  int s2d;
};

// A convolution as the MFMA kernels see it (stride 1): C = effective (padded or space-to-depth) input
// channels, ks = effective window, K = output channels; Creal / ksr describe the flat filter [K][Creal][ksr][ksr].
struct VConv {
  int C, ks, K, s2d, Creal, ksr;
};

// Source index, in the flat [K][Creal][ksr][ksr] filter, of packed element (n, tap, cp) of a virtual
// stride-1 layer, or -1 for padding.  s2d > 1: the layer is a strided one seen through a
// space-to-depth input: channel cp = (dy*s2d + dx)*Creal + c, tap = (KY, KX), kh = s2d*KY + dy.
__host__ __device__ inline int64_t filter_src(const VConv& v, int n, int tap, int cp) {
  int kh, kw, c;
  if (v.s2d == 1) {
    if (cp >= v.Creal) return -1;
    c = cp; kh = tap / v.ks; kw = tap % v.ks;
  } else {
    int g = cp / v.Creal;
    c = cp % v.Creal;
    if (g >= v.s2d * v.s2d) return -1;
    kh = v.s2d * (tap / v.ks) + g / v.s2d;
    kw = v.s2d * (tap % v.ks) + g % v.s2d;
    if (kh >= v.ksr || kw >= v.ksr) return -1;
  }
  return (((int64_t)n * v.Creal + c) * v.ksr + kh) * v.ksr + kw;
}

// One implicit GEMM: D[m][n] = sum_k im2col(t)[m][k] * B(n, k).  t = NHWC tensor [*][H][W][C] at a_off (elements
// of bf16 from the workspace base), output positions OH x OW, window ks, zero padding pad, stride 1.
struct IGemm {
  size_t a_off;
  int64_t b_off;            // elements of bf16 from the learner's weight-version base
  int M, Ncols;             // M = images * OH * OW
  int H, W, C, OH, OW, ks, pad;
  int Kchunks, CPT;         // ks*ks*C/8 and C/8
  int ldb;                  // row length of B in elements
  // Split of the contraction over `splits` workgroups per tile (fills the chip when there are few tiles):
  // each writes an fp32 partial tile to scratch (byte offset from the workspace base), a second kernel adds
  // them in split order and applies the epilogue, so the result does not depend on scheduling.
  int splits;
  size_t scratch_off;
  // multipliers for division by CPT, ks, OW, OH without a divide (set by igemm_set_magics)
  uint32_t mg_cpt, mg_ks, mg_ow, mg_oh;
  // 256 bytes of zeros inside the workspace (elements of bf16 from its base): the address out-of-range chunk
  // loads are redirected to, so that no load is conditional and no loaded value needs patching
  size_t zero_off;
  // byte sizes of the gathered tensor (one learner) and of the fragment-packed B, for hardware-bounds-checked
  // buffer loads (both below 2 GiB)
  uint32_t a_bytes, b_bytes;
};

// floor(n / d) == (n * magic(d)) >> 32 for all 0 <= n with n * d < 2^32 (d >= 2); d == 1 is handled apart.
inline uint32_t magic_u32(int d) { return d <= 1 ? 0u : (uint32_t)((((uint64_t)1) << 32) / (uint32_t)d + 1u); }
inline void igemm_set_magics(IGemm& g, int elem_bytes) {
  if (g.OH > 0 && g.OW > 0) g.a_bytes = (uint32_t)((int64_t)(g.M / (g.OH * g.OW)) * g.H * g.W * g.C * elem_bytes);
  g.b_bytes = (uint32_t)((int64_t)((g.Ncols + 31) & ~31) * g.ldb * 2);
  g.mg_cpt = magic_u32(g.CPT);
  g.mg_ks = magic_u32(g.ks);
  g.mg_ow = magic_u32(g.OW);
  g.mg_oh = magic_u32(g.OH);
}

struct Epilogue {
  size_t out_off, mask_off; // elements of bf16 from the workspace base
  int64_t bias_off;         // elements of bf16 from the weight-version base
  int has_bias, relu, use_mask, out_f32;
};

// is_bf16 selects T.  All offsets are in elements of T from the learner's workspace base, except where noted.
hipError_t launch_pack_input(bool is_bf16, const CPtrTab& images, const PtrTab& ws, size_t out_off, int count, int N,
                             const InPack& ip, const float* mean, hipStream_t s);

// ---- bf16 MFMA path (conv_mfma.hip)
// One launch repacks the filters of every MFMA convolution of a weight version.
struct PackJob {
  VConv v;
  int64_t w_off, fwd_off, bwd_off;   // flat source, fragment destinations (elements)
  int64_t start;                     // first global element index of this layer in the launch
  int Kp, Kpt;                       // padded row lengths; Kpt == 0: no transposed copy
};
constexpr int kMaxPackJobs = 24;
struct PackTable {
  PackJob job[kMaxPackJobs];
  int count;
  int64_t total;
};
// Several weight versions in one launch (blockIdx.y): flat bf16 vector and packed-filter region of each.
constexpr int kMaxPackVersions = 8;
struct PackVersions {
  const void* flat[kMaxPackVersions];
  void* packed[kMaxPackVersions];
};
hipError_t launch_pack_filters(const PackVersions& pv, int versions, const PackTable& t, hipStream_t s);
// ---- fp32 MFMA path (conv_mfma_f32.hip); dgrad: g gathers over dy, the filter is read transposed and flipped
hipError_t launch_igemm_f32(const PtrTab& ws, const CPtrTab& wts, const IGemm& g, const VConv& v, const Epilogue& ep, int64_t w_off,
                            bool dgrad, int count, hipStream_t s);
hipError_t launch_igemm_wgrad_f32(const PtrTab& ws, const PtrTab& grads, const IGemm& g, const VConv& v, size_t dy_off, int64_t w_off,
                                  int64_t b_off, int count, hipStream_t s);
hipError_t launch_igemm_frag(const PtrTab& ws, const CPtrTab& wts, const IGemm& g, const Epilogue& ep, int count, hipStream_t s);
hipError_t launch_igemm(const PtrTab& ws, const CPtrTab& wts, const IGemm& g, const Epilogue& ep, bool b_transposed, int count,
                        hipStream_t s);
// dW and db of one layer (the bias gradient rides along as one extra im2col column of ones).
hipError_t launch_igemm_wgrad(const PtrTab& ws, const PtrTab& grads, const IGemm& g, const VConv& v, size_t dy_off, int64_t w_off,
                              int64_t b_off, int count, hipStream_t s);
// Split choice: enough workgroups for the chip, bounded by the contraction length and the scratch size.
int choose_splits(int64_t tiles, int count, int steps, size_t bytes_per_split, size_t scratch_bytes, int64_t target = 600);

// y = conv(x, w) + b, optional ReLU.  w_off / b_off: element offsets into the learner's flat weight vector.
// out_f32: y is stored as fp32 whatever T is (class scores).
hipError_t launch_conv_fwd_simple(bool is_bf16, const PtrTab& ws, const CPtrTab& wts, size_t x_off, size_t y_off, int64_t w_off,
                                  int64_t b_off, const ConvShape& sh, bool relu, bool out_f32, int count, hipStream_t s);
// dx = conv^T(dy, w), optionally zeroed where mask (the forward tensor at mask_off) <= 0.
hipError_t launch_conv_dgrad_simple(bool is_bf16, const PtrTab& ws, const CPtrTab& wts, size_t dy_off, size_t dx_off, int64_t w_off,
                                    const ConvShape& sh, bool use_mask, size_t mask_off, int count, hipStream_t s);
// dW, db into the learner's fp32 gradient vector at w_off / b_off.
hipError_t launch_conv_wgrad_simple(bool is_bf16, const PtrTab& ws, const PtrTab& grads, size_t x_off, size_t dy_off, int64_t w_off,
                                    int64_t b_off, const ConvShape& sh, int count, hipStream_t s);

hipError_t launch_pool_fwd(bool is_bf16, bool is_max, const PtrTab& ws, size_t x_off, size_t y_off, size_t arg_byte_off,
                           const PoolShape& sh, bool relu, int count, hipStream_t s);
hipError_t launch_pool_bwd(bool is_bf16, bool is_max, const PtrTab& ws, size_t dy_off, size_t dx_off, size_t arg_byte_off,
                           const PoolShape& sh, bool use_mask, size_t mask_off, int count, hipStream_t s);

// NHWC [N][H][W][C] <-> [N][C*H*W] (C,H,W order), the flattening the fully connected weights expect.
hipError_t launch_flatten_fwd(bool is_bf16, const PtrTab& ws, size_t x_off, size_t y_off, int N, int C, int H, int W, int count,
                              hipStream_t s);
hipError_t launch_flatten_bwd(bool is_bf16, const PtrTab& ws, size_t dy_off, size_t dx_off, int N, int C, int H, int W, bool use_mask,
                              size_t mask_off, int count, hipStream_t s);

// loss[l] = mean_n -log softmax(z_n)[label_n];  dz = (softmax(z) - onehot) / N.  loss_out may be null.
// z_f32: the scores at z_off (an offset in elements of T) are fp32; dz is always of type T.
// loss_byte_off: N floats of per-image losses in the workspace (bytes from its base).
hipError_t launch_softmax_ce(bool is_bf16, bool z_f32, const PtrTab& ws, const CPtrTab& labels, size_t z_off, size_t dz_off,
                             size_t loss_byte_off, int N, int K, float* loss_out, int count, hipStream_t s);
hipError_t launch_label_rank(bool is_bf16, bool z_f32, const PtrTab& ws, const CPtrTab& labels, size_t z_off, int N, int K,
                             int32_t* rank_out, int count, hipStream_t s);
// ---- fully connected layers grouped by weight version (fc_group.hip)
// Group k = members first[k] .. first[k] + members[k] - 1 of the pointer tables handed to the launch (learners that read
// one weight version, listed next to each other); at most kMaxGroupRows image rows per group.
constexpr int kMaxGroupRows = 128;
struct GroupTab {
  uint8_t first[kMaxLearners];
  uint8_t members[kMaxLearners];
};
// A layer of `in` inputs and `out` units on mini-batches of mu images that the grouped kernels take.
bool fc_group_layer_ok(int mu, int in, int out);
// y = x W^T + b (optional ReLU, optional fp32 output) for every group; g = the layer's forward GEMM of ONE learner
// (M = mu).  scratch_off / scratch_bytes: the split-partial area of a workspace (the first member's is used).
hipError_t launch_fc_group_fwd(const PtrTab& ws, const CPtrTab& wts, const GroupTab& gt, int groups, const IGemm& g, const Epilogue& ep,
                               size_t scratch_off, size_t scratch_bytes, hipStream_t s);
// dx = dy W (optionally zeroed where the forward tensor at ep.mask_off is <= 0); g = the layer's input-gradient GEMM of
// one learner with a_off = offset of dy.
hipError_t launch_fc_group_dgrad(const PtrTab& ws, const CPtrTab& wts, const GroupTab& gt, int groups, const IGemm& g, const Epilogue& ep,
                                 size_t scratch_off, size_t scratch_bytes, hipStream_t s);

// Copies [bytes_per_member] between every member's workspace (at member_off_bytes) and consecutive pieces of `stage`.
hipError_t launch_stack_rows(const PtrTab& members, int count, size_t member_off_bytes, void* stage, int64_t bytes_per_member,
                             bool to_stage, hipStream_t s);
hipError_t launch_fc_save_factors(const PtrTab& ws, const PtrTab& grads, size_t x_off, size_t dy_off, size_t fx_off, size_t fdy_off,
                                  int64_t b_off, int N, int in, int out, int NP, int count, hipStream_t s);
hipError_t launch_fc_expand_factors(const void* fx, const void* fdy, float* dw, int N, int in, int out, int NP, hipStream_t s);

}  // namespace sasgd
