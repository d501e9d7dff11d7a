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

// is_bf16 selects T.  All offsets are in elements of T from the learner's workspace base, except where noted.
hipError_t launch_pack_input(bool is_bf16, const CPtrTab& images, const PtrTab& ws, size_t out_off, int count, int N, int C,
                             int H, int W, hipStream_t s);

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
hipError_t launch_softmax_ce(bool is_bf16, bool z_f32, const PtrTab& ws, const CPtrTab& labels, size_t z_off, size_t dz_off, int N,
                             int K, float* loss_out, int count, hipStream_t s);

}  // namespace sasgd
