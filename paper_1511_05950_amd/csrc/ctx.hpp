// Internal state of a sasgd context (host side).  Not part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/sasgd.h"

namespace sasgd {

constexpr int kMaxLearners = 64;   // also the largest c one applyUpdate launch reduces

typedef uint16_t bf16_t;           // raw bf16 bits in HBM

// ---------------------------------------------------------------- fused server update (update.hip)
struct UpdateLaunch {
  const float* theta_in;   // theta_i  [P]
  float* theta_out;        // theta_{i+1} [P] (may alias theta_in)
  float* v;                // momentum [P], updated in place
  bf16_t* shadow_out;      // optional bf16 copy of theta_{i+1} [P], or nullptr
  int64_t P;
  int32_t c;
  const float* grads[kMaxLearners];
  float coef[kMaxLearners];
  float momentum;
  float decay;             // (sum_l coef_l) * weight_decay
  int reverse;             // walk the vector from its end (same result; see apply_update_kernel)
  float* sum_buf;          // kSumStretch floats for the two-pass form of long windows, or nullptr: always one pass
};
// Several consecutive updates in ONE pass over the vector ("fused steps"): theta and v are read once, the steps are applied
// one after the other in registers -- the arithmetic of the single launches in the same order, bit-identical -- and
// written once; every step still writes its own weight version (ring slot / bf16 copy).  Step t owns the gradient-table
// entries [first[t], first[t + 1]).
constexpr int kMaxFusedSteps = 8;
struct StepTable {
  int32_t steps;
  int32_t first[kMaxFusedSteps + 1];
  float decay[kMaxFusedSteps];          // (sum of the step's coefficients) * weight_decay
  float* theta_out[kMaxFusedSteps];     // fp32 weights after step t (ring slot), or nullptr: not kept (fp32 master in place)
  bf16_t* shadow_out[kMaxFusedSteps];   // bf16 copy of the weights after step t, or nullptr
};
// Windows of at least kTwoPassMinC gradients are applied in two passes per stretch of kSumStretch parameters.
constexpr int kTwoPassMinC = 25;
constexpr int64_t kSumStretch = (int64_t)1 << 21;   // 8 MiB of sums: 512 workgroups of 4 096 parameters
hipError_t launch_apply_update(const UpdateLaunch& u, hipStream_t stream);
// Fused steps over a flat stretch: u supplies theta_in, v, P, momentum, the gradient table (u.c entries in all, at most
// kMaxLearners) -- its theta_out / shadow_out / decay are ignored in favour of st's per-step ones; the weights after the
// last step are also written to `final_theta` (may be theta_in).
hipError_t launch_apply_updates_fused(const UpdateLaunch& u, const StepTable& st, float* final_theta, hipStream_t stream);
// Device address, on the current device, of the library's statically allocated buffer of kSumStretch floats (looked up
// once per device; no allocation).  Every caller on a device shares it: launches that use it must not overlap.
hipError_t static_sum_buffer(float** out);
// Update of the fully connected layers (each: weights [out][in] followed by the bias [out]) whose gradients are kept as
// factors, all layers in ONE launch.  theta_in / theta_out / v / shadow_out / grads address element 0 of the flat vector.
constexpr int kMaxFactoredLayers = 16;   // further fully connected layers write their gradient out
struct FcUpdateLaunch {
  const float* theta_in;
  float* theta_out;
  float* v;
  bf16_t* shadow_out;      // optional
  int N, NP;               // N images per mini-batch, factor rows padded to NP
  int layers;
  int in[kMaxFactoredLayers], out[kMaxFactoredLayers];
  int64_t w_off[kMaxFactoredLayers];                     // first weight of the layer in the flat vector
  size_t fx_off[kMaxFactoredLayers], fdy_off[kMaxFactoredLayers];   // the layer's factors, bf16 elements from factors[l]
  int32_t c;
  const float* grads[kMaxLearners];     // written-out gradient of every pending gradient (bias part always used)
  const bf16_t* factors[kMaxLearners];  // base of the pending gradient's factors (x transposed [in][NP] at fx_off, dy
                                        // transposed [out][NP] at fdy_off), or nullptr: use the written-out weights gradient
  float coef[kMaxLearners];
  float momentum;
  float decay;
};
// st == nullptr: one step (u.shadow_out, u.decay).  Otherwise fused steps: st's first / decay / shadow_out are used (its
// theta_out is ignored: the weights are written once, to u.theta_out).
hipError_t launch_apply_update_fc(const FcUpdateLaunch& u, hipStream_t stream, const StepTable* st = nullptr);
hipError_t launch_fp32_to_bf16(const float* src, bf16_t* dst, int64_t n, hipStream_t stream);
hipError_t launch_bf16_to_fp32(const bf16_t* src, float* dst, int64_t n, hipStream_t stream);

// ---------------------------------------------------------------- network (net.cpp)
struct Net;   // layer plan + per-learner workspaces
struct LearnerBind {
  const float* images;     // [mu][C][H][W] fp32, caller-owned
  const int32_t* labels;   // [mu]
  const void* weights;     // bound weight version (fp32 or bf16 flat vector, plus packed copies)
  int64_t version;
  float* grad;             // [P] fp32 output
};
int net_create(const sasgd_config& cfg, Net** out, int64_t* out_P, size_t* out_pack_elems, std::string& err);
void net_destroy(Net* net);
// Device memory the net needs per learner, in bytes (activations, gradient activations, argmax).
size_t net_workspace_bytes(const Net* net);
// Staging area in which learners that share a weight version stack their mini-batches for the fully connected layers
// (bytes; 0 if the network has no such layer).  One per context.
size_t net_group_workspace_bytes(const Net* net);
hipError_t net_set_group_workspace(Net* net, void* ws, hipStream_t stream);
// Registers a learner's workspace and initialises it (zeros, plus the constant blocks the kernels read).
hipError_t net_set_workspace(Net* net, int learner, void* ws, hipStream_t stream);
// Per weight version: derive the kernel-friendly copies (bf16 repacked conv filters) from the flat vector.
hipError_t net_prepare_version(Net* net, const void* flat, void* packed, hipStream_t stream);
// The same for several versions in one launch per kernel.
hipError_t net_prepare_versions(Net* net, const void* const* flat, void* const* packed, int versions, hipStream_t stream);
// out_rank_dev == nullptr: forward, loss, backward (gradients into binds[k].grad).
// out_rank_dev != nullptr: evaluation pass, forward and loss only, plus the rank of each image's true class.
hipError_t net_calc_gradient(Net* net, const int* learners, const LearnerBind* binds, int count,
                             float* out_loss_dev, int32_t* out_rank_dev, hipStream_t stream);
// Fully connected layers whose weight gradient calcGradient leaves as factors in the learner's workspace
// (bf16 element offsets from the workspace base): weights at w_off [out][in], bias right behind them.
struct FactoredLayer {
  int64_t w_off;
  int in, out, N, NP;
  size_t fx_off, fdy_off;
};
int net_factored_layers(const Net* net, FactoredLayer* out, int max);
// dW [out][in] fp32 from the factors (layers.hip); used by the getters that hand out a written-out gradient
hipError_t launch_fc_expand_factors(const void* fx, const void* fdy, float* dw, int N, int in, int out, int NP, hipStream_t s);
void net_set_pixel_mean(Net* net, const float* mean_dev);
void net_input_shape(const Net* net, int* C, int* H, int* W);

// ---------------------------------------------------------------- context
enum GradState { GRAD_NONE = 0, GRAD_COMPUTED = 1, GRAD_PENDING = 2 };

struct Learner {
  const float* images = nullptr;
  const int32_t* labels = nullptr;
  bool has_weights = false;
  int64_t pulled_version = -1;
  bool evaluated = false;      // the pulled version has served an evaluation pass: it may leave the ring (see sasgd_evaluate)
  int64_t grad_timestamp = -1;
  GradState grad_state = GRAD_NONE;
  float* grad = nullptr;       // [P] fp32 (nullptr for NET_NONE)
  void* workspace = nullptr;
  bool fc_expanded = false;    // the factored parts of the current gradient have been written out into `grad`
};

struct Pending;
// An update whose window is closed and whose host bookkeeping is done, but whose device work has not been enqueued yet.
struct DeferredUpdate;

struct Pending {
  const void* factors_ws;   // workspace holding the fully connected factors of this gradient, or nullptr (written out)
  const float* grad;
  int64_t timestamp;   // j
  int32_t staleness;   // tau = i - j at push time
  int32_t learner;     // -1 for external gradients
};

struct DeferredUpdate {
  int64_t i = 0;                 // timestamp before the update: it makes version i + 1
  std::vector<Pending> grads;    // the window, in arrival order
  std::vector<float> coef;
  float decay = 0.f;             // (sum of coefficients) * weight_decay
};

}  // namespace sasgd

struct sasgd_ctx {
  sasgd_config cfg;
  int32_t c = 1;
  int64_t P = 0;
  int64_t timestamp = 0;             // i
  hipStream_t stream = nullptr;
  int device = 0;
  // weight versions
  float* ring_f32 = nullptr;         // FP32 compute: [R][P]; BF16 compute: [1][P] master
  sasgd::bf16_t* ring_b16 = nullptr; // BF16 compute: [R][P + pack] shadow copies
  size_t slot_elems_b16 = 0;         // elements per bf16 slot (P rounded up + packed filters)
  size_t slot_elems_f32 = 0;         // FP32 compute: elements per ring slot (P rounded up to 64)
  float* v = nullptr;                // momentum [P]
  float* sum_buf = nullptr;          // [kSumStretch] partial result of long windows (c >= kTwoPassMinC), else nullptr
  std::vector<sasgd::Learner> learners;
  std::vector<sasgd::Pending> pending;
  std::vector<sasgd::DeferredUpdate> deferred;   // updates applied on the host whose kernels are not launched yet
  bool window_closed = false;
  int32_t window_count = 0;
  float window_coef[sasgd::kMaxLearners];
  sasgd::Net* net = nullptr;
  std::vector<void*> allocations;
  std::string error;
  // profiling
  bool profiling = false;
  struct EvPair { hipEvent_t a, b; int which; int count; };
  std::vector<EvPair> events;
  double phase_ms[2] = {0, 0};
  int64_t phase_calls[2] = {0, 0};
  int64_t update_passes = 0;         // launches groups of the update phase (one pass may apply several updates)
};
