// C ABI of the staleness-aware n-softsync ASGD hot path: host-side protocol state (timestamps,
// staleness, the pending-gradient window, the ring of weight versions) and the launches of the
// device work.  Section references are to the paper (Sections 2.1, 2.2, 2.4, 3).
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <cmath>
#include <new>

#include "ctx.hpp"

using namespace sasgd;

namespace {

int fail(sasgd_ctx* ctx, int code, const std::string& msg) {
  if (ctx) ctx->error = msg;
  return code;
}

int fail_hip(sasgd_ctx* ctx, hipError_t e, const char* what) {
  return fail(ctx, SASGD_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

void* ctx_alloc(sasgd_ctx* ctx, size_t bytes) {
  void* p = nullptr;
  if (bytes == 0) bytes = 256;
  if (ctx->cfg.alloc) {
    p = ctx->cfg.alloc(bytes, ctx->cfg.alloc_user);
  } else if (hipMalloc(&p, bytes) != hipSuccess) {
    (void)hipGetLastError();
    p = nullptr;
  }
  if (p) ctx->allocations.push_back(p);
  return p;
}

void ctx_free_all(sasgd_ctx* ctx) {
  for (void* p : ctx->allocations) {
    if (ctx->cfg.release) ctx->cfg.release(p, ctx->cfg.alloc_user);
    else if (!ctx->cfg.alloc) (void)hipFree(p);
  }
  ctx->allocations.clear();
}

bool is_device_pointer(const void* p) {
  hipPointerAttribute_t attr;
  hipError_t e = hipPointerGetAttributes(&attr, p);
  if (e != hipSuccess) {
    (void)hipGetLastError();   // plain host memory is reported as an error: clear it
    return false;
  }
  return attr.type == hipMemoryTypeDevice;
}

inline int slot_of(const sasgd_ctx* ctx, int64_t version) { return (int)(version % ctx->cfg.ring_depth); }

inline bool version_in_ring(const sasgd_ctx* ctx, int64_t version) {
  return version >= 0 && version <= ctx->timestamp && ctx->timestamp - version < ctx->cfg.ring_depth;
}

// Device address of the weights a learner reads for `version`.
const void* version_ptr(const sasgd_ctx* ctx, int64_t version) {
  if (ctx->cfg.compute == SASGD_BF16) return ctx->ring_b16 + (size_t)slot_of(ctx, version) * ctx->slot_elems_b16;
  return ctx->ring_f32 + (size_t)slot_of(ctx, version) * ctx->slot_elems_f32;
}

void prof_begin(sasgd_ctx* ctx, int which, int count = 1) {
  if (!ctx->profiling) return;
  sasgd_ctx::EvPair ev;
  ev.which = which;
  ev.count = count;
  if (hipEventCreate(&ev.a) != hipSuccess || hipEventCreate(&ev.b) != hipSuccess) return;
  (void)hipEventRecord(ev.a, ctx->stream);
  ctx->events.push_back(ev);
}
void prof_end(sasgd_ctx* ctx) {
  if (!ctx->profiling || ctx->events.empty()) return;
  (void)hipEventRecord(ctx->events.back().b, ctx->stream);
}
void prof_collect(sasgd_ctx* ctx) {
  for (auto& ev : ctx->events) {
    float ms = 0.f;
    if (hipEventSynchronize(ev.b) == hipSuccess && hipEventElapsedTime(&ms, ev.a, ev.b) == hipSuccess) {
      ctx->phase_ms[ev.which] += ms;
      ctx->phase_calls[ev.which] += ev.count;
      if (ev.which == 1) ctx->update_passes += 1;
    }
    (void)hipEventDestroy(ev.a);
    (void)hipEventDestroy(ev.b);
  }
  ctx->events.clear();
}

// coef_l = alpha(tau_l) / c with alpha(tau) = alpha0 / tau for tau > 0 (Section 2.4) and alpha0 at tau = 0; the two
// other rate modes replace alpha(tau_l) by alpha0 / mean(tau) or by alpha0.
void window_coefficients(int lr_mode, float a0, int c, const int32_t* tau, float* coef) {
  if (lr_mode == SASGD_LR_MEAN_STALENESS) {
    int64_t sum = 0;
    for (int l = 0; l < c; l++) sum += tau[l];
    const float mean = (float)((double)sum / (double)c);
    const float a = a0 / std::max(mean, 1.0f);
    for (int l = 0; l < c; l++) coef[l] = a / (float)c;
  } else {
    for (int l = 0; l < c; l++) {
      const float a = lr_mode == SASGD_LR_CONSTANT ? a0 : a0 / (float)std::max(tau[l], 1);
      coef[l] = a / (float)c;
    }
  }
}


// Device work of `n` consecutive updates ctx->deferred[0 .. n): one launch per piece of the vector (flat stretch or
// factored fully connected layer) that applies the n steps in order, then the per-version filter repack.
hipError_t enqueue_updates(sasgd_ctx* ctx, int n) {
  const std::vector<DeferredUpdate>& D = ctx->deferred;
  const bool bf = ctx->cfg.compute == SASGD_BF16;
  const size_t Ppad = ((size_t)ctx->P + 63) & ~(size_t)63;
  UpdateLaunch u;
  StepTable st;
  memset(&st, 0, sizeof(st));
  st.steps = n;
  const Pending* src[kMaxLearners];
  int total = 0;
  bf16_t* slots_b16[kMaxFusedSteps] = {nullptr};
  for (int t = 0; t < n; t++) {
    st.first[t] = total;
    for (size_t l = 0; l < D[(size_t)t].grads.size(); l++) {
      src[total] = &D[(size_t)t].grads[l];
      u.grads[total] = D[(size_t)t].grads[l].grad;
      u.coef[total] = D[(size_t)t].coef[l];
      total++;
    }
    st.decay[t] = D[(size_t)t].decay;
    const int64_t made = D[(size_t)t].i + 1;
    if (bf) {
      slots_b16[t] = ctx->ring_b16 + (size_t)slot_of(ctx, made) * ctx->slot_elems_b16;
      st.shadow_out[t] = slots_b16[t];
    } else {
      st.theta_out[t] = ctx->ring_f32 + (size_t)slot_of(ctx, made) * ctx->slot_elems_f32;
    }
  }
  st.first[n] = total;
  if (!bf)   // a ring slot that a later step of this pass takes again is not written twice
    for (int t = 0; t < n; t++)
      for (int t2 = t + 1; t2 < n; t2++)
        if (st.theta_out[t2] == st.theta_out[t]) st.theta_out[t] = nullptr;
  const int64_t i0 = D[0].i;
  u.P = ctx->P;
  u.c = total;
  u.momentum = ctx->cfg.momentum;
  u.decay = st.decay[0];
  u.v = ctx->v;
  u.sum_buf = ctx->sum_buf;
  u.reverse = (int)(i0 & 1);   // consecutive single updates walk in opposite directions (last-level cache reuse)
  u.theta_in = bf ? ctx->ring_f32 : ctx->ring_f32 + (size_t)slot_of(ctx, i0) * ctx->slot_elems_f32;
  u.theta_out = bf ? ctx->ring_f32 : ctx->ring_f32 + (size_t)slot_of(ctx, i0 + 1) * ctx->slot_elems_f32;
  u.shadow_out = st.shadow_out[0];
  float* final_theta = bf ? ctx->ring_f32 : nullptr;   // fp32 compute: the last step's ring slot holds the result
  // Layers whose gradients are kept as factors get their own launch; the stretches of the flat vector between them
  // go through the streaming kernel.
  FactoredLayer fl[kMaxFactoredLayers];
  const int nfl = ctx->net ? net_factored_layers(ctx->net, fl, kMaxFactoredLayers) : 0;
  prof_begin(ctx, 1, n);
  hipError_t e = hipSuccess;
  auto flat_range = [&](int64_t begin, int64_t end) {
    if (end <= begin) return hipSuccess;
    UpdateLaunch r = u;
    r.theta_in += begin;
    r.theta_out += begin;
    r.v += begin;
    if (r.shadow_out) r.shadow_out += begin;
    for (int l = 0; l < total; l++) r.grads[l] += begin;
    r.P = end - begin;
    if (n == 1) return launch_apply_update(r, ctx->stream);
    StepTable sr = st;
    for (int t = 0; t < n; t++) {
      if (sr.theta_out[t]) sr.theta_out[t] += begin;
      if (sr.shadow_out[t]) sr.shadow_out[t] += begin;
    }
    return launch_apply_updates_fused(r, sr, final_theta ? final_theta + begin : nullptr, ctx->stream);
  };
  // every stretch of the flat vector between the factored layers, then all factored layers in one launch
  int64_t cursor = 0;
  for (int k = 0; k < nfl && e == hipSuccess; k++) {
    e = flat_range(cursor, fl[k].w_off);
    cursor = fl[k].w_off + (int64_t)fl[k].out * fl[k].in + fl[k].out;
  }
  if (nfl > 0 && e == hipSuccess) {
    FcUpdateLaunch fu;
    fu.theta_in = u.theta_in;
    fu.theta_out = u.theta_out;
    fu.v = u.v;
    fu.shadow_out = u.shadow_out;
    fu.N = fl[0].N; fu.NP = fl[0].NP;
    fu.layers = nfl;
    for (int k = 0; k < nfl; k++) {
      fu.in[k] = fl[k].in; fu.out[k] = fl[k].out; fu.w_off[k] = fl[k].w_off;
      fu.fx_off[k] = fl[k].fx_off; fu.fdy_off[k] = fl[k].fdy_off;
    }
    fu.c = total;
    for (int l = 0; l < total; l++) {
      fu.grads[l] = src[l]->grad;
      fu.coef[l] = u.coef[l];
      fu.factors[l] = (const bf16_t*)src[l]->factors_ws;
    }
    fu.momentum = u.momentum;
    fu.decay = u.decay;
    e = launch_apply_update_fc(fu, ctx->stream, &st);
  }
  if (e == hipSuccess) e = flat_range(cursor, ctx->P);
  prof_end(ctx);
  if (e == hipSuccess && bf && ctx->net) {
    const void* flat[kMaxFusedSteps];
    void* packed[kMaxFusedSteps];
    for (int t = 0; t < n; t++) { flat[t] = slots_b16[t]; packed[t] = slots_b16[t] + Ppad; }
    e = net_prepare_versions(ctx->net, flat, packed, n, ctx->stream);
  }
  return e;
}

// Launches the kernels of every deferred update, in order, as few passes over the vector as the tables allow.
int flush_updates(sasgd_ctx* ctx) {
  while (!ctx->deferred.empty()) {
    int n = 0, total = 0;
    while (n < (int)ctx->deferred.size() && n < kMaxFusedSteps && total + (int)ctx->deferred[(size_t)n].grads.size() <= kMaxLearners) {
      total += (int)ctx->deferred[(size_t)n].grads.size();
      n++;
    }
    if ((int)ctx->deferred[0].grads.size() >= kTwoPassMinC) n = 1;   // long windows go alone (two-pass form)
    else
      for (int t = 1; t < n; t++)
        if ((int)ctx->deferred[(size_t)t].grads.size() >= kTwoPassMinC) { n = t; break; }
    if (n < 1) n = 1;
    hipError_t e = enqueue_updates(ctx, n);
    ctx->deferred.erase(ctx->deferred.begin(), ctx->deferred.begin() + n);
    if (e != hipSuccess) return fail_hip(ctx, e, "applyUpdate");
  }
  return SASGD_OK;
}

}  // namespace

extern "C" {

const char* sasgd_version(void) { return "sasgd-gfx950 0.1"; }

const char* sasgd_last_error(sasgd_ctx* ctx) { return ctx ? ctx->error.c_str() : "null context"; }

int sasgd_create(const sasgd_config* cfg, const float* init_weights, sasgd_ctx** out) {
  if (!cfg || !out || !init_weights) return SASGD_EINVAL;
  *out = nullptr;
  if (cfg->lambda < 1 || cfg->lambda > kMaxLearners) return SASGD_EINVAL;
  if (cfg->n < 1 || cfg->n > cfg->lambda) return SASGD_EINVAL;
  if (cfg->ring_depth < 1) return SASGD_EINVAL;
  if (cfg->compute != SASGD_FP32 && cfg->compute != SASGD_BF16) return SASGD_EINVAL;
  if (cfg->lr_mode < SASGD_LR_PER_GRADIENT || cfg->lr_mode > SASGD_LR_CONSTANT) return SASGD_EINVAL;
  if (cfg->net < SASGD_NET_NONE || cfg->net > SASGD_NET_CUSTOM) return SASGD_EINVAL;
  if (cfg->net != SASGD_NET_NONE && cfg->mu < 1) return SASGD_EINVAL;
  if (cfg->net == SASGD_NET_NONE && cfg->num_params < 1) return SASGD_EINVAL;
  if (!(cfg->alpha0 >= 0.f) || !(cfg->momentum >= 0.f) || !(cfg->weight_decay >= 0.f)) return SASGD_EINVAL;
  if ((cfg->alloc == nullptr) != (cfg->release == nullptr)) return SASGD_EINVAL;

  sasgd_ctx* ctx = new (std::nothrow) sasgd_ctx();
  if (!ctx) return SASGD_ENOMEM;
  ctx->cfg = *cfg;
  ctx->cfg.layers = nullptr;   // the layer table is copied into the net plan; never dereferenced later
  ctx->c = cfg->lambda / cfg->n;   // c = floor(lambda / n), Section 2.2
  ctx->stream = (hipStream_t)cfg->stream;
  ctx->timestamp = 0;
  if (hipGetDevice(&ctx->device) != hipSuccess) {
    (void)hipGetLastError();
    delete ctx;
    return SASGD_EHIP;
  }

  {
    // look up this device's statically allocated buffer now, so that a later sasgd_applyUpdateNoAlloc (possibly under
    // stream capture) finds the address cached
    float* unused = nullptr;
    if (static_sum_buffer(&unused) != hipSuccess) (void)hipGetLastError();
  }
  int rc = SASGD_OK;
  size_t pack_elems = 0;
  do {
    if (cfg->net == SASGD_NET_NONE) {
      ctx->P = cfg->num_params;
    } else {
      int64_t P = 0;
      std::string err;
      rc = net_create(*cfg, &ctx->net, &P, &pack_elems, err);
      if (rc != SASGD_OK) { ctx->error = err; break; }
      if (cfg->num_params != 0 && cfg->num_params != P) {
        rc = fail(ctx, SASGD_EINVAL, "num_params does not match the network"); break;
      }
      ctx->P = P;
    }
    const size_t P = (size_t)ctx->P;
    const size_t R = (size_t)cfg->ring_depth;
    const size_t Ppad = (P + 63) & ~(size_t)63;
    if (cfg->compute == SASGD_BF16) {
      ctx->ring_f32 = (float*)ctx_alloc(ctx, P * sizeof(float));
      ctx->slot_elems_b16 = Ppad + ((pack_elems + 63) & ~(size_t)63);
      ctx->ring_b16 = (bf16_t*)ctx_alloc(ctx, R * ctx->slot_elems_b16 * sizeof(bf16_t));
      if (!ctx->ring_b16) { rc = fail(ctx, SASGD_ENOMEM, "weight ring (bf16)"); break; }
    } else {
      ctx->slot_elems_f32 = Ppad;       // every slot starts 256-byte aligned (the kernels move 16 bytes per lane)
      ctx->ring_f32 = (float*)ctx_alloc(ctx, R * Ppad * sizeof(float));
    }
    ctx->v = (float*)ctx_alloc(ctx, P * sizeof(float));
    if (!ctx->ring_f32 || !ctx->v) { rc = fail(ctx, SASGD_ENOMEM, "weight ring / momentum"); break; }
    if (cfg->lambda / cfg->n >= kTwoPassMinC) {
      ctx->sum_buf = (float*)ctx_alloc(ctx, (size_t)kSumStretch * sizeof(float));
      if (!ctx->sum_buf) { rc = fail(ctx, SASGD_ENOMEM, "buffer of the two-pass update"); break; }
    }

    hipError_t e = hipMemcpyAsync(ctx->ring_f32, init_weights, P * sizeof(float),
                                  is_device_pointer(init_weights) ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice,
                                  ctx->stream);
    if (e == hipSuccess) e = hipMemsetAsync(ctx->v, 0, P * sizeof(float), ctx->stream);
    if (e == hipSuccess && cfg->compute == SASGD_BF16) {
      if (ctx->slot_elems_b16 > P)
        e = hipMemsetAsync(ctx->ring_b16, 0, R * ctx->slot_elems_b16 * sizeof(bf16_t), ctx->stream);
      if (e == hipSuccess) e = launch_fp32_to_bf16(ctx->ring_f32, ctx->ring_b16, ctx->P, ctx->stream);
      if (e == hipSuccess && ctx->net) e = net_prepare_version(ctx->net, ctx->ring_b16, ctx->ring_b16 + Ppad, ctx->stream);
    }
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);   // init_weights may be freed by the caller
    if (e != hipSuccess) { rc = fail_hip(ctx, e, "initialising weights"); break; }

    ctx->learners.resize((size_t)cfg->lambda);
    if (ctx->net) {
      size_t ws = net_workspace_bytes(ctx->net);
      for (int l = 0; l < cfg->lambda; l++) {
        Learner& L = ctx->learners[(size_t)l];
        L.grad = (float*)ctx_alloc(ctx, P * sizeof(float));
        L.workspace = ctx_alloc(ctx, ws);
        if (!L.grad || !L.workspace) { rc = fail(ctx, SASGD_ENOMEM, "learner buffers"); break; }
        // the workspace starts as zeros: the kernels rely on one never-written block of zeros inside it
        hipError_t ez = net_set_workspace(ctx->net, l, L.workspace, ctx->stream);
        if (ez != hipSuccess) { rc = fail_hip(ctx, ez, "clearing workspace"); break; }
      }
      if (rc != SASGD_OK) break;
      if (net_group_workspace_bytes(ctx->net) > 0) {
        void* g = ctx_alloc(ctx, net_group_workspace_bytes(ctx->net));
        if (!g) { rc = fail(ctx, SASGD_ENOMEM, "group staging area"); break; }
        hipError_t eg = net_set_group_workspace(ctx->net, g, ctx->stream);
        if (eg != hipSuccess) { rc = fail_hip(ctx, eg, "clearing the group staging area"); break; }
      }
      hipError_t ez = hipStreamSynchronize(ctx->stream);
      if (ez != hipSuccess) { rc = fail_hip(ctx, ez, "clearing workspace"); break; }
    }
  } while (0);

  if (rc != SASGD_OK) {
    // keep the message reachable: the caller gets no context on failure, so print it
    fprintf(stderr, "sasgd_create failed: %s\n", ctx->error.c_str());
    if (ctx->net) net_destroy(ctx->net);
    ctx_free_all(ctx);
    delete ctx;
    return rc;
  }
  *out = ctx;
  return SASGD_OK;
}

int sasgd_destroy(sasgd_ctx* ctx) {
  if (!ctx) return SASGD_EINVAL;
  (void)flush_updates(ctx);
  (void)hipStreamSynchronize(ctx->stream);
  prof_collect(ctx);
  if (ctx->net) net_destroy(ctx->net);
  ctx_free_all(ctx);
  delete ctx;
  return SASGD_OK;
}

int sasgd_getMinibatch(sasgd_ctx* ctx, int32_t learner, const float* images_dev, const int32_t* labels_dev) {
  if (!ctx) return SASGD_EINVAL;
  if (!ctx->net) return fail(ctx, SASGD_EINVAL, "getMinibatch: context has no network");
  if (learner < 0 || learner >= ctx->cfg.lambda || !images_dev || !labels_dev)
    return fail(ctx, SASGD_EINVAL, "getMinibatch: bad learner or null buffer");
  if (((uintptr_t)images_dev & 3) || ((uintptr_t)labels_dev & 3))
    return fail(ctx, SASGD_EINVAL, "getMinibatch: buffers must be 4-byte aligned");
  Learner& L = ctx->learners[(size_t)learner];
  L.images = images_dev;
  L.labels = labels_dev;
  return SASGD_OK;
}

int sasgd_pullWeights(sasgd_ctx* ctx, int32_t learner, int32_t staleness_request, int64_t* out_timestamp) {
  if (!ctx) return SASGD_EINVAL;
  if (!ctx->net) return fail(ctx, SASGD_EINVAL, "pullWeights: context has no network");
  if (learner < 0 || learner >= ctx->cfg.lambda || staleness_request < 0)
    return fail(ctx, SASGD_EINVAL, "pullWeights: bad learner or negative staleness");
  // a learner cannot hold weights older than theta_0: clamp, so that j >= 0 (Section 2.1: tau = i - j >= 0)
  const int64_t tau = std::min<int64_t>(staleness_request, ctx->timestamp);
  const int64_t j = ctx->timestamp - tau;
  if (!version_in_ring(ctx, j)) return fail(ctx, SASGD_ERANGE, "pullWeights: version has left the ring");
  Learner& L = ctx->learners[(size_t)learner];
  L.has_weights = true;
  L.evaluated = false;
  L.pulled_version = j;
  if (out_timestamp) *out_timestamp = j;
  return SASGD_OK;
}

int sasgd_calcGradient(sasgd_ctx* ctx, const int32_t* learners, int32_t count, float* out_loss_dev) {
  if (!ctx) return SASGD_EINVAL;
  if (!ctx->net) return fail(ctx, SASGD_EINVAL, "calcGradient: context has no network");
  if (!learners || count < 1 || count > ctx->cfg.lambda) return fail(ctx, SASGD_EINVAL, "calcGradient: bad learner list");
  {   // the weight versions these learners read, and the buffers they overwrite, belong to updates that may still be deferred
    const int rc = flush_updates(ctx);
    if (rc != SASGD_OK) return rc;
  }
  bool seen[kMaxLearners] = {false};
  LearnerBind binds[kMaxLearners];
  int ids[kMaxLearners];
  for (int k = 0; k < count; k++) {
    const int l = learners[k];
    if (l < 0 || l >= ctx->cfg.lambda || seen[l]) return fail(ctx, SASGD_EINVAL, "calcGradient: bad or duplicate learner");
    seen[l] = true;
    const Learner& L = ctx->learners[(size_t)l];
    if (!L.images || !L.has_weights) return fail(ctx, SASGD_ESTATE, "calcGradient: learner has no mini-batch or no weights bound");
    if (L.grad_state == GRAD_PENDING) return fail(ctx, SASGD_ESTATE, "calcGradient: learner's previous gradient is still pending at the server");
    if (!version_in_ring(ctx, L.pulled_version)) return fail(ctx, SASGD_ERANGE, "calcGradient: pulled version has left the ring");
    ids[k] = l;
    binds[k].images = L.images;
    binds[k].labels = L.labels;
    binds[k].weights = version_ptr(ctx, L.pulled_version);
    binds[k].version = L.pulled_version;
    binds[k].grad = L.grad;
  }
  prof_begin(ctx, 0);
  hipError_t e = net_calc_gradient(ctx->net, ids, binds, count, out_loss_dev, nullptr, ctx->stream);
  prof_end(ctx);
  if (e != hipSuccess) return fail_hip(ctx, e, "calcGradient");
  for (int k = 0; k < count; k++) {
    Learner& L = ctx->learners[(size_t)ids[k]];
    L.grad_timestamp = L.pulled_version;   // gradient timestamp = timestamp of the weights used (Section 2.1)
    L.grad_state = GRAD_COMPUTED;
    L.fc_expanded = false;
    L.has_weights = false;                 // one mini-batch per push: nothing is accrued at the learner
    L.images = nullptr;
    L.labels = nullptr;
  }
  return SASGD_OK;
}

int sasgd_evaluate(sasgd_ctx* ctx, const int32_t* learners, int32_t count, float* out_loss_dev, int32_t* out_rank_dev) {
  if (!ctx) return SASGD_EINVAL;
  if (!ctx->net) return fail(ctx, SASGD_EINVAL, "evaluate: context has no network");
  if (!learners || count < 1 || count > ctx->cfg.lambda) return fail(ctx, SASGD_EINVAL, "evaluate: bad learner list");
  if (!out_rank_dev || ((uintptr_t)out_rank_dev & 3)) return fail(ctx, SASGD_EINVAL, "evaluate: out_rank_dev must be a device int32 array");
  {
    const int rc = flush_updates(ctx);
    if (rc != SASGD_OK) return rc;
  }
  bool seen[kMaxLearners] = {false};
  LearnerBind binds[kMaxLearners];
  int ids[kMaxLearners];
  for (int k = 0; k < count; k++) {
    const int l = learners[k];
    if (l < 0 || l >= ctx->cfg.lambda || seen[l]) return fail(ctx, SASGD_EINVAL, "evaluate: bad or duplicate learner");
    seen[l] = true;
    const Learner& L = ctx->learners[(size_t)l];
    if (!L.images || !L.has_weights) return fail(ctx, SASGD_ESTATE, "evaluate: learner has no mini-batch or no weights bound");
    if (!version_in_ring(ctx, L.pulled_version)) return fail(ctx, SASGD_ERANGE, "evaluate: pulled version has left the ring");
    ids[k] = l;
    binds[k].images = L.images;
    binds[k].labels = L.labels;
    binds[k].weights = version_ptr(ctx, L.pulled_version);
    binds[k].version = L.pulled_version;
    binds[k].grad = nullptr;             // the evaluation pass writes no gradient
  }
  hipError_t e = net_calc_gradient(ctx->net, ids, binds, count, out_loss_dev, out_rank_dev, ctx->stream);
  if (e != hipSuccess) return fail_hip(ctx, e, "evaluate");
  // The bindings stay, but a binding that an evaluation has used no longer keeps its version in the ring: a training
  // loop evaluates and moves on, and must not be stopped by applyUpdate's eviction check many updates later.
  for (int k = 0; k < count; k++) ctx->learners[(size_t)ids[k]].evaluated = true;
  return SASGD_OK;
}

int sasgd_setBaseRate(sasgd_ctx* ctx, float alpha0) {
  if (!ctx) return SASGD_EINVAL;
  if (!(alpha0 >= 0.f) || !std::isfinite(alpha0)) return fail(ctx, SASGD_EINVAL, "setBaseRate: alpha0 must be finite and not negative");
  if (ctx->window_closed) return fail(ctx, SASGD_ESTATE, "setBaseRate: a window is closed; call applyUpdate first");
  ctx->cfg.alpha0 = alpha0;
  return SASGD_OK;
}

int sasgd_setPixelMean(sasgd_ctx* ctx, const float* mean_dev) {
  if (!ctx) return SASGD_EINVAL;
  if (!ctx->net) return fail(ctx, SASGD_EINVAL, "setPixelMean: context has no network");
  if ((uintptr_t)mean_dev & 3) return fail(ctx, SASGD_EINVAL, "setPixelMean: pointer must be 4-byte aligned");
  net_set_pixel_mean(ctx->net, mean_dev);
  return SASGD_OK;
}

int sasgd_pushGradient(sasgd_ctx* ctx, int32_t learner, int32_t* out_staleness) {
  if (!ctx) return SASGD_EINVAL;
  if (learner < 0 || learner >= ctx->cfg.lambda || !ctx->net) return fail(ctx, SASGD_EINVAL, "pushGradient: bad learner");
  Learner& L = ctx->learners[(size_t)learner];
  if (L.grad_state != GRAD_COMPUTED) return fail(ctx, SASGD_ESTATE, "pushGradient: no freshly computed gradient");
  if ((int)ctx->pending.size() >= kMaxLearners) return fail(ctx, SASGD_ESTATE, "pushGradient: pending queue full");
  Pending p;
  p.factors_ws = L.workspace;   // fully connected factors, if the network keeps any, live in the learner's workspace
  p.grad = L.grad;
  p.timestamp = L.grad_timestamp;
  p.staleness = (int32_t)(ctx->timestamp - L.grad_timestamp);   // tau = i - j
  p.learner = learner;
  ctx->pending.push_back(p);
  L.grad_state = GRAD_PENDING;
  if (out_staleness) *out_staleness = p.staleness;
  return SASGD_OK;
}

int sasgd_pushGradientExternal(sasgd_ctx* ctx, const float* grad_dev, int64_t timestamp, int32_t* out_staleness) {
  if (!ctx) return SASGD_EINVAL;
  if (!grad_dev || ((uintptr_t)grad_dev & 15)) return fail(ctx, SASGD_EINVAL, "pushGradientExternal: gradient must be a 16-byte aligned device pointer");
  if (timestamp < 0 || timestamp > ctx->timestamp) return fail(ctx, SASGD_EINVAL, "pushGradientExternal: timestamp must lie in [0, i]");
  if ((int)ctx->pending.size() >= kMaxLearners) return fail(ctx, SASGD_ESTATE, "pushGradientExternal: pending queue full");
  Pending p;
  p.factors_ws = nullptr;
  p.grad = grad_dev;
  p.timestamp = timestamp;
  p.staleness = (int32_t)(ctx->timestamp - timestamp);
  p.learner = -1;
  ctx->pending.push_back(p);
  if (out_staleness) *out_staleness = p.staleness;
  return SASGD_OK;
}

int sasgd_sumGradients(sasgd_ctx* ctx, int32_t* out_pending) {
  if (!ctx) return SASGD_EINVAL;
  if (out_pending) *out_pending = (int32_t)ctx->pending.size();
  if (ctx->window_closed) return fail(ctx, SASGD_ESTATE, "sumGradients: window already closed; call applyUpdate");
  const int c = ctx->c;
  if ((int)ctx->pending.size() < c) return fail(ctx, SASGD_ENOTREADY, "sumGradients: fewer than c gradients pending");
  int32_t taus[kMaxLearners];
  for (int l = 0; l < c; l++) taus[l] = ctx->pending[(size_t)l].staleness;
  window_coefficients(ctx->cfg.lr_mode, ctx->cfg.alpha0, c, taus, ctx->window_coef);
  ctx->window_count = c;
  ctx->window_closed = true;
  return SASGD_OK;
}

int sasgd_applyUpdate(sasgd_ctx* ctx, int64_t* out_new_timestamp) {
  if (!ctx) return SASGD_EINVAL;
  if (!ctx->window_closed) return fail(ctx, SASGD_ESTATE, "applyUpdate: no closed window; call sumGradients first");
  const int64_t i = ctx->timestamp;
  const int R = ctx->cfg.ring_depth;
  const int64_t evicted = i + 1 - R;   // version whose slot theta_{i+1} takes
  if (evicted >= 0 && R > 1) {
    for (const Learner& L : ctx->learners)
      if (L.has_weights && !L.evaluated && L.pulled_version == evicted)
        return fail(ctx, SASGD_ERANGE, "applyUpdate: a learner still holds the version this update would overwrite");
  }
  DeferredUpdate d;
  d.i = i;
  float abar = 0.f;
  bool own = true;                       // every gradient of the window lives in a learner's buffers
  for (int l = 0; l < ctx->window_count; l++) {
    d.grads.push_back(ctx->pending[(size_t)l]);
    d.coef.push_back(ctx->window_coef[l]);
    abar += ctx->window_coef[l];
    own = own && ctx->pending[(size_t)l].learner >= 0;
  }
  d.decay = abar * ctx->cfg.weight_decay;
  // Deferral: the kernels of consecutive updates are launched together, as one pass over the vector (fused steps),
  // once something needs their result.  Only windows whose gradients the library owns wait (a caller's buffer may
  // change as soon as this call returns), and long windows keep their two-pass form.
  const bool defer = !(ctx->cfg.flags & SASGD_FLAG_EAGER_UPDATES) && own && ctx->window_count < kTwoPassMinC;
  int queued = 0;
  for (const DeferredUpdate& q : ctx->deferred) queued += (int)q.grads.size();
  if (!defer || (int)ctx->deferred.size() == kMaxFusedSteps || queued + ctx->window_count > kMaxLearners) {
    const int rc = flush_updates(ctx);
    if (rc != SASGD_OK) return rc;
  }
  const int c_now = ctx->window_count;
  ctx->deferred.push_back(std::move(d));
  if (!defer) {
    const int rc = flush_updates(ctx);
    if (rc != SASGD_OK) { ctx->deferred.clear(); return rc; }
  }
  for (int l = 0; l < c_now; l++) {
    const int lr = ctx->pending[(size_t)l].learner;
    if (lr >= 0) ctx->learners[(size_t)lr].grad_state = GRAD_NONE;
  }
  ctx->pending.erase(ctx->pending.begin(), ctx->pending.begin() + c_now);
  ctx->window_closed = false;
  ctx->window_count = 0;
  ctx->timestamp = i + 1;   // every weight update increments the timestamp by one (Section 2.1)
  if (out_new_timestamp) *out_new_timestamp = ctx->timestamp;
  return SASGD_OK;
}

int sasgd_flush(sasgd_ctx* ctx) {
  if (!ctx) return SASGD_EINVAL;
  return flush_updates(ctx);
}

int sasgd_applyUpdateNoAlloc(const float* theta_in_dev, float* theta_out_dev, float* v_dev, uint16_t* shadow_out_dev,
                             int64_t num_params, int32_t c, const float* const* grads_dev, const int32_t* staleness,
                             int32_t lr_mode, float alpha0, float momentum, float weight_decay, void* stream,
                             char* err, size_t err_len) {
  auto refuse = [&](int code, const char* msg) {
    if (err && err_len > 0) snprintf(err, err_len, "applyUpdateNoAlloc: %s", msg);
    return code;
  };
  if (!theta_in_dev || !theta_out_dev || !v_dev || !grads_dev || !staleness) return refuse(SASGD_EINVAL, "null argument");
  if (c < 1 || c > SASGD_NOALLOC_MAX_GRADIENTS) return refuse(SASGD_EINVAL, "c must lie in 1..64");
  if (num_params < 1 || num_params > SASGD_NOALLOC_MAX_PARAMS) return refuse(SASGD_EINVAL, "num_params must lie in 1..2^32");
  if (lr_mode < SASGD_LR_PER_GRADIENT || lr_mode > SASGD_LR_CONSTANT) return refuse(SASGD_EINVAL, "unknown lr_mode");
  if (!(alpha0 >= 0.f) || !(momentum >= 0.f) || !(weight_decay >= 0.f)) return refuse(SASGD_EINVAL, "alpha0, momentum and weight_decay must not be negative");
  if (((uintptr_t)theta_in_dev | (uintptr_t)theta_out_dev | (uintptr_t)v_dev) & 15) return refuse(SASGD_EINVAL, "theta and v must be 16-byte aligned");
  if ((uintptr_t)shadow_out_dev & 7) return refuse(SASGD_EINVAL, "shadow_out_dev must be 8-byte aligned");
  UpdateLaunch u;
  for (int l = 0; l < c; l++) {
    if (!grads_dev[l] || ((uintptr_t)grads_dev[l] & 15)) return refuse(SASGD_EINVAL, "every gradient must be a 16-byte aligned device pointer");
    if (staleness[l] < 0) return refuse(SASGD_EINVAL, "negative staleness");
    u.grads[l] = grads_dev[l];
  }
  window_coefficients(lr_mode, alpha0, c, staleness, u.coef);
  float abar = 0.f;
  for (int l = 0; l < c; l++) abar += u.coef[l];
  float* sums = nullptr;
  hipError_t e = static_sum_buffer(&sums);   // a lookup after the first call on this device; never an allocation
  if (e != hipSuccess) return refuse(SASGD_EHIP, hipGetErrorString(e));
  u.theta_in = theta_in_dev;
  u.theta_out = theta_out_dev;
  u.v = v_dev;
  u.shadow_out = shadow_out_dev;
  u.P = num_params;
  u.c = c;
  u.momentum = momentum;
  u.decay = abar * weight_decay;
  u.reverse = 0;
  u.sum_buf = sums;
  e = launch_apply_update(u, (hipStream_t)stream);
  if (e != hipSuccess) return refuse(SASGD_EHIP, hipGetErrorString(e));
  return SASGD_OK;
}

int sasgd_timestamp(sasgd_ctx* ctx, int64_t* out) {
  if (!ctx || !out) return SASGD_EINVAL;
  *out = ctx->timestamp;
  return SASGD_OK;
}

int sasgd_numParams(sasgd_ctx* ctx, int64_t* out) {
  if (!ctx || !out) return SASGD_EINVAL;
  *out = ctx->P;
  return SASGD_OK;
}

int sasgd_gradientsPerUpdate(sasgd_ctx* ctx, int32_t* out_c) {
  if (!ctx || !out_c) return SASGD_EINVAL;
  *out_c = ctx->c;
  return SASGD_OK;
}

int sasgd_factoredParams(sasgd_ctx* ctx, int64_t* out) {
  if (!ctx || !out) return SASGD_EINVAL;
  *out = 0;
  if (ctx->net) {
    FactoredLayer fl[kMaxFactoredLayers];
    const int nfl = net_factored_layers(ctx->net, fl, kMaxFactoredLayers);
    for (int k = 0; k < nfl; k++) *out += (int64_t)fl[k].in * fl[k].out;
  }
  return SASGD_OK;
}

int sasgd_gradientTimestamp(sasgd_ctx* ctx, int32_t learner, int64_t* out) {
  if (!ctx || !out || learner < 0 || learner >= ctx->cfg.lambda) return SASGD_EINVAL;
  const Learner& L = ctx->learners[(size_t)learner];
  *out = L.grad_state == GRAD_NONE ? -1 : L.grad_timestamp;
  return SASGD_OK;
}

int sasgd_copyWeights(sasgd_ctx* ctx, int64_t version, float* host_out) {
  if (!ctx || !host_out) return SASGD_EINVAL;
  if (!version_in_ring(ctx, version)) return fail(ctx, SASGD_ERANGE, "copyWeights: version not in the ring");
  {
    const int rc = flush_updates(ctx);
    if (rc != SASGD_OK) return rc;
  }
  const size_t bytes = (size_t)ctx->P * sizeof(float);
  hipError_t e;
  if (ctx->cfg.compute == SASGD_BF16 && version != ctx->timestamp) {
    // only the bf16 copy of an old version exists: fetch it and widen on the host
    std::vector<bf16_t> tmp((size_t)ctx->P);
    e = hipMemcpyAsync(tmp.data(), ctx->ring_b16 + (size_t)slot_of(ctx, version) * ctx->slot_elems_b16,
                       (size_t)ctx->P * sizeof(bf16_t), hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    if (e == hipSuccess)
      for (size_t k = 0; k < (size_t)ctx->P; k++) {
        uint32_t u = (uint32_t)tmp[k] << 16;
        memcpy(&host_out[k], &u, 4);
      }
  } else {
    const float* src = ctx->cfg.compute == SASGD_BF16 ? ctx->ring_f32
                                                      : ctx->ring_f32 + (size_t)slot_of(ctx, version) * ctx->slot_elems_f32;
    e = hipMemcpyAsync(host_out, src, bytes, hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  }
  if (e != hipSuccess) return fail_hip(ctx, e, "copyWeights");
  return SASGD_OK;
}

// Writes the fully connected weight gradients that the learner holds as factors into its flat gradient buffer.
static hipError_t expand_factored(sasgd_ctx* ctx, Learner& L) {
  if (!ctx->net || L.fc_expanded || L.grad_timestamp < 0) return hipSuccess;
  FactoredLayer fl[kMaxFactoredLayers];
  const int nfl = net_factored_layers(ctx->net, fl, kMaxFactoredLayers);
  for (int k = 0; k < nfl; k++) {
    const FactoredLayer& F = fl[k];
    hipError_t e = launch_fc_expand_factors((const bf16_t*)L.workspace + F.fx_off, (const bf16_t*)L.workspace + F.fdy_off,
                                            L.grad + F.w_off, F.N, F.in, F.out, F.NP, ctx->stream);
    if (e != hipSuccess) return e;
  }
  L.fc_expanded = true;
  return hipSuccess;
}

int sasgd_copyGradient(sasgd_ctx* ctx, int32_t learner, float* host_out) {
  if (!ctx || !host_out || learner < 0 || learner >= ctx->cfg.lambda) return SASGD_EINVAL;
  Learner& L = ctx->learners[(size_t)learner];
  if (!L.grad) return fail(ctx, SASGD_EINVAL, "copyGradient: context has no network");
  if (L.grad_timestamp < 0) return fail(ctx, SASGD_ESTATE, "copyGradient: learner has not computed a gradient");
  {
    const int rc = flush_updates(ctx);
    if (rc != SASGD_OK) return rc;
  }
  hipError_t e = expand_factored(ctx, L);
  if (e == hipSuccess) e = hipMemcpyAsync(host_out, L.grad, (size_t)ctx->P * sizeof(float), hipMemcpyDeviceToHost, ctx->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return fail_hip(ctx, e, "copyGradient");
  return SASGD_OK;
}

int sasgd_copyMomentum(sasgd_ctx* ctx, float* host_out) {
  if (!ctx || !host_out) return SASGD_EINVAL;
  {
    const int rc = flush_updates(ctx);
    if (rc != SASGD_OK) return rc;
  }
  hipError_t e = hipMemcpyAsync(host_out, ctx->v, (size_t)ctx->P * sizeof(float), hipMemcpyDeviceToHost, ctx->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return fail_hip(ctx, e, "copyMomentum");
  return SASGD_OK;
}

int sasgd_gradientPtr(sasgd_ctx* ctx, int32_t learner, float** out_dev) {
  if (!ctx || !out_dev || learner < 0 || learner >= ctx->cfg.lambda) return SASGD_EINVAL;
  if (!ctx->learners[(size_t)learner].grad) return fail(ctx, SASGD_EINVAL, "gradientPtr: context has no network");
  {
    const int rc = flush_updates(ctx);
    if (rc != SASGD_OK) return rc;
  }
  hipError_t e = expand_factored(ctx, ctx->learners[(size_t)learner]);
  if (e != hipSuccess) return fail_hip(ctx, e, "gradientPtr");
  *out_dev = ctx->learners[(size_t)learner].grad;
  return SASGD_OK;
}

int sasgd_setProfiling(sasgd_ctx* ctx, int32_t on) {
  if (!ctx) return SASGD_EINVAL;
  (void)flush_updates(ctx);
  prof_collect(ctx);
  ctx->profiling = on != 0;
  ctx->phase_ms[0] = ctx->phase_ms[1] = 0.0;
  ctx->phase_calls[0] = ctx->phase_calls[1] = 0;
  ctx->update_passes = 0;
  return SASGD_OK;
}

int sasgd_phaseTime(sasgd_ctx* ctx, int32_t which, double* out_ms_total, int64_t* out_calls) {
  if (!ctx || which < 0 || which > 2) return SASGD_EINVAL;
  (void)flush_updates(ctx);
  prof_collect(ctx);
  if (out_ms_total) *out_ms_total = ctx->phase_ms[which == 2 ? 1 : which];
  if (out_calls) *out_calls = which == 2 ? ctx->update_passes : ctx->phase_calls[which];
  return SASGD_OK;
}

}  // extern "C"
