/*
 * sasgd.h -- C ABI of the staleness-aware n-softsync ASGD hot path on one MI355X (gfx950).
 *
 * The calls carry the names of the protocol steps of the paper's Section 2.1:
 *   learner:           getMinibatch, pullWeights, calcGradient, pushGradient
 *   parameter server:  sumGradients, applyUpdate
 * lambda learners are simulated on one GPU.  The server keeps the weight versions
 * theta_i, theta_{i-1}, ... in a ring buffer in HBM; a learner that "pulls" binds one of
 * those versions, so the staleness tau = i - j of Section 2.1 is reproduced exactly.
 *
 * Conventions
 *  - Plain C.  Every call returns 0 (SASGD_OK) or a negative SASGD_E* code; nothing aborts or
 *    throws.  sasgd_last_error() gives a message for the last failure on a context.
 *  - "dev" pointers are device (HBM) addresses, "host" pointers are ordinary host memory.
 *  - All device work is enqueued on the hipStream_t given at creation (passed as void*).
 *    Calls return without waiting for the device, except the copy* getters, which block.
 *  - The context owns the weight ring, momentum, per-learner gradient buffers and
 *    workspaces (and, when floor(lambda / n) >= 25, an 8 MiB buffer of partial sums for the
 *    update of long windows); all are allocated in sasgd_create and freed in sasgd_destroy; no other
 *    call allocates device memory.  The caller owns mini-batch buffers and externally
 *    pushed gradients and keeps them alive until the work that reads them has completed
 *    on the stream.
 *  - A context is not thread-safe.
 *
 * Flat parameter order (weights, gradients, momentum alike): layers in network order; for
 * each convolution the weights [Cout][Cin][kh][kw] then the bias [Cout]; for each fully
 * connected layer the weights [out][in] (in = C,H,W flattened in that order) then the bias.
 */
#ifndef SASGD_H
#define SASGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sasgd_ctx sasgd_ctx;

enum {
  SASGD_OK = 0,
  SASGD_EINVAL = -1,    /* bad argument or configuration                                   */
  SASGD_ESTATE = -2,    /* protocol order violated (e.g. calcGradient before pullWeights)   */
  SASGD_ENOTREADY = -3, /* fewer than c gradients pending                                  */
  SASGD_ERANGE = -4,    /* weight version not (or no longer) in the ring                   */
  SASGD_EHIP = -5,      /* a HIP runtime call failed                                       */
  SASGD_ENOMEM = -6     /* allocation failed                                               */
};

enum { SASGD_NET_NONE = 0, SASGD_NET_CIFAR3 = 1, SASGD_NET_ALEX8 = 2, SASGD_NET_CUSTOM = 3 };
enum { SASGD_FP32 = 0, SASGD_BF16 = 1 };
enum { SASGD_LR_PER_GRADIENT = 0, SASGD_LR_MEAN_STALENESS = 1, SASGD_LR_CONSTANT = 2 };
enum { SASGD_CONV = 0, SASGD_MAXPOOL = 1, SASGD_AVGPOOL = 2, SASGD_RELU = 3, SASGD_FC = 4 };
/* flags */
enum { SASGD_FLAG_FLAT_FC_GRADIENT = 1, SASGD_FLAG_EAGER_UPDATES = 2 };   /* see sasgd_config.flags */

/* One layer of a custom network (SASGD_NET_CUSTOM).  The loss, softmax cross-entropy averaged
 * over the mini-batch, follows the last layer implicitly.
 *   CONV:    units = output channels, window x window kernel, stride, pad (zero padding)
 *   MAXPOOL / AVGPOOL: window, stride; output size ceil((H - window)/stride) + 1, windows clipped
 *            at the border, the average taken over the in-bounds elements
 *   RELU:    must directly follow a CONV, FC or pooling layer
 *   FC:      units = outputs                                                              */
typedef struct {
  int32_t kind, units, window, stride, pad;
} sasgd_layer;

typedef struct {
  int32_t lambda;       /* number of learners (Section 2.1), 1..64                                   */
  int32_t mu;           /* mini-batch size per learner (Section 2.1); ignored for NET_NONE           */
  int32_t n;            /* splitting parameter of n-softsync, 1..lambda; c = floor(lambda / n)
                           gradients enter one update (Section 2.2)                                  */
  int32_t ring_depth;   /* R >= 1 weight versions kept; a pull of staleness tau needs tau < R        */
  int32_t net;          /* SASGD_NET_*; NET_NONE = server only (gradients pushed externally)         */
  int32_t compute;      /* SASGD_FP32, or SASGD_BF16 = bf16 operands, fp32 accumulation; master
                           weights, momentum and gradients are fp32 either way                       */
  int32_t lr_mode;      /* PER_GRADIENT: alpha0 / tau_l for each gradient (Section 2.4);
                           MEAN_STALENESS: alpha0 / mean_l(tau_l); CONSTANT: alpha0.  A staleness
                           of 0 uses alpha0 unmodulated in every mode.                               */
  int32_t flags;        /* 0, or SASGD_FLAG_FLAT_FC_GRADIENT.  By default (BF16 compute, mu <= 32) the weight
                           gradient of a fully connected layer is not written out: with a mini-batch of mu
                           images it is the rank-mu product dy^T x, so calcGradient keeps the two factors
                           (mu x out and mu x in values) and applyUpdate forms the product on the fly in the
                           same fp32 arithmetic.  The 4 bytes per weight of gradient written by the learner
                           and read by the server disappear; copyGradient / gradientPtr expand the product on
                           demand.  The flag forces the written-out gradient instead.
                           SASGD_FLAG_EAGER_UPDATES: applyUpdate enqueues its kernels before it returns.  By default
                           the kernels of an update whose gradients all come from the library's learners wait until
                           something needs their result (see sasgd_applyUpdate).                              */
  int64_t num_params;   /* NET_NONE: length P of the parameter vector; otherwise 0 or the expected
                           P, checked against the network                                            */
  float alpha0;         /* base learning rate                                                        */
  float momentum;       /* m in  v <- m v + sum_l coef_l g_l + (sum_l coef_l) wd theta               */
  float weight_decay;   /* wd; theta_{i+1} = theta_i - v                                             */
  float reserved1;
  void* stream;         /* hipStream_t; NULL = the default stream                                    */
  /* NET_CUSTOM only */
  const sasgd_layer* layers;
  int32_t num_layers;
  int32_t in_channels, in_height, in_width;
  /* optional allocator (e.g. backed by a tensor library); NULL = hipMalloc / hipFree */
  void* (*alloc)(size_t bytes, void* user);
  void (*release)(void* ptr, void* user);
  void* alloc_user;
} sasgd_config;

/* Create a context.  init_weights: P floats in flat parameter order, host or device memory
 * (detected); copied into weight version 0.  Momentum starts at 0, the timestamp at 0.
 * Errors: EINVAL (configuration), ENOMEM, EHIP. */
int sasgd_create(const sasgd_config* cfg, const float* init_weights, sasgd_ctx** out);
int sasgd_destroy(sasgd_ctx* ctx);

/* ---- learner side (Section 2.1) ------------------------------------------------------- */

/* getMinibatch: bind the mini-batch learner `learner` will use in its next calcGradient.
 * images_dev: float32 [mu][C][H][W]; labels_dev: int32 [mu], each in [0, classes).  No copy is
 * made.  (Random selection from a dataset is the caller's business.) */
int sasgd_getMinibatch(sasgd_ctx* ctx, int32_t learner, const float* images_dev, const int32_t* labels_dev);

/* pullWeights: bind weight version j = i - min(staleness_request, i), i = current timestamp;
 * the gradient computed next carries timestamp j (Section 2.1).  staleness_request = 0 is the
 * paper's "pull the current weights"; a positive request stands in for a learner that pulled
 * that many updates ago.  Errors: ERANGE if version j has left the ring. */
int sasgd_pullWeights(sasgd_ctx* ctx, int32_t learner, int32_t staleness_request, int64_t* out_timestamp);

/* calcGradient: forward and backward pass of the network over the bound mini-batches of the
 * `count` listed learners (each on its own bound weight version), all in one batch of kernel
 * launches.  Each learner's result is the gradient of the mean loss over its mini-batch, i.e.
 * already divided by mu (Section 2.1; inner term of the server-view update, Section 3).
 * out_loss_dev: optional device float[count], the mean loss of each listed learner.
 * Errors: ESTATE if a listed learner has no mini-batch or weights bound, or still has a
 * gradient pending at the server; EINVAL for duplicates or NET_NONE. */
int sasgd_calcGradient(sasgd_ctx* ctx, const int32_t* learners, int32_t count, float* out_loss_dev);

/* pushGradient: hand the learner's gradient and its timestamp j to the server.  The staleness
 * tau = i - j (i = server timestamp now) is fixed here and returned.  No data moves. */
int sasgd_pushGradient(sasgd_ctx* ctx, int32_t learner, int32_t* out_staleness);

/* Push a caller-owned device gradient (float32 [P]) with timestamp j <= i (server microbenchmark,
 * or gradients produced elsewhere). */
int sasgd_pushGradientExternal(sasgd_ctx* ctx, const float* grad_dev, int64_t timestamp, int32_t* out_staleness);

/* ---- parameter-server side (Section 2.1, 2.2, 2.4) ------------------------------------ */

/* sumGradients: close the accumulation window.  Needs at least c pending gradients, takes the
 * first c in arrival order and fixes their coefficients coef_l = alpha(tau_l) / c.  The sum itself
 * is carried out inside applyUpdate's single pass.  out_pending: gradients pending before the call.
 * Errors: ENOTREADY when fewer than c are pending (nothing changes). */
int sasgd_sumGradients(sasgd_ctx* ctx, int32_t* out_pending);

/* applyUpdate: theta_{i+1} = theta_i - v with v <- m v + sum_l coef_l g_l + (sum_l coef_l) wd theta_i
 * (the n-softsync rule of Section 2.2 when m = wd = 0), written to ring slot (i+1) mod R; the
 * timestamp becomes i+1.  Errors: ESTATE without a closed window; ERANGE if the slot to be
 * overwritten holds a version some learner has pulled but not yet used.
 * Deferred launch: when every gradient of the window was computed by the library's learners (pushGradient) and the
 * window has fewer than 25 gradients, the host bookkeeping is done at once but the kernels are enqueued later --
 * at the next calcGradient, evaluate, getter, sasgd_flush or sasgd_destroy, or when 8 updates or 64 gradients have
 * gathered -- so that consecutive updates become ONE pass over theta and v: they are read once, the steps are applied
 * in order in registers (the arithmetic of the separate launches, bit for bit) and written once, and every step still
 * writes its weight version.  With n = lambda (one gradient per update) this is most of the server's memory traffic.
 * Windows holding a gradient pushed from outside (pushGradientExternal) are never deferred: their kernels are enqueued
 * before applyUpdate returns, as SASGD_FLAG_EAGER_UPDATES makes every update do. */
int sasgd_applyUpdate(sasgd_ctx* ctx, int64_t* out_new_timestamp);

/* Enqueue the kernels of all deferred updates now (no-op if there are none).  Call it before waiting on the stream for
 * the server's work, e.g. in front of a timing point. */
int sasgd_flush(sasgd_ctx* ctx);

/* applyUpdateNoAlloc: the server update for callers that cannot allocate device memory or create library objects
 * around a call -- code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  It is
 * sumGradients + applyUpdate on caller-owned vectors, without a context:
 *     coef_l = alpha(tau_l) / c   (lr_mode, alpha0 and the staleness tau_l = staleness[l] as in sumGradients)
 *     v <- momentum v + sum_l coef_l g_l + (sum_l coef_l) weight_decay theta_in;   theta_out = theta_in - v
 * run by the kernels of sasgd_applyUpdate: same arithmetic, same order, bit-identical results.  Windows of 25 and
 * more gradients over at least 2 Mi parameters take the two-launch form, whose 8 MiB of partial sums live in an array
 * compiled into the library (one copy per GPU, held until the process ends) instead of in a context's allocation.
 *   theta_in_dev, theta_out_dev, v_dev: device float32 [num_params], 16-byte aligned; theta_out may be theta_in.
 *   shadow_out_dev: optional device bf16 [num_params] (8-byte aligned) receiving theta_out rounded to nearest even.
 *   grads_dev: HOST array of c device pointers (float32 [num_params] each, 16-byte aligned); staleness: HOST int32 [c].
 *   stream: hipStream_t the launches are enqueued on (NULL = default stream); the call does not wait for them.
 *   err / err_len: optional host buffer that receives a message when the call fails.
 * Limits: 1 <= c <= SASGD_NOALLOC_MAX_GRADIENTS, 1 <= num_params <= SASGD_NOALLOC_MAX_PARAMS; anything beyond is
 * refused with EINVAL and a message.  Calls no hipMalloc / hipFree and no allocating library routine.
 * All calls on one GPU share that GPU's array: two calls whose kernels may overlap in time on one GPU (different
 * streams, different threads) race on it; calls on one stream are ordered and safe.  Nothing in it needs clearing:
 * every launch that reads a stretch of sums follows the launch that wrote exactly that stretch. */
#define SASGD_NOALLOC_MAX_GRADIENTS 64
#define SASGD_NOALLOC_MAX_PARAMS ((int64_t)1 << 32)
int sasgd_applyUpdateNoAlloc(const float* theta_in_dev, float* theta_out_dev, float* v_dev, uint16_t* shadow_out_dev,
                             int64_t num_params, int32_t c, const float* const* grads_dev, const int32_t* staleness,
                             int32_t lr_mode, float alpha0, float momentum, float weight_decay, void* stream,
                             char* err, size_t err_len);

/* ---- training-loop pieces around the hot path (Sections 4.1 - 4.3) ---------------------- */

/* evaluate: forward pass only over the bound mini-batches of the listed learners, each on its
 * bound weight version (the test / validation error curves of Section 4.3).  Nothing is
 * consumed: bindings, gradients and the protocol state stay as they are, except that a binding an
 * evaluation has used no longer holds its version in the ring (applyUpdate may overwrite it; a later
 * calcGradient on that binding then fails with ERANGE until the learner pulls again).
 * out_loss_dev: optional device float[count], mean loss per listed learner.
 * out_rank_dev: device int32[count * mu]; entry k*mu + s is the number of classes that precede
 * the true class of image s of learners[k] when the class scores are sorted in descending
 * order (equal scores: lower class index first).  rank >= 1 is a top-1 error, rank >= 5 a
 * top-5 error; a label outside [0, classes) gets rank = classes.
 * Errors: ESTATE if a listed learner has no mini-batch or weights bound; EINVAL as calcGradient. */
int sasgd_evaluate(sasgd_ctx* ctx, const int32_t* learners, int32_t count, float* out_loss_dev, int32_t* out_rank_dev);

/* Step decay of the base learning rate alpha0 (Section 4.3 lowers it by a constant factor at
 * fixed epochs).  Takes effect from the next sumGradients.  Errors: EINVAL unless finite and >= 0;
 * ESTATE while a window is closed (its coefficients are already fixed). */
int sasgd_setBaseRate(sasgd_ctx* ctx, float alpha0);

/* Per-pixel mean (Section 4.1 preprocessing): mean_dev is device float32 [C][H][W], subtracted
 * in fp32 from every image while calcGradient / evaluate re-lay out their input; NULL switches
 * it off.  Caller-owned; must stay valid while in use.  Errors: EINVAL for NET_NONE or a
 * pointer that is not 4-byte aligned. */
int sasgd_setPixelMean(sasgd_ctx* ctx, const float* mean_dev);

/* ---- getters -------------------------------------------------------------------------- */
int sasgd_timestamp(sasgd_ctx* ctx, int64_t* out);
int sasgd_numParams(sasgd_ctx* ctx, int64_t* out);
int sasgd_gradientsPerUpdate(sasgd_ctx* ctx, int32_t* out_c);
/* Number of parameters (fully connected weights) whose gradients are kept as factors (see flags); 0 if none. */
int sasgd_factoredParams(sasgd_ctx* ctx, int64_t* out);
/* Timestamp of the learner's last computed gradient (-1 if none). */
int sasgd_gradientTimestamp(sasgd_ctx* ctx, int32_t learner, int64_t* out);
/* Blocking copies to host float[P].  copyWeights: version must be in the ring; with BF16 compute
 * only the current version is held in fp32, older ones are returned from their bf16 copies. */
int sasgd_copyWeights(sasgd_ctx* ctx, int64_t version, float* host_out);
int sasgd_copyGradient(sasgd_ctx* ctx, int32_t learner, float* host_out);
int sasgd_copyMomentum(sasgd_ctx* ctx, float* host_out);
/* Device address of a learner's gradient buffer (float32 [P]); valid for the context's lifetime.
 * Fully connected weight gradients kept as factors (see flags) are expanded into the buffer by
 * this call and by copyGradient (enqueued on the context's stream). */
int sasgd_gradientPtr(sasgd_ctx* ctx, int32_t learner, float** out_dev);

/* Accumulated device time of the two hot phases since the last reset, measured with HIP events
 * on the context's stream when profiling is on (blocking query).
 * which: 0 = calcGradient launches (calls = calcGradient calls), 1 = applyUpdate kernels (calls = updates applied),
 * 2 = the same time as 1 with calls = passes over the vector (a pass applies one or several deferred updates). */
int sasgd_setProfiling(sasgd_ctx* ctx, int32_t on);
int sasgd_phaseTime(sasgd_ctx* ctx, int32_t which, double* out_ms_total, int64_t* out_calls);

const char* sasgd_last_error(sasgd_ctx* ctx);
const char* sasgd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SASGD_H */
