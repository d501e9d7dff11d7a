/*
 * CPU oracle for calcGradient -- TEST INFRASTRUCTURE, not part of the product.
 *
 * A plain, slow, double-precision implementation of what a learner computes in the
 * calcGradient step of Section 2.1: the gradient of the mini-batch loss with respect
 * to every trainable parameter, divided by the mini-batch size (the inner brace of
 * the server-view update equation in Section 3).  The networks are the layer types the
 * experimental section names (Section 4.1): convolution, max/average pooling, ReLU,
 * fully connected, softmax output with cross-entropy loss.
 *
 * Every layer is the textbook definition written as nested loops; the backward pass
 * is the chain rule applied layer by layer.  No im2col, no GEMM, no blocking.
 * OpenMP only spreads independent outer iterations over cores.
 *
 * Only tests, the smoke check and the bench's cpu_baseline leg may call this file.
 * It shares nothing with the HIP path.
 *
 * Tensor layout: images [N][C][H][W], conv weights [Cout][Cin][kh][kw], fc weights
 * [out][in] with `in` flattened as (C,H,W); flat parameter vector = for each layer in
 * network order, weights then bias.
 *
 * Readings of points on which the paper is silent (parity rests on them):
 *  - pooling windows: output size ceil((H-k)/s)+1, windows clipped at the border;
 *    the average pool divides by the number of in-bounds elements;
 *  - max-pool ties go to the first element in row-major window order; ReLU'(0) = 0;
 *  - loss = mean over the mini-batch of -log softmax(z)[label].
 *
 * Reduced-precision mode (round_bf16 != 0).  "bf16 compute" means that every tensor kept in
 * memory between layers is a bfloat16 number (8 significant bits, round to nearest even) while
 * sums are carried in higher precision.  In this mode the oracle rounds, and only rounds: the
 * images, the parameters, the output of every layer except the final class scores, the gradient
 * of the loss with respect to the class scores, and every activation gradient handed from one
 * layer to the previous one.  All sums stay in double precision and the parameter gradient is
 * not rounded.  ReLU signs and max-pool winners are therefore decided on bfloat16 values, the
 * precision in which a bf16 implementation has to take them.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

enum { L_CONV = 0, L_MAXPOOL = 1, L_AVGPOOL = 2, L_RELU = 3, L_FC = 4 };

/* One row of the layer table passed in from Python: type, a, b, c, d
 *   conv: a=cout b=k c=stride d=pad;  pool: a=k b=stride;  fc: a=out            */
typedef struct { int type, a, b, c, d; } olayer;

static int pool_out(int n, int k, int s) {
  int o = (n - k + s - 1) / s + 1;          /* ceil((n-k)/s) + 1 */
  if ((o - 1) * s >= n) o -= 1;             /* last window must start inside */
  return o < 1 ? 1 : o;
}

/* round a double to the nearest bfloat16 (ties to even), going through float as hardware does */
double round_to_bf16(double v) {
  float f = (float)v;
  unsigned int u;
  memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return v;             /* NaN stays NaN */
  u += 0x7fffu + ((u >> 16) & 1u);
  u &= 0xffff0000u;
  memcpy(&f, &u, 4);
  return (double)f;
}
static void round_array(double* a, size_t n, int on) {
  if (!on) return;
  for (size_t i = 0; i < n; i++) a[i] = round_to_bf16(a[i]);
}

/* ------------------------------------------------------------------ convolution */
void conv_forward(const double* x, const double* w, const double* b, double* y,
                  int N, int C, int H, int W, int Co, int k, int s, int p) {
  int OH = (H + 2 * p - k) / s + 1, OW = (W + 2 * p - k) / s + 1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; n++)
    for (int co = 0; co < Co; co++) {
      double* yo = y + ((size_t)n * Co + co) * OH * OW;
      for (int i = 0; i < OH * OW; i++) yo[i] = b[co];
      for (int ci = 0; ci < C; ci++)
        for (int kh = 0; kh < k; kh++)
          for (int kw = 0; kw < k; kw++) {
            double wv = w[(((size_t)co * C + ci) * k + kh) * k + kw];
            const double* xi = x + ((size_t)n * C + ci) * H * W;
            for (int oh = 0; oh < OH; oh++) {
              int ih = oh * s + kh - p;
              if (ih < 0 || ih >= H) continue;
              for (int ow = 0; ow < OW; ow++) {
                int iw = ow * s + kw - p;
                if (iw < 0 || iw >= W) continue;
                yo[oh * OW + ow] += wv * xi[ih * W + iw];
              }
            }
          }
    }
}

/* dx may be NULL (first layer).  dw, db are overwritten. */
void conv_backward(const double* x, const double* w, const double* dy, double* dx,
                   double* dw, double* db, int N, int C, int H, int W, int Co, int k,
                   int s, int p) {
  int OH = (H + 2 * p - k) / s + 1, OW = (W + 2 * p - k) / s + 1;
  /* dw[co][ci][kh][kw] = sum_{n,oh,ow} dy[n][co][oh][ow] * x[n][ci][ih][iw];  db[co] = sum dy */
#pragma omp parallel for schedule(static)
  for (int co = 0; co < Co; co++) {
    double sb = 0.0;
    for (int n = 0; n < N; n++) {
      const double* d = dy + ((size_t)n * Co + co) * OH * OW;
      for (int i = 0; i < OH * OW; i++) sb += d[i];
    }
    db[co] = sb;
    for (int ci = 0; ci < C; ci++)
      for (int kh = 0; kh < k; kh++)
        for (int kw = 0; kw < k; kw++) {
          double acc = 0.0;
          for (int n = 0; n < N; n++) {
            const double* d = dy + ((size_t)n * Co + co) * OH * OW;
            const double* xi = x + ((size_t)n * C + ci) * H * W;
            for (int oh = 0; oh < OH; oh++) {
              int ih = oh * s + kh - p;
              if (ih < 0 || ih >= H) continue;
              for (int ow = 0; ow < OW; ow++) {
                int iw = ow * s + kw - p;
                if (iw < 0 || iw >= W) continue;
                acc += d[oh * OW + ow] * xi[ih * W + iw];
              }
            }
          }
          dw[(((size_t)co * C + ci) * k + kh) * k + kw] = acc;
        }
  }
  if (!dx) return;
  /* dx[n][ci][ih][iw] = sum_{co,kh,kw} dy[n][co][oh][ow] * w[co][ci][kh][kw] */
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; n++)
    for (int ci = 0; ci < C; ci++) {
      double* dxi = dx + ((size_t)n * C + ci) * H * W;
      for (int i = 0; i < H * W; i++) dxi[i] = 0.0;
      for (int co = 0; co < Co; co++) {
        const double* d = dy + ((size_t)n * Co + co) * OH * OW;
        for (int kh = 0; kh < k; kh++)
          for (int kw = 0; kw < k; kw++) {
            double wv = w[(((size_t)co * C + ci) * k + kh) * k + kw];
            for (int oh = 0; oh < OH; oh++) {
              int ih = oh * s + kh - p;
              if (ih < 0 || ih >= H) continue;
              for (int ow = 0; ow < OW; ow++) {
                int iw = ow * s + kw - p;
                if (iw < 0 || iw >= W) continue;
                dxi[ih * W + iw] += wv * d[oh * OW + ow];
              }
            }
          }
      }
    }
}

/* ------------------------------------------------------------------ pooling */
void maxpool_forward(const double* x, double* y, int* arg, int NC, int H, int W, int k, int s) {
  int OH = pool_out(H, k, s), OW = pool_out(W, k, s);
#pragma omp parallel for schedule(static)
  for (int nc = 0; nc < NC; nc++) {
    const double* xi = x + (size_t)nc * H * W;
    for (int oh = 0; oh < OH; oh++)
      for (int ow = 0; ow < OW; ow++) {
        int best = -1;
        double bv = 0.0;
        for (int ih = oh * s; ih < oh * s + k && ih < H; ih++)
          for (int iw = ow * s; iw < ow * s + k && iw < W; iw++) {
            double v = xi[ih * W + iw];
            if (best < 0 || v > bv) { best = ih * W + iw; bv = v; }   /* first maximum wins */
          }
        y[((size_t)nc * OH + oh) * OW + ow] = bv;
        arg[((size_t)nc * OH + oh) * OW + ow] = best;
      }
  }
}

void maxpool_backward(const double* dy, const int* arg, double* dx, int NC, int H, int W, int k,
                      int s) {
  int OH = pool_out(H, k, s), OW = pool_out(W, k, s);
#pragma omp parallel for schedule(static)
  for (int nc = 0; nc < NC; nc++) {
    double* dxi = dx + (size_t)nc * H * W;
    for (int i = 0; i < H * W; i++) dxi[i] = 0.0;
    for (int o = 0; o < OH * OW; o++) dxi[arg[(size_t)nc * OH * OW + o]] += dy[(size_t)nc * OH * OW + o];
  }
}

void avgpool_forward(const double* x, double* y, int NC, int H, int W, int k, int s) {
  int OH = pool_out(H, k, s), OW = pool_out(W, k, s);
#pragma omp parallel for schedule(static)
  for (int nc = 0; nc < NC; nc++) {
    const double* xi = x + (size_t)nc * H * W;
    for (int oh = 0; oh < OH; oh++)
      for (int ow = 0; ow < OW; ow++) {
        double acc = 0.0;
        int cnt = 0;
        for (int ih = oh * s; ih < oh * s + k && ih < H; ih++)
          for (int iw = ow * s; iw < ow * s + k && iw < W; iw++) { acc += xi[ih * W + iw]; cnt++; }
        y[((size_t)nc * OH + oh) * OW + ow] = acc / cnt;
      }
  }
}

void avgpool_backward(const double* dy, double* dx, int NC, int H, int W, int k, int s) {
  int OH = pool_out(H, k, s), OW = pool_out(W, k, s);
#pragma omp parallel for schedule(static)
  for (int nc = 0; nc < NC; nc++) {
    double* dxi = dx + (size_t)nc * H * W;
    for (int i = 0; i < H * W; i++) dxi[i] = 0.0;
    for (int oh = 0; oh < OH; oh++)
      for (int ow = 0; ow < OW; ow++) {
        int cnt = 0;
        for (int ih = oh * s; ih < oh * s + k && ih < H; ih++)
          for (int iw = ow * s; iw < ow * s + k && iw < W; iw++) cnt++;
        double g = dy[((size_t)nc * OH + oh) * OW + ow] / cnt;
        for (int ih = oh * s; ih < oh * s + k && ih < H; ih++)
          for (int iw = ow * s; iw < ow * s + k && iw < W; iw++) dxi[ih * W + iw] += g;
      }
  }
}

/* ------------------------------------------------------------------ relu, fc, loss */
void relu_forward(const double* x, double* y, size_t n) {
  for (size_t i = 0; i < n; i++) y[i] = x[i] > 0.0 ? x[i] : 0.0;
}
void relu_backward(const double* x, const double* dy, double* dx, size_t n) {
  for (size_t i = 0; i < n; i++) dx[i] = x[i] > 0.0 ? dy[i] : 0.0;
}

void fc_forward(const double* x, const double* w, const double* b, double* y, int N, int In, int Out) {
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; n++)
    for (int o = 0; o < Out; o++) {
      double acc = b[o];
      for (int i = 0; i < In; i++) acc += w[(size_t)o * In + i] * x[(size_t)n * In + i];
      y[(size_t)n * Out + o] = acc;
    }
}

void fc_backward(const double* x, const double* w, const double* dy, double* dx, double* dw, double* db,
                 int N, int In, int Out) {
#pragma omp parallel for schedule(static)
  for (int o = 0; o < Out; o++) {
    double sb = 0.0;
    for (int n = 0; n < N; n++) sb += dy[(size_t)n * Out + o];
    db[o] = sb;
    for (int i = 0; i < In; i++) {
      double acc = 0.0;
      for (int n = 0; n < N; n++) acc += dy[(size_t)n * Out + o] * x[(size_t)n * In + i];
      dw[(size_t)o * In + i] = acc;
    }
  }
  if (!dx) return;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; n++)
    for (int i = 0; i < In; i++) {
      double acc = 0.0;
      for (int o = 0; o < Out; o++) acc += dy[(size_t)n * Out + o] * w[(size_t)o * In + i];
      dx[(size_t)n * In + i] = acc;
    }
}

/* loss = (1/N) sum_n -log softmax(z_n)[y_n];   dz = (softmax(z) - onehot) / N */
double softmax_ce(const double* z, const int* label, double* dz, int N, int K) {
  double loss = 0.0;
  for (int n = 0; n < N; n++) {
    const double* zn = z + (size_t)n * K;
    double m = zn[0];
    for (int j = 1; j < K; j++) if (zn[j] > m) m = zn[j];
    double sum = 0.0;
    for (int j = 0; j < K; j++) sum += exp(zn[j] - m);
    loss += -(zn[label[n]] - m - log(sum));
    for (int j = 0; j < K; j++)
      dz[(size_t)n * K + j] = (exp(zn[j] - m) / sum - (j == label[n] ? 1.0 : 0.0)) / N;
  }
  return loss / N;
}

/* ------------------------------------------------------------------ whole network */
/*
 * calcGradient of one learner: mean-over-mini-batch loss and its gradient.
 *   layers/nlayers : layer table;   C,H,W : input shape;   N : mini-batch size (mu)
 *   theta [P]      : flat parameters;  x [N][C][H][W];  label [N]
 *   grad [P]       : output (may be NULL for a forward-only loss evaluation)
 * Returns the loss, or NaN when P does not match the network.
 */
static double loss_gradient_scores(const olayer* layers, int nlayers, int C, int H, int W, int N,
                                   const double* theta_in, long P, const double* x, const int* label,
                                   double* grad, double* scores, int round_bf16) {
  double* theta = (double*)malloc(sizeof(double) * (size_t)P);
  memcpy(theta, theta_in, sizeof(double) * (size_t)P);
  round_array(theta, (size_t)P, round_bf16);
  /* forward: keep every layer's input */
  double** act = (double**)calloc((size_t)nlayers + 1, sizeof(double*));
  int** argm = (int**)calloc((size_t)nlayers, sizeof(int*));
  int* sc = (int*)malloc(sizeof(int) * ((size_t)nlayers + 1) * 3);
  long* off = (long*)malloc(sizeof(long) * (size_t)nlayers);
  size_t n0 = (size_t)N * C * H * W;
  act[0] = (double*)malloc(sizeof(double) * n0);
  memcpy(act[0], x, sizeof(double) * n0);
  round_array(act[0], n0, round_bf16);
  sc[0] = C; sc[1] = H; sc[2] = W;
  long pos = 0;
  for (int li = 0; li < nlayers; li++) {
    const olayer* L = &layers[li];
    int c = sc[3 * li], h = sc[3 * li + 1], w = sc[3 * li + 2], oc = c, oh = h, ow = w;
    off[li] = pos;
    if (L->type == L_CONV) { oc = L->a; oh = (h + 2 * L->d - L->b) / L->c + 1; ow = (w + 2 * L->d - L->b) / L->c + 1; }
    else if (L->type == L_MAXPOOL || L->type == L_AVGPOOL) { oh = pool_out(h, L->a, L->b); ow = pool_out(w, L->a, L->b); }
    else if (L->type == L_FC) { oc = L->a; oh = 1; ow = 1; }
    size_t no = (size_t)N * oc * oh * ow;
    act[li + 1] = (double*)malloc(sizeof(double) * no);
    switch (L->type) {
      case L_CONV: {
        long nw = (long)oc * c * L->b * L->b;
        if (pos + nw + oc <= P)
          conv_forward(act[li], theta + pos, theta + pos + nw, act[li + 1], N, c, h, w, oc, L->b, L->c, L->d);
        pos += nw + oc;
      } break;
      case L_MAXPOOL:
        argm[li] = (int*)malloc(sizeof(int) * no);
        maxpool_forward(act[li], act[li + 1], argm[li], N * c, h, w, L->a, L->b);
        break;
      case L_AVGPOOL: avgpool_forward(act[li], act[li + 1], N * c, h, w, L->a, L->b); break;
      case L_RELU: relu_forward(act[li], act[li + 1], no); break;
      case L_FC: {
        long nw = (long)oc * c * h * w;
        if (pos + nw + oc <= P)
          fc_forward(act[li], theta + pos, theta + pos + nw, act[li + 1], N, c * h * w, oc);
        pos += nw + oc;
      } break;
    }
    if (li + 1 < nlayers) round_array(act[li + 1], no, round_bf16);   /* the class scores stay unrounded */
    sc[3 * (li + 1)] = oc; sc[3 * (li + 1) + 1] = oh; sc[3 * (li + 1) + 2] = ow;
  }
  double loss = NAN;
  if (pos == P) {
    int K = sc[3 * nlayers] * sc[3 * nlayers + 1] * sc[3 * nlayers + 2];
    double* d = (double*)malloc(sizeof(double) * (size_t)N * K);
    if (scores) memcpy(scores, act[nlayers], sizeof(double) * (size_t)N * K);
    loss = softmax_ce(act[nlayers], label, d, N, K);
    round_array(d, (size_t)N * K, round_bf16);
    /* backward */
    for (int li = nlayers - 1; li >= 0 && grad; li--) {
      const olayer* L = &layers[li];
      int c = sc[3 * li], h = sc[3 * li + 1], w = sc[3 * li + 2];
      int oc = sc[3 * li + 3];
      size_t ni = (size_t)N * c * h * w;
      double* dprev = li > 0 ? (double*)malloc(sizeof(double) * ni) : NULL;
      switch (L->type) {
        case L_CONV: {
          long nw = (long)oc * c * L->b * L->b;
          conv_backward(act[li], theta + off[li], d, dprev, grad + off[li], grad + off[li] + nw, N, c, h, w, oc, L->b, L->c, L->d);
        } break;
        case L_MAXPOOL: if (dprev) maxpool_backward(d, argm[li], dprev, N * c, h, w, L->a, L->b); break;
        case L_AVGPOOL: if (dprev) avgpool_backward(d, dprev, N * c, h, w, L->a, L->b); break;
        case L_RELU: if (dprev) relu_backward(act[li], d, dprev, ni); break;
        case L_FC: {
          long nw = (long)oc * c * h * w;
          fc_backward(act[li], theta + off[li], d, dprev, grad + off[li], grad + off[li] + nw, N, c * h * w, oc);
        } break;
      }
      free(d);
      d = dprev;
      if (d) round_array(d, ni, round_bf16);
    }
    free(d);
  }
  for (int li = 0; li <= nlayers; li++) free(act[li]);
  for (int li = 0; li < nlayers; li++) free(argm[li]);
  free(act); free(argm); free(sc); free(off); free(theta);
  return loss;
}

double cnn_loss_and_gradient(const olayer* layers, int nlayers, int C, int H, int W, int N,
                             const double* theta_in, long P, const double* x, const int* label,
                             double* grad, int round_bf16) {
  return loss_gradient_scores(layers, nlayers, C, H, W, N, theta_in, P, x, label, grad, NULL, round_bf16);
}

/*
 * Evaluation pass (the test / validation error of Section 4.3): forward only.
 *   scores [N][K] : output of the last layer (K classes), the input of the softmax
 * Returns the mean loss, or NaN when P does not match the network.
 */
double cnn_class_scores(const olayer* layers, int nlayers, int C, int H, int W, int N,
                        const double* theta_in, long P, const double* x, const int* label,
                        double* scores, int round_bf16) {
  return loss_gradient_scores(layers, nlayers, C, H, W, N, theta_in, P, x, label, NULL, scores, round_bf16);
}

/*
 * Diagnostic for the fp32 parity tests, not part of the method: how close to zero does any ReLU input of this case
 * lie, relative to the size of the terms it is summed from?  A ReLU input v = b + sum_k w_k x_k whose magnitude is
 * below the rounding error of its own sum (about 1e-7 sum_k |w_k x_k| in float) has no defined sign: two correct fp32
 * evaluations that add in different orders may disagree on it, and one flipped ReLU changes the gradient by a whole
 * term.  The tests ask for this number and take only cases in which every ReLU input is decided.
 * Exact mode only.  Returns min over all ReLU inputs with a non-zero term sum of |v| / (|b| + sum_k |w_k x_k|), where
 * the sum is that of the convolution or fully connected layer in front of the ReLU (a max pool in between passes the
 * winner's sum on, an average pool the average of its window's sums); 1.0 if the network has no ReLU; NaN when P does
 * not match.
 */
double cnn_min_relu_margin(const olayer* layers, int nlayers, int C, int H, int W, int N,
                           const double* theta, long P, const double* x) {
  size_t n0 = (size_t)N * C * H * W;
  double* act = (double*)malloc(sizeof(double) * n0);
  double* mag = (double*)malloc(sizeof(double) * n0);
  memcpy(act, x, sizeof(double) * n0);
  for (size_t i = 0; i < n0; i++) mag[i] = fabs(x[i]);
  int c = C, h = H, w = W;
  long pos = 0;
  double worst = 1.0;
  for (int li = 0; li < nlayers; li++) {
    const olayer* L = &layers[li];
    int oc = c, oh = h, ow = w;
    if (L->type == L_CONV) { oc = L->a; oh = (h + 2 * L->d - L->b) / L->c + 1; ow = (w + 2 * L->d - L->b) / L->c + 1; }
    else if (L->type == L_MAXPOOL || L->type == L_AVGPOOL) { oh = pool_out(h, L->a, L->b); ow = pool_out(w, L->a, L->b); }
    else if (L->type == L_FC) { oc = L->a; oh = 1; ow = 1; }
    size_t no = (size_t)N * oc * oh * ow, ni = (size_t)N * c * h * w;
    double* out = (double*)malloc(sizeof(double) * no);
    double* mout = (double*)malloc(sizeof(double) * no);
    if (L->type == L_CONV || L->type == L_FC) {
      long nw = L->type == L_CONV ? (long)oc * c * L->b * L->b : (long)oc * c * h * w;
      if (pos + nw + oc > P) { free(out); free(mout); free(act); free(mag); return NAN; }
      double* aw = (double*)malloc(sizeof(double) * (size_t)(nw + oc));
      double* ax = (double*)malloc(sizeof(double) * ni);
      for (long i = 0; i < nw + oc; i++) aw[i] = fabs(theta[pos + i]);
      for (size_t i = 0; i < ni; i++) ax[i] = fabs(act[i]);
      if (L->type == L_CONV) {
        conv_forward(act, theta + pos, theta + pos + nw, out, N, c, h, w, oc, L->b, L->c, L->d);
        conv_forward(ax, aw, aw + nw, mout, N, c, h, w, oc, L->b, L->c, L->d);
      } else {
        fc_forward(act, theta + pos, theta + pos + nw, out, N, c * h * w, oc);
        fc_forward(ax, aw, aw + nw, mout, N, c * h * w, oc);
      }
      free(aw); free(ax);
      pos += nw + oc;
    } else if (L->type == L_MAXPOOL) {
      int* arg = (int*)malloc(sizeof(int) * no);
      maxpool_forward(act, out, arg, N * c, h, w, L->a, L->b);
      for (size_t o = 0; o < no; o++) mout[o] = mag[(o / ((size_t)oh * ow)) * h * w + arg[o]];
      free(arg);
    } else if (L->type == L_AVGPOOL) {
      avgpool_forward(act, out, N * c, h, w, L->a, L->b);
      avgpool_forward(mag, mout, N * c, h, w, L->a, L->b);
    } else {   /* L_RELU */
      for (size_t i = 0; i < ni; i++) {
        if (mag[i] > 0.0) { double m = fabs(act[i]) / mag[i]; if (m < worst) worst = m; }
        out[i] = act[i] > 0.0 ? act[i] : 0.0;
        mout[i] = out[i];
      }
    }
    free(act); free(mag);
    act = out; mag = mout;
    c = oc; h = oh; w = ow;
  }
  free(act); free(mag);
  return pos == P ? worst : NAN;
}

/* number of parameters of a layer table (for the parameter-count pins) */
long cnn_num_params(const olayer* layers, int nlayers, int C, int H, int W) {
  long pos = 0;
  int c = C, h = H, w = W;
  for (int li = 0; li < nlayers; li++) {
    const olayer* L = &layers[li];
    if (L->type == L_CONV) { pos += (long)L->a * c * L->b * L->b + L->a; h = (h + 2 * L->d - L->b) / L->c + 1; w = (w + 2 * L->d - L->b) / L->c + 1; c = L->a; }
    else if (L->type == L_MAXPOOL || L->type == L_AVGPOOL) { h = pool_out(h, L->a, L->b); w = pool_out(w, L->a, L->b); }
    else if (L->type == L_FC) { pos += (long)L->a * c * h * w + L->a; c = L->a; h = 1; w = 1; }
  }
  return pos;
}
