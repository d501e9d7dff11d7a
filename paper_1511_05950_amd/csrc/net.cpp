// Network plan and executor of calcGradient (Section 2.1): the layer list is turned into a list of
// device operations with fixed offsets into one per-learner workspace; a calcGradient call walks the list
// forward and backward, every launch covering all listed learners at once.  ReLU layers are fused into the
// operation that produces their input (its output is stored after the ReLU; the backward mask is applied
// by whichever kernel produces the gradient of that tensor).
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <vector>

#include "kernels.hpp"

namespace sasgd {

enum OpKind { OP_CONV, OP_POOL_MAX, OP_POOL_AVG, OP_FLATTEN };

struct Op {
  OpKind kind;
  bool relu = false;           // output stored after ReLU
  bool is_fc = false;
  bool out_f32 = false;        // output kept in fp32 (class scores)
  ConvShape cs{};              // OP_CONV
  PoolShape ps{};              // pools; OP_FLATTEN uses N,C,H,W
  int64_t w_off = 0, b_off = 0;
  int in_t = 0, out_t = 0;     // tensor indices
  size_t arg_off = 0;          // byte offset of the max-pool argmax, from the workspace base
  // bf16 MFMA path (conv / fc ops that qualify)
  bool mfma = false;
  VConv vc{};
  IGemm gf{};                  // forward implicit GEMM
  IGemm gd{};                  // input-gradient implicit GEMM
  bool dgrad_bt = false;       // fc: B operand is the flat weight matrix read transposed
  int64_t pack_fwd = -1, pack_bwd = -1;   // element offsets in the packed-filter region of a version slot
  int Kp = 0, Kpt = 0;
  // fully connected layer whose weight gradient is kept as the factors x^T [in][NP] and dy^T [out][NP]
  bool factored = false;
  size_t fx_off = 0, fdy_off = 0;         // element offsets of the two factor copies in the workspace
  int NP = 0;
  // fully connected layer that learners on one weight version run as ONE product on their stacked mini-batches:
  // element offset of the stacked layer input in the group staging area
  bool stacked = false;
  size_t gx_off = 0;
  // fully connected layer on the grouped kernels (small mini-batches): learners of one weight version share every read
  // of its weights without any copy; takes precedence over `stacked`
  bool grouped = false;
};

struct Tensor {
  size_t off = 0;              // element offset in the workspace
  size_t elems = 0;
  bool relu = false;           // values are post-ReLU (a gradient flowing into it must be masked)
};

struct Net {
  int mu = 0;
  bool bf16 = false;
  int classes = 0;
  bool scores_f32 = false;
  int64_t P = 0;
  std::vector<Op> ops;
  std::vector<Tensor> tensors; // tensor 0 = re-laid-out input
  int inC = 0, inH = 0, inW = 0;
  InPack inpack{};
  size_t Ppad = 0;             // start of the packed-filter region inside a version slot (elements)
  PackTable pack{};            // filter repacking jobs of one weight version
  size_t pack_elems = 0;
  size_t grad_a = 0, grad_b = 0, grad_elems = 0;   // two gradient-activation buffers (element offsets)
  size_t ws_bytes = 0;
  size_t loss_off = 0;         // per-image losses, mu floats (byte offset)
  size_t zero_off = 0;         // 256 zero bytes (element offset), target of out-of-range loads
  size_t scratch_off = 0, scratch_bytes = 0;   // split-contraction partials (bytes from the workspace base)
  // group staging area (one per context): a block of zeros, the stacked input of every stacked layer (kept for the
  // backward pass), stacked output / output gradient / input gradient, split partials.  Element offsets of bf16.
  int lambda = 0;
  void* group_ws = nullptr;
  size_t g_bytes = 0, g_zero_off = 0, g_y_off = 0, g_dy_off = 0, g_dx_off = 0, g_scratch_off = 0, g_scratch_bytes = 0;
  void* ws[kMaxLearners] = {nullptr};
  const float* pixel_mean = nullptr;   // optional [C][H][W] fp32, subtracted while the input is re-laid out
};

static int pool_out_size(int n, int k, int s) {
  int o = (n - k + s - 1) / s + 1;
  if ((o - 1) * s >= n) o--;
  return o < 1 ? 1 : o;
}

static const sasgd_layer kCifar3[] = {
    {SASGD_CONV, 32, 5, 1, 2}, {SASGD_MAXPOOL, 0, 3, 2, 0}, {SASGD_RELU, 0, 0, 0, 0},
    {SASGD_CONV, 32, 5, 1, 2}, {SASGD_RELU, 0, 0, 0, 0},    {SASGD_AVGPOOL, 0, 3, 2, 0},
    {SASGD_CONV, 64, 5, 1, 2}, {SASGD_RELU, 0, 0, 0, 0},    {SASGD_AVGPOOL, 0, 3, 2, 0},
    {SASGD_FC, 10, 0, 0, 0}};

static const sasgd_layer kAlex8[] = {
    {SASGD_CONV, 96, 11, 4, 0}, {SASGD_RELU, 0, 0, 0, 0}, {SASGD_MAXPOOL, 0, 3, 2, 0},
    {SASGD_CONV, 256, 5, 1, 2}, {SASGD_RELU, 0, 0, 0, 0}, {SASGD_MAXPOOL, 0, 3, 2, 0},
    {SASGD_CONV, 384, 3, 1, 1}, {SASGD_RELU, 0, 0, 0, 0},
    {SASGD_CONV, 384, 3, 1, 1}, {SASGD_RELU, 0, 0, 0, 0},
    {SASGD_CONV, 256, 3, 1, 1}, {SASGD_RELU, 0, 0, 0, 0}, {SASGD_MAXPOOL, 0, 3, 2, 0},
    {SASGD_FC, 4096, 0, 0, 0},  {SASGD_RELU, 0, 0, 0, 0},
    {SASGD_FC, 4096, 0, 0, 0},  {SASGD_RELU, 0, 0, 0, 0},
    {SASGD_FC, 1000, 0, 0, 0}};

int net_create(const sasgd_config& cfg, Net** out, int64_t* out_P, size_t* out_pack_elems, std::string& err) {
  const sasgd_layer* layers = nullptr;
  int nl = 0, C = 0, H = 0, W = 0;
  if (cfg.net == SASGD_NET_CIFAR3) {
    layers = kCifar3; nl = (int)(sizeof(kCifar3) / sizeof(kCifar3[0])); C = 3; H = 32; W = 32;
  } else if (cfg.net == SASGD_NET_ALEX8) {
    layers = kAlex8; nl = (int)(sizeof(kAlex8) / sizeof(kAlex8[0])); C = 3; H = 224; W = 224;
  } else if (cfg.net == SASGD_NET_CUSTOM) {
    layers = cfg.layers; nl = cfg.num_layers; C = cfg.in_channels; H = cfg.in_height; W = cfg.in_width;
    if (!layers || nl < 1 || nl > 256 || C < 1 || H < 1 || W < 1) { err = "custom network: bad layer table or input shape"; return SASGD_EINVAL; }
  } else {
    err = "unknown network"; return SASGD_EINVAL;
  }
  if (cfg.mu < 1 || cfg.mu > 4096) { err = "mu out of range (1..4096)"; return SASGD_EINVAL; }

  Net* net = new Net();
  net->mu = cfg.mu;
  net->bf16 = cfg.compute == SASGD_BF16;
  net->inC = C; net->inH = H; net->inW = W;
  const int N = cfg.mu;
  size_t cursor = 0;       // elements of T
  auto new_tensor = [&](size_t elems) {
    Tensor t;
    t.off = cursor;
    t.elems = elems;
    cursor += (elems + 63) & ~(size_t)63;
    net->tensors.push_back(t);
    return (int)net->tensors.size() - 1;
  };
  // The MFMA kernels gather 16-byte chunks of `chunk` channels (8 bf16 or 4 fp32).  The first convolution runs on
  // the MFMA path when it can: its input is channel-padded to a multiple of the chunk (stride 1) or
  // space-to-depth transformed (stride s, no padding).
  const int chunk = net->bf16 ? 8 : 4;
  int n_factored = 0;
  auto round_chunk = [&](int x) { return (x + chunk - 1) / chunk * chunk; };
  net->inpack = InPack{C, H, W, C, H, W, 1};
  bool first_mfma = false;
  if (layers[0].kind == SASGD_CONV && layers[0].units % chunk == 0 && layers[0].window >= 1 && layers[0].stride >= 1) {
    const sasgd_layer& L0 = layers[0];
    if (L0.stride == 1) {
      net->inpack.Cp = round_chunk(C);
      first_mfma = true;
    } else if (L0.pad == 0 && L0.window <= H && L0.window <= W) {
      const int sd = L0.stride;
      net->inpack = InPack{C, H, W, round_chunk(sd * sd * C), (H + sd - 1) / sd, (W + sd - 1) / sd, sd};
      first_mfma = true;
    }
  }
  int cur = new_tensor((size_t)N * net->inpack.Cp * net->inpack.Hp * net->inpack.Wp);
  bool flat = false;       // current tensor already in (C,H,W)-flattened order (after a flatten or an fc)
  size_t pack_cursor = 0;
  auto round32 = [](int x) { return (x + 31) & ~31; };
  int64_t P = 0;
  size_t arg_bytes = 0;
  for (int li = 0; li < nl; li++) {
    const sasgd_layer& L = layers[li];
    if (L.kind == SASGD_RELU) {
      if (net->ops.empty() || net->tensors[(size_t)cur].relu) { delete net; err = "relu must directly follow a conv, fc or pooling layer"; return SASGD_EINVAL; }
      net->ops.back().relu = true;
      net->tensors[(size_t)cur].relu = true;
      continue;
    }
    Op op;
    if (L.kind == SASGD_CONV) {
      if (flat || L.units < 1 || L.window < 1 || L.stride < 1 || L.pad < 0 || L.pad >= L.window || H + 2 * L.pad < L.window || W + 2 * L.pad < L.window) {
        delete net; err = "conv layer: bad shape"; return SASGD_EINVAL;
      }
      op.kind = OP_CONV;
      op.cs = ConvShape{N, C, H, W, L.units, (H + 2 * L.pad - L.window) / L.stride + 1, (W + 2 * L.pad - L.window) / L.stride + 1, L.window, L.stride, L.pad};
      op.w_off = P;
      P += (int64_t)L.units * C * L.window * L.window;
      op.b_off = P;
      P += L.units;
      op.in_t = cur;
      if (cur == 0 && first_mfma) {
        const InPack& ip = net->inpack;
        const int kse = (L.window + ip.s2d - 1) / ip.s2d;
        op.mfma = true;
        op.vc = VConv{ip.Cp, kse, L.units, ip.s2d, C, L.window};
        op.gf = IGemm{0, 0, N * op.cs.OH * op.cs.OW, L.units, ip.Hp, ip.Wp, ip.Cp, op.cs.OH, op.cs.OW, kse, ip.s2d == 1 ? L.pad : 0,
                      kse * kse * ip.Cp / chunk, ip.Cp / chunk, 0};
        if (net->bf16) {
          op.Kp = round32(kse * kse * ip.Cp);
          op.pack_fwd = (int64_t)pack_cursor;
          pack_cursor += (size_t)round32(L.units) * op.Kp;
        }
      } else if (cur != 0 && L.stride == 1 && C % chunk == 0 && L.units % chunk == 0) {
        op.mfma = true;
        op.vc = VConv{C, L.window, L.units, 1, C, L.window};
        op.gf = IGemm{0, 0, N * op.cs.OH * op.cs.OW, L.units, H, W, C, op.cs.OH, op.cs.OW, L.window, L.pad,
                      L.window * L.window * C / chunk, C / chunk, 0};
        op.gd = IGemm{0, 0, N * H * W, C, op.cs.OH, op.cs.OW, L.units, H, W, L.window, L.window - 1 - L.pad,
                      L.window * L.window * L.units / chunk, L.units / chunk, 0};
        if (net->bf16) {
          op.Kp = round32(L.window * L.window * C);
          op.Kpt = round32(L.window * L.window * L.units);
          op.pack_fwd = (int64_t)pack_cursor;
          pack_cursor += (size_t)round32(L.units) * op.Kp;
          op.pack_bwd = (int64_t)pack_cursor;
          pack_cursor += (size_t)round32(C) * op.Kpt;
        }
      }
      C = L.units; H = op.cs.OH; W = op.cs.OW;
      cur = op.out_t = new_tensor((size_t)N * C * H * W);
    } else if (L.kind == SASGD_MAXPOOL || L.kind == SASGD_AVGPOOL) {
      if (flat || L.window < 1 || L.window > 15 || L.stride < 1 || L.window > H || L.window > W) { delete net; err = "pooling layer: bad shape"; return SASGD_EINVAL; }
      op.kind = L.kind == SASGD_MAXPOOL ? OP_POOL_MAX : OP_POOL_AVG;
      op.ps = PoolShape{N, C, H, W, pool_out_size(H, L.window, L.stride), pool_out_size(W, L.window, L.stride), L.window, L.stride};
      op.in_t = cur;
      H = op.ps.OH; W = op.ps.OW;
      cur = op.out_t = new_tensor((size_t)N * C * H * W);
      if (op.kind == OP_POOL_MAX) { op.arg_off = arg_bytes; arg_bytes += ((size_t)N * C * H * W + 255) & ~(size_t)255; }
    } else if (L.kind == SASGD_FC) {
      if (L.units < 1) { delete net; err = "fc layer: bad shape"; return SASGD_EINVAL; }
      if (!flat && H * W > 1) {           // bring the tensor into the (C,H,W) order of the fc weights
        Op fl;
        fl.kind = OP_FLATTEN;
        fl.ps = PoolShape{N, C, H, W, 0, 0, 0, 0};
        fl.in_t = cur;
        cur = fl.out_t = new_tensor((size_t)N * C * H * W);
        net->ops.push_back(fl);
      }
      const int in = C * H * W;
      op.kind = OP_CONV;
      op.is_fc = true;
      op.cs = ConvShape{N, in, 1, 1, L.units, 1, 1, 1, 1, 0};
      op.w_off = P;
      P += (int64_t)L.units * in;
      op.b_off = P;
      P += L.units;
      op.in_t = cur;
      if (cur != 0 && in % chunk == 0 && L.units % chunk == 0 && (!net->bf16 || op.w_off % 8 == 0)) {
        // fully connected: the flat weight matrix [out][in] is the B operand as it lies (forward), and is read
        // transposed for the input gradient; no packed copy
        op.mfma = true;
        op.dgrad_bt = true;
        op.vc = VConv{in, 1, L.units, 1, in, 1};
        op.gf = IGemm{0, op.w_off, N, L.units, 1, 1, in, 1, 1, 1, 0, in / chunk, in / chunk, in};
        op.gd = IGemm{0, op.w_off, N, in, 1, 1, L.units, 1, 1, 1, 0, L.units / chunk, L.units / chunk, in};
        op.grouped = net->bf16 && fc_group_layer_ok(N, in, L.units);
        // rank-N weight gradient kept as factors: worth it while the N FMAs per weight and pending gradient stay far
        // below what the update's streaming rate leaves room for
        const int c_upd = cfg.lambda / cfg.n;
        if (net->bf16 && !(cfg.flags & SASGD_FLAG_FLAT_FC_GRADIENT) && N <= 32 && (int64_t)c_upd * N <= 1024 && op.w_off % 4 == 0 &&
            L.units % 4 == 0 && in % 8 == 0 && n_factored < kMaxFactoredLayers) {
          op.factored = true;
          op.NP = (N + 7) & ~7;
          n_factored++;
        }
      }
      C = L.units; H = 1; W = 1;
      flat = true;
      cur = op.out_t = new_tensor((size_t)N * C);
    } else {
      delete net; err = "unknown layer kind"; return SASGD_EINVAL;
    }
    net->ops.push_back(op);
  }
  if (P < 1) { delete net; err = "network has no parameters"; return SASGD_EINVAL; }
  if (net->tensors[(size_t)cur].relu) { delete net; err = "the class scores must not pass through a relu"; return SASGD_EINVAL; }
  net->classes = C * H * W;
  if (net->classes < 2) { delete net; err = "network output must have at least two classes"; return SASGD_EINVAL; }
  if (!flat && H * W > 1) {               // scores must be one vector per image in class order
    Op fl;
    fl.kind = OP_FLATTEN;
    fl.ps = PoolShape{N, C, H, W, 0, 0, 0, 0};
    fl.in_t = cur;
    cur = fl.out_t = new_tensor((size_t)N * C * H * W);
    net->ops.push_back(fl);
  }
  if (net->ops.back().kind == OP_CONV) {   // class scores produced by a conv / fc: keep them in fp32
    net->ops.back().out_f32 = true;
    net->scores_f32 = true;
    if (net->bf16) { new_tensor(net->tensors[(size_t)cur].elems); }   // room for the wider elements (tensor is last in the arena)
  }
  for (Op& op : net->ops) {
    if (!op.factored) continue;
    op.fx_off = net->tensors[(size_t)new_tensor((size_t)op.cs.C * op.NP)].off;
    op.fdy_off = net->tensors[(size_t)new_tensor((size_t)op.cs.K * op.NP)].off;
  }
  net->P = P;
  net->Ppad = ((size_t)P + 63) & ~(size_t)63;
  net->pack_elems = pack_cursor;
  for (Op& op : net->ops) {
    if (!op.mfma) continue;
    op.gf.zero_off = op.gd.zero_off = 0;   // filled below, once the arena is laid out
    const Tensor& ti = net->tensors[(size_t)op.in_t];
    op.gf.a_off = ti.off;
    if (!op.dgrad_bt && net->bf16) {
      op.gf.b_off = (int64_t)(net->Ppad + (size_t)op.pack_fwd);
      op.gf.ldb = op.Kp;
      if (op.pack_bwd >= 0) { op.gd.b_off = (int64_t)(net->Ppad + (size_t)op.pack_bwd); op.gd.ldb = op.Kpt; }
    }
    igemm_set_magics(op.gf, net->bf16 ? 2 : 4);
    igemm_set_magics(op.gd, net->bf16 ? 2 : 4);
    if (!net->bf16)   // the fp32 kernels read the flat filter itself: its byte size bounds their loads
      op.gf.b_bytes = op.gd.b_bytes = (uint32_t)((int64_t)op.vc.K * op.vc.Creal * op.vc.ksr * op.vc.ksr * 4);
  }
  size_t maxe = 0;
  for (const Tensor& t : net->tensors) maxe = t.elems > maxe ? t.elems : maxe;
  // the kernels address an activation tensor through 32-bit byte offsets with the top bit reserved for "out of range"
  if (maxe * 4 >= ((size_t)1 << 31)) { delete net; err = "an activation tensor of mu images exceeds 2 GiB: lower mu"; return SASGD_ERANGE; }
  net->grad_elems = (maxe + 63) & ~(size_t)63;
  net->grad_a = cursor;
  net->grad_b = cursor + net->grad_elems;
  cursor += 2 * net->grad_elems;
  net->zero_off = cursor;
  cursor += 256;
  for (Op& op : net->ops) op.gf.zero_off = op.gd.zero_off = net->zero_off;
  for (const Op& op : net->ops) {
    if (!op.mfma || op.pack_fwd < 0) continue;
    if (net->pack.count == kMaxPackJobs) { delete net; err = "too many convolution layers for the MFMA path"; return SASGD_EINVAL; }
    PackJob& jb = net->pack.job[net->pack.count++];
    jb.v = op.vc;
    jb.w_off = op.w_off;
    jb.fwd_off = op.pack_fwd;
    jb.bwd_off = op.pack_bwd < 0 ? 0 : op.pack_bwd;
    jb.Kp = op.Kp;
    jb.Kpt = op.pack_bwd < 0 ? 0 : op.Kpt;
    jb.start = net->pack.total;
    net->pack.total += (int64_t)((op.vc.K + 31) & ~31) * op.Kp + (op.pack_bwd < 0 ? 0 : (int64_t)((op.vc.C + 31) & ~31) * op.Kpt);
  }
  const size_t esz = net->bf16 ? 2 : 4;
  size_t bytes = (cursor * esz + 255) & ~(size_t)255;
  for (Op& op : net->ops) op.arg_off += bytes;
  bytes += arg_bytes;
  net->loss_off = bytes;
  bytes += ((size_t)N * 4 + 255) & ~(size_t)255;
  // scratch for split contractions: room for 8 partial copies of the largest output, within 16..128 MiB
  size_t need = 0;
  const int cw = net->bf16 ? 8 : 4;                // channels per im2col chunk
  for (const Op& op : net->ops) {
    if (!op.mfma) continue;
    size_t fwd = (size_t)op.gf.M * op.gf.Ncols * 4, wg = (size_t)op.gf.Ncols * (op.gf.Kchunks * cw + cw) * 4;
    size_t dg = (size_t)op.gd.M * op.gd.Ncols * 4;
    need = fwd > need ? fwd : need;
    need = wg > need ? wg : need;
    need = dg > need ? dg : need;
  }
  if (need > 0) {
    size_t sb = need * 8;
    if (sb > ((size_t)128 << 20)) sb = need > ((size_t)128 << 20) ? need : ((size_t)128 << 20);
    net->scratch_off = (bytes + 255) & ~(size_t)255;
    net->scratch_bytes = sb;
    bytes = net->scratch_off + sb;
  }
  net->ws_bytes = bytes + 256;
  // group staging area
  net->lambda = cfg.lambda;
  if (net->bf16 && cfg.lambda > 1) {
    const size_t R = (size_t)cfg.lambda * N;
    size_t g = 256, max_in = 0, max_out = 0;
    net->g_zero_off = 0;
    for (Op& op : net->ops) {
      if (!(op.is_fc && op.mfma) || op.grouped) continue;
      const size_t in = (size_t)op.cs.C, outn = (size_t)op.cs.K;
      if ((N * in * 2) % 16 || (N * outn * (op.out_f32 ? 4 : 2)) % 16 || R * std::max(in, outn) * 4 >= ((size_t)1 << 31)) continue;
      op.stacked = true;
      op.gx_off = g;
      g += (R * in + 63) & ~(size_t)63;
      max_in = std::max(max_in, in);
      max_out = std::max(max_out, outn);
    }
    if (max_in > 0) {
      net->g_y_off = g;  g += (2 * R * max_out + 63) & ~(size_t)63;     // room for fp32 class scores
      net->g_dy_off = g; g += (R * max_out + 63) & ~(size_t)63;
      net->g_dx_off = g; g += (R * max_in + 63) & ~(size_t)63;
      net->g_scratch_off = (g * 2 + 255) & ~(size_t)255;
      net->g_scratch_bytes = std::min((size_t)128 << 20, 8 * R * std::max(max_in, max_out) * 4);
      net->g_bytes = net->g_scratch_off + net->g_scratch_bytes + 256;
    }
  }
  *out = net;
  *out_P = P;
  *out_pack_elems = net->pack_elems;
  return SASGD_OK;
}

void net_destroy(Net* net) { delete net; }
size_t net_group_workspace_bytes(const Net* net) { return net->g_bytes; }
hipError_t net_set_group_workspace(Net* net, void* ws, hipStream_t stream) {
  net->group_ws = ws;
  return hipMemsetAsync(ws, 0, net->g_bytes, stream);   // the kernels rely on its block of zeros
}
size_t net_workspace_bytes(const Net* net) { return net->ws_bytes; }
hipError_t net_set_workspace(Net* net, int learner, void* ws, hipStream_t stream) {
  net->ws[learner] = ws;
  hipError_t e = hipMemsetAsync(ws, 0, net->ws_bytes, stream);
  if (e != hipSuccess) return e;
  // second half of the constant block: one 16-byte chunk holding 1.0 followed by zeros (the im2col "bias column")
  static const uint16_t one_bf16 = 0x3F80;
  static const float one_f32 = 1.0f;
  if (net->bf16) return hipMemcpyAsync((char*)ws + (net->zero_off + 128) * 2, &one_bf16, 2, hipMemcpyHostToDevice, stream);
  return hipMemcpyAsync((char*)ws + (net->zero_off + 128) * 4, &one_f32, 4, hipMemcpyHostToDevice, stream);
}

#define TRY(x) do { hipError_t e__ = (x); if (e__ != hipSuccess) return e__; } while (0)

// Derive the packed bf16 filters of every MFMA convolution from the flat bf16 copy of one weight version.
hipError_t net_prepare_versions(Net* net, const void* const* flat, void* const* packed, int versions, hipStream_t stream) {
  if (net->pack.count == 0) return hipSuccess;
  for (int v0 = 0; v0 < versions; v0 += kMaxPackVersions) {
    PackVersions pv;
    memset(&pv, 0, sizeof(pv));
    const int nv = std::min(kMaxPackVersions, versions - v0);
    for (int k = 0; k < nv; k++) { pv.flat[k] = flat[v0 + k]; pv.packed[k] = packed[v0 + k]; }
    TRY(launch_pack_filters(pv, nv, net->pack, stream));
  }
  return hipSuccess;
}
hipError_t net_prepare_version(Net* net, const void* flat, void* packed, hipStream_t stream) {
  return net_prepare_versions(net, &flat, &packed, 1, stream);
}

// fp32 MFMA path: 128 x 32 tiles, contraction steps of 16 (four 4-channel chunks)
static void set_splits_f32(const Net* net, IGemm& g, int count) {
  const int64_t tiles = (int64_t)((g.M + 127) / 128) * ((g.Ncols + 31) / 32);
  g.scratch_off = net->scratch_off;
  g.splits = choose_splits(tiles, count, (g.Kchunks + 3) / 4, (size_t)g.M * g.Ncols * 4, net->scratch_bytes);
}

static void set_splits(const Net* net, IGemm& g, int steps, int count) {
  const int bm = g.M <= 32 ? 32 : 128, bn = g.M <= 32 ? 128 : (g.Ncols <= 32 ? 32 : (g.Ncols <= 64 ? 64 : (g.Ncols % 256 == 0 ? 256 : 128)));
  const int64_t tiles = (int64_t)((g.M + bm - 1) / bm) * ((g.Ncols + bn - 1) / bn);
  g.scratch_off = net->scratch_off;
  g.splits = choose_splits(tiles, count, steps, (size_t)g.M * g.Ncols * 4, net->scratch_bytes);
}

int net_factored_layers(const Net* net, FactoredLayer* out, int max) {
  int k = 0;
  for (const Op& op : net->ops) {
    if (!op.factored) continue;
    if (k < max) out[k] = FactoredLayer{op.w_off, op.cs.C, op.cs.K, op.cs.N, op.NP, op.fx_off, op.fdy_off};
    k++;
  }
  return k;
}

void net_set_pixel_mean(Net* net, const float* mean_dev) { net->pixel_mean = mean_dev; }
void net_input_shape(const Net* net, int* C, int* H, int* W) { *C = net->inC; *H = net->inH; *W = net->inW; }

// Forward pass, loss and (unless out_rank_dev is given, which makes this an evaluation pass) backward pass.
hipError_t net_calc_gradient(Net* net, const int* learners, const LearnerBind* binds, int count, float* out_loss_dev,
                             int32_t* out_rank_dev, hipStream_t stream) {
  PtrTab ws, grads;
  CPtrTab wts, imgs, labs;
  memset(&ws, 0, sizeof(ws)); memset(&grads, 0, sizeof(grads));
  memset(&wts, 0, sizeof(wts)); memset(&imgs, 0, sizeof(imgs)); memset(&labs, 0, sizeof(labs));
  for (int k = 0; k < count; k++) {
    ws.p[k] = net->ws[learners[k]];
    grads.p[k] = binds[k].grad;
    wts.p[k] = binds[k].weights;
    imgs.p[k] = binds[k].images;
    labs.p[k] = binds[k].labels;
  }
  const bool bf = net->bf16;
  const std::vector<Tensor>& T = net->tensors;
  // Learners that read the same weight version: the stacked fully connected layers take each such group (two members
  // and more) as one matrix product; `single` lists the others.  Groups lie one after the other in the staging area.
  struct Group { int first_row_block; std::vector<int> idx; };
  std::vector<Group> groups;
  std::vector<int> single;
  if (net->group_ws && count > 1) {
    std::vector<char> taken((size_t)count, 0);
    int blocks = 0;
    for (int a = 0; a < count; a++) {
      if (taken[(size_t)a]) continue;
      Group g;
      g.first_row_block = blocks;
      for (int b2 = a; b2 < count; b2++)
        if (!taken[(size_t)b2] && wts.p[b2] == wts.p[a]) { g.idx.push_back(b2); taken[(size_t)b2] = 1; }
      if (g.idx.size() >= 2) { blocks += (int)g.idx.size(); groups.push_back(g); }
      else single.push_back(a);
    }
  }
  // The grouped fully connected kernels take every learner of the call, those of one weight version next to each
  // other: `wsG` / `wtsG` list the learners in that order, `gtab` cuts the list into groups of at most 128 image rows;
  // the learners of a version that has more are dealt out evenly (18 learners of 16 images: three groups of six).
  // (Measured against that: kernels that take up to 512 rows in one group, the row blocks dealt out to the wavefronts --
  // every 32-unit workgroup then walks an input tensor larger than an L2, and the fully connected launches of 18 learners
  // on one version took 438 us against 369 us.)
  PtrTab wsG;
  CPtrTab wtsG;
  GroupTab gtab;
  int ngroups = 0;
  bool any_grouped = false;
  for (const Op& op : net->ops) any_grouped = any_grouped || op.grouped;
  if (any_grouped) {
    memset(&wsG, 0, sizeof(wsG)); memset(&wtsG, 0, sizeof(wtsG)); memset(&gtab, 0, sizeof(gtab));
    const int cap = std::max(1, kMaxGroupRows / net->mu);
    std::vector<char> taken((size_t)count, 0);
    int pos = 0;
    for (int a = 0; a < count; a++) {
      if (taken[(size_t)a]) continue;
      std::vector<int> same;
      for (int b2 = a; b2 < count; b2++)
        if (!taken[(size_t)b2] && wts.p[b2] == wts.p[a]) { same.push_back(b2); taken[(size_t)b2] = 1; }
      const int n = (int)same.size(), chunks = (n + cap - 1) / cap;
      for (int ch = 0, at = 0; ch < chunks; ch++) {
        const int len = (n - at + (chunks - ch) - 1) / (chunks - ch);     // the remaining learners, evenly
        gtab.first[ngroups] = (uint8_t)pos;
        gtab.members[ngroups] = (uint8_t)len;
        ngroups++;
        for (int k = 0; k < len; k++, at++, pos++) {
          wsG.p[pos] = ws.p[same[(size_t)at]];
          wtsG.p[pos] = wts.p[same[(size_t)at]];
        }
      }
    }
  }
  PtrTab ws1, grads1;
  CPtrTab wts1;
  memset(&ws1, 0, sizeof(ws1)); memset(&grads1, 0, sizeof(grads1)); memset(&wts1, 0, sizeof(wts1));
  for (size_t k = 0; k < single.size(); k++) {
    ws1.p[k] = ws.p[single[k]]; grads1.p[k] = grads.p[single[k]]; wts1.p[k] = wts.p[single[k]];
  }
  const int count1 = (int)single.size();
  // One stacked fully connected product of a group: rows from every member's workspace (element offset src_off, `width`
  // values per image) are stacked at stage_in, the product runs on the staging area against the group's weights, and
  // the result rows (out_width values of out_esz bytes per image, at stage_out) go back to dst_off of every member.
  auto stacked_product = [&](const Group& G, IGemm g, Epilogue ep, bool bt, size_t src_off, size_t stage_in, int width, size_t dst_off,
                             size_t stage_out, int out_width, int out_esz) -> hipError_t {
    PtrTab mem, gws;
    CPtrTab gwt;
    memset(&mem, 0, sizeof(mem)); memset(&gws, 0, sizeof(gws)); memset(&gwt, 0, sizeof(gwt));
    const int k = (int)G.idx.size();
    for (int q = 0; q < k; q++) mem.p[q] = ws.p[G.idx[(size_t)q]];
    gws.p[0] = net->group_ws;
    gwt.p[0] = wts.p[G.idx[0]];
    const size_t row0 = (size_t)G.first_row_block * net->mu;
    if (stage_in != (size_t)-1)
      TRY(launch_stack_rows(mem, k, src_off * 2, (char*)net->group_ws + (stage_in + row0 * width) * 2, (int64_t)net->mu * width * 2, true, stream));
    g.M = net->mu * k;
    g.zero_off = net->g_zero_off;
    igemm_set_magics(g, 2);
    const int bm = 128, bn = g.Ncols <= 32 ? 32 : (g.Ncols <= 64 ? 64 : 128);
    const int64_t tiles = (int64_t)((g.M + bm - 1) / bm) * ((g.Ncols + bn - 1) / bn);
    g.scratch_off = net->g_scratch_off;
    g.splits = choose_splits(tiles, 1, (g.Kchunks + 3) / 4, (size_t)g.M * g.Ncols * 4, net->g_scratch_bytes);
    ep.out_off = stage_out + row0 * out_width * (out_esz / 2);
    TRY(launch_igemm(gws, gwt, g, ep, bt, 1, stream));
    return launch_stack_rows(mem, k, dst_off * 2, (char*)net->group_ws + ep.out_off * 2, (int64_t)net->mu * out_width * out_esz, false, stream);
  };
  // ---- forward
  TRY(launch_pack_input(bf, imgs, ws, T[0].off, count, net->mu, net->inpack, net->pixel_mean, stream));
  for (const Op& op : net->ops) {
    const size_t xi = T[(size_t)op.in_t].off, yo = T[(size_t)op.out_t].off;
    switch (op.kind) {
      case OP_CONV:
        if (op.mfma && !bf) {
          Epilogue ep{yo, 0, op.b_off, 1, op.relu ? 1 : 0, 0, 1};
          IGemm gf = op.gf;
          set_splits_f32(net, gf, count);
          TRY(launch_igemm_f32(ws, wts, gf, op.vc, ep, op.w_off, false, count, stream));
        } else if (op.mfma && op.grouped) {
          Epilogue ep{yo, 0, op.b_off, 1, op.relu ? 1 : 0, 0, op.out_f32 ? 1 : 0};
          TRY(launch_fc_group_fwd(wsG, wtsG, gtab, ngroups, op.gf, ep, net->scratch_off, net->scratch_bytes, stream));
        } else if (op.mfma && op.stacked && !groups.empty()) {
          Epilogue ep{yo, 0, op.b_off, 1, op.relu ? 1 : 0, 0, op.out_f32 ? 1 : 0};
          if (count1 > 0) {
            IGemm gf = op.gf;
            set_splits(net, gf, (gf.Kchunks + 3) / 4, count1);
            TRY(launch_igemm(ws1, wts1, gf, ep, false, count1, stream));
          }
          for (const Group& G : groups) {
            IGemm gf = op.gf;
            gf.a_off = op.gx_off + (size_t)G.first_row_block * net->mu * op.cs.C;
            TRY(stacked_product(G, gf, ep, false, xi, op.gx_off, op.cs.C, yo, net->g_y_off, op.cs.K, op.out_f32 ? 4 : 2));
          }
        } else if (op.mfma) {
          Epilogue ep{yo, 0, op.b_off, 1, op.relu ? 1 : 0, 0, op.out_f32 ? 1 : 0};
          IGemm gf = op.gf;
          set_splits(net, gf, (gf.Kchunks + 3) / 4, count);
          if (op.pack_fwd >= 0) TRY(launch_igemm_frag(ws, wts, gf, ep, count, stream));
          else TRY(launch_igemm(ws, wts, gf, ep, false, count, stream));
        } else {
          TRY(launch_conv_fwd_simple(bf, ws, wts, xi, yo, op.w_off, op.b_off, op.cs, op.relu, op.out_f32, count, stream));
        }
        break;
      case OP_POOL_MAX:
      case OP_POOL_AVG:
        TRY(launch_pool_fwd(bf, op.kind == OP_POOL_MAX, ws, xi, yo, op.arg_off, op.ps, op.relu, count, stream));
        break;
      case OP_FLATTEN:
        TRY(launch_flatten_fwd(bf, ws, xi, yo, op.ps.N, op.ps.C, op.ps.H, op.ps.W, count, stream));
        break;
    }
  }
  // ---- loss and its gradient with respect to the class scores
  size_t dy = net->grad_a, dx = net->grad_b;
  TRY(launch_softmax_ce(bf, net->scores_f32, ws, labs, T[(size_t)net->ops.back().out_t].off, dy, net->loss_off, net->mu, net->classes,
                        out_loss_dev, count, stream));
  if (out_rank_dev)
    return launch_label_rank(bf, net->scores_f32, ws, labs, T[(size_t)net->ops.back().out_t].off, net->mu, net->classes, out_rank_dev,
                             count, stream);
  // ---- backward
  // input gradient of a fully connected layer on the MFMA path: per learner, or stacked per group of one weight version
  auto fc_dgrad = [&](const Op& op, const Tensor& tin, size_t dy_off, size_t dx_off) -> hipError_t {
    Epilogue ep{dx_off, tin.off, 0, 0, 0, tin.relu ? 1 : 0, 0};
    if (op.grouped) {
      IGemm gd = op.gd;
      gd.a_off = dy_off;
      return launch_fc_group_dgrad(wsG, wtsG, gtab, ngroups, gd, ep, net->scratch_off, net->scratch_bytes, stream);
    }
    if (!(op.stacked && !groups.empty())) {
      IGemm gd = op.gd;
      gd.a_off = dy_off;
      set_splits(net, gd, (gd.Kchunks + 3) / 4, count);
      return launch_igemm(ws, wts, gd, ep, op.dgrad_bt, count, stream);
    }
    if (count1 > 0) {
      IGemm gd = op.gd;
      gd.a_off = dy_off;
      set_splits(net, gd, (gd.Kchunks + 3) / 4, count1);
      TRY(launch_igemm(ws1, wts1, gd, ep, op.dgrad_bt, count1, stream));
    }
    for (const Group& G : groups) {
      const size_t row0 = (size_t)G.first_row_block * net->mu;
      IGemm gd = op.gd;
      gd.a_off = net->g_dy_off + row0 * op.cs.K;
      Epilogue eg = ep;
      eg.mask_off = op.gx_off + row0 * op.cs.C;      // the layer's stacked input, kept from the forward pass
      TRY(stacked_product(G, gd, eg, op.dgrad_bt, dy_off, net->g_dy_off, op.cs.K, dx_off, net->g_dx_off, op.cs.C, 2));
    }
    return hipSuccess;
  };
  for (int k = (int)net->ops.size() - 1; k >= 0; k--) {
    const Op& op = net->ops[(size_t)k];
    const Tensor& tin = T[(size_t)op.in_t];
    const bool need_dx = op.in_t != 0;          // the network input needs no gradient
    switch (op.kind) {
      case OP_CONV:
        if (op.mfma && !bf) {
          {
            IGemm gw = op.gf;
            const int64_t tiles = (int64_t)((gw.Ncols + 31) / 32) * ((gw.Kchunks * 4 + 1 + 127) / 128);
            gw.scratch_off = net->scratch_off;
            gw.splits = choose_splits(tiles, count, (gw.M + 15) / 16, (size_t)gw.Ncols * (gw.Kchunks * 4 + 4) * 4, net->scratch_bytes);
            TRY(launch_igemm_wgrad_f32(ws, grads, gw, op.vc, dy, op.w_off, op.b_off, count, stream));
          }
          if (need_dx) {
            IGemm gd = op.gd;
            gd.a_off = dy;
            set_splits_f32(net, gd, count);
            Epilogue ep{dx, tin.off, 0, 0, 0, tin.relu ? 1 : 0, 1};
            TRY(launch_igemm_f32(ws, wts, gd, op.vc, ep, op.w_off, true, count, stream));
          }
        } else if (op.mfma && op.factored) {
          TRY(launch_fc_save_factors(ws, grads, tin.off, dy, op.fx_off, op.fdy_off, op.b_off, op.cs.N, op.cs.C, op.cs.K, op.NP, count, stream));
          if (need_dx) TRY(fc_dgrad(op, tin, dy, dx));
        } else if (op.mfma) {
          IGemm gw = op.gf;
          {
            const int64_t tiles = (int64_t)((gw.Ncols + 127) / 128) * ((gw.Kchunks * 8 + 1 + 127) / 128);
            gw.scratch_off = net->scratch_off;
            // narrow layers run small tiles (24-32 KiB of LDS, few registers): six and more workgroups fit a compute
            // unit and each one alone is latency-bound, so they want more of them
            // (CIFAR-shaped layers, 18 learners x 128 images: 1200 workgroups against 600 take conv1 from 148 to 97 us and
            // conv2 from 112 to 80 us; 900 and 1500 are slower again)
            const int64_t target = gw.Ncols <= 64 ? 1200 : 600;
            gw.splits = choose_splits(tiles, count, (gw.M + 31) / 32, (size_t)gw.Ncols * (gw.Kchunks * 8 + 8) * 4, net->scratch_bytes, target);
          }
          TRY(launch_igemm_wgrad(ws, grads, gw, op.vc, dy, op.w_off, op.b_off, count, stream));
          if (need_dx && op.is_fc) {
            TRY(fc_dgrad(op, tin, dy, dx));
          } else if (need_dx) {
            IGemm gd = op.gd;
            gd.a_off = dy;
            set_splits(net, gd, (gd.Kchunks + 3) / 4, count);
            Epilogue ep{dx, tin.off, 0, 0, 0, tin.relu ? 1 : 0, 0};
            if (op.pack_bwd >= 0) TRY(launch_igemm_frag(ws, wts, gd, ep, count, stream));
            else TRY(launch_igemm(ws, wts, gd, ep, op.dgrad_bt, count, stream));
          }
        } else {
          TRY(launch_conv_wgrad_simple(bf, ws, grads, tin.off, dy, op.w_off, op.b_off, op.cs, count, stream));
          if (need_dx) TRY(launch_conv_dgrad_simple(bf, ws, wts, dy, dx, op.w_off, op.cs, tin.relu, tin.off, count, stream));
        }
        break;
      case OP_POOL_MAX:
      case OP_POOL_AVG:
        if (need_dx) TRY(launch_pool_bwd(bf, op.kind == OP_POOL_MAX, ws, dy, dx, op.arg_off, op.ps, tin.relu, tin.off, count, stream));
        break;
      case OP_FLATTEN:
        if (need_dx) TRY(launch_flatten_bwd(bf, ws, dy, dx, op.ps.N, op.ps.C, op.ps.H, op.ps.W, tin.relu, tin.off, count, stream));
        break;
    }
    if (need_dx) { size_t t = dy; dy = dx; dx = t; }
  }
  return hipSuccess;
}

}  // namespace sasgd
