// Host side of one FDG module worker: descriptor validation, workspace plan, the FIFO ring of saved
// forwards, and the launch sequences of forward / delayed backward / update (Section III-A, Eq. 10,
// Eq. 11 and Eq. 15 of arXiv 1906.09108).  This file holds no arithmetic: every number is produced
// by the kernels in conv_kernels.hip and stream_kernels.hip.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <new>
#include <vector>

#include "../../include/fdg.h"
#include "fdg_internal.h"
#include <string.h>

using namespace fdg;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int round8(int c) { return (c + 7) / 8 * 8; }

struct ConvInfo {
  ConvShape sh;
  size_t p_off;                // fp32 master [Co][T][Ci] in the parameter arena (elements)
  size_t w_off, wt_off;        // bf16 copies in a slot's weight arena (elements)
  int stem7_ci = 0;            // > 0: the 7x7 stride-2 stem over stem7_ci channels, held as a 1x1 convolution over the
                               // 448 = 7 x 8 x 8 (row, column, stored channel) elements that launch_im2col7 lays out per pixel
  bool depthwise = false;      // sh = {Co = C, Ci = 1, T = 9}: one 3x3 filter per channel, run by the dwconv3 kernels
};
struct BnInfo {
  int C, M;
  size_t gamma_off, beta_off;  // parameter arena (elements)
  size_t stat_off;             // offset of this BN's [2C] block in every per-BN fp32 array
};
struct ParamTensor {           // one tensor of the external flat order
  size_t ext_off, int_off, count;   // count: elements of the external tensor
  int conv;                    // index into convs, or -1 (stored as is)
};
struct LayerPlan {
  int kind, c_in, c_out, stride;
  int Hi, Wi, Ho, Wo;
  bool projects;
  int conv[4];                 // conv1, conv2, projection (or stem conv in [0]); bottleneck: conv3 in [3]
  int bn[4];                   // bn1, bn2, bnp (stem / head bn in [0]); bottleneck: bn3 in [3]
  size_t act[6];               // byte offsets of saved bf16 tensors in a slot (meaning depends on kind)
  size_t out_b;                // byte offset of this layer's bf16 output in a slot (stream copy)
  size_t fc_w_off, fc_b_off;   // parameter arena (elements)
};

struct Plan {
  fdg_module_desc d;
  std::vector<fdg_layer_desc> layers;
  std::vector<LayerPlan> L;
  std::vector<ConvInfo> convs;
  std::vector<BnInfo> bns;
  std::vector<ParamTensor> ptensors;
  bool is_top = false;
  bool replay = false;         // a saved forward is its input and weight snapshot; the backward runs the forward again
  bool shared_weights = false; // ablation: saved forwards keep no weight snapshot; every pass reads the module's one copy
  int Cp_in = 0;               // channel pitch of the module input copy
  int out_c = 0, out_h = 0, out_w = 0;
  size_t ext_params = 0;       // external parameter count
  size_t conv_elems = 0;       // fp32 conv region (elements)
  size_t P = 0;                // internal parameter arena (elements, multiple of 4)
  size_t small_off = 0, small_count = 0;
  size_t stat_floats = 0;      // 2 * sum of BN channels
  int stat_rep = 0;            // stat_t elements between the copies of the sums arrays: all of them where the narrow kernels run
                               // (hundreds of small workgroups add into the sums), else 0 = a single copy
  size_t warena_elems = 0;     // bf16 elements of one slot's weight arena
  size_t emit_blocks = 0;
  size_t maxE = 0;             // largest activation tensor in elements
  int head_C = 0, head_HW = 0;
  // workspace byte offsets
  size_t o_params = 0, o_mom = 0, o_grads = 0, o_bsums = 0, o_running = 0, o_table = 0, o_slots = 0, slot_bytes = 0;
  // per saved forward: weight snapshot, small-parameter snapshot, labels, (replay) the fp32 NCHW input
  size_t s_warena = 0, s_small = 0, s_labels = 0, s_xcopy = 0;
  size_t o_warena = 0, o_small = 0;   // shared_weights: the module's one bf16 copy of the weights and of the small parameters
  // intermediates: inside every slot, or (replay) once per module at o_inter
  size_t s_sums = 0, s_xin = 0, s_acts = 0, s_pooled = 0, s_dl = 0, s_logits = 0;
  size_t o_inter = 0, inter_bytes = 0;
  size_t o_S[2] = {0, 0}, o_G[2] = {0, 0}, o_GB[2] = {0, 0}, o_T[3] = {0, 0, 0}, o_TP = 0, o_TPB = 0, o_dp = 0;
  size_t o_wscratch = 0, wscratch_bytes = 0;   // partial sums of the split weight gradient
  int wscratch_buffers = 1;
  size_t o_dwscratch = 0, dwscratch_bytes = 0; // the same for depthwise convolutions (they run on the caller's stream)
  size_t o_col = 0, o_colb = 0, col_bytes = 0; // operand rows of a 7x7 stem (launch_im2col7): the forward's and the backward's copy
  size_t total = 0;
  // layout of a caller-provided trace buffer (parity accessors): per layer the fp32 output of the forward and the fp32
  // input gradient of the backward, [L.size()] = the gradient that entered the module, all NHWC as the kernels leave them
  std::vector<size_t> tr_fwd, tr_bwd;
  size_t trace_total = 0;
};

bool build_plan(const fdg_module_desc* desc, int save_mode, Plan& p, fdg_status* why) {
  *why = FDG_ERR_INVALID_ARG;
  if (save_mode != FDG_SAVE_ACTIVATIONS && save_mode != FDG_SAVE_INPUT_AND_REPLAY &&
      save_mode != FDG_SAVE_ACTIVATIONS_CURRENT_WEIGHTS) return false;
  p.replay = save_mode == FDG_SAVE_INPUT_AND_REPLAY;
  p.shared_weights = save_mode == FDG_SAVE_ACTIVATIONS_CURRENT_WEIGHTS;
  if (!desc || !desc->layers || desc->num_layers <= 0) return false;
  if (desc->n <= 0 || desc->c_in <= 0 || desc->h_in <= 0 || desc->w_in <= 0 || desc->delay < 0) return false;
  if (!(desc->beta > 0.f && desc->beta <= 1.f) || !(desc->bn_eps > 0.f)) return false;
  if (desc->momentum < 0.f || desc->weight_decay < 0.f || desc->bn_momentum < 0.f || desc->bn_momentum > 1.f) return false;
  p.d = *desc;
  p.layers.assign(desc->layers, desc->layers + desc->num_layers);
  p.d.layers = nullptr;
  const int N = desc->n;
  int c = desc->c_in, h = desc->h_in, w = desc->w_in;
  p.Cp_in = round8(c);
  p.maxE = (size_t)N * h * w * p.Cp_in;
  size_t act_bytes = 0, ext = 0, small = 0;
  auto add_conv = [&](int Co, int Ci, int T, int stride, int Hi, int Wi) {
    ConvInfo ci{};
    ci.sh = ConvShape{N, Hi, Wi, Ci, round8(Ci), Co, T, stride};
    ci.p_off = p.conv_elems;
    p.conv_elems += (size_t)Co * T * Ci;
    ci.w_off = p.warena_elems;
    p.warena_elems += align_up((size_t)Co * T * ci.sh.Cip, 128);
    ci.wt_off = p.warena_elems;
    p.warena_elems += align_up((size_t)ci.sh.Cip * T * Co, 128);
    p.convs.push_back(ci);
    return (int)p.convs.size() - 1;
  };
  auto add_bn = [&](int C, int M) {
    BnInfo b{};
    b.C = C; b.M = M;
    b.stat_off = p.stat_floats;
    p.stat_floats += 2 * (size_t)C;
    p.bns.push_back(b);
    return (int)p.bns.size() - 1;
  };
  auto save = [&](size_t elems) {  // bf16 tensor saved in the slot
    const size_t off = act_bytes;
    act_bytes += align_up(elems * 2, kAlign);
    if (elems > p.maxE) p.maxE = elems;
    return off;
  };
  // external tensors are appended in the documented order; small tensors get their internal offset later
  struct Pending { int kind; int conv; int bn; int which; size_t count; };  // which: 0 gamma, 1 beta, 2 fc_w, 3 fc_b
  std::vector<Pending> pend;
  for (int i = 0; i < desc->num_layers; ++i) {
    const fdg_layer_desc& ld = p.layers[i];
    LayerPlan lp{};
    lp.kind = ld.kind; lp.c_in = ld.c_in; lp.c_out = ld.c_out; lp.stride = ld.stride;
    lp.conv[0] = lp.conv[1] = lp.conv[2] = lp.conv[3] = -1;
    lp.bn[0] = lp.bn[1] = lp.bn[2] = lp.bn[3] = -1;
    if (ld.c_in != c) return false;
    const bool head = ld.kind == FDG_HEAD_POSTACT || ld.kind == FDG_HEAD_PREACT;
    if (head) {
      if (i != desc->num_layers - 1 || desc->num_classes <= 0 || desc->num_classes > 1024) return false;
      if (c % 8 != 0 || c > 2048) { *why = FDG_ERR_UNSUPPORTED; return false; }
      lp.Hi = lp.Ho = h; lp.Wi = lp.Wo = w;
      p.is_top = true;
      p.head_C = c; p.head_HW = h * w;
      if (ld.kind == FDG_HEAD_PREACT) {
        lp.bn[0] = add_bn(c, N * h * w);
        pend.push_back({0, -1, lp.bn[0], 0, (size_t)c});
        pend.push_back({0, -1, lp.bn[0], 1, (size_t)c});
        lp.act[0] = save((size_t)N * h * w * c);  // o = relu(bn(x))
      }
      pend.push_back({0, -1, i, 2, (size_t)desc->num_classes * c});
      pend.push_back({0, -1, i, 3, (size_t)desc->num_classes});
      p.L.push_back(lp);
      break;
    }
    if (ld.kind != FDG_STEM_CONV_BN_RELU && ld.kind != FDG_BASIC_POSTACT && ld.kind != FDG_BASIC_PREACT &&
        ld.kind != FDG_BOTTLENECK_POSTACT && ld.kind != FDG_STEM_POOL && ld.kind != FDG_INVERTED_RESIDUAL) return false;
    if (ld.kind == FDG_BOTTLENECK_POSTACT && ld.c_out % 32 != 0) { *why = FDG_ERR_UNSUPPORTED; return false; }
    if (ld.kind == FDG_STEM_POOL) {
      if (ld.stride != 4 || ld.c_out <= 0) return false;
      if (i != 0 || !desc->is_bottom || c > 8) { *why = FDG_ERR_UNSUPPORTED; return false; }
    } else if (ld.c_out <= 0 || (ld.stride != 1 && ld.stride != 2)) return false;
    if (ld.c_out % 8 != 0 || ld.c_out > 2048) { *why = FDG_ERR_UNSUPPORTED; return false; }
    if (ld.kind != FDG_STEM_CONV_BN_RELU && ld.kind != FDG_STEM_POOL && (c % 8 != 0 || c > 2048)) { *why = FDG_ERR_UNSUPPORTED; return false; }
    if (ld.kind == FDG_INVERTED_RESIDUAL && 6 * c > 2048) { *why = FDG_ERR_UNSUPPORTED; return false; }
    const int ho = (h - 1) / ld.stride + 1, wo = (w - 1) / ld.stride + 1;
    lp.Hi = h; lp.Wi = w; lp.Ho = ho; lp.Wo = wo;
    lp.projects = (ld.kind == FDG_BASIC_POSTACT || ld.kind == FDG_BASIC_PREACT || ld.kind == FDG_BOTTLENECK_POSTACT) &&
                  (ld.stride != 1 || ld.c_in != ld.c_out);   // blocks with a shortcut only
    const size_t Ein = (size_t)N * h * w * round8(c), Eout = (size_t)N * ho * wo * ld.c_out;
    if (ld.kind == FDG_STEM_CONV_BN_RELU) {
      lp.conv[0] = add_conv(ld.c_out, c, 9, ld.stride, h, w);
      lp.bn[0] = add_bn(ld.c_out, N * ho * wo);
      pend.push_back({1, lp.conv[0], -1, 0, 0});
      pend.push_back({0, -1, lp.bn[0], 0, (size_t)ld.c_out});
      pend.push_back({0, -1, lp.bn[0], 1, (size_t)ld.c_out});
      lp.act[0] = save(Eout);  // c0
    } else if (ld.kind == FDG_BASIC_POSTACT) {
      lp.conv[0] = add_conv(ld.c_out, c, 9, ld.stride, h, w);
      lp.bn[0] = add_bn(ld.c_out, N * ho * wo);
      lp.conv[1] = add_conv(ld.c_out, ld.c_out, 9, 1, ho, wo);
      lp.bn[1] = add_bn(ld.c_out, N * ho * wo);
      pend.push_back({1, lp.conv[0], -1, 0, 0});
      pend.push_back({0, -1, lp.bn[0], 0, (size_t)ld.c_out});
      pend.push_back({0, -1, lp.bn[0], 1, (size_t)ld.c_out});
      pend.push_back({1, lp.conv[1], -1, 0, 0});
      pend.push_back({0, -1, lp.bn[1], 0, (size_t)ld.c_out});
      pend.push_back({0, -1, lp.bn[1], 1, (size_t)ld.c_out});
      lp.act[0] = save(Eout);  // c1
      lp.act[1] = save(Eout);  // a1
      lp.act[2] = save(Eout);  // c2
      if (lp.projects) {
        lp.conv[2] = add_conv(ld.c_out, c, 1, ld.stride, h, w);
        lp.bn[2] = add_bn(ld.c_out, N * ho * wo);
        pend.push_back({1, lp.conv[2], -1, 0, 0});
        pend.push_back({0, -1, lp.bn[2], 0, (size_t)ld.c_out});
        pend.push_back({0, -1, lp.bn[2], 1, (size_t)ld.c_out});
        lp.act[3] = save(Eout);  // p
      }
    } else if (ld.kind == FDG_STEM_POOL) {
      // the convolution as a 1x1 contraction over the 448 gathered elements of an output pixel, at half the input resolution
      const int hc = (h - 1) / 2 + 1, wc = (w - 1) / 2 + 1;
      lp.conv[0] = add_conv(ld.c_out, 448, 1, 1, hc, wc);
      p.convs[lp.conv[0]].stem7_ci = c;
      lp.bn[0] = add_bn(ld.c_out, N * hc * wc);
      pend.push_back({1, lp.conv[0], -1, 0, 0});
      pend.push_back({0, -1, lp.bn[0], 0, (size_t)ld.c_out});
      pend.push_back({0, -1, lp.bn[0], 1, (size_t)ld.c_out});
      lp.act[0] = save((size_t)N * hc * wc * ld.c_out);  // conv output
      lp.act[1] = save((size_t)N * hc * wc * ld.c_out);  // relu(bn): what the pool reads
      p.col_bytes = std::max(p.col_bytes, (size_t)N * hc * wc * 448 * 2);
    } else if (ld.kind == FDG_INVERTED_RESIDUAL) {
      const int cm = 6 * c;
      const size_t Emid_in = (size_t)N * h * w * cm, Emid = (size_t)N * ho * wo * cm;
      lp.conv[0] = add_conv(cm, c, 1, 1, h, w);
      lp.bn[0] = add_bn(cm, N * h * w);
      lp.conv[1] = add_conv(cm, 1, 9, ld.stride, h, w);
      p.convs[lp.conv[1]].depthwise = true;
      lp.bn[1] = add_bn(cm, N * ho * wo);
      lp.conv[3] = add_conv(ld.c_out, cm, 1, 1, ho, wo);
      lp.bn[3] = add_bn(ld.c_out, N * ho * wo);
      const int order[3] = {0, 1, 3};
      for (int q = 0; q < 3; ++q) {
        const int bn = lp.bn[order[q]];
        pend.push_back({1, lp.conv[order[q]], -1, 0, 0});
        pend.push_back({0, -1, bn, 0, (size_t)p.bns[bn].C});
        pend.push_back({0, -1, bn, 1, (size_t)p.bns[bn].C});
      }
      lp.act[0] = save(Emid_in);  // conv1 output
      lp.act[1] = save(Emid_in);  // relu6(bn1)
      lp.act[2] = save(Emid);     // depthwise output
      lp.act[4] = save(Emid);     // relu6(bn2)
      lp.act[5] = save(Eout);     // conv3 output
      p.dwscratch_bytes = std::max(p.dwscratch_bytes, dwconv3_wgrad_scratch_bytes(N, h, w, cm, ld.stride));
    } else if (ld.kind == FDG_BOTTLENECK_POSTACT) {
      const int cm = ld.c_out / 4;
      const size_t Emid_in = (size_t)N * h * w * cm, Emid = (size_t)N * ho * wo * cm;
      lp.conv[0] = add_conv(cm, c, 1, 1, h, w);
      lp.bn[0] = add_bn(cm, N * h * w);
      lp.conv[1] = add_conv(cm, cm, 9, ld.stride, h, w);
      lp.bn[1] = add_bn(cm, N * ho * wo);
      lp.conv[3] = add_conv(ld.c_out, cm, 1, 1, ho, wo);
      lp.bn[3] = add_bn(ld.c_out, N * ho * wo);
      const int order[3] = {0, 1, 3};
      for (int q = 0; q < 3; ++q) {
        const int bn = lp.bn[order[q]];
        pend.push_back({1, lp.conv[order[q]], -1, 0, 0});
        pend.push_back({0, -1, bn, 0, (size_t)p.bns[bn].C});
        pend.push_back({0, -1, bn, 1, (size_t)p.bns[bn].C});
      }
      lp.act[0] = save(Emid_in);  // c1
      lp.act[1] = save(Emid_in);  // a1
      lp.act[2] = save(Emid);     // c2
      lp.act[4] = save(Emid);     // a2
      lp.act[5] = save(Eout);     // c3
      if (lp.projects) {
        lp.conv[2] = add_conv(ld.c_out, c, 1, ld.stride, h, w);
        lp.bn[2] = add_bn(ld.c_out, N * ho * wo);
        pend.push_back({1, lp.conv[2], -1, 0, 0});
        pend.push_back({0, -1, lp.bn[2], 0, (size_t)ld.c_out});
        pend.push_back({0, -1, lp.bn[2], 1, (size_t)ld.c_out});
        lp.act[3] = save(Eout);  // p
      }
    } else {  // pre-activation
      lp.bn[0] = add_bn(c, N * h * w);
      lp.conv[0] = add_conv(ld.c_out, c, 9, ld.stride, h, w);
      lp.bn[1] = add_bn(ld.c_out, N * ho * wo);
      lp.conv[1] = add_conv(ld.c_out, ld.c_out, 9, 1, ho, wo);
      pend.push_back({0, -1, lp.bn[0], 0, (size_t)c});
      pend.push_back({0, -1, lp.bn[0], 1, (size_t)c});
      pend.push_back({1, lp.conv[0], -1, 0, 0});
      pend.push_back({0, -1, lp.bn[1], 0, (size_t)ld.c_out});
      pend.push_back({0, -1, lp.bn[1], 1, (size_t)ld.c_out});
      pend.push_back({1, lp.conv[1], -1, 0, 0});
      lp.act[0] = save(Ein);   // o1
      lp.act[1] = save(Eout);  // c1
      lp.act[2] = save(Eout);  // o2
      if (lp.projects) {
        lp.conv[2] = add_conv(ld.c_out, c, 1, ld.stride, h, w);
        pend.push_back({1, lp.conv[2], -1, 0, 0});
      }
    }
    lp.out_b = save(Eout);  // bf16 copy of the layer output (next layer's MFMA / BN operand, ReLU mask)
    p.L.push_back(lp);
    c = ld.c_out; h = ho; w = wo;
  }
  if (p.is_top) { p.out_c = 1; p.out_h = 1; p.out_w = 1 + N * desc->num_classes; }
  else { p.out_c = c; p.out_h = h; p.out_w = w; }
  // parameter arena: conv region, then the small tensors in external order
  p.small_off = align_up(p.conv_elems, 4);
  size_t soff = p.small_off;
  for (const Pending& q : pend) {
    ParamTensor t{};
    t.ext_off = ext;
    if (q.kind == 1) {
      const ConvInfo& ci = p.convs[q.conv];
      t.count = ci.stem7_ci ? (size_t)ci.sh.Co * ci.stem7_ci * 49 : (size_t)ci.sh.Co * ci.sh.T * ci.sh.Ci;
      t.int_off = ci.p_off;
      t.conv = q.conv;
    } else {
      t.count = q.count;
      t.int_off = soff;
      t.conv = -1;
      if (q.which == 0) p.bns[q.bn].gamma_off = soff;
      else if (q.which == 1) p.bns[q.bn].beta_off = soff;
      else if (q.which == 2) p.L[q.bn].fc_w_off = soff;
      else p.L[q.bn].fc_b_off = soff;
      soff += q.count;
      small += q.count;
    }
    ext += t.count;
    p.ptensors.push_back(t);
  }
  p.ext_params = ext;
  p.small_count = align_up(small, 4);
  p.P = p.small_off + p.small_count;
  if (p.P >= (1ull << 31) || p.warena_elems >= (1ull << 32) || p.maxE >= (1ull << 31)) { *why = FDG_ERR_UNSUPPORTED; return false; }
  for (const ConvInfo& ci : p.convs) p.emit_blocks += emit_blocks_for(ci.sh.Co, ci.sh.Cip, ci.sh.T);
  for (const ConvInfo& ci : p.convs)
    if (!ci.depthwise && conv_dgrad_feeds_next(ci.sh)) p.stat_rep = (int)(p.stat_floats * kStatWords);
  const size_t stat_copies = p.stat_rep ? kStatReplicas : 1;
  // workspace layout
  size_t o = 0;
  auto take = [&](size_t bytes) { const size_t at = o; o += align_up(bytes, kAlign); return at; };
  p.o_params = take(p.P * 4);
  p.o_mom = take(p.P * 4);
  p.o_grads = take(p.P * 4);
  p.o_bsums = take(p.stat_floats * kStatWords * sizeof(stat_t) * stat_copies);   // exact sums (stat_t pairs), copy after copy
  p.o_running = take(p.stat_floats * 4);
  p.o_table = take(p.convs.size() * sizeof(WeightEmitEntry));
  {  // one slot; the intermediates follow the snapshots inside it, or form a region of their own (replay)
    size_t so = 0, io = 0;
    auto stake = [&](size_t bytes) { const size_t at = so; so += align_up(bytes, kAlign); return at; };
    auto itake = [&](size_t bytes) {
      size_t& o2 = p.replay ? io : so;
      const size_t at = o2; o2 += align_up(bytes, kAlign); return at;
    };
    if (!p.shared_weights) {
      p.s_warena = stake(p.warena_elems * 2);
      p.s_small = stake(p.small_count * 4);
    }
    if (p.is_top) p.s_labels = stake((size_t)N * 4);
    if (p.replay) p.s_xcopy = stake((size_t)N * desc->c_in * desc->h_in * desc->w_in * 4);
    p.s_sums = itake(p.stat_floats * kStatWords * sizeof(stat_t) * stat_copies);
    p.s_xin = itake((size_t)N * desc->h_in * desc->w_in * p.Cp_in * 2);
    p.s_acts = itake(act_bytes);
    if (p.is_top) {
      p.s_pooled = itake((size_t)N * p.head_C * 4);
      p.s_dl = itake((size_t)N * desc->num_classes * 4);
      p.s_logits = itake((size_t)N * desc->num_classes * 4);
    }
    p.slot_bytes = so;
    p.inter_bytes = io;
  }
  p.o_slots = take(p.slot_bytes * (size_t)(desc->delay + 1));
  p.o_inter = take(p.inter_bytes);
  if (p.shared_weights) {
    p.o_warena = take(p.warena_elems * 2);
    p.o_small = take(p.small_count * 4);
  }
  for (int i = 0; i < 2; ++i) p.o_S[i] = take(p.maxE * 4);
  for (int i = 0; i < 2; ++i) p.o_G[i] = take(p.maxE * 4);
  for (int i = 0; i < 2; ++i) p.o_GB[i] = take(p.maxE * 2);
  for (int i = 0; i < 3; ++i) p.o_T[i] = take(p.maxE * 2);
  p.o_TP = take(std::max(p.maxE, p.is_top ? (size_t)1 + (size_t)N * desc->num_classes : (size_t)0) * 4);
  // the backward's own copy: a forward and a delayed backward of different contexts share no temporary, so they may
  // run on two streams at once (delay >= 1, stored form)
  p.o_TPB = take(desc->delay >= 1 && !p.replay ? p.maxE * 4 : 0);
  p.o_dp = take(p.is_top ? (size_t)N * p.head_C * 4 : 0);
  for (const ConvInfo& ci : p.convs)
    if (!ci.depthwise) p.wscratch_bytes = std::max(p.wscratch_bytes, conv_wgrad_scratch_bytes(ci.sh));
  // two buffers where weight gradients leave their slices to be added up by the next one (WgradDebt): the slices still owed
  // and the ones being written
  bool defers = false;
  for (const ConvInfo& ci : p.convs) defers = defers || (!ci.depthwise && conv_wgrad_defers(ci.sh));
  p.wscratch_bytes = align_up(p.wscratch_bytes, kAlign);
  p.o_wscratch = take(p.wscratch_bytes * (defers ? 2 : 1));
  p.wscratch_buffers = defers ? 2 : 1;
  p.o_dwscratch = take(p.dwscratch_bytes);
  p.o_col = take(p.col_bytes);
  p.o_colb = (desc->delay >= 1 && !p.replay) ? take(p.col_bytes) : p.o_col;   // as o_TPB: the two may run on two streams
  p.total = o;
  {
    size_t to = 0;
    auto ttake = [&](size_t bytes) { const size_t at = to; to += align_up(bytes, kAlign); return at; };
    for (const LayerPlan& L : p.L) {
      const bool head = L.kind == FDG_HEAD_POSTACT || L.kind == FDG_HEAD_PREACT;
      p.tr_fwd.push_back(ttake(head ? 0 : (size_t)N * L.Ho * L.Wo * L.c_out * 4));
      p.tr_bwd.push_back(ttake((size_t)N * L.Hi * L.Wi * round8(L.c_in) * 4));
    }
    p.tr_bwd.push_back(ttake(p.is_top ? 0 : (size_t)N * p.out_h * p.out_w * p.out_c * 4));
    p.trace_total = to;
  }
  *why = FDG_OK;
  return true;
}

}  // namespace

// Optional per-kernel-class timing with HIP events on the stream the kernels run on.
enum ProfClass { PC_CONV_FWD = 0, PC_CONV_DGRAD, PC_CONV_WGRAD, PC_BN_STATS, PC_BN_APPLY, PC_BN_BWD, PC_SGD,
                 PC_WEIGHT_SNAPSHOT, PC_LAYOUT, PC_HEAD, PC_FILL, PC_COUNT };
static const char* const kProfNames[PC_COUNT] = {"conv_fwd", "conv_dgrad", "conv_wgrad", "bn_stats", "bn_apply", "bn_bwd",
                                                 "sgd", "weight_snapshot", "layout", "head", "fill"};
struct ProfRecord { int cls; double flops, bytes; hipEvent_t e0, e1; char kernel[80]; };
struct Profiler {
  bool on = false;
  bool overflow = false;
  std::vector<ProfRecord> recs;
  std::vector<hipEvent_t> pool;
  size_t used = 0;
  hipEvent_t take() {
    if (used == pool.size()) {
      hipEvent_t e = nullptr;
      if (hipEventCreate(&e) != hipSuccess) return nullptr;
      pool.push_back(e);
    }
    return pool[used++];
  }
  void reset() { recs.clear(); used = 0; overflow = false; }
  ~Profiler() { for (hipEvent_t e : pool) (void)hipEventDestroy(e); }
};

// Weight gradients run on a second stream of the module.  A weight gradient depends only on tensors that exist
// when it is launched and nothing but the update needs its result, so it may overlap the data-gradient / batch-norm
// chain that follows it: while the workgroups of one kernel are in their HBM-bound output stage (or its grid
// leaves compute units idle), workgroups of the other keep the matrix cores busy.  Two rules keep it correct:
// the side stream waits for everything enqueued on the caller's stream before the launch, and a kernel on the
// caller's stream that overwrites a buffer a pending weight gradient reads first waits for that weight gradient.
struct SideStream {
  hipStream_t stream = nullptr;
  hipEvent_t ready = nullptr, joined = nullptr;
  struct Reader { const void* buf = nullptr; hipEvent_t done = nullptr; bool active = false; };
  Reader readers[4];
  bool busy = false;
  bool usable = false;
  bool wanted = true;    // fdg_overlap_enable
  ~SideStream() {
    if (stream) { (void)hipStreamSynchronize(stream); (void)hipStreamDestroy(stream); }
    if (ready) (void)hipEventDestroy(ready);
    if (joined) (void)hipEventDestroy(joined);
    for (Reader& r : readers)
      if (r.done) (void)hipEventDestroy(r.done);
    (void)hipGetLastError();
  }
};

struct fdg_module {
  Plan p;
  mutable Profiler prof;
  mutable SideStream side;
  mutable WgradDebt debt;               // slices of the last narrow weight gradient, not yet added up (on debt_stream)
  mutable hipStream_t debt_stream = nullptr;
  mutable int debt_buffer = 0;          // the scratch buffer the next deferring weight gradient writes
  char* ws = nullptr;
  int64_t seq_fwd = 0, seq_bwd = 0;
  bool has_grad = false;
  int64_t snapshot_seq = -1;          // the forward with this sequence number finds its weight snapshot already in its slot
  bool shared_valid = false;          // shared_weights: the module's bf16 copy is that of the present parameters
                                      // (written by the update before it); -1: none
  hipStream_t last_stream = nullptr;
  hipStream_t fwd_stream = nullptr;   // the forward's last stream (it may differ from the backward's)
  unsigned long long fwd_capture = 0, bwd_capture = 0;   // id of the stream capture the last forward / backward-side call
                                                         // was recorded in (0: it was not being captured)
  char* trace = nullptr;              // attached trace buffer (parity accessors), or nullptr
  std::vector<char> tr_gated;         // per layer: the traced input gradient is already gated by the layer below
  bool tr_fwd_valid = false, tr_bwd_valid = false;

  float* params() const { return reinterpret_cast<float*>(ws + p.o_params); }
  float* mom() const { return reinterpret_cast<float*>(ws + p.o_mom); }
  float* grads() const { return reinterpret_cast<float*>(ws + p.o_grads); }
  stat_t* bsums(const BnInfo& b) const { return reinterpret_cast<stat_t*>(ws + p.o_bsums) + b.stat_off * kStatWords; }
  float* running() const { return reinterpret_cast<float*>(ws + p.o_running); }
  char* slot(int64_t seq) const { return ws + p.o_slots + p.slot_bytes * (size_t)(seq % (p.d.delay + 1)); }
  float* S(int i) const { return reinterpret_cast<float*>(ws + p.o_S[i]); }
  float* G(int i) const { return reinterpret_cast<float*>(ws + p.o_G[i]); }
  bf16_t* GB(int i) const { return reinterpret_cast<bf16_t*>(ws + p.o_GB[i]); }
  bf16_t* T(int i) const { return reinterpret_cast<bf16_t*>(ws + p.o_T[i]); }
  float* TP() const { return reinterpret_cast<float*>(ws + p.o_TP); }
  // projection-shortcut temporary of the backward: its own where forward and backward may overlap
  float* TPB() const { return reinterpret_cast<float*>(ws + ((p.d.delay >= 1 && !p.replay) ? p.o_TPB : p.o_TP)); }
};

namespace {

#define FDG_TRY(expr)                      \
  do {                                     \
    hipError_t e__ = (expr);               \
    if (e__ != hipSuccess) {               \
      (void)hipGetLastError();             \
      return FDG_ERR_HIP;                  \
    }                                      \
  } while (0)

// Id of the capture `s` is being recorded into (hipStreamBeginCapture .. EndCapture), 0 if it is not.
unsigned long long capture_of(hipStream_t s) {
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  unsigned long long id = 0;
  if (hipStreamGetCaptureInfo(s, &st, &id) != hipSuccess) {
    (void)hipGetLastError();
    return 0;
  }
  return st == hipStreamCaptureStatusActive ? id : 0;
}
// One capture that holds the forward on one stream and the backward side on another is refused (see fdg.h, "Two
// streams"): `other` / `other_capture` are the stream and capture id of the last call of the other side.
bool two_streams_in_one_capture(unsigned long long capture, hipStream_t s, unsigned long long other_capture, hipStream_t other) {
  return capture != 0 && capture == other_capture && s != other;
}

// views into one saved forward: `base` its slot, `inter` where its intermediates live
struct SlotView {
  const fdg_module* m;
  char* base;
  char* inter;
  bf16_t* warena() const { return reinterpret_cast<bf16_t*>(m->p.shared_weights ? m->ws + m->p.o_warena : base + m->p.s_warena); }
  bf16_t* W(const ConvInfo& c) const { return warena() + c.w_off; }
  bf16_t* Wt(const ConvInfo& c) const { return warena() + c.wt_off; }
  float* small() const { return reinterpret_cast<float*>(m->p.shared_weights ? m->ws + m->p.o_small : base + m->p.s_small); }
  // snapshot of a small parameter given its offset in the parameter arena
  float* snap(size_t arena_off) const { return small() + (arena_off - m->p.small_off); }
  stat_t* sums(const BnInfo& b) const { return reinterpret_cast<stat_t*>(inter + m->p.s_sums) + b.stat_off * kStatWords; }
  bf16_t* xin() const { return reinterpret_cast<bf16_t*>(inter + m->p.s_xin); }
  bf16_t* act(size_t off) const { return reinterpret_cast<bf16_t*>(inter + m->p.s_acts + off); }
  float* pooled() const { return reinterpret_cast<float*>(inter + m->p.s_pooled); }
  float* dl() const { return reinterpret_cast<float*>(inter + m->p.s_dl); }
  float* logits() const { return reinterpret_cast<float*>(inter + m->p.s_logits); }
  int32_t* labels() const { return reinterpret_cast<int32_t*>(base + m->p.s_labels); }
  float* xcopy() const { return reinterpret_cast<float*>(base + m->p.s_xcopy); }
};
inline SlotView view_of(const fdg_module* m, int64_t seq) {
  char* base = m->slot(seq);
  return SlotView{m, base, m->p.replay ? m->ws + m->p.o_inter : base};
}

// Brackets the launches made in its lifetime with two events when profiling is on.
struct ProfScope {
  Profiler* pr = nullptr;
  hipStream_t s;
  hipEvent_t e1 = nullptr;
  size_t rec = 0;
  // convolutions: which kernel ran, on which layer shape (call after the launch)
  void label(const ConvShape& c) {
    if (!pr) return;
    snprintf(pr->recs[rec].kernel, sizeof(pr->recs[rec].kernel), "%s %d>%d k%d s%d @%dx%d", last_kernel(), c.Ci, c.Co,
             c.T == 9 ? 3 : 1, c.stride, c.Ho(), c.Wo());
  }
  ProfScope(const fdg_module* m, int cls, double flops, double bytes, hipStream_t stream) : s(stream) {
    Profiler& p = m->prof;
    if (!p.on) return;
    if (p.recs.size() >= (1u << 18)) { p.overflow = true; return; }
    hipEvent_t e0 = p.take();
    e1 = p.take();
    if (!e0 || !e1) { e1 = nullptr; return; }
    pr = &p;
    p.recs.push_back(ProfRecord{cls, flops, bytes, e0, e1, {0}});
    rec = p.recs.size() - 1;
    (void)hipEventRecord(e0, s);
  }
  ~ProfScope() { if (pr && e1) (void)hipEventRecord(e1, s); }
};

inline double conv_flops(const ConvShape& c) { return 2.0 * c.N * c.Ho() * c.Wo() * (double)c.Co * c.Ci * c.T; }
inline double conv_in_elems(const ConvShape& c) { return (double)c.N * c.Hi * c.Wi * c.Cip; }
inline double conv_out_elems(const ConvShape& c) { return (double)c.N * c.Ho() * c.Wo() * c.Co; }
inline double conv_w_elems(const ConvShape& c) { return (double)c.Co * c.T * c.Cip; }

hipError_t mconv_forward(const fdg_module* m, const ConvInfo& c, const bf16_t* x, const bf16_t* w, const float* addend,
                         float* out_f32, bf16_t* out_b16, stat_t* stats, hipStream_t s) {
  const double bytes = 2 * conv_in_elems(c.sh) + 2 * conv_w_elems(c.sh) +
                       conv_out_elems(c.sh) * ((addend ? 4 : 0) + (out_f32 ? 4 : 0) + (out_b16 ? 2 : 0));
  ProfScope ps(m, PC_CONV_FWD, conv_flops(c.sh), bytes, s);
  const hipError_t e = conv_forward(c.sh, x, w, addend, out_f32, out_b16, stats, s, m->p.stat_rep);
  ps.label(c.sh);
  return e;
}
// relu(batchnorm_b(x_raw)) -> act_out and the convolution of it, in one launch where the narrow kernel takes the batch-norm
// pass on its patch (conv_forward_bn_applies); false: the caller runs the two launches
bool forward_bn_fuses(const ConvInfo& c, const BnInfo& b, bool with_residual = false) {
  return b.C == c.sh.Cip && (long long)b.M == (long long)c.sh.N * c.sh.Hi * c.sh.Wi && conv_forward_bn_applies(c.sh, with_residual);
}
// res (optional, fp32) is added before the ReLU and act_out_f32 (optional) receives the activation in fp32: the end of the
// layer BELOW (its last batch norm, shortcut and ReLU) done on the patch of this layer's first convolution
hipError_t mconv_forward_after_bn(const fdg_module* m, const SlotView& v, const ConvInfo& c, const BnInfo& b, const bf16_t* x_raw,
                                  bf16_t* act_out, const bf16_t* w, bf16_t* out_b16, stat_t* stats, bool replayed, hipStream_t s,
                                  const float* res = nullptr, float* act_out_f32 = nullptr) {
  ConvInputBn bn{};
  bn.res_f32 = res; bn.act_out_f32 = act_out_f32;
  bn.x_raw = x_raw; bn.sums = v.sums(b); bn.gamma = v.snap(b.gamma_off); bn.beta = v.snap(b.beta_off); bn.act_out = act_out;
  if (!replayed) { bn.run_mean = m->running() + b.stat_off; bn.run_var = m->running() + b.stat_off + b.C; }
  bn.eps = m->p.d.bn_eps; bn.momentum = m->p.d.bn_momentum; bn.rep_stride = m->p.stat_rep;
  const double bytes = conv_in_elems(c.sh) * (2 + 2 + (res ? 4 : 0) + (act_out_f32 ? 4 : 0)) + 2 * conv_w_elems(c.sh) +
                       conv_out_elems(c.sh) * (out_b16 ? 2 : 0);
  ProfScope ps(m, PC_CONV_FWD, conv_flops(c.sh), bytes, s);
  const hipError_t e = conv_forward_bn(c.sh, bn, w, nullptr, nullptr, out_b16, stats, s, m->p.stat_rep);
  ps.label(c.sh);
  return e;
}
// ---- the side stream of the weight gradients (see SideStream) ----
bool side_create(SideStream& sd) {
  bool ok = hipStreamCreateWithFlags(&sd.stream, hipStreamNonBlocking) == hipSuccess;
  ok = ok && hipEventCreateWithFlags(&sd.ready, hipEventDisableTiming) == hipSuccess;
  ok = ok && hipEventCreateWithFlags(&sd.joined, hipEventDisableTiming) == hipSuccess;
  for (SideStream::Reader& r : sd.readers) ok = ok && hipEventCreateWithFlags(&r.done, hipEventDisableTiming) == hipSuccess;
  sd.usable = ok;
  if (!ok) (void)hipGetLastError();
  return ok;
}
// `s` waits for the pending weight gradient that reads `buf`, if there is one: call before overwriting buf.
hipError_t side_wait_readers(const fdg_module* m, const void* buf, hipStream_t s) {
  if (!buf) return hipSuccess;
  for (SideStream::Reader& r : m->side.readers)
    if (r.active && r.buf == buf) {
      r.active = false;
      return hipStreamWaitEvent(s, r.done, 0);
    }
  return hipSuccess;
}
// `s` waits for everything on the side stream (end of a backward; start of any other call after a failed one).
hipError_t side_join(const fdg_module* m, hipStream_t s) {
  SideStream& sd = m->side;
  if (!sd.busy) return hipSuccess;
  hipError_t e = hipEventRecord(sd.joined, sd.stream);
  if (e == hipSuccess) e = hipStreamWaitEvent(s, sd.joined, 0);
  for (SideStream::Reader& r : sd.readers) r.active = false;
  sd.busy = false;
  return e;
}

hipError_t mconv_dgrad(const fdg_module* m, const ConvInfo& c, const bf16_t* dy, const bf16_t* wt, const float* addend,
                       const bf16_t* addmask, float* out_f32, bf16_t* out_b16, hipStream_t s) {
  if (hipError_t e = side_wait_readers(m, out_b16, s); e != hipSuccess) return e;
  const double bytes = 2 * conv_out_elems(c.sh) + 2 * conv_w_elems(c.sh) +
                       conv_in_elems(c.sh) * ((addend ? 4 : 0) + (addmask ? 2 : 0) + (out_f32 ? 4 : 0) + (out_b16 ? 2 : 0));
  ProfScope ps(m, PC_CONV_DGRAD, conv_flops(c.sh), bytes, s);
  const hipError_t e = conv_dgrad(c.sh, dy, wt, addend, addmask, out_f32, out_b16, s);
  ps.label(c.sh);
  return e;
}
// the weight gradient of c on stream ws; narrow layers leave their slices for the next such call on the same stream
hipError_t wgrad_on(const fdg_module* m, const ConvInfo& c, const bf16_t* x, const bf16_t* dy, hipStream_t ws) {
  const Plan& p = m->p;
  if (m->debt.slices > 0 && m->debt_stream != ws) {   // the stream changed under a debt: settle it where it was made
    if (hipError_t e = conv_wgrad_settle(m->debt, m->debt_stream); e != hipSuccess) return e;
    if (hipError_t e = hipStreamSynchronize(m->debt_stream); e != hipSuccess) return e;
  }
  const bool defers = p.wscratch_buffers == 2 && conv_wgrad_defers(c.sh);
  float* scratch = reinterpret_cast<float*>(m->ws + p.o_wscratch + (defers ? (size_t)m->debt_buffer * p.wscratch_bytes : 0));
  if (!defers && m->debt.slices > 0 && m->debt.partial == scratch) {
    // buffer 0 is about to be reused by a kernel that does not take part: what is owed there is added up first
    if (hipError_t e = conv_wgrad_settle(m->debt, ws); e != hipSuccess) return e;
  }
  const hipError_t e = conv_wgrad(c.sh, x, dy, m->grads() + c.p_off, scratch, p.wscratch_bytes, /*overwrite=*/true, ws, &m->debt);
  if (e == hipSuccess) {
    m->debt_stream = ws;
    if (defers && m->debt.partial == scratch) m->debt_buffer ^= 1;
  }
  return e;
}

hipError_t mconv_wgrad(const fdg_module* m, const ConvInfo& c, const bf16_t* x, const bf16_t* dy, hipStream_t s) {
  const double bytes = 2 * conv_in_elems(c.sh) + 2 * conv_out_elems(c.sh) + 4.0 * c.sh.Co * c.sh.T * c.sh.Ci;
  SideStream& sd = m->side;
  if (sd.usable && sd.wanted && !m->prof.on) {   // while timing kernels everything stays on one stream: a kernel's time is its own
    hipError_t e = hipEventRecord(sd.ready, s);
    if (e == hipSuccess) e = hipStreamWaitEvent(sd.stream, sd.ready, 0);
    if (e != hipSuccess) return e;
    sd.busy = true;
    e = wgrad_on(m, c, x, dy, sd.stream);
    if (e != hipSuccess) return e;
    // remember who reads dy: the entry of the same buffer (its earlier reader ran before this one on the side
    // stream), else a free one, else the whole side stream is waited for at the next overwrite of anything
    SideStream::Reader* slot = nullptr;
    for (SideStream::Reader& r : sd.readers)
      if (r.active && r.buf == dy) slot = &r;
    if (!slot)
      for (SideStream::Reader& r : sd.readers)
        if (!r.active) { slot = &r; break; }
    if (!slot) return side_join(m, s);
    slot->buf = dy;
    slot->active = true;
    return hipEventRecord(slot->done, sd.stream);
  }
  ProfScope ps(m, PC_CONV_WGRAD, conv_flops(c.sh), bytes, s);
  const hipError_t e = wgrad_on(m, c, x, dy, s);
  ps.label(c.sh);
  return e;
}
// what the weight gradients of this call still owe (the slices of the last narrow one) is added up: before the side stream
// is joined at the end of a backward
hipError_t settle_wgrad_debt(const fdg_module* m) {
  if (m->debt.slices <= 0) return hipSuccess;
  return conv_wgrad_settle(m->debt, m->debt_stream);
}

hipError_t bn_stats(const SlotView& v, const BnInfo& b, const bf16_t* x, hipStream_t s) {
  ProfScope ps(v.m, PC_BN_STATS, 0, 2.0 * b.M * b.C, s);
  return launch_bn_stats(x, v.sums(b), b.M, b.C, s);
}

// forward apply with the parameters of the slot's snapshot (taken from the current ones just before the forward);
// moves the running statistics unless this is the replay of a saved forward
hipError_t bn_apply(const fdg_module* m, const SlotView& v, const BnInfo& b, const bf16_t* x, const float* res,
                    const BnInfo* b2, const bf16_t* x2, float* out_f32, bf16_t* out_b16, bool replayed, hipStream_t s,
                    int relu = 1) {
  BnApplyArgs a{};
  a.x = x; a.sums = v.sums(b); a.gamma = v.snap(b.gamma_off); a.beta = v.snap(b.beta_off);
  a.res_f32 = res;
  if (b2) {
    a.x2 = x2; a.sums2 = v.sums(*b2); a.gamma2 = v.snap(b2->gamma_off); a.beta2 = v.snap(b2->beta_off);
    if (!replayed) { a.run_mean2 = m->running() + b2->stat_off; a.run_var2 = m->running() + b2->stat_off + b2->C; }
  }
  a.out_f32 = out_f32; a.out_b16 = out_b16;
  if (!replayed) { a.run_mean = m->running() + b.stat_off; a.run_var = m->running() + b.stat_off + b.C; }
  a.M = b.M; a.C = b.C; a.eps = m->p.d.bn_eps; a.momentum = m->p.d.bn_momentum; a.relu = relu;
  a.rep_stride = m->p.stat_rep;
  ProfScope ps(m, PC_BN_APPLY, 0, (double)b.M * b.C * (2 + (res ? 4 : 0) + (b2 ? 2 : 0) + (out_f32 ? 4 : 0) + (out_b16 ? 2 : 0)), s);
  return launch_bn_apply(a, s);
}

// backward through ReLU (mask; gate_hi = 6 for ReLU6; mask == nullptr: no activation to gate by) and BN with the slot's gamma
// snapshot
hipError_t bn_backward(const fdg_module* m, const SlotView& v, const BnInfo& b, const void* dy, bool dy_f32,
                       const bf16_t* mask, const bf16_t* x, const float* addend, float* out_f32, bf16_t* out_b16,
                       hipStream_t s, float gate_hi = 0.f) {
  BnBwdArgs a{};
  a.dy = dy; a.dy_is_f32 = dy_f32 ? 1 : 0; a.mask = mask; a.x = x; a.sums = v.sums(b);
  a.gate_hi = gate_hi;
  a.dy_gated = mask ? 0 : 1;
  a.gamma = v.snap(b.gamma_off);
  a.bsums = m->bsums(b);
  a.addend = addend; a.out_f32 = out_f32; a.out_b16 = out_b16;
  a.dgamma = m->grads() + b.gamma_off; a.dbeta = m->grads() + b.beta_off;
  a.M = b.M; a.C = b.C; a.eps = m->p.d.bn_eps;
  a.rep_stride = a.brep_stride = m->p.stat_rep;
  if (hipError_t e = side_wait_readers(m, out_b16, s); e != hipSuccess) return e;
  // the reduce pass reads dy, gate and x; the apply pass reads them again and writes dx
  const double rd = (dy_f32 ? 4 : 2) + 2 + 2;
  ProfScope ps(m, PC_BN_BWD, 0, (double)b.M * b.C * (rd + ((out_f32 || out_b16) ? rd : 0) + (addend ? 4 : 0) +
                                                     (out_f32 ? 4 : 0) + (out_b16 ? 2 : 0)), s);
  hipError_t e = launch_bn_bwd_reduce(a, s);
  if (e != hipSuccess) return e;
  return launch_bn_bwd_apply(a, s);
}

// The same when dy came out of a gated data gradient (conv_dgrad_gated): it is already zero where the ReLU
// was closed and the two sums are in the module's bsums, so only the apply pass runs.
hipError_t bn_backward_after_gated_dgrad(const fdg_module* m, const SlotView& v, const BnInfo& b, const bf16_t* g,
                                         const bf16_t* x, const float* addend, float* out_f32, bf16_t* out_b16,
                                         hipStream_t s) {
  BnBwdArgs a{};
  a.dy = g; a.dy_is_f32 = 0; a.mask = nullptr; a.x = x; a.sums = v.sums(b);
  a.gamma = v.snap(b.gamma_off);
  a.bsums = m->bsums(b);
  a.addend = addend; a.out_f32 = out_f32; a.out_b16 = out_b16;
  a.dgamma = m->grads() + b.gamma_off; a.dbeta = m->grads() + b.beta_off;
  a.M = b.M; a.C = b.C; a.eps = m->p.d.bn_eps;
  a.rep_stride = a.brep_stride = m->p.stat_rep;
  a.dy_gated = 1; a.raw_sums = 1;
  if (hipError_t e = side_wait_readers(m, out_b16, s); e != hipSuccess) return e;
  ProfScope ps(m, PC_BN_BWD, 0, (double)b.M * b.C * ((out_f32 || out_b16 ? 4 : 0) + (addend ? 4 : 0) + (out_f32 ? 4 : 0) +
                                                     (out_b16 ? 2 : 0)), s);
  return launch_bn_bwd_apply(a, s);
}

// The same for an fp32 gradient that the data gradient of the layer above left gated, with the two sums taken from
// the fp32 values (conv_dgrad_feeding_next).
hipError_t bn_backward_fed_from_above(const fdg_module* m, const SlotView& v, const BnInfo& b, const float* g, const bf16_t* x,
                                      bf16_t* out_b16, hipStream_t s) {
  BnBwdArgs a{};
  a.dy = g; a.dy_is_f32 = 1; a.mask = nullptr; a.x = x; a.sums = v.sums(b);
  a.gamma = v.snap(b.gamma_off);
  a.bsums = m->bsums(b);
  a.out_b16 = out_b16;
  a.dgamma = m->grads() + b.gamma_off; a.dbeta = m->grads() + b.beta_off;
  a.M = b.M; a.C = b.C; a.eps = m->p.d.bn_eps;
  a.rep_stride = a.brep_stride = m->p.stat_rep;
  a.dy_gated = 1; a.raw_sums = 1;
  if (hipError_t e = side_wait_readers(m, out_b16, s); e != hipSuccess) return e;
  ProfScope ps(m, PC_BN_BWD, 0, (double)b.M * b.C * (4 + 2 + 2), s);
  return launch_bn_bwd_apply(a, s);
}

// Data gradient of convolution c into g (bf16), then the backward of the ReLU (gate = its output) and of the batch
// norm b (input x) that precede the convolution.  Where the wide kernels run, the gate and the two sums of the
// batch-norm backward are taken in the data gradient's output stage and one pass over g is saved.
// first half of the function below where the data gradient's output stage gates and sums: g = gate > 0 ? dgrad + addend : 0
// (bf16) and the two sums of batch norm b's backward in the module's bsums
bool dgrad_gates_for(const ConvInfo& c, const BnInfo& b) { return conv_dgrad_gates(c.sh) && b.C == c.sh.Cip; }
hipError_t gated_dgrad(const fdg_module* m, const ConvInfo& c, const bf16_t* dy, const bf16_t* wt, const float* dgrad_addend,
                       const BnInfo& b, const bf16_t* gate, const bf16_t* x, bf16_t* g, hipStream_t s) {
  if (hipError_t e = side_wait_readers(m, g, s); e != hipSuccess) return e;
  const double bytes = 2 * conv_out_elems(c.sh) + 2 * conv_w_elems(c.sh) + conv_in_elems(c.sh) * ((dgrad_addend ? 4 : 0) + 2 + 2 + 2);
  ProfScope ps(m, PC_CONV_DGRAD, conv_flops(c.sh), bytes, s);
  const hipError_t e = conv_dgrad_gated(c.sh, dy, wt, dgrad_addend, gate, x, m->bsums(b), nullptr, g, s, m->p.stat_rep);
  ps.label(c.sh);
  return e;
}
// The batch-norm backward of b (input x, gated gradient g with its two sums in bsums) as the input transform of the data
// gradient that consumes it (conv_dgrad_after_bn): where the narrow kernel takes it, dy never makes a pass of its own
ConvInputBnBwd bn_bwd_input(const fdg_module* m, const SlotView& v, const BnInfo& b, const void* g, bool g_f32, const bf16_t* x,
                            bf16_t* dy_out) {
  ConvInputBnBwd bn{};
  bn.g = g; bn.g_is_f32 = g_f32 ? 1 : 0; bn.x = x; bn.sums = v.sums(b); bn.bsums = m->bsums(b); bn.gamma = v.snap(b.gamma_off);
  bn.dgamma = m->grads() + b.gamma_off; bn.dbeta = m->grads() + b.beta_off; bn.dy_out = dy_out;
  bn.eps = m->p.d.bn_eps; bn.rep_stride = m->p.stat_rep;
  return bn;
}
bool bwd_bn_fuses(const ConvInfo& c, const BnInfo& b, bool g_f32) {
  return b.C == c.sh.Co && (long long)b.M == (long long)c.sh.N * c.sh.Ho() * c.sh.Wo() && conv_dgrad_bn_applies(c.sh, g_f32);
}

hipError_t dgrad_relu_bn_backward(const fdg_module* m, const SlotView& v, const ConvInfo& c, const bf16_t* dy, const bf16_t* wt,
                                  const float* dgrad_addend, const BnInfo& b, const bf16_t* gate, const bf16_t* x, bf16_t* g,
                                  const float* bn_addend, float* out_f32, bf16_t* out_b16, hipStream_t s) {
  if (dgrad_gates_for(c, b)) {
    if (hipError_t e = gated_dgrad(m, c, dy, wt, dgrad_addend, b, gate, x, g, s); e != hipSuccess) return e;
    return bn_backward_after_gated_dgrad(m, v, b, g, x, bn_addend, out_f32, out_b16, s);
  }
  hipError_t e = mconv_dgrad(m, c, dy, wt, dgrad_addend, nullptr, nullptr, g, s);
  if (e != hipSuccess) return e;
  return bn_backward(m, v, b, g, false, gate, x, bn_addend, out_f32, out_b16, s);
}

// The last batch norm of a layer that ends in batch norm + ReLU, and the input of that batch norm in slot v (nullptr:
// the layer does not end that way).
const BnInfo* closing_bn(const Plan& p, const SlotView& v, const LayerPlan& L, const bf16_t** bnx) {
  int bn = -1;
  size_t x = 0;
  if (L.kind == FDG_STEM_CONV_BN_RELU) { bn = L.bn[0]; x = L.act[0]; }
  else if (L.kind == FDG_BASIC_POSTACT) { bn = L.bn[1]; x = L.act[2]; }
  else if (L.kind == FDG_BOTTLENECK_POSTACT) { bn = L.bn[3]; x = L.act[5]; }
  if (bn < 0) return nullptr;
  *bnx = v.act(x);
  return &p.bns[bn];
}

// The layers of the module on x (fp32 NCHW) with the weights of slot v, every intermediate the backward needs
// written where v keeps them.  `replayed`: this forward ran before (v's snapshot and labels are in place); running
// statistics stay as they are and y_dev may be NULL (a head then needs it as scratch for loss and logits).
fdg_status forward_pass(fdg_module* m, const SlotView& v, const float* x_dev, float* y_dev, bool replayed, hipStream_t s) {
  const Plan& p = m->p;
  const int N = p.d.n;
  if (p.stat_floats)
    FDG_TRY(launch_fill_zero(v.sums(p.bns[0]), p.stat_floats * kStatWords * sizeof(stat_t) * (p.stat_rep ? kStatReplicas : 1), s));
  // module input: fp32 NCHW -> fp32 NHWC stream + bf16 NHWC copy (kept for the backward)
  int cur = 0;
  FDG_TRY(launch_nchw_to_nhwc(x_dev, (p.d.c_in % 8 == 0) ? m->S(cur) : nullptr, v.xin(), N, p.d.c_in, p.d.h_in * p.d.w_in,
                              p.Cp_in, 1.f, s));
  const bf16_t* cur_b = v.xin();
  bool stats_ready = false;   // the sums of this layer's leading BN were taken by the producer of its input
  // The last pass of a layer (batch norm [+ shortcut] + ReLU into the fp32 stream and its bf16 copy) is left to the first
  // convolution of the layer ABOVE where that is a basic block whose narrow kernel takes it on its patch: `pend` is that pass,
  // owed from the end of one iteration to the start of the next.
  struct { bool owed = false; const BnInfo* b = nullptr; const bf16_t* x_raw = nullptr; const float* res = nullptr; size_t layer = 0; } pend;
  auto above_takes = [&](size_t li, const BnInfo& b, bool with_res) {
    if (li + 1 >= p.L.size()) return false;
    const LayerPlan& up = p.L[li + 1];
    return up.kind == FDG_BASIC_POSTACT && forward_bn_fuses(p.convs[up.conv[0]], b, with_res);
  };
  for (size_t li = 0; li < p.L.size(); ++li) {
    const LayerPlan& L = p.L[li];
    const int nxt = cur ^ 1;
    bool next_ready = false;
    bool owes = false;
    if (L.kind == FDG_STEM_CONV_BN_RELU) {
      const ConvInfo& c0 = p.convs[L.conv[0]];
      const BnInfo& b0 = p.bns[L.bn[0]];
      FDG_TRY(mconv_forward(m, c0, cur_b, v.W(c0), nullptr, nullptr, v.act(L.act[0]), v.sums(b0), s));
      if (above_takes(li, b0, false)) {
        pend.owed = owes = true; pend.b = &b0; pend.x_raw = v.act(L.act[0]); pend.res = nullptr; pend.layer = li;
      } else {
        FDG_TRY(bn_apply(m, v, b0, v.act(L.act[0]), nullptr, nullptr, nullptr, m->S(nxt), v.act(L.out_b), replayed, s));
      }
    } else if (L.kind == FDG_BASIC_POSTACT) {
      const ConvInfo &c1 = p.convs[L.conv[0]], &c2 = p.convs[L.conv[1]];
      const BnInfo &b1 = p.bns[L.bn[0]], &b2 = p.bns[L.bn[1]];
      bf16_t *t_c1 = v.act(L.act[0]), *t_a1 = v.act(L.act[1]), *t_c2 = v.act(L.act[2]);
      if (pend.owed) {
        // this layer's input (fp32 stream S(cur) and its bf16 copy cur_b) is written here, by the convolution that reads it
        const LayerPlan& below = p.L[pend.layer];
        FDG_TRY(mconv_forward_after_bn(m, v, c1, *pend.b, pend.x_raw, v.act(below.out_b), v.W(c1), t_c1, v.sums(b1), replayed, s,
                                       pend.res, m->S(cur)));
        if (m->trace && !replayed)
          FDG_TRY(hipMemcpyAsync(m->trace + p.tr_fwd[pend.layer], m->S(cur), (size_t)N * below.Ho * below.Wo * below.c_out * 4,
                                 hipMemcpyDeviceToDevice, s));
        pend.owed = false;
      } else {
        FDG_TRY(mconv_forward(m, c1, cur_b, v.W(c1), nullptr, nullptr, t_c1, v.sums(b1), s));
      }
      if (forward_bn_fuses(c2, b1)) {   // BN1 + ReLU on the patch of the second convolution
        FDG_TRY(mconv_forward_after_bn(m, v, c2, b1, t_c1, t_a1, v.W(c2), t_c2, v.sums(b2), replayed, s));
      } else {
        FDG_TRY(bn_apply(m, v, b1, t_c1, nullptr, nullptr, nullptr, nullptr, t_a1, replayed, s));
        FDG_TRY(mconv_forward(m, c2, t_a1, v.W(c2), nullptr, nullptr, t_c2, v.sums(b2), s));
      }
      if (L.projects) {
        const ConvInfo& cp = p.convs[L.conv[2]];
        const BnInfo& bp = p.bns[L.bn[2]];
        bf16_t* t_p = v.act(L.act[3]);
        FDG_TRY(mconv_forward(m, cp, cur_b, v.W(cp), nullptr, nullptr, t_p, v.sums(bp), s));
        FDG_TRY(bn_apply(m, v, b2, t_c2, nullptr, &bp, t_p, m->S(nxt), v.act(L.out_b), replayed, s));
      } else if (above_takes(li, b2, true)) {
        pend.owed = owes = true; pend.b = &b2; pend.x_raw = t_c2; pend.res = m->S(cur); pend.layer = li;
      } else {
        FDG_TRY(bn_apply(m, v, b2, t_c2, m->S(cur), nullptr, nullptr, m->S(nxt), v.act(L.out_b), replayed, s));
      }
    } else if (L.kind == FDG_BOTTLENECK_POSTACT) {
      const ConvInfo &c1 = p.convs[L.conv[0]], &c2 = p.convs[L.conv[1]], &c3 = p.convs[L.conv[3]];
      const BnInfo &b1 = p.bns[L.bn[0]], &b2 = p.bns[L.bn[1]], &b3 = p.bns[L.bn[3]];
      bf16_t *t_c1 = v.act(L.act[0]), *t_a1 = v.act(L.act[1]), *t_c2 = v.act(L.act[2]), *t_a2 = v.act(L.act[4]),
             *t_c3 = v.act(L.act[5]);
      FDG_TRY(mconv_forward(m, c1, cur_b, v.W(c1), nullptr, nullptr, t_c1, v.sums(b1), s));
      FDG_TRY(bn_apply(m, v, b1, t_c1, nullptr, nullptr, nullptr, nullptr, t_a1, replayed, s));
      FDG_TRY(mconv_forward(m, c2, t_a1, v.W(c2), nullptr, nullptr, t_c2, v.sums(b2), s));
      FDG_TRY(bn_apply(m, v, b2, t_c2, nullptr, nullptr, nullptr, nullptr, t_a2, replayed, s));
      FDG_TRY(mconv_forward(m, c3, t_a2, v.W(c3), nullptr, nullptr, t_c3, v.sums(b3), s));
      if (L.projects) {
        const ConvInfo& cp = p.convs[L.conv[2]];
        const BnInfo& bp = p.bns[L.bn[2]];
        bf16_t* t_p = v.act(L.act[3]);
        FDG_TRY(mconv_forward(m, cp, cur_b, v.W(cp), nullptr, nullptr, t_p, v.sums(bp), s));
        FDG_TRY(bn_apply(m, v, b3, t_c3, nullptr, &bp, t_p, m->S(nxt), v.act(L.out_b), replayed, s));
      } else {
        FDG_TRY(bn_apply(m, v, b3, t_c3, m->S(cur), nullptr, nullptr, m->S(nxt), v.act(L.out_b), replayed, s));
      }
    } else if (L.kind == FDG_STEM_POOL) {
      const ConvInfo& c0 = p.convs[L.conv[0]];
      const BnInfo& b0 = p.bns[L.bn[0]];
      bf16_t* col = reinterpret_cast<bf16_t*>(m->ws + p.o_col);
      bf16_t *t_c = v.act(L.act[0]), *t_a = v.act(L.act[1]);
      FDG_TRY(side_wait_readers(m, col, s));
      FDG_TRY(launch_im2col7(cur_b, col, N, L.Hi, L.Wi, s));
      FDG_TRY(mconv_forward(m, c0, col, v.W(c0), nullptr, nullptr, t_c, v.sums(b0), s));
      FDG_TRY(bn_apply(m, v, b0, t_c, nullptr, nullptr, nullptr, nullptr, t_a, replayed, s));
      FDG_TRY(launch_maxpool3s2(t_a, m->S(nxt), v.act(L.out_b), N, c0.sh.Hi, c0.sh.Wi, L.c_out, s));
    } else if (L.kind == FDG_INVERTED_RESIDUAL) {
      const ConvInfo &c1 = p.convs[L.conv[0]], &c2 = p.convs[L.conv[1]], &c3 = p.convs[L.conv[3]];
      const BnInfo &b1 = p.bns[L.bn[0]], &b2 = p.bns[L.bn[1]], &b3 = p.bns[L.bn[3]];
      bf16_t *t_c1 = v.act(L.act[0]), *t_a1 = v.act(L.act[1]), *t_c2 = v.act(L.act[2]), *t_a2 = v.act(L.act[4]),
             *t_c3 = v.act(L.act[5]);
      FDG_TRY(mconv_forward(m, c1, cur_b, v.W(c1), nullptr, nullptr, t_c1, v.sums(b1), s));
      FDG_TRY(bn_apply(m, v, b1, t_c1, nullptr, nullptr, nullptr, nullptr, t_a1, replayed, s, /*relu6*/ 2));
      FDG_TRY(launch_dwconv3_fwd(t_a1, v.Wt(c2), t_c2, N, L.Hi, L.Wi, c2.sh.Co, L.stride, s));
      FDG_TRY(bn_stats(v, b2, t_c2, s));
      FDG_TRY(bn_apply(m, v, b2, t_c2, nullptr, nullptr, nullptr, nullptr, t_a2, replayed, s, /*relu6*/ 2));
      FDG_TRY(mconv_forward(m, c3, t_a2, v.W(c3), nullptr, nullptr, t_c3, v.sums(b3), s));
      const bool adds = L.stride == 1 && L.c_in == L.c_out;
      FDG_TRY(bn_apply(m, v, b3, t_c3, adds ? m->S(cur) : nullptr, nullptr, nullptr, m->S(nxt), v.act(L.out_b), replayed, s, /*no activation*/ 0));
    } else if (L.kind == FDG_BASIC_PREACT) {
      const ConvInfo &c1 = p.convs[L.conv[0]], &c2 = p.convs[L.conv[1]];
      const BnInfo &b1 = p.bns[L.bn[0]], &b2 = p.bns[L.bn[1]];
      bf16_t *t_o1 = v.act(L.act[0]), *t_c1 = v.act(L.act[1]), *t_o2 = v.act(L.act[2]);
      if (!stats_ready) FDG_TRY(bn_stats(v, b1, cur_b, s));
      FDG_TRY(bn_apply(m, v, b1, cur_b, nullptr, nullptr, nullptr, nullptr, t_o1, replayed, s));
      FDG_TRY(mconv_forward(m, c1, t_o1, v.W(c1), nullptr, nullptr, t_c1, v.sums(b2), s));
      FDG_TRY(bn_apply(m, v, b2, t_c1, nullptr, nullptr, nullptr, nullptr, t_o2, replayed, s));
      const float* shortcut = m->S(cur);
      if (L.projects) {
        const ConvInfo& cp = p.convs[L.conv[2]];
        FDG_TRY(mconv_forward(m, cp, t_o1, v.W(cp), nullptr, m->TP(), nullptr, nullptr, s));
        shortcut = m->TP();
      }
      // the block output is the next layer's BN input when that layer is pre-activated: take its sums here
      stat_t* next_stats = nullptr;
      if (li + 1 < p.L.size() && (p.L[li + 1].kind == FDG_BASIC_PREACT || p.L[li + 1].kind == FDG_HEAD_PREACT))
        next_stats = v.sums(p.bns[p.L[li + 1].bn[0]]);
      FDG_TRY(mconv_forward(m, c2, t_o2, v.W(c2), shortcut, m->S(nxt), v.act(L.out_b), next_stats, s));
      next_ready = next_stats != nullptr;
    } else {  // heads
      const bf16_t* o = cur_b;
      if (L.kind == FDG_HEAD_PREACT) {
        const BnInfo& b0 = p.bns[L.bn[0]];
        if (!stats_ready) FDG_TRY(bn_stats(v, b0, cur_b, s));
        FDG_TRY(bn_apply(m, v, b0, cur_b, nullptr, nullptr, nullptr, nullptr, v.act(L.act[0]), replayed, s));
        o = v.act(L.act[0]);
      }
      const int J = p.d.num_classes;
      FDG_TRY(launch_avgpool(o, v.pooled(), N, p.head_HW, p.head_C, s));
      FDG_TRY(launch_fc_fwd(v.pooled(), v.snap(L.fc_w_off), v.snap(L.fc_b_off), v.logits(), N, p.head_C, J, s));
      FDG_TRY(launch_softmax_ce(v.logits(), v.labels(), y_dev, v.dl(), N, J, s));
      break;
    }
    if (m->trace && !replayed && !owes)
      FDG_TRY(hipMemcpyAsync(m->trace + p.tr_fwd[li], m->S(nxt), (size_t)N * L.Ho * L.Wo * L.c_out * 4, hipMemcpyDeviceToDevice, s));
    cur = nxt;
    cur_b = v.act(L.out_b);
    stats_ready = next_ready;
  }
  if (m->trace && !replayed) m->tr_fwd_valid = true;
  if (!p.is_top && y_dev) FDG_TRY(launch_nhwc_to_nchw(m->S(cur), y_dev, N, p.out_c, p.out_h * p.out_w, p.out_c, s));
  return FDG_OK;
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// C ABI
// ------------------------------------------------------------------------------------------------
// bf16 copy of the present convolution weights (both layouts) and fp32 copy of the small parameters into v's snapshot
static fdg_status emit_snapshot(fdg_module* m, const SlotView& v, hipStream_t s) {
  const Plan& p = m->p;
  {
    ProfScope ps(m, PC_WEIGHT_SNAPSHOT, 0, 4.0 * p.conv_elems + 2.0 * p.warena_elems, s);
    FDG_TRY(launch_emit_weights(m->params(), v.warena(), reinterpret_cast<const WeightEmitEntry*>(m->ws + p.o_table),
                                (int)p.convs.size(), (int)p.emit_blocks, s));
  }
  if (p.small_count)
    FDG_TRY(hipMemcpyAsync(v.small(), m->params() + p.small_off, p.small_count * 4, hipMemcpyDeviceToDevice, s));
  return FDG_OK;
}

extern "C" {

size_t fdg_module_workspace_bytes_ex(const fdg_module_desc* desc, int32_t save_mode) {
  Plan p;
  fdg_status why;
  if (!build_plan(desc, save_mode, p, &why)) return 0;
  return p.total;
}
size_t fdg_module_workspace_bytes(const fdg_module_desc* desc) { return fdg_module_workspace_bytes_ex(desc, FDG_SAVE_ACTIVATIONS); }

fdg_status fdg_module_create(const fdg_module_desc* desc, void* dev_workspace, size_t bytes, void* hip_stream,
                             fdg_module** out) {
  return fdg_module_create_ex(desc, FDG_SAVE_ACTIVATIONS, dev_workspace, bytes, hip_stream, out);
}

fdg_status fdg_module_create_ex(const fdg_module_desc* desc, int32_t save_mode, void* dev_workspace, size_t bytes,
                                void* hip_stream, fdg_module** out) {
  if (!out) return FDG_ERR_INVALID_ARG;
  *out = nullptr;
  fdg_module* m = new (std::nothrow) fdg_module();
  if (!m) return FDG_ERR_INVALID_ARG;
  fdg_status why;
  if (!build_plan(desc, save_mode, m->p, &why)) {
    delete m;
    return why;
  }
  if (!dev_workspace || bytes < m->p.total || (reinterpret_cast<uintptr_t>(dev_workspace) % kAlign) != 0) {
    delete m;
    return dev_workspace ? FDG_ERR_WORKSPACE_TOO_SMALL : FDG_ERR_INVALID_ARG;
  }
  m->ws = static_cast<char*>(dev_workspace);
  m->tr_gated.assign(m->p.L.size(), 0);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  m->last_stream = s;
  m->fwd_stream = s;
  (void)side_create(m->side);   // without it the weight gradients simply stay on the caller's stream
  const Plan& p = m->p;
  // parameters, momentum, gradients, backward sums, running statistics (mean 0, var 1), emit table
  hipError_t e = launch_fill_zero(m->ws, p.o_running, s);
  if (e == hipSuccess) e = launch_fill_zero(m->ws + p.o_running, align_up(p.stat_floats * 4, kAlign), s);
  for (const BnInfo& b : p.bns)
    if (e == hipSuccess) e = launch_fill_f32(m->running() + b.stat_off + b.C, b.C, 1.f, s);
  if (e == hipSuccess && !p.convs.empty()) {
    std::vector<WeightEmitEntry> tab(p.convs.size());
    uint32_t blk = 0;
    for (size_t i = 0; i < p.convs.size(); ++i) {
      const ConvInfo& c = p.convs[i];
      tab[i].src_off = (uint32_t)c.p_off; tab[i].w_off = (uint32_t)c.w_off; tab[i].wt_off = (uint32_t)c.wt_off;
      tab[i].Co = c.sh.Co; tab[i].T = c.sh.T; tab[i].Ci = c.sh.Ci; tab[i].Cip = c.sh.Cip;
      tab[i].block_start = blk;
      blk += emit_blocks_for(c.sh.Co, c.sh.Cip, c.sh.T);
    }
    e = hipMemcpyAsync(m->ws + p.o_table, tab.data(), tab.size() * sizeof(WeightEmitEntry), hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);  // tab is a host temporary
  }
  if (e != hipSuccess) {
    (void)hipGetLastError();
    delete m;
    return FDG_ERR_HIP;
  }
  *out = m;
  return FDG_OK;
}

void fdg_destroy(fdg_module* m) { delete m; }

fdg_status fdg_forward(fdg_module* m, const float* x_dev, const int32_t* labels_dev, float* y_dev, void* hip_stream) {
  if (!m || !x_dev || !y_dev) return FDG_ERR_INVALID_ARG;
  const Plan& p = m->p;
  if (p.is_top != (labels_dev != nullptr)) return FDG_ERR_INVALID_ARG;
  if (m->seq_fwd - m->seq_bwd >= p.d.delay + 1) return FDG_ERR_QUEUE_FULL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const unsigned long long cap = capture_of(s);
  if (two_streams_in_one_capture(cap, s, m->bwd_capture, m->last_stream)) return FDG_ERR_UNSUPPORTED;
  m->fwd_capture = cap;
  m->fwd_stream = s;
  FDG_TRY(side_join(m, s));
  SlotView v = view_of(m, m->seq_fwd);
  const int N = p.d.n;
  // snapshot of the weights this forward uses (Eq. 10 evaluates the backward at these), unless the update that produced
  // them has already left it in this slot
  if (m->p.shared_weights ? !m->shared_valid : m->snapshot_seq != m->seq_fwd) if (fdg_status st = emit_snapshot(m, v, s); st != FDG_OK) return st;
  m->snapshot_seq = -1;
  m->shared_valid = true;
  if (p.is_top) FDG_TRY(hipMemcpyAsync(v.labels(), labels_dev, (size_t)N * 4, hipMemcpyDeviceToDevice, s));
  if (p.replay) FDG_TRY(hipMemcpyAsync(v.xcopy(), x_dev, (size_t)N * p.d.c_in * p.d.h_in * p.d.w_in * 4, hipMemcpyDeviceToDevice, s));
  if (fdg_status st = forward_pass(m, v, x_dev, y_dev, /*replayed=*/false, s); st != FDG_OK) return st;
  ++m->seq_fwd;
  return FDG_OK;
}

fdg_status fdg_backward_delayed(fdg_module* m, const float* grad_out_dev, float* grad_in_dev, void* hip_stream) {
  if (!m) return FDG_ERR_INVALID_ARG;
  const Plan& p = m->p;
  if (p.is_top ? grad_out_dev != nullptr : grad_out_dev == nullptr) return FDG_ERR_INVALID_ARG;
  if (m->seq_fwd == m->seq_bwd) return FDG_ERR_QUEUE_EMPTY;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const unsigned long long cap = capture_of(s);
  if (two_streams_in_one_capture(cap, s, m->fwd_capture, m->fwd_stream)) return FDG_ERR_UNSUPPORTED;
  m->bwd_capture = cap;
  m->last_stream = s;
  SlotView v = view_of(m, m->seq_bwd);  // the OLDEST saved forward
  const int N = p.d.n;
  // the backward sums of batch norm accumulate with atomics and start at zero; every gradient is written
  // (not accumulated) by the kernel that produces it
  FDG_TRY(side_join(m, s));
  if (p.shared_weights && !m->shared_valid) {   // the parameters were set from outside since the copy was made
    if (fdg_status st = emit_snapshot(m, v, s); st != FDG_OK) return st;
    m->shared_valid = true;
  }
  if (p.replay) {   // the saved forward is its input and its weights: run it again into the module's one set of intermediates
    if (fdg_status st = forward_pass(m, v, v.xcopy(), p.is_top ? m->TP() : nullptr, /*replayed=*/true, s); st != FDG_OK) return st;
  }
  FDG_TRY(launch_fill_zero(m->ws + p.o_bsums, p.o_running - p.o_bsums, s));
  int cur = 0;
  if (!p.is_top)  // gradient shrinking of Eq. 15: multiply by beta before anything else
    FDG_TRY(launch_nchw_to_nhwc(grad_out_dev, m->G(cur), m->GB(cur), N, p.out_c, p.out_h * p.out_w, p.out_c, p.d.beta, s));
  if (m->trace && !p.is_top)
    FDG_TRY(hipMemcpyAsync(m->trace + p.tr_bwd[p.L.size()], m->G(cur), (size_t)N * p.out_h * p.out_w * p.out_c * 4,
                           hipMemcpyDeviceToDevice, s));
  bool fed = false;   // G(cur) came from the layer above already gated by this layer's output, with this layer's
                      // last batch norm's two sums in bsums
  for (int li = (int)p.L.size() - 1; li >= 0; --li) {
    const LayerPlan& L = p.L[li];
    const int nxt = cur ^ 1;
    const bf16_t* in_b = li == 0 ? v.xin() : v.act(p.L[li - 1].out_b);  // bf16 copy of this layer's input
    const bool need_dx = !(li == 0 && p.d.is_bottom);
    const bool fed_here = fed;
    fed = false;
    if (L.kind == FDG_HEAD_POSTACT || L.kind == FDG_HEAD_PREACT) {
      const int J = p.d.num_classes;
      float* dp = reinterpret_cast<float*>(m->ws + p.o_dp);
      FDG_TRY(launch_fc_bwd(v.pooled(), v.snap(L.fc_w_off), v.dl(), m->grads() + L.fc_w_off, m->grads() + L.fc_b_off, dp, N,
                            p.head_C, J, s));
      if (L.kind == FDG_HEAD_PREACT) {
        const BnInfo& b0 = p.bns[L.bn[0]];
        FDG_TRY(launch_pool_bwd(dp, m->TPB(), nullptr, N, p.head_HW, p.head_C, s));
        FDG_TRY(bn_backward(m, v, b0, m->TPB(), true, v.act(L.act[0]), in_b, nullptr, m->G(nxt), m->GB(nxt), s));
      } else {
        FDG_TRY(side_wait_readers(m, m->GB(nxt), s));
        FDG_TRY(launch_pool_bwd(dp, m->G(nxt), m->GB(nxt), N, p.head_HW, p.head_C, s));
      }
    } else if (L.kind == FDG_STEM_CONV_BN_RELU) {
      const ConvInfo& c0 = p.convs[L.conv[0]];
      const BnInfo& b0 = p.bns[L.bn[0]];
      if (fed_here) FDG_TRY(bn_backward_fed_from_above(m, v, b0, m->G(cur), v.act(L.act[0]), m->T(0), s));
      else FDG_TRY(bn_backward(m, v, b0, m->G(cur), true, v.act(L.out_b), v.act(L.act[0]), nullptr, nullptr, m->T(0), s));
      FDG_TRY(mconv_wgrad(m, c0, in_b, m->T(0), s));
      if (need_dx) FDG_TRY(mconv_dgrad(m, c0, m->T(0), v.Wt(c0), nullptr, nullptr, m->G(nxt), m->GB(nxt), s));
    } else if (L.kind == FDG_BASIC_POSTACT) {
      const ConvInfo &c1 = p.convs[L.conv[0]], &c2 = p.convs[L.conv[1]];
      const BnInfo &b1 = p.bns[L.bn[0]], &b2 = p.bns[L.bn[1]];
      const bf16_t *t_c1 = v.act(L.act[0]), *t_a1 = v.act(L.act[1]), *t_c2 = v.act(L.act[2]), *t_y = v.act(L.out_b);
      // final ReLU mask (y > 0) then BN2; weight gradient and data gradient of conv2 (through ReLU and BN1); weight gradient
      // and data gradient of conv1.  Where the narrow kernel runs, the apply half of each batch-norm backward is done on
      // the patch of the data gradient that consumes it (fuse2: BN2 into conv2's, fuse1: BN1 into conv1's); that kernel
      // also writes the batch norm's result, which the weight gradient of the same convolution reads afterwards.
      // In the narrow layers the gated gradient g between conv2's data gradient and BN1's backward stays in fp32 (gf): a
      // bf16 g whose batch-norm backward is rounded to bf16 again is rounded twice, and the second rounding is then biased
      // (g sits on a grid of 256 mantissas, the batch norm's small per-channel terms fall below half a step of it), a bias
      // that conv1's weight gradient adds up coherently over all pixels: 2e-2 .. 4e-2 of it at 131072 pixels.
      const bool gated = dgrad_gates_for(c2, b1);
      const bool g32 = gated && conv_dgrad_feeds_next(c2.sh);
      float* gf = m->TPB();
      const bool fuse2 = fed_here && gated && bwd_bn_fuses(c2, b2, /*g_f32=*/true);
      const bool fuse1 = gated && !L.projects && need_dx && bwd_bn_fuses(c1, b1, /*g_f32=*/g32);
      bf16_t* dy_c1 = m->T(0);
      if (fuse2) {
        FDG_TRY(side_wait_readers(m, m->T(0), s));
        FDG_TRY(side_wait_readers(m, m->T(1), s));
        {
          const ConvInputBnBwd bn = bn_bwd_input(m, v, b2, m->G(cur), true, t_c2, m->T(0));
          const double bytes = conv_out_elems(c2.sh) * (4 + 2 + 2) + 2 * conv_w_elems(c2.sh) + conv_in_elems(c2.sh) * (2 + 2 + 2);
          ProfScope ps(m, PC_CONV_DGRAD, conv_flops(c2.sh), bytes, s);
          const hipError_t e = conv_dgrad_after_bn(c2.sh, bn, v.Wt(c2), nullptr, nullptr, t_a1, t_c1, m->bsums(b1), g32, g32 ? gf : nullptr,
                                                   g32 ? nullptr : m->T(1), s, p.stat_rep);
          ps.label(c2.sh);
          FDG_TRY(e);
        }
        FDG_TRY(mconv_wgrad(m, c2, t_a1, m->T(0), s));
      } else {
        if (fed_here) FDG_TRY(bn_backward_fed_from_above(m, v, b2, m->G(cur), t_c2, m->T(0), s));
        else FDG_TRY(bn_backward(m, v, b2, m->G(cur), true, t_y, t_c2, nullptr, nullptr, m->T(0), s));
        FDG_TRY(mconv_wgrad(m, c2, t_a1, m->T(0), s));
        if (g32) {
          const double bytes = 2 * conv_out_elems(c2.sh) + 2 * conv_w_elems(c2.sh) + conv_in_elems(c2.sh) * (4 + 2 + 2);
          ProfScope ps(m, PC_CONV_DGRAD, conv_flops(c2.sh), bytes, s);
          const hipError_t e = conv_dgrad_feeding_next(c2.sh, m->T(0), v.Wt(c2), nullptr, nullptr, t_a1, t_c1, m->bsums(b1), gf, nullptr, s,
                                                       p.stat_rep);
          ps.label(c2.sh);
          FDG_TRY(e);
        } else if (gated) FDG_TRY(gated_dgrad(m, c2, m->T(0), v.Wt(c2), nullptr, b1, t_a1, t_c1, m->T(1), s));
        else FDG_TRY(dgrad_relu_bn_backward(m, v, c2, m->T(0), v.Wt(c2), nullptr, b1, t_a1, t_c1, m->T(1), nullptr, nullptr, m->T(0), s));
      }
      if (fuse1) {
        dy_c1 = m->T(2);   // written by conv1's data gradient below; T(0) may still be read by conv2's weight gradient
      } else {
        if (g32) FDG_TRY(bn_backward_fed_from_above(m, v, b1, gf, t_c1, m->T(0), s));
        else if (gated) FDG_TRY(bn_backward_after_gated_dgrad(m, v, b1, m->T(1), t_c1, nullptr, nullptr, m->T(0), s));
        FDG_TRY(mconv_wgrad(m, c1, in_b, dy_c1, s));
      }
      if (L.projects) {
        const ConvInfo& cp = p.convs[L.conv[2]];
        const BnInfo& bp = p.bns[L.bn[2]];
        FDG_TRY(bn_backward(m, v, bp, m->G(cur), true, t_y, v.act(L.act[3]), nullptr, nullptr, m->T(1), s));
        FDG_TRY(mconv_wgrad(m, cp, in_b, m->T(1), s));
        if (need_dx && conv_dgrad_pair_applies(c1.sh, cp.sh)) {
          // the data gradients of the 3x3 and of the projection beside it, both stride 2, in one launch
          FDG_TRY(side_wait_readers(m, m->GB(nxt), s));
          const double bytes = 2 * (conv_out_elems(c1.sh) + conv_out_elems(cp.sh)) + 2 * (conv_w_elems(c1.sh) + conv_w_elems(cp.sh)) +
                               conv_in_elems(c1.sh) * (4 + 2);
          ProfScope ps(m, PC_CONV_DGRAD, conv_flops(c1.sh) + conv_flops(cp.sh), bytes, s);
          const hipError_t e = conv_dgrad_gated_pair(c1.sh, m->T(0), v.Wt(c1), cp.sh, m->T(1), v.Wt(cp), nullptr, nullptr, nullptr,
                                                     m->G(nxt), m->GB(nxt), s);
          ps.label(c1.sh);
          FDG_TRY(e);
        } else if (need_dx) {
          FDG_TRY(mconv_dgrad(m, cp, m->T(1), v.Wt(cp), nullptr, nullptr, m->TPB(), nullptr, s));
          FDG_TRY(mconv_dgrad(m, c1, m->T(0), v.Wt(c1), m->TPB(), nullptr, m->G(nxt), m->GB(nxt), s));
        }
      } else if (need_dx) {
        // identity shortcut: the masked incoming gradient joins the branch gradient.  Where the narrow kernel runs
        // and the layer below ends in batch norm + ReLU, its output stage also does the first half of that layer's
        // backward: the ReLU gate and the two sums of the batch norm.
        const bf16_t* bnx = nullptr;
        const BnInfo* bb = li > 0 ? closing_bn(p, v, p.L[li - 1], &bnx) : nullptr;
        const bool feeds = bb && bb->C == c1.sh.Cip && conv_dgrad_feeds_next(c1.sh);
        if (fuse1) {
          FDG_TRY(side_wait_readers(m, m->T(2), s));
          FDG_TRY(side_wait_readers(m, m->GB(nxt), s));
          {
            const ConvInputBnBwd bn = g32 ? bn_bwd_input(m, v, b1, gf, true, t_c1, m->T(2)) : bn_bwd_input(m, v, b1, m->T(1), false, t_c1, m->T(2));
            const double bytes = conv_out_elems(c1.sh) * (2 + 2 + 2) + 2 * conv_w_elems(c1.sh) +
                                 conv_in_elems(c1.sh) * (4 + 2 + (feeds ? 2 + 2 : 0) + 4 + 2);
            ProfScope ps(m, PC_CONV_DGRAD, conv_flops(c1.sh), bytes, s);
            const hipError_t e = conv_dgrad_after_bn(c1.sh, bn, v.Wt(c1), m->G(cur), t_y, feeds ? in_b : nullptr, feeds ? bnx : nullptr,
                                                     feeds ? m->bsums(*bb) : nullptr, feeds, m->G(nxt), m->GB(nxt), s, p.stat_rep);
            ps.label(c1.sh);
            FDG_TRY(e);
          }
          fed = feeds;
          FDG_TRY(mconv_wgrad(m, c1, in_b, m->T(2), s));
        } else if (feeds) {
          FDG_TRY(side_wait_readers(m, m->GB(nxt), s));
          const double bytes = 2 * conv_out_elems(c1.sh) + 2 * conv_w_elems(c1.sh) + conv_in_elems(c1.sh) * (4 + 2 + 2 + 2 + 4 + 2);
          ProfScope ps(m, PC_CONV_DGRAD, conv_flops(c1.sh), bytes, s);
          const hipError_t e = conv_dgrad_feeding_next(c1.sh, m->T(0), v.Wt(c1), m->G(cur), t_y, in_b, bnx,
                                                       m->bsums(*bb), m->G(nxt), m->GB(nxt), s, p.stat_rep);
          ps.label(c1.sh);
          FDG_TRY(e);
          fed = true;
        } else {
          FDG_TRY(mconv_dgrad(m, c1, m->T(0), v.Wt(c1), m->G(cur), t_y, m->G(nxt), m->GB(nxt), s));
        }
      }
    } else if (L.kind == FDG_BOTTLENECK_POSTACT) {
      const ConvInfo &c1 = p.convs[L.conv[0]], &c2 = p.convs[L.conv[1]], &c3 = p.convs[L.conv[3]];
      const BnInfo &b1 = p.bns[L.bn[0]], &b2 = p.bns[L.bn[1]], &b3 = p.bns[L.bn[3]];
      const bf16_t *t_c1 = v.act(L.act[0]), *t_a1 = v.act(L.act[1]), *t_c2 = v.act(L.act[2]), *t_a2 = v.act(L.act[4]),
                   *t_c3 = v.act(L.act[5]), *t_y = v.act(L.out_b);
      // final ReLU mask (y > 0) then BN3; then twice: weight gradient, data gradient through ReLU and batch norm
      if (fed_here) FDG_TRY(bn_backward_fed_from_above(m, v, b3, m->G(cur), t_c3, m->T(0), s));
      else FDG_TRY(bn_backward(m, v, b3, m->G(cur), true, t_y, t_c3, nullptr, nullptr, m->T(0), s));
      FDG_TRY(mconv_wgrad(m, c3, t_a2, m->T(0), s));
      FDG_TRY(dgrad_relu_bn_backward(m, v, c3, m->T(0), v.Wt(c3), nullptr, b2, t_a2, t_c2, m->T(1), nullptr, nullptr, m->T(0), s));
      FDG_TRY(mconv_wgrad(m, c2, t_a1, m->T(0), s));
      FDG_TRY(dgrad_relu_bn_backward(m, v, c2, m->T(0), v.Wt(c2), nullptr, b1, t_a1, t_c1, m->T(1), nullptr, nullptr, m->T(0), s));
      FDG_TRY(mconv_wgrad(m, c1, in_b, m->T(0), s));
      if (L.projects) {
        const ConvInfo& cp = p.convs[L.conv[2]];
        const BnInfo& bp = p.bns[L.bn[2]];
        FDG_TRY(bn_backward(m, v, bp, m->G(cur), true, t_y, v.act(L.act[3]), nullptr, nullptr, m->T(1), s));
        FDG_TRY(mconv_wgrad(m, cp, in_b, m->T(1), s));
        if (need_dx) {
          FDG_TRY(mconv_dgrad(m, cp, m->T(1), v.Wt(cp), nullptr, nullptr, m->TPB(), nullptr, s));
          FDG_TRY(mconv_dgrad(m, c1, m->T(0), v.Wt(c1), m->TPB(), nullptr, m->G(nxt), m->GB(nxt), s));
        }
      } else if (need_dx) {
        // identity shortcut: as in the basic block, the data gradient that ends this block's backward can also gate by
        // the output of the layer below and take the two sums of that layer's last batch norm
        const bf16_t* bnx = nullptr;
        const BnInfo* bb = li > 0 ? closing_bn(p, v, p.L[li - 1], &bnx) : nullptr;
        if (bb && bb->C == c1.sh.Cip && conv_dgrad_feeds_next(c1.sh)) {
          FDG_TRY(side_wait_readers(m, m->GB(nxt), s));
          const double bytes = 2 * conv_out_elems(c1.sh) + 2 * conv_w_elems(c1.sh) + conv_in_elems(c1.sh) * (4 + 2 + 2 + 2 + 4 + 2);
          ProfScope ps(m, PC_CONV_DGRAD, conv_flops(c1.sh), bytes, s);
          const hipError_t e = conv_dgrad_feeding_next(c1.sh, m->T(0), v.Wt(c1), m->G(cur), t_y, in_b, bnx,
                                                       m->bsums(*bb), m->G(nxt), m->GB(nxt), s, p.stat_rep);
          ps.label(c1.sh);
          FDG_TRY(e);
          fed = true;
        } else {
          FDG_TRY(mconv_dgrad(m, c1, m->T(0), v.Wt(c1), m->G(cur), t_y, m->G(nxt), m->GB(nxt), s));
        }
      }
    } else if (L.kind == FDG_STEM_POOL) {
      // the pool hands every window's gradient to its first maximum; then ReLU, batch norm, and the weight gradient of
      // the convolution as a 1x1 contraction over the gathered operand rows (gathered again: they are not kept)
      const ConvInfo& c0 = p.convs[L.conv[0]];
      const BnInfo& b0 = p.bns[L.bn[0]];
      bf16_t* col = reinterpret_cast<bf16_t*>(m->ws + p.o_colb);
      const bf16_t *t_c = v.act(L.act[0]), *t_a = v.act(L.act[1]);
      FDG_TRY(launch_maxpool3s2_bwd(t_a, m->G(cur), m->TPB(), N, c0.sh.Hi, c0.sh.Wi, L.c_out, s));
      FDG_TRY(bn_backward(m, v, b0, m->TPB(), true, t_a, t_c, nullptr, nullptr, m->T(0), s));
      FDG_TRY(side_wait_readers(m, col, s));
      FDG_TRY(launch_im2col7(in_b, col, N, L.Hi, L.Wi, s));
      FDG_TRY(mconv_wgrad(m, c0, col, m->T(0), s));
    } else if (L.kind == FDG_INVERTED_RESIDUAL) {
      const ConvInfo &c1 = p.convs[L.conv[0]], &c2 = p.convs[L.conv[1]], &c3 = p.convs[L.conv[3]];
      const BnInfo &b1 = p.bns[L.bn[0]], &b2 = p.bns[L.bn[1]], &b3 = p.bns[L.bn[3]];
      const bf16_t *t_c1 = v.act(L.act[0]), *t_a1 = v.act(L.act[1]), *t_c2 = v.act(L.act[2]), *t_a2 = v.act(L.act[4]),
                   *t_c3 = v.act(L.act[5]);
      const bool adds = L.stride == 1 && L.c_in == L.c_out;
      // the block ends in a batch norm: nothing gates the incoming gradient
      FDG_TRY(bn_backward(m, v, b3, m->G(cur), true, nullptr, t_c3, nullptr, nullptr, m->T(0), s));
      FDG_TRY(mconv_wgrad(m, c3, t_a2, m->T(0), s));
      // the gradients that go into a gate and a batch-norm backward stay in fp32 (a bf16 one, rounded again after that
      // backward, is rounded with a bias that the per-channel sums of this block's many pixels add up)
      float* gf = m->TPB();
      FDG_TRY(mconv_dgrad(m, c3, m->T(0), v.Wt(c3), nullptr, nullptr, gf, nullptr, s));
      FDG_TRY(bn_backward(m, v, b2, gf, true, t_a2, t_c2, nullptr, nullptr, m->T(0), s, 6.f));
      FDG_TRY(launch_dwconv3_wgrad(t_a1, m->T(0), m->grads() + c2.p_off, reinterpret_cast<float*>(m->ws + p.o_dwscratch),
                                   p.dwscratch_bytes, N, L.Hi, L.Wi, c2.sh.Co, L.stride, s));
      FDG_TRY(launch_dwconv3_dgrad(m->T(0), v.Wt(c2), nullptr, N, L.Hi, L.Wi, c2.sh.Co, L.stride, s, gf));
      FDG_TRY(bn_backward(m, v, b1, gf, true, t_a1, t_c1, nullptr, nullptr, m->T(0), s, 6.f));
      FDG_TRY(mconv_wgrad(m, c1, in_b, m->T(0), s));
      if (need_dx) FDG_TRY(mconv_dgrad(m, c1, m->T(0), v.Wt(c1), adds ? m->G(cur) : nullptr, nullptr, m->G(nxt), m->GB(nxt), s));
    } else {  // pre-activation block: y = conv2(o2) + shortcut
      const ConvInfo &c1 = p.convs[L.conv[0]], &c2 = p.convs[L.conv[1]];
      const BnInfo &b1 = p.bns[L.bn[0]], &b2 = p.bns[L.bn[1]];
      const bf16_t *t_o1 = v.act(L.act[0]), *t_c1 = v.act(L.act[1]), *t_o2 = v.act(L.act[2]);
      FDG_TRY(mconv_wgrad(m, c2, t_o2, m->GB(cur), s));
      FDG_TRY(dgrad_relu_bn_backward(m, v, c2, m->GB(cur), v.Wt(c2), nullptr, b2, t_o2, t_c1, m->T(0), nullptr, nullptr, m->T(1), s));
      FDG_TRY(mconv_wgrad(m, c1, t_o1, m->T(1), s));
      if (L.projects) {
        const ConvInfo& cp = p.convs[L.conv[2]];
        FDG_TRY(mconv_wgrad(m, cp, t_o1, m->GB(cur), s));
        if (conv_dgrad_pair_applies(c1.sh, cp.sh) && b1.C == c1.sh.Cip) {
          // both data gradients into the block's input (3x3 and projection, stride 2) in one launch, gated, with the sums of BN1
          FDG_TRY(side_wait_readers(m, m->T(0), s));
          {
            const double bytes = 2 * (conv_out_elems(c1.sh) + conv_out_elems(cp.sh)) + 2 * (conv_w_elems(c1.sh) + conv_w_elems(cp.sh)) +
                                 conv_in_elems(c1.sh) * (2 + 2 + 2);
            ProfScope ps(m, PC_CONV_DGRAD, conv_flops(c1.sh) + conv_flops(cp.sh), bytes, s);
            const hipError_t e = conv_dgrad_gated_pair(c1.sh, m->T(1), v.Wt(c1), cp.sh, m->GB(cur), v.Wt(cp), t_o1, in_b,
                                                       m->bsums(b1), nullptr, m->T(0), s, p.stat_rep);
            ps.label(c1.sh);
            FDG_TRY(e);
          }
          FDG_TRY(bn_backward_after_gated_dgrad(m, v, b1, m->T(0), in_b, nullptr, need_dx ? m->G(nxt) : nullptr,
                                                need_dx ? m->GB(nxt) : nullptr, s));
        } else {
          FDG_TRY(mconv_dgrad(m, cp, m->GB(cur), v.Wt(cp), nullptr, nullptr, m->TPB(), nullptr, s));
          FDG_TRY(dgrad_relu_bn_backward(m, v, c1, m->T(1), v.Wt(c1), m->TPB(), b1, t_o1, in_b, m->T(0), nullptr,
                                         need_dx ? m->G(nxt) : nullptr, need_dx ? m->GB(nxt) : nullptr, s));
        }
      } else {
        FDG_TRY(dgrad_relu_bn_backward(m, v, c1, m->T(1), v.Wt(c1), nullptr, b1, t_o1, in_b, m->T(0), m->G(cur),
                                       need_dx ? m->G(nxt) : nullptr, need_dx ? m->GB(nxt) : nullptr, s));
      }
    }
    if (m->trace && need_dx) {
      FDG_TRY(hipMemcpyAsync(m->trace + p.tr_bwd[li], m->G(nxt), (size_t)N * L.Hi * L.Wi * round8(L.c_in) * 4,
                             hipMemcpyDeviceToDevice, s));
      m->tr_gated[li] = fed ? 1 : 0;
    }
    cur = nxt;
  }
  if (m->trace) m->tr_bwd_valid = true;
  if (grad_in_dev && !p.d.is_bottom)
    FDG_TRY(launch_nhwc_to_nchw(m->G(cur), grad_in_dev, N, p.d.c_in, p.d.h_in * p.d.w_in, p.Cp_in, s));
  FDG_TRY(settle_wgrad_debt(m));
  FDG_TRY(side_join(m, s));   // the gradient is complete when the call's stream gets here
  ++m->seq_bwd;
  m->has_grad = true;
  return FDG_OK;
}

fdg_status fdg_update(fdg_module* m, float lr, void* hip_stream) {
  if (!m) return FDG_ERR_INVALID_ARG;
  if (!m->has_grad) return FDG_ERR_NO_GRAD;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const unsigned long long cap = capture_of(s);
  if (two_streams_in_one_capture(cap, s, m->fwd_capture, m->fwd_stream)) return FDG_ERR_UNSUPPORTED;
  m->bwd_capture = cap;
  m->last_stream = s;
  FDG_TRY(side_join(m, s));
  const Plan& p = m->p;
  if (p.shared_weights || m->seq_fwd - m->seq_bwd <= p.d.delay) {
    // (Ablation with one copy of the weights per module: that copy follows every update.)
    // The slot of the NEXT forward holds no saved forward that still waits for its backward (the last backward, which
    // this update is ordered after, was its last reader), so the update also leaves that forward's weight snapshot
    // there: theta is read once for both.
    const SlotView v = view_of(m, m->seq_fwd);
    ProfScope ps(m, PC_SGD, 0, 20.0 * p.P + 2.0 * p.warena_elems + 4.0 * p.small_count, s);
    FDG_TRY(launch_sgd_emit(m->params(), m->mom(), m->grads(), v.warena(), v.small(),
                            reinterpret_cast<const WeightEmitEntry*>(m->ws + p.o_table), (int)p.convs.size(), (int)p.emit_blocks,
                            p.small_off, p.small_count, lr, p.d.momentum, p.d.weight_decay, s));
    m->snapshot_seq = m->seq_fwd;
    m->shared_valid = true;
  } else {   // the ring is full: the next forward cannot start before another backward, and takes its own snapshot
    ProfScope ps(m, PC_SGD, 0, 20.0 * p.P, s);   // read theta, v, g; write theta, v
    FDG_TRY(launch_sgd(m->params(), m->mom(), m->grads(), p.P, lr, p.d.momentum, p.d.weight_decay, s));
    m->snapshot_seq = -1;
  }
  m->has_grad = false;
  return FDG_OK;
}

size_t fdg_param_count(const fdg_module* m) { return m ? m->p.ext_params : 0; }

// external flat order <-> internal arena order
static void ext_to_int(const Plan& p, const float* ext, float* in) {
  for (const ParamTensor& t : p.ptensors) {
    if (t.conv < 0) {
      for (size_t i = 0; i < t.count; ++i) in[t.int_off + i] = ext[t.ext_off + i];
    } else if (const int s7 = p.convs[t.conv].stem7_ci) {
      // [Co, ci, 7, 7] -> [Co][kh][kw of 8][c of 8]; the eighth column and the channels beyond ci stay zero
      const ConvShape& c = p.convs[t.conv].sh;
      for (int co = 0; co < c.Co; ++co)
        for (int ci = 0; ci < s7; ++ci)
          for (int kh = 0; kh < 7; ++kh)
            for (int kw = 0; kw < 7; ++kw)
              in[t.int_off + (size_t)co * 448 + kh * 64 + kw * 8 + ci] = ext[t.ext_off + (((size_t)co * s7 + ci) * 7 + kh) * 7 + kw];
    } else {
      const ConvShape& c = p.convs[t.conv].sh;
      for (int co = 0; co < c.Co; ++co)
        for (int ci = 0; ci < c.Ci; ++ci)
          for (int k = 0; k < c.T; ++k)
            in[t.int_off + ((size_t)co * c.T + k) * c.Ci + ci] = ext[t.ext_off + ((size_t)co * c.Ci + ci) * c.T + k];
    }
  }
}
static void int_to_ext(const Plan& p, const float* in, float* ext) {
  for (const ParamTensor& t : p.ptensors) {
    if (t.conv < 0) {
      for (size_t i = 0; i < t.count; ++i) ext[t.ext_off + i] = in[t.int_off + i];
    } else if (const int s7 = p.convs[t.conv].stem7_ci) {
      const ConvShape& c = p.convs[t.conv].sh;
      for (int co = 0; co < c.Co; ++co)
        for (int ci = 0; ci < s7; ++ci)
          for (int kh = 0; kh < 7; ++kh)
            for (int kw = 0; kw < 7; ++kw)
              ext[t.ext_off + (((size_t)co * s7 + ci) * 7 + kh) * 7 + kw] = in[t.int_off + (size_t)co * 448 + kh * 64 + kw * 8 + ci];
    } else {
      const ConvShape& c = p.convs[t.conv].sh;
      for (int co = 0; co < c.Co; ++co)
        for (int ci = 0; ci < c.Ci; ++ci)
          for (int k = 0; k < c.T; ++k)
            ext[t.ext_off + ((size_t)co * c.Ci + ci) * c.T + k] = in[t.int_off + ((size_t)co * c.T + k) * c.Ci + ci];
    }
  }
}

fdg_status fdg_set_params(fdg_module* m, const float* host_src, size_t count) {
  if (!m || !host_src || count != m->p.ext_params) return FDG_ERR_INVALID_ARG;
  std::vector<float> buf(m->p.P, 0.f);
  ext_to_int(m->p, host_src, buf.data());
  FDG_TRY(hipStreamSynchronize(m->last_stream));
  if (m->fwd_stream != m->last_stream) FDG_TRY(hipStreamSynchronize(m->fwd_stream));
  FDG_TRY(hipMemcpy(m->params(), buf.data(), m->p.P * 4, hipMemcpyHostToDevice));
  m->snapshot_seq = -1;   // a snapshot the last update left for the next forward is of the old parameters
  m->shared_valid = false;
  FDG_TRY(hipMemset(m->mom(), 0, m->p.P * 4));
  FDG_TRY(hipDeviceSynchronize());
  return FDG_OK;
}

static fdg_status read_arena(const fdg_module* m, const float* dev, float* host_dst, size_t count) {
  if (!m || !host_dst || count != m->p.ext_params) return FDG_ERR_INVALID_ARG;
  std::vector<float> buf(m->p.P);
  FDG_TRY(hipStreamSynchronize(m->last_stream));
  if (m->fwd_stream != m->last_stream) FDG_TRY(hipStreamSynchronize(m->fwd_stream));
  FDG_TRY(hipMemcpy(buf.data(), dev, m->p.P * 4, hipMemcpyDeviceToHost));
  int_to_ext(m->p, buf.data(), host_dst);
  return FDG_OK;
}
fdg_status fdg_get_params(const fdg_module* m, float* host_dst, size_t count) {
  return read_arena(m, m ? m->params() : nullptr, host_dst, count);
}
fdg_status fdg_get_grads(const fdg_module* m, float* host_dst, size_t count) {
  return read_arena(m, m ? m->grads() : nullptr, host_dst, count);
}
fdg_status fdg_get_momentum(const fdg_module* m, float* host_dst, size_t count) {
  return read_arena(m, m ? m->mom() : nullptr, host_dst, count);
}

size_t fdg_bn_stat_count(const fdg_module* m) { return m ? m->p.stat_floats : 0; }
fdg_status fdg_get_bn_running(const fdg_module* m, float* host_dst, size_t count) {
  if (!m || !host_dst || count != m->p.stat_floats) return FDG_ERR_INVALID_ARG;
  if (count == 0) return FDG_OK;
  // the arena holds the BNs in creation order; report them in parameter order
  std::vector<float> buf(count);
  FDG_TRY(hipStreamSynchronize(m->last_stream));
  if (m->fwd_stream != m->last_stream) FDG_TRY(hipStreamSynchronize(m->fwd_stream));
  FDG_TRY(hipMemcpy(buf.data(), m->running(), count * 4, hipMemcpyDeviceToHost));
  size_t o = 0;
  for (const ParamTensor& t : m->p.ptensors) {
    if (t.conv >= 0) continue;
    for (const BnInfo& b : m->p.bns)
      if (b.gamma_off == t.int_off) {
        for (int i = 0; i < 2 * b.C; ++i) host_dst[o++] = buf[b.stat_off + i];
        break;
      }
  }
  return o == count ? FDG_OK : FDG_ERR_INVALID_ARG;
}

fdg_status fdg_output_shape(const fdg_module* m, int32_t out[4]) {
  if (!m || !out) return FDG_ERR_INVALID_ARG;
  out[0] = m->p.is_top ? 1 : m->p.d.n;
  out[1] = m->p.out_c; out[2] = m->p.out_h; out[3] = m->p.out_w;
  return FDG_OK;
}

fdg_status fdg_input_shape(const fdg_module* m, int32_t out[4]) {
  if (!m || !out) return FDG_ERR_INVALID_ARG;
  out[0] = m->p.d.n; out[1] = m->p.d.c_in; out[2] = m->p.d.h_in; out[3] = m->p.d.w_in;
  return FDG_OK;
}

fdg_status fdg_module_traits(const fdg_module* m, int32_t* delay, int32_t* is_bottom, int32_t* is_top) {
  if (!m) return FDG_ERR_INVALID_ARG;
  if (delay) *delay = m->p.d.delay;
  if (is_bottom) *is_bottom = m->p.d.is_bottom ? 1 : 0;
  if (is_top) *is_top = m->p.is_top ? 1 : 0;
  return FDG_OK;
}

fdg_status fdg_queue_state(const fdg_module* m, int32_t* outstanding, int64_t* oldest_seq, int64_t* newest_seq) {
  if (!m) return FDG_ERR_INVALID_ARG;
  const int64_t n = m->seq_fwd - m->seq_bwd;
  if (outstanding) *outstanding = (int32_t)n;
  if (oldest_seq) *oldest_seq = n ? m->seq_bwd : -1;
  if (newest_seq) *newest_seq = n ? m->seq_fwd - 1 : -1;
  return FDG_OK;
}

// ---- parity accessors ----
static fdg_status sync_streams(const fdg_module* m) {
  FDG_TRY(hipStreamSynchronize(m->last_stream));
  if (m->fwd_stream != m->last_stream) FDG_TRY(hipStreamSynchronize(m->fwd_stream));
  return FDG_OK;
}
// device [n, hw, cp] (bf16 or fp32) -> host fp32 [n, c, hw]
static fdg_status read_nhwc(const void* dev, bool is_b16, int n, int c, int cp, int hw, float* host_dst) {
  const size_t elems = (size_t)n * hw * cp;
  std::vector<float> f(elems);
  if (is_b16) {
    std::vector<uint16_t> raw(elems);
    FDG_TRY(hipMemcpy(raw.data(), dev, elems * 2, hipMemcpyDeviceToHost));
    for (size_t i = 0; i < elems; ++i) {
      const uint32_t u = (uint32_t)raw[i] << 16;
      memcpy(&f[i], &u, 4);
    }
  } else {
    FDG_TRY(hipMemcpy(f.data(), dev, elems * 4, hipMemcpyDeviceToHost));
  }
  for (int i = 0; i < n; ++i)
    for (int q = 0; q < hw; ++q)
      for (int k = 0; k < c; ++k) host_dst[((size_t)i * c + k) * hw + q] = f[((size_t)i * hw + q) * cp + k];
  return FDG_OK;
}

fdg_status fdg_saved_read(const fdg_module* m, int64_t seq, int32_t layer, int32_t which, float* host_dst, size_t count,
                          int32_t shape[4]) {
  if (!m || !host_dst || layer < 0 || layer >= (int)m->p.L.size()) return FDG_ERR_INVALID_ARG;
  const Plan& p = m->p;
  if (seq < 0 || seq >= m->seq_fwd || seq < m->seq_fwd - (p.d.delay + 1)) return FDG_ERR_INVALID_ARG;
  if (p.replay && seq != m->seq_bwd - 1) return FDG_ERR_INVALID_ARG;   // one set of intermediates: the last replayed context's
  const LayerPlan& L = p.L[layer];
  const SlotView v = view_of(m, seq);
  const int N = p.d.n;
  const bool head = L.kind == FDG_HEAD_POSTACT || L.kind == FDG_HEAD_PREACT;
  const void* dev = nullptr;
  bool b16 = true;
  int c = 0, h = 0, w = 0;
  const int cm = L.c_out / 4;
  if (which >= 0 && which <= 5) {
    // which intermediates a layer kind has, with their shapes
    bool has = false;
    c = L.c_out; h = L.Ho; w = L.Wo;
    switch (L.kind) {
      case FDG_STEM_CONV_BN_RELU: has = which == 0; break;
      case FDG_BASIC_POSTACT: has = which <= 2 || (which == 3 && L.projects); break;
      case FDG_BASIC_PREACT:
        has = which <= 2;
        if (which == 0) { c = L.c_in; h = L.Hi; w = L.Wi; }
        break;
      case FDG_BOTTLENECK_POSTACT:
        has = which != 3 || L.projects;
        if (which == 0 || which == 1) { c = cm; h = L.Hi; w = L.Wi; }
        if (which == 2 || which == 4) c = cm;
        break;
      case FDG_HEAD_PREACT: has = which == 0; c = L.c_in; h = L.Hi; w = L.Wi; break;
      case FDG_STEM_POOL: has = which <= 1; h = (L.Hi - 1) / 2 + 1; w = (L.Wi - 1) / 2 + 1; break;
      case FDG_INVERTED_RESIDUAL:
        has = which != 3;
        if (which == 0 || which == 1) { c = 6 * L.c_in; h = L.Hi; w = L.Wi; }
        if (which == 2 || which == 4) c = 6 * L.c_in;
        break;
      default: break;
    }
    if (!has) return FDG_ERR_INVALID_ARG;
    dev = v.act(L.act[which]);
  } else if (which == 6) {
    if (head) return FDG_ERR_INVALID_ARG;
    c = L.c_out; h = L.Ho; w = L.Wo;
    dev = v.act(L.out_b);
  } else if (which == 7) {
    c = L.c_in; h = L.Hi; w = L.Wi;
    dev = layer == 0 ? v.xin() : v.act(p.L[layer - 1].out_b);
  } else if (which == 8 || which == 9) {
    if (!head) return FDG_ERR_INVALID_ARG;
    b16 = false;
    c = which == 8 ? p.head_C : p.d.num_classes; h = w = 1;
    dev = which == 8 ? v.pooled() : v.dl();
  } else {
    return FDG_ERR_INVALID_ARG;
  }
  if (shape) { shape[0] = N; shape[1] = c; shape[2] = h; shape[3] = w; }
  if (count != (size_t)N * c * h * w) return FDG_ERR_INVALID_ARG;
  if (fdg_status st = sync_streams(m); st != FDG_OK) return st;
  return read_nhwc(dev, b16, N, c, b16 ? round8(c) : c, h * w, host_dst);   // the head's fp32 tensors are dense
}

size_t fdg_trace_bytes(const fdg_module* m) { return m ? m->p.trace_total : 0; }

fdg_status fdg_trace_attach(fdg_module* m, void* dev_trace, size_t bytes) {
  if (!m) return FDG_ERR_INVALID_ARG;
  if (dev_trace && (bytes < m->p.trace_total || (reinterpret_cast<uintptr_t>(dev_trace) % kAlign) != 0))
    return FDG_ERR_WORKSPACE_TOO_SMALL;
  if (fdg_status st = sync_streams(m); st != FDG_OK) return st;
  m->trace = static_cast<char*>(dev_trace);
  m->tr_fwd_valid = m->tr_bwd_valid = false;
  return FDG_OK;
}

fdg_status fdg_trace_read(const fdg_module* m, int32_t dir, int32_t layer, float* host_dst, size_t count, int32_t shape[4],
                          int32_t* gated) {
  if (!m || !host_dst || !m->trace || (dir != 0 && dir != 1)) return FDG_ERR_INVALID_ARG;
  const Plan& p = m->p;
  const int nl = (int)p.L.size(), N = p.d.n;
  int c = 0, h = 0, w = 0;
  size_t off = 0;
  int g = 0;
  if (dir == 0) {
    if (layer < 0 || layer >= nl || !m->tr_fwd_valid) return FDG_ERR_INVALID_ARG;
    const LayerPlan& L = p.L[layer];
    if (L.kind == FDG_HEAD_POSTACT || L.kind == FDG_HEAD_PREACT) return FDG_ERR_INVALID_ARG;
    c = L.c_out; h = L.Ho; w = L.Wo; off = p.tr_fwd[layer];
  } else {
    if (layer < 0 || layer > nl || !m->tr_bwd_valid) return FDG_ERR_INVALID_ARG;
    if (layer == nl) {
      if (p.is_top) return FDG_ERR_INVALID_ARG;
      c = p.out_c; h = p.out_h; w = p.out_w;
    } else {
      if (layer == 0 && p.d.is_bottom) return FDG_ERR_INVALID_ARG;
      const LayerPlan& L = p.L[layer];
      c = L.c_in; h = L.Hi; w = L.Wi;
      g = m->tr_gated[layer];
    }
    off = p.tr_bwd[layer];
  }
  if (shape) { shape[0] = N; shape[1] = c; shape[2] = h; shape[3] = w; }
  if (gated) *gated = g;
  if (count != (size_t)N * c * h * w) return FDG_ERR_INVALID_ARG;
  if (fdg_status st = sync_streams(m); st != FDG_OK) return st;
  return read_nhwc(m->trace + off, false, N, c, round8(c), h * w, host_dst);
}

fdg_status fdg_profile_enable(fdg_module* m, int enable) {
  if (!m) return FDG_ERR_INVALID_ARG;
  FDG_TRY(hipStreamSynchronize(m->last_stream));
  if (m->fwd_stream != m->last_stream) FDG_TRY(hipStreamSynchronize(m->fwd_stream));
  m->prof.reset();
  m->prof.on = enable != 0;
  return FDG_OK;
}

fdg_status fdg_overlap_enable(fdg_module* m, int enable) {
  if (!m) return FDG_ERR_INVALID_ARG;
  if (fdg_status st = sync_streams(m); st != FDG_OK) return st;
  if (m->side.stream) FDG_TRY(hipStreamSynchronize(m->side.stream));
  m->side.wanted = enable != 0;
  return FDG_OK;
}

fdg_status fdg_profile_read(fdg_module* m, fdg_profile_entry* out, int32_t capacity, int32_t* count) {
  if (!m || !count || (capacity > 0 && !out)) return FDG_ERR_INVALID_ARG;
  FDG_TRY(hipStreamSynchronize(m->last_stream));
  if (m->fwd_stream != m->last_stream) FDG_TRY(hipStreamSynchronize(m->fwd_stream));
  // one entry per (class, kernel and layer shape)
  std::vector<fdg_profile_entry> acc;
  for (const ProfRecord& r : m->prof.recs) {
    float ms = 0.f;
    FDG_TRY(hipEventElapsedTime(&ms, r.e0, r.e1));
    size_t i = 0;
    for (; i < acc.size(); ++i)
      if (strcmp(acc[i].name, kProfNames[r.cls]) == 0 && strcmp(acc[i].kernel, r.kernel) == 0) break;
    if (i == acc.size()) {
      acc.push_back(fdg_profile_entry{});
      snprintf(acc[i].name, sizeof(acc[i].name), "%s", kProfNames[r.cls]);
      snprintf(acc[i].kernel, sizeof(acc[i].kernel), "%s", r.kernel);
    }
    acc[i].calls += 1;
    acc[i].total_ms += ms;
    acc[i].flops += r.flops;
    acc[i].bytes += r.bytes;
  }
  int n = 0;
  for (const fdg_profile_entry& e : acc) {
    if (n < capacity) out[n] = e;
    ++n;
  }
  *count = n;
  return m->prof.overflow ? FDG_ERR_UNSUPPORTED : FDG_OK;
}

const char* fdg_status_string(fdg_status s) {
  switch (s) {
    case FDG_OK: return "ok";
    case FDG_ERR_INVALID_ARG: return "invalid argument";
    case FDG_ERR_UNSUPPORTED: return "unsupported layer shape";
    case FDG_ERR_WORKSPACE_TOO_SMALL: return "workspace too small or misaligned";
    case FDG_ERR_QUEUE_FULL: return "history queue full";
    case FDG_ERR_QUEUE_EMPTY: return "history queue empty";
    case FDG_ERR_NO_GRAD: return "no gradient since the last update";
    case FDG_ERR_HIP: return "HIP error";
  }
  return "unknown status";
}

}  // extern "C"
