// Internal launch interface between the host-side module object and the gfx950 kernels.
// Everything here works on device pointers; activations are NHWC, bf16 for MFMA operands and
// fp32 for the residual stream.  Nothing in this header is part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace fdg {

typedef __bf16 bf16_t;

// One filter tap of a gather-form convolution: input pixel = (oh*in_stride + dh, ow*in_stride + dw),
// weight k-offset = kofs * Ci.  Packed as (dh+8) | (dw+8) << 8 | kofs << 16.
__host__ __device__ static inline int pack_tap(int dh, int dw, int kofs) { return (dh + 8) | ((dw + 8) << 8) | (kofs << 16); }

// out[pix(m), c] = sum_{tap, k} in[pixel(m, tap), k] * w[c, kofs(tap)*Ci + k]  (+ addend)
// Rows m enumerate an output grid [N, OH, OW]; the output pixel of row (n, oh, ow) is
// (n, oh*out_stride + ooh, ow*out_stride + oow) in a tensor [N, OHf, OWf, Co].  Forward convolution,
// stride-1 data gradient and each parity class of a stride-2 data gradient are all of this form.
// Per-channel sums (batch-norm statistics, the two sums of a batch-norm backward) are taken over many workgroups.
// Each workgroup adds ITS fp32 partial sum, reduced in a fixed order inside the workgroup, into the total -- and the
// total is kept EXACTLY, in 64-bit fixed point: the partial s is split into hi = rint(s * 2^11) and
// lo = rint((s - hi * 2^-11) * 2^62) (exact for 2^-39 <= |s| < 2^39; smaller partials are rounded to 2^-62) and both
// words are added with integer atomics.  Integer addition is associative, so the total does not depend on the order in
// which workgroups arrive: two runs on the same input give the same bits, which no fp32 atomic sum does.  Up to 4096
// partials fit.  A partial of 2^39 (5.5e11) or more -- a network that is blowing up -- goes to a third word, a double
// added with a floating-point atomic: still a sum, no longer order independent.
// A sums array for C channels is stat_t[3][2][C] (word, which of the two sums, channel), zero before the producers run;
// value = big + hi * 2^-11 + lo * 2^-62.
// Hundreds of workgroups onto one cache line serialise at the memory side (6 - 11 us per launch for the narrow
// layers), so an array may exist in kStatReplicas copies, rep_stride stat_t elements apart: workgroup b adds into copy
// b % kStatReplicas and whoever reads the sums adds the copies (integers again).  rep_stride = 0: a single copy.
constexpr int kStatReplicas = 8;
typedef long long stat_t;
constexpr int kStatWords = 3;                                   // stat_t per sum: hi, lo, big (a double)
inline size_t stat_elems(size_t channels) { return 2 * channels * kStatWords; }   // stat_t of a sums array

#if defined(__HIPCC__)
// total[which][c] += s, for the sums array of C channels starting at `stats`
__device__ __forceinline__ void stat_add(stat_t* stats, int C, int which, int c, float s) {
  const double d = (double)s;
  stat_t* p = stats + (size_t)which * C + c;
  if (fabs(d) < 0x1p39) {
    const double h = rint(d * 0x1p11);
    const long long hi = (long long)h, lo = (long long)rint((d - h * 0x1p-11) * 0x1p62);
    atomicAdd(reinterpret_cast<unsigned long long*>(p), (unsigned long long)hi);
    atomicAdd(reinterpret_cast<unsigned long long*>(p + 2 * (size_t)C), (unsigned long long)lo);
  } else {
    atomicAdd(reinterpret_cast<double*>(p + 4 * (size_t)C), d);
  }
}
__device__ __forceinline__ double stat_value(long long hi, long long lo, long long big) {
  return __builtin_bit_cast(double, big) + ((double)hi * 0x1p-11 + (double)lo * 0x1p-62);
}
// the total of channel c, copies added
__device__ __forceinline__ double stat_load(const stat_t* stats, int C, int which, int c, int rep_stride) {
  const stat_t* p = stats + (size_t)which * C + c;
  long long hi = p[0], lo = p[2 * (size_t)C];
  double big = __builtin_bit_cast(double, p[4 * (size_t)C]);
  if (rep_stride > 0)
    for (int r = 1; r < kStatReplicas; ++r) {
      const stat_t* q = p + (size_t)r * rep_stride;
      hi += q[0]; lo += q[2 * (size_t)C];
      big += __builtin_bit_cast(double, q[4 * (size_t)C]);
    }
  return stat_value(hi, lo, __builtin_bit_cast(long long, big));
}
#endif

struct GatherConvArgs {
  const bf16_t* in;      // [N, Hi, Wi, Ci] bf16, Ci % 8 == 0
  const bf16_t* w;       // [w_rows, Kw] bf16, k contiguous
  const float* addend;   // optional fp32 tensor indexed like the output
  const bf16_t* addmask; // optional: addend counts only where this bf16 tensor (output indexing) is > 0
  float* out_f32;        // optional fp32 output
  bf16_t* out_b16;       // optional bf16 output
  stat_t* stats;         // optional sums array of Co channels: += per-channel sum and sum of squares of the bf16-rounded output
  // Data gradient that ends in the ReLU and batch norm it back-propagates into next (wide kernels only):
  const bf16_t* gate;    // optional (output indexing): the output is kept where gate > 0 and is zero elsewhere
  const bf16_t* bnx;     // optional (output indexing), with stats: stats[Co + c] += sum of output * bnx instead of
                         // the squares -- with stats[c] the two sums the batch-norm backward needs
  int stats_rep_stride;  // stat_t elements between the copies of stats (0: one copy)
  int stats_f32;         // with bnx, narrow / generic output stage: the sums are of the fp32 values, not of the bf16 output
  int N, Hi, Wi, Ci;
  int OH, OW, in_stride;
  int OHf, OWf, out_stride, ooh, oow;
  int Co;                // output channel pitch, % 4 == 0
  int w_rows;            // weight rows that exist (<= Co); the other output channels are zero
  int Kw;                // weight row pitch in elements
  int ntaps;
  int tap[9];
  // Several output geometries in one launch (the four parity classes of a stride-2 data gradient), wide
  // kernel only.  nclass <= 1: the single geometry above.  Otherwise class i owns the tiles cls_start[i] ..
  // cls_start[i+1]-1 and replaces OH, OW, ooh, oow, ntaps and the tap list (a class may have no tap at all:
  // its outputs are the addend, or zero).
  int nclass;
  int cls_start[5];
  int cOH[4], cOW[4], cooh[4], coow[4], cntaps[4];
  int ctap[4][4];
  // A second contraction into the same outputs, wide pipelined kernel with nclass > 1 only: after its own taps, class
  // cls2 also adds in2[pixel at tap (0, 0), k] * w2[c, k] over the Ci channels of in2 [N, Hi, Wi, Ci] (indexed like
  // `in`), w2 [w_rows, Kw2].  That is the data gradient of a 1x1 stride-2 projection next to the 3x3 stride-2
  // convolution that reads the same input.  in2 == nullptr: none.
  const bf16_t* in2;
  const bf16_t* w2;
  int Kw2, cls2;
  // Input transform, narrow kernel only (tr_mode != 0; `in` is not read): the convolution's input is
  //   y = act(A[c] * p + B[c] * q + C[c]), rounded to bf16,
  // worked out in LDS from the raw patches of p (tr_p: bf16, or fp32 with tr_p_f32) and q (tr_q, bf16, mode 2 only),
  // both [N, Hi, Wi, Ci], with per-channel coefficients from batch-norm sums; every workgroup also writes the y of its
  // own pixels to tr_out (bf16 [N, Hi, Wi, Ci]), which is then what a batch-norm pass of its own would have left.
  //   mode 1: forward batch norm + ReLU of p.  A = gamma * invstd, B = 0, C = beta - mean * A from tr_sums (sums of p);
  //           act = max(., 0); tr_run_mean / tr_run_var (optional) take one running-statistics step.  With tr_q given, tr_q
  //           is an fp32 residual [N, Hi, Wi, Ci] added before the ReLU (the end of a basic block); tr_out_f32 (optional)
  //           receives y in fp32 as well (the residual stream).
  //   mode 2: backward of the batch norm whose input was q, applied to the gated gradient p.  A, B, C from tr_sums
  //           (forward sums of q) and tr_bsums (sum p, sum p*q) as in BnBwdArgs with raw_sums; no act; tr_dgamma and
  //           tr_dbeta are written.
  int tr_mode, tr_p_f32;
  const void* tr_p;
  const void* tr_q;
  bf16_t* tr_out;
  float* tr_out_f32;
  const stat_t* tr_sums;
  const stat_t* tr_bsums;
  const float* tr_gamma;
  const float* tr_beta;
  float* tr_run_mean;
  float* tr_run_var;
  float* tr_dgamma;
  float* tr_dbeta;
  float tr_eps, tr_momentum;
  int tr_rep_stride;     // stat_t elements between the copies of tr_sums and tr_bsums (0: one copy)
};
// whether the narrow kernel takes this layer with an input transform (a geometry conv_narrow_applies accepts, real input
// channels, one tile per workgroup, LDS for the raw patches)
bool conv_narrow_transforms(const GatherConvArgs& a, int var);   // var: 0 mode 1; 1 / 2 mode 2 with bf16 / fp32 p; 3 mode 1 with a residual
hipError_t launch_conv_gather(const GatherConvArgs& a, hipStream_t s);
// narrow layers (16 / 32 / 64 channels in and out, 3x3, unit stride): whole patch and whole filter on chip
bool conv_narrow_applies(const GatherConvArgs& a);
hipError_t launch_conv_narrow(const GatherConvArgs& a, hipStream_t s);

// dw[co, tap, ci] += sum_m dy[m, co] * x[pixel(m, tap), ci]   (fp32 atomics; dw must be pre-zeroed)
struct WgradArgs {
  const bf16_t* dy;  // [N, OH, OW, Co] bf16, Co % 8 == 0
  const bf16_t* x;   // [N, Hi, Wi, Cx] bf16, Cx % 8 == 0
  float* dw;         // [Co, ntaps, Ci] fp32
  int N, OH, OW, Co;
  int Hi, Wi, Cx, Ci; // Ci = real input channels (<= Cx)
  int stride;
  int ntaps;
  int tap[9];        // pack_tap(dh, dw, 0)
  float* scratch;    // optional device scratch for split partial sums (see conv_wgrad_scratch_bytes)
  size_t scratch_bytes;
  int overwrite;     // 1: dw = sum (no need to zero dw first);  0: dw += sum
  // narrow kernel only: the slices of an EARLIER narrow weight gradient on the same stream, added up by this launch
  // while its own loads are in flight (see WgradDebt); prev_slices == 0: none
  float* prev_dw;
  const float* prev_partial;
  int prev_n4, prev_slices, prev_overwrite;
  size_t prev_stride4;
  int defer_reduce;  // narrow kernel only: leave this launch's slices in scratch, the caller has them added up later
};
// The narrow weight-gradient kernel leaves one slice of partial sums per workgroup, and adding them up is a small launch
// of its own -- unless the NEXT narrow weight gradient on the same stream does it while its own loads are in flight.  A
// WgradDebt carries that from one conv_wgrad call to the next: a call that runs the narrow kernel first settles the debt it
// is handed inside its launch and then leaves its own (its scratch must be another buffer than the one still owed); any
// other call, and conv_wgrad_settle, launch the plain reduction for what is owed.  Same sums in the same order either way.
struct WgradDebt {
  float* dw = nullptr;
  const float* partial = nullptr;
  int n4 = 0, slices = 0, overwrite = 0;
  size_t stride4 = 0;
};
hipError_t conv_wgrad_settle(WgradDebt& debt, hipStream_t s);
hipError_t launch_conv_wgrad(const WgradArgs& a, hipStream_t s);
// narrow layers (16 / 32 / 64 channels in and out, 3x3, unit stride): all nine taps of a range of image rows per
// workgroup, per-workgroup slices in a.scratch added by a second kernel
bool conv_wgrad_narrow_applies(const WgradArgs& a);
size_t conv_wgrad_narrow_scratch_bytes(const WgradArgs& a);
hipError_t launch_conv_wgrad_narrow(const WgradArgs& a, hipStream_t s);
int conv_wgrad_narrow_slices(const WgradArgs& a);   // slices (workgroups) that launch writes; 0 where it does not apply
// dw (+)= sum of `slices` slices of n4 float4 each, stride4 float4 apart, in the narrow kernel's fixed order
hipError_t launch_wgrad_slices_reduce(float* dw, const float* partial, int n4, int slices, size_t stride4, int overwrite, hipStream_t s);

// One convolution of a module: 3x3 with padding 1 (T = 9) or 1x1 with padding 0 (T = 1), stride 1 or 2.
// Activations carry Cip = Ci rounded up to 8 channels (the padding channels hold zeros).
struct ConvShape {
  int N, Hi, Wi, Ci, Cip, Co, T, stride;
  int Ho() const { return (Hi - 1) / stride + 1; }
  int Wo() const { return (Wi - 1) / stride + 1; }
};
// y[N,Ho,Wo,Co] = conv(x[N,Hi,Wi,Cip], w[Co][T][Cip]) (+ addend)
// stats (optional, [2*Co], pre-zeroed): += per-channel sum and sum of squares of the bf16-rounded result,
// i.e. the batch-norm statistics of the tensor just produced
hipError_t conv_forward(const ConvShape& c, const bf16_t* x, const bf16_t* w, const float* addend, float* out_f32,
                        bf16_t* out_b16, stat_t* stats, hipStream_t s, int stats_rep_stride = 0);
// The same convolution of relu(batchnorm(x_raw)) with the batch-norm pass done on the patch in LDS (narrow layers, see
// GatherConvArgs::tr_mode = 1): act_out receives relu(batchnorm(x_raw)) in bf16 as a pass of its own would have written
// it; run_mean / run_var (optional) take one running-statistics step.  conv_forward_bn_applies says where.
struct ConvInputBn {
  const float* res_f32;  // optional [N, Hi, Wi, Cip]: added to the normalised value before the ReLU
  float* act_out_f32;    // optional [N, Hi, Wi, Cip]: the activation in fp32 as well
  const bf16_t* x_raw;   // [N, Hi, Wi, Cip] the batch norm's input
  const stat_t* sums;    // its sums array (sum, sum of squares), complete
  const float* gamma;
  const float* beta;
  bf16_t* act_out;       // [N, Hi, Wi, Cip]
  float* run_mean;
  float* run_var;
  float eps, momentum;
  int rep_stride;        // stat_t elements between the copies of sums (0: one copy)
};
bool conv_forward_bn_applies(const ConvShape& c, bool with_residual = false);
hipError_t conv_forward_bn(const ConvShape& c, const ConvInputBn& bn, const bf16_t* w, const float* addend, float* out_f32,
                           bf16_t* out_b16, stat_t* stats, hipStream_t s, int stats_rep_stride = 0);
// A data gradient whose input dy is the apply half of a batch-norm backward, done on the patch in LDS (narrow layers,
// see GatherConvArgs::tr_mode = 2): dy = gamma*invstd*(g - sum g / M - xhat * sum(g xhat) / M) for the gated gradient g at
// the batch norm's output and its input x, with the sums of g and g*x already in bsums (as a gated data gradient leaves
// them).  dy_out receives dy in bf16 (what the weight gradient of the same convolution reads), dgamma / dbeta are
// written.  Passed to the conv_dgrad_* calls below in place of their dy argument.
struct ConvInputBnBwd {
  const void* g;         // [N, Ho, Wo, Co] gated gradient, bf16 or fp32 (g_is_f32)
  int g_is_f32;
  const bf16_t* x;       // [N, Ho, Wo, Co] the batch norm's input
  const stat_t* sums;    // forward sums of x
  const stat_t* bsums;   // sum g, sum g*x
  const float* gamma;
  float* dgamma;
  float* dbeta;
  bf16_t* dy_out;        // [N, Ho, Wo, Co]
  float eps;
  int rep_stride;        // stat_t elements between the copies of sums and of bsums (0: one copy)
};
// whether the data gradient of c takes such an input (unit stride 3x3 narrow layer, one tile per workgroup)
bool conv_dgrad_bn_applies(const ConvShape& c, bool g_is_f32);
// conv_dgrad (gate, bnx, gsums all nullptr), conv_dgrad_gated (sums of the bf16 values) or conv_dgrad_feeding_next
// (sums_of_f32: of the fp32 values, out_f32 required) with that input
hipError_t conv_dgrad_after_bn(const ConvShape& c, const ConvInputBnBwd& bn, const bf16_t* wt, const float* addend,
                               const bf16_t* addmask, const bf16_t* gate, const bf16_t* bnx, stat_t* gsums, bool sums_of_f32,
                               float* out_f32, bf16_t* out_b16, hipStream_t s, int gsums_rep_stride = 0);
// dx[N,Hi,Wi,Cip] = conv^T(dy[N,Ho,Wo,Co], wt[Cip][T][Co]) (+ addend, optionally only where addmask > 0)
hipError_t conv_dgrad(const ConvShape& c, const bf16_t* dy, const bf16_t* wt, const float* addend,
                      const bf16_t* addmask, float* out_f32, bf16_t* out_b16, hipStream_t s);
// The same, ending in the gate of the ReLU below and the two sums of the batch norm below it:
//   dx = gate > 0 ? dgrad + addend : 0;  gsums[c] += sum bf16(dx[.., c]);  gsums[Cip + c] += sum bf16(dx[.., c]) * bnx[.., c].
// Only where conv_dgrad_gates(c) (the wide kernels); hipErrorInvalidValue otherwise.
// The narrow kernel runs this data gradient, so its fp32 result can be gated by the output of the layer below and
// carry the two sums of that layer's last batch norm (conv_dgrad_feeding_next).
bool conv_dgrad_feeds_next(const ConvShape& c);
hipError_t conv_dgrad_feeding_next(const ConvShape& c, const bf16_t* dy, const bf16_t* wt, const float* addend,
                                   const bf16_t* addmask, const bf16_t* gate, const bf16_t* bnx, stat_t* gsums, float* out_f32,
                                   bf16_t* out_b16, hipStream_t s, int gsums_rep_stride = 0);
bool conv_dgrad_gates(const ConvShape& c);
// conv_dgrad_gated of c (3x3, stride 2) with the data gradient of the 1x1 stride-2 projection cp beside it (same input
// tensor, same output grid) added before the gate, in one launch:
//   dx = gate > 0 ? dgrad(c; dy, wt) + dgrad(cp; dy2, wt2) : 0,  sums as conv_dgrad_gated;
// with gate, bnx and gsums all nullptr the plain sum of the two data gradients.
// Only where conv_dgrad_pair_applies (wide layers); hipErrorInvalidValue otherwise.
bool conv_dgrad_pair_applies(const ConvShape& c, const ConvShape& cp);
hipError_t conv_dgrad_gated_pair(const ConvShape& c, const bf16_t* dy, const bf16_t* wt, const ConvShape& cp, const bf16_t* dy2,
                                 const bf16_t* wt2, const bf16_t* gate, const bf16_t* bnx, stat_t* gsums, float* out_f32,
                                 bf16_t* out_b16, hipStream_t s, int gsums_rep_stride = 0);
hipError_t conv_dgrad_gated(const ConvShape& c, const bf16_t* dy, const bf16_t* wt, const float* addend, const bf16_t* gate,
                            const bf16_t* bnx, stat_t* gsums, float* out_f32, bf16_t* out_b16, hipStream_t s,
                            int gsums_rep_stride = 0);
// dw[Co][T][Ci] (+)= sum over pixels of dy * x.  overwrite = false: accumulated into dw (fp32 atomics where the
// pixel dimension is split), dw zeroed by the caller;  overwrite = true: dw is written, whatever it held.
// scratch (optional): device memory for the partial sums of the pixel splits; without it they are added
// with atomics.  conv_wgrad_scratch_bytes gives the useful size for a shape (0: the shape never uses it).
hipError_t conv_wgrad(const ConvShape& c, const bf16_t* x, const bf16_t* dy, float* dw, float* scratch,
                      size_t scratch_bytes, bool overwrite, hipStream_t s, WgradDebt* debt = nullptr);
// whether conv_wgrad of this shape runs the narrow kernel (and so takes part in a WgradDebt)
bool conv_wgrad_defers(const ConvShape& c);
size_t conv_wgrad_scratch_bytes(const ConvShape& c);

// Batch-norm pieces on [M, C] NHWC tensors (C % 8 == 0, C <= 2048).
// sums = a sums array of C channels (sum, sum of squares), pre-zeroed; accumulated exactly (see stat_t).
hipError_t launch_bn_stats(const bf16_t* x, stat_t* sums, int M, int C, hipStream_t s);

struct BnApplyArgs {
  const bf16_t* x;       // [M, C]
  const stat_t* sums;    // sums array of x
  const float* gamma;    // [C]
  const float* beta;     // [C]
  const float* res_f32;  // optional fp32 residual [M, C]
  const bf16_t* x2;      // optional second normalised operand (projection shortcut) [M, C]
  const stat_t* sums2;   // its sums, gamma, beta
  const float* gamma2;
  const float* beta2;
  float* out_f32;        // optional
  bf16_t* out_b16;       // optional
  float* run_mean;       // optional running statistics of x (updated by block 0)
  float* run_var;
  float* run_mean2;      // optional running statistics of x2
  float* run_var2;
  int M, C;
  float eps, momentum;
  int relu;              // 0: none, 1: max(y, 0), 2: min(max(y, 0), 6)
  int rep_stride;        // stat_t elements between the copies of sums and of sums2 (0: one copy)
};
hipError_t launch_bn_apply(const BnApplyArgs& a, hipStream_t s);

// Backward: g = dy * [mask > 0];  bsums = sums array [sum g | sum g*xhat] (pre-zeroed)
struct BnBwdArgs {
  const void* dy;        // [M, C] fp32 or bf16 (dy_is_f32)
  int dy_is_f32;
  const bf16_t* mask;    // [M, C] ReLU output (or pre-activation sign carrier); required
  const bf16_t* x;       // [M, C] the BN input saved by the forward
  const stat_t* sums;    // forward sums of x
  const float* gamma;    // snapshot gamma
  stat_t* bsums;         // sums array of C channels
  const float* addend;   // optional fp32 [M, C] added to dx (apply only)
  float* out_f32;        // optional dx
  bf16_t* out_b16;       // optional dx
  float* dgamma;         // [C] written by apply
  float* dbeta;          // [C]
  int M, C;
  float eps;
  float gate_hi;         // > 0: the gate is also closed where mask >= gate_hi (ReLU6: 6); 0: open above
  int dy_gated;          // dy needs no gate: it is already zero where the gate is closed, or there is none (mask is not read)
  int raw_sums;          // apply only: bsums holds sum g and sum g*x (not g*xhat), as a gated data gradient leaves them
  int rep_stride;        // stat_t elements between the copies of sums (0: one copy)
  int brep_stride;       // apply only: stat_t elements between the copies of bsums (0: one copy); the reduce pass adds into copy 0
};
hipError_t launch_bn_bwd_reduce(const BnBwdArgs& a, hipStream_t s);
hipError_t launch_bn_bwd_apply(const BnBwdArgs& a, hipStream_t s);

// Layout changes at the module boundary.  scale multiplies every element (beta of Eq. 15).
hipError_t launch_nchw_to_nhwc(const float* src, float* dst_f32, bf16_t* dst_b16, int N, int C, int HW, int Cp,
                               float scale, hipStream_t s);
hipError_t launch_nhwc_to_nchw(const float* src, float* dst, int N, int C, int HW, int Cp, hipStream_t s);

// Head: pooled[n,c] = mean_hw o[n,hw,c];  logits = pooled W^T + b;  softmax cross-entropy.
hipError_t launch_avgpool(const bf16_t* o, float* pooled, int N, int HW, int C, hipStream_t s);
hipError_t launch_fc_fwd(const float* pooled, const float* W, const float* b, float* logits, int N, int C, int J,
                         hipStream_t s);
// y[0] = mean loss, y[1 + n*J + j] = logits; dl[n,j] = (softmax - onehot)/N
hipError_t launch_softmax_ce(const float* logits, const int32_t* labels, float* y, float* dl, int N, int J,
                             hipStream_t s);
hipError_t launch_fc_bwd(const float* pooled, const float* W, const float* dl, float* dW, float* db, float* dp,
                         int N, int C, int J, hipStream_t s);
// g[n,hw,c] = dp[n,c]/HW
hipError_t launch_pool_bwd(const float* dp, float* g_f32, bf16_t* g_b16, int N, int HW, int C, hipStream_t s);

// theta, v, g flat fp32 (count % 4 == 0):  g' = g + wd*theta;  v = mu*v + g';  theta -= lr*v
hipError_t launch_sgd(float* theta, float* v, const float* g, size_t count, float lr, float mu, float wd,
                      hipStream_t s);

// bf16 copies of every convolution weight of the module, one launch.  Entry i describes one conv.
struct WeightEmitEntry {
  uint32_t src_off;    // fp32 master [Co][T][Ci], element offset in the parameter arena
  uint32_t w_off;      // bf16 [Co][T][Cip] element offset in the slot's weight arena (forward / wgrad layout)
  uint32_t wt_off;     // bf16 [Cip][T][Co] element offset (data-gradient layout)
  int32_t Co, T, Ci, Cip;
  uint32_t block_start; // first block of this conv in the launch
};
// blocks the snapshot kernel needs for one convolution (64 x 64 tiles per tap)
inline uint32_t emit_blocks_for(int Co, int Cip, int T) { return (uint32_t)(((Co + 63) / 64) * ((Cip + 63) / 64) * T); }
hipError_t launch_emit_weights(const float* params, bf16_t* warena, const WeightEmitEntry* table_dev, int nconv,
                               int total_blocks, hipStream_t s);

// launch_sgd over the whole parameter arena and the snapshot in one pass: the updated convolution weights are also
// written as bf16 into warena (both layouts, as launch_emit_weights) and the updated small parameters
// [small_off, small_off + small_count) as fp32 into small_snap.  conv_blocks = the blocks launch_emit_weights would take.
hipError_t launch_sgd_emit(float* params, float* mom, const float* grads, bf16_t* warena, float* small_snap,
                           const WeightEmitEntry* table_dev, int nconv, int conv_blocks, size_t small_off, size_t small_count,
                           float lr, float mu, float wd, hipStream_t s);

// ---- layers of the Tiny-ImageNet networks (layer_kernels.hip) ----
// col[m, kh, kw8, c8] of a 7x7 stride-2 padding-3 convolution over x8 [N, H, W, 8]: 448 bf16 per output pixel m = (n, oh, ow),
// the column kw = 7 and everything outside the image zero
hipError_t launch_im2col7(const bf16_t* x8, bf16_t* col, int N, int H, int W, hipStream_t s);
// 3x3 max-pool, stride 2, padding 1 over x [N, H, W, C] (C % 8 == 0); backward: dy fp32 [N, Ho, Wo, C] to the first maximum
// of each window in scan order, dx fp32 [N, H, W, C] written everywhere
hipError_t launch_maxpool3s2(const bf16_t* x, float* y_f32, bf16_t* y_b16, int N, int H, int W, int C, hipStream_t s);
hipError_t launch_maxpool3s2_bwd(const bf16_t* x, const float* dy, float* dx, int N, int H, int W, int C, hipStream_t s);
// depthwise 3x3 convolution, padding 1, stride 1 or 2; wt bf16 [9][C] (tap-major), dw fp32 [C][9]
hipError_t launch_dwconv3_fwd(const bf16_t* x, const bf16_t* wt, bf16_t* y, int N, int H, int W, int C, int stride, hipStream_t s);
// dx (bf16) and / or dx_f32 (fp32), at least one
hipError_t launch_dwconv3_dgrad(const bf16_t* dy, const bf16_t* wt, bf16_t* dx, int N, int H, int W, int C, int stride, hipStream_t s,
                                float* dx_f32 = nullptr);
size_t dwconv3_wgrad_scratch_bytes(int N, int H, int W, int C, int stride);
hipError_t launch_dwconv3_wgrad(const bf16_t* x, const bf16_t* dy, float* dw, float* scratch, size_t scratch_bytes, int N, int H, int W,
                                int C, int stride, hipStream_t s);

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);  // bytes % 16 == 0

// Name of the convolution kernel the calling thread launched last (as a profiler prints it), for the
// per-kernel timing records of the module; a literal with static lifetime.
void note_kernel(const char* name);
const char* last_kernel();
hipError_t launch_fill_f32(float* p, size_t count, float v, hipStream_t s);

}  // namespace fdg
