/*
 * fdg.h -- C ABI of one FDG module worker on one MI355X (gfx950).
 *
 * FDG (fully decoupled learning with delayed gradients, arXiv 1906.09108) splits a network into K
 * modules.  Section III-A of the paper states what one module does per iteration:
 *   forward   : run the module's layers on the newest input and keep what the later backward needs
 *               (the "saved computation graph" of Fig. 1(b));
 *   backward  : resume back-propagation on an OLDER batch with the gradient received from the
 *               module above, every factor evaluated at that older batch (Eq. 10), after the
 *               gradient was multiplied by the shrinking factor beta (Eq. 15);
 *   update    : apply the resulting delayed gradient to the CURRENT weights (Eq. 11 / Eq. 12).
 * This library is that worker.  A module is a list of ResNet-style layers; the history of saved
 * forwards is a FIFO ring of delay+1 contexts.
 *
 * Conventions that hold for every entry point
 *   - Pointers named *_dev are DEVICE pointers (HBM); pointers named host_* are HOST pointers.
 *   - Boundary tensors are fp32, NCHW, dense.
 *   - The caller owns every device buffer, including the single workspace arena given at create.
 *     The library never allocates or frees device memory; fdg_destroy frees only the host object.
 *   - `hip_stream` is a hipStream_t cast to void* (NULL = the null stream).  All device work of a
 *     call is enqueued on it and the call returns without waiting, except the host accessors
 *     (fdg_get_*, fdg_set_params) which synchronise that module's last used stream.
 *   - Errors are status codes; nothing throws or aborts.  Argument and queue errors are detected
 *     before anything is enqueued, so a failed call leaves the module unchanged.
 *   - A module object is not thread safe; calls on one module must be serialised by the caller.
 *   - Two streams.  The forward of the newest batch and the delayed backward of the oldest one touch different
 *     contexts (Fig. 1(b)) -- that independence is what the method is about -- and share no temporary when the
 *     module has delay >= 1 and the stored form (FDG_SAVE_ACTIVATIONS).  The host calls stay serialised, but such a
 *     module's fdg_forward and fdg_backward_delayed may be given DIFFERENT streams and then overlap on the GPU.  The
 *     caller orders, with events: fdg_update after that backward (same stream is enough) AND after the forward
 *     (the forward snapshots the weights the update moves); the next fdg_forward after that update; a
 *     fdg_backward_delayed after the forward whose context it pops (only an issue at delay-many steps' distance).
 *     With delay 0, or FDG_SAVE_INPUT_AND_REPLAY, give all calls of a step one stream (or order them fully).
 *   - Stream capture.  Every entry point may be recorded into a HIP graph (hipStreamBeginCapture on its stream): the
 *     library allocates nothing, clears memory with kernels and forks / joins its own second stream with events.  A
 *     step on ONE stream records as it is.  Recording the forward on one stream and the backward side (backward,
 *     update) on another inside the SAME capture is not supported: the call that would put the second stream of a
 *     module into a capture returns FDG_ERR_UNSUPPORTED and enqueues nothing.  Record the two streams' work as two
 *     graphs, or use one stream under capture.
 */
#ifndef FDG_H_
#define FDG_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fdg_module fdg_module; /* opaque, host memory, library-owned */

typedef enum {
  FDG_OK = 0,
  FDG_ERR_INVALID_ARG = 1,         /* NULL where a pointer is required, bad descriptor, bad count */
  FDG_ERR_UNSUPPORTED = 2,         /* a layer shape this build has no kernel for; two streams of a module in one capture */
  FDG_ERR_WORKSPACE_TOO_SMALL = 3, /* bytes < fdg_module_workspace_bytes(desc) or misaligned */
  FDG_ERR_QUEUE_FULL = 4,          /* forward with delay+1 contexts outstanding */
  FDG_ERR_QUEUE_EMPTY = 5,         /* backward with no context outstanding */
  FDG_ERR_NO_GRAD = 6,             /* update with no backward since the last update */
  FDG_ERR_HIP = 7                  /* a HIP call or kernel launch failed */
} fdg_status;

/* Layer kinds.  All convolutions are bias-free.  BN = training-mode batch normalisation.
 *   STEM_CONV_BN_RELU : conv3x3(c_in->c_out, stride) -> BN -> ReLU
 *   BASIC_POSTACT     : conv3x3(stride) -> BN -> ReLU -> conv3x3 -> BN -> (+shortcut) -> ReLU,
 *                       shortcut = identity, or conv1x1(stride)+BN when stride!=1 or c_in!=c_out
 *   BASIC_PREACT      : o=ReLU(BN(x)); conv3x3(o,stride) -> BN -> ReLU -> conv3x3, + shortcut,
 *                       shortcut = x, or conv1x1(o, stride) when stride!=1 or c_in!=c_out
 *   HEAD_POSTACT      : global average pool -> FC(c_in->num_classes)+bias -> softmax cross-entropy
 *   HEAD_PREACT       : BN -> ReLU -> the same head
 *   BOTTLENECK_POSTACT: conv1x1(c_in->c_out/4) -> BN -> ReLU -> conv3x3(c_out/4->c_out/4, stride) -> BN -> ReLU ->
 *                       conv1x1(c_out/4->c_out) -> BN -> (+shortcut) -> ReLU, shortcut as in BASIC_POSTACT; the
 *                       block of ResNet-101 (Section V-C, Table VII); c_out must be a multiple of 32
 *   STEM_POOL         : conv7x7(c_in->c_out, stride 2, padding 3) -> BN -> ReLU -> max-pool 3x3 (stride 2, padding 1): the
 *                       ImageNet stem of ResNet-18 / ResNet-101 (Table V, Table VII).  `stride` must be 4 (the two halvings);
 *                       c_in <= 8; only as the first layer of a bottom module (it has no input gradient: it is the first
 *                       layer of its network), else FDG_ERR_UNSUPPORTED.  Parameters: conv.w [c_out, c_in, 7, 7], gamma, beta
 *   INVERTED_RESIDUAL : conv1x1(c_in->6 c_in) -> BN -> ReLU6 -> depthwise conv3x3(stride) -> BN -> ReLU6 ->
 *                       conv1x1(6 c_in->c_out) -> BN, plus the input when stride == 1 and c_in == c_out: the block of
 *                       MobileNet-v2 (Table V) with its expansion factor 6.  Parameters: conv1.w [6 c_in, c_in, 1, 1], bn1,
 *                       conv2.w [6 c_in, 1, 3, 3], bn2, conv3.w [c_out, 6 c_in, 1, 1], bn3 (gamma, beta each)
 * A head, if present, must be the last layer; the module is then a TOP module (Section III-B:
 * its gradient is not shrunk and it needs no gradient from above).                              */
typedef enum {
  FDG_STEM_CONV_BN_RELU = 0,
  FDG_BASIC_POSTACT = 1,
  FDG_BASIC_PREACT = 2,
  FDG_HEAD_POSTACT = 3,
  FDG_HEAD_PREACT = 4,
  FDG_BOTTLENECK_POSTACT = 5,
  FDG_STEM_POOL = 6,
  FDG_INVERTED_RESIDUAL = 7
} fdg_layer_kind;

typedef struct {
  int32_t kind;   /* fdg_layer_kind */
  int32_t c_in;   /* input channels; must equal the previous layer's c_out */
  int32_t c_out;  /* output channels (heads: ignored, num_classes is used) */
  int32_t stride; /* 1 or 2 (heads: ignored; STEM_POOL: 4) */
} fdg_layer_desc;

typedef struct {
  int32_t n, c_in, h_in, w_in;  /* module input shape, NCHW */
  int32_t num_layers;
  const fdg_layer_desc* layers; /* HOST pointer; copied at create */
  int32_t delay;                /* d >= 0: the ring holds d+1 saved forwards */
  int32_t is_bottom;            /* 1: the gradient of the module input is never computed */
  int32_t num_classes;          /* heads only */
  float beta;                   /* gradient shrinking factor of Eq. 15, 0 < beta <= 1 */
  float momentum;               /* SGD momentum mu */
  float weight_decay;           /* L2 coefficient added to the gradient of every parameter */
  float bn_eps;                 /* added to the batch variance */
  float bn_momentum;            /* running-statistics momentum */
} fdg_module_desc;

/* Bytes of device workspace a module of this shape needs (parameters, momentum, gradients, the
 * ring of saved forwards with their bf16 weight snapshots, temporaries).  0 on an invalid or
 * unsupported descriptor.  The arena must be aligned to 256 bytes.                               */
size_t fdg_module_workspace_bytes(const fdg_module_desc* desc);

/* Build the host object over `dev_workspace` (DEVICE memory, `bytes` long, caller-owned, must
 * outlive the module).  Parameters, momentum, gradients and running statistics start at zero
 * (running variance at one); call fdg_set_params before the first forward.  Enqueues the zero
 * fill on `hip_stream`.                                                                          */
fdg_status fdg_module_create(const fdg_module_desc* desc, void* dev_workspace, size_t bytes,
                             void* hip_stream, fdg_module** out);

/* What a saved forward (the "saved computation graph" of Fig. 1(b)) consists of.
 *   FDG_SAVE_ACTIVATIONS      : every intermediate the backward reads, written once by the forward.  The ring costs
 *                               delay+1 sets of activations.
 *   FDG_SAVE_INPUT_AND_REPLAY : the module input (fp32, as given) and the weight snapshot only.  The delayed backward
 *                               first runs the forward again on that input with that snapshot (the recomputation of
 *                               feature replay, Section II, here with FDG's own stale weights, so Eq. 10 is unchanged)
 *                               into ONE set of activations shared by all contexts.  Results are those of
 *                               FDG_SAVE_ACTIVATIONS up to the order of floating-point sums; the running statistics of
 *                               batch normalisation move only in fdg_forward.  Costs one more forward per backward.
 *   FDG_SAVE_ACTIVATIONS_CURRENT_WEIGHTS : an ABLATION, not the method.  As FDG_SAVE_ACTIVATIONS, but a saved forward
 *                               keeps no weight snapshot: the module holds ONE bf16 copy of its weights, which follows
 *                               every fdg_update and fdg_set_params, and the delayed backward reads the convolution
 *                               weights, batch-norm scales and classifier weights as they are when it runs (stale
 *                               activations and batch statistics with current weights: what back-propagating through a
 *                               saved graph gives when weights are updated in place).  Eq. 10 carries the stale index on
 *                               the parameters too, so for delay >= 1 this is not the gradient of Eq. 10; with delay 0
 *                               and the call order forward, backward, update it is bit for bit FDG_SAVE_ACTIVATIONS.
 *                               Saves delay+1 weight copies (2 bytes per parameter and layout each).
 * fdg_module_workspace_bytes / fdg_module_create are the _ex forms with FDG_SAVE_ACTIVATIONS; everything said
 * there holds here.  Any other save_mode: 0 bytes / FDG_ERR_INVALID_ARG.                                          */
typedef enum { FDG_SAVE_ACTIVATIONS = 0, FDG_SAVE_INPUT_AND_REPLAY = 1, FDG_SAVE_ACTIVATIONS_CURRENT_WEIGHTS = 2 } fdg_save_mode;
size_t fdg_module_workspace_bytes_ex(const fdg_module_desc* desc, int32_t save_mode);
fdg_status fdg_module_create_ex(const fdg_module_desc* desc, int32_t save_mode, void* dev_workspace, size_t bytes,
                                void* hip_stream, fdg_module** out);

/* Forward step of Section III-A: run the layers on x with the CURRENT weights and push a context
 * (saved activations, batch statistics, and a snapshot of the weights used) into the ring.
 *   x_dev      : [n, c_in, h_in, w_in] fp32 NCHW, read only.
 *   labels_dev : [n] int32 class ids in [0, num_classes) for a top module, else NULL.
 *   y_dev      : output.  Non-top: [n, c_out, h_out, w_out] fp32 NCHW.  Top: 1 + n*num_classes
 *                floats = mean loss followed by the logits, row major [n][num_classes].
 * FDG_ERR_QUEUE_FULL if delay+1 contexts are outstanding.                                       */
fdg_status fdg_forward(fdg_module* m, const float* x_dev, const int32_t* labels_dev, float* y_dev,
                       void* hip_stream);

/* Delayed backward of Eq. 10 with the shrinking of Eq. 15: pops the OLDEST context, multiplies
 * grad_out by beta, back-propagates through that context's saved activations and weight
 * snapshot, leaves the parameter gradient in the module (fdg_get_grads) and, unless is_bottom or
 * grad_in_dev is NULL, writes the gradient of the module input (it carries this module's beta,
 * so a chain of modules compounds to beta^(K-k), Eq. 16).
 *   grad_out_dev : same shape as the forward's y, fp32 NCHW.  Must be NULL for a top module
 *                  (its gradient starts at the loss inside the module).
 *   grad_in_dev  : [n, c_in, h_in, w_in] fp32 NCHW or NULL.
 * FDG_ERR_QUEUE_EMPTY if nothing is outstanding.                                                */
fdg_status fdg_backward_delayed(fdg_module* m, const float* grad_out_dev, float* grad_in_dev,
                                void* hip_stream);

/* Update of Eq. 11 / Eq. 12 on the CURRENT parameters with the last delayed gradient g:
 *   g' = g + weight_decay*theta;  v = momentum*v + g';  theta = theta - lr*v
 * (momentum, weight decay: Section V-A).  FDG_ERR_NO_GRAD if no backward ran since the last
 * update.                                                                                       */
fdg_status fdg_update(fdg_module* m, float lr, void* hip_stream);

/* Frees the host object only (NULL is allowed).  The workspace stays with the caller. */
void fdg_destroy(fdg_module* m);

/* ---- host accessors (parity, checkpointing).  Flat parameter order: layers in order; inside a
 * layer the tensors in this order, each row major in its stated shape:
 *   STEM          : conv w[c_out,c_in,3,3], bn gamma[c_out], bn beta[c_out]
 *   BASIC_POSTACT : conv1 w[c_out,c_in,3,3], bn1 gamma, bn1 beta, conv2 w[c_out,c_out,3,3],
 *                   bn2 gamma, bn2 beta, then if projecting: proj w[c_out,c_in,1,1], bnp gamma,
 *                   bnp beta
 *   BASIC_PREACT  : bn1 gamma[c_in], bn1 beta[c_in], conv1 w[c_out,c_in,3,3], bn2 gamma[c_out],
 *                   bn2 beta[c_out], conv2 w[c_out,c_out,3,3], then if projecting:
 *                   proj w[c_out,c_in,1,1]
 *   HEAD_POSTACT  : fc W[num_classes,c_in], fc b[num_classes]
 *   HEAD_PREACT   : bn gamma[c_in], bn beta[c_in], fc W, fc b
 *   BOTTLENECK_POSTACT : with m = c_out/4: conv1 w[m,c_in,1,1], bn1 gamma[m], bn1 beta[m], conv2 w[m,m,3,3], bn2 gamma,
 *                   bn2 beta, conv3 w[c_out,m,1,1], bn3 gamma[c_out], bn3 beta[c_out], then if projecting:
 *                   proj w[c_out,c_in,1,1], bnp gamma, bnp beta
 * `count` must equal fdg_param_count.                                                           */
size_t fdg_param_count(const fdg_module* m);
fdg_status fdg_set_params(fdg_module* m, const float* host_src, size_t count); /* momentum := 0 */
fdg_status fdg_get_params(const fdg_module* m, float* host_dst, size_t count);
fdg_status fdg_get_grads(const fdg_module* m, float* host_dst, size_t count); /* beta-scaled, before weight decay */
fdg_status fdg_get_momentum(const fdg_module* m, float* host_dst, size_t count);

/* Running BN statistics, flat: for every BN in the parameter order above, mean[c] then var[c]. */
size_t fdg_bn_stat_count(const fdg_module* m);
fdg_status fdg_get_bn_running(const fdg_module* m, float* host_dst, size_t count);

/* Shape of the forward's y: out[0..3] = n, c, h, w (top module: 1, 1, 1, 1 + n*num_classes). */
fdg_status fdg_output_shape(const fdg_module* m, int32_t out[4]);

/* Shape of the forward's x: out[0..3] = n, c_in, h_in, w_in. */
fdg_status fdg_input_shape(const fdg_module* m, int32_t out[4]);

/* What the module was created as: the ring depth `delay`, whether it is a bottom module (no input
 * gradient) and whether it is a top module (ends in the loss).  Any output pointer may be NULL.   */
fdg_status fdg_module_traits(const fdg_module* m, int32_t* delay, int32_t* is_bottom, int32_t* is_top);

/* Ring state: number of outstanding contexts and the sequence numbers (0-based count of forwards)
 * of the oldest and newest one (-1 when empty).  Any of the three output pointers may be NULL.
 * A forward with sequence number s is stored in ring slot s mod (delay+1).                       */
fdg_status fdg_queue_state(const fdg_module* m, int32_t* outstanding, int64_t* oldest_seq,
                           int64_t* newest_seq);

/* ---- parity accessors: the tensors inside a step, layer by layer ------------------------------------------
 * Eq. 8 / Eq. 9 / Eq. 10 are a chain over the layers of a module; these accessors expose every link of that chain
 * so that each layer of a real step can be checked by itself: given the input the layer actually saw, did it produce
 * the output, the input gradient and the parameter gradient its definition gives?  All results are HOST fp32,
 * NCHW, dense, with the padding channels of the internal layout dropped; bf16 tensors are widened exactly.  Every
 * call synchronises the module's streams.  `shape` (optional) receives n, c, h, w; `count` must be n*c*h*w.
 *
 * fdg_saved_read: a tensor of the saved forward with sequence number `seq` (it must still be in the ring:
 * newest_seq - delay <= seq <= newest_seq; a context stays readable after its backward until a forward reuses its
 * slot).  Not available with FDG_SAVE_INPUT_AND_REPLAY before the backward of that context has replayed it.
 *   which 0..5 : the layer's saved intermediates (bf16), by layer kind
 *        STEM               0 = conv output
 *        BASIC_POSTACT      0 = conv1 output, 1 = relu(bn1), 2 = conv2 output, 3 = projection output (if projecting)
 *        BASIC_PREACT       0 = relu(bn1(x)), 1 = conv1 output, 2 = relu(bn2)
 *        BOTTLENECK_POSTACT 0 = conv1 output, 1 = relu(bn1), 2 = conv2 output, 3 = projection output, 4 = relu(bn2),
 *                           5 = conv3 output
 *        HEAD_PREACT        0 = relu(bn(x))
 *        STEM_POOL          0 = conv output, 1 = relu(bn) (the pool's input), both at half the input resolution
 *        INVERTED_RESIDUAL  0 = conv1 output, 1 = relu6(bn1), 2 = depthwise output, 4 = relu6(bn2), 5 = conv3 output
 *   which 6    : the bf16 copy of the layer's output (the next layer's operand and ReLU gate); not for heads
 *   which 7    : the bf16 copy of the layer's input
 *   which 8    : heads: the pooled features [n, c, 1, 1] (fp32)
 *   which 9    : heads: d loss / d logits [n, classes, 1, 1] (fp32)
 * FDG_ERR_INVALID_ARG for a tensor the layer does not have, a seq outside the ring, or a wrong count.
 *
 * fdg_trace_*: the fp32 tensors that travel BETWEEN layers are temporaries of a call; while a trace buffer is
 * attached (DEVICE memory, caller-owned, fdg_trace_bytes long, 256-byte aligned; NULL detaches) fdg_forward copies
 * every layer's fp32 output into it and fdg_backward_delayed every layer's input gradient, with plain device copies
 * on the call's stream after the kernel that produced them (for measurements: detach).  fdg_trace_read:
 *   dir 0, layer i             : fp32 output of layer i of the last traced forward (not for heads);
 *   dir 1, layer i             : gradient of the loss with respect to the INPUT of layer i, as the last traced
 *                                backward left it (absent for layer 0 of a bottom module);
 *   dir 1, layer = num_layers  : the gradient that entered the last layer: beta * grad_out (Eq. 15) (not for top modules).
 * *gated (optional) is set to 1 when a dir-1 tensor was already multiplied by the ReLU gate of the layer below
 * (its producer did that layer's first backward step, see fdg_kernels.h), else 0.                                */
fdg_status fdg_saved_read(const fdg_module* m, int64_t seq, int32_t layer, int32_t which, float* host_dst, size_t count,
                          int32_t shape[4]);
size_t fdg_trace_bytes(const fdg_module* m);
fdg_status fdg_trace_attach(fdg_module* m, void* dev_trace, size_t bytes);
fdg_status fdg_trace_read(const fdg_module* m, int32_t dir, int32_t layer, float* host_dst, size_t count, int32_t shape[4],
                          int32_t* gated);

/* Per-kernel timing, for measurement only. While enabled, every launch group of a call is bracketed by
 * two HIP events on the call's stream (this costs a few microseconds per launch, so throughput is
 * measured with profiling off).  fdg_profile_enable synchronises the module's stream and clears the
 * records.  fdg_profile_read synchronises, then sums the records into at most `capacity` entries of host
 * memory, one per kernel class and -- for convolutions -- per kernel and layer shape, and stores the number
 * of entries that exist in *count (call with capacity 0 to size the array):
 *   name     = class ("conv_fwd", "conv_dgrad", "conv_wgrad", "bn_apply", ...),
 *   kernel   = convolutions: "<kernel as a profiler names it> <ci>><co> k<ksize> s<stride> @<ho>x<wo>", else "",
 *   calls    = launch groups (a stride-2 data gradient is one call of four kernels),
 *   total_ms = summed event time,  flops = algorithmic multiply-add flops (2 per MAC; convolutions only),
 *   bytes    = algorithmic HBM bytes (every operand read once, every result written once).          */
typedef struct {
  char name[32];
  char kernel[80];
  int64_t calls;
  double total_ms;
  double flops;
  double bytes;
} fdg_profile_entry;
fdg_status fdg_profile_enable(fdg_module* m, int enable);
/* Weight gradients normally run on a second stream of the module and overlap the rest of the backward (they depend only
 * on tensors that exist when they are launched, and only the update reads their result).  enable = 0 keeps them on
 * the caller's stream -- a kernel's duration in an external profiler's trace is then its own -- enable = 1 (the
 * default) restores the overlap.  Results are the same bits either way.  Synchronises the module's streams.          */
fdg_status fdg_overlap_enable(fdg_module* m, int enable);
fdg_status fdg_profile_read(fdg_module* m, fdg_profile_entry* host_out, int32_t capacity, int32_t* count);

const char* fdg_status_string(fdg_status s);

#ifdef __cplusplus
}
#endif
#endif /* FDG_H_ */
