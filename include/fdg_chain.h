/*
 * fdg_chain.h -- C ABI of K FDG module workers run together on one GPU as Algorithm I of
 * arXiv 1906.09108 runs them on K devices.
 *
 * Every iteration t = 1, 2, ... each module k does, in the order of Algorithm I,
 *   (1) the delayed backward (Eq. 10, shrunk by the module's beta, Eq. 15) with the gradient it
 *       received at the end of the previous iteration, and the update (Eq. 11) -- if one was received;
 *   (2) the forward on the input it received at the end of the previous iteration (module 0: batch t)
 *       -- if one was received;
 * and, as the last thing an iteration does (Section III-A, communication; Fig. 1(a)), its output goes to
 * module k+1 and the gradient of its input to module k-1.  The last module ends in the loss: it
 * forwards its input, back-propagates the loss gradient of that same batch and updates (delay 0,
 * not shrunk: Section III-B).  So module k (counted from 1) forwards batch t-k+1 and back-propagates
 * batch t-2K+k+1; until those indices reach 1 the module idles for that part.
 *
 * The modules are ordinary fdg_module objects that the caller created (fdg.h) and still owns; the
 * chain borrows them.  Module k runs on a HIP stream of its own (created here, default priority), so
 * the K modules of an iteration overlap on the GPU as far as it has room; the iteration starts after
 * the work already enqueued on the caller's stream and the caller's stream waits for its end.  The
 * mailboxes are double buffered in caller-owned device memory: what is written in iteration t is read
 * in iteration t+1, so the exchange itself moves no data.  The library allocates no device memory.
 *
 * Pointers named *_dev are DEVICE pointers.  Errors are status codes (fdg_status of fdg.h).  A chain
 * is not thread safe, and while it exists nobody else may call the hot-path entry points of its
 * modules.
 */
#ifndef FDG_CHAIN_H_
#define FDG_CHAIN_H_

#include "fdg.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fdg_chain fdg_chain; /* opaque, host memory, library-owned */

/* Bytes of device memory for the mailboxes of these K modules: per boundary two activation and two
 * gradient tensors (fp32, the lower module's output shape) and K label vectors; every part aligned
 * to 256 bytes.  0 if the modules do not form a chain (see fdg_chain_create).                      */
size_t fdg_chain_mailbox_bytes(fdg_module* const* modules, int32_t K);

/* Bind K >= 1 modules, given from the input side, into a chain.  Requirements (else
 * FDG_ERR_INVALID_ARG): module 0 and only module 0 is a bottom module; module K-1 and only it is a top
 * module; the output shape of module k is the input shape of module k+1; no context is outstanding in
 * any module; module k was created with delay >= 2(K-1-k), the number of forwards that wait for their
 * gradient in Fig. 1(a).  `mailbox_dev` (256-byte aligned, `bytes` >= fdg_chain_mailbox_bytes) is
 * caller-owned and must outlive the chain; FDG_ERR_WORKSPACE_TOO_SMALL otherwise.                  */
fdg_status fdg_chain_create(fdg_module* const* modules, int32_t K, void* mailbox_dev, size_t bytes,
                            fdg_chain** out);

/* One iteration of Algorithm I.
 *   x_dev, labels_dev : batch t: module 0's input [n, c_in, h_in, w_in] fp32 NCHW and the n int32 class
 *                       ids of that batch (kept by the chain until the last module sees the batch).
 *   lr                : learning rate of every update of this iteration.
 *   top_y_dev         : where the last module writes its output, 1 + n*num_classes floats (mean loss,
 *                       then the logits), if it forwards a batch in this iteration; untouched otherwise.
 *   top_batch         : HOST pointer or NULL: receives the 1-based number of that batch, 0 if the last
 *                       module is still idle (t < K).
 * Everything is enqueued and the call returns; `hip_stream` waits for the iteration's end.  If a module
 * call fails its status is returned and the chain must not be stepped again.                       */
fdg_status fdg_chain_step(fdg_chain* c, const float* x_dev, const int32_t* labels_dev, float lr,
                          float* top_y_dev, int32_t* top_batch, void* hip_stream);

/* What happened in the last iteration: its number t (0 before the first step) and, per module, the
 * 1-based batch it forwarded and the one it back-propagated (0 = idle).  Host arrays of K entries;
 * any pointer may be NULL.                                                                         */
fdg_status fdg_chain_state(const fdg_chain* c, int64_t* iteration, int32_t* fwd_batch, int32_t* bwd_batch);

/* Waits for the chain's streams, destroys them and frees the host object (NULL allowed).  The modules
 * and the mailbox memory stay with the caller.                                                     */
void fdg_chain_destroy(fdg_chain* c);

/* Learning rate of the paper's training runs (Section V-A) for a 0-based epoch of the 300: 0.1, divided by 10 at
 * epochs 150, 225 and 275; with warmup_epochs > 0 (the paper: 3, for ResNet-110, ResNet-1202 and K = 3, 4) the
 * first warmup_epochs epochs run at 0.01.  Host arithmetic only; negative arguments count as 0.                */
float fdg_lr_schedule(int32_t epoch, int32_t warmup_epochs);

#ifdef __cplusplus
}
#endif
#endif /* FDG_CHAIN_H_ */
