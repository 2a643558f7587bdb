// K module workers on one GPU run as Algorithm I of arXiv 1906.09108: per module backward + update, forward,
// exchange at the end of the iteration (Section III-A).  Host code only: it sequences the entry points of
// fdg.h on one stream per module and keeps the double-buffered mailboxes; it holds no arithmetic.
#include <hip/hip_runtime.h>

#include <new>
#include <vector>

#include "../../include/fdg_chain.h"

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Shapes {
  std::vector<size_t> boundary_bytes;   // fp32 bytes of the tensor between module k and k+1
  size_t label_bytes = 0;               // one batch of labels
  size_t total = 0;
};

// Validates the chain and sizes its mailboxes.
bool plan(fdg_module* const* mods, int32_t K, Shapes* sh) {
  if (!mods || K < 1) return false;
  sh->boundary_bytes.clear();
  size_t total = 0;
  int32_t n0 = 0;
  for (int32_t k = 0; k < K; ++k) {
    if (!mods[k]) return false;
    int32_t delay = 0, bottom = 0, top = 0, in[4], out[4], outstanding = 0;
    if (fdg_module_traits(mods[k], &delay, &bottom, &top) != FDG_OK) return false;
    if (fdg_input_shape(mods[k], in) != FDG_OK || fdg_output_shape(mods[k], out) != FDG_OK) return false;
    if (fdg_queue_state(mods[k], &outstanding, nullptr, nullptr) != FDG_OK || outstanding != 0) return false;
    if ((bottom != 0) != (k == 0) || (top != 0) != (k == K - 1)) return false;
    if (delay < 2 * (K - 1 - k)) return false;
    if (k == 0) n0 = in[0];
    if (in[0] != n0) return false;
    if (k + 1 < K) {
      int32_t nin[4];
      if (!mods[k + 1] || fdg_input_shape(mods[k + 1], nin) != FDG_OK) return false;
      for (int i = 0; i < 4; ++i)
        if (nin[i] != out[i]) return false;
      const size_t bytes = align_up((size_t)out[0] * out[1] * out[2] * out[3] * sizeof(float), kAlign);
      sh->boundary_bytes.push_back(bytes);
      total += 4 * bytes;   // activation and gradient, two buffers each
    }
  }
  sh->label_bytes = align_up((size_t)n0 * sizeof(int32_t), kAlign);
  total += (size_t)K * sh->label_bytes;
  sh->total = total;
  return true;
}

}  // namespace

struct fdg_chain {
  int32_t K = 0;
  std::vector<fdg_module*> mods;
  std::vector<hipStream_t> streams;     // one per module
  std::vector<hipEvent_t> done;         // end of module k's part of an iteration
  hipEvent_t start = nullptr;           // the caller's stream at the start of an iteration
  // mailboxes: act[k][s] = output of module k (input of k+1), grad[k][s] = gradient of that tensor (from k+1),
  // s = iteration parity of the writer
  std::vector<float*> act[2], grad[2];
  std::vector<int32_t> act_batch[2], grad_batch[2];   // batch held by that buffer, 0 = nothing
  std::vector<int32_t*> labels;          // K buffers, batch b lives in labels[b % K]
  int64_t t = 0;
  std::vector<int32_t> fwd_batch, bwd_batch;
  bool broken = false;
};

extern "C" size_t fdg_chain_mailbox_bytes(fdg_module* const* modules, int32_t K) {
  Shapes sh;
  return plan(modules, K, &sh) ? sh.total : 0;
}

extern "C" fdg_status fdg_chain_create(fdg_module* const* modules, int32_t K, void* mailbox_dev, size_t bytes,
                                       fdg_chain** out) {
  if (!out) return FDG_ERR_INVALID_ARG;
  *out = nullptr;
  Shapes sh;
  if (!plan(modules, K, &sh)) return FDG_ERR_INVALID_ARG;
  if (sh.total > 0 && (!mailbox_dev || bytes < sh.total || reinterpret_cast<uintptr_t>(mailbox_dev) % kAlign))
    return FDG_ERR_WORKSPACE_TOO_SMALL;
  fdg_chain* c = new (std::nothrow) fdg_chain;
  if (!c) return FDG_ERR_INVALID_ARG;
  c->K = K;
  c->mods.assign(modules, modules + K);
  c->fwd_batch.assign(K, 0);
  c->bwd_batch.assign(K, 0);
  char* p = static_cast<char*>(mailbox_dev);
  for (int s = 0; s < 2; ++s) {
    c->act[s].resize(K > 0 ? K - 1 : 0);
    c->grad[s].resize(K > 0 ? K - 1 : 0);
    c->act_batch[s].assign(K > 0 ? K - 1 : 0, 0);
    c->grad_batch[s].assign(K > 0 ? K - 1 : 0, 0);
  }
  for (int32_t k = 0; k + 1 < K; ++k)
    for (int s = 0; s < 2; ++s) {
      c->act[s][k] = reinterpret_cast<float*>(p); p += sh.boundary_bytes[k];
      c->grad[s][k] = reinterpret_cast<float*>(p); p += sh.boundary_bytes[k];
    }
  for (int32_t k = 0; k < K; ++k) { c->labels.push_back(reinterpret_cast<int32_t*>(p)); p += sh.label_bytes; }
  bool ok = hipEventCreateWithFlags(&c->start, hipEventDisableTiming) == hipSuccess;
  for (int32_t k = 0; k < K && ok; ++k) {
    hipStream_t s = nullptr;
    hipEvent_t e = nullptr;
    ok = hipStreamCreateWithFlags(&s, hipStreamNonBlocking) == hipSuccess;
    if (ok) c->streams.push_back(s);
    ok = ok && hipEventCreateWithFlags(&e, hipEventDisableTiming) == hipSuccess;
    if (e) c->done.push_back(e);
  }
  if (!ok) {
    (void)hipGetLastError();
    fdg_chain_destroy(c);
    return FDG_ERR_HIP;
  }
  *out = c;
  return FDG_OK;
}

#define CHAIN_HIP(expr)                   \
  do {                                    \
    if ((expr) != hipSuccess) {           \
      (void)hipGetLastError();            \
      c->broken = true;                   \
      return FDG_ERR_HIP;                 \
    }                                     \
  } while (0)
#define CHAIN_FDG(expr)                   \
  do {                                    \
    const fdg_status st__ = (expr);       \
    if (st__ != FDG_OK) {                 \
      c->broken = true;                   \
      return st__;                        \
    }                                     \
  } while (0)

extern "C" fdg_status fdg_chain_step(fdg_chain* c, const float* x_dev, const int32_t* labels_dev, float lr,
                                     float* top_y_dev, int32_t* top_batch, void* hip_stream) {
  if (!c || !x_dev || !labels_dev || !top_y_dev || c->broken) return FDG_ERR_INVALID_ARG;
  hipStream_t main = static_cast<hipStream_t>(hip_stream);
  const int32_t K = c->K;
  const int64_t t = c->t + 1;
  const int w = (int)(t & 1), r = w ^ 1;   // buffers written in this iteration / written in the previous one
  // the labels of batch t wait in the chain until the last module forwards that batch (iteration t+K-1)
  const size_t n_labels = [&] { int32_t in[4]; (void)fdg_input_shape(c->mods[0], in); return (size_t)in[0]; }();
  CHAIN_HIP(hipMemcpyAsync(c->labels[t % K], labels_dev, n_labels * sizeof(int32_t), hipMemcpyDeviceToDevice, main));
  CHAIN_HIP(hipEventRecord(c->start, main));
  if (top_batch) *top_batch = 0;
  for (int32_t k = 0; k < K; ++k) {
    fdg_module* m = c->mods[k];
    hipStream_t s = c->streams[k];
    CHAIN_HIP(hipStreamWaitEvent(s, c->start, 0));
    c->fwd_batch[k] = c->bwd_batch[k] = 0;
    const int32_t in_batch = k == 0 ? (int32_t)t : c->act_batch[r][k - 1];
    const float* in = k == 0 ? x_dev : c->act[r][k - 1];
    float* grad_in = k == 0 ? nullptr : c->grad[w][k - 1];
    if (k > 0) c->grad_batch[w][k - 1] = 0;
    if (k + 1 < K) c->act_batch[w][k] = 0;
    if (k == K - 1) {
      if (in_batch) {
        CHAIN_FDG(fdg_forward(m, in, c->labels[in_batch % K], top_y_dev, s));
        CHAIN_FDG(fdg_backward_delayed(m, nullptr, grad_in, s));
        CHAIN_FDG(fdg_update(m, lr, s));
        c->fwd_batch[k] = c->bwd_batch[k] = in_batch;
        if (k > 0) c->grad_batch[w][k - 1] = in_batch;
        if (top_batch) *top_batch = in_batch;
      }
    } else {
      const int32_t g_batch = c->grad_batch[r][k];
      if (g_batch) {
        CHAIN_FDG(fdg_backward_delayed(m, c->grad[r][k], grad_in, s));
        CHAIN_FDG(fdg_update(m, lr, s));
        c->bwd_batch[k] = g_batch;
        if (k > 0) c->grad_batch[w][k - 1] = g_batch;
      }
      if (in_batch) {
        CHAIN_FDG(fdg_forward(m, in, nullptr, c->act[w][k], s));
        c->fwd_batch[k] = in_batch;
        c->act_batch[w][k] = in_batch;
      }
    }
    CHAIN_HIP(hipEventRecord(c->done[k], s));
  }
  // the communication of Section III-A: the iteration ends when every module is done; the buffers written now
  // are the ones read next
  for (int32_t k = 0; k < K; ++k) CHAIN_HIP(hipStreamWaitEvent(main, c->done[k], 0));
  c->t = t;
  return FDG_OK;
}

extern "C" fdg_status fdg_chain_state(const fdg_chain* c, int64_t* iteration, int32_t* fwd_batch, int32_t* bwd_batch) {
  if (!c) return FDG_ERR_INVALID_ARG;
  if (iteration) *iteration = c->t;
  for (int32_t k = 0; k < c->K; ++k) {
    if (fwd_batch) fwd_batch[k] = c->fwd_batch[k];
    if (bwd_batch) bwd_batch[k] = c->bwd_batch[k];
  }
  return FDG_OK;
}

extern "C" void fdg_chain_destroy(fdg_chain* c) {
  if (!c) return;
  for (hipStream_t s : c->streams) {
    (void)hipStreamSynchronize(s);
    (void)hipStreamDestroy(s);
  }
  for (hipEvent_t e : c->done) (void)hipEventDestroy(e);
  if (c->start) (void)hipEventDestroy(c->start);
  (void)hipGetLastError();
  delete c;
}

extern "C" float fdg_lr_schedule(int32_t epoch, int32_t warmup_epochs) {
  if (epoch < 0) epoch = 0;
  if (epoch < warmup_epochs) return 0.01f;
  if (epoch < 150) return 0.1f;
  if (epoch < 225) return 0.01f;
  if (epoch < 275) return 0.001f;
  return 0.0001f;
}
