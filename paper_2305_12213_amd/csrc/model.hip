// Model handle: layer plan, workspace carving, and the per-step orchestration of
// dynb_forward_backward (forward, loss, backward per worker) on one stream.
//
// Forward and the activation-gradient pass treat the global batch as one matrix of sum(b)
// rows (rows are independent and all workers share the weights); only the loss scaling 1/b_k
// and the weight/bias gradients are per worker.
//
// Every activation and activation-gradient is kept twice: row-major [rows][features] (the
// k-contiguous operand of forward / activation-gradient GEMMs) and transposed
// [features][padded rows] (the k-contiguous operands of the per-worker weight-gradient GEMMs,
// whose reduction runs over the worker's rows).  In the transposed copies worker k's b_k rows
// sit at columns [poff_k, poff_k + b_k), poff_k = sum_{j<k} round_up(b_j, 8), so that every
// worker's segment starts on a 16-byte boundary; the padding columns are written as zero.
#include <hip/hip_runtime.h>

#include <new>
#include <vector>

#include "dynb_internal.h"

using namespace dynb;

struct DenseLayer {
  int n_in, n_out;
  int64_t ld_in, ld_out;   // padded leading dimensions of the activations
  int64_t w_off, b_off;    // offsets into the flat parameter vector
  bool relu;
  void* Wn = nullptr;      // T [n_in][ld_out]   (B operand of the activation-gradient GEMM)
  void* Wt = nullptr;      // T [n_out][ld_in]   (B operand of the forward GEMM)
};

struct dynb_model {
  int dtype = DYNB_F32;
  int in_features = 0, n_classes = 0;
  std::vector<DenseLayer> layers;
  int64_t P = 0, P_pad = 0;

  bool bound = false;
  float* params = nullptr;
  int max_batch = 0, max_workers = 0;
  int64_t rows_cap = 0;    // padded row capacity (multiple of 64)
  std::vector<void*> act, actT;   // act[l]: input of layer l   (l = 0..L-1)
  std::vector<void*> dy, dyT;     // dy[l]: gradient wrt the output of layer l (after the mask)
  float* logits = nullptr;
  float* rowloss = nullptr;
  float* loss = nullptr;
};

namespace {

int elem_size(int dtype) { return dtype == DYNB_BF16 ? 2 : 4; }

struct Carver {
  char* base;
  size_t used = 0;
  explicit Carver(void* b) : base((char*)b) {}
  void* take(size_t bytes) {
    void* p = base ? base + used : nullptr;
    used += (size_t)round_up((int64_t)bytes, 256);
    return p;
  }
};

// Lays out the workspace; with base == nullptr only the size is computed.
size_t carve(dynb_model* m, void* base, int max_batch, int max_workers) {
  Carver c(base);
  const int es = elem_size(m->dtype);
  const int64_t rows = round_up((int64_t)max_batch + (int64_t)(ROW_PAD - 1) * max_workers, 64);
  const size_t L = m->layers.size();
  m->act.assign(L, nullptr); m->actT.assign(L, nullptr);
  m->dy.assign(L, nullptr);  m->dyT.assign(L, nullptr);
  for (size_t l = 0; l < L; ++l) {
    DenseLayer& D = m->layers[l];
    m->act[l] = c.take((size_t)rows * D.ld_in * es);
    m->actT[l] = c.take((size_t)D.n_in * rows * es);
    m->dy[l] = c.take((size_t)rows * D.ld_out * es);
    m->dyT[l] = c.take((size_t)D.n_out * rows * es);
    D.Wn = c.take((size_t)D.n_in * D.ld_out * es);
    D.Wt = c.take((size_t)D.n_out * D.ld_in * es);
  }
  const int64_t ldc = m->layers.back().ld_out;
  m->logits = (float*)c.take((size_t)rows * ldc * 4);
  m->rowloss = (float*)c.take((size_t)rows * 4);
  m->loss = (float*)c.take((size_t)DYNB_MAX_WORKERS * 4);
  if (base) m->rows_cap = rows;
  return c.used;
}

int build_segs(const int32_t* b, int K, Segs& s) {
  s.K = K;
  s.off[0] = 0;
  s.poff[0] = 0;
  for (int k = 0; k < K; ++k) {
    if (b[k] < 0) return fail(DYNB_ERR_BADARG, "negative batch size for worker %d", k);
    s.off[k + 1] = s.off[k] + b[k];
    s.poff[k + 1] = s.poff[k] + (int)round_up(b[k], ROW_PAD);
  }
  for (int k = K + 1; k <= DYNB_MAX_WORKERS; ++k) {
    s.off[k] = s.off[K];
    s.poff[k] = s.poff[K];
  }
  return DYNB_OK;
}

}  // namespace

extern "C" int dynb_model_create(const dynb_model_desc* d, dynb_model** out) {
  if (!d || !out || !d->layers) return fail(DYNB_ERR_BADARG, "model_create: null pointer");
  if (d->dtype != DYNB_F32 && d->dtype != DYNB_BF16)
    return fail(DYNB_ERR_BADARG, "model_create: unknown dtype");
  if (d->n_layers < 1 || d->n_layers > DYNB_MAX_LAYERS)
    return fail(DYNB_ERR_BADARG, "model_create: n_layers out of range");
  if (d->in_h < 1 || d->in_w < 1 || d->in_c < 1 || d->n_classes < 1)
    return fail(DYNB_ERR_BADARG, "model_create: bad input shape or class count");
  dynb_model* m = new (std::nothrow) dynb_model();
  if (!m) return fail(DYNB_ERR_BADARG, "model_create: out of host memory");
  m->dtype = d->dtype;
  m->n_classes = d->n_classes;
  m->in_features = d->in_h * d->in_w * d->in_c;
  int64_t feat = m->in_features, off = 0;
  for (int l = 0; l < d->n_layers; ++l) {
    const dynb_layer_desc& L = d->layers[l];
    if (L.kind != DYNB_LAYER_DENSE) {
      delete m;
      return fail(DYNB_ERR_UNSUPPORTED, "model_create: layer %d: only dense layers are built", l);
    }
    if (L.n_in != feat || L.n_out < 1) {
      delete m;
      return fail(DYNB_ERR_BADARG, "model_create: layer %d: n_in %d does not match %lld", l,
                  L.n_in, (long long)feat);
    }
    DenseLayer D;
    D.n_in = L.n_in; D.n_out = L.n_out;
    D.ld_in = round_up(L.n_in, COL_PAD); D.ld_out = round_up(L.n_out, COL_PAD);
    D.w_off = off; D.b_off = off + (int64_t)L.n_in * L.n_out;
    D.relu = L.relu != 0;
    off = D.b_off + L.n_out;
    feat = L.n_out;
    m->layers.push_back(D);
  }
  if (feat != d->n_classes) {
    delete m;
    return fail(DYNB_ERR_BADARG, "model_create: last layer has %lld outputs, n_classes is %d",
                (long long)feat, d->n_classes);
  }
  m->P = off;
  m->P_pad = round_up(off, 256);
  *out = m;
  return DYNB_OK;
}

extern "C" void dynb_model_destroy(dynb_model* m) { delete m; }
extern "C" int64_t dynb_model_num_params(const dynb_model* m) { return m ? m->P : 0; }
extern "C" int64_t dynb_model_padded_params(const dynb_model* m) { return m ? m->P_pad : 0; }
extern "C" const float* dynb_model_worker_loss(const dynb_model* m) {
  return (m && m->bound) ? m->loss : nullptr;
}

extern "C" int dynb_model_read_worker_loss(const dynb_model* m, float* host_loss, int32_t K,
                                           void* stream) {
  if (!m || !host_loss) return fail(DYNB_ERR_BADARG, "read_worker_loss: null pointer");
  if (!m->bound) return fail(DYNB_ERR_STATE, "read_worker_loss: model not bound");
  if (K < 1 || K > m->max_workers) return fail(DYNB_ERR_BADARG, "read_worker_loss: K out of range");
  if (hipMemcpyAsync(host_loss, m->loss, sizeof(float) * K, hipMemcpyDeviceToHost,
                     (hipStream_t)stream) != hipSuccess ||
      hipStreamSynchronize((hipStream_t)stream) != hipSuccess)
    return fail(DYNB_ERR_HIP, "read_worker_loss: copy failed");
  return DYNB_OK;
}

extern "C" size_t dynb_model_workspace_bytes(const dynb_model* m, int32_t max_batch,
                                             int32_t max_workers) {
  if (!m || max_batch < 1 || max_workers < 1 || max_workers > DYNB_MAX_WORKERS) return 0;
  dynb_model tmp = *m;
  return carve(&tmp, nullptr, max_batch, max_workers);
}

extern "C" int dynb_model_sync_weights(dynb_model* m, void* stream) {
  if (!m) return fail(DYNB_ERR_BADARG, "sync_weights: null model");
  if (!m->bound) return fail(DYNB_ERR_STATE, "sync_weights: model not bound");
  for (DenseLayer& D : m->layers) {
    int rc = launch_weight_cast(m->dtype, m->params + D.w_off, D.n_in, D.n_out, D.Wn, D.ld_out,
                                D.Wt, D.ld_in, stream);
    if (rc) return rc;
  }
  return DYNB_OK;
}

extern "C" int dynb_model_bind(dynb_model* m, float* params, void* ws, size_t ws_bytes,
                               int32_t max_batch, int32_t max_workers, void* stream) {
  if (!m || !params || !ws) return fail(DYNB_ERR_BADARG, "bind: null pointer");
  if (max_batch < 1 || max_workers < 1 || max_workers > DYNB_MAX_WORKERS)
    return fail(DYNB_ERR_BADARG, "bind: bad max_global_batch / max_workers");
  if (((uintptr_t)ws & 255) || ((uintptr_t)params & 15))
    return fail(DYNB_ERR_BADARG, "bind: workspace must be 256-byte and params 16-byte aligned");
  const size_t need = dynb_model_workspace_bytes(m, max_batch, max_workers);
  if (ws_bytes < need)
    return fail(DYNB_ERR_BADARG, "bind: workspace has %zu bytes, %zu needed", ws_bytes, need);
  carve(m, ws, max_batch, max_workers);
  m->params = params;
  m->max_batch = max_batch;
  m->max_workers = max_workers;
  // Padding (columns beyond a layer's width, rows beyond a worker's segment) must hold
  // finite values: it is multiplied by exact zeros.  Clearing once is enough, kernels
  // never write non-finite padding.
  if (hipMemsetAsync(ws, 0, need, (hipStream_t)stream) != hipSuccess)
    return fail(DYNB_ERR_HIP, "bind: hipMemsetAsync failed");
  m->bound = true;
  return dynb_model_sync_weights(m, stream);
}

extern "C" int dynb_forward_backward(dynb_model* m, const float* x, const int32_t* y,
                                     const int32_t* b, int32_t K, float* grads, void* stream) {
  if (!m || !x || !y || !b || !grads) return fail(DYNB_ERR_BADARG, "forward_backward: null pointer");
  if (!m->bound) return fail(DYNB_ERR_STATE, "forward_backward: model not bound");
  if (K < 1 || K > m->max_workers)
    return fail(DYNB_ERR_BADARG, "forward_backward: K=%d outside [1, %d]", K, m->max_workers);
  if ((uintptr_t)grads & 15) return fail(DYNB_ERR_BADARG, "forward_backward: grads must be 16-byte aligned");
  Segs s;
  int rc = build_segs(b, K, s);
  if (rc) return rc;
  if (s.off[K] > m->max_batch)
    return fail(DYNB_ERR_BADARG, "forward_backward: sum(b)=%d exceeds max_global_batch=%d",
                s.off[K], m->max_batch);
  const int Mp = s.off[K];    // rows of the global batch
  const int dt = m->dtype;
  const size_t L = m->layers.size();
  const int64_t ldT = m->rows_cap;

  if (Mp > 0) {
    // ---- forward ----
    rc = launch_pack_rows(dt, x, Mp, m->in_features, m->act[0], m->layers[0].ld_in, stream);
    if (rc) return rc;
    rc = launch_transpose(dt, m->act[0], m->layers[0].ld_in, m->layers[0].n_in, m->actT[0], ldT, s,
                          stream);
    if (rc) return rc;
    for (size_t l = 0; l < L; ++l) {
      const DenseLayer& D = m->layers[l];
      const bool last = l + 1 == L;
      GemmArgs g = {};
      g.A = m->act[l]; g.lda = D.ld_in; g.M = Mp;
      g.B = D.Wt; g.ldb = D.ld_in; g.N = D.n_out;
      g.K = (int)D.ld_in;
      g.mode = MODE_FWD;
      g.bias = m->params + D.b_off;
      g.relu = D.relu;
      if (last) { g.Cf = m->logits; g.ldcf = D.ld_out; }
      else { g.C = m->act[l + 1]; g.ldc = D.ld_out; }
      rc = launch_gemm(dt, g, s, stream);
      if (rc) return rc;
      if (!last) {
        rc = launch_transpose(dt, m->act[l + 1], D.ld_out, D.n_out, m->actT[l + 1], ldT, s, stream);
        if (rc) return rc;
      }
    }
    // ---- loss and dlogits (mean over each worker's own b_k samples) ----
    const DenseLayer& Z = m->layers[L - 1];
    rc = launch_softmax_xent(dt, m->logits, Z.ld_out, y, m->n_classes, m->dy[L - 1], Z.ld_out,
                             (int)Z.ld_out, m->rowloss, s, stream);
    if (rc) return rc;
    // ---- backward ----
    for (size_t l = L; l-- > 0;) {
      const DenseLayer& D = m->layers[l];
      rc = launch_transpose(dt, m->dy[l], D.ld_out, D.n_out, m->dyT[l], ldT, s, stream);
      if (rc) return rc;
      if (l > 0) {  // gradient wrt this layer's input, masked by the ReLU of the layer below
        const DenseLayer& Dp = m->layers[l - 1];
        GemmArgs g = {};
        g.A = m->dy[l]; g.lda = D.ld_out; g.M = Mp;
        g.B = D.Wn; g.ldb = D.ld_out; g.N = D.n_in;
        g.K = (int)D.ld_out;
        g.mode = MODE_DGRAD;
        g.C = m->dy[l - 1]; g.ldc = Dp.ld_out;
        if (Dp.relu) { g.mask = m->act[l]; g.ldmask = D.ld_in; }
        rc = launch_gemm(dt, g, s, stream);
        if (rc) return rc;
      }
    }
  }
  // ---- per-worker weight and bias gradients ----
  for (size_t l = 0; l < L; ++l) {
    const DenseLayer& D = m->layers[l];
    GemmArgs g = {};
    g.A = m->dyT[l]; g.lda = ldT; g.M = D.n_out;
    g.B = m->actT[l]; g.ldb = ldT; g.N = D.n_in;
    g.mode = MODE_WGRAD;
    g.Cf = grads + D.w_off; g.ldcf = D.n_out;
    g.group_stride = m->P_pad;
    rc = launch_gemm(dt, g, s, stream);
    if (rc) return rc;
    rc = launch_bias_grad(dt, m->dyT[l], ldT, D.n_out, grads + D.b_off, m->P_pad, s, stream);
    if (rc) return rc;
  }
  return launch_finalize(m->rowloss, m->loss, grads, m->P, m->P_pad, s, stream);
}

extern "C" int dynb_model_sgd_update(dynb_model* m, const float* g, float lr, float mu,
                                     float* velocity, void* stream) {
  if (!m || !g) return fail(DYNB_ERR_BADARG, "model_sgd_update: null pointer");
  if (!m->bound) return fail(DYNB_ERR_STATE, "model_sgd_update: model not bound");
  int rc = velocity ? dynb_sgd_momentum_update(m->params, velocity, g, m->P_pad, lr, mu, stream)
                    : dynb_sgd_update(m->params, g, m->P_pad, lr, stream);
  if (rc) return rc;
  return dynb_model_sync_weights(m, stream);
}
