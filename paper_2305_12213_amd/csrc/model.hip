// Model handle: layer plan, workspace carving, and the per-step orchestration of
// dynb_forward_backward (forward, loss, backward per worker) on one stream.
//
// Forward and the activation-gradient pass treat the global batch as one matrix (rows are
// independent and all workers share the weights); only the loss scaling 1/b_k and the
// weight/bias gradients are per worker.  A "row" is a sample for dense layers and a pixel
// (sample, y, x) for convolutions (NHWC with the channel pitch padded to 64).
//
// bf16 models: the per-worker weight-gradient kernels reduce over the rows of the row-major
// activations and gradients themselves.  fp32 models: every operand of a per-worker
// weight-gradient GEMM is kept transposed, [features][padded rows]; in these copies worker k's
// rows sit at columns [poff_k, poff_k + rows_k), poff_k = sum_{j<k} round_up(rows_j, 8), so that
// every worker's segment starts on a 16-byte boundary; the padding columns are written as zero.
#include <hip/hip_runtime.h>

#include <cmath>
#include <mutex>
#include <new>
#include <vector>

#include "dynb_internal.h"

using namespace dynb;

struct Layer {
  int kind = DYNB_LAYER_DENSE;
  int n_in = 0, n_out = 0;           // features (dense) or channels (conv, pool)
  int h_in = 1, w_in = 1, h_out = 1, w_out = 1, stride = 1;
  int hw_in = 1, hw_out = 1;         // rows per sample of the input / output
  int64_t ld_in = 0, ld_out = 0;     // channel pitch of input / output rows
  int cin_p = 0, cout_p = 0;         // conv: channels per tap, padded to 8
  int kf = 0, kd = 0;                // conv: reduction length forward / input gradient (x64)
  int wg_rows = 0;                   // rows of the transposed weight-gradient operand
  int64_t w_off = 0, b_off = 0;      // offsets into the flat parameter vector
  bool relu = false, has_params = false;
  void* Wn = nullptr;                // B operand of the input-gradient GEMM
  void* Wt = nullptr;                // B operand of the forward GEMM
  void* out = nullptr;               // T [rows_out][ld_out]: stored output (not for the last layer)
  void* inT = nullptr;               // T [wg_rows][cap]: transposed input (dense layers)
  void* dy = nullptr;                // T [rows_out][ld_out]: gradient wrt the output, masked
  void* dyT = nullptr;               // T [n_out][cap]
  int64_t capT = 0;                  // padded row capacity of inT / dyT
  int max_split = 1;                 // most chunks a worker's weight-gradient reduction is cut into
  int conv_chunk = 0;                // rows per chunk of a convolution's weight gradient
  // batch normalisation: scale at w_off, shift at b_off (n_out floats each); per-worker statistics
  float eps = 0.f;
  float* bn_mean = nullptr;          // fp32 [max_workers][n_out]
  float* bn_rstd = nullptr;
  // residual addition: this layer adds the stored output of layer skip_from; the source layer
  // receives the gradient of that branch in dy_skip and merges it into dy
  int skip_from = -1;
  bool skip_source = false;
  void* dy_skip = nullptr;           // T [rows_out][ld_out]; not needed when skip_fused
  // the layer above a skip source is a matrix product: its input-gradient kernel adds the
  // residual branch's gradient while writing this layer's dy (no separate pass)
  bool skip_fused = false;
  // a normalisation without ReLU directly in front of a residual addition: both run in one
  // kernel and the normalised tensor itself is never stored
  bool add_fused = false;
};

struct dynb_model {
  int dtype = DYNB_F32;
  int in_h = 1, in_w = 1, in_c = 1, n_classes = 0;
  std::vector<Layer> layers;
  int64_t P = 0, P_pad = 0;
  int first_param_layer = 0;

  bool bound = false;
  float* params = nullptr;
  int max_batch = 0, max_workers = 0;
  void* act0 = nullptr;              // packed input, T [B * in_h * in_w][ld]
  int64_t ld0 = 0;
  float* logits = nullptr;
  float* rowloss = nullptr;
  float* loss = nullptr;
  float* partial = nullptr;          // scratch of the split weight-gradient reductions
  int64_t partial_floats = 0;
  float* row_scratch = nullptr;       // chunk partials of the per-worker column reductions over pixel rows
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

int64_t padded_cap(int64_t max_batch, int64_t hw, int max_workers) {
  return round_up(max_batch * hw + (int64_t)(ROW_PAD - 1) * max_workers, 64);
}

// Lays out the workspace; with base == nullptr only the size is computed.
size_t carve(dynb_model* m, void* base, int max_batch, int max_workers) {
  Carver c(base);
  const int es = elem_size(m->dtype);
  m->act0 = c.take((size_t)max_batch * m->in_h * m->in_w * m->ld0 * es);
  for (size_t l = 0; l < m->layers.size(); ++l) {
    Layer& L = m->layers[l];
    const bool last = l + 1 == m->layers.size();
    const int64_t rows_out = (int64_t)max_batch * L.hw_out;
    if (!last && !L.add_fused) L.out = c.take((size_t)rows_out * L.ld_out * es);
    L.dy = c.take((size_t)rows_out * L.ld_out * es);
    if (L.skip_source && !L.skip_fused) L.dy_skip = c.take((size_t)rows_out * L.ld_out * es);
    if (L.kind == DYNB_LAYER_BN) {
      L.bn_mean = (float*)c.take((size_t)max_workers * L.n_out * 4);
      L.bn_rstd = (float*)c.take((size_t)max_workers * L.n_out * 4);
    }
    if (L.has_params) {
      if (L.kind == DYNB_LAYER_DENSE && m->dtype != DYNB_BF16) {   // (bf16 weight gradients read the
                                                                   // row-major tensors themselves)
        L.capT = padded_cap(max_batch, L.hw_out, max_workers);
        L.inT = c.take((size_t)L.wg_rows * L.capT * es);
        L.dyT = c.take((size_t)L.n_out * L.capT * es);
      }
      if (L.kind == DYNB_LAYER_DENSE) {
        L.Wn = c.take((size_t)L.n_in * L.ld_out * es);
        L.Wt = c.take((size_t)L.n_out * L.ld_in * es);
      } else {
        L.Wt = c.take((size_t)L.n_out * L.kf * es);
        L.Wn = c.take((size_t)L.n_in * L.kd * es);
      }
    }
  }
  int64_t bn_floats = 0;
  for (Layer& L : m->layers)
    if (L.kind == DYNB_LAYER_BN) {
      const int64_t need = row_scratch_floats((int64_t)max_batch * L.hw_out, max_workers, L.n_out);
      if (need > bn_floats) bn_floats = need;
    }
  m->row_scratch = bn_floats ? (float*)c.take((size_t)bn_floats * 4) : nullptr;
  const int64_t ldc = m->layers.back().ld_out;
  m->logits = (float*)c.take((size_t)max_batch * ldc * 4);
  m->rowloss = (float*)c.take((size_t)max_batch * 4);
  m->loss = (float*)c.take((size_t)DYNB_MAX_WORKERS * 4);
  // Scratch of the weight gradients that are reduced in chunks (one area serves all layers): a
  // dense layer with few weight-gradient tiles splits each worker's reduction over workgroups;
  // a convolution sums over every pixel of every sample and always works in row chunks.  The
  // chunk results are added afterwards in a fixed order.
  m->partial_floats = 0;
  for (Layer& L : m->layers) {
    if (!L.has_params || m->dtype != DYNB_BF16) continue;
    int64_t need = 0;
    if (L.kind == DYNB_LAYER_CONV3X3) {
      const int64_t rows = (int64_t)max_batch * L.hw_out;
      L.conv_chunk = conv_wgrad_chunk_rows(rows);
      need = conv_wgrad_scratch_floats(rows, max_workers, L.n_in, L.n_out);
    } else {
      const int64_t tiles = ((L.n_out + 127) / 128) * (int64_t)((L.wg_rows + 127) / 128);
      L.max_split = tiles >= 32 ? 1 : (int)(256 / tiles > 64 ? 64 : 256 / tiles);
      if (L.max_split > 1)
        need = round_up((int64_t)L.wg_rows * L.n_out, 64) * L.max_split * max_workers;
    }
    if (need > m->partial_floats) m->partial_floats = need;
  }
  m->partial = (float*)c.take((size_t)m->partial_floats * 4);
  return c.used;
}

// Segments in a row space with `hw` rows per sample.
int build_segs(const int32_t* b, int K, int hw, Segs& s) {
  s.K = K;
  s.off[0] = 0;
  s.poff[0] = 0;
  for (int k = 0; k < K; ++k) {
    if (b[k] < 0) return fail(DYNB_ERR_BADARG, "negative batch size for worker %d", k);
    s.off[k + 1] = s.off[k] + b[k] * hw;
    s.poff[k + 1] = s.poff[k] + (int)round_up((int64_t)b[k] * hw, ROW_PAD);
  }
  for (int k = K + 1; k <= DYNB_MAX_WORKERS; ++k) {
    s.off[k] = s.off[K];
    s.poff[k] = s.poff[K];
  }
  return DYNB_OK;
}

int bad_model(dynb_model* m, int code, const char* msg, int layer) {
  delete m;
  return fail(code, "model_create: layer %d: %s", layer, msg);
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
  m->in_h = d->in_h; m->in_w = d->in_w; m->in_c = d->in_c;
  bool has_conv = false;
  for (int l = 0; l < d->n_layers; ++l)
    has_conv |= d->layers[l].kind == DYNB_LAYER_CONV3X3 || d->layers[l].kind == DYNB_LAYER_GAP;
  // current activation geometry: h x w pixels of c channels per sample; a dense-only model
  // treats the whole input as one row of h*w*c features
  int h = has_conv ? d->in_h : 1, w = has_conv ? d->in_w : 1;
  int c = has_conv ? d->in_c : d->in_h * d->in_w * d->in_c;
  if (!has_conv) { m->in_c = c; m->in_h = 1; m->in_w = 1; }
  m->ld0 = round_up(c, COL_PAD);
  int64_t off = 0;
  bool seen_param = false, norm_params = false;
  for (int l = 0; l < d->n_layers; ++l) {
    const dynb_layer_desc& S = d->layers[l];
    Layer L;
    L.kind = S.kind;
    L.relu = S.relu != 0;
    L.h_in = h; L.w_in = w; L.hw_in = h * w;
    L.n_in = c;
    L.ld_in = round_up(c, COL_PAD);
    if (S.kind == DYNB_LAYER_DENSE) {
      if (h * w != 1) return bad_model(m, DYNB_ERR_UNSUPPORTED, "dense layer on a spatial input (pool first)", l);
      if (S.n_in != c || S.n_out < 1) return bad_model(m, DYNB_ERR_BADARG, "n_in does not match the incoming features", l);
      L.n_out = S.n_out;
      L.has_params = true;
      L.wg_rows = L.n_in;
      L.w_off = off; L.b_off = off + (int64_t)L.n_in * L.n_out;
      off = L.b_off + L.n_out;
    } else if (S.kind == DYNB_LAYER_CONV3X3) {
      if (d->dtype != DYNB_BF16) return bad_model(m, DYNB_ERR_UNSUPPORTED, "convolutions are built for bf16 models only", l);
      if (S.n_in != c || S.n_out < 1) return bad_model(m, DYNB_ERR_BADARG, "c_in does not match the incoming channels", l);
      if (S.stride != 1 && S.stride != 2) return bad_model(m, DYNB_ERR_BADARG, "stride must be 1 or 2", l);
      L.n_out = S.n_out;
      L.stride = S.stride;
      h = (h + 2 - 3) / S.stride + 1;
      w = (w + 2 - 3) / S.stride + 1;
      L.cin_p = (int)round_up(L.n_in, 8); L.cout_p = (int)round_up(L.n_out, 8);
      L.kf = (int)round_up(9 * L.cin_p, 64); L.kd = (int)round_up(9 * L.cout_p, 64);
      L.has_params = true;
      L.wg_rows = 9 * L.n_in;
      L.w_off = off; L.b_off = off + (int64_t)9 * L.n_in * L.n_out;
      off = L.b_off + L.n_out;
    } else if (S.kind == DYNB_LAYER_GAP) {
      if (d->dtype != DYNB_BF16) return bad_model(m, DYNB_ERR_UNSUPPORTED, "pooling is built for bf16 models only", l);
      if (S.relu) return bad_model(m, DYNB_ERR_UNSUPPORTED, "ReLU on a pooling layer", l);
      L.n_out = c;
      h = 1; w = 1;
    } else if (S.kind == DYNB_LAYER_BN) {
      if (d->dtype != DYNB_BF16) return bad_model(m, DYNB_ERR_UNSUPPORTED, "batch normalisation is built for bf16 models only", l);
      if (S.n_in != c || S.n_out != c) return bad_model(m, DYNB_ERR_BADARG, "channel count does not match the incoming channels", l);
      if (!(S.eps >= 0.f) || !std::isfinite(S.eps)) return bad_model(m, DYNB_ERR_BADARG, "eps must be finite and >= 0", l);
      L.n_out = c;
      L.eps = S.eps;
      L.w_off = off; L.b_off = off + c;
      off = L.b_off + c;
      norm_params = true;
    } else if (S.kind == DYNB_LAYER_ADD) {
      if (d->dtype != DYNB_BF16) return bad_model(m, DYNB_ERR_UNSUPPORTED, "residual additions are built for bf16 models only", l);
      if (S.skip_from < 0 || S.skip_from > l - 2) return bad_model(m, DYNB_ERR_BADARG, "skip_from must name a layer at least two below", l);
      Layer& Src = m->layers[S.skip_from];
      if (Src.n_out != c || Src.h_out != h || Src.w_out != w) return bad_model(m, DYNB_ERR_BADARG, "the skipped output has another shape", l);
      if (Src.skip_source) return bad_model(m, DYNB_ERR_UNSUPPORTED, "one residual addition per source layer", l);
      Src.skip_source = true;
      L.skip_from = S.skip_from;
      L.n_out = c;
    } else {
      return bad_model(m, DYNB_ERR_BADARG, "unknown layer kind", l);
    }
    L.h_out = h; L.w_out = w; L.hw_out = h * w;
    L.ld_out = round_up(L.n_out, COL_PAD);
    c = L.n_out;
    if ((L.has_params || norm_params) && !seen_param) { m->first_param_layer = l; seen_param = true; }
    norm_params = false;
    m->layers.push_back(L);
  }
  if (!seen_param) return bad_model(m, DYNB_ERR_BADARG, "model has no parameters", 0);
  const Layer& Z = m->layers.back();
  if (Z.kind != DYNB_LAYER_DENSE || Z.n_out != d->n_classes || Z.hw_out != 1)
    return bad_model(m, DYNB_ERR_BADARG, "the last layer must be dense with n_classes outputs", d->n_layers - 1);
  // what the layer graph allows to be fused (see Layer)
  for (size_t l = 0; l + 1 < m->layers.size(); ++l) {
    Layer& L = m->layers[l];
    const Layer& Up = m->layers[l + 1];
    if (L.skip_source && (Up.kind == DYNB_LAYER_DENSE || Up.kind == DYNB_LAYER_CONV3X3) &&
        (int)l + 1 > m->first_param_layer)
      L.skip_fused = true;
    if (L.kind == DYNB_LAYER_BN && !L.relu && !L.skip_source && Up.kind == DYNB_LAYER_ADD)
      L.add_fused = true;
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
  for (Layer& L : m->layers) {
    if (!L.has_params) continue;
    int rc;
    if (L.kind == DYNB_LAYER_DENSE)
      rc = launch_weight_cast(m->dtype, m->params + L.w_off, L.n_in, L.n_out, L.Wn, L.ld_out, L.Wt,
                              L.ld_in, stream);
    else
      rc = launch_conv_weight_cast(m->params + L.w_off, L.n_in, L.n_out, L.cin_p, L.cout_p, L.Wt,
                                   L.kf, L.Wn, L.kd, stream);
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
  int64_t max_hw = (int64_t)m->in_h * m->in_w;
  for (const Layer& L : m->layers) max_hw = L.hw_out > max_hw ? L.hw_out : max_hw;
  if ((int64_t)max_batch * max_hw > (int64_t)1 << 30)
    return fail(DYNB_ERR_UNSUPPORTED, "bind: max_global_batch * pixels exceeds 2^30 rows");
  if (m->dtype == DYNB_BF16) {   // the bf16 kernels keep byte offsets into an activation in 31 bits
    int64_t largest = (int64_t)max_batch * m->in_h * m->in_w * m->ld0 * 2;
    for (const Layer& L : m->layers) {
      const int64_t bytes = (int64_t)max_batch * L.hw_out * L.ld_out * 2;
      largest = bytes > largest ? bytes : largest;
    }
    if (largest >= (int64_t)1 << 31)
      return fail(DYNB_ERR_UNSUPPORTED,
                  "bind: an activation tensor of %lld bytes (2 GiB or more) is not supported; "
                  "lower max_global_batch", (long long)largest);
  }
  const size_t need = dynb_model_workspace_bytes(m, max_batch, max_workers);
  if (ws_bytes < need)
    return fail(DYNB_ERR_BADARG, "bind: workspace has %zu bytes, %zu needed", ws_bytes, need);
  carve(m, ws, max_batch, max_workers);
  m->params = params;
  m->max_batch = max_batch;
  m->max_workers = max_workers;
  // Padding columns (beyond a layer's width) are operands of the GEMMs and are multiplied by
  // zero weights: they must hold finite values.  Clearing once is enough, no kernel writes them.
  if (hipMemsetAsync(ws, 0, need, (hipStream_t)stream) != hipSuccess)
    return fail(DYNB_ERR_HIP, "bind: hipMemsetAsync failed");
  m->bound = true;
  return dynb_model_sync_weights(m, stream);
}

namespace {
// Forward, loss, backward and the per-worker gradients; with `agg` also the weighted aggregate
// agg[p] = sum_k (b_k / sum b) grads[k][p] (Eq. 2).
int run_forward_backward(dynb_model* m, const float* x, const int32_t* y, const int32_t* b,
                         int32_t K, float* grads, float* agg, void* stream);
}  // namespace

extern "C" int dynb_forward_backward(dynb_model* m, const float* x, const int32_t* y,
                                     const int32_t* b, int32_t K, float* grads, void* stream) {
  return run_forward_backward(m, x, y, b, K, grads, nullptr, stream);
}

extern "C" int dynb_forward_backward_aggregate(dynb_model* m, const float* x, const int32_t* y,
                                               const int32_t* b, int32_t K, float* grads,
                                               float* out, void* stream) {
  if (!out) return fail(DYNB_ERR_BADARG, "forward_backward_aggregate: null pointer");
  if ((uintptr_t)out & 15)
    return fail(DYNB_ERR_BADARG, "forward_backward_aggregate: out must be 16-byte aligned");
  return run_forward_backward(m, x, y, b, K, grads, out, stream);
}

namespace {
int run_forward_backward(dynb_model* m, const float* x, const int32_t* y, const int32_t* b,
                         int32_t K, float* grads, float* agg, void* stream) {
  if (!m || !x || !y || !b || !grads) return fail(DYNB_ERR_BADARG, "forward_backward: null pointer");
  if (!m->bound) return fail(DYNB_ERR_STATE, "forward_backward: model not bound");
  if (K < 1 || K > m->max_workers)
    return fail(DYNB_ERR_BADARG, "forward_backward: K=%d outside [1, %d]", K, m->max_workers);
  if ((uintptr_t)grads & 15) return fail(DYNB_ERR_BADARG, "forward_backward: grads must be 16-byte aligned");
  Segs s1;   // sample-level segments
  int rc = build_segs(b, K, 1, s1);
  if (rc) return rc;
  const int B = s1.off[K];
  if (B > m->max_batch)
    return fail(DYNB_ERR_BADARG, "forward_backward: sum(b)=%d exceeds max_global_batch=%d", B,
                m->max_batch);
  const int dt = m->dtype, es = elem_size(dt);
  const size_t nL = m->layers.size();
  std::vector<Segs> segs(nL);   // row-level segments of every layer's output
  for (size_t l = 0; l < nL; ++l) {
    rc = build_segs(b, K, m->layers[l].hw_out, segs[l]);
    if (rc) return rc;
  }
  auto in_act = [&](size_t l) -> const void* { return l == 0 ? m->act0 : m->layers[l - 1].out; };

  // dyv[l]: where layer l's gradient is read from -- its own buffer, or (no copy) the buffer of
  // the residual addition above it.  skip_grad[l]: the gradient that reaches a fused skip source
  // over the residual branch; the input-gradient kernel of the layer above adds it.
  std::vector<const void*> dyv(nL), skip_grad(nL, nullptr);
  for (size_t l = 0; l < nL; ++l) dyv[l] = m->layers[l].dy;
  // ---- per-worker weight and bias gradients ----
  Lambdas lam;                  // Eq. 2: lambda_k = b_k / sum_i b_i
  lam.K = K;
  for (int k = 0; k < K; ++k) lam.w[k] = B > 0 ? (float)((double)b[k] / (double)B) : 0.f;
  if (agg && B <= 0) return fail(DYNB_ERR_BADARG, "forward_backward_aggregate: sum(b) must be positive");
  // aggregates of the small tensors (biases, small weights, padding): one launch for all
  Ranges small;
  small.n = 0;
  auto flush_small = [&]() {
    const int r = small.n ? launch_aggregate_ranges(grads, m->P_pad, lam, small, agg, stream) : DYNB_OK;
    small.n = 0;
    return r;
  };
  auto add_small = [&](int64_t off, int64_t len) {
    if (len <= 0) return (int)DYNB_OK;
    small.off[small.n] = off;
    small.len[small.n] = len;
    return ++small.n == MAX_RANGES ? flush_small() : (int)DYNB_OK;
  };
  // Per-worker weight and bias gradients of layer l (and, with `agg`, their aggregate).  Needs
  // the layer's input and the finished gradient wrt its output.
  std::vector<char> wgrad_done(nL, 0);
  auto weight_gradient = [&](size_t l) -> int {
    wgrad_done[l] = 1;
    Layer& L = m->layers[l];
    if (L.kind == DYNB_LAYER_BN) {
      if (B == 0) {   // no backward pass ran: the scale / shift gradients of idle workers are zero
        rc = launch_bn_backward(L.dy, L.ld_out, in_act(l), L.ld_in, L.n_out, m->params + L.w_off,
                                L.bn_mean, L.bn_rstd, m->row_scratch, grads + L.w_off,
                                grads + L.b_off, m->P_pad, 0, 0, nullptr, 0, segs[l], stream);
        if (rc) return rc;
      }
      if (agg) {
        rc = add_small(L.w_off, 2 * (int64_t)L.n_out);
        if (rc) return rc;
      }
      return (int)DYNB_OK;
    }
    if (!L.has_params) return (int)DYNB_OK;
    if (L.kind == DYNB_LAYER_CONV3X3) {
      rc = launch_conv_wgrad(in_act(l), L.ld_in, L.n_in, L.h_in, L.w_in, dyv[l], L.ld_out, L.n_out,
                             L.h_out, L.w_out, L.stride, L.conv_chunk, m->partial, m->partial_floats,
                             grads + L.w_off, grads + L.b_off, m->P_pad, segs[l],
                             2.0 * B * L.hw_out * L.wg_rows * L.n_out,
                             (double)K * L.wg_rows * L.n_out * 4 +
                                 (double)B * (L.hw_in * L.n_in + L.hw_out * L.n_out) * es,
                             stream);
      if (rc) return rc;
      if (agg) {
        rc = add_small(L.w_off, (int64_t)L.wg_rows * L.n_out);
        if (!rc) rc = add_small(L.b_off, L.n_out);
        if (rc) return rc;
      }
      return (int)DYNB_OK;
    }
    GemmArgs g = {};
    g.mode = MODE_WGRAD;
    if (dt == DYNB_BF16) {   // the row-major tensors themselves, reduced over each worker's rows
      g.A = dyv[l]; g.lda = L.ld_out;
      g.B = in_act(l); g.ldb = L.ld_in;
    } else {
      g.A = L.dyT; g.lda = L.capT;
      g.B = L.inT; g.ldb = L.capT;
    }
    g.M = L.n_out; g.N = L.wg_rows;
    g.Cf = grads + L.w_off; g.ldcf = L.n_out;
    g.group_stride = m->P_pad;
    g.alg_flops = 2.0 * B * L.hw_out * L.wg_rows * L.n_out;
    g.alg_bytes = (double)K * L.wg_rows * L.n_out * 4 + (double)B * L.hw_out * (L.wg_rows + L.n_out) * es;
    int deepest = 0;
    for (int k = 0; k < K; ++k) {
      const int d = dt == DYNB_BF16 ? segs[l].off[k + 1] - segs[l].off[k] : segs[l].poff[k + 1] - segs[l].poff[k];
      deepest = d > deepest ? d : deepest;
    }
    int split = (deepest + 255) / 256;               // chunks of at least eight 32-deep stages
    split = split > L.max_split ? L.max_split : split;
    if (split > 1) {
      g.split = split;
      g.chunk = (int)round_up((deepest + split - 1) / split, 64);
      g.partial = m->partial;
      g.partial_stride = round_up((int64_t)L.wg_rows * L.n_out, 64);
    }
    // the aggregate of this weight: in the same kernel while the per-worker tiles are in
    // registers where the launch shape allows it, else by a pass over what was written
    const bool fold = agg && gemm_fuses_aggregate(dt, g, segs[l]);
    if (fold) {
      g.alg_bytes += (double)L.wg_rows * L.n_out * 4;   // the aggregated tile is written too
      g.agg = agg + L.w_off;
      for (int k = 0; k < K; ++k) g.lam[k] = lam.w[k];
    }
    // bf16, unsplit: the bias gradient is formed by the same kernel
    const bool bias_inside = dt == DYNB_BF16 && split <= 1;
    if (bias_inside) g.bias_grad = grads + L.b_off;
    rc = launch_gemm(dt, g, segs[l], stream);
    if (rc) return rc;
    if (split > 1) {
      rc = launch_wgrad_reduce(m->partial, split, g.partial_stride, (int64_t)L.wg_rows * L.n_out,
                               grads + L.w_off, m->P_pad, K, stream);
      if (rc) return rc;
    }
    if (bias_inside)
      rc = DYNB_OK;
    else if (dt == DYNB_BF16)
      rc = launch_bias_grad_rows(dyv[l], L.ld_out, L.n_out, grads + L.b_off, m->P_pad, segs[l], stream);
    else
      rc = launch_bias_grad(dt, L.dyT, L.capT, L.n_out, grads + L.b_off, m->P_pad, segs[l], stream);
    if (rc) return rc;
    if (agg) {
      const int64_t nw = (int64_t)L.wg_rows * L.n_out;
      if (!fold && nw >= 65536) {
        rc = launch_aggregate_range(grads + L.w_off, m->P_pad, lam, nw, agg + L.w_off, stream);
        if (rc) return rc;
      } else if (!fold) {
        rc = add_small(L.w_off, nw);
        if (rc) return rc;
      }
      rc = add_small(L.b_off, L.n_out);
      if (rc) return rc;
    }
    return (int)DYNB_OK;
  };
  if (B > 0) {
    // ---- forward ----
    rc = launch_pack_rows(dt, x, B * m->in_h * m->in_w, m->in_c, m->act0, m->ld0, stream);
    if (rc) return rc;
    for (size_t l = 0; l < nL; ++l) {
      Layer& L = m->layers[l];
      const bool last = l + 1 == nL;
      const int rows_out = B * L.hw_out;
      if (L.kind == DYNB_LAYER_GAP) {
        rc = launch_gap_forward(in_act(l), L.ld_in, L.hw_in, L.n_in, B, L.out, L.ld_out, stream);
        if (rc) return rc;
        continue;
      }
      if (L.kind == DYNB_LAYER_BN) {
        if (L.add_fused) {   // normalisation and the addition behind it in one pass
          const Layer& Add = m->layers[l + 1];
          const Layer& Src = m->layers[Add.skip_from];
          rc = launch_bn_forward(in_act(l), L.ld_in, L.n_out, m->params + L.w_off, m->params + L.b_off,
                                 L.eps, L.relu, L.bn_mean, L.bn_rstd, m->row_scratch, Src.out,
                                 Src.ld_out, Add.relu, Add.out, Add.ld_out, segs[l], stream);
        } else {
          rc = launch_bn_forward(in_act(l), L.ld_in, L.n_out, m->params + L.w_off, m->params + L.b_off,
                                 L.eps, L.relu, L.bn_mean, L.bn_rstd, m->row_scratch, nullptr, 0, 0,
                                 L.out, L.ld_out, segs[l], stream);
        }
        if (rc) return rc;
        continue;
      }
      if (L.kind == DYNB_LAYER_ADD) {
        if (m->layers[l - 1].add_fused) continue;
        const Layer& Src = m->layers[L.skip_from];
        rc = launch_add_forward(in_act(l), L.ld_in, Src.out, Src.ld_out, L.ld_out, rows_out, L.relu,
                                L.out, L.ld_out, stream);
        if (rc) return rc;
        continue;
      }
      GemmArgs g = {};
      g.mode = MODE_FWD;
      g.M = rows_out;
      g.N = L.n_out;
      g.bias = m->params + L.b_off;
      g.relu = L.relu;
      if (last) { g.Cf = m->logits; g.ldcf = L.ld_out; }
      else { g.C = L.out; g.ldc = L.ld_out; }
      if (L.kind == DYNB_LAYER_DENSE) {
        if (dt != DYNB_BF16) {
          rc = launch_transpose(dt, in_act(l), L.ld_in, L.n_in, L.inT, L.capT, segs[l], stream);
          if (rc) return rc;
        }
        g.A = in_act(l); g.lda = L.ld_in;
        g.B = L.Wt; g.ldb = L.ld_in;
        g.K = (int)L.ld_in;
        g.alg_flops = 2.0 * rows_out * L.n_in * L.n_out;
        g.alg_bytes = ((double)rows_out * (L.n_in + L.n_out) + (double)L.n_in * L.n_out) * es;
      } else {
        g.A = in_act(l); g.lda = L.ld_in;
        g.B = L.Wt; g.ldb = L.kf;
        g.K = L.kf;
        g.conv = 1; g.src_h = L.h_in; g.src_w = L.w_in; g.row_h = L.h_out; g.row_w = L.w_out;
        g.stride = L.stride; g.cp = L.cin_p;
        g.alg_flops = 2.0 * rows_out * 9 * L.n_in * L.n_out;
        g.alg_bytes = ((double)B * L.hw_in * L.n_in + (double)rows_out * L.n_out +
                       9.0 * L.n_in * L.n_out) * es;
      }
      rc = launch_gemm(dt, g, s1, stream);
      if (rc) return rc;
    }
    // ---- loss and dlogits (mean over each worker's own b_k samples) ----
    const Layer& Z = m->layers[nL - 1];
    rc = launch_softmax_xent(dt, m->logits, Z.ld_out, y, m->n_classes, Z.dy, Z.ld_out,
                             (int)Z.ld_out, m->rowloss, s1, stream);
    if (rc) return rc;
    // ---- backward: gradient wrt every layer's output, masked by that layer's ReLU ----
    for (size_t l = nL; l-- > 0;) {
      Layer& L = m->layers[l];
      if (L.skip_source && !L.skip_fused) {   // the gradient of the residual branch joins in
        rc = launch_grad_route(L.dy_skip, L.ld_out, nullptr, 0, L.ld_out, (int64_t)B * L.hw_out, 0, 1,
                               L.dy, L.ld_out, stream);
        if (rc) return rc;
      }
      if (L.kind == DYNB_LAYER_DENSE && dt != DYNB_BF16) {
        rc = launch_transpose(dt, dyv[l], L.ld_out, L.n_out, L.dyT, L.capT, segs[l], stream);
        if (rc) return rc;
      }
      const bool below = (int)l > m->first_param_layer;   // does anything below need a gradient?
      if (L.kind == DYNB_LAYER_BN) {
        Layer* Lq = l > 0 ? &m->layers[l - 1] : nullptr;
        rc = launch_bn_backward(dyv[l], L.ld_out, in_act(l), L.ld_in, L.n_out, m->params + L.w_off,
                                L.bn_mean, L.bn_rstd, m->row_scratch, grads + L.w_off,
                                grads + L.b_off, m->P_pad, below, Lq ? Lq->relu : 0,
                                Lq ? Lq->dy : nullptr, Lq ? Lq->ld_out : 0, segs[l], stream);
        if (rc) return rc;
        continue;
      }
      if (!below) continue;
      Layer& Lp = m->layers[l - 1];                   // producer of this layer's input
      const int rows_in = B * L.hw_in;
      if (L.kind == DYNB_LAYER_ADD) {                 // the same gradient goes down both branches
        Layer& Src = m->layers[L.skip_from];
        if (!Lp.relu && !Lp.skip_source) {
          dyv[l - 1] = dyv[l];                        // unchanged: read it where it is
        } else {
          rc = launch_grad_route(dyv[l], L.ld_out, Lp.out, Lp.ld_out, L.ld_out, rows_in, Lp.relu, 0,
                                 Lp.dy, Lp.ld_out, stream);
          if (rc) return rc;
        }
        if (Src.skip_fused) {
          skip_grad[L.skip_from] = dyv[l];
        } else {
          rc = launch_grad_route(dyv[l], L.ld_out, Src.out, Src.ld_out, L.ld_out, rows_in, Src.relu, 0,
                                 Src.dy_skip, Src.ld_out, stream);
          if (rc) return rc;
        }
        continue;
      }
      if (L.kind == DYNB_LAYER_GAP) {
        rc = launch_gap_backward(dyv[l], L.ld_out, Lp.out, Lp.ld_out, L.hw_in, L.n_in, B, Lp.relu,
                                 Lp.dy, Lp.ld_out, stream);
        if (rc) return rc;
        continue;
      }
      GemmArgs g = {};
      g.mode = MODE_DGRAD;
      g.M = rows_in;
      g.N = L.n_in;
      g.C = Lp.dy; g.ldc = Lp.ld_out;
      if (Lp.relu) { g.mask = Lp.out; g.ldmask = Lp.ld_out; }
      if (Lp.skip_source && Lp.skip_fused) { g.addend = skip_grad[l - 1]; g.ldadd = Lp.ld_out; }
      if (L.kind == DYNB_LAYER_DENSE) {
        g.A = dyv[l]; g.lda = L.ld_out;
        g.B = L.Wn; g.ldb = L.ld_out;
        g.K = (int)L.ld_out;
        g.alg_flops = 2.0 * rows_in * L.n_in * L.n_out;
        g.alg_bytes = ((double)rows_in * (L.n_in + L.n_out) + (double)L.n_in * L.n_out) * es;
      } else {
        g.A = dyv[l]; g.lda = L.ld_out;
        g.B = L.Wn; g.ldb = L.kd;
        g.K = L.kd;
        g.conv = 2; g.src_h = L.h_out; g.src_w = L.w_out; g.row_h = L.h_in; g.row_w = L.w_in;
        g.stride = L.stride; g.cp = L.cout_p;
        g.alg_flops = 2.0 * B * L.hw_out * 9 * L.n_in * L.n_out;
        g.alg_bytes = ((double)rows_in * L.n_in + (double)B * L.hw_out * L.n_out +
                       9.0 * L.n_in * L.n_out) * es;
      }
      rc = launch_gemm(dt, g, s1, stream);
      if (rc) return rc;
      // A dense layer's weight gradient right behind its input gradient.  That launch has just
      // read both of the weight gradient's operands in full -- the gradient wrt the layer's
      // output as its own operand, the layer's input as the ReLU mask of its epilogue -- so they
      // sit in the 256 MB last-level cache, from which the eight L2s then re-fetch their panels
      // (five to six times the operands' size per launch).  After the whole chain of input
      // gradients, and after other weight gradients have streamed gigabytes past that cache,
      // those re-fetches come from HBM and compete with the tile stores: 0.29 - 0.31 ms per
      // 4096 x 4096 launch instead of 0.24 - 0.28.
      if (L.kind == DYNB_LAYER_DENSE && dt == DYNB_BF16) {
        // (no ReLU below: the input gradient had no mask to read, so the layer's input gets its
        // own sequential read, as the first layer's does further down)
        const int64_t in_bytes = (int64_t)rows_in * L.ld_in * es;
        if (!Lp.relu && in_bytes >= ((int64_t)16 << 20)) {
          rc = launch_touch(in_act(l), in_bytes, stream);
          if (rc) return rc;
        }
        rc = weight_gradient(l);
        if (rc) return rc;
      }
    }
  }
  // ---- per-worker weight and bias gradients (of the layers the backward pass has not done) ----
  for (size_t l = 0; l < nL; ++l)
    if (!wgrad_done[l]) {
      // (a large first dense layer: no input gradient has read its input, so one sequential
      // pass brings it into the last-level cache first -- 8 us for 32 MB, 50 us off the launch)
      const Layer& L = m->layers[l];
      const int64_t in_bytes = (int64_t)B * L.hw_in * L.ld_in * es;
      if (L.kind == DYNB_LAYER_DENSE && dt == DYNB_BF16 && in_bytes >= ((int64_t)16 << 20)) {
        rc = launch_touch(in_act(l), in_bytes, stream);
        if (rc) return rc;
      }
      rc = weight_gradient(l);
      if (rc) return rc;
    }
  // per-worker losses and zero padding; with an aggregate: the small tensors still on the list
  // and the aggregate's padding [P, P_pad) in the same launch
  return launch_finalize(m->rowloss, m->loss, grads, m->P, m->P_pad, s1, agg ? &lam : nullptr,
                         agg ? &small : nullptr, agg, stream);
}
}  // namespace

// ---- the per-worker gradients without a caller workspace ----------------------------------
// For callers that cannot allocate device memory.  Everything dynb_forward_backward keeps in its
// bound workspace (packed input, stored activations and their gradients, 16-bit weight copies,
// logits, chunk partials) lives in this array instead; each device holds its own copy until the
// process ends.  Host code never uses the array's name as an address: scratch_base() asks the
// runtime for the address on the current device, once per device.
static __device__ __align__(256) unsigned char scratch[DYNB_STATIC_SCRATCH_BYTES];

namespace {

__global__ __launch_bounds__(256) void clear_bytes_kernel(uint4* dst, size_t n16) {
  const uint4 z = {0u, 0u, 0u, 0u};
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16;
       i += (size_t)gridDim.x * blockDim.x)
    dst[i] = z;
}

void* scratch_base() {
  static std::mutex mu;
  static void* known[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> lk(mu);
  if (!known[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
    known[dev] = p;
  }
  return known[dev];
}

}  // namespace

extern "C" size_t dynb_static_scratch_bytes(void) { return DYNB_STATIC_SCRATCH_BYTES; }

extern "C" int dynb_forward_backward_static(const dynb_model* m, const float* params,
                                            const float* x, const int32_t* y, const int32_t* b,
                                            int32_t K, float* grads, void* stream) {
  if (!m || !params || !x || !y || !b || !grads)
    return fail(DYNB_ERR_BADARG, "forward_backward_static: null pointer");
  if (K < 1 || K > DYNB_MAX_WORKERS)
    return fail(DYNB_ERR_BADARG, "forward_backward_static: K=%d outside [1, %d]", K, DYNB_MAX_WORKERS);
  if ((uintptr_t)params & 15)
    return fail(DYNB_ERR_BADARG, "forward_backward_static: params must be 16-byte aligned");
  int64_t B = 0;
  for (int k = 0; k < K; ++k) {
    if (b[k] < 0) return fail(DYNB_ERR_BADARG, "forward_backward_static: negative batch size for worker %d", k);
    B += b[k];
  }
  if (B > ((int64_t)1 << 24))
    return fail(DYNB_ERR_UNSUPPORTED, "forward_backward_static: sum(b) too large");
  const int cap = B > 0 ? (int)B : 1;
  int64_t max_hw = (int64_t)m->in_h * m->in_w;
  for (const Layer& L : m->layers) max_hw = L.hw_out > max_hw ? L.hw_out : max_hw;
  if ((int64_t)cap * max_hw > (int64_t)1 << 30)
    return fail(DYNB_ERR_UNSUPPORTED, "forward_backward_static: sum(b) * pixels exceeds 2^30 rows");
  // a private copy of the plan, laid out for exactly this call's batch and worker count
  dynb_model plan = *m;
  const size_t need = carve(&plan, nullptr, cap, K);
  if (need > (size_t)DYNB_STATIC_SCRATCH_BYTES)
    return fail(DYNB_ERR_UNSUPPORTED,
                "forward_backward_static: this model and batch need %zu bytes of scratch, the "
                "static area holds %zu (use dynb_model_bind + dynb_forward_backward)",
                need, (size_t)DYNB_STATIC_SCRATCH_BYTES);
  void* base = scratch_base();
  if (!base) return fail(DYNB_ERR_HIP, "forward_backward_static: no address for the static scratch area");
  carve(&plan, base, cap, K);
  plan.params = const_cast<float*>(params);   // (read only on this path)
  plan.max_batch = cap;
  plan.max_workers = K;
  plan.bound = true;
  // The area still holds the previous call's contents in another layout: the padding columns the
  // kernels read but never write must be zero again.  A kernel, not a memset node, so that the
  // call can be recorded into a graph.
  const size_t n16 = need / 16;   // (carve() rounds every piece to 256 bytes)
  const unsigned blocks = (unsigned)((n16 + 255) / 256 < 2048 ? (n16 + 255) / 256 : 2048);
  hipLaunchKernelGGL(clear_bytes_kernel, dim3(blocks ? blocks : 1), dim3(256), 0, (hipStream_t)stream,
                     (uint4*)base, n16);
  if (hipGetLastError() != hipSuccess) return fail(DYNB_ERR_HIP, "forward_backward_static: clear failed");
  if (int rc = dynb_model_sync_weights(&plan, stream)) return rc;
  return run_forward_backward(&plan, x, y, b, K, grads, nullptr, stream);
}

namespace {

int make_rule(const dynb_optimizer* opt, const float* s1, const float* s2, UpdateRule& r) {
  if (!opt) return fail(DYNB_ERR_BADARG, "update: null optimizer");
  r = UpdateRule{};
  r.kind = opt->kind;
  r.lr = opt->lr;
  r.mu = opt->momentum;
  switch (opt->kind) {
    case DYNB_OPT_SGD:
      break;
    case DYNB_OPT_MOMENTUM:
      if (!s1) return fail(DYNB_ERR_BADARG, "update: momentum needs state1 (velocity)");
      break;
    case DYNB_OPT_ADAM: {
      if (!s1 || !s2) return fail(DYNB_ERR_BADARG, "update: Adam needs state1 and state2");
      if (opt->step < 1) return fail(DYNB_ERR_BADARG, "update: Adam step numbers start at 1");
      if (!(opt->beta1 >= 0.0 && opt->beta1 < 1.0 && opt->beta2 >= 0.0 && opt->beta2 < 1.0))
        return fail(DYNB_ERR_BADARG, "update: Adam betas must lie in [0, 1)");
      set_adam(r, opt->beta1, opt->beta2, opt->eps, opt->step);
      break;
    }
    default:
      return fail(DYNB_ERR_BADARG, "update: unknown optimizer kind %d", opt->kind);
  }
  if (((uintptr_t)s1 & 15) || ((uintptr_t)s2 & 15))
    return fail(DYNB_ERR_BADARG, "update: optimizer state must be 16-byte aligned");
  return DYNB_OK;
}

// One step over all layers.  Dense weight matrices: the step and both 16-bit copies in one
// pass, MAX_CAST_MATS matrices per launch; the first such launch also steps the small tensors
// (biases, convolution weights, normalisation parameters), whose 16-bit layouts follow.
int update_layers(dynb_model* m, const GradSource& src, const UpdateRule& rule, float* s1,
                  float* s2, void* stream) {
  Ranges r;
  r.n = 0;
  CastMats mats;
  mats.n = 0;
  bool any_dense = false;
  for (Layer& L : m->layers) any_dense = any_dense || (L.has_params && L.kind == DYNB_LAYER_DENSE);
  // without a dense layer, or with more small tensors than one launch takes: element-wise launches
  auto flush_small = [&]() {
    const int rc = r.n ? launch_update_ranges(m->params, r, src, rule, s1, s2, stream) : DYNB_OK;
    r.n = 0;
    return rc;
  };
  auto add = [&](int64_t off, int64_t len) {
    if (len <= 0) return (int)DYNB_OK;
    if (r.n == MAX_RANGES)
      if (int rc = flush_small()) return rc;
    r.off[r.n] = off;
    r.len[r.n] = len;
    ++r.n;
    return (int)DYNB_OK;
  };
  for (Layer& L : m->layers) {
    if (L.kind == DYNB_LAYER_BN) {
      if (int rc = add(L.w_off, 2 * (int64_t)L.n_out)) return rc;
      continue;
    }
    if (!L.has_params) continue;
    int rc = add(L.b_off, L.n_out);
    if (!rc && L.kind != DYNB_LAYER_DENSE) rc = add(L.w_off, (int64_t)9 * L.n_in * L.n_out);
    if (rc) return rc;
  }
  if (!any_dense)
    if (int rc = flush_small()) return rc;
  auto flush_mats = [&]() {
    const int rc = launch_update_cast(m->dtype, m->params, mats, r, src, rule, s1, s2, stream);
    mats.n = 0;
    r.n = 0;   // (the small tensors went with this launch)
    return rc;
  };
  // (last layer first: the first layer's copies are then the most recently written when the next
  // step's forward pass starts with them -- measured 1.5 % of a step on the wide MLP)
  for (size_t li = m->layers.size(); li-- > 0;) {
    Layer& L = m->layers[li];
    if (!L.has_params || L.kind != DYNB_LAYER_DENSE) continue;
    const int i = mats.n++;
    mats.off[i] = L.w_off;
    mats.R[i] = L.n_in;
    mats.C[i] = L.n_out;
    mats.Wn[i] = L.Wn;
    mats.ldn[i] = L.ld_out;
    mats.Wt[i] = L.Wt;
    mats.ldt[i] = L.ld_in;
    if (mats.n == MAX_CAST_MATS)
      if (int rc = flush_mats()) return rc;
  }
  if (mats.n)
    if (int rc = flush_mats()) return rc;
  for (Layer& L : m->layers) {
    if (!L.has_params || L.kind == DYNB_LAYER_DENSE) continue;
    if (int rc = launch_conv_weight_cast(m->params + L.w_off, L.n_in, L.n_out, L.cin_p, L.cout_p, L.Wt,
                                         L.kf, L.Wn, L.kd, stream))
      return rc;
  }
  return DYNB_OK;
}

}  // namespace

extern "C" int dynb_model_update(dynb_model* m, const float* g, const dynb_optimizer* opt,
                                 float* state1, float* state2, void* stream) {
  if (!m || !g) return fail(DYNB_ERR_BADARG, "model_update: null pointer");
  if (!m->bound) return fail(DYNB_ERR_STATE, "model_update: model not bound");
  if ((uintptr_t)g & 15) return fail(DYNB_ERR_BADARG, "model_update: g must be 16-byte aligned");
  UpdateRule rule;
  if (int rc = make_rule(opt, state1, state2, rule)) return rc;
  GradSource src;
  src.g = g;
  src.worker_stride = 0;
  src.lam.K = 0;
  return update_layers(m, src, rule, state1, state2, stream);
}

extern "C" int dynb_model_aggregate_update(dynb_model* m, const float* grads, const int32_t* b,
                                           int32_t K, const dynb_optimizer* opt, float* state1,
                                           float* state2, void* stream) {
  if (!m || !grads || !b) return fail(DYNB_ERR_BADARG, "model_aggregate_update: null pointer");
  if (!m->bound) return fail(DYNB_ERR_STATE, "model_aggregate_update: model not bound");
  if (K < 1 || K > DYNB_MAX_WORKERS) return fail(DYNB_ERR_BADARG, "model_aggregate_update: K out of range");
  if ((uintptr_t)grads & 15)
    return fail(DYNB_ERR_BADARG, "model_aggregate_update: grads must be 16-byte aligned");
  int64_t total = 0;
  for (int k = 0; k < K; ++k) {
    if (b[k] < 0) return fail(DYNB_ERR_BADARG, "model_aggregate_update: negative batch size");
    total += b[k];
  }
  if (total <= 0) return fail(DYNB_ERR_BADARG, "model_aggregate_update: sum(b) must be positive");
  UpdateRule rule;
  if (int rc = make_rule(opt, state1, state2, rule)) return rc;
  GradSource src;
  src.g = grads;
  src.worker_stride = m->P_pad;
  src.lam.K = K;
  for (int k = 0; k < K; ++k) src.lam.w[k] = (float)((double)b[k] / (double)total);   // Eq. 2
  return update_layers(m, src, rule, state1, state2, stream);
}

extern "C" int dynb_model_sgd_update(dynb_model* m, const float* g, float lr, float mu,
                                     float* velocity, void* stream) {
  dynb_optimizer opt{};
  opt.kind = velocity ? DYNB_OPT_MOMENTUM : DYNB_OPT_SGD;
  opt.lr = lr;
  opt.momentum = mu;
  return dynb_model_update(m, g, &opt, velocity, nullptr, stream);
}
