// Internal declarations shared by the library's translation units (not part of the ABI).
#ifndef DYNB_INTERNAL_H
#define DYNB_INTERNAL_H

#include <cstddef>
#include <cstdint>

#include "../../include/dynb.h"

namespace dynb {

// Records a thread-local message and returns `code`.
int fail(int code, const char* fmt, ...);

constexpr int ROW_PAD = 8;    // every worker's row segment is padded to a multiple of this
constexpr int COL_PAD = 64;   // leading dimensions are padded to a multiple of this

inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }

// Row segments of the K workers, passed to kernels by value.
//   off[k]  : first row of worker k in the caller's (dense) batch, off[K] = sum(b)
//   poff[k] : first row of worker k in the padded row space, poff[k+1]-poff[k] = round_up(b_k, 8)
struct Segs {
  int K;
  int off[DYNB_MAX_WORKERS + 1];
  int poff[DYNB_MAX_WORKERS + 1];
};

struct Lambdas {
  int K;
  float w[DYNB_MAX_WORKERS];
};

// A list of index ranges [off, off + len) of the flat parameter vector, passed to kernels by
// value: one launch serves all the small tensors (biases, padding) of a model.
constexpr int MAX_RANGES = 48;
struct Ranges {
  int n;
  int64_t off[MAX_RANGES];
  int64_t len[MAX_RANGES];
};

// Kernel classes for the timing aid.
enum KClass {
  KC_GEMM_FWD = 0,
  KC_GEMM_DGRAD,
  KC_GEMM_WGRAD,
  KC_PACK,
  KC_TRANSPOSE,
  KC_SOFTMAX,
  KC_BIAS_GRAD,
  KC_FINALIZE,
  KC_AGGREGATE,
  KC_UPDATE,
  KC_WEIGHT_CAST,
  KC_CONV_AUX,
  KC_NORM,
  KC_GEMM_WGRAD_SMALL,   // bf16 weight gradients that run on the 128 x 128-tile kernels
  KC_GEMM_SMALL,         // bf16 forward / input-gradient products on the 128 x 128-tile kernel
  KC_COUNT
};

// Brackets one launch with events when timing is on.  flops/bytes are the algorithmic
// work of the launch (accumulated per class).
struct Timed {
  Timed(KClass cls, void* stream, double flops, double bytes);
  ~Timed();
  int cls;             // -1: timing is off
  void* stream;
  void* start;         // hipEvent_t, owned until the destructor queues the pair
  void* stop;
};

enum { MODE_FWD = 0, MODE_DGRAD = 1, MODE_WGRAD = 2 };

// C'[i][j] = sum_k A[i][k] * B[j][k]; both operands are k-contiguous with 16-byte aligned
// rows.  Meaning of (i, j) and of the outputs depends on `mode`:
//   FWD   : i = batch row, j = output feature.  v = acc + bias[j], optional ReLU;
//           C[i*ldc + j] = T(v) if C; Cf[i*ldcf + j] = v if Cf.
//   DGRAD : i = batch row, j = input feature.  v = mask[i*ldmask + j] > 0 ? acc : 0 (mask
//           optional); C[i*ldc + j] = T(v).  With `addend` (bf16 only: the gradient that reaches
//           the same tensor over a residual branch) acc is first rounded to T and
//           addend[i*ldadd + j] added, then the mask is applied.
//   WGRAD : one group per worker g; i = output feature, j = input feature;
//           Cf[g*group_stride + j*ldcf + i] = acc.  fp32: A = dy^T, B = input^T (features x
//           padded rows), operands start at column poff[g], depth poff[g+1]-poff[g].  bf16:
//           A = dy and B = the input as they are, ROW-MAJOR [batch rows][lda / ldb]; worker g
//           owns rows [off[g], off[g+1]) (no transposed copies).
struct GemmArgs {
  const void* A; int64_t lda; int M;   // rows of A  (i)
  const void* B; int64_t ldb; int N;   // rows of B  (j)
  int K;                               // reduction length (FWD/DGRAD), multiple of 8
  int mode;
  const float* bias; int relu;
  void* C; int64_t ldc;
  float* Cf; int64_t ldcf;
  const void* mask; int64_t ldmask;
  const void* addend; int64_t ldadd;   // DGRAD, bf16: see above
  int64_t group_stride;
  int groups_per_block;                // WGRAD, bf16 kernel: workers streamed by one workgroup
  // WGRAD, bf16, unsplit, optional: also write the bias gradient bias_grad[g*group_stride + i] =
  // sum over worker g's rows of A[row][i] (formed in the same kernel as one more column of the
  // product; its weighted aggregate is left to the pass over the small tensors)
  float* bias_grad;
  // Implicit-GEMM gather of operand A for a 3x3 convolution with zero padding 1 (bf16 only).
  // conv == 0: A is a plain matrix.  conv == 1 (forward): row i is output pixel (n, y, x) of a
  // row_h x row_w grid and reduction index k = (kh*3 + kw)*cp + c reads channel c of source
  // pixel (y*stride + kh - 1, x*stride + kw - 1).  conv == 2 (input gradient): row i is input
  // pixel (n, y, x) and k reads channel c of output pixel ((y + 1 - kh)/stride,
  // (x + 1 - kw)/stride) when both divisions are exact.  Out-of-range taps read zero.
  // A points at the source tensor [n * src_h * src_w][lda]; cp is a multiple of 8.
  int conv, src_h, src_w, row_h, row_w, stride, cp;
  // set by launch_gemm: log2(cp) when the cheap addressing applies (cp a power of two >= 32,
  // so that a 32-deep stage lies within one tap; the source pixel of a tap is the row's own
  // pixel plus an offset that is the same for all rows; source tensor below 2 GiB), else -1
  int gather_log2cp;
  double alg_flops, alg_bytes;         // algorithmic work of the launch (timing aid only)
  // WGRAD, bf16 kernel: split every worker's reduction into `split` chunks of `chunk` columns
  // (a multiple of 64).  Chunk c of worker g writes its tile to partial + (g*split + c) *
  // partial_stride (row pitch ldcf); launch_wgrad_reduce sums the chunks in a fixed order.
  // split <= 1: no split, tiles go straight to Cf.
  int split, chunk;
  float* partial;
  int64_t partial_stride;
  // WGRAD, bf16 kernel, optional: also write agg[j*ldcf + i] = sum_g lam[g] * (tile of worker g),
  // summed in a fixed, tile-dependent rotation of ascending g (the weighted aggregation of Eq. 2
  // while the per-worker tiles are still in registers).  Only when gemm_fuses_aggregate() says so.
  float* agg;
  float lam[DYNB_MAX_WORKERS];
  const void* zeros;   // 16 bytes of zeros in device memory (set by launch_gemm): what copies
                       // fetch for rows past a worker's last and taps outside an image
};

int launch_gemm(int dtype, const GemmArgs& a, const Segs& s, void* stream);
// Whether a weight-gradient launch of these dimensions can take GemmArgs::agg.
bool gemm_fuses_aggregate(int dtype, const GemmArgs& a, const Segs& s);
// out[e] = sum_k lam.w[k] * g[k*worker_stride + e], e < n, ascending k (any alignment)
int launch_aggregate_range(const float* g, int64_t worker_stride, const Lambdas& lam, int64_t n,
                           float* out, void* stream);
// the same over every range r: out[off_r + e] from g[k*worker_stride + off_r + e]
int launch_aggregate_ranges(const float* g, int64_t worker_stride, const Lambdas& lam,
                            const Ranges& r, float* out, void* stream);

// x fp32 [rows][D] -> out T [rows][ld]
int launch_pack_rows(int dtype, const float* x, int rows, int D, void* out, int64_t ld,
                     void* stream);
// in T [rows][ldi] -> out T [C][ldo] over the padded row space: out[c][poff_k + r] =
// in[off_k + r][c] for r < b_k, zero for the padding positions of each worker's segment
int launch_transpose(int dtype, const void* in, int64_t ldi, int C, void* out, int64_t ldo,
                     const Segs& s, void* stream);
// logits fp32 [rows][ldz] -> dz T [rows][ldd] (pad columns zero), rowloss[rows]
int launch_softmax_xent(int dtype, const float* logits, int64_t ldz, const int32_t* y, int C,
                        void* dz, int64_t ldd, int ld_cols, float* rowloss, const Segs& s,
                        void* stream);
// grads[g*group_stride + n] = sum over worker g's rows of dyT[n][row]
// ... and from the row-major gradient dy [rows][ld] (bf16; ld a multiple of 64, zeros in the
// padding columns)
int launch_bias_grad_rows(const void* dy, int64_t ld, int N, float* grads, int64_t group_stride,
                          const Segs& s, void* stream);
int launch_bias_grad(int dtype, const void* dyT, int64_t ld, int N, float* grads,
                     int64_t group_stride, const Segs& s, void* stream);
// Reads `bytes` (a multiple of 16, 16-byte aligned) and discards them: what a launch is about to
// fetch several times over, brought into the last-level cache by one sequential pass.
int launch_touch(const void* p, int64_t bytes, void* stream);
// loss[g] = mean of rowloss over worker g's rows; grads[g][P..P_pad) = 0.  With `out` (and lam,
// small): also out[range] = sum_k lam_k grads[k][range] for every range of `small`, and
// out[P..P_pad) = 0, in the same launch.
int launch_finalize(const float* rowloss, float* loss, float* grads, int64_t P, int64_t P_pad,
                    const Segs& s, const Lambdas* lam, const Ranges* small, float* out, void* stream);
int launch_aggregate(const float* grads, const Lambdas& lam, int64_t n, float* out, void* stream);
int launch_sgd(float* params, const float* g, int64_t n, float lr, void* stream);
int launch_momentum(float* params, float* v, const float* g, int64_t n, float lr, float mu,
                    void* stream);
// W fp32 [R][C] (dense) -> Wn T [R][ldn] and Wt T [C][ldt]
int launch_weight_cast(int dtype, const float* W, int R, int C, void* Wn, int64_t ldn, void* Wt,
                       int64_t ldt, void* stream);

// One optimizer step per parameter.  kind: DYNB_OPT_*.  s1 = velocity (momentum) or first
// moment (Adam), s2 = second moment (Adam).  Adam's bias corrections are passed as
// inv_c1 = 1/(1 - beta1^t), inv_c2 = 1/(1 - beta2^t), and omb = 1 - beta, all formed in double.
struct UpdateRule {
  int kind;
  float lr, mu;
  float beta1, beta2, omb1, omb2, eps, inv_c1, inv_c2;
};
// Fills the Adam fields of r for step t (t >= 1, betas in [0, 1)).
void set_adam(UpdateRule& r, double beta1, double beta2, float eps, int64_t t);
// Where the gradient of a parameter comes from: a finished vector g (lam.K == 0), or the K
// per-worker gradients g + k*worker_stride, summed with weights lam.w[k] in ascending k
// (the weighted aggregation of Eq. 2 done on the fly).
struct GradSource {
  const float* g;
  int64_t worker_stride;
  Lambdas lam;
};

// Dense weights W fp32 [R][C] at parameter offset `off`, each with its copies Wn T [R][ldn] and
// Wt T [C][ldt] (T = the model's storage type), passed to the kernel by value.
constexpr int MAX_CAST_MATS = 8;
struct CastMats {
  int n;
  int64_t off[MAX_CAST_MATS];
  int R[MAX_CAST_MATS], C[MAX_CAST_MATS];
  void* Wn[MAX_CAST_MATS];
  int64_t ldn[MAX_CAST_MATS];
  void* Wt[MAX_CAST_MATS];
  int64_t ldt[MAX_CAST_MATS];
  int first_block[MAX_CAST_MATS + 1];   // first workgroup of each matrix (set by the launcher)
};
// One launch: the optimizer step of every matrix of `mats` fused with the refresh of its two
// copies, and the element-wise step of every range of `small`; s1/s2 point at the state of
// parameter 0 (may be null when the rule has no such state)
int launch_update_cast(int dtype, float* params, CastMats& mats, const Ranges& small,
                       const GradSource& src, const UpdateRule& rule, float* s1, float* s2,
                       void* stream);
// element-wise step of parameters [off, off + n) (any alignment)
int launch_update_range(float* params, int64_t off, const GradSource& src, const UpdateRule& rule,
                        float* s1, float* s2, int64_t n, void* stream);
// element-wise step of every range of r
int launch_update_ranges(float* params, const Ranges& r, const GradSource& src, const UpdateRule& rule,
                         float* s1, float* s2, void* stream);
// plain streaming Adam over n parameters (n a multiple of 4, 16-byte aligned pointers)
int launch_adam(float* params, float* m, float* v, const float* g, int64_t n,
                const UpdateRule& rule, void* stream);
// out[g*group_stride + e] = sum_{c < split} partial[(g*split + c)*partial_stride + e], e < n
int launch_wgrad_reduce(const float* partial, int split, int64_t partial_stride, int64_t n,
                        float* out, int64_t group_stride, int K, void* stream);

// ---- convolution helpers (bf16 storage) ----
// out bf16 [9*C][ldo]: transposed patch matrix over the padded pixel positions of segments s
int launch_gap_forward(const void* act, int64_t lda, int HW, int C, int samples, void* pooled,
                       int64_t ldp, void* stream);
int launch_gap_backward(const void* dpooled, int64_t ldp, const void* act, int64_t lda, int HW,
                        int C, int samples, int relu, void* dact, int64_t ldd, void* stream);
int launch_conv_weight_cast(const float* W, int Cin, int Cout, int cin_p, int cout_p, void* Wf,
                            int kf, void* Wd, int kd, void* stream);

// Forward / input gradient of a 3x3 convolution from one halo tile in LDS (conv_direct.hip):
// takes the same description as the gathered-operand GEMM where conv_direct_applies() says so.
bool conv_direct_applies(int dtype, const GemmArgs& a);
int launch_conv_direct(const GemmArgs& a, void* stream);

// The rows of every worker cut into chunks of `rows` rows: first[k] = index of worker k's first
// chunk, first[K] = number of chunks (chunk c of worker k starts at off[k] + (c - first[k]) * rows).
struct RowChunks {
  int rows;
  int first[DYNB_MAX_WORKERS + 1];
};
RowChunks make_row_chunks(const Segs& s, int rows);

// Per-worker weight gradient of a 3x3 convolution straight from the row-major activations
// (bf16 in: [samples*H*W][ldi], dy: [samples*Ho*Wo][ldd]; dW[k * group_stride + (tap*Cin +
// ci)*Cout + co] and the bias gradient db[k * group_stride + co], fp32).  chunk_rows =
// conv_wgrad_chunk_rows(largest row count of the model's plan); scratch:
// conv_wgrad_scratch_floats() floats.
int conv_wgrad_chunk_rows(int64_t max_rows);
int64_t conv_wgrad_scratch_floats(int64_t max_rows, int max_workers, int Cin, int Cout);
int launch_conv_wgrad(const void* in, int64_t ldi, int Cin, int H, int W, const void* dy, int64_t ldd,
                      int Cout, int Ho, int Wo, int stride, int chunk_rows, float* scratch,
                      int64_t scratch_floats, float* dW, float* db, int64_t group_stride,
                      const Segs& s, double flops, double bytes, void* stream);

// Batch normalisation over each worker's own rows (bf16; x: T [rows][ldx], y: T [rows][ldy]):
// writes mean / rstd [k][C] (kept for the backward pass).  `scratch`: row_scratch_floats() floats
// (the partial results of the row chunks), shared by forward and backward.
constexpr int BN_CHUNK_ROWS = 256;
int64_t row_scratch_floats(int64_t max_rows, int max_workers, int C);
// With `skip` (a residual addition fused in): y = relu_sum?(T(normalised) + skip).
int launch_bn_forward(const void* x, int64_t ldx, int C, const float* gamma, const float* beta,
                      float eps, int relu, float* mean, float* rstd, float* scratch,
                      const void* skip, int64_t lds_, int relu_sum, void* y, int64_t ldy,
                      const Segs& s, void* stream);
// dgamma / dbeta[k * group_stride + c] (fp32, per worker) from dy (already masked by the layer's
// own ReLU); with need_dx also dx (T [rows][ldo]), masked by x > 0 when relu_below
int launch_bn_backward(const void* dy, int64_t ldd, const void* x, int64_t ldx, int C,
                       const float* gamma, const float* mean, const float* rstd, float* scratch,
                       float* dgamma, float* dbeta, int64_t group_stride, int need_dx,
                       int relu_below, void* dx, int64_t ldo, const Segs& s, void* stream);
// out = relu?(a + b) over `width` (padded, a multiple of 8) columns of `rows` rows
int launch_add_forward(const void* a, int64_t lda, const void* b, int64_t ldb, int64_t width,
                       int64_t rows, int relu, void* out, int64_t ldo, void* stream);
// dst = (accumulate ? dst : 0) + (relu ? src where act > 0 : src), same extent convention
int launch_grad_route(const void* src, int64_t lds_, const void* act, int64_t lda, int64_t width,
                      int64_t rows, int relu, int accumulate, void* dst, int64_t ldd, void* stream);

}  // namespace dynb

#endif
