// Internal declarations shared by the host code and the kernel launchers of libvf.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "vf.h"

namespace vf {

// ---------------------------------------------------------------------------------------
// errors
// ---------------------------------------------------------------------------------------
void set_last_error(const char* what, hipError_t e, const char* file, int line);
void set_last_error_text(const std::string& s);

#define VF_HIP(expr)                                              \
  do {                                                            \
    hipError_t e__ = (expr);                                      \
    if (e__ != hipSuccess) {                                      \
      ::vf::set_last_error(#expr, e__, __FILE__, __LINE__);       \
      return VF_EDEVICE;                                          \
    }                                                             \
  } while (0)

#define VF_TRY(expr)            \
  do {                          \
    int rc__ = (expr);          \
    if (rc__ != VF_OK) return rc__; \
  } while (0)

#define VF_LAUNCH_CHECK() VF_HIP(hipGetLastError())

// ---------------------------------------------------------------------------------------
// element types
// ---------------------------------------------------------------------------------------
typedef uint16_t bf16_t;   // raw bfloat16 bits

// Where a gradient-producing kernel puts a value v for flat index p:
//   accumulate == 0 :  dst[p] = alpha * v            (written as fma(alpha, v, 0))
//   accumulate != 0 :  dst[p] = fma(alpha, v, dst[p])
// With the staging vector: alpha = 1, accumulate = 0.  Fused into the gradient buffer:
// alpha = b_i/B, accumulate = (node index > 0).
struct GradOut {
  float* dst;
  float alpha;
  int accumulate;
};

// Epilogue of a GEMM:  C[m,n] = fma(alpha, acc[m,n], fma(beta, R[m,n], bias[n]))
// (with bias = 0 and beta = 1 this is the single fused multiply-add R + alpha*acc).
struct Epilogue {
  float alpha = 1.f;
  const float* bias = nullptr;   // fp32 [N] or null
  int bias_round_bf16 = 0;       // round bias values to bf16 before adding
  const float* R = nullptr;      // fp32 addend (may alias C) or null
  int64_t ldr = 0;
  float beta = 0.f;
  void* C = nullptr;
  int64_t ldc = 0;
  int c_is_bf16 = 0;             // store C as bf16 (RNE) instead of fp32
  int stream_c = 0;              // store C with the non-temporal hint (it is not kept in the L2s)
};

// BatchNorm + ReLU backward of whole nodes of 128 rows, taken inside the epilogue of the product that
// computes the incoming gradient (launch_gemm_bf16_bn_bwd): the layer's stored pre-activations and
// per-node statistics in, the bf16 gradient at the pre-activation and its transposed copy out, and
// per node the two column sums that the scale / shift (or bias) gradients are made of.
struct BnBwdArgs {
  const float* z = nullptr;      // pre-activations [M, N], fp32
  int64_t ldz = 0;
  const float* mean = nullptr;   // [nodes, N] (unused without BatchNorm)
  const float* rstd = nullptr;
  const float* gamma = nullptr;  // [N], or null: ReLU only
  const float* beta = nullptr;
  int round_params = 0;          // gamma, beta rounded to bf16 first
  bf16_t* dz = nullptr;          // [M, N]
  int64_t lddz = 0;
  bf16_t* dzT = nullptr;         // [N, ldt]: column = row of the unit, values times tscale
  int64_t ldt = 0;
  float tscale = 1.f;
  float* sums = nullptr;         // [nodes][2][N]: sum over the node's rows of dr * xhat, and of dr
};

// BatchNorm + ReLU forward of whole nodes of 128 rows inside the epilogue of the product that computes
// the layer's pre-activations (launch_gemm_bf16_bn_fwd): the pre-activations are stored as usual (the
// backward pass needs them), and with them the bf16 activation, its transposed copy and the per-node
// statistics; `var` receives the per-node biased variances for the small launch that blends the
// moving statistics in node order.
struct BnFwdArgs {
  float* z = nullptr;            // pre-activations [M, N], fp32 (written)
  int64_t ldz = 0;
  const float* gamma = nullptr;  // [N], or null: bias + ReLU only
  const float* beta = nullptr;
  const float* bias = nullptr;   // [N] or null (layers without BatchNorm)
  int round_params = 0;          // gamma, beta, bias rounded to bf16 first
  float eps = 0.f;
  bf16_t* a = nullptr;           // activation [M, N]
  int64_t lda = 0;
  bf16_t* aT = nullptr;          // [N, ldt]: column = row of the unit
  int64_t ldt = 0;
  float* mean = nullptr;         // [nodes, N] (BatchNorm only)
  float* rstd = nullptr;
  float* var = nullptr;          // [nodes, N] scratch (BatchNorm only)
};

// ---------------------------------------------------------------------------------------
// kernel launchers (each returns VF_OK or VF_EDEVICE/VF_EINVAL); all asynchronous
// ---------------------------------------------------------------------------------------

// k_accum_opt.hip
int launch_accumulate(float* buf, const float* g, float w, int64_t n, int first, hipStream_t s);
int launch_sgdm(float* theta, float* v, const float* G, float lr, float mu, int64_t n, hipStream_t s);
int launch_adam(float* theta, float* m, float* u, const float* G, float lr, float b1, float b2,
                float eps, float inv_c1, float inv_c2, int64_t n, hipStream_t s);
int launch_fill_f32(float* p, float value, int64_t n, hipStream_t s);

// k_gemm_f32.hip:  acc[m,n] = sum_k A[m*sam + k*sak] * B[n*sbn + k*sbk]   (fp32)
// The contraction may be cut into nsplit slices as for the bf16 kernel (slab s at
// ep.C + s*slab_stride elements; no R with nsplit > 1).
int launch_gemm_f32(const float* A, int64_t sam, int64_t sak, const float* B, int64_t sbn,
                    int64_t sbk, int M, int N, int K, int nsplit, int64_t slab_stride,
                    const Epilogue& ep, hipStream_t s);
int gemm_f32_pick_split(int M, int N, int K);

// k_gemm_bf16.hip: acc[m,n] = sum_k A[m*lda + k] * B[n*ldb + k]  (bf16 operands, fp32 MFMA
// accumulation).  lda, ldb multiples of 8, A and B 16-byte aligned.  The contraction is cut
// into nsplit slices; slice s goes to ep.C + s*slab_stride elements (the consumer adds the
// slabs in order).  With nsplit > 1 the epilogue may not add R; the bias goes to slab 0.
int launch_gemm_bf16(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, int M, int N,
                     int K, int nsplit, int64_t slab_stride, const Epilogue& ep, hipStream_t s);
// The product A B^T [M, N] (no bias, no addend, unsliced) followed, tile by tile inside the kernel, by
// the BatchNorm + ReLU backward pass of the layer it arrives at; every node has 128 rows.
// gemm_bf16_bn_bwd_takes: whether the fused kernel takes these operands (whole 256 x 256 tiles, enough
// of them, alignments); the launch returns VF_EINVAL otherwise.
bool gemm_bf16_bn_bwd_takes(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, int M, int N, int K,
                            const BnBwdArgs& fa);
int launch_gemm_bf16_bn_bwd(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, int M, int N, int K,
                            const BnBwdArgs& fa, hipStream_t s);
// The same for the forward pass: A B^T [M, N] stored as the pre-activations, and BatchNorm + ReLU of
// whole nodes of 128 rows applied to it tile by tile inside the kernel.
bool gemm_bf16_bn_fwd_takes(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, int M, int N, int K,
                            const BnFwdArgs& fa);
int launch_gemm_bf16_bn_fwd(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, int M, int N, int K,
                            const BnFwdArgs& fa, hipStream_t s);
// Moving statistics blended with the per-node batch statistics, node after node (Section 4.1).
int launch_bn_stats_finish(const float* mean, const float* var, int nodes, int C, float* run_mean, float* run_var,
                           float run_mix, hipStream_t s);
// Scale / shift (or bias) gradients from the per-node column sums, added up in node order.
int launch_bn_sums_finish(const float* sums, int nodes, int C, GradOut gout_g, GradOut gout_b, hipStream_t s);
// Number of slices that fills the chip for this shape (1 when the tile grid already does).
int gemm_bf16_pick_split(int M, int N, int K);

// Weight gradients of `count` consecutive nodes folded into C in one pass over it:
//   C <- fma(w[count-1], A[count-1] B[count-1]^T, ... fma(w[0], A[0] B[0]^T, overwrite ? 0 : C))
// A[j]: bf16 [M, ld] (rows = input features, K[j] <= 128 node rows contiguous), B[j]: bf16 [N, ld].
constexpr int kFoldMax = 8;
struct FoldArgs {
  const bf16_t* A[kFoldMax];
  const bf16_t* B[kFoldMax];
  int K[kFoldMax];
  float w[kFoldMax];
  int count;
  int overwrite;
};
int launch_gemm_bf16_fold(const FoldArgs& fa, int64_t ld, int M, int N, float* C, int64_t ldc, hipStream_t s);
// 3x3 convolution (stride 1, zero padding 1) of a channels-last bf16 image stack x [rows, Cin],
// rows = images*H*W, Cin % 64 == 0, with filters Wk [N, 9*Cin] (row pitch ldb), as a product
// whose first operand is read straight from x; epilogue as launch_gemm_bf16.  zeros: 128 bytes
// of device memory holding 0.  With `stats` (room for kConvStatsChunks * 2 * N floats) the kernel
// that takes the shape may also leave per-chunk, per-channel (mean, sum of squared deviations) of
// what it stored, chunk k covering rows [k * *stats_rows, (k + 1) * *stats_rows): *stats_chunks
// chunks (0: none were written), in the layout launch_bn2d_stats_finish reads.
constexpr int kConvStatsChunks = 256;
int launch_conv3x3_bf16(const bf16_t* x, int64_t rows, int H, int W, int Cin, const bf16_t* Wk, int64_t ldb, int N,
                        const Epilogue& ep, const bf16_t* zeros, hipStream_t s, float* stats = nullptr,
                        int* stats_chunks = nullptr, int* stats_rows = nullptr);

// The small per-node launches of a fold window, batched: `count` nodes, node j with rows[j] rows.
struct NodeList {
  const bf16_t* src[kFoldMax];
  bf16_t* dst[kFoldMax];
  int rows[kFoldMax];
  float w[kFoldMax];
  int count;
  int overwrite;
};
// dst[j][c*ldo + r] = src[j][r*ldi + c] for every node j (r < rows[j], c < C): k_elem.hip
int launch_transpose_nodes(const NodeList& nl, int64_t ldi, int64_t ldo, int C, hipStream_t s);
// out[r] <- fma(w[count-1], S_{count-1}[r], ... fma(w[0], S_0[r], overwrite ? 0 : out[r])) with
// S_j[r] = sum over c < rows[j] of src[j][r*ld + c], r < R (bias gradients of a window from the
// transposed output gradients; the same chain as one launch per node): k_norm.hip
int launch_rowsum_nodes(const NodeList& nl, int64_t ld, int R, float* out, hipStream_t s);

// k_elem.hip
// out[c*ldo + r] = in[r*ldi + c]  for r < R, c < C
// Up to kTransposeJobs bf16 matrices [R, C_j] (row pitch ldi_j) transposed in one launch into
// out_j [C_j, ldo]: column counts and pitches multiples of 8, ldo >= R rounded up to 8, bases
// 16-byte aligned (VF_EINVAL otherwise: the caller transposes one by one).
constexpr int kTransposeJobs = 4;
struct TransposeJobs {
  const bf16_t* in[kTransposeJobs];
  int64_t ldi[kTransposeJobs];
  bf16_t* out[kTransposeJobs];
  int C[kTransposeJobs];
  int count;
  int R;
  int64_t ldo;
};
int launch_transpose_bf16_jobs(const TransposeJobs& tj, hipStream_t s);
int launch_transpose_bf16(const bf16_t* in, int64_t ldi, bf16_t* out, int64_t ldo, int R, int C,
                          hipStream_t s);
// fp32 [R,C] (ld = C) -> bf16 natural copy [R, ldn] and transposed copy [C, ldt]
int launch_cast_weight(const float* w, int R, int C, bf16_t* nat, int64_t ldn, bf16_t* tr,
                       int64_t ldt, hipStream_t s);
// fp32 [R,C] -> bf16 [R,C] with the given leading dimensions
int launch_cast_bf16(const float* in, int64_t ldi, bf16_t* out, int64_t ldo, int R, int C,
                     hipStream_t s);

// k_norm.hip -- T is float or bf16_t (is_bf16 selects)
// BatchNorm over the R rows given + ReLU.  zp: nsplit partial slabs (slab elements apart,
// leading dimension ldzp) of the Linear output; their sum is written to z (saved for the
// backward pass; with one slab, zp may be z itself and nothing is copied).  a = relu(gamma*xhat + beta) as T; aT (optional, bf16 only) the same
// transposed, [C, ldt].  Saves mean, rstd.  With gamma == nullptr: a = relu(z).
// run_mean / run_var (both or neither): moving statistics, blended in place with the pass's
// own: run += run_mix * (stat - run), biased variance.
// group = 2 .. 8 (bf16): the rows are `group` nodes one after the other, of R rows each or, with
// node_rows (host array), of node_rows[n] rows (each at most 128, multiples of 8 when aT is
// given); statistics, the blend of the moving statistics and (in the backward kernel) the
// small-vector gradients are taken per node in node order; mean and rstd hold `group` vectors of
// C, the transposed copies every node's rows at the columns of its rows.
int launch_bn_relu_fwd(const float* zp, int nsplit, int64_t slab, int64_t ldzp, int R, int C,
                       const float* gamma, const float* beta, int round_params, float eps, float* z,
                       int64_t ldz, void* a, int64_t lda, int a_is_bf16, bf16_t* aT, int64_t ldt,
                       float* mean, float* rstd, float* run_mean, float* run_var, float run_mix,
                       hipStream_t s, int group = 1, const int* node_rows = nullptr);
// Backward of the above.  dap: nsplit partial slabs of the fp32 gradient w.r.t. a (slab 0 is
// overwritten when nsplit > 1).  Writes dz (T), dzT (optional, bf16, [C, ldt]) and, with
// BatchNorm, dgamma/dbeta through GradOut; without BatchNorm (gamma == nullptr) the bias
// gradient (column sums of dz) through gout_b.  nsplit must be a power of two <= 32.
// tscale: the transposed copy holds tscale * dz (rounded once, from the fp32 value).
int launch_bn_relu_bwd(float* dap, int nsplit, int64_t slab, int64_t ldda, const float* z,
                       int64_t ldz, int R, int C, const float* gamma, const float* beta,
                       int round_params, const float* mean, const float* rstd, void* dz, int64_t lddz,
                       int dz_is_bf16, bf16_t* dzT, int64_t ldt, GradOut gout_g, GradOut gout_b,
                       hipStream_t s, float tscale = 1.f, int group = 1, const int* node_rows = nullptr);
// out[r] = sum_c x[r*ld + c] through GradOut (bias gradient from a transposed bf16 gradient)
int launch_rowsum_bf16(const bf16_t* x, int64_t ld, int R, int C, GradOut out, hipStream_t s);
// out[c] = sum_r x[r*ld + c] through GradOut (x is T)
int launch_colsum(const void* x, int64_t ld, int x_is_bf16, int R, int C, GradOut out,
                  hipStream_t s);

// k_conv.hip -- the convolutional family: 3x3 convolutions (stride 1, zero padding 1, NHWC) as
// products over patch rows, BatchNorm over a node's n*H*W positions in chunks of rows.
int conv_chunks(int64_t rows);     // row chunks of the tall reductions: sizes their partial buffers (2*C floats each)
// cols[r, (kh*3+kw)*C + c] = x[n, h+kh-1, w+kw-1, c] or 0; row pitch Kp >= 9C, a multiple of 8
int launch_im2col3x3(const bf16_t* x, int64_t rows, int H, int W, int C, bf16_t* cols, int64_t Kp, hipStream_t s);
// the same patches transposed, [9C, ldo] (positions along the row), from the transposed input
// xT [C, ldx]; the padding of a row up to ldo is written as 0
int launch_im2col3x3_transposed(const bf16_t* xT, int64_t ldx, int64_t rows, int H, int W, int C, bf16_t* colsT,
                                int64_t ldo, hipStream_t s);
// bf16 copies of fp32 filters [Cout, 3, 3, Cin]: as they are (row pitch Kp) and, if flip != null,
// turned by 180 degrees with the channel roles exchanged, [Cin, 3, 3, Cout] (row pitch Kpf)
int launch_conv_weight_copies(const float* Wf, int Cout, int Cin, bf16_t* nat, int Kp, bf16_t* flip, int Kpf,
                              hipStream_t s);
// per-column mean and 1/sqrt(biased variance + eps) of y [rows, C]; moving statistics blended
int launch_bn2d_stats(const float* y, int64_t rows, int C, float eps, float* partial, float* mean, float* rstd,
                      float* run_mean, float* run_var, float run_mix, hipStream_t s);
// the second half of the above alone: per-chunk (mean, sum of squared deviations) already in
// `partial` ([chunk][2][C]), chunk k covering rows [k * rows_per_chunk, (k + 1) * rows_per_chunk)
int launch_bn2d_stats_finish(const float* partial, int nchunk, int rows_per_chunk, int64_t rows, int C, float eps,
                             float* mean, float* rstd, float* run_mean, float* run_var, float run_mix, hipStream_t s);
// a = relu(gamma * (y - mean) * rstd + beta (+ skip)) as bf16
int launch_bn2d_apply_fwd(const float* y, int64_t rows, int C, const float* gamma, const float* beta, int round_params,
                          const float* mean, const float* rstd, const bf16_t* skip, bf16_t* a, hipStream_t s);
// backward of the above given da (gradient w.r.t. a): dgamma, dbeta into the gradient; dy (bf16)
// the gradient w.r.t. y; with keep_dpre, da is replaced by the gradient w.r.t. the ReLU's input
int launch_bn2d_bwd(float* da, const bf16_t* a, const float* y, int64_t rows, int C, const float* gamma,
                    int round_params, const float* mean, const float* rstd, float* partial, float* sums,
                    int keep_dpre, bf16_t* dy, GradOut gout_g, GradOut gout_b, hipStream_t s);
int launch_avgpool_fwd(const bf16_t* a, int n_img, int HW, int C, bf16_t* pooled, int64_t ldp, hipStream_t s);
int launch_avgpool_bwd(const float* dpooled, int64_t ldd, int n_img, int HW, int C, float* da, hipStream_t s);
// dW[o, (kh, kw, c)] = sum over positions of dy[r, o] * x[r + (kh-1) W + (kw-1), c] (0 outside the
// image) straight from dy [rows, Cout] and x [rows, Cin] (bf16, channels last), as up to max_split
// slabs [Cout, 9 Cin] (slab_stride floats apart) of partial sums over slices of the positions, to
// be added in order; *nsplit_out slabs are written.  `zeros`: 128 bytes of 0.
// conv_wgrad_direct_fits: Cout % 64 == 0, Cin % 64 == 0, W in {8, 16, 32, 64}, H a multiple of
// 64 / W, rows a multiple of 64.
bool conv_wgrad_direct_fits(int Cout, int Cin, int H, int W, int64_t rows);
int launch_conv_wgrad_direct(const bf16_t* dy, int Cout, const bf16_t* x, int Cin, int64_t rows, int H, int W,
                             const bf16_t* zeros, float* slabs, int64_t slab_stride, int max_split, int* nsplit_out,
                             hipStream_t s);
// out (+)= alpha * (slab 0 + slab 1 + ...), slabs in order
int launch_fold_slabs(const float* slabs, int nsplit, int64_t stride, int64_t n, GradOut out, hipStream_t s);

// k_loss.hip
// Softmax cross-entropy over R rows of fp32 logits with C classes.  zp: nsplit partial slabs
// of the logits (summed into z, which may be slab 0 itself):
//   rowloss[r] = logsumexp(z_r) - z_r[label_r];  dz[r,c] = (softmax(z_r)[c] - [c==label_r]) / R
// dzT (optional, bf16 only): tscale times the same gradient (rounded once, from the fp32 value),
// transposed, [C, ldt].
// With node_loss != null the node's loss bookkeeping (launch_loss_reduce) follows.
int launch_softmax_xent(const float* zp, int nsplit, int64_t slab, int64_t ldzp, float* z, int64_t ldz,
                        const int32_t* labels, int R, int C, float* rowloss, void* dz, int64_t lddz,
                        int dz_is_bf16, bf16_t* dzT, int64_t ldt, float w, int node, float* node_loss,
                        float* total, hipStream_t s, float tscale = 1.f);
// node_loss[i] = (1/R) sum_r rowloss[r];  total = (i == 0 ? 0 : total) + w * node_loss[i]
// The same for nodes first .. first+count-1 in one launch (rows of node j at rowloss + off[j]).
constexpr int kLossNodes = 32;
struct LossNodes {
  int32_t off[kLossNodes];
  int32_t rows[kLossNodes];
  float w[kLossNodes];
  int32_t first, count;
};
int launch_loss_reduce_nodes(const float* rowloss, const LossNodes& ln, float* node_loss, float* total,
                             hipStream_t s);
int launch_loss_reduce(const float* rowloss, int R, float w, int node, float* node_loss,
                       float* total, hipStream_t s);

// k_bgemm.hip -- batched strided GEMM for the attention contractions.
// Element [b][i,k] of an operand lives at p + (b / inner)*outer + (b % inner)*inner + i*rs + k*cs.
struct BMat {
  const void* p;
  int is_bf16;
  int64_t outer, inner, rs, cs;
  int round_bf16 = 0;   // fp32 storage, but values enter the product rounded to bf16
};
// C[b][m,n] = alpha * sum_k A[b][m,k] * B[b][n,k], b < batch (<= 65535)
int launch_bgemm(const BMat& A, const BMat& B, const BMat& C, int M, int N, int K, int batch, int inner,
                 float alpha, hipStream_t s);

// k_attn.hip -- fused self-attention on the matrix cores (bf16, head size 64, sequence length
// 32, 64 or 128).  qkv: [n_seq*T, 3d] (q | k | v, heads side by side); prob: [n_seq*heads, T, T]
// softmax probabilities (written by the forward pass, read by the backward pass); om: [n_seq*T, d].
bool attn_mfma_supported(int seq_len, int d_head);
int launch_attn_fwd(const bf16_t* qkv, int n_seq, int seq_len, int d, int n_heads, bf16_t* prob, bf16_t* om,
                    float scale, hipStream_t s);
// dO: fp32 [n_seq*T, d] gradient w.r.t. om (rounded to bf16 as it is staged); dqkv: [n_seq*T, 3d]
int launch_attn_bwd(const float* dO, const bf16_t* qkv, const bf16_t* prob, int n_seq, int seq_len, int d,
                    int n_heads, bf16_t* dqkv, float scale, hipStream_t s);

// k_encoder.hip -- element-wise and row-wise kernels of the encoder
// h[r,:] = tok[ids[r]] + pos[r % T]   (table values rounded to bf16 when round_params)
int launch_embed_fwd(const int32_t* ids, const float* tok, const float* pos, int R, int T, int d,
                     int vocab, int round_params, float* h, hipStream_t s);
// pos table gradient: gpos[t,:] = sum over sequences of dh[seq*T + t, :]
int launch_embed_pos_bwd(const float* dh, int nseq, int T, int d, GradOut out, hipStream_t s);
// token table gradient: row ids[r] += dh[r,:], duplicates added in increasing r (deterministic)
int launch_embed_tok_bwd(const int32_t* ids, const float* dh, int R, int d, int vocab, GradOut out,
                         hipStream_t s);
// rowidx[s*m + j] = s*T + pos(s,j);  labels[s*m + j] = target(s,j)   from y [nseq, 2, m]
int launch_extract_masked(const int32_t* y, int nseq, int m, int T, int vocab, int32_t* rowidx,
                          int32_t* labels, hipStream_t s);
// LayerNorm over the last axis.  x row for output row r is x[row_map ? row_map[r] : r].
int launch_layernorm_fwd(const float* x, int64_t ldx, const int32_t* row_map, int R, int d,
                         const float* gamma, const float* beta, int round_params, float eps, void* y,
                         int64_t ldy, int y_is_bf16, float* mean, float* rstd, hipStream_t s);
// Row-chunked reductions: column sums use a scratch of kReduceChunks * columns floats, the
// LayerNorm backward one of 2 * kLnChunks * d floats.
constexpr int kReduceChunks = 128;
constexpr int kLnChunks = 1024;
// The second, small kernel of a row-chunked reduction (chunk partials of a column added in a
// fixed order, result through GradOut) can be put off: a launcher that is handed a FinishList and
// finds room in it writes its partials to a slice of the list's scratch, notes the job and
// returns; launch_finish_jobs then runs all noted jobs in ONE launch -- each with the arithmetic
// of the kernel it stands for -- and empties the list.  Everything on one stream; a job's target
// must not be read before that launch.  A full list (jobs or scratch) makes the launcher finish
// at once, as without a list.
struct FinishJob {
  const float* partial;
  int64_t pstride;       // LayerNorm parameters: distance from the gamma partials to the beta partials
  int nchunk, C, kind;   // kind 0: column sums (GradOut a); 1: LayerNorm gamma (a) and beta (b)
  GradOut a, b;
};
constexpr int kFinishJobs = 32;
struct FinishList {
  FinishJob job[kFinishJobs];
  int count = 0;
  float* scratch = nullptr;
  size_t cap = 0, used = 0;          // floats
  float* take(size_t n) {
    if (!scratch || count >= kFinishJobs || used + n > cap) return nullptr;
    float* p = scratch + used;
    used += (n + 3) & ~(size_t)3;    // slices stay 16-byte aligned
    return p;
  }
};
int launch_finish_jobs(FinishList& list, hipStream_t s);

// dx[orow] = LNbwd(sum of dy slabs)[r] (+ dres[orow]),  orow = row_map ? row_map[r] : r; also
// dgamma[c] = sum_r dy[r,c]*xhat[r,c] and dbeta[c] = sum_r dy[r,c] through GradOut (row chunks
// added in order).  d <= 1024.  scratch: 2 * kLnChunks * d floats.
int launch_layernorm_bwd(const float* dyp, int nsplit, int64_t slab, int64_t lddy, const float* x,
                         int64_t ldx, const int32_t* row_map, int R, int d, const float* gamma,
                         int round_params, const float* mean, const float* rstd, const float* dres,
                         float* dx, int64_t lddx, float* scratch, GradOut gout_g, GradOut gout_b,
                         hipStream_t s, FinishList* defer = nullptr);
// out[c] = sum_r x[r*ld + c] for many rows: partial sums per row chunk, then the chunks in order.
// scratch: kReduceChunks * C floats.
int launch_colsum_rows(const void* x, int64_t ld, int x_is_bf16, int R, int C, float* scratch, GradOut out,
                       hipStream_t s, FinishList* defer = nullptr);
// The gradient dy [R, C] at the output of a Linear layer, prepared for that layer's backward pass
// in one pass: transposed bf16 copy tr [C, ldt], (fp32 dy) bf16 copy nat [R, ldn], and the column
// sums (the bias gradient) through GradOut, 64-row tiles added in order.  dy_prepare_fits says
// whether the shapes qualify (alignment of the leading dimensions, at most kReduceChunks row
// tiles); bases 16-byte aligned; scratch: kReduceChunks * C floats.
bool dy_prepare_fits(int dy_is_f32, int64_t ldi, int64_t ldn, int64_t ldt, int R, int C);
int launch_dy_prepare(const void* dy, int dy_is_f32, int64_t ldi, int R, int C, bf16_t* nat, int64_t ldn,
                      bf16_t* tr, int64_t ldt, float* scratch, GradOut out, hipStream_t s,
                      FinishList* defer = nullptr);
// exact GELU: g = 0.5 u (1 + erf(u / sqrt 2));  u fp32 (a Linear layer's output), g T
int launch_gelu_fwd(const float* u, void* g, int g_is_bf16, int64_t n, hipStream_t s);
// du = dg * (Phi(u) + u phi(u));  dg and u fp32, du T
int launch_gelu_bwd(const float* dg, const float* u, void* du, int du_is_bf16, int64_t n, hipStream_t s);
// row softmax in place over fp32 S [rows, n] -> P written as T to p (and nothing else)
int launch_softmax_rows(const float* S, void* P, int p_is_bf16, int64_t rows, int n, hipStream_t s);
// dS = P * (dP - sum_j dP*P) in place over dP (fp32); P is T
int launch_softmax_rows_bwd(float* dP, const void* P, int p_is_bf16, int64_t rows, int n, hipStream_t s);
// out[r,c] = sum of slabs
int launch_reduce_slabs(const float* in, int nsplit, int64_t slab, int64_t n, float* out, hipStream_t s);

}  // namespace vf
