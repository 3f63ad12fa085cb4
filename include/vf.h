/*
 * libvf -- virtual-node training step on one AMD MI355X (gfx950).
 *
 * One step of the method of "VirtualFlow: Decoupling Deep Learning Models from the
 * Underlying Hardware" (arxiv 2009.09523), Section 3.2 (virtual node execution,
 * steps 1-5 of its Figure 4) with the size weights of Section 5.2:
 *
 *   a batch of B samples is split into V virtual nodes of sizes b_i (sum b_i = B);
 *   the nodes are run one after another on the accelerator, each with its own forward
 *   and backward pass (BatchNorm statistics over that node's rows only, Section 4.1);
 *   each node's gradient g_i is folded into one model-sized fp32 gradient buffer with
 *   weight b_i / B; one optimizer update is applied after the last node.
 *
 * Conventions for every entry point
 *   - returns VF_OK (0) or a negative VF_E* code; never throws or aborts;
 *   - "device" pointers are HIP device memory on the device current at vf_init;
 *     "host" pointers are ordinary host memory;
 *   - the caller owns params, batch and output buffers; the library owns its context
 *     (workspace, gradient buffer, staging, optimizer state, bf16 weight copies), all
 *     allocated in vf_init and freed in vf_destroy; vf_step allocates no device memory
 *     (on the host it fills a few small vectors of node sizes, offsets and weights);
 *   - all device work is enqueued on the stream given in the configuration.
 *
 * Flat parameter layout (fp32, also the layout of vf_grads and vf_opt_state):
 *   tensors in forward order; a Linear is W[K_in, N_out] row-major, then its bias, then
 *   the scale and shift of the normalisation that follows it.
 *   MLP:     per hidden layer W, bias (only without BatchNorm), gamma, beta (only with
 *            BatchNorm); last layer W, bias.
 *   encoder: tok_emb[vocab,d], pos_emb[T,d]; per layer ln1.gamma, ln1.beta, Wqkv[d,3d],
 *            bqkv, Wo[d,d], bo, ln2.gamma, ln2.beta, W1[d,ffn], b1, W2[ffn,d], b2; then
 *            lnf.gamma, lnf.beta, Wout[d,vocab], bout.
 *   conv:    a residual network of 3x3 convolutions (stride 1, zero padding 1, no bias, each
 *            followed by BatchNorm over the node's n*img*img positions): stem filters
 *            [width, 3, 3, in_ch], gamma, beta; per block filters1 [width, 3, 3, width], gamma1,
 *            beta1, filters2, gamma2, beta2 (block: convolution, BatchNorm, ReLU, convolution,
 *            BatchNorm, add the block's input, ReLU); then the classifier on the mean over the
 *            positions: W[width, classes], bias.
 *
 * Environment variables.  None is needed in normal use; the kernel choices change at most the
 * order of floating-point sums inside a product, never which operation is computed.  They
 * are read once per process, when the code that looks at them first runs.
 *   debugging
 *     VF_SYNC_EACH=all | tag[,tag...]   the host waits for the stream after every kernel launch
 *                        (or after the launches with one of the named profile tags), so that a
 *                        device error is reported by the launch that caused it
 *     VF_ARENA_GUARD=<bytes>            leaves that many bytes (rounded down to 256), filled with a
 *                        pattern that is no valid float, between the buffers of the workspace, so
 *                        that a read past a buffer's end shows in the results
 *   kernel selection, for measurements (every choice gives results that pass the same tests)
 *     VF_GEMM_TILE=128x128|128x64|64x128|64x64|32x128   forces one tile of the general bf16 product
 *     VF_GEMM_SHORTK=0     weight gradients go to the general kernel, not the short-contraction one
 *     VF_GEMM_DL=0|3|4|5   LDS-direct product kernel off, or its ring depth (default 4)
 *     VF_GEMM_PIPE=0..4    ring depth of the register-staged product kernel (default 3, 0 = off)
 *     VF_GEMM_SPLIT_TARGET=<n>   workgroups a small product is sliced up to (default 256)
 *     VF_GEMM_WIDE=0|1|128|256   256-row product kernel off / on (default) / with 128 or 256 columns
 *     VF_GEMM_WIDE_V=1|2   256 x 256 tiles on the ring of three 32-element stages (1) or on the whole-line kernel
 *                          with the 32x32x16 instruction (2) instead of the whole-line kernel with 16x16x32
 *     VF_GEMM_NT=1         fp32 results of the bf16 products stored with the non-temporal hint
 *     VF_CONV_LDS=0        3x3 convolutions without the filters-resident-in-LDS kernel
 *     VF_CONV_EXPLICIT=1   convolutions always write the patch matrix and call the product kernel
 *     VF_LN_WGS=<n>        workgroups of the LayerNorm backward kernel (default 256)
 *     VF_BN_SUBGROUPS=2|4  sub-groups of 256 threads per workgroup of the grouped BatchNorm kernels
 *     VF_BN_PAIR=0|1       grouped BatchNorm kernels with two columns per thread: never | for every even width
 *                          (default: for layers of at least 6144 columns)
 *     VF_BN_FUSE=0         the BatchNorm backward pass as a kernel of its own also where the input-gradient
 *                          product's epilogue would take it (units of whole 128-row nodes on wide layers)
 *     VF_BN_FUSE_FWD=0     the same for the forward pass
 *     VF_FLAT_NT=0|1       accumulate and optimizer kernels with non-temporal accesses: never | always
 *                          (default: for vectors of 64 MB and more)
 */
#ifndef VF_H
#define VF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#pragma GCC visibility push(default)

#define VF_OK        0
#define VF_EINVAL   (-1)   /* bad argument (null pointer, sizes that are not a partition, ...) */
#define VF_ENOMEM   (-2)   /* device or host allocation failed */
#define VF_EDEVICE  (-3)   /* a HIP call failed; vf_last_error() has the text */
#define VF_ESTATE   (-4)   /* call made in the wrong state (e.g. vf_grads before any vf_step) */

#define VF_MLP      0
#define VF_ENCODER  1
#define VF_CONV     2

#define VF_F32      0      /* fp32 operands and arithmetic throughout */
#define VF_BF16     1      /* bf16 GEMM operands (round-to-nearest-even), fp32 accumulation,
                              fp32 master parameters, gradients and optimizer */

#define VF_SGDM     0      /* v <- mu v + G;  theta <- theta - lr v */
#define VF_ADAM     1      /* bias-corrected Adam, t counted from 1 */

#define VF_MAX_DIMS 16

/* flags */
#define VF_FLAG_FUSED_ACCUMULATE 1u  /* weight-gradient kernels add w_i*g_i straight into the
                                        gradient buffer instead of writing a staging vector that
                                        the accumulate kernel folds in; same arithmetic per
                                        element (one fused multiply-add), same node order */
#define VF_FLAG_NO_GRAPH         2u  /* launch kernels one by one instead of replaying a
                                        captured HIP graph */
#define VF_FLAG_OVERLAP          4u  /* two streams (bf16 MLP and bf16 encoder; same results bit
                                        for bit as one stream):
                                        the forward passes run on the caller's stream, the
                                        backward passes and weight gradients on a second,
                                        library-owned stream, so that node i+1's forward pass
                                        runs beside node i's backward pass.  Nodes still start
                                        and finish in order, and every accumulation whose order
                                        matters stays on one stream; the tensors that pass from a
                                        node's forward to its backward pass are kept twice. */
#define VF_FLAG_ORDERED_FOLD     8u  /* inside a fold window keep the node-by-node chain of
                                        roundings, G <- fma(b_i/B, g_i, G) node after node.
                                        Without this flag a window (bf16 MLP) whose node sizes
                                        are multiples of 8 takes its weight gradients as ONE
                                        product over all the window's rows.  Nodes of one size:
                                        times the common weight, the same sum with fewer
                                        roundings, equal to the node-by-node result to fp32
                                        rounding.  Nodes of several sizes: with b_i/B folded into
                                        the bf16 output gradients of node i before the product
                                        (rounded once from fp32), one bf16 rounding apart from
                                        the node-by-node result.  Neither is bit for bit. */

typedef struct vf_ctx vf_ctx;

/* Plain data, copied by vf_init. */
typedef struct vf_config {
  int32_t model_kind;            /* VF_MLP | VF_ENCODER | VF_CONV */
  int32_t n_dims;                /* MLP: number of entries of dims (layers + 1), 2..VF_MAX_DIMS */
  int32_t dims[VF_MAX_DIMS];     /* MLP: [in, h1, ..., out] */
  int32_t batchnorm;             /* MLP: 1 = every hidden Linear (no bias) is followed by
                                    BatchNorm (statistics per virtual node) and ReLU;
                                    0 = Linear with bias, then ReLU */
  int32_t n_layers, d_model, n_heads, d_ffn, seq_len, vocab, n_masked;   /* encoder */
  int32_t img, in_ch, width, n_blocks, classes;   /* conv: img x img inputs with in_ch channels,
                                    `width` channels in every convolution (a multiple of 8, at
                                    most 256), n_blocks residual blocks; VF_BF16 only */
  int32_t dtype;                 /* VF_F32 | VF_BF16 */
  int32_t optimizer;             /* VF_SGDM | VF_ADAM */
  float   lr, momentum, beta1, beta2, adam_eps, bn_eps, ln_eps;
  float   bn_momentum;           /* MLP with BatchNorm: share of a pass's statistics blended into
                                    the moving mean / variance after every virtual node, in
                                    [0, 1]; 0 freezes them */
  int32_t max_batch;             /* largest B a step may use */
  int32_t max_node_size;         /* largest b_i; sizes the per-node workspace */
  int32_t max_nodes;             /* largest V */
  int32_t fold_window;           /* MLP, bf16, fused fold: the weight gradients of this many
                                    consecutive nodes (1..8; 0 = 1; with node_group > 1: of this
                                    many units of grouped nodes) are folded into the gradient
                                    buffer in one pass over it: nodes of one size (one weight
                                    b_i/B) as ONE product over all their rows, nodes of several
                                    sizes (multiples of 8) as one product with the weights folded
                                    into the transposed output gradients, other sizes -- or any
                                    with VF_FLAG_ORDERED_FOLD -- as the chain of fused
                                    multiply-adds of the node-by-node fold (bitwise its result).
                                    1/window of the buffer traffic; the transposed bf16 operands of
                                    the window's nodes are kept until then, so the workspace grows
                                    with the window (not with V). */
  int32_t node_group;            /* MLP (bf16) and encoder: up to this many CONSECUTIVE nodes (1, 2, 4,
                                    8, 16 or 32; 0 = 1) go through their passes together as one unit: their
                                    rows form one operand of every product, so the weights are read
                                    once per unit instead of once per node.  Everything a node owns
                                    stays per node -- BatchNorm statistics and their moving averages
                                    (node after node), the node losses, the weight b_i/B -- so the
                                    step computes what it computes node by node, up to the order of
                                    additions and (nodes of different sizes) one bf16 rounding of
                                    the output gradients, which carry 1/rows of the unit instead of
                                    1/b_i.  MLP: nodes of at most 128 rows, a multiple of 8, of any
                                    mix of sizes; other nodes go alone (units of 16 or 32 nodes: the
                                    staged fold then differs from the fused one by fp32 rounding in the
                                    BatchNorm scale / shift gradients, and a fold window holds at most
                                    as many units as a batch has).  Encoder: runs of 2 or 4
                                    nodes of one size.  The per-node workspace grows by this factor
                                    (not with V). */
  uint32_t flags;                /* VF_FLAG_* */
  void*   stream;                /* hipStream_t; NULL = the default stream */
} vf_config;

/* S0 of the step, host only (Section 3.2: the batch is split among the virtual nodes;
 * Section 5.2: node i's mean gradient is weighted by b_i/B).  node_sizes: host, length V.
 * off_out: host, V+1 entries, off[0]=0, off[i+1]=off[i]+b_i: node i owns the contiguous
 * batch rows off[i]..off[i+1]-1.  w_out: host, V entries, the single IEEE fp32 division
 * (float)b_i/(float)B.  Either output may be NULL.  VF_EINVAL if V<1, any b_i<1 or
 * sum b_i != B; outputs are then untouched. */
int vf_partition(const int32_t* node_sizes, int32_t V, int32_t B, int32_t* off_out, float* w_out);

/* Creates a context on the current HIP device: validates the configuration, lays out the
 * parameters and allocates every buffer a step needs (sized by max_node_size and max_batch,
 * not by the number of nodes: Section 3.3, the gradient buffer is one model-sized vector
 * shared by all nodes).  *out is NULL on failure. */
int vf_init(const vf_config* cfg, vf_ctx** out);

/* One training step (Section 3.2 steps 1-3 and 5; step 4, the cross-device exchange, is the
 * identity on one device).
 *   params      device, fp32 [vf_num_params], IN/OUT: master parameters, updated in place.
 *   batch_x     device. MLP: [B, dims[0]] row-major, fp32 for VF_F32, bf16 for VF_BF16.
 *               encoder: int32 token ids [B, seq_len], masked positions already replaced.
 *               conv: bf16 [B, img, img, in_ch] (channels last).
 *   batch_y     device, int32. MLP and conv: [B] class labels in [0, dims[last]) / [0, classes).
 *               encoder: [B, 2, n_masked]: [s,0,:] masked positions in [0, seq_len), distinct
 *               per sequence; [s,1,:] target ids in [0, vocab).
 *   B, V        batch size and number of virtual nodes.
 *   node_sizes  host, length V.
 * Validation (as vf_partition, plus V <= max_nodes, b_i <= max_node_size, B <= max_batch)
 * happens before any device work: a rejected call leaves params and all state untouched.
 * Label and id values are not validated (they live on the device); out-of-range values are
 * clamped into range by the kernels.  Asynchronous: returns once the work is enqueued. */
int vf_step(vf_ctx* ctx, void* params, const void* batch_x, const int32_t* batch_y,
            int32_t B, int32_t V, const int32_t* node_sizes);

/* Input prefetch (Section 3.2 step 1 / Figure 4: while one batch is processed the next one is
 * fetched in the background).  vf_prefetch copies the NEXT batch (same element types and layout
 * as vf_step's batch_x / batch_y) from HOST memory into one of two device staging buffers of the
 * context, on a copy stream of the library's own, and returns at once; the host buffers must
 * stay untouched until that copy is done, and should be pinned (hipHostMalloc), else the copy
 * is not asynchronous.  vf_step_prefetched runs vf_step on the staged batch (its stream waits
 * for the copy) and frees the other pair of buffers for the next vf_prefetch, so the pattern is
 *     vf_prefetch(b0); loop t: vf_step_prefetched(...); vf_prefetch(b_{t+1});   -- or prefetch first:
 *     vf_prefetch(b_{t+1}) may be called as soon as vf_step_prefetched(t) has returned.
 * At most one batch is staged ahead: a second vf_prefetch before the staged batch is consumed
 * returns VF_ESTATE, as does vf_step_prefetched with nothing staged.  A rejected step
 * (VF_EINVAL, as vf_step) leaves the batch staged.  The staging buffers are allocated at the
 * first vf_prefetch (VF_ENOMEM if that fails) and sized for max_batch. */
int vf_prefetch(vf_ctx* ctx, const void* host_x, const int32_t* host_y, int32_t B);
int vf_step_prefetched(vf_ctx* ctx, void* params, int32_t V, const int32_t* node_sizes);

/* Combined gradient G = sum_i (b_i/B) g_i of the last step (the value the update used): the
 * node gradients folded with the size weights of Section 5.2, which make G the gradient over the
 * whole batch also when the nodes differ in size (Section 3.2 step 3 has the fold itself),
 * fp32 [vf_num_params] copied to `out`, which may be a device or a host pointer.
 * Synchronises the stream.  VF_ESTATE before the first step. */
int vf_grads(vf_ctx* ctx, float* out);

/* Combined loss L = sum_i (b_i/B) L_i of the last step, L_i the mean loss over node i's
 * samples (encoder: over its masked positions); the weights are those of Section 5.2, so L is
 * the mean over the batch for nodes of any sizes.  out: host, one float.  Synchronises. */
int vf_loss(vf_ctx* ctx, float* out);

/* Per-node mean losses L_i of the last step.  out: host, V floats (V of the last step). */
int vf_node_losses(vf_ctx* ctx, float* out, int32_t V);

/* Optimizer state after the last step, fp32 [vf_num_params], device or host `out`.
 * which = 0: SGD-momentum velocity v, or Adam first moment m;  which = 1: Adam second
 * moment u (VF_EINVAL for SGD-momentum).  Synchronises. */
int vf_opt_state(vf_ctx* ctx, int32_t which, float* out);

/* Per-kernel timing of the steps run between the two calls (the library's counterpart of the
 * offline profiling of Section 5.1.1: how long each part of a node's pass takes on this
 * device).  While enabled, every kernel launch is bracketed by two events on the stream it goes
 * to and launches are made one by one instead of by graph replay, so step time itself is
 * slower than normal.  With VF_FLAG_OVERLAP the two streams stay in use, so a kernel's time
 * includes whatever it loses to the kernel running beside it.  vf_profile_stop synchronises and
 * writes a JSON object
 * {"<kernel tag>": {"launches": n, "total_ms": t}, ...} into `json` (host, `cap` bytes,
 * NUL-terminated); VF_EINVAL if it does not fit. */
int vf_profile_start(vf_ctx* ctx);
int vf_profile_stop(vf_ctx* ctx, char* json, size_t cap);

/* Number of optimizer updates applied so far (one per successful vf_step). */
int64_t vf_step_count(const vf_ctx* ctx);
/* The fold window in effect (1 when the configuration's model, dtype or mode has no windowed path). */
int32_t vf_fold_window(const vf_ctx* ctx);
/* Streams the node passes of a step are spread over: 2 when VF_FLAG_OVERLAP is in effect
 * (asked for, a non-default stream given, and the model supports it), else 1; 0 for NULL. */
int32_t vf_streams(const vf_ctx* ctx);

int64_t vf_num_params(const vf_ctx* ctx);

/* Bytes of device memory the context holds.  Depends on the model, max_node_size and
 * max_batch only -- never on the number of virtual nodes (Section 3.3). */
size_t vf_workspace_bytes(const vf_ctx* ctx);

void vf_destroy(vf_ctx* ctx);

const char* vf_strerror(int code);
/* Text of the last device error seen by this thread ("" if none). */
const char* vf_last_error(void);

/* ---- the two bandwidth-bound kernels of the step, callable on their own -------------- */

/* Step 3 of Section 3.2 with the weight of Section 5.2 over a flat fp32 vector:
 *   first != 0:  buf[p] = w * g[p]          first == 0:  buf[p] = buf[p] + w * g[p]
 * (one fused multiply-add per element).  buf, g: device, n floats, 16-byte aligned. */
int vf_accumulate(float* buf, const float* g, float w, int64_t n, int32_t first, void* stream);

/* Step 5 of Section 3.2 over flat fp32 vectors (device, n floats each):
 *   v <- momentum*v + G ;  theta <- theta - lr*v. */
int vf_sgdm_update(float* theta, float* v, const float* G, float lr, float momentum,
                   int64_t n, void* stream);
/*   m <- beta1*m + (1-beta1)*G ;  u <- beta2*u + (1-beta2)*G*G ;
 *   theta <- theta - lr * (m/(1-beta1^t)) / (sqrt(u/(1-beta2^t)) + eps),  t >= 1. */
int vf_adam_update(float* theta, float* m, float* u, const float* G, float lr, float beta1,
                   float beta2, float eps, int64_t t, int64_t n, void* stream);

/* The contraction every Linear layer of a virtual node's forward and backward pass uses
 * (Section 3.2 steps 1-2), callable on its own:
 *     C[m,n] = alpha * sum_k A[m*lda + k] * B[n*ldb + k]  (+ C[m,n] if accumulate != 0)
 * i.e. C = alpha * A * B^T (+ C) with both operands contiguous along the contraction.
 * dtype VF_BF16: A, B bf16 (device, 16-byte aligned, lda and ldb multiples of 8), products
 * accumulated in fp32 on the matrix cores; VF_F32: A, B fp32.  C: device fp32 [M, ldc].
 * Forward y = x W uses B = W^T; input gradient dx = dy W^T uses B = W; weight gradient
 * dW = x^T dy uses A = x^T, B = dy^T with alpha = b_i/B and accumulate = 1 to fold a node's
 * gradient straight into the gradient buffer.
 * nsplit >= 1 cuts the contraction into nsplit slices (bf16 only, accumulate must be 0):
 * C is then [nsplit][M][ldc] and slab s holds slice s's partial product; the caller adds
 * the slabs (the library's consumers do so in slab order).  This is how the skinny products
 * of a small virtual node are spread over all compute units. */
int vf_gemm(int32_t dtype, const void* A, int64_t lda, const void* B, int64_t ldb, float* C,
            int64_t ldc, int32_t M, int32_t N, int32_t K, float alpha, int32_t accumulate,
            int32_t nsplit, void* stream);

/* The sliced contraction of vf_gemm for callers that cannot allocate device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Computes
 *     C[m,n] = alpha * sum_k A[m*lda + k] * B[n*ldb + k]  (+ C[m,n] if accumulate != 0)
 * for bf16 A, B (device, 16-byte aligned, lda and ldb multiples of 8) and a DENSE fp32 C [M, N]
 * (device, row pitch N), with the contraction cut into nsplit slices exactly as vf_gemm cuts it;
 * the slabs of partial products, which vf_gemm hands to its caller, stay in a device array of
 * VF_NOALLOC_SCRATCH_BYTES that is part of the library's image (every GPU the library runs on
 * holds it until the process ends) and are added in slab order: C = fma(alpha, slab_0 + slab_1
 * + ... , accumulate ? C : 0), bit for bit what a caller of vf_gemm gets who adds the slabs in
 * that order.  The call allocates nothing (no hipMalloc / hipFree, no allocating library
 * routine); all work is enqueued on `stream`.  VF_EINVAL, with nothing enqueued, if
 * nsplit * M * N * 4 exceeds VF_NOALLOC_SCRATCH_BYTES or an argument is malformed.
 * All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU (two
 * streams, two threads) race; calls on one stream are ordered and safe.  Nothing needs to be
 * cleared between calls (every slice overwrites its whole slab). */
#define VF_NOALLOC_SCRATCH_BYTES (32 * 1024 * 1024)
int vf_gemm_noalloc(const void* A, int64_t lda, const void* B, int64_t ldb, float* C, int32_t M,
                    int32_t N, int32_t K, float alpha, int32_t accumulate, int32_t nsplit,
                    void* stream);

/* ---- training state of this device (Section 4.1) ---------------------------------------
 * What a device that joins a job has to receive before it can continue the job's steps: the
 * master parameters, the optimizer state, and the state the passes themselves carry (the
 * BatchNorm moving mean and variance, which every device updates on its own, once per virtual
 * node in node order, from that node's statistics:  moving += bn_momentum * (node - moving),
 * biased variance; start: mean 0, variance 1.  The paper does not say how several nodes on one
 * device share the moving statistics; this is the reading of a framework that runs the nodes
 * as consecutive passes).  Payload, little endian, VF_STATE_HEADER_BYTES + 4*(P + n_opt*P + 2*S)
 * bytes:
 *   int64 header[8] = { VF_STATE_MAGIC, P, n_opt (1 SGD-momentum, 2 Adam), S (summed width of
 *                       the BatchNorm layers), completed steps, optimizer, 0, 0 }
 *   fp32 theta[P]; fp32 opt[n_opt][P] (v | m, u); fp32 moving_mean[S]; fp32 moving_var[S]
 * (BatchNorm layers in forward order). */
#define VF_STATE_MAGIC        0x3145544154534656LL   /* "VFSTATE1" */
#define VF_STATE_HEADER_BYTES 64

/* Size of the payload for this context. */
int64_t vf_state_bytes(const vf_ctx* ctx);

/* Writes the payload to dst (device or host pointer, `bytes` >= vf_state_bytes).  params: device,
 * the master parameters the caller owns.  Synchronises the context's stream. */
int vf_state_export(vf_ctx* ctx, const float* params, void* dst, int64_t bytes);

/* Reads a payload (device or host pointer) written by vf_state_export of a context with the same
 * model and optimizer: overwrites params (device), the optimizer state, the moving statistics
 * and the step count (Adam's bias correction depends on it).  VF_EINVAL and nothing changed if
 * the header does not match this context.  Synchronises the context's stream. */
int vf_state_import(vf_ctx* ctx, float* params, const void* src, int64_t bytes);

/* ---- heterogeneous split solver (host only) ---------------------------------------------- */

/* Offline profile of one accelerator type (Section 5.1.1): the time of one virtual-node pass
 * for the node batch sizes that fit in its memory.  batch ascending, step_time > 0 (any unit). */
typedef struct vf_device_profile {
  int32_t n_devices;            /* n_i: accelerators of this type in the job */
  int32_t n_points;
  const int32_t* batch;         /* host, n_points node batch sizes */
  const double* step_time;      /* host, t_i(batch[k]) */
} vf_device_profile;

/* Section 5.1.2: minimise max_i ( t_i(b_i / v_i) * v_i ) + comm subject to sum_i n_i b_i = B over
 * the per-device batch b_i and the virtual nodes per device v_i of every type.  Reading of the
 * paper's formula (it prints t_i(b_i) * v_i): t_i is evaluated at the node batch b_i / v_i, which
 * is what its "virtual nodes on a GPU run sequentially" explanation and its Table 4 (per-GPU
 * batch and nodes per GPU) imply.  b_i ranges over 0 (type unused: the homogeneous fallback)
 * and the power-of-2 and power-of-2-like sizes 1,2,3,4,6,8,12,16,24,... the profiler considers;
 * b_i / v_i must be a profiled size.  comm (>= 0, same unit) is added when more than one
 * device takes part.  Among equal optima the first in lexicographic order of (b_0, b_1, ...)
 * ascending is returned, and for a given b_i the smallest v_i.
 * types: host, n_types (1..8) entries.  b_out, v_out: host, n_types entries (v = 0 for an unused
 * type).  step_time_out: host, optional.  VF_EINVAL for malformed input, VF_ESTATE when no
 * combination of profiled sizes adds up to B. */
int vf_solve_split(const vf_device_profile* types, int32_t n_types, int32_t B, double comm,
                   int32_t* b_out, int32_t* v_out, double* step_time_out);

#pragma GCC visibility pop

#ifdef __cplusplus
}
#endif
#endif /* VF_H */
