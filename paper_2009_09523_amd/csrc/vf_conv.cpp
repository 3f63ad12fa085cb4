// Residual network of 3x3 convolutions with per-node BatchNorm: buffers and the launch sequence
// of one virtual node (forward, loss, backward), Section 3.2 steps 1-3.  Every BatchNorm takes
// its statistics over the n*H*W positions of the node that is running (Section 4.1).
//
// A convolution is a product over patch rows (per output position the 3x3 neighbourhood of the
// bf16, channels-last input: 9*Cin values) with the filters.  When the input channels are a
// multiple of 64 the kernels read the patches straight from the activation (no patch matrix) --
// with 64 channels and an image side of 8 to 64, a kernel that keeps the filters in LDS and
// stages the input once per 64 positions; otherwise (the first layer) im2col writes them.  The
// input gradient is the same convolution of the output gradient with the filters turned by 180
// degrees and the channel roles exchanged (a second bf16 copy of the filters, made once per
// step).  The weight gradient contracts over all positions of the node, cut into slabs that are
// added in order: channel counts that are multiples of 64 (and image sides of 8 to 64) take a
// kernel that reads the output gradient and the stored input as they are; the others the product
// of the transposed output gradient with the transposed patch matrix (written row by row from
// the transposed input).  Where the convolution kernel supports it, it also leaves the
// BatchNorm statistics partials of what it stored.
#include <algorithm>
#include <cstdlib>

#include "vf_ctx.h"

namespace vf {
namespace {

inline int64_t round8(int64_t v) { return (v + 7) & ~int64_t(7); }

struct ConvLayer {
  int Cin = 0, C = 0;              // channels in, out
  int Kc = 0, Kp = 0;              // 9*Cin and its row pitch (a multiple of 8)
  int Kpf = 0;                     // 9*C: row pitch of the turned filters (0: no input gradient needed)
  int64_t w_off = 0, g_off = 0, be_off = 0;   // flat parameter offsets: filters, gamma, beta
  int64_t s_off = 0;               // offset of the moving statistics within a state half
  bf16_t* wnat = nullptr;          // [C, Kp]    filters as they are
  bf16_t* wflip = nullptr;         // [Cin, Kpf] turned filters
  const bf16_t* in = nullptr;      // the input of the node in flight ([rows, Cin], set by the forward pass)
  float* y = nullptr;              // [rows, C]  convolution output
  float* mean = nullptr;           // [C]
  float* rstd = nullptr;           // [C]
  bf16_t* a = nullptr;             // [rows, C]  after BatchNorm (+ skip) and ReLU
};

class Conv final : public Model {
 public:
  explicit Conv(const vf_config& cfg) : cfg_(cfg) {
    H_ = cfg.img; HW_ = cfg.img * cfg.img; C_ = cfg.width;
    const int nl = 1 + 2 * cfg.n_blocks;
    layers_.resize(nl);
    int64_t off = 0;
    for (int l = 0; l < nl; ++l) {
      ConvLayer& L = layers_[l];
      L.Cin = l == 0 ? cfg.in_ch : C_;
      L.C = C_;
      L.Kc = 9 * L.Cin;
      L.Kp = (int)round8(L.Kc);
      L.Kpf = l == 0 ? 0 : 9 * C_;
      L.w_off = off; off += (int64_t)C_ * L.Kc;
      L.g_off = off; off += C_;
      L.be_off = off; off += C_;
      L.s_off = (int64_t)l * C_;
    }
    fc_w_off_ = off; off += (int64_t)C_ * cfg.classes;
    fc_b_off_ = off; off += cfg.classes;
    P_ = off;
    rows_max_ = (int64_t)cfg.max_node_size * HW_;
    ldr_ = round8(rows_max_);
    ldb_ = round8(cfg.max_node_size);
    ldc_ = round8(C_);
    ldz_ = round8(cfg.classes);
  }

  int64_t num_params() const override { return P_; }

  void request_buffers(Arena& a) override {
    const size_t rows = (size_t)rows_max_;
    int kp_max = 0;
    for (ConvLayer& L : layers_) {
      a.request(&L.wnat, (size_t)L.C * L.Kp);
      if (L.Kpf) a.request(&L.wflip, (size_t)L.Cin * L.Kpf);
      a.request(&L.y, rows * L.C);
      a.request(&L.mean, (size_t)L.C);
      a.request(&L.rstd, (size_t)L.C);
      a.request(&L.a, rows * L.C);
      kp_max = std::max(kp_max, std::max(L.Kp, L.Kpf));
    }
    a.request(&cols_, rows * (size_t)kp_max);
    a.request(&zeros_, (size_t)64);
    a.request(&colsT_, (size_t)kp_max * ldr_);
    a.request(&dyT_, (size_t)C_ * ldr_);
    a.request(&inT_, (size_t)std::max(C_, cfg_.in_ch) * ldr_);
    a.request(&dy_, rows * C_);
    a.request(&gA_, rows * C_);
    a.request(&gB_, rows * C_);
    a.request(&partial_, (size_t)std::max(conv_chunks(rows_max_), kConvStatsChunks) * 2 * C_);
    a.request(&sums_, (size_t)2 * C_);
    // contraction slabs of a weight gradient: up to kMaxSplit from the product over the transposed
    // patch matrix, up to kDirectSplit per 64 x 64 channel block from the direct kernel
    const size_t per_slab = (size_t)C_ * (kp_max > 9 * C_ ? kp_max : 9 * C_);
    const int blocks64 = std::max(1, (C_ / 64) * (C_ / 64));
    a.request(&slabs_, per_slab * (size_t)std::max(kMaxSplit, (kDirectSplit + blocks64 - 1) / blocks64));
    a.request(&fc_wnat_, (size_t)C_ * ldz_);
    a.request(&fc_wtr_, (size_t)cfg_.classes * ldc_);
    a.request(&pooled_, (size_t)cfg_.max_node_size * ldc_);
    a.request(&pooledT_, (size_t)C_ * ldb_);
    a.request(&zslab_, (size_t)cfg_.max_node_size * ldz_);
    a.request(&z_, (size_t)cfg_.max_node_size * ldz_);
    a.request(&dz_, (size_t)cfg_.max_node_size * ldz_);
    a.request(&dzT_, (size_t)cfg_.classes * ldb_);
    a.request(&dpooled_, (size_t)cfg_.max_node_size * ldc_);
    a.request(&state_, (size_t)2 * layers_.size() * C_);
  }

  int64_t state_floats() const override { return 2 * (int64_t)layers_.size() * C_; }
  float* state_ptr() const override { return state_; }
  int init_state(hipStream_t st) override {   // moving mean 0, moving variance 1
    const int64_t S = (int64_t)layers_.size() * C_;
    VF_TRY(launch_fill_f32(state_, 0.f, S, st));
    return launch_fill_f32(state_ + S, 1.f, S, st);
  }

  int prepare(Ctx& c, const float* params, hipStream_t st) override {
    // the element-wise kernels read gamma, beta and the statistics four at a time
    if (reinterpret_cast<uintptr_t>(params) & 15) return VF_EINVAL;
    for (ConvLayer& L : layers_)
      VF_KS(c, st, "cast_weight", launch_conv_weight_copies(params + L.w_off, L.C, L.Cin, L.wnat, L.Kp, L.wflip, L.Kpf, st));
    VF_KS(c, st, "cast_weight", launch_cast_weight(params + fc_w_off_, C_, cfg_.classes, fc_wnat_, ldz_, fc_wtr_, ldc_, st));
    return VF_OK;
  }

  int run_node_main(Ctx& c, const StepArgs& s, int i, hipStream_t st) override {
    VF_TRY(forward(c, s, i, st));
    return backward(c, s, i, st);
  }

  int run_nodes_side(Ctx& c, const StepArgs& s, int i0, int count, hipStream_t st) override {
    for (int i = i0; i < i0 + count; ++i) VF_TRY(c.fold(i, s.w[i], st));   // staged mode only
    return VF_OK;
  }

 private:
  static constexpr int kMaxSplit = 32;
  static constexpr int kDirectSplit = 256;

  // y = patches(in) x filters^T; statistics over the node's rows; a = relu(BatchNorm(y) (+ skip))
  int conv_bn_relu(Ctx& c, ConvLayer& L, const bf16_t* in, const bf16_t* skip, int rows, const float* P,
                   hipStream_t st) {
    L.in = in;
    Epilogue ep;
    ep.C = L.y; ep.ldc = L.C;
    int chunks = 0, chunk_rows = 0;     // statistics partials that the convolution kernel leaves, if it does
    if (L.Cin % 64 == 0 && !explicit_) {
      VF_KS(c, st, "gemm_fwd", launch_conv3x3_bf16(in, rows, H_, H_, L.Cin, L.wnat, L.Kp, L.C, ep, zeros_, st, partial_,
                                                   &chunks, &chunk_rows));
    } else {
      VF_KS(c, st, "im2col", launch_im2col3x3(in, rows, H_, H_, L.Cin, cols_, L.Kp, st));
      VF_KS(c, st, "gemm_fwd", launch_gemm_bf16(cols_, L.Kp, L.wnat, L.Kp, rows, L.C, L.Kp, 1, 0, ep, st));
    }
    const int64_t S = (int64_t)layers_.size() * C_;
    if (chunks > 0)
      VF_KS(c, st, "bn_stats", launch_bn2d_stats_finish(partial_, chunks, chunk_rows, rows, L.C, cfg_.bn_eps, L.mean, L.rstd,
                                                        state_ + L.s_off, state_ + S + L.s_off, cfg_.bn_momentum, st));
    else
      VF_KS(c, st, "bn_stats", launch_bn2d_stats(L.y, rows, L.C, cfg_.bn_eps, partial_, L.mean, L.rstd,
                                                 state_ + L.s_off, state_ + S + L.s_off, cfg_.bn_momentum, st));
    VF_KS(c, st, "bn_apply", launch_bn2d_apply_fwd(L.y, rows, L.C, P + L.g_off, P + L.be_off, 1, L.mean, L.rstd,
                                                   skip, L.a, st));
    return VF_OK;
  }

  int forward(Ctx& c, const StepArgs& s, int i, hipStream_t st) {
    const int b = s.sizes[i];
    const int rows = b * HW_;
    const int64_t row0 = s.off[i];
    const float* P = s.params;
    const bf16_t* x = static_cast<const bf16_t*>(s.x) + row0 * HW_ * cfg_.in_ch;
    VF_TRY(conv_bn_relu(c, layers_[0], x, nullptr, rows, P, st));
    for (int blk = 0; blk < cfg_.n_blocks; ++blk) {
      const bf16_t* in = layers_[2 * blk].a;                  // the block's input: the previous stored activation
      VF_TRY(conv_bn_relu(c, layers_[1 + 2 * blk], in, nullptr, rows, P, st));
      VF_TRY(conv_bn_relu(c, layers_[2 + 2 * blk], layers_[1 + 2 * blk].a, in, rows, P, st));
    }
    VF_KS(c, st, "avgpool", launch_avgpool_fwd(layers_.back().a, b, HW_, C_, pooled_, ldc_, st));
    Epilogue ep;
    ep.C = zslab_; ep.ldc = ldz_;
    ep.bias = P + fc_b_off_; ep.bias_round_bf16 = 1;
    VF_KS(c, st, "gemm_fc", launch_gemm_bf16(pooled_, ldc_, fc_wtr_, ldc_, b, cfg_.classes, C_, 1, 0, ep, st));
    VF_KS(c, st, "softmax_xent", launch_softmax_xent(zslab_, 1, 0, ldz_, z_, ldz_, s.y + row0, b, cfg_.classes,
                                                     c.rowloss + row0, dz_, ldz_, 1, dzT_, ldb_, s.w[i], i, nullptr,
                                                     nullptr, st));
    if (i == s.V - 1) {   // loss bookkeeping of the whole step, in node order (Section 5.2)
      for (int first = 0; first < s.V; first += kLossNodes) {
        LossNodes ln{};
        ln.first = first;
        ln.count = std::min(kLossNodes, s.V - first);
        for (int j = 0; j < ln.count; ++j) {
          ln.off[j] = s.off[first + j]; ln.rows[j] = s.sizes[first + j]; ln.w[j] = s.w[first + j];
        }
        VF_KS(c, st, "loss_reduce", launch_loss_reduce_nodes(c.rowloss, ln, c.node_loss, c.loss_total, st));
      }
    }
    return VF_OK;
  }

  // dW[o, (kh,kw,c)] = sum over the node's positions of dy[r, o] * patches[r, (kh,kw,c)]
  int conv_wgrad(Ctx& c, ConvLayer& L, int rows, float w, int node, hipStream_t st) {
    const int64_t slab = (int64_t)L.C * L.Kc;
    if (!explicit_ && conv_wgrad_direct_fits(L.C, L.Cin, H_, H_, rows)) {
      // straight from dy and the stored input: no transposes, no patch matrix
      const int blocks64 = (L.C / 64) * (L.Cin / 64);
      int split = 0;
      VF_KS(c, st, "gemm_wgrad", launch_conv_wgrad_direct(dy_, L.C, L.in, L.Cin, rows, H_, H_, zeros_, slabs_, slab,
                                                          std::max(1, kDirectSplit / blocks64), &split, st));
      VF_KS(c, st, "fold_slabs", launch_fold_slabs(slabs_, split, slab, slab, c.gout(L.w_off, w, node), st));
      return VF_OK;
    }
    VF_KS(c, st, "transpose", launch_transpose_bf16(L.in, L.Cin, inT_, ldr_, rows, L.Cin, st));
    VF_KS(c, st, "im2col", launch_im2col3x3_transposed(inT_, ldr_, rows, H_, H_, L.Cin, colsT_, ldr_, st));
    VF_KS(c, st, "transpose", launch_transpose_bf16(dy_, L.C, dyT_, ldr_, rows, L.C, st));
    int split = std::min(kMaxSplit, gemm_bf16_pick_split(L.C, L.Kc, rows));
    Epilogue ep;
    ep.C = slabs_; ep.ldc = L.Kc;
    VF_KS(c, st, "gemm_wgrad", launch_gemm_bf16(dyT_, ldr_, colsT_, ldr_, L.C, L.Kc, rows, split, slab, ep, st));
    VF_KS(c, st, "fold_slabs", launch_fold_slabs(slabs_, split, slab, slab, c.gout(L.w_off, w, node), st));
    return VF_OK;
  }

  // out = (addend +) the convolution of dy with the turned filters
  int conv_dgrad(Ctx& c, ConvLayer& L, int rows, float* out, const float* addend, hipStream_t st) {
    Epilogue ep;
    ep.C = out; ep.ldc = L.Cin;
    if (addend) { ep.R = addend; ep.ldr = L.Cin; ep.beta = 1.f; }
    if (L.C % 64 == 0 && !explicit_) {
      VF_KS(c, st, "gemm_dgrad", launch_conv3x3_bf16(dy_, rows, H_, H_, L.C, L.wflip, L.Kpf, L.Cin, ep, zeros_, st));
    } else {
      VF_KS(c, st, "im2col", launch_im2col3x3(dy_, rows, H_, H_, L.C, cols_, L.Kpf, st));
      VF_KS(c, st, "gemm_dgrad", launch_gemm_bf16(cols_, L.Kpf, L.wflip, L.Kpf, rows, L.Cin, L.Kpf, 1, 0, ep, st));
    }
    return VF_OK;
  }

  int bn_bwd(Ctx& c, ConvLayer& L, float* da, int rows, int keep_dpre, const float* P, float w, int node,
             hipStream_t st) {
    VF_KS(c, st, "bn_bwd", launch_bn2d_bwd(da, L.a, L.y, rows, L.C, P + L.g_off, 1, L.mean, L.rstd, partial_, sums_,
                                           keep_dpre, dy_, c.gout(L.g_off, w, node), c.gout(L.be_off, w, node), st));
    return VF_OK;
  }

  int backward(Ctx& c, const StepArgs& s, int i, hipStream_t st) {
    const int b = s.sizes[i];
    const int rows = b * HW_;
    const float w = s.w[i];
    const float* P = s.params;
    // classifier: the gradient of the pooled features first (right behind the kernel that wrote
    // dz), then the bias and weight gradients
    {
      Epilogue ep;
      ep.C = dpooled_; ep.ldc = ldc_;
      VF_KS(c, st, "gemm_dgrad", launch_gemm_bf16(dz_, ldz_, fc_wnat_, ldz_, b, C_, cfg_.classes, 1, 0, ep, st));
    }
    VF_KS(c, st, "bias_grad", launch_rowsum_bf16(dzT_, ldb_, cfg_.classes, b, c.gout(fc_b_off_, w, i), st));
    VF_KS(c, st, "transpose", launch_transpose_bf16(pooled_, ldc_, pooledT_, ldb_, b, C_, st));
    {
      GradOut go = c.gout(fc_w_off_, w, i);
      Epilogue ep;
      ep.C = go.dst; ep.ldc = cfg_.classes; ep.alpha = go.alpha;
      if (go.accumulate) { ep.R = go.dst; ep.ldr = cfg_.classes; ep.beta = 1.f; }
      VF_KS(c, st, "gemm_wgrad", launch_gemm_bf16(pooledT_, ldb_, dzT_, ldb_, C_, cfg_.classes, b, 1, 0, ep, st));
    }
    VF_KS(c, st, "avgpool", launch_avgpool_bwd(dpooled_, ldc_, b, HW_, C_, gA_, st));
    for (int blk = cfg_.n_blocks - 1; blk >= 0; --blk) {
      ConvLayer& L1 = layers_[1 + 2 * blk];
      ConvLayer& L2 = layers_[2 + 2 * blk];
      // gA_: gradient w.r.t. the block's output; afterwards (keep_dpre) w.r.t. the sum before its ReLU,
      // which is also what flows through the skip connection
      VF_TRY(bn_bwd(c, L2, gA_, rows, 1, P, w, i, st));
      VF_TRY(conv_wgrad(c, L2, rows, w, i, st));
      VF_TRY(conv_dgrad(c, L2, rows, gB_, nullptr, st));
      VF_TRY(bn_bwd(c, L1, gB_, rows, 0, P, w, i, st));
      VF_TRY(conv_wgrad(c, L1, rows, w, i, st));
      VF_TRY(conv_dgrad(c, L1, rows, gA_, gA_, st));          // through the convolutions + through the skip
    }
    VF_TRY(bn_bwd(c, layers_[0], gA_, rows, 0, P, w, i, st));
    VF_TRY(conv_wgrad(c, layers_[0], rows, w, i, st));
    return VF_OK;
  }

  vf_config cfg_;
  bool explicit_ = std::getenv("VF_CONV_EXPLICIT") != nullptr;   // tuning aid: always write the patch matrix
  int H_ = 0, HW_ = 0, C_ = 0;
  int64_t P_ = 0, rows_max_ = 0;
  int64_t ldr_ = 0;                // pitch of the transposed [channels, rows] operands
  int64_t ldb_ = 0, ldc_ = 0, ldz_ = 0;   // pitches: node rows, channels, classes (rounded to 8)
  int64_t fc_w_off_ = 0, fc_b_off_ = 0;
  std::vector<ConvLayer> layers_;
  bf16_t* cols_ = nullptr;         // [rows, Kp] patch matrix (of a layer's input, or of an output gradient)
  bf16_t* zeros_ = nullptr;        // 128 bytes of 0: what the product kernel reads outside the image
  bf16_t* colsT_ = nullptr;        // [Kp, ldr]  patches transposed
  bf16_t* dyT_ = nullptr;          // [C, ldr]   output gradient transposed
  bf16_t* inT_ = nullptr;          // [Cin, ldr] a layer's input transposed
  bf16_t* dy_ = nullptr;           // [rows, C]  gradient w.r.t. a convolution output
  float* gA_ = nullptr;            // [rows, C]  gradients w.r.t. activations (two, alternating)
  float* gB_ = nullptr;
  float* partial_ = nullptr;       // per-chunk partial results of the tall reductions
  float* sums_ = nullptr;          // [2, C]
  float* slabs_ = nullptr;         // contraction slabs of a weight gradient
  bf16_t* fc_wnat_ = nullptr;      // classifier W [C, ldz]
  bf16_t* fc_wtr_ = nullptr;       // classifier W^T [classes, ldc]
  bf16_t* pooled_ = nullptr;       // [b, ldc]
  bf16_t* pooledT_ = nullptr;      // [C, ldb]
  float* zslab_ = nullptr;         // [b, ldz] logits as the product leaves them
  float* z_ = nullptr;             // [b, ldz]
  bf16_t* dz_ = nullptr;           // [b, ldz]
  bf16_t* dzT_ = nullptr;          // [classes, ldb]
  float* dpooled_ = nullptr;       // [b, ldc]
  float* state_ = nullptr;         // moving means of all layers, then moving variances
};

}  // namespace

std::unique_ptr<Model> make_conv(const vf_config& cfg) { return std::unique_ptr<Model>(new Conv(cfg)); }

}  // namespace vf
