// MLP with optional per-node BatchNorm: buffers and the launch sequence of one virtual node
// (forward, loss, backward), Section 3.2 steps 1-3.
#include <algorithm>

#include "vf_ctx.h"

namespace vf {
namespace {

inline int64_t round8(int64_t v) { return (v + 7) & ~int64_t(7); }

struct Layer {
  int K = 0, N = 0;
  bool hidden = false, has_bias = false, has_bn = false;
  int64_t w_off = -1, b_off = -1, g_off = -1, be_off = -1;   // flat parameter offsets
  int64_t ldn = 0, ldt = 0;        // leading dims of the bf16 weight copies
  bf16_t* wnat = nullptr;          // bf16 W  [K, ldn]   (contraction = N: input gradients)
  bf16_t* wtr = nullptr;           // bf16 W^T [N, ldt]  (contraction = K: forward)
  int64_t ld = 0;                  // leading dim of this layer's [b, N] buffers (N rounded to 8)
  // Tensors that pass from a node's forward part to its backward part come in two sets
  // (Ctx::aset): with two streams the next node's forward part runs beside this node's backward.
  float* z[2] = {nullptr, nullptr};     // fp32 [max_b, ld]: Linear output (logits for the last layer)
  float* mean[2] = {nullptr, nullptr};  // [N]
  float* rstd[2] = {nullptr, nullptr};  // [N]
  int64_t s_off = 0;               // offset of this layer's moving statistics within a state half
  void* a[2] = {nullptr, nullptr};      // T [max_b, ld]: activation after BatchNorm/ReLU
  // T [max_b, ld]: gradient w.r.t. z.  Two sets only for the last layer (the softmax of the
  // forward part writes it); the hidden layers' are written and read by the backward part.
  void* dz[2] = {nullptr, nullptr};
  // Weight-gradient operands, transposed: one wide matrix [N, ldw] each, in which node i owns
  // the columns of copy Ctx::slot(i) (Mlp::cols), its rows contiguous along the matrix row.  So
  // the operands of a whole fold window are still there when its weight gradients are taken in
  // one pass, or (two streams) the second stream can read node i's operands while the first
  // produces those of node i+1; and the nodes of a window of equal sizes lie side by side, one
  // long contraction.
  bf16_t* aT = nullptr;      // a transposed
  bf16_t* dzT = nullptr;     // dz transposed
};

class Mlp final : public Model {
 public:
  explicit Mlp(const vf_config& cfg) : cfg_(cfg) {
    bf16_ = cfg.dtype == VF_BF16;
    // a unit of the passes is one node of any size, or up to node_group nodes of at most 128 rows each
    // (max_group), and never has more rows than a batch: every per-unit buffer is sized for that
    group_ = bf16_ ? std::max(1, cfg.node_group) : 1;
    const int64_t grouped = std::min<int64_t>((int64_t)std::min(cfg.max_node_size, 128) * group_,
                                              std::max(cfg.max_batch, cfg.max_node_size));
    max_rows_ = (int)std::max<int64_t>(cfg.max_node_size, group_ > 1 ? grouped : 0);
    // as many copies of the weight-gradient operands as Ctx::copies() will ask for
    copies_ = std::max((cfg.flags & VF_FLAG_OVERLAP) ? 2 : 1, cfg.fold_window);
    const int nl = cfg.n_dims - 1;
    int64_t off = 0;
    layers_.resize(nl);
    for (int l = 0; l < nl; ++l) {
      Layer& L = layers_[l];
      L.K = cfg.dims[l];
      L.N = cfg.dims[l + 1];
      L.hidden = l < nl - 1;
      L.has_bn = L.hidden && cfg.batchnorm;
      L.has_bias = !L.has_bn;
      L.w_off = off; off += (int64_t)L.K * L.N;
      if (L.has_bias) { L.b_off = off; off += L.N; }
      if (L.has_bn) { L.g_off = off; off += L.N; L.be_off = off; off += L.N; }
      L.ld = round8(L.N);
      L.ldn = round8(L.N);
      L.ldt = round8(L.K);
      // The class dimension is the contraction of the last layer's input-gradient product: with both
      // operands' rows padded to whole 64-element stages (the padding stays zero: the arena starts
      // zeroed and no kernel writes anything else there) that product has no ragged contraction
      // and runs on the 256-row kernel (2048 x 8192 x 1000: 85 us; x 1024: 38 us).
      if (bf16_ && !L.hidden) L.ld = L.ldn = (L.N + 63) / 64 * 64;
    }
    P_ = off;
    for (Layer& L : layers_)
      if (L.has_bn) { L.s_off = bn_width_; bn_width_ += L.N; }
    ldb_ = round8(max_rows_);
    ldw_ = ldb_ * copies_;
    ordered_ = (cfg.flags & VF_FLAG_ORDERED_FOLD) != 0;
    // Scratch for GEMM outputs that arrive as partial slabs: the largest split * rows * ld
    // over the forward (N_l columns) and input-gradient (K_l columns) products.
    slab_elems_ = 0;
    for (const Layer& L : layers_) {
      slab_elems_ = std::max(slab_elems_, slab_need(max_rows_, L.N, L.K, L.ld));
      slab_elems_ = std::max(slab_elems_, slab_need(max_rows_, L.K, kdim(L), round8(L.K)));
    }
  }

  // split * rows * ld maximised over node sizes up to max_b (the split only changes when the
  // number of row tiles does)
  int64_t slab_need(int max_b, int N, int K, int64_t ld) const {
    int64_t need = 0;
    auto probe = [&](int m) {
      if (m > max_b) m = max_b;
      int split = bf16_ ? gemm_bf16_pick_split(m, N, K) : gemm_f32_pick_split(m, N, K);
      need = std::max(need, (int64_t)split * m * ld);
    };
    probe(32); probe(64);
    for (int m = 128; m < max_b + 128; m += 128) probe(m);
    return need;
  }

  // contraction length of layer L's input-gradient product (the last layer's rows are zero-padded)
  int kdim(const Layer& L) const { return (bf16_ && !L.hidden) ? (int)L.ld : L.N; }

  int split_for(int b, int N, int K, int64_t ld) const {
    int split = bf16_ ? gemm_bf16_pick_split(b, N, K) : gemm_f32_pick_split(b, N, K);
    while (split > 1 && (int64_t)split * b * ld > slab_elems_) split /= 2;
    return split;
  }

  int64_t num_params() const override { return P_; }
  bool supports_overlap() const override { return bf16_; }
  // groups of nodes: the BatchNorm kernels keep a node of up to 128 rows in registers, and the
  // transposed copies want node boundaries on 16-byte boundaries
  int max_group(int rows) const override { return (bf16_ && rows <= 128 && (rows & 7) == 0) ? 32 : 1; }
  bool groups_unequal() const override { return true; }
  int max_window() const override { return bf16_ ? kFoldMax : 1; }

  // The side part finishes the layers from the last to the first; a layer's stretch of the
  // parameter vector (its weights and the small vectors after them) can be updated then.  A
  // layer whose stretch does not start on a 16-byte boundary goes with the layer before it.
  void update_ranges(std::vector<UpdateRange>* out) const override {
    out->clear();
    range_layer_.clear();
    int64_t end = P_;
    for (int l = (int)layers_.size() - 1; l >= 0; --l) {
      const int64_t start = l == 0 ? 0 : layers_[l].w_off;
      if (start & 3) continue;
      UpdateRange r;
      r.off = start; r.n = end - start;
      out->push_back(r);
      range_layer_.push_back(l);
      end = start;
    }
  }

  void request_buffers(Arena& a) override {
    const size_t mb = (size_t)max_rows_;
    const size_t esz = bf16_ ? 2 : 4;
    const int sets = (bf16_ && (cfg_.flags & VF_FLAG_OVERLAP)) ? 2 : 1;
    for (Layer& L : layers_) {
      for (int q = 0; q < sets; ++q) {
        a.request(&L.z[q], mb * L.ld);
        if (q == 0 || !L.hidden) a.request(reinterpret_cast<char**>(&L.dz[q]), mb * L.ld * esz);
        if (L.hidden) {
          a.request(&L.mean[q], (size_t)L.N * group_);      // per node of a group
          a.request(&L.rstd[q], (size_t)L.N * group_);
          a.request(reinterpret_cast<char**>(&L.a[q]), mb * L.ld * esz);
        }
      }
      if (bf16_) {
        a.request(&L.wnat, (size_t)L.K * L.ldn);
        a.request(&L.wtr, (size_t)L.N * L.ldt);
        a.request(&L.dzT, (size_t)L.N * ldw_);
        if (L.hidden) a.request(&L.aT, (size_t)L.N * ldw_);
      }
    }
    if (bf16_) a.request(&xT_, (size_t)cfg_.dims[0] * ldw_);
    for (int q = 0; q < sets; ++q) a.request(&slab_[q], (size_t)slab_elems_);
    sets_ = sets;
    if (bn_width_) a.request(&state_, (size_t)(2 * bn_width_));
  }

  int64_t state_floats() const override { return 2 * bn_width_; }
  float* state_ptr() const override { return state_; }
  int init_state(hipStream_t st) override {   // moving mean 0, moving variance 1
    if (!bn_width_) return VF_OK;
    VF_TRY(launch_fill_f32(state_, 0.f, bn_width_, st));
    return launch_fill_f32(state_ + bn_width_, 1.f, bn_width_, st);
  }

  int prepare(Ctx& c, const float* params, hipStream_t st) override {
    if (!bf16_) return VF_OK;
    for (Layer& L : layers_)
      VF_KS(c, st, "cast_weight", launch_cast_weight(params + L.w_off, L.K, L.N, L.wnat, L.ldn, L.wtr, L.ldt, st));
    return VF_OK;
  }

  // The first layer's copies on `first`; the others on `second`, each followed by an event that
  // node 0's forward part waits for before that layer's product.  (The backward parts run on
  // `second`, behind the copies.)
  int prepare_split(Ctx& c, const float* params, hipStream_t first, hipStream_t second) override {
    if (!bf16_) return VF_OK;
    const int nl = (int)layers_.size();
    for (int l = 0; l < nl; ++l) {
      Layer& L = layers_[l];
      hipStream_t st = l == 0 ? first : second;
      VF_KS(c, st, "cast_weight", launch_cast_weight(params + L.w_off, L.K, L.N, L.wnat, L.ldn, L.wtr, L.ldt, st));
      if (l == 0) continue;
      if (!cast_done_[l]) VF_HIP(hipEventCreateWithFlags(&cast_done_[l], hipEventDisableTiming));
      VF_HIP(hipEventRecord(cast_done_[l], st));
    }
    wait_casts_ = true;
    return VF_OK;
  }

  ~Mlp() override {
    for (hipEvent_t e : cast_done_)
      if (e) (void)hipEventDestroy(e);
  }

  int run_node_main(Ctx& c, const StepArgs& s, int i, hipStream_t st) override {
    VF_TRY(run_node_fwd(c, s, i, st));
    return run_node_bwd(c, s, i, st);
  }

  // Forward pass and loss of node i.
  int run_node_fwd(Ctx& c, const StepArgs& s, int i, hipStream_t st) override {
    const int64_t pc = cols(c, s, i);        // where node i's copy of the side part's operands starts
    const int q = std::min(c.aset(i), sets_ - 1);
    float* slab_buf = slab_[0];
    const int b = s.sizes[i];
    const int64_t row0 = s.off[i];
    const float w = s.w[i];
    const float* P = s.params;
    const int nl = (int)layers_.size();
    const int D = cfg_.dims[0];
    const void* x = bf16_ ? (const void*)(static_cast<const bf16_t*>(s.x) + row0 * D)
                          : (const void*)(static_cast<const float*>(s.x) + row0 * D);
    const int32_t* y = s.y + row0;

    for (int l = 0; l < nl; ++l) {
      Layer& L = layers_[l];
      const void* in = l == 0 ? x : layers_[l - 1].a[q];
      const int64_t ldin = l == 0 ? D : layers_[l - 1].ld;
      const int split = split_for(b, L.N, L.K, L.ld);
      const int64_t slab = (int64_t)b * L.ld;
      if (wait_casts_ && l >= 1) VF_HIP(hipStreamWaitEvent(st, cast_done_[l], 0));
      // an unsliced product of a hidden layer writes the pre-activation where it is kept: the
      // normalisation kernel then has nothing to copy
      float* zsrc = (split == 1 && L.hidden) ? L.z[q] : slab_buf;
      // A unit of whole nodes of 128 rows on a wide layer: the product's epilogue takes BatchNorm and
      // ReLU itself (the pre-activations are stored and not read again in this pass); the scratch
      // holds the per-node variances for the small launch that blends the moving statistics.
      bool whole = bf16_ && L.hidden && split == 1 && s.group(i) >= 2 && b == 128 * s.group(i);
      for (int n = 0; n < s.group(i) && whole; ++n) whole = s.rows_of(i)[n] == 128;
      if (whole) {
        BnFwdArgs ff;
        ff.z = L.z[q]; ff.ldz = L.ld;
        if (L.has_bn) { ff.gamma = P + L.g_off; ff.beta = P + L.be_off; }
        else if (L.has_bias) ff.bias = P + L.b_off;
        ff.round_params = bf16_;
        ff.eps = cfg_.bn_eps;
        ff.a = static_cast<bf16_t*>(L.a[q]); ff.lda = L.ld;
        ff.aT = L.aT + pc; ff.ldt = ldw_;
        ff.mean = L.mean[q]; ff.rstd = L.rstd[q]; ff.var = slab_buf;
        if (gemm_bf16_bn_fwd_takes(static_cast<const bf16_t*>(in), ldin, L.wtr, L.ldt, b, L.N, L.K, ff)) {
          VF_KS(c, st, "gemm_fwd_bn", launch_gemm_bf16_bn_fwd(static_cast<const bf16_t*>(in), ldin, L.wtr, L.ldt, b, L.N, L.K, ff, st));
          if (L.has_bn)
            VF_KS(c, st, "bn_stats_finish", launch_bn_stats_finish(L.mean[q], slab_buf, s.group(i), L.N, state_ + L.s_off,
                                                                   state_ + bn_width_ + L.s_off, cfg_.bn_momentum, st));
          continue;
        }
      }
      Epilogue ep;
      ep.C = zsrc; ep.ldc = L.ld;
      if (L.has_bias) { ep.bias = P + L.b_off; ep.bias_round_bf16 = bf16_; }
      if (bf16_)
        VF_KS(c, st, "gemm_fwd", launch_gemm_bf16(static_cast<const bf16_t*>(in), ldin, L.wtr, L.ldt, b, L.N, L.K,
                                                  split, slab, ep, st));
      else
        VF_KS(c, st, "gemm_fwd", launch_gemm_f32(static_cast<const float*>(in), ldin, 1, P + L.w_off, 1, L.N, b, L.N, L.K, split, slab, ep, st));
      if (L.hidden)
        VF_KS(c, st, "bn_relu_fwd", launch_bn_relu_fwd(zsrc, split, slab, L.ld, s.seg[i], L.N,
                                       L.has_bn ? P + L.g_off : nullptr, L.has_bn ? P + L.be_off : nullptr,
                                       bf16_, cfg_.bn_eps, L.z[q], L.ld, L.a[q], L.ld, bf16_, bf16_ ? L.aT + pc : nullptr, ldw_,
                                       L.mean[q], L.rstd[q], L.has_bn ? state_ + L.s_off : nullptr,
                                       L.has_bn ? state_ + bn_width_ + L.s_off : nullptr, cfg_.bn_momentum, st,
                                       s.group(i), s.rows_of(i)));
      else
        VF_KS(c, st, "softmax_xent", launch_softmax_xent(slab_buf, split, slab, L.ld, L.z[q], L.ld, y, b, L.N,
                                                         c.rowloss + row0, L.dz[q], L.ld, bf16_, bf16_ ? L.dzT + pc : nullptr, ldw_, w, i,
                                                         nullptr, nullptr, st, tscale(c, s, i)));
    }
    wait_casts_ = false;
    // loss bookkeeping of the whole step after the last node's rows are in: node losses and
    // their weighted sum (Section 5.2), in node order
    if (i == s.V - 1) {
      for (int first = 0; first < s.nodes; first += kLossNodes) {
        LossNodes ln{};
        ln.first = first;
        ln.count = std::min(kLossNodes, s.nodes - first);
        for (int j = 0; j < ln.count; ++j) {
          ln.off[j] = s.node_off[first + j]; ln.rows[j] = s.node_sizes[first + j]; ln.w[j] = s.node_w[first + j];
        }
        VF_KS(c, st, "loss_reduce", launch_loss_reduce_nodes(c.rowloss, ln, c.node_loss, c.loss_total, st));
      }
    }
    return VF_OK;
  }

  // The input-gradient chain of node i (with the small-vector gradients the BatchNorm/ReLU
  // backward kernels fold into the gradient buffer on the way).
  int run_node_bwd(Ctx& c, const StepArgs& s, int i, hipStream_t st) override {
    const int64_t pc = cols(c, s, i);
    const int q = std::min(c.aset(i), sets_ - 1);
    float* slab_buf = slab_[sets_ - 1];      // the backward stream's own scratch when there are two
    const int b = s.sizes[i];
    const float w = s.w[i];
    const float* P = s.params;
    const int nl = (int)layers_.size();
    for (int l = nl - 1; l >= 1; --l) {
      Layer& L = layers_[l];
      // input gradient da[l-1][b,K] = dz W^T, then through ReLU / BatchNorm of layer l-1
      Layer& Pv = layers_[l - 1];
      const void* dz_in = L.hidden ? L.dz[0] : L.dz[q];
      const int split = split_for(b, L.K, kdim(L), Pv.ld);
      const int64_t slab = (int64_t)b * Pv.ld;
      Epilogue ed;
      ed.C = slab_buf; ed.ldc = Pv.ld;
      GradOut gg = Pv.has_bn ? c.gout(Pv.g_off, w, i) : GradOut{nullptr, 0.f, 0};
      GradOut gb = c.gout(Pv.has_bn ? Pv.be_off : Pv.b_off, w, i);
      // A unit of whole nodes of 128 rows on a wide layer: the product's epilogue takes the BatchNorm /
      // ReLU backward pass itself (the incoming gradient is never stored); the scratch holds the
      // per-node column sums for the small launch that makes the scale / shift gradients of them.
      bool whole = bf16_ && split == 1 && s.group(i) >= 2 && b == 128 * s.group(i);
      for (int n = 0; n < s.group(i) && whole; ++n) whole = s.rows_of(i)[n] == 128;
      if (whole) {
        BnBwdArgs fa;
        fa.z = Pv.z[q]; fa.ldz = Pv.ld;
        fa.mean = Pv.mean[q]; fa.rstd = Pv.rstd[q];
        fa.gamma = Pv.has_bn ? P + Pv.g_off : nullptr; fa.beta = Pv.has_bn ? P + Pv.be_off : nullptr;
        fa.round_params = bf16_;
        fa.dz = static_cast<bf16_t*>(Pv.dz[0]); fa.lddz = Pv.ld;
        fa.dzT = Pv.dzT + pc; fa.ldt = ldw_;
        fa.tscale = tscale(c, s, i);
        fa.sums = slab_buf;
        if (gemm_bf16_bn_bwd_takes(static_cast<const bf16_t*>(dz_in), L.ld, L.wnat, L.ldn, b, L.K, kdim(L), fa)) {
          VF_KS(c, st, "gemm_dgrad_bn", launch_gemm_bf16_bn_bwd(static_cast<const bf16_t*>(dz_in), L.ld, L.wnat, L.ldn, b, L.K,
                                                             kdim(L), fa, st));
          VF_KS(c, st, "bn_sums_finish", launch_bn_sums_finish(slab_buf, s.group(i), Pv.N, gg, gb, st));
          continue;
        }
      }
      if (bf16_)
        VF_KS(c, st, "gemm_dgrad", launch_gemm_bf16(static_cast<const bf16_t*>(dz_in), L.ld, L.wnat, L.ldn, b, L.K, kdim(L),
                                                    split, slab, ed, st));
      else
        VF_KS(c, st, "gemm_dgrad", launch_gemm_f32(static_cast<const float*>(dz_in), L.ld, 1, P + L.w_off, L.N, 1, b, L.K, L.N, split, slab, ed, st));
      VF_KS(c, st, "bn_relu_bwd", launch_bn_relu_bwd(slab_buf, split, slab, Pv.ld, Pv.z[q], Pv.ld, s.seg[i], Pv.N,
                                     Pv.has_bn ? P + Pv.g_off : nullptr, Pv.has_bn ? P + Pv.be_off : nullptr,
                                     bf16_, Pv.mean[q], Pv.rstd[q], Pv.dz[0], Pv.ld, bf16_, bf16_ ? Pv.dzT + pc : nullptr, ldw_,
                                     gg, gb, st, tscale(c, s, i), s.group(i), s.rows_of(i)));
    }
    return VF_OK;
  }

  // Weight gradients, the last layer's bias gradient, and (staged mode) the fold, of nodes
  // i0 .. i0+count-1.  Reads the transposed operands (bf16) that their main parts wrote.
  int run_nodes_side(Ctx& c, const StepArgs& s, int i0, int count, hipStream_t st) override {
    const int nl = (int)layers_.size();
    const int D = cfg_.dims[0];
    // One pass over the gradient buffer for the whole window: fused fold, bf16, every node short
    // enough for the single-trip kernel, shapes the 16-byte epilogue accepts.
    bool fold = bf16_ && c.fused && count > 1;
    for (int i = i0; i < i0 + count && fold; ++i) fold = s.sizes[i] <= 128;
    for (const Layer& L : layers_) fold = fold && (L.N & 3) == 0 && ((L.w_off & 3) == 0);
    // Nodes of one size have one weight w, and their operand copies lie side by side: the
    // window's weighted sum is w times ONE product over all its rows.
    const int kind = join_kind(c, s, i0, count);
    const bool joined = kind != kJoinNone;
    if (joined) fold = false;
    // after the step's last window layer l's gradient is final
    const bool last_window = i0 + count == s.V;
    auto layer_done = [&](int l) -> int {
      if (!last_window) return VF_OK;
      for (size_t k = 0; k < range_layer_.size(); ++k)
        if (range_layer_[k] == l) return c.mark_range((int)k, st);
      return VF_OK;
    };

    if (fold) {   // the window's small launches batched, then one fold per layer
      NodeList xs{}, ds{};
      xs.count = ds.count = count;
      ds.overwrite = i0 == 0;
      const Layer& last = layers_[nl - 1];
      for (int j = 0; j < count; ++j) {
        const int64_t pc = cols(c, s, i0 + j);
        xs.src[j] = static_cast<const bf16_t*>(s.x) + (int64_t)s.off[i0 + j] * D;
        xs.dst[j] = xT_ + pc;
        ds.src[j] = last.dzT + pc;
        xs.rows[j] = ds.rows[j] = s.sizes[i0 + j];
        ds.w[j] = s.w[i0 + j];
      }
      VF_KS(c, st, "transpose", launch_transpose_nodes(xs, D, ldw_, D, st));
      VF_KS(c, st, "bias_grad", launch_rowsum_nodes(ds, ldw_, last.N, c.gbuf + last.b_off, st));
    }
    if (joined) {
      // x of the whole window is one contiguous block of rows: one transpose
      const int rows = (int)(s.off[i0 + count - 1] + s.sizes[i0 + count - 1] - s.off[i0]);
      const float w = kind == kJoinScaled ? 1.f : s.w[i0];    // scaled: the weights are in the operand
      const int64_t pc = cols(c, s, i0);
      VF_KS(c, st, "transpose", launch_transpose_bf16(static_cast<const bf16_t*>(s.x) + (int64_t)s.off[i0] * D, D,
                                                      xT_ + pc, ldw_, rows, D, st));
      for (int l = nl - 1; l >= 0; --l) {
        Layer& L = layers_[l];
        GradOut go = c.gout(L.w_off, w, i0);
        if (!L.hidden)
          VF_KS(c, st, "bias_grad", launch_rowsum_bf16(L.dzT + pc, ldw_, L.N, rows, c.gout(L.b_off, w, i0), st));
        Epilogue ep;
        ep.C = go.dst; ep.ldc = L.N; ep.alpha = go.alpha;
        if (go.accumulate) { ep.R = go.dst; ep.ldr = L.N; ep.beta = 1.f; }
        VF_KS(c, st, "gemm_wgrad", launch_gemm_bf16((l == 0 ? xT_ : layers_[l - 1].aT) + pc, ldw_, L.dzT + pc, ldw_,
                                                    L.K, L.N, rows, 1, 0, ep, st));
        VF_TRY(layer_done(l));
      }
      return VF_OK;
    }
    for (int i = i0; i < i0 + count && !fold; ++i) {
      const int64_t pc = cols(c, s, i);
      const int b = s.sizes[i];
      const int64_t row0 = s.off[i];
      const float w = s.w[i];
      const void* x = bf16_ ? (const void*)(static_cast<const bf16_t*>(s.x) + row0 * D)
                            : (const void*)(static_cast<const float*>(s.x) + row0 * D);
      if (bf16_)
        VF_KS(c, st, "transpose", launch_transpose_bf16(static_cast<const bf16_t*>(x), D, xT_ + pc, ldw_, b, D, st));
      for (int l = nl - 1; l >= 0; --l) {
        Layer& L = layers_[l];
        const void* in = l == 0 ? x : layers_[l - 1].a[0];   // fp32 path: one tensor set
        const int64_t ldin = l == 0 ? D : layers_[l - 1].ld;
        if (!L.hidden) {   // last layer: bias gradient = sums over the node of dlogits
          if (bf16_) VF_KS(c, st, "bias_grad", launch_rowsum_bf16(L.dzT + pc, ldw_, L.N, b, c.gout(L.b_off, w, i), st));
          else       VF_KS(c, st, "bias_grad", launch_colsum(L.dz[0], L.ld, 0, b, L.N, c.gout(L.b_off, w, i), st));
        }
        GradOut go = c.gout(L.w_off, w, i);
        Epilogue ep;
        ep.C = go.dst; ep.ldc = L.N; ep.alpha = go.alpha;
        if (go.accumulate) { ep.R = go.dst; ep.ldr = L.N; ep.beta = 1.f; }
        if (bf16_) {
          const bf16_t* inT = (l == 0 ? xT_ : layers_[l - 1].aT) + pc;
          VF_KS(c, st, "gemm_wgrad", launch_gemm_bf16(inT, ldw_, L.dzT + pc, ldw_, L.K, L.N, b, 1, 0, ep, st));
        } else {
          VF_KS(c, st, "gemm_wgrad", launch_gemm_f32(static_cast<const float*>(in), 1, ldin,
                                                     static_cast<const float*>(L.dz[0]), 1, L.ld, L.K, L.N, b, 1, 0, ep, st));
        }
        if (c.fused && i == i0 + count - 1) VF_TRY(layer_done(l));
      }
      VF_TRY(c.fold(i, w, st));
      if (!c.fused && i == i0 + count - 1)
        for (int l = nl - 1; l >= 0; --l) VF_TRY(layer_done(l));
    }
    if (fold) {
      for (int l = nl - 1; l >= 0; --l) {
        Layer& L = layers_[l];
        FoldArgs fa{};
        fa.count = count;
        fa.overwrite = i0 == 0;
        for (int j = 0; j < count; ++j) {
          const int64_t pc = cols(c, s, i0 + j);
          fa.A[j] = (l == 0 ? xT_ : layers_[l - 1].aT) + pc;
          fa.B[j] = L.dzT + pc;
          fa.K[j] = s.sizes[i0 + j];
          fa.w[j] = s.w[i0 + j];
        }
        VF_KS(c, st, "gemm_wgrad", launch_gemm_bf16_fold(fa, ldw_, L.K, L.N, c.gbuf + L.w_off, L.N, st));
        VF_TRY(layer_done(l));
      }
    }
    return VF_OK;
  }

 private:
  // The window of node i (first node, node count).
  static void window_of(const Ctx& c, const StepArgs& s, int i, int* i0, int* count) {
    *i0 = i / c.window * c.window;
    *count = std::min(c.window, s.V - *i0);
  }
  // How the weighted gradient sum of the window i0 .. i0+count-1 is taken:
  //   kJoinNone    node by node (or the chain kernel),
  //   kJoinEqual   several nodes of ONE size (hence one weight b_i/B): the weight times one product
  //                over all the window's rows,
  //   kJoinScaled  nodes of several sizes: one product over all the window's rows, each node's rows
  //                of the transposed output gradients holding w_i dz (the per-sample gradient of the
  //                step's loss, Section 5.2) instead of dz.
  // Both joined kinds need node sizes that keep the operand copies 16-byte aligned.
  enum { kJoinNone = 0, kJoinEqual = 1, kJoinScaled = 2 };
  int join_kind(const Ctx& c, const StepArgs& s, int i0, int count) const {
    if (!bf16_ || !c.fused || ordered_ || count < 2) return kJoinNone;
    bool equal = true;
    for (int i = i0; i < i0 + count; ++i) {
      if (s.sizes[i] & 7) return kJoinNone;
      equal = equal && s.sizes[i] == s.sizes[i0];
    }
    return equal ? kJoinEqual : kJoinScaled;
  }
  bool side_by_side(const Ctx& c, const StepArgs& s, int i0, int count) const {
    return join_kind(c, s, i0, count) != kJoinNone;
  }
  // What the transposed output gradients of node i are scaled by (see join_kind).
  float tscale(const Ctx& c, const StepArgs& s, int i) const {
    int i0, count;
    window_of(c, s, i, &i0, &count);
    return join_kind(c, s, i0, count) == kJoinScaled ? s.w[i] : 1.f;
  }
  // First column of node i's copy in the wide transposed operands: copies are ldb_ columns
  // apart, or packed one after the other when the window's nodes are to lie side by side.
  int64_t cols(const Ctx& c, const StepArgs& s, int i) const {
    int i0, count;
    window_of(c, s, i, &i0, &count);
    switch (join_kind(c, s, i0, count)) {
      case kJoinEqual: return (int64_t)c.slot(i) * s.sizes[i0];
      case kJoinScaled: return (int64_t)c.slot(i0) * ldb_ + (s.off[i] - s.off[i0]);
      default: return (int64_t)c.slot(i) * ldb_;
    }
  }

  vf_config cfg_;
  bool bf16_ = false;
  int64_t P_ = 0;
  int64_t ldb_ = 0;
  std::vector<Layer> layers_;
  int copies_ = 2;
  bf16_t* xT_ = nullptr;           // the batch rows of the nodes in flight, transposed [D, ldw_]
  int64_t ldw_ = 0;                // leading dim of the wide transposed operands: copies_ * ldb_
  bool ordered_ = false;           // VF_FLAG_ORDERED_FOLD
  int group_ = 1;                  // nodes per unit of the passes (vf_config::node_group)
  int max_rows_ = 0;               // rows of the largest unit
  hipEvent_t cast_done_[VF_MAX_DIMS] = {};   // prepare_split: layer l's bf16 weight copies are written
  bool wait_casts_ = false;                  // the next forward part waits for them
  mutable std::vector<int> range_layer_;   // update_ranges: the layer that completes stretch k
  float* slab_[2] = {nullptr, nullptr};   // split-contraction scratch of the forward / backward stream
  int sets_ = 1;
  int64_t slab_elems_ = 0;
  int64_t bn_width_ = 0;           // summed width of the BatchNorm layers
  float* state_ = nullptr;         // [2 * bn_width_]: moving means, then moving variances
};

}  // namespace

std::unique_ptr<Model> make_mlp(const vf_config& cfg) { return std::unique_ptr<Model>(new Mlp(cfg)); }

}  // namespace vf
