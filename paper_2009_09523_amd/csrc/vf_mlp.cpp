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
  float* z = nullptr;              // fp32 [max_b, ld]: Linear output (logits for the last layer)
  float* mean = nullptr;           // [N]
  float* rstd = nullptr;           // [N]
  int64_t s_off = 0;               // offset of this layer's moving statistics within a state half
  void* a = nullptr;               // T [max_b, ld]: activation after BatchNorm/ReLU
  void* dz = nullptr;              // T [max_b, ld]: gradient w.r.t. z
  // Weight-gradient operands, transposed ([N, ldb], rows of the node contiguous).  Several
  // copies (Ctx::copies): node i writes copy Ctx::slot(i), so that the operands of a whole fold
  // window are still there when its weight gradients are taken in one pass, or (two streams) the
  // side stream can read node i's operands while the main stream produces those of node i+1.
  bf16_t* aT[kFoldMax] = {};     // a transposed
  bf16_t* dzT[kFoldMax] = {};    // dz transposed
};

class Mlp final : public Model {
 public:
  explicit Mlp(const vf_config& cfg) : cfg_(cfg) {
    bf16_ = cfg.dtype == VF_BF16;
    // as many copies of the weight-gradient operands as Ctx::copies() will ask for
    copies_ = std::max(2, cfg.fold_window);
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
    }
    P_ = off;
    for (Layer& L : layers_)
      if (L.has_bn) { L.s_off = bn_width_; bn_width_ += L.N; }
    ldb_ = round8(cfg.max_node_size);
    // Scratch for GEMM outputs that arrive as partial slabs: the largest split * rows * ld
    // over the forward (N_l columns) and input-gradient (K_l columns) products.
    slab_elems_ = 0;
    for (const Layer& L : layers_) {
      slab_elems_ = std::max(slab_elems_, slab_need(cfg.max_node_size, L.N, L.K, L.ld));
      slab_elems_ = std::max(slab_elems_, slab_need(cfg.max_node_size, L.K, L.N, round8(L.K)));
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

  int split_for(int b, int N, int K, int64_t ld) const {
    int split = bf16_ ? gemm_bf16_pick_split(b, N, K) : gemm_f32_pick_split(b, N, K);
    while (split > 1 && (int64_t)split * b * ld > slab_elems_) split /= 2;
    return split;
  }

  int64_t num_params() const override { return P_; }
  bool supports_overlap() const override { return bf16_; }
  int max_window() const override { return bf16_ ? copies_ : 1; }

  void request_buffers(Arena& a) override {
    const size_t mb = (size_t)cfg_.max_node_size;
    const size_t esz = bf16_ ? 2 : 4;
    for (Layer& L : layers_) {
      a.request(&L.z, mb * L.ld);
      a.request(reinterpret_cast<char**>(&L.dz), mb * L.ld * esz);
      if (L.hidden) {
        a.request(&L.mean, (size_t)L.N);
        a.request(&L.rstd, (size_t)L.N);
        a.request(reinterpret_cast<char**>(&L.a), mb * L.ld * esz);
      }
      if (bf16_) {
        a.request(&L.wnat, (size_t)L.K * L.ldn);
        a.request(&L.wtr, (size_t)L.N * L.ldt);
        for (int k = 0; k < copies_; ++k) {
          a.request(&L.dzT[k], (size_t)L.N * ldb_);
          if (L.hidden) a.request(&L.aT[k], (size_t)L.N * ldb_);
        }
      }
    }
    if (bf16_)
      for (int k = 0; k < copies_; ++k) a.request(&xT_[k], (size_t)cfg_.dims[0] * ldb_);
    a.request(&slab_, (size_t)slab_elems_);
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

  // Forward pass, loss, and the input-gradient chain (with the small-vector gradients the
  // BatchNorm/ReLU backward kernels produce on the way).
  int run_node_main(Ctx& c, const StepArgs& s, int i, hipStream_t st) override {
    const int p = c.slot(i);                 // which copy of the side part's operands
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
      const void* in = l == 0 ? x : layers_[l - 1].a;
      const int64_t ldin = l == 0 ? D : layers_[l - 1].ld;
      const int split = split_for(b, L.N, L.K, L.ld);
      const int64_t slab = (int64_t)b * L.ld;
      Epilogue ep;
      ep.C = slab_; ep.ldc = L.ld;
      if (L.has_bias) { ep.bias = P + L.b_off; ep.bias_round_bf16 = bf16_; }
      if (bf16_)
        VF_KS(c, st, "gemm_fwd", launch_gemm_bf16(static_cast<const bf16_t*>(in), ldin, L.wtr, L.ldt, b, L.N, L.K,
                                                  split, slab, ep, st));
      else
        VF_KS(c, st, "gemm_fwd", launch_gemm_f32(static_cast<const float*>(in), ldin, 1, P + L.w_off, 1, L.N, b, L.N, L.K, split, slab, ep, st));
      if (L.hidden)
        VF_KS(c, st, "bn_relu_fwd", launch_bn_relu_fwd(slab_, split, slab, L.ld, b, L.N,
                                       L.has_bn ? P + L.g_off : nullptr, L.has_bn ? P + L.be_off : nullptr,
                                       bf16_, cfg_.bn_eps, L.z, L.ld, L.a, L.ld, bf16_, L.aT[p], ldb_,
                                       L.mean, L.rstd, L.has_bn ? state_ + L.s_off : nullptr,
                                       L.has_bn ? state_ + bn_width_ + L.s_off : nullptr, cfg_.bn_momentum, st));
      else
        VF_KS(c, st, "softmax_xent", launch_softmax_xent(slab_, split, slab, L.ld, L.z, L.ld, y, b, L.N,
                                                         c.rowloss, L.dz, L.ld, bf16_, L.dzT[p], ldb_, w, i,
                                                         c.node_loss, c.loss_total, st));
    }

    for (int l = nl - 1; l >= 1; --l) {
      Layer& L = layers_[l];
      // input gradient da[l-1][b,K] = dz W^T, then through ReLU / BatchNorm of layer l-1
      Layer& Pv = layers_[l - 1];
      const int split = split_for(b, L.K, L.N, Pv.ld);
      const int64_t slab = (int64_t)b * Pv.ld;
      Epilogue ed;
      ed.C = slab_; ed.ldc = Pv.ld;
      if (bf16_)
        VF_KS(c, st, "gemm_dgrad", launch_gemm_bf16(static_cast<const bf16_t*>(L.dz), L.ld, L.wnat, L.ldn, b, L.K, L.N,
                                                    split, slab, ed, st));
      else
        VF_KS(c, st, "gemm_dgrad", launch_gemm_f32(static_cast<const float*>(L.dz), L.ld, 1, P + L.w_off, L.N, 1, b, L.K, L.N, split, slab, ed, st));
      GradOut gg = Pv.has_bn ? c.gout(Pv.g_off, w, i) : GradOut{nullptr, 0.f, 0};
      GradOut gb = c.gout(Pv.has_bn ? Pv.be_off : Pv.b_off, w, i);
      VF_KS(c, st, "bn_relu_bwd", launch_bn_relu_bwd(slab_, split, slab, Pv.ld, Pv.z, Pv.ld, b, Pv.N,
                                     Pv.has_bn ? P + Pv.g_off : nullptr, Pv.has_bn ? P + Pv.be_off : nullptr,
                                     bf16_, Pv.mean, Pv.rstd, Pv.dz, Pv.ld, bf16_, bf16_ ? Pv.dzT[p] : nullptr, ldb_,
                                     gg, gb, st));
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

    if (fold) {   // the window's small launches batched, then one fold per layer
      NodeList xs{}, ds{};
      xs.count = ds.count = count;
      ds.overwrite = i0 == 0;
      const Layer& last = layers_[nl - 1];
      for (int j = 0; j < count; ++j) {
        const int p = c.slot(i0 + j);
        xs.src[j] = static_cast<const bf16_t*>(s.x) + (int64_t)s.off[i0 + j] * D;
        xs.dst[j] = xT_[p];
        ds.src[j] = last.dzT[p];
        xs.rows[j] = ds.rows[j] = s.sizes[i0 + j];
        ds.w[j] = s.w[i0 + j];
      }
      VF_KS(c, st, "transpose", launch_transpose_nodes(xs, D, ldb_, D, st));
      VF_KS(c, st, "bias_grad", launch_rowsum_nodes(ds, ldb_, last.N, c.gbuf + last.b_off, st));
    }
    for (int i = i0; i < i0 + count && !fold; ++i) {
      const int p = c.slot(i);
      const int b = s.sizes[i];
      const int64_t row0 = s.off[i];
      const float w = s.w[i];
      const void* x = bf16_ ? (const void*)(static_cast<const bf16_t*>(s.x) + row0 * D)
                            : (const void*)(static_cast<const float*>(s.x) + row0 * D);
      if (bf16_)
        VF_KS(c, st, "transpose", launch_transpose_bf16(static_cast<const bf16_t*>(x), D, xT_[p], ldb_, b, D, st));
      for (int l = nl - 1; l >= 0; --l) {
        Layer& L = layers_[l];
        const void* in = l == 0 ? x : layers_[l - 1].a;
        const int64_t ldin = l == 0 ? D : layers_[l - 1].ld;
        if (!L.hidden) {   // last layer: bias gradient = sums over the node of dlogits
          if (bf16_) VF_KS(c, st, "bias_grad", launch_rowsum_bf16(L.dzT[p], ldb_, L.N, b, c.gout(L.b_off, w, i), st));
          else       VF_KS(c, st, "bias_grad", launch_colsum(L.dz, L.ld, 0, b, L.N, c.gout(L.b_off, w, i), st));
        }
        GradOut go = c.gout(L.w_off, w, i);
        Epilogue ep;
        ep.C = go.dst; ep.ldc = L.N; ep.alpha = go.alpha;
        if (go.accumulate) { ep.R = go.dst; ep.ldr = L.N; ep.beta = 1.f; }
        if (bf16_) {
          const bf16_t* inT = l == 0 ? xT_[p] : layers_[l - 1].aT[p];
          VF_KS(c, st, "gemm_wgrad", launch_gemm_bf16(inT, ldb_, L.dzT[p], ldb_, L.K, L.N, b, 1, 0, ep, st));
        } else {
          VF_KS(c, st, "gemm_wgrad", launch_gemm_f32(static_cast<const float*>(in), 1, ldin,
                                                     static_cast<const float*>(L.dz), 1, L.ld, L.K, L.N, b, 1, 0, ep, st));
        }
      }
      VF_TRY(c.fold(i, w, st));
    }
    if (fold) {
      for (int l = nl - 1; l >= 0; --l) {
        Layer& L = layers_[l];
        FoldArgs fa{};
        fa.count = count;
        fa.overwrite = i0 == 0;
        for (int j = 0; j < count; ++j) {
          const int p = c.slot(i0 + j);
          fa.A[j] = l == 0 ? xT_[p] : layers_[l - 1].aT[p];
          fa.B[j] = L.dzT[p];
          fa.K[j] = s.sizes[i0 + j];
          fa.w[j] = s.w[i0 + j];
        }
        VF_KS(c, st, "gemm_wgrad", launch_gemm_bf16_fold(fa, ldb_, L.K, L.N, c.gbuf + L.w_off, L.N, st));
      }
    }
    return VF_OK;
  }

 private:
  vf_config cfg_;
  bool bf16_ = false;
  int64_t P_ = 0;
  int64_t ldb_ = 0;
  std::vector<Layer> layers_;
  int copies_ = 2;
  bf16_t* xT_[kFoldMax] = {};
  float* slab_ = nullptr;
  int64_t slab_elems_ = 0;
  int64_t bn_width_ = 0;           // summed width of the BatchNorm layers
  float* state_ = nullptr;         // [2 * bn_width_]: moving means, then moving variances
};

}  // namespace

std::unique_ptr<Model> make_mlp(const vf_config& cfg) { return std::unique_ptr<Model>(new Mlp(cfg)); }

}  // namespace vf
