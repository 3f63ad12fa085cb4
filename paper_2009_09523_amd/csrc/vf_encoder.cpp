// Pre-LayerNorm transformer encoder with a masked-position cross-entropy head: buffers and the
// launch sequence of one virtual node (forward, loss, backward), Section 3.2 steps 1-3.
//
//   h = tok_emb[ids] + pos_emb;  per layer: h += Wo . attention(LN1(h));  h += W2 . gelu(W1 . LN2(h));
//   logits = Wout . LNf(h[masked positions]);  L_i = mean cross-entropy over the node's masked rows.
#include <algorithm>
#include <cmath>

#include "vf_ctx.h"

namespace vf {
namespace {

inline int64_t round8(int64_t v) { return (v + 7) & ~int64_t(7); }

struct Lin {
  int K = 0, N = 0;
  int64_t w_off = -1, b_off = -1;
  int64_t ldn = 0, ldt = 0;
  bf16_t* wnat = nullptr;   // bf16 W   [K, ldn]
  bf16_t* wtr = nullptr;    // bf16 W^T [N, ldt]
};

// What a node's forward part leaves for its backward part, per block (one set per node in flight).
struct BlockActs {
  float* hin = nullptr;                 // fp32 [R, d] input of the block (residual stream)
  float *mean1 = nullptr, *rstd1 = nullptr, *mean2 = nullptr, *rstd2 = nullptr;
  void* a = nullptr;                    // T [R, d]   LN1 output
  void* qkv_act = nullptr;              // T [R, 3d]
  void* prob = nullptr;                 // T [b*heads, T, T] attention probabilities
  void* om = nullptr;                   // T [R, d]   attention output, heads merged
  float* hmid = nullptr;                // fp32 [R, d] after the attention residual
  void* f = nullptr;                    // T [R, d]   LN2 output
  float* u = nullptr;                   // fp32 [R, ffn] FFN pre-activation (a Linear output: not an operand of a product)
  void* g = nullptr;                    // T [R, ffn] gelu(u)
  // ... and what its backward part leaves for weight gradients taken later (deferred mode):
  // the transposed output gradients [N, ldR] of w2, w1, o, qkv
  bf16_t* dyT[4] = {nullptr, nullptr, nullptr, nullptr};
};

struct Block {
  int64_t ln1_g, ln1_b, ln2_g, ln2_b;
  Lin qkv, o, w1, w2;
  BlockActs x[2];
};

// ... and after the blocks: the masked rows, their statistics, labels and logit gradients.
struct HeadActs {
  float* hlast = nullptr;               // fp32 [R, d] output of the last block
  int32_t *rowidx = nullptr, *labels = nullptr;
  float *meanf = nullptr, *rstdf = nullptr;
  void* rows = nullptr;                 // T [Rm, d] final LayerNorm of the masked rows
  void* dlogits = nullptr;              // T [Rm, ldV]
};

class Encoder final : public Model {
 public:
  explicit Encoder(const vf_config& cfg) : cfg_(cfg) {
    bf16_ = cfg.dtype == VF_BF16;
    d_ = cfg.d_model; f_ = cfg.d_ffn; T_ = cfg.seq_len; V_ = cfg.vocab; m_ = cfg.n_masked;
    nh_ = cfg.n_heads; dh_ = d_ / nh_;
    int64_t off = 0;
    tok_off_ = off; off += (int64_t)V_ * d_;
    pos_off_ = off; off += (int64_t)T_ * d_;
    blocks_.resize(cfg.n_layers);
    auto lin = [&](Lin& L, int K, int N) {
      L.K = K; L.N = N;
      L.w_off = off; off += (int64_t)K * N;
      L.b_off = off; off += N;
      L.ldn = round8(N); L.ldt = round8(K);
      lins_.push_back(&L);
    };
    for (Block& B : blocks_) {
      B.ln1_g = off; off += d_; B.ln1_b = off; off += d_;
      lin(B.qkv, d_, 3 * d_);
      lin(B.o, d_, d_);
      B.ln2_g = off; off += d_; B.ln2_b = off; off += d_;
      lin(B.w1, d_, f_);
      lin(B.w2, f_, d_);
    }
    lnf_g_ = off; off += d_; lnf_b_ = off; off += d_;
    lin(out_, d_, V_);
    P_ = off;
    // a unit of the passes is up to node_group nodes (their sequences are independent: only the
    // loss bookkeeping tells them apart): every per-unit buffer is sized for that many sequences
    max_seqs_ = cfg.max_node_size * std::min(4, std::max(1, cfg.node_group));
    maxR_ = (int64_t)max_seqs_ * T_;
    maxRm_ = (int64_t)max_seqs_ * m_;
    ldR_ = round8(maxR_);
    ldV_ = round8(V_);
    out_split_max_ = 32;
    mfma_attn_ = bf16_ && attn_mfma_supported(T_, dh_);
    // two nodes in flight (forward of one beside the backward of the other) need two sets of
    // what passes from a forward to its backward part
    sets_ = (supports_overlap() && (cfg.flags & VF_FLAG_OVERLAP)) ? 2 : 1;
  }

  int64_t num_params() const override { return P_; }
  // (the row-chunked reductions of the backward pass take units of up to 8192 tokens)
  int max_group(int) const override { return 4; }
  // the forward part of the fp32 / non-MFMA attention path shares its score scratch with the backward part
  bool supports_overlap() const override { return bf16_ && mfma_attn_; }

  void request_buffers(Arena& a) override {
    const size_t esz = bf16_ ? 2 : 4;
    const size_t R = (size_t)maxR_, Rm = (size_t)maxRm_;
    const size_t heads = (size_t)max_seqs_ * nh_;
    auto act = [&](void** p, size_t n) { a.request(reinterpret_cast<char**>(p), n * esz); };
    for (int q = 0; q < sets_; ++q) {
      for (Block& B : blocks_) {
        BlockActs& X = B.x[q];
        a.request(&X.hin, R * d_);
        a.request(&X.mean1, R); a.request(&X.rstd1, R); a.request(&X.mean2, R); a.request(&X.rstd2, R);
        act(&X.a, R * d_); act(&X.qkv_act, R * 3 * d_); act(&X.prob, heads * T_ * T_); act(&X.om, R * d_);
        a.request(&X.hmid, R * d_);
        act(&X.f, R * d_); a.request(&X.u, R * f_); act(&X.g, R * f_);
        if (sets_ == 2) {
          const int widths[4] = {d_, f_, d_, 3 * d_};
          for (int k = 0; k < 4; ++k) a.request(&X.dyT[k], (size_t)widths[k] * ldR_);
        }
      }
      HeadActs& H = head_[q];
      a.request(&H.hlast, R * d_);
      a.request(&H.rowidx, Rm); a.request(&H.labels, Rm);
      a.request(&H.meanf, Rm); a.request(&H.rstdf, Rm);
      act(&H.rows, Rm * d_);
      act(&H.dlogits, Rm * ldV_);
    }
    a.request(&logits_, Rm * ldV_);
    a.request(&scores_, heads * T_ * T_);
    a.request(&dh_buf_, R * d_);
    a.request(&dmid_, R * d_);
    a.request(&tmp32_, R * (size_t)std::max(f_, 3 * d_));
    act(&du_, R * f_);
    act(&dqkv_, R * 3 * d_);
    a.request(&drows_, (size_t)out_split_max_ * Rm * d_);
    a.request(&red_, std::max((size_t)kReduceChunks * std::max(std::max(V_, 3 * d_), f_), (size_t)2 * kLnChunks * d_));
    // room for one node's put-off finish steps (bias and LayerNorm-parameter gradients): the head's
    // column sums, 2 LayerNorms per block + 1, four Linear layers per block
    {
      const size_t ln_chunks = std::min<size_t>(kLnChunks, (size_t)(maxR_ + 3) / 4);
      const size_t nl = blocks_.size();
      fin_.cap = (size_t)kReduceChunks * V_ + (2 * nl + 1) * 2 * ln_chunks * d_ +
                 nl * (size_t)((maxR_ + 63) / 64) * (size_t)(6 * d_ + f_) + 4 * kFinishJobs;
      a.request(&fin_.scratch, fin_.cap);
    }
    if (bf16_) {
      act(&cast_, R * d_);
      const size_t maxdim = (size_t)std::max(std::max(d_, f_), 3 * d_);
      a.request(&tA_, maxdim * ldR_);
      a.request(&tB_, std::max(maxdim * (size_t)ldR_, (size_t)V_ * round8(maxRm_)));
      // contraction slabs of a weight gradient whose tile grid alone would leave most compute
      // units idle (few output tiles, long contraction): one set per stream that takes such products
      wslab_elems_ = 0;
      for (const Lin* L : lins_)
        if (L != &out_)
          wslab_elems_ = std::max(wslab_elems_, (size_t)gemm_bf16_pick_split(L->K, L->N, (int)maxR_) * L->K * L->N);
      if (wslab_elems_) {
        a.request(&wslab_[0], wslab_elems_);
        if (sets_ == 2) a.request(&wslab_[1], wslab_elems_);
      }
      if (sets_ == 2) {   // the deferred weight gradients run beside a backward part: scratch of their own
        a.request(&tA2_, (size_t)(f_ + 3 * d_) * ldR_);   // the four transposed inputs of a block side by side
        a.request(&tB2_, std::max(maxdim * (size_t)ldR_, (size_t)V_ * round8(maxRm_)));
      }
      for (Lin* L : lins_) {
        a.request(&L->wnat, (size_t)L->K * L->ldn);
        a.request(&L->wtr, (size_t)L->N * L->ldt);
      }
    }
  }

  int prepare(Ctx& c, const float* params, hipStream_t st) override {
    if (!bf16_) return VF_OK;
    for (Lin* L : lins_)
      VF_KS(c, st, "cast_weight", launch_cast_weight(params + L->w_off, L->K, L->N, L->wnat, L->ldn, L->wtr,
                                                     L->ldt, st));
    return VF_OK;
  }

  // Two streams and the fused fold: the weight gradients of node i are not taken inside its
  // backward part (the longer of the two parts) but as its side part, which the step enqueues on
  // the forward stream behind the next node's forward part.  The backward part leaves them the
  // transposed output gradients; the layers' inputs are still in the node's tensor set.
  bool side_beside_forward(const Ctx& c) const override { return sets_ == 2 && c.overlap && c.fused; }

  int run_nodes_side(Ctx& c, const StepArgs& s, int i0, int count, hipStream_t st) override {
    for (int i = i0; i < i0 + count; ++i) {
      if (side_beside_forward(c)) VF_TRY(deferred_wgrads(c, s, i, st));
      VF_TRY(c.fold(i, s.w[i], st));   // staged mode only
    }
    return VF_OK;
  }

  int run_node_main(Ctx& c, const StepArgs& s, int i, hipStream_t st) override {
    VF_TRY(run_node_fwd(c, s, i, st));
    return run_node_bwd(c, s, i, st);
  }

  // Forward pass and loss of node i.
  int run_node_fwd(Ctx& c, const StepArgs& s, int i, hipStream_t st) override {
    stream_ = st;
    const int q = std::min(c.aset(i), sets_ - 1);
    HeadActs& H = head_[q];
    const int b = s.sizes[i];
    const int64_t row0 = s.off[i];
    const float w = s.w[i];
    const float* P = s.params;
    const int R = b * T_, Rm = b * m_;
    const int nl = (int)blocks_.size();
    const int heads = b * nh_;
    const int32_t* ids = static_cast<const int32_t*>(s.x) + row0 * T_;
    const int32_t* y = s.y + row0 * 2 * m_;
    const float scale = 1.0f / std::sqrt((float)dh_);

    // ---- forward -----------------------------------------------------------------------
    VF_KS(c, st, "extract_masked", launch_extract_masked(y, b, m_, T_, V_, H.rowidx, H.labels, st));
    VF_KS(c, st, "embed_fwd", launch_embed_fwd(ids, P + tok_off_, P + pos_off_, R, T_, d_, V_, bf16_,
                                          blocks_[0].x[q].hin, st));
    for (int l = 0; l < nl; ++l) {
      Block& B = blocks_[l];
      BlockActs& X = B.x[q];
      float* hnext = l + 1 < nl ? blocks_[l + 1].x[q].hin : H.hlast;
      VF_KS(c, st, "layernorm_fwd", launch_layernorm_fwd(X.hin, d_, nullptr, R, d_, P + B.ln1_g, P + B.ln1_b, bf16_,
                                                    cfg_.ln_eps, X.a, d_, bf16_, X.mean1, X.rstd1, st));
      VF_TRY(lin_fwd(c, "gemm_fwd", B.qkv, P, X.a, d_, R, X.qkv_act, 3 * d_, true, nullptr));
      if (mfma_attn_) {
        VF_KS(c, st, "attn_fwd", launch_attn_fwd(static_cast<const bf16_t*>(X.qkv_act), b, T_, d_, nh_,
                                            static_cast<bf16_t*>(X.prob), static_cast<bf16_t*>(X.om), scale, st));
      } else {
        VF_KS(c, st, "attn_scores", launch_bgemm(qkv_mat(X.qkv_act, 0), qkv_mat(X.qkv_act, 1), score_mat(scores_, 0, false),
                                            T_, T_, dh_, heads, nh_, scale, st));
        VF_KS(c, st, "attn_softmax", launch_softmax_rows(scores_, X.prob, bf16_, (int64_t)heads * T_, T_, st));
        VF_KS(c, st, "attn_pv", launch_bgemm(score_mat(X.prob, 0, bf16_), vt_mat(X.qkv_act), merged_mat(X.om, bf16_),
                                        T_, dh_, T_, heads, nh_, 1.0f, st));
      }
      VF_TRY(lin_fwd(c, "gemm_fwd", B.o, P, X.om, d_, R, X.hmid, d_, false, X.hin));
      VF_KS(c, st, "layernorm_fwd", launch_layernorm_fwd(X.hmid, d_, nullptr, R, d_, P + B.ln2_g, P + B.ln2_b, bf16_,
                                                    cfg_.ln_eps, X.f, d_, bf16_, X.mean2, X.rstd2, st));
      VF_TRY(lin_fwd(c, "gemm_fwd", B.w1, P, X.f, d_, R, X.u, f_, false, nullptr));
      VF_KS(c, st, "gelu_fwd", launch_gelu_fwd(X.u, X.g, bf16_, (int64_t)R * f_, st));
      VF_TRY(lin_fwd(c, "gemm_fwd", B.w2, P, X.g, f_, R, hnext, d_, false, X.hmid));
    }
    VF_KS(c, st, "layernorm_fwd", launch_layernorm_fwd(H.hlast, d_, H.rowidx, Rm, d_, P + lnf_g_, P + lnf_b_, bf16_,
                                                  cfg_.ln_eps, H.rows, d_, bf16_, H.meanf, H.rstdf, st));
    VF_TRY(lin_fwd(c, "gemm_head", out_, P, H.rows, d_, Rm, logits_, ldV_, false, nullptr));
    VF_KS(c, st, "softmax_xent", launch_softmax_xent(logits_, 1, 0, ldV_, logits_, ldV_, H.labels, Rm, V_, c.rowloss,
                                                H.dlogits, ldV_, bf16_, nullptr, 0, w, i, nullptr, nullptr, st));
    // loss bookkeeping per virtual node (Section 5.2), in node order
    for (int j = 0; j < s.group(i); ++j) {
      const int node = s.first[i] + j, rows = s.seg[i] * m_;
      VF_KS(c, st, "loss_reduce", launch_loss_reduce(c.rowloss + (int64_t)j * rows, rows, s.node_w[node], node, c.node_loss,
                                                     c.loss_total, st));
    }

    return VF_OK;
  }

  // Backward pass of node i: every gradient through GradOut, in node order on one stream.
  int run_node_bwd(Ctx& c, const StepArgs& s, int i, hipStream_t st) override {
    stream_ = st;
    const int q = std::min(c.aset(i), sets_ - 1);
    HeadActs& H = head_[q];
    const int b = s.sizes[i];
    const int64_t row0 = s.off[i];
    const float w = s.w[i];
    const float* P = s.params;
    const int R = b * T_, Rm = b * m_;
    const int nl = (int)blocks_.size();
    const int heads = b * nh_;
    const int32_t* ids = static_cast<const int32_t*>(s.x) + row0 * T_;
    const float scale = 1.0f / std::sqrt((float)dh_);
    (void)heads;

    fin_.count = 0; fin_.used = 0;   // nothing is left over from a pass that ended in an error
    // ---- backward: output head -----------------------------------------------------------
    VF_KS(c, st, "colsum", launch_colsum_rows(H.dlogits, ldV_, bf16_, Rm, V_, red_, c.gout(out_.b_off, w, i), st, &fin_));
    const bool defer = side_beside_forward(c);
    sA_ = tA_; sB_ = tB_;
    VF_TRY(lin_bwd_w(c, "gemm_head_wgrad", out_, H.rows, d_, H.dlogits, ldV_, Rm, c.gout(out_.w_off, w, i)));
    int osplit = 1;
    VF_TRY(lin_bwd_x(c, "gemm_head_dgrad", out_, P, H.dlogits, ldV_, Rm, drows_, d_, &osplit));
    const int64_t oslab = (int64_t)Rm * d_;
    VF_KS(c, st, "fill", launch_fill_f32(dh_buf_, 0.f, (int64_t)R * d_, st));
    VF_KS(c, st, "layernorm_bwd", launch_layernorm_bwd(drows_, osplit, oslab, d_, H.hlast, d_, H.rowidx, Rm, d_,
                                                  P + lnf_g_, bf16_, H.meanf, H.rstdf, nullptr, dh_buf_, d_, red_,
                                                  c.gout(lnf_g_, w, i), c.gout(lnf_b_, w, i), st, &fin_));

    // ---- backward: blocks -------------------------------------------------------------------
    for (int l = nl - 1; l >= 0; --l) {
      Block& B = blocks_[l];
      BlockActs& X = B.x[q];
      // FFN
      const void* dh_op = dh_buf_;
      bool dyT = false;
      VF_TRY(prepare_dy(c, dh_buf_, true, d_, R, d_, c.gout(B.w2.b_off, w, i), defer ? X.dyT[0] : nullptr, &dh_op, &dyT));
      if (!(defer && dyT)) VF_TRY(lin_bwd_w(c, "gemm_wgrad", B.w2, X.g, f_, dh_op, d_, R, c.gout(B.w2.w_off, w, i), dyT));
      VF_TRY(lin_bwd_x(c, "gemm_dgrad", B.w2, P, dh_op, d_, R, tmp32_, f_, nullptr));
      VF_KS(c, st, "gelu_bwd", launch_gelu_bwd(tmp32_, X.u, du_, bf16_, (int64_t)R * f_, st));
      const void* du_op = du_;
      VF_TRY(prepare_dy(c, du_, !bf16_, f_, R, f_, c.gout(B.w1.b_off, w, i), defer ? X.dyT[1] : nullptr, &du_op, &dyT));
      if (!(defer && dyT)) VF_TRY(lin_bwd_w(c, "gemm_wgrad", B.w1, X.f, d_, du_, f_, R, c.gout(B.w1.w_off, w, i), dyT));
      VF_TRY(lin_bwd_x(c, "gemm_dgrad", B.w1, P, du_, f_, R, tmp32_, d_, nullptr));
      VF_KS(c, st, "layernorm_bwd", launch_layernorm_bwd(tmp32_, 1, 0, d_, X.hmid, d_, nullptr, R, d_, P + B.ln2_g,
                                                    bf16_, X.mean2, X.rstd2, dh_buf_, dmid_, d_, red_,
                                                    c.gout(B.ln2_g, w, i), c.gout(B.ln2_b, w, i), st, &fin_));
      // attention
      const void* dmid_op = dmid_;
      VF_TRY(prepare_dy(c, dmid_, true, d_, R, d_, c.gout(B.o.b_off, w, i), defer ? X.dyT[2] : nullptr, &dmid_op, &dyT));
      if (!(defer && dyT)) VF_TRY(lin_bwd_w(c, "gemm_wgrad", B.o, X.om, d_, dmid_op, d_, R, c.gout(B.o.w_off, w, i), dyT));
      VF_TRY(lin_bwd_x(c, "gemm_dgrad", B.o, P, dmid_op, d_, R, tmp32_, d_, nullptr));   // d(om), fp32
      // dP = dO V^T ; dV = P^T dO ; dS = P (dP - rowsum(dP P)) ; dQ = dS K / sqrt(dh) ; dK = dS^T Q / sqrt(dh)
      if (mfma_attn_) {
        VF_KS(c, st, "attn_bwd", launch_attn_bwd(tmp32_, static_cast<const bf16_t*>(X.qkv_act),
                                            static_cast<const bf16_t*>(X.prob), b, T_, d_, nh_,
                                            static_cast<bf16_t*>(dqkv_), scale, st));
      } else {
      VF_KS(c, st, "attn_bwd_dp", launch_bgemm(merged_mat(tmp32_, false, true), qkv_mat(X.qkv_act, 2), score_mat(scores_, 0, false),
                                          T_, T_, dh_, heads, nh_, 1.0f, st));
      VF_KS(c, st, "attn_bwd_dv", launch_bgemm(score_mat(X.prob, 1, bf16_), merged_t_mat(tmp32_), qkv_mat(dqkv_, 2),
                                          T_, dh_, T_, heads, nh_, 1.0f, st));
      VF_KS(c, st, "attn_softmax_bwd", launch_softmax_rows_bwd(scores_, X.prob, bf16_, (int64_t)heads * T_, T_, st));
      VF_KS(c, st, "attn_bwd_dq", launch_bgemm(score_mat(scores_, 0, false, true), kt_mat(X.qkv_act, 1), qkv_mat(dqkv_, 0),
                                          T_, dh_, T_, heads, nh_, scale, st));
      VF_KS(c, st, "attn_bwd_dk", launch_bgemm(score_mat(scores_, 1, false, true), kt_mat(X.qkv_act, 0), qkv_mat(dqkv_, 1),
                                          T_, dh_, T_, heads, nh_, scale, st));
      }
      const void* dqkv_op = dqkv_;
      VF_TRY(prepare_dy(c, dqkv_, !bf16_, 3 * d_, R, 3 * d_, c.gout(B.qkv.b_off, w, i), defer ? X.dyT[3] : nullptr, &dqkv_op, &dyT));
      if (!(defer && dyT)) VF_TRY(lin_bwd_w(c, "gemm_wgrad", B.qkv, X.a, d_, dqkv_, 3 * d_, R, c.gout(B.qkv.w_off, w, i), dyT));
      VF_TRY(lin_bwd_x(c, "gemm_dgrad", B.qkv, P, dqkv_, 3 * d_, R, tmp32_, d_, nullptr));
      VF_KS(c, st, "layernorm_bwd", launch_layernorm_bwd(tmp32_, 1, 0, d_, X.hin, d_, nullptr, R, d_, P + B.ln1_g,
                                                    bf16_, X.mean1, X.rstd1, dmid_, dh_buf_, d_, red_,
                                                    c.gout(B.ln1_g, w, i), c.gout(B.ln1_b, w, i), st, &fin_));
    }
    // ---- backward: embeddings ----------------------------------------------------------------
    VF_KS(c, st, "embed_bwd", launch_embed_pos_bwd(dh_buf_, b, T_, d_, c.gout(pos_off_, w, i), st));
    GradOut gt = c.gout(tok_off_, w, i);
    if (!c.fused || i == 0) VF_KS(c, st, "fill", launch_fill_f32(gt.dst, 0.f, (int64_t)V_ * d_, st));
    VF_KS(c, st, "embed_bwd", launch_embed_tok_bwd(ids, dh_buf_, R, d_, V_, gt, st));
    // the put-off finish steps of this node's bias and LayerNorm-parameter gradients, one launch
    VF_KS(c, st, "grad_finish", launch_finish_jobs(fin_, st));
    return VF_OK;
  }

 private:
  // ---- operand views for the batched attention products (batch = sequence * heads + head) ------
  const void* at(const void* p, int64_t elems, bool is16) const {
    return static_cast<const char*>(p) + elems * (is16 ? 2 : 4);
  }
  // [t, e] window of Q (which=0), K (1) or V (2) inside qkv [R, 3d]
  BMat qkv_mat(const void* qkv, int which) const {
    return BMat{at(qkv, (int64_t)which * d_, bf16_), bf16_, (int64_t)T_ * 3 * d_, dh_, 3 * (int64_t)d_, 1};
  }
  // the same window read as [e, t] (rows = feature, contraction = token)
  BMat kt_mat(const void* qkv, int which) const {
    return BMat{at(qkv, (int64_t)which * d_, bf16_), bf16_, (int64_t)T_ * 3 * d_, dh_, 1, 3 * (int64_t)d_};
  }
  BMat vt_mat(const void* qkv) const { return kt_mat(qkv, 2); }
  // [q, j] scores / probabilities; transposed = 1 reads them as [j, q]
  BMat score_mat(const void* p, int transposed, bool is16, bool round_operand = false) const {
    const int64_t TT = (int64_t)T_ * T_;
    return BMat{p, is16, nh_ * TT, TT, transposed ? 1 : (int64_t)T_, transposed ? (int64_t)T_ : 1,
                round_operand && bf16_};
  }
  // [t, e] window of one head inside a [R, d] tensor
  BMat merged_mat(const void* p, bool is16, bool round_operand = false) const {
    return BMat{p, is16, (int64_t)T_ * d_, dh_, d_, 1, round_operand && bf16_};
  }
  // fp32 [R, d] tensor read as [e, t]; values enter the product as bf16 in bf16 workloads
  BMat merged_t_mat(const void* p) const { return BMat{p, 0, (int64_t)T_ * d_, dh_, 1, d_, bf16_}; }

  // out[R, N] = in[R, K] W + bias (+ residual); out is T (out_act) or fp32
  int lin_fwd(Ctx& c, const char* tag, const Lin& L, const float* P, const void* in, int64_t ldin, int R,
              void* out, int64_t ldo, bool out_act, const float* residual) {
    Epilogue ep;
    ep.C = out; ep.ldc = ldo;
    ep.c_is_bf16 = out_act && bf16_;
    ep.bias = P + L.b_off; ep.bias_round_bf16 = bf16_;
    if (residual) { ep.R = residual; ep.ldr = ldo; ep.beta = 1.f; }
    if (bf16_)
      VF_KS(c, stream_, tag, launch_gemm_bf16(static_cast<const bf16_t*>(in), ldin, L.wtr, L.ldt, R, L.N, L.K, 1, 0, ep,
                                    stream_));
    else
      VF_KS(c, stream_, tag, launch_gemm_f32(static_cast<const float*>(in), ldin, 1, P + L.w_off, 1, L.N, R, L.N, L.K, 1, 0, ep,
                                   stream_));
    return VF_OK;
  }

  // The gradient dy [R, C] at a Linear layer's output (fp32, or the workload's type), readied for
  // that layer's backward pass: the bias gradient through gb, *op = what the products read as dy
  // (a bf16 copy of an fp32 dy in bf16 workloads), *transposed = whether tB_ already holds dy^T
  // (or `keep`, if given) for the weight gradient.  bf16 workloads whose shapes qualify get all of
  // it from one pass.
  int prepare_dy(Ctx& c, const void* dy, bool dy_is_f32, int64_t lddy, int R, int C, GradOut gb,
                 bf16_t* keep, const void** op, bool* transposed) {
    hipStream_t st = stream_;
    const int64_t ldr = round8(R);
    *op = dy;
    *transposed = false;
    if (bf16_ && dy_prepare_fits(dy_is_f32, lddy, lddy, ldr, R, C)) {
      // `keep`: where the transposed copy goes when the weight gradient is taken later
      VF_KS(c, stream_, "dy_prepare", launch_dy_prepare(dy, dy_is_f32, lddy, R, C, static_cast<bf16_t*>(cast_), lddy,
                                              keep ? keep : sB_, ldr, red_, gb, st, &fin_));
      if (dy_is_f32) *op = cast_;
      *transposed = true;
      return VF_OK;
    }
    if (bf16_ && dy_is_f32) {
      VF_KS(c, stream_, "cast", launch_cast_bf16(static_cast<const float*>(dy), lddy, static_cast<bf16_t*>(cast_), lddy, R, C, st));
      *op = cast_;
    }
    VF_KS(c, stream_, "colsum", launch_colsum_rows(dy, lddy, dy_is_f32 ? 0 : bf16_, R, C, red_, gb, st, &fin_));
    return VF_OK;
  }

  // dW[K, N] = in^T dy through GradOut.  dy_transposed: dy^T is already there, in `dyT` if given,
  // else in the scratch sB_; inT: in^T is already there (row pitch R rounded up to 8).
  int lin_bwd_w(Ctx& c, const char* tag, const Lin& L, const void* in, int64_t ldin, const void* dy,
                int64_t lddy, int R, GradOut go, bool dy_transposed = false, const bf16_t* dyT = nullptr,
                const bf16_t* inT = nullptr) {
    Epilogue ep;
    ep.C = go.dst; ep.ldc = L.N; ep.alpha = go.alpha;
    if (go.accumulate) { ep.R = go.dst; ep.ldr = L.N; ep.beta = 1.f; }
    if (bf16_) {
      const int64_t ldr = round8(R);
      if (!inT)
        VF_KS(c, stream_, "transpose", launch_transpose_bf16(static_cast<const bf16_t*>(in), ldin, sA_, ldr, R, L.K, stream_));
      if (!dy_transposed)
        VF_KS(c, stream_, "transpose", launch_transpose_bf16(static_cast<const bf16_t*>(dy), lddy, sB_, ldr, R, L.N, stream_));
      const bf16_t* At = inT ? inT : sA_;
      const bf16_t* Bt = dy_transposed && dyT ? dyT : sB_;
      float* slabs = wslab_[sA_ == tA2_ && tA2_ ? 1 : 0];
      const int64_t each = (int64_t)L.K * L.N;
      int ns = (slabs && &L != &out_) ? gemm_bf16_pick_split(L.K, L.N, R) : 1;
      while (ns > 1 && (size_t)ns * each > wslab_elems_) ns /= 2;
      if (ns > 1) {
        // slices of the contraction into slabs, added in slab order into the gradient
        Epilogue es;
        es.C = slabs; es.ldc = L.N;
        VF_KS(c, stream_, tag, launch_gemm_bf16(At, ldr, Bt, ldr, L.K, L.N, R, ns, each, es, stream_));
        VF_KS(c, stream_, "fold_slabs", launch_fold_slabs(slabs, ns, each, each, go, stream_));
      } else {
        VF_KS(c, stream_, tag, launch_gemm_bf16(At, ldr, Bt, ldr, L.K, L.N, R, 1, 0, ep, stream_));
      }
    } else {
      VF_KS(c, stream_, tag, launch_gemm_f32(static_cast<const float*>(in), 1, ldin, static_cast<const float*>(dy), 1, lddy,
                                   L.K, L.N, R, 1, 0, ep, stream_));
    }
    return VF_OK;
  }

  // The blocks' weight gradients that node i's backward part left out (see side_beside_forward),
  // in the order the backward part would have taken them.
  int deferred_wgrads(Ctx& c, const StepArgs& s, int i, hipStream_t st) {
    stream_ = st;
    sA_ = tA2_; sB_ = tB2_;
    const int q = std::min(c.aset(i), sets_ - 1);
    const float w = s.w[i];
    const int R = s.sizes[i] * T_;
    const int64_t ldr = round8(R);
    for (int l = (int)blocks_.size() - 1; l >= 0; --l) {
      Block& B = blocks_[l];
      BlockActs& X = B.x[q];
      const Lin* lins[4] = {&B.w2, &B.w1, &B.o, &B.qkv};
      const void* ins[4] = {X.g, X.f, X.om, X.a};
      const int64_t ldins[4] = {f_, d_, d_, d_};
      const bool f32dy[4] = {true, false, true, false};
      // the backward part took a gradient itself when its shapes did not qualify for the one-pass preparation
      bool mine[4];
      bool all = true;
      for (int k = 0; k < 4; ++k) {
        mine[k] = dy_prepare_fits(f32dy[k], lins[k]->N, lins[k]->N, ldr, R, lins[k]->N);
        all = all && mine[k];
      }
      // all four: their inputs are transposed by one launch, side by side in the scratch
      const bf16_t* inT[4] = {nullptr, nullptr, nullptr, nullptr};
      if (all) {
        TransposeJobs tj{};
        size_t off = 0;
        for (int k = 0; k < 4; ++k) {
          tj.in[k] = static_cast<const bf16_t*>(ins[k]); tj.ldi[k] = ldins[k];
          tj.out[k] = tA2_ + off; tj.C[k] = lins[k]->K;
          off += (size_t)lins[k]->K * ldr;
          inT[k] = tj.out[k];
        }
        tj.count = 4; tj.R = R; tj.ldo = ldr;
        VF_KS(c, st, "transpose", launch_transpose_bf16_jobs(tj, st));
      }
      for (int k = 0; k < 4; ++k) {
        const Lin& L = *lins[k];
        if (!mine[k]) continue;
        VF_TRY(lin_bwd_w(c, "gemm_wgrad", L, ins[k], ldins[k], nullptr, 0, R, c.gout(L.w_off, w, i), true, X.dyT[k], inT[k]));
      }
    }
    return VF_OK;
  }

  // dx[R, K] (fp32) = dy W^T.  With `split` the product may arrive as partial slabs.
  int lin_bwd_x(Ctx& c, const char* tag, const Lin& L, const float* P, const void* dy, int64_t lddy, int R,
                float* dx, int64_t lddx, int* split) {
    Epilogue ep;
    ep.C = dx; ep.ldc = lddx;
    int ns = 1;
    if (bf16_) {
      if (split) {
        ns = std::min(gemm_bf16_pick_split(R, L.K, L.N), out_split_max_);
        *split = ns;
      }
      VF_KS(c, stream_, tag, launch_gemm_bf16(static_cast<const bf16_t*>(dy), lddy, L.wnat, L.ldn, R, L.K, L.N, ns,
                                    (int64_t)R * lddx, ep, stream_));
    } else {
      if (split) *split = 1;
      VF_KS(c, stream_, tag, launch_gemm_f32(static_cast<const float*>(dy), lddy, 1, P + L.w_off, L.N, 1, R, L.K, L.N, 1, 0, ep,
                                   stream_));
    }
    return VF_OK;
  }

  vf_config cfg_;
  hipStream_t stream_ = nullptr;        // stream of the part being enqueued
  bool bf16_ = false;
  int d_ = 0, f_ = 0, T_ = 0, V_ = 0, m_ = 0, nh_ = 0, dh_ = 0;
  int64_t P_ = 0, tok_off_ = 0, pos_off_ = 0, lnf_g_ = 0, lnf_b_ = 0;
  int max_seqs_ = 0;               // sequences of the largest unit of the passes
  int64_t maxR_ = 0, maxRm_ = 0, ldR_ = 0, ldV_ = 0;
  int out_split_max_ = 32;
  bool mfma_attn_ = false;              // fused matrix-core attention kernels apply
  std::vector<Block> blocks_;
  std::vector<Lin*> lins_;
  Lin out_;
  HeadActs head_[2];
  int sets_ = 1;
  float* logits_ = nullptr;
  float* scores_ = nullptr;
  float *dh_buf_ = nullptr, *dmid_ = nullptr, *tmp32_ = nullptr;
  void *du_ = nullptr, *dqkv_ = nullptr, *cast_ = nullptr;
  float* drows_ = nullptr;
  float* red_ = nullptr;                // scratch of the row-chunked reductions
  FinishList fin_;                      // their finish steps of one node's backward pass, run as one launch
  bf16_t *tA_ = nullptr, *tB_ = nullptr;
  bf16_t *tA2_ = nullptr, *tB2_ = nullptr;   // the same scratch for weight gradients taken beside a backward part
  float* wslab_[2] = {nullptr, nullptr};     // contraction slabs of weight gradients ([1]: those taken beside a backward part)
  size_t wslab_elems_ = 0;
  bf16_t *sA_ = nullptr, *sB_ = nullptr;     // the scratch pair of the part being enqueued
};

}  // namespace

std::unique_ptr<Model> make_encoder(const vf_config& cfg) { return std::unique_ptr<Model>(new Encoder(cfg)); }

}  // namespace vf
