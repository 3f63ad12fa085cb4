// The library context: configuration, parameter layout, device buffers, per-model runners.
#pragma once

#include <algorithm>
#include <cstdlib>
#include <memory>
#include <string>
#include <vector>

#include "vf_internal.h"

namespace vf {

// Collects buffer requests, then carves them out of one device allocation.
class Arena {
 public:
  template <typename T>
  void request(T** target, size_t count) {
    size_t bytes = (count * sizeof(T) + 255) & ~size_t(255);
    reqs_.push_back({reinterpret_cast<void**>(target), total_, count * sizeof(T)});
    total_ += bytes + guard();
  }
  size_t total() const { return total_; }
  void assign(char* base) {
    for (auto& r : reqs_) *r.target = base + r.offset;
  }
  // Debugging aid: VF_ARENA_GUARD=<bytes> (a multiple of 256) leaves that much room after every
  // buffer; vf_init then fills the whole arena with the byte 0x7f (huge values in every
  // floating-point type) and zeroes exactly the bytes each buffer asked for, so that a read past
  // a buffer's end shows in the results.
  static size_t guard() {
    static const size_t g = std::getenv("VF_ARENA_GUARD") ? (size_t)std::atoll(std::getenv("VF_ARENA_GUARD")) & ~size_t(255) : 0;
    return g;
  }
  template <typename F>
  void for_each_buffer(F f) const {
    for (const auto& r : reqs_) f(r.offset, r.bytes);
  }

 private:
  struct Req { void** target; size_t offset; size_t bytes; };
  std::vector<Req> reqs_;
  size_t total_ = 0;
};

// What the passes of a step iterate over.  V, sizes, off, w describe the UNITS that go through the
// passes one after another: the virtual nodes themselves, or -- with node_group > 1 -- groups of
// consecutive nodes taken together (sizes[i] rows = the rows of its count[i] nodes; w[i] =
// sizes[i] / B, the sum of its nodes' weights, so a unit's loss is the mean over all its rows).
// What stays per node reads the node lists: first[i] is the unit's first node, its nodes are
// node_sizes[first[i]] .. node_sizes[first[i] + count[i] - 1] (BatchNorm statistics, losses).
struct StepArgs {
  float* params;
  const void* x;
  const int32_t* y;
  int32_t B, V;
  std::vector<int32_t> sizes, off;
  std::vector<float> w;
  std::vector<int32_t> seg;               // rows of unit i's first node (== sizes[i] without groups)
  std::vector<int32_t> first;             // index of unit i's first node
  std::vector<int32_t> count;             // nodes in unit i
  int32_t nodes;                          // the virtual nodes of the step ...
  std::vector<int32_t> node_sizes, node_off;
  std::vector<float> node_w;              // ... with their offsets and weights b_i/B
  int group(int i) const { return count[i]; }
  const int32_t* rows_of(int i) const { return node_sizes.data() + first[i]; }
};

struct Ctx;

// A stretch of the flat parameter vector whose gradient is complete before the rest is.
struct UpdateRange { int64_t off = 0, n = 0; };

// A model = parameter layout + buffers + the launch sequence of one virtual node.
class Model {
 public:
  virtual ~Model() {}
  virtual int64_t num_params() const = 0;
  virtual void request_buffers(Arena& a) = 0;
  // Refresh whatever the passes read instead of the fp32 master (bf16 weight copies).
  virtual int prepare(Ctx& c, const float* params, hipStream_t st) = 0;
  // Node `i` (rows off..off+b), each part a plain sequence of launches on ONE stream:
  //   forward part:  forward pass and loss bookkeeping (it also leaves the transposed operands of
  //                  the weight gradients it produces in copy c.slot(i));
  //   backward part: the input-gradient chain with the small-vector gradients (BatchNorm scale and
  //                  shift, hidden biases) folded into the gradient buffer on the way;
  //   side part:     what only the gradient buffer waits for -- weight gradients and, in staged
  //                  mode, the fold c.fold(i, ...) -- for `count` consecutive nodes i0 .. i0+count-1
  //                  (the fold window): a model may fold their weight gradients in one pass.
  // One stream: fwd(i), bwd(i) for the nodes of a window, then side(window).  Two streams
  // (overlap): the forward parts run on the caller's stream, the backward and side parts on the
  // library's second stream, so that fwd(i+1) runs beside bwd(i); every chain whose order matters
  // (moving statistics and loss in the forward parts, small-vector gradients in the backward
  // parts) stays on one stream in node order.  A model that supports this keeps the tensors that
  // pass from a node's forward to its backward part in two sets, c.aset(i).
  // run_node_main = forward part + backward part on one stream.
  virtual int run_node_main(Ctx& c, const StepArgs& a, int i, hipStream_t st) = 0;
  virtual int run_node_fwd(Ctx& c, const StepArgs& a, int i, hipStream_t st) { return run_node_main(c, a, i, st); }
  virtual int run_node_bwd(Ctx&, const StepArgs&, int, hipStream_t) { return VF_OK; }
  virtual int run_nodes_side(Ctx& c, const StepArgs& a, int i0, int count, hipStream_t st) = 0;
  // Two streams, launches made one by one: the same preparation with only what the first
  // launch of node 0's forward part needs on `first`, the rest on `second` (the model then
  // makes node 0's forward part wait for each piece where it first reads it).
  virtual int prepare_split(Ctx& c, const float* params, hipStream_t first, hipStream_t second) {
    (void)second;
    return prepare(c, params, first);
  }
  virtual bool supports_overlap() const { return false; }
  // Two streams: whether the side part of node i goes onto the forward stream, behind the forward
  // part of node i+1 (and after waiting for backward part i), instead of following backward part
  // i on the second stream.  For models whose backward part is the longer one.  Window 1 only.
  virtual bool side_beside_forward(const Ctx&) const { return false; }
  // Stretches of the parameter vector (16-byte aligned starts, together all of it) in the order
  // in which the last side part of a step completes their gradients; the model calls
  // Ctx::mark_range(k) at that point.  Empty: the gradient is complete when the side part ends.
  virtual void update_ranges(std::vector<UpdateRange>* out) const { out->clear(); }
  // Largest fold window the side part can take (it must keep that many nodes' operands).
  virtual int max_window() const { return 1; }
  // How many nodes of `rows` rows the passes take as one unit at most (1: none) ...
  virtual int max_group(int rows) const { (void)rows; return 1; }
  // ... and whether the nodes of a unit may differ in size.
  virtual bool groups_unequal() const { return false; }
  // State that the passes themselves carry from step to step on this device (BatchNorm moving
  // mean and variance, Section 4.1): `state_floats` fp32 values at `state_ptr`, laid out as all
  // layers' means then all layers' variances; init_state sets the starting values.
  virtual int64_t state_floats() const { return 0; }
  virtual float* state_ptr() const { return nullptr; }
  virtual int init_state(hipStream_t) { return VF_OK; }
};

// Optional per-kernel timing: while enabled, every launch made through VF_K is bracketed by
// two events on the context's stream and kernels are launched one by one (no graph replay).
struct Profiler {
  struct Rec { const char* tag; hipEvent_t a, b; };
  bool enabled = false;
  std::vector<Rec> recs;
  std::vector<hipEvent_t> pool;
  size_t used = 0;
  int take(hipEvent_t* e) {
    if (used == pool.size()) {
      hipEvent_t ev;
      VF_HIP(hipEventCreate(&ev));
      pool.push_back(ev);
    }
    *e = pool[used++];
    return VF_OK;
  }
};

struct Ctx {
  vf_config cfg;
  Profiler prof;
  hipStream_t stream = nullptr;
  int device = 0;
  bool bf16 = false;
  bool fused = false;
  int64_t P = 0;
  std::unique_ptr<Model> model;

  char* arena = nullptr;
  size_t arena_bytes = 0;
  float* gbuf = nullptr;      // combined gradient G (the shared gradient buffer)
  float* gstage = nullptr;    // one node's gradient g_i (unused when fused)
  float* opt0 = nullptr;      // v (SGD-momentum) or m (Adam)
  float* opt1 = nullptr;      // u (Adam)
  float* rowloss = nullptr;   // per-row losses of the node in flight
  float* node_loss = nullptr; // [max_nodes]
  float* loss_total = nullptr;

  int64_t steps = 0;
  int32_t last_V = 0;

  // Second stream (library-owned, default priority): with overlap the backward parts and the
  // weight gradients run there while the caller's stream goes on with the next node's forward.
  hipStream_t side = nullptr;
  bool overlap = false;
  hipEvent_t fwd_done[2] = {nullptr, nullptr};   // forward part of the node using set q is complete
  hipEvent_t bwd_done[2] = {nullptr, nullptr};   // backward part of the node using set q is complete
  hipEvent_t side_done[2] = {nullptr, nullptr};  // side part of window w (parity) is complete
  hipEvent_t prep_done = nullptr;                // weight preparation

  int group = 1;                          // consecutive equal-sized nodes taken through their passes together
  int window = 1;                         // nodes whose weight gradients are folded in one pass
  // copies of the side part's operands: one window's worth, and two with overlap at window 1
  int copies() const { return overlap ? std::max(2, window) : window; }
  int slot(int node) const { return node % copies(); }
  int aset(int node) const { return overlap ? (node & 1) : 0; }           // forward -> backward tensor set

  bool overlapping() const { return overlap; }
  float* stage_for(int) const { return gstage; }

  // Graph replay: one captured launch sequence per part (weight preparation, main(i), side(i)),
  // each a single-stream chain, so replay keeps the two streams apart exactly as eager
  // launches do.
  // Two captured sets are kept (a caller that alternates between two input buffers, as the
  // prefetching entry points do, replays instead of recapturing); `cur` is the one in use.
  struct GraphSet {
    std::vector<hipGraphExec_t> graphs;     // one graph, or [0] prepare, [1+2i] fwd(i), [2+2i] bwd(i), [1+2V+w] side(w)
    std::vector<int32_t> sizes, node_sizes;
    const void* params = nullptr;
    const void* x = nullptr;
    const void* y = nullptr;
  };
  GraphSet gsets[2];
  int cur = 0;
  GraphSet& gs() { return gsets[cur]; }
  const GraphSet& gs() const { return gsets[cur]; }

  // Input prefetch (Section 3.2 step 1: the next batch is fetched while this one is processed):
  // a copy stream and two pairs of device staging buffers, created on first use.
  struct Prefetch {
    hipStream_t stream = nullptr;
    void* x[2] = {nullptr, nullptr};
    void* y[2] = {nullptr, nullptr};
    hipEvent_t copied[2] = {nullptr, nullptr};     // the copy into pair k is complete
    hipEvent_t consumed[2] = {nullptr, nullptr};   // the step that read pair k is complete
    bool used[2] = {false, false};
    int next = 0;                                  // the pair the next prefetch fills / next step reads
    bool pending = false;                          // a batch is staged and not yet consumed
    int32_t pending_B = 0;
  } pf;

  // Destination of node i's gradient entry at flat offset `off`.
  GradOut gout(int64_t off, float w, int node) const {
    if (fused) return GradOut{gbuf + off, w, node > 0 ? 1 : 0};
    return GradOut{stage_for(node) + off, 1.0f, 0};
  }
  // Staged mode: fold node i's staging vector into the gradient buffer on stream `st`
  // (Section 3.2 step 3 with the weight of Section 5.2).  No-op in fused mode.
  int fold(int node, float w, hipStream_t st);

  // Two streams, launches made one by one: the update of a stretch of the parameters
  // (Section 3.2 step 5 is elementwise) starts on the first stream as soon as the second
  // stream has completed that stretch's gradient, beside the weight gradients still to come.
  std::vector<UpdateRange> ranges;
  std::vector<hipEvent_t> range_done;
  bool marking = false;          // this step's side part records range_done
  hipEvent_t last_side = nullptr;   // the event that ends the second stream's work of this step
  int mark_range(int k, hipStream_t st);
};

// Debugging aid: with VF_SYNC_EACH set in the environment the host waits after every launch
// (VF_SYNC_EACH=all), or after the launches whose tag the variable names (comma separated).
inline bool debug_sync_each(const char* tag) {
  static const char* spec = std::getenv("VF_SYNC_EACH");
  if (!spec) return false;
  const std::string s(spec);
  if (s == "all") return true;
  return ("," + s + ",").find("," + std::string(tag) + ",") != std::string::npos;
}

// Launch `call` (an expression returning a status) under the tag `name`; the launch goes to
// stream `strm` (VF_K: the context's main stream).
#define VF_K(ctx, name, call) VF_KS(ctx, (ctx).stream, name, call)
#define VF_KS(ctx, strm, name, call)                                             \
  do {                                                                    \
    if ((ctx).prof.enabled) {                                             \
      ::vf::Profiler::Rec r__{name, nullptr, nullptr};                    \
      VF_TRY((ctx).prof.take(&r__.a));                                    \
      VF_TRY((ctx).prof.take(&r__.b));                                    \
      VF_HIP(hipEventRecord(r__.a, (strm)));                              \
      VF_TRY(call);                                                       \
      VF_HIP(hipEventRecord(r__.b, (strm)));                              \
      (ctx).prof.recs.push_back(r__);                                     \
    } else {                                                              \
      VF_TRY(call);                                                       \
      if (::vf::debug_sync_each(name)) VF_HIP(hipStreamSynchronize((strm))); \
    }                                                                     \
  } while (0)

std::unique_ptr<Model> make_mlp(const vf_config& cfg);
std::unique_ptr<Model> make_encoder(const vf_config& cfg);
std::unique_ptr<Model> make_conv(const vf_config& cfg);

}  // namespace vf

struct vf_ctx {
  vf::Ctx c;
};
