// C ABI of libvf: argument checks, partition (S0), context set-up, and the step executor
// that strings the per-node launch sequences, the accumulate kernel and the optimizer
// update together (Section 3.2, steps 1-5; weights of Section 5.2).
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>

#include "vf_ctx.h"

namespace vf {

static thread_local std::string g_last_error;

void set_last_error(const char* what, hipError_t e, const char* file, int line) {
  char buf[512];
  snprintf(buf, sizeof buf, "%s failed: %s (%s:%d)", what, hipGetErrorString(e), file, line);
  g_last_error = buf;
}
void set_last_error_text(const std::string& s) { g_last_error = s; }

namespace {

int check_partition(const int32_t* sizes, int32_t V, int32_t B) {
  if (!sizes || V < 1 || B < 1) return VF_EINVAL;
  int64_t sum = 0;
  for (int32_t i = 0; i < V; ++i) {
    if (sizes[i] < 1) return VF_EINVAL;
    sum += sizes[i];
  }
  return sum == (int64_t)B ? VF_OK : VF_EINVAL;
}

int validate_config(const vf_config& c) {
  if (c.dtype != VF_F32 && c.dtype != VF_BF16) return VF_EINVAL;
  if (c.optimizer != VF_SGDM && c.optimizer != VF_ADAM) return VF_EINVAL;
  if (c.max_batch < 1 || c.max_node_size < 1 || c.max_nodes < 1) return VF_EINVAL;
  if (c.max_node_size > c.max_batch) return VF_EINVAL;
  if (!(c.bn_momentum >= 0.f && c.bn_momentum <= 1.f)) return VF_EINVAL;
  if (c.fold_window < 0 || c.fold_window > kFoldMax) return VF_EINVAL;
  if (c.node_group != 0 && c.node_group != 1 && c.node_group != 2 && c.node_group != 4 && c.node_group != 8 &&
      c.node_group != 16 && c.node_group != 32)
    return VF_EINVAL;
  if (c.model_kind == VF_MLP) {
    if (c.n_dims < 2 || c.n_dims > VF_MAX_DIMS) return VF_EINVAL;
    for (int i = 0; i < c.n_dims; ++i)
      if (c.dims[i] < 1) return VF_EINVAL;
    // bf16 rows of the batch are read with 16-byte loads
    if (c.dtype == VF_BF16 && (c.dims[0] % 8) != 0) return VF_EINVAL;
    return VF_OK;
  }
  if (c.model_kind == VF_ENCODER) {
    if (c.n_layers < 1 || c.d_model < 1 || c.n_heads < 1 || c.d_ffn < 1 || c.seq_len < 1 ||
        c.vocab < 1 || c.n_masked < 1)
      return VF_EINVAL;
    if (c.d_model % c.n_heads) return VF_EINVAL;
    if (c.d_model > 1024) return VF_EINVAL;                       // LayerNorm kernels keep a row in registers
    if ((int64_t)c.max_node_size * std::min(4, std::max(1, c.node_group)) * c.seq_len > 65536) return VF_EINVAL;   // token bitmap of the embedding backward
    if (c.n_masked > c.seq_len) return VF_EINVAL;
    if (c.dtype == VF_BF16 && ((c.d_model % 8) || (c.d_ffn % 8) || ((c.d_model / c.n_heads) % 8)))
      return VF_EINVAL;
    return VF_OK;
  }
  if (c.model_kind == VF_CONV) {
    if (c.dtype != VF_BF16) return VF_EINVAL;
    if (c.img < 1 || c.img > 1024 || c.in_ch < 1 || c.n_blocks < 0 || c.n_blocks > 64 || c.classes < 1) return VF_EINVAL;
    if (c.width < 8 || c.width > 256 || (c.width % 8)) return VF_EINVAL;
    return VF_OK;
  }
  return VF_EINVAL;
}

bool set_matches(const Ctx::GraphSet& g, const StepArgs& a) {
  return !g.graphs.empty() && g.params == a.params && g.x == a.x && g.y == a.y && g.sizes == a.sizes &&
         g.node_sizes == a.node_sizes;
}

// Selects the captured set that fits this call, if there is one.
bool graph_matches(Ctx& c, const StepArgs& a) {
  if (set_matches(c.gs(), a)) return true;
  if (set_matches(c.gsets[c.cur ^ 1], a)) { c.cur ^= 1; return true; }
  if (!c.gs().graphs.empty()) c.cur ^= 1;      // capture into the older set, keep the latest one
  return false;
}

void release_streams(Ctx& c) {
  hipEvent_t* evs[] = {&c.fwd_done[0], &c.fwd_done[1], &c.bwd_done[0], &c.bwd_done[1],
                       &c.side_done[0], &c.side_done[1], &c.prep_done};
  for (hipEvent_t* e : evs)
    if (*e) { (void)hipEventDestroy(*e); *e = nullptr; }
  for (hipEvent_t e : c.range_done)
    if (e) (void)hipEventDestroy(e);
  c.range_done.clear();
  if (c.side) { (void)hipStreamDestroy(c.side); c.side = nullptr; }
}

void release_prefetch(Ctx& c) {
  Ctx::Prefetch& p = c.pf;
  for (int k = 0; k < 2; ++k) {
    if (p.copied[k]) (void)hipEventDestroy(p.copied[k]);
    if (p.consumed[k]) (void)hipEventDestroy(p.consumed[k]);
    if (p.x[k]) (void)hipFree(p.x[k]);
    if (p.y[k]) (void)hipFree(p.y[k]);
    p.copied[k] = p.consumed[k] = nullptr;
    p.x[k] = nullptr; p.y[k] = nullptr;
  }
  if (p.stream) (void)hipStreamDestroy(p.stream);
  p.stream = nullptr;
}

// Bytes of one batch of B samples as vf_step reads it.
size_t batch_x_bytes(const vf_config& f, int64_t B) {
  if (f.model_kind == VF_MLP) return (size_t)B * f.dims[0] * (f.dtype == VF_BF16 ? 2 : 4);
  if (f.model_kind == VF_CONV) return (size_t)B * f.img * f.img * f.in_ch * 2;
  return (size_t)B * f.seq_len * sizeof(int32_t);
}
size_t batch_y_bytes(const vf_config& f, int64_t B) {
  if (f.model_kind != VF_ENCODER) return (size_t)B * sizeof(int32_t);
  return (size_t)B * 2 * f.n_masked * sizeof(int32_t);
}

// First use: the copy stream (default priority), two pairs of device staging buffers sized for
// max_batch, and the events that order copies against the steps that read them.
int init_prefetch(Ctx& c) {
  Ctx::Prefetch& p = c.pf;
  if (p.stream) return VF_OK;
  hipError_t e = hipStreamCreateWithFlags(&p.stream, hipStreamNonBlocking);
  for (int k = 0; k < 2 && e == hipSuccess; ++k) {
    e = hipEventCreateWithFlags(&p.copied[k], hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&p.consumed[k], hipEventDisableTiming);
    if (e == hipSuccess) e = hipMalloc(&p.x[k], batch_x_bytes(c.cfg, c.cfg.max_batch));
    if (e == hipSuccess) e = hipMalloc(&p.y[k], batch_y_bytes(c.cfg, c.cfg.max_batch));
  }
  if (e != hipSuccess) {
    set_last_error("prefetch set-up", e, __FILE__, __LINE__);
    (void)hipGetLastError();
    release_prefetch(c);
    return e == hipErrorOutOfMemory ? VF_ENOMEM : VF_EDEVICE;
  }
  return VF_OK;
}

void drop_graph(Ctx& c) {
  for (hipGraphExec_t g : c.gs().graphs)
    if (g) (void)hipGraphExecDestroy(g);
  c.gs().graphs.clear();
}

// The kinds of launch sequence of a step; `part` 0 = weight preparation, 1 = fwd(i), 2 = bwd(i),
// 3 = side(window i).  Each runs on one stream.
int enqueue_part(Ctx& c, const StepArgs& a, int part, int idx, hipStream_t st) {
  if (part == 0) return c.model->prepare(c, a.params, st);
  if (part == 1) return c.model->run_node_fwd(c, a, idx, st);
  if (part == 2) return c.model->run_node_bwd(c, a, idx, st);
  const int i0 = idx * c.window;
  return c.model->run_nodes_side(c, a, i0, std::min(c.window, a.V - i0), st);
}

// Record one part into a graph (captured on the main stream; replayed on whichever stream).
int capture_part(Ctx& c, const StepArgs& a, int part, int node, hipGraphExec_t* out) {
  hipGraph_t graph = nullptr;
  VF_HIP(hipStreamBeginCapture(c.stream, hipStreamCaptureModeThreadLocal));
  int rc = enqueue_part(c, a, part, node, c.stream);
  hipError_t e = hipStreamEndCapture(c.stream, &graph);
  if (rc != VF_OK) {
    if (graph) (void)hipGraphDestroy(graph);
    return rc;
  }
  if (e != hipSuccess) {
    set_last_error("hipStreamEndCapture", e, __FILE__, __LINE__);
    return VF_EDEVICE;
  }
  e = hipGraphInstantiate(out, graph, nullptr, nullptr, 0);
  (void)hipGraphDestroy(graph);
  if (e != hipSuccess) {
    *out = nullptr;
    set_last_error("hipGraphInstantiate", e, __FILE__, __LINE__);
    return VF_EDEVICE;
  }
  return VF_OK;
}

int enqueue_nodes(Ctx& c, const StepArgs& a, bool use_graph);

// Without overlap the whole step (minus the update) is one single-stream chain: one graph.
int capture_whole_step(Ctx& c, const StepArgs& a) {
  drop_graph(c);
  c.gs().graphs.assign(1, nullptr);
  hipGraph_t graph = nullptr;
  VF_HIP(hipStreamBeginCapture(c.stream, hipStreamCaptureModeThreadLocal));
  int rc = enqueue_nodes(c, a, false);
  hipError_t e = hipStreamEndCapture(c.stream, &graph);
  if (rc == VF_OK && e != hipSuccess) {
    set_last_error("hipStreamEndCapture", e, __FILE__, __LINE__);
    rc = VF_EDEVICE;
  }
  if (rc == VF_OK) {
    e = hipGraphInstantiate(&c.gs().graphs[0], graph, nullptr, nullptr, 0);
    if (e != hipSuccess) {
      set_last_error("hipGraphInstantiate", e, __FILE__, __LINE__);
      rc = VF_EDEVICE;
    }
  }
  if (graph) (void)hipGraphDestroy(graph);
  if (rc != VF_OK) {
    c.gs().graphs.clear();
    return rc;
  }
  c.gs().params = a.params; c.gs().x = a.x; c.gs().y = a.y; c.gs().sizes = a.sizes; c.gs().node_sizes = a.node_sizes;
  return VF_OK;
}

int capture_graphs(Ctx& c, const StepArgs& a) {
  if (!c.overlapping()) return capture_whole_step(c, a);
  drop_graph(c);
  const int nwin = (a.V + c.window - 1) / c.window;
  c.gs().graphs.assign((size_t)1 + 2 * a.V + nwin, nullptr);
  int rc = capture_part(c, a, 0, 0, &c.gs().graphs[0]);
  for (int i = 0; i < a.V && rc == VF_OK; ++i) {
    rc = capture_part(c, a, 1, i, &c.gs().graphs[1 + 2 * i]);
    if (rc == VF_OK) rc = capture_part(c, a, 2, i, &c.gs().graphs[2 + 2 * i]);
  }
  for (int w = 0; w < nwin && rc == VF_OK; ++w) rc = capture_part(c, a, 3, w, &c.gs().graphs[1 + 2 * a.V + w]);
  if (rc != VF_OK) {
    drop_graph(c);
    return rc;
  }
  c.gs().params = a.params; c.gs().x = a.x; c.gs().y = a.y; c.gs().sizes = a.sizes; c.gs().node_sizes = a.node_sizes;
  return VF_OK;
}

// Run one part: replay its graph, or launch its kernels one by one.
int run_part(Ctx& c, const StepArgs& a, bool use_graph, int part, int idx, hipStream_t st) {
  if (!use_graph) return enqueue_part(c, a, part, idx, st);
  const size_t at = part == 0 ? 0 : (part == 3 ? (size_t)1 + 2 * a.V + idx : (size_t)part + 2 * idx);
  VF_HIP(hipGraphLaunch(c.gs().graphs[at], st));
  return VF_OK;
}

// Everything of one step except the optimizer update (Section 3.2 steps 1-3).  One stream: the
// nodes one after another, each window of nodes followed by its side part.  Two streams: the
// forward parts on the caller's stream, the backward and side parts on the second one.
int enqueue_nodes(Ctx& c, const StepArgs& a, bool use_graph) {
  const bool ov = c.overlapping();
  if (use_graph && !ov) {          // the whole step is one captured chain
    VF_HIP(hipGraphLaunch(c.gs().graphs[0], c.stream));
    return VF_OK;
  }
  if (!ov || use_graph) VF_TRY(run_part(c, a, use_graph, 0, 0, c.stream));
  if (!ov) {
    for (int i0 = 0; i0 < a.V; i0 += c.window) {
      const int count = std::min(c.window, a.V - i0);
      for (int i = i0; i < i0 + count; ++i) VF_TRY(c.model->run_node_main(c, a, i, c.stream));
      VF_TRY(c.model->run_nodes_side(c, a, i0, count, c.stream));
    }
    return VF_OK;
  }
  // prep_done: the previous step's update is complete (and, replaying graphs, this step's
  // preparation too)
  VF_HIP(hipEventRecord(c.prep_done, c.stream));
  VF_HIP(hipStreamWaitEvent(c.side, c.prep_done, 0));
  if (!use_graph) VF_TRY(c.model->prepare_split(c, a.params, c.stream, c.side));
  c.marking = !use_graph && !c.ranges.empty();
  const int nwin = (a.V + c.window - 1) / c.window;
  const int reach = std::max(1, std::min(2, c.copies() / c.window));
  // Side part i on the forward stream, behind forward part i+1: it reads tensor set i & 1, which
  // forward part i+2 -- enqueued after it on the same stream -- writes next, and what backward
  // part i left for it, which backward part i+2 overwrites only after forward part i+2.
  const bool beside = c.window == 1 && c.model->side_beside_forward(c);
  if (beside) {
    for (int i = 0; i < a.V; ++i) {
      const int q = c.aset(i);
      if (i >= 2) VF_HIP(hipStreamWaitEvent(c.stream, c.bwd_done[q], 0));
      VF_TRY(run_part(c, a, use_graph, 1, i, c.stream));
      VF_HIP(hipEventRecord(c.fwd_done[q], c.stream));
      VF_HIP(hipStreamWaitEvent(c.side, c.fwd_done[q], 0));
      VF_TRY(run_part(c, a, use_graph, 2, i, c.side));
      VF_HIP(hipEventRecord(c.bwd_done[q], c.side));
      if (i >= 1) {
        VF_HIP(hipStreamWaitEvent(c.stream, c.bwd_done[q ^ 1], 0));
        VF_TRY(run_part(c, a, use_graph, 3, i - 1, c.stream));
      }
    }
    // join: the last backward part ends the second stream's work
    c.last_side = c.bwd_done[c.aset(a.V - 1)];
    VF_HIP(hipStreamWaitEvent(c.stream, c.last_side, 0));
    VF_TRY(run_part(c, a, use_graph, 3, a.V - 1, c.stream));
    return VF_OK;
  }
  for (int w = 0; w < nwin; ++w) {
    const int i0 = w * c.window, i1 = std::min(a.V, i0 + c.window);
    // This window's forward parts overwrite operand copies that an earlier side part reads: the
    // one `reach` windows back, where `reach` windows fit into the copies.
    if (w >= reach) VF_HIP(hipStreamWaitEvent(c.stream, c.side_done[(w - reach) & 1], 0));
    for (int i = i0; i < i1; ++i) {
      const int q = c.aset(i);
      // the tensors of set q were last read by bwd(i-2)
      if (i >= 2) VF_HIP(hipStreamWaitEvent(c.stream, c.bwd_done[q], 0));
      VF_TRY(run_part(c, a, use_graph, 1, i, c.stream));
      VF_HIP(hipEventRecord(c.fwd_done[q], c.stream));
      VF_HIP(hipStreamWaitEvent(c.side, c.fwd_done[q], 0));
      VF_TRY(run_part(c, a, use_graph, 2, i, c.side));
      VF_HIP(hipEventRecord(c.bwd_done[q], c.side));
    }
    // The window's weight gradients follow its backward parts on the second stream (a staged
    // node's gradient lives in the one staging vector that the next backward part writes again).
    VF_TRY(run_part(c, a, use_graph, 3, w, c.side));
    VF_HIP(hipEventRecord(c.side_done[w & 1], c.side));
  }
  // join: the last side part is the last thing on the second stream (when the update goes
  // stretch by stretch it joins after its last launch)
  c.last_side = c.side_done[(nwin - 1) & 1];
  if (!c.marking) VF_HIP(hipStreamWaitEvent(c.stream, c.last_side, 0));
  return VF_OK;
}

int update_stretch(Ctx& c, float* params, int64_t off, int64_t n) {
  const vf_config& f = c.cfg;
  if (f.optimizer == VF_SGDM) {
    VF_K(c, "optimizer", launch_sgdm(params + off, c.opt0 + off, c.gbuf + off, f.lr, f.momentum, n, c.stream));
    return VF_OK;
  }
  const double t = (double)(c.steps + 1);
  const float inv_c1 = (float)(1.0 / (1.0 - std::pow((double)f.beta1, t)));
  const float inv_c2 = (float)(1.0 / (1.0 - std::pow((double)f.beta2, t)));
  VF_K(c, "optimizer", launch_adam(params + off, c.opt0 + off, c.opt1 + off, c.gbuf + off, f.lr, f.beta1, f.beta2,
                                   f.adam_eps, inv_c1, inv_c2, n, c.stream));
  return VF_OK;
}

// The one update of a step (Section 3.2 step 5): elementwise, so it may go stretch by stretch,
// each as soon as its gradient is complete.
int enqueue_update(Ctx& c, float* params) {
  if (!c.marking) return update_stretch(c, params, 0, c.P);
  c.marking = false;
  for (size_t k = 0; k < c.ranges.size(); ++k) {
    VF_HIP(hipStreamWaitEvent(c.stream, c.range_done[k], 0));
    VF_TRY(update_stretch(c, params, c.ranges[k].off, c.ranges[k].n));
  }
  VF_HIP(hipStreamWaitEvent(c.stream, c.last_side, 0));
  return VF_OK;
}

int copy_out(Ctx& c, const float* src, float* out, size_t count) {
  VF_HIP(hipMemcpyAsync(out, src, count * sizeof(float), hipMemcpyDefault, c.stream));
  VF_HIP(hipStreamSynchronize(c.stream));
  return VF_OK;
}

}  // namespace

int Ctx::mark_range(int k, hipStream_t st) {
  if (!marking || k < 0 || k >= (int)range_done.size()) return VF_OK;
  VF_HIP(hipEventRecord(range_done[k], st));
  return VF_OK;
}

int Ctx::fold(int node, float w, hipStream_t st) {
  if (fused) return VF_OK;
  VF_KS(*this, st, "accumulate", launch_accumulate(gbuf, stage_for(node), w, P, node == 0, st));
  return VF_OK;
}

}  // namespace vf

using namespace vf;

extern "C" {

int vf_partition(const int32_t* node_sizes, int32_t V, int32_t B, int32_t* off_out, float* w_out) {
  int rc = check_partition(node_sizes, V, B);
  if (rc != VF_OK) return rc;
  if (off_out) {
    off_out[0] = 0;
    for (int32_t i = 0; i < V; ++i) off_out[i + 1] = off_out[i] + node_sizes[i];
  }
  if (w_out)
    for (int32_t i = 0; i < V; ++i) w_out[i] = (float)node_sizes[i] / (float)B;
  return VF_OK;
}

int vf_init(const vf_config* cfg, vf_ctx** out) {
  if (out) *out = nullptr;
  if (!cfg || !out) return VF_EINVAL;
  int rc = validate_config(*cfg);
  if (rc != VF_OK) return rc;
  vf_ctx* h = new (std::nothrow) vf_ctx();
  if (!h) return VF_ENOMEM;
  Ctx& c = h->c;
  c.cfg = *cfg;
  // Units of 16 or 32 nodes: a fold window never needs more units than a batch has (the window's
  // transposed operand copies are sized by window x largest unit).
  if (c.cfg.node_group >= 16 && c.cfg.fold_window > 1) {
    const int64_t unit = (int64_t)c.cfg.max_node_size * c.cfg.node_group;
    c.cfg.fold_window = (int32_t)std::max<int64_t>(1, std::min<int64_t>(c.cfg.fold_window, (c.cfg.max_batch + unit - 1) / unit));
  }
  cfg = &c.cfg;
  c.stream = static_cast<hipStream_t>(cfg->stream);
  if (!c.stream) c.cfg.flags |= VF_FLAG_NO_GRAPH;   // the default stream cannot be captured
  c.bf16 = cfg->dtype == VF_BF16;
  c.fused = (cfg->flags & VF_FLAG_FUSED_ACCUMULATE) != 0;
  hipError_t e = hipGetDevice(&c.device);
  if (e != hipSuccess) {
    set_last_error("hipGetDevice", e, __FILE__, __LINE__);
    delete h;
    return VF_EDEVICE;
  }
  c.model = cfg->model_kind == VF_MLP ? make_mlp(*cfg) : cfg->model_kind == VF_CONV ? make_conv(*cfg) : make_encoder(*cfg);
  if (!c.model) { delete h; return VF_EINVAL; }
  c.P = c.model->num_params();
  c.group = std::max(1, cfg->node_group);
  if (cfg->model_kind == VF_ENCODER) c.group = std::min(c.group, 4);   // its units are at most four nodes
  // Overlap needs a capturable main stream and a model that double-buffers what the side
  // stream reads (the bf16 MLP and the bf16 encoder do).
  c.overlap = c.stream != nullptr && (cfg->flags & VF_FLAG_OVERLAP) && c.model->supports_overlap();
  // A window needs the fused fold: a staged node's gradient lives in one staging vector.
  c.window = (!c.fused || cfg->fold_window < 1) ? 1 : std::min(cfg->fold_window, c.model->max_window());
  if (c.overlap) {
    e = hipStreamCreateWithFlags(&c.side, hipStreamNonBlocking);
    hipEvent_t* evs[] = {&c.fwd_done[0], &c.fwd_done[1], &c.bwd_done[0], &c.bwd_done[1],
                         &c.side_done[0], &c.side_done[1], &c.prep_done};
    for (hipEvent_t* ev : evs)
      if (e == hipSuccess) e = hipEventCreateWithFlags(ev, hipEventDisableTiming);
    c.model->update_ranges(&c.ranges);
    c.range_done.assign(c.ranges.size(), nullptr);
    for (hipEvent_t& ev : c.range_done)
      if (e == hipSuccess) e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
    if (e != hipSuccess) {
      set_last_error("side stream set-up", e, __FILE__, __LINE__);
      release_streams(c);
      delete h;
      return VF_EDEVICE;
    }
  }

  Arena arena;
  arena.request(&c.gbuf, (size_t)c.P);
  if (!c.fused) arena.request(&c.gstage, (size_t)c.P);
  arena.request(&c.opt0, (size_t)c.P);
  if (cfg->optimizer == VF_ADAM) arena.request(&c.opt1, (size_t)c.P);
  // per-row losses: of the whole batch (MLP: reduced once, after the last node's forward pass)
  size_t loss_rows = (size_t)cfg->max_batch;
  if (cfg->model_kind == VF_ENCODER) loss_rows = (size_t)cfg->max_node_size * c.group * (size_t)cfg->n_masked;
  arena.request(&c.rowloss, loss_rows);
  arena.request(&c.node_loss, (size_t)cfg->max_nodes);
  arena.request(&c.loss_total, 1);
  c.model->request_buffers(arena);
  c.arena_bytes = arena.total();
  e = hipMalloc(reinterpret_cast<void**>(&c.arena), c.arena_bytes);
  if (e != hipSuccess) {
    set_last_error("hipMalloc", e, __FILE__, __LINE__);
    c.arena = nullptr;
    (void)hipGetLastError();
    release_streams(c);
    delete h;
    return VF_ENOMEM;
  }
  arena.assign(c.arena);
  // optimizer state and loss cells start at zero
  if (Arena::guard()) {
    e = hipMemsetAsync(c.arena, 0x7f, c.arena_bytes, c.stream);
    arena.for_each_buffer([&](size_t off, size_t bytes) {
      if (e == hipSuccess && bytes) e = hipMemsetAsync(c.arena + off, 0, bytes, c.stream);
    });
  } else {
    e = hipMemsetAsync(c.arena, 0, c.arena_bytes, c.stream);
  }
  if (e == hipSuccess && c.model->init_state(c.stream) != VF_OK) e = hipErrorUnknown;
  if (e == hipSuccess) e = hipStreamSynchronize(c.stream);
  if (e != hipSuccess) {
    set_last_error("hipMemsetAsync", e, __FILE__, __LINE__);
    (void)hipGetLastError();
    release_streams(c);
    (void)hipFree(c.arena);
    delete h;
    return VF_EDEVICE;
  }
  *out = h;
  return VF_OK;
}

namespace {
// Everything vf_step checks before any device work.
int check_step(const Ctx& c, const void* params, int32_t B, int32_t V, const int32_t* node_sizes) {
  int rc = check_partition(node_sizes, V, B);
  if (rc != VF_OK) return rc;
  if (V > c.cfg.max_nodes || B > c.cfg.max_batch) return VF_EINVAL;
  for (int32_t i = 0; i < V; ++i)
    if (node_sizes[i] > c.cfg.max_node_size) return VF_EINVAL;
  if (reinterpret_cast<uintptr_t>(params) & 15) return VF_EINVAL;
  return VF_OK;
}
}  // namespace

int vf_prefetch(vf_ctx* h, const void* host_x, const int32_t* host_y, int32_t B) {
  if (!h || !host_x || !host_y || B < 1 || B > h->c.cfg.max_batch) return VF_EINVAL;
  Ctx& c = h->c;
  Ctx::Prefetch& p = c.pf;
  if (p.pending) return VF_ESTATE;                 // one batch ahead: the staged one has not been used
  VF_TRY(init_prefetch(c));
  const int k = p.next;
  // the step that last read this pair of buffers has to be through with them
  if (p.used[k]) VF_HIP(hipStreamWaitEvent(p.stream, p.consumed[k], 0));
  VF_HIP(hipMemcpyAsync(p.x[k], host_x, batch_x_bytes(c.cfg, B), hipMemcpyHostToDevice, p.stream));
  VF_HIP(hipMemcpyAsync(p.y[k], host_y, batch_y_bytes(c.cfg, B), hipMemcpyHostToDevice, p.stream));
  VF_HIP(hipEventRecord(p.copied[k], p.stream));
  p.pending = true;
  p.pending_B = B;
  return VF_OK;
}

int vf_step_prefetched(vf_ctx* h, void* params, int32_t V, const int32_t* node_sizes) {
  if (!h || !params) return VF_EINVAL;
  Ctx& c = h->c;
  Ctx::Prefetch& p = c.pf;
  if (!p.pending) return VF_ESTATE;
  int rc = check_step(c, params, p.pending_B, V, node_sizes);
  if (rc != VF_OK) return rc;                      // the staged batch stays staged
  const int k = p.next;
  VF_HIP(hipStreamWaitEvent(c.stream, p.copied[k], 0));
  rc = vf_step(h, params, p.x[k], static_cast<const int32_t*>(p.y[k]), p.pending_B, V, node_sizes);
  if (rc != VF_OK) return rc;
  VF_HIP(hipEventRecord(p.consumed[k], c.stream));
  p.used[k] = true;
  p.pending = false;
  p.next = k ^ 1;
  return VF_OK;
}

int vf_step(vf_ctx* h, void* params, const void* batch_x, const int32_t* batch_y, int32_t B,
            int32_t V, const int32_t* node_sizes) {
  if (!h || !params || !batch_x || !batch_y) return VF_EINVAL;
  Ctx& c = h->c;
  int rc = check_step(c, params, B, V, node_sizes);
  if (rc != VF_OK) return rc;

  StepArgs a;
  a.params = static_cast<float*>(params);
  a.x = batch_x; a.y = batch_y; a.B = B;
  a.nodes = V;
  a.node_sizes.assign(node_sizes, node_sizes + V);
  a.node_off.resize(V + 1);
  a.node_w.resize(V);
  vf_partition(node_sizes, V, B, a.node_off.data(), a.node_w.data());
  // the units of the passes: the nodes, or runs of up to `group` consecutive nodes -- of any sizes the
  // model takes together, or (models that want equal sizes) 2, 4 or 8 nodes of one size
  for (int32_t i = 0; i < V;) {
    int take = 1;
    const int most = std::min(c.group, c.model->max_group(node_sizes[i]));
    if (most > 1) {
      int run = 1;
      if (c.model->groups_unequal()) {
        while (i + run < V && run < most && c.model->max_group(node_sizes[i + run]) > 1) ++run;
        take = run;
      } else {
        while (i + run < V && run < most && node_sizes[i + run] == node_sizes[i]) ++run;
        take = run >= 8 ? 8 : (run >= 4 ? 4 : (run >= 2 ? 2 : 1));
      }
    }
    int32_t rows = 0;
    for (int j = 0; j < take; ++j) rows += node_sizes[i + j];
    a.sizes.push_back(rows);
    a.seg.push_back(node_sizes[i]);
    a.first.push_back(i);
    a.count.push_back(take);
    i += take;
  }
  a.V = (int32_t)a.sizes.size();
  a.off.resize(a.V + 1);
  a.w.resize(a.V);
  vf_partition(a.sizes.data(), a.V, B, a.off.data(), a.w.data());

  const bool use_graph = !((c.cfg.flags & VF_FLAG_NO_GRAPH) || c.prof.enabled);
  if (use_graph && !graph_matches(c, a)) VF_TRY(capture_graphs(c, a));
  VF_TRY(enqueue_nodes(c, a, use_graph));
  VF_TRY(enqueue_update(c, a.params));
  c.steps += 1;
  c.last_V = V;
  return VF_OK;
}

int vf_grads(vf_ctx* h, float* out) {
  if (!h || !out) return VF_EINVAL;
  if (h->c.steps == 0) return VF_ESTATE;
  return copy_out(h->c, h->c.gbuf, out, (size_t)h->c.P);
}

int vf_loss(vf_ctx* h, float* out) {
  if (!h || !out) return VF_EINVAL;
  if (h->c.steps == 0) return VF_ESTATE;
  return copy_out(h->c, h->c.loss_total, out, 1);
}

int vf_node_losses(vf_ctx* h, float* out, int32_t V) {
  if (!h || !out) return VF_EINVAL;
  if (h->c.steps == 0) return VF_ESTATE;
  if (V != h->c.last_V) return VF_EINVAL;
  return copy_out(h->c, h->c.node_loss, out, (size_t)V);
}

int vf_opt_state(vf_ctx* h, int32_t which, float* out) {
  if (!h || !out) return VF_EINVAL;
  Ctx& c = h->c;
  if (which == 0) return copy_out(c, c.opt0, out, (size_t)c.P);
  if (which == 1 && c.cfg.optimizer == VF_ADAM) return copy_out(c, c.opt1, out, (size_t)c.P);
  return VF_EINVAL;
}

int vf_profile_start(vf_ctx* h) {
  if (!h) return VF_EINVAL;
  Profiler& p = h->c.prof;
  p.enabled = true;
  p.recs.clear();
  p.used = 0;
  return VF_OK;
}

int vf_profile_stop(vf_ctx* h, char* out, size_t cap) {
  if (!h || !out || cap < 2) return VF_EINVAL;
  Ctx& c = h->c;
  Profiler& p = c.prof;
  p.enabled = false;
  VF_HIP(hipStreamSynchronize(c.stream));
  struct Agg { const char* tag; double ms; int64_t n; };
  std::vector<Agg> agg;
  for (const Profiler::Rec& r : p.recs) {
    float ms = 0.f;
    VF_HIP(hipEventElapsedTime(&ms, r.a, r.b));
    Agg* hit = nullptr;
    for (Agg& a : agg)
      if (std::strcmp(a.tag, r.tag) == 0) { hit = &a; break; }
    if (!hit) { agg.push_back({r.tag, 0.0, 0}); hit = &agg.back(); }
    hit->ms += ms;
    hit->n += 1;
  }
  p.recs.clear();
  p.used = 0;
  std::string js = "{";
  for (size_t i = 0; i < agg.size(); ++i) {
    char buf[160];
    snprintf(buf, sizeof buf, "%s\"%s\": {\"launches\": %lld, \"total_ms\": %.6f}", i ? ", " : "",
             agg[i].tag, (long long)agg[i].n, agg[i].ms);
    js += buf;
  }
  js += "}";
  if (js.size() + 1 > cap) return VF_EINVAL;
  std::memcpy(out, js.c_str(), js.size() + 1);
  return VF_OK;
}

int64_t vf_state_bytes(const vf_ctx* h) {
  if (!h) return 0;
  const Ctx& c = h->c;
  const int64_t n_opt = c.cfg.optimizer == VF_ADAM ? 2 : 1;
  return VF_STATE_HEADER_BYTES + 4 * (c.P + n_opt * c.P + c.model->state_floats());
}

int vf_state_export(vf_ctx* h, const float* params, void* dst, int64_t bytes) {
  if (!h || !params || !dst || bytes < vf_state_bytes(h)) return VF_EINVAL;
  Ctx& c = h->c;
  const int64_t n_opt = c.cfg.optimizer == VF_ADAM ? 2 : 1;
  const int64_t S2 = c.model->state_floats();
  const int64_t header[8] = {VF_STATE_MAGIC, c.P, n_opt, S2 / 2, c.steps, c.cfg.optimizer, 0, 0};
  char* out = static_cast<char*>(dst);
  const size_t pb = (size_t)c.P * sizeof(float);
  VF_HIP(hipMemcpyAsync(out, header, sizeof header, hipMemcpyDefault, c.stream));
  out += VF_STATE_HEADER_BYTES;
  VF_HIP(hipMemcpyAsync(out, params, pb, hipMemcpyDefault, c.stream)); out += pb;
  VF_HIP(hipMemcpyAsync(out, c.opt0, pb, hipMemcpyDefault, c.stream)); out += pb;
  if (n_opt == 2) { VF_HIP(hipMemcpyAsync(out, c.opt1, pb, hipMemcpyDefault, c.stream)); out += pb; }
  if (S2) VF_HIP(hipMemcpyAsync(out, c.model->state_ptr(), (size_t)S2 * sizeof(float), hipMemcpyDefault, c.stream));
  VF_HIP(hipStreamSynchronize(c.stream));   // `header` lives on this frame
  return VF_OK;
}

int vf_state_import(vf_ctx* h, float* params, const void* src, int64_t bytes) {
  if (!h || !params || !src || bytes < vf_state_bytes(h)) return VF_EINVAL;
  Ctx& c = h->c;
  const int64_t n_opt = c.cfg.optimizer == VF_ADAM ? 2 : 1;
  const int64_t S2 = c.model->state_floats();
  int64_t header[8];
  VF_HIP(hipStreamSynchronize(c.stream));
  VF_HIP(hipMemcpy(header, src, sizeof header, hipMemcpyDefault));
  if (header[0] != VF_STATE_MAGIC || header[1] != c.P || header[2] != n_opt || header[3] != S2 / 2 ||
      header[4] < 0 || header[5] != c.cfg.optimizer)
    return VF_EINVAL;
  const char* in = static_cast<const char*>(src) + VF_STATE_HEADER_BYTES;
  const size_t pb = (size_t)c.P * sizeof(float);
  VF_HIP(hipMemcpyAsync(params, in, pb, hipMemcpyDefault, c.stream)); in += pb;
  VF_HIP(hipMemcpyAsync(c.opt0, in, pb, hipMemcpyDefault, c.stream)); in += pb;
  if (n_opt == 2) { VF_HIP(hipMemcpyAsync(c.opt1, in, pb, hipMemcpyDefault, c.stream)); in += pb; }
  if (S2) VF_HIP(hipMemcpyAsync(c.model->state_ptr(), in, (size_t)S2 * sizeof(float), hipMemcpyDefault, c.stream));
  VF_HIP(hipStreamSynchronize(c.stream));
  c.steps = header[4];
  return VF_OK;
}

int64_t vf_step_count(const vf_ctx* h) { return h ? h->c.steps : 0; }
int32_t vf_fold_window(const vf_ctx* h) { return h ? h->c.window : 0; }
int32_t vf_streams(const vf_ctx* h) { return h ? (h->c.overlap ? 2 : 1) : 0; }
int64_t vf_num_params(const vf_ctx* h) { return h ? h->c.P : 0; }
size_t vf_workspace_bytes(const vf_ctx* h) { return h ? h->c.arena_bytes : 0; }

void vf_destroy(vf_ctx* h) {
  if (!h) return;
  Ctx& c = h->c;
  if (c.arena) {
    (void)hipStreamSynchronize(c.stream);
    if (c.side) (void)hipStreamSynchronize(c.side);
    drop_graph(c);
    c.cur ^= 1;
    drop_graph(c);
    release_streams(c);
    release_prefetch(c);
    for (hipEvent_t e : c.prof.pool) (void)hipEventDestroy(e);
    (void)hipFree(c.arena);
  }
  delete h;
}

const char* vf_strerror(int code) {
  switch (code) {
    case VF_OK: return "ok";
    case VF_EINVAL: return "invalid argument";
    case VF_ENOMEM: return "out of memory";
    case VF_EDEVICE: return "device error";
    case VF_ESTATE: return "call made in the wrong state";
    default: return "unknown error";
  }
}

const char* vf_last_error(void) { return g_last_error.c_str(); }

int vf_accumulate(float* buf, const float* g, float w, int64_t n, int32_t first, void* stream) {
  return launch_accumulate(buf, g, w, n, first, static_cast<hipStream_t>(stream));
}

int vf_sgdm_update(float* theta, float* v, const float* G, float lr, float momentum, int64_t n,
                   void* stream) {
  return launch_sgdm(theta, v, G, lr, momentum, n, static_cast<hipStream_t>(stream));
}

int vf_adam_update(float* theta, float* m, float* u, const float* G, float lr, float beta1,
                   float beta2, float eps, int64_t t, int64_t n, void* stream) {
  if (t < 1) return VF_EINVAL;
  const float inv_c1 = (float)(1.0 / (1.0 - std::pow((double)beta1, (double)t)));
  const float inv_c2 = (float)(1.0 / (1.0 - std::pow((double)beta2, (double)t)));
  return launch_adam(theta, m, u, G, lr, beta1, beta2, eps, inv_c1, inv_c2, n,
                     static_cast<hipStream_t>(stream));
}

int vf_gemm(int32_t dtype, const void* A, int64_t lda, const void* B, int64_t ldb, float* C,
            int64_t ldc, int32_t M, int32_t N, int32_t K, float alpha, int32_t accumulate,
            int32_t nsplit, void* stream) {
  if (!A || !B || !C || M < 1 || N < 1 || K < 1 || lda < K || ldb < K || ldc < N) return VF_EINVAL;
  if (nsplit < 1 || (nsplit > 1 && (accumulate || dtype != VF_BF16))) return VF_EINVAL;
  Epilogue ep;
  ep.C = C; ep.ldc = ldc; ep.alpha = alpha;
  if (accumulate) { ep.R = C; ep.ldr = ldc; ep.beta = 1.f; }
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dtype == VF_BF16)
    return launch_gemm_bf16(static_cast<const bf16_t*>(A), lda, static_cast<const bf16_t*>(B), ldb,
                            M, N, K, nsplit, (int64_t)M * ldc, ep, s);
  if (dtype == VF_F32)
    return launch_gemm_f32(static_cast<const float*>(A), lda, 1, static_cast<const float*>(B), ldb, 1,
                           M, N, K, 1, 0, ep, s);
  return VF_EINVAL;
}

}  // extern "C"
