// Host-side checks of the C ABI, built with AddressSanitizer and UndefinedBehaviorSanitizer on the
// host code (no device code is compiled in, nothing is launched): argument validation of every
// entry point, the partition arithmetic, and the split solver against an exhaustive search.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <limits>
#include <vector>

#include "vf.h"

static int failures = 0;
#define CHECK(cond)                                                         \
  do {                                                                      \
    if (!(cond)) { std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); ++failures; } \
  } while (0)

static vf_config small_config() {
  vf_config c;
  std::memset(&c, 0, sizeof c);
  c.model_kind = VF_MLP; c.n_dims = 3; c.dims[0] = 8; c.dims[1] = 16; c.dims[2] = 4;
  c.dtype = VF_F32; c.optimizer = VF_SGDM; c.lr = 0.1f; c.momentum = 0.9f; c.bn_eps = 1e-5f;
  c.bn_momentum = 0.1f; c.max_batch = 16; c.max_node_size = 8; c.max_nodes = 4;
  return c;
}

static void partition_checks() {
  const int32_t sizes[] = {48, 48, 32, 32, 16, 16, 48, 16};
  int32_t off[9];
  float w[8];
  CHECK(vf_partition(sizes, 8, 256, off, w) == VF_OK);
  int32_t at = 0;
  for (int i = 0; i < 8; ++i) {
    CHECK(off[i] == at);
    const float want = (float)sizes[i] / 256.0f;
    CHECK(std::memcmp(&w[i], &want, 4) == 0);
    at += sizes[i];
  }
  CHECK(off[8] == 256);
  CHECK(vf_partition(sizes, 8, 256, nullptr, nullptr) == VF_OK);
  CHECK(vf_partition(sizes, 8, 255, off, w) == VF_EINVAL);
  CHECK(vf_partition(sizes, 0, 256, off, w) == VF_EINVAL);
  CHECK(vf_partition(nullptr, 8, 256, off, w) == VF_EINVAL);
  const int32_t bad[] = {4, 0, 4};
  CHECK(vf_partition(bad, 3, 8, off, w) == VF_EINVAL);
  const int32_t big[] = {std::numeric_limits<int32_t>::max(), std::numeric_limits<int32_t>::max()};
  CHECK(vf_partition(big, 2, -2, off, w) == VF_EINVAL);        // the sum is taken in 64 bits
}

static void config_checks() {
  vf_ctx* h = reinterpret_cast<vf_ctx*>(0x1);
  CHECK(vf_init(nullptr, &h) == VF_EINVAL && h == nullptr);
  vf_config c = small_config();
  CHECK(vf_init(&c, nullptr) == VF_EINVAL);
  struct Edit { void (*apply)(vf_config&); };
  const Edit edits[] = {
      {[](vf_config& f) { f.dtype = 9; }},          {[](vf_config& f) { f.optimizer = -1; }},
      {[](vf_config& f) { f.max_nodes = 0; }},      {[](vf_config& f) { f.max_node_size = 0; }},
      {[](vf_config& f) { f.max_node_size = 32; }}, {[](vf_config& f) { f.n_dims = 1; }},
      {[](vf_config& f) { f.n_dims = VF_MAX_DIMS + 1; }}, {[](vf_config& f) { f.dims[1] = 0; }},
      {[](vf_config& f) { f.model_kind = 7; }},     {[](vf_config& f) { f.bn_momentum = 1.5f; }},
      {[](vf_config& f) { f.bn_momentum = std::nanf(""); }}, {[](vf_config& f) { f.fold_window = 9; }},
      {[](vf_config& f) { f.fold_window = -1; }},   {[](vf_config& f) { f.node_group = 3; }},
      {[](vf_config& f) { f.dtype = VF_BF16; f.dims[0] = 12; }},
      {[](vf_config& f) { f.model_kind = VF_ENCODER; }},
      {[](vf_config& f) { f.model_kind = VF_CONV; f.dtype = VF_BF16; f.img = 8; f.in_ch = 3; f.width = 12; f.classes = 4; }},
  };
  for (const Edit& e : edits) {
    vf_config f = small_config();
    e.apply(f);
    h = reinterpret_cast<vf_ctx*>(0x1);
    CHECK(vf_init(&f, &h) == VF_EINVAL && h == nullptr);
  }
  // a valid configuration: with no device to run on the call fails after validation, cleanly
  h = nullptr;
  const int rc = vf_init(&c, &h);
  CHECK(rc == VF_OK || rc == VF_EDEVICE || rc == VF_ENOMEM);
  if (rc == VF_OK) vf_destroy(h);
  else CHECK(h == nullptr);
}

static void null_handle_checks() {
  float f = 0.f;
  int32_t one = 1;
  CHECK(vf_step(nullptr, &f, &f, &one, 1, 1, &one) == VF_EINVAL);
  CHECK(vf_prefetch(nullptr, &f, &one, 1) == VF_EINVAL);
  CHECK(vf_step_prefetched(nullptr, &f, 1, &one) == VF_EINVAL);
  CHECK(vf_grads(nullptr, &f) == VF_EINVAL);
  CHECK(vf_loss(nullptr, &f) == VF_EINVAL);
  CHECK(vf_node_losses(nullptr, &f, 1) == VF_EINVAL);
  CHECK(vf_opt_state(nullptr, 0, &f) == VF_EINVAL);
  CHECK(vf_profile_start(nullptr) == VF_EINVAL);
  char buf[8];
  CHECK(vf_profile_stop(nullptr, buf, sizeof buf) == VF_EINVAL);
  CHECK(vf_step_count(nullptr) == 0 && vf_fold_window(nullptr) == 0 && vf_streams(nullptr) == 0);
  CHECK(vf_num_params(nullptr) == 0 && vf_workspace_bytes(nullptr) == 0 && vf_state_bytes(nullptr) == 0);
  CHECK(vf_state_export(nullptr, &f, buf, 8) == VF_EINVAL);
  CHECK(vf_state_import(nullptr, &f, buf, 8) == VF_EINVAL);
  vf_destroy(nullptr);
  CHECK(std::strcmp(vf_strerror(VF_OK), vf_strerror(VF_EINVAL)) != 0);
  CHECK(vf_strerror(-99) != nullptr && vf_last_error() != nullptr);
  // stand-alone kernels: malformed arguments are rejected before anything is launched
  CHECK(vf_accumulate(nullptr, &f, 1.f, 4, 1, nullptr) == VF_EINVAL);
  CHECK(vf_sgdm_update(nullptr, &f, &f, 0.1f, 0.9f, 4, nullptr) == VF_EINVAL);
  CHECK(vf_adam_update(&f, &f, &f, &f, 0.1f, 0.9f, 0.999f, 1e-8f, 0, 4, nullptr) == VF_EINVAL);
  CHECK(vf_gemm(VF_BF16, nullptr, 8, &f, 8, &f, 8, 1, 1, 8, 1.f, 0, 1, nullptr) == VF_EINVAL);
  CHECK(vf_gemm(VF_F32, &f, 8, &f, 8, &f, 8, 1, 1, 8, 1.f, 1, 2, nullptr) == VF_EINVAL);
  CHECK(vf_gemm_noalloc(&f, 8, &f, 8, &f, 4096, 4096, 8, 1.f, 0, 1, nullptr) == VF_EINVAL);   // 64 MiB of slabs
  CHECK(vf_gemm_noalloc(nullptr, 8, &f, 8, &f, 1, 1, 8, 1.f, 0, 1, nullptr) == VF_EINVAL);
}

// exhaustive search over every per-device batch 0..B, the definition of Section 5.1.2
static double brute(const std::vector<vf_device_profile>& t, int32_t B, double comm) {
  double best = std::numeric_limits<double>::infinity();
  std::vector<int32_t> b(t.size(), 0);
  auto like = [](int32_t v) {
    if (v == 0) return true;
    while (v % 2 == 0) v /= 2;
    return v == 1 || v == 3;
  };
  std::vector<int32_t> idx(t.size(), 0);
  while (true) {
    int64_t sum = 0;
    double worst = 0.0;
    int devices = 0;
    bool ok = true;
    for (size_t i = 0; i < t.size() && ok; ++i) {
      const int32_t bi = idx[i];
      if (!like(bi)) { ok = false; break; }
      if (bi == 0) continue;
      sum += (int64_t)t[i].n_devices * bi;
      devices += t[i].n_devices;
      double ti = std::numeric_limits<double>::infinity();
      for (int k = 0; k < t[i].n_points; ++k)
        if (bi % t[i].batch[k] == 0) ti = std::fmin(ti, t[i].step_time[k] * (bi / t[i].batch[k]));
      if (!std::isfinite(ti)) ok = false;
      worst = std::fmax(worst, ti);
    }
    if (ok && sum == B && devices > 0) best = std::fmin(best, worst + (devices > 1 ? comm : 0.0));
    size_t i = 0;
    while (i < idx.size() && ++idx[i] > B) idx[i++] = 0;
    if (i == idx.size()) break;
  }
  return best;
}

static void solver_checks() {
  const int32_t nodes[] = {2, 3, 4, 6, 8};
  const double fast[] = {1.0, 1.4, 1.7, 2.4, 3.0}, slow[] = {3.9, 5.8, 7.1, 10.2, 13.0};
  std::vector<vf_device_profile> t = {{2, 5, nodes, fast}, {3, 5, nodes, slow}};
  for (int32_t B : {12, 24, 30, 48, 60}) {
    for (double comm : {0.0, 0.5}) {
      int32_t b[2], v[2];
      double got = -1.0;
      const int rc = vf_solve_split(t.data(), 2, B, comm, b, v, &got);
      const double want = brute(t, B, comm);
      if (std::isfinite(want)) {
        CHECK(rc == VF_OK && got == want);
        CHECK(t[0].n_devices * b[0] + t[1].n_devices * b[1] == B);
      } else {
        CHECK(rc == VF_ESTATE);
      }
    }
  }
  int32_t b[2], v[2];
  CHECK(vf_solve_split(nullptr, 2, 12, 0.0, b, v, nullptr) == VF_EINVAL);
  CHECK(vf_solve_split(t.data(), 0, 12, 0.0, b, v, nullptr) == VF_EINVAL);
  CHECK(vf_solve_split(t.data(), 9, 12, 0.0, b, v, nullptr) == VF_EINVAL);
  CHECK(vf_solve_split(t.data(), 2, 0, 0.0, b, v, nullptr) == VF_EINVAL);
  CHECK(vf_solve_split(t.data(), 2, 12, -1.0, b, v, nullptr) == VF_EINVAL);
  CHECK(vf_solve_split(t.data(), 2, 12, 0.0, nullptr, v, nullptr) == VF_EINVAL);
  std::vector<vf_device_profile> broken = t;
  broken[0].n_points = 0;
  CHECK(vf_solve_split(broken.data(), 2, 12, 0.0, b, v, nullptr) == VF_EINVAL);
  const double neg[] = {1.0, -1.0, 1.7, 2.4, 3.0};
  broken = t;
  broken[1].step_time = neg;
  CHECK(vf_solve_split(broken.data(), 2, 12, 0.0, b, v, nullptr) == VF_EINVAL);
}

int main() {
  partition_checks();
  config_checks();
  null_handle_checks();
  solver_checks();
  if (failures) { std::printf("%d checks failed\n", failures); return 1; }
  std::printf("host checks ok\n");
  return 0;
}
