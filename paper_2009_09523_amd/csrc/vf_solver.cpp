// Heterogeneous split solver (Section 5.1.2): given per-accelerator-type offline profiles
// (time of one virtual-node pass against node batch size, Section 5.1.1), choose the per-device
// batch b_i and the number of virtual nodes v_i per device of every type so that
//     max_i ( t_i(b_i / v_i) * v_i + comm )     is minimal, subject to   sum_i n_i * b_i = B.
// Host code only.  Exhaustive search over power-of-2 and power-of-2-like per-device batches
// (the sizes the paper's profiler considers), a type may stay unused (b_i = 0: the
// homogeneous fallback of the paper).
#include <cmath>
#include <limits>
#include <vector>

#include "vf.h"

namespace {

// 1, 2, 3, 4, 6, 8, 12, 16, 24, ... up to `limit`
std::vector<int32_t> candidate_batches(int32_t limit) {
  std::vector<int32_t> c;
  for (int64_t p = 1; p <= limit; p *= 2) {
    c.push_back((int32_t)p);
    if (p >= 2 && p + p / 2 <= limit) c.push_back((int32_t)(p + p / 2));
  }
  return c;
}

struct Choice { int32_t v; double t; };   // best node count for one per-device batch

// Fewest sequential passes' total time for a device batch b: min over v with b % v == 0 and
// b / v in the profile of t(b / v) * v; ties go to the smaller v.
bool best_nodes(const vf_device_profile& p, int32_t b, Choice* out) {
  bool found = false;
  for (int32_t k = p.n_points - 1; k >= 0; --k) {      // large nodes first = small v first
    const int32_t node = p.batch[k];
    if (node < 1 || b % node) continue;
    const int32_t v = b / node;
    const double t = p.step_time[k] * (double)v;
    if (!found || t < out->t) { out->v = v; out->t = t; found = true; }
  }
  return found;
}

struct Search {
  const vf_device_profile* types;
  int32_t n_types, B;
  double comm;
  std::vector<std::vector<int32_t>> cand;        // per type: 0 and the candidate batches
  std::vector<std::vector<Choice>> choice;       // per type, per candidate
  std::vector<int32_t> cur, best_b, best_v;
  std::vector<int32_t> cur_v;
  double best = std::numeric_limits<double>::infinity();

  void rec(int i, int64_t assigned, double worst, int devices) {
    if (i == n_types) {
      if (assigned != B || devices == 0) return;
      const double total = worst + (devices > 1 ? comm : 0.0);
      if (total < best) { best = total; best_b = cur; best_v = cur_v; }
      return;
    }
    for (size_t k = 0; k < cand[i].size(); ++k) {
      const int32_t b = cand[i][k];
      const int64_t a = assigned + (int64_t)types[i].n_devices * b;
      if (a > B) break;                            // candidates ascend
      cur[i] = b;
      cur_v[i] = b ? choice[i][k].v : 0;
      rec(i + 1, a, b ? std::fmax(worst, choice[i][k].t) : worst, devices + (b ? types[i].n_devices : 0));
    }
  }
};

}  // namespace

extern "C" int vf_solve_split(const vf_device_profile* types, int32_t n_types, int32_t B, double comm,
                              int32_t* b_out, int32_t* v_out, double* step_time_out) {
  if (!types || n_types < 1 || n_types > 8 || B < 1 || !(comm >= 0.0) || !b_out || !v_out) return VF_EINVAL;
  for (int32_t i = 0; i < n_types; ++i) {
    const vf_device_profile& p = types[i];
    if (p.n_devices < 1 || p.n_points < 1 || !p.batch || !p.step_time) return VF_EINVAL;
    for (int32_t k = 0; k < p.n_points; ++k) {
      if (p.batch[k] < 1 || !(p.step_time[k] > 0.0)) return VF_EINVAL;
      if (k && p.batch[k] <= p.batch[k - 1]) return VF_EINVAL;
    }
  }
  Search s;
  s.types = types; s.n_types = n_types; s.B = B; s.comm = comm;
  s.cand.resize(n_types); s.choice.resize(n_types);
  s.cur.assign(n_types, 0); s.cur_v.assign(n_types, 0);
  const std::vector<int32_t> all = candidate_batches(B);
  for (int32_t i = 0; i < n_types; ++i) {
    s.cand[i].push_back(0);
    s.choice[i].push_back(Choice{0, 0.0});
    for (int32_t b : all) {
      Choice c;
      if (best_nodes(types[i], b, &c)) { s.cand[i].push_back(b); s.choice[i].push_back(c); }
    }
  }
  s.rec(0, 0, 0.0, 0);
  if (!(s.best < std::numeric_limits<double>::infinity())) return VF_ESTATE;   // no feasible split
  for (int32_t i = 0; i < n_types; ++i) { b_out[i] = s.best_b[i]; v_out[i] = s.best_v[i]; }
  if (step_time_out) *step_time_out = s.best;
  return VF_OK;
}
