// Layer partitioner (Section 3.2, "Partitioning algorithm"): pure host arithmetic on the per-layer profile.
//
// A(j, m) = time of the slowest stage of the best pipeline over layers 1..j on exactly m machines:
//   one stage replicated m times:        T(1 -> j, m)
//   or, over split points i and m':      max( A(i, m - m'),  2 C_i,  T(i+1 -> j, m') )
// with T(i -> j, m) = max(sum T_l, sum W_l^m) / m,  W_l^m = 4 (m-1) |w_l| / (m * bandwidth),  C_l = a_l / bandwidth.
// Layer sums come from prefix sums, so the table costs O(N^2 M^2) constant-time candidates.
#include <cmath>
#include <cstdint>
#include <vector>

#include "../../include/pd.h"
#include "pd_error.h"

namespace {

struct Problem {
  int N, M;
  double bw;
  std::vector<double> pre_t, pre_w;  // pre[k] = sum over the first k layers
  const double* a;

  // stage holding layers i+1..j (0 <= i < j <= N) on m machines
  double stage(int i, int j, int m) const {
    const double compute = pre_t[j] - pre_t[i];
    const double sync = m > 1 ? 4.0 * (m - 1) * (pre_w[j] - pre_w[i]) / m / bw : 0.0;
    return (compute > sync ? compute : sync) / m;
  }
  double boundary(int i) const { return 2.0 * a[i - 1] / bw; }  // after layer i (1-based)
};

}  // namespace

extern "C" int pd_partition(int32_t n_layers, int32_t n_machines, const double* t_layer, const double* act_bytes,
                            const double* param_bytes, double bandwidth, double* slowest_out,
                            pd_stage_assign* stages_out, size_t cap, size_t* n_stages_out, int32_t* noam_out) {
  using pd::fail;
  if (n_layers < 1 || n_machines < 1) return fail(PD_EINVAL, "partition: need at least one layer and one machine");
  if (!t_layer || !act_bytes || !param_bytes) return fail(PD_EINVAL, "partition: profile array is null");
  if (!(bandwidth > 0.0) || !std::isfinite(bandwidth)) return fail(PD_EINVAL, "partition: bandwidth must be positive");
  if ((int64_t)n_layers * n_machines > ((int64_t)1 << 24)) return fail(PD_EINVAL, "partition: problem too large");
  for (int l = 0; l < n_layers; ++l)
    if (!(t_layer[l] >= 0.0) || !(act_bytes[l] >= 0.0) || !(param_bytes[l] >= 0.0) || !std::isfinite(t_layer[l]) ||
        !std::isfinite(act_bytes[l]) || !std::isfinite(param_bytes[l]))
      return fail(PD_EINVAL, "partition: layer %d has a negative or non-finite profile value", l);

  Problem p;
  p.N = n_layers; p.M = n_machines; p.bw = bandwidth; p.a = act_bytes;
  p.pre_t.assign(n_layers + 1, 0.0);
  p.pre_w.assign(n_layers + 1, 0.0);
  for (int l = 0; l < n_layers; ++l) {
    p.pre_t[l + 1] = p.pre_t[l] + t_layer[l];
    p.pre_w[l + 1] = p.pre_w[l] + param_bytes[l];
  }
  const int N = p.N, M = p.M, ld = M + 1;
  std::vector<double> A((size_t)(N + 1) * ld, 0.0);
  std::vector<int32_t> cut((size_t)(N + 1) * ld, 0), rep((size_t)(N + 1) * ld, 0);  // cut = 0: a single stage
  for (int j = 1; j <= N; ++j)
    for (int m = 1; m <= M; ++m) {
      double best = p.stage(0, j, m);
      int bi = 0, bm = m;
      for (int i = 1; i < j; ++i) {
        const double c2 = p.boundary(i);
        if (c2 >= best) continue;  // no split here can win
        for (int mp = 1; mp < m; ++mp) {
          double cand = A[(size_t)i * ld + (m - mp)];
          if (c2 > cand) cand = c2;
          const double tail = p.stage(i, j, mp);
          if (tail > cand) cand = tail;
          if (cand < best) { best = cand; bi = i; bm = mp; }
        }
      }
      A[(size_t)j * ld + m] = best;
      cut[(size_t)j * ld + m] = bi;
      rep[(size_t)j * ld + m] = bm;
    }

  // walk the choices back from (N, M); stages come out last first
  std::vector<pd_stage_assign> rev;
  for (int j = N, m = M; j > 0;) {
    const int i = cut[(size_t)j * ld + m], r = rep[(size_t)j * ld + m];
    rev.push_back({i, j - 1, r});
    j = i;
    m -= r;
  }
  const size_t ns = rev.size();
  if (slowest_out) *slowest_out = A[(size_t)N * ld + M];
  if (n_stages_out) *n_stages_out = ns;
  if (noam_out) *noam_out = (n_machines + rev.back().replicas - 1) / rev.back().replicas;  // ceil(M / input-stage machines)
  if (ns > cap) return fail(PD_ENOMEM, "partition: %zu stages, capacity %zu", ns, cap);
  if (!stages_out) return fail(PD_EINVAL, "partition: stages_out is null");
  for (size_t k = 0; k < ns; ++k) stages_out[k] = rev[ns - 1 - k];
  return PD_OK;
}
