// Host-only part of libla_verify: the step-level controller and the budget planner.  No device code; these run
// on the CPU between passes.
//
//   la_step_select      Algorithm 1, verification and output construction: j* = first draft step the verifier
//                       rejected (all accepted: the target's bonus step), and what la_kv_commit has to append for it.
//   la_step_select_tree the same walk over a draft tree (Section 3.1, multi-branch drafting).
//   la_speedup_*        Section 3.2 (step level, sync and async) and Section 3.3 (token level) closed forms.
//   la_plan_budget      Section 3.3: argmax over (k1, k2) of f(k1) g(k2) under ParallelDim_f * k2 <= M.
#include <math.h>

#include <vector>

#include "la_verify.h"

namespace {

inline bool rate_ok(double alpha, double c) {
  return alpha > 0.0 && alpha < 1.0 && c > 0.0 && c < 1.0 && isfinite(alpha) && isfinite(c);
}

// (1 - a^k) / (1 - a) = 1 + a + ... + a^(k-1), by Horner: no cancellation near a = 1, exact for k = 1
inline double geometric_sum(double a, int k) {
  double s = 1.0;
  for (int i = 1; i < k; ++i) s = s * a + 1.0;
  return s;
}

// Leviathan-style form shared by f_sync and g: expected steps per cycle over the cycle's cost
inline double sync_form(double a, double c, int k) { return geometric_sum(a, k) / (1.0 - c + c * k); }

inline int depth_limit(double c) { return (int)ceil(1.0 / c); }

double async_form(double a, double c, int k) {
  if (k >= depth_limit(c)) return 1.0 / (c + (1.0 - c) * (1.0 - a));  // S_1: the draft is the slower side
  // S_2, numerator and denominator divided by (1 - a):
  //   E[X mod k] (1 - a^k) = sum_{r<k} r a^r (1 - a)  =  a (1 + a + .. + a^(k-1)) - k a^k
  const double gs = geometric_sum(a, k);
  const double ak = pow(a, k);
  return gs / (1.0 + c * (a * gs - k * ak));
}

}  // namespace

extern "C" {

la_status la_step_select(int32_t num_requests, int32_t num_branches, const uint8_t *verdicts,
                         const int32_t *chain_vis, const int32_t *own_len, int32_t *j_star, int32_t *src_branch,
                         int32_t *n_chain, int32_t *n_own) {
  if (num_requests < 1 || num_branches < 1) return LA_ERR_INVALID_ARG;
  if ((num_branches > 1 && !verdicts) || !j_star) return LA_ERR_INVALID_ARG;
  if ((n_chain && !chain_vis) || (n_own && !own_len)) return LA_ERR_INVALID_ARG;
  const int drafts = num_branches - 1;  // branch j < drafts verifies draft j; the last branch is the bonus step
  for (int b = 0; b < num_requests; ++b) {
    int j = 0;
    while (j < drafts && verdicts[(size_t)b * drafts + j]) ++j;
    j_star[b] = j;
    if (src_branch) src_branch[b] = j;
    if (n_chain) n_chain[b] = chain_vis[(size_t)b * num_branches + j];
    if (n_own) n_own[b] = own_len[(size_t)b * num_branches + j];
  }
  return LA_OK;
}

la_status la_step_select_tree(int32_t num_requests, int32_t num_nodes, const int32_t *parent,
                              const uint8_t *verdicts, const int32_t *own_len, int32_t *depth,
                              uint64_t *commit_mask, int32_t *src_branch, int32_t *n_own) {
  if (num_requests < 1 || num_nodes < 0 || num_nodes > 64) return LA_ERR_INVALID_ARG;
  if ((num_nodes > 0 && (!parent || !verdicts)) || !depth || !commit_mask || (n_own && !own_len))
    return LA_ERR_INVALID_ARG;
  for (int n = 0; n < num_nodes; ++n)
    if (parent[n] < -1 || parent[n] >= n) return LA_ERR_INVALID_ARG;
  for (int b = 0; b < num_requests; ++b) {
    const uint8_t *v = verdicts + (size_t)b * num_nodes;
    int at = -1, steps = 0;  // -1: the root (nothing drafted accepted yet)
    uint64_t mask = 0;
    // parents come before children, so one sweep in node order follows the path downwards and meets the
    // alternatives of each position in ascending order: the first accepted one wins
    for (int n = 0; n < num_nodes; ++n) {
      if (parent[n] == at && v[n]) {
        at = n;
        mask |= (uint64_t)1 << n;
        ++steps;
      }
    }
    depth[b] = steps;
    commit_mask[b] = mask;
    if (src_branch) src_branch[b] = at + 1;
    if (n_own) n_own[b] = own_len[(size_t)b * (num_nodes + 1) + at + 1];
  }
  return LA_OK;
}

la_status la_speedup_step_sync(double alpha1, double c1, int32_t k1, double *speedup) {
  if (!speedup || !rate_ok(alpha1, c1) || k1 < 1) return LA_ERR_INVALID_ARG;
  *speedup = sync_form(alpha1, c1, k1);
  return LA_OK;
}

la_status la_speedup_step_async(double alpha1, double c1, int32_t k1, double *speedup) {
  if (!speedup || !rate_ok(alpha1, c1) || k1 < 1) return LA_ERR_INVALID_ARG;
  *speedup = async_form(alpha1, c1, k1);
  return LA_OK;
}

la_status la_speedup_token(double alpha2, double c2, int32_t k2, double *speedup) {
  if (!speedup || !rate_ok(alpha2, c2) || k2 < 1) return LA_ERR_INVALID_ARG;
  *speedup = sync_form(alpha2, c2, k2);
  return LA_OK;
}

la_status la_plan_budget(const la_plan_desc *d, int32_t *k1_out, int32_t *k2_out, double *speedup) {
  if (!d || !k1_out || !k2_out) return LA_ERR_INVALID_ARG;
  if (!rate_ok(d->alpha1, d->c1) || !rate_ok(d->alpha2, d->c2) || d->budget < 1 || d->budget > (1 << 20))
    return LA_ERR_INVALID_ARG;
  const int M = d->budget;
  const bool asyn = d->asynchronous != 0;
  // beyond the depth limit the async form and its parallel dimension are both constant: nothing new to try
  const int k1_max = asyn ? (depth_limit(d->c1) < M ? depth_limit(d->c1) : M) : M;
  std::vector<double> g(M + 1);
  for (int k2 = 1; k2 <= M; ++k2) g[k2] = sync_form(d->alpha2, d->c2, k2);
  double best = -1.0;
  int b1 = 1, b2 = 1;
  for (int k1 = 1; k1 <= k1_max; ++k1) {
    const double f = asyn ? async_form(d->alpha1, d->c1, k1) : sync_form(d->alpha1, d->c1, k1);
    const int dim_f = k1;  // async: k1 <= depth limit here, so min(ceil(1/c1), k1) = k1
    for (int k2 = 1; k2 <= M / dim_f; ++k2) {
      const double h = f * g[k2];
      if (h > best) best = h, b1 = k1, b2 = k2;  // strict: ties keep the smallest k1, then the smallest k2
    }
  }
  *k1_out = b1;
  *k2_out = b2;
  if (speedup) *speedup = best;
  return LA_OK;
}

}  // extern "C"
