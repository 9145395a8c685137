// Search over the pipeline hyper-parameters (S, M, D) of Sec. 3 (workflow steps 2-5): every feasible
// combination is partitioned (dp_partition_solve with a fixed stage count), its FIFO-1F1B iteration simulated
// (dp_bubbles_1f1b), its bubbles filled with the non-trainable components (dp_bubbles_fill), and the
// combination with the least iteration time is reported.  Host code only; it composes the library's own
// entry points and adds the walk over the combinations.
#include "../../include/dpipe.h"
#include "dp_errors.h"

#include <algorithm>
#include <map>
#include <utility>
#include <vector>

extern "C" int dp_schedule_search(const dp_layer_cost* rows, int n_rows, const dp_search_opts* opts, dp_search_candidate* cands,
                                  int max_cands, int* n_cands, int* best) {
  using dp::set_error;
  if (!rows || n_rows <= 0 || !opts || !cands || !n_cands || !best || max_cands <= 0) return set_error(DP_EINVAL, "dp_schedule_search: null argument");
  const dp_search_opts& o = *opts;
  if (o.world_size <= 0 || o.training_batch <= 0 || !o.group_sizes || o.n_group_sizes <= 0 || !o.micro_batch_counts || o.n_micro_batch_counts <= 0 ||
      o.max_stages < 0 || o.min_bubble_ms < 0.0 || o.n_dep_pairs < 0 || (o.n_dep_pairs > 0 && !o.dep_pairs))
    return set_error(DP_EINVAL, "dp_schedule_search: sizes must be positive, candidate lists non-empty");
  if (o.n_group_sizes > 4096 || o.n_micro_batch_counts > 4096) return set_error(DP_EUNSUPPORTED, "dp_schedule_search: candidate lists longer than 4096");
  *n_cands = 0; *best = -1;
  int rc = DP_OK;
  try {
    // backbone rows by (batch, layer), for the stage times of a plan
    std::map<std::pair<int, int>, const dp_layer_cost*> at;
    int L = 0;
    for (int i = 0; i < n_rows; ++i)
      if (rows[i].component == 0) { at[{rows[i].batch, rows[i].layer}] = &rows[i]; L = std::max(L, rows[i].layer + 1); }
    if (L == 0) return set_error(DP_EINVAL, "dp_schedule_search: no rows of component 0");
    bool frozen = false;
    for (int i = 0; i < n_rows; ++i) frozen = frozen || rows[i].component >= 1;
    if (!frozen) return set_error(DP_EINVAL, "dp_schedule_search: no rows of a non-trainable component (component >= 1)");
    int count = 0;
    for (int di = 0; di < o.n_group_sizes; ++di) {
      const int D = o.group_sizes[di];
      if (D <= 0 || D > DP_MAX_STAGES || o.world_size % D || ((long)o.training_batch * D) % o.world_size) continue;
      const int group_batch = (int)((long)o.training_batch * D / o.world_size);
      for (int mi = 0; mi < o.n_micro_batch_counts; ++mi) {
        const int M = o.micro_batch_counts[mi];
        if (M <= 0 || group_batch % M || group_batch / M == 0) continue;
        const int B = group_batch / M;
        const int s_max = std::min(std::min(L, D), o.max_stages > 0 ? o.max_stages : DP_MAX_STAGES);
        for (int S = 1; S <= s_max; ++S) {
          dp_partition_opts po;
          po.micro_batch = B; po.n_micro_batches = M; po.n_devices = D; po.max_stages = o.max_stages;
          po.uniform_replication = o.uniform_replication; po.p2p_gbps = o.p2p_gbps; po.p2p_latency_ms = o.p2p_latency_ms;
          po.ar_gbps = o.ar_gbps; po.ar_latency_ms = o.ar_latency_ms; po.self_cond_prob = o.self_cond_prob; po.exact_stages = S;
          if (o.self_cond_prob > 0.0 && !at.count({B, L - 1})) continue;   // no profile of the feedback transfer at this micro-batch size
          dp_search_candidate c;
          const int prc = dp_partition_solve(rows, n_rows, &po, &c.plan);
          if (prc == DP_EUNSUPPORTED) continue;                            // no feasible partition into S stages
          if (prc != DP_OK) return prc;
          if (c.plan.n_stages != S) continue;
          // step 3: stage and transfer times of the plan, then the simulated iteration
          std::vector<double> f(S), b(S), tail(S), cf(std::max(S - 1, 0)), cb(std::max(S - 1, 0));
          std::vector<int> reps(S);
          bool ok = true;
          for (int s = 0; s < S && ok; ++s) {
            const int lo = c.plan.first_layer[s], hi = lo + c.plan.n_layers[s], lb = B / c.plan.replicas[s];
            reps[s] = c.plan.replicas[s];
            double pf = 0.0, pb = 0.0, g = 0.0;
            for (int l = lo; l < hi; ++l) {
              auto it = at.find({lb, l});
              if (it == at.end()) { ok = false; break; }
              pf += (double)it->second->fwd_ms; pb += (double)it->second->bwd_ms; g += (double)it->second->grad_bytes;
            }
            if (!ok) break;
            f[s] = (1.0 + o.self_cond_prob) * pf; b[s] = pb;
            tail[s] = g / (o.ar_gbps * 1e9) * 1e3 + o.ar_latency_ms;
            if (s) {
              const dp_layer_cost* r = at[{lb, lo - 1}];
              cf[s - 1] = (double)r->cf_bytes / (o.p2p_gbps * 1e9) * 1e3 + o.p2p_latency_ms;
              cb[s - 1] = (double)r->cb_bytes / (o.p2p_gbps * 1e9) * 1e3 + o.p2p_latency_ms;
            }
          }
          if (!ok) continue;
          std::vector<dp_bubble> bub(256);
          int nb = 0;
          double t_pipe = 0.0;
          int brc = dp_bubbles_1f1b(S, f.data(), b.data(), reps.data(), M, S > 1 ? cf.data() : nullptr, S > 1 ? cb.data() : nullptr, tail.data(),
                                    o.min_bubble_ms, bub.data(), (int)bub.size(), &nb, &t_pipe);
          if (brc == DP_EWORKSPACE) {
            bub.resize(nb);
            brc = dp_bubbles_1f1b(S, f.data(), b.data(), reps.data(), M, S > 1 ? cf.data() : nullptr, S > 1 ? cb.data() : nullptr, tail.data(),
                                  o.min_bubble_ms, bub.data(), (int)bub.size(), &nb, &t_pipe);
          }
          if (brc != DP_OK) return brc;
          // step 4: the non-trainable part into the bubbles
          std::vector<dp_fill> fills(1024);
          dp_fill_summary sum;
          int frc = dp_bubbles_fill(bub.data(), nb, rows, n_rows, o.dep_pairs, o.n_dep_pairs, group_batch, D, fills.data(), (int)fills.size(), &sum);
          if (frc == DP_EWORKSPACE) {
            fills.resize(sum.n_fills);
            frc = dp_bubbles_fill(bub.data(), nb, rows, n_rows, o.dep_pairs, o.n_dep_pairs, group_batch, D, fills.data(), (int)fills.size(), &sum);
          }
          if (frc != DP_OK) return frc;
          c.n_stages = S; c.n_micro_batches = M; c.group_size = D; c.micro_batch = B;
          c.pipeline_ms = t_pipe; c.leftover_ms = sum.leftover_ms; c.iteration_ms = t_pipe + sum.leftover_ms;
          c.bubble_ratio = sum.bubble_device_ms / (D * t_pipe);
          c.bubble_ratio_filled = (sum.bubble_device_ms - sum.filled_device_ms) / (D * c.iteration_ms);
          if (count < max_cands) {
            cands[count] = c;
            if (*best < 0 || c.iteration_ms < cands[*best].iteration_ms) *best = count;   // step 5
          } else rc = DP_EWORKSPACE;
          ++count;
        }
      }
    }
    *n_cands = count;
    if (count == 0) return set_error(DP_EUNSUPPORTED, "dp_schedule_search: no feasible combination of stages, micro-batches and group size");
    if (rc == DP_EWORKSPACE) return set_error(DP_EWORKSPACE, "dp_schedule_search: more candidates than rows to write them to");
  } catch (...) {
    return set_error(DP_EINVAL, "dp_schedule_search: out of host memory");
  }
  return rc;
}
