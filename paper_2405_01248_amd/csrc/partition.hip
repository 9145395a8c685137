// Backbone partitioner: the dynamic programme of Sec. 4.1 (Eq. 1-9) with the self-conditioning terms of
// Sec. 4.3 (Eq. 17-18), run on the host over cost-profile rows (dp_layer_cost, component 0) such as
// dp_stage_profile writes.  No device code: this file only rides in the same library.
//
// State (l, s, r, d): the first l layers in s stages on devices 1..d, the last stage replicated on the last
// r devices.  It keeps W = T_0, W_SC = T_0 under self-conditioning and Y = T_0^{S-C} of the best
// sub-partition found for it, "best" by the objective of the whole problem,
//   (M + 2S - 2) (p W_SC + (1 - p) W) + Y,
// with S the total stage count of the run; the programme is run once per S.
#include "../../include/dpipe.h"
#include "dp_errors.h"

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <map>
#include <vector>

namespace {

struct Terms { double t0, t0_sc, gap; bool ok; };

struct Problem {
  int L = 0, D = 0;
  const dp_partition_opts* o = nullptr;
  // per replication r = 1..D (index r - 1): terms of the stage [lo, hi) at local batch B / r
  std::vector<std::vector<Terms>> terms;     // [r - 1][lo * (L + 1) + hi]
  const Terms& at(int r, int lo, int hi) const { return terms[r - 1][(size_t)lo * (L + 1) + hi]; }
};

inline double bytes_ms(double bytes, double gbps) { return bytes / (gbps * 1e9) * 1e3; }

inline double objective(const dp_partition_opts& o, int S, double w, double w_sc, double y) {
  const double p = o.self_cond_prob;
  return (o.n_micro_batches + 2 * S - 2) * (p * w_sc + (1.0 - p) * w) + y;
}

struct State { double w, w_sc, y; int parent_l, parent_r; bool ok; };

}  // namespace

static int partition_solve_impl(const dp_layer_cost* rows, int n_rows, const dp_partition_opts* opts, dp_partition_plan* plan);

// No C++ exception crosses the C boundary: an allocation failure becomes an error code.
extern "C" int dp_partition_solve(const dp_layer_cost* rows, int n_rows, const dp_partition_opts* opts, dp_partition_plan* plan) {
  try {
    return partition_solve_impl(rows, n_rows, opts, plan);
  } catch (...) {
    return dp::set_error(DP_EINVAL, "dp_partition_solve: out of host memory");
  }
}

static int partition_solve_impl(const dp_layer_cost* rows, int n_rows, const dp_partition_opts* opts, dp_partition_plan* plan) {
  using dp::set_error;
  if (!rows || n_rows <= 0 || !opts || !plan) return set_error(DP_EINVAL, "dp_partition_solve: null argument");
  const dp_partition_opts& o = *opts;
  if (o.micro_batch <= 0 || o.n_micro_batches <= 0 || o.n_devices <= 0 || o.n_devices > DP_MAX_STAGES || o.max_stages < 0 || o.exact_stages < 0)
    return set_error(DP_EINVAL, "dp_partition_solve: micro_batch, n_micro_batches > 0; 1 <= n_devices <= DP_MAX_STAGES; max_stages, exact_stages >= 0");
  if (!(o.p2p_gbps > 0.0) || !(o.ar_gbps > 0.0) || o.p2p_latency_ms < 0.0 || o.ar_latency_ms < 0.0 || o.self_cond_prob < 0.0 ||
      o.self_cond_prob > 1.0)
    return set_error(DP_EINVAL, "dp_partition_solve: bandwidths > 0, latencies >= 0, 0 <= self_cond_prob <= 1");

  // ---- the profile: rows of component 0, one per (layer, batch); every batch size must cover layers 0..L-1
  std::map<int, std::vector<const dp_layer_cost*>> by_batch;
  int L = 0;
  for (int i = 0; i < n_rows; ++i)
    if (rows[i].component == 0) {
      if (rows[i].layer < 0 || rows[i].batch <= 0) return set_error(DP_EINVAL, "dp_partition_solve: bad layer or batch in a row");
      L = std::max(L, rows[i].layer + 1);
    }
  if (L == 0) return set_error(DP_EINVAL, "dp_partition_solve: no rows of component 0");
  if (L > 4096) return set_error(DP_EUNSUPPORTED, "dp_partition_solve: more than 4096 layers");
  for (int i = 0; i < n_rows; ++i) {
    if (rows[i].component != 0) continue;
    auto& v = by_batch[rows[i].batch];
    if (v.empty()) v.assign(L, nullptr);
    if (v[rows[i].layer]) return set_error(DP_EINVAL, "dp_partition_solve: duplicate (layer, batch) row");
    if (!(rows[i].fwd_ms >= 0.f) || !(rows[i].bwd_ms >= 0.f) || rows[i].cf_bytes < 0 || rows[i].cb_bytes < 0 || rows[i].grad_bytes < 0 ||
        rows[i].out_bytes < 0)
      return set_error(DP_EINVAL, "dp_partition_solve: negative or NaN cost in a row");
    v[rows[i].layer] = &rows[i];
  }
  for (auto& kv : by_batch)
    for (const dp_layer_cost* r : kv.second)
      if (!r) return set_error(DP_EINVAL, "dp_partition_solve: a batch size lacks rows for some layers");

  const int D = o.n_devices;
  const int s_max = std::min(std::min(L, D), o.max_stages > 0 ? o.max_stages : DP_MAX_STAGES);
  // what is allocated (stage terms: D x (L + 1)^2 entries; states: S x D^2 x L) and what is looped over (S^2 x D^3 x L^2 / 4)
  if ((double)s_max * D * D * L > 64e6 || (double)D * (L + 1) * (L + 1) > 8e6 || (double)s_max * s_max * D * D * D * L * L / 4.0 > 2e10)
    return set_error(DP_EUNSUPPORTED, "dp_partition_solve: problem too large (stages x devices^2 x layers > 64M, devices x layers^2 > 8M, or stages^2 x devices^3 x layers^2 > 8e10)");

  double tf = 0.0;                                        // T_F = O_L(B) / R_p2p + L_p2p   (Sec. 4.3)
  if (o.self_cond_prob > 0.0) {
    auto it = by_batch.find(o.micro_batch);
    if (it == by_batch.end()) return set_error(DP_EINVAL, "dp_partition_solve: self-conditioning needs rows at the micro-batch size (feedback transfer)");
    tf = bytes_ms((double)it->second[L - 1]->out_bytes, o.p2p_gbps) + o.p2p_latency_ms;
  }

  // ---- stage terms (Eq. 3-6, 17) for every layer range and replication
  Problem pb;
  pb.L = L; pb.D = D; pb.o = opts;
  pb.terms.assign(D, std::vector<Terms>((size_t)(L + 1) * (L + 1), Terms{0, 0, 0, false}));
  for (int r = 1; r <= D; ++r) {
    if (o.micro_batch % r) continue;
    auto it = by_batch.find(o.micro_batch / r);
    if (it == by_batch.end()) continue;
    const auto& lay = it->second;
    for (int lo = 0; lo < L; ++lo) {
      double pf = 0.0, pbk = 0.0, g = 0.0;
      double comm = 0.0, comm_sc = 0.0;
      if (lo > 0) {
        const double cf = (double)lay[lo - 1]->cf_bytes, cb = (double)lay[lo - 1]->cb_bytes;
        comm = bytes_ms(cf + cb, o.p2p_gbps) + 2 * o.p2p_latency_ms;
        comm_sc = bytes_ms(2 * cf + cb, o.p2p_gbps) + 3 * o.p2p_latency_ms;
      }
      for (int hi = lo + 1; hi <= L; ++hi) {
        pf += (double)lay[hi - 1]->fwd_ms; pbk += (double)lay[hi - 1]->bwd_ms; g += (double)lay[hi - 1]->grad_bytes;
        Terms& t = pb.terms[r - 1][(size_t)lo * (L + 1) + hi];
        t.t0 = std::max(pf + pbk, comm);                                   // Eq. 3
        t.t0_sc = std::max(2 * pf + pbk, comm_sc);                         // Eq. 17
        const double ts = bytes_ms(g, o.ar_gbps) + o.ar_latency_ms;        // Eq. 4
        t.gap = std::max(ts - pbk, 0.0);                                   // Eq. 5, 6 (clamped at zero)
        t.ok = true;
      }
    }
  }

  // ---- the programme, once per total stage count S
  const double inf = std::numeric_limits<double>::infinity();
  double best_val = inf;
  dp_partition_plan best;
  best.n_stages = 0;
  auto idx = [&](int s, int d, int r, int l) { return (((size_t)(s - 1) * (D + 1) + d) * (D + 1) + r) * (L + 1) + l; };
  std::vector<State> tab;
  for (int S = o.exact_stages > 0 ? o.exact_stages : 1; S <= (o.exact_stages > 0 ? std::min(o.exact_stages, s_max) : s_max); ++S) {
    tab.assign((size_t)S * (D + 1) * (D + 1) * (L + 1), State{0, 0, 0, -1, -1, false});
    for (int d = 1; d <= D; ++d)
      for (int l = 1; l <= L; ++l) {
        const Terms& t = pb.at(d, 0, l);
        if (t.ok) tab[idx(1, d, d, l)] = State{t.t0, t.t0_sc, t.gap, -1, -1, true};
      }
    for (int s = 2; s <= S; ++s)
      for (int d = s; d <= D; ++d)
        for (int r = 1; r <= d - (s - 1); ++r)
          for (int l_end = s; l_end <= L; ++l_end) {
            State pick{0, 0, 0, -1, -1, false};
            double pick_val = inf;
            for (int l = s - 1; l < l_end; ++l) {                          // Eq. 9: cut before the last stage
              const Terms& t = pb.at(r, l, l_end);
              if (!t.ok) continue;
              for (int rp = 1; rp <= d - r; ++rp) {                        // Eq. 9: replication of the stage before
                if (o.uniform_replication && rp != r) continue;
                const State& sub = tab[idx(s - 1, d - r, rp, l)];
                if (!sub.ok) continue;
                const double w = std::max(sub.w, t.t0), w_sc = std::max(sub.w_sc, t.t0_sc), y = std::max(sub.y, t.gap);   // Eq. 7, 8
                const double val = objective(o, S, w, w_sc, y);
                if (!pick.ok || val < pick_val) { pick = State{w, w_sc, y, l, rp, true}; pick_val = val; }
              }
            }
            if (pick.ok) tab[idx(s, d, r, l_end)] = pick;
          }
    for (int r = 1; r <= D; ++r) {                                         // Eq. 2
      const State& st = tab[idx(S, D, r, L)];
      if (!st.ok) continue;
      const double val = objective(o, S, st.w, st.w_sc, st.y) + o.self_cond_prob * tf;
      if (val < best_val) {
        best_val = val;
        best.n_stages = S;
        best.t0_ms = st.w; best.t0_sc_ms = st.w_sc; best.gap_ms = st.y; best.tf_ms = tf; best.t_max_ms = val;
        int s = S, d = D, rr = r, hi = L;
        while (s >= 1) {
          const State& cur = tab[idx(s, d, rr, hi)];
          const int lo = s > 1 ? cur.parent_l : 0;
          best.first_layer[s - 1] = lo; best.n_layers[s - 1] = hi - lo; best.replicas[s - 1] = rr;
          const int nd = d - rr, nr = cur.parent_r;
          hi = lo; d = nd; rr = nr; --s;
        }
      }
    }
  }
  if (best.n_stages == 0) return set_error(DP_EUNSUPPORTED, "dp_partition_solve: no feasible partition (micro_batch / replicas must be a profiled batch size)");
  for (int i = best.n_stages; i < DP_MAX_STAGES; ++i) best.first_layer[i] = best.n_layers[i] = best.replicas[i] = 0;
  *plan = best;
  return DP_OK;
}


// ------------------------------------------------------------------ two backbones, bidirectional pipelining (Sec. 4.2, Eq. 10-16)
namespace {

struct Rows {                                      // one backbone's profile: batch -> rows by layer
  std::map<int, std::vector<const dp_layer_cost*>> by_batch;
  int L = 0;
};

int collect_rows(const dp_layer_cost* rows, int n_rows, Rows& out, const char* who) {
  using dp::set_errorf;
  for (int i = 0; i < n_rows; ++i)
    if (rows[i].component == 0) {
      if (rows[i].layer < 0 || rows[i].batch <= 0) return set_errorf(DP_EINVAL, "%s: bad layer or batch in a row", who);
      out.L = std::max(out.L, rows[i].layer + 1);
    }
  if (out.L == 0) return set_errorf(DP_EINVAL, "%s: no rows of component 0", who);
  if (out.L > 256) return set_errorf(DP_EUNSUPPORTED, "%s: more than 256 layers", who);
  for (int i = 0; i < n_rows; ++i) {
    if (rows[i].component != 0) continue;
    auto& v = out.by_batch[rows[i].batch];
    if (v.empty()) v.assign(out.L, nullptr);
    if (v[rows[i].layer]) return set_errorf(DP_EINVAL, "%s: duplicate (layer, batch) row", who);
    if (!(rows[i].fwd_ms >= 0.f) || !(rows[i].bwd_ms >= 0.f) || rows[i].cf_bytes < 0 || rows[i].cb_bytes < 0 || rows[i].grad_bytes < 0)
      return set_errorf(DP_EINVAL, "%s: negative or NaN cost in a row", who);
    v[rows[i].layer] = &rows[i];
  }
  for (auto& kv : out.by_batch)
    for (const dp_layer_cost* r : kv.second)
      if (!r) return set_errorf(DP_EINVAL, "%s: a batch size lacks rows for some layers", who);
  return DP_OK;
}

struct PairTerms { double t0, gap; bool ok; };

// (T_0, T_0^{S-C}) of every stage [lo, hi) of one backbone at replication r, communication time doubled
void fill_bidir_terms(const Rows& R, const dp_partition_opts& o, int r, std::vector<PairTerms>& t) {
  const int L = R.L;
  t.assign((size_t)(L + 1) * (L + 1), PairTerms{0, 0, false});
  if (o.micro_batch % r) return;
  auto it = R.by_batch.find(o.micro_batch / r);
  if (it == R.by_batch.end()) return;
  const auto& lay = it->second;
  for (int lo = 0; lo < L; ++lo) {
    double pf = 0.0, pbk = 0.0, g = 0.0, comm = 0.0;
    if (lo > 0) comm = 2.0 * (bytes_ms((double)lay[lo - 1]->cf_bytes + (double)lay[lo - 1]->cb_bytes, o.p2p_gbps) + 2 * o.p2p_latency_ms);
    for (int hi = lo + 1; hi <= L; ++hi) {
      pf += (double)lay[hi - 1]->fwd_ms; pbk += (double)lay[hi - 1]->bwd_ms; g += (double)lay[hi - 1]->grad_bytes;
      PairTerms& x = t[(size_t)lo * (L + 1) + hi];
      x.t0 = std::max(pf + pbk, comm);
      x.gap = std::max(bytes_ms(g, o.ar_gbps) + o.ar_latency_ms - pbk, 0.0);
      x.ok = true;
    }
  }
}

struct BState { double w, y; int pd, pu, pr; bool ok; };

}  // namespace

extern "C" int dp_partition_solve_bidirectional(const dp_layer_cost* rows_down, int n_down, const dp_layer_cost* rows_up, int n_up,
                                                const dp_partition_opts* opts, dp_bidir_plan* plan) {
  using dp::set_error;
  if (!rows_down || n_down <= 0 || !rows_up || n_up <= 0 || !opts || !plan) return set_error(DP_EINVAL, "dp_partition_solve_bidirectional: null argument");
  const dp_partition_opts& o = *opts;
  if (o.micro_batch <= 0 || o.n_micro_batches <= 0 || o.n_devices <= 0 || o.n_devices > DP_MAX_STAGES || o.max_stages < 0 || o.exact_stages < 0)
    return set_error(DP_EINVAL, "dp_partition_solve_bidirectional: micro_batch, n_micro_batches > 0; 1 <= n_devices <= DP_MAX_STAGES; max_stages, exact_stages >= 0");
  if (!(o.p2p_gbps > 0.0) || !(o.ar_gbps > 0.0) || o.p2p_latency_ms < 0.0 || o.ar_latency_ms < 0.0)
    return set_error(DP_EINVAL, "dp_partition_solve_bidirectional: bandwidths > 0, latencies >= 0");
  if (o.self_cond_prob != 0.0) return set_error(DP_EUNSUPPORTED, "dp_partition_solve_bidirectional: self-conditioning is not combined with bidirectional pipelining");
  try {
    Rows Rd, Ru;
    if (int e = collect_rows(rows_down, n_down, Rd, "dp_partition_solve_bidirectional (down)")) return e;
    if (int e = collect_rows(rows_up, n_up, Ru, "dp_partition_solve_bidirectional (up)")) return e;
    const int Ld = Rd.L, Lu = Ru.L, D = o.n_devices;
    const int s_cap = std::min(std::min(std::min(Ld, Lu), D), o.max_stages > 0 ? o.max_stages : DP_MAX_STAGES);
    // work ~ S x D^3 x (Ld Lu)^2 / 4, memory ~ S x D^2 x Ld Lu states
    const double work = (double)s_cap * D * D * D * (double)Ld * Ld * Lu * Lu / 4.0, mem = (double)s_cap * (D + 1) * (D + 1) * (Ld + 1) * (Lu + 1);
    if (work > 4e9 || mem > 5e7) return set_error(DP_EUNSUPPORTED, "dp_partition_solve_bidirectional: problem too large (stages x devices^3 x (layers_down x layers_up)^2 > 1.6e10)");
    std::vector<std::vector<PairTerms>> td(D), tu(D);
    for (int r = 1; r <= D; ++r) { fill_bidir_terms(Rd, o, r, td[r - 1]); fill_bidir_terms(Ru, o, r, tu[r - 1]); }
    // the chain position holding down layers [d0, d1) and the up layers [u0, u1) counted from the up backbone's end
    auto pair = [&](int r, int d0, int d1, int u0, int u1, double& t0, double& gap) {
      const PairTerms& a = td[r - 1][(size_t)d0 * (Ld + 1) + d1];
      const PairTerms& b = tu[r - 1][(size_t)(Lu - u1) * (Lu + 1) + (Lu - u0)];
      if (!a.ok || !b.ok) return false;
      t0 = std::max(a.t0, b.t0); gap = std::max(a.gap, b.gap);
      return true;
    };
    const double inf = std::numeric_limits<double>::infinity();
    double best_val = inf;
    dp_bidir_plan best;
    best.n_stages = 0;
    std::vector<BState> tab;
    for (int S = o.exact_stages > 0 ? o.exact_stages : 1; S <= (o.exact_stages > 0 ? std::min(o.exact_stages, s_cap) : s_cap); ++S) {
      auto idx = [&](int s, int d, int r, int ld, int lu) { return ((((size_t)(s - 1) * (D + 1) + d) * (D + 1) + r) * (Ld + 1) + ld) * (Lu + 1) + lu; };
      auto obj = [&](double w, double y) { return (o.n_micro_batches + 2 * S - 2) * w + y; };
      tab.assign((size_t)S * (D + 1) * (D + 1) * (Ld + 1) * (Lu + 1), BState{0, 0, -1, -1, -1, false});
      for (int d = 1; d <= D; ++d)
        for (int ld = 1; ld <= Ld; ++ld)
          for (int lu = 1; lu <= Lu; ++lu) {
            double t0, gap;
            if (pair(d, 0, ld, 0, lu, t0, gap)) tab[idx(1, d, d, ld, lu)] = BState{t0, gap, -1, -1, -1, true};
          }
      for (int s = 2; s <= S; ++s)
        for (int d = s; d <= D; ++d)
          for (int r = 1; r <= d - (s - 1); ++r)
            for (int ld = s; ld <= Ld; ++ld)
              for (int lu = s; lu <= Lu; ++lu) {
                BState pick{0, 0, -1, -1, -1, false};
                double pick_val = inf;
                for (int pd = s - 1; pd < ld; ++pd)                       // Eq. 16
                  for (int pu = s - 1; pu < lu; ++pu) {
                    double t0, gap;
                    if (!pair(r, pd, ld, pu, lu, t0, gap)) continue;
                    for (int rp = 1; rp <= d - r; ++rp) {
                      if (o.uniform_replication && rp != r) continue;
                      const BState& sub = tab[idx(s - 1, d - r, rp, pd, pu)];
                      if (!sub.ok) continue;
                      const double w = std::max(sub.w, t0), y = std::max(sub.y, gap);   // Eq. 14, 15
                      const double val = obj(w, y);
                      if (!pick.ok || val < pick_val) { pick = BState{w, y, pd, pu, rp, true}; pick_val = val; }
                    }
                  }
                if (pick.ok) tab[idx(s, d, r, ld, lu)] = pick;
              }
      for (int r = 1; r <= D; ++r) {                                      // Eq. 13
        const BState& st = tab[idx(S, D, r, Ld, Lu)];
        if (!st.ok) continue;
        const double val = obj(st.w, st.y);
        if (val < best_val) {
          best_val = val;
          best.n_stages = S; best.t0_ms = st.w; best.gap_ms = st.y; best.t_max_ms = val;
          int s = S, d = D, rr = r, ld = Ld, lu = Lu;
          while (s >= 1) {
            const BState& cur = tab[idx(s, d, rr, ld, lu)];
            const int pd = s > 1 ? cur.pd : 0, pu = s > 1 ? cur.pu : 0;
            best.first_layer_down[s - 1] = pd; best.n_layers_down[s - 1] = ld - pd;
            best.first_layer_up[s - 1] = Lu - lu; best.n_layers_up[s - 1] = lu - pu;
            best.replicas[s - 1] = rr;
            const int nd = d - rr, nr = cur.pr;
            ld = pd; lu = pu; d = nd; rr = nr; --s;
          }
        }
      }
    }
    if (best.n_stages == 0) return set_error(DP_EUNSUPPORTED, "dp_partition_solve_bidirectional: no feasible partition (micro_batch / replicas must be a profiled batch size of both backbones)");
    for (int i = best.n_stages; i < DP_MAX_STAGES; ++i)
      best.first_layer_down[i] = best.n_layers_down[i] = best.first_layer_up[i] = best.n_layers_up[i] = best.replicas[i] = 0;
    *plan = best;
  } catch (...) {
    return set_error(DP_EINVAL, "dp_partition_solve_bidirectional: out of host memory");
  }
  return DP_OK;
}
