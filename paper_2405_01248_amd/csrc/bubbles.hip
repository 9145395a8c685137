// Pipeline bubbles and their filling with the frozen components (Sec. 5, Algorithms 1 and 2), host code.
//
// dp_bubbles_1f1b simulates one iteration of the FIFO-1F1B schedule from per-stage forward / backward times
// and cuts the idle time into bubbles (start, end, idle devices).  dp_bubbles_fill walks the bubbles in
// chronological order; for each it lists the whole-batch candidates of the ready components (Algorithm 2),
// extends every candidate by at most one partial-batch layer with the largest regular sample count that
// fits (Algorithm 1), and keeps the longest.  The candidates are walked by an odometer over prefix-time tables.  A layer begun on part of the batch stays the first ready layer
// of its component and counts as a whole-batch layer on the remaining samples.  No device code here.
#include "../../include/dpipe.h"
#include "dp_errors.h"

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <map>
#include <set>
#include <vector>

namespace {

using dp::set_error;

struct Op { char kind; int mb; };
struct Busy { double start, end; };

// stage s of S: min(S - 1 - s, M) warm-up forwards, then one forward / one backward alternately, then the
// remaining backwards; micro-batches in order
std::vector<Op> order_1f1b(int s, int S, int M) {
  const int warm = std::min(S - 1 - s, M);
  std::vector<Op> ops;
  for (int m = 0; m < warm; ++m) ops.push_back({'F', m});
  for (int i = 0; i < M - warm; ++i) { ops.push_back({'F', warm + i}); ops.push_back({'B', i}); }
  for (int m = M - warm; m < M; ++m) ops.push_back({'B', m});
  return ops;
}

const int kRegular[] = {4, 8, 12, 16, 24, 32, 48, 64, 96};   // regular local batch sizes of a partial-batch layer

struct Comp {
  int id = 0, n_layers = 0;
  std::vector<int> sizes;                       // profiled local batch sizes, ascending
  std::vector<std::vector<double>> ms;          // [size index][layer]
  std::vector<int> deps;                        // component indices
};

double layer_time(const Comp& c, int layer, int b) {
  const auto it = std::lower_bound(c.sizes.begin(), c.sizes.end(), b);
  if (it != c.sizes.end() && *it == b) return c.ms[it - c.sizes.begin()][layer];
  if (it == c.sizes.begin()) return c.ms[0][layer];
  if (it == c.sizes.end()) return c.ms.back()[layer] * b / c.sizes.back();
  const int hi = (int)(it - c.sizes.begin()), lo = hi - 1;
  const double w = (double)(b - c.sizes[lo]) / (c.sizes[hi] - c.sizes[lo]);
  return c.ms[lo][layer] * (1 - w) + c.ms[hi][layer] * w;
}

struct State { int batch; std::vector<int> u, rem; };

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// time of the j-th unfinished layer of component i as a whole-batch layer on d devices
double full_time(const std::vector<Comp>& cs, const State& st, int i, int j, int d) {
  const int n = j == 0 ? st.rem[i] : st.batch;
  return layer_time(cs[i], st.u[i] + j, ceil_div(n, d));
}

// Whole-batch packings of a bubble, the candidate set of Algorithm 2: the layer counts (k_0 .. k_{n-1}) of the
// ready components whose summed whole-batch time fits the bubble, every component before the last one walked from
// its largest feasible count down to zero (for the time its predecessors leave) and the last one always at its
// largest count.  Instead of recursing, an odometer runs over per-component tables of prefix times: digit x counts
// layers of component x; after a visit the right-most non-zero digit (the last one excepted) is decreased and the
// digits to its right are reset to their maxima for the new remainder -- the same order as the recursive listing,
// which matters because the first of several equally long candidates is kept.
struct PrefixTimes { std::vector<double> t; };     // t[k] = time of the component's first k unfinished layers, whole batch

std::vector<PrefixTimes> prefix_times(const std::vector<Comp>& cs, const State& st, const std::vector<int>& ready, int d) {
  std::vector<PrefixTimes> out(ready.size());
  for (size_t x = 0; x < ready.size(); ++x) {
    const int i = ready[x], left = cs[i].n_layers - st.u[i];
    out[x].t.assign(1, 0.0);
    for (int j = 0; j < left; ++j) out[x].t.push_back(out[x].t.back() + full_time(cs, st, i, j, d));
  }
  return out;
}

// largest k whose prefix time fits the budget (prefix times are non-decreasing)
inline int largest_fit(const PrefixTimes& p, double budget) {
  int k = 0;
  while (k + 1 < (int)p.t.size() && p.t[k + 1] <= budget) ++k;
  return k;
}

constexpr long kMaxPackings = 1000000;   // a bubble with more candidates than this is refused, not enumerated

// Calls visit(k) for every packing; false if there are more than kMaxPackings.
template <class Visit>
bool for_each_packing(const std::vector<PrefixTimes>& tab, double t_b, Visit visit) {
  const int n = (int)tab.size();
  std::vector<int> k(n, 0);
  std::vector<double> budget(n, 0.0);
  budget[0] = t_b;
  k[0] = largest_fit(tab[0], t_b);
  long count = 0;
  for (int from = 0;;) {
    for (int x = from; x + 1 < n; ++x) {
      budget[x + 1] = budget[x] - tab[x].t[k[x]];
      k[x + 1] = largest_fit(tab[x + 1], budget[x + 1]);
    }
    if (++count > kMaxPackings) return false;
    visit(k);
    int x = n - 2;
    while (x >= 0 && k[x] == 0) --x;
    if (x < 0) return true;
    --k[x];
    from = x;
  }
}

struct Pick { std::vector<int> k; int ph = -1, player = -1, pb = 0; double t = -1.0; bool ok = false; bool too_many = false; };

// Algorithm 1: every packing, alone or extended by one partial-batch layer (the next layer of one ready component
// on the largest regular sample count that still fits); the candidate that runs longest wins, the first on ties.
Pick fill_one(const std::vector<Comp>& cs, const State& st, const std::vector<int>& ready, double t_b, int d) {
  const std::vector<PrefixTimes> tab = prefix_times(cs, st, ready, d);
  Pick best;
  const bool all = for_each_packing(tab, t_b, [&](const std::vector<int>& k) {
    double t_full = 0.0;
    for (size_t x = 0; x < ready.size(); ++x)
      for (int j = 0; j < k[x]; ++j) t_full += full_time(cs, st, ready[x], j, d);
    if (!best.ok || t_full > best.t) { best.k = k; best.ph = -1; best.player = -1; best.pb = 0; best.t = t_full; best.ok = true; }
    for (size_t x = 0; x < ready.size(); ++x) {
      const int h = ready[x], layer = st.u[h] + k[x];
      if (layer >= cs[h].n_layers) continue;
      const int left = k[x] == 0 ? st.rem[h] : st.batch;
      int b_best = 0;
      for (int r : kRegular) {
        const int b = r * d;
        if (b < left && t_full + layer_time(cs[h], layer, r) <= t_b) b_best = std::max(b_best, b);
      }
      if (!b_best) continue;
      const double t = t_full + layer_time(cs[h], layer, b_best / d);
      if (t > best.t) { best.k = k; best.ph = h; best.player = layer; best.pb = b_best; best.t = t; }
    }
  });
  best.too_many = !all;
  return best;
}

}  // namespace

static int bubbles_1f1b_impl(int n_stages, const double* fwd_ms, const double* bwd_ms, const int* replicas, int n_micro_batches,
                               const double* comm_fwd_ms, const double* comm_bwd_ms, const double* tail_ms, double min_ms,
                               dp_bubble* out, int max_out, int* n_out, double* iteration_ms) {
  if (!fwd_ms || !bwd_ms || !replicas || !n_out || (max_out > 0 && !out)) return set_error(DP_EINVAL, "dp_bubbles_1f1b: null argument");
  const int S = n_stages, M = n_micro_batches;
  if (S < 1 || S > DP_MAX_STAGES || M < 1 || max_out < 0 || !(min_ms >= 0.0)) return set_error(DP_EINVAL, "dp_bubbles_1f1b: 1 <= n_stages <= DP_MAX_STAGES, n_micro_batches >= 1, min_ms >= 0");
  for (int s = 0; s < S; ++s) {
    if (!(fwd_ms[s] >= 0.0) || !(bwd_ms[s] >= 0.0) || replicas[s] < 1 || (tail_ms && !(tail_ms[s] >= 0.0)))
      return set_error(DP_EINVAL, "dp_bubbles_1f1b: times >= 0 and replicas >= 1");
    if (s + 1 < S && ((comm_fwd_ms && !(comm_fwd_ms[s] >= 0.0)) || (comm_bwd_ms && !(comm_bwd_ms[s] >= 0.0))))
      return set_error(DP_EINVAL, "dp_bubbles_1f1b: transfer times >= 0");
  }
  std::vector<std::vector<Op>> orders(S);
  for (int s = 0; s < S; ++s) orders[s] = order_1f1b(s, S, M);
  std::vector<size_t> pos(S, 0);
  std::vector<double> free_at(S, 0.0);
  // done[kind][s][m] = end time, < 0 while not run
  std::vector<std::vector<double>> done_f(S, std::vector<double>(M, -1.0)), done_b(S, std::vector<double>(M, -1.0));
  std::vector<std::vector<Busy>> busy(S);
  bool progress = true;
  while (progress) {
    progress = false;
    for (int s = 0; s < S; ++s)
      while (pos[s] < orders[s].size()) {
        const Op op = orders[s][pos[s]];
        double ready;
        if (op.kind == 'F') {
          if (s == 0) ready = 0.0;
          else if (done_f[s - 1][op.mb] >= 0.0) ready = done_f[s - 1][op.mb] + (comm_fwd_ms ? comm_fwd_ms[s - 1] : 0.0);
          else break;
        } else if (s == S - 1) {
          if (done_f[s][op.mb] < 0.0) break;
          ready = done_f[s][op.mb];
        } else {
          if (done_b[s + 1][op.mb] < 0.0) break;
          ready = done_b[s + 1][op.mb] + (comm_bwd_ms ? comm_bwd_ms[s] : 0.0);
        }
        const double start = std::max(free_at[s], ready), end = start + (op.kind == 'F' ? fwd_ms[s] : bwd_ms[s]);
        busy[s].push_back({start, end});
        (op.kind == 'F' ? done_f : done_b)[s][op.mb] = end;
        free_at[s] = end;
        ++pos[s];
        progress = true;
      }
  }
  for (int s = 0; s < S; ++s)
    if (pos[s] != orders[s].size()) return set_error(DP_EINVAL, "dp_bubbles_1f1b: schedule did not complete");
  if (tail_ms)
    for (int s = 0; s < S; ++s)
      if (tail_ms[s] > 0.0) { busy[s].push_back({free_at[s], free_at[s] + tail_ms[s]}); free_at[s] += tail_ms[s]; }
  const double t_end = *std::max_element(free_at.begin(), free_at.end());
  if (iteration_ms) *iteration_ms = t_end;

  // maximal spans with a constant, non-empty set of idle stages
  std::set<double> cutset = {0.0, t_end};
  for (int s = 0; s < S; ++s)
    for (const Busy& b : busy[s]) { cutset.insert(b.start); cutset.insert(b.end); }
  const std::vector<double> cuts(cutset.begin(), cutset.end());
  std::vector<dp_bubble> all;
  for (size_t c = 0; c + 1 < cuts.size(); ++c) {
    const double a = cuts[c], b = cuts[c + 1], mid = 0.5 * (a + b);
    uint64_t mask = 0;
    int dev = 0;
    for (int s = 0; s < S; ++s) {
      bool is_busy = false;
      for (const Busy& x : busy[s])
        if (x.start <= mid && mid < x.end) { is_busy = true; break; }
      if (!is_busy) { mask |= 1ull << s; dev += replicas[s]; }
    }
    if (!mask) continue;
    if (!all.empty() && all.back().stage_mask == mask && all.back().end_ms == a) all.back().end_ms = b;
    else all.push_back(dp_bubble{a, b, dev, mask});
  }
  int n = 0;
  for (const dp_bubble& b : all)
    if (b.end_ms - b.start_ms >= min_ms) {
      if (n < max_out) out[n] = b;
      ++n;
    }
  *n_out = n;
  if (n > max_out) return set_error(DP_EWORKSPACE, "dp_bubbles_1f1b: more bubbles than max_out (n_out holds the count)");
  return DP_OK;
}

static int bubbles_fill_impl(const dp_bubble* bubbles, int n_bubbles, const dp_layer_cost* rows, int n_rows, const int* dep_pairs,
                               int n_dep_pairs, int batch, int n_devices, dp_fill* fills, int max_fills, dp_fill_summary* summary) {
  if ((n_bubbles > 0 && !bubbles) || !rows || n_rows <= 0 || !summary || (max_fills > 0 && !fills) || (n_dep_pairs > 0 && !dep_pairs))
    return set_error(DP_EINVAL, "dp_bubbles_fill: null argument");
  if (n_bubbles < 0 || batch < 1 || n_devices < 1 || max_fills < 0 || n_dep_pairs < 0) return set_error(DP_EINVAL, "dp_bubbles_fill: bad size");

  // ---- components: rows with component >= 1, ascending id; every profiled batch size must cover layers 0..L-1
  std::map<int, std::map<int, std::map<int, double>>> tab;     // id -> batch -> layer -> ms
  for (int i = 0; i < n_rows; ++i) {
    const dp_layer_cost& r = rows[i];
    if (r.component < 1) continue;
    if (r.layer < 0 || r.batch < 1 || !(r.fwd_ms >= 0.f)) return set_error(DP_EINVAL, "dp_bubbles_fill: bad layer, batch or time in a row");
    if (!tab[r.component][r.batch].emplace(r.layer, (double)r.fwd_ms).second) return set_error(DP_EINVAL, "dp_bubbles_fill: duplicate (component, layer, batch) row");
  }
  if (tab.empty()) return set_error(DP_EINVAL, "dp_bubbles_fill: no rows of a non-trainable component (component >= 1)");
  if (tab.size() > 8) return set_error(DP_EUNSUPPORTED, "dp_bubbles_fill: more than 8 components");
  std::vector<Comp> cs;
  std::map<int, int> index_of;
  for (const auto& kv : tab) {
    Comp c;
    c.id = kv.first;
    for (const auto& bl : kv.second) c.n_layers = std::max(c.n_layers, bl.second.rbegin()->first + 1);
    for (const auto& bl : kv.second) {
      if ((int)bl.second.size() != c.n_layers) return set_error(DP_EINVAL, "dp_bubbles_fill: a batch size lacks rows for some layers");
      c.sizes.push_back(bl.first);
      std::vector<double> v;
      for (const auto& lm : bl.second) v.push_back(lm.second);
      c.ms.push_back(v);
    }
    index_of[c.id] = (int)cs.size();
    cs.push_back(c);
  }
  for (int i = 0; i < n_dep_pairs; ++i) {
    const auto a = index_of.find(dep_pairs[2 * i]), b = index_of.find(dep_pairs[2 * i + 1]);
    if (a == index_of.end() || b == index_of.end() || a->second == b->second) return set_error(DP_EINVAL, "dp_bubbles_fill: dependency names an unknown component or itself");
    cs[a->second].deps.push_back(b->second);
  }
  for (int i = 0; i < n_bubbles; ++i) {
    if (!(bubbles[i].end_ms >= bubbles[i].start_ms) || bubbles[i].n_devices < 1) return set_error(DP_EINVAL, "dp_bubbles_fill: bad bubble");
    if (i && bubbles[i].start_ms < bubbles[i - 1].start_ms) return set_error(DP_EINVAL, "dp_bubbles_fill: bubbles must be in chronological order");
  }

  State st{batch, std::vector<int>(cs.size(), 0), std::vector<int>(cs.size(), batch)};
  dp_fill_summary sum{0.0, 0.0, 0.0, 0};
  int n = 0;
  auto emit = [&](const dp_fill& f) { if (n < max_fills) fills[n] = f; ++n; };
  for (int bi = 0; bi < n_bubbles; ++bi) {
    const dp_bubble& bub = bubbles[bi];
    const double len = bub.end_ms - bub.start_ms;
    sum.bubble_device_ms += len * bub.n_devices;
    std::vector<int> ready;
    for (size_t i = 0; i < cs.size(); ++i) {
      if (st.u[i] >= cs[i].n_layers) continue;
      bool ok = true;
      for (int j : cs[i].deps) ok = ok && st.u[j] >= cs[j].n_layers;
      if (ok) ready.push_back((int)i);
    }
    if (ready.empty()) continue;
    const Pick p = fill_one(cs, st, ready, len, bub.n_devices);
    if (p.too_many) return set_error(DP_EUNSUPPORTED, "dp_bubbles_fill: a bubble has more than a million whole-batch packings");
    if (!p.ok || !(p.t > 0.0)) continue;
    for (size_t x = 0; x < ready.size(); ++x) {
      const int i = ready[x];
      if (!p.k[x]) continue;
      emit(dp_fill{bi, cs[i].id, st.u[i], p.k[x], st.rem[i], 0, p.t});
      st.u[i] += p.k[x];
      st.rem[i] = batch;
    }
    if (p.ph >= 0) {
      emit(dp_fill{bi, cs[p.ph].id, p.player, 1, p.pb, 1, p.t});
      st.rem[p.ph] -= p.pb;
    }
    sum.filled_device_ms += p.t * bub.n_devices;
  }
  for (size_t i = 0; i < cs.size(); ++i)
    for (int j = 0; j < cs[i].n_layers - st.u[i]; ++j) sum.leftover_ms += full_time(cs, st, (int)i, j, n_devices);
  sum.n_fills = n;
  *summary = sum;
  if (n > max_fills) return set_error(DP_EWORKSPACE, "dp_bubbles_fill: more fill rows than max_fills (summary.n_fills holds the count)");
  return DP_OK;
}


// No C++ exception crosses the C boundary: an allocation failure becomes an error code.
extern "C" int dp_bubbles_1f1b(int n_stages, const double* fwd_ms, const double* bwd_ms, const int* replicas, int n_micro_batches,
                               const double* comm_fwd_ms, const double* comm_bwd_ms, const double* tail_ms, double min_ms, dp_bubble* out,
                               int max_out, int* n_out, double* iteration_ms) {
  try {
    return bubbles_1f1b_impl(n_stages, fwd_ms, bwd_ms, replicas, n_micro_batches, comm_fwd_ms, comm_bwd_ms, tail_ms, min_ms, out, max_out, n_out,
                             iteration_ms);
  } catch (...) {
    return set_error(DP_EINVAL, "dp_bubbles_1f1b: out of host memory");
  }
}

extern "C" int dp_bubbles_fill(const dp_bubble* bubbles, int n_bubbles, const dp_layer_cost* rows, int n_rows, const int* dep_pairs,
                               int n_dep_pairs, int batch, int n_devices, dp_fill* fills, int max_fills, dp_fill_summary* summary) {
  try {
    return bubbles_fill_impl(bubbles, n_bubbles, rows, n_rows, dep_pairs, n_dep_pairs, batch, n_devices, fills, max_fills, summary);
  } catch (...) {
    return set_error(DP_EINVAL, "dp_bubbles_fill: out of host memory");
  }
}
