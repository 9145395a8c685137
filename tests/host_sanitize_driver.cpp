// Driver for the sanitizer build of the library's host-only code (partitioner, bidirectional partitioner,
// schedule simulation, bubble filling, hyper-parameter search): seeded random problems, error paths and
// sizes at the guards, run under AddressSanitizer and UndefinedBehaviorSanitizer.  It checks only cheap
// invariants itself (the numerical agreement with the oracle is the other tests' job); its purpose is
// that every path runs under the sanitizers.  Exit code 0 = nothing was reported.
#include "../include/dpipe.h"

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

static uint64_t g_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd() { g_state = g_state * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(g_state >> 33); }
static int rint_(int lo, int hi) { return lo + (int)(rnd() % (uint32_t)(hi - lo + 1)); }
static double runi(double lo, double hi) { return lo + (hi - lo) * (rnd() / 2147483648.0); }

#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "check failed at line %d: %s (%s)\n", __LINE__, #cond, dp_last_error()); return 1; } } while (0)

static std::vector<dp_layer_cost> backbone_rows(int L, const std::vector<int>& batches) {
  std::vector<dp_layer_cost> rows;
  for (int l = 0; l < L; ++l) {
    const double f = runi(0.1, 2.0), b = runi(0.2, 4.0);
    const int64_t act = (int64_t)runi(1e5, 4e6), g = (int64_t)runi(1e6, 3e7);
    for (int bs : batches) rows.push_back(dp_layer_cost{0, l, bs, (float)(f * bs), (float)(b * bs), act * bs, act * bs, act * bs, g});
  }
  return rows;
}

static void add_component(std::vector<dp_layer_cost>& rows, int id, int nl) {
  for (int l = 0; l < nl; ++l) {
    const double t = runi(0.05, 3.0);
    for (int bs : {4, 16, 64}) rows.push_back(dp_layer_cost{id, l, bs, (float)(t * (0.4 + 0.6 * bs / 16.0)), 0.f, 0, 0, 0, 0});
  }
}

int main() {
  const std::vector<int> batches = {1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 64};
  int solved = 0;
  for (int it = 0; it < 60; ++it) {
    const int L = rint_(1, 9), D = rint_(1, 8);
    std::vector<dp_layer_cost> rows = backbone_rows(L, batches);
    dp_partition_opts o{};
    o.micro_batch = (int[]){8, 12, 16, 24}[rnd() % 4]; o.n_micro_batches = rint_(1, 16); o.n_devices = D; o.max_stages = (int[]){0, 0, 2, 3}[rnd() % 4];
    o.uniform_replication = rnd() % 3 == 0; o.p2p_gbps = 25.0; o.p2p_latency_ms = 0.02; o.ar_gbps = 50.0; o.ar_latency_ms = 0.1;
    o.self_cond_prob = (double[]){0.0, 0.5, 1.0}[rnd() % 3]; o.exact_stages = (int[]){0, 0, 0, 1, 2}[rnd() % 5];
    dp_partition_plan plan;
    int rc = dp_partition_solve(rows.data(), (int)rows.size(), &o, &plan);
    CHECK(rc == DP_OK || rc == DP_EUNSUPPORTED);
    if (rc == DP_OK) {
      int layers = 0, devs = 0;
      for (int s = 0; s < plan.n_stages; ++s) { layers += plan.n_layers[s]; devs += plan.replicas[s]; }
      CHECK(layers == L && devs == D && plan.t_max_ms > 0.0);
      ++solved;
    }
    // two backbones
    std::vector<dp_layer_cost> up = backbone_rows(rint_(1, 6), batches);
    dp_partition_opts ob = o; ob.self_cond_prob = 0.0;
    dp_bidir_plan bp;
    rc = dp_partition_solve_bidirectional(rows.data(), (int)rows.size(), up.data(), (int)up.size(), &ob, &bp);
    CHECK(rc == DP_OK || rc == DP_EUNSUPPORTED);
    // schedule simulation and filling, also with outputs that are too small
    const int S = rint_(1, 6), M = rint_(1, 9);
    std::vector<double> f(S), b(S), tail(S), cf(S), cb(S);
    std::vector<int> reps(S);
    for (int s = 0; s < S; ++s) { f[s] = runi(0.5, 5); b[s] = runi(1, 9); tail[s] = runi(0, 1); cf[s] = runi(0, 0.5); cb[s] = runi(0, 0.5); reps[s] = rint_(1, 3); }
    std::vector<dp_bubble> bub(512);
    int nb = 0; double t_iter = 0;
    rc = dp_bubbles_1f1b(S, f.data(), b.data(), reps.data(), M, cf.data(), cb.data(), tail.data(), 0.0, bub.data(), (int)bub.size(), &nb, &t_iter);
    CHECK(rc == DP_OK && t_iter > 0.0);
    int nb0 = 0;
    rc = dp_bubbles_1f1b(S, f.data(), b.data(), reps.data(), M, nullptr, nullptr, nullptr, 0.0, nullptr, 0, &nb0, nullptr);
    CHECK(rc == (nb0 > 0 ? DP_EWORKSPACE : DP_OK));
    add_component(rows, 1, rint_(1, 5));
    if (rnd() % 2) add_component(rows, 2, rint_(1, 4));
    const int dep[2] = {2, 1};
    const bool two = rows.back().component == 2;
    std::vector<dp_fill> fills(2048);
    dp_fill_summary sum;
    int devs = 0; for (int r : reps) devs += r;
    rc = dp_bubbles_fill(bub.data(), nb, rows.data(), (int)rows.size(), two ? dep : nullptr, two ? 1 : 0, 64 * rint_(1, 4), devs, fills.data(), (int)fills.size(), &sum);
    CHECK(rc == DP_OK && sum.filled_device_ms <= sum.bubble_device_ms * (1 + 1e-9) + 1e-9);
    rc = dp_bubbles_fill(bub.data(), nb, rows.data(), (int)rows.size(), nullptr, 0, 64, devs, nullptr, 0, &sum);
    CHECK(rc == (sum.n_fills > 0 ? DP_EWORKSPACE : DP_OK));
    // the search over (S, M, D)
    const int gs[] = {1, 2, 4, 8, 3}, ms[] = {1, 2, 4, 8};
    dp_search_opts so{};
    so.world_size = 8; so.training_batch = 8 * (int[]){4, 8, 16}[rnd() % 3]; so.group_sizes = gs; so.n_group_sizes = 5; so.micro_batch_counts = ms;
    so.n_micro_batch_counts = 4; so.max_stages = (int[]){0, 2}[rnd() % 2]; so.uniform_replication = 1; so.p2p_gbps = 50; so.p2p_latency_ms = 0.01;
    so.ar_gbps = 100; so.ar_latency_ms = 0.05; so.self_cond_prob = (double[]){0.0, 0.5}[rnd() % 2]; so.min_bubble_ms = 0.0;
    so.dep_pairs = two ? dep : nullptr; so.n_dep_pairs = two ? 1 : 0;
    std::vector<dp_search_candidate> cands(512);
    int nc = 0, best = -1;
    rc = dp_schedule_search(rows.data(), (int)rows.size(), &so, cands.data(), (int)cands.size(), &nc, &best);
    CHECK(rc == DP_OK || rc == DP_EUNSUPPORTED);
    if (rc == DP_OK) {
      CHECK(best >= 0 && best < nc);
      for (int i = 0; i < nc; ++i) CHECK(cands[best].iteration_ms <= cands[i].iteration_ms);
      rc = dp_schedule_search(rows.data(), (int)rows.size(), &so, cands.data(), 1, &nc, &best);
      CHECK(rc == (nc > 1 ? DP_EWORKSPACE : DP_OK));
    }
  }
  CHECK(solved > 20);
  // ---- sizes at the guards: refused at once when too large, solved when just inside
  {
    dp_partition_opts o{};
    o.micro_batch = 8; o.n_micro_batches = 4; o.n_devices = 8; o.p2p_gbps = 25; o.ar_gbps = 50;
    dp_partition_plan plan;
    std::vector<dp_layer_cost> big = backbone_rows(4096, {8});
    CHECK(dp_partition_solve(big.data(), (int)big.size(), &o, &plan) == DP_EUNSUPPORTED);
    std::vector<dp_layer_cost> over = backbone_rows(4097, {8});
    CHECK(dp_partition_solve(over.data(), (int)over.size(), &o, &plan) == DP_EUNSUPPORTED);
    std::vector<dp_layer_cost> mid = backbone_rows(300, {8, 4, 2, 1});
    o.max_stages = 3;
    CHECK(dp_partition_solve(mid.data(), (int)mid.size(), &o, &plan) == DP_OK && plan.n_stages >= 1);
    std::vector<dp_layer_cost> a = backbone_rows(200, {8}), b2 = backbone_rows(200, {8});
    dp_bidir_plan bp;
    o.max_stages = 0;
    CHECK(dp_partition_solve_bidirectional(a.data(), (int)a.size(), b2.data(), (int)b2.size(), &o, &bp) == DP_EUNSUPPORTED);
    std::vector<dp_layer_cost> c257 = backbone_rows(257, {8});
    CHECK(dp_partition_solve_bidirectional(c257.data(), (int)c257.size(), a.data(), (int)a.size(), &o, &bp) == DP_EUNSUPPORTED);
  }
  // ---- a bubble with more whole-batch packings than the filler enumerates: 8 components of 40 very short layers
  {
    std::vector<dp_layer_cost> rows;
    for (int id = 1; id <= 8; ++id)
      for (int l = 0; l < 40; ++l) rows.push_back(dp_layer_cost{id, l, 4, 0.001f, 0.f, 0, 0, 0, 0});
    dp_bubble one{0.0, 10.0, 1, 1};
    std::vector<dp_fill> fills(512);
    dp_fill_summary sum;
    CHECK(dp_bubbles_fill(&one, 1, rows.data(), (int)rows.size(), nullptr, 0, 4, 1, fills.data(), (int)fills.size(), &sum) == DP_EUNSUPPORTED);
    // nine components are refused before anything is enumerated
    for (int l = 0; l < 2; ++l) rows.push_back(dp_layer_cost{9, l, 4, 0.001f, 0.f, 0, 0, 0, 0});
    CHECK(dp_bubbles_fill(&one, 1, rows.data(), (int)rows.size(), nullptr, 0, 4, 1, fills.data(), (int)fills.size(), &sum) == DP_EUNSUPPORTED);
  }
  // ---- null and nonsense arguments
  {
    dp_partition_plan plan; dp_partition_opts o{};
    CHECK(dp_partition_solve(nullptr, 0, &o, &plan) == DP_EINVAL);
    int n = 0;
    CHECK(dp_bubbles_1f1b(0, nullptr, nullptr, nullptr, 1, nullptr, nullptr, nullptr, 0.0, nullptr, 0, &n, nullptr) == DP_EINVAL);
    dp_fill_summary sum;
    CHECK(dp_bubbles_fill(nullptr, 0, nullptr, 0, nullptr, 0, 1, 1, nullptr, 0, &sum) == DP_EINVAL);
    CHECK(dp_schedule_search(nullptr, 0, nullptr, nullptr, 0, nullptr, nullptr) == DP_EINVAL);
    CHECK(dp_last_error()[0] != 0);
  }
  printf("host sanitizer driver: ok (%d partitions solved)\n", solved);
  return 0;
}
