// Per-launch kernel timing records (measurement aid; not thread-safe by design: one
// measuring thread enables it, runs the path, and collects).
#include "dp_ktime.h"
#include "dp_errors.h"
#include <algorithm>
#include <vector>

namespace dp {

struct KRec { int kind, m, n, k; double flops, bytes; hipEvent_t e0, e1; hipStream_t s; };
static std::vector<KRec> g_recs;
static size_t g_used = 0;
static bool g_on = false;
static float g_overhead_ms = 0.f;   // elapsed time of an empty event pair, measured by the last dp_ktime_end

bool ktime_enabled() { return g_on; }

void ktime_open(int kind, double flops, double bytes, int m, int n, int k, hipStream_t s) {
  if (g_used >= g_recs.size()) return;
  KRec& r = g_recs[g_used];
  r.kind = kind; r.flops = flops; r.bytes = bytes; r.m = m; r.n = n; r.k = k; r.s = s;
  (void)hipEventRecord(r.e0, s);
}
void ktime_close(hipStream_t s) {
  if (g_used >= g_recs.size()) return;
  (void)hipEventRecord(g_recs[g_used].e1, s);
  ++g_used;
}

static void ktime_free() {
  for (auto& r : g_recs) { (void)hipEventDestroy(r.e0); (void)hipEventDestroy(r.e1); }
  g_recs.clear();
  g_used = 0;
  g_on = false;
}

}  // namespace dp

using namespace dp;

extern "C" int dp_ktime_begin(int max_records) {
  if (max_records <= 0 || max_records > (1 << 20)) return set_error(DP_EINVAL, "dp_ktime_begin: max_records out of range");
  ktime_free();
  g_recs.resize(max_records);
  for (int i = 0; i < max_records; ++i) {
    if (hipEventCreate(&g_recs[i].e0) != hipSuccess || hipEventCreate(&g_recs[i].e1) != hipSuccess) {
      g_recs.resize(i);
      ktime_free();
      return set_error(DP_EHIP, "hipEventCreate failed");
    }
  }
  g_on = true;
  return DP_OK;
}

extern "C" int dp_ktime_end(dp_kernel_time* out, int max, int* n) {
  if (!out || !n || max < 0) return set_error(DP_EINVAL, "dp_ktime_end: bad argument");
  g_on = false;
  if (hipDeviceSynchronize() != hipSuccess) { ktime_free(); return set_error(DP_EHIP, "hipDeviceSynchronize failed"); }
  // What a pair of events reads by itself: empty pairs on the stream of the first record, from the unused
  // tail of the pool.  Reported beside the records, not taken off them: a record's two events bracket one
  // dispatch gap fewer than an empty pair suggests, so subtracting it would understate the durations.
  g_overhead_ms = 0.f;
  {
    const size_t spare = std::min<size_t>(g_recs.size() - g_used, 33);
    if (g_used > 0 && spare >= 3) {
      hipStream_t cs = g_recs[0].s;
      for (size_t i = 0; i < spare; ++i) {
        (void)hipEventRecord(g_recs[g_used + i].e0, cs);
        (void)hipEventRecord(g_recs[g_used + i].e1, cs);
      }
      if (hipStreamSynchronize(cs) == hipSuccess) {
        std::vector<float> v;
        for (size_t i = 0; i < spare; ++i) {
          float ms = 0.f;
          if (hipEventElapsedTime(&ms, g_recs[g_used + i].e0, g_recs[g_used + i].e1) == hipSuccess) v.push_back(ms);
        }
        if (!v.empty()) { std::sort(v.begin(), v.end()); g_overhead_ms = v[v.size() / 2]; }
      }
    }
  }
  int cnt = 0;
  for (size_t i = 0; i < g_used && cnt < max; ++i) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, g_recs[i].e0, g_recs[i].e1) != hipSuccess) continue;
    out[cnt++] = dp_kernel_time{g_recs[i].kind, g_recs[i].m, g_recs[i].n, g_recs[i].k, ms, g_recs[i].flops, g_recs[i].bytes};
  }
  *n = cnt;
  ktime_free();
  return DP_OK;
}

extern "C" float dp_ktime_event_overhead_ms(void) { return g_overhead_ms; }
