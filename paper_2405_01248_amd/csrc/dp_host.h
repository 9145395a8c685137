// Host-side helpers shared by the translation units that implement the C ABI: early-return macro,
// the bump planner that carves a caller-provided workspace, parameter tables, pointer checks.
#pragma once
#include "dp_errors.h"

#include <algorithm>
#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

#define DP_TRY(expr) do { int _e = (expr); if (_e != DP_OK) return _e; } while (0)

namespace dp {

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Bump planner over the caller's workspace; the same code computes sizes (base = nullptr)
// and pointers.
struct Plan {
  char* base; size_t off = 0;
  explicit Plan(void* b) : base((char*)b) {}
  void* take(size_t bytes) {
    void* p = base ? base + off : nullptr;
    off += align_up(bytes, 256);
    return p;
  }
};

struct ParamInfo { std::string name; int64_t rows, cols; };

inline int check_ptr(const void* p, const char* what, size_t align = 16) {
  if (!p) return set_errorf(DP_EINVAL, "%s is NULL", what);
  if ((uintptr_t)p % align) return set_errorf(DP_EALIGN, "%s is not %zu-byte aligned", what, align);
  return DP_OK;
}

inline float median(std::vector<float>& v) {
  std::sort(v.begin(), v.end());
  const size_t n = v.size();
  return n % 2 ? v[n / 2] : 0.5f * (v[n / 2 - 1] + v[n / 2]);
}

}  // namespace dp
