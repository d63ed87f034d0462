// Driver for the sanitizer build of the library's host-only trace simulator (tests/test_host_sanitizers.py).
// Reads cases from stdin:  n_cases, then per case  T K N C policy n_init  init[n_init]  trace[T*K];
// prints per case:  rc misses lifetime_sum evictions.  Also walks the argument-error paths.
#include <cstdio>
#include <vector>

#include "moe_cache.h"

int main() {
  int n_cases = 0;
  if (scanf("%d", &n_cases) != 1) return 2;
  for (int c = 0; c < n_cases; ++c) {
    long long T;
    int K, N, C, policy, n_init;
    if (scanf("%lld %d %d %d %d %d", &T, &K, &N, &C, &policy, &n_init) != 6) return 2;
    std::vector<int32_t> init(n_init > 0 ? n_init : 0), trace((size_t)(T * K));
    for (auto &v : init)
      if (scanf("%d", &v) != 1) return 2;
    for (auto &v : trace)
      if (scanf("%d", &v) != 1) return 2;
    int64_t misses = -1, life = -1, ev = -1;
    // exact-size heap buffers: any read past the trace or the initial list is caught by the sanitizer
    static const int32_t none = 0;  // an empty trace still needs a non-NULL pointer (never read)
    const int rc = moe_trace_misses(trace.empty() ? &none : trace.data(), T, K, N, C, policy,
                                    init.empty() ? nullptr : init.data(), n_init, &misses, &life, &ev);
    printf("%d %lld %lld %lld\n", rc, (long long)misses, (long long)life, (long long)ev);
  }
  // error paths: nothing may be touched before the arguments are validated
  int64_t m = 0;
  const int32_t one[2] = {0, 1};
  int bad = 0;
  bad += moe_trace_misses(nullptr, 1, 2, 3, 2, MOE_POLICY_LRU, nullptr, 0, &m, nullptr, nullptr) != MOE_EINVAL;
  bad += moe_trace_misses(one, 1, 2, 3, 2, MOE_POLICY_LRU, nullptr, 0, nullptr, nullptr, nullptr) != MOE_EINVAL;
  bad += moe_trace_misses(one, 1, 2, 3, 4, MOE_POLICY_LRU, nullptr, 0, &m, nullptr, nullptr) != MOE_EINVAL;
  bad += moe_trace_misses(one, 1, 2, 3, 1, MOE_POLICY_FARTHEST, nullptr, 0, &m, nullptr, nullptr) != MOE_EINVAL;
  bad += moe_trace_misses(one, 1, 2, 3, 2, 7, nullptr, 0, &m, nullptr, nullptr) != MOE_EINVAL;
  bad += moe_trace_misses(one, 1, 2, 1, 1, MOE_POLICY_LRU, nullptr, 0, &m, nullptr, nullptr) != MOE_EINVAL;
  bad += moe_trace_misses(one, 1, 2, 3, 2, MOE_POLICY_LRU, nullptr, 1, &m, nullptr, nullptr) != MOE_EINVAL;
  printf("errors %d\n", bad);
  return bad ? 1 : 0;
}
