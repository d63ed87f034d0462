// Offline cache analysis on a recorded selection trace: host code only, no GPU work.
//
// A trace lists, token by token, the K distinct experts a layer selected, in the order the cache touches them
// (descending router weight, Sec. 4.2).  Misses are counted per token against the cache as it was before the token
// (Eq. 4).  Two eviction policies: least recently used (the policy of Sec. 4.2, also for capacities below K, where
// only the most recently touched experts of a token stay: the cache-size sweep of Sec. 4.8) and farthest next use
// (the optimal-eviction bound the paper compares against in Sec. 4.8).
#include <stdint.h>

#include <limits>
#include <vector>

#include "moe_cache.h"

namespace {

struct Residency {
  std::vector<uint8_t> in;     // expert is in the cache
  std::vector<int64_t> born;   // token at which it was loaded
  int count = 0;
  int64_t lifetime_sum = 0, evictions = 0;

  explicit Residency(int n) : in(n, 0), born(n, 0) {}
  void load(int e, int64_t t) {
    in[e] = 1;
    born[e] = t;
    ++count;
  }
  void evict(int e, int64_t t) {
    in[e] = 0;
    --count;
    lifetime_sum += t - born[e];
    ++evictions;
  }
};

}  // namespace

extern "C" int moe_trace_misses(const int32_t *trace, int64_t n_tokens, int32_t top_k, int32_t n_experts,
                                int32_t capacity, int32_t policy, const int32_t *initial, int32_t n_initial,
                                int64_t *misses, int64_t *lifetime_sum, int64_t *evictions) {
  if (!trace || !misses || n_tokens < 0 || top_k <= 0 || n_experts <= 0 || top_k > n_experts || capacity <= 0 ||
      capacity > n_experts || n_initial < 0 || n_initial > capacity || (n_initial > 0 && !initial))
    return MOE_EINVAL;
  if (policy != MOE_POLICY_LRU && policy != MOE_POLICY_FARTHEST) return MOE_EINVAL;
  if (policy == MOE_POLICY_FARTHEST && capacity < top_k) return MOE_EINVAL;
  const int N = n_experts, K = top_k;
  std::vector<uint8_t> seen(N);
  for (int64_t t = 0; t < n_tokens; ++t) {
    std::fill(seen.begin(), seen.end(), 0);
    for (int k = 0; k < K; ++k) {
      const int e = trace[t * K + k];
      if (e < 0 || e >= N || seen[e]) return MOE_EINVAL;
      seen[e] = 1;
    }
  }
  Residency res(N);
  std::fill(seen.begin(), seen.end(), 0);
  for (int i = 0; i < n_initial; ++i) {
    const int e = initial[i];
    if (e < 0 || e >= N || seen[e]) return MOE_EINVAL;
    seen[e] = 1;
    res.load(e, 0);
  }
  int64_t miss_total = 0;

  if (policy == MOE_POLICY_LRU) {
    // recency as a stamp per expert; initial residents are older than any token, in list order
    std::vector<int64_t> stamp(N, 0);
    for (int i = 0; i < n_initial; ++i) stamp[initial[i]] = (int64_t)i - n_initial;
    for (int64_t t = 0; t < n_tokens; ++t) {
      const int32_t *tok = trace + t * K;
      for (int k = 0; k < K; ++k) miss_total += !res.in[tok[k]];
      for (int k = 0; k < K; ++k) {
        const int e = tok[k];
        if (!res.in[e]) res.load(e, t);
        stamp[e] = t * K + k;
      }
      while (res.count > capacity) {
        int victim = -1;
        for (int e = 0; e < N; ++e)
          if (res.in[e] && (victim < 0 || stamp[e] < stamp[victim])) victim = e;
        res.evict(victim, t);
      }
    }
  } else {
    // next[t*K+k]: the next token that selects the same expert again, or "never"
    const int64_t never = std::numeric_limits<int64_t>::max();
    std::vector<int64_t> next((size_t)n_tokens * K), upcoming(N, never);
    for (int64_t t = n_tokens - 1; t >= 0; --t)
      for (int k = 0; k < K; ++k) {
        const int e = trace[t * K + k];
        next[t * K + k] = upcoming[e];
        upcoming[e] = t;
      }
    std::vector<int64_t> use = upcoming;  // per expert: its next use from now on (first use, at the start)
    std::vector<uint8_t> now(N);
    for (int64_t t = 0; t < n_tokens; ++t) {
      const int32_t *tok = trace + t * K;
      std::fill(now.begin(), now.end(), 0);
      for (int k = 0; k < K; ++k) {
        now[tok[k]] = 1;
        miss_total += !res.in[tok[k]];
      }
      for (int k = 0; k < K; ++k) {
        const int e = tok[k];
        use[e] = next[t * K + k];
        if (res.in[e]) continue;
        if (res.count >= capacity) {
          int victim = -1;  // farthest next use among the experts this token does not need; ties: lowest id
          for (int c = 0; c < N; ++c)
            if (res.in[c] && !now[c] && (victim < 0 || use[c] > use[victim])) victim = c;
          res.evict(victim, t);
        }
        res.load(e, t);
      }
    }
  }
  *misses = miss_total;
  if (lifetime_sum) *lifetime_sum = res.lifetime_sum;
  if (evictions) *evictions = res.evictions;
  return MOE_OK;
}
