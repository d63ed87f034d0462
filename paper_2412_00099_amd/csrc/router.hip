// Fused router kernel: gate GEMV, softmax, logit range, cache prior, top-K, hit/miss accounting,
// LRU slot-table update (paper Eq. 3, Eq. 10, Eq. 9, Eq. 2, Eq. 4, Sec. 4.2), one launch per layer-token.
//
// This file is compiled with floating-point contraction off: the steps that decide which expert is
// selected are single fp32 operations in a fixed order (subtract, add, divide, multiply, add), so the
// decisions are reproducible bit for bit from the same fp32 logits.
//
// Layout of the work: one workgroup.  All its wavefronts compute rows of z = W_gate x (128-bit loads,
// fp32 accumulation, wavefront reduction); wavefront 0 then does the routing with lane e <-> expert e
// and lane s <-> slot s (N <= 64, C <= 64), entirely in registers, and writes the decision both to
// device memory (read by the expert kernel) and to host-mapped memory (read by the host to issue fills).
#include "common.h"

namespace moe {
namespace {

__device__ __forceinline__ uint64_t ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }
__device__ __forceinline__ int readlane_i(int v, int l) { return __builtin_amdgcn_readlane(v, l); }
__device__ __forceinline__ float readlane_f(float v, int l) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}
__device__ __forceinline__ int64_t readlane_i64(int64_t v, int l) {
  uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, l);
  uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)v >> 32), l);
  return (int64_t)(((uint64_t)hi << 32) | lo);
}

template <int CTRL>
__device__ __forceinline__ float dppf(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dppf<0x128>(v));
  v = fmaxf(v, dppf<0x124>(v));
  v = fmaxf(v, dppf<0x122>(v));
  v = fmaxf(v, dppf<0x121>(v));
  return fmaxf(fmaxf(readlane_f(v, 0), readlane_f(v, 16)), fmaxf(readlane_f(v, 32), readlane_f(v, 48)));
}
__device__ __forceinline__ float wave_min(float v) { return -wave_max(-v); }

// Position of each lane's key in the descending order of (key, lower lane first) over lanes < n.
__device__ __forceinline__ int rank_desc(float key, int lane, int n) {
  int r = 0;
  for (int j = 0; j < n; ++j) {
    float kj = readlane_f(key, j);
    r += (kj > key) || (kj == key && j < lane);
  }
  return r;
}
// Same for ascending integer keys (unique keys expected).
__device__ __forceinline__ int rank_asc_i(int key, int n) {
  int r = 0;
  for (int j = 0; j < n; ++j) r += readlane_i(key, j) < key;
  return r;
}

__device__ __forceinline__ float gate_row_dot(const void *gate_w, const void *x, int row, int d, int act_fmt,
                                              int lane) {
  float acc = 0.f;
  if (act_fmt == MOE_A_BF16) {
    const uint4 *w = reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(gate_w) + (size_t)row * d);
    const uint4 *xv = reinterpret_cast<const uint4 *>(x);
    for (int c = lane; c < d / 8; c += kWave) {
      uint4 a = w[c], b = xv[c];
      acc = __builtin_fmaf(bf16_lo(a.x), bf16_lo(b.x), acc);
      acc = __builtin_fmaf(bf16_hi(a.x), bf16_hi(b.x), acc);
      acc = __builtin_fmaf(bf16_lo(a.y), bf16_lo(b.y), acc);
      acc = __builtin_fmaf(bf16_hi(a.y), bf16_hi(b.y), acc);
      acc = __builtin_fmaf(bf16_lo(a.z), bf16_lo(b.z), acc);
      acc = __builtin_fmaf(bf16_hi(a.z), bf16_hi(b.z), acc);
      acc = __builtin_fmaf(bf16_lo(a.w), bf16_lo(b.w), acc);
      acc = __builtin_fmaf(bf16_hi(a.w), bf16_hi(b.w), acc);
    }
  } else {
    const float4 *w = reinterpret_cast<const float4 *>(static_cast<const float *>(gate_w) + (size_t)row * d);
    const float4 *xv = reinterpret_cast<const float4 *>(x);
    for (int c = lane; c < d / 4; c += kWave) {
      float4 a = w[c], b = xv[c];
      acc = __builtin_fmaf(a.x, b.x, acc);
      acc = __builtin_fmaf(a.y, b.y, acc);
      acc = __builtin_fmaf(a.z, b.z, acc);
      acc = __builtin_fmaf(a.w, b.w, acc);
    }
  }
  return wave_sum(acc);
}

__global__ __launch_bounds__(1024) void route_kernel(RouteParams p, const void *gate_w, const void *x,
                                                     const float *logits_in, LayerState *st,
                                                     moe_route_out_t *out_dev, moe_route_out_t *out_host) {
  __shared__ float z_s[MOE_MAX_EXPERTS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n_waves = blockDim.x >> 6;
  const int N = p.n_experts, K = p.top_k, C = p.capacity;

  if (logits_in != nullptr) {
    if (tid < N) z_s[tid] = logits_in[tid];
  } else {
    for (int row = wave; row < N; row += n_waves) {
      float v = gate_row_dot(gate_w, x, row, p.hidden, p.act_fmt, lane);
      if (lane == 0) z_s[row] = v;
    }
  }
  __syncthreads();
  if (wave != 0) return;

  // ---- lane e <-> expert e ------------------------------------------------------------------
  const bool active = lane < N;
  const float z = active ? z_s[lane] : -INFINITY;

  // softmax of the unmodified logits (Eq. 3); feeds only the expert weights
  const float zmax = wave_max(z);
  const float zmin = wave_min(active ? z : INFINITY);
  const float pe = active ? expf(z - zmax) : 0.f;
  const float psum = wave_sum(pe);
  float w = pe / psum;

  // Delta_avg (Eq. 10): cumulative mean of the logit range, current token included
  const float range = zmax - zmin;
  const float dsum = st->delta_sum + range;
  const int t = st->count;
  const int cnt = t + 1;
  const float delta = (p.delta_mode == MOE_DELTA_FIXED) ? p.delta_fixed : dsum / (float)cnt;

  int my_slot = active ? st->expert_slot[lane] : -1;
  const bool resident = my_slot >= 0;
  int64_t stamp = st->stamp[lane];
  int slot_exp = (lane < C) ? st->slot_expert[lane] : -1;
  uint64_t ever_used = st->ever_used;

  // ranking by the router (Eq. 2), ties -> lower index
  const int rank_z = rank_desc(z, lane, N);
  const bool top_j = active && rank_z < p.top_j;

  int rank_p;      // position in the altered ranking r'
  float zp = z;    // altered logits (Cache-Prior only)
  if (p.route_mode == MOE_ROUTE_CACHE_PRIOR) {
    const float bias = p.lambda * delta;            // one rounding
    if (active && (resident || top_j)) zp = z + bias;  // one rounding (Eq. 9)
    rank_p = rank_desc(zp, lane, N);
  } else {
    // Max-Rank (Eq. 6-7) / Cumsum-Threshold (Eq. 8): two promote() passes = a three-class stable partition
    int M = p.max_rank;
    if (p.route_mode == MOE_ROUTE_CUMSUM) {
      // cumulative weight up to and including my rank; M = number of experts whose preceding mass < p
      float before = 0.f;
      for (int r = 0; r < N; ++r) {
        uint64_t m = ballot(active && rank_z == r);
        float wr = readlane_f(w, (int)__builtin_ctzll(m));
        if (rank_z > r) before += wr;
      }
      M = (int)__builtin_popcountll(ballot(active && before < p.cumsum_p));
    }
    const int cls = top_j ? 0 : ((resident && rank_z < M) ? 1 : 2);
    rank_p = rank_asc_i(active ? cls * 64 + rank_z : 0x7fffffff, kWave);
  }
  const bool sel = active && rank_p < K;
  const uint64_t sel_mask = ballot(sel);
  const bool miss = sel && !resident;
  const uint64_t miss_mask = ballot(miss);
  const int n_miss = (int)__builtin_popcountll(miss_mask);

  // margin between the K-th and (K+1)-th altered logit (tie logging)
  float margin = INFINITY;
  if (K < N && p.route_mode == MOE_ROUTE_CACHE_PRIOR) {
    float a = readlane_f(zp, (int)__builtin_ctzll(ballot(active && rank_p == K - 1)));
    float b = readlane_f(zp, (int)__builtin_ctzll(ballot(active && rank_p == K)));
    margin = a - b;
  }

  // expert weights from the unmodified logits (Sec. 3.3), optional renormalisation (Sec. 2.1)
  if (p.renormalize) {
    const float s = wave_sum(sel ? w : 0.f);
    w = w / s;
  }

  // ---- LRU update (Sec. 4.2) ----------------------------------------------------------------
  // touch order inside the token: descending original logit -> position pos; stamp = t*K + pos
  int pos = 0;
  for (uint64_t m = sel_mask; m; m &= m - 1) pos += readlane_i(rank_z, (int)__builtin_ctzll(m)) < rank_z;
  if (sel) stamp = (int64_t)t * K + pos;
  int ordinal = 0;  // among the misses, in touch order
  for (uint64_t m = miss_mask; m; m &= m - 1) ordinal += readlane_i(pos, (int)__builtin_ctzll(m)) < pos;

  uint64_t empty_mask = ballot(lane < C && slot_exp < 0);
  const int n_empty = (int)__builtin_popcountll(empty_mask);
  const bool eligible = resident && !sel;  // selected experts are never victims
  const uint64_t elig_mask = ballot(eligible);
  int vrank = 0;  // eligible experts ordered by stamp, oldest first
  if (n_miss > n_empty) {
    for (uint64_t m = elig_mask; m; m &= m - 1) vrank += readlane_i64(stamp, (int)__builtin_ctzll(m)) < stamp;
  }
  int my_evicted = -1;
  int cold = 0, evictions = 0;
  for (int q = 0; q < n_miss; ++q) {
    const int ml = (int)__builtin_ctzll(ballot(miss && ordinal == q));
    int s, victim = -1;
    if (q < n_empty) {
      s = (int)__builtin_ctzll(empty_mask);
      empty_mask &= empty_mask - 1;
      cold += !((ever_used >> s) & 1);
    } else {
      victim = (int)__builtin_ctzll(ballot(eligible && vrank == q - n_empty));
      s = readlane_i(my_slot, victim);
      if (lane == victim) my_slot = -1;
      ++evictions;
    }
    if (lane == ml) {
      my_slot = s;
      my_evicted = victim;
    }
    if (lane == s) slot_exp = ml;
    ever_used |= 1ull << s;
  }

  // ---- write the decision and the state -----------------------------------------------------
  if (active) {
    st->expert_slot[lane] = my_slot;
    st->stamp[lane] = stamp;
    out_dev->logits[lane] = z;
    out_host->logits[lane] = z;
  }
  if (lane < C) st->slot_expert[lane] = slot_exp;
  if (sel) {
    const int k = rank_p;
    out_dev->sel_expert[k] = lane;
    out_dev->sel_slot[k] = my_slot;
    out_dev->sel_weight[k] = w;
    out_dev->miss[k] = miss;
    out_dev->evicted[k] = my_evicted;
    out_host->sel_expert[k] = lane;
    out_host->sel_slot[k] = my_slot;
    out_host->sel_weight[k] = w;
    out_host->miss[k] = miss;
    out_host->evicted[k] = my_evicted;
  }
  if (lane == 0) {
    st->ever_used = ever_used;
    st->delta_sum = dsum;
    st->count = cnt;
    st->selections += K;
    st->hits += K - n_miss;
    st->misses += n_miss;
    st->cold_misses += cold;
    st->evictions += evictions;
    out_dev->n_miss = n_miss;
    out_dev->token = t;
    out_dev->delta = delta;
    out_dev->margin = margin;
    out_host->n_miss = n_miss;
    out_host->token = t;
    out_host->delta = delta;
    out_host->margin = margin;
  }
  __threadfence_system();
  __builtin_amdgcn_wave_barrier();
  if (lane == 0) {
    out_dev->seq = p.seq;
    __hip_atomic_store(&out_host->seq, p.seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
  }
}

__global__ void state_init_kernel(LayerState *state, int n_layers, const int32_t *initial, int n_initial) {
  const int layer = blockIdx.x, lane = threadIdx.x;
  if (layer >= n_layers) return;
  LayerState *st = state + layer;
  st->expert_slot[lane] = -1;
  st->slot_expert[lane] = -1;
  st->stamp[lane] = 0;
  __syncthreads();
  if (lane < n_initial) {
    const int e = initial[layer * n_initial + lane];
    st->expert_slot[e] = lane;
    st->slot_expert[lane] = e;
    st->stamp[e] = (int64_t)lane - n_initial;  // -n .. -1 in list order: the first listed is the oldest
  }
  if (lane == 0) {
    st->ever_used = n_initial >= 64 ? ~0ull : ((1ull << n_initial) - 1ull);
    st->delta_sum = 0.f;
    st->count = 0;
    st->selections = st->hits = st->misses = st->cold_misses = st->evictions = 0;
  }
}

}  // namespace

hipError_t launch_route(const RouteParams &p, const void *gate_w, const void *x, const float *logits,
                        LayerState *state, moe_route_out_t *out_dev, moe_route_out_t *out_host_mapped,
                        hipStream_t s) {
  // enough wavefronts that every row of the gate matrix has all its loads in flight at once
  int waves = logits ? 1 : (p.n_experts + 3) / 4;
  if (waves > 16) waves = 16;
  if (waves < 1) waves = 1;
  hipLaunchKernelGGL(route_kernel, dim3(1), dim3(waves * kWave), 0, s, p, gate_w, x, logits, state, out_dev,
                     out_host_mapped);
  return hipGetLastError();
}

hipError_t launch_state_init(LayerState *state, int n_layers, const int32_t *initial_dev, int n_initial,
                             hipStream_t s) {
  hipLaunchKernelGGL(state_init_kernel, dim3(n_layers), dim3(MOE_MAX_EXPERTS), 0, s, state, n_layers, initial_dev,
                     n_initial);
  return hipGetLastError();
}

}  // namespace moe
