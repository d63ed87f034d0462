// Device code of the routing step (paper Eq. 3, Eq. 10, Eq. 9, Eq. 2, Eq. 4, Sec. 4.2), shared by the router
// kernels and by the expert kernels that run the layer boundary in their first workgroup.
//
// The steps that decide which expert is selected are single fp32 operations in a fixed order (subtract, add,
// divide, multiply, add) with floating-point contraction off, so the decisions are reproducible bit for bit from
// the same fp32 logits.
//
// Routing is done by one wavefront with lane e <-> expert e and lane s <-> slot s (N <= 64, C <= 64), entirely in
// registers.  Full rankings (baseline modes) are counted with one 64-bit compare per pair: the key is the logit
// mapped to an order-preserving unsigned integer, with 63 - lane below it so that equal logits rank the lower
// index first.  The decision record is assembled in LDS and written with 16-byte stores to device memory; what
// the host needs goes to host-mapped memory as three self-tagged 8-byte words.
#pragma once

#include "common.h"
#include "gemv_common.h"

namespace moe {
namespace rt {

constexpr int kRecWords = sizeof(moe_route_out_t) / 4;
static_assert(sizeof(moe_route_out_t) % 16 == 0, "route record is copied in 16-byte chunks");
// word offsets inside moe_route_out_t
constexpr int W_EXPERT = 0, W_SLOT = 8, W_WEIGHT = 16, W_MISS = 24, W_EVICT = 32, W_NMISS = 40, W_TOKEN = 41,
              W_DELTA = 42, W_MARGIN = 43, W_LOGITS = 44, W_SEQ = 44 + MOE_MAX_EXPERTS;
static_assert(W_SEQ * 4 == offsetof(moe_route_out_t, opaque), "record layout");
static_assert(W_LOGITS * 4 == offsetof(moe_route_out_t, logits), "record layout");

__device__ __forceinline__ uint64_t ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }
__device__ __forceinline__ int readlane_i(int v, int l) { return __builtin_amdgcn_readlane(v, l); }
__device__ __forceinline__ float readlane_f(float v, int l) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}
__device__ __forceinline__ uint64_t readlane_u64(uint64_t v, int l) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, l);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), l);
  return ((uint64_t)hi << 32) | lo;
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

// Order-preserving map of a finite float to uint32 (+0 and -0 must have been merged by the caller).
__device__ __forceinline__ uint32_t sortable(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
// key: larger = earlier in a descending ranking; equal values rank the lower lane first
__device__ __forceinline__ uint64_t rank_key(float v, int lane, bool active) {
  return active ? (((uint64_t)sortable(v + 0.f) << 32) | (uint32_t)(63 - lane)) : 0ull;
}
// number of lanes < n whose key is larger than mine = my position in the descending ranking
// (lanes >= n hold key 0, which is larger than no key, so all 64 lanes are always compared: no loop-carried branch)
__device__ __forceinline__ int rank_of(uint64_t key) {
  int r = 0;
#pragma unroll
  for (int j = 0; j < kWave; ++j) r += readlane_u64(key, j) > key;
  return r;
}

__device__ __forceinline__ float dot2(uint32_t w, uint32_t x, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), __builtin_bit_cast(bf16x2, x), acc, false);
}

// Up to R consecutive rows of z = W_gate x for one wavefront, all loads of a chunk column issued together.
template <int R>
__device__ __forceinline__ void gate_rows(const void *gate_w, const void *x, int row0, int nrows, int d, int act_fmt,
                                          int lane, float *out) {
  float acc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = 0.f;
  if (act_fmt == MOE_A_BF16) {
    const int nch = d / 8;
    const u32x4 *xv = reinterpret_cast<const u32x4 *>(x);
    const u32x4 *w = reinterpret_cast<const u32x4 *>(gate_w) + (size_t)row0 * nch;
#pragma unroll 4
    for (int c = lane; c < nch; c += kWave) {
      const u32x4 b = xv[c];
#pragma unroll
      for (int r = 0; r < R; ++r) {
        // rows past the last one re-read the last row (always in bounds); their sums are discarded
        const u32x4 a = w[(size_t)(r < nrows ? r : nrows - 1) * nch + c];
        acc[r] = dot2(a.x, b.x, acc[r]);
        acc[r] = dot2(a.y, b.y, acc[r]);
        acc[r] = dot2(a.z, b.z, acc[r]);
        acc[r] = dot2(a.w, b.w, acc[r]);
      }
    }
  } else {
    const int nch = d / 4;
    const float4 *xv = reinterpret_cast<const float4 *>(x);
    const float4 *w = reinterpret_cast<const float4 *>(gate_w) + (size_t)row0 * nch;
#pragma unroll 4
    for (int c = lane; c < nch; c += kWave) {
      const float4 b = xv[c];
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const float4 a = w[(size_t)(r < nrows ? r : nrows - 1) * nch + c];
        acc[r] = __builtin_fmaf(a.x, b.x, acc[r]);
        acc[r] = __builtin_fmaf(a.y, b.y, acc[r]);
        acc[r] = __builtin_fmaf(a.z, b.z, acc[r]);
        acc[r] = __builtin_fmaf(a.w, b.w, acc[r]);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < R; ++r) out[r] = wave_sum(acc[r]);
}

// z = W_gate x by all wavefronts of the workgroup, at most four rows each
__device__ __forceinline__ void gate_gemv(const void *gate_w, const void *x, const RouteParams &p, int wave, int n_waves,
                                          int lane, float *z_s) {
  constexpr int R = 4;
  const int N = p.n_experts;
  const int rpw = (N + n_waves - 1) / n_waves;  // rows per wavefront
  for (int row0 = wave * rpw; row0 < min(N, (wave + 1) * rpw); row0 += R) {
    float v[R];
    const int nrows = min(R, min(N, (wave + 1) * rpw) - row0);
    gate_rows<R>(gate_w, x, row0, nrows, p.hidden, p.act_fmt, lane, v);
#pragma unroll
    for (int r = 0; r < R; ++r)
      if (lane == 0 && r < nrows) z_s[row0 + r] = v[r];
  }
}

// Cache state of one layer as held by wavefront 0 (lane e: expert e, lane s: slot s).
struct CacheRegs {
  int my_slot, slot_exp, t, born;
  int64_t stamp;
  uint64_t ever_used;
  float dsum_prev;
  int64_t counter;  // lanes 0..5: selections, hits, misses, cold misses, evictions, lifetime sum
};

__device__ __forceinline__ CacheRegs load_cache_regs(const LayerState *st, int lane, int N, int C) {
  // every lane loads (the tables have 64 entries, the counter index is clamped) and masks afterwards: loads
  // inside branches would make later waits cover all outstanding loads
  CacheRegs cr;
  const int my_slot = st->expert_slot[lane];
  const int64_t stamp = st->stamp[lane];
  const int born = st->born[lane];
  const int slot_exp = st->slot_expert[lane];
  const int64_t counter = (&st->selections)[lane < 6 ? lane : 5];
  cr.ever_used = st->ever_used;
  cr.dsum_prev = st->delta_sum;
  cr.t = st->count;
  cr.my_slot = lane < N ? my_slot : -1;
  cr.stamp = lane < N ? stamp : 0;
  cr.born = lane < N ? born : 0;
  cr.slot_exp = lane < C ? slot_exp : -1;
  cr.counter = lane < 6 ? counter : 0;
  return cr;
}

// Where a layer-boundary step hands its decision to the other workgroups of the same launch (expert kernels that
// run the boundary in their first workgroup): what they need - the K slots, the miss flags and the K weights - as
// eight 8-byte words, each complete in itself: bits 0..15 = the tag of this hand-over (a per-layer count, so the
// words' previous content never carries it), bits 16..63 = 48 bits of payload
//     word 0: slots of positions 0..5 (8 bits each)      word 1: slots of positions 6, 7 | miss flags << 16
//     words 2..7: the eight fp32 weights as one 256-bit string, 48 bits per word
// A reader accepts the eight words only when all carry the tag it waits for, so no order between the stores is
// assumed: 8-byte atomic stores and loads, no fence.  The block is written kHandoverCopies times, 64 bytes apart,
// by one store instruction; workgroup b reads copy b % kHandoverCopies (hundreds of wavefronts polling one line
// serialise in the memory system).  handover = nullptr when nobody waits (separate router launch).
struct BoundaryFlags {
  uint64_t *handover;
  uint32_t tag;  // 16 bits
};
constexpr int kHandoverCopies = 8;
static_assert(kHandoverCopies * 8 == kWave, "one lane per word of every copy");

// Everything after the logits (Eq. 3 softmax, Eq. 10, Eq. 9, Eq. 2, Eq. 4, Sec. 4.2), run by one wavefront.
// note == nullptr: nobody on the host waits for this step (a token inside a batch).  carry != nullptr: receives the
// cache state as this step leaves it, so that a batch continues from registers; store_state = false then leaves the
// state in device memory as it was.  n_miss_out, when given, receives the number of misses of the step.  out_dev may
// point into LDS (a record that is copied out later, or dropped).
__device__ __forceinline__ void route_wave(const RouteParams &p, const float *z_s, const CacheRegs &cr, LayerState *st,
                                           moe_route_out_t *out_dev, HostNote *note, uint32_t *rec_s, int lane,
                                           BoundaryFlags flags = BoundaryFlags{nullptr, 0}, CacheRegs *carry = nullptr,
                                           bool store_state = true, int *n_miss_out = nullptr) {
#pragma clang fp contract(off)
  const int N = p.n_experts, K = p.top_k, C = p.capacity;
  int my_slot = cr.my_slot, slot_exp = cr.slot_exp;
  const int t = cr.t;
  int64_t stamp = cr.stamp;
  uint64_t ever_used = cr.ever_used;
  const float dsum_prev = cr.dsum_prev;

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
  const float dsum = dsum_prev + range;
  const int cnt = t + 1;
  const float delta = p.delta_mode == MOE_DELTA_FIXED ? p.delta_fixed
                      : p.delta_mode == MOE_DELTA_TOKEN ? range
                                                        : dsum / (float)cnt;

  const bool resident = my_slot >= 0;

  // router's own top-J (Sec. 3.3): J rounds of arg-max, ties -> lower index
  uint64_t topj_mask = 0;
  for (int j = 0; j < p.top_j; ++j) {
    const bool cand = active && !((topj_mask >> lane) & 1);
    const float m = wave_max(cand ? z : -INFINITY);
    topj_mask |= 1ull << __builtin_ctzll(ballot(cand && z == m));
  }
  const bool top_j = (topj_mask >> lane) & 1;

  int rank_p;    // position in the altered ranking r' (exact for the first K positions, >= K otherwise)
  float zp = z;  // altered logits (Cache-Prior only)
  float margin = INFINITY;  // between the K-th and (K+1)-th altered logit (tie logging)
  uint64_t taken = 0;       // Cache-Prior: the experts placed so far
  float kth = 0.f;
  if (p.route_mode == MOE_ROUTE_CACHE_PRIOR) {
    const float bias = p.lambda * delta;               // one rounding
    if (active && (resident || top_j)) zp = z + bias;  // one rounding (Eq. 9)
    // only the head of r' matters: K rounds of arg-max, ties -> lower index (one more round, for the margin,
    // follows once the decision has been handed on)
    rank_p = N;
    for (int k = 0; k < K; ++k) {
      const bool cand = active && !((taken >> lane) & 1);
      const float m = wave_max(cand ? zp : -INFINITY);
      const int l = (int)__builtin_ctzll(ballot(cand && zp == m));
      taken |= 1ull << l;
      if (lane == l) rank_p = k;
      kth = m;
    }
  } else {
    // Max-Rank (Eq. 6-7) / Cumsum-Threshold (Eq. 8): two promote() passes = a three-class stable partition
    const int rank_z = rank_of(rank_key(z, lane, active));
    int M = p.max_rank;
    if (p.route_mode == MOE_ROUTE_CUMSUM) {
      // mass ranked before me; M = number of experts whose preceding mass is still below p
      float before = 0.f;
      for (int r = 0; r < N; ++r) {
        const float wr = readlane_f(w, (int)__builtin_ctzll(ballot(active && rank_z == r)));
        if (rank_z > r) before += wr;
      }
      M = (int)__builtin_popcountll(ballot(active && before < p.cumsum_p));
    }
    const int cls = top_j ? 0 : ((resident && rank_z < M) ? 1 : 2);
    const uint64_t key = active ? (((uint64_t)(2 - cls) << 32) | (uint32_t)(63 - rank_z)) : 0ull;
    rank_p = rank_of(key);
  }
  const bool sel = active && rank_p < K;
  const uint64_t sel_mask = ballot(sel);
  const bool miss = sel && !resident;
  const uint64_t miss_mask = ballot(miss);
  const int n_miss = (int)__builtin_popcountll(miss_mask);
  if (n_miss_out != nullptr) *n_miss_out = n_miss;

  // expert weights from the unmodified logits (Sec. 3.3), optional renormalisation (Sec. 2.1)
  if (p.renormalize) {
    const float s = wave_sum(sel ? w : 0.f);
    w = w / s;
  }

  // ---- LRU update (Sec. 4.2) ----------------------------------------------------------------
  // touch order inside the token: descending original logit (ties -> lower index) -> position pos
  const uint64_t zkey = rank_key(z, lane, active);
  int pos = 0;
  for (uint64_t m = sel_mask; m; m &= m - 1) pos += readlane_u64(zkey, (int)__builtin_ctzll(m)) > zkey;
  if (sel) stamp = (int64_t)t * K + pos;
  int ordinal = 0;  // among the misses, in touch order
  for (uint64_t m = miss_mask; m; m &= m - 1) ordinal += readlane_i(pos, (int)__builtin_ctzll(m)) < pos;

  uint64_t empty_mask = ballot(lane < C && slot_exp < 0);
  const int n_empty = (int)__builtin_popcountll(empty_mask);
  const bool eligible = resident && !sel;  // selected experts are never victims
  const uint64_t elig_mask = ballot(eligible);
  int vrank = 0;  // eligible experts ordered by stamp, oldest first
  if (n_miss > n_empty) {
    for (uint64_t m = elig_mask; m; m &= m - 1)
      vrank += (int64_t)readlane_u64((uint64_t)stamp, (int)__builtin_ctzll(m)) < stamp;
  }
  int my_evicted = -1;
  int born = cr.born;
  int cold = 0, evictions = 0, lifetime = 0;  // lifetime: tokens the evicted experts had stayed (Sec. 4.6)
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
      lifetime += t - readlane_i(born, victim);
      if (lane == victim) my_slot = -1;
      ++evictions;
    }
    if (lane == ml) {
      my_slot = s;
      my_evicted = victim;
      born = t;
    }
    if (lane == s) slot_exp = ml;
    ever_used |= 1ull << s;
  }

  // ---- the decision in selection order, into the record being assembled in LDS ----------------------------
  rec_s[lane] = 0;
  if (lane + 64 < kRecWords) rec_s[lane + 64] = 0;
  __builtin_amdgcn_wave_barrier();
  if (lane < MOE_MAX_TOPK) rec_s[W_EVICT + lane] = (uint32_t)-1;
  if (active) rec_s[W_LOGITS + lane] = __float_as_uint(z);
  __builtin_amdgcn_wave_barrier();
  if (sel) {
    const int k = rank_p;
    rec_s[W_EXPERT + k] = (uint32_t)lane;
    rec_s[W_SLOT + k] = (uint32_t)my_slot;
    rec_s[W_WEIGHT + k] = __float_as_uint(w);
    rec_s[W_MISS + k] = miss ? 1u : 0u;
    rec_s[W_EVICT + k] = (uint32_t)my_evicted;
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  // ---- what the host needs (experts, slots, miss flags in selection order): three tagged 8-byte words ----
  // stored to mapped host memory as early as possible, so the trip over the host link overlaps the rest.  Every
  // lane packs them from the K entries just written (the same LDS words for all lanes: broadcast reads; a loop over
  // the selected lanes with lane reads costs three times as long)
  uint32_t lo = 0, hi = 0, mm = 0;
  uint64_t ew = 0, sw = 0;
#pragma unroll
  for (int k = 0; k < MOE_MAX_TOPK; ++k) {
    if (k < K) {
      const uint32_t e = rec_s[W_EXPERT + k], s8 = rec_s[W_SLOT + k] & 0xffu;
      if (k < 4) lo |= s8 << (8 * k); else hi |= s8 << (8 * (k - 4));
      mm |= rec_s[W_MISS + k] << k;
      ew |= (uint64_t)e << (16 + 6 * k);
      sw |= (uint64_t)(s8 & 63u) << (16 + 6 * k);
    }
  }
  if (note != nullptr && lane < 3) {
    const uint64_t tag = p.seq & 0xffffu;
    const uint64_t w0 = (uint64_t)p.seq | ((uint64_t)n_miss << 32) | ((uint64_t)mm << 40);
    const uint64_t v = lane == 0 ? w0 : (tag | (lane == 1 ? ew : sw));
    __hip_atomic_store(&note->w[lane], v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  }

  // ---- expert kernels waiting in the same launch need weights, slots and miss flags (see BoundaryFlags)
  if (flags.handover != nullptr) {
    const int word = lane & 7;  // lane = copy * 8 + word
    uint64_t payload;
    if (word == 0) {
      payload = ((uint64_t)lo | ((uint64_t)hi << 32)) & 0xffffffffffffull;
    } else if (word == 1) {
      payload = (uint64_t)(hi >> 16) | ((uint64_t)(mm & 0xffu) << 16);
    } else {
      const int bit = 48 * (word - 2), i = bit >> 5, sh = bit & 31;  // position in the 256-bit weight string
      const uint32_t next = i + 1 < MOE_MAX_TOPK ? rec_s[W_WEIGHT + i + 1] : 0u;  // (the string ends with weight 7)
      const uint64_t two = (uint64_t)rec_s[W_WEIGHT + i] | ((uint64_t)next << 32);
      payload = (two >> sh) & 0xffffffffffffull;
    }
    __hip_atomic_store(flags.handover + lane, (payload << 16) | (uint64_t)(flags.tag & 0xffffu), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
  }

  // margin between the K-th and (K+1)-th altered logit: one more arg-max round
  if (p.route_mode == MOE_ROUTE_CACHE_PRIOR && K < N) {
    const bool cand = active && !((taken >> lane) & 1);
    margin = kth - wave_max(cand ? zp : -INFINITY);
  }

  // ---- state back to device memory ------------------------------------------------------------
  const int inc = lane == 0 ? K : lane == 1 ? K - n_miss : lane == 2 ? n_miss : lane == 3 ? cold
                : lane == 4 ? evictions : lifetime;
  if (store_state) {
    if (active) {
      st->expert_slot[lane] = my_slot;
      st->stamp[lane] = stamp;
      st->born[lane] = born;
    }
    if (lane < C) st->slot_expert[lane] = slot_exp;
    if (lane == 0) {
      st->ever_used = ever_used;
      st->delta_sum = dsum;
      st->count = cnt;
    }
    if (lane < 6) (&st->selections)[lane] = cr.counter + inc;
  }
  if (carry != nullptr) {
    carry->my_slot = my_slot;
    carry->slot_exp = slot_exp;
    carry->t = cnt;
    carry->born = born;
    carry->stamp = stamp;
    carry->ever_used = ever_used;
    carry->dsum_prev = dsum;
    carry->counter = lane < 6 ? cr.counter + inc : 0;
  }

  // ---- full decision record in device memory: assembled in LDS, copied out in 16-byte chunks ----
  if (lane == 0) {
    // compact copy for the expert kernels: slots 8 bits each in selection order, miss flags as a mask
    rec_s[W_SEQ] = p.seq;
    rec_s[W_SEQ + 1] = lo;
    rec_s[W_SEQ + 2] = hi;
    rec_s[W_SEQ + 3] = mm;
    rec_s[W_NMISS] = (uint32_t)n_miss;
    rec_s[W_TOKEN] = (uint32_t)t;
    rec_s[W_DELTA] = __float_as_uint(delta);
    rec_s[W_MARGIN] = __float_as_uint(margin);
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  if (lane < kRecWords / 4) reinterpret_cast<u32x4 *>(out_dev)[lane] = reinterpret_cast<const u32x4 *>(rec_s)[lane];
}

// Gate rows of one wavefront held in registers: loaded before x exists, used once x is in LDS.
template <int R, int CH>
struct GateRegs {
  u32x4 w[R][CH];
};
template <int R, int CH>
__device__ __forceinline__ void gate_prefetch(const void *gate_w, int row0, int nrows, int lane, GateRegs<R, CH> &g) {
  const u32x4 *w = reinterpret_cast<const u32x4 *>(gate_w) + (size_t)row0 * (CH * kWave);
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int c = 0; c < CH; ++c) g.w[r][c] = w[(size_t)(r < nrows ? r : nrows - 1) * (CH * kWave) + c * kWave + lane];
}
template <int R, int CH>
__device__ __forceinline__ void gate_dot(const GateRegs<R, CH> &g, const uint32_t *x_s, int act_fmt, int lane, float *out) {
  float acc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = 0.f;
#pragma unroll
  for (int c = 0; c < CH; ++c) {
    const u32x4 b = reinterpret_cast<const u32x4 *>(x_s)[c * kWave + lane];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const u32x4 a = g.w[r][c];
      if (act_fmt == MOE_A_BF16) {
        acc[r] = dot2(a.x, b.x, acc[r]);
        acc[r] = dot2(a.y, b.y, acc[r]);
        acc[r] = dot2(a.z, b.z, acc[r]);
        acc[r] = dot2(a.w, b.w, acc[r]);
      } else {
        acc[r] = __builtin_fmaf(__uint_as_float(a.x), __uint_as_float(b.x), acc[r]);
        acc[r] = __builtin_fmaf(__uint_as_float(a.y), __uint_as_float(b.y), acc[r]);
        acc[r] = __builtin_fmaf(__uint_as_float(a.z), __uint_as_float(b.z), acc[r]);
        acc[r] = __builtin_fmaf(__uint_as_float(a.w), __uint_as_float(b.w), acc[r]);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < R; ++r) out[r] = wave_sum(acc[r]);
}

// PER consecutive values for one thread, fetched with one load
template <int PER>
__device__ __forceinline__ void load_f32(const float *p, float *out) {
  if constexpr (PER == 1) {
    out[0] = p[0];
  } else if constexpr (PER == 2) {
    const float2 v = *reinterpret_cast<const float2 *>(p);
    out[0] = v.x; out[1] = v.y;
  } else {
#pragma unroll
    for (int i = 0; i < PER / 4; ++i) {
      const float4 v = reinterpret_cast<const float4 *>(p)[i];
      out[4 * i] = v.x; out[4 * i + 1] = v.y; out[4 * i + 2] = v.z; out[4 * i + 3] = v.w;
    }
  }
}
template <int PER>
__device__ __forceinline__ void load_bf16(const uint16_t *p, float *out) {
  if constexpr (PER == 1) {
    out[0] = __uint_as_float((uint32_t)p[0] << 16);
  } else if constexpr (PER == 2) {
    const uint32_t v = *reinterpret_cast<const uint32_t *>(p);
    out[0] = bf16_lo(v); out[1] = bf16_hi(v);
  } else {
#pragma unroll
    for (int i = 0; i < PER / 4; ++i) {
      const u32x2 v = reinterpret_cast<const u32x2 *>(p)[i];
      out[4 * i] = bf16_lo(v.x); out[4 * i + 1] = bf16_hi(v.x); out[4 * i + 2] = bf16_lo(v.y);
      out[4 * i + 3] = bf16_hi(v.y);
    }
  }
}
template <int PER>
__device__ __forceinline__ void store_f32(float *p, const float *v) {
  if constexpr (PER == 1) p[0] = v[0];
  else if constexpr (PER == 2) *reinterpret_cast<float2 *>(p) = make_float2(v[0], v[1]);
  else {
#pragma unroll
    for (int i = 0; i < PER / 4; ++i)
      reinterpret_cast<float4 *>(p)[i] = make_float4(v[4 * i], v[4 * i + 1], v[4 * i + 2], v[4 * i + 3]);
  }
}
template <int PER>
__device__ __forceinline__ void store_bf16(uint16_t *p, const float *v) {
  if constexpr (PER == 1) {
    p[0] = f32_to_bf16_rne(v[0]);
  } else if constexpr (PER == 2) {
    *reinterpret_cast<uint32_t *>(p) = (uint32_t)f32_to_bf16_rne(v[0]) | ((uint32_t)f32_to_bf16_rne(v[1]) << 16);
  } else {
#pragma unroll
    for (int i = 0; i < PER / 4; ++i) {
      u32x2 o;
      o.x = (uint32_t)f32_to_bf16_rne(v[4 * i]) | ((uint32_t)f32_to_bf16_rne(v[4 * i + 1]) << 16);
      o.y = (uint32_t)f32_to_bf16_rne(v[4 * i + 2]) | ((uint32_t)f32_to_bf16_rne(v[4 * i + 3]) << 16);
      reinterpret_cast<u32x2 *>(p)[i] = o;
    }
  }
}


// LDS the boundary needs (the caller provides it): logits, record staging, per-wavefront partial sums, x.
struct BoundaryLds {
  float *z_s;        // [MOE_MAX_EXPERTS]
  uint32_t *rec_s;   // [kRecWords], 16-byte aligned
  float *part_s;     // [NW]
  uint32_t *x_s;     // [hidden] in act_fmt (bf16 uses half of it), 16-byte aligned
};
constexpr int kBoundaryLdsWords = MOE_MAX_EXPERTS + kRecWords + 16 + kFusedMaxHidden;
__device__ __forceinline__ BoundaryLds carve_boundary_lds(uint32_t *base) {  // base 16-byte aligned
  BoundaryLds l;
  l.rec_s = base;
  l.x_s = base + kRecWords;
  l.z_s = reinterpret_cast<float *>(base + kRecWords + kFusedMaxHidden);
  l.part_s = l.z_s + MOE_MAX_EXPERTS;
  return l;
}

// Layer boundary of a stack by one workgroup of NW wavefronts: the residual / perturbation / RMS-normalisation
// glue and the routing of this layer (the previous layer's expert output y has been summed by
// partial_reduce_kernel).
//   h = carry ? h + y + perturb*a : perturb*a ;  x = h / sqrt(mean(h^2) + 1e-6) -> x_out and LDS ;  route on x.
// CH > 0: 16-byte chunks per gate row per lane (d = CH*64*VEC); the wavefront's gate rows are then loaded into
// registers at the very start, so the weight fetch overlaps the glue.  CH == 0: any d, rows loaded afterwards.
// PER > 0: d = NW*64*PER and thread t owns the PER consecutive columns t*PER...; all loads of the first phase
// (cache state, glue operands, gate rows) are then issued unconditionally and in that order, so each use waits
// only for the loads ahead of it (a load inside a branch makes the compiler wait for all outstanding loads,
// which would serialise the memory round trips).  PER == 0: any d, columns t, t + NW*64, ... per thread.
// PRE: the glue has been done by reduce_glue_kernel (f.h is the new residual stream, f.ss its sums of squares
// per 64 columns); only x is formed here, with the same operations in the same order as the expert kernels use
// to form their own copy of x, so that both are bit-identical.
// All threads of the workgroup must call it; only wavefront 0 returns late (after the routing).
template <int NW, int CH, int PER, bool PRE = false>
__device__ __forceinline__ void fused_boundary(const RouteParams &p, const FusedParams &f, const void *gate_w,
                                               LayerState *st, moe_route_out_t *out_dev, HostNote *note,
                                               BoundaryFlags flags, const BoundaryLds &lds) {
#pragma clang fp contract(off)
  constexpr int NT = NW * kWave;
  constexpr int R = (MOE_MAX_EXPERTS + NW - 1) / NW;  // gate rows per wavefront
  float *z_s = lds.z_s, *part_s = lds.part_s;
  uint32_t *x_s = lds.x_s;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int d = p.hidden, N = p.n_experts;
  const bool bf16 = p.act_fmt == MOE_A_BF16;
  const int rpw = (N + NW - 1) / NW;  // rows per wavefront (<= R)
  const int row0 = wave * rpw, nrows = min(rpw, N - row0);
  const bool with_y = f.y != nullptr && f.carry;
  constexpr int kMaxPer = PER > 0 ? PER : kFusedMaxHidden / NT;
  float hv[kMaxPer], yv[kMaxPer], av[kMaxPer];
  CacheRegs cr{};
  GateRegs<R, (CH > 0 ? CH : 1)> greg;

  float tot_pre = 0.f;
  if constexpr (PRE) {
    static_assert(PER > 0, "the precomputed-glue path is only built for the vectorised column split");
    cr = load_cache_regs(st, lane, N, p.capacity);
    load_f32<PER>(f.h + tid * PER, hv);
    OrderedSum<NW * PER> blocks;  // d / 64 = NW * PER blocks of 64 columns
    blocks.fetch(f.ss, lane);
    __builtin_amdgcn_sched_barrier(0);  // the small loads stay ahead of the gate rows
    if constexpr (CH > 0) {
      const int r0 = min(row0, N - 1);
      gate_prefetch<R, (CH > 0 ? CH : 1)>(gate_w, r0, max(1, min(R, N - r0)), lane, greg);
    }
    tot_pre = blocks.total();
  } else if constexpr (PER > 0) {
    // every wavefront loads the cache state (only wavefront 0 uses it): unconditional, and the oldest loads
    cr = load_cache_regs(st, lane, N, p.capacity);
    // operands that are absent are read from h instead (any valid address) and masked out below
    const int j0 = tid * PER;
    load_f32<PER>(f.h + j0, hv);
    // y as PER bf16 values and as PER floats, the reading that does not apply taken from h
    const uint8_t *yb = with_y ? static_cast<const uint8_t *>(f.y) : reinterpret_cast<const uint8_t *>(f.h);
    const uint8_t *hb = reinterpret_cast<const uint8_t *>(f.h);
    load_f32<PER>(reinterpret_cast<const float *>((bf16 ? hb : yb) + (size_t)j0 * 4), yv);
    float y16[PER];
    load_bf16<PER>(reinterpret_cast<const uint16_t *>((bf16 ? yb : hb) + (size_t)j0 * 2), y16);
    load_f32<PER>((f.a != nullptr ? f.a : f.h) + j0, av);
    if constexpr (CH > 0) {
      // wavefronts past the last gate row re-read the last row
      const int r0 = min(row0, N - 1);
      gate_prefetch<R, (CH > 0 ? CH : 1)>(gate_w, r0, max(1, min(R, N - r0)), lane, greg);
    }
#pragma unroll
    for (int i = 0; i < PER; ++i) {  // (masks, not a select: see below)
      const uint32_t mb = bf16 ? 0xffffffffu : 0u;
      yv[i] = __uint_as_float((__float_as_uint(y16[i]) & mb) | (__float_as_uint(yv[i]) & ~mb));
    }
  } else {
#pragma unroll
    for (int i = 0; i < kMaxPer; ++i) {
      const int j = tid + i * NT;
      hv[i] = yv[i] = av[i] = 0.f;
      if (j < d) {
        if (f.carry) hv[i] = f.h[j];
        if (with_y)
          yv[i] = bf16 ? __uint_as_float((uint32_t) static_cast<const uint16_t *>(f.y)[j] << 16)
                       : static_cast<const float *>(f.y)[j];
        if (f.a != nullptr) av[i] = f.a[j];
      }
    }
    if (wave == 0) cr = load_cache_regs(st, lane, N, p.capacity);
    if (CH > 0 && nrows > 0) gate_prefetch<R, (CH > 0 ? CH : 1)>(gate_w, row0, nrows, lane, greg);
  }

  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < (PRE ? 0 : kMaxPer); ++i) {
    const int j = PER > 0 ? tid * PER + i : tid + i * NT;
    if (PER > 0 || j < d) {
      float v;
      if constexpr (PER > 0) {
        // absent operands are masked to +0 with bit masks: a select or a branch lets the compiler sink the load
        // into it, and a load inside a branch makes the next wait cover all outstanding loads
        const uint32_t mh = f.carry ? 0xffffffffu : 0u, my = with_y ? 0xffffffffu : 0u,
                       ma = f.a != nullptr ? 0xffffffffu : 0u;
        v = __uint_as_float(__float_as_uint(hv[i]) & mh) + __uint_as_float(__float_as_uint(yv[i]) & my);
        v = __builtin_fmaf(f.perturb, __uint_as_float(__float_as_uint(av[i]) & ma), v);
      } else {
        v = hv[i];
        if (with_y) v += yv[i];
        if (f.a != nullptr) v = __builtin_fmaf(f.perturb, av[i], v);
      }
      hv[i] = v;
      ss = __builtin_fmaf(v, v, ss);
      if (PER == 0) f.h[j] = v;
    }
  }
  float tot = tot_pre;
  if constexpr (!PRE) {
    if constexpr (PER > 0) store_f32<PER>(f.h + tid * PER, hv);
    ss = wave_sum(ss);
    if (lane == 0) part_s[wave] = ss;
    __syncthreads();
    for (int w = 0; w < NW; ++w) tot += part_s[w];
  }
  const float scale = 1.0f / sqrtf(tot / (float)d + 1e-6f);
  if constexpr (PER > 0) {
    float xv[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) xv[i] = hv[i] * scale;
    const int j0 = tid * PER;
    if (bf16) {
      store_bf16<PER>(static_cast<uint16_t *>(f.x_out) + j0, xv);
      store_bf16<PER>(reinterpret_cast<uint16_t *>(x_s) + j0, xv);
    } else {
      store_f32<PER>(static_cast<float *>(f.x_out) + j0, xv);
      store_f32<PER>(reinterpret_cast<float *>(x_s) + j0, xv);
    }
  } else {
#pragma unroll
    for (int i = 0; i < kMaxPer; ++i) {
      const int j = tid + i * NT;
      if (j < d) {
        const float v = hv[i] * scale;
        if (bf16) {
          const uint16_t q = f32_to_bf16_rne(v);
          static_cast<uint16_t *>(f.x_out)[j] = q;
          reinterpret_cast<uint16_t *>(x_s)[j] = q;
        } else {
          static_cast<float *>(f.x_out)[j] = v;
          reinterpret_cast<float *>(x_s)[j] = v;
        }
      }
    }
  }
  // x is in LDS: a workgroup barrier that waits for the LDS writes only (__syncthreads would also wait for the gate
  // rows still on their way and for the stores of x)
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");

  // ---- gate GEMV on x in LDS ----------------------------------------------------------------------
  if (nrows > 0) {
    float v[R];
    if (CH > 0)
      gate_dot<R, (CH > 0 ? CH : 1)>(greg, x_s, p.act_fmt, lane, v);
    else
      gate_rows<R>(gate_w, x_s, row0, nrows, d, p.act_fmt, lane, v);
#pragma unroll
    for (int r = 0; r < R; ++r)
      if (lane == 0 && r < nrows) z_s[row0 + r] = v[r];
  }
  __syncthreads();
  if (wave != 0) return;
  route_wave(p, z_s, cr, st, out_dev, note, lds.rec_s, lane, flags);
}

// Workgroup 0 of an expert launch that carries the layer boundary (NW wavefronts; d = NW*64*PER with bf16
// activations): forms x, routes, hands the record on, writes its (empty) partial row, then touches what the next
// layer's boundary will read first.  `red` is the launch's reduction buffer in LDS, borrowed.
template <int NW, int CH, int PER>
__device__ __forceinline__ void boundary_workgroup(const GemvParams &p, float *red) {
  const int tid = threadIdx.x, d = p.hidden;
  fused_boundary<NW, CH, PER, true>(p.b.route, p.b.glue, p.b.gate_w, p.b.state, p.b.out_dev, p.b.note,
                                    BoundaryFlags{p.b.handover, p.b.hand_tag},
                                    carve_boundary_lds(reinterpret_cast<uint32_t *>(red)));
  float *row = p.partial + (int64_t)p.row_offset * d;  // this workgroup's partial row: nothing to add
  for (int j = tid; j < d; j += NW * kWave) row[j] = 0.f;
  if (p.b.next_gate_w != nullptr) {
    // this compute unit is idle for the rest of the launch: pull what the next boundary reads first towards it
    const u32x4 *g = static_cast<const u32x4 *>(p.b.next_gate_w);
    uint32_t acc = 0;
    for (int64_t i = tid; i < p.b.gate_bytes / 16; i += NW * kWave) {
      const u32x4 v = g[i];
      acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    for (int i = tid; i < (int)(sizeof(LayerState) / 4); i += NW * kWave)
      acc ^= reinterpret_cast<const uint32_t *>(p.b.next_state)[i];
    if (acc == 0x9e3779b9u && p.b.gate_bytes < 0) row[0] = 1.f;  // never true: keeps the loads
  }
}

}  // namespace rt
}  // namespace moe
