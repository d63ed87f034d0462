// Prompt phase: a batch of B tokens through one MoE layer (paper Sec. 4.5 applies the cache-aware routing during
// generation and lets prompt processing use batched kernels; App. F looks at the prompt length).  The routing of the
// batch is the routing of its tokens one after the other - the cache bitmask m_t of Sec. 3.3 is the state after
// token t-1, also inside a batch - so every decision, slot and miss count equals what B single-token steps give;
// only the arithmetic is batched: the gate logits of all tokens by one small GEMM, the experts by a
// weights-stationary small GEMM per expert over the tokens routed to it (Eq. 1), both on the matrix cores.
//
//  gate_gemm_kernel    logits[B, N] = X[B, d] W_gate[N, d]^T, bf16 inputs, fp32 accumulation
//                      (v_mfma_f32_16x16x32_bf16: a 16-token x 16-expert tile per eight wavefronts, which split d).
//  route_batch_kernel  sixteen wavefronts route sixteen tokens at a time through rt::route_wave against the current
//                      cache state; a token that misses an expert is routed alone and updates the state (see there);
//                      one routing record per token.
//  expert_batch_kernel one workgroup (8 wavefronts) per unit = (expert blob, up to 128 consecutive records, tile of up
//                      to 16 tokens routed to that expert).  Per block of 16 records: all its weights are requested
//                      at once; g, u = W_gate/up block x X tile^T with the 16x16x32 bf16 MFMA, the hidden dimension
//                      split over the wavefronts and summed through LDS; h = silu(g) u w; then the block's columns of
//                      W_down (the record layout keeps them as rows) are applied with the 16x16x4 fp32 MFMA, whose
//                      operands hold one value per lane, so the rows need no transposition; each wavefront owns d/8
//                      output columns and keeps their 16-token accumulators in registers over the whole unit.  Every
//                      unit writes its 16 x d tile to its own rows of a partial buffer.
//  reduce_batch_kernel adds each token's partial rows in a fixed order (deterministic y) and rounds to bf16.
#include <type_traits>

#include "common.h"
#include "gemv_common.h"
#include "route_device.h"

namespace moe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4 mfma_bf16(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma_f32(float a, float b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// ---- gate logits of the batch -------------------------------------------------------------------
// grid = (token tiles of 16, expert tiles of 16), block = kGateSplit wavefronts: wavefront ks multiplies the ks-th
// part of the hidden dimension, all its operands requested at once (one round trip); the parts are added through LDS
// in a fixed order.  A-operand lane l: token l % 16, columns k0 + 8 (l / 16) .. + 8; B-operand lane l: expert
// n0 + l % 16, the same columns; result lane l: expert n0 + l % 16, tokens 4 (l / 16) + v.  Rows past the last token /
// expert re-read the last one and are not stored.
constexpr int kGateSplit = 8;
// STEPS: 32-column steps per wavefront (hidden = 32 * kGateSplit * STEPS)
template <int STEPS>
__global__ __launch_bounds__(kGateSplit *kWave) void gate_gemm_kernel(const uint16_t *x, const uint16_t *gate_w,
                                                                     float *logits, int B, int N, int d) {
  __shared__ f32x4 part[kGateSplit][kWave];
  const int lane = threadIdx.x & 63, ks = threadIdx.x >> 6;
  const int t0 = blockIdx.x * 16, n0 = blockIdx.y * 16;
  const int tok = min(t0 + (lane & 15), B - 1), exp = min(n0 + (lane & 15), N - 1);
  const u32x4 *xa = reinterpret_cast<const u32x4 *>(x + (size_t)tok * d) + (lane >> 4) + (size_t)ks * STEPS * 4;
  const u32x4 *wb = reinterpret_cast<const u32x4 *>(gate_w + (size_t)exp * d) + (lane >> 4) + (size_t)ks * STEPS * 4;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  u32x4 a[STEPS], b[STEPS];
#pragma unroll
  for (int s = 0; s < STEPS; ++s) {
    a[s] = xa[s * 4];
    b[s] = wb[s * 4];
  }
#pragma unroll
  for (int s = 0; s < STEPS; ++s) acc = mfma_bf16(a[s], b[s], acc);
  part[ks][lane] = acc;
  __syncthreads();
  if (ks != 0) return;
#pragma unroll
  for (int q = 1; q < kGateSplit; ++q) {
    const f32x4 t = part[q][lane];
    acc[0] += t[0];
    acc[1] += t[1];
    acc[2] += t[2];
    acc[3] += t[3];
  }
  const int e = n0 + (lane & 15);
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int t = t0 + 4 * (lane >> 4) + v;
    if (t < B && e < N) logits[(size_t)t * N + e] = acc[v];
  }
}

// ---- routing of the batch ---------------------------------------------------------------------------
// The decisions are those of the tokens routed one after the other (the cache mask of Sec. 3.3 is the state after the
// previous token), but a token that misses nothing leaves the cache as it found it except for the recency stamps of
// its experts - and stamps only matter to a later miss.  So sixteen wavefronts route the next sixteen tokens at once
// against the current state (rt::route_wave, unchanged, its record kept in LDS); the tokens up to the first one that
// misses an expert are accepted as they are: records copied out, stamps merged (a later token's stamp is larger, so
// the merge is a maximum), counters advanced.  The token with the miss is then routed by one wavefront against the
// merged state, which it updates, and the window moves on behind it.  What does not depend on the cache - Eq. 10's
// running sum of logit ranges - is prepared for all tokens first (the same additions in the same order).
// Miss-free batches cost one round per sixteen tokens; a miss costs one extra round.
constexpr int kRouteWaves = 16;
struct BatchCacheState {  // LayerState's tables while the batch is routed (LDS)
  int32_t my_slot[MOE_MAX_EXPERTS], slot_exp[MOE_MAX_EXPERTS], born[MOE_MAX_EXPERTS];
  long long stamp[MOE_MAX_EXPERTS];
  long long counter[6];
  uint64_t ever_used;
  int32_t count0;  // tokens routed before this batch
};

__device__ __forceinline__ rt::CacheRegs batch_cache_regs(const BatchCacheState &s, int lane, int t, float dsum_prev) {
  rt::CacheRegs cr;
  cr.my_slot = s.my_slot[lane];
  cr.slot_exp = s.slot_exp[lane];
  cr.born = s.born[lane];
  cr.stamp = s.stamp[lane];
  cr.counter = lane < 6 ? s.counter[lane] : 0;
  cr.ever_used = s.ever_used;
  cr.t = s.count0 + t;
  cr.dsum_prev = dsum_prev;
  return cr;
}

__global__ __launch_bounds__(kRouteWaves *kWave) void route_batch_kernel(RouteParams p, const float *logits, int B,
                                                                         LayerState *st, moe_route_out_t *out) {
  __shared__ float z_all[kMaxBatch * MOE_MAX_EXPERTS];
  __shared__ float range_s[kMaxBatch];
  __shared__ float dsum_s[kMaxBatch + 1];  // Eq. 10's sum before token t
  __shared__ __attribute__((aligned(16))) uint32_t asm_s[kRouteWaves][rt::kRecWords];    // route_wave's work buffer
  __shared__ __attribute__((aligned(16))) uint32_t stage_s[kRouteWaves][rt::kRecWords];  // a wavefront's record
  __shared__ BatchCacheState cs;
  __shared__ int first_miss_s;
  const int tid = threadIdx.x, lane = tid & 63, N = p.n_experts, K = p.top_k;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  if (wave == 0) {
    const rt::CacheRegs cr = rt::load_cache_regs(st, lane, N, p.capacity);
    cs.my_slot[lane] = cr.my_slot;
    cs.slot_exp[lane] = cr.slot_exp;
    cs.born[lane] = cr.born;
    cs.stamp[lane] = cr.stamp;
    if (lane < 6) cs.counter[lane] = cr.counter;
    if (lane == 0) {
      cs.ever_used = cr.ever_used;
      cs.count0 = cr.t;
      dsum_s[0] = cr.dsum_prev;
    }
  }
  for (int i = tid; i < B * N; i += kRouteWaves * kWave) {
    const int t = i / N;
    z_all[t * MOE_MAX_EXPERTS + (i - t * N)] = logits[i];
  }
  __syncthreads();
  for (int t = wave; t < B; t += kRouteWaves) {
    const bool active = lane < N;
    const float z = active ? z_all[t * MOE_MAX_EXPERTS + lane] : 0.f;
    const float r = rt::wave_max(active ? z : -INFINITY) - rt::wave_min(active ? z : INFINITY);
    if (lane == 0) range_s[t] = r;
  }
  __syncthreads();
  if (tid == 0) {
#pragma clang fp contract(off)
    float acc = dsum_s[0];
    for (int t = 0; t < B; ++t) {
      acc = acc + range_s[t];
      dsum_s[t + 1] = acc;
    }
  }

  int t0 = 0;
  while (t0 < B) {  // (t0 and everything that steers the loop is the same in every thread)
    if (tid == 0) first_miss_s = B;
    __syncthreads();
    const int t = t0 + wave;
    rt::CacheRegs cr, next;
    if (t < B) {
      cr = batch_cache_regs(cs, lane, t, dsum_s[t]);
      int n_miss = 0;
      rt::route_wave(p, z_all + t * MOE_MAX_EXPERTS, cr, st, reinterpret_cast<moe_route_out_t *>(stage_s[wave]), nullptr,
                     asm_s[wave], lane, rt::BoundaryFlags{nullptr, 0}, &next, false, &n_miss);
      if (n_miss > 0 && lane == 0) atomicMin(&first_miss_s, t);
    }
    __syncthreads();
    const int window_end = min(t0 + kRouteWaves, B);
    const int fm = min(first_miss_s, window_end);  // tokens t0 .. fm-1 stand as they are
    if (t < fm) {
      if (lane < rt::kRecWords / 4)
        reinterpret_cast<u32x4 *>(out + t)[lane] = reinterpret_cast<const u32x4 *>(stage_s[wave])[lane];
      if (lane < N && next.stamp != cr.stamp) atomicMax(&cs.stamp[lane], (long long)next.stamp);
    }
    if (tid < 2) cs.counter[tid] += (long long)K * (fm - t0);  // selections and hits
    __syncthreads();
    t0 = fm;
    if (fm < window_end) {
      // token fm misses at least one expert: routed against the merged state, which it updates
      if (wave == 0) {
        cr = batch_cache_regs(cs, lane, fm, dsum_s[fm]);
        rt::route_wave(p, z_all + fm * MOE_MAX_EXPERTS, cr, st, out + fm, nullptr, asm_s[0], lane,
                       rt::BoundaryFlags{nullptr, 0}, &next, false);
        cs.my_slot[lane] = next.my_slot;
        cs.slot_exp[lane] = next.slot_exp;
        cs.born[lane] = next.born;
        cs.stamp[lane] = next.stamp;
        if (lane < 6) cs.counter[lane] = next.counter;
        if (lane == 0) cs.ever_used = next.ever_used;
      }
      t0 = fm + 1;
    }
  }
  __syncthreads();
  if (wave == 0) {
    if (lane < N) {
      st->expert_slot[lane] = cs.my_slot[lane];
      st->stamp[lane] = cs.stamp[lane];
      st->born[lane] = cs.born[lane];
    }
    if (lane < p.capacity) st->slot_expert[lane] = cs.slot_exp[lane];
    if (lane < 6) (&st->selections)[lane] = cs.counter[lane];
    if (lane == 0) {
      st->ever_used = cs.ever_used;
      st->delta_sum = dsum_s[B];
      st->count = cs.count0 + B;
    }
  }
}

// ---- experts of the batch ---------------------------------------------------------------------------
constexpr int kBatchWaves = 8;
constexpr int kXPad = 8;  // bf16 elements of padding per X row in LDS (16 bytes: rows start in different banks)

// CBW: blocks of 128 output columns per wavefront (d = 8 * 128 * CBW)
template <int CBW>
__global__ __launch_bounds__(kBatchWaves *kWave) void expert_batch_kernel(BatchParams p) {
  constexpr int NW = kBatchWaves;
  constexpr int D = NW * 128 * CBW;   // hidden size
  constexpr int KS = D / (NW * 32);   // 32-column steps of the gate / up products per wavefront
  constexpr int XS = D + kXPad;       // LDS row stride of the X tile, in bf16 elements
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  uint16_t *xs = reinterpret_cast<uint16_t *>(lds);                              // [16][XS] bf16
  f32x4 *red = reinterpret_cast<f32x4 *>(lds + 16 * XS * 2);                     // [2][NW][2][64]
  float *hs = reinterpret_cast<float *>(lds + 16 * XS * 2 + 2 * NW * 2 * 64 * 16);  // [NW][16][16]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int unit = p.unit_base + (int)blockIdx.x;
  const BatchUnit u = p.units[unit];
  const TokenTile *tile = p.tiles + u.tile;
  const int n_tok = tile->n;
  const uint8_t *blob = u.slot < 0 ? p.shared_blob : p.slot_pool + (int64_t)u.slot * p.slot_bytes;
  const int64_t row_bytes = (int64_t)D * 2, rec_bytes = 3 * row_bytes;
  const float wt = (lane & 15) < n_tok ? tile->w[lane & 15] : 0.f;  // weight of token lane % 16 for this expert


  f32x4 acc[CBW][8];
#pragma unroll
  for (int cb = 0; cb < CBW; ++cb)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[cb][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int m16 = lane & 15, kq = lane >> 4;
  float *hw = hs + wave * 256;
  // The loads of a block: gate and up rows for this wavefront's slice of the hidden dimension, and its columns of the
  // down rows.  They are requested as early as their registers are free - gate / up of the next block right after
  // this block's gate / up products, down of the next block right after this block's down products - so that the
  // barrier, the reduction and the arithmetic of a block overlap the transfer of the next.
  u32x4 ag[KS], au[KS], dn[4][CBW];
  auto load_gu = [&](int r0) {
    const uint8_t *row = blob + (int64_t)(r0 + m16) * rec_bytes + ((int64_t)wave * (D / NW) + kq * 8) * 2;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      // (plain loads, not the streaming ones: a load covers 64 bytes of each of 16 rows, and the other half of every
      // 128-byte line is wanted by the next step - with an L1 allocation it is found there; measured 10 % faster)
      ag[s] = *reinterpret_cast<const u32x4 *>(row + s * 64);
      au[s] = *reinterpret_cast<const u32x4 *>(row + row_bytes + s * 64);
    }
  };
  auto load_dn = [&](int r0) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const uint8_t *drow = blob + (int64_t)(r0 + 4 * s + kq) * rec_bytes + 2 * row_bytes +
                            ((int64_t)wave * (D / NW) + m16 * 8) * 2;
#pragma unroll
      for (int cb = 0; cb < CBW; ++cb) dn[s][cb] = stream_load(reinterpret_cast<const u32x4 *>(drow + cb * 256));
    }
  };
  const uint16_t *xrow = xs + m16 * XS + wave * (D / NW) + kq * 8;
  int parity = 0;
  // one block of 16 records; NEXT: there is a block after it, whose loads are requested on the way
  auto block = [&](int r_next, auto next_tag) {
    constexpr bool NEXT = decltype(next_tag)::value;
    // gate / up: this wavefront's slice of the hidden dimension
    f32x4 g = {0.f, 0.f, 0.f, 0.f}, up = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const u32x4 b = *reinterpret_cast<const u32x4 *>(xrow + s * 32);
      g = mfma_bf16(ag[s], b, g);
      up = mfma_bf16(au[s], b, up);
    }
    if constexpr (NEXT) load_gu(r_next);
    f32x4 *rb = red + (size_t)parity * (NW * 2 * 64);
    parity ^= 1;
    rb[(wave * 2 + 0) * 64 + lane] = g;
    rb[(wave * 2 + 1) * 64 + lane] = up;
    // (the buffer alternates between blocks, so one barrier per block is enough; it waits for LDS only, not for
    // the weight loads in flight)
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    g = rb[lane];
    up = rb[64 + lane];
#pragma unroll
    for (int w = 1; w < NW; ++w) {
      const f32x4 tg = rb[(w * 2 + 0) * 64 + lane], tu = rb[(w * 2 + 1) * 64 + lane];
      g += tg;
      up += tu;
    }
    // h for records 4 (lane / 16) + v and token lane % 16, stored as [record][token] for this wavefront
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const float h = g[v] / (1.f + __expf(-g[v])) * up[v] * wt;
      hw[(4 * kq + v) * 16 + m16] = h;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // down: y[token][column] += sum over the block's records of h[record][token] * W_down[column][record]
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const float a = hw[(4 * s + kq) * 16 + m16];  // A operand: token lane % 16, record 4 s + lane / 16
#pragma unroll
      for (int cb = 0; cb < CBW; ++cb) {
        const uint32_t w4[4] = {dn[s][cb].x, dn[s][cb].y, dn[s][cb].z, dn[s][cb].w};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const float b = (j & 1) ? bf16_hi(w4[j >> 1]) : bf16_lo(w4[j >> 1]);
          acc[cb][j] = mfma_f32(a, b, acc[cb][j]);
        }
      }
    }
    if constexpr (NEXT) load_dn(r_next);
    __builtin_amdgcn_wave_barrier();
  };
  // the first block's weights do not depend on the tokens: requested before the X tile is staged
  load_gu(u.rec0);
  load_dn(u.rec0);
  // X tile: row t = activations of the tile's t-th token (zeros past the last token); a thread's token indices first,
  // then all its chunks of x at once (two round trips in all)
  {
    constexpr int PT = 16 * (D / 8) / (NW * kWave);  // 16-byte chunks per thread
    int tok_of[PT];
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int t = (tid + i * NW * kWave) / (D / 8);
      tok_of[i] = tile->tok[t < n_tok ? t : 0];
    }
    u32x4 v[PT];
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int c = tid + i * NW * kWave, t = c / (D / 8), k8 = c - t * (D / 8);
      v[i] = *(reinterpret_cast<const u32x4 *>(p.x + (size_t)tok_of[i] * D) + k8);
      if (t >= n_tok) v[i] = u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int c = tid + i * NW * kWave, t = c / (D / 8), k8 = c - t * (D / 8);
      *reinterpret_cast<u32x4 *>(xs + t * XS + k8 * 8) = v[i];
    }
  }
  __syncthreads();
  for (int blk = 16; blk < u.n_rec; blk += 16) block(u.rec0 + blk, std::true_type{});
  block(0, std::false_type{});

  // The unit's tile goes to its own rows of the partial buffer (result lane l: tokens 4 (l / 16) + v, column
  // wave * d/8 + cb * 128 + (l % 16) * 8 + j); reduce_batch_kernel adds the tiles of a token in a fixed order.
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int t = 4 * kq + v;
    if (t < n_tok) {
      float *yrow = p.partial + ((size_t)unit * 16 + t) * D + wave * (D / NW) + m16 * 8;
#pragma unroll
      for (int cb = 0; cb < CBW; ++cb) {
        *reinterpret_cast<f32x4 *>(yrow + cb * 128) = f32x4{acc[cb][0][v], acc[cb][1][v], acc[cb][2][v], acc[cb][3][v]};
        *reinterpret_cast<f32x4 *>(yrow + cb * 128 + 4) = f32x4{acc[cb][4][v], acc[cb][5][v], acc[cb][6][v], acc[cb][7][v]};
      }
    }
  }
}

// y[t] = the sum of token t's partial rows, rounded to bf16.  contrib[t * max_contrib + i] is a row index into the
// partial buffer (unit * 16 + row of the token in the unit's tile); grid = (tokens, d / 256), eight wavefronts per
// workgroup: wavefront g adds the g-th eighth of the list in list order (several loads in flight), the eight sums are
// added in order of g - a fixed tree, so y does not change from run to run.
constexpr int kReduceGroups = 8;
__global__ __launch_bounds__(kReduceGroups *kWave) void reduce_batch_kernel(const float *partial, const int32_t *contrib,
                                                                           const int32_t *n_contrib, int max_contrib,
                                                                           uint16_t *y, int d, int t_first) {
  __shared__ f32x4 part_s[kReduceGroups][kWave];
  const int t = blockIdx.x, lane = threadIdx.x & 63, g = threadIdx.x >> 6;
  const int col = blockIdx.y * 256 + lane * 4;
  const int32_t *list = contrib + (size_t)t * max_contrib;
  const int n = n_contrib[t], chunk = (n + kReduceGroups - 1) / kReduceGroups;
  const int i0 = g * chunk, i1 = min(n, i0 + chunk);
  f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
  for (int i = i0; i < i1; ++i) s += *reinterpret_cast<const f32x4 *>(partial + (size_t)list[i] * d + col);
  part_s[g][lane] = s;
  __syncthreads();
  if (g != 0) return;
#pragma unroll
  for (int k = 1; k < kReduceGroups; ++k) s += part_s[k][lane];
  u32x2 o;
  o.x = (uint32_t)f32_to_bf16_rne(s[0]) | ((uint32_t)f32_to_bf16_rne(s[1]) << 16);
  o.y = (uint32_t)f32_to_bf16_rne(s[2]) | ((uint32_t)f32_to_bf16_rne(s[3]) << 16);
  *reinterpret_cast<u32x2 *>(y + (size_t)(t_first + t) * d + col) = o;
}

template <int CBW>
constexpr size_t batch_lds_bytes() {
  return (size_t)16 * (kBatchWaves * 128 * CBW + kXPad) * 2 + 2 * kBatchWaves * 2 * 64 * 16 + kBatchWaves * 256 * 4;
}

}  // namespace

bool batch_shape_supported(int weight_fmt, int act_fmt, int hidden, int inter, int shared_inter) {
  return weight_fmt == MOE_W_BF16 && act_fmt == MOE_A_BF16 && (hidden == 1024 || hidden == 2048) && inter % 16 == 0 &&
         shared_inter % 16 == 0;
}

hipError_t launch_gate_gemm(const void *x, const void *gate_w, float *logits, int B, int N, int hidden, hipStream_t s) {
  if (B <= 0 || N <= 0 || N > MOE_MAX_EXPERTS) return hipErrorInvalidValue;
  const dim3 g((B + 15) / 16, (N + 15) / 16), blk(kWave * kGateSplit);
  const uint16_t *xp = static_cast<const uint16_t *>(x), *wp = static_cast<const uint16_t *>(gate_w);
  if (hidden == 32 * kGateSplit * 8)
    hipLaunchKernelGGL(gate_gemm_kernel<8>, g, blk, 0, s, xp, wp, logits, B, N, hidden);
  else if (hidden == 32 * kGateSplit * 4)
    hipLaunchKernelGGL(gate_gemm_kernel<4>, g, blk, 0, s, xp, wp, logits, B, N, hidden);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_route_batch(const RouteParams &p, const float *logits, int B, LayerState *state, moe_route_out_t *out,
                              hipStream_t s) {
  if (B <= 0 || B > kMaxBatch) return hipErrorInvalidValue;
  hipLaunchKernelGGL(route_batch_kernel, dim3(1), dim3(kRouteWaves * kWave), 0, s, p, logits, B, state, out);
  return hipGetLastError();
}

// the kernel's LDS (X tile, partial sums, h) exceeds the default limit of a launch: raised once per instantiation
template <int CBW>
hipError_t launch_expert_batch_t(const BatchParams &p, hipStream_t s) {
  static bool raised = false;
  if (!raised) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&expert_batch_kernel<CBW>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)batch_lds_bytes<CBW>());
    if (e != hipSuccess) return e;
    raised = true;
  }
  hipLaunchKernelGGL(expert_batch_kernel<CBW>, dim3(p.n_units), dim3(kBatchWaves * kWave), batch_lds_bytes<CBW>(), s, p);
  return hipGetLastError();
}

hipError_t launch_expert_batch(const BatchParams &p, hipStream_t s) {
  if (p.n_units <= 0) return hipSuccess;
  if (p.hidden == 2048) return launch_expert_batch_t<2>(p, s);
  if (p.hidden == 1024) return launch_expert_batch_t<1>(p, s);
  return hipErrorInvalidValue;
}

hipError_t launch_reduce_batch(const float *partial, const int32_t *contrib, const int32_t *n_contrib, int max_contrib,
                               void *y, int hidden, int t_first, int n_tokens, hipStream_t s) {
  if (n_tokens <= 0) return hipSuccess;
  hipLaunchKernelGGL(reduce_batch_kernel, dim3(n_tokens, hidden / 256), dim3(kReduceGroups * kWave), 0, s, partial, contrib, n_contrib,
                     max_contrib, static_cast<uint16_t *>(y), hidden, t_first);
  return hipGetLastError();
}

}  // namespace moe
