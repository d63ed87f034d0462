// Internal declarations shared by the translation units of libmoe_cache (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "moe_cache.h"

namespace moe {

constexpr int kWave = 64;

// Per-layer cache state, device resident.  One wavefront owns it during a routing step:
// lane e holds expert e's entries, lane s holds slot s's entry.
struct LayerState {
  int32_t expert_slot[MOE_MAX_EXPERTS];  // expert -> slot, -1 = not resident
  int32_t slot_expert[MOE_MAX_EXPERTS];  // slot -> expert, -1 = empty
  int64_t stamp[MOE_MAX_EXPERTS];        // recency stamp per expert (valid while resident)
  int32_t born[MOE_MAX_EXPERTS];         // token at which the expert was loaded (valid while resident)
  uint64_t ever_used;                    // bit s: slot s has held an expert
  float delta_sum;                       // Eq. 10 accumulator
  int32_t count;                         // tokens routed
  int64_t selections, hits, misses, cold_misses, evictions, lifetime_sum;  // contiguous: updated lane-wise
};

struct RouteParams {
  int32_t n_experts, top_k, top_j, capacity, hidden;
  int32_t act_fmt, renormalize, delta_mode, route_mode, max_rank;
  float lambda, delta_fixed, cumsum_p;
  uint32_t seq;
};

// Glue of a stack fused in front of the router (see fused_route_kernel).
constexpr int kFusedMaxHidden = 8192;
struct FusedParams {
  const void *y;    // [d] act_fmt, the previous layer's expert output, or nullptr
  float *h;         // [d] fp32 residual stream, updated in place
  const float *a;   // [d] fp32 perturbation or nullptr
  float perturb;
  int32_t carry;    // 0: a new token starts, h = perturb * a
  void *x_out;      // [d] act_fmt, the normalised vector (input of this layer)
  // When the glue has been done by reduce_glue_kernel: h already holds the new residual stream and ss its sums
  // of squares over consecutive blocks of 64 columns (n_ss = d / 64 of them); y, a, perturb, carry are unused.
  const float *ss;
  int32_t n_ss;
};

// The layer boundary (x from the new residual stream + routing step, see rt::fused_boundary) when it is run by
// workgroup 0 of the expert launch itself: the other workgroups compute x for themselves, stream the shared
// expert's records meanwhile, and wait for its decision before the first routed record.
struct BoundaryArgs {
  RouteParams route;
  FusedParams glue;
  const void *gate_w;
  LayerState *state;
  moe_route_out_t *out_dev;  // the layer's device record (= GemvParams::route)
  struct HostNote *note;     // the layer's words in mapped host memory
  uint64_t *handover;        // the layer's self-tagged words with slots, miss flags and weights (8 copies of 8)
  uint32_t hand_tag;         // 16-bit tag of this hand-over: the count of the layer's hand-overs so far, so that
                             // what the words still hold (the previous one) can never pass for it
  uint32_t *gave_up;         // mapped host word set when a wavefront stopped waiting for the hand-over
  int spin_limit;            // polls of the hand-over before a wavefront stops waiting (a test lowers it)
  // what the boundary of the layer that follows will read first (its gate matrix and cache state): workgroup 0
  // touches it once its own work is done, which measurably shortens that boundary (nullptr: don't)
  const void *next_gate_w;
  const LayerState *next_state;
  int64_t gate_bytes;
};

struct GemvParams {
  const uint8_t *slot_pool;      // this layer's slots
  const uint8_t *shared_blob;    // or nullptr
  const moe_route_out_t *route;  // device record of the layer's routing step (slots, weights, miss flags)
  const void *x;                 // [d] act_fmt
  float *partial;                // [grid][d] fp32
  int32_t hidden, inter, shared_inter, top_k, act_fmt;
  int64_t slot_bytes;
  int32_t pass;        // 0: shared expert + experts that were resident; 1: experts whose slot was just filled
  int32_t row_offset;  // first partial row this launch writes
  int32_t fused;       // workgroup 0 runs the layer boundary `b` and writes a zero partial row
  BoundaryArgs b;
};

// Blob geometry (see moe_blob_bytes).
struct BlobLayout {
  int64_t rec_bytes;    // bytes of one record (gate row | up row | down column [| inline scales])
  int64_t row_bytes;    // bytes of one d-long row of weights
  int64_t tail_offset;  // start of the out-of-record scales
  int64_t total;        // whole blob, multiple of 256
};
BlobLayout blob_layout(int fmt, int hidden, int inter);
// int4: bytes of one record - three rows of nibbles and the record's (gate, up) fp16 scale pairs, one pair per group of
// 128 columns, padded so that every record starts on a 128-byte line (a wavefront's 1 KB load then covers 8 lines, not 9)
__host__ __device__ constexpr int64_t int4_record_bytes(int64_t d) { return 3 * (d / 2) + ((d / 128) * 4 + 127) / 128 * 128; }

// What the host needs of a routing decision, written by the router into mapped host memory as three 8-byte words,
// each complete in itself (no ordering between them is assumed):
//   w[0] = seq | n_miss << 32 | miss flags by selection position << 40
//   w[1] = (seq & 0xffff) | expert of position k << (16 + 6k)
//   w[2] = (seq & 0xffff) | slot of position k   << (16 + 6k)
// The host has the decision once all three carry the tag of the step it waits for.
struct HostNote {
  uint64_t w[4];
};

// launchers (each returns the hipError_t of the launch)
hipError_t launch_route(const RouteParams &p, const void *gate_w, const void *x, const float *logits,
                        LayerState *state, moe_route_out_t *out_dev, HostNote *note_mapped,
                        hipStream_t s);
// launch shape of the expert GEMV
constexpr int kGemvWaves = 8;  // wavefronts per workgroup
constexpr int kGemvDepth = 2;  // records in flight per wavefront (fp32 / bf16 kernels)
struct GemvPlan {
  int grid;   // workgroups (= fp32 partial rows written): one per compute unit
  bool dot2;  // packed bf16 dot products (bf16 weights and activations)
};
GemvPlan gemv_plan(int n_cus, int total_records, int weight_fmt, int act_fmt);
bool gemv_fused_supported(int weight_fmt, int act_fmt, int hidden, const GemvPlan &plan);  // a launch variant with the boundary in workgroup 0
// f.ss != nullptr: the glue has been done by launch_reduce_glue (needs fused_route_pre_supported(hidden))
bool fused_route_pre_supported(int hidden);
hipError_t launch_fused_route(const RouteParams &p, const FusedParams &f, const void *gate_w, LayerState *state,
                              moe_route_out_t *out_dev, HostNote *note_mapped, hipStream_t s);
hipError_t launch_expert_gemv(const GemvParams &p, int weight_fmt, const GemvPlan &plan, hipStream_t s,
                              hipEvent_t start = nullptr, hipEvent_t stop = nullptr);
hipError_t launch_partial_reduce(const float *partial, int n_partial, void *y, int hidden, int act_fmt,
                                 hipStream_t s);
// the same plus the residual glue: h = (carry ? h + y : 0) + perturb * a in place, ss[b] = sum of h^2 over columns
// 64b .. 64b+63 (y may be NULL: not stored; n_partial may be 0: y = nothing)
hipError_t launch_reduce_glue(const float *partial, int n_partial, void *y, int hidden, int act_fmt, float *h,
                              const float *a, float perturb, int carry, float *ss, hipStream_t s);
hipError_t launch_pack(int fmt, int hidden, int inter, const void *gate, const void *up, const void *down,
                       const void *gs, const void *us, const void *ds, void *blob, hipStream_t s);
hipError_t launch_residual_rmsnorm(float *h, const void *y, const float *a, float perturb, int carry, void *x,
                                   int hidden, int act_fmt, hipStream_t s);
hipError_t launch_state_init(LayerState *state, int n_layers, const int32_t *initial_dev, int n_initial,
                             hipStream_t s);
// ---- prompt phase (expert_batch.hip): a batch of tokens through one layer ----
constexpr int kMaxBatch = 128;        // tokens per moe_route_batch / moe_expert_forward_batch call
// records of one expert handled by one workgroup of the batched expert kernel: the host picks a multiple of 16 between
// kBatchMinUnitRecords and kBatchMaxUnitRecords per launch; buffers are sized for kBatchUnitRecords and up
constexpr int kBatchUnitRecords = 128;
constexpr int kBatchMinUnitRecords = 32;
constexpr int kBatchMaxUnitRecords = 512;
// up to 16 tokens routed to one expert (or any 16 tokens, for the shared expert) and their weights for it
struct TokenTile {
  int32_t tok[16];
  float w[16];
  int32_t n, pad[3];
};
// one workgroup's work: n_rec (a multiple of 16) records from rec0 of the expert in `slot` (-1: the shared expert),
// applied to the tokens of tile `tile`
struct BatchUnit {
  int32_t slot, rec0, n_rec, tile;
};
struct BatchParams {
  const uint8_t *slot_pool, *shared_blob;
  const uint16_t *x;  // [B, d] bf16
  float *partial;     // [n_units][16][d] fp32: every unit's output tile
  const BatchUnit *units;
  const TokenTile *tiles;
  int32_t hidden, inter, shared_inter;
  int32_t n_units, unit_base;  // the launch covers units unit_base .. unit_base + n_units - 1
  int64_t slot_bytes;
};
bool batch_shape_supported(int weight_fmt, int act_fmt, int hidden, int inter, int shared_inter);
hipError_t launch_gate_gemm(const void *x, const void *gate_w, float *logits, int B, int N, int hidden, hipStream_t s);
hipError_t launch_route_batch(const RouteParams &p, const float *logits, int B, LayerState *state, moe_route_out_t *out,
                              hipStream_t s);
hipError_t launch_expert_batch(const BatchParams &p, hipStream_t s);
// y[t_first + t] = sum of the partial rows contrib[t][0 .. n_contrib[t]) in that order, for t < n_tokens
hipError_t launch_reduce_batch(const float *partial, const int32_t *contrib, const int32_t *n_contrib, int max_contrib,
                               void *y, int hidden, int t_first, int n_tokens, hipStream_t s);

// the allocation-free entry point (expert_static.hip): device address of its fixed scratch array and the compute-unit
// count of device `dev` (which must be current), looked up once per device
hipError_t static_scratch_setup(int dev, void **ptr, int *cus);
hipError_t launch_expert_forward_static(int weight_fmt, int act_fmt, int hidden, int inter, int shared_inter, int top_k,
                                        const void *slot_pool, int64_t slot_bytes, const void *shared_blob,
                                        const int32_t *sel_slot, const float *sel_weight, const void *x, void *y,
                                        hipStream_t s);
int static_max_hidden();
bool gemv_shape_supported(int weight_fmt, int hidden);
bool gemv_inter_supported(int weight_fmt, int inter);
hipError_t launch_expert_gemv_quant(const GemvParams &p, int weight_fmt, const GemvPlan &plan, hipStream_t s,
                                    hipEvent_t start, hipEvent_t stop);

// ---- device helpers -------------------------------------------------------------------------
#if defined(__HIPCC__)
__device__ __forceinline__ float bf16_lo(uint32_t v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t v) { return __uint_as_float(v & 0xffff0000u); }
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
// Sum over the 64 lanes, result in every lane, fixed order (rotations inside rows of 16, then rows).
// Sum of N <= 64 floats in index order, the same in every wavefront that computes it: fetch() has lane i load
// entry i (clamped: no branch around the load), total() adds the entries one by one through lane reads.  N is a
// compile-time constant so that neither part ends up inside a branch.
template <int N>
struct OrderedSum {
  static_assert(N >= 1 && N <= 64, "one entry per lane");
  float s;
  __device__ __forceinline__ void fetch(const float *v, int lane) { s = v[lane < N ? lane : 0]; }
  __device__ __forceinline__ float total() const {
    float tot = 0.f;
#pragma unroll
    for (int i = 0; i < N; ++i) tot += __int_as_float(__builtin_amdgcn_readlane(__float_as_int(s), i));
    return tot;
  }
};

__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f32<0x128>(v);  // row_ror:8
  v += dpp_f32<0x124>(v);  // row_ror:4
  v += dpp_f32<0x122>(v);  // row_ror:2
  v += dpp_f32<0x121>(v);  // row_ror:1
  float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
  float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
  float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
  float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
  return (r0 + r1) + (r2 + r3);
}
#endif

}  // namespace moe
