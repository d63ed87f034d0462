// Fused router kernel: gate GEMV, softmax, logit range, cache prior, top-K, hit/miss accounting,
// LRU slot-table update (paper Eq. 3, Eq. 10, Eq. 9, Eq. 2, Eq. 4, Sec. 4.2), one launch per layer-token.
//
// This file is compiled with floating-point contraction off: the steps that decide which expert is
// selected are single fp32 operations in a fixed order (subtract, add, divide, multiply, add), so the
// decisions are reproducible bit for bit from the same fp32 logits.
//
// Layout of the work: one workgroup.  All its wavefronts compute rows of z = W_gate x (128-bit loads, up to
// four rows per wavefront with all their loads in flight together, fp32 accumulation, DPP reduction);
// wavefront 0 then does the routing with lane e <-> expert e and lane s <-> slot s (N <= 64, C <= 64),
// entirely in registers.  Rankings are counted with one 64-bit compare per pair: the key is the logit
// mapped to an order-preserving unsigned integer, with 63 - lane below it so that equal logits rank the
// lower index first.  What the host needs (experts, slots, miss flags) goes to host-mapped memory as three
// self-tagged 8-byte words, each complete in itself, as soon as the victims are known; the full decision record is
// assembled in LDS and written with 16-byte stores to device memory.
#include "route_device.h"

namespace moe {
namespace {

using namespace rt;


__global__ __launch_bounds__(1024) void route_kernel(RouteParams p, const void *gate_w, const void *x,
                                                     const float *logits_in, LayerState *st,
                                                     moe_route_out_t *out_dev, HostNote *note) {
  __shared__ float z_s[MOE_MAX_EXPERTS];
  __shared__ __attribute__((aligned(16))) uint32_t rec_s[kRecWords];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), n_waves = blockDim.x >> 6;
  const int N = p.n_experts;

  // wavefront 0 owns the cache state; its loads are issued before the GEMV so their latency overlaps it
  CacheRegs cr{};
  if (wave == 0) cr = load_cache_regs(st, lane, N, p.capacity);

  if (logits_in != nullptr) {
    if (tid < N) z_s[tid] = logits_in[tid];
  } else {
    gate_gemv(gate_w, x, p, wave, n_waves, lane, z_s);
  }
  __syncthreads();
  if (wave != 0) return;
  route_wave(p, z_s, cr, st, out_dev, note, rec_s, lane);
}


// The layer boundary as a launch of its own (one workgroup of 16 wavefronts): see fused_boundary.  PRE: the residual
// glue and the sums of squares were left by reduce_glue_kernel; the boundary starts from h.
template <int CH, int PER, bool PRE>
__global__ __launch_bounds__(1024) void fused_route_kernel(RouteParams p, FusedParams f, const void *gate_w,
                                                           LayerState *st, moe_route_out_t *out_dev,
                                                           HostNote *note) {
  __shared__ __attribute__((aligned(16))) uint32_t lds[kBoundaryLdsWords];
  fused_boundary<16, CH, PER, PRE>(p, f, gate_w, st, out_dev, note, BoundaryFlags{nullptr, 0},
                                   carve_boundary_lds(lds));
}

__global__ void state_init_kernel(LayerState *state, int n_layers, const int32_t *initial, int n_initial) {
  const int layer = blockIdx.x, lane = threadIdx.x;
  if (layer >= n_layers) return;
  LayerState *st = state + layer;
  st->expert_slot[lane] = -1;
  st->slot_expert[lane] = -1;
  st->stamp[lane] = 0;
  st->born[lane] = 0;
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
    st->selections = st->hits = st->misses = st->cold_misses = st->evictions = st->lifetime_sum = 0;
  }
}

}  // namespace

hipError_t launch_route(const RouteParams &p, const void *gate_w, const void *x, const float *logits,
                        LayerState *state, moe_route_out_t *out_dev, HostNote *note_mapped,
                        hipStream_t s) {
  // at most four rows of the gate matrix per wavefront, so that all of a wavefront's loads are in flight at once
  int waves = logits ? 1 : (p.n_experts + 3) / 4;
  if (waves > 16) waves = 16;
  if (waves < 1) waves = 1;
  hipLaunchKernelGGL(route_kernel, dim3(1), dim3(waves * kWave), 0, s, p, gate_w, x, logits, state, out_dev,
                     note_mapped);
  return hipGetLastError();
}

// hidden sizes for which the boundary can start from what reduce_glue_kernel leaves: 16 wavefronts x PER columns
// per thread with PER in {1, 2, 4}, one sum of squares per 64 columns
bool fused_route_pre_supported(int hidden) { return hidden == 1024 || hidden == 2048 || hidden == 4096; }

hipError_t launch_fused_route(const RouteParams &p, const FusedParams &f, const void *gate_w, LayerState *state,
                              moe_route_out_t *out_dev, HostNote *note_mapped, hipStream_t s) {
  if (p.hidden > kFusedMaxHidden || p.hidden % 8 != 0) return hipErrorInvalidValue;
  // 16 wavefronts, at most four gate rows each (N <= 64)
  const dim3 g(1), b(1024);
  const int vec = p.act_fmt == MOE_A_BF16 ? 8 : 4;
  int ch = p.hidden % (kWave * vec) == 0 ? p.hidden / (kWave * vec) : 0;
  if (ch != 1 && ch != 2 && ch != 4) ch = 0;  // more than 4 chunks per row: gate rows are not held in registers
  const int per = (p.hidden % 1024 == 0 && (p.hidden / 1024 == 1 || p.hidden / 1024 == 2 || p.hidden / 1024 == 4))
                      ? p.hidden / 1024 : 0;
  const bool pre = f.ss != nullptr;
  if (pre && !fused_route_pre_supported(p.hidden)) return hipErrorInvalidValue;
#define MOE_FUSED(CH_, PER_, PRE_)                                                                              \
  hipLaunchKernelGGL((fused_route_kernel<CH_, PER_, PRE_>), g, b, 0, s, p, f, gate_w, state, out_dev, note_mapped)
#define MOE_FUSED2(CH_, PER_)                                                                                   \
  do {                                                                                                          \
    if (pre) MOE_FUSED(CH_, PER_, true);                                                                        \
    else MOE_FUSED(CH_, PER_, false);                                                                           \
  } while (0)
  switch (ch * 10 + per) {  // (bf16: d = 512 ch; fp32: d = 256 ch)
    case 42: MOE_FUSED2(4, 2); break;         // bf16 d = 2048
    case 41: MOE_FUSED2(4, 1); break;         // fp32 d = 1024
    case 21: MOE_FUSED2(2, 1); break;         // bf16 d = 1024
    case 20: MOE_FUSED(2, 0, false); break;   // fp32 d = 512
    case 10: MOE_FUSED(1, 0, false); break;   // bf16 d = 512, fp32 d = 256
    default:
      if (per == 2) MOE_FUSED2(0, 2);         // fp32 d = 2048
      else if (per == 4) MOE_FUSED2(0, 4);    // d = 4096
      else MOE_FUSED(0, 0, false);
  }
#undef MOE_FUSED2
#undef MOE_FUSED
  return hipGetLastError();
}

hipError_t launch_state_init(LayerState *state, int n_layers, const int32_t *initial_dev, int n_initial,
                             hipStream_t s) {
  hipLaunchKernelGGL(state_init_kernel, dim3(n_layers), dim3(MOE_MAX_EXPERTS), 0, s, state, n_layers, initial_dev,
                     n_initial);
  return hipGetLastError();
}

}  // namespace moe
