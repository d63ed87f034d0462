// Device helpers shared by the expert GEMV kernels (all weight formats).
#pragma once

#include "common.h"

namespace moe {

constexpr int kRedFloats = 16384;  // LDS floats (64 KB) shared by the wavefronts' rows in the final reduction

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// weights are read once: mark the loads non-temporal so they do not displace x and the partial rows in L2
__device__ __forceinline__ u32x4 stream_load(const u32x4 *p) { return __builtin_nontemporal_load(p); }

__device__ __forceinline__ float dot2_bf16(uint32_t w, uint32_t x, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), __builtin_bit_cast(bf16x2, x), acc, false);
}

// sums a and b over the wavefront (both results in every lane), the two chains interleaved
__device__ __forceinline__ void wave_sum2(float &a, float &b) {
  a += dpp_f32<0x128>(a);
  b += dpp_f32<0x128>(b);
  a += dpp_f32<0x124>(a);
  b += dpp_f32<0x124>(b);
  a += dpp_f32<0x122>(a);
  b += dpp_f32<0x122>(b);
  a += dpp_f32<0x121>(a);
  b += dpp_f32<0x121>(b);
  float a0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(a), 0));
  float a1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(a), 16));
  float a2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(a), 32));
  float a3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(a), 48));
  float b0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(b), 0));
  float b1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(b), 16));
  float b2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(b), 32));
  float b3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(b), 48));
  a = (a0 + a1) + (a2 + a3);
  b = (b0 + b1) + (b2 + b3);
}


// Walks the records one wavefront owns in one launch.
//
// Every workgroup owns a share of the shared expert's records followed by a share of the routed records (the K
// selected slots side by side, I records each); its wavefronts take list entries wave, wave+NW, ...  Shared
// records need nothing from the routing step, so streaming starts at once while the loads of the routing
// record are in flight; the record is unpacked when the first routed entry comes up.  Pass 0 covers the
// shared expert and the experts that were resident; pass 1 covers only the experts whose slots were filled
// for this token, so the first pass can run while the fills stream.
//
// Shares are equal and fixed.  With equal shares the workgroups do not finish together: the mean finish time of
// a workgroup depends on its XCD (about 1.4 us between the fastest and the slowest of 8, the same from launch to
// launch, nothing else systematic), plus about 0.9 us of launch-to-launch noise.  Neither of the two remedies
// pays: handing records out dynamically with device-scope atomics is far slower (an atomic on a contended
// address costs about 200 ns while HBM is saturated), and shares proportional to measured per-XCD rates (or
// skewed by XCD parity) leave the kernel time unchanged - the XCDs that finish early free bandwidth for the
// late ones, so the spread is not lost time.  Fixed shares keep the summation order of y, hence y itself,
// identical from run to run.
__device__ __forceinline__ u32x4 ld128(const void *p) { return *static_cast<const u32x4 *>(p); }
__device__ __forceinline__ u32x2 ld64(const void *p) { return *static_cast<const u32x2 *>(p); }

// FUSED: workgroup 0 of the launch runs the layer boundary; the records are shared among workgroups 1..G-1 and
// the decision is fetched only when the first routed entry comes up, once workgroup 0 has handed it over.
// STEP: distance between a wavefront's consecutive list entries.  NW (the default) interleaves the wavefronts over
// the workgroup's list; 1 gives every wavefront one contiguous block of it, so that its records stay inside one
// expert and, for int4, inside one scale group of 128 records as far as possible.
//
// The walk is organised in runs - consecutive entries of the wavefront inside one blob (the shared expert, or one
// selected expert) - so that the per-record work is an increment and a decrement; slot, weight and the split of the
// routed index into (expert, row) are worked out once per run.  All of it is wavefront-uniform (scalar registers).
template <int NW, bool FUSED = false, int STEP = NW>
struct RecordWalker {
  static_assert(STEP == NW || STEP == 1, "interleaved or blocked");
  int sh_at, n_sh;   // the wavefront's shared records: first row, how many (not yet started)
  int r, n_rt;       // its routed entries: next index into the K*I routed records, how many are left to start
  int left;          // records left in the current run
  int next_at;       // row of the current run's next record
  bool run_wanted;   // the pass covers the current run's expert
  bool decided;      // the routing decision has been unpacked
  // the routing record: loaded at kernel start, unpacked when the first routed run comes up
  u32x4 rw0, rw1, rd;  // sel_weight[0..3], sel_weight[4..7], {tag, slots lo, slots hi, miss mask}
  uint64_t slots;
  uint32_t miss_mask;
  // the record found by step() / next()
  const uint8_t *base;  // blob of the record's expert
  int rows, at;
  float wt;

  // start of part b of n records split into G parts (b * n < 2^32: the host limits n to 2^22 and G to 2^10)
  static __device__ __forceinline__ int bound(int b, int n, int G) {
    return (int)((uint32_t)b * (uint32_t)n / (uint32_t)G);
  }

  // The record is the same for every lane and was written by an earlier launch: it is read through the scalar data
  // path (constant address space), whose completion is counted apart from the vector loads - waiting for it does not
  // wait for the weight loads already queued, and the values arrive in scalar registers.
  __device__ __forceinline__ void load_record(const GemvParams &p) {
    typedef const __attribute__((address_space(4))) u32x4 *cvec;
    cvec rr = (cvec)(reinterpret_cast<uintptr_t>(p.route));
    rw0 = rr[offsetof(moe_route_out_t, sel_weight) / 16];
    rw1 = rr[offsetof(moe_route_out_t, sel_weight) / 16 + 1];
    rd = rr[offsetof(moe_route_out_t, opaque) / 16];
  }

  // FUSED: the decision as workgroup 0 of this launch hands it over - eight 8-byte words, each carrying the
  // hand-over's 16-bit tag beside 48 bits of payload (layout: rt::BoundaryFlags).  The words are taken only when all
  // eight carry the tag, whatever order their stores arrived in; re-read until they do, at most spin_limit times.
  // No agent-scope acquire is involved (it would invalidate the XCD's L2 under thirty-two streaming compute
  // units - measured: the launch ran at half speed): the words are read with agent-scope atomic loads.
  __device__ __forceinline__ bool load_handover(const uint64_t *words, uint32_t tag, int spin_limit) {
    const uint32_t want = tag & 0xffffu;
    for (int i = 0; i < spin_limit; ++i) {
      uint64_t q[8];
      uint32_t tags_ok = 1;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        q[j] = __hip_atomic_load(words + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        tags_ok &= (uint32_t)(((uint32_t)q[j] & 0xffffu) == want);
      }
      if (__builtin_amdgcn_readfirstlane((int)tags_ok)) {
        // the same in every lane: kept in scalar registers from here on
#pragma unroll
        for (int j = 0; j < 8; ++j)
          q[j] = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(q[j] >> 32)) << 16) |
                 (uint64_t)((uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)q[j]) >> 16);
        rd.x = tag;
        rd.y = (uint32_t)q[0];
        rd.z = (uint32_t)(q[0] >> 32) | ((uint32_t)(q[1] & 0xffffu) << 16);
        rd.w = (uint32_t)(q[1] >> 16) & 0xffu;
        rw0.x = (uint32_t)q[2];
        rw0.y = (uint32_t)(q[2] >> 32) | ((uint32_t)q[3] << 16);
        rw0.z = (uint32_t)(q[3] >> 16);
        rw0.w = (uint32_t)q[4];
        rw1.x = (uint32_t)(q[4] >> 32) | ((uint32_t)q[5] << 16);
        rw1.y = (uint32_t)(q[5] >> 16);
        rw1.z = (uint32_t)q[6];
        rw1.w = (uint32_t)(q[6] >> 32) | ((uint32_t)q[7] << 16);
        return true;
      }
      __builtin_amdgcn_s_sleep(2);
    }
    return false;
  }

  __device__ __forceinline__ void init(const GemvParams &p, int wave) {
    const int G = FUSED ? (int)gridDim.x - 1 : (int)gridDim.x, b = FUSED ? (int)blockIdx.x - 1 : (int)blockIdx.x;
    // the routing record first: it is on its way while the shared records are set up
    if constexpr (!FUSED) load_record(p);
    const int routed = p.top_k * p.inter;
    const int shared = p.pass == 0 ? p.shared_inter : 0;
    // the workgroup's list: ns shared records from row s0, then nr routed entries from q0
    const int s0 = bound(b, shared, G), ns = bound(b + 1, shared, G) - s0;
    const int q0 = bound(b, routed, G), nl = ns + bound(b + 1, routed, G) - q0;
    int first_sh, first_rt;  // list indices
    if constexpr (STEP == 1) {
      const int lb = wave * nl / NW, le = (wave + 1) * nl / NW;
      first_sh = lb;
      n_sh = max(0, min(le, ns) - lb);
      first_rt = max(lb, ns);
      n_rt = max(0, le - first_rt);
    } else {
      first_sh = wave;
      n_sh = wave < ns ? (ns - wave + NW - 1) / NW : 0;
      first_rt = wave + n_sh * NW;
      n_rt = first_rt < nl ? (nl - first_rt + NW - 1) / NW : 0;
    }
    sh_at = s0 + first_sh;
    r = q0 + (first_rt - ns);
    left = 0;
    next_at = 0;
    run_wanted = true;
    decided = false;
  }

  // masks instead of a select chain: a chain over adjacent members is turned into an indexed load from a
  // memory copy of the struct, which then lives in scratch
  __device__ __forceinline__ float pick_weight(int k) const {
    uint32_t v = 0;
    v |= rw0.x & (0u - (uint32_t)(k == 0));
    v |= rw0.y & (0u - (uint32_t)(k == 1));
    v |= rw0.z & (0u - (uint32_t)(k == 2));
    v |= rw0.w & (0u - (uint32_t)(k == 3));
    v |= rw1.x & (0u - (uint32_t)(k == 4));
    v |= rw1.y & (0u - (uint32_t)(k == 5));
    v |= rw1.z & (0u - (uint32_t)(k == 6));
    v |= rw1.w & (0u - (uint32_t)(k == 7));
    return __uint_as_float(v);
  }

  // list entries this wavefront still owns
  __device__ __forceinline__ int remaining() const { return left + n_sh + n_rt; }

  // the wavefront's next run (there must be one): its shared records first, then its routed entries expert by expert
  __device__ __forceinline__ void start_run(const GemvParams &p) {
    if (n_sh > 0) {
      base = p.shared_blob;
      rows = p.shared_inter;
      next_at = sh_at;
      left = n_sh;
      n_sh = 0;
      wt = 1.f;
      run_wanted = true;
      return;
    }
    if (!decided) {  // first routed run: unpack the routing record
      bool ok = true;
      if constexpr (FUSED) {
        // (one wavefront per workgroup fetching for all eight through LDS was measured: no faster)
        ok = load_handover(p.b.handover + 8 * ((int)blockIdx.x % 8), p.b.hand_tag, p.b.spin_limit);
      }
      slots = (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)rd.y) |
              ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)rd.z) << 32);
      miss_mask = (uint32_t)__builtin_amdgcn_readfirstlane((int)rd.w);
      if (!ok) {  // no record: read slot 0 and use nothing of it
        slots = 0;
        miss_mask = p.pass == 1 ? 0u : ~0u;
        *p.b.gave_up = 1u;
      }
      decided = true;
    }
    const int I = p.inter;
    const int seg = (int)((uint32_t)r / (uint32_t)I), row = r - seg * I;
    const int in_seg = (I - row + STEP - 1) / STEP;  // this wavefront's entries inside expert `seg` from here on
    left = min(in_seg, n_rt);
    n_rt -= left;
    r += left * STEP;
    base = p.slot_pool + (int64_t)((slots >> (8 * seg)) & 0xffu) * p.slot_bytes;
    rows = I;
    next_at = row;
    wt = pick_weight(seg);
    run_wanted = (((miss_mask >> seg) & 1u) != 0) == (p.pass == 1);
  }

  // Move to this wavefront's next list entry (there must be one: see remaining()) and describe its record, whether
  // the pass covers it or not; returns whether it does.  The caller loads the record in any case, so that the
  // number of loads in flight does not depend on the routing decision, and only skips the arithmetic.
  __device__ __forceinline__ bool step(const GemvParams &p) {
    if (left == 0) start_run(p);
    at = next_at;
    next_at += STEP;
    --left;
    return run_wanted;
  }

  // advance to this wavefront's next record of the pass, skipping the others; false when the list is exhausted
  __device__ __forceinline__ bool next(const GemvParams &p) {
    for (;;) {
      if (left == 0) {
        if (n_sh + n_rt == 0) return false;
        start_run(p);
      }
      if (run_wanted) {
        at = next_at;
        next_at += STEP;
        --left;
        return true;
      }
      left = 0;  // the pass does not cover this expert: drop the whole run
    }
  }
};

// Sum the wavefronts' private outputs through LDS (one barrier per pass) and write the workgroup's fp32
// partial row.  y holds, for load index c and v < VEC, column (c*64 + lane)*VEC + v at y[c*VEC + v].
// Slot (cv*64 + lane) of a wavefront's LDS row holds 4 columns with cv = c_in_pass*(VEC/4) + v4, so
// consecutive lanes hit consecutive 16-byte slots.  Wavefronts are added in index order (deterministic).
template <int NW, int VEC, int LPR>
__device__ __forceinline__ void reduce_and_store(const float *y, float *red, float *out, int tid, int lane, int wave) {
  constexpr int kRedCols = kRedFloats / NW;      // columns per LDS pass
  constexpr int CBF = kRedCols / (kWave * VEC);  // load indices c per pass (0 if a chunk exceeds a pass)
  constexpr int CB = CBF > 0 ? CBF : 1;
  static_assert(CBF > 0, "one 16-byte chunk per lane must fit an LDS pass");
  constexpr int PASSES = (LPR + CB - 1) / CB;
  constexpr int CPP = (LPR < CB ? LPR : CB);  // c per pass actually present
  constexpr int SLOTS = kRedCols / 4;         // float4 slots per wavefront row
  float4 *red4 = reinterpret_cast<float4 *>(red);
#pragma unroll
  for (int ps = 0; ps < PASSES; ++ps) {
    if (ps > 0) __syncthreads();
    float4 *dst = red4 + wave * SLOTS;
#pragma unroll
    for (int cc = 0; cc < CPP; ++cc)
#pragma unroll
      for (int v4 = 0; v4 < VEC / 4; ++v4) {
        const int j = (ps * CB + cc) * VEC + v4 * 4;
        dst[(cc * (VEC / 4) + v4) * kWave + lane] = make_float4(y[j], y[j + 1], y[j + 2], y[j + 3]);
      }
    __syncthreads();
    for (int sl = tid; sl < CPP * (VEC / 4) * kWave; sl += NW * kWave) {
      float4 acc = red4[sl];
#pragma unroll
      for (int w = 1; w < NW; ++w) {
        const float4 t = red4[w * SLOTS + sl];
        acc.x += t.x;
        acc.y += t.y;
        acc.z += t.z;
        acc.w += t.w;
      }
      const int cv = sl / kWave, ln = sl % kWave;
      const int c = ps * CB + cv / (VEC / 4), v4 = cv % (VEC / 4);
      *reinterpret_cast<float4 *>(out + (c * kWave + ln) * VEC + v4 * 4) = acc;
    }
  }
}

}  // namespace moe
