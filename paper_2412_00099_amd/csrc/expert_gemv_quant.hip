// Weight-only quantised variants of the expert SwiGLU GEMV (paper Eq. 1; Sec. 4.5 deploys 4- and 8-bit
// experts).  Same decomposition as the bf16 kernel - one wavefront per record [gate row | up row | column of
// W_down], DPP reduction of the two dot products, private output accumulators, LDS sum, one fp32 partial
// row per workgroup - with the dequantisation folded into the arithmetic:
//
//  int8 (per output channel fp16 scales).  Bytes are stored offset-binary (u = q + 128).  Two bytes become a
//  packed fp16 pair (1024 + u) with one byte permute; the dot products use the two-way fp16 dot instruction
//  with fp32 accumulation against fp16-packed activations, and the constant (1024 + 128) * sum(x) is removed
//  once per row.  The row scale multiplies the reduced dot product.  For the down projection each byte is
//  converted to fp32 and accumulated unscaled; the per-column scale is applied when the wavefront leaves
//  an expert (scales differ per expert) and at the end.
//
//  int4 (group-128 symmetric, fp16 scales, nibble = q + 8).  A lane's 32 columns of a row lie in one
//  group.  Nibble pairs (t, t+4) of a dword become packed bf16 (128 + n) with one and-or (plus a shift);
//  dot products use the two-way bf16 dot instruction against bf16-packed activations arranged in the same
//  pair order, the constant (128 + 8) * sum(x) is removed per lane, then the lane's group scale is applied
//  before the wavefront reduction.  For the down projection the pairs are formed as fp16 (1024 + n) and
//  consumed by mixed-precision FMAs; accumulators are unscaled within a group of 128 records and flushed with
//  the group's per-column scales (and the constant (1024 + 8) * sum(h) removed) when the group or expert
//  changes and at the end.
#include "common.h"
#include "gemv_common.h"
#include "route_device.h"

namespace moe {
namespace {

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float dot2_f16(uint32_t a, uint32_t b, float acc) {
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, a), __builtin_bit_cast(f16x2, b), acc, false);
}
__device__ __forceinline__ float f16_lo(uint32_t v) { return (float)__builtin_bit_cast(f16x2, v).x; }
__device__ __forceinline__ float f16_hi(uint32_t v) { return (float)__builtin_bit_cast(f16x2, v).y; }
__device__ __forceinline__ float f16_bits(uint16_t v) { return (float)__builtin_bit_cast(_Float16, v); }
__device__ __forceinline__ uint32_t pack_f16(float a, float b) {
  // saturate: activations beyond the fp16 range would turn into infinities
  a = fminf(fmaxf(a, -65504.f), 65504.f);
  b = fminf(fmaxf(b, -65504.f), 65504.f);
  f16x2 v = {(_Float16)a, (_Float16)b};
  return __builtin_bit_cast(uint32_t, v);
}
// N consecutive activations starting at column col (a multiple of 8), in two steps so that other loads can be
// issued between the fetch (16-byte loads into raw registers) and the conversion to float
template <int N>
struct XRaw {
  u32x4 v[N / 4];
};
template <int N>
__device__ __forceinline__ void fetch_x(const void *x, int act_fmt, int col, XRaw<N> &r) {
  if (act_fmt == MOE_A_BF16) {
    const u32x4 *q = reinterpret_cast<const u32x4 *>(static_cast<const uint16_t *>(x) + col);
#pragma unroll
    for (int i = 0; i < N / 8; ++i) r.v[i] = q[i];
  } else {
    const u32x4 *q = reinterpret_cast<const u32x4 *>(static_cast<const float *>(x) + col);
#pragma unroll
    for (int i = 0; i < N / 4; ++i) r.v[i] = q[i];
  }
}
template <int N>
__device__ __forceinline__ void unpack_x(const XRaw<N> &r, int act_fmt, float *out) {
  if (act_fmt == MOE_A_BF16) {
#pragma unroll
    for (int i = 0; i < N / 8; ++i) {
      const u32x4 v = r.v[i];
      out[8 * i + 0] = bf16_lo(v.x); out[8 * i + 1] = bf16_hi(v.x); out[8 * i + 2] = bf16_lo(v.y);
      out[8 * i + 3] = bf16_hi(v.y); out[8 * i + 4] = bf16_lo(v.z); out[8 * i + 5] = bf16_hi(v.z);
      out[8 * i + 6] = bf16_lo(v.w); out[8 * i + 7] = bf16_hi(v.w);
    }
  } else {
#pragma unroll
    for (int i = 0; i < N / 4; ++i) {
      const u32x4 v = r.v[i];
      out[4 * i + 0] = __uint_as_float(v.x); out[4 * i + 1] = __uint_as_float(v.y);
      out[4 * i + 2] = __uint_as_float(v.z); out[4 * i + 3] = __uint_as_float(v.w);
    }
  }
}

// FUSED launches (layer boundary in workgroup 0, see expert_gemv_kernel): N consecutive columns of the residual
// stream, fetched early, and the activations made of them - h * scale rounded to the activation type - with the
// same operations as workgroup 0 uses for the copy of x it writes to memory.
template <int N>
struct HRaw {
  float4 v[N / 4];
};
template <int N>
__device__ __forceinline__ void fetch_h(const float *h, int col, HRaw<N> &r) {
  const float4 *q = reinterpret_cast<const float4 *>(h + col);
#pragma unroll
  for (int i = 0; i < N / 4; ++i) r.v[i] = q[i];
}
template <int N>
__device__ __forceinline__ void x_from_h(const HRaw<N> &r, float scale, int act_fmt, float *out) {
#pragma unroll
  for (int i = 0; i < N / 4; ++i) {
    const float t[4] = {r.v[i].x * scale, r.v[i].y * scale, r.v[i].z * scale, r.v[i].w * scale};
#pragma unroll
    for (int k = 0; k < 4; ++k)
      out[4 * i + k] = act_fmt == MOE_A_BF16 ? __uint_as_float((uint32_t)f32_to_bf16_rne(t[k]) << 16) : t[k];
  }
}
// gate-matrix chunks per row per lane / columns per thread of workgroup 0 for hidden size d (bf16 activations,
// 8 wavefronts): d = 512 * PER; the gate rows are held in registers (CH = PER) up to d = 2048
constexpr int boundary_per(int d) { return d / 512; }
constexpr int boundary_ch(int d) { return d / 512 <= 4 ? d / 512 : 0; }

// =================================================================================================
// int8
// =================================================================================================
template <int LPR>
struct RecI8 {
  u32x4 g[LPR], u[LPR], dn[LPR];
  float sg, su, wt;
  const uint8_t *base;  // blob of the record's expert (its tail holds the down scales)
  int rows;
};

// PRE: the per-column scales of W_down are fetched when the wavefront enters an expert, so that the flush at the
// next change finds them in registers (costs 2*LPR 16-byte registers per lane)
template <int LPR, int NW, int DEPTH, bool PRE, bool FUSED>
__global__ __launch_bounds__(NW *kWave) void expert_gemv_int8_kernel(GemvParams p) {
  constexpr int VEC = 16, CPL = LPR * VEC;
  __shared__ __attribute__((aligned(16))) float red[kRedFloats];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int d = p.hidden;
  if constexpr (FUSED) {
    if (blockIdx.x == 0) {
      rt::boundary_workgroup<NW, boundary_ch(CPL * kWave), boundary_per(CPL * kWave)>(p, red);
      return;
    }
  }
  const int64_t row16 = d / VEC;
  const int64_t rec_bytes = 3 * row16 * 16;
  RecordWalker<NW, FUSED> walk;
  walk.init(p, wave);

  auto issue = [&](RecI8<LPR> &R) {
    const uint16_t *tail = reinterpret_cast<const uint16_t *>(walk.base + (int64_t)walk.rows * rec_bytes);
    R.wt = walk.wt;
    R.base = walk.base;
    R.rows = walk.rows;
    const u32x4 *q = reinterpret_cast<const u32x4 *>(walk.base + (int64_t)walk.at * rec_bytes) + lane;
#pragma unroll
    for (int c = 0; c < LPR; ++c) R.g[c] = stream_load(q + c * kWave);
    q += row16;
#pragma unroll
    for (int c = 0; c < LPR; ++c) R.u[c] = stream_load(q + c * kWave);
    q += row16;
#pragma unroll
    for (int c = 0; c < LPR; ++c) R.dn[c] = stream_load(q + c * kWave);
    R.sg = f16_bits(tail[walk.at]);              // gate scales [rows]
    R.su = f16_bits(tail[walk.rows + walk.at]);  // up scales [rows]
  };

  // the activations' few loads go out ahead of the weights (loads complete in order, and the first routed record
  // has to wait for the routing record); they are converted after the ring has been filled
  XRaw<VEC> xraw[FUSED ? 1 : LPR];
  HRaw<VEC> hraw[FUSED ? LPR : 1];
  OrderedSum<FUSED ? CPL : 1> blocks;  // FUSED: d / 64 = CPL sums of squares of the residual stream
  if constexpr (FUSED) {
    blocks.fetch(p.b.glue.ss, lane);
#pragma unroll
    for (int c = 0; c < LPR; ++c) fetch_h<VEC>(p.b.glue.h, (c * kWave + lane) * VEC, hraw[c]);
    __builtin_amdgcn_sched_barrier(0);
  } else {
#pragma unroll
    for (int c = 0; c < LPR; ++c) fetch_x<VEC>(p.x, p.act_fmt, (c * kWave + lane) * VEC, xraw[c]);
  }

  RecI8<LPR> ring[DEPTH];
  bool live[DEPTH];
#pragma unroll
  for (int j = 0; j < DEPTH; ++j) {
    live[j] = walk.next(p);
    if (live[j]) issue(ring[j]);
  }

  // activations as packed fp16 pairs in column order, and their sum over this lane's columns
  uint32_t xh[CPL / 2];
  float xsum = 0.f;
  float x_scale = 0.f;
  if constexpr (FUSED) x_scale = 1.0f / sqrtf(blocks.total() / (float)d + 1e-6f);
#pragma unroll
  for (int c = 0; c < LPR; ++c) {
    float xf[VEC];
    if constexpr (FUSED) x_from_h<VEC>(hraw[c], x_scale, p.act_fmt, xf);
    else unpack_x<VEC>(xraw[c], p.act_fmt, xf);
#pragma unroll
    for (int v = 0; v < VEC; v += 2) {
      const uint32_t pr = pack_f16(xf[v], xf[v + 1]);
      xh[(c * VEC + v) / 2] = pr;
      xsum += f16_lo(pr) + f16_hi(pr);
    }
  }
  const float xoff = -(1024.f + 128.f) * xsum;

  float y[CPL], acc[CPL];
#pragma unroll
  for (int j = 0; j < CPL; ++j) y[j] = acc[j] = 0.f;
  float hsum = 0.f;
  const uint8_t *cur_base = nullptr;
  int cur_rows = 0;

  u32x4 dsc[PRE ? 2 * LPR : 1];
  auto load_scales = [&](const uint8_t *base, int rows) {
    const uint16_t *sd = reinterpret_cast<const uint16_t *>(base + (int64_t)rows * rec_bytes) + 2 * rows;
#pragma unroll
    for (int c = 0; c < (PRE ? LPR : 0); ++c) {
      const u32x4 *sp = reinterpret_cast<const u32x4 *>(sd + (c * kWave + lane) * VEC);
      dsc[2 * c] = sp[0];
      dsc[2 * c + 1] = sp[1];
    }
  };

  // y += scale_col * (acc - 128*hsum) with the per-column scales of the expert whose blob is `base`
  auto flush = [&](const uint8_t *base, int rows) {
    const uint16_t *sd = reinterpret_cast<const uint16_t *>(base + (int64_t)rows * rec_bytes) + 2 * rows;
    const float off = 128.f * hsum;
#pragma unroll
    for (int c = 0; c < LPR; ++c) {
      const u32x4 *sp = reinterpret_cast<const u32x4 *>(sd + (c * kWave + lane) * VEC);
      const u32x4 s0 = PRE ? dsc[PRE ? 2 * c : 0] : sp[0], s1 = PRE ? dsc[PRE ? 2 * c + 1 : 0] : sp[1];
      const uint32_t sw[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
#pragma unroll
      for (int v = 0; v < VEC; v += 2) {
        const int j = c * VEC + v;
        y[j] = __builtin_fmaf(f16_lo(sw[v / 2]), acc[j] - off, y[j]);
        y[j + 1] = __builtin_fmaf(f16_hi(sw[v / 2]), acc[j + 1] - off, y[j + 1]);
        acc[j] = acc[j + 1] = 0.f;
      }
    }
    hsum = 0.f;
  };

  auto consume = [&](const RecI8<LPR> &R) {
    if (R.base != cur_base) {
      if (cur_base) flush(cur_base, cur_rows);
      cur_base = R.base;
      cur_rows = R.rows;
      load_scales(cur_base, cur_rows);
    }
    float g0 = 0.f, g1 = 0.f, u0 = 0.f, u1 = 0.f;
#pragma unroll
    for (int c = 0; c < LPR; ++c) {
      const uint32_t gw[4] = {R.g[c].x, R.g[c].y, R.g[c].z, R.g[c].w};
      const uint32_t uw[4] = {R.u[c].x, R.u[c].y, R.u[c].z, R.u[c].w};
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        // bytes (b0,b1) and (b2,b3) of the dword -> fp16 pairs (1024+b)
        const uint32_t glo = __builtin_amdgcn_perm(gw[w], 0x64646464u, 0x00050004u);
        const uint32_t ghi = __builtin_amdgcn_perm(gw[w], 0x64646464u, 0x00070006u);
        const uint32_t ulo = __builtin_amdgcn_perm(uw[w], 0x64646464u, 0x00050004u);
        const uint32_t uhi = __builtin_amdgcn_perm(uw[w], 0x64646464u, 0x00070006u);
        g0 = dot2_f16(glo, xh[c * 8 + w * 2], g0);
        g1 = dot2_f16(ghi, xh[c * 8 + w * 2 + 1], g1);
        u0 = dot2_f16(ulo, xh[c * 8 + w * 2], u0);
        u1 = dot2_f16(uhi, xh[c * 8 + w * 2 + 1], u1);
      }
    }
    float g = (g0 + g1) + xoff, u = (u0 + u1) + xoff;
    wave_sum2(g, u);
    g *= R.sg;
    u *= R.su;
    const float h = g / (1.f + __expf(-g)) * u * R.wt;
    hsum += h;
#pragma unroll
    for (int c = 0; c < LPR; ++c) {
      const uint32_t dw[4] = {R.dn[c].x, R.dn[c].y, R.dn[c].z, R.dn[c].w};
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const int j = c * VEC + w * 4;
        acc[j] = __builtin_fmaf(h, (float)(dw[w] & 0xffu), acc[j]);
        acc[j + 1] = __builtin_fmaf(h, (float)((dw[w] >> 8) & 0xffu), acc[j + 1]);
        acc[j + 2] = __builtin_fmaf(h, (float)((dw[w] >> 16) & 0xffu), acc[j + 2]);
        acc[j + 3] = __builtin_fmaf(h, (float)(dw[w] >> 24), acc[j + 3]);
      }
    }
  };

  while (live[0]) {
#pragma unroll
    for (int j = 0; j < DEPTH; ++j) {
      if (live[j]) {
        consume(ring[j]);
        live[j] = walk.next(p);
        if (live[j]) issue(ring[j]);
      }
    }
  }
  if (cur_base) flush(cur_base, cur_rows);
  reduce_and_store<NW, VEC, LPR>(y, red, p.partial + (int64_t)(p.row_offset + blockIdx.x) * d, tid, lane, wave);
}

// =================================================================================================
// int4, group 128
// =================================================================================================
// A dword holds the nibbles n0..n7 of eight consecutive columns.  Four masked copies of it are four fp16 pairs:
//     (w      & 0x000f000f) | 0x64006400  =  (1024 +      n0, 1024 +      n4)
//     (w      & 0x00f000f0) | 0x64006400  =  (1024 + 16 * n1, 1024 + 16 * n5)
//     (w >> 8 & 0x000f000f) | 0x64006400  =  (1024 +      n2, 1024 +      n6)
//     (w >> 8 & 0x00f000f0) | 0x64006400  =  (1024 + 16 * n3, 1024 + 16 * n7)
// one shift and four and-or operations per eight weights.  The factor 16 of the odd columns is undone in the other
// operand: the activations of odd columns are stored divided by 16 (gate / up rows), the down scales of odd columns
// are divided by 16 when the accumulators are flushed.  The constants (1024 and the zero point 8) are removed through
// sums of the activations (per lane and chunk, once) and of h (per group).
constexpr uint32_t kNibMaskLo = 0x000f000fu, kNibMaskHi = 0x00f000f0u, kF16Bias = 0x64006400u;

// (w & mask) | bias as one operation: mask and bias are handed over as register values so that the three-operand
// form is chosen (it takes no literal constants)
__device__ __forceinline__ uint32_t and_or(uint32_t w, uint32_t mask, uint32_t bias) { return (w & mask) | bias; }

template <int LPR>
struct RecI4 {
  u32x4 g[LPR], u[LPR], dn[LPR];
  uint32_t sc[LPR];  // (gate scale, up scale) fp16 pair of this lane's group, per chunk
  float wt;
  const uint8_t *base;  // blob of the record's expert (its tail holds the down scales)
  int rows, grp;
};

template <int LPR, int NW, int DEPTH, bool PRE, bool FUSED>
__global__ __launch_bounds__(NW *kWave) void expert_gemv_int4_kernel(GemvParams p) {
  constexpr int VEC = 32, CPL = LPR * VEC;
  __shared__ __attribute__((aligned(16))) float red[kRedFloats];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int d = p.hidden;
  if constexpr (FUSED) {
    if (blockIdx.x == 0) {
      rt::boundary_workgroup<NW, boundary_ch(CPL * kWave), boundary_per(CPL * kWave)>(p, red);
      return;
    }
  }
  const int64_t row16 = d / VEC;                             // 16-byte chunks per row of nibbles
  const int64_t rec_bytes = int4_record_bytes(d);            // three rows + (gate, up) scale pairs, padded
  RecordWalker<NW, FUSED, 1> walk;  // a contiguous block of records per wavefront: few changes of scale group
  walk.init(p, wave);

  auto issue = [&](RecI4<LPR> &R) {
    const uint8_t *rec = walk.base + (int64_t)walk.at * rec_bytes;
    R.wt = walk.wt;
    R.base = walk.base;
    R.rows = walk.rows;
    R.grp = walk.at >> 7;
    const u32x4 *q = reinterpret_cast<const u32x4 *>(rec) + lane;
#pragma unroll
    for (int c = 0; c < LPR; ++c) R.g[c] = stream_load(q + c * kWave);
    q += row16;
#pragma unroll
    for (int c = 0; c < LPR; ++c) R.u[c] = stream_load(q + c * kWave);
    q += row16;
#pragma unroll
    for (int c = 0; c < LPR; ++c) R.dn[c] = stream_load(q + c * kWave);
    const uint32_t *sc = reinterpret_cast<const uint32_t *>(rec + 3 * row16 * 16);
#pragma unroll
    for (int c = 0; c < LPR; ++c) R.sc[c] = sc[(c * kWave + lane) >> 2];  // 4 lanes (128 columns) per group
  };

  XRaw<VEC> xraw[FUSED ? 1 : LPR];  // fetched ahead of the weights, converted after the ring has been filled
  HRaw<VEC> hraw[FUSED ? LPR : 1];
  OrderedSum<FUSED ? CPL : 1> blocks;
  if constexpr (FUSED) {
    blocks.fetch(p.b.glue.ss, lane);
#pragma unroll
    for (int c = 0; c < LPR; ++c) fetch_h<VEC>(p.b.glue.h, (c * kWave + lane) * VEC, hraw[c]);
    __builtin_amdgcn_sched_barrier(0);
  } else {
#pragma unroll
    for (int c = 0; c < LPR; ++c) fetch_x<VEC>(p.x, p.act_fmt, (c * kWave + lane) * VEC, xraw[c]);
  }

  // Pass 0 loads every list entry of the wavefront, also the rare ones whose expert is only being filled (their
  // arithmetic is skipped), so that the steady-state loop issues its loads unconditionally and each use waits for
  // the oldest record only.  Pass 1 (the experts just filled) skips the other records without loading them.
  const bool all = p.pass == 0;
  int todo = all ? walk.remaining() : 0;
  RecI4<LPR> ring[DEPTH];
  bool live[DEPTH], want[DEPTH];
  auto advance = [&](int j) {
    if (all) {
      live[j] = todo > 0;
      if (live[j]) {
        --todo;
        want[j] = walk.step(p);
      }
    } else {
      live[j] = walk.next(p);
      want[j] = true;
    }
    if (live[j]) issue(ring[j]);
  };
#pragma unroll
  for (int j = 0; j < DEPTH; ++j) advance(j);
  // the down scales of the first record's group travel with the first records
  const uint8_t *cur_base = nullptr;
  int cur_rows = 0, cur_grp = -1;
  u32x4 dsc[PRE ? 4 * LPR : 1];
  auto load_scales = [&](const uint8_t *base, int rows, int grp) {
    const uint16_t *sd = reinterpret_cast<const uint16_t *>(base + (int64_t)rows * rec_bytes) + (int64_t)grp * d;
#pragma unroll
    for (int c = 0; c < (PRE ? LPR : 0); ++c) {
      const u32x4 *sp = reinterpret_cast<const u32x4 *>(sd + (c * kWave + lane) * VEC);
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) dsc[4 * c + q4] = sp[q4];
    }
  };
  if (live[0]) {
    cur_base = ring[0].base;
    cur_rows = ring[0].rows;
    cur_grp = ring[0].grp;
    load_scales(cur_base, cur_rows, cur_grp);
  }

  // mask and bias of the nibble unpacking as register values (see and_or)
  uint32_t mask_lo = kNibMaskLo, mask_hi = kNibMaskHi, bias = kF16Bias;
  asm volatile("" : "+s"(mask_lo), "+s"(mask_hi));
  asm volatile("" : "+v"(bias));

  // Activations as packed fp16 pairs in the order the unpacking produces the weights: per dword of eight columns
  // (x0, x4), (x1, x5) / 16, (x2, x6), (x3, x7) / 16.  xoff[c] removes, per chunk, what the biased weights add:
  // 1024 * (sum of the even-column entries) + 64 * (sum of the odd-column entries, which are x / 16 times 1024)
  // and the zero point 8 * (sum of all x).
  uint32_t xp[CPL / 2];
  float xoff[LPR];
  float x_scale = 0.f;
  if constexpr (FUSED) x_scale = 1.0f / sqrtf(blocks.total() / (float)d + 1e-6f);
#pragma unroll
  for (int c = 0; c < LPR; ++c) {
    float xf[VEC];
    if constexpr (FUSED) x_from_h<VEC>(hraw[c], x_scale, p.act_fmt, xf);
    else unpack_x<VEC>(xraw[c], p.act_fmt, xf);
    float s_even = 0.f, s_odd = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w)
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const float k = (t & 1) ? 0.0625f : 1.f;
        const uint32_t pr = pack_f16(xf[w * 8 + t] * k, xf[w * 8 + t + 4] * k);
        xp[c * 16 + w * 4 + t] = pr;
        if (t & 1) s_odd += f16_lo(pr) + f16_hi(pr); else s_even += f16_lo(pr) + f16_hi(pr);
      }
    // odd entries hold x / 16: 1024 * (x / 16) = 64 x of bias, and 8 x = 128 * (x / 16) of zero point
    xoff[c] = -((1024.f + 8.f) * s_even + (1024.f + 128.f) * s_odd);
  }

  float y[CPL], acc[CPL];
#pragma unroll
  for (int j = 0; j < CPL; ++j) y[j] = acc[j] = 0.f;
  float hsum = 0.f;
  bool dirty = false;  // acc holds something (scales of a group nothing was taken from are never applied)

  // even columns: y += s * (acc - (1024 + 8) * hsum);  odd columns (weights taken 16-fold):
  // y += (s / 16) * (acc - (1024 + 128) * hsum)
  auto flush = [&](const uint8_t *base, int rows, int grp) {
    const uint16_t *sd = reinterpret_cast<const uint16_t *>(base + (int64_t)rows * rec_bytes) + (int64_t)grp * d;
    const float off_even = (1024.f + 8.f) * hsum, off_odd = (1024.f + 128.f) * hsum;
#pragma unroll
    for (int c = 0; c < LPR; ++c) {
      const u32x4 *sp = reinterpret_cast<const u32x4 *>(sd + (c * kWave + lane) * VEC);
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const u32x4 sv = PRE ? dsc[PRE ? 4 * c + q4 : 0] : sp[q4];
        const uint32_t sw[4] = {sv.x, sv.y, sv.z, sv.w};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int j = c * VEC + q4 * 8 + t * 2;
          y[j] = __builtin_fmaf(f16_lo(sw[t]), acc[j] - off_even, y[j]);
          y[j + 1] = __builtin_fmaf(f16_hi(sw[t]) * 0.0625f, acc[j + 1] - off_odd, y[j + 1]);
          acc[j] = acc[j + 1] = 0.f;
        }
      }
    }
    hsum = 0.f;
    dirty = false;
  };

  auto consume = [&](const RecI4<LPR> &R) {
    if (R.base != cur_base || R.grp != cur_grp) {
      if (dirty) flush(cur_base, cur_rows, cur_grp);
      cur_base = R.base;
      cur_rows = R.rows;
      cur_grp = R.grp;
      load_scales(cur_base, cur_rows, cur_grp);
    }
    float g = 0.f, u = 0.f;
#pragma unroll
    for (int c = 0; c < LPR; ++c) {
      const uint32_t gw[4] = {R.g[c].x, R.g[c].y, R.g[c].z, R.g[c].w};
      const uint32_t uw[4] = {R.u[c].x, R.u[c].y, R.u[c].z, R.u[c].w};
      float g0 = 0.f, g1 = 0.f, u0 = 0.f, u1 = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t *xw = &xp[c * 16 + w * 4];
        const uint32_t g8 = gw[w] >> 8, u8 = uw[w] >> 8;
        g0 = dot2_f16(and_or(gw[w], mask_lo, bias), xw[0], g0);
        g1 = dot2_f16(and_or(gw[w], mask_hi, bias), xw[1], g1);
        g0 = dot2_f16(and_or(g8, mask_lo, bias), xw[2], g0);
        g1 = dot2_f16(and_or(g8, mask_hi, bias), xw[3], g1);
        u0 = dot2_f16(and_or(uw[w], mask_lo, bias), xw[0], u0);
        u1 = dot2_f16(and_or(uw[w], mask_hi, bias), xw[1], u1);
        u0 = dot2_f16(and_or(u8, mask_lo, bias), xw[2], u0);
        u1 = dot2_f16(and_or(u8, mask_hi, bias), xw[3], u1);
      }
      g = __builtin_fmaf((g0 + g1) + xoff[c], f16_lo(R.sc[c]), g);
      u = __builtin_fmaf((u0 + u1) + xoff[c], f16_hi(R.sc[c]), u);
    }
    wave_sum2(g, u);
    const float h = g / (1.f + __expf(-g)) * u * R.wt;
    hsum += h;
    dirty = true;
#pragma unroll
    for (int c = 0; c < LPR; ++c) {
      const uint32_t dw[4] = {R.dn[c].x, R.dn[c].y, R.dn[c].z, R.dn[c].w};
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t d8 = dw[w] >> 8;
        const uint32_t pr[4] = {and_or(dw[w], mask_lo, bias), and_or(dw[w], mask_hi, bias), and_or(d8, mask_lo, bias),
                                and_or(d8, mask_hi, bias)};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          // pair t = columns t and t + 4 of the dword (odd t: 16-fold), consumed by mixed-precision FMAs
          const int j = c * VEC + w * 8 + t;
          acc[j] = __builtin_fmaf(f16_lo(pr[t]), h, acc[j]);
          acc[j + 4] = __builtin_fmaf(f16_hi(pr[t]), h, acc[j + 4]);
        }
      }
    }
  };

  // steady state of pass 0: all ring entries live and at least DEPTH more entries to fetch
  if (all && live[DEPTH - 1]) {
    while (todo >= DEPTH) {
#pragma unroll
      for (int j = 0; j < DEPTH; ++j) {
        if (want[j]) consume(ring[j]);
        want[j] = walk.step(p);
        issue(ring[j]);
      }
      todo -= DEPTH;
    }
  }
  // start-up of short lists, tail, and pass 1.  ring[0] is always the oldest record in flight
  while (live[0]) {
#pragma unroll
    for (int j = 0; j < DEPTH; ++j) {
      if (live[j]) {
        if (want[j]) consume(ring[j]);
        advance(j);
      }
    }
  }
  if (dirty) flush(cur_base, cur_rows, cur_grp);
  reduce_and_store<NW, VEC, LPR>(y, red, p.partial + (int64_t)(p.row_offset + blockIdx.x) * d, tid, lane, wave);
}

}  // namespace

hipError_t launch_expert_gemv_quant(const GemvParams &p, int weight_fmt, const GemvPlan &plan, hipStream_t s,
                                    hipEvent_t e0, hipEvent_t e1) {
  const dim3 g(plan.grid), b(8 * kWave);
#define MOE_Q(KERNEL, ...)                                                                      \
  do {                                                                                          \
    if (p.fused) hipExtLaunchKernelGGL((KERNEL<__VA_ARGS__, true>), g, b, 0, s, e0, e1, 0, p);  \
    else hipExtLaunchKernelGGL((KERNEL<__VA_ARGS__, false>), g, b, 0, s, e0, e1, 0, p);         \
  } while (0)
  if (p.fused && (plan.grid < 2 || p.act_fmt != MOE_A_BF16)) return hipErrorInvalidValue;
  if (weight_fmt == MOE_W_INT8_PC) {
    switch (p.hidden / (kWave * 16)) {
      case 1: MOE_Q(expert_gemv_int8_kernel, 1, 8, 2, true); break;
      case 2: MOE_Q(expert_gemv_int8_kernel, 2, 8, 2, false); break;
      case 4: MOE_Q(expert_gemv_int8_kernel, 4, 8, 1, false); break;
      default: return hipErrorInvalidValue;
    }
  } else if (weight_fmt == MOE_W_INT4_G128) {
    switch (p.hidden / (kWave * 32)) {
      case 1: MOE_Q(expert_gemv_int4_kernel, 1, 8, 6, true); break;
      case 2: MOE_Q(expert_gemv_int4_kernel, 2, 8, 2, false); break;
      default: return hipErrorInvalidValue;
    }
  } else {
    return hipErrorInvalidValue;
  }
#undef MOE_Q
  return hipGetLastError();
}

}  // namespace moe
