// Expert SwiGLU GEMV for one token: y = sum_k w_k W_down,k ( silu(W_gate,k x) * (W_up,k x) ) + shared(x)
// (paper Eq. 1 with SwiGLU experts).  Memory bound: every weight byte of the K selected slots and of the
// shared expert is read exactly once, in 128-bit loads, and nothing else of size moves.
//
// Blob layout ("records"): expert = I records, record i = [gate row i | up row i | column i of W_down],
// each d weights.  One wavefront owns a record: lane l, load c covers columns (c*64 + l)*VEC .. +VEC of all
// three rows (VEC weights = 16 bytes).  The two dot products are reduced across the wavefront with DPP
// rotations, h_i = silu(g_i) * u_i * w_k is formed in every lane, and the lane accumulates h_i * down_i
// into its private d/64 outputs: no barrier between the up and the down projection.  Records of all
// selected experts and of the shared expert form one index space that is split evenly over the workgroups;
// inside a workgroup records are interleaved over the wavefronts, so a workgroup streams one contiguous span.
// Each wavefront keeps DEPTH records' loads in flight in a register ring.  The wavefronts' private outputs
// are tree-reduced through LDS, each workgroup writes one fp32 partial row, and a second small kernel adds
// the partial rows in a fixed order (deterministic result).
#include "common.h"
#include "gemv_common.h"
#include "route_device.h"

namespace moe {
namespace {

// ---- per-format arithmetic on one 16-byte chunk --------------------------------------------------
// X holds the lane's activations for one chunk: XW registers.  dot() accumulates the chunk's partial
// dot product into two chains; axpy() adds h * chunk to the VEC outputs.
template <int FMT, bool DOT2>
struct Chunk;

template <>
struct Chunk<MOE_W_FP32, false> {
  static constexpr int VEC = 4, XW = 4;
  static __device__ __forceinline__ void load_x(const void *x, int act_fmt, int col, float *xr) {
    if (act_fmt == MOE_A_BF16) {
      const u32x2 v = ld64(static_cast<const uint16_t *>(x) + col);
      xr[0] = bf16_lo(v.x); xr[1] = bf16_hi(v.x); xr[2] = bf16_lo(v.y); xr[3] = bf16_hi(v.y);
    } else {
      const u32x4 v = ld128(static_cast<const float *>(x) + col);
      xr[0] = __uint_as_float(v.x); xr[1] = __uint_as_float(v.y); xr[2] = __uint_as_float(v.z);
      xr[3] = __uint_as_float(v.w);
    }
  }
  // x entries of VEC consecutive columns from the residual stream: h * scale, rounded to the activation type
  static __device__ __forceinline__ void load_h(const float *h, int col, float *out) {
    const float4 v = *reinterpret_cast<const float4 *>(h + col);
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
  }
  static __device__ __forceinline__ void make_x(const float *hv, float scale, int act_fmt, float *xr) {
    const float t[4] = {hv[0] * scale, hv[1] * scale, hv[2] * scale, hv[3] * scale};
#pragma unroll
    for (int i = 0; i < 4; ++i)
      xr[i] = act_fmt == MOE_A_BF16 ? __uint_as_float((uint32_t)f32_to_bf16_rne(t[i]) << 16) : t[i];
  }
  static __device__ __forceinline__ void dot(const u32x4 &w, const float *xr, float &a0, float &a1) {
    a0 = __builtin_fmaf(__uint_as_float(w.x), xr[0], a0);
    a1 = __builtin_fmaf(__uint_as_float(w.y), xr[1], a1);
    a0 = __builtin_fmaf(__uint_as_float(w.z), xr[2], a0);
    a1 = __builtin_fmaf(__uint_as_float(w.w), xr[3], a1);
  }
  static __device__ __forceinline__ void axpy(float h, const u32x4 &w, float *y) {
    y[0] = __builtin_fmaf(h, __uint_as_float(w.x), y[0]);
    y[1] = __builtin_fmaf(h, __uint_as_float(w.y), y[1]);
    y[2] = __builtin_fmaf(h, __uint_as_float(w.z), y[2]);
    y[3] = __builtin_fmaf(h, __uint_as_float(w.w), y[3]);
  }
};

template <>
struct Chunk<MOE_W_BF16, false> {
  static constexpr int VEC = 8, XW = 8;
  static __device__ __forceinline__ void load_x(const void *x, int act_fmt, int col, float *xr) {
    if (act_fmt == MOE_A_BF16) {
      const u32x4 v = ld128(static_cast<const uint16_t *>(x) + col);
      xr[0] = bf16_lo(v.x); xr[1] = bf16_hi(v.x); xr[2] = bf16_lo(v.y); xr[3] = bf16_hi(v.y);
      xr[4] = bf16_lo(v.z); xr[5] = bf16_hi(v.z); xr[6] = bf16_lo(v.w); xr[7] = bf16_hi(v.w);
    } else {
      const float *p = static_cast<const float *>(x) + col;
      const u32x4 a = ld128(p), b = ld128(p + 4);
      xr[0] = __uint_as_float(a.x); xr[1] = __uint_as_float(a.y); xr[2] = __uint_as_float(a.z);
      xr[3] = __uint_as_float(a.w); xr[4] = __uint_as_float(b.x); xr[5] = __uint_as_float(b.y);
      xr[6] = __uint_as_float(b.z); xr[7] = __uint_as_float(b.w);
    }
  }
  static __device__ __forceinline__ void load_h(const float *h, int col, float *out) {
    const float4 *q = reinterpret_cast<const float4 *>(h + col);
    const float4 a = q[0], b = q[1];
    out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w; out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
  }
  static __device__ __forceinline__ void make_x(const float *hv, float scale, int act_fmt, float *xr) {
    float t[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = hv[i] * scale;
#pragma unroll
    for (int i = 0; i < 8; ++i)
      xr[i] = act_fmt == MOE_A_BF16 ? __uint_as_float((uint32_t)f32_to_bf16_rne(t[i]) << 16) : t[i];
  }
  static __device__ __forceinline__ void dot(const u32x4 &w, const float *xr, float &a0, float &a1) {
    a0 = __builtin_fmaf(bf16_lo(w.x), xr[0], a0);
    a1 = __builtin_fmaf(bf16_hi(w.x), xr[1], a1);
    a0 = __builtin_fmaf(bf16_lo(w.y), xr[2], a0);
    a1 = __builtin_fmaf(bf16_hi(w.y), xr[3], a1);
    a0 = __builtin_fmaf(bf16_lo(w.z), xr[4], a0);
    a1 = __builtin_fmaf(bf16_hi(w.z), xr[5], a1);
    a0 = __builtin_fmaf(bf16_lo(w.w), xr[6], a0);
    a1 = __builtin_fmaf(bf16_hi(w.w), xr[7], a1);
  }
  static __device__ __forceinline__ void axpy(float h, const u32x4 &w, float *y) {
    y[0] = __builtin_fmaf(h, bf16_lo(w.x), y[0]);
    y[1] = __builtin_fmaf(h, bf16_hi(w.x), y[1]);
    y[2] = __builtin_fmaf(h, bf16_lo(w.y), y[2]);
    y[3] = __builtin_fmaf(h, bf16_hi(w.y), y[3]);
    y[4] = __builtin_fmaf(h, bf16_lo(w.z), y[4]);
    y[5] = __builtin_fmaf(h, bf16_hi(w.z), y[5]);
    y[6] = __builtin_fmaf(h, bf16_lo(w.w), y[6]);
    y[7] = __builtin_fmaf(h, bf16_hi(w.w), y[7]);
  }
};

// bf16 weights with bf16 activations: the activations stay packed (two per register) and the dot products
// use the two-way bf16 dot instruction with fp32 accumulation (products of bf16 values are exact in fp32).
template <>
struct Chunk<MOE_W_BF16, true> {
  static constexpr int VEC = 8, XW = 4;
  static __device__ __forceinline__ void load_x(const void *x, int, int col, float *xr) {
    const u32x4 v = ld128(static_cast<const uint16_t *>(x) + col);
    xr[0] = __uint_as_float(v.x); xr[1] = __uint_as_float(v.y); xr[2] = __uint_as_float(v.z); xr[3] = __uint_as_float(v.w);
  }
  static __device__ __forceinline__ void load_h(const float *h, int col, float *out) {
    Chunk<MOE_W_BF16, false>::load_h(h, col, out);
  }
  static __device__ __forceinline__ void make_x(const float *hv, float scale, int, float *xr) {
    float t[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = hv[i] * scale;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      xr[i] = __uint_as_float((uint32_t)f32_to_bf16_rne(t[2 * i]) | ((uint32_t)f32_to_bf16_rne(t[2 * i + 1]) << 16));
  }
  static __device__ __forceinline__ void dot(const u32x4 &w, const float *xr, float &a0, float &a1) {
    a0 = dot2_bf16(w.x, __float_as_uint(xr[0]), a0);
    a1 = dot2_bf16(w.y, __float_as_uint(xr[1]), a1);
    a0 = dot2_bf16(w.z, __float_as_uint(xr[2]), a0);
    a1 = dot2_bf16(w.w, __float_as_uint(xr[3]), a1);
  }
  static __device__ __forceinline__ void axpy(float h, const u32x4 &w, float *y) {
    Chunk<MOE_W_BF16, false>::axpy(h, w, y);
  }
};

template <int LPR>
struct RecRegs {
  u32x4 g[LPR], u[LPR], dn[LPR];
  float wt;
};

// FMT: weight format; LPR: 16-byte loads per row per lane (d = LPR*64*VEC); NW: wavefronts per workgroup;
// DEPTH: records in flight per wavefront; DOT2: packed bf16 dot products.
// FUSED: workgroup 0 runs the layer boundary (x, gate GEMV, routing: rt::fused_boundary) instead of streaming
// records.  The residual glue has been done by reduce_glue_kernel; every workgroup forms x for itself from the
// new residual stream and its sums of squares (same operations in the same order everywhere, so all copies are
// bit-identical), starts on the shared expert's records at once, and waits for workgroup 0's decision only before
// its first routed record (RecordWalker::load_handover), so the boundary costs the launch little.  The wait is
// on workgroup 0 only, which is dispatched first, and is bounded.
template <int FMT, int LPR, int NW, int DEPTH, bool DOT2, bool FUSED>
__global__ __launch_bounds__(NW *kWave) void expert_gemv_kernel(GemvParams p) {
  using F = Chunk<FMT, DOT2>;
  constexpr int VEC = F::VEC, XW = F::XW;
  constexpr int CPL = LPR * VEC;  // columns per lane
  __shared__ __attribute__((aligned(16))) float red[kRedFloats];
  static_assert(rt::kBoundaryLdsWords <= kRedFloats, "the boundary borrows the reduction buffer");

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront-uniform: keeps record addressing scalar
  const int d = p.hidden;
  if constexpr (FUSED) {
    if (blockIdx.x == 0) {
      // with packed bf16 arithmetic the gate matrix has LPR 16-byte chunks per row per lane, and with NW = 8 each
      // thread owns d / 512 = LPR columns
      static_assert(DOT2 && NW == 8 && LPR <= 4, "the launch variant with the boundary exists for this case only");
      rt::boundary_workgroup<NW, LPR, LPR>(p, red);
      return;
    }
  }
  const int64_t row16 = (int64_t)d / VEC;  // 16-byte chunks per row
  const int64_t rec_bytes = 3 * row16 * 16;
  RecordWalker<NW, FUSED> walk;
  walk.init(p, wave);
  // FUSED: the operands of x (this lane's columns of the residual stream, its sums of squares per 64 columns) are
  // fetched first: a few small loads that complete before the weights queued behind them
  OrderedSum<(FUSED && CPL <= 64) ? CPL : 1> blocks;  // d / 64 = CPL blocks of 64 columns
  float hraw[FUSED ? CPL : 1];
  if constexpr (FUSED) {
    blocks.fetch(p.b.glue.ss, lane);
#pragma unroll
    for (int c = 0; c < LPR; ++c) F::load_h(p.b.glue.h, (c * kWave + lane) * VEC, &hraw[c * VEC]);
    __builtin_amdgcn_sched_barrier(0);  // ... and stay ahead of them in the instruction stream
  }

  auto issue = [&](RecRegs<LPR> &R) {
    R.wt = walk.wt;
    const u32x4 *q = reinterpret_cast<const u32x4 *>(walk.base + (int64_t)walk.at * rec_bytes) + lane;
#pragma unroll
    for (int c = 0; c < LPR; ++c) R.g[c] = stream_load(q + c * kWave);
    q += row16;
#pragma unroll
    for (int c = 0; c < LPR; ++c) R.u[c] = stream_load(q + c * kWave);
    q += row16;
#pragma unroll
    for (int c = 0; c < LPR; ++c) R.dn[c] = stream_load(q + c * kWave);
  };

  // Pass 0 loads every list entry of the wavefront, also the rare ones whose expert is only being filled (their
  // arithmetic is skipped): the number of records is then known up front, the steady-state loop below issues
  // its loads unconditionally, and the compiler can wait for exactly the oldest record in flight instead of for
  // all loads.  Pass 1 (only the experts just filled) skips the other records without loading them.
  const bool all = p.pass == 0;
  int todo = all ? walk.remaining() : 0;  // entries not issued yet (pass 0)
  RecRegs<LPR> ring[DEPTH];
  bool live[DEPTH], want[DEPTH];
  auto advance = [&](int j) {  // next record into ring[j], if there is one
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
  for (int j = 0; j < DEPTH; ++j) advance(j);  // weights first: they do not depend on x

  // activations: the lane keeps the x entries of its own columns in registers
  float xr[LPR * XW];
  if constexpr (FUSED) {
    const float scale = 1.0f / sqrtf(blocks.total() / (float)d + 1e-6f);
#pragma unroll
    for (int c = 0; c < LPR; ++c) F::make_x(&hraw[c * VEC], scale, p.act_fmt, &xr[c * XW]);
  } else {
#pragma unroll
    for (int c = 0; c < LPR; ++c) F::load_x(p.x, p.act_fmt, (c * kWave + lane) * VEC, &xr[c * XW]);
  }

  float y[CPL];
#pragma unroll
  for (int j = 0; j < CPL; ++j) y[j] = 0.f;

  auto consume = [&](const RecRegs<LPR> &R) {
    float g0 = 0.f, g1 = 0.f, u0 = 0.f, u1 = 0.f;
#pragma unroll
    for (int c = 0; c < LPR; ++c) {
      F::dot(R.g[c], &xr[c * XW], g0, g1);
      F::dot(R.u[c], &xr[c * XW], u0, u1);
    }
    float g = g0 + g1, u = u0 + u1;
    wave_sum2(g, u);
    const float h = g / (1.f + __expf(-g)) * u * R.wt;
#pragma unroll
    for (int c = 0; c < LPR; ++c) F::axpy(h, R.dn[c], &y[c * VEC]);
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
  // start-up of short lists, tail, and pass 1.  ring[0] is always the oldest record in flight: when it is dead,
  // all are
  while (live[0]) {
#pragma unroll
    for (int j = 0; j < DEPTH; ++j) {
      if (live[j]) {
        if (want[j]) consume(ring[j]);
        advance(j);
      }
    }
  }

  reduce_and_store<NW, VEC, LPR>(y, red, p.partial + (int64_t)(p.row_offset + blockIdx.x) * d, tid, lane, wave);
}

// y[j] = sum over partial rows in index order, rounded to the activation type.
// Block: 256 threads = 16 row groups x 16 lanes, each lane 4 columns (64 columns per block).
__global__ __launch_bounds__(256) void partial_reduce_kernel(const float *partial, int n_partial, void *y, int d,
                                                             int act_fmt) {
  __shared__ float4 acc_s[16][16];
  const int tid = threadIdx.x, cl = tid & 15, rg = tid >> 4;
  const int col = blockIdx.x * 64 + cl * 4;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  // rows rg*chunk .. (rg+1)*chunk: contiguous chunks keep the overall order a fixed left-to-right tree
  const int chunk = (n_partial + 15) / 16;
  const int b0 = rg * chunk, b1 = min(n_partial, b0 + chunk);
#pragma unroll 8
  for (int b = b0; b < b1; ++b) {
    const float4 t = *reinterpret_cast<const float4 *>(partial + (int64_t)b * d + col);
    acc.x += t.x;
    acc.y += t.y;
    acc.z += t.z;
    acc.w += t.w;
  }
  acc_s[rg][cl] = acc;
  __syncthreads();
  if (rg == 0) {
    float4 s = acc_s[0][cl];
#pragma unroll
    for (int g = 1; g < 16; ++g) {
      const float4 t = acc_s[g][cl];
      s.x += t.x;
      s.y += t.y;
      s.z += t.z;
      s.w += t.w;
    }
    if (act_fmt == MOE_A_BF16) {
      uint2 o;
      o.x = (uint32_t)f32_to_bf16_rne(s.x) | ((uint32_t)f32_to_bf16_rne(s.y) << 16);
      o.y = (uint32_t)f32_to_bf16_rne(s.z) | ((uint32_t)f32_to_bf16_rne(s.w) << 16);
      *reinterpret_cast<uint2 *>(static_cast<uint16_t *>(y) + col) = o;
    } else {
      *reinterpret_cast<float4 *>(static_cast<float *>(y) + col) = s;
    }
  }
}

// partial_reduce_kernel plus the residual glue of a stack for the same 64 columns:
//   y = sum of the partial rows, rounded to the activation type (stored if y != nullptr)
//   h = (carry ? h + y : 0) + perturb * a   (in place; y taken as 0 when there are no partial rows; a may be null)
//   ss[block] = sum of h^2 over the block's 64 columns, in a fixed order
__global__ __launch_bounds__(256) void reduce_glue_kernel(const float *partial, int n_partial, void *y, int d,
                                                          int act_fmt, float *h, const float *a, float perturb,
                                                          int carry, float *ss) {
  __shared__ float4 acc_s[16][16];
  __shared__ float sq_s[16];
  const int tid = threadIdx.x, cl = tid & 15, rg = tid >> 4;
  const int col = blockIdx.x * 64 + cl * 4;
  // the glue operands are fetched by every thread at the very start (absent ones read from h and ignored), so
  // that they are there when the sum is: only the threads of the first row group use them
  const float4 hv = *reinterpret_cast<const float4 *>(h + col);
  const float4 av = *reinterpret_cast<const float4 *>((a != nullptr ? a : h) + col);
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  const int chunk = (n_partial + 15) / 16;
  const int b0 = rg * chunk, b1 = min(n_partial, b0 + chunk);
  if (chunk == 16 && b1 - b0 == 16) {
    // the usual case (one partial row per compute unit of a 256-unit device): all sixteen rows requested at once,
    // added in the same order as below
    float4 t[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) t[i] = *reinterpret_cast<const float4 *>(partial + (int64_t)(b0 + i) * d + col);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      acc.x += t[i].x;
      acc.y += t[i].y;
      acc.z += t[i].z;
      acc.w += t[i].w;
    }
  } else {
#pragma unroll 8
    for (int b = b0; b < b1; ++b) {
      const float4 t = *reinterpret_cast<const float4 *>(partial + (int64_t)b * d + col);
      acc.x += t.x;
      acc.y += t.y;
      acc.z += t.z;
      acc.w += t.w;
    }
  }
  // (keeps the two early loads where they are: without a use here they are moved into the branch below)
  asm volatile("" ::"v"(hv.x), "v"(hv.y), "v"(hv.z), "v"(hv.w), "v"(av.x), "v"(av.y), "v"(av.z), "v"(av.w));
  acc_s[rg][cl] = acc;
  __syncthreads();
  if (rg == 0) {
    float4 s = acc_s[0][cl];
#pragma unroll
    for (int g = 1; g < 16; ++g) {
      const float4 t = acc_s[g][cl];
      s.x += t.x;
      s.y += t.y;
      s.z += t.z;
      s.w += t.w;
    }
    float yv[4] = {s.x, s.y, s.z, s.w};
    if (act_fmt == MOE_A_BF16) {
      uint16_t q[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        q[i] = f32_to_bf16_rne(yv[i]);
        yv[i] = __uint_as_float((uint32_t)q[i] << 16);
      }
      if (y != nullptr) {
        uint2 o;
        o.x = (uint32_t)q[0] | ((uint32_t)q[1] << 16);
        o.y = (uint32_t)q[2] | ((uint32_t)q[3] << 16);
        *reinterpret_cast<uint2 *>(static_cast<uint16_t *>(y) + col) = o;
      }
    } else if (y != nullptr) {
      *reinterpret_cast<float4 *>(static_cast<float *>(y) + col) = s;
    }
    const bool with_y = carry && n_partial > 0;
    float v[4] = {hv.x, hv.y, hv.z, hv.w};
    if (!carry) v[0] = v[1] = v[2] = v[3] = 0.f;
    const float aa[4] = {av.x, av.y, av.z, av.w};
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (with_y) v[i] += yv[i];
      if (a != nullptr) v[i] = __builtin_fmaf(perturb, aa[i], v[i]);
      sq = __builtin_fmaf(v[i], v[i], sq);
    }
    *reinterpret_cast<float4 *>(h + col) = make_float4(v[0], v[1], v[2], v[3]);
    sq_s[cl] = sq;
  }
  __syncthreads();
  if (tid == 0) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) t += sq_s[i];
    ss[blockIdx.x] = t;
  }
}

template <int FMT, int LPR, int NW, int DEPTH, bool DOT2, bool FUSED = false>
void launch_one(const GemvParams &p, int grid, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  hipExtLaunchKernelGGL((expert_gemv_kernel<FMT, LPR, NW, DEPTH, DOT2, FUSED>), dim3(grid), dim3(NW * kWave), 0, s,
                        e0, e1, 0, p);
}

template <int FMT, int LPR, bool DOT2>
hipError_t launch_plan(const GemvParams &p, const GemvPlan &plan, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  if (p.fused) {  // the variant with the boundary in workgroup 0 exists for packed bf16 arithmetic, d <= 2048
    if constexpr (LPR <= 4 && DOT2) {
      if (plan.grid < 2) return hipErrorInvalidValue;
      launch_one<FMT, LPR, kGemvWaves, kGemvDepth, DOT2, true>(p, plan.grid, s, e0, e1);
      return hipGetLastError();
    } else {
      return hipErrorInvalidValue;
    }
  }
  launch_one<FMT, LPR, kGemvWaves, kGemvDepth, DOT2>(p, plan.grid, s, e0, e1);
  return hipGetLastError();
}

// start/stop, when given, receive the kernel's own begin and end timestamps
template <int FMT, bool DOT2>
hipError_t launch_fmt(const GemvParams &p, const GemvPlan &plan, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  constexpr int VEC = Chunk<FMT, DOT2>::VEC;
  const int lpr = p.hidden / (kWave * VEC);
  switch (lpr) {
    case 1: return launch_plan<FMT, 1, DOT2>(p, plan, s, e0, e1);
    case 2: return launch_plan<FMT, 2, DOT2>(p, plan, s, e0, e1);
    case 4: return launch_plan<FMT, 4, DOT2>(p, plan, s, e0, e1);
    case 8: return launch_plan<FMT, 8, DOT2>(p, plan, s, e0, e1);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

bool gemv_shape_supported(int weight_fmt, int hidden) {
  int vec, max_lpr;
  switch (weight_fmt) {
    case MOE_W_FP32: vec = 4; max_lpr = 8; break;
    case MOE_W_BF16: vec = 8; max_lpr = 8; break;
    case MOE_W_INT8_PC: vec = 16; max_lpr = 4; break;
    case MOE_W_INT4_G128: vec = 32; max_lpr = 2; break;
    default: return false;
  }
  if (hidden <= 0 || hidden % (kWave * vec) != 0) return false;
  const int lpr = hidden / (kWave * vec);
  return (lpr == 1 || lpr == 2 || lpr == 4 || lpr == 8) && lpr <= max_lpr;
}

// int8 keeps 16-byte alignment of its scale tail with rows % 8 == 0; int4 groups 128 rows of W_down
bool gemv_inter_supported(int weight_fmt, int inter) {
  if (inter <= 0) return false;
  if (weight_fmt == MOE_W_INT8_PC) return inter % 8 == 0;
  if (weight_fmt == MOE_W_INT4_G128) return inter % 128 == 0;
  return true;
}

// Launch shape: one workgroup of 8 wavefronts per compute unit, two records in flight per wavefront
// (measured best on MI355X among 4/8/16 wavefronts, depths 1-3 and 1-4 workgroups per compute unit).
GemvPlan gemv_plan(int n_cus, int total_records, int weight_fmt, int act_fmt) {
  GemvPlan pl{};
  pl.grid = n_cus < total_records ? n_cus : total_records;
  if (pl.grid < 1) pl.grid = 1;
  if (pl.grid > 1024) pl.grid = 1024;  // (the record split multiplies workgroup index and record count in 32 bits)
  pl.dot2 = weight_fmt == MOE_W_BF16 && act_fmt == MOE_A_BF16;
  return pl;
}

bool gemv_fused_supported(int weight_fmt, int act_fmt, int hidden, const GemvPlan &plan) {
  if (act_fmt != MOE_A_BF16 || plan.grid < 2 || hidden % 512 != 0) return false;
  switch (weight_fmt) {
    case MOE_W_BF16:  // packed bf16 arithmetic, up to 4 loads per row per lane
      return plan.dot2 && hidden / (kWave * 8) <= 4;
    case MOE_W_INT8_PC:
    case MOE_W_INT4_G128: return hidden <= 4096;  // 8 wavefronts, at most 8 columns per thread of workgroup 0
    default: return false;
  }
}

hipError_t launch_expert_gemv(const GemvParams &p, int weight_fmt, const GemvPlan &plan, hipStream_t s,
                              hipEvent_t e0, hipEvent_t e1) {
  if (!gemv_shape_supported(weight_fmt, p.hidden)) return hipErrorInvalidValue;
  switch (weight_fmt) {
    case MOE_W_FP32: return launch_fmt<MOE_W_FP32, false>(p, plan, s, e0, e1);
    case MOE_W_BF16:
      return plan.dot2 ? launch_fmt<MOE_W_BF16, true>(p, plan, s, e0, e1)
                       : launch_fmt<MOE_W_BF16, false>(p, plan, s, e0, e1);
    case MOE_W_INT8_PC:
    case MOE_W_INT4_G128: return launch_expert_gemv_quant(p, weight_fmt, plan, s, e0, e1);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_partial_reduce(const float *partial, int n_partial, void *y, int hidden, int act_fmt,
                                 hipStream_t s) {
  if (hidden % 64 != 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(partial_reduce_kernel, dim3(hidden / 64), dim3(256), 0, s, partial, n_partial, y, hidden,
                     act_fmt);
  return hipGetLastError();
}

hipError_t launch_reduce_glue(const float *partial, int n_partial, void *y, int hidden, int act_fmt, float *h,
                              const float *a, float perturb, int carry, float *ss, hipStream_t s) {
  if (hidden % 64 != 0 || hidden / 64 > 128) return hipErrorInvalidValue;
  hipLaunchKernelGGL(reduce_glue_kernel, dim3(hidden / 64), dim3(256), 0, s, partial, n_partial, y, hidden, act_fmt, h,
                     a, perturb, carry, ss);
  return hipGetLastError();
}

}  // namespace moe
