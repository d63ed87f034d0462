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
// The wavefronts' private outputs are tree-reduced through LDS, each workgroup writes one fp32 partial row,
// and a second small kernel adds the partial rows in a fixed order (deterministic result).
#include "common.h"

namespace moe {
namespace {

constexpr int kGemvWaves = 8;
constexpr int kRedCols = 2048;  // columns reduced per LDS pass

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <int FMT>
struct WFmt;
template <>
struct WFmt<MOE_W_FP32> {
  static constexpr int VEC = 4;
  static __device__ __forceinline__ void decode(const u32x4 &v, float (&f)[4]) {
    f[0] = __uint_as_float(v.x);
    f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z);
    f[3] = __uint_as_float(v.w);
  }
};
template <>
struct WFmt<MOE_W_BF16> {
  static constexpr int VEC = 8;
  static __device__ __forceinline__ void decode(const u32x4 &v, float (&f)[8]) {
    f[0] = bf16_lo(v.x);
    f[1] = bf16_hi(v.x);
    f[2] = bf16_lo(v.y);
    f[3] = bf16_hi(v.y);
    f[4] = bf16_lo(v.z);
    f[5] = bf16_hi(v.z);
    f[6] = bf16_lo(v.w);
    f[7] = bf16_hi(v.w);
  }
};


// weights are read once: mark the loads non-temporal so they do not displace x and the partial rows in L2
__device__ __forceinline__ u32x4 stream_load(const u32x4 *p) { return __builtin_nontemporal_load(p); }

// VEC consecutive activations starting at element `col`, widened to fp32
template <int VEC>
__device__ __forceinline__ void load_x(const void *x, int act_fmt, int col, float *out) {
  if (act_fmt == MOE_A_BF16) {
    const uint16_t *xb = static_cast<const uint16_t *>(x) + col;
    if constexpr (VEC == 4) {
      const u32x2 v = *reinterpret_cast<const u32x2 *>(xb);
      out[0] = bf16_lo(v.x); out[1] = bf16_hi(v.x); out[2] = bf16_lo(v.y); out[3] = bf16_hi(v.y);
    } else {
#pragma unroll
      for (int i = 0; i < VEC / 8; ++i) {
        const u32x4 v = reinterpret_cast<const u32x4 *>(xb)[i];
        out[i * 8 + 0] = bf16_lo(v.x); out[i * 8 + 1] = bf16_hi(v.x);
        out[i * 8 + 2] = bf16_lo(v.y); out[i * 8 + 3] = bf16_hi(v.y);
        out[i * 8 + 4] = bf16_lo(v.z); out[i * 8 + 5] = bf16_hi(v.z);
        out[i * 8 + 6] = bf16_lo(v.w); out[i * 8 + 7] = bf16_hi(v.w);
      }
    }
  } else {
    const float4 *xf = reinterpret_cast<const float4 *>(static_cast<const float *>(x) + col);
#pragma unroll
    for (int i = 0; i < VEC / 4; ++i) {
      const float4 v = xf[i];
      out[i * 4 + 0] = v.x; out[i * 4 + 1] = v.y; out[i * 4 + 2] = v.z; out[i * 4 + 3] = v.w;
    }
  }
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

template <int LPR>
struct RecRegs {
  u32x4 g[LPR], u[LPR], dn[LPR];
  float wt;
};

// FMT: weight format, LPR: 16-byte loads per row per lane (d = LPR * 64 * VEC)
template <int FMT, int LPR>
__global__ __launch_bounds__(kGemvWaves * kWave) void expert_gemv_kernel(GemvParams p) {
  using F = WFmt<FMT>;
  constexpr int VEC = F::VEC;
  constexpr int CPL = LPR * VEC;  // columns per lane
  constexpr int NW = kGemvWaves;
  __shared__ float red[(NW / 2) * kRedCols];
  __shared__ int64_t seg_off[MOE_MAX_TOPK];
  __shared__ float seg_w[MOE_MAX_TOPK];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int d = p.hidden, I = p.inter, K = p.top_k;
  const int64_t row_bytes = (int64_t)d * 16 / VEC;
  const int64_t rec_bytes = 3 * row_bytes;
  const int routed = K * I;
  const int total = routed + p.shared_inter;
  const int r0 = (int)((int64_t)blockIdx.x * total / gridDim.x);
  const int r1 = (int)((int64_t)(blockIdx.x + 1) * total / gridDim.x);

  if (tid < K) {
    seg_off[tid] = (int64_t)p.route->sel_slot[tid] * p.slot_bytes;
    seg_w[tid] = p.route->sel_weight[tid];
  }
  __syncthreads();

  auto issue = [&](int r, RecRegs<LPR> &R) {
    const uint8_t *rec;
    if (r < routed) {
      const int k = r / I, i = r - k * I;
      rec = p.slot_pool + seg_off[k] + (int64_t)i * rec_bytes;
      R.wt = seg_w[k];
    } else {
      rec = p.shared_blob + (int64_t)(r - routed) * rec_bytes;
      R.wt = 1.f;
    }
    const u32x4 *q = reinterpret_cast<const u32x4 *>(rec) + lane;
#pragma unroll
    for (int c = 0; c < LPR; ++c) R.g[c] = stream_load(q + c * kWave);
    q += row_bytes / 16;
#pragma unroll
    for (int c = 0; c < LPR; ++c) R.u[c] = stream_load(q + c * kWave);
    q += row_bytes / 16;
#pragma unroll
    for (int c = 0; c < LPR; ++c) R.dn[c] = stream_load(q + c * kWave);
  };

  int r = r0 + wave;
  RecRegs<LPR> A, B;
  if (r < r1) issue(r, A);  // weights first: they do not depend on x

  // activations: lane keeps the x entries of its own columns in registers
  float xr[CPL];
#pragma unroll
  for (int c = 0; c < LPR; ++c) load_x<VEC>(p.x, p.act_fmt, (c * kWave + lane) * VEC, &xr[c * VEC]);

  float y[CPL];
#pragma unroll
  for (int j = 0; j < CPL; ++j) y[j] = 0.f;

  auto consume = [&](const RecRegs<LPR> &R) {
    float g0 = 0.f, g1 = 0.f, u0 = 0.f, u1 = 0.f;
#pragma unroll
    for (int c = 0; c < LPR; ++c) {
      float gw[VEC], uw[VEC];
      F::decode(R.g[c], gw);
      F::decode(R.u[c], uw);
#pragma unroll
      for (int v = 0; v < VEC; v += 2) {
        g0 = __builtin_fmaf(gw[v], xr[c * VEC + v], g0);
        g1 = __builtin_fmaf(gw[v + 1], xr[c * VEC + v + 1], g1);
        u0 = __builtin_fmaf(uw[v], xr[c * VEC + v], u0);
        u1 = __builtin_fmaf(uw[v + 1], xr[c * VEC + v + 1], u1);
      }
    }
    float g = g0 + g1, u = u0 + u1;
    wave_sum2(g, u);
    const float h = g / (1.f + __expf(-g)) * u * R.wt;
#pragma unroll
    for (int c = 0; c < LPR; ++c) {
      float dw[VEC];
      F::decode(R.dn[c], dw);
#pragma unroll
      for (int v = 0; v < VEC; ++v) y[c * VEC + v] = __builtin_fmaf(h, dw[v], y[c * VEC + v]);
    }
  };

  for (; r < r1; r += 2 * NW) {
    const bool has_b = r + NW < r1;
    if (has_b) issue(r + NW, B);
    consume(A);
    if (has_b) {
      if (r + 2 * NW < r1) issue(r + 2 * NW, A);
      consume(B);
    }
  }

  // ---- tree reduction of the wavefronts' outputs through LDS, kRedCols columns per pass ----------
  constexpr int CB = kRedCols / (kWave * VEC);            // load indices c per pass
  constexpr int PASSES = (LPR + CB - 1) / CB;
  constexpr int CPP = (LPR < CB ? LPR : CB);              // c per pass actually present
  float4 *red4 = reinterpret_cast<float4 *>(red);
  float *out = p.partial + (int64_t)blockIdx.x * d;
#pragma unroll
  for (int ps = 0; ps < PASSES; ++ps) {
#pragma unroll
    for (int s = NW / 2; s >= 1; s >>= 1) {
      if (wave >= s && wave < 2 * s) {
        float4 *dst = red4 + (int64_t)(wave - s) * (kRedCols / 4);
#pragma unroll
        for (int cc = 0; cc < CPP; ++cc)
#pragma unroll
          for (int v4 = 0; v4 < VEC / 4; ++v4) {
            const int j = (ps * CB + cc) * VEC + v4 * 4;
            dst[(cc * (VEC / 4) + v4) * kWave + lane] = make_float4(y[j], y[j + 1], y[j + 2], y[j + 3]);
          }
      }
      __syncthreads();
      if (wave < s) {
        const float4 *src = red4 + (int64_t)wave * (kRedCols / 4);
#pragma unroll
        for (int cc = 0; cc < CPP; ++cc)
#pragma unroll
          for (int v4 = 0; v4 < VEC / 4; ++v4) {
            const int j = (ps * CB + cc) * VEC + v4 * 4;
            const float4 t = src[(cc * (VEC / 4) + v4) * kWave + lane];
            y[j] += t.x;
            y[j + 1] += t.y;
            y[j + 2] += t.z;
            y[j + 3] += t.w;
          }
      }
      __syncthreads();
    }
  }
  if (wave == 0) {
#pragma unroll
    for (int c = 0; c < LPR; ++c)
#pragma unroll
      for (int v4 = 0; v4 < VEC / 4; ++v4) {
        const int j = c * VEC + v4 * 4;
        float4 *o = reinterpret_cast<float4 *>(out + (c * kWave + lane) * VEC + v4 * 4);
        *o = make_float4(y[j], y[j + 1], y[j + 2], y[j + 3]);
      }
  }
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

template <int FMT>
hipError_t launch_fmt(const GemvParams &p, int grid, hipStream_t s) {
  constexpr int VEC = WFmt<FMT>::VEC;
  const int lpr = p.hidden / (kWave * VEC);
  dim3 g(grid), b(kGemvWaves * kWave);
  switch (lpr) {
    case 1: hipLaunchKernelGGL((expert_gemv_kernel<FMT, 1>), g, b, 0, s, p); break;
    case 2: hipLaunchKernelGGL((expert_gemv_kernel<FMT, 2>), g, b, 0, s, p); break;
    case 4: hipLaunchKernelGGL((expert_gemv_kernel<FMT, 4>), g, b, 0, s, p); break;
    case 8: hipLaunchKernelGGL((expert_gemv_kernel<FMT, 8>), g, b, 0, s, p); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace

bool gemv_shape_supported(int weight_fmt, int hidden) {
  int vec;
  switch (weight_fmt) {
    case MOE_W_FP32: vec = 4; break;
    case MOE_W_BF16: vec = 8; break;
    default: return false;
  }
  if (hidden <= 0 || hidden % (kWave * vec) != 0) return false;
  const int lpr = hidden / (kWave * vec);
  return lpr == 1 || lpr == 2 || lpr == 4 || lpr == 8;
}

hipError_t launch_expert_gemv(const GemvParams &p, int weight_fmt, int grid, hipStream_t s) {
  if (!gemv_shape_supported(weight_fmt, p.hidden)) return hipErrorInvalidValue;
  switch (weight_fmt) {
    case MOE_W_FP32: return launch_fmt<MOE_W_FP32>(p, grid, s);
    case MOE_W_BF16: return launch_fmt<MOE_W_BF16>(p, grid, s);
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

}  // namespace moe
