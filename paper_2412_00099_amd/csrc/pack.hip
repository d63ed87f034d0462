// Blob geometry, the canonical -> record-layout packer, and the synthetic-stack glue kernel.
#include "common.h"

namespace moe {

BlobLayout blob_layout(int fmt, int hidden, int inter) {
  BlobLayout L{};
  const int64_t d = hidden, I = inter;
  switch (fmt) {
    case MOE_W_FP32: L.row_bytes = d * 4; break;
    case MOE_W_BF16: L.row_bytes = d * 2; break;
    default: return L;
  }
  L.rec_bytes = 3 * L.row_bytes;
  L.tail_offset = I * L.rec_bytes;
  L.total = (L.tail_offset + 255) / 256 * 256;
  return L;
}

namespace {

// One thread per 16-byte chunk of the blob.  gate/up chunks are straight copies of a row segment;
// a down chunk gathers column i of the [d, I] matrix (strided reads: this runs once per expert, off the
// decode path).
template <typename T>
__global__ void pack_plain_kernel(const T *gate, const T *up, const T *down, T *blob, int d, int I) {
  constexpr int VEC = 16 / sizeof(T);
  const int64_t chunks_per_row = d / VEC;
  const int64_t n_chunks = (int64_t)I * 3 * chunks_per_row;
  for (int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; c < n_chunks; c += (int64_t)gridDim.x * blockDim.x) {
    const int64_t rec = c / (3 * chunks_per_row);
    const int64_t rem = c - rec * 3 * chunks_per_row;
    const int sec = (int)(rem / chunks_per_row);
    const int64_t col = (rem - sec * chunks_per_row) * VEC;
    T v[VEC];
    if (sec == 0) {
#pragma unroll
      for (int j = 0; j < VEC; ++j) v[j] = gate[rec * d + col + j];
    } else if (sec == 1) {
#pragma unroll
      for (int j = 0; j < VEC; ++j) v[j] = up[rec * d + col + j];
    } else {
#pragma unroll
      for (int j = 0; j < VEC; ++j) v[j] = down[(col + j) * I + rec];
    }
    T *o = blob + (rec * 3 + sec) * d + col;
#pragma unroll
    for (int j = 0; j < VEC; ++j) o[j] = v[j];
  }
}

// h = (carry ? h : 0) + y + perturb*a ; x = h / sqrt(mean(h^2) + 1e-6) in act_fmt.  One workgroup.
__global__ __launch_bounds__(1024) void residual_rmsnorm_kernel(float *h, const void *y, const float *a,
                                                                float perturb, int carry, void *x, int d,
                                                                int act_fmt) {
  __shared__ float part[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float ss = 0.f;
  for (int j = tid; j < d; j += blockDim.x) {
    float v = carry ? h[j] : 0.f;
    if (y) v += (act_fmt == MOE_A_BF16) ? __uint_as_float((uint32_t) static_cast<const uint16_t *>(y)[j] << 16)
                                        : static_cast<const float *>(y)[j];
    if (a) v = __builtin_fmaf(perturb, a[j], v);
    h[j] = v;
    ss = __builtin_fmaf(v, v, ss);
  }
  ss = wave_sum(ss);
  if (lane == 0) part[wave] = ss;
  __syncthreads();
  float tot = 0.f;
  for (int w = 0; w < (int)(blockDim.x >> 6); ++w) tot += part[w];
  const float scale = 1.0f / sqrtf(tot / (float)d + 1e-6f);
  for (int j = tid; j < d; j += blockDim.x) {
    const float v = h[j] * scale;
    if (act_fmt == MOE_A_BF16)
      static_cast<uint16_t *>(x)[j] = f32_to_bf16_rne(v);
    else
      static_cast<float *>(x)[j] = v;
  }
}

}  // namespace

hipError_t launch_pack(int fmt, int hidden, int inter, const void *gate, const void *up, const void *down,
                       const void *gs, const void *us, const void *ds, void *blob, hipStream_t s) {
  (void)gs;
  (void)us;
  (void)ds;
  const int64_t chunks = (int64_t)inter * 3 * hidden / (fmt == MOE_W_FP32 ? 4 : 8);
  int grid = (int)((chunks + 255) / 256);
  if (grid > 65535) grid = 65535;
  if (fmt == MOE_W_FP32) {
    hipLaunchKernelGGL(pack_plain_kernel<float>, dim3(grid), dim3(256), 0, s, static_cast<const float *>(gate),
                       static_cast<const float *>(up), static_cast<const float *>(down), static_cast<float *>(blob),
                       hidden, inter);
  } else if (fmt == MOE_W_BF16) {
    hipLaunchKernelGGL(pack_plain_kernel<uint16_t>, dim3(grid), dim3(256), 0, s,
                       static_cast<const uint16_t *>(gate), static_cast<const uint16_t *>(up),
                       static_cast<const uint16_t *>(down), static_cast<uint16_t *>(blob), hidden, inter);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_residual_rmsnorm(float *h, const void *y, const float *a, float perturb, int carry, void *x,
                                   int hidden, int act_fmt, hipStream_t s) {
  hipLaunchKernelGGL(residual_rmsnorm_kernel, dim3(1), dim3(1024), 0, s, h, y, a, perturb, carry, x, hidden,
                     act_fmt);
  return hipGetLastError();
}

}  // namespace moe
