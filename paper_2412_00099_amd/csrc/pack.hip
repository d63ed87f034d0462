// Blob geometry, the canonical -> record-layout packer, and the synthetic-stack glue kernel.
#include "common.h"

namespace moe {

BlobLayout blob_layout(int fmt, int hidden, int inter) {
  BlobLayout L{};
  const int64_t d = hidden, I = inter;
  int64_t tail_bytes = 0;
  switch (fmt) {
    case MOE_W_FP32:
      L.row_bytes = d * 4;
      L.rec_bytes = 3 * L.row_bytes;
      break;
    case MOE_W_BF16:
      L.row_bytes = d * 2;
      L.rec_bytes = 3 * L.row_bytes;
      break;
    case MOE_W_INT8_PC:  // tail: gate scales [I], up scales [I], down scales [d], fp16
      L.row_bytes = d;
      L.rec_bytes = 3 * L.row_bytes;
      tail_bytes = (2 * I + d) * 2;
      break;
    case MOE_W_INT4_G128:  // record carries its (gate, up) group scales; tail: down scales [I/128][d], fp16
      L.row_bytes = d / 2;
      L.rec_bytes = int4_record_bytes(d);
      tail_bytes = (I / 128) * d * 2;
      break;
    default: return L;
  }
  L.tail_offset = I * L.rec_bytes;
  L.total = (L.tail_offset + tail_bytes + 255) / 256 * 256;
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

// int8: values become offset-binary bytes (q + 128); scales go to the tail.
__global__ void pack_int8_kernel(const int8_t *gate, const int8_t *up, const int8_t *down, const uint16_t *gs,
                                 const uint16_t *us, const uint16_t *ds, uint8_t *blob, int d, int I) {
  const int64_t chunks_per_row = d / 16;
  const int64_t n_chunks = (int64_t)I * 3 * chunks_per_row;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (int64_t c = gid; c < n_chunks; c += stride) {
    const int64_t rec = c / (3 * chunks_per_row);
    const int64_t rem = c - rec * 3 * chunks_per_row;
    const int sec = (int)(rem / chunks_per_row);
    const int64_t col = (rem - sec * chunks_per_row) * 16;
    uint8_t *o = blob + (rec * 3 + sec) * d + col;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int8_t q = sec == 0 ? gate[rec * d + col + j] : sec == 1 ? up[rec * d + col + j] : down[(col + j) * I + rec];
      o[j] = (uint8_t)q ^ 0x80u;
    }
  }
  uint16_t *tail = reinterpret_cast<uint16_t *>(blob + (int64_t)I * 3 * d);
  for (int64_t i = gid; i < 2 * (int64_t)I + d; i += stride)
    tail[i] = i < I ? gs[i] : i < 2 * (int64_t)I ? us[i - I] : ds[i - 2 * I];
}

// int4: canonical bytes hold two nibbles (even column low); gate/up rows are copied, the down column is
// gathered nibble by nibble; the record ends with its (gate, up) scale pairs, the down scales form the tail.
__global__ void pack_int4_kernel(const uint8_t *gate, const uint8_t *up, const uint8_t *down, const uint16_t *gs,
                                 const uint16_t *us, const uint16_t *ds, uint8_t *blob, int d, int I) {
  const int64_t row_bytes = d / 2, groups = d / 128, rec_bytes = int4_record_bytes(d);
  const int64_t chunks_per_row = row_bytes / 16;
  const int64_t n_chunks = (int64_t)I * 3 * chunks_per_row;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (int64_t c = gid; c < n_chunks; c += stride) {
    const int64_t rec = c / (3 * chunks_per_row);
    const int64_t rem = c - rec * 3 * chunks_per_row;
    const int sec = (int)(rem / chunks_per_row);
    const int64_t b0 = (rem - sec * chunks_per_row) * 16;  // first byte of the chunk inside the row
    uint8_t *o = blob + rec * rec_bytes + sec * row_bytes + b0;
    if (sec < 2) {
      const uint8_t *src = (sec == 0 ? gate : up) + rec * row_bytes + b0;
#pragma unroll
      for (int j = 0; j < 16; ++j) o[j] = src[j];
    } else {
      const int64_t in_row = I / 2;  // bytes per row of the canonical [d, I/2] matrix
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int64_t c0 = (b0 + j) * 2;  // two output columns share a byte
        const uint8_t a = down[c0 * in_row + rec / 2], b = down[(c0 + 1) * in_row + rec / 2];
        const int sh = (rec & 1) * 4;
        o[j] = (uint8_t)(((a >> sh) & 0xf) | (((b >> sh) & 0xf) << 4));
      }
    }
  }
  for (int64_t i = gid; i < (int64_t)I * groups; i += stride) {
    const int64_t rec = i / groups, g = i - rec * groups;
    uint16_t *o = reinterpret_cast<uint16_t *>(blob + rec * rec_bytes + 3 * row_bytes + g * 4);
    o[0] = gs[rec * groups + g];
    o[1] = us[rec * groups + g];
  }
  uint16_t *tail = reinterpret_cast<uint16_t *>(blob + (int64_t)I * rec_bytes);
  const int64_t rgroups = I / 128;
  for (int64_t i = gid; i < rgroups * d; i += stride) {
    const int64_t g = i / d, col = i - g * d;
    tail[i] = ds[col * rgroups + g];
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
  const int per16 = fmt == MOE_W_FP32 ? 4 : fmt == MOE_W_BF16 ? 8 : fmt == MOE_W_INT8_PC ? 16 : 32;
  const int64_t chunks = (int64_t)inter * 3 * hidden / per16;
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
  } else if (fmt == MOE_W_INT8_PC) {
    hipLaunchKernelGGL(pack_int8_kernel, dim3(grid), dim3(256), 0, s, static_cast<const int8_t *>(gate),
                       static_cast<const int8_t *>(up), static_cast<const int8_t *>(down),
                       static_cast<const uint16_t *>(gs), static_cast<const uint16_t *>(us),
                       static_cast<const uint16_t *>(ds), static_cast<uint8_t *>(blob), hidden, inter);
  } else if (fmt == MOE_W_INT4_G128) {
    hipLaunchKernelGGL(pack_int4_kernel, dim3(grid), dim3(256), 0, s, static_cast<const uint8_t *>(gate),
                       static_cast<const uint8_t *>(up), static_cast<const uint8_t *>(down),
                       static_cast<const uint16_t *>(gs), static_cast<const uint16_t *>(us),
                       static_cast<const uint16_t *>(ds), static_cast<uint8_t *>(blob), hidden, inter);
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
