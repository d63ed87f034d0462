// moe_expert_forward_static: the expert computation of one layer-token (paper Eq. 1) for callers that may not
// allocate - code under HIP graph capture, tight serving loops.  It runs the same kernels as moe_expert_forward;
// what that call keeps in memory the context allocated (the compact routing record the kernels read and the fp32
// partial rows, one per workgroup) lives here in a fixed device array that is part of the library's code object.
#include <mutex>

#include "common.h"

namespace moe {
namespace {

constexpr int kStaticMaxHidden = 4096;  // every workload shape; bounds the scratch array
constexpr int kStaticMaxGrid = 256;     // workgroups = partial rows
constexpr size_t kRecordBytes = 512;    // moe_route_out_t, padded
static_assert(sizeof(moe_route_out_t) <= kRecordBytes, "record area");
constexpr size_t kScratchBytes = kRecordBytes + sizeof(float) * (size_t)kStaticMaxGrid * kStaticMaxHidden;

// [ routing record | partial rows ]: 4 MiB + 512 B per GPU, held until the process ends
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
struct PerDevice {
  void *ptr = nullptr;  // device address of `scratch` on this GPU (each GPU has its own copy of the array)
  int cus = 0;
};
PerDevice g_dev[kMaxDevices];
std::mutex g_mu;

struct Selection {
  int32_t slot[MOE_MAX_TOPK];
  float weight[MOE_MAX_TOPK];
};

// the routing record as the expert kernels read it: the K weights, the K slots 8 bits each, no expert missing
__global__ void static_record_kernel(moe_route_out_t *rec, Selection sel, int top_k) {
  const int i = threadIdx.x;
  uint32_t *w = reinterpret_cast<uint32_t *>(rec);
  if (i < (int)(sizeof(moe_route_out_t) / 4)) w[i] = 0u;
  __syncthreads();
  if (i < top_k) {
    rec->sel_slot[i] = sel.slot[i];
    rec->sel_weight[i] = sel.weight[i];
  }
  if (i == 0) {
    uint32_t lo = 0, hi = 0;
    for (int k = 0; k < top_k; ++k) {
      const uint32_t s8 = (uint32_t)sel.slot[k] & 0xffu;
      if (k < 4) lo |= s8 << (8 * k); else hi |= s8 << (8 * (k - 4));
    }
    rec->opaque[0] = 1u;
    rec->opaque[1] = lo;
    rec->opaque[2] = hi;
    rec->opaque[3] = 0u;  // miss mask: every selected expert is in its slot
  }
}

}  // namespace

// Once per device, with that device current: the device address of the scratch array and the number of compute
// units.  The array's name is a host-side handle, not an address; only the address obtained here may be given to
// kernels.  Allocates nothing.
hipError_t static_scratch_setup(int dev, void **ptr, int *cus) {
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_mu);
  PerDevice &d = g_dev[dev];
  if (d.ptr == nullptr) {
    void *p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    int n = 0;
    e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    d.cus = n;
    d.ptr = p;
  }
  if (ptr) *ptr = d.ptr;
  if (cus) *cus = d.cus;
  return hipSuccess;
}

hipError_t launch_expert_forward_static(int weight_fmt, int act_fmt, int hidden, int inter, int shared_inter, int top_k,
                                        const void *slot_pool, int64_t slot_bytes, const void *shared_blob,
                                        const int32_t *sel_slot, const float *sel_weight, const void *x, void *y,
                                        hipStream_t s) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  void *base = nullptr;
  int cus = 0;
  e = static_scratch_setup(dev, &base, &cus);
  if (e != hipSuccess) return e;
  moe_route_out_t *rec = static_cast<moe_route_out_t *>(base);
  float *partial = reinterpret_cast<float *>(static_cast<unsigned char *>(base) + kRecordBytes);
  GemvPlan plan = gemv_plan(cus, top_k * inter + shared_inter, weight_fmt, act_fmt);
  if (plan.grid > kStaticMaxGrid) plan.grid = kStaticMaxGrid;
  Selection sel{};
  for (int k = 0; k < top_k; ++k) {
    sel.slot[k] = sel_slot[k];
    sel.weight[k] = sel_weight[k];
  }
  hipLaunchKernelGGL(static_record_kernel, dim3(1), dim3(128), 0, s, rec, sel, top_k);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  GemvParams p{};
  p.slot_pool = static_cast<const uint8_t *>(slot_pool);
  p.shared_blob = shared_inter > 0 ? static_cast<const uint8_t *>(shared_blob) : nullptr;
  p.route = rec;
  p.x = x;
  p.partial = partial;
  p.hidden = hidden;
  p.inter = inter;
  p.shared_inter = shared_inter;
  p.top_k = top_k;
  p.act_fmt = act_fmt;
  p.slot_bytes = slot_bytes;
  p.pass = 0;
  p.row_offset = 0;
  p.fused = 0;
  e = launch_expert_gemv(p, weight_fmt, plan, s);
  if (e != hipSuccess) return e;
  return launch_partial_reduce(partial, plan.grid, y, hidden, act_fmt, s);
}

int static_max_hidden() { return kStaticMaxHidden; }

}  // namespace moe
