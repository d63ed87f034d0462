// Host side of libmoe_cache: argument checking, the context, the per-layer step sequence
// (route kernel -> host learns the misses -> fills on the copy stream -> expert kernels) and statistics.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <algorithm>
#include <chrono>
#include <new>
#include <string>
#include <vector>

#include "common.h"

using namespace moe;

namespace {

thread_local std::string g_err;

int fail(int code, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

#define HIP_TRY(expr)                                                                        \
  do {                                                                                       \
    hipError_t e_ = (expr);                                                                  \
    if (e_ != hipSuccess) return fail(MOE_EHIP, "%s: %s", #expr, hipGetErrorString(e_));     \
  } while (0)

// Keeps the compute stream busy for about `ticks` periods of the 100 MHz wall clock (bounded by the iteration
// count whatever the clock does).  Enqueued ahead of a launch that is timed with events: the start event of such
// a launch is a marker of its own, enqueued a few microseconds of host time before the kernel, and on an idle
// stream it would be stamped that much before the kernel starts.  Behind this kernel both are queued by the time
// the marker is reached.
__global__ void hold_stream_kernel(uint64_t ticks) {
  const uint64_t t0 = wall_clock64();
  for (int i = 0; i < 4096 && wall_clock64() - t0 < ticks; ++i) __builtin_amdgcn_s_sleep(8);
}

bool valid_wfmt(int f) { return f >= MOE_W_FP32 && f <= MOE_W_INT4_G128; }
bool valid_afmt(int f) { return f == MOE_A_FP32 || f == MOE_A_BF16; }

}  // namespace

struct moe_cache {
  moe_cache_config_t cfg{};
  std::vector<const void *> host_blob;
  std::vector<void *> slot_pool;
  std::vector<const void *> gate_w;
  std::vector<const void *> shared_blob;
  std::vector<int32_t> initial;
  int32_t n_initial = 0;
  BlobLayout slot_layout{};
  hipStream_t compute = nullptr, copy = nullptr;

  LayerState *d_state = nullptr;
  moe_route_out_t *d_route = nullptr;
  HostNote *h_note = nullptr;      // pinned, mapped: the router's message to the host, one per layer
  HostNote *h_note_dev = nullptr;  // device view of h_note
  struct Decision {                // h_note decoded
    int n_miss = 0;
    uint8_t miss_mask = 0;
    uint8_t expert[MOE_MAX_TOPK] = {}, slot[MOE_MAX_TOPK] = {};
  };
  std::vector<Decision> decided;
  // layer boundaries deferred into the expert launch (see BoundaryArgs)
  std::vector<BoundaryArgs> boundary;
  uint64_t *d_handover = nullptr;   // [n_layers][64] self-tagged words: a boundary's decision for its own launch
  float *d_ss = nullptr;            // [128] sums of squares of the residual stream per 64 columns
  uint32_t *h_gave_up = nullptr;    // pinned, mapped: set by a wavefront that stopped waiting for the hand-over
  uint32_t *h_gave_up_dev = nullptr;
  bool fuse_boundary = true;        // run deferred boundaries inside the expert launch (see moe_cache_init)
  bool poison_fills = false;        // debugging aid: a slot is overwritten with NaN patterns before its fill (MOE_POISON_FILLS)
  int tag_spins = 1 << 18;          // polls (about a tenth of a second) before a workgroup stops waiting for
                                    // workgroup 0; MOE_TAG_SPINS lowers it so that tests reach the error path
  int32_t *d_initial = nullptr;
  float *d_partial = nullptr;
  int pending_rows = 0;            // partial rows of an expert output not reduced yet (y_dev was NULL)
  void *d_y = nullptr;             // [d] act_fmt: a pending expert output once summed, when the caller gave no y_dev
  GemvPlan plan{};
  hipEvent_t ev_route = nullptr;
  std::vector<hipEvent_t> ev_copy;
  std::vector<uint8_t> routed;        // per layer: 0 idle, 1 routed (decision on the host), 2 routed (not collected
                                      // yet), 3 boundary deferred into the expert launch
  std::vector<uint32_t> route_seq;    // per layer: completion tag of the pending route step
  std::vector<uint32_t> hand_count;   // per layer: hand-overs inside an expert launch so far
  std::vector<int64_t> bytes_filled;
  uint32_t seq = 0;
  bool poll = false;

  // prompt phase (moe_route_batch / moe_expert_forward_batch); allocated only for shapes the batched kernels take
  bool batch_ok = false;
  float *d_logits_batch = nullptr;          // [kMaxBatch][n_experts]
  moe_route_out_t *batch_rec = nullptr;      // [kMaxBatch] the decisions of the batch routed last: pinned host memory
  moe_route_out_t *batch_rec_dev = nullptr;  // the routing kernel's view of it (the records go straight to the host)
  float *d_bpartial = nullptr;              // [max_units][16][hidden]: the output tile of every unit
  // the tables of a launch, one block of pinned memory and its device copy (one transfer per launch):
  //   [max_tiles] tiles | [max_units] units | [kMaxBatch] partial rows per token | [kMaxBatch][max_contrib] their lists
  uint8_t *h_tables = nullptr, *d_tables = nullptr;
  size_t off_units = 0, off_contrib = 0;
  TokenTile *d_tiles = nullptr, *h_tiles = nullptr;
  BatchUnit *d_units = nullptr, *h_units = nullptr;
  int32_t *d_contrib = nullptr, *h_contrib = nullptr;
  int max_tiles = 0, max_units = 0, max_contrib = 0;
  int n_cus = 0;
  std::vector<BatchUnit> units_built;       // the units of a segment in the order they are made (tile by tile)
  std::vector<int32_t> unit_pos;            // their places in the launch
  std::vector<int32_t> xcd_queue[8];        // units per XCD, while the launch order is worked out
  std::vector<int32_t> unit_group_owner;    // per (blob, block of records): the XCD of its group
  std::vector<int32_t> tile_slot, tile_first_unit;
  int batch_layer = -1, batch_n = 0;
  hipEvent_t ev_batch = nullptr;            // compute stream has finished reading the slots (before fills overwrite them)

  // optional timing of the expert GEMV launches
  int profiling = 0;      // 0 = off, n = events on every n-th expert launch of a layer's first pass
  uint64_t prof_tick = 0;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> prof_events;
  std::vector<uint8_t> prof_full;  // launch covered the whole layer (no expert was missing)
  size_t prof_used = 0;
};

namespace {

int check_layer(const moe_cache_t *ctx, int32_t layer) {
  if (!ctx) return fail(MOE_EINVAL, "context is NULL");
  if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(MOE_EINVAL, "layer %d out of range [0,%d)", layer, ctx->cfg.n_layers);
  if (ctx->h_gave_up && __atomic_load_n(ctx->h_gave_up, __ATOMIC_RELAXED) != 0)
    return fail(MOE_EHIP, "an expert kernel gave up waiting for the layer boundary of its own launch: outputs since then are invalid");
  return MOE_OK;
}

int do_reset(moe_cache_t *c) {
  HIP_TRY(hipStreamSynchronize(c->compute));
  HIP_TRY(hipStreamSynchronize(c->copy));
  if (c->n_initial > 0)
    HIP_TRY(hipMemcpy(c->d_initial, c->initial.data(), c->initial.size() * sizeof(int32_t), hipMemcpyHostToDevice));
  HIP_TRY(launch_state_init(c->d_state, c->cfg.n_layers, c->d_initial, c->n_initial, c->compute));
  if (c->h_gave_up) __atomic_store_n(c->h_gave_up, 0u, __ATOMIC_RELAXED);
  c->pending_rows = 0;
  c->batch_layer = -1;
  c->batch_n = 0;
  const int N = c->cfg.n_experts;
  for (int l = 0; l < c->cfg.n_layers; ++l) {
    for (int i = 0; i < c->n_initial; ++i) {
      const int e = c->initial[(size_t)l * c->n_initial + i];
      HIP_TRY(hipMemcpy(static_cast<uint8_t *>(c->slot_pool[l]) + (size_t)i * c->slot_layout.total,
                        c->host_blob[(size_t)l * N + e], c->slot_layout.total, hipMemcpyHostToDevice));
    }
    c->routed[l] = 0;
    c->bytes_filled[l] = 0;
  }
  HIP_TRY(hipStreamSynchronize(c->compute));
  return MOE_OK;
}

}  // namespace

extern "C" {

const char *moe_last_error(void) { return g_err.c_str(); }

size_t moe_blob_bytes(int32_t weight_fmt, int32_t hidden, int32_t inter) {
  if (!valid_wfmt(weight_fmt) || hidden <= 0 || inter <= 0) return 0;
  if (!gemv_shape_supported(weight_fmt, hidden) || !gemv_inter_supported(weight_fmt, inter)) return 0;
  return (size_t)blob_layout(weight_fmt, hidden, inter).total;
}

size_t moe_slot_bytes(const moe_cache_config_t *cfg) {
  if (!cfg) return 0;
  return moe_blob_bytes(cfg->weight_fmt, cfg->hidden, cfg->inter);
}

int moe_pack_expert(int32_t weight_fmt, int32_t hidden, int32_t inter, const void *gate, const void *up,
                    const void *down, const void *gate_s, const void *up_s, const void *down_s, void *blob_dev,
                    void *stream) {
  if (!valid_wfmt(weight_fmt)) return fail(MOE_EINVAL, "unknown weight format %d", weight_fmt);
  if (hidden <= 0 || inter <= 0 || !gemv_shape_supported(weight_fmt, hidden) ||
      !gemv_inter_supported(weight_fmt, inter))
    return fail(MOE_EINVAL, "unsupported shape hidden=%d inter=%d for weight format %d", hidden, inter, weight_fmt);
  if (!gate || !up || !down || !blob_dev) return fail(MOE_EINVAL, "NULL weight or blob pointer");
  const bool quant = weight_fmt == MOE_W_INT8_PC || weight_fmt == MOE_W_INT4_G128;
  if (quant && (!gate_s || !up_s || !down_s)) return fail(MOE_EINVAL, "quantised format needs scale pointers");
  HIP_TRY(launch_pack(weight_fmt, hidden, inter, gate, up, down, gate_s, up_s, down_s, blob_dev,
                      static_cast<hipStream_t>(stream)));
  return MOE_OK;
}

int moe_cache_init(const moe_cache_config_t *cfg, const moe_cache_buffers_t *b, moe_cache_t **out) {
  if (!out) return fail(MOE_EINVAL, "out is NULL");
  *out = nullptr;
  if (!cfg || !b) return fail(MOE_EINVAL, "config or buffers is NULL");
  // ---- everything below is checked before the first HIP call ----
  if (cfg->n_layers <= 0) return fail(MOE_EINVAL, "n_layers must be positive");
  if (cfg->n_experts <= 0 || cfg->n_experts > MOE_MAX_EXPERTS)
    return fail(MOE_EINVAL, "n_experts must be in 1..%d", MOE_MAX_EXPERTS);
  if (cfg->top_k <= 0 || cfg->top_k > MOE_MAX_TOPK) return fail(MOE_EINVAL, "top_k must be in 1..%d", MOE_MAX_TOPK);
  if (cfg->top_j < 0 || cfg->top_j > cfg->top_k) return fail(MOE_EINVAL, "top_j must be in 0..top_k");
  if (cfg->capacity < cfg->top_k) return fail(MOE_EINVAL, "capacity %d < top_k %d: a token's experts must all be resident", cfg->capacity, cfg->top_k);
  if (cfg->capacity > cfg->n_experts) return fail(MOE_EINVAL, "capacity exceeds n_experts");
  if (!valid_wfmt(cfg->weight_fmt) || !valid_afmt(cfg->act_fmt)) return fail(MOE_EINVAL, "unknown weight or activation format");
  if (cfg->inter <= 0 || cfg->shared_inter < 0) return fail(MOE_EINVAL, "bad intermediate size");
  if (!gemv_shape_supported(cfg->weight_fmt, cfg->hidden))
    return fail(MOE_EINVAL, "hidden=%d unsupported for weight format %d (needs 64*{1,2,4,8} 16-byte loads per row)", cfg->hidden, cfg->weight_fmt);
  if (!gemv_inter_supported(cfg->weight_fmt, cfg->inter) ||
      (cfg->shared_inter > 0 && !gemv_inter_supported(cfg->weight_fmt, cfg->shared_inter)))
    return fail(MOE_EINVAL, "intermediate size unsupported for this weight format (int8: multiple of 8, int4: multiple of 128)");
  if ((int64_t)cfg->top_k * cfg->inter + cfg->shared_inter > (int64_t)1 << 22)
    return fail(MOE_EINVAL, "more than 2^22 expert records per layer-token");
  if (!(cfg->lambda >= 0.f) || !std::isfinite(cfg->lambda)) return fail(MOE_EINVAL, "lambda must be finite and >= 0");
  if (cfg->delta_mode < MOE_DELTA_RUNNING_MEAN || cfg->delta_mode > MOE_DELTA_TOKEN) return fail(MOE_EINVAL, "bad delta_mode");
  if (cfg->delta_mode == MOE_DELTA_FIXED && !std::isfinite(cfg->delta_fixed)) return fail(MOE_EINVAL, "delta_fixed must be finite");
  if (cfg->route_mode < MOE_ROUTE_CACHE_PRIOR || cfg->route_mode > MOE_ROUTE_CUMSUM) return fail(MOE_EINVAL, "bad route_mode");
  if (cfg->route_mode == MOE_ROUTE_MAX_RANK && (cfg->max_rank < 0 || cfg->max_rank > cfg->n_experts))
    return fail(MOE_EINVAL, "max_rank must be in 0..n_experts");
  if (cfg->route_mode == MOE_ROUTE_CUMSUM && !(cfg->cumsum_p >= 0.f)) return fail(MOE_EINVAL, "cumsum_p must be >= 0");
  if (cfg->renormalize != 0 && cfg->renormalize != 1) return fail(MOE_EINVAL, "renormalize must be 0 or 1");
  if (cfg->compute_stream == cfg->copy_stream) return fail(MOE_EINVAL, "copy_stream must differ from compute_stream");
  if (!b->host_expert_blob || !b->slot_pool || !b->gate_w) return fail(MOE_EINVAL, "NULL buffer table");
  if (cfg->shared_inter > 0 && !b->shared_blob) return fail(MOE_EINVAL, "shared_inter > 0 needs shared_blob");
  if (b->n_initial < 0 || b->n_initial > cfg->capacity) return fail(MOE_EINVAL, "n_initial must be in 0..capacity");
  if (b->n_initial > 0 && !b->initial_resident) return fail(MOE_EINVAL, "n_initial > 0 needs initial_resident");
  const int L = cfg->n_layers, N = cfg->n_experts;
  for (int l = 0; l < L; ++l) {
    if (!b->slot_pool[l] || !b->gate_w[l]) return fail(MOE_EINVAL, "NULL slot pool or gate matrix for layer %d", l);
    if (reinterpret_cast<uintptr_t>(b->slot_pool[l]) % 256 != 0) return fail(MOE_EINVAL, "slot pool of layer %d not 256-byte aligned", l);
    if (cfg->shared_inter > 0 && !b->shared_blob[l]) return fail(MOE_EINVAL, "NULL shared blob for layer %d", l);
    for (int e = 0; e < N; ++e)
      if (!b->host_expert_blob[(size_t)l * N + e]) return fail(MOE_EINVAL, "NULL host blob for layer %d expert %d", l, e);
    uint64_t seen = 0;
    for (int i = 0; i < b->n_initial; ++i) {
      const int e = b->initial_resident[(size_t)l * b->n_initial + i];
      if (e < 0 || e >= N || ((seen >> e) & 1)) return fail(MOE_EINVAL, "initial_resident of layer %d: bad or repeated expert %d", l, e);
      seen |= 1ull << e;
    }
  }

  moe_cache_t *c = new (std::nothrow) moe_cache;
  if (!c) return fail(MOE_ENOMEM, "out of host memory");
  c->cfg = *cfg;
  c->host_blob.assign(b->host_expert_blob, b->host_expert_blob + (size_t)L * N);
  c->slot_pool.assign(b->slot_pool, b->slot_pool + L);
  c->gate_w.assign(b->gate_w, b->gate_w + L);
  if (cfg->shared_inter > 0) c->shared_blob.assign(b->shared_blob, b->shared_blob + L);
  c->n_initial = b->n_initial;
  if (b->n_initial > 0) c->initial.assign(b->initial_resident, b->initial_resident + (size_t)L * b->n_initial);
  c->slot_layout = blob_layout(cfg->weight_fmt, cfg->hidden, cfg->inter);
  c->compute = static_cast<hipStream_t>(cfg->compute_stream);
  c->copy = static_cast<hipStream_t>(cfg->copy_stream);
  c->routed.assign(L, 0);
  c->route_seq.assign(L, 0);
  c->hand_count.assign(L, 0);
  c->decided.assign(L, {});
  c->boundary.assign(L, BoundaryArgs{});
  c->bytes_filled.assign(L, 0);
  c->ev_copy.assign(L, nullptr);

  auto bail = [&](int code) {
    moe_cache_destroy(c);
    return code;
  };
#define HIP_INIT(expr)                                                                      \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) {                                                                 \
      fail(e_ == hipErrorOutOfMemory ? MOE_ENOMEM : MOE_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
      return bail(e_ == hipErrorOutOfMemory ? MOE_ENOMEM : MOE_EHIP);                       \
    }                                                                                       \
  } while (0)

  int dev = 0;
  HIP_INIT(hipGetDevice(&dev));
  int cus = 0;
  HIP_INIT(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  HIP_INIT(static_scratch_setup(dev, nullptr, nullptr));  // moe_expert_forward_static's scratch array on this device
  c->n_cus = cus;
  c->plan = gemv_plan(cus, cfg->top_k * cfg->inter + cfg->shared_inter, cfg->weight_fmt, cfg->act_fmt);
  // the host learns a routing decision by polling the three self-tagged words the router stores into mapped host
  // memory (each complete in itself, no ordering between them); MOE_HOST_SYNC=event waits on a stream event instead
  c->poll = true;
  if (const char *s = getenv("MOE_HOST_SYNC")) c->poll = strcmp(s, "event") != 0;

  HIP_INIT(hipMalloc(&c->d_state, sizeof(LayerState) * L));
  HIP_INIT(hipMalloc(&c->d_route, sizeof(moe_route_out_t) * L));
  HIP_INIT(hipMemset(c->d_route, 0, sizeof(moe_route_out_t) * L));
  HIP_INIT(hipHostMalloc(reinterpret_cast<void **>(&c->h_note), sizeof(HostNote) * L,
                         hipHostMallocMapped | hipHostMallocCoherent));
  memset(c->h_note, 0, sizeof(HostNote) * L);
  HIP_INIT(hipHostGetDevicePointer(reinterpret_cast<void **>(&c->h_note_dev), c->h_note, 0));
  HIP_INIT(hipMalloc(&c->d_handover, sizeof(uint64_t) * 64 * (size_t)L));
  HIP_INIT(hipMemset(c->d_handover, 0, sizeof(uint64_t) * 64 * (size_t)L));
  HIP_INIT(hipMalloc(&c->d_ss, sizeof(float) * 128));
  HIP_INIT(hipMemset(c->d_ss, 0, sizeof(float) * 128));
  HIP_INIT(hipHostMalloc(reinterpret_cast<void **>(&c->h_gave_up), sizeof(uint32_t),
                         hipHostMallocMapped | hipHostMallocCoherent));
  *c->h_gave_up = 0;
  HIP_INIT(hipHostGetDevicePointer(reinterpret_cast<void **>(&c->h_gave_up_dev), c->h_gave_up, 0));
  // The boundary inside the expert launch pays off when the shared expert gives the other workgroups enough to do
  // until the routing record exists (measured: a gain of 20 % at one half of the records, none at one quarter).
  // MOE_FUSE_BOUNDARY=0 / 1 in the environment overrides the rule.
  c->fuse_boundary = 3 * (int64_t)cfg->shared_inter >= (int64_t)cfg->top_k * cfg->inter + cfg->shared_inter;
  if (const char *s = getenv("MOE_FUSE_BOUNDARY")) c->fuse_boundary = atoi(s) != 0;
  if (const char *s = getenv("MOE_POISON_FILLS")) c->poison_fills = atoi(s) != 0;
  if (const char *s = getenv("MOE_TAG_SPINS")) if (atoi(s) > 0) c->tag_spins = atoi(s);
  HIP_INIT(hipMalloc(&c->d_initial, sizeof(int32_t) * (size_t)L * (b->n_initial > 0 ? b->n_initial : 1)));
  HIP_INIT(hipMalloc(&c->d_partial, sizeof(float) * 2 * (size_t)c->plan.grid * cfg->hidden));
  HIP_INIT(hipMalloc(&c->d_y, sizeof(float) * (size_t)cfg->hidden));
  c->batch_ok = batch_shape_supported(cfg->weight_fmt, cfg->act_fmt, cfg->hidden, cfg->inter, cfg->shared_inter);
  if (c->batch_ok) {
    // (units of fewer records are only made while a launch stays within one workgroup per compute unit, below)
    const int chunks = std::max((cfg->inter + kBatchUnitRecords - 1) / kBatchUnitRecords, 1);
    const int schunks = std::max((cfg->shared_inter + kBatchUnitRecords - 1) / kBatchUnitRecords, cfg->shared_inter > 0 ? 1 : 0);
    // a tile is 16 tokens of one slot: at most one partly filled tile per slot plus the full ones
    const int routed_tiles = cfg->capacity + kMaxBatch * cfg->top_k / 16, shared_tiles = kMaxBatch / 16;
    c->max_tiles = routed_tiles + shared_tiles;
    c->max_units = std::max(routed_tiles * chunks + shared_tiles * schunks, cus);
    HIP_INIT(hipMalloc(&c->d_logits_batch, sizeof(float) * kMaxBatch * MOE_MAX_EXPERTS));
    HIP_INIT(hipHostMalloc(reinterpret_cast<void **>(&c->batch_rec), sizeof(moe_route_out_t) * kMaxBatch, hipHostMallocMapped));
    HIP_INIT(hipHostGetDevicePointer(reinterpret_cast<void **>(&c->batch_rec_dev), c->batch_rec, 0));
    c->max_contrib = std::max(cfg->top_k * chunks + schunks, cus);
    HIP_INIT(hipMalloc(&c->d_bpartial, sizeof(float) * (size_t)c->max_units * 16 * cfg->hidden));
    c->off_units = (sizeof(TokenTile) * c->max_tiles + 255) / 256 * 256;
    c->off_contrib = (c->off_units + sizeof(BatchUnit) * c->max_units + 255) / 256 * 256;
    const size_t table_bytes = c->off_contrib + sizeof(int32_t) * (size_t)kMaxBatch * (c->max_contrib + 1);
    HIP_INIT(hipMalloc(&c->d_tables, table_bytes));
    HIP_INIT(hipHostMalloc(reinterpret_cast<void **>(&c->h_tables), table_bytes, hipHostMallocDefault));
    c->h_tiles = reinterpret_cast<TokenTile *>(c->h_tables);
    c->d_tiles = reinterpret_cast<TokenTile *>(c->d_tables);
    c->h_units = reinterpret_cast<BatchUnit *>(c->h_tables + c->off_units);
    c->d_units = reinterpret_cast<BatchUnit *>(c->d_tables + c->off_units);
    c->h_contrib = reinterpret_cast<int32_t *>(c->h_tables + c->off_contrib);
    c->d_contrib = reinterpret_cast<int32_t *>(c->d_tables + c->off_contrib);
    HIP_INIT(hipEventCreateWithFlags(&c->ev_batch, hipEventDisableTiming));
  }
  HIP_INIT(hipEventCreateWithFlags(&c->ev_route, hipEventDisableTiming));
  for (int l = 0; l < L; ++l) HIP_INIT(hipEventCreateWithFlags(&c->ev_copy[l], hipEventDisableTiming));
#undef HIP_INIT
  int rc = do_reset(c);
  if (rc != MOE_OK) return bail(rc);
  *out = c;
  return MOE_OK;
}

void moe_cache_destroy(moe_cache_t *c) {
  if (!c) return;
  (void)hipStreamSynchronize(c->compute);
  (void)hipStreamSynchronize(c->copy);
  if (c->d_state) (void)hipFree(c->d_state);
  if (c->d_route) (void)hipFree(c->d_route);
  if (c->h_note) (void)hipHostFree(c->h_note);
  if (c->d_handover) (void)hipFree(c->d_handover);
  if (c->d_ss) (void)hipFree(c->d_ss);
  if (c->h_gave_up) (void)hipHostFree(c->h_gave_up);
  if (c->d_initial) (void)hipFree(c->d_initial);
  if (c->d_partial) (void)hipFree(c->d_partial);
  if (c->d_y) (void)hipFree(c->d_y);
  if (c->d_logits_batch) (void)hipFree(c->d_logits_batch);
  if (c->batch_rec) (void)hipHostFree(c->batch_rec);
  if (c->d_bpartial) (void)hipFree(c->d_bpartial);
  if (c->d_tables) (void)hipFree(c->d_tables);
  if (c->h_tables) (void)hipHostFree(c->h_tables);
  if (c->ev_batch) (void)hipEventDestroy(c->ev_batch);
  if (c->ev_route) (void)hipEventDestroy(c->ev_route);
  for (hipEvent_t e : c->ev_copy)
    if (e) (void)hipEventDestroy(e);
  for (auto &pr : c->prof_events) {
    (void)hipEventDestroy(pr.first);
    (void)hipEventDestroy(pr.second);
  }
  delete c;
}

// Wait until the routing decision of `layer` (tag `seq`) is visible on the host, decode it, then enqueue the fills
// of the missed experts on the copy stream.  Returns the number of misses through *n_miss.
static int collect_route(moe_cache_t *c, int32_t layer, uint32_t seq, int *n_miss) {
  const moe_cache_config_t &g = c->cfg;
  const HostNote *h = c->h_note + layer;
  const uint64_t tag = seq & 0xffffu;
  uint64_t w0 = 0, w1 = 0, w2 = 0;
  auto arrived = [&]() {
    w0 = __atomic_load_n(&h->w[0], __ATOMIC_ACQUIRE);
    w1 = __atomic_load_n(&h->w[1], __ATOMIC_ACQUIRE);
    w2 = __atomic_load_n(&h->w[2], __ATOMIC_ACQUIRE);
    return (uint32_t)w0 == seq && (w1 & 0xffffu) == tag && (w2 & 0xffffu) == tag;
  };
  bool seen = false;
  if (c->poll) {
    const auto t0 = std::chrono::steady_clock::now();
    for (uint32_t spin = 0;; ++spin) {
      if (arrived()) {
        seen = true;
        break;
      }
      if ((spin & 0x3ff) == 0x3ff && std::chrono::steady_clock::now() - t0 > std::chrono::milliseconds(200))
        break;  // fall back to a stream synchronisation (also surfaces launch errors)
    }
  }
  if (!seen) {
    HIP_TRY(hipEventRecord(c->ev_route, c->compute));
    HIP_TRY(hipEventSynchronize(c->ev_route));
    if (!arrived()) return fail(MOE_EHIP, "route kernel of layer %d did not publish its result", layer);
  }
  moe_cache::Decision &d = c->decided[layer];
  d.n_miss = (int)((w0 >> 32) & 0xff);
  d.miss_mask = (uint8_t)((w0 >> 40) & 0xff);
  for (int k = 0; k < g.top_k; ++k) {
    d.expert[k] = (uint8_t)((w1 >> (16 + 6 * k)) & 63);
    d.slot[k] = (uint8_t)((w2 >> (16 + 6 * k)) & 63);
  }
  const size_t slot_bytes = (size_t)c->slot_layout.total;
  if (d.n_miss > 0) {
    for (int k = 0; k < g.top_k; ++k) {
      if (!((d.miss_mask >> k) & 1)) continue;
      const int e = d.expert[k], s = d.slot[k];
      if (e >= g.n_experts || s >= g.capacity)
        return fail(MOE_EHIP, "route kernel returned expert %d slot %d out of range", e, s);
      // (debugging aid: whatever uses the slot before the fill has landed then computes NaNs, which no parity
      // test lets pass)
      if (c->poison_fills)
        HIP_TRY(hipMemsetAsync(static_cast<uint8_t *>(c->slot_pool[layer]) + (size_t)s * slot_bytes, 0xff, slot_bytes, c->copy));
      HIP_TRY(hipMemcpyAsync(static_cast<uint8_t *>(c->slot_pool[layer]) + (size_t)s * slot_bytes,
                             c->host_blob[(size_t)layer * g.n_experts + e], slot_bytes, hipMemcpyHostToDevice,
                             c->copy));
      c->bytes_filled[layer] += (int64_t)slot_bytes;
    }
    HIP_TRY(hipEventRecord(c->ev_copy[layer], c->copy));
  }
  *n_miss = d.n_miss;
  return MOE_OK;
}

// the full decision record of a layer, from device memory (waits for the compute stream)
static int fetch_record(moe_cache_t *c, int32_t layer, moe_route_out_t *out) {
  HIP_TRY(hipMemcpyAsync(out, c->d_route + layer, sizeof *out, hipMemcpyDeviceToHost, c->compute));
  HIP_TRY(hipStreamSynchronize(c->compute));
  return MOE_OK;
}

static RouteParams make_route_params(moe_cache_t *c) {
  const moe_cache_config_t &g = c->cfg;
  RouteParams p{};
  p.n_experts = g.n_experts;
  p.top_k = g.top_k;
  p.top_j = g.top_j;
  p.capacity = g.capacity;
  p.hidden = g.hidden;
  p.act_fmt = g.act_fmt;
  p.renormalize = g.renormalize;
  p.delta_mode = g.delta_mode;
  p.route_mode = g.route_mode;
  p.max_rank = g.max_rank;
  p.lambda = g.lambda;
  p.delta_fixed = g.delta_fixed;
  p.cumsum_p = g.cumsum_p;
  if (++c->seq == 0) c->seq = 1;
  p.seq = c->seq;
  return p;
}

// after the router launch: either leave the decision for moe_expert_forward, or wait for it now
static int finish_route_call(moe_cache_t *c, int32_t layer, uint32_t seq, moe_route_out_t *out_host) {
  c->route_seq[layer] = seq;
  if (!out_host) {
    c->routed[layer] = 2;  // decision collected by moe_expert_forward, behind the first expert launch
    return MOE_OK;
  }
  int n_miss = 0;
  if (int rc = collect_route(c, layer, seq, &n_miss)) return rc;
  c->routed[layer] = 1;
  return fetch_record(c, layer, out_host);
}

int moe_route_step(moe_cache_t *c, int32_t layer, const void *x_dev, const float *logits_dev,
                   moe_route_out_t *out_host) {
  if (int rc = check_layer(c, layer)) return rc;
  if ((x_dev == nullptr) == (logits_dev == nullptr)) return fail(MOE_EINVAL, "exactly one of x_dev and logits_dev must be given");
  if (c->routed[layer]) return fail(MOE_ESTATE, "layer %d: previous route step not followed by moe_expert_forward", layer);
  if (c->pending_rows) return fail(MOE_ESTATE, "an expert output is pending: the next routing call must be moe_stack_route_step");
  if (c->batch_layer >= 0) return fail(MOE_ESTATE, "a routed batch is pending: call moe_expert_forward_batch first");
  const RouteParams p = make_route_params(c);
  HIP_TRY(launch_route(p, c->gate_w[layer], x_dev, logits_dev, c->d_state + layer, c->d_route + layer,
                       c->h_note_dev + layer, c->compute));
  return finish_route_call(c, layer, p.seq, out_host);
}

int moe_stack_route_step(moe_cache_t *c, int32_t layer, float *h_dev, const float *a_dev, float perturb,
                         int32_t carry, void *x_dev, void *y_dev, moe_route_out_t *out_host) {
  if (int rc = check_layer(c, layer)) return rc;
  if (!h_dev || !x_dev) return fail(MOE_EINVAL, "h_dev or x_dev is NULL");
  if (c->cfg.hidden > kFusedMaxHidden) return fail(MOE_EINVAL, "hidden exceeds %d", kFusedMaxHidden);
  if (c->routed[layer]) return fail(MOE_ESTATE, "layer %d: previous route step not followed by moe_expert_forward", layer);
  if (c->batch_layer >= 0) return fail(MOE_ESTATE, "a routed batch is pending: call moe_expert_forward_batch first");
  const RouteParams p = make_route_params(c);
  const bool in_launch = !out_host && c->fuse_boundary &&
                         gemv_fused_supported(c->cfg.weight_fmt, c->cfg.act_fmt, c->cfg.hidden, c->plan) && c->cfg.hidden % 64 == 0;
  // the pending expert output is summed first (into y_dev if given, else into the library's own buffer)
  void *y = nullptr;
  if (c->pending_rows > 0) y = y_dev ? y_dev : c->d_y;
  FusedParams f{};
  f.h = h_dev;
  f.x_out = x_dev;
  if (in_launch) {
    // nobody waits for the decision here: the sum of the pending output and the residual glue are one launch, and
    // the rest of the boundary (x, gate GEMV, routing) runs in workgroup 0 of the layer's expert launch
    HIP_TRY(launch_reduce_glue(c->d_partial, c->pending_rows, y, c->cfg.hidden, c->cfg.act_fmt, h_dev, a_dev, perturb,
                               carry, c->d_ss, c->compute));
    c->pending_rows = 0;
    f.ss = c->d_ss;
    f.n_ss = c->cfg.hidden / 64;
    BoundaryArgs &b = c->boundary[layer];
    b.route = p;
    b.glue = f;
    b.gate_w = c->gate_w[layer];
    b.state = c->d_state + layer;
    b.out_dev = c->d_route + layer;
    b.note = c->h_note_dev + layer;
    b.handover = c->d_handover + 64 * (size_t)layer;
    b.hand_tag = ++c->hand_count[layer] & 0xffffu;  // the words hold count - 1 (0 at first): never equal
    b.gave_up = c->h_gave_up_dev;
    b.spin_limit = c->tag_spins;
    b.next_gate_w = c->gate_w[(layer + 1) % c->cfg.n_layers];
    b.next_state = c->d_state + (layer + 1) % c->cfg.n_layers;
    b.gate_bytes = (int64_t)c->cfg.n_experts * c->cfg.hidden * (c->cfg.act_fmt == MOE_A_BF16 ? 2 : 4);
    c->route_seq[layer] = p.seq;
    c->routed[layer] = 3;
    return MOE_OK;
  }
  if (fused_route_pre_supported(c->cfg.hidden)) {
    // the sum of the pending output and the residual glue spread over d / 64 workgroups; the single-workgroup
    // boundary launch then starts from h and the sums of squares
    HIP_TRY(launch_reduce_glue(c->d_partial, c->pending_rows, y, c->cfg.hidden, c->cfg.act_fmt, h_dev, a_dev, perturb,
                               carry, c->d_ss, c->compute));
    f.ss = c->d_ss;
    f.n_ss = c->cfg.hidden / 64;
  } else {
    if (c->pending_rows > 0)
      HIP_TRY(launch_partial_reduce(c->d_partial, c->pending_rows, y, c->cfg.hidden, c->cfg.act_fmt, c->compute));
    f.y = y;
    f.a = a_dev;
    f.perturb = perturb;
    f.carry = carry;
  }
  c->pending_rows = 0;
  HIP_TRY(launch_fused_route(p, f, c->gate_w[layer], c->d_state + layer, c->d_route + layer, c->h_note_dev + layer,
                             c->compute));
  return finish_route_call(c, layer, p.seq, out_host);
}

int moe_expert_forward(moe_cache_t *c, int32_t layer, const void *x_dev, void *y_dev) {
  if (int rc = check_layer(c, layer)) return rc;
  if (!x_dev) return fail(MOE_EINVAL, "x_dev is NULL");
  if (!c->routed[layer]) return fail(MOE_ESTATE, "layer %d: moe_expert_forward without a preceding moe_route_step", layer);
  if (c->pending_rows) return fail(MOE_ESTATE, "an expert output is pending: call moe_stack_route_step first");
  const moe_cache_config_t &g = c->cfg;
  GemvParams p{};
  p.slot_pool = static_cast<const uint8_t *>(c->slot_pool[layer]);
  p.shared_blob = g.shared_inter > 0 ? static_cast<const uint8_t *>(c->shared_blob[layer]) : nullptr;
  p.route = c->d_route + layer;
  p.x = x_dev;
  p.partial = c->d_partial;
  p.hidden = g.hidden;
  p.inter = g.inter;
  p.shared_inter = g.shared_inter;
  p.top_k = g.top_k;
  p.act_fmt = g.act_fmt;
  p.slot_bytes = c->slot_layout.total;
  // pass 0: the shared expert and the experts that were resident; it reads slots, weights and miss flags from
  // the device record, so it is launched before the host knows the decision
  p.pass = 0;
  p.row_offset = 0;
  if (c->routed[layer] == 3) {
    if (x_dev != c->boundary[layer].glue.x_out)
      return fail(MOE_EINVAL, "layer %d: x_dev must be the vector moe_stack_route_step wrote", layer);
    p.fused = 1;
    p.b = c->boundary[layer];
  }
  const bool prof = c->profiling && c->prof_tick++ % (uint64_t)c->profiling == 0 && c->prof_used < c->prof_events.size();
  if (prof) {
    hipLaunchKernelGGL(hold_stream_kernel, dim3(1), dim3(64), 0, c->compute, (uint64_t)5000);  // 50 us
    HIP_TRY(hipGetLastError());
    HIP_TRY(launch_expert_gemv(p, g.weight_fmt, c->plan, c->compute, c->prof_events[c->prof_used].first,
                               c->prof_events[c->prof_used].second));
  } else {
    HIP_TRY(launch_expert_gemv(p, g.weight_fmt, c->plan, c->compute));
  }
  p.fused = 0;
  int n_miss = c->decided[layer].n_miss;
  if (c->routed[layer] >= 2) {
    if (int rc = collect_route(c, layer, c->route_seq[layer], &n_miss)) return rc;
  }
  if (prof) c->prof_full[c->prof_used++] = n_miss == 0;
  int rows = c->plan.grid;
  if (n_miss > 0) {
    // pass 1: the experts whose slots are being filled, once the fills have landed
    HIP_TRY(hipStreamWaitEvent(c->compute, c->ev_copy[layer], 0));
    p.pass = 1;
    p.row_offset = c->plan.grid;
    HIP_TRY(launch_expert_gemv(p, g.weight_fmt, c->plan, c->compute));
    rows = 2 * c->plan.grid;
  }
  if (y_dev)
    HIP_TRY(launch_partial_reduce(c->d_partial, rows, y_dev, g.hidden, g.act_fmt, c->compute));
  else
    c->pending_rows = rows;  // finished by the next moe_stack_route_step
  c->routed[layer] = 0;
  return MOE_OK;
}

int moe_expert_forward_static(int32_t weight_fmt, int32_t act_fmt, int32_t hidden, int32_t inter, int32_t shared_inter,
                              int32_t top_k, const void *slot_pool_dev, int32_t n_slots, const void *shared_blob_dev,
                              const int32_t *sel_slot_host, const float *sel_weight_host, const void *x_dev,
                              void *y_dev, void *stream) {
  if (!valid_wfmt(weight_fmt) || !valid_afmt(act_fmt)) return fail(MOE_EINVAL, "unknown weight or activation format");
  if (hidden <= 0 || hidden > static_max_hidden())
    return fail(MOE_EINVAL, "hidden=%d beyond the fixed scratch buffer of this entry point (at most %d)", hidden, static_max_hidden());
  if (!gemv_shape_supported(weight_fmt, hidden)) return fail(MOE_EINVAL, "hidden=%d unsupported for weight format %d", hidden, weight_fmt);
  if (inter <= 0 || shared_inter < 0 || !gemv_inter_supported(weight_fmt, inter) ||
      (shared_inter > 0 && !gemv_inter_supported(weight_fmt, shared_inter)))
    return fail(MOE_EINVAL, "intermediate size unsupported for this weight format");
  if (top_k <= 0 || top_k > MOE_MAX_TOPK) return fail(MOE_EINVAL, "top_k must be in 1..%d", MOE_MAX_TOPK);
  if ((int64_t)top_k * inter + shared_inter > (int64_t)1 << 22) return fail(MOE_EINVAL, "more than 2^22 expert records");
  if (n_slots <= 0 || n_slots > 256) return fail(MOE_EINVAL, "n_slots must be in 1..256");
  if (!slot_pool_dev || !sel_slot_host || !sel_weight_host || !x_dev || !y_dev) return fail(MOE_EINVAL, "NULL argument");
  if (shared_inter > 0 && !shared_blob_dev) return fail(MOE_EINVAL, "shared_inter > 0 needs shared_blob_dev");
  for (int k = 0; k < top_k; ++k) {
    if (sel_slot_host[k] < 0 || sel_slot_host[k] >= n_slots) return fail(MOE_EINVAL, "sel_slot[%d]=%d outside 0..%d", k, sel_slot_host[k], n_slots - 1);
    if (!std::isfinite(sel_weight_host[k])) return fail(MOE_EINVAL, "sel_weight[%d] is not finite", k);
  }
  const int64_t slot_bytes = blob_layout(weight_fmt, hidden, inter).total;
  HIP_TRY(launch_expert_forward_static(weight_fmt, act_fmt, hidden, inter, shared_inter, top_k, slot_pool_dev, slot_bytes,
                                       shared_blob_dev, sel_slot_host, sel_weight_host, x_dev, y_dev,
                                       static_cast<hipStream_t>(stream)));
  return MOE_OK;
}

int moe_route_batch(moe_cache_t *c, int32_t layer, const void *x_dev, const float *logits_dev, int32_t n_tokens,
                    moe_route_out_t *out_host) {
  if (int rc = check_layer(c, layer)) return rc;
  if (!c->batch_ok) return fail(MOE_EINVAL, "the prompt-phase kernels take bf16 weights and activations, hidden 1024 or 2048, intermediate sizes that are multiples of 16");
  if ((x_dev == nullptr) == (logits_dev == nullptr)) return fail(MOE_EINVAL, "exactly one of x_dev and logits_dev must be given");
  if (n_tokens <= 0 || n_tokens > kMaxBatch) return fail(MOE_EINVAL, "n_tokens must be in 1..%d", kMaxBatch);
  if (c->routed[layer] || c->pending_rows || c->batch_layer >= 0)
    return fail(MOE_ESTATE, "layer %d: a routing step, an expert output or a routed batch is pending", layer);
  const float *z = logits_dev;
  if (x_dev) {
    HIP_TRY(launch_gate_gemm(x_dev, c->gate_w[layer], c->d_logits_batch, n_tokens, c->cfg.n_experts, c->cfg.hidden, c->compute));
    z = c->d_logits_batch;
  }
  const RouteParams p = make_route_params(c);
  HIP_TRY(launch_route_batch(p, z, n_tokens, c->d_state + layer, c->batch_rec_dev, c->compute));
  HIP_TRY(hipStreamSynchronize(c->compute));
  const moe_cache_config_t &g = c->cfg;
  for (int t = 0; t < n_tokens; ++t)
    for (int k = 0; k < g.top_k; ++k) {
      const moe_route_out_t &r = c->batch_rec[t];
      if (r.sel_expert[k] < 0 || r.sel_expert[k] >= g.n_experts || r.sel_slot[k] < 0 || r.sel_slot[k] >= g.capacity)
        return fail(MOE_EHIP, "batch routing returned expert %d slot %d out of range", r.sel_expert[k], r.sel_slot[k]);
    }
  if (out_host) memcpy(out_host, c->batch_rec, sizeof(moe_route_out_t) * n_tokens);
  c->batch_layer = layer;
  c->batch_n = n_tokens;
  return MOE_OK;
}

int moe_expert_forward_batch(moe_cache_t *c, int32_t layer, const void *x_dev, void *y_dev, int32_t n_tokens) {
  if (int rc = check_layer(c, layer)) return rc;
  if (!x_dev || !y_dev) return fail(MOE_EINVAL, "x_dev or y_dev is NULL");
  if (c->batch_layer != layer || c->batch_n != n_tokens)
    return fail(MOE_ESTATE, "layer %d: moe_expert_forward_batch without a preceding moe_route_batch of %d tokens", layer, n_tokens);
  const moe_cache_config_t &g = c->cfg;
  const int K = g.top_k, d = g.hidden;
  const size_t slot_bytes = (size_t)c->slot_layout.total;
  HIP_TRY(hipEventRecord(c->ev_batch, c->compute));  // whatever read the slots before this call is ahead of this point
  BatchParams bp{};
  bp.slot_pool = static_cast<const uint8_t *>(c->slot_pool[layer]);
  bp.shared_blob = g.shared_inter > 0 ? static_cast<const uint8_t *>(c->shared_blob[layer]) : nullptr;
  bp.x = static_cast<const uint16_t *>(x_dev);
  bp.partial = c->d_bpartial;
  bp.units = c->d_units;
  bp.tiles = c->d_tiles;
  bp.hidden = d;
  bp.inter = g.inter;
  bp.shared_inter = g.shared_inter;
  bp.slot_bytes = (int64_t)slot_bytes;
  // Segments: maximal runs of tokens during which no slot is refilled after a token of the run has read it, so that
  // all experts a segment needs are in their slots at once.  One expert launch per segment, behind its fills.
  int t0 = 0;
  bool first = true;
  while (t0 < n_tokens) {
    uint64_t read = 0;
    int t1 = t0;
    for (; t1 < n_tokens; ++t1) {
      const moe_route_out_t &r = c->batch_rec[t1];
      bool conflict = false;
      for (int k = 0; k < K; ++k) conflict |= r.miss[k] && ((read >> r.sel_slot[k]) & 1);
      if (conflict) break;
      for (int k = 0; k < K; ++k) read |= 1ull << r.sel_slot[k];
    }
    // fills of the segment's misses, once the compute stream has finished with the slots' previous contents
    int n_fill = 0;
    uint64_t filled = 0;  // slots that receive an expert in this segment
    for (int t = t0; t < t1; ++t) {
      const moe_route_out_t &r = c->batch_rec[t];
      for (int k = 0; k < K; ++k) {
        if (!r.miss[k]) continue;
        filled |= 1ull << r.sel_slot[k];
        if (n_fill++ == 0) HIP_TRY(hipStreamWaitEvent(c->copy, c->ev_batch, 0));
        if (c->poison_fills)
          HIP_TRY(hipMemsetAsync(static_cast<uint8_t *>(c->slot_pool[layer]) + (size_t)r.sel_slot[k] * slot_bytes, 0xff,
                                 slot_bytes, c->copy));
        HIP_TRY(hipMemcpyAsync(static_cast<uint8_t *>(c->slot_pool[layer]) + (size_t)r.sel_slot[k] * slot_bytes,
                               c->host_blob[(size_t)layer * g.n_experts + r.sel_expert[k]], slot_bytes,
                               hipMemcpyHostToDevice, c->copy));
        c->bytes_filled[layer] += (int64_t)slot_bytes;
      }
    }
    if (n_fill > 0) HIP_TRY(hipEventRecord(c->ev_copy[layer], c->copy));
    // token tiles per slot and for the shared expert, units per tile; the staging buffers are free again once the
    // previous segment's copies have been consumed
    if (!first) HIP_TRY(hipStreamSynchronize(c->compute));
    first = false;
    int n_tiles = 0, n_units = 0;
    const int n_seg = t1 - t0, mc = c->max_contrib;
    int32_t *n_contrib = c->h_contrib;                 // [kMaxBatch] counts, then the lists
    int32_t *contrib = c->h_contrib + kMaxBatch;       // [n_seg][mc]
    for (int i = 0; i < n_seg; ++i) n_contrib[i] = 0;
    // tiles first: per slot the tokens routed to it, sixteen to a tile; then the shared expert's
    std::vector<int32_t> &tile_slot = c->tile_slot;  // -1: the shared expert
    tile_slot.clear();
    auto new_tile = [&](int slot) -> TokenTile * {
      if (n_tiles >= c->max_tiles) return nullptr;
      TokenTile *tile = &c->h_tiles[n_tiles++];
      memset(tile, 0, sizeof *tile);
      tile_slot.push_back(slot);
      return tile;
    };
    for (int s = 0; s < g.capacity; ++s) {
      if (!((read >> s) & 1)) continue;
      TokenTile *tile = nullptr;
      for (int t = t0; t < t1; ++t) {
        const moe_route_out_t &r = c->batch_rec[t];
        for (int k = 0; k < K; ++k) {
          if (r.sel_slot[k] != s) continue;
          if (!tile || tile->n == 16) tile = new_tile(s);
          if (!tile) return fail(MOE_EHIP, "batch tables overflow (tiles)");
          tile->tok[tile->n] = t;
          tile->w[tile->n++] = r.sel_weight[k];
        }
      }
    }
    if (g.shared_inter > 0) {
      for (int t = t0; t < t1; t += 16) {
        TokenTile *tile = new_tile(-1);
        if (!tile) return fail(MOE_EHIP, "batch tables overflow (tiles)");
        for (int i = t; i < std::min(t + 16, t1); ++i) {
          tile->tok[tile->n] = i;
          tile->w[tile->n++] = 1.f;
        }
      }
    }
    // Records per unit.  A unit costs about 8 us of start-up plus 0.5 us per record, and the launch runs in rounds of
    // one workgroup per compute unit: take the size (a multiple of 16) with the smallest estimate rounds x unit time,
    // the larger one when two are equal (fewer partial tiles to add up).  A short batch thus spreads over all
    // compute units with small units, a long one avoids a last round that is nearly empty.
    int unit_rec = kBatchUnitRecords;
    {
      double best = 1e30;
      for (int cand = kBatchMinUnitRecords; cand <= kBatchMaxUnitRecords; cand += 16) {
        int total = 0;
        for (int i = 0; i < n_tiles; ++i) {
          const int rows = tile_slot[i] < 0 ? g.shared_inter : g.inter;
          total += (rows + cand - 1) / cand;
        }
        const int per_token = K * ((g.inter + cand - 1) / cand) + (g.shared_inter + cand - 1) / cand;
        if (total > c->max_units || per_token > mc) continue;  // (what the tables are sized for)
        const int rounds = (total + c->n_cus - 1) / c->n_cus;
        const double est = rounds * (8.0 + 0.5 * cand);
        if (est <= best) {
          best = est;
          unit_rec = cand;
        }
      }
    }
    c->units_built.clear();
    c->tile_first_unit.assign(n_tiles + 1, 0);
    for (int i = 0; i < n_tiles; ++i) {
      const int rows = tile_slot[i] < 0 ? g.shared_inter : g.inter;
      c->tile_first_unit[i] = n_units;
      for (int r0 = 0; r0 < rows; r0 += unit_rec, ++n_units)
        c->units_built.push_back(BatchUnit{tile_slot[i], r0, std::min(unit_rec, rows - r0), i});
    }
    c->tile_first_unit[n_tiles] = n_units;
    if (n_units > c->max_units) return fail(MOE_EHIP, "batch tables overflow (%d units)", n_units);
    // Launch order.  The units that read the same records (one blob, one block of records; one unit per token tile)
    // should share them in an L2: workgroups go to the XCDs round-robin by index, so such a group gets consecutive
    // places of one XCD (indices 8 apart), the groups spread over the XCDs by length.  Made tile by tile, the units
    // of a group would sit a tile's unit count apart - at C2 on eight different XCDs, each fetching the block from HBM.
    // Two groups: first the units whose experts were in their slots already (and the shared expert's), launched at
    // once; behind them the units of the slots being filled, launched behind the fill event - so the first group
    // computes while the fills stream.
    std::vector<int32_t> &pos = c->unit_pos;
    int n_ready = 0;
    {
      const int max_chunks = (std::max(g.inter, g.shared_inter) + unit_rec - 1) / unit_rec;
      pos.assign(n_units, -1);
      std::vector<int32_t> &owner = c->unit_group_owner;  // per (blob, block of records): the XCD of its group
      auto key = [&](const BatchUnit &bu) { return (bu.slot + 1) * max_chunks + bu.rec0 / unit_rec; };
      int placed = 0;
      for (int pass = 0; pass < 2; ++pass) {
        for (auto &q : c->xcd_queue) q.clear();
        owner.assign((size_t)(g.capacity + 1) * max_chunks, -1);
        for (int u = 0; u < n_units; ++u) {
          const BatchUnit &bu = c->units_built[u];
          const bool waits = bu.slot >= 0 && ((filled >> bu.slot) & 1);
          if (waits != (pass == 1)) continue;
          int32_t &x = owner[(size_t)key(bu)];
          if (x < 0) {  // a new group: to the XCD with the shortest queue
            x = 0;
            for (int i = 1; i < 8; ++i)
              if (c->xcd_queue[i].size() < c->xcd_queue[x].size()) x = i;
          }
          c->xcd_queue[x].push_back(u);
        }
        for (auto &q : c->xcd_queue)  // a group's units side by side in its queue
          std::stable_sort(q.begin(), q.end(), [&](int32_t ua, int32_t ub) { return key(c->units_built[ua]) < key(c->units_built[ub]); });
        size_t longest = 0;
        for (auto &q : c->xcd_queue) longest = std::max(longest, q.size());
        for (size_t i = 0; i < longest; ++i)
          for (int x = 0; x < 8; ++x)
            if (i < c->xcd_queue[x].size()) {
              const int32_t u = c->xcd_queue[x][i];
              pos[u] = placed;
              c->h_units[placed++] = c->units_built[u];
            }
        if (pass == 0) n_ready = placed;
      }
    }
    // per token: the rows of the partial buffer that hold its share of y (unit place * 16 + row in the tile), in a
    // fixed order: tiles in the order made, a tile's units by record
    for (int i = 0; i < n_tiles; ++i) {
      const TokenTile &tile = c->h_tiles[i];
      for (int row = 0; row < tile.n; ++row) {
        const int t = tile.tok[row];
        for (int u = c->tile_first_unit[i]; u < c->tile_first_unit[i + 1]; ++u) {
          int32_t &n = n_contrib[t - t0];
          if (n < mc) contrib[(size_t)(t - t0) * mc + n] = pos[u] * 16 + row;
          ++n;
        }
      }
    }
    for (int i = 0; i < n_seg; ++i)
      if (n_contrib[i] > mc) return fail(MOE_EHIP, "batch tables overflow (%d partial rows for one token)", n_contrib[i]);
    HIP_TRY(hipMemcpyAsync(c->d_tables, c->h_tables, c->off_contrib + sizeof(int32_t) * ((size_t)kMaxBatch + (size_t)n_seg * mc),
                           hipMemcpyHostToDevice, c->compute));
    bp.unit_base = 0;
    bp.n_units = n_ready;
    HIP_TRY(launch_expert_batch(bp, c->compute));
    if (n_fill > 0) HIP_TRY(hipStreamWaitEvent(c->compute, c->ev_copy[layer], 0));
    bp.unit_base = n_ready;
    bp.n_units = n_units - n_ready;
    HIP_TRY(launch_expert_batch(bp, c->compute));
    HIP_TRY(launch_reduce_batch(c->d_bpartial, c->d_contrib + kMaxBatch, c->d_contrib, mc, y_dev, d, t0, n_seg,
                                c->compute));
    HIP_TRY(hipEventRecord(c->ev_batch, c->compute));
    t0 = t1;
  }
  HIP_TRY(hipStreamSynchronize(c->compute));
  c->batch_layer = -1;
  c->batch_n = 0;
  return MOE_OK;
}

int moe_cache_last_route(moe_cache_t *c, int32_t layer, moe_route_out_t *out) {
  if (int rc = check_layer(c, layer)) return rc;
  if (!out) return fail(MOE_EINVAL, "out is NULL");
  if (c->routed[layer] >= 2) return fail(MOE_ESTATE, "layer %d: routing decision not collected yet", layer);
  return fetch_record(c, layer, out);
}

int moe_cache_stats(moe_cache_t *c, int32_t layer, moe_cache_stats_t *out) {
  if (!c || !out) return fail(MOE_EINVAL, "NULL argument");
  if (int rc = check_layer(c, layer == -1 ? 0 : layer)) return rc;  // also refuses a context whose hand-over was abandoned
  HIP_TRY(hipStreamSynchronize(c->compute));
  std::vector<LayerState> st(c->cfg.n_layers);
  HIP_TRY(hipMemcpy(st.data(), c->d_state, sizeof(LayerState) * st.size(), hipMemcpyDeviceToHost));
  memset(out, 0, sizeof *out);
  for (int l = 0; l < c->cfg.n_layers; ++l) {
    if (layer != -1 && l != layer) continue;
    out->tokens += st[l].count;
    out->selections += st[l].selections;
    out->hits += st[l].hits;
    out->misses += st[l].misses;
    out->cold_misses += st[l].cold_misses;
    out->evictions += st[l].evictions;
    out->lifetime_sum += st[l].lifetime_sum;
    out->bytes_filled += c->bytes_filled[l];
  }
  return MOE_OK;
}

int moe_cache_tables(moe_cache_t *c, int32_t layer, moe_cache_tables_t *out) {
  if (int rc = check_layer(c, layer)) return rc;
  if (!out) return fail(MOE_EINVAL, "out is NULL");
  HIP_TRY(hipStreamSynchronize(c->compute));
  LayerState st;
  HIP_TRY(hipMemcpy(&st, c->d_state + layer, sizeof st, hipMemcpyDeviceToHost));
  memcpy(out->expert_slot, st.expert_slot, sizeof out->expert_slot);
  memcpy(out->slot_expert, st.slot_expert, sizeof out->slot_expert);
  memcpy(out->stamp, st.stamp, sizeof out->stamp);
  out->delta_sum = st.delta_sum;
  out->count = st.count;
  return MOE_OK;
}

namespace {
struct SnapshotHeader {
  uint32_t magic, version;
  int32_t n_experts, capacity, top_k, reserved;
};
constexpr uint32_t kSnapMagic = 0x43454f4du, kSnapVersion = 1;  // "MOEC"
constexpr size_t kSnapBytes = sizeof(SnapshotHeader) + sizeof(LayerState);
}  // namespace

int moe_cache_snapshot(moe_cache_t *c, int32_t layer, void *buf, size_t *bytes) {
  if (int rc = check_layer(c, layer)) return rc;
  if (!bytes) return fail(MOE_EINVAL, "bytes is NULL");
  const size_t have = *bytes;
  *bytes = kSnapBytes;
  if (!buf) return MOE_OK;
  if (have < kSnapBytes) return fail(MOE_EINVAL, "snapshot needs %zu bytes, buffer has %zu", kSnapBytes, have);
  HIP_TRY(hipStreamSynchronize(c->compute));
  SnapshotHeader hd{kSnapMagic, kSnapVersion, c->cfg.n_experts, c->cfg.capacity, c->cfg.top_k, 0};
  memcpy(buf, &hd, sizeof hd);
  HIP_TRY(hipMemcpy(static_cast<uint8_t *>(buf) + sizeof hd, c->d_state + layer, sizeof(LayerState),
                    hipMemcpyDeviceToHost));
  return MOE_OK;
}

int moe_cache_restore(moe_cache_t *c, int32_t layer, const void *buf, size_t bytes) {
  if (int rc = check_layer(c, layer)) return rc;
  if (!buf || bytes < kSnapBytes) return fail(MOE_EINVAL, "snapshot buffer is NULL or shorter than %zu bytes", kSnapBytes);
  if (c->routed[layer] || c->pending_rows) return fail(MOE_ESTATE, "layer %d: a routing step or an expert output is pending", layer);
  const moe_cache_config_t &g = c->cfg;
  SnapshotHeader hd;
  memcpy(&hd, buf, sizeof hd);
  if (hd.magic != kSnapMagic || hd.version != kSnapVersion) return fail(MOE_EINVAL, "not a cache snapshot");
  if (hd.n_experts != g.n_experts || hd.capacity != g.capacity || hd.top_k != g.top_k)
    return fail(MOE_EINVAL, "snapshot is for n_experts=%d capacity=%d top_k=%d", hd.n_experts, hd.capacity, hd.top_k);
  LayerState st;
  memcpy(&st, static_cast<const uint8_t *>(buf) + sizeof hd, sizeof st);
  // the two tables must describe one partial bijection expert <-> slot inside the configured ranges
  for (int e = 0; e < MOE_MAX_EXPERTS; ++e) {
    const int s = st.expert_slot[e];
    const bool ok = e < g.n_experts ? (s == -1 || (s >= 0 && s < g.capacity && st.slot_expert[s] == e)) : s == -1;
    if (!ok) return fail(MOE_EINVAL, "snapshot tables inconsistent at expert %d", e);
  }
  for (int s = 0; s < MOE_MAX_EXPERTS; ++s) {
    const int e = st.slot_expert[s];
    const bool ok = s < g.capacity ? (e == -1 || (e >= 0 && e < g.n_experts && st.expert_slot[e] == s &&
                                                   ((st.ever_used >> s) & 1)))
                                   : e == -1;
    if (!ok) return fail(MOE_EINVAL, "snapshot tables inconsistent at slot %d", s);
  }
  if (st.count < 0 || st.selections < 0 || st.misses < 0) return fail(MOE_EINVAL, "snapshot counters negative");
  HIP_TRY(hipStreamSynchronize(c->compute));
  HIP_TRY(hipStreamSynchronize(c->copy));
  HIP_TRY(hipMemcpy(c->d_state + layer, &st, sizeof st, hipMemcpyHostToDevice));
  const size_t slot_bytes = (size_t)c->slot_layout.total;
  for (int s = 0; s < g.capacity; ++s) {
    const int e = st.slot_expert[s];
    if (e < 0) continue;
    HIP_TRY(hipMemcpy(static_cast<uint8_t *>(c->slot_pool[layer]) + (size_t)s * slot_bytes,
                      c->host_blob[(size_t)layer * g.n_experts + e], slot_bytes, hipMemcpyHostToDevice));
  }
  return MOE_OK;
}

int moe_cache_set_lambda(moe_cache_t *c, float lambda) {
  if (!c) return fail(MOE_EINVAL, "context is NULL");
  if (!(lambda >= 0.f) || !std::isfinite(lambda)) return fail(MOE_EINVAL, "lambda must be finite and >= 0");
  c->cfg.lambda = lambda;
  return MOE_OK;
}

int moe_cache_set_baseline(moe_cache_t *c, int32_t route_mode, int32_t max_rank, float cumsum_p) {
  if (!c) return fail(MOE_EINVAL, "context is NULL");
  if (route_mode < MOE_ROUTE_CACHE_PRIOR || route_mode > MOE_ROUTE_CUMSUM) return fail(MOE_EINVAL, "bad route_mode");
  if (route_mode == MOE_ROUTE_MAX_RANK && (max_rank < 0 || max_rank > c->cfg.n_experts))
    return fail(MOE_EINVAL, "max_rank must be in 0..n_experts");
  if (route_mode == MOE_ROUTE_CUMSUM && !(cumsum_p >= 0.f)) return fail(MOE_EINVAL, "cumsum_p must be >= 0");
  c->cfg.route_mode = route_mode;
  c->cfg.max_rank = max_rank;
  c->cfg.cumsum_p = cumsum_p;
  return MOE_OK;
}

int moe_cache_reset(moe_cache_t *c) {
  if (!c) return fail(MOE_EINVAL, "context is NULL");
  return do_reset(c);
}

int moe_residual_rmsnorm(float *h_dev, const void *y_dev, const float *a_dev, float perturb, int32_t carry,
                         void *x_dev, int32_t hidden, int32_t act_fmt, void *stream) {
  if (!h_dev || !x_dev) return fail(MOE_EINVAL, "h_dev or x_dev is NULL");
  if (hidden <= 0 || !valid_afmt(act_fmt)) return fail(MOE_EINVAL, "bad hidden or act_fmt");
  HIP_TRY(launch_residual_rmsnorm(h_dev, y_dev, a_dev, perturb, carry, x_dev, hidden, act_fmt,
                                  static_cast<hipStream_t>(stream)));
  return MOE_OK;
}

int moe_cache_plan(moe_cache_t *c, moe_cache_plan_t *out) {
  if (!c || !out) return fail(MOE_EINVAL, "NULL argument");
  out->grid = c->plan.grid;
  out->wavefronts = kGemvWaves;
  out->depth = kGemvDepth;
  out->packed_bf16_dot = c->plan.dot2;
  out->boundary_in_expert_launch = c->fuse_boundary && c->cfg.hidden % 64 == 0 && c->cfg.hidden <= kFusedMaxHidden &&
                                   gemv_fused_supported(c->cfg.weight_fmt, c->cfg.act_fmt, c->cfg.hidden, c->plan);
  return MOE_OK;
}

namespace {
constexpr size_t kProfEvents = 1u << 15;  // launches timed between two resets
}

int moe_cache_profile(moe_cache_t *c, int32_t enable, int32_t reset, double *avg_us, int64_t *launches) {
  if (!c) return fail(MOE_EINVAL, "context is NULL");
  HIP_TRY(hipStreamSynchronize(c->compute));
  double total_ms = 0.0;
  int64_t n_full = 0;
  for (size_t i = 0; i < c->prof_used; ++i) {
    if (!c->prof_full[i]) continue;  // a launch that left out missing experts moved fewer bytes
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, c->prof_events[i].first, c->prof_events[i].second));
    total_ms += ms;
    ++n_full;
  }
  if (avg_us) *avg_us = n_full ? total_ms * 1000.0 / (double)n_full : 0.0;
  if (launches) *launches = n_full;
  if (reset) c->prof_used = 0;
  c->profiling = enable > 0 ? enable : 0;
  c->prof_tick = 0;
  // the events are made here, not between the launches they time
  while (c->profiling && c->prof_events.size() < kProfEvents) {
    hipEvent_t a, b;
    HIP_TRY(hipEventCreate(&a));
    HIP_TRY(hipEventCreate(&b));
    c->prof_events.emplace_back(a, b);
    c->prof_full.push_back(0);
  }
  return MOE_OK;
}

}  // extern "C"
