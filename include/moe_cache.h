/*
 * moe_cache.h - C ABI of the batch-1 MoE decode path with cache-conditional routing.
 *
 * One MoE layer step for one token is
 *   z = W_gate x, w = softmax(z)                                  (paper Eq. 3)
 *   z' = z + lambda * Delta_avg * m~_t, select top-K of z'          (Sec. 3.3, Eq. 9, Eq. 10)
 *   hits/misses against the cache as it stood before the token     (Sec. 2.2, Eq. 4)
 *   LRU update of the expert cache                                 (Sec. 4.2)
 *   y = sum_k w_k E_k(x) (+ shared expert), E = SwiGLU             (Eq. 1)
 * The paper's DRAM tier is a pool of `capacity` expert slots per layer in device memory,
 * its Flash tier is pinned host memory holding every expert; a miss is filled by an
 * asynchronous host-to-device copy on `copy_stream`.
 *
 * Conventions
 *  - Every function returns MOE_OK or a negative moe_status; nothing throws or aborts.
 *    moe_last_error() gives a message for the calling thread's last failure.
 *  - "device" pointers are HIP device memory, "host" pointers ordinary host memory, "pinned"
 *    is page-locked host memory.  All buffers handed in are BORROWED: the caller allocates them,
 *    keeps them alive until moe_cache_destroy and frees them afterwards.  The library allocates
 *    only its own small tables (state, route records, partial sums).
 *  - Streams are hipStream_t passed as void*; both are borrowed.  Calls on one context must come
 *    from one thread at a time.
 *  - Expert ids are 0..n_experts-1, slots 0..capacity-1.  n_experts <= 64, top_k <= 8.
 *  - Environment variables read by moe_cache_init (all optional):
 *      MOE_HOST_SYNC=event     the host waits for a routing decision on a stream event instead of polling the
 *                              words the router stores into mapped host memory
 *      MOE_FUSE_BOUNDARY=0|1   overrides the rule that decides whether a non-blocking moe_stack_route_step runs
 *                              inside the layer's expert launch (see moe_cache_plan)
 *      MOE_POISON_FILLS=1      debugging aid: a slot is overwritten with 0xff bytes (NaNs in every format's
 *                              scales or weights) on the copy stream right before its fill, so that anything
 *                              computed from a slot before its fill has landed shows up as NaN in the output
 *      MOE_TAG_SPINS=n         polls before a workgroup stops waiting for the first workgroup of its own launch
 *                              (a test lowers it to reach the error path described at moe_stack_route_step)
 */
#ifndef MOE_CACHE_H
#define MOE_CACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_MAX_EXPERTS 64
#define MOE_MAX_TOPK 8

typedef struct moe_cache moe_cache_t; /* opaque, owned by the library */

enum moe_status { MOE_OK = 0, MOE_EINVAL = -1, MOE_ENOMEM = -2, MOE_EHIP = -3, MOE_ESTATE = -4 };
enum moe_weight_fmt { MOE_W_FP32 = 0, MOE_W_BF16 = 1, MOE_W_INT8_PC = 2, MOE_W_INT4_G128 = 3 };
enum moe_act_fmt { MOE_A_FP32 = 0, MOE_A_BF16 = 1 };
/* The logit range Delta that scales the prior (Eq. 9-10; App. D on the choice of the estimate): the running mean
 * over the tokens seen since the last reset (the paper's method), a fixed value given by the caller (e.g. from a
 * calibration set), or the current token's own range max z - min z. */
enum moe_delta_mode { MOE_DELTA_RUNNING_MEAN = 0, MOE_DELTA_FIXED = 1, MOE_DELTA_TOKEN = 2 };
/* How the ranking vector is altered before the top-K cut.  CACHE_PRIOR is the paper's method
 * (Sec. 3.3); MAX_RANK (Sec. 3.1, Eq. 6-7) and CUMSUM (Sec. 3.2, Eq. 8) are its two baselines. */
enum moe_route_mode { MOE_ROUTE_CACHE_PRIOR = 0, MOE_ROUTE_MAX_RANK = 1, MOE_ROUTE_CUMSUM = 2 };

typedef struct moe_cache_config {
  int32_t n_layers;
  int32_t hidden;       /* d; a multiple of 64 * (16 / bytes per weight) */
  int32_t n_experts;    /* N <= 64 */
  int32_t inter;        /* I, SwiGLU intermediate of a routed expert */
  int32_t shared_inter; /* intermediate of the always-on shared expert, 0 = none */
  int32_t top_k;        /* K <= 8 */
  int32_t top_j;        /* router's own top-J always selected (Sec. 3.3), 0..top_k */
  int32_t capacity;     /* expert slots per layer, top_k <= capacity <= n_experts */
  int32_t weight_fmt;   /* moe_weight_fmt of expert blobs */
  int32_t act_fmt;      /* moe_act_fmt of x, y and the router matrix */
  int32_t renormalize;  /* 1: divide the K weights by their sum (Sec. 2.1) */
  int32_t delta_mode;   /* moe_delta_mode */
  int32_t route_mode;   /* moe_route_mode */
  int32_t max_rank;     /* M of Eq. 6 (MOE_ROUTE_MAX_RANK) */
  float lambda;         /* >= 0, strength of the cache prior (Eq. 9) */
  float delta_fixed;    /* Delta_avg when delta_mode == MOE_DELTA_FIXED */
  float cumsum_p;       /* p of Eq. 8 (MOE_ROUTE_CUMSUM) */
  int32_t reserved;
  void *compute_stream; /* hipStream_t for kernels */
  void *copy_stream;    /* hipStream_t for miss fills; must differ from compute_stream */
} moe_cache_config_t;

typedef struct moe_cache_buffers {
  const void *const *host_expert_blob; /* [n_layers*n_experts] pinned host, packed blobs (moe_pack_expert) */
  void *const *slot_pool;              /* [n_layers] device, capacity*moe_slot_bytes(cfg) each, 256-byte aligned */
  const void *const *gate_w;           /* [n_layers] device, router matrix [N,d] row-major, act_fmt */
  const void *const *shared_blob;      /* [n_layers] device packed blob of the shared expert, or NULL */
  const int32_t *initial_resident;     /* host [n_layers*n_initial] experts preloaded into slots 0.., or NULL */
  int32_t n_initial;                   /* 0..capacity (App. G: empty or random initial cache) */
} moe_cache_buffers_t;

/* What one routing step decided; entries 0..top_k-1 are valid, ranked by the altered logits. */
typedef struct moe_route_out {
  int32_t sel_expert[MOE_MAX_TOPK];
  int32_t sel_slot[MOE_MAX_TOPK];   /* slot each selected expert occupies after the step */
  float sel_weight[MOE_MAX_TOPK];   /* softmax of the UNMODIFIED logits (Sec. 3.3), renormalised if asked */
  int32_t miss[MOE_MAX_TOPK];       /* 1 if the expert was not resident before the step (Eq. 4) */
  int32_t evicted[MOE_MAX_TOPK];    /* expert that lost its slot to this one, or -1 */
  int32_t n_miss;
  int32_t token;                    /* index of this step within the layer, from 0 */
  float delta;                      /* Delta_avg used (Eq. 10) */
  float margin;                     /* gap between the K-th and (K+1)-th altered logit */
  float logits[MOE_MAX_EXPERTS];    /* z, as used */
  uint32_t opaque[4];               /* the library's own compact copy of the decision (read by its expert kernels);
                                     * not part of the interface: do not interpret, do not rely on */
} moe_route_out_t;

typedef struct moe_cache_stats {
  int64_t tokens, selections, hits, misses, cold_misses, evictions, bytes_filled;
  int64_t lifetime_sum; /* over the evictions: tokens between an expert's load and its eviction; divided by
                         * `evictions` it is the average cache lifetime of Sec. 4.6 / Table 2 */
} moe_cache_stats_t;

/* Per-layer tables, for checking against a reference (host struct). */
typedef struct moe_cache_tables {
  int32_t expert_slot[MOE_MAX_EXPERTS]; /* expert -> slot or -1 */
  int32_t slot_expert[MOE_MAX_EXPERTS]; /* slot -> expert or -1 */
  int64_t stamp[MOE_MAX_EXPERTS];       /* recency stamp of resident experts: token*K + position */
  float delta_sum;                      /* running sum of max(z)-min(z) (Eq. 10) */
  int32_t count;                        /* tokens seen */
} moe_cache_tables_t;

/* Bytes of one packed expert with intermediate size `inter` (0 on invalid arguments).  A slot and a
 * host blob are moe_blob_bytes(fmt, hidden, cfg.inter); the shared blob uses cfg.shared_inter. */
size_t moe_blob_bytes(int32_t weight_fmt, int32_t hidden, int32_t inter);
/* Bytes of one expert slot of the fast tier for this configuration (Sec. 2.2: the cache holds whole experts), so
 * that the caller can size slot_pool (capacity * moe_slot_bytes per layer) and the host blobs.  Only weight_fmt,
 * hidden and inter are read.  0 on NULL or an unsupported shape. */
size_t moe_slot_bytes(const moe_cache_config_t *cfg);

/* Pack one expert from canonical row-major weights into the blob layout the kernels stream
 * (record i = gate row i | up row i | column i of down).  All pointers are device memory:
 *  fp32/bf16: gate,up [I,d], down [d,I] of that type; scale pointers NULL.
 *  int8: int8 values as above, fp16 scales gate_s,up_s [I], down_s [d] (one per output row).
 *  int4: bytes [I,d/2], [I,d/2], [d,I/2] (nibble = q+8, even column low), fp16 scales
 *        [I,d/128], [I,d/128], [d,I/128] (Sec. 4.5 names 4- and 8-bit weights; the format is ours).
 * Runs asynchronously on `stream`.  MOE_EINVAL on bad shapes/NULLs, MOE_EHIP on launch failure. */
int moe_pack_expert(int32_t weight_fmt, int32_t hidden, int32_t inter, const void *gate, const void *up,
                    const void *down, const void *gate_s, const void *up_s, const void *down_s, void *blob_dev,
                    void *stream);

/* Create a context (problem statement of Sec. 2.1-2.2 and 3.3).  Validates everything before touching
 * the GPU (MOE_EINVAL), preloads initial residents synchronously, leaves the cache otherwise empty. */
int moe_cache_init(const moe_cache_config_t *cfg, const moe_cache_buffers_t *bufs, moe_cache_t **out);
void moe_cache_destroy(moe_cache_t *ctx);

/* Routing step of one layer for one token (Eq. 3, Eq. 9-10, Eq. 4, Sec. 4.2): exactly one of x_dev
 * (device [d], act_fmt: the router GEMV is computed) and logits_dev (device [N] fp32: used as z) is
 * non-NULL; the buffer must stay unchanged until the layer's moe_expert_forward has been called.
 * With out_host non-NULL the call returns once the decision is known on the host (written to *out_host)
 * and the copies filling missed experts' slots are enqueued on copy_stream.  With out_host NULL the call
 * only enqueues the router kernel; the decision is collected, and the fills enqueued, inside
 * moe_expert_forward.  MOE_ESTATE if the layer's previous step has not been followed by moe_expert_forward. */
int moe_route_step(moe_cache_t *ctx, int32_t layer, const void *x_dev, const float *logits_dev,
                   moe_route_out_t *out_host);

/* Eq. 1 for the layer's last routing step: y = sum_k w_k E_k(x) + shared(x); x_dev (the vector given to
 * moe_route_step), y_dev device [d] in act_fmt.  The kernels are asynchronous on compute_stream: a first
 * launch covers the shared expert and the experts that were resident, a second one (after the fills) the
 * experts that were missing.  The call returns once the routing decision has reached the host (it is needed
 * to enqueue the fills), not when y is ready.  MOE_ESTATE without a preceding moe_route_step.
 * y_dev may be NULL: the output then stays inside the library as fp32 partial sums and is finished by the next
 * moe_stack_route_step (of any layer), which must follow before another moe_expert_forward. */
int moe_expert_forward(moe_cache_t *ctx, int32_t layer, const void *x_dev, void *y_dev);

/* Prompt phase: n_tokens (1..128) tokens of one layer in one call.  The paper applies its routing during generation and
 * leaves prompt processing to batched kernels (Sec. 4.5; App. F varies the prompt length); here a batch is routed as
 * its tokens one after the other - the cache bitmask m_t of Sec. 3.3 is the state after token t-1, also inside a batch -
 * so decisions, slots, evictions, Delta_avg (Eq. 10) and the miss counts of Eq. 4 are exactly those of n_tokens calls of
 * moe_route_step in the same order; only the arithmetic is batched (matrix cores).
 * moe_route_batch: exactly one of x_dev (device [n_tokens, d], act_fmt: the gate logits are computed) and logits_dev
 *   (device [n_tokens, N] fp32) is non-NULL.  Returns once all decisions are on the host; out_host (may be NULL)
 *   receives n_tokens records.  x_dev must stay unchanged until moe_expert_forward_batch.
 * moe_expert_forward_batch: y[t] = sum_k w_k E_k(x[t]) + shared(x[t]) (Eq. 1) for every token of the batch routed
 *   last; x_dev as given to moe_route_batch, y_dev device [n_tokens, d] in act_fmt.  Tokens are grouped per expert;
 *   where a slot is refilled inside the batch after an earlier token has read it, the batch is cut there and the
 *   parts run one after the other; within a part the experts that are resident (and the shared expert) are computed
 *   while the part's fills stream, the filled ones behind them.  The partial results are added in a fixed order (y
 *   is reproducible bit for bit).  Returns when y is complete.
 * Shapes: bf16 weights and activations, hidden 1024 or 2048, intermediate sizes that are multiples of 16;
 * MOE_EINVAL otherwise.  MOE_ESTATE if a single-token step of the layer or an expert output is pending, or if
 * moe_expert_forward_batch does not follow a moe_route_batch of the same layer and size. */
int moe_route_batch(moe_cache_t *ctx, int32_t layer, const void *x_dev, const float *logits_dev, int32_t n_tokens,
                    moe_route_out_t *out_host);
int moe_expert_forward_batch(moe_cache_t *ctx, int32_t layer, const void *x_dev, void *y_dev, int32_t n_tokens);

/* moe_expert_forward for callers that cannot allocate device memory or hold a context: code under HIP graph capture,
 * tight serving loops, harnesses that forbid allocation.  Computes y = sum_k w_k E_k(x) + shared(x) for experts that are
 * all in their slots, with the kernels moe_expert_forward uses.  The call allocates nothing (no hipMalloc / hipFree, no
 * memset): the routing record its kernels read and their fp32 partial rows live in a fixed 4 MiB + 512 B device array
 * inside the library, one per GPU, held until the process ends.  Hence the limits: hidden <= 4096, at most 256
 * workgroups; larger shapes are refused with MOE_EINVAL.  Every call on a GPU shares that GPU's array: calls that
 * overlap in time on one GPU (different streams, different threads) race; calls on one stream are ordered.
 *   slot_pool_dev   device, n_slots slots of moe_blob_bytes(weight_fmt, hidden, inter) each, 256-byte aligned
 *   shared_blob_dev device packed shared expert (shared_inter > 0) or NULL
 *   sel_slot_host, sel_weight_host   HOST arrays [top_k]: the slot of each selected expert and its weight (read
 *                   before the call returns; slots are checked against n_slots)
 *   x_dev, y_dev    device [hidden] in act_fmt; y is complete when `stream` reaches the end of the three kernels
 *                   this call enqueues.  The device of `stream` must be current. */
int moe_expert_forward_static(int32_t weight_fmt, int32_t act_fmt, int32_t hidden, int32_t inter, int32_t shared_inter,
                              int32_t top_k, const void *slot_pool_dev, int32_t n_slots, const void *shared_blob_dev,
                              const int32_t *sel_slot_host, const float *sel_weight_host, const void *x_dev,
                              void *y_dev, void *stream);

/* Layer boundary of a multi-layer stack (workload glue fused with the router kernel: Eq. 3, 9, 10, 4, Sec. 4.2):
 *   y  = the expert output left pending by moe_expert_forward(..., y_dev = NULL), if any
 *   h  = carry ? h + y + perturb * a : perturb * a  (a may be NULL; carry = 0 starts a new token)
 *   x  = h / sqrt(mean(h^2) + 1e-6), rounded to act_fmt, written to x_dev
 *   then the routing step of `layer` on x, exactly as moe_route_step(ctx, layer, x_dev, NULL, out_host).
 * h_dev: device fp32 [d] in/out; a_dev: device fp32 [d] or NULL; x_dev: device act_fmt [d] (pass it to the
 * layer's moe_expert_forward); y_dev: device act_fmt [d] or NULL, receives the finished pending output.
 * hidden must be at most 8192.  Same blocking rule and errors as moe_route_step.
 * With out_host NULL the library may defer x and the routing into the layer's expert launch (its first workgroup
 * does them while the others already stream the shared expert; see moe_cache_plan): x_dev and the routing record
 * are then written by the kernels moe_expert_forward enqueues, not by this call's, so nothing but
 * moe_expert_forward(ctx, layer, x_dev, ...) may use x_dev in between, and that call must be given the same x_dev.
 * The other workgroups' wait for the first one is bounded; should it ever run out, they finish without the routed
 * experts, and every later call that names a layer returns MOE_EHIP until moe_cache_reset. */
int moe_stack_route_step(moe_cache_t *ctx, int32_t layer, float *h_dev, const float *a_dev, float perturb,
                         int32_t carry, void *x_dev, void *y_dev, moe_route_out_t *out_host);

/* The last routing decision of a layer that has reached the host (after a blocking moe_route_step, or after
 * the moe_expert_forward that followed a non-blocking one).  MOE_ESTATE if a decision is still pending. */
int moe_cache_last_route(moe_cache_t *ctx, int32_t layer, moe_route_out_t *out_host);

/* Counters of one layer, or summed over layers with layer = -1 (Eq. 4 numerators/denominators).
 * Synchronises compute_stream.  MOE_EHIP after an abandoned hand-over (see moe_stack_route_step), like every
 * other call on a context in that state. */
int moe_cache_stats(moe_cache_t *ctx, int32_t layer, moe_cache_stats_t *out_host);
/* Slot table, stamps and Delta accumulator of one layer.  Synchronises compute_stream. */
int moe_cache_tables(moe_cache_t *ctx, int32_t layer, moe_cache_tables_t *out_host);
/* Save / restore the cache state of one layer (slot tables, stamps, Delta_avg accumulator of Eq. 10, counters of
 * Eq. 4) as an opaque host blob, e.g. to resume a decode or to start a comparison from a recorded state.
 * moe_cache_snapshot: *bytes holds the size of buf_host on entry and the size of the blob on return; with
 * buf_host NULL only the size is returned.  MOE_EINVAL if the buffer is too small.  Synchronises compute_stream.
 * moe_cache_restore: checks that the blob was taken from a context of the same n_experts / capacity / top_k and
 * that its tables are consistent (MOE_EINVAL otherwise, nothing changed), then installs it and copies every
 * resident expert's blob from the host tier into its slot, synchronously.  MOE_ESTATE while a routing step of
 * the layer or an expert output is pending. */
int moe_cache_snapshot(moe_cache_t *ctx, int32_t layer, void *buf_host, size_t *bytes);
int moe_cache_restore(moe_cache_t *ctx, int32_t layer, const void *buf_host, size_t bytes);
/* Change the strength lambda of the cache prior (Eq. 9: z' = z + lambda * Delta_avg * m~_t; Sec. 3.3 sweeps it as
 * the knob between the original routing, lambda = 0, and fully cache-driven routing) from the next routing step on.
 * Finite and >= 0, else MOE_EINVAL.  Does not touch the cache or Delta_avg. */
int moe_cache_set_lambda(moe_cache_t *ctx, float lambda);
/* Switch between the paper's method and its two list-based baselines (Sec. 3.1-3.2) and set M of Eq. 6 / p of Eq. 8. */
int moe_cache_set_baseline(moe_cache_t *ctx, int32_t route_mode, int32_t max_rank, float cumsum_p);
/* Start a new evaluation: empty every layer's cache (then preload the initial residents again, App. G), restart
 * the running mean Delta_avg of Eq. 10 (sum and token count to zero) and the hit/miss counters of Eq. 4; drops
 * pending steps and outputs and clears the error state described at moe_stack_route_step.  Synchronises both
 * streams. */
int moe_cache_reset(moe_cache_t *ctx);

/* Workload glue for multi-layer synthetic stacks (not part of the paper's method):
 * h = (carry ? h : 0) + y + perturb * a (y, a may be NULL); x = h / sqrt(mean(h^2) + 1e-6) rounded to act_fmt.
 * h: device fp32 [d] in/out; y: device act_fmt [d] or NULL; a: device fp32 [d] or NULL; x: device act_fmt [d].
 * carry = 0 starts a new token (h is overwritten). */
int moe_residual_rmsnorm(float *h_dev, const void *y_dev, const float *a_dev, float perturb, int32_t carry,
                         void *x_dev, int32_t hidden, int32_t act_fmt, void *stream);

/* Offline analysis of a recorded selection trace; host memory only, no GPU work, no context.
 * trace[t*top_k + k]: the experts one layer selected at token t (distinct, each in 0..n_experts-1), in the order
 * the cache touches them (descending router weight, Sec. 4.2).  Misses are counted per token against the cache
 * before the token (Eq. 4), starting from `initial` (n_initial experts, may be NULL/0).
 *   MOE_POLICY_LRU       least-recently-used eviction as in Sec. 4.2; any capacity in 1..n_experts (below top_k
 *                        only the most recently touched experts of a token stay: the cache-size sweep of Sec. 4.8)
 *   MOE_POLICY_FARTHEST  evict the resident expert, not needed by the current token, whose next use is farthest
 *                        (never again first, ties to the lowest id): the optimal-eviction bound of Sec. 4.8;
 *                        needs capacity >= top_k
 * Outputs: *misses; optionally (may be NULL) *lifetime_sum and *evictions as in moe_cache_stats_t.
 * MOE_EINVAL on NULL/out-of-range arguments or a token with repeated experts. */
enum { MOE_POLICY_LRU = 0, MOE_POLICY_FARTHEST = 1 };
int moe_trace_misses(const int32_t *trace, int64_t n_tokens, int32_t top_k, int32_t n_experts, int32_t capacity,
                     int32_t policy, const int32_t *initial, int32_t n_initial, int64_t *misses,
                     int64_t *lifetime_sum, int64_t *evictions);

/* The launch shape the context chose for the expert kernels, and whether a moe_stack_route_step without out_host
 * runs its routing inside the layer's expert launch (bf16 activations, a supported shape, and a shared expert of at
 * least a third of the layer's records; MOE_FUSE_BOUNDARY=0 or 1 in the environment at moe_cache_init overrides
 * the last condition). */
typedef struct moe_cache_plan {
  int32_t grid, wavefronts, depth, packed_bf16_dot, boundary_in_expert_launch;
} moe_cache_plan_t;
int moe_cache_plan(moe_cache_t *ctx, moe_cache_plan_t *out_host);

/* Average duration in microseconds of the timed expert-GEMV launches that covered a whole layer (no expert missing)
 * since the last call with reset != 0, and their count; measured with start/stop events attached to the launches
 * on compute_stream.  enable = 0 switches the timing off, enable = n > 0 times every n-th first-pass launch from
 * this call on (1 = all of them; events on every launch slow the host down to where the device idles between
 * launches, a stride co-prime to the layer count samples every layer without that); at most 32768 launches are
 * timed between two resets, later ones run untimed.  Each timed launch is preceded by a 50 us hold of the stream,
 * so that the kernel is already queued behind its start marker when the device reaches the marker. */
int moe_cache_profile(moe_cache_t *ctx, int32_t enable, int32_t reset, double *avg_us, int64_t *launches);

const char *moe_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MOE_CACHE_H */
