/*
 * coe.h - C ABI of the MI355X (gfx950) library for dependency-routed batched expert inference,
 * the data-parallel hot path of CoServe-style Collaboration-of-Experts (CoE) serving.
 *
 * Model (paper, Section 2.1): a CoE model is a set of experts plus routing rules.  A request first
 * runs on a preliminary expert; that expert's output either selects the next expert or is the final
 * result.  Experts of one architecture differ only in their weights (Section 4.5, "profiled only
 * once"); every expert has a usage probability and a memory footprint (Section 4.5); the memory that
 * may hold experts on the device is capped (Sections 2.2, 4.3), and a request for an expert that is
 * not on the device forces an expert switch (Section 4.1, "Online").
 *
 * One context drives one GPU.  A context is not thread-safe.  All functions return 0 (COE_OK), a
 * positive informational code, or a negative error code; coe_last_error() then holds a message.
 * Nothing throws across this boundary.  Unless a parameter says "device", pointers are host pointers
 * owned by the caller, read or written during the call only, and may be freed when the call returns.
 * After COE_EDEVICE (a HIP call failed) the context must be destroyed; after any other error it
 * stays usable.
 */
#ifndef COE_H
#define COE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define COE_OK 0
#define COE_DONE 1      /* coe_step: no request is pending */
#define COE_EINVAL (-1) /* bad argument */
#define COE_ENOMEM (-2) /* host/device allocation failed, or an expert cannot fit the cache */
#define COE_ESTATE (-3) /* call order (e.g. submit before the graph is set) */
#define COE_EGRAPH (-4) /* dependency graph invalid: id out of range, cycle, more routes than classes */
#define COE_EDEVICE (-5)/* a HIP runtime call failed */
#define COE_ERANGE (-6) /* a caller buffer or a configured capacity is too small */
#define COE_EIO (-7)    /* the backing file of the host tier could not be created, written or read */

typedef struct coe_ctx coe_ctx;

/* ---- architecture descriptor: a flat layer list over numbered activation buffers ---------------------------
 * Buffer 0 is the request's input image [in_h][in_w][in_c] (NHWC).  Buffers 1..7 are scratch.
 * Activations are NHWC; a token tensor [T][D] is an image of height T, width 1, D channels.
 *   op COE_OP_CONV     dst = act(conv(src) + bias (+ res)); cross-correlation, zero padding, k filters r x s
 *   op COE_OP_MAXPOOL  dst = max over r x s windows of src (padding never wins), k = channels of src
 *   op COE_OP_HEAD     logits[k] = FC(global average pool of src); ends the program
 *   op COE_OP_TOKENS   dst = [class token; src tokens] + position embedding
 *   op COE_OP_LAYERNORM dst = layer norm of src over channels, eps 1e-6
 *   op COE_OP_ATTENTION src = [T][3D] (q|k|v), aux0 = heads; dst = softmax(q k^T / sqrt(D/heads)) v
 *   op COE_OP_HEAD_CLS logits[k] = FC(layer norm(token 0 of src)); ends the program
 *   op COE_OP_CONCAT   dst = [src | res] along channels (same height and width; k = channels of dst)
 *   op COE_OP_UPSAMPLE dst = src upsampled by two, nearest neighbour (k = channels)
 *   op COE_OP_HEAD_DET src (and res, if >= 0) are detection maps with aux0 anchors x (5 + k) channels per position (4 box
 *                      terms, objectness, k class logits): logits[c] = max over maps, positions and anchors of
 *                      sigmoid(objectness) * sigmoid(class c); k <= 251; no weights; ends the program
 * (the last three serve detector-shaped experts, the paper's object-detection experts downstream of its classifiers,
 * Section 5.1; bf16 only, channel counts multiples of 8)
 * act: 0 none, 1 ReLU, 2 GELU (erf form), 3 SiLU.  res = -1 for none; for a CONV, res must have dst's shape.
 * dtype: 0 = fp32 everywhere; 1 = bf16 weights and stored activations, fp32 accumulation, bias, residual add
 * and activation in fp32, one round-to-nearest-even to bf16 per stored activation, fp32 logits. */
enum { COE_OP_CONV = 1, COE_OP_MAXPOOL = 2, COE_OP_HEAD = 3, COE_OP_TOKENS = 4, COE_OP_LAYERNORM = 5,
       COE_OP_ATTENTION = 6, COE_OP_HEAD_CLS = 7, COE_OP_CONCAT = 8, COE_OP_UPSAMPLE = 9, COE_OP_HEAD_DET = 10 };
enum { COE_DT_F32 = 0, COE_DT_BF16 = 1 };

typedef struct {
    int32_t op, src, dst, res, k, r, s, stride, pad, act, aux0, aux1;
} coe_layer;

typedef struct {
    int32_t dtype, in_h, in_w, in_c, n_classes, n_layers;
    const coe_layer* layers; /* [n_layers] */
} coe_arch_desc;

/* Expert weights ("host_weights" of coe_register_expert) are one blob: the tensors of the layers in order,
 * each starting at the next multiple of 256 bytes.
 *   CONV      W[k][r][s][c] in the arch dtype, bias[k] fp32
 *   HEAD      W[k][c] in the arch dtype, bias[k] fp32
 *   TOKENS    cls[c], pos[T][c] in the arch dtype
 *   LAYERNORM gamma[c], beta[c] fp32
 *   HEAD_CLS  gamma[c], beta[c] fp32, W[k][c] arch dtype, bias[k] fp32
 * coe_arch_blob_bytes() returns the total (a multiple of 256). */

typedef struct {
    int32_t device;            /* HIP device ordinal */
    int32_t max_requests;      /* capacity of the request store (requests submitted and not yet collected) */
    int32_t max_batch;         /* request splitting (paper Section 4.2 "Request splitting"): largest batch one expert
                                * launch sequence handles (0 = 256).  Per architecture the library lowers it to what 31-bit
                                * byte offsets into the largest tensor of a launch allow, and cuts a group into the fewest
                                * sequences that fit, of equal size.  The activation workspace is sized for it. */
    int32_t max_stages;        /* longest path through the dependency graph that is recorded per request */
    int32_t cache_cap_experts; /* device expert cache: at most this many resident experts (0 = no limit) */
    int32_t profile;           /* k > 0: time every k-th launch of each kernel class with events (1 = all; see
                                * coe_profile_read); 0: no events */
    int64_t cache_cap_bytes;   /* and at most this many bytes of expert weights (0 = no limit).  The device memory behind the
                                * cache is one arena, allocated when the dependency graph is set: per distinct blob size as
                                * many slots as the caps let be resident at once (without caps: one per expert) */
    void* compute_stream;      /* borrowed hipStream_t for kernels, or NULL: the library creates one */
    void* copy_stream;         /* borrowed hipStream_t for expert switches, or NULL: the library creates one */
    int32_t group_small;       /* request arranging leaves many groups of a few requests: groups of at most this many
                                * requests whose experts share an architecture run as ONE launch per layer (0 = 64,
                                * negative = never).  Results do not depend on it. */
    int32_t eviction;          /* replacement rule of the expert cache: 0 = the two-stage rule of paper Section 4.3;
                                * 1 = least recently used, 2 = first in first out (the rules of the systems the paper
                                * compares with, Section 5.1; for measuring what the two-stage rule buys) */
    int32_t prefetch_depth;    /* expert switches are issued ahead of the groups that need them, so that the copy runs
                                * while earlier groups compute (paper Section 4.2: an expert can be loaded during the
                                * processing of a preceding request).  The experts of this many groups right before a
                                * missing one in the plan count as in use while its copy is in flight and are not
                                * evicted for it; 0 = only groups that have not run yet in the stage are protected, and
                                * consecutive misses then reuse one slot: each copy waits for the group before it. */
    int32_t executors;         /* executors (paper Section 4.1): launch sequences of different groups run on this many
                                * streams, each with its own activation workspace, so that small launches overlap on the
                                * device; 0 or 1 = one (the compute stream), at most 3.  Results do not depend on it. */
} coe_config;

typedef struct {
    int32_t n_pending;   /* requests queued for a stage when the step began (those of waiting groups included) */
    int32_t n_groups;    /* experts whose group ran in this step */
    int32_t n_chunks;    /* batches after splitting */
    int32_t n_hits;      /* groups whose expert was resident */
    int32_t n_misses;    /* groups that needed an expert switch */
    int32_t n_evictions; /* experts evicted */
    int64_t bytes_switched; /* host-to-device bytes of the switches */
    double host_plan_us; /* host time spent planning (cache policy, splitting) */
    int32_t n_grouped;   /* groups that shared their launches with other small groups */
    int32_t n_group_sets; /* launch sequences those groups were packed into */
    int32_t n_deferred_groups;   /* groups left queued by the arranging window (see coe_set_arranging) */
    int32_t n_deferred_requests; /* their requests; these are counted in n_pending but ran no stage in this step */
    int32_t n_executors_used;    /* executors that ran at least one launch sequence in this step */
    int32_t n_device_allocs;     /* device allocations made during this step: 0, because the expert arena (one slot class per
                                  * blob size), the request store and the activation workspaces are allocated when the
                                  * dependency graph is set (paper Section 5.5: expert management must stay a negligible
                                  * share of the time) */
    int32_t n_host_misses;       /* with a host tier (coe_set_host_tier): switches whose expert had to be read from the backing
                                  * file first */
    int64_t bytes_read;          /* bytes read from the backing file */
    double read_us;              /* host time spent in those reads */
} coe_step_stats;

/* Create / destroy a context.  coe_create fails with COE_EDEVICE when no GPU is usable. */
int coe_create(const coe_config* cfg, coe_ctx** out);
void coe_destroy(coe_ctx* ctx);
const char* coe_last_error(const coe_ctx* ctx); /* valid until the next call on ctx; "" if none.  ctx == NULL: the message of
                                                  * the calling thread's last failed call that takes no context */

/* Register an architecture shared by many experts (paper Section 4.5: experts of the same architecture are
 * profiled once).  All architectures of a context take the same input shape and dtype.  The descriptor is copied.
 * Errors: COE_EINVAL for a malformed layer list (bad buffer ids, shape mismatch of a residual, unknown op). */
int coe_register_arch(coe_ctx* ctx, const coe_arch_desc* desc, int32_t* arch_id);
/* Bytes of a weight blob of that architecture; negative error code on failure. */
int64_t coe_arch_blob_bytes(const coe_ctx* ctx, int32_t arch_id);

/* Register expert `expert_id` (ids must be dense, 0..E-1, any order).  host_weights is the canonical blob
 * (nbytes must equal coe_arch_blob_bytes); the library copies it into its own pinned host store, from which
 * expert switches are served.  usage_prob is the pre-assessed usage probability (paper Section 4.5) used for
 * the initial cache fill and for eviction. */
int coe_register_expert(coe_ctx* ctx, int32_t expert_id, int32_t arch_id, const void* host_weights, size_t nbytes,
                        float usage_prob);

/* Third storage tier (paper Section 1: experts are offloaded to CPU memory or SSD; Section 5.1: where CPU memory cannot
 * hold every expert either, it serves as a cache in front of the SSD).  Without this call every expert keeps a pinned host
 * copy.  With it, host memory holds at most host_cap_experts experts in pinned slots (a slot class per blob size, allocated
 * when the dependency graph is set) and every expert's blob lives in the file at backing_path, which the library creates,
 * truncates, fills at registration, and removes in coe_destroy.  A device switch whose expert has no host slot has the
 * blob read from the file into one first: the reads of a step are queued, in switch order, on a loader thread of the context
 * when the step is planned, and coe_step waits for one only when the next group cannot be launched without it.  The host tier is a cache of the same kind one level down: its requests
 * are the device tier's switches, one at a time in the order they are issued; replacement by the same rule as the device
 * tier (coe_config.eviction), applied to host residency; its initial fill is by descending usage probability (Section 4.1)
 * and precedes the device's.  Must be called before the first coe_register_expert.  coe_debug_forward then serves
 * device-resident experts only and coe_debug_layer_output is not available (COE_ESTATE).
 * Errors: COE_EINVAL (cap <= 0, null or overlong path), COE_ESTATE (experts already registered), COE_EIO (file). */
int coe_set_host_tier(coe_ctx* ctx, int32_t host_cap_experts, const char* backing_path);

/* Routing rules (paper Sections 2.1, 4.5 "Routing rules"): CSR successor lists.  Expert e routes on the argmax
 * over its first n_route = succ_off[e+1]-succ_off[e] logits (lowest index wins ties); the request goes to
 * succ[succ_off[e]+argmax], or is final when that entry is -1 or n_route is 0.  Every stage's expert consumes the
 * request's original input.  Must be called after all n_experts experts are registered.  Allocates every device buffer the
 * step path uses (expert arena, request store, activation workspaces): coe_submit and coe_step allocate nothing.
 * Errors: COE_EGRAPH (id out of range, cycle, n_route > classes of e), COE_ESTATE (experts missing), COE_ENOMEM. */
int coe_set_dependency_graph(coe_ctx* ctx, int32_t n_experts, const int32_t* succ_off, const int32_t* succ);

/* Append n requests.  inputs: [n][in_h][in_w][in_c] in the context dtype, a device pointer if on_device != 0,
 * else a host pointer; copied into the request store (stream-ordered; a device source must stay valid until
 * coe_sync or coe_collect, and the call returns without waiting; a host source has been read when the call returns).  first_expert: [n] host array of preliminary experts, or NULL = expert 0.
 * *first_request_id (nullable) receives the id of the first request; ids are consecutive.
 * Errors: COE_ERANGE when the store is full, COE_ESTATE before the graph is set. */
int coe_submit(coe_ctx* ctx, int32_t n, const void* inputs, int on_device, const int32_t* first_expert,
               int64_t* first_request_id);

/* Run ONE stage for every pending request: regroup by expert (paper Section 4.2 "Request arranging"), split
 * groups into batches ("Request splitting"), serve experts from the device cache (hits first; misses are
 * switched in on the copy stream while earlier groups compute; victims by two-stage eviction, Section 4.3),
 * run each expert on its batches, and route.  Work is enqueued asynchronously except for one small count
 * read-back.  Returns COE_DONE when nothing is pending.  stats is nullable. */
int coe_step(coe_ctx* ctx, coe_step_stats* stats);

/* Arranging window (paper Section 4.2, "Request arranging": a new request is placed behind the queued requests of
 * the same expert, so that they run together and the expert is loaded at most once for all of them).  coe_step
 * runs every queued group, so requests only meet the ones that arrived before the same step.  With a window, a group
 * of an expert of architecture arch_id that is still small stays queued instead: it is skipped in a step when it
 * holds fewer than min_group_resident requests (expert on the device) or min_group_missing requests (expert not on
 * the device: running it costs a switch), unless its oldest request has already waited max_wait_steps steps
 * (age = number of coe_step calls since the one that first saw the request; a request never waits longer).  Later
 * arrivals for the same expert join the queued group before it runs.  The thresholds are what the latency model of
 * Section 4.2 (K n + B per batch, plus the load time of a missing expert) says about when the fixed cost per request
 * has become small; a profiler computes them offline.  max_wait_steps = 0 (the default) switches the window off.
 * Results per request do not depend on any of this.  Errors: COE_EINVAL (unknown architecture, negative value). */
int coe_set_arranging(coe_ctx* ctx, int32_t arch_id, int32_t min_group_resident, int32_t min_group_missing,
                      int32_t max_wait_steps);

/* Latency model of an architecture (paper Section 4.2 "Prediction of additional inference latency"): a batch of n requests
 * of one expert takes k_ns * n + b_ns, a missing expert adds load_ns; measured offline (Section 4.5).  With several
 * executors, coe_step gives every launch sequence (a group, or a set of small groups sharing launches) to the executor
 * whose queue is predicted to finish first ("Request assigning": the assignment that minimises the longest queue; ties go
 * to the lowest-numbered executor); a group's sequences stay on one executor.  Defaults: k_ns = 1000, b_ns = load_ns = 0
 * (balance request counts).  Errors: COE_EINVAL (unknown architecture, negative value). */
int coe_set_latency_model(coe_ctx* ctx, int32_t arch_id, int64_t k_ns, int64_t b_ns, int64_t load_ns);

/* Wait for all enqueued work. */
int coe_sync(coe_ctx* ctx);

/* Copy out finished requests not yet collected, in request-id order, at most cap.  logits: [cap][max_classes]
 * fp32 of the last expert run (zero padded); path: [cap][max_stages] expert ids, -1 padded.  max_classes is the
 * largest n_classes over registered architectures.  Synchronises.  Any of the three output arrays may be NULL. */
int coe_collect(coe_ctx* ctx, int32_t cap, int64_t* request_id, float* logits, int32_t* path, int32_t* n_out);

/* Forget all requests (finished or not); experts, graph and cache contents stay. */
int coe_reset_requests(coe_ctx* ctx);

/* ---- inspection used by tests and the benchmark --------------------------------------------------------------- */
/* Result of the last step's regroup: cnt[E], off[E+1], perm[n_pending], inv[n_live] (-1 for non-pending).
 * perm/inv index request slots (request id minus the id of the oldest uncollected-store base).  Nullable outputs. */
int coe_debug_last_regroup(coe_ctx* ctx, int32_t* n_pending, int32_t* n_live, int32_t* cnt, int32_t* off,
                           int32_t* perm, int32_t* inv, int32_t perm_cap);
/* Switch log since creation: flat words {expert, n_victims, victims...} per switch, initial fill included.
 * Writes at most cap words; *n_words receives the total. */
int coe_debug_switch_log(coe_ctx* ctx, int32_t cap, int32_t* log, int32_t* n_words);
/* The same for the host tier (empty without one): {expert, n_victims, victims...} per read from the backing file. */
int coe_debug_host_log(coe_ctx* ctx, int32_t cap, int32_t* log, int32_t* n_words);
/* Which experts are resident: out[E] bytes (0/1). */
int coe_debug_resident(coe_ctx* ctx, uint8_t* out);
/* Run one expert on n inputs (device pointer, context dtype) without routing: logits_out [n][n_classes] fp32 (host). */
int coe_debug_forward(coe_ctx* ctx, int32_t expert_id, int32_t n, const void* device_inputs, float* logits_out);
/* Run the first `layer + 1` layers of an expert on n <= max_batch inputs (device pointer) and copy that layer's output
 * tensor [n][p][q][k] (context dtype) to `out` (host, out_bytes must match).  Heads and fused layers have none. */
int coe_debug_layer_output(coe_ctx* ctx, int32_t expert_id, int32_t n, const void* device_inputs, int32_t layer, void* out,
                           size_t out_bytes);
/* One convolution layer with the library's kernel selection, on host tensors (uploaded, run `repeat` times, read back):
 * x [n][h][w][c], w [k][r][s][c] (canonical order), bias [k] fp32, res [n][p][q][k] or NULL, y [n][p][q][k]; x, w, res,
 * y in `dtype`.  *kernel_class (nullable) receives the COE_K_* class that ran.  Timed under cfg.profile like any launch. */
int coe_debug_conv(coe_ctx* ctx, int32_t dtype, const void* x, const void* w, const float* bias, const void* res, void* y,
                   int32_t n, int32_t h, int32_t wd, int32_t c, int32_t k, int32_t r, int32_t s, int32_t stride,
                   int32_t pad, int32_t act, int32_t repeat, int32_t* kernel_class);
/* Stand-alone regroup on a host key vector (uploaded, regrouped on the device, read back): same outputs as above. */
int coe_debug_regroup(coe_ctx* ctx, int32_t n, const int32_t* cur, int32_t n_experts, int32_t* cnt, int32_t* off,
                      int32_t* perm, int32_t* inv);

/* Batches of the last step after request splitting (paper Section 4.2 "Request splitting"), in launch order: words
 * {expert, first row of the batch in the regrouped order, requests} per batch.  A group of n requests whose architecture takes
 * at most m per launch sequence is cut into ceil(n / m) batches of ceil(n / ceil(n / m)) requests, the last one holding the
 * rest.  Writes at most cap batches; *n_chunks receives the total. */
int coe_debug_last_chunks(coe_ctx* ctx, int32_t cap, int32_t* chunks, int32_t* n_chunks);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): the index part of request arranging, as coe_debug_regroup computes it, on DEVICE arrays and without a context.
 * cur [n] (expert id in [0, n_experts) = queued, anything else = not queued), cnt [n_experts], off [n_experts + 1],
 * perm [n], inv [n] are device pointers owned by the caller; the kernels are enqueued on `stream` (a hipStream_t, NULL = the
 * default stream) of the current device and the call returns without waiting.  The per-workgroup histograms, which the other
 * entry points keep in a buffer the context allocates, live in a static device array of COE_STATIC_SCRATCH_BYTES that every
 * GPU the library has run this call on holds until the process ends.  The call allocates nothing, frees nothing and
 * synchronises nothing.  All calls on one GPU share that array: calls that overlap there (two streams, two threads) race;
 * calls on one stream are ordered and need no clearing in between.
 * Errors: COE_ERANGE when ceil(n / 256) * n_experts * 4 exceeds COE_STATIC_SCRATCH_BYTES, COE_EINVAL (null pointer, n < 0,
 * n_experts outside 1..2048), COE_EDEVICE (a HIP call failed); coe_last_error(NULL) holds the message (per thread). */
#define COE_STATIC_SCRATCH_BYTES (4u << 20)
int coe_regroup_static(int32_t n, const int32_t* cur, int32_t n_experts, int32_t* cnt, int32_t* off, int32_t* perm,
                       int32_t* inv, void* stream);

/* Launch sequences of the last step in launch order: the first expert of each, its predicted cost and the executor it ran
 * on.  Writes at most cap entries (arrays nullable); *n_units receives the total. */
int coe_debug_last_assignment(coe_ctx* ctx, int32_t cap, int32_t* first_expert, int64_t* cost_ns, int32_t* executor,
                              int32_t* n_units);

/* Kernel classes timed when cfg.profile != 0. */
enum { COE_K_REGROUP_INDEX = 0, COE_K_REGROUP_GATHER = 1, COE_K_CONV_MFMA = 2, COE_K_CONV_DIRECT = 3, COE_K_POOL = 4,
       COE_K_HEAD = 5, COE_K_SWITCH = 6, COE_K_CONV_STEM = 7, COE_K_ATTENTION = 8, COE_K_TOKEN_OPS = 9, COE_K_CONV_SLAB = 10,
       COE_K_SWITCH_WAIT = 11, /* not a kernel: the time an executor's stream stood still waiting for an expert's copy to land
                                * (from the end of its previous work to the end of the copy); what is left of the switch time
                                * after the overlap with compute */
       COE_K_COUNT = 12 };
/* Synchronises, then returns and clears the accumulated TIMED launches, their milliseconds and algorithmic work of a class
 * (flops for the conv and attention classes, bytes for the others). */
int coe_profile_read(coe_ctx* ctx, int32_t kernel_class, int64_t* launches, double* ms, double* work);
/* Returns and clears the number of launches of a class since the last call, timed or not (cfg.profile != 0). */
int coe_profile_issued(coe_ctx* ctx, int32_t kernel_class, int64_t* issued);

/* ---- host-only pieces (no GPU needed) -------------------------------------------------------------------------- */
/* Graph check used by coe_set_dependency_graph.  n_classes: [n_experts] or NULL (skip the route-count check). */
int coe_validate_graph(int32_t n_experts, const int32_t* succ_off, const int32_t* succ, const int32_t* n_classes);

/* The arranging window's rule on its own: for every expert e with count[e] > 0 queued requests, age[e] steps waited by
 * the oldest of them, resident[e] != 0 when the expert is on the device, and its architecture's thresholds (arrays
 * indexed by expert), defer[e] = 1 when the group stays queued in this step, else 0.  Returns the number deferred. */
int coe_arrange_defer(int32_t n_experts, const int32_t* count, const int32_t* age, const uint8_t* resident,
                      const int32_t* min_group_resident, const int32_t* min_group_missing, const int32_t* max_wait_steps,
                      uint8_t* defer);

/* The assignment rule on its own: unit u (in order) goes to the executor with the least cost assigned so far, the
 * lowest-numbered among equals; executor[u] receives it. */
int coe_assign_executors(int32_t n_units, const int64_t* cost_ns, int32_t n_executors, int32_t* executor);

/* ---- offline profiler arithmetic (paper Section 4.5 "Expert performance metrics", Section 4.4 "Efficient Memory Management") ----
 * The profiler measures through the calls above (coe_debug_forward over batch sizes, switches with cfg.profile) and hands
 * the numbers to these host-only functions.
 * coe_profiler_fit_latency: least-squares line latency = K n + B through n >= 2 (batch size, latency) points (Section 4.2:
 * a batch of one expert scales linearly with the number of requests).  COE_EINVAL when all batch sizes are equal.
 * coe_profiler_max_batch: the maximum batch size of Section 4.5 (average latency per request stops falling): the smallest
 * measured batch whose latency per request is within `tol` (relative) of the best one measured.
 * coe_profiler_arranging_window: thresholds for coe_set_arranging from the model: a group of n requests spends the share
 * K n / (K n + B [+ load]) on its requests; the smallest n for which that share reaches `efficiency` (in [0, 1)) with the
 * expert on the device, and with the load of a missing expert added. */
int coe_profiler_fit_latency(int32_t n, const int32_t* batch, const double* latency_us, double* k_us, double* b_us);
int coe_profiler_max_batch(int32_t n, const int32_t* batch, const double* latency_us, double tol, int32_t* max_batch);
int coe_profiler_arranging_window(double k_us, double b_us, double load_us, double efficiency, int32_t* min_group_resident,
                                  int32_t* min_group_missing);

/* Memory scores (Section 4.5: an expert's memory footprint is normalised to its memory score; Section 4.3's eviction figure
 * and the user-configurable memory allocation are stated in them).  The unit is the smallest footprint among the experts, so
 * score[e] = nbytes[e] / unit >= 1; *unit_bytes receives it.  A memory allocation of s scores is cache_cap_bytes =
 * floor(s * unit).  COE_EINVAL for n <= 0, a null pointer or a footprint <= 0.
 * coe_profiler_expert_budget: memory allocation under limited computation performance (Section 4.4): inference runs at the
 * maximum batch size and everything else goes to experts: total_bytes - reserve_bytes - max_batch * bytes_per_request
 * (activation workspace of one request), never below 0.  *budget_scores (nullable) receives it in memory scores of
 * unit_bytes.  COE_EINVAL for negative sizes or unit_bytes <= 0. */
int coe_profiler_memory_scores(int32_t n, const int64_t* nbytes, double* score, int64_t* unit_bytes);
/* The current maximum executable batch size (Section 4.2 "Request splitting"): the smaller of the largest batch the
 * available memory holds (free_bytes / bytes_per_request, rounded down) and the maximum batch size the profiler measured;
 * at least 0.  This is the value for coe_config.max_batch.  COE_EINVAL for negative sizes or bytes_per_request <= 0. */
int coe_profiler_executable_batch(int64_t free_bytes, int64_t bytes_per_request, int32_t profiled_max_batch, int32_t* batch);
int coe_profiler_expert_budget(int64_t total_bytes, int64_t reserve_bytes, int64_t bytes_per_request, int32_t max_batch,
                               int64_t unit_bytes, int64_t* budget_bytes, double* budget_scores);

/* Expert usage probabilities from a sample run (Section 4.5 "Expert information": where the routing rules do not give the
 * probabilities in closed form, the CoE is run on a small sample and each expert's use is recorded).  path: [n_requests]
 * [max_stages] expert ids as coe_collect returns them (-1 padded); prob[e] = share of the sampled requests whose path
 * visits expert e.  COE_EINVAL for a null pointer, non-positive sizes or an id outside [-1, n_experts). */
int coe_profiler_usage_probabilities(int32_t n_requests, int32_t max_stages, const int32_t* path, int32_t n_experts, float* prob);

/* Decay-window search for the number of experts to keep on the device when their memory competes with the memory of large
 * batches (Section 4.4, "Memory allocation under sufficient computation performance").  The window slides along the number
 * of experts (sorted by descending usage probability): window k covers [sum of the earlier sizes, + size_k) with
 * size_k = initial_window * decay^k and decay = 1 - initial_window / 100 (Eq. 1).  For every window the caller loads as many
 * experts as the window's upper bound (rounded up, at most n_experts_total), runs sample requests and appends the measured
 * throughput.  Once `fit_points` (>= 2) earlier values exist, a least-squares line through the earlier values over their
 * index (Eq. 2) predicts the newest one; the search stops at the first window whose value falls short of the prediction by
 * more than error_margin, relative (Eq. 3), or when a window has loaded every expert.  The number of experts to keep is
 * then any value in [n_low, n_high] of the final window.  The function is stateless: call it with the throughputs measured
 * so far (n_measured = 0 first); status says whether to measure again (at n_next experts) or which way the search ended. */
enum { COE_WINDOW_MEASURE = 0, COE_WINDOW_SHORTFALL = 1, COE_WINDOW_END = 2 };
typedef struct {
    int32_t status;        /* COE_WINDOW_* */
    int32_t n_next;        /* COE_WINDOW_MEASURE: experts to load for the next measurement */
    double window_low;     /* bounds, on the expert axis, of the window measured last (of the first window when n_measured = 0) */
    double window_high;
    int32_t n_low, n_high; /* the same as whole experts (rounded up, clipped to 1..n_experts_total) */
    double linear_error;   /* Eq. 3's left side for the newest value (0 while fewer than fit_points earlier values exist) */
} coe_window_state;
int coe_profiler_window_step(int32_t n_experts_total, double initial_window, double error_margin, int32_t fit_points,
                             int32_t n_measured, const double* throughput, coe_window_state* out);

/* The expert-cache policy on its own (paper Section 4.1 initial fill, Section 4.3 two-stage eviction).
 * coe_policy_stage: has_group[E] marks experts with pending requests; order[E] receives the execution order
 * (resident first, then missing, each by ascending id), *n_order its length; log receives {expert, n_victims,
 * victims...} per switch, at most log_cap words; returns the number of words, or COE_ENOMEM / COE_ERANGE. */
typedef struct coe_policy coe_policy;
coe_policy* coe_policy_create(int32_t n_experts, const int64_t* nbytes, const float* usage_prob,
                              const int32_t* succ_off, const int32_t* succ, int32_t cap_experts, int64_t cap_bytes);
void coe_policy_destroy(coe_policy* p);
int coe_policy_init_fill(coe_policy* p, int32_t* loaded /*[E]*/);
int coe_policy_stage(coe_policy* p, const uint8_t* has_group, int32_t* order, int32_t* n_order, int32_t* log,
                     int32_t log_cap);
int coe_policy_resident(const coe_policy* p, uint8_t* out /*[E]*/);
/* Replacement rule as in coe_config.eviction; COE_EINVAL for an unknown kind.  Call before the first stage. */
int coe_policy_set_eviction(coe_policy* p, int32_t kind);
/* As coe_config.prefetch_depth; COE_EINVAL for a negative depth. */
int coe_policy_set_in_use_depth(coe_policy* p, int32_t depth);

#ifdef __cplusplus
}
#endif
#endif /* COE_H */
