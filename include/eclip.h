/*
 * libeclip -- co-located DNN inference on a pre-allocated pool of CU-masked HIP
 * streams, for AMD Instinct MI355X (gfx950).
 *
 * The calls follow the problem statement of the ECLIP paper:
 *   - a pool of streams whose CU masks are fixed at start-up, so that changing a
 *     kernel group's CU share at run time is a table write and never a driver call
 *     (Sec. III-A, "Pre-allocated CU Masked Streams");
 *   - a model = its kernels in execution order, partitioned into kernel groups; a
 *     lookup table names the pooled stream each group runs on (Sec. III-A,
 *     "Redirecting Kernel Dispatch", and Sec. III-B);
 *   - data dependencies between consecutive kernels that land on different streams
 *     are enforced by the library (Sec. III-A, "Enforcing Data Dependencies");
 *   - requests of one model are served in order by that model's worker; different
 *     models run concurrently (Sec. III-A);
 *   - the CU configuration of every group is chosen by the resource-allocation model
 *     of Sec. III-B, solved exactly on the CPU.
 *
 * Conventions
 *   - Every function returns an eclip_status, never throws and never aborts; a
 *     description of the last failure on the calling thread is at eclip_last_error().
 *   - "host" / "device" is stated for every pointer.  Sizes are in elements unless
 *     the name says bytes.
 *   - Handles are owned by the library and released by the matching destroy/free
 *     call; passing a released handle is undefined.
 *   - Thread safety: calls on different models may run on different threads at once;
 *     calls on one model are serialised inside the library.  Pool creation and
 *     destruction are not thread safe with respect to calls on the same pool.
 *
 * Environment variables (read by the library; for tuning and tests, never needed in service)
 *   ECLIP_GEMM_FORCE="kind,variant,n"  every matrix-core layer takes this plan instead of the planner's or the tuned
 *                         one: kind 0 = LDS-tiled kernel (variant = tile id, n = K slices), kind 1 = wave-split-K
 *                         kernel (variant = tile id, n = 4, 8 or 16 wavefronts); also turns launch sharing off
 *   ECLIP_NO_PAIRS=1      independent layers never share a launch (pairs of convolutions, pool + classifier, first
 *                         convolution reading the caller's tensor)
 *   ECLIP_GCONV_DIRECT=1  read at eclip_model_load: grouped convolutions take the direct kernel, not the matrix cores
 *   ECLIP_CONCAT_COPY=1   read at eclip_model_load: every CONCAT layer copies its operands (no concatenation in place)
 *   ECLIP_SHUFFLE_KERNEL=1  read at eclip_model_load: every SHUFFLE layer runs its kernel (no folding into weights)
 *   ECLIP_SWITCH_EVENTS=1   read at eclip_model_load / eclip_bench_switch: stream switches are ordered by an event pair
 *                         instead of stream memory operations (write / wait on a word of signal memory)
 *   ECLIP_TRACE=1         the set-up steps of the library (pool, model load) on stderr
 */
#ifndef ECLIP_H
#define ECLIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ECLIP_OK = 0,
    ECLIP_EINVAL = 1,   /* malformed argument or descriptor                                  */
    ECLIP_ENOMEM = 2,   /* host or device allocation failed                                  */
    ECLIP_EHIP = 3,     /* a HIP runtime call failed (text in eclip_last_error)              */
    ECLIP_ESTATE = 4,   /* call not valid in the object's current state                      */
    ECLIP_ETIMEOUT = 5, /* eclip_wait deadline passed; the request is still pending          */
    ECLIP_ELIMIT = 6    /* a documented capacity limit was exceeded                          */
} eclip_status;

/* Thread-local, NUL-terminated description of the last non-OK status on this thread. */
const char *eclip_last_error(void);

typedef struct eclip_pool eclip_pool;
typedef struct eclip_model eclip_model;
typedef struct eclip_req eclip_req;

/* ------------------------------------------------------------------------------------------
 * Stream pool (Sec. III-A, "Pre-allocated CU Masked Streams")
 * ---------------------------------------------------------------------------------------- */

/* One CU mask: bit i of words[i/32] set = CU i enabled (the bit order of
 * hipExtStreamCreateWithCUMask).  n_words == 0 asks for an unmasked stream (all CUs), the
 * analogue of the paper's shared default stream.  `owner` is the worker the mask was laid
 * out for, or -1 when shared; it is informational.  `words` is a host pointer, read during
 * the call only. */
typedef struct {
    const uint32_t *words;
    uint32_t n_words;
    int32_t owner;
} eclip_mask;

#define ECLIP_MAX_POOL_STREAMS 64u

/* Create one HIP stream per mask on `device`.  All masks are applied here, once.
 * Errors: EINVAL (null pointers, n_masks == 0, a mask with no bit set, a bit at or above the
 * device's CU count, a mask that leaves one of the device's XCDs without a CU -- the XCD count is read
 * from the device, and when the runtime cannot report it every masked stream is refused with EHIP),
 * ELIMIT (n_masks > ECLIP_MAX_POOL_STREAMS), EHIP.  Validation that
 * needs no device (null, zero masks, empty mask, limit) happens before any HIP call. */
eclip_status eclip_pool_create(int device, const eclip_mask *masks, uint32_t n_masks, eclip_pool **out);

/* HIP stream handle (hipStream_t, as void*) and enabled-CU count of pool entry `mask_id`.
 * Either output pointer may be NULL.  EINVAL for an unknown id. */
eclip_status eclip_pool_stream(const eclip_pool *pool, uint32_t mask_id, void **hip_stream, uint32_t *n_cu);

/* Number of CUs of the pool's device. */
eclip_status eclip_pool_device_cus(const eclip_pool *pool, uint32_t *n_cu);

/* Destroys every stream.  ESTATE while models loaded on the pool are still alive. */
eclip_status eclip_pool_destroy(eclip_pool *pool);

/* Hardware-queue sharing (Sec. II-C, Observation 2, as measured on MI355X).  Every masked stream owns an
 * HSA queue; the queues are dealt to the compute pipes of the command processor in creation order, and a
 * pipe serves one queue at a time: a queue that sits on a barrier (waiting for an event of another stream)
 * keeps its pipe, so two streams of one pipe that are in use in the same period slow each other down by
 * 3-5x (measured: two co-located ResNet-18 workers, 193 us per step on 4 distinct pipes, 600-930 us with
 * two active streams on one pipe).  *pipe receives the creation rank of the masked stream among the
 * pool's masked streams modulo ECLIP_N_PIPES, UINT32_MAX for an unmasked stream (it uses one of the
 * runtime's shared queues).  Tables installed with eclip_alloc_set on co-located models should use streams of
 * pairwise different pipes. */
#define ECLIP_N_PIPES 4u
eclip_status eclip_pool_pipe(const eclip_pool *pool, uint32_t mask_id, uint32_t *pipe);

/* Observation 2's experiment: a chain of `iters` dependent, trivially short kernels dealt round-robin to the
 * n pool entries mask_ids[0..n), each kernel waiting for its predecessor through an event.  *ns_per_kernel
 * receives the wall-clock time per kernel.  Host pointers. */
eclip_status eclip_bench_streams(eclip_pool *pool, const uint32_t *mask_ids, uint32_t n, uint32_t iters,
                                 double *ns_per_kernel);

/* Host-only helper: the per-worker mask layout of Sec. III-A.  The device's CUs are cut into
 * n_granules = total_cus / granule equal granules (the paper: 4 shader engines of 15 CUs).
 * Worker `worker` of `n_workers` claims granules in a fixed order chosen so that two workers
 * start at opposite ends and their masks of a and b granules share exactly
 * max(0, a + b - n_granules) granules; for 2 workers and 4 granules this reproduces the paper's
 * example (worker 1: SE 1 / 1,3 / 1,2,3; worker 2: SE 4 / 2,4 / 2,3,4).  The mask with
 * `take` granules is written to words_out[0..n_words).
 *   stripe == 0: granule g = CU bits [g*granule, (g+1)*granule)
 *   stripe  > 0: granule g = the runs of `stripe` consecutive bits number g, g + n_granules, ...:
 *                bits { stripe*(g + n_granules*j) + x : x < stripe, j < granule/stripe }
 * On MI355X mask bit i is CU (i/32) of shader engine (i/8) % 4 of XCD i % 8 (measured with
 * eclip_pool_probe), and a mask must keep at least one CU in every XCD.  So stripe = 0 with a
 * granule of 32 gives every worker one more CU in every shader engine of every XCD per granule, and
 * stripe = 8 with a granule of 64 gives it one whole shader engine in every XCD per granule (the
 * closest analogue of the paper's SE-aligned masks).
 * EINVAL: granule does not divide total_cus, stripe does not divide granule, take > n_granules or
 * 0, worker >= n_workers, n_words too small. */
eclip_status eclip_mask_layout(uint32_t total_cus, uint32_t granule, uint32_t n_workers, uint32_t worker,
                               uint32_t take, uint32_t stripe, uint32_t *words_out, uint32_t n_words);

/* Diagnostic: launch `n_blocks` one-wave workgroups on pool entry `mask_id` and report, per
 * workgroup, where it ran: out[i] = (xcc_id << 16) | (shader_engine << 8) | (shader_array << 4) | cu_id as read from
 * the wave's hardware-id registers.  `out` is a host array of n_blocks words. */
eclip_status eclip_pool_probe(eclip_pool *pool, uint32_t mask_id, uint32_t n_blocks, uint32_t *out);

/* The same probe, launched as a HIP graph captured from and replayed on the pool entry's stream: shows that replayed
 * kernels stay on the stream's CUs (what eclip_model_graphs relies on). */
eclip_status eclip_pool_probe_graph(eclip_pool *pool, uint32_t mask_id, uint32_t n_blocks, uint32_t *out);

/* ------------------------------------------------------------------------------------------
 * Models (Sec. III-A "Redirecting Kernel Dispatch"; kernel groups: Sec. III-B)
 * ---------------------------------------------------------------------------------------- */

enum { ECLIP_OP_CONV = 1, ECLIP_OP_LINEAR, ECLIP_OP_MAXPOOL, ECLIP_OP_GAP, ECLIP_OP_LAYERNORM,
       ECLIP_OP_SOFTMAX, ECLIP_OP_ATTENTION, ECLIP_OP_EMBED, ECLIP_OP_ELTWISE, ECLIP_OP_CONCAT,
       ECLIP_OP_SHUFFLE };
enum { ECLIP_ACT_NONE = 0, ECLIP_ACT_RELU, ECLIP_ACT_RELU6, ECLIP_ACT_GELU };
enum { ECLIP_F32 = 0, ECLIP_BF16 = 1, ECLIP_F16 = 2 };
enum { ECLIP_KIND_IMAGE = 0, ECLIP_KIND_SEQ = 1, ECLIP_KIND_VEC = 2 };
enum { ECLIP_IN_IMAGE = 0, ECLIP_IN_TOKENS = 1, ECLIP_IN_SEQ = 2, ECLIP_IN_VEC = 3 };

/* One layer = one kernel of the model, in execution order.  Logical tensor layouts:
 * IMAGE [B][C][H][W]; SEQ [B][S][Hd] described as c = Hd, h = 1, w = S; VEC [B][n] as c = n.
 *   CONV       y = act(conv2d(x, W[c][cin/groups][kh][kw], stride, pad) + b + in1); zero padding;
 *              groups = 1 (matrix cores), cin == c == groups (depthwise kernel) or any common
 *              divisor of cin and c (grouped convolution, direct kernel; 16-bit models)
 *   LINEAR     y = act(x W[c][k]^T + b + in1); an IMAGE input is flattened in (C,H,W) order,
 *              a SEQ input is transformed per token
 *   MAXPOOL    kh x kw window, stride, pad (padding never wins the max)
 *   GAP        mean over H*W -> VEC
 *   LAYERNORM  over the last axis of (x + in1): biased variance, eps, gamma at g_off, beta at be_off
 *   SOFTMAX    over the last axis
 *   ATTENTION  x = SEQ with c = 3*Hd laid out [q | k | v], each head-major with `heads` heads;
 *              per head softmax(q k^T / sqrt(d)) v
 *   EMBED      input = int32 token ids [B][S]; y = tok[id] + pos[s] + typ[0]; tables at w_off
 *              (aux0 rows), g_off (aux1 rows), be_off (2 rows)
 *   ELTWISE    y = act(x + b + in1)
 *   CONCAT     y = [x | in1] along the channel axis (second workload family: dense blocks)
 *   SHUFFLE    channel shuffle with `groups` groups: y[.., j] = x[.., (j % groups) * (c / groups) + j / groups]
 * in0/in1 index earlier layers; -1 = the model input; in1 = -2 = absent.  Offsets are element
 * offsets into the weight blob, -1 = absent (treated as zero bias / gamma 1 / beta 0). */
typedef struct {
    int32_t op, in0, in1, kind;
    int32_t c, h, w;
    int32_t kh, kw, stride, pad, groups;
    int32_t act, heads;
    int64_t w_off, b_off, g_off, be_off;
    float eps;
    int32_t aux0, aux1;
} eclip_layer;

typedef struct {
    int32_t dtype;                  /* storage and MFMA input type of activations and weights */
    int32_t in_kind;                /* ECLIP_IN_* */
    int32_t in_c, in_h, in_w;       /* IMAGE: C,H,W; SEQ/TOKENS: c = Hd, h = 1, w = S; VEC: c = n */
    const eclip_layer *layers;      /* host, n_layers entries, execution order */
    uint32_t n_layers;
    const uint32_t *group_of_layer; /* host, non-decreasing, starts at 0, covers 0..n_groups-1 */
    uint32_t n_groups;
    uint32_t max_batch;             /* largest batch a request may carry (>= 1) */
    uint32_t max_inflight;          /* submitted-but-not-waited requests allowed at once (>= 1) */
} eclip_model_desc;

/* Validate the descriptor, copy the weights into a device layout of the library's choosing and
 * allocate activation and workspace buffers for max_batch.  `weights` holds weight_bytes bytes of
 * `dtype` elements (host pointer, or device pointer when weights_on_device != 0); the caller may
 * free it after the call.  Descriptor validation needs no device and precedes every HIP call.
 * EINVAL: bad op/shape/offset, non-monotone groups, unsupported combination (16-bit models need
 * channel counts that are multiples of 8 on every tensor that feeds another layer; attention needs
 * head size 32 or 64 and S <= 512 and a 16-bit dtype; normalisation rows <= 8192 elements). */
eclip_status eclip_model_load(eclip_pool *pool, const eclip_model_desc *desc, const void *weights,
                              size_t weight_bytes, int weights_on_device, eclip_model **out);

/* ESTATE while requests are in flight. */
eclip_status eclip_model_free(eclip_model *model);

/* Move a loaded model to another pool of the same device (weights and buffers stay where they are; only the
 * streams change).  The group -> stream table is cleared: call eclip_alloc_set again.  Lets a serving pool of
 * a few streams on distinct pipes replace the wide pool used for profiling.  ESTATE while requests are in
 * flight, EINVAL for a pool on another device. */
eclip_status eclip_model_rebind(eclip_model *model, eclip_pool *new_pool);

/* Install the lookup table group -> pooled stream (the optimizer's output, Sec. III-B).  Takes
 * effect for the next eclip_submit; no stream is created or re-masked.  EINVAL: n_groups differs
 * from the model's, unknown mask id. */
eclip_status eclip_alloc_set(eclip_model *model, const uint32_t *mask_id_of_group, uint32_t n_groups);

/* Number of stream switches (cross-stream dependencies) one request incurs under the current table. */
eclip_status eclip_model_switches(const eclip_model *model, uint32_t *n_switches);

/* Enqueue one request.  d_in: device pointer, logical layout, `dtype` elements for IMAGE/SEQ/VEC
 * inputs ([B][C][H][W] / [B][S][Hd] / [B][n]) or int32 token ids [B][S].  d_out: device pointer to
 * float32 in the last layer's logical layout.  Both stay owned by the caller and must remain valid
 * until eclip_wait succeeds.  Returns at once; kernels of group g run on the stream named by the
 * table, and consecutive groups on different streams are ordered by an event.  Requests of one
 * model execute in submission order.  ESTATE before eclip_alloc_set; EINVAL batch == 0 or
 * > max_batch; ELIMIT more than max_inflight requests outstanding.  EHIP when a launch fails part-way: the
 * library then drains the device, drops the request (its slot stays free, nothing of it remains queued) and
 * leaves earlier requests of the model waitable. */
eclip_status eclip_submit(eclip_model *model, const void *d_in, void *d_out, uint32_t batch, eclip_req **out);

/* The same request with every kernel's scratch memory (the partial sums of K slices and of the global average
 * pool) in a static device array of ECLIP_STATIC_SCRATCH_BYTES that the library holds on each GPU it has a pool
 * on, instead of the workspace eclip_model_load allocated.  For callers that must not allocate device memory:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The call itself allocates
 * nothing, on the host side of the runtime or on the device.  Arguments, ordering and results are those of
 * eclip_submit (bit for bit: the kernels and their plans are the same).  Every call on a GPU shares that GPU's
 * array, whose content is whatever the last call left (every kernel writes its partial sums before reading
 * them, so nothing has to be cleared): requests issued through this call on different models of one GPU must not
 * overlap in time -- wait for one before submitting the next -- or they race on the array.
 * ELIMIT: the model's kernels need more scratch than the array holds (the need is fixed at load: it grows with
 * max_batch); otherwise the errors of eclip_submit. */
#define ECLIP_STATIC_SCRATCH_BYTES (16u << 20)
eclip_status eclip_submit_static(eclip_model *model, const void *d_in, void *d_out, uint32_t batch, eclip_req **out);

/* Replay instead of re-launch (Sec. III-A: the cost of dispatch is first-order for kernels that last microseconds).
 * While on, eclip_submit captures a request the first time it sees a combination of (d_in, d_out, batch) under the
 * current table -- one HIP graph per run of kernel groups that share a pooled stream -- and afterwards replays the
 * graphs on those streams, with the same events between them at the stream switches.  The kernels, their order,
 * their streams (and therefore their CU masks) and the results are those of the plain path, bit for bit.  Up to 8
 * captured requests are kept per model (least recently used first out); eclip_alloc_set with a different table,
 * eclip_model_rebind and eclip_model_tune discard them.  Off after load.  ESTATE while requests are in flight. */
eclip_status eclip_model_graphs(eclip_model *model, int enable);

/* Timestamps cost a marker packet at both ends of every request, so requests carry them only while this is on
 * (off after load).  Takes effect for the next eclip_submit. */
eclip_status eclip_model_timing(eclip_model *model, int enable);

typedef struct {
    uint64_t gpu_ns;       /* first kernel start to last kernel end, device clock; 0 unless eclip_model_timing was on at submit */
    uint32_t n_kernels;    /* kernels launched */
    uint32_t n_switches;   /* cross-stream dependencies inserted */
} eclip_timing;

/* Block until the request has finished or timeout_ns has passed (UINT64_MAX = no limit).  On OK
 * the request handle is consumed.  On ETIMEOUT it stays valid and may be waited again. */
eclip_status eclip_wait(eclip_req *req, uint64_t timeout_ns, eclip_timing *opt_out);

/* Solo latency of each kernel of `group` on pool entry `mask_id` (Sec. III-B, "Minimum CU
 * Threshold Profiling"): median over `iters` timed samples, integer nanoseconds, one value per
 * kernel of the group in execution order (host array).  A sample is the HIP-event time of 8
 * back-to-back launches of the kernel on that stream, divided by 8 (an event pair around one
 * microsecond-scale kernel would mostly time the events).  Runs one untimed forward pass on zero
 * input first so every buffer is initialised.  Must not overlap other requests of this model. */
eclip_status eclip_profile_group(eclip_model *model, uint32_t group, uint32_t mask_id, uint32_t batch,
                                 uint32_t iters, uint64_t *ns_per_kernel_out);

/* Measured plan selection for the matrix-core layers (an extension of the profiling step of Sec. III-B: the library
 * writes its own kernels, so next to "how long does this kernel take on c CUs" it can also ask "which of my tile
 * shapes is fastest on c CUs").  For every distinct GEMM problem (M, N, K) among the model's CONV / LINEAR layers
 * at `batch`, every candidate launch plan is timed on pool entry `mask_id` (minimum over `iters` samples of 6
 * back-to-back launches) and the fastest is remembered for streams of that CU count -- unless the cost model's own
 * choice is within 5 % of it, in which case that one stays.  Later eclip_submit / eclip_profile_* / kernel_info
 * calls use the remembered plans; problems or CU counts never tuned keep the cost model's plans.  Results stay
 * within the same tolerances (a different tile only reassociates the fp32 sums).  *n_tuned_out (optional) receives
 * the number of problems timed.  Same preconditions as eclip_profile_group. */
eclip_status eclip_model_tune(eclip_model *model, uint32_t mask_id, uint32_t batch, uint32_t iters, uint32_t *n_tuned_out);

/* The group as eclip_submit serves it (Sec. III-B: the allocator's beta of a unit): all launches of `group` in
 * order on pool entry `mask_id` -- including the input re-layout in group 0, two independent layers sharing a
 * launch, pool + classifier in one launch -- timed as one interval; median over `iters` samples in integer
 * nanoseconds to *group_ns_out, and the number of kernels launched per pass to *n_launches_out (optional; the
 * kernel count the allocator's CUAverage should weigh the unit with).  Same preconditions as
 * eclip_profile_group. */
eclip_status eclip_profile_group_served(eclip_model *model, uint32_t group, uint32_t mask_id, uint32_t batch,
                                        uint32_t iters, uint64_t *group_ns_out, uint32_t *n_launches_out);

/* Number of layers (kernels before any launch sharing) in `group`. */
eclip_status eclip_model_group_size(const eclip_model *model, uint32_t group, uint32_t *n_kernels);

/* How layer `layer` would be launched for `batch` samples on pool entry `mask_id`: which kernel and
 * with what shape.  For reporting; nothing is launched. */
typedef struct {
    char kernel[48];        /* kernel function name, e.g. "conv_wsk_kernel" */
    uint32_t launches;      /* kernels launched for this layer (2 when K is split over the grid) */
    uint32_t workgroups;    /* workgroups of the main kernel */
    uint32_t threads;       /* threads per workgroup of the main kernel */
    uint32_t tile_m, tile_n;/* output tile of a matrix-core kernel, else 0 */
    uint32_t k_splits;      /* grid-level K slices (matrix-core LDS-tiled kernel), else 1 */
    uint64_t m, n, k;       /* GEMM view of a CONV / LINEAR layer, else 0 */
} eclip_kernel_info;
eclip_status eclip_model_kernel_info(const eclip_model *model, uint32_t layer, uint32_t mask_id, uint32_t batch,
                                     eclip_kernel_info *out);

/* ------------------------------------------------------------------------------------------
 * Resource-allocation optimizer (Sec. III-B, "Optimization Formulation"); CPU only
 * ---------------------------------------------------------------------------------------- */

enum { ECLIP_OVERLAP_EXCESS = 0, ECLIP_OVERLAP_LITERAL = 1, ECLIP_OVERLAP_TABLE = 2 };

typedef struct { uint64_t lo, hi; } eclip_u128;

/* A unit is a run of n_kernels >= 1 consecutive kernels that share one configuration (n_kernels
 * == 1 everywhere is the paper's per-kernel model).  Arrays are host pointers.
 *   configs[n_configs]            strictly increasing CU counts (the paper: 15,30,45,60)
 *   units_of_worker[n_workers]    units per worker; units are stored worker-major below
 *   n_kernels[sum units]          kernels per unit
 *   beta[sum units][n_configs]    profiled solo latency of the unit at each configuration, ns
 *   switch_max                    barrier-packet budget per worker per request
 *   overlap_mode                  EXCESS:  CUOverlap = max(0, sum_w CUAverage_w - total_cus)
 *                                 LITERAL: CUOverlap = sum_w CUAverage_w (as printed)
 *                                 TABLE:   alpha = alpha_ppm[min(n_alpha-1, floor(EXCESS overlap / granule))] / 1e6,
 *                                          alpha_ppm non-decreasing
 * Objective: sum over workers of sum over units of beta * (1 + alpha), alpha = CUOverlap / total_cus.
 * Ties: smaller sum of CU averages, then the lexicographically smallest index vector. */
typedef struct {
    uint32_t total_cus;
    const uint32_t *configs;
    uint32_t n_configs;
    uint32_t n_workers;
    const uint32_t *units_of_worker;
    const uint32_t *n_kernels;
    const uint64_t *beta;
    uint32_t switch_max;
    uint32_t overlap_mode;
    const uint64_t *alpha_ppm;
    uint32_t n_alpha;
    uint32_t granule;
    /* Extensions, 0 = the model as printed.
     * max_configs:    a worker may use at most this many distinct configurations in one request.  Every
     *                 (worker, configuration) pair in use is one pooled stream, and only a few streams run
     *                 without oversubscribing the hardware queues (Sec. II-C, Observation 2: 7 on MI50;
     *                 on MI355X 4, one per compute pipe, see eclip_bench_streams).
     * switch_cost_ns: added to a worker's solo time at every configuration switch (factor (iii) of
     *                 Sec. III-B, which the printed model bounds through switch_max only). */
    uint32_t max_configs;
    uint64_t switch_cost_ns;
    /* max_configs_of_worker[n_workers] (host, optional): the same limit per worker; when given it replaces max_configs
     * (0 = no limit for that worker).  Lets a caller spend a global stream budget unevenly: with 4 usable streams and 3
     * workers, solve for (2,1,1), (1,2,1) and (1,1,2) and keep the best objective. */
    const uint32_t *max_configs_of_worker;
} eclip_alloc_problem;

/* Exact minimiser.  cfg_idx_out[sum units] receives the configuration index of every unit
 * (worker-major); objective_out (optional) the objective as the exact integer
 *   (sum of chosen betas) * (total_cus*D + Ov_D)      EXCESS / LITERAL, D = lcm of the workers' kernel counts
 *   (sum of chosen betas) * (10^6 + alpha_ppm)        TABLE
 * and switches_out[n_workers] (optional) each worker's switch count.
 * EINVAL on malformed input; ELIMIT when the instance exceeds the solver's state budget or the
 * objective would not fit 128 bits. */
eclip_status eclip_alloc_solve(const eclip_alloc_problem *problem, uint32_t *cfg_idx_out,
                               eclip_u128 *objective_out, uint32_t *switches_out);

/* The two partitioning scenarios the paper compares its optimizer with (Sec. IV, "Spatial Partitioning Scenarios";
 * switch counts as in Table I), computed from the same problem description; only configs, units_of_worker and
 * beta are read.  Exact integer comparisons, no search.  cfg_idx_out[sum units] and switches_out[n_workers]
 * (optional) as for eclip_alloc_solve.  EINVAL on malformed input.
 *
 * Model-Wise (Sec. II-A, Sec. IV): every worker keeps one configuration for the whole request -- the smallest CU
 * count c with  slo_den * sum_g beta[g][c] <= slo_num * sum_g beta[g][largest]  (the QoS convention of Sec. II-A
 * is 3x the solo latency: slo_num = 3, slo_den = 1); the largest configuration always qualifies.  No switches. */
eclip_status eclip_alloc_model_wise(const eclip_alloc_problem *problem, uint32_t slo_num, uint32_t slo_den,
                                    uint32_t *cfg_idx_out, uint32_t *switches_out);

/* Kernel-Wise on pre-allocated streams (Sec. IV, KW-Prealloc): every unit runs at its own minimum-CU threshold
 * (Sec. III-B, "Minimum CU Threshold Profiling": the fewest CUs without noticeable slowdown), read as the smallest
 * c with  100 * beta[c] <= (100 + tol_pct) * beta[largest]  (tol_pct = 5 by default in the benchmark); a switch is
 * counted wherever consecutive units of a worker differ. */
eclip_status eclip_alloc_kernel_wise(const eclip_alloc_problem *problem, uint32_t tol_pct, uint32_t *cfg_idx_out,
                                     uint32_t *switches_out);

/* ------------------------------------------------------------------------------------------
 * Repartitioning overhead (Sec. II-C, Observation 1)
 * ---------------------------------------------------------------------------------------- */

/* Measures, with a trivially short kernel, the wall-clock cost per kernel of three ways of running
 * a chain of `iters` dependent kernels:
 *   same_stream_ns  all on pool entry mask_a (no repartitioning);
 *   pooled_ns       alternating between pool entries mask_a and mask_b, ordered the way eclip_submit orders a
 *                   stream switch (switching through the pre-allocated pool);
 *   create_ns       every kernel on a stream created with mask_b's CU mask for that kernel (applying the mask
 *                   at run time): host time to create the stream and queue the dependent kernel on it; draining
 *                   and destroying the previous stream is not counted.
 * Host pointers; any output may be NULL. */
eclip_status eclip_bench_switch(eclip_pool *pool, uint32_t mask_a, uint32_t mask_b, uint32_t iters,
                                double *same_stream_ns, double *pooled_ns, double *create_ns);

#ifdef __cplusplus
}
#endif
#endif /* ECLIP_H */
