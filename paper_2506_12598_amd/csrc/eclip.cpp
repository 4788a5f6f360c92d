// libeclip host side: stream pool, model loader, executor, profiler, C ABI.
#include "eclip.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <array>
#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "kernels.h"

namespace eclip {
std::string solve_alloc(const eclip_alloc_problem *p, uint32_t *cfg_out, eclip_u128 *obj_out, uint32_t *sw_out, bool *limit);
std::string policy_model_wise(const eclip_alloc_problem *p, uint32_t slo_num, uint32_t slo_den, uint32_t *cfg_out, uint32_t *sw_out);
std::string policy_kernel_wise(const eclip_alloc_problem *p, uint32_t tol_pct, uint32_t *cfg_out, uint32_t *sw_out);
}
using namespace eclip;

// ------------------------------------------------------------------------------------------------
// errors
// ------------------------------------------------------------------------------------------------
static thread_local std::string g_err;

static eclip_status fail(eclip_status st, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return st;
}
#define HIP_TRY(call)                                                                                         \
    do {                                                                                                      \
        hipError_t e_ = (call);                                                                               \
        if (e_ != hipSuccess) return fail(ECLIP_EHIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
    } while (0)

extern "C" const char *eclip_last_error(void) { return g_err.c_str(); }

// ECLIP_TRACE=1 in the environment prints the library's set-up steps to stderr.
static bool trace_on()
{
    static const bool on = getenv("ECLIP_TRACE") != nullptr;
    return on;
}
#define TRACE(...)                                                        \
    do {                                                                  \
        if (trace_on()) { fprintf(stderr, "[eclip] " __VA_ARGS__); fputc('\n', stderr); fflush(stderr); } \
    } while (0)

// ------------------------------------------------------------------------------------------------
// pool
// ------------------------------------------------------------------------------------------------
struct PoolStream {
    hipStream_t stream = nullptr;
    uint32_t n_cu = 0;
    uint32_t pipe = UINT32_MAX;          // creation rank among the pool's masked streams, modulo ECLIP_N_PIPES
    std::vector<uint32_t> words;
    int32_t owner = -1;
};
struct eclip_pool {
    int device = 0;
    uint32_t device_cus = 0;
    std::vector<PoolStream> streams;
    void *scratch = nullptr;             // this device's static scratch (eclip_submit_static)
    int n_models = 0;
    std::mutex mu;
};

static uint32_t popcount_words(const uint32_t *w, uint32_t n)
{
    uint32_t c = 0;
    for (uint32_t i = 0; i < n; ++i) c += (uint32_t)__builtin_popcount(w[i]);
    return c;
}

// Scratch for eclip_submit_static: the K-slice partial sums of the matrix-core kernels and the partial sums of the
// global average pool go here instead of the workspace eclip_model_load allocated.  One array per GPU, held until the
// process ends.  In host code this name only stands for the symbol: its device address is looked up once per device in
// eclip_pool_create (static_scratch_of) and only that address is handed to kernels.
static __device__ __align__(256) unsigned char scratch[ECLIP_STATIC_SCRATCH_BYTES];

static std::mutex g_scratch_mu;
static void *g_scratch_ptr[64] = {nullptr};

// Address of `scratch` on `device` (which must be the current device), looked up on first use.
static hipError_t static_scratch_of(int device, void **ptr)
{
    if (device < 0 || device >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = p;
    }
    *ptr = g_scratch_ptr[device];
    return hipSuccess;
}

extern "C" eclip_status eclip_pool_create(int device, const eclip_mask *masks, uint32_t n_masks, eclip_pool **out)
{
    if (!out) return fail(ECLIP_EINVAL, "out is null");
    *out = nullptr;
    if (!masks || n_masks == 0) return fail(ECLIP_EINVAL, "no masks given");
    if (n_masks > ECLIP_MAX_POOL_STREAMS) return fail(ECLIP_ELIMIT, "%u masks exceed the pool limit of %u streams", n_masks, ECLIP_MAX_POOL_STREAMS);
    for (uint32_t i = 0; i < n_masks; ++i) {
        if (masks[i].n_words && !masks[i].words) return fail(ECLIP_EINVAL, "mask %u: words is null", i);
        if (masks[i].n_words && popcount_words(masks[i].words, masks[i].n_words) == 0)
            return fail(ECLIP_EINVAL, "mask %u enables no CU", i);
    }
    int n_dev = 0;
    TRACE("pool_create: %u masks", n_masks);
    HIP_TRY(hipGetDeviceCount(&n_dev));
    TRACE("devices: %d", n_dev);
    if (device < 0 || device >= n_dev) return fail(ECLIP_EINVAL, "device %d out of range (%d devices)", device, n_dev);
    HIP_TRY(hipSetDevice(device));
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDeviceProperties(&prop, device));
    const uint32_t cus = (uint32_t)prop.multiProcessorCount;
    TRACE("device %d: %s, %u CUs", device, prop.name, cus);
    for (uint32_t i = 0; i < n_masks; ++i)
        for (uint32_t wd = 0; wd < masks[i].n_words; ++wd)
            for (uint32_t b = 0; b < 32; ++b)
                if ((masks[i].words[wd] >> b & 1u) && wd * 32 + b >= cus)
                    return fail(ECLIP_EINVAL, "mask %u enables CU %u but the device has %u", i, wd * 32 + b, cus);
    // Consecutive mask bits rotate over the device's XCDs (bit i belongs to XCD i % n_xcc); the runtime does
    // not survive a queue mask that leaves an XCD without any CU, so such masks are refused here.  The XCD count
    // comes from the device; when the runtime cannot tell it, masked streams are refused altogether.
    bool any_masked = false;
    for (uint32_t i = 0; i < n_masks; ++i) any_masked |= masks[i].n_words != 0;
    if (any_masked) {
        int xcc = 0;
        const hipError_t xe = hipDeviceGetAttribute(&xcc, hipDeviceAttributeNumberOfXccs, device);
        if (xe != hipSuccess || xcc < 1 || cus % (uint32_t)xcc)
            return fail(ECLIP_EHIP, "cannot read the XCD count of device %d (%s, value %d): CU-masked streams are refused", device,
                        hipGetErrorString(xe), xcc);
        const uint32_t n_xcc = (uint32_t)xcc;
        TRACE("device %d: %u XCDs", device, n_xcc);
        for (uint32_t i = 0; i < n_masks; ++i) {
            if (masks[i].n_words == 0) continue;
            std::vector<uint32_t> per(n_xcc, 0u);
            for (uint32_t b = 0; b < masks[i].n_words * 32; ++b)
                if (masks[i].words[b / 32] >> (b % 32) & 1u) per[b % n_xcc]++;
            for (uint32_t x = 0; x < n_xcc; ++x)
                if (per[x] == 0) return fail(ECLIP_EINVAL, "mask %u leaves XCD %u (mask bits congruent to %u modulo %u) without a CU", i, x, x, n_xcc);
        }
    }
    void *scratch_ptr = nullptr;
    HIP_TRY(static_scratch_of(device, &scratch_ptr));
    HIP_TRY(attention_init());
    HIP_TRY(conv_gemm_init());
    HIP_TRY(conv_wsk_init());
    TRACE("kernel attributes set");
    eclip_pool *p = new (std::nothrow) eclip_pool;
    if (!p) return fail(ECLIP_ENOMEM, "out of host memory");
    p->device = device;
    p->device_cus = cus;
    p->scratch = scratch_ptr;
    p->streams.resize(n_masks);
    uint32_t n_masked = 0;
    for (uint32_t i = 0; i < n_masks; ++i) {
        PoolStream &s = p->streams[i];
        s.owner = masks[i].owner;
        if (masks[i].n_words) s.pipe = n_masked++ % ECLIP_N_PIPES;
        hipError_t e;
        if (masks[i].n_words == 0) {
            s.n_cu = cus;
            e = hipStreamCreateWithFlags(&s.stream, hipStreamNonBlocking);
        } else {
            s.words.assign(masks[i].words, masks[i].words + masks[i].n_words);
            s.n_cu = popcount_words(s.words.data(), masks[i].n_words);
            e = hipExtStreamCreateWithCUMask(&s.stream, masks[i].n_words, s.words.data());
        }
        TRACE("stream %u: %u CUs, %s", i, s.n_cu, hipGetErrorString(e));
        if (e != hipSuccess) {
            for (uint32_t j = 0; j < i; ++j) (void)hipStreamDestroy(p->streams[j].stream);
            delete p;
            return fail(ECLIP_EHIP, "creating pool stream %u failed: %s", i, hipGetErrorString(e));
        }
    }
    *out = p;
    return ECLIP_OK;
}

extern "C" eclip_status eclip_pool_stream(const eclip_pool *pool, uint32_t mask_id, void **hip_stream, uint32_t *n_cu)
{
    if (!pool) return fail(ECLIP_EINVAL, "pool is null");
    if (mask_id >= pool->streams.size()) return fail(ECLIP_EINVAL, "unknown mask id %u", mask_id);
    if (hip_stream) *hip_stream = (void *)pool->streams[mask_id].stream;
    if (n_cu) *n_cu = pool->streams[mask_id].n_cu;
    return ECLIP_OK;
}

extern "C" eclip_status eclip_pool_device_cus(const eclip_pool *pool, uint32_t *n_cu)
{
    if (!pool || !n_cu) return fail(ECLIP_EINVAL, "null argument");
    *n_cu = pool->device_cus;
    return ECLIP_OK;
}

extern "C" eclip_status eclip_pool_pipe(const eclip_pool *pool, uint32_t mask_id, uint32_t *pipe)
{
    if (!pool || !pipe) return fail(ECLIP_EINVAL, "null argument");
    if (mask_id >= pool->streams.size()) return fail(ECLIP_EINVAL, "unknown mask id %u", mask_id);
    *pipe = pool->streams[mask_id].pipe;
    return ECLIP_OK;
}

// A dependency between two streams ("the next kernel group waits for everything queued so far on the stream it leaves").
// With stream memory operations (hipStreamWriteValue64 on the stream that is left, hipStreamWaitValue64 on the one that
// is entered, on a word of signal memory) a hop costs about 6 us on top of the kernel, with an event pair about 13 us
// (dependent chain of trivial kernels alternating between two masked streams: 9.0 against 16.3 us per kernel).  Values
// grow by one per hop, and a hop's write is always queued before its wait, on a stream that has itself passed every
// earlier wait of the chain, so the word only ever grows and no wait can be left behind unanswered.  Falls back to
// events where the device lacks the operations or ECLIP_SWITCH_EVENTS is set.
struct HopSignal {
    uint64_t *word = nullptr;                // device, signal memory
    uint64_t seq = 0;
    hipError_t init(int device)
    {
        int can = 0;
        if (getenv("ECLIP_SWITCH_EVENTS") || hipDeviceGetAttribute(&can, hipDeviceAttributeCanUseStreamWaitValue, device) != hipSuccess || !can) {
            (void)hipGetLastError();
            return hipSuccess;
        }
        hipError_t e = hipExtMallocWithFlags((void **)&word, 8, hipMallocSignalMemory);
        if (e != hipSuccess) { word = nullptr; (void)hipGetLastError(); return hipSuccess; }
        const uint64_t zero = 0;
        e = hipMemcpy(word, &zero, 8, hipMemcpyHostToDevice);
        if (e != hipSuccess) { (void)hipFree(word); word = nullptr; }
        return e;
    }
    void release()
    {
        if (word) (void)hipFree(word);
        word = nullptr;
    }
    // `ev` is the event used when stream memory operations are not available
    hipError_t hop(hipStream_t from, hipStream_t to, hipEvent_t ev)
    {
        if (word) {
            const uint64_t v = ++seq;
            hipError_t e = hipStreamWriteValue64(from, word, v, 0);
            if (e != hipSuccess) return e;
            return hipStreamWaitValue64(to, word, v, hipStreamWaitValueGte, ~(uint64_t)0);
        }
        hipError_t e = hipEventRecord(ev, from);
        if (e != hipSuccess) return e;
        return hipStreamWaitEvent(to, ev, 0);
    }
};

extern "C" eclip_status eclip_bench_streams(eclip_pool *pool, const uint32_t *mask_ids, uint32_t n, uint32_t iters,
                                            double *ns_per_kernel)
{
    if (!pool || !mask_ids || !ns_per_kernel) return fail(ECLIP_EINVAL, "null argument");
    if (n == 0 || n > ECLIP_MAX_POOL_STREAMS) return fail(ECLIP_EINVAL, "n must be 1..%u", ECLIP_MAX_POOL_STREAMS);
    if (iters == 0 || iters > 100000) return fail(ECLIP_EINVAL, "iters must be 1..100000");
    for (uint32_t i = 0; i < n; ++i)
        if (mask_ids[i] >= pool->streams.size()) return fail(ECLIP_EINVAL, "unknown mask id %u", mask_ids[i]);
    HIP_TRY(hipSetDevice(pool->device));
    uint32_t *d = nullptr;
    HIP_TRY(hipMalloc(&d, 256));
    hipError_t e = hipMemset(d, 0, 256);
    std::vector<hipEvent_t> ev(n, nullptr);
    for (uint32_t i = 0; i < n && e == hipSuccess; ++i) e = hipEventCreateWithFlags(&ev[i], hipEventDisableTiming);
    HopSignal hops;                                  // the same dependency mechanism eclip_submit uses
    if (e == hipSuccess) e = hops.init(pool->device);
    double result = 0.0;
    for (int pass = 0; pass < 2 && e == hipSuccess; ++pass) {          // pass 0 warms every queue up
        const uint32_t count = pass == 0 ? std::min<uint32_t>(iters, 4 * n) : iters;
        const auto t0 = std::chrono::steady_clock::now();
        for (uint32_t i = 0; i < count && e == hipSuccess; ++i) {
            const hipStream_t cur = pool->streams[mask_ids[i % n]].stream;
            if (i && n > 1) {
                const hipStream_t prev = pool->streams[mask_ids[(i - 1) % n]].stream;
                e = hops.hop(prev, cur, ev[i % n]);
            }
            if (e == hipSuccess) e = launch_tick(d, cur);
        }
        for (uint32_t i = 0; i < n && e == hipSuccess; ++i) e = hipStreamSynchronize(pool->streams[mask_ids[i]].stream);
        result = (double)std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now() - t0).count() / count;
    }
    for (hipEvent_t x : ev)
        if (x) (void)hipEventDestroy(x);
    (void)hipDeviceSynchronize();
    hops.release();
    (void)hipFree(d);
    if (e != hipSuccess) return fail(ECLIP_EHIP, "stream bench failed: %s", hipGetErrorString(e));
    *ns_per_kernel = result;
    return ECLIP_OK;
}

extern "C" eclip_status eclip_pool_destroy(eclip_pool *pool)
{
    if (!pool) return fail(ECLIP_EINVAL, "pool is null");
    if (pool->n_models > 0) return fail(ECLIP_ESTATE, "%d models are still loaded on this pool", pool->n_models);
    HIP_TRY(hipSetDevice(pool->device));
    for (PoolStream &s : pool->streams) {
        (void)hipStreamSynchronize(s.stream);
        (void)hipStreamDestroy(s.stream);
    }
    delete pool;
    return ECLIP_OK;
}

// The granule order of worker 0: odd granules (1-based) ascending, then even ones; worker 1 walks it
// backwards, so that the two start at opposite ends (Sec. III-A: SE 1,3,2 against SE 4,2,3).  Further
// pairs of workers use the same two walks rotated.
extern "C" eclip_status eclip_mask_layout(uint32_t total_cus, uint32_t granule, uint32_t n_workers, uint32_t worker,
                                          uint32_t take, uint32_t stripe, uint32_t *words_out, uint32_t n_words)
{
    if (!words_out) return fail(ECLIP_EINVAL, "words_out is null");
    if (granule == 0 || total_cus == 0 || total_cus % granule) return fail(ECLIP_EINVAL, "granule %u does not divide %u CUs", granule, total_cus);
    const uint32_t ng = total_cus / granule;
    if (n_workers == 0 || worker >= n_workers) return fail(ECLIP_EINVAL, "worker %u of %u", worker, n_workers);
    if (take == 0 || take > ng) return fail(ECLIP_EINVAL, "take %u of %u granules", take, ng);
    if ((uint64_t)n_words * 32 < total_cus) return fail(ECLIP_EINVAL, "n_words too small for %u CUs", total_cus);
    if (stripe && granule % stripe) return fail(ECLIP_EINVAL, "stripe %u does not divide the granule of %u CUs", stripe, granule);
    std::vector<uint32_t> order;
    for (uint32_t g = 0; g < ng; g += 2) order.push_back(g);
    for (uint32_t g = 1; g < ng; g += 2) order.push_back(g);
    if (worker & 1u) std::reverse(order.begin(), order.end());
    const uint32_t pairs = (n_workers + 1) / 2;
    const uint32_t rot = (worker / 2) * (ng / pairs) % ng;
    std::rotate(order.begin(), order.begin() + rot, order.end());
    std::fill(words_out, words_out + n_words, 0u);
    for (uint32_t i = 0; i < take; ++i) {
        const uint32_t g = order[i];
        for (uint32_t j = 0; j < granule; ++j) {
            const uint32_t bit = stripe ? stripe * (g + ng * (j / stripe)) + j % stripe : g * granule + j;
            words_out[bit / 32] |= 1u << (bit % 32);
        }
    }
    return ECLIP_OK;
}

extern "C" eclip_status eclip_pool_probe(eclip_pool *pool, uint32_t mask_id, uint32_t n_blocks, uint32_t *out)
{
    if (!pool || !out) return fail(ECLIP_EINVAL, "null argument");
    if (mask_id >= pool->streams.size()) return fail(ECLIP_EINVAL, "unknown mask id %u", mask_id);
    if (n_blocks == 0 || n_blocks > 65536) return fail(ECLIP_EINVAL, "n_blocks must be 1..65536");
    HIP_TRY(hipSetDevice(pool->device));
    uint32_t *d = nullptr;
    HIP_TRY(hipMalloc(&d, (size_t)n_blocks * 4));
    hipStream_t s = pool->streams[mask_id].stream;
    hipError_t e = launch_probe(d, (int)n_blocks, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e == hipSuccess) e = hipMemcpy(out, d, (size_t)n_blocks * 4, hipMemcpyDeviceToHost);
    (void)hipFree(d);
    if (e != hipSuccess) return fail(ECLIP_EHIP, "probe failed: %s", hipGetErrorString(e));
    return ECLIP_OK;
}

extern "C" eclip_status eclip_pool_probe_graph(eclip_pool *pool, uint32_t mask_id, uint32_t n_blocks, uint32_t *out)
{
    if (!pool || !out) return fail(ECLIP_EINVAL, "null argument");
    if (mask_id >= pool->streams.size()) return fail(ECLIP_EINVAL, "unknown mask id %u", mask_id);
    if (n_blocks == 0 || n_blocks > 65536) return fail(ECLIP_EINVAL, "n_blocks must be 1..65536");
    HIP_TRY(hipSetDevice(pool->device));
    uint32_t *d = nullptr;
    HIP_TRY(hipMalloc(&d, (size_t)n_blocks * 4));
    hipStream_t s = pool->streams[mask_id].stream;
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    hipError_t e = hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal);
    if (e == hipSuccess) {
        const hipError_t le = launch_probe(d, (int)n_blocks, s);
        e = hipStreamEndCapture(s, &graph);
        if (le != hipSuccess) e = le;
    }
    if (e == hipSuccess) e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    if (e == hipSuccess) e = hipGraphLaunch(exec, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e == hipSuccess) e = hipMemcpy(out, d, (size_t)n_blocks * 4, hipMemcpyDeviceToHost);
    if (exec) (void)hipGraphExecDestroy(exec);
    if (graph) (void)hipGraphDestroy(graph);
    (void)hipFree(d);
    if (e != hipSuccess) return fail(ECLIP_EHIP, "graph probe failed: %s", hipGetErrorString(e));
    return ECLIP_OK;
}

// ------------------------------------------------------------------------------------------------
// model
// ------------------------------------------------------------------------------------------------
static const size_t NONE = (size_t)-1;

struct Dims { int kind, c, h, w; };   // c as stored (the network input's channels may be padded)

struct LayerPlan {
    eclip_layer L;
    Dims in, out;
    int in_c_logical = 0;      // channels of the input before padding
    size_t out_off = 0;        // byte offset of this layer's output in the activation arena
    size_t w_dev = NONE, b_dev = NONE, g_dev = NONE, be_dev = NONE;   // byte offsets in the device weight arena
    bool gemm = false;         // runs on the matrix-core GEMM kernel
    int gc_super = 0;          // grouped CONV on the matrix cores: groups per super-group (0: the direct kernel)
    // Concatenation in place: the output of a layer may be a channel range of another layer's (wider) buffer.
    int buf = -1;              // layer whose arena buffer holds this layer's output (itself unless in place)
    int ld = 0;                // channels between consecutive pixels of that buffer (0: this layer's own channel count)
    int c_off = 0;             // first channel of this layer's output in it
    bool concat_copy = false;  // CONCAT in place, head of a chain: the first operand is copied into the buffer, the second is there
    bool concat_noop = false;  // CONCAT in place whose operands are both already in the buffer: nothing to launch
    // Channel shuffle folded into weights: the SHUFFLE layer launches nothing and its readers' weights are permuted at load.
    bool shuffle_noop = false;
    int perm_groups = 0;       // > 0: this layer's input arrives NOT shuffled; its weights are laid out for that order
    bool pair_next = false;    // this layer and the next are independent GEMM layers of one group: one launch may carry both
    bool gapfc_next = false;   // global average pool whose only reader is the linear layer that follows: one launch may do both
};

struct eclip_req {
    eclip_model *model = nullptr;
    hipEvent_t done = nullptr;                       // completion only (no timestamps): what eclip_wait blocks on
    hipEvent_t t_start = nullptr, t_done = nullptr;  // timestamped pair, recorded only while the model's timing is on
    bool pending = false, timed = false;
    uint32_t n_kernels = 0, n_switches = 0;
};

struct eclip_model {
    eclip_pool *pool = nullptr;
    int dtype = 0, esize = 2;
    int in_kind = 0, in_c = 0, in_h = 0, in_w = 0, in_cp = 0;
    uint32_t max_batch = 1;
    std::vector<LayerPlan> layers;
    std::vector<uint32_t> group_of_layer;
    uint32_t n_groups = 0;
    std::vector<uint32_t> mask_of_group;
    bool has_alloc = false;
    bool stem_direct = false;      // layer 0 is the only reader of an IMAGE input of <= 4 channels and a matrix-core convolution:
                                   // it may read the caller's tensor itself instead of the channels-last copy

    char *d_weights = nullptr;
    char *d_act = nullptr;
    char *d_in_stage = nullptr;    // channels-last copy of an IMAGE input
    float *d_ws = nullptr;
    float *ws = nullptr;           // workspace the launches use: d_ws, or the device's static scratch for the duration of
                                   // an eclip_submit_static call
    size_t ws_floats = 0;
    bool timing = false;           // requests record timing events (eclip_model_timing)
    // Captured requests (eclip_model_graphs): a request is cut into segments, one per run of kernel groups on the same
    // pooled stream; each segment is a HIP graph captured once and replayed on that stream.  An entry is good for one
    // (input buffer, output buffer, batch, workspace) under the table and plans it was captured with (`stamp`).
    struct GraphSeg { hipGraphExec_t exec; uint32_t mask_id; uint32_t first_group; };
    struct GraphEntry {
        const void *d_in; void *d_out; uint32_t batch; float *ws; uint64_t stamp, last_use;
        uint32_t n_kernels;
        std::vector<GraphSeg> segs;
    };
    bool use_graphs = false;
    hipStream_t capture_stream = nullptr;  // private to the model: requests are captured here and replayed on pooled streams
    uint64_t stamp = 1, use_clock = 0;     // stamp changes whenever the table, the pool or the plans change
    std::vector<GraphEntry> graphs;
    // plans chosen by measurement (eclip_model_tune), keyed by (M, N, K, CUs of the stream); the cost model decides the rest
    std::map<std::array<long, 4>, GemmPlan> tuned;
    void *d_self_in = nullptr;     // zero input / scratch output for profiling
    float *d_self_out = nullptr;

    std::vector<eclip_req> reqs;
    std::vector<hipEvent_t> switch_events;
    HopSignal hops;                     // cross-stream dependencies at group boundaries that change stream
    hipEvent_t last_done = nullptr;     // done event of the most recent request (owned by its req)
    hipStream_t last_stream = nullptr;
    uint32_t inflight = 0;
    std::mutex mu;
};

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static int elem_size(int dtype) { return dtype == ECLIP_F32 ? 4 : 2; }

static size_t out_elems(const eclip_model *m) {
    const Dims &d = m->layers.back().out;
    return (size_t)d.c * d.h * d.w;
}
static size_t in_elems(const eclip_model *m) {
    if (m->in_kind == ECLIP_IN_TOKENS) return (size_t)m->in_w;
    return (size_t)m->in_c * m->in_h * m->in_w;
}

static void drop_graphs(eclip_model *m)
{
    for (auto &g : m->graphs)
        for (auto &sg : g.segs)
            if (sg.exec) (void)hipGraphExecDestroy(sg.exec);
    m->graphs.clear();
}

static void free_model(eclip_model *m)
{
    if (!m) return;
    drop_graphs(m);
    if (m->capture_stream) (void)hipStreamDestroy(m->capture_stream);
    (void)hipFree(m->d_weights);
    (void)hipFree(m->d_act);
    (void)hipFree(m->d_in_stage);
    (void)hipFree(m->d_ws);
    (void)hipFree(m->d_self_in);
    (void)hipFree(m->d_self_out);
    for (eclip_req &r : m->reqs) {
        if (r.done) (void)hipEventDestroy(r.done);
        if (r.t_start) (void)hipEventDestroy(r.t_start);
        if (r.t_done) (void)hipEventDestroy(r.t_done);
    }
    for (hipEvent_t e : m->switch_events)
        if (e) (void)hipEventDestroy(e);
    m->hops.release();
    delete m;
}

// Validates the descriptor and fills the per-layer plans (shapes only).  No HIP call.
static eclip_status plan_model(const eclip_model_desc *d, size_t weight_elems, eclip_model *m)
{
    if (d->dtype < ECLIP_F32 || d->dtype > ECLIP_F16) return fail(ECLIP_EINVAL, "unknown dtype %d", d->dtype);
    if (d->in_kind < ECLIP_IN_IMAGE || d->in_kind > ECLIP_IN_VEC) return fail(ECLIP_EINVAL, "unknown input kind %d", d->in_kind);
    if (!d->layers || d->n_layers == 0) return fail(ECLIP_EINVAL, "model has no layers");
    if (d->n_layers > 4096) return fail(ECLIP_ELIMIT, "more than 4096 layers");
    if (!d->group_of_layer || d->n_groups == 0) return fail(ECLIP_EINVAL, "no kernel-group partition");
    if (d->max_batch == 0 || d->max_inflight == 0) return fail(ECLIP_EINVAL, "max_batch and max_inflight must be >= 1");
    if (d->max_inflight > 1024) return fail(ECLIP_ELIMIT, "max_inflight above 1024");
    if (d->in_c <= 0 || d->in_h <= 0 || d->in_w <= 0) return fail(ECLIP_EINVAL, "non-positive input dims");
    if (d->group_of_layer[0] != 0) return fail(ECLIP_EINVAL, "group_of_layer must start at 0");
    for (uint32_t i = 1; i < d->n_layers; ++i) {
        const uint32_t a = d->group_of_layer[i - 1], b = d->group_of_layer[i];
        if (b != a && b != a + 1) return fail(ECLIP_EINVAL, "group_of_layer not non-decreasing in steps of one at layer %u", i);
    }
    if (d->group_of_layer[d->n_layers - 1] != d->n_groups - 1) return fail(ECLIP_EINVAL, "group_of_layer does not end at n_groups-1");

    const bool f32 = d->dtype == ECLIP_F32;
    m->dtype = d->dtype;
    m->esize = elem_size(d->dtype);
    m->in_kind = d->in_kind; m->in_c = d->in_c; m->in_h = d->in_h; m->in_w = d->in_w;
    // a 16-bit image input is staged with its channel count rounded up to 8 when a matrix-core layer reads it
    bool gemm_reads_input = false;
    for (uint32_t i = 0; i < d->n_layers; ++i) {
        const eclip_layer &L = d->layers[i];
        if (L.in0 == -1 && ((L.op == ECLIP_OP_CONV && L.groups == 1) || L.op == ECLIP_OP_LINEAR)) gemm_reads_input = true;
    }
    m->in_cp = (d->in_kind == ECLIP_IN_IMAGE && !f32 && gemm_reads_input) ? (int)align_up((size_t)d->in_c, 8) : d->in_c;
    m->max_batch = d->max_batch;
    m->n_groups = d->n_groups;
    m->group_of_layer.assign(d->group_of_layer, d->group_of_layer + d->n_layers);
    m->layers.resize(d->n_layers);

    Dims in_dims;
    if (d->in_kind == ECLIP_IN_IMAGE) in_dims = Dims{ECLIP_KIND_IMAGE, m->in_cp, d->in_h, d->in_w};
    else if (d->in_kind == ECLIP_IN_VEC) {
        if (d->in_h != 1 || d->in_w != 1) return fail(ECLIP_EINVAL, "VEC input needs h = w = 1");
        in_dims = Dims{ECLIP_KIND_VEC, d->in_c, 1, 1};
    } else {
        if (d->in_h != 1) return fail(ECLIP_EINVAL, "SEQ/TOKENS input needs h = 1");
        in_dims = Dims{ECLIP_KIND_SEQ, d->in_c, 1, d->in_w};
    }
    auto check_off = [&](int64_t off, size_t n, const char *what, uint32_t i) -> eclip_status {
        if (off < 0 || (size_t)off + n > weight_elems)
            return fail(ECLIP_EINVAL, "layer %u: %s offset %lld (+%zu) outside the weight blob of %zu elements", i, what, (long long)off, n, weight_elems);
        return ECLIP_OK;
    };
    for (uint32_t i = 0; i < d->n_layers; ++i) {
        const eclip_layer &L = d->layers[i];
        LayerPlan &P = m->layers[i];
        P.L = L;
        if (L.in0 < -1 || L.in0 >= (int)i) return fail(ECLIP_EINVAL, "layer %u: in0 = %d is not an earlier layer", i, L.in0);
        if (L.in1 != -2 && (L.in1 < -1 || L.in1 >= (int)i)) return fail(ECLIP_EINVAL, "layer %u: in1 = %d is not an earlier layer", i, L.in1);
        if (L.in0 == -1 && d->in_kind == ECLIP_IN_TOKENS && L.op != ECLIP_OP_EMBED)
            return fail(ECLIP_EINVAL, "layer %u: only EMBED may read token ids", i);
        const Dims in = L.in0 == -1 ? in_dims : m->layers[L.in0].out;
        P.in = in;
        P.in_c_logical = (L.in0 == -1 && d->in_kind == ECLIP_IN_IMAGE) ? d->in_c : in.c;
        P.buf = (int)i;
        Dims out{L.kind, L.c, L.h, L.w};
        if (L.c <= 0 || L.h <= 0 || L.w <= 0) return fail(ECLIP_EINVAL, "layer %u: non-positive output dims", i);
        if (L.act < ECLIP_ACT_NONE || L.act > ECLIP_ACT_GELU) return fail(ECLIP_EINVAL, "layer %u: unknown activation %d", i, L.act);
        eclip_status st;
        switch (L.op) {
        case ECLIP_OP_CONV: {
            if (in.kind != ECLIP_KIND_IMAGE || L.kind != ECLIP_KIND_IMAGE) return fail(ECLIP_EINVAL, "layer %u: CONV needs IMAGE input and output", i);
            if (L.kh <= 0 || L.kw <= 0 || L.stride <= 0 || L.pad < 0) return fail(ECLIP_EINVAL, "layer %u: bad conv geometry", i);
            if (in.h + 2 * L.pad < L.kh || in.w + 2 * L.pad < L.kw) return fail(ECLIP_EINVAL, "layer %u: kernel larger than padded input", i);
            const int ho = (in.h + 2 * L.pad - L.kh) / L.stride + 1, wo = (in.w + 2 * L.pad - L.kw) / L.stride + 1;
            if (L.h != ho || L.w != wo) return fail(ECLIP_EINVAL, "layer %u: CONV output %dx%d declared, %dx%d expected", i, L.h, L.w, ho, wo);
            if (L.groups < 1 || P.in_c_logical % L.groups || L.c % L.groups)
                return fail(ECLIP_EINVAL, "layer %u: groups must divide both channel counts", i);
            const bool dw = L.groups > 1 && L.groups == P.in_c_logical && L.c == L.groups;     // depthwise kernel
            const bool grouped = L.groups > 1 && !dw;                                            // direct grouped kernel
            if (L.groups > 1 && in.c != P.in_c_logical) return fail(ECLIP_EINVAL, "layer %u: grouped CONV directly on a channel-padded network input is not supported", i);
            if (grouped && f32) return fail(ECLIP_EINVAL, "layer %u: grouped CONV (1 < groups < channels) needs a 16-bit model", i);
            if ((st = check_off(L.w_off, (size_t)L.c * (P.in_c_logical / L.groups) * L.kh * L.kw, "weight", i))) return st;
            if (L.b_off >= 0 && (st = check_off(L.b_off, L.c, "bias", i))) return st;
            if (!f32 && L.groups == 1 && in.c % 8) return fail(ECLIP_EINVAL, "layer %u: 16-bit CONV needs an input channel count that is a multiple of 8 (got %d)", i, in.c);
            P.gemm = !f32 && L.groups == 1;
            if (grouped && !getenv("ECLIP_GCONV_DIRECT")) {
                int S = 0;
                if (gconv_mfma_pick(L.groups, P.in_c_logical / L.groups, L.c / L.groups, &S)) P.gc_super = S;
            }
            break;
        }
        case ECLIP_OP_LINEAR: {
            const bool seq = in.kind == ECLIP_KIND_SEQ;
            if (seq) { if (L.kind != ECLIP_KIND_SEQ || L.h != 1 || L.w != in.w) return fail(ECLIP_EINVAL, "layer %u: LINEAR on a sequence keeps [S] (w)", i); }
            else if (L.kind != ECLIP_KIND_VEC || L.h != 1 || L.w != 1) return fail(ECLIP_EINVAL, "layer %u: LINEAR on an image/vector yields a VEC", i);
            const size_t k_logical = seq ? (size_t)in.c : (size_t)P.in_c_logical * in.h * in.w;
            if ((st = check_off(L.w_off, (size_t)L.c * k_logical, "weight", i))) return st;
            if (L.b_off >= 0 && (st = check_off(L.b_off, L.c, "bias", i))) return st;
            if (!f32 && in.c % 8) return fail(ECLIP_EINVAL, "layer %u: 16-bit LINEAR needs an input channel count that is a multiple of 8 (got %d)", i, in.c);
            P.gemm = !f32;
            break;
        }
        case ECLIP_OP_MAXPOOL: {
            if (in.kind != ECLIP_KIND_IMAGE || L.kind != ECLIP_KIND_IMAGE) return fail(ECLIP_EINVAL, "layer %u: MAXPOOL needs IMAGE tensors", i);
            if (L.kh <= 0 || L.kw <= 0 || L.stride <= 0 || L.pad < 0 || 2 * L.pad > std::min(L.kh, L.kw))
                return fail(ECLIP_EINVAL, "layer %u: bad pooling geometry", i);
            if (in.h + 2 * L.pad < L.kh || in.w + 2 * L.pad < L.kw) return fail(ECLIP_EINVAL, "layer %u: window larger than padded input", i);
            const int ho = (in.h + 2 * L.pad - L.kh) / L.stride + 1, wo = (in.w + 2 * L.pad - L.kw) / L.stride + 1;
            if (L.h != ho || L.w != wo || L.c != in.c) return fail(ECLIP_EINVAL, "layer %u: MAXPOOL output dims mismatch", i);
            if (in.c != P.in_c_logical) return fail(ECLIP_EINVAL, "layer %u: MAXPOOL directly on a channel-padded network input is not supported", i);
            break;
        }
        case ECLIP_OP_GAP:
            if (in.kind != ECLIP_KIND_IMAGE || L.kind != ECLIP_KIND_VEC || L.c != in.c || L.h != 1 || L.w != 1)
                return fail(ECLIP_EINVAL, "layer %u: GAP maps IMAGE [C,H,W] to VEC [C]", i);
            if (in.c != P.in_c_logical) return fail(ECLIP_EINVAL, "layer %u: GAP directly on a channel-padded network input is not supported", i);
            break;
        case ECLIP_OP_LAYERNORM:
        case ECLIP_OP_SOFTMAX: {
            if (in.kind == ECLIP_KIND_IMAGE) return fail(ECLIP_EINVAL, "layer %u: row operators need SEQ or VEC tensors", i);
            if (L.kind != in.kind || L.c != in.c || L.h != in.h || L.w != in.w) return fail(ECLIP_EINVAL, "layer %u: row operator changes shape", i);
            const int v = f32 ? (in.c % 4 ? 1 : 4) : (in.c % 8 ? 1 : 8);
            if ((in.c / v + 63) / 64 > 16) return fail(ECLIP_EINVAL, "layer %u: row of %d elements exceeds the kernel's register budget", i, in.c);
            if (L.op == ECLIP_OP_LAYERNORM) {
                if (L.g_off >= 0 && (st = check_off(L.g_off, L.c, "gamma", i))) return st;
                if (L.be_off >= 0 && (st = check_off(L.be_off, L.c, "beta", i))) return st;
                if (!(L.eps >= 0.0f)) return fail(ECLIP_EINVAL, "layer %u: negative eps", i);
            }
            break;
        }
        case ECLIP_OP_ATTENTION: {
            if (f32) return fail(ECLIP_EINVAL, "layer %u: ATTENTION needs a 16-bit model", i);
            if (in.kind != ECLIP_KIND_SEQ || L.kind != ECLIP_KIND_SEQ || in.c % 3 || L.c != in.c / 3 || L.w != in.w || L.h != 1)
                return fail(ECLIP_EINVAL, "layer %u: ATTENTION maps SEQ [S,3*Hd] to SEQ [S,Hd]", i);
            if (L.heads <= 0 || L.c % L.heads) return fail(ECLIP_EINVAL, "layer %u: heads must divide the hidden size", i);
            const int dh = L.c / L.heads;
            if (dh != 32 && dh != 64) return fail(ECLIP_EINVAL, "layer %u: head size %d not supported (32 or 64)", i, dh);
            if (in.w > 512) return fail(ECLIP_EINVAL, "layer %u: sequence length %d above 512", i, in.w);
            break;
        }
        case ECLIP_OP_EMBED: {
            if (L.in0 != -1 || d->in_kind != ECLIP_IN_TOKENS) return fail(ECLIP_EINVAL, "layer %u: EMBED reads the token-id input", i);
            if (L.kind != ECLIP_KIND_SEQ || L.h != 1 || L.w != d->in_w || L.c != d->in_c) return fail(ECLIP_EINVAL, "layer %u: EMBED output must be SEQ [S,Hd]", i);
            if (L.aux0 <= 0 || L.aux1 < d->in_w) return fail(ECLIP_EINVAL, "layer %u: EMBED needs vocab > 0 and at least S positions", i);
            if ((st = check_off(L.w_off, (size_t)L.aux0 * L.c, "token table", i))) return st;
            if ((st = check_off(L.g_off, (size_t)L.aux1 * L.c, "position table", i))) return st;
            if ((st = check_off(L.be_off, (size_t)2 * L.c, "type table", i))) return st;
            break;
        }
        case ECLIP_OP_ELTWISE:
            if (L.kind != in.kind || L.c != in.c || L.h != in.h || L.w != in.w) return fail(ECLIP_EINVAL, "layer %u: ELTWISE changes shape", i);
            if (in.c != P.in_c_logical) return fail(ECLIP_EINVAL, "layer %u: ELTWISE directly on a channel-padded network input is not supported", i);
            if (L.b_off >= 0 && (st = check_off(L.b_off, L.c, "bias", i))) return st;
            break;
        case ECLIP_OP_CONCAT: {
            if (L.in1 == -2) return fail(ECLIP_EINVAL, "layer %u: CONCAT needs two inputs", i);
            if (L.in1 == -1 && d->in_kind == ECLIP_IN_TOKENS) return fail(ECLIP_EINVAL, "layer %u: token ids cannot be concatenated", i);
            const Dims r = L.in1 == -1 ? in_dims : m->layers[L.in1].out;
            if (r.kind != in.kind || r.h != in.h || r.w != in.w) return fail(ECLIP_EINVAL, "layer %u: CONCAT inputs differ in shape", i);
            if (L.kind != in.kind || L.h != in.h || L.w != in.w || L.c != in.c + r.c) return fail(ECLIP_EINVAL, "layer %u: CONCAT output must have the summed channel count", i);
            if (in.c != P.in_c_logical || (L.in1 == -1 && d->in_kind == ECLIP_IN_IMAGE && in_dims.c != (int)d->in_c))
                return fail(ECLIP_EINVAL, "layer %u: CONCAT directly on a channel-padded network input is not supported", i);
            break;
        }
        case ECLIP_OP_SHUFFLE:
            if (L.kind != in.kind || L.c != in.c || L.h != in.h || L.w != in.w) return fail(ECLIP_EINVAL, "layer %u: SHUFFLE changes shape", i);
            if (L.groups < 1 || L.c % L.groups) return fail(ECLIP_EINVAL, "layer %u: SHUFFLE groups must divide the channel count", i);
            if (in.c != P.in_c_logical) return fail(ECLIP_EINVAL, "layer %u: SHUFFLE directly on a channel-padded network input is not supported", i);
            break;
        default:
            return fail(ECLIP_EINVAL, "layer %u: unknown op %d", i, L.op);
        }
        if (L.in1 != -2 && L.op != ECLIP_OP_CONCAT) {
            if (L.op == ECLIP_OP_SHUFFLE || L.op == ECLIP_OP_MAXPOOL || L.op == ECLIP_OP_GAP || L.op == ECLIP_OP_SOFTMAX || L.op == ECLIP_OP_ATTENTION || L.op == ECLIP_OP_EMBED)
                return fail(ECLIP_EINVAL, "layer %u: this op takes no second input", i);
            if (L.in1 == -1 && d->in_kind == ECLIP_IN_TOKENS) return fail(ECLIP_EINVAL, "layer %u: token ids cannot be a residual", i);
            const Dims r = L.in1 == -1 ? in_dims : m->layers[L.in1].out;
            if (r.kind != out.kind || r.c != out.c || r.h != out.h || r.w != out.w)
                return fail(ECLIP_EINVAL, "layer %u: residual input shape differs from the output shape", i);
        }
        if ((size_t)out.c * out.h * out.w * d->max_batch >= ((size_t)1 << 30)) return fail(ECLIP_ELIMIT, "layer %u: tensor of 2^30 elements or more", i);
        P.out = out;
    }
    // Horizontal fusion candidates: consecutive matrix-core layers of one kernel group, the second not reading the
    // first (e.g. the projection shortcut and the first convolution of a residual block), neither being the last
    // layer (whose output goes to the caller).
    for (uint32_t i = 0; i + 2 < d->n_layers; ++i) {
        LayerPlan &A = m->layers[i];
        const LayerPlan &B = m->layers[i + 1];
        A.pair_next = A.gemm && B.gemm && d->group_of_layer[i] == d->group_of_layer[i + 1] && B.L.in0 != (int)i && B.L.in1 != (int)i;
    }
    {
        const LayerPlan &S = m->layers[0];
        bool only_reader = true;
        for (uint32_t j = 1; j < d->n_layers; ++j) only_reader &= m->layers[j].L.in0 != -1 && m->layers[j].L.in1 != -1;
        m->stem_direct = d->in_kind == ECLIP_IN_IMAGE && d->in_c <= 4 && m->in_cp == 8 && S.L.op == ECLIP_OP_CONV && S.gemm &&
                         S.L.in0 == -1 && S.L.in1 != -1 && only_reader && d->n_layers > 1;
    }
    // Pool + classifier candidates: a GAP layer read only by the matrix-core linear layer right after it, same group,
    // the linear layer taking no second operand.  Whether the fused kernel pays depends on the batch (decided per request).
    for (uint32_t i = 0; i + 1 < d->n_layers; ++i) {
        LayerPlan &A = m->layers[i];
        const LayerPlan &B = m->layers[i + 1];
        if (A.L.op != ECLIP_OP_GAP || B.L.op != ECLIP_OP_LINEAR || !B.gemm || B.L.in0 != (int)i || B.L.in1 >= 0) continue;
        if (d->group_of_layer[i] != d->group_of_layer[i + 1] || B.in.kind == ECLIP_KIND_IMAGE) continue;
        bool other_reader = false;
        for (uint32_t j = i + 2; j < d->n_layers; ++j) other_reader |= m->layers[j].L.in0 == (int)i || m->layers[j].L.in1 == (int)i;
        A.gapfc_next = !other_reader;
    }
    // Concatenation in place (DenseNet-style blocks: y = concat(x, f(x)), again and again).  Copying makes the block
    // quadratic in traffic and costs a launch per layer.  Instead a chain of concatenations shares ONE buffer with the
    // channel count of the last of them: the matrix-core convolution that produces a second operand writes its channels
    // straight into its range of that buffer (row pitch = the buffer's channel count), every earlier concatenation of
    // the chain is the buffer's first channels, read with that pitch, and the CONCAT layers themselves launch nothing,
    // except the head of a chain, which copies its first operand in.  Conditions, all checked here: 16-bit model; the
    // second operand comes from a matrix-core CONV without residual that nobody else reads; channel counts are multiples
    // of 8; and a concatenation that is not the last of its chain is read only by the next concatenation (as its first
    // operand) and by matrix-core convolutions (as their input), the two readers that know about the pitch.
    if (m->dtype != ECLIP_F32 && !getenv("ECLIP_CONCAT_COPY")) {
        const int n = (int)d->n_layers;
        std::vector<std::vector<int>> readers(n);
        for (int j = 0; j < n; ++j) {
            const eclip_layer &L = m->layers[j].L;
            if (L.in0 >= 0) readers[L.in0].push_back(j);
            if (L.in1 >= 0 && L.in1 != L.in0) readers[L.in1].push_back(j);
        }
        std::vector<int> chain(n, -1);
        std::vector<char> extended(n, 0);
        for (int i = 0; i < n; ++i) {
            LayerPlan &C = m->layers[i];
            if (C.L.op != ECLIP_OP_CONCAT) continue;
            const int a = C.L.in0, b = C.L.in1;
            if (a < 0 || b < 0 || a == b) continue;
            const LayerPlan &B = m->layers[b];
            if (B.L.op != ECLIP_OP_CONV || !B.gemm || B.L.in1 != -2 || readers[b].size() != 1 || b == n - 1) continue;
            if (C.in.c % 8 || B.out.c % 8) continue;
            bool extend = m->layers[a].L.op == ECLIP_OP_CONCAT && chain[a] >= 0 && !extended[a];
            if (extend)
                for (int r : readers[a]) {
                    const LayerPlan &R = m->layers[r];
                    const bool next_concat = r == i;
                    const bool conv_input = R.L.op == ECLIP_OP_CONV && R.gemm && R.L.in0 == a && R.L.in1 != a;
                    extend &= next_concat || conv_input;
                }
            chain[i] = extend ? chain[a] : i;
            if (extend) extended[a] = 1;
            C.concat_noop = extend;
            C.concat_copy = !extend;
        }
        for (int i = n - 1; i >= 0; --i) {
            if (chain[i] < 0) continue;
            int last = i;                                       // the last concatenation of this layer's chain owns the buffer
            for (int j = n - 1; j > i; --j)
                if (chain[j] == chain[i]) { last = j; break; }
            const int ld = m->layers[last].out.c;
            LayerPlan &C = m->layers[i];
            C.buf = last;
            C.ld = i == last ? 0 : ld;
            LayerPlan &B = m->layers[C.L.in1];
            B.buf = last;
            B.ld = ld;
            B.c_off = C.in.c;
        }
    }
    // Channel shuffle folded into weights (ShuffleNet-style units: grouped 1x1 -> shuffle -> depthwise -> grouped 1x1).
    // A shuffle is a fixed permutation of channels, y[j] = x[s(j)].  A depthwise convolution treats channels one by one,
    // so dw(shuffle(x)) = shuffle(dw'(x)) with dw' = dw with its per-channel filters permuted; and a convolution that sums
    // over ALL of its input channels (dense, or grouped with every group inside one super-group of the matrix-core
    // kernel, whose weight block is stored dense anyway) absorbs a permutation of its input into the order of its weight
    // columns.  So when a SHUFFLE is read only by a depthwise CONV (no residual) that is read only by such a convolution,
    // the two filters are permuted once at load and the SHUFFLE layer is its input, untouched: no launch, no traffic.
    if (m->dtype != ECLIP_F32 && !getenv("ECLIP_SHUFFLE_KERNEL")) {
        const int n = (int)d->n_layers;
        auto readers_of = [&](int idx, int *only) {
            int cnt = 0;
            for (int j = 0; j < n; ++j)
                if (m->layers[j].L.in0 == idx || m->layers[j].L.in1 == idx) { ++cnt; *only = j; }
            return cnt;
        };
        for (int i = 0; i + 2 < n; ++i) {
            LayerPlan &S = m->layers[i];
            if (S.L.op != ECLIP_OP_SHUFFLE || S.L.in0 < 0 || S.L.groups < 2) continue;
            const LayerPlan &A = m->layers[S.L.in0];
            if (A.buf != S.L.in0 || A.ld) continue;                        // the input is a plain tensor of its own
            int dwi = -1, g2 = -1;
            if (readers_of(i, &dwi) != 1) continue;
            LayerPlan &D = m->layers[dwi];
            const bool is_dw = D.L.op == ECLIP_OP_CONV && D.L.groups > 1 && D.L.groups == D.in.c && D.L.c == D.L.groups;
            if (!is_dw || D.L.in0 != i || D.L.in1 != -2 || dwi == n - 1) continue;
            if (readers_of(dwi, &g2) != 1) continue;
            LayerPlan &Gc = m->layers[g2];
            if (Gc.L.op != ECLIP_OP_CONV || Gc.L.in0 != dwi || Gc.L.in1 == dwi) continue;
            const bool dense = Gc.gemm && Gc.L.groups == 1;
            const bool grouped = Gc.L.groups > 1 && !(Gc.L.groups == Gc.in.c && Gc.L.c == Gc.L.groups);
            const bool one_super_group = grouped && Gc.L.groups <= 16 && Gc.in.c % 32 == 0 && Gc.L.c % 16 == 0 && !getenv("ECLIP_GCONV_DIRECT");
            if (!dense && !one_super_group) continue;
            if (one_super_group) Gc.gc_super = Gc.L.groups;
            S.shuffle_noop = true;
            S.buf = S.L.in0;
            D.perm_groups = S.L.groups;
            Gc.perm_groups = S.L.groups;
        }
    }
    return ECLIP_OK;
}

// Converts one 16-bit or 32-bit element array; helpers for the weight re-layout (host side).
static void put(std::vector<char> &arena, size_t &cursor, const void *src, size_t bytes, size_t *off_out)
{
    cursor = align_up(cursor, 256);
    if (arena.size() < cursor + bytes) arena.resize(cursor + bytes);
    if (src) memcpy(arena.data() + cursor, src, bytes);
    *off_out = cursor;
    cursor += bytes;
}

template <typename E>
static void relayout_weights(eclip_model *m, const E *w, std::vector<char> &arena, size_t &cursor)
{
    const bool f32 = m->dtype == ECLIP_F32;
    for (LayerPlan &P : m->layers) {
        const eclip_layer &L = P.L;
        const size_t es = sizeof(E);
        if (L.op == ECLIP_OP_CONV || L.op == ECLIP_OP_LINEAR) {
            // logical [cout][cin_g][kh][kw]; a LINEAR on an image is a convolution whose window is the image
            int kh = L.kh, kw = L.kw;
            const int cin_l = P.in_c_logical, cin_s = P.in.c;
            if (L.op == ECLIP_OP_LINEAR) { kh = (P.in.kind == ECLIP_KIND_IMAGE) ? P.in.h : 1; kw = (P.in.kind == ECLIP_KIND_IMAGE) ? P.in.w : 1; }
            const bool dw = L.op == ECLIP_OP_CONV && L.groups > 1 && L.groups == cin_l && L.c == L.groups;
            const bool grouped = L.op == ECLIP_OP_CONV && L.groups > 1 && !dw;
            const E *src = w + L.w_off;
            // input channel i of this layer, as it arrives, is channel unshuf(i) of the tensor the weights were made for
            // (identity unless a channel shuffle in front of the layer was folded away: shuffled[j] = x[(j % G)(c/G) + j/G])
            const int pg = P.perm_groups, pcg = pg ? cin_l / pg : 1;
            auto unshuf = [&](int i) { return pg ? (i % pcg) * pg + i / pcg : i; };
            if (grouped && P.gc_super) {
                // Block-diagonal dense weights of every super-group (gc_super neighbouring groups), in the 1 KB blocks of
                // 16 output channels x 32 k that the matrix instruction consumes: block (sg, nb, t) at
                // ((sg * NB + nb) * KT + t) KB with t = tap * (SI / 32) + kb; lane l of a block owns
                // W[16 nb + (l & 15)][32 kb + 8 (l >> 4) .. +7] of the super-group's SO x SI block of that tap, which is
                // zero wherever output and input channel belong to different groups.
                const int cig = cin_l / L.groups, cog = L.c / L.groups, S = P.gc_super;
                const size_t SI = (size_t)S * cig, SO = (size_t)S * cog, n_sg = (size_t)L.groups / S;
                const size_t KBS = SI / 32, NB = SO / 16, KT = (size_t)kh * kw * KBS;
                size_t off;
                put(arena, cursor, nullptr, n_sg * NB * KT * 512 * es, &off);
                E *dst = reinterpret_cast<E *>(arena.data() + off);
                memset(dst, 0, n_sg * NB * KT * 512 * es);
                for (size_t sg = 0; sg < n_sg; ++sg)
                    for (size_t nb = 0; nb < NB; ++nb)
                        for (size_t t = 0; t < KT; ++t)
                            for (int l = 0; l < 64; ++l) {
                                const size_t tap = t / KBS, kb = t % KBS;
                                const size_t n = nb * 16 + (size_t)(l & 15), k0 = kb * 32 + (size_t)(l >> 4) * 8;
                                E *d8 = dst + (((sg * NB + nb) * KT + t) * 64 + (size_t)l) * 8;
                                for (int e = 0; e < 8; ++e) {
                                    const size_t k = k0 + e;
                                    const size_t kk = pg ? (size_t)unshuf((int)k) : k;          // pg: one super-group, k is the layer's channel
                                    if (n / cog != kk / cig) continue;                 // off the diagonal
                                    const size_t co = sg * SO + n, ci = kk % cig;
                                    d8[e] = src[(co * cig + ci) * kh * kw + tap];
                                }
                            }
                P.w_dev = off;
            } else
            if (grouped) {                              // [cout][cig][kh][kw] -> [cout][kh][kw][cig]
                const int cig = cin_l / L.groups;
                std::vector<E> t((size_t)L.c * kh * kw * cig);
                for (int co = 0; co < L.c; ++co)
                    for (int ci = 0; ci < cig; ++ci)
                        for (int i = 0; i < kh * kw; ++i)
                            t[((size_t)co * kh * kw + i) * cig + ci] = src[((size_t)co * cig + ci) * kh * kw + i];
                put(arena, cursor, t.data(), t.size() * es, &P.w_dev);
            } else
            if (dw) {                                   // -> [kh][kw][c]
                std::vector<E> t((size_t)kh * kw * L.c);
                for (int c = 0; c < L.c; ++c)
                    for (int i = 0; i < kh * kw; ++i) t[(size_t)i * L.c + c] = src[(size_t)unshuf(c) * kh * kw + i];
                put(arena, cursor, t.data(), t.size() * es, &P.w_dev);
            } else if (f32) {                           // -> [kh][kw][cin][cout]
                std::vector<E> t((size_t)kh * kw * cin_s * L.c);
                for (int co = 0; co < L.c; ++co)
                    for (int ci = 0; ci < cin_l; ++ci)
                        for (int i = 0; i < kh * kw; ++i)
                            t[((size_t)i * cin_s + ci) * L.c + co] = src[((size_t)co * cin_l + ci) * kh * kw + i];
                put(arena, cursor, t.data(), t.size() * es, &P.w_dev);
            } else {
                // GEMM operand W[n][k], k = (kh, kw, ci_stored) with padded channels zero, stored in the order the
                // matrix instruction consumes it: blocks of 16 rows x 32 k, block (nb, kb) at ((nb * KB + kb) * 1 KB),
                // and inside a block lane l of a wavefront owns the 16 bytes W[16 nb + (l & 15)][32 kb + 8 (l >> 4) .. +7].
                // A wavefront then fetches one block with one fully contiguous 1 KB load.  N is padded to 16 and K to
                // 32 with zeros.
                const size_t K = (size_t)kh * kw * cin_s;
                const size_t KB = (K + 31) / 32, NB = ((size_t)L.c + 15) / 16;
                std::vector<E> plain((size_t)L.c * K, 0);
                if (kh * kw == 1 && cin_l == cin_s && !pg) {
                    memcpy(plain.data(), src, plain.size() * es);
                } else {
                    for (int co = 0; co < L.c; ++co)
                        for (int ci = 0; ci < cin_l; ++ci)
                            for (int i = 0; i < kh * kw; ++i)
                                plain[(size_t)co * K + (size_t)i * cin_s + ci] = src[((size_t)co * cin_l + unshuf(ci)) * kh * kw + i];
                }
                size_t off;
                put(arena, cursor, nullptr, NB * KB * 512 * es, &off);
                E *dst = reinterpret_cast<E *>(arena.data() + off);
                memset(dst, 0, NB * KB * 512 * es);
                for (size_t nb = 0; nb < NB; ++nb)
                    for (size_t kb = 0; kb < KB; ++kb)
                        for (int l = 0; l < 64; ++l) {
                            const size_t n = nb * 16 + (size_t)(l & 15), k0 = kb * 32 + (size_t)(l >> 4) * 8;
                            if (n >= (size_t)L.c) continue;
                            E *d8 = dst + ((nb * KB + kb) * 64 + (size_t)l) * 8;
                            for (int e = 0; e < 8; ++e)
                                if (k0 + e < K) d8[e] = plain[n * K + k0 + e];
                        }
                P.w_dev = off;
            }
            if (L.b_off >= 0 && dw && pg) {             // a depthwise layer's channels moved with its input's: so does its bias
                std::vector<E> t((size_t)L.c);
                for (int c = 0; c < L.c; ++c) t[c] = w[L.b_off + unshuf(c)];
                put(arena, cursor, t.data(), t.size() * es, &P.b_dev);
            } else if (L.b_off >= 0) put(arena, cursor, w + L.b_off, (size_t)L.c * es, &P.b_dev);
        } else if (L.op == ECLIP_OP_LAYERNORM) {
            if (L.g_off >= 0) put(arena, cursor, w + L.g_off, (size_t)L.c * es, &P.g_dev);
            if (L.be_off >= 0) put(arena, cursor, w + L.be_off, (size_t)L.c * es, &P.be_dev);
        } else if (L.op == ECLIP_OP_EMBED) {
            put(arena, cursor, w + L.w_off, (size_t)L.aux0 * L.c * es, &P.w_dev);
            put(arena, cursor, w + L.g_off, (size_t)L.aux1 * L.c * es, &P.g_dev);
            put(arena, cursor, w + L.be_off, (size_t)2 * L.c * es, &P.be_dev);
        } else if (L.op == ECLIP_OP_ELTWISE) {
            if (L.b_off >= 0) put(arena, cursor, w + L.b_off, (size_t)L.c * es, &P.b_dev);
        }
    }
}

// GEMM view of a CONV / LINEAR layer
struct GemmShape { int B, H, W, Cin, Ho, Wo, Cout, KH, KW, stride, pad; };
static GemmShape gemm_shape(const LayerPlan &P, int batch)
{
    const eclip_layer &L = P.L;
    GemmShape g;
    g.B = batch; g.Cin = P.in.c; g.Cout = L.c;
    if (L.op == ECLIP_OP_CONV) {
        g.H = P.in.h; g.W = P.in.w; g.Ho = L.h; g.Wo = L.w; g.KH = L.kh; g.KW = L.kw; g.stride = L.stride; g.pad = L.pad;
    } else if (P.in.kind == ECLIP_KIND_IMAGE) {
        g.H = P.in.h; g.W = P.in.w; g.Ho = 1; g.Wo = 1; g.KH = P.in.h; g.KW = P.in.w; g.stride = 1; g.pad = 0;
    } else {
        g.H = 1; g.W = P.in.w; g.Ho = 1; g.Wo = P.in.w; g.KH = 1; g.KW = 1; g.stride = 1; g.pad = 0;
    }
    return g;
}

// The launch plan of a matrix-core layer: the measured choice when eclip_model_tune has seen this problem on a stream of
// this CU count, else the planner's cost model.
static GemmPlan plan_of(const eclip_model *m, long M, long N, long K, int n_cu)
{
    if (!m->tuned.empty() && !getenv("ECLIP_GEMM_FORCE")) {
        const auto it = m->tuned.find(std::array<long, 4>{M, N, K, (long)n_cu});
        if (it != m->tuned.end()) return it->second;
    }
    return conv_gemm_plan(M, N, K, n_cu, m->ws_floats);
}

extern "C" eclip_status eclip_model_load(eclip_pool *pool, const eclip_model_desc *desc, const void *weights,
                                         size_t weight_bytes, int weights_on_device, eclip_model **out)
{
    if (!out) return fail(ECLIP_EINVAL, "out is null");
    *out = nullptr;
    if (!desc) return fail(ECLIP_EINVAL, "descriptor is null");
    if (!weights && weight_bytes) return fail(ECLIP_EINVAL, "weights is null");
    eclip_model *m = new (std::nothrow) eclip_model;
    if (!m) return fail(ECLIP_ENOMEM, "out of host memory");
    const int es = (desc->dtype == ECLIP_F32) ? 4 : 2;
    eclip_status st = plan_model(desc, weight_bytes / (size_t)es, m);
    if (st != ECLIP_OK) { delete m; return st; }
    if (!pool) { delete m; return fail(ECLIP_EINVAL, "pool is null"); }
    m->pool = pool;

#define LOAD_TRY(call)                                                                                   \
    do {                                                                                                 \
        hipError_t e_ = (call);                                                                          \
        if (e_ != hipSuccess) {                                                                          \
            free_model(m);                                                                               \
            return fail(e_ == hipErrorOutOfMemory ? ECLIP_ENOMEM : ECLIP_EHIP, "%s failed: %s", #call, hipGetErrorString(e_)); \
        }                                                                                                \
    } while (0)

    LOAD_TRY(hipSetDevice(pool->device));
    // ---- weights: host copy -> re-layout -> device arena
    std::vector<char> host_copy;
    const void *w_host = weights;
    if (weights_on_device) {
        host_copy.resize(weight_bytes);
        LOAD_TRY(hipMemcpy(host_copy.data(), weights, weight_bytes, hipMemcpyDeviceToHost));
        w_host = host_copy.data();
    }
    std::vector<char> arena;
    size_t cursor = 0;
    if (es == 4) relayout_weights<uint32_t>(m, (const uint32_t *)w_host, arena, cursor);
    else relayout_weights<uint16_t>(m, (const uint16_t *)w_host, arena, cursor);
    LOAD_TRY(hipMalloc((void **)&m->d_weights, std::max<size_t>(cursor, 256)));
    if (cursor) LOAD_TRY(hipMemcpy(m->d_weights, arena.data(), cursor, hipMemcpyHostToDevice));
    std::vector<char>().swap(arena);

    // ---- activation arena: one buffer per layer, sized for max_batch
    size_t act = 0;
    for (LayerPlan &P : m->layers) {
        P.out_off = act;
        if (&m->layers[P.buf] != &P) continue;               // in place: lives in another layer's buffer
        act += align_up((size_t)P.out.c * P.out.h * P.out.w * m->max_batch * (size_t)es, 256);
    }
    LOAD_TRY(hipMalloc((void **)&m->d_act, std::max<size_t>(act, 256)));
    if (m->in_kind == ECLIP_IN_IMAGE)
        LOAD_TRY(hipMalloc((void **)&m->d_in_stage, (size_t)m->in_cp * m->in_h * m->in_w * m->max_batch * (size_t)es));

    // ---- split-K workspace: enough for the most demanding GEMM layer at any CU count, capped
    size_t ws = 0;
    for (const LayerPlan &P : m->layers) {
        if (P.L.op == ECLIP_OP_GAP) ws = std::max(ws, (size_t)m->max_batch * 64 * (size_t)P.L.c);
        if (!P.gemm) continue;
        const GemmShape g = gemm_shape(P, (int)m->max_batch);
        const size_t MN = (size_t)g.B * g.Ho * g.Wo * g.Cout;
        const size_t KT = ((size_t)g.KH * g.KW * g.Cin + 63) / 64;
        if (MN <= (size_t)256 * 64 * 64) ws = std::max(ws, MN * std::min<size_t>(32, std::max<size_t>(1, KT / 3)));
        if (KT >= 4 && 2 * MN <= ((size_t)16 << 20)) ws = std::max(ws, 2 * MN);       // K cut in two for mid-size layers
    }
    m->ws_floats = std::min<size_t>(ws, (size_t)16 << 20);
    LOAD_TRY(hipMalloc((void **)&m->d_ws, std::max<size_t>(m->ws_floats * 4, 256)));
    m->ws = m->d_ws;

    // ---- profiling buffers, requests, events
    const size_t in_bytes = in_elems(m) * m->max_batch * (size_t)(m->in_kind == ECLIP_IN_TOKENS ? 4 : es);
    LOAD_TRY(hipMalloc(&m->d_self_in, std::max<size_t>(in_bytes, 256)));
    LOAD_TRY(hipMemset(m->d_self_in, 0, std::max<size_t>(in_bytes, 256)));
    LOAD_TRY(hipMalloc((void **)&m->d_self_out, std::max<size_t>(out_elems(m) * m->max_batch * 4, 256)));
    m->reqs.resize(desc->max_inflight);
    for (eclip_req &r : m->reqs) {
        r.model = m;
        LOAD_TRY(hipEventCreateWithFlags(&r.done, hipEventDisableTiming));
        LOAD_TRY(hipEventCreate(&r.t_start));
        LOAD_TRY(hipEventCreate(&r.t_done));
    }
    m->switch_events.assign(m->n_groups, nullptr);
    for (hipEvent_t &e : m->switch_events) LOAD_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
    LOAD_TRY(m->hops.init(pool->device));
    LOAD_TRY(hipDeviceSynchronize());
#undef LOAD_TRY
    {
        std::lock_guard<std::mutex> lk(pool->mu);
        pool->n_models++;
    }
    *out = m;
    return ECLIP_OK;
}

extern "C" eclip_status eclip_model_free(eclip_model *model)
{
    if (!model) return fail(ECLIP_EINVAL, "model is null");
    {
        std::lock_guard<std::mutex> lk(model->mu);
        if (model->inflight) return fail(ECLIP_ESTATE, "%u requests still in flight", model->inflight);
    }
    eclip_pool *pool = model->pool;
    HIP_TRY(hipSetDevice(pool->device));
    HIP_TRY(hipDeviceSynchronize());
    free_model(model);
    std::lock_guard<std::mutex> lk(pool->mu);
    pool->n_models--;
    return ECLIP_OK;
}

extern "C" eclip_status eclip_model_rebind(eclip_model *model, eclip_pool *new_pool)
{
    if (!model || !new_pool) return fail(ECLIP_EINVAL, "null argument");
    if (new_pool->device != model->pool->device) return fail(ECLIP_EINVAL, "the new pool is on another device");
    std::lock_guard<std::mutex> lk(model->mu);
    if (model->inflight) return fail(ECLIP_ESTATE, "%u requests still in flight", model->inflight);
    HIP_TRY(hipSetDevice(new_pool->device));
    HIP_TRY(hipDeviceSynchronize());
    eclip_pool *old = model->pool;
    if (old != new_pool) {
        { std::lock_guard<std::mutex> l2(old->mu); old->n_models--; }
        { std::lock_guard<std::mutex> l2(new_pool->mu); new_pool->n_models++; }
        model->pool = new_pool;
    }
    model->has_alloc = false;
    model->mask_of_group.clear();
    model->last_done = nullptr;
    model->last_stream = nullptr;
    model->stamp++;
    drop_graphs(model);
    return ECLIP_OK;
}

extern "C" eclip_status eclip_alloc_set(eclip_model *model, const uint32_t *mask_id_of_group, uint32_t n_groups)
{
    if (!model || !mask_id_of_group) return fail(ECLIP_EINVAL, "null argument");
    if (n_groups != model->n_groups) return fail(ECLIP_EINVAL, "table has %u groups, the model %u", n_groups, model->n_groups);
    for (uint32_t g = 0; g < n_groups; ++g)
        if (mask_id_of_group[g] >= model->pool->streams.size())
            return fail(ECLIP_EINVAL, "group %u: unknown mask id %u", g, mask_id_of_group[g]);
    std::lock_guard<std::mutex> lk(model->mu);
    if (!model->has_alloc || !std::equal(model->mask_of_group.begin(), model->mask_of_group.end(), mask_id_of_group)) model->stamp++;
    model->mask_of_group.assign(mask_id_of_group, mask_id_of_group + n_groups);
    model->has_alloc = true;
    return ECLIP_OK;
}

extern "C" eclip_status eclip_model_switches(const eclip_model *model, uint32_t *n_switches)
{
    if (!model || !n_switches) return fail(ECLIP_EINVAL, "null argument");
    if (!model->has_alloc) return fail(ECLIP_ESTATE, "no allocation table installed");
    uint32_t n = 0;
    for (uint32_t g = 1; g < model->n_groups; ++g) n += model->mask_of_group[g] != model->mask_of_group[g - 1];
    *n_switches = n;
    return ECLIP_OK;
}

extern "C" eclip_status eclip_model_group_size(const eclip_model *model, uint32_t group, uint32_t *n_kernels)
{
    if (!model || !n_kernels) return fail(ECLIP_EINVAL, "null argument");
    if (group >= model->n_groups) return fail(ECLIP_EINVAL, "unknown group %u", group);
    *n_kernels = (uint32_t)std::count(model->group_of_layer.begin(), model->group_of_layer.end(), group);
    return ECLIP_OK;
}

extern "C" eclip_status eclip_model_kernel_info(const eclip_model *model, uint32_t layer, uint32_t mask_id, uint32_t batch,
                                                eclip_kernel_info *out)
{
    if (!model || !out) return fail(ECLIP_EINVAL, "null argument");
    if (layer >= model->layers.size()) return fail(ECLIP_EINVAL, "unknown layer %u", layer);
    if (mask_id >= model->pool->streams.size()) return fail(ECLIP_EINVAL, "unknown mask id %u", mask_id);
    if (batch == 0 || batch > model->max_batch) return fail(ECLIP_EINVAL, "batch %u outside 1..%u", batch, model->max_batch);
    const LayerPlan &P = model->layers[layer];
    memset(out, 0, sizeof *out);
    out->launches = 1;
    out->k_splits = 1;
    out->threads = 256;
    const char *name = "";
    const long rows = (long)batch * P.out.h * P.out.w;
    switch (P.L.op) {
    case ECLIP_OP_CONV:
    case ECLIP_OP_LINEAR: {
        const GemmShape g = gemm_shape(P, (int)batch);
        out->m = (uint64_t)g.B * g.Ho * g.Wo; out->n = (uint64_t)g.Cout; out->k = (uint64_t)g.KH * g.KW * g.Cin;
        if (P.gemm) {
            const GemmPlan pl = plan_of(model, (long)out->m, (long)out->n, (long)out->k, (int)model->pool->streams[mask_id].n_cu);
            int bm, bn, bk;
            if (pl.kind == 1) { conv_wsk_tile(pl.variant, &bm, &bn); name = "conv_wsk_kernel"; out->threads = (uint32_t)pl.nw * 64; }
            else { conv_gemm_tile(pl.variant, &bm, &bn, &bk); name = "conv_gemm_kernel"; }
            out->tile_m = (uint32_t)bm; out->tile_n = (uint32_t)bn;
            out->k_splits = (uint32_t)pl.splits;
            out->workgroups = (uint32_t)pl.tiles * (uint32_t)pl.splits;
            out->launches = pl.splits > 1 ? 2 : 1;
        } else if (P.L.op == ECLIP_OP_CONV && P.L.groups > 1 && !(P.L.groups == P.in.c && P.L.c == P.L.groups)) {
            name = P.gc_super ? "gconv_mfma_kernel" : "gconv_kernel";
            out->workgroups = (uint32_t)((rows * P.L.c + 255) / 256);
            if (P.gc_super)
                out->workgroups = (uint32_t)gconv_mfma_workgroups(rows, P.L.groups, P.L.c / P.L.groups, P.gc_super,
                                                                  (int)model->pool->streams[mask_id].n_cu);
        } else if (P.L.op == ECLIP_OP_CONV && P.L.groups > 1) {
            DwConvArgs da{};
            da.B = (int)batch; da.C = P.L.c; da.Ho = P.L.h; da.Wo = P.L.w; da.KH = P.L.kh; da.KW = P.L.kw; da.stride = P.L.stride;
            da.dtype = model->dtype == ECLIP_F32 ? DT_F32 : (model->dtype == ECLIP_BF16 ? DT_BF16 : DT_F16);
            const int dw_cu = (int)model->pool->streams[mask_id].n_cu;
            name = dwconv_strip_rows(da, dw_cu) ? "dwconv3_strip_kernel" : dwconv_pixels_per_thread(da, dw_cu) == 4 ? "dwconv3_row_kernel" : "dwconv_kernel";
            out->workgroups = (uint32_t)((rows * (P.L.c / ((P.L.c % 8 || model->dtype == ECLIP_F32) ? (model->dtype == ECLIP_F32 && P.L.c % 4 == 0 ? 4 : 1) : 8)) + 255) / 256);
        } else {
            name = "conv_f32_kernel";
            out->workgroups = (uint32_t)((rows * P.L.c + 255) / 256);
        }
        break;
    }
    case ECLIP_OP_MAXPOOL:
        // 3x3 windows at stride 2 on vector-width channels: two outputs per thread (see launch_maxpool)
        name = (P.L.kh == 3 && P.L.kw == 3 && P.L.stride == 2 && P.L.c % (model->dtype == ECLIP_F32 ? 4 : 8) == 0) ? "maxpool3s2_block_kernel" : "maxpool_kernel";
        break;
    case ECLIP_OP_GAP: name = "gap_kernel"; break;
    case ECLIP_OP_LAYERNORM:
    case ECLIP_OP_SOFTMAX: {
        // 4 wavefronts per workgroup, each carrying 64 / (lanes per row) rows (see launch_row)
        const int v = model->dtype == ECLIP_F32 ? (P.in.c % 4 ? 1 : 4) : (P.in.c % 8 ? 1 : 8);
        const int nchunk = P.in.c / v, lpr = nchunk <= 48 ? 16 : 64;
        const long per_wg = 4 * (64 / lpr);
        name = "row_kernel";
        out->workgroups = (uint32_t)((rows + per_wg - 1) / per_wg);
        break;
    }
    case ECLIP_OP_ATTENTION: name = (P.in.w + 31) / 32 * 32 > 256 ? "attention_chunk_kernel" : "attention_kernel"; break;   // see launch_attention
    case ECLIP_OP_EMBED: name = "embed_kernel"; break;
    case ECLIP_OP_ELTWISE: name = "eltwise_kernel"; break;
    case ECLIP_OP_CONCAT:
        name = P.concat_noop ? "(in place)" : P.concat_copy ? "chancopy_kernel" : "concat_kernel";
        if (P.concat_noop) out->launches = 0;
        break;
    case ECLIP_OP_SHUFFLE:
        name = P.shuffle_noop ? "(folded into weights)" : "shuffle_kernel";
        if (P.shuffle_noop) out->launches = 0;
        break;
    default: break;
    }
    snprintf(out->kernel, sizeof out->kernel, "%s", name);
    return ECLIP_OK;
}

// ------------------------------------------------------------------------------------------------
// executor
// ------------------------------------------------------------------------------------------------
static const void *wptr(const eclip_model *m, size_t off) { return off == NONE ? nullptr : (const void *)(m->d_weights + off); }
// where layer P's output lives: its own buffer, or its channel range of the buffer of a concatenation done in place
static char *out_ptr(const eclip_model *m, const LayerPlan &P)
{
    return m->d_act + m->layers[P.buf].out_off + (size_t)P.c_off * (size_t)m->esize;
}
// pixel pitch (in channels) a reader of layer idx must use, 0 when the tensor is contiguous
static int pitch_of(const eclip_model *m, int idx) { return idx >= 0 ? m->layers[idx].ld : 0; }

// Launches layer i on `s`.  `d_out32` non-null: this is the last layer and its result goes to the caller.
static hipError_t launch_layer(eclip_model *m, uint32_t i, int batch, hipStream_t s, int n_cu, const void *d_in, float *d_out32,
                               uint32_t *n_launched)
{
    LayerPlan &P = m->layers[i];
    const eclip_layer &L = P.L;
    const int dt = m->dtype;
    auto src = [&](int idx) -> const void * {
        if (idx == -2) return nullptr;
        if (idx == -1) return m->in_kind == ECLIP_IN_IMAGE ? (const void *)m->d_in_stage : d_in;
        return (const void *)out_ptr(m, m->layers[idx]);
    };
    void *y = out_ptr(m, P);
    // the last layer writes float32 straight into the caller's buffer when its internal layout is the
    // logical one (SEQ / VEC) and its kernel has a float output path
    const bool chan_last_out = P.out.kind != ECLIP_KIND_IMAGE || (P.out.h == 1 && P.out.w == 1);
    float *y32 = nullptr;
    hipError_t e = hipSuccess;
    const long rows = (long)batch * P.out.h * P.out.w;
    *n_launched += 1;
    switch (L.op) {
    case ECLIP_OP_CONV:
    case ECLIP_OP_LINEAR: {
        const GemmShape g = gemm_shape(P, batch);
        if (P.gemm) {
            if (d_out32 && chan_last_out) y32 = d_out32;
            ConvGemmArgs a{src(L.in0), wptr(m, P.w_dev), wptr(m, P.b_dev), src(L.in1), y32 ? nullptr : y, y32, m->ws,
                           g.B, g.H, g.W, g.Cin, g.Ho, g.Wo, g.Cout, g.KH, g.KW, g.stride, g.pad, L.act, dt};
            a.ldx = pitch_of(m, L.in0);
            a.ldy = P.ld;
            const GemmPlan pl = plan_of(m, (long)g.B * g.Ho * g.Wo, g.Cout, (long)g.KH * g.KW * g.Cin, n_cu);
            *n_launched -= 1;
            e = launch_conv_gemm(a, pl, s, n_launched);
        } else if (L.op == ECLIP_OP_CONV && L.groups > 1 && !(L.groups == g.Cin && L.c == L.groups)) {
            GConvArgs a{src(L.in0), wptr(m, P.w_dev), wptr(m, P.b_dev), src(L.in1), y, g.B, g.H, g.W, g.Cin, g.Ho, g.Wo, g.Cout,
                        g.KH, g.KW, g.stride, g.pad, L.groups, L.act, dt};
            e = P.gc_super ? launch_gconv_mfma(a, P.gc_super, n_cu, s) : launch_gconv(a, n_cu, s);
        } else if (L.op == ECLIP_OP_CONV && L.groups > 1) {
            DwConvArgs a{src(L.in0), wptr(m, P.w_dev), wptr(m, P.b_dev), src(L.in1), y, g.B, g.H, g.W, L.c, g.Ho, g.Wo, g.KH, g.KW, g.stride, g.pad, L.act, dt};
            e = launch_dwconv(a, n_cu, s);
        } else {
            float *yf = (float *)y;
            if (d_out32 && chan_last_out) { yf = d_out32; y32 = d_out32; }
            ConvF32Args a{(const float *)src(L.in0), (const float *)wptr(m, P.w_dev), (const float *)wptr(m, P.b_dev), (const float *)src(L.in1), yf,
                          g.B, g.H, g.W, g.Cin, g.Ho, g.Wo, g.Cout, g.KH, g.KW, g.stride, g.pad, L.act};
            e = launch_conv_f32(a, s);
        }
        break;
    }
    case ECLIP_OP_MAXPOOL: {
        PoolArgs a{src(L.in0), y, batch, P.in.h, P.in.w, L.c, L.h, L.w, L.kh, L.kw, L.stride, L.pad, dt};
        e = launch_maxpool(a, n_cu, s);
        break;
    }
    case ECLIP_OP_GAP:
        if (d_out32) y32 = d_out32;
        *n_launched -= 1;
        e = launch_gap(src(L.in0), y, y32, m->ws, m->ws_floats, batch, P.in.h * P.in.w, L.c, dt, n_cu, s, n_launched);
        break;
    case ECLIP_OP_LAYERNORM:
    case ECLIP_OP_SOFTMAX: {
        if (d_out32) y32 = d_out32;
        RowArgs a{src(L.in0), src(L.in1), wptr(m, P.g_dev), wptr(m, P.be_dev), y, y32, rows, L.c, L.eps, dt};
        e = L.op == ECLIP_OP_LAYERNORM ? launch_layernorm(a, n_cu, s) : launch_softmax(a, n_cu, s);
        break;
    }
    case ECLIP_OP_ATTENTION: {
        if (d_out32) y32 = d_out32;
        AttnArgs a{src(L.in0), y, y32, batch, P.in.w, L.c, L.heads, dt};
        e = launch_attention(a, n_cu, s);
        break;
    }
    case ECLIP_OP_EMBED: {
        EmbedArgs a{(const int32_t *)d_in, wptr(m, P.w_dev), wptr(m, P.g_dev), wptr(m, P.be_dev), y, batch, P.out.w, L.c, L.aux0, dt};
        e = launch_embed(a, n_cu, s);
        break;
    }
    case ECLIP_OP_ELTWISE: {
        if (d_out32 && chan_last_out) y32 = d_out32;
        EltArgs a{src(L.in0), wptr(m, P.b_dev), src(L.in1), y, y32, rows, L.c, L.act, dt};
        e = launch_eltwise(a, n_cu, s);
        break;
    }
    case ECLIP_OP_CONCAT:
        if (P.concat_noop) *n_launched -= 1;                 // both operands were written into this buffer by their producers
        else if (P.concat_copy) e = launch_chancopy(src(L.in0), y, rows, P.in.c, P.ld ? P.ld : L.c, dt, s);
        else e = launch_concat(src(L.in0), src(L.in1), y, rows, P.in.c, L.c - P.in.c, dt, s);
        break;
    case ECLIP_OP_SHUFFLE:
        if (P.shuffle_noop) *n_launched -= 1;                // folded into the weights of the layers that read it
        else e = launch_shuffle(src(L.in0), y, rows, L.c, L.groups, dt, s);
        break;
    default:
        e = hipErrorInvalidValue;
    }
    if (e != hipSuccess || !d_out32 || y32) return e;
    // the layer could not write the caller's buffer itself: convert its internal output
    *n_launched += 1;
    if (P.out.kind == ECLIP_KIND_IMAGE && !chan_last_out) return launch_nhwc_to_nchw_f32(y, d_out32, batch, P.out.c, P.out.h, P.out.w, dt, s);
    return launch_to_f32(y, d_out32, rows * P.out.c, dt, s);
}

// Launches layers i and i + 1 (pair_next) in one kernel when the planner finds a common plan; *done tells whether it did.
static hipError_t launch_pair(eclip_model *m, uint32_t i, int batch, hipStream_t s, int n_cu, const void *d_in, uint32_t *n_launched, bool *done)
{
    *done = false;
    ConvGemmArgs a[2];
    GemmPlan own[2], pl[2];
    long mnk[2][3];
    for (int k = 0; k < 2; ++k) {
        const LayerPlan &P = m->layers[i + k];
        const eclip_layer &L = P.L;
        auto src = [&](int idx) -> const void * {
            if (idx == -2) return nullptr;
            if (idx == -1) return m->in_kind == ECLIP_IN_IMAGE ? (const void *)m->d_in_stage : d_in;
            return (const void *)out_ptr(m, m->layers[idx]);
        };
        const GemmShape g = gemm_shape(P, batch);
        a[k] = ConvGemmArgs{src(L.in0), wptr(m, P.w_dev), wptr(m, P.b_dev), src(L.in1), out_ptr(m, P), nullptr, m->ws,
                            g.B, g.H, g.W, g.Cin, g.Ho, g.Wo, g.Cout, g.KH, g.KW, g.stride, g.pad, L.act, m->dtype};
        a[k].ldx = pitch_of(m, L.in0);
        a[k].ldy = P.ld;
        mnk[k][0] = (long)g.B * g.Ho * g.Wo; mnk[k][1] = g.Cout; mnk[k][2] = (long)g.KH * g.KW * g.Cin;
        own[k] = plan_of(m, mnk[k][0], mnk[k][1], mnk[k][2], n_cu);
    }
    if (!conv_gemm_plan_pair(own[0], mnk[0][0], mnk[0][1], mnk[0][2], own[1], mnk[1][0], mnk[1][1], mnk[1][2], n_cu, &pl[0], &pl[1]))
        return hipSuccess;
    *done = true;
    return launch_conv_gemm_pair(a[0], pl[0], a[1], pl[1], s, n_launched);
}

// Launches the GAP layer i and the linear layer i + 1 (gapfc_next) as one kernel when the shape suits it.
static hipError_t launch_gapfc_pair(eclip_model *m, uint32_t i, int batch, hipStream_t s, const void *d_in, float *d_out32, uint32_t *n_launched, bool *done)
{
    *done = false;
    const LayerPlan &G = m->layers[i], &F = m->layers[i + 1];
    const int HW = G.in.h * G.in.w, C = G.L.c;
    if (getenv("ECLIP_NO_PAIRS") || !gapfc_supported(batch, HW, C, m->dtype)) return hipSuccess;
    const void *x = G.L.in0 == -1 ? (m->in_kind == ECLIP_IN_IMAGE ? (const void *)m->d_in_stage : d_in) : (const void *)out_ptr(m, m->layers[G.L.in0]);
    *done = true;
    *n_launched += 1;
    return launch_gapfc(x, wptr(m, F.w_dev), wptr(m, F.b_dev), d_out32 ? nullptr : (void *)out_ptr(m, F), d_out32, batch, HW, C, F.L.c, F.L.act,
                        m->dtype, s);
}

// First layer straight from the caller's NCHW tensor (stem_direct), when a plan of that form is within the cost of the
// re-layout kernel it saves; *done tells whether it was launched.
static hipError_t launch_stem_direct(eclip_model *m, int batch, hipStream_t s, int n_cu, const void *d_in, uint32_t *n_launched, bool *done)
{
    *done = false;
    const LayerPlan &P = m->layers[0];
    const GemmShape g = gemm_shape(P, batch);
    GemmPlan pl;
    if (!conv_gemm_plan_stem((long)g.B * g.Ho * g.Wo, g.Cout, (long)g.KH * g.KW * g.Cin, n_cu, m->ws_floats, 2.0, &pl)) return hipSuccess;
    ConvGemmArgs a{d_in, wptr(m, P.w_dev), wptr(m, P.b_dev), nullptr, out_ptr(m, P), nullptr, m->ws,
                   g.B, g.H, g.W, g.Cin, g.Ho, g.Wo, g.Cout, g.KH, g.KW, g.stride, g.pad, P.L.act, m->dtype};
    a.nchw_c = m->in_c;
    *done = true;
    return launch_conv_gemm(a, pl, s, n_launched);
}

static hipError_t launch_input_stage(eclip_model *m, int batch, const void *d_in, hipStream_t s, uint32_t *n_launched)
{
    if (m->in_kind != ECLIP_IN_IMAGE) return hipSuccess;
    *n_launched += 1;
    return launch_nchw_to_nhwc(d_in, m->d_in_stage, batch, m->in_c, m->in_h, m->in_w, m->in_cp, m->dtype, s);
}

// One launch unit of the served path, starting at layer i: the first layer together with the input re-layout it needs
// (or reading the caller's tensor itself), two independent matrix-core layers in one launch, pool + classifier in one
// launch, or a single layer.  *consumed receives the number of layers the unit covered.  eclip_submit and the profiler
// both walk a model through this function, so what is profiled is what is served.
static hipError_t launch_unit(eclip_model *m, uint32_t i, int batch, hipStream_t s, int n_cu, const void *d_in, float *d_out,
                              uint32_t *n_launched, uint32_t *consumed)
{
    const uint32_t n_layers = (uint32_t)m->layers.size();
    hipError_t e;
    *consumed = 1;
    if (i == 0) {
        bool stem_done = false;
        if (m->stem_direct) {
            if ((e = launch_stem_direct(m, batch, s, n_cu, d_in, n_launched, &stem_done)) != hipSuccess) return e;
            if (stem_done) return hipSuccess;
        }
        if ((e = launch_input_stage(m, batch, d_in, s, n_launched)) != hipSuccess) return e;
    }
    if (m->layers[i].pair_next) {
        bool paired = false;
        if ((e = launch_pair(m, i, batch, s, n_cu, d_in, n_launched, &paired)) != hipSuccess) return e;
        if (paired) { *consumed = 2; return hipSuccess; }
    }
    if (m->layers[i].gapfc_next) {
        bool fused = false;
        if ((e = launch_gapfc_pair(m, i, batch, s, d_in, i + 2 == n_layers ? d_out : nullptr, n_launched, &fused)) != hipSuccess) return e;
        if (fused) { *consumed = 2; return hipSuccess; }
    }
    return launch_layer(m, i, batch, s, n_cu, d_in, i + 1 == n_layers ? d_out : nullptr, n_launched);
}

// The captured form of a request on (d_in, d_out, batch) under the current table, plans and workspace: looked up, or
// captured now.  Every run of kernel groups that shares a pooled stream becomes one HIP graph.  It is captured from a
// stream private to the model, in thread-local mode -- pooled streams may be shared by several workers, whose launches
// must not land in (or break) another worker's capture -- and replayed on the pooled stream, whose queue is what
// confines the kernels to its CUs; the cross-stream dependencies stay outside the graphs, as events between the segments.
// Nothing runs during capture: the caller replays the entry right away.  At most 8 entries per model, least recently
// used first out.
static hipError_t graph_entry(eclip_model *m, const void *d_in, void *d_out, uint32_t batch, eclip_model::GraphEntry **out)
{
    *out = nullptr;
    for (auto &g : m->graphs)
        if (g.d_in == d_in && g.d_out == d_out && g.batch == batch && g.ws == m->ws && g.stamp == m->stamp) {
            g.last_use = ++m->use_clock;
            *out = &g;
            return hipSuccess;
        }
    // stale entries (older stamp) and, beyond 8, the least recently used one make room
    for (size_t k = 0; k < m->graphs.size();) {
        if (m->graphs[k].stamp != m->stamp) {
            for (auto &sg : m->graphs[k].segs) (void)hipGraphExecDestroy(sg.exec);
            m->graphs.erase(m->graphs.begin() + k);
        } else ++k;
    }
    if (m->graphs.size() >= 8) {
        size_t lru = 0;
        for (size_t k = 1; k < m->graphs.size(); ++k)
            if (m->graphs[k].last_use < m->graphs[lru].last_use) lru = k;
        for (auto &sg : m->graphs[lru].segs) (void)hipGraphExecDestroy(sg.exec);
        m->graphs.erase(m->graphs.begin() + lru);
    }
    eclip_model::GraphEntry ge{d_in, d_out, batch, m->ws, m->stamp, ++m->use_clock, 0, {}};
    const uint32_t n_layers = (uint32_t)m->layers.size();
    hipError_t e = hipSuccess;
    for (uint32_t i = 0; i < n_layers && e == hipSuccess;) {
        const uint32_t g0 = m->group_of_layer[i];
        const uint32_t mask_id = m->mask_of_group[g0];
        const PoolStream &ps = m->pool->streams[mask_id];
        e = hipStreamBeginCapture(m->capture_stream, hipStreamCaptureModeThreadLocal);
        if (e != hipSuccess) break;
        hipError_t le = hipSuccess;
        while (i < n_layers && le == hipSuccess && m->pool->streams[m->mask_of_group[m->group_of_layer[i]]].stream == ps.stream) {
            uint32_t consumed = 1;
            le = launch_unit(m, i, (int)batch, m->capture_stream, (int)ps.n_cu, d_in, (float *)d_out, &ge.n_kernels, &consumed);
            i += consumed;
        }
        hipGraph_t graph = nullptr;
        e = hipStreamEndCapture(m->capture_stream, &graph);  // always ended, so that the stream is usable again
        if (le != hipSuccess) e = le;
        hipGraphExec_t exec = nullptr;
        if (e == hipSuccess) e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
        if (graph) (void)hipGraphDestroy(graph);
        if (e == hipSuccess) ge.segs.push_back(eclip_model::GraphSeg{exec, mask_id, g0});
    }
    if (e != hipSuccess) {
        for (auto &sg : ge.segs) (void)hipGraphExecDestroy(sg.exec);
        return e;
    }
    m->graphs.push_back(std::move(ge));
    *out = &m->graphs.back();
    return hipSuccess;
}

// The body of eclip_submit, with the model's mutex held.
static eclip_status submit_locked(eclip_model *model, const void *d_in, void *d_out, uint32_t batch, eclip_req **out)
{
    if (!model->has_alloc) return fail(ECLIP_ESTATE, "eclip_alloc_set has not been called");
    eclip_req *r = nullptr;
    for (eclip_req &q : model->reqs)
        if (!q.pending) { r = &q; break; }
    if (!r) return fail(ECLIP_ELIMIT, "more than %zu requests in flight", model->reqs.size());
    eclip_pool *pool = model->pool;
    HIP_TRY(hipSetDevice(pool->device));

    const uint32_t n_layers = (uint32_t)model->layers.size();
    hipStream_t cur = pool->streams[model->mask_of_group[0]].stream;
    r->n_kernels = 0;
    r->n_switches = 0;
    r->timed = model->timing;
    // Once the first call below has been made, a failure leaves work queued that this request can no longer account
    // for: the device is drained, the chain to the previous request is dropped (nothing is outstanding after the
    // drain, and earlier requests keep their own completion events), the slot stays free, and the caller gets EHIP.
    hipError_t e = hipSuccess;
    const char *what = "";
#define SUB_TRY(call)                                                          \
    do {                                                                       \
        if (e == hipSuccess && (e = (call)) != hipSuccess) what = #call;       \
    } while (0)
    // requests of one model run in order: the first kernel waits for the previous request when that
    // one ended on another stream (on the same stream, queue order already serialises them)
    if (model->last_done && model->last_stream != cur) SUB_TRY(hipStreamWaitEvent(cur, model->last_done, 0));
    if (r->timed) SUB_TRY(hipEventRecord(r->t_start, cur));
    if (model->use_graphs) {
        eclip_model::GraphEntry *ge = nullptr;
        SUB_TRY(graph_entry(model, d_in, d_out, batch, &ge));
        for (size_t k = 0; ge && k < ge->segs.size() && e == hipSuccess; ++k) {
            const eclip_model::GraphSeg &sg = ge->segs[k];
            const PoolStream &ps = pool->streams[sg.mask_id];
            if (ps.stream != cur) {
                SUB_TRY(model->hops.hop(cur, ps.stream, model->switch_events[sg.first_group]));
                cur = ps.stream;
                r->n_switches++;
            }
            SUB_TRY(hipGraphLaunch(sg.exec, cur));
        }
        if (ge) r->n_kernels = ge->n_kernels;
    } else {
    uint32_t prev_group = 0;
    for (uint32_t i = 0; i < n_layers && e == hipSuccess;) {
        const uint32_t g = model->group_of_layer[i];
        const PoolStream &ps = pool->streams[model->mask_of_group[g]];
        if (g != prev_group && ps.stream != cur) {
            // group boundary that changes stream: the next group waits for everything queued so far
            SUB_TRY(model->hops.hop(cur, ps.stream, model->switch_events[g]));
            cur = ps.stream;
            r->n_switches++;
        }
        prev_group = g;
        uint32_t consumed = 1;
        SUB_TRY(launch_unit(model, i, (int)batch, cur, (int)ps.n_cu, d_in, (float *)d_out, &r->n_kernels, &consumed));
        i += consumed;
    }
    }
    if (r->timed) SUB_TRY(hipEventRecord(r->t_done, cur));
    SUB_TRY(hipEventRecord(r->done, cur));
#undef SUB_TRY
    if (e != hipSuccess) {
        (void)hipDeviceSynchronize();
        (void)hipGetLastError();
        model->last_done = nullptr;
        model->last_stream = nullptr;
        return fail(ECLIP_EHIP, "%s failed: %s; the device was drained and the request dropped", what, hipGetErrorString(e));
    }
    r->pending = true;
    model->inflight++;
    model->last_done = r->done;
    model->last_stream = cur;
    *out = r;
    return ECLIP_OK;
}

extern "C" eclip_status eclip_submit(eclip_model *model, const void *d_in, void *d_out, uint32_t batch, eclip_req **out)
{
    if (!model || !out) return fail(ECLIP_EINVAL, "null argument");
    *out = nullptr;
    if (!d_in || !d_out) return fail(ECLIP_EINVAL, "null device buffer");
    if (batch == 0 || batch > model->max_batch) return fail(ECLIP_EINVAL, "batch %u outside 1..%u", batch, model->max_batch);
    std::lock_guard<std::mutex> lk(model->mu);
    return submit_locked(model, d_in, d_out, batch, out);
}

// ------------------------------------------------------------------------------------------------
// the entry point that allocates nothing
// ------------------------------------------------------------------------------------------------
extern "C" eclip_status eclip_submit_static(eclip_model *model, const void *d_in, void *d_out, uint32_t batch, eclip_req **out)
{
    if (!model || !out) return fail(ECLIP_EINVAL, "null argument");
    *out = nullptr;
    if (!d_in || !d_out) return fail(ECLIP_EINVAL, "null device buffer");
    if (batch == 0 || batch > model->max_batch) return fail(ECLIP_EINVAL, "batch %u outside 1..%u", batch, model->max_batch);
    if (model->ws_floats * sizeof(float) > (size_t)ECLIP_STATIC_SCRATCH_BYTES)
        return fail(ECLIP_ELIMIT, "the model's kernels need %zu bytes of scratch, the static scratch holds %zu", model->ws_floats * sizeof(float),
                    (size_t)ECLIP_STATIC_SCRATCH_BYTES);
    void *sp = model->pool->scratch;
    if (!sp) return fail(ECLIP_ESTATE, "the pool has no static scratch address");
    std::lock_guard<std::mutex> lk(model->mu);
    model->ws = (float *)sp;
    const eclip_status st = submit_locked(model, d_in, d_out, batch, out);
    model->ws = model->d_ws;
    return st;
}

extern "C" eclip_status eclip_model_graphs(eclip_model *model, int enable)
{
    if (!model) return fail(ECLIP_EINVAL, "model is null");
    std::lock_guard<std::mutex> lk(model->mu);
    if (model->inflight) return fail(ECLIP_ESTATE, "%u requests still in flight", model->inflight);
    HIP_TRY(hipSetDevice(model->pool->device));
    if (enable && !model->capture_stream) HIP_TRY(hipStreamCreateWithFlags(&model->capture_stream, hipStreamNonBlocking));
    model->use_graphs = enable != 0;
    if (!enable) {
        HIP_TRY(hipDeviceSynchronize());
        drop_graphs(model);
    }
    return ECLIP_OK;
}

extern "C" eclip_status eclip_model_timing(eclip_model *model, int enable)
{
    if (!model) return fail(ECLIP_EINVAL, "model is null");
    std::lock_guard<std::mutex> lk(model->mu);
    model->timing = enable != 0;
    return ECLIP_OK;
}

extern "C" eclip_status eclip_wait(eclip_req *req, uint64_t timeout_ns, eclip_timing *opt_out)
{
    if (!req || !req->model) return fail(ECLIP_EINVAL, "request is null");
    eclip_model *m = req->model;
    if (!req->pending) return fail(ECLIP_ESTATE, "request is not pending");
    if (timeout_ns == UINT64_MAX) {
        HIP_TRY(hipEventSynchronize(req->done));
    } else {
        const auto deadline = std::chrono::steady_clock::now() + std::chrono::nanoseconds(timeout_ns);
        for (;;) {
            const hipError_t e = hipEventQuery(req->done);
            if (e == hipSuccess) break;
            if (e != hipErrorNotReady) return fail(ECLIP_EHIP, "hipEventQuery failed: %s", hipGetErrorString(e));
            if (std::chrono::steady_clock::now() >= deadline) return fail(ECLIP_ETIMEOUT, "request still running after %llu ns", (unsigned long long)timeout_ns);
            std::this_thread::yield();
        }
    }
    if (opt_out) {
        opt_out->gpu_ns = 0;
        if (req->timed) {
            float ms = 0.0f;
            HIP_TRY(hipEventElapsedTime(&ms, req->t_start, req->t_done));
            opt_out->gpu_ns = (uint64_t)((double)ms * 1e6);
        }
        opt_out->n_kernels = req->n_kernels;
        opt_out->n_switches = req->n_switches;
    }
    std::lock_guard<std::mutex> lk(m->mu);
    req->pending = false;
    m->inflight--;
    return ECLIP_OK;
}

// Shared front end of the two profilers: argument checks, the lock, and one untimed pass of the whole model through
// the served launch sequence so that every activation buffer holds finite data.
static eclip_status profile_prepare(eclip_model *model, uint32_t group, uint32_t mask_id, uint32_t batch, uint32_t iters)
{
    if (group >= model->n_groups) return fail(ECLIP_EINVAL, "unknown group %u", group);
    if (mask_id >= model->pool->streams.size()) return fail(ECLIP_EINVAL, "unknown mask id %u", mask_id);
    if (batch == 0 || batch > model->max_batch) return fail(ECLIP_EINVAL, "batch %u outside 1..%u", batch, model->max_batch);
    if (iters == 0 || iters > 10000) return fail(ECLIP_EINVAL, "iters must be 1..10000");
    if (model->inflight) return fail(ECLIP_ESTATE, "requests in flight");
    eclip_pool *pool = model->pool;
    HIP_TRY(hipSetDevice(pool->device));
    const PoolStream &ps = pool->streams[mask_id];
    const uint32_t n_layers = (uint32_t)model->layers.size();
    uint32_t dummy = 0;
    for (uint32_t i = 0; i < n_layers;) {
        uint32_t consumed = 1;
        HIP_TRY(launch_unit(model, i, (int)batch, ps.stream, (int)ps.n_cu, model->d_self_in, model->d_self_out, &dummy, &consumed));
        i += consumed;
    }
    HIP_TRY(hipStreamSynchronize(ps.stream));
    return ECLIP_OK;
}

extern "C" eclip_status eclip_profile_group(eclip_model *model, uint32_t group, uint32_t mask_id, uint32_t batch,
                                            uint32_t iters, uint64_t *ns_per_kernel_out)
{
    if (!model || !ns_per_kernel_out) return fail(ECLIP_EINVAL, "null argument");
    std::lock_guard<std::mutex> lk(model->mu);
    eclip_status st = profile_prepare(model, group, mask_id, batch, iters);
    if (st != ECLIP_OK) return st;
    const PoolStream &ps = model->pool->streams[mask_id];
    const uint32_t n_layers = (uint32_t)model->layers.size();
    uint32_t dummy = 0;
    std::vector<uint32_t> idx;
    for (uint32_t i = 0; i < n_layers; ++i)
        if (model->group_of_layer[i] == group) idx.push_back(i);
    const size_t nk = idx.size();
    std::vector<hipEvent_t> ev(2 * nk, nullptr);
    for (hipEvent_t &e : ev)
        if (hipEventCreate(&e) != hipSuccess) st = fail(ECLIP_EHIP, "hipEventCreate failed");
    std::vector<std::vector<float>> samples(nk);
    // An event pair around a single microsecond-scale kernel mostly measures the two event markers, so
    // every kernel is launched REPS times back to back between its two events and the elapsed time is
    // divided by REPS: the figure is the kernel's cost as one link of an in-order chain, launch gap included.
    const uint32_t REPS = 8;
    for (uint32_t it = 0; it < iters + 2 && st == ECLIP_OK; ++it) {       // two warm-up rounds
        hipError_t e = hipSuccess;
        for (size_t k = 0; k < nk && e == hipSuccess; ++k) {
            const uint32_t i = idx[k];
            e = hipEventRecord(ev[2 * k], ps.stream);
            for (uint32_t r = 0; r < REPS && e == hipSuccess; ++r)
                e = launch_layer(model, i, (int)batch, ps.stream, (int)ps.n_cu, model->d_self_in, i + 1 == n_layers ? model->d_self_out : nullptr, &dummy);
            if (e == hipSuccess) e = hipEventRecord(ev[2 * k + 1], ps.stream);
        }
        if (e == hipSuccess) e = hipStreamSynchronize(ps.stream);
        if (e != hipSuccess) { st = fail(ECLIP_EHIP, "profiling launch failed: %s", hipGetErrorString(e)); break; }
        if (it < 2) continue;
        for (size_t k = 0; k < nk; ++k) {
            float ms = 0.0f;
            if (hipEventElapsedTime(&ms, ev[2 * k], ev[2 * k + 1]) != hipSuccess) { st = fail(ECLIP_EHIP, "hipEventElapsedTime failed"); break; }
            samples[k].push_back(ms / (float)REPS);
        }
    }
    for (hipEvent_t e : ev)
        if (e) (void)hipEventDestroy(e);
    if (st != ECLIP_OK) return st;
    for (size_t k = 0; k < nk; ++k) {
        std::sort(samples[k].begin(), samples[k].end());
        ns_per_kernel_out[k] = (uint64_t)std::llround((double)samples[k][samples[k].size() / 2] * 1e6);
    }
    return ECLIP_OK;
}

extern "C" eclip_status eclip_model_tune(eclip_model *model, uint32_t mask_id, uint32_t batch, uint32_t iters, uint32_t *n_tuned_out)
{
    if (!model) return fail(ECLIP_EINVAL, "model is null");
    std::lock_guard<std::mutex> lk(model->mu);
    eclip_status st = profile_prepare(model, 0, mask_id, batch, iters);
    if (st != ECLIP_OK) return st;
    const PoolStream &ps = model->pool->streams[mask_id];
    const int n_cu = (int)ps.n_cu;
    const uint32_t n_layers = (uint32_t)model->layers.size();
    hipEvent_t ev[2] = {nullptr, nullptr};
    if (hipEventCreate(&ev[0]) != hipSuccess || hipEventCreate(&ev[1]) != hipSuccess) st = fail(ECLIP_EHIP, "hipEventCreate failed");
    uint32_t n_tuned = 0;
    const uint32_t REPS = 6;
    for (uint32_t i = 0; i < n_layers && st == ECLIP_OK; ++i) {
        const LayerPlan &P = model->layers[i];
        if (!P.gemm) continue;
        const eclip_layer &L = P.L;
        const GemmShape g = gemm_shape(P, (int)batch);
        const long M = (long)g.B * g.Ho * g.Wo, N = g.Cout, K = (long)g.KH * g.KW * g.Cin;
        const std::array<long, 4> key{M, N, K, (long)n_cu};
        if (model->tuned.count(key)) continue;
        auto src = [&](int idx) -> const void * {
            if (idx == -2) return nullptr;
            if (idx == -1) return model->in_kind == ECLIP_IN_IMAGE ? (const void *)model->d_in_stage : (const void *)model->d_self_in;
            return (const void *)out_ptr(model, model->layers[idx]);
        };
        const bool last = i + 1 == n_layers;
        const bool chan_last_out = P.out.kind != ECLIP_KIND_IMAGE || (P.out.h == 1 && P.out.w == 1);
        float *y32 = (last && chan_last_out) ? model->d_self_out : nullptr;
        ConvGemmArgs a{src(L.in0), wptr(model, P.w_dev), wptr(model, P.b_dev), src(L.in1), y32 ? nullptr : (void *)out_ptr(model, P), y32,
                       model->ws, g.B, g.H, g.W, g.Cin, g.Ho, g.Wo, g.Cout, g.KH, g.KW, g.stride, g.pad, L.act, model->dtype};
        a.ldx = pitch_of(model, L.in0);
        a.ldy = P.ld;
        const GemmPlan own = conv_gemm_plan(M, N, K, n_cu, model->ws_floats);
        std::vector<GemmPlan> cand = conv_gemm_candidates(M, N, K, n_cu, model->ws_floats);
        cand.insert(cand.begin(), own);
        float best_ms = 1e30f, own_ms = 1e30f;
        size_t best = 0;
        for (size_t c = 0; c < cand.size() && st == ECLIP_OK; ++c) {
            float t_min = 1e30f;
            for (uint32_t it = 0; it < iters + 1; ++it) {
                // the first sample is a single launch: it warms the code and the caches up, and a candidate that takes more
                // than three times the best so far per launch is dropped there and then (the cost model's own plan is timed
                // first, so the bar is set early)
                const uint32_t reps = it ? REPS : 1;
                hipError_t e = hipEventRecord(ev[0], ps.stream);
                for (uint32_t r = 0; r < reps && e == hipSuccess; ++r) e = launch_conv_gemm(a, cand[c], ps.stream, nullptr);
                if (e == hipSuccess) e = hipEventRecord(ev[1], ps.stream);
                if (e == hipSuccess) e = hipStreamSynchronize(ps.stream);
                float ms = 0.0f;
                if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev[0], ev[1]);
                if (e != hipSuccess) { st = fail(ECLIP_EHIP, "tuning launch failed: %s", hipGetErrorString(e)); break; }
                if (it) t_min = std::min(t_min, ms / (float)REPS);
                else if (ms > 3.0f * best_ms + 0.02f) break;
            }
            if (c == 0) own_ms = t_min;
            if (t_min < best_ms) { best_ms = t_min; best = c; }
        }
        if (st != ECLIP_OK) break;
        // the cost model's plan stays unless a measured one beats it clearly: its picks keep independent layers on the
        // kernel that can share a launch, which a per-layer timing does not see
        model->tuned[key] = best_ms < 0.95f * own_ms ? cand[best] : own;
        model->stamp++;
        ++n_tuned;
    }
    for (hipEvent_t e : ev)
        if (e) (void)hipEventDestroy(e);
    if (st == ECLIP_OK && n_tuned_out) *n_tuned_out = n_tuned;
    return st;
}

extern "C" eclip_status eclip_profile_group_served(eclip_model *model, uint32_t group, uint32_t mask_id, uint32_t batch,
                                                   uint32_t iters, uint64_t *group_ns_out, uint32_t *n_launches_out)
{
    if (!model || !group_ns_out) return fail(ECLIP_EINVAL, "null argument");
    std::lock_guard<std::mutex> lk(model->mu);
    eclip_status st = profile_prepare(model, group, mask_id, batch, iters);
    if (st != ECLIP_OK) return st;
    const PoolStream &ps = model->pool->streams[mask_id];
    const uint32_t n_layers = (uint32_t)model->layers.size();
    uint32_t first = n_layers, last = 0;
    for (uint32_t i = 0; i < n_layers; ++i)
        if (model->group_of_layer[i] == group) { first = std::min(first, i); last = i; }
    hipEvent_t ev[2] = {nullptr, nullptr};
    if (hipEventCreate(&ev[0]) != hipSuccess || hipEventCreate(&ev[1]) != hipSuccess) st = fail(ECLIP_EHIP, "hipEventCreate failed");
    std::vector<float> samples;
    uint32_t launches = 0;
    // the group's launch units in order, as eclip_submit issues them (pairs never straddle a group boundary), twice
    // back to back per sample so that the two event markers weigh less against a short group
    const uint32_t REPS = 2;
    for (uint32_t it = 0; it < iters + 2 && st == ECLIP_OK; ++it) {       // two warm-up rounds
        hipError_t e = hipEventRecord(ev[0], ps.stream);
        launches = 0;
        for (uint32_t r = 0; r < REPS && e == hipSuccess; ++r)
            for (uint32_t i = first; i <= last && e == hipSuccess;) {
                uint32_t consumed = 1;
                e = launch_unit(model, i, (int)batch, ps.stream, (int)ps.n_cu, model->d_self_in, model->d_self_out, &launches, &consumed);
                i += consumed;
            }
        if (e == hipSuccess) e = hipEventRecord(ev[1], ps.stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ps.stream);
        if (e != hipSuccess) { st = fail(ECLIP_EHIP, "profiling launch failed: %s", hipGetErrorString(e)); break; }
        if (it < 2) continue;
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, ev[0], ev[1]) != hipSuccess) { st = fail(ECLIP_EHIP, "hipEventElapsedTime failed"); break; }
        samples.push_back(ms / (float)REPS);
    }
    for (hipEvent_t e : ev)
        if (e) (void)hipEventDestroy(e);
    if (st != ECLIP_OK) return st;
    std::sort(samples.begin(), samples.end());
    *group_ns_out = (uint64_t)std::llround((double)samples[samples.size() / 2] * 1e6);
    if (n_launches_out) *n_launches_out = launches / REPS;
    return ECLIP_OK;
}

// ------------------------------------------------------------------------------------------------
// allocator entry point
// ------------------------------------------------------------------------------------------------
extern "C" eclip_status eclip_alloc_solve(const eclip_alloc_problem *problem, uint32_t *cfg_idx_out,
                                          eclip_u128 *objective_out, uint32_t *switches_out)
{
    bool limit = false;
    std::string err;
    try {
        err = solve_alloc(problem, cfg_idx_out, objective_out, switches_out, &limit);
    } catch (const std::bad_alloc &) {
        return fail(ECLIP_ENOMEM, "allocation solver ran out of memory");
    }
    if (err.empty()) return ECLIP_OK;
    return fail(limit ? ECLIP_ELIMIT : ECLIP_EINVAL, "%s", err.c_str());
}

extern "C" eclip_status eclip_alloc_model_wise(const eclip_alloc_problem *problem, uint32_t slo_num, uint32_t slo_den,
                                               uint32_t *cfg_idx_out, uint32_t *switches_out)
{
    const std::string err = policy_model_wise(problem, slo_num, slo_den, cfg_idx_out, switches_out);
    return err.empty() ? ECLIP_OK : fail(ECLIP_EINVAL, "%s", err.c_str());
}

extern "C" eclip_status eclip_alloc_kernel_wise(const eclip_alloc_problem *problem, uint32_t tol_pct, uint32_t *cfg_idx_out,
                                                uint32_t *switches_out)
{
    const std::string err = policy_kernel_wise(problem, tol_pct, cfg_idx_out, switches_out);
    return err.empty() ? ECLIP_OK : fail(ECLIP_EINVAL, "%s", err.c_str());
}

// ------------------------------------------------------------------------------------------------
// repartitioning overhead
// ------------------------------------------------------------------------------------------------
extern "C" eclip_status eclip_bench_switch(eclip_pool *pool, uint32_t mask_a, uint32_t mask_b, uint32_t iters,
                                           double *same_stream_ns, double *pooled_ns, double *create_ns)
{
    if (!pool) return fail(ECLIP_EINVAL, "pool is null");
    if (mask_a >= pool->streams.size() || mask_b >= pool->streams.size()) return fail(ECLIP_EINVAL, "unknown mask id");
    if (iters == 0 || iters > 100000) return fail(ECLIP_EINVAL, "iters must be 1..100000");
    HIP_TRY(hipSetDevice(pool->device));
    const PoolStream &A = pool->streams[mask_a], &B = pool->streams[mask_b];
    uint32_t *d = nullptr;
    HIP_TRY(hipMalloc(&d, 256));
    HIP_TRY(hipMemset(d, 0, 256));
    hipEvent_t ev[2] = {nullptr, nullptr};
    HopSignal hops;                                  // the same dependency mechanism eclip_submit uses
    hipStream_t prev = nullptr, fresh = nullptr;     // streams of leg (3), destroyed at `done` whatever happens
    eclip_status st = ECLIP_OK;
    auto now = [] { return std::chrono::steady_clock::now(); };
    auto ns = [](std::chrono::steady_clock::time_point a, std::chrono::steady_clock::time_point b) {
        return (double)std::chrono::duration_cast<std::chrono::nanoseconds>(b - a).count();
    };
#define B_TRY(call)                                                                                       \
    do {                                                                                                  \
        hipError_t e_ = (call);                                                                           \
        if (e_ != hipSuccess) { st = fail(ECLIP_EHIP, "%s failed: %s", #call, hipGetErrorString(e_)); goto done; } \
    } while (0)
    B_TRY(hipEventCreateWithFlags(&ev[0], hipEventDisableTiming));
    B_TRY(hipEventCreateWithFlags(&ev[1], hipEventDisableTiming));
    B_TRY(hops.init(pool->device));
    {
        // warm-up
        for (int i = 0; i < 16; ++i) { B_TRY(launch_tick(d, A.stream)); }
        B_TRY(hipStreamSynchronize(A.stream));
        // (1) no repartitioning
        auto t0 = now();
        for (uint32_t i = 0; i < iters; ++i) B_TRY(launch_tick(d, A.stream));
        B_TRY(hipStreamSynchronize(A.stream));
        auto t1 = now();
        if (same_stream_ns) *same_stream_ns = ns(t0, t1) / iters;
        // (2) alternate between two pooled streams; each kernel waits for the previous one
        t0 = now();
        for (uint32_t i = 0; i < iters; ++i) {
            const hipStream_t cur = (i & 1) ? B.stream : A.stream, prev = (i & 1) ? A.stream : B.stream;
            if (i) B_TRY(hops.hop(prev, cur, ev[i & 1]));
            B_TRY(launch_tick(d, cur));
        }
        B_TRY(hipStreamSynchronize(A.stream));
        B_TRY(hipStreamSynchronize(B.stream));
        t1 = now();
        if (pooled_ns) *pooled_ns = ns(t0, t1) / iters;
        // (3) apply the mask at run time: a fresh masked stream per kernel
        if (create_ns) {
            const uint32_t n = std::min<uint32_t>(iters, 2000);
            std::vector<uint32_t> all_words((pool->device_cus + 31) / 32, 0u);
            const std::vector<uint32_t> *words = &B.words;
            if (B.words.empty()) {
                for (uint32_t c = 0; c < pool->device_cus; ++c) all_words[c / 32] |= 1u << (c % 32);
                words = &all_words;
            }
            // Timed: creating the masked stream and queueing the dependent kernel on it -- what applying a mask at run
            // time adds to a launch.  Draining and destroying the previous stream happen outside the accumulated
            // interval: that is teardown, not repartitioning.
            double acc = 0.0;
            for (uint32_t i = 0; i < n; ++i) {
                t0 = now();
                B_TRY(hipExtStreamCreateWithCUMask(&fresh, (uint32_t)words->size(), words->data()));
                if (prev) B_TRY(hipStreamWaitEvent(fresh, ev[0], 0));
                B_TRY(launch_tick(d, fresh));
                B_TRY(hipEventRecord(ev[0], fresh));
                t1 = now();
                acc += ns(t0, t1);
                if (prev) { B_TRY(hipStreamSynchronize(prev)); B_TRY(hipStreamDestroy(prev)); }
                prev = fresh;
                fresh = nullptr;
            }
            B_TRY(hipStreamSynchronize(prev));
            *create_ns = acc / n;
        }
    }
done:
#undef B_TRY
    if (fresh) { (void)hipStreamSynchronize(fresh); (void)hipStreamDestroy(fresh); }
    if (prev) { (void)hipStreamSynchronize(prev); (void)hipStreamDestroy(prev); }
    if (ev[0]) (void)hipEventDestroy(ev[0]);
    if (ev[1]) (void)hipEventDestroy(ev[1]);
    (void)hipDeviceSynchronize();
    hops.release();
    (void)hipFree(d);
    return st;
}
