// Context life cycle, stream status and the commit-and-drain step.
#include "hx_common.hpp"
#include "hx_search.hpp"
#include "hx_cp.hpp"
#include "hx_append.hpp"

void hx_dag_release(hx_ctx *ctx);   // hx_dag.hip
int hx_score_init();                // hx_score.hip
int hx_reveal_search(hx_ctx *ctx, const hx_model *model, const hx_calls *calls,
                     const hx_prefill_tab *pre, const hx_decode_tab *dec, const hx_links *links,
                     const float *tail, const float *horizon, int32_t n_nodes, int32_t n_wf,
                     int32_t *best_p, int32_t *best_d, float *best_cost, float *ratio,
                     const HxHorizonsPlan *reveal, bool *revealed, void *stream);   // hx_score.hip
int hx_relax_search(hx_ctx *ctx, const hx_model *model, const hx_calls *calls,
                    const hx_prefill_tab *pre, const hx_decode_tab *dec, const hx_links *links,
                    const float *tail, const float *horizon, int32_t n_nodes, int32_t n_wf,
                    int32_t *best_p, int32_t *best_d, float *best_cost, float *ratio,
                    const HxAppendPlan *walks, bool *merged, void *stream);         // hx_score.hip
int hx_plan_init();                 // hx_plan.hip
int hx_decode_init();               // hx_decode.hip

namespace {

char g_create_err[256] = "NULL context";   // why the last hx_ctx_create failed

int create_fail(const char *what, hipError_t e)
{
    snprintf(g_create_err, sizeof(g_create_err), "hx_ctx_create: %s: %s", what, hipGetErrorString(e));
    return HX_ERR_DEVICE;
}

__global__ void hx_clear_status_kernel(int32_t *status) { *status = 0; }

struct CommitArgs {
    int C, P, D;
    const int32_t *L_in, *L_out, *best_p, *best_d;
    int32_t *backlog, *used, *batch, *qd;
    const int32_t *drain_p, *drain_q, *release;
    int tokens_per_seq, max_batch;
    unsigned long long *acc;    // [P] backlog, [D] used, [D] qd additions of this round
    int32_t *status;
    int32_t *ticket;            // workgroups of the adding kernel that have delivered their sums (0 between launches); NULL: a drain launch follows
};

// The urgency fold of the same calls (Eq. (2)), for a round whose search ran before its horizons were there: the
// commit kernels form it as they pass over the calls.  ratio == NULL: no fold.
struct RatioArgs {
    const int32_t *node, *wf;
    const float *elapsed, *tail, *horizon, *best_cost;
    int n_nodes, n_wf;
    float *ratio;
};

__global__ __launch_bounds__(256) void hx_commit_clear_kernel(CommitArgs a)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < a.P + 2 * a.D) a.acc[i] = 0ull;
}

// sum of x over the lanes of `members` (all lanes of the wave take part)
__device__ __forceinline__ unsigned long long hx_wave_sum(unsigned long long x)
{
#pragma unroll
    for (int off = HX_WAVE / 2; off > 0; off >>= 1) x += __shfl_xor(x, off);
    return x;
}

// Adds, per distinct key among the lanes of the wave, the lanes' values into
// acc[key] with one LDS atomic per key (chosen placements concentrate on a few
// instances: 64 atomics on one address would serialise).
__device__ __forceinline__ void hx_add_by_key(unsigned long long *acc, bool valid, int key,
                                              unsigned long long v0, unsigned long long *acc1, unsigned long long v1)
{
    unsigned long long todo = __ballot(valid);
    const int lane = threadIdx.x & (HX_WAVE - 1);
    while (todo) {
        const int leader = __ffsll((long long)todo) - 1;
        const int k = __shfl(key, leader);
        const bool mine = valid && key == k;
        const unsigned long long s0 = hx_wave_sum(mine ? v0 : 0ull);
        const unsigned long long s1 = acc1 ? hx_wave_sum(mine ? v1 : 0ull) : 0ull;
        if (lane == leader) {
            atomicAdd(&acc[k], s0);
            if (acc1) atomicAdd(&acc1[k], s1);
        }
        todo &= ~__ballot(mine);
    }
}

__device__ __forceinline__ int hx_add_sat_drain(int cur, unsigned long long add, int drain, int32_t *status)
{
    unsigned long long total = (unsigned long long)(cur < 0 ? 0 : cur) + add;
    if (total > 2147483647ull) { hx_raise(status, HX_ERR_OVERFLOW); total = 2147483647ull; }
    long long left = (long long)total - (long long)drain;
    return left < 0 ? 0 : (left > 2147483647LL ? 2147483647 : (int)left);
}

// The state update of Algorithm 1 for all calls of the round at once: integer
// additions commute, so the result does not depend on call order.  Every wave
// first combines its calls per instance, every block sums into an LDS copy of
// the counters, and only the non-zero sums reach the global accumulators.
__global__ __launch_bounds__(256) void hx_commit_add_kernel(CommitArgs a, RatioArgs rt)
{
    __shared__ unsigned long long s_acc[3 * HX_MAX_INSTANCES];
    const int n_acc = a.P + 2 * a.D;
    for (int i = threadIdx.x; i < n_acc; i += blockDim.x) s_acc[i] = 0ull;
    __syncthreads();
    bool bad = false;
    const int stride = gridDim.x * blockDim.x;
    const int rounds = (a.C + stride - 1) / stride;          // the same trip count for every lane of a wave
    for (int it = 0; it < rounds; ++it) {
        const int c = it * stride + blockIdx.x * blockDim.x + threadIdx.x;
        int p = -1, d = -1, L = 0, O = 0;
        if (c < a.C) { p = a.best_p[c]; d = a.best_d[c]; L = a.L_in[c]; O = a.L_out[c]; }
        if (rt.ratio && c < a.C)
            hx_projected_ratio(rt.node, rt.wf, rt.elapsed, rt.tail, rt.horizon, rt.n_nodes, rt.n_wf, c, rt.best_cost[c], a.status, rt.ratio);
        bool valid = p >= 0 && d >= 0;                      // otherwise the call stays queued
        if (valid && (p >= a.P || d >= a.D || L < 0 || O < 0)) { bad = true; valid = false; }
        hx_add_by_key(s_acc, valid, p, (unsigned long long)L, nullptr, 0ull);
        hx_add_by_key(s_acc + a.P, valid, d, (unsigned long long)L + (unsigned long long)O,
                      s_acc + a.P + a.D, (unsigned long long)O);
    }
    if (bad) hx_raise(a.status, HX_ERR_INDEX);
    __syncthreads();
    unsigned long long seen = 0ull;
    for (int i = threadIdx.x; i < n_acc; i += blockDim.x)
        if (s_acc[i]) seen ^= atomicAdd(&a.acc[i], s_acc[i]);
    if (!a.ticket) return;
    // The workgroup that delivers last applies the drains: no second launch.  Everything the workgroups
    // exchange goes through device-scope atomics (the sums above, the ticket, and the accumulators read back with
    // an exchange that also leaves them at zero), so no cache has to be written back in between.  A workgroup
    // takes its ticket only after every one of its additions has returned its old value, i.e. has been
    // performed: the empty statement below needs those values, and the barrier follows it.
    asm volatile("" ::"v"((unsigned)(seen ^ (seen >> 32))) : "memory");
    __shared__ int s_last;
    __syncthreads();
    if (threadIdx.x == 0) {
        const int t = atomicAdd(a.ticket, 1);
        s_last = t == (int)gridDim.x - 1;
        if (s_last) __hip_atomic_store(a.ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (!s_last) return;
    for (int i = threadIdx.x; i < (a.P > a.D ? a.P : a.D); i += blockDim.x) {
        if (i < a.P) a.backlog[i] = hx_add_sat_drain(a.backlog[i], atomicExch(&a.acc[i], 0ull), a.drain_p ? a.drain_p[i] : 0, a.status);
        if (i < a.D) {
            a.qd[i] = hx_add_sat_drain(a.qd[i], atomicExch(&a.acc[a.P + a.D + i], 0ull), a.drain_q ? a.drain_q[i] : 0, a.status);
            const int used = hx_add_sat_drain(a.used[i], atomicExch(&a.acc[a.P + i], 0ull), a.release ? a.release[i] : 0, a.status);
            a.used[i] = used;
            long long b = ((long long)used + a.tokens_per_seq - 1) / a.tokens_per_seq;
            a.batch[i] = (int)(b > a.max_batch ? a.max_batch : b);
        }
    }
}

// Both steps in one workgroup, for rounds small enough that one compute unit adds them up as fast as a launch
// takes: the additions go into the workgroup's LDS counters with LDS atomics, and the same threads then apply
// the drains -- no global accumulators, one launch instead of two.  Same integer results.
constexpr int COMMIT_ONE_THREADS = 1024;
// rounds of at most this many calls are committed by the one-workgroup kernel: a launch saved (3-4 us of a small
// round).  Measured: 4096 calls already take it 2 us longer than the two launches (chosen placements concentrate
// on few instances, and lanes that meet on a counter wait for each other), 16384 calls 30 us longer.
constexpr int HX_COMMIT_ONE_LAUNCH = 1024;
__global__ __launch_bounds__(COMMIT_ONE_THREADS) void hx_commit_one_kernel(CommitArgs a, RatioArgs rt)
{
    __shared__ unsigned long long s_acc[3 * HX_MAX_INSTANCES];
    const int n_acc = a.P + 2 * a.D;
    for (int i = threadIdx.x; i < n_acc; i += COMMIT_ONE_THREADS) s_acc[i] = 0ull;
    __syncthreads();
    bool bad = false;
    const int rounds = (a.C + COMMIT_ONE_THREADS - 1) / COMMIT_ONE_THREADS;     // the same trip count for every lane
    for (int it = 0; it < rounds; ++it) {
        const int c = it * COMMIT_ONE_THREADS + threadIdx.x;
        int p = -1, d = -1, L = 0, O = 0;
        if (c < a.C) { p = a.best_p[c]; d = a.best_d[c]; L = a.L_in[c]; O = a.L_out[c]; }
        if (rt.ratio && c < a.C)
            hx_projected_ratio(rt.node, rt.wf, rt.elapsed, rt.tail, rt.horizon, rt.n_nodes, rt.n_wf, c, rt.best_cost[c], a.status, rt.ratio);
        bool valid = p >= 0 && d >= 0;
        if (valid && (p >= a.P || d >= a.D || L < 0 || O < 0)) { bad = true; valid = false; }
        if (valid) {       // LDS atomics: lanes that meet on a counter are serialised there, nowhere else
            atomicAdd(&s_acc[p], (unsigned long long)L);
            atomicAdd(&s_acc[a.P + d], (unsigned long long)L + (unsigned long long)O);
            atomicAdd(&s_acc[a.P + a.D + d], (unsigned long long)O);
        }
    }
    if (bad) hx_raise(a.status, HX_ERR_INDEX);
    __syncthreads();
    const int i = threadIdx.x;
    if (i < a.P) a.backlog[i] = hx_add_sat_drain(a.backlog[i], s_acc[i], a.drain_p ? a.drain_p[i] : 0, a.status);
    if (i < a.D) {
        a.qd[i] = hx_add_sat_drain(a.qd[i], s_acc[a.P + a.D + i], a.drain_q ? a.drain_q[i] : 0, a.status);
        const int used = hx_add_sat_drain(a.used[i], s_acc[a.P + i], a.release ? a.release[i] : 0, a.status);
        a.used[i] = used;
        long long b = ((long long)used + a.tokens_per_seq - 1) / a.tokens_per_seq;
        a.batch[i] = (int)(b > a.max_batch ? a.max_batch : b);
    }
}

__global__ __launch_bounds__(256) void hx_commit_drain_kernel(CommitArgs a)
{
    // the accumulators are left at zero for the next round
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < a.P) {
        a.backlog[i] = hx_add_sat_drain(a.backlog[i], a.acc[i], a.drain_p ? a.drain_p[i] : 0, a.status);
        a.acc[i] = 0ull;
    }
    if (i < a.D) {
        a.qd[i] = hx_add_sat_drain(a.qd[i], a.acc[a.P + a.D + i], a.drain_q ? a.drain_q[i] : 0, a.status);
        const int used = hx_add_sat_drain(a.used[i], a.acc[a.P + i], a.release ? a.release[i] : 0, a.status);
        a.used[i] = used;
        a.acc[a.P + i] = 0ull;
        a.acc[a.P + a.D + i] = 0ull;
        long long b = ((long long)used + a.tokens_per_seq - 1) / a.tokens_per_seq;
        a.batch[i] = (int)(b > a.max_batch ? a.max_batch : b);
    }
}

// ---- element-by-element check of a round's inputs (debug entry point) ----

struct ValidateArgs {
    int C, P, D, T, n_nodes, n_wf;
    const int32_t *L_in, *L_out, *node, *wf;
    const float *elapsed;
    const float *p_flops, *p_hbm;
    const int32_t *p_backlog, *p_type;
    const float *d_flops, *d_hbm;
    const int32_t *d_used, *d_cap, *d_batch, *d_qd, *d_type;
    const float *bw, *lat;
    int32_t *count;          // [HX_VALIDATE_FIELDS]
};

// classification on the bit pattern: the build assumes that no arithmetic sees a NaN
__device__ __forceinline__ bool hx_is_rate(float x)          // finite and > 0
{
    const unsigned b = __float_as_uint(x);
    return b > 0u && b < 0x7f800000u;
}
__device__ __forceinline__ bool hx_is_span(float x)          // finite and >= 0
{
    const unsigned b = __float_as_uint(x);
    return b < 0x7f800000u || b == 0x80000000u;
}

__global__ __launch_bounds__(256) void hx_validate_clear_kernel(int32_t *count)
{
    if (threadIdx.x < HX_VALIDATE_FIELDS) count[threadIdx.x] = 0;
}

__global__ __launch_bounds__(256) void hx_validate_kernel(ValidateArgs a)
{
    int bad[HX_VALIDATE_FIELDS];
#pragma unroll
    for (int k = 0; k < HX_VALIDATE_FIELDS; ++k) bad[k] = 0;
    const int stride = gridDim.x * blockDim.x;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < a.C; i += stride) {
        bad[HX_BAD_L_IN] += a.L_in[i] < 0;
        bad[HX_BAD_L_OUT] += a.L_out[i] < 0;
        if (a.node) bad[HX_BAD_NODE] += a.node[i] < 0 || a.node[i] >= a.n_nodes;
        if (a.wf) bad[HX_BAD_WF] += a.wf[i] < 0 || a.wf[i] >= a.n_wf;
        if (a.elapsed) bad[HX_BAD_ELAPSED] += !hx_is_span(a.elapsed[i]);
    }
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < a.P; i += stride) {
        bad[HX_BAD_PREFILL_RATE] += !hx_is_rate(a.p_flops[i]) || !hx_is_rate(a.p_hbm[i]);
        bad[HX_BAD_PREFILL_BACKLOG] += a.p_backlog[i] < 0;
        bad[HX_BAD_PREFILL_TYPE] += a.p_type[i] < 0 || a.p_type[i] >= a.T;
    }
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < a.D; i += stride) {
        bad[HX_BAD_DECODE_RATE] += !hx_is_rate(a.d_flops[i]) || !hx_is_rate(a.d_hbm[i]);
        bad[HX_BAD_DECODE_STATE] += a.d_used[i] < 0 || a.d_cap[i] < 0 || a.d_batch[i] < 0 || a.d_qd[i] < 0;
        bad[HX_BAD_DECODE_TYPE] += a.d_type[i] < 0 || a.d_type[i] >= a.T;
    }
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < a.T * a.T; i += stride)
        bad[HX_BAD_LINK] += !hx_is_rate(a.bw[i]) || (a.lat && !hx_is_span(a.lat[i]));
#pragma unroll
    for (int k = 0; k < HX_VALIDATE_FIELDS; ++k) {
        int v = bad[k];
#pragma unroll
        for (int off = HX_WAVE / 2; off > 0; off >>= 1) v += __shfl_xor(v, off);
        if ((threadIdx.x & (HX_WAVE - 1)) == 0 && v) atomicAdd(&a.count[k], v);
    }
}

// Scratch of hx_commit_static, the commit for callers that cannot allocate: the
// accumulators of one round, [P] backlog, [D] used, [D] qd additions, then a
// spare word that takes the status of a caller who passes none.  Each GPU the
// library runs on holds its own copy (25 KB) until the process ends.  In host
// code the array's name is only a handle for hipGetSymbolAddress; kernels get
// the address that call returned for the current device.
constexpr int HX_STATIC_ACC = 3 * HX_MAX_INSTANCES;
static __device__ __align__(256) unsigned long long scratch[HX_STATIC_ACC + 32];

constexpr int HX_MAX_DEVICES = 64;
unsigned long long *g_scratch_ptr[HX_MAX_DEVICES];   // device address of `scratch`, per device; NULL = not asked yet

// address of `scratch` on `device`, which must be the current device
hipError_t hx_static_scratch(int device, unsigned long long **out)
{
    unsigned long long *p = __atomic_load_n(&g_scratch_ptr[device], __ATOMIC_ACQUIRE);
    if (!p) {
        void *sym = nullptr;
        const hipError_t e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!sym) return hipErrorInvalidSymbol;
        p = (unsigned long long *)sym;
        __atomic_store_n(&g_scratch_ptr[device], p, __ATOMIC_RELEASE);   // every thread gets the same answer
    }
    *out = p;
    return hipSuccess;
}

int static_fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_create_err, sizeof(g_create_err), fmt, ap);
    va_end(ap);
    return code;
}

}  // namespace

extern "C" int hx_ctx_create(hx_ctx **out, int device)
{
    if (!out) return HX_ERR_INVALID_ARG;
    *out = nullptr;
    int count = 0;
    hipError_t e = hipGetDeviceCount(&count);
    if (e != hipSuccess) return create_fail("hipGetDeviceCount", e);
    if (device < 0 || device >= count) return create_fail("no such device", hipErrorInvalidDevice);
    HxDeviceGuard guard(device);
    if (!guard.ok) return create_fail("hipSetDevice", hipErrorInvalidDevice);
    hx_ctx *ctx = new (std::nothrow) hx_ctx();
    if (!ctx) return create_fail("out of host memory", hipErrorOutOfMemory);
    ctx->device = device;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) == hipSuccess && prop.multiProcessorCount > 0)
        ctx->num_cu = prop.multiProcessorCount;
    const char *what = "hipMalloc(status)";
    e = hipMalloc((void **)&ctx->d_status, sizeof(int32_t));
    if (e == hipSuccess) { what = "hipHostMalloc(status)"; e = hipHostMalloc((void **)&ctx->h_status, sizeof(int32_t), hipHostMallocDefault); }
    if (e == hipSuccess) { what = "hipMalloc(tables)"; e = hipMalloc((void **)&ctx->d_prep, sizeof(HxPrepTables)); }
    if (e == hipSuccess) { what = "hipMalloc(flags)"; e = hipMalloc((void **)&ctx->d_flags, HX_MAX_SWEEP_FLAGS * sizeof(int32_t)); }
    if (e == hipSuccess) { what = "hipMalloc(ticket)"; e = hipMalloc((void **)&ctx->d_ticket, sizeof(int32_t)); }
    if (e == hipSuccess) { what = "hipMalloc(accumulators)"; e = hipMalloc((void **)&ctx->d_acc, 3 * HX_MAX_INSTANCES * sizeof(unsigned long long)); }
    if (e == hipSuccess && device < HX_MAX_DEVICES) {     // set-up for hx_commit_static on this device
        what = "hipGetSymbolAddress(scratch)";
        unsigned long long *p = nullptr;
        e = hx_static_scratch(device, &p);
    }
    if (e == hipSuccess && (hx_score_init() != HX_OK || hx_plan_init() != HX_OK || hx_decode_init() != HX_OK)) { what = "hipFuncSetAttribute(LDS size)"; e = hipErrorInvalidValue; }
    if (e == hipSuccess) {
        what = "launch of hx_clear_status_kernel";
        CommitArgs z{};
        z.P = HX_MAX_INSTANCES; z.D = HX_MAX_INSTANCES; z.acc = ctx->d_acc;
        hx_commit_clear_kernel<<<(3 * HX_MAX_INSTANCES + 255) / 256, 256, 0, nullptr>>>(z);
        hx_clear_status_kernel<<<1, 1, 0, nullptr>>>(ctx->d_status);
        hx_clear_status_kernel<<<1, 1, 0, nullptr>>>(ctx->d_ticket);
        e = hipGetLastError();
    }
    if (e == hipSuccess) { what = "hipStreamSynchronize"; e = hipStreamSynchronize(nullptr); }
    if (e != hipSuccess) {
        hx_ctx_destroy(ctx);
        return create_fail(what, e);
    }
    *out = ctx;
    return HX_OK;
}

extern "C" int hx_ctx_destroy(hx_ctx *ctx)
{
    if (!ctx) return HX_ERR_INVALID_ARG;
    HxDeviceGuard guard(ctx->device);
    hx_dag_release(ctx);
    if (ctx->d_status) (void)hipFree(ctx->d_status);
    if (ctx->h_status) (void)hipHostFree(ctx->h_status);
    if (ctx->d_prep) (void)hipFree(ctx->d_prep);
    if (ctx->d_flags) (void)hipFree(ctx->d_flags);
    if (ctx->d_ticket) (void)hipFree(ctx->d_ticket);
    if (ctx->d_acc) (void)hipFree(ctx->d_acc);
    if (ctx->d_dpart) (void)hipFree(ctx->d_dpart);
    if (ctx->d_dtl) (void)hipFree(ctx->d_dtl);
    if (ctx->d_dtab) (void)hipFree(ctx->d_dtab);
    if (ctx->d_rkey) (void)hipFree(ctx->d_rkey);
    delete ctx;
    return HX_OK;
}

extern "C" const char *hx_last_error(const hx_ctx *ctx)
{
    return ctx ? ctx->err : g_create_err;
}

extern "C" int hx_stream_status(hx_ctx *ctx, void *stream_)
{
    if (!ctx) return HX_ERR_INVALID_ARG;
    HxDeviceGuard guard(ctx->device);
    HX_REQUIRE(ctx, guard.ok, HX_ERR_DEVICE, "cannot select device %d", ctx->device);
    hipStream_t stream = (hipStream_t)stream_;
    HX_HIP(ctx, hipMemcpyAsync(ctx->h_status, ctx->d_status, sizeof(int32_t), hipMemcpyDeviceToHost, stream));
    hx_clear_status_kernel<<<1, 1, 0, stream>>>(ctx->d_status);
    HX_HIP(ctx, hipStreamSynchronize(stream));
    const int code = *ctx->h_status;
    if (code != HX_OK) {
        const char *what = code == HX_ERR_NOT_DAG ? "an edge breaks the DAG order, or no fixed point within the sweep limit"
                         : code == HX_ERR_INDEX ? "an index held in a device array is out of range"
                         : code == HX_ERR_OVERFLOW ? "an instance counter exceeded INT32_MAX"
                         : code == HX_ERR_CAPACITY ? "a limit was hit on the device: propagation did not finish within max_depth sweeps, or an interval list is full"
                                                   : "device status";
        return hx_fail(ctx, code, "%s", what);
    }
    return HX_OK;
}

namespace {

// hx_commit, with the urgency fold of the same calls in the same launch when rt.ratio is given
int commit_round(hx_ctx *ctx, const hx_calls *calls, const int32_t *best_p, const int32_t *best_d,
                 int32_t P, int32_t *backlog_tok,
                 int32_t D, int32_t *used_tok, int32_t *batch, int32_t *qd_tok,
                 const int32_t *drain_prefill, const int32_t *drain_decode_q,
                 const int32_t *release_tok, int32_t tokens_per_seq, int32_t max_batch,
                 const RatioArgs &rt, void *stream_)
{
    HX_REQUIRE(ctx, calls, HX_ERR_INVALID_ARG, "NULL calls");
    const int C = calls->n;
    HX_REQUIRE(ctx, C >= 0 && P >= 0 && D >= 0, HX_ERR_INVALID_ARG, "negative size");
    HX_REQUIRE(ctx, P <= HX_MAX_INSTANCES && D <= HX_MAX_INSTANCES, HX_ERR_SHAPE,
               "pool %d x %d beyond %d instances per side", P, D, HX_MAX_INSTANCES);
    HX_REQUIRE(ctx, tokens_per_seq > 0 && max_batch >= 0, HX_ERR_INVALID_ARG, "tokens_per_seq must be positive");
    HX_REQUIRE(ctx, C == 0 || (calls->L_in && calls->L_out && best_p && best_d), HX_ERR_INVALID_ARG, "NULL call array");
    HX_REQUIRE(ctx, P == 0 || backlog_tok, HX_ERR_INVALID_ARG, "NULL backlog_tok");
    HX_REQUIRE(ctx, D == 0 || (used_tok && batch && qd_tok), HX_ERR_INVALID_ARG, "NULL decode array");
    if (P + D == 0) return HX_OK;
    HxDeviceGuard guard(ctx->device);
    HX_REQUIRE(ctx, guard.ok, HX_ERR_DEVICE, "cannot select device %d", ctx->device);
    hipStream_t stream = (hipStream_t)stream_;
    CommitArgs a{C, P, D, calls->L_in, calls->L_out, best_p, best_d, backlog_tok, used_tok, batch, qd_tok,
                 drain_prefill, drain_decode_q, release_tok, tokens_per_seq, max_batch, ctx->d_acc, ctx->d_status, nullptr};
    if (C <= HX_COMMIT_ONE_LAUNCH) {
        hx_commit_one_kernel<<<1, COMMIT_ONE_THREADS, 0, stream>>>(a, rt);
        return hx_check_launch(ctx, "hx_commit_one_kernel");
    }
    int grid = (C + 255) / 256;
    grid = grid > ctx->num_cu ? ctx->num_cu : grid;
    a.ticket = ctx->d_ticket;                  // the workgroup that finishes last applies the drains
    hx_commit_add_kernel<<<grid, 256, 0, stream>>>(a, rt);
    return hx_check_launch(ctx, "hx_commit_add_kernel");
}

}  // namespace

extern "C" int hx_commit(hx_ctx *ctx, const hx_calls *calls, const int32_t *best_p, const int32_t *best_d,
                         int32_t P, int32_t *backlog_tok,
                         int32_t D, int32_t *used_tok, int32_t *batch, int32_t *qd_tok,
                         const int32_t *drain_prefill, const int32_t *drain_decode_q,
                         const int32_t *release_tok, int32_t tokens_per_seq, int32_t max_batch,
                         void *stream_)
{
    if (!ctx) return HX_ERR_INVALID_ARG;
    return commit_round(ctx, calls, best_p, best_d, P, backlog_tok, D, used_tok, batch, qd_tok, drain_prefill, drain_decode_q,
                        release_tok, tokens_per_seq, max_batch, RatioArgs{}, stream_);
}

extern "C" int hx_commit_static(const hx_calls *calls, const int32_t *best_p, const int32_t *best_d,
                                int32_t P, int32_t *backlog_tok,
                                int32_t D, int32_t *used_tok, int32_t *batch, int32_t *qd_tok,
                                const int32_t *drain_prefill, const int32_t *drain_decode_q,
                                const int32_t *release_tok, int32_t tokens_per_seq, int32_t max_batch,
                                int32_t *status, void *stream_)
{
    if (!calls) return static_fail(HX_ERR_INVALID_ARG, "hx_commit_static: NULL calls");
    const int C = calls->n;
    if (C < 0 || P < 0 || D < 0) return static_fail(HX_ERR_INVALID_ARG, "hx_commit_static: negative size");
    if (P > HX_MAX_INSTANCES || D > HX_MAX_INSTANCES)
        return static_fail(HX_ERR_SHAPE, "hx_commit_static: pool %d x %d beyond the %d instances per side its static scratch holds",
                           P, D, HX_MAX_INSTANCES);
    if (tokens_per_seq <= 0 || max_batch < 0) return static_fail(HX_ERR_INVALID_ARG, "hx_commit_static: tokens_per_seq must be positive");
    if (C > 0 && !(calls->L_in && calls->L_out && best_p && best_d)) return static_fail(HX_ERR_INVALID_ARG, "hx_commit_static: NULL call array");
    if (P > 0 && !backlog_tok) return static_fail(HX_ERR_INVALID_ARG, "hx_commit_static: NULL backlog_tok");
    if (D > 0 && !(used_tok && batch && qd_tok)) return static_fail(HX_ERR_INVALID_ARG, "hx_commit_static: NULL decode array");
    if (P + D == 0) return HX_OK;
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return static_fail(HX_ERR_DEVICE, "hx_commit_static: hipGetDevice: %s", hipGetErrorString(e));
    if (device < 0 || device >= HX_MAX_DEVICES) return static_fail(HX_ERR_SHAPE, "hx_commit_static: device %d beyond the %d it keeps scratch for", device, HX_MAX_DEVICES);
    unsigned long long *acc = nullptr;
    e = hx_static_scratch(device, &acc);
    if (e != hipSuccess) return static_fail(HX_ERR_DEVICE, "hx_commit_static: hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    hipStream_t stream = (hipStream_t)stream_;
    CommitArgs a{C, P, D, calls->L_in, calls->L_out, best_p, best_d, backlog_tok, used_tok, batch, qd_tok,
                 drain_prefill, drain_decode_q, release_tok, tokens_per_seq, max_batch, acc,
                 status ? status : (int32_t *)(acc + HX_STATIC_ACC), nullptr};
    // the array keeps what the last call left: start from zero whatever that was
    // (a fill kernel, so that the call can be captured in a graph)
    hx_commit_clear_kernel<<<(P + 2 * D + 255) / 256, 256, 0, stream>>>(a);
    if (C > 0) {
        int grid = (C + 255) / 256;
        grid = grid > 256 ? 256 : grid;
        hx_commit_add_kernel<<<grid, 256, 0, stream>>>(a, RatioArgs{});
    }
    const int n_inst = P > D ? P : D;
    hx_commit_drain_kernel<<<(n_inst + 255) / 256, 256, 0, stream>>>(a);
    e = hipGetLastError();
    if (e != hipSuccess) return static_fail(HX_ERR_DEVICE, "hx_commit_static: launch: %s", hipGetErrorString(e));
    return HX_OK;
}

extern "C" int hx_validate_round(hx_ctx *ctx, const hx_calls *calls, const hx_prefill_tab *pre, const hx_decode_tab *dec,
                                 const hx_links *links, int32_t n_nodes, int32_t n_wf, int32_t *report, void *stream_)
{
    if (!ctx) return HX_ERR_INVALID_ARG;
    HX_REQUIRE(ctx, calls && pre && dec && links && report, HX_ERR_INVALID_ARG, "NULL table or report");
    const int C = calls->n, P = pre->n, D = dec->n, T = links->n_types;
    HX_REQUIRE(ctx, C >= 0 && P >= 0 && D >= 0 && n_nodes >= 0 && n_wf >= 0, HX_ERR_INVALID_ARG, "negative size");
    HX_REQUIRE(ctx, T >= 1 && T <= HX_MAX_TYPES, HX_ERR_SHAPE, "n_types %d outside 1..%d", T, HX_MAX_TYPES);
    HX_REQUIRE(ctx, C == 0 || (calls->L_in && calls->L_out), HX_ERR_INVALID_ARG, "NULL call array");
    HX_REQUIRE(ctx, P == 0 || (pre->flops && pre->hbm_bw && pre->backlog_tok && pre->type), HX_ERR_INVALID_ARG,
               "NULL member in prefill table");
    HX_REQUIRE(ctx, D == 0 || (dec->flops && dec->hbm_bw && dec->used_tok && dec->cap_tok && dec->batch && dec->qd_tok && dec->type),
               HX_ERR_INVALID_ARG, "NULL member in decode table");
    HX_REQUIRE(ctx, links->bw, HX_ERR_INVALID_ARG, "links.bw is NULL");
    HxDeviceGuard guard(ctx->device);
    HX_REQUIRE(ctx, guard.ok, HX_ERR_DEVICE, "cannot select device %d", ctx->device);
    hipStream_t stream = (hipStream_t)stream_;
    ValidateArgs a{C, P, D, T, n_nodes, n_wf, calls->L_in, calls->L_out, calls->node, calls->wf, calls->elapsed,
                   pre->flops, pre->hbm_bw, pre->backlog_tok, pre->type,
                   dec->flops, dec->hbm_bw, dec->used_tok, dec->cap_tok, dec->batch, dec->qd_tok, dec->type,
                   links->bw, links->latency, ctx->d_flags};
    int n = C > P ? C : P;
    n = n > D ? n : D;
    n = n > T * T ? n : T * T;
    int grid = (n + 255) / 256;
    grid = grid > ctx->num_cu * 4 ? ctx->num_cu * 4 : grid;
    hx_validate_clear_kernel<<<1, 256, 0, stream>>>(ctx->d_flags);
    hx_validate_kernel<<<grid, 256, 0, stream>>>(a);
    if (int rc = hx_check_launch(ctx, "hx_validate_kernel")) return rc;
    HX_HIP(ctx, hipMemcpyAsync(report, ctx->d_flags, HX_VALIDATE_FIELDS * sizeof(int32_t), hipMemcpyDeviceToHost, stream));
    HX_HIP(ctx, hipStreamSynchronize(stream));
    static const char *const what[HX_VALIDATE_FIELDS] = {
        "negative L_in", "negative L_out", "node outside 0..n_nodes-1", "wf outside 0..n_wf-1", "elapsed negative or not finite",
        "prefill flops or hbm_bw not a positive finite number", "negative backlog_tok", "prefill type outside 0..n_types-1",
        "decode flops or hbm_bw not a positive finite number", "negative used_tok, cap_tok, batch or qd_tok",
        "decode type outside 0..n_types-1", "link bandwidth not positive and finite, or latency negative or not finite"};
    for (int k = 0; k < HX_VALIDATE_FIELDS; ++k)
        if (report[k]) return hx_fail(ctx, HX_ERR_INVALID_ARG, "%d element(s): %s", report[k], what[k]);
    return HX_OK;
}

extern "C" int hx_round(hx_ctx *ctx, const hx_model *model, const hx_round_args *r, void *stream)
{
    if (!ctx) return HX_ERR_INVALID_ARG;
    HX_REQUIRE(ctx, model && r, HX_ERR_INVALID_ARG, "NULL model or round");
    HX_REQUIRE(ctx, r->n_new >= 0 && r->n_wf >= 0 && r->n_nodes >= 0, HX_ERR_INVALID_ARG, "negative size");
    HX_REQUIRE(ctx, r->n_new == 0 || r->n_nodes == 0, HX_ERR_INVALID_ARG,
               "a round reveals new nodes (n_new) or brings its whole graph (n_nodes), not both");
    int rc = HX_OK;
    const float *tail = nullptr, *horizon = nullptr;
    int32_t n_nodes = 0;
    if (r->n_nodes > 0) {
        // A small round's horizon refresh rides in the search's launch and its ratio in the commit's: two launches
        // instead of three, the two chains of memory round trips side by side.  Only where every argument check of
        // the three calls passes and the round fits (else nothing has been launched and the calls follow one
        // after the other, each reporting what it finds).
        HxHorizonsPlan plan;
        const int P = r->prefill.n, D = r->decode.n;
        const bool commit_ok = r->calls.n > 0 && P > 0 && D > 0 && P <= HX_MAX_INSTANCES && D <= HX_MAX_INSTANCES &&
                               r->tokens_per_seq > 0 && r->max_batch >= 0 && r->backlog_tok && r->used_tok && r->batch && r->qd_tok;
        bool revealed = false;
        if (commit_ok &&
            hx_horizons_plan(ctx, model, r->n_nodes, r->n_edges, r->succ_row_ptr, r->succ_col_idx, r->node_L_in, r->node_L_out,
                             r->n_types, r->type_flops, r->type_hbm_bw, &r->links, r->n_wf, r->wf_ptr,
                             r->node_cost, r->rem, r->tail, r->level, r->horizon, &plan) == HX_OK &&
            hx_reveal_search(ctx, model, &r->calls, &r->prefill, &r->decode, &r->links, r->tail, r->horizon, r->n_nodes, r->n_wf,
                             r->best_p, r->best_d, r->best_cost, r->ratio, &plan, &revealed, stream) == HX_OK &&
            revealed) {
            const RatioArgs rt{r->calls.node, r->calls.wf, r->calls.elapsed, r->tail, r->horizon, r->best_cost,
                               r->n_nodes, r->n_wf, r->ratio};
            return commit_round(ctx, &r->calls, r->best_p, r->best_d, P, r->backlog_tok, D, r->used_tok, r->batch, r->qd_tok,
                                r->drain_prefill, r->drain_decode_q, r->release_tok, r->tokens_per_seq, r->max_batch, rt, stream);
        }
        rc = hx_horizons(ctx, model, r->n_nodes, r->n_edges, r->succ_row_ptr, r->succ_col_idx, r->node_L_in, r->node_L_out,
                         r->n_types, r->type_flops, r->type_hbm_bw, &r->links, r->n_wf, r->wf_ptr,
                         r->node_cost, r->rem, r->tail, r->level, r->horizon, stream);
        if (rc != HX_OK) return rc;
        if (r->ratio) { tail = r->tail; horizon = r->horizon; n_nodes = r->n_nodes; }
    } else {
        // The append's walks ride in the search's launch, and the ratio in the commit's, where every argument check
        // passes and the search is large enough beside them: four launches instead of five, the walks' chain of
        // memory round trips under the search.  Else the walks are a launch of their own and the calls follow.
        HxAppendPlan ap{};
        bool merged = false;
        if (r->n_new > 0) {
            rc = hx_dag_append_begin(ctx, model, r->n_new, r->n_new_edges, r->parent_row_ptr, r->parent_col_idx,
                                     r->new_L_in, r->new_L_out, r->n_types, r->type_flops, r->type_hbm_bw, &r->links,
                                     r->new_cost, r->new_wf, &ap, stream);
            if (rc != HX_OK) return rc;
        }
        if (ap.grid > 0) {
            const int P = r->prefill.n, D = r->decode.n;
            const bool commit_ok = r->calls.n > 0 && P > 0 && D > 0 && P <= HX_MAX_INSTANCES && D <= HX_MAX_INSTANCES &&
                                   r->tokens_per_seq > 0 && r->max_batch >= 0 && r->backlog_tok && r->used_tok && r->batch && r->qd_tok;
            const float *g_tail = nullptr, *g_hor = nullptr;
            int32_t g_nodes = 0;
            if (commit_ok && hx_dag_view(ctx, nullptr, &g_tail, nullptr, &g_hor, &g_nodes) == HX_OK &&
                hx_relax_search(ctx, model, &r->calls, &r->prefill, &r->decode, &r->links, g_tail, g_hor, g_nodes + r->n_new, r->n_wf,
                                r->best_p, r->best_d, r->best_cost, r->ratio, &ap, &merged, stream) != HX_OK)
                merged = false;
            if (!merged) {
                rc = hx_dag_append_walks(ctx, &ap, stream);
                if (rc != HX_OK) return rc;
            }
            rc = hx_dag_append_end(ctx, &ap, stream);
            if (rc != HX_OK) return rc;
            if (merged) {
                rc = hx_dag_view(ctx, nullptr, &g_tail, nullptr, &g_hor, &g_nodes);
                if (rc != HX_OK) return rc;
                const RatioArgs rt{r->calls.node, r->calls.wf, r->calls.elapsed, g_tail, g_hor, r->best_cost, g_nodes, r->n_wf, r->ratio};
                return commit_round(ctx, &r->calls, r->best_p, r->best_d, P, r->backlog_tok, D, r->used_tok, r->batch, r->qd_tok,
                                    r->drain_prefill, r->drain_decode_q, r->release_tok, r->tokens_per_seq, r->max_batch, rt, stream);
            }
        }
        if (r->ratio) {
            rc = hx_dag_view(ctx, nullptr, &tail, nullptr, &horizon, &n_nodes);
            if (rc != HX_OK) return rc;
        }
    }
    rc = hx_score_placements(ctx, model, &r->calls, &r->prefill, &r->decode, &r->links, tail, horizon, n_nodes, r->n_wf,
                             nullptr, nullptr, r->best_p, r->best_d, r->best_cost, r->ratio, stream);
    if (rc != HX_OK) return rc;
    return hx_commit(ctx, &r->calls, r->best_p, r->best_d, r->prefill.n, r->backlog_tok, r->decode.n, r->used_tok, r->batch,
                     r->qd_tok, r->drain_prefill, r->drain_decode_q, r->release_tok, r->tokens_per_seq, r->max_batch, stream);
}
