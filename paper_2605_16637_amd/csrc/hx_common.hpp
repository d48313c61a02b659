// Shared host-side plumbing of the library: the context, error reporting and
// launch helpers.  Device arithmetic lives in hx_terms.hpp and the .hip files.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstring>

#include "../../include/hx.h"

constexpr int HX_WAVE = 64;
// decode entries are grouped by GPU class and each class segment is padded to
// a multiple of this many entries, so the inner search loop needs no tail
constexpr int HX_DGROUP = 8;
constexpr int HX_DPAD = HX_MAX_INSTANCES + HX_MAX_TYPES * HX_DGROUP;   // padded decode entries, upper bound

// Per-round tables the prepare kernel derives from the raw snapshots; one copy
// lives in the context's scratch and every scoring kernel stages it into LDS.
struct HxPrepTables {
    // prefill side, by instance
    float pre_wait[HX_MAX_INSTANCES];   // backlog_tok * phi / F
    float pre_invF[HX_MAX_INSTANCES];
    float pre_invB[HX_MAX_INSTANCES];
    int32_t pre_type[HX_MAX_INSTANCES];
    // decode side, by entry (grouped by class, padded); pads have orig = -1, free = -1
    float dec_wait[HX_DPAD];            // decode availability hint
    float dec_c1[HX_DPAD];              // phi * (batch + 1) / F
    float dec_c2[HX_DPAD];              // (omega + kappa * used) / B
    float dec_kB[HX_DPAD];              // kappa / B
    int32_t dec_free[HX_DPAD];          // cap_tok - used_tok
    int32_t dec_orig[HX_DPAD];          // instance index of the entry
    int32_t dec_type[HX_DPAD];          // class of the entry
    int32_t dec_pos[HX_MAX_INSTANCES];  // entry of instance d
    int32_t seg[HX_MAX_TYPES + 1];      // class t owns entries seg[t] .. seg[t+1]-1
    float link_invbw[HX_MAX_TYPES * HX_MAX_TYPES];
    float link_lat[HX_MAX_TYPES * HX_MAX_TYPES];
    int32_t n_entries;                  // seg[T]
};

struct HxDagStore {
    int32_t cap_nodes = 0, cap_edges = 0, cap_wf = 0, max_depth = 0;
    int32_t n_nodes = 0, n_edges = 0;
    float *cost = nullptr, *rem = nullptr, *tail = nullptr, *horizon = nullptr;
    int32_t *level = nullptr, *wf = nullptr, *parent_row_ptr = nullptr, *parent_col = nullptr;
    int32_t *parent0 = nullptr;        // [cap_nodes] a node's first parent (-1: none), beside its row of parent_col
    int32_t *mark = nullptr, *list[2] = {nullptr, nullptr};
    int32_t *counters = nullptr;       // [4]: list sizes (3, rotating) + epoch
    uint32_t epoch = 0;
};

struct hx_ctx {
    int device = 0;
    char err[256] = "no error";
    int32_t *d_status = nullptr;       // sticky device status word
    int32_t *h_status = nullptr;       // pinned copy
    HxPrepTables *d_prep = nullptr;
    int32_t *d_flags = nullptr;        // sweep "changed" flags, [HX_MAX_SWEEP_FLAGS]
    unsigned long long *d_acc = nullptr;   // commit accumulators, [3 * HX_MAX_INSTANCES]
    int32_t *d_ticket = nullptr;           // commit: workgroups that have delivered their sums; 0 between launches
    int32_t *d_dpart = nullptr;            // decode-stage free list and per-group partial results, dpart_cap words
    size_t dpart_cap = 0;
    unsigned long long *d_rkey = nullptr;  // sorted tiles of ordering keys, [rkey_cap]
    size_t rkey_cap = 0;
    void *d_dtl = nullptr;                 // decode-stage timelines (entries, lengths, stretches, sorted occupancies), dtl_cap entries
    size_t dtl_cap = 0;
    float *d_dtab = nullptr;               // decode-stage first-room tables, dtab_cap instances
    int dtab_cap = 0;
    int num_cu = 256;
    HxDagStore dag;
};

constexpr int HX_MAX_SWEEP_FLAGS = 4096;

inline int hx_fail(hx_ctx *ctx, int code, const char *fmt, ...)
{
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return code;
}

#define HX_HIP(ctx, call)                                                                  \
    do {                                                                                   \
        hipError_t e_ = (call);                                                            \
        if (e_ != hipSuccess)                                                              \
            return hx_fail((ctx), HX_ERR_DEVICE, "%s: %s", #call, hipGetErrorString(e_));  \
    } while (0)

#define HX_REQUIRE(ctx, cond, code, ...)                \
    do {                                                \
        if (!(cond)) return hx_fail((ctx), (code), __VA_ARGS__); \
    } while (0)

// Every kernel that can meet a bad element records the first error here.
__device__ inline void hx_raise(int32_t *status, int32_t code)
{
    // read first: when many threads meet the same bad input only a few reach the atomic
    if (__hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) atomicCAS(status, 0, code);
}

inline int hx_check_launch(hx_ctx *ctx, const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hx_fail(ctx, HX_ERR_DEVICE, "launch of %s: %s", what, hipGetErrorString(e));
    return HX_OK;
}

// hx_score.hip: validate the pool tables and enqueue the per-round table kernel (fills ctx->d_prep)
int hx_prepare_pool(hx_ctx *ctx, const hx_model *model, const hx_prefill_tab *pre, const hx_decode_tab *dec,
                    const hx_links *links, hipStream_t stream);

// set the device of the context for the duration of a call
struct HxDeviceGuard {
    int prev = -1;
    bool ok = true;
    explicit HxDeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) != hipSuccess) { ok = false; return; }
        if (prev != dev && hipSetDevice(dev) != hipSuccess) ok = false;
    }
    ~HxDeviceGuard()
    {
        int cur = -1;
        if (prev >= 0 && hipGetDevice(&cur) == hipSuccess && cur != prev) (void)hipSetDevice(prev);
    }
};
