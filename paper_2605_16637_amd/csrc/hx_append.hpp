// Device code of the incremental append's walks (Sec. 4.1, online reveal; Sec. 5.1, the horizon is refreshed at every
// reveal), shared by the append's own kernels in hx_dag.hip and by the scheduling round's merged launch in
// hx_score.hip.
#pragma once

#include "hx_common.hpp"

struct AppendArgs {
    int n_old, n_new, e_old, n_new_edges, cap_wf;
    const int32_t *new_row_ptr, *new_col, *new_wf;
    const float *new_cost;
    float *cost, *rem, *tail, *horizon;
    int32_t *level, *wf, *prow, *pcol, *parent0, *mark;
    int32_t *list_in, *list_out;
    int32_t *counters;      // [0..2] rotating list sizes
    int cin, cout, czero;   // which counter is read, appended to, cleared
    uint32_t epoch;
    int32_t *status;
};

// non-negative fp32 values order like their bit patterns
__device__ __forceinline__ bool hx_raise_max_f32(float *addr, float v)
{
    unsigned old = atomicMax((unsigned *)addr, __float_as_uint(v));
    return __float_as_uint(v) > old;
}

// push the (new) rem and level of node v to its parent u; enqueue u if it grew.  The lanes of a
// wavefront that enqueue at the same moment take their list slots with one atomic between them
// (the list counter is a single address: one atomic per lane would serialise the whole sweep).
// SCOPED: the list entry is written with a device-scope store (for the single-workgroup loop,
// whose later steps read the list back).
template <bool SCOPED>
__device__ __forceinline__ void hx_push_parent_t(const AppendArgs &a, int u, float rem_v, int level_v)
{
    bool grew = hx_raise_max_f32(&a.tail[u], rem_v);
    int old = atomicMax(&a.level[u], level_v + 1);
    grew = grew || (level_v + 1 > old);
    const bool want = grew && (uint32_t)atomicExch(&a.mark[u], (int)a.epoch) != a.epoch;
    const unsigned long long m = __builtin_amdgcn_ballot_w64(want);      // of the lanes active here
    if (m) {
        const int lane = (int)(threadIdx.x & (HX_WAVE - 1));
        const int leader = __ffsll((long long)m) - 1;
        int base = 0;
        if (lane == leader) base = atomicAdd(&a.counters[a.cout], __popcll(m));
        base = __shfl(base, leader);
        if (want) {
            const int slot = base + __popcll(m & ((1ull << lane) - 1ull));   // at most one entry per node and sweep:
            if (SCOPED) __hip_atomic_store(&a.list_out[slot], u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            else a.list_out[slot] = u;                                        // never beyond cap_nodes
        }
    }
}

// node u onto the worklist of the next sweep, once per sweep (rare path: one atomic per entry)
__device__ __forceinline__ void hx_enqueue(const AppendArgs &a, int u)
{
    if ((uint32_t)atomicExch(&a.mark[u], (int)a.epoch) != a.epoch) {
        const int slot = atomicAdd(&a.counters[a.cout], 1);
        a.list_out[slot] = u;
    }
}

__device__ __forceinline__ void hx_push_parent_scoped(const AppendArgs &a, int u, float rem_v, int level_v)
{
    hx_push_parent_t<true>(a, u, rem_v, level_v);
}

// Second phase of an append (a kernel boundary after init, so that a new node whose parent is
// also new finds that parent initialised).  Asynchronous propagation: every new node walks up from itself, one thread per new node.  A visit
// of node u recomputes rem[u] from the tail u has now, raises its workflow's horizon, and raises the
// tail and level of u's parents; a parent that grew is visited next (further grown parents wait on a
// small stack).  Whoever raises a node visits it afterwards with a tail at least as large as the one it left there, so
// every increase is carried upwards by someone, and a thread whose value did not raise anything
// stops: the fixed point is the same as that of the level-by-level sweeps, maxima are exact, and no
// launch or barrier separates the levels.  A walk that outgrows its stack or its step budget hands
// the remaining nodes to the worklist, which the sweeps after this kernel finish.
//
// A walk is a chain of memory round trips, and most of it goes up through first parents.  One round trip per
// level on that path: a node's first parent is kept beside its row of parents, so it is known when the node is
// reached; the two atomics that raise the parent return what it held before, which together with the raised value
// is what it holds now; and everything else the visit of the parent needs (cost, workflow, its own row and first
// parent -- nothing an append changes) is asked for together with those atomics.  Further parents, and nodes
// taken from the stack, pay the extra trips.
constexpr int RELAX_STACK = 16;
constexpr int RELAX_STEPS = 1024;

struct HxVisit {
    float cost, tl;
    int lv, w, e0, e1, q0;
};

// what a visit needs of node u that no append changes
__device__ __forceinline__ void hx_visit_fixed(const AppendArgs &a, int u, HxVisit &x)
{
    x.cost = a.cost[u]; x.w = a.wf[u]; x.e0 = a.prow[u]; x.e1 = a.prow[u + 1]; x.q0 = a.parent0[u];
}

// block, n_blocks: the workgroup's place among those that walk (the launch may hold other workgroups too)
__device__ __forceinline__ void hx_append_relax_body(const AppendArgs &a, int block, int n_blocks)
{
    for (int i = block * (int)blockDim.x + (int)threadIdx.x; i < a.n_new; i += n_blocks * (int)blockDim.x) {
        int stack[RELAX_STACK];
        int sp = 0, steps = 0;
        int u = a.n_old + i;
        HxVisit x;
        bool have = false;                   // x already describes u (reached through its child's first-parent slot)
        while (u >= 0) {
            if (!have) {
                x.tl = __hip_atomic_load(&a.tail[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                x.lv = __hip_atomic_load(&a.level[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                hx_visit_fixed(a, u, x);
            }
            const float r = x.cost + x.tl;
            const int lv = x.lv;
            hx_raise_max_f32(&a.rem[u], r);
            if (x.w >= 0) hx_raise_max_f32(&a.horizon[x.w], r);
            ++steps;
            int next = -1;
            have = false;
            const int e0 = x.e0, e1 = x.e1, q0 = x.q0;
            if (e1 > e0 && q0 >= 0) {
                // the first parent: raised, and its own visit prepared, in one round trip
                const unsigned old_t = atomicMax((unsigned *)&a.tail[q0], __float_as_uint(r));
                const int old_l = atomicMax(&a.level[q0], lv + 1);
                HxVisit y;
                hx_visit_fixed(a, q0, y);
                if (__float_as_uint(r) > old_t || lv + 1 > old_l) {
                    if (steps >= RELAX_STEPS) {
                        hx_enqueue(a, q0);
                    } else {
                        y.tl = __uint_as_float(max(old_t, __float_as_uint(r)));
                        y.lv = max(old_l, lv + 1);
                        x = y; next = q0; have = true;
                    }
                }
            }
            for (int e = e0 + 1; e < e1; ++e) {
                const int q = a.pcol[e];
                if (q < 0) continue;
                bool grew = hx_raise_max_f32(&a.tail[q], r);
                const int old = atomicMax(&a.level[q], lv + 1);
                grew = grew || (lv + 1 > old);
                if (!grew) continue;
                if (steps >= RELAX_STEPS) hx_enqueue(a, q);
                else if (next < 0) next = q;
                else if (sp < RELAX_STACK) stack[sp++] = q;
                else hx_enqueue(a, q);
            }
            u = next >= 0 ? next : (sp > 0 ? stack[--sp] : -1);
        }
    }
}


// An append in progress (hx_dag.hip): its first kernel has been launched, the walks and what follows them have
// not.  For the scheduling round, whose search can take the walks into its own launch.
struct HxAppendPlan {
    AppendArgs a;
    int grid;               // workgroups of 256 threads the walks would be launched with
    int n_new, n_new_edges;
};

int hx_dag_append_begin(hx_ctx *ctx, const hx_model *model, int32_t n_new, int32_t n_new_edges,
                        const int32_t *parent_row_ptr, const int32_t *parent_col_idx,
                        const int32_t *new_L_in, const int32_t *new_L_out,
                        int32_t n_types, const float *type_flops, const float *type_hbm_bw, const hx_links *links,
                        float *new_cost, const int32_t *new_wf, HxAppendPlan *plan, void *stream);
int hx_dag_append_walks(hx_ctx *ctx, const HxAppendPlan *plan, void *stream);
int hx_dag_append_end(hx_ctx *ctx, const HxAppendPlan *plan, void *stream);
