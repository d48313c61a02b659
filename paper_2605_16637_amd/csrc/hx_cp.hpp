// Device code of the standalone node cost and of the single-pass critical path (Sec. 5.1: the horizon H_w is the
// longest cost-weighted path of the revealed sub-DAG, rem[v] = cost[v] + max over successors of rem), shared by
// the kernels of hx_dag.hip and by the scheduling round's first kernel in hx_score.hip.
#pragma once

#include "hx_common.hpp"
#include "hx_terms.hpp"

#include <cmath>

constexpr int kT = HX_MAX_TYPES;

// ---- standalone node cost -----------------------------------------------------

struct NodeCostArgs {
    HxModelF m;
    int n, T;
    const int32_t *L_in, *L_out;
    const float *tF, *tB, *bw, *lat;
    float *cost;
};

// Per-class tables of the standalone cost, padded to kT x kT (a pair with a class
// that does not exist has infinite transfer latency), so that the pair loop
// unrolls completely and its table reads are LDS broadcasts.
struct CostTables {
    float invF[kT], invB[kT], c1[kT], c2[kT], kB[kT];
    float invbw[kT * kT], lat[kT * kT];
};

// filled by the first kT * kT threads of the block; a barrier follows at the caller's
__device__ __forceinline__ void hx_cost_tables_fill(CostTables &t, const NodeCostArgs &a, int tid)
{
    if (tid < kT) {
        const bool in = tid < a.T;
        float invF = in ? 1.0f / a.tF[tid] : 0.0f, invB = in ? 1.0f / a.tB[tid] : 0.0f;
        HxDecF d = hx_decode_terms(a.m, 0, 0, 0, invF, invB);
        t.invF[tid] = invF; t.invB[tid] = invB;
        // a padded class is excluded by an infinite link latency below; its own terms stay finite (0)
        t.c1[tid] = in ? d.c1 : 0.0f; t.c2[tid] = in ? d.c2 : 0.0f; t.kB[tid] = in ? d.kB : 0.0f;
    }
    if (tid < kT * kT) {
        const int tp = tid / kT, td = tid % kT;
        const bool in = tp < a.T && td < a.T;
        t.invbw[tid] = in ? 1.0f / a.bw[tp * a.T + td] : 0.0f;
        t.lat[tid] = in ? (a.lat ? a.lat[tp * a.T + td] : 0.0f) : INFINITY;
    }
}

// min over class pairs of prefill + transfer + decode on an idle pool.  T: classes in use (wave-uniform); the
// pairs beyond them would lose anyway (infinite latency in the padded tables) and are not evaluated.
__device__ __forceinline__ float hx_node_cost_eval(const HxModelF &m, const CostTables &t, int T, int L, int O)
{
    const HxCallF cf = hx_call_terms(m, L, O);
    float dec[kT];
#pragma unroll
    for (int td = 0; td < kT; ++td) dec[td] = td < T ? hx_decode_time(cf, t.c1[td], t.c2[td], t.kB[td]) : INFINITY;
    float best = INFINITY;
#pragma unroll
    for (int tp = 0; tp < kT; ++tp) {
        if (tp < T) {
            const float done = hx_prefill_done(cf, 0.0f, t.invF[tp], t.invB[tp]);
#pragma unroll
            for (int td = 0; td < kT; ++td) {
                if (td < T) {
                    const float x = hx_transfer(cf, t.invbw[tp * kT + td], t.lat[tp * kT + td]);
                    best = fminf(best, hx_candidate(done + x, 0.0f, dec[td]));
                }
            }
        }
    }
    return best;
}


// The same minimum with the prefill classes taken one after the other instead of all pairs at once: some twenty
// registers instead of two hundred, for kernels whose other work sets the register budget.  Every pair's cost is
// formed by the same functions on the same values, and a minimum does not depend on the order: the same bits.
__device__ __forceinline__ float hx_node_cost_eval_rolled(const HxModelF &m, const CostTables &t, int T, int L, int O)
{
    const HxCallF cf = hx_call_terms(m, L, O);
    float dec[kT];
#pragma unroll
    for (int td = 0; td < kT; ++td) dec[td] = td < T ? hx_decode_time(cf, t.c1[td], t.c2[td], t.kB[td]) : INFINITY;
    float best = INFINITY;
#pragma unroll 1
    for (int tp = 0; tp < T; ++tp) {
        const float done = hx_prefill_done(cf, 0.0f, t.invF[tp], t.invB[tp]);
#pragma unroll
        for (int td = 0; td < kT; ++td) {
            if (td < T) {
                const float x = hx_transfer(cf, t.invbw[tp * kT + td], t.lat[tp * kT + td]);
                best = fminf(best, hx_candidate(done + x, 0.0f, dec[td]));
            }
        }
    }
    return best;
}

// ---- critical path, single pass ---------------------------------------------------

struct CpArgs {
    int n_nodes, n_edges, n_wf;
    const int32_t *row_ptr, *col, *wf_ptr;
    const float *cost;
    float *rem, *tail, *horizon;
    int32_t *level;
    int32_t *status;
};

constexpr int CP_THREADS = 256;      // threads per block
constexpr int CP_WPB = 64;           // at most this many workflows per block, one walking lane each
constexpr int CP_NMAX = 1400;        // nodes staged per block
constexpr int CP_NMAX_COST = 1344;   // the same where the block also holds the class tables of the node cost
constexpr int CP_DEG = 4;            // successors a walking lane combines per step

// A node in LDS.  Before the walk reaches it: (cost, left); after: (rem, level, tail).
// s01/s23 hold its CP_DEG successors as 16-bit byte offsets of their records in
// the block's array, 0 for an empty slot: record 0 is (0, -1), what a node
// without successors takes its maximum over.  `left` marks a node whose slots
// are empty because staging left its row to the walk, which reads it from
// global memory: a node with more than CP_DEG successors, or one whose row
// starts within the last CP_DEG - 1 ids of the whole array.
struct __align__(16) CpNode { int rem_bits; int lvl; unsigned s01, s23; };
static_assert((CP_NMAX + 1) * sizeof(CpNode) <= 65536, "successor offsets are 16 bits");

// The walk of one lane over its workflow [ws, we), records in LDS at `base` (record 0 = the empty
// successor, node n0 + i at record i + 1).  LEFT: some node of the run was left to the walk (more
// successors than a record holds, or a row at the very end of the id array): such a node's row is
// read from global memory, edge by edge.  Returns whether an edge left the workflow.
template <bool LEFT>
__device__ __forceinline__ bool hx_cp_walk(const CpArgs &a, char *base, int n0, int ws, int we, float &hmax)
{
    bool not_dag = false;
    const unsigned lo = (unsigned)(ws - n0 + 1) * (unsigned)sizeof(CpNode);
    const unsigned hi = (unsigned)(we - n0 + 1) * (unsigned)sizeof(CpNode);
    int hbits = 0;
    unsigned umax = 0;
    uint4 cur = *(const uint4 *)(base + hi - sizeof(CpNode));
    for (unsigned p = hi - (unsigned)sizeof(CpNode); p >= lo; p -= (unsigned)sizeof(CpNode)) {
        // the node before this one (record 0 before the run's first: read, not used)
        const uint4 nxt = *(const uint4 *)(base + p - sizeof(CpNode));
        const unsigned u0 = cur.z & 0xffffu, u1 = cur.z >> 16, u2 = cur.w & 0xffffu, u3 = cur.w >> 16;
        const int2 g0 = *(const int2 *)(base + u0), g1 = *(const int2 *)(base + u1);
        const int2 g2 = *(const int2 *)(base + u2), g3 = *(const int2 *)(base + u3);
        umax = max(max(umax, u0), max(max(u1, u2), u3));
        int tb = max(max(g0.x, g1.x), max(max(g2.x, g3.x), 0));      // 0: the tail is never negative, whatever the costs
        int lv = max(max(g0.y, g1.y), max(g2.y, g3.y));
        if (LEFT && cur.y != 0) {
            const int v = (int)(p / (unsigned)sizeof(CpNode)) - 1;
            const int r0 = a.row_ptr[n0 + v], r1 = a.row_ptr[n0 + v + 1];       // found in range when staged
            for (int e = r0; e < r1; ++e) {
                const unsigned t = (unsigned)a.col[e] - (unsigned)(n0 + v + 1);   // distance beyond v + 1
                if (t < (unsigned)(we - n0 - v - 1)) {
                    const int2 g = *(const int2 *)(base + p + (t + 1) * (unsigned)sizeof(CpNode));
                    tb = max(tb, g.x); lv = max(lv, g.y);
                } else {
                    not_dag = true;
                }
            }
        }
        const float rv = __int_as_float((int)cur.x) + __int_as_float(tb);
        // (rem, level, tail): the successors of a finished node are not read again
        *(int2 *)(base + p) = make_int2(__float_as_int(rv), lv + 1);
        *(int *)(base + p + 8) = tb;
        hbits = max(hbits, __float_as_int(rv));
        cur = nxt;
    }
    hmax = __int_as_float(hbits);
    return not_dag || umax >= hi;                       // or an edge into a later workflow of the run
}

// One block takes `wpb` consecutive workflows; their nodes are a contiguous
// slice of the node arrays.
//  stage  one thread per node (a few nodes each, strided so that neighbouring
//         lanes read neighbouring words): cost and both ends of the node's row,
//         then its successor ids, every load of a stage issued before the first
//         is used.  The thread checks each edge as far as it can without
//         knowing the node's workflow (successor later than the node, inside the
//         block's slice) and parks the node in LDS as one 16-byte record.
//  walk   one lane per workflow (the lanes of one wave, a different wave in
//         consecutive blocks so that the walkers of a CU spread over its
//         SIMDs) walks the nodes from the last to the first.  A step is one
//         16-byte read (cost and successors of the next node, asked for one
//         step ahead), four 8-byte gathers, two three-way maxima each for rem
//         and level on integer bit patterns (max(0, .) of fp32 values that are
//         not NaN is the signed integer maximum of their bits with 0), and one
//         12-byte write.  What staging could not check -- a successor in a later
//         workflow of the same block -- shows in the largest offset the lane
//         has followed.  tail takes the place of the node's first successors.
//  store  every thread writes rem, level and tail of a few nodes, coalesced.
// Workflows that together exceed CP_NMAX nodes are taken in several runs, each
// as long as fits, one after the other; a single workflow of more than CP_NMAX
// nodes is walked in global memory by one lane (and so is every workflow, a
// lane each, of a graph with fewer than CP_DEG edges in all).
// COST: the node costs are not read but worked out here from the nodes' lengths (and written out as
// well), `nc` and `tab` being the arguments and the class tables of the standalone cost.
// STREAM: rem, level and tail leave with stores that do not claim cache lines (see the store phase).
// ROLLED: the cost's class pairs one after the other (hx_node_cost_eval_rolled), for a kernel with few registers to spare.
template <int NMAX, bool COST, bool STREAM, bool ROLLED = false>
__device__ __forceinline__ void hx_cp_local_body(const CpArgs &a, int wpb, CpNode *s_node, int &s_any,
                                                 const NodeCostArgs *nc, CostTables *tab, int block)
{
    // COST: the class tables are filled once, by the block's first run, after that run's own loads have been asked
    // for (the tables' loads and divisions then run under those instead of in front of them); block-uniform
    bool tab_ready = !COST;
    constexpr int CP_NMAX = NMAX;             // nodes staged per run
    constexpr int CP_NPT = (NMAX + CP_THREADS - 1) / CP_THREADS;
    const int tid = threadIdx.x;
    const int w0 = block * wpb;
    const int w1 = min(w0 + wpb, a.n_wf);
    // the walking lanes: wave (block mod 4), lane = workflow within the run
    const int wl = tid - ((block & 3) << 6);
    bool not_dag = false, bad_index = false;
    if (tid == 0) s_node[0] = CpNode{0, -1, 0u, 0u};
    char *const base = (char *)s_node;

    // the first run's bounds are read before anything is written: uniform loads of memory the kernel
    // has not touched go through the scalar cache
    const int n0_first = w0 < w1 ? a.wf_ptr[w0] : 0, n1_first = w0 < w1 ? a.wf_ptr[w1] : 0;
    for (int wa = w0; wa < w1;) {
        // the run [wa, wb): normally all of the block's workflows
        int wb = w1;
        // a walking lane's own bounds are asked for together with the run's (none of them waits for the other)
        int ws = 0, we = 0;
        if (wl >= 0 && wl < w1 - wa) { ws = a.wf_ptr[wa + wl]; we = a.wf_ptr[wa + wl + 1]; }
        const int n0 = wa == w0 ? n0_first : a.wf_ptr[wa];
        int n1 = wa == w0 ? n1_first : a.wf_ptr[wb];
        if (n0 >= 0 && n1 >= n0 && n1 - n0 > CP_NMAX) {
            int lo = wa, hi = wb;                       // wf_ptr[lo] - n0 fits, wf_ptr[hi] - n0 does not
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                const int x = a.wf_ptr[mid];
                if (x >= n0 && x - n0 <= CP_NMAX) lo = mid; else hi = mid;
            }
            wb = max(lo, wa + 1);
            n1 = a.wf_ptr[wb];
        }
        const bool walker = wl >= 0 && wl < wb - wa;
        // the slice of the run: malformed -> nothing is read, the error is reported
        if (n0 < 0 || n1 > a.n_nodes || n0 > n1) {
            bad_index = true;
            if (walker) a.horizon[wa + wl] = 0.0f;
            wa = wb;
            continue;
        }
        const int nn = n1 - n0;
        if (!walker) ws = we = n0;
        if (ws < n0 || we > n1 || ws > we) { bad_index = true; ws = we = n0; }   // this workflow is skipped
        float hmax = 0.0f;

        if (nn <= CP_NMAX && a.n_edges >= CP_DEG) {
            if (nn > 0) {
                float c[CP_NPT];
                int len_in[COST ? CP_NPT : 1], len_out[COST ? CP_NPT : 1];
                int ra[CP_NPT], rb[CP_NPT];
#pragma unroll
                for (int k = 0; k < CP_NPT; ++k) {
                    const int i = min(k * CP_THREADS + tid, nn - 1);   // a thread past the end repeats the last node
                    if constexpr (COST) { len_in[k] = nc->L_in[n0 + i]; len_out[k] = nc->L_out[n0 + i]; }
                    else c[k] = a.cost[n0 + i];
                    ra[k] = a.row_ptr[n0 + i];
                    rb[k] = a.row_ptr[n0 + i + 1];
                }
                // the first CP_DEG ids of each row in one 16-byte load.  A row of more than CP_DEG ids, or one
                // that starts within the last CP_DEG - 1 ids of the whole array (where such a load would run
                // past the end), is left to the walk.
                int ed[CP_NPT][CP_DEG];
                int deg[CP_NPT];
                const int e_last4 = a.n_edges - CP_DEG;
#pragma unroll
                for (int k = 0; k < CP_NPT; ++k) {
                    if (ra[k] < 0 || rb[k] > a.n_edges || ra[k] > rb[k]) { bad_index = true; ra[k] = rb[k] = 0; }
                    __builtin_memcpy(ed[k], a.col + min(ra[k], e_last4), sizeof(int) * CP_DEG);
                    deg[k] = rb[k] - ra[k];
                    if (deg[k] > CP_DEG || (deg[k] > 0 && ra[k] > e_last4)) { deg[k] = -1; s_any = wa + 1; }
                }
                if constexpr (COST) if (!tab_ready) {
                    hx_cost_tables_fill(*tab, *nc, tid);
                    __syncthreads();
                    tab_ready = true;
                }
                // the costs are worked out (COST) and parked while the ids are on their way
#pragma unroll
                for (int k = 0; k < CP_NPT; ++k) {
                    const int i = k * CP_THREADS + tid;
                    if constexpr (COST) if (i < nn) {
                        c[k] = ROLLED ? hx_node_cost_eval_rolled(nc->m, *tab, nc->T, len_in[k], len_out[k])
                                      : hx_node_cost_eval(nc->m, *tab, nc->T, len_in[k], len_out[k]);
                        nc->cost[n0 + i] = c[k];
                    }
                    if (i < nn) *(int2 *)&s_node[i + 1] = make_int2(__float_as_int(c[k]), deg[k] < 0);
                    deg[k] = max(deg[k], 0);                         // a node left to the walk keeps no slots
                }
#pragma unroll
                for (int k = 0; k < CP_NPT; ++k) {
                    const int i = k * CP_THREADS + tid;
                    const int ic = min(i, nn - 1);
                    // a legal successor is one of ic+1 .. nn-1: one unsigned compare of its distance beyond ic+1
                    const int first = n0 + ic + 1;
                    const unsigned span = (unsigned)(nn - 1 - ic);
                    const unsigned off = (unsigned)(ic + 2) * (unsigned)sizeof(CpNode);
                    unsigned slot[CP_DEG];
                    int n_ok = 0;
#pragma unroll
                    for (int j = 0; j < CP_DEG; ++j) {
                        const unsigned t = (unsigned)ed[k][j] - (unsigned)first;
                        const bool ok = t < (deg[k] > j ? span : 0u);   // a slot past the end of the row has no legal id
                        n_ok += ok;
                        slot[j] = ok ? t * (unsigned)sizeof(CpNode) + off : 0u;
                    }
                    if (n_ok != deg[k]) not_dag = true;              // an edge backwards or out of the run's slice
                    if (i < nn) *(uint2 *)&s_node[i + 1].s01 = make_uint2(slot[0] | (slot[1] << 16), slot[2] | (slot[3] << 16));
                }
            }
            __syncthreads();

            if (we > ws) {                              // a walking lane with a non-empty workflow
                const bool bad = s_any == wa + 1 ? hx_cp_walk<true>(a, base, n0, ws, we, hmax)
                                                 : hx_cp_walk<false>(a, base, n0, ws, we, hmax);
                not_dag = not_dag || bad;
            }
            __syncthreads();
#pragma unroll
            for (int k = 0; k < CP_NPT; ++k) {
                const int i = k * CP_THREADS + tid;
                if (i < nn) {
                    const int4 me = *(const int4 *)&s_node[i + 1];
                    if constexpr (STREAM) {
                        // a graph far larger than the caches: stores that do not claim cache lines (measured on the
                        // 2 M-node stress graph: 17.2 -> 14.4 us per launch; the same hint on the loads of a stage
                        // costs 2-5 us).  A round's graph of 10^4 - 10^5 nodes is read again by the next kernel of
                        // the round and is better left in the caches.
                        __builtin_nontemporal_store(__int_as_float(me.x), &a.rem[n0 + i]);
                        __builtin_nontemporal_store(me.y, &a.level[n0 + i]);
                        __builtin_nontemporal_store(__int_as_float(me.z), &a.tail[n0 + i]);
                    } else {
                        a.rem[n0 + i] = __int_as_float(me.x);
                        a.level[n0 + i] = me.y;
                        a.tail[n0 + i] = __int_as_float(me.z);
                    }
                }
            }
            __syncthreads();                            // the next run stages over these records
        } else {
            // walked in global memory
            if constexpr (COST) if (!tab_ready) {
                hx_cost_tables_fill(*tab, *nc, tid);
                __syncthreads();
                tab_ready = true;
            }
            for (int v = we - 1; v >= ws; --v) {
                int r0 = a.row_ptr[v], r1 = a.row_ptr[v + 1];
                if (r0 < 0 || r1 > a.n_edges || r0 > r1) { bad_index = true; r0 = r1 = 0; }
                float tl = 0.0f;
                int lv = 0;
                for (int e = r0; e < r1; ++e) {
                    int u = a.col[e];
                    if (u <= v || u >= we) { not_dag = true; continue; }
                    tl = fmaxf(tl, a.rem[u]);          // written earlier by this same thread
                    lv = max(lv, a.level[u] + 1);
                }
                float cv;
                if constexpr (COST) {
                    cv = ROLLED ? hx_node_cost_eval_rolled(nc->m, *tab, nc->T, nc->L_in[v], nc->L_out[v])
                                : hx_node_cost_eval(nc->m, *tab, nc->T, nc->L_in[v], nc->L_out[v]);
                    nc->cost[v] = cv;
                }
                else cv = a.cost[v];
                float rv = cv + tl;
                a.rem[v] = rv; a.tail[v] = tl; a.level[v] = lv;
                hmax = fmaxf(hmax, rv);
            }
        }
        if (walker) a.horizon[wa + wl] = hmax;
        wa = wb;
    }
    if (not_dag) hx_raise(a.status, HX_ERR_NOT_DAG);
    if (bad_index) hx_raise(a.status, HX_ERR_INDEX);
}

// seven blocks of 22.4 KB per compute unit, 72 vector registers

// hx_horizons as its argument checks and launch shape without the launch (hx_dag.hip): for the scheduling round's
// first kernel, whose first workgroups do the same work.  grid == 0: there is nothing to launch.
struct HxHorizonsPlan {
    CpArgs a;
    NodeCostArgs nc;
    int wpb, grid;
};

int hx_horizons_plan(hx_ctx *ctx, const hx_model *model, int32_t n_nodes, int32_t n_edges,
                     const int32_t *succ_row_ptr, const int32_t *succ_col_idx,
                     const int32_t *L_in, const int32_t *L_out,
                     int32_t n_types, const float *type_flops, const float *type_hbm_bw, const hx_links *links,
                     int32_t n_wf, const int32_t *wf_ptr,
                     float *node_cost, float *rem, float *tail, int32_t *level, float *horizon, HxHorizonsPlan *plan);
