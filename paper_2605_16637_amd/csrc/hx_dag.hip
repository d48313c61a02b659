// Workflow horizons: standalone node cost, the max-plus critical-path pass
// (single-pass workflow-local form and level-synchronous general form) and the
// incremental append for DAGs revealed at run time.
//
// What is computed: Sec. 5.1 of the paper.  H_w(t) is the completion time of
// the revealed sub-DAG of workflow w served in isolation; it is recomputed when
// calls are revealed and can only grow.  Here that is the longest
// cost-weighted path, with rem[v] = cost[v] + max over successors of rem.
//
// rem is one fp32 addition of an exact maximum, so every evaluation order --
// the single pass, the sweeps, the incremental propagation -- gives the same
// bits.
#include "hx_common.hpp"
#include "hx_terms.hpp"
#include "hx_cp.hpp"
#include "hx_append.hpp"

#include <cmath>

namespace {

// ---- standalone node cost -----------------------------------------------------

__global__ __launch_bounds__(256) void hx_node_cost_kernel(NodeCostArgs a)
{
    __shared__ CostTables s_tab;
    const int tid = threadIdx.x;
    // the first node's lengths are on their way while the class tables are set up
    const int v0 = blockIdx.x * blockDim.x + tid;
    int L = v0 < a.n ? a.L_in[v0] : 0, O = v0 < a.n ? a.L_out[v0] : 0;
    hx_cost_tables_fill(s_tab, a, tid);
    __syncthreads();
    for (int v = v0; v < a.n; v += gridDim.x * blockDim.x) {
        const int Lv = L, Ov = O;
        const int vn = v + gridDim.x * blockDim.x;
        if (vn < a.n) { L = a.L_in[vn]; O = a.L_out[vn]; }
        a.cost[v] = hx_node_cost_eval(a.m, s_tab, a.T, Lv, Ov);
    }
}


// ---- critical path, single pass ---------------------------------------------------

template <bool STREAM>
__global__ __launch_bounds__(CP_THREADS) __attribute__((amdgpu_waves_per_eu(7, 8)))
void hx_cp_local_kernel(CpArgs a, int wpb)
{
    __shared__ CpNode s_node[CP_NMAX + 1];
    __shared__ int s_any;                     // == first workflow of the run + 1: a node of this run was left to the walk
    hx_cp_local_body<CP_NMAX, false, STREAM>(a, wpb, s_node, s_any, nullptr, nullptr, (int)blockIdx.x);
}

// The same pass with the standalone node cost worked out while staging instead of being read:
// one launch for what hx_node_cost_kernel and hx_cp_local_kernel do one after the other.  The
// evaluation of 64 class pairs per node wants more registers than seven blocks per compute unit
// leave; the launch is meant for the graphs of a scheduling round (tens of thousands of nodes,
// spread over all compute units), where the latency of a launch counts and residency does not.
__global__ __launch_bounds__(CP_THREADS)
void hx_cp_cost_kernel(CpArgs a, NodeCostArgs nc, int wpb)
{
    __shared__ CpNode s_node[CP_NMAX_COST + 1];
    __shared__ int s_any;
    __shared__ CostTables s_tab;
    hx_cp_local_body<CP_NMAX_COST, true, false>(a, wpb, s_node, s_any, &nc, &s_tab, (int)blockIdx.x);
}

// ---- critical path, level-synchronous sweeps ------------------------------------------

__global__ __launch_bounds__(256) void hx_cp_init_kernel(CpArgs a, int32_t *flags, int n_flags)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < a.n_nodes) { a.rem[i] = a.cost[i]; a.tail[i] = 0.0f; a.level[i] = 0; }
    if (i < n_flags) flags[i] = (i == 0) ? 1 : 0;      // flags[s] != 0: sweep s changed something
}

// Sweep s: every node pulls from its successors.  Values only grow towards the
// fixed point; a sweep in which nothing changed has read only final values.
// Runs only if the previous sweep changed something.
__global__ __launch_bounds__(256) void hx_cp_sweep_kernel(CpArgs a, int32_t *flags, int s)
{
    if (__hip_atomic_load(&flags[s - 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) return;
    bool changed = false, bad = false;
    for (int v = blockIdx.x * blockDim.x + threadIdx.x; v < a.n_nodes; v += gridDim.x * blockDim.x) {
        int r0 = a.row_ptr[v], r1 = a.row_ptr[v + 1];
        if (r0 < 0 || r1 > a.n_edges || r0 > r1) { bad = true; continue; }
        float tl = 0.0f;
        int lv = 0;
        for (int e = r0; e < r1; ++e) {
            int u = a.col[e];
            if (u < 0 || u >= a.n_nodes) { bad = true; continue; }
            tl = fmaxf(tl, __hip_atomic_load(&a.rem[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            lv = max(lv, __hip_atomic_load(&a.level[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1);
        }
        // a level beyond the node count can only come from a cycle: stop growing
        lv = min(lv, a.n_nodes);
        if (tl != a.tail[v] || lv != a.level[v]) {
            changed = true;
            a.tail[v] = tl;
            __hip_atomic_store(&a.level[v], lv, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&a.rem[v], a.cost[v] + tl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if (changed) flags[s] = 1;
    if (bad) hx_raise(a.status, HX_ERR_INDEX);
}

__global__ __launch_bounds__(256) void hx_cp_finish_kernel(CpArgs a, const int32_t *flags, int last)
{
    const int w = blockIdx.x * blockDim.x + threadIdx.x;
    if (w == 0 && flags[last] != 0) hx_raise(a.status, HX_ERR_NOT_DAG);
    if (w >= a.n_wf) return;
    int s = a.wf_ptr[w], e = a.wf_ptr[w + 1];
    if (s < 0 || e > a.n_nodes || s > e) { hx_raise(a.status, HX_ERR_INDEX); a.horizon[w] = 0.0f; return; }
    float h = 0.0f;
    for (int v = s; v < e; ++v) h = fmaxf(h, a.rem[v]);
    a.horizon[w] = h;
}

// ---- incremental append ------------------------------------------------------------------

// First phase of an append: the new nodes' own entries.  The two list counters the append needs at zero (the
// one the walks append to, the one the first sweep after them clears) are cleared here: the walks are a launch
// of their own after this one, so no launch is spent on the counters.
// COST: the nodes' standalone costs are not read but worked out here from their lengths, exactly as
// hx_node_cost_kernel does, and written to the caller's array as well (one launch less in front of the walks, where
// every launch of a round still waits for the host).
template <bool COST>
__global__ __launch_bounds__(256) void hx_append_init_kernel(AppendArgs a, NodeCostArgs nc)
{
    __shared__ CostTables s_tab;
    if constexpr (COST) {
        hx_cost_tables_fill(s_tab, nc, threadIdx.x);
        __syncthreads();
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) { a.counters[a.czero] = 0; a.counters[a.cout] = 0; }
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < a.n_new; i += gridDim.x * blockDim.x) {
        const int v = a.n_old + i;
        float c;
        if constexpr (COST) {
            c = hx_node_cost_eval(nc.m, s_tab, nc.T, nc.L_in[i], nc.L_out[i]);
            nc.cost[i] = c;
        } else {
            c = a.new_cost[i];
        }
        int w = a.new_wf[i];
        int r0 = a.new_row_ptr[i], r1 = a.new_row_ptr[i + 1];
        if (r0 < 0 || r1 > a.n_new_edges || r0 > r1) { hx_raise(a.status, HX_ERR_INDEX); r0 = r1 = min(max(r0, 0), a.n_new_edges); }
        a.cost[v] = c; a.rem[v] = c; a.tail[v] = 0.0f; a.level[v] = 0; a.mark[v] = 0;
        a.prow[v + 1] = a.e_old + r1;
        if (w < 0 || w >= a.cap_wf) { hx_raise(a.status, HX_ERR_INDEX); w = -1; }
        a.wf[v] = w;
        if (w >= 0) hx_raise_max_f32(&a.horizon[w], c);
        int first = -1;
        for (int e = r0; e < r1; ++e) {
            int u = a.new_col[e];
            if (u < 0 || u >= v) { hx_raise(a.status, HX_ERR_NOT_DAG); u = -1; }
            a.pcol[a.e_old + e] = u;
            if (e == r0) first = u;
        }
        a.parent0[v] = first;
    }
}

__global__ __launch_bounds__(256) void hx_append_relax_kernel(AppendArgs a)
{
    hx_append_relax_body(a, (int)blockIdx.x, (int)gridDim.x);
}

__global__ void hx_append_finish_kernel(AppendArgs a)
{
    if (threadIdx.x == 0 && a.counters[a.cin] != 0) hx_raise(a.status, HX_ERR_CAPACITY);
}

// The remaining sweeps in one workgroup: after a few grid-wide sweeps the lists
// are short, and what is left is a chain of dependent steps -- one launch loops
// over them until the list is empty (or `sweeps` steps are done) instead of one
// launch per step.  Every value another thread may have written is read with a
// device-scope load.
__global__ __launch_bounds__(1024) void hx_append_tail_kernel(AppendArgs a, int32_t *list0, int32_t *list1,
                                                              int first, int sweeps)
{
    __shared__ int s_n;
    for (int s = first; s < first + sweeps; ++s) {
        a.cin = (s + 1) % 3; a.cout = (s + 2) % 3; a.czero = s % 3;
        a.list_in = (s & 1) ? list1 : list0;
        a.list_out = (s & 1) ? list0 : list1;
        a.epoch += 1;
        if (threadIdx.x == 0) {
            s_n = __hip_atomic_load(&a.counters[a.cin], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&a.counters[a.czero], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        const int n = s_n;
        if (n == 0) break;                                   // uniform: nothing left to propagate
        for (int i = threadIdx.x; i < n; i += blockDim.x) {
            const int u = __hip_atomic_load(&a.list_in[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const float tl = __hip_atomic_load(&a.tail[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int lv = __hip_atomic_load(&a.level[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const float r = a.cost[u] + tl;
            a.rem[u] = r;
            const int w = a.wf[u];
            if (w >= 0) hx_raise_max_f32(&a.horizon[w], r);
            for (int e = a.prow[u]; e < a.prow[u + 1]; ++e) {
                int q = a.pcol[e];
                if (q >= 0) hx_push_parent_scoped(a, q, r, lv);
            }
        }
        __threadfence();
        __syncthreads();
    }
    // the list the last step wrote must be empty, or the depth limit was too small
    if (threadIdx.x == 0) {
        const int last = (first + sweeps + 1) % 3;
        if (__hip_atomic_load(&a.counters[last], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0 &&
            s_n != 0) hx_raise(a.status, HX_ERR_CAPACITY);
    }
}

// cost of existing nodes replaced by observed values (an id outside the graph is skipped and reported)
__global__ __launch_bounds__(256) void hx_set_cost_kernel(int n, const int32_t *ids, const float *value, float *cost, int n_nodes,
                                                          int32_t *status)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int v = ids[i];
    if (v < 0 || v >= n_nodes) { hx_raise(status, HX_ERR_INDEX); return; }
    cost[v] = value[i];
}

// everything the costs determine back to its starting point: rem = cost, no tail, no horizon
__global__ __launch_bounds__(256) void hx_refresh_reset_kernel(AppendArgs a, int n_wf)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < a.n_new) { a.rem[i] = a.cost[i]; a.tail[i] = 0.0f; }
    if (i < n_wf) a.horizon[i] = 0.0f;
    if (i < 3) a.counters[i] = 0;
}

__global__ __launch_bounds__(256) void hx_fill_i32_kernel(int32_t *p, size_t n, int32_t v)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

template <typename T>
int dev_alloc(hx_ctx *ctx, T **p, size_t n)
{
    *p = nullptr;
    HX_HIP(ctx, hipMalloc((void **)p, (n ? n : 1) * sizeof(T)));
    return HX_OK;
}

void dag_free(HxDagStore &g)
{
    void *ptrs[] = {g.cost, g.rem, g.tail, g.horizon, g.level, g.wf, g.parent_row_ptr, g.parent_col, g.parent0,
                    g.mark, g.list[0], g.list[1], g.counters};
    for (void *p : ptrs) if (p) (void)hipFree(p);
    g = HxDagStore{};
}

}  // namespace

void hx_dag_release(hx_ctx *ctx) { dag_free(ctx->dag); }

namespace {

// the argument checks of the standalone cost, and its kernel arguments
int node_cost_args(hx_ctx *ctx, const hx_model *model, int32_t n, const int32_t *L_in, const int32_t *L_out,
                   int32_t n_types, const float *type_flops, const float *type_hbm_bw, const hx_links *links, float *cost,
                   NodeCostArgs *out)
{
    HX_REQUIRE(ctx, model && links && links->bw && type_flops && type_hbm_bw, HX_ERR_INVALID_ARG, "NULL table");
    HX_REQUIRE(ctx, n >= 0, HX_ERR_INVALID_ARG, "negative n");
    HX_REQUIRE(ctx, n_types >= 1 && n_types <= HX_MAX_TYPES && links->n_types == n_types, HX_ERR_SHAPE,
               "n_types %d (links %d) outside 1..%d", n_types, links->n_types, HX_MAX_TYPES);
    HX_REQUIRE(ctx, n == 0 || (L_in && L_out && cost), HX_ERR_INVALID_ARG, "NULL array");
    NodeCostArgs a{};
    a.m = HxModelF{model->kv_bytes_per_token, model->flops_per_token, model->attn_flops_per_token2,
                   model->weight_bytes, model->nominal_batch};
    a.n = n; a.T = n_types; a.L_in = L_in; a.L_out = L_out; a.tF = type_flops; a.tB = type_hbm_bw;
    a.bw = links->bw; a.lat = links->latency; a.cost = cost;
    *out = a;
    return HX_OK;
}

}  // namespace

extern "C" int hx_node_cost(hx_ctx *ctx, const hx_model *model, int32_t n,
                            const int32_t *L_in, const int32_t *L_out,
                            int32_t n_types, const float *type_flops, const float *type_hbm_bw,
                            const hx_links *links, float *cost, void *stream_)
{
    if (!ctx) return HX_ERR_INVALID_ARG;
    NodeCostArgs a{};
    if (int rc = node_cost_args(ctx, model, n, L_in, L_out, n_types, type_flops, type_hbm_bw, links, cost, &a)) return rc;
    if (n == 0) return HX_OK;
    HxDeviceGuard guard(ctx->device);
    HX_REQUIRE(ctx, guard.ok, HX_ERR_DEVICE, "cannot select device %d", ctx->device);
    int grid = (n + 255) / 256;
    grid = grid > ctx->num_cu * 8 ? ctx->num_cu * 8 : grid;
    hx_node_cost_kernel<<<grid, 256, 0, (hipStream_t)stream_>>>(a);
    return hx_check_launch(ctx, "hx_node_cost_kernel");
}

extern "C" int hx_critical_path(hx_ctx *ctx, int32_t n_nodes, int32_t n_edges,
                                const int32_t *succ_row_ptr, const int32_t *succ_col_idx,
                                const float *node_cost, int32_t n_wf, const int32_t *wf_ptr,
                                int32_t max_sweeps,
                                float *rem, float *tail, int32_t *level, float *horizon, void *stream_)
{
    if (!ctx) return HX_ERR_INVALID_ARG;
    HX_REQUIRE(ctx, n_nodes >= 0 && n_edges >= 0 && n_wf >= 0 && max_sweeps >= 0, HX_ERR_INVALID_ARG, "negative size");
    HX_REQUIRE(ctx, max_sweeps < HX_MAX_SWEEP_FLAGS, HX_ERR_SHAPE, "max_sweeps beyond %d", HX_MAX_SWEEP_FLAGS - 1);
    HX_REQUIRE(ctx, succ_row_ptr && wf_ptr, HX_ERR_INVALID_ARG, "NULL row_ptr or wf_ptr");
    HX_REQUIRE(ctx, n_edges == 0 || succ_col_idx, HX_ERR_INVALID_ARG, "NULL col_idx");
    HX_REQUIRE(ctx, n_nodes == 0 || (node_cost && rem && tail && level), HX_ERR_INVALID_ARG, "NULL node array");
    HX_REQUIRE(ctx, n_wf == 0 || horizon, HX_ERR_INVALID_ARG, "NULL horizon");
    if (n_wf == 0 && (n_nodes == 0 || max_sweeps == 0)) return HX_OK;
    HxDeviceGuard guard(ctx->device);
    HX_REQUIRE(ctx, guard.ok, HX_ERR_DEVICE, "cannot select device %d", ctx->device);
    hipStream_t stream = (hipStream_t)stream_;
    CpArgs a{n_nodes, n_edges, n_wf, succ_row_ptr, succ_col_idx, wf_ptr, node_cost, rem, tail, horizon, level,
             ctx->d_status};
    if (max_sweeps == 0) {
        // workflows per block: as many as fit the staged slice at the average workflow size
        long long fit = n_nodes > 0 ? (long long)(CP_NMAX * 41 / 50) * n_wf / n_nodes : CP_WPB;
        const int wpb = (int)(fit < 1 ? 1 : (fit > CP_WPB ? CP_WPB : fit));
        const int grid = (n_wf + wpb - 1) / wpb;
        // results of 12 MB and more are streamed out past the caches
        if (n_nodes >= (1 << 20)) hx_cp_local_kernel<true><<<grid, CP_THREADS, 0, stream>>>(a, wpb);
        else hx_cp_local_kernel<false><<<grid, CP_THREADS, 0, stream>>>(a, wpb);
        return hx_check_launch(ctx, "hx_cp_local_kernel");
    }
    const int nmax = n_nodes > max_sweeps + 1 ? n_nodes : max_sweeps + 1;
    hx_cp_init_kernel<<<(nmax + 255) / 256, 256, 0, stream>>>(a, ctx->d_flags, max_sweeps + 1);
    if (int rc = hx_check_launch(ctx, "hx_cp_init_kernel")) return rc;
    int grid = (n_nodes + 255) / 256;
    grid = grid > ctx->num_cu * 8 ? ctx->num_cu * 8 : (grid < 1 ? 1 : grid);
    for (int s = 1; s <= max_sweeps; ++s) {
        hx_cp_sweep_kernel<<<grid, 256, 0, stream>>>(a, ctx->d_flags, s);
        if (int rc = hx_check_launch(ctx, "hx_cp_sweep_kernel")) return rc;
    }
    hx_cp_finish_kernel<<<(n_wf + 255) / 256 + 1, 256, 0, stream>>>(a, ctx->d_flags, max_sweeps);
    return hx_check_launch(ctx, "hx_cp_finish_kernel");
}

int hx_horizons_plan(hx_ctx *ctx, const hx_model *model, int32_t n_nodes, int32_t n_edges,
                     const int32_t *succ_row_ptr, const int32_t *succ_col_idx,
                     const int32_t *L_in, const int32_t *L_out,
                     int32_t n_types, const float *type_flops, const float *type_hbm_bw, const hx_links *links,
                     int32_t n_wf, const int32_t *wf_ptr,
                     float *node_cost, float *rem, float *tail, int32_t *level, float *horizon, HxHorizonsPlan *plan)
{
    HX_REQUIRE(ctx, model && links && links->bw && type_flops && type_hbm_bw, HX_ERR_INVALID_ARG, "NULL table");
    HX_REQUIRE(ctx, n_nodes >= 0 && n_edges >= 0 && n_wf >= 0, HX_ERR_INVALID_ARG, "negative size");
    HX_REQUIRE(ctx, n_types >= 1 && n_types <= HX_MAX_TYPES && links->n_types == n_types, HX_ERR_SHAPE,
               "n_types %d (links %d) outside 1..%d", n_types, links->n_types, HX_MAX_TYPES);
    HX_REQUIRE(ctx, succ_row_ptr && wf_ptr, HX_ERR_INVALID_ARG, "NULL row_ptr or wf_ptr");
    HX_REQUIRE(ctx, n_edges == 0 || succ_col_idx, HX_ERR_INVALID_ARG, "NULL col_idx");
    HX_REQUIRE(ctx, n_nodes == 0 || (L_in && L_out && node_cost && rem && tail && level), HX_ERR_INVALID_ARG, "NULL node array");
    HX_REQUIRE(ctx, n_wf == 0 || horizon, HX_ERR_INVALID_ARG, "NULL horizon");
    *plan = HxHorizonsPlan{};
    if (n_wf == 0) return HX_OK;
    plan->a = CpArgs{n_nodes, n_edges, n_wf, succ_row_ptr, succ_col_idx, wf_ptr, node_cost, rem, tail, horizon, level,
                     ctx->d_status};
    NodeCostArgs nc{};
    nc.m = HxModelF{model->kv_bytes_per_token, model->flops_per_token, model->attn_flops_per_token2,
                    model->weight_bytes, model->nominal_batch};
    nc.n = n_nodes; nc.T = n_types; nc.L_in = L_in; nc.L_out = L_out; nc.tF = type_flops; nc.tB = type_hbm_bw;
    nc.bw = links->bw; nc.lat = links->latency; nc.cost = node_cost;
    plan->nc = nc;
    // workflows per block: as many as fit the staged slice at the average workflow size, but no more
    // than it takes to give every compute unit a block (a thread evaluates the cost of each of its nodes)
    long long fit = n_nodes > 0 ? (long long)(CP_NMAX_COST * 41 / 50) * n_wf / n_nodes : CP_WPB;
    const long long spread = n_wf / ctx->num_cu;
    fit = fit > spread ? (spread < 1 ? 1 : spread) : fit;
    plan->wpb = (int)(fit < 1 ? 1 : (fit > CP_WPB ? CP_WPB : fit));
    plan->grid = (n_wf + plan->wpb - 1) / plan->wpb;
    return HX_OK;
}

extern "C" int hx_horizons(hx_ctx *ctx, const hx_model *model, int32_t n_nodes, int32_t n_edges,
                           const int32_t *succ_row_ptr, const int32_t *succ_col_idx,
                           const int32_t *L_in, const int32_t *L_out,
                           int32_t n_types, const float *type_flops, const float *type_hbm_bw, const hx_links *links,
                           int32_t n_wf, const int32_t *wf_ptr,
                           float *node_cost, float *rem, float *tail, int32_t *level, float *horizon, void *stream_)
{
    if (!ctx) return HX_ERR_INVALID_ARG;
    HxHorizonsPlan plan;
    if (int rc = hx_horizons_plan(ctx, model, n_nodes, n_edges, succ_row_ptr, succ_col_idx, L_in, L_out, n_types, type_flops,
                                  type_hbm_bw, links, n_wf, wf_ptr, node_cost, rem, tail, level, horizon, &plan))
        return rc;
    if (plan.grid == 0) return HX_OK;
    HxDeviceGuard guard(ctx->device);
    HX_REQUIRE(ctx, guard.ok, HX_ERR_DEVICE, "cannot select device %d", ctx->device);
    hx_cp_cost_kernel<<<plan.grid, CP_THREADS, 0, (hipStream_t)stream_>>>(plan.a, plan.nc, plan.wpb);
    return hx_check_launch(ctx, "hx_cp_cost_kernel");
}

extern "C" int hx_dag_reserve(hx_ctx *ctx, int32_t max_nodes, int32_t max_edges, int32_t max_wf,
                              int32_t max_depth, void *stream_)
{
    if (!ctx) return HX_ERR_INVALID_ARG;
    HX_REQUIRE(ctx, max_nodes >= 0 && max_edges >= 0 && max_wf >= 0 && max_depth >= 0, HX_ERR_INVALID_ARG, "negative size");
    HX_REQUIRE(ctx, max_depth <= 4096, HX_ERR_SHAPE, "max_depth beyond 4096");
    HxDeviceGuard guard(ctx->device);
    HX_REQUIRE(ctx, guard.ok, HX_ERR_DEVICE, "cannot select device %d", ctx->device);
    hipStream_t stream = (hipStream_t)stream_;
    HX_HIP(ctx, hipStreamSynchronize(stream));
    HxDagStore &g = ctx->dag;
    dag_free(g);
    int rc = HX_OK;
    const size_t N = (size_t)max_nodes, E = (size_t)max_edges, W = (size_t)max_wf;
    if ((rc = dev_alloc(ctx, &g.cost, N)) || (rc = dev_alloc(ctx, &g.rem, N)) || (rc = dev_alloc(ctx, &g.tail, N)) ||
        (rc = dev_alloc(ctx, &g.horizon, W)) || (rc = dev_alloc(ctx, &g.level, N)) || (rc = dev_alloc(ctx, &g.wf, N)) ||
        (rc = dev_alloc(ctx, &g.parent_row_ptr, N + 1)) || (rc = dev_alloc(ctx, &g.parent_col, E)) ||
        (rc = dev_alloc(ctx, &g.parent0, N)) || (rc = dev_alloc(ctx, &g.mark, N)) || (rc = dev_alloc(ctx, &g.list[0], N)) ||
        (rc = dev_alloc(ctx, &g.list[1], N)) || (rc = dev_alloc(ctx, &g.counters, (size_t)4))) {
        dag_free(g);
        return rc;
    }
    g.cap_nodes = max_nodes; g.cap_edges = max_edges; g.cap_wf = max_wf; g.max_depth = max_depth;
    g.n_nodes = 0; g.n_edges = 0; g.epoch = 0;
    // horizon of every workflow starts at 0; parent_row_ptr[0] = 0 (fill kernels, no memset nodes)
    hx_fill_i32_kernel<<<256, 256, 0, stream>>>((int32_t *)g.horizon, W, 0);
    hx_fill_i32_kernel<<<1, 64, 0, stream>>>(g.parent_row_ptr, 1, 0);
    hx_fill_i32_kernel<<<1, 64, 0, stream>>>(g.counters, 4, 0);
    return hx_check_launch(ctx, "hx_fill_i32_kernel");
}

namespace {

// The append's first kernel.  nc: NULL, or the arguments of the standalone cost of the new nodes, which that kernel
// then works out itself (new_cost is nc->cost then, written as well as used).  plan->grid == 0: nothing to append.
int dag_append_begin(hx_ctx *ctx, int32_t n_new, int32_t n_new_edges, const int32_t *parent_row_ptr, const int32_t *parent_col_idx,
                     const float *new_cost, const int32_t *new_wf, const NodeCostArgs *nc, HxAppendPlan *plan, hipStream_t stream)
{
    *plan = HxAppendPlan{};
    HxDagStore &g = ctx->dag;
    HX_REQUIRE(ctx, g.cost, HX_ERR_INVALID_ARG, "hx_dag_reserve has not been called");
    HX_REQUIRE(ctx, n_new >= 0 && n_new_edges >= 0, HX_ERR_INVALID_ARG, "negative size");
    HX_REQUIRE(ctx, n_new == 0 || (parent_row_ptr && new_cost && new_wf), HX_ERR_INVALID_ARG, "NULL array");
    HX_REQUIRE(ctx, n_new_edges == 0 || parent_col_idx, HX_ERR_INVALID_ARG, "NULL parent_col_idx");
    HX_REQUIRE(ctx, (long long)g.n_nodes + n_new <= g.cap_nodes, HX_ERR_CAPACITY,
               "%d + %d nodes beyond the reserved %d", g.n_nodes, n_new, g.cap_nodes);
    HX_REQUIRE(ctx, (long long)g.n_edges + n_new_edges <= g.cap_edges, HX_ERR_CAPACITY,
               "%d + %d edges beyond the reserved %d", g.n_edges, n_new_edges, g.cap_edges);
    if (n_new == 0) return HX_OK;
    HxDeviceGuard guard(ctx->device);
    HX_REQUIRE(ctx, guard.ok, HX_ERR_DEVICE, "cannot select device %d", ctx->device);

    AppendArgs a{};
    a.n_old = g.n_nodes; a.n_new = n_new; a.e_old = g.n_edges; a.n_new_edges = n_new_edges; a.cap_wf = g.cap_wf;
    a.new_row_ptr = parent_row_ptr; a.new_col = parent_col_idx; a.new_wf = new_wf; a.new_cost = new_cost;
    a.cost = g.cost; a.rem = g.rem; a.tail = g.tail; a.horizon = g.horizon;
    a.level = g.level; a.wf = g.wf; a.prow = g.parent_row_ptr; a.pcol = g.parent_col; a.parent0 = g.parent0; a.mark = g.mark;
    a.counters = g.counters; a.status = ctx->d_status;

    int grid = (n_new + 255) / 256;
    grid = grid > ctx->num_cu * 8 ? ctx->num_cu * 8 : grid;
    a.cin = 0; a.cout = 1; a.czero = 2; a.epoch = ++g.epoch;
    a.list_in = g.list[1]; a.list_out = g.list[0];
    if (nc) hx_append_init_kernel<true><<<grid, 256, 0, stream>>>(a, *nc);
    else hx_append_init_kernel<false><<<grid, 256, 0, stream>>>(a, NodeCostArgs{});
    if (int rc = hx_check_launch(ctx, "hx_append_init_kernel")) return rc;
    plan->a = a; plan->grid = grid; plan->n_new = n_new; plan->n_new_edges = n_new_edges;
    return HX_OK;
}

int dag_append(hx_ctx *ctx, int32_t n_new, int32_t n_new_edges, const int32_t *parent_row_ptr, const int32_t *parent_col_idx,
               const float *new_cost, const int32_t *new_wf, const NodeCostArgs *nc, hipStream_t stream)
{
    HxAppendPlan plan;
    if (int rc = dag_append_begin(ctx, n_new, n_new_edges, parent_row_ptr, parent_col_idx, new_cost, new_wf, nc, &plan, stream)) return rc;
    if (plan.grid == 0) return HX_OK;
    if (int rc = hx_dag_append_walks(ctx, &plan, stream)) return rc;
    return hx_dag_append_end(ctx, &plan, stream);
}

}  // namespace

// the walks of an append that has begun, as a launch of their own
int hx_dag_append_walks(hx_ctx *ctx, const HxAppendPlan *plan, void *stream)
{
    HxDeviceGuard guard(ctx->device);
    HX_REQUIRE(ctx, guard.ok, HX_ERR_DEVICE, "cannot select device %d", ctx->device);
    hx_append_relax_kernel<<<plan->grid, 256, 0, (hipStream_t)stream>>>(plan->a);
    return hx_check_launch(ctx, "hx_append_relax_kernel");
}

// what follows the walks: what they handed over (normally nothing) is finished level by level in one workgroup --
// sweep k reads the list sweep k-1 wrote, max_depth sweeps reach every ancestor -- and the graph has grown
int hx_dag_append_end(hx_ctx *ctx, const HxAppendPlan *plan, void *stream_)
{
    HxDeviceGuard guard(ctx->device);
    HX_REQUIRE(ctx, guard.ok, HX_ERR_DEVICE, "cannot select device %d", ctx->device);
    hipStream_t stream = (hipStream_t)stream_;
    HxDagStore &g = ctx->dag;
    AppendArgs a = plan->a;
    if (g.max_depth > 0) {
        a.epoch = g.epoch;                       // the loop advances it once per step
        hx_append_tail_kernel<<<1, 1024, 0, stream>>>(a, g.list[0], g.list[1], 0, g.max_depth);
        g.epoch += (uint32_t)g.max_depth;
    } else {
        a.cin = 1;
        hx_append_finish_kernel<<<1, 64, 0, stream>>>(a);
    }
    if (int rc = hx_check_launch(ctx, "hx_dag_append kernels")) return rc;
    g.n_nodes += plan->n_new;
    g.n_edges += plan->n_new_edges;
    return HX_OK;
}

extern "C" int hx_dag_append(hx_ctx *ctx, int32_t n_new, int32_t n_new_edges,
                             const int32_t *parent_row_ptr, const int32_t *parent_col_idx,
                             const float *new_cost, const int32_t *new_wf, void *stream_)
{
    if (!ctx) return HX_ERR_INVALID_ARG;
    return dag_append(ctx, n_new, n_new_edges, parent_row_ptr, parent_col_idx, new_cost, new_wf, nullptr, (hipStream_t)stream_);
}

// hx_node_cost of the new nodes followed by the first kernel of hx_dag_append, the cost worked out by that kernel: the
// same checks and the same results as the two calls, one launch less (for hx_round, which goes on with
// hx_dag_append_walks -- or takes the walks into its search's launch -- and hx_dag_append_end)
int hx_dag_append_begin(hx_ctx *ctx, const hx_model *model, int32_t n_new, int32_t n_new_edges,
                        const int32_t *parent_row_ptr, const int32_t *parent_col_idx,
                        const int32_t *new_L_in, const int32_t *new_L_out,
                        int32_t n_types, const float *type_flops, const float *type_hbm_bw, const hx_links *links,
                        float *new_cost, const int32_t *new_wf, HxAppendPlan *plan, void *stream_)
{
    *plan = HxAppendPlan{};
    NodeCostArgs nc{};
    if (int rc = node_cost_args(ctx, model, n_new, new_L_in, new_L_out, n_types, type_flops, type_hbm_bw, links, new_cost, &nc))
        return rc;
    return dag_append_begin(ctx, n_new, n_new_edges, parent_row_ptr, parent_col_idx, new_cost, new_wf, &nc, plan, (hipStream_t)stream_);
}

extern "C" int hx_dag_set_cost(hx_ctx *ctx, int32_t n, const int32_t *node_ids, const float *cost, void *stream_)
{
    if (!ctx) return HX_ERR_INVALID_ARG;
    HxDagStore &g = ctx->dag;
    HX_REQUIRE(ctx, g.cost, HX_ERR_INVALID_ARG, "hx_dag_reserve has not been called");
    HX_REQUIRE(ctx, n >= 0, HX_ERR_INVALID_ARG, "negative size");
    HX_REQUIRE(ctx, n == 0 || (node_ids && cost), HX_ERR_INVALID_ARG, "NULL array");
    if (n == 0 || g.n_nodes == 0) return HX_OK;
    HxDeviceGuard guard(ctx->device);
    HX_REQUIRE(ctx, guard.ok, HX_ERR_DEVICE, "cannot select device %d", ctx->device);
    hipStream_t stream = (hipStream_t)stream_;
    hx_set_cost_kernel<<<(n + 255) / 256, 256, 0, stream>>>(n, node_ids, cost, g.cost, g.n_nodes, ctx->d_status);
    // a cost may have gone down, so nothing can be kept: every node starts again from rem = cost and walks up
    // (levels do not depend on costs and stay)
    AppendArgs a{};
    a.n_old = 0; a.n_new = g.n_nodes; a.cap_wf = g.cap_wf;
    a.cost = g.cost; a.rem = g.rem; a.tail = g.tail; a.horizon = g.horizon;
    a.level = g.level; a.wf = g.wf; a.prow = g.parent_row_ptr; a.pcol = g.parent_col; a.parent0 = g.parent0; a.mark = g.mark;
    a.counters = g.counters; a.status = ctx->d_status;
    a.cin = 0; a.cout = 1; a.czero = 2; a.epoch = ++g.epoch;
    a.list_in = g.list[1]; a.list_out = g.list[0];
    const int m = g.n_nodes > g.cap_wf ? g.n_nodes : g.cap_wf;
    hx_refresh_reset_kernel<<<(m + 255) / 256, 256, 0, stream>>>(a, g.cap_wf);
    int grid = (g.n_nodes + 255) / 256;
    grid = grid > ctx->num_cu * 8 ? ctx->num_cu * 8 : grid;
    hx_append_relax_kernel<<<grid, 256, 0, stream>>>(a);
    if (g.max_depth > 0) {
        a.epoch = g.epoch;
        hx_append_tail_kernel<<<1, 1024, 0, stream>>>(a, g.list[0], g.list[1], 0, g.max_depth);
        g.epoch += (uint32_t)g.max_depth;
    } else {
        a.cin = 1;
        hx_append_finish_kernel<<<1, 64, 0, stream>>>(a);
    }
    return hx_check_launch(ctx, "hx_dag_set_cost kernels");
}

extern "C" int hx_dag_view(hx_ctx *ctx, const float **rem, const float **tail, const int32_t **level,
                           const float **horizon, int32_t *n_nodes)
{
    if (!ctx) return HX_ERR_INVALID_ARG;
    HxDagStore &g = ctx->dag;
    HX_REQUIRE(ctx, g.cost, HX_ERR_INVALID_ARG, "hx_dag_reserve has not been called");
    if (rem) *rem = g.rem;
    if (tail) *tail = g.tail;
    if (level) *level = g.level;
    if (horizon) *horizon = g.horizon;
    if (n_nodes) *n_nodes = g.n_nodes;
    return HX_OK;
}
