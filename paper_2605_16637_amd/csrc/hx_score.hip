// Scoring of placement candidates: prepare (per-round tables), fused search
// (score + per-call argmin, no tensor written), materialised tensor, select.
//
// What is computed: Sec. 5.3 of the paper (enumerate prefill x decode
// instances, prefill finish + transfer, earliest decode finish, keep the
// earliest pair), feasibility per Sec. 5.4 Eq. (3),(4), projected ratio per
// Sec. 5.1 Eq. (2).  How it is laid out is specific to gfx950:
//
//  * One wavefront owns one call at a time.  Lanes are prefill instances
//    (KP per lane), so everything that depends on the decode instance only --
//    its availability hint and the call's decode time there -- is the same
//    for all 64 lanes and is read from LDS as a broadcast.
//  * Transfer time depends on the two GPU classes only, so a lane keeps
//    ready[class] = prefill finish + transfer for the <= 8 decode classes in
//    registers, and decode instances are visited grouped by class: inside a
//    class segment the inner loop is  t = max(ready, avail_d) + dec_d ;
//    best = min(best, t)  with no index bookkeeping.
//  * The index is recovered afterwards: the wave minimum fixes the winning
//    prefill instance (lowest p among lanes that hold the minimum), and one
//    pass of the wave over that instance's D candidates finds the lowest d
//    that reproduces the minimum bit for bit.  This gives exactly the
//    lexicographic minimum of (cost, p*D + d).
#include "hx_common.hpp"
#include "hx_terms.hpp"
#include "hx_search.hpp"
#include "hx_cp.hpp"
#include "hx_append.hpp"

#include <cfloat>
#include <cmath>

namespace {

// ---- prepare ------------------------------------------------------------------

struct PrepArgs {
    HxModelF m;
    int P, D, T;
    const float *p_flops, *p_hbm;
    const int32_t *p_backlog, *p_type;
    const float *d_flops, *d_hbm;
    const int32_t *d_used, *d_cap, *d_batch, *d_qd, *d_type;
    const float *bw, *lat;
    HxPrepTables *out;
    int32_t *status;
};

// One workgroup of 1024 threads, one thread per instance of either side (at most HX_MAX_INSTANCES each).
// Everything is read at the top and written at the bottom: the three barriers in between (class counts,
// class segments) then wait for neither loads nor stores.
__global__ __launch_bounds__(1024) void hx_prepare_kernel(PrepArgs a)
{
    __shared__ int s_cnt[kT], s_seg[kT + 1];
    __shared__ int s_wcnt[HX_MAX_INSTANCES / HX_WAVE][kT];
    const int tid = threadIdx.x;
    const int lane = tid & (HX_WAVE - 1), wv = tid >> 6;
    HxPrepTables *o = a.out;

    // ---- reads
    const bool has_link = tid < kT * kT;
    const int tp = tid / kT, td = tid % kT;
    const bool link_in = has_link && tp < a.T && td < a.T;
    const float l_bw = link_in ? a.bw[tp * a.T + td] : 1.0f;
    const float l_lat = (link_in && a.lat) ? a.lat[tp * a.T + td] : 0.0f;
    const bool has_p = tid < a.P;
    int p_t = has_p ? a.p_type[tid] : 0;
    const float p_flops = has_p ? a.p_flops[tid] : 1.0f, p_hbm = has_p ? a.p_hbm[tid] : 1.0f;
    const int p_backlog = has_p ? a.p_backlog[tid] : 0;
    const bool has_d = tid < a.D;
    int my_t = has_d ? a.d_type[tid] : -1;
    const int d_used = has_d ? a.d_used[tid] : 0, d_batch = has_d ? a.d_batch[tid] : 0, d_qd = has_d ? a.d_qd[tid] : 0;
    const int d_cap = has_d ? a.d_cap[tid] : 0;
    const float d_flops = has_d ? a.d_flops[tid] : 1.0f, d_hbm = has_d ? a.d_hbm[tid] : 1.0f;
    if (has_p && (p_t < 0 || p_t >= a.T)) { hx_raise(a.status, HX_ERR_INDEX); p_t = 0; }
    if (has_d && (my_t < 0 || my_t >= a.T)) { hx_raise(a.status, HX_ERR_INDEX); my_t = 0; }

    // ---- decode instances ranked by class: per-wave class counts (ballots), class sizes, class segments
    int my_rank = 0;                     // instances of my class before me in my wave
#pragma unroll
    for (int t = 0; t < kT; ++t) {
        unsigned long long b = __ballot(my_t == t);
        if (lane == 0) s_wcnt[wv][t] = __popcll(b);
        if (my_t == t) my_rank = __popcll(b & ((1ull << lane) - 1ull));
    }
    __syncthreads();
    // class sizes: one thread per class adds up the waves' counts, then one thread lays out the segments
    if (tid < kT) {
        int n = 0;
        for (int k = 0; k < (a.D + HX_WAVE - 1) / HX_WAVE; ++k) {
            const int here = s_wcnt[k][tid];
            s_wcnt[k][tid] = n;                      // instances of the class in earlier waves
            n += here;
        }
        s_cnt[tid] = n;
    }
    __syncthreads();
    if (tid == 0) {
        int e = 0;
        for (int t = 0; t < kT; ++t) {
            s_seg[t] = e;
            e += (s_cnt[t] + HX_DGROUP - 1) / HX_DGROUP * HX_DGROUP;
        }
        s_seg[kT] = e;
    }
    __syncthreads();

    // ---- writes
    if (has_link) {
        o->link_invbw[tid] = link_in ? 1.0f / l_bw : 0.0f;
        o->link_lat[tid] = l_lat;
    }
    if (has_p) {
        const float invF = 1.0f / p_flops;
        o->pre_invF[tid] = invF;
        o->pre_invB[tid] = 1.0f / p_hbm;
        o->pre_wait[tid] = hx_prefill_wait(a.m, p_backlog, invF);
        o->pre_type[tid] = p_t;
    }
    if (tid <= kT) o->seg[tid] = s_seg[tid];
    const int n_entries = s_seg[kT];
    if (tid == 0) o->n_entries = n_entries;
    // pads (real entries below: disjoint indices)
    for (int e = tid; e < n_entries; e += blockDim.x) {
        int t = 0;
        while (t + 1 < kT && e >= s_seg[t + 1]) ++t;
        if (e >= s_seg[t] + s_cnt[t]) {
            o->dec_wait[e] = 0.0f; o->dec_c1[e] = 0.0f; o->dec_c2[e] = 0.0f; o->dec_kB[e] = 0.0f;
            o->dec_free[e] = -1; o->dec_orig[e] = -1; o->dec_type[e] = t;
        }
    }
    if (has_d) {
        const int d = tid, t = my_t;
        int e = s_seg[t] + s_wcnt[wv][t] + my_rank;
        HxDecF x = hx_decode_terms(a.m, d_used, d_batch, d_qd, 1.0f / d_flops, 1.0f / d_hbm);
        o->dec_wait[e] = x.wait; o->dec_c1[e] = x.c1; o->dec_c2[e] = x.c2; o->dec_kB[e] = x.kB;
        long long fr = (long long)d_cap - (long long)d_used;
        o->dec_free[e] = fr < -1 ? -1 : (fr > 2147483647LL ? 2147483647 : (int)fr);
        o->dec_orig[e] = d; o->dec_type[e] = t; o->dec_pos[d] = e;
    }
}

// The same tables, built by the first 256 threads of a workgroup straight into its own LDS arrays (the fused search
// does this itself instead of reading what hx_prepare_kernel wrote: a launch less per round, for a few
// barriers more per workgroup).  Entry order is the one above: classes ascending, instances of a class
// ascending.  s_scratch: [(HX_MAX_INSTANCES / HX_WAVE) * kT + kT] ints.  Ends with a barrier.
struct PrepLds {
    float *wait, *c1, *c2, *kB;
    int *free, *orig, *dtype;
    float *pw, *pinvF, *pinvB;
    int *ptype;
    float *invbw, *lat;
    int *seg;            // [kT + 1]
    int *scratch;
    int Pp;
};

__device__ __forceinline__ void hx_prepare_into_lds(const PrepArgs &a, const PrepLds &o)
{
    constexpr int NCH = HX_MAX_INSTANCES / 256;          // chunks of 256 instances
    // the first 256 threads of the workgroup do the work; wavefronts beyond them only keep the barriers company
    const bool worker = threadIdx.x < 256;
    const int tid = worker ? (int)threadIdx.x : (1 << 24);      // beyond every size: all the tests below fail
    const int lane = threadIdx.x & (HX_WAVE - 1), wv = (threadIdx.x >> 6) & 3;
    int *s_wcnt = o.scratch;                             // [NCH * 4 waves][kT]
    int *s_cnt = o.scratch + NCH * 4 * kT;               // [kT]

    // ---- reads (all of them before the first barrier)
    const bool has_link = tid < kT * kT;
    const int tp = tid / kT, td = tid % kT;
    const bool link_in = has_link && tp < a.T && td < a.T;
    const float l_bw = link_in ? a.bw[tp * a.T + td] : 1.0f;
    const float l_lat = (link_in && a.lat) ? a.lat[tp * a.T + td] : 0.0f;
    int my_t[NCH], d_used[NCH], d_batch[NCH], d_qd[NCH], d_cap[NCH];
    float d_flops[NCH], d_hbm[NCH];
    bool bad = false;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        const int d = j * 256 + tid;
        const bool has_d = d < a.D;
        my_t[j] = has_d ? a.d_type[d] : -1;
        d_used[j] = has_d ? a.d_used[d] : 0; d_batch[j] = has_d ? a.d_batch[d] : 0; d_qd[j] = has_d ? a.d_qd[d] : 0;
        d_cap[j] = has_d ? a.d_cap[d] : 0;
        d_flops[j] = has_d ? a.d_flops[d] : 1.0f; d_hbm[j] = has_d ? a.d_hbm[d] : 1.0f;
        if (has_d && (my_t[j] < 0 || my_t[j] >= a.T)) { bad = true; my_t[j] = 0; }
    }
    for (int p = tid; p < o.Pp; p += 256) {
        const bool in = p < a.P;
        int p_t = in ? a.p_type[p] : 0;
        if (in && (p_t < 0 || p_t >= a.T)) { bad = true; p_t = 0; }
        const float invF = in ? 1.0f / a.p_flops[p] : 0.0f;
        o.pinvF[p] = invF;
        o.pinvB[p] = in ? 1.0f / a.p_hbm[p] : 0.0f;
        o.pw[p] = in ? hx_prefill_wait(a.m, a.p_backlog[p], invF) : INFINITY;    // lanes beyond P never win
        o.ptype[p] = p_t;
    }
    if (bad) hx_raise(a.status, HX_ERR_INDEX);
    if (has_link) {
        o.invbw[tid] = link_in ? 1.0f / l_bw : 0.0f;
        o.lat[tid] = l_lat;
    }

    // ---- decode instances ranked by class: per-wave class counts (ballots), class sizes, class segments
    int my_rank[NCH];
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        my_rank[j] = 0;
        if (j * 256 < a.D) {
#pragma unroll
            for (int t = 0; t < kT; ++t) {
                const unsigned long long b = __ballot(my_t[j] == t);
                if (lane == 0 && worker) s_wcnt[(j * 4 + wv) * kT + t] = __popcll(b);
                if (my_t[j] == t) my_rank[j] = __popcll(b & ((1ull << lane) - 1ull));
            }
        }
    }
    __syncthreads();
    const int n_slots = (a.D + HX_WAVE - 1) / HX_WAVE;   // waves of instances, in instance order
    if (tid < HX_WAVE) {                                 // the first wave: lane t < kT owns class t
        int n = 0;
        if (tid < kT)
            for (int k = 0; k < n_slots; ++k) n += s_wcnt[k * kT + tid];     // independent reads
        if (tid < kT) s_cnt[tid] = n;
        // class segments: running sum of the padded class sizes over the lanes
        const int padded = tid < kT ? (n + HX_DGROUP - 1) / HX_DGROUP * HX_DGROUP : 0;
        int incl = padded;
#pragma unroll
        for (int off = 1; off < kT; off <<= 1) {
            const int up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        if (tid < kT) o.seg[tid] = incl - padded;
        if (tid == kT - 1) o.seg[kT] = incl;
    }
    __syncthreads();

    // ---- entries: pads, then the instances (disjoint indices)
    int seg[kT + 1], cnt[kT];
#pragma unroll
    for (int t = 0; t <= kT; ++t) seg[t] = o.seg[t];
#pragma unroll
    for (int t = 0; t < kT; ++t) cnt[t] = s_cnt[t];
    const int n_entries = seg[kT];
    for (int e = tid; e < n_entries; e += 256) {
        int t = 0, first = 0, used = cnt[0];
#pragma unroll
        for (int k = 1; k < kT; ++k)
            if (e >= seg[k]) { t = k; first = seg[k]; used = cnt[k]; }
        if (e >= first + used) {
            o.wait[e] = 0.0f; o.c1[e] = 0.0f; o.c2[e] = 0.0f; o.kB[e] = 0.0f;
            o.free[e] = -1; o.orig[e] = -1; o.dtype[e] = t;
        }
    }
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        const int d = j * 256 + tid;
        if (d < a.D) {
            const int t = my_t[j];
            int e = o.seg[t] + my_rank[j];
            for (int k = 0; k < j * 4 + wv; ++k) e += s_wcnt[k * kT + t];        // instances of the class in earlier waves
            const HxDecF x = hx_decode_terms(a.m, d_used[j], d_batch[j], d_qd[j], 1.0f / d_flops[j], 1.0f / d_hbm[j]);
            o.wait[e] = x.wait; o.c1[e] = x.c1; o.c2[e] = x.c2; o.kB[e] = x.kB;
            const long long fr = (long long)d_cap[j] - (long long)d_used[j];
            o.free[e] = fr < -1 ? -1 : (fr > 2147483647LL ? 2147483647 : (int)fr);
            o.orig[e] = d; o.dtype[e] = t;
        }
    }
    __syncthreads();
}

// ---- common argument block of the scoring kernels ------------------------------

struct ScoreArgs {
    HxModelF m;
    int C, P, D;
    const int32_t *L_in, *L_out, *node, *wf;
    const float *elapsed, *tail, *horizon;
    int n_nodes, n_wf;
    const HxPrepTables *prep;
    int32_t *best_p, *best_d;
    float *best_cost, *ratio;
    float *cost;          // materialised tensor or NULL
    uint8_t *feas;        // materialised mask or NULL
    int32_t *status;
};

// projected ratio, Eq. (2), with the downstream tail of the call's node
__device__ __forceinline__ void hx_ratio(const ScoreArgs &a, int c, float best)
{
    hx_projected_ratio(a.node, a.wf, a.elapsed, a.tail, a.horizon, a.n_nodes, a.n_wf, c, best, a.status, a.ratio);
}

// ---- fused search ----------------------------------------------------------------

// LDS carve-up shared by host (size) and device (offsets)
struct FusedLds {
    int Dp, Pp;
    __host__ __device__ FusedLds(int n_entries_bound, int P)
        : Dp(n_entries_bound), Pp((P + HX_WAVE - 1) / HX_WAVE * HX_WAVE) {}
    __host__ __device__ size_t block_floats() const { return (size_t)7 * Dp + (size_t)4 * Pp + 2 * kT * kT + 16; }
    __host__ __device__ size_t wave_floats() const { return (size_t)Dp + kT * kT; }
    __host__ __device__ size_t bytes(int waves) const { return 4 * (block_floats() + waves * wave_floats()); }
};

// block, n_blocks: the workgroup's place among those that search (the launch may hold other workgroups too)
template <int KP>
__device__ __forceinline__ void hx_fused_search_body(const ScoreArgs &a, const PrepArgs &pa, int dp_bound, float *smem,
                                                     int block, int n_blocks)
{
    const FusedLds lay(dp_bound, a.P);
    float *s_wait = smem;                  // 7 decode arrays of dp_bound entries
    float *s_c1 = s_wait + lay.Dp;
    float *s_c2 = s_c1 + lay.Dp;
    float *s_kB = s_c2 + lay.Dp;
    int *s_free = (int *)(s_kB + lay.Dp);
    int *s_orig = s_free + lay.Dp;
    int *s_dtype = s_orig + lay.Dp;
    float *s_pw = (float *)(s_dtype + lay.Dp);   // 4 prefill arrays of Pp entries
    float *s_pinvF = s_pw + lay.Pp;
    float *s_pinvB = s_pinvF + lay.Pp;
    int *s_ptype = (int *)(s_pinvB + lay.Pp);
    float *s_invbw = (float *)(s_ptype + lay.Pp);
    float *s_lat = s_invbw + kT * kT;
    int *s_seg = (int *)(s_lat + kT * kT);       // kT+1 used, 16 reserved
    float *s_wave = (float *)(s_seg + 16);

    const int tid = threadIdx.x;
    const int lane = tid & (HX_WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int waves_per_block = blockDim.x >> 6;
    float *dbuf = s_wave + (size_t)wave * lay.wave_floats();    // the call's decode time per entry
    float *xbuf = dbuf + lay.Dp;                                // transfer per class pair

    // What the wave's first call says of itself is asked for before the pool's tables are derived, and every
    // later call's while the call before it is searched: the loads are wave-uniform (scalar), and none of the
    // kernel's chains of dependent memory round trips waits for them on its own.
    const int gw = block * waves_per_block + wave;
    const int nw = n_blocks * waves_per_block;
    const bool want_ratio = a.ratio != nullptr;
    int c = gw;
    int L = 0, O = 0, nd = 0, w = 0;
    float el = 0.0f;
    if (c < a.C) {
        L = a.L_in[c]; O = a.L_out[c];
        if (want_ratio) { nd = a.node[c]; w = a.wf[c]; el = a.elapsed[c]; }
    }

    // the per-round tables of the pool, derived here; the class counts of the derivation borrow the
    // waves' buffers, which nothing has used yet
    const PrepLds out{s_wait, s_c1, s_c2, s_kB, s_free, s_orig, s_dtype, s_pw, s_pinvF, s_pinvB, s_ptype,
                      s_invbw, s_lat, s_seg, (int *)s_wave, lay.Pp};
    hx_prepare_into_lds(pa, out);
    const int Dp = s_seg[kT];              // <= dp_bound by construction

    int seg[kT + 1];
#pragma unroll
    for (int k = 0; k <= kT; ++k) seg[k] = __builtin_amdgcn_readfirstlane(s_seg[k]);
    const HxPoolLds pool{s_wait, s_c1, s_c2, s_kB, s_free, s_orig, s_dtype, s_pw, s_pinvF, s_pinvB, s_ptype,
                         s_invbw, s_lat, Dp, a.P, lay.Pp};

    while (c < a.C) {
        // the downstream tail and the horizon of the call's workflow travel while the call is searched
        const bool ok = !want_ratio || (nd >= 0 && nd < a.n_nodes && w >= 0 && w < a.n_wf);
        float tl = 0.0f, hz = 1.0f;
        if (want_ratio && ok) { tl = a.tail[nd]; hz = a.horizon[w]; }
        const int cn = c + nw;
        int Ln = 0, On = 0, ndn = 0, wn = 0;
        float eln = 0.0f;
        if (cn < a.C) {
            Ln = a.L_in[cn]; On = a.L_out[cn];
            if (want_ratio) { ndn = a.node[cn]; wn = a.wf[cn]; eln = a.elapsed[cn]; }
        }
        const HxBest b = hx_search_call<KP>(a.m, pool, seg, dbuf, xbuf, L, O, lane);
        if (lane == 0) {
            a.best_p[c] = b.p;
            a.best_d[c] = b.d;
            a.best_cost[c] = b.cost;
            if (want_ratio) {
                if (!ok) hx_raise(a.status, HX_ERR_INDEX);
                hx_store_bits(a.ratio, c, hx_ratio_bits(el, b.cost, tl, hz, ok));      // Eq. (2), as hx_projected_ratio forms it
            }
        }
        c = cn; L = Ln; O = On; nd = ndn; w = wn; el = eln;
    }
}

template <int KP>
__global__ __launch_bounds__(512) void hx_fused_search_kernel(ScoreArgs a, PrepArgs pa, int dp_bound)
{
    extern __shared__ __align__(16) float smem[];
    hx_fused_search_body<KP>(a, pa, dp_bound, smem, (int)blockIdx.x, (int)gridDim.x);
}

// ---- the first kernel of a scheduling round that brings its whole graph: reveal and search in one launch ----
//
// The horizon refresh (node cost + critical path, what hx_cp_cost_kernel does) and the search do not depend on each
// other -- only the ratio needs both, and it is formed by the commit kernel that follows -- so they share a launch:
// n_reveal workgroups take workflows exactly as hx_cp_cost_kernel's do (same body, the cost's prefill classes one
// after the other to stay within the search's registers), the others search.  Same results as the two kernels,
// one launch and the gap before it less.  On a small round (every wavefront has at most one call, all workgroups
// resident at once) both halves are chains of memory round trips, which now run side by side; on a large one the
// reveal's workgroups, the last of the grid then, take the places of the searching workgroups that end first
// (those whose wavefronts were dealt one call fewer) while the rest of the chip goes on searching.
constexpr int RV_NMAX = 512;             // nodes staged per run of a reveal workgroup

struct RevealLds {
    CpNode node[RV_NMAX + 1];
    CostTables tab;
    int any;
};

// FIRST: the reveal's workgroups are the first n_reveal of the grid (else the last)
template <int KP, bool FIRST>
__global__ __launch_bounds__(CP_THREADS) void hx_reveal_search_kernel(ScoreArgs a, PrepArgs pa, int dp_bound, CpArgs cp,
                                                                      NodeCostArgs nc, int wpb, int n_reveal)
{
    extern __shared__ __align__(16) float smem[];
    const int n_search = (int)gridDim.x - n_reveal;
    const int block = FIRST ? (int)blockIdx.x - n_reveal : (int)blockIdx.x;              // among the searching ones
    if (FIRST ? block < 0 : block >= n_search) {
        RevealLds *l = (RevealLds *)smem;
        hx_cp_local_body<RV_NMAX, true, false, true>(cp, wpb, l->node, l->any, &nc, &l->tab,
                                                     FIRST ? (int)blockIdx.x : block - n_search);
        return;
    }
    hx_fused_search_body<KP>(a, pa, dp_bound, smem, block, n_search);
}

// The same for a round that appends to the context's graph: the append's walks (hx_append_relax_kernel's work: one
// thread per new node, a chain of device-scope atomics up its ancestors) take the first n_lead workgroups of the
// search's launch.  They are all latency and no arithmetic, and where the search fills the chip the workgroups they
// displace are again the ones with the fewest calls.
template <int KP>
__global__ __launch_bounds__(512) void hx_relax_search_kernel(ScoreArgs a, PrepArgs pa, int dp_bound, AppendArgs ap, int n_lead)
{
    extern __shared__ __align__(16) float smem[];
    if ((int)blockIdx.x < n_lead) {
        hx_append_relax_body(ap, (int)blockIdx.x, n_lead);
        return;
    }
    hx_fused_search_body<KP>(a, pa, dp_bound, smem, (int)blockIdx.x - n_lead, (int)gridDim.x - n_lead);
}

// ---- materialised tensor ------------------------------------------------------------

// A workgroup takes nc calls at a time (nc = 4 on small pools, where one call's share of the tensor is a few
// KB and the barriers and the per-call tables would otherwise cost as much as the stores; 1 on large ones).
// LDS: per call of the batch the prefill finish per instance, the decode time per instance and the class-pair
// transfer times, each worked out by 256 / nc threads; beside them what does not depend on the call (waits,
// per-token terms, classes; original instance order), staged once per workgroup.
__global__ __launch_bounds__(256) void hx_materialise_kernel(ScoreArgs a, int nc)
{
    extern __shared__ __align__(16) float smem[];
    const HxPrepTables *__restrict__ t = a.prep;
    const int P4 = (a.P + 3) & ~3, D4 = (a.D + 3) & ~3;      // every array starts on a 16-byte boundary
    float *s_done = smem;                       // [nc][P4] per call
    float *s_dec = s_done + nc * P4;            // [nc][D4] per call
    float *s_x = s_dec + nc * D4;               // [nc][kT*kT] per call
    float *s_wait = s_x + nc * kT * kT;         // [D]
    int *s_ptype = (int *)(s_wait + D4);        // [P]
    int *s_dtype = s_ptype + P4;                // [D]
    float *s_pw = (float *)(s_dtype + D4);      // [P] prefill wait, 1/F, 1/B
    float *s_pF = s_pw + P4;
    float *s_pB = s_pF + P4;
    float *s_c1 = s_pB + P4;                    // [D] decode per-token terms and free tokens, by instance
    float *s_c2 = s_c1 + D4;
    float *s_kB = s_c2 + D4;
    int *s_free = (int *)(s_kB + D4);
    float *s_lbw = (float *)(s_free + D4);      // [kT*kT] link tables
    float *s_llat = s_lbw + kT * kT;
    const int tid = threadIdx.x;
    // rows of the tensor are 16-byte aligned and a whole number of quads long
    const bool vec4 = (a.D & 3) == 0 && a.D >= 4 && (reinterpret_cast<uintptr_t>(a.cost) & 15) == 0;
    for (int p = tid; p < a.P; p += blockDim.x) {
        s_pw[p] = t->pre_wait[p]; s_pF[p] = t->pre_invF[p]; s_pB[p] = t->pre_invB[p]; s_ptype[p] = t->pre_type[p];
    }
    for (int d = tid; d < a.D; d += blockDim.x) {
        const int e = t->dec_pos[d];
        s_c1[d] = t->dec_c1[e]; s_c2[d] = t->dec_c2[e]; s_kB[d] = t->dec_kB[e]; s_free[d] = t->dec_free[e];
        s_wait[d] = t->dec_wait[e]; s_dtype[d] = t->dec_type[e];
    }
    if (tid < kT * kT) { s_lbw[tid] = t->link_invbw[tid]; s_llat[tid] = t->link_lat[tid]; }
    // the part of the workgroup that works out the tables of one call of the batch
    const int per_call = blockDim.x / nc;
    const int slot = tid / per_call, tq = tid - slot * per_call;
    for (int c0 = blockIdx.x * nc; c0 < a.C; c0 += gridDim.x * nc) {
        const int cs = c0 + slot;
        const bool live = cs < a.C;
        const int L = live ? a.L_in[cs] : 0, O = live ? a.L_out[cs] : 0;
        const HxCallF cf = hx_call_terms(a.m, L, O);
        __syncthreads();
        if (live) {
            for (int p = tq; p < a.P; p += per_call) s_done[slot * P4 + p] = hx_prefill_done(cf, s_pw[p], s_pF[p], s_pB[p]);
            for (int d = tq; d < a.D; d += per_call) {
                const bool fits = hx_fits(L, O, s_free[d]);
                s_dec[slot * D4 + d] = fits ? hx_decode_time(cf, s_c1[d], s_c2[d], s_kB[d]) : INFINITY;
                if (a.feas) a.feas[(size_t)cs * a.D + d] = fits ? 1 : 0;
            }
            for (int i = tq; i < kT * kT; i += per_call) s_x[slot * kT * kT + i] = hx_transfer(cf, s_lbw[i], s_llat[i]);
        }
        __syncthreads();
        if (a.cost) {
            const int n_here = min(nc, a.C - c0);
            for (int s = 0; s < n_here; ++s) {
                float *out = a.cost + (size_t)(c0 + s) * a.P * a.D;
                const float *done_s = s_done + s * P4, *dec_s = s_dec + s * D4, *x_s = s_x + s * kT * kT;
                // (p, d) of the elements a thread writes advance without a division: by blockDim positions at a time
                if (vec4) {
                    // four neighbouring decode instances per step, one 16-byte store
                    const int dq = a.D >> 2;
                    const int step_p = blockDim.x / dq, step_q = blockDim.x % dq;
                    int p = tid / dq, q = tid - p * dq;
                    for (; p < a.P; p += step_p) {
                        const float done = done_s[p];
                        const float *xr = x_s + s_ptype[p] * kT;
                        const float4 w = reinterpret_cast<const float4 *>(s_wait)[q];
                        const float4 tm = reinterpret_cast<const float4 *>(dec_s)[q];
                        const int4 k = reinterpret_cast<const int4 *>(s_dtype)[q];
                        float4 v;
                        v.x = hx_candidate(done + xr[k.x], w.x, tm.x);
                        v.y = hx_candidate(done + xr[k.y], w.y, tm.y);
                        v.z = hx_candidate(done + xr[k.z], w.z, tm.z);
                        v.w = hx_candidate(done + xr[k.w], w.w, tm.w);
                        reinterpret_cast<float4 *>(out + (size_t)p * a.D)[q] = v;
                        q += step_q;
                        if (q >= dq) { q -= dq; ++p; }
                    }
                } else {
                    const int step_p = blockDim.x / a.D, step_d = blockDim.x % a.D;
                    int p = tid / a.D, d = tid - p * a.D;
                    for (; p < a.P; p += step_p) {
                        out[(size_t)p * a.D + d] = hx_candidate(done_s[p] + x_s[s_ptype[p] * kT + s_dtype[d]], s_wait[d], dec_s[d]);
                        d += step_d;
                        if (d >= a.D) { d -= a.D; ++p; }
                    }
                }
            }
        }
    }
}
__global__ __launch_bounds__(256) void hx_select_kernel(ScoreArgs a)
{
    __shared__ float s_v[4];
    __shared__ int s_i[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = a.P * a.D;
    const bool vec4 = (n & 3) == 0 && (reinterpret_cast<uintptr_t>(a.cost) & 15) == 0;
    for (int c = blockIdx.x; c < a.C; c += gridDim.x) {
        const float *row = a.cost + (size_t)c * n;
        float bv = INFINITY;
        int bi = 0x7fffffff;
        if (vec4) {
            // 16-byte loads, two in flight per thread; indices grow within a quad and from quad to quad
            const float4 *row4 = reinterpret_cast<const float4 *>(row);
            const int n4 = n >> 2;
            int i4 = tid;
            for (; i4 + (int)blockDim.x < n4; i4 += 2 * blockDim.x) {
                const float4 x = row4[i4], y = row4[i4 + blockDim.x];
                const int i = i4 << 2, j = (i4 + blockDim.x) << 2;
                if (x.x < bv) { bv = x.x; bi = i; }
                if (x.y < bv) { bv = x.y; bi = i + 1; }
                if (x.z < bv) { bv = x.z; bi = i + 2; }
                if (x.w < bv) { bv = x.w; bi = i + 3; }
                if (y.x < bv) { bv = y.x; bi = j; }
                if (y.y < bv) { bv = y.y; bi = j + 1; }
                if (y.z < bv) { bv = y.z; bi = j + 2; }
                if (y.w < bv) { bv = y.w; bi = j + 3; }
            }
            if (i4 < n4) {
                const float4 x = row4[i4];
                const int i = i4 << 2;
                if (x.x < bv) { bv = x.x; bi = i; }
                if (x.y < bv) { bv = x.y; bi = i + 1; }
                if (x.z < bv) { bv = x.z; bi = i + 2; }
                if (x.w < bv) { bv = x.w; bi = i + 3; }
            }
        } else {
            for (int i = tid; i < n; i += blockDim.x) {     // i grows: "<" keeps the lowest index of this thread
                float v = row[i];
                if (v < bv) { bv = v; bi = i; }
            }
        }
#pragma unroll
        for (int off = HX_WAVE / 2; off > 0; off >>= 1) {
            float ov = __shfl_xor(bv, off);
            int oi = __shfl_xor(bi, off);
            bool take = ov < bv || (ov == bv && oi < bi);
            bv = take ? ov : bv;
            bi = take ? oi : bi;
        }
        __syncthreads();
        if (lane == 0) { s_v[wave] = bv; s_i[wave] = bi; }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < (int)(blockDim.x >> 6); ++w)
                if (s_v[w] < bv || (s_v[w] == bv && s_i[w] < bi)) { bv = s_v[w]; bi = s_i[w]; }
            bool any = bv < INFINITY;
            a.best_p[c] = any ? bi / a.D : -1;
            a.best_d[c] = any ? bi % a.D : -1;
            a.best_cost[c] = bv;
            if (a.ratio) hx_ratio(a, c, bv);
        }
    }
}

// the urgency fold on its own: Eq. (2) from best costs found earlier
__global__ __launch_bounds__(256) void hx_urgency_kernel(const int32_t *node, const int32_t *wf, const float *elapsed,
                                                         const float *best_cost, const float *tail, const float *horizon,
                                                         int n_nodes, int n_wf, int C, float *ratio, int32_t *status)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c < C) hx_projected_ratio(node, wf, elapsed, tail, horizon, n_nodes, n_wf, c, best_cost[c], status, ratio);
}

// fused outputs when the pool is empty: nothing is feasible
__global__ void hx_no_pool_kernel(ScoreArgs a)
{
    int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= a.C) return;
    a.best_p[c] = -1; a.best_d[c] = -1; a.best_cost[c] = INFINITY;
    if (a.ratio) hx_ratio(a, c, INFINITY);
}

HxModelF to_model(const hx_model *m)
{
    return HxModelF{m->kv_bytes_per_token, m->flops_per_token, m->attn_flops_per_token2,
                    m->weight_bytes, m->nominal_batch};
}

// the pool tables as the table derivation reads them (pointers checked by the caller)
PrepArgs make_prep_args(hx_ctx *ctx, const hx_model *model, const hx_prefill_tab *pre, const hx_decode_tab *dec,
                        const hx_links *links)
{
    PrepArgs pa{};
    pa.m = to_model(model); pa.P = pre->n; pa.D = dec->n; pa.T = links->n_types;
    pa.p_flops = pre->flops; pa.p_hbm = pre->hbm_bw; pa.p_backlog = pre->backlog_tok; pa.p_type = pre->type;
    pa.d_flops = dec->flops; pa.d_hbm = dec->hbm_bw; pa.d_used = dec->used_tok; pa.d_cap = dec->cap_tok;
    pa.d_batch = dec->batch; pa.d_qd = dec->qd_tok; pa.d_type = dec->type;
    pa.bw = links->bw; pa.lat = links->latency; pa.out = ctx->d_prep; pa.status = ctx->d_status;
    return pa;
}

int check_ratio_inputs(hx_ctx *ctx, const hx_calls *calls, const float *tail, const float *horizon,
                       int32_t n_nodes, int32_t n_wf, const float *ratio)
{
    if (!ratio) return HX_OK;
    HX_REQUIRE(ctx, calls && calls->node && calls->wf && calls->elapsed && tail && horizon,
               HX_ERR_INVALID_ARG, "ratio needs calls.node, calls.wf, calls.elapsed, tail and horizon");
    HX_REQUIRE(ctx, n_nodes >= 0 && n_wf >= 0, HX_ERR_INVALID_ARG, "negative n_nodes or n_wf");
    return HX_OK;
}

}  // namespace

// Validates the pool tables and enqueues the kernel that derives the per-round
// tables (ctx->d_prep) from them.  Shared by every entry point that scores.
int hx_prepare_pool(hx_ctx *ctx, const hx_model *model, const hx_prefill_tab *pre, const hx_decode_tab *dec,
                    const hx_links *links, hipStream_t stream)
{
    HX_REQUIRE(ctx, model && pre && dec && links, HX_ERR_INVALID_ARG, "NULL table");
    const int P = pre->n, D = dec->n, T = links->n_types;
    HX_REQUIRE(ctx, P >= 0 && D >= 0, HX_ERR_INVALID_ARG, "negative size");
    HX_REQUIRE(ctx, T >= 1 && T <= HX_MAX_TYPES, HX_ERR_SHAPE, "n_types %d outside 1..%d", T, HX_MAX_TYPES);
    HX_REQUIRE(ctx, P <= HX_MAX_INSTANCES && D <= HX_MAX_INSTANCES, HX_ERR_SHAPE,
               "pool %d x %d beyond %d instances per side", P, D, HX_MAX_INSTANCES);
    HX_REQUIRE(ctx, P == 0 || (pre->flops && pre->hbm_bw && pre->backlog_tok && pre->type),
               HX_ERR_INVALID_ARG, "NULL member in prefill table");
    HX_REQUIRE(ctx, D == 0 || (dec->flops && dec->hbm_bw && dec->used_tok && dec->cap_tok && dec->batch &&
                               dec->qd_tok && dec->type), HX_ERR_INVALID_ARG, "NULL member in decode table");
    HX_REQUIRE(ctx, links->bw, HX_ERR_INVALID_ARG, "links.bw is NULL");
    const PrepArgs pa = make_prep_args(ctx, model, pre, dec, links);
    hx_prepare_kernel<<<1, 1024, 0, stream>>>(pa);
    return hx_check_launch(ctx, "hx_prepare_kernel");
}

// the fused search may use all 160 KB of LDS; said once per process, outside any stream work
int hx_score_init()
{
    const int lds = 160 * 1024;
    const void *kernels[] = {
        reinterpret_cast<const void *>(hx_fused_search_kernel<1>), reinterpret_cast<const void *>(hx_fused_search_kernel<2>),
        reinterpret_cast<const void *>(hx_fused_search_kernel<4>),
        reinterpret_cast<const void *>(hx_reveal_search_kernel<1, true>), reinterpret_cast<const void *>(hx_reveal_search_kernel<2, true>),
        reinterpret_cast<const void *>(hx_reveal_search_kernel<4, true>),
        reinterpret_cast<const void *>(hx_reveal_search_kernel<1, false>), reinterpret_cast<const void *>(hx_reveal_search_kernel<2, false>),
        reinterpret_cast<const void *>(hx_reveal_search_kernel<4, false>),
        reinterpret_cast<const void *>(hx_relax_search_kernel<1>), reinterpret_cast<const void *>(hx_relax_search_kernel<2>),
        reinterpret_cast<const void *>(hx_relax_search_kernel<4>)};
    hipError_t e = hipSuccess;
    for (const void *k : kernels)
        if (e == hipSuccess) e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    return e == hipSuccess ? HX_OK : HX_ERR_DEVICE;
}

namespace {

// reveal: NULL, or the horizon refresh of the same round (hx_horizons_plan), to ride in the search's launch if the
// round is small enough for that: *revealed says whether it did.  walks: NULL, or an append of the same round that
// has begun (hx_dag_append_begin), whose walks are to ride in the search's launch likewise.  With a reveal the ratio is only checked, not
// written -- the horizons are not there yet; the caller forms it afterwards -- and nothing but the fused search is
// launched: if the reveal does not fit, nothing at all is, and the caller makes the calls one after the other.
int score_placements(hx_ctx *ctx, const hx_model *model, const hx_calls *calls,
                     const hx_prefill_tab *pre, const hx_decode_tab *dec, const hx_links *links,
                     const float *tail, const float *horizon, int32_t n_nodes, int32_t n_wf,
                     float *cost, uint8_t *feas,
                     int32_t *best_p, int32_t *best_d, float *best_cost, float *ratio,
                     const HxHorizonsPlan *reveal, const HxAppendPlan *walks, bool *revealed, void *stream_)
{
    HX_REQUIRE(ctx, model && calls && pre && dec && links, HX_ERR_INVALID_ARG, "NULL table");
    const int C = calls->n, P = pre->n, D = dec->n, T = links->n_types;
    HX_REQUIRE(ctx, C >= 0 && P >= 0 && D >= 0, HX_ERR_INVALID_ARG, "negative size");
    HX_REQUIRE(ctx, T >= 1 && T <= HX_MAX_TYPES, HX_ERR_SHAPE, "n_types %d outside 1..%d", T, HX_MAX_TYPES);
    HX_REQUIRE(ctx, P <= HX_MAX_INSTANCES && D <= HX_MAX_INSTANCES, HX_ERR_SHAPE,
               "pool %d x %d beyond %d instances per side", P, D, HX_MAX_INSTANCES);
    const bool fused = best_p || best_d || best_cost;
    HX_REQUIRE(ctx, !fused || (best_p && best_d && best_cost), HX_ERR_INVALID_ARG,
               "best_p, best_d, best_cost must be given together");
    HX_REQUIRE(ctx, fused || cost || feas, HX_ERR_INVALID_ARG, "no output requested");
    HX_REQUIRE(ctx, !ratio || fused, HX_ERR_INVALID_ARG, "ratio needs the fused outputs");
    HX_REQUIRE(ctx, C == 0 || (calls->L_in && calls->L_out), HX_ERR_INVALID_ARG, "calls.L_in / L_out is NULL");
    HX_REQUIRE(ctx, P == 0 || (pre->flops && pre->hbm_bw && pre->backlog_tok && pre->type),
               HX_ERR_INVALID_ARG, "NULL member in prefill table");
    HX_REQUIRE(ctx, D == 0 || (dec->flops && dec->hbm_bw && dec->used_tok && dec->cap_tok && dec->batch &&
                               dec->qd_tok && dec->type), HX_ERR_INVALID_ARG, "NULL member in decode table");
    HX_REQUIRE(ctx, links->bw, HX_ERR_INVALID_ARG, "links.bw is NULL");
    HX_REQUIRE(ctx, !cost || (double)C * P * D < 9.0e18, HX_ERR_SHAPE, "tensor too large");
    HX_REQUIRE(ctx, (long long)P * D <= 2147483647LL, HX_ERR_SHAPE, "P*D beyond int32");
    if (int rc = check_ratio_inputs(ctx, calls, tail, horizon, n_nodes, n_wf, ratio)) return rc;
    if (C == 0) return HX_OK;

    HxDeviceGuard guard(ctx->device);
    HX_REQUIRE(ctx, guard.ok, HX_ERR_DEVICE, "cannot select device %d", ctx->device);
    hipStream_t stream = (hipStream_t)stream_;

    ScoreArgs a{};
    a.m = to_model(model);
    a.C = C; a.P = P; a.D = D;
    a.L_in = calls->L_in; a.L_out = calls->L_out; a.node = calls->node; a.wf = calls->wf;
    a.elapsed = calls->elapsed; a.tail = tail; a.horizon = horizon; a.n_nodes = n_nodes; a.n_wf = n_wf;
    a.prep = ctx->d_prep;
    a.best_p = best_p; a.best_d = best_d; a.best_cost = best_cost; a.ratio = (reveal || walks) ? nullptr : ratio;
    a.cost = cost; a.feas = feas; a.status = ctx->d_status;

    if (reveal && (P == 0 || D == 0 || !fused || cost || feas || reveal->grid == 0)) return HX_OK;      // not this way
    if (walks && (P == 0 || D == 0 || !fused || cost || feas || walks->grid == 0)) return HX_OK;
    if (P == 0 || D == 0) {
        if (fused) {
            hx_no_pool_kernel<<<(C + 255) / 256, 256, 0, stream>>>(a);
            return hx_check_launch(ctx, "hx_no_pool_kernel");
        }
        return HX_OK;
    }

    if (fused) {
        // the search derives the per-round tables of the pool in its own workgroups: no launch of its own for them
        const PrepArgs pa = make_prep_args(ctx, model, pre, dec, links);
        // upper bound of the padded decode entries, known on the host without reading the device
        const int dp_bound = (D + HX_DGROUP - 1) / HX_DGROUP * HX_DGROUP + (T - 1) * HX_DGROUP;
        // Workgroups of 4 or 8 wavefronts (one or two per SIMD), as many per compute unit as local memory allows up
        // to 6 wavefronts per SIMD (registers would allow 7; measured no faster, and 6 divides into either
        // workgroup size): the pool tables are per workgroup, a wavefront adds its decode-time and transfer
        // buffers.  Whichever size puts more wavefronts on a SIMD, the larger on a tie (half as many workgroups derive
        // the pool's tables).
        const FusedLds lay(dp_bound, P);
        if (reveal) {
            // Workgroups of four wavefronts, as many searching ones as are resident at once (six per compute unit, or
            // what local memory allows) or as the calls need, whichever is less.  Where all of the launch is resident
            // at once the reveal's workgroups are the first of the grid.  Where the searching workgroups alone fill
            // the chip they are the last: they start as the first searching workgroups end -- those whose wavefronts
            // have the fewest calls (calls are dealt c, c + n, ...) -- in places that would stand empty for the rest of
            // the launch, and are done before the wavefronts with one call more (in front of the grid they held up
            // that many searching workgroups from the start: 73 us against 71 for the large round's launch).  Not this
            // way if the reveal's units are too large for its staging area or its workgroups more than a third of
            // the searching ones.
            const size_t lds4 = lay.bytes(4) > sizeof(RevealLds) ? lay.bytes(4) : sizeof(RevealLds);
            if (lds4 > 160 * 1024) return HX_OK;
            const long long by_lds = (long long)(160 * 1024) / (long long)lds4;
            const long long resident = (by_lds < 6 ? by_lds : 6) * ctx->num_cu;
            const long long need4 = (C + 3) / 4;
            const int n_search = (int)(need4 < resident ? need4 : resident);
            const long long nodes_per_unit = (long long)reveal->a.n_nodes * reveal->wpb / (reveal->a.n_wf > 0 ? reveal->a.n_wf : 1);
            const bool all_resident = need4 + reveal->grid <= resident;
            if (nodes_per_unit > RV_NMAX * 7 / 10 || !(all_resident || 3LL * reveal->grid <= n_search)) return HX_OK;
            auto launch = [&](auto kern) {
                kern<<<reveal->grid + n_search, CP_THREADS, lds4, stream>>>(a, pa, dp_bound, reveal->a, reveal->nc, reveal->wpb,
                                                                            reveal->grid);
            };
            if (all_resident) {
                if (P <= 64) launch(hx_reveal_search_kernel<1, true>);
                else if (P <= 128) launch(hx_reveal_search_kernel<2, true>);
                else launch(hx_reveal_search_kernel<4, true>);
            } else {
                if (P <= 64) launch(hx_reveal_search_kernel<1, false>);
                else if (P <= 128) launch(hx_reveal_search_kernel<2, false>);
                else launch(hx_reveal_search_kernel<4, false>);
            }
            if (int rc = hx_check_launch(ctx, "hx_reveal_search_kernel")) return rc;
            *revealed = true;
            return HX_OK;
        }
        const int reg_limit = 6 * 4;                               // wavefronts per compute unit
        int waves = 4, blocks_per_cu = 1, best_on_cu = 0;
        for (int w = 4; w <= 8; w += 4) {
            const size_t need_lds = lay.bytes(w);
            if (need_lds > 160 * 1024) continue;
            int b = (int)((160 * 1024) / need_lds);
            b = b > reg_limit / w ? reg_limit / w : b;
            if (b * w >= best_on_cu) { best_on_cu = b * w; waves = w; blocks_per_cu = b; }
        }
        const size_t lds = lay.bytes(waves);
        HX_REQUIRE(ctx, best_on_cu > 0, HX_ERR_SHAPE, "pool needs %zu B of LDS", lds);
        int grid = ctx->num_cu * blocks_per_cu;
        const int need = (C + waves - 1) / waves;
        grid = grid > need ? need : grid;
        if (walks) {
            // the walks' threads take several new nodes each if need be; not this way if they would be more than a
            // third of the launch (a small search behind a large append: the two launches are then the better way)
            const int threads = waves * HX_WAVE;
            const int n_lead = (walks->a.n_new + threads - 1) / threads;
            if (3LL * n_lead > grid) return HX_OK;
            auto launch_w = [&](auto kern) { kern<<<n_lead + grid, threads, lds, stream>>>(a, pa, dp_bound, walks->a, n_lead); };
            if (P <= 64) launch_w(hx_relax_search_kernel<1>);
            else if (P <= 128) launch_w(hx_relax_search_kernel<2>);
            else launch_w(hx_relax_search_kernel<4>);
            if (int rc = hx_check_launch(ctx, "hx_relax_search_kernel")) return rc;
            *revealed = true;
            return HX_OK;
        }
        auto launch = [&](auto kern) { kern<<<grid, waves * HX_WAVE, lds, stream>>>(a, pa, dp_bound); };
        if (P <= 64) launch(hx_fused_search_kernel<1>);
        else if (P <= 128) launch(hx_fused_search_kernel<2>);
        else launch(hx_fused_search_kernel<4>);
        if (int rc = hx_check_launch(ctx, "hx_fused_search_kernel")) return rc;
    }
    if (cost || feas) {
        if (int rc = hx_prepare_pool(ctx, model, pre, dec, links, stream)) return rc;
        const int P4 = (P + 3) & ~3, D4 = (D + 3) & ~3;
        const int nc = (long long)P * D <= 16384 && C >= 4 * ctx->num_cu * 4 ? 4 : 1;      // calls per workgroup at a time
        const size_t lds = 4 * ((size_t)nc * (P4 + D4 + kT * kT) + 4 * P4 + 6 * D4 + 2 * kT * kT);
        const int batches = (C + nc - 1) / nc;
        const int grid = batches < ctx->num_cu * 8 ? batches : ctx->num_cu * 8;
        hx_materialise_kernel<<<grid, 256, lds, stream>>>(a, nc);
        if (int rc = hx_check_launch(ctx, "hx_materialise_kernel")) return rc;
    }
    return HX_OK;
}

}  // namespace

extern "C" int hx_score_placements(hx_ctx *ctx, const hx_model *model, const hx_calls *calls,
                                   const hx_prefill_tab *pre, const hx_decode_tab *dec,
                                   const hx_links *links,
                                   const float *tail, const float *horizon, int32_t n_nodes, int32_t n_wf,
                                   float *cost, uint8_t *feas,
                                   int32_t *best_p, int32_t *best_d, float *best_cost, float *ratio,
                                   void *stream_)
{
    if (!ctx) return HX_ERR_INVALID_ARG;
    return score_placements(ctx, model, calls, pre, dec, links, tail, horizon, n_nodes, n_wf, cost, feas,
                            best_p, best_d, best_cost, ratio, nullptr, nullptr, nullptr, stream_);
}

// The horizon refresh `reveal` and hx_score_placements (fused outputs) in one launch, where the round is small
// enough (*revealed; otherwise nothing has been launched).  ratio is checked like hx_score_placements' but not
// written: the caller forms it once the launch has produced the horizons (the commit kernel does).
int hx_reveal_search(hx_ctx *ctx, const hx_model *model, const hx_calls *calls,
                     const hx_prefill_tab *pre, const hx_decode_tab *dec, const hx_links *links,
                     const float *tail, const float *horizon, int32_t n_nodes, int32_t n_wf,
                     int32_t *best_p, int32_t *best_d, float *best_cost, float *ratio,
                     const HxHorizonsPlan *reveal, bool *revealed, void *stream_)
{
    *revealed = false;
    return score_placements(ctx, model, calls, pre, dec, links, tail, horizon, n_nodes, n_wf, nullptr, nullptr,
                            best_p, best_d, best_cost, ratio, reveal, nullptr, revealed, stream_);
}

// The walks of an append that has begun and hx_score_placements (fused outputs) in one launch, where the search is
// large enough beside them (*merged; otherwise nothing has been launched).  ratio: checked, not written, as above.
int hx_relax_search(hx_ctx *ctx, const hx_model *model, const hx_calls *calls,
                    const hx_prefill_tab *pre, const hx_decode_tab *dec, const hx_links *links,
                    const float *tail, const float *horizon, int32_t n_nodes, int32_t n_wf,
                    int32_t *best_p, int32_t *best_d, float *best_cost, float *ratio,
                    const HxAppendPlan *walks, bool *merged, void *stream_)
{
    *merged = false;
    return score_placements(ctx, model, calls, pre, dec, links, tail, horizon, n_nodes, n_wf, nullptr, nullptr,
                            best_p, best_d, best_cost, ratio, nullptr, walks, merged, stream_);
}

extern "C" int hx_select(hx_ctx *ctx, int32_t C, int32_t P, int32_t D, const float *cost,
                         const hx_calls *calls, const float *tail, const float *horizon,
                         int32_t n_nodes, int32_t n_wf,
                         int32_t *best_p, int32_t *best_d, float *best_cost, float *ratio, void *stream_)
{
    if (!ctx) return HX_ERR_INVALID_ARG;
    HX_REQUIRE(ctx, C >= 0 && P >= 0 && D >= 0, HX_ERR_INVALID_ARG, "negative size");
    HX_REQUIRE(ctx, (long long)P * D <= 2147483647LL, HX_ERR_SHAPE, "P*D beyond int32");
    HX_REQUIRE(ctx, best_p && best_d && best_cost, HX_ERR_INVALID_ARG, "NULL output");
    HX_REQUIRE(ctx, cost || (long long)C * P * D == 0, HX_ERR_INVALID_ARG, "cost is NULL");
    if (int rc = check_ratio_inputs(ctx, calls, tail, horizon, n_nodes, n_wf, ratio)) return rc;
    HX_REQUIRE(ctx, !calls || calls->n == C, HX_ERR_INVALID_ARG, "calls.n differs from C");
    if (C == 0) return HX_OK;
    HxDeviceGuard guard(ctx->device);
    HX_REQUIRE(ctx, guard.ok, HX_ERR_DEVICE, "cannot select device %d", ctx->device);
    hipStream_t stream = (hipStream_t)stream_;
    ScoreArgs a{};
    a.C = C; a.P = P; a.D = D; a.cost = const_cast<float *>(cost);
    if (calls) { a.node = calls->node; a.wf = calls->wf; a.elapsed = calls->elapsed; }
    a.tail = tail; a.horizon = horizon; a.n_nodes = n_nodes; a.n_wf = n_wf;
    a.best_p = best_p; a.best_d = best_d; a.best_cost = best_cost; a.ratio = ratio; a.status = ctx->d_status;
    const int grid = C < ctx->num_cu * 8 ? C : ctx->num_cu * 8;
    hx_select_kernel<<<grid, 256, 0, stream>>>(a);
    return hx_check_launch(ctx, "hx_select_kernel");
}

extern "C" int hx_urgency(hx_ctx *ctx, const hx_calls *calls, const float *best_cost,
                          const float *tail, const float *horizon, int32_t n_nodes, int32_t n_wf,
                          float *ratio, void *stream_)
{
    if (!ctx) return HX_ERR_INVALID_ARG;
    HX_REQUIRE(ctx, calls, HX_ERR_INVALID_ARG, "NULL calls");
    const int C = calls->n;
    HX_REQUIRE(ctx, C >= 0 && n_nodes >= 0 && n_wf >= 0, HX_ERR_INVALID_ARG, "negative size");
    HX_REQUIRE(ctx, C == 0 || (calls->node && calls->wf && calls->elapsed && best_cost && tail && horizon && ratio),
               HX_ERR_INVALID_ARG, "the ratio needs node, wf, elapsed, best_cost, tail and horizon");
    if (C == 0) return HX_OK;
    HxDeviceGuard guard(ctx->device);
    HX_REQUIRE(ctx, guard.ok, HX_ERR_DEVICE, "cannot select device %d", ctx->device);
    hx_urgency_kernel<<<(C + 255) / 256, 256, 0, (hipStream_t)stream_>>>(calls->node, calls->wf, calls->elapsed, best_cost, tail, horizon,
                                                                       n_nodes, n_wf, C, ratio, ctx->d_status);
    return hx_check_launch(ctx, "hx_urgency_kernel");
}
