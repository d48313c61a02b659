// The search of one call over the whole pool by one wavefront: the inner part
// of the fused scoring kernel, shared with the recomputing-greedy planner so
// that both compare exactly the same fp32 costs.
//
// Lanes are prefill instances (KP per lane, in chunks of 64*KP beyond that).
// What depends on the decode instance only is the same for all 64 lanes and is
// read from LDS as broadcasts: the instance's availability hint (from the
// workgroup's pool tables, it does not depend on the call) and the call's
// decode time there (+inf where the call does not fit), written once per call
// into the wave's own buffer; decode entries are grouped by GPU class, so the transfer time
// leaves the inner loop, which is  t = max(ready, avail_d) + dec_d ;
// best = min(best, t)  with no index bookkeeping.  The index is recovered
// afterwards: the wave minimum fixes the winning prefill instance (lowest p
// among the lanes that hold the minimum), and one pass over that instance's
// candidates finds the lowest d that reproduces the minimum bit for bit --
// exactly the lexicographic minimum of (cost, p*D + d).
#pragma once

#include "hx_common.hpp"
#include "hx_terms.hpp"

#include <cmath>

// Minimum over the 64 lanes of a wavefront with data-parallel-primitive lane
// moves (no LDS traffic): two quad swaps and two row mirrors leave every row
// of 16 lanes holding its minimum, two row broadcasts carry it to lane 63,
// which is read back as a wave-uniform value.  Each step is one instruction,
// the minimum itself taking its first operand through the lane move (lanes
// a row mask leaves out keep their value: the destination is the operand).
// A lane move may read a register two cycles after a vector instruction wrote
// it at the earliest, and five after one wrote the execution mask; the
// compiler does not see inside these statements, so they carry their own waits
// (and one at the end, before the lane read that follows).
#define HX_DPP_MIN_CHAIN(OP)                                                                  \
    "s_nop 4\n\t" OP " %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"        \
    "s_nop 1\n\t" OP " %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"        \
    "s_nop 1\n\t" OP " %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"            \
    "s_nop 1\n\t" OP " %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\t"                 \
    "s_nop 1\n\t" OP " %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"               \
    "s_nop 1\n\t" OP " %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"               \
    "s_nop 1"

__device__ __forceinline__ float hx_wave_min(float x)
{
    asm volatile(HX_DPP_MIN_CHAIN("v_min_f32_dpp") : "+v"(x));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

__device__ __forceinline__ int hx_wave_min(int x)
{
    asm volatile(HX_DPP_MIN_CHAIN("v_min_i32_dpp") : "+v"(x));
    return __builtin_amdgcn_readlane(x, 63);
}

__device__ __forceinline__ float hx_wave_max(float x)
{
    asm volatile(HX_DPP_MIN_CHAIN("v_max_f32_dpp") : "+v"(x));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

// The wavefront's largest value and the lowest index that has it, in every lane.  A lane without a
// candidate passes (-inf, INT_MAX): it loses to every candidate, also to one whose value is -inf.
// Every lane of the wavefront must be active.
__device__ __forceinline__ void hx_wave_argmax(float &v, int &i)
{
    const float top = hx_wave_max(v);
    i = hx_wave_min(v == top ? i : 0x7fffffff);
    v = top;
}

// views of the pool tables staged in LDS
struct HxPoolLds {
    const float *wait, *c1, *c2, *kB;      // decode entries (grouped by class, padded): availability hint and per-token terms
    const int *free, *orig, *dtype;        // free KV tokens, instance index (-1 = pad), class
    const float *pw, *pinvF, *pinvB;       // prefill instances, padded to Pp: wait, 1/F, 1/B
    const int *ptype;
    const float *invbw, *lat;              // [kT*kT] class-pair transfer tables
    int Dp, P, Pp;
};

struct HxBest {
    float cost;    // +inf when no pair is feasible
    int p, d;      // -1, -1 then
};

// One instruction each, in the order written (the compiler keeps volatile statements in order): the fold below
// fixes its instruction sequence by hand.  Same operations as hx_candidate and fminf, hence the same bits.
#define HX_VMAX(d, a, b) asm volatile("v_max_f32 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b))
#define HX_VADD(d, a, b) asm volatile("v_add_f32 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b))
#define HX_VMIN3(d, a, b, c) asm volatile("v_min3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c))

// Folds the eight candidates of one group of decode entries, availability in a0, a1, decode time in d0, d1, into the
// running minimum of each of the lane's KP prefill instances: t = max(ready, avail) + dec, three-input minima.
// A SIMD's main pipe issues the maxima and minima (one per 4 cycles); an addition can issue at the same time
// on the second fp32 pipe, for another wavefront.  The three kinds are therefore mixed finely -- the additions
// and minima of a slot between the maxima of the next -- so that whatever point of the sequence the other
// wavefronts of the SIMD are at, one of them is likely to offer an instruction of the other kind.
template <int KP>
__device__ __forceinline__ void hx_fold_group(const float (&r)[KP], float (&best)[KP],
                                              const float4 &a0, const float4 &a1, const float4 &d0, const float4 &d1)
{
    const float av[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
    const float dv[8] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
    float t[KP][8], m1[KP], m2[KP];
#pragma unroll
    for (int j = 0; j < KP; ++j) {
        HX_VMAX(t[j][0], r[j], av[0]);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (e + 1 < 8) HX_VMAX(t[j][e + 1], r[j], av[e + 1]);
            HX_VADD(t[j][e], t[j][e], dv[e]);
            if (j > 0 && e == 1) HX_VMIN3(best[j - 1], best[j - 1], t[j - 1][0], t[j - 1][1]);
            if (j > 0 && e == 3) HX_VMIN3(m1[j - 1], t[j - 1][2], t[j - 1][3], t[j - 1][4]);
            if (j > 0 && e == 5) HX_VMIN3(m2[j - 1], t[j - 1][5], t[j - 1][6], t[j - 1][7]);
            if (j > 0 && e == 7) HX_VMIN3(best[j - 1], best[j - 1], m1[j - 1], m2[j - 1]);
        }
    }
    HX_VMIN3(best[KP - 1], best[KP - 1], t[KP - 1][0], t[KP - 1][1]);
    HX_VMIN3(m1[KP - 1], t[KP - 1][2], t[KP - 1][3], t[KP - 1][4]);
    HX_VMIN3(m2[KP - 1], t[KP - 1][5], t[KP - 1][6], t[KP - 1][7]);
    HX_VMIN3(best[KP - 1], best[KP - 1], m1[KP - 1], m2[KP - 1]);
}

// dbuf: the wave's [Dp] decode times of the call (16-byte aligned); xbuf: the wave's [kT*kT] transfer times.
// s.wait (availability per decode entry) is read as it stands in the pool view: a caller that changes the
// pool between calls changes it there.  seg: class segments, wave-uniform.
template <int KP>
__device__ __forceinline__ HxBest hx_search_call(const HxModelF &m, const HxPoolLds &s,
                                                 const int (&seg)[HX_MAX_TYPES + 1],
                                                 float *dbuf, float *xbuf, int L, int O, int lane)
{
    constexpr int kT = HX_MAX_TYPES;
    const HxCallF cf = hx_call_terms(m, L, O);
    const int Dp = s.Dp;

    // decode time of this call on every decode entry (+inf where it does not fit), four entries per lane and
    // step (Dp is a multiple of the group size, the tables are 16-byte aligned)
    for (int e = 4 * lane; e < Dp; e += 4 * HX_WAVE) {
        const int4 fr = *(const int4 *)(s.free + e);
        const float4 c1 = *(const float4 *)(s.c1 + e), c2 = *(const float4 *)(s.c2 + e), kB = *(const float4 *)(s.kB + e);
        float4 t;
        t.x = hx_fits(L, O, fr.x) ? hx_decode_time(cf, c1.x, c2.x, kB.x) : INFINITY;
        t.y = hx_fits(L, O, fr.y) ? hx_decode_time(cf, c1.y, c2.y, kB.y) : INFINITY;
        t.z = hx_fits(L, O, fr.z) ? hx_decode_time(cf, c1.z, c2.z, kB.z) : INFINITY;
        t.w = hx_fits(L, O, fr.w) ? hx_decode_time(cf, c1.w, c2.w, kB.w) : INFINITY;
        *(float4 *)(dbuf + e) = t;
    }
    xbuf[lane] = hx_transfer(cf, s.invbw[lane], s.lat[lane]);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    float bestv = INFINITY;
    int bestp = -1;
    for (int chunk = 0; chunk < s.P; chunk += HX_WAVE * KP) {
        // per prefill instance of the lane: its finish time, and where its row of transfer times starts
        float done[KP], bj[KP];
        const float *xr[KP];
#pragma unroll
        for (int j = 0; j < KP; ++j) {
            int p = chunk + j * HX_WAVE + lane;
            p = p < s.Pp ? p : s.Pp - 1;            // stays inside the staged (padded) table
            const bool in = chunk + j * HX_WAVE + lane < s.P;
            done[j] = in ? hx_prefill_done(cf, s.pw[p], s.pinvF[p], s.pinvB[p]) : INFINITY;
            xr[j] = xbuf + s.ptype[p] * kT;
            bj[j] = INFINITY;
        }
#pragma unroll
        for (int k = 0; k < kT; ++k) {
            const float4 *qa = (const float4 *)(s.wait + seg[k]);
            const float4 *qd = (const float4 *)(dbuf + seg[k]);
            const int ngroups = (seg[k + 1] - seg[k]) / HX_DGROUP;
            // ready time at an instance of decode class k: prefill finish + transfer (formed per class rather than
            // kept for all classes: registers are what limits the wavefronts per SIMD)
            float rk[KP];
#pragma unroll
            for (int j = 0; j < KP; ++j) rk[j] = done[j] + xr[j][k];
            for (int g = 0; g < ngroups; ++g, qa += 2, qd += 2) hx_fold_group<KP>(rk, bj, qa[0], qa[1], qd[0], qd[1]);
        }
#pragma unroll
        for (int j = 0; j < KP; ++j) {
            // p grows with j and with chunk: "<" keeps the lowest p of this lane
            if (bj[j] < bestv) { bestv = bj[j]; bestp = chunk + j * HX_WAVE + lane; }
        }
    }
    // wave minimum of (cost, p): the minimum cost, then the lowest p among the lanes that hold it
    const float lane_best = bestv;
    bestv = hx_wave_min(lane_best);
    bestp = hx_wave_min(lane_best == bestv ? bestp : 0x7fffffff);
    HxBest out{bestv, -1, -1};
    if (bestv < INFINITY) {
        out.p = bestp;
        // lowest d of instance p* that reproduces the minimum exactly
        const float done = hx_prefill_done(cf, s.pw[bestp], s.pinvF[bestp], s.pinvB[bestp]);
        const float *xr = xbuf + s.ptype[bestp] * kT;
        int dmin = 0x7fffffff;
        // four entries per lane and step: a group of entries is of one class (pads have no decode time and never match)
        for (int e = 4 * lane; e < Dp; e += 4 * HX_WAVE) {
            const float ready = done + xr[s.dtype[e]];
            const float4 w = *(const float4 *)(s.wait + e), t = *(const float4 *)(dbuf + e);
            const int4 og = *(const int4 *)(s.orig + e);
            if (hx_candidate(ready, w.x, t.x) == bestv) dmin = min(dmin, og.x);
            if (hx_candidate(ready, w.y, t.y) == bestv) dmin = min(dmin, og.y);
            if (hx_candidate(ready, w.z, t.z) == bestv) dmin = min(dmin, og.z);
            if (hx_candidate(ready, w.w, t.w) == bestv) dmin = min(dmin, og.w);
        }
        out.d = hx_wave_min(dmin);
    }
    // the next call of this wave rewrites the buffers: order its writes after these reads
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    return out;
}

// The same result -- the lexicographic minimum of (cost, p, d) over the whole pool, bit for bit -- found
// class by class instead of pair by pair (for planners, which need the result, not the P x D costs).
// A candidate's cost is max(done_p + x[class_p][class_d], avail_d) + dec_d, non-decreasing in its first
// operand, and that operand depends on the decode instance through its class only: so the minimum over p
// for a decode entry is max(r[class_d], avail_d) + dec_d with r[k] = min over p of done_p + x[class_p][k],
// exactly (max and min round nothing, and the one addition is applied to the same operands).  P x T
// additions for r, D candidates, and for the (usually one) entry that attains the minimum a pass over p to
// find the lowest prefill instance that attains it there.
// dbuf, xbuf as in hx_search_call; rbuf: the wave's [HX_MAX_TYPES] floats.
__device__ __forceinline__ HxBest hx_search_call_by_class(const HxModelF &m, const HxPoolLds &s, float *dbuf, float *xbuf,
                                                          float *rbuf, int L, int O, int lane)
{
    constexpr int kT = HX_MAX_TYPES;
    const HxCallF cf = hx_call_terms(m, L, O);
    const int Dp = s.Dp;
    for (int e = lane; e < Dp; e += HX_WAVE)
        dbuf[e] = hx_fits(L, O, s.free[e]) ? hx_decode_time(cf, s.c1[e], s.c2[e], s.kB[e]) : INFINITY;
    xbuf[lane] = hx_transfer(cf, s.invbw[lane], s.lat[lane]);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // r[k]: the earliest the call's KV can be at an instance of decode class k
    float r[kT];
#pragma unroll
    for (int k = 0; k < kT; ++k) r[k] = INFINITY;
    for (int chunk = 0; chunk < s.P; chunk += HX_WAVE) {
        const int p = min(chunk + lane, s.Pp - 1);
        const float done = chunk + lane < s.P ? hx_prefill_done(cf, s.pw[p], s.pinvF[p], s.pinvB[p]) : INFINITY;
        const float *xr = xbuf + s.ptype[p] * kT;
#pragma unroll
        for (int k = 0; k < kT; ++k) r[k] = fminf(r[k], done + xr[k]);
    }
#pragma unroll
    for (int k = 0; k < kT; ++k) r[k] = hx_wave_min(r[k]);
    if (lane < kT) {
        float mine = r[0];
#pragma unroll
        for (int k = 1; k < kT; ++k) mine = lane == k ? r[k] : mine;
        rbuf[lane] = mine;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    float bv = INFINITY;
    for (int e = lane; e < Dp; e += HX_WAVE)
        bv = fminf(bv, hx_candidate(rbuf[s.dtype[e] & (kT - 1)], s.wait[e], dbuf[e]));
    bv = hx_wave_min(bv);
    HxBest out{bv, -1, -1};
    if (bv < INFINITY) {
        int best_p = 0x7fffffff, best_d = 0x7fffffff;
        for (int e0 = 0; e0 < Dp; e0 += HX_WAVE) {
            const int e = e0 + lane;
            bool hit = false;
            if (e < Dp) hit = s.orig[e] >= 0 && hx_candidate(rbuf[s.dtype[e] & (kT - 1)], s.wait[e], dbuf[e]) == bv;
            unsigned long long todo = __builtin_amdgcn_ballot_w64(hit);
            while (todo) {
                const int ee = e0 + __builtin_ctzll(todo);          // an entry that attains the minimum (wave-uniform)
                todo &= todo - 1;
                const float q_wait = s.wait[ee], q_dec = dbuf[ee];
                const int k = s.dtype[ee] & (kT - 1);
                int p_low = 0x7fffffff;
                for (int chunk = 0; chunk < s.P; chunk += HX_WAVE) {
                    const int p = min(chunk + lane, s.Pp - 1);
                    const float done = hx_prefill_done(cf, s.pw[p], s.pinvF[p], s.pinvB[p]);
                    const float v = hx_candidate(done + xbuf[s.ptype[p] * kT + k], q_wait, q_dec);
                    if (chunk + lane < s.P && v == bv) p_low = min(p_low, chunk + lane);
                }
                p_low = hx_wave_min(p_low);
                const int d = s.orig[ee];
                if (p_low < best_p || (p_low == best_p && d < best_d)) { best_p = p_low; best_d = d; }
            }
        }
        out.p = best_p; out.d = best_d;
    }
    // the next call of this wave rewrites the buffers: order its writes after these reads
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    return out;
}

// Cost of one pair (prefill instance p, decode entry e) for a call, by the same functions in the same
// order as the search above, hence bit-identical to what the search computes for that pair.
__device__ __forceinline__ float hx_pair_cost(const HxModelF &m, const HxPoolLds &s, int L, int O, int p, int e)
{
    constexpr int kT = HX_MAX_TYPES;
    const HxCallF cf = hx_call_terms(m, L, O);
    const float done = hx_prefill_done(cf, s.pw[p], s.pinvF[p], s.pinvB[p]);
    const int k = s.ptype[p] * kT + s.dtype[e];
    const float x = hx_transfer(cf, s.invbw[k], s.lat[k]);
    const float dec = hx_fits(L, O, s.free[e]) ? hx_decode_time(cf, s.c1[e], s.c2[e], s.kB[e]) : INFINITY;
    return hx_candidate(done + x, s.wait[e], dec);
}

// The library is built on the assumption that no arithmetic ever sees a NaN, so
// the NaN that marks a bad index is chosen among integers and stored as bits.
constexpr unsigned HX_QNAN_BITS = 0x7fc00000u;

// Eq. (2) with the downstream tail of the call's node, as bits: (elapsed + best
// + tail) / horizon; a workflow without a horizon (0: nothing it has revealed
// costs anything) makes its calls as urgent as can be, +inf; !ok gives the NaN.
__device__ __forceinline__ unsigned hx_ratio_bits(float elapsed, float best, float tail, float horizon, bool ok)
{
    const float r = horizon > 0.0f ? ((elapsed + best) + tail) / horizon : INFINITY;
    return ok ? __float_as_uint(r) : HX_QNAN_BITS;
}

__device__ __forceinline__ void hx_store_bits(float *out, int i, unsigned bits) { ((unsigned *)out)[i] = bits; }

// projected ratio of call c, stored to ratio[c].  A node or workflow index
// outside the arrays gives NaN and raises HX_ERR_INDEX.
__device__ __forceinline__ void hx_projected_ratio(const int32_t *node, const int32_t *wf, const float *elapsed,
                                                   const float *tail, const float *horizon, int n_nodes, int n_wf,
                                                   int c, float best, int32_t *status, float *ratio)
{
    const int nd = node[c], w = wf[c];
    const bool ok = nd >= 0 && nd < n_nodes && w >= 0 && w < n_wf;
    if (!ok) hx_raise(status, HX_ERR_INDEX);
    hx_store_bits(ratio, c, hx_ratio_bits(elapsed[c], best, ok ? tail[nd] : 0.0f, ok ? horizon[w] : 1.0f, ok));
}

// ordering key of a ratio: a NaN (raised elsewhere as a bad index) sorts with +inf
__device__ __forceinline__ float hx_rank_key(float r)
{
    const unsigned b = __float_as_uint(r);                       // chosen among integers: r may be the NaN
    return __uint_as_float((b & 0x7fffffffu) > 0x7f800000u ? 0x7f800000u : b);
}
