// The decode stage (Sec. 5.4): calls whose KV has arrived wait for decode
// admission.  A call needs L_in + L_out tokens of KV (Eq. 3) under the
// instance's capacity (Eq. 4) for as long as it decodes; each instance carries
// token-capacity intervals (who holds how many tokens from when to when), and
// the earliest capacity-feasible start on an instance is the first moment from
// which the call fits for its whole decode time.  Projected finish = that start
// + decode time (Sec. 5.1: waiting for decode capacity plus decode execution);
// a call locked to an instance during prefill planning may only go there.
//
// Per instance the intervals are turned into a timeline: the distinct event
// times >= now in increasing order with the occupancy from each time to the
// next.  A start is feasible when a run of consecutive timeline segments that
// all leave room covers the decode time; a run can only begin where occupancy
// drops, i.e. now or at the end of an interval.
#include "hx_common.hpp"
#include "hx_terms.hpp"
#include "hx_search.hpp"

#include <climits>
#include <cmath>

namespace {

typedef unsigned long long u64;

// ---- timeline of one instance, built in LDS by a whole workgroup --------------------

// scratch for 2*cnt + 1 events (the extra one is "now")
struct TlScratch {
    u64 *key;        // (time bits, end-before-start flag, event id): unique, orders the events
    int *delta;      // +tok at a start, -tok at an end
    float *ts;       // sorted: time
    int *ds;         //         delta
};

// compact timeline: entry i covers [t_i, t_{i+1}) (the last one has no end) with occupancy occ_i
struct Tl {
    int2 *e;         // (time bits, occupancy)
};

__host__ __device__ inline size_t hx_align16(size_t x) { return (x + 15) & ~(size_t)15; }

// The scans read whole groups of entries, one group ahead: a timeline of up to ne entries is
// stored in ne rounded up to a multiple of eight, plus sixteen, the rest filled with (never, empty).
__host__ __device__ inline int hx_tl_len(int ne) { return ((ne + 7) & ~7) + 16; }

__device__ inline TlScratch hx_carve_scratch(unsigned char *p, int ne)
{
    TlScratch w;
    w.key = (u64 *)p;                 p += hx_align16((size_t)ne * 8);
    w.delta = (int *)p;               p += hx_align16((size_t)ne * 4);
    w.ts = (float *)p;                p += hx_align16((size_t)ne * 4);
    w.ds = (int *)p;
    return w;
}
__host__ __device__ inline size_t hx_scratch_bytes(int ne)
{
    return hx_align16((size_t)ne * 8) + 3 * hx_align16((size_t)ne * 4);
}

template <bool COHERENT, typename T> __device__ __forceinline__ T hx_ld(const T *p)
{
    // COHERENT: the value may have been written by another wave of this workgroup a moment ago
    if (COHERENT) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return *p;
}

// Counting against all of n keys, one key per group of `parts` neighbouring lanes: 4 or 2 lanes per key where the
// workgroup has that many threads to spare (a power of two, so a group lies inside a quad of lanes).
__device__ __forceinline__ int hx_count_parts(int n, int nthreads) { return 4 * n <= nthreads ? 4 : (2 * n <= nthreads ? 2 : 1); }

// the sum over the lanes of a group (lane moves inside the quad; every lane of the group is active)
__device__ __forceinline__ int hx_parts_sum(int r, int parts)
{
    if (parts >= 2) r += __builtin_amdgcn_update_dpp(0, r, 0xB1, 0xf, 0xf, false);      // quad_perm [1,0,3,2]
    if (parts >= 4) r += __builtin_amdgcn_update_dpp(0, r, 0x4E, 0xf, 0xf, false);      // quad_perm [2,3,0,1]
    return r;
}

// All threads of the workgroup call this.  cnt entries of one instance -> compact timeline in
// `out`, its length in *n_out (LDS).  Ends the call with a barrier.
template <bool COHERENT>
__device__ void hx_build_timeline(int cnt, const float *st, const float *en, const int32_t *tk,
                                  TlScratch w, Tl out, int *n_out, int32_t *status)
{
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const int n_ev = 2 * cnt + 1;
    for (int i = tid; i < n_ev; i += nthreads) {
        float time = 0.0f;
        int delta = 0;
        unsigned is_end = 1;                               // event 0 is "now"
        if (i > 0) {
            const int j = (i - 1) >> 1;
            is_end = (unsigned)(i - 1) & 1u;
            const float s = hx_ld<COHERENT>(st + j), e = hx_ld<COHERENT>(en + j);
            const int k = hx_ld<COHERENT>(tk + j);
            if (s < e && k > 0) {                          // anything else (NaN times included) holds nothing
                const float x = is_end ? e : s;
                time = x > 0.0f ? x : 0.0f;                // the past is folded onto now
                delta = is_end ? -k : k;
            }
        }
        // at equal times starts sort before ends, so the last event of a time is an end if there is one
        w.key[i] = ((u64)__float_as_uint(time) << 32) | ((u64)is_end << 31) | (unsigned)i;
        w.delta[i] = delta;
    }
    __syncthreads();
    // position of every event = number of smaller keys (keys are unique); with threads to spare, the 2 or 4
    // neighbouring lanes of an event count a part of the keys each
    const int parts = hx_count_parts(n_ev, nthreads);
    const int share = ((n_ev + parts - 1) / parts + 7) & ~7;
    for (int i = tid / parts; i < n_ev; i += nthreads / parts) {
        const u64 ki = w.key[i];
        const int j_lo = min((tid & (parts - 1)) * share, n_ev), j_hi = min(j_lo + share, n_ev);
        int r = 0;
        int j = j_lo;
        for (; j + 8 <= j_hi; j += 8) {                   // eight independent reads in flight
            u64 kk[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) kk[u] = w.key[j + u];
#pragma unroll
            for (int u = 0; u < 8; ++u) r += kk[u] < ki;
        }
        for (; j < j_hi; ++j) r += w.key[j] < ki;
        r = hx_parts_sum(r, parts);
        if ((tid & (parts - 1)) == 0) {
            w.ts[r] = __uint_as_float((unsigned)(ki >> 32));
            w.ds[r] = w.delta[i];
        }
    }
    __syncthreads();
    // one wavefront: running occupancy, and one entry per distinct time (the last event of that time)
    if (tid < HX_WAVE) {
        const int per = (n_ev + HX_WAVE - 1) / HX_WAVE;
        const int lo = min(tid * per, n_ev), hi = min(lo + per, n_ev);
        long long sum = 0;
        int heads = 0;
        for (int i = lo; i < hi; ++i) {
            sum += w.ds[i];
            heads += (i == n_ev - 1) || (w.ts[i + 1] != w.ts[i]);
        }
        long long psum = sum;
        int ph = heads;
#pragma unroll
        for (int off = 1; off < HX_WAVE; off <<= 1) {
            const long long o = __shfl_up(psum, off);
            const int oh = __shfl_up(ph, off);
            if (tid >= off) { psum += o; ph += oh; }
        }
        long long run = psum - sum;
        int pos = ph - heads;
        for (int i = lo; i < hi; ++i) {
            run += w.ds[i];
            if ((i == n_ev - 1) || (w.ts[i + 1] != w.ts[i])) {
                if (run > (long long)INT_MAX) hx_raise(status, HX_ERR_OVERFLOW);
                const int occ = run > (long long)INT_MAX ? INT_MAX : (int)run;
                out.e[pos] = make_int2(__float_as_int(w.ts[i]), occ);
                ++pos;
            }
        }
        if (tid == HX_WAVE - 1) *n_out = pos;
    }
    __syncthreads();
    for (int i = *n_out + tid; i < hx_tl_len(n_ev); i += nthreads) out.e[i] = make_int2(0x7f800000, 0);
    __syncthreads();
}

// ---- earliest capacity-feasible start, one lane per (call, instance) ------------------

struct HxSlot {
    float S;     // start, +inf if none
    bool found;
};

// thr = tokens the call may find occupied (capacity - demand), < 0: never fits.  T = decode time.
// Lanes of a wavefront may scan different timelines (e 16-byte aligned, padded as hx_tl_len says).
//
// Straight-line arithmetic per entry, no flags: rs is the start of the run of entries with room
// that the scan is in, +inf while it is in none (a run begins at the first entry with room:
// min(+inf, t_i) = t_i; inside a run t_i > rs leaves rs alone); the run is long enough once the next
// entry's time reaches rs + T, which cannot happen outside a run (rs + T = +inf, and the entry
// whose successor is "never" always has room: everything has ended by then).  Run starts only
// grow along the timeline, so the earliest start is the minimum over all hits.  The loop ends when
// every lane has its answer or has passed the end of its timeline.
__device__ __forceinline__ HxSlot hx_earliest_start(const int2 *e, int n, int thr, float T, bool active)
{
    const bool open = active && thr >= 0;
    float rs = INFINITY, ans = INFINITY;
#define HX_TL_STEP(cur_, occ_, nxt_)                                              \
    {                                                                             \
        rs = (occ_) <= thr ? fminf(rs, __int_as_float(cur_)) : INFINITY;          \
        ans = fminf(ans, __int_as_float(nxt_) >= rs + T ? rs : INFINITY);         \
    }
    // eight entries per step, the next eight already on their way (lanes that are through read entry 0 on)
    const int4 *q = reinterpret_cast<const int4 *>(e);
    int4 c0 = q[0], c1 = q[1], c2 = q[2], c3 = q[3];
    for (int i0 = 0;; i0 += 8) {
        const bool going = open && i0 < n && !(ans < INFINITY);
        if (__builtin_amdgcn_ballot_w64(going) == 0) break;
        const int at = going ? (i0 >> 1) + 4 : 0;
        const int4 n0 = q[at], n1 = q[at + 1], n2 = q[at + 2], n3 = q[at + 3];
        const float keep = ans;
        HX_TL_STEP(c0.x, c0.y, c0.z)
        HX_TL_STEP(c0.z, c0.w, c1.x)
        HX_TL_STEP(c1.x, c1.y, c1.z)
        HX_TL_STEP(c1.z, c1.w, c2.x)
        HX_TL_STEP(c2.x, c2.y, c2.z)
        HX_TL_STEP(c2.z, c2.w, c3.x)
        HX_TL_STEP(c3.x, c3.y, c3.z)
        HX_TL_STEP(c3.z, c3.w, n0.x)
        ans = going ? ans : keep;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
#undef HX_TL_STEP
    const bool found = open && ans < INFINITY;
    return HxSlot{found ? ans : INFINITY, found};
}

// ---- one scoring pass over (queue x instances) -----------------------------------------

struct DecodeArgs {
    HxModelF m;
    int Q, D, stride;
    const int32_t *L_in, *L_out, *lock;
    const float *d_flops, *d_hbm;
    const int32_t *d_used, *d_cap, *d_batch;
    const int32_t *iv_count;
    const float *iv_start, *iv_end;
    const int32_t *iv_tok;
    float *start, *cost;
    // The free calls (valid, not locked) of the queue in queue order: the queue is cut into D slices of `per`
    // calls, slice d's free calls are free_c[d*per ..], n_free[d] of them.  Unused when there are no locks.
    int32_t *free_c, *n_free;
    int per;
    // Best candidate of every call within each group of gd consecutive instances: [group][Q] each.
    int gd, n_groups;
    float *part_cost, *part_start;
    int32_t *part_d;
    int32_t *status;
};

// what a lane knows of its call on an instance
struct HxDecodeCand {
    float T;
    int thr;
    bool legal;
};

__device__ __forceinline__ HxDecodeCand hx_decode_candidate(const HxModelF &m, int L, int O, int lk, int d, int D,
                                                            const HxDecF &x, int cap, int32_t *status)
{
    HxDecodeCand c;
    bool ok = L >= 0 && O >= 0 && lk >= -1 && lk < D;
    if (!ok) hx_raise(status, HX_ERR_INDEX);
    c.legal = ok && (lk < 0 || lk == d);
    const HxCallF cf = hx_call_terms(m, ok ? L : 0, ok ? O : 0);
    c.T = hx_decode_time(cf, x.c1, x.c2, x.kB);
    const long long room = (long long)cap - ((long long)L + (long long)O);
    c.thr = (!ok || room < 0) ? -1 : (room > (long long)INT_MAX ? INT_MAX : (int)room);
    return c;
}

// How the scoring kernel searches an instance's timeline, decided here per instance.
constexpr int HX_TAB = 4096;          // entries of the first-room table at most
constexpr int HX_TAB_MAX_N = 512;     // timeline entries at most for the table (their occupancies are ranked all against all)
constexpr int HX_TAB_FLAG = 1 << 16;  // added to the stretch count in an instance's record: the table was written

struct TlOut {
    int2 *e;         // [D][nt] timeline entries, padded
    int *n;          // [D] entries
    int *seg;        // [D][nt] heads of the stretches, then n
    int2 *head;      // [D][nt] per stretch: (time of its head, rank of the head's occupancy), padded with (-inf, 0)
    int *sorted;     // [D][nt] the n occupancies in increasing order
    float *G;        // [D][HX_TAB] first-room table
    int *meta;       // [D][8] what the scoring kernel reads first of an instance: n, m (+flag), capacity, decode terms c1, c2, kB
};

// Workgroup d: everything the scoring kernel needs of instance d -- its timeline, built in LDS; the timeline's
// stretches of non-increasing occupancy; where that is small enough, the first-room table; a record of the
// instance's sizes and decode terms -- and the free calls among the d-th slice of the queue, in order.
constexpr int TL_THREADS = 512;
__global__ __launch_bounds__(TL_THREADS) void hx_decode_timeline_kernel(DecodeArgs a, TlOut o, int nt)
{
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int s_n, s_m;
    const int tid = threadIdx.x;
    const int d = blockIdx.x;
    const int ne = 2 * a.stride + 1;
    TlScratch w = hx_carve_scratch(smem, ne);
    Tl tl;
    tl.e = (int2 *)(smem + hx_scratch_bytes(ne));
    int cnt = a.iv_count[d];
    if (cnt < 0 || cnt > a.stride) {
        if (tid == 0) hx_raise(a.status, HX_ERR_INDEX);
        cnt = cnt < 0 ? 0 : a.stride;
    }
    // this workgroup's slice of the queue (see below): its first calls are asked for now and used after the build
    const int c_lo = d * a.per, c_hi = min(a.Q, (d + 1) * a.per);
    const bool pre_in = a.lock && c_lo + tid < c_hi;
    const int pre_L = pre_in ? a.L_in[c_lo + tid] : 0, pre_O = pre_in ? a.L_out[c_lo + tid] : 0;
    const int pre_lk = pre_in ? a.lock[c_lo + tid] : -1;
    const size_t at = (size_t)d * a.stride;
    hx_build_timeline<false>(cnt, a.iv_start + at, a.iv_end + at, a.iv_tok + at, w, tl, &s_n, a.status);
    const int n = s_n;
    // Everything below is worked out in LDS and registers first and written to memory at the very end: a
    // barrier waits for the stores before it, and there are several barriers to come.

    // This workgroup's slice of the queue: its free calls, in order.  A thread keeps the place of its call of
    // the first 512 (few slices are longer) and writes it with the rest.
    int my_place = -1, n_free = 0;
    if (a.lock) {
        __shared__ int s_wave_n[TL_THREADS / HX_WAVE];
        const int lane = tid & (HX_WAVE - 1), wave = tid >> 6;
        for (int base = c_lo; base < c_hi; base += blockDim.x) {
            const int c = base + tid;
            const bool in = c < c_hi;
            const bool first = base == c_lo;
            const int L = first ? pre_L : (in ? a.L_in[c] : 0), O = first ? pre_O : (in ? a.L_out[c] : 0);
            const int lk = first ? pre_lk : (in ? a.lock[c] : -1);
            const bool ok = L >= 0 && O >= 0 && lk >= -1 && lk < a.D;
            if (!ok) hx_raise(a.status, HX_ERR_INDEX);
            const bool is_free = in && ok && lk < 0;
            const u64 mf = __builtin_amdgcn_ballot_w64(is_free);
            if (lane == 0) s_wave_n[wave] = __popcll(mf);
            __syncthreads();
            int before = n_free;
            for (int w2 = 0; w2 < wave; ++w2) before += s_wave_n[w2];
            const int place = before + __popcll(mf & ((1ull << lane) - 1ull));
            if (is_free) {
                if (first) my_place = place;
                else a.free_c[d * a.per + place] = c;
            }
            for (int w2 = 0; w2 < TL_THREADS / HX_WAVE; ++w2) n_free += s_wave_n[w2];
            __syncthreads();
        }
    }

    // Occupancy rises only where a planned interval starts; between two such entries it never rises.  The
    // heads of these stretches (entry 0 and every entry above its predecessor), in order, and n as the last one.
    // The builder's scratch is free again: seg_l, rank and sorted live there.
    short *seg_l = (short *)w.ds;
    if (tid < HX_WAVE) {
        const int per_lane = (n + HX_WAVE - 1) / HX_WAVE;
        const int lo = min(tid * per_lane, n), hi = min(lo + per_lane, n);
        int heads = 0;
        for (int i = lo; i < hi; ++i) heads += i == 0 || tl.e[i].y > tl.e[i - 1].y;
        int incl = heads;
#pragma unroll
        for (int off = 1; off < HX_WAVE; off <<= 1) {
            const int up = __shfl_up(incl, off);
            if (tid >= off) incl += up;
        }
        int pos = incl - heads;
        for (int i = lo; i < hi; ++i)
            if (i == 0 || tl.e[i].y > tl.e[i - 1].y) seg_l[pos++] = (short)i;
        if (tid == HX_WAVE - 1) { seg_l[incl] = (short)n; s_m = incl; }
    }
    // (occupancy, entry) as one key, for the ranks below
    for (int i = tid; i < n; i += blockDim.x) w.key[i] = ((u64)(unsigned)tl.e[i].y << 16) | (unsigned)i;
    __syncthreads();
    const int m = s_m;
    // Few stretches over a timeline of moderate length: the table below fits and the scoring kernel uses it.
    const bool table = n <= HX_TAB_MAX_N && m * (n + 1) <= HX_TAB;
    // Whether an entry leaves room for a call depends only on how the call's threshold ranks among the n
    // occupancies: with r = the number of occupancies <= threshold, entry i has room exactly when
    // rank_i = #{j : occ_j <= occ_i} is <= r.  The keys below an entry's own give its place in increasing
    // order, the keys below (occupancy + 1, 0) its rank.
    int *rank = w.delta, *sorted = (int *)w.ts;
    if (table) {
        const int parts = hx_count_parts(n, TL_THREADS);
        const int share = ((n + parts - 1) / parts + 7) & ~7;
        for (int i = tid / parts; i < n; i += TL_THREADS / parts) {
            const u64 mine = w.key[i], above = ((mine >> 16) + 1) << 16;
            const int j_lo = min((tid & (parts - 1)) * share, n), j_hi = min(j_lo + share, n);
            int place = 0, le = 0;
            int j = j_lo;
            for (; j + 8 <= j_hi; j += 8) {                // eight independent reads in flight
                u64 other[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) other[u] = w.key[j + u];
#pragma unroll
                for (int u = 0; u < 8; ++u) { place += other[u] < mine; le += other[u] < above; }
            }
            for (; j < j_hi; ++j) { const u64 other = w.key[j]; place += other < mine; le += other < above; }
            place = hx_parts_sum(place, parts); le = hx_parts_sum(le, parts);
            if ((tid & (parts - 1)) == 0) {
                rank[i] = le;
                sorted[place] = (int)(mine >> 16);
            }
        }
        __syncthreads();
    }

    // ---- the last barrier is behind: everything goes to memory
    for (int i = tid; i < hx_tl_len(2 * cnt + 1); i += blockDim.x) o.e[(size_t)d * nt + i] = tl.e[i];
    for (int k = tid; k <= m; k += blockDim.x) o.seg[(size_t)d * nt + k] = (int)seg_l[k];
    if (my_place >= 0) a.free_c[d * a.per + my_place] = c_lo + tid;
    if (tid == 0) {
        o.n[d] = n;
        if (a.lock) a.n_free[d] = n_free;
        // the instance's decode terms are the same for every call: worked out here, once
        const HxDecF x = hx_decode_terms(a.m, a.d_used[d], a.d_batch[d], 0, 1.0f / a.d_flops[d], 1.0f / a.d_hbm[d]);
        int *meta = o.meta + 8 * d;
        meta[0] = n; meta[1] = table ? (m | HX_TAB_FLAG) : m; meta[2] = a.d_cap[d];
        meta[3] = __float_as_int(x.c1); meta[4] = __float_as_int(x.c2); meta[5] = __float_as_int(x.kB); meta[6] = 0; meta[7] = 0;
    }
    if (!table) return;
    for (int i = tid; i < n; i += blockDim.x) o.sorted[(size_t)d * nt + i] = sorted[i];
    for (int k = tid; k < hx_tl_len(m); k += blockDim.x)
        o.head[(size_t)d * nt + k] = k < m ? make_int2(tl.e[seg_l[k]].x, rank[seg_l[k]]) : make_int2((int)0xff800000u, 0);
    // G[k][r]: the time of the first entry of stretch k that has room at threshold rank r, +inf if none has.
    // Ranks never rise inside a stretch, so that entry is found by bisection.
    const int width = n + 1;
    for (int idx = tid; idx < m * width; idx += blockDim.x) {
        const int k = idx / width, r = idx - k * width;
        const int last = seg_l[k + 1];
        int lo = seg_l[k], hi = last;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (rank[mid] <= r) hi = mid; else lo = mid + 1;
        }
        o.G[(size_t)d * HX_TAB + idx] = lo < last ? __int_as_float(tl.e[lo].x) : INFINITY;
    }
}

// The same scan as hx_earliest_start for a timeline every lane of the wavefront shares.  The
// timeline was written by an earlier kernel and nothing writes it now, so it is read through the
// constant address space: with wave-uniform addresses the entries arrive as scalars, cost no vector
// memory or LDS traffic, and feed the vector arithmetic as scalar operands.  Eight entries per
// step, the next eight already on their way.
typedef int HxTlGroup __attribute__((ext_vector_type(16)));      // eight (time, occupancy) entries
typedef __attribute__((address_space(4))) const HxTlGroup *hx_tl_group_cp;

__device__ __forceinline__ float hx_earliest_start_shared(const int2 *__restrict__ e, int n, int thr, float T, bool active)
{
    const bool open = active && thr >= 0;
    float rs = INFINITY, ans = INFINITY;
#define HX_TL_STEP(cur_, occ_, nxt_)                                              \
    {                                                                             \
        rs = (occ_) <= thr ? fminf(rs, __int_as_float(cur_)) : INFINITY;          \
        ans = fminf(ans, __int_as_float(nxt_) >= rs + T ? rs : INFINITY);         \
    }
    const hx_tl_group_cp g = (hx_tl_group_cp)(unsigned long long)e;
    HxTlGroup cur = g[0];
    for (int i0 = 0; i0 < n; i0 += 8) {
        if (__builtin_amdgcn_ballot_w64(open && !(ans < INFINITY)) == 0) break;
        const HxTlGroup nxt = g[(i0 >> 3) + 1];
        // a lane that already has its answer keeps it: later hits have later starts
        HX_TL_STEP(cur[0], cur[1], cur[2])
        HX_TL_STEP(cur[2], cur[3], cur[4])
        HX_TL_STEP(cur[4], cur[5], cur[6])
        HX_TL_STEP(cur[6], cur[7], cur[8])
        HX_TL_STEP(cur[8], cur[9], cur[10])
        HX_TL_STEP(cur[10], cur[11], cur[12])
        HX_TL_STEP(cur[12], cur[13], cur[14])
        HX_TL_STEP(cur[14], cur[15], nxt[0])
        cur = nxt;
    }
#undef HX_TL_STEP
    return open ? ans : INFINITY;
}

// The start from the first-room table (see the timeline kernel).  r: the rank of the call's threshold.
// Stretch by stretch: a run that reaches a head lasted until then, which is where its length is tested
// (the entry-by-entry scan tests it at every entry, but a run long enough at an entry inside a stretch
// is still the same run, and long enough, at the next head or at the end); the run survives the head if
// the head has room; otherwise the next run begins at the stretch's first entry with room, G[k][r].
// Inside a run that entry is the head itself, later than the run's start, so one minimum serves both
// cases.  The same comparisons on the same values as the scan: the same start bit for bit.
// head: per stretch (time, rank) in groups of eight, read as scalars; G, sorted: LDS.
// first: the first eight heads, which the caller asked for ahead of time.
__device__ __forceinline__ float hx_earliest_start_table(const int2 *__restrict__ head, HxTlGroup first, const float *G,
                                                         const int *sorted, int n, int m, int thr, float T, bool active)
{
    const bool open = active && thr >= 0;
    int r = 0;
    {
        int lo = 0, hi = n;                                // first position of sorted[] above thr = #{occ <= thr}
        while (__builtin_amdgcn_ballot_w64(lo < hi) != 0) {
            const int mid = (lo + hi) >> 1;
            const bool le = sorted[min(mid, n - 1)] <= thr;
            if (lo < hi) { if (le) lo = mid + 1; else hi = mid; }
        }
        r = open ? lo : 0;                                 // rank 0: no entry has room
    }
    const float *Gr = G + r;
    const int width = n + 1;
    float rs = INFINITY, ans = INFINITY;
    // Eight stretches per step: their heads arrive as scalars, their table entries are read together.  Past the
    // last stretch the heads are (-inf, rank 0) and the table row is the last one again: no hit, the run
    // kept, and a minimum with a value that is already in it.
#define HX_HEAD_STEP(u_)                                                          \
    {                                                                             \
        ans = fminf(ans, __int_as_float(cur[2 * (u_)]) >= rs + T ? rs : INFINITY); \
        rs = cur[2 * (u_) + 1] <= r ? rs : INFINITY;                              \
        rs = fminf(rs, gv[u_]);                                                   \
    }
    const hx_tl_group_cp g = (hx_tl_group_cp)(unsigned long long)head;
    HxTlGroup cur = first;
    for (int k0 = 0; k0 < m; k0 += 8) {
        if (__builtin_amdgcn_ballot_w64(open && !(ans < INFINITY)) == 0) break;
        const HxTlGroup nxt = g[(k0 >> 3) + 1];
        float gv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) gv[u] = Gr[min(k0 + u, m - 1) * width];
        HX_HEAD_STEP(0) HX_HEAD_STEP(1) HX_HEAD_STEP(2) HX_HEAD_STEP(3)
        HX_HEAD_STEP(4) HX_HEAD_STEP(5) HX_HEAD_STEP(6) HX_HEAD_STEP(7)
        cur = nxt;
    }
#undef HX_HEAD_STEP
    ans = fminf(ans, INFINITY >= rs + T ? rs : INFINITY);  // the last run reaches the end of the timeline
    return open ? ans : INFINITY;
}

// The same result by stretches instead of entries.  Inside a stretch occupancy never rises, so the
// entries with room are its tail, found by bisection; a run that has begun continues through every
// later stretch whose head still has room and ends at the first head that has not, which is where
// its length is tested (a run long enough at any earlier entry is long enough there).  All
// comparisons are the ones the entry-by-entry scan makes, on the same values, so the start is the
// same bit for bit; the work per (call, instance) is a few operations per stretch plus the
// bisections instead of seven per entry.  e: the timeline in LDS; seg[0..m]: heads and n.
__device__ __forceinline__ float hx_earliest_start_stretches(const int2 *e, const int *seg, int n, int m, int thr, float T, bool active)
{
    const bool open = active && thr >= 0;
    float rs = INFINITY, ans = INFINITY;
    for (int k = 0; k < m; ++k) {
        if (__builtin_amdgcn_ballot_w64(open && !(ans < INFINITY)) == 0) break;
        const int first = seg[k], last = seg[k + 1];
        const int2 head = e[first];
        const bool head_room = head.y <= thr;
        // a run that reaches a head lasted until then (rs = +inf outside a run: no hit)
        ans = fminf(ans, __int_as_float(head.x) >= rs + T ? rs : INFINITY);
        rs = head_room ? rs : INFINITY;
        // lanes outside a run take the first entry with room in this stretch, if there is one
        const bool need = open && !(rs < INFINITY);
        if (__builtin_amdgcn_ballot_w64(need) != 0) {
            int lo = first, hi = last;
            while (__builtin_amdgcn_ballot_w64(need && lo < hi) != 0) {
                const int mid = (lo + hi) >> 1;
                const bool room = e[min(mid, n - 1)].y <= thr;
                if (lo < hi) { if (room) hi = mid; else lo = mid + 1; }
            }
            if (need && lo < last) rs = __int_as_float(e[lo].x);
        }
    }
    ans = fminf(ans, INFINITY >= rs + T ? rs : INFINITY);  // the last run reaches the end of the timeline
    return open ? ans : INFINITY;
}

// What the scoring kernel knows of an instance: one 32-byte record, written by the timeline kernel and read
// as scalars.
typedef int HxMetaRec __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(4))) const HxMetaRec *hx_meta_cp;

struct HxInst {
    int n, m_flag, cap;
    float c1, c2, kB;              // the instance's part of the decode time of a call (hx_decode_terms)
    __device__ __forceinline__ int m() const { return m_flag & (HX_TAB_FLAG - 1); }
    // with the table: a few operations per stretch.  Else few long stretches: search them; many short ones
    // (most entries are starts): the plain scan, straight from memory.
    __device__ __forceinline__ bool by_table() const { return (m_flag & HX_TAB_FLAG) != 0; }
    __device__ __forceinline__ bool by_stretch() const { return !by_table() && 4 * m() <= n; }
};

__device__ __forceinline__ HxInst hx_inst_load(const TlOut &o, int d)
{
    const HxMetaRec r = ((hx_meta_cp)(unsigned long long)o.meta)[d];
    HxInst it;
    it.n = r[0]; it.m_flag = r[1]; it.cap = r[2];
    it.c1 = __int_as_float(r[3]); it.c2 = __int_as_float(r[4]); it.kB = __int_as_float(r[5]);
    return it;
}

// An instance's tables, copied to LDS by the whole workgroup.  With the table: its cells, then the sorted
// occupancies; for the stretch search: the timeline's (time, occupancy) pairs, then the stretch heads.
constexpr int DS_THREADS = 256;
constexpr int DS_OFF_SORTED = HX_TAB, DS_OFF_SEG = 2 * (2 * HX_MAX_INTERVALS + 2);   // words into the staging buffer
constexpr int DS_BUF = HX_TAB + HX_TAB_MAX_N;
static_assert(DS_BUF >= DS_OFF_SEG + HX_MAX_INTERVALS + 2, "the stretch search's arrays fit in the table's place");

// n words from memory to LDS by the whole workgroup, eight loads per thread asked for before the first is
// stored (one memory round trip per 2048 words); from[0] must be readable
__device__ __forceinline__ void hx_copy_words(int *to, const int *__restrict__ from, int n, int tid)
{
    for (int base = 0; base < n; base += 8 * DS_THREADS) {
        int v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = base + u * DS_THREADS + tid;
            v[u] = from[i < n ? i : 0];                    // past the end: the first word again, not stored
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = base + u * DS_THREADS + tid;
            if (i < n) to[i] = v[u];
        }
    }
}

__device__ __forceinline__ void hx_inst_stage(int *buf, const TlOut &o, int d, int nt, const HxInst &it, int tid)
{
    const int n = it.n, m = it.m();
    if (it.by_table()) {
        // the sorted occupancies (at most two per thread) ride with the table's first 2048 cells: one round trip
        const int *G = (const int *)(o.G + (size_t)d * HX_TAB), *sorted = o.sorted + (size_t)d * nt;
        const int cells = m * (n + 1);
        int v[8], s2[2];
#pragma unroll
        for (int u = 0; u < 8; ++u) { const int i = u * DS_THREADS + tid; v[u] = G[i < cells ? i : 0]; }
#pragma unroll
        for (int u = 0; u < 2; ++u) { const int i = u * DS_THREADS + tid; s2[u] = sorted[i < n ? i : 0]; }
#pragma unroll
        for (int u = 0; u < 8; ++u) { const int i = u * DS_THREADS + tid; if (i < cells) buf[i] = v[u]; }
#pragma unroll
        for (int u = 0; u < 2; ++u) { const int i = u * DS_THREADS + tid; if (i < n) buf[DS_OFF_SORTED + i] = s2[u]; }
        if (cells > 8 * DS_THREADS) hx_copy_words(buf + 8 * DS_THREADS, G + 8 * DS_THREADS, cells - 8 * DS_THREADS, tid);
    } else if (it.by_stretch()) {
        hx_copy_words(buf, (const int *)(o.e + (size_t)d * nt), 2 * n, tid);
        hx_copy_words(buf + DS_OFF_SEG, o.seg + (size_t)d * nt, m + 1, tid);
    }
}
static_assert(HX_TAB_MAX_N <= 2 * DS_THREADS, "two sorted occupancies per thread");

// Selection without atomics: a workgroup takes 256 free calls, one per lane, through a group of gd consecutive
// instances, one instance after the other, and every lane keeps the best (finish, instance, start) it has
// seen -- instances ascend, so "strictly smaller" keeps the lowest instance among equal finishes.  The lane's
// result for the group goes to part_*[group][call]; the finish kernel takes the minimum over the groups in
// the same order.  (Asking for an instance's tables while the one before it is searched, into a second
// buffer, was measured and gained nothing: with four workgroups to a compute unit the waits are already
// covered, and the extra address arithmetic costs what the overlap saves.)
//
// The first n_lock workgroups of the grid are for the locked calls instead, one lane per call of the queue
// (lanes of free calls idle): a locked call has its one instance, so each lane reads that instance's
// timeline for itself, and its result is the call's result (group 0's place).
__global__ __launch_bounds__(DS_THREADS) void hx_decode_score_kernel(DecodeArgs a, TlOut o, int nt, int n_lock)
{
    __shared__ __align__(16) int s_buf[DS_BUF];
    int *s_pref = s_buf;                                   // free calls before each slice of the queue: done with before the buffer is filled
    static_assert(DS_BUF >= HX_MAX_INSTANCES + 1, "the slice prefixes fit in the staging buffer");
    __shared__ int s_wave_n[DS_THREADS / HX_WAVE];
    const int tid = threadIdx.x;
    if ((int)blockIdx.x < n_lock) {
        const int c = (int)blockIdx.x * DS_THREADS + tid;
        const bool in = c < a.Q;
        const int L = in ? a.L_in[c] : 0, O = in ? a.L_out[c] : 0;
        const int lk = in ? a.lock[c] : -1;
        const bool ok = L >= 0 && O >= 0 && lk >= -1 && lk < a.D;              // an error is already raised
        const bool legal = in && ok && lk >= 0;
        const int d = legal ? lk : 0;
        const HxDecF x = hx_decode_terms(a.m, a.d_used[d], a.d_batch[d], 0, 1.0f / a.d_flops[d], 1.0f / a.d_hbm[d]);
        const HxDecodeCand k = hx_decode_candidate(a.m, legal ? L : 0, legal ? O : 0, -1, d, a.D, x, a.d_cap[d], a.status);
        const HxSlot s = hx_earliest_start(o.e + (size_t)d * nt, o.n[d], k.thr, k.T, legal);
        const float v = s.S + k.T;
        const bool placed = legal && s.found && v < INFINITY;
        if (in && !(ok && lk < 0)) {                       // locked or invalid: this lane speaks for the call
            a.part_cost[c] = placed ? v : INFINITY;
            a.part_start[c] = placed ? s.S : INFINITY;
            a.part_d[c] = placed ? d : -1;
            if (a.start || a.cost)
                for (int j = 0; j < a.D; ++j) {
                    const bool here = legal && j == d;
                    if (a.start) a.start[(size_t)c * a.D + j] = here ? s.S : INFINITY;
                    if (a.cost) a.cost[(size_t)c * a.D + j] = (here && s.found) ? v : INFINITY;
                }
        }
        return;
    }
    const int b = (int)blockIdx.x - n_lock;
    const int tile = b / a.n_groups, grp = b - tile * a.n_groups;
    const int lane = tid & (HX_WAVE - 1), wave = tid >> 6;
    const int d_lo = grp * a.gd, d_hi = min(a.D, (grp + 1) * a.gd);
    // which call this lane has: position tile*256 + tid of the free calls
    int c = tile * DS_THREADS + tid;
    bool in = c < a.Q;
    if (a.lock) {
        // free calls before each slice: an inclusive scan of the D slice counts, four per thread
        int v[4], sum = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int idx = tid * 4 + j;
            v[j] = idx < a.D ? a.n_free[idx] : 0;
            sum += v[j];
        }
        int incl = sum;
#pragma unroll
        for (int off = 1; off < HX_WAVE; off <<= 1) {
            const int up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        if (lane == HX_WAVE - 1) s_wave_n[wave] = incl;
        __syncthreads();
        int run = incl - sum;
        for (int w2 = 0; w2 < wave; ++w2) run += s_wave_n[w2];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int idx = tid * 4 + j;
            if (idx < a.D) s_pref[idx] = run;
            run += v[j];
            if (idx == a.D - 1) s_pref[a.D] = run;
        }
        __syncthreads();
        const int n_all = s_pref[a.D];
        const int p = tile * DS_THREADS + tid;
        if (tile * DS_THREADS >= n_all) return;            // the whole workgroup: the grid is sized for a queue without locks
        in = p < n_all;
        // the last slice that begins at or before position p
        int lo = 0, hi = a.D - 1;
        while (__builtin_amdgcn_ballot_w64(lo < hi) != 0) {
            const int mid = (lo + hi + 1) >> 1;
            const bool le = s_pref[mid] <= p;
            if (lo < hi) { if (le) lo = mid; else hi = mid - 1; }
        }
        c = in ? a.free_c[lo * a.per + (p - s_pref[lo])] : 0;
    } else if (tile * DS_THREADS >= a.Q) {
        return;
    }
    const bool has = in;                                   // a call of its own: writes a result, if only "none"
    int L = in ? a.L_in[c] : 0, O = in ? a.L_out[c] : 0;
    if (!a.lock && (L < 0 || O < 0)) { hx_raise(a.status, HX_ERR_INDEX); in = false; }
    if (!in) { L = 0; O = 0; }
    const HxCallF cf = hx_call_terms(a.m, L, O);
    const long long need = (long long)L + (long long)O;
    float best_v = INFINITY, best_S = INFINITY;
    int best_d = -1;
    HxInst cur = hx_inst_load(o, d_lo);
    for (int d = d_lo; d < d_hi; ++d) {
        const int *buf = s_buf;
        __syncthreads();                                   // the slice prefixes, or the last instance's tables, are done with
        hx_inst_stage(s_buf, o, d, nt, cur, tid);
        // (scalars, on their way while the tables land: the first heads of this instance, the next instance's record)
        const HxTlGroup heads = *(hx_tl_group_cp)(unsigned long long)(o.head + (size_t)d * nt);
        const HxInst nxt = hx_inst_load(o, min(d + 1, d_hi - 1));
        __syncthreads();
        const float T = hx_decode_time(cf, cur.c1, cur.c2, cur.kB);
        const long long room = (long long)cur.cap - need;
        const int thr = room < 0 ? -1 : (room > (long long)INT_MAX ? INT_MAX : (int)room);
        const int n = cur.n, m = cur.m();
        const float S = cur.by_table()     ? hx_earliest_start_table(o.head + (size_t)d * nt, heads, (const float *)buf, buf + DS_OFF_SORTED,
                                                                     n, m, thr, T, in)
                        : cur.by_stretch() ? hx_earliest_start_stretches((const int2 *)buf, buf + DS_OFF_SEG, n, m, thr, T, in)
                                           : hx_earliest_start_shared(o.e + (size_t)d * nt, n, thr, T, in);
        const float v = S + T;                             // +inf when there is no start
        if (in) {
            if (a.start) a.start[(size_t)c * a.D + d] = S;
            if (a.cost) a.cost[(size_t)c * a.D + d] = S < INFINITY ? v : INFINITY;
            if (S < INFINITY && v < best_v) { best_v = v; best_S = S; best_d = d; }
        }
        cur = nxt;
    }
    if (has) {
        const size_t at = (size_t)grp * a.Q + c;
        a.part_cost[at] = best_v; a.part_start[at] = best_S; a.part_d[at] = best_d;
    }
}

struct DecodeFinishArgs {
    int Q, D, n_groups;
    const int32_t *L_in, *L_out, *lock;
    const float *part_cost, *part_start;
    const int32_t *part_d;
    const int32_t *node, *wf;
    const float *elapsed, *tail, *horizon;
    int n_nodes, n_wf;
    int32_t *best_d;
    float *best_start, *best_cost, *ratio;
    int32_t *status;
};

// the best of the groups' candidates (one place only for a call that is not free); n_groups = 0: there are no instances
__global__ __launch_bounds__(64) void hx_decode_finish_kernel(DecodeFinishArgs a)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= a.Q) return;
    int d = -1;
    float S = INFINITY, v = INFINITY;
    const int lk = a.lock ? a.lock[c] : -1;
    const bool is_free = a.L_in[c] >= 0 && a.L_out[c] >= 0 && lk == -1;
    const int groups = is_free ? a.n_groups : min(a.n_groups, 1);
    // groups ascend in instance: "strictly smaller" keeps the lowest instance among equal finishes
    int g_best = -1;
    int g = 0;
    for (; g + 8 <= groups; g += 8) {
        float pv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) pv[u] = a.part_cost[(size_t)(g + u) * a.Q + c];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (pv[u] < v) { v = pv[u]; g_best = g + u; }
    }
    for (; g < groups; ++g) {
        const float pv = a.part_cost[(size_t)g * a.Q + c];
        if (pv < v) { v = pv; g_best = g; }
    }
    if (g_best >= 0) {
        S = a.part_start[(size_t)g_best * a.Q + c];
        d = a.part_d[(size_t)g_best * a.Q + c];
    }
    a.best_d[c] = d; a.best_start[c] = S; a.best_cost[c] = v;
    if (a.ratio)
        hx_projected_ratio(a.node, a.wf, a.elapsed, a.tail, a.horizon, a.n_nodes, a.n_wf, c, v, a.status, a.ratio);
}

// ---- recomputing greedy of the decode stage, one workgroup -----------------------------

constexpr int DG_THREADS = 1024;
constexpr int DG_WAVES = DG_THREADS / HX_WAVE;

struct DGreedyArgs {
    HxModelF m;
    int Q, D, stride;
    const int32_t *L_in, *L_out, *lock, *node, *wf;
    const float *elapsed, *tail, *horizon;
    int n_nodes, n_wf;
    const float *d_flops, *d_hbm;
    const int32_t *d_used, *d_cap, *d_batch;
    int32_t *iv_count;
    float *iv_start, *iv_end;
    int32_t *iv_tok;
    int32_t *best_d, *rank;
    float *best_start, *best_cost, *ratio;
    int32_t *status;
};

// LDS carve-up shared by host (size) and device (offsets)
struct DGreedyLds {
    int ne, nt, D, Q;      // events per instance, stored timeline length, padded sizes
    __host__ __device__ DGreedyLds(int stride, int D_, int Q_)
        : ne(2 * stride + 1), nt(hx_tl_len(2 * stride + 1) + 2), D((D_ + 3) & ~3), Q((Q_ + 3) & ~3) {}
    // + 2: the lanes of a wavefront scan different timelines with 16-byte reads; with a timeline length of
    // 4k + 2 entries neighbouring timelines start 16 bytes apart modulo the banks instead of on the same ones
    __host__ __device__ size_t off_tl() const { return hx_scratch_bytes(ne); }
    __host__ __device__ size_t off_inst() const { return off_tl() + hx_align16((size_t)D * nt * 8); }
    __host__ __device__ size_t off_call() const { return off_inst() + (size_t)6 * D * 4; }
    __host__ __device__ size_t off_red() const { return off_call() + (size_t)11 * Q * 4; }
    __host__ __device__ size_t off_mat() const { return hx_align16(off_red() + (size_t)(2 * DG_WAVES + 8) * 4); }
    __host__ __device__ size_t bytes() const { return off_mat(); }
    // with the start of every (instance, call) pair kept: [D][Q] floats more
    __host__ __device__ size_t bytes_with_matrix() const { return off_mat() + (size_t)D * Q * 4; }
};

enum : int { DG_ALIVE = 1, DG_DIRTY = 2 };

// An added interval can only delay starts on the instance that received it; everything else stands.
// keep_all (when LDS has room for the start of every (instance, call) pair): after a step only that
// instance's column is computed again, one call per lane, all lanes on the same timeline; a call whose best
// was there takes the minimum of its row again (start + the call's decode time on the instance, the sum its
// finish was when the pair was scored); the start of the call that is picked is read from its row.  Otherwise: a call is scored again, on every instance, if its instance is the one that changed.
// Both ways give the same plan: the same functions on the same timelines, the same (finish, instance) rule.
__global__ __launch_bounds__(DG_THREADS) void hx_decode_plan_kernel(DGreedyArgs a, int keep_all)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const DGreedyLds lay(a.stride, a.D, a.Q);
    TlScratch w = hx_carve_scratch(smem, lay.ne);
    int2 *s_tl = (int2 *)(smem + lay.off_tl());
    int *s_n = (int *)(smem + lay.off_inst());
    int *s_cnt = s_n + lay.D;
    int *s_cap = s_cnt + lay.D;
    float *s_c1 = (float *)(s_cap + lay.D);
    float *s_c2 = s_c1 + lay.D;
    float *s_kB = s_c2 + lay.D;
    int *s_bd = (int *)(smem + lay.off_call());
    float *s_bs = (float *)(s_bd + lay.Q);
    float *s_bc = s_bs + lay.Q;
    float *s_ratio = s_bc + lay.Q;
    int *s_flags = (int *)(s_ratio + lay.Q);
    int *s_L = s_flags + lay.Q;                            // what the queue says of a call, read once
    int *s_O = s_L + lay.Q;
    int *s_lk = s_O + lay.Q;
    float *s_el = (float *)(s_lk + lay.Q);
    float *s_tail = s_el + lay.Q;                          // tail of its node, horizon of its workflow (-1: index out of range)
    float *s_hz = s_tail + lay.Q;
    float *s_redv = (float *)(smem + lay.off_red());
    int *s_redi = (int *)(s_redv + DG_WAVES);
    int *s_pick = s_redi + DG_WAVES;
    float *s_mat = (float *)(smem + lay.off_mat());       // [lay.D][lay.Q] start of call c on instance d, +inf: none (keep_all)

    const int tid = threadIdx.x;
    const int lane = tid & (HX_WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    for (int d = tid; d < a.D; d += DG_THREADS) {
        int cnt = a.iv_count[d];
        if (cnt < 0 || cnt > a.stride) { hx_raise(a.status, HX_ERR_INDEX); cnt = cnt < 0 ? 0 : a.stride; }
        s_cnt[d] = cnt;
        s_cap[d] = a.d_cap[d];
        const HxDecF x = hx_decode_terms(a.m, a.d_used[d], a.d_batch[d], 0, 1.0f / a.d_flops[d], 1.0f / a.d_hbm[d]);
        s_c1[d] = x.c1; s_c2[d] = x.c2; s_kB[d] = x.kB;
    }
    for (int c = tid; c < a.Q; c += DG_THREADS) {
        s_flags[c] = DG_ALIVE | DG_DIRTY;
        s_L[c] = a.L_in[c]; s_O[c] = a.L_out[c]; s_lk[c] = a.lock ? a.lock[c] : -1; s_el[c] = a.elapsed[c];
        const int nd = a.node[c], w = a.wf[c];
        const bool ok = nd >= 0 && nd < a.n_nodes && w >= 0 && w < a.n_wf;
        if (!ok) hx_raise(a.status, HX_ERR_INDEX);
        s_tail[c] = ok ? a.tail[nd] : 0.0f;
        s_hz[c] = ok ? fmaxf(a.horizon[w], 0.0f) : -1.0f;
    }
    __syncthreads();
    for (int d = 0; d < a.D; ++d) {
        const size_t at = (size_t)d * a.stride;
        Tl tl{s_tl + (size_t)d * lay.nt};
        hx_build_timeline<false>(s_cnt[d], a.iv_start + at, a.iv_end + at, a.iv_tok + at, w, tl, &s_n[d], a.status);
    }

    for (int k = 0; k < a.Q; ++k) {
        // (1) score the calls whose instance changed (keep_all: every call, once): one wavefront per call, lanes over instances
        for (int c = wave; c < a.Q && (!keep_all || k == 0); c += DG_WAVES) {
            if (s_flags[c] != (DG_ALIVE | DG_DIRTY)) continue;     // wave-uniform
            const int L = s_L[c], O = s_O[c];
            const int lk = s_lk[c];
            float bv = INFINITY, bS = INFINITY;
            int bd = INT_MAX;
            for (int d0 = 0; d0 < a.D; d0 += HX_WAVE) {
                const int d = d0 + lane;
                const bool in = d < a.D;
                const int dd = in ? d : 0;
                HxDecF x;
                x.wait = 0.0f; x.c1 = s_c1[dd]; x.c2 = s_c2[dd]; x.kB = s_kB[dd];
                const HxDecodeCand q = hx_decode_candidate(a.m, L, O, lk, dd, a.D, x, s_cap[dd], a.status);
                const HxSlot s = hx_earliest_start(s_tl + (size_t)dd * lay.nt, s_n[dd],
                                                   q.thr, q.T, in && q.legal);
                const float v = s.S + q.T;
                if (keep_all && in) s_mat[(size_t)d * lay.Q + c] = s.found ? s.S : INFINITY;
                if (in && s.found && v < bv) { bv = v; bS = s.S; bd = d; }
            }
            const float best = hx_wave_min(bv);
            const int best_d = hx_wave_min(bv == best && best < INFINITY ? bd : INT_MAX);
            const float best_S = __shfl(bS, best_d == INT_MAX ? 0 : (best_d & (HX_WAVE - 1)));
            if (lane == 0) {
                const bool any = best_d != INT_MAX;
                s_bd[c] = any ? best_d : -1;
                s_bs[c] = any ? best_S : INFINITY;
                s_bc[c] = any ? best : INFINITY;
                hx_store_bits(s_ratio, c, hx_ratio_bits(s_el[c], any ? best : INFINITY, s_tail[c], s_hz[c], s_hz[c] >= 0.0f));   // Eq. (2)
                s_flags[c] = DG_ALIVE;
            }
        }
        __syncthreads();
        // (2) the most urgent remaining call: largest ratio, lowest index among equals
        float rv = -INFINITY;
        int ri = INT_MAX;
        for (int c = tid; c < a.Q; c += DG_THREADS) {
            if (s_flags[c] & DG_ALIVE) {
                const float r = hx_rank_key(s_ratio[c]);
                if (ri == INT_MAX || r > rv) { rv = r; ri = c; }
            }
        }
        hx_wave_argmax(rv, ri);
        if (lane == 0) { s_redv[wave] = rv; s_redi[wave] = ri; }
        __syncthreads();
        // (3) the first wavefront takes the best of the wavefronts' candidates (one per lane, the same rule), and its
        // first lane records the pick and appends its interval
        if (wave == 0) {
            rv = lane < DG_WAVES ? s_redv[lane] : -INFINITY;
            ri = lane < DG_WAVES ? s_redi[lane] : INT_MAX;
            hx_wave_argmax(rv, ri);
        }
        if (tid == 0) {
            const int c = ri, d = s_bd[c];
            // its best may have moved since its start was last written: the start on the instance it has now
            if (keep_all && d >= 0) s_bs[c] = s_mat[(size_t)d * lay.Q + c];
            a.best_d[c] = d; a.best_start[c] = s_bs[c]; a.best_cost[c] = s_bc[c]; hx_store_bits(a.ratio, c, __float_as_uint(s_ratio[c])); a.rank[c] = k;
            s_flags[c] = 0;
            int changed = -1;
            if (d >= 0) {
                if (s_cnt[d] >= a.stride) {
                    hx_raise(a.status, HX_ERR_CAPACITY);
                } else {
                    const size_t at = (size_t)d * a.stride + s_cnt[d];
                    const long long need = (long long)s_L[c] + (long long)s_O[c];
                    a.iv_start[at] = s_bs[c];
                    a.iv_end[at] = s_bc[c];
                    a.iv_tok[at] = need > (long long)INT_MAX ? INT_MAX : (int)need;
                    s_cnt[d] += 1;
                    changed = d;
                    // The usual case -- the interval holds something, starts now or later, ends at a finite time, and
                    // the timeline has at most one entry per thread -- is inserted into the timeline below;
                    // anything else has the timeline built again from the instance's intervals.
                    const float S = s_bs[c], E = s_bc[c];
                    s_pick[1] = (S >= 0.0f && S < E && E < INFINITY && need > 0 && s_n[d] <= DG_THREADS) ? 1 : 0;
                    if (!s_pick[1]) __threadfence();                 // the other threads are about to read the interval from memory
                    s_pick[2] = s_n[d]; s_pick[3] = s_n[d];          // entries before S, before E: all, unless an entry says otherwise
                    s_pick[4] = __float_as_int(S > 0.0f ? S : 0.0f); s_pick[5] = __float_as_int(E);
                    s_pick[6] = need > (long long)INT_MAX ? INT_MAX : (int)need;
                }
            }
            s_pick[0] = changed;
        }
        __syncthreads();
        // (4) the timeline of the instance that took the call, and who has to look again
        const int pd = s_pick[0];
        if (pd >= 0) {
            const size_t at = (size_t)pd * a.stride;
            Tl tl{s_tl + (size_t)pd * lay.nt};
            if (s_pick[1]) {
                // The compact timeline is a function of the instance's events, so adding the two events of the new
                // interval (S, E, tok) to it gives what building it again would: entries from S up to E hold tok
                // more; S and E become entries of their own unless the timeline already has an entry at that time
                // (S: the occupancy before it plus tok; E: the occupancy that stood before E).
                const int n = s_n[pd];
                const float S = __int_as_float(s_pick[4]), E = __int_as_float(s_pick[5]);
                const int tok = s_pick[6];
                const bool in = tid < n;
                const int2 me = in ? tl.e[tid] : make_int2(0x7f800000, 0);
                const float t = __int_as_float(me.x);
                const float before = (in && tid > 0) ? __int_as_float(tl.e[tid - 1].x) : -1.0f;
                if (in && t >= S && before < S) s_pick[2] = tid;
                if (in && t >= E && before < E) s_pick[3] = tid;
                __syncthreads();
                const int pos_s = s_pick[2], pos_e = s_pick[3];                   // pos_e >= 1: entry 0 is now, and E > 0
                const bool has_s = pos_s < n && __int_as_float(tl.e[pos_s].x) == S;
                const bool has_e = pos_e < n && __int_as_float(tl.e[pos_e].x) == E;
                const int occ_before_s = tl.e[pos_s > 0 ? pos_s - 1 : 0].y, occ_before_e = tl.e[pos_e - 1].y;
                const int old_len = hx_tl_len(2 * s_cnt[pd] - 1), new_len = hx_tl_len(2 * s_cnt[pd] + 1);
                __syncthreads();                                                  // every old entry has been read
                const int n_new = n + (has_s ? 0 : 1) + (has_e ? 0 : 1);
                if (in) {
                    const int at_new = tid + ((!has_s && tid >= pos_s) ? 1 : 0) + ((!has_e && tid >= pos_e) ? 1 : 0);
                    long long occ = me.y;
                    if (tid >= pos_s && tid < pos_e) occ += tok;
                    if (occ > (long long)INT_MAX) { hx_raise(a.status, HX_ERR_OVERFLOW); occ = INT_MAX; }
                    tl.e[at_new] = make_int2(me.x, (int)occ);
                }
                if (tid == 0 && !has_s) {
                    long long occ = (long long)occ_before_s + tok;
                    if (occ > (long long)INT_MAX) { hx_raise(a.status, HX_ERR_OVERFLOW); occ = INT_MAX; }
                    tl.e[pos_s] = make_int2(s_pick[4], (int)occ);
                }
                if (tid == HX_WAVE && !has_e) {
                    const int at_e = pos_e + (has_s ? 0 : 1);
                    tl.e[at_e] = make_int2(s_pick[5], occ_before_e);
                }
                // the filler behind the entries reaches as far as a timeline of two more events may be read
                for (int i = old_len + tid; i < new_len; i += DG_THREADS)
                    if (i >= n_new) tl.e[i] = make_int2(0x7f800000, 0);
                if (tid == 2 * HX_WAVE) s_n[pd] = n_new;
                __syncthreads();
            } else {
                hx_build_timeline<true>(s_cnt[pd], a.iv_start + at, a.iv_end + at, a.iv_tok + at, w, tl, &s_n[pd], a.status);
            }
            if (!keep_all) {
                for (int c = tid; c < a.Q; c += DG_THREADS)
                    if ((s_flags[c] & DG_ALIVE) && s_bd[c] == pd) s_flags[c] = DG_ALIVE | DG_DIRTY;
            } else {
                HxDecF x;
                x.wait = 0.0f; x.c1 = s_c1[pd]; x.c2 = s_c2[pd]; x.kB = s_kB[pd];
                const int cap = s_cap[pd], n = s_n[pd];
                for (int base = 0; base < a.Q; base += DG_THREADS) {
                    const int c = base + tid;
                    const bool live = c < a.Q && (s_flags[c] & DG_ALIVE);
                    const int L = live ? s_L[c] : 0, O = live ? s_O[c] : 0;
                    const int lk = live ? s_lk[c] : -1;
                    const HxDecodeCand q = hx_decode_candidate(a.m, L, O, live ? lk : -1, pd, a.D, x, cap, a.status);
                    const HxSlot s = hx_earliest_start(tl.e, n, q.thr, q.T, live && q.legal);
                    if (live) {
                        s_mat[(size_t)pd * lay.Q + c] = s.found ? s.S : INFINITY;
                        if (s_bd[c] == pd) {
                            // lowest instance among equal finishes: ascending, strictly smaller (the finish is the kept
                            // start plus the call's decode time there, the same sum as when the pair was scored)
                            const HxCallF cf = hx_call_terms(a.m, L, O);
                            float bv = INFINITY;
                            int bd = -1;
                            int d = 0;
                            for (; d + 8 <= a.D; d += 8) {                    // eight instances' reads in flight
                                float S8[8], c1[8], c2[8], kB[8];
#pragma unroll
                                for (int u = 0; u < 8; ++u) {
                                    S8[u] = s_mat[(size_t)(d + u) * lay.Q + c];
                                    c1[u] = s_c1[d + u]; c2[u] = s_c2[d + u]; kB[u] = s_kB[d + u];
                                }
#pragma unroll
                                for (int u = 0; u < 8; ++u) {
                                    const float v = S8[u] + hx_decode_time(cf, c1[u], c2[u], kB[u]);
                                    if (v < bv) { bv = v; bd = d + u; }
                                }
                            }
                            for (; d < a.D; ++d) {
                                const float v = s_mat[(size_t)d * lay.Q + c] + hx_decode_time(cf, s_c1[d], s_c2[d], s_kB[d]);
                                if (v < bv) { bv = v; bd = d; }
                            }
                            s_bd[c] = bd;
                            s_bc[c] = bv;
                            hx_store_bits(s_ratio, c, hx_ratio_bits(s_el[c], bv, s_tail[c], s_hz[c], s_hz[c] >= 0.0f));   // Eq. (2)
                        }
                    }
                }
            }
        }
        __syncthreads();
    }
    for (int d = tid; d < a.D; d += DG_THREADS) a.iv_count[d] = s_cnt[d];
}

__global__ __launch_bounds__(256) void hx_decode_no_instance_kernel(DGreedyArgs a)
{
    // no decode instance at all: nothing is feasible, every call has infinite ratio and is ranked by index
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= a.Q) return;
    a.best_d[c] = -1; a.best_start[c] = INFINITY; a.best_cost[c] = INFINITY; a.rank[c] = c;
    hx_projected_ratio(a.node, a.wf, a.elapsed, a.tail, a.horizon, a.n_nodes, a.n_wf, c, INFINITY, a.status, a.ratio);
}

HxModelF to_model(const hx_model *m)
{
    return HxModelF{m->kv_bytes_per_token, m->flops_per_token, m->attn_flops_per_token2, m->weight_bytes, m->nominal_batch};
}

int check_tables(hx_ctx *ctx, const hx_calls *q, const hx_decode_tab *dec, const hx_intervals *iv)
{
    HX_REQUIRE(ctx, q->n >= 0 && dec->n >= 0, HX_ERR_INVALID_ARG, "negative size");
    HX_REQUIRE(ctx, dec->n <= HX_MAX_INSTANCES, HX_ERR_SHAPE, "%d decode instances, at most %d", dec->n, HX_MAX_INSTANCES);
    HX_REQUIRE(ctx, iv->stride >= 0 && iv->stride <= HX_MAX_INTERVALS, HX_ERR_SHAPE,
               "interval stride %d outside 0..%d", iv->stride, HX_MAX_INTERVALS);
    HX_REQUIRE(ctx, q->n == 0 || (q->L_in && q->L_out), HX_ERR_INVALID_ARG, "NULL call lengths");
    HX_REQUIRE(ctx, dec->n == 0 || (dec->flops && dec->hbm_bw && dec->used_tok && dec->cap_tok && dec->batch && iv->count),
               HX_ERR_INVALID_ARG, "NULL decode table or interval count");
    HX_REQUIRE(ctx, dec->n == 0 || iv->stride == 0 || (iv->start && iv->end && iv->tok), HX_ERR_INVALID_ARG, "NULL interval array");
    return HX_OK;
}

}  // namespace

// the decode planner may use all of a CU's LDS; said once per process
int hx_decode_init()
{
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(hx_decode_plan_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    return e == hipSuccess ? HX_OK : HX_ERR_DEVICE;
}

extern "C" int hx_decode_score(hx_ctx *ctx, const hx_model *model, const hx_calls *queue, const int32_t *lock,
                               const hx_decode_tab *dec, const hx_intervals *iv,
                               const float *tail, const float *horizon, int32_t n_nodes, int32_t n_wf,
                               float *start, float *cost,
                               int32_t *best_d, float *best_start, float *best_cost, float *ratio, void *stream_)
{
    if (!ctx) return HX_ERR_INVALID_ARG;
    HX_REQUIRE(ctx, model && queue && dec && iv, HX_ERR_INVALID_ARG, "NULL table");
    if (int rc = check_tables(ctx, queue, dec, iv)) return rc;
    const int Q = queue->n, D = dec->n;
    HX_REQUIRE(ctx, Q == 0 || (best_d && best_start && best_cost), HX_ERR_INVALID_ARG, "NULL output");
    HX_REQUIRE(ctx, !ratio || Q == 0 || (queue->node && queue->wf && queue->elapsed && tail && horizon), HX_ERR_INVALID_ARG,
               "a ratio needs node, wf, elapsed, tail and horizon");
    HX_REQUIRE(ctx, n_nodes >= 0 && n_wf >= 0, HX_ERR_INVALID_ARG, "negative n_nodes or n_wf");
    if (Q == 0) return HX_OK;
    HxDeviceGuard guard(ctx->device);
    HX_REQUIRE(ctx, guard.ok, HX_ERR_DEVICE, "cannot select device %d", ctx->device);
    hipStream_t stream = (hipStream_t)stream_;
    const int ne = 2 * iv->stride + 1, nt = hx_tl_len(ne);
    // Groups of instances: enough workgroups (tiles of 256 calls x groups) to fill the chip several times over,
    // at most 64 groups (the finish kernel reads one partial result per group and call).
    const int tiles = (Q + DS_THREADS - 1) / DS_THREADS;
    int n_groups = 0, gd = 1;
    if (D > 0) {
        n_groups = (8 * ctx->num_cu + tiles - 1) / tiles;
        if (n_groups > 64) n_groups = 64;
        if (n_groups > D) n_groups = D;
        gd = (D + n_groups - 1) / n_groups;
        n_groups = (D + gd - 1) / gd;
    }
    const int per = D > 0 ? (Q + D - 1) / D : Q;
    // words of scratch per pass: the free list (D slices of `per` places) and three partial results per group and call
    const size_t part_need = (size_t)(D > 0 ? D : 1) * per + 3 * (size_t)(n_groups > 0 ? n_groups : 1) * Q;
    const size_t tl_need = (size_t)(D > 0 ? D : 1) * nt;
    if (part_need > ctx->dpart_cap || tl_need > ctx->dtl_cap || D > ctx->dtab_cap) {
        // grown, never shrunk; work queued on the old blocks has to finish before they go
        HX_HIP(ctx, hipDeviceSynchronize());
        if (part_need > ctx->dpart_cap) {
            if (ctx->d_dpart) { HX_HIP(ctx, hipFree(ctx->d_dpart)); ctx->d_dpart = nullptr; ctx->dpart_cap = 0; }
            const size_t want = part_need < 65536 ? 65536 : part_need;
            HX_HIP(ctx, hipMalloc((void **)&ctx->d_dpart, want * sizeof(int32_t)));
            ctx->dpart_cap = want;
        }
        if (tl_need > ctx->dtl_cap) {
            if (ctx->d_dtl) { HX_HIP(ctx, hipFree(ctx->d_dtl)); ctx->d_dtl = nullptr; ctx->dtl_cap = 0; }
            // per entry: (time, occupancy) and (head time, head rank) 8 bytes each, sorted occupancy and stretch head 4
            // each, source 2; per instance two counts and a record of eight words
            HX_HIP(ctx, hipMalloc((void **)&ctx->d_dtl, tl_need * 24 + (2 + 8) * (size_t)HX_MAX_INSTANCES * sizeof(int) + 64));
            ctx->dtl_cap = tl_need;
        }
        if (D > ctx->dtab_cap) {
            if (ctx->d_dtab) { HX_HIP(ctx, hipFree(ctx->d_dtab)); ctx->d_dtab = nullptr; ctx->dtab_cap = 0; }
            const int want = D < 64 ? 64 : D;
            HX_HIP(ctx, hipMalloc((void **)&ctx->d_dtab, (size_t)want * HX_TAB * sizeof(float)));
            ctx->dtab_cap = want;
        }
    }
    TlOut o{};
    int32_t *n_free = nullptr;
    {
        unsigned char *p = (unsigned char *)ctx->d_dtl;
        const size_t cap = ctx->dtl_cap;                      // a multiple of 8: every block below stays 16-byte aligned
        o.e = (int2 *)p;        p += cap * 8;
        o.head = (int2 *)p;     p += cap * 8;
        o.n = (int *)p;         p += (size_t)HX_MAX_INSTANCES * sizeof(int);
        n_free = (int32_t *)p;  p += (size_t)HX_MAX_INSTANCES * sizeof(int);
        o.meta = (int *)p;      p += 8 * (size_t)HX_MAX_INSTANCES * sizeof(int);
        o.sorted = (int *)p;    p += cap * 4;
        o.seg = (int *)p;       p += cap * 4;
        o.G = ctx->d_dtab;
    }
    int32_t *free_c = ctx->d_dpart;
    float *part_cost = (float *)(ctx->d_dpart + (size_t)(D > 0 ? D : 1) * per);
    float *part_start = part_cost + (size_t)(n_groups > 0 ? n_groups : 1) * Q;
    int32_t *part_d = (int32_t *)(part_start + (size_t)(n_groups > 0 ? n_groups : 1) * Q);
    if (D > 0) {
        DecodeArgs a{};
        a.m = to_model(model); a.Q = Q; a.D = D; a.stride = iv->stride;
        a.L_in = queue->L_in; a.L_out = queue->L_out; a.lock = lock;
        a.d_flops = dec->flops; a.d_hbm = dec->hbm_bw; a.d_used = dec->used_tok; a.d_cap = dec->cap_tok; a.d_batch = dec->batch;
        a.iv_count = iv->count; a.iv_start = iv->start; a.iv_end = iv->end; a.iv_tok = iv->tok;
        a.start = start; a.cost = cost; a.status = ctx->d_status;
        a.free_c = free_c; a.n_free = n_free; a.per = per;
        a.gd = gd; a.n_groups = n_groups; a.part_cost = part_cost; a.part_start = part_start; a.part_d = part_d;
        const size_t lds = hx_scratch_bytes(ne) + hx_align16((size_t)nt * 8);
        hx_decode_timeline_kernel<<<D, TL_THREADS, lds, stream>>>(a, o, nt);
        const int n_lock = lock ? tiles : 0;
        hx_decode_score_kernel<<<n_lock + tiles * n_groups, DS_THREADS, 0, stream>>>(a, o, nt, n_lock);
    }
    DecodeFinishArgs f{};
    f.Q = Q; f.D = D; f.n_groups = n_groups;
    f.L_in = queue->L_in; f.L_out = queue->L_out; f.lock = lock;
    f.part_cost = part_cost; f.part_start = part_start; f.part_d = part_d;
    f.node = queue->node; f.wf = queue->wf; f.elapsed = queue->elapsed; f.tail = tail; f.horizon = horizon;
    f.n_nodes = n_nodes; f.n_wf = n_wf;
    f.best_d = best_d; f.best_start = best_start; f.best_cost = best_cost; f.ratio = ratio; f.status = ctx->d_status;
    hx_decode_finish_kernel<<<(Q + 63) / 64, 64, 0, stream>>>(f);
    return hx_check_launch(ctx, "hx_decode_score kernels");
}

extern "C" int hx_decode_plan_greedy(hx_ctx *ctx, const hx_model *model, const hx_calls *queue, const int32_t *lock,
                                     const hx_decode_tab *dec, const hx_intervals *iv,
                                     const float *tail, const float *horizon, int32_t n_nodes, int32_t n_wf,
                                     int32_t *best_d, float *best_start, float *best_cost, float *ratio, int32_t *rank,
                                     void *stream_)
{
    if (!ctx) return HX_ERR_INVALID_ARG;
    HX_REQUIRE(ctx, model && queue && dec && iv, HX_ERR_INVALID_ARG, "NULL table");
    if (int rc = check_tables(ctx, queue, dec, iv)) return rc;
    const int Q = queue->n, D = dec->n;
    HX_REQUIRE(ctx, Q <= HX_DECODE_GREEDY_MAX_CALLS, HX_ERR_SHAPE, "%d calls beyond the %d the decode planner takes", Q,
               HX_DECODE_GREEDY_MAX_CALLS);
    HX_REQUIRE(ctx, Q == 0 || (best_d && best_start && best_cost && ratio && rank), HX_ERR_INVALID_ARG, "NULL output");
    HX_REQUIRE(ctx, Q == 0 || (queue->node && queue->wf && queue->elapsed && tail && horizon), HX_ERR_INVALID_ARG,
               "the planner needs node, wf, elapsed, tail and horizon");
    HX_REQUIRE(ctx, n_nodes >= 0 && n_wf >= 0, HX_ERR_INVALID_ARG, "negative n_nodes or n_wf");
    if (Q == 0) return HX_OK;
    const DGreedyLds lay(iv->stride, D, Q);
    HX_REQUIRE(ctx, lay.bytes() <= (size_t)160 * 1024, HX_ERR_SHAPE,
               "%d instances x %d entries (+ %d calls) need %zu bytes of local memory, at most %d", D, iv->stride, Q,
               lay.bytes(), 160 * 1024);
    HxDeviceGuard guard(ctx->device);
    HX_REQUIRE(ctx, guard.ok, HX_ERR_DEVICE, "cannot select device %d", ctx->device);
    hipStream_t stream = (hipStream_t)stream_;
    DGreedyArgs a{};
    a.m = to_model(model); a.Q = Q; a.D = D; a.stride = iv->stride;
    a.L_in = queue->L_in; a.L_out = queue->L_out; a.lock = lock; a.node = queue->node; a.wf = queue->wf;
    a.elapsed = queue->elapsed; a.tail = tail; a.horizon = horizon; a.n_nodes = n_nodes; a.n_wf = n_wf;
    a.d_flops = dec->flops; a.d_hbm = dec->hbm_bw; a.d_used = dec->used_tok; a.d_cap = dec->cap_tok; a.d_batch = dec->batch;
    a.iv_count = iv->count; a.iv_start = iv->start; a.iv_end = iv->end; a.iv_tok = iv->tok;
    a.best_d = best_d; a.best_start = best_start; a.best_cost = best_cost; a.ratio = ratio; a.rank = rank;
    a.status = ctx->d_status;
    if (D == 0) {
        hx_decode_no_instance_kernel<<<(Q + 255) / 256, 256, 0, stream>>>(a);
    } else {
        const bool keep_all = lay.bytes_with_matrix() <= (size_t)160 * 1024;
        hx_decode_plan_kernel<<<1, DG_THREADS, keep_all ? lay.bytes_with_matrix() : lay.bytes(), stream>>>(a, keep_all ? 1 : 0);
    }
    return hx_check_launch(ctx, "hx_decode_plan_greedy kernel");
}
