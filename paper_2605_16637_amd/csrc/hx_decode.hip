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
    short *su, *ss;  // unsorted / sorted: 1 + index of the interval that ends here, 0 = now
};

// compact timeline: entry i covers [t_i, t_{i+1}) (the last one has no end) with occupancy occ_i
struct Tl {
    int2 *e;         // (time bits, occupancy)
    short *src;      // which interval's end t_i is (1 + index), 0 = now
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
    w.ds = (int *)p;                  p += hx_align16((size_t)ne * 4);
    w.su = (short *)p;                p += hx_align16((size_t)ne * 2);
    w.ss = (short *)p;
    return w;
}
__host__ __device__ inline size_t hx_scratch_bytes(int ne)
{
    return hx_align16((size_t)ne * 8) + 3 * hx_align16((size_t)ne * 4) + 2 * hx_align16((size_t)ne * 2);
}

template <bool COHERENT, typename T> __device__ __forceinline__ T hx_ld(const T *p)
{
    // COHERENT: the value may have been written by another wave of this workgroup a moment ago
    if (COHERENT) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return *p;
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
        int delta = 0, src = 0;
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
                src = (is_end && e > 0.0f) ? j + 1 : 0;
            }
        }
        // at equal times starts sort before ends, so the last event of a time is an end if there is one
        w.key[i] = ((u64)__float_as_uint(time) << 32) | ((u64)is_end << 31) | (unsigned)i;
        w.delta[i] = delta;
        w.su[i] = (short)src;
    }
    __syncthreads();
    // position of every event = number of smaller keys (keys are unique)
    for (int i = tid; i < n_ev; i += nthreads) {
        const u64 ki = w.key[i];
        int r = 0;
        int j = 0;
        for (; j + 8 <= n_ev; j += 8) {                   // eight independent reads in flight
            u64 kk[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) kk[u] = w.key[j + u];
#pragma unroll
            for (int u = 0; u < 8; ++u) r += kk[u] < ki;
        }
        for (; j < n_ev; ++j) r += w.key[j] < ki;
        w.ts[r] = __uint_as_float((unsigned)(ki >> 32));
        w.ds[r] = w.delta[i];
        w.ss[r] = w.su[i];
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
                out.src[pos] = w.ss[i];
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
    int src;     // 1 + index of the interval whose end S is, 0 = now, -1 if none
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
__device__ __forceinline__ HxSlot hx_earliest_start(const int2 *e, const short *src, int n, int thr, float T, bool active)
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
    HxSlot r{INFINITY, -1};
    if (open && ans < INFINITY) {
        // which entry the start is: times are strictly increasing, so a bisection finds it
        int lo = 0, hi = n - 1;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (__int_as_float(e[mid].x) < ans) lo = mid + 1; else hi = mid;
        }
        r.S = ans;
        r.src = src[lo];
    }
    return r;
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
    u64 *key;
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

// selection key: lexicographic minimum of (cost, instance); the start rides along as the interval it is the end of
__device__ __forceinline__ u64 hx_decode_key(float cost, int d, int src)
{
    return ((u64)__float_as_uint(cost) << 32) | ((u64)(unsigned)d << 16) | (unsigned)src;
}

__global__ __launch_bounds__(256) void hx_decode_key_init_kernel(u64 *key, int Q)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c < Q) key[c] = ~0ull;
}

// Workgroup d: the timeline of instance d, built in LDS and written to the library's scratch
// (nt entries per instance, padded); the workgroups also set the selection keys to "nothing yet".
__global__ __launch_bounds__(256) void hx_decode_timeline_kernel(DecodeArgs a, int2 *tl_e, short *tl_src, int *tl_n, int nt)
{
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int s_n;
    const int tid = threadIdx.x;
    const int d = blockIdx.x;
    const int ne = 2 * a.stride + 1;
    TlScratch w = hx_carve_scratch(smem, ne);
    Tl tl;
    tl.e = (int2 *)(smem + hx_scratch_bytes(ne));
    tl.src = (short *)(smem + hx_scratch_bytes(ne) + hx_align16((size_t)hx_tl_len(ne) * 8));
    int cnt = a.iv_count[d];
    if (cnt < 0 || cnt > a.stride) {
        if (tid == 0) hx_raise(a.status, HX_ERR_INDEX);
        cnt = cnt < 0 ? 0 : a.stride;
    }
    const size_t at = (size_t)d * a.stride;
    hx_build_timeline<false>(cnt, a.iv_start + at, a.iv_end + at, a.iv_tok + at, w, tl, &s_n, a.status);
    const int n = s_n;
    for (int i = tid; i < hx_tl_len(2 * cnt + 1); i += blockDim.x) tl_e[(size_t)d * nt + i] = tl.e[i];
    for (int i = tid; i < n; i += blockDim.x) tl_src[(size_t)d * ne + i] = tl.src[i];
    if (tid == 0) tl_n[d] = n;
    const int per = (a.Q + a.D - 1) / a.D;
    for (int c = d * per + tid; c < min(a.Q, (d + 1) * per); c += blockDim.x) a.key[c] = ~0ull;
}

// The same scan as hx_earliest_start for a timeline every lane of the wavefront shares.  The
// timeline was written by an earlier kernel and nothing writes it now, so it is read through the
// constant address space: with wave-uniform addresses the entries arrive as scalars, cost no vector
// memory or LDS traffic, and feed the vector arithmetic as scalar operands.  Eight entries per
// step, the next eight already on their way.
typedef int HxTlGroup __attribute__((ext_vector_type(16)));      // eight (time, occupancy) entries
typedef __attribute__((address_space(4))) const HxTlGroup *hx_tl_group_cp;

__device__ __forceinline__ HxSlot hx_earliest_start_shared(const int2 *__restrict__ e, const float *lds_t, const short *lds_src,
                                                           int n, int thr, float T, bool active)
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
    HxSlot r{INFINITY, -1};
    if (open && ans < INFINITY) {
        // which entry the start is: times are strictly increasing, a bisection over the copy in LDS finds it
        int lo = 0, hi = n - 1;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (lds_t[mid] < ans) lo = mid + 1; else hi = mid;
        }
        r.S = ans;
        r.src = lds_src[lo];
    }
    return r;
}

// Workgroup (d, part): calls part*chunk .. of the queue against instance d.  The calls that may
// go to d (free ones and those locked to d) are first gathered in LDS, so that the scan runs with
// full wavefronts however many calls are locked elsewhere; then one call per lane.
constexpr int DS_CHUNK = 1024;        // calls per workgroup at most

__global__ __launch_bounds__(256) void hx_decode_score_kernel(DecodeArgs a, const int2 *__restrict__ tl_e,
                                                              const short *__restrict__ tl_src, const int *__restrict__ tl_n,
                                                              int nt, int splits, int chunk)
{
    __shared__ int s_c[DS_CHUNK], s_L[DS_CHUNK], s_O[DS_CHUNK];
    __shared__ float s_t[2 * HX_MAX_INTERVALS + 2];        // the timeline's times and sources, for the bisection
    __shared__ short s_src[2 * HX_MAX_INTERVALS + 2];
    __shared__ int s_count;
    const int tid = threadIdx.x;
    const int lane = tid & (HX_WAVE - 1);
    const int d = blockIdx.x / splits, part = blockIdx.x - d * splits;
    const int ne = 2 * a.stride + 1;
    const int2 *__restrict__ e = tl_e + (size_t)d * nt;
    const short *__restrict__ src = tl_src + (size_t)d * ne;
    const int n = tl_n[d];
    const float invF = 1.0f / a.d_flops[d], invB = 1.0f / a.d_hbm[d];
    const HxDecF x = hx_decode_terms(a.m, a.d_used[d], a.d_batch[d], 0, invF, invB);
    const int cap = a.d_cap[d];
    const int c_lo = part * chunk, c_hi = min(a.Q, c_lo + chunk);
    if (tid == 0) s_count = 0;
    for (int i = tid; i < n; i += blockDim.x) { s_t[i] = __int_as_float(e[i].x); s_src[i] = src[i]; }
    __syncthreads();
    for (int base = c_lo; base < c_hi; base += blockDim.x) {
        const int c = base + tid;
        const bool in = c < c_hi;
        const int L = in ? a.L_in[c] : 0, O = in ? a.L_out[c] : 0;
        const int lk = (in && a.lock) ? a.lock[c] : -1;
        const bool ok = L >= 0 && O >= 0 && lk >= -1 && lk < a.D;
        if (!ok) hx_raise(a.status, HX_ERR_INDEX);
        const bool legal = in && ok && (lk < 0 || lk == d);
        const unsigned long long m = __builtin_amdgcn_ballot_w64(legal);
        int at = 0;
        if (lane == 0 && m) at = atomicAdd(&s_count, __popcll(m));
        at = __builtin_amdgcn_readfirstlane(at) + __popcll(m & ((1ull << lane) - 1ull));
        if (legal) { s_c[at] = c; s_L[at] = L; s_O[at] = O; }
        if (in && !legal) {
            if (a.start) a.start[(size_t)c * a.D + d] = INFINITY;
            if (a.cost) a.cost[(size_t)c * a.D + d] = INFINITY;
        }
    }
    __syncthreads();
    const int n_legal = s_count;
    for (int base = 0; base < n_legal; base += blockDim.x) {
        const int i = base + tid;
        const bool in = i < n_legal;
        const int c = in ? s_c[i] : 0, L = in ? s_L[i] : 0, O = in ? s_O[i] : 0;
        const HxDecodeCand k = hx_decode_candidate(a.m, L, O, -1, d, a.D, x, cap, a.status);
        const HxSlot s = hx_earliest_start_shared(e, s_t, s_src, n, k.thr, k.T, in);
        const float v = s.S + k.T;                         // +inf when there is no start
        if (in) {
            if (a.start) a.start[(size_t)c * a.D + d] = s.S;
            if (a.cost) a.cost[(size_t)c * a.D + d] = s.src >= 0 ? v : INFINITY;
            if (s.src >= 0 && v < INFINITY) {
                // read first: most candidates do not improve on what other instances have already written
                const u64 mine = hx_decode_key(v, d, s.src);
                if (__hip_atomic_load(&a.key[c], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) > mine) atomicMin(&a.key[c], mine);
            }
        }
    }
}

struct DecodeFinishArgs {
    int Q, D, stride;
    const u64 *key;
    const float *iv_end;
    const int32_t *node, *wf;
    const float *elapsed, *tail, *horizon;
    int n_nodes, n_wf;
    int32_t *best_d;
    float *best_start, *best_cost, *ratio;
    int32_t *status;
};

__global__ __launch_bounds__(256) void hx_decode_finish_kernel(DecodeFinishArgs a)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= a.Q) return;
    const u64 k = a.key[c];
    int d = -1;
    float S = INFINITY, v = INFINITY;
    if (k != ~0ull) {
        d = (int)((k >> 16) & 0xffffu);
        const int src = (int)(k & 0xffffu);
        v = __uint_as_float((unsigned)(k >> 32));
        S = src == 0 ? 0.0f : a.iv_end[(size_t)d * a.stride + (src - 1)];
    }
    a.best_d[c] = d; a.best_start[c] = S; a.best_cost[c] = v;
    if (a.ratio)
        a.ratio[c] = hx_projected_ratio(a.node, a.wf, a.elapsed, a.tail, a.horizon, a.n_nodes, a.n_wf, c, v, a.status);
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
    __host__ __device__ size_t off_src() const { return off_tl() + hx_align16((size_t)D * nt * 8); }
    __host__ __device__ size_t off_inst() const { return off_src() + hx_align16((size_t)D * ne * 2); }
    __host__ __device__ size_t off_call() const { return off_inst() + (size_t)6 * D * 4; }
    __host__ __device__ size_t off_red() const { return off_call() + (size_t)5 * Q * 4; }
    __host__ __device__ size_t bytes() const { return off_red() + (size_t)(2 * DG_WAVES + 8) * 4; }
};

enum : int { DG_ALIVE = 1, DG_DIRTY = 2 };

// A call is scored again only if its instance is the one that just received an interval:
// an added interval can only delay starts on that instance, every other call keeps its result.
__global__ __launch_bounds__(DG_THREADS) void hx_decode_plan_kernel(DGreedyArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const DGreedyLds lay(a.stride, a.D, a.Q);
    TlScratch w = hx_carve_scratch(smem, lay.ne);
    int2 *s_tl = (int2 *)(smem + lay.off_tl());
    short *s_src = (short *)(smem + lay.off_src());
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
    float *s_redv = (float *)(smem + lay.off_red());
    int *s_redi = (int *)(s_redv + DG_WAVES);
    int *s_pick = s_redi + DG_WAVES;

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
    for (int c = tid; c < a.Q; c += DG_THREADS) s_flags[c] = DG_ALIVE | DG_DIRTY;
    __syncthreads();
    for (int d = 0; d < a.D; ++d) {
        const size_t at = (size_t)d * a.stride;
        Tl tl{s_tl + (size_t)d * lay.nt, s_src + (size_t)d * lay.ne};
        hx_build_timeline<false>(s_cnt[d], a.iv_start + at, a.iv_end + at, a.iv_tok + at, w, tl, &s_n[d], a.status);
    }

    for (int k = 0; k < a.Q; ++k) {
        // (1) score the calls whose instance changed: one wavefront per call, lanes over instances
        for (int c = wave; c < a.Q; c += DG_WAVES) {
            if (s_flags[c] != (DG_ALIVE | DG_DIRTY)) continue;     // wave-uniform
            const int L = a.L_in[c], O = a.L_out[c];
            const int lk = a.lock ? a.lock[c] : -1;
            float bv = INFINITY, bS = INFINITY;
            int bd = INT_MAX;
            for (int d0 = 0; d0 < a.D; d0 += HX_WAVE) {
                const int d = d0 + lane;
                const bool in = d < a.D;
                const int dd = in ? d : 0;
                HxDecF x;
                x.wait = 0.0f; x.c1 = s_c1[dd]; x.c2 = s_c2[dd]; x.kB = s_kB[dd];
                const HxDecodeCand q = hx_decode_candidate(a.m, L, O, lk, dd, a.D, x, s_cap[dd], a.status);
                const HxSlot s = hx_earliest_start(s_tl + (size_t)dd * lay.nt, s_src + (size_t)dd * lay.ne, s_n[dd],
                                                   q.thr, q.T, in && q.legal);
                const float v = s.S + q.T;
                if (in && s.src >= 0 && v < bv) { bv = v; bS = s.S; bd = d; }
            }
            const float best = hx_wave_min(bv);
            const int best_d = hx_wave_min(bv == best && best < INFINITY ? bd : INT_MAX);
            const float best_S = __shfl(bS, best_d == INT_MAX ? 0 : (best_d & (HX_WAVE - 1)));
            if (lane == 0) {
                const bool any = best_d != INT_MAX;
                s_bd[c] = any ? best_d : -1;
                s_bs[c] = any ? best_S : INFINITY;
                s_bc[c] = any ? best : INFINITY;
                s_ratio[c] = hx_projected_ratio(a.node, a.wf, a.elapsed, a.tail, a.horizon, a.n_nodes, a.n_wf, c,
                                                any ? best : INFINITY, a.status);
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
#pragma unroll
        for (int off = HX_WAVE / 2; off > 0; off >>= 1) {
            const float ov = __shfl_xor(rv, off);
            const int oi = __shfl_xor(ri, off);
            const bool take = oi != INT_MAX && (ri == INT_MAX || ov > rv || (ov == rv && oi < ri));
            rv = take ? ov : rv;
            ri = take ? oi : ri;
        }
        if (lane == 0) { s_redv[wave] = rv; s_redi[wave] = ri; }
        __syncthreads();
        // (3) one thread records the pick and appends its interval
        if (tid == 0) {
            for (int wv = 1; wv < DG_WAVES; ++wv) {
                const float ov = s_redv[wv];
                const int oi = s_redi[wv];
                if (oi != INT_MAX && (ri == INT_MAX || ov > rv || (ov == rv && oi < ri))) { rv = ov; ri = oi; }
            }
            const int c = ri, d = s_bd[c];
            a.best_d[c] = d; a.best_start[c] = s_bs[c]; a.best_cost[c] = s_bc[c]; a.ratio[c] = s_ratio[c]; a.rank[c] = k;
            s_flags[c] = 0;
            int changed = -1;
            if (d >= 0) {
                if (s_cnt[d] >= a.stride) {
                    hx_raise(a.status, HX_ERR_CAPACITY);
                } else {
                    const size_t at = (size_t)d * a.stride + s_cnt[d];
                    const long long need = (long long)a.L_in[c] + (long long)a.L_out[c];
                    a.iv_start[at] = s_bs[c];
                    a.iv_end[at] = s_bc[c];
                    a.iv_tok[at] = need > (long long)INT_MAX ? INT_MAX : (int)need;
                    s_cnt[d] += 1;
                    changed = d;
                    __threadfence();
                }
            }
            s_pick[0] = changed;
        }
        __syncthreads();
        // (4) the timeline of the instance that took the call, and who has to look again
        const int pd = s_pick[0];
        if (pd >= 0) {
            const size_t at = (size_t)pd * a.stride;
            Tl tl{s_tl + (size_t)pd * lay.nt, s_src + (size_t)pd * lay.ne};
            hx_build_timeline<true>(s_cnt[pd], a.iv_start + at, a.iv_end + at, a.iv_tok + at, w, tl, &s_n[pd], a.status);
            for (int c = tid; c < a.Q; c += DG_THREADS)
                if ((s_flags[c] & DG_ALIVE) && s_bd[c] == pd) s_flags[c] = DG_ALIVE | DG_DIRTY;
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
    a.ratio[c] = hx_projected_ratio(a.node, a.wf, a.elapsed, a.tail, a.horizon, a.n_nodes, a.n_wf, c, INFINITY, a.status);
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
    const size_t tl_need = (size_t)(D > 0 ? D : 1) * nt;
    if (Q > ctx->dkey_cap || tl_need > ctx->dtl_cap) {
        // grown, never shrunk; work queued on the old blocks has to finish before they go
        HX_HIP(ctx, hipDeviceSynchronize());
        if (Q > ctx->dkey_cap) {
            if (ctx->d_dkey) { HX_HIP(ctx, hipFree(ctx->d_dkey)); ctx->d_dkey = nullptr; ctx->dkey_cap = 0; }
            const int want = Q < 4096 ? 4096 : Q;
            HX_HIP(ctx, hipMalloc((void **)&ctx->d_dkey, (size_t)want * sizeof(u64)));
            ctx->dkey_cap = want;
        }
        if (tl_need > ctx->dtl_cap) {
            if (ctx->d_dtl) { HX_HIP(ctx, hipFree(ctx->d_dtl)); ctx->d_dtl = nullptr; ctx->dtl_cap = 0; }
            // per entry: (time, occupancy) 8 bytes + source 2 bytes; per instance one length
            HX_HIP(ctx, hipMalloc((void **)&ctx->d_dtl, tl_need * 10 + (size_t)HX_MAX_INSTANCES * sizeof(int) + 64));
            ctx->dtl_cap = tl_need;
        }
    }
    int2 *tl_e = (int2 *)ctx->d_dtl;
    int *tl_n = (int *)((unsigned char *)ctx->d_dtl + ctx->dtl_cap * 8);
    short *tl_src = (short *)((unsigned char *)ctx->d_dtl + ctx->dtl_cap * 8 + (size_t)HX_MAX_INSTANCES * sizeof(int));
    if (D > 0) {
        DecodeArgs a{};
        a.m = to_model(model); a.Q = Q; a.D = D; a.stride = iv->stride;
        a.L_in = queue->L_in; a.L_out = queue->L_out; a.lock = lock;
        a.d_flops = dec->flops; a.d_hbm = dec->hbm_bw; a.d_used = dec->used_tok; a.d_cap = dec->cap_tok; a.d_batch = dec->batch;
        a.iv_count = iv->count; a.iv_start = iv->start; a.iv_end = iv->end; a.iv_tok = iv->tok;
        a.start = start; a.cost = cost; a.key = ctx->d_dkey; a.status = ctx->d_status;
        const size_t lds = hx_scratch_bytes(ne) + hx_align16((size_t)nt * 8) + hx_align16((size_t)ne * 2);
        hx_decode_timeline_kernel<<<D, 256, lds, stream>>>(a, tl_e, tl_src, tl_n, nt);
        // enough workgroups to fill the chip, each with at least one full pass of calls
        int splits = (8 * ctx->num_cu + D - 1) / D;
        const int max_splits = (Q + 255) / 256, min_splits = (Q + DS_CHUNK - 1) / DS_CHUNK;
        if (splits > max_splits) splits = max_splits;
        if (splits < min_splits) splits = min_splits;
        int chunk = (Q + splits - 1) / splits;
        chunk = (chunk + 255) / 256 * 256;                // <= DS_CHUNK, a multiple of 256 itself
        splits = (Q + chunk - 1) / chunk;
        hx_decode_score_kernel<<<D * splits, 256, 0, stream>>>(a, tl_e, tl_src, tl_n, nt, splits, chunk);
    } else {
        hx_decode_key_init_kernel<<<(Q + 255) / 256, 256, 0, stream>>>(ctx->d_dkey, Q);
    }
    DecodeFinishArgs f{};
    f.Q = Q; f.D = D; f.stride = iv->stride; f.key = ctx->d_dkey; f.iv_end = iv->end;
    f.node = queue->node; f.wf = queue->wf; f.elapsed = queue->elapsed; f.tail = tail; f.horizon = horizon;
    f.n_nodes = n_nodes; f.n_wf = n_wf;
    f.best_d = best_d; f.best_start = best_start; f.best_cost = best_cost; f.ratio = ratio; f.status = ctx->d_status;
    hx_decode_finish_kernel<<<(Q + 255) / 256, 256, 0, stream>>>(f);
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
    if (D == 0)
        hx_decode_no_instance_kernel<<<(Q + 255) / 256, 256, 0, stream>>>(a);
    else
        hx_decode_plan_kernel<<<1, DG_THREADS, lay.bytes(), stream>>>(a);
    return hx_check_launch(ctx, "hx_decode_plan_greedy kernel");
}
