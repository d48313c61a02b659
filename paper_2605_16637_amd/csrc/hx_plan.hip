// The planner around the scoring loop (Algorithm 1 main loop; Sec. 5.3):
// one-pass ordering of the calls by their projected ratio, and the recomputing
// greedy loop for small queues -- pick the most urgent call, give it the pair
// with the earliest projected decode finish, add it to a simulated copy of the
// pool state, score again.
#include "hx_common.hpp"
#include "hx_terms.hpp"
#include "hx_search.hpp"

#include <cmath>

namespace {

constexpr int kT = HX_MAX_TYPES;

// ---- one-pass ordering -----------------------------------------------------------

constexpr int RANK_TILE = 2048;      // calls compared against per block, at most
constexpr int RANK_SMALL = 16384;    // queues up to this size are ranked by all-pairs counting

__global__ __launch_bounds__(256) void hx_rank_zero_kernel(int32_t *rank, int C)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c < C) rank[c] = 0;
}

// (ratio, index) as one unsigned 64-bit key that orders like "larger ratio first,
// then lower index": the float bits made monotone, then the complemented index
__device__ __forceinline__ unsigned long long hx_rank_key64(float r, int idx)
{
    unsigned b = __float_as_uint(hx_rank_key(r));
    b ^= (b & 0x80000000u) ? 0xffffffffu : 0x80000000u;
    return ((unsigned long long)b << 32) | (unsigned)(0xffffffffu - (unsigned)idx);
}

// rank[c] = number of calls ahead of c: larger ratio, or equal ratio and lower
// index.  Block (i, j) counts, for 256 calls, those ahead of them among the
// `tile` calls of tile j; the partial counts are added up with integer atomics.
__global__ __launch_bounds__(256) void hx_rank_count_kernel(const float *ratio, int32_t *rank, int C, int tile)
{
    __shared__ unsigned long long s_key[RANK_TILE];
    const int k0 = blockIdx.y * tile;
    const int kn = min(tile, C - k0);
    for (int i = threadIdx.x; i < kn; i += blockDim.x) s_key[i] = hx_rank_key64(ratio[k0 + i], k0 + i);
    __syncthreads();
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    const unsigned long long mine = hx_rank_key64(ratio[c], c);
    int ahead = 0;
#pragma unroll 8
    for (int i = 0; i < kn; ++i) ahead += s_key[i] > mine;
    if (ahead) atomicAdd(&rank[c], ahead);
}

// Larger queues: sample sort.  256 evenly spaced calls are sorted and serve as splitters; every call
// finds its bucket among them, takes a slot in it, and is moved next to the other members of its
// bucket; a workgroup per bucket then counts, for every member, the larger keys inside the bucket and
// adds the sizes of all higher buckets.  Keys are unique (they end in the call index), so buckets stay
// balanced however many ratios are equal, and the ranks do not depend on the order the slots were
// taken in.
constexpr int RANK_SPLIT = 256;                  // splitters; buckets 0 .. RANK_SPLIT
constexpr int RANK_BUCKETS = RANK_SPLIT + 1;
constexpr int RANK_CHUNK = 2048;                 // bucket members held in LDS at a time

struct RankScratch {
    unsigned long long *split;                   // [RANK_SPLIT] ascending
    unsigned long long *bkey;                    // [C] keys grouped by bucket
    int *hist;                                   // [RANK_BUCKETS] bucket sizes
};

__global__ __launch_bounds__(RANK_SPLIT) void hx_rank_splitters_kernel(const float *ratio, int C, RankScratch w)
{
    __shared__ unsigned long long s[RANK_SPLIT];
    const int t = threadIdx.x;
    const int c = (int)(((long long)t * C) / RANK_SPLIT);
    s[t] = hx_rank_key64(ratio[c], c);
    w.hist[t] = 0;
    if (t == 0) w.hist[RANK_SPLIT] = 0;
    __syncthreads();
    for (int k = 2; k <= RANK_SPLIT; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            const int l = t ^ j;
            const unsigned long long x = s[t], y = s[l];
            __syncthreads();
            // ascending bitonic network: the lower index of a pair keeps the smaller key when (t & k) == 0
            const bool keep_small = ((t & k) == 0) == (t < l);
            s[t] = keep_small ? (x < y ? x : y) : (x < y ? y : x);
            __syncthreads();
        }
    }
    w.split[t] = s[t];
}

// bucket of a key: the number of splitters below it
__device__ __forceinline__ int hx_rank_bucket(const unsigned long long *split, unsigned long long key)
{
    int lo = 0, hi = RANK_SPLIT;                  // first splitter that is not below the key
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (split[mid] < key) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// every call takes a slot in its bucket; the slot is parked in rank[c].  The calls of a workgroup first
// count themselves per bucket in LDS, then the workgroup reserves its share of every bucket with one
// global atomic per non-empty bucket (one atomic per call would queue up on 257 addresses).
__global__ __launch_bounds__(1024) void hx_rank_slot_kernel(const float *ratio, int32_t *rank, int C, RankScratch w)
{
    __shared__ unsigned long long s_split[RANK_SPLIT];
    __shared__ int s_cnt[RANK_BUCKETS], s_base[RANK_BUCKETS];
    const int t = threadIdx.x;
    if (t < RANK_SPLIT) s_split[t] = w.split[t];
    if (t < RANK_BUCKETS) s_cnt[t] = 0;
    __syncthreads();
    const int c = blockIdx.x * blockDim.x + t;
    int b = 0, local = 0;
    if (c < C) {
        b = hx_rank_bucket(s_split, hx_rank_key64(ratio[c], c));
        local = atomicAdd(&s_cnt[b], 1);
    }
    __syncthreads();
    if (t < RANK_BUCKETS && s_cnt[t] > 0) s_base[t] = atomicAdd(&w.hist[t], s_cnt[t]);
    __syncthreads();
    if (c < C) rank[c] = s_base[b] + local;
}

// exclusive prefix of the bucket sizes, by every workgroup for itself (257 values)
__device__ __forceinline__ void hx_rank_starts(const int *hist, int *s_start)
{
    __shared__ int s_part[4];
    const int t = threadIdx.x;                    // the first 256 threads: bucket t (bucket 256 rides with thread 255)
    const int lane = t & (HX_WAVE - 1), wv = t >> 6;
    const int h = t < RANK_SPLIT ? hist[t] : 0;
    int incl = h;
#pragma unroll
    for (int off = 1; off < HX_WAVE; off <<= 1) {
        const int o = __shfl_up(incl, off);
        if (lane >= off) incl += o;
    }
    if (t < RANK_SPLIT && lane == HX_WAVE - 1) s_part[wv] = incl;
    __syncthreads();
    if (t < RANK_SPLIT) {
        int base = 0;
        for (int k = 0; k < wv; ++k) base += s_part[k];
        s_start[t] = base + incl - h;
        if (t == RANK_SPLIT - 1) { s_start[RANK_SPLIT] = base + incl; s_start[RANK_BUCKETS] = base + incl + hist[RANK_SPLIT]; }
    }
    __syncthreads();
}

__global__ __launch_bounds__(256) void hx_rank_scatter_kernel(const float *ratio, const int32_t *rank, int C, RankScratch w)
{
    __shared__ unsigned long long s_split[RANK_SPLIT];
    __shared__ int s_start[RANK_BUCKETS + 1];
    s_split[threadIdx.x] = w.split[threadIdx.x];
    hx_rank_starts(w.hist, s_start);
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    const unsigned long long key = hx_rank_key64(ratio[c], c);
    w.bkey[s_start[hx_rank_bucket(s_split, key)] + rank[c]] = key;
}

// workgroup b: rank of every member of bucket b = keys in higher buckets + larger keys in its own
__global__ __launch_bounds__(1024) void hx_rank_within_kernel(int32_t *rank, int C, RankScratch w)
{
    __shared__ unsigned long long s_key[RANK_CHUNK];
    __shared__ int s_start[RANK_BUCKETS + 1];
    hx_rank_starts(w.hist, s_start);
    const int b = blockIdx.x;
    const int m0 = s_start[b], m1 = s_start[b + 1];
    const int higher = C - m1;
    // members in rounds of one per thread, each compared with the whole bucket, which passes through LDS in chunks
    for (int base = m0; base < m1; base += blockDim.x) {                   // same trip count for all threads
        const int i = base + threadIdx.x;
        const unsigned long long mine = i < m1 ? w.bkey[i] : ~0ull;
        int ahead = 0;
        for (int k0 = m0; k0 < m1; k0 += RANK_CHUNK) {
            const int kn = min(RANK_CHUNK, m1 - k0);
            __syncthreads();
            for (int k = threadIdx.x; k < kn; k += blockDim.x) s_key[k] = w.bkey[k0 + k];
            __syncthreads();
            int k = 0;
            for (; k + 8 <= kn; k += 8) {                  // eight independent reads in flight
                unsigned long long kk[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) kk[u] = s_key[k + u];
#pragma unroll
                for (int u = 0; u < 8; ++u) ahead += kk[u] > mine;
            }
            for (; k < kn; ++k) ahead += s_key[k] > mine;
        }
        if (i < m1) rank[0xffffffffu - (unsigned)(mine & 0xffffffffull)] = higher + ahead;
    }
}

// ---- recomputing greedy -------------------------------------------------------------

constexpr int GREEDY_THREADS = 1024;
constexpr int GREEDY_WAVES = GREEDY_THREADS / HX_WAVE;

struct GreedyArgs {
    HxModelF m;
    int C, P, D;
    const int32_t *L_in, *L_out, *node, *wf;
    const float *elapsed, *tail, *horizon;
    int n_nodes, n_wf;
    const HxPrepTables *prep;
    const float *d_flops, *d_hbm;
    const int32_t *p_backlog, *d_used, *d_cap, *d_batch, *d_qd;
    int tokens_per_seq, max_batch;
    int32_t *best_p, *best_d, *rank;
    float *best_cost, *ratio;
    int32_t *backlog_out, *used_out, *batch_out, *qd_out;
    int32_t *status;
};

// LDS carve-up shared by host (size) and device (offsets), in 4-byte words
struct GreedyLds {
    int Dp, Pp, C, P, D;      // lengths of the LDS arrays (not the problem sizes)
    __host__ __device__ GreedyLds(int dp_bound, int P_, int D_, int C_)
        : Dp(dp_bound), Pp((P_ + HX_WAVE - 1) / HX_WAVE * HX_WAVE),
          C((C_ + 3) & ~3), P((P_ + 3) & ~3), D((D_ + 3) & ~3) {}      // array lengths, kept 16-byte aligned
    __host__ __device__ size_t words() const
    {
        return (size_t)7 * Dp + 4 * Pp + 2 * kT * kT + 16     // pool view, as in the fused search
             + P + 7 * (size_t)D                               // simulated state and what is needed to re-derive an entry
             + 11 * (size_t)C                                  // per call: pair, cost, ratio, flags; lengths, elapsed, tail, horizon; the list of calls to score again
             + 4 * GREEDY_WAVES                                // reduction scratch
             + (size_t)GREEDY_WAVES * (Dp + kT * kT + kT);     // per-wave search buffers
    }
};

enum : int { ALIVE = 1, DIRTY = 2 };

// One block plans the whole queue: the pool tables, the simulated state and the
// per-call results live in LDS, there is no launch between iterations.  A call
// is scored again only if its current pair touches an instance a commit just
// changed and the pair's cost moved: while commits only add load they can only
// raise costs, so every other call keeps its pair and cost exactly.  A commit
// that lowers a term of its decode instance (a snapshot batch above the batch
// rule's value) has every remaining call scored again.
template <int KP>
__global__ __launch_bounds__(GREEDY_THREADS) void hx_plan_greedy_kernel(GreedyArgs a, int dp_bound)
{
    extern __shared__ __align__(16) float smem[];
    const HxPrepTables *__restrict__ t = a.prep;
    const int Dp = t->n_entries;
    const GreedyLds lay(dp_bound, a.P, a.D, a.C);
    float *s_wait = smem;
    float *s_c1 = s_wait + lay.Dp;
    float *s_c2 = s_c1 + lay.Dp;
    float *s_kB = s_c2 + lay.Dp;
    int *s_free = (int *)(s_kB + lay.Dp);
    int *s_orig = s_free + lay.Dp;
    int *s_dtype = s_orig + lay.Dp;
    float *s_pw = (float *)(s_dtype + lay.Dp);
    float *s_pinvF = s_pw + lay.Pp;
    float *s_pinvB = s_pinvF + lay.Pp;
    int *s_ptype = (int *)(s_pinvB + lay.Pp);
    float *s_invbw = (float *)(s_ptype + lay.Pp);
    float *s_lat = s_invbw + kT * kT;
    int *s_seg = (int *)(s_lat + kT * kT);
    int *s_backlog = s_seg + 16;                       // simulated state
    int *s_used = s_backlog + lay.P;
    int *s_batch = s_used + lay.D;
    int *s_qd = s_batch + lay.D;
    int *s_cap = s_qd + lay.D;
    int *s_pos = s_cap + lay.D;                        // entry of decode instance d
    float *s_dinvF = (float *)(s_pos + lay.D);
    float *s_dinvB = s_dinvF + lay.D;
    int *s_bp = (int *)(s_dinvB + lay.D);              // per call
    int *s_bd = s_bp + lay.C;
    float *s_bc = (float *)(s_bd + lay.C);
    float *s_ratio = s_bc + lay.C;
    int *s_flags = (int *)(s_ratio + lay.C);
    int *s_L = s_flags + lay.C;                        // what the queue says of a call, read once
    int *s_O = s_L + lay.C;
    float *s_el = (float *)(s_O + lay.C);
    float *s_tl = s_el + lay.C;                        // tail of its node, horizon of its workflow (-1: index out of range)
    float *s_hz = s_tl + lay.C;
    int *s_list = (int *)(s_hz + lay.C);               // the calls to score again, in any order: dealt to the wavefronts evenly
    float *s_redv = (float *)(s_list + lay.C);         // reduction scratch, then the pick
    int *s_redi = (int *)(s_redv + GREEDY_WAVES);
    int *s_pick = s_redi + GREEDY_WAVES;               // [0] call, [1] p, [2] d
    float *s_wave = (float *)(s_pick + 2 * GREEDY_WAVES);

    const int tid = threadIdx.x;
    const int lane = tid & (HX_WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    float *dbuf = s_wave + (size_t)wave * (lay.Dp + kT * kT + kT);
    float *xbuf = dbuf + lay.Dp;
    float *rbuf = xbuf + kT * kT;

    for (int e = tid; e < Dp; e += GREEDY_THREADS) {
        s_wait[e] = t->dec_wait[e]; s_c1[e] = t->dec_c1[e]; s_c2[e] = t->dec_c2[e]; s_kB[e] = t->dec_kB[e];
        s_free[e] = t->dec_free[e]; s_orig[e] = t->dec_orig[e]; s_dtype[e] = t->dec_type[e];
    }
    for (int p = tid; p < lay.Pp; p += GREEDY_THREADS) {
        const bool in = p < a.P;
        s_pw[p] = in ? t->pre_wait[p] : INFINITY;
        s_pinvF[p] = in ? t->pre_invF[p] : 0.0f;
        s_pinvB[p] = in ? t->pre_invB[p] : 0.0f;
        s_ptype[p] = in ? t->pre_type[p] : 0;
        if (in) s_backlog[p] = a.p_backlog[p];
    }
    for (int d = tid; d < a.D; d += GREEDY_THREADS) {
        s_used[d] = a.d_used[d]; s_batch[d] = a.d_batch[d]; s_qd[d] = a.d_qd[d]; s_cap[d] = a.d_cap[d];
        s_pos[d] = t->dec_pos[d];
        s_dinvF[d] = 1.0f / a.d_flops[d]; s_dinvB[d] = 1.0f / a.d_hbm[d];
    }
    if (tid < kT * kT) { s_invbw[tid] = t->link_invbw[tid]; s_lat[tid] = t->link_lat[tid]; }
    if (tid <= kT) s_seg[tid] = t->seg[tid];
    for (int c = tid; c < a.C; c += GREEDY_THREADS) {
        s_flags[c] = ALIVE | DIRTY;
        s_list[c] = c;
        s_L[c] = a.L_in[c]; s_O[c] = a.L_out[c]; s_el[c] = a.elapsed[c];
        const int nd = a.node[c], w = a.wf[c];
        const bool ok = nd >= 0 && nd < a.n_nodes && w >= 0 && w < a.n_wf;
        if (!ok) hx_raise(a.status, HX_ERR_INDEX);
        s_tl[c] = ok ? a.tail[nd] : 0.0f;
        s_hz[c] = ok ? fmaxf(a.horizon[w], 0.0f) : -1.0f;
    }
    __syncthreads();

    int seg[kT + 1];
#pragma unroll
    for (int k = 0; k <= kT; ++k) seg[k] = __builtin_amdgcn_readfirstlane(s_seg[k]);
    const HxPoolLds pool{s_wait, s_c1, s_c2, s_kB, s_free, s_orig, s_dtype, s_pw, s_pinvF, s_pinvB, s_ptype,
                         s_invbw, s_lat, Dp, a.P, lay.Pp};

    int n_dirty = a.C;                                 // every call at first (uniform; s_pick[4] carries it from step to step)
    for (int k = 0; k < a.C; ++k) {
        // (1) score the calls whose pair may have changed, on the simulated state: the list deals them to the
        // wavefronts evenly (by call index, a wavefront could find all of its calls dirty and its neighbour none)
        for (int i = wave; i < n_dirty; i += GREEDY_WAVES) {
            const int c = s_list[i];
            if (s_flags[c] != (ALIVE | DIRTY)) continue;           // wave-uniform: c depends on the wave only
            // large pools: class by class (KP = 0); small ones: pair by pair, whose inner loop costs less than the
            // class search's reductions up to about 64 x 64 pairs
            HxBest b;
            if constexpr (KP == 0) b = hx_search_call_by_class(a.m, pool, dbuf, xbuf, rbuf, s_L[c], s_O[c], lane);
            else b = hx_search_call<KP>(a.m, pool, seg, dbuf, xbuf, s_L[c], s_O[c], lane);
            if (lane == 0) {
                s_bp[c] = b.p; s_bd[c] = b.d; s_bc[c] = b.cost;
                hx_store_bits(s_ratio, c, hx_ratio_bits(s_el[c], b.cost, s_tl[c], s_hz[c], s_hz[c] >= 0.0f));       // Eq. (2)
                s_flags[c] = ALIVE;
            }
        }
        __syncthreads();
        // (2) the most urgent remaining call: largest ratio, lowest index among equals
        float bv = -INFINITY;
        int bi = 0x7fffffff;
        for (int c = tid; c < a.C; c += GREEDY_THREADS) {
            if (s_flags[c] & ALIVE) {
                const float r = hx_rank_key(s_ratio[c]);
                if (bi == 0x7fffffff || r > bv) { bv = r; bi = c; }
            }
        }
        hx_wave_argmax(bv, bi);
        if (lane == 0) { s_redv[wave] = bv; s_redi[wave] = bi; }
        __syncthreads();
        // (3) the first two wavefronts take the best of the wavefronts' candidates (one per lane, the same rule); the
        // first lane of one records the pick and adds it to the prefill side of the simulated state, the first lane
        // of the other to the decode side (two chains of dependent LDS reads side by side)
        if (wave < 2) {
            bv = lane < GREEDY_WAVES ? s_redv[lane] : -INFINITY;
            bi = lane < GREEDY_WAVES ? s_redi[lane] : 0x7fffffff;
            hx_wave_argmax(bv, bi);
        }
        if (tid == 0) {
            const int c = bi, p = s_bp[c], d = s_bd[c];
            a.best_p[c] = p; a.best_d[c] = d; a.best_cost[c] = s_bc[c]; hx_store_bits(a.ratio, c, __float_as_uint(s_ratio[c])); a.rank[c] = k;
            s_flags[c] = 0;
            s_pick[0] = c; s_pick[1] = p; s_pick[2] = d;
            s_pick[4] = 0;                                  // the next step's list starts empty
            if (p >= 0) {
                const int L = s_L[c];
                long long bl = (long long)s_backlog[p] + L;
                if (L < 0 || s_O[c] < 0) bl = s_backlog[p];            // raised by the other lane
                if (bl > 2147483647LL) { hx_raise(a.status, HX_ERR_OVERFLOW); bl = 2147483647LL; }
                s_backlog[p] = (int)bl;
                // the derived table entry of the prefill instance, by the function the per-round prepare uses
                s_pw[p] = hx_prefill_wait(a.m, s_backlog[p], s_pinvF[p]);
            }
        }
        if (tid == HX_WAVE) {
            const int c = bi, p = s_bp[c], d = s_bd[c];
            s_pick[3] = 0;
            if (p >= 0) {
                const int L = s_L[c], O = s_O[c];
                long long qd = (long long)s_qd[d] + O, us = (long long)s_used[d] + L + O;
                if (L < 0 || O < 0) { hx_raise(a.status, HX_ERR_INDEX); qd = s_qd[d]; us = s_used[d]; }
                if (qd > 2147483647LL || us > 2147483647LL) {
                    hx_raise(a.status, HX_ERR_OVERFLOW);
                    qd = min(qd, 2147483647LL); us = min(us, 2147483647LL);
                }
                s_qd[d] = (int)qd; s_used[d] = (int)us;
                // us >= 0 and tokens_per_seq are below 2^31, their sum fits 32 unsigned bits: no 64-bit division
                const long long nb = us >= 0 ? (long long)(((unsigned)us + (unsigned)a.tokens_per_seq - 1u) / (unsigned)a.tokens_per_seq)
                                             : (us + a.tokens_per_seq - 1) / a.tokens_per_seq;
                s_batch[d] = (int)(nb > a.max_batch ? a.max_batch : nb);
                // the derived table entry of the decode instance, by the function the per-round prepare uses
                const HxDecF x = hx_decode_terms(a.m, s_used[d], s_batch[d], s_qd[d], s_dinvF[d], s_dinvB[d]);
                const int e = s_pos[d];
                const long long fr = (long long)s_cap[d] - us;
                const int nfree = fr < -1 ? -1 : (int)fr;
                // A commit normally only adds load.  It lowers a term when the snapshot's batch stood above what
                // the batch rule gives for the new occupancy (the caller's batch is only required to be >= 0):
                // then pairs on d get cheaper and any call may prefer d now.
                s_pick[3] = (x.wait < s_wait[e] || x.c1 < s_c1[e] || x.c2 < s_c2[e] || nfree > s_free[e]) ? 1 : 0;
                s_wait[e] = x.wait; s_c1[e] = x.c1; s_c2[e] = x.c2; s_kB[e] = x.kB;
                s_free[e] = nfree;
            }
        }
        __syncthreads();
        // (4) which calls are scored again
        const int pp = s_pick[1], pd = s_pick[2];
        if (pp >= 0 && s_pick[3]) {
            // a term of the decode instance fell: nothing can be kept
            for (int c = tid; c < a.C; c += GREEDY_THREADS)
                if (s_flags[c] & ALIVE) { s_flags[c] = ALIVE | DIRTY; s_list[atomicAdd(&s_pick[4], 1)] = c; }
        } else if (pp >= 0) {
            // load was only added: every pair costs what it did or more, so only calls whose pair touches one of
            // the two instances can lose their minimum -- and not even those if the cost of their pair came out
            // the same (e.g. the decode instance's availability still dominates a longer prefill queue)
            for (int c = tid; c < a.C; c += GREEDY_THREADS)
                if ((s_flags[c] & ALIVE) && (s_bp[c] == pp || s_bd[c] == pd) &&
                    hx_pair_cost(a.m, pool, s_L[c], s_O[c], s_bp[c], s_pos[s_bd[c]]) != s_bc[c]) {
                    s_flags[c] = ALIVE | DIRTY;
                    s_list[atomicAdd(&s_pick[4], 1)] = c;
                }
        }
        __syncthreads();
        n_dirty = s_pick[4];
    }
    // the simulated state the plan leaves
    for (int p = tid; p < a.P; p += GREEDY_THREADS) if (a.backlog_out) a.backlog_out[p] = s_backlog[p];
    for (int d = tid; d < a.D; d += GREEDY_THREADS) {
        if (a.used_out) a.used_out[d] = s_used[d];
        if (a.batch_out) a.batch_out[d] = s_batch[d];
        if (a.qd_out) a.qd_out[d] = s_qd[d];
    }
}

__global__ __launch_bounds__(256) void hx_plan_no_pool_kernel(GreedyArgs a)
{
    // with an empty pool nothing is feasible: every call has infinite ratio and is ranked by index
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= a.C) return;
    a.best_p[c] = -1; a.best_d[c] = -1; a.best_cost[c] = INFINITY; a.rank[c] = c;
    hx_projected_ratio(a.node, a.wf, a.elapsed, a.tail, a.horizon, a.n_nodes, a.n_wf, c, INFINITY, a.status, a.ratio);
}

__global__ __launch_bounds__(256) void hx_copy_i32_kernel(const int32_t *src, int32_t *dst, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

}  // namespace

// the planner kernel may use all of a CU's LDS; said once per process
int hx_plan_init()
{
    const int lds = 160 * 1024;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(hx_plan_greedy_kernel<0>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(hx_plan_greedy_kernel<1>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(hx_plan_greedy_kernel<2>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(hx_plan_greedy_kernel<4>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    return e == hipSuccess ? HX_OK : HX_ERR_DEVICE;
}

extern "C" int hx_rank(hx_ctx *ctx, int32_t C, const float *ratio, int32_t *rank, void *stream_)
{
    if (!ctx) return HX_ERR_INVALID_ARG;
    HX_REQUIRE(ctx, C >= 0, HX_ERR_INVALID_ARG, "negative size");
    HX_REQUIRE(ctx, C == 0 || (ratio && rank), HX_ERR_INVALID_ARG, "NULL array");
    if (C == 0) return HX_OK;
    HxDeviceGuard guard(ctx->device);
    HX_REQUIRE(ctx, guard.ok, HX_ERR_DEVICE, "cannot select device %d", ctx->device);
    hipStream_t stream = (hipStream_t)stream_;
    const int bx = (C + 255) / 256;
    if (C <= RANK_SMALL) {
        // small queues: every call against every call, no scratch.  Tiles short enough for a few thousand
        // workgroups (a workgroup's time is its tile's length, whatever the queue's), long enough to be worth
        // their atomics.
        int tile = (C / 32 + 63) / 64 * 64;
        if (tile < 64) tile = 64;
        if (tile > RANK_TILE) tile = RANK_TILE;
        const int by = (C + tile - 1) / tile;
        hx_rank_zero_kernel<<<bx, 256, 0, stream>>>(rank, C);
        hx_rank_count_kernel<<<dim3(bx, by), 256, 0, stream>>>(ratio, rank, C, tile);
        return hx_check_launch(ctx, "hx_rank kernels");
    }
    const size_t need = (size_t)C + RANK_SPLIT + (RANK_BUCKETS + 1) / 2 + 8;      // keys, splitters, bucket sizes (two ints per word)
    if (need > ctx->rkey_cap) {
        // grown, never shrunk; work queued on the old block has to finish before it goes
        HX_HIP(ctx, hipDeviceSynchronize());
        if (ctx->d_rkey) { HX_HIP(ctx, hipFree(ctx->d_rkey)); ctx->d_rkey = nullptr; ctx->rkey_cap = 0; }
        HX_HIP(ctx, hipMalloc((void **)&ctx->d_rkey, need * sizeof(unsigned long long)));
        ctx->rkey_cap = need;
    }
    RankScratch w;
    w.split = ctx->d_rkey;
    w.bkey = ctx->d_rkey + RANK_SPLIT;
    w.hist = (int *)(ctx->d_rkey + RANK_SPLIT + C);
    hx_rank_splitters_kernel<<<1, RANK_SPLIT, 0, stream>>>(ratio, C, w);
    hx_rank_slot_kernel<<<(C + 1023) / 1024, 1024, 0, stream>>>(ratio, rank, C, w);
    hx_rank_scatter_kernel<<<bx, 256, 0, stream>>>(ratio, rank, C, w);
    hx_rank_within_kernel<<<RANK_BUCKETS, 1024, 0, stream>>>(rank, C, w);
    return hx_check_launch(ctx, "hx_rank kernels");
}

extern "C" int hx_plan_greedy(hx_ctx *ctx, const hx_model *model, const hx_calls *calls,
                              const hx_prefill_tab *pre, const hx_decode_tab *dec, const hx_links *links,
                              const float *tail, const float *horizon, int32_t n_nodes, int32_t n_wf,
                              int32_t tokens_per_seq, int32_t max_batch,
                              int32_t *best_p, int32_t *best_d, float *best_cost, float *ratio, int32_t *rank,
                              int32_t *backlog_tok_out, int32_t *used_tok_out, int32_t *batch_out, int32_t *qd_tok_out,
                              void *stream_)
{
    if (!ctx) return HX_ERR_INVALID_ARG;
    HX_REQUIRE(ctx, model && calls && pre && dec && links, HX_ERR_INVALID_ARG, "NULL table");
    const int C = calls->n, P = pre->n, D = dec->n, T = links->n_types;
    HX_REQUIRE(ctx, C >= 0, HX_ERR_INVALID_ARG, "negative size");
    HX_REQUIRE(ctx, C <= HX_GREEDY_MAX_CALLS, HX_ERR_SHAPE, "%d calls beyond the %d the recomputing planner takes", C,
               HX_GREEDY_MAX_CALLS);
    HX_REQUIRE(ctx, P <= HX_GREEDY_MAX_INSTANCES && D <= HX_GREEDY_MAX_INSTANCES, HX_ERR_SHAPE,
               "pool %d x %d beyond the %d instances per side the recomputing planner takes", P, D, HX_GREEDY_MAX_INSTANCES);
    HX_REQUIRE(ctx, tokens_per_seq > 0 && max_batch >= 0, HX_ERR_INVALID_ARG, "tokens_per_seq must be positive");
    HX_REQUIRE(ctx, best_p && best_d && best_cost && ratio && rank, HX_ERR_INVALID_ARG, "NULL output");
    HX_REQUIRE(ctx, C == 0 || (calls->L_in && calls->L_out && calls->node && calls->wf && calls->elapsed && tail && horizon),
               HX_ERR_INVALID_ARG, "the planner needs L_in, L_out, node, wf, elapsed, tail and horizon");
    HX_REQUIRE(ctx, n_nodes >= 0 && n_wf >= 0, HX_ERR_INVALID_ARG, "negative n_nodes or n_wf");
    HxDeviceGuard guard(ctx->device);
    HX_REQUIRE(ctx, guard.ok, HX_ERR_DEVICE, "cannot select device %d", ctx->device);
    hipStream_t stream = (hipStream_t)stream_;

    GreedyArgs a{};
    a.m = HxModelF{model->kv_bytes_per_token, model->flops_per_token, model->attn_flops_per_token2,
                   model->weight_bytes, model->nominal_batch};
    a.C = C; a.P = P; a.D = D;
    a.L_in = calls->L_in; a.L_out = calls->L_out; a.node = calls->node; a.wf = calls->wf; a.elapsed = calls->elapsed;
    a.tail = tail; a.horizon = horizon; a.n_nodes = n_nodes; a.n_wf = n_wf;
    a.prep = ctx->d_prep; a.d_flops = dec->flops; a.d_hbm = dec->hbm_bw;
    a.p_backlog = pre->backlog_tok; a.d_used = dec->used_tok; a.d_cap = dec->cap_tok; a.d_batch = dec->batch; a.d_qd = dec->qd_tok;
    a.tokens_per_seq = tokens_per_seq; a.max_batch = max_batch;
    a.best_p = best_p; a.best_d = best_d; a.rank = rank; a.best_cost = best_cost; a.ratio = ratio;
    a.backlog_out = backlog_tok_out; a.used_out = used_tok_out; a.batch_out = batch_out; a.qd_out = qd_tok_out;
    a.status = ctx->d_status;

    if (P == 0 || D == 0) {
        // an empty side: nothing is feasible, the state is returned unchanged
        if (P) HX_REQUIRE(ctx, pre->backlog_tok, HX_ERR_INVALID_ARG, "NULL member in prefill table");
        if (D) HX_REQUIRE(ctx, dec->used_tok && dec->batch && dec->qd_tok, HX_ERR_INVALID_ARG, "NULL member in decode table");
        if (C) hx_plan_no_pool_kernel<<<(C + 255) / 256, 256, 0, stream>>>(a);
        if (P && backlog_tok_out) hx_copy_i32_kernel<<<(P + 255) / 256, 256, 0, stream>>>(pre->backlog_tok, backlog_tok_out, P);
        if (D && used_tok_out) hx_copy_i32_kernel<<<(D + 255) / 256, 256, 0, stream>>>(dec->used_tok, used_tok_out, D);
        if (D && batch_out) hx_copy_i32_kernel<<<(D + 255) / 256, 256, 0, stream>>>(dec->batch, batch_out, D);
        if (D && qd_tok_out) hx_copy_i32_kernel<<<(D + 255) / 256, 256, 0, stream>>>(dec->qd_tok, qd_tok_out, D);
        return hx_check_launch(ctx, "hx_plan_no_pool_kernel");
    }
    if (int rc = hx_prepare_pool(ctx, model, pre, dec, links, stream)) return rc;
    const int dp_bound = (D + HX_DGROUP - 1) / HX_DGROUP * HX_DGROUP + (T - 1) * HX_DGROUP;
    const GreedyLds lay(dp_bound, P, D, C);
    const size_t lds = 4 * lay.words();
    HX_REQUIRE(ctx, lds <= 160 * 1024, HX_ERR_SHAPE, "queue and pool need %zu B of LDS", lds);
    if ((long long)P * D > 64 * 64) hx_plan_greedy_kernel<0><<<1, GREEDY_THREADS, lds, stream>>>(a, dp_bound);
    else if (P <= 64) hx_plan_greedy_kernel<1><<<1, GREEDY_THREADS, lds, stream>>>(a, dp_bound);
    else if (P <= 128) hx_plan_greedy_kernel<2><<<1, GREEDY_THREADS, lds, stream>>>(a, dp_bound);
    else hx_plan_greedy_kernel<4><<<1, GREEDY_THREADS, lds, stream>>>(a, dp_bound);
    return hx_check_launch(ctx, "hx_plan_greedy_kernel");
}
