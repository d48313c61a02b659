/*
 * hx_oracle.c -- CPU oracle for the per-round placement search of a workflow-
 * and heterogeneity-aware scheduler on a prefill-decode disaggregated pool.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, obviously-correct
 * statement of what the search computes.  It is used by the tests, by the
 * smoke check and by the CPU-baseline leg of the benchmark; nothing on the
 * product path may call it.  It shares no code, header, table or constant
 * with the GPU implementation.
 *
 * Arithmetic: every latency term is evaluated in fp64 directly from its
 * definition, once per (call, prefill, decode) candidate, with no hoisting,
 * blocking or reordering.  Feasibility, levels and state updates are int32.
 * The critical-path pass can round every sum to fp32 on request, because
 * the workload definition fixes fp32 for that pass.
 *
 * What the paper fixes and what it leaves open
 * --------------------------------------------
 * The paper gives the structure of the computation:
 *   - Sec. 4.2 "Scheduler internals": an Estimator turns per-call input and
 *     output length plus instance snapshots into prefill time, decode time,
 *     KV-transfer latency and decode memory demand with a roofline-style
 *     model;
 *   - Sec. 4.2 "Heterogeneous resource modelling": a prefill instance is a
 *     single server with a queue, a decode instance does batched decoding
 *     under a KV-capacity limit, transfer latency is KV size over the
 *     effective bandwidth between the two GPU classes;
 *   - Sec. 5.1, Eq. (2): projected ratio R = ((t - a_w) + Delta) / H_w(t);
 *   - Sec. 5.1 (online workflow horizon): H_w(t) is the completion time of
 *     the revealed sub-DAG when nothing else runs on the cluster;
 *   - Sec. 5.3: enumerate candidate prefill x decode instances, estimate the
 *     prefill finish, add transfer latency, project the earliest decode
 *     finish from decode availability hints, choose the pair with the
 *     earliest projected decode finish;
 *   - Sec. 5.4, Eq. (3),(4): demand m(c) = L_in + L_out_hat, feasible on d
 *     only if m(c) <= Cap(d);
 *   - Algorithm 1: per invocation, update horizons, then for every waiting
 *     call project the best feasible placement and compute R.
 * It prints no formula for the estimator.  The readings below fill that gap;
 * they are the literal roofline form (time = max of compute-bound time and
 * bandwidth-bound time) over the four per-class quantities a pool
 * description provides (FLOP/s, memory B/s, KV capacity, NIC B/s).
 *
 *  R1  prefill wait      Wp(p)      = backlog_tok[p] * phi / F_p
 *  R2  prefill service   Tpre(c,p)  = max((phi*L + a*L^2)/F_p,
 *                                         (omega + kappa*L)/B_p)
 *  R3  KV transfer       X(c,p,d)   = kappa*L / bw[tp][td] + lat[tp][td]
 *  R4  decode hint       step(d)    = max(phi*batch_d/F_d,
 *                                         (omega + kappa*used_d)/B_d)
 *                        waitD(d)   = qd_tok[d] * step(d) / Bbar
 *  R5  decode per token  ttok(c,d)  = max(phi*(batch_d+1)/F_d,
 *                              (omega + kappa*(used_d + L + O/2))/B_d)
 *                        Tdec(c,d)  = O * ttok(c,d)
 *  R6  feasibility       used_d + L + O <= cap_d   (tokens, integers);
 *                        Eq. (4) with Cap(d) read as the capacity still
 *                        free; equals Eq. (4) when used_d = 0
 *  R7  candidate cost    Delta      = max(Wp + Tpre + X, waitD) + Tdec,
 *                                     +infinity when infeasible
 *  R8  selection         lexicographic minimum of (Delta, p*D + d);
 *                        no feasible pair -> (-1, -1, +infinity)
 *  R9  standalone cost   cost(v)    = min over class pairs (tp,td) of
 *                        Tpre + X + O*max(phi/F_td,
 *                                  (omega + kappa*(L + O/2))/B_td)
 *                        i.e. R2,R3,R5 on an idle pool
 *  R10 critical path     tail(v) = max(0, max_{u in succ(v)} rem(u)),
 *                        rem(v) = cost(v) + tail(v),
 *                        level(v) = 0 without successors, else
 *                        1 + max level(u);  H(w) = max_{v in w} rem(v)
 *  R11 urgency           R(c) = (elapsed_c + Delta*_c + tail(node_c)) / H(wf_c); +inf where H(wf_c) = 0
 *                        = Eq. (2) whenever the call is a leaf of the
 *                        revealed DAG (tail = 0)
 *  R12 commit and drain  integer bookkeeping of chosen placements, see
 *                        hxo_commit
 *  R13 recomputing greedy (Algorithm 1 main loop; Sec. 5.3, small queues):
 *                        repeat: score every remaining call on the simulated
 *                        state (R7, R8, R11); take the call of largest R,
 *                        equal R by lowest call index; record its pair, cost,
 *                        R and its rank (0 = first); add it to the state
 *                        (backlog[p*] += L, qd[d*] += O, used[d*] += L + O,
 *                        batch[d*] = R12's rule; no drain).  A call with no
 *                        feasible pair has R = +infinity: it is ranked at
 *                        once, keeps (-1,-1) and changes nothing.
 *  R14 one-pass ordering (Sec. 5.3, larger queues): rank = position by
 *                        decreasing R, equal R by increasing call index
 *
 * Decode stage (Sec. 5.4; calls whose KV has arrived and that wait for decode
 * admission).  Times are seconds from now.
 *  R22 token-capacity intervals: decode instance d holds intervals
 *                        j = (s_j, e_j, m_j): m_j tokens of KV occupied on
 *                        s_j <= tau < e_j (resident sequences have s_j <= 0,
 *                        planned ones start later);
 *                        occ_d(tau) = sum of m_j over the intervals holding tau
 *  R23 capacity-feasible start: t is feasible for call c on d when
 *                        occ_d(tau) + m(c) <= cap_d for every tau in
 *                        [t, t + Tdec(c,d)), m(c) = L + O (Eq. 3);
 *                        S(c,d) = the earliest feasible t >= 0.  Occupancy only
 *                        drops where an interval ends, so S is 0 or some e_j.
 *                        m(c) > cap_d (Eq. 4): never feasible, S = +infinity
 *  R24 decode-stage cost Delta_D(c,d) = S(c,d) + Tdec(c,d): waiting for decode
 *                        capacity plus decode execution (Sec. 5.1), Tdec by R5
 *                        on the snapshot (batch_d, used_d)
 *  R25 legal instances   a call locked to d (Sec. 5.4) may only go to d; a free
 *                        call to any instance; best = lexicographic minimum of
 *                        (Delta_D, d); nothing legal and feasible -> (-1, +inf)
 *  R26 decode greedy     (Sec. 5.4, small queues) repeat: score every remaining
 *                        call on the simulated intervals; take the call of
 *                        largest R = (elapsed + Delta_D + tail)/H, equal R by
 *                        lowest index; record instance, start, finish, R, rank;
 *                        append (S, S + Tdec, m(c)) to that instance.  Only the
 *                        intervals are simulated (batch_d, used_d of R5 stay as
 *                        in the snapshot).  A call with nothing feasible is
 *                        ranked at once with (-1, +inf) and changes nothing.
 *                        Larger queues: one scoring pass, then R14.
 *
 * The choice of these formulas cannot be checked against printed values of
 * the paper (it prints none): parity with "the paper's estimator" is
 * unpinned, and so are the tie rules of R8, R13, R14, R25, R26, the
 * commit/drain rule R12 and the interval layout R22.  What the tests pin is
 * that this file computes R1..R14 and R22..R26 as written: round-number
 * cases worked by hand, closed forms, brute force on small inputs, an
 * integer-time simulation of the intervals, monotonicity and scaling
 * invariants, validity of finished plans.
 *
 * L = L_in, O = predicted output length, kappa = KV bytes per token,
 * phi = FLOP per token, a = attention FLOP per token^2, omega = weight
 * bytes, Bbar = nominal decode batch.  Rates are in FLOP/s and B/s.
 */

#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    double kv_bytes_per_token;     /* kappa */
    double flops_per_token;        /* phi   */
    double attn_flops_per_token2;  /* a     */
    double weight_bytes;           /* omega */
    double nominal_batch;          /* Bbar  */
} hxo_model;

/* ---- the latency terms, one function per reading ---------------------- */

/* R1: queue of a single-server prefill instance (Sec. 4.2 resource model;
 * the waiting part of the prefill projection in Sec. 5.1). */
double hxo_prefill_wait(const hxo_model *m, int32_t backlog_tok, double F)
{
    return (double)backlog_tok * m->flops_per_token / F;
}

/* R2: roofline prefill time (Sec. 4.2 Estimator; Sec. 6). */
double hxo_prefill_time(const hxo_model *m, int32_t L, double F, double B)
{
    double l = (double)L;
    double t_compute = (m->flops_per_token * l + m->attn_flops_per_token2 * l * l) / F;
    double t_memory = (m->weight_bytes + m->kv_bytes_per_token * l) / B;
    return t_compute > t_memory ? t_compute : t_memory;
}

/* R3: KV size over class-pair bandwidth (Sec. 4.2 resource model). */
double hxo_transfer_time(const hxo_model *m, int32_t L, double bw, double lat)
{
    return m->kv_bytes_per_token * (double)L / bw + lat;
}

/* R4: time of one decode iteration of the batch now resident on d. */
double hxo_decode_step(const hxo_model *m, int32_t batch, int32_t used_tok, double F, double B)
{
    double t_compute = m->flops_per_token * (double)batch / F;
    double t_memory = (m->weight_bytes + m->kv_bytes_per_token * (double)used_tok) / B;
    return t_compute > t_memory ? t_compute : t_memory;
}

/* R4: decode availability hint (Sec. 5.3): queued decode tokens drained
 * Bbar at a time. */
double hxo_decode_wait(const hxo_model *m, int32_t qd_tok, int32_t batch, int32_t used_tok,
                       double F, double B)
{
    return (double)qd_tok * hxo_decode_step(m, batch, used_tok, F, B) / m->nominal_batch;
}

/* R5: per-token decode time once call (L,O) has joined the batch on d; its
 * own context averages L + O/2 over the generation. */
double hxo_decode_token_time(const hxo_model *m, int32_t L, int32_t O, int32_t batch,
                             int32_t used_tok, double F, double B)
{
    double t_compute = m->flops_per_token * ((double)batch + 1.0) / F;
    double ctx = (double)used_tok + (double)L + (double)O / 2.0;
    double t_memory = (m->weight_bytes + m->kv_bytes_per_token * ctx) / B;
    return t_compute > t_memory ? t_compute : t_memory;
}

/* R6: Eq. (3),(4) in tokens, against the capacity still free.  64-bit sum so
 * that no int32 overflow can turn an infeasible pair feasible. */
int hxo_feasible(int32_t L, int32_t O, int32_t used_tok, int32_t cap_tok)
{
    int64_t need = (int64_t)used_tok + (int64_t)L + (int64_t)O;
    return need <= (int64_t)cap_tok;
}

/* R7: projected time from now until decode finishes on the pair (p,d)
 * (Sec. 5.3: prefill finish + transfer, then earliest decode finish). */
double hxo_candidate_cost(const hxo_model *m, int32_t L, int32_t O,
                          double pF, double pB, int32_t p_backlog,
                          double dF, double dB, int32_t d_used, int32_t d_cap,
                          int32_t d_batch, int32_t d_qd,
                          double link_bw, double link_lat)
{
    if (!hxo_feasible(L, O, d_used, d_cap))
        return INFINITY;
    double ready = hxo_prefill_wait(m, p_backlog, pF) + hxo_prefill_time(m, L, pF, pB)
                 + hxo_transfer_time(m, L, link_bw, link_lat);
    double avail = hxo_decode_wait(m, d_qd, d_batch, d_used, dF, dB);
    double start = ready > avail ? ready : avail;
    return start + (double)O * hxo_decode_token_time(m, L, O, d_batch, d_used, dF, dB);
}

/* ---- the enumeration (Algorithm 1 inner loop; Sec. 5.3) ---------------- */

/*
 * For every call c, every prefill p and every decode d evaluate R7 and keep
 * the lexicographic minimum of (cost, p*D + d)  (R8).
 *
 * cost      [C*P*D] fp64, row-major (c, p, d); may be NULL
 * feas      [C*D]   1 = feasible;              may be NULL
 * best_p/d  [C]     -1 when no pair is feasible
 * best_cost [C]     +inf when no pair is feasible
 * second    [C]     smallest cost among the other candidates (+inf if none);
 *                   may be NULL.  Lets a checker see how close a tie was.
 * link_lat  [T*T] or NULL (= 0)
 * Returns 0, or -1 on a bad argument (negative size, type out of range).
 */
int hxo_score(const hxo_model *m,
              int32_t C, const int32_t *L_in, const int32_t *L_out,
              int32_t P, const float *pF, const float *pB,
              const int32_t *p_backlog, const int32_t *p_type,
              int32_t D, const float *dF, const float *dB,
              const int32_t *d_used, const int32_t *d_cap,
              const int32_t *d_batch, const int32_t *d_qd, const int32_t *d_type,
              int32_t T, const float *link_bw, const float *link_lat,
              double *cost, uint8_t *feas,
              int32_t *best_p, int32_t *best_d, double *best_cost, double *second,
              int32_t nthreads)
{
    if (C < 0 || P < 0 || D < 0 || T <= 0) return -1;
    for (int32_t p = 0; p < P; ++p) if (p_type[p] < 0 || p_type[p] >= T) return -1;
    for (int32_t d = 0; d < D; ++d) if (d_type[d] < 0 || d_type[d] >= T) return -1;
    (void)nthreads;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#pragma omp parallel for schedule(static)
#endif
    for (int32_t c = 0; c < C; ++c) {
        double bc = INFINITY, sc = INFINITY;
        int32_t bp = -1, bd = -1;
        for (int32_t d = 0; d < D && feas; ++d)
            feas[(size_t)c * D + d] = (uint8_t)hxo_feasible(L_in[c], L_out[c], d_used[d], d_cap[d]);
        for (int32_t p = 0; p < P; ++p) {
            for (int32_t d = 0; d < D; ++d) {
                int32_t tp = p_type[p], td = d_type[d];
                double lat = link_lat ? (double)link_lat[tp * T + td] : 0.0;
                double v = hxo_candidate_cost(m, L_in[c], L_out[c],
                                              (double)pF[p], (double)pB[p], p_backlog[p],
                                              (double)dF[d], (double)dB[d], d_used[d], d_cap[d],
                                              d_batch[d], d_qd[d],
                                              (double)link_bw[tp * T + td], lat);
                if (cost) cost[((size_t)c * P + p) * D + d] = v;
                /* candidates are visited in increasing flat index, so a strict
                 * "<" keeps the lowest flat index among equal costs */
                if (v < bc) { sc = bc; bc = v; bp = p; bd = d; }
                else if (v < sc) { sc = v; }
            }
        }
        best_p[c] = bp; best_d[c] = bd; best_cost[c] = bc;
        if (second) second[c] = sc;
    }
    return 0;
}

/* One candidate by index, for spot checks of very large rounds. */
double hxo_score_one(const hxo_model *m, int32_t L, int32_t O,
                     int32_t p, const float *pF, const float *pB,
                     const int32_t *p_backlog, const int32_t *p_type,
                     int32_t d, const float *dF, const float *dB,
                     const int32_t *d_used, const int32_t *d_cap,
                     const int32_t *d_batch, const int32_t *d_qd, const int32_t *d_type,
                     int32_t T, const float *link_bw, const float *link_lat)
{
    int32_t tp = p_type[p], td = d_type[d];
    double lat = link_lat ? (double)link_lat[tp * T + td] : 0.0;
    return hxo_candidate_cost(m, L, O, (double)pF[p], (double)pB[p], p_backlog[p],
                              (double)dF[d], (double)dB[d], d_used[d], d_cap[d],
                              d_batch[d], d_qd[d], (double)link_bw[tp * T + td], lat);
}

/* R8 on a tensor that already exists: first index of the minimum. */
int hxo_select(int32_t C, int32_t P, int32_t D, const double *cost,
               int32_t *best_p, int32_t *best_d, double *best_cost)
{
    if (C < 0 || P < 0 || D < 0) return -1;
    for (int32_t c = 0; c < C; ++c) {
        double bc = INFINITY;
        int64_t bi = -1;
        const double *row = cost + (size_t)c * P * D;
        for (int64_t i = 0; i < (int64_t)P * D; ++i)
            if (row[i] < bc) { bc = row[i]; bi = i; }
        best_p[c] = bi < 0 ? -1 : (int32_t)(bi / D);
        best_d[c] = bi < 0 ? -1 : (int32_t)(bi % D);
        best_cost[c] = bc;
    }
    return 0;
}

/* R9: cost of one call on an idle pool, best class pair (the per-node term of
 * the standalone horizon, Sec. 5.1). */
int hxo_node_cost(const hxo_model *m, int32_t n, const int32_t *L_in, const int32_t *L_out,
                  int32_t T, const float *tF, const float *tB,
                  const float *link_bw, const float *link_lat, double *cost)
{
    if (n < 0 || T <= 0) return -1;
    for (int32_t v = 0; v < n; ++v) {
        double best = INFINITY;
        for (int32_t tp = 0; tp < T; ++tp) {
            for (int32_t td = 0; td < T; ++td) {
                double lat = link_lat ? (double)link_lat[tp * T + td] : 0.0;
                double t = hxo_prefill_time(m, L_in[v], (double)tF[tp], (double)tB[tp])
                         + hxo_transfer_time(m, L_in[v], (double)link_bw[tp * T + td], lat)
                         + (double)L_out[v] * hxo_decode_token_time(m, L_in[v], L_out[v], 0, 0,
                                                                    (double)tF[td], (double)tB[td]);
                if (t < best) best = t;
            }
        }
        cost[v] = best;
    }
    return 0;
}

/* ---- critical path (R10; Sec. 5.1 horizon; horizon-update step of Algorithm 1) */

/*
 * Longest remaining path over a DAG given as successor lists.  Makes no
 * assumption on node numbering: nodes are finished in depth-first post-order,
 * so every successor is final before its predecessor is.
 *
 * row_ptr [n+1], col [row_ptr[n]]  successor CSR
 * cost    [n]     per-node cost (already fp32-representable when
 *                 round_f32 != 0)
 * wf_ptr  [n_wf+1] nodes of workflow w are wf_ptr[w] .. wf_ptr[w+1]-1
 * rem, tail [n], horizon [n_wf]  fp64 holders; with round_f32 != 0 every sum
 *                 is rounded to fp32 first (one rounding per node; the max is
 *                 exact), so the values are exactly the fp32 results
 * level   [n]
 * Returns 0; -1 bad argument; -2 the graph has a cycle; -3 out of memory.
 */
int hxo_critical_path(int32_t n, const int32_t *row_ptr, const int32_t *col, const double *cost,
                      int32_t n_wf, const int32_t *wf_ptr, int round_f32,
                      double *rem, double *tail, int32_t *level, double *horizon)
{
    if (n < 0 || n_wf < 0) return -1;
    for (int32_t v = 0; v < n; ++v) {
        if (row_ptr[v] > row_ptr[v + 1] || row_ptr[v] < 0) return -1;
        for (int32_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e)
            if (col[e] < 0 || col[e] >= n) return -1;
    }
    /* state: 0 = untouched, 1 = on the stack, 2 = final */
    uint8_t *state = (uint8_t *)calloc((size_t)n + 1, 1);
    int32_t *stack = (int32_t *)malloc(((size_t)n + 1) * sizeof(int32_t));
    int32_t *next_edge = (int32_t *)malloc(((size_t)n + 1) * sizeof(int32_t));
    if (!state || !stack || !next_edge) { free(state); free(stack); free(next_edge); return -3; }
    int rc = 0;
    for (int32_t root = 0; root < n && rc == 0; ++root) {
        if (state[root]) continue;
        int32_t top = 0;
        stack[top] = root; state[root] = 1; next_edge[root] = row_ptr[root];
        while (top >= 0) {
            int32_t v = stack[top];
            if (next_edge[v] < row_ptr[v + 1]) {
                int32_t u = col[next_edge[v]++];
                if (state[u] == 1) { rc = -2; break; }          /* back edge */
                if (state[u] == 0) {
                    state[u] = 1; next_edge[u] = row_ptr[u]; stack[++top] = u;
                }
            } else {
                double t = 0.0;
                int32_t lv = 0;
                for (int32_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
                    int32_t u = col[e];
                    if (rem[u] > t) t = rem[u];
                    if (level[u] + 1 > lv) lv = level[u] + 1;
                }
                double r = cost[v] + t;
                if (round_f32) r = (double)(float)r;
                tail[v] = t; rem[v] = r; level[v] = lv;
                state[v] = 2; --top;
            }
        }
    }
    free(state); free(stack); free(next_edge);
    if (rc) return rc;
    for (int32_t w = 0; w < n_wf; ++w) {
        double h = 0.0;
        if (wf_ptr[w] < 0 || wf_ptr[w + 1] > n || wf_ptr[w] > wf_ptr[w + 1]) return -1;
        for (int32_t v = wf_ptr[w]; v < wf_ptr[w + 1]; ++v)
            if (rem[v] > h) h = rem[v];
        horizon[w] = h;
    }
    return 0;
}

/* Same pass when workflow membership is a per-node id instead of ranges
 * (nodes appended at run time are not contiguous per workflow). */
int hxo_horizon_by_id(int32_t n, const double *rem, const int32_t *wf_of_node,
                      int32_t n_wf, double *horizon)
{
    for (int32_t w = 0; w < n_wf; ++w) horizon[w] = 0.0;
    for (int32_t v = 0; v < n; ++v) {
        int32_t w = wf_of_node[v];
        if (w < 0 || w >= n_wf) return -1;
        if (rem[v] > horizon[w]) horizon[w] = rem[v];
    }
    return 0;
}

/* R10 on a graph in reveal order (Sec. 4.1: a call is revealed after its
 * parents, so every parent has a smaller id than its child), given as parent
 * lists with a per-node workflow id: the same definition as hxo_critical_path,
 * evaluated by one pass from the last node to the first.  When node v is
 * reached every successor of v (a larger id) is final and has already offered
 * its rem and level to v, so tail[v] and level[v] are complete; rem[v] is then
 * one addition and v offers it to its own parents.  For long-lived graphs of
 * tens of millions of nodes, where the depth-first form's transposition of the
 * parent lists is what costs.
 * Returns 0; -1 bad argument (a parent id not below its child's, a workflow id
 * out of range). */
int hxo_critical_path_revealed(int32_t n, const int32_t *parent_row_ptr, const int32_t *parent_col,
                               const double *cost, const int32_t *wf_of_node, int32_t n_wf, int round_f32,
                               double *rem, double *tail, int32_t *level, double *horizon)
{
    if (n < 0 || n_wf < 0) return -1;
    for (int32_t v = 0; v < n; ++v) {
        if (parent_row_ptr[v] > parent_row_ptr[v + 1] || parent_row_ptr[v] < 0) return -1;
        for (int32_t e = parent_row_ptr[v]; e < parent_row_ptr[v + 1]; ++e)
            if (parent_col[e] < 0 || parent_col[e] >= v) return -1;
        if (wf_of_node[v] < 0 || wf_of_node[v] >= n_wf) return -1;
        tail[v] = 0.0; level[v] = 0;
    }
    for (int32_t w = 0; w < n_wf; ++w) horizon[w] = 0.0;
    for (int32_t v = n - 1; v >= 0; --v) {
        double r = cost[v] + tail[v];
        if (round_f32) r = (double)(float)r;
        rem[v] = r;
        if (r > horizon[wf_of_node[v]]) horizon[wf_of_node[v]] = r;
        for (int32_t e = parent_row_ptr[v]; e < parent_row_ptr[v + 1]; ++e) {
            int32_t u = parent_col[e];
            if (r > tail[u]) tail[u] = r;
            if (level[v] + 1 > level[u]) level[u] = level[v] + 1;
        }
    }
    return 0;
}

/* R11: Eq. (2) with the downstream tail of the call's node added.  Eq. (2)
 * divides by the workflow's horizon and says nothing of a horizon of zero (a
 * workflow whose revealed calls all cost nothing); the reading taken here: such
 * a call is as urgent as can be, R = +infinity, whatever the numerator. */
static double ratio_r11(double elapsed, double cost, double tail, double horizon)
{
    if (!(horizon > 0.0)) return INFINITY;
    return (elapsed + cost + tail) / horizon;
}

int hxo_urgency(int32_t C, const double *elapsed, const double *best_cost,
                const int32_t *node, const int32_t *wf,
                const double *tail, const double *horizon, double *ratio)
{
    for (int32_t c = 0; c < C; ++c)
        ratio[c] = ratio_r11(elapsed[c], best_cost[c], tail[node[c]], horizon[wf[c]]);
    return 0;
}

/* ---- R12: commit the chosen placements, then drain (the simulated-state
 * update of Algorithm 1, batched once per round) -------------------------- */

/*
 * For every call with a placement: backlog_tok[p*] += L; qd_tok[d*] += O;
 * used_tok[d*] += L + O.  Then per instance: backlog = max(0, backlog -
 * drain_prefill), qd = max(0, qd - drain_decode_q), used = max(0, used -
 * release_tok), batch = ceil(used / tokens_per_seq) clipped to [0, max_batch].
 * All int32 with 64-bit intermediates.  A total above INT32_MAX is an error
 * (return -4); the tables then hold the saturated values.
 */
static int32_t sat32(int64_t x)
{
    if (x > 2147483647LL) return 2147483647;
    if (x < 0) return 0;
    return (int32_t)x;
}

int hxo_commit(int32_t C, const int32_t *L_in, const int32_t *L_out,
               const int32_t *best_p, const int32_t *best_d,
               int32_t P, int32_t *backlog_tok,
               int32_t D, int32_t *used_tok, int32_t *batch, int32_t *qd_tok,
               const int32_t *drain_prefill, const int32_t *drain_decode_q,
               const int32_t *release_tok, int32_t tokens_per_seq, int32_t max_batch)
{
    if (tokens_per_seq <= 0) return -1;
    int64_t *bl = (int64_t *)calloc((size_t)P + 1, sizeof(int64_t));
    int64_t *us = (int64_t *)calloc((size_t)D + 1, sizeof(int64_t));
    int64_t *qd = (int64_t *)calloc((size_t)D + 1, sizeof(int64_t));
    if (!bl || !us || !qd) { free(bl); free(us); free(qd); return -3; }
    for (int32_t p = 0; p < P; ++p) bl[p] = backlog_tok[p];
    for (int32_t d = 0; d < D; ++d) { us[d] = used_tok[d]; qd[d] = qd_tok[d]; }
    int rc = 0;
    for (int32_t c = 0; c < C; ++c) {
        int32_t p = best_p[c], d = best_d[c];
        if (p < 0 || d < 0) continue;
        if (p >= P || d >= D) { rc = -1; break; }
        bl[p] += L_in[c];
        qd[d] += L_out[c];
        us[d] += (int64_t)L_in[c] + L_out[c];
    }
    if (rc == 0) {
        for (int32_t p = 0; p < P; ++p) if (bl[p] > 2147483647LL) rc = -4;
        for (int32_t d = 0; d < D; ++d) if (us[d] > 2147483647LL || qd[d] > 2147483647LL) rc = -4;
        for (int32_t p = 0; p < P; ++p)
            backlog_tok[p] = sat32(sat32(bl[p]) - (int64_t)drain_prefill[p]);
        for (int32_t d = 0; d < D; ++d) {
            qd_tok[d] = sat32(sat32(qd[d]) - (int64_t)drain_decode_q[d]);
            used_tok[d] = sat32(sat32(us[d]) - (int64_t)release_tok[d]);
            int64_t b = ((int64_t)used_tok[d] + tokens_per_seq - 1) / tokens_per_seq;
            if (b > max_batch) b = max_batch;
            batch[d] = (int32_t)b;
        }
    }
    free(bl); free(us); free(qd);
    return rc;
}

/* ---- R14: one-pass ordering by the risk score (Sec. 5.3) ----------------- */

int hxo_rank(int32_t C, const double *ratio, int32_t *rank)
{
    if (C < 0) return -1;
    for (int32_t c = 0; c < C; ++c) {
        int32_t ahead = 0;
        for (int32_t k = 0; k < C; ++k)
            if (ratio[k] > ratio[c] || (ratio[k] == ratio[c] && k < c)) ++ahead;
        rank[c] = ahead;
    }
    return 0;
}

/* ---- R13: the recomputing greedy loop of Algorithm 1 (Sec. 5.3) ---------- */

/*
 * p_backlog [P], d_used, d_batch, d_qd [D] are the simulated state: read, and
 * left as the plan leaves them.  Outputs per call, as of the moment the call
 * was picked: best_p, best_d, best_cost, ratio, rank.
 * Returns 0; -1 bad argument; -3 out of memory; -4 an int32 counter overflowed.
 */
int hxo_plan_greedy(const hxo_model *m,
                    int32_t C, const int32_t *L_in, const int32_t *L_out,
                    const double *elapsed, const int32_t *node, const int32_t *wf,
                    const double *tail, const double *horizon,
                    int32_t P, const float *pF, const float *pB, int32_t *p_backlog, const int32_t *p_type,
                    int32_t D, const float *dF, const float *dB, int32_t *d_used, const int32_t *d_cap,
                    int32_t *d_batch, int32_t *d_qd, const int32_t *d_type,
                    int32_t T, const float *link_bw, const float *link_lat,
                    int32_t tokens_per_seq, int32_t max_batch,
                    int32_t *best_p, int32_t *best_d, double *best_cost, double *ratio, int32_t *rank)
{
    if (C < 0 || P < 0 || D < 0 || T <= 0 || tokens_per_seq <= 0) return -1;
    uint8_t *done = (uint8_t *)calloc((size_t)C + 1, 1);
    if (!done) return -3;
    int rc = 0;
    for (int32_t k = 0; k < C && rc == 0; ++k) {
        int32_t pick = -1, pick_p = -1, pick_d = -1;
        double pick_r = 0.0, pick_cost = 0.0;
        for (int32_t c = 0; c < C; ++c) {
            if (done[c]) continue;
            double bc = INFINITY;
            int32_t bp = -1, bd = -1;
            for (int32_t p = 0; p < P; ++p)
                for (int32_t d = 0; d < D; ++d) {
                    int32_t tp = p_type[p], td = d_type[d];
                    double lat = link_lat ? (double)link_lat[tp * T + td] : 0.0;
                    double v = hxo_candidate_cost(m, L_in[c], L_out[c], (double)pF[p], (double)pB[p], p_backlog[p],
                                                  (double)dF[d], (double)dB[d], d_used[d], d_cap[d], d_batch[d], d_qd[d],
                                                  (double)link_bw[tp * T + td], lat);
                    if (v < bc) { bc = v; bp = p; bd = d; }
                }
            double r = ratio_r11(elapsed[c], bc, tail[node[c]], horizon[wf[c]]);
            if (pick < 0 || r > pick_r) { pick = c; pick_r = r; pick_cost = bc; pick_p = bp; pick_d = bd; }
        }
        done[pick] = 1;
        best_p[pick] = pick_p; best_d[pick] = pick_d; best_cost[pick] = pick_cost; ratio[pick] = pick_r; rank[pick] = k;
        if (pick_p >= 0) {
            int64_t bl = (int64_t)p_backlog[pick_p] + L_in[pick];
            int64_t qd = (int64_t)d_qd[pick_d] + L_out[pick];
            int64_t us = (int64_t)d_used[pick_d] + L_in[pick] + L_out[pick];
            if (bl > 2147483647LL || qd > 2147483647LL || us > 2147483647LL) { rc = -4; break; }
            p_backlog[pick_p] = (int32_t)bl; d_qd[pick_d] = (int32_t)qd; d_used[pick_d] = (int32_t)us;
            int64_t b = (us + tokens_per_seq - 1) / tokens_per_seq;
            d_batch[pick_d] = (int32_t)(b > max_batch ? max_batch : b);
        }
    }
    free(done);
    return rc;
}

/* ---- decode stage (Sec. 5.4): capacity intervals, locks, greedy ------------- */

/* R22: tokens occupied on an instance at time tau. */
int64_t hxo_occupancy(int32_t K, const double *iv_start, const double *iv_end, const int32_t *iv_tok, double tau)
{
    int64_t occ = 0;
    for (int32_t j = 0; j < K; ++j)
        if (iv_start[j] <= tau && tau < iv_end[j]) occ += iv_tok[j];
    return occ;
}

/* R23: is a start at t capacity-feasible for a call of m_tok tokens decoding
 * for T seconds?  Occupancy only rises where an interval starts, so the window
 * [t, t + T) is checked at t and at every interval start inside it. */
int hxo_start_is_feasible(int32_t m_tok, double T, int32_t cap_tok, double t,
                          int32_t K, const double *iv_start, const double *iv_end, const int32_t *iv_tok)
{
    if (hxo_occupancy(K, iv_start, iv_end, iv_tok, t) + (int64_t)m_tok > (int64_t)cap_tok) return 0;
    for (int32_t j = 0; j < K; ++j)
        if (iv_start[j] > t && iv_start[j] < t + T &&
            hxo_occupancy(K, iv_start, iv_end, iv_tok, iv_start[j]) + (int64_t)m_tok > (int64_t)cap_tok) return 0;
    return 1;
}

/* R23: earliest capacity-feasible start, by trying now and every interval end. */
double hxo_decode_start(int32_t m_tok, double T, int32_t cap_tok,
                        int32_t K, const double *iv_start, const double *iv_end, const int32_t *iv_tok)
{
    if ((int64_t)m_tok > (int64_t)cap_tok) return INFINITY;
    double best = INFINITY;
    if (hxo_start_is_feasible(m_tok, T, cap_tok, 0.0, K, iv_start, iv_end, iv_tok)) best = 0.0;
    for (int32_t j = 0; j < K; ++j) {
        double t = iv_end[j];
        if (t > 0.0 && t < best && hxo_start_is_feasible(m_tok, T, cap_tok, t, K, iv_start, iv_end, iv_tok)) best = t;
    }
    return best;
}

/*
 * R24, R25: decode-stage score of every (call, instance).  Interval lists are
 * stored with a fixed stride: instance d owns entries d*stride .. d*stride +
 * iv_count[d] - 1.  start, cost: [Q*D] or NULL; best_*: [Q].  Returns -3 on a
 * lock outside [-1, D).
 */
int hxo_decode_score(const hxo_model *m, int32_t Q, const int32_t *L_in, const int32_t *L_out, const int32_t *lock,
                     int32_t D, const float *dF, const float *dB, const int32_t *d_used, const int32_t *d_cap,
                     const int32_t *d_batch,
                     int32_t stride, const int32_t *iv_count, const double *iv_start, const double *iv_end,
                     const int32_t *iv_tok,
                     double *start, double *cost, int32_t *best_d, double *best_start, double *best_cost)
{
    if (Q < 0 || D < 0 || stride < 0) return -1;
    for (int32_t c = 0; c < Q; ++c)
        if (lock && (lock[c] < -1 || lock[c] >= D)) return -3;
    for (int32_t c = 0; c < Q; ++c) {
        double bc = INFINITY, bs = INFINITY;
        int32_t bd = -1;
        for (int32_t d = 0; d < D; ++d) {
            double S = INFINITY, v = INFINITY;
            if (!lock || lock[c] < 0 || lock[c] == d) {
                double T = (double)L_out[c] *
                           hxo_decode_token_time(m, L_in[c], L_out[c], d_batch[d], d_used[d], (double)dF[d], (double)dB[d]);
                int64_t need = (int64_t)L_in[c] + (int64_t)L_out[c];
                int32_t m_tok = need > 2147483647LL ? 2147483647 : (int32_t)need;
                if (need <= (int64_t)d_cap[d])
                    S = hxo_decode_start(m_tok, T, d_cap[d], iv_count[d], iv_start + (size_t)d * stride,
                                         iv_end + (size_t)d * stride, iv_tok + (size_t)d * stride);
                v = S + T;
            }
            if (start) start[(size_t)c * D + d] = S;
            if (cost) cost[(size_t)c * D + d] = v;
            if (v < bc) { bc = v; bs = S; bd = d; }
        }
        best_d[c] = bd; best_start[c] = bs; best_cost[c] = bc;
    }
    return 0;
}

/*
 * Not part of the method: hxo_decode_score with every decode time replaced by
 * max(0, t_scale * Tdec + t_shift), for the parity tests of a finished plan,
 * which bracket what fp32 rounding of Tdec and of start + Tdec can decide
 * differently (a plan creates exact ties: a call placed where another of the
 * same decode time ended).  At (1, 0) it returns what hxo_decode_score returns.
 */
int hxo_decode_score_bracket(const hxo_model *m, int32_t Q, const int32_t *L_in, const int32_t *L_out, const int32_t *lock,
                             int32_t D, const float *dF, const float *dB, const int32_t *d_used, const int32_t *d_cap,
                             const int32_t *d_batch,
                             int32_t stride, const int32_t *iv_count, const double *iv_start, const double *iv_end,
                             const int32_t *iv_tok, double t_scale, double t_shift,
                             double *start, double *cost, int32_t *best_d, double *best_start, double *best_cost)
{
    if (Q < 0 || D < 0 || stride < 0) return -1;
    for (int32_t c = 0; c < Q; ++c)
        if (lock && (lock[c] < -1 || lock[c] >= D)) return -3;
    for (int32_t c = 0; c < Q; ++c) {
        double bc = INFINITY, bs = INFINITY;
        int32_t bd = -1;
        for (int32_t d = 0; d < D; ++d) {
            double S = INFINITY, v = INFINITY;
            if (!lock || lock[c] < 0 || lock[c] == d) {
                double T = t_scale * (double)L_out[c] *
                           hxo_decode_token_time(m, L_in[c], L_out[c], d_batch[d], d_used[d], (double)dF[d], (double)dB[d]) + t_shift;
                if (T < 0.0) T = 0.0;
                int64_t need = (int64_t)L_in[c] + (int64_t)L_out[c];
                int32_t m_tok = need > 2147483647LL ? 2147483647 : (int32_t)need;
                if (need <= (int64_t)d_cap[d])
                    S = hxo_decode_start(m_tok, T, d_cap[d], iv_count[d], iv_start + (size_t)d * stride,
                                         iv_end + (size_t)d * stride, iv_tok + (size_t)d * stride);
                v = S + T;
            }
            if (start) start[(size_t)c * D + d] = S;
            if (cost) cost[(size_t)c * D + d] = v;
            if (v < bc) { bc = v; bs = S; bd = d; }
        }
        best_d[c] = bd; best_start[c] = bs; best_cost[c] = bc;
    }
    return 0;
}

/*
 * R26: recomputing greedy of the decode stage.  The interval lists are
 * extended in place (iv_count grows); -4 when an instance's list is full.
 */
int hxo_decode_plan_greedy(const hxo_model *m, int32_t Q, const int32_t *L_in, const int32_t *L_out, const int32_t *lock,
                           const double *elapsed, const int32_t *node, const int32_t *wf,
                           const double *tail, const double *horizon,
                           int32_t D, const float *dF, const float *dB, const int32_t *d_used, const int32_t *d_cap,
                           const int32_t *d_batch,
                           int32_t stride, int32_t *iv_count, double *iv_start, double *iv_end, int32_t *iv_tok,
                           int32_t *best_d, double *best_start, double *best_cost, double *ratio, int32_t *rank)
{
    if (Q < 0 || D < 0 || stride < 0) return -1;
    uint8_t *done = (uint8_t *)calloc((size_t)Q + 1, 1);
    if (!done) return -3;
    int rc = 0;
    for (int32_t k = 0; k < Q && rc == 0; ++k) {
        int32_t pick = -1, pick_d = -1;
        double pick_r = 0.0, pick_s = 0.0, pick_cost = 0.0;
        for (int32_t c = 0; c < Q; ++c) {
            if (done[c]) continue;
            int32_t bd;
            double bs, bc;
            rc = hxo_decode_score(m, 1, L_in + c, L_out + c, lock ? lock + c : NULL, D, dF, dB, d_used, d_cap, d_batch,
                                  stride, iv_count, iv_start, iv_end, iv_tok, NULL, NULL, &bd, &bs, &bc);
            if (rc) break;
            double r = ratio_r11(elapsed[c], bc, tail[node[c]], horizon[wf[c]]);
            if (pick < 0 || r > pick_r) { pick = c; pick_r = r; pick_d = bd; pick_s = bs; pick_cost = bc; }
        }
        if (rc) break;
        done[pick] = 1;
        best_d[pick] = pick_d; best_start[pick] = pick_s; best_cost[pick] = pick_cost; ratio[pick] = pick_r; rank[pick] = k;
        if (pick_d >= 0) {
            if (iv_count[pick_d] >= stride) { rc = -4; break; }
            size_t at = (size_t)pick_d * stride + iv_count[pick_d];
            iv_start[at] = pick_s; iv_end[at] = pick_cost; iv_tok[at] = L_in[pick] + L_out[pick];
            iv_count[pick_d] += 1;
        }
    }
    free(done);
    return rc;
}
