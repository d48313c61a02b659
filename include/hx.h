/*
 * hx.h -- C ABI of the GPU placement search (AMD MI355X / gfx950).
 *
 * The library evaluates, for one scheduling invocation of a workflow- and
 * heterogeneity-aware scheduler on a prefill-decode disaggregated pool, the
 * search the paper's Algorithm 1 runs for every waiting call: enumerate every
 * (prefill instance, decode instance) pair, estimate the time until decode
 * finishes there, keep the earliest feasible pair, and turn it into the
 * call's projected ratio against its workflow horizon.
 *
 * Conventions for every entry point
 * ---------------------------------
 *  - Returns HX_OK (0) or a negative HX_ERR_* code; never throws; a failed
 *    call has launched nothing.  hx_last_error(ctx) describes the last
 *    failure of that context.
 *  - "device" pointers are device memory of the GPU the context was created
 *    on, owned by the caller, valid until the work enqueued on `stream` has
 *    finished.  "host" pointers are ordinary host memory read during the
 *    call.  The structs hx_model / hx_calls / hx_prefill_tab / hx_decode_tab /
 *    hx_links / hx_intervals themselves live in host memory; their pointer members are
 *    device pointers.  The library never returns memory the caller must free
 *    (hx_dag_view returns borrowed pointers into the context).
 *  - `stream` is a hipStream_t (NULL = the default stream).  Work is enqueued
 *    on it and the call returns without waiting.  Conditions that only the
 *    GPU can see (an index out of range inside an array, a graph that is not
 *    a DAG, a sweep limit reached) never fault: the offending element is
 *    skipped, a sticky status word is set on the device, and
 *    hx_stream_status() reports it after synchronising the stream.
 *  - Indices are int32; -1 means "none".  Costs are fp32 seconds, +infinity
 *    for an infeasible pair.  Rates are FLOP/s and B/s, lengths and
 *    capacities are tokens.
 *  - Calls on one context must not overlap in time on different streams: the
 *    context owns scratch that consecutive calls reuse.  One exception, for
 *    rounds that refresh horizons beside the search: hx_node_cost,
 *    hx_critical_path (single pass), hx_horizons, hx_dag_append and
 *    hx_dag_set_cost may run on one stream while hx_score_placements with
 *    fused outputs only, or hx_urgency, runs on another (they share nothing
 *    but the status word, which kernels update atomically).  A context is not
 *    thread-safe.
 *  - Device memory is allocated by hx_ctx_create and hx_dag_reserve, and by
 *    hx_decode_score and hx_rank (beyond 16384 calls) the first time they meet
 *    a larger problem than before; every other call only launches kernels and
 *    can be captured in a HIP graph (hx_validate_round and hx_stream_status
 *    wait for the stream and cannot).
 */
#ifndef HX_H
#define HX_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HX_OK               0
#define HX_ERR_INVALID_ARG (-1)  /* NULL where a pointer is required, negative size, bad flag      */
#define HX_ERR_SHAPE       (-2)  /* a size beyond HX_MAX_TYPES / HX_MAX_INSTANCES / int32 indexing */
#define HX_ERR_NOT_DAG     (-3)  /* successor not later than its node / no fixed point in time      */
#define HX_ERR_CAPACITY    (-4)  /* reserved store, scratch or sweep limit exceeded                 */
#define HX_ERR_DEVICE      (-5)  /* a HIP call failed; hx_last_error has its text                   */
#define HX_ERR_INDEX       (-6)  /* an index held in a device array is out of range                 */
#define HX_ERR_OVERFLOW    (-7)  /* an int32 instance counter would exceed INT32_MAX                */

#define HX_MAX_TYPES      8      /* GPU classes in a pool                      */
#define HX_MAX_INSTANCES  1024   /* prefill instances, and decode instances    */
#define HX_GREEDY_MAX_CALLS      1024   /* queue length hx_plan_greedy takes            */
#define HX_GREEDY_MAX_INSTANCES  256    /* instances per side hx_plan_greedy takes      */
#define HX_MAX_INTERVALS         511    /* entries per decode instance in hx_intervals  */
#define HX_DECODE_GREEDY_MAX_CALLS 1024 /* queue length hx_decode_plan_greedy takes     */

typedef struct hx_ctx hx_ctx;

/* Model descriptor of the estimator (Sec. 4.2 "Scheduler internals": a
 * roofline-style model over per-call input and output length). */
typedef struct {
    float kv_bytes_per_token;      /* kappa: KV-cache bytes one token occupies           */
    float flops_per_token;         /* phi:   FLOP per token, linear part                 */
    float attn_flops_per_token2;   /* a:     FLOP per token^2, attention part of prefill */
    float weight_bytes;            /* omega: bytes read per forward pass                 */
    float nominal_batch;           /* Bbar:  decode-queue tokens retired per decode step */
} hx_model;

/* Ready calls, structure of arrays, n entries each (Sec. 7.1: a call is
 * annotated with input length, output length and workflow identity). */
typedef struct {
    int32_t n;
    const int32_t *L_in;      /* device [n] prompt tokens, >= 0                        */
    const int32_t *L_out;     /* device [n] predicted output tokens, >= 0              */
    const int32_t *node;      /* device [n] DAG node of the call; NULL if no ratio     */
    const int32_t *wf;        /* device [n] workflow of the call;  NULL if no ratio    */
    const float   *elapsed;   /* device [n] t - a_w of Eq. (2);    NULL if no ratio    */
} hx_calls;

/* Prefill pool snapshot: single-server instances with a queue (Sec. 4.2
 * "Heterogeneous resource modelling"). */
typedef struct {
    int32_t n;                    /* P, 0..HX_MAX_INSTANCES                            */
    const float   *flops;         /* device [n] FLOP/s, > 0                            */
    const float   *hbm_bw;        /* device [n] B/s, > 0                               */
    const int32_t *backlog_tok;   /* device [n] prompt tokens queued ahead, >= 0       */
    const int32_t *type;          /* device [n] GPU class, 0..n_types-1                */
} hx_prefill_tab;

/* Decode pool snapshot: batched decoding under a KV-capacity limit. */
typedef struct {
    int32_t n;                    /* D, 0..HX_MAX_INSTANCES                            */
    const float   *flops;         /* device [n] FLOP/s, > 0                            */
    const float   *hbm_bw;        /* device [n] B/s, > 0                               */
    const int32_t *used_tok;      /* device [n] KV tokens resident, >= 0               */
    const int32_t *cap_tok;       /* device [n] KV capacity in tokens, Cap(d) of Eq. (4) */
    const int32_t *batch;         /* device [n] sequences in the running batch, >= 0   */
    const int32_t *qd_tok;        /* device [n] output tokens queued for decode, >= 0  */
    const int32_t *type;          /* device [n] GPU class, 0..n_types-1                */
} hx_decode_tab;

/* Effective KV-transfer bandwidth between GPU classes (Sec. 4.2): row =
 * class of the prefill side, column = class of the decode side. */
typedef struct {
    int32_t n_types;              /* T, 1..HX_MAX_TYPES                                */
    const float *bw;              /* device [T*T] B/s, > 0                             */
    const float *latency;         /* device [T*T] seconds added per transfer, or NULL  */
} hx_links;

/* ---- context ------------------------------------------------------------ */

/* Creates a context on HIP device `device` (allocates a few KB of scratch and
 * a pinned status word).  *out is NULL on failure. */
int hx_ctx_create(hx_ctx **out, int device);

/* Frees everything the context owns.  The caller has synchronised its streams. */
int hx_ctx_destroy(hx_ctx *ctx);

/* Text of the last error of this context (static storage, never NULL); with
 * ctx == NULL, why the last hx_ctx_create or hx_commit_static of this process failed. */
const char *hx_last_error(const hx_ctx *ctx);

/* Synchronises `stream`, returns the sticky device status (HX_OK or the first
 * HX_ERR_* a kernel raised since the last call) and clears it. */
int hx_stream_status(hx_ctx *ctx, void *stream);

/* ---- (1) critical path: CSR DAGs + per-node cost -> remaining latency ---- */

/*
 * Standalone cost of each call: its prefill, KV transfer and decode time on
 * an idle pool, on the best pair of GPU classes.  This is the per-node term
 * of the workflow horizon H_w(t) of Sec. 5.1, which is defined on the same
 * cluster with no other workflow present.
 *   n, L_in, L_out      device [n] lengths of the nodes
 *   n_types, type_flops, type_hbm_bw   device [n_types] per-class rates
 *   links               class-pair bandwidth (same n_types)
 *   cost                device [n] out, seconds
 */
int hx_node_cost(hx_ctx *ctx, const hx_model *model, int32_t n,
                 const int32_t *L_in, const int32_t *L_out,
                 int32_t n_types, const float *type_flops, const float *type_hbm_bw,
                 const hx_links *links, float *cost, void *stream);

/*
 * Longest remaining path of every node (max-plus pass from the sinks up) and
 * the horizon of every workflow (Sec. 5.1; the horizon-update step of
 * Algorithm 1):
 *   tail[v]  = max(0, max over successors u of rem[u])
 *   rem[v]   = node_cost[v] + tail[v]          (one fp32 addition)
 *   level[v] = 0 without successors, else 1 + max level[u]
 *   horizon[w] = max rem[v] over the nodes of w
 * Inputs (device): successor lists in CSR form, succ_row_ptr [n_nodes+1]
 * non-decreasing with succ_row_ptr[0] = 0 and succ_row_ptr[n_nodes] =
 * n_edges, succ_col_idx [n_edges]; node_cost [n_nodes] >= 0; wf_ptr [n_wf+1]:
 * workflow w owns the contiguous nodes wf_ptr[w] .. wf_ptr[w+1]-1.
 * Outputs (device): rem, tail [n_nodes] fp32; level [n_nodes]; horizon [n_wf].
 *
 * max_sweeps == 0: single pass.  Requires what online reveal gives by
 *   construction: every successor has a larger id than its node and belongs
 *   to the same workflow.  An edge that breaks this raises HX_ERR_NOT_DAG in
 *   the stream status; what is then written for the workflow the edge starts
 *   in is unspecified (no other workflow is affected, nothing faults).  Any
 *   workflow size and any number of successors per node are accepted; the
 *   pass is fastest when a node has at most 4.
 * max_sweeps  > 0: level-synchronous relaxation for any numbering; successors
 *   may be anywhere.  Sweeps until nothing changes, at most max_sweeps times
 *   (a DAG of depth L needs L+2); still changing then -> HX_ERR_NOT_DAG in the
 *   stream status (a cycle, or the limit was too small).
 * Both give bit-identical results on inputs both accept.
 */
int hx_critical_path(hx_ctx *ctx, int32_t n_nodes, int32_t n_edges,
                     const int32_t *succ_row_ptr, const int32_t *succ_col_idx,
                     const float *node_cost, int32_t n_wf, const int32_t *wf_ptr,
                     int32_t max_sweeps,
                     float *rem, float *tail, int32_t *level, float *horizon, void *stream);

/*
 * hx_node_cost followed by hx_critical_path (max_sweeps = 0) in one launch:
 * the standalone cost of every node is worked out from its lengths while the
 * pass stages the node, written to node_cost (device [n_nodes], out) and used
 * at once.  Same arguments, same requirements on the numbering, same results
 * bit for bit, same error reporting as the two calls; a node that no workflow
 * of wf_ptr covers gets no cost (the pass does not visit it).  Meant for the graphs
 * of a scheduling round, where a launch saved counts; on graphs of millions
 * of nodes the two separate calls are faster (the cost evaluation needs
 * registers that the pass alone gives to more resident workgroups).
 */
int hx_horizons(hx_ctx *ctx, const hx_model *model, int32_t n_nodes, int32_t n_edges,
                const int32_t *succ_row_ptr, const int32_t *succ_col_idx,
                const int32_t *L_in, const int32_t *L_out,
                int32_t n_types, const float *type_flops, const float *type_hbm_bw, const hx_links *links,
                int32_t n_wf, const int32_t *wf_ptr,
                float *node_cost, float *rem, float *tail, int32_t *level, float *horizon, void *stream);

/*
 * Incremental form for DAGs revealed at run time (Sec. 4.1, online reveal;
 * Sec. 5.1, the horizon is refreshed at every reveal).  The graph lives
 * in the context.  hx_dag_reserve sizes it (allocates; not for the hot loop)
 * and empties it.  An append propagates with one walk per new node, of any
 * depth; only a walk that is cut short (more than 16 parents waiting at once,
 * or more than 1024 nodes visited) hands over to level-by-level sweeps, of
 * which at most max_depth run: if they do not finish, the stream status gets
 * HX_ERR_CAPACITY.  max_depth = longest path in edges is always enough.
 */
int hx_dag_reserve(hx_ctx *ctx, int32_t max_nodes, int32_t max_edges, int32_t max_wf,
                   int32_t max_depth, void *stream);

/*
 * Appends n_new nodes with ids n_old .. n_old+n_new-1.  New nodes have no
 * successors yet (rem = cost, level 0); tail, level and rem of their
 * ancestors and the horizons of their workflows are raised to what a full
 * recomputation on the grown graph gives, bit for bit.
 *   parent_row_ptr device [n_new+1], parent_row_ptr[0] = 0,
 *                  parent_row_ptr[n_new] = n_new_edges
 *   parent_col_idx device [n_new_edges] parents of each new node; a parent id
 *                  must be smaller than the child's id (else the edge is
 *                  skipped and HX_ERR_NOT_DAG raised in the stream status)
 *   new_cost       device [n_new] >= 0
 *   new_wf         device [n_new] workflow ids, 0 .. max_wf-1
 * HX_ERR_CAPACITY if the reserved store would overflow.
 */
int hx_dag_append(hx_ctx *ctx, int32_t n_new, int32_t n_new_edges,
                  const int32_t *parent_row_ptr, const int32_t *parent_col_idx,
                  const float *new_cost, const int32_t *new_wf, void *stream);

/*
 * Replaces the cost of n nodes of the context's graph (Sec. 5.1: when true
 * service times become available the horizon is corrected by replacing
 * estimates with observed latencies) and recomputes rem, tail and every
 * horizon from the new costs -- a cost may have gone down, so nothing is kept
 * but the levels, which do not depend on costs.  Results equal a full
 * recomputation, bit for bit.
 *   node_ids device [n], 0 .. nodes appended so far - 1 (others are skipped,
 *            HX_ERR_INDEX in the stream status); cost device [n] >= 0.
 * Work grows with the whole graph, not with n: meant for the occasional
 * correction, not for every round.
 */
int hx_dag_set_cost(hx_ctx *ctx, int32_t n, const int32_t *node_ids, const float *cost, void *stream);

/* Borrowed device pointers into the context's graph (valid until the next
 * hx_dag_reserve or hx_ctx_destroy) and the number of nodes appended so far.
 * Any out pointer may be NULL. */
int hx_dag_view(hx_ctx *ctx, const float **rem, const float **tail, const int32_t **level,
                const float **horizon, int32_t *n_nodes);

/* ---- (2) scoring: calls x prefill x decode -> cost tensor or best pair ---- */

/*
 * Evaluates the latency model for every candidate (c, p, d) (Sec. 5.3: all
 * prefill x decode instance pairs, prefill finish plus KV transfer, then the
 * earliest decode finish given decode availability; feasibility per Sec. 5.4
 * Eq. (3),(4) against the KV capacity still free on d):
 *   cost(c,p,d) = max(wait_p + prefill(c,p) + transfer(c,p,d), avail_d)
 *                 + L_out * token_time(c,d)      if used_d + L_in + L_out <= cap_d
 *               = +infinity                      otherwise
 * Fused outputs (no tensor is written): best_p, best_d [C] = the pair of
 * minimum cost, ties to the lowest p*D + d, (-1,-1) when no pair is feasible;
 * best_cost [C]; ratio [C] = (elapsed + best_cost + tail[node]) / horizon[wf]
 * (Eq. (2) with the downstream tail of the call's node; needs tail [n_nodes],
 * horizon [n_wf] and the node/wf/elapsed members of `calls`; a node or
 * workflow index outside those lengths gives NaN and raises HX_ERR_INDEX in
 * the stream status; a workflow whose horizon is 0 gives +infinity).  best_p, best_d, best_cost are
 * all NULL or all non-NULL; ratio may be NULL on its own.
 * Materialised outputs, each may be NULL: cost [C*P*D] row-major (c,p,d) --
 * bit-identical to what the fused search compares; feas [C*D] 1/0.
 * At least one output must be requested.  P or D of 0 gives (-1,-1,+inf).
 */
int hx_score_placements(hx_ctx *ctx, const hx_model *model, const hx_calls *calls,
                        const hx_prefill_tab *prefill, const hx_decode_tab *decode,
                        const hx_links *links,
                        const float *tail, const float *horizon, int32_t n_nodes, int32_t n_wf,
                        float *cost, uint8_t *feas,
                        int32_t *best_p, int32_t *best_d, float *best_cost, float *ratio,
                        void *stream);

/*
 * Debug entry point: element-by-element check of a round's inputs.  The
 * scoring calls check sizes and pointers only and tolerate out-of-range
 * elements without faulting (their results for such elements are
 * unspecified); this call counts them.  report: host [HX_VALIDATE_FIELDS] out,
 * the number of offending elements per category below.  calls->node, wf and
 * elapsed, and links->latency, are checked when not NULL.  Synchronises
 * `stream`.  Returns HX_OK when every count is zero, else HX_ERR_INVALID_ARG
 * with hx_last_error naming the first non-empty category.  Not for the hot
 * loop: it reads every input array once and waits for the result.
 */
enum {
    HX_BAD_L_IN = 0,          /* L_in < 0                                             */
    HX_BAD_L_OUT,             /* L_out < 0                                            */
    HX_BAD_NODE,              /* node outside 0..n_nodes-1                            */
    HX_BAD_WF,                /* wf outside 0..n_wf-1                                 */
    HX_BAD_ELAPSED,           /* elapsed negative, infinite or NaN                    */
    HX_BAD_PREFILL_RATE,      /* prefill flops or hbm_bw not finite and > 0           */
    HX_BAD_PREFILL_BACKLOG,   /* backlog_tok < 0                                      */
    HX_BAD_PREFILL_TYPE,      /* prefill type outside 0..n_types-1                    */
    HX_BAD_DECODE_RATE,       /* decode flops or hbm_bw not finite and > 0            */
    HX_BAD_DECODE_STATE,      /* used_tok, cap_tok, batch or qd_tok < 0               */
    HX_BAD_DECODE_TYPE,       /* decode type outside 0..n_types-1                     */
    HX_BAD_LINK,              /* bw not finite and > 0, latency negative or not finite */
    HX_VALIDATE_FIELDS
};
int hx_validate_round(hx_ctx *ctx, const hx_calls *calls, const hx_prefill_tab *prefill,
                      const hx_decode_tab *decode, const hx_links *links,
                      int32_t n_nodes, int32_t n_wf, int32_t *report, void *stream);

/* ---- (3) select: per-call argmin over a materialised tensor --------------- */

/*
 * best pair of each call from cost [C*P*D] (device, row-major (c,p,d), values
 * >= 0 or +infinity): minimum cost, ties to the lowest flat index p*D + d
 * (Sec. 5.3: a call goes to the pair whose projected decode finish is
 * earliest).  Outputs as in hx_score_placements; `calls`, tail, horizon and
 * ratio may all be NULL when no ratio is wanted.
 */
int hx_select(hx_ctx *ctx, int32_t C, int32_t P, int32_t D, const float *cost,
              const hx_calls *calls, const float *tail, const float *horizon,
              int32_t n_nodes, int32_t n_wf,
              int32_t *best_p, int32_t *best_d, float *best_cost, float *ratio, void *stream);

/* ---- (4) commit the chosen placements into the snapshots ------------------ */

/*
 * The simulated-state update of Algorithm 1, applied once for the whole round:
 * every call with best_p >= 0 adds L_in to backlog_tok[best_p], L_out to
 * qd_tok[best_d] and L_in + L_out to used_tok[best_d]; then each instance
 * drains: backlog = max(0, backlog - drain_prefill), qd = max(0, qd -
 * drain_decode_q), used = max(0, used - release_tok), batch =
 * min(max_batch, ceil(used / tokens_per_seq)).  Integer arithmetic; the
 * result does not depend on the order of the calls.  backlog_tok [P],
 * used_tok, batch, qd_tok [D] are device arrays updated in place; the drain
 * arrays are device inputs or NULL (= 0).  A total above INT32_MAX saturates
 * and raises HX_ERR_OVERFLOW in the stream status; a placement index outside
 * the pool is skipped and raises HX_ERR_INDEX.
 */
int hx_commit(hx_ctx *ctx, const hx_calls *calls, const int32_t *best_p, const int32_t *best_d,
              int32_t P, int32_t *backlog_tok,
              int32_t D, int32_t *used_tok, int32_t *batch, int32_t *qd_tok,
              const int32_t *drain_prefill, const int32_t *drain_decode_q,
              const int32_t *release_tok, int32_t tokens_per_seq, int32_t max_batch,
              void *stream);

/*
 * One scheduling invocation of Algorithm 1 in one call, for callers that pay for
 * every crossing of this boundary: the calls revealed since
 * the last invocation are priced and appended to the context's graph (horizons
 * of the affected workflows refreshed: Sec. 4.1, 5.1), every ready call is
 * projected onto its best feasible (prefill, decode) pair with its ratio
 * (Sec. 5.3, 5.4, Eq. (2)), and the chosen pairs are committed to the pool
 * snapshot (the simulated-state update, once for the round).  The results,
 * argument meaning and error reporting are exactly those of
 *   hx_node_cost(new_L_in, new_L_out -> new_cost); hx_dag_append(new nodes);
 *   hx_score_placements(fused outputs, tail and horizon = the context's graph);
 *   hx_commit(calls, best_p, best_d, the snapshot's counters, the drains)
 * made on `stream` in that order (the first one that fails ends the call; what
 * was enqueued before it stays enqueued), in fewer launches: the new nodes'
 * costs are worked out by the append's first kernel, and -- where every
 * argument check of the calls passes and the search is large enough beside
 * the append -- the append's walks up the graph share the search's launch (the
 * search does not depend on them; only the ratio does) and the ratio is formed
 * by the commit's launch.  n_new may be 0 (nothing is revealed), calls.n may
 * be 0.  The counters of `prefill` and `decode` that
 * the commit updates are passed once more as writable pointers (they may be
 * the same memory as the tables' own backlog_tok, used_tok, batch, qd_tok: the
 * search has read them by then).
 * A round may instead bring its whole graph (n_nodes > 0, n_new = 0; a
 * scheduler that rebuilds the ready workflows' DAGs per invocation): then the
 * reveal is hx_horizons on the arrays given (same requirements on the
 * numbering, same outputs) and the ratio uses their tail and horizon;
 * hx_dag_reserve is needed for the first form only.  Such a round is made in
 * two launches instead of three where every argument check of the three calls
 * passes and the graph's workflows are small enough to be staged 512 nodes at
 * a time: the horizon refresh and the search, which do not depend on each
 * other, share a launch, and the ratio is formed by the commit's launch.  The
 * results are the same bit for bit; in any other case the three calls are made
 * one after the other.
 */
typedef struct {
    /* reveal */
    int32_t n_new, n_new_edges;
    const int32_t *parent_row_ptr;   /* device [n_new+1]                        */
    const int32_t *parent_col_idx;   /* device [n_new_edges]                    */
    const int32_t *new_L_in;         /* device [n_new]                          */
    const int32_t *new_L_out;        /* device [n_new]                          */
    const int32_t *new_wf;           /* device [n_new]                          */
    float         *new_cost;         /* device [n_new] out: standalone costs    */
    int32_t n_types;                 /* classes of type_flops / type_hbm_bw     */
    const float   *type_flops;       /* device [n_types]                        */
    const float   *type_hbm_bw;      /* device [n_types]                        */
    int32_t n_wf;                    /* workflows numbered so far (horizon length used for the ratio) */
    /* reveal, the other form: the whole graph of the round, arguments as hx_horizons (n_nodes > 0 selects it) */
    int32_t n_nodes, n_edges;
    const int32_t *succ_row_ptr;     /* device [n_nodes+1]                      */
    const int32_t *succ_col_idx;     /* device [n_edges]                        */
    const int32_t *wf_ptr;           /* device [n_wf+1]                         */
    const int32_t *node_L_in;        /* device [n_nodes]                        */
    const int32_t *node_L_out;       /* device [n_nodes]                        */
    float   *node_cost, *rem, *tail; /* device [n_nodes] out                    */
    int32_t *level;                  /* device [n_nodes] out                    */
    float   *horizon;                /* device [n_wf] out                       */
    /* search */
    hx_calls        calls;           /* node, wf, elapsed required when ratio != NULL */
    hx_prefill_tab  prefill;
    hx_decode_tab   decode;
    hx_links        links;
    int32_t *best_p, *best_d;        /* device [calls.n] out                    */
    float   *best_cost, *ratio;      /* device [calls.n] out; ratio may be NULL */
    /* commit */
    int32_t *backlog_tok;            /* device [prefill.n], updated in place    */
    int32_t *used_tok, *batch, *qd_tok;   /* device [decode.n], updated in place */
    const int32_t *drain_prefill, *drain_decode_q, *release_tok;   /* device or NULL */
    int32_t tokens_per_seq, max_batch;
} hx_round_args;

int hx_round(hx_ctx *ctx, const hx_model *model, const hx_round_args *round, void *stream);

/*
 * hx_commit for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Takes
 * no context and allocates nothing, now or earlier: the per-round accumulators
 * (one 64-bit word per backlog, used and queue counter, 24 KB) are a static
 * device array inside the library, one copy per GPU, held until the process
 * ends.  Same arguments, arithmetic and results as hx_commit, on the current
 * HIP device; P and D at most HX_MAX_INSTANCES (HX_ERR_SHAPE beyond, nothing
 * launched).  status: device int32 or NULL; takes the first HX_ERR_INDEX /
 * HX_ERR_OVERFLOW a kernel raises if it holds 0 (the caller clears and reads
 * it); with NULL such conditions go unreported (the elements are still
 * skipped or saturated).  Launches three kernels on `stream` (the first clears
 * the accumulators: they keep what the last call left) and no memset or copy.
 * All calls on one GPU share the one array: calls that overlap in time on that
 * GPU (two streams, two threads) race; calls in stream order do not.  The text
 * of a failure is returned by hx_last_error(NULL).
 */
int hx_commit_static(const hx_calls *calls, const int32_t *best_p, const int32_t *best_d,
                     int32_t P, int32_t *backlog_tok,
                     int32_t D, int32_t *used_tok, int32_t *batch, int32_t *qd_tok,
                     const int32_t *drain_prefill, const int32_t *drain_decode_q,
                     const int32_t *release_tok, int32_t tokens_per_seq, int32_t max_batch,
                     int32_t *status, void *stream);

/*
 * The urgency fold on its own (Eq. (2) with the downstream tail of the call's
 * node): ratio[c] = (elapsed[c] + best_cost[c] + tail[node[c]]) / horizon[wf[c]],
 * the same arithmetic as the ratio output of hx_score_placements and hx_select.
 * For callers that run the search (which needs no horizon) on one stream while
 * the horizons of the round are still being refreshed on another, and fold
 * them in afterwards.  calls->node, wf, elapsed, best_cost, ratio: device [C];
 * a node or workflow outside 0..n_nodes-1 / 0..n_wf-1 gives NaN and raises
 * HX_ERR_INDEX in the stream status; a horizon of 0 gives +infinity (Eq. (2)
 * is undefined there: such a call counts as most urgent).
 */
int hx_urgency(hx_ctx *ctx, const hx_calls *calls, const float *best_cost,
               const float *tail, const float *horizon, int32_t n_nodes, int32_t n_wf,
               float *ratio, void *stream);

/* ---- (5) the planner around the scoring loop ------------------------------- */

/*
 * One-pass ordering for larger queues (Sec. 5.3: calls are ordered once by the
 * same risk score): rank[c] = position of call c when the calls are sorted by
 * decreasing ratio, equal ratios by increasing call index (0 = most urgent).
 * ratio [C] device in (as written by hx_score_placements or hx_select; +inf =
 * nothing feasible, ranked first), rank [C] device out.  Up to 16384 calls every
 * call is compared with every call (no scratch).  Beyond that the calls are
 * split into 257 buckets by 256 sampled splitters and compared within their
 * bucket; the library then keeps 8 bytes of scratch per call, and a call with a
 * larger C than any before it allocates, after waiting for the device, and is
 * then not capturable in a graph.
 */
int hx_rank(hx_ctx *ctx, int32_t C, const float *ratio, int32_t *rank, void *stream);

/*
 * Recomputing greedy for small queues (the main loop of Algorithm 1; Sec. 5.3):
 * repeat C times -- score every remaining call on a simulated copy of the pool
 * state, take the call of largest projected ratio (equal ratios: lowest call
 * index), record its pair, cost, ratio and rank (0 = first), and add it to the
 * simulated state: backlog_tok[p] += L_in, qd_tok[d] += L_out, used_tok[d] +=
 * L_in + L_out, batch[d] = min(max_batch, ceil(used_tok[d] / tokens_per_seq)).
 * A call with no feasible pair has ratio +inf: it is ranked at once, keeps
 * (-1, -1) and changes nothing.  Inputs as in hx_score_placements (tail,
 * horizon and the node/wf/elapsed members of `calls` are required; the pool
 * tables are read only).  Outputs [C]: best_p, best_d, best_cost, ratio as of
 * the moment the call was picked, and rank.  backlog_tok_out [P], used_tok_out,
 * batch_out, qd_tok_out [D] receive the simulated state the plan leaves; each
 * may be NULL.  At most HX_GREEDY_MAX_CALLS calls and HX_GREEDY_MAX_INSTANCES
 * instances per side (HX_ERR_SHAPE beyond): the whole loop runs in one
 * workgroup with no launch between iterations.
 */
int hx_plan_greedy(hx_ctx *ctx, const hx_model *model, const hx_calls *calls,
                   const hx_prefill_tab *prefill, const hx_decode_tab *decode, const hx_links *links,
                   const float *tail, const float *horizon, int32_t n_nodes, int32_t n_wf,
                   int32_t tokens_per_seq, int32_t max_batch,
                   int32_t *best_p, int32_t *best_d, float *best_cost, float *ratio, int32_t *rank,
                   int32_t *backlog_tok_out, int32_t *used_tok_out, int32_t *batch_out, int32_t *qd_tok_out,
                   void *stream);

/* ---- (6) the decode stage (Sec. 5.4) ---------------------------------------- */

/*
 * Decode token-capacity intervals (Sec. 5.4 "simulated decode intervals"; Sec. 6:
 * the estimator keeps decode token-capacity intervals per instance).  Instance d
 * owns entries d*stride .. d*stride + count[d] - 1; entry j says that tok[j] KV
 * tokens are held on start[j] <= t < end[j], seconds from now (resident
 * sequences have start <= 0, planned ones start later).  An entry with
 * start >= end or tok <= 0 holds nothing.  All arrays are device memory owned by
 * the caller; hx_decode_score only reads them, hx_decode_plan_greedy appends.
 */
typedef struct {
    int32_t  stride;   /* entries reserved per instance, 0..HX_MAX_INTERVALS     */
    int32_t *count;    /* device [D] entries in use, 0..stride                   */
    float   *start;    /* device [D*stride]                                      */
    float   *end;      /* device [D*stride]                                      */
    int32_t *tok;      /* device [D*stride]                                      */
} hx_intervals;

/*
 * Decode-stage scoring of a queue of calls whose KV has arrived (Sec. 5.4;
 * Sec. 5.1: for decode scheduling the projection is waiting for decode capacity
 * plus decode execution on the candidate instance).  For call c and instance d
 *   T(c,d)  = L_out * per-token decode time on d's snapshot (batch, used_tok),
 *   S(c,d)  = the earliest t >= 0 such that the intervals of d leave room for
 *             L_in + L_out more tokens (Eq. 3) under cap_tok[d] (Eq. 4) at every
 *             instant of [t, t + T); it is 0 or the end of one of d's entries;
 *             +inf when L_in + L_out > cap_tok[d].  The window is half open and
 *             t + T is formed and compared in fp32: a call fits exactly between
 *             two entries when fl(t + T) equals the next entry's start,
 *   cost    = S + T.
 * lock [Q] device or NULL: lock[c] = d restricts call c to instance d (a call
 * locked during prefill planning cannot migrate), -1 leaves it free; any other
 * value raises HX_ERR_INDEX in the status word and the call gets no instance.
 * Per call the result is the lexicographic minimum of (cost, d) over its legal
 * instances: best_d (-1 if none), best_start, best_cost (+inf if none) and,
 * when ratio != NULL, ratio = (elapsed + best_cost + tail[node]) / horizon[wf]
 * (Eq. 2 at the decode stage; needs the node/wf/elapsed members of `queue`,
 * tail and horizon).  start, cost: device [Q*D] row-major or NULL, every pair
 * (+inf for an instance the lock excludes).  decode->qd_tok and decode->type are
 * not read.  The library keeps scratch for this call: per instance its sorted
 * timeline and what is derived from it (about 60 bytes per interval, and a
 * 16 KiB search table), per call a place in the list of free calls and the
 * best candidate within each of up to 64 groups of instances (12 bytes per
 * group).  A call with a larger Q, D or D * stride than any before it
 * allocates, after waiting for the device, and is then not capturable in a
 * graph.  The selection uses no atomics: results do not depend on timing.
 */
int hx_decode_score(hx_ctx *ctx, const hx_model *model, const hx_calls *queue, const int32_t *lock,
                    const hx_decode_tab *decode, const hx_intervals *intervals,
                    const float *tail, const float *horizon, int32_t n_nodes, int32_t n_wf,
                    float *start, float *cost,
                    int32_t *best_d, float *best_start, float *best_cost, float *ratio, void *stream);

/*
 * Recomputing greedy of the decode stage for small queues (Sec. 5.4 "Adaptive
 * greedy decode assignment"): repeat Q times -- score every remaining call as
 * hx_decode_score does, on the simulated intervals; take the call of largest
 * ratio (equal ratios: lowest index); record its instance, start, finish
 * (best_cost), ratio and rank (0 = first); append (start, finish, L_in + L_out)
 * to that instance's entries and count[d] += 1.  A call with no feasible legal
 * instance has ratio +inf: it is ranked at once with (-1, +inf) and changes
 * nothing.  If an instance's list is full the status word gets HX_ERR_CAPACITY
 * and that entry is not appended.  Only the intervals are simulated: the
 * per-token time keeps the snapshot's batch and used_tok.  At most
 * HX_DECODE_GREEDY_MAX_CALLS calls, and D * (2*stride + 1) must fit the
 * workgroup's local memory (HX_ERR_SHAPE otherwise; e.g. 64 instances x 90
 * entries, 16 x 370): the whole loop is one workgroup with no launch between
 * iterations.  Larger queues: hx_decode_score once, then hx_rank.
 */
int hx_decode_plan_greedy(hx_ctx *ctx, const hx_model *model, const hx_calls *queue, const int32_t *lock,
                          const hx_decode_tab *decode, const hx_intervals *intervals,
                          const float *tail, const float *horizon, int32_t n_nodes, int32_t n_wf,
                          int32_t *best_d, float *best_start, float *best_cost, float *ratio, int32_t *rank,
                          void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HX_H */
