// fp32 latency terms of the estimator, as device functions shared by every
// scoring kernel so that the fused search, the materialised tensor and the
// per-node standalone cost round identically.
//
// The paper names the terms (Sec. 4.2 "Scheduler internals": prefill time,
// decode time, KV-transfer latency, decode memory demand from a roofline-style
// model; Sec. 4.2 "Heterogeneous resource modelling": single-server prefill
// queue, batched decode under a KV limit, KV size over class-pair bandwidth)
// and prints no formula; each term below is the plain roofline form
// time = max(compute-bound, bandwidth-bound).
//
// All files including this header are compiled with -ffp-contract=off; every
// fused multiply-add is written out as fmaf so the rounding sequence is fixed.
#pragma once

#include <hip/hip_runtime.h>

struct HxModelF {
    float kappa;   // KV bytes per token
    float phi;     // FLOP per token
    float attn;    // FLOP per token^2
    float omega;   // weight bytes
    float bbar;    // nominal decode batch
};

// ---- per prefill instance (once per round) ----------------------------------

// queue of a single-server prefill instance: backlog_tok * phi / F
__device__ __forceinline__ float hx_prefill_wait(const HxModelF &m, int backlog_tok, float invF)
{
    return ((float)backlog_tok * m.phi) * invF;
}

// ---- per call ---------------------------------------------------------------

struct HxCallF {
    float L, O;
    float comp;      // phi*L + a*L^2   [FLOP]
    float mem;       // omega + kappa*L [B]
    float kvL;       // kappa*L         [B]   KV size to transfer
    float ctx;       // L + O/2         [tok] own context averaged over the generation
};

__device__ __forceinline__ HxCallF hx_call_terms(const HxModelF &m, int L_in, int L_out)
{
    HxCallF c;
    c.L = (float)L_in;
    c.O = (float)L_out;
    c.comp = fmaf(m.attn * c.L, c.L, m.phi * c.L);
    c.mem = fmaf(m.kappa, c.L, m.omega);
    c.kvL = m.kappa * c.L;
    c.ctx = fmaf(0.5f, c.O, c.L);
    return c;
}

// ---- per (call, prefill instance) -------------------------------------------

// prefill wait + roofline prefill service time
__device__ __forceinline__ float hx_prefill_done(const HxCallF &c, float wait, float invF, float invB)
{
    return wait + fmaxf(c.comp * invF, c.mem * invB);
}

// ---- per (call, prefill class, decode class) ----------------------------------

// KV size over the effective bandwidth between the two classes (+ latency)
__device__ __forceinline__ float hx_transfer(const HxCallF &c, float inv_bw, float lat)
{
    return fmaf(c.kvL, inv_bw, lat);
}

// ---- per decode instance (once per round) -------------------------------------

struct HxDecF {
    float wait;   // availability hint: qd_tok * step / Bbar
    float c1;     // phi*(batch+1)/F          compute-bound time per token
    float c2;     // (omega + kappa*used)/B   bandwidth-bound time per token before the call's own context
    float kB;     // kappa/B
};

__device__ __forceinline__ HxDecF hx_decode_terms(const HxModelF &m, int used_tok, int batch, int qd_tok,
                                                  float invF, float invB)
{
    HxDecF d;
    float resident = fmaf(m.kappa, (float)used_tok, m.omega) * invB;
    float step = fmaxf((m.phi * (float)batch) * invF, resident);
    d.wait = ((float)qd_tok * step) / m.bbar;
    d.c1 = (m.phi * ((float)batch + 1.0f)) * invF;
    d.c2 = resident;
    d.kB = m.kappa * invB;
    return d;
}

// ---- per (call, decode instance) -----------------------------------------------

// decode execution time L_out * per-token time, or +inf when the call does not
// fit the KV capacity still free (Sec. 5.4 Eq. (3),(4): demand L_in + L_out)
__device__ __forceinline__ bool hx_fits(int L_in, int L_out, int free_tok)
{
    // both lengths are >= 0, so the unsigned sum cannot wrap
    return free_tok >= 0 && ((unsigned)L_in + (unsigned)L_out) <= (unsigned)free_tok;
}

__device__ __forceinline__ float hx_decode_time(const HxCallF &c, float c1, float c2, float kB)
{
    return c.O * fmaxf(c1, fmaf(kB, c.ctx, c2));
}

// ---- per candidate ---------------------------------------------------------------

// projected decode finish: decode starts when both the KV has arrived and the
// instance is available (Sec. 5.3)
__device__ __forceinline__ float hx_candidate(float ready, float dec_wait, float dec_time)
{
    return fmaxf(ready, dec_wait) + dec_time;
}
