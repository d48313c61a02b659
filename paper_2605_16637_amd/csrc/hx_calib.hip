// Benchmark-only calibration kernels, built into their own small library (not part of the placement
// search and not declared in hx.h):
//   hx_calib_valu    streams of plain fp32 vector instructions (no memory, no packed or fused forms) of known
//                    length per lane, to measure the rate at which the chip issues each kind under load;
//   hx_calib_search  the arithmetic of the fused search's inner loop on registers alone -- the ceiling that
//                    kernel is held against;
//   hx_calib_copy  a plain device copy of known size, the reference for HBM byte counters and for what a
//                  launch of a given size can reach.
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

namespace {

constexpr int CALIB_THREADS = 256;

#define HX_VMAX(d, a, b) asm volatile("v_max_f32 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b))
#define HX_VADD(d, a, b) asm volatile("v_add_f32 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b))
#define HX_VMIN3(d, a, b, c) asm volatile("v_min3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c))

// One iteration = 32 instructions per lane on 16 independent registers.
// MIX 0: v_max_f32 only.   MIX 1: v_add_f32 only.   MIX 2: v_max_f32 and v_add_f32 alternating.
template <int MIX>
__global__ __launch_bounds__(CALIB_THREADS) void hx_calib_valu_kernel(float *sink, int iters, float a, float b)
{
    float x[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) x[j] = (float)(threadIdx.x + j);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            if (MIX == 0) { HX_VMAX(x[j], x[j], a); }
            else if (MIX == 1) { HX_VADD(x[j], x[j], b); }
            else if (j & 1) { HX_VADD(x[j], x[j], b); }
            else { HX_VMAX(x[j], x[j], a); }
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            if (MIX == 0) { HX_VMAX(x[j], x[j], b); }
            else if (MIX == 1) { HX_VADD(x[j], x[j], a); }
            else if (j & 1) { HX_VMAX(x[j], x[j], a); }
            else { HX_VADD(x[j], x[j], b); }
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < 16; ++j) s += x[j];
    sink[(size_t)blockIdx.x * CALIB_THREADS + threadIdx.x] = s;
}

// The arithmetic of the search's inner loop on registers alone: per iteration 8 decode entries x 4 prefill
// slots = 32 candidates per lane, each t = max(ready, avail) + dec folded into a running minimum with
// three-input minima: 32 v_max_f32, 32 v_add_f32, 16 v_min3_f32, the additions and minima of one slot
// placed between the maxima of the next.  No memory, no per-call work.
__global__ __launch_bounds__(CALIB_THREADS) void hx_calib_search_kernel(float *sink, int iters, float a0, float d0)
{
    float r[4], best[4], av[8], dv[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) { r[j] = (float)(threadIdx.x + j); best[j] = 1e30f; }
#pragma unroll
    for (int e = 0; e < 8; ++e) { av[e] = a0 + (float)e; dv[e] = d0 + (float)e; }
    for (int it = 0; it < iters; ++it) {
        float t[4][8], m1[4], m2[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
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
        HX_VMIN3(best[3], best[3], t[3][0], t[3][1]);
        HX_VMIN3(m1[3], t[3][2], t[3][3], t[3][4]);
        HX_VMIN3(m2[3], t[3][5], t[3][6], t[3][7]);
        HX_VMIN3(best[3], best[3], m1[3], m2[3]);
    }
    sink[(size_t)blockIdx.x * CALIB_THREADS + threadIdx.x] = (best[0] + best[1]) + (best[2] + best[3]);
}

__global__ __launch_bounds__(256) void hx_calib_copy_kernel(const float4 *__restrict__ src, float4 *__restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace

// Enqueues an instruction stream on `stream`: blocks x 256 lanes, `iters` iterations of 32 instructions per
// lane; mix 0 = v_max_f32 only, 1 = v_add_f32 only, 2 = the two alternating.
// sink: device [blocks * 256] floats.  Returns 0, or -1 for a bad argument, -5 if the launch failed.
extern "C" int hx_calib_valu(int blocks, int iters, int mix, float *sink, void *stream)
{
    if (blocks <= 0 || iters < 0 || !sink || mix < 0 || mix > 2) return -1;
    hipStream_t st = (hipStream_t)stream;
    if (mix == 0) hx_calib_valu_kernel<0><<<blocks, CALIB_THREADS, 0, st>>>(sink, iters, 1.0f, 0.25f);
    else if (mix == 1) hx_calib_valu_kernel<1><<<blocks, CALIB_THREADS, 0, st>>>(sink, iters, 1.0f, 0.25f);
    else hx_calib_valu_kernel<2><<<blocks, CALIB_THREADS, 0, st>>>(sink, iters, 1.0f, 0.25f);
    return hipGetLastError() == hipSuccess ? 0 : -5;
}

// Enqueues the search loop's arithmetic on registers: blocks x 256 lanes, `iters` iterations of 32 candidates
// per lane (32 v_max_f32 + 32 v_add_f32 + 16 v_min3_f32).  sink as above.
extern "C" int hx_calib_search(int blocks, int iters, float *sink, void *stream)
{
    if (blocks <= 0 || iters < 0 || !sink) return -1;
    hx_calib_search_kernel<<<blocks, CALIB_THREADS, 0, (hipStream_t)stream>>>(sink, iters, 1.0f, 0.25f);
    return hipGetLastError() == hipSuccess ? 0 : -5;
}

// Enqueues a copy of n16 16-byte words from src to dst (device, 16-byte aligned) with `blocks` workgroups.
extern "C" int hx_calib_copy(const void *src, void *dst, size_t n16, int blocks, void *stream)
{
    if (!src || !dst || blocks <= 0) return -1;
    hx_calib_copy_kernel<<<blocks, 256, 0, (hipStream_t)stream>>>((const float4 *)src, (float4 *)dst, n16);
    return hipGetLastError() == hipSuccess ? 0 : -5;
}
