// Sustained vector-ALU issue rate of the GPU, measured: the denominator bench.py prints
// beside the paper figure of 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz.  Not part of libjsv:
// built into libjsv_probe.so and loaded by bench.py --peak-probe only.
//
// Every lane runs eight independent chains of one instruction, 64 instructions per loop
// iteration, nothing else but the scalar loop counter; inline asm keeps the compiler from
// folding the chains into a closed form.  Lane-operations per second = lanes x iterations
// x 64 / kernel time (HIP events, best of `repeats`).
//
// Four instructions, because they do not issue at one rate on this chip: v_add_u32 (like
// v_and_b32, v_xor_b32, v_mov_b32 with register or constant operands) goes through at about
// 2.4 cycles per wave64 instruction and SIMD, while v_min_u32 and v_cmp_le_u32 - the two
// instructions the enumeration spends per candidate - and v_fma_f64 take about 4.2 and 4.7.
// The enumeration's roofline is therefore the v_min_u32 / v_cmp figure, not the v_add_u32 one.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr int CHAINS = 8;
constexpr int UNROLL = 8;      // CHAINS * UNROLL = 64 vector instructions per iteration

__global__ void __launch_bounds__(256) probe_add_u32(uint32_t iters, uint32_t* sink)
{
    const uint32_t x = threadIdx.x * 2654435761u + blockIdx.x + 1u;
    uint32_t a[CHAINS];
#pragma unroll
    for (int c = 0; c < CHAINS; ++c) a[c] = x + c;
    for (uint32_t i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
#pragma unroll
            for (int c = 0; c < CHAINS; ++c)
                asm volatile("v_add_u32_e32 %0, %1, %0" : "+v"(a[c]) : "v"(x));
    }
    uint32_t r = 0;
#pragma unroll
    for (int c = 0; c < CHAINS; ++c) r ^= a[c];
    sink[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

__global__ void __launch_bounds__(256) probe_fma_f64(uint32_t iters, uint32_t* sink)
{
    const double x = 1.0 + 1e-9 * (double)(threadIdx.x + 1u);
    const double y = 1e-12 * (double)(blockIdx.x + 1u);
    double a[CHAINS];
#pragma unroll
    for (int c = 0; c < CHAINS; ++c) a[c] = 0.5 + 0.01 * c;
    for (uint32_t i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
#pragma unroll
            for (int c = 0; c < CHAINS; ++c)
                asm volatile("v_fma_f64 %0, %0, %1, %2" : "+v"(a[c]) : "v"(x), "v"(y));
    }
    double r = 0.0;
#pragma unroll
    for (int c = 0; c < CHAINS; ++c) r += a[c];
    sink[blockIdx.x * blockDim.x + threadIdx.x] = (uint32_t)__double2loint(r);
}

__global__ void __launch_bounds__(256) probe_min_u32(uint32_t iters, uint32_t* sink)
{
    const uint32_t x = threadIdx.x * 2654435761u + blockIdx.x + 1u;
    uint32_t a[CHAINS];
#pragma unroll
    for (int c = 0; c < CHAINS; ++c) a[c] = ~x + c;
    for (uint32_t i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
#pragma unroll
            for (int c = 0; c < CHAINS; ++c)
                asm volatile("v_min_u32_e32 %0, %1, %0" : "+v"(a[c]) : "v"(x));
    }
    uint32_t r = 0;
#pragma unroll
    for (int c = 0; c < CHAINS; ++c) r ^= a[c];
    sink[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

__global__ void __launch_bounds__(256) probe_cmp_u32(uint32_t iters, uint32_t* sink)
{
    const uint32_t x = threadIdx.x * 2654435761u + blockIdx.x + 1u;
    uint32_t a[CHAINS];
#pragma unroll
    for (int c = 0; c < CHAINS; ++c) a[c] = x + c;
    for (uint32_t i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
#pragma unroll
            for (int c = 0; c < CHAINS; ++c)
                asm volatile("v_cmp_le_u32_e32 vcc, %0, %1" : : "v"(a[c]), "v"(x) : "vcc");
    }
    uint32_t r = 0;
#pragma unroll
    for (int c = 0; c < CHAINS; ++c) r ^= a[c];
    sink[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

}  // namespace

// kind 0: v_add_u32, kind 1: v_fma_f64, kind 2: v_min_u32, kind 3: v_cmp_le_u32.  blocks x 256 lanes, `iters` iterations of 64
// instructions each, `repeats` launches on the default stream of the current device.
// Outputs: seconds of the fastest launch, lane-operations of one launch.  Returns a hipError_t.
extern "C" __attribute__((visibility("default")))
int jsv_probe_valu(int kind, uint32_t blocks, uint32_t iters, int repeats, double* best_seconds, double* lane_ops)
{
    if (!best_seconds || !lane_ops || blocks == 0 || repeats < 1 || kind < 0 || kind > 3) return (int)hipErrorInvalidValue;
    uint32_t* sink = nullptr;
    hipError_t e = hipMalloc(&sink, (size_t)blocks * 256 * sizeof(uint32_t));
    if (e != hipSuccess) return (int)e;
    hipEvent_t t0 = nullptr, t1 = nullptr;
    e = hipEventCreate(&t0);
    if (e == hipSuccess) e = hipEventCreate(&t1);
    float best = 0.f;
    for (int r = 0; r <= repeats && e == hipSuccess; ++r) {        // launch 0 warms up
        e = hipEventRecord(t0, nullptr);
        if (kind == 0) hipLaunchKernelGGL(probe_add_u32, dim3(blocks), dim3(256), 0, nullptr, iters, sink);
        else if (kind == 1) hipLaunchKernelGGL(probe_fma_f64, dim3(blocks), dim3(256), 0, nullptr, iters, sink);
        else if (kind == 2) hipLaunchKernelGGL(probe_min_u32, dim3(blocks), dim3(256), 0, nullptr, iters, sink);
        else hipLaunchKernelGGL(probe_cmp_u32, dim3(blocks), dim3(256), 0, nullptr, iters, sink);
        if (e == hipSuccess) e = hipGetLastError();
        if (e == hipSuccess) e = hipEventRecord(t1, nullptr);
        if (e == hipSuccess) e = hipEventSynchronize(t1);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, t0, t1);
        if (r >= 1 && (best == 0.f || ms < best)) best = ms;
    }
    if (t0) (void)hipEventDestroy(t0);
    if (t1) (void)hipEventDestroy(t1);
    (void)hipFree(sink);
    *best_seconds = best * 1e-3;
    *lane_ops = (double)blocks * 256.0 * (double)iters * (double)(CHAINS * UNROLL);
    return (int)e;
}
