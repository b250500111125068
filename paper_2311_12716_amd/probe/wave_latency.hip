// Measurement code, not part of the product: what one wave on an otherwise idle compute unit pays
// per instruction.  `bench.py --wave-latency` runs it; the rollout's dynamics stage is one such
// wave whose step-to-step chain bounds small launches, and these figures are what that chain is
// made of.  Each test runs a loop of N iterations on one wave and reports shader clocks
// (s_memtime) and nanoseconds (the constant-rate clock) per iteration.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace {

constexpr int N = 4096;
constexpr int TESTS = 6;

// opaque to the optimiser: keeps a dependent chain a chain
#define KEEP(x) asm volatile("" : "+v"(x))

__global__ __launch_bounds__(64) void k_wave_latency(uint64_t *out, uint32_t seed)
{
    __shared__ uint32_t lds[1024];
    const int lane = threadIdx.x;
    for (int i = lane; i < 1024; i += 64) lds[i] = (i + 64) & 1023;      // lane-private chains of indices
    __syncthreads();
    uint64_t clk[TESTS], ns[TESTS];
    uint32_t x = seed + lane, y = seed * 3 + lane, z = lane | 1, w = 7 + lane, p = lane;
    uint64_t c0, t0;
#define BEGIN c0 = clock64(); t0 = wall_clock64();
#define END(j) clk[j] = clock64() - c0; ns[j] = (wall_clock64() - t0) * 10;
    // 0: one add that needs the previous add's result
    BEGIN
#pragma unroll 16
    for (int i = 0; i < N; ++i) { x = x + z; KEEP(x); }
    END(0)
    // 1: four adds that do not depend on each other
    BEGIN
#pragma unroll 4
    for (int i = 0; i < N; ++i) { x += 3; y += 5; z += 7; w += 9; KEEP(x); KEEP(y); KEEP(z); KEEP(w); }
    END(1)
    // 2: an LDS read whose address is the previous read's result
    BEGIN
#pragma unroll 8
    for (int i = 0; i < N; ++i) p = lds[p];
    END(2)
    // 3: compare -> select on the compare's mask -> add, each needing the one before
    BEGIN
#pragma unroll 16
    for (int i = 0; i < N; ++i) { x = (x > y) ? z : x + 1; KEEP(x); }
    END(3)
    // 4: two compares, the masks combined on the scalar unit, then the select
    BEGIN
#pragma unroll 16
    for (int i = 0; i < N; ++i) { const bool a = x > y, b = x != w; x = (a & b) ? z : x + 1; KEEP(x); }
    END(4)
    // 5: an LDS write followed by a read of the same address
    BEGIN
#pragma unroll 8
    for (int i = 0; i < N; ++i) { lds[lane] = p; asm volatile("" ::: "memory"); p = lds[lane] + 1; }
    END(5)
    if (lane == 0)
        for (int j = 0; j < TESTS; ++j) { out[2 * j] = clk[j]; out[2 * j + 1] = ns[j]; }
    if (x + y + z + w + p == 0x12345u) out[2 * TESTS] = 1;               // keeps the results alive
}

}  // namespace

// d_out: device buffer of 13 uint64: per test the shader clocks and the nanoseconds of its
// 4096 iterations (tests: dependent add, four independent adds, dependent LDS read,
// compare-select-add chain, two compares + scalar and + select chain, LDS write then read).
// Returns 0, or -1 without a buffer.
extern "C" int waveprobe_run(uint64_t *d_out, void *stream)
{
    if (!d_out) return -1;
    hipLaunchKernelGGL(k_wave_latency, dim3(1), dim3(64), 0, (hipStream_t)stream, d_out, 1u);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

extern "C" int waveprobe_iterations(void) { return N; }
