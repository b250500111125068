// Store-pattern probe: measurement code of bench.py (--store-patterns), not part of the product
// library.  It writes an output buffer of the rollout's size in the rollout's pattern with
// nothing else going on -- no dynamics, no LDS, constants as data -- so that what the memory
// system does with the pattern can be told apart from what the kernels add, and hardware
// counters can be read per pattern (each variant is a kernel of its own name).
//
//   k_probe_fill            one-shot: every workgroup fills 4 KB, the whole buffer once
//   k_probe_slab<NT, PACED> persistent: `workgroups` workgroups, each writing its chunk
//                           (bytes_per_step / workgroups, a multiple of 16) of every step's slab,
//                           10 store waves, one barrier per 8 steps -- the store stage of the
//                           student rollout.  NT: streaming stores (sc0 sc1 nt) instead of plain
//                           ones.  PACED: sleep_units of s_sleep 1 after each step's store.
//   k_probe_contiguous      persistent, the same chunks, but a workgroup's steps back to back in
//                           memory (the layout [N][T][...] the interface does not have): shows
//                           that the slab stride is not what costs.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace {

typedef uint32_t u4 __attribute__((ext_vector_type(4)));
constexpr int STORE_WAVES = 10, STEPS_PER_BARRIER = 8;

// The data registers of every store here hold one constant that is never rewritten, so the
// assembly form needs no more than its own wait states after it.
template <int NT>
__device__ __forceinline__ void put(char *p, u4 v)
{
    if (NT) asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
    else *(u4 *)p = v;
}

__global__ __launch_bounds__(256) void k_probe_fill(u4 *p, size_t pieces)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const u4 v = {1, 2, 3, 4};
    if (i < pieces) p[i] = v;
}

template <int NT, int PACED>
__global__ __launch_bounds__(64 * STORE_WAVES) void k_probe_slab(char *p, int steps, size_t slab, int chunk,
                                                                 int sleep_units)
{
    const u4 v = {1, 2, 3, 4};
    char *base = p + (size_t)blockIdx.x * chunk;
    for (int s0 = 0; s0 < steps; s0 += STEPS_PER_BARRIER) {
        for (int u = 0; u < STEPS_PER_BARRIER && s0 + u < steps; ++u) {
            for (int off = (int)threadIdx.x * 16; off < chunk; off += 64 * STORE_WAVES * 16)
                put<NT>(base + (size_t)u * slab + off, v);
            if (PACED)
                for (int q = 0; q < sleep_units; ++q) __builtin_amdgcn_s_sleep(1);
        }
        base += (size_t)STEPS_PER_BARRIER * slab;
        __syncthreads();
    }
}

__global__ __launch_bounds__(64 * STORE_WAVES) void k_probe_contiguous(char *p, int steps, int chunk)
{
    const u4 v = {1, 2, 3, 4};
    char *base = p + (size_t)blockIdx.x * chunk * steps;
    for (int s0 = 0; s0 < steps; s0 += STEPS_PER_BARRIER) {
        for (int u = 0; u < STEPS_PER_BARRIER && s0 + u < steps; ++u)
            for (int off = (int)threadIdx.x * 16; off < chunk; off += 64 * STORE_WAVES * 16)
                put<0>(base + (size_t)u * chunk + off, v);
        base += (size_t)STEPS_PER_BARRIER * chunk;
        __syncthreads();
    }
}

}  // namespace

// pattern 0 fill, 1 slab with plain stores, 2 slab with streaming stores, 3 contiguous per
// workgroup.  d_buf: device buffer of steps * bytes_per_step bytes, 16-byte aligned;
// bytes_per_step a multiple of 16 * workgroups.  Returns 0, or -1 for arguments out of range.
extern "C" int storeprobe_run(int pattern, void *d_buf, size_t bytes_per_step, int workgroups, int steps,
                              int sleep_units, void *stream)
{
    if (!d_buf || workgroups < 1 || steps < 1 || sleep_units < 0 || sleep_units > 4096) return -1;
    if (bytes_per_step == 0 || bytes_per_step % ((size_t)16 * workgroups) != 0 || ((uintptr_t)d_buf & 15)) return -1;
    const size_t chunk = bytes_per_step / workgroups;
    if (chunk > (1u << 30)) return -1;
    hipStream_t st = (hipStream_t)stream;
    char *p = (char *)d_buf;
    const dim3 block(64 * STORE_WAVES);
    switch (pattern) {
    case 0: {
        const size_t pieces = bytes_per_step * steps / 16;
        hipLaunchKernelGGL(k_probe_fill, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, st, (u4 *)p, pieces);
        break;
    }
    case 1:
        if (sleep_units) hipLaunchKernelGGL((k_probe_slab<0, 1>), dim3(workgroups), block, 0, st, p, steps, bytes_per_step, (int)chunk, sleep_units);
        else hipLaunchKernelGGL((k_probe_slab<0, 0>), dim3(workgroups), block, 0, st, p, steps, bytes_per_step, (int)chunk, 0);
        break;
    case 2:
        if (sleep_units) hipLaunchKernelGGL((k_probe_slab<1, 1>), dim3(workgroups), block, 0, st, p, steps, bytes_per_step, (int)chunk, sleep_units);
        else hipLaunchKernelGGL((k_probe_slab<1, 0>), dim3(workgroups), block, 0, st, p, steps, bytes_per_step, (int)chunk, 0);
        break;
    case 3:
        hipLaunchKernelGGL(k_probe_contiguous, dim3(workgroups), block, 0, st, p, steps, (int)chunk);
        break;
    default: return -1;
    }
    return hipGetLastError() == hipSuccess ? 0 : -4;
}
