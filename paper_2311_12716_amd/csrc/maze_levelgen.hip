// Levels made on the device: the random level generator, level mutations and the
// level setter of the teacher editor env.
//
// Random numbers come from a counter-based generator (Philox-4x32, 10 rounds: Salmon,
// Moraes, Dror, Shaw, SC'11): key = seed, counter = (level id low, level id high,
// draw index / 4, purpose), draw `index` = output word index % 4; purpose 0 =
// generation, 1 = mutation.  A level's draws therefore depend on its id alone, not on
// the batch or the GPU it is drawn on.  A draw u becomes a cell index as
// floor(u * cells / 2^32).
#include "maze_internal.h"
#include "maze_editor_device.h"

namespace {

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;       // round multipliers
    constexpr uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;       // key increments
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
        const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += W0;
        k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

__device__ __forceinline__ int draw_below(uint32_t u, int n) { return (int)__umulhi(u, (uint32_t)n); }

enum { GENERATE = 0, MUTATE = 1 };

// One lane per env; the envs' bit streams are edited in LDS (stride odd: lanes hit
// different banks) and copied in and out of global memory by the whole workgroup.
// EPB = envs per workgroup (at most 64, fewer when the streams are long).
template <int MODE>
__global__ __launch_bounds__(64) void k_levelgen(EditorDev p, int EPB, uint32_t seed_lo, uint32_t seed_hi,
                                                 uint64_t first_id, int n_edits)
{
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x;
    const int env0 = blockIdx.x * EPB;
    const int count = min(EPB, p.N - env0);
    const int SW = p.SW, stride = SW | 1;
    for (int i = lane; i < count * SW; i += 64) {
        const int e = i / SW, o = i - e * SW;
        lds[e * stride + o] = (MODE == MUTATE) ? p.stream[(size_t)(env0 + e) * SW + o] : 0u;
    }
    __syncthreads();
    if (lane < count) {
        const int n = env0 + lane;
        uint32_t *s = lds + lane * stride;
        const uint64_t id = first_id + (uint64_t)n;
        const uint32_t id_lo = (uint32_t)id, id_hi = (uint32_t)(id >> 32);
        uint32_t out[4];
        if (MODE == GENERATE) {
            int32_t t = 0, ac = -1, gc = -1;
            int dir = 0;
            const int last = p.n_walls + 2;              // draws 0..last-1 place, draw `last` = heading
            for (int b = 0; 4 * b <= last; ++b) {
                philox4x32_10(id_lo, id_hi, (uint32_t)b, GENERATE, seed_lo, seed_hi, out);
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const int j = 4 * b + w;
                    if (j < last) editor_apply(p, s, t, ac, gc, draw_below(out[w], p.cells));
                    else if (j == last) dir = (int)(out[w] & 3);
                }
            }
            p.t[n] = t;
            p.agent_cell[n] = ac;
            p.goal_cell[n] = gc;
            p.dir_init[n] = (int8_t)dir;
        } else {
            const int ac = p.agent_cell[n], gc = p.goal_cell[n];
            for (int b = 0; 4 * b < n_edits; ++b) {
                philox4x32_10(id_lo, id_hi, (uint32_t)b, MUTATE, seed_lo, seed_hi, out);
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const int j = 4 * b + w;
                    if (j >= n_edits) continue;
                    const int c = draw_below(out[w], p.cells);
                    if (c == ac || c == gc) continue;    // the agent's and the goal's cells stay free
                    s[(3 * c) >> 5] ^= 1u << ((3 * c) & 31);
                }
            }
        }
    }
    __syncthreads();
    for (int i = lane; i < count * SW; i += 64) {
        const int e = i / SW, o = i - e * SW;
        p.stream[(size_t)(env0 + e) * SW + o] = lds[e * stride + o];
    }
}

// One thread per stream dword: bit 3c+ch = channel ch (wall, goal, agent) of cell c.
__global__ void k_editor_set_levels(EditorDev p, const int8_t *__restrict__ walls,
                                    const int32_t *__restrict__ agent_xy,
                                    const int8_t *__restrict__ agent_dir,
                                    const int32_t *__restrict__ goal_xy)
{
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= (long long)p.N * p.SW) return;
    const int n = (int)(gid / p.SW), o = (int)(gid - (long long)n * p.SW);
    const int ax = min(max(agent_xy[2 * n], 0), p.W - 1), ay = min(max(agent_xy[2 * n + 1], 0), p.H - 1);
    const int gx = min(max(goal_xy[2 * n], 0), p.W - 1), gy = min(max(goal_xy[2 * n + 1], 0), p.H - 1);
    const int ac = ay * p.W + ax, gc = gy * p.W + gx;
    const int8_t *w = walls + (size_t)n * p.cells;
    uint32_t bits = 0;
    int c = (32 * o) / 3, ch = 32 * o - 3 * c;
    for (int i = 0; i < 32 && c < p.cells; ++i) {
        const bool on = ch == 0 ? (w[c] != 0) : (ch == 1 ? c == gc : c == ac);
        bits |= (on ? 1u : 0u) << i;
        if (++ch == 3) { ch = 0; ++c; }
    }
    p.stream[gid] = bits;
    if (o == 0) {
        p.agent_cell[n] = ac;
        p.goal_cell[n] = gc;
        p.t[n] = p.n_walls + 2;
        p.dir_init[n] = agent_dir[n] & 3;
    }
}

int levelgen_launch(const editor_ctx *ctx, int mode, uint64_t seed, uint64_t first_id, int n_edits,
                    hipStream_t st)
{
    const EditorDev &p = ctx->dev;
    const size_t per_env = 4 * (size_t)(p.SW | 1);
    int EPB = (int)((60 * 1024) / per_env);
    if (EPB > 64) EPB = 64;
    const size_t shmem = per_env * EPB;
    const dim3 grid((p.N + EPB - 1) / EPB), block(64);
    const uint32_t lo = (uint32_t)seed, hi = (uint32_t)(seed >> 32);
    if (mode == GENERATE)
        hipLaunchKernelGGL(k_levelgen<GENERATE>, grid, block, shmem, st, p, EPB, lo, hi, first_id, 0);
    else
        hipLaunchKernelGGL(k_levelgen<MUTATE>, grid, block, shmem, st, p, EPB, lo, hi, first_id, n_edits);
    MAZE_HIP_CHECK(hipGetLastError());
    return MAZE_OK;
}

}  // namespace

extern "C" int editor_random_levels(editor_ctx *ctx, uint64_t seed, uint64_t first_level_id, void *stream)
{
    if (!ctx) return MAZE_ENULL;
    MAZE_DEVICE_CHECK(ctx);
    return levelgen_launch(ctx, GENERATE, seed, first_level_id, 0, (hipStream_t)stream);
}

extern "C" int editor_mutate_levels(editor_ctx *ctx, uint64_t seed, uint64_t first_level_id, int n_edits,
                                    void *stream)
{
    if (!ctx) return MAZE_ENULL;
    MAZE_DEVICE_CHECK(ctx);
    if (n_edits < 0) return MAZE_EINVAL;
    if (n_edits == 0) return MAZE_OK;
    return levelgen_launch(ctx, MUTATE, seed, first_level_id, n_edits, (hipStream_t)stream);
}

extern "C" int editor_set_levels(editor_ctx *ctx, const int8_t *d_walls, const int32_t *d_agent_xy,
                                 const int8_t *d_agent_dir, const int32_t *d_goal_xy, void *stream)
{
    if (!ctx || !d_walls || !d_agent_xy || !d_agent_dir || !d_goal_xy) return MAZE_ENULL;
    MAZE_DEVICE_CHECK(ctx);
    const EditorDev &p = ctx->dev;
    const long long total = (long long)p.N * p.SW;
    hipLaunchKernelGGL(k_editor_set_levels, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       (hipStream_t)stream, p, d_walls, d_agent_xy, d_agent_dir, d_goal_xy);
    MAZE_HIP_CHECK(hipGetLastError());
    return MAZE_OK;
}
