// Teacher editor env: host entry points and per-cell kernels.
#include "maze_internal.h"
#include "maze_editor_device.h"

#include <new>

struct EditorLayout { size_t stream, agent, goal, t, dir, total; };

static int editor_dims(int N, int H, int W, EditorDev *d)
{
    if (N <= 0 || H <= 0 || W <= 0) return MAZE_EINVAL;
    long long cells = (long long)H * W;
    if (cells < 2) return MAZE_EINVAL;
    if (cells > 4096) return MAZE_ESIZE;
    d->N = N; d->H = H; d->W = W; d->cells = (int)cells;
    d->SW = (3 * (int)cells + 31) / 32;
    return MAZE_OK;
}

static EditorLayout editor_layout(const EditorDev &d)
{
    EditorLayout L;
    size_t off = 0, n = (size_t)d.N;
    L.stream = off; off = maze_align_up(off + n * d.SW * 4, 256);
    L.agent = off;  off = maze_align_up(off + n * 4, 256);
    L.goal = off;   off = maze_align_up(off + n * 4, 256);
    L.t = off;      off = maze_align_up(off + n * 4, 256);
    L.dir = off;    off = maze_align_up(off + n, 256);
    L.total = off;
    return L;
}

extern "C" int editor_workspace_bytes(int N, int H, int W, size_t *out)
{
    if (!out) return MAZE_ENULL;
    EditorDev d;
    int rc = editor_dims(N, H, W, &d);
    if (rc != MAZE_OK) return rc;
    *out = editor_layout(d).total;
    return MAZE_OK;
}

extern "C" int editor_create(editor_ctx **out, int N, int H, int W, int n_walls,
                             void *d_workspace, size_t workspace_bytes)
{
    if (!out) return MAZE_ENULL;
    *out = nullptr;
    if (!d_workspace) return MAZE_ENULL;
    EditorDev d;
    int rc = editor_dims(N, H, W, &d);
    if (rc != MAZE_OK) return rc;
    if (n_walls < 0 || n_walls > (1 << 24)) return MAZE_EINVAL;
    if (((uintptr_t)d_workspace & 255) != 0) return MAZE_EINVAL;
    EditorLayout L = editor_layout(d);
    if (workspace_bytes < L.total) return MAZE_ESIZE;
    editor_ctx *c = new (std::nothrow) editor_ctx;
    if (!c) return MAZE_EINVAL;
    char *ws = (char *)d_workspace;
    d.n_walls = n_walls;
    d.stream = (uint32_t *)(ws + L.stream);
    d.agent_cell = (int32_t *)(ws + L.agent);
    d.goal_cell = (int32_t *)(ws + L.goal);
    d.t = (int32_t *)(ws + L.t);
    d.dir_init = (int8_t *)(ws + L.dir);
    c->dev = d;
    c->workspace_bytes = workspace_bytes;
    if (hipGetDevice(&c->device) != hipSuccess) { delete c; return MAZE_EHIP; }
    c->cus = 0;
    c->clock_khz = 0;
    if (hipDeviceGetAttribute(&c->cus, hipDeviceAttributeMultiprocessorCount, c->device) != hipSuccess ||
        hipDeviceGetAttribute(&c->clock_khz, hipDeviceAttributeWallClockRate, c->device) != hipSuccess)
        c->clock_khz = 0;                         // unknown: the store waves are not paced
    int lds = 0;
    if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, c->device) != hipSuccess)
        lds = 64 * 1024;
    c->lds_per_cu = (size_t)lds;
    *out = c;
    return MAZE_OK;
}

extern "C" int editor_destroy(editor_ctx *ctx)
{
    if (!ctx) return MAZE_ENULL;
    delete ctx;
    return MAZE_OK;
}

__global__ void k_editor_reset(EditorDev p, const int8_t *__restrict__ dir_init)
{
    long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    long long total = (long long)p.N * p.SW;
    if (gid < total) p.stream[gid] = 0;
    if (gid < p.N) {
        p.agent_cell[gid] = -1;
        p.goal_cell[gid] = -1;
        p.t[gid] = 0;
        p.dir_init[gid] = dir_init[gid] & 3;
    }
}

extern "C" int editor_reset(editor_ctx *ctx, const int8_t *d_agent_dir_init, void *stream)
{
    if (!ctx || !d_agent_dir_init) return MAZE_ENULL;
    MAZE_DEVICE_CHECK(ctx);
    const EditorDev &p = ctx->dev;
    long long total = (long long)p.N * p.SW;
    hipLaunchKernelGGL(k_editor_reset, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       (hipStream_t)stream, p, d_agent_dir_init);
    MAZE_HIP_CHECK(hipGetLastError());
    return MAZE_OK;
}

// One lane per env; the stream stays in global memory (L2) and the observation is
// written byte by byte.  Correct for every supported shape.
__global__ void k_editor_percell(EditorDev p, int n_begin, const int32_t *__restrict__ actions,
                                 int n_steps, int8_t *__restrict__ obs,
                                 int32_t *__restrict__ t_out, uint8_t *__restrict__ done)
{
    int n = n_begin + blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= p.N) return;
    uint32_t *s = p.stream + (size_t)n * p.SW;
    int32_t t = p.t[n], ac = p.agent_cell[n], gc = p.goal_cell[n];
    const int nbytes = 3 * p.cells;
    for (int st = 0; st < n_steps; ++st) {
        size_t i = (size_t)st * p.N + n;
        editor_apply(p, s, t, ac, gc, actions[i]);
        if (t_out) t_out[i] = t;
        if (done) done[i] = (t == p.n_walls + 2) ? 1 : 0;
        if (obs) {
            int8_t *o = obs + i * nbytes;
            for (int b = 0; b < nbytes; ++b) o[b] = (int8_t)((s[b >> 5] >> (b & 31)) & 1);
        }
    }
    p.t[n] = t;
    p.agent_cell[n] = ac;
    p.goal_cell[n] = gc;
}

// Implemented in maze_editor_tiled.hip: runs the tiled kernel on the first *covered envs.
int editor_tiled_launch(const editor_ctx *ctx, const int32_t *d_actions, int n_steps,
                        int8_t *d_obs, int32_t *d_t, uint8_t *d_done, int *covered, hipStream_t st);

extern "C" int editor_step(editor_ctx *ctx, const int32_t *d_actions, int n_steps, int8_t *d_obs,
                           int32_t *d_t, uint8_t *d_done, void *stream)
{
    if (!ctx || !d_actions) return MAZE_ENULL;
    MAZE_DEVICE_CHECK(ctx);
    if (n_steps < 1) return MAZE_EINVAL;
    const EditorDev &p = ctx->dev;
    hipStream_t st = (hipStream_t)stream;
    int covered = 0;
    editor_tiled_launch(ctx, d_actions, n_steps, d_obs, d_t, d_done, &covered, st);
    if (covered < p.N)
        hipLaunchKernelGGL(k_editor_percell, dim3((p.N - covered + 63) / 64), dim3(64), 0, st, p,
                           covered, d_actions, n_steps, d_obs, d_t, d_done);
    MAZE_HIP_CHECK(hipGetLastError());
    return MAZE_OK;
}

__global__ void k_editor_get_walls(EditorDev p, int8_t *walls)
{
    long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    long long total = (long long)p.N * p.cells;
    if (gid >= total) return;
    int c = (int)(gid % p.cells);
    int n = (int)(gid / p.cells);
    const uint32_t *s = p.stream + (size_t)n * p.SW;
    walls[gid] = (int8_t)((s[(3 * c) >> 5] >> ((3 * c) & 31)) & 1);
}

__global__ void k_editor_get_poses(EditorDev p, int32_t *agent_xy, int8_t *agent_dir,
                                   int32_t *goal_xy)
{
    int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= p.N) return;
    int ac = p.agent_cell[n], gc = p.goal_cell[n];
    if (agent_xy) {
        agent_xy[2 * n] = ac < 0 ? -1 : ac % p.W;
        agent_xy[2 * n + 1] = ac < 0 ? -1 : ac / p.W;
    }
    if (agent_dir) agent_dir[n] = ac < 0 ? 0 : p.dir_init[n];
    if (goal_xy) {
        goal_xy[2 * n] = gc < 0 ? -1 : gc % p.W;
        goal_xy[2 * n + 1] = gc < 0 ? -1 : gc / p.W;
    }
}

extern "C" int editor_get_levels(editor_ctx *ctx, int8_t *d_walls, int32_t *d_agent_xy,
                                 int8_t *d_agent_dir, int32_t *d_goal_xy, void *stream)
{
    if (!ctx) return MAZE_ENULL;
    MAZE_DEVICE_CHECK(ctx);
    const EditorDev &p = ctx->dev;
    hipStream_t st = (hipStream_t)stream;
    if (d_walls) {
        long long total = (long long)p.N * p.cells;
        hipLaunchKernelGGL(k_editor_get_walls, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                           st, p, d_walls);
    }
    hipLaunchKernelGGL(k_editor_get_poses, dim3((p.N + 255) / 256), dim3(256), 0, st, p,
                       d_agent_xy, d_agent_dir, d_goal_xy);
    MAZE_HIP_CHECK(hipGetLastError());
    return MAZE_OK;
}
