// Student maze env: host entry points, level packing, per-cell kernels and the
// getters.  The tiled store-layout rollout kernels live in maze_student_tiled.hip.
#include "maze_internal.h"
#include "maze_student_device.h"

#include <new>

// ------------------------------------------------------------------ host side
static int student_dims(int N, int H, int W, int view, StudentDev *d, int *word64)
{
    if (N <= 0 || H <= 0 || W <= 0 || view <= 0 || (view & 1) == 0) return MAZE_EINVAL;
    int P = view - 1;
    int HP = H + 2 * P, WP = W + 2 * P;
    if (HP > 64 || WP > 64) return MAZE_ESIZE;
    d->N = N; d->H = H; d->W = W; d->k = view;
    d->P = P; d->HP = HP; d->WP = WP; d->SP = HP > WP ? HP : WP;
    *word64 = (d->SP > 32);
    return MAZE_OK;
}

struct StudentLayout { size_t pose, tcount, start, goalrot, grids, total; };

static StudentLayout student_layout(const StudentDev &d, int word64)
{
    StudentLayout L;
    size_t off = 0;
    size_t n = (size_t)d.N;
    L.pose = off;    off = maze_align_up(off + n * 4, 256);
    L.tcount = off;  off = maze_align_up(off + n * 4, 256);
    L.start = off;   off = maze_align_up(off + n * 4, 256);
    L.goalrot = off; off = maze_align_up(off + n * 16, 256);
    L.grids = off;   off = maze_align_up(off + n * 4 * d.SP * (word64 ? 8 : 4), 256);
    L.total = off;
    return L;
}

extern "C" int maze_workspace_bytes(int N, int H, int W, int view, size_t *out)
{
    if (!out) return MAZE_ENULL;
    StudentDev d;
    int w64;
    int rc = student_dims(N, H, W, view, &d, &w64);
    if (rc != MAZE_OK) return rc;
    *out = student_layout(d, w64).total;
    return MAZE_OK;
}

extern "C" int maze_create(maze_ctx **out, int N, int H, int W, int view, int max_steps,
                           void *d_workspace, size_t workspace_bytes)
{
    if (!out) return MAZE_ENULL;
    *out = nullptr;
    if (!d_workspace) return MAZE_ENULL;
    StudentDev d;
    int w64;
    int rc = student_dims(N, H, W, view, &d, &w64);
    if (rc != MAZE_OK) return rc;
    if (max_steps < 1 || max_steps >= (1 << 24)) return MAZE_EINVAL;
    if (((uintptr_t)d_workspace & 255) != 0) return MAZE_EINVAL;
    StudentLayout L = student_layout(d, w64);
    if (workspace_bytes < L.total) return MAZE_ESIZE;
    maze_ctx *c = new (std::nothrow) maze_ctx;
    if (!c) return MAZE_EINVAL;
    char *ws = (char *)d_workspace;
    d.max_steps = max_steps;
    d.pose = (uint32_t *)(ws + L.pose);
    d.tcount = (uint32_t *)(ws + L.tcount);
    d.start = (uint32_t *)(ws + L.start);
    d.goalrot = (uint32_t *)(ws + L.goalrot);
    d.grids = ws + L.grids;
    d.reward_slope = 0.9 / (double)max_steps;
    c->dev = d;
    c->word64 = w64;
    c->variant = 0;
    c->dev.obs_encoding = 0;
    c->dev.obs_occlusion = 0;
    c->workspace_bytes = workspace_bytes;
    if (hipGetDevice(&c->device) != hipSuccess) { delete c; return MAZE_EHIP; }
    *out = c;
    return MAZE_OK;
}

extern "C" int maze_destroy(maze_ctx *ctx)
{
    if (!ctx) return MAZE_ENULL;
    delete ctx;
    return MAZE_OK;
}

extern "C" int maze_set_kernel_variant(maze_ctx *ctx, int variant)
{
    if (!ctx) return MAZE_ENULL;
    if (variant < 0 || variant > 1) return MAZE_EINVAL;
    ctx->variant = variant;
    return MAZE_OK;
}

extern "C" int maze_set_obs_mode(maze_ctx *ctx, int encoding, int occlusion)
{
    if (!ctx) return MAZE_ENULL;
    if (encoding < 0 || encoding > 1 || occlusion < 0 || occlusion > 1) return MAZE_EINVAL;
    ctx->dev.obs_encoding = encoding;
    ctx->dev.obs_occlusion = occlusion;
    return MAZE_OK;
}

// ------------------------------------------------------------- level packing
// One wavefront per env.  The H*W wall bytes are turned into two bitmaps with wave
// ballots -- row-major (bit y*W + x) and column-major (bit x*H + y) -- 64 cells per
// ballot, kept in the wave's slice of LDS.  Every row of the four heading frames is
// then one field of one of the bitmaps (reversed for the two frames that look
// against the axis), shifted into the ring of border walls.  Lane 0 also packs the
// start pose and the goal's position in the four frames.
constexpr int PACK_WAVES = 4;                 // waves (= envs) per workgroup
constexpr int PACK_BM_DWORDS = 4096 / 32 + 4;  // bitmap of up to 64x64 cells + zero tail

__device__ __forceinline__ uint64_t bitmap_field(const uint32_t *bm, int offset, int len)
{
    const int w = offset >> 5, sh = offset & 31;
    const uint64_t lo = ((uint64_t)bm[w + 1] << 32) | bm[w];
    const uint64_t hi = bm[w + 2];
    uint64_t v = lo >> sh;
    if (sh) v |= hi << (64 - sh);
    return len >= 64 ? v : (v & (((uint64_t)1 << len) - 1));
}

template <typename Word>
__global__ __launch_bounds__(64 * PACK_WAVES) void k_pack_levels(
    StudentDev p, const int8_t *__restrict__ walls, const int32_t *__restrict__ agent_xy,
    const int8_t *__restrict__ agent_dir, const int32_t *__restrict__ goal_xy)
{
    __shared__ uint32_t lds[PACK_WAVES][2][PACK_BM_DWORDS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = blockIdx.x * PACK_WAVES + wave;
    if (n >= p.N) return;                        // whole wave leaves together
    uint32_t *bm_rm = lds[wave][0], *bm_cm = lds[wave][1];
    const int cells = p.H * p.W;
    const int8_t *g = walls + (size_t)n * cells;
    const int chunks = (cells + 63) >> 6;
    for (int c = 0; c <= chunks; ++c) {          // one extra chunk of zeros as the tail
        const int idx = c * 64 + lane;
        const bool valid = idx < cells;
        const int x = valid ? idx / p.H : 0, y = valid ? idx - x * p.H : 0;
        const bool rm = valid && g[idx] != 0;
        const bool cm = valid && g[y * p.W + x] != 0;
        const uint64_t m_rm = __ballot(rm), m_cm = __ballot(cm);
        if (lane == 0) {
            bm_rm[2 * c] = (uint32_t)m_rm; bm_rm[2 * c + 1] = (uint32_t)(m_rm >> 32);
            bm_cm[2 * c] = (uint32_t)m_cm; bm_cm[2 * c + 1] = (uint32_t)(m_cm >> 32);
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    Word *out = (Word *)p.grids + (size_t)n * 4 * p.SP;
    for (int task = lane; task < 4 * p.SP; task += 64) {
        const int d = task / p.SP, row = task - d * p.SP;
        const int rows = (d & 1) ? p.HP : p.WP;  // shape of frame d
        const int len = (d & 1) ? p.W : p.H;     // interior cells per row of frame d
        uint64_t word = ~(uint64_t)0;            // border rows and rows beyond the frame: solid
        const int r = row - p.P;                 // interior line of the frame
        if (row < rows && r >= 0 && r < rows - 2 * p.P) {
            uint64_t f;
            if (d == 3) f = bitmap_field(bm_rm, r * p.W, p.W);
            else if (d == 1) f = __brevll(bitmap_field(bm_rm, (p.H - 1 - r) * p.W, p.W)) >> (64 - p.W);
            else if (d == 0) f = bitmap_field(bm_cm, (p.W - 1 - r) * p.H, p.H);
            else f = __brevll(bitmap_field(bm_cm, r * p.H, p.H)) >> (64 - p.H);
            const uint64_t field_mask = (((uint64_t)1 << len) - 1) << p.P;
            word = (f << p.P) | ~field_mask;
        }
        out[task] = (Word)word;
    }
    if (lane == 0) {
        int ax = min(max(agent_xy[2 * n], 0), p.W - 1) + p.P;
        int ay = min(max(agent_xy[2 * n + 1], 0), p.H - 1) + p.P;
        int gx = min(max(goal_xy[2 * n], 0), p.W - 1) + p.P;
        int gy = min(max(goal_xy[2 * n + 1], 0), p.H - 1) + p.P;
        int d = agent_dir[n] & 3;
        int xd, yd;
        padded_to_frame(p, d, ax, ay, xd, yd);
        uint32_t s = (uint32_t)xd | ((uint32_t)yd << 8) | ((uint32_t)d << 16);
        p.start[n] = s;
        p.pose[n] = s;
        p.tcount[n] = 0;
        for (int f = 0; f < 4; ++f) {
            padded_to_frame(p, f, gx, gy, xd, yd);
            p.goalrot[4 * n + f] = (uint32_t)xd | ((uint32_t)yd << 8);
        }
    }
}

extern "C" int maze_reset_to_levels(maze_ctx *ctx, const int8_t *d_walls,
                                    const int32_t *d_agent_xy, const int8_t *d_agent_dir,
                                    const int32_t *d_goal_xy, void *stream)
{
    if (!ctx || !d_walls || !d_agent_xy || !d_agent_dir || !d_goal_xy) return MAZE_ENULL;
    hipStream_t st = (hipStream_t)stream;
    const StudentDev &p = ctx->dev;
    dim3 grid((p.N + PACK_WAVES - 1) / PACK_WAVES), block(64 * PACK_WAVES);
    if (ctx->word64)
        hipLaunchKernelGGL(k_pack_levels<uint64_t>, grid, block, 0, st, p, d_walls, d_agent_xy,
                           d_agent_dir, d_goal_xy);
    else
        hipLaunchKernelGGL(k_pack_levels<uint32_t>, grid, block, 0, st, p, d_walls, d_agent_xy,
                           d_agent_dir, d_goal_xy);
    MAZE_HIP_CHECK(hipGetLastError());
    return MAZE_OK;
}

// ---------------------------------------------------------- per-cell kernels
// One lane per env, state in registers across the n_steps loop, walls read from
// the packed grids in global memory (they stay in L2), observation written one
// byte at a time.  Correct for every supported shape; the tiled kernels are
// the fast path.
template <typename Word>
__device__ __forceinline__ void render_cells(const StudentDev &p, const Word *__restrict__ grid_n,
                                             uint32_t pose, uint32_t goal, int8_t *__restrict__ o)
{
    const int k = p.k, h = k >> 1;
    int xd = pose & 255, yd = (pose >> 8) & 255, d = (pose >> 16) & 3;
    int gxd = goal & 255, gyd = (goal >> 8) & 255;
    const Word *g = grid_n + d * p.SP;
    if (!p.obs_encoding && !p.obs_occlusion) {
        for (int r = 0; r < k; ++r) {
            int row = yd - (k - 1) + r;
            Word w = g[row] >> (xd - h);
            for (int c = 0; c < k; ++c) {
                int wall = (int)((w >> c) & 1);
                int isgoal = (!wall) && (row == gyd) && (xd - h + c == gxd);
                o[0] = (int8_t)wall;
                o[1] = (int8_t)isgoal;
                o[2] = (int8_t)(!wall && !isgoal);
                o += 3;
            }
        }
        return;
    }
    // Variants.  Occlusion: view rows are settled from the agent's row outwards, each as a bit
    // mask: the cells seen so far spread sideways through cells that are not walls (a seen wall
    // spreads nothing), then every seen non-wall cell makes the three cells touching it in the
    // next row ahead seen.  The agent's own cell spreads whatever it holds.
    const uint32_t all = (1u << k) - 1;
    uint32_t from_below = 1u << h;
    for (int r = k - 1; r >= 0; --r) {
        const int row = yd - (k - 1) + r;
        const uint32_t wall = (uint32_t)(g[row] >> (xd - h)) & all;
        uint32_t open = ~wall & all;
        if (r == k - 1) open |= 1u << h;
        uint32_t seen = all;
        if (p.obs_occlusion) {
            seen = from_below;
            for (int it = 1; it < k; ++it) {
                const uint32_t src = seen & open;
                seen |= ((src << 1) | (src >> 1)) & all;
            }
            const uint32_t src = seen & open;
            from_below = (src | (src << 1) | (src >> 1)) & all;
        }
        int8_t *q = o + (size_t)r * k * 3;
        for (int c = 0; c < k; ++c) {
            const int vis = (seen >> c) & 1, is_wall = (wall >> c) & 1;
            const int is_goal = !is_wall && row == gyd && xd - h + c == gxd;
            if (p.obs_encoding == 0) {
                q[0] = (int8_t)(vis & is_wall);
                q[1] = (int8_t)(vis & is_goal);
                q[2] = (int8_t)(vis & !is_wall & !is_goal);
            } else {
                // MiniGrid's indices: wall (2, grey 5), goal (8, green 1), empty (1, 0); unseen 0
                q[0] = (int8_t)(vis ? (is_wall ? 2 : (is_goal ? 8 : 1)) : 0);
                q[1] = (int8_t)(vis ? (is_wall ? 5 : (is_goal ? 1 : 0)) : 0);
                q[2] = 0;
            }
            q += 3;
        }
    }
}

template <typename Word>
__global__ void k_student_percell(StudentDev p, int n_begin, const int8_t *__restrict__ actions,
                                  int n_steps, float *__restrict__ reward,
                                  uint8_t *__restrict__ done, int8_t *__restrict__ obs)
{
    int n = n_begin + blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= p.N) return;
    const Word *grid_n = (const Word *)p.grids + (size_t)n * 4 * p.SP;
    uint32_t pose = p.pose[n];
    uint32_t t = p.tcount[n];
    const uint32_t start = p.start[n];
    uint32_t gr[4];
    for (int f = 0; f < 4; ++f) gr[f] = p.goalrot[4 * n + f];
    const size_t obs_env = (size_t)p.k * p.k * 3;
    // actions are fetched four steps ahead: the loop otherwise waits a full memory round
    // trip per step for one byte
    constexpr int AHEAD = 4;
    int a_q[AHEAD];
#pragma unroll
    for (int j = 0; j < AHEAD; ++j) a_q[j] = actions[(size_t)min(j, n_steps - 1) * p.N + n];
    for (int s = 0; s < n_steps; ++s) {
        const int a = a_q[0];
#pragma unroll
        for (int j = 0; j + 1 < AHEAD; ++j) a_q[j] = a_q[j + 1];
        a_q[AHEAD - 1] = actions[(size_t)min(s + AHEAD, n_steps - 1) * p.N + n];
        int xd = pose & 255, yd = (pose >> 8) & 255, d = (pose >> 16) & 3;
        bool blocked = (grid_n[d * p.SP + yd - 1] >> xd) & 1;
        pose = student_move(p, pose, a, blocked);
        t += 1;
        d = (pose >> 16) & 3;
        bool reached = (pose & 0xFFFF) == gr[d];
        float r = reached ? (float)(1.0 - (double)t * p.reward_slope) : 0.0f;
        bool dn = reached || t >= (uint32_t)p.max_steps;
        if (dn) { pose = start; t = 0; }
        reward[(size_t)s * p.N + n] = r;
        done[(size_t)s * p.N + n] = dn ? 1 : 0;
        if (obs)
            render_cells<Word>(p, grid_n, pose, gr[(pose >> 16) & 3],
                               obs + ((size_t)s * p.N + n) * obs_env);
    }
    p.pose[n] = pose;
    p.tcount[n] = t;
}

template <typename Word>
__global__ void k_render_percell(StudentDev p, int n_begin, int8_t *__restrict__ obs)
{
    int n = n_begin + blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= p.N) return;
    const Word *grid_n = (const Word *)p.grids + (size_t)n * 4 * p.SP;
    uint32_t pose = p.pose[n];
    uint32_t goal = p.goalrot[4 * n + ((pose >> 16) & 3)];
    render_cells<Word>(p, grid_n, pose, goal, obs + (size_t)n * p.k * p.k * 3);
}

// Implemented in maze_student_tiled.hip: launches the tiled kernel on the first
// *covered envs (a multiple of the workgroup size; 0 if the shape is not covered) and returns 1 if
// it launched.  n_steps == 0 renders the current state.
int student_tiled_launch(const maze_ctx *ctx, const int8_t *d_actions, int n_steps,
                         float *d_reward, uint8_t *d_done, int8_t *d_obs, int *covered,
                         hipStream_t st);

extern "C" int maze_step(maze_ctx *ctx, const int8_t *d_actions, int n_steps, float *d_reward,
                         uint8_t *d_done, int8_t *d_obs, void *stream)
{
    if (!ctx || !d_actions || !d_reward || !d_done) return MAZE_ENULL;
    if (n_steps < 1) return MAZE_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    const StudentDev &p = ctx->dev;
    int covered = 0;
    if (ctx->variant == 0)
        student_tiled_launch(ctx, d_actions, n_steps, d_reward, d_done, d_obs, &covered, st);
    if (covered < p.N) {
        dim3 grid((p.N - covered + 63) / 64), block(64);
        if (ctx->word64)
            hipLaunchKernelGGL(k_student_percell<uint64_t>, grid, block, 0, st, p, covered,
                               d_actions, n_steps, d_reward, d_done, d_obs);
        else
            hipLaunchKernelGGL(k_student_percell<uint32_t>, grid, block, 0, st, p, covered,
                               d_actions, n_steps, d_reward, d_done, d_obs);
    }
    MAZE_HIP_CHECK(hipGetLastError());
    return MAZE_OK;
}

extern "C" int maze_render_obs(maze_ctx *ctx, int8_t *d_obs, void *stream)
{
    if (!ctx || !d_obs) return MAZE_ENULL;
    hipStream_t st = (hipStream_t)stream;
    const StudentDev &p = ctx->dev;
    int covered = 0;
    if (ctx->variant == 0)
        student_tiled_launch(ctx, nullptr, 0, nullptr, nullptr, d_obs, &covered, st);
    if (covered < p.N) {
        dim3 grid((p.N - covered + 63) / 64), block(64);
        if (ctx->word64)
            hipLaunchKernelGGL(k_render_percell<uint64_t>, grid, block, 0, st, p, covered, d_obs);
        else
            hipLaunchKernelGGL(k_render_percell<uint32_t>, grid, block, 0, st, p, covered, d_obs);
    }
    MAZE_HIP_CHECK(hipGetLastError());
    return MAZE_OK;
}

// -------------------------------------------------------------------- getters
__global__ void k_get_state(StudentDev p, int32_t *xy, int8_t *dir, int32_t *t)
{
    int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= p.N) return;
    uint32_t pose = p.pose[n];
    int d = (pose >> 16) & 3, X, Y;
    frame_to_padded(p, d, pose & 255, (pose >> 8) & 255, X, Y);
    if (xy) { xy[2 * n] = X - p.P; xy[2 * n + 1] = Y - p.P; }
    if (dir) dir[n] = (int8_t)d;
    if (t) t[n] = (int32_t)p.tcount[n];
}

template <typename Word>
__global__ void k_get_walls(StudentDev p, int8_t *walls)
{
    long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    long long total = (long long)p.N * p.H * p.W;
    if (gid >= total) return;
    int x = (int)(gid % p.W);
    int y = (int)((gid / p.W) % p.H);
    int n = (int)(gid / ((long long)p.W * p.H));
    const Word *g3 = (const Word *)p.grids + ((size_t)n * 4 + 3) * p.SP;   // frame 3 = unrotated
    walls[gid] = (int8_t)((g3[y + p.P] >> (x + p.P)) & 1);
}

__global__ void k_get_level_poses(StudentDev p, int32_t *agent_xy, int8_t *agent_dir,
                                  int32_t *goal_xy)
{
    int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= p.N) return;
    uint32_t s = p.start[n];
    int d = (s >> 16) & 3, X, Y;
    frame_to_padded(p, d, s & 255, (s >> 8) & 255, X, Y);
    if (agent_xy) { agent_xy[2 * n] = X - p.P; agent_xy[2 * n + 1] = Y - p.P; }
    if (agent_dir) agent_dir[n] = (int8_t)d;
    if (goal_xy) {
        uint32_t g = p.goalrot[4 * n + 3];
        goal_xy[2 * n] = (int)(g & 255) - p.P;
        goal_xy[2 * n + 1] = (int)((g >> 8) & 255) - p.P;
    }
}

extern "C" int maze_get_state(maze_ctx *ctx, int32_t *d_xy, int8_t *d_dir, int32_t *d_t,
                              void *stream)
{
    if (!ctx) return MAZE_ENULL;
    const StudentDev &p = ctx->dev;
    hipLaunchKernelGGL(k_get_state, dim3((p.N + 255) / 256), dim3(256), 0, (hipStream_t)stream, p,
                       d_xy, d_dir, d_t);
    MAZE_HIP_CHECK(hipGetLastError());
    return MAZE_OK;
}

extern "C" int maze_get_levels(maze_ctx *ctx, int8_t *d_walls, int32_t *d_agent_xy,
                               int8_t *d_agent_dir, int32_t *d_goal_xy, void *stream)
{
    if (!ctx) return MAZE_ENULL;
    const StudentDev &p = ctx->dev;
    hipStream_t st = (hipStream_t)stream;
    if (d_walls) {
        long long total = (long long)p.N * p.H * p.W;
        unsigned blocks = (unsigned)((total + 255) / 256);
        if (ctx->word64)
            hipLaunchKernelGGL(k_get_walls<uint64_t>, dim3(blocks), dim3(256), 0, st, p, d_walls);
        else
            hipLaunchKernelGGL(k_get_walls<uint32_t>, dim3(blocks), dim3(256), 0, st, p, d_walls);
    }
    hipLaunchKernelGGL(k_get_level_poses, dim3((p.N + 255) / 256), dim3(256), 0, st, p, d_agent_xy,
                       d_agent_dir, d_goal_xy);
    MAZE_HIP_CHECK(hipGetLastError());
    return MAZE_OK;
}

extern "C" const char *maze_strerror(int code)
{
    switch (code) {
    case MAZE_OK: return "ok";
    case MAZE_EINVAL: return "argument out of range";
    case MAZE_ENULL: return "required pointer is NULL";
    case MAZE_ESIZE: return "grid or view too large for the packed layout, or workspace too small";
    case MAZE_EHIP: return "HIP runtime call failed";
    default: return "unknown error code";
    }
}
