// Student maze env: host entry points, level packing, per-cell kernels and the
// getters.  The tiled store-layout rollout kernels live in maze_student_tiled.hip.
#include "maze_internal.h"
#include "maze_student_device.h"

#include <atomic>
#include <new>

// ------------------------------------------------------------------ host side
static int student_dims(int N, int H, int W, int view, StudentDev *d, int *word64)
{
    // view >= 3: the padding of view - 1 rings of wall is also what stops a forward step at the
    // edge of the interior, so a 1 x 1 view (no ring) is not a shape this layout can hold
    if (N <= 0 || H <= 0 || W <= 0 || view < 3 || (view & 1) == 0) return MAZE_EINVAL;
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

// Point a context at its workspace (device memory laid out by student_layout) with the
// defaults of a fresh env: automatic kernel choice, plain observation.
static void student_bind(maze_ctx *c, StudentDev d, int word64, int max_steps, void *d_workspace,
                         const StudentLayout &L)
{
    char *ws = (char *)d_workspace;
    d.max_steps = max_steps;
    d.pose = (uint32_t *)(ws + L.pose);
    d.tcount = (uint32_t *)(ws + L.tcount);
    d.start = (uint32_t *)(ws + L.start);
    d.goalrot = (uint32_t *)(ws + L.goalrot);
    d.grids = ws + L.grids;
    d.reward_slope = 0.9 / (double)max_steps;
    d.obs_encoding = 0;
    d.obs_occlusion = 0;
    c->dev = d;
    c->word64 = word64;
    c->variant = 0;
    c->workspace_bytes = L.total;
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
    student_bind(c, d, w64, max_steps, d_workspace, L);
    c->workspace_bytes = workspace_bytes;
    hipDeviceProp_t prop;
    if (hipGetDevice(&c->device) != hipSuccess ||
        hipGetDeviceProperties(&prop, c->device) != hipSuccess) { delete c; return MAZE_EHIP; }
    c->cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 1;
    c->lds_per_cu = prop.maxSharedMemoryPerMultiProcessor;
    c->clock_khz = 0;
    if (hipDeviceGetAttribute(&c->clock_khz, hipDeviceAttributeWallClockRate, c->device) != hipSuccess)
        c->clock_khz = 0;
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
constexpr int PACK_WAVES = 4;                 // waves per workgroup

// Level packing for grids whose padded rows fit 32-bit words (every 13 x 13 configuration).
// G = 16 or 32 lanes per env, max(H, W) <= G: lane l assembles row l of the wall grid as a
// bit mask from the wall bytes (parked in LDS by the whole wave, one coalesced read of the
// wave's envs), a log2(G)-stage butterfly over the env's lanes transposes the G x G bit matrix
// so that lane l also holds column l, and the four heading frames follow directly: frame 3
// holds the rows, frame 1 the rows reversed in both directions, frames 0 and 2 the columns
// (one of them reversed each way).  The frames are staged in LDS and leave as 16-byte pieces
// of one contiguous run per wave.  No loop over cells, no 64-bit arithmetic.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// value of lane (id ^ J) within groups of 32 lanes (the LDS crossbar's bit-mode swizzle)
template <int J>
__device__ __forceinline__ uint32_t lane_xor(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x1F | (J << 10));
}

// One butterfly stage of the bit-matrix transpose: blocks of J x J off the diagonal swap.
template <int J>
__device__ __forceinline__ uint32_t transpose_stage(uint32_t r, int l)
{
    constexpr uint32_t keep = J == 16 ? 0x0000FFFFu : J == 8 ? 0x00FF00FFu : J == 4 ? 0x0F0F0F0Fu
                            : J == 2 ? 0x33333333u : 0x55555555u;     // columns x with (x & J) == 0
    const uint32_t t = lane_xor<J>(r);
    const uint32_t lower = (r & keep) | ((t & keep) << J);            // lanes with (l & J) == 0
    const uint32_t upper = (r & (keep << J)) | ((t >> J) & keep);
    return (l & J) ? upper : lower;
}

template <int G>
__global__ __launch_bounds__(64 * PACK_WAVES) void k_pack_levels_rows(
    StudentDev p, const int8_t *__restrict__ walls, const int32_t *__restrict__ agent_xy,
    const int8_t *__restrict__ agent_dir, const int32_t *__restrict__ goal_xy)
{
    constexpr int EPV = 64 / G;                      // envs per wave
    constexpr int IN_DWORDS = EPV * G * G / 4;       // wall bytes of a wave's envs, at most
    constexpr int OUT_DWORDS = EPV * 4 * 32;         // their frames, at most (SP <= 32)
    __shared__ uint32_t in_lds[PACK_WAVES][IN_DWORDS];
    __shared__ __align__(16) uint32_t out_lds[PACK_WAVES][OUT_DWORDS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane / G, l = lane % G;
    const int n0 = (blockIdx.x * PACK_WAVES + wave) * EPV;      // first env of the wave
    if (n0 >= p.N) return;                                      // (no workgroup barrier below)
    const int live_envs = min(EPV, p.N - n0);
    const bool live = sub < live_envs;
    const int n = n0 + (live ? sub : 0);
    // the five pose lanes of an env request their inputs first
    const int32_t *pos_src = l < 4 ? goal_xy : agent_xy;
    const int pos_x = l < 5 ? pos_src[2 * n] : 0, pos_y = l < 5 ? pos_src[2 * n + 1] : 0;
    const int start_dir = agent_dir[n] & 3;
    const int H = p.H, W = p.W, P = p.P, SP = p.SP, cells = H * W;
    // wall bytes of the wave's envs: one contiguous run, a dword per lane and round (of any
    // alignment; the run's last bytes singly, so that nothing beyond the array is read)
    const int bytes = live_envs * cells;
    const int8_t *src = walls + (size_t)n0 * cells;
    uint32_t *in = in_lds[wave];
    for (int i = lane; 4 * i < bytes; i += 64) {
        uint32_t v = 0;
        if (4 * i + 4 <= bytes) {
            __builtin_memcpy(&v, src + 4 * i, 4);
        } else {
            for (int b = 0; 4 * i + b < bytes; ++b) v |= (uint32_t)(uint8_t)src[4 * i + b] << (8 * b);
        }
        in[i] = v;
    }
    wave_lds_sync();
    uint32_t r = 0;                                  // row l: bit x = wall(x, l)
    if (live && l < H) {
        const uint8_t *row = (const uint8_t *)in + sub * cells + l * W;
        for (int x0 = 0; x0 < W; x0 += 8) {
            uint32_t b[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) b[u] = row[min(x0 + u, W - 1)];
#pragma unroll
            for (int u = 0; u < 8; ++u) r |= (b[u] ? 1u : 0u) << (x0 + u);
        }
        r &= (1u << W) - 1u;
    }
    uint32_t c = r;                                  // column l after the transpose: bit y = wall(l, y)
    if (G == 32) c = transpose_stage<16>(c, l);
    c = transpose_stage<8>(c, l);
    c = transpose_stage<4>(c, l);
    c = transpose_stage<2>(c, l);
    c = transpose_stage<1>(c, l);
    // frames: everything outside the interior is wall
    uint32_t *out = out_lds[wave];
    const int per_env = 4 * SP;
    for (int i = lane; i < live_envs * per_env; i += 64) out[i] = ~0u;
    wave_lds_sync();
    if (live) {
        uint32_t *o = out + sub * per_env;
        if (l < H) {
            const uint32_t field = ((1u << W) - 1u) << P;
            o[3 * SP + P + l] = (r << P) | ~field;
            o[1 * SP + (p.HP - 1 - P - l)] = ((__brev(r) >> (32 - W)) << P) | ~field;
        }
        if (l < W) {
            const uint32_t field = ((1u << H) - 1u) << P;
            o[0 * SP + (p.WP - 1 - P - l)] = (c << P) | ~field;
            o[2 * SP + P + l] = ((__brev(c) >> (32 - H)) << P) | ~field;
        }
    }
    wave_lds_sync();
    uint4 *dst = (uint4 *)((uint32_t *)p.grids + (size_t)n0 * per_env);
    for (int i = lane; i < live_envs * SP; i += 64) dst[i] = ((const uint4 *)out)[i];
    if (l < 5 && live) {
        const int X = min(max(pos_x, 0), W - 1) + P;
        const int Y = min(max(pos_y, 0), H - 1) + P;
        const int d = l < 4 ? l : start_dir;
        int xd, yd;
        padded_to_frame(p, d, X, Y, xd, yd);
        const uint32_t v = (uint32_t)xd | ((uint32_t)yd << 8);
        if (l < 4) {
            p.goalrot[4 * n + l] = v;
        } else {
            const uint32_t st = v | ((uint32_t)d << 16);
            p.start[n] = st;
            p.pose[n] = st;
            p.tcount[n] = 0;
        }
    }
}

// The same for padded rows of 33 to 64 bits (grids up to 60 x 60): one env per wave, lane l takes
// row l and column l, a line of bits is two 32-bit halves; the 64 x 64 bit matrix is transposed
// by one exchange across the wave's halves (blocks of 32) and the five butterfly stages on
// either half.
__global__ __launch_bounds__(64 * PACK_WAVES) void k_pack_levels_rows64(
    StudentDev p, const int8_t *__restrict__ walls, const int32_t *__restrict__ agent_xy,
    const int8_t *__restrict__ agent_dir, const int32_t *__restrict__ goal_xy)
{
    constexpr int IN_DWORDS = 64 * 64 / 4;           // wall bytes of an env, at most
    constexpr int OUT_DWORDS = 4 * 64 * 2;           // its frames, at most (SP <= 64 words of 64 bits)
    __shared__ uint32_t in_lds[PACK_WAVES][IN_DWORDS];
    __shared__ __align__(16) uint32_t out_lds[PACK_WAVES][OUT_DWORDS];
    const int l = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = blockIdx.x * PACK_WAVES + wave;
    if (n >= p.N) return;                            // (no workgroup barrier below)
    const int32_t *pos_src = l < 4 ? goal_xy : agent_xy;
    const int pos_x = l < 5 ? pos_src[2 * n] : 0, pos_y = l < 5 ? pos_src[2 * n + 1] : 0;
    const int start_dir = agent_dir[n] & 3;
    const int H = p.H, W = p.W, P = p.P, SP = p.SP, cells = H * W;
    const int8_t *src = walls + (size_t)n * cells;
    uint32_t *in = in_lds[wave];
    for (int i = l; 4 * i < cells; i += 64) {
        uint32_t v = 0;
        if (4 * i + 4 <= cells) {
            __builtin_memcpy(&v, src + 4 * i, 4);
        } else {
            for (int b = 0; 4 * i + b < cells; ++b) v |= (uint32_t)(uint8_t)src[4 * i + b] << (8 * b);
        }
        in[i] = v;
    }
    wave_lds_sync();
    uint32_t rlo = 0, rhi = 0;                       // row l: bit x = wall(x, l), x < 32 in rlo
    if (l < H) {
        const uint8_t *row = (const uint8_t *)in + l * W;
        for (int x0 = 0; x0 < W; x0 += 8) {
            uint32_t b[8], part = 0;
#pragma unroll
            for (int u = 0; u < 8; ++u) b[u] = row[min(x0 + u, W - 1)];
#pragma unroll
            for (int u = 0; u < 8; ++u) part |= (b[u] ? 1u : 0u) << u;
            if (x0 < 32) rlo |= part << x0;
            else rhi |= part << (x0 - 32);
        }
        // (the last group repeated the row's last cell beyond its end: cut that off)
        if (W < 32) { rlo &= (1u << W) - 1u; rhi = 0; }
        else if (W < 64) rhi &= (1u << (W - 32)) - 1u;
    }
    // column l after the transpose: bit y = wall(l, y)
    uint32_t clo = rlo, chi = rhi;
    {
        const uint32_t give = (l & 32) ? clo : chi;
        const uint32_t got = (uint32_t)__builtin_amdgcn_ds_bpermute(4 * (l ^ 32), (int)give);
        if (l & 32) clo = got; else chi = got;
    }
    clo = transpose_stage<16>(clo, l); chi = transpose_stage<16>(chi, l);
    clo = transpose_stage<8>(clo, l);  chi = transpose_stage<8>(chi, l);
    clo = transpose_stage<4>(clo, l);  chi = transpose_stage<4>(chi, l);
    clo = transpose_stage<2>(clo, l);  chi = transpose_stage<2>(chi, l);
    clo = transpose_stage<1>(clo, l);  chi = transpose_stage<1>(chi, l);
    const uint64_t r = ((uint64_t)rhi << 32) | rlo, c = ((uint64_t)chi << 32) | clo;
    uint64_t *out = (uint64_t *)out_lds[wave];
    for (int i = l; i < 4 * SP; i += 64) out[i] = ~(uint64_t)0;
    wave_lds_sync();
    if (l < H) {                                     // (W, H <= 60: every shift below is < 64)
        const uint64_t field = (((uint64_t)1 << W) - 1u) << P;
        out[3 * SP + P + l] = (r << P) | ~field;
        out[1 * SP + (p.HP - 1 - P - l)] = ((__brevll(r) >> (64 - W)) << P) | ~field;
    }
    if (l < W) {
        const uint64_t field = (((uint64_t)1 << H) - 1u) << P;
        out[0 * SP + (p.WP - 1 - P - l)] = (c << P) | ~field;
        out[2 * SP + P + l] = ((__brevll(c) >> (64 - H)) << P) | ~field;
    }
    wave_lds_sync();
    uint4 *dst = (uint4 *)((uint64_t *)p.grids + (size_t)n * 4 * SP);
    for (int i = l; i < 2 * SP; i += 64) dst[i] = ((const uint4 *)out)[i];
    if (l < 5) {
        const int X = min(max(pos_x, 0), W - 1) + P;
        const int Y = min(max(pos_y, 0), H - 1) + P;
        const int d = l < 4 ? l : start_dir;
        int xd, yd;
        padded_to_frame(p, d, X, Y, xd, yd);
        const uint32_t v = (uint32_t)xd | ((uint32_t)yd << 8);
        if (l < 4) {
            p.goalrot[4 * n + l] = v;
        } else {
            const uint32_t st = v | ((uint32_t)d << 16);
            p.start[n] = st;
            p.pose[n] = st;
            p.tcount[n] = 0;
        }
    }
}

extern "C" int maze_reset_to_levels(maze_ctx *ctx, const int8_t *d_walls,
                                    const int32_t *d_agent_xy, const int8_t *d_agent_dir,
                                    const int32_t *d_goal_xy, void *stream)
{
    if (!ctx || !d_walls || !d_agent_xy || !d_agent_dir || !d_goal_xy) return MAZE_ENULL;
    MAZE_DEVICE_CHECK(ctx);
    hipStream_t st = (hipStream_t)stream;
    const StudentDev &p = ctx->dev;
    const dim3 block(64 * PACK_WAVES);
    auto blocks = [&](int envs_per_wave) {
        const int per_block = PACK_WAVES * envs_per_wave;
        return dim3((p.N + per_block - 1) / per_block);
    };
    if (ctx->word64) {
        // 64-bit rows: SP <= 64, so max(H, W) <= 60
        hipLaunchKernelGGL(k_pack_levels_rows64, blocks(1), block, 0, st, p, d_walls, d_agent_xy,
                           d_agent_dir, d_goal_xy);
    } else {
        // 32-bit rows: SP <= 32, so max(H, W) <= 28
        if (p.H <= 16 && p.W <= 16)
            hipLaunchKernelGGL(k_pack_levels_rows<16>, blocks(4), block, 0, st, p, d_walls, d_agent_xy,
                               d_agent_dir, d_goal_xy);
        else
            hipLaunchKernelGGL(k_pack_levels_rows<32>, blocks(2), block, 0, st, p, d_walls, d_agent_xy,
                               d_agent_dir, d_goal_xy);
    }
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

// Implemented in maze_student_tiled.hip: launches the tiled kernels on the first *covered envs
// (0 if the call is not one they take) and returns 1 if it launched, 0 if not, or a negative
// error code.  n_steps == 0 renders the current state.
int student_tiled_launch(const maze_ctx *ctx, const int8_t *d_actions, int n_steps,
                         float *d_reward, uint8_t *d_done, int8_t *d_obs, int *covered,
                         hipStream_t st);

int student_tiled_plan(int k, int N, int SP, bool typed, bool occlusion, int cus, size_t budget,
                       int *epw, size_t *lds_bytes);

extern "C" int maze_rollout_plan(int N, int H, int W, int view, int encoding, int occlusion, int cus,
                                 size_t lds_per_cu, int *envs_per_workgroup, size_t *lds_bytes)
{
    if (!envs_per_workgroup || !lds_bytes) return MAZE_ENULL;
    StudentDev d;
    int w64;
    const int rc = student_dims(N, H, W, view, &d, &w64);
    if (rc != MAZE_OK) return rc;
    if (cus < 1 || encoding < 0 || encoding > 1 || occlusion < 0 || occlusion > 1) return MAZE_EINVAL;
    const size_t budget = lds_per_cu > 1024 ? lds_per_cu - 1024 : 0;
    return student_tiled_plan(view, N, d.SP, encoding != 0, occlusion != 0, cus, budget,
                              envs_per_workgroup, lds_bytes);
}

extern "C" int maze_step(maze_ctx *ctx, const int8_t *d_actions, int n_steps, float *d_reward,
                         uint8_t *d_done, int8_t *d_obs, void *stream)
{
    if (!ctx || !d_actions || !d_reward || !d_done) return MAZE_ENULL;
    if (n_steps < 1) return MAZE_EINVAL;
    MAZE_DEVICE_CHECK(ctx);
    hipStream_t st = (hipStream_t)stream;
    const StudentDev &p = ctx->dev;
    int covered = 0;
    if (ctx->variant == 0) {
        const int rc = student_tiled_launch(ctx, d_actions, n_steps, d_reward, d_done, d_obs, &covered, st);
        if (rc < 0) return rc;
    }
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
    MAZE_DEVICE_CHECK(ctx);
    hipStream_t st = (hipStream_t)stream;
    const StudentDev &p = ctx->dev;
    int covered = 0;
    if (ctx->variant == 0) {
        const int rc = student_tiled_launch(ctx, nullptr, 0, nullptr, nullptr, d_obs, &covered, st);
        if (rc < 0) return rc;
    }
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

// ------------------------------------------- rollout without context or workspace
// For callers that cannot allocate device memory: the packed levels and the env state of
// one rollout live in a static device array instead of a caller's workspace.  Each GPU
// holds its own copy of the array at its own address; the address is looked up once per
// device (with that device current) and used from then on -- the array's name itself is
// only a host-side stand-in and never goes to a kernel.
static __device__ __align__(256) unsigned char scratch[MAZE_STATIC_WORKSPACE_BYTES];

namespace {
struct StaticDevice {
    std::atomic<int> ready{0};
    void *scratch_ptr = nullptr;
    int cus = 0;
    size_t lds_per_cu = 0;
    int clock_khz = 0;
};
StaticDevice static_devices[16];
}  // namespace

extern "C" int maze_rollout_static(int N, int H, int W, int view, int max_steps,
                                   const int8_t *d_walls, const int32_t *d_agent_xy,
                                   const int8_t *d_agent_dir, const int32_t *d_goal_xy,
                                   const int8_t *d_actions, int n_steps, float *d_reward,
                                   uint8_t *d_done, int8_t *d_obs, void *stream)
{
    if (!d_walls || !d_agent_xy || !d_agent_dir || !d_goal_xy || !d_actions || !d_reward || !d_done)
        return MAZE_ENULL;
    StudentDev d;
    int w64;
    const int rc = student_dims(N, H, W, view, &d, &w64);
    if (rc != MAZE_OK) return rc;
    if (max_steps < 1 || max_steps >= (1 << 24) || n_steps < 1) return MAZE_EINVAL;
    const StudentLayout L = student_layout(d, w64);
    if (L.total > (size_t)MAZE_STATIC_WORKSPACE_BYTES) return MAZE_ESIZE;
    int device = -1;
    MAZE_HIP_CHECK(hipGetDevice(&device));
    if (device < 0 || device >= 16) return MAZE_EINVAL;
    StaticDevice &sd = static_devices[device];
    if (!sd.ready.load(std::memory_order_acquire)) {
        // first call on this device (two threads racing here look up the same values)
        void *ptr = nullptr;
        MAZE_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr || ((uintptr_t)ptr & 255) != 0) return MAZE_EHIP;
        hipDeviceProp_t prop;
        MAZE_HIP_CHECK(hipGetDeviceProperties(&prop, device));
        sd.scratch_ptr = ptr;
        sd.cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 1;
        sd.lds_per_cu = prop.maxSharedMemoryPerMultiProcessor;
        if (hipDeviceGetAttribute(&sd.clock_khz, hipDeviceAttributeWallClockRate, device) != hipSuccess)
            sd.clock_khz = 0;
        sd.ready.store(1, std::memory_order_release);
    }
    maze_ctx ctx;                                   // on the stack: nothing is allocated
    student_bind(&ctx, d, w64, max_steps, sd.scratch_ptr, L);
    ctx.device = device;
    ctx.cus = sd.cus;
    ctx.lds_per_cu = sd.lds_per_cu;
    ctx.clock_khz = sd.clock_khz;
    // every word of the array that the rollout reads is written by the packing kernel first
    // (state and grids of envs 0..N-1), so contents left by an earlier call do not matter
    int rc2 = maze_reset_to_levels(&ctx, d_walls, d_agent_xy, d_agent_dir, d_goal_xy, stream);
    if (rc2 != MAZE_OK) return rc2;
    return maze_step(&ctx, d_actions, n_steps, d_reward, d_done, d_obs, stream);
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

// The setter that goes with k_get_state: parts given as nullptr are kept.
__global__ void k_set_state(StudentDev p, const int32_t *xy, const int8_t *dir, const int32_t *t)
{
    int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= p.N) return;
    const uint32_t pose = p.pose[n];
    int d = (pose >> 16) & 3, X, Y;
    frame_to_padded(p, d, pose & 255, (pose >> 8) & 255, X, Y);
    if (xy) {
        X = min(max(xy[2 * n], 0), p.W - 1) + p.P;
        Y = min(max(xy[2 * n + 1], 0), p.H - 1) + p.P;
    }
    if (dir) d = dir[n] & 3;
    int xd, yd;
    padded_to_frame(p, d, X, Y, xd, yd);
    p.pose[n] = (uint32_t)xd | ((uint32_t)yd << 8) | ((uint32_t)d << 16);
    if (t) p.tcount[n] = (uint32_t)min(max(t[n], 0), p.max_steps - 1);
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
    MAZE_DEVICE_CHECK(ctx);
    const StudentDev &p = ctx->dev;
    hipLaunchKernelGGL(k_get_state, dim3((p.N + 255) / 256), dim3(256), 0, (hipStream_t)stream, p,
                       d_xy, d_dir, d_t);
    MAZE_HIP_CHECK(hipGetLastError());
    return MAZE_OK;
}

extern "C" int maze_set_state(maze_ctx *ctx, const int32_t *d_xy, const int8_t *d_dir,
                              const int32_t *d_t, void *stream)
{
    if (!ctx) return MAZE_ENULL;
    if (!d_xy && !d_dir && !d_t) return MAZE_OK;
    MAZE_DEVICE_CHECK(ctx);
    const StudentDev &p = ctx->dev;
    hipLaunchKernelGGL(k_set_state, dim3((p.N + 255) / 256), dim3(256), 0, (hipStream_t)stream, p,
                       d_xy, d_dir, d_t);
    MAZE_HIP_CHECK(hipGetLastError());
    return MAZE_OK;
}

extern "C" int maze_get_levels(maze_ctx *ctx, int8_t *d_walls, int32_t *d_agent_xy,
                               int8_t *d_agent_dir, int32_t *d_goal_xy, void *stream)
{
    if (!ctx) return MAZE_ENULL;
    MAZE_DEVICE_CHECK(ctx);
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
