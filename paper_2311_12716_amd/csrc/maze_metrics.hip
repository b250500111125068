// Level metrics of the student env's current levels: number of walls and shortest
// path length from the start cell to the goal cell.
//
// The wall grid is already held as one bit per cell, one word per row, so the
// breadth-first search is a flood over row bitmaps: a lane owns one row of one env
// and repeats
//     reach' = (reach | reach << 1 | reach >> 1 | row above | row below) & free
// where the neighbouring rows come from the neighbouring lanes of the wave.  The
// number of rounds until the goal's bit appears is the path length; a round that
// changes nothing means the goal cannot be reached.
#include "maze_internal.h"
#include "maze_student_device.h"

namespace {

template <typename Word>
__device__ __forceinline__ Word shuffle_up1(Word v)
{
    if (sizeof(Word) == 4) return (Word)__shfl_up((unsigned)v, 1);
    return (Word)__shfl_up((unsigned long long)v, 1);
}

template <typename Word>
__device__ __forceinline__ Word shuffle_down1(Word v)
{
    if (sizeof(Word) == 4) return (Word)__shfl_down((unsigned)v, 1);
    return (Word)__shfl_down((unsigned long long)v, 1);
}

// G = lanes per env (a power of two >= H, at most 64); a wave serves 64 / G envs.
template <typename Word>
__global__ __launch_bounds__(256) void k_level_metrics(StudentDev p, int G, int32_t *__restrict__ n_walls,
                                                       int32_t *__restrict__ path_len)
{
    const int lane = threadIdx.x & 63;
    const int wave_global = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int per_wave = 64 / G;
    const int group = lane / G, r = lane - group * G;          // env within the wave, row
    const int n_raw = wave_global * per_wave + group;
    const bool env_live = n_raw < p.N;
    const int n = env_live ? n_raw : p.N - 1;
    const bool row_live = env_live && r < p.H;
    const uint64_t gmask = (G == 64 ? ~0ull : ((1ull << G) - 1)) << (group * G);

    // interior of row r of the unrotated grid (frame 3), bit x = cell (x, r) is free
    const Word *grid = (const Word *)p.grids + ((size_t)n * 4 + 3) * p.SP;
    const Word interior = (Word)(((Word)1 << p.W) - 1);
    const Word wall = row_live ? (Word)((grid[p.P + (row_live ? r : 0)] >> p.P) & interior) : (Word)0;
    const Word free_cells = row_live ? (Word)(~wall & interior) : (Word)0;

    // wall count: sum over the env's lanes
    int count = sizeof(Word) == 4 ? __popc((unsigned)wall) : __popcll((unsigned long long)wall);
    for (int off = 1; off < G; off <<= 1) count += __shfl_xor(count, off);

    // start and goal cells in interior coordinates
    const uint32_t start = p.start[n];
    int SX, SY;
    frame_to_padded(p, (start >> 16) & 3, start & 255, (start >> 8) & 255, SX, SY);
    const int sx = SX - p.P, sy = SY - p.P;
    const uint32_t goal = p.goalrot[4 * (size_t)n + 3];
    const int gx = (int)(goal & 255) - p.P, gy = (int)((goal >> 8) & 255) - p.P;

    Word reach = (row_live && r == sy) ? (Word)(((Word)1 << sx) & free_cells) : (Word)0;
    const Word goal_bit = (row_live && r == gy) ? (Word)((Word)1 << gx) : (Word)0;
    int dist = -1;
    bool running = env_live;
    const int max_rounds = p.H * p.W;            // a shortest path visits no cell twice
    for (int round = 0; round <= max_rounds; ++round) {
        const uint64_t found = __ballot((reach & goal_bit) != 0) & gmask;
        if (running && found) { dist = round; running = false; }
        Word up = shuffle_up1(reach), down = shuffle_down1(reach);
        if (r == 0) up = 0;
        if (r >= p.H - 1) down = 0;
        const Word grown = (Word)((reach | (reach << 1) | (reach >> 1) | up | down) & free_cells);
        const uint64_t changed = __ballot(grown != reach) & gmask;
        if (running && !changed) running = false;            // flood complete, goal not in it
        reach = grown;
        if (!__any(running)) break;
    }
    if (env_live && r == 0) {
        if (n_walls) n_walls[n] = count;
        if (path_len) path_len[n] = dist;
    }
}

}  // namespace

extern "C" int maze_level_metrics(maze_ctx *ctx, int32_t *d_n_walls, int32_t *d_path_len, void *stream)
{
    if (!ctx) return MAZE_ENULL;
    if (!d_n_walls && !d_path_len) return MAZE_OK;
    const StudentDev &p = ctx->dev;
    if (p.H > 64) return MAZE_ESIZE;             // one lane per row of an env
    int G = 1;
    while (G < p.H) G <<= 1;
    const int per_wave = 64 / G;
    const long long waves = ((long long)p.N + per_wave - 1) / per_wave;
    const unsigned blocks = (unsigned)((waves + 3) / 4);
    hipStream_t st = (hipStream_t)stream;
    if (ctx->word64)
        hipLaunchKernelGGL(k_level_metrics<uint64_t>, dim3(blocks), dim3(256), 0, st, p, G, d_n_walls,
                           d_path_len);
    else
        hipLaunchKernelGGL(k_level_metrics<uint32_t>, dim3(blocks), dim3(256), 0, st, p, G, d_n_walls,
                           d_path_len);
    MAZE_HIP_CHECK(hipGetLastError());
    return MAZE_OK;
}
