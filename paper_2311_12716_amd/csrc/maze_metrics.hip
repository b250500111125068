// Level metrics of the student env's current levels: number of walls and shortest
// path length from the start cell to the goal cell.
//
// The wall grid is already held as one bit per cell, one word per row, so the
// breadth-first search is a flood over row bitmaps: a lane owns one row of one env
// and repeats
//     reach' = (reach | reach << 1 | reach >> 1 | row above | row below) & free
// where the neighbouring rows come from the neighbouring lanes of the wave (DPP wave
// shifts).  The number of rounds until the goal's bit appears is the path length; rounds
// that change nothing mean the goal cannot be reached.
#include "maze_internal.h"
#include "maze_student_device.h"

namespace {

// The value of a neighbouring lane by a DPP wave shift (one full-rate instruction per dword,
// no LDS crossbar).  SHR = true: lane i reads lane i-1; false: lane i reads lane i+1.  Which
// lane a shift really delivers is not assumed: the kernel shifts the lane numbers once and
// derives its edge masks from what arrives.
template <bool SHR>
__device__ __forceinline__ uint32_t wave_shift1(uint32_t v)
{
    return __builtin_amdgcn_update_dpp(0u, v, SHR ? 0x138 /* wave_shr:1 */ : 0x130 /* wave_shl:1 */, 0xf,
                                       0xf, true);
}
template <bool SHR, typename Word>
__device__ __forceinline__ Word wave_shift1_word(Word v)
{
    if (sizeof(Word) == 4) return (Word)wave_shift1<SHR>((uint32_t)v);
    const uint32_t lo = wave_shift1<SHR>((uint32_t)v), hi = wave_shift1<SHR>((uint32_t)((uint64_t)v >> 32));
    return (Word)(((uint64_t)hi << 32) | lo);
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

    // A shifted value counts only if it comes from the row above or below in the same env (lane
    // numbers differ by one, same group, row inside the grid).  Lane numbers travel as lane + 1,
    // so a lane at the wave's edge, which receives 0, reads "no lane".
    const uint32_t from_a = wave_shift1<true>((uint32_t)lane + 1) - 1, from_b = wave_shift1<false>((uint32_t)lane + 1) - 1;
    auto neighbour_ok = [&](uint32_t from) {
        const int fg = (int)from / G, fr = (int)from - fg * G;
        return from < 64u && fg == group && (fr == r - 1 || fr == r + 1) && fr < p.H && row_live;
    };
    const Word keep_a = neighbour_ok(from_a) ? ~(Word)0 : (Word)0;
    const Word keep_b = neighbour_ok(from_b) ? ~(Word)0 : (Word)0;

    Word reach = (row_live && r == sy) ? (Word)(((Word)1 << sx) & free_cells) : (Word)0;
    const Word goal_bit = (row_live && r == gy) ? (Word)((Word)1 << gx) : (Word)0;
    int dist = -1;                               // set by the goal's lane in the round its bit appears
    bool running = env_live;
    const int max_rounds = p.H * p.W;            // a shortest path visits no cell twice
    // rounds between two looks at who is done: more on the large grids, whose paths are long
    constexpr int CHECK = sizeof(Word) == 8 ? 16 : 4;
    // One round of the flood.  With one env per wave (G = 64) nothing has to be masked: a lane
    // at the wave's edge receives 0 from the shift, and the lanes of rows beyond the grid hold
    // no free cell, so they never hold or pass on a reached one.
    auto flood = [&](Word from) {
        Word a = wave_shift1_word<true>(from), b = wave_shift1_word<false>(from);
        if (G != 64) { a &= keep_a; b &= keep_b; }
        return (Word)((from | (from << 1) | (from >> 1) | a | b) & free_cells);
    };
    for (int round0 = 0; round0 <= max_rounds; round0 += CHECK) {
        // the goal's bit is looked for once per CHECK rounds; the lane that finds it then
        // replays the rounds since the last look (the wave's other lanes replay with it, their
        // results are not used) to learn in which of them it appeared
        const Word before = reach;
        const bool here = dist < 0 && (reach & goal_bit) != 0;       // reached by round0
#pragma unroll
        for (int i = 0; i < CHECK; ++i) reach = flood(reach);
        const bool changed = reach != before;    // the flood only grows: no change over these rounds = none in any
        if (here) dist = round0;
        const bool late = dist < 0 && (reach & goal_bit) != 0;       // reached in rounds round0+1 .. round0+CHECK
        if (__any(late)) {
            Word again = before;
#pragma unroll
            for (int i = 1; i <= CHECK; ++i) {
                again = flood(again);
                if (late && dist < 0 && (again & goal_bit) != 0) dist = round0 + i;
            }
        }
        // an env is done when its goal lane has a distance or nothing changed in these rounds
        const uint64_t found = __ballot(dist >= 0) & gmask, moving = __ballot(changed) & gmask;
        if (found || !moving) running = false;
        if (!__any(running)) break;
    }
    // the goal's lane holds the distance; hand it to the env's first lane
    const uint64_t holder = __ballot(dist >= 0) & gmask;
    const int src_lane = holder ? __ffsll((long long)holder) - 1 : lane;
    dist = __shfl(dist, src_lane);
    if (env_live && r == 0) {
        if (n_walls) n_walls[n] = count;
        if (path_len) path_len[n] = dist;
    }
}

}  // namespace

extern "C" int maze_level_metrics(maze_ctx *ctx, int32_t *d_n_walls, int32_t *d_path_len, void *stream)
{
    if (!ctx) return MAZE_ENULL;
    MAZE_DEVICE_CHECK(ctx);
    if (!d_n_walls && !d_path_len) return MAZE_OK;
    const StudentDev &p = ctx->dev;
    // one lane per row of an env: H <= 64 holds for every context maze_create makes
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
