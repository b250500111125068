// Tiled store-layout kernels of the student env.
//
// One wavefront owns 64 consecutive envs for the whole rollout.  Per step each
// lane advances its own env (state in registers, wall rows from LDS), builds the
// env's observation as a BIT STREAM -- bit i of the stream is byte i of the
// env's k*k*3 observation, which is 0 or 1 -- and leaves it in LDS.  The wave's
// 64 streams, concatenated, are exactly the 64*3k^2 contiguous output bytes of
// this time step, so the lanes then switch roles: lane m takes 32 consecutive
// stream bits (they may straddle two envs), expands each bit to a byte and
// writes 32 contiguous bytes with two 16-byte stores.  Every obs byte leaves the
// CU in an aligned, fully used 16-byte store.
#include "maze_internal.h"
#include "maze_student_device.h"

namespace {

template <int K>
struct View {
    static constexpr int CELLS = K * K;
    static constexpr int SB = 3 * CELLS;           // stream bits (= obs bytes) per env
    static constexpr int ND = (SB + 31) / 32;      // data dwords per env record
    static constexpr int REC = ND + 1;             // record = data dwords + one zero dword
    static constexpr int NSD = 2 * SB;             // stream dwords per 64-env wave-step
    static constexpr int ROUNDS = (NSD + 63) / 64;
    static constexpr int LUTN = 1 << K;            // row pattern -> 3K stream bits
    static constexpr int ROWBITS = 3 * K;
};

// 4 stream bits -> 4 bytes (bit j -> byte j).  The four shifted copies do not
// overlap, so the multiply carries nothing.
__device__ __forceinline__ uint32_t expand_nibble(uint32_t nib)
{
    return (nib * 0x00204081u) & 0x01010101u;
}

template <typename Word> struct WordOps;
template <> struct WordOps<uint32_t> { static constexpr int DW = 1; };
template <> struct WordOps<uint64_t> { static constexpr int DW = 2; };

// Per-wave LDS carve-up (dword offsets).
template <int K, typename Word>
struct Lds {
    static constexpr int LUT = 0;
    static constexpr int REC0 = View<K>::LUTN;
    static constexpr int GRID0 = REC0 + 64 * View<K>::REC;
    __host__ __device__ static int grid_stride(int SP)       // dwords per env, odd
    {
        return (4 * SP * WordOps<Word>::DW + 4) | 1;
    }
    __host__ static size_t bytes(int SP, bool grid_in_lds)
    {
        return 4 * (size_t)(GRID0 + (grid_in_lds ? 64 * grid_stride(SP) : 64 * 5));
    }
};

// Row r of the view of an env (r = 0 farthest).  The words come from LDS or, for
// grids too large to stage, from the packed grids in global memory.
template <int K, typename Word, bool GRID_LDS>
__device__ __forceinline__ void load_view_rows(const uint32_t *lds_env, const Word *glob_env, int SP,
                                               int d, int yd, Word (&rows)[K])
{
    int first = d * SP + yd - (K - 1);
    if (GRID_LDS) {
        if (sizeof(Word) == 4) {
#pragma unroll
            for (int r = 0; r < K; ++r) rows[r] = (Word)lds_env[first + r];
        } else {
#pragma unroll
            for (int r = 0; r < K; ++r) {
                uint32_t lo = lds_env[2 * (first + r)], hi = lds_env[2 * (first + r) + 1];
                rows[r] = (Word)(((uint64_t)hi << 32) | lo);
            }
        }
    } else {
#pragma unroll
        for (int r = 0; r < K; ++r) rows[r] = glob_env[first + r];
    }
}

// Build the env's stream record from its view rows and leave it in LDS.
template <int K, typename Word>
__device__ __forceinline__ void produce_record(uint32_t *lds, int lane, const Word (&rows)[K], int xd,
                                               int yd, uint32_t goal)
{
    using V = View<K>;
    constexpr int h = K / 2;
    uint32_t D[V::REC];
#pragma unroll
    for (int q = 0; q < V::REC; ++q) D[q] = 0;
    const int sh = xd - h;
#pragma unroll
    for (int r = 0; r < K; ++r) {
        uint32_t idx = (uint32_t)(rows[r] >> sh) & (V::LUTN - 1);
        uint32_t piece = lds[Lds<K, Word>::LUT + idx];
        constexpr int dummy = 0; (void)dummy;
        const int off = V::ROWBITS * r, q = off >> 5, b = off & 31;
        D[q] |= piece << b;
        if (b + V::ROWBITS > 32) D[q + 1] |= piece >> (32 - b);
    }
    uint32_t *rec = lds + Lds<K, Word>::REC0 + lane * V::REC;
#pragma unroll
    for (int q = 0; q < V::REC; ++q) rec[q] = D[q];
    // goal: an empty cell (100b) becomes a goal cell (010b): flip stream bits 3c+1, 3c+2
    int f = yd - (int)(goal >> 8);                 // rows ahead of the agent
    int c = (int)(goal & 255) - xd + h;            // view column
    bool inview = ((unsigned)f < (unsigned)K) & ((unsigned)c < (unsigned)K);
    int cell = (K - 1 - f) * K + c;
    int bit = 3 * cell + 1;
    if (inview) {
        int q = bit >> 5, b = bit & 31;
        atomicXor(&rec[q], 3u << b);
        if (b == 31) atomicXor(&rec[q + 1], 1u);
    }
}

// Lane-constant description of the 32 stream bits a lane expands in one round.
struct Window {
    int addr0;      // dword index in LDS of the first dword holding the window (env e0)
    int addr1;      // dword index of env e0+1's first dword, or of a zero dword
    int sh;         // bit offset of the window inside addr0's dword
    int rem;        // bits the window takes from env e0 (capped at 32)
    int active;     // window exists (last round is partial)
    uint32_t out;   // byte offset of the window's 32 output bytes in the wave's block
};

template <int K, typename Word>
__device__ __forceinline__ Window make_window(int lane, int round)
{
    using V = View<K>;
    Window w;
    int m = round * 64 + lane;
    w.active = m < V::NSD;
    int mm = w.active ? m : 0;
    int bitpos = 32 * mm;
    int e0 = bitpos / V::SB;
    int s = bitpos - e0 * V::SB;
    int rec0 = Lds<K, Word>::REC0 + e0 * V::REC;
    w.addr0 = rec0 + (s >> 5);
    w.sh = s & 31;
    int rem = V::SB - s;
    w.rem = rem < 32 ? rem : 32;
    w.addr1 = rem < 32 ? rec0 + V::REC : rec0 + V::ND;     // next env, or e0's zero dword
    w.out = 32u * mm;
    return w;
}

template <int K, typename Word>
__device__ __forceinline__ void consume_window(const uint32_t *lds, const Window &w, int8_t *block)
{
    uint32_t lo = lds[w.addr0], hi = lds[w.addr0 + 1], nx = lds[w.addr1];
    uint32_t bits = __builtin_amdgcn_alignbit(hi, lo, w.sh);
    bits |= (w.rem < 32) ? (nx << w.rem) : 0u;
    uint4 a, b;
    a.x = expand_nibble(bits & 15);          a.y = expand_nibble((bits >> 4) & 15);
    a.z = expand_nibble((bits >> 8) & 15);   a.w = expand_nibble((bits >> 12) & 15);
    b.x = expand_nibble((bits >> 16) & 15);  b.y = expand_nibble((bits >> 20) & 15);
    b.z = expand_nibble((bits >> 24) & 15);  b.w = expand_nibble(bits >> 28);
    uint4 *dst = (uint4 *)(block + w.out);
    dst[0] = a;
    dst[1] = b;
}

template <int K, typename Word>
__device__ __forceinline__ void fill_lut(uint32_t *lds, int lane)
{
    using V = View<K>;
    for (int i = lane; i < V::LUTN; i += 64) {
        uint32_t v = 0;
#pragma unroll
        for (int c = 0; c < K; ++c) v |= (((i >> c) & 1) ? 1u : 4u) << (3 * c);
        lds[Lds<K, Word>::LUT + i] = v;
    }
}

// Copy the wave's 64 envs' grids (and their goal tables) into LDS.
template <int K, typename Word>
__device__ __forceinline__ void stage_grids(const StudentDev &p, uint32_t *lds, int lane, int env0,
                                            bool grid_in_lds)
{
    const int gs = grid_in_lds ? Lds<K, Word>::grid_stride(p.SP) : 5;
    const int goff = grid_in_lds ? 4 * p.SP * WordOps<Word>::DW : 0;
    uint32_t *base = lds + Lds<K, Word>::GRID0;
    if (grid_in_lds) {
        const int per_env = 4 * p.SP * WordOps<Word>::DW;
        const uint32_t *src = (const uint32_t *)p.grids + (size_t)env0 * per_env;
        int e = 0, o = lane;
        while (o >= per_env) { o -= per_env; ++e; }
        while (e < 64) {
            base[e * gs + o] = src[(size_t)e * per_env + o];
            o += 64;
            while (o >= per_env) { o -= per_env; ++e; }
        }
    }
    for (int f = 0; f < 4; ++f) base[lane * gs + goff + f] = p.goalrot[4 * (size_t)(env0 + lane) + f];
}

// ------------------------------------------------------------------ rollout
template <int K, typename Word, bool GRID_LDS>
__global__ __launch_bounds__(64) void k_student_tiled(StudentDev p, const int8_t *__restrict__ actions,
                                                      int n_steps, float *__restrict__ reward,
                                                      uint8_t *__restrict__ done,
                                                      int8_t *__restrict__ obs)
{
    using V = View<K>;
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x;
    const int env0 = blockIdx.x * 64;
    const int n = env0 + lane;
    const int gs = GRID_LDS ? Lds<K, Word>::grid_stride(p.SP) : 5;
    const int goff = GRID_LDS ? 4 * p.SP * WordOps<Word>::DW : 0;

    fill_lut<K, Word>(lds, lane);
    stage_grids<K, Word>(p, lds, lane, env0, GRID_LDS);
    __syncthreads();

    const uint32_t *lds_env = lds + Lds<K, Word>::GRID0 + lane * gs;
    const Word *glob_env = (const Word *)p.grids + (size_t)n * 4 * p.SP;
    Window win[V::ROUNDS];
#pragma unroll
    for (int j = 0; j < V::ROUNDS; ++j) win[j] = make_window<K, Word>(lane, j);

    uint32_t pose = p.pose[n];
    int xd = pose & 255, yd = (pose >> 8) & 255, d = (pose >> 16) & 3;
    uint32_t t = p.tcount[n];
    const uint32_t start = p.start[n];
    const int sxd = start & 255, syd = (start >> 8) & 255, sd = (start >> 16) & 3;
    const uint32_t sgoal = lds_env[goff + sd];
    const uint32_t tmax = (uint32_t)p.max_steps;
    const double slope = p.reward_slope;
    const int HPm1 = p.HP - 1, WPm1 = p.WP - 1;

    // wall word of the row just ahead of the agent, for the first step
    Word rows[K];
    load_view_rows<K, Word, GRID_LDS>(lds_env, glob_env, p.SP, d, yd, rows);
    Word ahead = rows[K - 2];

    const size_t step_obs = (size_t)p.N * V::SB;
    int8_t *block = obs + (size_t)env0 * V::SB;
    const int8_t *act = actions + n;
    float *rw = reward + n;
    uint8_t *dn = done + n;

    int a_next = act[0];
    for (int s = 0; s < n_steps; ++s) {
        const int a = a_next;
        if (s + 1 < n_steps) a_next = act[(size_t)(s + 1) * p.N];
        // ---- dynamics
        t += 1;
        const bool blocked = (ahead >> xd) & 1;
        const int rows_m1 = (d & 1) ? HPm1 : WPm1;
        const int bits_m1 = (d & 1) ? WPm1 : HPm1;
        const bool tl = (a == 0), tr = (a == 1), fw = (a == 2) & !blocked;
        const int nx = tl ? rows_m1 - yd : (tr ? yd : xd);
        const int ny = tl ? xd : (tr ? bits_m1 - xd : yd - (fw ? 1 : 0));
        d = (d + (tl ? 3 : 0) + (tr ? 1 : 0)) & 3;
        uint32_t goal = lds_env[goff + d];
        const bool reached = ((uint32_t)nx | ((uint32_t)ny << 8)) == goal;
        const float r = reached ? (float)(1.0 - (double)t * slope) : 0.0f;
        const bool fin = reached | (t >= tmax);
        xd = fin ? sxd : nx;
        yd = fin ? syd : ny;
        d = fin ? sd : d;
        t = fin ? 0u : t;
        goal = fin ? sgoal : goal;
        rw[(size_t)s * p.N] = r;
        dn[(size_t)s * p.N] = fin ? 1 : 0;
        // ---- observation of the new state
        load_view_rows<K, Word, GRID_LDS>(lds_env, glob_env, p.SP, d, yd, rows);
        ahead = rows[K - 2];
        produce_record<K, Word>(lds, lane, rows, xd, yd, goal);
        __syncthreads();
#pragma unroll
        for (int j = 0; j < V::ROUNDS; ++j)
            if (win[j].active) consume_window<K, Word>(lds, win[j], block);
        __syncthreads();
        block += step_obs;
    }
    p.pose[n] = (uint32_t)xd | ((uint32_t)yd << 8) | ((uint32_t)d << 16);
    p.tcount[n] = t;
}

// ---------------------------------------------------- observation of the state
template <int K, typename Word, bool GRID_LDS>
__global__ __launch_bounds__(64) void k_render_tiled(StudentDev p, int8_t *__restrict__ obs)
{
    using V = View<K>;
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x;
    const int env0 = blockIdx.x * 64;
    const int n = env0 + lane;
    fill_lut<K, Word>(lds, lane);
    __syncthreads();
    const Word *glob_env = (const Word *)p.grids + (size_t)n * 4 * p.SP;
    uint32_t pose = p.pose[n];
    int xd = pose & 255, yd = (pose >> 8) & 255, d = (pose >> 16) & 3;
    Word rows[K];
    load_view_rows<K, Word, false>(nullptr, glob_env, p.SP, d, yd, rows);
    produce_record<K, Word>(lds, lane, rows, xd, yd, p.goalrot[4 * (size_t)n + d]);
    __syncthreads();
    int8_t *block = obs + (size_t)env0 * V::SB;
#pragma unroll
    for (int j = 0; j < V::ROUNDS; ++j) {
        Window w = make_window<K, Word>(lane, j);
        if (w.active) consume_window<K, Word>(lds, w, block);
    }
}

template <int K, typename Word>
int launch_k(const maze_ctx *ctx, const int8_t *d_actions, int n_steps, float *d_reward,
             uint8_t *d_done, int8_t *d_obs, int full_waves, hipStream_t st)
{
    const StudentDev &p = ctx->dev;
    // stage the grids in LDS when a wave's 64 envs fit in 64 KB, else read rows from L2
    size_t with_grid = Lds<K, Word>::bytes(p.SP, true);
    bool grid_lds = with_grid <= 64 * 1024;
    size_t shmem = Lds<K, Word>::bytes(p.SP, grid_lds);
    size_t shmem_render = Lds<K, Word>::bytes(p.SP, false);
    if (n_steps == 0) {
        hipLaunchKernelGGL((k_render_tiled<K, Word, false>), dim3(full_waves), dim3(64),
                           shmem_render, st, p, d_obs);
    } else if (grid_lds) {
        hipLaunchKernelGGL((k_student_tiled<K, Word, true>), dim3(full_waves), dim3(64), shmem, st, p,
                           d_actions, n_steps, d_reward, d_done, d_obs);
    } else {
        hipLaunchKernelGGL((k_student_tiled<K, Word, false>), dim3(full_waves), dim3(64), shmem, st, p,
                           d_actions, n_steps, d_reward, d_done, d_obs);
    }
    return 1;
}

}  // namespace

// Launch the tiled kernel on the first `*covered` envs (a multiple of 64) and
// report how many it took; the caller runs the per-cell kernel on the rest.
// n_steps == 0 renders the current state.  Returns 0 if no tiled kernel applies.
int student_tiled_launch(const maze_ctx *ctx, const int8_t *d_actions, int n_steps, float *d_reward,
                         uint8_t *d_done, int8_t *d_obs, int *covered, hipStream_t st)
{
    const StudentDev &p = ctx->dev;
    *covered = 0;
    if (!d_obs) return 0;
    const int K = p.k;
    if (K != 3 && K != 5 && K != 7) return 0;
    // 16-byte stores: every time step's block and the buffer itself must be 16-byte aligned
    if ((((size_t)p.N * 3 * K * K) & 15) != 0 || ((uintptr_t)d_obs & 15) != 0) return 0;
    int full = p.N / 64;
    if (full == 0) return 0;
    int rc;
    if (ctx->word64) {
        if (K == 3) rc = launch_k<3, uint64_t>(ctx, d_actions, n_steps, d_reward, d_done, d_obs, full, st);
        else if (K == 5) rc = launch_k<5, uint64_t>(ctx, d_actions, n_steps, d_reward, d_done, d_obs, full, st);
        else rc = launch_k<7, uint64_t>(ctx, d_actions, n_steps, d_reward, d_done, d_obs, full, st);
    } else {
        if (K == 3) rc = launch_k<3, uint32_t>(ctx, d_actions, n_steps, d_reward, d_done, d_obs, full, st);
        else if (K == 5) rc = launch_k<5, uint32_t>(ctx, d_actions, n_steps, d_reward, d_done, d_obs, full, st);
        else rc = launch_k<7, uint32_t>(ctx, d_actions, n_steps, d_reward, d_done, d_obs, full, st);
    }
    if (rc) *covered = full * 64;
    return rc;
}
