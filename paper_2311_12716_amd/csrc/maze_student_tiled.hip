// Tiled store-layout kernels of the student env.
//
// A workgroup owns 64 consecutive envs for the whole rollout.  Per step one lane
// per env advances the env (state in registers, wall rows from LDS) and builds
// its observation as a BIT STREAM -- bit i of the stream is byte i of the env's
// k*k*3 observation, which is 0 or 1 -- and leaves it in LDS.  The 64 streams,
// concatenated, are exactly the 64*3k^2 contiguous output bytes of this time
// step, so other lanes then take 16 consecutive stream bits each (they may
// straddle two envs), expand each bit to a byte and write 16 contiguous bytes;
// consecutive lanes take consecutive pieces, so one store instruction of a wave
// writes 1 KB of contiguous, aligned output.
#include "maze_internal.h"
#include "maze_student_device.h"

namespace {

template <int K>
struct View {
    static constexpr int CELLS = K * K;
    static constexpr int SB = 3 * CELLS;           // stream bits (= obs bytes) per env
    static constexpr int ND = (SB + 31) / 32;      // data dwords per env record
    static constexpr int REC = ND + 1;             // record = data dwords + one zero dword
    static constexpr int NWIN = 4 * SB;            // 16-bit windows per 64-env step
    static constexpr int ROUNDS = (NWIN + 63) / 64;
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

// Per-workgroup LDS carve-up (dword offsets).  Two record buffers so that the
// producer wave can build step s+1 while the consumer waves drain step s; each
// buffer also carries the step's reward (float bits) and done flag per env.
template <int K, typename Word>
struct Lds {
    static constexpr int LUT = 0;
    static constexpr int BUF_REC = 0;                             // inside a buffer
    static constexpr int BUF_REW = 64 * View<K>::REC;
    static constexpr int BUF_DONE = BUF_REW + 64;
    static constexpr int BUF_SIZE = BUF_DONE + 64;
    static constexpr int BUF0 = View<K>::LUTN;
    static constexpr int GRID0 = BUF0 + 2 * BUF_SIZE;
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
__device__ __forceinline__ void produce_record(const uint32_t *lut, uint32_t *rec,
                                               const Word (&rows)[K], int xd, int gf, int gc)
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
        uint32_t piece = lut[idx];
        const int off = V::ROWBITS * r, q = off >> 5, b = off & 31;
        D[q] |= piece << b;
        if (b + V::ROWBITS > 32) D[q + 1] |= piece >> (32 - b);
    }
#pragma unroll
    for (int q = 0; q < V::REC; ++q) rec[q] = D[q];
    // goal: an empty cell (100b) becomes a goal cell (010b): flip stream bits 3c+1, 3c+2
    // (gf, gc) = goal position relative to the agent: cells ahead, cells to the right
    int f = gf;
    int c = gc + h;                                // view column
    bool inview = ((unsigned)f < (unsigned)K) & ((unsigned)c < (unsigned)K);
    int cell = (K - 1 - f) * K + c;
    int bit = 3 * cell + 1;
    if (inview) {
        int q = bit >> 5, b = bit & 31;
        atomicXor(&rec[q], 3u << b);
        if (b == 31) atomicXor(&rec[q + 1], 1u);
    }
}

// Lane-constant description of the 16 stream bits a lane expands in one round.
// In round j lane l takes window 64*j + l, so one store instruction of the wave
// writes 64 consecutive 16-byte pieces = 1 KB of contiguous output.
// Dword indices are relative to the first record of the buffer.
struct Window {
    int addr0;      // first dword holding the window (in env e0's record)
    int addr1;      // env e0+1's first dword, or e0's zero dword when the window ends in e0
    int sh;         // bit offset of the window inside addr0's dword
    int rem;        // bits taken from env e0 when fewer than 16, else 0 (then addr1 reads zero)
    int active;     // window exists (the last round is partial)
    uint32_t out;   // byte offset of the window's 16 output bytes in the workgroup's block
};

template <int K>
__device__ __forceinline__ Window make_window(int lane, int round)
{
    using V = View<K>;
    Window w;
    int m = round * 64 + lane;
    w.active = m < V::NWIN;
    int mm = w.active ? m : 0;
    int bitpos = 16 * mm;
    int e0 = bitpos / V::SB;
    int s = bitpos - e0 * V::SB;
    int rec0 = e0 * V::REC;
    w.addr0 = rec0 + (s >> 5);
    w.sh = s & 31;
    int rem = V::SB - s;
    w.rem = rem < 16 ? rem : 0;
    w.addr1 = rem < 16 ? rec0 + V::REC : rec0 + V::ND;
    w.out = 16u * mm;
    return w;
}

// Expand one 16-bit window of the concatenated streams into 16 output bytes.
__device__ __forceinline__ void consume_window(const uint32_t *recs, const Window &w, int8_t *block)
{
    uint32_t lo = recs[w.addr0], hi = recs[w.addr0 + 1], nx = recs[w.addr1];
    // bits [s, s+16) of env e0 (zero beyond its end), then env e0+1 from bit 0; when the
    // window ends inside e0, nx is e0's zero dword and the shift amount is irrelevant
    uint32_t bits = __builtin_amdgcn_alignbit(hi, lo, w.sh) | (nx << w.rem);
    uint4 a;
    a.x = expand_nibble(bits & 15);          a.y = expand_nibble((bits >> 4) & 15);
    a.z = expand_nibble((bits >> 8) & 15);   a.w = expand_nibble((bits >> 12) & 15);
    *(uint4 *)(block + w.out) = a;
}

template <int K, typename Word>
__device__ __forceinline__ void fill_lut(uint32_t *lds, int tid, int nthreads)
{
    using V = View<K>;
    for (int i = tid; i < V::LUTN; i += nthreads) {
        uint32_t v = 0;
#pragma unroll
        for (int c = 0; c < K; ++c) v |= (((i >> c) & 1) ? 1u : 4u) << (3 * c);
        lds[Lds<K, Word>::LUT + i] = v;
    }
}

// Copy the workgroup's 64 envs' grids into LDS (all threads take part).
template <int K, typename Word>
__device__ __forceinline__ void stage_grids(const StudentDev &p, uint32_t *lds, int tid, int nthreads,
                                            int env0)
{
    const int gs = Lds<K, Word>::grid_stride(p.SP);
    uint32_t *base = lds + Lds<K, Word>::GRID0;
    const int per_env = 4 * p.SP * WordOps<Word>::DW;
    const uint32_t *src = (const uint32_t *)p.grids + (size_t)env0 * per_env;
    int e = 0, o = tid;
    while (o >= per_env) { o -= per_env; ++e; }
    while (e < 64) {
        base[e * gs + o] = src[(size_t)e * per_env + o];
        o += nthreads;
        while (o >= per_env) { o -= per_env; ++e; }
    }
}

constexpr int ACT_RING = 8;   // action prefetch distance of the producer wave, in steps

// ------------------------------------------------------------------ rollout
// Workgroup = 64 envs = one PRODUCER wave + NC CONSUMER waves.
//   producer : lane = env.  Per step: action -> move -> goal/done/reset -> view rows
//              -> stream record, reward, done into LDS buffer s&1.  Its only global
//              traffic is the action byte, prefetched ACT_RING steps ahead, so it never
//              waits for a store to be acknowledged.
//   consumer : after the step's barrier, expands buffer s&1 into the step's
//              64*3k^2 contiguous obs bytes, 1 KB per store instruction (round j
//              of the windows goes to consumer j % NC); the last consumer also writes the
//              reward and done rows.  Consumers never load from global memory.
// One barrier per step: the producer arrives after building step s, the consumers
// after draining step s-1, so buffer s&1 is rewritten (step s+2) only after its
// readers have passed the next barrier.
template <int K, typename Word, bool GRID_LDS, int NC>
__global__ __launch_bounds__(64 * (1 + NC)) void k_student_rollout(
    StudentDev p, const int8_t *__restrict__ actions, int n_steps, float *__restrict__ reward,
    uint8_t *__restrict__ done, int8_t *__restrict__ obs)
{
    using V = View<K>;
    using L = Lds<K, Word>;
    extern __shared__ uint32_t lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int env0 = blockIdx.x * 64;

    fill_lut<K, Word>(lds, tid, 64 * (1 + NC));
    if (GRID_LDS) stage_grids<K, Word>(p, lds, tid, 64 * (1 + NC), env0);
    __syncthreads();

    if (wave == 0) {
        // ------------------------------------------------------------ producer
        const int n = env0 + lane;
        const int gs = GRID_LDS ? L::grid_stride(p.SP) : 0;
        const uint32_t *lds_env = lds + L::GRID0 + lane * gs;
        const Word *glob_env = (const Word *)p.grids + (size_t)n * 4 * p.SP;
        const uint32_t *lut = lds + L::LUT;
        uint32_t pose = p.pose[n];
        int xd = pose & 255, yd = (pose >> 8) & 255, d = (pose >> 16) & 3;
        uint32_t t = p.tcount[n];
        const uint32_t start = p.start[n];
        const int sxd = start & 255, syd = (start >> 8) & 255, sd = (start >> 16) & 3;
        // goal relative to the agent in the agent's own frame: gf cells ahead, gc cells to
        // the right.  Turning rotates this vector, moving forward shortens gf; no goal
        // coordinates are needed inside the loop.
        const uint32_t g_now = p.goalrot[4 * (size_t)n + d], g_start = p.goalrot[4 * (size_t)n + sd];
        int gf = yd - (int)(g_now >> 8), gc = (int)(g_now & 255) - xd;
        const int sgf = syd - (int)(g_start >> 8), sgc = (int)(g_start & 255) - sxd;
        const uint32_t tmax = (uint32_t)p.max_steps;
        const double slope = p.reward_slope;
        const int HPm1 = p.HP - 1, WPm1 = p.WP - 1;

        Word rows[K];
        load_view_rows<K, Word, GRID_LDS>(lds_env, glob_env, p.SP, d, yd, rows);
        Word ahead = rows[K - 2];           // wall word of the row just ahead of the agent

        // one env step + observation record into LDS buffer s&1, then the step's barrier
        auto step = [&](int s, uint32_t a) __attribute__((always_inline)) {
            // ---- dynamics (branch-free)
            t += 1;
            const int blocked = (int)((ahead >> xd) & 1);
            const int odd = d & 1;
            const int rows_m1 = odd ? HPm1 : WPm1;
            const int bits_m1 = odd ? WPm1 : HPm1;
            const int tl = (a == 0), tr = (a == 1), fw = (a == 2) & (blocked ^ 1);
            const int x_l = rows_m1 - yd, y_r = bits_m1 - xd, y_f = yd - fw;
            const int nx = tl ? x_l : (tr ? yd : xd);
            const int ny = tl ? xd : (tr ? y_r : y_f);
            const int nf = tl ? -gc : (tr ? gc : gf - fw);
            const int nc = tl ? gf : (tr ? -gf : gc);
            d = (d + 3 * tl + tr) & 3;
            const int reached = ((nf | nc) == 0);
            const int fin = reached | (t >= tmax);
            const float r = reached ? (float)(1.0 - (double)t * slope) : 0.0f;
            xd = fin ? sxd : nx;
            yd = fin ? syd : ny;
            d = fin ? sd : d;
            t = fin ? 0u : t;
            gf = fin ? sgf : nf;
            gc = fin ? sgc : nc;
            // ---- observation of the new state -> LDS buffer s&1
            uint32_t *buf = lds + L::BUF0 + (s & 1) * L::BUF_SIZE;
            load_view_rows<K, Word, GRID_LDS>(lds_env, glob_env, p.SP, d, yd, rows);
            ahead = rows[K - 2];
            buf[L::BUF_REW + lane] = __float_as_uint(r);
            buf[L::BUF_DONE + lane] = (uint32_t)fin;
            produce_record<K, Word>(lut, buf + L::BUF_REC + lane * V::REC, rows, xd, gf, gc);
            __syncthreads();
        };

        // actions are prefetched ACT_RING steps ahead (indices clamped to the last step, so
        // every load is unconditional and stays in flight across the steps in between)
        // (read as unsigned bytes: values other than 0, 1, 2 are no-ops either way)
        const uint8_t *act = (const uint8_t *)actions + n;
        const int last = n_steps - 1;
        uint32_t ring[ACT_RING];
#pragma unroll
        for (int i = 0; i < ACT_RING; ++i) ring[i] = act[(size_t)min(i, last) * p.N];
        int s = 0;
        for (; s + ACT_RING <= n_steps; s += ACT_RING) {
#pragma unroll
            for (int i = 0; i < ACT_RING; ++i) {
                const uint32_t a = ring[i];
                ring[i] = act[(size_t)min(s + i + ACT_RING, last) * p.N];
                step(s + i, a);
            }
        }
        // fewer than ACT_RING steps left: their actions are ring[0..]
#pragma unroll
        for (int i = 0; i < ACT_RING - 1; ++i)
            if (s + i < n_steps) step(s + i, ring[i]);
        p.pose[n] = (uint32_t)xd | ((uint32_t)yd << 8) | ((uint32_t)d << 16);
        p.tcount[n] = t;
        __syncthreads();
    } else {
        // ------------------------------------------------------------ consumer
        const int c = wave - 1;
        constexpr int MYR = (V::ROUNDS + NC - 1) / NC;     // rounds per consumer, at most
        Window win[MYR];
#pragma unroll
        for (int j = 0; j < MYR; ++j) {
            int round = c + j * NC;
            win[j] = make_window<K>(lane, round < V::ROUNDS ? round : 0);
            if (round >= V::ROUNDS) win[j].active = 0;
        }
        const size_t step_obs = (size_t)p.N * V::SB;
        int8_t *block = obs + (size_t)env0 * V::SB;
        float *rw = reward + env0 + lane;
        uint8_t *dn = done + env0 + lane;
        for (int s = 0; s < n_steps; ++s) {
            __syncthreads();
            const uint32_t *buf = lds + L::BUF0 + (s & 1) * L::BUF_SIZE;
#pragma unroll
            for (int j = 0; j < MYR; ++j)
                if (win[j].active) consume_window(buf + L::BUF_REC, win[j], block);
            if (c == NC - 1) {
                *rw = __uint_as_float(buf[L::BUF_REW + lane]);
                *dn = (uint8_t)buf[L::BUF_DONE + lane];
            }
            block += step_obs;
            rw += p.N;
            dn += p.N;
        }
        __syncthreads();
    }
}

// ---------------------------------------------------- observation of the state
// One wave per 64 envs: produce the records, then expand them (no time loop).
template <int K, typename Word>
__global__ __launch_bounds__(64) void k_render_tiled(StudentDev p, int8_t *__restrict__ obs)
{
    using V = View<K>;
    using L = Lds<K, Word>;
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x;
    const int env0 = blockIdx.x * 64;
    const int n = env0 + lane;
    fill_lut<K, Word>(lds, lane, 64);
    __syncthreads();
    const Word *glob_env = (const Word *)p.grids + (size_t)n * 4 * p.SP;
    uint32_t pose = p.pose[n];
    int xd = pose & 255, yd = (pose >> 8) & 255, d = (pose >> 16) & 3;
    Word rows[K];
    load_view_rows<K, Word, false>(nullptr, glob_env, p.SP, d, yd, rows);
    uint32_t *buf = lds + L::BUF0;
    const uint32_t g = p.goalrot[4 * (size_t)n + d];
    produce_record<K, Word>(lds + L::LUT, buf + L::BUF_REC + lane * V::REC, rows, xd,
                            yd - (int)(g >> 8), (int)(g & 255) - xd);
    __syncthreads();
    int8_t *block = obs + (size_t)env0 * V::SB;
#pragma unroll
    for (int j = 0; j < V::ROUNDS; ++j) {
        Window w = make_window<K>(lane, j);
        if (w.active) consume_window(buf + L::BUF_REC, w, block);
    }
}

template <int K, typename Word>
int launch_k(const maze_ctx *ctx, const int8_t *d_actions, int n_steps, float *d_reward,
             uint8_t *d_done, int8_t *d_obs, int groups, hipStream_t st)
{
    using V = View<K>;
    constexpr int NC = V::ROUNDS < 3 ? V::ROUNDS : 3;      // consumer waves per workgroup
    const StudentDev &p = ctx->dev;
    // stage the grids in LDS when the workgroup's 64 envs fit in 64 KB, else read rows from L2
    bool grid_lds = Lds<K, Word>::bytes(p.SP, true) <= 64 * 1024;
    size_t shmem = Lds<K, Word>::bytes(p.SP, grid_lds);
    size_t shmem_render = Lds<K, Word>::bytes(p.SP, false);
    dim3 grid(groups), block(64 * (1 + NC));
    if (n_steps == 0) {
        hipLaunchKernelGGL((k_render_tiled<K, Word>), grid, dim3(64), shmem_render, st, p, d_obs);
    } else if (grid_lds) {
        hipLaunchKernelGGL((k_student_rollout<K, Word, true, NC>), grid, block, shmem, st, p,
                           d_actions, n_steps, d_reward, d_done, d_obs);
    } else {
        hipLaunchKernelGGL((k_student_rollout<K, Word, false, NC>), grid, block, shmem, st, p,
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
