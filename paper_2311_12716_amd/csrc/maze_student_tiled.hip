// Tiled store-layout kernels of the student env.
//
// A workgroup owns EPW consecutive envs for the whole rollout: 128 when the batch is
// large enough to fill the GPU that way (128 * 3k^2 bytes per step is a whole number
// of 128-byte lines, so no line of the output is shared between workgroups), 64 or
// 32 for smaller batches or grids whose LDS copy would not fit.  Per step one lane per env advances the env (state in
// registers, wall rows from LDS) and its observation is built as a BIT STREAM --
// bit i of the stream is byte i of the env's k*k*3 observation, which is 0 or 1 --
// and left in LDS.  The EPW streams, concatenated, are exactly the EPW*3k^2
// contiguous output bytes of this time step, so other lanes then take 16 consecutive stream bits each (they may
// straddle two envs), expand each bit to a byte and write 16 contiguous bytes;
// consecutive lanes take consecutive pieces, so one store instruction of a wave
// writes 1 KB of contiguous, aligned output.
//
// The per-step work is a three-stage pipeline over the waves of the workgroup,
// advanced by one barrier per block of SPB steps:
//   first  ("dynamics") block b  : action, move, goal/done/reset, read the K
//                                     wall rows of the new view and publish the
//                                     K x K view bits, the goal offset, reward, done
//   next   ("records")  block b-1: view bits -> stream record (row lookup table),
//                                     goal cell patched in; store reward and done
//   rest   ("stores")   block b-2: expand records to bytes, store obs
// (one dynamics and one records wave per 64 envs)
// Only the dynamics wave carries a dependency from step to step, so the time per
// step is that wave's short chain; the store waves never load from global memory
// and the dynamics wave touches it once every 16 steps (actions, staged in LDS).
#include "maze_internal.h"
#include "maze_student_device.h"

#include <type_traits>

// Compile-time knobs (overridable for measurements).
#ifndef MAZE_SPB
#define MAZE_SPB 2
#endif
#ifndef MAZE_STORE_WAVES
#define MAZE_STORE_WAVES 10
#endif

namespace {

constexpr int SPB = MAZE_SPB;   // steps per barrier: every stage handles SPB steps between barriers

// Compile-time shape of a workgroup: view size K, EPW envs.
template <int K, int EPW>
struct View {
    static constexpr int CELLS = K * K;
    static constexpr int SB = 3 * CELLS;           // stream bits (= obs bytes) per env
    static constexpr int ND = (SB + 31) / 32;      // data dwords per env record
    static constexpr int REC = ND + 1;             // record = data dwords + one zero dword
    static constexpr int LUTN = 1 << K;            // row pattern -> 3K stream bits
    static constexpr int ROWBITS = 3 * K;
    static constexpr int RPD = 32 / K;             // view rows packed per dword
    static constexpr int WV = (K + RPD - 1) / RPD; // dwords of packed view bits
    static constexpr int LA = EPW < 64 ? EPW : 64; // envs (= active lanes) of a dynamics / records wave
    static constexpr int NDYN = EPW / LA;          // dynamics waves (and records waves)
    static constexpr int NWIN = EPW * SB / 16;     // 16-bit windows per workgroup step
    static constexpr int ROUNDS = (NWIN + 63) / 64;
    static constexpr int NC = ROUNDS < MAZE_STORE_WAVES ? ROUNDS : MAZE_STORE_WAVES;   // store waves
    static constexpr int WAVES = 2 * NDYN + NC;
    // actions: one 16-byte load per lane covers 16 envs of one step, so a dynamics wave
    // stages ACT_BLOCK steps of its LA envs per load
    static constexpr int ACT_LPR = LA / 16;
    static constexpr int ACT_BLOCK = 64 / ACT_LPR;
    static_assert((EPW * SB) % 16 == 0, "a step's chunk must be a whole number of 16-byte pieces");
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

// Per-workgroup LDS carve-up (dword offsets).  ST and REC hold SPB steps each and
// are double buffered by block parity (a block = the SPB steps between two barriers).
template <int K, typename Word, int EPW>
struct Lds {
    using V = View<K, EPW>;
    static constexpr int LUT = 0;                                  // [LUTN]
    static constexpr int ACT = LUT + V::LUTN;                      // [2][ACT_BLOCK][EPW] action bytes
    static constexpr int ACT_ROW = EPW;                            // bytes per step
    static constexpr int ST = ACT + 2 * V::ACT_BLOCK * EPW / 4;    // [2][SPB][WV+2][EPW] view bits, goal, out
    static constexpr int ST_SIZE = (V::WV + 2) * EPW;
    static constexpr int REC = ST + 2 * SPB * ST_SIZE;             // [2][SPB][EPW*REC] stream records
    static constexpr int REC_SIZE = EPW * V::REC;
    static constexpr int GRID0 = REC + 2 * SPB * REC_SIZE;         // [EPW][grid_stride]
    __host__ __device__ static int grid_stride(int SP)             // dwords per env, odd
    {
        return (4 * SP * WordOps<Word>::DW) | 1;
    }
    __host__ static size_t bytes(int SP, bool grid_in_lds)
    {
        return 4 * (size_t)(GRID0 + (grid_in_lds ? EPW * grid_stride(SP) : 0));
    }
};

// The K wall words of an env's view (row 0 farthest).  From LDS or, for grids too
// large to stage, from the packed grids in global memory.
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

// K x K view bits (row r, column c -> bit K*(r % RPD) + c of dword r / RPD).
template <int K, typename Word>
__device__ __forceinline__ void pack_view(const Word (&rows)[K], int xd, uint32_t (&vw)[View<K, 64>::WV])
{
    using V = View<K, 64>;
    const int sh = xd - K / 2;
#pragma unroll
    for (int q = 0; q < V::WV; ++q) vw[q] = 0;
#pragma unroll
    for (int r = 0; r < K; ++r) {
        uint32_t bits = sizeof(Word) == 4 ? __builtin_amdgcn_ubfe((uint32_t)rows[r], sh, K)
                                          : (uint32_t)(rows[r] >> sh) & (V::LUTN - 1);
        vw[r / V::RPD] |= bits << (K * (r % V::RPD));
    }
}

// Stream record of one env from its view bits; goal at (gf cells ahead, gc cells to
// the right) of the agent.  An empty cell is 100b, a wall 001b, the goal 010b.
template <int K>
__device__ __forceinline__ void produce_record(const uint32_t *lut, uint32_t *rec,
                                               const uint32_t (&vw)[View<K, 64>::WV], int gf, int gc)
{
    using V = View<K, 64>;
    uint32_t D[V::REC];
#pragma unroll
    for (int q = 0; q < V::REC; ++q) D[q] = 0;
#pragma unroll
    for (int r = 0; r < K; ++r) {
        uint32_t idx = (vw[r / V::RPD] >> (K * (r % V::RPD))) & (V::LUTN - 1);
        uint32_t piece = lut[idx];
        const int off = V::ROWBITS * r, q = off >> 5, b = off & 31;
        D[q] |= piece << b;
        if (b + V::ROWBITS > 32) D[q + 1] |= piece >> (32 - b);
    }
#pragma unroll
    for (int q = 0; q < V::REC; ++q) rec[q] = D[q];
    // goal: the empty cell (100b) becomes a goal cell (010b): flip stream bits 3c+1, 3c+2
    // (a goal that sits on a wall cell -- a level the caller should not build -- shows as wall)
    int c = gc + K / 2;                            // view column
    bool inview = ((unsigned)gf < (unsigned)K) & ((unsigned)c < (unsigned)K);
    const int grow = inview ? K - 1 - gf : 0;      // view row of the goal
    const uint32_t gword = (V::WV == 1 || grow < V::RPD) ? vw[0] : vw[V::WV - 1];
    const int gshift = K * (grow < V::RPD ? grow : grow - V::RPD) + c;
    inview = inview & !((gword >> (gshift & 31)) & 1);
    int cell = (K - 1 - gf) * K + c;
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

template <int K, int EPW>
__device__ __forceinline__ Window make_window(int lane, int round)
{
    using V = View<K, EPW>;
    Window w;
    int m = round * 64 + lane;
    w.active = (round < V::ROUNDS) && (m < V::NWIN);
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

template <int K>
__device__ __forceinline__ void fill_lut(uint32_t *lut, int tid, int nthreads)
{
    using V = View<K, 64>;
    for (int i = tid; i < V::LUTN; i += nthreads) {
        uint32_t v = 0;
#pragma unroll
        for (int c = 0; c < K; ++c) v |= (((i >> c) & 1) ? 1u : 4u) << (3 * c);
        lut[i] = v;
    }
}

// Copy the workgroup's envs' grids into LDS (all threads take part).
template <int K, typename Word, int EPW>
__device__ __forceinline__ void stage_grids(const StudentDev &p, uint32_t *lds, int tid, int nthreads,
                                            int env0)
{
    const int gs = Lds<K, Word, EPW>::grid_stride(p.SP);
    uint32_t *base = lds + Lds<K, Word, EPW>::GRID0;
    const int per_env = 4 * p.SP * WordOps<Word>::DW;
    const uint32_t *src = (const uint32_t *)p.grids + (size_t)env0 * per_env;
    int e = 0, o = tid;
    while (o >= per_env) { o -= per_env; ++e; }
    while (e < EPW) {
        base[e * gs + o] = src[(size_t)e * per_env + o];
        o += nthreads;
        while (o >= per_env) { o -= per_env; ++e; }
    }
}

// ------------------------------------------------------------------ rollout
// Each role runs its own loop over blocks of SPB steps; every wave passes exactly
// ceil(n_steps / SPB) + 3 barriers.
//   between barriers b and b+1:  dynamics builds block b   -> ST[b&1]
//                                records  builds block b-1 -> REC[(b-1)&1]  (reads ST[(b-1)&1])
//                                stores   drain  block b-2                  (read REC[(b-2)&1])
// so no buffer is written while it is read.  The block loops are unrolled by two so
// every LDS address is a lane constant plus an immediate.
template <int K, typename Word, int EPW, bool GRID_LDS, bool SQUARE>
__global__ __launch_bounds__((64 * View<K, EPW>::WAVES)) void k_student_rollout(
    StudentDev p, const int8_t *__restrict__ actions, int n_steps, float *__restrict__ reward,
    uint8_t *__restrict__ done, int8_t *__restrict__ obs)
{
    using V = View<K, EPW>;
    using L = Lds<K, Word, EPW>;
    constexpr int NT = 64 * V::WAVES;
    constexpr int ACT_BLOCK = V::ACT_BLOCK;
    extern __shared__ uint32_t lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int env0 = blockIdx.x * EPW;

    fill_lut<K>(lds + L::LUT, tid, NT);
    if (GRID_LDS) stage_grids<K, Word, EPW>(p, lds, tid, NT, env0);

    if (wave < V::NDYN) {
        // ================================================================ dynamics
        const bool active = lane < V::LA;          // a wave serves LA envs
        const int e = wave * 64 + (active ? lane : 0);   // env within the workgroup
        const int n = env0 + e;
        const int last = n_steps - 1;
        uint32_t pose = p.pose[n];
        int xd = pose & 255, yd = (pose >> 8) & 255, d = (pose >> 16) & 3;
        uint32_t t = p.tcount[n];
        const uint32_t start = p.start[n];
        const int sxd = start & 255, syd = (start >> 8) & 255, sd = (start >> 16) & 3;
        // goal relative to the agent in the agent's own frame: gf cells ahead, gc cells to
        // the right.  Turning rotates this vector, moving forward shortens gf.
        const uint32_t g_now = p.goalrot[4 * (size_t)n + d], g_start = p.goalrot[4 * (size_t)n + sd];
        int gf = yd - (int)(g_now >> 8), gc = (int)(g_now & 255) - xd;
        const int sgf = syd - (int)(g_start >> 8), sgc = (int)(g_start & 255) - sxd;
        const uint32_t tmax = (uint32_t)p.max_steps;
        const int HPm1 = p.HP - 1, WPm1 = p.WP - 1;
        const uint32_t *lds_env = lds + L::GRID0 + e * (GRID_LDS ? L::grid_stride(p.SP) : 0);
        const Word *glob_env = (const Word *)p.grids + (size_t)n * 4 * p.SP;
        // actions: lane l of this wave stages the bytes of step block*ACT_BLOCK + l/ACT_LPR
        // for 16 of the wave's envs (all 64 lanes stage, whatever LA is)
        const int stage_row = lane / V::ACT_LPR;
        const int stage_col = wave * 64 + 16 * (lane % V::ACT_LPR);
        const int8_t *act_lane = actions + env0 + stage_col;
        uint8_t *act_stage = (uint8_t *)(lds + L::ACT) + stage_row * L::ACT_ROW + stage_col;
        auto load_actions = [&](int block) {
            int s = min(block * ACT_BLOCK + stage_row, last);
            return *(const uint4 *)(act_lane + (size_t)s * p.N);
        };
        *(uint4 *)act_stage = load_actions(0);
        uint4 act_regs = load_actions(1);
        __syncthreads();                                             // barrier 0 (set-up)
        Word rows[K];
        load_view_rows<K, Word, GRID_LDS>(lds_env, glob_env, p.SP, d, yd, rows);
        Word ahead = rows[K - 2];          // wall word of the row just ahead of the agent
        const uint8_t *act_lds = (const uint8_t *)(lds + L::ACT) + e;
        uint32_t act_off = 0;              // byte offset of the current step's row in the ring
        uint32_t a_next = act_lds[0];

        auto env_step = [&](int slot) {
            const uint32_t a = a_next;
            act_off = (act_off + L::ACT_ROW) & (2 * ACT_BLOCK * L::ACT_ROW - 1);
            a_next = act_lds[act_off];     // next step's action (staged >= 8 steps ago)
            t += 1;
            const int blocked = sizeof(Word) == 4 ? (int)__builtin_amdgcn_ubfe((uint32_t)ahead, xd, 1)
                                                  : (int)((ahead >> xd) & 1);
            const bool tl = (a == 0), tr = (a == 1);
            const int fw = (a == 2) ? (blocked ^ 1) : 0;
            int rows_m1 = WPm1, bits_m1 = WPm1;
            if (!SQUARE) {
                const bool odd = d & 1;
                rows_m1 = odd ? HPm1 : WPm1;
                bits_m1 = odd ? WPm1 : HPm1;
            }
            const int nx = tl ? rows_m1 - yd : (tr ? yd : xd);
            const int ny = tl ? xd : (tr ? bits_m1 - xd : yd - fw);
            const int nf = tl ? -gc : (tr ? gc : gf - fw);
            const int nc = tl ? gf : (tr ? -gf : gc);
            d = (d + (tl ? 3 : 0) + (tr ? 1 : 0)) & 3;
            const bool reached = ((nf | nc) == 0);
            const bool fin = reached | (t >= tmax);
            // out word: step count if the goal was reached, done in bit 31
            const uint32_t out = (reached ? t : 0u) | (fin ? 0x80000000u : 0u);
            xd = fin ? sxd : nx;
            yd = fin ? syd : ny;
            d = fin ? sd : d;
            t = fin ? 0u : t;
            gf = fin ? sgf : nf;
            gc = fin ? sgc : nc;
            load_view_rows<K, Word, GRID_LDS>(lds_env, glob_env, p.SP, d, yd, rows);
            ahead = rows[K - 2];
            uint32_t vw[V::WV];
            pack_view<K, Word>(rows, xd, vw);
            uint32_t *st = lds + L::ST + slot * L::ST_SIZE + e;
#pragma unroll
            for (int q = 0; q < V::WV; ++q) st[q * EPW] = vw[q];
            st[V::WV * EPW] = (uint32_t)(gf & 0xFFFF) | ((uint32_t)gc << 16);
            st[(V::WV + 1) * EPW] = out;
        };
        auto step = [&](int i, int slot) {
            if (active) env_step(slot);
            // stage the next block of actions half way through the current one
            if ((i & (ACT_BLOCK - 1)) == ACT_BLOCK / 2) {
                const int nb = i / ACT_BLOCK + 1;
                *(uint4 *)(act_stage + (nb & 1) * (ACT_BLOCK * L::ACT_ROW)) = act_regs;
                act_regs = load_actions(nb + 1);
            }
        };
        auto block = [&](int i0, auto PAR) {
#pragma unroll
            for (int u = 0; u < SPB; ++u)
                if (i0 + u < n_steps) step(i0 + u, decltype(PAR)::value * SPB + u);
            __syncthreads();
        };
        int i = 0;
        for (; i + SPB < n_steps; i += 2 * SPB) {
            block(i, std::integral_constant<int, 0>());
            block(i + SPB, std::integral_constant<int, 1>());
        }
        if (i < n_steps) block(i, std::integral_constant<int, 0>());
        if (active) {
            p.pose[n] = (uint32_t)xd | ((uint32_t)yd << 8) | ((uint32_t)d << 16);
            p.tcount[n] = t;
        }
        __syncthreads();
        __syncthreads();
    } else if (wave < 2 * V::NDYN) {
        // ================================================================= records
        const bool active = lane < V::LA;
        const int e = (wave - V::NDYN) * 64 + (active ? lane : 0);
        float *rw = reward + env0 + e;
        uint8_t *dn = done + env0 + e;
        const double slope = p.reward_slope;
        __syncthreads();                                             // barrier 0 (set-up)
        __syncthreads();                                             // block 0 published
        auto step = [&](int slot) {
            const uint32_t *st = lds + L::ST + slot * L::ST_SIZE + e;
            uint32_t vw[V::WV];
#pragma unroll
            for (int q = 0; q < V::WV; ++q) vw[q] = st[q * EPW];
            const uint32_t g = st[V::WV * EPW];
            const uint32_t out = st[(V::WV + 1) * EPW];
            produce_record<K>(lds + L::LUT, lds + L::REC + slot * L::REC_SIZE + e * V::REC, vw,
                              (int)(int16_t)(g & 0xFFFF), (int)g >> 16);
            const uint32_t tr = out & 0x7FFFFFFFu;
            *rw = tr ? (float)(1.0 - (double)tr * slope) : 0.0f;
            *dn = (uint8_t)(out >> 31);
            rw += p.N;
            dn += p.N;
        };
        auto block = [&](int s0, auto PAR) {
#pragma unroll
            for (int u = 0; u < SPB; ++u)
                if (s0 + u < n_steps && active) step(decltype(PAR)::value * SPB + u);
            __syncthreads();
        };
        int s = 0;
        for (; s + SPB < n_steps; s += 2 * SPB) {
            block(s, std::integral_constant<int, 0>());
            block(s + SPB, std::integral_constant<int, 1>());
        }
        if (s < n_steps) block(s, std::integral_constant<int, 0>());
        __syncthreads();
    } else {
        // ================================================================== stores
        const int c = wave - 2 * V::NDYN;
        constexpr int MYR = (V::ROUNDS + V::NC - 1) / V::NC;     // rounds per store wave, at most
        Window win[MYR];
#pragma unroll
        for (int j = 0; j < MYR; ++j) win[j] = make_window<K, EPW>(lane, c + j * V::NC);
        const size_t step_obs = (size_t)p.N * V::SB;
        int8_t *out_block = obs + (size_t)env0 * V::SB;
        __syncthreads();                                             // barrier 0 (set-up)
        __syncthreads();                                             // block 0 published
        __syncthreads();                                             // block 0 recorded
        auto step = [&](int slot) {
            const uint32_t *rec = lds + L::REC + slot * L::REC_SIZE;
#pragma unroll
            for (int j = 0; j < MYR; ++j)
                if (win[j].active) consume_window(rec, win[j], out_block);
            out_block += step_obs;
        };
        auto block = [&](int s0, auto PAR) {
#pragma unroll
            for (int u = 0; u < SPB; ++u)
                if (s0 + u < n_steps) step(decltype(PAR)::value * SPB + u);
            __syncthreads();
        };
        int s = 0;
        for (; s + SPB < n_steps; s += 2 * SPB) {
            block(s, std::integral_constant<int, 0>());
            block(s + SPB, std::integral_constant<int, 1>());
        }
        if (s < n_steps) block(s, std::integral_constant<int, 0>());
    }
}

// ------------------------------- observation of the state / one step + observation
// One workgroup of REPW threads per REPW envs, no time loop: optionally advance every
// env by one step (the call a policy loop makes: state in and out of global memory, wall
// rows from the packed grids in L2), then produce the records and expand them.
constexpr int REPW = 64;

template <int K, typename Word, bool DO_STEP>
__global__ __launch_bounds__(REPW) void k_step_render_tiled(
    StudentDev p, const int8_t *__restrict__ actions, float *__restrict__ reward,
    uint8_t *__restrict__ done, int8_t *__restrict__ obs)
{
    using V = View<K, REPW>;
    using L = Lds<K, Word, REPW>;
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x;
    const int env0 = blockIdx.x * REPW;
    const int n = env0 + lane;
    fill_lut<K>(lds + L::LUT, lane, REPW);
    __syncthreads();
    const Word *glob_env = (const Word *)p.grids + (size_t)n * 4 * p.SP;
    uint32_t pose = p.pose[n];
    if (DO_STEP) {
        const int a = actions[n];
        const int xd0 = pose & 255, yd0 = (pose >> 8) & 255, d0 = (pose >> 16) & 3;
        const bool blocked = (glob_env[d0 * p.SP + yd0 - 1] >> xd0) & 1;
        pose = student_move(p, pose, a, blocked);
        uint32_t t = p.tcount[n] + 1;
        const bool reached = (pose & 0xFFFF) == p.goalrot[4 * (size_t)n + ((pose >> 16) & 3)];
        const bool fin = reached || t >= (uint32_t)p.max_steps;
        reward[n] = reached ? (float)(1.0 - (double)t * p.reward_slope) : 0.0f;
        done[n] = fin ? 1 : 0;
        if (fin) { pose = p.start[n]; t = 0; }
        p.pose[n] = pose;
        p.tcount[n] = t;
    }
    const int xd = pose & 255, yd = (pose >> 8) & 255, d = (pose >> 16) & 3;
    Word rows[K];
    load_view_rows<K, Word, false>(nullptr, glob_env, p.SP, d, yd, rows);
    uint32_t vw[V::WV];
    pack_view<K, Word>(rows, xd, vw);
    const uint32_t g = p.goalrot[4 * (size_t)n + d];
    produce_record<K>(lds + L::LUT, lds + L::REC + lane * V::REC, vw, yd - (int)(g >> 8),
                      (int)(g & 255) - xd);
    __syncthreads();
    int8_t *block = obs + (size_t)env0 * V::SB;
    for (int j = 0; j < V::ROUNDS; ++j) {
        Window w = make_window<K, REPW>(lane, j);
        if (w.active) consume_window(lds + L::REC, w, block);
    }
}

constexpr size_t LDS_PER_CU = 160 * 1024;     // gfx950

// Raise a kernel's dynamic LDS limit above the 64 KB default (remembered in *granted).
template <typename Kernel>
bool allow_large_lds(Kernel kernel, size_t bytes, size_t *granted)
{
    if (bytes <= 64 * 1024 || bytes <= *granted) return true;
    if (hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)bytes) != hipSuccess)
        return false;
    *granted = bytes;
    return true;
}

template <int K, typename Word, int EPW>
int launch_rollout(const maze_ctx *ctx, const int8_t *d_actions, int n_steps, float *d_reward,
                   uint8_t *d_done, int8_t *d_obs, hipStream_t st)
{
    using V = View<K, EPW>;
    using L = Lds<K, Word, EPW>;
    const StudentDev &p = ctx->dev;
    const bool grid_lds = L::bytes(p.SP, true) <= LDS_PER_CU - 1024;
    const size_t shmem = L::bytes(p.SP, grid_lds);
    const dim3 grid(p.N / EPW), block(64 * V::WAVES);
    const bool square = p.HP == p.WP;
    static size_t granted[2] = {0, 0};
    if (grid_lds && square) {
        auto kern = k_student_rollout<K, Word, EPW, true, true>;
        if (!allow_large_lds(kern, shmem, &granted[0])) return 0;
        hipLaunchKernelGGL(kern, grid, block, shmem, st, p, d_actions, n_steps, d_reward, d_done, d_obs);
    } else if (grid_lds) {
        auto kern = k_student_rollout<K, Word, EPW, true, false>;
        if (!allow_large_lds(kern, shmem, &granted[1])) return 0;
        hipLaunchKernelGGL(kern, grid, block, shmem, st, p, d_actions, n_steps, d_reward, d_done, d_obs);
    } else {
        auto kern = k_student_rollout<K, Word, EPW, false, false>;
        hipLaunchKernelGGL(kern, grid, block, shmem, st, p, d_actions, n_steps, d_reward, d_done, d_obs);
    }
    return EPW * (p.N / EPW);
}

// Envs per workgroup: the largest of 128 / 64 / 32 whose grids fit in LDS and that still
// gives every CU a workgroup; small batches take 32 so that more CUs take part.
template <int K, typename Word>
int launch_k(const maze_ctx *ctx, const int8_t *d_actions, int n_steps, float *d_reward,
             uint8_t *d_done, int8_t *d_obs, hipStream_t st)
{
    const StudentDev &p = ctx->dev;
    if (n_steps <= 1) {
        // render only (0) or the single step of a policy loop (1): one light launch
        if (p.N < REPW) return 0;
        const size_t shmem_render = Lds<K, Word, REPW>::bytes(p.SP, false);
        const dim3 grid(p.N / REPW), block(REPW);
        if (n_steps == 0)
            hipLaunchKernelGGL((k_step_render_tiled<K, Word, false>), grid, block, shmem_render, st, p,
                               d_actions, d_reward, d_done, d_obs);
        else
            hipLaunchKernelGGL((k_step_render_tiled<K, Word, true>), grid, block, shmem_render, st, p,
                               d_actions, d_reward, d_done, d_obs);
        return REPW * (p.N / REPW);
    }
    const int cus = 256;
    const bool fit128 = Lds<K, Word, 128>::bytes(p.SP, true) <= LDS_PER_CU - 1024;
    const bool fit64 = Lds<K, Word, 64>::bytes(p.SP, true) <= LDS_PER_CU - 1024;
    const bool fit32 = Lds<K, Word, 32>::bytes(p.SP, true) <= LDS_PER_CU - 1024;
    if (p.N >= 128 * cus && fit128)
        return launch_rollout<K, Word, 128>(ctx, d_actions, n_steps, d_reward, d_done, d_obs, st);
    if (p.N >= 64 * cus && fit64)
        return launch_rollout<K, Word, 64>(ctx, d_actions, n_steps, d_reward, d_done, d_obs, st);
    if (p.N >= 32 && (fit32 || !fit64))
        return launch_rollout<K, Word, 32>(ctx, d_actions, n_steps, d_reward, d_done, d_obs, st);
    if (p.N >= 64)
        return launch_rollout<K, Word, 64>(ctx, d_actions, n_steps, d_reward, d_done, d_obs, st);
    return 0;
}

}  // namespace

// Launch the tiled kernel on the first `*covered` envs (a multiple of the workgroup's
// envs) and report how many it took; the caller runs the per-cell kernel on the rest.
// n_steps == 0 renders the current state; n_steps == 1 is one step + observation in one
// light launch.  Returns 0 if no tiled kernel applies.
int student_tiled_launch(const maze_ctx *ctx, const int8_t *d_actions, int n_steps, float *d_reward,
                         uint8_t *d_done, int8_t *d_obs, int *covered, hipStream_t st)
{
    const StudentDev &p = ctx->dev;
    *covered = 0;
    if (!d_obs) return 0;
    const int K = p.k;
    if (K != 3 && K != 5 && K != 7) return 0;
    // 16-byte accesses: every time step's obs block, the obs buffer and each step's row of
    // actions must be 16-byte aligned
    if ((((size_t)p.N * 3 * K * K) & 15) != 0 || ((uintptr_t)d_obs & 15) != 0) return 0;
    if (n_steps > 1 && ((p.N & 15) != 0 || ((uintptr_t)d_actions & 15) != 0)) return 0;
    int done_envs;
    if (ctx->word64) {
        if (K == 3) done_envs = launch_k<3, uint64_t>(ctx, d_actions, n_steps, d_reward, d_done, d_obs, st);
        else if (K == 5) done_envs = launch_k<5, uint64_t>(ctx, d_actions, n_steps, d_reward, d_done, d_obs, st);
        else done_envs = launch_k<7, uint64_t>(ctx, d_actions, n_steps, d_reward, d_done, d_obs, st);
    } else {
        if (K == 3) done_envs = launch_k<3, uint32_t>(ctx, d_actions, n_steps, d_reward, d_done, d_obs, st);
        else if (K == 5) done_envs = launch_k<5, uint32_t>(ctx, d_actions, n_steps, d_reward, d_done, d_obs, st);
        else done_envs = launch_k<7, uint32_t>(ctx, d_actions, n_steps, d_reward, d_done, d_obs, st);
    }
    *covered = done_envs;
    return done_envs > 0;
}
