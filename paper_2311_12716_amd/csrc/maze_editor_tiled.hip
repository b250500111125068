// Tiled store-layout kernel of the teacher editor env.
//
// The editor's state per env IS the bit stream its observation expands from: bit
// 3*c + ch of the stream is channel ch (wall, goal, agent) of cell c, i.e. byte
// 3*c + ch of the env's H*W*3 observation.  A workgroup keeps the streams of
// EPW = 128 consecutive envs in LDS for the whole call (128 * 3*H*W bytes per step
// is a whole number of 128-byte lines).  Per step
//   2 "edit" waves (one lane per env) apply the placement to their env's stream
//     with LDS bit atomics and write the step's t and done,
//   NS "store" waves then expand the 128 concatenated streams to bytes: lane l of
//     round j takes stream bits [16*(64*j+l), +16) -- they may straddle two envs --
//     and writes 16 bytes, so one store instruction of a wave writes 1 KB of
//     contiguous output.
// The streams are kept twice, and the two copies alternate: while the store waves expand
// copy s & 1 -- the grid after step s -- the edit waves bring the other copy up to step
// s + 1 (it lags one edit behind, so they apply the previous placement and the new one).
// One barrier per step; the store waves never wait for an edit, so the output stream has
// no gap at the step boundaries.
#include "maze_internal.h"
#include "maze_store_device.h"

namespace {

constexpr int EPW = 128;        // envs per workgroup
constexpr int NE = EPW / 64;    // edit waves
constexpr int NS = 12;          // store waves
constexpr int NWAVES = NE + NS;

__device__ __forceinline__ void lds_set_bit(uint32_t *rec, int bit)
{
    atomicOr(&rec[bit >> 5], 1u << (bit & 31));
}

__device__ __forceinline__ void lds_clear_bit(uint32_t *rec, int bit)
{
    atomicAnd(&rec[bit >> 5], ~(1u << (bit & 31)));
}

__global__ __launch_bounds__(64 * NWAVES) void k_editor_tiled(
    EditorDev p, const int32_t *__restrict__ actions, int n_steps, int8_t *__restrict__ obs,
    int32_t *__restrict__ t_out, uint8_t *__restrict__ done, uint32_t pace_fp)
{
    extern __shared__ uint32_t lds[];            // [2][EPW][REC], REC = SW + 1 (last dword stays 0)
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int env0 = xcd_contiguous(blockIdx.x, gridDim.x) * EPW;
    const int SW = p.SW, REC = SW + 1;
    const int SB = 3 * p.cells;                  // stream bits = obs bytes per env
    const int count = min(EPW, p.N - env0);      // envs of this workgroup (the last one may be partly filled)

    const int COPY = EPW * REC;                  // dwords of one copy of the streams
    // stage the streams into both copies (and zero the pad dwords; streams of absent envs
    // read as empty)
    for (int i = tid; i < COPY; i += 64 * NWAVES) {
        int e = i / REC, o = i - e * REC;
        const uint32_t v = (o < SW && e < count) ? p.stream[(size_t)(env0 + e) * SW + o] : 0u;
        lds[i] = v;
        lds[COPY + i] = v;
    }
    __syncthreads();

    if (wave < NE) {
        // ==================================================================== edit
        const int e = wave * 64 + lane;
        const bool present = e < count;
        const int n = env0 + (present ? e : 0);  // absent lanes repeat env 0's reads, write nothing
        uint32_t *rec0 = lds + e * REC;          // this env's record in copy 0; copy 1 is COPY further
        int32_t t = p.t[n], ac = p.agent_cell[n], gc = p.goal_cell[n];
        const int32_t *act = actions + n;
        int32_t a_next = act[0];
        int prev_clear = -1, prev_set = -1;      // the placement the other copy has not seen yet
        for (int s = 0; s < n_steps; ++s) {
            const int32_t action = a_next;
            if (s + 1 < n_steps) a_next = act[(size_t)(s + 1) * p.N];
            const int a = min(max(action, 0), p.cells - 1);
            int clear = -1, set = -1;
            if (t < p.n_walls) {
                set = 3 * a;
            } else if (t == p.n_walls) {
                ac = a;
                clear = 3 * a;
                set = 3 * a + 2;
            } else if (t == p.n_walls + 1) {
                const int j = (a == ac) ? ((a + 1 == p.cells) ? 0 : a + 1) : a;
                gc = j;
                clear = 3 * j;
                set = 3 * j + 1;
            }
            // copy s & 1 becomes the grid after step s: the placement it missed, then this one
            // (in this order: a later placement may clear what an earlier one set)
            uint32_t *rec = rec0 + (s & 1) * COPY;
            if (prev_clear >= 0) lds_clear_bit(rec, prev_clear);
            if (prev_set >= 0) lds_set_bit(rec, prev_set);
            if (clear >= 0) lds_clear_bit(rec, clear);
            if (set >= 0) lds_set_bit(rec, set);
            prev_clear = clear;
            prev_set = set;
            if (t < p.n_walls + 2) t += 1;
            if (t_out && present) t_out[(size_t)s * p.N + n] = t;
            if (done && present) done[(size_t)s * p.N + n] = (t == p.n_walls + 2) ? 1 : 0;
            __syncthreads();                     // copy s & 1 is ready; the other is free to edit
        }
        // write the state back (the copy of the last step is complete)
        if (present) {
            p.t[n] = t;
            p.agent_cell[n] = ac;
            p.goal_cell[n] = gc;
            const uint32_t *rec = rec0 + ((n_steps - 1) & 1) * COPY;
            for (int o = 0; o < SW; ++o) p.stream[(size_t)n * SW + o] = rec[o];
        }
    } else {
        // =================================================================== store
        const int c = wave - NE;
        const int block_bytes = count * SB;      // obs bytes of the workgroup per step
        const int nwin = (block_bytes + 15) / 16;  // 16-bit windows per step (the last may be cut)
        // window m = c*64 + lane, then every NS*64 windows; its position is kept as
        // (env e0, bit s inside the env) and advanced without divisions
        const int adv_bits = 16 * NS * 64;
        const int adv_q = adv_bits / SB, adv_r = adv_bits - adv_q * SB;
        const int m0 = c * 64 + lane;
        const int e_first = (16 * m0) / SB, s_first = 16 * m0 - e_first * SB;
        const size_t step_obs = (size_t)p.N * SB;
        int8_t *out_block = obs + (size_t)env0 * SB;
        // rounds of windows per step, and whether the lines fall the same way at every step (then
        // a window whose 128-byte line is written whole by one store instruction of this wave --
        // 64 windows, 1 KB -- is stored in the streaming form)
        const int max_rounds = (nwin + NS * 64 - 1) / (NS * 64);
        const bool steady = step_obs % 128 == 0;
        const uintptr_t chunk_lo = (uintptr_t)out_block, chunk_hi = chunk_lo + (size_t)block_bytes;
        StorePacer pacer;                         // (see maze_store_device.h)
        pacer.init(pace_fp);
        for (int s = 0; s < n_steps; ++s) {
            __syncthreads();                     // copy s & 1 holds the grid after step s
            const uint32_t *copy = lds + (s & 1) * COPY;
            const uint32_t units = pacer.begin(1, (uint32_t)max_rounds * 63u);
            const uint32_t per_round = units / (uint32_t)max_rounds, extra = units % (uint32_t)max_rounds;
            int e0 = e_first, bs = s_first;
            uint32_t round = 0;
            for (int m = m0; m < nwin; m += NS * 64, ++round) {
                const uint32_t *r0 = copy + e0 * REC;
                const int rem = SB - bs;
                const bool spill = rem < 16;     // window runs into the next env
                uint32_t lo = r0[bs >> 5], hi = r0[(bs >> 5) + 1];
                uint32_t nx = spill ? r0[REC] : 0u;
                uint32_t bits = __builtin_amdgcn_alignbit(hi, lo, bs & 31) | (nx << (spill ? rem : 0));
                uint4 v;
                v.x = expand_nibble(bits & 15);          v.y = expand_nibble((bits >> 4) & 15);
                v.z = expand_nibble((bits >> 8) & 15);   v.w = expand_nibble((bits >> 12) & 15);
                const int valid = block_bytes - 16 * m;
                const uintptr_t line = (chunk_lo + 16 * (size_t)m) & ~(uintptr_t)127;
                const uintptr_t piece_lo = chunk_lo + 16 * (size_t)(m - lane);
                const uintptr_t piece_hi = piece_lo + 1024 < chunk_hi ? piece_lo + 1024 : chunk_hi;
                if (steady && valid >= 16 && line >= piece_lo && line + 128 <= piece_hi)
                    store16_stream(out_block, 16u * (uint32_t)m, v);
                else if (valid >= 16) store16(out_block + 16 * (size_t)m, v);
                else store_bytes(out_block + 16 * (size_t)m, v, valid);
                bs += adv_r;
                e0 += adv_q;
                if (bs >= SB) { bs -= SB; e0 += 1; }
                if (units) StorePacer::nap(per_round + (round < extra ? 1u : 0u));
            }
            pacer.end();
            out_block += step_obs;
        }
    }
}

}  // namespace

// Returns 1 if the tiled kernel was launched (on all envs: *covered = N; the last workgroup
// may be partly filled), 0 if the shape is not covered (the caller runs the per-cell kernel).
int editor_tiled_launch(const editor_ctx *ctx, const int32_t *d_actions, int n_steps,
                        int8_t *d_obs, int32_t *d_t, uint8_t *d_done, int *covered, hipStream_t st)
{
    const EditorDev &p = ctx->dev;
    *covered = 0;
    if (!d_obs) return 0;
    // two copies of the streams of 128 envs; above the 64 KB default the kernel's LDS limit is
    // raised once per device; streams too large for that go to the per-cell kernel
    const size_t shmem = 2 * 4 * (size_t)EPW * (p.SW + 1);
    if (shmem > 120 * 1024 || shmem + 1024 > ctx->lds_per_cu) return 0;
    static size_t granted[16] = {};
    if (shmem > 64 * 1024 && shmem > granted[ctx->device & 15]) {
        if (hipFuncSetAttribute((const void *)k_editor_tiled, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)shmem) != hipSuccess)
            return 0;
        granted[ctx->device & 15] = shmem;
    }
    if (3 * p.cells < 16) return 0;              // a 16-bit window must not span more than two envs
    const int groups = (p.N + EPW - 1) / EPW;
    // store waves paced like the student rollout's: the workgroups resident at once (one per
    // CU: 14 waves each) write their obs, t and done of a step and read its actions
    const double resident = (double)(groups < ctx->cus ? groups : ctx->cus);
    const uint32_t pace_fp = maze_pace_fp(ctx->clock_khz, resident * EPW * (3.0 * p.cells + 9.0),
                                          (double)p.N * n_steps * (3.0 * p.cells + 5.0), MAZE_PACED_GBS_EDITOR);
    hipLaunchKernelGGL(k_editor_tiled, dim3(groups), dim3(64 * NWAVES), shmem, st, p, d_actions,
                       n_steps, d_obs, d_t, d_done, pace_fp);
    *covered = p.N;
    return 1;
}
