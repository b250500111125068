// Tiled store-layout kernels of the student env (templates; included by one translation
// unit per view size, which instantiates them).
//
// A workgroup owns EPW consecutive envs for the whole rollout: 128 when the batch is
// large enough to fill the GPU that way (128 * 3k^2 bytes per step is a whole number
// of 128-byte lines, so no line of the output is shared between workgroups), 64 or
// 32 for smaller batches or grids whose LDS copy would not fit, 16 when even those
// would leave compute units without a workgroup.  Per step one lane
// per env advances the env (state in registers, wall rows from LDS) and its
// observation is built as a BIT STREAM -- bit i of the stream is byte i of the env's
// k*k*3 observation, which is 0 or 1 -- and left in LDS.  The EPW streams,
// concatenated, are exactly the EPW*3k^2 contiguous output bytes of this time step,
// so other lanes then take 16 consecutive stream bits each (they may straddle two
// envs), expand each bit to a byte and write 16 contiguous bytes; consecutive lanes
// take consecutive pieces, so one store instruction of a wave writes 1 KB of
// contiguous, aligned output.
//
// The per-step work is a four-stage pipeline over the waves of the workgroup,
// advanced by one barrier per block of SPB steps:
//   first  ("dynamics") block b  : action, move (one wall word: the row of the cell ahead),
//                                  goal/done/reset, in the grid's own coordinates; publish
//                                  position, forward vector, outcome
//   next   ("views")    block b-1: position and goal offset in the heading's frame; K wall
//                                  rows of that frame -> K x K view bits
//   next   ("records")  block b-2: view bits -> stream record (row lookup table),
//                                  goal cell patched in; store reward and done
//   rest   ("stores")   block b-3: expand records to bytes, store obs
// (one dynamics, one views and one records wave per 64 envs -- two records waves in small
// workgroups of the observation variants; every stage has at most two dependent LDS round trips)
// Only the dynamics wave carries a dependency from step to step, so the time per
// step is that wave's short chain; the store waves never load from global memory
// and the dynamics wave touches it once every 16 steps (actions, staged in LDS).
//
// Large launches are bound by how the memory system takes the observation stream, and
// for them the store stage does two more things (maze_store_device.h): lines that one
// store instruction writes whole go out as streaming stores, and the store waves keep
// a clock schedule just under the write rate the memory sustains (StorePacer) instead
// of storing as fast as the queues accept.
#pragma once

#include "maze_internal.h"
#include "maze_store_device.h"
#include "maze_student_device.h"

namespace {

constexpr int SPB = 8;            // steps per barrier: every stage handles SPB steps between barriers
constexpr int STORE_WAVES = 10;   // store waves of a workgroup, at most
// Steps a stage handles together (all reads, then all writes): the largest power of two
// that divides SPB and keeps the group's registers within `budget` dwords.
constexpr int step_group(int dwords_per_step, int budget)
{
    int g = 1;
    while (2 * g <= SPB && SPB % (2 * g) == 0 && 2 * g * dwords_per_step <= budget) g *= 2;
    return g;
}

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
    static constexpr int NC = ROUNDS < STORE_WAVES ? ROUNDS : STORE_WAVES;   // store waves
    // actions: one 16-byte load per lane covers 16 envs of one step, so a dynamics wave
    // stages ACT_BLOCK steps of its LA envs per load
    static constexpr int ACT_LPR = LA / 16;
    static constexpr int ACT_BLOCK = 64 / ACT_LPR;
    static_assert((EPW * SB) % 16 == 0, "a step's chunk must be a whole number of 16-byte pieces");
};

// 16 action bytes of one step (row clamped to the last step), from a lane's first column on.
template <bool PARTIAL>
__device__ __forceinline__ uint4 load_actions(const int8_t *act_lane, int row, int last, int N, int valid)
{
    const int8_t *src = act_lane + (size_t)min(row, last) * N;
    return (!PARTIAL || valid >= 16) ? load16(src) : load_bytes(src, valid);
}


template <typename Word> struct WordOps;
template <> struct WordOps<uint32_t> { static constexpr int DW = 1; };
template <> struct WordOps<uint64_t> { static constexpr int DW = 2; };

// Per-workgroup LDS carve-up (dword offsets).  ST and REC hold SPB steps each and
// are double buffered by block parity (a block = the SPB steps between two barriers).
template <int K, typename Word, int EPW, int MODE = 0>
struct Lds {
    using V = View<K, EPW>;
    static constexpr int LUT = 0;                                  // [LUTN]
    // the rollout of the observation variants (MODE 1) keeps two more tables
    static constexpr int TYPED = LUT + V::LUTN;                    // [3][128] typed dwords (typed_table)
    static constexpr int TYPED_N = MODE == 1 ? 3 * 128 : 0;
    static constexpr int VIS = TYPED + TYPED_N;                    // [2^(2K)] 16-bit rows (visibility_table)
    static constexpr int VIS_N = MODE == 1 ? (1 << (2 * K)) / 2 : 0;
    // action ring: per env the bytes of 2 * ACT_BLOCK consecutive steps, so that one dword holds
    // the actions of four steps; an env's ring is one dword longer than that (odd pitch)
    static constexpr int ACT = VIS + VIS_N;                        // [EPW][ACT_PITCH] dwords
    static constexpr int ACT_PITCH = V::ACT_BLOCK / 2 + 1;         // dwords per env
    static constexpr int ST = ACT + EPW * ACT_PITCH;               // [2][SPB][EPW][4] cell, forward vector, step count, -
    static constexpr int ST_SIZE = 4 * EPW;                        // (four dwords per env: one 16-byte access)
    static constexpr int VW = ST + 2 * SPB * ST_SIZE;              // [2][SPB][WV+2][EPW] view bits, goal, out
    static constexpr int VW_SIZE = (V::WV + 2) * EPW;
    static constexpr int REC = VW + 2 * SPB * VW_SIZE;             // [2][SPB][EPW*REC] stream records
    static constexpr int REC_SIZE = EPW * V::REC;
    static constexpr int GRID0 = REC + 2 * SPB * REC_SIZE;         // [EPW][grid_stride]
    __host__ __device__ static int grid_stride(int SP)             // dwords per env, odd
    {
        return (4 * SP * WordOps<Word>::DW) | 1;
    }
    // with the staged grids of the EPW envs / without (the single-step kernel reads them from L2)
    __host__ static size_t bytes(int SP) { return 4 * (size_t)(GRID0 + EPW * grid_stride(SP)); }
    __host__ static size_t bytes_without_grids() { return 4 * (size_t)GRID0; }
};

// The K wall words of an env's view (row 0 farthest): from the grids staged in LDS (the
// rollout) or from the packed grids in global memory (the single-step kernel).
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
// record_lookup() only reads (the row table), record_finish() only computes, so a caller
// that builds several records can issue all table reads before the first write.
template <int K>
__device__ __forceinline__ void record_lookup(const uint32_t *lut, const uint32_t (&vw)[View<K, 64>::WV],
                                              uint32_t (&piece)[K])
{
    using V = View<K, 64>;
#pragma unroll
    for (int r = 0; r < K; ++r)
        piece[r] = lut[(vw[r / V::RPD] >> (K * (r % V::RPD))) & (V::LUTN - 1)];
}

// Occluded view: an unseen cell's three stream bits are cleared.  The row table entry of a
// mask has bit 3c set for every 1 of the mask (the wall pattern 001b); times 7 gives 111b.
template <int K>
__device__ __forceinline__ void mask_unseen(const uint32_t *lut, const uint32_t (&seenw)[View<K, 64>::WV],
                                            uint32_t (&piece)[K])
{
    using V = View<K, 64>;
    constexpr uint32_t first_of_three = 0x49249249u & ((1u << V::ROWBITS) - 1);
#pragma unroll
    for (int r = 0; r < K; ++r) {
        const uint32_t seen = (seenw[r / V::RPD] >> (K * (r % V::RPD))) & (V::LUTN - 1);
        piece[r] &= (lut[seen] & first_of_three) * 7u;
    }
}

// seenw: the seen cells (occluded view) packed like vw, or nullptr when every cell is shown.
template <int K>
__device__ __forceinline__ void record_finish(const uint32_t (&piece)[K],
                                              const uint32_t (&vw)[View<K, 64>::WV], int gf, int gc,
                                              uint32_t (&D)[View<K, 64>::ND], uint32_t *rec,
                                              const uint32_t *seenw = nullptr)
{
    using V = View<K, 64>;
#pragma unroll
    for (int q = 0; q < V::ND; ++q) D[q] = 0;
#pragma unroll
    for (int r = 0; r < K; ++r) {
        const int off = V::ROWBITS * r, q = off >> 5, b = off & 31;
        D[q] |= piece[r] << b;
        if (b + V::ROWBITS > 32) D[q + 1] |= piece[r] >> (32 - b);
    }
    // goal: the empty cell (100b) becomes a goal cell (010b): flip stream bits 3c+1, 3c+2
    // (a goal that sits on a wall cell -- a level the caller should not build -- shows as wall)
    const int c = gc + K / 2;                      // view column
    bool inview = ((unsigned)gf < (unsigned)K) & ((unsigned)c < (unsigned)K);
    const int grow = inview ? K - 1 - gf : 0;      // view row of the goal
    const uint32_t vw_first = vw[0], vw_last = vw[V::WV - 1];   // scalars: no indexed select
    const uint32_t gword = (V::WV == 1 || grow < V::RPD) ? vw_first : vw_last;
    const int gshift = K * (grow < V::RPD ? grow : grow - V::RPD) + c;
    inview = inview & !((gword >> (gshift & 31)) & 1);
    if (seenw) {                                   // an unseen goal is not shown
        const uint32_t sw_first = seenw[0], sw_last = seenw[V::WV - 1];
        const uint32_t sword = (V::WV == 1 || grow < V::RPD) ? sw_first : sw_last;
        inview = inview & ((sword >> (gshift & 31)) & 1);
    }
    const int bit = inview ? 3 * (grow * K + c) + 1 : 0;
    const uint64_t flip = inview ? (uint64_t)3 << (bit & 31) : 0;
    const int fq = bit >> 5;
#pragma unroll
    for (int q = 0; q < V::ND; ++q) {
        uint32_t m = (q == fq) ? (uint32_t)flip : 0u;
        if (q > 0) m |= (q - 1 == fq) ? (uint32_t)(flip >> 32) : 0u;
        rec[q] = D[q] ^ m;
    }
}

template <int K>
__device__ __forceinline__ void produce_record(const uint32_t *lut, uint32_t *rec,
                                               const uint32_t (&vw)[View<K, 64>::WV], int gf, int gc)
{
    using V = View<K, 64>;
    uint32_t piece[K], D[V::ND];
    record_lookup<K>(lut, vw, piece);
    record_finish<K>(piece, vw, gf, gc, D, rec);
    rec[V::ND] = 0;
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
    // typed encoding only: which of the window's 16 bytes are a cell's first (type) and second
    // (colour) byte; a cell is three bytes and every env starts a new cell
    uint32_t type_pos, colour_pos;
    int typed_row[4];   // per output dword: first entry of its phase's row of the typed table
    int valid;      // bytes of the window that exist: 16, fewer in a partly filled workgroup
    bool stream;    // the window's 128-byte output line is written by this workgroup alone, at
                    // every step: its stores take the streaming form
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
    w.valid = 16;
    w.stream = false;
    const int phase = bitpos % 3;                // stream bit 16*mm is byte `phase` of its cell
    const uint32_t every_third = 0x9249u;        // bits 0, 3, 6, 9, 12, 15
    w.type_pos = phase == 0 ? every_third : (phase == 1 ? 0x4924u : 0x2492u);
    w.colour_pos = phase == 0 ? 0x2492u : (phase == 1 ? every_third : 0x4924u);
#pragma unroll
    for (int q = 0; q < 4; ++q) w.typed_row[q] = 128 * ((phase + q) % 3);   // 4 bytes on: phase + 1
    return w;
}

// block: the workgroup's output block of this step (the same for all lanes)
__device__ __forceinline__ void store_window(int8_t *block, const uint4 &a, const Window &w)
{
    if (w.stream) store16_stream(block, w.out, a);
    else if (w.valid >= 16) store16(block + w.out, a);
    else store_bytes(block + w.out, a, w.valid);
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
    store_window(block, a, w);
}

// The same window written in the (type, colour, state) encoding.  The one-hot stream holds,
// per cell, the bits (wall, goal, empty); the typed bytes are
//     type = 1*empty + 2*wall + 8*goal,  colour = 5*wall + 1*goal,  state = 0,
// so bit planes 0..3 of the output bytes are picked from the stream bits of the same cell
// one or two positions away, masked to the type / colour positions, expanded like the
// plain stream and combined.  A cell never straddles two envs, so the bits needed beyond
// the window come from the same records.
__device__ __forceinline__ void consume_window_typed(const uint32_t *recs, const Window &w, int8_t *block)
{
    const uint32_t lo = recs[w.addr0], hi = recs[w.addr0 + 1], nx = recs[w.addr1];
    const uint32_t prev = recs[w.addr0 > 0 ? w.addr0 - 1 : 0];
    const uint32_t bits = __builtin_amdgcn_alignbit(hi, lo, w.sh) | (nx << w.rem);   // stream bits p, p+1, ...
    const uint32_t below = w.sh ? (lo >> (w.sh - 1)) & 1u : prev >> 31;               // stream bit p-1
    const uint32_t x = bits & 0xFFFFu, up1 = (bits >> 1) & 0xFFFFu, up2 = (bits >> 2) & 0xFFFFu;
    const uint32_t down1 = ((bits << 1) | below) & 0xFFFFu;
    const uint32_t p0 = (up2 & w.type_pos) | ((down1 | x) & w.colour_pos);   // empty -> 1; wall or goal -> colour bit 0
    const uint32_t p1 = x & w.type_pos;                                      // wall -> type 2
    const uint32_t p2 = down1 & w.colour_pos;                                // wall -> colour 4 (+1 = grey 5)
    const uint32_t p3 = up1 & w.type_pos;                                    // goal -> type 8
    uint32_t out[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int sh = 4 * q;
        out[q] = expand_nibble((p0 >> sh) & 15) | (expand_nibble((p1 >> sh) & 15) << 1) |
                 (expand_nibble((p2 >> sh) & 15) << 2) | (expand_nibble((p3 >> sh) & 15) << 3);
    }
    const uint4 a = make_uint4(out[0], out[1], out[2], out[3]);
    store_window(block, a, w);
}

// The typed bytes of one output dword depend on the phase of its first byte (which of type,
// colour, state it is) and on 7 stream bits: the one before the dword's first, its own four and
// two more.  typed_table[phase][those bits] holds the dword, so a window is four table reads.
__device__ __forceinline__ void fill_typed_table(uint32_t *table, int tid, int nthreads)
{
    for (int i = tid; i < 3 * 128; i += nthreads) {
        const int phase = i >> 7, s = i & 127;             // bit j of s: stream bit (first - 1 + j)
        uint32_t v = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int role = (phase + b) % 3;              // 0 type, 1 colour, 2 state
            const int before = (s >> b) & 1, own = (s >> (b + 1)) & 1, next = (s >> (b + 2)) & 1,
                      after = (s >> (b + 3)) & 1;
            // a cell's stream bits are (wall, goal, empty): at its type byte own = wall, next = goal,
            // after = empty; at its colour byte before = wall, own = goal
            const int byte = role == 0 ? 2 * own + 8 * next + after : (role == 1 ? 5 * before + own : 0);
            v |= (uint32_t)byte << (8 * b);
        }
        table[i] = v;
    }
}

__device__ __forceinline__ void consume_window_typed(const uint32_t *recs, const Window &w, int8_t *block,
                                                     const uint32_t *typed_table)
{
    const uint32_t lo = recs[w.addr0], hi = recs[w.addr0 + 1], nx = recs[w.addr1];
    const uint32_t prev = recs[w.addr0 > 0 ? w.addr0 - 1 : 0];
    const uint32_t bits = __builtin_amdgcn_alignbit(hi, lo, w.sh) | (nx << w.rem);   // stream bits p, p+1, ...
    const uint32_t below = w.sh ? (lo >> (w.sh - 1)) & 1u : prev >> 31;               // stream bit p-1
    const uint32_t from_below = (bits << 1) | below;                                  // bit j: stream bit p-1+j
    uint4 a;
    a.x = typed_table[w.typed_row[0] + (from_below & 127)];
    a.y = typed_table[w.typed_row[1] + ((from_below >> 4) & 127)];
    a.z = typed_table[w.typed_row[2] + ((from_below >> 8) & 127)];
    a.w = typed_table[w.typed_row[3] + ((from_below >> 12) & 127)];
    store_window(block, a, w);
}

// Which cells of the view are seen (occluded view): rows are settled from the agent's row
// outwards as K-bit masks.  Seen cells spread sideways through cells that are not walls (a
// seen wall spreads nothing), then every seen non-wall cell makes the three cells touching
// it in the next row ahead seen.  The agent's own cell spreads whatever it holds.  Returns
// the masks packed like the view bits (row r at bit K*(r % RPD) of dword r / RPD).
// One row: `wall` its wall cells, `from_below` the cells made seen by the row behind it.
template <int K>
__device__ __forceinline__ void visible_row(uint32_t wall, uint32_t from_below, uint32_t &seen,
                                            uint32_t &to_next)
{
    constexpr uint32_t all = (1u << K) - 1;
    const uint32_t open = ~wall & all;
    seen = from_below;
#pragma unroll
    for (int it = 1; it < K; ++it) {
        const uint32_t src = seen & open;
        seen |= ((src << 1) | (src >> 1)) & all;
    }
    const uint32_t src = seen & open;
    to_next = (src | (src << 1) | (src >> 1)) & all;
}

template <int K>
__device__ __forceinline__ void visible_cells(const uint32_t (&vw)[View<K, 64>::WV],
                                              uint32_t (&seenw)[View<K, 64>::WV])
{
    using V = View<K, 64>;
    constexpr uint32_t all = (1u << K) - 1, centre = 1u << (K / 2);
#pragma unroll
    for (int q = 0; q < V::WV; ++q) seenw[q] = 0;
    uint32_t from_below = centre;
#pragma unroll
    for (int r = K - 1; r >= 0; --r) {
        uint32_t wall = (vw[r / V::RPD] >> (K * (r % V::RPD))) & all;
        if (r == K - 1) wall &= ~centre;           // the agent's cell spreads whatever it holds
        uint32_t seen;
        visible_row<K>(wall, from_below, seen, from_below);
        seenw[r / V::RPD] |= seen << (K * (r % V::RPD));
    }
}

// visibility_table[wall | from_below << K] = seen | to_next << K: a row of the occluded view is
// one 16-bit table read in the rollout (2^(2K) entries).
template <int K>
__device__ __forceinline__ void fill_visibility_table(uint16_t *table, int tid, int nthreads)
{
    constexpr uint32_t all = (1u << K) - 1;
    for (int i = tid; i < (1 << (2 * K)); i += nthreads) {
        uint32_t seen, to_next;
        visible_row<K>(i & all, (uint32_t)i >> K, seen, to_next);
        table[i] = (uint16_t)(seen | (to_next << K));
    }
}

// visible_cells() for G views at once through the table: the G chains of K dependent reads
// run side by side.
template <int K, int G>
__device__ __forceinline__ void visible_cells_tabled(const uint16_t *table,
                                                     const uint32_t (&vw)[G][View<K, 64>::WV],
                                                     uint32_t (&seenw)[G][View<K, 64>::WV])
{
    using V = View<K, 64>;
    constexpr uint32_t all = (1u << K) - 1, centre = 1u << (K / 2);
    uint32_t from_below[G];
#pragma unroll
    for (int w = 0; w < G; ++w) {
        from_below[w] = centre;
#pragma unroll
        for (int q = 0; q < V::WV; ++q) seenw[w][q] = 0;
    }
#pragma unroll
    for (int r = K - 1; r >= 0; --r) {
#pragma unroll
        for (int w = 0; w < G; ++w) {
            uint32_t wall = (vw[w][r / V::RPD] >> (K * (r % V::RPD))) & all;
            if (r == K - 1) wall &= ~centre;
            const uint32_t e = table[wall | (from_below[w] << K)];
            seenw[w][r / V::RPD] |= (e & all) << (K * (r % V::RPD));
            from_below[w] = e >> K;
        }
    }
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

// Copy the workgroup's envs' grids into LDS (all threads take part).  In global memory the
// `count` grids are one contiguous run of 16-byte pieces (an env's four frames are a multiple of
// four dwords and the array is 256-byte aligned); a thread takes every nthreads-th piece, four
// of its pieces in flight at a time, and puts each into its env's slot (slots are one dword
// longer than a grid, so a piece is written as four dwords).
template <typename L, typename Word>
__device__ __forceinline__ void stage_grids(const StudentDev &p, uint32_t *lds, int tid, int nthreads,
                                            int env0, int count)
{
    uint32_t *base = lds + L::GRID0;
    const int per_env = 4 * p.SP * WordOps<Word>::DW;          // dwords, a multiple of 4
    const uint4 *src = (const uint4 *)((const uint32_t *)p.grids + (size_t)env0 * per_env);
    const int pieces = count * (per_env >> 2);
    // dword index of the piece in the run, and the env it falls in (advanced without dividing)
    const int stride = 4 * nthreads, stride_envs = stride / per_env, stride_rest = stride - stride_envs * per_env;
    int idx = 4 * tid, e = idx / per_env, o = idx - e * per_env;
    constexpr int BATCH = 4;
    for (int i0 = tid; i0 < pieces; i0 += BATCH * nthreads) {
        uint4 v[BATCH];
#pragma unroll
        for (int u = 0; u < BATCH; ++u)
            if (i0 + u * nthreads < pieces) v[u] = src[i0 + u * nthreads];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            if (i0 + u * nthreads < pieces) {
                uint32_t *dst = base + idx + e;                  // e slots precede it, one extra dword each
                dst[0] = v[u].x; dst[1] = v[u].y; dst[2] = v[u].z; dst[3] = v[u].w;
            }
            idx += stride; e += stride_envs; o += stride_rest;
            if (o >= per_env) { o -= per_env; ++e; }
        }
    }
}

// ------------------------------------------------------------------ rollout
// Two 16-bit numbers in one register; arithmetic on them compiles to packed instructions
// (one multiply-add turns a pair, the swap of its halves is an operand modifier).
typedef short pair16 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ pair16 as_pair(uint32_t v) { return __builtin_bit_cast(pair16, v); }
__device__ __forceinline__ uint32_t as_word(pair16 v) { return __builtin_bit_cast(uint32_t, v); }

// Per-lane state of the dynamics stage (one env per lane).  The stage works in the padded
// grid's own coordinates -- a move is one add, the wall test one word of the unrotated grid
// -- and leaves the change to the heading's frame, which only the view needs, to the views
// stage, where nothing waits for the previous step.
template <typename Word>
struct DynState {
    uint32_t pos;             // X | Y << 16, padded-grid coordinates
    uint32_t dv;              // one step forward, (dx, dy) as two 16-bit numbers
    uint32_t t;               // steps since the episode began
    // The row of the cell ahead decides whether a forward step is blocked.  It is fetched one
    // step early: as soon as the action is known, the row ahead of the pose the action leads
    // to -- taking a forward step as successful -- is requested (`spec`), and the choice
    // between that word, the previous one (the forward step hit a wall: pose unchanged) and
    // the start pose's word (episode ended) is made at the top of the next step, when the LDS
    // read has returned.
    Word row_keep, spec;
    bool use_start, use_keep;
};

template <typename Word>
struct DynConst {
    uint32_t start_pos, start_dv;      // the level's start pose, packed as above
    uint32_t goal_pos;                 // the goal cell, packed like pos
    Word row_start;                    // row of the cell ahead of the start pose
    uint32_t tmax;
    const uint32_t *rows;              // this env's unrotated grid (frame 3) in LDS
};

// Word of row `y` of an env's unrotated grid.
template <typename Word>
__device__ __forceinline__ Word grid_row(const uint32_t *rows, uint32_t y)
{
    if (sizeof(Word) == 4) return (Word)rows[y];
    return (Word)(((uint64_t)rows[2 * y + 1] << 32) | rows[2 * y]);
}

// What the dynamics stage hands to the views stage per env and step (12 bytes in a 16-byte
// slot: one LDS instruction each way).
struct alignas(16) Published { uint32_t cell, dv, t; };

// Forward vectors of the headings 0..3 (+x, +y, -x, -y) as (dx, dy) pairs of 16-bit numbers.
__device__ __forceinline__ uint32_t heading_vector(int d)
{
    return d == 0 ? 0x00000001u : d == 1 ? 0x00010000u : d == 2 ? 0x0000FFFFu : 0xFFFF0000u;
}

// Dynamics stage -> views stage, per env and step one 16-byte piece (written and read with one
// LDS instruction each): the cell the agent is in after the action (X | Y << 16), the forward
// vector after the action (dx | dy << 16), the episode's step count including this step -- all
// before the reset that an episode's end brings -- and one dword unused.
//
// One env step of the dynamics stage.  A right turn maps the forward vector (dx, dy) to
// (-dy, dx), a left turn to (dy, -dx): one packed multiply of the swapped pair.  The stage
// keeps its own state right across episode ends but publishes what it has before the reset
// (the cell the agent moved to, the heading after the action, the step count): whether the
// goal was reached, whether the episode ended and the pose the observation then shows follow
// from these and the level's constants in the views stage, off the step-to-step chain.
template <typename Word, int EPW>
__device__ __forceinline__ void dyn_step(DynState<Word> &s, const DynConst<Word> &c, uint32_t a, uint32_t *st)
{
    const bool tl = (a == 0), tr = (a == 1), f2 = (a == 2);
    const pair16 dv = as_pair(s.dv), swapped = dv.yx;
    const uint32_t right = as_word(swapped * (pair16){-1, 1}), left = as_word(swapped * (pair16){1, -1});
    uint32_t ndv = tr ? right : s.dv;
    ndv = tl ? left : ndv;
    const uint32_t ahead = as_word(as_pair(s.pos) + dv);
    const uint32_t next = f2 ? ahead : s.pos;
    const Word row = s.use_start ? c.row_start : (s.use_keep ? s.row_keep : s.spec);
    s.spec = grid_row<Word>(c.rows, as_word(as_pair(next) + as_pair(ndv)) >> 16);
    // (the bit-field extract takes its position from the low 5 bits of `ahead`: its X half)
    const uint32_t blocked = sizeof(Word) == 4 ? __builtin_amdgcn_ubfe((uint32_t)row, ahead, 1)
                                               : (uint32_t)(row >> (ahead & 63u)) & 1u;
    const bool stay = f2 & (blocked != 0);
    const uint32_t moved = stay ? s.pos : next;
    const uint32_t t1 = s.t + 1;
    const bool reached = moved == c.goal_pos;
    const bool fin = reached | (t1 >= c.tmax);
    s.pos = fin ? c.start_pos : moved;
    s.dv = fin ? c.start_dv : ndv;
    s.t = fin ? 0u : t1;
    s.use_start = fin;
    s.use_keep = stay;
    s.row_keep = row;
    *(Published *)st = Published{moved, ndv, t1};
}

// What the views stage makes of a published pose: the heading, the position in the heading's
// frame (Xd | Yd << 16) and the goal's offset in that frame (cells ahead | cells to the
// right << 16).  g0..g3: the goal cell in each frame, packed like the position.
// (All alternatives first, then plain selects on values: a conditional expression with work
// in its arms compiles to a branch, an array indexed by the heading to a stack slot.)
struct FramePose { int d; uint32_t pos, goal; };
__device__ __forceinline__ FramePose to_frame(uint32_t pos, uint32_t dv, uint32_t g0, uint32_t g1, uint32_t g2,
                                              uint32_t g3, int HPm1, int WPm1)
{
    const bool h0 = dv == 0x00000001u, h1 = dv == 0x00010000u, h2 = dv == 0x0000FFFFu;
    const pair16 p = as_pair(pos), swapped = p.yx;
    // frame 0: (Y, WP-1-X); frame 1: (WP-1-X, HP-1-Y); frame 2: (HP-1-Y, X); frame 3: (X, Y)
    const uint32_t f0 = as_word(swapped * (pair16){1, -1} + (pair16){0, (short)WPm1});
    const uint32_t f1 = as_word((pair16){(short)WPm1, (short)HPm1} - p);
    const uint32_t f2 = as_word(swapped * (pair16){-1, 1} + (pair16){(short)HPm1, 0});
    FramePose r;
    int d = h2 ? 2 : 3;
    d = h1 ? 1 : d;
    r.d = h0 ? 0 : d;
    uint32_t fp = h2 ? f2 : pos;
    fp = h1 ? f1 : fp;
    r.pos = h0 ? f0 : fp;
    uint32_t g = h2 ? g2 : g3;
    g = h1 ? g1 : g;
    g = h0 ? g0 : g;
    // (gxd - xd, gyd - yd) -> ahead = yd - gyd, right = gxd - xd
    const pair16 diff = as_pair(g) - as_pair(r.pos);
    r.goal = as_word(diff.yx * (pair16){-1, 1});
    return r;
}

// Each role runs its own loop over blocks of SPB steps; every wave passes exactly
// ceil(n_steps / SPB) + 4 barriers.
//   between barriers b and b+1:  dynamics builds block b   -> ST[b&1]
//                                views    builds block b-1 -> VW[(b-1)&1]   (reads ST[(b-1)&1])
//                                records  builds block b-2 -> REC[(b-2)&1]  (reads VW[(b-2)&1])
//                                stores   drain  block b-3                  (read REC[(b-3)&1])
// so no buffer is written while it is read.  The block loops are unrolled by two so
// every LDS address is a lane constant plus an immediate.
// The body of a role handles one block: it sees i0 (the block's first step), par (the
// block's parity: its buffers), and `full` (a compile-time flag: every one of the SPB
// steps exists; otherwise step i0+u must be tested against n_steps).  Bodies are written
// in phases over the block's steps -- all reads, then all writes -- so that independent
// steps overlap their LDS round trips.
#define MAZE_STEP_ON(u) (full || i0 + (u) < n_steps)
#define MAZE_FOR_EACH_BLOCK(...)                                                           \
    for (int blk0 = 0; blk0 < n_steps; blk0 += 2 * SPB) {                                  \
        _Pragma("unroll") for (int par = 0; par < 2; ++par) {                              \
            const int i0 = blk0 + par * SPB;                                               \
            if (i0 + SPB <= n_steps) {                                                     \
                constexpr bool full = true;                                                \
                { __VA_ARGS__; }                                                           \
                __syncthreads();                                                           \
            } else if (i0 < n_steps) {                                                     \
                constexpr bool full = false;                                               \
                { __VA_ARGS__; }                                                           \
                __syncthreads();                                                           \
            }                                                                              \
        }                                                                                  \
    }

// Records waves per dynamics wave, and the waves of a rollout workgroup.  With occlusion the
// records stage is the one that is busy all the time (98 % of a launch, every other stage under
// 60 %).  Workgroups of 16 or 32 envs get two records waves for it, each taking half of a block's
// passes: config 5 occluded 152 -> 100 us, 8192 envs x 256 steps occluded 58.7 -> 38.8.  At 64
// envs per workgroup a second wave gains nothing (config 3 occluded 118 either way, and 127 ->
// 137 us with typed bytes as well: the table reads, not the instruction issue, are the limit
// there), and at 128 the workgroup has no threads left for one.
template <int EPW, int MODE> constexpr int records_split() { return (MODE == 1 && EPW <= 32) ? 2 : 1; }
template <int K, int EPW, int MODE> constexpr int rollout_waves()
{
    return (2 + records_split<EPW, MODE>()) * View<K, EPW>::NDYN + View<K, EPW>::NC;
}

// MODE 0: the default observation.  MODE 1: the observation variants (p.obs_occlusion: unseen
// cells cleared in the records stage; p.obs_encoding: typed bytes in the stores stage).
// PARTIAL: the workgroup may hold fewer than EPW envs (the last envs of a batch, n_end - env0 of
// them): idle lanes repeat env 0 of the workgroup and write nothing, pieces beyond the last
// env's bytes are not stored.
// BIG (workgroups of 32 envs only; the larger ones always have it): the flavour for launches whose
// output is too large for the memory-side cache to absorb, with streaming stores and paced
// store waves.  Small launches are bound by latency and keep the plain store stage.
template <int K, typename Word, int EPW, int MODE = 0, bool PARTIAL = false, bool BIG = false>
__global__ __launch_bounds__((64 * rollout_waves<K, EPW, MODE>())) void k_student_rollout(
    StudentDev p, int n_begin, int n_end, const int8_t *__restrict__ actions, int n_steps,
    float *__restrict__ reward, uint8_t *__restrict__ done, int8_t *__restrict__ obs, uint32_t pace_fp)
{
    using V = View<K, EPW>;
    using L = Lds<K, Word, EPW, MODE>;
    constexpr int RSPLIT = records_split<EPW, MODE>();
    constexpr int NT = 64 * rollout_waves<K, EPW, MODE>();
    constexpr bool LARGE = EPW >= 64 || BIG;
    constexpr int ACT_BLOCK = V::ACT_BLOCK;
    constexpr int UGV = step_group(K * WordOps<Word>::DW + 4, 40);   // views: wall rows + pose in frame + outcome
    // records: table words + view (+ the seen cells and the chain state of the occluded view)
    constexpr int UGR = step_group(K + V::WV + 2 + (MODE == 1 ? V::WV + 2 : 0), 48);
    // steps per pass of a views / records wave: the wave's 64 lanes take 64 / LA steps of a
    // block at once when the workgroup has fewer than 64 envs
    constexpr int UPL = SPB % (64 / V::LA) == 0 ? 64 / V::LA : 1;
    constexpr int UGVP = UGV > SPB / UPL ? SPB / UPL : UGV;
    constexpr int PASSES_R = SPB / UPL / RSPLIT;                 // passes of a records wave per block
    static_assert(PASSES_R >= 1, "a records wave needs a pass per block");
    constexpr int UGRP = UGR > PASSES_R ? PASSES_R : UGR;
    extern __shared__ __align__(16) uint32_t lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wg = xcd_contiguous(blockIdx.x, gridDim.x);
    const int env0 = n_begin + wg * EPW;             // n_begin: a multiple of 32 (16-byte pieces)
    const int SP = p.SP, N = p.N;
    const int count = PARTIAL ? min(EPW, n_end - env0) : EPW;       // envs of this workgroup
    const int live_lanes = PARTIAL ? min((int)V::LA, count) : V::LA; // (PARTIAL: one wave per stage)
    static_assert(!PARTIAL || V::NDYN == 1, "partly filled workgroups: 64 envs at most");

    fill_lut<K>(lds + L::LUT, tid, NT);
    stage_grids<L, Word>(p, lds, tid, NT, env0, count);
    if (MODE == 1) {
        fill_typed_table(lds + L::TYPED, tid, NT);
        if (p.obs_occlusion) fill_visibility_table<K>((uint16_t *)(lds + L::VIS), tid, NT);
    }

    if (wave < V::NDYN) {
        // ================================================================ dynamics
        const bool active = lane < live_lanes;     // a wave serves LA envs
        const int e = wave * 64 + (active ? lane : 0);   // env within the workgroup
        const int n = env0 + e;
        const int last = n_steps - 1;
        DynState<Word> s;
        DynConst<Word> c;
        // poses are kept in the frame of their heading between launches (pose = Xd | Yd << 8 |
        // d << 16); frame 3 is the padded grid itself
        const uint32_t pose = p.pose[n], start = p.start[n], goal3 = p.goalrot[4 * (size_t)n + 3];
        int X, Y;
        frame_to_padded(p, (pose >> 16) & 3, pose & 255, (pose >> 8) & 255, X, Y);
        s.pos = (uint32_t)X | ((uint32_t)Y << 16);
        s.dv = heading_vector((pose >> 16) & 3);
        s.t = p.tcount[n];
        frame_to_padded(p, (start >> 16) & 3, start & 255, (start >> 8) & 255, X, Y);
        c.start_pos = (uint32_t)X | ((uint32_t)Y << 16);
        c.start_dv = heading_vector((start >> 16) & 3);
        c.goal_pos = (goal3 & 255u) | ((goal3 >> 8) << 16);
        c.tmax = (uint32_t)p.max_steps;
        c.rows = lds + L::GRID0 + e * L::grid_stride(SP) + 3 * SP * WordOps<Word>::DW;
        // Actions.  Global memory holds them step-major; lane l of this wave loads the 16 bytes
        // of step block * ACT_BLOCK + l / ACT_LPR for 16 of the wave's envs (all 64 lanes load,
        // whatever LA is) and writes them, byte by byte, into those envs' rings, where an env's
        // consecutive steps are consecutive bytes: the step loop then reads one dword per four
        // steps.  A block of ACT_BLOCK steps is staged half a block of them before its first
        // step, into the half of the ring the block before the previous one has left.
        const int stage_row = lane / V::ACT_LPR;
        const int stage_col = wave * 64 + 16 * (lane % V::ACT_LPR);
        const int8_t *act_lane = actions + env0 + stage_col;
        uint8_t *act_stage = (uint8_t *)(lds + L::ACT) + stage_col * (4 * L::ACT_PITCH) + stage_row;
        // bytes of a row that exist from this lane's first column on (PARTIAL: may be < 16)
        const int act_valid = PARTIAL ? N - (env0 + stage_col) : 16;
        auto stage_actions = [&](int half, const uint4 &v) {
            const uint32_t dw[4] = {v.x, v.y, v.z, v.w};
            _Pragma("unroll") for (int j = 0; j < 16; ++j)
                act_stage[half * ACT_BLOCK + j * (4 * L::ACT_PITCH)] = (uint8_t)(dw[j >> 2] >> (8 * (j & 3)));
        };
        stage_actions(0, load_actions<PARTIAL>(act_lane, stage_row, last, N, act_valid));
        uint4 act_regs = load_actions<PARTIAL>(act_lane, ACT_BLOCK + stage_row, last, N, act_valid);
        __syncthreads();                                             // barrier 0 (set-up)
        c.row_start = grid_row<Word>(c.rows, as_word(as_pair(c.start_pos) + as_pair(c.start_dv)) >> 16);
        s.row_keep = grid_row<Word>(c.rows, as_word(as_pair(s.pos) + as_pair(s.dv)) >> 16);
        s.spec = s.row_keep;
        s.use_start = false; s.use_keep = true;
        const uint32_t *act_ring = lds + L::ACT + e * L::ACT_PITCH;
        constexpr int RING_MASK = 2 * ACT_BLOCK - 1;                 // ring length in steps - 1
        uint32_t act_w0 = act_ring[0], act_w1 = act_ring[1];         // the actions of the block's 8 steps
        static_assert(SPB == 8, "two action dwords per block");
        uint32_t *st_e = lds + L::ST + 4 * e;
        MAZE_FOR_EACH_BLOCK(
            const uint32_t w0 = act_w0; const uint32_t w1 = act_w1;
            _Pragma("unroll") for (int u = 0; u < SPB; ++u) {
                const int i = i0 + u;
                if (MAZE_STEP_ON(u)) {
                    // (idle lanes of a partly filled wave repeat env 0 of the workgroup: the same
                    // values to the same addresses; stepping all lanes keeps the flags plain masks)
                    dyn_step<Word, EPW>(s, c, ((u < 4 ? w0 : w1) >> (8 * (u & 3))) & 255u,
                                        st_e + (par * SPB + u) * L::ST_SIZE);
                }
                // the next block's actions, half a block early (staged at least half a block ago)
                if (u == SPB / 2 - 1) {
                    const int at = ((i0 + SPB) & RING_MASK) >> 2;
                    act_w0 = act_ring[at];
                    act_w1 = act_ring[at + 1];
                }
                // stage the next block of actions half way through the current one
                if ((i & (ACT_BLOCK - 1)) == ACT_BLOCK / 2) {
                    const int nb = i / ACT_BLOCK + 1;
                    stage_actions(nb & 1, act_regs);
                    act_regs = load_actions<PARTIAL>(act_lane, (nb + 1) * ACT_BLOCK + stage_row, last, N, act_valid);
                }
            })
        if (active) {
            const int d = s.dv == heading_vector(0) ? 0 : s.dv == heading_vector(1) ? 1 : s.dv == heading_vector(2) ? 2 : 3;
            int xd, yd;
            padded_to_frame(p, d, (int)(s.pos & 0xFFFFu), (int)(s.pos >> 16), xd, yd);
            p.pose[n] = (uint32_t)xd | ((uint32_t)yd << 8) | ((uint32_t)d << 16);
            p.tcount[n] = s.t;
        }
        __syncthreads();
        __syncthreads();
        __syncthreads();
    } else if (wave < 2 * V::NDYN) {
        // =================================================================== views
        // With fewer than 64 envs per workgroup the wave's lanes beyond the first LA take the
        // next steps of a block (UPL steps per pass: `half` is the step within the pass), so
        // the stage issues 1 / UPL of the instructions per step.
        const int half = UPL > 1 ? lane / V::LA : 0;
        const int el = UPL > 1 ? lane % V::LA : lane;
        const bool active = el < live_lanes;
        const int e = (wave - V::NDYN) * 64 + (active ? el : 0);
        const uint32_t *lds_env = lds + L::GRID0 + e * L::grid_stride(SP);
        const uint32_t *st_lane = lds + L::ST + half * L::ST_SIZE + 4 * e;
        uint32_t *vw_lane = lds + L::VW + half * L::VW_SIZE + e;
        // the goal cell in each heading's frame, Xd | Yd << 16
        const uint4 gr = *(const uint4 *)(p.goalrot + 4 * (size_t)(env0 + e));
        uint32_t goal0 = (gr.x & 255u) | ((gr.x >> 8) << 16), goal1 = (gr.y & 255u) | ((gr.y >> 8) << 16);
        uint32_t goal2 = (gr.z & 255u) | ((gr.z >> 8) << 16), goal3 = (gr.w & 255u) | ((gr.w >> 8) << 16);
        // (the compiler is not to know that the four were one vector: it would turn the selects
        // between them into an indexed read of a copy on the stack)
        asm volatile("" : "+v"(goal0), "+v"(goal1), "+v"(goal2), "+v"(goal3));
        const int HPm1 = p.HP - 1, WPm1 = p.WP - 1;
        const uint32_t tmax = (uint32_t)p.max_steps, goal_abs = goal3;      // frame 3 is the grid itself
        uint32_t start_abs, start_dv;
        {
            const uint32_t start = p.start[env0 + e];
            int X, Y;
            frame_to_padded(p, (start >> 16) & 3, start & 255, (start >> 8) & 255, X, Y);
            start_abs = (uint32_t)X | ((uint32_t)Y << 16);
            start_dv = heading_vector((start >> 16) & 3);
        }
        __syncthreads();                                             // barrier 0 (set-up)
        __syncthreads();                                             // block 0 published
        MAZE_FOR_EACH_BLOCK(
            if (active) {
                _Pragma("unroll") for (int u0 = 0; u0 < SPB / UPL; u0 += UGVP) {
                    FramePose f[UGVP];
                    uint32_t out[UGVP];
                    Word rows[UGVP][K];
                    _Pragma("unroll") for (int w = 0; w < UGVP; ++w) if (MAZE_STEP_ON((u0 + w) * UPL + half)) {
                        const uint32_t *st = st_lane + (par * SPB + (u0 + w) * UPL) * L::ST_SIZE;
                        const Published pub = *(const Published *)st;
                        const bool reached = pub.cell == goal_abs, fin = reached | (pub.t >= tmax);
                        f[w] = to_frame(fin ? start_abs : pub.cell, fin ? start_dv : pub.dv, goal0, goal1, goal2,
                                        goal3, HPm1, WPm1);
                        out[w] = (reached ? pub.t : 0u) | (fin ? 0x80000000u : 0u);
                    }
                    _Pragma("unroll") for (int w = 0; w < UGVP; ++w) if (MAZE_STEP_ON((u0 + w) * UPL + half))
                        load_view_rows<K, Word, true>(lds_env, nullptr, SP, f[w].d, f[w].pos >> 16, rows[w]);
                    _Pragma("unroll") for (int w = 0; w < UGVP; ++w) if (MAZE_STEP_ON((u0 + w) * UPL + half)) {
                        uint32_t vw[V::WV];
                        pack_view<K, Word>(rows[w], f[w].pos & 0xFFFF, vw);
                        uint32_t *v = vw_lane + (par * SPB + (u0 + w) * UPL) * L::VW_SIZE;
                        _Pragma("unroll") for (int q = 0; q < V::WV; ++q) v[q * EPW] = vw[q];
                        v[V::WV * EPW] = f[w].goal;
                        v[(V::WV + 1) * EPW] = out[w];
                    }
                }
            })
        __syncthreads();
        __syncthreads();
    } else if (wave < (2 + RSPLIT) * V::NDYN) {
        // ================================================================= records
        const int half = UPL > 1 ? lane / V::LA : 0;
        const int el = UPL > 1 ? lane % V::LA : lane;
        const bool active = el < live_lanes;
        // (RSPLIT records waves per 64 envs: wave `rsel` of them takes that part of a block's passes)
        const int rsel = RSPLIT > 1 ? (wave - 2 * V::NDYN) / V::NDYN : 0;
        const int e = (wave - (2 + rsel) * V::NDYN) * 64 + (active ? el : 0);
        float *rw = reward + env0 + e + (size_t)half * N;
        uint8_t *dn = done + env0 + e + (size_t)half * N;
        const double slope = p.reward_slope;
        const uint32_t *vw_lane = lds + L::VW + half * L::VW_SIZE + e;
        uint32_t *rec_lane = lds + L::REC + half * L::REC_SIZE + e * V::REC;
        // the zero dword that ends every record is written once
        if (active && half == 0 && rsel == 0)
            for (int sl = 0; sl < 2 * SPB; ++sl) lds[L::REC + sl * L::REC_SIZE + e * V::REC + V::ND] = 0;
        __syncthreads();                                             // barrier 0 (set-up)
        __syncthreads();                                             // block 0 published
        __syncthreads();                                             // block 0 viewed
        MAZE_FOR_EACH_BLOCK(
            if (active) {
                _Pragma("unroll") for (int uu = 0; uu < PASSES_R; uu += UGRP) {
                    const int u0 = rsel * PASSES_R + uu;
                    uint32_t vw[UGRP][V::WV], g[UGRP], out[UGRP], piece[UGRP][K];
                    _Pragma("unroll") for (int w = 0; w < UGRP; ++w) if (MAZE_STEP_ON((u0 + w) * UPL + half)) {
                        const uint32_t *v = vw_lane + (par * SPB + (u0 + w) * UPL) * L::VW_SIZE;
                        _Pragma("unroll") for (int q = 0; q < V::WV; ++q) vw[w][q] = v[q * EPW];
                        g[w] = v[V::WV * EPW]; out[w] = v[(V::WV + 1) * EPW];
                    }
                    _Pragma("unroll") for (int w = 0; w < UGRP; ++w) if (MAZE_STEP_ON((u0 + w) * UPL + half))
                        record_lookup<K>(lds + L::LUT, vw[w], piece[w]);
                    uint32_t seenw[UGRP][V::WV];
                    if constexpr (MODE == 1) if (p.obs_occlusion) {
                        // (steps beyond the rollout's end hold the block's stale views: their
                        // table reads stay inside the table, their results are dropped)
                        _Pragma("unroll") for (int w = 0; w < UGRP; ++w) if (!MAZE_STEP_ON((u0 + w) * UPL + half))
                            _Pragma("unroll") for (int q = 0; q < V::WV; ++q) vw[w][q] = 0;
                        visible_cells_tabled<K, UGRP>((const uint16_t *)(lds + L::VIS), vw, seenw);
                    }
                    _Pragma("unroll") for (int w = 0; w < UGRP; ++w) if (MAZE_STEP_ON((u0 + w) * UPL + half)) {
                        uint32_t D[V::ND];
                        uint32_t *rec = rec_lane + (par * SPB + (u0 + w) * UPL) * L::REC_SIZE;
                        if (MODE == 1 && p.obs_occlusion) {
                            mask_unseen<K>(lds + L::LUT, seenw[w], piece[w]);
                            record_finish<K>(piece[w], vw[w], (int)(int16_t)(g[w] & 0xFFFF),
                                             (int)g[w] >> 16, D, rec, seenw[w]);
                        } else
                        record_finish<K>(piece[w], vw[w], (int)(int16_t)(g[w] & 0xFFFF), (int)g[w] >> 16,
                                         D, rec);
                        const uint32_t tr = out[w] & 0x7FFFFFFFu;
                        rw[(size_t)((u0 + w) * UPL) * N] = tr ? (float)(1.0 - (double)tr * slope) : 0.0f;
                        dn[(size_t)((u0 + w) * UPL) * N] = (uint8_t)(out[w] >> 31);
                    }
                }
                rw += (size_t)SPB * N;
                dn += (size_t)SPB * N;
            })
        __syncthreads();
    } else {
        // ================================================================== stores
        const int cw = wave - (2 + RSPLIT) * V::NDYN;
        constexpr int MYR = (V::ROUNDS + V::NC - 1) / V::NC;     // rounds per store wave, at most
        Window win[MYR];
#pragma unroll
        for (int j = 0; j < MYR; ++j) {
            win[j] = make_window<K, EPW>(lane, cw + j * V::NC);
            if (PARTIAL) {
                const int left = count * V::SB - (int)win[j].out;   // bytes of the block from this piece on
                win[j].valid = min(16, left);
                win[j].active = win[j].active && left > 0;
            }
        }
        const size_t step_obs = (size_t)N * V::SB;
        int8_t *out_block = obs + (size_t)env0 * V::SB;
        // Streaming stores for the windows whose 128-byte line is written whole by one store
        // instruction of this wave -- decided once, which needs the lines to fall the same way at
        // every step.  (A line that two instructions share must stay in the L2 until both have
        // written it: streamed, its parts reach memory one by one; with every inner line of a
        // chunk streamed, whichever instruction wrote it, config 5 took 166 instead of 124 us.)
        if (LARGE && step_obs % 128 == 0) {
            const uintptr_t chunk_lo = (uintptr_t)out_block, chunk_hi = chunk_lo + (size_t)count * V::SB;
#pragma unroll
            for (int j = 0; j < MYR; ++j) {
                // the line must be written whole by this one store instruction of the wave (its
                // 64 windows, 1 KB from the wave's first window on)
                const uintptr_t line = (chunk_lo + win[j].out) & ~(uintptr_t)127;
                const uintptr_t piece_lo = chunk_lo + (win[j].out - 16u * (uint32_t)lane);
                const uintptr_t piece_hi = piece_lo + 1024 < chunk_hi ? piece_lo + 1024 : chunk_hi;
                win[j].stream = win[j].active && win[j].valid >= 16 && line >= piece_lo && line + 128 <= piece_hi;
            }
        }
        __syncthreads();                                             // barrier 0 (set-up)
        __syncthreads();                                             // block 0 published
        __syncthreads();                                             // block 0 viewed
        __syncthreads();                                             // block 0 recorded
        StorePacer pacer;                      // (see maze_store_device.h)
        pacer.init(LARGE ? pace_fp : 0u);
        MAZE_FOR_EACH_BLOCK(
            constexpr uint32_t SLOTS = SPB * MYR;  // stores of a wave per block
            const uint32_t units = LARGE ? pacer.begin(full ? SPB : n_steps - i0, SLOTS * 63u) : 0u;
            if (units == 0) {
                // (kept apart: without the sleep loops between them the compiler overlaps the
                // LDS reads of the block's steps)
                _Pragma("unroll") for (int u = 0; u < SPB; ++u) if (MAZE_STEP_ON(u)) {
                    const uint32_t *rec = lds + L::REC + (par * SPB + u) * L::REC_SIZE;
                    _Pragma("unroll") for (int j = 0; j < MYR; ++j) {
                        if (!win[j].active) continue;
                        if (MODE == 1 && p.obs_encoding)
                            consume_window_typed(rec, win[j], out_block + u * step_obs, lds + L::TYPED);
                        else consume_window(rec, win[j], out_block + u * step_obs);
                    }
                }
            } else {
                const uint32_t per_slot = units / SLOTS, extra = units % SLOTS;
                _Pragma("unroll") for (int u = 0; u < SPB; ++u) if (MAZE_STEP_ON(u)) {
                    const uint32_t *rec = lds + L::REC + (par * SPB + u) * L::REC_SIZE;
                    _Pragma("unroll") for (int j = 0; j < MYR; ++j) {
                        if (win[j].active) {
                            if (MODE == 1 && p.obs_encoding)
                                consume_window_typed(rec, win[j], out_block + u * step_obs, lds + L::TYPED);
                            else consume_window(rec, win[j], out_block + u * step_obs);
                        }
                        StorePacer::nap(per_slot + ((uint32_t)(u * MYR + j) < extra ? 1u : 0u));
                    }
                }
            }
            if (LARGE) pacer.end();
            out_block += SPB * step_obs;)
    }
}

// ------------------------------- observation of the state / one step + observation
// One workgroup of REPW threads per REPW envs, no time loop: optionally advance every
// env by one step (the call a policy loop makes: state in and out of global memory, wall
// rows from the packed grids in L2), then produce the records and expand them.
constexpr int REPW = 64;

template <int K, typename Word, bool DO_STEP, int MODE = 0>
__global__ __launch_bounds__(REPW) void k_step_render_tiled(
    StudentDev p, const int8_t *__restrict__ actions, float *__restrict__ reward,
    uint8_t *__restrict__ done, int8_t *__restrict__ obs)
{
    using V = View<K, REPW>;
    using L = Lds<K, Word, REPW>;
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x;
    const int env0 = xcd_contiguous(blockIdx.x, gridDim.x) * REPW;
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
    uint32_t *rec = lds + L::REC + lane * V::REC;
    if (MODE == 1 && p.obs_occlusion) {
        uint32_t piece[K], D[V::ND], seenw[V::WV];
        record_lookup<K>(lds + L::LUT, vw, piece);
        visible_cells<K>(vw, seenw);
        mask_unseen<K>(lds + L::LUT, seenw, piece);
        record_finish<K>(piece, vw, yd - (int)(g >> 8), (int)(g & 255) - xd, D, rec, seenw);
        rec[V::ND] = 0;
    } else {
        produce_record<K>(lds + L::LUT, rec, vw, yd - (int)(g >> 8), (int)(g & 255) - xd);
    }
    __syncthreads();
    int8_t *block = obs + (size_t)env0 * V::SB;
    for (int j = 0; j < V::ROUNDS; ++j) {
        Window w = make_window<K, REPW>(lane, j);
        if (!w.active) continue;
        if (MODE == 1 && p.obs_encoding) consume_window_typed(lds + L::REC, w, block);
        else consume_window(lds + L::REC, w, block);
    }
}

// LDS a workgroup of a rollout may use on this device: what a CU has, less 1 KB that the
// runtime may claim for itself.
inline size_t lds_budget(const maze_ctx *ctx) { return ctx->lds_per_cu > 1024 ? ctx->lds_per_cu - 1024 : 0; }

// The largest grids (64 rows of 64 bits in each of the four frames) of 32 envs fit beside the
// pipeline buffers of every flavour in the 160 KB of a gfx950 CU, so a rollout with 32 envs per
// workgroup exists for every shape the library accepts.
static_assert(Lds<7, uint64_t, 32, 1>::GRID0 * 4 + 32 * 4 * ((4 * 64 * 2) | 1) <= 159 * 1024,
              "32 envs per workgroup must fit in LDS for every supported shape");

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

// Runs the rollout kernel on envs [n_begin, n_begin + EPW * (n_envs / EPW)) -- with PARTIAL on all
// n_envs, the last workgroup partly filled -- and returns how many envs that is, or MAZE_EHIP
// if the device does not grant the LDS the workgroup needs.
template <int K, typename Word, int EPW, int MODE = 0, bool PARTIAL = false, bool BIG = false>
int launch_rollout(const maze_ctx *ctx, int n_begin, int n_envs, const int8_t *d_actions, int n_steps,
                   float *d_reward, uint8_t *d_done, int8_t *d_obs, hipStream_t st)
{
    using V = View<K, EPW>;
    using L = Lds<K, Word, EPW, MODE>;
    const StudentDev &p = ctx->dev;
    const int groups = PARTIAL ? (n_envs + EPW - 1) / EPW : n_envs / EPW;
    if (groups < 1) return 0;
    const int n_end = PARTIAL ? n_begin + n_envs : n_begin + groups * EPW;
    const size_t shmem = L::bytes(p.SP);
    if (shmem > lds_budget(ctx)) return MAZE_EHIP;
    const dim3 grid(groups), block(64 * rollout_waves<K, EPW, MODE>());
    // Pacing of the store waves (see the kernel's stores stage): the time one step of the launch
    // should take if the workgroups resident at once write their chunks, reward and done at
    // MAZE_PACED_GBS (MAZE_PACED_GBS_TYPED for the typed observation).  Paced are launches that
    // write more than twice what the 256 MB memory-side cache holds (a smaller output is absorbed
    // there and leaves the chip later: 16384 envs x 256 steps take 52 us unpaced, 57 paced) and do
    // not build the occluded view (there the records stage sets the pace: 117 us unpaced, 120
    // paced).
    const double out_bytes = (double)(n_end - n_begin) * n_steps * (V::SB + 5);
    uint32_t pace_fp = 0;
    if (!p.obs_occlusion) {
        const size_t per_cu = max((size_t)1, min(lds_budget(ctx) / shmem, (size_t)(32 / rollout_waves<K, EPW, MODE>())));
        const double resident = (double)min((long long)groups, (long long)ctx->cus * (long long)per_cu);
        pace_fp = maze_pace_fp(ctx->clock_khz, resident * EPW * (V::SB + 6), out_bytes,
                               p.obs_encoding ? MAZE_PACED_GBS_TYPED : MAZE_PACED_GBS);
    }
    // Workgroups of 32 envs: launches too large for the memory-side cache go to the flavour with
    // streaming stores and pacing, the others (bound by latency: 4096 envs x 256 steps take 39.6 us
    // with the plain store stage, 42.1 with the other) keep the plain one.
    if constexpr (EPW == 32 && !PARTIAL && !BIG) {
        if (out_bytes > MAZE_CACHE_ABSORBS_BYTES)
            return launch_rollout<K, Word, EPW, MODE, PARTIAL, true>(ctx, n_begin, n_envs, d_actions, n_steps,
                                                                     d_reward, d_done, d_obs, st);
    }
    // largest LDS size granted so far, per device (the attribute belongs to the kernel on one
    // device); a race between host threads only repeats the call
    static size_t granted_all[16] = {};         // (one table per instantiation of this function)
    auto kern = k_student_rollout<K, Word, EPW, MODE, PARTIAL, BIG>;
    if (!allow_large_lds(kern, shmem, &granted_all[ctx->device & 15])) return MAZE_EHIP;
    hipLaunchKernelGGL(kern, grid, block, shmem, st, p, n_begin, n_end, d_actions, n_steps, d_reward,
                       d_done, d_obs, pace_fp);
    return n_end - n_begin;
}

// The envs the large workgroups left over, and small batches: workgroups of 32 in one more
// launch on the same stream; if their number is not a multiple of 32 the flavour whose last
// workgroup may be partly filled takes them all.
template <int K, typename Word, int MODE>
int launch_rest(const maze_ctx *ctx, int covered, const int8_t *d_actions, int n_steps, float *d_reward,
                uint8_t *d_done, int8_t *d_obs, hipStream_t st)
{
    if (covered < 0) return covered;
    const int rest = ctx->dev.N - covered;
    if (rest <= 0) return covered;
    const int more = rest % 32 == 0
        ? launch_rollout<K, Word, 32, MODE>(ctx, covered, rest, d_actions, n_steps, d_reward, d_done, d_obs, st)
        : launch_rollout<K, Word, 32, MODE, true>(ctx, covered, rest, d_actions, n_steps, d_reward, d_done,
                                                  d_obs, st);
    return more < 0 ? more : covered + more;
}

// Envs per workgroup of a rollout's main launch: the largest of 128 / 64 / 32 whose grids fit
// in LDS and that still gives every CU a workgroup; small batches take 32 so that more CUs
// take part.  Observation variants: 128 for typed bytes alone (as fast as the plain
// observation), at most 64 with occlusion (the records stage is the slow one there: more
// workgroups do better).  MAZE_EHIP if not even 32 envs fit into `budget` bytes of LDS.
template <int K, typename Word>
int plan_k(int N, int SP, bool typed, bool occlusion, int cus, size_t budget, int *epw, size_t *lds_bytes)
{
    const bool variant = typed || occlusion;
    const size_t b128 = variant ? Lds<K, Word, 128, 1>::bytes(SP) : Lds<K, Word, 128>::bytes(SP);
    const size_t b64 = variant ? Lds<K, Word, 64, 1>::bytes(SP) : Lds<K, Word, 64>::bytes(SP);
    const size_t b32 = variant ? Lds<K, Word, 32, 1>::bytes(SP) : Lds<K, Word, 32>::bytes(SP);
    const size_t b16 = variant ? Lds<K, Word, 16, 1>::bytes(SP) : Lds<K, Word, 16>::bytes(SP);
    if (b32 > budget) return MAZE_EHIP;
    if (!occlusion && N >= 128 * (long long)cus && b128 <= budget) { *epw = 128; *lds_bytes = b128; }
    // (the occluded view alone does better with 32 envs per workgroup and their two records
    // waves than with 64 and one: config 3 118 -> 112 us; with typed bytes as well 128 -> 140)
    else if (!(occlusion && !typed) && N >= 64 * (long long)cus && b64 <= budget) { *epw = 64; *lds_bytes = b64; }
    else if (N >= 16 && N <= 16 * (long long)cus) { *epw = 16; *lds_bytes = b16; }
    else { *epw = 32; *lds_bytes = b32; }
    return MAZE_OK;
}

template <int K>
int plan_view_size(int N, int SP, bool typed, bool occlusion, int cus, size_t budget, int *epw,
                   size_t *lds_bytes)
{
    return SP > 32 ? plan_k<K, uint64_t>(N, SP, typed, occlusion, cus, budget, epw, lds_bytes)
                   : plan_k<K, uint32_t>(N, SP, typed, occlusion, cus, budget, epw, lds_bytes);
}

// Returns the number of envs covered (all of them for a rollout) or a negative error code.
template <int K, typename Word>
int launch_k(const maze_ctx *ctx, const int8_t *d_actions, int n_steps, float *d_reward,
             uint8_t *d_done, int8_t *d_obs, hipStream_t st)
{
    const StudentDev &p = ctx->dev;
    if (n_steps <= 1) {
        // render only (0) or the single step of a policy loop (1): one light launch
        if (p.N < REPW) return 0;
        const size_t shmem_render = Lds<K, Word, REPW>::bytes_without_grids();
        const dim3 grid(p.N / REPW), block(REPW);
        const bool variant = p.obs_encoding || p.obs_occlusion;
        if (n_steps == 0 && !variant)
            hipLaunchKernelGGL((k_step_render_tiled<K, Word, false>), grid, block, shmem_render, st, p,
                               d_actions, d_reward, d_done, d_obs);
        else if (n_steps == 0)
            hipLaunchKernelGGL((k_step_render_tiled<K, Word, false, 1>), grid, block, shmem_render, st, p,
                               d_actions, d_reward, d_done, d_obs);
        else if (!variant)
            hipLaunchKernelGGL((k_step_render_tiled<K, Word, true>), grid, block, shmem_render, st, p,
                               d_actions, d_reward, d_done, d_obs);
        else
            hipLaunchKernelGGL((k_step_render_tiled<K, Word, true, 1>), grid, block, shmem_render, st, p,
                               d_actions, d_reward, d_done, d_obs);
        return REPW * (p.N / REPW);
    }
    const bool variant = p.obs_encoding || p.obs_occlusion;
    int epw = 0, covered = 0;
    size_t lds_bytes = 0;
    const int rc = plan_k<K, Word>(p.N, p.SP, p.obs_encoding != 0, p.obs_occlusion != 0, ctx->cus, lds_budget(ctx), &epw,
                                   &lds_bytes);
    if (rc != MAZE_OK) return rc;
    if (variant) {
        if (epw == 128)
            covered = launch_rollout<K, Word, 128, 1>(ctx, 0, p.N, d_actions, n_steps, d_reward, d_done,
                                                      d_obs, st);
        else if (epw == 64)
            covered = launch_rollout<K, Word, 64, 1>(ctx, 0, p.N, d_actions, n_steps, d_reward, d_done,
                                                     d_obs, st);
        else if (epw == 16)
            covered = launch_rollout<K, Word, 16, 1>(ctx, 0, p.N, d_actions, n_steps, d_reward, d_done,
                                                     d_obs, st);
        return launch_rest<K, Word, 1>(ctx, covered, d_actions, n_steps, d_reward, d_done, d_obs, st);
    }
    if (epw == 128)
        covered = launch_rollout<K, Word, 128>(ctx, 0, p.N, d_actions, n_steps, d_reward, d_done, d_obs, st);
    else if (epw == 64)
        covered = launch_rollout<K, Word, 64>(ctx, 0, p.N, d_actions, n_steps, d_reward, d_done, d_obs, st);
    else if (epw == 16)
        covered = launch_rollout<K, Word, 16>(ctx, 0, p.N, d_actions, n_steps, d_reward, d_done, d_obs, st);
    return launch_rest<K, Word, 0>(ctx, covered, d_actions, n_steps, d_reward, d_done, d_obs, st);
}

// Word size dispatch for one view size; the translation units maze_student_tiled_k*.hip wrap it.
template <int K>
int launch_view_size(const maze_ctx *ctx, const int8_t *d_actions, int n_steps, float *d_reward,
                     uint8_t *d_done, int8_t *d_obs, hipStream_t st)
{
    return ctx->word64 ? launch_k<K, uint64_t>(ctx, d_actions, n_steps, d_reward, d_done, d_obs, st)
                       : launch_k<K, uint32_t>(ctx, d_actions, n_steps, d_reward, d_done, d_obs, st);
}

}  // namespace
