// Device helpers of the store-layout kernels (student and editor): bit-to-byte expansion
// and 16-byte global accesses of any alignment.
#pragma once

#include "maze_internal.h"

// 4 stream bits -> 4 bytes (bit j -> byte j).  The four shifted copies do not
// overlap, so the multiply carries nothing.
__device__ __forceinline__ uint32_t expand_nibble(uint32_t nib)
{
    return (nib * 0x00204081u) & 0x01010101u;
}

// 16-byte global accesses at addresses of any alignment (a batch size or a buffer offset that
// is not a multiple of 16 shifts every step's block): a plain 16-byte copy, which compiles to
// one dwordx4 instruction on this target whatever the alignment.
__device__ __forceinline__ void store16(int8_t *dst, const uint4 &v) { __builtin_memcpy(dst, &v, 16); }

// The same store for output that is a pure stream -- nothing on the chip reads it back -- and
// whose 128-byte line is written completely by one store instruction of a wave:
// non-temporal, system scope (written through, nothing of it kept).  Each of the 8 XCDs has
// an L2 of its own, so a kernel's output has to leave them before the next kernel starts;
// without the hint the rollout's output collects there as dirty lines and is written back
// when the kernel ends.  Measured on config 3, 256-step rollout, launches back to back: plain
// stores 133.5 us, nt 127.1, sc0 sc1 nt 125.2, sc0 sc1 alone 134.3.  Lines that two store
// instructions share must not carry the hint: they would leave the L2 half written and be
// merged in memory (config 5, whose 4704-byte chunks end inside lines: 129 -> 152 us with nt
// on every store; the same on the rollout's 4-byte reward and 1-byte done stores: 127 -> 135).
//
// base: the same for every lane of the wave (a workgroup's block of a step); offset: this
// lane's byte offset in it, at any alignment.  A raw buffer store whose descriptor spans
// [base, base + 2^32) and whose cache bits are an argument (buffer_store_dwordx4 ... offen
// sc0 nt sc1).  It is a builtin, not inline assembly, on purpose: the compiler places the
// wait states a 16-byte store needs before its data registers may be overwritten only for
// instructions it knows, and a store written as assembly text had later lanes' data
// overwritten in flight.
typedef uint32_t maze_u4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store16_stream(int8_t *base, uint32_t offset, const uint4 &v)
{
    const uint64_t b = (uint64_t)(uintptr_t)base;
    const uint64_t uniform = ((uint64_t)__builtin_amdgcn_readfirstlane((int)(b >> 32)) << 32) |
                             (uint32_t)__builtin_amdgcn_readfirstlane((int)b);
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)(uintptr_t)uniform, 0, -1, 0x00020000);
    const maze_u4 t = {v.x, v.y, v.z, v.w};
    __builtin_amdgcn_raw_buffer_store_b128(t, rsrc, (int)offset, 0, 0x13);      // sc0 | nt | sc1
}
__device__ __forceinline__ uint4 load16(const int8_t *src)
{
    uint4 v;
    __builtin_memcpy(&v, src, 16);
    return v;
}

// Pacing of a store wave.  The memory system takes the observation stream fastest when it is
// offered at a steady rate just below what it can sustain; offered more -- every wave storing
// as fast as the queues accept -- its throughput drops by a fifth (config 3: 125 us per
// rollout launch unpaced, 110 paced).  So a store wave keeps to a schedule: pace_fp is the time
// one step of the whole launch should take (ticks of the constant-rate clock, 8 fractional
// bits; 0 = no pacing); a block of steps gets that much time, and what the wave does not need
// for its own work -- the previous block's time less its sleep -- it sleeps, in units spread
// between the block's stores.  The schedule is absolute, so errors do not add up; a wave that
// falls a whole block behind restarts it instead of catching up in a burst; a wave that
// cannot keep it at all (the launch is bound by something else) drops it after four blocks
// and costs nothing from then on.
struct StorePacer {
    uint32_t pace;        // ticks per step (8 fractional bits), 0 = off
    uint32_t unit_fp;     // one sleep unit (s_sleep 1) in the same measure, calibrated at the start
    uint32_t work_fp;     // the previous block's duration less its sleep
    uint64_t sched_fp;    // when the current block's stores should be out
    uint64_t t_begin;
    uint32_t units;       // sleep units of the current block
    int behind;           // blocks in a row without time to sleep (-1: before the first block)

    __device__ __forceinline__ static uint64_t now_fp() { return __builtin_amdgcn_s_memrealtime() << 8; }
    __device__ __forceinline__ static void nap(uint32_t n)
    {
        for (uint32_t q = 0; q < n; ++q) __builtin_amdgcn_s_sleep(1);
    }
    __device__ __forceinline__ void init(uint32_t pace_fp)
    {
        pace = pace_fp; unit_fp = 256; work_fp = 0; sched_fp = 0; t_begin = 0; units = 0; behind = -1;
        if (pace) {
            const uint64_t c0 = now_fp();
#pragma unroll
            for (int q = 0; q < 16; ++q) __builtin_amdgcn_s_sleep(1);
            unit_fp = max(16u, (uint32_t)((now_fp() - c0) >> 4));
        }
    }
    // Start a block of `steps` steps; returns the sleep units to spread over it (at most max_units).
    __device__ __forceinline__ uint32_t begin(uint32_t steps, uint32_t max_units)
    {
        units = 0;
        if (!pace) return 0;
        t_begin = now_fp();
        const uint64_t block_fp = (uint64_t)steps * pace;
        if (behind < 0) { sched_fp = t_begin; behind = 0; }
        sched_fp += block_fp;
        const int64_t spare = (int64_t)(sched_fp - t_begin) - (int64_t)work_fp;
        if (spare >= (int64_t)unit_fp) {
            units = min(max_units, (uint32_t)(spare / unit_fp));
            behind = 0;
        } else {
            if (spare < -(int64_t)block_fp) sched_fp = t_begin + block_fp;
            if (++behind >= 4) pace = 0;
        }
        return units;
    }
    __device__ __forceinline__ void end()
    {
        if (!pace) return;
        const uint64_t took = now_fp() - t_begin, slept = (uint64_t)units * unit_fp;
        work_fp = took > slept ? (uint32_t)min((uint64_t)0x7FFFFFFF, took - slept) : 0u;
    }
};

// The same for a piece of which only the first `valid` (< 16) bytes exist (the last, partly
// filled workgroup of a batch).
__device__ __forceinline__ void store_bytes(int8_t *dst, const uint4 &v, int valid)
{
    // 8, 4, 2 and 1 bytes as the bits of `valid` say: at most four stores
    uint64_t cur = ((uint64_t)v.y << 32) | v.x;
    if (valid & 8) {
        __builtin_memcpy(dst, &cur, 8);
        dst += 8;
        cur = ((uint64_t)v.w << 32) | v.z;
    }
    if (valid & 4) {
        const uint32_t w = (uint32_t)cur;
        __builtin_memcpy(dst, &w, 4);
        dst += 4;
        cur >>= 32;
    }
    if (valid & 2) {
        const uint16_t h = (uint16_t)cur;
        __builtin_memcpy(dst, &h, 2);
        dst += 2;
        cur >>= 16;
    }
    if (valid & 1) *dst = (int8_t)cur;
}

// The first `valid` (< 16) bytes at src, the rest zero.
__device__ __forceinline__ uint4 load_bytes(const int8_t *src, int valid)
{
    uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
    for (int b = 0; b < 16; ++b)
        if (b < valid) w[b >> 2] |= (uint32_t)(uint8_t)src[b] << (8 * (b & 3));
    return make_uint4(w[0], w[1], w[2], w[3]);
}

// The hardware hands consecutive workgroups of a launch to the 8 XCDs in turn, each with an L2 of
// its own.  Neighbouring workgroups write neighbouring byte ranges whose ends share a 128-byte
// line unless the range is a whole number of lines (32 student envs x 147 B is not); this renumbering
// gives every XCD a contiguous range of workgroups, so that such a line is completed within one L2
// instead of leaving two of them in parts.  (If the assignment were different the result would
// be the same, only the gain lost.)
__device__ __forceinline__ int xcd_contiguous(int block, int blocks)
{
    const int xcd = block & 7, turn = block >> 3;
    const int each = blocks >> 3, extra = blocks & 7;       // the first `extra` XCDs get one more
    return xcd * each + min(xcd, extra) + turn;
}
