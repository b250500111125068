// Internal definitions shared by the translation units of libmaze_cdna4.
// Not part of the public boundary (see include/maze_cdna4.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "maze_cdna4.h"

#define MAZE_HIP_CHECK(expr)                      \
    do {                                          \
        hipError_t e__ = (expr);                  \
        if (e__ != hipSuccess) return MAZE_EHIP;  \
    } while (0)

static inline size_t maze_align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---------------------------------------------------------------------------
// Student env: device-side layout.
//
// The wall grid is padded with P = k-1 rings of wall cells so that a k x k view
// never leaves the array, and kept as one bit per cell, one machine word per
// padded row.  Four copies are stored, one per heading d, each rotated so that
// heading d points towards smaller row indices ("up") and the agent's right
// hand towards larger bit indices.  In frame d an agent at padded (X,Y) sits at
//     d = 3 (-y): (Xd,Yd) = (X,        Y       )   rows HP, bits WP
//     d = 0 (+x): (Xd,Yd) = (Y,        WP-1-X  )   rows WP, bits HP
//     d = 1 (+y): (Xd,Yd) = (WP-1-X,   HP-1-Y  )   rows HP, bits WP
//     d = 2 (-x): (Xd,Yd) = (HP-1-Y,   X       )   rows WP, bits HP
// and its view is rows Yd-(k-1)..Yd, bits Xd-k/2..Xd+k/2 of grid d, whatever d.
// The dynamic state is kept in the frame of the current heading:
//     pose = Xd | Yd << 8 | d << 16.
// ---------------------------------------------------------------------------
struct StudentDev {
    int N, H, W, k, max_steps;
    int P, HP, WP, SP;      // pad, padded height/width, rows stored per rotated grid
    uint32_t *pose;         // [N] current pose (frame of current heading)
    uint32_t *tcount;       // [N] steps since the episode began
    uint32_t *start;        // [N] start pose (frame of the start heading)
    uint32_t *goalrot;      // [N][4] goal position Xd | Yd << 8 in each frame
    void *grids;            // [N][4][SP] words (uint32_t or uint64_t)
    double reward_slope;    // 0.9 / max_steps
    int obs_encoding;       // 0 one-hot (wall, goal, empty), 1 (type, colour, state)
    int obs_occlusion;      // 0 whole window, 1 cells behind walls are unseen
};

struct maze_ctx {
    StudentDev dev;
    int word64;             // rows need 64-bit words
    int variant;            // 0 auto, 1 per-cell kernels only
    int device;             // the device that was current at maze_create; every call must run on it
    int cus;                // its compute units and the LDS of one of them (device properties):
    size_t lds_per_cu;      // they decide how many envs a workgroup of the rollout takes
    int clock_khz;          // rate of the constant-rate clock kernels read (the rollout paces its stores by it)
    size_t workspace_bytes;
};

// MAZE_OK if the calling thread's current device is the one the context was created on.
static inline int maze_same_device(int ctx_device)
{
    int now = -1;
    if (hipGetDevice(&now) != hipSuccess) return MAZE_EHIP;
    return now == ctx_device ? MAZE_OK : MAZE_EINVAL;
}
#define MAZE_DEVICE_CHECK(ctx)                          \
    do {                                                \
        int rc__ = maze_same_device((ctx)->device);     \
        if (rc__ != MAZE_OK) return rc__;               \
    } while (0)

// The write rate the store waves of a large launch are paced to (see StorePacer).  Rollout
// launches back to back, us per launch, by rate in GB/s (unpaced: config 3 takes 125):
//                                            6900   7000   7100   7200   7300   7500
//   config 3 (256 workgroups x 9600 B/step)  110.7  109.2  108.1  106.6  105.4  103.5
//   65536 envs x 128 steps                   119.1  117.3  117.4  117.8  121.7  125.0
//   view 7 on 20 x 20 grids, 128 steps       113.4  112.8  112.2  112.3  112.7  119.3
//   config 5                                 104.7  103.5  102.5  101.8  101.9  101.7
//   config 3, typed observation              111.8  116.8  118.1  118.5  118.6  117.0
// Past a shape-dependent point the stream falls back towards the unpaced rate, so each constant
// stays below the lowest such point of its kind of launch; the typed observation's store waves
// look every byte up in a table and have less time to spare per block.
#define MAZE_PACED_GBS 7200.0
#define MAZE_PACED_GBS_TYPED 6900.0
// The editor's stream (64896 B per workgroup and step at 13 x 13) turns earlier and sharply:
// config 4, us per reset + step after a long warm-up: 163 unpaced and at 6900 or 7200, 158 at
// 6700, 143.4 at 6550, 146.5 at 6400, 150.9 at 6200 (there and below the schedule alone sets
// the time); the constant keeps a margin to the turn.
#define MAZE_PACED_GBS_EDITOR 6400.0

// Time one step of a launch should take, in ticks of the device's constant-rate clock with 8
// fractional bits, if the workgroups resident at once move bytes_per_step at rate_gbs;
// 0 = do not pace: no clock, an output small enough for the 256 MB memory-side cache to absorb
// most of it (it leaves the chip later: 16384 envs x 256 steps take 52 us unpaced, 57 paced), or
// steps scheduled shorter than a pipeline's own latency per step (such a launch can never be
// ahead of its schedule).
#define MAZE_CACHE_ABSORBS_BYTES (2.0 * 256.0 * 1048576.0)
static inline uint32_t maze_pace_fp(int clock_khz, double bytes_per_step, double out_bytes_total,
                                    double rate_gbs)
{
    if (clock_khz <= 0 || out_bytes_total <= MAZE_CACHE_ABSORBS_BYTES) return 0;
    const double step_ns = bytes_per_step / rate_gbs;                 // bytes / (GB/s) = ns
    const double ticks_fp = step_ns * 1e-6 * clock_khz * 256.0;
    return step_ns >= 150.0 && ticks_fp < 4.0e9 ? (uint32_t)ticks_fp : 0u;
}

// ---------------------------------------------------------------------------
// Teacher editor env: device-side layout.
//
// Per env the grid is kept as the bit stream its observation expands from:
// bit 3*c + ch of the stream is channel ch (0 wall, 1 goal, 2 agent) of cell c.
// ---------------------------------------------------------------------------
struct EditorDev {
    int N, H, W, n_walls;
    int cells;              // H*W
    int SW;                 // stream dwords per env = ceil(3*cells/32)
    uint32_t *stream;       // [N][SW]
    int32_t *agent_cell;    // [N], -1 until placed
    int32_t *goal_cell;     // [N], -1 until placed
    int32_t *t;             // [N]
    int8_t *dir_init;       // [N]
};

struct editor_ctx {
    EditorDev dev;
    int device;
    int cus;                // compute units and clock rate of the device (pacing of the store waves)
    int clock_khz;
    size_t lds_per_cu;      // LDS of a compute unit (the tiled kernel keeps two copies of 128 envs' streams)
    size_t workspace_bytes;
};
