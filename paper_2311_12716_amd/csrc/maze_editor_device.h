// Device helpers of the teacher editor env shared by its kernels.
#pragma once

#include "maze_internal.h"

// One placement applied to an env's bit stream (bit 3c+ch = channel ch of cell c).
__device__ __forceinline__ void editor_apply(const EditorDev &p, uint32_t *__restrict__ s,
                                             int32_t &t, int32_t &ac, int32_t &gc, int action)
{
    int a = min(max(action, 0), p.cells - 1);
    if (t < p.n_walls) {
        s[(3 * a) >> 5] |= 1u << ((3 * a) & 31);
    } else if (t == p.n_walls) {
        ac = a;
        s[(3 * a) >> 5] &= ~(1u << ((3 * a) & 31));
        s[(3 * a + 2) >> 5] |= 1u << ((3 * a + 2) & 31);
    } else if (t == p.n_walls + 1) {
        int j = (a == ac) ? ((a + 1 == p.cells) ? 0 : a + 1) : a;
        gc = j;
        s[(3 * j) >> 5] &= ~(1u << ((3 * j) & 31));
        s[(3 * j + 1) >> 5] |= 1u << ((3 * j + 1) & 31);
    }
    if (t < p.n_walls + 2) t += 1;
}
