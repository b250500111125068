// Device helpers of the student env shared by its kernels: conversions between
// padded grid coordinates and the four heading frames, and the move rule.
#pragma once

#include "maze_internal.h"

// Frame d coordinates of the padded cell (X,Y).
__device__ __forceinline__ void padded_to_frame(const StudentDev &p, int d, int X, int Y, int &xd,
                                                int &yd)
{
    switch (d & 3) {
    case 0: xd = Y; yd = p.WP - 1 - X; break;
    case 1: xd = p.WP - 1 - X; yd = p.HP - 1 - Y; break;
    case 2: xd = p.HP - 1 - Y; yd = X; break;
    default: xd = X; yd = Y; break;
    }
}

// Padded cell of frame d coordinates (xd,yd).
__device__ __forceinline__ void frame_to_padded(const StudentDev &p, int d, int xd, int yd, int &X,
                                                int &Y)
{
    switch (d & 3) {
    case 0: X = p.WP - 1 - yd; Y = xd; break;
    case 1: X = p.WP - 1 - xd; Y = p.HP - 1 - yd; break;
    case 2: X = yd; Y = p.HP - 1 - xd; break;
    default: X = xd; Y = yd; break;
    }
}

// One action applied to a pose (Xd | Yd << 8 | d << 16) kept in the frame of its
// heading.  Turning changes the frame: a right turn maps (Xd,Yd) to
// (Yd, bits-1-Xd), a left turn to (rows-1-Yd, Xd), where rows x bits is the shape
// of the current frame's grid.  Forward is one row up unless `blocked`.
__device__ __forceinline__ uint32_t student_move(const StudentDev &p, uint32_t pose, int action,
                                                 bool blocked)
{
    int xd = pose & 255, yd = (pose >> 8) & 255, d = (pose >> 16) & 3;
    int rows_m1 = (d & 1) ? p.HP - 1 : p.WP - 1;
    int bits_m1 = (d & 1) ? p.WP - 1 : p.HP - 1;
    if (action == 0) {
        int nx = rows_m1 - yd, ny = xd;
        xd = nx; yd = ny; d = (d + 3) & 3;
    } else if (action == 1) {
        int nx = yd, ny = bits_m1 - xd;
        xd = nx; yd = ny; d = (d + 1) & 3;
    } else if (action == 2) {
        if (!blocked) yd -= 1;
    }
    return (uint32_t)xd | ((uint32_t)yd << 8) | ((uint32_t)d << 16);
}
