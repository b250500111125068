// Tiled student kernels for a 3 x 3 view (one translation unit per view size, so that they
// compile side by side).
#include "maze_student_tiled.h"

int student_tiled_launch_k3(const maze_ctx *ctx, const int8_t *d_actions, int n_steps, float *d_reward,
                             uint8_t *d_done, int8_t *d_obs, hipStream_t st)
{
    return launch_view_size<3>(ctx, d_actions, n_steps, d_reward, d_done, d_obs, st);
}

int student_tiled_plan_k3(int N, int SP, bool typed, bool occlusion, int cus, size_t budget, int *epw,
                          size_t *lds_bytes)
{
    return plan_view_size<3>(N, SP, typed, occlusion, cus, budget, epw, lds_bytes);
}
