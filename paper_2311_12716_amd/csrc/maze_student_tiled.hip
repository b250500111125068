// Entry of the tiled store-layout kernels of the student env: picks the view size.
#include "maze_internal.h"

#define MAZE_DECLARE_VIEW_SIZE(K)                                                                  \
    int student_tiled_launch_k##K(const maze_ctx *ctx, const int8_t *d_actions, int n_steps,        \
                                  float *d_reward, uint8_t *d_done, int8_t *d_obs, hipStream_t st); \
    int student_tiled_plan_k##K(int N, int SP, bool typed, bool occlusion, int cus, size_t budget, \
                                int *epw, size_t *lds_bytes);
MAZE_DECLARE_VIEW_SIZE(3)
MAZE_DECLARE_VIEW_SIZE(5)
MAZE_DECLARE_VIEW_SIZE(7)

// Launch the tiled kernels on the first `*covered` envs and report how many they took; the
// caller runs the per-cell kernel on the rest.  n_steps == 0 renders the current state;
// n_steps == 1 is one step + observation in one light launch (whole groups of 64 envs).
// Returns 1 if it launched, 0 if no tiled kernel applies (no observation wanted, or a view
// size other than 3, 5, 7), or a negative error code (MAZE_EHIP: the device refused the LDS
// a workgroup needs) -- never a silent switch to the slow kernel for a shape it covers.
int student_tiled_launch(const maze_ctx *ctx, const int8_t *d_actions, int n_steps, float *d_reward,
                         uint8_t *d_done, int8_t *d_obs, int *covered, hipStream_t st)
{
    *covered = 0;
    if (!d_obs) return 0;
    if (ctx->dev.max_steps >= (1 << 29)) return 0;   // the step count shares a word with heading and done
    int done_envs;
    switch (ctx->dev.k) {
    case 3: done_envs = student_tiled_launch_k3(ctx, d_actions, n_steps, d_reward, d_done, d_obs, st); break;
    case 5: done_envs = student_tiled_launch_k5(ctx, d_actions, n_steps, d_reward, d_done, d_obs, st); break;
    case 7: done_envs = student_tiled_launch_k7(ctx, d_actions, n_steps, d_reward, d_done, d_obs, st); break;
    default: return 0;
    }
    if (done_envs < 0) return done_envs;
    *covered = done_envs;
    return done_envs > 0;
}

// The shape of a rollout launch for one view size (see maze_rollout_plan in the header).
int student_tiled_plan(int k, int N, int SP, bool typed, bool occlusion, int cus, size_t budget,
                       int *epw, size_t *lds_bytes)
{
    switch (k) {
    case 3: return student_tiled_plan_k3(N, SP, typed, occlusion, cus, budget, epw, lds_bytes);
    case 5: return student_tiled_plan_k5(N, SP, typed, occlusion, cus, budget, epw, lds_bytes);
    case 7: return student_tiled_plan_k7(N, SP, typed, occlusion, cus, budget, epw, lds_bytes);
    default: *epw = 0; *lds_bytes = 0; return MAZE_OK;
    }
}
