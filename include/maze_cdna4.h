/*
 * maze_cdna4 -- batched MiniGrid-style maze environment for AMD CDNA4 (gfx950).
 *
 * C ABI of the data-parallel hot path of unsupervised-environment-design
 * training on mazes (the "AMaze" benchmark of the minimax paper, Section 3):
 * the student's step + egocentric observation, the teacher's sequential level
 * editor (Section 2.2), and generalised advantage estimation (appendix on
 * hyperparameters).  All compute runs in HIP kernels; this header has no C++
 * or framework types in it.
 *
 * Conventions shared by every call
 *   - Pointers named d_* are DEVICE pointers owned by the caller; the library
 *     never frees or retains them beyond the call, except the workspace given
 *     to *_create, which must stay alive until *_destroy.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls validate their arguments on the host, enqueue kernels on `stream`
 *     and return without synchronising.  Two calls on the same context must be
 *     ordered by the caller (same stream, or events).
 *   - A context belongs to the device that was current at *_create; every later
 *     call on it must be made with that device current (MAZE_EINVAL otherwise)
 *     and with a stream of that device.
 *   - Return value: MAZE_OK (0) or a negative MAZE_E* code; nothing aborts or
 *     throws.  maze_strerror() names a code.
 *   - Coordinates: x = column (grows right), y = row (grows down); interior
 *     cells 0 <= x < W, 0 <= y < H; everything outside the interior is wall.
 *     Heading: 0 = +x, 1 = +y, 2 = -x, 3 = -y.  Batched arrays are env-major
 *     within a time step: [n_steps][N]...
 */
#ifndef MAZE_CDNA4_H
#define MAZE_CDNA4_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MAZE_OK       0
#define MAZE_EINVAL  (-1)   /* argument out of range                         */
#define MAZE_ENULL   (-2)   /* required pointer is NULL                       */
#define MAZE_ESIZE   (-3)   /* grid/view too large for the packed layout, or
                               workspace too small                             */
#define MAZE_EHIP    (-4)   /* a HIP runtime call failed                      */

typedef struct maze_ctx maze_ctx;       /* small host-side handle */
typedef struct editor_ctx editor_ctx;   /* small host-side handle */

const char *maze_strerror(int code);

/* ------------------------------------------------------------------ student
 * Static parameters (paper Section 2.2: fixed at initialisation): number of
 * envs N, interior size H x W, odd view size k >= 3, episode cap max_steps (250
 * in the paper's experiments, Section 4).  Limits: W + 2(k-1) <= 64 and
 * H + 2(k-1) <= 64 (the walls are kept as one machine word per padded row),
 * 1 <= max_steps < 2^24; k = 1 or even k: MAZE_EINVAL (the k-1 rings of wall the
 * layout pads the grid with are also what bounds the agent's moves).
 *
 * maze_workspace_bytes: device bytes maze_create needs for these parameters.
 * maze_create: builds the host handle; d_workspace must be 256-byte aligned.
 * The state is undefined until the first maze_reset_to_levels.               */
int maze_workspace_bytes(int N, int H, int W, int view, size_t *out);
int maze_create(maze_ctx **out, int N, int H, int W, int view, int max_steps,
                void *d_workspace, size_t workspace_bytes);
int maze_destroy(maze_ctx *ctx);

/* Set every env's free parameters (its level) and put the agent on the start
 * pose with t = 0 -- the state setter of Section 2.2, and the hand-off target
 * of the teacher's final design.
 *   d_walls     int8  [N,H,W]  non-zero = wall
 *   d_agent_xy  int32 [N,2]    start (x,y)
 *   d_agent_dir int8  [N]      start heading
 *   d_goal_xy   int32 [N,2]
 * Preconditions (caller's): agent and goal inside the interior, on free,
 * distinct cells.  For memory safety coordinates are clamped into the interior
 * and the heading is taken modulo 4.  Other violations are simulated as they
 * stand: a goal on a wall cell is never reached and renders as wall; an agent
 * that starts on the goal finishes the episode on its first step.             */
int maze_reset_to_levels(maze_ctx *ctx, const int8_t *d_walls, const int32_t *d_agent_xy,
                         const int8_t *d_agent_dir, const int32_t *d_goal_xy, void *stream);

/* n_steps >= 1 environment steps for all N envs (Section 3: goal-reaching maze
 * with MiniGrid semantics).  Per env and step:
 *   t += 1; action 0 = turn left, 1 = turn right, 2 = forward unless the cell
 *   ahead is a wall; any other value changes nothing but still counts a step;
 *   reached = agent on goal; reward = 1 - 0.9*t/max_steps if reached else 0;
 *   done = reached or t >= max_steps; if done the agent returns to the level's
 *   start pose and t = 0 (same level).
 *   d_actions int8  [n_steps,N]
 *   d_reward  float [n_steps,N]
 *   d_done    uint8 [n_steps,N]
 *   d_obs     int8  [n_steps,N,k,k,3] or NULL: observation AFTER each step (of
 *             the reset state when done), same encoding as maze_render_obs.
 * n_steps > 1 runs the whole open-loop rollout in one launch with the state
 * held on chip; n_steps = 1 is the plain step a policy loop calls.
 * Speed: calls with d_obs and k in {3, 5, 7} run the store-layout kernels (the
 * observation leaves the chip as 16-byte pieces of contiguous runs); calls
 * without d_obs, other view sizes and the last N mod 64 envs of a single step
 * run a one-lane-per-env kernel that writes the observation byte by byte --
 * same results, several times slower.  MAZE_EHIP if the device does not grant
 * the LDS a workgroup of the rollout needs (up to 127 KB; never a silent switch
 * of kernels).                                                                */
int maze_step(maze_ctx *ctx, const int8_t *d_actions, int n_steps, float *d_reward,
              uint8_t *d_done, int8_t *d_obs, void *stream);

/* How a rollout (maze_step with d_obs and n_steps > 1) of these static parameters would be
 * launched on a device with `cus` compute units and lds_per_cu bytes of LDS per unit (what
 * maze_create reads from the device properties): envs per workgroup of the main launch (128,
 * 64, 32 or 16; 0 if the view size is not one the store-layout kernels take, the one-lane-per-env
 * kernel then runs) and the LDS bytes such a workgroup needs.  Host arithmetic only, no GPU
 * is touched.  MAZE_EHIP if even 32 envs per workgroup do not fit -- the error maze_step
 * returns on such a device; argument errors as for maze_create and maze_set_obs_mode.     */
int maze_rollout_plan(int N, int H, int W, int view, int encoding, int occlusion, int cus,
                      size_t lds_per_cu, int *envs_per_workgroup, size_t *lds_bytes);

/* For callers that cannot allocate device memory -- code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc: maze_reset_to_levels followed by maze_step
 * on a fresh env, with no context and no workspace.  The packed levels and the env state are
 * kept in a static device array of MAZE_STATIC_WORKSPACE_BYTES inside the library (each GPU
 * the library runs on holds its copy until the process ends); the call allocates nothing on
 * the host or the device.  Arguments as for maze_create (N, H, W, view, max_steps),
 * maze_reset_to_levels (the levels) and maze_step (d_actions [n_steps,N], d_reward, d_done,
 * d_obs or NULL); all d_* are device pointers owned by the caller; the kernels are enqueued
 * on `stream` of the current device and nothing synchronises.  The env state is not kept
 * for a later call: every call starts from the levels' start poses with t = 0, with the
 * default observation (one-hot, no occlusion).
 * Limit: maze_workspace_bytes(N, H, W, view) <= MAZE_STATIC_WORKSPACE_BYTES (16 MiB), which
 * holds e.g. 32768 envs of 13 x 13 with view 5 (11.9 MB) or 8192 envs of 51 x 51 with view 7
 * (16.7 MB); MAZE_ESIZE beyond it.  Other errors as for the three calls it stands for.
 * All calls on one GPU share the one array: two calls that may overlap in time (different
 * streams, or host threads without ordering) race and give undefined results; calls on one
 * stream are safe back to back.                                                         */
#define MAZE_STATIC_WORKSPACE_BYTES (16u << 20)
int maze_rollout_static(int N, int H, int W, int view, int max_steps, const int8_t *d_walls,
                        const int32_t *d_agent_xy, const int8_t *d_agent_dir,
                        const int32_t *d_goal_xy, const int8_t *d_actions, int n_steps,
                        float *d_reward, uint8_t *d_done, int8_t *d_obs, void *stream);

/* Egocentric k x k observation of the current state (Section 3: partially
 * observable).  d_obs int8 [N,k,k,3]; view row 0 is farthest ahead, the agent
 * is at row k-1, column k/2, facing row 0; column 0 is on its left.  Channels
 * are one-hot (wall, goal, empty); the agent's own cell reads empty; cells
 * outside the interior are wall; no occlusion.                                */
int maze_render_obs(maze_ctx *ctx, int8_t *d_obs, void *stream);

/* State / level getters (Section 2.2).  d_xy int32 [N,2], d_dir int8 [N],
 * d_t int32 [N]; level arrays as in maze_reset_to_levels.  Any pointer may be
 * NULL to skip that output.                                                   */
int maze_get_state(maze_ctx *ctx, int32_t *d_xy, int8_t *d_dir, int32_t *d_t, void *stream);

/* State setter (Section 2.2: the env exposes a getter and a setter for its state).
 * Overwrites the running state of every env -- position, heading, steps taken in
 * the current episode -- and leaves the levels (walls, start pose, goal) as they
 * are, so that a state read with maze_get_state, or any other, can be continued
 * from.  d_xy int32 [N,2] (x, y), clamped into the interior; d_dir int8 [N],
 * taken mod 4; d_t int32 [N], clamped to [0, max_steps - 1].  A NULL pointer
 * keeps that part of the state.  Device pointers, owned by the caller; enqueued
 * on stream.  Returns MAZE_ENULL for a NULL ctx.                              */
int maze_set_state(maze_ctx *ctx, const int32_t *d_xy, const int8_t *d_dir, const int32_t *d_t,
                   void *stream);
int maze_get_levels(maze_ctx *ctx, int8_t *d_walls, int32_t *d_agent_xy, int8_t *d_agent_dir,
                    int32_t *d_goal_xy, void *stream);

/* Level metrics of the levels held by ctx (Section 2.2: per-level metrics such as
 * the number of walls; Section 3: shortest paths, which the paper computes with a
 * matrix-based all-pairs algorithm -- the distance between two given cells is the
 * same number whichever way it is found).
 *   d_n_walls  int32 [N]: interior wall cells
 *   d_path_len int32 [N]: fewest moves between 4-neighbouring non-wall cells from
 *                         the level's start cell to its goal cell (turns are free);
 *                         0 if they coincide, -1 if the goal cannot be reached or
 *                         the start cell is a wall.
 * Either pointer may be NULL.  Depends only on the levels, not on the current
 * state.                                                                         */
int maze_level_metrics(maze_ctx *ctx, int32_t *d_n_walls, int32_t *d_path_len, void *stream);

/* Choose the kernel family used by maze_step / maze_render_obs: 0 = automatic
 * (the tiled store-layout kernels when the shape allows, else the per-cell
 * kernel), 1 = always the per-cell kernel.  Results are identical; meant for
 * tests and measurements.                                                     */
int maze_set_kernel_variant(maze_ctx *ctx, int variant);

/* Observation variants (Section 3: the maze reproduces the MiniGrid mazes of prior
 * work, whose observation hides what lies behind walls and describes a cell by
 * object type, colour and state), for maze_step and maze_render_obs from the next
 * call on.  Shape and index order of d_obs do not change.
 *   encoding  0 (default): one-hot (wall, goal, empty)
 *             1: (type, colour, state) with MiniGrid's indices: empty (1,0,0),
 *                wall (2,5,0), goal (8,1,0), unseen (0,0,0)
 *   occlusion 0 (default): every cell of the window is shown
 *             1: a cell is seen if a chain of seen non-wall cells leads to it from
 *                the agent's cell, each link going sideways within a view row or to
 *                one of the three touching cells of the next row ahead; seen walls
 *                pass nothing on; an unseen cell reads zero in all channels.
 * MAZE_EINVAL for other values.                                                 */
int maze_set_obs_mode(maze_ctx *ctx, int encoding, int occlusion);

/* ------------------------------------------------------------------- teacher
 * The teacher's design MDP (Section 2.2): an empty H x W grid on which the
 * teacher places n_walls walls, then the agent, then the goal, one cell index
 * (row-major, y*W + x) per step.  Limits: H*W <= 4096, n_walls >= 0.
 *
 * Per env and step, with t the number of placements made so far:
 *   the action is clamped into [0, H*W);
 *   t <  n_walls   : the cell becomes a wall (again, if it already is one);
 *   t == n_walls   : the agent is put there with heading agent_dir_init, a wall
 *                    on that cell is removed;
 *   t == n_walls+1 : the goal is put there; if that is the agent's cell the goal
 *                    moves on to the next cell in row-major order (cyclically);
 *                    a wall on the goal's cell is removed;
 *   t <- t+1 while t < n_walls+2; later steps change nothing.
 *   done = (t == n_walls+2).                                                  */
int editor_workspace_bytes(int N, int H, int W, size_t *out);
int editor_create(editor_ctx **out, int N, int H, int W, int n_walls,
                  void *d_workspace, size_t workspace_bytes);
int editor_destroy(editor_ctx *ctx);

/* Empty grid, nothing placed, t = 0; latches the heading each env's agent will
 * get (d_agent_dir_init int8 [N], taken modulo 4).                            */
int editor_reset(editor_ctx *ctx, const int8_t *d_agent_dir_init, void *stream);

/*   d_actions int32 [n_steps,N]
 *   d_obs     int8  [n_steps,N,H,W,3] or NULL: full grid after each step,
 *             channels (wall, goal, agent)
 *   d_t       int32 [n_steps,N] or NULL: t after each step
 *   d_done    uint8 [n_steps,N] or NULL                                        */
int editor_step(editor_ctx *ctx, const int32_t *d_actions, int n_steps, int8_t *d_obs,
                int32_t *d_t, uint8_t *d_done, void *stream);

/* The designed levels in exactly the layout maze_reset_to_levels takes (the
 * reset_student hand-off of Section 2.2).  Before the agent / goal is placed
 * its coordinates read (-1,-1) and the heading 0.                             */
int editor_get_levels(editor_ctx *ctx, int8_t *d_walls, int32_t *d_agent_xy,
                      int8_t *d_agent_dir, int32_t *d_goal_xy, void *stream);

/* Load finished levels into the editor env (Section 2.2: setter of the free
 * parameters), e.g. levels of a replay buffer that are to be mutated.  Arrays as
 * in maze_reset_to_levels; any non-zero wall byte is a wall; coordinates are
 * clamped into the interior; the heading is taken modulo 4; everything else is
 * copied as it is.  Afterwards the design episode counts as finished
 * (t = n_walls + 2).                                                             */
int editor_set_levels(editor_ctx *ctx, const int8_t *d_walls, const int32_t *d_agent_xy,
                      const int8_t *d_agent_dir, const int32_t *d_goal_xy, void *stream);

/* Random levels drawn on the device (Section 3: mazes with randomly sampled wall,
 * goal and agent positions; the random generator of the DR and replay baselines).
 * Env n becomes level first_level_id + n of the generator `seed`: the outcome of a
 * design episode under uniformly random actions -- n_walls wall placements
 * (repeats allowed), the agent, the goal -- with a uniformly random heading.  The
 * draws come from the counter-based generator Philox-4x32-10 with key = seed and
 * counter = (id low, id high, draw / 4, 0), draw j = word j % 4; draws 0 ..
 * n_walls+1 are the placements, draw n_walls+2 the heading (low two bits); a draw
 * u selects cell floor(u * H*W / 2^32).  A level depends on (seed, id, H, W,
 * n_walls) only, not on N.  Replaces the env's whole state; no observation is
 * written.                                                                       */
int editor_random_levels(editor_ctx *ctx, uint64_t seed, uint64_t first_level_id, void *stream);

/* Mutate the levels held by the editor env (the mutations of the ACCEL baseline,
 * "number of mutations" in the hyperparameter tables): n_edits times, draw a cell
 * uniformly (counter (id low, id high, draw / 4, 1) of the same generator); if it
 * holds the agent or the goal nothing happens, otherwise its wall bit is flipped.
 * n_edits >= 0 (MAZE_EINVAL otherwise).                                          */
int editor_mutate_levels(editor_ctx *ctx, uint64_t seed, uint64_t first_level_id, int n_edits,
                         void *stream);

/* ----------------------------------------------------------------------- GAE
 * Generalised advantage estimation (PPO with GAE, appendix on hyperparameters;
 * gamma, lambda as in the hyperparameter table).  Per env, backwards in time:
 *   delta_t = r_t + gamma * V_{t+1} * (1 - d_t) - V_t
 *   A_t     = delta_t + gamma * lambda * (1 - d_t) * A_{t+1},   A_T = 0
 *   ret_t   = A_t + V_t
 *   d_rewards float [T,N], d_values float [T+1,N], d_dones uint8 [T,N],
 *   d_adv float [T,N], d_returns float [T,N] or NULL.
 * The recurrence is carried in double and rounded to float on output.         */
int compute_gae(const float *d_rewards, const float *d_values, const uint8_t *d_dones,
                int T, int N, double gamma, double lambda, float *d_adv, float *d_returns,
                void *stream);

/* Replay scores of a rollout, one per env = per level (Appendix, hyperparameters:
 * the PLR scoring function is MaxMC, the maximum Monte Carlo regret estimator, or
 * PVL, the positive value loss estimator).  Inputs as for compute_gae plus its
 * advantages d_adv float [T,N]; evaluated in double, rounded once to float:
 *   G_t   = r_t + gamma (1-d_t) G_{t+1},  G_T = V_T   (Monte Carlo return; an episode
 *           cut off by the end of the rollout is completed with the value estimate)
 *   best  = max(max_t G_t, d_rmax_in[n] if d_rmax_in is not NULL)
 *   d_rmax_out[n] = best;  d_maxmc[n] = best - mean_t V_t;  d_pvl[n] = mean_t max(A_t, 0)
 * Means run over all T steps.  d_rmax_in may be NULL (no return seen yet) and may
 * alias d_rmax_out; any output may be NULL.  T, N >= 1 (MAZE_EINVAL otherwise).   */
int replay_scores(const float *d_rewards, const float *d_values, const uint8_t *d_dones,
                  const float *d_adv, int T, int N, double gamma, const float *d_rmax_in,
                  float *d_rmax_out, float *d_maxmc, float *d_pvl, void *stream);

/* Probability of replaying each of the K levels of a buffer (Appendix, hyperparameter
 * tables: prioritization rank or proportional, temperature beta, staleness
 * coefficient rho; formulas of the prioritized-level-replay work the paper cites):
 *   h_i = 1 / rank_i (rank 1 = highest score; equal scores: lower index first), or
 *         max(score_i, 0) if rank_prioritization == 0
 *   P_S = h_i^(1/beta) / sum_j h_j^(1/beta)          (uniform if the sum is 0)
 *   P_C = (now - last_seen_i) / sum_j (now - last_seen_j)
 *   d_prob[i] = (1 - rho) P_S + rho P_C              (P_S alone if the second sum is 0)
 * d_scores float [K], d_last_seen int32 [K] (<= now), d_prob float [K]; double
 * arithmetic, rounded once.  1 <= K <= 16384 (MAZE_ESIZE above), beta > 0,
 * 0 <= rho <= 1 (MAZE_EINVAL otherwise).                                           */
int replay_distribution(const float *d_scores, const int32_t *d_last_seen, int K, int now,
                        int rank_prioritization, double temperature, double staleness_coef,
                        float *d_prob, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MAZE_CDNA4_H */
