/*
 * CPU oracle for the batched maze hot path.  TEST INFRASTRUCTURE ONLY: the
 * product (the HIP library) never includes, links or calls anything here.
 *
 * One env at a time, one byte per grid cell, scalar loops, no bit tricks,
 * no blocking.  Each function is the plain definition of one operation of the
 * tensorised maze benchmark of the paper (Section 3, "Maze as an Accelerated
 * Petri Dish"; environment interface Section 2.2; PPO+GAE Appendix "Choice of
 * Architecture and Hyperparameters").  Where the paper is silent the reading
 * taken is written next to the code.
 *
 * Conventions: x = column (grows right), y = row (grows down); interior cells
 * 0<=x<W, 0<=y<H; everything outside the interior is wall.  Arrays are
 * row-major [y][x].  dir: 0 = +x, 1 = +y, 2 = -x, 3 = -y.
 *
 * Floating point: rewards and GAE are evaluated in double (the paper fixes no
 * precision); rewards are rounded once to float at the end because the
 * interface type is float32.
 *
 * Parity pins (tests/, "not gpu"): BFS shortest paths on hand-built mazes,
 * scripted levels with known step counts and rewards, rotation / turn
 * invariants, hand-derived observation crops, GAE closed forms, editor
 * scripted cases; level metrics against closed forms, scipy's graph routines
 * and the matrix all-pairs recursion; the random generator against its
 * published known-answer vectors, generated and mutated levels by invariants
 * and statistics; replay scores by closed forms and against GAE at lambda = 1;
 * observation variants by hand-derived visibility masks and graph
 * reachability.  No function here is without a pin.
 */
#include <stdint.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* unit vectors of the four headings, index = dir */
static const int DX[4] = { 1, 0, -1, 0 };
static const int DY[4] = { 0, 1, 0, -1 };

enum { CELL_WALL = 0, CELL_GOAL = 1, CELL_EMPTY = 2 };

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* Is (x,y) a wall for the env whose grid is `walls` (H*W bytes)?  Anything
 * outside the interior is wall: a WxH interior is a (W+2)x(H+2) MiniGrid
 * room whose border is solid, and the view may reach further out still. */
static int is_wall(const int8_t *walls, int H, int W, int x, int y)
{
    if (x < 0 || x >= W || y < 0 || y >= H) return 1;
    return walls[y * W + x] != 0;
}

/* ---------------------------------------------------------------------------
 * Student dynamics, one env, one step (Section 3: goal-reaching maze based on
 * MiniGrid; episode cap, Section 4 "S5 policies": 250 steps).
 *
 *   t <- t+1
 *   action 0: turn left, 1: turn right, 2: forward if the cell ahead is free;
 *   any other value: nothing (the step still counts)
 *   reached = agent on goal;  reward = 1 - 0.9*t/max_steps if reached else 0
 *   done = reached or t >= max_steps
 *   if done: agent back to the level's start pose, t <- 0 (same level)
 * ------------------------------------------------------------------------- */
static void step_one(int H, int W, int max_steps, const int8_t *walls,
                     int sx, int sy, int sdir, int gx, int gy,
                     int *x, int *y, int *dir, int *t, int action,
                     float *reward, uint8_t *done)
{
    *t += 1;
    if (action == 0) {
        *dir = (*dir + 3) % 4;
    } else if (action == 1) {
        *dir = (*dir + 1) % 4;
    } else if (action == 2) {
        int cx = *x + DX[*dir];
        int cy = *y + DY[*dir];
        if (!is_wall(walls, H, W, cx, cy)) {
            *x = cx;
            *y = cy;
        }
    }
    int reached = (*x == gx && *y == gy);
    double r = 0.0;
    if (reached) r = 1.0 - 0.9 * (double)(*t) / (double)max_steps;
    *reward = (float)r;
    int d = reached || (*t >= max_steps);
    *done = (uint8_t)d;
    if (d) {
        *x = sx;
        *y = sy;
        *dir = sdir;
        *t = 0;
    }
}

/* ---------------------------------------------------------------------------
 * Egocentric k x k observation of one env in its current pose (Section 3:
 * "partially-observable").  View row 0 is the row farthest ahead, the agent
 * sits in row k-1, column k/2, looking towards row 0.  View column 0 is on
 * the agent's far left.  Each cell is one-hot over (wall, goal, empty); the
 * agent's own cell shows what it stands on (empty, or goal never happens after
 * a step because that ends the episode).  No occlusion.
 * ------------------------------------------------------------------------- */
static void render_one(int H, int W, int k, const int8_t *walls, int gx, int gy,
                       int x, int y, int dir, int8_t *obs /* [k][k][3] */)
{
    int rdir = (dir + 1) % 4; /* heading of the agent's right hand */
    for (int r = 0; r < k; ++r) {
        for (int c = 0; c < k; ++c) {
            int ahead = (k - 1) - r;
            int side = c - k / 2;
            int wx = x + ahead * DX[dir] + side * DX[rdir];
            int wy = y + ahead * DY[dir] + side * DY[rdir];
            int cell;
            if (is_wall(walls, H, W, wx, wy)) cell = CELL_WALL;
            else if (wx == gx && wy == gy) cell = CELL_GOAL;
            else cell = CELL_EMPTY;
            int8_t *o = obs + ((size_t)r * k + c) * 3;
            o[0] = (cell == CELL_WALL);
            o[1] = (cell == CELL_GOAL);
            o[2] = (cell == CELL_EMPTY);
        }
    }
}

/* Batched single step over N envs.  State (xy, dir, t) is updated in place. */
void orc_maze_step(int N, int H, int W, int max_steps,
                   const int8_t *walls /* [N,H,W] */,
                   const int32_t *start_xy /* [N,2] */, const int8_t *start_dir /* [N] */,
                   const int32_t *goal_xy /* [N,2] */,
                   int32_t *xy /* [N,2] */, int8_t *dir /* [N] */, int32_t *t /* [N] */,
                   const int8_t *actions /* [N] */,
                   float *reward /* [N] */, uint8_t *done /* [N] */)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        int x = xy[2 * n], y = xy[2 * n + 1], d = dir[n], tt = t[n];
        step_one(H, W, max_steps, walls + (size_t)n * H * W,
                 start_xy[2 * n], start_xy[2 * n + 1], start_dir[n],
                 goal_xy[2 * n], goal_xy[2 * n + 1],
                 &x, &y, &d, &tt, actions[n], &reward[n], &done[n]);
        xy[2 * n] = x;
        xy[2 * n + 1] = y;
        dir[n] = (int8_t)d;
        t[n] = tt;
    }
}

/* Batched observation of the current state. */
void orc_maze_render(int N, int H, int W, int k,
                     const int8_t *walls, const int32_t *goal_xy,
                     const int32_t *xy, const int8_t *dir,
                     int8_t *obs /* [N,k,k,3] */)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        render_one(H, W, k, walls + (size_t)n * H * W, goal_xy[2 * n], goal_xy[2 * n + 1],
                   xy[2 * n], xy[2 * n + 1], dir[n], obs + (size_t)n * k * k * 3);
    }
}

/* n_steps of (step, then observe the state after the step and its reset).
 * actions [n_steps,N]; reward, done [n_steps,N]; obs [n_steps,N,k,k,3] or NULL. */
void orc_maze_rollout(int N, int H, int W, int k, int max_steps, int n_steps,
                      const int8_t *walls, const int32_t *start_xy, const int8_t *start_dir,
                      const int32_t *goal_xy, int32_t *xy, int8_t *dir, int32_t *t,
                      const int8_t *actions, float *reward, uint8_t *done, int8_t *obs)
{
    for (int s = 0; s < n_steps; ++s) {
        orc_maze_step(N, H, W, max_steps, walls, start_xy, start_dir, goal_xy, xy, dir, t,
                      actions + (size_t)s * N, reward + (size_t)s * N, done + (size_t)s * N);
        if (obs)
            orc_maze_render(N, H, W, k, walls, goal_xy, xy, dir,
                            obs + (size_t)s * N * k * k * 3);
    }
}

/* ---------------------------------------------------------------------------
 * Observation variants (Section 3: the maze reproduces the MiniGrid mazes of
 * prior work; MiniGrid's own observation hides what lies behind walls and
 * describes a cell by (object type, colour, state)).
 *
 * occlusion = 1: a cell of the k x k view is seen if the agent's own cell is
 * connected to it by a chain of seen cells that are not walls, where a seen
 * non-wall cell passes sight on to its left and right neighbours in its view
 * row and to the three cells of the next row ahead that touch it.  (Walls are
 * seen but pass nothing on; a single pillar therefore hides nothing, a closed
 * wall hides everything behind it.)  Rows are settled from the agent's row
 * outwards.  An unseen cell has all three channels zero.
 *
 * encoding = 1: channels are (type, colour, state) with MiniGrid's published
 * indices: unseen (0,0,0), empty (1,0,0), wall (2,5,0) -- grey --, goal
 * (8,1,0) -- green.  encoding = 0: the one-hot (wall, goal, empty) channels.
 * ------------------------------------------------------------------------- */
enum { MAX_VIEW = 31 };

static void view_cells(int H, int W, int k, const int8_t *walls, int gx, int gy,
                       int x, int y, int dir, int cell[MAX_VIEW][MAX_VIEW])
{
    int rdir = (dir + 1) % 4;
    for (int r = 0; r < k; ++r) {
        for (int c = 0; c < k; ++c) {
            int ahead = (k - 1) - r, side = c - k / 2;
            int wx = x + ahead * DX[dir] + side * DX[rdir];
            int wy = y + ahead * DY[dir] + side * DY[rdir];
            if (is_wall(walls, H, W, wx, wy)) cell[r][c] = CELL_WALL;
            else if (wx == gx && wy == gy) cell[r][c] = CELL_GOAL;
            else cell[r][c] = CELL_EMPTY;
        }
    }
}

static void view_visibility(int k, int cell[MAX_VIEW][MAX_VIEW], int seen[MAX_VIEW][MAX_VIEW])
{
    for (int r = 0; r < k; ++r)
        for (int c = 0; c < k; ++c) seen[r][c] = 0;
    seen[k - 1][k / 2] = 1;                       /* the agent's own cell */
    for (int r = k - 1; r >= 0; --r) {
        /* the agent's cell passes sight on whatever it holds */
        int changed = 1;
        while (changed) {                         /* sideways, until the row is settled */
            changed = 0;
            for (int c = 0; c < k; ++c) {
                int open = cell[r][c] != CELL_WALL || (r == k - 1 && c == k / 2);
                if (!seen[r][c] || !open) continue;
                if (c > 0 && !seen[r][c - 1]) { seen[r][c - 1] = 1; changed = 1; }
                if (c + 1 < k && !seen[r][c + 1]) { seen[r][c + 1] = 1; changed = 1; }
            }
        }
        if (r == 0) break;
        for (int c = 0; c < k; ++c) {             /* on to the next row ahead */
            int open = cell[r][c] != CELL_WALL || (r == k - 1 && c == k / 2);
            if (!seen[r][c] || !open) continue;
            for (int cc = c - 1; cc <= c + 1; ++cc)
                if (cc >= 0 && cc < k) seen[r - 1][cc] = 1;
        }
    }
}

void orc_maze_render_variant(int N, int H, int W, int k, int encoding, int occlusion,
                             const int8_t *walls, const int32_t *goal_xy,
                             const int32_t *xy, const int8_t *dir, int8_t *obs /* [N,k,k,3] */)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        int cell[MAX_VIEW][MAX_VIEW], seen[MAX_VIEW][MAX_VIEW];
        view_cells(H, W, k, walls + (size_t)n * H * W, goal_xy[2 * n], goal_xy[2 * n + 1],
                   xy[2 * n], xy[2 * n + 1], dir[n], cell);
        if (occlusion) view_visibility(k, cell, seen);
        for (int r = 0; r < k; ++r) {
            for (int c = 0; c < k; ++c) {
                int8_t *o = obs + (((size_t)n * k + r) * k + c) * 3;
                int vis = !occlusion || seen[r][c];
                int kind = cell[r][c];
                if (encoding == 0) {
                    o[0] = vis && kind == CELL_WALL;
                    o[1] = vis && kind == CELL_GOAL;
                    o[2] = vis && kind == CELL_EMPTY;
                } else {
                    static const int8_t code[3][3] = { { 2, 5, 0 }, { 8, 1, 0 }, { 1, 0, 0 } };
                    for (int ch = 0; ch < 3; ++ch) o[ch] = vis ? code[kind][ch] : 0;
                }
            }
        }
    }
}

/* ---------------------------------------------------------------------------
 * Teacher's design MDP (Section 2.2: the teacher's decision process is its own
 * environment whose final instance becomes the student's level).
 *
 * Placement order: n_walls wall steps, then the agent, then the goal.  Action
 * = cell index in row-major order, clamped into range.  A wall on a wall
 * changes nothing; the agent clears the wall under it; a goal aimed at the
 * agent's cell moves on cyclically to the next cell, and clears a wall under
 * it.  After the goal is placed further steps change nothing.
 *
 * agent_xy / goal_xy hold -1,-1 until placed.
 * ------------------------------------------------------------------------- */
static void editor_step_one(int H, int W, int n_walls, int8_t *walls,
                            int32_t *agent_xy, int8_t *agent_dir, int32_t *goal_xy,
                            int32_t *t, int dir_init, int action)
{
    int cells = H * W;
    int a = action;
    if (a < 0) a = 0;
    if (a > cells - 1) a = cells - 1;
    if (*t < n_walls) {
        walls[a] = 1;
    } else if (*t == n_walls) {
        agent_xy[0] = a % W;
        agent_xy[1] = a / W;
        *agent_dir = (int8_t)dir_init;
        walls[a] = 0;
    } else if (*t == n_walls + 1) {
        int j = a;
        while (j % W == agent_xy[0] && j / W == agent_xy[1]) j = (j + 1) % cells;
        goal_xy[0] = j % W;
        goal_xy[1] = j / W;
        walls[j] = 0;
    }
    if (*t < n_walls + 2) *t += 1;
}

/* Full-grid teacher observation: channels (wall, goal, agent). */
static void editor_obs_one(int H, int W, const int8_t *walls, const int32_t *agent_xy,
                           const int32_t *goal_xy, int8_t *obs /* [H][W][3] */)
{
    for (int y = 0; y < H; ++y) {
        for (int x = 0; x < W; ++x) {
            int8_t *o = obs + ((size_t)y * W + x) * 3;
            o[0] = walls[y * W + x] != 0;
            o[1] = (goal_xy[0] == x && goal_xy[1] == y);
            o[2] = (agent_xy[0] == x && agent_xy[1] == y);
        }
    }
}

void orc_editor_reset(int N, int H, int W, int8_t *walls, int32_t *agent_xy, int8_t *agent_dir,
                      int32_t *goal_xy, int32_t *t)
{
    for (int n = 0; n < N; ++n) {
        for (int c = 0; c < H * W; ++c) walls[(size_t)n * H * W + c] = 0;
        agent_xy[2 * n] = agent_xy[2 * n + 1] = -1;
        goal_xy[2 * n] = goal_xy[2 * n + 1] = -1;
        agent_dir[n] = 0;
        t[n] = 0;
    }
}

/* n_steps editor steps.  actions [n_steps,N] int32; obs [n_steps,N,H,W,3];
 * t_out, done [n_steps,N] (either may be NULL). */
void orc_editor_rollout(int N, int H, int W, int n_walls, int n_steps,
                        const int8_t *dir_init /* [N] */,
                        int8_t *walls, int32_t *agent_xy, int8_t *agent_dir, int32_t *goal_xy,
                        int32_t *t, const int32_t *actions,
                        int8_t *obs, int32_t *t_out, uint8_t *done)
{
    for (int s = 0; s < n_steps; ++s) {
#pragma omp parallel for schedule(static)
        for (int n = 0; n < N; ++n) {
            editor_step_one(H, W, n_walls, walls + (size_t)n * H * W, agent_xy + 2 * n,
                            agent_dir + n, goal_xy + 2 * n, t + n, dir_init[n],
                            actions[(size_t)s * N + n]);
            if (obs)
                editor_obs_one(H, W, walls + (size_t)n * H * W, agent_xy + 2 * n, goal_xy + 2 * n,
                               obs + ((size_t)s * N + n) * H * W * 3);
            if (t_out) t_out[(size_t)s * N + n] = t[n];
            if (done) done[(size_t)s * N + n] = (t[n] == n_walls + 2);
        }
    }
}

/* ---------------------------------------------------------------------------
 * Generalised advantage estimation (Appendix "Choice of Architecture and
 * Hyperparameters": PPO with GAE, gamma and lambda_GAE of the hyperparameter
 * table).  Per env, backwards in time, in double:
 *   delta_t = r_t + gamma * V_{t+1} * (1-d_t) - V_t
 *   A_t     = delta_t + gamma*lambda * (1-d_t) * A_{t+1},   A_T = 0
 *   ret_t   = A_t + V_t
 * d_t = 1 cuts both the bootstrap and the trace (a time-out counts as an end).
 * ------------------------------------------------------------------------- */
void orc_gae(int T, int N, double gamma, double lambda,
             const float *rewards /* [T,N] */, const float *values /* [T+1,N] */,
             const uint8_t *dones /* [T,N] */,
             double *adv /* [T,N] */, double *ret /* [T,N] or NULL */)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        double A = 0.0;
        for (int s = T - 1; s >= 0; --s) {
            size_t i = (size_t)s * N + n;
            double nd = dones[i] ? 0.0 : 1.0;
            double delta = (double)rewards[i] + gamma * (double)values[i + N] * nd
                           - (double)values[i];
            A = delta + gamma * lambda * nd * A;
            adv[i] = A;
            if (ret) ret[i] = A + (double)values[i];
        }
    }
}

/* ---------------------------------------------------------------------------
 * Level metrics (Section 2.2: environments may report per-level metrics such
 * as the number of walls; Section 3 and the shortest-path figure of Section 4:
 * shortest path length of a maze).
 *
 *   n_walls[n]  = number of interior wall cells
 *   path_len[n] = fewest forward moves that take the agent from its start cell
 *                 to the goal cell through cells that are not walls, moving
 *                 between 4-neighbours; turns cost nothing; 0 if start = goal;
 *                 -1 if the goal cannot be reached.
 *
 * The paper obtains the distances with a matrix-based all-pairs algorithm; a
 * breadth-first search from the start cell defines the same number and is what
 * is written here.  `queue` is caller-provided scratch of H*W ints per thread.
 * ------------------------------------------------------------------------- */
static int bfs_one(int H, int W, const int8_t *walls, int sx, int sy, int gx, int gy,
                   int32_t *dist /* [H*W] */, int32_t *queue /* [H*W] */)
{
    for (int i = 0; i < H * W; ++i) dist[i] = -1;
    if (is_wall(walls, H, W, sx, sy)) return -1;
    int head = 0, tail = 0;
    dist[sy * W + sx] = 0;
    queue[tail++] = sy * W + sx;
    while (head < tail) {
        int c = queue[head++];
        int x = c % W, y = c / W;
        if (x == gx && y == gy) return dist[c];
        for (int d = 0; d < 4; ++d) {
            int nx = x + DX[d], ny = y + DY[d];
            if (is_wall(walls, H, W, nx, ny)) continue;
            if (dist[ny * W + nx] >= 0) continue;
            dist[ny * W + nx] = dist[c] + 1;
            queue[tail++] = ny * W + nx;
        }
    }
    return -1;
}

void orc_level_metrics(int N, int H, int W, const int8_t *walls /* [N,H,W] */,
                       const int32_t *agent_xy /* [N,2] */, const int32_t *goal_xy /* [N,2] */,
                       int32_t *n_walls /* [N] */, int32_t *path_len /* [N] */,
                       int32_t *scratch /* [threads, 2*H*W] */)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
#ifdef _OPENMP
        int32_t *s = scratch + (size_t)omp_get_thread_num() * 2 * H * W;
#else
        int32_t *s = scratch;
#endif
        const int8_t *w = walls + (size_t)n * H * W;
        int count = 0;
        for (int i = 0; i < H * W; ++i) count += w[i] ? 1 : 0;
        n_walls[n] = count;
        path_len[n] = bfs_one(H, W, w, agent_xy[2 * n], agent_xy[2 * n + 1],
                              goal_xy[2 * n], goal_xy[2 * n + 1], s, s + H * W);
    }
}

/* ---------------------------------------------------------------------------
 * Random levels and level mutations drawn on the device (Section 3: mazes with
 * randomly sampled wall, goal and agent positions; Table of baselines: DR uses a
 * random generator, ACCEL mutates levels of its buffer; hyperparameter table:
 * number of mutations).
 *
 * The paper fixes neither the random number generator nor the sampling rule;
 * the readings taken here:
 *
 *  - Random numbers are counter based, so a level's draws depend only on
 *    (seed, level id, purpose, draw index), never on the batch it is part of:
 *    Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random
 *    numbers: as easy as 1, 2, 3", SC'11), key = seed (low, high word),
 *    counter = (level id low, level id high, draw index / 4, purpose), and draw
 *    `index` is output word index % 4.  purpose 0 = generation, 1 = mutation.
 *  - A 32-bit draw u becomes an integer below n as floor(u * n / 2^32).
 *  - A random level is what the teacher's design episode produces under
 *    uniformly random actions: n_walls wall placements (repeats allowed), then
 *    the agent, then the goal, each a uniformly drawn cell (draws 0 ..
 *    n_walls+1); the agent's heading is draw n_walls+2 modulo 4.
 *  - One mutation draws a cell uniformly; if it holds the agent or the goal
 *    nothing happens, otherwise its wall bit is flipped.
 * ------------------------------------------------------------------------- */
static void mulhilo32(uint32_t a, uint32_t b, uint32_t *hi, uint32_t *lo)
{
    uint64_t p = (uint64_t)a * (uint64_t)b;
    *hi = (uint32_t)(p >> 32);
    *lo = (uint32_t)p;
}

void orc_philox4x32(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint32_t hi0, lo0, hi1, lo1;
        mulhilo32(0xD2511F53u, c0, &hi0, &lo0);
        mulhilo32(0xCD9E8D57u, c2, &hi1, &lo1);
        uint32_t n0 = hi1 ^ c1 ^ k0, n1 = lo1, n2 = hi0 ^ c3 ^ k1, n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;          /* key schedule: golden-ratio and sqrt(3)-1 increments */
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

uint32_t orc_level_draw(uint64_t seed, uint64_t level_id, uint32_t purpose, uint32_t index)
{
    uint32_t ctr[4] = { (uint32_t)level_id, (uint32_t)(level_id >> 32), index / 4, purpose };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    orc_philox4x32(ctr, key, out);
    return out[index % 4];
}

uint32_t orc_draw_below(uint32_t u, uint32_t n)
{
    return (uint32_t)(((uint64_t)u * (uint64_t)n) >> 32);
}

/* Levels first_id .. first_id+N-1 of the random generator; the arrays end up in
 * the state of a finished design episode (t = n_walls + 2). */
void orc_editor_random_levels(int N, int H, int W, int n_walls, uint64_t seed, uint64_t first_id,
                              int8_t *walls, int32_t *agent_xy, int8_t *agent_dir,
                              int32_t *goal_xy, int32_t *t, int8_t *dir_init)
{
    orc_editor_reset(N, H, W, walls, agent_xy, agent_dir, goal_xy, t);
    for (int n = 0; n < N; ++n) {
        uint64_t id = first_id + (uint64_t)n;
        dir_init[n] = (int8_t)(orc_level_draw(seed, id, 0, (uint32_t)n_walls + 2) & 3);
        for (int j = 0; j < n_walls + 2; ++j) {
            int action = (int)orc_draw_below(orc_level_draw(seed, id, 0, (uint32_t)j),
                                             (uint32_t)(H * W));
            editor_step_one(H, W, n_walls, walls + (size_t)n * H * W, agent_xy + 2 * n,
                            agent_dir + n, goal_xy + 2 * n, t + n, dir_init[n], action);
        }
    }
}

/* n_edits mutations of each level; mutation draws of level first_id+n. */
void orc_editor_mutate(int N, int H, int W, uint64_t seed, uint64_t first_id, int n_edits,
                       int8_t *walls, const int32_t *agent_xy, const int32_t *goal_xy)
{
    for (int n = 0; n < N; ++n) {
        int8_t *w = walls + (size_t)n * H * W;
        for (int j = 0; j < n_edits; ++j) {
            int c = (int)orc_draw_below(orc_level_draw(seed, first_id + (uint64_t)n, 1, (uint32_t)j),
                                        (uint32_t)(H * W));
            int x = c % W, y = c / W;
            if (x == agent_xy[2 * n] && y == agent_xy[2 * n + 1]) continue;
            if (x == goal_xy[2 * n] && y == goal_xy[2 * n + 1]) continue;
            w[c] = w[c] ? 0 : 1;
        }
    }
}

/* ---------------------------------------------------------------------------
 * Replay scores of a rollout (Appendix, hyperparameters: the PLR scoring
 * function is MaxMC, the maximum Monte Carlo regret estimator, or PVL, the
 * positive value loss estimator; the paper names them and cites prior work for
 * the formulas).  Per env (= per level, an env keeps its level for the whole
 * rollout), in double:
 *
 *   G_t      = r_t + gamma * (1-d_t) * G_{t+1},   G_T = V_T
 *              (Monte Carlo return; an episode cut off by the end of the
 *               rollout is completed with the value estimate)
 *   R_max    = max(R_max before, max_t G_t)       (best return seen on the level)
 *   MaxMC    = mean_t (R_max - V_t)
 *   PVL      = mean_t max(A_t, 0)                 (A_t = the GAE advantage)
 *
 * Readings: the mean runs over all T steps of the rollout; R_max includes this
 * rollout's returns before the mean is taken.
 * ------------------------------------------------------------------------- */
void orc_replay_scores(int T, int N, double gamma,
                       const float *rewards /* [T,N] */, const float *values /* [T+1,N] */,
                       const uint8_t *dones /* [T,N] */, const float *adv /* [T,N] */,
                       const float *rmax_in /* [N] or NULL: no return seen yet */,
                       double *rmax_out /* [N] */, double *maxmc /* [N] */, double *pvl /* [N] */)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        double G = (double)values[(size_t)T * N + n];
        int have = rmax_in != NULL;
        double best = have ? (double)rmax_in[n] : 0.0;
        double sum_v = 0.0, sum_pos = 0.0;
        for (int s = T - 1; s >= 0; --s) {
            size_t i = (size_t)s * N + n;
            G = (double)rewards[i] + gamma * (dones[i] ? 0.0 : 1.0) * G;
            if (!have || G > best) { best = G; have = 1; }
            sum_v += (double)values[i];
            double a = (double)adv[i];
            sum_pos += a > 0.0 ? a : 0.0;
        }
        rmax_out[n] = best;
        maxmc[n] = best - sum_v / T;
        pvl[n] = sum_pos / T;
    }
}
