// Generalised advantage estimation and the replay scores of a rollout: reverse scans
// over time, parallel over envs and over segments of the time axis.
#include "maze_internal.h"

namespace {

constexpr int SEG = 16;         // time steps per segment (held in registers)
constexpr int MAX_SEGS = 16;    // segments (= waves) per workgroup

// A_t = delta_t + c_t * A_{t+1},  c_t = gamma*lambda*(1-d_t),  A_T = 0.
//
// A workgroup takes 64 envs; wave j takes one segment of SEG consecutive steps of a
// "super-block" of S*SEG steps.  Each wave scans its segment backwards as if nothing
// followed it (A = 0 after its last step) and records, per step, that local A_t and
// the product P_t of the c's from t to the segment's end.  The true value is
// A_t = local A_t + P_t * (true A just after the segment), and those carry-ins follow
// from the segments' first (A, P) pairs by a short serial combine through LDS.  All
// loads of a segment are independent of the recurrence, so they are in flight
// together; inputs are read once, outputs written once.
//
// Arithmetic is in double (inputs widened exactly, outputs rounded to float once);
// an episode end (d_t = 1) makes P_t = 0, so nothing leaks across it.
__global__ __launch_bounds__(64 * MAX_SEGS) void k_gae_scan(
    const float *__restrict__ rewards, const float *__restrict__ values,
    const uint8_t *__restrict__ dones, int T, int N, int S, double gamma, double gl,
    float *__restrict__ adv, float *__restrict__ ret)
{
    __shared__ double sA[MAX_SEGS][64], sP[MAX_SEGS][64], sCarry[64];
    const int lane = threadIdx.x & 63;
    const int j = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_raw = blockIdx.x * 64 + lane;
    const bool live = n_raw < N;
    const size_t n = live ? n_raw : N - 1;       // idle lanes read a valid column, store nothing
    if (j == 0) sCarry[lane] = 0.0;
    for (int sb_end = T; sb_end > 0; sb_end -= S * SEG) {
        // wave j's segment: steps [seg_end - SEG, seg_end), clipped at 0; wave S-1 is the latest
        const int seg_end = sb_end - (S - 1 - j) * SEG;
        double a[SEG], pp[SEG];
        float v[SEG];
        double A = 0.0, P = 1.0;
        if (seg_end > 0) {
            double vnext = (double)values[(size_t)seg_end * N + n];
#pragma unroll
            for (int u = 0; u < SEG; ++u) {
                const int t = seg_end - 1 - u;
                if (t >= 0) {
                    const size_t i = (size_t)t * N + n;
                    const float vf = values[i];
                    const double nd = dones[i] ? 0.0 : 1.0;
                    const double delta = (double)rewards[i] + gamma * vnext * nd - (double)vf;
                    const double c = gl * nd;
                    A = delta + c * A;
                    P = c * P;
                    vnext = (double)vf;
                    v[u] = vf;
                }
                a[u] = A;
                pp[u] = P;
            }
        }
        sA[j][lane] = A;
        sP[j][lane] = P;
        __syncthreads();
        // true advantage just after this wave's segment
        double carry = sCarry[lane];
        for (int jj = S - 1; jj > j; --jj) carry = sA[jj][lane] + sP[jj][lane] * carry;
        if (seg_end > 0 && live) {
#pragma unroll
            for (int u = 0; u < SEG; ++u) {
                const int t = seg_end - 1 - u;
                if (t >= 0) {
                    const size_t i = (size_t)t * N + n;
                    const double At = a[u] + pp[u] * carry;
                    adv[i] = (float)At;
                    if (ret) ret[i] = (float)(At + (double)v[u]);
                }
            }
        }
        __syncthreads();
        // true advantage at the super-block's first step; read again only after the next
        // iteration's first barrier
        if (j == 0) sCarry[lane] = A + P * carry;
    }
}

// Replay scores of a rollout, per env:  G_t = r_t + gamma (1-d_t) G_{t+1} with G_T = V_T,
// best = max_t G_t (and the best return seen before, if given), MaxMC = best - mean_t V_t,
// PVL = mean_t max(A_t, 0).  Same decomposition of the time axis as the advantage scan:
// every wave scans one segment as if G were 0 after it and keeps, per step, that local
// return and the product of the discount factors up to the segment's end; the true
// return is local + product * (true return just after the segment).
__global__ __launch_bounds__(64 * MAX_SEGS) void k_replay_scores(
    const float *__restrict__ rewards, const float *__restrict__ values,
    const uint8_t *__restrict__ dones, const float *__restrict__ adv, int T, int N, int S,
    double gamma, const float *rmax_in, float *rmax_out, float *__restrict__ maxmc,
    float *__restrict__ pvl)
{
    __shared__ double sA[MAX_SEGS][64], sP[MAX_SEGS][64], sCarry[64];
    const int lane = threadIdx.x & 63;
    const int j = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_raw = blockIdx.x * 64 + lane;
    const bool live = n_raw < N;
    const size_t n = live ? n_raw : N - 1;
    if (j == 0) sCarry[lane] = (double)values[(size_t)T * N + n];      // G_T = V_T
    double best = -INFINITY, sum_v = 0.0, sum_pos = 0.0;
    for (int sb_end = T; sb_end > 0; sb_end -= S * SEG) {
        const int seg_end = sb_end - (S - 1 - j) * SEG;
        double a[SEG], pp[SEG];
        double A = 0.0, P = 1.0;
        if (seg_end > 0) {
#pragma unroll
            for (int u = 0; u < SEG; ++u) {
                const int t = seg_end - 1 - u;
                if (t >= 0) {
                    const size_t i = (size_t)t * N + n;
                    const double c = dones[i] ? 0.0 : gamma;
                    A = (double)rewards[i] + c * A;
                    P = c * P;
                    sum_v += (double)values[i];
                    const double ad = (double)adv[i];
                    sum_pos += ad > 0.0 ? ad : 0.0;
                }
                a[u] = A;
                pp[u] = P;
            }
        }
        sA[j][lane] = A;
        sP[j][lane] = P;
        __syncthreads();
        double carry = sCarry[lane];
        for (int jj = S - 1; jj > j; --jj) carry = sA[jj][lane] + sP[jj][lane] * carry;
        if (seg_end > 0) {
#pragma unroll
            for (int u = 0; u < SEG; ++u)
                if (seg_end - 1 - u >= 0) best = fmax(best, a[u] + pp[u] * carry);
        }
        __syncthreads();
        if (j == 0) sCarry[lane] = A + P * carry;
    }
    // combine the waves' partial results (sA, sP are free again; sCarry is read by nobody)
    __shared__ double sV[MAX_SEGS][64];
    sA[j][lane] = best;
    sP[j][lane] = sum_pos;
    sV[j][lane] = sum_v;
    __syncthreads();
    if (j == 0 && live) {
        for (int jj = 1; jj < S; ++jj) {
            best = fmax(best, sA[jj][lane]);
            sum_pos += sP[jj][lane];
            sum_v += sV[jj][lane];
        }
        if (rmax_in) best = fmax(best, (double)rmax_in[n]);
        if (rmax_out) rmax_out[n] = (float)best;
        if (maxmc) maxmc[n] = (float)(best - sum_v / T);
        if (pvl) pvl[n] = (float)(sum_pos / T);
    }
}

}  // namespace

extern "C" int replay_scores(const float *d_rewards, const float *d_values, const uint8_t *d_dones,
                             const float *d_adv, int T, int N, double gamma, const float *d_rmax_in,
                             float *d_rmax_out, float *d_maxmc, float *d_pvl, void *stream)
{
    if (!d_rewards || !d_values || !d_dones || !d_adv) return MAZE_ENULL;
    if (T < 1 || N < 1) return MAZE_EINVAL;
    int S = (T + SEG - 1) / SEG;
    if (S > MAX_SEGS) S = MAX_SEGS;
    hipLaunchKernelGGL(k_replay_scores, dim3((N + 63) / 64), dim3(64 * S), 0, (hipStream_t)stream,
                       d_rewards, d_values, d_dones, d_adv, T, N, S, gamma, d_rmax_in, d_rmax_out,
                       d_maxmc, d_pvl);
    MAZE_HIP_CHECK(hipGetLastError());
    return MAZE_OK;
}

extern "C" int compute_gae(const float *d_rewards, const float *d_values, const uint8_t *d_dones,
                           int T, int N, double gamma, double lambda, float *d_adv,
                           float *d_returns, void *stream)
{
    if (!d_rewards || !d_values || !d_dones || !d_adv) return MAZE_ENULL;
    if (T < 1 || N < 1) return MAZE_EINVAL;
    int S = (T + SEG - 1) / SEG;
    if (S > MAX_SEGS) S = MAX_SEGS;
    hipLaunchKernelGGL(k_gae_scan, dim3((N + 63) / 64), dim3(64 * S), 0, (hipStream_t)stream,
                       d_rewards, d_values, d_dones, T, N, S, gamma, gamma * lambda, d_adv,
                       d_returns);
    MAZE_HIP_CHECK(hipGetLastError());
    return MAZE_OK;
}
