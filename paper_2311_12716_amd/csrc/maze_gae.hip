// Generalised advantage estimation: reverse scan over time, parallel over envs and
// over segments of the time axis.
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

}  // namespace

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
