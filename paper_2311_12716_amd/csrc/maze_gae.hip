// Generalised advantage estimation: one lane per env, reverse scan over time.
#include "maze_internal.h"

// The recurrence A_t = delta_t + gamma*lambda*(1-d_t)*A_{t+1} is carried in double
// (inputs are widened exactly, the result is rounded to float once per element),
// so the float output does not depend on how the scan is scheduled.
__global__ void k_gae_scan(const float *__restrict__ rewards, const float *__restrict__ values,
                           const uint8_t *__restrict__ dones, int T, int N, double gamma,
                           double gl, float *__restrict__ adv, float *__restrict__ ret)
{
    int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    double A = 0.0;
    double vnext = (double)values[(size_t)T * N + n];
    for (int s = T - 1; s >= 0; --s) {
        size_t i = (size_t)s * N + n;
        double v = (double)values[i];
        double nd = dones[i] ? 0.0 : 1.0;
        double delta = (double)rewards[i] + gamma * vnext * nd - v;
        A = delta + gl * nd * A;
        adv[i] = (float)A;
        if (ret) ret[i] = (float)(A + v);
        vnext = v;
    }
}

extern "C" int compute_gae(const float *d_rewards, const float *d_values, const uint8_t *d_dones,
                           int T, int N, double gamma, double lambda, float *d_adv,
                           float *d_returns, void *stream)
{
    if (!d_rewards || !d_values || !d_dones || !d_adv) return MAZE_ENULL;
    if (T < 1 || N < 1) return MAZE_EINVAL;
    hipLaunchKernelGGL(k_gae_scan, dim3((N + 63) / 64), dim3(64), 0, (hipStream_t)stream,
                       d_rewards, d_values, d_dones, T, N, gamma, gamma * lambda, d_adv,
                       d_returns);
    MAZE_HIP_CHECK(hipGetLastError());
    return MAZE_OK;
}
