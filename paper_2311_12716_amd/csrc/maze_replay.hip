// Replay distribution of a level buffer: rank (or proportional) prioritisation of the
// levels' scores with a temperature, mixed with a staleness term.
//
// The buffer is small (K = 4000 in the paper's tables), so one workgroup does the whole
// job with the scores in LDS: a level's rank is one plus the number of levels that beat
// it (higher score, or equal score and lower index), found by counting -- K comparisons
// per level, spread over 1024 lanes -- and the two normalising sums are block
// reductions in a fixed order, so the result does not depend on timing.
#include "maze_internal.h"

namespace {

constexpr int RD_THREADS = 1024;
constexpr int RD_MAX_K = 12288;          // scores (4 B) + last-seen (4 B) in LDS, plus reduction space

__device__ __forceinline__ double block_sum(double v, double *red, int tid)
{
    // lanes of a wave first (fixed butterfly order), then the 16 waves by thread 0
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    __syncthreads();
    if ((tid & 63) == 0) red[tid >> 6] = v;
    __syncthreads();
    double tot = 0.0;
    for (int w = 0; w < RD_THREADS / 64; ++w) tot += red[w];
    return tot;
}

__global__ __launch_bounds__(RD_THREADS) void k_replay_distribution(
    const float *__restrict__ scores, const int32_t *__restrict__ last_seen, int K, int now,
    int use_rank, double inv_temperature, double rho, float *__restrict__ prob)
{
    extern __shared__ uint32_t lds[];
    float *s = (float *)lds;                                 // [K]
    double *red = (double *)(lds + ((K + 1) & ~1));          // [16], 8-byte aligned
    const int tid = threadIdx.x;
    for (int i = tid; i < K; i += RD_THREADS) s[i] = scores[i];
    __syncthreads();
    constexpr int PER = (RD_MAX_K + RD_THREADS - 1) / RD_THREADS;
    double w[PER], stale[PER];
    double wsum = 0.0, ssum = 0.0;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const int i = tid + q * RD_THREADS;
        w[q] = 0.0;
        stale[q] = 0.0;
        if (i < K) {
            const float si = s[i];
            double h;
            if (use_rank) {
                int better = 0;
                for (int j = 0; j < K; ++j) {
                    const float sj = s[j];
                    better += (sj > si || (sj == si && j < i)) ? 1 : 0;
                }
                h = 1.0 / (double)(better + 1);
            } else {
                h = si > 0.0f ? (double)si : 0.0;
            }
            w[q] = pow(h, inv_temperature);
            stale[q] = (double)((long long)now - (long long)last_seen[i]);
            wsum += w[q];
            ssum += stale[q];
        }
    }
    const double wtot = block_sum(wsum, red, tid);
    const double stot = block_sum(ssum, red, tid);
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const int i = tid + q * RD_THREADS;
        if (i < K) {
            const double ps = wtot > 0.0 ? w[q] / wtot : 1.0 / (double)K;
            const double p = stot > 0.0 ? (1.0 - rho) * ps + rho * (stale[q] / stot) : ps;
            prob[i] = (float)p;
        }
    }
}

}  // namespace

extern "C" int replay_distribution(const float *d_scores, const int32_t *d_last_seen, int K, int now,
                                   int rank_prioritization, double temperature, double staleness_coef,
                                   float *d_prob, void *stream)
{
    if (!d_scores || !d_last_seen || !d_prob) return MAZE_ENULL;
    if (K < 1 || !(temperature > 0.0) || !(staleness_coef >= 0.0 && staleness_coef <= 1.0))
        return MAZE_EINVAL;
    if (K > RD_MAX_K) return MAZE_ESIZE;
    const size_t shmem = 4 * (size_t)((K + 1) & ~1) + 8 * (RD_THREADS / 64);
    hipLaunchKernelGGL(k_replay_distribution, dim3(1), dim3(RD_THREADS), shmem, (hipStream_t)stream,
                       d_scores, d_last_seen, K, now, rank_prioritization ? 1 : 0, 1.0 / temperature,
                       staleness_coef, d_prob);
    MAZE_HIP_CHECK(hipGetLastError());
    return MAZE_OK;
}
