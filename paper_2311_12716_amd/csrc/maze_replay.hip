// Replay distribution of a level buffer: rank (or proportional) prioritisation of the
// levels' scores with a temperature, mixed with a staleness term.
//
// The buffer is small (K = 4000 in the paper's tables), so one workgroup does the whole
// job in LDS.  Ranks come from a bitonic sort of 64-bit keys (score, descending, in the
// high word; level index in the low word), so equal scores are ordered by index and the
// result does not depend on timing: the level whose key ends up at position p has rank
// p + 1.  The two normalising sums are block reductions in a fixed order.
#include "maze_internal.h"

namespace {

constexpr int RD_THREADS = 1024;
constexpr int RD_MAX_K = 16384;          // 8-byte keys of the padded buffer: 128 KB of LDS

__device__ __forceinline__ double block_sum(double v, double *red, int tid)
{
    // lanes of a wave first (fixed butterfly order), then the 16 waves in order
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    __syncthreads();
    if ((tid & 63) == 0) red[tid >> 6] = v;
    __syncthreads();
    double tot = 0.0;
    for (int w = 0; w < RD_THREADS / 64; ++w) tot += red[w];
    return tot;
}

// Key that sorts ascending exactly when the score sorts descending (index ascending among
// equal scores).  -0 counts as +0.
__device__ __forceinline__ uint64_t rank_key(float score, int index)
{
    uint32_t u = __float_as_uint(score + 0.0f);
    u ^= (u >> 31) ? 0xFFFFFFFFu : 0x80000000u;          // unsigned order = float order
    return ((uint64_t)(~u) << 32) | (uint32_t)index;
}

__global__ __launch_bounds__(RD_THREADS) void k_replay_distribution(
    const float *__restrict__ scores, const int32_t *__restrict__ last_seen, int K, int n2, int now,
    int use_rank, double inv_temperature, double rho, float *__restrict__ prob)
{
    extern __shared__ uint64_t keys[];                       // [n2] (rank mode)
    __shared__ double red[RD_THREADS / 64];
    const int tid = threadIdx.x;
    if (use_rank) {
        for (int i = tid; i < n2; i += RD_THREADS) keys[i] = i < K ? rank_key(scores[i], i) : ~0ull;
        __syncthreads();
        for (int k = 2; k <= n2; k <<= 1) {
            for (int j = k >> 1; j > 0; j >>= 1) {
                for (int t = tid; t < n2 / 2; t += RD_THREADS) {
                    const int lo = ((t & ~(j - 1)) << 1) | (t & (j - 1)), hi = lo | j;
                    const uint64_t a = keys[lo], b = keys[hi];
                    const bool ascending = (lo & k) == 0;
                    if ((a > b) == ascending) { keys[lo] = b; keys[hi] = a; }
                }
                __syncthreads();
            }
        }
    }
    // weights: by position in rank mode (position p holds the level of rank p + 1), by level
    // otherwise; staleness by level
    double wsum = 0.0, ssum = 0.0;
    for (int i = tid; i < K; i += RD_THREADS) {
        double h;
        if (use_rank) {
            h = 1.0 / (double)(i + 1);
        } else {
            const float si = scores[i];
            h = si > 0.0f ? (double)si : 0.0;
        }
        wsum += pow(h, inv_temperature);
        ssum += (double)((long long)now - (long long)last_seen[i]);
    }
    const double wtot = block_sum(wsum, red, tid);
    const double stot = block_sum(ssum, red, tid);
    for (int p = tid; p < K; p += RD_THREADS) {
        const int i = use_rank ? (int)(uint32_t)keys[p] : p;
        double h;
        if (use_rank) {
            h = 1.0 / (double)(p + 1);
        } else {
            const float si = scores[i];
            h = si > 0.0f ? (double)si : 0.0;
        }
        const double ps = wtot > 0.0 ? pow(h, inv_temperature) / wtot : 1.0 / (double)K;
        const double stale = (double)((long long)now - (long long)last_seen[i]);
        prob[i] = (float)(stot > 0.0 ? (1.0 - rho) * ps + rho * (stale / stot) : ps);
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
    int n2 = 2;
    while (n2 < K) n2 <<= 1;
    const size_t shmem = rank_prioritization ? 8 * (size_t)n2 : 0;
    // dynamic LDS above 64 KB needs an opt-in, once per device
    static size_t granted[16] = {};
    int device = 0;
    MAZE_HIP_CHECK(hipGetDevice(&device));
    if (shmem > 60 * 1024 && shmem > granted[device & 15]) {
        MAZE_HIP_CHECK(hipFuncSetAttribute((const void *)k_replay_distribution,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem));
        granted[device & 15] = shmem;
    }
    hipLaunchKernelGGL(k_replay_distribution, dim3(1), dim3(RD_THREADS), shmem, (hipStream_t)stream,
                       d_scores, d_last_seen, K, n2, now, rank_prioritization ? 1 : 0, 1.0 / temperature,
                       staleness_coef, d_prob);
    MAZE_HIP_CHECK(hipGetLastError());
    return MAZE_OK;
}
