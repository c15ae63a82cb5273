// Advantages over the kept rollouts (Sec. 3.2): a = (r - mu_S) / (sigma_S + std_eps), with the
// mean and the population standard deviation of the m kept rewards of each prompt group; or, as
// the "Before" variant of App. "On Advantage Normalization", with the statistics of all n
// rewards of the group.  One wavefront per group; statistics are accumulated in double precision.
#include "common.h"

namespace pods {
namespace {

__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
    for (int off = kWave / 2; off >= 1; off >>= 1) x += __shfl_xor(x, off, kWave);
    return x;
}

constexpr int kWavesPerBlock = 4;

__global__ __launch_bounds__(kWavesPerBlock* kWave) void advantage_kernel(
    const float* __restrict__ rewards, const int32_t* __restrict__ sel_idx, int B, int n, int m,
    float std_eps, int stats_from_all, float* __restrict__ adv) {
    const int lane = threadIdx.x & (kWave - 1);
    const int group = blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
    if (group >= B) return;
    const float* r = rewards + (size_t)group * n;
    const int32_t* s = sel_idx + (size_t)group * m;
    float* a = adv + (size_t)group * m;

    // the population the statistics are taken over: the m kept rewards, or all n
    const int cnt = stats_from_all ? n : m;
    auto sample = [&](int j) { return stats_from_all ? r[j] : r[s[j]]; };

    double sum = 0.0;
    float lo = __builtin_huge_valf(), hi = -__builtin_huge_valf();
    for (int j = lane; j < cnt; j += kWave) {
        const float x = sample(j);
        sum += (double)x;
        lo = fminf(lo, x);
        hi = fmaxf(hi, x);
    }
    sum = wave_sum(sum);
#pragma unroll
    for (int off = kWave / 2; off >= 1; off >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, off, kWave));
        hi = fmaxf(hi, __shfl_xor(hi, off, kWave));
    }
    if (lo == hi) {  // sigma_S = 0: decided by comparison, never by a tolerance
        for (int j = lane; j < m; j += kWave) a[j] = 0.0f;
        return;
    }
    const double mu = sum / (double)cnt;
    double ss = 0.0;
    for (int j = lane; j < cnt; j += kWave) {
        const double x = (double)sample(j) - mu;
        ss += x * x;
    }
    ss = wave_sum(ss);
    const double sigma = sqrt(ss / (double)cnt);
    const double inv = 1.0 / (sigma + (double)std_eps);
    for (int j = lane; j < m; j += kWave) a[j] = (float)(((double)r[s[j]] - mu) * inv);
}

}  // namespace

pods_status launch_advantage(const float* rewards, const int32_t* sel_idx, int32_t B, int32_t n,
                             int32_t m, float std_eps, bool stats_from_all, float* adv, hipStream_t stream) {
    const unsigned grid = (unsigned)ceil_div(B, kWavesPerBlock);
    PODS_LAUNCH("pods_advantage", stream, advantage_kernel, dim3(grid), dim3(kWavesPerBlock * kWave), 0, stream,
                rewards, sel_idx, B, n, m, std_eps, stats_from_all ? 1 : 0, adv);
    return check_launch("pods_advantage");
}

}  // namespace pods
