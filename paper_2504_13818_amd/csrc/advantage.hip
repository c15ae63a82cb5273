// Advantages over the kept rollouts (Sec. 3.2): a = (r - mu_S) / (sigma_S + std_eps), with the
// mean and the population standard deviation of the m kept rewards of each prompt group; or, as
// the "Before" variant of App. "On Advantage Normalization", with the statistics of all n
// rewards of the group.  One wavefront per group; statistics are accumulated in double precision.
// Also here: the copy that concatenates the kept rollouts' records (Sec. 3.2).
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

// One word from src to dst, both streamed past the L2 (read once, written once: nothing here reads them again).
template <typename W>
__device__ __forceinline__ void copy_streaming(const W* s, W* d) {
    if constexpr (sizeof(W) == 16) {
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        __builtin_nontemporal_store(__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(s)),
                                    reinterpret_cast<u32x4*>(d));
    } else {
        __builtin_nontemporal_store(__builtin_nontemporal_load(s), d);
    }
}

// Kept rollouts' records, concatenated over the prompts (Sec. 3.2).  blockIdx.x = output row
// b*m + j, blockIdx.y = a slab of 1024 words of the row; W is the access word.
template <typename W>
__global__ __launch_bounds__(256) void gather_rows_kernel(const W* __restrict__ src,
                                                          const int32_t* __restrict__ sel_idx, int n, int m,
                                                          size_t row_words, W* __restrict__ dst) {
    const size_t out_row = blockIdx.x;
    const size_t b = out_row / (size_t)m;
    const size_t in_row = b * (size_t)n + (size_t)sel_idx[out_row];
    const W* s = src + in_row * row_words;
    W* d = dst + out_row * row_words;
    constexpr int kPerThread = 4;
    const size_t first = ((size_t)blockIdx.y * 256 * kPerThread) + threadIdx.x;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
        const size_t w = first + (size_t)i * 256;
        if (w < row_words) copy_streaming(s + w, d + w);
    }
}

// Optional argument check for the selection step: rewards that are NaN or infinite (for which the
// down-sampling rules define nothing) are counted, and the flat index of the first one is kept.
__global__ void check_rewards_init_kernel(int32_t* __restrict__ report) {
    report[0] = 0;
    report[1] = -1;
}
__global__ __launch_bounds__(256) void check_rewards_kernel(const float* __restrict__ rewards, int64_t count,
                                                            int32_t* __restrict__ report) {
    int bad = 0;
    uint32_t first = 0xFFFFFFFFu;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) {
        if ((__float_as_uint(rewards[i]) & 0x7F800000u) == 0x7F800000u) {
            ++bad;
            first = min(first, (uint32_t)i);
        }
    }
    if (bad != 0) {   // integer count and minimum: order-independent
        atomicAdd(&report[0], bad);
        atomicMin(reinterpret_cast<uint32_t*>(&report[1]), first);   // -1 reads as the largest unsigned
    }
}

template <typename W>
void launch_gather_width(const void* src, const int32_t* sel_idx, int32_t B, int32_t n, int32_t m,
                         size_t row_bytes, void* dst, hipStream_t stream) {
    const size_t row_words = row_bytes / sizeof(W);
    const unsigned slabs = (unsigned)ceil_div((int64_t)row_words, 256 * 4);
    PODS_LAUNCH("pods_gather_rows", stream, gather_rows_kernel<W>, dim3((unsigned)((int64_t)B * m), slabs), dim3(256),
                0, stream, static_cast<const W*>(src), sel_idx, n, m, row_words, static_cast<W*>(dst));
}

}  // namespace

pods_status launch_gather_rows(const void* src, const int32_t* sel_idx, int32_t B, int32_t n, int32_t m,
                               size_t row_bytes, void* dst, hipStream_t stream) {
    const uintptr_t bits = reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst) | row_bytes;
    if (ceil_div((int64_t)row_bytes, 1024) > 65535)   // slabs of at least 1 KiB ride on grid.y
        return fail(PODS_ERR_UNSUPPORTED, "pods_gather_rows: row_bytes = %zu exceeds 64 MiB", row_bytes);
    if ((bits & 15) == 0) launch_gather_width<uint4>(src, sel_idx, B, n, m, row_bytes, dst, stream);
    else if ((bits & 3) == 0) launch_gather_width<uint32_t>(src, sel_idx, B, n, m, row_bytes, dst, stream);
    else launch_gather_width<uint8_t>(src, sel_idx, B, n, m, row_bytes, dst, stream);
    return check_launch("pods_gather_rows");
}

pods_status launch_check_rewards(const float* rewards, int64_t count, int32_t* report, hipStream_t stream) {
    PODS_LAUNCH("pods_check_rewards (init)", stream, check_rewards_init_kernel, dim3(1), dim3(1), 0, stream, report);
    pods_status st = check_launch("pods_check_rewards (init)");
    if (st != PODS_OK) return st;
    const unsigned grid = (unsigned)(ceil_div(count, 256) < 2048 ? ceil_div(count, 256) : 2048);
    PODS_LAUNCH("pods_check_rewards", stream, check_rewards_kernel, dim3(grid), dim3(256), 0, stream, rewards, count,
                report);
    return check_launch("pods_check_rewards");
}

pods_status launch_advantage(const float* rewards, const int32_t* sel_idx, int32_t B, int32_t n,
                             int32_t m, float std_eps, bool stats_from_all, float* adv, hipStream_t stream) {
    const unsigned grid = (unsigned)ceil_div(B, kWavesPerBlock);
    PODS_LAUNCH("pods_advantage", stream, advantage_kernel, dim3(grid), dim3(kWavesPerBlock * kWave), 0, stream,
                rewards, sel_idx, B, n, m, std_eps, stats_from_all ? 1 : 0, adv);
    return check_launch("pods_advantage");
}

}  // namespace pods
