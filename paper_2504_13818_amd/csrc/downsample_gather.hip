// Steps 3 and 4 of Algorithm 1 in one launch: down-sample each prompt group by the chosen rule
// (Sec. 3.2, Sec. 3.3), normalise the kept rewards into advantages (Sec. 3.2, or the "Before"
// variant of App. "On Advantage Normalization"), and copy the kept rollouts' records into the
// concatenated layout the policy update reads.
//
// One workgroup per group.  The group's (key, index) pairs are sorted in LDS by a bitonic network,
// the two prefix-sum tables of Theorem 1 are built by a block scan, every split k of Algorithm 2 is
// scored by one thread, and then all threads copy the m kept rows of every record.  The selection
// arithmetic (double-precision m*sum(x^2) - (sum x)^2, a split whose multiset equals the previous
// split's is never preferred, smallest maximising k) is the batched selector's; only the way the
// work is spread over lanes differs, because here the copy, not the sort, decides the launch shape.
#include "common.h"

#include <climits>

namespace pods {
namespace {

constexpr int kThreads = 256;

struct DeviceRecord {
    const void* src;
    void* dst;
    uint32_t row_words;   // row_bytes / word_bytes
    uint32_t word_bytes;  // 16, 4 or 1: the widest access src, dst and row_bytes allow
};
struct DeviceRecords {
    DeviceRecord r[PODS_MAX_RECORDS];
    int count;
};

// 64-bit sort key: the reward mapped to an unsigned integer of the same order (-0.0 first made
// +0.0) in the high word, the rollout's index in the low word.
__device__ __forceinline__ uint64_t reward_key(float r, uint32_t e) {
    r = r + 0.0f;
    const uint32_t b = __float_as_uint(r);
    const uint32_t ordered = b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
    return ((uint64_t)ordered << 32) | e;
}
__device__ __forceinline__ float key_reward(uint64_t key) {
    const uint32_t ordered = (uint32_t)(key >> 32);
    return __uint_as_float(ordered ^ ((ordered >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}
__device__ __forceinline__ int32_t key_index(uint64_t key) { return (int32_t)(uint32_t)key; }

__device__ __forceinline__ double block_sum(double x, double* scratch) {
    const int tid = threadIdx.x;
    __syncthreads();
    scratch[tid] = x;
    __syncthreads();
    for (int off = kThreads / 2; off >= 1; off >>= 1) {
        if (tid < off) scratch[tid] += scratch[tid + off];
        __syncthreads();
    }
    return scratch[0];
}

// out1[j] = sum of value(0 .. j-1), out2[j] the same of the squares, j = 0 .. len.
template <class F>
__device__ __forceinline__ void prefix_tables(F value, int len, double* out1, double* out2, double* s1,
                                              double* s2) {
    const int tid = threadIdx.x;
    const int per = (len + kThreads - 1) / kThreads;
    const int j0 = min(tid * per, len), j1 = min(j0 + per, len);
    double b1 = 0.0, b2 = 0.0;
    for (int j = j0; j < j1; ++j) {
        const double x = value(j);
        b1 += x;
        b2 += x * x;
    }
    __syncthreads();
    s1[tid] = b1;
    s2[tid] = b2;
    __syncthreads();
    for (int off = 1; off < kThreads; off <<= 1) {
        const double a1 = tid >= off ? s1[tid - off] : 0.0;
        const double a2 = tid >= off ? s2[tid - off] : 0.0;
        __syncthreads();
        s1[tid] += a1;
        s2[tid] += a2;
        __syncthreads();
    }
    double r1 = tid > 0 ? s1[tid - 1] : 0.0;
    double r2 = tid > 0 ? s2[tid - 1] : 0.0;
    if (tid == 0) {
        out1[0] = 0.0;
        out2[0] = 0.0;
    }
    for (int j = j0; j < j1; ++j) {
        const double x = value(j);
        r1 += x;
        r2 += x * x;
        out1[j + 1] = r1;
        out2[j + 1] = r2;
    }
    __syncthreads();
}

// dst rows (b*m + j) <- src rows (b*n + sel[j]), j < m; four words in flight per thread.
template <class W, class I>
__device__ __forceinline__ void copy_rows(const W* __restrict__ src, W* __restrict__ dst, size_t b, int n, int m,
                                          uint32_t row_words, const int32_t* sel) {
    const I total = (I)m * (I)row_words;
    const W* s = src + b * (size_t)n * row_words;
    W* d = dst + b * (size_t)m * row_words;
    constexpr int kInFlight = 4;
    for (I f = threadIdx.x; f < total; f += (I)kThreads * kInFlight) {
        W v[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            const I i = f + (I)u * kThreads;
            if (i < total) {
                const I row = i / (I)row_words;
                const I w = i - row * (I)row_words;
                v[u] = s[(size_t)sel[row] * row_words + w];
            }
        }
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            const I i = f + (I)u * kThreads;
            if (i < total) d[i] = v[u];
        }
    }
}

template <class W>
__device__ __forceinline__ void copy_record(const DeviceRecord& rec, size_t b, int n, int m, const int32_t* sel) {
    const W* src = static_cast<const W*>(rec.src);
    W* dst = static_cast<W*>(rec.dst);
    if ((uint64_t)m * rec.row_words <= 0xFFFFFFFFull) copy_rows<W, uint32_t>(src, dst, b, n, m, rec.row_words, sel);
    else copy_rows<W, uint64_t>(src, dst, b, n, m, rec.row_words, sel);
}

__global__ __launch_bounds__(kThreads) void downsample_gather_kernel(
    const float* __restrict__ rewards, const uint32_t* __restrict__ rand_keys, int n, int n2, int m, int rule,
    float std_eps, int stats_from_all, DeviceRecords recs, int32_t* __restrict__ sel_idx,
    int32_t* __restrict__ sel_k, float* __restrict__ adv) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    uint64_t* key = reinterpret_cast<uint64_t*>(lds_raw);   // [n2] sorted (key, index)
    double* lo1 = reinterpret_cast<double*>(key + n2);      // [m+1] sum of the j lowest rewards
    double* lo2 = lo1 + (m + 1);                            // ... of their squares
    double* hi1 = lo2 + (m + 1);                            // [m+1] sum of the k highest rewards
    double* hi2 = hi1 + (m + 1);
    int32_t* sel = reinterpret_cast<int32_t*>(hi2 + (m + 1));   // [m] kept indices, output order
    __shared__ double s1[kThreads], s2[kThreads];
    __shared__ int sk[kThreads];

    const int tid = threadIdx.x;
    const size_t b = blockIdx.x;
    const float* r = rewards + b * (size_t)n;

    // ---- order the group by (key, index) ----
    for (int e = tid; e < n2; e += kThreads) {
        uint64_t k = ~0ull;   // padding sorts behind every rollout
        if (e < n)
            k = rule == PODS_RULE_RAND ? (((uint64_t)rand_keys[b * (size_t)n + e] << 32) | (uint32_t)e)
                                       : reward_key(r[e], (uint32_t)e);
        key[e] = k;
    }
    for (int k = 2; k <= n2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            __syncthreads();
            for (int i = tid; i < n2 / 2; i += kThreads) {
                const int lo = ((i & ~(j - 1)) << 1) | (i & (j - 1));
                const int hi = lo | j;
                const bool ascending = (lo & k) == 0;
                const uint64_t a = key[lo], c = key[hi];
                if ((a > c) == ascending) {
                    key[lo] = c;
                    key[hi] = a;
                }
            }
        }
    }
    __syncthreads();

    // ---- the rule's positions in that order ----
    int best_k = -1;
    if (rule == PODS_RULE_MAXVAR) {
        prefix_tables([&](int j) { return (double)key_reward(key[j]); }, m, lo1, lo2, s1, s2);
        prefix_tables([&](int j) { return (double)key_reward(key[n - 1 - j]); }, m, hi1, hi2, s1, s2);
        // score every split k (the m-k lowest with the k highest); first strict maximum wins
        const double dm = (double)m;
        double best = -__builtin_huge_val();
        int mine = INT_MAX;
        for (int k = tid; k <= m; k += kThreads) {
            if (k > 0 && key_reward(key[n - k]) == key_reward(key[m - k])) continue;  // same multiset as split k-1
            const double S = lo1[m - k] + hi1[k];
            const double Q = lo2[m - k] + hi2[k];
            const double D = dm * Q - S * S;
            if (D > best) {
                best = D;
                mine = k;
            }
        }
        s1[tid] = best;
        sk[tid] = mine;
        __syncthreads();
        for (int off = kThreads / 2; off >= 1; off >>= 1) {
            if (tid < off) {
                const double od = s1[tid + off];
                const int ok = sk[tid + off];
                if (od > s1[tid] || (od == s1[tid] && ok < sk[tid])) {
                    s1[tid] = od;
                    sk[tid] = ok;
                }
            }
            __syncthreads();
        }
        best_k = sk[0];
    } else if (rule == PODS_RULE_MAXR) {
        best_k = m;
    }
    for (int j = tid; j < m; j += kThreads) {
        int pos;
        if (rule == PODS_RULE_MAXVAR) pos = j < m - best_k ? j : n - m + j;
        else if (rule == PODS_RULE_MAXR) pos = n - m + j;
        else if (rule == PODS_RULE_PERC) pos = (int)(((int64_t)(2 * j + 1) * n) / (2 * (int64_t)m));
        else pos = j;
        const int32_t idx = key_index(key[pos]);
        sel[j] = idx;
        sel_idx[b * (size_t)m + j] = idx;
    }
    if (sel_k != nullptr && tid == 0) sel_k[b] = best_k;
    __syncthreads();

    // ---- advantages: statistics over the kept rewards, or over all n ----
    {
        const int cnt = stats_from_all ? n : m;
        auto sample = [&](int j) { return stats_from_all ? r[j] : r[sel[j]]; };
        double sum = 0.0;
        float lo = __builtin_huge_valf(), hi = -__builtin_huge_valf();
        for (int j = tid; j < cnt; j += kThreads) {
            const float x = sample(j);
            sum += (double)x;
            lo = fminf(lo, x);
            hi = fmaxf(hi, x);
        }
        sum = block_sum(sum, s1);
        // range of the population, through the same scratch
        __syncthreads();
        s1[tid] = (double)lo;
        s2[tid] = (double)hi;
        __syncthreads();
        for (int off = kThreads / 2; off >= 1; off >>= 1) {
            if (tid < off) {
                s1[tid] = fmin(s1[tid], s1[tid + off]);
                s2[tid] = fmax(s2[tid], s2[tid + off]);
            }
            __syncthreads();
        }
        const bool flat = s1[0] == s2[0];   // sigma = 0: decided by comparison, never by a tolerance
        float* a = adv + b * (size_t)m;
        if (flat) {
            for (int j = tid; j < m; j += kThreads) a[j] = 0.0f;
        } else {
            const double mu = sum / (double)cnt;
            double ss = 0.0;
            for (int j = tid; j < cnt; j += kThreads) {
                const double x = (double)sample(j) - mu;
                ss += x * x;
            }
            ss = block_sum(ss, s1);
            const double inv = 1.0 / (sqrt(ss / (double)cnt) + (double)std_eps);
            for (int j = tid; j < m; j += kThreads) a[j] = (float)(((double)r[sel[j]] - mu) * inv);
        }
    }

    // ---- the kept rollouts' records ----
    for (int q = 0; q < recs.count; ++q) {
        const DeviceRecord& rec = recs.r[q];
        if (rec.word_bytes == 16) copy_record<uint4>(rec, b, n, m, sel);
        else if (rec.word_bytes == 4) copy_record<uint32_t>(rec, b, n, m, sel);
        else copy_record<uint8_t>(rec, b, n, m, sel);
    }
}

}  // namespace

pods_status launch_downsample_gather(const float* rewards, const uint32_t* rand_keys, int32_t B, int32_t n, int32_t m,
                                     int32_t rule, float std_eps, bool stats_from_all, const pods_record* records,
                                     int32_t num_records, int32_t* sel_idx, int32_t* sel_k, float* adv,
                                     hipStream_t stream) {
    DeviceRecords recs{};
    recs.count = num_records;
    for (int q = 0; q < num_records; ++q) {
        const pods_record& in = records[q];
        const uintptr_t bits =
            reinterpret_cast<uintptr_t>(in.src) | reinterpret_cast<uintptr_t>(in.dst) | (uintptr_t)in.row_bytes;
        const uint32_t word = (bits & 15) == 0 ? 16u : (bits & 3) == 0 ? 4u : 1u;
        if (in.row_bytes / word > 0xFFFFFFFFull)
            return fail(PODS_ERR_UNSUPPORTED, "pods_downsample_gather: record %d: row_bytes = %zu is too large", q,
                        in.row_bytes);
        recs.r[q] = DeviceRecord{in.src, in.dst, (uint32_t)(in.row_bytes / word), word};
    }
    int n2 = 1;
    while (n2 < n) n2 <<= 1;
    const size_t lds = (size_t)n2 * sizeof(uint64_t) + 4 * (size_t)(m + 1) * sizeof(double) + (size_t)m * sizeof(int32_t);
    PODS_LAUNCH("pods_downsample_gather", stream, downsample_gather_kernel, dim3((unsigned)B), dim3(kThreads), lds,
                stream, rewards, rand_keys, n, n2, m, rule, std_eps, stats_from_all ? 1 : 0, recs, sel_idx, sel_k,
                adv);
    return check_launch("pods_downsample_gather");
}

}  // namespace pods
