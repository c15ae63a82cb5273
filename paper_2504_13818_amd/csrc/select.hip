// Down-sampling rules, one prompt group per wavefront: max-variance (Sec. 3.3: Lemma 3.1,
// Algorithm 2, Theorem 1) and, on the same sorted order, max-reward, percentile and random
// (Sec. 3.2).
//
// Each lane holds KPL consecutive elements of the group as 64-bit sort keys.  A key is the
// order-preserving integer image of the float32 reward followed by the element's index, laid
// into the mantissa of a double in [2, 4): for such doubles floating-point order equals integer
// order, so an in-lane compare-exchange is one v_min_f64 and one v_max_f64 and a cross-lane one is
// one v_cmp_lt_f64 and two selects.  The index in the low bits makes every key distinct and gives
// the (reward, index) order the tie rule asks for.  Partner values travel by DPP moves where the
// lane pattern allows, else through the LDS crossbar (ds_swizzle / ds_bpermute).
// A bitonic network sorts the 64*KPL keys in registers; the sorted rewards and indices are staged
// in LDS; prefix sums of r and r^2 over the m lowest and running sums over the k highest are
// scanned in double precision (DPP row shifts and row broadcasts, no LDS traffic); one candidate
// split k per lane is scored as m*Q - S^2 (m^2 times its variance), candidates that repeat the
// previous multiset are passed over, and the wave's maximum plus the first lane that attains it
// (smallest k on equal scores) picks k.
#include "common.h"

namespace pods {
namespace {

constexpr int kIdxBits = 12;  // n <= 4096

__device__ __forceinline__ double make_key(float r, uint32_t e) {
    r = r + 0.0f;  // -0.0 -> +0.0
    uint32_t b = __float_as_uint(r);
    uint32_t ou = b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);  // unsigned order == float order
    uint64_t k = (1ull << 62) | ((uint64_t)ou << kIdxBits) | e;
    return __longlong_as_double((long long)k);
}
__device__ __forceinline__ double make_key_u32(uint32_t ou, uint32_t e) {
    uint64_t k = (1ull << 62) | ((uint64_t)ou << kIdxBits) | e;
    return __longlong_as_double((long long)k);
}
__device__ __forceinline__ double pad_key(uint32_t e) {
    uint64_t k = (1ull << 62) | ((uint64_t)0xFFFFFFFFu << kIdxBits) | e;  // after every real reward
    return __longlong_as_double((long long)k);
}
__device__ __forceinline__ float key_reward(double key) {
    uint64_t k = (uint64_t)__double_as_longlong(key);
    uint32_t ou = (uint32_t)(k >> kIdxBits);
    uint32_t b = ou ^ ((ou >> 31) ? 0x80000000u : 0xFFFFFFFFu);
    return __uint_as_float(b);
}
__device__ __forceinline__ uint32_t key_index(double key) {
    return (uint32_t)__double_as_longlong(key) & ((1u << kIdxBits) - 1u);
}

__device__ __forceinline__ void cmp_exchange(double& lo, double& hi) {
    double a = fmin(lo, hi), b = fmax(lo, hi);
    lo = a;
    hi = b;
}

// Value of `x` held by lane (lane ^ LM).  Masks that a DPP modifier can express (1, 2, 3 within a
// quad, 7 and 15 as half-row / row mirrors) cost one VALU move; other masks below 32 go through the
// LDS crossbar without touching LDS memory (ds_swizzle, bit mode); masks that cross the two
// 32-lane halves use ds_bpermute with the partner's lane index.
template <int LM>
__device__ __forceinline__ uint32_t lane_xor(uint32_t x, int lane) {
    if constexpr (LM == 1) return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0xB1, 0xF, 0xF, true);
    else if constexpr (LM == 2) return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x4E, 0xF, 0xF, true);
    else if constexpr (LM == 3) return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x1B, 0xF, 0xF, true);
    else if constexpr (LM == 7) return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x141, 0xF, 0xF, true);
    else if constexpr (LM == 15) return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x140, 0xF, 0xF, true);
    else if constexpr (LM < 32) return (uint32_t)__builtin_amdgcn_ds_swizzle((int)x, 0x1F | (LM << 10));
    else return (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ LM) << 2, (int)x);
}
template <int LM>
__device__ __forceinline__ double lane_xor(double x, int lane) {
    const uint32_t lo = lane_xor<LM>((uint32_t)__double2loint(x), lane);
    const uint32_t hi = lane_xor<LM>((uint32_t)__double2hiint(x), lane);
    return __hiloint2double((int)hi, (int)lo);
}

// Keys are pairwise distinct, so "mine < other" decides; the lower lane of a pair keeps the smaller.
__device__ __forceinline__ double keep(double mine, double other, bool lower) {
    return ((mine < other) == lower) ? mine : other;
}

// First step of a bitonic merge of blocks of `SIZE`: element e meets e ^ (SIZE-1).
template <int KPL, int SIZE>
__device__ __forceinline__ void stage_mirror(double (&key)[KPL], int lane) {
    if constexpr (SIZE <= KPL) {
#pragma unroll
        for (int j = 0; j < KPL; ++j) {
            const int p = j ^ (SIZE - 1);
            if (j < p) cmp_exchange(key[j], key[p]);
        }
    } else {
        constexpr int LM = SIZE / KPL - 1;          // lane ^ LM, register KPL-1-j
        const bool lower = (lane & ((LM + 1) >> 1)) == 0;
        double other[KPL];
#pragma unroll
        for (int j = 0; j < KPL; ++j) other[j] = lane_xor<LM>(key[KPL - 1 - j], lane);
#pragma unroll
        for (int j = 0; j < KPL; ++j) key[j] = keep(key[j], other[j], lower);
    }
}

// Later steps of a merge: element e meets e ^ STRIDE.
template <int KPL, int STRIDE>
__device__ __forceinline__ void stage_xor(double (&key)[KPL], int lane) {
    if constexpr (STRIDE < KPL) {
#pragma unroll
        for (int j = 0; j < KPL; ++j) {
            const int p = j ^ STRIDE;
            if (j < p) cmp_exchange(key[j], key[p]);
        }
    } else {
        constexpr int LM = STRIDE / KPL;
        const bool lower = (lane & LM) == 0;
#pragma unroll
        for (int j = 0; j < KPL; ++j) key[j] = keep(key[j], lane_xor<LM>(key[j], lane), lower);
    }
}

template <int KPL, int SIZE, int STRIDE>
__device__ __forceinline__ void merge_steps(double (&key)[KPL], int lane) {
    if constexpr (STRIDE >= 1) {
        stage_xor<KPL, STRIDE>(key, lane);
        merge_steps<KPL, SIZE, STRIDE / 2>(key, lane);
    }
}

template <int KPL, int SIZE>
__device__ __forceinline__ void sort_from(double (&key)[KPL], int lane) {
    if constexpr (SIZE <= kWave * KPL) {
        stage_mirror<KPL, SIZE>(key, lane);
        merge_steps<KPL, SIZE, SIZE / 4>(key, lane);
        sort_from<KPL, SIZE * 2>(key, lane);
    }
}

// x of another lane under a DPP control word; lanes the pattern leaves without a source get `fill`.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_f64(double x, double fill) {
    const int lo = __builtin_amdgcn_update_dpp(__double2loint(fill), __double2loint(x), CTRL, ROW_MASK, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(__double2hiint(fill), __double2hiint(x), CTRL, ROW_MASK, 0xF, false);
    return __hiloint2double(hi, lo);
}

// Inclusive scan over the 64 lanes: shifts by 1, 2, 4, 8 inside each row of 16 lanes, then lane 15
// of rows 0 and 2 is broadcast into rows 1 and 3, then lane 31 into rows 2 and 3.
__device__ __forceinline__ double wave_inclusive_scan(double x) {
    x += dpp_f64<0x111, 0xF>(x, 0.0);   // row_shr:1
    x += dpp_f64<0x112, 0xF>(x, 0.0);   // row_shr:2
    x += dpp_f64<0x114, 0xF>(x, 0.0);   // row_shr:4
    x += dpp_f64<0x118, 0xF>(x, 0.0);   // row_shr:8
    x += dpp_f64<0x142, 0xA>(x, 0.0);   // row_bcast:15 into rows 1, 3
    x += dpp_f64<0x143, 0xC>(x, 0.0);   // row_bcast:31 into rows 2, 3
    return x;
}

// Maximum over the 64 lanes, returned wave-uniform (same data movement as the scan; lane 63 ends
// up with the maximum of everything before it).
__device__ __forceinline__ double wave_max(double x) {
    const double ninf = -__builtin_huge_val();
    x = fmax(x, dpp_f64<0x111, 0xF>(x, ninf));
    x = fmax(x, dpp_f64<0x112, 0xF>(x, ninf));
    x = fmax(x, dpp_f64<0x114, 0xF>(x, ninf));
    x = fmax(x, dpp_f64<0x118, 0xF>(x, ninf));
    x = fmax(x, dpp_f64<0x142, 0xA>(x, ninf));
    x = fmax(x, dpp_f64<0x143, 0xC>(x, ninf));
    const int lo = __builtin_amdgcn_readlane(__double2loint(x), kWave - 1);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(x), kWave - 1);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double lane_value(double x, int src_lane) {   // src_lane wave-uniform
    const int lo = __builtin_amdgcn_readlane(__double2loint(x), src_lane);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(x), src_lane);
    return __hiloint2double(hi, lo);
}

// Dynamic LDS per wave: float val[N]; uint16 idx[N]; double p1[m+1]; double p2[m+1].
__host__ __device__ inline size_t wave_lds_bytes(int N, int m) {
    size_t b = (size_t)N * 4 + (size_t)N * 2;
    b = (b + 7) / 8 * 8;
    return b + 2 * (size_t)(m + 1) * 8;
}

template <int KPL, int WAVES>
__global__ __launch_bounds__(WAVES* kWave) void select_kernel(const float* __restrict__ rewards,
                                                              const uint32_t* __restrict__ rand_keys,
                                                              int B, int n, int m, int rule,
                                                              int32_t* __restrict__ sel_idx,
                                                              int32_t* __restrict__ sel_k) {
    constexpr int N = kWave * KPL;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int group = blockIdx.x * WAVES + wave;
    const bool live = group < B;  // dead waves still take every barrier

    unsigned char* base = lds_raw + (size_t)wave * wave_lds_bytes(N, m);
    float* s_val = reinterpret_cast<float*>(base);
    uint16_t* s_idx = reinterpret_cast<uint16_t*>(base + (size_t)N * 4);
    double* p1 = reinterpret_cast<double*>(base + ((size_t)N * 6 + 7) / 8 * 8);
    double* p2 = p1 + (m + 1);

    // ---- load and key (Alg. 2 step 1 input) ----
    double key[KPL];
    if (rule == PODS_RULE_RAND) {   // the m smallest of the caller's random keys, ties by index
        const uint32_t* row = rand_keys + (size_t)(live ? group : 0) * n;
#pragma unroll
        for (int j = 0; j < KPL; ++j) {
            const int e = lane * KPL + j;
            key[j] = (e < n) ? make_key_u32(row[e], (uint32_t)e) : pad_key((uint32_t)e);
        }
    } else {
        const float* row = rewards + (size_t)(live ? group : 0) * n;
#pragma unroll
        for (int j = 0; j < KPL; ++j) {
            const int e = lane * KPL + j;
            key[j] = (e < n) ? make_key(row[e], (uint32_t)e) : pad_key((uint32_t)e);
        }
    }

    // ---- argsort ascending by (reward, index) ----
    sort_from<KPL, 2>(key, lane);

#pragma unroll
    for (int j = 0; j < KPL; ++j) {
        const int e = lane * KPL + j;
        s_val[e] = key_reward(key[j]);
        s_idx[e] = (uint16_t)key_index(key[j]);
    }
    __syncthreads();

    if (rule != PODS_RULE_MAXVAR) {
        // Sec. 3.2's other rules are positions of the sorted order: the m highest (max-reward), the
        // (j + 1/2)/m quantiles taken as position floor((2j + 1) n / (2m)) (percentile), and the m
        // lowest of the random keys (random).
        if (live) {
            int32_t* out = sel_idx + (size_t)group * m;
            for (int j = lane; j < m; j += kWave) {
                int pos = j;
                if (rule == PODS_RULE_MAXR) pos = n - m + j;
                if (rule == PODS_RULE_PERC) pos = (int)(((int64_t)(2 * j + 1) * n) / (2 * m));
                out[j] = (int32_t)s_idx[pos];
            }
            if (sel_k != nullptr && lane == 0) sel_k[group] = (rule == PODS_RULE_MAXR) ? m : -1;
        }
        return;
    }

    // ---- Theorem 1: prefix sums of r and r^2 over the m lowest ----
    double c1 = 0.0, c2 = 0.0;
    if (lane == 0) { p1[0] = 0.0; p2[0] = 0.0; }
    for (int e0 = 0; e0 < m; e0 += kWave) {
        const int e = e0 + lane;
        const double x = (e < m) ? (double)s_val[e] : 0.0;
        const double a1 = wave_inclusive_scan(x) + c1;
        const double a2 = wave_inclusive_scan(x * x) + c2;
        if (e < m) { p1[e + 1] = a1; p2[e + 1] = a2; }
        c1 = lane_value(a1, kWave - 1);
        c2 = lane_value(a2, kWave - 1);
    }
    __syncthreads();

    // ---- Alg. 2 steps 2-6: score every split k, keep the first strict maximum ----
    // k = 0 (the m lowest) is the starting candidate; lane l of pass k0 scores k = k0 + l + 1.
    const double dm = (double)m;
    double best = dm * c2 - c1 * c1;   // wave-uniform
    int best_k = 0;
    c1 = 0.0;
    c2 = 0.0;
    for (int k0 = 0; k0 < m; k0 += kWave) {
        const int k = k0 + lane + 1;
        const bool in = k <= m;
        const float top = in ? s_val[n - k] : 0.0f;
        const double x = (double)top;
        const double u1 = wave_inclusive_scan(x) + c1;   // sum of the k highest
        const double u2 = wave_inclusive_scan(x * x) + c2;
        c1 = lane_value(u1, kWave - 1);
        c2 = lane_value(u2, kWave - 1);
        double D = -__builtin_huge_val();
        if (in && top != s_val[m - k]) {   // else same multiset as split k-1
            const double S = p1[m - k] + u1;
            const double Q = p2[m - k] + u2;
            D = dm * Q - S * S;
        }
        const double top_d = wave_max(D);
        if (top_d > best) {   // strictly larger only: an earlier (smaller) k keeps its place on ties
            best = top_d;
            best_k = k0 + 1 + (int)__builtin_ctzll(__ballot(D == top_d));
        }
    }

    // ---- emit the (m-k) lowest then the k highest ----
    if (live) {
        int32_t* out = sel_idx + (size_t)group * m;
        for (int j = lane; j < m; j += kWave)
            out[j] = (j < m - best_k) ? (int32_t)s_idx[j] : (int32_t)s_idx[n - m + j];
        if (sel_k != nullptr && lane == 0) sel_k[group] = best_k;
    }
}

template <int KPL, int WAVES>
pods_status launch_variant(const float* rewards, const uint32_t* rand_keys, int32_t B, int32_t n, int32_t m,
                           int32_t rule, int32_t* sel_idx, int32_t* sel_k, hipStream_t stream) {
    const size_t lds = (size_t)WAVES * wave_lds_bytes(kWave * KPL, m);
    if (lds > 160 * 1024) return fail(PODS_ERR_UNSUPPORTED, "pods_select: LDS need %zu B", lds);
    auto kernel = select_kernel<KPL, WAVES>;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess)
            return fail(PODS_ERR_RUNTIME, "pods_select: cannot reserve %zu B of LDS: %s", lds,
                        hipGetErrorString(e));
    }
    const unsigned grid = (unsigned)ceil_div(B, WAVES);
    PODS_LAUNCH("pods_select", stream, kernel, dim3(grid), dim3(WAVES * kWave), lds, stream, rewards, rand_keys,
                B, n, m, rule, sel_idx, sel_k);
    return check_launch("pods_select");
}

}  // namespace

pods_status launch_select(const float* rewards, const uint32_t* rand_keys, int32_t B, int32_t n, int32_t m,
                          int32_t rule, int32_t* sel_idx, int32_t* sel_k, hipStream_t stream) {
    if (n <= 64) return launch_variant<1, 4>(rewards, rand_keys, B, n, m, rule, sel_idx, sel_k, stream);
    if (n <= 128) return launch_variant<2, 4>(rewards, rand_keys, B, n, m, rule, sel_idx, sel_k, stream);
    if (n <= 256) return launch_variant<4, 4>(rewards, rand_keys, B, n, m, rule, sel_idx, sel_k, stream);
    if (n <= 512) return launch_variant<8, 2>(rewards, rand_keys, B, n, m, rule, sel_idx, sel_k, stream);
    if (n <= 1024) return launch_variant<16, 2>(rewards, rand_keys, B, n, m, rule, sel_idx, sel_k, stream);
    if (n <= 2048) return launch_variant<32, 1>(rewards, rand_keys, B, n, m, rule, sel_idx, sel_k, stream);
    if (n <= 4096) return launch_variant<64, 1>(rewards, rand_keys, B, n, m, rule, sel_idx, sel_k, stream);
    return fail(PODS_ERR_UNSUPPORTED, "pods_select: n = %d exceeds 4096", n);
}

}  // namespace pods
