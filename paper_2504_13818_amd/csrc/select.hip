// Down-sampling rules: max-variance (Sec. 3.3: Lemma 3.1, Algorithm 2, Theorem 1) and, on the
// same sorted order, max-reward, percentile and random (Sec. 3.2).
//
// A prompt group is sorted by G lanes of a wavefront, KPL keys per lane (G * KPL >= n), so one
// wavefront handles 64 / G groups at once.  Few lanes per group is the point: a compare-exchange
// between two keys of the same lane is one v_min_f64 plus one v_max_f64, one between lanes costs
// two data moves, a minimum and a sign flip per key, so for n = 256 eight lanes with 32 keys each
// run 30 of the 36 bitonic stages inside the lane.  (Between lanes the compare is avoided too: see
// set_sign.)
//
// A key is the order-preserving integer image of the float32 reward followed by the element's
// index, laid into the mantissa of a double in [2, 4): for such doubles floating-point order equals
// integer order.  The index in the low bits makes every key distinct and gives the (reward, index)
// order the tie rule asks for.  Partner values travel by DPP moves (every lane pattern inside a
// row of 16 lanes has one), through the LDS crossbar (ds_swizzle) up to 32 lanes, by ds_bpermute
// beyond.
//
// After the sort the keys at the m lowest and the m highest positions of each group are staged in
// LDS.  Each lane of the group then owns a contiguous block of the candidate splits k: it sums its
// block of the lowest / highest rewards and their squares in double precision, a scan over the G
// lanes turns block sums into block offsets, and the lane walks its candidates in ascending k,
// scoring m*Q - S^2 (m^2 times the variance) from the prefix sums of Theorem 1.  Candidates that
// repeat the previous multiset are passed over; a strictly larger score replaces the running best,
// and across lanes the larger score, or on equal scores the smaller k, wins.
#include "common.h"

namespace pods {
namespace {

constexpr int kIdxBits = 12;  // n <= 4096

__device__ __forceinline__ double make_key_u32(uint32_t ou, uint32_t e) {
    uint64_t k = (1ull << 62) | ((uint64_t)ou << kIdxBits) | e;
    return __longlong_as_double((long long)k);
}
__device__ __forceinline__ double make_key(float r, uint32_t e) {
    r = r + 0.0f;  // -0.0 -> +0.0
    uint32_t b = __float_as_uint(r);
    return make_key_u32(b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u), e);  // unsigned order == float order
}
__device__ __forceinline__ double pad_key(uint32_t e) { return make_key_u32(0xFFFFFFFFu, e); }  // after every real key
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

// Value of `x` held by lane (lane ^ LM).  Inside a row of 16 lanes every mask the network uses has
// a DPP form: quad permutes (1, 2, 3), half-row and row mirrors (7, 15), a row rotation (8), and for
// 4 a shift up plus a shift down, each written to the banks of lanes it is right for.
template <int LM>
__device__ __forceinline__ uint32_t lane_xor(uint32_t x, int lane) {
    if constexpr (LM == 1) return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0xB1, 0xF, 0xF, true);
    else if constexpr (LM == 2) return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x4E, 0xF, 0xF, true);
    else if constexpr (LM == 3) return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x1B, 0xF, 0xF, true);
    else if constexpr (LM == 7) return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x141, 0xF, 0xF, true);
    else if constexpr (LM == 15) return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x140, 0xF, 0xF, true);
    else if constexpr (LM == 8) return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x128, 0xF, 0xF, true);  // row_ror:8
    else if constexpr (LM == 4) {
        const int up = __builtin_amdgcn_update_dpp((int)x, (int)x, 0x104, 0xF, 0x5, false);   // row_shl:4 -> lanes 0-3, 8-11
        return (uint32_t)__builtin_amdgcn_update_dpp(up, (int)x, 0x114, 0xF, 0xA, false);    // row_shr:4 -> lanes 4-7, 12-15
    }
    else if constexpr (LM < 32) return (uint32_t)__builtin_amdgcn_ds_swizzle((int)x, 0x1F | (LM << 10));
    else return (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ LM) << 2, (int)x);
}
template <int LM>
__device__ __forceinline__ double lane_xor(double x, int lane) {
    const uint32_t lo = lane_xor<LM>((uint32_t)__double2loint(x), lane);
    const uint32_t hi = lane_xor<LM>((uint32_t)__double2hiint(x), lane);
    return __hiloint2double((int)hi, (int)lo);
}

// Compare-exchange between lanes without a compare: for the duration of a cross-lane stage the
// lane that is to keep the larger key of its pair holds its keys negated (sign bit flipped, which
// reverses the order of these never-zero doubles).  Then both lanes of a pair compute
// min(mine, -other): the lower lane gets min(a, b), the upper one min(-b, -a) = -max(a, b).
// `sign` is the flip this lane's keys currently carry; moving to another stage costs one XOR per key.
template <int KPL>
__device__ __forceinline__ void set_sign(double (&key)[KPL], uint32_t& sign, uint32_t want) {
    const uint32_t delta = sign ^ want;
#pragma unroll
    for (int j = 0; j < KPL; ++j)
        key[j] = __hiloint2double((int)((uint32_t)__double2hiint(key[j]) ^ delta), __double2loint(key[j]));
    sign = want;
}

// First step of a bitonic merge of blocks of `SIZE`: element e meets e ^ (SIZE-1).
template <int KPL, int SIZE>
__device__ __forceinline__ void stage_mirror(double (&key)[KPL], uint32_t& sign, int lane) {
    if constexpr (SIZE <= KPL) {
#pragma unroll
        for (int j = 0; j < KPL; ++j) {
            const int p = j ^ (SIZE - 1);
            if (j < p) cmp_exchange(key[j], key[p]);
        }
    } else {
        constexpr int LM = SIZE / KPL - 1;          // lane ^ LM, register KPL-1-j
        set_sign<KPL>(key, sign, (lane & ((LM + 1) >> 1)) ? 0x80000000u : 0u);
#pragma unroll
        for (int j = 0; j < KPL / 2; ++j) {
            const double oa = lane_xor<LM>(key[KPL - 1 - j], lane);
            const double ob = lane_xor<LM>(key[j], lane);
            key[j] = fmin(key[j], -oa);
            key[KPL - 1 - j] = fmin(key[KPL - 1 - j], -ob);
        }
    }
}

// Later steps of a merge: element e meets e ^ STRIDE.
template <int KPL, int STRIDE, bool CROSSED>
__device__ __forceinline__ void stage_xor(double (&key)[KPL], uint32_t& sign, int lane) {
    if constexpr (STRIDE < KPL) {
        // first in-lane step after cross-lane ones: back to true keys
        if constexpr (CROSSED && STRIDE == KPL / 2) set_sign<KPL>(key, sign, 0u);
#pragma unroll
        for (int j = 0; j < KPL; ++j) {
            const int p = j ^ STRIDE;
            if (j < p) cmp_exchange(key[j], key[p]);
        }
    } else {
        constexpr int LM = STRIDE / KPL;
        set_sign<KPL>(key, sign, (lane & LM) ? 0x80000000u : 0u);
#pragma unroll
        for (int j = 0; j < KPL; ++j) key[j] = fmin(key[j], -lane_xor<LM>(key[j], lane));
    }
}

template <int KPL, int STRIDE, bool CROSSED>
__device__ __forceinline__ void merge_steps(double (&key)[KPL], uint32_t& sign, int lane) {
    if constexpr (STRIDE >= 1) {
        stage_xor<KPL, STRIDE, CROSSED>(key, sign, lane);
        merge_steps<KPL, STRIDE / 2, CROSSED>(key, sign, lane);
    }
}

// Bitonic sort of the G*KPL keys held by each aligned run of G lanes (element e = lane-in-run * KPL + j).
template <int KPL, int G, int SIZE>
__device__ __forceinline__ void sort_from(double (&key)[KPL], uint32_t& sign, int lane) {
    static_assert(KPL >= 2, "the sign is restored by the first in-lane step of each merge");
    if constexpr (SIZE <= G * KPL) {
        stage_mirror<KPL, SIZE>(key, sign, lane);
        merge_steps<KPL, SIZE / 4, (SIZE > KPL)>(key, sign, lane);
        sort_from<KPL, G, SIZE * 2>(key, sign, lane);
    }
}

// x of lane (lane - OFF), OFF < 16, 0.0 where that lane lies before the start of the row of 16 lanes
// or, for runs shorter than a row, before the start of the run.
template <int G, int OFF>
__device__ __forceinline__ double run_shift_up(double x, int gl) {
    static_assert(OFF < 16 && OFF < G, "shift inside a row and inside the run");
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(x), 0x110 + OFF, 0xF, 0xF, true);   // row_shr:OFF
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(x), 0x110 + OFF, 0xF, 0xF, true);
    if constexpr (G >= 16) return __hiloint2double(hi, lo);
    const bool has = gl >= OFF;
    return __hiloint2double(has ? hi : 0, has ? lo : 0);
}

// Exclusive prefix sum of x over the lanes of each run of G lanes (lane 0 of the run gets 0).
template <int G>
__device__ __forceinline__ double run_exclusive_scan(double x, int gl, int lane) {
    if constexpr (G >= 2) x += run_shift_up<G, 1>(x, gl);
    if constexpr (G >= 4) x += run_shift_up<G, 2>(x, gl);
    if constexpr (G >= 8) x += run_shift_up<G, 4>(x, gl);
    if constexpr (G >= 16) x += run_shift_up<G, 8>(x, gl);
    if constexpr (G >= 32) {           // lane 15 of rows 0 and 2 into rows 1 and 3
        const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(x), 0x142, 0xA, 0xF, false);
        const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(x), 0x142, 0xA, 0xF, false);
        x += __hiloint2double(hi, lo);
    }
    if constexpr (G >= 64) {           // lane 31 into rows 2 and 3
        const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(x), 0x143, 0xC, 0xF, false);
        const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(x), 0x143, 0xC, 0xF, false);
        x += __hiloint2double(hi, lo);
    }
    // inclusive -> exclusive: the left neighbour's value
    const int lo = __builtin_amdgcn_ds_bpermute(((lane - 1) & (kWave - 1)) << 2, __double2loint(x));
    const int hi = __builtin_amdgcn_ds_bpermute(((lane - 1) & (kWave - 1)) << 2, __double2hiint(x));
    return gl == 0 ? 0.0 : __hiloint2double(hi, lo);
}

// The same sum taken from the other end of the run: over the lanes above this one.
template <int G>
__device__ __forceinline__ double run_exclusive_scan_down(double x, int gl, int lane) {
    const double y = run_exclusive_scan<G>(lane_xor<G - 1>(x, lane), gl, lane);
    return lane_xor<G - 1>(y, lane);
}

// Best (score, k) over the lanes of a run: the larger score, on equal scores the smaller k.
template <int LM>
__device__ __forceinline__ void run_best(double& best, int& best_k, int lane) {
    if constexpr (LM >= 1) {
        const double ob = lane_xor<LM>(best, lane);
        const int ok = (int)lane_xor<LM>((uint32_t)best_k, lane);
        if (ob > best || (ob == best && ok < best_k)) { best = ob; best_k = ok; }
        run_best<LM / 2>(best, best_k, lane);
    }
}

// Keys at sorted positions [first, first + count) to LDS; this lane holds positions e0 .. e0 + KPL - 1,
// which usually lie wholly inside or wholly outside the range.
template <int KPL>
__device__ __forceinline__ void stage_range(const double (&key)[KPL], int e0, int first, int count, double* dst) {
    if (e0 >= first && e0 + KPL <= first + count) {
#pragma unroll
        for (int j = 0; j < KPL; ++j) dst[e0 - first + j] = key[j];
    } else if (e0 + KPL > first && e0 < first + count) {
#pragma unroll
        for (int j = 0; j < KPL; ++j) {
            const int p = e0 + j;
            if (p >= first && p < first + count) dst[p - first] = key[j];
        }
    }
}

constexpr int kBlockMax = 8;   // candidates per lane that the register-resident scan covers

// LDS per group.  Max-variance: the keys at the m lowest and the m highest sorted positions, then,
// when a lane owns more than kBlockMax candidates, double p1[m+1], p2[m+1].  Other rules: uint16 idx[n].
__host__ __device__ inline size_t group_lds_bytes(int n, int m, int rule, int G) {
    if (rule != PODS_RULE_MAXVAR) return ((size_t)n * 2 + 15) / 16 * 16;
    const bool in_registers = (m + G - 1) / G <= kBlockMax;
    return (size_t)m * 16 + (in_registers ? 0 : 2 * (size_t)(m + 1) * 8);
}

template <int KPL, int G>
__global__ __launch_bounds__(256) void select_kernel(const float* __restrict__ rewards,
                                                     const uint32_t* __restrict__ rand_keys,
                                                     int B, int n, int m, int rule,
                                                     int32_t* __restrict__ sel_idx,
                                                     int32_t* __restrict__ sel_k) {
    constexpr int kGroupsPerWave = kWave / G;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int waves = blockDim.x / kWave;
    const int gl = lane & (G - 1);                 // lane within the group's run
    const int slot = wave * kGroupsPerWave + lane / G;
    const int64_t group = (int64_t)blockIdx.x * (waves * kGroupsPerWave) + slot;
    const bool live = group < B;                   // dead runs still take every barrier

    // ---- load and key (Alg. 2 step 1 input): lane gl holds elements gl*KPL .. gl*KPL + KPL-1 ----
    double key[KPL];
    const int e0 = gl * KPL;
    if (rule == PODS_RULE_RAND) {   // the m smallest of the caller's random keys, ties by index
        const uint32_t* row = rand_keys + (size_t)(live ? group : 0) * n;
#pragma unroll
        for (int j = 0; j < KPL; ++j)
            key[j] = (e0 + j < n) ? make_key_u32(row[e0 + j], (uint32_t)(e0 + j)) : pad_key((uint32_t)(e0 + j));
    } else {
        const float* row = rewards + (size_t)(live ? group : 0) * n;
        if (KPL >= 4 && n == G * KPL && (reinterpret_cast<uintptr_t>(rewards) & 15) == 0) {
            // full rows of 16-byte-aligned lane blocks
#pragma unroll
            for (int j = 0; j + 3 < KPL; j += 4) {
                const float4 v = *reinterpret_cast<const float4*>(row + e0 + j);
                key[j] = make_key(v.x, (uint32_t)(e0 + j));
                key[j + 1] = make_key(v.y, (uint32_t)(e0 + j + 1));
                key[j + 2] = make_key(v.z, (uint32_t)(e0 + j + 2));
                key[j + 3] = make_key(v.w, (uint32_t)(e0 + j + 3));
            }
        } else {
#pragma unroll
            for (int j = 0; j < KPL; ++j)
                key[j] = (e0 + j < n) ? make_key(row[e0 + j], (uint32_t)(e0 + j)) : pad_key((uint32_t)(e0 + j));
        }
    }

    // ---- argsort ascending by (key, index): sorted position p = gl*KPL + j ----
    uint32_t sign = 0u;
    sort_from<KPL, G, 2>(key, sign, lane);

    unsigned char* base = lds_raw + (size_t)slot * group_lds_bytes(n, m, rule, G);
    if (rule != PODS_RULE_MAXVAR) {
        // Sec. 3.2's other rules are positions of the sorted order: the m highest (max-reward), the
        // (j + 1/2)/m quantiles taken as position floor((2j + 1) n / (2m)) (percentile), and the m
        // lowest of the random keys (random).
        uint16_t* s_idx = reinterpret_cast<uint16_t*>(base);
#pragma unroll
        for (int j = 0; j < KPL; ++j)
            if (e0 + j < n) s_idx[e0 + j] = (uint16_t)key_index(key[j]);
        __syncthreads();
        if (live) {
            int32_t* out = sel_idx + (size_t)group * m;
            for (int j = gl; j < m; j += G) {
                int pos = j;
                if (rule == PODS_RULE_MAXR) pos = n - m + j;
                if (rule == PODS_RULE_PERC) pos = (int)(((int64_t)(2 * j + 1) * n) / (2 * m));
                out[j] = (int32_t)s_idx[pos];
            }
            if (sel_k != nullptr && gl == 0) sel_k[group] = (rule == PODS_RULE_MAXR) ? m : -1;
        }
        return;
    }

    double* k_lo = reinterpret_cast<double*>(base);   // keys at positions 0 .. m-1
    double* k_hi = k_lo + m;                          // keys at positions n-m .. n-1
    double* p1 = k_hi + m;
    double* p2 = p1 + (m + 1);
    stage_range<KPL>(key, e0, 0, m, k_lo);
    stage_range<KPL>(key, e0, n - m, m, k_hi);
    __syncthreads();

    // ---- Theorem 1 and Alg. 2 steps 2-6 ----
    // Lane gl scores the candidates k = j0+1 .. j1.  Candidate k reads sorted positions m-k of the low
    // and of the high staged range (the reward that leaves, the reward that enters), so the lane owns
    // offsets [a, b) = [m-j1, m-j0) of both ranges.
    const int per_lane = (m + G - 1) / G;
    const int j0 = min(m, gl * per_lane), j1 = min(m, j0 + per_lane);
    const double dm = (double)m;
    double best = -__builtin_huge_val();
    int best_k = 0x7fffffff;
    if (per_lane <= kBlockMax) {
        // Everything in registers: the block's rewards, its prefix sums of the low range (ascending
        // position) and its running sums of the high range (ascending k, i.e. descending position).
        const int a = m - j1, cnt = j1 - j0;
        double lo_r[kBlockMax], hi_r[kBlockMax];
#pragma unroll
        for (int i = 0; i < kBlockMax; ++i) {
            const int pos = min(a + i, m - 1);   // slots past the block are read in bounds and not used
            lo_r[i] = (i < cnt) ? (double)key_reward(k_lo[pos]) : 0.0;
            hi_r[i] = (i < cnt) ? (double)key_reward(k_hi[pos]) : 0.0;
        }
        double bl1 = 0.0, bl2 = 0.0, bh1 = 0.0, bh2 = 0.0;
#pragma unroll
        for (int i = 0; i < kBlockMax; ++i) {
            bl1 += lo_r[i];
            bl2 += lo_r[i] * lo_r[i];
        }
#pragma unroll
        for (int i = kBlockMax - 1; i >= 0; --i) {
            bh1 += hi_r[i];
            bh2 += hi_r[i] * hi_r[i];
        }
        // lower positions of the low range belong to the lanes above; smaller k to the lanes below
        double r1 = run_exclusive_scan_down<G>(bl1, gl, lane);
        double r2 = run_exclusive_scan_down<G>(bl2, gl, lane);
        double u1 = run_exclusive_scan<G>(bh1, gl, lane);
        double u2 = run_exclusive_scan<G>(bh2, gl, lane);
        double pp1[kBlockMax], pp2[kBlockMax];   // sums of the low range below position a + i
#pragma unroll
        for (int i = 0; i < kBlockMax; ++i) {
            pp1[i] = r1;
            pp2[i] = r2;
            r1 += lo_r[i];
            r2 += lo_r[i] * lo_r[i];
        }
        if (gl == 0) {   // k = 0, the m lowest: lane 0's block ends at position m
            best = dm * r2 - r1 * r1;
            best_k = 0;
        }
#pragma unroll
        for (int i = kBlockMax - 1; i >= 0; --i) {   // ascending k = m - (a + i)
            u1 += hi_r[i];
            u2 += hi_r[i] * hi_r[i];
            if (i < cnt && hi_r[i] != lo_r[i]) {   // else same multiset as split k-1
                const double S = pp1[i] + u1;
                const double Q = pp2[i] + u2;
                const double D = dm * Q - S * S;
                if (D > best) { best = D; best_k = m - (a + i); }
            }
        }
    } else {
        // Larger blocks: the prefix sums go through LDS.
        double b1 = 0.0, b2 = 0.0;
        for (int j = j0; j < j1; ++j) {
            const double x = (double)key_reward(k_lo[j]);
            b1 += x;
            b2 += x * x;
        }
        double r1 = run_exclusive_scan<G>(b1, gl, lane);
        double r2 = run_exclusive_scan<G>(b2, gl, lane);
        if (gl == 0) { p1[0] = 0.0; p2[0] = 0.0; }
        for (int j = j0; j < j1; ++j) {
            const double x = (double)key_reward(k_lo[j]);
            r1 += x;
            r2 += x * x;
            p1[j + 1] = r1;
            p2[j + 1] = r2;
        }
        // sums of the k highest up to the start of this lane's block of candidates k = j0+1 .. j1
        b1 = 0.0;
        b2 = 0.0;
        for (int k = j0 + 1; k <= j1; ++k) {
            const double x = (double)key_reward(k_hi[m - k]);
            b1 += x;
            b2 += x * x;
        }
        double u1 = run_exclusive_scan<G>(b1, gl, lane);
        double u2 = run_exclusive_scan<G>(b2, gl, lane);
        __syncthreads();

        // score every split k, keep the first strict maximum
        if (gl == 0) {   // k = 0: the m lowest
            best = dm * p2[m] - p1[m] * p1[m];
            best_k = 0;
        }
        for (int k = j0 + 1; k <= j1; ++k) {
            const float top = key_reward(k_hi[m - k]);
            const double x = (double)top;
            u1 += x;
            u2 += x * x;
            if (top != key_reward(k_lo[m - k])) {   // else same multiset as split k-1
                const double S = p1[m - k] + u1;
                const double Q = p2[m - k] + u2;
                const double D = dm * Q - S * S;
                if (D > best) { best = D; best_k = k; }
            }
        }
    }
    run_best<G / 2>(best, best_k, lane);

    // ---- emit the (m-k) lowest then the k highest ----
    if (live) {
        int32_t* out = sel_idx + (size_t)group * m;
        for (int j = gl; j < m; j += G) out[j] = (int32_t)key_index((j < m - best_k) ? k_lo[j] : k_hi[j]);
        if (sel_k != nullptr && gl == 0) sel_k[group] = best_k;
    }
}

// ------------------------------------------------------------------------------------------------
// Max-variance selection of m = n/4 out of n = 16, 32, ... 256 (the paper's own ratios: 64 -> 16,
// 32 -> 8, 256 -> 64), with the whole network inside the lanes.
//
// Four lanes hold a group, KPL = n/4 keys each, and they sit 16 lanes apart (lanes s, s+16, s+32, s+48:
// 16 groups per wavefront), because two lane bits at those distances can be exchanged with a register
// bit by v_permlane16_swap / v_permlane32_swap: one instruction per 32-bit register pair moves the
// upper half of one register's lanes into the lower half of the other's.  A compare-exchange between
// two lanes then becomes: transpose (one swap per key word), compare-exchange between two registers of
// the same lane.  Each lane first sorts its KPL keys with Batcher's odd-even merge sort (543
// compare-exchanges for 64 keys against 672 of the bitonic network), then two bitonic merges (2 KPL,
// 4 KPL) run on element-index bits that are register bits when their turn comes; the bit parked in the
// lane meanwhile is one whose turn is far off, so a merge costs two or three transpositions, not one
// per stage.
// Direction: every compare-exchange is ascending in the value as stored.  A run that must descend for
// the next merge is sorted ascending on negated keys and then has its sign flipped (one XOR per key):
// these keys are doubles in [2, 4), never zero, so negation reverses their order exactly.
// The last merge starts with one half-cleaner across the two runs' lower halves and one across their upper
// halves, which separates the lowest and the highest quarter from the middle half; Theorem 1 never reads the
// middle half, so its registers are dropped, and the remaining stages run on half the keys.
// The last transpositions leave lane L = 0..3 of the group with sorted positions [L n/16, (L+1) n/16) of
// the lowest quarter and the same offsets of the highest quarter in registers, which is exactly the
// block of candidate splits k a lane scores (split k drops the low position m-k and adds the high
// position n-k): prefix sums, scores and the emitted indices never leave the registers; no LDS.
// ------------------------------------------------------------------------------------------------
template <int WHICH>   // 0: the lane bit 16 apart, 1: the lane bit 32 apart
__device__ __forceinline__ void lane_reg_swap(double& a, double& b) {
    unsigned alo = (unsigned)__double2loint(a), ahi = (unsigned)__double2hiint(a);
    unsigned blo = (unsigned)__double2loint(b), bhi = (unsigned)__double2hiint(b);
    if constexpr (WHICH == 0) {
        const auto lo = __builtin_amdgcn_permlane16_swap(alo, blo, false, false);
        const auto hi = __builtin_amdgcn_permlane16_swap(ahi, bhi, false, false);
        alo = lo[0]; blo = lo[1]; ahi = hi[0]; bhi = hi[1];
    } else {
        const auto lo = __builtin_amdgcn_permlane32_swap(alo, blo, false, false);
        const auto hi = __builtin_amdgcn_permlane32_swap(ahi, bhi, false, false);
        alo = lo[0]; blo = lo[1]; ahi = hi[0]; bhi = hi[1];
    }
    a = __hiloint2double((int)ahi, (int)alo);
    b = __hiloint2double((int)bhi, (int)blo);
}

// Exchange of the element-index bit held by a lane bit with the one held by register bit RB, over the
// registers for which live(r) holds: afterwards key[r | 1<<RB] of a lane whose bit is 0 holds what
// key[r] of the partner lane (bit 1) held, and vice versa.
template <int KPL, int WHICH, int RB, typename Live>
__device__ __forceinline__ void transpose_bit(double (&key)[KPL], Live live) {
#pragma unroll
    for (int r = 0; r < KPL; ++r)
        if ((r & (1 << RB)) == 0 && live(r)) lane_reg_swap<WHICH>(key[r], key[r | (1 << RB)]);
}
// Compare-exchange along register bit RB: the register with the bit clear keeps the smaller key.
template <int KPL, int RB, typename Live>
__device__ __forceinline__ void stage_reg_bit(double (&key)[KPL], Live live) {
#pragma unroll
    for (int r = 0; r < KPL; ++r)
        if ((r & (1 << RB)) == 0 && live(r)) cmp_exchange(key[r], key[r | (1 << RB)]);
}
template <int KPL, int RB_HI, int RB_LO, typename Live>
__device__ __forceinline__ void stages_reg_bits(double (&key)[KPL], Live live) {
    if constexpr (RB_HI >= RB_LO) {
        stage_reg_bit<KPL, RB_HI>(key, live);
        stages_reg_bits<KPL, RB_HI - 1, RB_LO>(key, live);
    }
}

// Batcher's odd-even merge sort of key[LO .. LO + N), ascending (all indices are compile-time constants).
template <int KPL, int LO, int N, int R>
__device__ __forceinline__ void oddeven_merge(double (&key)[KPL]) {
    constexpr int kStep = R * 2;
    if constexpr (kStep < N) {
        oddeven_merge<KPL, LO, N, kStep>(key);
        oddeven_merge<KPL, LO + R, N, kStep>(key);
#pragma unroll
        for (int i = LO + R; i + R < LO + N; i += kStep) cmp_exchange(key[i], key[i + R]);
    } else {
        cmp_exchange(key[LO], key[LO + R]);
    }
}
template <int KPL, int LO, int N>
__device__ __forceinline__ void oddeven_sort(double (&key)[KPL]) {
    if constexpr (N > 1) {
        oddeven_sort<KPL, LO, N / 2>(key);
        oddeven_sort<KPL, LO + N / 2, N / 2>(key);
        oddeven_merge<KPL, LO, N, 1>(key);
    }
}

constexpr int ilog2(int x) { return x <= 1 ? 0 : 1 + ilog2(x / 2); }

template <int KPL>
__device__ __forceinline__ void flip_sign(double (&key)[KPL], uint32_t mask) {
#pragma unroll
    for (int r = 0; r < KPL; ++r)
        key[r] = __hiloint2double((int)((uint32_t)__double2hiint(key[r]) ^ mask), __double2loint(key[r]));
}

// Value of x in the lane `lane ^ MASK` (MASK = 16 or 32).
template <int MASK>
__device__ __forceinline__ double partner(double x, int lane) {
    const int lo = __builtin_amdgcn_ds_bpermute((lane ^ MASK) << 2, __double2loint(x));
    const int hi = __builtin_amdgcn_ds_bpermute((lane ^ MASK) << 2, __double2hiint(x));
    return __hiloint2double(hi, lo);
}

// Between the phases nothing is to be moved: with free rein the scheduler stretches live ranges across them
// and the kernel no longer fits two wavefronts per SIMD without spilling.
#define PODS_PHASE_FENCE() __builtin_amdgcn_sched_barrier(0)
// Two wavefronts per SIMD (the 64 keys alone take 128 registers); three fit only with spills and measured
// slower, and 4096 wavefronts fill two rounds of two exactly.
template <int KPL>
__global__ __launch_bounds__(256, 2) void select_quarter_kernel(const float* __restrict__ rewards, int B,
                                                             int32_t* __restrict__ sel_idx,
                                                             int32_t* __restrict__ sel_k) {
    constexpr int kR = ilog2(KPL);         // register bits
    constexpr int kN = 4 * KPL, kM = KPL;  // n rollouts, m kept
    constexpr int kPer = KPL / 4;          // sorted positions of each outer quarter, and candidates, per lane
    static_assert(kR >= 2 && (1 << kR) == KPL, "KPL is a power of two, at least 4");
    const int lane = threadIdx.x & (kWave - 1);
    const int l0 = (lane >> 4) & 1, l1 = lane >> 5;     // the two lane bits of the group
    const int64_t group = ((int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave) * 16 + (lane & 15);
    const bool live = group < B;

    // ---- load and key: the lane takes every fourth float4 of the row (the group's four lanes read 64
    // contiguous bytes per instruction); the element's index rides in the key, so which lane sorts
    // which elements is free.  Lanes whose run must come out descending start with negated keys.
    const float4* row = reinterpret_cast<const float4*>(rewards + (size_t)(live ? group : 0) * kN);
    const int quad = 2 * l1 + l0;
    const uint32_t sign_a = ((l0 ^ l1) != 0) ? 0x80000000u : 0u;
    double key[KPL];
#pragma unroll
    for (int i = 0; i < KPL / 4; ++i) {
        const float4 v = row[4 * i + quad];
        const float x[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t b = __float_as_uint(x[c] + 0.0f);   // -0.0 -> +0.0
            const uint32_t ou = b ^ ((uint32_t)((int32_t)b >> 31) | 0x80000000u);   // unsigned order == float order
            const uint32_t lo = (ou << kIdxBits) | (uint32_t)(quad << 2) | (uint32_t)(16 * i + c);
            const uint32_t hi = (ou >> (32 - kIdxBits)) | 0x40000000u | sign_a;
            key[4 * i + c] = __hiloint2double((int)hi, (int)lo);
        }
    }
    auto all = [](int) { return true; };
    PODS_PHASE_FENCE();

    // ---- each lane: KPL keys ascending as stored
    oddeven_sort<KPL, 0, KPL>(key);

    // ---- merge of pairs of lanes (16 apart) into runs of 2 KPL.  Element bit kR sits in lane bit 0.
    flip_sign<KPL>(key, l0 ? 0x80000000u : 0u);                  // odd lanes now descend
    transpose_bit<KPL, 0, 0>(key, all);                          // lane bit 0 <- e0, register bit 0 <- e(kR)
    stage_reg_bit<KPL, 0>(key, all);                             // stride KPL
    stages_reg_bits<KPL, kR - 1, 1>(key, all);                   // strides KPL/2 .. 2
    transpose_bit<KPL, 0, 1>(key, all);                          // lane bit 0 <- e1, register bit 1 <- e0
    stage_reg_bit<KPL, 1>(key, all);                             // stride 1
    // now: lane bit 1 = e(kR+1), lane bit 0 = e1, register bit 0 = e(kR), bit 1 = e0, bit j = ej (j >= 2)

    // ---- merge of the two runs of 2 KPL (lanes 32 apart) into the sorted group, outer quarters only
    flip_sign<KPL>(key, l1 ? 0x80000000u : 0u);                  // the upper run now descends (all keys true)
    transpose_bit<KPL, 1, 1>(key, all);                          // lane bit 1 <- e0, register bit 1 <- e(kR+1)
    // Registers with bits (1, 0) = 00, 01 now hold the lower and the upper half of the ascending run, 10 and 11 the
    // upper and the lower half of the descending one.  Theorem 1 reads the m lowest and the m highest of the group
    // only: the m lowest lie in the two lower halves, and one half-cleaner across them (ascending half against
    // descending half, element by element) leaves exactly them, as a bitonic sequence, in its minima; likewise the
    // m highest in the maxima across the two upper halves.  (The full merge would spend two stages, three times as
    // many instructions, to get the same two quarters.)
#pragma unroll
    for (int r = 0; r < KPL; r += 4) {
        key[r] = fmin(key[r], key[r | 3]);                       // the lowest quarter
        key[r | 3] = fmax(key[r | 1], key[r | 2]);               // the highest quarter
    }
    // registers with bits (1, 0) = 00 hold the lowest quarter, 11 the highest; 01 and 10 are never read again
    auto outer = [](int r) { return (r & 3) == 0 || (r & 3) == 3; };
    stages_reg_bits<KPL, kR - 1, 2>(key, outer);                 // strides KPL/2 .. 4
    transpose_bit<KPL, 1, kR - 1>(key, outer);                   // lane bit 1 <- e(kR-1), register bit kR-1 <- e0
    transpose_bit<KPL, 0, kR - 2>(key, outer);                   // lane bit 0 <- e(kR-2), register bit kR-2 <- e1
    stage_reg_bit<KPL, kR - 2>(key, outer);                      // stride 2
    stage_reg_bit<KPL, kR - 1>(key, outer);                      // stride 1
    // Sorted position p: bit kR+1 = register bit 1, bit kR = register bit 0, bits kR-1, kR-2 = lane bits 1, 0,
    // bits kR-3 .. 2 = the same register bits, bit 1 = register bit kR-2, bit 0 = register bit kR-1.
    PODS_PHASE_FENCE();
    auto reg_of = [](int i, bool high) {   // register holding offset i (0 .. kPer-1) of this lane's block
        int r = high ? 3 : 0;
        r |= (i & ~3) & ((1 << (kR - 2)) - 1);                   // offset bits kR-3 .. 2
        r |= ((i >> 1) & 1) << (kR - 2);
        r |= (i & 1) << (kR - 1);
        return r;
    };

    // ---- Theorem 1 and Alg. 2 steps 2-6.  This lane owns offsets [a, a + kPer) of the m lowest and of the
    // m highest sorted positions, i.e. the candidate splits k = m - (a + i), i = 0 .. kPer-1.
    const int a = kPer * quad;
    // rewards as float32 and the keys' low words (which end in the index): 3 registers per position instead
    // of the 6 that double-precision rewards and separate indices would take
    float lo_r[kPer], hi_r[kPer];
    uint32_t lo_w[kPer], hi_w[kPer];
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        lo_r[i] = key_reward(key[reg_of(i, false)]);
        hi_r[i] = key_reward(key[reg_of(i, true)]);
        lo_w[i] = (uint32_t)__double2loint(key[reg_of(i, false)]);
        hi_w[i] = (uint32_t)__double2loint(key[reg_of(i, true)]);
    }
    PODS_PHASE_FENCE();
    double bl1 = 0.0, bl2 = 0.0, bh1 = 0.0, bh2 = 0.0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        const double x = (double)lo_r[i];
        bl1 += x;
        bl2 += x * x;
    }
#pragma unroll
    for (int i = kPer - 1; i >= 0; --i) {
        const double x = (double)hi_r[i];
        bh1 += x;
        bh2 += x * x;
    }
    PODS_PHASE_FENCE();
    // sums of the low range below this lane's block, of the high range above it
    const double tl1 = partner<16>(bl1, lane), tl2 = partner<16>(bl2, lane);
    const double th1 = partner<16>(bh1, lane), th2 = partner<16>(bh2, lane);
    const double ul1 = partner<32>(bl1 + tl1, lane), ul2 = partner<32>(bl2 + tl2, lane);
    const double uh1 = partner<32>(bh1 + th1, lane), uh2 = partner<32>(bh2 + th2, lane);
    double p1 = (l1 ? ul1 : 0.0) + (l0 ? tl1 : 0.0);     // low positions before offset a
    double p2 = (l1 ? ul2 : 0.0) + (l0 ? tl2 : 0.0);
    double u1 = (l1 ? 0.0 : uh1) + (l0 ? 0.0 : th1);     // high positions from offset a + kPer on
    double u2 = (l1 ? 0.0 : uh2) + (l0 ? 0.0 : th2);
    p1 += bl1;                                           // low positions before offset a + kPer
    p2 += bl2;
    const double dm = (double)kM;
    double best = -__builtin_huge_val();
    int best_k = 0x7fffffff;
    if (quad == 3) {   // k = 0, the m lowest: the last lane's block ends at position m
        best = dm * p2 - p1 * p1;
        best_k = 0;
    }
#pragma unroll
    for (int i = kPer - 1; i >= 0; --i) {   // ascending k = m - (a + i)
        const double xl = (double)lo_r[i], xh = (double)hi_r[i];
        p1 -= xl;                            // low positions before offset a + i
        p2 -= xl * xl;
        u1 += xh;                            // high positions from offset a + i on
        u2 += xh * xh;
        if (hi_r[i] != lo_r[i]) {            // else same multiset as split k-1
            const double S = p1 + u1;
            const double Q = p2 + u2;
            const double D = dm * Q - S * S;
            if (D > best) { best = D; best_k = kM - (a + i); }
        }
    }
    // best over the group's four lanes: the larger score, on equal scores the smaller k
#pragma unroll
    for (int step = 0; step < 2; ++step) {
        const double ob = step == 0 ? partner<16>(best, lane) : partner<32>(best, lane);
        const int ok = __builtin_amdgcn_ds_bpermute((lane ^ (step == 0 ? 16 : 32)) << 2, best_k);
        if (ob > best || (ob == best && ok < best_k)) { best = ob; best_k = ok; }
    }

    PODS_PHASE_FENCE();
    // ---- emit the (m-k) lowest then the k highest: output slot j = a + i.  The lane holds kPer consecutive slots
    // as pieces of four; the pieces are transposed among the group's four lanes first (lane bit <-> piece bit, one
    // swap per word), so that a store instruction writes 64 contiguous bytes per group instead of four 16-byte
    // pieces 64 bytes apart: the stores go past the L2 (nontemporal: no dirty lines wait for the kernel's end),
    // where nothing would merge such pieces into whole lines.
    constexpr int kPieces = kPer / 4;
    constexpr uint32_t kIdxMask = (1u << kIdxBits) - 1u;
    uint32_t piece[kPieces][4];
#pragma unroll
    for (int i = 0; i < kPer; ++i)
        piece[i / 4][i % 4] = ((a + i < kM - best_k) ? lo_w[i] : hi_w[i]) & kIdxMask;
    if constexpr (kPieces >= 2) {      // lane bit 0 <-> piece bit 0
#pragma unroll
        for (int p = 0; p < kPieces; p += 2)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const auto r = __builtin_amdgcn_permlane16_swap(piece[p][c], piece[p + 1][c], false, false);
                piece[p][c] = r[0];
                piece[p + 1][c] = r[1];
            }
    }
    if constexpr (kPieces >= 4) {      // lane bit 1 <-> piece bit 1
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const auto r = __builtin_amdgcn_permlane32_swap(piece[p][c], piece[p + 2][c], false, false);
                piece[p][c] = r[0];
                piece[p + 2][c] = r[1];
            }
    }
    static_assert(kPieces == 1 || kPieces == 2 || kPieces == 4, "16, 32 or 64 keys per lane");
    if (live) {
        int32_t* out = sel_idx + (size_t)group * kM;
        typedef int i32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int p = 0; p < kPieces; ++p) {
            // piece p now holds: 4 pieces: lane quad p's piece `quad`; 2 pieces: lane (l1, p)'s piece l0; 1: its own
            const int slot = kPieces == 4 ? 16 * p + 4 * quad : kPieces == 2 ? 8 * (2 * l1 + p) + 4 * l0 : 4 * quad;
            i32x4 w;
            w[0] = (int)piece[p][0]; w[1] = (int)piece[p][1]; w[2] = (int)piece[p][2]; w[3] = (int)piece[p][3];
            __builtin_nontemporal_store(w, reinterpret_cast<i32x4*>(out + slot));
        }
        if (sel_k != nullptr && quad == 0) __builtin_nontemporal_store(best_k, sel_k + group);
    }
}

template <int KPL>
pods_status launch_quarter(const float* rewards, int32_t B, int32_t* sel_idx, int32_t* sel_k, hipStream_t stream) {
    const unsigned grid = (unsigned)ceil_div(B, 4 * 16);   // 4 waves of 16 groups
    PODS_LAUNCH("pods_select", stream, select_quarter_kernel<KPL>, dim3(grid), dim3(256), 0, stream, rewards, B, sel_idx,
                sel_k);
    return check_launch("pods_select");
}

template <int KPL, int G>
pods_status launch_variant(const float* rewards, const uint32_t* rand_keys, int32_t B, int32_t n, int32_t m,
                           int32_t rule, int32_t* sel_idx, int32_t* sel_k, hipStream_t stream) {
    constexpr int kGroupsPerWave = kWave / G;
    const size_t per_wave = (size_t)kGroupsPerWave * group_lds_bytes(n, m, rule, G);
    int waves = 4;                                  // as many waves per workgroup as keep its LDS within 64 KiB
    while (waves > 1 && waves * per_wave > 64 * 1024) waves /= 2;
    const size_t lds = waves * per_wave;
    if (lds > 160 * 1024) return fail(PODS_ERR_UNSUPPORTED, "pods_select: LDS need %zu B", lds);
    auto kernel = select_kernel<KPL, G>;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess)
            return fail(PODS_ERR_RUNTIME, "pods_select: cannot reserve %zu B of LDS: %s", lds,
                        hipGetErrorString(e));
    }
    const unsigned grid = (unsigned)ceil_div(B, (int64_t)waves * kGroupsPerWave);
    PODS_LAUNCH("pods_select", stream, kernel, dim3(grid), dim3(waves * kWave), lds, stream, rewards, rand_keys,
                B, n, m, rule, sel_idx, sel_k);
    return check_launch("pods_select");
}

}  // namespace

pods_status launch_select(const float* rewards, const uint32_t* rand_keys, int32_t B, int32_t n, int32_t m,
                          int32_t rule, int32_t* sel_idx, int32_t* sel_k, hipStream_t stream) {
#define PODS_SELECT_VARIANT(KPL, G) \
    return launch_variant<KPL, G>(rewards, rand_keys, B, n, m, rule, sel_idx, sel_k, stream)
    // max-variance, a quarter kept, 16-byte-aligned rows: the all-in-lane kernel
    if (rule == PODS_RULE_MAXVAR && n == 4 * m && ((reinterpret_cast<uintptr_t>(rewards) | reinterpret_cast<uintptr_t>(sel_idx)) & 15) == 0) {
        if (n == 256) return launch_quarter<64>(rewards, B, sel_idx, sel_k, stream);
        if (n == 128) return launch_quarter<32>(rewards, B, sel_idx, sel_k, stream);
        if (n == 64) return launch_quarter<16>(rewards, B, sel_idx, sel_k, stream);
    }
    if (n <= 16) PODS_SELECT_VARIANT(4, 4);
    if (n <= 32) PODS_SELECT_VARIANT(8, 4);
    if (n <= 64) PODS_SELECT_VARIANT(16, 4);
    if (n <= 128) PODS_SELECT_VARIANT(32, 4);
    if (n <= 256) PODS_SELECT_VARIANT(32, 8);
    if (n <= 512) PODS_SELECT_VARIANT(32, 16);
    if (n <= 1024) PODS_SELECT_VARIANT(32, 32);
    if (n <= 2048) PODS_SELECT_VARIANT(32, 64);
    if (n <= 4096) PODS_SELECT_VARIANT(64, 64);
#undef PODS_SELECT_VARIANT
    return fail(PODS_ERR_UNSUPPORTED, "pods_select: n = %d exceeds 4096", n);
}

}  // namespace pods
