// Plain kernels for the GRPO-PODS token loss: fp32 arithmetic on the vector ALUs, any shape.
// They serve fp32 inputs and shapes the matrix-core path does not cover.  One workgroup per
// token (forward, d_hidden) or per vocabulary row (d_w_lm); dot products are one per wavefront.
//
// Forward : z_v = <h, W_v>, running (max, sum exp) over v, z_y captured          (log pi = z_y - lse)
// Backward: dz_v = g (1[v = y] - exp(z_v - lse));  d_hidden = sum_v dz_v W_v;  d_W_v = sum_t dz_tv h_t
#include "loss.h"

namespace pods {
namespace {

__device__ __forceinline__ float load_elem(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_elem(const uint16_t* p, size_t i) {
    return __uint_as_float((uint32_t)p[i] << 16);  // bf16 -> fp32, exact
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

constexpr int kChunk = 1024;

template <typename E>
__global__ __launch_bounds__(256) void simple_fwd_kernel(const LossHeader* __restrict__ hdr,
                                                         const int32_t* __restrict__ row_map,
                                                         const int32_t* __restrict__ tok,
                                                         const E* __restrict__ hidden,
                                                         const E* __restrict__ w, int d, int V,
                                                         float* __restrict__ pmax,
                                                         float* __restrict__ psum,
                                                         float* __restrict__ zy) {
    extern __shared__ float lds[];
    float* hs = lds;
    __shared__ float red_m[4], red_s[4];
    const int p = blockIdx.x;
    if (p >= hdr->n_valid) return;
    const size_t hrow = (size_t)row_map[p] * d;
    for (int k = threadIdx.x; k < d; k += 256) hs[k] = load_elem(hidden, hrow + k);
    __syncthreads();
    const int y = tok[p];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float M = -__builtin_huge_valf(), L = 0.0f;
    for (int v = wave; v < V; v += 4) {
        float acc = 0.0f;
        const size_t wrow = (size_t)v * d;
        for (int k = lane; k < d; k += 64) acc += hs[k] * load_elem(w, wrow + k);
        acc = wave_sum(acc);
        if (v == y && lane == 0) zy[p] = acc;
        const float Mn = fmaxf(M, acc);
        L = L * expf(M - Mn) + expf(acc - Mn);
        M = Mn;
    }
    if (lane == 0) { red_m[wave] = M; red_s[wave] = L; }
    __syncthreads();
    if (threadIdx.x == 0) {
        float Mt = fmaxf(fmaxf(red_m[0], red_m[1]), fmaxf(red_m[2], red_m[3]));
        float Lt = 0.0f;
        for (int i = 0; i < 4; ++i)
            if (red_m[i] > -__builtin_huge_valf()) Lt += red_s[i] * expf(red_m[i] - Mt);
        pmax[p] = Mt;
        psum[p] = Lt;
    }
}

template <typename E>
__global__ __launch_bounds__(256) void simple_dh_kernel(const LossHeader* __restrict__ hdr,
                                                        const int32_t* __restrict__ row_map,
                                                        const int32_t* __restrict__ tok,
                                                        const float* __restrict__ lse,
                                                        const float* __restrict__ g,
                                                        const E* __restrict__ hidden,
                                                        const E* __restrict__ w, int d, int V,
                                                        float* __restrict__ d_hidden) {
    extern __shared__ float lds[];
    float* hs = lds;            // [d]
    float* acc = lds + d;       // [d]
    float* dzs = lds + 2 * d;   // [kChunk]
    const int p = blockIdx.x;
    if (p >= hdr->n_bwd) return;
    const size_t hrow = (size_t)row_map[p] * d;
    const float gp = g[p];
    if (gp == 0.0f) {  // clipped token or zero advantage: exact zero row
        for (int k = threadIdx.x; k < d; k += 256) d_hidden[hrow + k] = 0.0f;
        return;
    }
    for (int k = threadIdx.x; k < d; k += 256) { hs[k] = load_elem(hidden, hrow + k); acc[k] = 0.0f; }
    __syncthreads();
    const int y = tok[p];
    const float ls = lse[p];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int v0 = 0; v0 < V; v0 += kChunk) {
        const int cnt = min(kChunk, V - v0);
        for (int j = wave; j < cnt; j += 4) {
            const int v = v0 + j;
            float z = 0.0f;
            const size_t wrow = (size_t)v * d;
            for (int k = lane; k < d; k += 64) z += hs[k] * load_elem(w, wrow + k);
            z = wave_sum(z);
            if (lane == 0) dzs[j] = gp * ((v == y ? 1.0f : 0.0f) - expf(z - ls));
        }
        __syncthreads();
        for (int k = threadIdx.x; k < d; k += 256) {
            float s = 0.0f;
            for (int j = 0; j < cnt; ++j) s += dzs[j] * load_elem(w, (size_t)(v0 + j) * d + k);
            acc[k] += s;
        }
        __syncthreads();
    }
    for (int k = threadIdx.x; k < d; k += 256) d_hidden[hrow + k] = acc[k];
}

template <typename E>
__global__ __launch_bounds__(256) void simple_dw_kernel(const LossHeader* __restrict__ hdr,
                                                        const int32_t* __restrict__ row_map,
                                                        const int32_t* __restrict__ tok,
                                                        const float* __restrict__ lse,
                                                        const float* __restrict__ g,
                                                        const E* __restrict__ hidden,
                                                        const E* __restrict__ w, int d, int V,
                                                        int accumulate, float* __restrict__ d_w) {
    extern __shared__ float lds[];
    float* ws = lds;            // [d]
    float* acc = lds + d;       // [d]
    float* dzs = lds + 2 * d;   // [kChunk]
    const int v = blockIdx.x;
    const int n_valid = hdr->n_bwd;
    const size_t wrow = (size_t)v * d;
    for (int k = threadIdx.x; k < d; k += 256) { ws[k] = load_elem(w, wrow + k); acc[k] = 0.0f; }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int p0 = 0; p0 < n_valid; p0 += kChunk) {
        const int cnt = min(kChunk, n_valid - p0);
        for (int j = wave; j < cnt; j += 4) {
            const int p = p0 + j;
            const float gp = g[p];
            float dz = 0.0f;
            if (gp != 0.0f) {
                const size_t hrow = (size_t)row_map[p] * d;
                float z = 0.0f;
                for (int k = lane; k < d; k += 64) z += ws[k] * load_elem(hidden, hrow + k);
                z = wave_sum(z);
                dz = gp * ((v == tok[p] ? 1.0f : 0.0f) - expf(z - lse[p]));
            }
            if (lane == 0) dzs[j] = dz;
        }
        __syncthreads();
        for (int k = threadIdx.x; k < d; k += 256) {
            float s = 0.0f;
            for (int j = 0; j < cnt; ++j) {
                const float dz = dzs[j];
                if (dz != 0.0f) s += dz * load_elem(hidden, (size_t)row_map[p0 + j] * d + k);
            }
            acc[k] += s;
        }
        __syncthreads();
    }
    for (int k = threadIdx.x; k < d; k += 256) d_w[wrow + k] = accumulate ? d_w[wrow + k] + acc[k] : acc[k];
}

template <typename K>
pods_status reserve_lds(K kernel, size_t bytes, const char* what) {
    if (bytes > 160 * 1024) return fail(PODS_ERR_UNSUPPORTED, "%s: needs %zu B of LDS", what, bytes);
    if (bytes > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e != hipSuccess) return fail(PODS_ERR_RUNTIME, "%s: %s", what, hipGetErrorString(e));
    }
    return PODS_OK;
}

template <typename E>
pods_status forward_t(const LossArgs& a, const LossPlan& p) {
    unsigned char* ws = a.workspace;
    const size_t lds = sizeof(float) * (size_t)a.d;
    auto kernel = simple_fwd_kernel<E>;
    pods_status st = reserve_lds(kernel, lds, "token loss forward (plain)");
    if (st != PODS_OK) return st;
    PODS_LAUNCH("token loss forward (plain)", a.stream, kernel, dim3((unsigned)p.ncap), dim3(256), lds, a.stream,
                       reinterpret_cast<const LossHeader*>(ws + p.off_hdr),
                       reinterpret_cast<const int32_t*>(ws + p.off_rowmap),
                       reinterpret_cast<const int32_t*>(ws + p.off_tok),
                       static_cast<const E*>(a.hidden), static_cast<const E*>(a.w_lm), a.d, a.V,
                       reinterpret_cast<float*>(ws + p.off_pmax),
                       reinterpret_cast<float*>(ws + p.off_psum),
                       reinterpret_cast<float*>(ws + p.off_zy));
    return check_launch("token loss forward (plain)");
}

template <typename E>
pods_status backward_t(const LossArgs& a, const LossPlan& p) {
    unsigned char* ws = a.workspace;
    const size_t lds = sizeof(float) * (2 * (size_t)a.d + kChunk);
    auto* hdr = reinterpret_cast<const LossHeader*>(ws + p.off_hdr);
    auto* row_map = reinterpret_cast<const int32_t*>(ws + p.off_rowmap);
    auto* tok = reinterpret_cast<const int32_t*>(ws + p.off_tok);
    auto* lse = reinterpret_cast<const float*>(ws + p.off_lse);
    auto* g = reinterpret_cast<const float*>(ws + p.off_g);
    auto kdh = simple_dh_kernel<E>;
    auto kdw = simple_dw_kernel<E>;
    pods_status st = reserve_lds(kdh, lds, "token loss d_hidden (plain)");
    if (st != PODS_OK) return st;
    st = reserve_lds(kdw, lds, "token loss d_w_lm (plain)");
    if (st != PODS_OK) return st;
    PODS_LAUNCH("token loss d_hidden (plain)", a.stream, kdh, dim3((unsigned)p.ncap), dim3(256), lds, a.stream, hdr, row_map, tok, lse,
                       g, static_cast<const E*>(a.hidden), static_cast<const E*>(a.w_lm), a.d, a.V,
                       a.d_hidden);
    if ((st = check_launch("token loss d_hidden (plain)")) != PODS_OK) return st;
    PODS_LAUNCH("token loss d_w_lm (plain)", a.stream, kdw, dim3((unsigned)a.V), dim3(256), lds, a.stream, hdr, row_map, tok, lse, g,
                       static_cast<const E*>(a.hidden), static_cast<const E*>(a.w_lm), a.d, a.V,
                       a.accumulate_d_w ? 1 : 0, a.d_w_lm);
    return check_launch("token loss d_w_lm (plain)");
}

}  // namespace

pods_status simple_forward(const LossArgs& a, const LossPlan& p) {
    return a.dt == PODS_F32 ? forward_t<float>(a, p) : forward_t<uint16_t>(a, p);
}
pods_status simple_backward(const LossArgs& a, const LossPlan& p) {
    return a.dt == PODS_F32 ? backward_t<float>(a, p) : backward_t<uint16_t>(a, p);
}

}  // namespace pods
