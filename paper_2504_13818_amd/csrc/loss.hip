// GRPO-PODS token loss: workspace plan, row compaction, the surrogate (clipped importance-ratio)
// step and the loss reduction.  The two contraction-heavy parts (log-sum-exp over the vocabulary,
// and the gradients) live in loss_simple.hip and loss_mfma.hip.
#include "loss.h"

namespace pods {

LossPlan plan_loss(int32_t R, int32_t T, int32_t d, int32_t V, pods_dtype dt, size_t mode) {
    LossPlan p{};
    p.ncap = (int64_t)R * T;
    p.ncap_ld = (p.ncap + kTile - 1) / kTile * kTile;
    // the matrix-core path reads 16-byte granules of the bf16 rows; its working copies pad d to a multiple of 64
    p.mfma = (dt == PODS_BF16) && (d % 8 == 0);
    p.dk = (d + 63) / 64 * 64;
    p.slots = p.mfma ? (int)(((int64_t)V + kTile - 1) / kTile) : 1;   // one partial per vocabulary tile
    p.loss_blocks = (int)ceil_div(p.ncap, 256);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes, 256);
        return o;
    };
    p.off_hdr = take(sizeof(LossHeader));
    p.off_offsets = take(sizeof(int32_t) * ((size_t)R + 1));
    p.off_rowmap = take(sizeof(int32_t) * (size_t)p.ncap_ld);
    p.off_tok = take(sizeof(int32_t) * (size_t)p.ncap_ld);
    p.off_lse = take(sizeof(float) * (size_t)p.ncap_ld);
    p.off_zy = take(sizeof(float) * (size_t)p.ncap_ld);
    p.off_g = take(sizeof(float) * (size_t)p.ncap_ld);
    p.off_coef = take(sizeof(float) * (size_t)p.ncap_ld);
    p.off_cscale = take(sizeof(float) * (size_t)p.ncap_ld);
    // matrix-core path: the exponent a token's vocabulary tiles agree on after the first forward launch
    p.off_efix = take(p.mfma ? sizeof(float) * (size_t)p.ncap_ld : 0);
    p.off_pmax = take(sizeof(float) * (size_t)p.ncap_ld * p.slots);
    p.off_psum = take(sizeof(float) * (size_t)p.ncap_ld * p.slots);
    // matrix-core path: fp16 power-of-two factor per (vocabulary tile, token) of the softmax numerators
    p.off_qscale = take(p.mfma ? sizeof(uint16_t) * (size_t)p.ncap_ld * p.slots : 0);
    p.off_losspart = take(sizeof(double) * (size_t)p.loss_blocks);
    // per-block maxima of |g|: one entry per kTile rows covers every possible block size
    p.off_gmax = take(sizeof(uint32_t) * (size_t)(p.ncap_ld / kTile));
    if (!p.mfma) {
        p.nb = p.ncap_ld; p.nblocks = 1; p.ldq = 0; p.vld = 0;
        p.off_wtt = p.off_htt = p.off_wt = p.off_ht = p.off_dz = off;
        p.total = off;
        return p;
    }
    const int64_t vround = ((int64_t)V + kTile - 1) / kTile * kTile;
    p.vld = vround;
    p.ldq = vround + kTile;
    p.off_wtt = take(2 * (size_t)p.dk * (size_t)vround);     // transposed bf16 weight, [vround/256][dk][256]
    p.off_htt = take(2 * (size_t)p.dk * (size_t)p.ncap_ld);  // transposed bf16 hidden, [ncap_ld/256][dk][256]
    p.off_wt = take(2 * (size_t)p.dk * (size_t)vround);      // fp16 weight copy [vround][dk] (zero rows past V)
    p.off_ht = take(2 * (size_t)p.dk * (size_t)p.ncap_ld);   // fp16 packed, g-scaled hidden [ncap_ld][dk]
    p.off_dz = off;                                          // q[nb][ldq] fp16, the last array
    const size_t row_bytes = 2 * (size_t)p.ldq;
    const int64_t rec_nb = p.ncap_ld < kDefaultTokenBlock ? p.ncap_ld : kDefaultTokenBlock;
    int64_t nb;
    if (mode == 0) {
        nb = rec_nb;
    } else if (mode == 1) {
        nb = kTile;
    } else {
        // the largest block (whole tiles, at most the recommended one) whose q fits in what is left;
        // one tile of rows is the minimum the entry point has already checked against
        const size_t left = mode > off ? mode - off : 0;
        nb = (int64_t)(left / row_bytes) / kTile * kTile;
        if (nb > rec_nb) nb = rec_nb;
        if (nb < kTile) nb = kTile;
    }
    p.nb = nb;
    p.nblocks = (int)ceil_div(p.ncap_ld, nb);
    p.total = align_up(off + (size_t)nb * row_bytes, 256);
    return p;
}

namespace {

// Exclusive prefix sum of the rollout lengths: offsets[i] = first packed row of rollout i.  With
// `skip`, rollouts whose advantage is non-zero are packed first (one pass for them, one for the
// rest) and the backward pass stops after them: a zero advantage makes every per-token weight of
// the rollout zero, so its gradient terms vanish identically.
__global__ __launch_bounds__(1024) void scan_lengths_kernel(const int32_t* __restrict__ lengths,
                                                            const float* __restrict__ adv, int skip,
                                                            int R, int T,
                                                            int32_t* __restrict__ offsets,
                                                            uint32_t* __restrict__ gmax_block, int ngmax,
                                                            LossHeader* __restrict__ hdr) {
    __shared__ int32_t wave_tot[16];
    __shared__ int32_t carry;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry = 0;
    for (int b = tid; b < ngmax; b += 1024) gmax_block[b] = 0u;
    __syncthreads();
    int32_t n_live = 0;
    for (int pass = 0; pass < (skip ? 2 : 1); ++pass) {
        for (int base = 0; base < R; base += 1024) {
            const int i = base + tid;
            const bool mine = i < R && (!skip || ((adv[i] != 0.0f) == (pass == 0)));
            int32_t len = 0;
            if (mine) len = rollout_len(lengths, i, T);
            int32_t x = len;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                int32_t t = __shfl_up(x, off, 64);
                if (lane >= off) x += t;
            }
            if (lane == 63) wave_tot[wave] = x;
            __syncthreads();
            int32_t before = carry;
            for (int w = 0; w < wave; ++w) before += wave_tot[w];
            if (mine) offsets[i] = before + x - len;
            __syncthreads();
            if (tid == 1023) carry = before + x;
            __syncthreads();
        }
        if (pass == 0) n_live = carry;
    }
    if (tid == 0) {
        offsets[R] = carry;
        hdr->n_valid = carry;
        hdr->n_bwd = skip ? n_live : carry;
        hdr->clipped = 0;
        hdr->bad_lengths = 0;
        hdr->bad_tokens = 0;
        hdr->gmax_bits = 0u;
        hdr->wmax_bits = 0u;
        hdr->hmax_bits = 0u;
    }
}

// Packed row -> flat position map and packed token ids; clears logp_out at padded positions.  Lengths
// outside [0, T] and token ids outside [0, V) are taken as clamped (nothing downstream can then index out
// of bounds) and counted in the header.
__global__ __launch_bounds__(256) void fill_rows_kernel(LossHeader* __restrict__ hdr,
                                                        const int32_t* __restrict__ lengths,
                                                        const int32_t* __restrict__ tokens,
                                                        const int32_t* __restrict__ offsets, int T, int V,
                                                        int32_t* __restrict__ row_map,
                                                        int32_t* __restrict__ tok,
                                                        float* __restrict__ logp_out) {
    const int i = blockIdx.x;                       // rollouts ride on grid.x (no 65535 limit)
    const int t = blockIdx.y * 256 + threadIdx.x;
    if (t == 0 && lengths != nullptr && (lengths[i] < 0 || lengths[i] > T)) atomicAdd(&hdr->bad_lengths, 1);
    if (t >= T) return;
    const int len = rollout_len(lengths, i, T);
    const int64_t flat = (int64_t)i * T + t;
    if (t < len) {
        const int p = offsets[i] + t;
        row_map[p] = (int32_t)flat;
        int y = tokens[flat];
        if ((unsigned)y >= (unsigned)V) {
            atomicAdd(&hdr->bad_tokens, 1);         // an integer count: order-independent
            y = y < 0 ? 0 : V - 1;
        }
        tok[p] = y;
    } else if (logp_out != nullptr) {
        logp_out[flat] = 0.0f;
    }
}

// d_hidden rows of padded positions, and of rollouts the backward pass skips, are zero.
__global__ __launch_bounds__(256) void zero_pad_rows_kernel(const int32_t* __restrict__ lengths,
                                                            const float* __restrict__ adv, int skip,
                                                            int T, int d,
                                                            float* __restrict__ d_hidden) {
    const int64_t flat = blockIdx.x;
    const int i = (int)(flat / T), t = (int)(flat % T);
    const int len = rollout_len(lengths, i, T);
    if (t < len && !(skip && adv[i] == 0.0f)) return;
    float* row = d_hidden + flat * d;
    if ((d & 3) == 0) {
        float4* r4 = reinterpret_cast<float4*>(row);
        for (int k = threadIdx.x; k < d / 4; k += 256) r4[k] = make_float4(0.f, 0.f, 0.f, 0.f);
    } else {
        for (int k = threadIdx.x; k < d; k += 256) row[k] = 0.0f;
    }
}

// Per valid token of the rows [row0, row_end): the forward pass's partials, one per vocabulary tile, merged
// into log-sum-exp.  64 tokens per workgroup; its 16 waves take every sixteenth partial each (coalesced across
// tokens, many loads in flight) and are merged through LDS in a fixed order.
// BASE2 = false (plain path): a partial is (m, sum exp(z - m)).
// BASE2 = true (matrix-core path): a partial is (E, sum exp(z) 2^-E) with E an integer, so partials combine
// by exact powers of two; besides lse the kernel writes, for the softmax numerators 2^14 exp(z) 2^-E kept by
// the forward pass: Eref = the largest E among the token's tiles, cscale[p] = 2^Eref exp(-lse) (below 32, at
// least 1/V: the largest logit lies within 5 binades below 2^Eref), and qscale[tile][p] = 2^(E - Eref) <= 1
// in fp16 (exact; 0 below 2^-24), so that 2^14 softmax = numerator * qscale * cscale.  Every tile that
// already used Eref, which after the first forward launch of a token block is the rule, has qscale = 1.
constexpr int kLseWaves = 16;
template <bool BASE2>
__global__ __launch_bounds__(64 * kLseWaves) void lse_kernel(const LossHeader* __restrict__ hdr,
                                                  const float* __restrict__ pmax,
                                                  const float* __restrict__ psum, int slots,
                                                  int64_t slot_stride, int64_t row0, int64_t row_end,
                                                  float* __restrict__ lse_out, float* __restrict__ cscale,
                                                  _Float16* __restrict__ qscale) {
    __shared__ float sm[kLseWaves][64], sl[kLseWaves][64];
    const int64_t n_valid = hdr->n_valid < row_end ? hdr->n_valid : row_end;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t p = row0 + (int64_t)blockIdx.x * 64 + lane;
    float M = -__builtin_huge_valf(), L = 0.0f;
    if (p < n_valid) {
#pragma unroll 4
        for (int s = w; s < slots; s += kLseWaves) {
            const float m = pmax[s * slot_stride + p];
            const float l = psum[s * slot_stride + p];
            if (m > -__builtin_huge_valf()) {
                const float Mn = fmaxf(M, m);
                if constexpr (BASE2) L = ldexpf(L, (int)fmaxf(M - Mn, -200.0f)) + ldexpf(l, (int)(m - Mn));
                else L = L * __expf(M - Mn) + l * __expf(m - Mn);
                M = Mn;
            }
        }
    }
    sm[w][lane] = M;
    sl[w][lane] = L;
    __syncthreads();
    float eref = 0.0f;
    if (p < n_valid) {   // every wave merges the waves' partial results the same way
        float Mt = sm[0][lane];
#pragma unroll
        for (int i = 1; i < kLseWaves; ++i) Mt = fmaxf(Mt, sm[i][lane]);
        float Lt = 0.0f;
#pragma unroll
        for (int i = 0; i < kLseWaves; ++i)
            if (sm[i][lane] > -__builtin_huge_valf())
                Lt += BASE2 ? ldexpf(sl[i][lane], (int)(sm[i][lane] - Mt)) : sl[i][lane] * expf(sm[i][lane] - Mt);
        if constexpr (BASE2) {
            const float lse2 = Mt + log2f(Lt);
            eref = Mt;
            if (w == 0) {
                lse_out[p] = lse2 * 0.6931471805599453f;
                cscale[p] = exp2f(eref - lse2);
            }
        } else if (w == 0) {
            lse_out[p] = Mt + logf(Lt);
        }
    }
    if constexpr (BASE2) {
        // rows past N up to the end of the last token tile are read by the gradient kernels (against zero
        // operands): their factors are zeros, not whatever the workspace held
        const int64_t tile_end = (hdr->n_valid + 255) / 256 * 256;
        if (p < n_valid) {
            for (int s = w; s < slots; s += kLseWaves) {
                const float e = pmax[s * slot_stride + p];
                qscale[s * slot_stride + p] = (_Float16)ldexpf(1.0f, (int)fmaxf(e - eref, -30.0f));
            }
        } else if (p >= hdr->n_valid && p < tile_end && p < row_end) {
            for (int s = w; s < slots; s += kLseWaves) qscale[s * slot_stride + p] = (_Float16)0.0f;
        }
    }
}

// Per valid token: the surrogate of
// Sec. 3.2: rho = exp(logp - old_logp), min[rho a, clip(rho, 1-eps, 1+eps) a], its weight
// 1/(R len_i), and g = d loss / d logp; with a reference policy, minus kl_coef times the per-token
// KL estimator (Table 2 lists the coefficient).  Block partial sums of the loss in double.
__global__ __launch_bounds__(256) void surrogate_kernel(
    LossHeader* __restrict__ hdr, const int32_t* __restrict__ row_map,
    const float* __restrict__ lse_in, const float* __restrict__ cscale, const float* __restrict__ zy, const float* __restrict__ old_logp, const float* __restrict__ ref_logp,
    float kl_coef, const float* __restrict__ adv,
    const int32_t* __restrict__ lengths, int R, int T, float clip_eps, float grad_scale,
    float* __restrict__ g_out, float* __restrict__ coef_out,
    float* __restrict__ logp_out, double* __restrict__ loss_part, int64_t row0, int64_t row_end,
    uint32_t* __restrict__ gmax_block) {
    __shared__ double red[4];
    __shared__ float redg[4], redq[4];
    __shared__ int redc[4];
    const int64_t n_valid = hdr->n_valid < row_end ? hdr->n_valid : row_end;
    const int64_t p = row0 + (int64_t)blockIdx.x * 256 + threadIdx.x;
    double contrib = 0.0;
    float gabs = 0.0f, gqabs = 0.0f;
    bool cut = false;
    if (p < n_valid) {
        const float lse = lse_in[p];
        const int flat = row_map[p];
        const int i = flat / T;
        const int len = rollout_len(lengths, i, T);
        const float a = adv[i];
        const float c = 1.0f / ((float)R * (float)len);
        const float logp = zy[p] - lse;
        const float rho = expf(logp - old_logp[flat]);
        const float lo = 1.0f - clip_eps, hi = 1.0f + clip_eps;
        float obj = fminf(rho * a, fminf(fmaxf(rho, lo), hi) * a);
        const bool inactive = (a > 0.0f && rho > hi) || (a < 0.0f && rho < lo);
        cut = inactive;
        float dobj = inactive ? 0.0f : a * rho;   // d obj / d logp
        if (ref_logp != nullptr) {
            // KL penalty, per token: exp(x) - x - 1 with x = log pi_ref(y) - log pi_theta(y)
            const float x = ref_logp[flat] - logp;
            const float em1 = expm1f(x);
            obj -= kl_coef * (em1 - x);
            dobj += kl_coef * em1;
        }
        const float gp = -c * dobj * grad_scale;
        // the matrix-core path's softmax operand lacks a per-token factor in [1, 2): it rides on the weight
        const float gq = cscale != nullptr ? gp * cscale[p] : gp;
        g_out[p] = gq;
        coef_out[p] = gp * -expm1f(logp);  // d loss / d z_y = g (1 - softmax_y)
        gabs = fabsf(gp);
        gqabs = fabsf(gq);
        if (logp_out != nullptr) logp_out[flat] = logp;
        contrib = -(double)c * (double)obj;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        contrib += __shfl_xor(contrib, off, 64);
        gabs = fmaxf(gabs, __shfl_xor(gabs, off, 64));
        gqabs = fmaxf(gqabs, __shfl_xor(gqabs, off, 64));
    }
    const int ncut = __popcll(__ballot(cut));
    if ((threadIdx.x & 63) == 0) {
        red[threadIdx.x >> 6] = contrib;
        redg[threadIdx.x >> 6] = gabs;
        redq[threadIdx.x >> 6] = gqabs;
        redc[threadIdx.x >> 6] = ncut;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        loss_part[row0 / 256 + blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
        const int nc = redc[0] + redc[1] + redc[2] + redc[3];
        if (nc > 0) atomicAdd(&hdr->clipped, nc);   // an integer count: order-independent
        const float gm = fmaxf(fmaxf(redg[0], redg[1]), fmaxf(redg[2], redg[3]));
        const float gq = fmaxf(fmaxf(redq[0], redq[1]), fmaxf(redq[2], redq[3]));
        if (gm > 0.0f) atomicMax(&hdr->gmax_bits, __float_as_uint(gm));   // maxima: order-independent
        if (gq > 0.0f) atomicMax(gmax_block, __float_as_uint(gq));
    }
}

__global__ __launch_bounds__(1024) void finalize_loss_kernel(const double* __restrict__ loss_part,
                                                             int nblocks, float* __restrict__ loss) {
    __shared__ double red[1024];
    double acc = 0.0;
    for (int b = threadIdx.x; b < nblocks; b += 1024) acc += loss_part[b];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int s = 512; s >= 1; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) loss[0] = (float)red[0];
}

}  // namespace

pods_status launch_surrogate(const LossArgs& a, const LossPlan& p, int64_t row0, int64_t nrows, int block) {
    unsigned char* ws = a.workspace;
    float* cscale = p.mfma ? reinterpret_cast<float*>(ws + p.off_cscale) : nullptr;
    if (p.mfma)
        PODS_LAUNCH("log-sum-exp", a.stream, lse_kernel<true>, dim3((unsigned)ceil_div(nrows, 64)), dim3(64 * kLseWaves), 0, a.stream,
                    reinterpret_cast<const LossHeader*>(ws + p.off_hdr), reinterpret_cast<const float*>(ws + p.off_pmax),
                    reinterpret_cast<const float*>(ws + p.off_psum), p.slots, p.ncap_ld, row0, row0 + nrows,
                    reinterpret_cast<float*>(ws + p.off_lse), cscale, reinterpret_cast<_Float16*>(ws + p.off_qscale));
    else
        PODS_LAUNCH("log-sum-exp", a.stream, lse_kernel<false>, dim3((unsigned)ceil_div(nrows, 64)), dim3(64 * kLseWaves), 0, a.stream,
                    reinterpret_cast<const LossHeader*>(ws + p.off_hdr), reinterpret_cast<const float*>(ws + p.off_pmax),
                    reinterpret_cast<const float*>(ws + p.off_psum), p.slots, p.ncap_ld, row0, row0 + nrows,
                    reinterpret_cast<float*>(ws + p.off_lse), nullptr, nullptr);
    pods_status st = check_launch("log-sum-exp");
    if (st != PODS_OK) return st;
    PODS_LAUNCH("surrogate", a.stream, surrogate_kernel, dim3((unsigned)ceil_div(nrows, 256)), dim3(256), 0, a.stream,
                reinterpret_cast<LossHeader*>(ws + p.off_hdr), reinterpret_cast<const int32_t*>(ws + p.off_rowmap),
                reinterpret_cast<const float*>(ws + p.off_lse), cscale, reinterpret_cast<const float*>(ws + p.off_zy), a.old_logp, a.ref_logp, a.kl_coef,
                a.adv, a.lengths, a.R, a.T, a.clip_eps, a.grad_scale,
                reinterpret_cast<float*>(ws + p.off_g), reinterpret_cast<float*>(ws + p.off_coef), a.logp_out,
                reinterpret_cast<double*>(ws + p.off_losspart), row0, row0 + nrows,
                reinterpret_cast<uint32_t*>(ws + p.off_gmax) + block);
    return check_launch("surrogate");
}

pods_status run_loss(const LossArgs& a) {
    const LossPlan p = plan_loss(a.R, a.T, a.d, a.V, a.dt, a.workspace_bytes);
    if (p.total > a.workspace_bytes)
        return fail(PODS_ERR_WORKSPACE, "grpo_token_loss_fwd_bwd: layout needs %zu B, workspace has %zu B", p.total,
                    a.workspace_bytes);
    unsigned char* ws = a.workspace;
    auto* hdr = reinterpret_cast<LossHeader*>(ws + p.off_hdr);
    auto* offsets = reinterpret_cast<int32_t*>(ws + p.off_offsets);
    auto* row_map = reinterpret_cast<int32_t*>(ws + p.off_rowmap);
    auto* tok = reinterpret_cast<int32_t*>(ws + p.off_tok);
    auto* loss_part = reinterpret_cast<double*>(ws + p.off_losspart);
    pods_status st;

    PODS_LAUNCH("scan_lengths", a.stream, scan_lengths_kernel, dim3(1), dim3(1024), 0, a.stream, a.lengths, a.adv,
                a.skip_zero_adv ? 1 : 0, a.R, a.T, offsets, reinterpret_cast<uint32_t*>(ws + p.off_gmax),
                (int)(p.ncap_ld / kTile), hdr);
    if ((st = check_launch("scan_lengths")) != PODS_OK) return st;
    PODS_LAUNCH("fill_rows", a.stream, fill_rows_kernel, dim3((unsigned)a.R, (unsigned)ceil_div(a.T, 256)), dim3(256),
                       0, a.stream, hdr, a.lengths, a.tokens, offsets, a.T, a.V, row_map, tok, a.logp_out);
    if ((st = check_launch("fill_rows")) != PODS_OK) return st;
    if (a.lengths != nullptr || a.skip_zero_adv) {
        PODS_LAUNCH("zero_pad_rows", a.stream, zero_pad_rows_kernel, dim3((unsigned)p.ncap), dim3(256), 0, a.stream,
                           a.lengths, a.adv, a.skip_zero_adv ? 1 : 0, a.T, a.d, a.d_hidden);
        if ((st = check_launch("zero_pad_rows")) != PODS_OK) return st;
    }

    if (p.mfma) {
        if ((st = mfma_forward_backward(a, p)) != PODS_OK) return st;
    } else {
        if ((st = simple_forward(a, p)) != PODS_OK) return st;
        if ((st = launch_surrogate(a, p, 0, p.ncap_ld, 0)) != PODS_OK) return st;
        if ((st = simple_backward(a, p)) != PODS_OK) return st;
    }
    PODS_LAUNCH("finalize_loss", a.stream, finalize_loss_kernel, dim3(1), dim3(1024), 0, a.stream, loss_part,
                       p.loss_blocks, a.loss);
    return check_launch("finalize_loss");
}

}  // namespace pods
