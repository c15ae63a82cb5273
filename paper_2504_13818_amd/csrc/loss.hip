// GRPO-PODS token loss: workspace plan, row compaction, the surrogate (clipped importance-ratio)
// step and the loss reduction.  The two contraction-heavy parts (log-sum-exp over the vocabulary,
// and the gradients) live in loss_simple.hip and loss_mfma.hip.
#include "loss.h"

namespace pods {

LossPlan plan_loss(int32_t R, int32_t T, int32_t d, int32_t V, pods_dtype dt, size_t mode) {
    LossPlan p{};
    p.ncap = (int64_t)R * T;
    p.ncap_ld = (p.ncap + kTile - 1) / kTile * kTile;
    p.mfma = (dt == PODS_BF16) && (d % 64 == 0);
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
    p.off_pmax = take(sizeof(float) * (size_t)p.ncap_ld * p.slots);
    p.off_psum = take(sizeof(float) * (size_t)p.ncap_ld * p.slots);
    p.off_losspart = take(sizeof(double) * (size_t)p.loss_blocks);
    if (!p.mfma) {
        p.vc = 0; p.nchunks = 0; p.ldq = 0; p.vld = 0; p.vld_t = 0;
        p.off_wtt = p.off_htt = p.off_wt = p.off_ht = p.off_dz = off;
        p.total = off;
        return p;
    }
    const int64_t vround = ((int64_t)V + kTile - 1) / kTile * kTile;
    p.vld_t = vround;
    p.off_wtt = take(2 * (size_t)d * (size_t)vround);        // transposed fp16 weight, [vround/256][d][256]
    p.off_htt = take(2 * (size_t)d * (size_t)p.ncap_ld);     // transposed fp16 hidden, [ncap_ld/256][d][256]
    // Fixed part: fp16 weight copy (vld rows, at most vround + vc) and fp16 packed, g-scaled hidden.
    auto total_for = [&](int vc, LossPlan& q) {
        size_t o = off;
        auto tk = [&](size_t bytes) { size_t r = o; o = align_up(o + bytes, 256); return r; };
        q.vc = vc;
        q.nchunks = (int)ceil_div(vround, vc);
        q.vld = (int64_t)q.nchunks * vc;
        q.off_wt = tk(2 * (size_t)d * (size_t)q.vld);
        q.off_ht = tk(2 * (size_t)d * (size_t)p.ncap_ld);
        q.ldq = vc + kTile;
        q.off_dz = tk(2 * (size_t)p.ncap_ld * (size_t)q.ldq);
        q.total = o;
    };
    int vc;
    if (mode == 0) {
        // The d_w_lm launch of a chunk has (vc / 256) x ceil(d / 256) tiles of equal, long duration: pick
        // the chunk, near the default, whose tile count fills whole rounds of the 256 CUs best
        // (d = 3584: 36 x 14 = 504 tiles, not 32 x 14 = 448).
        const int64_t nd = ((int64_t)d + kTile - 1) / kTile;
        const int64_t nv0 = kDefaultVocabChunk / kTile;
        int64_t best_nv = nv0;
        double best_eff = -1.0;
        for (int64_t nv = nv0 - nv0 / 4; nv <= nv0 + nv0 / 4; ++nv) {
            const int64_t tiles = nv * nd;
            const double eff = (double)tiles / (double)((tiles + 255) / 256 * 256);
            const bool closer = llabs(nv - nv0) < llabs(best_nv - nv0);
            if (eff > best_eff + 1e-9 || (eff > best_eff - 1e-9 && closer)) { best_eff = eff; best_nv = nv; }
        }
        const int64_t want = best_nv * kTile;
        vc = (int)(vround < want ? vround : want);
    } else if (mode == 1) {
        vc = kTile;
    } else {
        // A caller-given workspace at least as large as the recommendation gets the recommended chunk.
        // Below it: the largest chunk (at most four default chunks) whose layout fits.  The layout is not
        // monotone in the chunk (the fp16 weight copy has nchunks * vc rows, which can grow when vc
        // shrinks), so every candidate is laid out and checked; vc = kTile is the minimum the entry point
        // has already checked against.
        const LossPlan rec = plan_loss(R, T, d, V, dt, 0);
        if (rec.total <= mode) return rec;
        const int64_t cap = vround < 4 * kDefaultVocabChunk ? vround : 4 * kDefaultVocabChunk;
        vc = kTile;
        LossPlan q = p;
        for (int64_t c = cap; c > kTile; c -= kTile) {
            total_for((int)c, q);
            if (q.total <= mode) { vc = (int)c; break; }
        }
    }
    total_for(vc, p);
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
                                                            LossHeader* __restrict__ hdr) {
    __shared__ int32_t wave_tot[16];
    __shared__ int32_t carry;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry = 0;
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

// Per valid token: combine the forward partials into log-sum-exp, then the surrogate of
// Sec. 3.2: rho = exp(logp - old_logp), min[rho a, clip(rho, 1-eps, 1+eps) a], its weight
// 1/(R len_i), and g = d loss / d logp; with a reference policy, minus kl_coef times the per-token
// KL estimator (Table 2 lists the coefficient).  Block partial sums of the loss in double.
__global__ __launch_bounds__(256) void surrogate_kernel(
    LossHeader* __restrict__ hdr, const int32_t* __restrict__ row_map,
    const float* __restrict__ pmax, const float* __restrict__ psum, int slots, int64_t slot_stride,
    const float* __restrict__ zy, const float* __restrict__ old_logp, const float* __restrict__ ref_logp,
    float kl_coef, const float* __restrict__ adv,
    const int32_t* __restrict__ lengths, int R, int T, float clip_eps, float grad_scale,
    float* __restrict__ lse_out, float* __restrict__ g_out, float* __restrict__ coef_out,
    float* __restrict__ logp_out, double* __restrict__ loss_part) {
    __shared__ double red[4];
    __shared__ float redg[4];
    __shared__ int redc[4];
    const int n_valid = hdr->n_valid;
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    double contrib = 0.0;
    float gabs = 0.0f;
    bool cut = false;
    if (p < n_valid) {
        float M = -__builtin_huge_valf();
        for (int s = 0; s < slots; ++s) M = fmaxf(M, pmax[s * slot_stride + p]);
        float L = 0.0f;
        for (int s = 0; s < slots; ++s) {
            const float ms = pmax[s * slot_stride + p];
            if (ms > -__builtin_huge_valf()) L += psum[s * slot_stride + p] * expf(ms - M);
        }
        const float lse = M + logf(L);
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
        lse_out[p] = lse;
        g_out[p] = gp;
        coef_out[p] = gp * -expm1f(logp);  // d loss / d z_y = g (1 - softmax_y)
        gabs = fabsf(gp);
        if (logp_out != nullptr) logp_out[flat] = logp;
        contrib = -(double)c * (double)obj;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        contrib += __shfl_xor(contrib, off, 64);
        gabs = fmaxf(gabs, __shfl_xor(gabs, off, 64));
    }
    const int ncut = __popcll(__ballot(cut));
    if ((threadIdx.x & 63) == 0) {
        red[threadIdx.x >> 6] = contrib;
        redg[threadIdx.x >> 6] = gabs;
        redc[threadIdx.x >> 6] = ncut;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        loss_part[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
        const int nc = redc[0] + redc[1] + redc[2] + redc[3];
        if (nc > 0) atomicAdd(&hdr->clipped, nc);   // an integer count: order-independent
        const float gm = fmaxf(fmaxf(redg[0], redg[1]), fmaxf(redg[2], redg[3]));
        if (gm > 0.0f) atomicMax(&hdr->gmax_bits, __float_as_uint(gm));  // a max: order-independent
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
    auto* lse = reinterpret_cast<float*>(ws + p.off_lse);
    auto* zy = reinterpret_cast<float*>(ws + p.off_zy);
    auto* g = reinterpret_cast<float*>(ws + p.off_g);
    auto* coef = reinterpret_cast<float*>(ws + p.off_coef);
    auto* pmax = reinterpret_cast<float*>(ws + p.off_pmax);
    auto* psum = reinterpret_cast<float*>(ws + p.off_psum);
    auto* loss_part = reinterpret_cast<double*>(ws + p.off_losspart);
    pods_status st;

    PODS_LAUNCH("scan_lengths", a.stream, scan_lengths_kernel, dim3(1), dim3(1024), 0, a.stream, a.lengths, a.adv,
                       a.skip_zero_adv ? 1 : 0, a.R, a.T, offsets, hdr);
    if ((st = check_launch("scan_lengths")) != PODS_OK) return st;
    PODS_LAUNCH("fill_rows", a.stream, fill_rows_kernel, dim3((unsigned)a.R, (unsigned)ceil_div(a.T, 256)), dim3(256),
                       0, a.stream, hdr, a.lengths, a.tokens, offsets, a.T, a.V, row_map, tok, a.logp_out);
    if ((st = check_launch("fill_rows")) != PODS_OK) return st;
    if (a.lengths != nullptr || a.skip_zero_adv) {
        PODS_LAUNCH("zero_pad_rows", a.stream, zero_pad_rows_kernel, dim3((unsigned)p.ncap), dim3(256), 0, a.stream,
                           a.lengths, a.adv, a.skip_zero_adv ? 1 : 0, a.T, a.d, a.d_hidden);
        if ((st = check_launch("zero_pad_rows")) != PODS_OK) return st;
    }

    st = p.mfma ? mfma_forward(a, p) : simple_forward(a, p);
    if (st != PODS_OK) return st;

    PODS_LAUNCH("surrogate", a.stream, surrogate_kernel, dim3((unsigned)p.loss_blocks), dim3(256), 0, a.stream, hdr,
                       row_map, pmax, psum, p.slots, p.ncap_ld, zy, a.old_logp, a.ref_logp, a.kl_coef, a.adv, a.lengths, a.R,
                       a.T, a.clip_eps, a.grad_scale, lse, g, coef, a.logp_out, loss_part);
    if ((st = check_launch("surrogate")) != PODS_OK) return st;
    PODS_LAUNCH("finalize_loss", a.stream, finalize_loss_kernel, dim3(1), dim3(1024), 0, a.stream, loss_part,
                       p.loss_blocks, a.loss);
    if ((st = check_launch("finalize_loss")) != PODS_OK) return st;

    return p.mfma ? mfma_backward(a, p) : simple_backward(a, p);
}

}  // namespace pods
