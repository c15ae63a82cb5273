// GRPO-PODS token loss (objective of Sec. 3.2): host-side plan and the kernel families behind
// grpo_token_loss_fwd_bwd.
//
// Notation: R kept rollouts, T padded length, N = sum of lengths (valid token positions, known
// only on the device), d hidden size, V vocabulary.  Valid positions are packed into rows
// p = 0..N-1 (rollout-major; when zero-advantage rollouts are skipped, the others first); every
// kernel is launched for the worst case R*T rows and returns early for rows at or beyond N.
#pragma once

#include "common.h"

namespace pods {

struct LossArgs {
    const void* hidden;
    const void* w_lm;
    const int32_t* tokens;
    const float* old_logp;
    const float* ref_logp;   // log pi_ref(y) for the KL penalty, or null
    float kl_coef;
    const float* adv;
    const int32_t* lengths;
    int32_t R, T, d, V;
    pods_dtype dt;
    float clip_eps, grad_scale;
    float* loss;
    float* logp_out;
    float* d_hidden;
    float* d_w_lm;
    bool accumulate_d_w;   // d_w_lm += gradient instead of d_w_lm = gradient
    bool skip_zero_adv;    // rollouts with a_i == 0 take no part in the backward pass
    unsigned char* workspace;
    size_t workspace_bytes;
    hipStream_t stream;
};

// Device header at the start of the workspace.  Its first 64 bytes are the public pods_loss_report.
struct LossHeader {
    int32_t n_valid;       // N
    int32_t n_bwd;         // packed rows the backward pass covers: N, or only the rows of rollouts with
                           // a non-zero advantage (they are packed first when those are skipped)
    int32_t clipped;       // valid tokens whose clipped term is the selected one (no gradient)
    int32_t bad_lengths;   // rollouts whose length lay outside [0, T] (taken as clamped)
    int32_t bad_tokens;    // valid positions whose token id lay outside [0, V) (taken as clamped)
    uint32_t gmax_bits;    // bit patterns of max_t |g_t|, max |W_lm|, max |h| over valid rows
    uint32_t wmax_bits;    // (non-negative floats order as integers; the last two on the bf16
    uint32_t hmax_bits;    //  matrix-core path only)
    int32_t pad[56];
};
static_assert(sizeof(LossHeader) == 256, "the header is one 256-byte slot of the workspace");
static_assert(sizeof(pods_loss_report) == 64, "the report is the head of the header");

// Valid prefix length of rollout i: lengths[i] clamped to [0, T] (T when lengths is null).
__device__ __forceinline__ int rollout_len(const int32_t* lengths, int i, int T) {
    if (lengths == nullptr) return T;
    const int len = lengths[i];
    return len < 0 ? 0 : (len > T ? T : len);
}

// 2^(target - floor(log2 x)) for the float with bit pattern `bits` (x >= 0): brings x into
// [2^target, 2^(target+1)).  1 for x = 0; the exponent of the result is kept inside [-100, 100], and a
// non-finite x is treated as the largest finite binade.
__device__ __forceinline__ int float_exponent(uint32_t bits) {
    const int e = (int)((bits >> 23) & 0xFFu);
    return (e == 0 ? 1 : (e == 255 ? 254 : e)) - 127;
}
__device__ __forceinline__ float pow2(int e) {
    e = e < -100 ? -100 : (e > 100 ? 100 : e);
    return __uint_as_float((uint32_t)(e + 127) << 23);
}

// Power-of-two range scales of the two fp16 gradient operands (exact for bf16 data that stays in fp16's
// normal range, i.e. within 2^-22 of the largest element):
//   W16 = fp16(s_w W),  s_w brings max |W| into [2^8, 2^9)
//   H16 = fp16(s_h g_t h_t),  s_h brings (max |g|) (max |h|) below 2^14 (and at least to 2^12); the
//         maximum of |g| is taken per token block, whose d_w_lm contribution is scaled back by 1 / s_h
__device__ __forceinline__ float w_range_scale(const LossHeader* hdr) {
    if (hdr->wmax_bits == 0u) return 1.0f;
    return pow2(8 - float_exponent(hdr->wmax_bits));
}
__device__ __forceinline__ float g_range_scale(uint32_t gmax_bits, const LossHeader* hdr) {
    if (gmax_bits == 0u || hdr->hmax_bits == 0u) return 1.0f;
    return pow2(12 - float_exponent(gmax_bits) - float_exponent(hdr->hmax_bits));
}

// Fixed power-of-two scale of the fp16 softmax operand of the two gradient contractions.
constexpr float kQScale = 16384.0f;  // q = kQScale softmax (0 at v = y): 0 <= q <= 2^14

constexpr int kTile = 256;          // token / vocab / hidden tile edge of the matrix-core kernels
constexpr int kDefaultVocabChunk = 8192;    // vocabulary columns per forward launch of the matrix-core path
constexpr int kDefaultTokenBlock = 32768;   // packed token rows whose softmax numerators are held at a time

struct LossPlan {
    int64_t ncap;     // R*T
    int64_t ncap_ld;  // ncap rounded up to kTile: rows of the per-token arrays
    bool mfma;        // bf16 inputs with d % 8 == 0 take the matrix-core path
    int slots;        // forward partial slots per token (one per vocabulary tile on the matrix-core path)
    int64_t nb;       // matrix-core path: packed token rows per block (multiple of kTile); the block's softmax
                      // numerators q[nb][ldq] are the only [tokens, vocabulary]-shaped array that ever exists
    int nblocks;      // token blocks = ceil(ncap_ld / nb); 1 on the plain path
    int64_t ldq;      // row pitch of q in elements: the padded vocabulary plus one tile, so rows do not sit a
                      // power of two apart
    int64_t vld;      // V rounded up to kTile: rows of the fp16 weight copy, columns of the transposed one
    int dk;           // d rounded up to 64: the contraction length of the working copies (zero beyond d)
    int loss_blocks;
    size_t off_hdr, off_gmax, off_offsets, off_rowmap, off_tok, off_lse, off_zy, off_g, off_coef, off_cscale, off_efix, off_pmax,
        off_psum, off_qscale, off_losspart, off_wtt, off_htt, off_wt, off_ht, off_dz, total;
};

// mode 0: recommended size; mode 1: minimum size; otherwise `mode` is the number of bytes
// available and the largest token block (up to the recommended one) that fits is chosen.
LossPlan plan_loss(int32_t R, int32_t T, int32_t d, int32_t V, pods_dtype dt, size_t mode);

pods_status run_loss(const LossArgs& a);

// Surrogate step (loss.hip) for the packed rows [row0, row0 + nrows): log-sum-exp from the forward partials,
// the clipped objective, g, the y-logit coefficient, log-probs, loss partial sums; max |g| of the rows goes to
// entry `block` of the per-block maxima.
pods_status launch_surrogate(const LossArgs& a, const LossPlan& p, int64_t row0, int64_t nrows, int block);

// Plain kernels (fp32 arithmetic, any shape): loss_simple.hip
pods_status simple_forward(const LossArgs& a, const LossPlan& p);
pods_status simple_backward(const LossArgs& a, const LossPlan& p);

// Matrix-core kernels (bf16 inputs): loss_mfma.hip.  Forward, surrogate and backward, token block by
// token block.
pods_status mfma_forward_backward(const LossArgs& a, const LossPlan& p);

}  // namespace pods
