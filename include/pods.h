/* pods.h - C ABI of the PODS hot path on one AMD MI355X (gfx950).
 *
 * PODS ("Policy Optimization with Down-Sampling") generates n rollouts per prompt, keeps m < n
 * of them by a down-sampling rule, and runs the GRPO policy update on the kept ones only.
 * This library is the device side of that update's data-parallel hot path:
 *
 *   pods_select               max-variance down-sampling, batched over prompt groups
 *                             (Sec. 3.3: definition, Lemma 3.1, Algorithm 2, Theorem 1)
 *   pods_downsample           the same selection step under any of the paper's rules: max-variance,
 *                             max-reward, percentile, random (Sec. 3.2)
 *   pods_gather_rows          the kept rollouts' records, concatenated over prompts (Sec. 3.2)
 *   pods_downsample_gather    down-sampling, advantages and the records' copy in one launch
 *                             (Algorithm 1, steps 3-4)
 *   pods_advantage            group-normalised advantages over the kept rollouts (Sec. 3.2)
 *   pods_advantage_before     the "Before" variant: statistics from all n rollouts of the group
 *                             (App. "On Advantage Normalization")
 *   grpo_token_loss_fwd_bwd   the GRPO-PODS objective L_PODS(theta, S) (Sec. 3.2, and L_GRPO in
 *                             Sec. 3.1) taken through the policy's last layer: the lm_head
 *                             projection, log-softmax, importance ratio, clipped surrogate, and
 *                             the gradients w.r.t. the hidden states and the lm_head weight,
 *                             without ever holding the [tokens, vocab] logits in memory.
 *                             (_accumulate: d_w_lm +=; _kl: with a KL penalty; _ex: every option)
 *
 * Conventions for every entry point
 *   - Every pointer is a DEVICE pointer unless marked "host".  `stream` is a hipStream_t passed
 *     as void* (NULL = the default stream).  Calls only enqueue work on `stream`: no host
 *     synchronisation, no host read of device data, no device allocation.
 *   - The caller owns every buffer, including the workspace.  The library keeps no device memory
 *     and no state between calls, with two stated exceptions: the built-in working array of
 *     grpo_token_loss_fwd_bwd_static, and the benchmark hooks of pods_profile.h.  Outputs are
 *     overwritten, inputs are never modified.  Arrays are dense, row-major, 0-based indices (the paper is 1-based).
 *   - The return value is a pods_status; nothing throws or aborts across this boundary.
 *     Conditions the host can see (null pointers, non-positive sizes, m > n, a workspace that
 *     is too small, a shape no kernel variant covers) are reported before anything is launched.
 *     Conditions that live in device data cannot be reported by a call that never waits for the
 *     device.  The token loss takes a length outside [0, T] and a token id outside [0, V) as
 *     clamped to the nearest valid value, so that nothing is read or written out of bounds, and
 *     counts them in its report (grpo_token_loss_report); its results are then meaningless.  NaN or
 *     infinite rewards give undefined selections and advantages (but no out-of-bounds access);
 *     pods_check_rewards is the optional launch that finds them.
 *   - pods_last_error() returns a host string describing the last failure on this thread.
 */
#ifndef PODS_H_
#define PODS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PODS_OK = 0,
    PODS_ERR_INVALID_ARG = 1,  /* null pointer, size <= 0, m > n, negative clip_eps, ...        */
    PODS_ERR_UNSUPPORTED = 2,  /* a shape outside what the kernels cover (limits stated below)  */
    PODS_ERR_WORKSPACE = 3,    /* workspace pointer null / misaligned / smaller than required   */
    PODS_ERR_RUNTIME = 4       /* a HIP launch failed; pods_last_error() has the HIP message    */
} pods_status;

/* The last member of each enum only widens it to 32 bits, so that any int a caller passes is a value the
 * library may inspect and reject; it is not a value to pass. */
typedef enum { PODS_F32 = 0, PODS_BF16 = 1, PODS_DTYPE_INT32_ = 0x7fffffff } pods_dtype;

/* Max-variance down-sampling D_maxv (Sec. 3.3).  For each of B prompt groups, chooses the m of
 * n rewards whose (population) variance is maximal.  By Lemma 3.1 the optimum is the (m-k)
 * lowest plus the k highest rewards of the sorted order for some k; Algorithm 2 scans k = 0..m
 * and keeps a candidate only when its variance is strictly larger, so the smallest maximising k
 * wins; Theorem 1's prefix sums make each candidate O(1).
 *
 * Tie rule (the paper leaves it open): the sort order is ascending (reward, index), -0.0 equal
 * to +0.0.  Hence among equal rewards the low part takes the lowest indices, the high part the
 * highest.  Candidate variances are compared as m*sum(x^2) - (sum x)^2 in double precision; a
 * candidate whose multiset equals the previous candidate's is never preferred.
 *
 *   rewards  [B, n] float32, in
 *   sel_idx  [B, m] int32, out: ind[0 .. m-k) followed by ind[n-k .. n) of the sorted order
 *   sel_k    [B]    int32, out: the chosen k; may be NULL
 *   1 <= m <= n <= 4096 (PODS_ERR_UNSUPPORTED above that).  m == n is accepted (k = 0).
 */
pods_status pods_select(const float* rewards, int32_t B, int32_t n, int32_t m,
                        int32_t* sel_idx, int32_t* sel_k, void* stream);

/* Optional argument check for the calls above and below that read rewards: counts the rewards that are
 * NaN or infinite, which Sec. 3.2's rules and advantages define nothing for.  One extra launch on
 * `stream`; the caller reads the report when it next synchronises.
 *
 *   rewards  [B, n] float32, in
 *   report   [2] int32, out (device): report[0] = number of non-finite rewards, report[1] = flat
 *            index b*n + i of the first one, or -1.  B*n < 2^31.
 */
pods_status pods_check_rewards(const float* rewards, int32_t B, int32_t n, int32_t* report, void* stream);

/* The down-sampling step of the PODS framework (Algorithm 1, step 3) under a chosen rule
 * (Sec. 3.2 for the first three, Sec. 3.3 for max-variance).  All rules read positions of the
 * group's order ascending by (key, index), where the key is the reward (-0.0 equal to +0.0) or,
 * for PODS_RULE_RAND, the caller's random key:
 *
 *   PODS_RULE_MAXVAR  exactly pods_select.
 *   PODS_RULE_MAXR    D_maxr, the m highest rewards: positions n-m .. n-1 (so among equal rewards at
 *                     the cut, the highest indices are kept).  sel_k receives m.
 *   PODS_RULE_PERC    D_perc, the (j - 1/2)/m quantiles, j = 1..m.  The paper names no order
 *                     statistic for a quantile q; taken here as position floor(q n), i.e.
 *                     floor((2j - 1) n / (2m)) in integers.  sel_k receives -1.
 *   PODS_RULE_RAND    D_rand, m indices uniformly without replacement.  The library draws nothing:
 *                     the caller passes one 32-bit key per rollout (independent uniform draws) and
 *                     the m smallest (key, index) are kept; rewards may be NULL.  sel_k receives -1.
 *
 *   rewards    [B, n] float32, in (unused and may be NULL for PODS_RULE_RAND)
 *   rand_keys  [B, n] uint32, in (PODS_RULE_RAND only; NULL otherwise)
 *   sel_idx    [B, m] int32, out, in the order of the positions listed above
 *   sel_k      [B]    int32, out, may be NULL
 *   1 <= m <= n <= 4096.
 */
typedef enum {
    PODS_RULE_MAXVAR = 0,
    PODS_RULE_MAXR = 1,
    PODS_RULE_PERC = 2,
    PODS_RULE_RAND = 3,
    PODS_RULE_INT32_ = 0x7fffffff
} pods_rule;

pods_status pods_downsample(const float* rewards, const uint32_t* rand_keys, int32_t B, int32_t n,
                            int32_t m, pods_rule rule, int32_t* sel_idx, int32_t* sel_k, void* stream);

/* Advantages over the kept rollouts (Sec. 3.2): a_{S,i} = (r_i - mu_S) / (sigma_S + std_eps)
 * with mu_S, sigma_S the mean and population standard deviation of the m kept rewards, so each
 * group's advantages sum to zero.  A group whose kept rewards are all equal gets exactly 0.
 *
 *   rewards  [B, n] float32, in
 *   sel_idx  [B, m] int32, in (values in [0, n))
 *   adv      [B, m] float32, out, in sel_idx's order; read as adv[R], R = B*m, by the loss
 *   1 <= m <= n, m <= 4096.
 */
pods_status pods_advantage(const float* rewards, const int32_t* sel_idx, int32_t B, int32_t n,
                           int32_t m, float std_eps, float* adv, void* stream);

/* "Before" normalisation (App. "On Advantage Normalization"): a_i = (r_i - mu) / (sigma + std_eps)
 * for the kept i, with mu and the population sigma taken over all n rollouts of the group, i.e.
 * before down-sampling; a group's kept advantages then need not sum to zero.  A group whose n
 * rewards are all equal gets exactly 0.  Arguments as pods_advantage.
 */
pods_status pods_advantage_before(const float* rewards, const int32_t* sel_idx, int32_t B, int32_t n,
                                  int32_t m, float std_eps, float* adv, void* stream);

/* The kept rollouts of every prompt, concatenated (Sec. 3.2: the same procedure per prompt, then
 * the down-sampled rollouts are concatenated; Algorithm 1 steps 3-4).  Copies one fixed-size record
 * per kept rollout (its token ids, old log-probs, length, ...) into the [R, ...] layout the token
 * loss reads:  dst[(b*m + j) * row_bytes ...] = src[(b*n + sel_idx[b, j]) * row_bytes ...].
 *
 *   src        [B, n, row_bytes] bytes, in
 *   sel_idx    [B, m] int32, in (values in [0, n); not checked)
 *   dst        [B*m, row_bytes] bytes, out; must not overlap src
 *   row_bytes  > 0.  Rows are copied 16 bytes per lane when src, dst and row_bytes are multiples
 *              of 16, 4 bytes per lane when they are multiples of 4, else byte by byte.
 */
pods_status pods_gather_rows(const void* src, const int32_t* sel_idx, int32_t B, int32_t n, int32_t m,
                             size_t row_bytes, void* dst, void* stream);

/* Steps 3 and 4 of Algorithm 1 in one launch: pods_downsample, then pods_advantage (or
 * pods_advantage_before), then pods_gather_rows for each of up to PODS_MAX_RECORDS record arrays,
 * with the results of each step exactly as those calls define them.  One workgroup serves one
 * prompt group, so this is the call for a training step's handful of prompts with long records;
 * for very many small groups without records the separate pods_downsample is the faster selector.
 *
 *   rewards         [B, n] float32, in (needed by every rule: the advantages read it)
 *   rand_keys       [B, n] uint32, in (PODS_RULE_RAND only; NULL otherwise)
 *   stats_from_all  0: statistics of the m kept rewards; non-zero: of all n ("Before")
 *   records         HOST array of num_records descriptors; each src is [B, n, row_bytes] bytes on
 *                   the device, each dst [B*m, row_bytes] bytes on the device, not overlapping any
 *                   src; the array is read during the call and need not outlive it
 *   num_records     0 .. PODS_MAX_RECORDS
 *   sel_idx         [B, m] int32, out;  sel_k [B] int32, out, may be NULL;  adv [B, m] float32, out
 *   1 <= m <= n <= 1024 (PODS_ERR_UNSUPPORTED above that: use the separate calls).
 */
enum { PODS_MAX_RECORDS = 8 };
typedef struct {
    const void* src;
    void* dst;
    size_t row_bytes;
} pods_record;

pods_status pods_downsample_gather(const float* rewards, const uint32_t* rand_keys, int32_t B, int32_t n,
                                   int32_t m, pods_rule rule, float std_eps, int32_t stats_from_all,
                                   const pods_record* records, int32_t num_records, int32_t* sel_idx,
                                   int32_t* sel_k, float* adv, void* stream);

/* Bytes of workspace grpo_token_loss_fwd_bwd wants for these sizes (a recommendation: any
 * workspace of at least grpo_token_loss_workspace_min_bytes works; below the recommendation the
 * call works through the tokens in smaller blocks, above it nothing changes).  Returns 0 for invalid
 * sizes. */
size_t grpo_token_loss_workspace_bytes(int32_t R, int32_t T, int32_t d, int32_t V, pods_dtype dt);
size_t grpo_token_loss_workspace_min_bytes(int32_t R, int32_t T, int32_t d, int32_t V, pods_dtype dt);
/* Bytes of a workspace of workspace_bytes that a call with these sizes lays its working arrays out in
 * (never more than workspace_bytes; host arithmetic only).  Returns 0 for invalid sizes or a
 * workspace below the minimum. */
size_t grpo_token_loss_workspace_used_bytes(int32_t R, int32_t T, int32_t d, int32_t V, pods_dtype dt,
                                            size_t workspace_bytes);

/* GRPO-PODS token loss, forward and backward (objective of Sec. 3.2; with S = all rollouts it
 * is L_GRPO of Sec. 3.1).  For R kept rollouts (R = B*m over a batch of prompts, concatenated
 * as Sec. 3.2 prescribes), with logits z = W_lm h, log pi(y) = z_y - logsumexp(z),
 * rho = exp(log pi(y) - old_logp):
 *
 *   loss = -(1/R) sum_i (1/len_i) sum_{t < len_i} min[ rho_it a_i, clip(rho_it, 1-eps, 1+eps) a_i ]
 *
 * (minus the objective, which the paper maximises).  old_logp is a constant (pi_theta_fixed).
 * Gradient flows through a token iff the unclipped term is the selected one, i.e. unless
 * (a > 0 and rho > 1+eps) or (a < 0 and rho < 1-eps).  A rollout of length 0 contributes 0 and
 * still counts in R.
 *
 *   hidden    [R, T, d] dt, in: last-layer hidden state per position (right-padded rollouts)
 *   w_lm      [V, d]    dt, in: lm_head weight, logits = hidden . w_lm^T, no bias
 *   tokens    [R, T] int32, in: generated token per position, in [0, V)
 *   old_logp  [R, T] float32, in: log pi_theta_fixed of that token
 *   adv       [R]    float32, in: a_{S,i}
 *   lengths   [R]    int32, in: valid prefix length in [0, T]; NULL = every rollout has T
 *   clip_eps  >= 0;  grad_scale multiplies both gradients (upstream d/d loss, or a global 1/R fix)
 *   loss      [1]    float32, out (device)
 *   logp_out  [R, T] float32, out, log pi_theta(y) at valid positions, 0 at padded; may be NULL
 *   d_hidden  [R, T, d] float32, out: grad_scale * d loss / d hidden; padded rows are zero
 *   d_w_lm    [V, d]    float32, out: grad_scale * d loss / d w_lm
 *   workspace 256-byte aligned device buffer of workspace_bytes; contents undefined after the call
 *
 * bf16 inputs are multiplied on the matrix cores with fp32 accumulation; softmax statistics are
 * fp32.  The logits are computed once: the forward pass keeps the softmax numerators of one block of
 * tokens at a time in the workspace (fp16, under power-of-two scales so that they cannot overflow), and
 * the backward pass reads them.  For the two gradient contractions the softmax part of the per-logit
 * gradient is thus rounded to fp16, the weight and the token-weighted hidden state are
 * copied to fp16 under power-of-two scales taken from their largest magnitudes (exact for elements
 * within 2^22 of the largest, see pods_loss_report), and the generated token's own logit is applied
 * in fp32; results are deterministic (no floating-point atomics).  A bf16 call with d not a multiple
 * of 8, and every fp32 call, uses plain fp32 vector arithmetic throughout (orders of magnitude slower); bf16
 * with d a multiple of 8 runs on the matrix cores, the working copies padded with zeros to a multiple of 64
 * (hidden and w_lm must be 16-byte aligned).  d <= 16384, R*T <= 2^30,
 * T <= 16776960 (PODS_ERR_UNSUPPORTED beyond).
 */
pods_status grpo_token_loss_fwd_bwd(const void* hidden, const void* w_lm, const int32_t* tokens,
                                    const float* old_logp, const float* adv, const int32_t* lengths,
                                    int32_t R, int32_t T, int32_t d, int32_t V, pods_dtype dt,
                                    float clip_eps, float grad_scale, float* loss, float* logp_out,
                                    float* d_hidden, float* d_w_lm, void* workspace,
                                    size_t workspace_bytes, void* stream);

/* The same, for gradient accumulation over several rollout batches (App., "Note on gradient
 * accumulation": a prompt's rollouts arrive in batches, each is down-sampled and back-propagated
 * on its own): d_w_lm is read and the gradient is added to it; everything else is as above.
 * The caller zeroes d_w_lm before the first batch of an accumulation. */
pods_status grpo_token_loss_fwd_bwd_accumulate(const void* hidden, const void* w_lm, const int32_t* tokens,
                                               const float* old_logp, const float* adv,
                                               const int32_t* lengths, int32_t R, int32_t T, int32_t d,
                                               int32_t V, pods_dtype dt, float clip_eps, float grad_scale,
                                               float* loss, float* logp_out, float* d_hidden,
                                               float* d_w_lm, void* workspace, size_t workspace_bytes,
                                               void* stream);

/* The same with a KL penalty towards a reference policy.  Table 2 lists a KL coefficient (0.04 in one
 * setting, 0 in the others) but the paper gives no formula; taken here is the per-token estimator of the
 * GRPO objective the paper builds on: with x = ref_logp - log pi_theta(y), KL = exp(x) - x - 1 (>= 0),
 * and the token's term becomes min[...] - kl_coef * KL.
 *
 *   ref_logp        [R, T] float32, in: log pi_ref of the generated token (a constant)
 *   kl_coef         >= 0
 *   accumulate_d_w  non-zero: d_w_lm += gradient, as in grpo_token_loss_fwd_bwd_accumulate
 * Everything else as in grpo_token_loss_fwd_bwd. */
pods_status grpo_token_loss_fwd_bwd_kl(const void* hidden, const void* w_lm, const int32_t* tokens,
                                       const float* old_logp, const float* ref_logp, const float* adv,
                                       const int32_t* lengths, int32_t R, int32_t T, int32_t d, int32_t V,
                                       pods_dtype dt, float clip_eps, float kl_coef, float grad_scale,
                                       int32_t accumulate_d_w, float* loss, float* logp_out,
                                       float* d_hidden, float* d_w_lm, void* workspace,
                                       size_t workspace_bytes, void* stream);

/* The general form: every option of the three entry points above, plus the skipping of rollouts that
 * cannot contribute to the gradients.
 *
 *   ref_logp, kl_coef  as in grpo_token_loss_fwd_bwd_kl; ref_logp may be NULL when kl_coef == 0
 *   flags              PODS_LOSS_ACCUMULATE_D_W: d_w_lm += gradient.
 *                      PODS_LOSS_SKIP_ZERO_ADVANTAGE: a rollout with a_i == 0 (every kept rollout of a
 *                      prompt whose kept rewards are all equal, Sec. 3.2) has the per-token weight zero at
 *                      every position, so its terms of both gradients vanish identically; with this flag
 *                      the backward pass leaves those rollouts out (their d_hidden rows are written as
 *                      zero) instead of multiplying by zero.  The loss, logp_out and, up to the order of
 *                      floating-point summation over tokens in d_w_lm, the gradients are unchanged.  The
 *                      flag is ignored while a KL penalty is active (kl_coef != 0), because the penalty
 *                      gives such rollouts a gradient.
 */
enum { PODS_LOSS_ACCUMULATE_D_W = 1, PODS_LOSS_SKIP_ZERO_ADVANTAGE = 2 };
pods_status grpo_token_loss_fwd_bwd_ex(const void* hidden, const void* w_lm, const int32_t* tokens,
                                       const float* old_logp, const float* ref_logp, const float* adv,
                                       const int32_t* lengths, int32_t R, int32_t T, int32_t d, int32_t V,
                                       pods_dtype dt, float clip_eps, float kl_coef, float grad_scale,
                                       int32_t flags, float* loss, float* logp_out, float* d_hidden,
                                       float* d_w_lm, void* workspace, size_t workspace_bytes, void* stream);

/* What a token-loss call (any of the entry points above and below) found in its device-side arguments,
 * and its diagnostic counters; kept in the first 64 bytes of the workspace after the call.
 *
 *   valid_tokens      N = sum of the lengths (after clamping to [0, T])
 *   backward_tokens   valid tokens the backward pass covered (N unless zero-advantage rollouts were skipped)
 *   clipped_tokens    valid tokens at which the clipped term of the surrogate is the selected one, so no
 *                     gradient flows: (a > 0 and rho > 1+eps) or (a < 0 and rho < 1-eps).  Divided by
 *                     valid_tokens this is the clip fraction.
 *   bad_lengths       rollouts whose length lay outside [0, T];  bad_tokens: valid positions whose token
 *                     id lay outside [0, V).  Both were taken as clamped; non-zero means the results of
 *                     the call are meaningless.
 *   max_abs_g         max over valid tokens of |d loss / d log pi(y)| (times grad_scale)
 *   max_abs_w, max_abs_hidden   largest |w_lm| element and largest |hidden| element over valid positions
 *                     (bf16 matrix-core path only, 0 otherwise).  A NaN or infinity here means the inputs
 *                     held one.  The two fp16 operands of the gradient contractions are scaled by powers
 *                     of two chosen from these maxima, so no finite bf16 input overflows them; elements
 *                     more than 2^22 below the maximum lose low-order bits (fp16 subnormals).
 *
 * grpo_token_loss_report copies the report to HOST memory: it waits for `stream` (the only token-loss call
 * that synchronises with the device).  workspace = the workspace of the call to report on, or NULL for
 * the built-in one of grpo_token_loss_fwd_bwd_static on the current GPU. */
typedef struct {
    int32_t valid_tokens;
    int32_t backward_tokens;
    int32_t clipped_tokens;
    int32_t bad_lengths;
    int32_t bad_tokens;
    float max_abs_g;
    float max_abs_w;
    float max_abs_hidden;
    int32_t reserved[8];
} pods_loss_report;
pods_status grpo_token_loss_report(const void* workspace, pods_loss_report* report /* host */, void* stream);

/* grpo_token_loss_fwd_bwd for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): no workspace argument; the working arrays live
 * in a device array built into the library, PODS_STATIC_WORKSPACE_BYTES per GPU, which every GPU the
 * library runs on holds until the process ends.  The call allocates and frees nothing.  Sizes whose
 * minimal workspace (grpo_token_loss_workspace_min_bytes) exceeds that array are rejected with
 * PODS_ERR_UNSUPPORTED before anything is launched.  Within the array the call picks its token block
 * as grpo_token_loss_fwd_bwd does for a workspace of that size, so the results are those of that
 * call.  The array belongs to the GPU that is current when the call is made; all calls on one GPU share
 * it, so two calls that overlap in time on the same GPU (different streams or threads) race: serialise
 * them.  Each call writes every part of the array it later reads; nothing is kept between calls.
 * grpo_token_loss_static_workspace_bytes() returns PODS_STATIC_WORKSPACE_BYTES.  All other arguments as
 * in grpo_token_loss_fwd_bwd. */
#define PODS_STATIC_WORKSPACE_BYTES (64u << 20)
size_t grpo_token_loss_static_workspace_bytes(void);
pods_status grpo_token_loss_fwd_bwd_static(const void* hidden, const void* w_lm, const int32_t* tokens,
                                           const float* old_logp, const float* adv, const int32_t* lengths,
                                           int32_t R, int32_t T, int32_t d, int32_t V, pods_dtype dt,
                                           float clip_eps, float grad_scale, float* loss, float* logp_out,
                                           float* d_hidden, float* d_w_lm, void* stream);

/* Host string for the last error on the calling thread; valid until the next failing call. */
const char* pods_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PODS_H_ */
