// C ABI of the PODS HIP library: argument checks, then dispatch to the kernel families.
#include "common.h"
#include "loss.h"

#include <mutex>

namespace pods {
char* error_buffer() {
    static thread_local char buf[kErrorBufferBytes] = "";
    return buf;
}

}  // namespace pods

using namespace pods;

extern "C" {

const char* pods_last_error(void) { return error_buffer(); }

pods_status pods_select(const float* rewards, int32_t B, int32_t n, int32_t m, int32_t* sel_idx,
                        int32_t* sel_k, void* stream) {
    if (rewards == nullptr || sel_idx == nullptr)
        return fail(PODS_ERR_INVALID_ARG, "pods_select: rewards and sel_idx must not be null");
    if (B <= 0 || n <= 0 || m <= 0)
        return fail(PODS_ERR_INVALID_ARG, "pods_select: B=%d n=%d m=%d must be positive", B, n, m);
    if (m > n) return fail(PODS_ERR_INVALID_ARG, "pods_select: m=%d exceeds n=%d", m, n);
    if (n > 4096) return fail(PODS_ERR_UNSUPPORTED, "pods_select: n=%d exceeds 4096", n);
    return launch_select(rewards, nullptr, B, n, m, PODS_RULE_MAXVAR, sel_idx, sel_k,
                         static_cast<hipStream_t>(stream));
}

pods_status pods_check_rewards(const float* rewards, int32_t B, int32_t n, int32_t* report, void* stream) {
    if (rewards == nullptr || report == nullptr)
        return fail(PODS_ERR_INVALID_ARG, "pods_check_rewards: rewards and report must not be null");
    if (B <= 0 || n <= 0) return fail(PODS_ERR_INVALID_ARG, "pods_check_rewards: B=%d n=%d must be positive", B, n);
    if ((int64_t)B * n > (int64_t)0x7fffffff)
        return fail(PODS_ERR_UNSUPPORTED, "pods_check_rewards: more than 2^31 - 1 rewards");
    return launch_check_rewards(rewards, (int64_t)B * n, report, static_cast<hipStream_t>(stream));
}

pods_status pods_downsample(const float* rewards, const uint32_t* rand_keys, int32_t B, int32_t n,
                            int32_t m, pods_rule rule, int32_t* sel_idx, int32_t* sel_k, void* stream) {
    if (rule != PODS_RULE_MAXVAR && rule != PODS_RULE_MAXR && rule != PODS_RULE_PERC && rule != PODS_RULE_RAND)
        return fail(PODS_ERR_INVALID_ARG, "pods_downsample: unknown rule %d", (int)rule);
    if (sel_idx == nullptr) return fail(PODS_ERR_INVALID_ARG, "pods_downsample: sel_idx must not be null");
    if (rule == PODS_RULE_RAND && rand_keys == nullptr)
        return fail(PODS_ERR_INVALID_ARG, "pods_downsample: the random rule needs rand_keys");
    if (rule != PODS_RULE_RAND && rewards == nullptr)
        return fail(PODS_ERR_INVALID_ARG, "pods_downsample: rewards must not be null");
    if (B <= 0 || n <= 0 || m <= 0)
        return fail(PODS_ERR_INVALID_ARG, "pods_downsample: B=%d n=%d m=%d must be positive", B, n, m);
    if (m > n) return fail(PODS_ERR_INVALID_ARG, "pods_downsample: m=%d exceeds n=%d", m, n);
    if (n > 4096) return fail(PODS_ERR_UNSUPPORTED, "pods_downsample: n=%d exceeds 4096", n);
    return launch_select(rewards, rand_keys, B, n, m, (int32_t)rule, sel_idx, sel_k,
                         static_cast<hipStream_t>(stream));
}

static pods_status advantage_entry(const char* who, const float* rewards, const int32_t* sel_idx, int32_t B,
                                   int32_t n, int32_t m, float std_eps, bool stats_from_all, float* adv,
                                   void* stream) {
    if (rewards == nullptr || sel_idx == nullptr || adv == nullptr)
        return fail(PODS_ERR_INVALID_ARG, "%s: null pointer", who);
    if (B <= 0 || n <= 0 || m <= 0)
        return fail(PODS_ERR_INVALID_ARG, "%s: B=%d n=%d m=%d must be positive", who, B, n, m);
    if (m > n) return fail(PODS_ERR_INVALID_ARG, "%s: m=%d exceeds n=%d", who, m, n);
    if (m > 4096) return fail(PODS_ERR_UNSUPPORTED, "%s: m=%d exceeds 4096", who, m);
    if (!(std_eps >= 0.0f)) return fail(PODS_ERR_INVALID_ARG, "%s: std_eps < 0", who);
    return launch_advantage(rewards, sel_idx, B, n, m, std_eps, stats_from_all, adv,
                            static_cast<hipStream_t>(stream));
}

pods_status pods_advantage(const float* rewards, const int32_t* sel_idx, int32_t B, int32_t n,
                           int32_t m, float std_eps, float* adv, void* stream) {
    return advantage_entry("pods_advantage", rewards, sel_idx, B, n, m, std_eps, false, adv, stream);
}

pods_status pods_advantage_before(const float* rewards, const int32_t* sel_idx, int32_t B, int32_t n,
                                  int32_t m, float std_eps, float* adv, void* stream) {
    return advantage_entry("pods_advantage_before", rewards, sel_idx, B, n, m, std_eps, true, adv, stream);
}

pods_status pods_downsample_gather(const float* rewards, const uint32_t* rand_keys, int32_t B, int32_t n,
                                   int32_t m, pods_rule rule, float std_eps, int32_t stats_from_all,
                                   const pods_record* records, int32_t num_records, int32_t* sel_idx,
                                   int32_t* sel_k, float* adv, void* stream) {
    const char* who = "pods_downsample_gather";
    if (rule != PODS_RULE_MAXVAR && rule != PODS_RULE_MAXR && rule != PODS_RULE_PERC && rule != PODS_RULE_RAND)
        return fail(PODS_ERR_INVALID_ARG, "%s: unknown rule %d", who, (int)rule);
    if (rewards == nullptr || sel_idx == nullptr || adv == nullptr)
        return fail(PODS_ERR_INVALID_ARG, "%s: rewards, sel_idx and adv must not be null", who);
    if (rule == PODS_RULE_RAND && rand_keys == nullptr)
        return fail(PODS_ERR_INVALID_ARG, "%s: the random rule needs rand_keys", who);
    if (B <= 0 || n <= 0 || m <= 0)
        return fail(PODS_ERR_INVALID_ARG, "%s: B=%d n=%d m=%d must be positive", who, B, n, m);
    if (m > n) return fail(PODS_ERR_INVALID_ARG, "%s: m=%d exceeds n=%d", who, m, n);
    if (n > 1024) return fail(PODS_ERR_UNSUPPORTED, "%s: n=%d exceeds 1024", who, n);
    if (!(std_eps >= 0.0f)) return fail(PODS_ERR_INVALID_ARG, "%s: std_eps < 0", who);
    if (num_records < 0 || num_records > PODS_MAX_RECORDS)
        return fail(PODS_ERR_INVALID_ARG, "%s: num_records=%d outside [0, %d]", who, num_records,
                    (int)PODS_MAX_RECORDS);
    if (num_records > 0 && records == nullptr)
        return fail(PODS_ERR_INVALID_ARG, "%s: records must not be null", who);
    for (int32_t q = 0; q < num_records; ++q)
        if (records[q].src == nullptr || records[q].dst == nullptr || records[q].row_bytes == 0)
            return fail(PODS_ERR_INVALID_ARG, "%s: record %d has a null pointer or no bytes", who, q);
    return launch_downsample_gather(rewards, rand_keys, B, n, m, (int32_t)rule, std_eps, stats_from_all != 0,
                                    records, num_records, sel_idx, sel_k, adv, static_cast<hipStream_t>(stream));
}

static bool loss_sizes_ok(int32_t R, int32_t T, int32_t d, int32_t V, pods_dtype dt) {
    return R > 0 && T > 0 && d > 0 && V > 0 && (dt == PODS_F32 || dt == PODS_BF16) &&
           (int64_t)R * T <= (int64_t)1 << 30;
}

size_t grpo_token_loss_workspace_bytes(int32_t R, int32_t T, int32_t d, int32_t V, pods_dtype dt) {
    if (!loss_sizes_ok(R, T, d, V, dt)) return 0;
    return plan_loss(R, T, d, V, dt, 0).total;
}

size_t grpo_token_loss_workspace_min_bytes(int32_t R, int32_t T, int32_t d, int32_t V, pods_dtype dt) {
    if (!loss_sizes_ok(R, T, d, V, dt)) return 0;
    return plan_loss(R, T, d, V, dt, 1).total;
}

size_t grpo_token_loss_workspace_used_bytes(int32_t R, int32_t T, int32_t d, int32_t V, pods_dtype dt,
                                            size_t workspace_bytes) {
    if (!loss_sizes_ok(R, T, d, V, dt)) return 0;
    if (workspace_bytes < plan_loss(R, T, d, V, dt, 1).total) return 0;
    return plan_loss(R, T, d, V, dt, workspace_bytes).total;
}

static pods_status token_loss_entry(const void* hidden, const void* w_lm, const int32_t* tokens,
                                    const float* old_logp, const float* ref_logp, float kl_coef,
                                    const float* adv, const int32_t* lengths,
                                    int32_t R, int32_t T, int32_t d, int32_t V, pods_dtype dt,
                                    float clip_eps, float grad_scale, float* loss, float* logp_out,
                                    float* d_hidden, float* d_w_lm, int32_t flags, void* workspace,
                                    size_t workspace_bytes, void* stream) {
    if (hidden == nullptr || w_lm == nullptr || tokens == nullptr || old_logp == nullptr ||
        adv == nullptr || loss == nullptr || d_hidden == nullptr || d_w_lm == nullptr)
        return fail(PODS_ERR_INVALID_ARG, "grpo_token_loss_fwd_bwd: null pointer");
    if (R <= 0 || T <= 0 || d <= 0 || V <= 0)
        return fail(PODS_ERR_INVALID_ARG, "grpo_token_loss_fwd_bwd: R=%d T=%d d=%d V=%d must be positive",
                    R, T, d, V);
    if (dt != PODS_F32 && dt != PODS_BF16)
        return fail(PODS_ERR_INVALID_ARG, "grpo_token_loss_fwd_bwd: unknown dtype %d", (int)dt);
    if (!(clip_eps >= 0.0f)) return fail(PODS_ERR_INVALID_ARG, "grpo_token_loss_fwd_bwd: clip_eps < 0");
    if ((flags & ~(PODS_LOSS_ACCUMULATE_D_W | PODS_LOSS_SKIP_ZERO_ADVANTAGE)) != 0)
        return fail(PODS_ERR_INVALID_ARG, "grpo_token_loss_fwd_bwd: unknown flag bits in %d", flags);
    if (!(grad_scale == grad_scale)) return fail(PODS_ERR_INVALID_ARG, "grpo_token_loss_fwd_bwd: grad_scale is NaN");
    if (!loss_sizes_ok(R, T, d, V, dt))
        return fail(PODS_ERR_UNSUPPORTED, "grpo_token_loss_fwd_bwd: R*T exceeds 2^30 positions");
    if (d > 16384) return fail(PODS_ERR_UNSUPPORTED, "grpo_token_loss_fwd_bwd: d=%d exceeds 16384", d);
    if (T > 65535 * 256) return fail(PODS_ERR_UNSUPPORTED, "grpo_token_loss_fwd_bwd: T=%d exceeds 16776960", T);
    if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
        return fail(PODS_ERR_WORKSPACE, "grpo_token_loss_fwd_bwd: workspace null or not 256-byte aligned");
    const size_t need = plan_loss(R, T, d, V, dt, 1).total;
    if (workspace_bytes < need)
        return fail(PODS_ERR_WORKSPACE, "grpo_token_loss_fwd_bwd: workspace %zu B < required %zu B",
                    workspace_bytes, need);
    LossArgs a;
    a.hidden = hidden; a.w_lm = w_lm; a.tokens = tokens; a.old_logp = old_logp; a.adv = adv;
    a.ref_logp = (ref_logp != nullptr && kl_coef != 0.0f) ? ref_logp : nullptr; a.kl_coef = kl_coef;
    a.lengths = lengths; a.R = R; a.T = T; a.d = d; a.V = V; a.dt = dt; a.clip_eps = clip_eps;
    a.grad_scale = grad_scale; a.loss = loss; a.logp_out = logp_out; a.d_hidden = d_hidden;
    a.d_w_lm = d_w_lm; a.accumulate_d_w = (flags & PODS_LOSS_ACCUMULATE_D_W) != 0;
    // with a KL penalty a zero-advantage rollout still has a gradient: nothing can be skipped
    a.skip_zero_adv = (flags & PODS_LOSS_SKIP_ZERO_ADVANTAGE) != 0 && a.ref_logp == nullptr;
    a.workspace = static_cast<unsigned char*>(workspace);
    a.workspace_bytes = workspace_bytes; a.stream = static_cast<hipStream_t>(stream);
    return run_loss(a);
}

pods_status grpo_token_loss_fwd_bwd(const void* hidden, const void* w_lm, const int32_t* tokens,
                                    const float* old_logp, const float* adv, const int32_t* lengths,
                                    int32_t R, int32_t T, int32_t d, int32_t V, pods_dtype dt,
                                    float clip_eps, float grad_scale, float* loss, float* logp_out,
                                    float* d_hidden, float* d_w_lm, void* workspace,
                                    size_t workspace_bytes, void* stream) {
    return token_loss_entry(hidden, w_lm, tokens, old_logp, nullptr, 0.0f, adv, lengths, R, T, d, V, dt, clip_eps,
                            grad_scale, loss, logp_out, d_hidden, d_w_lm, 0, workspace, workspace_bytes, stream);
}

pods_status grpo_token_loss_fwd_bwd_accumulate(const void* hidden, const void* w_lm, const int32_t* tokens,
                                               const float* old_logp, const float* adv,
                                               const int32_t* lengths, int32_t R, int32_t T, int32_t d,
                                               int32_t V, pods_dtype dt, float clip_eps, float grad_scale,
                                               float* loss, float* logp_out, float* d_hidden,
                                               float* d_w_lm, void* workspace, size_t workspace_bytes,
                                               void* stream) {
    return token_loss_entry(hidden, w_lm, tokens, old_logp, nullptr, 0.0f, adv, lengths, R, T, d, V, dt, clip_eps,
                            grad_scale, loss, logp_out, d_hidden, d_w_lm, PODS_LOSS_ACCUMULATE_D_W, workspace, workspace_bytes, stream);
}

pods_status grpo_token_loss_fwd_bwd_kl(const void* hidden, const void* w_lm, const int32_t* tokens,
                                       const float* old_logp, const float* ref_logp, const float* adv,
                                       const int32_t* lengths, int32_t R, int32_t T, int32_t d, int32_t V,
                                       pods_dtype dt, float clip_eps, float kl_coef, float grad_scale,
                                       int32_t accumulate_d_w, float* loss, float* logp_out,
                                       float* d_hidden, float* d_w_lm, void* workspace,
                                       size_t workspace_bytes, void* stream) {
    if (ref_logp == nullptr) return fail(PODS_ERR_INVALID_ARG, "grpo_token_loss_fwd_bwd_kl: ref_logp is null");
    if (!(kl_coef >= 0.0f)) return fail(PODS_ERR_INVALID_ARG, "grpo_token_loss_fwd_bwd_kl: kl_coef < 0");
    return token_loss_entry(hidden, w_lm, tokens, old_logp, ref_logp, kl_coef, adv, lengths, R, T, d, V, dt, clip_eps,
                            grad_scale, loss, logp_out, d_hidden, d_w_lm,
                            accumulate_d_w != 0 ? PODS_LOSS_ACCUMULATE_D_W : 0, workspace, workspace_bytes, stream);
}

pods_status grpo_token_loss_fwd_bwd_ex(const void* hidden, const void* w_lm, const int32_t* tokens,
                                       const float* old_logp, const float* ref_logp, const float* adv,
                                       const int32_t* lengths, int32_t R, int32_t T, int32_t d, int32_t V,
                                       pods_dtype dt, float clip_eps, float kl_coef, float grad_scale,
                                       int32_t flags, float* loss, float* logp_out, float* d_hidden,
                                       float* d_w_lm, void* workspace, size_t workspace_bytes, void* stream) {
    if (!(kl_coef >= 0.0f)) return fail(PODS_ERR_INVALID_ARG, "grpo_token_loss_fwd_bwd_ex: kl_coef < 0");
    if (ref_logp == nullptr && kl_coef != 0.0f)
        return fail(PODS_ERR_INVALID_ARG, "grpo_token_loss_fwd_bwd_ex: kl_coef = %g needs ref_logp", (double)kl_coef);
    return token_loss_entry(hidden, w_lm, tokens, old_logp, ref_logp, kl_coef, adv, lengths, R, T, d, V, dt, clip_eps,
                            grad_scale, loss, logp_out, d_hidden, d_w_lm, flags, workspace, workspace_bytes, stream);
}

// ---- grpo_token_loss_fwd_bwd_static: the workspace is a device array of this library -----------------
namespace {
constexpr size_t kScratchBytes = (size_t)PODS_STATIC_WORKSPACE_BYTES;
constexpr int kMaxDevices = 64;
}  // namespace
// One copy per GPU, at that GPU's own address; in host code the name is only a handle for
// hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
namespace {
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each GPU, looked up once

pods_status scratch_on_current_device(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(PODS_ERR_RUNTIME, "grpo_token_loss_fwd_bwd_static: hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices)
        return fail(PODS_ERR_UNSUPPORTED, "grpo_token_loss_fwd_bwd_static: device %d outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || ptr == nullptr)
            return fail(PODS_ERR_RUNTIME, "grpo_token_loss_fwd_bwd_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return PODS_OK;
}
}  // namespace

size_t grpo_token_loss_static_workspace_bytes(void) { return kScratchBytes; }

pods_status grpo_token_loss_report(const void* workspace, pods_loss_report* report, void* stream) {
    if (report == nullptr) return fail(PODS_ERR_INVALID_ARG, "grpo_token_loss_report: report must not be null");
    const void* src = workspace;
    if (src == nullptr) {   // the built-in working array of grpo_token_loss_fwd_bwd_static
        void* ws = nullptr;
        pods_status st = scratch_on_current_device(&ws);
        if (st != PODS_OK) return st;
        src = ws;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = hipMemcpyAsync(report, src, sizeof(pods_loss_report), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return fail(PODS_ERR_RUNTIME, "grpo_token_loss_report: %s", hipGetErrorString(e));
    return PODS_OK;
}

pods_status grpo_token_loss_fwd_bwd_static(const void* hidden, const void* w_lm, const int32_t* tokens,
                                           const float* old_logp, const float* adv, const int32_t* lengths,
                                           int32_t R, int32_t T, int32_t d, int32_t V, pods_dtype dt,
                                           float clip_eps, float grad_scale, float* loss, float* logp_out,
                                           float* d_hidden, float* d_w_lm, void* stream) {
    if (!loss_sizes_ok(R, T, d, V, dt))
        return fail(PODS_ERR_INVALID_ARG, "grpo_token_loss_fwd_bwd_static: R=%d T=%d d=%d V=%d dtype=%d invalid", R, T, d,
                    V, (int)dt);
    const size_t need = plan_loss(R, T, d, V, dt, 1).total;
    if (need > kScratchBytes)
        return fail(PODS_ERR_UNSUPPORTED,
                    "grpo_token_loss_fwd_bwd_static: these sizes need %zu B of workspace, the built-in one has %zu B; "
                    "use grpo_token_loss_fwd_bwd with a workspace of the caller's",
                    need, kScratchBytes);
    void* ws = nullptr;
    pods_status st = scratch_on_current_device(&ws);
    if (st != PODS_OK) return st;
    return token_loss_entry(hidden, w_lm, tokens, old_logp, nullptr, 0.0f, adv, lengths, R, T, d, V, dt, clip_eps,
                            grad_scale, loss, logp_out, d_hidden, d_w_lm, 0, ws, kScratchBytes, stream);
}

pods_status pods_gather_rows(const void* src, const int32_t* sel_idx, int32_t B, int32_t n, int32_t m,
                             size_t row_bytes, void* dst, void* stream) {
    if (src == nullptr || sel_idx == nullptr || dst == nullptr)
        return fail(PODS_ERR_INVALID_ARG, "pods_gather_rows: null pointer");
    if (B <= 0 || n <= 0 || m <= 0 || row_bytes == 0)
        return fail(PODS_ERR_INVALID_ARG, "pods_gather_rows: B=%d n=%d m=%d row_bytes=%zu must be positive", B, n, m,
                    row_bytes);
    if (m > n) return fail(PODS_ERR_INVALID_ARG, "pods_gather_rows: m=%d exceeds n=%d", m, n);
    if ((int64_t)B * m > (int64_t)0x7fffffff)
        return fail(PODS_ERR_UNSUPPORTED, "pods_gather_rows: more than 2^31 - 1 kept rollouts");
    return launch_gather_rows(src, sel_idx, B, n, m, row_bytes, dst, static_cast<hipStream_t>(stream));
}

}  // extern "C"
