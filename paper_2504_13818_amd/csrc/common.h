// Shared host-side helpers of the PODS HIP library: error reporting and launch checks.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "pods.h"

namespace pods {

// Thread-local message behind pods_last_error().
char* error_buffer();
constexpr size_t kErrorBufferBytes = 512;

inline pods_status fail(pods_status code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(error_buffer(), kErrorBufferBytes, fmt, ap);
    va_end(ap);
    return code;
}

// Reports (and clears) a launch error of the kernel just enqueued.
inline pods_status check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(PODS_ERR_RUNTIME, "%s: %s", what, hipGetErrorString(e));
    return PODS_OK;
}

// Optional per-launch timing (pods_profile_*): when enabled on the calling thread, every kernel
// launch made through a StageTimer scope is bracketed by a pair of HIP events on its stream.
void profile_stage_begin(const char* name, hipStream_t stream);
void profile_stage_end(hipStream_t stream);
struct StageTimer {
    hipStream_t stream;
    StageTimer(const char* name, hipStream_t s) : stream(s) { profile_stage_begin(name, s); }
    ~StageTimer() { profile_stage_end(stream); }
};

#define PODS_LAUNCH(name, strm, ...)                        \
    do {                                                    \
        ::pods::StageTimer pods_stage_timer_(name, strm);   \
        hipLaunchKernelGGL(__VA_ARGS__);                    \
    } while (0)

constexpr int kWave = 64;  // CDNA wavefront width

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Kernel-family entry points (defined in select.hip, advantage.hip, loss_*.hip).
pods_status launch_select(const float* rewards, const uint32_t* rand_keys, int32_t B, int32_t n, int32_t m,
                          int32_t rule, int32_t* sel_idx, int32_t* sel_k, hipStream_t stream);
pods_status launch_advantage(const float* rewards, const int32_t* sel_idx, int32_t B, int32_t n,
                             int32_t m, float std_eps, bool stats_from_all, float* adv, hipStream_t stream);
pods_status launch_check_rewards(const float* rewards, int64_t count, int32_t* report, hipStream_t stream);
pods_status launch_gather_rows(const void* src, const int32_t* sel_idx, int32_t B, int32_t n, int32_t m,
                               size_t row_bytes, void* dst, hipStream_t stream);
pods_status launch_downsample_gather(const float* rewards, const uint32_t* rand_keys, int32_t B, int32_t n, int32_t m,
                                     int32_t rule, float std_eps, bool stats_from_all, const pods_record* records,
                                     int32_t num_records, int32_t* sel_idx, int32_t* sel_k, float* adv,
                                     hipStream_t stream);

}  // namespace pods
