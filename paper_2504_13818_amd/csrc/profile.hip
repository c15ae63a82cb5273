// Benchmark plumbing, apart from the method: per-launch HIP-event timing of the library's kernels
// (pods_profile.h) and a matrix-core-only loop that measures what the chip sustains with no memory
// traffic at all.
#include "common.h"
#include "pods_profile.h"

#include <vector>

namespace pods {
namespace {
struct Stage { const char* name; hipEvent_t start, stop; };
struct Profile {
    bool enabled = false;
    size_t used = 0;             // stages recorded since the last enable / reset
    std::vector<Stage> stages;   // event pairs are created once and reused
};
Profile& profile() {
    static thread_local Profile p;
    return p;
}
}  // namespace

void profile_stage_begin(const char* name, hipStream_t stream) {
    Profile& p = profile();
    if (!p.enabled) return;
    if (p.used == p.stages.size()) {
        Stage s{name, nullptr, nullptr};
        if (hipEventCreate(&s.start) != hipSuccess || hipEventCreate(&s.stop) != hipSuccess) {
            p.enabled = false;
            return;
        }
        p.stages.push_back(s);
    }
    p.stages[p.used].name = name;
    (void)hipEventRecord(p.stages[p.used].start, stream);
}

void profile_stage_end(hipStream_t stream) {
    Profile& p = profile();
    if (!p.enabled || p.used >= p.stages.size()) return;
    (void)hipEventRecord(p.stages[p.used].stop, stream);
    ++p.used;
}


namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Each wave multiplies 4 x 4 blocks of 32 x 32 x 16 bf16 from registers, `iters` times two k-steps: the
// instruction mix of the token loss's main loop with every load taken out.  Operands are pseudo-random
// values of both signs in [-2, 2) (the matrix pipe's power draw follows the operand bits).
__global__ __launch_bounds__(256, 1) void mfma_only_kernel(int iters, float* __restrict__ sink) {
    bf16x8 a[4], b[4];
    uint32_t x = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            x = x * 1664525u + 1013904223u;
            a[i][j] = (__bf16)((float)(int)(x >> 16 & 0xFFFu) * (1.0f / 1024.0f) - 2.0f);
            x = x * 1664525u + 1013904223u;
            b[i][j] = (__bf16)((float)(int)(x >> 16 & 0xFFFu) * (1.0f / 1024.0f) - 2.0f);
        }
    f32x16 acc[4][4];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                for (int ni = 0; ni < 4; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) s += acc[mi][ni][r];
    if (s == 123.456f) sink[0] = s;   // keeps the loop alive; practically never true
}

}  // namespace
}  // namespace pods

using namespace pods;

extern "C" {

pods_status pods_profile_enable(int32_t enable) {
    auto& p = profile();
    p.enabled = enable != 0;
    p.used = 0;
    if (!p.enabled) {   // switched off: the events go too
        for (Stage& s : p.stages) {
            (void)hipEventDestroy(s.start);
            (void)hipEventDestroy(s.stop);
        }
        p.stages.clear();
    }
    return PODS_OK;
}

int32_t pods_profile_count(void) { return (int32_t)profile().used; }

pods_status pods_profile_get(int32_t i, const char** name, float* ms) {
    auto& p = profile();
    if (i < 0 || (size_t)i >= p.used || name == nullptr || ms == nullptr)
        return fail(PODS_ERR_INVALID_ARG, "pods_profile_get: index %d outside [0, %zu)", i, p.used);
    hipError_t e = hipEventSynchronize(p.stages[i].stop);
    if (e == hipSuccess) e = hipEventElapsedTime(ms, p.stages[i].start, p.stages[i].stop);
    if (e != hipSuccess) return fail(PODS_ERR_RUNTIME, "pods_profile_get: %s", hipGetErrorString(e));
    *name = p.stages[i].name;
    return PODS_OK;
}

pods_status pods_profile_mfma_only(int32_t workgroups, int32_t iters, float* sink, double* flops, void* stream) {
    if (workgroups <= 0 || iters <= 0 || sink == nullptr || flops == nullptr)
        return fail(PODS_ERR_INVALID_ARG, "pods_profile_mfma_only: workgroups and iters must be positive, sink and flops not null");
    hipStream_t s = static_cast<hipStream_t>(stream);
    PODS_LAUNCH("mfma only", s, mfma_only_kernel, dim3((unsigned)workgroups), dim3(256), 0, s, iters, sink);
    *flops = (double)workgroups * 4.0 * (double)iters * 32.0 * (2.0 * 32 * 32 * 16);
    return check_launch("pods_profile_mfma_only");
}

}  // extern "C"
