// Calls every entry point of the C ABI with arguments that the host-side checks must refuse
// (and the queries with valid ones), in a build whose HOST code carries AddressSanitizer and
// UndefinedBehaviorSanitizer.  No kernel is launched and no GPU is needed: every call returns
// from its argument checks.  A wrong status, or a sanitizer report, ends the run non-zero.
// Built and run by tests/test_sanitizers_cpu.py.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "spo.h"

static int failures = 0;
#define EXPECT(call, want)                                                             \
    do {                                                                               \
        const long long got_ = (long long)(call);                                      \
        if (got_ != (long long)(want)) {                                               \
            std::fprintf(stderr, "%s:%d: %s = %lld, expected %lld\n", __FILE__, __LINE__, #call, got_, (long long)(want)); \
            ++failures;                                                                \
        }                                                                              \
    } while (0)

int main() {
    // non-NULL, aligned dummies: never dereferenced on the paths taken here
    float *f = reinterpret_cast<float *>(uintptr_t(4096));
    int32_t *i32 = reinterpret_cast<int32_t *>(uintptr_t(8192));
    void *ws = reinterpret_cast<void *>(uintptr_t(1) << 20);
    void *odd = reinterpret_cast<void *>((uintptr_t(1) << 20) + 8);

    for (int sc = 1; sc >= -8; --sc) EXPECT(std::strlen(spo_status_string(sc)) > 0, 1);

    // sampler
    EXPECT(spo_sample_prompts_workspace_bytes(0, 1), 0);
    EXPECT(spo_sample_prompts_workspace_bytes(int64_t(1) << 20, 4096) >= (size_t(12) << 20), 1);
    EXPECT(spo_sample_prompts(nullptr, f, 4, 1, 0.05, 0, 0, 0, 0, i32, nullptr, ws, 1 << 20, nullptr), SPO_ENULL);
    EXPECT(spo_sample_prompts(f, f, 0, 1, 0.05, 0, 0, 0, 0, i32, nullptr, ws, 1 << 20, nullptr), SPO_EINVAL);
    EXPECT(spo_sample_prompts(f, f, 4, 1, -0.1, 0, 0, 0, 0, i32, nullptr, ws, 1 << 20, nullptr), SPO_EINVAL);
    EXPECT(spo_sample_prompts(f, f, 4, 5, 0.05, 0, 0, 0, 0, i32, nullptr, ws, 1 << 20, nullptr), SPO_EINVAL);
    EXPECT(spo_sample_prompts(f, f, int64_t(1) << 20, 20000, 0.05, 0, 0, 0, 0, i32, nullptr, ws, size_t(1) << 30, nullptr), SPO_ERANGE);
    EXPECT(spo_sample_prompts(f, f, 4, 2, 0.05, 0, 0, 0, 0, i32, nullptr, nullptr, 0, nullptr), SPO_EWORKSPACE);
    EXPECT(spo_sample_prompts(f, f, 4, 2, 0.05, 0, 0, 0, 0, i32, nullptr, ws, 8, nullptr), SPO_EWORKSPACE);
    EXPECT(spo_sample_prompts(f, f, 4, 2, 0.05, 0, 0, 0, 0, i32, nullptr, odd, 1 << 20, nullptr), SPO_EINVAL);
    EXPECT(spo_sample_prompts_static(f, f, int64_t(SPO_SAMPLE_STATIC_MAX_N) + 1, 2, 0.05, 0, 0, 0, 0, i32, nullptr, nullptr), SPO_ERANGE);
    EXPECT(spo_sample_prompts_static(f, nullptr, 4, 2, 0.05, 0, 0, 0, 0, i32, nullptr, nullptr), SPO_ENULL);

    // advantages, diagnostics, tracker
    EXPECT(spo_advantages(nullptr, f, 4, i32, f, 1, 0, 0.0f, 1, nullptr, f, nullptr, nullptr, nullptr, 0, nullptr), SPO_ENULL);
    EXPECT(spo_advantages(f, f, 4, i32, f, 0, 0, 0.0f, 1, nullptr, f, nullptr, nullptr, nullptr, 0, nullptr), SPO_EINVAL);
    EXPECT(spo_advantages(f, f, 4, i32, f, 3, 2, 0.0f, 1, nullptr, f, nullptr, nullptr, nullptr, 0, nullptr), SPO_EINVAL);
    EXPECT(spo_advantages(f, f, 4, i32, f, 3, 0, -1.0f, 1, nullptr, f, nullptr, nullptr, nullptr, 0, nullptr), SPO_EINVAL);
    EXPECT(spo_advantages(f, f, 4, i32, f, 3, 0, 0.0f, 1, nullptr, f, nullptr, nullptr, ws, 8, nullptr), SPO_EWORKSPACE);
    EXPECT(spo_advantages(f, f, 4, i32, f, 3, 0, 0.0f, 1, nullptr, f, nullptr, nullptr, odd, 1 << 20, nullptr), SPO_EINVAL);
    EXPECT(spo_advantages_workspace_bytes(0), 0);
    EXPECT(spo_advantage_diagnostics(f, f, 4, 0.02f, 1e-4f, f, nullptr), SPO_EINVAL);
    EXPECT(spo_advantage_diagnostics(f, nullptr, 4, 1e-4f, 0.02f, f, nullptr), SPO_ENULL);
    EXPECT(spo_tracker_update_workspace_bytes(0), 0);
    EXPECT(spo_tracker_update_workspace_bytes(1000), 4096);
    EXPECT(spo_tracker_update(f, f, 4, i32, f, nullptr, 1, 0.25f, 0.875f, 0.96f, 1, nullptr, nullptr, nullptr, nullptr, 0, nullptr), SPO_ENULL);
    EXPECT(spo_tracker_update(f, f, 4, i32, f, f, 1, 0.0f, 0.875f, 0.96f, 1, nullptr, nullptr, nullptr, nullptr, 0, nullptr), SPO_EINVAL);
    EXPECT(spo_tracker_update(f, f, 4, i32, f, f, 1, 0.25f, 0.97f, 0.96f, 1, nullptr, nullptr, nullptr, nullptr, 0, nullptr), SPO_EINVAL);
    EXPECT(spo_tracker_update(f, f, 4, i32, f, f, 1, 0.25f, 0.875f, 1.5f, 1, nullptr, nullptr, nullptr, nullptr, 0, nullptr), SPO_EINVAL);
    EXPECT(spo_tracker_update(f, f, 4, i32, f, f, 1, 0.25f, 0.875f, 0.96f, 0, nullptr, nullptr, nullptr, nullptr, 0, nullptr), SPO_EWORKSPACE);
    EXPECT(spo_tracker_update(f, f, 1000, i32, f, f, 1, 0.25f, 0.875f, 0.96f, 0, nullptr, nullptr, nullptr, ws, 256, nullptr), SPO_EWORKSPACE);
    EXPECT(spo_tracker_update(f, f, 4, i32, f, f, 1, 0.25f, 0.875f, 0.96f, 1, nullptr, nullptr, nullptr, odd, 256, nullptr), SPO_EINVAL);
    EXPECT(spo_tracker_update_ema(f, f, 4, i32, f, f, 0, 0.25f, 0.875f, 0.96f, 1, nullptr, nullptr, nullptr, nullptr, 0, nullptr), SPO_EINVAL);
    EXPECT(spo_tracker_init(f, 4, 1.0f, f, f, nullptr), SPO_EINVAL);
    EXPECT(spo_tracker_init(nullptr, 4, 0.875f, f, f, nullptr), SPO_ENULL);

    // loss
    spo_pg_desc d;
    std::memset(&d, 0, sizeof d);
    EXPECT(spo_pg_loss_fwd(nullptr, f, f, f, nullptr, ws, 0, nullptr), SPO_ENULL);
    EXPECT(spo_pg_loss_fwd(&d, f, f, f, nullptr, ws, 0, nullptr), SPO_EINVAL);  // struct_size
    EXPECT(spo_pg_loss_fwd_workspace_bytes(&d), 0);
    d.struct_size = sizeof d;
    d.dtype = SPO_BF16; d.w_layout = SPO_W_VH; d.T = 512; d.H = 128; d.V = 1000; d.B = 8;
    d.eps_low = 0.2f; d.eps_high = 0.28f;
    EXPECT(spo_pg_loss_fwd(&d, f, f, f, nullptr, ws, 0, nullptr), SPO_ENULL);  // NULL arrays
    d.hidden = d.W = f; d.target = i32; d.old_logp = f; d.adv_norm = f; d.cu_seqlens = i32;
    EXPECT(spo_pg_loss_fwd_workspace_bytes(&d) > 0, 1);
    EXPECT(spo_pg_loss_bwd_workspace_bytes(&d, 0) > 0, 1);
    EXPECT(spo_pg_loss_bwd_workspace_bytes(&d, -1), 0);
    EXPECT(spo_pg_loss_bwd_workspace_bytes(&d, 256) <= spo_pg_loss_bwd_workspace_bytes(&d, 512), 1);
    EXPECT(spo_pg_loss_fwd(&d, f, f, f, nullptr, nullptr, 0, nullptr), SPO_EWORKSPACE);
    EXPECT(spo_pg_loss_fwd(&d, f, f, f, nullptr, odd, 1 << 20, nullptr), SPO_EINVAL);
    EXPECT(spo_pg_loss_fwd(&d, f, f, f, nullptr, ws, 16, nullptr), SPO_EWORKSPACE);
    EXPECT(spo_pg_loss_fwd(&d, nullptr, f, f, nullptr, ws, 1 << 20, nullptr), SPO_ENULL);
    EXPECT(spo_pg_loss_bwd(&d, f, f, 1.0f, f, SPO_BF16, f, SPO_FP32, 0, nullptr, -5, ws, 1 << 20, nullptr), SPO_EINVAL);
    EXPECT(spo_pg_loss_bwd(&d, f, f, 1.0f, f, 7, f, SPO_FP32, 0, nullptr, 0, ws, 1 << 20, nullptr), SPO_EINVAL);
    EXPECT(spo_pg_loss_bwd(&d, f, f, 1.0f, f, SPO_BF16, f, SPO_BF16, 1, nullptr, 0, ws, 1 << 20, nullptr), SPO_EINVAL);
    EXPECT(spo_pg_loss_bwd(&d, f, f, 1.0f, f, SPO_BF16, f, SPO_FP32, 0, nullptr, 0, ws, 16, nullptr), SPO_EWORKSPACE);
    EXPECT(spo_pg_loss_fwd_bwd_workspace_bytes(&d, 0) > 0, 1);
    EXPECT(spo_pg_loss_fwd_bwd_workspace_bytes(&d, -1), 0);
    EXPECT(spo_pg_loss_fwd_bwd(&d, 1.0f, f, f, f, nullptr, f, SPO_BF16, f, SPO_FP32, 0, -5, ws, 1 << 20, nullptr), SPO_EINVAL);
    EXPECT(spo_pg_loss_fwd_bwd(&d, 1.0f, f, f, f, nullptr, f, 7, f, SPO_FP32, 0, 0, ws, 1 << 20, nullptr), SPO_EINVAL);
    EXPECT(spo_pg_loss_fwd_bwd(&d, 1.0f, f, f, f, nullptr, f, SPO_BF16, f, SPO_BF16, 1, 0, ws, 1 << 20, nullptr), SPO_EINVAL);
    EXPECT(spo_pg_loss_fwd_bwd(&d, 1.0f, nullptr, f, f, nullptr, f, SPO_BF16, f, SPO_FP32, 0, 0, ws, 1 << 20, nullptr), SPO_ENULL);
    EXPECT(spo_pg_loss_fwd_bwd(&d, 1.0f, f, f, f, nullptr, f, SPO_BF16, f, SPO_FP32, 0, 0, ws, 16, nullptr), SPO_EWORKSPACE);
    EXPECT(spo_pg_loss_fwd_bwd(&d, 1.0f, f, f, f, nullptr, f, SPO_BF16, f, SPO_FP32, 0, 0, odd, 1 << 20, nullptr), SPO_EINVAL);
    d.H = 100;
    EXPECT(spo_pg_loss_fwd(&d, f, f, f, nullptr, ws, 1 << 20, nullptr), SPO_EUNSUPPORTED);
    d.H = 128; d.eps_low = -0.1f;
    EXPECT(spo_pg_loss_fwd(&d, f, f, f, nullptr, ws, 1 << 20, nullptr), SPO_EINVAL);
    d.eps_low = 0.2f; d.V = int64_t(1) << 31;
    EXPECT(spo_pg_loss_fwd(&d, f, f, f, nullptr, ws, 1 << 20, nullptr), SPO_ERANGE);
    d.V = 1000; d.dtype = 9;
    EXPECT(spo_pg_loss_fwd(&d, f, f, f, nullptr, ws, 1 << 20, nullptr), SPO_EINVAL);
    // logits-in form
    d.dtype = SPO_BF16; d.logits = f; d.hidden = d.W = nullptr; d.H = 0;
    EXPECT(spo_pg_loss_fwd_workspace_bytes(&d) > 0, 1);
    EXPECT(spo_pg_loss_fwd(&d, f, f, f, nullptr, ws, 16, nullptr), SPO_EWORKSPACE);
    EXPECT(spo_pg_loss_fwd_bwd_workspace_bytes(&d, 0), 0);
    EXPECT(spo_pg_loss_fwd_bwd(&d, 1.0f, f, f, f, nullptr, f, SPO_BF16, f, SPO_FP32, 0, 0, ws, 1 << 20, nullptr), SPO_EUNSUPPORTED);

    // timing aid
    EXPECT(spo_kernel_timing_enable(0), SPO_OK);
    EXPECT(spo_kernel_timing_read(nullptr, nullptr), SPO_ENULL);
    float ms[SPO_TIMING_CLASSES];
    int32_t n[SPO_TIMING_CLASSES];
    EXPECT(spo_kernel_timing_read(ms, n), SPO_OK);

    if (failures) return 1;
    std::printf("ABI host-side sanitizer run ok\n");
    return 0;
}
