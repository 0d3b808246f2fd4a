// Pieces shared by the fused and the logits-in forms of the clipped
// policy-gradient loss: the per-token surrogate, the masked reduction and the
// per-token gradient scale (Method, PPO-Clip objective with the normalised
// advantage of a response applied to each of its tokens).
#pragma once

#include "common.hpp"

namespace spo {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;  // finite stand-in for -inf in running maxima
constexpr int kTokThreads = 256;

struct Surrogate {
    float ratio, obj;
    bool active;  // the unclipped branch is the minimum: gradient flows
};

__device__ __forceinline__ Surrogate surrogate(float logp, float old_logp, float adv, float eps_low, float eps_high) {
    Surrogate r;
    r.ratio = expf(logp - old_logp);
    const float s1 = r.ratio * adv;
    const float c = fminf(fmaxf(r.ratio, 1.0f - eps_low), 1.0f + eps_high);
    const float s2 = c * adv;
    r.active = s1 <= s2;
    r.obj = r.active ? s1 : s2;
    return r;
}

// Per-block partial sums of the forward, reduced later in block order.
struct FwdPartial {
    double sum_obj, count, clipped, sum_ratio;
};

// One thread per token: merges the per-split (running max, sum of exponentials)
// pairs into lse, forms logp and the surrogate, and reduces this block's masked
// sums.  z_target[t] is the logit of the sampled token.  The per-token arrays start at token
// t_base of the batch (a multiple of the block size; 0 unless the batch is walked in pieces).
static __global__ void __launch_bounds__(kTokThreads)
token_loss_kernel(const float *__restrict__ part_max, const float *__restrict__ part_sum, int nsplit,
                  int64_t split_stride, const float *__restrict__ z_target, int64_t T,
                  const float *__restrict__ old_logp, const uint8_t *__restrict__ mask,
                  const float *__restrict__ adv_norm, const int32_t *__restrict__ cu, int B, float eps_low,
                  float eps_high, float *__restrict__ logp_out, float *__restrict__ lse_out,
                  FwdPartial *__restrict__ partials, int64_t t_base = 0) {
    __shared__ double scratch[kTokThreads / kWave];
    const int64_t t = static_cast<int64_t>(blockIdx.x) * kTokThreads + threadIdx.x;
    double so = 0.0, cnt = 0.0, clp = 0.0, sr = 0.0;
    if (t < T) {
        float mx = kNegBig;
        for (int i = 0; i < nsplit; ++i) mx = fmaxf(mx, part_max[i * split_stride + t]);
        float s = 0.0f;
        for (int i = 0; i < nsplit; ++i) s += part_sum[i * split_stride + t] * expf(part_max[i * split_stride + t] - mx);
        const float lse = mx + logf(s);
        const float logp = z_target[t] - lse;
        lse_out[t] = lse;
        logp_out[t] = logp;
        if (!mask || mask[t]) {
            const float adv = adv_norm[response_of_token(cu, B, t_base + t)];
            const Surrogate r = surrogate(logp, old_logp[t], adv, eps_low, eps_high);
            so = logp == logp ? r.obj : logp;  // a NaN log-prob (target id outside the vocabulary) reaches the loss
            cnt = 1.0;
            clp = r.active ? 0.0 : 1.0;
            sr = r.ratio;
        }
    }
    so = block_sum(so, scratch);
    cnt = block_sum(cnt, scratch);
    clp = block_sum(clp, scratch);
    sr = block_sum(sr, scratch);
    if (threadIdx.x == 0) partials[blockIdx.x] = FwdPartial{so, cnt, clp, sr};
}

// One workgroup sums the block partials in a fixed order and writes the loss.
static __global__ void __launch_bounds__(kTokThreads)
loss_finalize_kernel(const FwdPartial *__restrict__ partials, int64_t nblocks, float *__restrict__ loss,
                     float *__restrict__ stats) {
    __shared__ double scratch[kTokThreads / kWave];
    double so = 0.0, cnt = 0.0, clp = 0.0, sr = 0.0;
    for (int64_t i = threadIdx.x; i < nblocks; i += kTokThreads) {
        const FwdPartial p = partials[i];
        so += p.sum_obj; cnt += p.count; clp += p.clipped; sr += p.sum_ratio;
    }
    so = block_sum(so, scratch);
    cnt = block_sum(cnt, scratch);
    clp = block_sum(clp, scratch);
    sr = block_sum(sr, scratch);
    if (threadIdx.x == 0) {
        loss[0] = cnt > 0.0 ? static_cast<float>(-so / cnt) : 0.0f;
        if (stats) {
            stats[0] = static_cast<float>(cnt);
            stats[1] = cnt > 0.0 ? static_cast<float>(clp / cnt) : 0.0f;
            stats[2] = cnt > 0.0 ? static_cast<float>(sr / cnt) : 0.0f;
            stats[3] = static_cast<float>(so);
        }
    }
}

// count[0] = number of unmasked tokens.  One workgroup, fixed order.
static __global__ void __launch_bounds__(1024)
mask_count_kernel(const uint8_t *__restrict__ mask, int64_t T, double *__restrict__ count) {
    __shared__ double scratch[1024 / kWave];
    double c = 0.0;
    if (mask) {
        for (int64_t t = threadIdx.x; t < T; t += 1024) c += mask[t] ? 1.0 : 0.0;
        c = block_sum(c, scratch);
    } else {
        c = static_cast<double>(T);
    }
    if (threadIdx.x == 0) count[0] = c;
}

// g[t] = -(mask_t / M) * A * ratio_t * [unclipped branch is the minimum] * grad_loss;
// entries T <= t < T_pad are zero so that padded tokens contribute nothing.  t_base as above.
static __global__ void __launch_bounds__(kTokThreads)
grad_scale_kernel(const float *__restrict__ logp, const float *__restrict__ old_logp,
                  const uint8_t *__restrict__ mask, const float *__restrict__ adv_norm,
                  const int32_t *__restrict__ cu, int B, int64_t T, int64_t T_pad, float eps_low, float eps_high,
                  float grad_loss, const double *__restrict__ count, float *__restrict__ g, int64_t t_base = 0) {
    const int64_t t = static_cast<int64_t>(blockIdx.x) * kTokThreads + threadIdx.x;
    if (t >= T_pad) return;
    float out = 0.0f;
    const double M = count[0];
    if (t < T && M > 0.0 && (!mask || mask[t])) {
        const float adv = adv_norm[response_of_token(cu, B, t_base + t)];
        const Surrogate r = surrogate(logp[t], old_logp[t], adv, eps_low, eps_high);
        if (r.active) out = -(adv * r.ratio * grad_loss) / static_cast<float>(M);
    }
    g[t] = out;
}

// Host-side checks common to forward and backward.
static inline int validate_pg_desc(const spo_pg_desc *d) {
    if (!d) return SPO_ENULL;
    if (d->struct_size != sizeof(spo_pg_desc)) return SPO_EINVAL;
    if (d->dtype != SPO_BF16 && d->dtype != SPO_FP32) return SPO_EINVAL;
    if (d->T < 0 || d->V < 1 || d->B < 1) return SPO_EINVAL;
    if (d->T >= (int64_t(1) << 31) || d->V >= (int64_t(1) << 31)) return SPO_ERANGE;
    if (!(d->eps_low >= 0.0f) || !(d->eps_high >= 0.0f)) return SPO_EINVAL;
    if (!d->adv_norm || !d->cu_seqlens) return SPO_ENULL;
    if (d->T > 0 && (!d->target || !d->old_logp)) return SPO_ENULL;
    if (!d->logits) {
        if (d->w_layout != SPO_W_VH && d->w_layout != SPO_W_HV) return SPO_EINVAL;
        if (!d->W || (d->T > 0 && !d->hidden)) return SPO_ENULL;
        if (d->H < 1) return SPO_EINVAL;
        if (d->H % 64 != 0) return SPO_EUNSUPPORTED;
        if (d->H > 65536) return SPO_ERANGE;
    }
    return SPO_OK;
}

}  // namespace spo
