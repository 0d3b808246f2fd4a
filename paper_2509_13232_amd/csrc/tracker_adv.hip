// Beta value tracker (update, initialisation) and single-stream advantages.
// Method, "A KL-Adaptive Value Tracker" and "Advantage Estimation and Policy
// Optimization".  Plain ALU work on B <= a few thousand scattered entries:
// launch-latency bound, one small launch each.
#include "common.hpp"

namespace spo {

// rho = 2^(-D/D_half) kept inside [rho_min, rho_max]; fp64 so that the fp32
// result of rho*alpha + r carries a single rounding.
__device__ __forceinline__ double discount(float kl, double d_half, double rho_min, double rho_max) {
    const double d = kl > 0.0f ? static_cast<double>(kl) : 0.0;
    double rho = exp2(-d / d_half);
    rho = rho < rho_min ? rho_min : rho;
    rho = rho > rho_max ? rho_max : rho;
    return rho;
}

__device__ __forceinline__ void observe(float &a, float &b, float r, double rho) {
    const double rd = static_cast<double>(r);
    a = static_cast<float>(rho * static_cast<double>(a) + rd);
    b = static_cast<float>(rho * static_cast<double>(b) + (1.0 - rd));
}

// Moving-average form: v <- v + (r - v)/(rho n + 1), n <- rho n + 1.
__device__ __forceinline__ void observe_ema(float &v, float &n, float r, double rho) {
    const double vd = static_cast<double>(v), nd = static_cast<double>(n);
    const double eta = 1.0 / (rho * nd + 1.0);
    v = static_cast<float>(vd + eta * (static_cast<double>(r) - vd));
    n = static_cast<float>(rho * nd + 1.0);
}

// Both forms of the tracker share the update kernels: Ema = false keeps
// (alpha, beta), Ema = true keeps (v_hat, n_eff) in the same two arrays.
template <bool Ema>
__device__ __forceinline__ float mean_of(float a, float b) {
    if constexpr (Ema) return a;
    return static_cast<float>(static_cast<double>(a) / (static_cast<double>(a) + static_cast<double>(b)));
}

template <bool Ema>
__device__ __forceinline__ void apply(float &a, float &b, float r, double rho) {
    if constexpr (Ema) observe_ema(a, b, r, rho);
    else observe(a, b, r, rho);
}

// One thread per observation; ids are unique, so every thread owns its entry.
template <bool Ema>
__global__ void __launch_bounds__(256)
tracker_update_unique_kernel(float *__restrict__ alpha, float *__restrict__ beta,
                             const int32_t *__restrict__ idx, const float *__restrict__ reward,
                             const float *__restrict__ kl, int B, double d_half, double rho_min,
                             double rho_max, uint32_t *__restrict__ n_obs,
                             float *__restrict__ v_prev) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= B) return;
    const int64_t i = idx[k];
    float a = alpha[i], b = beta[i];
    if (v_prev) v_prev[k] = mean_of<Ema>(a, b);
    apply<Ema>(a, b, reward[k], discount(kl[k], d_half, rho_min, rho_max));
    alpha[i] = a;
    beta[i] = b;
    if (n_obs) n_obs[i] += 1u;
}

// Repeated ids: the thread of the FIRST occurrence of an id applies all of its
// observations one after the other in batch order; other threads do nothing.
template <bool Ema>
__global__ void __launch_bounds__(256)
tracker_update_ordered_kernel(float *__restrict__ alpha, float *__restrict__ beta,
                              const int32_t *__restrict__ idx, const float *__restrict__ reward,
                              const float *__restrict__ kl, int B, double d_half, double rho_min,
                              double rho_max, uint32_t *__restrict__ n_obs,
                              float *__restrict__ v_prev) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= B) return;
    const int32_t id = idx[k];
    for (int j = 0; j < k; ++j)
        if (idx[j] == id) return;  // an earlier thread owns this id
    float a = alpha[id], b = beta[id];
    uint32_t seen = 0;
    for (int j = k; j < B; ++j) {
        if (idx[j] != id) continue;
        if (v_prev) v_prev[j] = mean_of<Ema>(a, b);
        apply<Ema>(a, b, reward[j], discount(kl[j], d_half, rho_min, rho_max));
        ++seen;
    }
    alpha[id] = a;
    beta[id] = b;
    if (n_obs) n_obs[id] += seen;
}

__global__ void __launch_bounds__(256)
tracker_init_kernel(const float *__restrict__ v0, int64_t N, double n0, float *__restrict__ alpha,
                    float *__restrict__ beta) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= N) return;
    const double v = static_cast<double>(v0[i]);
    alpha[i] = static_cast<float>(n0 * v);
    beta[i] = static_cast<float>(n0 * (1.0 - v));
}

// One workgroup: raw advantages, then mean and standard deviation in fp64 with a
// fixed reduction order, then the normalised values.  The centred second pass
// avoids the cancellation of the sum-of-squares shortcut.
constexpr int kAdvThreads = 1024;

__global__ void __launch_bounds__(kAdvThreads)
advantages_kernel(const float *__restrict__ alpha, const float *__restrict__ beta,
                  const int32_t *__restrict__ idx, const float *__restrict__ reward, int B, int ddof,
                  double eps_norm, int use_baseline, float *__restrict__ adv_raw,
                  float *__restrict__ adv_norm, float *__restrict__ stats) {
    __shared__ double scratch[kAdvThreads / kWave];
    auto raw = [&](int k) -> double {
        double v = 0.0;
        if (use_baseline) {
            const int64_t i = idx[k];
            const double a = alpha[i];
            v = beta ? a / (a + static_cast<double>(beta[i])) : a;
        }
        return static_cast<double>(reward[k]) - v;
    };
    double s = 0.0;
    for (int k = threadIdx.x; k < B; k += kAdvThreads) {
        const double a = raw(k);
        if (adv_raw) adv_raw[k] = static_cast<float>(a);
        s += a;
    }
    const double mu = block_sum(s, scratch) / static_cast<double>(B);
    double ss = 0.0;
    for (int k = threadIdx.x; k < B; k += kAdvThreads) {
        const double d = raw(k) - mu;
        ss += d * d;
    }
    ss = block_sum(ss, scratch);
    const double dn = static_cast<double>(B - ddof);
    const double sigma = dn > 0.0 ? sqrt(ss / dn) : 0.0;
    const double den = sigma + eps_norm;
    for (int k = threadIdx.x; k < B; k += kAdvThreads)
        adv_norm[k] = den > 0.0 ? static_cast<float>((raw(k) - mu) / den) : 0.0f;
    if (stats && threadIdx.x == 0) {
        stats[0] = static_cast<float>(mu);
        stats[1] = static_cast<float>(sigma);
    }
}

// Diagnostics of the unnormalised advantages (one workgroup, fp64, fixed order).
__global__ void __launch_bounds__(kAdvThreads)
advantage_diagnostics_kernel(const float *__restrict__ adv_raw, const float *__restrict__ reward, int B,
                             float tau_tight, float tau_loose, float *__restrict__ diag) {
    __shared__ double scratch[kAdvThreads / kWave];
    double nt = 0.0, nl = 0.0, sa = 0.0, sr = 0.0;
    for (int k = threadIdx.x; k < B; k += kAdvThreads) {
        const float a = fabsf(adv_raw[k]);
        nt += a <= tau_tight ? 1.0 : 0.0;
        nl += a <= tau_loose ? 1.0 : 0.0;
        sa += static_cast<double>(adv_raw[k]);
        sr += static_cast<double>(reward[k]);
    }
    nt = block_sum(nt, scratch);
    nl = block_sum(nl, scratch);
    const double ma = block_sum(sa, scratch) / B, mr = block_sum(sr, scratch) / B;
    double va = 0.0, vr = 0.0;
    for (int k = threadIdx.x; k < B; k += kAdvThreads) {
        const double da = static_cast<double>(adv_raw[k]) - ma, dr = static_cast<double>(reward[k]) - mr;
        va += da * da;
        vr += dr * dr;
    }
    va = block_sum(va, scratch);
    vr = block_sum(vr, scratch);
    if (threadIdx.x == 0) {
        diag[0] = static_cast<float>(nt / B);
        diag[1] = static_cast<float>(nl / B);
        diag[2] = static_cast<float>(va / B);
        diag[3] = static_cast<float>(vr / B);
    }
}

}  // namespace spo

using namespace spo;

extern "C" int spo_advantage_diagnostics(const float *adv_raw, const float *reward, int32_t B, float tau_tight,
                                         float tau_loose, float *diag, spo_stream_t stream) {
    if (!adv_raw || !reward || !diag) return SPO_ENULL;
    if (B < 1 || !(tau_tight >= 0.0f) || !(tau_loose >= tau_tight)) return SPO_EINVAL;
    advantage_diagnostics_kernel<<<1, kAdvThreads, 0, as_stream(stream)>>>(adv_raw, reward, B, tau_tight, tau_loose, diag);
    return launch_status();
}

template <bool Ema>
static int tracker_update_launch(float *alpha, float *beta, int64_t N, const int32_t *idx,
                                 const float *reward, const float *kl, int32_t B, float d_half,
                                 float rho_min, float rho_max, int ids_unique, uint32_t *n_obs,
                                 float *v_prev_out, spo_stream_t stream) {
    if (!alpha || !beta || !idx || !reward || !kl) return SPO_ENULL;
    if (N < 1 || N >= (int64_t(1) << 31) || B < 1) return SPO_EINVAL;
    if (!(d_half > 0.0f) || !(rho_min >= 0.0f) || !(rho_max <= 1.0f) || !(rho_min <= rho_max))
        return SPO_EINVAL;
    const int threads = 256, blocks = (B + threads - 1) / threads;
    if (ids_unique)
        tracker_update_unique_kernel<Ema><<<blocks, threads, 0, as_stream(stream)>>>(
            alpha, beta, idx, reward, kl, B, d_half, rho_min, rho_max, n_obs, v_prev_out);
    else
        tracker_update_ordered_kernel<Ema><<<blocks, threads, 0, as_stream(stream)>>>(
            alpha, beta, idx, reward, kl, B, d_half, rho_min, rho_max, n_obs, v_prev_out);
    return launch_status();
}

extern "C" int spo_tracker_update(float *alpha, float *beta, int64_t N, const int32_t *idx,
                                  const float *reward, const float *kl, int32_t B, float d_half,
                                  float rho_min, float rho_max, int ids_unique, uint32_t *n_obs,
                                  float *v_prev_out, spo_stream_t stream) {
    return tracker_update_launch<false>(alpha, beta, N, idx, reward, kl, B, d_half, rho_min, rho_max,
                                        ids_unique, n_obs, v_prev_out, stream);
}

extern "C" int spo_tracker_update_ema(float *v_hat, float *n_eff, int64_t N, const int32_t *idx,
                                      const float *reward, const float *kl, int32_t B, float d_half,
                                      float rho_min, float rho_max, int ids_unique, uint32_t *n_obs,
                                      float *v_prev_out, spo_stream_t stream) {
    return tracker_update_launch<true>(v_hat, n_eff, N, idx, reward, kl, B, d_half, rho_min, rho_max,
                                       ids_unique, n_obs, v_prev_out, stream);
}

extern "C" int spo_tracker_init(const float *v0, int64_t N, float rho_min, float *alpha,
                                float *beta, spo_stream_t stream) {
    if (!v0 || !alpha || !beta) return SPO_ENULL;
    if (N < 1 || !(rho_min >= 0.0f) || !(rho_min < 1.0f)) return SPO_EINVAL;
    const int threads = 256;
    const int64_t blocks = ceil_div(N, threads);
    if (blocks >= (int64_t(1) << 31)) return SPO_ERANGE;
    tracker_init_kernel<<<static_cast<unsigned>(blocks), threads, 0, as_stream(stream)>>>(
        v0, N, 1.0 / (1.0 - static_cast<double>(rho_min)), alpha, beta);
    return launch_status();
}

extern "C" int spo_advantages(const float *alpha, const float *beta, int64_t N, const int32_t *idx,
                              const float *reward, int32_t B, int ddof, float eps_norm,
                              int use_baseline, float *adv_raw, float *adv_norm, float *stats,
                              spo_stream_t stream) {
    if (!reward || !adv_norm) return SPO_ENULL;
    if (use_baseline && (!alpha || !idx)) return SPO_ENULL;
    if (B < 1 || (use_baseline && N < 1) || ddof < 0 || ddof > 1 || !(eps_norm >= 0.0f))
        return SPO_EINVAL;
    advantages_kernel<<<1, kAdvThreads, 0, as_stream(stream)>>>(
        alpha, beta, idx, reward, B, ddof, eps_norm, use_baseline, adv_raw, adv_norm, stats);
    return launch_status();
}
