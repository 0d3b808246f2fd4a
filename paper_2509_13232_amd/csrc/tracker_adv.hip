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

constexpr int32_t kNoOwner = 0x7fffffff;
constexpr int kInfoRange = 1, kInfoRepeat = 2;  // bits of info[0]

__global__ void __launch_bounds__(256) fill_slots_kernel(int32_t *__restrict__ slot, int64_t N) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < N) slot[i] = kNoOwner;
}

__global__ void clear_info_kernel(int32_t *__restrict__ info) { info[0] = 0; }

// One thread per observation; ids are unique, so every thread owns its entry.  An id outside
// [0, N) is skipped and flagged.  With a slot table (all kNoOwner) a repeated id is flagged too:
// every observation files its number under its id and the ones that find another there raise
// the flag (the entries are left filed; the table is refilled before its next use).
template <bool Ema>
__global__ void __launch_bounds__(256)
tracker_update_unique_kernel(float *__restrict__ alpha, float *__restrict__ beta, int64_t N,
                             const int32_t *__restrict__ idx, const float *__restrict__ reward,
                             const float *__restrict__ kl, int B, double d_half, double rho_min,
                             double rho_max, uint32_t *__restrict__ n_obs,
                             float *__restrict__ v_prev, int32_t *__restrict__ info,
                             int32_t *__restrict__ slot) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= B) return;
    const int64_t i = idx[k];
    if (i < 0 || i >= N) {
        if (info) atomicOr(&info[0], kInfoRange);
        if (v_prev) v_prev[k] = __builtin_nanf("");
        return;
    }
    if (slot && info && atomicExch(&slot[i], k) != kNoOwner) atomicOr(&info[0], kInfoRepeat);
    float a = alpha[i], b = beta[i];
    if (v_prev) v_prev[k] = mean_of<Ema>(a, b);
    apply<Ema>(a, b, reward[k], discount(kl[k], d_half, rho_min, rho_max));
    alpha[i] = a;
    beta[i] = b;
    if (n_obs) n_obs[i] += 1u;
}

// Repeated ids, applied one after the other in batch order.  One workgroup works in rounds: every
// pending observation files its number under its id with an atomic minimum (slot table, all
// kNoOwner on entry and again on exit); the observation that finds its own number there is the
// earliest pending one of its id and is applied, by one thread, with no other thread touching that
// entry in this round.  The number of rounds is the largest number of repeats of an id (8 for
// batches that sample every prompt 8 times), the work per round the batch size; a batch larger
// than 32768 observations is taken in windows of that many, in order.  The minimum does not
// depend on the order of the atomics: the result is the same on every run.  Tracker entries and
// slots are read and written with L2-coherent accesses, since a later round's thread must see
// what an earlier round's thread wrote.
constexpr int kRoundThreads = 1024, kRoundPer = 32;

template <bool Ema>
__global__ void __launch_bounds__(kRoundThreads)
tracker_update_rounds_kernel(float *__restrict__ alpha, float *__restrict__ beta, int64_t N,
                             const int32_t *__restrict__ idx, const float *__restrict__ reward,
                             const float *__restrict__ kl, int B, double d_half, double rho_min,
                             double rho_max, uint32_t *__restrict__ n_obs, float *__restrict__ v_prev,
                             int32_t *__restrict__ info, int32_t *__restrict__ slot) {
    __shared__ int pending_flag[2];
    auto ld = [](const float *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
    auto st = [](float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
    if (threadIdx.x == 0) { pending_flag[0] = 0; pending_flag[1] = 0; }
    __syncthreads();
    for (int64_t w0 = 0; w0 < B; w0 += static_cast<int64_t>(kRoundThreads) * kRoundPer) {
        // observation j of this thread in the window: k = w0 + j * kRoundThreads + tid
        uint32_t pending = 0;
        for (int j = 0; j < kRoundPer; ++j) {
            const int64_t k = w0 + static_cast<int64_t>(j) * kRoundThreads + threadIdx.x;
            if (k >= B) break;
            const int64_t i = idx[k];
            if (i < 0 || i >= N) {
                if (info) atomicOr(&info[0], kInfoRange);
                if (v_prev) v_prev[k] = __builtin_nanf("");
            } else {
                pending |= 1u << j;
            }
        }
        for (int round = 0;; ++round) {
            for (int j = 0; j < kRoundPer; ++j)
                if (pending >> j & 1u) {
                    const int k = static_cast<int>(w0 + static_cast<int64_t>(j) * kRoundThreads + threadIdx.x);
                    atomicMin(&slot[idx[k]], k);
                }
            __threadfence();
            __syncthreads();  // every claim of this round is filed
            uint32_t won = 0;
            for (int j = 0; j < kRoundPer; ++j)
                if (pending >> j & 1u) {
                    const int k = static_cast<int>(w0 + static_cast<int64_t>(j) * kRoundThreads + threadIdx.x);
                    if (__hip_atomic_load(&slot[idx[k]], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == k) won |= 1u << j;
                }
            __syncthreads();  // every claim has been read
            for (int j = 0; j < kRoundPer; ++j)
                if (won >> j & 1u) {
                    const int k = static_cast<int>(w0 + static_cast<int64_t>(j) * kRoundThreads + threadIdx.x);
                    const int32_t i = idx[k];
                    __hip_atomic_store(&slot[i], kNoOwner, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    float a = ld(&alpha[i]), b = ld(&beta[i]);
                    if (v_prev) v_prev[k] = mean_of<Ema>(a, b);
                    apply<Ema>(a, b, reward[k], discount(kl[k], d_half, rho_min, rho_max));
                    st(&alpha[i], a);
                    st(&beta[i], b);
                    if (n_obs) atomicAdd(&n_obs[i], 1u);
                }
            pending &= ~won;
            int *flag = &pending_flag[round & 1];
            if (pending) *flag = 1;
            __threadfence();
            __syncthreads();  // the slots are clear again, the updates are visible, the flag is complete
            const bool again = *flag != 0;
            if (threadIdx.x == 0) pending_flag[(round + 1) & 1] = 0;
            __syncthreads();
            if (!again) break;
        }
    }
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

// Raw advantage of response k in fp64.  An id outside [0, N) reads nothing: its baseline is NaN
// (so are the batch statistics) and it is flagged.
__device__ __forceinline__ double raw_advantage(const float *__restrict__ alpha, const float *__restrict__ beta,
                                                const int32_t *__restrict__ idx, const float *__restrict__ reward,
                                                int use_baseline, int64_t N, int32_t *__restrict__ info, int k) {
    double v = 0.0;
    if (use_baseline) {
        const int64_t i = idx[k];
        if (i < 0 || i >= N) {
            if (info) info[0] = kInfoRange;
            return __builtin_nan("");
        }
        const double a = alpha[i];
        v = beta ? a / (a + static_cast<double>(beta[i])) : a;
    }
    return static_cast<double>(reward[k]) - v;
}

// One workgroup: raw advantages, then mean and standard deviation in fp64 with a
// fixed reduction order, then the normalised values.  The centred second pass
// avoids the cancellation of the sum-of-squares shortcut.
constexpr int kAdvThreads = 1024;

__global__ void __launch_bounds__(kAdvThreads)
advantages_kernel(const float *__restrict__ alpha, const float *__restrict__ beta,
                  const int32_t *__restrict__ idx, const float *__restrict__ reward, int B, int ddof,
                  double eps_norm, int use_baseline, float *__restrict__ adv_raw,
                  float *__restrict__ adv_norm, float *__restrict__ stats, int64_t N, int32_t *__restrict__ info) {
    __shared__ double scratch[kAdvThreads / kWave];
    auto raw = [&](int k) { return raw_advantage(alpha, beta, idx, reward, use_baseline, N, info, k); };
    if (info && threadIdx.x == 0) info[0] = 0;
    __syncthreads();
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
        adv_norm[k] = den == 0.0 ? 0.0f : static_cast<float>((raw(k) - mu) / den);  // den is >= 0, or NaN and says so
    if (stats && threadIdx.x == 0) {
        stats[0] = static_cast<float>(mu);
        stats[1] = static_cast<float>(sigma);
    }
}

// The same over many workgroups, for large batches: three launches, each workgroup over kAdvSpan
// responses.  part[0..nb) are the workgroups' sums of the raw advantages, part[nb..2nb) their
// sums of centred squares; every workgroup adds the partial sums it needs in the same fixed
// order, so all of them hold the same mean and deviation, bit for bit, in every run.  (The order
// differs from the one-workgroup kernel's: the two agree to fp64 rounding, not bitwise.)
constexpr int kAdvSpan = 4096;

__device__ __forceinline__ double ordered_total(const double *__restrict__ part, int nb, double *scratch) {
    double s = 0.0;
    for (int i = threadIdx.x; i < nb; i += kAdvThreads) s += part[i];
    return block_sum(s, scratch);
}

// phase 0: raw advantages and their partial sums; phase 1: partial sums of centred squares;
// phase 2: normalised values and the statistics
template <int Phase>
__global__ void __launch_bounds__(kAdvThreads)
advantages_wide_kernel(const float *__restrict__ alpha, const float *__restrict__ beta,
                       const int32_t *__restrict__ idx, const float *__restrict__ reward, int B, int ddof,
                       double eps_norm, int use_baseline, float *__restrict__ adv_raw, float *__restrict__ adv_norm,
                       float *__restrict__ stats, int64_t N, int32_t *__restrict__ info, double *__restrict__ part) {
    __shared__ double scratch[kAdvThreads / kWave];
    const int nb = gridDim.x;
    const int k0 = blockIdx.x * kAdvSpan, k1 = k0 + kAdvSpan < B ? k0 + kAdvSpan : B;
    auto raw = [&](int k) { return raw_advantage(alpha, beta, idx, reward, use_baseline, N, info, k); };
    if (Phase == 0) {
        double s = 0.0;
        for (int k = k0 + threadIdx.x; k < k1; k += kAdvThreads) {
            const double a = raw(k);
            if (adv_raw) adv_raw[k] = static_cast<float>(a);
            s += a;
        }
        s = block_sum(s, scratch);
        if (threadIdx.x == 0) part[blockIdx.x] = s;
        return;
    }
    const double mu = ordered_total(part, nb, scratch) / static_cast<double>(B);
    if (Phase == 1) {
        double ss = 0.0;
        for (int k = k0 + threadIdx.x; k < k1; k += kAdvThreads) {
            const double d = raw(k) - mu;
            ss += d * d;
        }
        ss = block_sum(ss, scratch);
        if (threadIdx.x == 0) part[nb + blockIdx.x] = ss;
        return;
    }
    const double dn = static_cast<double>(B - ddof);
    const double ss = ordered_total(part + nb, nb, scratch);
    const double sigma = dn > 0.0 ? sqrt(ss / dn) : 0.0;
    const double den = sigma + eps_norm;
    for (int k = k0 + threadIdx.x; k < k1; k += kAdvThreads)
        adv_norm[k] = den == 0.0 ? 0.0f : static_cast<float>((raw(k) - mu) / den);  // den is >= 0, or NaN and says so
    if (stats && blockIdx.x == 0 && threadIdx.x == 0) {
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

static size_t slot_table_bytes(int64_t N) { return align_up(static_cast<size_t>(N) * sizeof(int32_t), 256); }

template <bool Ema>
static int tracker_update_launch(float *alpha, float *beta, int64_t N, const int32_t *idx,
                                 const float *reward, const float *kl, int32_t B, float d_half,
                                 float rho_min, float rho_max, int ids_unique, uint32_t *n_obs,
                                 float *v_prev_out, int32_t *info, void *ws, size_t ws_bytes,
                                 spo_stream_t stream) {
    if (!alpha || !beta || !idx || !reward || !kl) return SPO_ENULL;
    if (N < 1 || N >= (int64_t(1) << 31) || B < 1) return SPO_EINVAL;
    if (!(d_half > 0.0f) || !(rho_min >= 0.0f) || !(rho_max <= 1.0f) || !(rho_min <= rho_max))
        return SPO_EINVAL;
    if (ws && (reinterpret_cast<uintptr_t>(ws) % 256 != 0)) return SPO_EINVAL;
    if ((ws || !ids_unique) && (!ws || ws_bytes < slot_table_bytes(N))) return SPO_EWORKSPACE;
    hipStream_t s = as_stream(stream);
    int32_t *slot = static_cast<int32_t *>(ws);
    if (info) clear_info_kernel<<<1, 1, 0, s>>>(info);
    if (slot) fill_slots_kernel<<<static_cast<unsigned>(ceil_div(N, 256)), 256, 0, s>>>(slot, N);
    if (ids_unique) {
        const int threads = 256, blocks = (B + threads - 1) / threads;
        tracker_update_unique_kernel<Ema><<<blocks, threads, 0, s>>>(alpha, beta, N, idx, reward, kl, B, d_half, rho_min,
                                                                      rho_max, n_obs, v_prev_out, info, slot);
    } else {
        tracker_update_rounds_kernel<Ema><<<1, kRoundThreads, 0, s>>>(alpha, beta, N, idx, reward, kl, B, d_half, rho_min,
                                                                       rho_max, n_obs, v_prev_out, info, slot);
    }
    return launch_status();
}

extern "C" size_t spo_tracker_update_workspace_bytes(int64_t N) { return N < 1 ? 0 : slot_table_bytes(N); }

extern "C" int spo_tracker_update(float *alpha, float *beta, int64_t N, const int32_t *idx,
                                  const float *reward, const float *kl, int32_t B, float d_half,
                                  float rho_min, float rho_max, int ids_unique, uint32_t *n_obs,
                                  float *v_prev_out, int32_t *info, void *ws, size_t ws_bytes,
                                  spo_stream_t stream) {
    return tracker_update_launch<false>(alpha, beta, N, idx, reward, kl, B, d_half, rho_min, rho_max,
                                        ids_unique, n_obs, v_prev_out, info, ws, ws_bytes, stream);
}

extern "C" int spo_tracker_update_ema(float *v_hat, float *n_eff, int64_t N, const int32_t *idx,
                                      const float *reward, const float *kl, int32_t B, float d_half,
                                      float rho_min, float rho_max, int ids_unique, uint32_t *n_obs,
                                      float *v_prev_out, int32_t *info, void *ws, size_t ws_bytes,
                                      spo_stream_t stream) {
    return tracker_update_launch<true>(v_hat, n_eff, N, idx, reward, kl, B, d_half, rho_min, rho_max,
                                       ids_unique, n_obs, v_prev_out, info, ws, ws_bytes, stream);
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

constexpr int kAdvWideMin = 4 * kAdvSpan;  // below this one workgroup is as fast

extern "C" size_t spo_advantages_workspace_bytes(int32_t B) {
    if (B < 1) return 0;
    return static_cast<size_t>(2 * ceil_div(B, kAdvSpan)) * sizeof(double);
}

extern "C" int spo_advantages(const float *alpha, const float *beta, int64_t N, const int32_t *idx,
                              const float *reward, int32_t B, int ddof, float eps_norm,
                              int use_baseline, float *adv_raw, float *adv_norm, float *stats,
                              int32_t *info, void *ws, size_t ws_bytes, spo_stream_t stream) {
    if (!reward || !adv_norm) return SPO_ENULL;
    if (use_baseline && (!alpha || !idx)) return SPO_ENULL;
    if (B < 1 || (use_baseline && N < 1) || ddof < 0 || ddof > 1 || !(eps_norm >= 0.0f))
        return SPO_EINVAL;
    if (ws && reinterpret_cast<uintptr_t>(ws) % 256 != 0) return SPO_EINVAL;
    if (ws && ws_bytes < spo_advantages_workspace_bytes(B)) return SPO_EWORKSPACE;
    hipStream_t s = as_stream(stream);
    if (!ws || B < kAdvWideMin) {
        advantages_kernel<<<1, kAdvThreads, 0, s>>>(alpha, beta, idx, reward, B, ddof, eps_norm, use_baseline, adv_raw,
                                                    adv_norm, stats, N, info);
        return launch_status();
    }
    const unsigned nb = static_cast<unsigned>(ceil_div(B, kAdvSpan));
    double *part = static_cast<double *>(ws);
    if (info) clear_info_kernel<<<1, 1, 0, s>>>(info);
    advantages_wide_kernel<0><<<nb, kAdvThreads, 0, s>>>(alpha, beta, idx, reward, B, ddof, eps_norm, use_baseline,
                                                        adv_raw, adv_norm, stats, N, info, part);
    advantages_wide_kernel<1><<<nb, kAdvThreads, 0, s>>>(alpha, beta, idx, reward, B, ddof, eps_norm, use_baseline,
                                                        adv_raw, adv_norm, stats, N, info, part);
    advantages_wide_kernel<2><<<nb, kAdvThreads, 0, s>>>(alpha, beta, idx, reward, B, ddof, eps_norm, use_baseline,
                                                        adv_raw, adv_norm, stats, N, info, part);
    return launch_status();
}
