// Logits-in form of the clipped policy-gradient loss: the [T x V] logits already
// exist and are streamed once (forward) or read once and written once
// (backward).  Pure HBM streaming; one workgroup per token row, 16-byte accesses.
#include <algorithm>

#include "pg_common.hpp"
#include "timing.hpp"

namespace spo {

constexpr int kRowThreads = 256;

template <typename T> struct Vec;
template <> struct Vec<bf16_t> {
    static constexpr int N = 8;
    __device__ static __forceinline__ void load(const bf16_t *p, float (&x)[8]) {
        const uint4 u = *reinterpret_cast<const uint4 *>(p);
        const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = __uint_as_float(w[i] << 16);
            x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    __device__ static __forceinline__ void store(bf16_t *p, const float (&x)[8]) {
        uint4 u;
        u.x = pack_bf16x2(x[0], x[1]); u.y = pack_bf16x2(x[2], x[3]);
        u.z = pack_bf16x2(x[4], x[5]); u.w = pack_bf16x2(x[6], x[7]);
        *reinterpret_cast<uint4 *>(p) = u;
    }
    __device__ static __forceinline__ float get(const bf16_t *p) { return bf16_to_f32(*p); }
    __device__ static __forceinline__ void put(bf16_t *p, float v) { *p = f32_to_bf16(v); }
};
template <> struct Vec<float> {
    static constexpr int N = 4;
    __device__ static __forceinline__ void load(const float *p, float (&x)[4]) {
        const float4 u = *reinterpret_cast<const float4 *>(p);
        x[0] = u.x; x[1] = u.y; x[2] = u.z; x[3] = u.w;
    }
    __device__ static __forceinline__ void store(float *p, const float (&x)[4]) {
        *reinterpret_cast<float4 *>(p) = make_float4(x[0], x[1], x[2], x[3]);
    }
    __device__ static __forceinline__ float get(const float *p) { return *p; }
    __device__ static __forceinline__ void put(float *p, float v) { *p = v; }
};

// running (max, sum of exp(x - max)) with one more value / merged with another pair
__device__ __forceinline__ void lse_merge(float &m, float &s, float om, float os) {
    const float nm = fmaxf(m, om);
    s = s * __builtin_amdgcn_exp2f((m - nm) * kLog2e) + os * __builtin_amdgcn_exp2f((om - nm) * kLog2e);
    m = nm;
}

// One row per workgroup: (max, sum-exp) of the row and the target's logit.
template <typename T, bool kVector>
__global__ void __launch_bounds__(kRowThreads)
logits_row_lse_kernel(const T *__restrict__ logits, int64_t V, const int32_t *__restrict__ target,
                      float *__restrict__ row_max, float *__restrict__ row_sum, float *__restrict__ z_target) {
    __shared__ float sm[kRowThreads / kWave], ss[kRowThreads / kWave];
    constexpr int N = Vec<T>::N;
    const int64_t t = blockIdx.x;
    const T *row = logits + t * V;
    float m = kNegBig, s = 0.0f;
    if (kVector) {
        // four independent 16-byte loads in flight per thread before any of them is used
        constexpr int U = 4;
        const int64_t step = static_cast<int64_t>(kRowThreads) * N;
        for (int64_t v0 = static_cast<int64_t>(threadIdx.x) * N; v0 < V; v0 += U * step) {
            float x[U][N];
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (v0 + u * step < V) Vec<T>::load(row + v0 + u * step, x[u]);
            // one new maximum and one rescaling of the running sum for the whole group of loads
            float mx = m;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (v0 + u * step >= V) break;
#pragma unroll
                for (int i = 0; i < N; ++i) mx = fmaxf(mx, x[u][i]);
            }
            const float nm2 = -mx * kLog2e;
            float a = 0.0f;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (v0 + u * step >= V) break;
#pragma unroll
                for (int i = 0; i < N; ++i) a += __builtin_amdgcn_exp2f(fmaf(x[u][i], kLog2e, nm2));
            }
            s = s * __builtin_amdgcn_exp2f((m - mx) * kLog2e) + a;
            m = mx;
        }
    } else {
        for (int64_t v = threadIdx.x; v < V; v += kRowThreads) lse_merge(m, s, Vec<T>::get(row + v), 1.0f);
    }
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) lse_merge(m, s, __shfl_xor(m, o, kWave), __shfl_xor(s, o, kWave));
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { sm[wave] = m; ss[wave] = s; }
    __syncthreads();
    if (threadIdx.x == 0) {
        float M = sm[0], S = ss[0];
        for (int w = 1; w < kRowThreads / kWave; ++w) lse_merge(M, S, sm[w], ss[w]);
        row_max[t] = M;
        row_sum[t] = S;
        const int64_t y = target[t];  // an id outside [0, V) gives NaN instead of a read out of bounds
        z_target[t] = (y >= 0 && y < V) ? Vec<T>::get(row + y) : __builtin_nanf("");
    }
}

// d_logits[t][v] = g[t] * ([v == target[t]] - exp(z[t][v] - lse[t])); rows whose
// scale is zero are written as zeros without being read.
template <typename T, bool kVector>
__global__ void __launch_bounds__(kRowThreads)
logits_row_grad_kernel(const T *__restrict__ logits, int64_t V, const int32_t *__restrict__ target,
                       const float *__restrict__ lse, const float *__restrict__ g, T *__restrict__ d_logits) {
    constexpr int N = Vec<T>::N;
    const int64_t t = blockIdx.x;
    const T *row = logits + t * V;
    T *out = d_logits + t * V;
    const float gt = g[t], nl = -lse[t] * kLog2e;
    const int64_t y = target[t];
    if (kVector) {
        constexpr int U = 4;
        const int64_t step = static_cast<int64_t>(kRowThreads) * N;
        for (int64_t v0 = static_cast<int64_t>(threadIdx.x) * N; v0 < V; v0 += U * step) {
            float x[U][N];
            if (gt != 0.0f) {
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (v0 + u * step < V) Vec<T>::load(row + v0 + u * step, x[u]);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t v = v0 + u * step;
                if (v >= V) break;
                if (gt != 0.0f) {
#pragma unroll
                    for (int i = 0; i < N; ++i)
                        x[u][i] = (v + i == y ? gt : 0.0f) - gt * __builtin_amdgcn_exp2f(fmaf(x[u][i], kLog2e, nl));
                } else {
#pragma unroll
                    for (int i = 0; i < N; ++i) x[u][i] = 0.0f;
                }
                Vec<T>::store(out + v, x[u]);
            }
        }
    } else {
        for (int64_t v = threadIdx.x; v < V; v += kRowThreads) {
            float x = 0.0f;
            if (gt != 0.0f) x = (v == y ? gt : 0.0f) - gt * __builtin_amdgcn_exp2f(fmaf(Vec<T>::get(row + v), kLog2e, nl));
            Vec<T>::put(out + v, x);
        }
    }
}

struct LogitsFwdPlan {
    float *row_max, *row_sum, *z_target;
    FwdPartial *partials;
    int64_t nblk_tok;
    size_t bytes;
};

static LogitsFwdPlan plan_logits_fwd(const spo_pg_desc *d, void *ws) {
    LogitsFwdPlan p;
    const int64_t Tn = std::max<int64_t>(d->T, 1);
    p.nblk_tok = ceil_div(Tn, kTokThreads);
    Arena a(ws);
    p.row_max = a.take<float>(Tn);
    p.row_sum = a.take<float>(Tn);
    p.z_target = a.take<float>(Tn);
    p.partials = a.take<FwdPartial>(p.nblk_tok);
    p.bytes = a.used;
    return p;
}

template <typename T>
static bool vector_ok(const void *p, int64_t V) {
    return V % Vec<T>::N == 0 && reinterpret_cast<uintptr_t>(p) % 16 == 0;
}

int logits_fwd_workspace(const spo_pg_desc *d, size_t *bytes) {
    *bytes = plan_logits_fwd(d, nullptr).bytes;
    return SPO_OK;
}

int logits_fwd(const spo_pg_desc *d, float *loss, float *logp, float *lse, float *stats, void *ws,
               size_t ws_bytes, hipStream_t s) {
    const LogitsFwdPlan p = plan_logits_fwd(d, ws);
    if (ws_bytes < p.bytes) return SPO_EWORKSPACE;
    if (d->T > 0) {
        const unsigned rows = static_cast<unsigned>(d->T);
        ScopedKernelTimer timer(kTimeLogitsFwd, s);
        if (d->dtype == SPO_BF16) {
            const bf16_t *lg = static_cast<const bf16_t *>(d->logits);
            if (vector_ok<bf16_t>(lg, d->V))
                logits_row_lse_kernel<bf16_t, true><<<rows, kRowThreads, 0, s>>>(lg, d->V, d->target, p.row_max, p.row_sum, p.z_target);
            else
                logits_row_lse_kernel<bf16_t, false><<<rows, kRowThreads, 0, s>>>(lg, d->V, d->target, p.row_max, p.row_sum, p.z_target);
        } else {
            const float *lg = static_cast<const float *>(d->logits);
            if (vector_ok<float>(lg, d->V))
                logits_row_lse_kernel<float, true><<<rows, kRowThreads, 0, s>>>(lg, d->V, d->target, p.row_max, p.row_sum, p.z_target);
            else
                logits_row_lse_kernel<float, false><<<rows, kRowThreads, 0, s>>>(lg, d->V, d->target, p.row_max, p.row_sum, p.z_target);
        }
    }
    token_loss_kernel<<<static_cast<unsigned>(p.nblk_tok), kTokThreads, 0, s>>>(
        p.row_max, p.row_sum, 1, 0, p.z_target, d->T, d->old_logp, d->mask, d->adv_norm, d->cu_seqlens, d->B,
        d->eps_low, d->eps_high, logp, lse, p.partials);
    loss_finalize_kernel<<<1, kTokThreads, 0, s>>>(p.partials, p.nblk_tok, loss, stats);
    return launch_status();
}

struct LogitsBwdPlan {
    double *count;
    float *g;
    size_t bytes;
};

static LogitsBwdPlan plan_logits_bwd(const spo_pg_desc *d, void *ws) {
    LogitsBwdPlan p;
    Arena a(ws);
    p.count = a.take<double>(1);
    p.g = a.take<float>(std::max<int64_t>(d->T, 1));
    p.bytes = a.used;
    return p;
}

int logits_bwd_workspace(const spo_pg_desc *d, size_t *bytes) {
    *bytes = plan_logits_bwd(d, nullptr).bytes;
    return SPO_OK;
}

int logits_bwd(const spo_pg_desc *d, const float *logp, const float *lse, float grad_loss, void *d_logits,
               void *ws, size_t ws_bytes, hipStream_t s) {
    if (!d_logits) return SPO_ENULL;
    const LogitsBwdPlan p = plan_logits_bwd(d, ws);
    if (ws_bytes < p.bytes) return SPO_EWORKSPACE;
    if (d->T == 0) return SPO_OK;
    mask_count_kernel<<<1, 1024, 0, s>>>(d->mask, d->T, p.count);
    grad_scale_kernel<<<static_cast<unsigned>(ceil_div(d->T, kTokThreads)), kTokThreads, 0, s>>>(
        logp, d->old_logp, d->mask, d->adv_norm, d->cu_seqlens, d->B, d->T, d->T, d->eps_low, d->eps_high, grad_loss,
        p.count, p.g);
    const unsigned rows = static_cast<unsigned>(d->T);
    ScopedKernelTimer timer(kTimeLogitsBwd, s);
    if (d->dtype == SPO_BF16) {
        const bf16_t *lg = static_cast<const bf16_t *>(d->logits);
        bf16_t *dl = static_cast<bf16_t *>(d_logits);
        if (vector_ok<bf16_t>(lg, d->V) && vector_ok<bf16_t>(dl, d->V))
            logits_row_grad_kernel<bf16_t, true><<<rows, kRowThreads, 0, s>>>(lg, d->V, d->target, lse, p.g, dl);
        else
            logits_row_grad_kernel<bf16_t, false><<<rows, kRowThreads, 0, s>>>(lg, d->V, d->target, lse, p.g, dl);
    } else {
        const float *lg = static_cast<const float *>(d->logits);
        float *dl = static_cast<float *>(d_logits);
        if (vector_ok<float>(lg, d->V) && vector_ok<float>(dl, d->V))
            logits_row_grad_kernel<float, true><<<rows, kRowThreads, 0, s>>>(lg, d->V, d->target, lse, p.g, dl);
        else
            logits_row_grad_kernel<float, false><<<rows, kRowThreads, 0, s>>>(lg, d->V, d->target, lse, p.g, dl);
    }
    return launch_status();
}

}  // namespace spo
