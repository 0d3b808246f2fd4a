// Prioritized prompt sampling: weights -> exact integer CDF -> Philox draws.
// Method, "Prioritized Prompt Sampling" (sampling-weight equation and the batch
// draw of the training loop).  The O(N) part (weights + scan) streams the tracker
// once per phase; the draw itself is B binary searches.
//
// Everything that decides an index is integer arithmetic or a single correctly
// rounded IEEE fp64 operation (add, divide, subtract, multiply, sqrt: no fused
// multiply-add can form because no product feeds an addition), so the indices do
// not depend on the machine, the launch shape or the order of summation.
#include <mutex>

#include "common.hpp"

namespace spo {

constexpr int kScanThreads = 256;
constexpr int kScanRows = 16;                               // rows of 256 items per block
constexpr int kScanItems = kScanThreads * kScanRows;        // 4096 items per block
constexpr int kMaxSlotsNoReplace = 16384;
constexpr int kResolveThreads = 1024;
constexpr int kSlotsPerThread = kMaxSlotsNoReplace / kResolveThreads;

__device__ __forceinline__ uint64_t weight_code(float alpha, float beta, double eps) {
    const double a = static_cast<double>(alpha), b = static_cast<double>(beta);
    const double s = a + b;
    double w = eps;
    if (s > 0.0) {
        const double v = a / s;
        const double q = 1.0 - v;
        const double p = v * q;
        w = sqrt(p) + eps;
    }
    return static_cast<uint64_t>(floor(w * 4294967296.0));
}

// Inclusive scan of one value per thread over a 256-thread block.
__device__ __forceinline__ uint64_t block_scan_inclusive(uint64_t x, uint64_t *wave_tot, uint64_t &total) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const uint64_t y = __shfl_up(x, o, kWave);
        if (lane >= o) x += y;
    }
    __syncthreads();
    if (lane == kWave - 1) wave_tot[wave] = x;
    __syncthreads();
    uint64_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kScanThreads / kWave; ++w) {
        const uint64_t t = wave_tot[w];
        if (w < wave) before += t;
        all += t;
    }
    total = all;
    return x + before;
}

// Phase 1: per-block sum of the weight codes.
__global__ void __launch_bounds__(kScanThreads)
weight_block_sums_kernel(const float *__restrict__ alpha, const float *__restrict__ beta, int64_t N,
                         double eps, uint64_t *__restrict__ block_sums) {
    __shared__ uint64_t scratch[kScanThreads / kWave];
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kScanItems;
    uint64_t s = 0;
#pragma unroll 4
    for (int r = 0; r < kScanRows; ++r) {
        const int64_t i = base + r * kScanThreads + threadIdx.x;
        if (i < N) s += weight_code(alpha[i], beta[i], eps);
    }
    s = block_sum(s, scratch);
    if (threadIdx.x == 0) block_sums[blockIdx.x] = s;
}

// Phase 2: exclusive scan of the block sums (one workgroup, carried in chunks).
__global__ void __launch_bounds__(kScanThreads)
scan_block_sums_kernel(uint64_t *__restrict__ block_sums, int64_t nblocks, uint64_t *__restrict__ total_out) {
    __shared__ uint64_t wave_tot[kScanThreads / kWave];
    uint64_t carry = 0;
    for (int64_t base = 0; base < nblocks; base += kScanThreads) {
        const int64_t i = base + threadIdx.x;
        const uint64_t x = i < nblocks ? block_sums[i] : 0;
        uint64_t tot;
        const uint64_t inc = block_scan_inclusive(x, wave_tot, tot);
        if (i < nblocks) block_sums[i] = carry + inc - x;
        carry += tot;
    }
    if (threadIdx.x == 0) *total_out = carry;
}

// Phase 3: inclusive CDF of the codes.
__global__ void __launch_bounds__(kScanThreads)
weight_cdf_kernel(const float *__restrict__ alpha, const float *__restrict__ beta, int64_t N, double eps,
                  const uint64_t *__restrict__ block_offsets, uint64_t *__restrict__ cdf) {
    __shared__ uint64_t wave_tot[kScanThreads / kWave];
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kScanItems;
    uint64_t carry = block_offsets[blockIdx.x];
    for (int r = 0; r < kScanRows; ++r) {
        const int64_t i = base + r * kScanThreads + threadIdx.x;
        const uint64_t x = i < N ? weight_code(alpha[i], beta[i], eps) : 0;
        uint64_t tot;
        const uint64_t inc = block_scan_inclusive(x, wave_tot, tot);
        if (i < N) cdf[i] = carry + inc;
        carry += tot;
    }
}

// Philox4x32-10 (Salmon et al., SC'11): ten rounds, each two 32x32->64 products
// whose halves are crossed with the other counter words and the round key; the
// key grows by the two Weyl constants after every round.
__device__ __forceinline__ uint64_t philox_bits(uint64_t seed, uint64_t iteration, uint32_t slot, uint32_t attempt) {
    uint32_t c0 = slot, c1 = attempt, c2 = static_cast<uint32_t>(iteration), c3 = static_cast<uint32_t>(iteration >> 32);
    uint32_t k0 = static_cast<uint32_t>(seed), k1 = static_cast<uint32_t>(seed >> 32);
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return static_cast<uint64_t>(c0) | (static_cast<uint64_t>(c1) << 32);
}

// index of draw (slot, attempt): first i with cdf[i] > floor(bits * total / 2^64)
__device__ __forceinline__ int32_t draw_index(const uint64_t *__restrict__ cdf, int64_t N, uint64_t total,
                                              uint64_t seed, uint64_t iteration, uint32_t slot, uint32_t attempt) {
    const uint64_t t = __umul64hi(philox_bits(seed, iteration, slot, attempt), total);
    int64_t lo = 0, hi = N;
    while (lo < hi) {
        const int64_t mid = lo + ((hi - lo) >> 1);
        if (cdf[mid] > t) hi = mid; else lo = mid + 1;
    }
    return static_cast<int32_t>(lo);
}

__global__ void __launch_bounds__(256)
draw_with_replacement_kernel(const uint64_t *__restrict__ cdf, int64_t N, const uint64_t *__restrict__ total,
                             uint64_t seed, uint64_t iteration, int B, int32_t *__restrict__ idx_out,
                             int32_t *__restrict__ info) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t tot = *total;  // zero: every weight is zero, nothing can be drawn
    if (k < B) idx_out[k] = tot ? draw_index(cdf, N, tot, seed, iteration, k, 0) : -1;
    if (info && k == 0) { info[0] = tot ? 0 : 1; info[1] = 0; }
}

// Successive sampling without replacement as a fixed point: every slot starts at
// attempt 0; in each sweep a slot whose candidate is also held by a LOWER slot
// moves to its next attempt.  A candidate that makes a slot move is always held
// for good by some lower slot (follow the chain of holders downwards), so the
// fixed point is the sequential definition "first attempt not taken by an
// earlier slot".  One workgroup; the loop ends because every sweep that does not
// end it raises some attempt counter and counters are capped by max_attempts.
//
// "Held by a lower slot" is decided through owner[N] (all kNoOwner on entry and
// again on exit): every live slot files its number under its candidate with an
// atomic minimum, then reads the minimum back.  The minimum does not depend on
// the order of the atomics, so the result is the same on every run.  The owner
// entries are read and cleared with L2-coherent accesses: the atomics act at the
// L2, a plain load could be served from the CU's own cache.
constexpr int32_t kNoOwner = 0x7fffffff;

__global__ void __launch_bounds__(256) fill_owner_kernel(int32_t *__restrict__ owner, int64_t N) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < N) owner[i] = kNoOwner;
}

__global__ void __launch_bounds__(kResolveThreads)
draw_without_replacement_kernel(const uint64_t *__restrict__ cdf, int64_t N, const uint64_t *__restrict__ total_p,
                                uint64_t seed, uint64_t iteration, int B, uint32_t max_attempts,
                                int32_t *__restrict__ idx_out, int32_t *__restrict__ info,
                                int32_t *__restrict__ owner) {
    __shared__ int changed_flag[2];
    __shared__ int failed_flag;
    const uint64_t total = *total_p;
    if (total == 0) {  // every weight is zero: nothing can be drawn (uniform exit, before any barrier)
        for (int k = threadIdx.x; k < B; k += kResolveThreads) idx_out[k] = -1;
        if (info && threadIdx.x == 0) { info[0] = 1; info[1] = 0; }
        return;
    }
    uint32_t attempt[kSlotsPerThread];
    int32_t cand[kSlotsPerThread];
    bool live[kSlotsPerThread];   // slot exists and has not run out of attempts
#pragma unroll
    for (int s = 0; s < kSlotsPerThread; ++s) {
        attempt[s] = 0;
        const int k = s * kResolveThreads + threadIdx.x;
        live[s] = k < B;
        cand[s] = live[s] ? draw_index(cdf, N, total, seed, iteration, k, 0) : -1;
    }
    if (threadIdx.x == 0) { changed_flag[0] = 0; changed_flag[1] = 0; failed_flag = 0; }
    __syncthreads();
    for (int sweep = 0;; ++sweep) {
#pragma unroll
        for (int s = 0; s < kSlotsPerThread; ++s)
            if (live[s]) atomicMin(&owner[cand[s]], s * kResolveThreads + static_cast<int>(threadIdx.x));
        __threadfence();
        __syncthreads();  // every claim of this sweep is filed
        bool conflict[kSlotsPerThread];
#pragma unroll
        for (int s = 0; s < kSlotsPerThread; ++s)
            conflict[s] = live[s] && __hip_atomic_load(&owner[cand[s]], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) <
                                         s * kResolveThreads + static_cast<int>(threadIdx.x);
        __syncthreads();  // every claim has been read
#pragma unroll
        for (int s = 0; s < kSlotsPerThread; ++s)
            if (live[s]) __hip_atomic_store(&owner[cand[s]], kNoOwner, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        bool any = false;
#pragma unroll
        for (int s = 0; s < kSlotsPerThread; ++s) {
            if (conflict[s]) {
                any = true;
                if (++attempt[s] >= max_attempts) {
                    live[s] = false;
                    cand[s] = -1;
                    failed_flag = 1;
                } else {
                    cand[s] = draw_index(cdf, N, total, seed, iteration, s * kResolveThreads + threadIdx.x, attempt[s]);
                }
            }
        }
        int *flag = &changed_flag[sweep & 1];
        if (any) *flag = 1;
        __threadfence();
        __syncthreads();  // owner is clear again; the flag is complete
        const bool again = *flag != 0;
        if (threadIdx.x == 0) changed_flag[(sweep + 1) & 1] = 0;
        if (!again) break;
        __syncthreads();
    }
    uint32_t amax = 0;
#pragma unroll
    for (int s = 0; s < kSlotsPerThread; ++s) {
        const int k = s * kResolveThreads + threadIdx.x;
        if (k < B) {
            idx_out[k] = cand[s];   // -1 for a slot that ran out of attempts
            amax = attempt[s] > amax ? attempt[s] : amax;
        }
    }
    if (info) {
        __shared__ uint32_t amax_sh;
        if (threadIdx.x == 0) amax_sh = 0;
        __syncthreads();
        atomicMax(&amax_sh, amax);
        __syncthreads();
        if (threadIdx.x == 0) { info[0] = failed_flag; info[1] = static_cast<int32_t>(amax_sh); }
    }
}

struct SamplerWorkspace {
    uint64_t *cdf, *block_sums, *total;
    int32_t *owner;
    size_t bytes;
};

static SamplerWorkspace sampler_layout(void *ws, int64_t N) {
    Arena a(ws);
    SamplerWorkspace w;
    w.cdf = a.take<uint64_t>(static_cast<size_t>(N));
    w.block_sums = a.take<uint64_t>(static_cast<size_t>(ceil_div(N, kScanItems)));
    w.total = a.take<uint64_t>(1);
    w.owner = a.take<int32_t>(static_cast<size_t>(N));
    w.bytes = a.used;
    return w;
}

}  // namespace spo

using namespace spo;

extern "C" size_t spo_sample_prompts_workspace_bytes(int64_t N, int32_t B) {
    (void)B;
    if (N < 1) return 0;
    return sampler_layout(nullptr, N).bytes;
}

// Checks and launches shared by the two entry points; ws holds sampler_layout(ws, N).
static int sample_launch(const float *alpha, const float *beta, int64_t N, int32_t B, double eps_explore,
                         uint64_t seed, uint64_t iteration, int replace, uint32_t max_attempts,
                         int32_t *idx_out, int32_t *info, void *ws, hipStream_t s) {
    const SamplerWorkspace w = sampler_layout(ws, N);
    if (max_attempts == 0) max_attempts = 1u << 16;  // a sweep per attempt level: bounds a hopeless draw to ~0.1 s
    const int64_t nblocks = ceil_div(N, kScanItems);
    weight_block_sums_kernel<<<static_cast<unsigned>(nblocks), kScanThreads, 0, s>>>(alpha, beta, N, eps_explore, w.block_sums);
    scan_block_sums_kernel<<<1, kScanThreads, 0, s>>>(w.block_sums, nblocks, w.total);
    weight_cdf_kernel<<<static_cast<unsigned>(nblocks), kScanThreads, 0, s>>>(alpha, beta, N, eps_explore, w.block_sums, w.cdf);
    if (replace) {
        draw_with_replacement_kernel<<<(B + 255) / 256, 256, 0, s>>>(w.cdf, N, w.total, seed, iteration, B, idx_out, info);
    } else {
        fill_owner_kernel<<<static_cast<unsigned>(ceil_div(N, 256)), 256, 0, s>>>(w.owner, N);
        draw_without_replacement_kernel<<<1, kResolveThreads, 0, s>>>(w.cdf, N, w.total, seed, iteration, B, max_attempts,
                                                                     idx_out, info, w.owner);
    }
    return launch_status();
}

static int sample_check(const float *alpha, const float *beta, int64_t N, int32_t B, double eps_explore,
                        int replace, const int32_t *idx_out) {
    if (!alpha || !beta || !idx_out) return SPO_ENULL;
    if (N < 1 || N >= (int64_t(1) << 31) || B < 1 || !(eps_explore >= 0.0) || !(eps_explore <= 1.0))
        return SPO_EINVAL;
    if (!replace && B > N) return SPO_EINVAL;
    if (!replace && B > kMaxSlotsNoReplace) return SPO_ERANGE;
    return SPO_OK;
}

extern "C" int spo_sample_prompts(const float *alpha, const float *beta, int64_t N, int32_t B,
                                  double eps_explore, uint64_t seed, uint64_t iteration, int replace,
                                  uint32_t max_attempts, int32_t *idx_out, int32_t *info, void *ws,
                                  size_t ws_bytes, spo_stream_t stream) {
    const int rc = sample_check(alpha, beta, N, B, eps_explore, replace, idx_out);
    if (rc) return rc;
    if (!ws) return SPO_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return SPO_EINVAL;
    if (ws_bytes < sampler_layout(nullptr, N).bytes) return SPO_EWORKSPACE;
    return sample_launch(alpha, beta, N, B, eps_explore, seed, iteration, replace, max_attempts, idx_out, info, ws,
                         as_stream(stream));
}

// ----------------------------------------------------------------------------
// The same draw for callers that cannot allocate: the CDF, the block sums and the
// owner table live in a fixed array in device memory that belongs to the library
// (one copy per GPU, held until the process ends).
// ----------------------------------------------------------------------------
namespace spo {

constexpr int64_t kStaticMaxN = SPO_SAMPLE_STATIC_MAX_N;
// what sampler_layout takes for kStaticMaxN prompts: 8 B (CDF) + 4 B (owner) per prompt,
// one 8-byte sum per 4096 prompts, the total, each block rounded up to 256 bytes
constexpr size_t kStaticBytes = static_cast<size_t>(kStaticMaxN) * 12 + (kStaticMaxN / kScanItems + 1) * 8 + 4 * 256;
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

// Device address of `scratch` on the current device.  In host code the array's name is only a
// handle for hipGetSymbolAddress; every GPU has its own copy at its own address, looked up
// once per device with that device current.
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void *g_scratch_ptr[kMaxDevices];

static int static_scratch(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SPO_EHIP;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SPO_EHIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return SPO_OK;
}

}  // namespace spo

extern "C" int spo_sample_prompts_static(const float *alpha, const float *beta, int64_t N, int32_t B,
                                         double eps_explore, uint64_t seed, uint64_t iteration, int replace,
                                         uint32_t max_attempts, int32_t *idx_out, int32_t *info,
                                         spo_stream_t stream) {
    int rc = sample_check(alpha, beta, N, B, eps_explore, replace, idx_out);
    if (rc) return rc;
    if (N > kStaticMaxN) return SPO_ERANGE;  // the fixed array holds the tables of at most this many prompts
    if (sampler_layout(nullptr, N).bytes > kStaticBytes) return SPO_ERANGE;
    void *ws = nullptr;
    if ((rc = static_scratch(&ws))) return rc;
    return sample_launch(alpha, beta, N, B, eps_explore, seed, iteration, replace, max_attempts, idx_out, info, ws,
                         as_stream(stream));
}
