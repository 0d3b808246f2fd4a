// Shared host/device helpers of the SPO HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spo.h"

namespace spo {

static inline hipStream_t as_stream(spo_stream_t s) { return reinterpret_cast<hipStream_t>(s); }

// Status of the launch that was just enqueued.
static inline int launch_status() {
    return hipGetLastError() == hipSuccess ? SPO_OK : SPO_EHIP;
}

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
__host__ __device__ static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Bump allocator over the caller's workspace; every block 256-byte aligned.  With a NULL
// base it only adds up sizes (the workspace queries) and hands out NULL.
struct Arena {
    char *base;
    size_t used;
    explicit Arena(void *p) : base(static_cast<char *>(p)), used(0) {}
    template <typename T>
    T *take(size_t count) {
        T *p = base ? reinterpret_cast<T *>(base + used) : nullptr;
        used += align_up(count * sizeof(T), 256);
        return p;
    }
};

typedef uint16_t bf16_t;  // raw bfloat16 bits

#if defined(__HIPCC__)

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_to_f32(bf16_t b) {
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<bf16_t>((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<bf16_t>(u >> 16);
}

// two floats -> packed bf16 pair, round-to-nearest-even in hardware (v_cvt_pk_bf16_f32)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2_rn(float lo, float hi) {
    const f32x2_t f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return static_cast<uint32_t>(f32_to_bf16(lo)) | (static_cast<uint32_t>(f32_to_bf16(hi)) << 16);
}

// Sum over the 64 lanes of a wavefront; every lane receives the total.
template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// Sum over a thread block in a fixed order (bitwise reproducible).  scratch holds
// one T per wavefront.  Every thread receives the total.
template <typename T>
__device__ __forceinline__ T block_sum(T v, T *scratch) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int nwave = (blockDim.x + kWave - 1) / kWave;
    v = wave_sum(v);
    __syncthreads();  // scratch may still be read by a previous reduction
    if (lane == 0) scratch[wave] = v;
    __syncthreads();
    T total = T(0);
    for (int w = 0; w < nwave; ++w) total += scratch[w];
    return total;
}

// Response that holds token t: largest b with cu[b]-cu[0] <= t (cu has B+1 entries).
__device__ __forceinline__ int response_of_token(const int32_t *cu, int B, int64_t t) {
    const int64_t base = cu[0];
    int lo = 0, hi = B;  // invariant: cu[lo]-base <= t, answer in [lo, hi)
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (static_cast<int64_t>(cu[mid]) - base <= t) lo = mid; else hi = mid;
    }
    return lo;
}

#endif  // __HIPCC__

}  // namespace spo
