// bf16 MFMA contraction core for gfx950 (CDNA4, 64-wide wavefronts).
//
// Computes a BM x BN tile of  D[m][n] = sum_k A[m][k] * B[n][k]  where both
// operands are row-major with the contraction index contiguous.  All three
// contractions of the loss (logits = W h, dHidden = dZ W, dW = dZ^T X) are
// brought to this form by the callers, so there is one main loop to tune.
//
// Data path per stage of 64 contraction elements (128 bytes = one cache line per
// operand row; half-line rows were measured to halve the L2->LDS rate):
//   HBM/L2 --global_load_lds_dwordx4--> LDS (two stages)  --ds_read_b128-->
//   VGPR fragments --v_mfma_f32_32x32x16_bf16--> fp32 accumulators.
// Global loads go straight to LDS without passing through registers.  A tile
// row is 8 chunks of 16 bytes; chunk c of row r is stored at chunk position
// c ^ swz(r), which makes both the 64 lanes x 16 B fragment reads and the
// linear DMA writes free of bank conflicts.  The swizzle is applied on the
// global side (each lane fetches the chunk that belongs at its LDS slot),
// because the DMA writes lane i at base + 16*i.
//
// Accumulator layout of one 32x32 block (v_mfma_f32_32x32x16_bf16): lane l
// holds column n = l % 32 and, in register r, row m = 8*(r/4) + 4*(l/32) + r%4.
// Callers put the index they reduce over or scale by per row of the tile
// (vocabulary entries) on m and the index with per-lane constants (tokens) on n.
#pragma once

#include "common.hpp"

namespace spo {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kBK = 64;      // contraction elements per stage
constexpr int kStages = 2;   // LDS stages
constexpr int kRowBytes = kBK * 2;
constexpr int kChunks = kRowBytes / 16;

// chunk swizzle of a tile row (3 bits): a bijection on 0..7 both over rows 0..7
// and over the rows of equal parity in 0..15, i.e. 16 consecutive rows reading
// the same chunk touch 16 different 16-byte slots of any 256-byte window, and 8
// consecutive rows 8 different slots of any 128-byte window
__device__ __forceinline__ int swz(int row) {
    return ((row >> 1) & 3) | (((row ^ (row >> 3)) & 1) << 2);
}

template <int BM_, int BN_, int WGM_, int WGN_>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, WGM = WGM_, WGN = WGN_;
    static constexpr int NWAVE = WGM * WGN, NT = NWAVE * kWave;
    static constexpr int WM = BM / WGM, WN = BN / WGN;     // wave tile
    static constexpr int FM = WM / 32, FN = WN / 32;       // 32x32 blocks per wave
    static constexpr int KK = kBK / 16;                    // MFMA k-slices per stage
    static constexpr int A_BYTES = BM * kRowBytes, B_BYTES = BN * kRowBytes;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = kStages * STAGE_BYTES;
    static constexpr int A_LOADS = BM * kChunks / NT, B_LOADS = BN * kChunks / NT;
    static constexpr int STAGE_LOADS = A_LOADS + B_LOADS;  // DMA instructions per thread and stage
    static_assert(BM * kChunks % NT == 0 && BN * kChunks % NT == 0, "tile rows must split evenly over the threads");
    static_assert((NT / kChunks) % 16 == 0, "swizzle must be the same for every load of a thread");
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile is made of 32x32 blocks");

    typedef f32x16_t Acc[FM][FN];

    __device__ static __forceinline__ int wave_id() {
        return __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x) / kWave);
    }
    __device__ static __forceinline__ int wave_m0() { return (wave_id() % WGM) * WM; }
    __device__ static __forceinline__ int wave_n0() { return (wave_id() / WGM) * WN; }
    // tile row of accumulator register r of block fm (add the block's tile origin)
    __device__ static __forceinline__ int acc_row(int fm, int r) {
        return wave_m0() + fm * 32 + 8 * (r >> 2) + 4 * ((threadIdx.x & 63) >> 5) + (r & 3);
    }
    // tile column of block fn
    __device__ static __forceinline__ int acc_col(int fn) {
        return wave_n0() + fn * 32 + (threadIdx.x & 31);
    }

    // Global -> LDS transfers of one tile: addressing and issue.
    // Slot q = i*NT + tid of a tile <-> (row q/kChunks, position q%kChunks).
    struct Dma {
        const char *a_tile, *b_tile;     // first row of the A / B panel (wave-uniform)
        uint32_t oa[A_LOADS], ob[B_LOADS];  // this lane's byte offsets inside the panels
        uint32_t lds_wave;               // LDS address of this wave's 1 KiB slice of stage 0

        __device__ __forceinline__ Dma(const char *A, int64_t lda_bytes, int64_t m0, int64_t M, const char *B,
                                       int64_t ldb_bytes, int64_t n0, int64_t N, char *lds) {
            const int tid = threadIdx.x;
            const int ld_row = tid / kChunks;
            const int ld_chunk = (tid % kChunks) ^ swz(ld_row & 15);
            // the tile origins are the same for every lane; say so, the DMA wants them in SGPRs
            auto uniform = [](const char *p) {
                const uint64_t u = reinterpret_cast<uint64_t>(p);
                const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(u));
                const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(u >> 32));
                return reinterpret_cast<const char *>((static_cast<uint64_t>(hi) << 32) | lo);
            };
            a_tile = uniform(A + m0 * lda_bytes);
            b_tile = uniform(B + n0 * ldb_bytes);
            // 32-bit byte offsets from the tile's first row (a tile spans < 4 GiB)
#pragma unroll
            for (int i = 0; i < A_LOADS; ++i) {
                int64_t r = i * (NT / kChunks) + ld_row;
                r = m0 + r < M ? r : M - 1 - m0;
                oa[i] = static_cast<uint32_t>(r * lda_bytes + ld_chunk * 16);
            }
#pragma unroll
            for (int i = 0; i < B_LOADS; ++i) {
                int64_t r = i * (NT / kChunks) + ld_row;
                r = n0 + r < N ? r : N - 1 - n0;
                ob[i] = static_cast<uint32_t>(r * ldb_bytes + ld_chunk * 16);
            }
            lds_wave = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) char *)lds)) +
                       wave_id() * (kWave * 16);
        }
        // The DMA is issued from inline assembly.  Issued through the compiler it would
        // make every later LDS read wait for ALL outstanding DMA (the wait-count pass
        // cannot tell the stages apart); here every vmcnt wait for these loads is
        // explicit instead.  M0 holds the LDS base of the 64 lanes x 16 bytes written.
        __device__ static __forceinline__ void dma(const char *base, uint32_t off, uint32_t lds_addr) {
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :
                         : "s"(lds_addr), "v"(off), "s"(base)
                         : "memory");
        }
        // DMA instruction i (0 .. STAGE_LOADS-1) of this thread's share of stage kt
        __device__ __forceinline__ void one(int kt, int i) const {
            const uint32_t la = lds_wave + (kt % kStages) * STAGE_BYTES;
            const int64_t koff = static_cast<int64_t>(kt) * kRowBytes;
            if (i < A_LOADS) dma(a_tile + koff, oa[i], la + i * (NT * 16));
            else dma(b_tile + koff, ob[i - A_LOADS], la + A_BYTES + (i - A_LOADS) * (NT * 16));
        }
        __device__ __forceinline__ void stage(int kt) const {
#pragma unroll
            for (int i = 0; i < STAGE_LOADS; ++i) one(kt, i);
        }
    };

    // Starts the transfer of stage 0 of a tile while the caller still works on the
    // previous tile's accumulators (its epilogue); the matching mainloop call passes
    // stage0_issued = true.  All threads of the block must call this together.
    __device__ static __forceinline__ void prefetch(const char *__restrict__ A, int64_t lda_bytes, int64_t m0, int64_t M,
                                                    const char *__restrict__ B, int64_t ldb_bytes, int64_t n0, int64_t N,
                                                    char *lds) {
        const Dma d(A, lda_bytes, m0, M, B, ldb_bytes, n0, N, lds);
        __syncthreads();  // every wave is done with the previous contents of lds
        d.stage(0);
    }

    // acc += A[m0.., :K] * B[n0.., :K]^T.  Rows beyond M / N are read from the last
    // valid row (the caller masks them).  K = kBK * KT.  lds: LDS_BYTES bytes,
    // 16-byte aligned.  All threads of the block must call this together.
    __device__ static __forceinline__ void mainloop(const char *__restrict__ A, int64_t lda_bytes, int64_t m0, int64_t M,
                                                    const char *__restrict__ B, int64_t ldb_bytes, int64_t n0, int64_t N,
                                                    int KT, char *lds, Acc &acc, bool stage0_issued = false) {
        const int lane = threadIdx.x & 63, wave = wave_id();
        const Dma d(A, lda_bytes, m0, M, B, ldb_bytes, n0, N, lds);
        auto wait_dma = [] { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };
        // ---- fragment addressing: lane reads row (l%32) of a 32-row block, chunk 2*kk + l/32
        const int fr_sw = swz(lane & 15);
        int fr_off[KK];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) fr_off[kk] = (lane & 31) * kRowBytes + (((2 * kk + (lane >> 5)) ^ fr_sw) * 16);
        const int a_base = wave_m0() * kRowBytes, b_base = A_BYTES + wave_n0() * kRowBytes;

        // Two groups of four wavefronts (one of each per SIMD) run half a step apart:
        // while one group multiplies, the other reads its fragments from LDS, so the
        // MFMA pipe of every SIMD always has a wavefront to serve.  Barrier j of one
        // group meets barrier j of the other; group 1 passes one extra barrier first
        // and group 0 one extra at the end.  With I(j) the interval after barrier j,
        // group 0 reads stage s in I(2s) and multiplies in I(2s+1); group 1 reads in
        // I(2s+1) and multiplies in I(2s+2).  The buffer of stage s+1 is free from
        // barrier 2s on and must be complete at barrier 2s+2, so its DMA is issued in
        // I(2s) and awaited at the end of I(2s+1).  The address unit takes about 16
        // cycles per DMA instruction and a burst of them blocks the issuing
        // wavefront: group 1, which multiplies during I(2s), feeds its share one
        // instruction per two MFMAs, and group 0 issues its share behind its
        // fragment reads.
        static_assert(NWAVE == 8, "the main loop is written for two groups of four wavefronts");
        static_assert(kStages == 2, "the schedule below is for two stages");
        const int group = wave >> 2;
        auto fence_barrier = [] {
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
        };
        if (!stage0_issued) {
            __syncthreads();  // every wave is done with the previous contents of lds
            d.stage(0);
        }
        wait_dma();
        fence_barrier();
        if (group == 1) {
            if (KT > 1) d.stage(1);
            fence_barrier();
        }
        for (int kt = 0; kt < KT; ++kt) {
            const char *st = lds + (kt % kStages) * STAGE_BYTES;
            bf16x8_t af[FM][KK], bf[FN][KK];
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
#pragma unroll
                for (int fm = 0; fm < FM; ++fm)
                    af[fm][kk] = *reinterpret_cast<const bf16x8_t *>(st + a_base + fm * (32 * kRowBytes) + fr_off[kk]);
#pragma unroll
                for (int fn = 0; fn < FN; ++fn)
                    bf[fn][kk] = *reinterpret_cast<const bf16x8_t *>(st + b_base + fn * (32 * kRowBytes) + fr_off[kk]);
            }
            if (group == 0) {
                if (kt + 1 < KT) d.stage(kt + 1);
            } else {
                wait_dma();  // my share of stage kt+1, issued during the previous multiply phase
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // fragments are in registers
            fence_barrier();
            __builtin_amdgcn_s_setprio(1);
            const bool feed = group == 1 && kt + 2 < KT;  // wave-uniform
#pragma unroll
            for (int j = 0; j < KK * FM * FN; ++j) {
                const int kk = j / (FM * FN), fm = (j / FN) % FM, fn = j % FN;
                if (j % 2 == 0 && j / 2 < STAGE_LOADS) {
                    if (feed) d.one(kt + 2, j / 2);
                    __builtin_amdgcn_sched_barrier(0);
                }
                acc[fm][fn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[fm][kk], bf[fn][kk], acc[fm][fn], 0, 0, 0);
            }
            __builtin_amdgcn_s_setprio(0);
            if (group == 0) wait_dma();  // my share of stage kt+1
            fence_barrier();
        }
        if (group == 0) fence_barrier();
    }

    __device__ static __forceinline__ void zero(Acc &acc) {
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
#pragma unroll
            for (int fn = 0; fn < FN; ++fn)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[fm][fn][r] = 0.0f;
    }
};

// Maps a linear workgroup id to a tile of an nM x nN tile grid so that the 32
// workgroups that run together on one XCD (ids equal mod 8 are dispatched to the
// same XCD and share its L2) form a 4 x 8 patch: 12 operand panels feed 32 tiles.
// Patches are walked along M first.  Returns false for ids beyond the grid.
struct TileOrder {
    int64_t nM, nN, pM, pN;  // tiles and patches per dimension
    __host__ __device__ TileOrder(int64_t nm, int64_t nn) : nM(nm), nN(nn), pM((nm + 3) / 4), pN((nn + 7) / 8) {}
    __host__ __device__ int64_t blocks() const { return (pM * pN + 7) / 8 * 8 * 32; }
    __device__ bool tile(int64_t bid, int64_t &tm, int64_t &tn) const {
        const int64_t xcd = bid & 7, q = bid >> 3;
        const int64_t patch = (q >> 5) * 8 + xcd, w = q & 31;
        if (patch >= pM * pN) return false;
        tm = (patch % pM) * 4 + (w >> 3);
        tn = (patch / pM) * 8 + (w & 7);
        return tm < nM && tn < nN;
    }
};

}  // namespace spo
