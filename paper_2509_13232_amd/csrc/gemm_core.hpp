// bf16 MFMA contraction core for gfx950 (CDNA4, 64-wide wavefronts).
//
// Computes a BM x BN tile of  D[m][n] = sum_k A[m][k] * B[n][k]  where both
// operands are row-major with the contraction index contiguous (mainloop: logits =
// W h and dHidden = dZ W), or of  D[m][n] = sum_k A[k][m] * B[k][n]  where the
// contraction index is the row index of both (mainloop_kmajor: dW = dZ^T X, which
// contracts over tokens: the rows of the hidden states and of the blocks of dZ).  The two
// loops share the tile shape, the schedule and the accumulator layout.
//
// Data path per stage of 64 contraction elements (128 bytes = one cache line per
// operand row; half-line rows were measured to halve the L2->LDS rate):
//   HBM/L2 --global_load_lds_dwordx4--> LDS (two stages)  --ds_read_b128-->
//   VGPR fragments --v_mfma_f32_16x16x32_bf16--> fp32 accumulators.
// Global loads go straight to LDS without passing through registers.  A tile
// row is 8 chunks of 16 bytes; chunk c of row r is stored at chunk position
// c ^ swz(r), which makes both the 64 lanes x 16 B fragment reads and the
// linear DMA writes free of bank conflicts.  The swizzle is applied on the
// global side (each lane fetches the chunk that belongs at its LDS slot),
// because the DMA writes lane i at base + 16*i.
//
// Accumulator layout of one 16x16 block (v_mfma_f32_16x16x32_bf16): lane l
// holds column n = l % 16 and, in register r, row m = 4*(l/16) + r.
// Callers put the index they reduce over or scale by per row of the tile
// (vocabulary entries) on m and the index with per-lane constants (tokens) on n.
#pragma once

#include <type_traits>

#include "common.hpp"

namespace spo {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kBK = 64;      // contraction elements per stage
constexpr int kStages = 2;   // LDS stages
constexpr int kRowBytes = kBK * 2;
constexpr int kChunks = kRowBytes / 16;
constexpr int kBlockK = kBK;  // contraction elements per block of a k-blocked operand: one stage

// chunk swizzle of a tile row (3 bits): a bijection on 0..7 both over rows 0..7
// and over the rows of equal parity in 0..15, i.e. 16 consecutive rows reading
// the same chunk touch 16 different 16-byte slots of any 256-byte window, and 8
// consecutive rows 8 different slots of any 128-byte window
__device__ __forceinline__ int swz(int row) {
    return ((row >> 1) & 3) | (((row ^ (row >> 3)) & 1) << 2);
}

// MI is the edge of the MFMA block: 16 for v_mfma_f32_16x16x32_bf16, the instruction the
// main loop is written for.  (The same tile on v_mfma_f32_32x32x16_bf16, with two
// phase-shifted groups of wavefronts, was 4-6 % slower on the same chip.)
template <int BM_, int BN_, int WGM_, int WGN_, int MI_ = 16>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, WGM = WGM_, WGN = WGN_, MI = MI_;
    static_assert(MI == 16, "the main loop issues 16x16x32 MFMAs");
    static constexpr int NWAVE = WGM * WGN, NT = NWAVE * kWave;
    static constexpr int WM = BM / WGM, WN = BN / WGN;     // wave tile
    static constexpr int FM = WM / MI, FN = WN / MI;       // MI x MI blocks per wave
    static constexpr int KK = kBK / (512 / MI);            // MFMA k-slices per stage (16 or 32 elements deep)
    static constexpr int ACC_R = MI * MI / kWave;          // accumulator registers per block and lane
    static constexpr int A_BYTES = BM * kRowBytes, B_BYTES = BN * kRowBytes;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = kStages * STAGE_BYTES;
    static constexpr int A_LOADS = BM * kChunks / NT, B_LOADS = BN * kChunks / NT;
    static constexpr int STAGE_LOADS = A_LOADS + B_LOADS;  // DMA instructions per thread and stage
    static_assert(BM * kChunks % NT == 0 && BN * kChunks % NT == 0, "tile rows must split evenly over the threads");
    static_assert((NT / kChunks) % 16 == 0, "swizzle must be the same for every load of a thread");
    static_assert(WM % MI == 0 && WN % MI == 0, "wave tile is made of MI x MI blocks");

    typedef float AccBlock __attribute__((ext_vector_type(ACC_R)));
    typedef AccBlock Acc[FM][FN];

    __device__ static __forceinline__ int wave_id() {
        return __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x) / kWave);
    }
    __device__ static __forceinline__ int wave_m0() { return (wave_id() % WGM) * WM; }
    __device__ static __forceinline__ int wave_n0() { return (wave_id() / WGM) * WN; }
    // Accumulator layout of a 16x16 block: lane l holds column l % 16 and, in register r, row
    // 4*(l/16) + r: a lane owns a run of four consecutive rows, a quad of lanes four consecutive
    // columns, and the four groups of 16 lanes hold different rows of the same columns.
    // tile row of accumulator register r of block fm
    __device__ static __forceinline__ int acc_row(int fm, int r) {
        return wave_m0() + fm * MI + 4 * ((threadIdx.x & 63) / MI) + r;
    }
    // tile column of block fn
    __device__ static __forceinline__ int acc_col(int fn) {
        return wave_n0() + fn * MI + (threadIdx.x & (MI - 1));
    }
    static constexpr int GROUPS = kWave / MI;  // lane groups that hold different rows of the same column
    static constexpr int RUNS = ACC_R / 4;     // runs of four consecutive rows per block and lane
    __device__ static __forceinline__ int lane_group() { return (threadIdx.x & 63) / MI; }
    // Row d of the wavefront's part of the tile (0 <= d < WM) lives in block fm, register r of
    // the lanes of group g.
    __device__ static __forceinline__ void locate(int d, int &fm, int &r, int &g) {
        fm = d / MI;
        g = (d >> 2) & (GROUPS - 1);
        r = d & 3;
    }

    // The two operand panels of one tile: A[m0.., :K] and B[n0.., :K], rows of ld bytes, M / N
    // valid rows in all (rows of the tile beyond them are fetched from the last valid row; the
    // caller masks them).  An operand may be stored in blocks of kBlockK contraction elements:
    // element k of row m at base + (k / kBlockK) * blk + m * ld + (k % kBlockK) * 2 bytes
    // (blk = 0: plain row-major).  With ld = 128 bytes a stage of a tile is then one contiguous
    // 32 KiB piece instead of 256 lines a whole matrix row apart: the 256 rows stay within a few
    // pages of the address translation and spread evenly over the memory channels.
    struct Operands {
        const char *A;
        int64_t lda_bytes, m0, M;
        const char *B;
        int64_t ldb_bytes, n0, N;
        int64_t a_blk, b_blk;
    };

    // Global -> LDS transfers of one tile: addressing and issue.
    // Slot q = i*NT + tid of a tile <-> (row q/kChunks, position q%kChunks).
    struct Dma {
        const char *a_tile, *b_tile;     // first row of the A / B panel (wave-uniform)
        int64_t a_blk, b_blk;            // bytes from one block of kBlockK contraction elements to the next
        uint32_t oa[A_LOADS], ob[B_LOADS];  // this lane's byte offsets inside the panels
        uint32_t lds_wave;               // LDS address of this wave's 1 KiB slice of buffer 0

        // the tile origins are the same for every lane; say so, the DMA wants them in SGPRs
        __device__ static __forceinline__ const char *uniform(const char *p) {
            const uint64_t u = reinterpret_cast<uint64_t>(p);
            const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(u));
            const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(u >> 32));
            return reinterpret_cast<const char *>((static_cast<uint64_t>(hi) << 32) | lo);
        }
        __device__ static __forceinline__ uint32_t lds_address(const char *p) {
            return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) const char *)p));
        }

        __device__ __forceinline__ Dma(const Operands &t, char *lds)
            : a_blk(t.a_blk ? t.a_blk : kBlockK * 2), b_blk(t.b_blk ? t.b_blk : kBlockK * 2) {
            // The thread index goes through an empty asm so that the compiler cannot trace what is
            // derived from it: hoisted out of a loop over tiles these few cheap values would sit
            // in registers across the main loop, where every register counts.
            int tid = threadIdx.x;
            asm volatile("" : "+v"(tid));
            const int ld_row = tid / kChunks;
            const uint32_t ld_chunk16 = static_cast<uint32_t>(((tid % kChunks) ^ swz(ld_row & 15)) * 16);
            a_tile = uniform(t.A + t.m0 * t.lda_bytes);
            b_tile = uniform(t.B + t.n0 * t.ldb_bytes);
            // 32-bit byte offsets from the tile's first row (a tile spans < 4 GiB); rows past the
            // operand's last row are fetched from that last row
            const uint32_t a_last = static_cast<uint32_t>(t.M - t.m0 >= BM ? BM - 1 : t.M - 1 - t.m0);
            const uint32_t b_last = static_cast<uint32_t>(t.N - t.n0 >= BN ? BN - 1 : t.N - 1 - t.n0);
            const uint32_t lda = static_cast<uint32_t>(t.lda_bytes), ldb = static_cast<uint32_t>(t.ldb_bytes);
#pragma unroll
            for (int i = 0; i < A_LOADS; ++i) {
                const uint32_t r = static_cast<uint32_t>(i * (NT / kChunks) + ld_row);
                oa[i] = (r < a_last ? r : a_last) * lda + ld_chunk16;
            }
#pragma unroll
            for (int i = 0; i < B_LOADS; ++i) {
                const uint32_t r = static_cast<uint32_t>(i * (NT / kChunks) + ld_row);
                ob[i] = (r < b_last ? r : b_last) * ldb + ld_chunk16;
            }
            lds_wave = lds_address(lds) + wave_id() * (kWave * 16);
        }
        // The DMA is issued from inline assembly.  Issued through the compiler it would
        // make every later LDS read wait for ALL outstanding DMA (the wait-count pass
        // cannot tell the stages apart); here every vmcnt wait for these loads is
        // explicit instead.  M0 holds the LDS base of the 64 lanes x 16 bytes written.  (M0 cannot
        // be named as a clobber: the compiler reserves the register and keeps no value of its
        // own in it across an asm statement; these kernels use nothing else that goes through M0.)
        __device__ static __forceinline__ void dma(const char *base, uint32_t off, uint32_t lds_addr) {
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :
                         : "s"(lds_addr), "v"(off), "s"(base)
                         : "memory");
        }
        // DMA instruction i (0 .. STAGE_LOADS-1) of this thread's share of stage kt, into LDS buffer buf
        __device__ __forceinline__ void one(int kt, int buf, int i) const {
            const uint32_t la = lds_wave + buf * STAGE_BYTES;
            static_assert(kBlockK == kBK, "one block per stage");
            if (i < A_LOADS) dma(a_tile + kt * a_blk, oa[i], la + i * (NT * 16));
            else dma(b_tile + kt * b_blk, ob[i - A_LOADS], la + A_BYTES + (i - A_LOADS) * (NT * 16));
        }
        __device__ __forceinline__ void stage(int kt, int buf) const {
#pragma unroll
            for (int i = 0; i < STAGE_LOADS; ++i) one(kt, buf, i);
        }
    };

    __device__ static __forceinline__ void fence_barrier() {
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    }

    // acc += A[m0.., :K] * B[n0.., :K]^T for ONE tile, K = kBK * KT.  lds: LDS_BYTES bytes,
    // 16-byte aligned.  All threads of the block must call this together.
    //
    // Schedule of a step: both wavefronts of a SIMD multiply at the same time and each hides its
    // own fragment reads between its MFMAs (one read per two MFMAs, into a second register set
    // for the next k-slice of 32); whenever one of them waits, at the barrier or for its
    // operands, the other keeps the MFMA pipe fed.  One barrier per step, between the two
    // k-slices: before it a wavefront has all its reads of stage s in registers and its share of
    // stage s+1 landed; after it stage s+1 may be read and the buffer of stage s is refilled with
    // stage s+2 (one DMA instruction per four MFMAs).
    __device__ static __forceinline__ void mainloop(const Operands &t, int KT, char *lds, Acc &acc) {
        static_assert(KK == 2 && kStages == 2, "two k-slices per stage, two stages");
        static_assert((FM + FN) * 2 <= FM * FN && STAGE_LOADS * 4 <= FM * FN, "reads and DMA fit between the MFMAs of a slice");
        const int lane = threadIdx.x & 63;
        const Dma d(t, lds);
        // lane reads row (l%16) of a 16-row block, chunk 4*kk + l/16
        const int fr_sw = swz(lane & 15);
        int fr_off[KK];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) fr_off[kk] = (lane & 15) * kRowBytes + (((4 * kk + (lane >> 4)) ^ fr_sw) * 16);
        const int a_base = wave_m0() * kRowBytes, b_base = A_BYTES + wave_n0() * kRowBytes;
        bf16x8_t af[2][FM], bf[2][FN];
        // fragment r (0..FM+FN-1) of k-slice kk of stage kt into register set buf
        auto read_frag = [&](int kt, int kk, int buf, int r) {
            const char *st = lds + (kt % kStages) * STAGE_BYTES;
            if (r < FM) af[buf][r] = *reinterpret_cast<const bf16x8_t *>(st + a_base + r * (16 * kRowBytes) + fr_off[kk]);
            else bf[buf][r - FM] = *reinterpret_cast<const bf16x8_t *>(st + b_base + (r - FM) * (16 * kRowBytes) + fr_off[kk]);
        };
        __syncthreads();  // every wave is done with the previous contents of lds
        d.stage(0, 0);
        if (KT > 1) {
            d.stage(1, 1);
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(STAGE_LOADS) : "memory");  // loads return in order: stage 0 has landed
        } else {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        fence_barrier();
#pragma unroll
        for (int r = 0; r < FM + FN; ++r) read_frag(0, 0, 0, r);
        // One step; MORE: a stage kt+1 exists, FEED: a stage kt+2 exists.  Compile-time flags: a
        // branch around every read and every DMA instruction costs the wavefront more issue time
        // than the instruction it guards, so the last two steps are peeled off the loop instead.
        auto step = [&](int kt, auto more_t, auto feed_t) {
            constexpr bool MORE = decltype(more_t)::value, FEED = decltype(feed_t)::value;
            // ---- slice 0 of stage kt, reading its slice 1 between the MFMAs
#pragma unroll
            for (int j = 0; j < FM * FN; ++j) {
                const int fm = j / FN, fn = j % FN;
                if (j % 2 == 0 && j / 2 < FM + FN) {
                    read_frag(kt, 1, 1, j / 2);
                    __builtin_amdgcn_sched_barrier(0);
                }
                acc[fm][fn] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[0][fm], bf[0][fn], acc[fm][fn], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
            fence_barrier();
            // ---- slice 1, reading slice 0 of stage kt+1 and feeding the DMA of stage kt+2
#pragma unroll
            for (int j = 0; j < FM * FN; ++j) {
                const int fm = j / FN, fn = j % FN;
                if (j % 2 == 0 && j / 2 < FM + FN) {
                    if (MORE) read_frag(kt + 1, 0, 0, j / 2);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (j % 4 == 1 && j / 4 < STAGE_LOADS) {
                    if (FEED) d.one(kt + 2, kt % kStages, j / 4);
                    __builtin_amdgcn_sched_barrier(0);
                }
                acc[fm][fn] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[1][fm], bf[1][fn], acc[fm][fn], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        int kt = 0;
        for (; kt + 2 < KT; ++kt) step(kt, std::true_type{}, std::true_type{});
        if (kt + 1 < KT) step(kt++, std::true_type{}, std::false_type{});
        step(kt, std::false_type{}, std::false_type{});
    }

    // ---- operands with the contraction index as the ROW index: A[k][m], B[k][n] ----
    // LDS stage of an operand: kBK rows of BM (BN) elements = 512 bytes = 32 chunks of 16 bytes,
    // chunk c of row r at position c ^ ksw(r).  ksw moves bits 1-2 of the position with the row
    // inside a group of four and bits 3-4 with the group of eight rows, so the 8-byte pieces a
    // transposing read collects (4 rows x 32 bytes per group of 16 lanes, the four groups 8 rows
    // apart) fall on distinct banks, and so do the linear DMA writes.
    __device__ static __forceinline__ int ksw(int r) { return ((r & 3) << 1) | (((r >> 3) & 3) << 3); }
    static constexpr int K_ROWB = BM * 2;                  // bytes per row of a stage
    static constexpr int K_CH = K_ROWB / 16;               // chunks per row
    static constexpr int K_LOADS = kBK * K_CH / NT;        // DMA instructions per thread, operand and stage
    static_assert(BM == BN && K_CH == 32 && kBK * K_CH % NT == 0 && 2 * K_LOADS == STAGE_LOADS,
                  "row-index-contracted stages have the size and DMA count of the others");

    // Global -> LDS transfers for mainloop_kmajor.  Slot q = i*NT + tid of an operand's stage
    // <-> (row q / K_CH, position q % K_CH): one instruction moves two whole rows of 512 bytes.
    struct DmaK {
        const char *a_col, *b_col;  // &A[0][m0], &B[0][n0] (wave-uniform)
        int64_t lda, ldb;           // row strides in bytes
        uint32_t oa[K_LOADS], ob[K_LOADS];
        uint32_t lds_wave;
        // Mr, Nr: readable length of a row of A, B (multiples of 8 elements); chunks past it are
        // fetched from the row's last readable chunk (the caller masks those columns).
        // a_sub / b_sub != 0: the operand's columns are stored in blocks of kBlockK (the k-blocked
        // layout of Dma seen from the other side): column c of row k at
        // base + (c / kBlockK) * sub + k * ld + (c % kBlockK) * 2 bytes, all BM (BN) columns readable.
        __device__ __forceinline__ DmaK(const char *A, int64_t lda_bytes, int64_t m0, int64_t Mr, const char *B,
                                        int64_t ldb_bytes, int64_t n0, int64_t Nr, char *lds, int64_t a_sub,
                                        int64_t b_sub) {
            const int tid = threadIdx.x;
            auto uniform = [](const char *p) {
                const uint64_t u = reinterpret_cast<uint64_t>(p);
                const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(u));
                const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(u >> 32));
                return reinterpret_cast<const char *>((static_cast<uint64_t>(hi) << 32) | lo);
            };
            a_col = uniform(A + m0 * 2);
            b_col = uniform(B + n0 * 2);
            lda = lda_bytes;
            ldb = ldb_bytes;
            const int a_last = (Mr - m0 >= BM ? K_CH : static_cast<int>(Mr - m0) / 8) - 1;
            const int b_last = (Nr - n0 >= BN ? K_CH : static_cast<int>(Nr - n0) / 8) - 1;
#pragma unroll
            for (int i = 0; i < K_LOADS; ++i) {
                const int q = i * NT + tid, row = q / K_CH, c = (q % K_CH) ^ ksw(row);
                constexpr int cpb = kBlockK / 8;  // 16-byte chunks per block of columns
                oa[i] = a_sub ? static_cast<uint32_t>((c / cpb) * a_sub + row * lda_bytes + (c % cpb) * 16)
                              : static_cast<uint32_t>(row * lda_bytes + (c < a_last ? c : a_last) * 16);
                ob[i] = b_sub ? static_cast<uint32_t>((c / cpb) * b_sub + row * ldb_bytes + (c % cpb) * 16)
                              : static_cast<uint32_t>(row * ldb_bytes + (c < b_last ? c : b_last) * 16);
            }
            lds_wave = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) char *)lds)) +
                       wave_id() * (kWave * 16);
        }
        __device__ __forceinline__ void one(int kt, int i) const {
            const uint32_t la = lds_wave + (kt % kStages) * STAGE_BYTES;
            if (i < K_LOADS) Dma::dma(a_col + static_cast<int64_t>(kt) * kBK * lda, oa[i], la + i * (NT * 16));
            else Dma::dma(b_col + static_cast<int64_t>(kt) * kBK * ldb, ob[i - K_LOADS], la + A_BYTES + (i - K_LOADS) * (NT * 16));
        }
        __device__ __forceinline__ void stage(int kt) const {
#pragma unroll
            for (int i = 0; i < STAGE_LOADS; ++i) one(kt, i);
        }
    };

    // acc += sum_k A[k][m0..] * B[k][n0..] over k < kBK*KT; every row k < kBK*KT of both operands
    // must be readable.  Same schedule as mainloop; the fragments come out of LDS with
    // ds_read_b64_tr_b16: within a group of 16 lanes, lane i receives element i%4 of the four
    // source lanes i/4, i/4+4, i/4+8, i/4+12.  Source lane s points at row k0 + s/4, columns
    // 4*(s%4).. of a 16-column block, so lane i ends up with rows k0..k0+3 of column i; the
    // group index selects k0 = 8*(l/16) and a second read 4 rows down completes the 8 values
    // per lane that the MFMA wants (two reads per fragment, one read per MFMA while they last).
    __device__ static __forceinline__ void mainloop_kmajor(const char *__restrict__ A, int64_t lda_bytes, int64_t m0, int64_t Mr,
                                                           const char *__restrict__ B, int64_t ldb_bytes, int64_t n0, int64_t Nr,
                                                           int KT, char *lds, Acc &acc, int64_t a_sub = 0, int64_t b_sub = 0) {
        typedef short v4s __attribute__((ext_vector_type(4)));
        typedef short v8s __attribute__((ext_vector_type(8)));
        static_assert(KK == 2 && kStages == 2, "two k-slices per stage, two stages");
        constexpr int NR = 2 * (FM + FN);  // reads per k-slice
        static_assert(NR <= FM * FN && STAGE_LOADS * 4 <= FM * FN, "reads and DMA fit between the MFMAs of a slice");
        static_assert((32 + 4) * K_ROWB < 65536, "slice and half offsets fit the read's offset field");
        const int lane = threadIdx.x & 63;
        const DmaK d(A, lda_bytes, m0, Mr, B, ldb_bytes, n0, Nr, lds, a_sub, b_sub);
        const int G = lane >> 4, sl = lane & 15;
        // LDS address of this lane's source piece of a block, slice 0, first half, stage 0.  The
        // slice adds 32 rows and the half 4 rows (neither changes ksw); the stage is toggled in.
        auto src_off = [&](int col0) {
            const int row = 8 * G + (sl >> 2);
            const int col = col0 + 4 * (sl & 3);
            return row * K_ROWB + (((col >> 3) ^ ksw(row)) << 4) + ((col >> 2) & 1) * 8;
        };
        const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) char *)lds));
        uint32_t a_addr[FM], b_addr[FN];
#pragma unroll
        for (int b = 0; b < FM; ++b) a_addr[b] = lds0 + src_off(wave_m0() + b * MI);
#pragma unroll
        for (int b = 0; b < FN; ++b) b_addr[b] = lds0 + A_BYTES + src_off(wave_n0() + b * MI);
        int to_other = STAGE_BYTES;  // distance to the stage the addresses do not point at
        auto other_stage = [&] {
#pragma unroll
            for (int b = 0; b < FM; ++b) a_addr[b] += to_other;
#pragma unroll
            for (int b = 0; b < FN; ++b) b_addr[b] += to_other;
            to_other = -to_other;
        };
        auto fence_barrier = [] {
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
        };
        v4s ah[2][FM][2], bh[2][FN][2];  // [register set][block][half of the 8 contraction values]
        // read r (0 .. NR-1) of k-slice kk of the stage the addresses point at, into register set buf
        auto read_half = [&](int kk, int buf, int r) {
            const int blk = r >> 1, h = r & 1;
            const int off = (32 * kk + 4 * h) * K_ROWB;
            if (blk < FM)
                ah[buf][blk][h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (v4s __attribute__((address_space(3))) *)(uintptr_t)(a_addr[blk] + off));
            else
                bh[buf][blk - FM][h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (v4s __attribute__((address_space(3))) *)(uintptr_t)(b_addr[blk - FM] + off));
        };
        auto frag = [](const v4s (&p)[2]) {
            const v8s v = __builtin_shufflevector(p[0], p[1], 0, 1, 2, 3, 4, 5, 6, 7);
            return __builtin_bit_cast(bf16x8_t, v);
        };
        __syncthreads();  // every wave is done with the previous contents of lds
        d.stage(0);
        if (KT > 1) {
            d.stage(1);
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(STAGE_LOADS) : "memory");  // loads return in order: stage 0 has landed
        } else {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        fence_barrier();
#pragma unroll
        for (int r = 0; r < NR; ++r) read_half(0, 0, r);
        auto step = [&](int kt, auto more_t, auto feed_t) {  // flags as in mainloop
            constexpr bool MORE = decltype(more_t)::value, FEED = decltype(feed_t)::value;
            // ---- slice 0 of stage kt, reading its slice 1 between the MFMAs
#pragma unroll
            for (int j = 0; j < FM * FN; ++j) {
                const int fm = j / FN, fn = j % FN;
                if (j < NR) {
                    read_half(1, 1, j);
                    __builtin_amdgcn_sched_barrier(0);
                }
                acc[fm][fn] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(frag(ah[0][fm]), frag(bh[0][fn]), acc[fm][fn], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
            fence_barrier();
            other_stage();
            // ---- slice 1, reading slice 0 of stage kt+1 and feeding the DMA of stage kt+2
#pragma unroll
            for (int j = 0; j < FM * FN; ++j) {
                const int fm = j / FN, fn = j % FN;
                if (j < NR) {
                    if (MORE) read_half(0, 0, j);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (j % 4 == 1 && j / 4 < STAGE_LOADS) {
                    if (FEED) d.one(kt + 2, j / 4);
                    __builtin_amdgcn_sched_barrier(0);
                }
                acc[fm][fn] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(frag(ah[1][fm]), frag(bh[1][fn]), acc[fm][fn], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        int kt = 0;
        for (; kt + 2 < KT; ++kt) step(kt, std::true_type{}, std::true_type{});
        if (kt + 1 < KT) step(kt++, std::true_type{}, std::false_type{});
        step(kt, std::false_type{}, std::false_type{});
    }

    __device__ static __forceinline__ void zero(Acc &acc) {
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
#pragma unroll
            for (int fn = 0; fn < FN; ++fn)
#pragma unroll
                for (int r = 0; r < ACC_R; ++r) acc[fm][fn][r] = 0.0f;
    }
};

// Maps a linear workgroup id to a tile of an nM x nN tile grid so that the 32
// workgroups that run together on one XCD (ids equal mod 8 are dispatched to the
// same XCD and share its L2) form a 4 x 8 patch: 12 operand panels feed 32 tiles.
// Patches are walked along N first: with N the short dimension (the 16 tiles of a
// hidden size of 4096 are two patches) the eight XCDs then work on few M panels and
// all N panels at the same time, so an M panel (rows of the logit gradients, the
// large operand of both backward contractions) is fetched from memory once instead
// of once per N patch (measured against walking M first: dHidden -1.6 %, dW -2.4 %).
// Returns false for ids beyond the grid.
struct TileOrder {
    int64_t nM, nN, pM, pN;  // tiles and patches per dimension
    __host__ __device__ TileOrder(int64_t nm, int64_t nn) : nM(nm), nN(nn), pM((nm + 3) / 4), pN((nn + 7) / 8) {}
    __host__ __device__ int64_t blocks() const { return (pM * pN + 7) / 8 * 8 * 32; }
    __device__ bool tile(int64_t bid, int64_t &tm, int64_t &tn) const {
        const int64_t xcd = bid & 7, q = bid >> 3;
        const int64_t patch = (q >> 5) * 8 + xcd, w = q & 31;
        if (patch >= pM * pN) return false;
        tm = (patch / pN) * 4 + (w >> 3);
        tn = (patch % pN) * 8 + (w & 7);
        return tm < nM && tn < nN;
    }
};

}  // namespace spo
