// Fused LM-head + clipped policy-gradient loss, forward and backward, on bf16
// MFMA (Method, PPO-Clip objective over the full vocabulary).  The [T x V] logits
// never exist in memory:
//   forward   sweeps vocabulary tiles, keeping a running (max, sum-exp) per token;
//             the sampled token's logit is one dot product per token beside it;
//   backward  recomputes the logits tile by tile, turns them into bf16 logit
//             gradients dZ for one chunk of tokens at a time, and contracts that
//             chunk twice (dHidden = dZ W, dW += dZ^T X);
//   forward and backward in one call (when d(total)/d(loss) is known up front)
//             walks the batch in pieces: the sweep of a piece also stores, at two
//             bytes per logit, what the two contractions of that piece then
//             read, so the logits are formed once.
// The logits and dHidden run through the main loop of gemm_core.hpp in the form
// D[m][n] = sum_k A[m][k] B[n][k] (a transposition kernel provides the head with
// the vocabulary contiguous for dHidden); dW contracts over tokens, the row index
// of both dZ and the hidden states, through the loop's second form
// D[m][n] = sum_k A[k][m] B[k][n], so neither is copied.
//
// fp32 inputs use the same bf16 main loop: every value is split into three bf16
// parts (x = x0 + x1 + x2) and the six leading cross products are laid side by
// side along the contraction index, which recovers fp32-grade logits.
#include <algorithm>

#include "gemm_core.hpp"
#include "pg_common.hpp"
#include "timing.hpp"

namespace spo {

// 8 wavefronts, each a 128 x 64 part of the tile, on 16x16x32 MFMAs (measured 4-6 % faster
// than the same tile on 32x32x16 on the same chip: the instruction draws less power).
typedef Tile<256, 256, 2, 4, 16> TL;
constexpr int kSplitTerms = 6;    // cross products kept by the fp32 split
constexpr int kSweepSplits = 16;  // vocabulary splits of the forward sweep on large problems (a multiple of 8)
// Default size of a backward chunk: as many tokens as keep the chunk's bf16 logit gradients
// (2 * V bytes per token) within this budget, in whole rounds of dHidden tiles on the chip's
// 256 compute units.  dW is read and rewritten once per chunk and every launch ends in a
// partly filled round of tiles, so larger chunks (the caller's choice) are a little faster:
// at H = 4096, V = 151936 the step takes about 1 % longer with 8 GiB than with 40 GB.
constexpr int64_t kDzBudgetBytes = int64_t(8) << 30;
constexpr int kChipCUs = 256;
constexpr int kTailTiles = kChipCUs;  // fp32 tiles of room for the parts of a short last round of tiles (see TailCut)

static int64_t gcd64(int64_t a, int64_t b) { return b ? gcd64(b, a % b) : a; }

// tokens per chunk when the caller leaves the choice to the library (a multiple of the tile)
static int64_t default_chunk_tokens(int64_t H, int64_t V_blk) {
    const int64_t fit = kDzBudgetBytes / (2 * V_blk) / TL::BN * TL::BN;  // tokens within the budget
    const int64_t nHt = (H + TL::BM - 1) / TL::BM;                        // dHidden tiles per token tile
    const int64_t round = TL::BN * (kChipCUs / gcd64(kChipCUs, nHt));     // tokens per full round of tiles
    if (fit >= round) return fit / round * round;
    return fit > TL::BN ? fit : TL::BN;
}

// ----------------------------------------------------------------------------
// operand preparation
// ----------------------------------------------------------------------------

// dst[r][j*K + k] = part_{sel(j)}(src[r][k]) with sel = {0,0,1,0,2,1} (side 0) or
// {0,1,0,2,0,1} (side 1): sum_j dst0[.][jK+k] * dst1[.][jK+k] keeps the products
// x0y0, x0y1, x1y0, x0y2, x2y0, x1y1 of the three-part bf16 splits of x and y.
__global__ void __launch_bounds__(256)
split_expand_kernel(const float *__restrict__ src, int64_t rows, int64_t K, bf16_t *__restrict__ dst, int side) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= rows * K) return;
    const int64_t r = i / K, k = i % K;
    const float x = src[i];
    const bf16_t p0 = f32_to_bf16(x);
    const float r1 = x - bf16_to_f32(p0);
    const bf16_t p1 = f32_to_bf16(r1);
    const bf16_t p2 = f32_to_bf16(r1 - bf16_to_f32(p1));
    bf16_t *o = dst + r * (kSplitTerms * K) + k;
    if (side == 0) {
        o[0] = p0; o[K] = p0; o[2 * K] = p1; o[3 * K] = p0; o[4 * K] = p2; o[5 * K] = p1;
    } else {
        o[0] = p0; o[K] = p1; o[2 * K] = p0; o[3 * K] = p2; o[4 * K] = p0; o[5 * K] = p1;
    }
}

__device__ __forceinline__ bf16_t load_as_bf16(const bf16_t *p) { return *p; }
__device__ __forceinline__ bf16_t load_as_bf16(const float *p) { return f32_to_bf16(*p); }

// dst[c][r] = bf16(src[r][c]) for r < R, c < C; dst[c][r] = 0 for R <= r < R_pad and
// for C <= c < C_pad (all r < R_pad).  dst has leading dimension ld_dst >= R_pad, or with
// ld_dst == 0 it is stored in blocks of kBlockK values of r (the layout the main loop reads
// as a k-blocked operand): dst[c][r] at (r / kBlockK) * C_pad * kBlockK + c * kBlockK + r % kBlockK.
template <typename SrcT>
__global__ void __launch_bounds__(256)
transpose_to_bf16_kernel(const SrcT *__restrict__ src, int64_t R, int64_t C, int64_t ld_src,
                         bf16_t *__restrict__ dst, int64_t R_pad, int64_t C_pad, int64_t ld_dst) {
    __shared__ bf16_t tile[64][66];
    const int64_t r0 = static_cast<int64_t>(blockIdx.x) * 64, c0 = static_cast<int64_t>(blockIdx.y) * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int i = ty; i < 64; i += 4) {
        const int64_t r = r0 + i, c = c0 + tx;
        tile[i][tx] = (r < R && c < C) ? load_as_bf16(src + r * ld_src + c) : bf16_t(0);
    }
    __syncthreads();
    for (int i = ty; i < 64; i += 4) {
        const int64_t c = c0 + i, r = r0 + tx;
        if (c < C_pad && r < R_pad)
            dst[ld_dst ? c * ld_dst + r : (r / kBlockK) * (C_pad * kBlockK) + c * kBlockK + r % kBlockK] = tile[tx][i];
    }
}

// dst[c][r] = src[r][c] (fp32, R x C -> C x R), 64 x 64 tiles through LDS.
__global__ void __launch_bounds__(256)
transpose_f32_kernel(const float *__restrict__ src, int64_t R, int64_t C, float *__restrict__ dst) {
    __shared__ float tile[64][65];
    const int64_t r0 = static_cast<int64_t>(blockIdx.x) * 64, c0 = static_cast<int64_t>(blockIdx.y) * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int i = ty; i < 64; i += 4)
        if (r0 + i < R && c0 + tx < C) tile[i][tx] = src[(r0 + i) * C + c0 + tx];
    __syncthreads();
    for (int i = ty; i < 64; i += 4)
        if (c0 + i < C && r0 + tx < R) dst[(c0 + i) * R + r0 + tx] = tile[tx][i];
}

__global__ void __launch_bounds__(256)
f32_to_bf16_kernel(const float *__restrict__ src, bf16_t *__restrict__ dst, int64_t n) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < n) dst[i] = f32_to_bf16(src[i]);
}

__global__ void __launch_bounds__(256) fill_zero_kernel(uint32_t *__restrict__ p, int64_t n_words) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < n_words) p[i] = 0u;
}

// ----------------------------------------------------------------------------
// backward: compaction of the tokens that carry a gradient
// ----------------------------------------------------------------------------
// Masked tokens, tokens on the clipped branch and tokens of a response with zero
// advantage have g = 0: their rows of dZ vanish, so the backward contractions run
// over the remaining ("active") tokens only, in their original order.

// act_idx[j] = index of the j-th token with g != 0; n_act[0] = their number.
// One workgroup walks the tokens 4096 at a time (order-preserving, deterministic).
__global__ void __launch_bounds__(1024)
compact_active_kernel(const float *__restrict__ g, int64_t T, int32_t *__restrict__ act_idx,
                      int32_t *__restrict__ n_act) {
    __shared__ int wave_cnt[16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int base = 0;
    for (int64_t t0 = 0; t0 < T; t0 += 4096) {
        const int64_t t = t0 + threadIdx.x * 4;
        bool on[4];
        int mine = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            on[i] = t + i < T && g[t + i] != 0.0f;
            mine += on[i] ? 1 : 0;
        }
        // exclusive prefix of `mine` over the wavefront, then over the 16 wavefronts
        int incl = mine;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const int up = __shfl_up(incl, d, kWave);
            if (lane >= d) incl += up;
        }
        if (lane == kWave - 1) wave_cnt[wave] = incl;
        __syncthreads();
        int off = 0, tot = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const int c = wave_cnt[w];
            off += w < wave ? c : 0;
            tot += c;
        }
        int pos = base + off + incl - mine;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (on[i]) act_idx[pos++] = static_cast<int32_t>(t + i);
        base += tot;
        __syncthreads();
    }
    if (threadIdx.x == 0) n_act[0] = base;
}

// Number of active tokens that fall into rows [row_base, row_base + cap) of the compact order.
__device__ __forceinline__ int64_t active_rows(const int32_t *n_act, int64_t row_base, int64_t cap) {
    const int64_t n = static_cast<int64_t>(*n_act) - row_base;
    return n < 0 ? 0 : (n > cap ? cap : n);
}

// Rows [row_base, row_base + rows) of the compact order as contiguous copies: the hidden
// states (Xc[r] = X[act_idx[row_base + r]]) and, packed into one 16-byte record per row, the
// per-token scalars the recompute needs: tok[r] = (|g|, log2|g| - lse * log2(e), target with the
// sign of g in the top bit (set: g > 0), 0): the gradient's softmax part -g * p is then
// -sign(g) * exp2(z * log2(e) + tok.y), one multiply-add and one exponential per logit.
// Rows past the last active token are filled with zeros and (0, -inf, no target): every
// exponential underflows to an exact zero.  One workgroup per row.
template <typename T_>
__global__ void __launch_bounds__(256)
gather_chunk_kernel(const T_ *__restrict__ X, int64_t H, const int32_t *__restrict__ act_idx,
                    const int32_t *__restrict__ n_act, int64_t row_base, int64_t rows,
                    const int32_t *__restrict__ target, const float *__restrict__ lse, const float *__restrict__ g,
                    T_ *__restrict__ Xc, float4 *__restrict__ tok) {
    const int64_t r = blockIdx.x;
    const bool live = r < active_rows(n_act, row_base, rows);
    const int64_t src = live ? act_idx[row_base + r] : 0;
    const int n16 = static_cast<int>(H * sizeof(T_) / 16);  // H is a multiple of 64
    const uint4 *in = reinterpret_cast<const uint4 *>(X + src * H);
    uint4 *out = reinterpret_cast<uint4 *>(Xc + r * H);
    for (int i = threadIdx.x; i < n16; i += 256) out[i] = live ? in[i] : make_uint4(0u, 0u, 0u, 0u);
    if (threadIdx.x == 0) {
        const float gs = live ? g[src] : 0.0f;
        const uint32_t ts = live ? (static_cast<uint32_t>(target[src]) & 0x7fffffffu) | (gs > 0.0f ? 0x80000000u : 0u)
                                 : 0x7fffffffu;
        tok[r] = make_float4(fabsf(gs), live ? log2f(fabsf(gs)) - lse[src] * kLog2e : -INFINITY, __uint_as_float(ts), 0.0f);
    }
}

// ----------------------------------------------------------------------------
// forward: logit of the sampled token
// ----------------------------------------------------------------------------
// z_target[t] = h_t . W[target[t]] (W with one row per vocabulary entry), one wavefront per
// token, products and sum in fp32.  The sweep below does not have to watch for this one
// entry of every row.  An id outside [0, V) gives NaN (the token's log-prob, and with it the
// loss, then say so instead of carrying an arbitrary number).
__device__ __forceinline__ float dot8(const uint4 a, const uint4 b) {
    const uint32_t x[4] = {a.x, a.y, a.z, a.w}, y[4] = {b.x, b.y, b.z, b.w};
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        s = fmaf(__uint_as_float(x[i] << 16), __uint_as_float(y[i] << 16), s);
        s = fmaf(__uint_as_float(x[i] & 0xffff0000u), __uint_as_float(y[i] & 0xffff0000u), s);
    }
    return s;
}

template <typename T_>
__global__ void __launch_bounds__(256)
target_logit_kernel(const T_ *__restrict__ X, const T_ *__restrict__ Wvh, int64_t H, int64_t V, int64_t T,
                    const int32_t *__restrict__ target, float *__restrict__ z_target) {
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (t >= T) return;
    const int64_t y = target[t];
    if (y < 0 || y >= V) {
        if (lane == 0) z_target[t] = __builtin_nanf("");
        return;
    }
    float s = 0.0f;
    if constexpr (sizeof(T_) == 2) {
        const uint4 *x = reinterpret_cast<const uint4 *>(X + t * H), *w = reinterpret_cast<const uint4 *>(Wvh + y * H);
        for (int i = lane; i < H / 8; i += kWave) s += dot8(x[i], w[i]);  // H is a multiple of 64
    } else {
        const float4 *x = reinterpret_cast<const float4 *>(X + t * H), *w = reinterpret_cast<const float4 *>(Wvh + y * H);
        for (int i = lane; i < H / 4; i += kWave) {
            const float4 a = x[i], b = w[i];
            s = fmaf(a.x, b.x, s); s = fmaf(a.y, b.y, s); s = fmaf(a.z, b.z, s); s = fmaf(a.w, b.w, s);
        }
    }
    s = wave_sum(s);
    if (lane == 0) z_target[t] = s;
}

// ----------------------------------------------------------------------------
// forward: vocabulary sweep with online log-sum-exp
// ----------------------------------------------------------------------------
// Tile rows (m) are vocabulary entries, tile columns (n) are tokens, so that each
// lane owns FN tokens and reduces over the vocabulary inside its own registers.

// Workgroup -> (token tile, vocabulary split) of the two kernels that form logits (the forward
// sweep and the backward's recompute): a workgroup keeps its token tile and walks the vocabulary
// tiles of its split.  Ids equal mod 8 run on the same XCD and share its L2: there, 32
// consecutive workgroups are a patch of 4 token tiles x 8 splits (each hidden-state panel feeds
// 8 of them, each head tile 4), and the eight XCDs work on the same splits of different token
// tiles at about the same time, so a head tile fetched from memory serves 32 token tiles out of
// the Infinity Cache.  (A 4 x 8 patch of tiles walked along the vocabulary, every head tile used by
// one XCD only, made the recompute 3.6 % slower.)  More than 8 splits shorten a workgroup's
// sweep: workgroups that share lines then have less time to drift apart.
struct SweepMap {
    int nsplit;
    int64_t nTt, nVt, per_xcd;
    // splits = 0: chosen here; otherwise the caller's number (kept when it is a multiple of 8 or below 8)
    __host__ __device__ SweepMap(int64_t token_tiles, int64_t vocab_tiles, int splits = 0)
        : nTt(token_tiles), nVt(vocab_tiles) {
        int64_t ns = (2048 + (nTt > 0 ? nTt : 1) - 1) / (nTt > 0 ? nTt : 1);  // small batches: more splits fill the chip
        ns = ns < kSweepSplits ? kSweepSplits : ns;
        if (splits > 0) ns = splits;
        ns = ns < nVt ? ns : nVt;
        nsplit = static_cast<int>(ns >= 8 ? ns / 8 * 8 : ns);  // whole groups of 8 splits whenever there are 8
        const int64_t x = (nTt + 7) / 8;
        per_xcd = nsplit % 8 == 0 ? (x + 3) / 4 * 4 : x;  // whole patches of 4 when the splits come in groups of 8
    }
    __host__ __device__ int64_t blocks() const { return per_xcd * 8 * nsplit; }
    // token tile jt and split of workgroup bid; false past the last token tile
    __device__ bool tile(int64_t bid, int &split, int64_t &jt) const {
        const int64_t xcd = bid & 7, q = bid >> 3;
        if (nsplit % 8 == 0) {
            const int groups = nsplit / 8, w = static_cast<int>(q & 31);
            const int64_t patch = q >> 5;
            split = static_cast<int>(patch % groups) * 8 + (w & 7);
            jt = ((patch / groups) * 4 + (w >> 3)) * 8 + xcd;
        } else {  // small problems: all splits of a token tile side by side
            split = static_cast<int>(q % nsplit);
            jt = (q / nsplit) * 8 + xcd;
        }
        return jt < nTt;
    }
    __host__ __device__ int64_t first_tile(int split) const { return split * nVt / nsplit; }
};

constexpr int kSweepLds = TL::LDS_BYTES + TL::NT * 32;       // operand stages + the per-thread running state
constexpr int kSweepLdsProbs = TL::LDS_BYTES + TL::NT * 48;  // ... + the per-token references

// Exchange between neighbouring groups of 16 lanes: v_permlane16_swap(a, b) swaps the odd groups
// of a with the even groups of b.  With a, b the values a lane holds for two consecutive MFMA
// blocks q, q+1, lane group g ends up with (in a, b) the values of block q + (g & 1) from lane
// groups (g & 2) and (g & 2) + 1.
__device__ __forceinline__ void swap_lane_groups(uint32_t &a, uint32_t &b) {
    typedef unsigned v2u __attribute__((ext_vector_type(2)));
    const v2u t = __builtin_amdgcn_permlane16_swap(a, b, false, false);
    a = t.x;
    b = t.y;
}

// two floats as a pair of IEEE halves, round to nearest even
__device__ __forceinline__ uint32_t pack_f16x2_rn(float lo, float hi) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    const h2 v = {static_cast<_Float16>(lo), static_cast<_Float16>(hi)};
    return __builtin_bit_cast(uint32_t, v);
}

// Emit = kEmitNone: the forward proper; the logits exist in registers only.
// The other two forms serve the one-call forward + backward: every finished tile is also
// written out, in the blocked layout of the logit gradients (token n of this launch, vocabulary
// entry v at Z + (v / 64) * z_blk + n * 64 + v % 64).
// Emit = kEmitLogits: fp16 of (logit - offset).  The offset is the running maximum of the token
// over the 128 vocabulary rows per tile that the wavefront has seen so far in its sweep, this
// tile included: one value per (vocabulary tile, half of the tile, token), written to
// offs[(tile * 2 + half) * T_pad + n].  Stored values are <= 0, and an entry within d of the
// row's largest logit is stored within d of zero, where fp16 resolves 2^-11 * d: the entries
// that carry the softmax are the most exact ones.  Rows past the vocabulary are stored as -inf.
// Emit = kEmitProbs: bf16 of exp(logit - r_n), with r_n a per-token reference known before the
// sweep (offs[n] = r_n * log2(e) on entry; see the host code for the choice that makes these
// the softmax probabilities divided by the token's importance ratio).  The exponentials are the
// ones the running sum needs anyway, times one factor per token and lane; exponents are capped
// at 126 so that nothing stored is infinite.  Rows past the vocabulary are stored as zeros.
constexpr int kEmitNone = 0, kEmitLogits = 1, kEmitProbs = 2;

template <int Emit>
__global__ void __launch_bounds__(TL::NT)
fwd_sweep_kernel(const char *__restrict__ W, int64_t ldw_bytes, int64_t V, const char *__restrict__ X,
                 int64_t ldx_bytes, int64_t T, int KT, int nsplit, int64_t nTt, int64_t nVt, int64_t T_pad,
                 float *__restrict__ part_max, float *__restrict__ part_sum, uint16_t *__restrict__ Z, int64_t z_blk,
                 float *__restrict__ offs) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const SweepMap map(nTt, nVt, nsplit);  // the host sized the partial results with the same map
    int split;
    int64_t jt;
    if (!map.tile(blockIdx.x, split, jt)) return;
    const int64_t n0 = jt * TL::BN;
    const int64_t vt0 = map.first_tile(split), vt1 = map.first_tile(split + 1);
    const int lane = threadIdx.x & 63;

    // Running (maximum, sum of exponentials) of this lane's FN tokens.  Between tiles they wait in
    // the LDS the operand stages leave free (a slot per thread): the main loop needs every register.
    static_assert(TL::FN == 4, "one 16-byte slot each for the maxima and the sums");
    auto state = [&] {
        int tid = threadIdx.x;
        asm volatile("" : "+v"(tid));  // not to be traced: the address is formed anew at every use
        return reinterpret_cast<float4 *>(lds + TL::LDS_BYTES) + (Emit == kEmitProbs ? 3 : 2) * tid;
    };
    state()[0] = make_float4(kNegBig, kNegBig, kNegBig, kNegBig);
    state()[1] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (Emit == kEmitProbs) {  // the references of this lane's four tokens: the workgroup keeps its token tile
        const float *r = offs + n0 + TL::wave_n0() + (lane & 15);
        state()[2] = make_float4(r[0], r[TL::MI], r[2 * TL::MI], r[3 * TL::MI]);
    }
    // One finished tile.  Online log-sum-exp over its rows: three operations per logit (multiply-add
    // into the exponent, exponential, add) plus its share of the maximum.  With Emit, the tile's
    // values also leave for memory, token column by token column as each is done, so that the stores
    // of one column are on their way while the next is being worked on.  A lane holds runs of four
    // consecutive vocabulary entries of one token; after an exchange between neighbouring lane
    // groups it holds 16 contiguous bytes of two 64-entry blocks out of four (the scheme of the
    // recompute's epilogue below).
    auto finish_tile = [&](TL::Acc &acc, int64_t vt) {
        const int64_t m0 = vt * TL::BM;
        if (m0 + TL::BM > V) {  // ragged last tile: rows past the vocabulary do not count
#pragma unroll
            for (int fm = 0; fm < TL::FM; ++fm)
#pragma unroll
                for (int r = 0; r < TL::ACC_R; ++r)
                    if (m0 + TL::acc_row(fm, r) >= V)
#pragma unroll
                        for (int fn = 0; fn < TL::FN; ++fn) acc[fm][fn][r] = -INFINITY;
        }
        int l = threadIdx.x & 63;
        asm volatile("" : "+v"(l));  // not to be traced: nothing derived from it lives through the main loop
        const int grp = l >> 4, col = l & 15;
        const int64_t wave_blk = vt * (TL::BM / kBlockK) + TL::wave_m0() / kBlockK;
        const int piece = (grp & 1) * 16 + (grp & 2) * 4;  // elements: byte offset 32 * (g & 1) + 8 * (g & 2)
        float4 *st = state();
        const float4 m4 = st[0], s4 = st[1];
        float m_run[TL::FN] = {m4.x, m4.y, m4.z, m4.w}, s_run[TL::FN] = {s4.x, s4.y, s4.z, s4.w};
        float ref[TL::FN] = {0.0f, 0.0f, 0.0f, 0.0f};
        if (Emit == kEmitProbs) {
            const float4 r4 = st[2];
            ref[0] = r4.x; ref[1] = r4.y; ref[2] = r4.z; ref[3] = r4.w;
        }
#pragma unroll
        for (int fn = 0; fn < TL::FN; ++fn) {
            float mx = -INFINITY;
#pragma unroll
            for (int fm = 0; fm < TL::FM; ++fm)
#pragma unroll
                for (int r = 0; r < TL::ACC_R; ++r) mx = fmaxf(mx, acc[fm][fn][r]);
            // the running maximum starts at a finite sentinel, so nm is finite even when every
            // row of the tile is masked (their logits are -inf and add exact zeros)
            const float nm = fmaxf(m_run[fn], mx);
            const float c = -nm * kLog2e;
            // what is stored of an entry: a * value + b, with value the exponential (kEmitProbs: times
            // exp(nm - r), capped) or the logit itself (kEmitLogits: minus the offset, the largest logit the
            // wavefront's 128 rows have shown for this token so far)
            float a = 0.0f, off = 0.0f;
            if (Emit == kEmitProbs) a = __builtin_amdgcn_exp2f(fminf(fmaf(nm, kLog2e, -ref[fn]), 126.0f));
            if (Emit == kEmitLogits) {
                off = fmaxf(nm, __shfl_xor(nm, 16, kWave));
                off = fmaxf(off, __shfl_xor(off, 32, kWave));
                if (grp == 0)
                    offs[(vt * TL::WGM + TL::wave_m0() / TL::WM) * T_pad + n0 + TL::wave_n0() + fn * TL::MI + col] = off;
            }
            float s = 0.0f;
            uint16_t *row = Emit ? Z + (n0 + TL::wave_n0() + fn * TL::MI + col) * kBlockK + piece : nullptr;
#pragma unroll
            for (int b = 0; b < TL::FM / 4; ++b) {
                uint32_t lo[4], hi[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float e[4], v[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        e[r] = __builtin_amdgcn_exp2f(fmaf(acc[4 * b + q][fn][r], kLog2e, c));
                        s += e[r];
                        v[r] = Emit == kEmitProbs ? e[r] * a : acc[4 * b + q][fn][r] - off;
                    }
                    if (Emit == kEmitProbs) {
                        lo[q] = pack_bf16x2_rn(v[0], v[1]);
                        hi[q] = pack_bf16x2_rn(v[2], v[3]);
                    }
                    if (Emit == kEmitLogits) {
                        lo[q] = pack_f16x2_rn(v[0], v[1]);
                        hi[q] = pack_f16x2_rn(v[2], v[3]);
                    }
                }
                if (Emit) {
                    swap_lane_groups(lo[0], lo[1]);
                    swap_lane_groups(hi[0], hi[1]);
                    swap_lane_groups(lo[2], lo[3]);
                    swap_lane_groups(hi[2], hi[3]);
                    uint16_t *out = row + (wave_blk + b) * z_blk;
                    *reinterpret_cast<uint4 *>(out) = make_uint4(lo[0], hi[0], lo[1], hi[1]);
                    *reinterpret_cast<uint4 *>(out + kBlockK / 2) = make_uint4(lo[2], hi[2], lo[3], hi[3]);
                }
            }
            s_run[fn] = s_run[fn] * __builtin_amdgcn_exp2f((m_run[fn] - nm) * kLog2e) + s;
            m_run[fn] = nm;
        }
        st[0] = make_float4(m_run[0], m_run[1], m_run[2], m_run[3]);
        st[1] = make_float4(s_run[0], s_run[1], s_run[2], s_run[3]);
    };
    auto tile_ops = [&](int64_t vt) { return typename TL::Operands{W, ldw_bytes, vt * TL::BM, V, X, ldx_bytes, n0, T, 0, 0}; };
    for (int64_t vt = vt0; vt < vt1; ++vt) {
        TL::Acc acc;
        TL::zero(acc);
        TL::mainloop(tile_ops(vt), KT, lds, acc);
        finish_tile(acc, vt);
    }
    // merge the lane groups that hold different rows of the same token, then the WGM
    // wavefronts that share a token column
    float *red_m = reinterpret_cast<float *>(lds);
    float *red_s = red_m + TL::WGM * TL::BN;
    const float4 m4 = state()[0], s4 = state()[1];
    const float m_run[TL::FN] = {m4.x, m4.y, m4.z, m4.w}, s_run[TL::FN] = {s4.x, s4.y, s4.z, s4.w};
    __syncthreads();  // operand stages are no longer read
#pragma unroll
    for (int fn = 0; fn < TL::FN; ++fn) {
        float m = m_run[fn], sum = s_run[fn];
#pragma unroll
        for (int o = TL::MI; o < kWave; o <<= 1) {
            const float om = __shfl_xor(m, o, kWave), os = __shfl_xor(sum, o, kWave);
            const float nm = fmaxf(m, om);
            sum = sum * __builtin_amdgcn_exp2f((m - nm) * kLog2e) + os * __builtin_amdgcn_exp2f((om - nm) * kLog2e);
            m = nm;
        }
        if (lane < TL::MI) {
            const int slot = (TL::wave_id() % TL::WGM) * TL::BN + TL::acc_col(fn);
            red_m[slot] = m;
            red_s[slot] = sum;
        }
    }
    __syncthreads();
    for (int c = threadIdx.x; c < TL::BN; c += TL::NT) {
        float nm = kNegBig;
#pragma unroll
        for (int w = 0; w < TL::WGM; ++w) nm = fmaxf(nm, red_m[w * TL::BN + c]);
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < TL::WGM; ++w)
            s += red_s[w * TL::BN + c] * __builtin_amdgcn_exp2f((red_m[w * TL::BN + c] - nm) * kLog2e);
        part_max[split * T_pad + n0 + c] = nm;
        part_sum[split * T_pad + n0 + c] = s;
    }
}

// ----------------------------------------------------------------------------
// backward, step 1: recompute the logits tile by tile and emit their bf16 gradient
// ----------------------------------------------------------------------------
// dz[t][v] = g[t] * ([v == target[t]] - exp(z[t][v] - lse[t])), written once, in blocks
// of kBlockK = 64 vocabulary entries: dz[t][v] at dZ + (v / 64) * dz_blk + t * 64 + v % 64
// (dz_blk elements per block = rows of the chunk * 64).  dHidden reads the blocks as a
// k-blocked operand (contraction over v: one block per k-step), dW reads four neighbouring
// blocks as a matrix with the tokens as rows (contraction over t).  Entries with v >= V and
// tokens past the active rows of their tile are written as zeros.  Token tiles that start at
// or after the number of active rows of this chunk (device value n_act[0] - row_base) are
// skipped altogether.
//
// Workgroups map to (token tile, vocabulary split) as in the forward sweep (SweepMap).  The
// gradients go from the accumulators to memory without a detour through LDS.

__global__ void __launch_bounds__(TL::NT)
recompute_dz_kernel(const char *__restrict__ W, int64_t ldw_bytes, int64_t V,
                    const char *__restrict__ X, int64_t ldx_bytes, int64_t T_valid, int KT,
                    const float4 *__restrict__ tok, int64_t nVt, int64_t nTt, bf16_t *__restrict__ dZ,
                    int64_t dz_blk, const int32_t *__restrict__ n_act, int64_t row_base) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    static_assert(TL::BM % kBlockK == 0 && kBlockK == 4 * TL::MI && TL::FM % 4 == 0,
                  "a block of dZ is four MFMA blocks of vocabulary rows");
    const int act = static_cast<int>(active_rows(n_act, row_base, T_valid));
    const SweepMap map(nTt, nVt);
    int split;
    int64_t jt;
    if (!map.tile(blockIdx.x, split, jt) || jt * TL::BN >= act) return;  // past the last active token
    const int tn = static_cast<int>(jt);
    const int vt0 = static_cast<int>(map.first_tile(split)), vt1 = static_cast<int>(map.first_tile(split + 1));
    auto tile_ops = [&](int tile_m, int tile_n) {
        return typename TL::Operands{W, ldw_bytes, static_cast<int64_t>(tile_m) * TL::BM, V, X, ldx_bytes,
                                     static_cast<int64_t>(tile_n) * TL::BN, T_valid, 0, 0};
    };
    // gradients of one finished tile
    auto emit = [&](TL::Acc &acc, int tile_m, int tile_n) {
        const int m0 = tile_m * TL::BM, n0 = tile_n * TL::BN;
        if (m0 + TL::BM > V) {  // ragged last tile: rows past the vocabulary get probability zero
#pragma unroll
            for (int fm = 0; fm < TL::FM; ++fm)
#pragma unroll
                for (int r = 0; r < TL::ACC_R; ++r)
                    if (m0 + TL::acc_row(fm, r) >= V)
#pragma unroll
                        for (int fn = 0; fn < TL::FN; ++fn) acc[fm][fn][r] = -INFINITY;
        }
        // A lane holds runs of four consecutive vocabulary entries (8 bytes of bf16) of ONE token,
        // at offset 32 * (fm % 4) + 8 * group inside that token's 128-byte row of a block of dZ.
        // After an exchange between neighbouring lane groups a lane holds 16 contiguous bytes of
        // two blocks out of four: per store instruction every token gets a contiguous 64-byte half
        // of its row.  (Everything that depends on the lane is derived here from a value the
        // compiler cannot trace, so that none of it is kept in registers across the main loop.)
        int lane = threadIdx.x & 63;
        asm volatile("" : "+v"(lane));
        const int grp = lane >> 4, col = lane & 15;
        const int wave_blk = tile_m * (TL::BM / kBlockK) + TL::wave_m0() / kBlockK;
        const int piece = (grp & 1) * 16 + (grp & 2) * 4;  // elements: byte offset 32 * (g & 1) + 8 * (g & 2)
        // the records of this wavefront's 64 tokens, one per lane (handed round with lane shuffles below)
        const float4 rec = tok[static_cast<int64_t>(n0) + TL::wave_n0() + lane];
#pragma unroll
        for (int fn = 0; fn < TL::FN; ++fn) {
            const int src = fn * TL::MI + col;
            const float ag = __shfl(rec.x, src, kWave), nl = __shfl(rec.y, src, kWave);
            const uint32_t ts = __float_as_uint(__shfl(rec.z, src, kWave));
            // the values are formed as |g| * p >= 0; the sign of -g is put on afterwards, two at a time
            const uint32_t sgn = (ts & 0x80000000u) ? 0x80008000u : 0u;
            // where the target's vocabulary row sits among this wave's rows, if it does
            const int dy = static_cast<int>(ts & 0x7fffffffu) - (m0 + TL::wave_m0());
            int fq = 0, rq = 0, gq = 0;
            const bool in_wave = static_cast<unsigned>(dy) < static_cast<unsigned>(TL::WM);
            if (in_wave) TL::locate(dy, fq, rq, gq);
            const bool mine = in_wave && gq == grp;
            bf16_t *row = dZ + static_cast<int64_t>(n0 + TL::wave_n0() + fn * TL::MI + col) * kBlockK + piece;
#pragma unroll
            for (int b = 0; b < TL::FM / 4; ++b) {
                uint32_t lo[4], hi[4];  // bf16 pairs: lo = rows +0,+1, hi = rows +2,+3 of the run of block 4b+q
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float e[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) e[i] = __builtin_amdgcn_exp2f(fmaf(acc[4 * b + q][fn][i], kLog2e, nl));
                    lo[q] = pack_bf16x2_rn(e[0], e[1]);
                    hi[q] = pack_bf16x2_rn(e[2], e[3]);
                }
                if (mine && (fq >> 2) == b) {  // rare: the one-hot term, |g| * (p - 1) before the sign goes on
                    float x = 0.0f;
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if ((fq & 3) == q && rq == i) x = acc[4 * b + q][fn][i];
                    const uint32_t v = f32_to_bf16(__builtin_amdgcn_exp2f(fmaf(x, kLog2e, nl)) - ag);
                    const uint32_t keep = (rq & 1) ? 0x0000ffffu : 0xffff0000u, put = (rq & 1) ? v << 16 : v;
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if ((fq & 3) == q) {
                            if (rq & 2) hi[q] = (hi[q] & keep) | put;
                            else lo[q] = (lo[q] & keep) | put;
                        }
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    lo[q] ^= sgn;
                    hi[q] ^= sgn;
                }
                swap_lane_groups(lo[0], lo[1]);
                swap_lane_groups(hi[0], hi[1]);
                swap_lane_groups(lo[2], lo[3]);
                swap_lane_groups(hi[2], hi[3]);
                bf16_t *out = row + (wave_blk + b) * dz_blk;
                *reinterpret_cast<uint4 *>(out) = make_uint4(lo[0], hi[0], lo[1], hi[1]);
                *reinterpret_cast<uint4 *>(out + kBlockK / 2) = make_uint4(lo[2], hi[2], lo[3], hi[3]);
            }
        }
    };
    for (int tm = vt0; tm < vt1; ++tm) {
        TL::Acc acc;
        TL::zero(acc);
        TL::mainloop(tile_ops(tm, tn), KT, lds, acc);
        emit(acc, tm, tn);
    }
}

// A launch ends in a partly filled round of tiles when its tile count is no multiple of the chip's
// compute units.  A short last round (at most half of the units busy) is cut off: the tiles
// before it run as they are, in whole rounds, and the `rem` tiles after them are each cut along the
// contraction into `parts` runs whose partial results are added in a fixed order afterwards.  Host
// and device code ask the same function, so the number of tiles may be known on the device only.
struct TailCut {
    int64_t whole;  // tiles that run in whole rounds (all of them when nothing is cut)
    int rem, parts;
    __host__ __device__ explicit TailCut(int64_t tiles) : whole(tiles), rem(0), parts(1) {
        const int r = static_cast<int>(tiles % kChipCUs);
        if (tiles > kChipCUs && r > 0 && r <= kChipCUs / 2) {
            whole = tiles - r;
            rem = r;
            parts = kChipCUs / r < 8 ? kChipCUs / r : 8;
        }
    }
};
constexpr int kTailNone = 0, kTailWhole = 1, kTailCut = 2;  // what a launch does about a short last round

// ----------------------------------------------------------------------------
// backward, steps 2 and 3: plain contraction with a store / accumulate epilogue
// ----------------------------------------------------------------------------
// out[row(m)*ldo + n] (=|+=) sum_k A[m][k] B[n][k], or with KMajor
// sum_k A[k][m] B[k][n] (rows of A and B are then readable up to the next multiple
// of 8 elements past M and N).  An operand with a_blk / b_blk != 0 is stored in blocks
// of kBlockK = 64 elements of its contiguous index, blk bytes apart, rows 128 bytes
// apart inside a block: for the plain form that index is k (see Dma), for KMajor it is
// m (n), and tile tm (tn) of the operand is made of the four blocks from 4 tm (4 tn) on
// (see DmaK).
// With n_act != NULL the extent that holds active tokens is read on the device
// (rows = active_rows(n_act, row_base, .)): limit == kLimitRows keeps only the first
// `rows` rows of A and stores row m at out row row_map[m] (dHidden: scatter back to the
// tokens' own rows); limit == kLimitK contracts only over the first `rows` values of
// the contraction index, rounded up to whole tiles of tokens (dW).  row_scale != NULL (stores that
// do not add to the output): row m of the product is multiplied by row_scale[m] on its way out.
constexpr int kLimitRows = 1, kLimitK = 2;

// With nsplit > 1 (plain form only) the contraction is cut into nsplit equal runs of k-steps;
// workgroup (tile, part) writes its fp32 partial tile to partials[part][m][n] (leading
// dimension N) and reduce_split_kernel adds the parts in a fixed order: shapes with fewer
// tiles than the chip has compute units still fill it, and the result does not depend on timing.
//
// Epilogue: the accumulators go out through LDS (the operand stages are free by then), half a
// tile at a time: a lane holds four consecutive ROWS of one column, so stored directly a
// wavefront would scatter 64-byte pieces over many rows per instruction; from LDS every
// wavefront writes (or reads, adds and rewrites) whole rows of 256 values, 16 bytes per lane.
// LDS layout of a half tile: 128 rows x 1024 bytes, the 64-byte piece c of row r at position
// c ^ ((r / 4) % 4): the four lane groups, whose rows lie 4 apart, hit different banks.
template <bool KMajor>
__global__ void __launch_bounds__(TL::NT)
gemm_store_kernel(const char *__restrict__ A, int64_t lda_bytes, int64_t M, const char *__restrict__ B,
                  int64_t ldb_bytes, int64_t N, int KT, void *__restrict__ out, int64_t ldo, int out_dtype,
                  int accumulate, const int32_t *__restrict__ n_act, int64_t row_base, int limit,
                  const int32_t *__restrict__ row_map, int64_t a_blk, int64_t b_blk, int nsplit,
                  float *__restrict__ partials, int tail, const float *__restrict__ row_scale) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    constexpr int bpt = TL::BM / kBlockK;  // blocks per tile edge
    static_assert(TL::BM % kBlockK == 0 && TL::BN == TL::BM, "a tile of a blocked operand is a whole number of blocks");
    static_assert(TL::WGM == 2 && TL::BN * 4 * (TL::BM / 2) <= TL::LDS_BYTES, "half a tile of fp32 fits the operand stages");
    const int64_t tiles_n = ceil_div(N, TL::BN);
    int64_t m_end = M;
    if (n_act && limit == kLimitRows) m_end = active_rows(n_act, row_base, M);
    // kTailWhole: the launch of the whole rounds; kTailCut: the launch of the cut tiles (workgroup
    // i * parts + p takes part p of tile whole + i of the row-major order); both see the same cut
    const TailCut cut(tail == kTailNone ? 0 : ceil_div(m_end, TL::BM) * tiles_n);
    int64_t tm, tn;
    int part;
    if (tail == kTailCut) {
        if (blockIdx.x >= static_cast<unsigned>(cut.rem * cut.parts)) return;
        part = static_cast<int>(blockIdx.x % cut.parts);
        const int64_t t = cut.whole + blockIdx.x / cut.parts;
        tm = t / tiles_n;
        tn = t % tiles_n;
    } else {
        const TileOrder ord(ceil_div(M, TL::BM), tiles_n);
        const int64_t per_part = ord.blocks();
        part = static_cast<int>(blockIdx.x / per_part);
        if (!ord.tile(blockIdx.x % per_part, tm, tn)) return;
        if (tail == kTailWhole && tm * tiles_n + tn >= cut.whole) return;  // left to the launch of the cut tiles
    }
    const int64_t m0 = tm * TL::BM, n0 = tn * TL::BN;
    if (m0 >= m_end) return;
    if (n_act && limit == kLimitK) {
        const int64_t k_rows = active_rows(n_act, row_base, static_cast<int64_t>(KT) * kBK);
        KT = __builtin_amdgcn_readfirstlane(static_cast<int>(ceil_div(k_rows, TL::BN) * (TL::BN / kBK)));
        if (KT == 0 && accumulate && tail != kTailCut) return;  // nothing to add
    }
    int kt0 = 0;
    const int parts = tail == kTailCut ? cut.parts : nsplit;
    if (parts > 1) {  // this part's run of k-steps
        const int per = (KT + parts - 1) / parts;
        kt0 = part * per;
        KT = KT - kt0 < per ? KT - kt0 : per;
    }
    TL::Acc acc;
    TL::zero(acc);
    if (KT > 0) {
        if (KMajor) {
            const int64_t Mr = (M + 7) & ~int64_t(7), Nr = (N + 7) & ~int64_t(7);
            const char *Ak = A + kt0 * (kBK * lda_bytes), *Bk = B + kt0 * (kBK * ldb_bytes);  // rows are the contraction index
            TL::mainloop_kmajor(a_blk ? Ak + tm * bpt * a_blk : Ak, lda_bytes, a_blk ? 0 : m0, a_blk ? TL::BM : Mr,
                                b_blk ? Bk + tn * bpt * b_blk : Bk, ldb_bytes, b_blk ? 0 : n0, b_blk ? TL::BN : Nr, KT, lds,
                                acc, a_blk, b_blk);
        } else {
            // k-step kt of an operand starts blk bytes (blocked) or one stage of 128 bytes (row-major) further on
            const int64_t sa = a_blk ? a_blk : kBK * 2, sb = b_blk ? b_blk : kBK * 2;
            TL::mainloop(typename TL::Operands{A + kt0 * sa, lda_bytes, m0, M, B + kt0 * sb, ldb_bytes, n0, N, a_blk, b_blk},
                         KT, lds, acc);
        }
    }
    // where the tile goes: its place in the output, or (parts of a contraction) a plain fp32 tile
    int64_t om0 = m0, on0 = n0, oN = N;
    if (nsplit > 1) {  // partial results [part][M][N], no row map
        out = partials + static_cast<int64_t>(part) * M * N;
        ldo = N;
        out_dtype = SPO_FP32;
        accumulate = 0;
        row_map = nullptr;
    }
    if (tail == kTailCut) {  // partial results [part][tile - whole][BM][BN]
        out = partials + (static_cast<int64_t>(part) * cut.rem + (tm * tiles_n + tn - cut.whole)) * (TL::BM * TL::BN);
        ldo = TL::BN;
        out_dtype = SPO_FP32;
        accumulate = 0;
        row_map = nullptr;
        om0 = on0 = 0;
        oN = TL::BN;
        m_end = TL::BM;
    }
    int lane = threadIdx.x & 63;
    asm volatile("" : "+v"(lane));  // not to be traced: nothing derived from it is to live through the main loop
    const int grp = lane >> 4, col = lane & 15;
    // whole groups of four columns can move as 16 (fp32) or 8 (bf16) bytes when the rows allow it
    const bool vec = ldo % 4 == 0 && oN % 4 == 0 && reinterpret_cast<uintptr_t>(out) % 16 == 0;
    constexpr int HALF = TL::BM / 2, ROWS = HALF / TL::NWAVE;
    // adding to fp32 rows: the old values of a wavefront's rows are all requested before the half
    // tile is staged, so that their latency passes once per half tile and behind the staging
    const bool rmw = accumulate && out_dtype == SPO_FP32 && vec;
    const int64_t n = on0 + 4 * lane;  // this lane's four columns
    __syncthreads();  // the operand stages are no longer read
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
        const int64_t m_first = om0 + half * HALF + TL::wave_id() * ROWS;  // this wavefront's rows of the half tile
        float4 old[ROWS];
        if (rmw) {
#pragma unroll
            for (int i = 0; i < ROWS; ++i) {
                old[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                if (m_first + i < m_end && n < oN) {
                    const int64_t m = row_map ? row_map[m_first + i] : m_first + i;
                    old[i] = *reinterpret_cast<const float4 *>(static_cast<const float *>(out) + m * ldo + n);
                }
            }
        }
        if (TL::wave_m0() == half * HALF) {
#pragma unroll
            for (int fm = 0; fm < TL::FM; ++fm)
#pragma unroll
                for (int fn = 0; fn < TL::FN; ++fn)
#pragma unroll
                    for (int r = 0; r < TL::ACC_R; ++r) {
                        const int row = fm * TL::MI + 4 * grp + r;                  // (row / 4) % 4 == grp
                        const int piece = (TL::wave_n0() / TL::MI + fn) ^ grp;     // 64-byte piece of the row
                        *reinterpret_cast<float *>(lds + row * (TL::BN * 4) + piece * 64 + col * 4) = acc[fm][fn][r];
                    }
        }
        __syncthreads();
        if (rmw) {
#pragma unroll
            for (int i = 0; i < ROWS; ++i) {
                const int row = TL::wave_id() * ROWS + i;
                if (m_first + i >= m_end || n >= oN) continue;
                const int64_t m = row_map ? row_map[m_first + i] : m_first + i;
                const float4 v = *reinterpret_cast<const float4 *>(lds + row * (TL::BN * 4) +
                                                                   (((lane >> 2) ^ ((row >> 2) & 3)) << 6) + (lane & 3) * 16);
                *reinterpret_cast<float4 *>(static_cast<float *>(out) + m * ldo + n) =
                    make_float4(old[i].x + v.x, old[i].y + v.y, old[i].z + v.z, old[i].w + v.w);
            }
        } else {
#pragma unroll 4
            for (int i = 0; i < ROWS; ++i) {
                const int row = TL::wave_id() * ROWS + i;
                int64_t m = m_first + i;
                if (m >= m_end) break;  // rows are in order: nothing further down either
                const float sc = row_scale && nsplit == 1 ? row_scale[m] : 1.0f;  // (parts are scaled when they are added)
                if (row_map) m = row_map[m];
                float4 v = *reinterpret_cast<const float4 *>(lds + row * (TL::BN * 4) +
                                                             (((lane >> 2) ^ ((row >> 2) & 3)) << 6) + (lane & 3) * 16);
                v = make_float4(v.x * sc, v.y * sc, v.z * sc, v.w * sc);
                if (n >= oN) continue;
                if (out_dtype == SPO_FP32) {
                    float *o = static_cast<float *>(out) + m * ldo + n;
                    if (vec) {
                        *reinterpret_cast<float4 *>(o) = v;
                    } else {
                        const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (n + j < oN) o[j] = accumulate ? o[j] + e[j] : e[j];
                    }
                } else {
                    bf16_t *o = static_cast<bf16_t *>(out) + m * ldo + n;
                    if (vec) {
                        *reinterpret_cast<uint2 *>(o) = make_uint2(pack_bf16x2_rn(v.x, v.y), pack_bf16x2_rn(v.z, v.w));
                    } else {
                        const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (n + j < oN) o[j] = f32_to_bf16(e[j]);
                    }
                }
            }
        }
        __syncthreads();  // the half tile has been read: its space may be written again
    }
}

// out[row_map[m]][n] = row_scale[m] * sum over the parts (in order) of partials[part][m][n] for m
// below the number of active rows (n_act, row_map, row_scale may each be NULL: all M rows, in
// place, unscaled); four values per thread (N is a multiple of 4 here).
__global__ void __launch_bounds__(256)
reduce_split_kernel(const float *__restrict__ partials, int nsplit, int64_t M, int64_t N,
                    const int32_t *__restrict__ n_act, int64_t row_base, const int32_t *__restrict__ row_map,
                    void *__restrict__ out, int64_t ldo, int out_dtype, const float *__restrict__ row_scale) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t per_row = N / 4, m = i / per_row, n = (i % per_row) * 4;
    if (m >= (n_act ? active_rows(n_act, row_base, M) : M)) return;
    float4 s = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    for (int p = 0; p < nsplit; ++p) {
        const float4 v = *reinterpret_cast<const float4 *>(partials + (static_cast<int64_t>(p) * M + m) * N + n);
        s = make_float4(s.x + v.x, s.y + v.y, s.z + v.z, s.w + v.w);
    }
    if (row_scale) {
        const float sc = row_scale[m];
        s = make_float4(s.x * sc, s.y * sc, s.z * sc, s.w * sc);
    }
    const int64_t mo = row_map ? row_map[m] : m;
    if (out_dtype == SPO_FP32) {
        *reinterpret_cast<float4 *>(static_cast<float *>(out) + mo * ldo + n) = s;
    } else {
        *reinterpret_cast<uint2 *>(static_cast<bf16_t *>(out) + mo * ldo + n) =
            make_uint2(pack_bf16x2_rn(s.x, s.y), pack_bf16x2_rn(s.z, s.w));
    }
}

// The cut tiles of a launch's short last round (TailCut): out[row_map[m]][n] (=|+=) row_scale[m] times
// the sum, in order, of partials[part][tile - whole][m % BM][n % BN] over the parts.  The launch is
// sized for the most tiles a cut can have; n_act (with limit == kLimitRows), row_map and row_scale
// may be NULL.  Four values per thread.
__global__ void __launch_bounds__(256)
reduce_tail_kernel(const float *__restrict__ partials, int64_t M, int64_t N, const int32_t *__restrict__ n_act,
                   int64_t row_base, int limit, const int32_t *__restrict__ row_map, void *__restrict__ out, int64_t ldo,
                   int out_dtype, int accumulate, const float *__restrict__ row_scale) {
    constexpr int64_t per_tile = TL::BM * TL::BN / 4;
    const int64_t m_end = n_act && limit == kLimitRows ? active_rows(n_act, row_base, M) : M;
    const int64_t tiles_n = ceil_div(N, TL::BN);
    const TailCut cut(ceil_div(m_end, TL::BM) * tiles_n);
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t tl = i / per_tile, r = (i % per_tile) / (TL::BN / 4), c = (i % (TL::BN / 4)) * 4;
    if (tl >= cut.rem) return;
    const int64_t t = cut.whole + tl;
    const int64_t m = (t / tiles_n) * TL::BM + r, n = (t % tiles_n) * TL::BN + c;
    if (m >= m_end || n >= N) return;
    float4 sum = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    for (int p = 0; p < cut.parts; ++p) {
        const float4 v = *reinterpret_cast<const float4 *>(
            partials + ((static_cast<int64_t>(p) * cut.rem + tl) * TL::BM + r) * TL::BN + c);
        sum = make_float4(sum.x + v.x, sum.y + v.y, sum.z + v.z, sum.w + v.w);
    }
    if (row_scale) {
        const float sc = row_scale[m];
        sum = make_float4(sum.x * sc, sum.y * sc, sum.z * sc, sum.w * sc);
    }
    const int64_t mo = row_map ? row_map[m] : m;
    const float e[4] = {sum.x, sum.y, sum.z, sum.w};
    const bool vec = ldo % 4 == 0 && n + 3 < N && reinterpret_cast<uintptr_t>(out) % 16 == 0;
    if (out_dtype == SPO_FP32) {
        float *o = static_cast<float *>(out) + mo * ldo + n;
        if (vec) {
            float4 w = sum;
            if (accumulate) {
                const float4 old = *reinterpret_cast<const float4 *>(o);
                w = make_float4(old.x + sum.x, old.y + sum.y, old.z + sum.z, old.w + sum.w);
            }
            *reinterpret_cast<float4 *>(o) = w;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (n + j < N) o[j] = accumulate ? o[j] + e[j] : e[j];
        }
    } else {  // bf16 outputs are never added to
        bf16_t *o = static_cast<bf16_t *>(out) + mo * ldo + n;
        if (vec) {
            *reinterpret_cast<uint2 *>(o) = make_uint2(pack_bf16x2_rn(e[0], e[1]), pack_bf16x2_rn(e[2], e[3]));
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (n + j < N) o[j] = f32_to_bf16(e[j]);
        }
    }
}

// ----------------------------------------------------------------------------
// one-call forward + backward: logit gradients from the logits the forward stored
// ----------------------------------------------------------------------------
// dZ[j][v] = g * ([v == target] - exp(z[v] - lse)) for the active tokens j of a piece of the
// batch, from the fp16 offsets written by fwd_sweep_kernel<kEmitLogits> (z = stored value + offset of
// the entry's half tile), into the blocked bf16 layout the two contractions read.
// Row j of the output is token act_idx[j] of the piece; tok[j] is its record (see
// gather_chunk_kernel); rows from the number of active tokens up to the next multiple of 256
// are written as zeros, rows beyond are left alone (no contraction reads them).  A wavefront
// moves 8 rows x 128 bytes of one 64-entry block per step (16 bytes per lane), a workgroup 32
// rows, over `per_wg` consecutive blocks.
__global__ void __launch_bounds__(256)
dz_from_logits_kernel(const uint16_t *__restrict__ Z, int64_t z_blk, const float *__restrict__ offs, int64_t off_stride,
                      const int32_t *__restrict__ act_idx,
                      const int32_t *__restrict__ n_act, int64_t rows_cap, const float4 *__restrict__ tok,
                      bf16_t *__restrict__ dZ, int64_t dz_blk, int64_t n_blk, int per_wg) {
    const int64_t act = active_rows(n_act, 0, rows_cap);
    const int64_t j = static_cast<int64_t>(blockIdx.x) * 32 + (threadIdx.x >> 3);
    if (static_cast<int64_t>(blockIdx.x) * 32 >= (act + TL::BN - 1) / TL::BN * TL::BN) return;
    const int part = threadIdx.x & 7;  // which 8 of the block's 64 entries
    const bool live = j < act;
    const int64_t src = live ? act_idx[j] : 0;
    const float4 rec = live ? tok[j] : make_float4(0.0f, -INFINITY, __uint_as_float(0x7fffffffu), 0.0f);
    const uint32_t ts = __float_as_uint(rec.z);
    const uint32_t sgn = (ts & 0x80000000u) ? 0x80008000u : 0u;  // the values are formed as |g| * p; the sign of -g goes on in pairs
    const int64_t y = ts & 0x7fffffffu;
    constexpr int bph = TL::WM / kBlockK;  // blocks per wavefront's half of a tile: one offset each
    const int64_t b0 = static_cast<int64_t>(blockIdx.y) * per_wg;
    for (int64_t b = b0; b < b0 + per_wg && b < n_blk; ++b) {
        uint4 o = make_uint4(0u, 0u, 0u, 0u);
        if (live) {
            const float off = offs[(b / bph) * off_stride + src];
            const float c = fmaf(off, kLog2e, rec.y);  // log2|g| + (offset - lse) * log2(e)
            const uint4 zz = *reinterpret_cast<const uint4 *>(Z + b * z_blk + src * kBlockK + part * 8);
            const uint32_t w[4] = {zz.x, zz.y, zz.z, zz.w};
            float e[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                typedef _Float16 h2 __attribute__((ext_vector_type(2)));
                const h2 h = __builtin_bit_cast(h2, w[i]);
                e[2 * i] = __builtin_amdgcn_exp2f(fmaf(static_cast<float>(h.x), kLog2e, c));
                e[2 * i + 1] = __builtin_amdgcn_exp2f(fmaf(static_cast<float>(h.y), kLog2e, c));
            }
            const int64_t dy = y - (b * kBlockK + part * 8);
            if (dy >= 0 && dy < 8) {  // the one-hot term: |g| * (p - 1) before the sign goes on
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (dy == i) e[i] -= rec.x;
            }
            o = make_uint4(pack_bf16x2_rn(e[0], e[1]) ^ sgn, pack_bf16x2_rn(e[2], e[3]) ^ sgn,
                           pack_bf16x2_rn(e[4], e[5]) ^ sgn, pack_bf16x2_rn(e[6], e[7]) ^ sgn);
        }
        *reinterpret_cast<uint4 *>(dZ + b * dz_blk + j * kBlockK + part * 8) = o;
    }
}

// ----------------------------------------------------------------------------
// one-call forward + backward without a loss mask: the sweep stores what the contractions read
// ----------------------------------------------------------------------------
// The reference of token t is r_t = z_t[y_t] - old_logp_t: the log-sum-exp the token would have if
// the policy had not moved since the behaviour policy sampled it.  Both terms are known before
// the sweep (the logit of the sampled token costs one dot product).  Then
//   Q[t][v] = exp(z[t][v] - r_t) = softmax(z_t)[v] / ratio_t,   ratio_t = exp(logp_t - old_logp_t),
// lies near the probabilities whatever the logits' scale (bf16 keeps 8 bits of each entry), and
//   dZ[t][v] = g_t ([v == y_t] - softmax[v]) = c_t (Q[t][v] - [v == y_t] / ratio_t),  c_t = -g_t ratio_t.
// So once a piece's log-probs are known, one entry per token is rewritten (Q[t][y_t] = exp(old_logp_t)
// by construction, so the new value is formed afresh in fp32 and rounded once) and the contractions
// run on Q itself: dHidden_t = c_t (Q_t W), dW = Q^T (c X).  No pass over the stored tile is needed;
// the price is that rows of tokens without a gradient (c_t = 0) are multiplied like the others,
// which is why this form serves batches without a loss mask.

// ref2[t] = r_t * log2(e); 0 where the token has no valid target logit, where old_logp is not
// finite, and for the padding rows Tv <= t < Tzp (their stored rows stay finite and are multiplied by 0).
__global__ void __launch_bounds__(kTokThreads)
probs_reference_kernel(const float *__restrict__ z_target, const float *__restrict__ old_logp, int64_t Tv, int64_t Tzp,
                       float *__restrict__ ref2) {
    const int64_t t = static_cast<int64_t>(blockIdx.x) * kTokThreads + threadIdx.x;
    if (t >= Tzp) return;
    float r = 0.0f;
    if (t < Tv) {
        r = (z_target[t] - old_logp[t]) * kLog2e;
        if (!(fabsf(r) < 3.0e38f)) r = 0.0f;  // NaN or infinite
    }
    ref2[t] = r;
}

// c[t] = -g[t] * ratio_t (0 for tokens without a gradient and for the padding rows), and for the
// tokens with a gradient Q[t][y_t] = exp(old_logp_t) - 1 / ratio_t.
__global__ void __launch_bounds__(kTokThreads)
probs_patch_kernel(const float *__restrict__ g, const float *__restrict__ logp, const float *__restrict__ old_logp,
                   const int32_t *__restrict__ target, int64_t V, int64_t Tv, int64_t Tzp, uint16_t *__restrict__ Q,
                   int64_t q_blk, float *__restrict__ c) {
    const int64_t t = static_cast<int64_t>(blockIdx.x) * kTokThreads + threadIdx.x;
    if (t >= Tzp) return;
    float ct = 0.0f;
    if (t < Tv && g[t] != 0.0f) {
        const float ratio = expf(logp[t] - old_logp[t]);  // as in the surrogate: finite and positive where g != 0
        ct = -g[t] * ratio;
        const int64_t y = target[t];
        if (y >= 0 && y < V) Q[(y / kBlockK) * q_blk + t * kBlockK + y % kBlockK] = f32_to_bf16(expf(old_logp[t]) - 1.0f / ratio);
    }
    c[t] = ct;
}

// dst[t][:] = bf16(c[t] * src[t][:]) for t < rows_pad (c is 0 from the last valid row on: zeros).
// One workgroup per row; H is a multiple of 64.
template <typename T_>
__global__ void __launch_bounds__(256)
scale_rows_kernel(const T_ *__restrict__ src, const float *__restrict__ c, int64_t rows, int64_t H,
                  bf16_t *__restrict__ dst) {
    const int64_t t = blockIdx.x;
    const float ct = c[t];
    const bool live = t < rows && ct != 0.0f;
    uint2 *out = reinterpret_cast<uint2 *>(dst + t * H);
    for (int i = threadIdx.x; i < H / 4; i += 256) {
        float x[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if (live) {
            if constexpr (sizeof(T_) == 2) {
                const uint2 v = reinterpret_cast<const uint2 *>(src + t * H)[i];
                x[0] = __uint_as_float(v.x << 16); x[1] = __uint_as_float(v.x & 0xffff0000u);
                x[2] = __uint_as_float(v.y << 16); x[3] = __uint_as_float(v.y & 0xffff0000u);
            } else {
                const float4 v = reinterpret_cast<const float4 *>(src + t * H)[i];
                x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
            }
        }
        out[i] = make_uint2(pack_bf16x2_rn(x[0] * ct, x[1] * ct), pack_bf16x2_rn(x[2] * ct, x[3] * ct));
    }
}

// ----------------------------------------------------------------------------
// host side
// ----------------------------------------------------------------------------
// The kernels use more dynamic LDS than the default limit allows.  The attribute belongs
// to the current device's copy of the kernel, so it is set on every call (a host-side
// table lookup) rather than remembered in a process-wide flag.
static int set_lds_limit() {
    hipError_t e = hipSuccess;
    e = e ? e : hipFuncSetAttribute(reinterpret_cast<const void *>(fwd_sweep_kernel<kEmitNone>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kSweepLds);
    e = e ? e : hipFuncSetAttribute(reinterpret_cast<const void *>(fwd_sweep_kernel<kEmitLogits>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kSweepLds);
    e = e ? e : hipFuncSetAttribute(reinterpret_cast<const void *>(fwd_sweep_kernel<kEmitProbs>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kSweepLdsProbs);
    e = e ? e : hipFuncSetAttribute(reinterpret_cast<const void *>(recompute_dz_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, TL::LDS_BYTES);
    e = e ? e : hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_store_kernel<false>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, TL::LDS_BYTES);
    e = e ? e : hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_store_kernel<true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, TL::LDS_BYTES);
    return e == hipSuccess ? SPO_OK : SPO_EHIP;
}

static inline int64_t round_up(int64_t x, int64_t a) { return ceil_div(x, a) * a; }
static inline unsigned grid1(int64_t n, int per = 256) { return static_cast<unsigned>(ceil_div(n, per)); }

struct FwdPlan {
    int64_t nTt, nVt, T_pad, Kc;  // Kc: contraction length seen by the main loop
    int nsplit;
    int64_t nblk_tok;
    // workspace
    float *part_max, *part_sum, *z_target;
    FwdPartial *partials;
    bf16_t *Xs, *Ws, *Wvh;  // split-expanded operands (fp32), [V,H] copy (HV layout)
    float *W32;             // [V,H] copy of an fp32 head given as [H,V]
    size_t bytes;
};

static FwdPlan plan_fwd(const spo_pg_desc *d, void *ws) {
    FwdPlan p;
    p.nTt = ceil_div(d->T, TL::BN);
    p.nVt = ceil_div(d->V, TL::BM);
    p.T_pad = p.nTt * TL::BN;
    p.nsplit = SweepMap(p.nTt, p.nVt).nsplit;
    p.Kc = d->dtype == SPO_FP32 ? kSplitTerms * d->H : d->H;
    p.nblk_tok = ceil_div(std::max<int64_t>(d->T, 1), kTokThreads);
    Arena a(ws);
    p.part_max = a.take<float>(static_cast<size_t>(p.nsplit) * p.T_pad);
    p.part_sum = a.take<float>(static_cast<size_t>(p.nsplit) * p.T_pad);
    p.z_target = a.take<float>(p.T_pad);
    p.partials = a.take<FwdPartial>(p.nblk_tok);
    p.Xs = p.Ws = p.Wvh = nullptr;
    p.W32 = nullptr;
    if (d->dtype == SPO_FP32) {
        p.Xs = a.take<bf16_t>(static_cast<size_t>(std::max<int64_t>(d->T, 1)) * p.Kc);
        p.Ws = a.take<bf16_t>(static_cast<size_t>(d->V) * p.Kc);
        if (d->w_layout == SPO_W_HV) p.W32 = a.take<float>(static_cast<size_t>(d->V) * d->H);
    } else if (d->w_layout == SPO_W_HV) {
        p.Wvh = a.take<bf16_t>(static_cast<size_t>(d->V) * d->H);
    }
    p.bytes = a.used;
    return p;
}

static int check_fused(const spo_pg_desc *d) {
    if (reinterpret_cast<uintptr_t>(d->hidden) % 16 || reinterpret_cast<uintptr_t>(d->W) % 16) return SPO_EINVAL;
    return SPO_OK;
}

int fused_fwd_workspace(const spo_pg_desc *d, size_t *bytes) {
    *bytes = plan_fwd(d, nullptr).bytes;
    return SPO_OK;
}

int fused_fwd(const spo_pg_desc *d, float *loss, float *logp, float *lse, float *stats, void *ws,
              size_t ws_bytes, hipStream_t s) {
    int rc = check_fused(d);
    if (rc) return rc;
    const FwdPlan p = plan_fwd(d, ws);
    if (ws_bytes < p.bytes) return SPO_EWORKSPACE;
    if ((rc = set_lds_limit())) return rc;
    if (d->T > 0) {
        const char *X, *W;
        if (d->dtype == SPO_FP32) {
            split_expand_kernel<<<grid1(d->T * d->H), 256, 0, s>>>(static_cast<const float *>(d->hidden), d->T, d->H, p.Xs, 1);
            const float *w32 = static_cast<const float *>(d->W);
            if (d->w_layout == SPO_W_HV) {
                transpose_f32_kernel<<<dim3(grid1(d->H, 64), grid1(d->V, 64)), 256, 0, s>>>(w32, d->H, d->V, p.W32);
                w32 = p.W32;
            }
            split_expand_kernel<<<grid1(d->V * d->H), 256, 0, s>>>(w32, d->V, d->H, p.Ws, 0);
            X = reinterpret_cast<const char *>(p.Xs);
            W = reinterpret_cast<const char *>(p.Ws);
        } else {
            X = static_cast<const char *>(d->hidden);
            if (d->w_layout == SPO_W_HV) {
                transpose_to_bf16_kernel<bf16_t><<<dim3(grid1(d->H, 64), grid1(d->V, 64)), 256, 0, s>>>(
                    static_cast<const bf16_t *>(d->W), d->H, d->V, d->V, p.Wvh, d->H, d->V, d->H);
                W = reinterpret_cast<const char *>(p.Wvh);
            } else {
                W = static_cast<const char *>(d->W);
            }
        }
        const int64_t blocks = SweepMap(p.nTt, p.nVt).blocks();
        ScopedKernelTimer timer(kTimeFwdSweep, s);
        fwd_sweep_kernel<kEmitNone><<<static_cast<unsigned>(blocks), TL::NT, kSweepLds, s>>>(
            W, p.Kc * 2, d->V, X, p.Kc * 2, d->T, static_cast<int>(p.Kc / kBK), p.nsplit, p.nTt, p.nVt, p.T_pad,
            p.part_max, p.part_sum, nullptr, 0, nullptr);
    }
    if (d->T > 0) {
        if (d->dtype == SPO_FP32)
            target_logit_kernel<float><<<grid1(d->T, 4), 256, 0, s>>>(
                static_cast<const float *>(d->hidden), d->w_layout == SPO_W_HV ? p.W32 : static_cast<const float *>(d->W),
                d->H, d->V, d->T, d->target, p.z_target);
        else
            target_logit_kernel<bf16_t><<<grid1(d->T, 4), 256, 0, s>>>(
                static_cast<const bf16_t *>(d->hidden), d->w_layout == SPO_W_HV ? p.Wvh : static_cast<const bf16_t *>(d->W),
                d->H, d->V, d->T, d->target, p.z_target);
    }
    token_loss_kernel<<<static_cast<unsigned>(p.nblk_tok), kTokThreads, 0, s>>>(
        p.part_max, p.part_sum, p.nsplit, p.T_pad, p.z_target, d->T, d->old_logp, d->mask, d->adv_norm,
        d->cu_seqlens, d->B, d->eps_low, d->eps_high, logp, lse, p.partials);
    loss_finalize_kernel<<<1, kTokThreads, 0, s>>>(p.partials, p.nblk_tok, loss, stats);
    return launch_status();
}

struct BwdPlan {
    int64_t Tc, V_pad, V_blk, Kc, T_pad;  // V rounded up to a k-step (64) and to whole tiles (256)
    double *count;
    float *g, *dW_acc;
    bf16_t *WT, *Xb, *dZ, *Xs, *Ws, *Wvh;  // Xb: bf16 copy of the gathered rows of an fp32 hidden
    float *W32;  // [V,H] copy of an fp32 head given as [H,V]
    int32_t *act_idx, *n_act;  // active-token list, its length
    float4 *tok;               // per-chunk records (g, -lse*log2e, target) of the gathered rows
    int dx_split;              // parts the dHidden contraction is cut into (1: not split)
    float *dx_part;            // their fp32 partial results [dx_split][Tc][H]
    float *dw_tail;            // partial tiles of a contraction's short last round (see launch_gemm)
    void *Xc;
    size_t bytes;
};

static BwdPlan plan_bwd(const spo_pg_desc *d, int64_t chunk_tokens, void *ws, bool need_dw_acc) {
    BwdPlan p;
    const int64_t Tmax = round_up(std::max<int64_t>(d->T, 1), TL::BN);
    p.T_pad = Tmax;
    p.V_pad = round_up(d->V, kBK);
    p.V_blk = round_up(d->V, TL::BM);
    const int64_t tc = chunk_tokens > 0 ? round_up(chunk_tokens, TL::BN) : default_chunk_tokens(d->H, p.V_blk);
    p.Tc = std::min(tc, Tmax);
    p.Kc = d->dtype == SPO_FP32 ? kSplitTerms * d->H : d->H;
    Arena a(ws);
    p.count = a.take<double>(1);
    p.g = a.take<float>(p.T_pad);
    p.act_idx = a.take<int32_t>(p.T_pad);
    p.n_act = a.take<int32_t>(1);
    p.tok = a.take<float4>(p.Tc);
    // dHidden has (Tc / 256) * ceil(H / 256) tiles; below three quarters of the chip's compute
    // units the contraction over the vocabulary is cut into parts (H a multiple of 4 is given)
    const int64_t dx_tiles = (p.Tc / TL::BN) * ceil_div(d->H, TL::BM);
    p.dx_split = dx_tiles * 4 < kChipCUs * 3 ? static_cast<int>(std::min<int64_t>(8, kChipCUs / dx_tiles)) : 1;
    p.dx_part = p.dx_split > 1 ? a.take<float>(static_cast<size_t>(p.dx_split) * p.Tc * d->H) : nullptr;
    p.Xc = a.take<char>(static_cast<size_t>(p.Tc) * d->H * (d->dtype == SPO_FP32 ? 4 : 2));
    p.WT = a.take<bf16_t>(static_cast<size_t>(d->H) * p.V_blk);   // [V_blk / 64][H][64]
    p.dZ = a.take<bf16_t>(static_cast<size_t>(p.Tc) * p.V_blk);  // [V_blk / 64][rows of the chunk][64]
    p.Xb = p.Xs = p.Ws = p.Wvh = nullptr;
    p.dW_acc = nullptr;
    p.W32 = nullptr;
    if (d->dtype == SPO_FP32) {
        p.Xb = a.take<bf16_t>(static_cast<size_t>(p.Tc) * d->H);
        p.Xs = a.take<bf16_t>(static_cast<size_t>(p.Tc) * p.Kc);
        p.Ws = a.take<bf16_t>(static_cast<size_t>(d->V) * p.Kc);
        if (d->w_layout == SPO_W_HV) p.W32 = a.take<float>(static_cast<size_t>(d->V) * d->H);
    } else if (d->w_layout == SPO_W_HV) {
        p.Wvh = a.take<bf16_t>(static_cast<size_t>(d->V) * d->H);
    }
    if (need_dw_acc) p.dW_acc = a.take<float>(static_cast<size_t>(d->V) * d->H);
    p.dw_tail = a.take<float>(static_cast<size_t>(kTailTiles) * TL::BM * TL::BN);
    p.bytes = a.used;
    return p;
}

int fused_bwd_workspace(const spo_pg_desc *d, int64_t chunk_tokens, size_t *bytes) {
    // sized for the larger case (bf16 d_W needs an fp32 accumulator)
    *bytes = plan_bwd(d, chunk_tokens, nullptr, true).bytes;
    return SPO_OK;
}

template <typename SrcT>
static void launch_transpose(const SrcT *src, int64_t R, int64_t C, int64_t ld_src, bf16_t *dst, int64_t R_pad,
                             int64_t C_pad, int64_t ld_dst, hipStream_t s) {
    transpose_to_bf16_kernel<SrcT><<<dim3(grid1(R_pad, 64), grid1(C_pad, 64)), 256, 0, s>>>(src, R, C, ld_src, dst,
                                                                                         R_pad, C_pad, ld_dst);
}

// `tail`: room for kTailTiles fp32 tiles; with it a short last round of tiles is cut along the
// contraction (TailCut): 9504 tiles of dW on 256 units take 37 rounds and an eighth instead of 38,
// and a dHidden launch whose number of active rows leaves a round nearly empty loses a fifth of a
// round instead of a whole one.  Where the tile count depends on n_act the two extra launches
// are made in any case and find out on the device that there is nothing to cut.
template <bool KMajor>
static void launch_gemm(const bf16_t *A, int64_t lda, int64_t M, const bf16_t *B, int64_t ldb, int64_t N, int64_t K,
                        void *out, int64_t ldo, int out_dtype, int accumulate, const int32_t *n_act, int64_t row_base,
                        int limit, const int32_t *row_map, int64_t a_blk_elems, int64_t b_blk_elems, hipStream_t s,
                        int nsplit = 1, float *partials = nullptr, float *tail = nullptr,
                        const float *row_scale = nullptr) {
    const TileOrder ord(ceil_div(M, TL::BM), ceil_div(N, TL::BN));
    const bool rows_on_device = n_act && limit == kLimitRows;
    const bool cut = tail && nsplit == 1 && (rows_on_device ? ord.nM * ord.nN > kChipCUs : TailCut(ord.nM * ord.nN).rem > 0);
    gemm_store_kernel<KMajor><<<static_cast<unsigned>(ord.blocks() * nsplit), TL::NT, TL::LDS_BYTES, s>>>(
        reinterpret_cast<const char *>(A), lda * 2, M, reinterpret_cast<const char *>(B), ldb * 2, N,
        static_cast<int>(K / kBK), out, ldo, out_dtype, accumulate, n_act, row_base, limit, row_map, a_blk_elems * 2,
        b_blk_elems * 2, nsplit, partials, cut ? kTailWhole : kTailNone, row_scale);
    if (nsplit > 1)
        reduce_split_kernel<<<grid1(M * (N / 4)), 256, 0, s>>>(partials, nsplit, M, N, n_act, row_base, row_map, out, ldo,
                                                               out_dtype, row_scale);
    if (cut) {
        // sized for the most a cut can be: half of the units' worth of tiles, as many part-tiles as units
        gemm_store_kernel<KMajor><<<kChipCUs, TL::NT, TL::LDS_BYTES, s>>>(
            reinterpret_cast<const char *>(A), lda * 2, M, reinterpret_cast<const char *>(B), ldb * 2, N,
            static_cast<int>(K / kBK), out, ldo, out_dtype, accumulate, n_act, row_base, limit, row_map, a_blk_elems * 2,
            b_blk_elems * 2, 1, tail, kTailCut, nullptr);
        reduce_tail_kernel<<<grid1((kChipCUs / 2) * (TL::BM * TL::BN / 4)), 256, 0, s>>>(
            tail, M, N, n_act, row_base, limit, row_map, out, ldo, out_dtype, accumulate, row_scale);
    }
}

int fused_bwd(const spo_pg_desc *d, const float *logp, const float *lse, float grad_loss, void *d_hidden,
              int d_hidden_dtype, void *d_W, int d_W_dtype, int accumulate_dW, int64_t chunk_tokens, void *ws,
              size_t ws_bytes, hipStream_t s) {
    int rc = check_fused(d);
    if (rc) return rc;
    if (accumulate_dW && d_W && d_W_dtype != SPO_FP32) return SPO_EINVAL;
    const bool need_acc = d_W && d_W_dtype == SPO_BF16;
    const BwdPlan p = plan_bwd(d, chunk_tokens, ws, need_acc);
    if (ws_bytes < p.bytes) return SPO_EWORKSPACE;
    if ((rc = set_lds_limit())) return rc;
    const int64_t H = d->H, V = d->V, T = d->T;
    float *dW32 = need_acc ? p.dW_acc : static_cast<float *>(d_W);
    if (T == 0) {
        if (d_W && !accumulate_dW) {
            const int64_t words = d_W_dtype == SPO_FP32 ? V * H : V * H / 2;
            fill_zero_kernel<<<grid1(words), 256, 0, s>>>(static_cast<uint32_t *>(d_W), words);
        }
        return launch_status();
    }
    mask_count_kernel<<<1, 1024, 0, s>>>(d->mask, T, p.count);
    grad_scale_kernel<<<grid1(p.T_pad, kTokThreads), kTokThreads, 0, s>>>(
        logp, d->old_logp, d->mask, d->adv_norm, d->cu_seqlens, d->B, T, p.T_pad, d->eps_low, d->eps_high, grad_loss,
        p.count, p.g);
    // vocabulary-major head for the recompute, hidden-major head for dHidden
    const bf16_t *Wk;
    if (d->dtype == SPO_FP32) {
        const float *w32 = static_cast<const float *>(d->W);
        if (d->w_layout == SPO_W_HV) {
            transpose_f32_kernel<<<dim3(grid1(H, 64), grid1(V, 64)), 256, 0, s>>>(w32, H, V, p.W32);
            w32 = p.W32;
        }
        split_expand_kernel<<<grid1(V * H), 256, 0, s>>>(w32, V, H, p.Ws, 0);
        Wk = p.Ws;
        if (d_hidden) launch_transpose(w32, V, H, H, p.WT, p.V_blk, H, 0, s);
    } else {
        const bf16_t *Wvh = static_cast<const bf16_t *>(d->W);
        if (d->w_layout == SPO_W_HV) {
            launch_transpose(static_cast<const bf16_t *>(d->W), H, V, V, p.Wvh, H, V, H, s);
            Wvh = p.Wvh;
        }
        Wk = Wvh;
        if (d_hidden) launch_transpose(Wvh, V, H, H, p.WT, p.V_blk, H, 0, s);
    }
    // the tokens that carry a gradient, in order; the chunks below run over this list
    compact_active_kernel<<<1, 1024, 0, s>>>(p.g, T, p.act_idx, p.n_act);
    if (d_hidden) {  // rows of the other tokens stay zero
        const int64_t words = T * H / (d_hidden_dtype == SPO_FP32 ? 1 : 2);
        fill_zero_kernel<<<grid1(words), 256, 0, s>>>(static_cast<uint32_t *>(d_hidden), words);
    }
    const int64_t nVt = ceil_div(V, TL::BM);
    for (int64_t t0 = 0, c = 0; t0 < T; t0 += p.Tc, ++c) {
        // rows [t0, t0 + Tcp) of the compact order; how many of them exist is known on the
        // device only, so every launch is sized for the most there can be and trims itself
        const int64_t Tcp = round_up(std::min(p.Tc, T - t0), TL::BN);
        const bf16_t *Xk, *Xrows;  // operand of the recompute; the rows as plain bf16 (operand of dW)
        if (d->dtype == SPO_FP32) {
            float *xc = static_cast<float *>(p.Xc);
            gather_chunk_kernel<float><<<static_cast<unsigned>(Tcp), 256, 0, s>>>(
                static_cast<const float *>(d->hidden), H, p.act_idx, p.n_act, t0, Tcp, d->target, lse, p.g, xc,
                p.tok);
            split_expand_kernel<<<grid1(Tcp * H), 256, 0, s>>>(xc, Tcp, H, p.Xs, 1);
            Xk = p.Xs;
            if (d_W) f32_to_bf16_kernel<<<grid1(Tcp * H), 256, 0, s>>>(xc, p.Xb, Tcp * H);
            Xrows = p.Xb;
        } else {
            bf16_t *xc = static_cast<bf16_t *>(p.Xc);
            gather_chunk_kernel<bf16_t><<<static_cast<unsigned>(Tcp), 256, 0, s>>>(
                static_cast<const bf16_t *>(d->hidden), H, p.act_idx, p.n_act, t0, Tcp, d->target, lse, p.g, xc,
                p.tok);
            Xk = Xrows = xc;
        }
        {
            const SweepMap map(Tcp / TL::BN, nVt);
            const int64_t wgs = map.blocks();
            ScopedKernelTimer timer(kTimeRecompute, s);
            recompute_dz_kernel<<<static_cast<unsigned>(wgs), TL::NT, TL::LDS_BYTES, s>>>(
                reinterpret_cast<const char *>(Wk), p.Kc * 2, V, reinterpret_cast<const char *>(Xk), p.Kc * 2,
                Tcp, static_cast<int>(p.Kc / kBK), p.tok, nVt, Tcp / TL::BN, p.dZ, Tcp * kBlockK, p.n_act, t0);
        }
        if (d_hidden) {
            ScopedKernelTimer timer(kTimeDHidden, s);
            // both operands k-blocked over the vocabulary: a stage of a tile is 32 KiB contiguous
            launch_gemm<false>(p.dZ, kBlockK, Tcp, p.WT, kBlockK, H, p.V_pad, d_hidden, H, d_hidden_dtype, 0, p.n_act, t0,
                               kLimitRows, p.act_idx + t0, Tcp * kBlockK, H * kBlockK, s, p.dx_split, p.dx_part, p.dw_tail);
        }
        if (d_W) {
            const int acc = (c > 0 || accumulate_dW) ? 1 : 0;
            ScopedKernelTimer timer(kTimeDW, s);
            // contraction over the chunk's tokens, the row index of both dZ and the gathered hidden rows
            if (d->w_layout == SPO_W_VH)
                launch_gemm<true>(p.dZ, kBlockK, V, Xrows, H, H, Tcp, dW32, H, SPO_FP32, acc, p.n_act, t0, kLimitK, nullptr,
                                  Tcp * kBlockK, 0, s, 1, nullptr, p.dw_tail);
            else
                launch_gemm<true>(Xrows, H, H, p.dZ, kBlockK, V, Tcp, dW32, V, SPO_FP32, acc, p.n_act, t0, kLimitK, nullptr,
                                  0, Tcp * kBlockK, s, 1, nullptr, p.dw_tail);
        }
    }
    if (need_acc) f32_to_bf16_kernel<<<grid1(V * H), 256, 0, s>>>(p.dW_acc, static_cast<bf16_t *>(d_W), V * H);
    return launch_status();
}

// ----------------------------------------------------------------------------
// forward and backward in one call
// ----------------------------------------------------------------------------
// With the gradient of the total w.r.t. the loss known up front, nothing has to be formed
// twice: the batch is walked in pieces of Tz tokens; the forward sweep of a piece also stores
// its logits (fp16 offsets, 2 * V bytes per token), the piece's log-probs give the gradient
// factors, one pass turns the stored logits of the piece's active tokens into bf16 logit
// gradients, and the two contractions follow: three products of size T x V x H instead of four.
// By default a piece's stored logits stay within kDzBudgetBytes, and so do its gradients.
// Without a loss mask the pass over the stored logits is left out as well: the sweep stores
// bf16 scaled probabilities that the contractions read as they are (probs_reference_kernel).
struct FbPlan {
    int64_t Tz, T_pad, V_pad, V_blk, Kc, nVt, nblk_tok;
    int nsplit;
    double *count;
    float *g, *z_target, *part_max, *part_sum, *offs, *dW_acc, *W32, *dx_part, *dw_tail, *cscale;
    bool dense;  // no loss mask: the sweep stores what the contractions read (see probs_reference_kernel)
    FwdPartial *partials;
    int32_t *act_idx, *n_act;
    float4 *tok;
    uint16_t *Z;
    bf16_t *dZ, *WT, *Xb, *Xs, *Ws, *Wvh;
    void *Xc;
    int dx_split;
    size_t bytes;
};

static FbPlan plan_fb(const spo_pg_desc *d, int64_t chunk_tokens, void *ws, bool need_dw_acc, bool want_dx) {
    FbPlan p;
    p.T_pad = round_up(std::max<int64_t>(d->T, 1), TL::BN);
    p.V_pad = round_up(d->V, kBK);
    p.V_blk = round_up(d->V, TL::BM);
    p.nVt = p.V_blk / TL::BM;
    p.Kc = d->dtype == SPO_FP32 ? kSplitTerms * d->H : d->H;
    // tokens per piece: a multiple of 4096 (16 splits x 16 token tiles = one round of workgroups
    // of the sweep on 256 compute units) that keeps the stored logits within the budget, and the
    // logit gradients likewise
    int64_t tz = chunk_tokens > 0 ? round_up(chunk_tokens, TL::BN) : kDzBudgetBytes / (2 * p.V_blk) / 4096 * 4096;
    if (tz < TL::BN) tz = TL::BN;
    p.Tz = std::min(tz, p.T_pad);
    // Vocabulary splits of a piece's sweep: a launch lasts (rounds of workgroups on the chip) x
    // (tiles of the longest workgroup); among the multiples of 8 that fill the chip the count
    // with the shortest launch, else what the sweep chooses for small problems.
    p.nsplit = 0;
    const int64_t nTz = p.Tz / TL::BN;
    int64_t best = 0;
    for (int ns = kSweepSplits; ns <= 64 && ns <= p.nVt && nTz * kSweepSplits >= kChipCUs; ns += 8) {
        const int64_t cost = ceil_div(nTz * ns, kChipCUs) * ceil_div(p.nVt, ns);
        if (!p.nsplit || cost < best) {
            best = cost;
            p.nsplit = ns;
        }
    }
    p.nsplit = SweepMap(nTz, p.nVt, p.nsplit).nsplit;
    p.nblk_tok = p.T_pad / kTokThreads;
    static_assert(TL::BN % kTokThreads == 0, "pieces start at a block of the per-token kernels");
    Arena a(ws);
    p.count = a.take<double>(1);
    p.g = a.take<float>(p.T_pad);
    p.z_target = a.take<float>(p.T_pad);
    p.partials = a.take<FwdPartial>(p.nblk_tok);
    p.part_max = a.take<float>(static_cast<size_t>(p.nsplit) * p.Tz);
    p.part_sum = a.take<float>(static_cast<size_t>(p.nsplit) * p.Tz);
    p.dense = d->mask == nullptr;
    p.offs = a.take<float>(p.dense ? p.Tz : static_cast<size_t>(p.nVt) * TL::WGM * p.Tz);
    p.cscale = p.dense ? a.take<float>(p.Tz) : nullptr;
    p.act_idx = a.take<int32_t>(p.Tz);
    p.n_act = a.take<int32_t>(1);
    p.tok = a.take<float4>(p.Tz);
    const int64_t dx_tiles = (p.Tz / TL::BN) * ceil_div(d->H, TL::BM);
    p.dx_split = want_dx && dx_tiles * 4 < kChipCUs * 3 ? static_cast<int>(std::min<int64_t>(8, kChipCUs / dx_tiles)) : 1;
    p.dx_part = p.dx_split > 1 ? a.take<float>(static_cast<size_t>(p.dx_split) * p.Tz * d->H) : nullptr;
    p.Xc = a.take<char>(static_cast<size_t>(p.Tz) * d->H * (d->dtype == SPO_FP32 ? 4 : 2));
    p.WT = want_dx ? a.take<bf16_t>(static_cast<size_t>(d->H) * p.V_blk) : nullptr;
    p.Z = a.take<uint16_t>(static_cast<size_t>(p.Tz) * p.V_blk);
    p.dZ = p.dense ? nullptr : a.take<bf16_t>(static_cast<size_t>(p.Tz) * p.V_blk);
    p.Xb = p.Xs = p.Ws = p.Wvh = nullptr;
    p.dW_acc = p.W32 = nullptr;
    if (d->dtype == SPO_FP32) {
        p.Xb = a.take<bf16_t>(static_cast<size_t>(p.Tz) * d->H);
        p.Xs = a.take<bf16_t>(static_cast<size_t>(p.Tz) * p.Kc);
        p.Ws = a.take<bf16_t>(static_cast<size_t>(d->V) * p.Kc);
        if (d->w_layout == SPO_W_HV) p.W32 = a.take<float>(static_cast<size_t>(d->V) * d->H);
    } else if (d->w_layout == SPO_W_HV) {
        p.Wvh = a.take<bf16_t>(static_cast<size_t>(d->V) * d->H);
    }
    if (need_dw_acc) p.dW_acc = a.take<float>(static_cast<size_t>(d->V) * d->H);
    p.dw_tail = a.take<float>(static_cast<size_t>(kTailTiles) * TL::BM * TL::BN);
    p.bytes = a.used;
    return p;
}

int fused_fwd_bwd_workspace(const spo_pg_desc *d, int64_t chunk_tokens, size_t *bytes) {
    *bytes = plan_fb(d, chunk_tokens, nullptr, true, true).bytes;  // sized for the larger case
    return SPO_OK;
}

int fused_fwd_bwd(const spo_pg_desc *d, float grad_loss, float *loss, float *logp, float *lse, float *stats,
                  void *d_hidden, int d_hidden_dtype, void *d_W, int d_W_dtype, int accumulate_dW,
                  int64_t chunk_tokens, void *ws, size_t ws_bytes, hipStream_t s) {
    int rc = check_fused(d);
    if (rc) return rc;
    if (accumulate_dW && d_W && d_W_dtype != SPO_FP32) return SPO_EINVAL;
    const bool need_acc = d_W && d_W_dtype == SPO_BF16;
    const FbPlan p = plan_fb(d, chunk_tokens, ws, need_acc, d_hidden != nullptr);
    if (ws_bytes < p.bytes) return SPO_EWORKSPACE;
    if ((rc = set_lds_limit())) return rc;
    const int64_t H = d->H, V = d->V, T = d->T;
    float *dW32 = need_acc ? p.dW_acc : static_cast<float *>(d_W);
    if (T == 0) {
        if (d_W && !accumulate_dW) {
            const int64_t words = d_W_dtype == SPO_FP32 ? V * H : V * H / 2;
            fill_zero_kernel<<<grid1(words), 256, 0, s>>>(static_cast<uint32_t *>(d_W), words);
        }
        loss_finalize_kernel<<<1, kTokThreads, 0, s>>>(p.partials, 0, loss, stats);
        return launch_status();
    }
    mask_count_kernel<<<1, 1024, 0, s>>>(d->mask, T, p.count);
    // the head as the kernels read it: one row per vocabulary entry for the logits, one row per
    // hidden unit (blocked over the vocabulary) for dHidden
    const char *Wk;
    if (d->dtype == SPO_FP32) {
        const float *w32 = static_cast<const float *>(d->W);
        if (d->w_layout == SPO_W_HV) {
            transpose_f32_kernel<<<dim3(grid1(H, 64), grid1(V, 64)), 256, 0, s>>>(w32, H, V, p.W32);
            w32 = p.W32;
        }
        split_expand_kernel<<<grid1(V * H), 256, 0, s>>>(w32, V, H, p.Ws, 0);
        Wk = reinterpret_cast<const char *>(p.Ws);
        if (d_hidden) launch_transpose(w32, V, H, H, p.WT, p.V_blk, H, 0, s);
        target_logit_kernel<float><<<grid1(T, 4), 256, 0, s>>>(static_cast<const float *>(d->hidden), w32, H, V, T,
                                                               d->target, p.z_target);
    } else {
        const bf16_t *Wvh = static_cast<const bf16_t *>(d->W);
        if (d->w_layout == SPO_W_HV) {
            launch_transpose(static_cast<const bf16_t *>(d->W), H, V, V, p.Wvh, H, V, H, s);
            Wvh = p.Wvh;
        }
        Wk = reinterpret_cast<const char *>(Wvh);
        if (d_hidden) launch_transpose(Wvh, V, H, H, p.WT, p.V_blk, H, 0, s);
        target_logit_kernel<bf16_t><<<grid1(T, 4), 256, 0, s>>>(static_cast<const bf16_t *>(d->hidden), Wvh, H, V, T,
                                                                d->target, p.z_target);
    }
    if (d_hidden && !p.dense) {  // rows of tokens without a gradient stay zero (without a mask every row is written)
        const int64_t words = T * H / (d_hidden_dtype == SPO_FP32 ? 1 : 2);
        fill_zero_kernel<<<grid1(words), 256, 0, s>>>(static_cast<uint32_t *>(d_hidden), words);
    }
    const size_t x_elt = d->dtype == SPO_FP32 ? 4 : 2, dx_elt = d_hidden_dtype == SPO_FP32 ? 4 : 2;
    for (int64_t t0 = 0, c = 0; t0 < T; t0 += p.Tz, ++c) {
        const int64_t Tv = std::min(p.Tz, T - t0), Tzp = round_up(Tv, TL::BN);
        const char *Xpiece = static_cast<const char *>(d->hidden) + t0 * H * x_elt;
        const char *Xk = Xpiece;
        if (d->dtype == SPO_FP32) {
            split_expand_kernel<<<grid1(Tv * H), 256, 0, s>>>(reinterpret_cast<const float *>(Xpiece), Tv, H, p.Xs, 1);
            Xk = reinterpret_cast<const char *>(p.Xs);
        }
        const SweepMap map(Tzp / TL::BN, p.nVt, p.nsplit);
        if (p.dense) probs_reference_kernel<<<grid1(Tzp, kTokThreads), kTokThreads, 0, s>>>(p.z_target + t0, d->old_logp + t0, Tv, Tzp, p.offs);
        {
            ScopedKernelTimer timer(kTimeFwdSweep, s);
            if (p.dense)
                fwd_sweep_kernel<kEmitProbs><<<static_cast<unsigned>(map.blocks()), TL::NT, kSweepLdsProbs, s>>>(
                    Wk, p.Kc * 2, V, Xk, p.Kc * 2, Tv, static_cast<int>(p.Kc / kBK), map.nsplit, map.nTt, map.nVt, Tzp,
                    p.part_max, p.part_sum, p.Z, Tzp * kBlockK, p.offs);
            else
                fwd_sweep_kernel<kEmitLogits><<<static_cast<unsigned>(map.blocks()), TL::NT, kSweepLds, s>>>(
                    Wk, p.Kc * 2, V, Xk, p.Kc * 2, Tv, static_cast<int>(p.Kc / kBK), map.nsplit, map.nTt, map.nVt, Tzp,
                    p.part_max, p.part_sum, p.Z, Tzp * kBlockK, p.offs);
        }
        token_loss_kernel<<<grid1(Tv, kTokThreads), kTokThreads, 0, s>>>(
            p.part_max, p.part_sum, map.nsplit, Tzp, p.z_target + t0, Tv, d->old_logp + t0, d->mask ? d->mask + t0 : nullptr,
            d->adv_norm, d->cu_seqlens, d->B, d->eps_low, d->eps_high, logp + t0, lse + t0, p.partials + t0 / kTokThreads,
            t0);
        if (!d_hidden && !d_W) continue;
        grad_scale_kernel<<<grid1(Tzp, kTokThreads), kTokThreads, 0, s>>>(
            logp + t0, d->old_logp + t0, d->mask ? d->mask + t0 : nullptr, d->adv_norm, d->cu_seqlens, d->B, Tv, Tzp,
            d->eps_low, d->eps_high, grad_loss, p.count, p.g + t0, t0);
        if (p.dense) {
            // the contractions run on what the sweep stored: every row of the piece, scaled by c_t
            probs_patch_kernel<<<grid1(Tzp, kTokThreads), kTokThreads, 0, s>>>(
                p.g + t0, logp + t0, d->old_logp + t0, d->target + t0, V, Tv, Tzp, p.Z, Tzp * kBlockK, p.cscale);
            const bf16_t *Q = p.Z;
            if (d_hidden) {
                ScopedKernelTimer timer(kTimeDHidden, s);
                launch_gemm<false>(Q, kBlockK, Tv, p.WT, kBlockK, H, p.V_pad, static_cast<char *>(d_hidden) + t0 * H * dx_elt, H,
                                   d_hidden_dtype, 0, nullptr, 0, 0, nullptr, Tzp * kBlockK, H * kBlockK, s, p.dx_split,
                                   p.dx_part, p.dw_tail, p.cscale);
            }
            if (d_W) {
                bf16_t *Xc = d->dtype == SPO_FP32 ? p.Xb : static_cast<bf16_t *>(p.Xc);  // c_t x_t, the rows past the piece zero
                if (d->dtype == SPO_FP32)
                    scale_rows_kernel<float><<<static_cast<unsigned>(Tzp), 256, 0, s>>>(
                        reinterpret_cast<const float *>(Xpiece), p.cscale, Tv, H, Xc);
                else
                    scale_rows_kernel<bf16_t><<<static_cast<unsigned>(Tzp), 256, 0, s>>>(
                        reinterpret_cast<const bf16_t *>(Xpiece), p.cscale, Tv, H, Xc);
                const int acc = (c > 0 || accumulate_dW) ? 1 : 0;
                ScopedKernelTimer timer(kTimeDW, s);
                if (d->w_layout == SPO_W_VH)
                    launch_gemm<true>(Q, kBlockK, V, Xc, H, H, Tzp, dW32, H, SPO_FP32, acc, nullptr, 0, 0, nullptr,
                                      Tzp * kBlockK, 0, s, 1, nullptr, p.dw_tail);
                else
                    launch_gemm<true>(Xc, H, H, Q, kBlockK, V, Tzp, dW32, V, SPO_FP32, acc, nullptr, 0, 0, nullptr, 0,
                                      Tzp * kBlockK, s, 1, nullptr, p.dw_tail);
            }
            continue;
        }
        compact_active_kernel<<<1, 1024, 0, s>>>(p.g + t0, Tv, p.act_idx, p.n_act);
        const bf16_t *Xrows;
        if (d->dtype == SPO_FP32) {
            float *xc = static_cast<float *>(p.Xc);
            gather_chunk_kernel<float><<<static_cast<unsigned>(Tzp), 256, 0, s>>>(
                reinterpret_cast<const float *>(Xpiece), H, p.act_idx, p.n_act, 0, Tzp, d->target + t0, lse + t0, p.g + t0,
                xc, p.tok);
            if (d_W) f32_to_bf16_kernel<<<grid1(Tzp * H), 256, 0, s>>>(xc, p.Xb, Tzp * H);
            Xrows = p.Xb;
        } else {
            bf16_t *xc = static_cast<bf16_t *>(p.Xc);
            gather_chunk_kernel<bf16_t><<<static_cast<unsigned>(Tzp), 256, 0, s>>>(
                reinterpret_cast<const bf16_t *>(Xpiece), H, p.act_idx, p.n_act, 0, Tzp, d->target + t0, lse + t0,
                p.g + t0, xc, p.tok);
            Xrows = xc;
        }
        {
            constexpr int per_wg = 8;
            const int64_t n_blk = p.V_blk / kBlockK;
            ScopedKernelTimer timer(kTimeLogitsToDz, s);
            dz_from_logits_kernel<<<dim3(static_cast<unsigned>(Tzp / 32), grid1(n_blk, per_wg)), 256, 0, s>>>(
                p.Z, Tzp * kBlockK, p.offs, Tzp, p.act_idx, p.n_act, Tzp, p.tok, p.dZ,
                Tzp * kBlockK, n_blk, per_wg);
        }
        if (d_hidden) {
            ScopedKernelTimer timer(kTimeDHidden, s);
            launch_gemm<false>(p.dZ, kBlockK, Tzp, p.WT, kBlockK, H, p.V_pad, static_cast<char *>(d_hidden) + t0 * H * dx_elt, H,
                               d_hidden_dtype, 0, p.n_act, 0, kLimitRows, p.act_idx, Tzp * kBlockK, H * kBlockK, s,
                               p.dx_split, p.dx_part, p.dw_tail);
        }
        if (d_W) {
            const int acc = (c > 0 || accumulate_dW) ? 1 : 0;
            ScopedKernelTimer timer(kTimeDW, s);
            if (d->w_layout == SPO_W_VH)
                launch_gemm<true>(p.dZ, kBlockK, V, Xrows, H, H, Tzp, dW32, H, SPO_FP32, acc, p.n_act, 0, kLimitK, nullptr,
                                  Tzp * kBlockK, 0, s, 1, nullptr, p.dw_tail);
            else
                launch_gemm<true>(Xrows, H, H, p.dZ, kBlockK, V, Tzp, dW32, V, SPO_FP32, acc, p.n_act, 0, kLimitK, nullptr,
                                  0, Tzp * kBlockK, s, 1, nullptr, p.dw_tail);
        }
    }
    loss_finalize_kernel<<<1, kTokThreads, 0, s>>>(p.partials, ceil_div(T, kTokThreads), loss, stats);
    if (need_acc) f32_to_bf16_kernel<<<grid1(V * H), 256, 0, s>>>(p.dW_acc, static_cast<bf16_t *>(d_W), V * H);
    return launch_status();
}

}  // namespace spo
