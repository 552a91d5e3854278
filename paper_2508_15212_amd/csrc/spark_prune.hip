// Prefill-time channel pruning of the key cache for gfx950 (wave64).
//
// [Sec. "Problem Formulation and Analysis": saliency w = |q^j| * |k^j|, Eq. (7), Top_T;
//  Sec. "SparK": mean query over the observation window, mask and pruned keys;
//  App. "Caching Pruned Channel Statistics": mean saliency of the pruned set.]
//
// Kernels
//   spark_window_stat_kernel  a[b,h,j] = mean_g | mean_t Q_win[b,g,t,j] |  in float64, stored
//                             as float32 together with 1/a (G*128 threads per (b, h)).
//   spark_prune_kernel        one wavefront per tile (64 tokens of one KV head).  For each
//                             token the 128 saliencies sit two per lane (channels 2l, 2l+1);
//                             the T-th largest is found on the float32 bit pattern, most
//                             significant bits first: the top 13 bits by a counting pass over
//                             LDS bins that four rows share, the rest (for the rows that need
//                             it) by probes of two wave ballots and two scalar popcounts each.
//                             The kept set is then a pair of 64-bit ballots = the channel
//                             mask, and a prefix popcount (mbcnt) gives each kept value its
//                             slot in the packed row.  Rows are staged in LDS and written out
//                             with lane = token, coalesced, every 64, 32 or 16 rows.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "spark_kernels.h"
#include "spark_layout.h"
#include "spark_wave.h"

namespace spark {

// ---------------------------------------------------------------- window statistic

// grid = batch * Hkv blocks, min(G, 8) * 128 threads: thread (g, j) sums head g's window column j in
// float64 (t ascending), thread (0, j) then adds the G absolute means in g order -- the same order
// of operations as a plain loop nest.  Every sum of bf16 inputs this short is exact in float64, so
// the single rounding to float32 at the end decides a's bits.
__global__ __launch_bounds__(8 * SPARK_D) void spark_window_stat_kernel(const uint16_t *__restrict__ qwin,
                                                                     int Hq, int Hkv, int W,
                                                                     uint8_t *__restrict__ packed,
                                                                     SparkLayout L)
{
    __shared__ double absmean[16][SPARK_D];
    const int bh = blockIdx.x;
    const int b = bh / Hkv, h = bh % Hkv;
    const int j = threadIdx.x % SPARK_D, g0 = threadIdx.x / SPARK_D;
    const int G = Hq / Hkv, GT = blockDim.x / SPARK_D;      // GT = min(G, 8) head slots
    for (int g = g0; g < G; g += GT) {
        const uint16_t *src = qwin + ((int64_t)(b * Hq + h * G + g) * W) * SPARK_D + j;
        double qs = 0.0;
        int t = 0;
        for (; t + 8 <= W; t += 8) {          // eight loads in flight, added in order
            uint16_t x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = src[(int64_t)(t + u) * SPARK_D];
#pragma unroll
            for (int u = 0; u < 8; ++u) qs += (double)bf16_bits_to_float(x[u]);
        }
        for (; t < W; ++t) qs += (double)bf16_bits_to_float(src[(int64_t)t * SPARK_D]);
        absmean[g][j] = fabs(qs / (double)W);
    }
    __syncthreads();
    if (g0 != 0) return;
    double s = 0.0;
    for (int gg = 0; gg < G; ++gg) s += absmean[gg][j];
    const float a32 = (float)(s / (double)G);
    float *a_out = reinterpret_cast<float *>(packed + L.off_a);
    float *inva_out = reinterpret_cast<float *>(packed + L.off_inva);
    a_out[(int64_t)bh * SPARK_D + j] = a32;
    inva_out[(int64_t)bh * SPARK_D + j] = (a32 != 0.0f) ? (1.0f / a32) : 0.0f;
    if (bh == 0 && j < 64) {
        uint32_t *hdr = reinterpret_cast<uint32_t *>(packed);
        uint32_t v = 0;
        if (j == 0) v = SPARK_MAGIC;
        if (j == 1) v = (uint32_t)L.T;
        if (j == 2) v = (uint32_t)L.int8;
        if (j == 3) v = (uint32_t)L.batch;
        if (j == 4) v = (uint32_t)L.n_kv_heads;
        if (j == 5) v = (uint32_t)L.total_tokens;
        if (j == 6) v = (uint32_t)L.ndw;
        if (j == 8) v = (uint32_t)L.stats;      // (word 7 = 0: a key cache)
        hdr[j] = v;
    }
}

// ---------------------------------------------------------------- top-T selection + pack

#ifndef SPARK_PRUNE_WAVES
#define SPARK_PRUNE_WAVES 4
#endif
constexpr int kPruneWaves = SPARK_PRUNE_WAVES;      // wavefronts per block, one tile each
constexpr int kHistBins = 128;      // digit bins of the counting pass, one 32-bit word per bin: 16 that collect the
                                    // keys above the window, then 112 = 3.5 octaves x 32 digits
constexpr int kOverBins = 16;
constexpr int kHistWords = kHistBins + 64;  // per wavefront: the bins, then one spare word per lane
constexpr int kBatch = 4;           // rows whose counting passes share the bins (one byte of every word each)

typedef __attribute__((address_space(3))) uint32_t lds_u32;
// LDS byte address of a pointer into shared memory, and back
__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}
__device__ __forceinline__ lds_u32 *lds_word(uint32_t byte_address) { return (lds_u32 *)(uintptr_t)byte_address; }

// a * b + c with a, b taken as signed 24-bit numbers (one instruction; b is a small constant here)
template <int B>
__device__ __forceinline__ int mad_i24(int a, int c)
{
    int r;
    asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(r) : "v"(a), "n"(B), "s"(c));
    return r;
}
// lanes whose byte R of x is >= y (wave-uniform), as a wave mask (one instruction: the compare selects the byte itself)
template <int R>
__device__ __forceinline__ uint64_t ballot_byte_ge(uint32_t x, uint32_t y)
{
    uint64_t m;
    if constexpr (R == 0) asm("v_cmp_ge_u32_sdwa %0, %1, %2 src0_sel:BYTE_0 src1_sel:DWORD" : "=s"(m) : "v"(x), "s"(y));
    if constexpr (R == 1) asm("v_cmp_ge_u32_sdwa %0, %1, %2 src0_sel:BYTE_1 src1_sel:DWORD" : "=s"(m) : "v"(x), "s"(y));
    if constexpr (R == 2) asm("v_cmp_ge_u32_sdwa %0, %1, %2 src0_sel:BYTE_2 src1_sel:DWORD" : "=s"(m) : "v"(x), "s"(y));
    if constexpr (R == 3) asm("v_cmp_ge_u32_sdwa %0, %1, %2 src0_sel:BYTE_3 src1_sel:DWORD" : "=s"(m) : "v"(x), "s"(y));
    return m;
}
// x clamped to [lo, hi] (one instruction; lo <= hi)
__device__ __forceinline__ int clamp_i32(int x, int lo, int hi)
{
    int r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "v"(lo), "v"(hi));
    return r;
}

// The search below the digit, one bit per step from bit 17 down to bit LAST.  On entry at least T keys are >= p and
// c (> T) of them are counted; every step tries p with one more bit set and keeps it if T or more keys are still
// >= it.  Ends as soon as exactly T keys are >= p, or after bit LAST (then p is the T-th largest key and it is
// tied).  p, c and the bit live in scalar registers; a step is two vector compares, nine scalar instructions and
// two branches (written out because the compiler's version of the loop condition costs six scalar instructions
// more, and the scalar unit is what bounds this kernel).  Leaves in kb0 / kb1 the wave masks of the keys >= p
// (taken here, in the same block, so that this rarely run path shares no code with the usual one).
template <uint32_t LAST>
__device__ __forceinline__ void probe_bits(uint32_t k0, uint32_t k1, uint32_t Tv, uint32_t &p, uint32_t &c,
                                           uint64_t &kb0, uint64_t &kb1)
{
    uint32_t bit = 1u << 17, cand, n0, n1;
    uint64_t m1;
    asm volatile(
        "1:\n\t"
        "s_or_b32 %[cand], %[p], %[bit]\n\t"
        "v_cmp_le_u32_e32 vcc, %[cand], %[k0]\n\t"
        "v_cmp_le_u32_e64 %[m1], %[cand], %[k1]\n\t"
        "s_bcnt1_i32_b64 %[n0], vcc\n\t"
        "s_bcnt1_i32_b64 %[n1], %[m1]\n\t"
        "s_add_i32 %[n0], %[n0], %[n1]\n\t"
        "s_cmp_lt_u32 %[n0], %[T]\n\t"
        "s_cselect_b32 %[p], %[p], %[cand]\n\t"
        "s_cselect_b32 %[c], %[c], %[n0]\n\t"
        "s_cmp_eq_u32 %[c], %[T]\n\t"
        "s_cbranch_scc1 2f\n\t"
        "s_lshr_b32 %[bit], %[bit], 1\n\t"          // (sets the condition code to "result not zero")
        "s_cmp_ge_u32 %[bit], %[last]\n\t"
        "s_cbranch_scc1 1b\n\t"
        "2:\n\t"
        "v_cmp_le_u32_e64 %[kb0], %[p], %[k0]\n\t"
        "v_cmp_le_u32_e64 %[kb1], %[p], %[k1]"
        : [p] "+s"(p), [c] "+s"(c), [bit] "+s"(bit), [cand] "=&s"(cand), [n0] "=&s"(n0), [n1] "=&s"(n1), [m1] "=&s"(m1),
          [kb0] "=&s"(kb0), [kb1] "=&s"(kb1)
        : [k0] "v"(k0), [k1] "v"(k1), [T] "s"(Tv), [last] "n"(LAST)
        : "vcc", "scc");
}

// words per token in the LDS staging row: mask, mu, (scale), then T bf16 values
__host__ __device__ inline int spark_stage_words(const SparkLayout &L)
{
    int w = L.val0 + (L.T + 1) / 2;
    if (w < L.ndw) w = L.ndw;
    return (w + 1) & ~1;
}

// Rows a wavefront stages in LDS before it writes them out (a whole tile of 64, or 32, or 16): the largest that
// leaves room for at least five wavefronts per SIMD (20 per compute unit of 160 KB), since the search is a
// chain of dependent cross-lane steps that needs other wavefronts to fill its gaps.
__host__ inline int spark_prune_rows_per_flush(const SparkLayout &L)
{
    for (int rows = SPARK_TILE_TOKENS; rows > 16; rows /= 2)
        if ((size_t)rows * spark_stage_words(L) * 4 + kHistWords * 4 <= 7000) return rows;
    return 16;
}

__host__ inline size_t spark_prune_lds_bytes(const SparkLayout &L)
{
    return (size_t)kPruneWaves *
           ((size_t)spark_prune_rows_per_flush(L) * spark_stage_words(L) * 4 + kHistWords * 4);
}

// One searched row goes to its staging place.  kb0 / kb1: wave masks of the lanes whose first / second value is
// kept; pos0: number of kept values in front of this lane's first one; row_a: LDS byte address of the row's
// first value slot (wave-uniform).  The lane's kept values are stored to their slots (16 bits each), and the
// two masks are filed in the registers (em, om) of the lane named by the one-hot `lane_bit`.
// The stores run under the keep masks and the two 64-bit moves under `lane_bit`; the execution mask is set
// back to all lanes afterwards: the kernel has wave-uniform control flow only, every lane is active here.
#ifndef SPARK_PRUNE_STAGE_VARIANT
#define SPARK_PRUNE_STAGE_VARIANT 2
#endif
__device__ __forceinline__ void stage_row(int pos0, uint32_t xx, uint64_t kb0, uint64_t kb1, uint32_t row_a,
                                          uint64_t lane_bit, uint32_t dump_a, uint64_t &em, uint64_t &om)
{
#if SPARK_PRUNE_STAGE_VARIANT == 2
    uint32_t a0, a1;
    asm volatile(
        "v_addc_co_u32 %[a1], vcc, 0, %[pos], %[kb0]\n\t"      // slot of the second value: + 1 if the first is kept
        "v_lshl_add_u32 %[a0], %[pos], 1, %[row]\n\t"
        "v_lshl_add_u32 %[a1], %[a1], 1, %[row]\n\t"
        "s_mov_b64 exec, %[kb0]\n\t"
        "ds_write_b16 %[a0], %[x]\n\t"
        "s_mov_b64 exec, %[kb1]\n\t"
        "ds_write_b16_d16_hi %[a1], %[x]\n\t"
        "s_mov_b64 exec, %[bit]\n\t"
        "v_mov_b64 %[e], %[kb0]\n\t"
        "v_mov_b64 %[o], %[kb1]\n\t"
        "s_mov_b64 exec, -1"
        : [e] "+v"(em), [o] "+v"(om), [a0] "=&v"(a0), [a1] "=&v"(a1)
        : [kb0] "s"(kb0), [kb1] "s"(kb1), [bit] "s"(lane_bit), [pos] "v"(pos0), [row] "s"(row_a), [x] "v"(xx)
        : "memory", "vcc");
    (void)dump_a;
#else
    // every lane stores; a pruned value goes to the lane's spare word instead of masking lanes off
    const bool keep0 = __builtin_amdgcn_inverse_ballot_w64(kb0);
    const bool keep1 = __builtin_amdgcn_inverse_ballot_w64(kb1);
    const uint32_t a0 = row_a + 2u * (uint32_t)pos0, a1 = a0 + (keep0 ? 2u : 0u);
    typedef __attribute__((address_space(3))) uint16_t lds_u16;
    *(lds_u16 *)(uintptr_t)(keep0 ? a0 : dump_a) = (uint16_t)xx;
    *(lds_u16 *)(uintptr_t)(keep1 ? a1 : dump_a) = (uint16_t)(xx >> 16);
#if SPARK_PRUNE_STAGE_VARIANT == 1
    asm volatile(
        "s_mov_b64 exec, %[bit]\n\t"
        "v_mov_b64 %[e], %[kb0]\n\t"
        "v_mov_b64 %[o], %[kb1]\n\t"
        "s_mov_b64 exec, -1"
        : [e] "+v"(em), [o] "+v"(om)
        : [kb0] "s"(kb0), [kb1] "s"(kb1), [bit] "s"(lane_bit));
#else
    const int lane_id = __builtin_ctzll(lane_bit);
    uint32_t e_lo = (uint32_t)em, e_hi = (uint32_t)(em >> 32), o_lo = (uint32_t)om, o_hi = (uint32_t)(om >> 32);
    asm("s_mov_b32 m0, %8\n\t"
        "v_writelane_b32 %0, %4, m0\n\t"
        "v_writelane_b32 %1, %5, m0\n\t"
        "v_writelane_b32 %2, %6, m0\n\t"
        "v_writelane_b32 %3, %7, m0"
        : "+v"(e_lo), "+v"(e_hi), "+v"(o_lo), "+v"(o_hi)
        : "s"((uint32_t)kb0), "s"((uint32_t)(kb0 >> 32)), "s"((uint32_t)kb1), "s"((uint32_t)(kb1 >> 32)), "s"(lane_id)
        : "m0");
    em = ((uint64_t)e_hi << 32) | e_lo;
    om = ((uint64_t)o_hi << 32) | o_lo;
#endif
#endif
}

// Pairwise step of a transposing reduction.  A and B hold one partial per lane for two tokens;
// the result holds A[l] + A[partner(l)] in the lanes where `hi` is false and B[l] + B[partner(l)]
// where it is true.  CTRL is a data-parallel-primitive pattern whose partner differs in exactly the
// lane bit that `hi` tests (and in no lower bit).  Four such steps fold 16 tokens x 64 lanes into
// one register with token (l & 15) summed over the 16 lanes of l's row.
template <int CTRL>
__device__ __forceinline__ float fold_pair(float A, float B, bool hi)
{
    const float stay = hi ? B : A, go = hi ? A : B;
    return stay + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(go), CTRL, 0xF, 0xF, true));
}
// The same step across the halves of the wavefront and across neighbouring rows of 16 lanes, where this chip's
// lane-swap instructions do the selecting for free (two instructions a step instead of three):
// fold_halves gives A[l] + A[l + 32] in lanes 0..31 and B[l - 32] + B[l] in lanes 32..63,
// fold_rows   gives A[l] + A[l ^ 16] in rows 0 and 2 and B[l ^ 16] + B[l] in rows 1 and 3.
__device__ __forceinline__ float fold_halves(float A, float B)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(A), __float_as_uint(B), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float fold_rows(float A, float B)
{
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(A), __float_as_uint(B), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// Four levels of these steps (halves, rows, row rotate by 4, row rotate by 8) and a sum over the lanes of every quad
// fold 16 tokens x 64 lanes into one register: token t of the sixteen (bits t0..t3) ends up in the four lanes
// 32 t0 + 16 t1 + 4 t2 + 8 t3 + {0, 1, 2, 3}.
__device__ __forceinline__ float quad_sum(float x)
{
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
    return x;
}

// One tile by one wavefront.  FULL: wavefront number wt (over tiles, then heads) of those that take the tiles which
// hold all 64 tokens (the first total_tokens / 64 of every head); otherwise wt = the KV head whose partly filled
// last tile this wavefront takes.  Two instantiations, so that the hot one carries no bounds logic.
// MODE: bit 0 = int8 codes + scale instead of bf16 kept entries; bit 1 = the rows also carry the all-channel mean
// and standard deviation of the row's saliencies (App. "Caching Pruned Channel Statistics", for the sampled recovery).
// VALUES: the rows are value-cache rows (App. "Pruning Value Cache Channels"): the score of a channel is
// |v| itself, there is no channel weight, no sequence bookkeeping and no statistic of the pruned set.
#ifndef SPARK_PRUNE_MIN_WAVES
#define SPARK_PRUNE_MIN_WAVES (MODE >= 2 ? 6 : 7)
#endif
template <int MODE, bool FULL, bool VALUES>
__device__ __forceinline__ void prune_tile(const uint16_t *__restrict__ k, int64_t k_tok_stride, int64_t k_head_stride,
                                           const int32_t *__restrict__ cu, uint8_t *__restrict__ packed,
                                           const SparkLayout &L, const int rows_per_flush, const int wave, const int64_t wt)
{
    constexpr bool INT8 = (MODE & 1) != 0, STATS = (MODE & 2) != 0;
    extern __shared__ __align__(16) uint8_t smem[];
    const int lane = threadIdx.x & 63;
    const int64_t full_tiles = L.total_tokens / SPARK_TILE_TOKENS;
    if (wt >= (FULL ? full_tiles : 1) * L.n_kv_heads) return;   // whole wavefront leaves; no block barrier is used
    if (VALUES && wt == 0 && (FULL || full_tiles == 0)) {
        // header of a value cache (the key cache's is written with the channel weights): first wavefront of
        // whichever launch comes first
        uint32_t v = 0;
        if (lane == 0) v = SPARK_MAGIC;
        if (lane == 1) v = (uint32_t)L.T;
        if (lane == 4) v = (uint32_t)L.n_kv_heads;
        if (lane == 5) v = (uint32_t)L.total_tokens;
        if (lane == 6) v = (uint32_t)L.ndw;
        if (lane == 7) v = 1u;   // value cache
        reinterpret_cast<uint32_t *>(packed)[lane] = v;
    }
    const int h = FULL ? (int)(wt / full_tiles) : (int)wt;
    const int64_t tile = FULL ? wt % full_tiles : full_tiles;
    const int T = L.T;
    const int B = L.batch;
    const int sw = spark_stage_words(L);
    uint32_t *stage = reinterpret_cast<uint32_t *>(smem) +
                      (size_t)wave * (rows_per_flush * sw + kHistWords);
    uint32_t *hist = stage + rows_per_flush * sw;        // [0, 128) bins, [128, 192) spare
    uint16_t *stage16 = reinterpret_cast<uint16_t *>(stage);

    const float2 *a_all = reinterpret_cast<const float2 *>(packed + L.off_a);
    const int64_t n0 = tile * SPARK_TILE_TOKENS;
    const int nvalid = FULL ? SPARK_TILE_TOKENS : (int)(L.total_tokens - n0);

    // sequence of the first token: largest b with cu[b] <= n0 (skips empty sequences)
    int b = 0;
    int seq_end_t = 0x7FFFFFFF;   // token index within the tile where the current sequence ends
    // lane l owns channels 2l (low half of its 32-bit load) and 2l+1 (high half)
    float2 a01 = make_float2(1.0f, 1.0f);
    if constexpr (!VALUES) {
        int lo = 0, hi = B;     // invariant: cu[lo] <= n0 < cu[hi]
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (cu[mid] <= n0) lo = mid; else hi = mid;
        }
        b = lo;
        seq_end_t = (int)((int64_t)cu[b + 1] - n0);   // total < 2^31
        a01 = a_all[((int64_t)b * L.n_kv_heads + h) * (SPARK_D / 2) + lane];
    }

    // Row addresses: a wave-uniform base (scalar registers) plus one 32-bit per-lane offset per row of
    // a block of PF rows, set up once; a block's eight loads then cost no address arithmetic.
    constexpr int PF = 8;
    const char *kbase = reinterpret_cast<const char *>(k + n0 * k_tok_stride + (int64_t)h * k_head_stride);
    const uint32_t stride_b = (uint32_t)k_tok_stride * 2u;   // bytes per token row (the host checks the range)
    uint32_t voff[PF];
#pragma unroll
    for (int u = 0; u < PF; ++u) voff[u] = (uint32_t)lane * 4u + (uint32_t)u * stride_b;
    // rows tb0 .. tb0+PF-1 of the tile into x; in a partly filled tile rows past the last token repeat
    // the last one
    auto load_block = [&](uint32_t (&x)[PF], int tb0) __attribute__((always_inline)) {
        if constexpr (FULL) {
            const char *sb = kbase + (size_t)((uint32_t)tb0 * stride_b);
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                asm volatile("" : "+v"(voff[u]));   // keeps the 32-bit offset next to its load (scalar base + offset form)
                x[u] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(sb + voff[u]));
            }
        } else {
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                const int tt = (tb0 + u < nvalid) ? (tb0 + u) : (nvalid - 1);
                const char *sb = kbase + (size_t)((uint32_t)tt * stride_b);
                asm volatile("" : "+v"(voff[0]));
                x[u] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(sb + voff[0]));
            }
        }
    };

    // lane t collects, for token t, the ballots of kept even channels (em) and kept odd channels (om)
    uint64_t em = 0, om = 0;
    uint64_t tok_bit = 1;                                   // one-hot: the lane of the row being searched
    float mureg = 0.0f;                                     // sums of pruned saliencies: token t in lane
                                                            // 32 t0 + 16 t1 + 4 t2 + 8 t3 + (t >> 4)
    uint32_t muall = 0;                                     // lane t: mean saliency over all channels (bits)
    float sqreg = 0.0f;                                     // sums of squared deviations from it, same places

    // Rows are fetched a block ahead: while one block of PF rows is searched the next is in flight,
    // in two register sets that swap roles.
    uint32_t xa[PF], xb[PF];
    load_block(xa, 0);

    // T-th largest key of a row.  The search is most-significant-bit first on the float32 bit pattern:
    // keep a prefix p such that at least T keys are >= p and extend it until exactly T keys are >= p (or all
    // 31 bits are fixed: a tie at the cut).  A probe of one candidate is two wave ballots and two scalar
    // popcounts.  The top 13 bits (exponent and five mantissa bits = the DIGIT of a key) are settled by one
    // counting pass: a window of 112 digits (3.5 octaves) is centred on the digit found for the row before
    // (rows of one head rarely differ by more than an octave or two); every lane adds its
    // two keys' digits to LDS bins, highest digit first, keys above the window into sixteen bins in front of
    // it (spread by lane) and keys below it into a per-lane spare word, so no lane is masked off and nothing
    // piles up on one address.  Lane l reads bins l and 64 + l, wave prefix sums turn them into "keys with
    // digit >= the bin's", and one ballot per row finds the bin where the count reaches T.  Four rows share a
    // pass: row r counts in byte r of every bin (a bin holds at most 128 keys), so zeroing, reading and the
    // prefix sums are paid once per four rows.  A row whose T-th key lies outside the window repeats the pass
    // alone with the window moved; its exponent is found by bisection if that fails as well.
    int D;    // digit (exponent and five mantissa bits) of the T-th key of the row before
    {   // first row: the exponent by bisection over the 256 exponents
        const uint32_t xx = xa[0];
        const uint32_t key0 = __float_as_uint(__fmul_rn(a01.x, fabsf(__uint_as_float(xx << 16))));
        const uint32_t key1 = __float_as_uint(__fmul_rn(a01.y, fabsf(__uint_as_float(xx & 0xFFFF0000u))));
        int lo = 0, hi = 256;   // at least T keys are >= lo << 23, fewer are >= hi << 23
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            const uint32_t x = (uint32_t)mid << 23;
            const int c = __popcll(__ballot(key0 >= x)) + __popcll(__ballot(key1 >= x));
            if (c >= T) lo = mid; else hi = mid;
        }
        D = (lo << 5) + 16;
    }
    const uint32_t bins_a = lds_address(hist);                                   // byte address of bin 0 (wave-uniform)
    const int lo_clamp = (int)(bins_a + 4u * (lane & (kOverBins - 1)));          // where a key far above the window counts
    const int hi_clamp = (int)(bins_a + 4u * kHistBins + 4u * lane);             // this lane's spare word, past the bins
    lds_u32 *const my_bin = lds_word(bins_a + 4u * lane);                        // bins l and 64 + l
    const uint32_t dump_a = lds_address(hist + kHistBins + lane);     // where pruned values go
    const uint32_t row_a0 = lds_address(stage16 + L.val0 * 2);
    uint32_t row_a = row_a0;                                          // LDS byte address of the current row's first value slot
    const uint32_t row_step = (uint32_t)sw * 4u;
    const uint32_t Tv = (uint32_t)T;

    // One counting pass.  key0 / key1 [NR]: the rows' keys; topd: digit of bin kOverBins (the window's highest).
    // Leaves in (sA, sB) the counts of keys with digit >= the digit of bins l and 64 + l, row r in byte r.
    auto count_pass = [&](auto nr_tag, const uint32_t *k0, const uint32_t *k1, const int topd, uint32_t &sA,
                          uint32_t &sB) __attribute__((always_inline)) {
        constexpr int NR = decltype(nr_tag)::value;
        my_bin[0] = 0u;
        my_bin[64] = 0u;
        prune_lds_sync();
        // byte address of the bin of digit d: bins_a + 4 * (kOverBins + topd - d)
        const int top_a = (int)bins_a + 4 * (kOverBins + topd);
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            const int a0 = clamp_i32(mad_i24<-4>((int)(k0[r] >> 18), top_a), lo_clamp, hi_clamp);
            const int a1 = clamp_i32(mad_i24<-4>((int)(k1[r] >> 18), top_a), lo_clamp, hi_clamp);
            __hip_atomic_fetch_add(lds_word((uint32_t)a0), 1u << (8 * r), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
            __hip_atomic_fetch_add(lds_word((uint32_t)a1), 1u << (8 * r), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
        }
        prune_lds_sync();
        const uint32_t hA = my_bin[0], hB = my_bin[64];
        prune_lds_sync();
        sA = wave_inclusive_sum(hA);
        sB = wave_inclusive_sum(hB) + (uint32_t)__builtin_amdgcn_readlane((int)sA, 63);   // (bytes cannot carry: <= 128 keys)
    };
    // Where row R's count reaches T.  Returns the 13-bit prefix of the T-th key, shifted to its place (topS = the
    // window's highest digit plus kOverBins, shifted likewise), and in cnt the number of keys >= that prefix;
    // sets bit R of miss_up if T or more keys lie above the window, of miss_down if fewer than T keys lie in or
    // above it.  (The usual case, a crossing in the lower 64 bins, is six scalar instructions.)
    auto crossing = [&](auto r_tag, const uint32_t sA, const uint32_t sB, const uint32_t topS, const uint32_t topS_low,
                        int &cnt, uint32_t &miss_up, uint32_t &miss_down) __attribute__((always_inline)) -> uint32_t {
        constexpr int R = decltype(r_tag)::value;
        const uint64_t rA = ballot_byte_ge<R>(sA, Tv);
        if (rA != 0) {
            const int l = __builtin_ctzll(rA);
            cnt = (int)(((uint32_t)__builtin_amdgcn_readlane((int)sA, l) >> (8 * R)) & 0xFFu);
            if (__builtin_expect(l < kOverBins, 0)) miss_up |= 1u << R;
            return topS - ((uint32_t)l << 18);
        }
        const uint64_t rB = ballot_byte_ge<R>(sB, Tv);
        if (__builtin_expect(rB == 0, 0)) {
            miss_down |= 1u << R;
            return 0u;
        }
        const int l = __builtin_ctzll(rB);
        cnt = (int)(((uint32_t)__builtin_amdgcn_readlane((int)sB, l) >> (8 * R)) & 0xFFu);
        return topS_low - ((uint32_t)l << 18);
    };

    // searches and stages rows u0 .. u0+3 of the block held in x (tokens tb+u0 ..); leaves their pruned-saliency
    // partials in ps (and, with statistics, the squared deviations in qs)
    auto do_batch = [&](const uint32_t (&x)[PF], const int u0, const int tb, float (&ps)[PF],
                        float (&qs)[PF]) __attribute__((always_inline)) {
        uint32_t key0[kBatch], key1[kBatch];
        // ---- saliency: one float32 multiply, never fused
        auto first_stage = [&](const int r, const bool may_cross) __attribute__((always_inline)) {
            const int t = tb + u0 + r;
            const uint32_t xx = x[u0 + r];
            if (!VALUES && may_cross && t >= seq_end_t) {    // the tile crosses into the next non-empty sequence
                if (t < nvalid) {
                    do {
                        ++b;
                        seq_end_t = (int)((int64_t)cu[b + 1] - n0);
                    } while (t >= seq_end_t);
                    a01 = a_all[((int64_t)b * L.n_kv_heads + h) * (SPARK_D / 2) + lane];
                    // finish this load here, inside the rare branch: otherwise the wait for it
                    // lands after the join and drains the prefetched K rows on every token
                    __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
                }
            }
            key0[r] = __float_as_uint(__fmul_rn(a01.x, fabsf(__uint_as_float(xx << 16))));
            key1[r] = __float_as_uint(__fmul_rn(a01.y, fabsf(__uint_as_float(xx & 0xFFFF0000u))));
        };
        if (!VALUES && __builtin_expect(tb + u0 + kBatch - 1 >= seq_end_t, 0)) {
#pragma unroll
            for (int r = 0; r < kBatch; ++r) first_stage(r, true);
        } else {
#pragma unroll
            for (int r = 0; r < kBatch; ++r) first_stage(r, false);
        }
        // ---- counting pass: exponent and five mantissa bits, four rows at once
        uint32_t pfx[kBatch];
        int geq[kBatch];
        uint32_t miss_up = 0, miss_down = 0;
        const int topd = D + 56;                  // the window's highest digit: the window is centred on D
        {
            uint32_t sA, sB;
            count_pass(std::integral_constant<int, kBatch>{}, key0, key1, topd, sA, sB);
            const uint32_t topS = (uint32_t)(topd + kOverBins) << 18;
            uint32_t topS_low = topS - (64u << 18);     // the same for the lower 64 bins
            asm volatile("" : "+s"(topS_low));          // (kept as a value of its own: one subtraction per row less)
            auto locate = [&](auto r_tag) __attribute__((always_inline)) {
                constexpr int R = decltype(r_tag)::value;
                int cnt = 0;
                pfx[R] = crossing(r_tag, sA, sB, topS, topS_low, cnt, miss_up, miss_down);
                geq[R] = cnt;
            };
            locate(std::integral_constant<int, 0>{});
            locate(std::integral_constant<int, 1>{});
            locate(std::integral_constant<int, 2>{});
            locate(std::integral_constant<int, 3>{});
        }
        // rows whose T-th key lies outside the window: one at a time, window moved by three octaves; if that is
        // not enough either, the exponent by bisection (a window whose top octave is that one cannot miss)
        uint32_t miss = miss_up | miss_down;
        while (__builtin_expect(miss != 0, 0)) {
            const int r = __builtin_ctz(miss);
            miss &= miss - 1;
            // (values, not references, are selected: the four rows' registers stay registers)
            auto pick = [&](auto v0, auto v1, auto v2, auto v3) { return r == 0 ? v0 : (r == 1 ? v1 : (r == 2 ? v2 : v3)); };
            const uint32_t k0[1] = {pick(key0[0], key0[1], key0[2], key0[3])};
            const uint32_t k1[1] = {pick(key1[0], key1[1], key1[2], key1[3])};
            int td = topd + (((miss_up >> r) & 1u) ? 96 : -96);
            uint32_t P = 0;
            int GE = 0;
            for (int round = 0;; ++round) {
                uint32_t sA, sB;
                count_pass(std::integral_constant<int, 1>{}, k0, k1, td, sA, sB);
                int cnt = 0;
                uint32_t up = 0, down = 0;
                const uint32_t pre = crossing(std::integral_constant<int, 0>{}, sA, sB, (uint32_t)(td + kOverBins) << 18,
                                              (uint32_t)(td + kOverBins - 64) << 18, cnt, up, down);
                if ((up | down) == 0) {
                    GE = cnt;
                    P = pre;
                    break;
                }
                if (round == 2) {   // cannot happen for keys below 2^31 (finite input); never spin
                    GE = T;
                    P = 0x7F800000u;
                    break;
                }
                int lo = 0, hi = 256;   // at least T keys are >= lo << 23, fewer are >= hi << 23
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    const uint32_t v = (uint32_t)mid << 23;
                    const int c = __popcll(__ballot(k0[0] >= v)) + __popcll(__ballot(k1[0] >= v));
                    if (c >= T) lo = mid; else hi = mid;
                }
                td = ((lo + 1) << 5) - 1;     // the T-th key has exponent lo: the window's first octave
            }
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                pfx[i] = (r == i) ? P : pfx[i];
                geq[i] = (r == i) ? GE : geq[i];
            }
        }
        D = (int)(pfx[kBatch - 1] >> 18);
        // ---- the rest of each row
#pragma unroll
        for (int r = 0; r < kBatch; ++r) {
            const int u = u0 + r, t = tb + u;
            const uint32_t xx = x[u];
            const uint32_t k0 = key0[r], k1 = key1[r];
            const float w0 = __uint_as_float(k0), w1 = __uint_as_float(k1);
            uint32_t p = (uint32_t)__builtin_amdgcn_readfirstlane((int)pfx[r]);
            uint32_t c = (uint32_t)__builtin_amdgcn_readfirstlane(geq[r]);      // keys >= p (at least T)
            // the usual case first: the digit's bin ends exactly at T keys (taken unconditionally: a plain
            // if-then compiles to one compare and one branch, an if-else here does not)
            uint64_t kb0 = __ballot(k0 >= p);
            uint64_t kb1 = __ballot(k1 >= p);
            if (__builtin_expect(c != Tv, 0)) {
                // remaining 18 bits: the digit's bin did not end exactly at T keys (|v| of a bf16 entry has no bits
                // below 16)
                probe_bits<(VALUES ? (1u << 16) : 1u)>(k0, k1, Tv, p, c, kb0, kb1);
                if (__builtin_expect(c != Tv, 0)) {
                    // all bits fixed and still more than T keys >= p: p is the T-th largest value and it is tied
                    const bool eq0 = (k0 == p), eq1 = (k1 == p);
                    const uint64_t q0 = __ballot(eq0), q1 = __ballot(eq1);
                    const int need = T - __popcll(__ballot(k0 > p)) - __popcll(__ballot(k1 > p));
                    // tied channels below 2l: both halves of every lower lane; below 2l+1: plus own even
                    const int r0 = mbcnt64(q0) + mbcnt64(q1);
                    const int r1 = r0 + (eq0 ? 1 : 0);
                    kb0 = __ballot((k0 > p) || (eq0 && r0 < need));   // lower channel first
                    kb1 = __ballot((k1 > p) || (eq1 && r1 < need));
                }
            }
            const bool keep0 = __builtin_amdgcn_inverse_ballot_w64(kb0);
            const bool keep1 = __builtin_amdgcn_inverse_ballot_w64(kb1);
            // slot of each kept value = number of kept channels below it
            const int pos0 = (int)__builtin_amdgcn_mbcnt_hi(
                (uint32_t)(kb1 >> 32),
                __builtin_amdgcn_mbcnt_lo((uint32_t)kb1,
                                          __builtin_amdgcn_mbcnt_hi((uint32_t)(kb0 >> 32),
                                                                    __builtin_amdgcn_mbcnt_lo((uint32_t)kb0, 0))));
            stage_row(pos0, xx, kb0, kb1, row_a, tok_bit, dump_a, em, om);
            tok_bit <<= 1;
            row_a += row_step;
            ps[u] = VALUES ? 0.0f : (keep0 ? 0.0f : w0) + (keep1 ? 0.0f : w1);
            qs[u] = 0.0f;
            if constexpr (STATS) {
                // mean over all 128 channels now (wave sum), squared deviations folded with the rest
                const float mrow = wave_total_f32(w0 + w1) * (1.0f / (float)SPARK_D);
                write_lane1(muall, (uint32_t)__builtin_amdgcn_readfirstlane(__float_as_int(mrow)), t);
                const float d0 = w0 - mrow, d1 = w1 - mrow;
                qs[u] = fmaf(d0, d0, d1 * d1);
            }
        }
    };

    // the PF rows held in x (tokens tb .. tb+PF-1); returns their pruned-saliency partials folded into one
    // register: row u (bits u0 u1 u2) in the lanes with l5 = u0, l4 = u1, l2 = u2
    auto fold8 = [&](const float (&p)[PF]) __attribute__((always_inline)) -> float {
        const float f01 = fold_halves(p[0], p[1]), f23 = fold_halves(p[2], p[3]);
        const float f45 = fold_halves(p[4], p[5]), f67 = fold_halves(p[6], p[7]);
        return fold_pair<0x124>(fold_rows(f01, f23), fold_rows(f45, f67), lane & 4);     // row_ror 4
    };
    auto do_block = [&](const uint32_t (&x)[PF], int tb) __attribute__((always_inline)) -> float2 {
        float ps[PF], qs[PF];
#pragma unroll
        for (int u0 = 0; u0 < PF; u0 += kBatch) do_batch(x, u0, tb, ps, qs);
        if constexpr (VALUES) return make_float2(0.0f, 0.0f);
        float q07 = 0.0f;
        if constexpr (STATS) q07 = fold8(qs);
        return make_float2(fold8(ps), q07);
    };

    // ---- rows t0 .. t0 + rows_per_flush - 1 leave the staging area, lane = token (the other lanes idle)
    uint8_t *const tile_out = packed + L.off_tiles + ((int64_t)h * L.n_tiles + tile) * L.tile_bytes;
    auto flush = [&](const int t0) __attribute__((always_inline)) {
        prune_lds_sync();
        // (the lane number is taken afresh here so that nothing of this rarely run part is computed ahead
        // of the row loop and kept in registers across it)
        int ln = lane;
        asm volatile("" : "+v"(ln));
        // lane = token fetches its row's sums from the lane the reduction left them in
        const int src_lane = 32 * (ln & 1) + 16 * ((ln >> 1) & 1) + 4 * ((ln >> 2) & 1) + 8 * ((ln >> 3) & 1) + (ln >> 4);
        const float mu_sum = VALUES ? 0.0f : __int_as_float(__builtin_amdgcn_ds_bpermute(src_lane * 4, __float_as_int(mureg)));
        const float sq_sum = STATS ? __int_as_float(__builtin_amdgcn_ds_bpermute(src_lane * 4, __float_as_int(sqreg))) : 0.0f;
        if (ln >= t0 && ln < t0 + rows_per_flush) {
            const bool valid = ln < nvalid;
            uint32_t *row = stage + (size_t)(ln - t0) * sw;
            const float mu = (!VALUES && valid && T < SPARK_D) ? (mu_sum / (float)(SPARK_D - T)) : 0.0f;
            // channel-ordered mask: bit 2l of the row = even ballot bit l, bit 2l+1 = odd ballot bit l.
            // Rows past the last token carry a well-formed mask (channels 0..T-1) and zero values, so a
            // reader that walks exactly T bits never runs off the mask.
            auto low_bits = [](int n) { return n <= 0 ? 0u : (n >= 32 ? 0xFFFFFFFFu : ((1u << n) - 1u)); };
            const uint32_t e_lo = (uint32_t)em, e_hi = (uint32_t)(em >> 32), o_lo = (uint32_t)om, o_hi = (uint32_t)(om >> 32);
            row[0] = valid ? (spread16(e_lo) | (spread16(o_lo) << 1)) : low_bits(T);
            row[1] = valid ? (spread16(e_lo >> 16) | (spread16(o_lo >> 16) << 1)) : low_bits(T - 32);
            row[2] = valid ? (spread16(e_hi) | (spread16(o_hi) << 1)) : low_bits(T - 64);
            row[3] = valid ? (spread16(e_hi >> 16) | (spread16(o_hi >> 16) << 1)) : low_bits(T - 96);
            if (!VALUES) row[4] = __float_as_uint(mu);
            if (STATS && valid) {
                row[INT8 ? 6 : 5] = muall;
                row[INT8 ? 7 : 6] = __float_as_uint(sqrtf(sq_sum * (1.0f / (float)SPARK_D)));
            }
            if (!valid) {
                for (int d = VALUES ? 4 : 5; d < sw; ++d) row[d] = 0u;
            } else {
                const int vend = L.val0 + (T + 1) / 2;               // one past the last staged bf16 word
                if (T & 1) row[vend - 1] &= 0xFFFFu;                 // unused upper half of the last word
                for (int d = vend; d < sw; ++d) row[d] = 0u;
                if (INT8) {
                    // absmax scale and round-to-nearest-even codes, decided in float32.  The staged bf16 words
                    // are read two at a time (four values; val0 is even, rows are 8-byte aligned, and the words
                    // behind the last kept value are zero up to the row's end).
                    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                    const u32x2 *vals2 = reinterpret_cast<const u32x2 *>(row + L.val0);
                    const int nquad = (T + 3) / 4;
                    float amax = 0.0f;
                    for (int c = 0; c < nquad; ++c) {
                        const u32x2 w = vals2[c];
                        amax = fmaxf(fmaxf(amax, fabsf(bf16_bits_to_float(w.x & 0xFFFFu))), fabsf(bf16_bits_to_float(w.x >> 16)));
                        amax = fmaxf(fmaxf(amax, fabsf(bf16_bits_to_float(w.y & 0xFFFFu))), fabsf(bf16_bits_to_float(w.y >> 16)));
                    }
                    const float scale = __fdiv_rn(amax, 127.0f);
                    row[5] = __float_as_uint(scale);
                    // The code is rint(fl32(v / scale)).  The exact division costs ten instructions a value, so the
                    // integer is first taken from v times an approximate reciprocal: that product and the exactly
                    // rounded quotient both lie within 3.1e-5 of v / scale (|v / scale| <= 127, reciprocal to one
                    // unit in the last place, two roundings), so unless the product comes within 6e-5 of a half
                    // integer the two round to the same integer; otherwise (and when the reciprocal is not
                    // finite) the lane divides exactly.
                    const float rs = __builtin_amdgcn_rcpf(scale);
                    auto code_of = [&](uint32_t bits) -> uint32_t {
                        const float v = bf16_bits_to_float(bits);
                        const float qa = v * rs;
                        float qf = rintf(qa);
                        if (!(fabsf(qa - qf) < 0.5f - 6e-5f)) qf = rintf(__fdiv_rn(v, scale));
                        // (|v| <= amax and scale = fl32(amax / 127), so |qf| <= 127 already: no clamp is needed)
                        return (uint32_t)(int)qf & 0xFFu;
                    };
                    for (int c = 0; c < nquad; ++c) {
                        const u32x2 w = vals2[c];      // values 4c .. 4c+3 (zero bits past the T-th: code 0)
                        uint32_t word = 0;
                        if (scale != 0.0f)
                            word = code_of(w.x & 0xFFFFu) | (code_of(w.x >> 16) << 8) | (code_of(w.y & 0xFFFFu) << 16) |
                                   (code_of(w.y >> 16) << 24);
                        row[L.val0 + c] = word;   // never ahead of the bf16 words still to be read
                    }
                    for (int d = L.val0 + L.nv; d < L.ndw; ++d) row[d] = 0u;
                }
            }
            // ---- coalesced tile write: section q holds words 4q..4q+3 of every token
            // (written once, read by another kernel much later: non-temporal, like the loads)
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
            for (int q = 0; q < L.nq; ++q) {
                u32x4 v;
                v.x = row[4 * q + 0];
                v.y = row[4 * q + 1];
                v.z = row[4 * q + 2];
                v.w = row[4 * q + 3];
                __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(tile_out + (size_t)q * 1024 + ln * 16));
            }
            if (L.tail2) {
                u32x2 v;
                v.x = row[4 * L.nq + 0];
                v.y = row[4 * L.nq + 1];
                __builtin_nontemporal_store(v, reinterpret_cast<u32x2 *>(tile_out + (size_t)L.nq * 1024 + ln * 8));
            }
        }
        prune_lds_sync();      // the staging rows are reused
    };

    // Every one of the 64 rows is processed; rows past the last token repeat the last one and are
    // overwritten by the epilogue.
    for (int tb = 0; tb < SPARK_TILE_TOKENS; tb += 2 * PF) {
        load_block(xb, tb + PF);
        const float2 fa = do_block(xa, tb);
        if (tb + 2 * PF < SPARK_TILE_TOKENS) load_block(xa, tb + 2 * PF);
        const float2 fb = do_block(xb, tb + PF);
        if constexpr (!VALUES) {
            // pruned-saliency sums of these 16 tokens: pair the two blocks, finish across the four rows
            // (the sixteen sums go to the lanes whose two low bits are the group's number, see quad_sum above)
            const float s = quad_sum(fold_pair<0x128>(fa.x, fb.x, lane & 8));              // row_ror 8
            if ((lane & 3) == (tb >> 4)) mureg = s;
            if constexpr (STATS) {
                const float s2 = quad_sum(fold_pair<0x128>(fa.y, fb.y, lane & 8));
                if ((lane & 3) == (tb >> 4)) sqreg = s2;
            }
        }
        if (((tb + 2 * PF) & (rows_per_flush - 1)) == 0) {
            flush(tb + 2 * PF - rows_per_flush);
            row_a = row_a0;
        }
    }
}


// One launch for a whole cache: the first tail_blocks blocks take the heads' partly filled last tiles (few
// wavefronts, each a long serial chain of rows: they start first and run beside the rest), the other blocks the
// tiles that hold 64 tokens.  Blocks are four independent wavefronts; nothing synchronises across them.
// (WITH_TAIL = false: the token count is a multiple of 64, there are no partly filled tiles, and the kernel holds
// the one instantiation only, which the register allocator then treats a little better.)
template <int MODE, bool VALUES, bool WITH_TAIL>
__global__ __launch_bounds__(kPruneWaves * 64, SPARK_PRUNE_MIN_WAVES) void spark_prune_kernel(
    const uint16_t *__restrict__ k, int64_t k_tok_stride, int64_t k_head_stride,
    const int32_t *__restrict__ cu, uint8_t *__restrict__ packed, SparkLayout L, int rows_per_flush, int tail_blocks)
{
    // the wavefront index is the same in all 64 lanes; saying so keeps everything derived from it
    // (tile, token loop, search state) in scalar registers
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (WITH_TAIL && (int)blockIdx.x < tail_blocks)
        prune_tile<MODE, false, VALUES>(k, k_tok_stride, k_head_stride, cu, packed, L, rows_per_flush, wave,
                                        (int64_t)blockIdx.x * kPruneWaves + wave);
    else
        prune_tile<MODE, true, VALUES>(k, k_tok_stride, k_head_stride, cu, packed, L, rows_per_flush, wave,
                                       (int64_t)((int)blockIdx.x - tail_blocks) * kPruneWaves + wave);
}

// ---------------------------------------------------------------- canonical export

// one thread per (token, KV head) row
__global__ void spark_unpack_kernel(const uint8_t *__restrict__ packed, SparkLayout L,
                                    uint32_t *mask_out, void *vals_out, float *mu_out,
                                    float *scale_out, float *a_out, float *mu_all_out, float *sigma_out)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t rows = L.total_tokens * L.n_kv_heads;
    if (a_out && idx < (int64_t)L.batch * L.n_kv_heads * SPARK_D)
        a_out[idx] = reinterpret_cast<const float *>(packed + L.off_a)[idx];
    if (idx >= rows) return;
    const int64_t n = idx / L.n_kv_heads;
    const int h = (int)(idx % L.n_kv_heads);
    const uint8_t *tile = packed + L.off_tiles + ((int64_t)h * L.n_tiles + n / SPARK_TILE_TOKENS) * L.tile_bytes;
    const int t = (int)(n % SPARK_TILE_TOKENS);
    auto word = [&](int d) {
        return *reinterpret_cast<const uint32_t *>(tile + spark_tile_word_offset(L, t, d));
    };
    if (mask_out)
        for (int m = 0; m < 4; ++m) mask_out[idx * 4 + m] = word(m);
    if (mu_out && !L.values) mu_out[idx] = __uint_as_float(word(4));
    if (L.stats) {
        if (mu_all_out) mu_all_out[idx] = __uint_as_float(word(L.int8 ? 6 : 5));
        if (sigma_out) sigma_out[idx] = __uint_as_float(word(L.int8 ? 7 : 6));
    }
    if (L.int8) {
        if (scale_out) scale_out[idx] = __uint_as_float(word(5));
        if (vals_out) {
            int8_t *o = reinterpret_cast<int8_t *>(vals_out) + idx * L.T;
            for (int i = 0; i < L.T; ++i) o[i] = (int8_t)((word(L.val0 + i / 4) >> (8 * (i & 3))) & 0xFF);
        }
    } else if (vals_out) {
        uint16_t *o = reinterpret_cast<uint16_t *>(vals_out) + idx * L.T;
        for (int i = 0; i < L.T; ++i) o[i] = (uint16_t)((word(L.val0 + i / 2) >> (16 * (i & 1))) & 0xFFFF);
    }
}


// ---------------------------------------------------------------- host-side launch

namespace {

// every tile of the cache in one launch
template <bool VALUES>
hipError_t launch_tiles(const uint16_t *x, int64_t tok_stride, int64_t head_stride, const int32_t *cu,
                        uint8_t *packed, const SparkLayout &L, hipStream_t st)
{
    const size_t lds = spark_prune_lds_bytes(L);
    const int64_t full_waves = (L.total_tokens / SPARK_TILE_TOKENS) * L.n_kv_heads;
    const int64_t tail_waves = (L.total_tokens % SPARK_TILE_TOKENS) ? L.n_kv_heads : 0;
    const int tail_blocks = (int)((tail_waves + kPruneWaves - 1) / kPruneWaves);
    const int64_t nblocks = tail_blocks + (full_waves + kPruneWaves - 1) / kPruneWaves;
    if (nblocks == 0) return hipSuccess;
    auto launch = [&](auto kern) -> hipError_t {
        if (lds > 48 * 1024) {
            hipError_t e2 = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e2 != hipSuccess) return e2;
        }
        hipLaunchKernelGGL(kern, dim3((unsigned)nblocks), dim3(kPruneWaves * 64), lds, st, x, tok_stride, head_stride, cu,
                           packed, L, spark_prune_rows_per_flush(L), tail_blocks);
        return hipGetLastError();
    };
    const int mode = VALUES ? 0 : (L.int8 ? 1 : 0) + (L.stats ? 2 : 0);
    if (tail_blocks == 0) {
        switch (mode) {
            case 0: return launch(&spark_prune_kernel<0, VALUES, false>);
            case 1: return launch(&spark_prune_kernel<1, false, false>);
            case 2: return launch(&spark_prune_kernel<2, false, false>);
            default: return launch(&spark_prune_kernel<3, false, false>);
        }
    }
    switch (mode) {
        case 0: return launch(&spark_prune_kernel<0, VALUES, true>);
        case 1: return launch(&spark_prune_kernel<1, false, true>);
        case 2: return launch(&spark_prune_kernel<2, false, true>);
        default: return launch(&spark_prune_kernel<3, false, true>);
    }
}

}  // namespace

hipError_t launch_window_stat(const uint16_t *qwin, uint8_t *packed, const SparkLayout &L, int Hq, int W, hipStream_t st)
{
    hipLaunchKernelGGL(spark_window_stat_kernel, dim3(L.batch * L.n_kv_heads),
                       dim3(((Hq / L.n_kv_heads) < 8 ? (Hq / L.n_kv_heads) : 8) * SPARK_D), 0, st, qwin, Hq,
                       L.n_kv_heads, W, packed, L);
    return hipGetLastError();
}

hipError_t launch_prune(const uint16_t *k, int64_t k_tok_stride, int64_t k_head_stride, const uint16_t *qwin,
                        const int32_t *cu, uint8_t *packed, const SparkLayout &L, int Hq, int W, hipStream_t st)
{
    const hipError_t e = launch_window_stat(qwin, packed, L, Hq, W, st);
    if (e != hipSuccess) return e;
    return launch_tiles<false>(k, k_tok_stride, k_head_stride, cu, packed, L, st);
}

hipError_t launch_prune_values(const uint16_t *v, int64_t v_tok_stride, int64_t v_head_stride, uint8_t *packed,
                               const SparkLayout &L, hipStream_t st)
{
    return launch_tiles<true>(v, v_tok_stride, v_head_stride, nullptr, packed, L, st);
}

hipError_t launch_unpack(const uint8_t *packed, const SparkLayout &L, uint32_t *mask_out, void *vals_out,
                         float *mu_out, float *scale_out, float *a_out, float *mu_all_out, float *sigma_out,
                         hipStream_t st)
{
    int64_t n = L.total_tokens * L.n_kv_heads;
    const int64_t na = (int64_t)L.batch * L.n_kv_heads * SPARK_D;
    if (a_out && na > n) n = na;
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(spark_unpack_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, packed, L,
                       mask_out, vals_out, mu_out, scale_out, a_out, mu_all_out, sigma_out);
    return hipGetLastError();
}

}  // namespace spark
