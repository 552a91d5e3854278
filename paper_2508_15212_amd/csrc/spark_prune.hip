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
//                             the T-th largest is found by a most-significant-bit-first
//                             search on the float32 bit pattern where every probe is two
//                             wave ballots and two scalar popcounts; the kept set is then a
//                             pair of 64-bit ballots = the channel mask, and a prefix
//                             popcount (mbcnt) gives each kept value its slot in the packed
//                             row.  Rows are staged in LDS and the finished tile is written
//                             with lane = token, coalesced.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "spark_kernels.h"
#include "spark_layout.h"

namespace spark {

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

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

constexpr int kPruneWaves = 4;      // wavefronts per block, one tile each
constexpr int kHistBins = 64;       // one 64-bin digit histogram per wavefront (+ 64 spare words)

// words per token in the LDS staging row: mask, mu, (scale), then T bf16 values
__host__ __device__ inline int spark_stage_words(const SparkLayout &L)
{
    int w = L.val0 + (L.T + 1) / 2;
    if (w < L.ndw) w = L.ndw;
    return (w + 1) & ~1;
}

__host__ inline size_t spark_prune_lds_bytes(const SparkLayout &L)
{
    return (size_t)kPruneWaves *
           ((size_t)SPARK_TILE_TOKENS * spark_stage_words(L) * 4 + 2 * kHistBins * 4);
}

// bits 0..15 of x spread to the even bit positions of a 32-bit word
__device__ __forceinline__ uint32_t spread16(uint32_t x)
{
    x &= 0xFFFFu;
    x = (x | (x << 8)) & 0x00FF00FFu;
    x = (x | (x << 4)) & 0x0F0F0F0Fu;
    x = (x | (x << 2)) & 0x33333333u;
    x = (x | (x << 1)) & 0x55555555u;
    return x;
}

__device__ __forceinline__ int mbcnt64(uint64_t m)   // set bits of m below this lane
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0));
}

// Inclusive prefix sum over the 64 lanes (lane l gets x_0 + ... + x_l) with data-parallel-primitive
// moves: shifts by 1, 2, 4, 8 inside each row of 16 lanes, then the last lane of row 0 / 2 is added
// to row 1 / 3 and the last lane of row 1 to rows 2 and 3.  Lanes with no source add 0.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t v)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, false);   // row_shr 1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, false);   // row_shr 2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, false);   // row_shr 4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, false);   // row_shr 8
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);   // row_bcast 15 -> rows 1, 3
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);   // row_bcast 31 -> rows 2, 3
    return v;
}

// Four wave-uniform values into lane `lane_id` (wave-uniform) of four registers; the other lanes
// keep theirs.  (The lane selector of v_writelane travels in M0 because the value is a scalar
// register already.)
__device__ __forceinline__ void write_lane4(uint32_t &a, uint32_t &b, uint32_t &c, uint32_t &d, uint32_t va,
                                            uint32_t vb, uint32_t vc, uint32_t vd, int lane_id)
{
    asm("s_mov_b32 m0, %8\n\t"
        "v_writelane_b32 %0, %4, m0\n\t"
        "v_writelane_b32 %1, %5, m0\n\t"
        "v_writelane_b32 %2, %6, m0\n\t"
        "v_writelane_b32 %3, %7, m0"
        : "+v"(a), "+v"(b), "+v"(c), "+v"(d)
        : "s"(va), "s"(vb), "s"(vc), "s"(vd), "s"(lane_id)
        : "m0");
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

// Sum over the 64 lanes, returned wave-uniform (same moves as the prefix sum; lane 63 ends with the total).
__device__ __forceinline__ float wave_total_f32(float v)
{
    auto step = [&](auto ctrl, auto rmask) {
        v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), decltype(ctrl)::value,
                                                        decltype(rmask)::value, 0xF, false));
    };
    step(std::integral_constant<int, 0x111>{}, std::integral_constant<int, 0xF>{});
    step(std::integral_constant<int, 0x112>{}, std::integral_constant<int, 0xF>{});
    step(std::integral_constant<int, 0x114>{}, std::integral_constant<int, 0xF>{});
    step(std::integral_constant<int, 0x118>{}, std::integral_constant<int, 0xF>{});
    step(std::integral_constant<int, 0x142>{}, std::integral_constant<int, 0xA>{});
    step(std::integral_constant<int, 0x143>{}, std::integral_constant<int, 0xC>{});
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// One wave-uniform value into lane `lane_id` of a register.
__device__ __forceinline__ void write_lane1(uint32_t &a, uint32_t va, int lane_id)
{
    asm("s_mov_b32 m0, %2\n\t"
        "v_writelane_b32 %0, %1, m0"
        : "+v"(a)
        : "s"(va), "s"(lane_id)
        : "m0");
}

__device__ __forceinline__ void prune_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// FULL: the launch covers the tiles that hold all 64 tokens (the first total_tokens / 64 of every head);
// otherwise it covers the one partly filled last tile of every head, one wavefront each.
// MODE: 0 = bf16 kept entries, 1 = int8 codes + scale, 2 = bf16 plus the all-channel mean and standard
// deviation of the row's saliencies (App. "Caching Pruned Channel Statistics", for the sampled recovery).
// VALUES: the rows are value-cache rows (App. "Pruning Value Cache Channels"): the score of a channel is
// |v| itself, there is no channel weight, no sequence bookkeeping and no statistic of the pruned set.
template <int MODE, bool FULL, bool VALUES>
__global__ __launch_bounds__(kPruneWaves * 64) void spark_prune_kernel(
    const uint16_t *__restrict__ k, int64_t k_tok_stride, int64_t k_head_stride,
    const int32_t *__restrict__ cu, uint8_t *__restrict__ packed, SparkLayout L)
{
    constexpr bool INT8 = (MODE == 1), STATS = (MODE == 2);
    extern __shared__ __align__(16) uint8_t smem[];
    const int lane = threadIdx.x & 63;
    // the wavefront index is the same in all 64 lanes; saying so keeps everything derived from it
    // (tile, token loop, search state) in scalar registers
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t wt = (int64_t)blockIdx.x * kPruneWaves + wave;
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
                      (size_t)wave * (SPARK_TILE_TOKENS * sw + 2 * kHistBins);
    uint32_t *hist = stage + SPARK_TILE_TOKENS * sw;
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

    // lane t collects, for token t, the ballots of kept even channels (e) and kept odd channels (o)
    uint32_t e_lo = 0, e_hi = 0, o_lo = 0, o_hi = 0;
    float mureg = 0.0f;                                     // lane t: sum of pruned saliencies
    uint32_t muall = 0;                                     // lane t: mean saliency over all channels (bits)
    float sqreg = 0.0f;                                     // lane t: sum of squared deviations from it

    // Rows are fetched a block ahead: while one block of PF rows is searched the next is in flight,
    // in two register sets that swap roles.
    uint32_t xa[PF], xb[PF];
    load_block(xa, 0);

    // T-th largest key of a row.  The search is most-significant-bit first on the float32 bit pattern:
    // keep a prefix p such that at least T keys are >= p and try to extend it; a probe is two wave
    // ballots and two scalar popcounts.  Two shortcuts settle the top 14 bits: the exponent E (largest
    // with at least T keys >= 2^E) is found by stepping from the previous row's -- rows of one head
    // rarely differ by more than an octave -- and the next six bits by one counting pass (lanes add
    // their keys' digits to a 64-bin LDS histogram stored highest digit first, lane l reads bin l, a
    // wave prefix sum turns that into "keys with digit >= d", a ballot finds the digit where the count
    // reaches what is still needed).  The search stops as soon as exactly T keys are >= p.
    int E;
    {   // first row: E by bisection over the 256 exponents
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
        E = lo;
    }

    // searches and stages the PF rows held in x (tokens tb .. tb+PF-1); returns their pruned-saliency
    // partials folded into one register (token tb + u in the lanes with l & 7 == u)
    auto do_block = [&](const uint32_t (&x)[PF], int tb) __attribute__((always_inline)) -> float2 {
        float ps[PF], qs[PF];
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int t = tb + u;
            const uint32_t xx = x[u];
            if (!VALUES && __builtin_expect(t >= seq_end_t, 0)) {    // rare: the tile crosses into the next non-empty sequence
                if (t < nvalid) {
                    do {
                        ++b;
                        seq_end_t = (int)((int64_t)cu[b + 1] - n0);
                    } while (t >= seq_end_t);
                    a01 = a_all[((int64_t)b * L.n_kv_heads + h) * (SPARK_D / 2) + lane];
                    // finish this load here, inside the rare branch: otherwise the wait for it
                    // lands after the join and drains the prefetched K rows on every token
                    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
                }
            }
            // saliency: one float32 multiply, never fused
            const float w0 = __fmul_rn(a01.x, fabsf(__uint_as_float(xx << 16)));
            const float w1 = __fmul_rn(a01.y, fabsf(__uint_as_float(xx & 0xFFFF0000u)));
            const uint32_t key0 = __float_as_uint(w0), key1 = __float_as_uint(w1);
            auto count_ge = [&](uint32_t x) {
                return __popcll(__ballot(key0 >= x)) + __popcll(__ballot(key1 >= x));
            };

            // exponent: in the common case the previous row's E still has (keys >= 2^E) >= T > above1
            int above1 = count_ge(((uint32_t)E + 1u) << 23);      // keys with exponent > E
            while (__builtin_expect(above1 >= T, 0)) {            // step up (2^256 is above every key)
                ++E;
                above1 = count_ge(((uint32_t)E + 1u) << 23);
            }
            // next six bits: counting pass over the keys whose exponent is E; the others land in a
            // spare word (bins 64..127) that is never read.  If the octave turns out to hold fewer
            // keys than are still needed, all of it counts as "above" and the pass moves one octave
            // down (octave 0 ends this: it holds every key not above it).
            uint32_t s2;
            uint64_t reached;
            for (;;) {
                hist[lane] = 0u;
                prune_lds_sync();
                {
                    const uint32_t top = ((uint32_t)E << 6) | 63u;
                    const uint32_t d0 = top - (key0 >> 17), d1 = top - (key1 >> 17);
                    const uint32_t spare = (uint32_t)(kHistBins + lane);   // one spare word per lane: no pile-up
                    atomicAdd(&hist[d0 < spare ? d0 : spare], 1u);
                    atomicAdd(&hist[d1 < spare ? d1 : spare], 1u);
                }
                prune_lds_sync();
                s2 = wave_inclusive_sum(hist[lane]);              // keys in octave E with digit >= 63 - lane
                prune_lds_sync();
                reached = __ballot(s2 >= (uint32_t)(T - above1)); // T - above1 >= 1
                if (__builtin_expect(reached != 0, 1)) break;
                above1 += __builtin_amdgcn_readlane((int)s2, 63);
                --E;
            }
            const int l2 = __builtin_ctzll(reached);
            const int ge = above1 + __builtin_amdgcn_readlane((int)s2, l2);   // keys >= p
            uint32_t p = ((uint32_t)E << 23) | ((uint32_t)(63 - l2) << 17);
            int tied = 0;
            if (ge != T) {
                // remaining 17 bits (a probe is 2 vector compares and ~8 scalar instructions, with
                // the candidate and the prefix held in scalar registers)
                tied = 1;
                uint32_t bit = 1u << 16;
#pragma nounroll
                do {
                    const uint32_t cand = p | bit;
                    const int c = count_ge(cand);
                    p = (c >= T) ? cand : p;
                    if (c == T) { tied = 0; break; }
                    bit >>= 1;
                } while (bit != (VALUES ? (1u << 15) : 0u));   // |v| of a bf16 entry has no bits below 16
            }
            // exactly T keys are >= p, unless p is the T-th largest value and it is tied
            uint64_t kb0 = __ballot(key0 >= p), kb1 = __ballot(key1 >= p);
            if (__builtin_expect(tied, 0)) {
                const bool eq0 = (key0 == p), eq1 = (key1 == p);
                const uint64_t q0 = __ballot(eq0), q1 = __ballot(eq1);
                const int need = T - __popcll(__ballot(key0 > p)) - __popcll(__ballot(key1 > p));
                // tied channels below 2l: both halves of every lower lane; below 2l+1: plus own even
                const int r0 = mbcnt64(q0) + mbcnt64(q1);
                const int r1 = r0 + (eq0 ? 1 : 0);
                kb0 = __ballot((key0 > p) || (eq0 && r0 < need));   // lower channel first
                kb1 = __ballot((key1 > p) || (eq1 && r1 < need));
            }
            const bool keep0 = __builtin_amdgcn_inverse_ballot_w64(kb0);
            const bool keep1 = __builtin_amdgcn_inverse_ballot_w64(kb1);
            // slot of each kept value = number of kept channels below it
            const int pos0 = (int)__builtin_amdgcn_mbcnt_hi(
                (uint32_t)(kb1 >> 32),
                __builtin_amdgcn_mbcnt_lo((uint32_t)kb1,
                                          __builtin_amdgcn_mbcnt_hi((uint32_t)(kb0 >> 32),
                                                                    __builtin_amdgcn_mbcnt_lo((uint32_t)kb0, 0))));
            const int pos1 = pos0 + (keep0 ? 1 : 0);
            uint16_t *vrow = stage16 + (size_t)t * sw * 2 + L.val0 * 2;
            // every lane stores; a pruned value goes to the lane's spare word instead of masking
            // lanes off around the store
            uint16_t *dump = reinterpret_cast<uint16_t *>(hist + kHistBins + lane);
            *(keep0 ? vrow + pos0 : dump) = (uint16_t)xx;
            *(keep1 ? vrow + pos1 : dump) = (uint16_t)(xx >> 16);
            // lane t keeps the ballots of token t
            write_lane4(e_lo, e_hi, o_lo, o_hi, (uint32_t)kb0, (uint32_t)(kb0 >> 32), (uint32_t)kb1,
                        (uint32_t)(kb1 >> 32), t);
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
        if constexpr (VALUES) return make_float2(0.0f, 0.0f);
        float q07 = 0.0f;
        if constexpr (STATS) {
            const float g01 = fold_pair<0xB1>(qs[0], qs[1], lane & 1);
            const float g23 = fold_pair<0xB1>(qs[2], qs[3], lane & 1);
            const float g45 = fold_pair<0xB1>(qs[4], qs[5], lane & 1);
            const float g67 = fold_pair<0xB1>(qs[6], qs[7], lane & 1);
            q07 = fold_pair<0x124>(fold_pair<0x4E>(g01, g23, lane & 2), fold_pair<0x4E>(g45, g67, lane & 2), lane & 4);
        }
        const float f01 = fold_pair<0xB1>(ps[0], ps[1], lane & 1);     // quad_perm [1,0,3,2]
        const float f23 = fold_pair<0xB1>(ps[2], ps[3], lane & 1);
        const float f45 = fold_pair<0xB1>(ps[4], ps[5], lane & 1);
        const float f67 = fold_pair<0xB1>(ps[6], ps[7], lane & 1);
        const float f03 = fold_pair<0x4E>(f01, f23, lane & 2);         // quad_perm [2,3,0,1]
        const float f47 = fold_pair<0x4E>(f45, f67, lane & 2);
        return make_float2(fold_pair<0x124>(f03, f47, lane & 4), q07);   // row_ror 4
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
            float s = fold_pair<0x128>(fa.x, fb.x, lane & 8);              // row_ror 8
            s += __shfl_xor(s, 16);
            s += __shfl_xor(s, 32);
            if ((lane >> 4) == (tb >> 4)) mureg = s;
            if constexpr (STATS) {
                float s2 = fold_pair<0x128>(fa.y, fb.y, lane & 8);
                s2 += __shfl_xor(s2, 16);
                s2 += __shfl_xor(s2, 32);
                if ((lane >> 4) == (tb >> 4)) sqreg = s2;
            }
        }
    }

    // ---- row epilogue, lane = token
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const bool valid = lane < nvalid;
    uint32_t *row = stage + (size_t)lane * sw;
    const float mu = (!VALUES && valid && T < SPARK_D) ? (mureg / (float)(SPARK_D - T)) : 0.0f;
    // channel-ordered mask: bit 2l of the row = even ballot bit l, bit 2l+1 = odd ballot bit l.
    // Rows past the last token carry a well-formed mask (channels 0..T-1) and zero values, so a
    // reader that walks exactly T bits never runs off the mask.
    auto low_bits = [](int n) { return n <= 0 ? 0u : (n >= 32 ? 0xFFFFFFFFu : ((1u << n) - 1u)); };
    row[0] = valid ? (spread16(e_lo) | (spread16(o_lo) << 1)) : low_bits(T);
    row[1] = valid ? (spread16(e_lo >> 16) | (spread16(o_lo >> 16) << 1)) : low_bits(T - 32);
    row[2] = valid ? (spread16(e_hi) | (spread16(o_hi) << 1)) : low_bits(T - 64);
    row[3] = valid ? (spread16(e_hi >> 16) | (spread16(o_hi >> 16) << 1)) : low_bits(T - 96);
    if (!VALUES) row[4] = __float_as_uint(mu);
    if (STATS) {
        row[5] = valid ? muall : 0u;
        row[6] = valid ? __float_as_uint(sqrtf(sqreg * (1.0f / (float)SPARK_D))) : 0u;
    }
    if (!valid) {
        for (int d = VALUES ? 4 : (STATS ? 7 : 5); d < sw; ++d) row[d] = 0u;
    } else {
        const int vend = L.val0 + (T + 1) / 2;               // one past the last staged bf16 word
        if (T & 1) row[vend - 1] &= 0xFFFFu;                 // unused upper half of the last word
        for (int d = vend; d < sw; ++d) row[d] = 0u;
        if (INT8) {
            // absmax scale and round-to-nearest-even codes, decided in float32
            auto val = [&](int i) {
                return bf16_bits_to_float((row[L.val0 + (i >> 1)] >> (16 * (i & 1))) & 0xFFFFu);
            };
            float amax = 0.0f;
            for (int i = 0; i < T; ++i) amax = fmaxf(amax, fabsf(val(i)));
            const float scale = __fdiv_rn(amax, 127.0f);
            row[5] = __float_as_uint(scale);
            for (int c = 0; c < L.nv; ++c) {
                uint32_t word = 0;
                for (int e = 0; e < 4; ++e) {
                    const int i = 4 * c + e;
                    int code = 0;
                    if (i < T && scale != 0.0f) {
                        float qf = rintf(__fdiv_rn(val(i), scale));
                        qf = fminf(fmaxf(qf, -127.0f), 127.0f);
                        code = (int)qf;
                    }
                    word |= ((uint32_t)code & 0xFFu) << (8 * e);
                }
                row[L.val0 + c] = word;   // never ahead of the bf16 words still to be read
            }
            for (int d = L.val0 + L.nv; d < L.ndw; ++d) row[d] = 0u;
        }
    }
    // ---- coalesced tile write: section q holds words 4q..4q+3 of every token
    uint8_t *tile_out = packed + L.off_tiles + ((int64_t)h * L.n_tiles + tile) * L.tile_bytes;
    // (written once, read by another kernel much later: non-temporal, like the loads)
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    for (int q = 0; q < L.nq; ++q) {
        u32x4 v;
        v.x = row[4 * q + 0];
        v.y = row[4 * q + 1];
        v.z = row[4 * q + 2];
        v.w = row[4 * q + 3];
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(tile_out + (size_t)q * 1024 + lane * 16));
    }
    if (L.tail2) {
        u32x2 v;
        v.x = row[4 * L.nq + 0];
        v.y = row[4 * L.nq + 1];
        __builtin_nontemporal_store(v, reinterpret_cast<u32x2 *>(tile_out + (size_t)L.nq * 1024 + lane * 8));
    }
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
        if (mu_all_out) mu_all_out[idx] = __uint_as_float(word(5));
        if (sigma_out) sigma_out[idx] = __uint_as_float(word(6));
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

// the tiles that hold 64 tokens, then (if the token count is not a multiple of 64) each head's last tile
template <bool VALUES>
hipError_t launch_tiles(const uint16_t *x, int64_t tok_stride, int64_t head_stride, const int32_t *cu,
                        uint8_t *packed, const SparkLayout &L, hipStream_t st)
{
    const size_t lds = spark_prune_lds_bytes(L);
    auto launch = [&](auto kern, int64_t waves) -> hipError_t {
        if (waves == 0) return hipSuccess;
        if (lds > 48 * 1024) {
            hipError_t e2 = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e2 != hipSuccess) return e2;
        }
        const int nblocks = (int)((waves + kPruneWaves - 1) / kPruneWaves);
        hipLaunchKernelGGL(kern, dim3(nblocks), dim3(kPruneWaves * 64), lds, st, x, tok_stride, head_stride, cu,
                           packed, L);
        return hipGetLastError();
    };
    const int64_t full_waves = (L.total_tokens / SPARK_TILE_TOKENS) * L.n_kv_heads;
    const int64_t tail_waves = (L.total_tokens % SPARK_TILE_TOKENS) ? L.n_kv_heads : 0;
    if (VALUES || (!L.int8 && !L.stats)) {
        const hipError_t e = launch(&spark_prune_kernel<0, true, VALUES>, full_waves);
        return e != hipSuccess ? e : launch(&spark_prune_kernel<0, false, VALUES>, tail_waves);
    }
    if (L.int8) {
        const hipError_t e = launch(&spark_prune_kernel<1, true, false>, full_waves);
        return e != hipSuccess ? e : launch(&spark_prune_kernel<1, false, false>, tail_waves);
    }
    const hipError_t e = launch(&spark_prune_kernel<2, true, false>, full_waves);
    return e != hipSuccess ? e : launch(&spark_prune_kernel<2, false, false>, tail_waves);
}

}  // namespace

hipError_t launch_prune(const uint16_t *k, int64_t k_tok_stride, int64_t k_head_stride, const uint16_t *qwin,
                        const int32_t *cu, uint8_t *packed, const SparkLayout &L, int Hq, int W, hipStream_t st)
{
    hipLaunchKernelGGL(spark_window_stat_kernel, dim3(L.batch * L.n_kv_heads),
                       dim3(((Hq / L.n_kv_heads) < 8 ? (Hq / L.n_kv_heads) : 8) * SPARK_D), 0, st, qwin, Hq,
                       L.n_kv_heads, W, packed, L);
    hipError_t e = hipGetLastError();
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
