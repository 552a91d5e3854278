// The top-p variant of the prefill pruning for gfx950 (wave64).
//
// [Sec. "Adaptive Variants of SparK": per token, the fewest most salient channels whose saliencies together
//  account for 99 % of the row's total saliency are kept; no fixed pruning ratio.]
//
// The count of a row is an integer decided by sums, so the sums are integers too: every saliency of a row is
// expressed in units of the last place of the row's largest saliency, rounded down (q < 2^24, a row's total
// below 2^31), and with p in basis points the row keeps the smallest m >= 1 whose m largest saliencies have
//     10000 * sum q  >=  p * (total of q),      i.e.   sum q >= need := ceil(p * total / 10000).
// Exact in any summation order, which is what a parallel reduction needs.  Ties: lower channel first.
//
// Kernels
//   spark_topp_select_kernel  one wavefront per tile of 64 tokens; per token a radix selection ON SUMS: the float32
//                             bit pattern of the smallest kept saliency is fixed level by level, each level
//                             adding the q of the still undecided keys to 64 LDS bins by their next digit; a wave
//                             prefix sum over the bins (highest digit first) and one ballot give the digit at
//                             which the running sum reaches `need`.  The first level takes ten bits (exponent
//                             and two mantissa bits) over a window of sixteen octaves below the row's largest
//                             key, the others six bits each; the levels end as soon as one key alone starts
//                             with the bits fixed so far.  Writes the rows' fixed part (mask, mean
//                             saliency of the pruned channels, count) and the tile's length in the value stream.
//   spark_topp_scan_kernel    exclusive prefix sum of the tile lengths of every KV head: the directory.
//   spark_topp_pack_kernel    one wavefront per row: reads the dense key row with one coalesced load; every lane
//                             finds the slots of its two channels from popcounts of the row's mask and stores its
//                             kept entries into the value stream at the place the directory and the counts of
//                             the tile's lower tokens give.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spark_kernels.h"
#include "spark_layout.h"
#include "spark_wave.h"

namespace spark {

namespace {

constexpr int kWaves = 4;     // wavefronts per block, one tile each

// Maximum over the 64 lanes, wave-uniform.  Data-parallel-primitive moves: two quad permutes and two row rotates
// leave each row of 16 lanes holding its row maximum, two row broadcasts fold the four rows into lane 63.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_max_u32_step(uint32_t x)
{
    const uint32_t y = (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, CTRL, ROW_MASK, 0xF, false);
    return x > y ? x : y;
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    v = dpp_max_u32_step<0xB1, 0xF>(v);    // quad_perm [1,0,3,2]
    v = dpp_max_u32_step<0x4E, 0xF>(v);    // quad_perm [2,3,0,1]
    v = dpp_max_u32_step<0x124, 0xF>(v);   // row_ror 4
    v = dpp_max_u32_step<0x128, 0xF>(v);   // row_ror 8
    v = dpp_max_u32_step<0x142, 0xA>(v);   // row_bcast 15 into rows 1 and 3
    v = dpp_max_u32_step<0x143, 0xC>(v);   // row_bcast 31 into rows 2 and 3
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// a saliency (float32 bits, sign clear) in units of 2^(emax - 150), rounded down; emax >= 1
__device__ __forceinline__ uint32_t quantise(uint32_t bits, int emax)
{
    const int e = (int)(bits >> 23);
    const uint32_t mant = (bits & 0x7FFFFFu) | (e ? 0x800000u : 0u);
    const int shift = emax - (e ? e : 1);
    return shift < 24 ? (mant >> shift) : 0u;
}

}  // namespace

template <bool FULL>
__global__ __launch_bounds__(kWaves * 64) void spark_topp_select_kernel(
    const uint16_t *__restrict__ k, int64_t k_tok_stride, int64_t k_head_stride, const int32_t *__restrict__ cu,
    uint8_t *__restrict__ packed, SparkLayout L, int p_bp)
{
    __shared__ uint32_t hist_all[kWaves][128];      // per wavefront: 64 bins, then one spare word per lane
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t wt = (int64_t)blockIdx.x * kWaves + wave;
    const int64_t full_tiles = L.total_tokens / SPARK_TILE_TOKENS;
    if (wt >= (FULL ? full_tiles : 1) * L.n_kv_heads) return;    // the whole wavefront leaves; no block barrier is used
    const int h = FULL ? (int)(wt / full_tiles) : (int)wt;
    const int64_t tile = FULL ? wt % full_tiles : full_tiles;
    const int64_t n0 = tile * SPARK_TILE_TOKENS;
    const int nvalid = FULL ? SPARK_TILE_TOKENS : (int)(L.total_tokens - n0);
    uint32_t *hist = hist_all[wave];

    // sequence of the first token: largest b with cu[b] <= n0 (skips empty sequences)
    int b;
    {
        int lo = 0, hi = L.batch;     // invariant: cu[lo] <= n0 < cu[hi]
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (cu[mid] <= n0) lo = mid; else hi = mid;
        }
        b = lo;
    }
    int seq_end_t = (int)((int64_t)cu[b + 1] - n0);
    const float2 *a_all = reinterpret_cast<const float2 *>(packed + L.off_a);
    // lane l owns channels 2l (low half of its 32-bit load) and 2l+1 (high half)
    float2 a01 = a_all[((int64_t)b * L.n_kv_heads + h) * (SPARK_D / 2) + lane];
    const uint16_t *kbase = k + n0 * k_tok_stride + (int64_t)h * k_head_stride + 2 * lane;

    uint32_t e_lo = 0, e_hi = 0, o_lo = 0, o_hi = 0;     // lane t: ballots of the kept even / odd channels of token t
    uint32_t mu_bits = 0, cnt_reg = 0;                     // lane t: mean pruned saliency, kept count of token t

    uint32_t xnext = *reinterpret_cast<const uint32_t *>(kbase);
    for (int t = 0; t < nvalid; ++t) {
        const uint32_t xx = xnext;
        if (t + 1 < nvalid) xnext = *reinterpret_cast<const uint32_t *>(kbase + (int64_t)(t + 1) * k_tok_stride);
        if (t >= seq_end_t) {       // the tile crosses into the next non-empty sequence
            do {
                ++b;
                seq_end_t = (int)((int64_t)cu[b + 1] - n0);
            } while (t >= seq_end_t);
            a01 = a_all[((int64_t)b * L.n_kv_heads + h) * (SPARK_D / 2) + lane];
        }
        // saliency: one float32 multiply, never fused
        const float w0 = __fmul_rn(a01.x, fabsf(__uint_as_float(xx << 16)));
        const float w1 = __fmul_rn(a01.y, fabsf(__uint_as_float(xx & 0xFFFF0000u)));
        const uint32_t k0 = __float_as_uint(w0), k1 = __float_as_uint(w1);
        // integer saliencies in units of the last place of the row's largest
        const uint32_t kmax = wave_max_u32(k0 > k1 ? k0 : k1);
        int emax = (int)(kmax >> 23);
        emax = emax < 1 ? 1 : emax;
        const uint32_t q0 = quantise(k0, emax), q1 = quantise(k1, emax);
        const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)wave_inclusive_sum(q0 + q1), 63);
        // need = ceil(total * p / 10000) without a 64-bit division: total = 10000 A + B, B * p < 2^27
        const uint32_t tA = total / 10000u, tB = total - tA * 10000u;
        const uint32_t need = tA * (uint32_t)p_bp + (tB * (uint32_t)p_bp + 9999u) / 10000u;

        uint64_t kb0, kb1;
        if (need == 0) {
            // an all-zero row: one channel is kept, the first
            kb0 = 1ull;
            kb1 = 0ull;
        } else {
            // radix selection on sums: theta = the largest bit pattern with sum{q : key >= theta} >= need
            uint32_t theta = 0;      // the bits fixed so far
            uint32_t above = 0;      // sum of q over the keys above every pattern that starts with theta's fixed bits
            auto level = [&](const int sh, const int nbits) __attribute__((always_inline)) -> bool {
                // undecided keys agree with theta above bit sh + nbits; their next digit is (key >> sh) & (2^nbits - 1).
                // Bins are laid out highest digit first, so lane l reads the bin of digit top - l.
                const uint32_t top = (theta >> sh) | ((1u << nbits) - 1u);
                const uint32_t spare = 64u + (uint32_t)lane;
                const uint32_t i0 = top - (k0 >> sh), i1 = top - (k1 >> sh);      // < 2^nbits exactly for the undecided keys
                hist[lane] = 0u;
                prune_lds_sync();
                atomicAdd(&hist[i0 < (1u << nbits) ? i0 : spare], q0);
                atomicAdd(&hist[i1 < (1u << nbits) ? i1 : spare], q1);
                prune_lds_sync();
                const uint32_t c = wave_inclusive_sum(hist[lane]);                // q of undecided keys with digit >= top - lane
                prune_lds_sync();
                const uint64_t reached = __ballot(above + c >= need);            // never empty: the undecided keys reach `need`
                const int l2 = __builtin_ctzll(reached);
                if (l2 > 0) above += (uint32_t)__builtin_amdgcn_readlane((int)c, l2 - 1);
                theta |= (((1u << nbits) - 1u) - (uint32_t)l2) << sh;
                // If one key alone starts with the bits fixed so far, it is the smallest kept one: the levels
                // below would only spell out its remaining bits.  (Usual after two or three levels.)
                const uint64_t in0 = __ballot((k0 >> sh) == (theta >> sh)), in1 = __ballot((k1 >> sh) == (theta >> sh));
                if (__popcll(in0) + __popcll(in1) != 1) return false;
                theta = in0 ? (uint32_t)__builtin_amdgcn_readlane((int)k0, __builtin_ctzll(in0))
                            : (uint32_t)__builtin_amdgcn_readlane((int)k1, __builtin_ctzll(in1 | (1ull << 63)));
                return true;
            };
            // First level: the exponent and two mantissa bits at once (four bins an octave), over the sixteen
            // octaves below the row's largest key.  All of a row's keys share their top bits, so a level on the
            // top six bits alone would drop nearly every key into one or two bins (and serialise the adds);
            // here they spread over some forty.  The window is that long because the cut of a row whose loud
            // channels hold nearly all of its saliency lies among the quiet ones, seven to ten octaves below
            // the largest (an outlier) key.  Keys further down go to the spare words; if the kept sum is not
            // reached inside the window, the row falls back to plain six-bit levels from the top.
            bool done;
            {
                constexpr int kSh = 21;
                const uint32_t dmax = kmax >> kSh;
                const uint32_t spare = 64u + (uint32_t)lane;
                const uint32_t i0 = dmax - (k0 >> kSh), i1 = dmax - (k1 >> kSh);
                hist[lane] = 0u;
                prune_lds_sync();
                atomicAdd(&hist[i0 < 64u ? i0 : spare], q0);
                atomicAdd(&hist[i1 < 64u ? i1 : spare], q1);
                prune_lds_sync();
                const uint32_t c = wave_inclusive_sum(hist[lane]);
                prune_lds_sync();
                const uint64_t reached = __ballot(c >= need);
                if (reached != 0ull) {
                    const int l2 = __builtin_ctzll(reached);
                    if (l2 > 0) above = (uint32_t)__builtin_amdgcn_readlane((int)c, l2 - 1);
                    theta = (dmax - (uint32_t)l2) << kSh;
                    const uint64_t in0 = __ballot((k0 >> kSh) == (theta >> kSh)), in1 = __ballot((k1 >> kSh) == (theta >> kSh));
                    done = (__popcll(in0) + __popcll(in1) == 1);
                    if (done)
                        theta = in0 ? (uint32_t)__builtin_amdgcn_readlane((int)k0, __builtin_ctzll(in0))
                                    : (uint32_t)__builtin_amdgcn_readlane((int)k1, __builtin_ctzll(in1 | (1ull << 63)));
                    else
                        done = level(15, 6) || level(9, 6) || level(3, 6) || level(0, 3);
                } else {
                    done = level(25, 6) || level(19, 6) || level(13, 6) || level(7, 6) || level(1, 6) || level(0, 1);
                }
            }
            (void)done;
            // `above` is now the sum over the keys > theta; the keys == theta (each worth q_theta) fill the rest,
            // lowest channels first
            const bool eq0 = (k0 == theta), eq1 = (k1 == theta);
            const uint64_t m0 = __ballot(eq0), m1 = __ballot(eq1);
            const uint32_t q_theta = quantise(theta, emax);
            int n_tie = 1;
            uint32_t acc = above + q_theta;
            const int n_eq = __popcll(m0) + __popcll(m1);
            while (acc < need && n_tie < n_eq) {
                acc += q_theta;
                ++n_tie;
            }
            // tied channels below 2l: both halves of every lower lane; below 2l+1: plus own even
            const int r0 = mbcnt64(m0) + mbcnt64(m1);
            const int r1 = r0 + (eq0 ? 1 : 0);
            kb0 = __ballot((k0 > theta) || (eq0 && r0 < n_tie));
            kb1 = __ballot((k1 > theta) || (eq1 && r1 < n_tie));
        }
        const bool keep0 = (kb0 >> lane) & 1ull, keep1 = (kb1 >> lane) & 1ull;
        const int cnt = __popcll(kb0) + __popcll(kb1);
        const float psum = wave_total_f32((keep0 ? 0.0f : w0) + (keep1 ? 0.0f : w1));
        const float mu = cnt < SPARK_D ? psum / (float)(SPARK_D - cnt) : 0.0f;
        write_lane1(e_lo, (uint32_t)kb0, t);
        write_lane1(e_hi, (uint32_t)(kb0 >> 32), t);
        write_lane1(o_lo, (uint32_t)kb1, t);
        write_lane1(o_hi, (uint32_t)(kb1 >> 32), t);
        write_lane1(mu_bits, (uint32_t)__builtin_amdgcn_readfirstlane(__float_as_int(mu)), t);
        write_lane1(cnt_reg, (uint32_t)cnt, t);
    }

    // ---- fixed part of the rows, lane = token (rows past the last token: empty mask, count 0)
    const bool valid = lane < nvalid;
    uint8_t *tile_out = packed + L.off_tiles + ((int64_t)h * L.n_tiles + tile) * L.tile_bytes;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    u32x4 m;
    // channel-ordered mask: bit 2l of the row = even ballot bit l, bit 2l+1 = odd ballot bit l
    m.x = valid ? (spread16(e_lo) | (spread16(o_lo) << 1)) : 0u;
    m.y = valid ? (spread16(e_lo >> 16) | (spread16(o_lo >> 16) << 1)) : 0u;
    m.z = valid ? (spread16(e_hi) | (spread16(o_hi) << 1)) : 0u;
    m.w = valid ? (spread16(e_hi >> 16) | (spread16(o_hi >> 16) << 1)) : 0u;
    *reinterpret_cast<u32x4 *>(tile_out + lane * 16) = m;
    u32x2 tail;
    tail.x = valid ? mu_bits : 0u;
    tail.y = valid ? cnt_reg : 0u;
    *reinterpret_cast<u32x2 *>(tile_out + 1024 + lane * 8) = tail;
    // words this tile takes in the head's value stream (every row rounded up to a whole word)
    const uint32_t words = valid ? (cnt_reg + 1u) / 2u : 0u;
    const uint32_t tile_words = (uint32_t)__builtin_amdgcn_readlane((int)wave_inclusive_sum(words), 63);
    if (lane == 0)
        reinterpret_cast<uint32_t *>(packed + L.off_dir)[(int64_t)h * (L.n_tiles + 1) + tile + 1] = tile_words;
    if (wt == 0 && (FULL || full_tiles == 0) && lane < 16) {
        // header (the channel weights are written by the window kernel that runs before)
        uint32_t v = 0;
        if (lane == 0) v = SPARK_MAGIC;
        if (lane == 3) v = (uint32_t)L.batch;
        if (lane == 4) v = (uint32_t)L.n_kv_heads;
        if (lane == 5) v = (uint32_t)L.total_tokens;
        if (lane == 6) v = (uint32_t)L.ndw;
        if (lane == 9) v = 1u;   // top-p cache
        if (lane == 10) v = (uint32_t)p_bp;
        reinterpret_cast<uint32_t *>(packed)[lane] = v;
    }
}

// One block per KV head: dir[h][0] = 0, dir[h][t + 1] = words of tiles 0 .. t (they arrive as per-tile counts).
__global__ __launch_bounds__(256) void spark_topp_scan_kernel(uint8_t *__restrict__ packed, SparkLayout L)
{
    __shared__ uint32_t part[256];
    uint32_t *dir = reinterpret_cast<uint32_t *>(packed + L.off_dir) + (int64_t)blockIdx.x * (L.n_tiles + 1);
    const int64_t n = L.n_tiles;
    const int64_t chunk = (n + 255) / 256;
    const int64_t i0 = (int64_t)threadIdx.x * chunk, i1 = (i0 + chunk < n) ? i0 + chunk : n;
    uint32_t s = 0;
    for (int64_t i = i0; i < i1; ++i) s += dir[i + 1];
    part[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (int i = 0; i < 256; ++i) {
            const uint32_t v = part[i];
            part[i] = run;
            run += v;
        }
        dir[0] = 0u;
    }
    __syncthreads();
    uint32_t run = part[threadIdx.x];
    for (int64_t i = i0; i < i1; ++i) {
        run += dir[i + 1];
        dir[i + 1] = run;
    }
}

// One wavefront per tile.  Lane = token reads the fixed parts (mask, count) and numbers the rows' places in the
// stream (a wave prefix sum of their lengths); then token by token the wavefront reads the dense key row as
// spark_topp_select_kernel did (lane l = channels 2l, 2l+1) and every lane stores its kept entries at the slots
// the mask gives them, so loads and stores both run over contiguous bytes.
__global__ __launch_bounds__(kWaves * 64) void spark_topp_pack_kernel(const uint16_t *__restrict__ k, int64_t k_tok_stride,
                                                                      int64_t k_head_stride, uint8_t *__restrict__ packed,
                                                                      SparkLayout L)
{
    const int lane = threadIdx.x & 63;
    const int64_t wt = (int64_t)blockIdx.x * kWaves + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (wt >= L.n_tiles * L.n_kv_heads) return;
    const int h = (int)(wt / L.n_tiles);
    const int64_t tile = wt % L.n_tiles;
    const int64_t n0 = tile * SPARK_TILE_TOKENS;
    const int64_t left = L.total_tokens - n0;
    const int nvalid = left < SPARK_TILE_TOKENS ? (int)left : SPARK_TILE_TOKENS;
    const uint8_t *tp = packed + L.off_tiles + ((int64_t)h * L.n_tiles + tile) * L.tile_bytes;
    const uint4 mk = *reinterpret_cast<const uint4 *>(tp + lane * 16);
    const uint32_t cnt = *reinterpret_cast<const uint32_t *>(tp + 1024 + lane * 8 + 4);
    const uint32_t words = (cnt + 1u) / 2u;
    const uint32_t before = wave_inclusive_sum(words) - words;       // words of the lower tokens of this tile
    const uint32_t base = reinterpret_cast<const uint32_t *>(packed + L.off_dir)[(int64_t)h * (L.n_tiles + 1) + tile];
    uint16_t *dst_tile = reinterpret_cast<uint16_t *>(reinterpret_cast<uint32_t *>(packed + L.off_vals) +
                                                     (int64_t)h * L.vals_head_words + base);
    const uint16_t *kbase = k + n0 * k_tok_stride + (int64_t)h * k_head_stride + 2 * lane;
    // this lane's two channels are bits 2l, 2l+1 of the 128-bit mask: bits sh, sh+1 of its lower or upper half
    const int sh = (2 * lane) & 63;
    const uint64_t below = (1ull << sh) - 1ull;
    uint32_t xnext = *reinterpret_cast<const uint32_t *>(kbase);
    for (int t = 0; t < nvalid; ++t) {
        const uint32_t xx = xnext;
        if (t + 1 < nvalid) xnext = *reinterpret_cast<const uint32_t *>(kbase + (int64_t)(t + 1) * k_tok_stride);
        const uint64_t lo = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)mk.y, t) << 32) |
                            (uint32_t)__builtin_amdgcn_readlane((int)mk.x, t);
        const uint64_t hi = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)mk.w, t) << 32) |
                            (uint32_t)__builtin_amdgcn_readlane((int)mk.z, t);
        const uint32_t cnt_t = (uint32_t)__builtin_amdgcn_readlane((int)cnt, t);
        uint16_t *dst = dst_tile + 2 * (size_t)(uint32_t)__builtin_amdgcn_readlane((int)before, t);
        const uint64_t mine = lane < 32 ? lo : hi;
        const uint32_t slot0 = (lane < 32 ? 0u : (uint32_t)__popcll(lo)) + (uint32_t)__popcll(mine & below);
        const bool keep0 = (mine >> sh) & 1ull, keep1 = (mine >> (sh + 1)) & 1ull;
        if (keep0) dst[slot0] = (uint16_t)xx;
        if (keep1) dst[slot0 + (keep0 ? 1u : 0u)] = (uint16_t)(xx >> 16);
        if (lane == 0 && (cnt_t & 1u)) dst[cnt_t] = 0;      // the unused half of the row's last word
    }
}

// canonical export, one thread per (token, KV head) row
__global__ void spark_topp_unpack_kernel(const uint8_t *__restrict__ packed, SparkLayout L, uint32_t *mask_out,
                                         int32_t *count_out, uint16_t *vals_out, float *mu_out, float *a_out)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t rows = L.total_tokens * L.n_kv_heads;
    if (a_out && idx < (int64_t)L.batch * L.n_kv_heads * SPARK_D)
        a_out[idx] = reinterpret_cast<const float *>(packed + L.off_a)[idx];
    if (idx >= rows) return;
    const int64_t n = idx / L.n_kv_heads;
    const int h = (int)(idx % L.n_kv_heads);
    const int64_t tile = n / SPARK_TILE_TOKENS;
    const int t = (int)(n % SPARK_TILE_TOKENS);
    const uint8_t *tp = packed + L.off_tiles + ((int64_t)h * L.n_tiles + tile) * L.tile_bytes;
    const uint32_t cnt = *reinterpret_cast<const uint32_t *>(tp + 1024 + t * 8 + 4);
    if (mask_out)
        for (int m = 0; m < 4; ++m) mask_out[idx * 4 + m] = *reinterpret_cast<const uint32_t *>(tp + t * 16 + m * 4);
    if (mu_out) mu_out[idx] = *reinterpret_cast<const float *>(tp + 1024 + t * 8);
    if (count_out) count_out[idx] = (int32_t)cnt;
    if (vals_out) {
        uint32_t before = 0;
        for (int u = 0; u < t; ++u) before += (*reinterpret_cast<const uint32_t *>(tp + 1024 + u * 8 + 4) + 1u) / 2u;
        const uint32_t base = reinterpret_cast<const uint32_t *>(packed + L.off_dir)[(int64_t)h * (L.n_tiles + 1) + tile];
        const uint32_t *src = reinterpret_cast<const uint32_t *>(packed + L.off_vals) + (int64_t)h * L.vals_head_words + base + before;
        uint16_t *o = vals_out + idx * SPARK_D;
        for (uint32_t i = 0; i < (uint32_t)SPARK_D; ++i)
            o[i] = i < cnt ? (uint16_t)((src[i >> 1] >> (16 * (i & 1))) & 0xFFFFu) : (uint16_t)0;
    }
}

// ---------------------------------------------------------------- host-side launch

hipError_t launch_prune_topp(const uint16_t *k, int64_t k_tok_stride, int64_t k_head_stride, const int32_t *cu,
                             uint8_t *packed, const SparkLayout &L, int p_bp, hipStream_t st)
{
    const int64_t full_waves = (L.total_tokens / SPARK_TILE_TOKENS) * L.n_kv_heads;
    const int64_t tail_waves = (L.total_tokens % SPARK_TILE_TOKENS) ? L.n_kv_heads : 0;
    if (full_waves) {
        hipLaunchKernelGGL(spark_topp_select_kernel<true>, dim3((unsigned)((full_waves + kWaves - 1) / kWaves)),
                           dim3(kWaves * 64), 0, st, k, k_tok_stride, k_head_stride, cu, packed, L, p_bp);
        if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    }
    if (tail_waves) {
        hipLaunchKernelGGL(spark_topp_select_kernel<false>, dim3((unsigned)((tail_waves + kWaves - 1) / kWaves)),
                           dim3(kWaves * 64), 0, st, k, k_tok_stride, k_head_stride, cu, packed, L, p_bp);
        if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    }
    if (L.n_tiles == 0) return hipSuccess;
    hipLaunchKernelGGL(spark_topp_scan_kernel, dim3(L.n_kv_heads), dim3(256), 0, st, packed, L);
    if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    const int64_t waves = L.n_tiles * L.n_kv_heads;
    hipLaunchKernelGGL(spark_topp_pack_kernel, dim3((unsigned)((waves + kWaves - 1) / kWaves)), dim3(kWaves * 64), 0, st, k,
                       k_tok_stride, k_head_stride, packed, L);
    return hipGetLastError();
}

hipError_t launch_unpack_topp(const uint8_t *packed, const SparkLayout &L, uint32_t *mask_out, int32_t *count_out,
                              uint16_t *vals_out, float *mu_out, float *a_out, hipStream_t st)
{
    int64_t n = L.total_tokens * L.n_kv_heads;
    const int64_t na = (int64_t)L.batch * L.n_kv_heads * SPARK_D;
    if (a_out && na > n) n = na;
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(spark_topp_unpack_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, packed, L, mask_out,
                       count_out, vals_out, mu_out, a_out);
    return hipGetLastError();
}

}  // namespace spark
