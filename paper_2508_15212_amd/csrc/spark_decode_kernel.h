// Decode attention over the packed (channel-pruned) key cache for gfx950 (wave64).
//
// [Sec. "SparK", "Channel Recovery": pruned entry (n, j) is rebuilt as mu_n / a_j (the
//  degenerate recovery function) and the scores are those of standard attention on the
//  rebuilt keys; Sec. "Preliminaries", Eq. (4): softmax over the cached tokens, then P V.]
//
// The rebuilt key row is never formed.  With d_nj = k_nj - mu_n / a_j for kept channels,
//     <q_g, ktilde_n> = sum_{j kept} q_gj d_nj + mu_n * R_g,   R_g = sum_j q_gj / a_j,
// so a token costs T gathers from a 128-entry table {q_0j .. q_(G-1)j, 1/a_j} held in LDS.
//
// Work decomposition: one block of 4 wavefronts per (batch, KV head, sequence split); each
// wavefront streams whole tiles of 64 tokens.  Per tile:
//   1. lane = token: read the packed row (coalesced, see spark_layout.h), walk its mask
//      bits, accumulate the G scores of the KV head's query group in float32;
//   2. online softmax per query head (running maximum m, per-lane partial sums l);
//   3. probabilities go through LDS into the A operand of the 16x16x32 bf16 MFMA (rows =
//      query heads, K = tokens), split into a high and a low bf16 part so P keeps ~16
//      significant bits; V rows are read 16 bytes per lane, transposed in registers with
//      byte permutes into B operands (K = tokens, N = channels) and accumulated in float32.
// With a channel-pruned VALUE cache (App. "Pruning Value Cache Channels": pruned entries are dropped, i.e.
// contribute 0) step 3 reads packed value rows instead (lane = token, coalesced), parks them in LDS and
// rebuilds the dense 16-byte pieces the MFMA path wants with lane = (token, group of 8 channels): the
// group's mask byte and the number of kept entries before it locate a window of 8 candidates in the
// packed row, and a 256-entry table of byte-permute selectors spreads the candidates to their channels
// (zeros elsewhere).  The cost does not depend on how many entries a row keeps.
// Split partials (m, l, unnormalised output) go to the workspace; the block that arrives last at
// its (batch, KV head) counter merges them and writes the output, so one launch does the step.
// Batches of many short sequences take another decomposition (the balanced mode, see DecodeParams::warm_waves):
// the tiles of a KV head, sequences back to back, are dealt out in equal contiguous ranges to wavefronts that
// work independently of their block - own query table, one partial per sequence touched, the wavefront that
// counts in last merges the pair - so the launch does not last as long as its longest sequence.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spark_kernels.h"
#include "spark_layout.h"

namespace spark {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct DecodeParams {
    const uint16_t *q;       // [B, Hq, 128] bf16
    const uint8_t *packed;   // packed key cache
    const uint16_t *v;       // dense values (NULL when the value cache is packed)
    const uint8_t *packed_v; // packed value cache (value-channel pruning), else NULL
    SparkLayout Lv;          // its layout
    int64_t v_tok_stride, v_head_stride;
    const int32_t *cu;       // [B+1]
    float *part_acc;         // [slots][128]   partial softmax states, see slot numbering below
    float *part_ml;          // [slots][2]     (m in log2 units, l)
    uint32_t *counters;      // [B*Hkv] arrival counters, zero between calls
    unsigned long long *trace;   // NULL, or eight 64-bit words per block of the grid for the timeline (see stamp())
    void *out;               // [B, Hq, 128] bf16 or float32
    int out_f32;
    int Hq, Hkv;
    // How sequences are cut into blocks.  A sequence that spans ntile tiles gets
    //   fixed_splits                           chunks if fixed_splits > 0,
    //   max(1, ceil(ntile / chunk_tiles))      chunks otherwise (long sequences get more blocks than short ones),
    // chunks are numbered through the batch (global chunk id), block = (global chunk, KV head); the host
    // launches nchunk_max >= the true count and blocks past the last chunk leave at once.
    // Slot of (global chunk c, q head) = c * Hq + head; the appended rows' slots follow at tail_base:
    // ((b * Hq + head) * tail_slots + part).
    int fixed_splits, chunk_tiles, nchunk_max;
    // Balanced mode (warm_waves > 0; ragged batches of many short sequences): the (sequence, tile) items of a KV
    // head, sequences back to back, are dealt out in equal contiguous ranges to warm_waves wavefronts, each of
    // which works on its own and leaves one partial per sequence it touches.  Wavefront w covers items
    // [w * I / warm_waves, (w + 1) * I / warm_waves) of the I items; the partial of (wavefront w, sequence b) has
    // chunk id w + b (both grow along the item list, so the ids of one sequence are consecutive and no two
    // pairs share one); a sequence without tokens has the single id warm_waves + batch + b: warm_waves + 2 * batch
    // ids in all.
    int warm_waves;
    int ntail;               // blocks per (batch, KV head) for the appended rows, 256 rows each (0: none)
    int tail_slots;          // slots reserved per (batch, q head) for them (>= max(1, ntail))
    int64_t tail_base;       // first of them: the number of chunk ids the workspace provides for, times Hq
    const uint16_t *tail_k, *tail_v;   // appended never-pruned rows [B, tail_cap, Hkv, 128] bf16, or NULL
    const int32_t *tail_len;           // [B]
    int tail_cap;
    int rec;                           // 0: degenerate recovery; 1 Gaussian, 2 Exponential (sampled)
    uint32_t seed_lo, seed_hi;         // seed of the sampled recovery
    float scale_log2;        // softmax scale * log2(e)
    SparkLayout L;
};

constexpr int kDecodeWaves = 4;

__device__ __forceinline__ void wave_lds_sync()
{
    // LDS operations of one wavefront execute in order; this only stops the compiler from
    // moving accesses across the point where lanes exchange data through LDS.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Maximum over the 64 lanes, returned wave-uniform.  Data-parallel-primitive moves: two quad
// permutes and two row rotates leave each row of 16 lanes holding its row maximum, two row
// broadcasts fold the four rows into lane 63.  Lanes a step does not address keep their value.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_max_step(float x)
{
    const int xi = __float_as_int(x);
    const float y = __int_as_float(__builtin_amdgcn_update_dpp(xi, xi, CTRL, ROW_MASK, 0xF, false));
    return fmaxf(x, y);
}

__device__ __forceinline__ float wave_max(float x)
{
    x = dpp_max_step<0xB1, 0xF>(x);    // quad_perm [1,0,3,2]
    x = dpp_max_step<0x4E, 0xF>(x);    // quad_perm [2,3,0,1]
    x = dpp_max_step<0x124, 0xF>(x);   // row_ror 4
    x = dpp_max_step<0x128, 0xF>(x);   // row_ror 8
    x = dpp_max_step<0x142, 0xA>(x);   // row_bcast 15 into rows 1 and 3
    x = dpp_max_step<0x143, 0xC>(x);   // row_bcast 31 into rows 2 and 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

// Sum over the 64 lanes, returned wave-uniform.  Data-parallel-primitive moves (shifts by 1, 2, 4, 8 inside each
// row of 16 lanes, then two row broadcasts) leave the total in lane 63; no LDS round trips.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add_step(float x)
{
    return x + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, ROW_MASK, 0xF, false));
}

__device__ __forceinline__ float wave_sum(float x)
{
    x = dpp_add_step<0x111, 0xF>(x);   // row_shr 1
    x = dpp_add_step<0x112, 0xF>(x);   // row_shr 2
    x = dpp_add_step<0x114, 0xF>(x);   // row_shr 4
    x = dpp_add_step<0x118, 0xF>(x);   // row_shr 8
    x = dpp_add_step<0x142, 0xA>(x);   // row_bcast 15 -> rows 1, 3
    x = dpp_add_step<0x143, 0xC>(x);   // row_bcast 31 -> rows 2, 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

// device-scope (all XCDs) relaxed store / load of one float
__device__ __forceinline__ void st_agent(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ uint32_t u4c(const uint4 &v, int c) { return c == 0 ? v.x : c == 1 ? v.y : c == 2 ? v.z : v.w; }
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }   // v_exp_f32; exp2(-inf) = 0
__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// Inclusive prefix sum over the 64 lanes (data-parallel-primitive moves: shifts by 1, 2, 4, 8 inside each row
// of 16 lanes, then the last lane of row 0 / 2 into row 1 / 3 and the last lane of row 1 into rows 2, 3).
__device__ __forceinline__ int wave_inclusive_sum_i32(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, false);   // row_shr 1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, false);   // row_shr 2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, false);   // row_shr 4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, false);   // row_shr 8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);   // row_bcast 15 -> rows 1, 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);   // row_bcast 31 -> rows 2, 3
    return v;
}

struct SeqChunks { int b, first, n, s0, s1; };   // sequence, global id of its first chunk, number of its chunks
                                                  // (0: none), its token range

// Finds the sequence that owns global chunk `gid` (want_b < 0) or describes sequence `want_b`.  Every lane of
// the wavefront calls it with the same arguments and gets the same answer: 64 sequences are sized per step
// (lane = sequence) and a wave prefix sum numbers their chunks.
__device__ __forceinline__ SeqChunks locate_chunks(const DecodeParams &P, int B, int gid, int want_b, int lane)
{
    SeqChunks r = {0, 0, 0, 0, 0};
    if (P.fixed_splits > 0) {
        const int b = (want_b >= 0) ? want_b : gid / P.fixed_splits;
        if (b < B) { r.b = b; r.first = b * P.fixed_splits; r.n = P.fixed_splits; r.s0 = P.cu[b]; r.s1 = P.cu[b + 1]; }
        return r;
    }
    int base = 0;
    for (int b0 = 0; b0 < B; b0 += 64) {
        const int bb = b0 + lane;
        int n = 0, s0 = 0, s1 = 0;
        if (bb < B) {
            s0 = P.cu[bb];
            s1 = P.cu[bb + 1];
            const int ntile = (s1 > s0) ? ((s1 - 1) / SPARK_TILE_TOKENS - s0 / SPARK_TILE_TOKENS + 1) : 0;
            n = (ntile + P.chunk_tiles - 1) / P.chunk_tiles;
            n = n < 1 ? 1 : n;     // an empty sequence still gets one block: somebody has to write its zeros
        }
        const int inc = wave_inclusive_sum_i32(n);
        uint64_t hit;
        if (want_b >= 0)
            hit = (want_b >= b0 && want_b < b0 + 64) ? (1ull << (want_b - b0)) : 0ull;
        else
            hit = __ballot(base + inc > gid);
        if (hit != 0ull) {
            const int l = __builtin_ctzll(hit);
            const int nn = __builtin_amdgcn_readlane(n, l), ii = __builtin_amdgcn_readlane(inc, l);
            r.b = b0 + l;
            r.first = base + ii - nn;
            r.n = nn;
            r.s0 = __builtin_amdgcn_readlane(s0, l);
            r.s1 = __builtin_amdgcn_readlane(s1, l);
            return r;
        }
        base += __builtin_amdgcn_readlane(inc, 63);
    }
    return r;
}

// ---------------------------------------------------------------- balanced mode: the batch as a list of items

// The batch's sequences in registers, lane = sequence 64 k + lane (the mode takes at most 256 sequences): token
// range and the number of items (tiles spanned; none for a sequence without tokens) up to and including the
// sequence.  Every lane of a wavefront builds the same table.
struct WarmSeqs {
    int s0[4], s1[4], inc[4];
    int total;
};
struct WarmSeq { int b, s0, s1, n, first_item; };
struct PairInfo { int b, first, nsplit; };   // sequence, chunk id of its first partial, number of its partials

__device__ __forceinline__ WarmSeqs warm_load(const DecodeParams &P, int B, int lane)
{
    WarmSeqs W;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int bb = 64 * k + lane;
        W.s0[k] = W.s1[k] = 0;
        if (bb < B) { W.s0[k] = P.cu[bb]; W.s1[k] = P.cu[bb + 1]; }
    }
    int base = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int n = (W.s1[k] > W.s0[k]) ? ((W.s1[k] - 1) / SPARK_TILE_TOKENS - W.s0[k] / SPARK_TILE_TOKENS + 1) : 0;
        W.inc[k] = base + wave_inclusive_sum_i32(n);
        base = __builtin_amdgcn_readlane(W.inc[k], 63);
    }
    W.total = base;
    return W;
}

// entry of sequence b (wave-uniform b)
__device__ __forceinline__ WarmSeq warm_get(const WarmSeqs &W, int b)
{
    const int k = b >> 6, l = b & 63;
    // (values, not references to the arrays: the table stays in registers)
    auto pick = [k, l](int a0, int a1, int a2, int a3) {
        int v = a0;
        v = (k == 1) ? a1 : v;
        v = (k == 2) ? a2 : v;
        v = (k == 3) ? a3 : v;
        return __builtin_amdgcn_readlane(v, l);
    };
    WarmSeq q;
    q.b = b;
    q.s0 = pick(W.s0[0], W.s0[1], W.s0[2], W.s0[3]);
    q.s1 = pick(W.s1[0], W.s1[1], W.s1[2], W.s1[3]);
    q.n = (q.s1 > q.s0) ? ((q.s1 - 1) / SPARK_TILE_TOKENS - q.s0 / SPARK_TILE_TOKENS + 1) : 0;
    q.first_item = pick(W.inc[0], W.inc[1], W.inc[2], W.inc[3]) - q.n;
    return q;
}

// the sequence that holds item `item` (0 <= item < W.total)
__device__ __forceinline__ WarmSeq warm_find(const WarmSeqs &W, int item)
{
    int b = 0;
    bool found = false;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint64_t hit = __ballot(W.inc[k] > item);
        if (!found && hit != 0ull) { b = 64 * k + __builtin_ctzll(hit); found = true; }
    }
    return warm_get(W, b);
}

// wavefront w of nw covers items [w * total / nw, (w + 1) * total / nw): the one that covers `item`
__device__ __forceinline__ int warm_wave_of(int item, int nw, int total)
{
    return (int)((((uint32_t)item + 1u) * (uint32_t)nw - 1u) / (uint32_t)total);
}

// Partials of sequence q: one per wavefront that covers some of its items.  `nwe` is the number of wavefronts that
// take part, min(warm_waves, total): with fewer items than wavefronts each of the first `total` takes one.
__device__ __forceinline__ PairInfo warm_pair(const DecodeParams &P, const WarmSeq &q, int B, int total)
{
    PairInfo pi;
    pi.b = q.b;
    if (q.n > 0) {
        const int nwe = P.warm_waves < total ? P.warm_waves : total;
        const int wf = warm_wave_of(q.first_item, nwe, total);
        const int wl = warm_wave_of(q.first_item + q.n - 1, nwe, total);
        pi.first = wf + q.b;
        pi.nsplit = wl - wf + 1;
    } else {
        pi.first = P.warm_waves + B + q.b;
        pi.nsplit = 1;
    }
    return pi;
}

// ---------------------------------------------------------------- appended (never pruned) rows

// [Sec. "Preliminaries": each decode step concatenates the new token's key and value to the cache; pruning
//  happens once, at prefill, so these rows stay dense.]  One extra block per (batch, KV head) of the decode
// grid runs plain attention over the sequence's appended rows and leaves the softmax state (m, l,
// unnormalised output) in the spare partial slot; it then takes part in the arrival count like a sequence
// split, so whichever block comes last folds it in.  qs [G][128] and Psh [4][G][64] are LDS scratch.
template <int G>
__device__ __forceinline__ void tail_partial(const DecodeParams &P, int b, int h, int part, float *qs, float *Psh,
                                             float (*red_m)[G], float (*red_l)[G], float *red_acc /* [4][G][128] */)
{
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int len = P.tail_len[b];
    len = len < 0 ? 0 : (len > P.tail_cap ? P.tail_cap : len);
    // this block's share: rows [256 * part, 256 * part + 256)
    const int first = part * kDecodeWaves * 64;
    len = (len < first + kDecodeWaves * 64) ? len : first + kDecodeWaves * 64;
    for (int idx = tid; idx < G * SPARK_D; idx += kDecodeWaves * 64) {
        const int g = idx / SPARK_D, j = idx % SPARK_D;
        qs[g * SPARK_D + j] = bf16lo(P.q[((int64_t)b * P.Hq + h * G + g) * SPARK_D + j]) * P.scale_log2;
    }
    __syncthreads();
    float m[G], l[G], acc[G][2];
#pragma unroll
    for (int g = 0; g < G; ++g) { m[g] = -INFINITY; l[g] = 0.0f; acc[g][0] = acc[g][1] = 0.0f; }
    const int64_t row0 = (int64_t)b * P.tail_cap;
    float *pw = Psh + wave * G * 64;
    for (int c0 = first + wave * 64; c0 < len; c0 += kDecodeWaves * 64) {   // (one pass)
        // scores, lane = token
        const int t = c0 + lane;
        const bool valid = t < len;
        const uint16_t *krow = P.tail_k + ((row0 + (valid ? t : len - 1)) * P.Hkv + h) * SPARK_D;
        float s[G];
#pragma unroll
        for (int g = 0; g < G; ++g) s[g] = 0.0f;
#pragma unroll 4
        for (int c = 0; c < SPARK_D / 8; ++c) {
            const uint4 x = *reinterpret_cast<const uint4 *>(krow + 8 * c);
            const float kf[8] = {bf16lo(x.x), bf16hi(x.x), bf16lo(x.y), bf16hi(x.y),
                                 bf16lo(x.z), bf16hi(x.z), bf16lo(x.w), bf16hi(x.w)};
#pragma unroll
            for (int e = 0; e < 8; ++e)
#pragma unroll
                for (int g = 0; g < G; ++g) s[g] = fmaf(qs[g * SPARK_D + 8 * c + e], kf[e], s[g]);
        }
        // online softmax (log2 domain); probabilities to LDS
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float sg = valid ? s[g] : -INFINITY;
            const float mnew = fmaxf(m[g], wave_max(sg));          // finite: lane 0 of the chunk is valid
            const float alpha = fast_exp2(m[g] - mnew);             // m = -inf -> 0
            const float p = fast_exp2(sg - mnew);
            m[g] = mnew;
            l[g] = fmaf(l[g], alpha, p);
            acc[g][0] *= alpha;
            acc[g][1] *= alpha;
            pw[g * 64 + lane] = p;
        }
        wave_lds_sync();
        // weighted sum, lane = channels 2l, 2l+1; eight value rows in flight
        const int nval = (len - c0 < 64) ? (len - c0) : 64;
        const uint16_t *vbase = P.tail_v + ((row0 + c0) * P.Hkv + h) * SPARK_D + 2 * lane;
        const int64_t vstep = (int64_t)P.Hkv * SPARK_D;
        for (int t0 = 0; t0 < nval; t0 += 8) {
            uint32_t vw[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int tt = (t0 + u < nval) ? (t0 + u) : (nval - 1);
                vw[u] = *reinterpret_cast<const uint32_t *>(vbase + tt * vstep);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const bool on = t0 + u < nval;
                const float v0 = bf16lo(vw[u]), v1 = bf16hi(vw[u]);
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const float p = on ? pw[g * 64 + ((t0 + u) & 63)] : 0.0f;
                    acc[g][0] = fmaf(p, v0, acc[g][0]);
                    acc[g][1] = fmaf(p, v1, acc[g][1]);
                }
            }
        }
        wave_lds_sync();
    }
    // merge the wavefronts and write the partial (device-scope stores, as the sequence splits do)
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const float lt = wave_sum(l[g]);
        if (lane == 0) { red_m[wave][g] = m[g]; red_l[wave][g] = lt; }
        red_acc[(wave * G + g) * SPARK_D + 2 * lane] = acc[g][0];
        red_acc[(wave * G + g) * SPARK_D + 2 * lane + 1] = acc[g][1];
    }
    __syncthreads();
    for (int idx = tid; idx < G * SPARK_D; idx += kDecodeWaves * 64) {
        const int g = idx / SPARK_D, ch = idx % SPARK_D;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < kDecodeWaves; ++w) M = fmaxf(M, red_m[w][g]);
        const float Ms = (M == -INFINITY) ? 0.0f : M;
        float Lsum = 0.0f, A = 0.0f;
#pragma unroll
        for (int w = 0; w < kDecodeWaves; ++w) {
            const float f = fast_exp2(red_m[w][g] - Ms);
            Lsum = fmaf(red_l[w][g], f, Lsum);
            A = fmaf(red_acc[(w * G + g) * SPARK_D + ch], f, A);
        }
        const int64_t slot = P.tail_base + ((int64_t)b * P.Hq + h * G + g) * P.tail_slots + part;
        st_agent(&P.part_acc[slot * SPARK_D + ch], A);
        if (ch == 0) { st_agent(&P.part_ml[slot * 2], M); st_agent(&P.part_ml[slot * 2 + 1], Lsum); }
    }
}

// resident blocks per compute unit the register budget is held to (three was measured no faster
// than two and spills once the table gathers are batched)
constexpr int decode_min_blocks(int, int) { return 2; }
// The cache is read once per step: the streaming loads carry the non-temporal hint so they do not
// displace each other in the L2 / memory-side cache (measured: 129 us -> 118 us on the 32K workload).
#define NT_LOAD(p) __builtin_nontemporal_load(p)

// Timeline of a launch (a measurement aid, off unless a buffer has been given through spark_decode_timeline):
// thread 0 of every block files the 100 MHz wall clock at five points - word 0 entry, 1 start of streaming,
// 2 end of streaming (wavefront 0), 3 partial stored, 4 exit - and, with word 5, its tile count (in the balanced
// mode: 1 << 32 | tiles of wavefront 0), 6 the hardware ids (XCC id << 32 | HW_ID), 7 whether it merged a
// (batch, KV head) pair.
__device__ __forceinline__ void stamp(const DecodeParams &P, int word, unsigned long long value)
{
    if (P.trace != nullptr && threadIdx.x == 0) P.trace[(size_t)blockIdx.x * 8 + word] = value;
}
// TVC: 0 = dense values; > 0 = packed values with that many kept channels per row (row held in registers);
// -1 = packed values, any count (row words read from memory as they are needed).
// REC: 0 = degenerate recovery (mu / a, folded into the score sum); 1 / 2 = Gaussian / Exponential recovery:
// a saliency is drawn for every pruned entry from the row's all-channel statistics with a counter-based
// generator keyed by (seed, token, head, channel), so the run can be repeated and checked.
// VAR: rows keep a per-row number of channels (the top-p variant, Sec. "Adaptive Variants of SparK"): the row's
// count sits in its sixth word and the kept entries in the head's value stream, located through the tile
// directory and a wave prefix sum of the lower tokens' lengths.
// WARM: balanced mode (see DecodeParams::warm_waves): the four wavefronts of a block work independently, each with
// its own query table, on a contiguous range of (sequence, tile) items; nothing in a block waits for another
// wavefront, and a sequence boundary inside a range costs one partial store and one table rebuild while the
// next tile is already in flight.
template <int G, int TCT, int INT8, int TVC, int REC = 0, int VAR = 0, int WARM = 0>
__global__ __launch_bounds__(kDecodeWaves * 64, decode_min_blocks(G, TCT)) void spark_decode_kernel(DecodeParams P)
{
    static_assert(!VAR || (TCT == 0 && INT8 == 0 && TVC == 0 && REC == 0), "variable-length rows: any-length bf16 path only");
    static_assert(!WARM || (TVC == 0 && REC == 0 && VAR == 0 && G <= 8), "balanced mode: dense values, degenerate recovery");
    constexpr bool PV = (TVC != 0);             // packed value cache
    constexpr int NVW = PV ? (TVC > 0 ? (((4 + (TVC + 1) / 2) + 1) & ~1) : 4) : 1;   // value-row words in registers
    // LDS row stride (words) of a parked value row.  A row kept whole in registers (NVW words) is parked word by
    // word at an ODD stride: the four tokens whose windows a wavefront reads together then start in banks of both
    // parities (with an even stride the window offsets, which advance by about two words per group, fell on even
    // banks only: 104 instead of 113 us at 26 kept value channels on the 32K shape, no change at 64).  Rows of any
    // length are read from memory in 16-byte pieces and keep a stride that is 4 mod 8; the longest is 68 words.
    constexpr int RSV = PV ? (TVC > 0 ? (NVW | 1) : 68) : 1;
    // floats per table entry: G queries, 1/a, pad -- a multiple of 4 (16-byte gathers) that is 4 mod 8, so
    // that the entries of different channels start in all eight 16-byte bank groups, not in half of them
    constexpr int GP = 8 * ((G + 1 + 3) / 8) + 4;
    constexpr int VAL0 = INT8 ? 6 : 5;
    constexpr int NV_CT = INT8 ? (TCT + 3) / 4 : (TCT + 1) / 2;
    constexpr int NDW_CT = (VAL0 + NV_CT + 1) & ~1;
    constexpr int NQ_CT = NDW_CT / 4;

    __shared__ __align__(16) float qtab[(WARM ? kDecodeWaves : 1) * SPARK_D * GP];   // (balanced mode: one per wavefront)
    __shared__ float Rsh[16];
    __shared__ __align__(16) uint16_t Pbuf[kDecodeWaves][2][G][64];
    // per wavefront: the accumulators at the end; with packed values, before that, the parked value rows
    // (+ slack: the candidate window may read 4 words past a row)
    constexpr int RED_BYTES = G * SPARK_D * 4, RAW_BYTES = (SPARK_TILE_TOKENS * RSV + 8) * 4;
    constexpr int WBUF = (PV && RAW_BYTES > RED_BYTES) ? RAW_BYTES : RED_BYTES;
    __shared__ __align__(16) uint8_t wbuf[kDecodeWaves][WBUF];
    // packed values: per token 16 x {kept entries before the group, the group's mask byte}; the selector
    // table in two arrays (four words and two words per entry, each read with one aligned access: either array's
    // entries then tile all 32 banks; one array of 12-word entries left half the banks idle on the short read)
    __shared__ __align__(16) uint32_t vmeta[PV ? kDecodeWaves : 1][PV ? SPARK_TILE_TOKENS * 8 : 1];
    __shared__ __align__(16) uint32_t vlut[PV ? 256 * 4 : 1];
    __shared__ __align__(16) uint32_t vlutb[PV ? 256 * 2 : 1];
    __shared__ float red_m[kDecodeWaves][G], red_l[kDecodeWaves][G];
    __shared__ int last_flag;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keep tile addressing scalar
    if (P.trace != nullptr) {
        stamp(P, 0, wall_clock64());
        stamp(P, 6, ((unsigned long long)__builtin_amdgcn_s_getreg(20 | (31 << 11)) << 32) |     // XCC_ID
                        (unsigned long long)__builtin_amdgcn_s_getreg(4 | (31 << 11)));              // HW_ID
        stamp(P, 7, 0ull);
    }
    const SparkLayout &L = P.L;
    const int T = TCT ? TCT : L.T;
    // blocks [0, nmain) stream the cache: (global chunk, KV head) pairs, or in the balanced mode (group of four
    // wavefronts, KV head); when rows have been appended after prefill, B * Hkv * ntail more blocks follow, each
    // taking 256 of a (batch, KV head)'s appended rows
    const int nmain = (WARM ? P.warm_waves / kDecodeWaves : P.nchunk_max) * P.Hkv;
    const bool is_tail = (int)blockIdx.x >= nmain;      // block-uniform
    const int tb = (int)blockIdx.x - nmain;
    const int gid = is_tail ? -1 : (int)(blockIdx.x / P.Hkv);
    const int h = is_tail ? (tb / P.ntail) % P.Hkv : (int)(blockIdx.x % P.Hkv);
    WarmSeqs W;
    PairInfo pi = {0, 0, 0};
    int s0 = 0, s1 = 0;                                  // token range of the sequence being streamed
    int split = 0;                                       // this block's (wavefront's) partial within its sequence
    float *const qt = qtab + (WARM ? wave * SPARK_D * GP : 0);
    if constexpr (WARM) {
        W = warm_load(P, L.batch, lane);
        if (is_tail) pi = warm_pair(P, warm_get(W, (tb / P.ntail) / P.Hkv), L.batch, W.total);
    } else {
        const SeqChunks sc = locate_chunks(P, L.batch, gid, is_tail ? (tb / P.ntail) / P.Hkv : -1, lane);
        if (sc.n == 0) return;                           // past the last chunk: the whole block leaves
        pi.b = sc.b;
        pi.first = sc.first;
        pi.nsplit = sc.n;                                // chunks of this sequence
        split = is_tail ? 0 : gid - sc.first;            // this block's chunk within its sequence
        s0 = sc.s0;
        s1 = sc.s1;
    }
    // partial slot of (q head index within the batch element's heads, i-th partial of a (batch, KV head))
    auto slot_of = [&](const PairInfo &pr, int qh, int i) -> int64_t {
        return (i < pr.nsplit) ? (int64_t)(pr.first + i) * P.Hq + qh
                               : P.tail_base + ((int64_t)pr.b * P.Hq + qh) * P.tail_slots + (i - pr.nsplit);
    };
    // Folds the nmerge partial states of pair pr for query head h * G + g and writes the output (one wavefront;
    // lane l takes the output channels 2l, 2l+1).  Up to 64 partial states are folded per round with the
    // running-maximum rule: lane i fetches the (m, l) pair of partial i - one 8-byte load per lane, the pair's
    // factor exp2(m_i - M) is then handed out by readlane - while every lane fetches its accumulator pair of
    // all the partials (64 independent 8-byte loads in flight; the accumulators of the main loop are dead
    // there, so the registers are there).  All loads are device-scope.  A pair with up to 64 partials is
    // merged in one memory round trip.
    auto merge_head = [&](const PairInfo &pr, int nmerge, int g) {
        constexpr int RN = 64;                   // partials per round
        const int c2 = lane;
        const int qh = h * G + g;
        const uint64_t *pa = reinterpret_cast<const uint64_t *>(P.part_acc + 2 * c2);
        const uint64_t *pm = reinterpret_cast<const uint64_t *>(P.part_ml);
        float M = -INFINITY, Lsum = 0.0f, A0 = 0.0f, A1 = 0.0f;
        for (int i0 = 0; i0 < nmerge; i0 += RN) {
            const int n = (nmerge - i0 < RN) ? nmerge - i0 : RN;
            float mi = -INFINITY, li = 0.0f;
            if (lane < n) {
                const uint64_t ml = __hip_atomic_load(pm + slot_of(pr, qh, i0 + lane), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                mi = __uint_as_float((uint32_t)ml);
                li = __uint_as_float((uint32_t)(ml >> 32));
            }
            uint64_t av[RN];
#pragma unroll
            for (int k0 = 0; k0 < RN; k0 += 8) {
                if (k0 < n) {                                      // (wave-uniform: whole groups of eight are skipped)
#pragma unroll
                    for (int k = k0; k < k0 + 8; ++k) {
                        const int i = i0 + ((k < n) ? k : n - 1);  // (past the batch: some valid slot, its factor is 0)
                        av[k] = __hip_atomic_load(pa + slot_of(pr, qh, i) * (SPARK_D / 2), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                } else {
#pragma unroll
                    for (int k = k0; k < k0 + 8; ++k) av[k] = 0ull;
                }
            }
            const float Mn = fmaxf(M, wave_max(mi));
            const float Ms = (Mn == -INFINITY) ? 0.0f : Mn;
            const float fo = fast_exp2(M - Ms);               // M = -inf -> 0
            M = Mn;
            const float fi = fast_exp2(mi - Ms);              // lane i: factor of partial i0 + i (0 past the batch)
            Lsum = fmaf(Lsum, fo, wave_sum(li * fi));
            A0 *= fo;
            A1 *= fo;
#pragma unroll
            for (int k0 = 0; k0 < RN; k0 += 8) {
                if (k0 < n) {
#pragma unroll
                    for (int k = k0; k < k0 + 8; ++k) {
                        const float f = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(fi), k));
                        A0 = fmaf(__uint_as_float((uint32_t)av[k]), f, A0);
                        A1 = fmaf(__uint_as_float((uint32_t)(av[k] >> 32)), f, A1);
                    }
                }
            }
        }
        const int64_t bq = (int64_t)pr.b * P.Hq + qh;
        const float o0 = (Lsum > 0.0f) ? (A0 / Lsum) : 0.0f, o1 = (Lsum > 0.0f) ? (A1 / Lsum) : 0.0f;
        if (P.out_f32) {
            reinterpret_cast<float2 *>(P.out)[bq * (SPARK_D / 2) + c2] = make_float2(o0, o1);
        } else {
            const uint32_t packed2 = (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)o0) |
                                     ((uint32_t)__builtin_bit_cast(uint16_t, (__bf16)o1) << 16);
            reinterpret_cast<uint32_t *>(P.out)[bq * (SPARK_D / 2) + c2] = packed2;
        }
    };
    const int b = pi.b;
    const int nsplit = pi.nsplit;
    const int nmerge = nsplit + P.ntail;                 // partial states the last arrival folds
    if (is_tail) {
        static_assert(sizeof(qtab) >= G * SPARK_D * 4 && sizeof(Pbuf) >= kDecodeWaves * G * 64 * 4, "LDS reuse");
        tail_partial<G>(P, b, h, tb % P.ntail, qtab, reinterpret_cast<float *>(&Pbuf[0][0][0][0]), red_m, red_l,
                        reinterpret_cast<float *>(&wbuf[0][0]));
    } else {
    float m[G], l[G], R[G];
    f32x4 acc[8];
#pragma unroll
    for (int g = 0; g < G; ++g) { m[g] = -INFINITY; l[g] = 0.0f; }
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int tg = lane >> 4, cn = lane & 15;
    // slot of this lane's token in the P buffer: MFMA lane group tg' = token % 4 holds, as its K
    // index i, token 32*ks + 4*i + tg' (the same order in which V rows are fetched)
    const int ppos = (lane & 32) | ((lane & 3) << 3) | ((lane & 31) >> 2);
    const uint8_t *tiles = P.packed + L.off_tiles + (int64_t)h * L.n_tiles * L.tile_bytes;
    const uint16_t *vbase = PV ? nullptr : P.v + (int64_t)h * P.v_head_stride + cn * 8;
    const SparkLayout &Lv = P.Lv;
    const uint8_t *vtiles = PV ? P.packed_v + Lv.off_tiles + (int64_t)h * Lv.n_tiles * Lv.tile_bytes : nullptr;
    const int rsv = (TVC > 0) ? RSV : 8 * ((Lv.ndw + 3) / 8) + 4;   // parked-row stride in words

    // Rows of any length: value words [w_lo, w_hi) of the row, fetched in the 16-byte sections they are stored
    // in, NLD sections (a batch) per request.  The first batch is requested with the row's fixed words.
    constexpr int NLD = 2;
    constexpr int per_word = INT8 ? 4 : 2;          // entries per value word
    const int w_lo = L.val0, w_hi = L.val0 + (T + per_word - 1) / per_word;
    auto load_batch = [&](int tile, int qd0, u32x4 (&wv)[NLD]) {
        const uint8_t *tp = tiles + (int64_t)tile * L.tile_bytes;
#pragma unroll
        for (int u = 0; u < NLD; ++u) {
            const int qd = qd0 + u;
            wv[u] = u32x4{0u, 0u, 0u, 0u};
            if (4 * qd < w_hi) {
                if (qd < L.nq) {
                    wv[u] = NT_LOAD(reinterpret_cast<const u32x4 *>(tp + qd * 1024 + lane * 16));
                } else {                           // the 2-word section at the end of the row
                    const uint2 x = *reinterpret_cast<const uint2 *>(tp + L.nq * 1024 + lane * 8);
                    wv[u].x = x.x;
                    wv[u].y = x.y;
                }
            }
        }
    };
    u32x4 wfirst[(TCT || VAR) ? 1 : NLD];            // (any length, fixed per cache: the first batch of the tile in flight)
    constexpr int NR = TCT ? NDW_CT : 6;    // row words held in registers
    auto load_row = [&](int tile, uint32_t (&r)[NR]) {
        const uint8_t *tp = tiles + (int64_t)tile * L.tile_bytes;
        if (TCT) {
#pragma unroll
            for (int qd = 0; qd < NQ_CT; ++qd) {
                const u32x4 x = NT_LOAD(reinterpret_cast<const u32x4 *>(tp + qd * 1024 + lane * 16));
                r[4 * qd + 0] = x.x; r[4 * qd + 1] = x.y; r[4 * qd + 2] = x.z; r[4 * qd + 3] = x.w;
            }
            if (NDW_CT % 4) {
                const uint2 x = *reinterpret_cast<const uint2 *>(tp + NQ_CT * 1024 + lane * 8);
                r[4 * NQ_CT + 0] = x.x; r[4 * NQ_CT + 1] = x.y;
            }
        } else {
#pragma unroll
            for (int d = 0; d < 6; ++d)
                r[d] = *reinterpret_cast<const uint32_t *>(tp + spark_tile_word_offset(L, lane, d));
            if constexpr (!TCT && !VAR && G <= 8) load_batch(tile, w_lo >> 2, wfirst);
        }
    };
    // half a tile of V: lane (tg, cn) takes 16 bytes (channels 8cn..8cn+7) of rows 4i + tg, so that
    // one load instruction of the wavefront covers 4 consecutive rows (1 KB when rows are contiguous)
    auto load_v = [&](int tile, int ks, uint4 (&vh)[8]) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            int n = tile * SPARK_TILE_TOKENS + 32 * ks + 4 * i + tg;
            n = (n < s0) ? s0 : n;
            n = (n > s1 - 1) ? (s1 - 1) : n;     // rows outside the sequence get p = 0
            const u32x4 x = NT_LOAD(reinterpret_cast<const u32x4 *>(vbase + (int64_t)n * P.v_tok_stride));
            vh[i] = make_uint4(x.x, x.y, x.z, x.w);
        }
    };

    // packed value row of this lane's token: mask words, then the kept entries (coalesced sections as for keys)
    auto load_vrow = [&](int tile, uint32_t (&r)[NVW]) {
        const uint8_t *tp = vtiles + (int64_t)tile * Lv.tile_bytes;
        if (TVC > 0) {
#pragma unroll
            for (int qd = 0; qd < NVW / 4; ++qd) {
                const u32x4 x = NT_LOAD(reinterpret_cast<const u32x4 *>(tp + qd * 1024 + lane * 16));
                r[4 * qd + 0] = x.x; r[4 * qd + 1] = x.y; r[4 * qd + 2] = x.z; r[4 * qd + 3] = x.w;
            }
            if (NVW % 4) {
                const uint2 x = *reinterpret_cast<const uint2 *>(tp + (NVW / 4) * 1024 + lane * 8);
                r[4 * (NVW / 4) + 0] = x.x; r[4 * (NVW / 4) + 1] = x.y;
            }
        } else {
            const u32x4 x = NT_LOAD(reinterpret_cast<const u32x4 *>(tp + lane * 16));   // the mask
            r[0] = x.x; r[1] = x.y; r[2] = x.z; r[3] = x.w;
        }
    };

    // A wavefront keeps one tile in flight: the loads of tile i+1 are issued when tile i is done.
    // (Requesting further ahead was measured slower: more outstanding requests per wavefront cost
    // more in DRAM efficiency than the extra overlap gained.)
    uint32_t rn[NR];
    uint4 vr[2][8];
    uint32_t vrow[NVW];
    auto prefetch = [&](int tile) {
        load_row(tile, rn);
        if constexpr (PV) {
            load_vrow(tile, vrow);
        } else {
            load_v(tile, 0, vr[0]);
            load_v(tile, 1, vr[1]);
        }
    };
    // One tile of sequence [s0, s1) whose rows have been requested by prefetch(): scores, online softmax, P V.
    auto process = [&](int tile) {
        const uint8_t *tp = tiles + (int64_t)tile * L.tile_bytes;
        const int n_lane = tile * SPARK_TILE_TOKENS + lane;
        const bool valid = (n_lane >= s0) && (n_lane < s1);

        uint32_t (&r)[NR] = rn;
        // ---- scores, lane = token
        const float mu = REC ? 0.0f : __uint_as_float(r[4]);   // sampled recovery: no mean term
        float s[G];
#pragma unroll
        for (int g = 0; g < G; ++g) s[g] = 0.0f;
        {
            uint64_t cur = ((uint64_t)r[1] << 32) | r[0];
            const uint64_t upper = ((uint64_t)r[3] << 32) | r[2];
            const int clo = __popc(r[0]) + __popc(r[1]);
            int jb = 0;
            float scale_row = 1.0f;
            if (INT8) scale_row = __uint_as_float(r[5]);
            // next kept channel of this lane's row (ascending); exactly T bits are set
            auto next_channel = [&](int i) {
                const bool sw = (i == clo);          // first entry of channels 64..127
                cur = sw ? upper : cur;
                jb = sw ? 64 : jb;
                const int j = (__builtin_ctzll((unsigned long long)cur) + jb) & (SPARK_D - 1);
                cur &= cur - 1;
                return j;
            };
            auto kept_value = [&](int i, uint32_t word) {
                if (INT8) return (float)(int)(int8_t)((word >> (8 * (i & 3))) & 0xFF) * scale_row;
                return (i & 1) ? bf16hi(word) : bf16lo(word);
            };
            auto entry = [&](int i, uint32_t word) {
                const float *e = &qt[next_channel(i) * GP];
                const float d = fmaf(-mu, e[G], kept_value(i, word));
#pragma unroll
                for (int g = 0; g < G; ++g) s[g] = fmaf(e[g], d, s[g]);
            };
            if (TCT) {
                // The mask walk is a dependent chain and the table gathers have LDS latency; doing the
                // walk and the gathers in batches keeps several gathers in flight at once.
                constexpr int BQ = (G <= 4) ? 8 : (G == 8 ? 4 : 2);   // gathers in flight, bounded by registers
#pragma unroll
                for (int i0 = 0; i0 < TCT; i0 += BQ) {
                    int off[BQ];
#pragma unroll
                    for (int u = 0; u < BQ; ++u)
                        if (i0 + u < TCT) off[u] = next_channel(i0 + u) * GP;
                    float ev[BQ][GP];
#pragma unroll
                    for (int u = 0; u < BQ; ++u)
                        if (i0 + u < TCT) {
#pragma unroll
                            for (int g = 0; g <= G; ++g) ev[u][g] = qt[off[u] + g];
                        }
#pragma unroll
                    for (int u = 0; u < BQ; ++u)
                        if (i0 + u < TCT) {
                            const int i = i0 + u;
                            const float d = fmaf(-mu, ev[u][G], kept_value(i, r[VAL0 + (INT8 ? i / 4 : i / 2)]));
#pragma unroll
                            for (int g = 0; g < G; ++g) s[g] = fmaf(ev[u][g], d, s[g]);
                        }
                }
            } else if constexpr (VAR) {
                // this row's kept entries: words [before, before + (count + 1) / 2) of the tile's part of the stream
                const uint32_t cnt = r[5] < (uint32_t)SPARK_D ? r[5] : (uint32_t)SPARK_D;     // (bounds the walk whatever the cache holds)
                const uint32_t words = (cnt + 1u) >> 1;
                const uint32_t before = (uint32_t)wave_inclusive_sum_i32((int)words) - words;
                const uint32_t *vsrc = reinterpret_cast<const uint32_t *>(P.packed + L.off_vals) + (int64_t)h * L.vals_head_words +
                                       reinterpret_cast<const uint32_t *>(P.packed + L.off_dir)[(int64_t)h * (L.n_tiles + 1) + tile] + before;
                const int tmax = (int)wave_max((float)cnt);     // (counts are at most 128: exact in float32)
                // The row's words are fetched 16 at a time (32 entries, four 16-byte loads in flight per lane: one
                // memory round trip per 32 entries instead of one per word); a load whose first word lies past the
                // lane's row is masked off, one that straddles the row's end reads at most three words of the next
                // row or of the stream's padding.  Entries are then taken eight at a time like the fixed-count path
                // (eight channel numbers off the mask, eight table gathers in flight, eight multiply-adds), a group
                // being skipped only when the whole wavefront is past it.  (Measured on the 32K shape with 110 kept
                // entries per row: 688 us with one load per word, 306 us with the batched loads, 262 us with the
                // grouped gathers; eight loads in flight instead of four changed nothing.)
                constexpr int NLD = 4;      // 16-byte loads in flight per lane
                typedef uint32_t u32x4u __attribute__((ext_vector_type(4), aligned(4)));
                for (int i0 = 0; i0 < tmax; i0 += 8 * NLD) {
                    u32x4u wv[NLD];
#pragma unroll
                    for (int u = 0; u < NLD; ++u) {
                        const uint32_t w0 = (uint32_t)(i0 >> 1) + 4u * u;
                        wv[u] = (w0 < words) ? *reinterpret_cast<const u32x4u *>(vsrc + w0) : u32x4u{0u, 0u, 0u, 0u};
                    }
#pragma unroll
                    for (int u = 0; u < NLD; ++u) {
                        if (i0 + 8 * u >= tmax) break;                // (wave-uniform; the groups of eight stay whole so
                                                                      //  that their table gathers are in flight together)
                        const uint32_t w4[4] = {wv[u].x, wv[u].y, wv[u].z, wv[u].w};
                        int off[8];
#pragma unroll
                        for (int k = 0; k < 8; ++k) {
                            // (as next_channel, but defined when the row's bits have run out: an idle lane reads some entry)
                            const bool sw = (i0 + 8 * u + k == clo);
                            cur = sw ? upper : cur;
                            jb = sw ? 64 : jb;
                            off[k] = ((__builtin_ctzll((unsigned long long)cur | (1ull << 63)) + jb) & (SPARK_D - 1)) * GP;
                            cur &= cur - 1;
                        }
                        float ev[8][G + 1];
#pragma unroll
                        for (int k = 0; k < 8; ++k)
#pragma unroll
                            for (int g = 0; g <= G; ++g) ev[k][g] = qt[off[k] + g];
#pragma unroll
                        for (int k = 0; k < 8; ++k) {
                            const bool on = (uint32_t)(i0 + 8 * u + k) < cnt;   // lanes whose row is shorter idle through the rest
                            const float d = on ? fmaf(-mu, ev[k][G], kept_value(k, w4[k >> 1])) : 0.0f;
#pragma unroll
                            for (int g = 0; g < G; ++g) s[g] = fmaf(ev[k][g], d, s[g]);
                        }
                    }
                }
            } else if constexpr (G > 8) {
                // Any row length, sixteen query heads: the registers leave no room for batches of sections; one
                // load per value word, one table gather at a time.
                uint32_t vw = 0;
                for (int i = 0; i < T; ++i) {
                    if (i % per_word == 0)
                        vw = *reinterpret_cast<const uint32_t *>(tp + spark_tile_word_offset(L, lane, L.val0 + i / per_word));
                    entry(i, vw);
                }
            } else {
                // Any row length: the row's value words come in batches of two 16-byte sections (coalesced 1 KB
                // requests; one load per word cost 1.5 x the time of a row-length instantiation).  The first batch
                // was requested with the row's fixed words; each further one is requested before the batch in
                // hand is worked on.  A section that holds value words only is taken like the fixed-length path
                // takes its entries - eight channel numbers off the mask, eight table gathers in flight, eight
                // multiply-adds; the first section (the row's fixed words come first) and the last one go entry
                // by entry.  Every lane has the same T, so all of this is wave-uniform.
                constexpr int per = per_word;
                // table gathers in flight, bounded by registers (as in the fixed-length path)
                constexpr int GS = (G <= 4) ? ((WARM && INT8) ? 4 : 8) : 4;
                auto do_batch = [&](int qd0, const u32x4 (&wv)[NLD]) {
#pragma unroll
                    for (int u = 0; u < NLD; ++u) {
                        const int wq = 4 * (qd0 + u);          // first word of this section
                        if (wq >= w_hi) break;
                        const uint32_t w4[4] = {wv[u].x, wv[u].y, wv[u].z, wv[u].w};
                        const int i_first = (wq - w_lo) * per; // entry its first word starts with
                        if (wq >= w_lo && i_first + 4 * per <= T) {
#pragma unroll
                            for (int grp = 0; grp < 4 * per / GS; ++grp) {
                                const int i0 = i_first + GS * grp;
                                int off[GS];
#pragma unroll
                                for (int k = 0; k < GS; ++k) off[k] = next_channel(i0 + k) * GP;
                                float ev[GS][G + 1];
#pragma unroll
                                for (int k = 0; k < GS; ++k)
#pragma unroll
                                    for (int g = 0; g <= G; ++g) ev[k][g] = qt[off[k] + g];
#pragma unroll
                                for (int k = 0; k < GS; ++k) {
                                    const float d = fmaf(-mu, ev[k][G], kept_value(i0 + k, w4[(GS * grp + k) / per]));
#pragma unroll
                                    for (int g = 0; g < G; ++g) s[g] = fmaf(ev[k][g], d, s[g]);
                                }
                            }
                        } else {
#pragma unroll
                            for (int c = 0; c < 4; ++c) {
                                const int w = wq + c;
                                if (w < w_lo || w >= w_hi) continue;
                                for (int e = 0; e < per; ++e) {
                                    const int i = (w - w_lo) * per + e;
                                    if (i < T) entry(i, w4[c]);
                                }
                            }
                        }
                    }
                };
                u32x4 wcur[NLD];
#pragma unroll
                for (int u = 0; u < NLD; ++u) wcur[u] = wfirst[u];
                if constexpr (G <= 4) {
                    u32x4 wnxt[NLD];
                    for (int qd0 = w_lo >> 2;;) {
                        const int qd1 = qd0 + NLD;
                        const bool further = 4 * qd1 < w_hi;       // (wave-uniform)
                        if (further) load_batch(tile, qd1, wnxt);
                        do_batch(qd0, wcur);
                        if (!further) break;
#pragma unroll
                        for (int u = 0; u < NLD; ++u) wcur[u] = wnxt[u];
                        qd0 = qd1;
                    }
                } else {
                    // (eight query heads: no registers for a second batch; it is requested when the first is done)
                    for (int qd0 = w_lo >> 2;;) {
                        do_batch(qd0, wcur);
                        qd0 += NLD;
                        if (4 * qd0 >= w_hi) break;
                        load_batch(tile, qd0, wcur);
                    }
                }
            }
        }
        if constexpr (REC != 0) {
            // ---- sampled recovery: every pruned entry j adds q_gj * w~_j / a_j
            constexpr uint32_t kGold = 0x9E3779B9u;
            auto mix = [](uint32_t x) {
                x ^= x >> 16; x *= 0x85EBCA6Bu; x ^= x >> 13; x *= 0xC2B2AE35u; x ^= x >> 16;
                return x;
            };
            const uint32_t base = mix(mix(mix((uint32_t)n_lane) + P.seed_lo) + (uint32_t)h * kGold + P.seed_hi);
            auto unif = [&](uint32_t c) {   // ((x >> 9) + 0.5) / 2^23: exact in float32
                return ((float)(mix(base + c * kGold) >> 9) + 0.5f) * (1.0f / 8388608.0f);
            };
            // (the statistics follow mu, and the scale where the kept entries are int8 codes)
            const float mu_a = INT8 ? __uint_as_float(*reinterpret_cast<const uint32_t *>(tp + spark_tile_word_offset(L, lane, 6)))
                                    : __uint_as_float(r[5]);
            const float sg = __uint_as_float(*reinterpret_cast<const uint32_t *>(tp + spark_tile_word_offset(L, lane, INT8 ? 7 : 6)));
            constexpr float kLn2 = 0.69314718055994530942f;
#pragma unroll
            for (int wd = 0; wd < 4; ++wd) {
                uint32_t mw = r[wd];
#pragma unroll 2
                for (int pp = 0; pp < 16; ++pp) {
                    const int j = 32 * wd + 2 * pp;
                    const float u1 = unif((uint32_t)j), u2 = unif((uint32_t)j + 1u);
                    float w0, w1;
                    if (REC == 1) {   // Box-Muller pair for channels j, j + 1
                        const float rr = __builtin_sqrtf(-2.0f * kLn2 * __builtin_amdgcn_logf(u1));
                        w0 = fmaf(sg, rr * __builtin_amdgcn_cosf(u2), mu_a);    // v_cos / v_sin take revolutions
                        w1 = fmaf(sg, rr * __builtin_amdgcn_sinf(u2), mu_a);
                    } else {          // rate 1 / mu
                        w0 = -mu_a * kLn2 * __builtin_amdgcn_logf(u1);
                        w1 = -mu_a * kLn2 * __builtin_amdgcn_logf(u2);
                    }
                    const float *e0 = &qt[j * GP], *e1 = &qt[(j + 1) * GP];
                    const float t0 = (mw & 1u) ? 0.0f : e0[G] * w0;
                    const float t1 = (mw & 2u) ? 0.0f : e1[G] * w1;
                    mw >>= 2;
#pragma unroll
                    for (int g = 0; g < G; ++g) s[g] = fmaf(e1[g], t1, fmaf(e0[g], t0, s[g]));
                }
            }
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            s[g] = fmaf(mu, R[g], s[g]);
            s[g] = valid ? s[g] : -INFINITY;
        }

        // ---- online softmax (log2 domain) and P -> LDS as bf16 high + low parts
        bool rescale = false;
        float alpha[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float tmax = wave_max(s[g]);
            const float mnew = fmaxf(m[g], tmax);
            const float msafe = (mnew == -INFINITY) ? 0.0f : mnew;
            alpha[g] = fast_exp2(m[g] - msafe);            // m = -inf -> 0
            rescale = rescale || (mnew != m[g]);
            m[g] = mnew;
            const float p = fast_exp2(s[g] - msafe);       // s = -inf -> 0
            l[g] = fmaf(l[g], alpha[g], p);
            const __bf16 ph = (__bf16)p;
            const __bf16 pl = (__bf16)(p - (float)ph);
            Pbuf[wave][0][g][ppos] = __builtin_bit_cast(uint16_t, ph);
            Pbuf[wave][1][g][ppos] = __builtin_bit_cast(uint16_t, pl);
        }
        if (rescale) {   // wave-uniform: m is the same in every lane
            float al[4];
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) al[rr] = 1.0f;
#pragma unroll
            for (int g = 0; g < G; ++g)
                if ((g >> 2) == tg) al[g & 3] = alpha[g];
#pragma unroll
            for (int e = 0; e < 8; ++e)
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) acc[e][rr] *= al[rr];
        }
        wave_lds_sync();

        if constexpr (PV) {
            // ---- packed values: park this token's row in LDS with its per-group bookkeeping
            uint32_t *raw = reinterpret_cast<uint32_t *>(wbuf[wave]);
            uint32_t mk[4];
            if (TVC > 0) {
#pragma unroll
                for (int d = 0; d < 4 * (NVW / 4); ++d) raw[lane * RSV + d] = vrow[d];    // (word stores: the stride is odd)
                if (NVW % 4) {
                    raw[lane * RSV + 4 * (NVW / 4)] = vrow[4 * (NVW / 4)];
                    raw[lane * RSV + 4 * (NVW / 4) + 1] = vrow[4 * (NVW / 4) + 1];
                }
            } else {
                // any row length: straight from memory, no prefetch
                const uint8_t *vtp = vtiles + (int64_t)tile * Lv.tile_bytes;
                for (int qd = 1; qd < Lv.nq; ++qd) {
                    const u32x4 x = NT_LOAD(reinterpret_cast<const u32x4 *>(vtp + qd * 1024 + lane * 16));
                    *reinterpret_cast<u32x4 *>(&raw[lane * rsv + 4 * qd]) = x;
                }
                if (Lv.tail2) {
                    const uint2 x = *reinterpret_cast<const uint2 *>(vtp + Lv.nq * 1024 + lane * 8);
                    raw[lane * rsv + 4 * Lv.nq] = x.x;
                    raw[lane * rsv + 4 * Lv.nq + 1] = x.y;
                }
            }
#pragma unroll
            for (int w4 = 0; w4 < 4; ++w4) mk[w4] = vrow[w4];
            {
                // 16 halfwords: (kept entries in lower groups) << 8 | mask byte of the group
                uint32_t meta[8];
                uint32_t before = 0;
#pragma unroll
                for (int c = 0; c < 16; ++c) {
                    const uint32_t byte = (mk[c >> 2] >> (8 * (c & 3))) & 0xFFu;
                    const uint32_t hw = (before << 8) | byte;
                    if (c & 1) meta[c >> 1] |= hw << 16; else meta[c >> 1] = hw;
                    before += __popc(byte);
                }
                u32x4 m0 = {meta[0], meta[1], meta[2], meta[3]}, m1 = {meta[4], meta[5], meta[6], meta[7]};
                *reinterpret_cast<u32x4 *>(&vmeta[wave][lane * 8]) = m0;
                *reinterpret_cast<u32x4 *>(&vmeta[wave][lane * 8 + 4]) = m1;
            }
            wave_lds_sync();
        }
        {
            // ---- P V on the matrix cores
    #pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                if constexpr (PV) {
                    // rebuild the dense pieces of this half tile: lane (tg, cn) makes channels 8cn..8cn+7 of
                    // tokens 32ks + 4i + tg (four at a time, to bound the registers in flight)
                    const uint32_t *raw = reinterpret_cast<const uint32_t *>(wbuf[wave]);
                    const uint16_t *meta16 = reinterpret_cast<const uint16_t *>(vmeta[wave]);
    #pragma unroll
                    for (int i0 = 0; i0 < 8; i0 += 4) {
    #pragma unroll
                        for (int i = i0; i < i0 + 4; ++i) {
                            const int t = 32 * ks + 4 * i + tg;
                            const uint32_t hw = meta16[t * 16 + cn];
                            const uint32_t byte = hw & 0xFFu, before = hw >> 8;
                            const uint32_t *win = &raw[t * rsv + 4 + (before >> 1)];   // 8 candidates start here ...
                            const uint32_t sh = (before & 1u) << 4;                     // ... or one halfword further
                            const uint32_t d0 = win[0], d1 = win[1], d2 = win[2], d3 = win[3], d4 = win[4];
                            const uint32_t q0 = __builtin_amdgcn_alignbit(d1, d0, sh);
                            const uint32_t q1 = __builtin_amdgcn_alignbit(d2, d1, sh);
                            const uint32_t q2 = __builtin_amdgcn_alignbit(d3, d2, sh);
                            const uint32_t q3 = __builtin_amdgcn_alignbit(d4, d3, sh);
                            const u32x4 sa = *reinterpret_cast<const u32x4 *>(&vlut[byte * 4]);
                            const uint2 sb = *reinterpret_cast<const uint2 *>(&vlutb[byte * 2]);
                            vr[ks][i].x = __builtin_amdgcn_perm(q1, q0, sa.x);
                            vr[ks][i].y = __builtin_amdgcn_perm(q1, q0, sa.y);
                            vr[ks][i].z = __builtin_amdgcn_perm(q1, q0, sa.z) | __builtin_amdgcn_perm(q3, q2, sa.w);
                            vr[ks][i].w = __builtin_amdgcn_perm(q1, q0, sb.x) | __builtin_amdgcn_perm(q3, q2, sb.y);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                uint4 ah = {0, 0, 0, 0}, alo = {0, 0, 0, 0};
                if (cn < G) {
                    ah = *reinterpret_cast<const uint4 *>(&Pbuf[wave][0][cn][32 * ks + 8 * tg]);
                    alo = *reinterpret_cast<const uint4 *>(&Pbuf[wave][1][cn][32 * ks + 8 * tg]);
                }
                const bf16x8 A_hi = __builtin_bit_cast(bf16x8, ah);
                const bf16x8 A_lo = __builtin_bit_cast(bf16x8, alo);
                // 8x8 transpose of this lane's (token, channel) block: B operand e = channel 8cn+e, K = tokens
                u32x4 bop[8];
    #pragma unroll
                for (int cp = 0; cp < 4; ++cp)
    #pragma unroll
                    for (int tp2 = 0; tp2 < 4; ++tp2) {
                        const uint32_t x = u4c(vr[ks][2 * tp2], cp);
                        const uint32_t y = u4c(vr[ks][2 * tp2 + 1], cp);
                        bop[2 * cp][tp2] = __builtin_amdgcn_perm(y, x, 0x05040100u);       // low halves  (x | y << 16)
                        bop[2 * cp + 1][tp2] = __builtin_amdgcn_perm(y, x, 0x07060302u);   // high halves
                    }
    #pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const bf16x8 B = __builtin_bit_cast(bf16x8, bop[e]);
                    acc[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A_hi, B, acc[e], 0, 0, 0);
                    acc[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A_lo, B, acc[e], 0, 0, 0);
                }
            }
        }
        wave_lds_sync();   // P buffer is rewritten by the next tile
    };
    if constexpr (WARM) {
        // ---- balanced mode: this wavefront's contiguous range of the head's (sequence, tile) items
        const int B = L.batch, NW = P.warm_waves, total = W.total;
        const int wid = (int)(blockIdx.x / P.Hkv) * kDecodeWaves + wave;       // wavefront number within the KV head
        const int nwe = NW < total ? NW : total;                               // wavefronts that get items
        int item = 0, item_end = 0;
        if (wid < nwe) {
            item = (int)(((uint32_t)wid * (uint32_t)total) / (uint32_t)nwe);
            item_end = (int)((((uint32_t)wid + 1u) * (uint32_t)total) / (uint32_t)nwe);
        }
        float *const red = reinterpret_cast<float *>(wbuf[wave]);              // [G][128] staging of the accumulators

        // query table {q_g[j] * scale * log2e, 1/a[j]} and R_g of a sequence, built by this wavefront alone.  The
        // inputs are requested before the sequence's first tile (loads return in order), the table is written
        // once the previous sequence's state has been stored.
        constexpr bool HOIST = G < 8 && TCT != 0;   // (eight query heads, or the any-length loop's buffers: the registers
                                                    //  to hold the query across the store are not there)
        float inva_r[2];
        uint16_t q_r[2][G];
        auto request_query = [&](int sb) {
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
                const int j = lane + 64 * jj;
                inva_r[jj] = reinterpret_cast<const float *>(P.packed + L.off_inva)[((int64_t)sb * P.Hkv + h) * SPARK_D + j];
#pragma unroll
                for (int g = 0; g < G; ++g) q_r[jj][g] = P.q[((int64_t)sb * P.Hq + h * G + g) * SPARK_D + j];
            }
        };
        auto build_query = [&]() {
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
                const int j = lane + 64 * jj;
#pragma unroll
                for (int g = 0; g < G; ++g) qt[j * GP + g] = bf16lo(q_r[jj][g]) * P.scale_log2;
                qt[j * GP + G] = inva_r[jj];
#pragma unroll
                for (int g = G + 1; g < GP; ++g) qt[j * GP + g] = 0.0f;
            }
            wave_lds_sync();
#pragma unroll
            for (int g = 0; g < G; ++g)
                R[g] = wave_sum(qt[lane * GP + g] * qt[lane * GP + G] + qt[(lane + 64) * GP + g] * qt[(lane + 64) * GP + G]);
        };
        auto reset_state = [&]() {
#pragma unroll
            for (int g = 0; g < G; ++g) { m[g] = -INFINITY; l[g] = 0.0f; }
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};
        };
        // A stored partial is counted in only after its stores have been acknowledged.  The wait is put off to
        // a point where nothing else of this wavefront is in flight (just before the next tile is requested, or
        // at the end), so it costs nothing; whoever counts last merges the pair.  (Looking at the count's answer
        // one tile later still, to save its round trip as well, was measured 30 % slower: a load result that is
        // live around the loop makes the compiler wait for all memory at the top of every iteration.)
        PairInfo pend = {0, 0, 0};
        int pend_n = 0;                      // partial states of the pending pair (0: nothing pending)
        // Folds the nm partial states of pair pr for all G query heads at once: 64 / G lanes per head, each with
        // 2 G output channels, every lane fetching the (m, l) pairs of its head (the lanes of a head read the same
        // words) and its channels of every partial - all loads of a round are independent, so a pair with up to
        // RN partials costs one memory round trip however many heads it has.
        auto merge_pair = [&](const PairInfo &pr, int nm) {
            constexpr int LPH = 64 / G, CPL = 2 * G, RN = (32 / G < 16) ? 32 / G : 16;
            const int g = lane / LPH, c = lane % LPH;
            const int qh = h * G + g;
            const uint64_t *pm = reinterpret_cast<const uint64_t *>(P.part_ml);
            float M = -INFINITY, Lsum = 0.0f, A[CPL];
#pragma unroll
            for (int e = 0; e < CPL; ++e) A[e] = 0.0f;
            for (int i0 = 0; i0 < nm; i0 += RN) {
                const int n = (nm - i0 < RN) ? nm - i0 : RN;
                uint64_t ml[RN], av[RN][G];
#pragma unroll
                for (int k = 0; k < RN; ++k) {
                    if (k < n) {                               // (wave-uniform)
                        const int64_t slot = slot_of(pr, qh, i0 + k);
                        ml[k] = __hip_atomic_load(pm + slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        const uint64_t *pa = reinterpret_cast<const uint64_t *>(P.part_acc + slot * SPARK_D + c * CPL);
#pragma unroll
                        for (int v = 0; v < G; ++v) av[k][v] = __hip_atomic_load(pa + v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    } else {
                        ml[k] = (uint64_t)__float_as_uint(-INFINITY);      // (m = -inf, l = 0: factor 0)
#pragma unroll
                        for (int v = 0; v < G; ++v) av[k][v] = 0ull;
                    }
                }
                float Mn = M;
#pragma unroll
                for (int k = 0; k < RN; ++k) Mn = fmaxf(Mn, __uint_as_float((uint32_t)ml[k]));
                const float Ms = (Mn == -INFINITY) ? 0.0f : Mn;
                const float fo = fast_exp2(M - Ms);            // M = -inf -> 0
                M = Mn;
                Lsum *= fo;
#pragma unroll
                for (int e = 0; e < CPL; ++e) A[e] *= fo;
#pragma unroll
                for (int k = 0; k < RN; ++k) {
                    const float f = fast_exp2(__uint_as_float((uint32_t)ml[k]) - Ms);
                    Lsum = fmaf(__uint_as_float((uint32_t)(ml[k] >> 32)), f, Lsum);
#pragma unroll
                    for (int v = 0; v < G; ++v) {
                        A[2 * v] = fmaf(__uint_as_float((uint32_t)av[k][v]), f, A[2 * v]);
                        A[2 * v + 1] = fmaf(__uint_as_float((uint32_t)(av[k][v] >> 32)), f, A[2 * v + 1]);
                    }
                }
            }
            const int64_t o2 = (((int64_t)pr.b * P.Hq + qh) * SPARK_D + c * CPL) / 2;      // in pairs of channels
#pragma unroll
            for (int v = 0; v < G; ++v) {
                const float o0 = (Lsum > 0.0f) ? (A[2 * v] / Lsum) : 0.0f, o1 = (Lsum > 0.0f) ? (A[2 * v + 1] / Lsum) : 0.0f;
                if (P.out_f32) {
                    reinterpret_cast<float2 *>(P.out)[o2 + v] = make_float2(o0, o1);
                } else {
                    reinterpret_cast<uint32_t *>(P.out)[o2 + v] = (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)o0) |
                                                                  ((uint32_t)__builtin_bit_cast(uint16_t, (__bf16)o1) << 16);
                }
            }
        };
        auto flush = [&]() {
            if (pend_n == 0) return;         // (wave-uniform)
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);   // this wavefront's stores have been acknowledged
            uint32_t old = 0u;
            if (lane == 0) old = atomicInc(&P.counters[pend.b * P.Hkv + h], (uint32_t)(pend_n - 1));
            old = (uint32_t)__builtin_amdgcn_readfirstlane((int)old);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            if (old == (uint32_t)(pend_n - 1)) {
                merge_pair(pend, pend_n);
                if (P.trace != nullptr) stamp(P, 7, 1ull);
            }
            pend_n = 0;
        };
        // this wavefront's state of pair pr: the output itself when nobody else contributes, else its partial
        auto finalize = [&](const PairInfo &pr, int my) {
            flush();                         // (one pair can be pending at a time)
            const int nm = pr.nsplit + P.ntail;
            float lt[G];
#pragma unroll
            for (int g = 0; g < G; ++g) lt[g] = wave_sum(l[g]);
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int g = 4 * tg + rr;
                if (g < G) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) red[g * SPARK_D + 8 * cn + e] = acc[e][rr];
                }
            }
            wave_lds_sync();
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float2 a2 = *reinterpret_cast<const float2 *>(&red[g * SPARK_D + 2 * lane]);
                const int qh = h * G + g;
                if (nm == 1) {
                    const float o0 = (lt[g] > 0.0f) ? (a2.x / lt[g]) : 0.0f, o1 = (lt[g] > 0.0f) ? (a2.y / lt[g]) : 0.0f;
                    const int64_t oi = ((int64_t)pr.b * P.Hq + qh) * (SPARK_D / 2) + lane;
                    if (P.out_f32) {
                        reinterpret_cast<float2 *>(P.out)[oi] = make_float2(o0, o1);
                    } else {
                        reinterpret_cast<uint32_t *>(P.out)[oi] = (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)o0) |
                                                                  ((uint32_t)__builtin_bit_cast(uint16_t, (__bf16)o1) << 16);
                    }
                } else {
                    const int64_t slot = slot_of(pr, qh, my);
                    const uint64_t two = (uint64_t)__float_as_uint(a2.x) | ((uint64_t)__float_as_uint(a2.y) << 32);
                    __hip_atomic_store(reinterpret_cast<uint64_t *>(P.part_acc + slot * SPARK_D) + lane, two, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                    if (lane == 0) {
                        const uint64_t ml = (uint64_t)__float_as_uint(m[g]) | ((uint64_t)__float_as_uint(lt[g]) << 32);
                        __hip_atomic_store(reinterpret_cast<uint64_t *>(P.part_ml) + slot, ml, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
            }
            wave_lds_sync();   // the staging area is reused
            if (nm > 1) { pend = pr; pend_n = nm; }
        };

        if (P.trace != nullptr) stamp(P, 5, (1ull << 32) | (unsigned long long)(item_end - item));   // (bit 32: balanced mode)
        if (item < item_end) {
            WarmSeq cur = warm_find(W, item);
            PairInfo pr = warm_pair(P, cur, B, total);
            int my = wid - (pr.first - cur.b);                 // this wavefront's partial within the pair
            s0 = cur.s0;
            s1 = cur.s1;
            int tile = s0 / SPARK_TILE_TOKENS + (item - cur.first_item);
            if (HOIST) request_query(cur.b);
            prefetch(tile);
            if (!HOIST) request_query(cur.b);
            build_query();
            reset_state();
            if (P.trace != nullptr) stamp(P, 1, wall_clock64());
            for (;;) {
                ++item;
                const bool more = item < item_end;
                const bool newseq = more && (item == cur.first_item + cur.n);   // (wave-uniform)
                WarmSeq nxt = cur;
                if (newseq) nxt = warm_find(W, item);
                const int tnext = newseq ? nxt.s0 / SPARK_TILE_TOKENS : tile + 1;
                process(tile);
                if (!more) break;
                s0 = nxt.s0;
                s1 = nxt.s1;
                tile = tnext;
                flush();                     // (nothing of this wavefront is in flight here, and no tile is held)
                if (HOIST && newseq) request_query(nxt.b);
                prefetch(tile);              // in flight while the finished sequence is stored and the table rebuilt
                if (newseq) {
                    finalize(pr, my);
                    cur = nxt;
                    pr = warm_pair(P, cur, B, total);
                    my = wid - (pr.first - cur.b);
                    if (!HOIST) request_query(cur.b);
                    build_query();
                    reset_state();
                }
            }
            if (P.trace != nullptr) stamp(P, 2, wall_clock64());
            // A pair whose partials are exactly this block's four wavefronts' last ones (batches of equal
            // sequences: every sequence is one block's share) needs no partials in memory: the four states are
            // folded through LDS and the output written, as the cut by length does with one block per sequence.
            // All four wavefronts see the same condition, and each meets the barrier once, at its end.
            const int wf = pr.first - cur.b;
            const bool block_pair = pr.nsplit == kDecodeWaves && (wf % kDecodeWaves) == 0 && P.ntail == 0 &&
                                    (int)((((uint32_t)wf + (uint32_t)kDecodeWaves) * (uint32_t)total) / (uint32_t)nwe) ==
                                        cur.first_item + cur.n;
            if (block_pair) {
                flush();
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const float lt = wave_sum(l[g]);
                    if (lane == 0) { red_m[wave][g] = m[g]; red_l[wave][g] = lt; }
                }
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const int g = 4 * tg + rr;
                    if (g < G) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) red[g * SPARK_D + 8 * cn + e] = acc[e][rr];
                    }
                }
                __syncthreads();
                for (int idx = tid; idx < G * SPARK_D; idx += kDecodeWaves * 64) {
                    const int g = idx / SPARK_D, ch = idx % SPARK_D;
                    float M = -INFINITY;
#pragma unroll
                    for (int w2 = 0; w2 < kDecodeWaves; ++w2) M = fmaxf(M, red_m[w2][g]);
                    const float Ms = (M == -INFINITY) ? 0.0f : M;
                    float Lsum = 0.0f, A = 0.0f;
#pragma unroll
                    for (int w2 = 0; w2 < kDecodeWaves; ++w2) {
                        const float f = fast_exp2(red_m[w2][g] - Ms);
                        Lsum = fmaf(red_l[w2][g], f, Lsum);
                        A = fmaf(reinterpret_cast<const float *>(wbuf[w2])[g * SPARK_D + ch], f, A);
                    }
                    const float o = (Lsum > 0.0f) ? (A / Lsum) : 0.0f;
                    const int64_t oi = ((int64_t)cur.b * P.Hq + h * G + g) * SPARK_D + ch;
                    if (P.out_f32)
                        reinterpret_cast<float *>(P.out)[oi] = o;
                    else
                        reinterpret_cast<uint16_t *>(P.out)[oi] = __builtin_bit_cast(uint16_t, (__bf16)o);
                }
                __syncthreads();             // (a wavefront that looks after an empty sequence next reuses its staging area)
            } else {
                finalize(pr, my);
            }
            if (P.trace != nullptr) stamp(P, 3, wall_clock64());
            flush();
        }
        // sequences without tokens have no item: wavefront b mod NW writes their zeros (or their empty partial)
        for (int sb = wid; sb < B; sb += NW) {
            const WarmSeq q = warm_get(W, sb);
            if (q.n == 0) {
                reset_state();
                finalize(warm_pair(P, q, B, total), 0);
                flush();
            }
        }
        if (P.trace != nullptr) stamp(P, 4, wall_clock64());
        return;
    }
    // ---- tiles of this split
    int t_begin = 0, t_end = 0;
    if (s1 > s0) {
        const int tf = s0 / SPARK_TILE_TOKENS, tl = (s1 - 1) / SPARK_TILE_TOKENS;
        const int ntile = tl - tf + 1;
        const int chunk = (ntile + nsplit - 1) / nsplit;
        t_begin = tf + split * chunk;
        t_end = t_begin + chunk;
        if (t_end > tl + 1) t_end = tl + 1;
    }

    // Tiles are visited in rotated order, a different rotation per block.  The order does not
    // matter to the running softmax, and it keeps the blocks (whose V chunks start at large
    // power-of-two distances) from sweeping the memory channels in lockstep.
    const int nts = t_end - t_begin;
    const int rot = nts > 0 ? (int)((blockIdx.x * 37u) % (uint32_t)nts) : 0;
    auto tile_of = [&](int k) { int li = k + rot; li = (li >= nts) ? li - nts : li; return t_begin + li; };
    int kidx = wave;
    int tile = tile_of(kidx);
    // The query and 1/a are requested before the first tile: loads return in order, so the table can be built
    // while the tile is still on its way.
    float inva_r = 0.0f;
    uint16_t q_r[G];
    if (tid < SPARK_D) {
        inva_r = reinterpret_cast<const float *>(P.packed + L.off_inva)[((int64_t)b * P.Hkv + h) * SPARK_D + tid];
#pragma unroll
        for (int g = 0; g < G; ++g) q_r[g] = P.q[((int64_t)b * P.Hq + h * G + g) * SPARK_D + tid];
    }
    if (kidx < nts) prefetch(tile);
    if constexpr (PV) {
        // Selector table, entry b = mask byte of a group of 8 channels.  The group's kept entries are the
        // first popcount(b) of a window of 8 candidates = 16 bytes Q0..Q3; output word o holds channels
        // 2o, 2o+1.  A byte-permute picks from two words (selector 0-3: second operand, 4-7: first, 0x0C:
        // zero): words 0, 1 need candidates 0..3 only -> one permute of (Q1, Q0); words 2, 3 may reach
        // into Q2, Q3 -> the OR of a permute of (Q1, Q0) and one of (Q3, Q2).
        const uint32_t bmask = (uint32_t)tid;
        uint32_t sel[6];
#pragma unroll
        for (int k = 0; k < 6; ++k) sel[k] = 0x0C0C0C0Cu;
        int rnk = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const bool on = (bmask >> e) & 1u;
            const int o = e >> 1, sh = (e & 1) * 16;      // output word, bit position of its half
            const int src = 2 * rnk;                       // candidate's first byte in the window
            const uint32_t two = (uint32_t)((src & 7) | (((src & 7) + 1) << 8)) << sh;
            const uint32_t keep = ~(0xFFFFu << sh);
            if (o < 2) {
                if (on) sel[o] = (sel[o] & keep) | two;
            } else {
                if (on && src < 8) sel[2 * o - 2] = (sel[2 * o - 2] & keep) | two;
                if (on && src >= 8) sel[2 * o - 1] = (sel[2 * o - 1] & keep) | two;
            }
            rnk += on ? 1 : 0;
        }
        u32x4 lo4 = {sel[0], sel[1], sel[2], sel[3]};
        *reinterpret_cast<u32x4 *>(&vlut[tid * 4]) = lo4;
        vlutb[tid * 2] = sel[4];
        vlutb[tid * 2 + 1] = sel[5];
    }
    // ---- per-step query prep: table {q_g[j] * scale * log2e, 1/a[j]} and R_g
    if (tid < SPARK_D) {
        const int j = tid;
#pragma unroll
        for (int g = 0; g < G; ++g) qt[j * GP + g] = bf16lo(q_r[g]) * P.scale_log2;
        qt[j * GP + G] = inva_r;
#pragma unroll
        for (int g = G + 1; g < GP; ++g) qt[j * GP + g] = 0.0f;
    }
    __syncthreads();
    for (int g = wave; g < G; g += kDecodeWaves) {
        float r = qt[lane * GP + g] * qt[lane * GP + G] +
                  qt[(lane + 64) * GP + g] * qt[(lane + 64) * GP + G];
        r = wave_sum(r);
        if (lane == 0) Rsh[g] = r;
    }
    __syncthreads();
#pragma unroll
    for (int g = 0; g < G; ++g) R[g] = Rsh[g];


    if (P.trace != nullptr) { stamp(P, 1, wall_clock64()); stamp(P, 5, (unsigned long long)nts); }
    for (; kidx < nts; kidx += kDecodeWaves) {
        tile = tile_of(kidx);
        const bool more = kidx + kDecodeWaves < nts;            // wave-uniform
        const int tnext = tile_of(more ? kidx + kDecodeWaves : kidx);
        process(tile);
        if (more) prefetch(tnext);   // request the next tile; its latency is covered by the other resident wavefronts
    }

    if (P.trace != nullptr) stamp(P, 2, wall_clock64());
    // ---- merge the 4 wavefronts, write the split partial
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const float lt = wave_sum(l[g]);
        if (lane == 0) { red_m[wave][g] = m[g]; red_l[wave][g] = lt; }
    }
    // accumulator layout: lane (tg, cn), register rr of acc[e] = head 4*tg + rr, channel 8*cn + e
    wave_lds_sync();   // this wavefront's parked value rows are no longer read
    auto red_acc = [&](int w, int g, int ch) -> float & {
        return reinterpret_cast<float *>(wbuf[w])[g * SPARK_D + ch];
    };
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const int g = 4 * tg + rr;
        if (g < G) {
#pragma unroll
            for (int e = 0; e < 8; ++e) red_acc(wave, g, 8 * cn + e) = acc[e][rr];
        }
    }
    __syncthreads();
    for (int idx = tid; idx < G * SPARK_D; idx += kDecodeWaves * 64) {
        const int g = idx / SPARK_D, ch = idx % SPARK_D;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < kDecodeWaves; ++w) M = fmaxf(M, red_m[w][g]);
        const float Ms = (M == -INFINITY) ? 0.0f : M;
        float Lsum = 0.0f, A = 0.0f;
#pragma unroll
        for (int w = 0; w < kDecodeWaves; ++w) {
            const float f = fast_exp2(red_m[w][g] - Ms);
            Lsum = fmaf(red_l[w][g], f, Lsum);
            A = fmaf(red_acc(w, g, ch), f, A);
        }
        if (nmerge == 1) {   // the only block of this (batch, KV head): the result is final
            const float o = (Lsum > 0.0f) ? (A / Lsum) : 0.0f;
            const int64_t oi = ((int64_t)b * P.Hq + h * G + g) * SPARK_D + ch;
            if (P.out_f32)
                reinterpret_cast<float *>(P.out)[oi] = o;
            else
                reinterpret_cast<uint16_t *>(P.out)[oi] = __builtin_bit_cast(uint16_t, (__bf16)o);
        } else {
            const int64_t slot = slot_of(pi, h * G + g, split);
            st_agent(&P.part_acc[slot * SPARK_D + ch], A);
            if (ch == 0) { st_agent(&P.part_ml[slot * 2], M); st_agent(&P.part_ml[slot * 2 + 1], Lsum); }
        }
    }
    }   // sequence split
    if (P.trace != nullptr) { const unsigned long long now = wall_clock64(); stamp(P, 3, now); stamp(P, 4, now); }
    if (nmerge == 1) return;   // (block-uniform)

    // ---- the last block of this (batch, KV head) to get here merges the splits.
    // The partials are written and read with device-scope accesses (they go to the point where
    // all the chip's L2 slices agree), each thread waits for its own stores to be acknowledged,
    // and only then is the block's arrival counted.  That orders partials before the count
    // without a device-wide cache write-back.  atomicInc wraps at the number of arrivals - 1, which leaves the
    // counter at zero for the next call.
    __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);   // this thread's stores have been acknowledged
    __syncthreads();
    if (tid == 0) {
        const uint32_t old = atomicInc(&P.counters[b * P.Hkv + h], (uint32_t)(nmerge - 1));
        last_flag = (old == (uint32_t)(nmerge - 1));
    }
    __syncthreads();
    if (P.trace != nullptr) stamp(P, 4, wall_clock64());
    if (!last_flag) return;
    // a wavefront takes one query head per pass
    for (int g = wave; g < G; g += kDecodeWaves) merge_head(pi, nmerge, g);
    if (P.trace != nullptr) { stamp(P, 4, wall_clock64()); stamp(P, 7, 1ull); }
}

// ---------------------------------------------------------------- host-side launch

template <int G, int TCT, int INT8, int TVC, int REC = 0, int VAR = 0, int WARM = 0>
static hipError_t launch_one(const DecodeParams &P, int nblocks, hipStream_t st)
{
    hipLaunchKernelGGL((spark_decode_kernel<G, TCT, INT8, TVC, REC, VAR, WARM>), dim3(nblocks), dim3(kDecodeWaves * 64), 0, st, P);
    return hipGetLastError();
}

// dense values, degenerate recovery, fixed row length: the chunked or the balanced decomposition
template <int G, int TCT, int INT8>
static hipError_t launch_plain(const DecodeParams &P, int nblocks, hipStream_t st)
{
    if constexpr (G <= 8) {
        if (P.warm_waves > 0) return launch_one<G, TCT, INT8, 0, 0, 0, 1>(P, nblocks, st);
    }
    return launch_one<G, TCT, INT8, 0>(P, nblocks, st);
}

// packed values: row lengths 64 / 38 / 26 with the row in registers, anything else generic
template <int G, int TCT, int INT8 = 0>
static hipError_t launch_pv(const DecodeParams &P, int nblocks, hipStream_t st)
{
    switch (P.Lv.T) {
        case 64: return launch_one<G, TCT, INT8, 64>(P, nblocks, st);
        case 38: return launch_one<G, TCT, INT8, 38>(P, nblocks, st);
        case 26: return launch_one<G, TCT, INT8, 26>(P, nblocks, st);
        default: return launch_one<G, TCT, INT8, -1>(P, nblocks, st);
    }
}

// One instantiation per query-group size G; each lives in its own translation unit (spark_decode_g*.hip) so
// that the units compile in parallel.
template <int G>
hipError_t launch_g(const DecodeParams &P, int nblocks, hipStream_t st)
{
    // rows that carry the all-channel statistics are longer: only the any-length instantiations read them
    const int T = P.L.stats ? -1 : P.L.T;
    if (P.L.topp) return launch_one<G, 0, 0, 0, 0, 1>(P, nblocks, st);
    if (P.rec == 1) return P.L.int8 ? launch_one<G, 0, 1, 0, 1>(P, nblocks, st) : launch_one<G, 0, 0, 0, 1>(P, nblocks, st);
    if (P.rec == 2) return P.L.int8 ? launch_one<G, 0, 1, 0, 2>(P, nblocks, st) : launch_one<G, 0, 0, 0, 2>(P, nblocks, st);
    if (P.packed_v) {
        if (P.L.int8) return T == 26 ? launch_pv<G, 26, 1>(P, nblocks, st) : launch_pv<G, 0, 1>(P, nblocks, st);
        if (T == 26) return launch_pv<G, 26>(P, nblocks, st);
        if (T == 64) return launch_pv<G, 64>(P, nblocks, st);
        return launch_pv<G, 0>(P, nblocks, st);
    }
    if (P.L.int8) {
        if (T == 26) return launch_plain<G, 26, 1>(P, nblocks, st);
        if (T == 38) return launch_plain<G, 38, 1>(P, nblocks, st);
        if (T == 64) return launch_plain<G, 64, 1>(P, nblocks, st);
        return launch_plain<G, 0, 1>(P, nblocks, st);
    }
    if (T == 26) return launch_plain<G, 26, 0>(P, nblocks, st);
    if (T == 25) return launch_plain<G, 25, 0>(P, nblocks, st);
    if (T == 38) return launch_plain<G, 38, 0>(P, nblocks, st);
    if (T == 64) return launch_plain<G, 64, 0>(P, nblocks, st);
    return launch_plain<G, 0, 0>(P, nblocks, st);
}

}  // namespace spark
