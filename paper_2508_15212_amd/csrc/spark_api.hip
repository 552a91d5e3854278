// C ABI of the library (see include/spark.h): argument checks on the host, buffer sizing,
// kernel launches on the caller's stream.  Nothing here allocates or synchronises.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <mutex>

#include "../../include/spark.h"
#include "spark_kernels.h"
#include "spark_layout.h"

namespace {

bool desc_ok(const spark_desc *d, spark_status *why)
{
    *why = SPARK_ERR_INVALID_ARG;
    if (!d) return false;
    if (d->batch < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1) return false;
    // token and tile indices are 32-bit in the kernels (a tile's last row index must still fit), block counts too
    if (d->total_tokens < 0 || d->total_tokens > ((int64_t)1 << 31) - 256) return false;
    if (d->batch > (1 << 18)) return false;
    if (d->keep < 1 || d->keep > d->head_dim) return false;
    if (d->n_q_heads % d->n_kv_heads) return false;
    if (d->n_splits < -1 || d->n_splits > 4096) return false;
    if (d->max_seqlen < 0) return false;
    if (d->keep_v < 0 || d->keep_v > d->head_dim) return false;
    if (d->tail_capacity < 0 || d->tail_capacity > (1 << 20)) return false;
    if (d->stats != 0 && d->stats != 1) return false;
    *why = SPARK_ERR_UNSUPPORTED;
    if (d->head_dim != SPARK_D) return false;
    const int G = d->n_q_heads / d->n_kv_heads;
    if (!(G == 1 || G == 2 || G == 4 || G == 8 || G == 16)) return false;
    if (d->pack_dtype != SPARK_PACK_BF16 && d->pack_dtype != SPARK_PACK_INT8) return false;
    if (d->out_dtype != SPARK_OUT_BF16 && d->out_dtype != SPARK_OUT_F32) return false;
    *why = SPARK_OK;
    return true;
}

SparkLayout layout_of(const spark_desc *d)
{
    return spark_make_layout(d->keep, d->pack_dtype == SPARK_PACK_INT8, d->batch, d->n_kv_heads, d->total_tokens,
                             d->stats);
}

SparkLayout topp_layout_of(const spark_desc *d)
{
    return spark_make_topp_layout(d->batch, d->n_kv_heads, d->total_tokens);
}

SparkLayout values_layout_of(const spark_desc *d)
{
    return spark_make_values_layout(d->keep_v, d->n_kv_heads, d->total_tokens);
}

bool strides_ok(int64_t tok, int64_t head)
{
    return tok >= SPARK_D && head >= SPARK_D && tok % 8 == 0 && head % 8 == 0;
}

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// How the decode grid cuts the batch into blocks.  The decode kernel keeps two 4-wave blocks resident per
// compute unit (256 CUs), so about 512 blocks stream the cache in a single round with no tail; a block should
// still see at least 4 tiles (one per wavefront).  Sequences are cut into chunks of chunk_tiles tiles, so long
// sequences of a ragged batch get more blocks than short ones; n_splits > 0 (or a batch too large for the
// in-kernel numbering of the chunks) asks for the same number of chunks for every sequence instead.
spark::DecodePlan plan_of(const spark_desc *d, bool allow_balanced = true)
{
    spark::DecodePlan p;
    p.tail_slots = d->tail_capacity > 0 ? (d->tail_capacity + 255) / 256 : 1;
    const int64_t tiles = (d->total_tokens + SPARK_TILE_TOKENS - 1) / SPARK_TILE_TOKENS;
    int64_t chunk = (tiles * d->n_kv_heads + 511) / 512;
    // With many (batch, KV head) pairs the blocks of an evenly cut batch would already exceed what is resident
    // at once, and every further round costs a block's fixed start-up and merge latency: then only sequences
    // well above the average length are cut.
    if ((int64_t)d->batch * d->n_kv_heads >= 256) chunk *= 2;
    if (chunk < 4) chunk = 4;     // one tile per wavefront: below that a block's start-up outweighs its work
    p.chunk_tiles = (int)chunk;
    p.fixed_splits = 0;
    if (d->n_splits > 0) {
        p.fixed_splits = d->n_splits;
    } else if (d->batch > 256) {
        const int64_t avg_tiles = (d->total_tokens / d->batch + SPARK_TILE_TOKENS - 1) / SPARK_TILE_TOKENS;
        int64_t n = (avg_tiles + chunk - 1) / chunk;
        p.fixed_splits = (int)(n < 1 ? 1 : (n > 4096 ? 4096 : n));
    }
    if (p.fixed_splits > 0)
        p.nchunk_max = d->batch * p.fixed_splits;
    else   // a sequence of len tokens spans at most len / 64 + 2 tiles, and rounding up costs at most one chunk
        p.nchunk_max = (int)((tiles + 2 * (int64_t)d->batch) / chunk + d->batch + 1);
    // Many sequences, each too short to be cut: one block per (sequence, KV head) would make the launch last as
    // long as its longest sequence.  Then (or on request, n_splits = -1) the (sequence, tile) items of a KV head
    // are dealt out evenly to as many wavefronts as are resident at once, 2048 over all heads.  The mode holds
    // the batch's sequence table in registers (at most 256 sequences) and numbers items in 32 bits.
    p.warm_waves = 0;
    p.chunk_ids = p.nchunk_max;
    const int64_t pairs = (int64_t)d->batch * d->n_kv_heads;
    // (a batch that its caller knows to be near-uniform is balanced with one block per sequence already)
    const bool even = d->max_seqlen > 0 && (int64_t)d->max_seqlen * d->batch * 8 <= d->total_tokens * 9;
    const bool wanted = d->n_splits == -1 || (d->n_splits == 0 && d->batch >= 32 && pairs >= 256 && !even);
    if (allow_balanced && wanted && d->batch <= 256 && d->n_q_heads / d->n_kv_heads <= 8) {
        const int per_head = 512 / d->n_kv_heads > 0 ? 512 / d->n_kv_heads : 1;     // blocks of four wavefronts
        const int64_t nw = 4 * (int64_t)per_head;
        // (unasked, only where a wavefront gets two tiles or more: with less the partials cost more than the
        //  balance gains - 32 sequences of 100 to 1000 tokens: 19.0 against 20.6 us)
        const bool enough = d->n_splits == -1 || tiles >= 2 * nw;
        if (enough && (tiles + 2 * (int64_t)d->batch + 1) * nw < ((int64_t)1 << 32)) {
            p.warm_waves = (int)nw;
            const int ids = (int)nw + 2 * d->batch;
            if (p.chunk_ids < ids) p.chunk_ids = ids;
        }
    }
    return p;
}

// chunks an average-length sequence is cut into; 0 for the balanced cut (what spark_decode_splits reports)
int pick_splits(const spark_desc *d)
{
    const spark::DecodePlan p = plan_of(d);
    if (p.warm_waves > 0) return 0;
    if (p.fixed_splits > 0) return p.fixed_splits;
    const int64_t avg_tiles = (d->total_tokens / d->batch + SPARK_TILE_TOKENS - 1) / SPARK_TILE_TOKENS;
    const int64_t n = (avg_tiles + p.chunk_tiles - 1) / p.chunk_tiles;
    return (int)(n < 1 ? 1 : n);
}

// partial slots in the workspace: one per (chunk, q head), then the appended rows' (one per 256 rows of
// capacity, at least one, per (batch, q head), so a workspace serves calls with and without appended rows)
size_t partial_slots(const spark_desc *d, bool allow_balanced = true)
{
    const spark::DecodePlan p = plan_of(d, allow_balanced);
    return (size_t)p.chunk_ids * d->n_q_heads + (size_t)d->batch * d->n_q_heads * p.tail_slots;
}

// The arrival counters sit at the START of the workspace, so their position depends on batch and n_kv_heads
// only and not on how a call cuts its sequences into blocks; the partial states follow at a 256-byte boundary.
size_t counter_bytes(const spark_desc *d)
{
    return (((size_t)d->batch * d->n_kv_heads * sizeof(uint32_t)) + 255) & ~(size_t)255;
}

}  // namespace

extern "C" {

const char *spark_status_string(spark_status s)
{
    switch (s) {
        case SPARK_OK: return "ok";
        case SPARK_ERR_INVALID_ARG: return "invalid argument";
        case SPARK_ERR_UNSUPPORTED: return "unsupported configuration";
        case SPARK_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case SPARK_ERR_HIP: return "HIP runtime error";
        case SPARK_ERR_MISMATCH: return "packed cache does not match the description";
    }
    return "unknown status";
}

size_t spark_packed_bytes(const spark_desc *desc)
{
    spark_status why;
    if (!desc_ok(desc, &why)) return 0;
    return (size_t)layout_of(desc).total_bytes;
}

size_t spark_prune_workspace(const spark_desc *desc)
{
    (void)desc;
    return 0;
}

int32_t spark_decode_splits(const spark_desc *desc)
{
    spark_status why;
    if (!desc_ok(desc, &why)) return 0;
    return pick_splits(desc);
}

size_t spark_decode_workspace(const spark_desc *desc)
{
    spark_status why;
    if (!desc_ok(desc, &why)) return 0;
    const size_t slots = partial_slots(desc);
    return slots * (SPARK_D + 2) * sizeof(float) + counter_bytes(desc);
}

spark_status spark_decode_workspace_init(const spark_desc *desc, void *workspace, size_t workspace_bytes,
                                         void *hip_stream)
{
    spark_status why;
    if (!desc_ok(desc, &why)) return why;
    if (!workspace || !aligned(workspace, 16)) return SPARK_ERR_INVALID_ARG;
    if (workspace_bytes < spark_decode_workspace(desc)) return SPARK_ERR_WORKSPACE_TOO_SMALL;
    uint32_t *counters = static_cast<uint32_t *>(workspace);
    const hipError_t e = spark::launch_zero_counters(counters, desc->batch * desc->n_kv_heads,
                                                     static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SPARK_OK : SPARK_ERR_HIP;
}

spark_status spark_prune(const spark_desc *desc, const void *k_bf16, const void *qwin_bf16,
                         const int32_t *cu_seqlens, void *packed_out, void *workspace, size_t workspace_bytes,
                         void *hip_stream)
{
    (void)workspace;
    (void)workspace_bytes;
    spark_status why;
    if (!desc_ok(desc, &why)) return why;
    if (!k_bf16 || !qwin_bf16 || !cu_seqlens || !packed_out) return SPARK_ERR_INVALID_ARG;
    if (desc->window < 1) return SPARK_ERR_INVALID_ARG;
    if (!strides_ok(desc->k_token_stride, desc->k_head_stride)) return SPARK_ERR_INVALID_ARG;
    // the prune kernel addresses the 64 rows of a tile with 32-bit byte offsets from the tile's first row
    if (desc->k_token_stride > ((int64_t)1 << 24)) return SPARK_ERR_UNSUPPORTED;
    if (!aligned(k_bf16, 16) || !aligned(qwin_bf16, 2) || !aligned(packed_out, 256)) return SPARK_ERR_INVALID_ARG;
    const SparkLayout L = layout_of(desc);
    const hipError_t e = spark::launch_prune(static_cast<const uint16_t *>(k_bf16), desc->k_token_stride,
                                             desc->k_head_stride, static_cast<const uint16_t *>(qwin_bf16),
                                             cu_seqlens, static_cast<uint8_t *>(packed_out), L, desc->n_q_heads,
                                             desc->window, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SPARK_OK : SPARK_ERR_HIP;
}

size_t spark_packed_values_bytes(const spark_desc *desc)
{
    spark_status why;
    if (!desc_ok(desc, &why) || desc->keep_v < 1) return 0;
    return (size_t)values_layout_of(desc).total_bytes;
}

spark_status spark_prune_values(const spark_desc *desc, const void *v_bf16, void *packed_v_out, void *hip_stream)
{
    spark_status why;
    if (!desc_ok(desc, &why)) return why;
    if (desc->keep_v < 1 || !v_bf16 || !packed_v_out) return SPARK_ERR_INVALID_ARG;
    if (!strides_ok(desc->v_token_stride, desc->v_head_stride)) return SPARK_ERR_INVALID_ARG;
    if (desc->v_token_stride > ((int64_t)1 << 24)) return SPARK_ERR_UNSUPPORTED;
    if (!aligned(v_bf16, 16) || !aligned(packed_v_out, 256)) return SPARK_ERR_INVALID_ARG;
    const hipError_t e = spark::launch_prune_values(static_cast<const uint16_t *>(v_bf16), desc->v_token_stride,
                                                    desc->v_head_stride, static_cast<uint8_t *>(packed_v_out),
                                                    values_layout_of(desc), static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SPARK_OK : SPARK_ERR_HIP;
}

spark_status spark_unpack_values(const spark_desc *desc, const void *packed_v, uint32_t *mask_out, void *vals_out,
                                 void *hip_stream)
{
    spark_status why;
    if (!desc_ok(desc, &why)) return why;
    if (desc->keep_v < 1 || !packed_v) return SPARK_ERR_INVALID_ARG;
    const hipError_t e = spark::launch_unpack(static_cast<const uint8_t *>(packed_v), values_layout_of(desc), mask_out,
                                              vals_out, nullptr, nullptr, nullptr, nullptr, nullptr, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SPARK_OK : SPARK_ERR_HIP;
}

namespace {

spark_status decode_common(const spark_desc *desc, const void *q_bf16, const void *packed, const void *v_bf16,
                           const void *packed_v, const int32_t *cu_seqlens, void *out, void *workspace,
                           size_t workspace_bytes, void *hip_stream, const void *tail_k = nullptr,
                           const void *tail_v = nullptr, const int32_t *tail_len = nullptr, int rec = 0,
                           uint64_t seed = 0, bool topp = false, bool allow_balanced = true)
{
    spark_status why;
    if (!desc_ok(desc, &why)) return why;
    if (!q_bf16 || !packed || !cu_seqlens || !out || !workspace) return SPARK_ERR_INVALID_ARG;
    if (packed_v) {
        if (desc->keep_v < 1) return SPARK_ERR_INVALID_ARG;
        if (!aligned(packed_v, 256)) return SPARK_ERR_INVALID_ARG;
    } else {
        if (!v_bf16) return SPARK_ERR_INVALID_ARG;
        if (!strides_ok(desc->v_token_stride, desc->v_head_stride)) return SPARK_ERR_INVALID_ARG;
        if (!aligned(v_bf16, 16)) return SPARK_ERR_INVALID_ARG;
    }
    if (!aligned(packed, 256) || !aligned(workspace, 16) || !aligned(q_bf16, 2) || !aligned(out, 8))
        return SPARK_ERR_INVALID_ARG;
    if (tail_k) {
        if (!tail_v || !tail_len || desc->tail_capacity < 1) return SPARK_ERR_INVALID_ARG;
        if (!aligned(tail_k, 16) || !aligned(tail_v, 16) || !aligned(tail_len, 4)) return SPARK_ERR_INVALID_ARG;
    }
    const size_t slots = partial_slots(desc, allow_balanced);
    if (workspace_bytes < slots * (SPARK_D + 2) * sizeof(float) + counter_bytes(desc)) return SPARK_ERR_WORKSPACE_TOO_SMALL;
    const SparkLayout L = topp ? topp_layout_of(desc) : layout_of(desc);
    SparkLayout Lv = L;
    if (packed_v) Lv = values_layout_of(desc);
    const spark::DecodePlan plan = plan_of(desc, allow_balanced);
    uint32_t *counters = static_cast<uint32_t *>(workspace);
    float *part_acc = reinterpret_cast<float *>(static_cast<uint8_t *>(workspace) + counter_bytes(desc));
    float *part_ml = part_acc + slots * SPARK_D;
    const float scale = desc->softmax_scale != 0.0f ? desc->softmax_scale : 1.0f / sqrtf((float)SPARK_D);
    const hipError_t e = spark::launch_decode_attn(
        static_cast<const uint16_t *>(q_bf16), static_cast<const uint8_t *>(packed),
        static_cast<const uint16_t *>(v_bf16), desc->v_token_stride, desc->v_head_stride,
        static_cast<const uint8_t *>(packed_v), packed_v ? &Lv : nullptr, cu_seqlens, part_acc, part_ml, counters,
        desc->n_q_heads, plan, scale, L, out, desc->out_dtype == SPARK_OUT_F32,
        static_cast<const uint16_t *>(tail_k), static_cast<const uint16_t *>(tail_v), tail_len,
        desc->tail_capacity, rec, seed, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SPARK_OK : SPARK_ERR_HIP;
}

}  // namespace

spark_status spark_decode_attn(const spark_desc *desc, const void *q_bf16, const void *packed, const void *v_bf16,
                               const int32_t *cu_seqlens, void *out, void *workspace, size_t workspace_bytes,
                               void *hip_stream)
{
    if (!v_bf16) return SPARK_ERR_INVALID_ARG;
    return decode_common(desc, q_bf16, packed, v_bf16, nullptr, cu_seqlens, out, workspace, workspace_bytes,
                         hip_stream);
}

spark_status spark_decode_attn_sampled(const spark_desc *desc, const void *q_bf16, const void *packed,
                                       const void *v_bf16, const int32_t *cu_seqlens, void *out, void *workspace,
                                       size_t workspace_bytes, int32_t recovery, uint64_t seed, void *hip_stream)
{
    if (!v_bf16) return SPARK_ERR_INVALID_ARG;
    if (recovery != SPARK_RECOVER_GAUSSIAN && recovery != SPARK_RECOVER_EXPONENTIAL) return SPARK_ERR_INVALID_ARG;
    if (desc && !desc->stats) return SPARK_ERR_INVALID_ARG;     // the cache must carry the all-channel statistics
    return decode_common(desc, q_bf16, packed, v_bf16, nullptr, cu_seqlens, out, workspace, workspace_bytes,
                         hip_stream, nullptr, nullptr, nullptr, recovery, seed);
}

spark_status spark_unpack_stats(const spark_desc *desc, const void *packed, float *mu_all_out, float *sigma_out,
                                void *hip_stream)
{
    spark_status why;
    if (!desc_ok(desc, &why)) return why;
    if (!packed || !desc->stats) return SPARK_ERR_INVALID_ARG;
    const hipError_t e = spark::launch_unpack(static_cast<const uint8_t *>(packed), layout_of(desc), nullptr, nullptr,
                                              nullptr, nullptr, nullptr, mu_all_out, sigma_out,
                                              static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SPARK_OK : SPARK_ERR_HIP;
}

spark_status spark_decode_attn_tail(const spark_desc *desc, const void *q_bf16, const void *packed, const void *v_bf16,
                                    const int32_t *cu_seqlens, const void *tail_k_bf16, const void *tail_v_bf16,
                                    const int32_t *tail_len, void *out, void *workspace, size_t workspace_bytes,
                                    void *hip_stream)
{
    if (!v_bf16 || !tail_k_bf16) return SPARK_ERR_INVALID_ARG;
    return decode_common(desc, q_bf16, packed, v_bf16, nullptr, cu_seqlens, out, workspace, workspace_bytes,
                         hip_stream, tail_k_bf16, tail_v_bf16, tail_len);
}

spark_status spark_decode_attn_values(const spark_desc *desc, const void *q_bf16, const void *packed,
                                      const void *packed_v, const int32_t *cu_seqlens, void *out, void *workspace,
                                      size_t workspace_bytes, void *hip_stream)
{
    if (!packed_v) return SPARK_ERR_INVALID_ARG;
    return decode_common(desc, q_bf16, packed, nullptr, packed_v, cu_seqlens, out, workspace, workspace_bytes,
                         hip_stream);
}

spark_status spark_decode_attn_values_tail(const spark_desc *desc, const void *q_bf16, const void *packed,
                                           const void *packed_v, const int32_t *cu_seqlens,
                                           const void *tail_k_bf16, const void *tail_v_bf16,
                                           const int32_t *tail_len, void *out, void *workspace,
                                           size_t workspace_bytes, void *hip_stream)
{
    if (!packed_v || !tail_k_bf16) return SPARK_ERR_INVALID_ARG;
    return decode_common(desc, q_bf16, packed, nullptr, packed_v, cu_seqlens, out, workspace, workspace_bytes,
                         hip_stream, tail_k_bf16, tail_v_bf16, tail_len);
}

spark_status spark_unpack(const spark_desc *desc, const void *packed, uint32_t *mask_out, void *vals_out,
                          float *mu_out, float *scale_out, float *a_out, void *hip_stream)
{
    spark_status why;
    if (!desc_ok(desc, &why)) return why;
    if (!packed) return SPARK_ERR_INVALID_ARG;
    const SparkLayout L = layout_of(desc);
    const hipError_t e = spark::launch_unpack(static_cast<const uint8_t *>(packed), L, mask_out, vals_out, mu_out,
                                              scale_out, a_out, nullptr, nullptr, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SPARK_OK : SPARK_ERR_HIP;
}

spark_status spark_check_packed(const spark_desc *desc, const void *packed, int32_t is_value_cache, void *hip_stream)
{
    spark_status why;
    if (!desc_ok(desc, &why)) return why;
    if (!packed || !aligned(packed, 256)) return SPARK_ERR_INVALID_ARG;
    if (is_value_cache && desc->keep_v < 1) return SPARK_ERR_INVALID_ARG;
    uint32_t hdr[16];
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (hipMemcpyAsync(hdr, packed, sizeof hdr, hipMemcpyDeviceToHost, st) != hipSuccess) return SPARK_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return SPARK_ERR_HIP;
    const SparkLayout L = is_value_cache ? values_layout_of(desc) : layout_of(desc);
    // header words: magic, T, int8, batch, Hkv, total_tokens, words per row, value-cache flag, statistics flag
    const uint32_t want[9] = {SPARK_MAGIC, (uint32_t)L.T, (uint32_t)L.int8, (uint32_t)L.batch, (uint32_t)L.n_kv_heads,
                              (uint32_t)L.total_tokens, (uint32_t)L.ndw, is_value_cache ? 1u : 0u, (uint32_t)L.stats};
    for (int i = 0; i < 9; ++i)
        if (hdr[i] != want[i]) return SPARK_ERR_MISMATCH;
    return SPARK_OK;
}

// ---------------------------------------------------------------- the top-p variant

size_t spark_packed_topp_bytes(const spark_desc *desc)
{
    spark_status why;
    if (!desc_ok(desc, &why)) return 0;
    return (size_t)topp_layout_of(desc).total_bytes;
}

spark_status spark_prune_topp(const spark_desc *desc, const void *k_bf16, const void *qwin_bf16,
                              const int32_t *cu_seqlens, int32_t p_basis_points, void *packed_out, void *hip_stream)
{
    spark_status why;
    if (!desc_ok(desc, &why)) return why;
    if (!k_bf16 || !qwin_bf16 || !cu_seqlens || !packed_out) return SPARK_ERR_INVALID_ARG;
    if (desc->window < 1 || p_basis_points < 1 || p_basis_points > 10000) return SPARK_ERR_INVALID_ARG;
    if (!strides_ok(desc->k_token_stride, desc->k_head_stride)) return SPARK_ERR_INVALID_ARG;
    if (desc->pack_dtype != SPARK_PACK_BF16 || desc->stats) return SPARK_ERR_UNSUPPORTED;
    if (!aligned(k_bf16, 16) || !aligned(qwin_bf16, 2) || !aligned(packed_out, 256)) return SPARK_ERR_INVALID_ARG;
    const SparkLayout L = topp_layout_of(desc);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    hipError_t e = spark::launch_window_stat(static_cast<const uint16_t *>(qwin_bf16), static_cast<uint8_t *>(packed_out), L,
                                             desc->n_q_heads, desc->window, st);
    if (e == hipSuccess)
        e = spark::launch_prune_topp(static_cast<const uint16_t *>(k_bf16), desc->k_token_stride, desc->k_head_stride,
                                     cu_seqlens, static_cast<uint8_t *>(packed_out), L, p_basis_points, st);
    return e == hipSuccess ? SPARK_OK : SPARK_ERR_HIP;
}

spark_status spark_decode_attn_topp(const spark_desc *desc, const void *q_bf16, const void *packed, const void *v_bf16,
                                    const int32_t *cu_seqlens, void *out, void *workspace, size_t workspace_bytes,
                                    void *hip_stream)
{
    if (!v_bf16) return SPARK_ERR_INVALID_ARG;
    if (desc && (desc->pack_dtype != SPARK_PACK_BF16 || desc->stats)) return SPARK_ERR_UNSUPPORTED;
    return decode_common(desc, q_bf16, packed, v_bf16, nullptr, cu_seqlens, out, workspace, workspace_bytes, hip_stream,
                         nullptr, nullptr, nullptr, 0, 0, true);
}

spark_status spark_unpack_topp(const spark_desc *desc, const void *packed, uint32_t *mask_out, int32_t *count_out,
                               void *vals_out, float *mu_out, float *a_out, void *hip_stream)
{
    spark_status why;
    if (!desc_ok(desc, &why)) return why;
    if (!packed) return SPARK_ERR_INVALID_ARG;
    const hipError_t e = spark::launch_unpack_topp(static_cast<const uint8_t *>(packed), topp_layout_of(desc), mask_out,
                                                   count_out, static_cast<uint16_t *>(vals_out), mu_out, a_out,
                                                   static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SPARK_OK : SPARK_ERR_HIP;
}

// ---------------------------------------------------------------- decode without a caller-provided workspace

// Split partials and arrival counters of spark_decode_attn_static: one array per GPU, held until the process
// ends.  In host code this name is only a handle for hipGetSymbolAddress; kernels get the looked-up address.
static __device__ __align__(256) unsigned char scratch[SPARK_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];      // device address of `scratch` on each GPU, looked up on first use
std::mutex g_scratch_mutex;

// address of this GPU's copy of the array (the current device's), or nullptr after a runtime error
void *scratch_address()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

spark_status spark_decode_attn_static(const spark_desc *desc, const void *q_bf16, const void *packed,
                                      const void *v_bf16, const int32_t *cu_seqlens, void *out, void *hip_stream)
{
    spark_status why;
    if (!desc_ok(desc, &why)) return why;
    if (!v_bf16) return SPARK_ERR_INVALID_ARG;
    // the balanced cut of a ragged batch needs more partial slots than the chunked one: where only the chunked
    // one fits the array, that one is used
    bool balanced = true;
    size_t need = spark_decode_workspace(desc);
    if (need > (size_t)SPARK_STATIC_WORKSPACE_BYTES) {
        balanced = false;
        need = partial_slots(desc, false) * (SPARK_D + 2) * sizeof(float) + counter_bytes(desc);
    }
    if (need > (size_t)SPARK_STATIC_WORKSPACE_BYTES) return SPARK_ERR_WORKSPACE_TOO_SMALL;
    void *ws = scratch_address();
    if (!ws) return SPARK_ERR_HIP;
    // the array keeps whatever the last call on this GPU left: the counters must start at zero (a small fill
    // kernel, not a memset node, so the call can be captured into a graph); partial states are written before
    // they are read
    if (spark::launch_zero_counters(static_cast<uint32_t *>(ws), desc->batch * desc->n_kv_heads,
                                    static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return SPARK_ERR_HIP;
    return decode_common(desc, q_bf16, packed, v_bf16, nullptr, cu_seqlens, out, ws, SPARK_STATIC_WORKSPACE_BYTES,
                         hip_stream, nullptr, nullptr, nullptr, 0, 0, false, balanced);
}

}  // extern "C"
