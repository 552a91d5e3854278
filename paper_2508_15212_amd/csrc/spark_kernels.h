// Internal: launch functions implemented next to their kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spark_layout.h"

namespace spark {

// Immediate of s_waitcnt on gfx9-family parts: vmcnt in bits [3:0] and [15:14] (vector memory loads AND stores
// of this wavefront still outstanding), expcnt in bits [6:4], lgkmcnt in bits [11:8] (LDS, scalar memory).  A
// field left at its maximum does not wait.  This one waits for vmcnt == 0 only: every global load has returned
// and every global store of the wavefront has been acknowledged by the memory system.
constexpr int kWaitVmcnt0 = (0 << 0) | (0 << 14) | (7 << 4) | (15 << 8);      // = 0x0F70

struct DecodeParams;

// How the decode grid cuts sequences into blocks (chosen on the host from the description alone).
struct DecodePlan {
    int fixed_splits;   // > 0: every sequence is cut into this many chunks
    int chunk_tiles;    // else: a sequence spanning ntile tiles gets max(1, ceil(ntile / chunk_tiles)) chunks
    int nchunk_max;     // upper bound on the number of chunks in the batch (grid = nchunk_max * Hkv + tail blocks)
    int tail_slots;     // partial slots reserved per (batch, q head) for appended rows
    int warm_waves;     // > 0: the balanced mode may be used, with this many wavefronts per KV head; the launch
                        // falls back to the chunked cut for the kernel variants that have no balanced form
    int chunk_ids;      // chunk ids the workspace has partial slots for: >= nchunk_max, and >= the balanced
                        // mode's warm_waves + 2 * batch; the appended rows' slots follow at chunk_ids * Hq
};

// measurement aid: later decode launches of this process file eight 64-bit words per block into `device_words`
// (room for `blocks` blocks; launches with more blocks file nothing); NULL switches it off
void set_decode_timeline(unsigned long long *device_words, size_t blocks);

hipError_t launch_prune(const uint16_t *k, int64_t k_tok_stride, int64_t k_head_stride, const uint16_t *qwin,
                        const int32_t *cu, uint8_t *packed, const SparkLayout &L, int Hq, int W, hipStream_t st);

// value-cache channel pruning: per (token, KV head) the L.T channels of largest |v| (L from spark_make_values_layout)
hipError_t launch_prune_values(const uint16_t *v, int64_t v_tok_stride, int64_t v_head_stride, uint8_t *packed,
                               const SparkLayout &L, hipStream_t st);

hipError_t launch_unpack(const uint8_t *packed, const SparkLayout &L, uint32_t *mask_out, void *vals_out,
                         float *mu_out, float *scale_out, float *a_out, float *mu_all_out, float *sigma_out,
                         hipStream_t st);

// q [B,Hq,128] bf16; the caller splits the workspace into part_acc / part_ml / counters.
// Values are either dense (v, strides; packed_v = NULL) or a packed value cache (packed_v, Lv; v = NULL).
// Partial slots: plan.chunk_ids * Hq, then batch * Hq * plan.tail_slots; tail_k != NULL adds the appended rows
// [B, tail_cap, Hkv, 128].
hipError_t launch_decode_attn(const uint16_t *q, const uint8_t *packed, const uint16_t *v, int64_t v_tok_stride,
                              int64_t v_head_stride, const uint8_t *packed_v, const SparkLayout *Lv,
                              const int32_t *cu, float *part_acc, float *part_ml,
                              uint32_t *counters, int Hq, const DecodePlan &plan, float softmax_scale, const SparkLayout &L,
                              void *out, int out_f32, const uint16_t *tail_k, const uint16_t *tail_v,
                              const int32_t *tail_len, int tail_cap, int rec, uint64_t seed, hipStream_t st);

hipError_t launch_zero_counters(uint32_t *counters, int n, hipStream_t st);

// channel weights a, 1/a (and the key cache's header) alone
hipError_t launch_window_stat(const uint16_t *qwin, uint8_t *packed, const SparkLayout &L, int Hq, int W, hipStream_t st);

// top-p variant (L from spark_make_topp_layout; the channel weights must have been written before)
hipError_t launch_prune_topp(const uint16_t *k, int64_t k_tok_stride, int64_t k_head_stride, const int32_t *cu,
                             uint8_t *packed, const SparkLayout &L, int p_bp, hipStream_t st);
hipError_t launch_unpack_topp(const uint8_t *packed, const SparkLayout &L, uint32_t *mask_out, int32_t *count_out,
                              uint16_t *vals_out, float *mu_out, float *a_out, hipStream_t st);

}  // namespace spark
