// Host side of decode attention: parameter block, choice of the query-group instantiation, counter reset.
// The kernel template is in spark_decode_kernel.h; its instantiations are compiled in spark_decode_g*.hip.
#include "spark_decode_kernel.h"

namespace spark {

extern template hipError_t launch_g<1>(const DecodeParams &, int, hipStream_t);
extern template hipError_t launch_g<2>(const DecodeParams &, int, hipStream_t);
extern template hipError_t launch_g<4>(const DecodeParams &, int, hipStream_t);
extern template hipError_t launch_g<8>(const DecodeParams &, int, hipStream_t);
extern template hipError_t launch_g<16>(const DecodeParams &, int, hipStream_t);

// Zeroes the arrival counters of a fresh workspace.
__global__ void spark_zero_kernel(uint32_t *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// Timeline buffer of the measurement aid spark_decode_timeline (process-wide; NULL = off)
namespace {
unsigned long long *g_timeline = nullptr;
size_t g_timeline_blocks = 0;
}  // namespace

void set_decode_timeline(unsigned long long *device_words, size_t blocks)
{
    g_timeline = device_words;
    g_timeline_blocks = device_words ? blocks : 0;
}

hipError_t launch_decode_attn(const uint16_t *q, const uint8_t *packed, const uint16_t *v, int64_t v_tok_stride,
                              int64_t v_head_stride, const uint8_t *packed_v, const SparkLayout *Lv,
                              const int32_t *cu, float *part_acc, float *part_ml,
                              uint32_t *counters, int Hq, const DecodePlan &plan, float softmax_scale, const SparkLayout &L,
                              void *out, int out_f32, const uint16_t *tail_k, const uint16_t *tail_v,
                              const int32_t *tail_len, int tail_cap, int rec, uint64_t seed, hipStream_t st)
{
    DecodeParams P;
    P.q = q;
    P.packed = packed;
    P.v = v;
    P.packed_v = packed_v;
    P.Lv = Lv ? *Lv : L;
    P.v_tok_stride = v_tok_stride;
    P.v_head_stride = v_head_stride;
    P.cu = cu;
    P.part_acc = part_acc;
    P.part_ml = part_ml;
    P.counters = counters;
    P.out = out;
    P.out_f32 = out_f32;
    P.Hq = Hq;
    P.Hkv = L.n_kv_heads;
    P.fixed_splits = plan.fixed_splits;
    P.chunk_tiles = plan.chunk_tiles;
    P.nchunk_max = plan.nchunk_max;
    // balanced mode: dense values, degenerate recovery, rows of one length, query groups up to 8 (else chunks)
    P.warm_waves = (!packed_v && rec == 0 && !L.topp && Hq / L.n_kv_heads <= 8) ? plan.warm_waves : 0;
    P.tail_slots = plan.tail_slots;
    P.ntail = tail_k ? plan.tail_slots : 0;
    P.tail_base = (int64_t)plan.chunk_ids * Hq;
    P.tail_k = tail_k;
    P.tail_v = tail_v;
    P.tail_len = tail_len;
    P.tail_cap = tail_cap;
    P.rec = rec;
    P.seed_lo = (uint32_t)seed;
    P.seed_hi = (uint32_t)(seed >> 32);
    P.scale_log2 = softmax_scale * 1.44269504088896340736f;
    P.L = L;
    const int G = P.Hq / P.Hkv;
    const int nblocks = P.Hkv * ((P.warm_waves > 0 ? P.warm_waves / kDecodeWaves : P.nchunk_max) + L.batch * P.ntail);
    P.trace = (g_timeline != nullptr && (size_t)nblocks <= g_timeline_blocks) ? g_timeline : nullptr;
    switch (G) {
        case 1: return launch_g<1>(P, nblocks, st);
        case 2: return launch_g<2>(P, nblocks, st);
        case 4: return launch_g<4>(P, nblocks, st);
        case 8: return launch_g<8>(P, nblocks, st);
        case 16: return launch_g<16>(P, nblocks, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_zero_counters(uint32_t *counters, int n, hipStream_t st)
{
    hipLaunchKernelGGL(spark_zero_kernel, dim3((n + 255) / 256), dim3(256), 0, st, counters, n);
    return hipGetLastError();
}

}  // namespace spark
