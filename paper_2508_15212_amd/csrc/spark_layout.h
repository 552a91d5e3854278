// Packed key-cache layout shared by the prune, decode and unpack kernels.
//
// The cache is a header, the per-(batch, KV head) channel weights a and 1/a, and an
// array of TILES.  A tile holds 64 consecutive global tokens of one KV head.  Every
// token owns one ROW of `ndw` 32-bit words:
//
//   bf16 storage : [ m0 m1 m2 m3 | mu | v0 v1 ... v(nv-1) | pad ]   nv = ceil(T/2)
//   int8 storage : [ m0 m1 m2 m3 | mu | scale | c0 ... c(nv-1) | pad ]   nv = ceil(T/4)
//   value cache  : [ m0 m1 m2 m3 | v0 v1 ... v(nv-1) | pad ]        (pruned entries are dropped: no statistic)
//   bf16 + stats : [ m0 m1 m2 m3 | mu | mu_all | sigma_all | v0 ... v(nv-1) | pad ]   (for the sampled recovery functions)
//   int8 + stats : [ m0 m1 m2 m3 | mu | scale | mu_all | sigma_all | c0 ... c(nv-1) | pad ]
//   top-p rows   : [ m0 m1 m2 m3 | mu | count ]        the kept entries live in a value stream, see below
//
// m0..m3 is the 128-bit channel mask (bit j%32 of word j/32 = channel j kept), mu the
// mean saliency of the pruned channels, v* the kept entries in ascending channel order
// (two bf16 per word, the lower channel in the low half; or four int8 codes per word).
// ndw is rounded up to an even number so a row is a whole number of 8-byte units.
//
// Inside a tile the rows are interleaved so that a wavefront whose lane l owns token l
// reads the tile with fully coalesced 16-byte (then one 8-byte) accesses:
//
//   word d of token t lives at   (d/4)*1024 + t*16 + (d%4)*4          for d <  4*nq
//                                nq*1024 + t*8 + (d - 4*nq)*4         for the 2-word tail
//
// with nq = ndw/4 full 16-byte sections.  Tiles are ordered [KV head][tile index]; the
// tile index of global token n is n/64, so a tile may straddle two sequences.
//
// The top-p variant keeps a different number of channels in every row.  Its tiles hold only the fixed part of
// the rows (24 bytes: mask, mu, count); the kept entries of a KV head form one VALUE STREAM of 32-bit words:
// tile by tile, inside a tile token by token, every row rounded up to a whole word (two bf16 per word, the
// lower channel in the low half, an unused upper half 0).  A DIRECTORY uint32 [Hkv][n_tiles + 1] gives the
// word offset of every tile in its head's stream (an exclusive prefix sum; the last entry is the head's
// length).  The stream is sized for the worst case (every row keeps all 128 channels); only its used part
// is ever read.
#pragma once
#include <stddef.h>
#include <stdint.h>

#define SPARK_D 128
#define SPARK_TILE_TOKENS 64
#define SPARK_MAGIC 0x53504B31u /* "SPK1" */

#if defined(__HIPCC__) || defined(__HIP__)
#define SPARK_HD __host__ __device__
#else
#define SPARK_HD
#endif

struct SparkLayout {
    int32_t T;            // kept channels per row
    int32_t int8;         // 1 = int8 codes + scale
    int32_t values;       // 1 = packed VALUE cache: rows carry no mu word and there is no a / 1/a section
    int32_t stats;        // 1 = rows also carry the mean and standard deviation of the saliency over all channels
    int32_t nv;           // value words per row
    int32_t val0;         // index of the first value word in a row
    int32_t ndw;          // words per row (even)
    int32_t nq;           // full 16-byte sections per row
    int32_t tail2;        // 1 if a 2-word tail section follows
    int32_t tile_bytes;   // 64 * 4 * ndw
    int32_t batch, n_kv_heads;
    int64_t total_tokens;
    int64_t n_tiles;      // ceil(total_tokens / 64)
    int64_t off_a;        // float [batch][Hkv][128]
    int64_t off_inva;     // float [batch][Hkv][128]   1/a, 0 where a == 0
    int64_t off_tiles;    // tiles [Hkv][n_tiles]
    int64_t total_bytes;
    // top-p variant only
    int32_t topp;         // 1 = rows keep a per-row number of channels (values in the stream)
    int32_t pad_;
    int64_t off_dir;      // uint32 [Hkv][n_tiles + 1]
    int64_t off_vals;     // value streams [Hkv][vals_head_words] 32-bit words
    int64_t vals_head_words;   // capacity of one head's stream: n_tiles * 64 rows * 64 words
};

static inline SPARK_HD SparkLayout spark_make_layout(int T, int int8, int batch, int n_kv_heads,
                                                     int64_t total_tokens, int stats = 0)
{
    SparkLayout L;
    L.T = T;
    L.int8 = int8;
    L.values = 0;
    L.stats = stats;
    L.nv = int8 ? (T + 3) / 4 : (T + 1) / 2;
    L.val0 = 5 + (int8 ? 1 : 0) + (stats ? 2 : 0);
    int ndw = L.val0 + L.nv;
    L.ndw = (ndw + 1) & ~1;
    L.nq = L.ndw / 4;
    L.tail2 = (L.ndw % 4) ? 1 : 0;
    L.tile_bytes = SPARK_TILE_TOKENS * 4 * L.ndw;
    L.batch = batch;
    L.n_kv_heads = n_kv_heads;
    L.total_tokens = total_tokens;
    L.n_tiles = (total_tokens + SPARK_TILE_TOKENS - 1) / SPARK_TILE_TOKENS;
    const int64_t abytes = (int64_t)batch * n_kv_heads * SPARK_D * 4;
    const int64_t apad = (abytes + 255) & ~(int64_t)255;
    L.off_a = 256;
    L.off_inva = L.off_a + apad;
    L.off_tiles = L.off_inva + apad;
    L.total_bytes = L.off_tiles + (int64_t)n_kv_heads * L.n_tiles * L.tile_bytes;
    L.topp = 0;
    L.pad_ = 0;
    L.off_dir = L.off_vals = L.vals_head_words = 0;
    return L;
}

// Top-p cache: rows [ m0 m1 m2 m3 | mu | count ] in the tiles, then the directory and the value streams.
static inline SPARK_HD SparkLayout spark_make_topp_layout(int batch, int n_kv_heads, int64_t total_tokens)
{
    SparkLayout L = spark_make_layout(SPARK_D, 0, batch, n_kv_heads, total_tokens);
    L.topp = 1;
    L.T = 0;              // no fixed count
    L.nv = 0;
    L.val0 = 6;
    L.ndw = 6;
    L.nq = 1;
    L.tail2 = 1;
    L.tile_bytes = SPARK_TILE_TOKENS * 4 * L.ndw;
    const int64_t tiles_end = L.off_tiles + (int64_t)n_kv_heads * L.n_tiles * L.tile_bytes;
    L.off_dir = (tiles_end + 255) & ~(int64_t)255;
    const int64_t dir_bytes = (int64_t)n_kv_heads * (L.n_tiles + 1) * 4;
    L.off_vals = (L.off_dir + dir_bytes + 255) & ~(int64_t)255;
    L.vals_head_words = L.n_tiles * SPARK_TILE_TOKENS * (SPARK_D / 2);
    // (256 bytes of padding behind the last stream: a reader may fetch whole 16-byte groups of a row's words)
    L.total_bytes = L.off_vals + (int64_t)n_kv_heads * L.vals_head_words * 4 + 256;
    return L;
}

// Packed value cache (value-channel pruning): same tiles, rows [ m0 m1 m2 m3 | v0 ... v(nv-1) | pad ].
static inline SPARK_HD SparkLayout spark_make_values_layout(int Tv, int n_kv_heads, int64_t total_tokens)
{
    SparkLayout L = spark_make_layout(Tv, 0, 0, n_kv_heads, total_tokens);
    L.values = 1;
    L.val0 = 4;
    const int ndw = L.val0 + L.nv;
    L.ndw = (ndw + 1) & ~1;
    L.nq = L.ndw / 4;
    L.tail2 = (L.ndw % 4) ? 1 : 0;
    L.tile_bytes = SPARK_TILE_TOKENS * 4 * L.ndw;
    L.total_bytes = L.off_tiles + (int64_t)n_kv_heads * L.n_tiles * L.tile_bytes;   // off_tiles = 256: batch = 0
    return L;
}

// byte offset of word d of token t inside a tile
static inline SPARK_HD int spark_tile_word_offset(const SparkLayout &L, int t, int d)
{
    const int q = d >> 2;
    if (q < L.nq) return q * 1024 + t * 16 + (d & 3) * 4;
    return L.nq * 1024 + t * 8 + (d - 4 * L.nq) * 4;
}
