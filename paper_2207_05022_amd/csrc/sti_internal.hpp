// Internal declarations shared by the translation units of libsti (HIP, gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include "sti.h"

namespace sti {

constexpr int kMaxShardsPerLayer = 64;   // sti_dims.n_heads upper bound
constexpr int kInlineShards = 64;        // shard tables up to this size travel as kernel arguments

// Device-side view of one shard version.
struct ShardDesc {
    const void *data;       // packed stream or float32 values
    const float *codebook;  // 2^bits centroids (unused for 32)
    int32_t bits;           // 2..6 or 32
    int32_t tag;            // original shard id inside its layer
    const uint32_t *outlier_pos;   // distinct offsets of the outlier dictionary
    const float *outlier_val;      // their original float32 weights
    uint32_t n_outliers;
    uint32_t pad;
};

struct InlineShardTable {
    ShardDesc d[kInlineShards];
};

// ---- decode.hip -----------------------------------------------------------
// Decode n_shards shards of n weights each into out[s*n + j].  `table` is a
// device pointer to n_shards descriptors, or NULL to use `inline_table`.
hipError_t launch_decode(const ShardDesc *table, const InlineShardTable *inline_table, int n_shards,
                         uint64_t n, void *out, sti_dtype out_dtype, hipStream_t stream);

// Put the bookkept outliers back: out[s*n + pos] = round_to(out_dtype, val) for every entry of
// every shard's outlier dictionary (offsets >= n are ignored).  Runs after launch_decode.
hipError_t launch_patch_outliers(const ShardDesc *table, const InlineShardTable *inline_table,
                                 int n_shards, uint32_t max_outliers, uint64_t n, void *out,
                                 sti_dtype out_dtype, hipStream_t stream);
// Same for the fragment-tiled binary16 working buffer written by launch_decode_tiled.
hipError_t launch_patch_outliers_tiled(const InlineShardTable &table, int n_shards,
                                       uint32_t max_outliers, int d, int dh, int f, void *out,
                                       hipStream_t stream);

// Decode n_shards shards of a layer (d, dh, f geometry) into the fragment-tiled binary16
// working buffer out[n_shards][Wsh] used by the matrix-core GEMM (see weight_loader.hpp).
hipError_t launch_decode_tiled(const InlineShardTable &table, int n_shards, int d, int dh, int f,
                               void *out, hipStream_t stream);
// Same with the table in device memory (any number of shards, e.g. every layer of a model in
// one launch): shard p is written at out + p * Wsh * 2 bytes.
hipError_t launch_decode_tiled_table(const ShardDesc *device_table, int n_shards, int d, int dh, int f,
                                     void *out, hipStream_t stream);

// ---- layer kernels ----------------------------------------------------------
// The four projections of a layer over its present shards, seen as GEMMs
// C[T x N] = A[T x K] * W^T whose weight operand is cut into per-shard blocks:
enum GemmKind : int32_t {
    GEMM_QKV = 0,       // blocks along N: block p = [3*dh x d] (Wq,Wk,Wv of shard p); + bq|bk|bv
    GEMM_FFN_UP = 1,    // blocks along N: block p = [f x d];   + b1 slice, then GELU
    GEMM_OUT = 2,       // blocks along K: block p = [d x dh];  + bo[n] + residual
    GEMM_FFN_DOWN = 3,  // blocks along K: block p = [d x f];   + b2[n] + residual
    // wide-tile kernel only, sequences of exactly 128 tokens: a 128 x 384 tile is the Q, K, V of
    // two heads of one sequence, and the workgroup goes on to those heads' attention; C is then
    // the context buffer [T x m*dh] and no Q/K/V buffer is written
    GEMM_QKV_ATTN = 4
};

struct GemmBlock {
    const void *w;          // start of the block's weights: float32 values, or a k-bit stream
    const float *codebook;  // centroids when bits <= 6
    int32_t bits;           // 2..6, 32; 17 = fragment-tiled binary16 working buffer
    int32_t shard;          // original shard id (selects the bias slice)
};

struct GemmBlocks {
    GemmBlock b[kMaxShardsPerLayer];
};

struct GemmProblem {
    GemmKind kind;
    int32_t T;          // rows of A and C
    int32_t n_blocks;   // present shards
    int32_t block_rows; // N-split: rows per block; K-split: N (= d)
    int32_t block_cols; // N-split: K (= d);        K-split: columns per block
    int32_t d_head;     // QKV bias selection
    const void *A;      // [T x K], row stride lda elements
    int32_t lda;
    void *C;            // [T x N], row stride ldc elements
    int32_t ldc;
    const float *bias0, *bias1, *bias2;  // QKV: bq,bk,bv; FFN_UP: b1; OUT/FFN_DOWN: bias[N]
    const void *resid;  // OUT/FFN_DOWN: [T x N] residual, row stride ldr
    int32_t ldr;
    // wide-tile kernel, OUT/FFN_DOWN only: with k_splits > 1 the K range is also split over
    // that many workgroups per tile, C is float32 and takes the raw partial sums of split s
    // at C + s * partial_stride (bias and residual are left to launch_layernorm)
    int32_t k_splits;
    int64_t partial_stride;
    const int32_t *key_lengths;   // GEMM_QKV_ATTN: real positions per sequence (device, may be null)
    // wide-tile kernel, GEMM_QKV and GEMM_QKV_ATTN: workgroups beyond those of the tiles (next_workgroups of them, on compute
    // units the tiles leave idle) decompress next_shards shards - the next layer's - from the device
    // table next_table into the working buffer next_out; next_workgroups == 0: nothing of the kind
    const ShardDesc *next_table;
    void *next_out;
    int32_t next_shards, next_workgroups, next_ffn_per_shard;
};

// float32 path (layer_f32.hip): A, C, resid are float32; weights are float32 blocks.
hipError_t launch_gemm_f32(const GemmProblem &p, const GemmBlocks &blocks, hipStream_t stream);
// qkv [T x m*3*dh] float32 (per shard: q, k, v each dh wide) -> ctx [T x m*dh] float32.
// key_lengths (device, [B], may be null): keys of sequence b beyond key_lengths[b] take no part.
hipError_t launch_attention_f32(const float *qkv, float *ctx, int B, int L, int m, int dh,
                                const int32_t *key_lengths, hipStream_t stream);

// binary16 MFMA path (gemm_wide.hip, attention_mfma.hip): A and C are binary16.  QKV / FFN_UP
// apply bias (and GELU); OUT / FFN_DOWN add bias[N] and the binary16 residual, leaving the
// LayerNorm to launch_layernorm_f16in (or, with k_splits > 1, leave float32 partial sums that
// launch_layernorm completes, like the few-token variant below).  Every block is a cell array
// of the fragment-tiled binary16 working buffer (bits == kTiledBits).
hipError_t launch_gemm_wide(const GemmProblem &p, const GemmBlocks &blocks, hipStream_t stream);
bool gemm_wide_supported(const GemmProblem &p, const GemmBlocks &blocks);
// whether the Q/K/V projection of B sequences of L tokens over m heads should go out as GEMM_QKV_ATTN
bool gemm_wide_fuses_attention(int B, int L, int m, int dh);
// workgroups a Q/K/V launch (GEMM_QKV or GEMM_QKV_ATTN; kind, T, n_blocks, block_rows, block_cols set)
// can give to the next layer's decompression: one per compute unit that its tiles leave idle (0: none to
// spare, decompress with a launch of its own)
int gemm_wide_spare_workgroups(const GemmProblem &p);
// K splits across workgroups the wide-tile kernel wants for this problem (1 = none), and the
// largest value it can return for T tokens and N output columns (workspace sizing)
int gemm_wide_k_splits(const GemmProblem &p);
int gemm_wide_max_k_splits(int64_t T, int N);
hipError_t launch_attention_mfma(const void *qkv, void *ctx, int B, int L, int m, int dh,
                                 const int32_t *key_lengths, hipStream_t stream);

// Few-token variant of the MFMA GEMM (gemm_skinny.hip): T <= kSkinnyMaxTokens, split-K inside the
// workgroup and, for the K-split kinds, across `k_splits` workgroups that write float32
// partial sums at C + s * partial_stride (to be added by launch_layernorm).
constexpr int kSkinnyMaxTokens = 256;
constexpr int kSkinnyMaxSplits = 8;
int skinny_k_splits(const GemmProblem &p);
hipError_t launch_gemm_skinny(const GemmProblem &p, const GemmBlocks &blocks, int k_splits,
                              int64_t partial_stride, hipStream_t stream);

// rowops.hip
// v = sum_{s < n_partials} pre[s * partial_stride + t*d + :] + bias[:] + resid[t][:]  (n_partials may be 0);
// y[t][:] = LayerNorm(v) * g + b.  pre float32; bias (float32 [d]) and resid_f16 (binary16
// [T x d]) may be NULL; y of out_dtype.
hipError_t launch_layernorm(const float *pre, int n_partials, int64_t partial_stride,
                            const float *bias, const void *resid_f16, void *y, sti_dtype out_dtype,
                            const float *g, const float *b, int T, int d, float eps,
                            hipStream_t stream);
// y[t][:] = LayerNorm(pre_f16[t][:]) * g + b for rows that already hold sum + bias + residual.
hipError_t launch_layernorm_f16in(const void *pre_f16, void *y, sti_dtype out_dtype, const float *g,
                                  const float *b, int T, int d, float eps, hipStream_t stream);
// elementwise conversion between activation types
hipError_t launch_convert(const void *src, sti_dtype src_dtype, void *dst, sti_dtype dst_dtype,
                          uint64_t n, hipStream_t stream);

// Kernel launches of the entry points go through launch(): while per-kernel timing is on
// (sti_profile_begin), the launch carries the two events the profiler handed out, which then
// hold the dispatch's own begin and end time stamps -- the same stamps a kernel trace reads.
// (Two events recorded around a launch read about 2.5 us more than the kernel lasts: the
// record-to-start latency.)  Without timing it is an ordinary launch.
struct LaunchEvents {
    hipEvent_t start = nullptr, stop = nullptr;
};
LaunchEvents take_launch_events();   // api.hip; nulls unless a timed launch is pending on this thread

template <typename... P, typename... A>
inline void launch(void (*kernel)(P...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream, A... args)
{
    const LaunchEvents ev = take_launch_events();
    if (ev.start)
        hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds_bytes, stream, ev.start, ev.stop, 0, (P)args...);
    else
        hipLaunchKernelGGL(kernel, grid, block, (uint32_t)lds_bytes, stream, (P)args...);
}

}  // namespace sti
