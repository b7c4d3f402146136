// Internal declarations shared by the translation units of libsti (HIP, gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
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
    int32_t tag;            // caller-defined (original shard id in layer kernels)
};

struct InlineShardTable {
    ShardDesc d[kInlineShards];
};

// ---- decode.hip -----------------------------------------------------------
// Decode n_shards shards of n weights each into out[s*n + j].  `table` is a
// device pointer to n_shards descriptors, or NULL to use `inline_table`.
hipError_t launch_decode(const ShardDesc *table, const InlineShardTable *inline_table, int n_shards,
                         uint64_t n, void *out, sti_dtype out_dtype, hipStream_t stream);

// ---- reference-precision (float32) layer kernels: layer_f32.hip -------------
struct GemmBlock {
    const void *w;          // weights of this block (float32 for the f32 path; stream/float32 for mfma)
    const float *codebook;  // mfma path only
    int32_t bits;           // mfma path only
    int32_t shard;          // original shard id (selects bias slices)
};

struct GemmBlocks {
    GemmBlock b[kMaxShardsPerLayer];
};

enum GemmKind : int32_t {
    GEMM_QKV = 0,      // N-split: block p holds [3*dh x d]; bias from bq/bk/bv of shard
    GEMM_FFN_UP = 1,   // N-split: block p holds [f x d]; bias b1 of shard; GELU
    GEMM_OUT = 2,      // K-split: block p holds [d x dh]; + bias[n] + residual
    GEMM_FFN_DOWN = 3  // K-split: block p holds [d x f];  + bias[n] + residual
};

struct LayerGeom {
    int32_t d, M, dh, f, m;   // m = number of present shards
    int32_t B, L, T;
    float eps;
};

}  // namespace sti
