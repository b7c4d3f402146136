// Host-side helpers shared by the entry points in api.hip and pipeline.hip.
#pragma once
#include "sti_internal.hpp"

namespace sti {

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline bool valid_packed_bits(int b) { return b >= 2 && b <= 6; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

#define STI_TRY(expr)                                 \
    do {                                              \
        if ((expr) != hipSuccess) return STI_ERR_HIP; \
    } while (0)

// Offsets of the scratch regions of one layer call inside the caller's workspace.
struct WorkspaceLayout {
    size_t w32 = 0, w16 = 0, act[2] = {0, 0}, qkv = 0, ctx = 0, pre = 0, h = 0, u = 0, table = 0, total = 0;
    int w16_layers = 1;   // layers the binary16 working buffer holds at once (a ring: layer l in slot l % w16_layers)
    int decode_group = 1; // layers that one decompression launch of sti_model_forward takes (<= w16_layers)
};
// model_layers > 1 (sti_model_forward with room for it): a ring of binary16 working buffers - as many
// layers as one decompression launch takes (64 MiB worth), at least two, so that a layer can be
// decompressed while the one before it computes - and the device copy of the whole model's shard table.
WorkspaceLayout workspace_layout(const sti_dims &d, int64_t T, sti_precision prec, int model_layers = 1);

sti_status check_dims(const sti_dims *dims, int batch, int seq, sti_precision prec);
sti_status check_decode_shard(const sti_shard &s);   // bitwidth 2..6 or 32, pointers, alignment
sti_status check_params(const sti_layer_params *p);
sti_status check_io(const void *x, void *y, sti_dtype io, int64_t T, int d);

// One layer over shards[M] (bitwidth 0 = absent), arguments already validated.  `in` is
// float32 (F32 precision) or binary16 (MFMA precision); `out` is written as out_dtype.
// What a layer's Q/K/V launch (many-token route) does on the compute units its tiles leave idle:
// decompress the following layer (n_shards shards of the device table into the working buffer `out`,
// dictionaries of outliers not applied) with `workgroups` workgroups.
struct NextLayerDecode {
    const ShardDesc *table;
    int n_shards;
    void *out;
    int workgroups;
};
// Workgroups such a launch has to spare for a layer of m present shards (0: the layer does not go
// through the many-token route, or its projection fills the chip).
int spare_decode_workgroups(const sti_dims &d, int B, int Lseq, int m, sti_precision prec);

sti_status run_layer(const sti_dims &d, const sti_shard *shards, const sti_layer_params &prm,
                     const void *in, void *out, sti_dtype out_dtype, int B, int Lseq,
                     sti_precision prec, uint8_t *ws, const WorkspaceLayout &wl, hipStream_t stream,
                     const void *predecoded = nullptr, const int32_t *key_lengths = nullptr,
                     const NextLayerDecode *next = nullptr);
// `predecoded`: the layer's present shards already sit there in fragment-tiled binary16 order
// (outliers applied); run_layer then decompresses nothing.
// `key_lengths` (device, [B]): real positions per padded sequence; null = every position is real.
// `next` (only with `predecoded`, and only when spare_decode_workgroups says so for this layer).
sti_status check_key_lengths(const int32_t *key_lengths);   // non-null, 4-byte aligned

}  // namespace sti
