// Shard decompression: k-bit dictionary indexes -> centroids (Section
// "quantization per shard"; the substitution loop of Section "Implementation").
//
// HBM-bound streaming kernel.  One workgroup decodes one chunk of one shard:
//  - the shard's codebook is rounded to the output type once and kept in LDS;
//  - work is cut into units of 8 indexes, which occupy exactly k bytes for
//    every k, so a unit is two aligned dword loads and a funnel shift;
//  - consecutive lanes take consecutive units, so each store instruction of a
//    wave writes one contiguous 1 KiB (f16/bf16) or 2 KiB (f32) span.
#include "sti_internal.hpp"
#include "weight_loader.hpp"

namespace sti {
namespace {

// 4 units per thread and nontemporal stores measured best on the 1 GiB stream (5.2 TB/s, the
// rate a plain kernel with the same 1 : 4.6 read : write ratio reaches on this chip).
#define STI_STORE(v, p) __builtin_nontemporal_store((v), (p))
constexpr int kThreads = 256;
constexpr int kUnitsPerThread = 4;                          // units of 8 weights
constexpr int kChunkUnits = kThreads * kUnitsPerThread;     // 1024 units = 8192 weights

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// ---- output element traits: LUT entries are stored as raw bit patterns ----
__device__ inline uint32_t f32_bits(float v) { return __builtin_bit_cast(uint32_t, v); }

__device__ inline uint16_t to_f16_bits(float v)
{
    uint32_t u = f32_bits(v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u)  // NaN: keep sign and top payload bits, set quiet bit
        return (uint16_t)(((u >> 16) & 0x8000u) | 0x7E00u | ((u & 0x7FFFFFu) >> 13));
    _Float16 h = (_Float16)v;  // v_cvt_f16_f32: round to nearest even, subnormals kept
    return __builtin_bit_cast(uint16_t, h);
}

__device__ inline uint16_t to_bf16_bits(float v)
{
    uint32_t u = f32_bits(v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    return (uint16_t)((u + 0x7FFFu + lsb) >> 16);
}

struct OutF32 {
    typedef uint32_t bits_t;
    static __device__ inline bits_t cvt(float v) { return f32_bits(v); }
};
struct OutF16 {
    typedef uint16_t bits_t;
    static __device__ inline bits_t cvt(float v) { return to_f16_bits(v); }
};
struct OutBF16 {
    typedef uint16_t bits_t;
    static __device__ inline bits_t cvt(float v) { return to_bf16_bits(v); }
};

// Store 8 consecutive outputs starting at element e (16-byte aligned address).
__device__ inline void store8(uint16_t *out, uint64_t e, const uint32_t v[8])
{
    u32x4 p;
    p.x = v[0] | (v[1] << 16);
    p.y = v[2] | (v[3] << 16);
    p.z = v[4] | (v[5] << 16);
    p.w = v[6] | (v[7] << 16);
    STI_STORE(p, (u32x4 *)(out + e));
}
__device__ inline void store8(uint32_t *out, uint64_t e, const uint32_t v[8])
{
    u32x4 a = {v[0], v[1], v[2], v[3]};
    u32x4 b = {v[4], v[5], v[6], v[7]};
    STI_STORE(a, (u32x4 *)(out + e));
    STI_STORE(b, (u32x4 *)(out + e + 4));
}

// 64-bit window holding the k bytes of unit u (bits beyond the stream read as 0).
template <int K>
__device__ inline uint64_t load_window(const uint8_t *data, uint64_t nbytes, uint64_t u)
{
    uint64_t b = u * (uint64_t)K;            // first byte of the unit
    uint64_t i0 = b >> 2;                    // dword holding it
    uint64_t ndw = nbytes >> 2;              // dwords lying fully inside the stream
    const uint32_t *dw = (const uint32_t *)data;
    if (i0 + 1 < ndw) {
        uint32_t lo = __builtin_nontemporal_load(dw + i0);
        uint32_t hi = __builtin_nontemporal_load(dw + i0 + 1);
        uint64_t w = ((uint64_t)hi << 32) | lo;
        return w >> ((uint32_t)(b & 3) * 8);
    }
    uint64_t w = 0;
    for (int t = 0; t < K; ++t)
        if (b + t < nbytes) w |= (uint64_t)data[b + t] << (8 * t);
    return w;
}

template <int K, typename Out>
__device__ inline void decode_packed_chunk(const uint8_t *data, uint64_t n, uint64_t unit0,
                                           const typename Out::bits_t *lut,
                                           typename Out::bits_t *out, bool vec_ok)
{
    const uint64_t nbytes = (n * K + 7) >> 3;
    const uint64_t n_units = (n + 7) >> 3;
    uint64_t w[kUnitsPerThread];
#pragma unroll
    for (int r = 0; r < kUnitsPerThread; ++r) {
        uint64_t u = unit0 + (uint64_t)r * kThreads + threadIdx.x;
        w[r] = (u < n_units) ? load_window<K>(data, nbytes, u) : 0;
    }
#pragma unroll
    for (int r = 0; r < kUnitsPerThread; ++r) {
        uint64_t u = unit0 + (uint64_t)r * kThreads + threadIdx.x;
        if (u >= n_units) continue;
        uint32_t v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = lut[(uint32_t)(w[r] >> (j * K)) & ((1u << K) - 1u)];
        uint64_t e = u * 8;
        if (vec_ok && e + 8 <= n) {
            store8(out, e, v);
        } else {
            for (int j = 0; j < 8; ++j)
                if (e + j < n) out[e + j] = (typename Out::bits_t)v[j];
        }
    }
}

template <typename Out>
__device__ inline void decode_raw_chunk(const float *data, uint64_t n, uint64_t unit0,
                                        typename Out::bits_t *out, bool vec_ok)
{
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const uint64_t n_units = (n + 7) >> 3;
#pragma unroll 4
    for (int r = 0; r < kUnitsPerThread; ++r) {
        uint64_t u = unit0 + (uint64_t)r * kThreads + threadIdx.x;
        if (u >= n_units) continue;
        uint64_t e = u * 8;
        uint32_t v[8];
        if (e + 8 <= n) {
            f32x4 a = __builtin_nontemporal_load((const f32x4 *)(data + e));
            f32x4 b = __builtin_nontemporal_load((const f32x4 *)(data + e + 4));
            v[0] = Out::cvt(a.x); v[1] = Out::cvt(a.y); v[2] = Out::cvt(a.z); v[3] = Out::cvt(a.w);
            v[4] = Out::cvt(b.x); v[5] = Out::cvt(b.y); v[6] = Out::cvt(b.z); v[7] = Out::cvt(b.w);
            if (vec_ok) {
                store8(out, e, v);
                continue;
            }
            for (int j = 0; j < 8; ++j) out[e + j] = (typename Out::bits_t)v[j];
        } else {
            for (int j = 0; j < 8; ++j)
                if (e + j < n) out[e + j] = Out::cvt(data[e + j]);
        }
    }
}

struct TableInline {
    InlineShardTable t;
    __device__ inline ShardDesc get(uint32_t s) const { return t.d[s]; }
};

template <typename Out, typename Table>
__global__ __launch_bounds__(kThreads) void decode_kernel(Table table, uint64_t n,
                                                          uint32_t chunks_per_shard,
                                                          typename Out::bits_t *out, int vec_ok)
{
    __shared__ typename Out::bits_t lut[64];
    const uint32_t s = blockIdx.x / chunks_per_shard;
    const uint32_t c = blockIdx.x - s * chunks_per_shard;
    const ShardDesc sd = table.get(s);
    const int bits = sd.bits;
    if (bits != 32) {
        if (threadIdx.x < (1u << bits)) lut[threadIdx.x] = Out::cvt(sd.codebook[threadIdx.x]);
        __syncthreads();
    }
    typename Out::bits_t *o = out + (uint64_t)s * n;
    const uint64_t unit0 = (uint64_t)c * kChunkUnits;
    const uint8_t *data = (const uint8_t *)sd.data;
    switch (bits) {
        case 2: decode_packed_chunk<2, Out>(data, n, unit0, lut, o, vec_ok); break;
        case 3: decode_packed_chunk<3, Out>(data, n, unit0, lut, o, vec_ok); break;
        case 4: decode_packed_chunk<4, Out>(data, n, unit0, lut, o, vec_ok); break;
        case 5: decode_packed_chunk<5, Out>(data, n, unit0, lut, o, vec_ok); break;
        case 6: decode_packed_chunk<6, Out>(data, n, unit0, lut, o, vec_ok); break;
        case 32: decode_raw_chunk<Out>((const float *)sd.data, n, unit0, o, vec_ok); break;
        default: break;
    }
}

template <typename Out>
hipError_t launch_typed(const ShardDesc *table, const InlineShardTable *inline_table, int n_shards,
                        uint64_t n, void *out, hipStream_t stream)
{
    const uint64_t n_units = (n + 7) / 8;
    const uint64_t chunks = (n_units + kChunkUnits - 1) / kChunkUnits;
    const uint64_t blocks = chunks * (uint64_t)n_shards;
    if (blocks == 0) return hipSuccess;
    if (blocks > 0x7FFFFFFFull || chunks > 0xFFFFFFFFull) return hipErrorInvalidValue;
    // vector stores need every shard's output to start on a 16-byte boundary
    const int vec_ok = (n % 8 == 0) ? 1 : 0;
    typedef typename Out::bits_t bits_t;
    if (table) {
        TablePtr t{table};
        launch((decode_kernel<Out, TablePtr>), dim3((uint32_t)blocks), dim3(kThreads), 0, stream, 
            t, n, (uint32_t)chunks, (bits_t *)out, vec_ok);
    } else {
        TableInline t;
        t.t = *inline_table;
        launch((decode_kernel<Out, TableInline>), dim3((uint32_t)blocks), dim3(kThreads), 0, stream, 
            t, n, (uint32_t)chunks, (bits_t *)out, vec_ok);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_decode(const ShardDesc *table, const InlineShardTable *inline_table, int n_shards,
                         uint64_t n, void *out, sti_dtype out_dtype, hipStream_t stream)
{
    switch (out_dtype) {
        case STI_F32: return launch_typed<OutF32>(table, inline_table, n_shards, n, out, stream);
        case STI_F16: return launch_typed<OutF16>(table, inline_table, n_shards, n, out, stream);
        case STI_BF16: return launch_typed<OutBF16>(table, inline_table, n_shards, n, out, stream);
    }
    return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------
// Working buffer for the matrix-core path (Section "Submodel execution": a buffer
// holding one layer of decompressed weights, shared by all layers) -- here binary16
// and fragment-tiled, so that the GEMM loads every weight fragment as one
// contiguous 1 KiB read.  One wave decodes one 32 x 64 cell with the same per-lane
// loader the fused GEMM uses.
// ---------------------------------------------------------------------------
namespace {

template <typename Table>
__global__ __launch_bounds__(256) void decode_tiled_kernel(Table tab, int total_cells,
                                                           int d, int dh, int f, uint8_t *out)
{
    __shared__ uint16_t lut[4][kLutEntries];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int cell = blockIdx.x * 4 + wave;
    if (cell >= total_cells) return;   // whole wave; no workgroup barrier is used
    decode_tiled_cell(tab, cell, d, dh, f, out, lut[wave], lane);
}

}  // namespace

// ---------------------------------------------------------------------------
// Outlier dictionary (Section "quantization per shard": the few weights that do not follow
// the Gaussian are preserved as-is; Section "Implementation": they keep a k-bit placeholder
// in the index matrix and their original weights and offsets are bookkept).  After the
// substitution pass the original weights are scattered back.  grid = shards x chunks, flattened
// (the shard count may pass the limit of the second grid dimension).
// ---------------------------------------------------------------------------
namespace {

template <typename Out, typename Table>
__global__ __launch_bounds__(256) void patch_outliers_kernel(Table table, uint64_t n, uint32_t chunks,
                                                             typename Out::bits_t *out)
{
    const uint32_t shard = blockIdx.x / chunks, chunk = blockIdx.x - shard * chunks;
    const ShardDesc sd = table.get(shard);
    typename Out::bits_t *o = out + (uint64_t)shard * n;
    for (uint32_t t = chunk * 256 + threadIdx.x; t < sd.n_outliers; t += chunks * 256) {
        const uint32_t pos = sd.outlier_pos[t];
        if (pos < n) o[pos] = Out::cvt(sd.outlier_val[t]);
    }
}

template <typename Out>
hipError_t patch_typed(const ShardDesc *table, const InlineShardTable *inline_table, int n_shards,
                       uint32_t max_outliers, uint64_t n, void *out, hipStream_t stream)
{
    uint32_t chunks = (max_outliers + 255) / 256;
    if (chunks > 1024) chunks = 1024;
    while ((uint64_t)chunks * (uint64_t)n_shards > 0x7FFFFFFFull) chunks = (chunks + 1) / 2;
    dim3 grid(chunks * (uint32_t)n_shards);
    typedef typename Out::bits_t bits_t;
    if (table) {
        TablePtr t{table};
        patch_outliers_kernel<Out, TablePtr><<<grid, 256, 0, stream>>>(t, n, chunks, (bits_t *)out);
    } else {
        TableInline t;
        t.t = *inline_table;
        patch_outliers_kernel<Out, TableInline><<<grid, 256, 0, stream>>>(t, n, chunks, (bits_t *)out);
    }
    return hipGetLastError();
}

// offset inside a shard -> byte offset inside its fragment-tiled image
__device__ inline int64_t tiled_byte_offset(uint32_t pos, int d, int dh, int f)
{
    const int64_t o_o = (int64_t)3 * dh * d, o_1 = (int64_t)4 * dh * d, o_2 = o_1 + (int64_t)f * d;
    int64_t sub_off;
    int cols;
    if (pos < o_o) { sub_off = 0; cols = d; }
    else if (pos < o_1) { sub_off = o_o; cols = dh; }
    else if (pos < o_2) { sub_off = o_1; cols = d; }
    else { sub_off = o_2; cols = f; }
    const int64_t rel = pos - sub_off;
    const int row = (int)(rel / cols), col = (int)(rel - (int64_t)row * cols);
    const int lane = ((col & 63) >> 5) * 32 + (row & 31), q = (col & 31) >> 3, e = col & 7;
    return sub_off * 2 + tiled_cell_offset(row >> 5, col >> 6, cols) + q * 1024 + lane * 16 + e * 2;
}

__global__ __launch_bounds__(256) void patch_outliers_tiled_kernel(InlineShardTable tab, int d,
                                                                   int dh, int f, uint8_t *out)
{
    const ShardDesc sd = tab.d[blockIdx.y];
    const int64_t wsh = (int64_t)d * (4 * dh + 2 * f);
    uint8_t *o = out + (int64_t)blockIdx.y * wsh * 2;
    for (uint32_t t = blockIdx.x * 256 + threadIdx.x; t < sd.n_outliers; t += gridDim.x * 256) {
        const uint32_t pos = sd.outlier_pos[t];
        if (pos < wsh) *(uint16_t *)(o + tiled_byte_offset(pos, d, dh, f)) = to_f16_bits(sd.outlier_val[t]);
    }
}

}  // namespace

hipError_t launch_patch_outliers(const ShardDesc *table, const InlineShardTable *inline_table,
                                 int n_shards, uint32_t max_outliers, uint64_t n, void *out,
                                 sti_dtype out_dtype, hipStream_t stream)
{
    if (n_shards <= 0 || max_outliers == 0 || n == 0) return hipSuccess;
    switch (out_dtype) {
        case STI_F32: return patch_typed<OutF32>(table, inline_table, n_shards, max_outliers, n, out, stream);
        case STI_F16: return patch_typed<OutF16>(table, inline_table, n_shards, max_outliers, n, out, stream);
        case STI_BF16: return patch_typed<OutBF16>(table, inline_table, n_shards, max_outliers, n, out, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_patch_outliers_tiled(const InlineShardTable &table, int n_shards,
                                       uint32_t max_outliers, int d, int dh, int f, void *out,
                                       hipStream_t stream)
{
    if (n_shards <= 0 || max_outliers == 0) return hipSuccess;
    uint32_t chunks = (max_outliers + 255) / 256;
    if (chunks > 1024) chunks = 1024;
    patch_outliers_tiled_kernel<<<dim3(chunks, n_shards), 256, 0, stream>>>(table, d, dh, f,
                                                                            (uint8_t *)out);
    return hipGetLastError();
}

hipError_t launch_decode_tiled(const InlineShardTable &table, int n_shards, int d, int dh, int f,
                               void *out, hipStream_t stream)
{
    const int64_t wsh = (int64_t)d * (4 * dh + 2 * f);
    const int64_t cells = wsh / 2048 * n_shards;
    if (cells == 0) return hipSuccess;
    if (d % 64 || dh % 64 || f % 64 || cells > 0x7FFFFFF0) return hipErrorInvalidValue;
    launch((decode_tiled_kernel<TableInline>), dim3((uint32_t)((cells + 3) / 4)), dim3(256), 0, stream, 
        TableInline{table}, (int)cells, d, dh, f, (uint8_t *)out);
    return hipGetLastError();
}

hipError_t launch_decode_tiled_table(const ShardDesc *device_table, int n_shards, int d, int dh, int f,
                                     void *out, hipStream_t stream)
{
    const int64_t wsh = (int64_t)d * (4 * dh + 2 * f);
    const int64_t cells = wsh / 2048 * n_shards;
    if (cells == 0) return hipSuccess;
    if (d % 64 || dh % 64 || f % 64 || cells > 0x7FFFFFF0) return hipErrorInvalidValue;
    launch((decode_tiled_kernel<TablePtr>), dim3((uint32_t)((cells + 3) / 4)), dim3(256), 0, stream, 
        TablePtr{device_table}, (int)cells, d, dh, f, (uint8_t *)out);
    return hipGetLastError();
}

}  // namespace sti
