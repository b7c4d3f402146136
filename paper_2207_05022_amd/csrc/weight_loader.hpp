// Per-lane weight loader shared by the fused GEMM and the working-buffer decoder:
// 32 consecutive weights of one row arrive as k dwords of a k-bit stream (or as
// float32 / binary16 values) and leave as four binary16 MFMA B fragments.
//
// Fragment-tiled working buffer: a [R x C] weight block (R % 32 == 0, C % 64 == 0)
// is stored as 4 KiB cells, one per (32-row strip, 64-column K tile); inside a cell
// fragment q (0..3) is 1 KiB and lane l owns 16 bytes of it, namely row l%32,
// columns (l/32)*32 + q*8 .. +8 of the cell.  A wave therefore loads or stores a
// whole fragment as one contiguous 1 KiB access.
#pragma once
#include "sti_internal.hpp"

namespace sti {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kLutEntries = 64;  // per block

__device__ inline uint32_t f16_bits(float v) { return __builtin_bit_cast(uint16_t, (_Float16)v); }
__device__ inline float gelu_erf(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752440f)); }

// 32 weights of one lane before decode, kept as four named vectors so that the
// loop-carried prefetch state stays in registers.
struct Raw {
    u32x4 a, b, c, d;
};

// ---- raw loads: 32 weights of one lane ------------------------------------
template <int BITS>
__device__ inline Raw load_raw(const void *p)
{
    const uint32_t *q = (const uint32_t *)p;
    Raw r;
    r.a = r.b = r.c = r.d = u32x4{0, 0, 0, 0};
    if constexpr (BITS == 2) {
        u32x2 v = *(const u32x2 *)q;
        r.a.x = v.x; r.a.y = v.y;
    } else if constexpr (BITS == 4) {
        r.a = *(const u32x4 *)q;
    } else if constexpr (BITS == 6) {
        u32x2 a = *(const u32x2 *)q, b = *(const u32x2 *)(q + 2), c = *(const u32x2 *)(q + 4);
        r.a = u32x4{a.x, a.y, b.x, b.y};
        r.b.x = c.x; r.b.y = c.y;
    } else if constexpr (BITS == 3) {
        r.a.x = q[0]; r.a.y = q[1]; r.a.z = q[2];
    } else if constexpr (BITS == 5) {
        r.a = u32x4{q[0], q[1], q[2], q[3]};
        r.b.x = q[4];
    } else if constexpr (BITS == 16) {   // binary16 working buffer
        r.a = *(const u32x4 *)q; r.b = *(const u32x4 *)(q + 4);
        r.c = *(const u32x4 *)(q + 8); r.d = *(const u32x4 *)(q + 12);
    } else {                             // 32: float32 weights, rounded to binary16 on arrival
        const f32x4 *f = (const f32x4 *)p;
        uint32_t h[16];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            f32x4 v = f[i];
            h[2 * i] = f16_bits(v.x) | (f16_bits(v.y) << 16);
            h[2 * i + 1] = f16_bits(v.z) | (f16_bits(v.w) << 16);
        }
        r.a = u32x4{h[0], h[1], h[2], h[3]}; r.b = u32x4{h[4], h[5], h[6], h[7]};
        r.c = u32x4{h[8], h[9], h[10], h[11]}; r.d = u32x4{h[12], h[13], h[14], h[15]};
    }
    return r;
}

__device__ inline Raw load_raw_any(int bits, const void *p)
{
    switch (bits) {
        case 2: return load_raw<2>(p);
        case 3: return load_raw<3>(p);
        case 4: return load_raw<4>(p);
        case 5: return load_raw<5>(p);
        case 6: return load_raw<6>(p);
        case 16: return load_raw<16>(p);
        default: return load_raw<32>(p);
    }
}

// ---- decode: raw -> four B fragments (32 binary16 weights) ------------------
template <int BITS>
__device__ inline void decode_raw(const Raw &r, const uint16_t *lut, half8 (&f)[4])
{
    if constexpr (BITS > 6) {
        f[0] = __builtin_bit_cast(half8, r.a); f[1] = __builtin_bit_cast(half8, r.b);
        f[2] = __builtin_bit_cast(half8, r.c); f[3] = __builtin_bit_cast(half8, r.d);
        return;
    }
    uint32_t w[16];
    const uint32_t rv[8] = {r.a.x, r.a.y, r.a.z, r.a.w, r.b.x, r.b.y, r.b.z, r.b.w};
    {
        constexpr uint32_t mask = (1u << BITS) - 1u;
#pragma unroll
        for (int j = 0; j < 32; j += 2) {
            uint32_t idx[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int bit = (j + t) * BITS;
                const int dw = bit >> 5, sh = bit & 31;
                uint32_t v = rv[dw] >> sh;
                if (sh + BITS > 32) v |= rv[dw + 1] << (32 - sh);
                idx[t] = v & mask;
            }
            w[j / 2] = (uint32_t)lut[idx[0]] | ((uint32_t)lut[idx[1]] << 16);
        }
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        u32x4 v = {w[4 * s], w[4 * s + 1], w[4 * s + 2], w[4 * s + 3]};
        f[s] = __builtin_bit_cast(half8, v);
    }
}

__device__ inline void decode_raw_any(int bits, const Raw &r, const uint16_t *lut, half8 (&f)[4])
{
    switch (bits) {
        case 2: decode_raw<2>(r, lut, f); break;
        case 3: decode_raw<3>(r, lut, f); break;
        case 4: decode_raw<4>(r, lut, f); break;
        case 5: decode_raw<5>(r, lut, f); break;
        case 6: decode_raw<6>(r, lut, f); break;
        default: decode_raw<16>(r, lut, f); break;
    }
}


constexpr int kTiledBits = 17;   // GemmBlock::bits value marking a fragment-tiled binary16 block

// byte offset of the cell (strip, kt) of a tiled block with C columns
__device__ inline int64_t tiled_cell_offset(int strip, int kt, int cols)
{
    return ((int64_t)strip * (cols >> 6) + kt) * 4096;
}

// Cells of the fragment-tiled binary16 working buffer (Section "Submodel execution": the working buffer a
// layer is decompressed into).  A cell is 32 rows x 64 columns = 4 KiB; cells are numbered shard by shard,
// and inside a shard over its four sub-blocks [3dh x d], [d x dh], [f x d], [d x f], strip by strip.
struct TiledCell {
    int shard;         // index into the run of shards
    int cols;          // columns of the sub-block
    int64_t sub_off;   // element offset of the sub-block inside the shard
    int strip, kt;     // 32-row strip and 64-column tile inside the sub-block
};

__device__ inline TiledCell locate_tiled_cell(int cell, int d, int dh, int f)
{
    const int c_qkv = (3 * dh / 32) * (d / 64), c_o = (d / 32) * (dh / 64);
    const int c_1 = (f / 32) * (d / 64), c_2 = (d / 32) * (f / 64);
    const int per_shard = c_qkv + c_o + c_1 + c_2;
    TiledCell t;
    t.shard = cell / per_shard;
    int c = cell - t.shard * per_shard;
    if (c < c_qkv) { t.cols = d; t.sub_off = 0; }
    else if (c < c_qkv + c_o) { c -= c_qkv; t.cols = dh; t.sub_off = (int64_t)3 * dh * d; }
    else if (c < c_qkv + c_o + c_1) { c -= c_qkv + c_o; t.cols = d; t.sub_off = (int64_t)4 * dh * d; }
    else { c -= c_qkv + c_o + c_1; t.cols = f; t.sub_off = (int64_t)4 * dh * d + (int64_t)f * d; }
    const int tiles = t.cols >> 6;
    t.strip = c / tiles;
    t.kt = c - t.strip * tiles;
    return t;
}

// this lane's 32 weights of the cell (row lane % 32, columns (lane / 32) * 32 .. + 32 of the tile), as stored
__device__ inline Raw load_tiled_cell_raw(const TiledCell &t, int bits, const void *data, int lane)
{
    const int64_t elem = t.sub_off + (int64_t)(t.strip * 32 + (lane & 31)) * t.cols + t.kt * 64 + (lane >> 5) * 32;
    return load_raw_any(bits, (const uint8_t *)data + (elem >> 5) * (bits * 4));
}

__device__ inline void store_tiled_cell(const TiledCell &t, int d, int dh, int f, const half8 (&fr)[4],
                                        uint8_t *out, int lane)
{
    const int64_t wsh = (int64_t)d * (4 * dh + 2 * f);
    uint8_t *cell_out = out + ((int64_t)t.shard * wsh + t.sub_off) * 2 + tiled_cell_offset(t.strip, t.kt, t.cols);
#pragma unroll
    for (int q = 0; q < 4; ++q)
        *((u32x4 *)(cell_out + q * 1024) + lane) = __builtin_bit_cast(u32x4, fr[q]);
}

// One wave decodes cell number `cell` into the working buffer at `out`.  lut: 64 entries of LDS that
// belong to this wave alone.
template <typename Table>
__device__ inline void decode_tiled_cell(const Table &tab, int cell, int d, int dh, int f, uint8_t *out,
                                         uint16_t *lut, int lane)
{
    const TiledCell t = locate_tiled_cell(cell, d, dh, f);
    const ShardDesc sd = tab.get(t.shard);
    const int bits = sd.bits;
    if (bits <= 6) {
        // (LDS serves a wave's accesses in order; the fences keep the compiler from moving this table's
        //  writes above the reads of the previous cell's table, and its reads above the writes)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (lane < (1 << bits)) lut[lane] = (uint16_t)f16_bits(sd.codebook[lane]);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    const Raw raw = load_tiled_cell_raw(t, bits, sd.data, lane);
    half8 fr[4];
    decode_raw_any(bits, raw, lut, fr);
    store_tiled_cell(t, d, dh, f, fr, out, lane);
}

// shard table in device memory
struct TablePtr {
    const ShardDesc *p;
    __device__ inline ShardDesc get(uint32_t s) const { return p[s]; }
};

// four fragments of one cell for this lane
__device__ inline Raw load_tiled(const void *cell, int lane)
{
    const u32x4 *q = (const u32x4 *)cell + lane;
    Raw r;
    r.a = q[0]; r.b = q[64]; r.c = q[128]; r.d = q[192];
    return r;
}

}  // namespace sti
