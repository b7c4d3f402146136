// Projections of the layer on the matrix cores with decompression fused into
// the weight loader (Section "quantization per shard": indexes are substituted
// by centroids before use; here that happens in registers, just before the
// MFMA that consumes the weights, so decoded weights never touch memory).
//
//   C[T x N] = A[T x K] * W^T,  A binary16, W block-structured k-bit / float32,
//   float32 accumulation in v_mfma_f32_32x32x16_f16.
//
// Workgroup = 4 waves arranged WM x WN; a wave owns a (RA*32) x (RB*32) tile:
//   - the A tile [BM x 64] goes global -> LDS (double buffered, padded rows) and
//     every A fragment read from LDS feeds RB MFMAs;
//   - a lane owns weight row n and 32 consecutive K positions per 64-wide K
//     tile (lanes 0-31 the first 32, lanes 32-63 the last 32); 32 k-bit indexes
//     are exactly k dwords, so the raw stream is loaded with aligned dword
//     loads, every field position is a compile-time constant, and every
//     decoded fragment feeds RA MFMAs;
//   - the raw dwords of K tile t+1 are in flight while tile t is decoded and
//     multiplied; codebooks of all blocks sit in LDS as binary16;
//   - the K order inside a tile is permuted identically for A and W, which a
//     dot product does not see.
#include <stdlib.h>
#include "sti_internal.hpp"

namespace sti {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 64;           // K positions per LDS stage
constexpr int LDA = BK + 8;      // padded LDS row (halves): 144 bytes, conflict-free b128 reads
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

template <int BM>
struct Smem {
    _Float16 a[2][BM][LDA];
    uint16_t lut[kMaxShardsPerLayer][kLutEntries];
};

template <int RA, int RB, int WM, int WN>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmProblem p, GemmBlocks blocks)
{
    static_assert(WM * WN == 4, "four waves per workgroup");
    constexpr int BM = WM * RA * 32, BN = WN * RB * 32;
    constexpr int A_PASSES = BM / 32;   // 16-byte pieces per thread per K tile
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    Smem<BM> &sm = *reinterpret_cast<Smem<BM> *>(smem_raw);

    const bool n_split = (p.kind == GEMM_QKV || p.kind == GEMM_FFN_UP);
    const int N = n_split ? p.n_blocks * p.block_rows : p.block_rows;
    const int K = n_split ? p.block_cols : p.n_blocks * p.block_cols;
    const int nkt = K / BK;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps block/bitwidth selection scalar
    const int g = lane >> 5, lr = lane & 31;
    const int wm = wave / WN, wn = wave % WN;
    // Workgroups are handed to the 8 XCDs round-robin by linear id.  Give each XCD one
    // contiguous range of the row-major tile order (a band of rows and all column
    // tiles), so that its private L2 keeps its band of A and streams W once.
    const int n_tiles = (N + BN - 1) / BN;
    const int m_tiles = (p.T + BM - 1) / BM;
    const int total_tiles = n_tiles * m_tiles;
    const int per_xcd = (total_tiles + 7) / 8;
    const int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || tile >= total_tiles) return;
    const int tile_m = tile / n_tiles, tile_n = tile - tile_m * n_tiles;
    const int m0 = tile_m * BM;
    const int mw = wm * RA * 32;                           // first row of this wave inside the tile
    // N and the block widths are multiples of RB*32, so a wave's columns are all inside
    // or all outside the matrix; a wave outside recomputes the first columns (no branch
    // in the K loop) and stores nothing
    const int nw_real = tile_n * BN + wn * RB * 32;
    const bool wave_active = nw_real < N;
    const int nw = wave_active ? nw_real : 0;              // first column of this wave

    // codebooks -> LDS (binary16)
    for (int i = tid; i < p.n_blocks * kLutEntries; i += 256) {
        const int b = i / kLutEntries, e = i % kLutEntries;
        const int bits = blocks.b[b].bits;
        if (bits <= 6 && e < (1 << bits)) sm.lut[b][e] = (uint16_t)f16_bits(blocks.b[b].codebook[e]);
    }

    // N-split: a wave stays inside one block for the whole K loop
    int nblk = 0, nrow0 = nw;
    if (n_split) {
        nblk = nw / p.block_rows;
        nrow0 = nw - nblk * p.block_rows;
    }
    const int tiles_per_kblock = n_split ? nkt : p.block_cols / BK;

    float16v acc[RA][RB];
#pragma unroll
    for (int i = 0; i < RA; ++i)
#pragma unroll
        for (int r = 0; r < RB; ++r)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][r][v] = 0.f;

    const _Float16 *A = (const _Float16 *)p.A;
    const int a_row = tid >> 3, a_col = (tid & 7) * 8;   // 16-byte piece of the A tile
    u32x4 a_regs[A_PASSES];
    auto load_a = [&](int kt) {
#pragma unroll
        for (int i = 0; i < A_PASSES; ++i) {
            const int m = m0 + i * 32 + a_row;
            u32x4 v = {0, 0, 0, 0};
            if (m < p.T) v = *(const u32x4 *)(A + (int64_t)m * p.lda + kt * BK + a_col);
            a_regs[i] = v;
        }
    };
    auto store_a = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_PASSES; ++i)
            *(u32x4 *)&sm.a[buf][i * 32 + a_row][a_col] = a_regs[i];
    };

    // stream position of this lane's 32 weights of strip r in K tile kt
    auto weight_src = [&](int kt, int r, int &bits, int &blk) -> const void * {
        int col;
        int64_t row_elems;
        if (n_split) {
            blk = nblk;
            col = kt * BK + g * 32;
            row_elems = (int64_t)(nrow0 + r * 32 + lr) * p.block_cols;
        } else {
            blk = kt / tiles_per_kblock;
            col = (kt - blk * tiles_per_kblock) * BK + g * 32;
            row_elems = (int64_t)(nw + r * 32 + lr) * p.block_cols;
        }
        bits = blocks.b[blk].bits;
        const int64_t elem = row_elems + col;   // multiple of 32
        return (const uint8_t *)blocks.b[blk].w + (elem >> 5) * (bits * 4);
    };

    Raw raw[RB];
    int cur_bits = 0, cur_blk = 0;
    if (nkt > 0) load_a(0);
    if (nkt > 0) {
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const void *src = weight_src(0, r, cur_bits, cur_blk);
            raw[r] = load_raw_any(cur_bits, src);
        }
    }
    __syncthreads();   // LUTs visible

    for (int kt = 0; kt < nkt; ++kt) {
        const int buf = kt & 1;
        store_a(buf);
        __syncthreads();
        if (kt + 1 < nkt) load_a(kt + 1);
        half8 bf[RB][4];
        const uint16_t *lut = sm.lut[cur_blk];
#pragma unroll
        for (int r = 0; r < RB; ++r) decode_raw_any(cur_bits, raw[r], lut, bf[r]);
        if (kt + 1 < nkt) {
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                const void *src = weight_src(kt + 1, r, cur_bits, cur_blk);
                raw[r] = load_raw_any(cur_bits, src);
            }
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) {
#pragma unroll
            for (int i = 0; i < RA; ++i) {
                half8 a = *(const half8 *)&sm.a[buf][mw + i * 32 + lr][g * 32 + s * 8];
#pragma unroll
                for (int r = 0; r < RB; ++r)
                    acc[i][r] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, bf[r][s], acc[i][r], 0, 0, 0);
            }
        }
    }
    if (!wave_active) return;

    // ---- epilogue: lane owns column n, rows mw + i*32 + (v/4)*8 + g*4 + v%4 ----
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        const int n = nw + r * 32 + lr;
        if (p.kind == GEMM_QKV || p.kind == GEMM_FFN_UP) {
            const int nrow = nrow0 + r * 32 + lr;
            float bias;
            if (p.kind == GEMM_QKV) {
                const int which = nrow / p.d_head, e = nrow - which * p.d_head;
                const float *bp = which == 0 ? p.bias0 : (which == 1 ? p.bias1 : p.bias2);
                bias = bp[blocks.b[nblk].shard * p.d_head + e];
            } else {
                bias = p.bias0[blocks.b[nblk].shard * p.block_rows + nrow];
            }
            _Float16 *C = (_Float16 *)p.C;
#pragma unroll
            for (int i = 0; i < RA; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + mw + i * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
                    if (m >= p.T) continue;
                    float x = acc[i][r][v] + bias;
                    if (p.kind == GEMM_FFN_UP) x = gelu_erf(x);
                    C[(int64_t)m * p.ldc + n] = (_Float16)x;
                }
        } else {
            const float bias = p.bias0[n];
            float *C = (float *)p.C;
            const _Float16 *R = (const _Float16 *)p.resid;
#pragma unroll
            for (int i = 0; i < RA; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + mw + i * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
                    if (m >= p.T) continue;
                    C[(int64_t)m * p.ldc + n] = acc[i][r][v] + bias + (float)R[(int64_t)m * p.ldr + n];
                }
        }
    }
}

template <int RA, int RB, int WM, int WN>
hipError_t launch_cfg(const GemmProblem &p, const GemmBlocks &blocks, int N, hipStream_t stream)
{
    constexpr int BM = WM * RA * 32, BN = WN * RB * 32;
    const int total = ((N + BN - 1) / BN) * ((p.T + BM - 1) / BM);
    dim3 grid(((total + 7) / 8) * 8);
    gemm_mfma_kernel<RA, RB, WM, WN><<<grid, dim3(256), sizeof(Smem<BM>), stream>>>(p, blocks);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_mfma(const GemmProblem &p, const GemmBlocks &blocks, hipStream_t stream)
{
    const bool n_split = (p.kind == GEMM_QKV || p.kind == GEMM_FFN_UP);
    const int N = n_split ? p.n_blocks * p.block_rows : p.block_rows;
    if (p.T <= 0 || N <= 0) return hipSuccess;
    if (N % 64 || p.block_rows % 64 || p.block_cols % BK || p.lda % 8 || p.n_blocks <= 0 && n_split)
        return hipErrorInvalidValue;
    static int cfg = -1;
    if (cfg < 0) { const char *e = getenv("STI_EXP_CFG"); cfg = e ? atoi(e) : 0; }
    switch (cfg) {
        case 1: return launch_cfg<4, 2, 1, 4>(p, blocks, N, stream);
        case 2: return launch_cfg<2, 2, 2, 2>(p, blocks, N, stream);
        case 3: return launch_cfg<4, 2, 2, 2>(p, blocks, N, stream);
        case 4: return launch_cfg<2, 1, 1, 4>(p, blocks, N, stream);
        default: return launch_cfg<4, 1, 1, 4>(p, blocks, N, stream);
    }
}

}  // namespace sti
