// Projections of the layer on the matrix cores with decompression fused into
// the weight loader (Section "quantization per shard": indexes are substituted
// by centroids before use; here that happens in registers, just before the
// MFMA that consumes the weights, so decoded weights never touch memory).
//
//   C[T x N] = A[T x K] * W^T,  A binary16, W block-structured k-bit / float32,
//   float32 accumulation in v_mfma_f32_32x32x16_f16.
//
// Workgroup = 4 waves, tile BM x 128; every wave owns all BM rows of a 32-column
// strip, so each weight is decoded exactly once per workgroup:
//   - A tile [BM x 64] goes global -> LDS (double buffered, padded rows);
//   - a lane owns weight row n and 32 consecutive K positions per 64-wide K
//     tile (lanes 0-31 the first 32, lanes 32-63 the last 32); 32 k-bit indexes
//     are exactly k dwords, so the raw stream is loaded with aligned dword
//     loads and every field position is a compile-time constant;
//   - codebooks of all blocks sit in LDS as binary16;
//   - the K order inside a tile is permuted identically for A and W, which a
//     dot product does not see.
#include "sti_internal.hpp"

namespace sti {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int BN = 128;          // columns per workgroup (4 waves x 32)
constexpr int BK = 64;           // K positions per LDS stage
constexpr int LDA = BK + 8;      // padded LDS row (halves): 144 bytes, conflict-free b128 reads
constexpr int kLutEntries = 64;  // per block

union Frag4 {        // the four B fragments (k16 steps) of one 64-wide K tile
    uint32_t u[16];
    half8 h[4];
};

__device__ inline uint16_t f16_bits(float v) { return __builtin_bit_cast(uint16_t, (_Float16)v); }
__device__ inline float gelu_erf(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752440f)); }

// ---- raw loads: 32 weights of one lane ------------------------------------
template <int BITS>
__device__ inline void load_raw(const void *p, uint32_t (&raw)[16])
{
    const uint32_t *q = (const uint32_t *)p;
    if constexpr (BITS == 2) {
        u32x2 v = *(const u32x2 *)q;
        raw[0] = v.x; raw[1] = v.y;
    } else if constexpr (BITS == 4) {
        u32x4 v = *(const u32x4 *)q;
        raw[0] = v.x; raw[1] = v.y; raw[2] = v.z; raw[3] = v.w;
    } else if constexpr (BITS == 6) {
        u32x2 a = *(const u32x2 *)q, b = *(const u32x2 *)(q + 2), c = *(const u32x2 *)(q + 4);
        raw[0] = a.x; raw[1] = a.y; raw[2] = b.x; raw[3] = b.y; raw[4] = c.x; raw[5] = c.y;
    } else if constexpr (BITS == 3 || BITS == 5) {
#pragma unroll
        for (int i = 0; i < BITS; ++i) raw[i] = q[i];
    } else if constexpr (BITS == 16) {   // binary16 working buffer
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            u32x4 v = *(const u32x4 *)(q + 4 * i);
            raw[4 * i] = v.x; raw[4 * i + 1] = v.y; raw[4 * i + 2] = v.z; raw[4 * i + 3] = v.w;
        }
    } else {                             // 32: float32 weights, rounded to binary16 here
        const f32x4 *f = (const f32x4 *)p;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            f32x4 v = f[i];
            raw[2 * i] = (uint32_t)f16_bits(v.x) | ((uint32_t)f16_bits(v.y) << 16);
            raw[2 * i + 1] = (uint32_t)f16_bits(v.z) | ((uint32_t)f16_bits(v.w) << 16);
        }
    }
}

// ---- decode: raw -> 32 binary16 weights in fragment order -------------------
template <int BITS>
__device__ inline void decode_raw(const uint32_t (&raw)[16], const uint16_t *lut, Frag4 &f)
{
    if constexpr (BITS == 16 || BITS == 32) {
#pragma unroll
        for (int i = 0; i < 16; ++i) f.u[i] = raw[i];
    } else {
        constexpr uint32_t mask = (1u << BITS) - 1u;
#pragma unroll
        for (int j = 0; j < 32; j += 2) {
            uint32_t idx[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int bit = (j + t) * BITS;
                const int dw = bit >> 5, sh = bit & 31;
                uint32_t v = raw[dw] >> sh;
                if (sh + BITS > 32) v |= raw[dw + 1] << (32 - sh);
                idx[t] = v & mask;
            }
            f.u[j / 2] = (uint32_t)lut[idx[0]] | ((uint32_t)lut[idx[1]] << 16);
        }
    }
}

// bytes of 32 consecutive weights
__host__ __device__ constexpr int bytes32(int bits) { return bits * 4; }

template <int MFRAGS>
struct Smem {
    _Float16 a[2][MFRAGS * 32][LDA];
    uint16_t lut[kMaxShardsPerLayer][kLutEntries];
};

template <int MFRAGS>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmProblem p, GemmBlocks blocks)
{
    constexpr int BM = MFRAGS * 32;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    Smem<MFRAGS> &sm = *reinterpret_cast<Smem<MFRAGS> *>(smem_raw);

    const bool n_split = (p.kind == GEMM_QKV || p.kind == GEMM_FFN_UP);
    const int N = n_split ? p.n_blocks * p.block_rows : p.block_rows;
    const int K = n_split ? p.block_cols : p.n_blocks * p.block_cols;
    const int nkt = K / BK;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int g = lane >> 5, lr = lane & 31;
    const int m0 = blockIdx.y * BM;
    const int nw = blockIdx.x * BN + wave * 32;   // first column of this wave
    const bool wave_active = nw < N;              // N is a multiple of 32
    const int n = nw + lr;                        // this lane's weight row / output column

    // codebooks -> LDS (binary16)
    for (int i = tid; i < p.n_blocks * kLutEntries; i += 256) {
        const int b = i / kLutEntries, e = i % kLutEntries;
        const int bits = blocks.b[b].bits;
        if (bits <= 6 && e < (1 << bits)) sm.lut[b][e] = f16_bits(blocks.b[b].codebook[e]);
    }

    // N-split: the wave stays inside one block for the whole K loop
    int nblk = 0, nrow = n;
    if (n_split && wave_active) {
        nblk = nw / p.block_rows;
        nrow = n - nblk * p.block_rows;
    }
    const int tiles_per_kblock = n_split ? nkt : p.block_cols / BK;

    float16v acc[MFRAGS];
#pragma unroll
    for (int i = 0; i < MFRAGS; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

    const _Float16 *A = (const _Float16 *)p.A;
    const int a_row = tid >> 3, a_col = (tid & 7) * 8;   // 16-byte piece of the A tile
    u32x4 a_regs[MFRAGS];
    auto load_a = [&](int kt) {
#pragma unroll
        for (int i = 0; i < MFRAGS; ++i) {
            const int m = m0 + i * 32 + a_row;
            u32x4 v = {0, 0, 0, 0};
            if (m < p.T) v = *(const u32x4 *)(A + (int64_t)m * p.lda + kt * BK + a_col);
            a_regs[i] = v;
        }
    };
    auto store_a = [&](int buf) {
#pragma unroll
        for (int i = 0; i < MFRAGS; ++i)
            *(u32x4 *)&sm.a[buf][i * 32 + a_row][a_col] = a_regs[i];
    };

    // weight stream position of this lane for K tile kt
    auto weight_src = [&](int kt, int &bits, const uint16_t *&lut) -> const void * {
        int blk, col;   // block and first K column inside the block row
        int64_t row_elems;
        if (n_split) {
            blk = nblk; col = kt * BK + g * 32;
            row_elems = (int64_t)nrow * p.block_cols;
        } else {
            blk = kt / tiles_per_kblock;
            col = (kt - blk * tiles_per_kblock) * BK + g * 32;
            row_elems = (int64_t)n * p.block_cols;
        }
        bits = blocks.b[blk].bits;
        lut = sm.lut[blk];
        const int64_t elem = row_elems + col;   // multiple of 32
        return (const uint8_t *)blocks.b[blk].w + (elem >> 5) * bytes32(bits);
    };

    uint32_t raw[16];
    int raw_bits = 0;
    const uint16_t *raw_lut = nullptr;
    auto fetch_b = [&](int kt) {
        const void *src = weight_src(kt, raw_bits, raw_lut);
        switch (raw_bits) {
            case 2: load_raw<2>(src, raw); break;
            case 3: load_raw<3>(src, raw); break;
            case 4: load_raw<4>(src, raw); break;
            case 5: load_raw<5>(src, raw); break;
            case 6: load_raw<6>(src, raw); break;
            case 16: load_raw<16>(src, raw); break;
            default: load_raw<32>(src, raw); break;
        }
    };

    if (nkt > 0) {
        load_a(0);
        if (wave_active) fetch_b(0);
    }
    __syncthreads();   // LUTs visible

    for (int kt = 0; kt < nkt; ++kt) {
        const int buf = kt & 1;
        store_a(buf);
        __syncthreads();
        if (kt + 1 < nkt) load_a(kt + 1);
        if (wave_active) {
            Frag4 bf;
            switch (raw_bits) {
                case 2: decode_raw<2>(raw, raw_lut, bf); break;
                case 3: decode_raw<3>(raw, raw_lut, bf); break;
                case 4: decode_raw<4>(raw, raw_lut, bf); break;
                case 5: decode_raw<5>(raw, raw_lut, bf); break;
                case 6: decode_raw<6>(raw, raw_lut, bf); break;
                default: decode_raw<16>(raw, raw_lut, bf); break;
            }
            if (kt + 1 < nkt) fetch_b(kt + 1);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
#pragma unroll
                for (int i = 0; i < MFRAGS; ++i) {
                    half8 a = *(const half8 *)&sm.a[buf][i * 32 + lr][g * 32 + s * 8];
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, bf.h[s], acc[i], 0, 0, 0);
                }
            }
        }
    }
    if (!wave_active) return;

    // ---- epilogue: lane owns column n, rows i*32 + (v/4)*8 + g*4 + v%4 ----
    if (p.kind == GEMM_QKV || p.kind == GEMM_FFN_UP) {
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
        for (int i = 0; i < MFRAGS; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + i * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
                if (m >= p.T) continue;
                float x = acc[i][v] + bias;
                if (p.kind == GEMM_FFN_UP) x = gelu_erf(x);
                C[(int64_t)m * p.ldc + n] = (_Float16)x;
            }
    } else {
        const float bias = p.bias0[n];
        float *C = (float *)p.C;
        const _Float16 *R = (const _Float16 *)p.resid;
#pragma unroll
        for (int i = 0; i < MFRAGS; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + i * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
                if (m >= p.T) continue;
                C[(int64_t)m * p.ldc + n] = acc[i][v] + bias + (float)R[(int64_t)m * p.ldr + n];
            }
    }
}

}  // namespace

hipError_t launch_gemm_mfma(const GemmProblem &p, const GemmBlocks &blocks, hipStream_t stream)
{
    const bool n_split = (p.kind == GEMM_QKV || p.kind == GEMM_FFN_UP);
    const int N = n_split ? p.n_blocks * p.block_rows : p.block_rows;
    if (p.T <= 0 || N <= 0) return hipSuccess;
    if (N % 32 || p.block_cols % BK || p.lda % 8) return hipErrorInvalidValue;
    constexpr int MFRAGS = 4;
    dim3 grid((N + BN - 1) / BN, (p.T + MFRAGS * 32 - 1) / (MFRAGS * 32));
    const size_t lds = sizeof(Smem<MFRAGS>);
    gemm_mfma_kernel<MFRAGS><<<grid, dim3(256), lds, stream>>>(p, blocks);
    return hipGetLastError();
}

}  // namespace sti
