// Projections of the layer on the matrix cores (Section "A primer on transformer":
// the Q/K/V, output and two FFN linear layers), over the present shards only.
//
//   C[T x N] = A[T x K] * W^T,  A binary16, float32 accumulation in
//   v_mfma_f32_32x32x16_f16, W cut into per-shard blocks that are either
//     - k-bit index streams / float32 values, decompressed in registers just before
//       the MFMA that consumes them (Section "quantization per shard": indexes are
//       substituted by centroids before use), or
//     - cells of the fragment-tiled binary16 working buffer (weight_loader.hpp).
//
// Workgroup = 4 waves arranged WM x WN; a wave owns a (RA*32) x (RB*32) tile:
//   - the A tile [BM x 64] goes global -> registers -> LDS (double buffered, padded
//     rows); every A fragment read from LDS feeds RB MFMAs;
//   - a lane owns weight row n and 32 consecutive K positions per 64-wide K tile
//     (lanes 0-31 the first 32, lanes 32-63 the last 32); 32 k-bit indexes are exactly
//     k dwords, so the raw stream is loaded with aligned dword loads, every field
//     position is a compile-time constant, and every decoded fragment feeds RA MFMAs;
//   - global loads of K tile t+1 are in flight while tile t is multiplied;
//   - the K order inside a tile is permuted identically for A and W, which a dot
//     product does not see;
//   - binary16 results leave through LDS so that every global store is 16 bytes of
//     one output row.
#include "sti_internal.hpp"
#include "weight_loader.hpp"

namespace sti {
namespace {

constexpr int BK = 64;           // K positions per LDS stage
constexpr int LDA = BK + 8;      // padded LDS row (halves): 144 bytes, conflict-free b128 reads

// erf by the rational approximation 7.1.26 of Abramowitz & Stegun (|error| < 1.5e-7),
// enough for results that are rounded to binary16.
__device__ inline float gelu_fast(float z)
{
    const float x = fabsf(z) * 0.70710678118654752440f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
    float poly = fmaf(1.061405429f, t, -1.453152027f);
    poly = fmaf(poly, t, 1.421413741f);
    poly = fmaf(poly, t, -0.284496736f);
    poly = fmaf(poly, t, 0.254829592f);
    const float e = __builtin_amdgcn_exp2f(-x * x * 1.44269504088896340736f);
    const float erf_abs = 1.0f - poly * t * e;
    const float erf_z = z < 0.f ? -erf_abs : erf_abs;
    return 0.5f * z * (1.0f + erf_z);
}

template <int BM>
struct Smem {
    _Float16 a[2][BM][LDA];
    uint16_t lut[kMaxShardsPerLayer][kLutEntries];
};

template <int KIND, int RA, int RB, int WM, int WN, bool TILED>
__global__ __launch_bounds__(256, (RA * RB >= 4 ? 2 : 3)) void gemm_mfma_kernel(GemmProblem p, GemmBlocks blocks)
{
    static_assert(WM * WN == 4, "four waves per workgroup");
    constexpr int BM = WM * RA * 32, BN = WN * RB * 32;
    constexpr int A_PASSES = BM / 32;   // 16-byte pieces per thread per K tile
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    Smem<BM> &sm = *reinterpret_cast<Smem<BM> *>(smem_raw);

    constexpr bool n_split = (KIND == GEMM_QKV || KIND == GEMM_FFN_UP);
    const int N = n_split ? p.n_blocks * p.block_rows : p.block_rows;
    const int K = n_split ? p.block_cols : p.n_blocks * p.block_cols;
    const int nkt = K / BK;
    const int tid = threadIdx.x, lane = tid & 63;
    // wave-uniform, so that block and bitwidth selection stay scalar
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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
    if constexpr (!TILED) {
        for (int i = tid; i < p.n_blocks * kLutEntries; i += 256) {
            const int b = i / kLutEntries, e = i % kLutEntries;
            const int bits = blocks.b[b].bits;
            if (bits <= 6 && e < (1 << bits)) sm.lut[b][e] = (uint16_t)f16_bits(blocks.b[b].codebook[e]);
        }
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
    struct AStage {
        u32x4 v[A_PASSES];
    };
    auto load_a = [&](int kt) -> AStage {
        AStage st;
#pragma unroll
        for (int i = 0; i < A_PASSES; ++i) {
            const int m = m0 + i * 32 + a_row;
            u32x4 v = {0, 0, 0, 0};
            if (m < p.T) v = *(const u32x4 *)(A + (int64_t)m * p.lda + kt * BK + a_col);
            st.v[i] = v;
        }
        return st;
    };
    auto store_a = [&](int buf, const AStage &st) {
#pragma unroll
        for (int i = 0; i < A_PASSES; ++i)
            *(u32x4 *)&sm.a[buf][i * 32 + a_row][a_col] = st.v[i];
    };

    struct BStage {
        Raw raw[RB];
        int bits, blk;
    };
    // the 32 weights of this lane for every strip of K tile kt
    auto fetch = [&](int kt) -> BStage {
        BStage st;
        int blk, ktb, row;   // block, K tile inside the block, first row inside the block
        if (n_split) {
            blk = nblk; ktb = kt; row = nrow0;
        } else {
            blk = kt / tiles_per_kblock; ktb = kt - blk * tiles_per_kblock; row = nw;
        }
        const int bits = blocks.b[blk].bits;
        st.bits = bits; st.blk = blk;
        const uint8_t *base = (const uint8_t *)blocks.b[blk].w;
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            if (TILED || bits == kTiledBits) {
                st.raw[r] = load_tiled(base + tiled_cell_offset((row >> 5) + r, ktb, p.block_cols), lane);
            } else {
                const int64_t elem = (int64_t)(row + r * 32 + lr) * p.block_cols + ktb * BK + g * 32;
                st.raw[r] = load_raw_any(bits, base + (elem >> 5) * (bits * 4));
            }
        }
        return st;
    };

    auto compute = [&](int buf, const BStage &st) {
        half8 bf[RB][4];
        const uint16_t *lut = sm.lut[st.blk];
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            if constexpr (TILED) decode_raw<16>(st.raw[r], lut, bf[r]);
            else decode_raw_any(st.bits, st.raw[r], lut, bf[r]);
        }
        // the A fragments of k-step s+1 are read from LDS while the MFMAs of step s run;
        // the scheduling barriers keep the reads ahead of the MFMAs they overlap
        half8 a_cur[RA], a_nxt[RA];
#pragma unroll
        for (int i = 0; i < RA; ++i) a_cur[i] = *(const half8 *)&sm.a[buf][mw + i * 32 + lr][g * 32];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if (s < 3) {
#pragma unroll
                for (int i = 0; i < RA; ++i)
                    a_nxt[i] = *(const half8 *)&sm.a[buf][mw + i * 32 + lr][g * 32 + (s + 1) * 8];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < RA; ++i)
#pragma unroll
                for (int r = 0; r < RB; ++r)
                    acc[i][r] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf[r][s], a_cur[i], acc[i][r], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (s < 3) {
#pragma unroll
                for (int i = 0; i < RA; ++i) a_cur[i] = a_nxt[i];
            }
        }
    };


    AStage a0;
    BStage b0;
    if (nkt > 0) { a0 = load_a(0); b0 = fetch(0); }
    __syncthreads();   // codebooks visible
    for (int kt = 0; kt < nkt; ++kt) {
        store_a(kt & 1, a0);
        __syncthreads();
        if (kt + 1 < nkt) a0 = load_a(kt + 1);
        const BStage cur = b0;
        if (kt + 1 < nkt) b0 = fetch(kt + 1);
        compute(kt & 1, cur);
    }

    // ---- epilogue ----
    // The weight fragment is the first MFMA operand, so the accumulator of a 32 x 32 block holds,
    // in lane l, token row lr and output columns (v/4)*8 + g*4 + v%4.  Exchanging registers
    // between lanes l and l+32 (v_permlane32_swap) turns that into runs of 8 consecutive columns
    // per lane: after the swap of the column groups 2q and 2q+1 the lane owns columns
    // 16q + 8g .. +8 of its row, i.e. one 16-byte piece of the output row.  Bias, GELU and the
    // residual are applied to that piece in registers; the pieces of the whole workgroup tile
    // are then collected in LDS so that every global store instruction writes whole rows of
    // the tile (stores of 32-byte row segments straight from the accumulator layout were
    // measured to be limited by the number of partial cache lines per instruction).
    constexpr int LDT = BN + 8;   // padded row of the staged tile (halves): conflict-free 16-byte writes
    static_assert(BM * LDT <= 2 * BM * LDA, "the staged tile fits in the A buffers");
    _Float16 *tile_out = &sm.a[0][0][0];
    const _Float16 *R = (const _Float16 *)p.resid;
    __syncthreads();   // every wave is done with the A tiles
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        f32x4 bias[2][2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int c = r * 32 + 16 * q + 8 * g;     // first column of the piece inside the wave's strip
            const float *bp;
            if constexpr (KIND == GEMM_QKV) {
                const int nrow = nrow0 + c;
                const int which = nrow / p.d_head, e0 = nrow - which * p.d_head;
                bp = (which == 0 ? p.bias0 : (which == 1 ? p.bias1 : p.bias2)) + blocks.b[nblk].shard * p.d_head + e0;
            } else if constexpr (KIND == GEMM_FFN_UP) {
                bp = p.bias0 + blocks.b[nblk].shard * p.block_rows + nrow0 + c;
            } else {
                bp = p.bias0 + nw + c;
            }
            bias[q][0] = *(const f32x4 *)bp;
            bias[q][1] = *(const f32x4 *)(bp + 4);
        }
#pragma unroll
        for (int i = 0; i < RA; ++i) {
            const int row = mw + i * 32 + lr;          // row inside the tile
            half8 res[2];
            if constexpr (!n_split) {
                const int m = m0 + row;
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    u32x4 v = {0, 0, 0, 0};
                    if (wave_active && m < p.T) v = *(const u32x4 *)(R + (int64_t)m * p.ldr + nw + r * 32 + 16 * q + 8 * g);
                    res[q] = __builtin_bit_cast(half8, v);
                }
            }
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                float x[8];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    // (element values first: a bit cast applied to a vector element itself reads element 0)
                    const float lo = acc[i][r][(2 * q) * 4 + e], hi = acc[i][r][(2 * q + 1) * 4 + e];
                    const auto sw = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(uint32_t, lo),
                                                                     __builtin_bit_cast(uint32_t, hi), false, false);
                    const uint32_t s0 = sw[0], s1 = sw[1];
                    x[e] = __builtin_bit_cast(float, s0);
                    x[4 + e] = __builtin_bit_cast(float, s1);
                }
                half8 o;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float y = x[e] + bias[q][e >> 2][e & 3];
                    if constexpr (KIND == GEMM_FFN_UP) y = gelu_fast(y);
                    if constexpr (!n_split) y += (float)res[q][e];
                    o[e] = (_Float16)y;
                }
                *(half8 *)(tile_out + row * LDT + (wn * RB + r) * 32 + 16 * q + 8 * g) = o;
            }
        }
    }
    __syncthreads();
    // 16 lanes per tile row: one store instruction writes 4 whole rows of the tile
    _Float16 *C = (_Float16 *)p.C;
    constexpr int PIECES_PER_ROW = BN / 8;
    constexpr int PASSES = BM * PIECES_PER_ROW / 256;
    u32x4 piece[PASSES];
#pragma unroll
    for (int j = 0; j < PASSES; ++j) {
        const int pc = tid + 256 * j;
        piece[j] = *(const u32x4 *)(tile_out + (pc / PIECES_PER_ROW) * LDT + (pc % PIECES_PER_ROW) * 8);
    }
#pragma unroll
    for (int j = 0; j < PASSES; ++j) {
        const int pc = tid + 256 * j;
        const int m = m0 + pc / PIECES_PER_ROW, n = tile_n * BN + (pc % PIECES_PER_ROW) * 8;
        if (m < p.T && n < N) *(u32x4 *)(C + (int64_t)m * p.ldc + n) = piece[j];
    }
}

template <int KIND, int RA, int RB, int WM, int WN>
hipError_t launch_kind(const GemmProblem &p, const GemmBlocks &blocks, int N, hipStream_t stream)
{
    constexpr int BM = WM * RA * 32, BN = WN * RB * 32;
    const int total = ((N + BN - 1) / BN) * ((p.T + BM - 1) / BM);
    dim3 grid(((total + 7) / 8) * 8);
    bool tiled = p.n_blocks > 0;
    for (int b = 0; b < p.n_blocks; ++b) tiled = tiled && blocks.b[b].bits == kTiledBits;
    if (tiled)
        gemm_mfma_kernel<KIND, RA, RB, WM, WN, true><<<grid, dim3(256), sizeof(Smem<BM>), stream>>>(p, blocks);
    else
        gemm_mfma_kernel<KIND, RA, RB, WM, WN, false><<<grid, dim3(256), sizeof(Smem<BM>), stream>>>(p, blocks);
    return hipGetLastError();
}

template <int RA, int RB, int WM, int WN>
hipError_t launch_cfg(const GemmProblem &p, const GemmBlocks &blocks, int N, hipStream_t stream)
{
    switch (p.kind) {
    case GEMM_QKV: return launch_kind<GEMM_QKV, RA, RB, WM, WN>(p, blocks, N, stream);
    case GEMM_FFN_UP: return launch_kind<GEMM_FFN_UP, RA, RB, WM, WN>(p, blocks, N, stream);
    case GEMM_OUT: return launch_kind<GEMM_OUT, RA, RB, WM, WN>(p, blocks, N, stream);
    case GEMM_FFN_DOWN: return launch_kind<GEMM_FFN_DOWN, RA, RB, WM, WN>(p, blocks, N, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_gemm_mfma(const GemmProblem &p, const GemmBlocks &blocks, hipStream_t stream)
{
    const bool n_split = (p.kind == GEMM_QKV || p.kind == GEMM_FFN_UP);
    const int N = n_split ? p.n_blocks * p.block_rows : p.block_rows;
    if (p.T <= 0 || N <= 0) return hipSuccess;
    if (N % 64 || p.block_rows % 64 || p.block_cols % BK || p.lda % 8 || p.ldc % 8)
        return hipErrorInvalidValue;
    if (gemm_wide_supported(p, blocks)) return launch_gemm_wide(p, blocks, stream);
    // Wide outputs (QKV, FFN1) take 128-row tiles; the d-wide outputs (O, FFN2) take 64-row
    // tiles so that the grid still covers the chip.
    if (N >= 2048 && p.T > 64) return launch_cfg<4, 1, 1, 4>(p, blocks, N, stream);
    return launch_cfg<2, 1, 1, 4>(p, blocks, N, stream);
}

}  // namespace sti
