// Projections for few tokens (up to 128-192, at most 256): the regime of single-sequence inference, where
// every weight is used once and the layer is bound by how fast the packed shards stream in
// (Section "Submodel execution" runs one input at a time).
//
// A workgroup owns one 32-column strip of the output, a 64-row block of tokens and a range of
// the K dimension; its eight waves take interleaved 64-wide K tiles of that range (split-K
// inside the workgroup, at most a few tiles per wave, the first two in flight from the start),
// decode their weights in registers with the shared per-lane loader, read their A fragments
// straight from global memory (A is a few hundred KiB and cache resident), and reduce the
// eight partial accumulators through LDS.  Long reductions (FFN2) are additionally split
// across workgroups; those write float32 partial sums that the LayerNorm kernel adds up in
// a fixed order, so results do not depend on scheduling.
#include "sti_internal.hpp"
#include "weight_loader.hpp"

namespace sti {
namespace {

constexpr int BK = 64;
constexpr int NW = 8;            // waves per workgroup
constexpr int ROWS = 64;         // token rows per workgroup

__device__ inline float gelu_fast(float z)
{
    // erf by Abramowitz & Stegun 7.1.26 (|error| < 1.5e-7); results are rounded to binary16
    const float x = fabsf(z) * 0.70710678118654752440f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
    float poly = fmaf(1.061405429f, t, -1.453152027f);
    poly = fmaf(poly, t, 1.421413741f);
    poly = fmaf(poly, t, -0.284496736f);
    poly = fmaf(poly, t, 0.254829592f);
    const float e = __builtin_amdgcn_exp2f(-x * x * 1.44269504088896340736f);
    const float erf_abs = 1.0f - poly * t * e;
    return 0.5f * z * (1.0f + (z < 0.f ? -erf_abs : erf_abs));
}

template <int RA>
struct SkinnySmem {
    float red[NW][RA][16][64];                       // partial accumulators of the waves
    uint16_t lut[NW][2][kLutEntries];                // codebooks (binary16) of each wave's current and next tile
    _Float16 stage[NW][32][40];                      // output staging, one 32 x 32 tile per wave
};

// grid: x = 32-column strip, y = K split, z = 64-row block of A
template <int RA>
__global__ __launch_bounds__(NW * 64) void gemm_skinny_kernel(
    // leading scalar arguments arrive preloaded in scalar registers: what the first loads of a
    // workgroup depend on (of p, only the other fields are read)
    const void *hot_A, int32_t hot_T, int32_t hot_lda, int32_t hot_n_blocks, int32_t hot_block_rows,
    int32_t hot_block_cols, int32_t hot_kind, int32_t k_splits, int64_t partial_stride,
    GemmProblem p, GemmBlocks blocks)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    SkinnySmem<RA> &sm = *reinterpret_cast<SkinnySmem<RA> *>(smem_raw);
    const bool n_split = (hot_kind == GEMM_QKV || hot_kind == GEMM_FFN_UP);
    const int K = n_split ? hot_block_cols : hot_n_blocks * hot_block_cols;
    const int nkt = K / BK;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 5, lr = lane & 31;
    const int nw = blockIdx.x * 32;             // first output column of the strip
    const int m0 = blockIdx.z * ROWS;           // first token row of this block
    const int split = blockIdx.y;
    const int kt_begin = (int)((int64_t)nkt * split / k_splits);
    const int kt_end = (int)((int64_t)nkt * (split + 1) / k_splits);

    int nblk = 0, nrow0 = nw;
    if (n_split) {
        nblk = nw / hot_block_rows;
        nrow0 = nw - nblk * hot_block_rows;
    }
    const int tiles_per_kblock = n_split ? nkt : hot_block_cols / BK;

    struct BStage {
        Raw raw;
        int bits;
        float centroid;   // entry `lane` of the block's codebook (k-bit blocks)
    };
    // weight block of K tile kt (wave-uniform)
    auto block_of = [&](int kt) -> int { return n_split ? nblk : kt / tiles_per_kblock; };
    auto fetch_b = [&](int kt, const GemmBlock &desc) -> BStage {
        BStage st;
        int blk, ktb, row;
        if (n_split) {
            blk = nblk; ktb = kt; row = nrow0;
        } else {
            blk = kt / tiles_per_kblock; ktb = kt - blk * tiles_per_kblock; row = nw;
        }
        const int bits = desc.bits;
        st.bits = bits;
        // this lane's centroid first: staging it into LDS then waits for this load only, not for
        // the weights behind it (blocks without a codebook read the activations: valid memory,
        // value unused)
        st.centroid = *(bits <= 6 ? desc.codebook + (lane & ((1 << bits) - 1)) : (const float *)hot_A + lane);
        const uint8_t *base = (const uint8_t *)desc.w;
        if (bits == kTiledBits) {
            st.raw = load_tiled(base + tiled_cell_offset(row >> 5, ktb, hot_block_cols), lane);
        } else {
            const int64_t elem = (int64_t)(row + lr) * hot_block_cols + ktb * BK + g * 32;
            st.raw = load_raw_any(bits, base + (elem >> 5) * (bits * 4));
        }
        return st;
    };
    struct AStage {
        u32x4 f[RA][4];
    };
    const _Float16 *A = (const _Float16 *)hot_A;
    auto fetch_a = [&](int kt) -> AStage {
        AStage st;
#pragma unroll
        for (int i = 0; i < RA; ++i) {
            const int m = min(m0 + i * 32 + lr, hot_T - 1);   // rows past T repeat row T-1; their results are not stored
            const _Float16 *src = A + (int64_t)m * hot_lda + kt * BK + g * 32;
#pragma unroll
            for (int s = 0; s < 4; ++s) st.f[i][s] = *(const u32x4 *)(src + s * 8);
        }
        return st;
    };

    float16v acc[RA];
#pragma unroll
    for (int i = 0; i < RA; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

    // Two tiles in flight before anything else is waited for.  Order of the requests: the A
    // fragments (they need nothing but the leading arguments), then every block descriptor this
    // wave will look at (those of its first two tiles and of the codebooks it stages) in one
    // round of scalar loads, then the weights, then the centroids.
    int kt = kt_begin + wave;
    AStage a_cur, a_nxt;
    BStage b_cur, b_nxt;
    if (kt < kt_end) a_cur = fetch_a(kt);
    if (kt + NW < kt_end) a_nxt = fetch_a(kt + NW);
    const int last_blk = hot_n_blocks - 1;
    const GemmBlock desc0 = blocks.b[min(block_of(min(kt, nkt - 1)), last_blk)];
    const GemmBlock desc1 = blocks.b[min(block_of(min(kt + NW, nkt - 1)), last_blk)];
    if (kt < kt_end) b_cur = fetch_b(kt, desc0);
    if (kt + NW < kt_end) b_nxt = fetch_b(kt + NW, desc1);
    // Each wave keeps the codebooks of its own current and next tile in LDS (binary16): no
    // workgroup-wide table, no barrier, and no descriptor beyond those of the tiles themselves.
    static_assert(kLutEntries == 64, "one lane per centroid");
    auto stage_lut = [&](int slot, const BStage &st) {
        if (st.bits <= 6) sm.lut[wave][slot][lane] = (uint16_t)f16_bits(st.centroid);
    };
    if (kt < kt_end) stage_lut(0, b_cur);
    if (kt + NW < kt_end) stage_lut(1, b_nxt);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    for (int slot = 0; kt < kt_end; kt += NW, slot ^= 1) {
        const BStage bs = b_cur;
        const AStage as = a_cur;
        b_cur = b_nxt; a_cur = a_nxt;
        half8 bf[4];
        decode_raw_any(bs.bits, bs.raw, sm.lut[wave][slot], bf);
        if (kt + 2 * NW < kt_end) {   // (a third tile per wave: rare; its codebook takes the slot just read)
            b_nxt = fetch_b(kt + 2 * NW, blocks.b[block_of(kt + 2 * NW)]);
            a_nxt = fetch_a(kt + 2 * NW);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            stage_lut(slot, b_nxt);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int i = 0; i < RA; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, as.f[i][s]),
                                                               bf[s], acc[i], 0, 0, 0);
    }

    // ---- reduce the partial accumulators; wave i finishes fragment i ----
#pragma unroll
    for (int i = 0; i < RA; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) sm.red[wave][i][v][lane] = acc[i][v];
    __syncthreads();

    float bias = 0.f;
    if (n_split) {
        const int nrow = nrow0 + lr;
        if (hot_kind == GEMM_QKV) {
            const int which = nrow / p.d_head, e = nrow - which * p.d_head;
            const float *bp = which == 0 ? p.bias0 : (which == 1 ? p.bias1 : p.bias2);
            bias = bp[blocks.b[nblk].shard * p.d_head + e];
        } else {
            bias = p.bias0[blocks.b[nblk].shard * hot_block_rows + nrow];
        }
    }
#pragma unroll
    for (int i = 0; i < RA; ++i) {
        if (i != wave) continue;   // wave-uniform
        float sum[16];
#pragma unroll
        for (int v = 0; v < 16; ++v)
            sum[v] = ((sm.red[0][i][v][lane] + sm.red[1][i][v][lane]) +
                      (sm.red[2][i][v][lane] + sm.red[3][i][v][lane])) +
                     ((sm.red[4][i][v][lane] + sm.red[5][i][v][lane]) +
                      (sm.red[6][i][v][lane] + sm.red[7][i][v][lane]));
        if (!n_split) {
            // raw float32 (partial) sums; bias, residual and LayerNorm follow in the row kernel
            float *C = (float *)p.C + (int64_t)split * partial_stride;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + i * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
                if (m < hot_T) C[(int64_t)m * p.ldc + nw + lr] = sum[v];
            }
        } else {
            _Float16 *st = &sm.stage[wave][0][0];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float x = sum[v] + bias;
                if (hot_kind == GEMM_FFN_UP) x = gelu_fast(x);
                st[((v >> 2) * 8 + g * 4 + (v & 3)) * 40 + lr] = (_Float16)x;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            _Float16 *C = (_Float16 *)p.C;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int c = lane + 64 * j;   // 16-byte chunk of the 32 x 32 tile
                const int row = c >> 2, cc = c & 3;
                const int m = m0 + i * 32 + row;
                if (m < hot_T)
                    *(u32x4 *)(C + (int64_t)m * p.ldc + nw + cc * 8) = *(const u32x4 *)(st + row * 40 + cc * 8);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
}

template <int RA>
hipError_t launch_ra(const GemmProblem &p, const GemmBlocks &blocks, int N, int k_splits,
                     int64_t partial_stride, hipStream_t stream)
{
    dim3 grid(N / 32, k_splits, (p.T + ROWS - 1) / ROWS);
    // more than 64 KiB of dynamic LDS needs an explicit opt-in: once per instantiation, and safe
    // when several host threads make their first call together
    static const hipError_t attr_status =
        hipFuncSetAttribute((const void *)gemm_skinny_kernel<RA>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)sizeof(SkinnySmem<RA>));
    if (attr_status != hipSuccess) return attr_status;
    launch((gemm_skinny_kernel<RA>), grid, dim3(NW * 64), sizeof(SkinnySmem<RA>), stream, p.A, p.T, p.lda, p.n_blocks,
           p.block_rows, p.block_cols, (int32_t)p.kind, k_splits, partial_stride, p, blocks);
    return hipGetLastError();
}

}  // namespace

int skinny_k_splits(const GemmProblem &p)
{
    const bool n_split = (p.kind == GEMM_QKV || p.kind == GEMM_FFN_UP);
    if (n_split) return 1;
    const int nkt = p.n_blocks * p.block_cols / BK;
    int s = nkt / (2 * NW);       // about two K tiles per wave
    if (s < 1) s = 1;
    if (s > kSkinnyMaxSplits) s = kSkinnyMaxSplits;
    return s;
}

hipError_t launch_gemm_skinny(const GemmProblem &p, const GemmBlocks &blocks, int k_splits,
                              int64_t partial_stride, hipStream_t stream)
{
    const bool n_split = (p.kind == GEMM_QKV || p.kind == GEMM_FFN_UP);
    const int N = n_split ? p.n_blocks * p.block_rows : p.block_rows;
    if (p.T <= 0 || N <= 0) return hipSuccess;
    if (N % 32 || p.block_rows % 32 || p.block_cols % BK || p.lda % 8 || p.ldc % 8 || k_splits < 1)
        return hipErrorInvalidValue;
    if (p.T <= 32) return launch_ra<1>(p, blocks, N, k_splits, partial_stride, stream);
    return launch_ra<2>(p, blocks, N, k_splits, partial_stride, stream);
}

}  // namespace sti
