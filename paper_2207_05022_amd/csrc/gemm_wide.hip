// Projections of the layer on the matrix cores for many tokens (Section "A primer on
// transformer": the Q/K/V, output and two FFN linear layers), with the weights taken from
// the per-layer fragment-tiled binary16 working buffer (Section "Submodel execution": a
// layer's shards are decompressed into a working buffer before the layer runs).
//
//   C[T x N] = A[T x K] * W^T,  float32 accumulation in v_mfma_f32_32x32x16_f16.
//
// One workgroup of NW waves owns a (RA*32) x (NW*32) tile and is sized so that a compute
// unit holds all its waves at once (12 wave slots at this register budget): all waves of a
// unit then move through the K loop in step, share one copy of the A tile and finish together.
//   - the A tile [BM x 64] goes global -> LDS directly (global_load_lds_dwordx4, no
//     registers, no LDS store instructions), three stages; its 16-byte chunks are XOR-swizzled
//     by row pair so that the unpadded rows read without bank conflicts;
//   - a wave's weight fragments are contiguous 1 KiB loads from the working buffer, two K
//     tiles ahead, straight into registers; both kinds of load address memory as a scalar
//     base plus a 32-bit lane offset (measured 1.5 % faster end to end than 64-bit lane
//     addresses);
//   - the A fragments of k-step s+1 are read from LDS while the MFMAs of step s run;
//   - the weight fragment is the first MFMA operand, so a lane's accumulators are runs of
//     output columns of one token row; v_permlane32_swap merges them into 16-byte pieces,
//     which get bias / GELU / residual in registers and leave through an LDS copy of the
//     whole tile, so that every global store instruction writes whole rows of the tile.
//
// Sequences of exactly 128 tokens (the padded length the paper profiles with): a 128-row tile is
// one whole sequence, so the Q/K/V projection is cut into 128 x 384 tiles = Q | K | V of two
// heads, and the workgroup that has multiplied such a tile keeps it in LDS and computes those
// heads' attention itself (kind GEMM_QKV_ATTN): no Q/K/V buffer in memory and no attention launch.
#include "sti_internal.hpp"
#include "weight_loader.hpp"
#include "attention_core.hpp"

// STI_PHASE_STAMPS (the phase-budget build libsti_phases.so only, never the product library): wave 0
// of every workgroup reads the shader clock counter at six points (kernel entry, prologue loads
// requested, first K tile landed, K loop done, epilogue arithmetic done, last store acknowledged)
// plus the 100 MHz wall clock at both ends, keeps the values in scalar registers (a store inside the
// K loop would count against its hand-written waits) and writes them once, at its exit.
#ifdef STI_PHASE_STAMPS
namespace {
constexpr int kStampKinds = 5, kStampSlots = 512, kStampWords = 8;
__device__ unsigned long long sti_phase_stamps[kStampKinds * kStampSlots * kStampWords];
}
// out: [kind][slot][8] = six clock stamps, wall clock at entry, wall clock at exit (0 = slot unused)
extern "C" int sti_phase_stamps_read(unsigned long long *out, int clear)
{
    hipError_t e = hipMemcpyFromSymbol(out, HIP_SYMBOL(sti_phase_stamps), sizeof(sti_phase_stamps));
    if (e == hipSuccess && clear) {
        void *dev = nullptr;
        e = hipGetSymbolAddress(&dev, HIP_SYMBOL(sti_phase_stamps));
        if (e == hipSuccess) e = hipMemset(dev, 0, sizeof(sti_phase_stamps));
    }
    return (int)e;
}
#define STI_STAMP(i) (stamp[i] = __builtin_amdgcn_s_memtime())
#define STI_STAMPS_OUT()                                                                               \
    do {                                                                                               \
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                                               \
        STI_STAMP(5);                                                                                  \
        const unsigned slot = blockIdx.y * gridDim.x + blockIdx.x;                                     \
        if (threadIdx.x == 0 && slot < (unsigned)kStampSlots) {                                        \
            unsigned long long *o = sti_phase_stamps + ((size_t)KIND * kStampSlots + slot) * kStampWords; \
            for (int i_ = 0; i_ < 6; ++i_) o[i_] = stamp[i_];                                          \
            o[6] = wall0;                                                                              \
            o[7] = wall_clock64();                                                                     \
        }                                                                                              \
    } while (0)
#else
#define STI_STAMP(i) ((void)0)
#define STI_STAMPS_OUT() ((void)0)
#endif

namespace sti {
namespace {

constexpr int BK = 64;   // K positions per LDS stage
constexpr int kComputeUnits = 256;
constexpr int kGroupRows = 8;   // row tiles per band of the tile order ...
constexpr int kRowMajorColumnTiles = 12;   // ... used beyond this many column tiles

typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) const void global_cptr;
typedef __attribute__((address_space(3))) void lds_ptr;

// GELU with the Gaussian CDF (the erf form, not the tanh form):  z * Phi(z),
// Phi(z) = 1/2 + z * R(z^2).  R is a degree-8 polynomial in u = 2 z^2 / 4.5^2 - 1, fitted in
// float64 (weighted least squares on Chebyshev nodes) to (Phi(z) - 1/2) / z on |z| <= 4.5;
// beyond that Phi is taken at the clamped argument (1 - Phi(4.5) = 3.4e-6).  Evaluated in
// float32 the absolute error of the result is below 5e-5 for all z (0.1 of a binary16 ulp at
// 0.35, the value at z = 0.6 where the error peaks) and its relative error below 1e-4 for
// z > -1; 13 arithmetic instructions per value and no transcendental ones, which matters
// because the epilogue of the FFN1 projection is bound by exactly these instructions.
__device__ inline float gelu_erf(float z)
{
    const float zc = __builtin_amdgcn_fmed3f(z, -4.5f, 4.5f);
    const float u = fmaf(zc * zc, 2.0f / 20.25f, -1.0f);
    float r = 3.174704981e-03f;
    r = fmaf(r, u, -9.158361878e-03f);
    r = fmaf(r, u, 1.244540513e-02f);
    r = fmaf(r, u, -1.696567595e-02f);
    r = fmaf(r, u, 2.754268719e-02f);
    r = fmaf(r, u, -4.047719455e-02f);
    r = fmaf(r, u, 5.482644199e-02f);
    r = fmaf(r, u, -7.717846451e-02f);
    r = fmaf(r, u, 1.569020774e-01f);
    return z * fmaf(zc, r, 0.5f);
}

// LDS of the attention that follows the Q/K/V tile (GEMM_QKV_ATTN): per head Q and K row-major
// with padded rows and V transposed, for 128 positions of 64 features
constexpr int ATT_L = 128, ATT_DH = 64, ATT_KPAD = ATT_DH + 8, ATT_VTS = ATT_L + 8;
constexpr int ATT_HEAD_HALVES = 2 * ATT_L * ATT_KPAD + ATT_DH * ATT_VTS;
constexpr size_t kAttentionLdsBytes = (size_t)2 * ATT_HEAD_HALVES * 2;

template <int RA, int NW, int KS>
constexpr size_t wide_lds_bytes()
{
    constexpr size_t stages = (size_t)KS * 3 * (RA * 32) * BK * 2;
    constexpr size_t tile = (size_t)(RA * 32) * (NW * 32 + 8) * 2;
    constexpr size_t partial = (size_t)(KS - 1) * (RA * 32) * (NW * 32) * 4;
    constexpr size_t m = stages > tile ? stages : tile;
    return m > partial ? m : partial;
}

// Workgroups of a Q/K/V launch beyond those of its tiles.  With 128-token sequences the launch has one
// 128 x 384 tile per sequence and pair of heads (192 for 32 sequences of BERT-base), with a few hundred
// tokens a few dozen tiles: fewer than the chip has compute units, so these land on units the tiles
// leave idle.  They decompress the next layer's shards into its working buffer (Section "Submodel
// execution": the next layer is made ready while the current one computes) - work that is bound by
// memory latency and bandwidth, beside a projection that is bound by the matrix cores.
// All waves of the workgroup come here.  LDS: the binary16 codebooks, bitwidths and data pointers of all
// shards, so that a cell costs one round trip to memory; a wave asks for three cells at a time, the first
// three together with the codebooks (a short projection must not end up waiting for these workgroups).
constexpr size_t kNextDecodeLdsBytes = (size_t)kMaxShardsPerLayer * (kLutEntries * 2 + 4 + 8);

template <int NWAVES>
__device__ inline void decode_next_layer(const GemmProblem &p, int d, unsigned char *smem, int worker)
{
    uint16_t *luts = (uint16_t *)smem;                                                    // [shards][64]
    int32_t *bits_of = (int32_t *)(smem + (size_t)kMaxShardsPerLayer * kLutEntries * 2);  // [shards]
    uint64_t *data_of = (uint64_t *)(smem + (size_t)kMaxShardsPerLayer * (kLutEntries * 2 + 4));
    // (pointers that come out of memory are taken as global-memory pointers by hand: the compiler would
    //  address through them with the slower flat instructions)
    auto as_global = [](uint64_t a) { return (const void *)(global_cptr *)a; };
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // round trip 1: the descriptors; round trip 2: the codebooks together with the first cells
    constexpr int SPW = (kMaxShardsPerLayer + NWAVES - 1) / NWAVES;   // shards a wave stages
    float centroid[SPW];
    int staged_bits[SPW];
#pragma unroll
    for (int j = 0; j < SPW; ++j) {
        const int s = wave + j * NWAVES;
        centroid[j] = 0.f;
        staged_bits[j] = 0;
        if (s < p.next_shards) {
            const ShardDesc sd = p.next_table[s];
            staged_bits[j] = sd.bits;
            if (lane == 0) {
                bits_of[s] = sd.bits;
                data_of[s] = (uint64_t)sd.data;
            }
            if (sd.bits <= 6 && lane < (1 << sd.bits)) centroid[j] = ((const float *)as_global((uint64_t)sd.codebook))[lane];
        }
    }
    __syncthreads();
    const int dh = p.d_head, f = p.next_ffn_per_shard;
    const int total = (int)((int64_t)d * (4 * dh + 2 * f) / 2048) * p.next_shards;
    const int stride = p.next_workgroups * NWAVES;
    constexpr int CH = 3;   // cells a wave asks for at a time
    TiledCell t[CH];
    int bits[CH];
    Raw raw[CH];
    auto request = [&](int first) {
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int cell = first + c * stride;
            bits[c] = 0;   // (no cell)
            if (cell < total) {
                t[c] = locate_tiled_cell(cell, d, dh, f);
                bits[c] = bits_of[t[c].shard];
                raw[c] = load_tiled_cell_raw(t[c], bits[c], as_global(data_of[t[c].shard]), lane);
            }
        }
    };
    int first = worker * NWAVES + wave;
    request(first);
#pragma unroll
    for (int j = 0; j < SPW; ++j) {
        const int s = wave + j * NWAVES;
        if (s < p.next_shards && staged_bits[j] <= 6 && lane < (1 << staged_bits[j]))
            luts[s * kLutEntries + lane] = (uint16_t)f16_bits(centroid[j]);
    }
    __syncthreads();
    while (first < total) {
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            if (bits[c] != 0) {
                half8 fr[4];
                decode_raw_any(bits[c], raw[c], luts + t[c].shard * kLutEntries, fr);
                store_tiled_cell(t[c], d, dh, f, fr, (uint8_t *)p.next_out, lane);
            }
        }
        first += CH * stride;
        if (first < total) request(first);
    }
}

// KS = 2 (outputs as narrow as d_model, long K): the workgroup has two groups of NW waves that
// each take one half of K for the same tile, with A stages of their own; the second group
// hands its accumulators over through LDS at the end.  Twice the waves per compute unit for
// a tile count that is fixed by the output size.
template <int KIND, int RA, int NW, int KS, bool EARLY>
__global__ __launch_bounds__(NW * KS * 64, 3) void gemm_wide_kernel(
    // what the first loads of a workgroup depend on, as leading scalar arguments: these arrive
    // preloaded in scalar registers (the build asks for kernel-argument preloading), so that the
    // first A fetches and weight loads are not behind a round trip to the argument buffer
    // (14 dwords fit: block_shape = block_rows | block_cols << 16, blocks_splits = n_blocks | k_splits << 16)
    const void *hot_A, const void *hot_w0, const void *hot_resid, const float *hot_bias0, int32_t hot_w_stride,
    int32_t hot_T, int32_t hot_lda, int32_t hot_ldr, uint32_t hot_block_shape, uint32_t hot_blocks_splits,
    GemmProblem p, GemmBlocks blocks)   // (of p, only the fields that are not among the leading arguments are read)
{
    const int hot_block_rows = hot_block_shape & 0xffff, hot_block_cols = hot_block_shape >> 16;
    const int hot_n_blocks = hot_blocks_splits & 0xffff, hot_k_splits = hot_blocks_splits >> 16;
#ifdef STI_PHASE_STAMPS
    unsigned long long stamp[6] = {0, 0, 0, 0, 0, 0};
    const unsigned long long wall0 = wall_clock64();
    STI_STAMP(0);
#endif
    constexpr int BM = RA * 32, BN = NW * 32, NT = NW * KS * 64, NTH = NW * 64;
    constexpr bool n_split = (KIND == GEMM_QKV || KIND == GEMM_FFN_UP || KIND == GEMM_QKV_ATTN);
    constexpr bool qkv = (KIND == GEMM_QKV || KIND == GEMM_QKV_ATTN);
    static_assert(KIND != GEMM_QKV_ATTN || (RA == 4 && NW == 12 && KS == 1), "two heads of one 128-token sequence per tile");
    constexpr int STAGE = BM * BK;              // halves per A stage
    constexpr int FETCHES = BM / 8;             // fetch instructions per A stage: 8 rows (1 KiB) each
    constexpr int FPW = (FETCHES + NW - 1) / NW;   // per wave: wave w issues fetches w, w + NW, ...
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];

    const int N = n_split ? hot_n_blocks * hot_block_rows : hot_block_rows;
    const int K = n_split ? hot_block_cols : hot_n_blocks * hot_block_cols;
    // K is split over the KS wave groups of the workgroup and, for few tiles, over
    // gridDim.y workgroups per tile as well (raw float32 partial sums, see the epilogue)
    const int splits = (!n_split && hot_k_splits > 1) ? hot_k_splits : 1;
    const int nkt = K / BK / KS / splits;  // K tiles of this wave's group
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = wave_all / NW, wave = wave_all - half * NW;   // K group, column strip
    const int kt0 = ((int)blockIdx.y * KS + half) * nkt;
    const int g = lane >> 5, lr = lane & 31;
    // Workgroups are handed to the 8 XCDs round-robin by linear id; give each XCD one
    // contiguous range of the tile order: row by row up to kRowMajorColumnTiles column tiles;
    // beyond that (d_model 2048: 22 column tiles) row by row would stream every weight column
    // through the L2 once per row tile, and the order walks bands of kGroupRows row tiles column
    // by column instead, so that the workgroups that run together share weight columns too
    // (measured at d_model 2048, 4096 tokens: 720 -> 617 us per layer; at 8 to 11 column
    // tiles the two orders measure the same within run-to-run noise).
    const int n_tiles = (N + BN - 1) / BN;
    const int m_tiles = (hot_T + BM - 1) / BM;
    const int total_tiles = n_tiles * m_tiles;
    const int per_xcd = (total_tiles + 7) / 8;
    const int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if constexpr (qkv) {
        if ((int)(blockIdx.x >> 3) >= per_xcd) {   // behind the tiles' workgroups: the next layer's decompression
            if (p.next_workgroups > 0) decode_next_layer<NW * KS>(p, hot_block_cols, smem_raw, (int)blockIdx.x - 8 * per_xcd);
            return;
        }
    }
    if ((int)(blockIdx.x >> 3) >= per_xcd || tile >= total_tiles) return;
    const int group = n_tiles > kRowMajorColumnTiles ? kGroupRows : 1;
    const int band = tile / (group * n_tiles);
    const int band_rows = min(group, m_tiles - band * group);   // the last band may be short
    const int in_band = tile - band * (group * n_tiles);
    const int tile_n = in_band / band_rows;
    const int tile_m = band * group + (in_band - tile_n * band_rows);
    const int m0 = tile_m * BM;
    // N and the block widths are multiples of 32, so a wave's columns are all inside or all
    // outside the matrix; a wave outside recomputes the first columns and its results are
    // dropped by the column mask of the stores
    const int nw_real = tile_n * BN + wave * 32;
    const int nw = nw_real < N ? nw_real : 0;
    int nblk = 0, nrow0 = nw;
    if (n_split) {
        nblk = nw / hot_block_rows;
        nrow0 = nw - nblk * hot_block_rows;
    }
    const int tiles_per_kblock = n_split ? nkt * KS : hot_block_cols / BK;

    float16v acc[RA];
#pragma unroll
    for (int i = 0; i < RA; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

    // ---- A tile: lane l of a fetch instruction fills LDS slot (row l/8, chunk l%8) of its 8
    //      rows with the chunk (l%8) ^ ((row/2)%8) of that row, so that the 16 rows that one
    //      quarter of a fragment read touches (128-byte rows, two per 64-bank line) fall on
    //      16 different bank groups; rows past T repeat row T-1 ----
    const _Float16 *A = (const _Float16 *)hot_A + (int64_t)m0 * hot_lda;   // first row of the tile
    uint32_t src[FPW];   // byte offset of this lane's chunk from the tile's first row and K tile
#pragma unroll
    for (int j = 0; j < FPW; ++j) {
        const int row = (wave + NW * j) * 8 + (lane >> 3);   // row inside the tile
        const int r = m0 + row < hot_T ? row : hot_T - 1 - m0;
        src[j] = (uint32_t)((r * hot_lda + (((lane & 7) ^ ((row >> 1) & 7)) * 8)) * 2);   // < 2^24 * 2
    }
    // The loads of the K loop are written as instructions rather than through the compiler:
    // its own bookkeeping would wait for every outstanding fetch into LDS before the next LDS
    // read, which is exactly the overlap this loop is built for.  The waits are in step().
    const uint32_t lds_base = (uint32_t)(size_t)(lds_ptr *)smem_raw;
    auto fetch_a = [&](int kt, int buf) {
#pragma unroll
        for (int j = 0; j < FPW; ++j) {
            if (wave + NW * j < FETCHES) {
                const _Float16 *gp = A + (kt0 + kt) * BK;   // scalar base, per-lane 32-bit offset
                const uint32_t dst = lds_base + (uint32_t)(((half * 3 + buf) * STAGE + (wave + NW * j) * 8 * BK) * 2);
                asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                             :: "v"(src[j]), "s"(gp), "s"(dst) : "memory", "m0");
            }
        }
    };
    // byte offset of this lane's fragment of k-step s inside row block 0 of a stage
    int frag_off[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) frag_off[s] = lr * (BK * 2) + (((g * 4 + s) ^ ((lr >> 1) & 7)) * 16);

    const uint32_t lane16 = lane * 16;
    auto frag_ptr = [&](int kt) -> const uint8_t * {
        int blk, ktb, row;
        kt += kt0;
        if (n_split) {
            blk = nblk; ktb = kt; row = nrow0;
        } else {
            blk = kt / tiles_per_kblock; ktb = kt - blk * tiles_per_kblock; row = nw;
        }
        // (the blocks of a working buffer lie at a constant distance: no look-up in the block table)
        const uint8_t *base = (const uint8_t *)hot_w0 + (int64_t)blk * hot_w_stride;   // (stride < 2^31)
        return base + tiled_cell_offset(row >> 5, ktb, hot_block_cols);   // wave-uniform
    };

    // Three A stages and three sets of weight fragment registers: the loads of K tile t+2 are
    // issued while tile t is multiplied (A fetches first, then the 4 fragment loads; with K
    // unsplit behind the MFMAs of the first k-step, so that those start right after the
    // barrier: measured 2 % faster end to end than issuing at the top, while the split-K
    // shapes are faster with the issue at the top).  The wait in front of the barrier is
    // written by hand: it lets the loads of tile t+1, the last ones issued, stay in flight.
    u32x4 bw[3][4];
    int n_fetch = 0;   // A fetches this wave issues per stage
#pragma unroll
    for (int j = 0; j < FPW; ++j) n_fetch += (wave + NW * j < FETCHES) ? 1 : 0;
    auto issue = [&](int kt, u32x4 (&dst)[4]) {
        fetch_a(kt, kt % 3);
        const uint8_t *q = frag_ptr(kt);
        asm volatile("global_load_dwordx4 %0, %4, %5\n\t"
                     "global_load_dwordx4 %1, %4, %5 offset:1024\n\t"
                     "global_load_dwordx4 %2, %4, %5 offset:2048\n\t"
                     "global_load_dwordx4 %3, %4, %5 offset:3072"
                     : "=&v"(dst[0]), "=&v"(dst[1]), "=&v"(dst[2]), "=&v"(dst[3]) : "v"(lane16), "s"(q) : "memory");
    };
#define STI_WAIT_LOADS(n) asm volatile("s_waitcnt vmcnt(" #n ")" ::: "memory")
    // EARLY (64-row tiles of the d_model-wide projections, K not split over workgroups): what
    // the epilogue adds (bias and residual rows) is asked for before the K loop: asked for in
    // the epilogue, these loads cost a whole round trip (3-4 thousand clocks of a 20-50 thousand
    // clock kernel).  They are the oldest loads in flight, so the first wait of the K loop
    // covers them.  (A variant of its own: with K split over workgroups nothing is added here.)
    constexpr bool PRE = EARLY;
    static_assert(!EARLY || (!n_split && RA <= 2), "early operands: 64-row tiles of OUT / FFN_DOWN");
    const _Float16 *R = (const _Float16 *)hot_resid;
    f32x4 bias[2][2];
    u32x4 resv[PRE ? RA : 1][2];
    auto load_epilogue_operands = [&]() {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int c = 16 * q + 8 * g;     // first column of the piece inside the wave's strip
            const float *bp;
            if constexpr (qkv) {
                const int nrow = nrow0 + c;
                const int which = nrow / p.d_head, e0 = nrow - which * p.d_head;
                bp = (which == 0 ? hot_bias0 : (which == 1 ? p.bias1 : p.bias2)) + blocks.b[nblk].shard * p.d_head + e0;
            } else if constexpr (KIND == GEMM_FFN_UP) {
                bp = hot_bias0 + blocks.b[nblk].shard * hot_block_rows + nrow0 + c;
            } else {
                bp = hot_bias0 + nw + c;
            }
            bias[q][0] = *(const f32x4 *)bp;
            bias[q][1] = *(const f32x4 *)(bp + 4);
        }
        if constexpr (PRE) {
#pragma unroll
            for (int i = 0; i < RA; ++i) {
                const int m = min(m0 + i * 32 + lr, hot_T - 1);   // (rows past T: row T-1 again, never stored)
#pragma unroll
                for (int q = 0; q < 2; ++q) resv[i][q] = *(const u32x4 *)(R + (int64_t)m * hot_ldr + nw + 16 * q + 8 * g);
            }
        }
    };
    auto step = [&](int kt, u32x4 (&bcur)[4], u32x4 (&bnew)[4]) {
        // the weight fragments and the A stage of tile kt have landed (the barrier below is a
        // scheduling boundary: no MFMA of this step is placed above the wait) ...
        if (kt + 1 < nkt) {
            if (n_fetch == 2) STI_WAIT_LOADS(6);
            else if (n_fetch == 1) STI_WAIT_LOADS(5);
            else STI_WAIT_LOADS(4);
        } else {
            STI_WAIT_LOADS(0);
        }
        // ... for every wave, and every wave is done reading the stage that is refilled next
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
#ifdef STI_PHASE_STAMPS
        if (kt == 0) STI_STAMP(2);
#endif
        if (KS == 2 && kt + 2 < nkt) issue(kt + 2, bnew);
        const unsigned char *stage = smem_raw + (half * 3 + kt % 3) * (STAGE * 2);
        half8 a_cur[RA], a_nxt[RA];
#pragma unroll
        for (int i = 0; i < RA; ++i) a_cur[i] = *(const half8 *)(stage + i * (32 * BK * 2) + frag_off[0]);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if (s < 3) {
#pragma unroll
                for (int i = 0; i < RA; ++i)
                    a_nxt[i] = *(const half8 *)(stage + i * (32 * BK * 2) + frag_off[s + 1]);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < RA; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, bcur[s]), a_cur[i],
                                                              acc[i], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (KS == 1 && s == 0 && kt + 2 < nkt) issue(kt + 2, bnew);
            __builtin_amdgcn_sched_barrier(0);
            if (s < 3) {
#pragma unroll
                for (int i = 0; i < RA; ++i) a_cur[i] = a_nxt[i];
            }
        }
    };
    static_assert(FPW <= 2, "the hand-written waits cover up to two A fetches per wave");
    if (PRE && half == 0) load_epilogue_operands();
    if (nkt > 0) issue(0, bw[0]);
    if (nkt > 1) issue(1, bw[1]);
    STI_STAMP(1);
    for (int kt = 0; kt < nkt; kt += 3) {
        step(kt, bw[0], bw[2]);
        if (kt + 1 < nkt) step(kt + 1, bw[1], bw[0]);
        if (kt + 2 < nkt) step(kt + 2, bw[2], bw[1]);
    }
#undef STI_WAIT_LOADS
    STI_STAMP(3);

    // ---- epilogue ----
    // Lane l holds token row lr and output columns (v/4)*8 + g*4 + v%4 of each 32 x 32 block.
    // Swapping the column groups 2q and 2q+1 between lanes l and l+32 leaves the lane with the
    // 8 consecutive columns 16q + 8g .. +8 of its row: one 16-byte piece of the output row.
    constexpr int LDT = BN + 8;   // padded row of the staged tile (halves): conflict-free 16-byte writes
    _Float16 *tile_out = (_Float16 *)smem_raw;
    // (also when K is split over workgroups and nothing is added here: leaving these loads out
    //  made those launches 2 % slower, measured twice)
    if (!PRE) load_epilogue_operands();
    __syncthreads();   // every wave is done with the A stages
    if constexpr (KIND == GEMM_QKV_ATTN) {
        // ---- the tile is Q | K | V of heads 2 tile_n and 2 tile_n + 1 for the 128 positions of
        //      sequence tile_m: leave them in LDS (binary16, bias added: the values the unfused
        //      route stores) and run the two heads' attention (Section "A primer on transformer":
        //      per-head attention scores) with eight of the twelve waves, 32 queries each ----
        _Float16 *hb = (_Float16 *)smem_raw + (wave / 6) * ATT_HEAD_HALVES;   // this wave's head
        const int part = (wave % 6) >> 1;      // 0 Q, 1 K, 2 V (wave-uniform)
        const int ch = (wave & 1) * 32;        // first feature of the wave's 32 columns
#pragma unroll
        for (int i = 0; i < RA; ++i) {
            const int row = i * 32 + lr;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                half8 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float lo = acc[i][(2 * q) * 4 + e], hi = acc[i][(2 * q + 1) * 4 + e];
                    const auto sw = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(uint32_t, lo),
                                                                     __builtin_bit_cast(uint32_t, hi), false, false);
                    const uint32_t s0 = sw[0], s1 = sw[1];
                    o[e] = (_Float16)(__builtin_bit_cast(float, s0) + bias[q][0][e]);
                    o[4 + e] = (_Float16)(__builtin_bit_cast(float, s1) + bias[q][1][e]);
                }
                const int c = ch + 16 * q + 8 * g;
                if (part < 2) {
                    *(half8 *)(hb + part * (ATT_L * ATT_KPAD) + row * ATT_KPAD + c) = o;
                } else {
                    _Float16 *vt = hb + 2 * (ATT_L * ATT_KPAD);
#pragma unroll
                    for (int e = 0; e < 8; ++e) vt[(c + e) * ATT_VTS + row] = o[e];
                }
            }
        }
        __syncthreads();
        STI_STAMP(4);   // (here: Q, K, V of the tile are in LDS; what follows is the attention)
        const int head = tile_n * 2 + (wave >> 2);          // present-head index of waves 0..7
        if (wave >= 8 || head >= hot_n_blocks) return;
        hb = (_Float16 *)smem_raw + (wave >> 2) * ATT_HEAD_HALVES;
        const _Float16 *Qs = hb, *Ks = hb + ATT_L * ATT_KPAD, *Vt = hb + 2 * (ATT_L * ATT_KPAD);
        int Lk = ATT_L;
        if (p.key_lengths) Lk = min(max(p.key_lengths[tile_m], 1), ATT_L);
        const int qrow = (wave & 3) * 32 + lr;
        half8 qf[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) qf[s] = *(const half8 *)(Qs + qrow * ATT_KPAD + s * 16 + g * 8);
        float16v ov[2];
        const float run_sum = attention_scores_in_registers<4>(qf, Ks, ATT_KPAD, Vt, ATT_VTS, Lk, lane, ov);
        const float inv = 1.0f / run_sum;
        _Float16 *out = (_Float16 *)p.C + (int64_t)(m0 + qrow) * p.ldc + head * ATT_DH;
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                half4 h;
#pragma unroll
                for (int i = 0; i < 4; ++i) h[i] = (_Float16)(ov[e][v4 * 4 + i] * inv);
                *(half4 *)(out + e * 32 + v4 * 8 + g * 4) = h;
            }
        STI_STAMPS_OUT();
        return;
    }
    if constexpr (KS == 2) {
        // second K group -> LDS -> first K group (same lane, same registers)
        float *part = (float *)smem_raw;
        const int th = tid - half * NTH;
        if (half == 1) {
#pragma unroll
            for (int i = 0; i < RA; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) part[(i * 16 + v) * NTH + th] = acc[i][v];
        }
        __syncthreads();
        if (half == 0) {
#pragma unroll
            for (int i = 0; i < RA; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][v] += part[(i * 16 + v) * NTH + th];
        }
        __syncthreads();   // the sums are in registers: the buffer can take the staged tile
    }
    if (splits > 1) {
        // one of several workgroups of this tile: raw float32 sums, 32 bytes per lane and piece
        if (half == 0 && nw_real < N) {
            float *Cf = (float *)p.C + (int64_t)blockIdx.y * p.partial_stride;
#pragma unroll
            for (int i = 0; i < RA; ++i) {
                const int m = m0 + i * 32 + lr;
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    float x[8];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float lo = acc[i][(2 * q) * 4 + e], hi = acc[i][(2 * q + 1) * 4 + e];
                        const auto sw = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(uint32_t, lo),
                                                                         __builtin_bit_cast(uint32_t, hi), false, false);
                        const uint32_t s0 = sw[0], s1 = sw[1];
                        x[e] = __builtin_bit_cast(float, s0);
                        x[4 + e] = __builtin_bit_cast(float, s1);
                    }
                    if (m < hot_T) {
                        float *dst = Cf + (int64_t)m * p.ldc + nw + 16 * q + 8 * g;
                        *(f32x4 *)dst = f32x4{x[0], x[1], x[2], x[3]};
                        *(f32x4 *)(dst + 4) = f32x4{x[4], x[5], x[6], x[7]};
                    }
                }
            }
        }
        STI_STAMP(4);
        STI_STAMPS_OUT();
        return;
    }
    if (half == 0) {
#pragma unroll
    for (int i = 0; i < RA; ++i) {
        const int row = i * 32 + lr;          // row inside the tile
        half8 res[2];
        if constexpr (PRE) {
            res[0] = __builtin_bit_cast(half8, resv[i][0]);
            res[1] = __builtin_bit_cast(half8, resv[i][1]);
        } else if constexpr (!n_split) {
            const int m = m0 + row;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                u32x4 v = {0, 0, 0, 0};
                if (m < hot_T) v = *(const u32x4 *)(R + (int64_t)m * hot_ldr + nw + 16 * q + 8 * g);
                res[q] = __builtin_bit_cast(half8, v);
            }
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            float x[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                // (element values first: a bit cast applied to a vector element itself reads element 0)
                const float lo = acc[i][(2 * q) * 4 + e], hi = acc[i][(2 * q + 1) * 4 + e];
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
                if constexpr (KIND == GEMM_FFN_UP) y = gelu_erf(y);
                if constexpr (!n_split) y += (float)res[q][e];
                o[e] = (_Float16)y;
            }
            *(half8 *)(tile_out + row * LDT + wave * 32 + 16 * q + 8 * g) = o;
        }
    }
    }
    __syncthreads();
    STI_STAMP(4);
    // BN/8 lanes per tile row: every store instruction writes whole rows of the tile
    _Float16 *C = (_Float16 *)p.C;
    constexpr int PIECES_PER_ROW = BN / 8;
    constexpr int PASSES = BM * PIECES_PER_ROW / NT;
    static_assert(PASSES * NT == BM * PIECES_PER_ROW, "whole passes");
    u32x4 piece[PASSES];
#pragma unroll
    for (int j = 0; j < PASSES; ++j) {
        const int pc = tid + NT * j;
        piece[j] = *(const u32x4 *)(tile_out + (pc / PIECES_PER_ROW) * LDT + (pc % PIECES_PER_ROW) * 8);
    }
#pragma unroll
    for (int j = 0; j < PASSES; ++j) {
        const int pc = tid + NT * j;
        const int m = m0 + pc / PIECES_PER_ROW, n = tile_n * BN + (pc % PIECES_PER_ROW) * 8;
        if (m < hot_T && n < N) *(u32x4 *)(C + (int64_t)m * p.ldc + n) = piece[j];
    }
    STI_STAMPS_OUT();
}

template <int KIND, int RA, int NW, int KS, bool EARLY>
hipError_t launch_variant(const GemmProblem &p, const GemmBlocks &blocks, int N, hipStream_t stream);

template <int KIND, int RA, int NW, int KS>
hipError_t launch_shape(const GemmProblem &p, const GemmBlocks &blocks, int N, hipStream_t stream)
{
    constexpr bool n_split = (KIND == GEMM_QKV || KIND == GEMM_FFN_UP || KIND == GEMM_QKV_ATTN);
    if constexpr (!n_split && RA <= 2) {
        if (p.k_splits <= 1) return launch_variant<KIND, RA, NW, KS, true>(p, blocks, N, stream);
    }
    return launch_variant<KIND, RA, NW, KS, false>(p, blocks, N, stream);
}

template <int KIND, int RA, int NW, int KS, bool EARLY>
hipError_t launch_variant(const GemmProblem &p, const GemmBlocks &blocks, int N, hipStream_t stream)
{
    constexpr int BM = RA * 32, BN = NW * 32;
    constexpr size_t lds = (KIND == GEMM_QKV_ATTN && kAttentionLdsBytes > wide_lds_bytes<RA, NW, KS>())
                               ? kAttentionLdsBytes : wide_lds_bytes<RA, NW, KS>();
    // once per instantiation, and safe when several host threads make their first call together
    static const hipError_t attr_status =
        hipFuncSetAttribute((const void *)gemm_wide_kernel<KIND, RA, NW, KS, EARLY>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (attr_status != hipSuccess) return attr_status;
    const int total = ((N + BN - 1) / BN) * ((p.T + BM - 1) / BM);
    const bool n_split = (KIND == GEMM_QKV || KIND == GEMM_FFN_UP || KIND == GEMM_QKV_ATTN);
    dim3 grid(((total + 7) / 8) * 8, (!n_split && p.k_splits > 1) ? p.k_splits : 1);
    if ((KIND == GEMM_QKV_ATTN || KIND == GEMM_QKV) && p.next_workgroups > 0) {
        static_assert((KIND != GEMM_QKV_ATTN && KIND != GEMM_QKV) || kNextDecodeLdsBytes <= lds, "the decompressing workgroups' tables fit");
        if (!p.next_table || !p.next_out || p.next_shards <= 0 || p.next_shards > kMaxShardsPerLayer ||
            p.next_ffn_per_shard <= 0 || p.next_ffn_per_shard % 64 || p.block_cols % 64 ||
            (int)grid.x + p.next_workgroups > kComputeUnits)
            return hipErrorInvalidValue;
        grid.x += p.next_workgroups;
    }
    const int64_t w_stride = p.n_blocks > 1 ? (const uint8_t *)blocks.b[1].w - (const uint8_t *)blocks.b[0].w : 0;
    launch((gemm_wide_kernel<KIND, RA, NW, KS, EARLY>), grid, dim3(NW * KS * 64), lds, stream, p.A, blocks.b[0].w,
           p.resid, p.bias0, (int32_t)w_stride, p.T, p.lda, p.ldr, (uint32_t)p.block_rows | (uint32_t)p.block_cols << 16,
           (uint32_t)p.n_blocks | (uint32_t)(p.k_splits > 1 ? p.k_splits : 1) << 16, p, blocks);
    return hipGetLastError();
}

template <int RA, int NW>
hipError_t launch_kind(const GemmProblem &p, const GemmBlocks &blocks, int N, hipStream_t stream)
{
    switch (p.kind) {
    case GEMM_QKV: return launch_shape<GEMM_QKV, RA, NW, 1>(p, blocks, N, stream);
    case GEMM_FFN_UP: return launch_shape<GEMM_FFN_UP, RA, NW, 1>(p, blocks, N, stream);
    case GEMM_OUT: return launch_shape<GEMM_OUT, RA, NW, 1>(p, blocks, N, stream);
    case GEMM_FFN_DOWN: return launch_shape<GEMM_FFN_DOWN, RA, NW, 1>(p, blocks, N, stream);
    case GEMM_QKV_ATTN: break;   // one shape only, launched by launch_gemm_wide itself
    }
    return hipErrorInvalidValue;
}

struct Shape {
    int ra, nw;
};
constexpr Shape kShapes[] = {{4, 12}, {4, 9}, {2, 12}, {2, 6}};
constexpr int kWaveSlots = 12;   // waves a compute unit holds at this kernel's register budget

}  // namespace

// Tile shape for a [T x N] output: the one whose busiest compute unit has the least MFMA
// work (workgroups are spread evenly over the units, floor(12 / NW) of them fit on one at a
// time); ties go to fewer rounds of workgroups on that unit, then to more rows per weight
// fragment, then to more waves per unit.
bool gemm_wide_supported(const GemmProblem &p, const GemmBlocks &blocks)
{
    if (p.n_blocks <= 0 || p.T <= 0) return false;
    for (int b = 0; b < p.n_blocks; ++b)
        if (blocks.b[b].bits != kTiledBits) return false;
    // the kernel addresses block b as block 0 + b * (distance of the first two)
    const int64_t stride = p.n_blocks > 1 ? (const uint8_t *)blocks.b[1].w - (const uint8_t *)blocks.b[0].w : 0;
    for (int b = 2; b < p.n_blocks; ++b)
        if ((const uint8_t *)blocks.b[b].w - (const uint8_t *)blocks.b[0].w != stride * b) return false;
    // ... and takes the stride and the block shape and count as 32- and 16-bit kernel arguments
    if (stride < 0 || stride > INT32_MAX || p.n_blocks > 0xffff || p.block_rows > 0xffff || p.block_cols > 0xffff ||
        p.k_splits > 0xffff)
        return false;
    return true;
}

namespace {

struct Choice {
    int shape;       // index into kShapes
    bool ks2;        // K split over two wave groups inside the workgroup
    long tiles;
    int nkt_total;
};

Choice choose(const GemmProblem &p, int N)
{
    const bool n_split = (p.kind == GEMM_QKV || p.kind == GEMM_FFN_UP || p.kind == GEMM_QKV_ATTN);
    int best = -1;
    long best_key[4] = {0, 0, 0, 0}, best_tiles = 0;
    for (int c = 0; c < (int)(sizeof(kShapes) / sizeof(kShapes[0])); ++c) {
        const int bm = kShapes[c].ra * 32, bn = kShapes[c].nw * 32;
        const long tiles = (long)((N + bn - 1) / bn) * ((p.T + bm - 1) / bm);
        const long per_cu = (tiles + kComputeUnits - 1) / kComputeUnits;        // workgroups on the busiest unit
        const long resident = kWaveSlots / kShapes[c].nw;
        const long key[4] = {per_cu * kShapes[c].nw * kShapes[c].ra,            // its MFMA work
                             (per_cu + resident - 1) / resident,                // rounds
                             -kShapes[c].ra,
                             -(per_cu < resident ? per_cu : resident) * kShapes[c].nw};
        bool better = best < 0;
        for (int i = 0; i < 4 && !better; ++i) {
            if (key[i] != best_key[i]) { better = key[i] < best_key[i]; break; }
        }
        if (better) {
            best = c;
            best_tiles = tiles;
            for (int i = 0; i < 4; ++i) best_key[i] = key[i];
        }
    }
    Choice ch;
    ch.shape = best;
    ch.tiles = best_tiles;
    ch.nkt_total = (n_split ? p.block_cols : p.n_blocks * p.block_cols) / BK;
    // one 6-wave workgroup per unit: split K inside the workgroup to fill the unit
    ch.ks2 = !n_split && kShapes[best].ra == 2 && kShapes[best].nw == 6 && best_key[1] == 1 &&
             best_key[0] == 12 && ch.nkt_total % 2 == 0 && ch.nkt_total >= 4;
    return ch;
}

}  // namespace

// With few tiles (few tokens) a workgroup of the d_model-wide projections would walk a long K
// range alone while most compute units idle (FFN2 at 256 tokens: 16 workgroups, 21 us): K is
// then split over 2 or 4 workgroups per tile as well, each with at least 3 K tiles per wave
// group, while they fill at most half the chip (measured: 3-6 % per layer from 256 to 1024
// tokens; 8 splits, or splitting up to the whole chip, cost more in the LayerNorm that adds
// the float32 partial sums than they save here).
int gemm_wide_k_splits(const GemmProblem &p)
{
    if (p.kind == GEMM_QKV || p.kind == GEMM_FFN_UP || p.kind == GEMM_QKV_ATTN || p.n_blocks <= 0 || p.T <= 0) return 1;
    const Choice ch = choose(p, p.block_rows);
    if (!ch.ks2) return 1;
    for (int s = 4; s >= 2; s >>= 1)
        if (ch.tiles * s <= kComputeUnits / 2 && ch.nkt_total % (2 * s) == 0 && ch.nkt_total / (2 * s) >= 3) return s;
    return 1;
}

int gemm_wide_max_k_splits(int64_t T, int N)
{
    const int64_t tiles = ((T + 63) / 64) * ((N + 191) / 192);
    for (int s = 4; s >= 2; s >>= 1)
        if (tiles * s <= kComputeUnits / 2) return s;
    return 1;
}

// The fused form pays once its 128 x 384 tiles (one per sequence and pair of heads) fill at least
// half of the compute units; below that the separate Q/K/V projection spreads over more of them.
bool gemm_wide_fuses_attention(int B, int L, int m, int dh)
{
    return L == ATT_L && dh == ATT_DH && m > 0 && (int64_t)B * ((m + 1) / 2) >= kComputeUnits / 2;
}

// Every workgroup of the launch, tiles and decompression, finds a compute unit in the first round;
// below an eighth of the chip the decompression would outlast the projection.
int gemm_wide_spare_workgroups(const GemmProblem &p)
{
    if (p.n_blocks <= 0 || p.T <= 0) return 0;
    int64_t tiles;
    if (p.kind == GEMM_QKV_ATTN) tiles = (int64_t)(p.T / ATT_L) * ((p.n_blocks + 1) / 2);
    else if (p.kind == GEMM_QKV) tiles = choose(p, p.n_blocks * p.block_rows).tiles;
    else return 0;
    const int64_t spare = kComputeUnits - (tiles + 7) / 8 * 8;
    return spare >= kComputeUnits / 8 ? (int)spare : 0;
}

hipError_t launch_gemm_wide(const GemmProblem &p, const GemmBlocks &blocks, hipStream_t stream)
{
    const bool n_split = (p.kind == GEMM_QKV || p.kind == GEMM_FFN_UP || p.kind == GEMM_QKV_ATTN);
    const int N = n_split ? p.n_blocks * p.block_rows : p.block_rows;
    if (p.T <= 0 || N <= 0) return hipSuccess;
    if (!gemm_wide_supported(p, blocks)) return hipErrorInvalidValue;
    if (N % 32 || p.block_rows % 32 || p.block_cols % BK || p.lda % 8 || p.ldc % 8) return hipErrorInvalidValue;
    if (p.kind == GEMM_QKV_ATTN) {
        if (p.T % ATT_L || p.block_rows != 3 * ATT_DH || p.d_head != ATT_DH || p.ldc < p.n_blocks * ATT_DH)
            return hipErrorInvalidValue;
        return launch_shape<GEMM_QKV_ATTN, 4, 12, 1>(p, blocks, N, stream);
    }
    const Choice ch = choose(p, N);
    if (p.k_splits > 1 && (!ch.ks2 || p.k_splits != gemm_wide_k_splits(p))) return hipErrorInvalidValue;
    if (ch.ks2) {
        return p.kind == GEMM_OUT ? launch_shape<GEMM_OUT, 2, 6, 2>(p, blocks, N, stream)
                                  : launch_shape<GEMM_FFN_DOWN, 2, 6, 2>(p, blocks, N, stream);
    }
    switch (ch.shape) {
    case 0: return launch_kind<4, 12>(p, blocks, N, stream);
    case 1: return launch_kind<4, 9>(p, blocks, N, stream);
    case 2: return launch_kind<2, 12>(p, blocks, N, stream);
    default: return launch_kind<2, 6>(p, blocks, N, stream);
    }
}

}  // namespace sti
