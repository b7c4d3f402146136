// float32 kernels of the layer: the decompress-into-a-working-buffer route of
// the paper (Section "Submodel execution": shards are decompressed into a
// buffer holding one layer of FP32 weights, then the layer is computed), with
// float32 storage and arithmetic throughout.  Any dimensions are accepted.
#include "sti_internal.hpp"

namespace sti {
namespace {

constexpr int BM = 64, BN = 64, BK = 16, TM = 4, TN = 4;

__device__ inline float gelu_erf(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752440f)); }

// Address of weight (n, kk) of the block-structured operand.
__device__ inline const float *weight_ptr(const GemmBlocks &blocks, bool n_split, int block_rows,
                                          int block_cols, int n, int kk)
{
    if (n_split) {
        int p = n / block_rows, r = n - p * block_rows;
        return (const float *)blocks.b[p].w + (int64_t)r * block_cols + kk;
    }
    int p = kk / block_cols, e = kk - p * block_cols;
    return (const float *)blocks.b[p].w + (int64_t)n * block_cols + e;
}

__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmProblem p, GemmBlocks blocks)
{
    __shared__ float As[BK][BM + 4];
    __shared__ float Bs[BK][BN + 4];
    const bool n_split = (p.kind == GEMM_QKV || p.kind == GEMM_FFN_UP);
    const int N = n_split ? p.n_blocks * p.block_rows : p.block_rows;
    const int K = n_split ? p.block_cols : p.n_blocks * p.block_cols;
    // one grid dimension, column tiles fastest (the row-tile count may pass the limit of the others)
    const int n_tiles = (N + BN - 1) / BN;
    const int tile_m = blockIdx.x / n_tiles, tile_n = blockIdx.x - tile_m * n_tiles;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int tid = threadIdx.x;
    const int tx = tid % 16, ty = tid / 16;
    const float *A = (const float *)p.A;

    float acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = 0.f;

    for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
        for (int i = 0; i < (BM * BK) / 256; ++i) {
            int idx = tid + i * 256;
            int r = idx / BK, c = idx % BK;
            int m = m0 + r, kk = k0 + c;
            As[c][r] = (m < p.T && kk < K) ? A[(int64_t)m * p.lda + kk] : 0.f;
            int n = n0 + r;
            Bs[c][r] = (n < N && kk < K)
                           ? *weight_ptr(blocks, n_split, p.block_rows, p.block_cols, n, kk)
                           : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < BK; ++c) {
            float a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = As[c][ty * TM + i];
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = Bs[c][tx * TN + j];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }

    float *C = (float *)p.C;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        int m = m0 + ty * TM + i;
        if (m >= p.T) continue;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            int n = n0 + tx * TN + j;
            if (n >= N) continue;
            float v = acc[i][j];
            if (p.kind == GEMM_QKV) {
                int blk = n / p.block_rows, r = n - blk * p.block_rows;
                int which = r / p.d_head, e = r - which * p.d_head;
                const float *bias = which == 0 ? p.bias0 : (which == 1 ? p.bias1 : p.bias2);
                v += bias[blocks.b[blk].shard * p.d_head + e];
            } else if (p.kind == GEMM_FFN_UP) {
                int blk = n / p.block_rows, r = n - blk * p.block_rows;
                v = gelu_erf(v + p.bias0[blocks.b[blk].shard * p.block_rows + r]);
            } else {
                v += p.bias0[n] + ((const float *)p.resid)[(int64_t)m * p.ldr + n];
            }
            C[(int64_t)m * p.ldc + n] = v;
        }
    }
}

__device__ inline float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// One wave per query row: scores over all keys, wavefront-reduction softmax,
// then the context row.  Dynamic LDS: 4 waves x (L + dh) floats.  With key_lengths, sequence b
// attends to its first key_lengths[b] positions only (clamped to 1..L).
__global__ __launch_bounds__(256) void attention_f32_kernel(const float *qkv, float *ctx, int L,
                                                            int m, int dh, const int32_t *key_lengths)
{
    extern __shared__ float smem[];
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    float *prob = smem + (size_t)wave * (L + dh);
    float *qrow = prob + L;
    const int b = blockIdx.z, p = blockIdx.y;
    const int i = blockIdx.x * 4 + wave;
    if (i >= L) return;  // whole wave leaves; no workgroup barrier below
    int Lk = L;
    if (key_lengths) Lk = min(max(key_lengths[b], 1), L);
    const int64_t ld = (int64_t)m * 3 * dh;
    const float *base = qkv + (int64_t)b * L * ld + (int64_t)p * 3 * dh;
    const float *q = base + (int64_t)i * ld;
    for (int e = lane; e < dh; e += 64) qrow[e] = q[e];
    __builtin_amdgcn_wave_barrier();
    const float scale = 1.0f / sqrtf((float)dh);
    float mx = -INFINITY;
    for (int j = lane; j < Lk; j += 64) {
        const float *k = base + (int64_t)j * ld + dh;
        float s = 0.f;
        for (int e = 0; e < dh; ++e) s = fmaf(qrow[e], k[e], s);
        s *= scale;
        prob[j] = s;
        mx = fmaxf(mx, s);
    }
    mx = wave_max(mx);
    float den = 0.f;
    for (int j = lane; j < Lk; j += 64) {
        float e = expf(prob[j] - mx);
        prob[j] = e;
        den += e;
    }
    den = wave_sum(den);
    const float inv = 1.0f / den;
    __builtin_amdgcn_wave_barrier();
    float *out = ctx + ((int64_t)b * L + i) * ((int64_t)m * dh) + (int64_t)p * dh;
    for (int e = lane; e < dh; e += 64) {
        float acc = 0.f;
        for (int j = 0; j < Lk; ++j) acc = fmaf(prob[j], base[(int64_t)j * ld + 2 * dh + e], acc);
        out[e] = acc * inv;
    }
}

}  // namespace

hipError_t launch_gemm_f32(const GemmProblem &p, const GemmBlocks &blocks, hipStream_t stream)
{
    const bool n_split = (p.kind == GEMM_QKV || p.kind == GEMM_FFN_UP);
    const int N = n_split ? p.n_blocks * p.block_rows : p.block_rows;
    if (p.T <= 0 || N <= 0) return hipSuccess;
    const int64_t tiles = (int64_t)((N + BN - 1) / BN) * ((p.T + BM - 1) / BM);
    if (tiles > 0x7FFFFFFF) return hipErrorInvalidValue;
    launch(gemm_f32_kernel, dim3((uint32_t)tiles), dim3(256), 0, stream, p, blocks);
    return hipGetLastError();
}

hipError_t launch_attention_f32(const float *qkv, float *ctx, int B, int L, int m, int dh,
                                const int32_t *key_lengths, hipStream_t stream)
{
    if (B <= 0 || L <= 0 || m <= 0) return hipSuccess;
    dim3 grid((L + 3) / 4, m, B);
    size_t lds = (size_t)4 * (L + dh) * sizeof(float);
    launch(attention_f32_kernel, grid, dim3(256), lds, stream, qkv, ctx, L, m, dh, key_lengths);
    return hipGetLastError();
}

}  // namespace sti
