// Per-head attention on the matrix cores: C = softmax(Q K^T / sqrt(dh)) V for
// one (sequence, present head) per workgroup column (Section "A primer on
// transformer": each head contributes its own attention score).
//
// Everything is computed transposed so that the softmax never crosses lanes:
//   S^T = K Q^T   -> a lane owns one query (MFMA column) and 16 keys per
//                    32-key block in its accumulator registers;
//   O^T = V^T P^T -> the probabilities are already in the register layout the
//                    B operand needs once the key order inside each k16 step
//                    is permuted, and V^T is read from LDS in that same order.
// The maximum and the sum of a query's row are per lane; lanes l and l^32 own the two
// halves of a query's keys and exchange their maxima (once per key block with the running
// maximum of the online softmax, once in all when the sequence is short, see SHORT).
//
// Padded sequences (the input length is fixed after padding, Section "Prerequisite: Offline
// Profiling"): with key_lengths, sequence b attends to its first key_lengths[b] positions only
// (clamped to 1..L); rows of padded positions are still computed, from those keys.
#include "sti_internal.hpp"
#include "attention_core.hpp"

namespace sti {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int DH = 64;
constexpr int KPAD = DH + 8;   // padded K row (halves)

__device__ inline int vt_stride(int Lp) { return Lp + 8; }

// NW waves per workgroup, 32 queries each.
// SHORT > 0 (at most 32 * SHORT keys; 4 or 8): all scores stay in registers, the row maximum is
// known before the first exponential, and the output accumulators are never rescaled.
template <int NW, int SHORT>
__global__ __launch_bounds__(NW * 64, 2) void attention_mfma_kernel(const _Float16 *qkv, _Float16 *ctx,
                                                                 int L, int Lp, int m,
                                                                 const int32_t *key_lengths)
{
    constexpr int QB = NW * 32;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    _Float16 *Ks = (_Float16 *)smem_raw;                 // [Lp][KPAD]
    _Float16 *Vt = Ks + (size_t)Lp * KPAD;               // [DH][Lp + 8]
    const int vts = vt_stride(Lp);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int g = lane >> 5, lr = lane & 31;
    const int b = blockIdx.z, p = blockIdx.y;
    const int64_t ld = (int64_t)m * 3 * DH;
    const _Float16 *base = qkv + (int64_t)b * L * ld + (int64_t)p * 3 * DH;
    int Lk = L;   // keys that take part
    if (key_lengths) Lk = min(max(key_lengths[b], 1), L);

    // this lane's query row as the B operand of S^T = K Q^T (asked for first: the loads below
    // and these share one round trip to memory)
    const int q = blockIdx.x * QB + wave * 32 + lr;
    half8 qf[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        u32x4 v = {0, 0, 0, 0};
        if (q < L) v = *(const u32x4 *)(base + (int64_t)q * ld + s * 16 + g * 8);
        qf[s] = __builtin_bit_cast(half8, v);
    }

    // Stage K (row-major; rows >= Lk are zero) and V transposed, 128 keys per pass: all loads
    // of a pass are issued before the first LDS store, so a pass costs one round trip.
    //   K: a thread takes 16 bytes of rows tid/8 + 8 NW j;
    //   V: a lane takes two consecutive keys and 8 features, so that the 64 lanes of one LDS
    //      store write consecutive dwords of one V^T row (no bank conflicts).
    constexpr int KJ = 16 / NW;           // K rows per thread and pass
    constexpr int VJ = 8 / NW;            // V key pairs per thread and pass
    const int kc = (tid & 7) * 8;
    const int v_items = (Lp / 2) * 8;
    for (int r0p = 0; r0p < Lp; r0p += 128) {
        u32x4 kreg[KJ], v0[VJ], v1[VJ];
#pragma unroll
        for (int j = 0; j < KJ; ++j) {
            const int r = r0p + (tid >> 3) + NW * 8 * j;
            kreg[j] = u32x4{0, 0, 0, 0};
            if (r < Lk) kreg[j] = *(const u32x4 *)(base + (int64_t)r * ld + DH + kc);
        }
#pragma unroll
        for (int j = 0; j < VJ; ++j) {
            const int item = (r0p / 128) * (NW * 64 * VJ) + tid + NW * 64 * j;
            const int pair = item % (Lp / 2), c = (item / (Lp / 2)) * 8;
            const int r0 = 2 * pair;
            v0[j] = u32x4{0, 0, 0, 0};
            v1[j] = u32x4{0, 0, 0, 0};
            if (item < v_items && r0 < Lk) v0[j] = *(const u32x4 *)(base + (int64_t)r0 * ld + 2 * DH + c);
            if (item < v_items && r0 + 1 < Lk) v1[j] = *(const u32x4 *)(base + (int64_t)(r0 + 1) * ld + 2 * DH + c);
        }
#pragma unroll
        for (int j = 0; j < KJ; ++j) {
            const int r = r0p + (tid >> 3) + NW * 8 * j;
            if (r < Lp) *(u32x4 *)(Ks + (size_t)r * KPAD + kc) = kreg[j];
        }
#pragma unroll
        for (int j = 0; j < VJ; ++j) {
            const int item = (r0p / 128) * (NW * 64 * VJ) + tid + NW * 64 * j;
            if (item >= v_items) continue;
            const int pair = item % (Lp / 2), c = (item / (Lp / 2)) * 8;
            const int r0 = 2 * pair;
            const uint32_t a[4] = {v0[j].x, v0[j].y, v0[j].z, v0[j].w}, bq[4] = {v1[j].x, v1[j].y, v1[j].z, v1[j].w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t lo = (a[i] & 0xFFFFu) | (bq[i] << 16);          // feature c + 2i
                const uint32_t hi = (a[i] >> 16) | (bq[i] & 0xFFFF0000u);      // feature c + 2i + 1
                *(uint32_t *)(Vt + (size_t)(c + 2 * i) * vts + r0) = lo;
                *(uint32_t *)(Vt + (size_t)(c + 2 * i + 1) * vts + r0) = hi;
            }
        }
    }
    __syncthreads();

    const float scale = 0.125f * 1.44269504088896340736f;   // 1/sqrt(64) * log2(e)
    float run_max = -INFINITY, run_sum = 0.f;
    float16v o[2];
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[e][v] = 0.f;

    const int nkb = (Lk + 31) / 32;   // key blocks beyond the last real key are skipped
    // O^T += V^T P^T over the two k16 steps of key block kb; pk = the block's probabilities
    auto add_pv = [&](int kb, const uint32_t (&pk)[8]) {
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            u32x4 pv = {pk[4 * s2], pk[4 * s2 + 1], pk[4 * s2 + 2], pk[4 * s2 + 3]};
            half8 pf = __builtin_bit_cast(half8, pv);
            const int key0 = kb * 32 + (2 * s2) * 8 + g * 4;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const _Float16 *vrow = Vt + (size_t)(e * 32 + lr) * vts + key0;
                u32x2 lo = *(const u32x2 *)vrow;
                u32x2 hi = *(const u32x2 *)(vrow + 8);
                u32x4 vv = {lo.x, lo.y, hi.x, hi.y};
                o[e] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, vv), pf,
                                                              o[e], 0, 0, 0);
            }
        }
    };
    if constexpr (SHORT > 0) {
        run_sum = attention_scores_in_registers<SHORT>(qf, Ks, KPAD, Vt, vts, Lk, lane, o);
    } else
    for (int kb = 0; kb < nkb; ++kb) {
        float16v s_acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) s_acc[v] = 0.f;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            half8 kf = *(const half8 *)(Ks + (size_t)(kb * 32 + lr) * KPAD + s * 16 + g * 8);
            s_acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qf[s], s_acc, 0, 0, 0);
        }
        // scores of keys kb*32 + (v/4)*8 + g*4 + v%4 for this lane's query
        float bmax = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int key = kb * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
            float x = s_acc[v] * scale;
            x = (key < Lk) ? x : -INFINITY;
            s_acc[v] = x;
            bmax = fmaxf(bmax, x);
        }
        bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
        const float new_max = fmaxf(run_max, bmax);
        const float alpha = __builtin_amdgcn_exp2f(run_max - new_max);
        run_max = new_max;
        float psum = 0.f;
        uint32_t pk[8];
#pragma unroll
        for (int v = 0; v < 16; v += 2) {
            float p0 = __builtin_amdgcn_exp2f(s_acc[v] - new_max);
            float p1 = __builtin_amdgcn_exp2f(s_acc[v + 1] - new_max);
            psum += p0 + p1;
            pk[v / 2] = (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)p0) |
                        ((uint32_t)__builtin_bit_cast(uint16_t, (_Float16)p1) << 16);
        }
        run_sum = run_sum * alpha + psum;
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[e][v] *= alpha;
        add_pv(kb, pk);
    }
    if constexpr (SHORT == 0) run_sum += __shfl_xor(run_sum, 32, 64);   // (the register-resident variant returns the pair's sum)
    if (q >= L) return;
    const float inv = 1.0f / run_sum;
    _Float16 *out = ctx + ((int64_t)b * L + q) * ((int64_t)m * DH) + (int64_t)p * DH;
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
            half4 h;
#pragma unroll
            for (int i = 0; i < 4; ++i) h[i] = (_Float16)(o[e][v4 * 4 + i] * inv);
            *(half4 *)(out + e * 32 + v4 * 8 + g * 4) = h;
        }
}

}  // namespace

hipError_t launch_attention_mfma(const void *qkv, void *ctx, int B, int L, int m, int dh,
                                 const int32_t *key_lengths, hipStream_t stream)
{
    if (B <= 0 || L <= 0 || m <= 0) return hipSuccess;
    if (dh != DH) return hipErrorInvalidValue;
    const int Lp = (L + 31) / 32 * 32;
    const size_t lds = ((size_t)Lp * KPAD + (size_t)DH * (Lp + 8)) * sizeof(_Float16);
    // once per process, and safe when several host threads make their first call together
    static const hipError_t attr_status = [] {
        hipError_t e = hipFuncSetAttribute((const void *)attention_mfma_kernel<4, 0>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)attention_mfma_kernel<2, 0>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        return e;
    }();
    if (attr_status != hipSuccess) return attr_status;
    // few (sequence, head) pairs: 64 queries per workgroup put twice as many workgroups on the chip
    const bool small_wg = (int64_t)B * m * ((L + 127) / 128) < 128 && L > 32;
    if (small_wg) {
        dim3 grid((L + 63) / 64, m, B);
        if (Lp <= 128)
            launch((attention_mfma_kernel<2, 4>), grid, dim3(128), lds, stream, (const _Float16 *)qkv,
                                                                          (_Float16 *)ctx, L, Lp, m, key_lengths);
        else if (Lp <= 256)
            launch((attention_mfma_kernel<2, 8>), grid, dim3(128), lds, stream, (const _Float16 *)qkv,
                                                                          (_Float16 *)ctx, L, Lp, m, key_lengths);
        else
            launch((attention_mfma_kernel<2, 0>), grid, dim3(128), lds, stream, (const _Float16 *)qkv,
                                                                          (_Float16 *)ctx, L, Lp, m, key_lengths);
    } else {
        dim3 grid((L + 127) / 128, m, B);
        if (Lp <= 128)
            launch((attention_mfma_kernel<4, 4>), grid, dim3(256), lds, stream, (const _Float16 *)qkv,
                                                                          (_Float16 *)ctx, L, Lp, m, key_lengths);
        else if (Lp <= 256)
            launch((attention_mfma_kernel<4, 8>), grid, dim3(256), lds, stream, (const _Float16 *)qkv,
                                                                          (_Float16 *)ctx, L, Lp, m, key_lengths);
        else
            launch((attention_mfma_kernel<4, 0>), grid, dim3(256), lds, stream, (const _Float16 *)qkv,
                                                                          (_Float16 *)ctx, L, Lp, m, key_lengths);
    }
    return hipGetLastError();
}

}  // namespace sti
