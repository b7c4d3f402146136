// Attention of 32 queries (one per lane pair l, l ^ 32) over at most 32 * NKB keys that sit in LDS,
// with every score kept in registers (Section "A primer on transformer": per-head attention
// scores).  Shared by the attention kernel and by the Q/K/V projection that runs the attention
// of the heads it has just produced.
//
// Everything is computed transposed so that the softmax never crosses lanes:
//   S^T = K Q^T   -> a lane owns one query (MFMA column) and 16 keys per 32-key block in its
//                    accumulator registers;
//   O^T = V^T P^T -> the probabilities are already in the register layout the B operand needs
//                    once the key order inside each k16 step is permuted, and V^T is read from
//                    LDS in that same order.
// The row maximum is known before the first exponential (lanes l and l ^ 32 exchange their
// maxima once), so the output accumulators are never rescaled.
#pragma once
#include "sti_internal.hpp"

namespace sti {

typedef _Float16 att_half8 __attribute__((ext_vector_type(8)));
typedef float att_float16v __attribute__((ext_vector_type(16)));
typedef uint32_t att_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t att_u32x2 __attribute__((ext_vector_type(2)));

// qf[s]  : this lane's query as the B operand of S^T = K Q^T (features s*16 + g*8 .. +8)
// Ks     : keys, row-major, `kpad` halves per row (rows >= Lk are never weighted)
// Vt     : values transposed, `vts` halves per feature row
// Lk     : keys that take part (1 .. 32 * NKB); key blocks behind the last one are skipped
// out    : o[e][v] = unnormalised context of feature e*32 + (v/4)*8 + g*4 + v%4; returns the row sum
//          of the lane pair (the caller divides)
template <int NKB>
__device__ inline float attention_scores_in_registers(const att_half8 (&qf)[4], const _Float16 *Ks, int kpad,
                                                      const _Float16 *Vt, int vts, int Lk, int lane,
                                                      att_float16v (&o)[2])
{
    const int g = lane >> 5, lr = lane & 31;
    const float scale = 0.125f * 1.44269504088896340736f;   // 1/sqrt(64) * log2(e)
    const int nkb = (Lk + 31) / 32;
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[e][v] = 0.f;
    att_float16v sc[NKB];
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
        if (kb >= nkb) break;
#pragma unroll
        for (int v = 0; v < 16; ++v) sc[kb][v] = 0.f;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const att_half8 kf = *(const att_half8 *)(Ks + (size_t)(kb * 32 + lr) * kpad + s * 16 + g * 8);
            sc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qf[s], sc[kb], 0, 0, 0);
        }
        if (kb * 32 + 32 > Lk) {   // keys past Lk sit in the last block only
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int key = kb * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
                sc[kb][v] = (key < Lk) ? sc[kb][v] : -INFINITY;
            }
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sc[kb][v]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float shift = -mx * scale;   // (scale > 0: the maximum of the scaled scores)
    float run_sum = 0.f;
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
        if (kb >= nkb) break;
        uint32_t pk[8];
#pragma unroll
        for (int v = 0; v < 16; v += 2) {
            const float p0 = __builtin_amdgcn_exp2f(fmaf(sc[kb][v], scale, shift));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(sc[kb][v + 1], scale, shift));
            run_sum += p0 + p1;
            pk[v / 2] = (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)p0) |
                        ((uint32_t)__builtin_bit_cast(uint16_t, (_Float16)p1) << 16);
        }
        // O^T += V^T P^T over the two k16 steps of key block kb
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            const att_u32x4 pv = {pk[4 * s2], pk[4 * s2 + 1], pk[4 * s2 + 2], pk[4 * s2 + 3]};
            const att_half8 pf = __builtin_bit_cast(att_half8, pv);
            const int key0 = kb * 32 + (2 * s2) * 8 + g * 4;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const _Float16 *vrow = Vt + (size_t)(e * 32 + lr) * vts + key0;
                const att_u32x2 lo = *(const att_u32x2 *)vrow;
                const att_u32x2 hi = *(const att_u32x2 *)(vrow + 8);
                const att_u32x4 vv = {lo.x, lo.y, hi.x, hi.y};
                o[e] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(att_half8, vv), pf, o[e], 0, 0, 0);
            }
        }
    }
    run_sum += __shfl_xor(run_sum, 32, 64);
    return run_sum;
}

}  // namespace sti
