// Row-wise and elementwise helpers of the layer: LayerNorm over d features
// (biased variance, Section "A primer on transformer" runs stock BERT layers)
// and activation type conversion.
#include <type_traits>
#include "sti_internal.hpp"

namespace sti {
namespace {

__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ inline uint16_t f32_to_bf16_bits(float v)
{
    uint32_t u = __builtin_bit_cast(uint32_t, v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}
__device__ inline float bf16_bits_to_f32(uint16_t b)
{
    return __builtin_bit_cast(float, (uint32_t)b << 16);
}

template <int DT> struct Elem;
template <> struct Elem<STI_F32> {
    typedef float type;
    static __device__ inline float load(const float *p) { return *p; }
    static __device__ inline void store(float *p, float v) { *p = v; }
};
template <> struct Elem<STI_F16> {
    typedef _Float16 type;
    static __device__ inline float load(const _Float16 *p) { return (float)*p; }
    static __device__ inline void store(_Float16 *p, float v) { *p = (_Float16)v; }
};
template <> struct Elem<STI_BF16> {
    typedef uint16_t type;
    static __device__ inline float load(const uint16_t *p) { return bf16_bits_to_f32(*p); }
    static __device__ inline void store(uint16_t *p, float v) { *p = f32_to_bf16_bits(v); }
};

// v[t][:] = pre[t][:] (+ bias[:]) (+ resid[t][:]);  y[t][:] = LayerNorm(v) * g + b.
// One wave per row; two-pass mean / variance in float32.  General sizes.
template <int DT>
__global__ __launch_bounds__(256) void layernorm_kernel(const float *pre, int n_partials,
                                                        int64_t partial_stride, const float *bias,
                                                        const _Float16 *resid,
                                                        typename Elem<DT>::type *y, const float *g,
                                                        const float *b, int T, int d, float eps)
{
    const int row = blockIdx.x * 4 + threadIdx.x / 64;
    const int lane = threadIdx.x % 64;
    if (row >= T) return;
    const float *r = pre + (int64_t)row * d;
    const _Float16 *rs = resid ? resid + (int64_t)row * d : nullptr;
    auto value = [&](int c) {
        float v = n_partials > 0 ? r[c] : 0.f;
        for (int s = 1; s < n_partials; ++s) v += r[(int64_t)s * partial_stride + c];
        if (bias) v += bias[c];
        if (rs) v += (float)rs[c];
        return v;
    };
    float s = 0.f;
    for (int c = lane; c < d; c += 64) s += value(c);
    const float mean = wave_sum(s) / (float)d;
    float q = 0.f;
    for (int c = lane; c < d; c += 64) {
        float t = value(c) - mean;
        q = fmaf(t, t, q);
    }
    const float var = wave_sum(q) / (float)d;
    const float inv = 1.0f / sqrtf(var + eps);
    typename Elem<DT>::type *o = y + (int64_t)row * d;
    for (int c = lane; c < d; c += 64) Elem<DT>::store(o + c, (value(c) - mean) * inv * g[c] + b[c]);
}

// Same, for d a multiple of 4 and at most 2048: the row is read once with 16-byte loads
// and kept in registers.
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));

// LPR lanes share one row (64, 32 or 16): fewer lanes per row keep more bytes in flight per
// lane and shorten the two reductions.
template <int LPR>
__device__ inline float row_sum(float v)
{
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

template <int DT, int LPR, int MAXC>   // MAXC = 16-byte chunks per lane: d <= 4 * LPR * MAXC
__global__ __launch_bounds__(256) void layernorm_vec_kernel(const float *pre, int n_partials,
                                                            int64_t partial_stride,
                                                            const float *bias, const _Float16 *resid,
                                                            typename Elem<DT>::type *y,
                                                            const float *g, const float *b, int T,
                                                            int d, float eps)
{
    constexpr int ROWS = 256 / LPR;               // rows per workgroup
    const int sub = threadIdx.x % LPR;
    const int row = blockIdx.x * ROWS + threadIdx.x / LPR;
    if (row >= T) return;   // whole row groups leave together; shuffles stay inside a group
    const int nchunk = d >> 2;
    // Every load of this row is independent of the others: they are issued in groups (bias and
    // residual first, then the partial sums two planes at a time) and only then added, in the
    // fixed order plane 0, 1, ..., bias, residual.  (Written as load-then-use per chunk, each of
    // up to 8 planes x 8 chunks cost a round trip to memory of its own.)  Lanes past the end of
    // the row load its last chunk and drop the value.
    const int last = nchunk - 1;
    int cj[MAXC];
#pragma unroll
    for (int j = 0; j < MAXC; ++j) cj[j] = min(sub + LPR * j, last);
    f32x4 bs[MAXC];
    half4 rs4[MAXC];
#pragma unroll
    for (int j = 0; j < MAXC; ++j) {
        bs[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        rs4[j] = half4{(_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f};
        if (bias) bs[j] = ((const f32x4 *)bias)[cj[j]];
        if (resid) rs4[j] = ((const half4 *)(resid + (int64_t)row * d))[cj[j]];
    }
    f32x4 gg[MAXC], bb[MAXC];
#pragma unroll
    for (int j = 0; j < MAXC; ++j) {
        gg[j] = ((const f32x4 *)g)[cj[j]];
        bb[j] = ((const f32x4 *)b)[cj[j]];
    }
    f32x4 v[MAXC];
#pragma unroll
    for (int j = 0; j < MAXC; ++j) v[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    const float *rp = pre + (int64_t)row * d;
    for (int sp = 0; sp < n_partials; sp += 2) {
        const bool two = sp + 1 < n_partials;   // uniform
        f32x4 t0[MAXC], t1[MAXC];
#pragma unroll
        for (int j = 0; j < MAXC; ++j) {
            t0[j] = *(const f32x4 *)(rp + (int64_t)sp * partial_stride + 4 * cj[j]);
            t1[j] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (two) t1[j] = *(const f32x4 *)(rp + (int64_t)(sp + 1) * partial_stride + 4 * cj[j]);
        }
#pragma unroll
        for (int j = 0; j < MAXC; ++j) {
            v[j] = sp == 0 ? t0[j] : v[j] + t0[j];
            if (two) v[j] += t1[j];
        }
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < MAXC; ++j) {
        f32x4 x = v[j];
        if (bias) x += bs[j];
        if (resid) x += f32x4{(float)rs4[j].x, (float)rs4[j].y, (float)rs4[j].z, (float)rs4[j].w};
        if (sub + LPR * j >= nchunk) x = f32x4{0.f, 0.f, 0.f, 0.f};
        v[j] = x;
        s += (x.x + x.y) + (x.z + x.w);
    }
    const float mean = row_sum<LPR>(s) / (float)d;
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < MAXC; ++j) {
        if (sub + LPR * j < nchunk) {
            f32x4 t = v[j] - mean;
            q += (t.x * t.x + t.y * t.y) + (t.z * t.z + t.w * t.w);
        }
    }
    const float var = row_sum<LPR>(q) / (float)d;
    const float inv = 1.0f / sqrtf(var + eps);
    typename Elem<DT>::type *o = y + (int64_t)row * d;
#pragma unroll
    for (int j = 0; j < MAXC; ++j) {
        const int c = sub + LPR * j;
        if (c < nchunk) {
            const f32x4 t = (v[j] - mean) * inv * gg[j] + bb[j];
            if constexpr (DT == STI_F32) {
                ((f32x4 *)o)[c] = t;
            } else if constexpr (DT == STI_F16) {
                ((half4 *)o)[c] = half4{(_Float16)t.x, (_Float16)t.y, (_Float16)t.z, (_Float16)t.w};
            } else {
                Elem<DT>::store(o + 4 * c, t.x); Elem<DT>::store(o + 4 * c + 1, t.y);
                Elem<DT>::store(o + 4 * c + 2, t.z); Elem<DT>::store(o + 4 * c + 3, t.w);
            }
        }
    }
}

// LayerNorm of rows that already hold sum + bias + residual in binary16 (written by the
// matrix-core GEMM); d a multiple of 8 and at most 8 * LPR * MAXC; LPR lanes per row.  All
// loads (the row, gains, shifts) are issued before the first use: one round trip to memory.
// Lanes past the end of the row load its last chunk and drop the value.
template <int DT, int LPR, int MAXC>
__global__ __launch_bounds__(256) void layernorm_f16in_kernel(const _Float16 *pre,
                                                              typename Elem<DT>::type *y,
                                                              const float *g, const float *b, int T,
                                                              int d, float eps)
{
    typedef _Float16 half8 __attribute__((ext_vector_type(8)));
    constexpr int ROWS = 256 / LPR;
    const int sub = threadIdx.x % LPR;
    const int row = blockIdx.x * ROWS + threadIdx.x / LPR;
    if (row >= T) return;   // whole row groups leave together; shuffles stay inside a group
    const int nchunk = d >> 3, last = nchunk - 1;
    const half8 *r = (const half8 *)(pre + (int64_t)row * d);
    half8 h[MAXC];
    f32x4 g0[MAXC], g1[MAXC], b0[MAXC], b1[MAXC];
#pragma unroll
    for (int j = 0; j < MAXC; ++j) h[j] = r[min(sub + LPR * j, last)];
#pragma unroll
    for (int j = 0; j < MAXC; ++j) {
        const int c = min(sub + LPR * j, last);
        g0[j] = ((const f32x4 *)g)[2 * c]; g1[j] = ((const f32x4 *)g)[2 * c + 1];
        b0[j] = ((const f32x4 *)b)[2 * c]; b1[j] = ((const f32x4 *)b)[2 * c + 1];
    }
    float v[MAXC][8];
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < MAXC; ++j) {
        const bool in = sub + LPR * j < nchunk;
#pragma unroll
        for (int e = 0; e < 8; ++e) { v[j][e] = in ? (float)h[j][e] : 0.f; s += v[j][e]; }
    }
    const float mean = row_sum<LPR>(s) / (float)d;
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < MAXC; ++j)
        if (sub + LPR * j < nchunk) {
#pragma unroll
            for (int e = 0; e < 8; ++e) { const float t = v[j][e] - mean; q = fmaf(t, t, q); }
        }
    const float var = row_sum<LPR>(q) / (float)d;
    const float inv = 1.0f / sqrtf(var + eps);
    typename Elem<DT>::type *o = y + (int64_t)row * d;
#pragma unroll
    for (int j = 0; j < MAXC; ++j) {
        const int c = sub + LPR * j;
        if (c < nchunk) {
            const float gg[8] = {g0[j].x, g0[j].y, g0[j].z, g0[j].w, g1[j].x, g1[j].y, g1[j].z, g1[j].w};
            const float bb[8] = {b0[j].x, b0[j].y, b0[j].z, b0[j].w, b1[j].x, b1[j].y, b1[j].z, b1[j].w};
            float t[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) t[e] = (v[j][e] - mean) * inv * gg[e] + bb[e];
            if constexpr (DT == STI_F16) {
                half8 o8;
#pragma unroll
                for (int e = 0; e < 8; ++e) o8[e] = (_Float16)t[e];
                ((half8 *)o)[c] = o8;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) Elem<DT>::store(o + 8 * c + e, t[e]);
            }
        }
    }
}

// Same for rows of any length (d a multiple of 8): the row is read three times (mean, variance,
// output) instead of being kept in registers.
template <int DT>
__global__ __launch_bounds__(256) void layernorm_f16in_long_kernel(const _Float16 *pre,
                                                                   typename Elem<DT>::type *y,
                                                                   const float *g, const float *b, int T,
                                                                   int d, float eps)
{
    typedef _Float16 half8 __attribute__((ext_vector_type(8)));
    const int lane = threadIdx.x % 64;
    const int row = blockIdx.x * 4 + threadIdx.x / 64;
    if (row >= T) return;
    const int nchunk = d >> 3;
    const half8 *r = (const half8 *)(pre + (int64_t)row * d);
    float s = 0.f;
    for (int c = lane; c < nchunk; c += 64) {
        const half8 h = r[c];
#pragma unroll
        for (int e = 0; e < 8; ++e) s += (float)h[e];
    }
    const float mean = wave_sum(s) / (float)d;
    float q = 0.f;
    for (int c = lane; c < nchunk; c += 64) {
        const half8 h = r[c];
#pragma unroll
        for (int e = 0; e < 8; ++e) { const float t = (float)h[e] - mean; q = fmaf(t, t, q); }
    }
    const float inv = 1.0f / sqrtf(wave_sum(q) / (float)d + eps);
    typename Elem<DT>::type *o = y + (int64_t)row * d;
    for (int c = lane; c < nchunk; c += 64) {
        const half8 h = r[c];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            Elem<DT>::store(o + 8 * c + e, ((float)h[e] - mean) * inv * g[8 * c + e] + b[8 * c + e]);
    }
}

template <int SRC, int DST>
__global__ __launch_bounds__(256) void convert_kernel(const typename Elem<SRC>::type *src,
                                                      typename Elem<DST>::type *dst, uint64_t n)
{
    uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * 256;
    for (; i < n; i += stride) Elem<DST>::store(dst + i, Elem<SRC>::load(src + i));
}

template <int SRC>
hipError_t convert_from(const void *src, void *dst, sti_dtype dst_dtype, uint64_t n, dim3 grid,
                        hipStream_t stream)
{
    typedef typename Elem<SRC>::type S;
    switch (dst_dtype) {
        case STI_F32:
            launch((convert_kernel<SRC, STI_F32>), grid, dim3(256), 0, stream, (const S *)src, (float *)dst, n);
            break;
        case STI_F16:
            launch((convert_kernel<SRC, STI_F16>), grid, dim3(256), 0, stream, (const S *)src, (_Float16 *)dst, n);
            break;
        case STI_BF16:
            launch((convert_kernel<SRC, STI_BF16>), grid, dim3(256), 0, stream, (const S *)src, (uint16_t *)dst, n);
            break;
    }
    return hipGetLastError();
}

}  // namespace

template <int DT>
void launch_ln_typed(const float *pre, int n_partials, int64_t partial_stride, const float *bias,
                     const void *resid, void *y, const float *g, const float *b, int T, int d, float eps,
                     bool vec, hipStream_t stream)
{
    typedef typename Elem<DT>::type O;
    dim3 grid((T + 3) / 4);
#define STI_LN_VEC(LPR, MAXC, GRID) \
    launch((layernorm_vec_kernel<DT, LPR, MAXC>), GRID, dim3(256), 0, stream, pre, n_partials, partial_stride, bias, \
           (const _Float16 *)resid, (O *)y, g, b, T, d, eps)
    // many rows: 32 lanes per row (8 rows per workgroup); few rows: a whole wave per row; chunks
    // per lane sized to the row, so that the registers hold no more loads in flight than it has
    if (vec && T >= 2048 && d <= 1024) {
        if (d <= 768) STI_LN_VEC(32, 6, dim3((T + 7) / 8));
        else STI_LN_VEC(32, 8, dim3((T + 7) / 8));
    } else if (vec) {
        if (d <= 768) STI_LN_VEC(64, 3, grid);
        else if (d <= 1024) STI_LN_VEC(64, 4, grid);
        else STI_LN_VEC(64, 8, grid);
    } else {
        launch((layernorm_kernel<DT>), grid, dim3(256), 0, stream, pre, n_partials, partial_stride, bias, (const _Float16 *)resid, (O *)y, g, b, T, d, eps);
    }
#undef STI_LN_VEC
}

hipError_t launch_layernorm(const float *pre, int n_partials, int64_t partial_stride,
                            const float *bias, const void *resid_f16, void *y, sti_dtype out_dtype,
                            const float *g, const float *b, int T, int d, float eps,
                            hipStream_t stream)
{
    if (T <= 0 || d <= 0) return hipSuccess;
    if (n_partials < 0 || (n_partials > 0 && !pre)) return hipErrorInvalidValue;
    auto al16 = [](const void *p) { return ((uintptr_t)p & 15) == 0; };
    const bool vec = d % 4 == 0 && d <= 2048 && partial_stride % 4 == 0 && al16(pre) && al16(g) && al16(b) && al16(y) &&
                     (!bias || al16(bias)) && (!resid_f16 || al16(resid_f16));
    switch (out_dtype) {
        case STI_F32: launch_ln_typed<STI_F32>(pre, n_partials, partial_stride, bias, resid_f16, y, g, b, T, d, eps, vec, stream); break;
        case STI_F16: launch_ln_typed<STI_F16>(pre, n_partials, partial_stride, bias, resid_f16, y, g, b, T, d, eps, vec, stream); break;
        case STI_BF16: launch_ln_typed<STI_BF16>(pre, n_partials, partial_stride, bias, resid_f16, y, g, b, T, d, eps, vec, stream); break;
    }
    return hipGetLastError();
}

hipError_t launch_layernorm_f16in(const void *pre_f16, void *y, sti_dtype out_dtype, const float *g,
                                  const float *b, int T, int d, float eps, hipStream_t stream)
{
    if (T <= 0 || d <= 0) return hipSuccess;
    if (d % 8) return hipErrorInvalidValue;
    dim3 grid((T + 3) / 4);
    const _Float16 *p = (const _Float16 *)pre_f16;
    if (d > 2048) {
        switch (out_dtype) {
            case STI_F32: launch((layernorm_f16in_long_kernel<STI_F32>), grid, dim3(256), 0, stream, p, (float *)y, g, b, T, d, eps); break;
            case STI_F16: launch((layernorm_f16in_long_kernel<STI_F16>), grid, dim3(256), 0, stream, p, (_Float16 *)y, g, b, T, d, eps); break;
            case STI_BF16: launch((layernorm_f16in_long_kernel<STI_BF16>), grid, dim3(256), 0, stream, p, (uint16_t *)y, g, b, T, d, eps); break;
        }
        return hipGetLastError();
    }
    // 32 lanes per row while the row fits 3 or 4 chunks of 8 per lane (every lane busy at d_model 768
    // and 1024), a whole wave per row beyond
    auto go = [&](auto dt) {
        constexpr int DT = decltype(dt)::value;
        typedef typename Elem<DT>::type O;
        if (d <= 768)
            launch((layernorm_f16in_kernel<DT, 32, 3>), dim3((T + 7) / 8), dim3(256), 0, stream, p, (O *)y, g, b, T, d, eps);
        else if (d <= 1024)
            launch((layernorm_f16in_kernel<DT, 32, 4>), dim3((T + 7) / 8), dim3(256), 0, stream, p, (O *)y, g, b, T, d, eps);
        else
            launch((layernorm_f16in_kernel<DT, 64, 4>), dim3((T + 3) / 4), dim3(256), 0, stream, p, (O *)y, g, b, T, d, eps);
    };
    switch (out_dtype) {
        case STI_F32: go(std::integral_constant<int, STI_F32>{}); break;
        case STI_F16: go(std::integral_constant<int, STI_F16>{}); break;
        case STI_BF16: go(std::integral_constant<int, STI_BF16>{}); break;
    }
    return hipGetLastError();
}

hipError_t launch_convert(const void *src, sti_dtype src_dtype, void *dst, sti_dtype dst_dtype,
                          uint64_t n, hipStream_t stream)
{
    if (n == 0) return hipSuccess;
    uint64_t blocks = (n + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    dim3 grid((uint32_t)blocks);
    switch (src_dtype) {
        case STI_F32: return convert_from<STI_F32>(src, dst, dst_dtype, n, grid, stream);
        case STI_F16: return convert_from<STI_F16>(src, dst, dst_dtype, n, grid, stream);
        case STI_BF16: return convert_from<STI_BF16>(src, dst, dst_dtype, n, grid, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace sti
