// Ceiling probes (libsti_probes.so): what this chip delivers for the two resources the hot path is
// bound by, measured with the simplest kernels that use nothing else.  Not part of libsti.so; bench.py
// --ceilings runs them next to the kernels they put into perspective.
//
//   sti_probe_mfma    a loop of v_mfma_f32_32x32x16_f16 on register operands only (no memory, no LDS,
//                     no barriers): the matrix-core rate at the clock the chip holds under that load.
//                     `varied` = 0: the same two operand registers in every MFMA; 1: four pseudo-random
//                     operand pairs of unit scale taken in turn (the clock the chip holds depends on how
//                     much the operands change from one instruction to the next).
//   sti_probe_stream  every thread reads 16 bytes and writes `ratio` x 16 bytes, coalesced, non-temporal:
//                     the HBM rate of a stream with the read : write mix of shard decompression
//                     (1 : 4.64 for the 2..6-bit mix of the decode-only configuration) beside a 1 : 1 copy.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// 4 independent accumulators per wave: consecutive MFMAs of a wave never wait for each other
template <bool VARIED>
__global__ __launch_bounds__(768) void mfma_loop_kernel(float *out, int iters)
{
    half8 a[4], b[4];
    uint32_t h = (blockIdx.x * 768u + threadIdx.x) * 2654435761u + 12345u;
    for (int j = 0; j < 4; ++j)
        for (int i = 0; i < 8; ++i) {
            if (VARIED) {
                h = h * 1664525u + 1013904223u;
                a[j][i] = (_Float16)(((int)(h >> 8) & 0xffff) * (4.0f / 65536.0f) - 2.0f);   // uniform in [-2, 2)
                h = h * 1664525u + 1013904223u;
                b[j][i] = (_Float16)(((int)(h >> 8) & 0xffff) * (4.0f / 65536.0f) - 2.0f);
            } else {
                a[j][i] = (_Float16)(threadIdx.x * 0.001f + i);
                b[j][i] = (_Float16)(i * 0.5f);
            }
        }
    float16v acc[4];
    for (int j = 0; j < 4; ++j)
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[VARIED ? j : 0], b[VARIED ? (j + 1) & 3 : 0], acc[j], 0, 0, 0);
    }
    float s = 0.f;
    for (int j = 0; j < 4; ++j)
        for (int v = 0; v < 16; ++v) s += acc[j][v];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <int RATIO>
__global__ __launch_bounds__(256) void stream_kernel(const u32x4 *in, u32x4 *out, size_t n_in)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_in) return;
    const u32x4 v = __builtin_nontemporal_load(in + i);
#pragma unroll
    for (int r = 0; r < RATIO; ++r) {
        const u32x4 w = v + (uint32_t)r;
        __builtin_nontemporal_store(w, out + ((size_t)blockIdx.x * RATIO + r) * 256 + threadIdx.x);
    }
}

template <typename F>
int time_launches(hipStream_t stream, int reps, double *ms_per_launch, F launch)
{
    hipEvent_t a = nullptr, b = nullptr;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return 1;
    launch();   // warm-up
    int rc = 0;
    if (hipEventRecord(a, stream) != hipSuccess) rc = 1;
    for (int i = 0; i < reps && !rc; ++i) launch();
    if (!rc && (hipGetLastError() != hipSuccess || hipEventRecord(b, stream) != hipSuccess ||
                hipEventSynchronize(b) != hipSuccess)) rc = 1;
    float ms = 0.f;
    if (!rc && hipEventElapsedTime(&ms, a, b) != hipSuccess) rc = 1;
    *ms_per_launch = ms / reps;
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    return rc;
}

}  // namespace

extern "C" {

// `blocks` workgroups of `waves` waves (1..12) run `iters` x 4 MFMAs per wave.  scratch: DEVICE,
// blocks * waves * 64 floats.  Returns 0 and the milliseconds per launch (average of `reps`), and the
// flops of one launch in *flops.
int sti_probe_mfma(int blocks, int waves, int iters, int reps, int varied, float *scratch, void *hip_stream,
                   double *ms_per_launch, double *flops)
{
    if (blocks <= 0 || waves <= 0 || waves > 12 || iters <= 0 || reps <= 0 || !scratch || !ms_per_launch || !flops)
        return 2;
    hipStream_t stream = (hipStream_t)hip_stream;
    *flops = (double)blocks * waves * iters * 4 * (2.0 * 32 * 32 * 16);
    return time_launches(stream, reps, ms_per_launch, [&] {
        if (varied) hipLaunchKernelGGL(mfma_loop_kernel<true>, dim3(blocks), dim3(waves * 64), 0, stream, scratch, iters);
        else hipLaunchKernelGGL(mfma_loop_kernel<false>, dim3(blocks), dim3(waves * 64), 0, stream, scratch, iters);
    });
}

// in: DEVICE, n_in * 16 bytes; out: DEVICE, n_in * 16 * ratio bytes (n_in a multiple of 256); ratio 1, 4 or 5.
int sti_probe_stream(const void *in, void *out, uint64_t n_in, int ratio, int reps, void *hip_stream,
                     double *ms_per_launch, double *bytes)
{
    if (!in || !out || n_in == 0 || n_in % 256 || reps <= 0 || !ms_per_launch || !bytes) return 2;
    if (ratio != 1 && ratio != 4 && ratio != 5) return 2;
    hipStream_t stream = (hipStream_t)hip_stream;
    const dim3 grid((uint32_t)(n_in / 256));
    *bytes = (double)n_in * 16 * (1 + ratio);
    return time_launches(stream, reps, ms_per_launch, [&] {
        if (ratio == 1) hipLaunchKernelGGL(stream_kernel<1>, grid, dim3(256), 0, stream, (const u32x4 *)in, (u32x4 *)out, (size_t)n_in);
        else if (ratio == 4) hipLaunchKernelGGL(stream_kernel<4>, grid, dim3(256), 0, stream, (const u32x4 *)in, (u32x4 *)out, (size_t)n_in);
        else hipLaunchKernelGGL(stream_kernel<5>, grid, dim3(256), 0, stream, (const u32x4 *)in, (u32x4 *)out, (size_t)n_in);
    });
}

}  // extern "C"
