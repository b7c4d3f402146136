// Layerwise load || compute pipeline with a preload buffer (Section "Elastic pipelining":
// the IO of layer k+1 overlaps the computation of layer k; a small preload buffer keeps the
// shards of the bottom layers across inferences; Section "Submodel execution": after an
// inference, loaded shards are kept from the bottom layers up until the buffer is full).
//
// Mapping onto this machine: the packed shard streams live in pinned host memory (the
// paper's flash); a library-owned copy stream moves the selected versions of layer k+1 over
// PCIe into one of a few staging slots in HBM while the caller's stream computes layer k;
// the first selected shards in (layer, shard) order that fit the preload buffer are placed
// there instead and found again by the next call with the same plan (no IO for them).
//
// A layer's shards are many small transfers (150 KB .. 2.4 MB each); issued one by one as
// DMA copies their fixed cost dominates.  Pinned host memory is mapped into the device's
// address space, so one gather kernel per layer pulls all of them over the link with a few
// hundred KB of reads in flight; host memory that is not mapped falls back to DMA copies.
#include <new>
#include <string.h>
#include <vector>

#include "api_internal.hpp"

constexpr int kMaxSlots = 8;

struct sti_pipeline {
    sti_dims dims;
    uint8_t *preload;
    size_t preload_bytes;
    uint8_t *staging;
    size_t slot_bytes;
    hipStream_t copy_stream;
    int n_slots;                       // staging ring depth (2 .. kMaxSlots)
    hipEvent_t loaded[kMaxSlots];      // copies of the layer using slot s have landed
    hipEvent_t computed[kMaxSlots];    // the layer using slot s has been computed
    hipEvent_t last_done;     // end of the previous call's compute
    bool has_last;
    struct Resident {
        int layer, shard, bits;
        const void *host;
        size_t off, bytes;
    };
    std::vector<Resident> resident;   // contents of the preload buffer, in placement order
    bool slot_used[kMaxSlots];
};

namespace sti {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct CopyItem {
    const uint8_t *src;   // device-visible address of pinned host memory
    uint8_t *dst;
    uint64_t bytes;
};
struct CopyTable {
    CopyItem item[kMaxShardsPerLayer];
};

constexpr int kCopyThreads = 1024;
constexpr int kCopyUnroll = 1;          // 16-byte loads in flight per thread
constexpr int kCopyChunk = kCopyThreads * kCopyUnroll;   // 16-byte units per workgroup step
constexpr int kCopyGrid = 8;            // 8 x 16 KiB in flight: measured to saturate the host link
constexpr int kCopyLdsClaim = 160 * 1024;

// A few workgroups walk all items of a layer in 16 KiB chunks.  Reads over the host link
// take microseconds; a compute wave that shares a compute unit with them waits behind them
// in the vector memory pipeline.  So the grid is small (the link is saturated by ~128 KiB in
// flight) and each workgroup claims a whole compute unit: 16 waves that are allotted 128
// vector registers each fill the register file of all four SIMDs, and the launch asks for
// the unit's whole LDS, so no wave of the other stream's kernels lands beside them.
__global__ __launch_bounds__(kCopyThreads) void gather_copy_kernel(const CopyTable table, int n_items)
{
    extern __shared__ unsigned char lds_claim[];
    (void)lds_claim;
    asm volatile("" ::: "v127");   // raises the kernel's register allotment to 128
    for (int e = 0; e < n_items; ++e) {
        const CopyItem it = table.item[e];
        const uint64_t n16 = it.bytes / 16;
        const u32x4 *src = (const u32x4 *)it.src;
        u32x4 *dst = (u32x4 *)it.dst;
        const uint64_t step = (uint64_t)gridDim.x * kCopyChunk;
        for (uint64_t base = (uint64_t)blockIdx.x * kCopyChunk + threadIdx.x; base < n16; base += step) {
            u32x4 v[kCopyUnroll];
#pragma unroll
            for (int j = 0; j < kCopyUnroll; ++j) {
                const uint64_t i = base + (uint64_t)j * kCopyThreads;
                if (i < n16) v[j] = src[i];
            }
#pragma unroll
            for (int j = 0; j < kCopyUnroll; ++j) {
                const uint64_t i = base + (uint64_t)j * kCopyThreads;
                if (i < n16) dst[i] = v[j];
            }
        }
        if (blockIdx.x == (unsigned)e % gridDim.x) {
            const uint64_t tail = n16 * 16 + threadIdx.x;
            if (tail < it.bytes) it.dst[tail] = it.src[tail];
        }
    }
}

inline size_t shard_bytes(const sti_dims &d, int bits)
{
    const size_t wsh = (size_t)d.d_model * (4 * (size_t)d.d_head + 2 * (size_t)d.ffn_per_shard);
    return bits == 32 ? wsh * 4 : (wsh * (size_t)bits + 7) / 8;
}

// The address a kernel can use for `host`, or nullptr when the memory is not mapped into the
// device's address space (then only the runtime's own copies can read it).  Asked on every
// copy: an address that was pinned memory once may be ordinary memory by the next call.
const void *device_view(const void *host)
{
    const void *view = nullptr;
    hipPointerAttribute_t attr;
    memset(&attr, 0, sizeof(attr));
    if (hipPointerGetAttributes(&attr, host) == hipSuccess) {
        if (attr.type == hipMemoryTypeHost && attr.devicePointer &&
            ((uintptr_t)attr.devicePointer & 15) == 0)
            view = attr.devicePointer;
    } else {
        (void)hipGetLastError();   // ordinary host memory: not an error of this call
    }
    return view;
}

}  // namespace
}  // namespace sti

using namespace sti;

extern "C" {

size_t sti_pipeline_staging_bytes(const sti_dims *dims)
{
    if (!dims || dims->d_model <= 0 || dims->d_head <= 0 || dims->ffn_per_shard <= 0 ||
        dims->n_heads <= 0 || dims->n_heads > kMaxShardsPerLayer)
        return 0;
    return 2 * align_up((size_t)dims->n_heads * align_up(shard_bytes(*dims, 32), 256), 256);
}

sti_status sti_pipeline_create(const sti_dims *dims, void *preload_buffer, size_t preload_bytes,
                               void *staging, size_t staging_bytes, sti_pipeline **out)
{
    if (!dims || !out) return STI_ERR_NULL;
    *out = nullptr;
    const size_t need = sti_pipeline_staging_bytes(dims);
    if (need == 0) return STI_ERR_DIMS;
    if (!staging || staging_bytes < need) return STI_ERR_WORKSPACE;
    if (preload_bytes != 0 && !preload_buffer) return STI_ERR_NULL;
    if (!aligned(staging, 256) || (preload_buffer && !aligned(preload_buffer, 256))) return STI_ERR_ALIGN;
    sti_pipeline *p = new (std::nothrow) sti_pipeline();
    if (!p) return STI_ERR_HIP;
    p->dims = *dims;
    p->preload = (uint8_t *)preload_buffer;
    p->preload_bytes = preload_buffer ? preload_bytes : 0;
    p->staging = (uint8_t *)staging;
    p->slot_bytes = need / 2;
    p->n_slots = (int)(staging_bytes / p->slot_bytes);
    if (p->n_slots > kMaxSlots) p->n_slots = kMaxSlots;
    p->copy_stream = nullptr;
    p->has_last = false;
    p->last_done = nullptr;
    for (int s = 0; s < kMaxSlots; ++s) {
        p->slot_used[s] = false;
        p->loaded[s] = p->computed[s] = nullptr;
    }
    bool ok = hipFuncSetAttribute((const void *)gather_copy_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                  kCopyLdsClaim) == hipSuccess;
    ok = ok && hipStreamCreateWithFlags(&p->copy_stream, hipStreamNonBlocking) == hipSuccess;
    for (int s = 0; s < p->n_slots && ok; ++s) {
        ok = hipEventCreateWithFlags(&p->loaded[s], hipEventDisableTiming) == hipSuccess &&
             hipEventCreateWithFlags(&p->computed[s], hipEventDisableTiming) == hipSuccess;
    }
    ok = ok && hipEventCreateWithFlags(&p->last_done, hipEventDisableTiming) == hipSuccess;
    if (!ok) {
        sti_pipeline_destroy(p);
        return STI_ERR_HIP;
    }
    *out = p;
    return STI_OK;
}

sti_status sti_pipeline_destroy(sti_pipeline *p)
{
    if (!p) return STI_OK;
    sti_status st = STI_OK;
    if (p->copy_stream) {
        if (hipStreamSynchronize(p->copy_stream) != hipSuccess) st = STI_ERR_HIP;
        if (hipStreamDestroy(p->copy_stream) != hipSuccess) st = STI_ERR_HIP;
    }
    for (int s = 0; s < kMaxSlots; ++s) {
        if (p->loaded[s] && hipEventDestroy(p->loaded[s]) != hipSuccess) st = STI_ERR_HIP;
        if (p->computed[s] && hipEventDestroy(p->computed[s]) != hipSuccess) st = STI_ERR_HIP;
    }
    if (p->last_done && hipEventDestroy(p->last_done) != hipSuccess) st = STI_ERR_HIP;
    delete p;
    return st;
}

}  // extern "C"

namespace {

// masked: the call came through sti_pipeline_forward_masked and key_lengths must be usable
sti_status pipeline_forward(sti_pipeline *pl, int n_layers, const sti_shard *store,
                            const sti_layer_params *params, const int8_t *plan, const void *x,
                            void *y, sti_dtype io_dtype, int batch, int seq, bool masked,
                            const int32_t *key_lengths, sti_precision precision, void *workspace,
                            size_t workspace_bytes, void *hip_stream, sti_pipeline_stats *stats)
{
    if (!pl) return STI_ERR_NULL;
    if (stats) memset(stats, 0, sizeof(*stats));
    const sti_dims *dims = &pl->dims;
    sti_status st = check_dims(dims, batch, seq, precision);
    if (st != STI_OK) return st;
    if (n_layers < 0) return STI_ERR_DIMS;
    const int64_t T = (int64_t)batch * seq;
    st = check_io(x, y, io_dtype, T, dims->d_model);
    if (st != STI_OK) return st;
    if (masked && T > 0) {
        st = check_key_lengths(key_lengths);
        if (st != STI_OK) return st;
    }
    const int M = dims->n_heads;
    if (n_layers > 0 && (!store || !params || !plan)) return STI_ERR_NULL;
    std::vector<sti_shard> chosen;
    try {
        chosen.resize((size_t)n_layers * M);
    } catch (const std::bad_alloc &) {
        return STI_ERR_HIP;
    }
    for (int l = 0; l < n_layers; ++l) {
        st = check_params(&params[l]);
        if (st != STI_OK) return st;
        for (int i = 0; i < M; ++i) {
            const int k = plan[(size_t)l * M + i];
            sti_shard &c = chosen[(size_t)l * M + i];
            memset(&c, 0, sizeof(c));
            if (k == 0) continue;
            int slot;
            if (valid_packed_bits(k)) slot = k - 2;
            else if (k == 32) slot = 5;
            else return STI_ERR_BITWIDTH;
            const sti_shard &v = store[((size_t)l * M + i) * 6 + slot];
            if (!v.data) return STI_ERR_MISSING_SHARD;
            if (v.bitwidth != k) return STI_ERR_BITWIDTH;
            st = check_decode_shard(v);   // pointer presence and alignment (data is a host address here)
            if (st != STI_OK) return st;
            c = v;
        }
    }
    const WorkspaceLayout wl = workspace_layout(*dims, T, precision);
    if (!workspace || workspace_bytes < wl.total) return STI_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return STI_ERR_ALIGN;
    if (T == 0) return STI_OK;

    hipStream_t stream = (hipStream_t)hip_stream;
    uint8_t *ws = (uint8_t *)workspace;
    const size_t io_bytes = (size_t)T * dims->d_model * (io_dtype == STI_F32 ? 4 : 2);
    if (n_layers == 0) {
        STI_TRY(hipMemcpyAsync(y, x, io_bytes, hipMemcpyDeviceToDevice, stream));
        return STI_OK;
    }

    // ---- which selected shards live in the preload buffer after this call: the longest
    //      prefix in (layer, shard) order that fits ----
    std::vector<sti_pipeline::Resident> want;
    {
        size_t cum = 0;
        bool full = false;
        for (int l = 0; l < n_layers && !full; ++l)
            for (int i = 0; i < M && !full; ++i) {
                const sti_shard &c = chosen[(size_t)l * M + i];
                if (c.bitwidth == 0) continue;
                const size_t bytes = shard_bytes(*dims, c.bitwidth);
                if (cum + bytes > pl->preload_bytes) { full = true; break; }
                want.push_back({l, i, c.bitwidth, c.data, cum, bytes});
                cum = align_up(cum + bytes, 256);
            }
    }
    auto is_hit = [&](size_t idx) {
        if (idx >= pl->resident.size()) return false;
        const auto &a = pl->resident[idx];
        const auto &b = want[idx];
        return a.layer == b.layer && a.shard == b.shard && a.bits == b.bits && a.host == b.host &&
               a.off == b.off && a.bytes == b.bytes;
    };

    // the copies of this call may overwrite what the previous call's kernels still read
    if (pl->has_last) STI_TRY(hipStreamWaitEvent(pl->copy_stream, pl->last_done, 0));

    const sti_dtype act = (precision == STI_PREC_F32) ? STI_F32 : STI_F16;
    const void *cur = x;
    int next_buf = 0;
    if (io_dtype != act) {
        STI_TRY(launch_convert(x, io_dtype, ws + wl.act[0], act, (uint64_t)T * dims->d_model, stream));
        cur = ws + wl.act[0];
        next_buf = 1;
    }
    size_t want_pos = 0;   // next entry of `want` (entries are in layer, shard order)
    for (int s = 0; s < kMaxSlots; ++s) pl->slot_used[s] = false;
    for (int l = 0; l < n_layers; ++l) {
        const int slot = l % pl->n_slots;
        sti_shard *row = &chosen[(size_t)l * M];
        CopyTable table;
        int n_gather = 0, n_copies = 0;
        size_t slot_off = 0;
        bool waited = false;
        for (int i = 0; i < M; ++i) {
            if (row[i].bitwidth == 0) continue;
            const size_t bytes = shard_bytes(*dims, row[i].bitwidth);
            uint8_t *dst;
            bool copy = true;
            if (want_pos < want.size() && want[want_pos].layer == l && want[want_pos].shard == i) {
                dst = pl->preload + want[want_pos].off;
                if (is_hit(want_pos)) {
                    copy = false;
                    if (stats) stats->shards_hit += 1;
                }
                if (stats) { stats->bytes_resident += bytes; stats->shards_preloaded += 1; }
                ++want_pos;
            } else {
                // the slot was last read by layer l - n_slots
                if (!waited && pl->slot_used[slot]) {
                    STI_TRY(hipStreamWaitEvent(pl->copy_stream, pl->computed[slot], 0));
                    waited = true;
                }
                dst = pl->staging + (size_t)slot * pl->slot_bytes + slot_off;
                slot_off = align_up(slot_off + bytes, 256);
            }
            if (copy) {
                const void *view = device_view(row[i].data);
                if (view) {
                    table.item[n_gather++] = {(const uint8_t *)view, dst, (uint64_t)bytes};
                } else {
                    STI_TRY(hipMemcpyAsync(dst, row[i].data, bytes, hipMemcpyHostToDevice, pl->copy_stream));
                }
                ++n_copies;
                if (stats) { stats->bytes_copied += bytes; stats->shards_copied += 1; }
            }
            row[i].data = dst;   // from here on the shard is a device shard
        }
        if (n_gather > 0) {
            gather_copy_kernel<<<dim3(kCopyGrid), dim3(kCopyThreads), kCopyLdsClaim, pl->copy_stream>>>(
                table, n_gather);
            STI_TRY(hipGetLastError());
        }
        if (n_copies > 0) {
            STI_TRY(hipEventRecord(pl->loaded[slot], pl->copy_stream));
            STI_TRY(hipStreamWaitEvent(stream, pl->loaded[slot], 0));
        }
        const bool last = (l == n_layers - 1);
        void *out = last ? y : (void *)(ws + wl.act[next_buf]);
        st = run_layer(*dims, row, params[l], cur, out, last ? io_dtype : act, batch, seq, precision,
                       ws, wl, stream, nullptr, masked ? key_lengths : nullptr);
        if (st != STI_OK) return st;
        if (slot_off > 0) {
            STI_TRY(hipEventRecord(pl->computed[slot], stream));
            pl->slot_used[slot] = true;
        }
        cur = out;
        next_buf ^= 1;
    }
    STI_TRY(hipEventRecord(pl->last_done, stream));
    pl->has_last = true;
    pl->resident.swap(want);
    return STI_OK;
}

}  // namespace

extern "C" {

sti_status sti_pipeline_forward(sti_pipeline *pl, int n_layers, const sti_shard *store,
                                const sti_layer_params *params, const int8_t *plan, const void *x,
                                void *y, sti_dtype io_dtype, int batch, int seq,
                                sti_precision precision, void *workspace, size_t workspace_bytes,
                                void *hip_stream, sti_pipeline_stats *stats)
{
    return pipeline_forward(pl, n_layers, store, params, plan, x, y, io_dtype, batch, seq, false, nullptr,
                            precision, workspace, workspace_bytes, hip_stream, stats);
}

sti_status sti_pipeline_forward_masked(sti_pipeline *pl, int n_layers, const sti_shard *store,
                                       const sti_layer_params *params, const int8_t *plan, const void *x,
                                       void *y, sti_dtype io_dtype, int batch, int seq,
                                       const int32_t *key_lengths, sti_precision precision,
                                       void *workspace, size_t workspace_bytes, void *hip_stream,
                                       sti_pipeline_stats *stats)
{
    return pipeline_forward(pl, n_layers, store, params, plan, x, y, io_dtype, batch, seq, true, key_lengths,
                            precision, workspace, workspace_bytes, hip_stream, stats);
}

}  // extern "C"
