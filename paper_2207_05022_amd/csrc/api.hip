// C ABI of libsti: argument validation, shard-table staging, kernel sequencing.
// Every check runs before the first launch; device work goes to the caller's stream.
#include <mutex>
#include <new>
#include <string.h>
#include <vector>

#include "sti_internal.hpp"

namespace sti {
namespace {

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

inline bool valid_packed_bits(int b) { return b >= 2 && b <= 6; }

// Pinned host ring through which shard tables larger than the inline limit are
// uploaded.  A slot is reused only after the copy that read it has completed.
class StagingRing {
public:
    static constexpr int kSlots = 4;
    hipError_t upload(const ShardDesc *src, size_t count, void *dst, hipStream_t stream)
    {
        std::lock_guard<std::mutex> lock(mu_);
        Slot &s = slots_[next_];
        next_ = (next_ + 1) % kSlots;
        const size_t bytes = count * sizeof(ShardDesc);
        hipError_t e;
        if (s.event) {
            e = hipEventSynchronize(s.event);
            if (e != hipSuccess) return e;
        } else {
            e = hipEventCreateWithFlags(&s.event, hipEventDisableTiming);
            if (e != hipSuccess) return e;
        }
        if (s.capacity < bytes) {
            if (s.ptr) {
                e = hipHostFree(s.ptr);
                s.ptr = nullptr;
                s.capacity = 0;
                if (e != hipSuccess) return e;
            }
            size_t cap = 1 << 16;
            while (cap < bytes) cap <<= 1;
            e = hipHostMalloc(&s.ptr, cap, hipHostMallocDefault);
            if (e != hipSuccess) return e;
            s.capacity = cap;
        }
        memcpy(s.ptr, src, bytes);
        e = hipMemcpyAsync(dst, s.ptr, bytes, hipMemcpyHostToDevice, stream);
        if (e != hipSuccess) return e;
        return hipEventRecord(s.event, stream);
    }

private:
    struct Slot {
        void *ptr = nullptr;
        size_t capacity = 0;
        hipEvent_t event = nullptr;
    };
    std::mutex mu_;
    Slot slots_[kSlots];
    int next_ = 0;
};

StagingRing &staging()
{
    static StagingRing ring;
    return ring;
}

sti_status check_decode_shard(const sti_shard &s)
{
    const int b = s.bitwidth;
    if (b != 32 && !valid_packed_bits(b)) return STI_ERR_BITWIDTH;
    if (!s.data) return STI_ERR_MISSING_SHARD;
    if (b != 32 && !s.codebook) return STI_ERR_MISSING_SHARD;
    if (s.n_outliers != 0 || s.outlier_pos || s.outlier_val) return STI_ERR_UNSUPPORTED;
    if (!aligned(s.data, 16)) return STI_ERR_ALIGN;
    if (b != 32 && !aligned(s.codebook, 4)) return STI_ERR_ALIGN;
    return STI_OK;
}

}  // namespace
}  // namespace sti

using namespace sti;

extern "C" {

const char *sti_status_string(sti_status s)
{
    switch (s) {
        case STI_OK: return "ok";
        case STI_ERR_NULL: return "required pointer is NULL";
        case STI_ERR_DIMS: return "invalid or unsupported dimensions";
        case STI_ERR_BITWIDTH: return "bitwidth outside {0,2,3,4,5,6,32}";
        case STI_ERR_MISSING_SHARD: return "selected shard version has no data";
        case STI_ERR_ALIGN: return "device pointer not aligned as documented";
        case STI_ERR_WORKSPACE: return "workspace missing or too small";
        case STI_ERR_DTYPE: return "unknown dtype or precision";
        case STI_ERR_HIP: return "HIP runtime call failed";
        case STI_ERR_UNSUPPORTED: return "request not implemented";
    }
    return "unknown status";
}

size_t sti_decode_workspace_bytes(int n_shards)
{
    if (n_shards <= kInlineShards) return 0;
    return (size_t)n_shards * sizeof(ShardDesc);
}

sti_status sti_decode_shards(const sti_shard *shards, int n_shards, uint64_t weights_per_shard,
                             void *out, sti_dtype out_dtype, void *workspace,
                             size_t workspace_bytes, void *hip_stream)
{
    if (n_shards < 0) return STI_ERR_DIMS;
    if (out_dtype != STI_F32 && out_dtype != STI_F16 && out_dtype != STI_BF16) return STI_ERR_DTYPE;
    if (n_shards == 0) return STI_OK;
    if (!shards) return STI_ERR_NULL;
    if (weights_per_shard > (1ull << 40)) return STI_ERR_DIMS;
    if (weights_per_shard != 0 && !out) return STI_ERR_NULL;
    if (out && !aligned(out, 16)) return STI_ERR_ALIGN;
    for (int s = 0; s < n_shards; ++s) {
        sti_status st = check_decode_shard(shards[s]);
        if (st != STI_OK) return st;
    }
    const size_t need = sti_decode_workspace_bytes(n_shards);
    if (need) {
        if (!workspace || workspace_bytes < need) return STI_ERR_WORKSPACE;
        if (!aligned(workspace, 16)) return STI_ERR_ALIGN;
    }
    if (weights_per_shard == 0) return STI_OK;

    hipStream_t stream = (hipStream_t)hip_stream;
    hipError_t e;
    if (need) {
        std::vector<ShardDesc> table;
        try {
            table.resize(n_shards);
        } catch (const std::bad_alloc &) {
            return STI_ERR_HIP;
        }
        for (int s = 0; s < n_shards; ++s)
            table[s] = ShardDesc{shards[s].data, shards[s].codebook, shards[s].bitwidth, s};
        e = staging().upload(table.data(), table.size(), workspace, stream);
        if (e != hipSuccess) return STI_ERR_HIP;
        e = launch_decode((const ShardDesc *)workspace, nullptr, n_shards, weights_per_shard, out,
                          out_dtype, stream);
    } else {
        InlineShardTable t;
        memset(&t, 0, sizeof(t));
        for (int s = 0; s < n_shards; ++s)
            t.d[s] = ShardDesc{shards[s].data, shards[s].codebook, shards[s].bitwidth, s};
        e = launch_decode(nullptr, &t, n_shards, weights_per_shard, out, out_dtype, stream);
    }
    return e == hipSuccess ? STI_OK : STI_ERR_HIP;
}

}  // extern "C"
