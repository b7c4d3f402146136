// Outlier-aware quantization of one layer's shards into a k-bit version (Section
// "quantization per shard"; Section "Implementation", preprocessing): a single Gaussian is
// fitted to all weights of the layer, weights whose log likelihood is below a threshold are
// outliers, the others are cut into 2^k clusters of equal population (by sorted rank), each
// cluster's centroid is the mean of its members, and every weight becomes the k-bit index of
// its cluster; outliers keep a placeholder index and are bookkept with offset and value.
//
// No sort is needed for equal-population clusters: only the 2^k - 1 boundary values are, and
// those are found by rank selection with two 16-bit histogram passes over an order-preserving
// integer image of the floats.  All passes stream the layer once (HBM bound):
//   moments -> outlier test + high-half histogram -> boundary bins -> low-half histograms of
//   those bins -> boundary values -> per-cluster sums -> centroids -> pack + outlier lists.
// Sums are accumulated in float64 in a fixed order, so a run is reproducible bit for bit.
#include "api_internal.hpp"

namespace sti {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kChunk = 1024;        // weights per workgroup in the streaming passes
constexpr int kMaxClusters = 64;
constexpr int kBins = 65536;

struct QuantState {
    double mu, var, r2;             // outlier iff (x - mu)^2 > r2
    unsigned long long n_total, n_inliers;
    uint32_t edge_key[kMaxClusters];    // [c-1]: key of the lowest member of cluster c, c = 1..C-1
    uint32_t edge_bin[kMaxClusters];
    uint32_t edge_rank[kMaxClusters];   // rank of that member inside its high-half bin
    uint32_t n_slots;
    uint32_t slot_bin[kMaxClusters];
    uint32_t error;                 // 1: no inliers
};

struct QuantLayout {
    size_t state, partials, hist_hi, bin_slot, hist_lo, chunk_count, chunk_off, csum, zero_begin, zero_end, total;
};

QuantLayout quant_layout(int64_t n_chunks, int n_blocks_moments)
{
    QuantLayout L;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t at = off; off = align_up(off + bytes, 256); return at; };
    L.state = take(sizeof(QuantState));
    L.partials = take((size_t)n_blocks_moments * 2 * sizeof(double));
    L.chunk_count = take((size_t)n_chunks * 4);
    L.chunk_off = take((size_t)n_chunks * 4);
    L.csum = take((size_t)n_chunks * kMaxClusters * (sizeof(double) + 4));
    L.zero_begin = off;
    L.hist_hi = take((size_t)kBins * 4);
    L.bin_slot = take((size_t)kBins);
    L.hist_lo = take((size_t)(kMaxClusters - 1) * kBins * 4);
    L.zero_end = off;
    L.total = off;
    return L;
}

// order-preserving image of a float (-0.0 counted as +0.0)
__device__ inline uint32_t order_key(float x)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, x + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ inline float key_value(uint32_t k)
{
    const uint32_t u = (k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k;
    return __builtin_bit_cast(float, u);
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = 0;
}

__device__ inline double block_sum_256(double v, double *lds)
{
    // fixed order: butterfly inside a wave, then the four waves in order
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds[wave] = v;
    __syncthreads();
    return lds[0] + lds[1] + lds[2] + lds[3];
}

__global__ __launch_bounds__(256) void moments_kernel(const float *w, uint64_t n, double *partials)
{
    __shared__ double lds[4];
    double s = 0.0, ss = 0.0;
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (uint64_t)gridDim.x * 256) {
        const double x = (double)w[i];
        s += x;
        ss += x * x;
    }
    const double bs = block_sum_256(s, lds);
    const double bss = block_sum_256(ss, lds);
    if (threadIdx.x == 0) { partials[2 * blockIdx.x] = bs; partials[2 * blockIdx.x + 1] = bss; }
}

__global__ __launch_bounds__(256) void fit_kernel(const double *partials, int n_blocks, uint64_t n, double threshold,
                                                  double reg_covar, QuantState *st)
{
    __shared__ double lds[4];
    double s = 0.0, ss = 0.0;
    for (int b = threadIdx.x; b < n_blocks; b += 256) { s += partials[2 * b]; ss += partials[2 * b + 1]; }
    const double ts = block_sum_256(s, lds);
    const double tss = block_sum_256(ss, lds);
    if (threadIdx.x == 0) {
        const double mu = ts / (double)n;
        const double var = tss / (double)n - mu * mu + reg_covar;
        st->mu = mu;
        st->var = var;
        // log N(x; mu, var) < threshold  <=>  (x - mu)^2 > 2 var (-threshold - log sqrt(2 pi var))
        st->r2 = 2.0 * var * (-threshold - 0.5 * log(2.0 * 3.14159265358979323846 * var));
        st->n_total = n;
        st->error = 0;
    }
}

// Outlier test, high-half histogram of the inliers, number of outliers per chunk of 1024
// weights.  A workgroup of 1024 threads walks chunks 4 at a time (grid-strided) and counts into
// a histogram of its own in LDS - the keys of Gaussian weights crowd into about a thousand of
// the 65536 bins, which serialises device-wide atomics - and adds the bins it touched to the
// global histogram at the end.  Two 16-bit counters per LDS word: the host sizes the grid so
// that a workgroup sees fewer than 65536 weights.
__global__ __launch_bounds__(1024) void classify_kernel(const float *w, const QuantState *st, int64_t n_chunks,
                                                        uint32_t *hist_hi, uint32_t *chunk_count)
{
    __shared__ uint32_t hist[kBins / 2];
    __shared__ uint32_t cnt[16];
    for (int i = threadIdx.x; i < kBins / 2; i += 1024) hist[i] = 0;
    __syncthreads();
    const double mu = st->mu, r2 = st->r2;
    const int wave = threadIdx.x >> 6;
    for (int64_t c0 = (int64_t)blockIdx.x * 4; c0 < n_chunks; c0 += (int64_t)gridDim.x * 4) {
        const int64_t chunk = c0 + (threadIdx.x >> 8);
        uint32_t outl = 0;
        if (chunk < n_chunks) {
            const f32x4 v = *(const f32x4 *)(w + (size_t)chunk * kChunk + (threadIdx.x & 255) * 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const double d = (double)v[e] - mu;
                if (d * d > r2) {
                    outl += 1;
                } else {
                    const uint32_t bin = order_key(v[e]) >> 16;
                    atomicAdd(&hist[bin >> 1], 1u << (16 * (bin & 1)));
                }
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) outl += __shfl_down(outl, o, 64);
        __syncthreads();
        if ((threadIdx.x & 63) == 0) cnt[wave] = outl;
        __syncthreads();
        if ((threadIdx.x & 255) == 0 && chunk < n_chunks)
            chunk_count[chunk] = cnt[wave] + cnt[wave + 1] + cnt[wave + 2] + cnt[wave + 3];
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kBins / 2; i += 1024) {
        const uint32_t h = hist[i];
        if (h & 0xFFFFu) atomicAdd(&hist_hi[2 * i], h & 0xFFFFu);
        if (h >> 16) atomicAdd(&hist_hi[2 * i + 1], h >> 16);
    }
}

// exclusive scan of 1024 per-thread values (returns the prefix of this thread; *total = sum)
__device__ inline uint64_t block_scan_1024(uint64_t v, uint64_t *lds, uint64_t *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint64_t inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint64_t t = __shfl_up(inc, o, 64);
        if (lane >= o) inc += t;
    }
    __syncthreads();
    if (lane == 63) lds[wave] = inc;
    __syncthreads();
    uint64_t base = 0;
    for (int i = 0; i < wave; ++i) base += lds[i];
    uint64_t tot = 0;
    for (int i = 0; i < 16; ++i) tot += lds[i];
    *total = tot;
    return base + inc - v;
}

// single workgroup: outlier list offsets per shard, number of inliers, and for every cluster
// boundary the high-half bin that holds its rank.  Laid out so that nothing waits on a chain
// of dependent global loads: one wave scans one shard's chunk counts, a thread keeps its 64
// bins in registers for the search, and the boundary bins reach the last step through LDS.
__global__ __launch_bounds__(1024) void select_bins_kernel(QuantState *st, const uint32_t *hist_hi, uint8_t *bin_slot,
                                                           const uint32_t *chunk_count, uint32_t *chunk_off,
                                                           int n_shards, int chunks_per_shard, int n_clusters,
                                                           uint32_t *outlier_count)
{
    __shared__ uint64_t lds[16];
    __shared__ uint32_t shard_outliers[kMaxShardsPerLayer];
    __shared__ uint32_t l_edge_bin[kMaxClusters];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // (a) outlier list offsets: exclusive scan of the chunk counts of each shard, 4 chunks per
    //     lane and step
    for (int s = wave; s < n_shards; s += 16) {
        const uint32_t *cnt = chunk_count + (size_t)s * chunks_per_shard;
        uint32_t *off = chunk_off + (size_t)s * chunks_per_shard;
        uint32_t carry = 0;
        for (int base = 0; base < chunks_per_shard; base += 256) {
            const int c0 = base + lane * 4;
            uint32_t v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = (c0 + j < chunks_per_shard) ? cnt[c0 + j] : 0;
            const uint32_t mine = v[0] + v[1] + v[2] + v[3];
            uint32_t inc = mine;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t up = __shfl_up(inc, o, 64);
                if (lane >= o) inc += up;
            }
            uint32_t p = carry + inc - mine;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (c0 + j < chunks_per_shard) off[c0 + j] = p;
                p += v[j];
            }
            carry += __shfl(inc, 63, 64);
        }
        if (lane == 0) {
            outlier_count[s] = carry;
            shard_outliers[s] = carry;
        }
    }
    __syncthreads();
    uint64_t n_out_total = 0;
    for (int s = 0; s < n_shards; ++s) n_out_total += shard_outliers[s];
    const uint64_t n_in = st->n_total - n_out_total;
    if (threadIdx.x == 0) {
        st->n_inliers = n_in;
        if (n_in == 0) st->error = 1;
    }
    if (n_in == 0) return;
    // (b) prefix of the 65536 bins, 64 consecutive bins per thread (kept in registers)
    uint32_t h[64];
    const uint4 *h4 = (const uint4 *)(hist_hi + threadIdx.x * 64);
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const uint4 x = h4[q];
        h[4 * q] = x.x; h[4 * q + 1] = x.y; h[4 * q + 2] = x.z; h[4 * q + 3] = x.w;
    }
    uint64_t own = 0;
#pragma unroll
    for (int b = 0; b < 64; ++b) own += h[b];
    uint64_t total;
    const uint64_t pre = block_scan_1024(own, lds, &total);
    for (int c = 1; c < n_clusters; ++c) {
        const uint64_t rank = ((uint64_t)c * n_in) / (uint64_t)n_clusters;
        if (rank >= pre && rank < pre + own) {
            const uint32_t rel = (uint32_t)(rank - pre);   // rank inside this thread's 64 bins
            uint32_t p = 0;
            int bin = -1;
            uint32_t rank_in_bin = 0;
#pragma unroll
            for (int b = 0; b < 64; ++b) {
                if (bin < 0 && rel < p + h[b]) {
                    bin = b;
                    rank_in_bin = rel - p;
                }
                p += h[b];
            }
            st->edge_bin[c - 1] = threadIdx.x * 64 + bin;
            st->edge_rank[c - 1] = rank_in_bin;
            l_edge_bin[c - 1] = threadIdx.x * 64 + bin;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t n_slots = 0, last_bin = 0;
        for (int c = 1; c < n_clusters; ++c) {
            const uint32_t bin = l_edge_bin[c - 1];
            if (n_slots == 0 || last_bin != bin) {   // boundary bins are non-decreasing
                st->slot_bin[n_slots] = bin;
                bin_slot[bin] = (uint8_t)(n_slots + 1);
                last_bin = bin;
                ++n_slots;
            }
        }
        st->n_slots = n_slots;
    }
}

__global__ __launch_bounds__(256) void hist_lo_kernel(const float *w, const QuantState *st, const uint8_t *bin_slot,
                                                      uint32_t *hist_lo)
{
    const double mu = st->mu, r2 = st->r2;
    const f32x4 v = *(const f32x4 *)(w + (size_t)blockIdx.x * kChunk + threadIdx.x * 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const double d = (double)v[e] - mu;
        if (d * d > r2) continue;
        const uint32_t key = order_key(v[e]);
        const uint32_t slot = bin_slot[key >> 16];
        if (slot) atomicAdd(&hist_lo[(size_t)(slot - 1) * kBins + (key & 0xFFFFu)], 1u);
    }
}

// one workgroup per boundary: the value at the boundary's rank
__global__ __launch_bounds__(1024) void select_values_kernel(QuantState *st, const uint8_t *bin_slot,
                                                             const uint32_t *hist_lo)
{
    __shared__ uint64_t lds[16];
    if (st->error) return;
    const int c = blockIdx.x + 1;
    const uint32_t bin = st->edge_bin[c - 1];
    const uint64_t rank = st->edge_rank[c - 1];
    const uint32_t *h = hist_lo + (size_t)(bin_slot[bin] - 1) * kBins;
    uint64_t own = 0;
    for (int b = 0; b < 64; ++b) own += h[threadIdx.x * 64 + b];
    uint64_t total;
    const uint64_t pre = block_scan_1024(own, lds, &total);
    if (rank >= pre && rank < pre + own) {
        uint64_t p = pre;
        for (int b = 0; b < 64; ++b) {
            const uint64_t x = h[threadIdx.x * 64 + b];
            if (rank < p + x) {
                st->edge_key[c - 1] = (bin << 16) | (uint32_t)(threadIdx.x * 64 + b);
                break;
            }
            p += x;
        }
    }
}

// number of boundaries whose key is <= key: the cluster index
__device__ inline int cluster_of(uint32_t key, const uint32_t *edges, int n_edges)
{
    int lo = 0, hi = n_edges;   // first edge with edge > key
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (edges[mid] <= key) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

// per chunk: float64 sum and count of the inliers of every cluster
__global__ __launch_bounds__(256) void cluster_sums_kernel(const float *w, const QuantState *st, int n_clusters,
                                                           double *csum, uint32_t *ccount)
{
    __shared__ uint32_t edges[kMaxClusters];
    __shared__ double wsum[4][kMaxClusters];
    __shared__ uint32_t wcnt[4][kMaxClusters];
    if (threadIdx.x < n_clusters - 1) edges[threadIdx.x] = st->edge_key[threadIdx.x];
    (&wsum[0][0])[threadIdx.x] = 0.0;   // 4 x kMaxClusters = 256 accumulators, one per thread
    (&wcnt[0][0])[threadIdx.x] = 0;
    __syncthreads();
    const double mu = st->mu, r2 = st->r2;
    const f32x4 v = *(const f32x4 *)(w + (size_t)blockIdx.x * kChunk + threadIdx.x * 4);
    int idx[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const double d = (double)v[e] - mu;
        idx[e] = (d * d > r2) ? -1 : cluster_of(order_key(v[e]), edges, n_clusters - 1);
    }
    const int wave = threadIdx.x >> 6;
    // every wave adds into accumulators of its own with LDS atomics (float64 add, integer add):
    // four instructions per kind and wave instead of a shuffle reduction per cluster.  Lanes
    // of one instruction that hit the same cluster are added in the order the LDS serialises
    // them; float64 sums of at most 256 float32 values agree to ~1e-16 relative in any order,
    // and the centroid is rounded to float32 once, from the sum over all chunks.
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (idx[e] >= 0) {
            unsafeAtomicAdd(&wsum[wave][idx[e]], (double)(v[e] + 0.0f));
            atomicAdd(&wcnt[wave][idx[e]], 1u);
        }
    }
    __syncthreads();
    if (threadIdx.x < n_clusters) {
        const int c = threadIdx.x;
        csum[(size_t)blockIdx.x * kMaxClusters + c] = wsum[0][c] + wsum[1][c] + wsum[2][c] + wsum[3][c];
        ccount[(size_t)blockIdx.x * kMaxClusters + c] = wcnt[0][c] + wcnt[1][c] + wcnt[2][c] + wcnt[3][c];
    }
}

// one workgroup per cluster: centroid = mean of the cluster (its lower boundary value if it is
// empty); the chunk partials are added in a fixed order
__global__ __launch_bounds__(1024) void centroids_kernel(const QuantState *st, const double *csum, const uint32_t *ccount,
                                                         int64_t n_chunks, float *codebook, sti_quant_stats *stats)
{
    __shared__ double ls[16];
    __shared__ uint64_t ln[16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = blockIdx.x;
    double s = 0.0;
    uint64_t n = 0;
    for (int64_t b = threadIdx.x; b < n_chunks; b += 1024) {
        s += csum[(size_t)b * kMaxClusters + c];
        n += ccount[(size_t)b * kMaxClusters + c];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { s += __shfl_down(s, o, 64); n += __shfl_down(n, o, 64); }
    if (lane == 0) { ls[wave] = s; ln[wave] = n; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double ts = 0.0;
        uint64_t tn = 0;
        for (int i = 0; i < 16; ++i) { ts += ls[i]; tn += ln[i]; }
        float cen;
        if (st->error) cen = 0.0f;
        else if (tn) cen = (float)(ts / (double)tn);
        else cen = key_value(st->edge_key[c > 0 ? c - 1 : 0]);
        codebook[c] = cen;
        if (c == 0 && stats) {
            stats->mean = st->mu;
            stats->variance = st->var;
            stats->n_outliers = st->n_total - st->n_inliers;
            stats->status = st->error;
        }
    }
}

// one workgroup of 128 threads per chunk: 8 weights -> k bytes per thread; outliers of the
// chunk are appended to the shard's dictionary in offset order
template <int K>
__global__ __launch_bounds__(128) void pack_kernel(const float *w, const QuantState *st, const uint32_t *chunk_off,
                                                   int chunks_per_shard, uint64_t wsh, uint8_t *packed,
                                                   uint32_t *outlier_pos, float *outlier_val, uint32_t max_outliers)
{
    __shared__ uint32_t edges[kMaxClusters];
    __shared__ uint32_t wave_tot[2];
    constexpr int C = 1 << K;
    if (threadIdx.x < C - 1) edges[threadIdx.x] = st->edge_key[threadIdx.x];
    __syncthreads();
    const double mu = st->mu, r2 = st->r2;
    const int shard = blockIdx.x / chunks_per_shard, chunk = blockIdx.x - shard * chunks_per_shard;
    const uint64_t in_shard = (uint64_t)chunk * kChunk + threadIdx.x * 8;
    const float *src = w + (uint64_t)shard * wsh + in_shard;
    const f32x4 a = *(const f32x4 *)src, b = *(const f32x4 *)(src + 4);
    const float x[8] = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
    uint64_t bits = 0;
    uint32_t flags = 0, n_out = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const double d = (double)x[e] - mu;
        if (d * d > r2) { flags |= 1u << e; n_out += 1; }
        bits |= (uint64_t)cluster_of(order_key(x[e]), edges, C - 1) << (e * K);
    }
    uint8_t *dst = packed + ((uint64_t)shard * wsh + in_shard) / 8 * K;
#pragma unroll
    for (int j = 0; j < K; ++j) dst[j] = (uint8_t)(bits >> (8 * j));
    // position of this thread's outliers in the shard's dictionary
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = n_out;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_up(inc, o, 64);
        if (lane >= o) inc += t;
    }
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    uint32_t pos = chunk_off[blockIdx.x] + (wave ? wave_tot[0] : 0) + inc - n_out;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if (flags & (1u << e)) {
            if (pos < max_outliers) {
                outlier_pos[(uint64_t)shard * max_outliers + pos] = (uint32_t)(in_shard + e);
                outlier_val[(uint64_t)shard * max_outliers + pos] = x[e];
            }
            ++pos;
        }
    }
}

int moments_blocks(uint64_t n)
{
    const uint64_t b = (n + 256 * 16 - 1) / (256 * 16);
    return (int)(b < 1 ? 1 : (b > 2048 ? 2048 : b));
}

}  // namespace
}  // namespace sti

using namespace sti;

extern "C" {

size_t sti_quantize_workspace_bytes(const sti_dims *dims)
{
    if (!dims || dims->d_model <= 0 || dims->d_head <= 0 || dims->ffn_per_shard <= 0 || dims->n_heads <= 0 ||
        dims->n_heads > kMaxShardsPerLayer)
        return 0;
    const uint64_t wsh = (uint64_t)dims->d_model * (4 * (uint64_t)dims->d_head + 2 * (uint64_t)dims->ffn_per_shard);
    if (wsh % kChunk) return 0;
    const uint64_t n = wsh * dims->n_heads;
    return quant_layout((int64_t)(n / kChunk), moments_blocks(n)).total;
}

sti_status sti_quantize_layer(const sti_dims *dims, const float *weights, int bitwidth, double loglik_threshold,
                              double reg_covar, uint8_t *packed, float *codebook, uint32_t *outlier_pos,
                              float *outlier_val, uint32_t max_outliers_per_shard, uint32_t *outlier_count,
                              sti_quant_stats *stats, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!dims || !weights || !packed || !codebook || !outlier_count) return STI_ERR_NULL;
    if (max_outliers_per_shard > 0 && (!outlier_pos || !outlier_val)) return STI_ERR_NULL;
    if (!valid_packed_bits(bitwidth)) return STI_ERR_BITWIDTH;
    if (dims->d_model <= 0 || dims->d_head <= 0 || dims->ffn_per_shard <= 0 || dims->n_heads <= 0 ||
        dims->n_heads > kMaxShardsPerLayer)
        return STI_ERR_DIMS;
    if (!(reg_covar >= 0.0) || !(loglik_threshold == loglik_threshold)) return STI_ERR_DIMS;
    const uint64_t wsh = (uint64_t)dims->d_model * (4 * (uint64_t)dims->d_head + 2 * (uint64_t)dims->ffn_per_shard);
    if (wsh % kChunk) return STI_ERR_UNSUPPORTED;
    const int M = dims->n_heads;
    const uint64_t n = wsh * M;
    if (n / kChunk > 0x7FFFFFFFull) return STI_ERR_DIMS;
    if (!aligned(weights, 16) || !aligned(packed, 16) || !aligned(workspace, 256)) return STI_ERR_ALIGN;
    const int nb = moments_blocks(n);
    const int64_t n_chunks = (int64_t)(n / kChunk);
    const int chunks_per_shard = (int)(wsh / kChunk);
    const QuantLayout L = quant_layout(n_chunks, nb);
    if (!workspace || workspace_bytes < L.total) return STI_ERR_WORKSPACE;

    hipStream_t stream = (hipStream_t)hip_stream;
    uint8_t *ws = (uint8_t *)workspace;
    QuantState *st = (QuantState *)(ws + L.state);
    double *partials = (double *)(ws + L.partials);
    uint32_t *hist_hi = (uint32_t *)(ws + L.hist_hi), *hist_lo = (uint32_t *)(ws + L.hist_lo);
    uint8_t *bin_slot = ws + L.bin_slot;
    uint32_t *chunk_count = (uint32_t *)(ws + L.chunk_count), *chunk_off = (uint32_t *)(ws + L.chunk_off);
    double *csum = (double *)(ws + L.csum);
    uint32_t *ccount = (uint32_t *)(csum + (size_t)n_chunks * kMaxClusters);
    const int C = 1 << bitwidth;

    fill_zero_kernel<<<dim3(1024), dim3(256), 0, stream>>>((uint32_t *)(ws + L.zero_begin), (L.zero_end - L.zero_begin) / 4);
    moments_kernel<<<dim3(nb), dim3(256), 0, stream>>>(weights, n, partials);
    fit_kernel<<<dim3(1), dim3(256), 0, stream>>>(partials, nb, n, loglik_threshold, reg_covar, st);
    // fewer than 65536 weights per workgroup (16-bit private counters), at least one chunk group each
    int64_t classify_groups = (n_chunks + 3) / 4;
    int64_t classify_grid = classify_groups < 512 ? classify_groups : 512;
    while ((classify_groups + classify_grid - 1) / classify_grid * 4 * kChunk >= 65536) classify_grid *= 2;
    classify_kernel<<<dim3((uint32_t)classify_grid), dim3(1024), 0, stream>>>(weights, st, n_chunks, hist_hi, chunk_count);
    select_bins_kernel<<<dim3(1), dim3(1024), 0, stream>>>(st, hist_hi, bin_slot, chunk_count, chunk_off, M,
                                                           chunks_per_shard, C, outlier_count);
    hist_lo_kernel<<<dim3((uint32_t)n_chunks), dim3(256), 0, stream>>>(weights, st, bin_slot, hist_lo);
    select_values_kernel<<<dim3(C - 1), dim3(1024), 0, stream>>>(st, bin_slot, hist_lo);
    cluster_sums_kernel<<<dim3((uint32_t)n_chunks), dim3(256), 0, stream>>>(weights, st, C, csum, ccount);
    centroids_kernel<<<dim3(C), dim3(1024), 0, stream>>>(st, csum, ccount, n_chunks, codebook, stats);
    const dim3 pg((uint32_t)n_chunks), pb(128);
    switch (bitwidth) {
    case 2: pack_kernel<2><<<pg, pb, 0, stream>>>(weights, st, chunk_off, chunks_per_shard, wsh, packed, outlier_pos, outlier_val, max_outliers_per_shard); break;
    case 3: pack_kernel<3><<<pg, pb, 0, stream>>>(weights, st, chunk_off, chunks_per_shard, wsh, packed, outlier_pos, outlier_val, max_outliers_per_shard); break;
    case 4: pack_kernel<4><<<pg, pb, 0, stream>>>(weights, st, chunk_off, chunks_per_shard, wsh, packed, outlier_pos, outlier_val, max_outliers_per_shard); break;
    case 5: pack_kernel<5><<<pg, pb, 0, stream>>>(weights, st, chunk_off, chunks_per_shard, wsh, packed, outlier_pos, outlier_val, max_outliers_per_shard); break;
    default: pack_kernel<6><<<pg, pb, 0, stream>>>(weights, st, chunk_off, chunks_per_shard, wsh, packed, outlier_pos, outlier_val, max_outliers_per_shard); break;
    }
    STI_TRY(hipGetLastError());
    return STI_OK;
}

}  // extern "C"
