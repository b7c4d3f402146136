// C ABI of libsti: argument validation, shard-table staging, kernel sequencing.
// Every check runs before the first launch; device work goes to the caller's stream.
#include <mutex>
#include <new>
#include <string.h>
#include <vector>

#include "sti_internal.hpp"
#include "api_internal.hpp"

namespace sti {


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

// Optional per-launch timing: while enabled, every kernel launch of the entry points carries
// two events that hold the dispatch's begin and end time stamps (see launch() in
// sti_internal.hpp); sti_profile_end() sums them per class.
class Profiler {
public:
    bool enabled() const { return on_; }
    hipError_t begin()
    {
        std::lock_guard<std::mutex> lock(mu_);
        used_ = 0;
        on_ = true;
        return hipSuccess;
    }
    // events for the next launch of class `cls` (nulls when timing is off)
    hipError_t next(int cls, LaunchEvents *ev)
    {
        std::lock_guard<std::mutex> lock(mu_);
        *ev = LaunchEvents{};
        if (!on_) return hipSuccess;
        if (used_ == recs_.size()) {
            Rec r;
            hipError_t e = hipEventCreate(&r.a);
            if (e != hipSuccess) return e;
            e = hipEventCreate(&r.b);
            if (e != hipSuccess) return e;
            recs_.push_back(r);
        }
        recs_[used_].cls = cls;
        ev->start = recs_[used_].a;
        ev->stop = recs_[used_].b;
        return hipSuccess;
    }
    // the launch took the events: count it
    void commit()
    {
        std::lock_guard<std::mutex> lock(mu_);
        if (on_ && used_ < recs_.size()) ++used_;
    }
    hipError_t end(sti_profile *out)
    {
        std::lock_guard<std::mutex> lock(mu_);
        on_ = false;
        memset(out, 0, sizeof(*out));
        for (size_t i = 0; i < used_; ++i) {
            hipError_t e = hipEventSynchronize(recs_[i].b);
            if (e != hipSuccess) return e;
            float ms = 0.f;
            e = hipEventElapsedTime(&ms, recs_[i].a, recs_[i].b);
            if (e != hipSuccess) return e;
            out->launches[recs_[i].cls] += 1;
            out->ms[recs_[i].cls] += ms;
        }
        used_ = 0;
        return hipSuccess;
    }

private:
    struct Rec {
        hipEvent_t a = nullptr, b = nullptr;
        int cls = 0;
    };
    std::mutex mu_;
    std::vector<Rec> recs_;
    size_t used_ = 0;
    bool on_ = false;
};

Profiler &profiler()
{
    static Profiler p;
    return p;
}

thread_local LaunchEvents pending_launch_events;

// Run `fn` (one kernel launch through launch(); returns hipError_t) with timing events when enabled.
template <typename F>
hipError_t timed(int cls, hipStream_t stream, F fn)
{
    (void)stream;
    Profiler &pr = profiler();
    if (!pr.enabled()) return fn();
    hipError_t e = pr.next(cls, &pending_launch_events);
    if (e != hipSuccess) return e;
    e = fn();
    if (pending_launch_events.start == nullptr) pr.commit();   // taken by the launch
    pending_launch_events = LaunchEvents{};                      // (nothing was launched: dropped)
    return e;
}

LaunchEvents take_launch_events()
{
    const LaunchEvents ev = pending_launch_events;
    pending_launch_events = LaunchEvents{};
    return ev;
}

// Whether `stream` is recording a graph.  The staging ring (a pinned slot that later calls
// overwrite, an event the host waits on) must not be recorded: a replay would read whatever
// table the slot holds by then.
inline hipError_t stream_is_capturing(hipStream_t stream, bool *capturing)
{
    hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
    const hipError_t e = hipStreamIsCapturing(stream, &status);
    *capturing = (status != hipStreamCaptureStatusNone);
    return e;
}

inline ShardDesc make_desc(const sti_shard &s, int tag)
{
    return ShardDesc{s.data, s.codebook, s.bitwidth, tag, s.outlier_pos, s.outlier_val, s.n_outliers, 0};
}

sti_status check_decode_shard(const sti_shard &s)
{
    const int b = s.bitwidth;
    if (b != 32 && !valid_packed_bits(b)) return STI_ERR_BITWIDTH;
    if (!s.data) return STI_ERR_MISSING_SHARD;
    if (b != 32 && !s.codebook) return STI_ERR_MISSING_SHARD;
    if (b == 32 && s.n_outliers != 0) return STI_ERR_UNSUPPORTED;   // raw shards have no dictionary
    if (s.n_outliers != 0 && (!s.outlier_pos || !s.outlier_val)) return STI_ERR_NULL;
    if (s.n_outliers != 0 && (!aligned(s.outlier_pos, 4) || !aligned(s.outlier_val, 4))) return STI_ERR_ALIGN;
    if (!aligned(s.data, 16)) return STI_ERR_ALIGN;
    if (b != 32 && !aligned(s.codebook, 4)) return STI_ERR_ALIGN;
    return STI_OK;
}


// ---------------------------------------------------------------------------
// Layer sequencing
// ---------------------------------------------------------------------------


// Offsets of the scratch regions of one layer call (sized for all M shards present).
WorkspaceLayout workspace_layout(const sti_dims &d, int64_t T, sti_precision prec, int model_layers)
{
    WorkspaceLayout L;
    const size_t es = (prec == STI_PREC_F32) ? 4 : 2;
    const size_t M = d.n_heads, dm = d.d_model, dh = d.d_head, f = d.ffn_per_shard;
    if (prec != STI_PREC_F32 && model_layers > 1) {
        // Layers are decompressed in groups, each group right before its first layer: working
        // buffers written shortly before they are read are still in the memory-side cache (the
        // FFN2 projection measured 7 % faster than with one launch for the whole model up front),
        // while one launch per layer is too short to keep HBM busy.  A group is as many layers as
        // fit 64 MiB of working buffers (4 layers of BERT-base).
        const size_t layer_w16_bytes = M * dm * (4 * dh + 2 * f) * 2;
        size_t group = ((size_t)64 << 20) / (layer_w16_bytes ? layer_w16_bytes : 1);
        if (group < 1) group = 1;
        if (group > (size_t)model_layers) group = (size_t)model_layers;
        L.decode_group = (int)group;
        L.w16_layers = (int)(group < 2 ? 2 : group);
    }
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    };
    if (prec == STI_PREC_F32) L.w32 = take(M * dm * (4 * dh + 2 * f) * 4);
    else L.w16 = take((size_t)L.w16_layers * M * dm * (4 * dh + 2 * f) * 2);
    L.act[0] = take((size_t)T * dm * es);
    L.act[1] = take((size_t)T * dm * es);
    L.qkv = take((size_t)T * M * 3 * dh * es);
    L.ctx = take((size_t)T * M * dh * es);
    {   // float32 sums before LayerNorm; the few-token GEMM may leave several partial sums
        size_t rows = (size_t)T;
        if (prec != STI_PREC_F32 && T <= kSkinnyMaxTokens) rows *= kSkinnyMaxSplits;
        if (prec != STI_PREC_F32) {   // ... and so may the wide-tile GEMM when it has few tiles
            const size_t wide_rows = (size_t)T * gemm_wide_max_k_splits(T, (int)dm);
            if (wide_rows > rows) rows = wide_rows;
        }
        L.pre = take(rows * dm * 4);
    }
    L.h = take((size_t)T * dm * es);
    L.u = take((size_t)T * M * f * es);
    if (L.w16_layers > 1) L.table = take((size_t)model_layers * M * sizeof(ShardDesc));
    L.total = off;
    return L;
}

sti_status check_dims(const sti_dims *dims, int batch, int seq, sti_precision prec)
{
    if (!dims) return STI_ERR_NULL;
    if (prec != STI_PREC_F32 && prec != STI_PREC_F16_MFMA) return STI_ERR_DTYPE;
    if (dims->d_model <= 0 || dims->d_head <= 0 || dims->ffn_per_shard <= 0) return STI_ERR_DIMS;
    if (dims->n_heads <= 0 || dims->n_heads > kMaxShardsPerLayer) return STI_ERR_DIMS;
    if (!(dims->ln_eps >= 0.0f)) return STI_ERR_DIMS;
    if (batch < 0 || seq < 0) return STI_ERR_DIMS;
    if (dims->d_model > (1 << 16) || dims->d_head > (1 << 12) || dims->ffn_per_shard > (1 << 16))
        return STI_ERR_DIMS;
    if ((int64_t)batch * seq > (1 << 24) || batch > 65535) return STI_ERR_DIMS;
    if (prec == STI_PREC_F32) {
        // the float32 attention kernel keeps one score row per wave in LDS
        if ((size_t)4 * ((size_t)seq + dims->d_head) * 4 > 65536) return STI_ERR_DIMS;
    } else {
        if (dims->d_model % 64 || dims->ffn_per_shard % 64) return STI_ERR_DIMS;
        if (dims->d_head != 64) return STI_ERR_DIMS;
        if (seq > 512) return STI_ERR_DIMS;
    }
    return STI_OK;
}

sti_status check_layer_shard(const sti_shard &s)
{
    if (s.bitwidth == 0) return STI_OK;
    return check_decode_shard(s);
}

sti_status check_params(const sti_layer_params *p)
{
    if (!p) return STI_ERR_NULL;
    const float *all[10] = {p->bq, p->bk, p->bv, p->bo, p->b1, p->b2,
                            p->ln1_g, p->ln1_b, p->ln2_g, p->ln2_b};
    for (const float *q : all) {
        if (!q) return STI_ERR_NULL;
        if (!aligned(q, 4)) return STI_ERR_ALIGN;
    }
    return STI_OK;
}

inline const void *block_start(const sti_shard &s, size_t elem_off)
{
    if (s.bitwidth == 32) return (const float *)s.data + elem_off;
    return (const uint8_t *)s.data + elem_off * (size_t)s.bitwidth / 8;
}

// From this many tokens on, a layer's shards are decompressed once into the binary16
// working buffer; below it, the GEMMs decode the streams themselves (every weight is then
// used by at most a few row tiles).
// Which GEMM family a matrix-core layer takes.  The few-token kernels decode every weight
// once per 64-row block and take partial sums through LayerNorm; from a couple of row blocks
// on it is cheaper to decompress the layer once into the working buffer and run the
// wide-tile kernels (measured per layer, BERT-base with 9 of 12 shards: 128 tokens 57 against
// 69 us, 192 tokens 60 against 63, 256 tokens 68 against 65, 384 tokens 164 -- with the
// decode fused into a tiled GEMM, as used before -- against 70; d_model 1024, 12 of 16 shards:
// 192 tokens 82 against 76, 256 tokens 92 against 77).
inline bool few_token_path(const sti_dims &d, int64_t T)
{
    return T <= 128 || (T <= 192 && d.d_model <= 768);
}
static_assert(kSkinnyMaxTokens >= 192, "the partial-sum planes are sized with kSkinnyMaxTokens");


// One layer, arguments already validated.  `in` is float32 (F32 precision) or
// binary16 (MFMA precision); `out` is written as out_dtype.
int spare_decode_workgroups(const sti_dims &d, int B, int Lseq, int m, sti_precision prec)
{
    if (prec != STI_PREC_F16_MFMA || m <= 0 || few_token_path(d, (int64_t)B * Lseq)) return 0;
    GemmProblem p;
    memset(&p, 0, sizeof(p));
    p.kind = gemm_wide_fuses_attention(B, Lseq, m, d.d_head) ? GEMM_QKV_ATTN : GEMM_QKV;
    p.T = B * Lseq; p.n_blocks = m; p.block_rows = 3 * d.d_head; p.block_cols = d.d_model;
    return gemm_wide_spare_workgroups(p);
}

sti_status run_layer(const sti_dims &d, const sti_shard *shards, const sti_layer_params &prm,
                     const void *in, void *out, sti_dtype out_dtype, int B, int Lseq,
                     sti_precision prec, uint8_t *ws, const WorkspaceLayout &wl, hipStream_t stream,
                     const void *predecoded, const int32_t *key_lengths, const NextLayerDecode *next)
{
    const int dm = d.d_model, M = d.n_heads, dh = d.d_head, f = d.ffn_per_shard;
    const int T = B * Lseq;
    if (T == 0) return STI_OK;
    const size_t wsh = (size_t)dm * (4 * dh + 2 * f);
    const size_t off_o = (size_t)3 * dh * dm, off_1 = (size_t)4 * dh * dm,
                 off_2 = (size_t)4 * dh * dm + (size_t)f * dm;
    int present[kMaxShardsPerLayer];
    int m = 0;
    for (int i = 0; i < M; ++i)
        if (shards[i].bitwidth != 0) present[m++] = i;

    GemmBlocks bq, bo, b1, b2;
    memset(&bq, 0, sizeof(bq)); memset(&bo, 0, sizeof(bo));
    memset(&b1, 0, sizeof(b1)); memset(&b2, 0, sizeof(b2));
    const bool f32 = (prec == STI_PREC_F32);
    // MFMA path: with many row tiles per weight it is cheaper to decompress the layer
    // once into a binary16 working buffer than to decode inside every row tile
    uint32_t max_outliers = 0;
    for (int p = 0; p < m; ++p)
        if (shards[present[p]].n_outliers > max_outliers) max_outliers = shards[present[p]].n_outliers;
    // shards with an outlier dictionary always go through the working buffer, where the
    // outliers are scattered back after the substitution pass
    const bool predecode = !f32 && m > 0 && (predecoded || !few_token_path(d, T) || max_outliers > 0);
    const _Float16 *w16 = predecoded ? (const _Float16 *)predecoded : (const _Float16 *)(ws + wl.w16);
    if (predecode && !predecoded) {
        InlineShardTable t;
        memset(&t, 0, sizeof(t));
        for (int p = 0; p < m; ++p) {
            const sti_shard &s = shards[present[p]];
            t.d[p] = make_desc(s, present[p]);
        }
        STI_TRY(timed(STI_K_DECODE, stream, [&] { return launch_decode_tiled(t, m, dm, dh, f, ws + wl.w16, stream); }));
        STI_TRY(launch_patch_outliers_tiled(t, m, max_outliers, dm, dh, f, ws + wl.w16, stream));
    }
    if (f32 && m > 0) {
        InlineShardTable t;
        memset(&t, 0, sizeof(t));
        for (int p = 0; p < m; ++p) {
            const sti_shard &s = shards[present[p]];
            t.d[p] = make_desc(s, present[p]);
        }
        STI_TRY(timed(STI_K_DECODE, stream, [&] { return launch_decode(nullptr, &t, m, wsh, ws + wl.w32, STI_F32, stream); }));
        STI_TRY(launch_patch_outliers(nullptr, &t, m, max_outliers, wsh, ws + wl.w32, STI_F32, stream));
    }
    for (int p = 0; p < m; ++p) {
        const sti_shard &s = shards[present[p]];
        if (f32) {
            const float *w = (const float *)(ws + wl.w32) + (size_t)p * wsh;
            bq.b[p] = GemmBlock{w, nullptr, 32, present[p]};
            bo.b[p] = GemmBlock{w + off_o, nullptr, 32, present[p]};
            b1.b[p] = GemmBlock{w + off_1, nullptr, 32, present[p]};
            b2.b[p] = GemmBlock{w + off_2, nullptr, 32, present[p]};
        } else if (predecode) {
            const _Float16 *w = w16 + (size_t)p * wsh;
            bq.b[p] = GemmBlock{w, nullptr, 17, present[p]};
            bo.b[p] = GemmBlock{w + off_o, nullptr, 17, present[p]};
            b1.b[p] = GemmBlock{w + off_1, nullptr, 17, present[p]};
            b2.b[p] = GemmBlock{w + off_2, nullptr, 17, present[p]};
        } else {
            bq.b[p] = GemmBlock{block_start(s, 0), s.codebook, s.bitwidth, present[p]};
            bo.b[p] = GemmBlock{block_start(s, off_o), s.codebook, s.bitwidth, present[p]};
            b1.b[p] = GemmBlock{block_start(s, off_1), s.codebook, s.bitwidth, present[p]};
            b2.b[p] = GemmBlock{block_start(s, off_2), s.codebook, s.bitwidth, present[p]};
        }
    }
    void *qkv = ws + wl.qkv, *ctx = ws + wl.ctx, *h = ws + wl.h, *u = ws + wl.u;
    float *pre = (float *)(ws + wl.pre);
    const sti_dtype act_dtype = f32 ? STI_F32 : STI_F16;
    // (a layer with every shard absent has nothing to multiply: on the matrix-core path its two
    //  LayerNorms run alone, over bias + residual, like those behind the few-token kernels)
    const bool skinny = !f32 && (few_token_path(d, T) || m == 0);
    const bool no_products = !f32 && m == 0;
    const int64_t partial_stride = (int64_t)T * dm;
    int pre_partials = 1;   // partial sums the last K-split GEMM left in `pre`
    auto gemm = [&](const GemmProblem &p, const GemmBlocks &blk) {
        static const int cls[5] = {STI_K_GEMM_QKV, STI_K_GEMM_FFN_UP, STI_K_GEMM_OUT,
                                   STI_K_GEMM_FFN_DOWN, STI_K_GEMM_QKV};
        return timed(cls[p.kind], stream, [&] {
            if (f32) return launch_gemm_f32(p, blk, stream);
            if (!skinny) {
                GemmProblem q = p;
                if (p.kind == GEMM_OUT || p.kind == GEMM_FFN_DOWN) {
                    q.k_splits = gemm_wide_k_splits(p);
                    q.partial_stride = partial_stride;
                    pre_partials = q.k_splits;
                }
                return launch_gemm_wide(q, blk, stream);
            }
            const int splits = skinny_k_splits(p);
            if (p.kind == GEMM_OUT || p.kind == GEMM_FFN_DOWN) pre_partials = splits;
            return launch_gemm_skinny(p, blk, splits, partial_stride, stream);
        });
    };
    // the MFMA GEMMs leave bias and residual to the LayerNorm kernel
    auto layernorm = [&](void *dst, sti_dtype dt, const float *g, const float *b,
                         const float *bias, const void *resid) {
        return timed(STI_K_LAYERNORM, stream, [&] {
            if (!f32 && !skinny && pre_partials == 1)   // the wide MFMA GEMM already added bias and residual
                return launch_layernorm_f16in(pre, dst, dt, g, b, T, dm, d.ln_eps, stream);
            return launch_layernorm(pre, pre_partials, partial_stride, f32 ? nullptr : bias,
                                    f32 ? nullptr : resid, dst, dt, g, b, T, dm, d.ln_eps, stream);
        });
    };

    GemmProblem p;
    if (m > 0) {
        memset(&p, 0, sizeof(p));
        p.kind = GEMM_QKV; p.T = T; p.n_blocks = m; p.block_rows = 3 * dh; p.block_cols = dm;
        p.d_head = dh; p.A = in; p.lda = dm; p.C = qkv; p.ldc = m * 3 * dh;
        p.bias0 = prm.bq; p.bias1 = prm.bk; p.bias2 = prm.bv;
        if (!f32 && !skinny && gemm_wide_fuses_attention(B, Lseq, m, dh)) {
            // sequences of 128 tokens: the projection's 128-row tiles are whole sequences, and its
            // workgroups go on to the attention of the heads they hold (no Q/K/V buffer)
            p.kind = GEMM_QKV_ATTN; p.C = ctx; p.ldc = m * dh; p.key_lengths = key_lengths;
            if (next && next->workgroups > 0 && next->n_shards > 0) {
                p.next_table = next->table; p.next_shards = next->n_shards; p.next_out = next->out;
                p.next_workgroups = next->workgroups; p.next_ffn_per_shard = f;
            }
            STI_TRY(gemm(p, bq));
        } else {
            if (next && next->workgroups > 0 && next->n_shards > 0) {
                if (f32 || skinny) return STI_ERR_UNSUPPORTED;   // (the caller asked spare_decode_workgroups first)
                p.next_table = next->table; p.next_shards = next->n_shards; p.next_out = next->out;
                p.next_workgroups = next->workgroups; p.next_ffn_per_shard = f;
            }
            STI_TRY(gemm(p, bq));
            STI_TRY(timed(STI_K_ATTENTION, stream, [&] {
                return f32 ? launch_attention_f32((const float *)qkv, (float *)ctx, B, Lseq, m, dh, key_lengths, stream)
                           : launch_attention_mfma(qkv, ctx, B, Lseq, m, dh, key_lengths, stream);
            }));
        }
    }
    memset(&p, 0, sizeof(p));
    p.kind = GEMM_OUT; p.T = T; p.n_blocks = m; p.block_rows = dm; p.block_cols = dh; p.d_head = dh;
    p.A = ctx; p.lda = m * dh; p.C = pre; p.ldc = dm; p.bias0 = prm.bo; p.resid = in; p.ldr = dm;
    if (no_products) pre_partials = 0;
    else STI_TRY(gemm(p, bo));
    STI_TRY(layernorm(h, act_dtype, prm.ln1_g, prm.ln1_b, prm.bo, in));
    if (m > 0) {
        memset(&p, 0, sizeof(p));
        p.kind = GEMM_FFN_UP; p.T = T; p.n_blocks = m; p.block_rows = f; p.block_cols = dm;
        p.d_head = dh; p.A = h; p.lda = dm; p.C = u; p.ldc = m * f; p.bias0 = prm.b1;
        STI_TRY(gemm(p, b1));
    }
    memset(&p, 0, sizeof(p));
    p.kind = GEMM_FFN_DOWN; p.T = T; p.n_blocks = m; p.block_rows = dm; p.block_cols = f;
    p.d_head = dh; p.A = u; p.lda = m * f; p.C = pre; p.ldc = dm; p.bias0 = prm.b2; p.resid = h;
    p.ldr = dm;
    if (no_products) pre_partials = 0;
    else STI_TRY(gemm(p, b2));
    STI_TRY(layernorm(out, out_dtype, prm.ln2_g, prm.ln2_b, prm.b2, h));
    return STI_OK;
}

sti_status check_io(const void *x, void *y, sti_dtype io, int64_t T, int d)
{
    if (io != STI_F32 && io != STI_F16 && io != STI_BF16) return STI_ERR_DTYPE;
    if (T == 0) return STI_OK;
    if (!x || !y) return STI_ERR_NULL;
    if (!aligned(x, 16) || !aligned(y, 16)) return STI_ERR_ALIGN;
    const size_t bytes = (size_t)T * d * (io == STI_F32 ? 4 : 2);
    const uintptr_t a = (uintptr_t)x, b = (uintptr_t)y;
    if (a < b + bytes && b < a + bytes) return STI_ERR_DIMS;  // x and y overlap
    return STI_OK;
}

sti_status check_key_lengths(const int32_t *key_lengths)
{
    if (!key_lengths) return STI_ERR_NULL;
    return aligned(key_lengths, 4) ? STI_OK : STI_ERR_ALIGN;
}

}  // namespace sti

using namespace sti;

namespace {

// Scratch memory of sti_layer_forward_static: what sti_layer_forward takes as `workspace`
// (working buffer, projections' outputs, partial sums), for callers that cannot allocate.
// One copy per GPU, at an address of its own on each, held until the process ends.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on the current device, looked up once per device (in host code
// the array's name is only a handle for this lookup, never an address a kernel may use).
hipError_t static_scratch(uint8_t **out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static uint8_t *per_device[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!per_device[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        per_device[dev] = (uint8_t *)ptr;
    }
    *out = per_device[dev];
    return hipSuccess;
}

// masked: the call came through a *_masked entry point and key_lengths must be usable
sti_status layer_forward(const sti_dims *dims, const sti_shard *shards,
                         const sti_layer_params *params, const void *x, void *y,
                         sti_dtype io_dtype, int batch, int seq, bool masked, const int32_t *key_lengths,
                         sti_precision precision, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    sti_status st = check_dims(dims, batch, seq, precision);
    if (st != STI_OK) return st;
    if (!shards) return STI_ERR_NULL;
    st = check_params(params);
    if (st != STI_OK) return st;
    const int64_t T = (int64_t)batch * seq;
    st = check_io(x, y, io_dtype, T, dims->d_model);
    if (st != STI_OK) return st;
    if (masked && T > 0) {
        st = check_key_lengths(key_lengths);
        if (st != STI_OK) return st;
    }
    for (int i = 0; i < dims->n_heads; ++i) {
        st = check_layer_shard(shards[i]);
        if (st != STI_OK) return st;
    }
    const WorkspaceLayout wl = workspace_layout(*dims, T, precision);
    if (!workspace || workspace_bytes < wl.total) return STI_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return STI_ERR_ALIGN;
    if (T == 0) return STI_OK;

    hipStream_t stream = (hipStream_t)hip_stream;
    uint8_t *ws = (uint8_t *)workspace;
    const sti_dtype act = (precision == STI_PREC_F32) ? STI_F32 : STI_F16;
    const void *in = x;
    if (io_dtype != act) {
        STI_TRY(timed(STI_K_CONVERT, stream, [&] { return launch_convert(x, io_dtype, ws + wl.act[0], act, (uint64_t)T * dims->d_model, stream); }));
        in = ws + wl.act[0];
    }
    return run_layer(*dims, shards, *params, in, y, io_dtype, batch, seq, precision, ws, wl, stream,
                     nullptr, masked ? key_lengths : nullptr);
}

sti_status model_forward(const sti_dims *dims, int n_layers, const sti_shard *store,
                         const sti_layer_params *params, const int8_t *plan, const void *x,
                         void *y, sti_dtype io_dtype, int batch, int seq, bool masked,
                         const int32_t *key_lengths, sti_precision precision, void *workspace,
                         size_t workspace_bytes, void *hip_stream);

}  // namespace

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
    hipStream_t stream = (hipStream_t)hip_stream;
    hipError_t e;
    if (need) {
        if (!workspace || workspace_bytes < need) return STI_ERR_WORKSPACE;
        if (!aligned(workspace, 16)) return STI_ERR_ALIGN;
        // the table of a large call is uploaded through the staging ring: not under capture
        bool capturing = false;
        if (stream_is_capturing(stream, &capturing) != hipSuccess) return STI_ERR_HIP;
        if (capturing) return STI_ERR_UNSUPPORTED;
    }
    if (weights_per_shard == 0) return STI_OK;

    uint32_t max_outliers = 0;
    for (int s = 0; s < n_shards; ++s)
        if (shards[s].n_outliers > max_outliers) max_outliers = shards[s].n_outliers;
    if (need) {
        std::vector<ShardDesc> table;
        try {
            table.resize(n_shards);
        } catch (const std::bad_alloc &) {
            return STI_ERR_HIP;
        }
        for (int s = 0; s < n_shards; ++s)
            table[s] = make_desc(shards[s], s);
        e = staging().upload(table.data(), table.size(), workspace, stream);
        if (e != hipSuccess) return STI_ERR_HIP;
        e = timed(STI_K_DECODE, stream, [&] {
            return launch_decode((const ShardDesc *)workspace, nullptr, n_shards, weights_per_shard,
                                 out, out_dtype, stream);
        });
        if (e == hipSuccess)
            e = launch_patch_outliers((const ShardDesc *)workspace, nullptr, n_shards, max_outliers,
                                      weights_per_shard, out, out_dtype, stream);
    } else {
        InlineShardTable t;
        memset(&t, 0, sizeof(t));
        for (int s = 0; s < n_shards; ++s)
            t.d[s] = make_desc(shards[s], s);
        e = timed(STI_K_DECODE, stream, [&] {
            return launch_decode(nullptr, &t, n_shards, weights_per_shard, out, out_dtype, stream);
        });
        if (e == hipSuccess)
            e = launch_patch_outliers(nullptr, &t, n_shards, max_outliers, weights_per_shard, out,
                                      out_dtype, stream);
    }
    return e == hipSuccess ? STI_OK : STI_ERR_HIP;
}

size_t sti_working_buffer_bytes(const sti_dims *dims)
{
    if (check_dims(dims, 0, 0, STI_PREC_F16_MFMA) != STI_OK) return 0;
    return (size_t)dims->n_heads * dims->d_model * (4 * (size_t)dims->d_head + 2 * (size_t)dims->ffn_per_shard) * 2;
}

int64_t sti_working_buffer_offset(const sti_dims *dims, uint64_t j)
{
    if (check_dims(dims, 0, 0, STI_PREC_F16_MFMA) != STI_OK) return -1;
    const uint64_t d = dims->d_model, dh = dims->d_head, f = dims->ffn_per_shard;
    if (j >= d * (4 * dh + 2 * f)) return -1;
    const uint64_t o_o = 3 * dh * d, o_1 = 4 * dh * d, o_2 = o_1 + f * d;
    uint64_t sub, cols;
    if (j < o_o) { sub = 0; cols = d; }
    else if (j < o_1) { sub = o_o; cols = dh; }
    else if (j < o_2) { sub = o_1; cols = d; }
    else { sub = o_2; cols = f; }
    const uint64_t row = (j - sub) / cols, col = (j - sub) % cols;
    const uint64_t cell = (row / 32) * (cols / 64) + col / 64;
    const uint64_t lane = ((col % 64) / 32) * 32 + row % 32, q = (col % 32) / 8;
    return (int64_t)(sub + cell * 2048 + q * 512 + lane * 8 + col % 8);
}

sti_status sti_decode_working_buffer(const sti_dims *dims, const sti_shard *shards, void *out,
                                     size_t out_bytes, void *hip_stream)
{
    sti_status st = check_dims(dims, 0, 0, STI_PREC_F16_MFMA);
    if (st != STI_OK) return st;
    if (!shards) return STI_ERR_NULL;
    const int M = dims->n_heads;
    InlineShardTable t;
    memset(&t, 0, sizeof(t));
    int m = 0;
    uint32_t max_outliers = 0;
    for (int i = 0; i < M; ++i) {
        st = check_layer_shard(shards[i]);
        if (st != STI_OK) return st;
        if (shards[i].bitwidth == 0) continue;
        if (shards[i].n_outliers > max_outliers) max_outliers = shards[i].n_outliers;
        t.d[m++] = make_desc(shards[i], i);
    }
    if (m == 0) return STI_OK;
    const size_t wsh = (size_t)dims->d_model * (4 * (size_t)dims->d_head + 2 * (size_t)dims->ffn_per_shard);
    if (!out) return STI_ERR_NULL;
    if (out_bytes < (size_t)m * wsh * 2) return STI_ERR_WORKSPACE;
    if (!aligned(out, 256)) return STI_ERR_ALIGN;
    hipStream_t stream = (hipStream_t)hip_stream;
    STI_TRY(timed(STI_K_DECODE, stream, [&] {
        return launch_decode_tiled(t, m, dims->d_model, dims->d_head, dims->ffn_per_shard, out, stream);
    }));
    STI_TRY(launch_patch_outliers_tiled(t, m, max_outliers, dims->d_model, dims->d_head, dims->ffn_per_shard,
                                        out, stream));
    return STI_OK;
}

size_t sti_workspace_bytes(const sti_dims *dims, int batch, int seq, sti_precision precision)
{
    if (check_dims(dims, batch, seq, precision) != STI_OK) return 0;
    size_t t = workspace_layout(*dims, (int64_t)batch * seq, precision).total;
    return t ? t : 256;
}

sti_status sti_layer_forward(const sti_dims *dims, const sti_shard *shards,
                             const sti_layer_params *params, const void *x, void *y,
                             sti_dtype io_dtype, int batch, int seq, sti_precision precision,
                             void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return layer_forward(dims, shards, params, x, y, io_dtype, batch, seq, false, nullptr, precision,
                         workspace, workspace_bytes, hip_stream);
}

sti_status sti_layer_forward_static(const sti_dims *dims, const sti_shard *shards,
                                    const sti_layer_params *params, const void *x, void *y,
                                    sti_dtype io_dtype, int batch, int seq, sti_precision precision,
                                    void *hip_stream)
{
    // everything that can be refused is refused before the scratch array is looked at
    sti_status st = check_dims(dims, batch, seq, precision);
    if (st != STI_OK) return st;
    const size_t need = workspace_layout(*dims, (int64_t)batch * seq, precision).total;
    if (need > kStaticScratchBytes) return STI_ERR_WORKSPACE;
    uint8_t *scratch_ptr = nullptr;
    if (static_scratch(&scratch_ptr) != hipSuccess) return STI_ERR_HIP;
    return layer_forward(dims, shards, params, x, y, io_dtype, batch, seq, false, nullptr, precision,
                         scratch_ptr, kStaticScratchBytes, hip_stream);
}

size_t sti_static_scratch_bytes(void) { return kStaticScratchBytes; }

sti_status sti_layer_forward_masked(const sti_dims *dims, const sti_shard *shards,
                                    const sti_layer_params *params, const void *x, void *y,
                                    sti_dtype io_dtype, int batch, int seq, const int32_t *key_lengths,
                                    sti_precision precision, void *workspace, size_t workspace_bytes,
                                    void *hip_stream)
{
    return layer_forward(dims, shards, params, x, y, io_dtype, batch, seq, true, key_lengths, precision,
                         workspace, workspace_bytes, hip_stream);
}

sti_status sti_model_forward(const sti_dims *dims, int n_layers, const sti_shard *store,
                             const sti_layer_params *params, const int8_t *plan, const void *x,
                             void *y, sti_dtype io_dtype, int batch, int seq,
                             sti_precision precision, void *workspace, size_t workspace_bytes,
                             void *hip_stream)
{
    return model_forward(dims, n_layers, store, params, plan, x, y, io_dtype, batch, seq, false, nullptr,
                         precision, workspace, workspace_bytes, hip_stream);
}

sti_status sti_model_forward_masked(const sti_dims *dims, int n_layers, const sti_shard *store,
                                    const sti_layer_params *params, const int8_t *plan, const void *x,
                                    void *y, sti_dtype io_dtype, int batch, int seq,
                                    const int32_t *key_lengths, sti_precision precision, void *workspace,
                                    size_t workspace_bytes, void *hip_stream)
{
    return model_forward(dims, n_layers, store, params, plan, x, y, io_dtype, batch, seq, true, key_lengths,
                         precision, workspace, workspace_bytes, hip_stream);
}

}  // extern "C"

namespace {

sti_status model_forward(const sti_dims *dims, int n_layers, const sti_shard *store,
                         const sti_layer_params *params, const int8_t *plan, const void *x,
                         void *y, sti_dtype io_dtype, int batch, int seq, bool masked,
                         const int32_t *key_lengths, sti_precision precision, void *workspace,
                         size_t workspace_bytes, void *hip_stream)
{
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
            st = check_decode_shard(v);
            if (st != STI_OK) return st;
            c = v;
        }
    }
    // With room for every layer's working buffer (sti_model_workspace_bytes) the model is
    // decompressed a few layers per launch (below); otherwise each layer decompresses into the
    // one buffer just before it runs.
    WorkspaceLayout wl = workspace_layout(*dims, T, precision);
    hipStream_t stream = (hipStream_t)hip_stream;
    // (under stream capture the grouped route, whose shard table goes through the staging
    //  ring, is not taken: the per-layer route records kernel launches only)
    bool whole_model_fits =
        precision == STI_PREC_F16_MFMA && !few_token_path(*dims, T) && n_layers > 1 && workspace &&
        aligned(workspace, 256) && workspace_bytes >= workspace_layout(*dims, T, precision, n_layers).total;
    if (whole_model_fits) {
        bool capturing = false;
        if (stream_is_capturing(stream, &capturing) != hipSuccess) return STI_ERR_HIP;
        if (capturing) whole_model_fits = false;
    }
    if (whole_model_fits) wl = workspace_layout(*dims, T, precision, n_layers);
    if (!workspace || workspace_bytes < wl.total) return STI_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return STI_ERR_ALIGN;
    if (T == 0) return STI_OK;

    uint8_t *ws = (uint8_t *)workspace;
    const size_t io_bytes = (size_t)T * dims->d_model * (io_dtype == STI_F32 ? 4 : 2);
    if (n_layers == 0) {
        STI_TRY(hipMemcpyAsync(y, x, io_bytes, hipMemcpyDeviceToDevice, stream));
        return STI_OK;
    }
    const size_t wsh = (size_t)dims->d_model * (4 * (size_t)dims->d_head + 2 * (size_t)dims->ffn_per_shard);
    std::vector<size_t> first_shard;   // index of a layer's first present shard in the model-wide table
    std::vector<ShardDesc> table;
    if (whole_model_fits) {
        try {
            first_shard.resize(n_layers);
            table.reserve((size_t)n_layers * M);
            for (int l = 0; l < n_layers; ++l) {
                first_shard[l] = table.size();
                for (int i = 0; i < M; ++i) {
                    const sti_shard &s = chosen[(size_t)l * M + i];
                    if (s.bitwidth != 0) table.push_back(make_desc(s, i));
                }
            }
        } catch (const std::bad_alloc &) {
            return STI_ERR_HIP;
        }
        if (!table.empty())
            STI_TRY(staging().upload(table.data(), table.size(), (ShardDesc *)(ws + wl.table), stream));
    }
    // Layer l's working buffer is slot l % w16_layers of a ring (a slot holds a full layer): a group of
    // decode_group <= w16_layers layers has slots of its own, the slot of layer l + 1 is not that of
    // layer l, and whatever a slot held before belongs to a layer whose launches are already behind on
    // the stream.  (A ring rather than a buffer per layer: less memory, and measured 1-2.5 % faster.)
    const int decode_group = wl.decode_group;
    auto w16_of = [&](int l) { return ws + wl.w16 + (size_t)(l % wl.w16_layers) * M * wsh * 2; };
    const ShardDesc *dev_table = (const ShardDesc *)(ws + wl.table);
    auto last_shard = [&](int l) { return (l + 1 < n_layers) ? first_shard[l + 1] : table.size(); };
    // put layer l's outlier dictionaries into its working buffer (absent in most stores)
    auto patch_layer = [&](int l) -> sti_status {
        const size_t a = first_shard[l], b = last_shard(l);
        uint32_t max_outliers = 0;
        InlineShardTable t;
        memset(&t, 0, sizeof(t));
        for (size_t e = a; e < b; ++e) {
            t.d[e - a] = table[e];
            if (table[e].n_outliers > max_outliers) max_outliers = table[e].n_outliers;
        }
        if (max_outliers > 0)
            STI_TRY(launch_patch_outliers_tiled(t, (int)(b - a), max_outliers, dims->d_model, dims->d_head,
                                                dims->ffn_per_shard, w16_of(l), stream));
        return STI_OK;
    };
    // decompress layers [l0, l1) into their working buffers and apply their outlier dictionaries
    auto decode_layers = [&](int l0, int l1) -> sti_status {
        // (the caller keeps a group inside the ring: slots l0 % w16_layers ... are consecutive)
        bool all_full = true;   // then the shards of the group lie back to back, as one launch writes them
        for (int l = l0; l < l1; ++l) all_full = all_full && last_shard(l) - first_shard[l] == (size_t)M;
        for (int l = l0; l < l1; ++l) {
            const int lend = all_full ? l1 : l + 1;   // one launch for the group, else one per layer
            const size_t lo = first_shard[l], hi = last_shard(lend - 1);
            if (hi > lo)
                STI_TRY(timed(STI_K_DECODE, stream, [&] {
                    return launch_decode_tiled_table(dev_table + lo, (int)(hi - lo), dims->d_model, dims->d_head,
                                                     dims->ffn_per_shard, w16_of(l), stream);
                }));
            for (int k = l; k < lend; ++k) {
                sti_status ps = patch_layer(k);
                if (ps != STI_OK) return ps;
            }
            l = lend - 1;
        }
        return STI_OK;
    };
    // A layer whose Q/K/V projection leaves compute units idle (spare_decode_workgroups) decompresses
    // the layer behind it on those units: then only the first layer (and whatever follows a layer that
    // cannot) is decompressed by a launch of its own.
    auto spare = [&](int l) {
        return spare_decode_workgroups(*dims, batch, seq, (int)(last_shard(l) - first_shard[l]), precision);
    };
    const sti_dtype act = (precision == STI_PREC_F32) ? STI_F32 : STI_F16;
    const void *cur = x;
    int next_buf = 0;
    if (io_dtype != act) {
        STI_TRY(timed(STI_K_CONVERT, stream, [&] { return launch_convert(x, io_dtype, ws + wl.act[0], act, (uint64_t)T * dims->d_model, stream); }));
        cur = ws + wl.act[0];
        next_buf = 1;
    }
    int decoded_upto = 0;   // layers [0, decoded_upto) have their working buffers (as far as the stream is concerned)
    for (int l = 0; l < n_layers; ++l) {
        const bool last = (l == n_layers - 1);
        void *out = last ? y : (void *)(ws + wl.act[next_buf]);
        NextLayerDecode next_decode = {nullptr, 0, nullptr, 0};
        if (whole_model_fits && !table.empty()) {
            const int spare_here = spare(l);
            if (l >= decoded_upto) {
                int l1 = l + decode_group < n_layers ? l + decode_group : n_layers;
                const int to_wrap = wl.w16_layers - l % wl.w16_layers;   // slots up to the end of the ring
                if (l1 > l + to_wrap) l1 = l + to_wrap;
                if (spare_here > 0) l1 = l + 1;   // the layers behind this one ride along with their predecessors
                st = decode_layers(l, l1);
                if (st != STI_OK) return st;
                decoded_upto = l1;
            }
            if (spare_here > 0 && l + 1 == decoded_upto && l + 1 < n_layers) {
                const size_t a = first_shard[l + 1], b = last_shard(l + 1);
                if (b > a) next_decode = {dev_table + a, (int)(b - a), w16_of(l + 1), spare_here};
                decoded_upto = l + 2;
            }
        }
        const void *predecoded = whole_model_fits ? (const void *)w16_of(l) : nullptr;
        st = run_layer(*dims, &chosen[(size_t)l * M], params[l], cur, out, last ? io_dtype : act,
                       batch, seq, precision, ws, wl, stream, predecoded, masked ? key_lengths : nullptr,
                       next_decode.workgroups > 0 ? &next_decode : nullptr);
        if (st != STI_OK) return st;
        if (next_decode.workgroups > 0) {
            st = patch_layer(l + 1);
            if (st != STI_OK) return st;
        }
        cur = out;
        next_buf ^= 1;
    }
    return STI_OK;
}

}  // namespace

extern "C" {

size_t sti_model_workspace_bytes(const sti_dims *dims, int n_layers, int batch, int seq, sti_precision precision)
{
    if (check_dims(dims, batch, seq, precision) != STI_OK || n_layers < 0) return 0;
    const int64_t T = (int64_t)batch * seq;
    const bool whole_model = precision == STI_PREC_F16_MFMA && !few_token_path(*dims, T) && n_layers > 1;
    return workspace_layout(*dims, T, precision, whole_model ? n_layers : 1).total;
}

sti_status sti_profile_begin(void)
{
    return profiler().begin() == hipSuccess ? STI_OK : STI_ERR_HIP;
}

sti_status sti_profile_end(sti_profile *out)
{
    if (!out) return STI_ERR_NULL;
    return profiler().end(out) == hipSuccess ? STI_OK : STI_ERR_HIP;
}

}  // extern "C"
