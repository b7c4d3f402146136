/*
 * sti.h - C ABI of the shard-decode + shard-subset encoder-layer library for
 * AMD MI355X (gfx950).
 *
 * The library executes the compute side of the paper's inference pipeline:
 * a model is stored as N x M x K shard versions (layer, vertical slice,
 * bitwidth; Section "storing shards per version"); a submodel selects, per
 * layer, a subset of the M shards and one fidelity version of each (Section
 * "vertical partitioning", "quantization per shard"); a layer is decompressed
 * and computed as one job and layers run in order (Section "Submodel
 * execution").  Biases and LayerNorm parameters are not part of shards and
 * stay resident in full precision (Section "Implementation", last paragraph).
 * Embeddings, pooler and task heads are outside this library.
 *
 * Conventions for every entry point
 * ---------------------------------
 *  - Pointers marked DEVICE are device (HBM) addresses owned by the caller;
 *    pointers marked HOST are ordinary host memory that is read only during
 *    the call and may be freed as soon as it returns.
 *  - `hip_stream` is a hipStream_t (NULL = the default stream).  All device
 *    work is enqueued on it; no entry point synchronises the device.  Results
 *    are valid once the stream has reached the end of the enqueued work.
 *  - Nothing is thrown or aborted across the ABI: the return code is the only
 *    error channel.  All argument validation happens before the first launch,
 *    so an argument error leaves the outputs untouched.
 *  - The library allocates no device memory.  Scratch space comes in through
 *    the `workspace` arguments; the only state it keeps is a small pinned host
 *    staging ring used to upload shard tables.  Two calls that are given the
 *    same workspace must be ordered (same stream, or caller-side events).
 *  - The call fails with STI_ERR_HIP when no gfx950 device code can run.
 *
 * Stream format of a k-bit shard (k = 2..6)
 * -----------------------------------------
 *  Index j of the shard occupies bits [j*k, j*k + k) of a gap-free bitstream;
 *  stream bit b is bit (b mod 8) of byte floor(b / 8) (least significant bit
 *  first; the two 4-bit indexes of a byte are low nibble first).  There is no
 *  per-row padding.  The stream is ceil(n*k/8) bytes and must start on a
 *  16-byte boundary.  A 32-bit shard is n raw float32 values.
 *
 * Logical layout of the decoded weights of a shard (Table 1)
 * ----------------------------------------------------------
 *  Six row-major [out_features][in_features] sub-blocks, in this order:
 *    Wq [dh x d]  Wk [dh x d]  Wv [dh x d]   rows of the layer's Q/K/V matrices of head i
 *    Wo [d x dh]                             columns of the output projection reading head i
 *    W1 [f x d]                              rows i*f .. (i+1)*f of FFN1
 *    W2 [d x f]                              columns i*f .. (i+1)*f of FFN2
 *  with d = d_model, dh = d_head, f = ffn_per_shard; d*(4*dh + 2*f) weights.
 */
#ifndef STI_H
#define STI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    STI_OK = 0,
    STI_ERR_NULL = 1,          /* a required pointer is NULL                               */
    STI_ERR_DIMS = 2,          /* a size is negative, zero where it may not be, or unsupported */
    STI_ERR_BITWIDTH = 3,      /* bitwidth outside {0, 2, 3, 4, 5, 6, 32} (0 only where absent is allowed) */
    STI_ERR_MISSING_SHARD = 4, /* the plan selects a version whose data pointer is NULL    */
    STI_ERR_ALIGN = 5,         /* a device pointer is not aligned as documented            */
    STI_ERR_WORKSPACE = 6,     /* workspace NULL or smaller than the query function says   */
    STI_ERR_DTYPE = 7,         /* unknown sti_dtype / sti_precision value                  */
    STI_ERR_HIP = 8,           /* a HIP runtime call failed (launch, copy, event)          */
    STI_ERR_UNSUPPORTED = 9    /* valid request that this build does not implement         */
} sti_status;

typedef enum { STI_F32 = 0, STI_F16 = 1, STI_BF16 = 2 } sti_dtype;

/* STI_PREC_F32: float32 storage and arithmetic end to end (decode to a float32
 *   working buffer, then float32 kernels); any dimensions.
 * STI_PREC_F16_MFMA: binary16 operands on the matrix cores with float32
 *   accumulation.  Up to 128 tokens per call (192 when d_model <= 768) the
 *   projections decode the packed streams inside their weight loader; with
 *   more tokens, and for shards that carry an outlier dictionary, a layer's
 *   shards are decompressed once into a binary16 working buffer in the
 *   workspace that the projections then read (every weight would otherwise be
 *   decoded once per 64 or 128 token rows).  Needs d_head == 64, d_model and
 *   ffn_per_shard multiples of 64 and seq <= 512 (STI_ERR_DIMS otherwise). */
typedef enum { STI_PREC_F32 = 0, STI_PREC_F16_MFMA = 1 } sti_precision;

typedef struct {
    int32_t d_model;       /* d  : hidden size                                   */
    int32_t n_heads;       /* M  : attention heads = shards per layer (<= 64)    */
    int32_t d_head;        /* dh : features per head (d_model need not equal M*dh) */
    int32_t ffn_per_shard; /* f  : FFN neurons per shard (d_ff / M)              */
    float ln_eps;          /* LayerNorm epsilon (BERT uses 1e-12)                */
} sti_dims;

/* One fidelity version of one shard (Figure "instantiating N x M x K model
 * shards": k-bit index matrix + centroid dictionary + outlier dictionary). */
typedef struct {
    int8_t bitwidth;             /* 0 = absent, 2..6 = packed indexes, 32 = raw float32          */
    const void *data;            /* DEVICE. ceil(n*k/8) bytes or n float32; 16-byte aligned      */
    const float *codebook;       /* DEVICE. 2^k float32 centroids, 4-byte aligned; ignored for 32 */
    uint32_t n_outliers;         /* entries of the outlier dictionary (0 = none; must be 0 for 32) */
    const uint32_t *outlier_pos; /* DEVICE. distinct offsets (< n) of the outliers inside the shard */
    const float *outlier_val;    /* DEVICE. their original float32 weights                         */
} sti_shard;

/* Resident full-precision parameters of one layer.  All DEVICE float32. */
typedef struct {
    const float *bq, *bk, *bv; /* [M*dh]  biases of the Q/K/V projections, head-major      */
    const float *bo;           /* [d]     bias of the output projection                    */
    const float *b1;           /* [M*f]   bias of FFN1, slice-major                        */
    const float *b2;           /* [d]     bias of FFN2                                     */
    const float *ln1_g, *ln1_b; /* [d]    LayerNorm after the attention block              */
    const float *ln2_g, *ln2_b; /* [d]    LayerNorm after the feed-forward block           */
} sti_layer_params;

/* Text for a status code (static storage, never NULL). */
const char *sti_status_string(sti_status s);

/* ---------------------------------------------------------------------------
 * Decompression (Section "quantization per shard": "substituting dictionary
 * indexes with floating point centroids"; Section "Implementation": the
 * index -> centroid substitution loop).
 *
 * For s in [0, n_shards), j in [0, weights_per_shard):
 *     out[s*weights_per_shard + j] = round_to(out_dtype, codebook_s[index_s[j]])
 * or the raw value for a 32-bit shard; then, for every entry t of the shard's
 * outlier dictionary (Section "Implementation": outliers keep a k-bit
 * placeholder; their original weights and offsets are bookkept),
 *     out[s*weights_per_shard + outlier_pos[t]] = round_to(out_dtype, outlier_val[t]).
 * Offsets must be distinct; offsets >= weights_per_shard are ignored.  The layer
 * entry points apply the same dictionary.  Rounding to F16/BF16 is to nearest,
 * ties to even, subnormals kept, overflow to infinity; F32 output is the
 * centroid bit for bit.
 *
 *  shards            HOST array [n_shards]; bitwidth 0 is NOT allowed here.
 *  weights_per_shard number of weights n of every shard (any value >= 0).
 *  out               DEVICE, n_shards*n elements of out_dtype, 16-byte aligned.
 *  workspace         DEVICE scratch of at least sti_decode_workspace_bytes(n_shards)
 *                    bytes, 16-byte aligned; may be NULL when that size is 0.
 *
 * Stream capture: a call with at most 64 shards enqueues kernels only and may be
 * captured into a graph.  A larger call uploads its shard table through a pinned
 * host buffer that later calls reuse, so it returns STI_ERR_UNSUPPORTED, before
 * enqueuing anything, when `hip_stream` is capturing.
 *
 * Errors: NULL / DIMS (negative counts) / BITWIDTH / MISSING_SHARD (data NULL,
 * or codebook NULL for k <= 6) / NULL (outlier arrays missing) / ALIGN /
 * WORKSPACE / DTYPE / UNSUPPORTED (outliers on a 32-bit shard; more than 64
 * shards under stream capture) / HIP.
 * ------------------------------------------------------------------------- */
size_t sti_decode_workspace_bytes(int n_shards);

sti_status sti_decode_shards(const sti_shard *shards, int n_shards, uint64_t weights_per_shard,
                             void *out, sti_dtype out_dtype, void *workspace,
                             size_t workspace_bytes, void *hip_stream);

/* ---------------------------------------------------------------------------
 * One encoder layer over a shard subset (Section "A primer on transformer":
 * per-head Q, K, V -> attention scores -> output projection O -> two FFN
 * linears; Section "vertical partitioning": any subset of a layer's shards
 * executes; Table 1).  With P the present shards and X the input [B*L x d]:
 *
 *   Q_i = X Wq_i^T + bq_i (same K_i, V_i);  C_i = softmax(Q_i K_i^T / sqrt(dh)) V_i  per sequence
 *   h   = LayerNorm1( X + bo + sum_{i in P} C_i Wo_i^T )
 *   U_i = gelu( h W1_i^T + b1_i ),  gelu(z) = z/2 (1 + erf(z / sqrt 2))
 *   y   = LayerNorm2( h + b2 + sum_{i in P} U_i W2_i^T )
 *
 * LayerNorm uses the biased variance over d and ln_eps.  An absent shard adds
 * nothing and nothing is rescaled; a layer with every shard absent is valid.
 *
 *  shards   HOST array [M]; bitwidth 0 = absent.
 *  params   HOST struct of DEVICE pointers.
 *  x, y     DEVICE [batch][seq][d_model] of io_dtype, 16-byte aligned, not aliased.
 *  workspace DEVICE, >= sti_workspace_bytes(dims, batch, seq, precision), 256-byte aligned.
 *
 * sti_workspace_bytes returns 0 for invalid arguments.
 * ------------------------------------------------------------------------- */
size_t sti_workspace_bytes(const sti_dims *dims, int batch, int seq, sti_precision precision);

sti_status sti_layer_forward(const sti_dims *dims, const sti_shard *shards,
                             const sti_layer_params *params, const void *x, void *y,
                             sti_dtype io_dtype, int batch, int seq, sti_precision precision,
                             void *workspace, size_t workspace_bytes, void *hip_stream);

/* ---------------------------------------------------------------------------
 * sti_layer_forward for callers that cannot allocate device memory (code under graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same layer, the
 * same kernels and the same results, with the workspace taken from an array that is
 * part of the library's device image instead of from the caller.  The call allocates
 * nothing (no device, pinned or pageable memory) and enqueues kernel launches only.
 *
 * The array holds sti_static_scratch_bytes() = 64 MiB on every GPU the library runs on,
 * from the first use of the library on that GPU until the process ends.  A call whose
 * sti_workspace_bytes(dims, batch, seq, precision) exceeds it returns STI_ERR_WORKSPACE
 * before anything is enqueued (BERT-base dimensions fit 20 x 128 tokens with
 * STI_PREC_F16_MFMA and 8 x 128 with STI_PREC_F32; d_model 1024 with 16 shards fits
 * 12 x 128 and 2 x 128).  All calls on one GPU share the one array:
 * calls whose kernels may overlap on that GPU (different streams, or several host
 * threads) race; calls on one stream are ordered and safe.  The array keeps the last
 * call's contents; no kernel of the layer reads scratch memory it has not written in
 * the same call, so nothing needs clearing.  The array's address on the current device is
 * looked up on the first call there, which should be made outside stream capture.
 * Other arguments and errors as for sti_layer_forward.
 * ------------------------------------------------------------------------- */
size_t sti_static_scratch_bytes(void);

sti_status sti_layer_forward_static(const sti_dims *dims, const sti_shard *shards,
                                    const sti_layer_params *params, const void *x, void *y,
                                    sti_dtype io_dtype, int batch, int seq, sti_precision precision,
                                    void *hip_stream);

/* ---------------------------------------------------------------------------
 * The working buffer of the matrix-core path by itself (Section "Submodel execution":
 * all selected shards of a layer are decompressed into a working buffer before the
 * layer's computation starts).  sti_decode_working_buffer writes what sti_layer_forward
 * (STI_PREC_F16_MFMA, working-buffer route) places in its workspace before the
 * projections run: the present shards, in slot order, compacted, each as
 * weights_per_shard = d*(4*dh + 2*f) binary16 values (codebook entries and outlier
 * weights rounded to nearest even), in a tiled order chosen so that one matrix-core
 * operand of a wave is one contiguous 1 KiB read:
 *
 *   weight j of a shard lies in one of the six row-major sub-blocks Wq|Wk|Wv [3dh x d],
 *   Wo [d x dh], W1 [f x d], W2 [d x f] (element offsets 0, 3*dh*d, 4*dh*d,
 *   4*dh*d + f*d; Wq, Wk, Wv form one block of 3*dh rows), at (row, col) of a block with
 *   C columns that starts at element offset `sub`.  Its place in the shard's image is
 *     sub + ((row/32)*(C/64) + col/64)*2048 + ((col%32)/8)*512
 *         + (((col%64)/32)*32 + row%32)*8 + col%8            (binary16 elements).
 *
 * sti_working_buffer_offset evaluates that formula (HOST; -1 for invalid dims or j out of
 * range); sti_working_buffer_bytes is the size for all M shards present (0 for invalid dims).
 * Dimensions as for STI_PREC_F16_MFMA.
 *
 *  shards    HOST array [M]; bitwidth 0 = absent (skipped, nothing written for it).
 *  out       DEVICE, 256-byte aligned, at least (present shards) * weights_per_shard * 2 bytes.
 * Errors: NULL / DIMS / BITWIDTH / MISSING_SHARD / ALIGN / WORKSPACE (out_bytes too small) / HIP.
 * Kernel launches only: may be captured.
 * ------------------------------------------------------------------------- */
size_t sti_working_buffer_bytes(const sti_dims *dims);
int64_t sti_working_buffer_offset(const sti_dims *dims, uint64_t j);
sti_status sti_decode_working_buffer(const sti_dims *dims, const sti_shard *shards, void *out,
                                     size_t out_bytes, void *hip_stream);

/* ---------------------------------------------------------------------------
 * Layers 0 .. n_layers-1 in order, the output of one feeding the next (Section
 * "Submodel execution").  A shallower submodel is run by passing fewer layers.
 *
 *  store   HOST array [n_layers][M][6]: the versions of shard (l, i) for
 *          k = 2, 3, 4, 5, 6, 32 in that order; data == NULL where a version is
 *          not stored.  The bitwidth field of a stored version must match its slot.
 *  params  HOST array [n_layers].
 *  plan    HOST int8 [n_layers][M]: 0 = absent, else the bitwidth to use.
 *  x, y    as for sti_layer_forward; n_layers == 0 copies x to y.
 * ------------------------------------------------------------------------- */
sti_status sti_model_forward(const sti_dims *dims, int n_layers, const sti_shard *store,
                             const sti_layer_params *params, const int8_t *plan, const void *x,
                             void *y, sti_dtype io_dtype, int batch, int seq,
                             sti_precision precision, void *workspace, size_t workspace_bytes,
                             void *hip_stream);

/* ---------------------------------------------------------------------------
 * Padded sequences.  The paper runs inputs padded to one fixed length (Section
 * "Prerequisite: Offline Profiling": the input length is fixed after padding, e.g. 128;
 * Section "Compute Planning").  With the variants below, sequence b holds key_lengths[b]
 * real positions followed by padding, and in every layer
 *
 *   C_i = softmax over the first key_lengths[b] keys only ( Q_i K_i^T / sqrt(dh) ) V_i,
 *
 * i.e. no query gives attention weight to a padded position.  The rows of padded
 * positions are computed like any other (from the real keys) and written to y; the real
 * rows do not depend on what the padding holds, as long as it is finite.
 *
 *  key_lengths  DEVICE int32 [batch], 4-byte aligned, read by the kernels when they run
 *               (it must stay unchanged until then).  Values are clamped to 1 .. seq.
 *               NULL is STI_ERR_NULL unless batch * seq == 0.
 * All other arguments, the workspace sizes and the error behaviour are those of the
 * entry point without the suffix, which is the case key_lengths[b] == seq for all b.
 * ------------------------------------------------------------------------- */
sti_status sti_layer_forward_masked(const sti_dims *dims, const sti_shard *shards,
                                    const sti_layer_params *params, const void *x, void *y,
                                    sti_dtype io_dtype, int batch, int seq, const int32_t *key_lengths,
                                    sti_precision precision, void *workspace, size_t workspace_bytes,
                                    void *hip_stream);

sti_status sti_model_forward_masked(const sti_dims *dims, int n_layers, const sti_shard *store,
                                    const sti_layer_params *params, const int8_t *plan, const void *x,
                                    void *y, sti_dtype io_dtype, int batch, int seq,
                                    const int32_t *key_lengths, sti_precision precision, void *workspace,
                                    size_t workspace_bytes, void *hip_stream);

/* Workspace size with which sti_model_forward keeps a ring of working buffers - two to four
 * layers' worth (64 MiB), never fewer than two - and the model's shard table in device memory
 * (Section "Submodel execution" keeps one layer's working buffer and decompresses a layer right
 * before it computes; with a second buffer a layer is decompressed while the layer before it
 * computes - by the workgroups that the Q/K/V launch of that layer has to spare, when it has at
 * least 32 of them - and otherwise a few layers are decompressed by one launch right before the
 * first of them runs).  Applies to STI_PREC_F16_MFMA whenever
 * the layer goes through the working buffer (more than 128 tokens, more than 192 when
 * d_model <= 768); otherwise, and for n_layers <= 1, it equals sti_workspace_bytes.
 * sti_model_forward takes this whole-model route whenever workspace_bytes is at least this value
 * and the per-layer route otherwise: same results either way.  The whole-model route uploads
 * a shard table through a pinned host buffer that later calls reuse and is therefore
 * never taken while `hip_stream` is capturing: a captured call runs the per-layer route
 * (kernel launches only), whatever the workspace size.  0 on invalid arguments. */
size_t sti_model_workspace_bytes(const sti_dims *dims, int n_layers, int batch, int seq,
                                 sti_precision precision);

/* ---------------------------------------------------------------------------
 * Layerwise load || compute pipeline with a preload buffer (Section "Elastic
 * pipelining": the IO of layer k+1 overlaps the computation of layer k, and a small
 * preload buffer keeps the shards of the bottom layers in memory across inferences;
 * Section "Submodel execution": after an inference the loaded shards are kept from
 * the bottom layers up until the buffer is full).
 *
 * Here the packed shard streams stay in HOST memory (pinned, so that copies are
 * asynchronous) and play the role of the paper's flash.  sti_pipeline_forward
 * computes exactly what sti_model_forward computes, but moves the selected version
 * of every shard of layer k+1 over the host link on a library-owned stream while
 * the caller's stream computes layer k.  The first selected shards in (layer,
 * shard) order that fit `preload_bytes` are placed in the preload buffer instead of
 * the two staging slots; a later call that selects the same versions from the same
 * host addresses finds them there and copies nothing for them.
 *
 *  preload_buffer DEVICE, 256-byte aligned, owned by the caller, must outlive the handle;
 *                 may be NULL with preload_bytes == 0 (every call starts cold).
 *  staging        DEVICE, 256-byte aligned, owned by the caller, must outlive the handle.
 *                 sti_pipeline_staging_bytes(dims) is the minimum: two slots of one
 *                 full-precision layer each.  Every further slot that fits (up to 8)
 *                 lets the copies run one more layer ahead of the computation.
 *  store          as for sti_model_forward, except that `data` of every version is a
 *                 HOST address (16-byte aligned); codebooks and outlier dictionaries
 *                 stay DEVICE resident like the biases (a few hundred bytes each).
 *  stats          HOST, optional: what this call copied and what it found resident.
 *
 * A handle serves one call at a time; calls on one handle may be enqueued back to
 * back (the copies of a call wait for the kernels of the previous one).  The
 * library-owned stream has default priority; the handle must not be used while a
 * stream capture is active.  Errors as for sti_model_forward.
 * ------------------------------------------------------------------------- */
typedef struct sti_pipeline sti_pipeline;

typedef struct {
    uint64_t bytes_copied;     /* host -> device bytes moved by this call                    */
    uint64_t bytes_resident;   /* bytes of the selected shards held by the preload buffer     */
    uint32_t shards_copied;    /* shards moved over the host link by this call                */
    uint32_t shards_hit;       /* selected shards found in the preload buffer (no copy)       */
    uint32_t shards_preloaded; /* selected shards in the preload buffer after this call       */
} sti_pipeline_stats;

size_t sti_pipeline_staging_bytes(const sti_dims *dims);

sti_status sti_pipeline_create(const sti_dims *dims, void *preload_buffer, size_t preload_bytes,
                               void *staging, size_t staging_bytes, sti_pipeline **out);

sti_status sti_pipeline_forward(sti_pipeline *pipeline, int n_layers, const sti_shard *store,
                                const sti_layer_params *params, const int8_t *plan, const void *x,
                                void *y, sti_dtype io_dtype, int batch, int seq,
                                sti_precision precision, void *workspace, size_t workspace_bytes,
                                void *hip_stream, sti_pipeline_stats *stats);

/* sti_pipeline_forward over padded sequences: key_lengths as for sti_model_forward_masked. */
sti_status sti_pipeline_forward_masked(sti_pipeline *pipeline, int n_layers, const sti_shard *store,
                                       const sti_layer_params *params, const int8_t *plan, const void *x,
                                       void *y, sti_dtype io_dtype, int batch, int seq,
                                       const int32_t *key_lengths, sti_precision precision,
                                       void *workspace, size_t workspace_bytes, void *hip_stream,
                                       sti_pipeline_stats *stats);

/* Waits for the handle's copies, then releases its stream and events (not the buffers). */
sti_status sti_pipeline_destroy(sti_pipeline *pipeline);

/* ---------------------------------------------------------------------------
 * Two-stage planning (Section "Compute Planning", Section "IO Planning").  Host
 * code only: HOST pointers, no device work, no stream.
 *
 * sti_plan_tables holds what the paper profiles once per device (Section
 * "Prerequisite: Offline Profiling"): the delay of loading one shard per
 * bitwidth and of decompressing + executing one layer of m shards (sentence
 * length and clock are fixed by whoever fills the table).
 *
 * sti_plan_submodel: of all n x m submodels (n layers of m shards) whose
 * computation meets the deadline, n * t_comp[m-1] <= deadline_s, the one with
 * the most shards; of those with equally many, the deepest.  n = m = 0 when even
 * 1 x 1 is too slow.
 *
 * sti_plan_bitwidths: fidelity versions for the submodel layers 0..n-1 x shards
 * 0..m-1.  AIB(0) is the IO time that filled the preload buffer (the preloaded
 * shards inside the submodel), AIB(k) = AIB(k-1) + t_comp[m-1]; a shard chosen at
 * layer l is charged to the budgets of layer l and of all later layers, and a
 * plan is valid while no budget is negative (Section "Accumulated IO Budgets").
 * Preloaded shards keep their version.  Pass 1 gives all others the highest
 * uniform bitwidth (2..6, 32) that is valid - 2 bits if none is, and then pass 2
 * is skipped; pass 2 walks `importance` (most important first) and raises a
 * shard to 32 bits whenever the budgets allow (Section "Selecting Optimal Shard
 * Versions").
 *
 *  preloaded   HOST [n_layers*n_shards], may be NULL: bitwidth of the version the
 *              preload buffer holds of shard (l, i), 0 = not held.
 *  importance  HOST [n_layers*n_shards]: a permutation of the shard ids
 *              l*n_shards + i (required when n > 0).
 *  plan        HOST out [n_layers*n_shards]: bitwidth, 0 = not in the submodel;
 *              the layout sti_model_forward and sti_pipeline_forward take.
 *  aib         HOST out [n], may be NULL: the budgets left after the allocation.
 * Errors: STI_ERR_NULL, STI_ERR_DIMS (sizes, negative or non-finite delays,
 * importance not a permutation), STI_ERR_BITWIDTH (preloaded).
 * ------------------------------------------------------------------------- */
typedef struct {
    int32_t n_layers;      /* N: layers of the full model                              */
    int32_t n_shards;      /* M: shards per layer                                      */
    double t_io[6];        /* seconds to load one shard at 2, 3, 4, 5, 6, 32 bits      */
    const double *t_comp;  /* HOST [n_shards]: t_comp[m-1] = seconds per layer of m shards */
} sti_plan_tables;

sti_status sti_plan_submodel(const sti_plan_tables *tables, double deadline_s, int32_t *n, int32_t *m);

sti_status sti_plan_bitwidths(const sti_plan_tables *tables, int32_t n, int32_t m, const int8_t *preloaded,
                              const int32_t *importance, int8_t *plan, double *aib);

/* ---------------------------------------------------------------------------
 * Quantizing a layer's shards into a k-bit version (Section "quantization per
 * shard"; Section "Implementation", preprocessing of the model): one Gaussian is
 * fitted to all weights of the layer (mean, biased variance + reg_covar); a weight
 * whose log likelihood under it is below `loglik_threshold` (the paper: -4) is an
 * outlier; the remaining weights are cut, in sorted order, into 2^k clusters of
 * equal population, cluster c starting at rank floor(c*n/2^k); the centroid of a
 * cluster is the arithmetic mean of its members; every weight is replaced by the
 * k-bit index of the cluster whose value range holds it (all copies of a value go
 * to one cluster; an outlier's placeholder follows the same rule) and outliers are
 * bookkept per shard as (offset inside the shard, original value), offsets
 * ascending.  The outputs are exactly what sti_shard takes: `packed` in the stream
 * format above, one codebook shared by the layer's shards, outlier dictionaries.
 *
 *  weights        DEVICE float32 [n_heads][Wsh]: the layer's shards at full precision
 *                 (the logical layout of Table 1), 16-byte aligned; Wsh % 1024 == 0
 *                 (STI_ERR_UNSUPPORTED otherwise); finite values.
 *  packed         DEVICE out [n_heads][Wsh*k/8] bytes.
 *  codebook       DEVICE out float32 [2^k], ascending.
 *  outlier_pos/val DEVICE out [n_heads][max_outliers_per_shard]; entries beyond a
 *                 shard's count are left untouched.  outlier_count DEVICE out
 *                 [n_heads]: the shard's number of outliers, which may exceed
 *                 max_outliers_per_shard (then the dictionary is truncated: call
 *                 again with more room).
 *  stats          DEVICE out, may be NULL; status 1 = every weight is an outlier
 *                 (nothing to cluster; packed and codebook are meaningless).
 *  workspace      DEVICE, >= sti_quantize_workspace_bytes(dims), 256-byte aligned.
 * The moments (mean, variance) are accumulated in float64 in a fixed order.  The
 * cluster sums are float64 too; within one wave the order in which weights of one
 * cluster are added is the hardware's (LDS atomics), the per-wave sums are then
 * combined in a fixed order.  Any order of such a sum of at most 256 float32 values
 * agrees to about 1e-16 relative, far below the one float32 rounding of the centroid:
 * streams, dictionaries and the outlier decisions are reproducible bit for bit, a
 * centroid could in principle differ in its last bit between calls (not observed).
 * Errors as for the other entry points.
 * ------------------------------------------------------------------------- */
typedef struct {
    double mean;          /* fitted mean                                   */
    double variance;      /* fitted variance (reg_covar included)          */
    uint64_t n_outliers;  /* over all shards of the layer                  */
    uint32_t status;      /* 0 ok, 1 no inliers                            */
} sti_quant_stats;

size_t sti_quantize_workspace_bytes(const sti_dims *dims);

sti_status sti_quantize_layer(const sti_dims *dims, const float *weights, int bitwidth, double loglik_threshold,
                              double reg_covar, uint8_t *packed, float *codebook, uint32_t *outlier_pos,
                              float *outlier_val, uint32_t max_outliers_per_shard, uint32_t *outlier_count,
                              sti_quant_stats *stats, void *workspace, size_t workspace_bytes, void *hip_stream);

/* ---------------------------------------------------------------------------
 * Per-kernel timing (the counterpart of the paper's one-time hardware profiling
 * of computation delays, Section "Prerequisite: offline profiling").  Between
 * sti_profile_begin() and sti_profile_end() every kernel launch of the entry
 * points above carries two events on the caller's stream that take the
 * dispatch's own begin and end time stamps; sti_profile_end() waits for them
 * and returns, per kernel class, the number of launches and the summed kernel
 * time in milliseconds.  Process wide, not re-entrant; meant for measurement
 * runs, not for production calls (nor for calls under stream capture).
 * ------------------------------------------------------------------------- */
typedef enum {
    STI_K_DECODE = 0,
    STI_K_GEMM_QKV = 1,
    STI_K_ATTENTION = 2,
    STI_K_GEMM_OUT = 3,
    STI_K_LAYERNORM = 4,
    STI_K_GEMM_FFN_UP = 5,
    STI_K_GEMM_FFN_DOWN = 6,
    STI_K_CONVERT = 7,
    STI_K_COUNT = 8
} sti_kernel_class;

typedef struct {
    uint64_t launches[STI_K_COUNT];
    double ms[STI_K_COUNT];
} sti_profile;

sti_status sti_profile_begin(void);
sti_status sti_profile_end(sti_profile *out); /* HOST out */

#ifdef __cplusplus
}
#endif
#endif /* STI_H */
