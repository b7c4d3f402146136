/*
 * CPU oracle for shard decode and the shard-subset encoder layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain definition of what the
 * GPU library computes, written from the paper, in double precision with
 * scalar loops.  It shares no code, header, table or helper with the HIP
 * path and is never called by it; only the tests, the smoke check and the
 * benchmark's CPU-baseline leg use it.  Nothing here is blocked, fused or
 * reordered beyond the definitions below (OpenMP only splits independent
 * output rows over cores, as the paper's own C/OpenMP decompressor splits
 * its substitution loop, Section "Implementation").
 *
 * What is defined
 * ---------------
 * Decode (Section "quantization per shard", "storing shards per version"):
 *   a k-bit shard is a gap-free bitstream of k-bit dictionary indexes, least
 *   significant bit first, plus 2^k float32 centroids; decompression
 *   substitutes each index by its centroid, then puts the bookkept outliers
 *   back at their offsets.  A 32-bit shard is raw float32.
 * Shard layout (Table 1): six row-major [out][in] sub-blocks
 *   Wq[dh x d] Wk[dh x d] Wv[dh x d] Wo[d x dh] W1[f x d] W2[d x f].
 * Layer (Section "A primer on transformer", "vertical partitioning"):
 *   post-LayerNorm BERT encoder layer restricted to the present shards;
 *   an absent shard contributes exactly nothing; biases of the output
 *   projection and of FFN2, both residuals and both LayerNorms always apply.
 * Model (Section "Submodel execution"): layers run in order, layer l+1
 *   consumes the output of layer l.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_ARG 1
#define ORACLE_ERR_MEM 2

#define ORACLE_F32 0
#define ORACLE_F16 1
#define ORACLE_BF16 2

/* One fidelity version of one shard; all pointers are host pointers. */
typedef struct {
    int32_t bitwidth;            /* 0 absent, 2..6 packed indexes, 32 raw float32        */
    const void *data;            /* ceil(n*k/8) bytes, or n float32                       */
    const float *codebook;       /* 2^k float32 centroids; unused for 32                  */
    uint32_t n_outliers;         /* outlier dictionary (Section "Implementation": outliers */
    const uint32_t *outlier_pos; /*   keep a k-bit placeholder; their original weights and */
    const float *outlier_val;    /*   offsets in the shard are bookkept); distinct offsets */
} oracle_shard;

/* Resident full-fidelity parameters of one layer (Section "Implementation",
 * last paragraph: biases and LayerNorm are kept in memory, not in shards). */
typedef struct {
    const float *bq, *bk, *bv; /* [M*dh] */
    const float *bo;           /* [d]    */
    const float *b1;           /* [M*f]  */
    const float *b2;           /* [d]    */
    const float *ln1_g, *ln1_b, *ln2_g, *ln2_b; /* [d] */
} oracle_layer_params;

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* Decode                                                              */
/* ------------------------------------------------------------------ */

/* Index j of a k-bit stream: bit t of the index is stream bit j*k + t,
 * where stream bit b is bit (b mod 8) of byte floor(b / 8). */
uint32_t oracle_unpack_index(const uint8_t *stream, int k, uint64_t j)
{
    uint32_t idx = 0;
    for (int t = 0; t < k; ++t) {
        uint64_t b = j * (uint64_t)k + (uint64_t)t;
        uint32_t bit = (stream[b >> 3] >> (b & 7)) & 1u;
        idx |= bit << t;
    }
    return idx;
}

/* float32 -> binary16, round to nearest, ties to even, subnormals kept,
 * overflow to infinity; done on the bit pattern with integer arithmetic.
 * NaN keeps its sign and the top ten payload bits, with the quiet bit set. */
uint16_t oracle_f32_to_f16(float v)
{
    uint32_t u;
    memcpy(&u, &v, 4);
    uint32_t sign = (u >> 16) & 0x8000u;
    uint32_t exp = (u >> 23) & 0xFFu;
    uint32_t man = u & 0x7FFFFFu;
    if (exp == 0xFFu) {
        if (man == 0) return (uint16_t)(sign | 0x7C00u);
        return (uint16_t)(sign | 0x7E00u | (man >> 13));
    }
    int e = (int)exp - 127; /* unbiased; value = 1.man * 2^e (exp != 0) */
    if (exp == 0) return (uint16_t)sign; /* |v| < 2^-126, far below half of 2^-24 */
    if (e > 15) return (uint16_t)(sign | 0x7C00u);
    uint32_t sig = man | 0x800000u; /* 24-bit significand, value = sig * 2^(e-23) */
    int shift;                      /* number of low bits of sig to drop         */
    uint32_t base;                  /* half bits before adding the kept fraction */
    if (e >= -14) {                 /* normal half: keep 10 fraction bits        */
        shift = 13;
        base = (uint32_t)(e + 15) << 10;
        sig &= 0x7FFFFFu;           /* implicit one is carried by the exponent   */
    } else {                        /* subnormal half: unit is 2^-24             */
        shift = -e - 1;             /* sig * 2^(e-23) / 2^-24 = sig >> (-e-1)    */
        base = 0;
        if (shift > 25) return (uint16_t)sign; /* below half of the smallest subnormal */
    }
    uint32_t kept = sig >> shift;
    uint32_t rem = sig & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (kept & 1u))) kept += 1;
    /* a carry out of the fraction correctly bumps the exponent (and reaches
     * infinity from the largest finite value) because the fields are adjacent */
    return (uint16_t)(sign | (base + kept));
}

/* float32 -> bfloat16, round to nearest even on the dropped 16 bits. */
uint16_t oracle_f32_to_bf16(float v)
{
    uint32_t u;
    memcpy(&u, &v, 4);
    if (((u >> 23) & 0xFFu) == 0xFFu && (u & 0x7FFFFFu) != 0)
        return (uint16_t)((u >> 16) | 0x0040u); /* NaN: keep top payload, set quiet bit */
    uint32_t kept = u >> 16;
    uint32_t rem = u & 0xFFFFu;
    if (rem > 0x8000u || (rem == 0x8000u && (kept & 1u))) kept += 1;
    return (uint16_t)kept;
}

/* Decode n weights of one shard to float32 (bit-for-bit centroid values). */
int oracle_decode_f32(const oracle_shard *sh, uint64_t n, float *out)
{
    if (!sh || !out || !sh->data) return ORACLE_ERR_ARG;
    int k = sh->bitwidth;
    if (k == 32) {
        memcpy(out, sh->data, n * sizeof(float));
        return ORACLE_OK;
    }
    if (k < 2 || k > 6 || !sh->codebook) return ORACLE_ERR_ARG;
    const uint8_t *s = (const uint8_t *)sh->data;
    const float *cb = sh->codebook;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < (int64_t)n; ++j)
        out[j] = cb[oracle_unpack_index(s, k, (uint64_t)j)];
    for (uint32_t t = 0; t < sh->n_outliers; ++t) {
        if (!sh->outlier_pos || !sh->outlier_val) return ORACLE_ERR_ARG;
        if (sh->outlier_pos[t] >= n) return ORACLE_ERR_ARG;
        out[sh->outlier_pos[t]] = sh->outlier_val[t];
    }
    return ORACLE_OK;
}

/* Decode n_shards shards of n weights each into out[n_shards][n] of the
 * requested element type.  Absent shards (bitwidth 0) are an error here. */
int oracle_decode_shards(const oracle_shard *shards, int n_shards, uint64_t n, void *out, int dtype)
{
    if (!shards || !out || n_shards < 0) return ORACLE_ERR_ARG;
    if (dtype != ORACLE_F32 && dtype != ORACLE_F16 && dtype != ORACLE_BF16) return ORACLE_ERR_ARG;
    float *tmp = (float *)malloc((n ? n : 1) * sizeof(float));
    if (!tmp) return ORACLE_ERR_MEM;
    for (int s = 0; s < n_shards; ++s) {
        int rc = oracle_decode_f32(&shards[s], n, tmp);   /* substitution + outliers */
        if (rc) { free(tmp); return rc; }
#pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < (int64_t)n; ++j) {
            uint64_t o = (uint64_t)s * n + (uint64_t)j;
            if (dtype == ORACLE_F32)
                ((float *)out)[o] = tmp[j];
            else if (dtype == ORACLE_F16)
                ((uint16_t *)out)[o] = oracle_f32_to_f16(tmp[j]);
            else
                ((uint16_t *)out)[o] = oracle_f32_to_bf16(tmp[j]);
        }
    }
    free(tmp);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* Layer                                                               */
/* ------------------------------------------------------------------ */

/* out[t][n] = bias[n] + sum_c in[t][c] * W[n][c]   (W row-major [rows][cols]) */
static void linear_rows(double *out, int64_t ldo, const double *in, int64_t ldi, int64_t T,
                        const double *W, int64_t rows, int64_t cols, const float *bias)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t t = 0; t < T; ++t)
        for (int64_t n = 0; n < rows; ++n) {
            double acc = 0.0;
            for (int64_t c = 0; c < cols; ++c) acc += in[t * ldi + c] * W[n * cols + c];
            out[t * ldo + n] = acc + (bias ? (double)bias[n] : 0.0);
        }
}

/* acc[t][n] += sum_c in[t][c] * W[n][c] */
static void linear_rows_accumulate(double *acc_out, int64_t ldo, const double *in, int64_t ldi,
                                   int64_t T, const double *W, int64_t rows, int64_t cols)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t t = 0; t < T; ++t)
        for (int64_t n = 0; n < rows; ++n) {
            double acc = 0.0;
            for (int64_t c = 0; c < cols; ++c) acc += in[t * ldi + c] * W[n * cols + c];
            acc_out[t * ldo + n] += acc;
        }
}

/* y[t][:] = (v - mean) / sqrt(var + eps) * g + b, biased variance over d */
static void layer_norm_rows(double *y, const double *v, int64_t T, int64_t d, const float *g,
                            const float *b, double eps)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const double *r = v + t * d;
        double mean = 0.0;
        for (int64_t c = 0; c < d; ++c) mean += r[c];
        mean /= (double)d;
        double var = 0.0;
        for (int64_t c = 0; c < d; ++c) var += (r[c] - mean) * (r[c] - mean);
        var /= (double)d;
        double inv = 1.0 / sqrt(var + eps);
        for (int64_t c = 0; c < d; ++c)
            y[t * d + c] = (r[c] - mean) * inv * (double)g[c] + (double)b[c];
    }
}

static double gelu_erf(double z) { return z * 0.5 * (1.0 + erf(z / sqrt(2.0))); }

/* Attention of one head over one sequence: C = softmax(Q K^T / sqrt(dh)) V.
 * q, k, v, c are [L][dh] with row stride ld.  Only the first Lk keys take part (Lk = L for a
 * sequence without padding): a padded position gets no attention weight from any query. */
static void attention_head(double *c, const double *q, const double *k, const double *v, int64_t L,
                           int64_t Lk, int64_t dh, int64_t ld, double *score_rows /* [L][L] scratch */)
{
    double scale = 1.0 / sqrt((double)dh);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < L; ++i) {
        double *s = score_rows + i * L;
        double mx = -INFINITY;
        for (int64_t j = 0; j < Lk; ++j) {
            double acc = 0.0;
            for (int64_t e = 0; e < dh; ++e) acc += q[i * ld + e] * k[j * ld + e];
            s[j] = acc * scale;
            if (s[j] > mx) mx = s[j];
        }
        double den = 0.0;
        for (int64_t j = 0; j < Lk; ++j) {
            s[j] = exp(s[j] - mx);
            den += s[j];
        }
        for (int64_t j = 0; j < Lk; ++j) s[j] /= den;
        for (int64_t e = 0; e < dh; ++e) {
            double acc = 0.0;
            for (int64_t j = 0; j < Lk; ++j) acc += s[j] * v[j * ld + e];
            c[i * ld + e] = acc;
        }
    }
}

/* One encoder layer over the present shards.
 * shards[M]: bitwidth 0 marks an absent shard.  x, y: [B][L][d] double.
 * Optional taps (may be NULL), all [B*L][d] double:
 *   attn_out = b_o + sum_i C_i Wo_i^T          (before residual and LayerNorm)
 *   h_out    = LayerNorm1(x + attn)
 *   ffn_out  = b_2 + sum_i U_i W2_i^T          (before residual and LayerNorm) */
static int layer_forward_impl(int32_t d, int32_t M, int32_t dh, int32_t f, double eps,
                              const oracle_shard *shards, const oracle_layer_params *p,
                              const double *x, double *y, int32_t B, int32_t L,
                              const int32_t *key_lengths /* [B] or NULL */, double *attn_out,
                              double *h_out, double *ffn_out)
{
    if (!shards || !p || !x || !y) return ORACLE_ERR_ARG;
    if (d <= 0 || M <= 0 || dh <= 0 || f <= 0 || B < 0 || L < 0) return ORACLE_ERR_ARG;
    if (key_lengths)
        for (int32_t b = 0; b < B; ++b)
            if (key_lengths[b] < 1 || key_lengths[b] > L) return ORACLE_ERR_ARG;
    for (int i = 0; i < M; ++i) {
        int k = shards[i].bitwidth;
        if (k == 0) continue;
        if (k != 32 && (k < 2 || k > 6)) return ORACLE_ERR_ARG;
        if (!shards[i].data || (k != 32 && !shards[i].codebook)) return ORACLE_ERR_ARG;
    }
    int64_t T = (int64_t)B * L;
    uint64_t wsh = (uint64_t)d * (uint64_t)(4 * dh + 2 * f);
    int64_t off_q = 0, off_k = (int64_t)dh * d, off_v = 2 * (int64_t)dh * d,
            off_o = 3 * (int64_t)dh * d, off_1 = 4 * (int64_t)dh * d,
            off_2 = 4 * (int64_t)dh * d + (int64_t)f * d;

    float *w32 = (float *)malloc(wsh * sizeof(float));
    double *w = (double *)malloc(wsh * sizeof(double));
    double *q = (double *)malloc((size_t)(T > 0 ? T : 1) * dh * sizeof(double));
    double *kk = (double *)malloc((size_t)(T > 0 ? T : 1) * dh * sizeof(double));
    double *v = (double *)malloc((size_t)(T > 0 ? T : 1) * dh * sizeof(double));
    double *c = (double *)malloc((size_t)(T > 0 ? T : 1) * dh * sizeof(double));
    double *u = (double *)malloc((size_t)(T > 0 ? T : 1) * f * sizeof(double));
    double *sc = (double *)malloc((size_t)(L > 0 ? L : 1) * (L > 0 ? L : 1) * sizeof(double));
    double *attn = (double *)malloc((size_t)(T > 0 ? T : 1) * d * sizeof(double));
    double *h = (double *)malloc((size_t)(T > 0 ? T : 1) * d * sizeof(double));
    double *ffn = (double *)malloc((size_t)(T > 0 ? T : 1) * d * sizeof(double));
    int rc = ORACLE_OK;
    if (!w32 || !w || !q || !kk || !v || !c || !u || !sc || !attn || !h || !ffn) {
        rc = ORACLE_ERR_MEM;
        goto done;
    }

    /* attention block: attn = b_o + sum over present heads of C_i Wo_i^T */
    for (int64_t t = 0; t < T; ++t)
        for (int64_t n = 0; n < d; ++n) attn[t * d + n] = (double)p->bo[n];
    for (int i = 0; i < M; ++i) {
        if (shards[i].bitwidth == 0) continue;
        rc = oracle_decode_f32(&shards[i], wsh, w32);
        if (rc) goto done;
        for (uint64_t j = 0; j < wsh; ++j) w[j] = (double)w32[j];
        linear_rows(q, dh, x, d, T, w + off_q, dh, d, p->bq + (int64_t)i * dh);
        linear_rows(kk, dh, x, d, T, w + off_k, dh, d, p->bk + (int64_t)i * dh);
        linear_rows(v, dh, x, d, T, w + off_v, dh, d, p->bv + (int64_t)i * dh);
        for (int64_t b = 0; b < B; ++b)
            attention_head(c + b * L * dh, q + b * L * dh, kk + b * L * dh, v + b * L * dh, L,
                           key_lengths ? key_lengths[b] : L, dh, dh, sc);
        linear_rows_accumulate(attn, d, c, dh, T, w + off_o, d, dh);
    }
    if (attn_out) memcpy(attn_out, attn, (size_t)T * d * sizeof(double));
    for (int64_t e = 0; e < T * d; ++e) attn[e] += x[e];
    layer_norm_rows(h, attn, T, d, p->ln1_g, p->ln1_b, eps);
    if (h_out) memcpy(h_out, h, (size_t)T * d * sizeof(double));

    /* feed-forward block: ffn = b_2 + sum over present slices of U_i W2_i^T */
    for (int64_t t = 0; t < T; ++t)
        for (int64_t n = 0; n < d; ++n) ffn[t * d + n] = (double)p->b2[n];
    for (int i = 0; i < M; ++i) {
        if (shards[i].bitwidth == 0) continue;
        rc = oracle_decode_f32(&shards[i], wsh, w32);
        if (rc) goto done;
        for (uint64_t j = 0; j < wsh; ++j) w[j] = (double)w32[j];
        linear_rows(u, f, h, d, T, w + off_1, f, d, p->b1 + (int64_t)i * f);
        for (int64_t e = 0; e < T * f; ++e) u[e] = gelu_erf(u[e]);
        linear_rows_accumulate(ffn, d, u, f, T, w + off_2, d, f);
    }
    if (ffn_out) memcpy(ffn_out, ffn, (size_t)T * d * sizeof(double));
    for (int64_t e = 0; e < T * d; ++e) ffn[e] += h[e];
    layer_norm_rows(y, ffn, T, d, p->ln2_g, p->ln2_b, eps);

done:
    free(w32); free(w); free(q); free(kk); free(v); free(c); free(u); free(sc);
    free(attn); free(h); free(ffn);
    return rc;
}

int oracle_layer_forward_taps(int32_t d, int32_t M, int32_t dh, int32_t f, double eps,
                              const oracle_shard *shards, const oracle_layer_params *p,
                              const double *x, double *y, int32_t B, int32_t L, double *attn_out,
                              double *h_out, double *ffn_out)
{
    return layer_forward_impl(d, M, dh, f, eps, shards, p, x, y, B, L, NULL, attn_out, h_out, ffn_out);
}

int oracle_layer_forward(int32_t d, int32_t M, int32_t dh, int32_t f, double eps,
                         const oracle_shard *shards, const oracle_layer_params *p, const double *x,
                         double *y, int32_t B, int32_t L)
{
    return layer_forward_impl(d, M, dh, f, eps, shards, p, x, y, B, L, NULL, NULL, NULL, NULL);
}

/* Inputs padded to a common length (Section "Prerequisite: Offline Profiling": the length is
 * fixed after padding): sequence b holds key_lengths[b] real positions, 1 <= key_lengths[b] <= L,
 * followed by padding.  Padded positions are computed like any other row but no query attends
 * to them. */
int oracle_layer_forward_masked(int32_t d, int32_t M, int32_t dh, int32_t f, double eps,
                                const oracle_shard *shards, const oracle_layer_params *p,
                                const double *x, double *y, int32_t B, int32_t L,
                                const int32_t *key_lengths)
{
    if (!key_lengths) return ORACLE_ERR_ARG;
    return layer_forward_impl(d, M, dh, f, eps, shards, p, x, y, B, L, key_lengths, NULL, NULL, NULL);
}

/* Layers 0 .. n_layers-1 in order; shards is [n_layers][M], params [n_layers]. */
static int model_forward_impl(int32_t d, int32_t M, int32_t dh, int32_t f, double eps, int32_t n_layers,
                              const oracle_shard *shards, const oracle_layer_params *params,
                              const double *x, double *y, int32_t B, int32_t L,
                              const int32_t *key_lengths)
{
    if (n_layers < 0 || !x || !y) return ORACLE_ERR_ARG;
    size_t n = (size_t)B * L * d;
    double *cur = (double *)malloc((n ? n : 1) * sizeof(double));
    double *nxt = (double *)malloc((n ? n : 1) * sizeof(double));
    if (!cur || !nxt) { free(cur); free(nxt); return ORACLE_ERR_MEM; }
    memcpy(cur, x, n * sizeof(double));
    int rc = ORACLE_OK;
    for (int l = 0; l < n_layers && rc == ORACLE_OK; ++l) {
        rc = layer_forward_impl(d, M, dh, f, eps, shards + (size_t)l * M, &params[l], cur, nxt, B, L,
                                key_lengths, NULL, NULL, NULL);
        double *t = cur; cur = nxt; nxt = t;
    }
    if (rc == ORACLE_OK) memcpy(y, cur, n * sizeof(double));
    free(cur); free(nxt);
    return rc;
}

int oracle_model_forward(int32_t d, int32_t M, int32_t dh, int32_t f, double eps, int32_t n_layers,
                         const oracle_shard *shards, const oracle_layer_params *params,
                         const double *x, double *y, int32_t B, int32_t L)
{
    return model_forward_impl(d, M, dh, f, eps, n_layers, shards, params, x, y, B, L, NULL);
}

/* The same key lengths in every layer. */
int oracle_model_forward_masked(int32_t d, int32_t M, int32_t dh, int32_t f, double eps,
                                int32_t n_layers, const oracle_shard *shards,
                                const oracle_layer_params *params, const double *x, double *y,
                                int32_t B, int32_t L, const int32_t *key_lengths)
{
    if (!key_lengths) return ORACLE_ERR_ARG;
    return model_forward_impl(d, M, dh, f, eps, n_layers, shards, params, x, y, B, L, key_lengths);
}
