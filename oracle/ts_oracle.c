/*
 * TEST INFRASTRUCTURE -- fp64 CPU oracle for the mixed paged-attention pass.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call this file.
 * It shares no code with the GPU library and never receives data produced by it.
 *
 * What it computes (the paper defines the batch, not the arithmetic; Sec. 2.1 says the
 * prefill phase builds the KV cache for all input tokens and each decode iteration adds
 * the last token's entry and reuses the rest; Sec. 3.4 / Sec. 4.4 put a chunked prefill
 * next to the decode batch of a Convertible Decoder):
 *
 *   append : for sequence s, new token i sits at position pos = prefix_s + i,
 *            prefix_s = ctx_len_s - q_len_s; it is stored in page block_table[s][pos/16],
 *            slot pos%16, for every KV head, after conversion to the cache element type.
 *   attend : query token i of sequence s, query head h, sees the n = prefix_s + i + 1 first
 *            keys of its sequence, through KV head h / (Hq/Hkv):
 *              z_j = sm_scale * <q, k_j>,  w_j = exp(z_j - max z),  out = sum w_j v_j / sum w_j.
 *
 * Everything is evaluated in double, one (row, head) at a time, straight from the definition.
 * Parity status: the paper prints no value for this path; the functions here are pinned by
 * the tests in tests/test_oracle_pins.py (dense brute force, closed forms, invariants,
 * exhaustive e4m3 nearest-value search).
 *
 * Cache element order (a choice of this library, the paper is silent): per (page, kv head)
 *   K tile: [D/x][16 slots][x]  with x = 16 bytes / element size  (dim-chunks of 16 bytes)
 *   V tile: [D][16 slots]       (token index fastest)
 * tiles ordered [page][kv head].
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { OR_F32 = 0, OR_BF16 = 1, OR_FP8_E4M3 = 2 };
#define OR_PAGE 16

typedef struct {
    int32_t num_q_heads, num_kv_heads, head_dim;
    int32_t q_dtype, kv_dtype;
    int64_t num_pages;
    int32_t max_pages_per_seq;
} or_desc;

static int elem_size(int dt) { return dt == OR_F32 ? 4 : (dt == OR_BF16 ? 2 : 1); }

/* ---- element decoders ------------------------------------------------------------------ */

double or_e4m3_to_double(uint8_t b)
{
    int sign = b >> 7, e = (b >> 3) & 15, m = b & 7;
    double v;
    if (e == 15 && m == 7) return NAN;               /* the only NaN pattern; there is no inf */
    if (e == 0) v = ldexp((double)m / 8.0, -6);      /* subnormal: m/8 * 2^-6 */
    else        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

static double bf16_to_double(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

static double load_elem(const void *base, int64_t idx, int dt)
{
    if (dt == OR_F32)  return (double)((const float *)base)[idx];
    if (dt == OR_BF16) return bf16_to_double(((const uint16_t *)base)[idx]);
    return or_e4m3_to_double(((const uint8_t *)base)[idx]);
}

static float load_as_float(const void *base, int64_t idx, int dt)
{
    if (dt == OR_F32) return ((const float *)base)[idx];
    return (float)bf16_to_double(((const uint16_t *)base)[idx]);
}

/* ---- e4m3 encoder: fp32 divide by the scale, then nearest-even onto the e4m3 grid -------- */

uint8_t or_e4m3_encode(float x, float scale)
{
    volatile float yf = x / scale;                   /* IEEE single division, rounded once */
    double y = (double)yf;
    uint8_t sign = signbit(y) ? 0x80 : 0x00;
    double a = fabs(y);
    if (isnan(y)) return sign | 0x7F;
    if (a >= 448.0) return sign | 0x7E;              /* saturate (also +-inf) to +-448 */
    if (a < ldexp(1.0, -6)) {                        /* subnormal range, spacing 2^-9 */
        int q = (int)nearbyint(ldexp(a, 9));         /* ties to even; q = 8 is the first normal */
        return sign | (uint8_t)q;
    }
    int ex;
    (void)frexp(a, &ex);                             /* a = f * 2^ex, f in [0.5,1) */
    int e = ex - 1;                                  /* a in [2^e, 2^(e+1)) */
    int q = (int)nearbyint(ldexp(a, 3 - e));         /* in [8,16], ties to even */
    if (q == 16) { q = 8; e += 1; }
    if (e > 8 || (e == 8 && q > 14)) return sign | 0x7E;
    return sign | (uint8_t)(((e + 7) << 3) | (q - 8));
}

/* ---- cache addressing ------------------------------------------------------------------ */

static int64_t k_index(const or_desc *d, int64_t page, int g, int slot, int dim)
{
    int x = 16 / elem_size(d->kv_dtype);
    int64_t tile = page * d->num_kv_heads + g;
    return (tile * (d->head_dim / x) + dim / x) * (OR_PAGE * x) + (int64_t)slot * x + dim % x;
}

static int64_t v_index(const or_desc *d, int64_t page, int g, int slot, int dim)
{
    int64_t tile = page * d->num_kv_heads + g;
    return (tile * d->head_dim + dim) * OR_PAGE + slot;
}

static void store_elem(void *cache, int64_t idx, int kv_dt, const void *src, int64_t sidx, int q_dt,
                       float scale)
{
    if (kv_dt == OR_F32)       ((float *)cache)[idx] = ((const float *)src)[sidx];
    else if (kv_dt == OR_BF16) ((uint16_t *)cache)[idx] = ((const uint16_t *)src)[sidx];
    else ((uint8_t *)cache)[idx] = or_e4m3_encode(load_as_float(src, sidx, q_dt), scale);
}

static int check_desc(const or_desc *d)
{
    if (d->num_q_heads <= 0 || d->num_kv_heads <= 0 || d->num_q_heads % d->num_kv_heads) return -1;
    if (d->head_dim <= 0 || d->head_dim % 16) return -1;
    if (d->kv_dtype == OR_F32 && d->q_dtype != OR_F32) return -1;
    if (d->kv_dtype == OR_BF16 && d->q_dtype != OR_BF16) return -1;
    if (d->kv_dtype == OR_FP8_E4M3 && d->q_dtype != OR_BF16 && d->q_dtype != OR_F32) return -1;
    return 0;
}

/* ---- append ---------------------------------------------------------------------------- */

int or_kv_append(const or_desc *d, const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                 const float *k_scale, const float *v_scale, const int32_t *block_table,
                 const int32_t *q_lens, const int32_t *ctx_lens, int num_seqs)
{
    if (check_desc(d)) return -1;
    int64_t row = 0;
    for (int s = 0; s < num_seqs; ++s) {
        int prefix = ctx_lens[s] - q_lens[s];
        if (q_lens[s] < 0 || prefix < 0) return -1;
        for (int i = 0; i < q_lens[s]; ++i, ++row) {
            int pos = prefix + i;
            if (pos / OR_PAGE >= d->max_pages_per_seq) return -2;
            int64_t page = block_table[(int64_t)s * d->max_pages_per_seq + pos / OR_PAGE];
            int slot = pos % OR_PAGE;
            if (page < 0 || page >= d->num_pages) return -3;
            for (int g = 0; g < d->num_kv_heads; ++g) {
                float ks = d->kv_dtype == OR_FP8_E4M3 ? k_scale[g] : 1.0f;
                float vs = d->kv_dtype == OR_FP8_E4M3 ? v_scale[g] : 1.0f;
                for (int dim = 0; dim < d->head_dim; ++dim) {
                    int64_t sidx = (row * d->num_kv_heads + g) * d->head_dim + dim;
                    store_elem(k_cache, k_index(d, page, g, slot, dim), d->kv_dtype, k_new, sidx,
                               d->q_dtype, ks);
                    store_elem(v_cache, v_index(d, page, g, slot, dim), d->kv_dtype, v_new, sidx,
                               d->q_dtype, vs);
                }
            }
        }
    }
    return 0;
}

/* ---- one (row, head) of attention ------------------------------------------------------ */

/* q_row: index of the query token in q [T,Hq,D]; bt_row: the sequence's page list; n_keys: how
 * many keys this row sees.  weights (may be NULL) receives the n_keys normalised weights. */
int or_attention_row(const or_desc *d, const void *q, const void *k_cache, const void *v_cache,
                     const float *k_scale, const float *v_scale, const int32_t *bt_row, int n_keys,
                     int64_t q_row, int h, double sm_scale, double *weights, double *out)
{
    int D = d->head_dim, G = d->num_q_heads / d->num_kv_heads, g = h / G;
    double ks = d->kv_dtype == OR_FP8_E4M3 ? (double)k_scale[g] : 1.0;
    double vs = d->kv_dtype == OR_FP8_E4M3 ? (double)v_scale[g] : 1.0;
    double *z = (double *)malloc(sizeof(double) * (size_t)(n_keys > 0 ? n_keys : 1));
    if (!z) return -4;
    double zmax = -INFINITY;
    for (int j = 0; j < n_keys; ++j) {
        int64_t page = bt_row[j / OR_PAGE];
        if (page < 0 || page >= d->num_pages) { free(z); return -3; }
        double acc = 0.0;
        for (int dim = 0; dim < D; ++dim) {
            double qv = load_elem(q, (q_row * d->num_q_heads + h) * D + dim, d->q_dtype);
            double kv = load_elem(k_cache, k_index(d, page, g, j % OR_PAGE, dim), d->kv_dtype) * ks;
            acc += qv * kv;
        }
        z[j] = sm_scale * acc;
        if (z[j] > zmax) zmax = z[j];
    }
    double denom = 0.0;
    for (int j = 0; j < n_keys; ++j) { z[j] = exp(z[j] - zmax); denom += z[j]; }
    for (int dim = 0; dim < D; ++dim) out[dim] = 0.0;
    for (int j = 0; j < n_keys; ++j) {
        int64_t page = bt_row[j / OR_PAGE];
        double w = z[j] / denom;
        if (weights) weights[j] = w;
        for (int dim = 0; dim < D; ++dim)
            out[dim] += w * (load_elem(v_cache, v_index(d, page, g, j % OR_PAGE, dim), d->kv_dtype) * vs);
    }
    free(z);
    return 0;
}

/* ---- the whole pass: every query token of every sequence, every head --------------------- */

/* Attends from the cache as it stands (run or_kv_append first for "append then attend").
 * out: double [T,Hq,D].  row_stride/row_offset select rows row_offset, row_offset+row_stride, ...
 * (row_stride = 1, row_offset = 0 for all rows) so that a bounded sample can be timed. */
int or_mixed_paged_attention(const or_desc *d, const void *q, const void *k_cache, const void *v_cache,
                             const float *k_scale, const float *v_scale, const int32_t *block_table,
                             const int32_t *q_lens, const int32_t *ctx_lens, int num_seqs,
                             double sm_scale, double *out, int64_t row_stride, int64_t row_offset)
{
    if (check_desc(d)) return -1;
    if (row_stride < 1) row_stride = 1;
    int64_t T = 0;
    for (int s = 0; s < num_seqs; ++s) {
        if (q_lens[s] < 0 || ctx_lens[s] < q_lens[s]) return -1;
        if ((ctx_lens[s] + OR_PAGE - 1) / OR_PAGE > d->max_pages_per_seq) return -2;
        T += q_lens[s];
    }
    if (T == 0) return 0;
    int32_t *row_seq = (int32_t *)malloc(sizeof(int32_t) * (size_t)T);
    int32_t *row_keys = (int32_t *)malloc(sizeof(int32_t) * (size_t)T);
    if (!row_seq || !row_keys) { free(row_seq); free(row_keys); return -4; }
    int64_t r = 0;
    for (int s = 0; s < num_seqs; ++s)
        for (int i = 0; i < q_lens[s]; ++i, ++r) {
            row_seq[r] = s;
            row_keys[r] = ctx_lens[s] - q_lens[s] + i + 1;
        }
    int H = d->num_q_heads, D = d->head_dim, rc = 0;
    int64_t n_rows = (T - row_offset + row_stride - 1) / row_stride;
    if (row_offset >= T) n_rows = 0;
    #pragma omp parallel for schedule(dynamic, 1)
    for (int64_t it = 0; it < n_rows * H; ++it) {
        int64_t row = row_offset + (it / H) * row_stride;
        int h = (int)(it % H);
        int e = or_attention_row(d, q, k_cache, v_cache, k_scale, v_scale,
                                 block_table + (int64_t)row_seq[row] * d->max_pages_per_seq,
                                 row_keys[row], row, h, sm_scale, NULL, out + (row * H + h) * D);
        if (e) {
            #pragma omp critical
            rc = e;
        }
    }
    free(row_seq);
    free(row_keys);
    return rc;
}

int or_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    #pragma omp parallel
    {
        #pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
