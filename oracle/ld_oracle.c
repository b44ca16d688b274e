/*
 * CPU oracle for the decode / chunked-prefill path of a decoder-only transformer
 * over a paged KV cache.  TEST INFRASTRUCTURE ONLY: it is called by the tests, by
 * the smoke check and by the benchmark's CPU-baseline leg, never by the product.
 * It shares no code with the GPU library.
 *
 * What it computes (paper section 2.1: each token's query is multiplied with the
 * keys of all preceding tokens, followed by a softmax and a weighted average of
 * the values; keys and values of processed tokens are cached; a request runs as a
 * prefill phase over the prompt and an autoregressive decode phase; section 2.2
 * step (g): tool observations are concatenated after prompt and plan and fed back;
 * section 4.1: temperature 0, i.e. greedy).  The paper does not describe the
 * decoder block; the block used here (RMSNorm, rotary position embedding in the
 * half-split pairing, SwiGLU, no biases, untied LM head) is the one fixed by the
 * workload definitions.  Section 4.1 names a model family whose attention is
 * grouped (several query heads per key/value head) and banded: with window W > 0 a
 * token at position p attends to positions max(0, p - W + 1) .. p only; W = 0 means
 * every preceding position.  The cache still keeps every position.
 *
 * Arithmetic: every floating-point step is done in double precision, one token at
 * a time, two-pass softmax, plain loops.  Weights are read as fp32 or as bf16 bit
 * patterns (both exact in double).  Keys and values are optionally rounded to the
 * storage grid of the cache (bf16 or fp32, round-to-nearest-even) when they are
 * appended, because the cache's element type is part of the data-structure
 * contract; with kv_round = 0 the cache keeps doubles (the pure definition).
 *
 * Parity status: every function below is pinned by tests/test_oracle_pins.py
 * (closed forms, invariants, library routines in float64, brute force).  The one
 * exception is the greedy token sequence on the full 7B/13B shapes, for which no
 * published values exist: "parity unpinned" beyond the agreement of this file with
 * the float64 whole-sequence re-derivation on the small shape.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_E_INVAL (-1)
#define ORC_E_NOMEM (-2)
#define ORC_E_STATE (-3)
#define ORC_E_RANGE (-5)

typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
    double rms_eps, rope_base;
    int32_t wdtype;   /* 0: matrices are float32, 1: matrices are bf16 bit patterns (uint16) */
    int32_t kv_round; /* 0: cache keeps doubles, 1: round k,v to bf16 on append, 2: round to fp32 */
    int32_t kv_block; /* tokens per cache block */
    int32_t window;   /* > 0: attend to the last `window` positions (own position included); 0: all */
} orc_config;

typedef struct {
    const void *embed, *lm_head;
    const float *final_norm;
    const float *const *attn_norm;
    const void *const *wqkv;
    const void *const *wo;
    const float *const *ffn_norm;
    const void *const *wgate_up;
    const void *const *wdown;
} orc_weights;

typedef struct {
    orc_config c;
    orc_weights w;
    const float **attn_norm, **ffn_norm;
    const void **wqkv, **wo, **wgate_up, **wdown;
} orc_model;

/* ---------------------------------------------------------------- scalars */

static double bf16_bits_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* Round a double to the nearest value with an 8-bit significand (bf16 grid),
 * ties to even, directly from double (no intermediate float rounding). */
double orc_round_bf16(double x)
{
    if (x == 0.0 || !isfinite(x)) return x;
    int e;
    double m = frexp(x, &e);             /* x = m * 2^e, 0.5 <= |m| < 1 */
    int shift = 8;
    if (e < -125) shift = 8 - (-125 - e); /* bf16 subnormals: fewer bits */
    if (shift < 0) return copysign(0.0, x);
    double r = nearbyint(ldexp(m, shift)); /* default rounding mode: nearest even */
    return ldexp(r, e - shift);
}

double orc_round_f32(double x) { return (double)(float)x; }

static double round_kv(double x, int mode)
{
    return mode == 1 ? orc_round_bf16(x) : mode == 2 ? orc_round_f32(x) : x;
}

static inline double welem(const void *w, int wdtype, int64_t i)
{
    return wdtype ? bf16_bits_to_double(((const uint16_t *)w)[i]) : (double)((const float *)w)[i];
}

/* ---------------------------------------------------------------- steps */

/* out_i = x_i / sqrt(mean_j x_j^2 + eps) * g_i  (eps inside the square root). */
void orc_rmsnorm(const double *x, const float *g, int32_t d, double eps, double *out)
{
    double ss = 0.0;
    for (int i = 0; i < d; i++) ss += x[i] * x[i];
    double r = 1.0 / sqrt(ss / d + eps);
    for (int i = 0; i < d; i++) out[i] = x[i] * r * (double)g[i];
}

/* Rotary embedding of one head at absolute position pos (0-based), in place.
 * Pair i is (u_i, u_{i+hd/2}), rotated by the angle pos * base^(-2i/hd). */
void orc_rope_head(double *u, int32_t hd, int64_t pos, double base)
{
    int half = hd / 2;
    for (int i = 0; i < half; i++) {
        double theta = pow(base, -2.0 * i / hd);
        double ang = (double)pos * theta;
        double c = cos(ang), s = sin(ang);
        double a = u[i], b = u[i + half];
        u[i] = a * c - b * s;
        u[i + half] = a * s + b * c;
    }
}

/* y = W x, W row-major [n, k]. */
void orc_matvec(const void *w, int32_t wdtype, int64_t n, int64_t k, const double *x, double *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n; r++) {
        double acc = 0.0;
        if (wdtype) {
            const uint16_t *row = (const uint16_t *)w + r * k;
#pragma omp simd reduction(+ : acc)
            for (int64_t j = 0; j < k; j++) {
                uint32_t u = (uint32_t)row[j] << 16;
                float f;
                memcpy(&f, &u, 4);
                acc += (double)f * x[j];
            }
        } else {
            const float *row = (const float *)w + r * k;
#pragma omp simd reduction(+ : acc)
            for (int64_t j = 0; j < k; j++) acc += (double)row[j] * x[j];
        }
        y[r] = acc;
    }
}

/* In place: s_j <- exp(s_j - max) / sum. */
void orc_softmax(double *s, int64_t n)
{
    double m = s[0];
    for (int64_t j = 1; j < n; j++) if (s[j] > m) m = s[j];
    double sum = 0.0;
    for (int64_t j = 0; j < n; j++) { s[j] = exp(s[j] - m); sum += s[j]; }
    for (int64_t j = 0; j < n; j++) s[j] /= sum;
}

double orc_silu(double z) { return z / (1.0 + exp(-z)); }

/* Smallest index attaining the maximum. */
int32_t orc_argmax(const double *x, int64_t n)
{
    int64_t best = 0;
    for (int64_t i = 1; i < n; i++) if (x[i] > x[best]) best = i;
    return (int32_t)best;
}

/* Sampling at temperature T > 0 (the paper decodes at temperature 0, section 4.1; this is the same
 * decision with noise): the token is argmax_i (logit_i / T + g_i) with independent standard Gumbel noise
 * g_i = -log(-log(u_i)), which draws i with probability softmax(logits / T)_i.  The uniforms come from a
 * counter-based generator, so a draw is a pure function of (seed, counter): u = (k + 1/2) / 2^23 with k
 * the top 23 bits of the SplitMix64 output function applied to seed + (counter + 1) * 0x9E3779B97F4A7C15
 * (Steele, Lea, Flood 2014).  The counter of vocabulary entry i for the token that will sit at position
 * pos is pos * n + i.  Smallest index on ties, as for the plain argmax. */
double orc_uniform(uint64_t seed, uint64_t counter)
{
    uint64_t z = seed + (counter + 1) * 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    z = z ^ (z >> 31);
    return ((double)(z >> 41) + 0.5) / 8388608.0;
}

int32_t orc_sample_gumbel(const double *logits, int64_t n, double temperature, uint64_t seed, int64_t pos)
{
    int64_t best = 0;
    double best_v = 0.0;
    for (int64_t i = 0; i < n; i++) {
        double u = orc_uniform(seed, (uint64_t)pos * (uint64_t)n + (uint64_t)i);
        double v = logits[i] / temperature - log(-log(u));
        if (i == 0 || v > best_v) { best = i; best_v = v; }
    }
    return (int32_t)best;
}

/* The scores orc_sample_gumbel takes the argmax of, written out: out[i] = logits[i] / T + g_i for the token
 * that will sit at position pos.  For the tests' near-tie diagnosis (how far apart were the two candidates
 * the decision was between); the sampler above does not call it. */
void orc_gumbel_scores(const double *logits, int64_t n, double temperature, uint64_t seed, int64_t pos, double *out)
{
    for (int64_t i = 0; i < n; i++) {
        double u = orc_uniform(seed, (uint64_t)pos * (uint64_t)n + (uint64_t)i);
        out[i] = logits[i] / temperature - log(-log(u));
    }
}

/* One query against n cached (key, value) rows given by pointer tables:
 * scores q.k_j / sqrt(hd), softmax, weighted average of the values. */
static void attend_rows(const double *q, const double *const *krow, const double *const *vrow,
                        int64_t n, int32_t hd, double *scores, double *out)
{
    double scale = 1.0 / sqrt((double)hd);
    for (int64_t j = 0; j < n; j++) {
        double s = 0.0;
        for (int i = 0; i < hd; i++) s += q[i] * krow[j][i];
        scores[j] = s * scale;
    }
    orc_softmax(scores, n);
    for (int i = 0; i < hd; i++) out[i] = 0.0;
    for (int64_t j = 0; j < n; j++)
        for (int i = 0; i < hd; i++) out[i] += scores[j] * vrow[j][i];
}

/* Contiguous single-head attention: K, V are [n, hd] doubles. */
void orc_attention_contig(const double *q, const double *K, const double *V, int64_t n, int32_t hd,
                          double *out)
{
    const double **kr = malloc(sizeof(*kr) * n), **vr = malloc(sizeof(*vr) * n);
    double *sc = malloc(sizeof(double) * n);
    for (int64_t j = 0; j < n; j++) { kr[j] = K + j * hd; vr[j] = V + j * hd; }
    attend_rows(q, kr, vr, n, hd, sc, out);
    free(kr); free(vr); free(sc);
}

/* Stand-alone paged attention for a batch of single-token queries.
 * q [B, H, hd] doubles.  The pools hold float32 (elem=0) or bf16 bit patterns (elem=1);
 * element (block, kv_head, slot, i) of a pool sits at
 *   block*stride_block + kv_head*stride_head + slot*stride_slot + i   (in elements).
 * block_table [B, table_stride]; ctx_len [B]; out [B, H, hd] doubles.
 * Token j of sequence b lives in physical block block_table[b][j / kv_block], slot j % kv_block. */
void orc_paged_attention(const double *q, const void *kpool, const void *vpool, int32_t elem,
                         int64_t stride_block, int64_t stride_head, int64_t stride_slot,
                         const int32_t *block_table, int32_t table_stride, const int32_t *ctx_len,
                         int32_t B, int32_t H, int32_t Hkv, int32_t hd, int32_t kv_block, int32_t window,
                         double *out)
{
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; b++) {
        for (int h = 0; h < H; h++) {
            /* the query is the token at position ctx_len - 1; it sees positions first .. ctx_len - 1 */
            int64_t last = ctx_len[b], first = (window > 0 && last > window) ? last - window : 0;
            int64_t n = last - first;
            int kvh = h / (H / Hkv);
            double *K = malloc(sizeof(double) * n * hd), *V = malloc(sizeof(double) * n * hd);
            for (int64_t j = 0; j < n; j++) {
                int64_t pos = first + j;
                int64_t blk = block_table[(int64_t)b * table_stride + pos / kv_block];
                int64_t off = blk * stride_block + kvh * stride_head + (pos % kv_block) * stride_slot;
                for (int i = 0; i < hd; i++) {
                    K[j * hd + i] = welem(kpool, elem, off + i);
                    V[j * hd + i] = welem(vpool, elem, off + i);
                }
            }
            orc_attention_contig(q + ((int64_t)b * H + h) * hd, K, V, n, hd,
                                 out + ((int64_t)b * H + h) * hd);
            free(K); free(V);
        }
    }
}

/* ---------------------------------------------------------------- model */

orc_model *orc_model_create(const orc_config *c, const orc_weights *w)
{
    if (!c || !w) return NULL;
    if (c->n_heads % c->n_kv_heads || c->head_dim % 2 || c->kv_block <= 0 || c->window < 0) return NULL;
    orc_model *m = calloc(1, sizeof(*m));
    m->c = *c;
    m->w = *w;
    int L = c->n_layers;
    m->attn_norm = malloc(sizeof(void *) * (L + 1)); m->ffn_norm = malloc(sizeof(void *) * (L + 1));
    m->wqkv = malloc(sizeof(void *) * (L + 1)); m->wo = malloc(sizeof(void *) * (L + 1));
    m->wgate_up = malloc(sizeof(void *) * (L + 1)); m->wdown = malloc(sizeof(void *) * (L + 1));
    for (int l = 0; l < L; l++) {
        m->attn_norm[l] = w->attn_norm[l]; m->ffn_norm[l] = w->ffn_norm[l];
        m->wqkv[l] = w->wqkv[l]; m->wo[l] = w->wo[l];
        m->wgate_up[l] = w->wgate_up[l]; m->wdown[l] = w->wdown[l];
    }
    return m;
}

void orc_model_destroy(orc_model *m)
{
    if (!m) return;
    free(m->attn_norm); free(m->ffn_norm); free(m->wqkv); free(m->wo); free(m->wgate_up); free(m->wdown);
    free(m);
}

/* The cache a token's forward pass appends to and reads from.  Two storage schemes
 * with identical arithmetic: a contiguous array indexed by position, or a paged pool
 * reached through a block table. */
typedef struct {
    int paged;
    /* contiguous: [layer][pos][2][kv_head][hd] */
    double *flat; int64_t flat_cap;
    /* paged: pool [layer][block][2][kv_head][slot][hd], table of physical block ids */
    double *pool; int64_t n_blocks; const int32_t *table;
} kv_view;

static double *kv_row(const orc_config *c, const kv_view *v, int layer, int which, int kvh, int64_t pos)
{
    int hd = c->head_dim, Hk = c->n_kv_heads;
    if (!v->paged)
        return v->flat + ((((int64_t)layer * v->flat_cap + pos) * 2 + which) * Hk + kvh) * hd;
    int64_t blk = v->table[pos / c->kv_block];
    int64_t slot = pos % c->kv_block;
    return v->pool + (((((int64_t)layer * v->n_blocks + blk) * 2 + which) * Hk + kvh) * c->kv_block + slot) * hd;
}

/* Forward pass of one token at absolute position pos.  Appends its keys and values to
 * the cache, attends over positions 0..pos (the last `window` of them if the model is
 * banded), and (if logits != NULL) writes the vocab logits of this position. */
static void forward_token(const orc_model *m, const kv_view *kv, int32_t token, int64_t pos, double *logits)
{
    const orc_config *c = &m->c;
    int d = c->d_model, H = c->n_heads, Hk = c->n_kv_heads, hd = c->head_dim, F = c->d_ffn;
    int nq = H * hd, nkv = Hk * hd, nqkv = nq + 2 * nkv;
    double *x = malloc(sizeof(double) * d), *h = malloc(sizeof(double) * d);
    double *qkv = malloc(sizeof(double) * nqkv), *att = malloc(sizeof(double) * nq);
    double *tmp = malloc(sizeof(double) * d), *gu = malloc(sizeof(double) * 2 * F), *a = malloc(sizeof(double) * F);
    int64_t first = (c->window > 0 && pos + 1 > c->window) ? pos + 1 - c->window : 0;
    int64_t n = pos + 1 - first;   /* visible positions: first .. pos */

    for (int i = 0; i < d; i++) x[i] = welem(m->w.embed, c->wdtype, (int64_t)token * d + i);

    for (int l = 0; l < c->n_layers; l++) {
        orc_rmsnorm(x, m->attn_norm[l], d, c->rms_eps, h);
        orc_matvec(m->wqkv[l], c->wdtype, nqkv, d, h, qkv);
        double *q = qkv, *k = qkv + nq, *v = qkv + nq + nkv;
        for (int hh = 0; hh < H; hh++) orc_rope_head(q + hh * hd, hd, pos, c->rope_base);
        for (int hh = 0; hh < Hk; hh++) orc_rope_head(k + hh * hd, hd, pos, c->rope_base);
        for (int hh = 0; hh < Hk; hh++) {
            double *kd = kv_row(c, kv, l, 0, hh, pos), *vd = kv_row(c, kv, l, 1, hh, pos);
            for (int i = 0; i < hd; i++) {
                kd[i] = round_kv(k[hh * hd + i], c->kv_round);
                vd[i] = round_kv(v[hh * hd + i], c->kv_round);
            }
        }
#pragma omp parallel for schedule(static)
        for (int hh = 0; hh < H; hh++) {
            int kvh = hh / (H / Hk);
            const double **kr = malloc(sizeof(*kr) * n), **vr = malloc(sizeof(*vr) * n);
            double *sc = malloc(sizeof(double) * n);
            for (int64_t j = 0; j < n; j++) {
                kr[j] = kv_row(c, kv, l, 0, kvh, first + j);
                vr[j] = kv_row(c, kv, l, 1, kvh, first + j);
            }
            attend_rows(q + hh * hd, kr, vr, n, hd, sc, att + hh * hd);
            free(kr); free(vr); free(sc);
        }
        orc_matvec(m->wo[l], c->wdtype, d, nq, att, tmp);
        for (int i = 0; i < d; i++) x[i] += tmp[i];

        orc_rmsnorm(x, m->ffn_norm[l], d, c->rms_eps, h);
        orc_matvec(m->wgate_up[l], c->wdtype, 2 * (int64_t)F, d, h, gu);
        for (int i = 0; i < F; i++) a[i] = orc_silu(gu[i]) * gu[F + i];
        orc_matvec(m->wdown[l], c->wdtype, d, F, a, tmp);
        for (int i = 0; i < d; i++) x[i] += tmp[i];
    }
    if (logits) {
        orc_rmsnorm(x, m->w.final_norm, d, c->rms_eps, h);
        orc_matvec(m->w.lm_head, c->wdtype, c->vocab, d, h, logits);
    }
    free(x); free(h); free(qkv); free(att); free(tmp); free(gu); free(a);
}

/* Whole sequence through a contiguous cache; logits_all [n, vocab] (every position). */
int32_t orc_forward_contig(const orc_model *m, const int32_t *tokens, int64_t n, double *logits_all)
{
    const orc_config *c = &m->c;
    for (int64_t p = 0; p < n; p++) if (tokens[p] < 0 || tokens[p] >= c->vocab) return ORC_E_RANGE;
    kv_view v = {0};
    v.flat_cap = n;
    v.flat = calloc((size_t)c->n_layers * n * 2 * c->n_kv_heads * c->head_dim, sizeof(double));
    if (!v.flat) return ORC_E_NOMEM;
    for (int64_t p = 0; p < n; p++) forward_token(m, &v, tokens[p], p, logits_all + p * c->vocab);
    free(v.flat);
    return ORC_OK;
}

/* ---------------------------------------------------------------- paged cache + sequence state
 *
 * Block allocator policy: the free list is a LIFO stack whose first pops return
 * 0, 1, 2, ...; a block is popped when a token is fed at a position whose logical
 * block has no physical block yet; freeing a sequence pushes its blocks back in
 * reverse logical order, so the next allocation gets them back in logical order.
 * Sequence state: n_cached tokens have their keys/values in the pool; `pending` is a
 * token that was emitted but not fed yet. */
typedef struct {
    int active, stopped, has_pending;
    int32_t pending;
    int64_t n_cached;
    int32_t n_mapped;
    int32_t first_block;  /* logical blocks below it were released by orc_kv_trim (attention band) */
    int32_t *table;
    int swapped;      /* keys/values live outside the pool; no block is held */
    double temperature; uint64_t seed;   /* temperature 0: greedy */
} orc_seq;

typedef struct {
    const orc_model *m;
    int64_t n_blocks;
    int32_t max_seqs, max_blocks_per_seq;
    double *pool;
    int32_t *free_stack; int64_t n_free;
    int32_t *refs;    /* sequences holding each block (prefix sharing); 0 = on the free list */
    orc_seq *seqs;
} orc_kv;

orc_kv *orc_kv_create(const orc_model *m, int64_t n_blocks, int32_t max_seqs, int32_t max_blocks_per_seq)
{
    if (!m || n_blocks <= 0 || max_seqs <= 0 || max_blocks_per_seq <= 0) return NULL;
    const orc_config *c = &m->c;
    orc_kv *kv = calloc(1, sizeof(*kv));
    kv->m = m; kv->n_blocks = n_blocks; kv->max_seqs = max_seqs; kv->max_blocks_per_seq = max_blocks_per_seq;
    size_t per_block = (size_t)2 * c->n_kv_heads * c->kv_block * c->head_dim;
    kv->pool = calloc((size_t)c->n_layers * n_blocks * per_block, sizeof(double));
    kv->free_stack = malloc(sizeof(int32_t) * n_blocks);
    kv->refs = calloc(n_blocks, sizeof(int32_t));
    for (int64_t i = 0; i < n_blocks; i++) kv->free_stack[i] = (int32_t)(n_blocks - 1 - i);
    kv->n_free = n_blocks;
    kv->seqs = calloc(max_seqs, sizeof(orc_seq));
    for (int s = 0; s < max_seqs; s++) {
        kv->seqs[s].table = malloc(sizeof(int32_t) * max_blocks_per_seq);
        for (int i = 0; i < max_blocks_per_seq; i++) kv->seqs[s].table[i] = -1;
    }
    if (!kv->pool) { free(kv); return NULL; }
    return kv;
}

void orc_kv_destroy(orc_kv *kv)
{
    if (!kv) return;
    for (int s = 0; s < kv->max_seqs; s++) free(kv->seqs[s].table);
    free(kv->seqs); free(kv->free_stack); free(kv->refs); free(kv->pool); free(kv);
}

static orc_seq *get_seq(orc_kv *kv, int32_t s)
{
    if (s < 0 || s >= kv->max_seqs || !kv->seqs[s].active) return NULL;
    return &kv->seqs[s];
}

/* Make sure logical blocks first_block..need-1 of a sequence have physical blocks. */
static int ensure_blocks(orc_kv *kv, orc_seq *q, int64_t need)
{
    if (need > kv->max_blocks_per_seq) return ORC_E_RANGE;
    int64_t missing = 0;
    for (int64_t i = q->first_block; i < need; i++) if (q->table[i] < 0) missing++;
    if (missing > kv->n_free) return ORC_E_NOMEM;
    for (int64_t i = q->first_block; i < need; i++)
        if (q->table[i] < 0) { q->table[i] = kv->free_stack[--kv->n_free]; kv->refs[q->table[i]] = 1; }
    if (need > q->n_mapped) q->n_mapped = (int32_t)need;
    return ORC_OK;
}

/* Drop every block a sequence holds, last logical block first; a block goes back to the free list when
 * its last holder drops it. */
static void release_blocks(orc_kv *kv, orc_seq *q)
{
    for (int i = kv->max_blocks_per_seq - 1; i >= 0; i--)
        if (q->table[i] >= 0) {
            if (--kv->refs[q->table[i]] == 0) kv->free_stack[kv->n_free++] = q->table[i];
            q->table[i] = -1;
        }
    q->n_mapped = 0;
}

/* Sliding-window memory (the model family of section 4.1 attends to a band of W positions): the blocks
 * whose positions all lie below n_cached - W + 1 can be seen by no later query of the sequence (the next
 * one sits at position n_cached) and are given up, lowest logical block first; a shared block returns to
 * the free list when its last holder gives it up.  Without a band nothing is released. */
int32_t orc_kv_trim(orc_kv *kv, int32_t s, int32_t *released)
{
    orc_seq *q = get_seq(kv, s);
    if (!q || !released) return ORC_E_INVAL;
    if (q->swapped) return ORC_E_STATE;
    *released = 0;
    const orc_config *c = &kv->m->c;
    int64_t low = q->n_cached - c->window + 1;
    if (c->window <= 0 || low <= 0) return ORC_OK;
    int64_t keep_from = low / c->kv_block;
    for (int64_t i = q->first_block; i < keep_from; i++)
        if (q->table[i] >= 0) {
            if (--kv->refs[q->table[i]] == 0) kv->free_stack[kv->n_free++] = q->table[i];
            q->table[i] = -1;
            (*released)++;
        }
    if (keep_from > q->first_block) q->first_block = (int32_t)keep_from;
    return ORC_OK;
}

int32_t orc_kv_alloc(orc_kv *kv, int64_t reserve_tokens, int32_t *out)
{
    if (reserve_tokens < 0) return ORC_E_INVAL;
    int s = 0;
    while (s < kv->max_seqs && kv->seqs[s].active) s++;
    if (s == kv->max_seqs) return ORC_E_NOMEM;
    orc_seq *q = &kv->seqs[s];
    int bs = kv->m->c.kv_block;
    q->n_mapped = 0; q->first_block = 0;
    int rc = ensure_blocks(kv, q, (reserve_tokens + bs - 1) / bs);
    if (rc) return rc;
    q->active = 1; q->stopped = 0; q->has_pending = 0; q->pending = -1; q->n_cached = 0; q->swapped = 0;
    q->temperature = 0.0; q->seed = 0;
    *out = s;
    return ORC_OK;
}

/* Test hook: force logical block -> physical block (takes the block out of the free list). */
int32_t orc_kv_map(orc_kv *kv, int32_t s, int32_t logical, int32_t physical)
{
    orc_seq *q = get_seq(kv, s);
    if (!q || logical < 0 || logical >= kv->max_blocks_per_seq) return ORC_E_INVAL;
    if (q->table[logical] >= 0) return ORC_E_STATE;
    int64_t at = -1;
    for (int64_t i = 0; i < kv->n_free; i++) if (kv->free_stack[i] == physical) { at = i; break; }
    if (at < 0) return ORC_E_NOMEM;
    memmove(kv->free_stack + at, kv->free_stack + at + 1, sizeof(int32_t) * (kv->n_free - at - 1));
    kv->n_free--;
    kv->refs[physical] = 1;
    q->table[logical] = physical;
    if (logical + 1 > q->n_mapped) q->n_mapped = logical + 1;
    return ORC_OK;
}

int32_t orc_kv_free(orc_kv *kv, int32_t s)
{
    orc_seq *q = get_seq(kv, s);
    if (!q) return ORC_E_INVAL;
    release_blocks(kv, q);
    q->active = 0; q->swapped = 0;
    return ORC_OK;
}

int32_t orc_kv_block_table(orc_kv *kv, int32_t s, int32_t *out, int32_t cap, int32_t *n)
{
    orc_seq *q = get_seq(kv, s);
    if (!q) return ORC_E_INVAL;
    if (cap < q->n_mapped) return ORC_E_RANGE;
    for (int i = 0; i < q->n_mapped; i++) out[i] = q->table[i];
    *n = q->n_mapped;
    return ORC_OK;
}

int64_t orc_kv_free_blocks(const orc_kv *kv) { return kv->n_free; }
int64_t orc_kv_len(orc_kv *kv, int32_t s) { orc_seq *q = get_seq(kv, s); return q ? q->n_cached : -1; }

/* Test hook: declare that the next n positions of a sequence are already cached, with keys and
 * values given as [n, layers, 2, kv_heads, hd] doubles (stored as given), and set the pending token. */
int32_t orc_kv_inject(orc_kv *kv, int32_t s, const double *kvdata, int64_t n, int32_t pending)
{
    orc_seq *q = get_seq(kv, s);
    const orc_config *c = &kv->m->c;
    if (!q || n < 0) return ORC_E_INVAL;
    if (q->swapped) return ORC_E_STATE;
    int rc = ensure_blocks(kv, q, (q->n_cached + n + c->kv_block - 1) / c->kv_block);
    if (rc) return rc;
    kv_view v = {0};
    v.paged = 1; v.pool = kv->pool; v.n_blocks = kv->n_blocks; v.table = q->table;
    int hd = c->head_dim, Hk = c->n_kv_heads;
    for (int64_t p = 0; p < n; p++)
        for (int l = 0; l < c->n_layers; l++)
            for (int w = 0; w < 2; w++)
                for (int hh = 0; hh < Hk; hh++)
                    memcpy(kv_row(c, &v, l, w, hh, q->n_cached + p),
                           kvdata + ((((p * c->n_layers + l) * 2 + w) * Hk) + hh) * hd, sizeof(double) * hd);
    q->n_cached += n;
    if (pending >= 0) { q->has_pending = 1; q->pending = pending; }
    return ORC_OK;
}

/* Read back one cached (key or value) row, for block-indexing checks. */
int32_t orc_kv_read(orc_kv *kv, int32_t s, int32_t layer, int32_t which, int32_t kvh, int64_t pos, double *out)
{
    orc_seq *q = get_seq(kv, s);
    const orc_config *c = &kv->m->c;
    if (!q || pos < 0 || pos >= q->n_cached) return ORC_E_INVAL;
    if (q->swapped || pos < (int64_t)q->first_block * c->kv_block) return ORC_E_STATE;
    kv_view v = {0};
    v.paged = 1; v.pool = kv->pool; v.n_blocks = kv->n_blocks; v.table = q->table;
    memcpy(out, kv_row(c, &v, layer, which, kvh, pos), sizeof(double) * c->head_dim);
    return ORC_OK;
}

/* KV retention across a tool call (section 2.2 describes systems that keep, swap to host memory or
 * discard the cache of a request that waits for a tool): swapping a sequence out moves the keys and values of its cached
 * positions from the pool into `store` and returns every block it holds to the free list in the order
 * orc_kv_free uses; the token state (length, pending token) stays.  Swapping in takes blocks for the
 * cached length in the order a reservation would and copies the contents back.  While swapped out the
 * sequence cannot be stepped.  store: [logical block][layer][2][kv_head][slot][hd] doubles,
 * orc_kv_swap_doubles() of them. */
static int64_t seq_token_blocks(const orc_kv *kv, const orc_seq *q)
{
    int bs = kv->m->c.kv_block;
    return (q->n_cached + bs - 1) / bs;
}
static size_t block_doubles(const orc_kv *kv)
{
    const orc_config *c = &kv->m->c;
    return (size_t)2 * c->n_kv_heads * c->kv_block * c->head_dim;
}
int64_t orc_kv_swap_doubles(orc_kv *kv, int32_t s)
{
    orc_seq *q = get_seq(kv, s);
    if (!q) return -1;
    return seq_token_blocks(kv, q) * kv->m->c.n_layers * (int64_t)block_doubles(kv);
}
int32_t orc_kv_swap_out(orc_kv *kv, int32_t s, double *store)
{
    orc_seq *q = get_seq(kv, s);
    if (!q || !store) return ORC_E_INVAL;
    if (q->swapped) return ORC_E_STATE;
    size_t per = block_doubles(kv);
    int L = kv->m->c.n_layers;
    int64_t nb = seq_token_blocks(kv, q);
    for (int64_t j = q->first_block; j < nb; j++)      /* released blocks: their part of the store is not written */
        for (int l = 0; l < L; l++)
            memcpy(store + (j * L + l) * per, kv->pool + ((size_t)l * kv->n_blocks + q->table[j]) * per,
                   sizeof(double) * per);
    release_blocks(kv, q);
    q->swapped = 1;
    return ORC_OK;
}
int32_t orc_kv_swap_in(orc_kv *kv, int32_t s, const double *store)
{
    orc_seq *q = get_seq(kv, s);
    if (!q || !store) return ORC_E_INVAL;
    if (!q->swapped) return ORC_E_STATE;
    int64_t nb = seq_token_blocks(kv, q);
    int rc = ensure_blocks(kv, q, nb);
    if (rc) return rc;
    size_t per = block_doubles(kv);
    int L = kv->m->c.n_layers;
    for (int64_t j = q->first_block; j < nb; j++)
        for (int l = 0; l < L; l++)
            memcpy(kv->pool + ((size_t)l * kv->n_blocks + q->table[j]) * per, store + (j * L + l) * per,
                   sizeof(double) * per);
    q->swapped = 0;
    return ORC_OK;
}

/* Prefix sharing (section 2.1 serves many requests at once; section 4.3 puts the same tool descriptions
 * into every prompt): a new sequence that starts with the first n_tokens cached positions of `parent`.
 * Blocks that the prefix fills completely are shared (their holder count goes up; nothing ever writes a
 * full block again); a last, partly filled block is copied into a block of the child's own, because both
 * sequences will append into their copy.  The child has no pending token. */
int32_t orc_kv_fork(orc_kv *kv, int32_t parent, int64_t n_tokens, int32_t *out)
{
    orc_seq *p = get_seq(kv, parent);
    if (!p || !out || n_tokens < 0 || n_tokens > p->n_cached) return ORC_E_INVAL;
    if (p->swapped) return ORC_E_STATE;
    int s = 0;
    while (s < kv->max_seqs && kv->seqs[s].active) s++;
    if (s == kv->max_seqs) return ORC_E_NOMEM;
    int bs = kv->m->c.kv_block;
    int64_t full = n_tokens / bs, tail = n_tokens % bs;
    if (p->first_block > 0) {   /* the child's next query must not need a block the parent has released */
        int64_t low = n_tokens - kv->m->c.window + 1;
        if ((low < 0 ? 0 : low) / bs < p->first_block) return ORC_E_STATE;
    }
    if (tail && kv->n_free < 1) return ORC_E_NOMEM;
    orc_seq *q = &kv->seqs[s];
    q->active = 1; q->stopped = 0; q->has_pending = 0; q->pending = -1; q->swapped = 0;
    q->temperature = 0.0; q->seed = 0;
    q->n_cached = n_tokens; q->n_mapped = (int32_t)(full + (tail ? 1 : 0));
    q->first_block = p->first_block;
    for (int64_t j = p->first_block; j < full; j++) { q->table[j] = p->table[j]; kv->refs[p->table[j]]++; }
    if (tail) {
        int32_t nb = kv->free_stack[--kv->n_free];
        kv->refs[nb] = 1;
        q->table[full] = nb;
        size_t per = block_doubles(kv);
        for (int l = 0; l < kv->m->c.n_layers; l++)
            memcpy(kv->pool + ((size_t)l * kv->n_blocks + nb) * per,
                   kv->pool + ((size_t)l * kv->n_blocks + p->table[full]) * per, sizeof(double) * per);
    }
    *out = s;
    return ORC_OK;
}

static int feed_tokens(orc_kv *kv, orc_seq *q, const int32_t *tok, int64_t n, double *logits_last)
{
    const orc_config *c = &kv->m->c;
    for (int64_t i = 0; i < n; i++) if (tok[i] < 0 || tok[i] >= c->vocab) return ORC_E_RANGE;
    int rc = ensure_blocks(kv, q, (q->n_cached + n + c->kv_block - 1) / c->kv_block);
    if (rc) return rc;
    kv_view v = {0};
    v.paged = 1; v.pool = kv->pool; v.n_blocks = kv->n_blocks; v.table = q->table;
    for (int64_t i = 0; i < n; i++) {
        forward_token(kv->m, &v, tok[i], q->n_cached, i == n - 1 ? logits_last : NULL);
        q->n_cached++;
    }
    return ORC_OK;
}

/* Prefill: feed [pending?] ++ tokens at the next positions, in order; emit the greedy token of the
 * last position, which becomes the new pending token.  logits_out [vocab] may be NULL. */
int32_t orc_prefill(orc_kv *kv, int32_t s, const int32_t *tokens, int64_t n, double *logits_out, int32_t *next)
{
    orc_seq *q = get_seq(kv, s);
    if (!q || n < 0 || (n == 0 && !q->has_pending)) return ORC_E_INVAL;
    if (q->stopped || q->swapped) return ORC_E_STATE;
    int64_t tot = n + (q->has_pending ? 1 : 0);
    int32_t *all = malloc(sizeof(int32_t) * tot);
    int64_t k = 0;
    if (q->has_pending) all[k++] = q->pending;
    for (int64_t i = 0; i < n; i++) all[k++] = tokens[i];
    double *lg = malloc(sizeof(double) * kv->m->c.vocab);
    int rc = feed_tokens(kv, q, all, tot, lg);
    if (rc == ORC_OK) {
        /* the emitted token will sit at position n_cached */
        q->pending = q->temperature > 0.0
                         ? orc_sample_gumbel(lg, kv->m->c.vocab, q->temperature, q->seed, q->n_cached)
                         : orc_argmax(lg, kv->m->c.vocab);
        q->has_pending = 1;
        if (next) *next = q->pending;
        if (logits_out) memcpy(logits_out, lg, sizeof(double) * kv->m->c.vocab);
    }
    free(all); free(lg);
    return rc;
}

/* Temperature and seed of a sequence's token choice (temperature 0: greedy, the default). */
int32_t orc_seq_set_sampling(orc_kv *kv, int32_t s, double temperature, uint64_t seed)
{
    orc_seq *q = get_seq(kv, s);
    if (!q || !(temperature >= 0.0)) return ORC_E_INVAL;
    q->temperature = temperature; q->seed = seed;
    return ORC_OK;
}

/* Decode: feed the pending token, emit the next one. */
int32_t orc_decode(orc_kv *kv, int32_t s, double *logits_out, int32_t *next)
{
    orc_seq *q = get_seq(kv, s);
    if (!q) return ORC_E_INVAL;
    if (q->stopped || q->swapped || !q->has_pending) return ORC_E_STATE;
    return orc_prefill(kv, s, NULL, 0, logits_out, next);
}

int32_t orc_seq_stop(orc_kv *kv, int32_t s)
{
    orc_seq *q = get_seq(kv, s);
    if (!q) return ORC_E_INVAL;
    q->stopped = 1;
    return ORC_OK;
}
