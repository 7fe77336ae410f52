/*
 * CPU oracle for one step of SUN's shared decode module.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU
 * library is checked against.  It shares no code with the HIP path and must
 * never be called from it; only the test-suite, the smoke check and the
 * benchmark's cpu-baseline leg may load it.
 *
 * What it computes: the decode module D_theta_d of Section 3.1 (Eq. 3): given
 * the most recent token y_{t-1} of every request and the KV cache of all
 * previously processed positions, produce the next-token logits and the KV
 * entry of the new position, which is appended to the cache (Eq. 4).  All
 * requests of a batch use the same decode parameters whatever prefill model
 * produced their cache (Section 3.2.1), so requests are evaluated
 * independently of one another and of their source-model tag.  QSUN (Section
 * 3.3, Eq. 8) is the same step with weight-only quantised projections: 4-bit
 * codes, groups of 128 along the input dimension, lm_head left unquantised
 * (Appendix A.1, "Quantization Configurations").
 *
 * The paper does not spell out the block; it names LLaMA-3.1 / Qwen3 class
 * decoder-only Transformers (Section 4).  The block evaluated here is the
 * pre-norm Llama block: RMSNorm, GQA attention with rotary embedding
 * (half-split pairing), SwiGLU feed-forward, final RMSNorm, untied lm_head.
 *
 * Arithmetic: every stored input (weights, embedding, cached K/V) is used at
 * the value it is stored with; everything computed is IEEE double.  The new
 * K/V entry is rounded to bfloat16 (round to nearest even) before it is
 * written and before this step attends to it, so the step consumes exactly
 * what later steps will read.  cos/sin of the rotary angle are evaluated in
 * double from a double angle and then rounded to float.
 * act_bf16 is NOT the definition any GPU parity test compares with (all of them
 * use the unrounded step above).  It is a second, separately pinned reading of
 * "16-bit" kept for sensitivity measurements only: the vector fed to each
 * projection (normalised hidden state, attention output, SwiGLU product) is
 * rounded to bfloat16 first, as in a deployment whose activations are 16-bit;
 * sums, the residual stream, softmax and norms stay double.  At the 8B shape its
 * logits lie 0.13 to 0.16 from the unrounded ones, which is why the GPU path
 * carries activations as two bf16 planes instead.
 *
 * orc_decode_step_peer is a harness option, like the forced tokens of a run: the
 * same step computed next to another implementation's cache, adopting that
 * implementation's stored bf16 code for a new entry where it is this step's own
 * rounding, its neighbour, or within a given bound (see stored_code), so that one
 * legitimate rounding flip is not carried through the remaining layers into
 * everything compared after it.
 *
 * Pins (see tests, "not gpu"): causal full forward == prefill + decode
 * (Eq. 1 vs Eq. 2+3 with theta_p = theta_d), library special cases
 * (scaled-dot-product attention, rms_norm, silu, matmul, complex rotation),
 * paged == contiguous, softmax row sums, Eq. 4 append, batch-mix invariance,
 * exact dequantisation on the integer grid, the peer rule entry by entry and
 * against the primitives chained by hand.
 * Parity unpinned: none of the functions; absolute logit values at the large
 * shapes have no reference other than these properties.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_F64 = 2, ORC_W4 = 3 };
enum { ORC_OK = 0, ORC_ERR_ARG = 1, ORC_ERR_PAGE = 2, ORC_ERR_TOKEN = 3, ORC_ERR_ALLOC = 4 };

typedef struct {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
    double rms_eps, rope_base;
    int32_t act_bf16; /* 16-bit configuration: the input of every projection is a bf16 value */
    int32_t qk_norm;  /* backbone option (Qwen3 class): RMSNorm over head_dim on every q and k head, with its
                         own gain per layer, applied before the rotation */
    int32_t rope_scaling;  /* backbone option (LLaMA-3.1 class): 0 = none, 1 = frequency-dependent scaling */
    int32_t rope_orig_max; /* original context length of the scaling rule */
    double rope_factor, rope_low_freq, rope_high_freq;
    int32_t qkv_bias;      /* backbone option (Qwen2 class): q, k and v projections add a bias vector */
    int32_t pad_;
} orc_cfg;

/* One parameter tensor, row-major [rows, cols]; y = M x contracts over cols. */
typedef struct {
    int32_t kind;        /* ORC_F32 | ORC_BF16 | ORC_F64 | ORC_W4 */
    int32_t rows, cols;
    int32_t group;       /* ORC_W4: group length along cols */
    const void *data;    /* dense kinds */
    const uint8_t *q;    /* ORC_W4: codes, [rows, cols/2], low nibble = even column */
    const uint16_t *s;   /* ORC_W4: fp16 scales  [rows, ceil(cols/group)] */
    const uint16_t *z;   /* ORC_W4: fp16 zero points, same shape */
} orc_mat;

/* Parameter table: mats[0]=E, then 14 per layer (g1,Wq,Wk,Wv,Wo,g2,Wg,Wu,Wd, the
 * head-norm gains qn, kn of length head_dim, read only under qk_norm, and the projection
 * biases bq, bk, bv, read only under qkv_bias), then g_f, W_lm. */
enum { M_G1 = 0, M_WQ, M_WK, M_WV, M_WO, M_G2, M_WG, M_WU, M_WD, M_QN, M_KN, M_BQ, M_BK, M_BV, M_PER_LAYER };
#define MAT_E(m) (&(m)[0])
#define MAT_L(m, l, w) (&(m)[1 + (l) * M_PER_LAYER + (w)])
#define MAT_GF(m, nl) (&(m)[1 + (nl) * M_PER_LAYER])
#define MAT_LM(m, nl) (&(m)[2 + (nl) * M_PER_LAYER])

/* bf16 KV pool addressed by element strides; K and V have separate strides. */
typedef struct {
    uint16_t *base;
    int64_t n_pages;
    int32_t page_tokens;
    int32_t pad_;
    int64_t k_off, k_layer, k_page, k_head, k_token, k_dim;
    int64_t v_off, v_layer, v_page, v_head, v_token, v_dim;
} orc_pool;

/* ---------- number formats ---------- */

static double bf16_to_double(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* Round a double to the nearest bfloat16 (ties to even), directly. */
static uint16_t double_to_bf16(double x) {
    if (isnan(x)) return 0x7FC0;
    float f = (float)x; /* used only for sign/inf/zero and as a starting point */
    if (isinf(f) || x == 0.0) {
        uint32_t u;
        memcpy(&u, &f, 4);
        return (uint16_t)(u >> 16);
    }
    /* Candidate by truncation of |x| toward zero in bf16, then pick the nearer
     * of it and its successor in exact double arithmetic. */
    double ax = fabs(x);
    float ft = (float)ax;
    if ((double)ft > ax) ft = nextafterf(ft, 0.0f);
    uint32_t u;
    memcpy(&u, &ft, 4);
    uint32_t lo = u & 0xFFFF0000u, hi = lo + 0x00010000u;
    float flo, fhi;
    memcpy(&flo, &lo, 4);
    memcpy(&fhi, &hi, 4);
    double dlo = ax - (double)flo, dhi = (double)fhi - ax;
    uint32_t pick;
    if (dlo < dhi) pick = lo;
    else if (dhi < dlo) pick = hi;
    else pick = ((lo >> 16) & 1u) ? hi : lo;
    uint16_t r = (uint16_t)(pick >> 16);
    if (x < 0) r |= 0x8000;
    return r;
}

static float half_to_float(uint16_t h) {
    uint32_t sign = (uint32_t)(h >> 15) & 1u, e = (h >> 10) & 0x1Fu, m = h & 0x3FFu;
    double v;
    if (e == 0) v = ldexp((double)m, -24);
    else if (e == 31) v = m ? NAN : INFINITY;
    else v = ldexp((double)(m | 0x400u), (int)e - 25);
    return (float)(sign ? -v : v);
}

/* float -> IEEE half, round to nearest even. */
static uint16_t float_to_half(float f) {
    if (isnan(f)) return 0x7E00;
    uint16_t sign = signbit(f) ? 0x8000 : 0;
    double a = fabs((double)f);
    if (a >= 65520.0) return sign | 0x7C00; /* rounds to inf */
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e); /* a = m * 2^e, m in [0.5,1) */
    int q = e - 11;     /* quantum exponent for 11 significant bits */
    if (q < -24) q = -24;
    double scaled = ldexp(a, -q);
    double r = nearbyint(scaled); /* ties to even in the default rounding mode */
    double v = ldexp(r, q);
    /* re-encode v, which is exactly representable */
    if (v == 0.0) return sign;
    (void)frexp(v, &e);
    int be = e - 1 + 15;
    if (be <= 0) return sign | (uint16_t)ldexp(v, 24);
    uint32_t mant = (uint32_t)ldexp(v, 11 - e) & 0x3FFu;
    return sign | (uint16_t)(be << 10) | (uint16_t)mant;
}

/* ---------- parameter access ---------- */

static int mat_groups(const orc_mat *m) { return (m->cols + m->group - 1) / m->group; }

/* Value of entry (r,c).  For ORC_W4 this is (Q - Z) * S evaluated in float,
 * which is exact: |Q-Z| <= 15 needs 4 bits, an fp16 scale has 11. */
static double mat_get(const orc_mat *m, int64_t r, int64_t c) {
    switch (m->kind) {
    case ORC_F32: return (double)((const float *)m->data)[r * m->cols + c];
    case ORC_BF16: return bf16_to_double(((const uint16_t *)m->data)[r * m->cols + c]);
    case ORC_F64: return ((const double *)m->data)[r * m->cols + c];
    default: {
        uint8_t byte = m->q[r * (int64_t)(m->cols / 2) + c / 2];
        int code = (c & 1) ? (byte >> 4) : (byte & 15);
        int64_t g = r * (int64_t)mat_groups(m) + c / m->group;
        float w = ((float)code - half_to_float(m->z[g])) * half_to_float(m->s[g]);
        return (double)w;
    }
    }
}

/* Y[b][r] = sum_c M[r][c] X[b][c], c ascending, one double accumulator. */
static void linear(const orc_mat *m, const double *X, int B, double *Y) {
    const int R = m->rows, C = m->cols;
#pragma omp parallel
    {
        double *row = (double *)malloc(sizeof(double) * (size_t)C);
#pragma omp for schedule(static)
        for (int r = 0; r < R; ++r) {
            for (int c = 0; c < C; ++c) row[c] = mat_get(m, r, c);
            for (int b = 0; b < B; ++b) {
                const double *x = X + (size_t)b * C;
                double acc = 0.0;
                for (int c = 0; c < C; ++c) acc += row[c] * x[c];
                Y[(size_t)b * R + r] = acc;
            }
        }
        free(row);
    }
}

/* h = x * rsqrt(mean(x^2) + eps) * g */
static void rmsnorm(const orc_mat *g, const double *x, int n, double eps, double *h) {
    double ss = 0.0;
    for (int j = 0; j < n; ++j) ss += x[j] * x[j];
    double r = 1.0 / sqrt(ss / n + eps);
    for (int j = 0; j < n; ++j) h[j] = x[j] * r * mat_get(g, 0, j);
}

/* Rotation frequency of pair j: base^(-2j/d), and under the LLaMA-3.1 rule rescaled by wavelength:
 * pairs whose wavelength is below orig/high_freq keep their frequency, pairs above orig/low_freq
 * are slowed by `factor`, and in between the two are blended linearly in orig/wavelength. */
static double rope_freq(const orc_cfg *c, int j) {
    const double pi = 3.14159265358979323846;
    double f = pow(c->rope_base, -2.0 * j / c->head_dim);
    if (c->rope_scaling != 1) return f;
    double wavelen = 2.0 * pi / f, orig = (double)c->rope_orig_max;
    if (wavelen < orig / c->rope_high_freq) return f;
    if (wavelen > orig / c->rope_low_freq) return f / c->rope_factor;
    double smooth = (orig / wavelen - c->rope_low_freq) / (c->rope_high_freq - c->rope_low_freq);
    return (1.0 - smooth) * f / c->rope_factor + smooth * f;
}

/* Rotary embedding of one head vector u[d] at 0-based position pos; pairs
 * (j, j+d/2), theta_j = rope_freq(j). */
static void rope(const orc_cfg *cf, double *u, int64_t pos) {
    int d = cf->head_dim, half = d / 2;
    for (int j = 0; j < half; ++j) {
        double theta = rope_freq(cf, j);
        double ang = (double)pos * theta;
        double c = (double)(float)cos(ang), s = (double)(float)sin(ang);
        double a = u[j], b = u[j + half];
        u[j] = a * c - b * s;
        u[j + half] = b * c + a * s;
    }
}

/* q and k heads of one position: optional head norm, then the rotation at pos */
static void norm_and_rotate(const orc_cfg *c, const orc_mat *mats, int l, double *q, double *k, int64_t pos) {
    const int d = c->head_dim;
    double tmp[1024];
    for (int h = 0; h < c->n_q_heads + c->n_kv_heads; ++h) {
        double *u = h < c->n_q_heads ? q + (size_t)h * d : k + (size_t)(h - c->n_q_heads) * d;
        if (c->qk_norm) {
            rmsnorm(MAT_L(mats, l, h < c->n_q_heads ? M_QN : M_KN), u, d, c->rms_eps, tmp);
            memcpy(u, tmp, sizeof(double) * d);
        }
        rope(c, u, pos);
    }
}

static double silu(double z) { return z / (1.0 + exp(-z)); }

/* q, k, v of B rows: the three projections of the normed input, plus their bias vectors if the block has them */
static void qkv_project(const orc_cfg *c, const orc_mat *mats, int l, const double *Hn, int B, double *Q, double *K,
                        double *V) {
    double *out[3] = {Q, K, V};
    const int width[3] = {c->n_q_heads * c->head_dim, c->n_kv_heads * c->head_dim, c->n_kv_heads * c->head_dim};
    for (int w = 0; w < 3; ++w) {
        linear(MAT_L(mats, l, M_WQ + w), Hn, B, out[w]);
        if (c->qkv_bias)
            for (int b = 0; b < B; ++b)
                for (int j = 0; j < width[w]; ++j) out[w][(size_t)b * width[w] + j] += mat_get(MAT_L(mats, l, M_BQ + w), 0, j);
    }
}

/* 16-bit configuration: a projection consumes bf16 activations. */
static void act_round(const orc_cfg *c, double *x, size_t n) {
    if (!c->act_bf16) return;
    for (size_t i = 0; i < n; ++i) x[i] = bf16_to_double(double_to_bf16(x[i]));
}

/* ---------- attention over one request, one layer ---------- */

/* softmax-weighted sum for one query head: scores[0..n-1] already scaled. */
static double softmax_inplace(double *s, int64_t n) {
    double m = s[0];
    for (int64_t t = 1; t < n; ++t) if (s[t] > m) m = s[t];
    double sum = 0.0;
    for (int64_t t = 0; t < n; ++t) { s[t] = exp(s[t] - m); sum += s[t]; }
    double check = 0.0;
    for (int64_t t = 0; t < n; ++t) { s[t] /= sum; check += s[t]; }
    return check;
}

/* Contiguous cache: Kc,Vc are [n][Hkv][d] doubles for this layer. */
static void attend_contig(const orc_cfg *c, const double *q, const double *Kc, const double *Vc,
                          int64_t n, double *a, double *rowsum, double *scratch) {
    const int d = c->head_dim, G = c->n_q_heads / c->n_kv_heads, Hkv = c->n_kv_heads;
    const double scale = 1.0 / sqrt((double)d);
    for (int h = 0; h < c->n_q_heads; ++h) {
        int kvh = h / G;
        for (int64_t t = 0; t < n; ++t) {
            const double *k = Kc + ((size_t)t * Hkv + kvh) * d;
            double acc = 0.0;
            for (int j = 0; j < d; ++j) acc += q[h * d + j] * k[j];
            scratch[t] = acc * scale;
        }
        double rs = softmax_inplace(scratch, n);
        if (rowsum) rowsum[h] = rs;
        for (int j = 0; j < d; ++j) {
            double acc = 0.0;
            for (int64_t t = 0; t < n; ++t) acc += scratch[t] * Vc[((size_t)t * Hkv + kvh) * d + j];
            a[h * d + j] = acc;
        }
    }
}

static uint16_t *pool_k(const orc_pool *p, int layer, int64_t page, int head, int slot) {
    return p->base + p->k_off + layer * p->k_layer + page * p->k_page + head * p->k_head + slot * p->k_token;
}
static uint16_t *pool_v(const orc_pool *p, int layer, int64_t page, int head, int slot) {
    return p->base + p->v_off + layer * p->v_layer + page * p->v_page + head * p->v_head + slot * p->v_token;
}

/* Paged cache: token t of the request lives in page pt[t / P], slot t % P.
 * Query heads h0 <= h < h1 (heads are independent of one another). */
static void attend_paged(const orc_cfg *c, const orc_pool *p, int layer, const int32_t *pt,
                         const double *q, int64_t n, double *a, double *rowsum, double *scratch, int h0, int h1) {
    const int d = c->head_dim, G = c->n_q_heads / c->n_kv_heads, P = p->page_tokens;
    const double scale = 1.0 / sqrt((double)d);
    for (int h = h0; h < h1; ++h) {
        int kvh = h / G;
        for (int64_t t = 0; t < n; ++t) {
            const uint16_t *k = pool_k(p, layer, pt[t / P], kvh, (int)(t % P));
            double acc = 0.0;
            for (int j = 0; j < d; ++j) acc += q[h * d + j] * bf16_to_double(k[j * p->k_dim]);
            scratch[t] = acc * scale;
        }
        double rs = softmax_inplace(scratch, n);
        if (rowsum) rowsum[h] = rs;
        for (int j = 0; j < d; ++j) {
            double acc = 0.0;
            for (int64_t t = 0; t < n; ++t) {
                const uint16_t *v = pool_v(p, layer, pt[t / P], kvh, (int)(t % P));
                acc += scratch[t] * bf16_to_double(v[j * p->v_dim]);
            }
            a[h * d + j] = acc;
        }
    }
}

/* ---------- shared pieces of the block ---------- */

static int32_t argmax_lowest(const double *v, int n) {
    int32_t best = 0;
    for (int i = 1; i < n; ++i) if (v[i] > v[best]) best = i;
    return best;
}

static int embed_rows(const orc_cfg *c, const orc_mat *mats, int B, const int32_t *tokens, double *X) {
    for (int b = 0; b < B; ++b) {
        if (tokens[b] < 0 || tokens[b] >= c->vocab) return ORC_ERR_TOKEN;
        for (int j = 0; j < c->hidden; ++j) X[(size_t)b * c->hidden + j] = mat_get(MAT_E(mats), tokens[b], j);
    }
    return ORC_OK;
}

/* x += Wd (silu(Wg h) * (Wu h)), h = rmsnorm(x; g2), for all rows of X. */
static void feed_forward(const orc_cfg *c, const orc_mat *mats, int l, int B, double *X,
                         double *Hn, double *Gt, double *Up, double *Dn) {
    const int H = c->hidden, F = c->ffn;
    for (int b = 0; b < B; ++b) rmsnorm(MAT_L(mats, l, M_G2), X + (size_t)b * H, H, c->rms_eps, Hn + (size_t)b * H);
    act_round(c, Hn, (size_t)B * H);
    linear(MAT_L(mats, l, M_WG), Hn, B, Gt);
    linear(MAT_L(mats, l, M_WU), Hn, B, Up);
    for (size_t i = 0; i < (size_t)B * F; ++i) Gt[i] = silu(Gt[i]) * Up[i];
    act_round(c, Gt, (size_t)B * F);
    linear(MAT_L(mats, l, M_WD), Gt, B, Dn);
    for (size_t i = 0; i < (size_t)B * H; ++i) X[i] += Dn[i];
}

static void final_logits(const orc_cfg *c, const orc_mat *mats, int B, const double *X, double *Hn,
                         double *logits, int32_t *next) {
    const int H = c->hidden, V = c->vocab, NL = c->n_layers;
    for (int b = 0; b < B; ++b) rmsnorm(MAT_GF(mats, NL), X + (size_t)b * H, H, c->rms_eps, Hn + (size_t)b * H);
    act_round(c, Hn, (size_t)B * H);
    linear(MAT_LM(mats, NL), Hn, B, logits);
    if (next) for (int b = 0; b < B; ++b) next[b] = argmax_lowest(logits + (size_t)b * V, V);
}

/* ---------- the decode step over a paged bf16 pool ---------- */

/*
 * One decode step for B requests (Eq. 3).  seq_lens[i] = L_i tokens already
 * cached; the new token sits at position L_i, its K/V (bf16-rounded) is written
 * to slot L_i % P of page page_tables[i][L_i / P] in every layer (Eq. 4), and
 * attention spans positions 0..L_i.  model_ids are accepted and ignored: the
 * decode parameters do not depend on them (Section 3.2.1).
 * mode 0: attention walks the page table.  mode 1: the request's cache is first
 * gathered into a contiguous array and attention runs on that.
 * logits: [B, vocab] doubles.  next: [B] or NULL.  rowsums: [B, NL, Hq] or NULL,
 * receives the sum of each softmax row.  attn_probe: [B, NL, Hq*d] or NULL,
 * receives the attention output of every layer.
 */
/* monotone integer code of a bf16 bit pattern: neighbouring values differ by one */
static int32_t bf16_ordered(uint16_t u) { return (u & 0x8000) ? -(int32_t)(u & 0x7FFF) : (int32_t)(u & 0x7FFF); }

/*
 * The entry the step stores for one new K or V value (Eq. 4: the cache holds bf16).  Without a peer: the
 * value rounded to nearest even.  With a peer (the same slot of another implementation's cache after the same
 * step): the stored bf16 code is a quantised decision that an implementation computing the value in fp32
 * may take one step away from this one where the value lies close to a rounding boundary, and an entry that
 * cancels to nearly zero may differ by more steps while being as close in value.  Both are correct stores.
 * If the peer's code is this rounding, its neighbour, or within tol_abs + tol_rel |value| of it, the peer's
 * code is stored (and this step's attention, like every later step, reads it), so that one legitimate
 * difference is not carried through the remaining layers into everything compared afterwards; otherwise this
 * implementation's own rounding is stored, and the comparison of the two caches shows the entry.
 * stats[0..3] count: equal, adopted neighbour, adopted by value, kept own (peer rejected).
 */
static uint16_t stored_code(double x, const uint16_t *peer, double tol_abs, double tol_rel, int64_t *stats) {
    const uint16_t own = double_to_bf16(x);
    if (!peer) return own;
    const uint16_t p = *peer;
    int which;
    if (p == own) which = 0;
    else if (abs(bf16_ordered(p) - bf16_ordered(own)) <= 1) which = 1;
    else if (fabs(bf16_to_double(p) - bf16_to_double(own)) <= tol_abs + tol_rel * fabs(bf16_to_double(own))) which = 2;
    else which = 3;
    if (stats) {
#pragma omp atomic
        stats[which] += 1;
    }
    return which == 3 ? own : p;
}

static int decode_step_impl(const orc_cfg *c, const orc_mat *mats, const orc_pool *pool, int B,
                    const int32_t *tokens, const int32_t *page_tables, int max_pages,
                    const int32_t *seq_lens, const int32_t *model_ids, int mode,
                    double *logits, int32_t *next, double *rowsums, double *attn_probe,
                    const orc_pool *peer, double peer_tol_abs, double peer_tol_rel, int64_t *peer_stats) {
    (void)model_ids;
    const int H = c->hidden, Hq = c->n_q_heads, Hkv = c->n_kv_heads, d = c->head_dim, F = c->ffn;
    const int NL = c->n_layers, P = pool->page_tokens, QD = Hq * d, KD = Hkv * d;
    if (B <= 0 || Hq % Hkv || d % 2 || QD <= 0) return ORC_ERR_ARG;
    int64_t maxn = 0;
    for (int b = 0; b < B; ++b) {
        int64_t n = (int64_t)seq_lens[b] + 1;
        if (seq_lens[b] < 0 || (n + P - 1) / P > max_pages) return ORC_ERR_ARG;
        for (int64_t pg = 0; pg < (n + P - 1) / P; ++pg) {
            int32_t id = page_tables[(size_t)b * max_pages + pg];
            if (id < 0 || id >= pool->n_pages) return ORC_ERR_PAGE;
        }
        if (n > maxn) maxn = n;
    }
    size_t nx = (size_t)B * H;
    double *X = malloc(sizeof(double) * nx), *Hn = malloc(sizeof(double) * nx);
    double *Q = malloc(sizeof(double) * B * QD), *K = malloc(sizeof(double) * B * KD), *Vv = malloc(sizeof(double) * B * KD);
    double *A = malloc(sizeof(double) * B * QD), *O = malloc(sizeof(double) * nx);
    double *Gt = malloc(sizeof(double) * B * F), *Up = malloc(sizeof(double) * B * F), *Dn = malloc(sizeof(double) * nx);
    if (!X || !Hn || !Q || !K || !Vv || !A || !O || !Gt || !Up || !Dn) return ORC_ERR_ALLOC;
    int rc = embed_rows(c, mats, B, tokens, X);
    for (int l = 0; l < NL && rc == ORC_OK; ++l) {
        for (int b = 0; b < B; ++b) rmsnorm(MAT_L(mats, l, M_G1), X + (size_t)b * H, H, c->rms_eps, Hn + (size_t)b * H);
        act_round(c, Hn, nx);
        qkv_project(c, mats, l, Hn, B, Q, K, Vv);
#pragma omp parallel for schedule(dynamic, 1)
        for (int b = 0; b < B; ++b) {
            const int64_t L = seq_lens[b], n = L + 1;
            const int32_t *pt = page_tables + (size_t)b * max_pages;
            double *q = Q + (size_t)b * QD, *k = K + (size_t)b * KD, *v = Vv + (size_t)b * KD;
            norm_and_rotate(c, mats, l, q, k, L);
            /* append: slot L of the request's cache, bf16 storage */
            for (int h = 0; h < Hkv; ++h) {
                uint16_t *kd = pool_k(pool, l, pt[L / P], h, (int)(L % P));
                uint16_t *vd = pool_v(pool, l, pt[L / P], h, (int)(L % P));
                const uint16_t *kp = peer ? pool_k(peer, l, pt[L / P], h, (int)(L % P)) : NULL;
                const uint16_t *vp = peer ? pool_v(peer, l, pt[L / P], h, (int)(L % P)) : NULL;
                for (int j = 0; j < d; ++j) {
                    kd[j * pool->k_dim] = stored_code(k[h * d + j], kp ? kp + j * peer->k_dim : NULL, peer_tol_abs, peer_tol_rel, peer_stats);
                    vd[j * pool->v_dim] = stored_code(v[h * d + j], vp ? vp + j * peer->v_dim : NULL, peer_tol_abs, peer_tol_rel, peer_stats);
                }
            }
            if (mode != 0) {
                double *scratch = malloc(sizeof(double) * (size_t)n);
                double *rs = rowsums ? rowsums + ((size_t)b * NL + l) * Hq : NULL;
                double *a = A + (size_t)b * QD;
                double *Kc = malloc(sizeof(double) * (size_t)n * KD), *Vc = malloc(sizeof(double) * (size_t)n * KD);
                for (int64_t t = 0; t < n; ++t)
                    for (int h = 0; h < Hkv; ++h) {
                        const uint16_t *ks = pool_k(pool, l, pt[t / P], h, (int)(t % P));
                        const uint16_t *vs = pool_v(pool, l, pt[t / P], h, (int)(t % P));
                        for (int j = 0; j < d; ++j) {
                            Kc[((size_t)t * Hkv + h) * d + j] = bf16_to_double(ks[j * pool->k_dim]);
                            Vc[((size_t)t * Hkv + h) * d + j] = bf16_to_double(vs[j * pool->v_dim]);
                        }
                    }
                attend_contig(c, q, Kc, Vc, n, a, rs, scratch);
                free(Kc);
                free(Vc);
                free(scratch);
            }
        }
        if (mode == 0) {
            /* every (request, query head) pair is independent: spread them over the cores */
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
            for (int b = 0; b < B; ++b)
                for (int h = 0; h < Hq; ++h) {
                    const int64_t n = (int64_t)seq_lens[b] + 1;
                    double *scratch = malloc(sizeof(double) * (size_t)n);
                    double *rs = rowsums ? rowsums + ((size_t)b * NL + l) * Hq : NULL;
                    attend_paged(c, pool, l, page_tables + (size_t)b * max_pages, Q + (size_t)b * QD, n,
                                 A + (size_t)b * QD, rs, scratch, h, h + 1);
                    free(scratch);
                }
        }
        if (attn_probe)
            for (int b = 0; b < B; ++b)
                memcpy(attn_probe + ((size_t)b * NL + l) * QD, A + (size_t)b * QD, sizeof(double) * QD);
        act_round(c, A, (size_t)B * QD);
        linear(MAT_L(mats, l, M_WO), A, B, O);
        for (size_t i = 0; i < nx; ++i) X[i] += O[i];
        feed_forward(c, mats, l, B, X, Hn, Gt, Up, Dn);
    }
    if (rc == ORC_OK) final_logits(c, mats, B, X, Hn, logits, next);
    free(X); free(Hn); free(Q); free(K); free(Vv); free(A); free(O); free(Gt); free(Up); free(Dn);
    return rc;
}

int orc_decode_step(const orc_cfg *c, const orc_mat *mats, const orc_pool *pool, int B,
                    const int32_t *tokens, const int32_t *page_tables, int max_pages,
                    const int32_t *seq_lens, const int32_t *model_ids, int mode,
                    double *logits, int32_t *next, double *rowsums, double *attn_probe) {
    return decode_step_impl(c, mats, pool, B, tokens, page_tables, max_pages, seq_lens, model_ids, mode, logits, next,
                            rowsums, attn_probe, NULL, 0.0, 0.0, NULL);
}

/*
 * The same step next to another implementation's cache (`peer`: same layout and page ids as `pool`, read
 * only, holding that implementation's entries for the positions this step writes): see stored_code().
 * peer_stats[4] is added to: entries equal, adopted as neighbour, adopted by value, kept (peer rejected).
 * A harness option like the forced tokens of a run: every value is still computed here, independently, and
 * the peer's entry is only taken after it has been checked against it.
 */
int orc_decode_step_peer(const orc_cfg *c, const orc_mat *mats, const orc_pool *pool, int B,
                         const int32_t *tokens, const int32_t *page_tables, int max_pages,
                         const int32_t *seq_lens, const int32_t *model_ids, int mode,
                         double *logits, int32_t *next, const orc_pool *peer, double peer_tol_abs,
                         double peer_tol_rel, int64_t *peer_stats) {
    if (!peer || peer->n_pages != pool->n_pages || peer->page_tokens != pool->page_tokens) return ORC_ERR_ARG;
    return decode_step_impl(c, mats, pool, B, tokens, page_tables, max_pages, seq_lens, model_ids, mode, logits, next,
                            NULL, NULL, peer, peer_tol_abs, peer_tol_rel, peer_stats);
}

/* ---------- decode step over a contiguous double cache (no paging) ---------- */

/*
 * One request, cache held as doubles: Kc,Vc are [NL][cap][Hkv][d] with the first
 * L positions filled; position L is written by this call.  round_kv != 0 rounds
 * the new entry to bf16 first.  Used to check the decomposition of Eq. 1 into
 * Eq. 2+3 free of storage rounding.
 */
int orc_decode_contig_f64(const orc_cfg *c, const orc_mat *mats, int32_t token, int64_t L, int64_t cap,
                          double *Kc, double *Vc, int round_kv, double *logits, int32_t *next) {
    const int H = c->hidden, Hq = c->n_q_heads, Hkv = c->n_kv_heads, d = c->head_dim, F = c->ffn;
    const int NL = c->n_layers, QD = Hq * d, KD = Hkv * d;
    if (L < 0 || L >= cap) return ORC_ERR_ARG;
    double *X = malloc(sizeof(double) * H), *Hn = malloc(sizeof(double) * H);
    double *q = malloc(sizeof(double) * QD), *k = malloc(sizeof(double) * KD), *v = malloc(sizeof(double) * KD);
    double *a = malloc(sizeof(double) * QD), *O = malloc(sizeof(double) * H);
    double *Gt = malloc(sizeof(double) * F), *Up = malloc(sizeof(double) * F), *Dn = malloc(sizeof(double) * H);
    double *scratch = malloc(sizeof(double) * (size_t)(L + 1));
    int rc = embed_rows(c, mats, 1, &token, X);
    for (int l = 0; l < NL && rc == ORC_OK; ++l) {
        rmsnorm(MAT_L(mats, l, M_G1), X, H, c->rms_eps, Hn);
        act_round(c, Hn, H);
        qkv_project(c, mats, l, Hn, 1, q, k, v);
        norm_and_rotate(c, mats, l, q, k, L);
        double *Kl = Kc + (size_t)l * cap * KD, *Vl = Vc + (size_t)l * cap * KD;
        for (int j = 0; j < KD; ++j) {
            Kl[(size_t)L * KD + j] = round_kv ? bf16_to_double(double_to_bf16(k[j])) : k[j];
            Vl[(size_t)L * KD + j] = round_kv ? bf16_to_double(double_to_bf16(v[j])) : v[j];
        }
        attend_contig(c, q, Kl, Vl, L + 1, a, NULL, scratch);
        act_round(c, a, QD);
        linear(MAT_L(mats, l, M_WO), a, 1, O);
        for (int j = 0; j < H; ++j) X[j] += O[j];
        feed_forward(c, mats, l, 1, X, Hn, Gt, Up, Dn);
    }
    if (rc == ORC_OK) final_logits(c, mats, 1, X, Hn, logits, next);
    free(X); free(Hn); free(q); free(k); free(v); free(a); free(O); free(Gt); free(Up); free(Dn); free(scratch);
    return rc;
}

/* ---------- brute force: causal forward over a whole sequence (Eq. 1) ---------- */

/*
 * No cache: every layer is evaluated for all T positions, position t attending
 * to positions 0..t.  logits: [T, vocab].  K_out, V_out: [NL][T][Hkv][d]
 * (post-rotary keys), may be NULL.  round_kv != 0 rounds every K/V to bf16
 * before it is attended to, as a bf16 cache would.
 */
int orc_full_forward(const orc_cfg *c, const orc_mat *mats, int T, const int32_t *tokens, int round_kv,
                     double *logits, double *K_out, double *V_out) {
    const int H = c->hidden, Hq = c->n_q_heads, Hkv = c->n_kv_heads, d = c->head_dim, F = c->ffn;
    const int NL = c->n_layers, QD = Hq * d, KD = Hkv * d, G = Hq / Hkv;
    size_t nx = (size_t)T * H;
    double *X = malloc(sizeof(double) * nx), *Hn = malloc(sizeof(double) * nx), *O = malloc(sizeof(double) * nx);
    double *Q = malloc(sizeof(double) * T * QD), *K = malloc(sizeof(double) * T * KD), *V = malloc(sizeof(double) * T * KD);
    double *A = malloc(sizeof(double) * T * QD), *sc = malloc(sizeof(double) * T);
    double *Gt = malloc(sizeof(double) * T * F), *Up = malloc(sizeof(double) * T * F), *Dn = malloc(sizeof(double) * nx);
    int rc = embed_rows(c, mats, T, tokens, X);
    for (int l = 0; l < NL && rc == ORC_OK; ++l) {
        for (int t = 0; t < T; ++t) rmsnorm(MAT_L(mats, l, M_G1), X + (size_t)t * H, H, c->rms_eps, Hn + (size_t)t * H);
        act_round(c, Hn, nx);
        qkv_project(c, mats, l, Hn, T, Q, K, V);
        for (int t = 0; t < T; ++t) {
            norm_and_rotate(c, mats, l, Q + (size_t)t * QD, K + (size_t)t * KD, t);
        }
        if (round_kv)
            for (size_t i = 0; i < (size_t)T * KD; ++i) {
                K[i] = bf16_to_double(double_to_bf16(K[i]));
                V[i] = bf16_to_double(double_to_bf16(V[i]));
            }
        if (K_out) memcpy(K_out + (size_t)l * T * KD, K, sizeof(double) * T * KD);
        if (V_out) memcpy(V_out + (size_t)l * T * KD, V, sizeof(double) * T * KD);
        for (int t = 0; t < T; ++t)
            for (int h = 0; h < Hq; ++h) {
                const double *q = Q + (size_t)t * QD + h * d;
                for (int u = 0; u <= t; ++u) {
                    double acc = 0.0;
                    for (int j = 0; j < d; ++j) acc += q[j] * K[(size_t)u * KD + (h / G) * d + j];
                    sc[u] = acc / sqrt((double)d);
                }
                softmax_inplace(sc, t + 1);
                for (int j = 0; j < d; ++j) {
                    double acc = 0.0;
                    for (int u = 0; u <= t; ++u) acc += sc[u] * V[(size_t)u * KD + (h / G) * d + j];
                    A[(size_t)t * QD + h * d + j] = acc;
                }
            }
        act_round(c, A, (size_t)T * QD);
        linear(MAT_L(mats, l, M_WO), A, T, O);
        for (size_t i = 0; i < nx; ++i) X[i] += O[i];
        feed_forward(c, mats, l, T, X, Hn, Gt, Up, Dn);
    }
    if (rc == ORC_OK) final_logits(c, mats, T, X, Hn, logits, NULL);
    free(X); free(Hn); free(O); free(Q); free(K); free(V); free(A); free(sc); free(Gt); free(Up); free(Dn);
    return rc;
}

/* ---------- single operations, exposed for pins and kernel-level parity ---------- */

void orc_rmsnorm(const double *x, const double *g, int n, double eps, double *h) {
    orc_mat gm = {ORC_F64, 1, n, 0, g, NULL, NULL, NULL};
    rmsnorm(&gm, x, n, eps, h);
}
void orc_rope(double *u, int d, int64_t pos, double base) {
    orc_cfg c;
    memset(&c, 0, sizeof c);
    c.head_dim = d;
    c.rope_base = base;
    rope(&c, u, pos);
}
void orc_rope_cfg(const orc_cfg *c, double *u, int64_t pos) { rope(c, u, pos); }
double orc_rope_freq(const orc_cfg *c, int j) { return rope_freq(c, j); }
double orc_silu(double z) { return silu(z); }
void orc_linear(const orc_mat *m, const double *X, int B, double *Y) { linear(m, X, B, Y); }
int32_t orc_argmax(const double *v, int n) { return argmax_lowest(v, n); }
uint16_t orc_double_to_bf16(double x) { return double_to_bf16(x); }
double orc_bf16_to_double(uint16_t b) { return bf16_to_double(b); }
uint16_t orc_float_to_half(float f) { return float_to_half(f); }
float orc_half_to_float(uint16_t h) { return half_to_float(h); }

/* Paged attention for one request and layer: q [Hq*d] (already rotated),
 * n = number of cached positions to attend to (all present in the pool). */
int orc_attention_paged(const orc_cfg *c, const orc_pool *pool, int layer, const int32_t *pt,
                        const double *q, int64_t n, double *a, double *rowsum) {
    double *scratch = malloc(sizeof(double) * (size_t)n);
    if (!scratch) return ORC_ERR_ALLOC;
    attend_paged(c, pool, layer, pt, q, n, a, rowsum, scratch, 0, c->n_q_heads);
    free(scratch);
    return ORC_OK;
}

/* ---------- 4-bit weight-only quantisation (QSUN) ---------- */

static float clampf(float x, float lo, float hi) { return x < lo ? lo : (x > hi ? hi : x); }

/*
 * Round-to-nearest group quantiser.  w: float [rows, cols]; groups of `group`
 * consecutive columns (the last may be short).  W_hat = (Q - Z) * S.
 * mode 0 (affine):    S = fp16((max-min)/15) (1 if that is 0),
 *                     Z = clamp(rne(-min/S),0,15), Q = clamp(rne(w/S)+Z,0,15).
 * mode 1 (symmetric): S = fp16(max|w|/7) (1 if 0), Z = 8, Q = clamp(rne(w/S)+8,0,15).
 * Divisions use the stored fp16 scale, in float; rne is round-half-to-even.
 * q: [rows, cols/2] bytes, low nibble = even column (cols must be even).
 */
int orc_quantize_w4(const float *w, int rows, int cols, int group, int mode,
                    uint8_t *q, uint16_t *s, uint16_t *z) {
    if (cols % 2 || group <= 0) return ORC_ERR_ARG;
    int ng = (cols + group - 1) / group;
#pragma omp parallel for schedule(static)
    for (int r = 0; r < rows; ++r) {
        const float *row = w + (size_t)r * cols;
        memset(q + (size_t)r * (cols / 2), 0, (size_t)cols / 2);
        for (int g = 0; g < ng; ++g) {
            int c0 = g * group, c1 = c0 + group < cols ? c0 + group : cols;
            float mn = row[c0], mx = row[c0], amax = fabsf(row[c0]);
            for (int cc = c0 + 1; cc < c1; ++cc) {
                if (row[cc] < mn) mn = row[cc];
                if (row[cc] > mx) mx = row[cc];
                if (fabsf(row[cc]) > amax) amax = fabsf(row[cc]);
            }
            float sf = (mode == 0) ? (mx - mn) / 15.0f : amax / 7.0f;
            uint16_t sh = float_to_half(sf);
            float S = half_to_float(sh);
            if (S == 0.0f) { S = 1.0f; sh = float_to_half(1.0f); }
            float Z = (mode == 0) ? clampf(nearbyintf(-mn / S), 0.0f, 15.0f) : 8.0f;
            if (Z == 0.0f) Z = 0.0f; /* the zero point is an integer code: store +0, never -0 */
            s[(size_t)r * ng + g] = sh;
            z[(size_t)r * ng + g] = float_to_half(Z);
            for (int cc = c0; cc < c1; ++cc) {
                int code = (int)clampf(nearbyintf(row[cc] / S) + Z, 0.0f, 15.0f);
                q[(size_t)r * (cols / 2) + cc / 2] |= (uint8_t)(code << ((cc & 1) * 4));
            }
        }
    }
    return ORC_OK;
}

/* out[r][c] = (Q - Z) * S as float (exact). */
void orc_dequantize_w4(const orc_mat *m, float *out) {
    for (int r = 0; r < m->rows; ++r)
        for (int c = 0; c < m->cols; ++c) out[(size_t)r * m->cols + c] = (float)mat_get(m, r, c);
}

int orc_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
