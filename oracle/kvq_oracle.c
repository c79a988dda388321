/*
 * kvq_oracle.c -- plain, slow CPU oracle for the mixed-precision KV-cache path.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only tests, the smoke check
 * and the benchmark's cpu_baseline leg may load it.  It shares no code with the
 * HIP library: it is written straight from the paper's equations.
 *
 * What it follows (KVTuner, arXiv 2502.04420):
 *   - Section 3.1, Eq. 1:  a = softmax(q K^T / sqrt(D)),  o = a V, with K and V
 *     the concatenation of every cached token and the current one (no mask for
 *     the single decode query).
 *   - Section 3.2, Eq. 2:  Q(X) = round((X - z) / s),  X^ = Q(X) * s + z,
 *     z = min(X),  s = (max(X) - min(X)) / (2^B - 1), taken along the channel
 *     dimension (values: one (s, z) per token per group of G channels) or along
 *     the token dimension (keys: one (s, z) per channel per group of G tokens),
 *     which is the KIVI mode the experimental-settings appendix selects with
 *     group size 32 and residual length 32.
 *   - Section 5.1: one (key bits, value bits) pair per layer.
 *
 * Readings where the paper is silent (each listed in the design notes):
 *   - "round" is round-half-to-even, and (x - z) / s, s itself and max - min are
 *     single IEEE fp32 operations on the fp16 inputs widened to fp32; codes are
 *     clamped to [0, 2^B - 1]; a constant group has s = 0 and all codes 0.
 *   - D in sqrt(D) is the per-head dimension.
 *   - the newest tokens stay in fp16: with T tokens appended so far,
 *     N_p = G * floor(max(T - R, 0) / G) tokens are quantized and the other
 *     T - N_p (at least R once T >= R) stay in full precision.  Key groups are
 *     therefore aligned to absolute positions [32 g, 32 g + 32).
 *   - 16 "bits" means the fp16 values are kept as they are.
 *   - key grouping: the KIVI mode above by default; a second mode groups keys per
 *     token like the values (the paper's per-token-asym mode).
 *   - prefill-stage attention (the prompt's own attention reading the dequantized cache, Section 5.3 and the
 *     experimental-settings appendix): evaluated over the cache as it stands when it is called; the query at
 *     absolute position p sees positions 0..p; a token enters as X^ if it is held quantized at that moment.
 *   - signed zeros: min(X) and max(X) are numbers; a zero minimum or maximum is stored as +0 whichever of +0 / -0
 *     the group holds and in whichever order (z and s then have one bit pattern per group).
 *   - metadata precision: s and z are fp32 by default.  A variant stores them as
 *     fp16 (z exactly, s rounded once); it encodes and decodes with the rounded s.
 *
 * Precision: s, z and the codes are fp32 / integer exactly as above; everything
 * in the attention (dequantisation c * s + z, dot products, softmax, weighted
 * sum) is fp64; the output is rounded once to fp16 (round-half-to-even).
 *
 * Parity pins live in tests/test_oracle_*.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ fp16 */

/* IEEE binary16 -> double, exact. */
static double half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);                 /* subnormal or zero */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m | 0x400), e - 25);
    return sign ? -v : v;
}

/* double -> IEEE binary16, one rounding, round-half-to-even. */
static uint16_t double_to_half(double x)
{
    uint16_t sign = signbit(x) ? 0x8000 : 0;
    double a = fabs(x);
    if (isnan(a)) return (uint16_t)(sign | 0x7e00);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00);   /* 65520 ties to 65536 = inf */
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                 /* a = f * 2^e, f in [0.5, 1) -> a in [2^(e-1), 2^e) */
    int be = e - 1;                     /* floor(log2(a)) */
    if (be < -14) be = -14;             /* subnormal range shares the quantum 2^-24 */
    double quantum = ldexp(1.0, be - 10);
    double n = nearbyint(a / quantum);  /* exact division by a power of two, then RNE */
    if (n == 0.0) return sign;
    double r = n * quantum;             /* the rounded value, exactly representable */
    (void)frexp(r, &e);
    be = e - 1;
    if (be < -14) {                     /* subnormal result */
        return (uint16_t)(sign | (uint16_t)(r / ldexp(1.0, -24)));
    }
    uint16_t mant = (uint16_t)(r / ldexp(1.0, be - 10)) & 0x3ff;
    return (uint16_t)(sign | ((uint16_t)(be + 15) << 10) | mant);
}

float kvo_half_to_float(uint16_t h) { return (float)half_to_double(h); }
uint16_t kvo_double_to_half(double x) { return double_to_half(x); }

/* ------------------------------------------------------------- quantizer */

/*
 * Eq. 2 on one group of n fp32 values with B = bits.  Writes the scale, the
 * zero-point (offset) and one code per element.
 *
 * scale_fp16 selects the narrow-metadata variant: the scale is rounded once to
 * fp16 (round-half-to-even) and that rounded value, widened back to fp32, is the
 * s used for encoding and decoding, so both sides agree.  The zero-point is the
 * minimum of fp16 inputs and needs no rounding.  With the rounded scale the
 * quotient can exceed 2^B - 1 (a scale that became subnormal in fp16 may be far
 * too small), which is where the clamp acts; a scale that rounds to zero gives
 * all codes 0 like a constant group.
 */
void kvo_quantize_group_ex(const float *x, int n, int bits, int scale_fp16, float *s_out, float *z_out, uint8_t *codes)
{
    float mn = x[0], mx = x[0];
    for (int i = 1; i < n; i++) {
        if (x[i] < mn) mn = x[i];
        if (x[i] > mx) mx = x[i];
    }
    /* Eq. 2 takes the minimum and maximum as numbers.  The number zero has two fp32 encodings; which of them a scan
     * meets first depends on the element order, which Eq. 2 does not know.  Reading: a zero extreme is stored as +0
     * (so z and s have one bit pattern per group whatever the order; codes and X^ are the same either way). */
    if (mn == 0.0f) mn = 0.0f;
    if (mx == 0.0f) mx = 0.0f;
    const int qmax = (1 << bits) - 1;
    const float z = mn;
    const float range = mx - mn;
    float s = range / (float)qmax;
    if (scale_fp16) s = kvo_half_to_float(double_to_half((double)s));
    for (int i = 0; i < n; i++) {
        long c = 0;
        if (s != 0.0f) {
            float t = (x[i] - z) / s;
            c = lrintf(t);              /* current rounding mode: nearest, ties to even */
            if (c < 0) c = 0;
            if (c > qmax) c = qmax;
        }
        codes[i] = (uint8_t)c;
    }
    *s_out = s;
    *z_out = z;
}

void kvo_quantize_group(const float *x, int n, int bits, float *s_out, float *z_out, uint8_t *codes)
{
    kvo_quantize_group_ex(x, n, bits, 0, s_out, z_out, codes);
}

/* X^ = Q(X) * s + z, evaluated in double. */
static inline double dequant(uint8_t c, float s, float z)
{
    return (double)c * (double)s + (double)z;
}

/* ------------------------------------------------------------ cache state */

typedef struct {
    int kbits, vbits;
    int T;          /* tokens appended so far (same for every sequence) */
    int Np;         /* tokens quantized so far, multiple of G */
    int cap;        /* allocated tokens */
    /* per (b, kv-head) arrays, index bh = b * Hkv + h, each [cap] tokens long */
    uint16_t *raw_k, *raw_v;     /* [BH][cap][D] every token as appended (fp16) */
    uint8_t *k_code, *v_code;    /* [BH][cap][D] one code per element (first Np tokens valid) */
    float *k_s, *k_z;            /* [BH][cap/G][D] per token-group, per channel */
    float *v_s, *v_z;            /* [BH][cap][D/G] per token, per channel-group */
} kvo_layer;

typedef struct kvo_cache {
    int L, B, Hq, Hkv, D, G, R;
    int scale_fp16;     /* narrow-metadata variant: scales rounded to fp16 */
    int key_per_token;  /* keys quantized like values: per token over each group of G channels */
    kvo_layer *layer;
} kvo_cache;

kvo_cache *kvo_create(int n_layers, int batch, int n_q_heads, int n_kv_heads, int head_dim,
                      int group, int residual, const uint8_t *kbits, const uint8_t *vbits)
{
    if (n_layers < 1 || batch < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads || group < 1 ||
        head_dim % group || residual < 0)
        return NULL;
    for (int l = 0; l < n_layers; l++) {
        int kb = kbits[l], vb = vbits[l];
        if ((kb != 2 && kb != 4 && kb != 8 && kb != 16) || (vb != 2 && vb != 4 && vb != 8 && vb != 16))
            return NULL;
    }
    kvo_cache *c = calloc(1, sizeof *c);
    c->L = n_layers; c->B = batch; c->Hq = n_q_heads; c->Hkv = n_kv_heads;
    c->D = head_dim; c->G = group; c->R = residual;
    c->layer = calloc((size_t)n_layers, sizeof(kvo_layer));
    for (int l = 0; l < n_layers; l++) {
        c->layer[l].kbits = kbits[l];
        c->layer[l].vbits = vbits[l];
    }
    return c;
}

/* Select the narrow-metadata variant (see kvo_quantize_group_ex).  Only while every layer is empty. */
int kvo_set_scale_fp16(kvo_cache *c, int on)
{
    for (int l = 0; l < c->L; l++)
        if (c->layer[l].T) return -1;
    c->scale_fp16 = on ? 1 : 0;
    return 0;
}

/*
 * Select the axis along which the keys are grouped for Eq. 2.  0 (default): per channel over G
 * consecutive tokens (the KIVI mode).  1: per token over each group of G channels, exactly as the
 * values (the paper's per-token-asym mode; its group size is not stated, the value grouping is
 * used).  Only while every layer is empty.  The key metadata then has the value metadata's shape.
 */
int kvo_set_key_per_token(kvo_cache *c, int on)
{
    for (int l = 0; l < c->L; l++)
        if (c->layer[l].T) return -1;
    c->key_per_token = on ? 1 : 0;
    return 0;
}

static void layer_free(kvo_layer *y)
{
    free(y->raw_k); free(y->raw_v); free(y->k_code); free(y->v_code);
    free(y->k_s); free(y->k_z); free(y->v_s); free(y->v_z);
    int kb = y->kbits, vb = y->vbits;
    memset(y, 0, sizeof *y);
    y->kbits = kb; y->vbits = vb;
}

void kvo_destroy(kvo_cache *c)
{
    if (!c) return;
    for (int l = 0; l < c->L; l++) layer_free(&c->layer[l]);
    free(c->layer);
    free(c);
}

int kvo_reset(kvo_cache *c, int layer)
{
    if (layer < -1 || layer >= c->L) return -1;
    for (int l = 0; l < c->L; l++)
        if (layer < 0 || l == layer) layer_free(&c->layer[l]);
    return 0;
}

/* Re-allocate every per-(b,h) array of a layer for `cap` tokens, keeping contents. */
static void layer_grow(const kvo_cache *c, kvo_layer *y, int cap)
{
    const size_t BH = (size_t)c->B * c->Hkv, D = (size_t)c->D, G = (size_t)c->G;
    const size_t ng_old = (size_t)y->cap / G, ng_new = ((size_t)cap + G - 1) / G;
    cap = (int)(ng_new * G);
    uint16_t *rk = calloc(BH * cap * D, 2), *rv = calloc(BH * cap * D, 2);
    uint8_t *kc = calloc(BH * cap * D, 1), *vc = calloc(BH * cap * D, 1);
    float *ks = calloc(BH * ng_new * D, 4), *kz = calloc(BH * ng_new * D, 4);
    float *vs = calloc(BH * cap * (D / G), 4), *vz = calloc(BH * cap * (D / G), 4);
    for (size_t bh = 0; bh < BH && y->cap; bh++) {
        memcpy(rk + bh * cap * D, y->raw_k + bh * y->cap * D, (size_t)y->cap * D * 2);
        memcpy(rv + bh * cap * D, y->raw_v + bh * y->cap * D, (size_t)y->cap * D * 2);
        memcpy(kc + bh * cap * D, y->k_code + bh * y->cap * D, (size_t)y->cap * D);
        memcpy(vc + bh * cap * D, y->v_code + bh * y->cap * D, (size_t)y->cap * D);
        memcpy(ks + bh * ng_new * D, y->k_s + bh * ng_old * D, ng_old * D * 4);
        memcpy(kz + bh * ng_new * D, y->k_z + bh * ng_old * D, ng_old * D * 4);
        memcpy(vs + bh * cap * (D / G), y->v_s + bh * y->cap * (D / G), (size_t)y->cap * (D / G) * 4);
        memcpy(vz + bh * cap * (D / G), y->v_z + bh * y->cap * (D / G), (size_t)y->cap * (D / G) * 4);
    }
    free(y->raw_k); free(y->raw_v); free(y->k_code); free(y->v_code);
    free(y->k_s); free(y->k_z); free(y->v_s); free(y->v_z);
    y->raw_k = rk; y->raw_v = rv; y->k_code = kc; y->v_code = vc;
    y->k_s = ks; y->k_z = kz; y->v_s = vs; y->v_z = vz;
    y->cap = cap;
}

/*
 * Quantize tokens [Np, Np + G) of one (b, kv-head): keys per channel over the G
 * tokens, values per token over each group of G channels (Eq. 2, KIVI mode).
 */
static void flush_group(const kvo_cache *c, kvo_layer *y, size_t bh)
{
    const int D = c->D, G = c->G;
    const size_t cap = (size_t)y->cap;
    const size_t t0 = (size_t)y->Np;
    const size_t g = t0 / G;
    float *buf = malloc(sizeof(float) * (size_t)(G > D ? G : D));
    uint8_t *cbuf = malloc((size_t)(G > D ? G : D));
    if (y->kbits < 16 && c->key_per_token) {
        for (int i = 0; i < G; i++) {
            for (int j = 0; j < D / G; j++) {
                for (int e = 0; e < G; e++)
                    buf[e] = kvo_half_to_float(y->raw_k[(bh * cap + t0 + i) * D + j * G + e]);
                float s, z;
                kvo_quantize_group_ex(buf, G, y->kbits, c->scale_fp16, &s, &z, cbuf);
                y->k_s[(bh * cap + t0 + i) * (D / G) + j] = s;      /* same element count as the per-channel shape */
                y->k_z[(bh * cap + t0 + i) * (D / G) + j] = z;
                for (int e = 0; e < G; e++)
                    y->k_code[(bh * cap + t0 + i) * D + j * G + e] = cbuf[e];
            }
        }
    } else if (y->kbits < 16) {
        for (int d = 0; d < D; d++) {
            for (int i = 0; i < G; i++)
                buf[i] = kvo_half_to_float(y->raw_k[(bh * cap + t0 + i) * D + d]);
            float s, z;
            kvo_quantize_group_ex(buf, G, y->kbits, c->scale_fp16, &s, &z, cbuf);
            y->k_s[(bh * (cap / G) + g) * D + d] = s;
            y->k_z[(bh * (cap / G) + g) * D + d] = z;
            for (int i = 0; i < G; i++)
                y->k_code[(bh * cap + t0 + i) * D + d] = cbuf[i];
        }
    }
    if (y->vbits < 16) {
        for (int i = 0; i < G; i++) {
            for (int j = 0; j < D / G; j++) {
                for (int e = 0; e < G; e++)
                    buf[e] = kvo_half_to_float(y->raw_v[(bh * cap + t0 + i) * D + j * G + e]);
                float s, z;
                kvo_quantize_group_ex(buf, G, y->vbits, c->scale_fp16, &s, &z, cbuf);
                y->v_s[(bh * cap + t0 + i) * (D / G) + j] = s;
                y->v_z[(bh * cap + t0 + i) * (D / G) + j] = z;
                for (int e = 0; e < G; e++)
                    y->v_code[(bh * cap + t0 + i) * D + j * G + e] = cbuf[e];
            }
        }
    }
    free(buf);
    free(cbuf);
}

/*
 * Append n tokens to a layer.  K, V: fp16 [B, Hkv, n, D].  Then quantize whole
 * groups of the oldest full-precision tokens while at least R + G of them remain.
 */
int kvo_quantize_append(kvo_cache *c, int layer, const uint16_t *K, const uint16_t *V, int n)
{
    if (layer < 0 || layer >= c->L || n < 1) return -1;
    kvo_layer *y = &c->layer[layer];
    const size_t BH = (size_t)c->B * c->Hkv, D = (size_t)c->D;
    if (y->T + n > y->cap) {
        int want = y->cap * 2;
        if (want < y->T + n) want = y->T + n;
        layer_grow(c, y, want);
    }
    const size_t cap = (size_t)y->cap;
    for (size_t bh = 0; bh < BH; bh++) {
        memcpy(y->raw_k + (bh * cap + y->T) * D, K + bh * n * D, (size_t)n * D * 2);
        memcpy(y->raw_v + (bh * cap + y->T) * D, V + bh * n * D, (size_t)n * D * 2);
    }
    y->T += n;
    while (y->T - y->Np >= c->R + c->G) {
#pragma omp parallel for schedule(static)
        for (long bh = 0; bh < (long)BH; bh++) flush_group(c, y, (size_t)bh);
        y->Np += c->G;
    }
    return 0;
}

int kvo_tokens(const kvo_cache *c, int layer, int *n_packed, int *n_residual)
{
    if (layer < 0 || layer >= c->L) return -1;
    *n_packed = c->layer[layer].Np;
    *n_residual = c->layer[layer].T - c->layer[layer].Np;
    return 0;
}

/* ---------------------------------------------------------------- attention */

/*
 * Eq. 1 for one query row against T rows of (already dequantised) K and V held
 * as doubles [T][D].  p (length T) receives the softmax row; o (length D) the output.
 */
static void attend_row(const double *q, const double *Kh, const double *Vh, int T, int D,
                       double *p, double *o)
{
    const double inv_sqrt_d = 1.0 / sqrt((double)D);
    double mx = -INFINITY;
    for (int t = 0; t < T; t++) {
        double acc = 0.0;
        for (int d = 0; d < D; d++) acc += q[d] * Kh[(size_t)t * D + d];
        p[t] = acc * inv_sqrt_d;
        if (p[t] > mx) mx = p[t];
    }
    double sum = 0.0;
    for (int t = 0; t < T; t++) {
        p[t] = exp(p[t] - mx);
        sum += p[t];
    }
    for (int t = 0; t < T; t++) p[t] /= sum;
    for (int d = 0; d < D; d++) o[d] = 0.0;
    for (int t = 0; t < T; t++)
        for (int d = 0; d < D; d++) o[d] += p[t] * Vh[(size_t)t * D + d];
}

/* The cache of one layer as attention sees it: X^ (Eq. 2) for quantized tokens, the fp16 values for the rest.
 * Kh, Vh: double [B, Hkv, T, D]. */
static void reconstruct_bh(const kvo_cache *c, const kvo_layer *y, size_t bh, double *Kh, double *Vh)
{
    const int D = c->D, G = c->G, T = y->T, Np = y->Np;
    const size_t cap = (size_t)y->cap;
    for (int t = 0; t < T; t++) {
        for (int d = 0; d < D; d++) {
            size_t e = (bh * cap + t) * D + d;
            if (t < Np && y->kbits < 16 && c->key_per_token)
                Kh[(size_t)t * D + d] = dequant(y->k_code[e], y->k_s[(bh * cap + t) * (D / G) + d / G],
                                                y->k_z[(bh * cap + t) * (D / G) + d / G]);
            else if (t < Np && y->kbits < 16)
                Kh[(size_t)t * D + d] = dequant(y->k_code[e], y->k_s[(bh * (cap / G) + t / G) * D + d],
                                                y->k_z[(bh * (cap / G) + t / G) * D + d]);
            else
                Kh[(size_t)t * D + d] = half_to_double(y->raw_k[e]);
            if (t < Np && y->vbits < 16)
                Vh[(size_t)t * D + d] = dequant(y->v_code[e], y->v_s[(bh * cap + t) * (D / G) + d / G],
                                                y->v_z[(bh * cap + t) * (D / G) + d / G]);
            else
                Vh[(size_t)t * D + d] = half_to_double(y->raw_v[e]);
        }
    }
}

int kvo_reconstruct(const kvo_cache *c, int layer, double *K_hat, double *V_hat)
{
    if (layer < 0 || layer >= c->L) return -1;
    const kvo_layer *y = &c->layer[layer];
    const size_t per = (size_t)y->T * c->D;
    for (long bh = 0; bh < (long)c->B * c->Hkv; bh++)
        reconstruct_bh(c, y, (size_t)bh, K_hat + (size_t)bh * per, V_hat + (size_t)bh * per);
    return 0;
}

/*
 * Decode attention of one layer over everything appended so far: quantized
 * tokens enter as X^ (Eq. 2), the rest as their fp16 values.
 * q: fp16 [B, Hq, D];  out: fp16 [B, Hq, D];
 * out_f64 (nullable): the unrounded outputs [B, Hq, D];
 * p_out (nullable): the softmax rows [B, Hq, T].
 */
int kvo_decode_attention(const kvo_cache *c, int layer, const uint16_t *q, uint16_t *out,
                         double *out_f64, double *p_out)
{
    if (layer < 0 || layer >= c->L) return -1;
    const kvo_layer *y = &c->layer[layer];
    if (y->T < 1) return -2;
    const int D = c->D, T = y->T, gq = c->Hq / c->Hkv;
    const long BH = (long)c->B * c->Hkv;
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < BH; bh++) {
        double *Kh = malloc(sizeof(double) * (size_t)T * D);
        double *Vh = malloc(sizeof(double) * (size_t)T * D);
        double *p = malloc(sizeof(double) * (size_t)T);
        double *qd = malloc(sizeof(double) * (size_t)D);
        double *o = malloc(sizeof(double) * (size_t)D);
        reconstruct_bh(c, y, (size_t)bh, Kh, Vh);
        const long b = bh / c->Hkv, h = bh % c->Hkv;
        for (int j = 0; j < gq; j++) {
            const size_t row = (size_t)b * c->Hq + (size_t)h * gq + j;   /* q head h*gq+j reads kv head h */
            for (int d = 0; d < D; d++) qd[d] = half_to_double(q[row * D + d]);
            attend_row(qd, Kh, Vh, T, D, p, o);
            for (int d = 0; d < D; d++) {
                out[row * D + d] = double_to_half(o[d]);
                if (out_f64) out_f64[row * D + d] = o[d];
            }
            if (p_out) memcpy(p_out + row * T, p, sizeof(double) * (size_t)T);
        }
        free(Kh); free(Vh); free(p); free(qd); free(o);
    }
    return 0;
}

/*
 * Prefill-stage attention of one layer over the cache as it stands.  The paper quantizes the cache in the
 * prefill stage as well as in decoding and lets the prompt's own attention read the dequantized K and V
 * (calibration design of Section 5.3, experimental-settings appendix).  Reading taken here: a query at absolute
 * position p attends to positions 0..p (Eq. 1 under the usual causal mask); a token enters as X^ (Eq. 2) if the
 * cache holds it quantized now, else as its fp16 value.
 * positions: n absolute positions (each in [0, T)), shared by all heads;
 * q: fp16 [B, Hq, n, D], row i is the query at positions[i];  out: fp16 [B, Hq, n, D];
 * out_f64 (nullable): the unrounded outputs.
 */
int kvo_prefill_attention_at(const kvo_cache *c, int layer, const uint16_t *q, const int *positions, int n,
                             uint16_t *out, double *out_f64)
{
    if (layer < 0 || layer >= c->L) return -1;
    const kvo_layer *y = &c->layer[layer];
    if (y->T < 1 || n < 1) return -2;
    for (int i = 0; i < n; i++)
        if (positions[i] < 0 || positions[i] >= y->T) return -2;
    const int D = c->D, T = y->T, gq = c->Hq / c->Hkv;
    const long BH = (long)c->B * c->Hkv;
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < BH; bh++) {
        double *Kh = malloc(sizeof(double) * (size_t)T * D);
        double *Vh = malloc(sizeof(double) * (size_t)T * D);
        double *p = malloc(sizeof(double) * (size_t)T);
        double *qd = malloc(sizeof(double) * (size_t)D);
        double *o = malloc(sizeof(double) * (size_t)D);
        reconstruct_bh(c, y, (size_t)bh, Kh, Vh);
        const long b = bh / c->Hkv, h = bh % c->Hkv;
        for (int j = 0; j < gq; j++) {
            const size_t head = (size_t)b * c->Hq + (size_t)h * gq + j;
            for (int i = 0; i < n; i++) {
                const size_t row = head * (size_t)n + (size_t)i;
                for (int d = 0; d < D; d++) qd[d] = half_to_double(q[row * D + d]);
                attend_row(qd, Kh, Vh, positions[i] + 1, D, p, o);       /* keys and values 0..position */
                for (int d = 0; d < D; d++) {
                    out[row * D + d] = double_to_half(o[d]);
                    if (out_f64) out_f64[row * D + d] = o[d];
                }
            }
        }
        free(Kh); free(Vh); free(p); free(qd); free(o);
    }
    return 0;
}

/* The same with the last n_q tokens appended as the queries: positions T - n_q .. T - 1. */
int kvo_prefill_attention(const kvo_cache *c, int layer, const uint16_t *q, int n_q, uint16_t *out, double *out_f64)
{
    if (layer < 0 || layer >= c->L) return -1;
    const int T = c->layer[layer].T;
    if (T < 1 || n_q < 1 || n_q > T) return -2;
    int *positions = malloc(sizeof(int) * (size_t)n_q);
    for (int i = 0; i < n_q; i++) positions[i] = T - n_q + i;
    const int rc = kvo_prefill_attention_at(c, layer, q, positions, n_q, out, out_f64);
    free(positions);
    return rc;
}

/*
 * Brute-force Eq. 1 on raw fp16 tensors, no quantization anywhere.
 * q [B,Hq,D], K,V [B,Hkv,T,D] fp16; outputs as in kvo_decode_attention.
 */
void kvo_attention_exact(const uint16_t *q, const uint16_t *K, const uint16_t *V, int B, int Hq,
                         int Hkv, int T, int D, uint16_t *out, double *out_f64, double *p_out)
{
    const int gq = Hq / Hkv;
    for (long bh = 0; bh < (long)B * Hkv; bh++) {
        double *Kh = malloc(sizeof(double) * (size_t)T * D);
        double *Vh = malloc(sizeof(double) * (size_t)T * D);
        double *p = malloc(sizeof(double) * (size_t)T);
        double *qd = malloc(sizeof(double) * (size_t)D);
        double *o = malloc(sizeof(double) * (size_t)D);
        for (size_t i = 0; i < (size_t)T * D; i++) {
            Kh[i] = half_to_double(K[(size_t)bh * T * D + i]);
            Vh[i] = half_to_double(V[(size_t)bh * T * D + i]);
        }
        const long b = bh / Hkv, h = bh % Hkv;
        for (int j = 0; j < gq; j++) {
            const size_t row = (size_t)b * Hq + (size_t)h * gq + j;
            for (int d = 0; d < D; d++) qd[d] = half_to_double(q[row * D + d]);
            attend_row(qd, Kh, Vh, T, D, p, o);
            for (int d = 0; d < D; d++) {
                if (out) out[row * D + d] = double_to_half(o[d]);
                if (out_f64) out_f64[row * D + d] = o[d];
            }
            if (p_out) memcpy(p_out + row * T, p, sizeof(double) * (size_t)T);
        }
        free(Kh); free(Vh); free(p); free(qd); free(o);
    }
}

/* ------------------------------------------------------------------ export */

/* Little-endian bit packing: element i occupies bits [i*bits, (i+1)*bits) of the stream. */
static void pack_bits(const uint8_t *codes, int n, int bits, uint8_t *dst)
{
    memset(dst, 0, (size_t)(n * bits + 7) / 8);
    for (int i = 0; i < n; i++) {
        int bit = i * bits;
        dst[bit >> 3] |= (uint8_t)(codes[i] << (bit & 7));   /* bits divides 8: never straddles */
    }
}

/*
 * Canonical dump of one layer (any pointer may be NULL to skip it):
 *   k_codes  kbits<16: [B,Hkv,Np/G,D][G*kbits/8 bytes]  the G tokens of a group, per channel
 *            kbits=16: fp16 [B,Hkv,Np,D]
 *   k_scale, k_zero    fp32 [B,Hkv,Np/G,D]              (kbits<16 only)
 *            with keys grouped per token: k_codes [B,Hkv,Np][D*kbits/8 bytes], k_scale, k_zero [B,Hkv,Np,D/G]
 *   v_codes  vbits<16: [B,Hkv,Np][D*vbits/8 bytes]      the D channels of a token
 *            vbits=16: fp16 [B,Hkv,Np,D]
 *   v_scale, v_zero    fp32 [B,Hkv,Np,D/G]              (vbits<16 only)
 *   k_res, v_res       fp16 [B,Hkv,Nr,D]                oldest first
 */
int kvo_export(const kvo_cache *c, int layer, uint8_t *k_codes, float *k_scale, float *k_zero,
               uint8_t *v_codes, float *v_scale, float *v_zero, uint16_t *k_res, uint16_t *v_res)
{
    if (layer < 0 || layer >= c->L) return -1;
    const kvo_layer *y = &c->layer[layer];
    const size_t BH = (size_t)c->B * c->Hkv, D = (size_t)c->D, G = (size_t)c->G;
    const size_t Np = (size_t)y->Np, Nr = (size_t)(y->T - y->Np), cap = (size_t)y->cap;
    uint8_t *tmp = malloc(G > D ? G : D);
    for (size_t bh = 0; bh < BH; bh++) {
        if (y->kbits < 16 && c->key_per_token) {
            const size_t tb = D * (size_t)y->kbits / 8;
            for (size_t t = 0; t < Np; t++) {
                if (k_codes) pack_bits(y->k_code + (bh * cap + t) * D, (int)D, y->kbits, k_codes + (bh * Np + t) * tb);
                for (size_t j = 0; j < D / G; j++) {
                    if (k_scale) k_scale[(bh * Np + t) * (D / G) + j] = y->k_s[(bh * cap + t) * (D / G) + j];
                    if (k_zero) k_zero[(bh * Np + t) * (D / G) + j] = y->k_z[(bh * cap + t) * (D / G) + j];
                }
            }
        } else if (y->kbits < 16) {
            const size_t gb = G * (size_t)y->kbits / 8;
            for (size_t g = 0; g < Np / G; g++)
                for (size_t d = 0; d < D; d++) {
                    size_t o = (bh * (Np / G) + g) * D + d;
                    if (k_codes) {
                        for (size_t i = 0; i < G; i++) tmp[i] = y->k_code[(bh * cap + g * G + i) * D + d];
                        pack_bits(tmp, (int)G, y->kbits, k_codes + o * gb);
                    }
                    if (k_scale) k_scale[o] = y->k_s[(bh * (cap / G) + g) * D + d];
                    if (k_zero) k_zero[o] = y->k_z[(bh * (cap / G) + g) * D + d];
                }
        } else if (k_codes) {
            memcpy(k_codes + bh * Np * D * 2, y->raw_k + bh * cap * D, Np * D * 2);
        }
        if (y->vbits < 16) {
            const size_t tb = D * (size_t)y->vbits / 8;
            for (size_t t = 0; t < Np; t++) {
                if (v_codes) pack_bits(y->v_code + (bh * cap + t) * D, (int)D, y->vbits, v_codes + (bh * Np + t) * tb);
                for (size_t j = 0; j < D / G; j++) {
                    if (v_scale) v_scale[(bh * Np + t) * (D / G) + j] = y->v_s[(bh * cap + t) * (D / G) + j];
                    if (v_zero) v_zero[(bh * Np + t) * (D / G) + j] = y->v_z[(bh * cap + t) * (D / G) + j];
                }
            }
        } else if (v_codes) {
            memcpy(v_codes + bh * Np * D * 2, y->raw_v + bh * cap * D, Np * D * 2);
        }
        if (k_res) memcpy(k_res + bh * Nr * D, y->raw_k + (bh * cap + Np) * D, Nr * D * 2);
        if (v_res) memcpy(v_res + bh * Nr * D, y->raw_v + (bh * cap + Np) * D, Nr * D * 2);
    }
    free(tmp);
    return 0;
}

int kvo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
