/*
 * TEST INFRASTRUCTURE ONLY -- plain, slow, double-precision CPU reference of the decoder
 * forward that ConfLayers' self-speculative decoding runs (draft with a layer skip set,
 * full-model verification, per-layer confidence).  Nothing in the product path may call
 * into this file; it shares no code with the HIP library.
 *
 * What it follows:
 *   - decoder: a Llama-style pre-norm block (RMSNorm, rotary embedding, KV-cache
 *     attention, SwiGLU MLP), the model family named in Section 4.1.1;
 *   - draft model = target model with the layers of the skip set S removed, a skipped
 *     layer leaving the residual stream untouched (Section 3, description of Figure 2);
 *   - verification = one forward pass of the full model over the drafted tokens
 *     (Section 1, speculative decoding paragraph);
 *   - confidence = 1 - H(softmax(logits)) / log K, with the logits cast to fp32-range
 *     values, clamped, soft-maxed (Eq. 1), entropy with epsilon inside the log (Eq. 2),
 *     normalised by H_max = log K (Eq. 3, Eq. 4); logits of a layer come from projecting
 *     its hidden state through the shared LM head (Section 3.1).
 *
 * All arithmetic is IEEE double, sums run left to right over the reduction index,
 * compiled with -ffp-contract=off so no fused multiply-add changes a rounding.
 * Matrices are row-major [out][in]; weights arrive as fp32 or as raw bf16 / fp16 bit patterns
 * (uint16) and are widened exactly.
 *
 * Storage precision of the K/V cache is a stated model parameter, orc_config.kv_storage:
 *   ORC_KV_EXACT (-1): the cache holds the fp64 values -- the plain definition of attention over
 *       the keys and values of Section 1 / Section 3, nothing rounded;
 *   0 / 1 / 2: the cache stores each K (after the rotary embedding) and V element rounded to
 *       fp32 / bf16 / fp16, round-to-nearest-even, via an fp32 intermediate as a half-precision
 *       tensor is produced from fp32 compute -- the reading of Section 4.1.1 (models evaluated in
 *       half precision, so the cache of such a model holds half-precision numbers) -- and
 *       attention reads those stored values, for the rows of the current block too.
 * Everything else stays in double in both modes.  Both modes are pinned by the CPU tests.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab, max_seq;
    double rms_eps, rope_base;
    int32_t weight_dtype; /* 0 = float32, 1 = bf16 stored as uint16, 2 = IEEE fp16 stored as uint16 */
    int32_t kv_storage;   /* ORC_KV_EXACT = cache in fp64; 0 / 1 / 2 = K, V rounded to fp32 / bf16 / fp16 when stored */
} orc_config;

#define ORC_KV_EXACT (-1)

typedef struct {
    orc_config c;
    const void *embed, *lm_head;
    const float *final_norm;
    const float **attn_norm, **mlp_norm;
    const void **wq, **wk, **wv, **wo, **wg, **wu, **wd;
    double *kcache, *vcache; /* [L][max_seq][d_kv] */
} orc_model;

static double widen_bf16(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* IEEE binary16 bit pattern -> double (exact): 1 sign, 5 exponent (bias 15), 10 fraction bits */
static double widen_fp16(uint16_t h)
{
    int sign = h >> 15, e = (h >> 10) & 31, f = h & 1023;
    double v;
    if (e == 0) v = ldexp((double)f, -24);                     /* zero and subnormals: f * 2^-24 */
    else if (e == 31) v = f ? NAN : INFINITY;
    else v = ldexp((double)(1024 + f), e - 25);               /* (1 + f/1024) * 2^(e-15) */
    return sign ? -v : v;
}

/* x rounded to fp32 and then to fp16 (round-to-nearest-even both times), returned as a double.
 * The fp16 step rounds the fp32 value on the fp16 grid: spacing 2^(e-10) for |x| in [2^e, 2^(e+1)),
 * e >= -14, and 2^-24 below 2^-14; values that round to 65520 or more become infinity. */
double orc_round_fp16(double x)
{
    float f = (float)x;
    if (!(f == f) || f == INFINITY || f == -INFINITY) return (double)f;
    double a = fabs((double)f);
    if (a == 0.0) return (double)f;
    int e;
    (void)frexp(a, &e);              /* a = m * 2^e, m in [0.5, 1): a in [2^(e-1), 2^e) */
    int ex = e - 1;
    if (ex < -14) ex = -14;
    double q = ldexp(1.0, ex - 10);  /* grid spacing */
    double r = nearbyint(a / q) * q; /* a / q is exact (power of two), nearbyint rounds half to even */
    if (r >= 65520.0) r = INFINITY;
    return f < 0 ? -r : r;
}

/* x rounded to fp32 and then to bf16 (round-to-nearest-even both times), returned as a double */
double orc_round_bf16(double x)
{
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7F800000u) == 0x7F800000u) return (double)f; /* inf / nan unchanged */
    u += 0x7FFFu + ((u >> 16) & 1u);
    u &= 0xFFFF0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

static double round_storage(double x, int kv_storage)
{
    if (kv_storage == ORC_KV_EXACT) return x;
    return kv_storage == 0 ? (double)(float)x : kv_storage == 1 ? orc_round_bf16(x) : orc_round_fp16(x);
}

/* The same conversion for all 65 536 bit patterns, tabulated once per process (the formula above, evaluated
 * ahead of the matrix products instead of inside their inner loop); filled by orc_create before any use. */
static double fp16_value[65536];
static int fp16_value_ready = 0;
static void fill_fp16_table(void)
{
    if (fp16_value_ready) return;
    for (int h = 0; h < 65536; h++) fp16_value[h] = widen_fp16((uint16_t)h);
    fp16_value_ready = 1;
}

/* Y[r][n] = sum_k W[n][k] * X[r][k]   (W: N x K row-major, X: R x K, Y: R x N).
 * Every output is its own left-to-right sum over k, exactly as written; up to ORC_RB rows r share one pass over the
 * weight row n (their sums advance side by side, none of them is reassociated), so the weight is widened once per
 * pass instead of once per row. */
#define ORC_RB 8
static void matmul_wt(const void *W, int dtype, int N, int K, const double *X, int R, double *Y)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; n++) {
        const float *wf = (const float *)W + (size_t)n * K;
        const uint16_t *wh = (const uint16_t *)W + (size_t)n * K;
        for (int r0 = 0; r0 < R; r0 += ORC_RB) {
            const int nr = R - r0 < ORC_RB ? R - r0 : ORC_RB;
            double acc[ORC_RB];
            const double *x[ORC_RB];
            for (int j = 0; j < nr; j++) { acc[j] = 0.0; x[j] = X + (size_t)(r0 + j) * K; }
            if (nr == 1) {   /* a single row: one scalar running sum */
                double a0 = 0.0;
                const double *x0 = x[0];
                for (int k = 0; k < K; k++) {
                    const double w = dtype == 0 ? (double)wf[k] : dtype == 1 ? widen_bf16(wh[k]) : fp16_value[wh[k]];
                    a0 += w * x0[k];
                }
                acc[0] = a0;
            } else if (nr == ORC_RB) {
                for (int k = 0; k < K; k++) {
                    const double w = dtype == 0 ? (double)wf[k] : dtype == 1 ? widen_bf16(wh[k]) : fp16_value[wh[k]];
                    for (int j = 0; j < ORC_RB; j++) acc[j] += w * x[j][k];
                }
            } else {
                for (int k = 0; k < K; k++) {
                    const double w = dtype == 0 ? (double)wf[k] : dtype == 1 ? widen_bf16(wh[k]) : fp16_value[wh[k]];
                    for (int j = 0; j < nr; j++) acc[j] += w * x[j][k];
                }
            }
            for (int j = 0; j < nr; j++) Y[(size_t)(r0 + j) * N + n] = acc[j];
        }
    }
}

/* out = x * rsqrt(mean(x^2) + eps) * gain */
static void rmsnorm(const double *x, const float *gain, int d, double eps, double *out)
{
    double ss = 0.0;
    for (int i = 0; i < d; i++) ss += x[i] * x[i];
    double s = 1.0 / sqrt(ss / (double)d + eps);
    for (int i = 0; i < d; i++) out[i] = x[i] * s * (double)gain[i];
}

/* Rotary embedding of one head vector at position p: element i pairs with i + hd/2 and the
 * pair is rotated by the angle p * base^(-2i/hd). */
static void rope_head(double *v, int hd, int p, double base)
{
    int half = hd / 2;
    for (int i = 0; i < half; i++) {
        double ang = (double)p * pow(base, -2.0 * (double)i / (double)hd);
        double c = cos(ang), s = sin(ang);
        double a = v[i], b = v[i + half];
        v[i] = a * c - b * s;
        v[i + half] = b * c + a * s;
    }
}

orc_model *orc_create(const orc_config *cfg, const void *embed, const void *lm_head,
                      const float *final_norm, const float **attn_norm, const void **wq,
                      const void **wk, const void **wv, const void **wo, const float **mlp_norm,
                      const void **wg, const void **wu, const void **wd)
{
    if (!cfg || cfg->n_heads % cfg->n_kv_heads || cfg->head_dim % 2) return NULL;
    if (cfg->kv_storage < ORC_KV_EXACT || cfg->kv_storage > 2) return NULL;
    orc_model *m = (orc_model *)calloc(1, sizeof(orc_model));
    m->c = *cfg;
    fill_fp16_table();
    int L = cfg->n_layers;
    m->embed = embed; m->lm_head = lm_head; m->final_norm = final_norm;
#define COPYP(field, type) m->field = (type)malloc(sizeof(void *) * L); memcpy((void *)m->field, field, sizeof(void *) * L)
    COPYP(attn_norm, const float **); COPYP(mlp_norm, const float **);
    COPYP(wq, const void **); COPYP(wk, const void **); COPYP(wv, const void **); COPYP(wo, const void **);
    COPYP(wg, const void **); COPYP(wu, const void **); COPYP(wd, const void **);
#undef COPYP
    size_t n = (size_t)L * cfg->max_seq * cfg->n_kv_heads * cfg->head_dim;
    m->kcache = (double *)calloc(n, sizeof(double));
    m->vcache = (double *)calloc(n, sizeof(double));
    if (!m->kcache || !m->vcache) return NULL;
    return m;
}

void orc_destroy(orc_model *m)
{
    if (!m) return;
    free((void *)m->attn_norm); free((void *)m->mlp_norm);
    free((void *)m->wq); free((void *)m->wk); free((void *)m->wv); free((void *)m->wo);
    free((void *)m->wg); free((void *)m->wu); free((void *)m->wd);
    free(m->kcache); free(m->vcache); free(m);
}

/* Overwrite every cache entry at positions >= from_pos with NaN (stale-entry safety tests). */
void orc_kv_poison(orc_model *m, int from_pos)
{
    int dkv = m->c.n_kv_heads * m->c.head_dim;
    for (int l = 0; l < m->c.n_layers; l++)
        for (int p = from_pos; p < m->c.max_seq; p++)
            for (int i = 0; i < dkv; i++) {
                size_t o = ((size_t)l * m->c.max_seq + p) * dkv + i;
                m->kcache[o] = NAN; m->vcache[o] = NAN;
            }
}

double *orc_kcache(orc_model *m) { return m->kcache; }
double *orc_vcache(orc_model *m) { return m->vcache; }

/*
 * Forward R token rows at positions pos0 .. pos0+R-1 (row r sees cache positions
 * 0 .. pos0+r, i.e. causal inside the block).  sub_skip (optional) has two entries per layer:
 * sub_skip[2l] != 0 leaves out the attention sub-block of layer l (no projections, no cache
 * write, residual unchanged), sub_skip[2l+1] != 0 its MLP sub-block -- the two modules whose
 * hidden states Section 3.1 scores separately; a layer of the skip set S of Section 3 has both
 * set.  Executed attention sub-blocks write their K/V rows into the cache at the rows' positions.
 *   taps   (optional) [R][L][2][d]: residual stream after the attention sub-block and
 *          after the MLP sub-block of every layer (for a skipped layer both equal its input)
 *   logits (optional) [R][V]
 *   hidden (optional) [R][d]: residual stream after the last layer (before the final norm)
 * Returns 0, or -1 on bad arguments.
 */
int orc_forward_sub(orc_model *m, const int32_t *tokens, int R, int pos0, const uint8_t *sub_skip,
                    double *taps, double *logits, double *hidden)
{
    const orc_config *c = &m->c;
    int L = c->n_layers, d = c->d_model, H = c->n_heads, Hkv = c->n_kv_heads, hd = c->head_dim;
    int dq = H * hd, dkv = Hkv * hd, f = c->d_ffn, V = c->vocab, wt = c->weight_dtype;
    if (R <= 0 || pos0 < 0 || pos0 + R > c->max_seq) return -1;
    for (int r = 0; r < R; r++) if (tokens[r] < 0 || tokens[r] >= V) return -1;

    double *x = (double *)malloc(sizeof(double) * R * d);
    double *h = (double *)malloc(sizeof(double) * R * d);
    double *q = (double *)malloc(sizeof(double) * R * dq);
    double *kk = (double *)malloc(sizeof(double) * R * dkv);
    double *vv = (double *)malloc(sizeof(double) * R * dkv);
    double *att = (double *)malloc(sizeof(double) * R * dq);
    double *t1 = (double *)malloc(sizeof(double) * R * d);
    double *gt = (double *)malloc(sizeof(double) * R * f);
    double *up = (double *)malloc(sizeof(double) * R * f);
    int group = H / Hkv;
    double inv_sqrt_hd = 1.0 / sqrt((double)hd);

    for (int r = 0; r < R; r++)
        for (int i = 0; i < d; i++) {
            size_t o = (size_t)tokens[r] * d + i;
            x[(size_t)r * d + i] = wt == 0   ? (double)((const float *)m->embed)[o]
                                   : wt == 1 ? widen_bf16(((const uint16_t *)m->embed)[o])
                                             : fp16_value[((const uint16_t *)m->embed)[o]];
        }

    for (int l = 0; l < L; l++) {
        const int skip_attn = sub_skip && sub_skip[2 * l], skip_mlp = sub_skip && sub_skip[2 * l + 1];
        double *Kc = m->kcache + (size_t)l * c->max_seq * dkv;
        double *Vc = m->vcache + (size_t)l * c->max_seq * dkv;
        /* attention sub-block */
        if (!skip_attn) {
        for (int r = 0; r < R; r++) rmsnorm(x + (size_t)r * d, m->attn_norm[l], d, c->rms_eps, h + (size_t)r * d);
        matmul_wt(m->wq[l], wt, dq, d, h, R, q);
        matmul_wt(m->wk[l], wt, dkv, d, h, R, kk);
        matmul_wt(m->wv[l], wt, dkv, d, h, R, vv);
        for (int r = 0; r < R; r++) {
            int p = pos0 + r;
            for (int hh = 0; hh < H; hh++) rope_head(q + (size_t)r * dq + hh * hd, hd, p, c->rope_base);
            for (int hh = 0; hh < Hkv; hh++) rope_head(kk + (size_t)r * dkv + hh * hd, hd, p, c->rope_base);
            for (int i = 0; i < dkv; i++) {
                Kc[(size_t)p * dkv + i] = round_storage(kk[(size_t)r * dkv + i], c->kv_storage);
                Vc[(size_t)p * dkv + i] = round_storage(vv[(size_t)r * dkv + i], c->kv_storage);
            }
        }
#pragma omp parallel for schedule(static) collapse(2)
        for (int r = 0; r < R; r++)
            for (int hh = 0; hh < H; hh++) {
                int p = pos0 + r, kvh = hh / group;
                const double *qv = q + (size_t)r * dq + hh * hd;
                double *s = (double *)malloc(sizeof(double) * (p + 1));
                double mx = -INFINITY;
                for (int j = 0; j <= p; j++) {
                    const double *kr = Kc + (size_t)j * dkv + kvh * hd;
                    double a = 0.0;
                    for (int i = 0; i < hd; i++) a += qv[i] * kr[i];
                    s[j] = a * inv_sqrt_hd;
                    if (s[j] > mx) mx = s[j];
                }
                double z = 0.0;
                for (int j = 0; j <= p; j++) { s[j] = exp(s[j] - mx); z += s[j]; }
                double *o = att + (size_t)r * dq + hh * hd;
                for (int i = 0; i < hd; i++) o[i] = 0.0;
                for (int j = 0; j <= p; j++) {
                    const double *vr = Vc + (size_t)j * dkv + kvh * hd;
                    double w = s[j] / z;
                    for (int i = 0; i < hd; i++) o[i] += w * vr[i];
                }
                free(s);
            }
        matmul_wt(m->wo[l], wt, d, dq, att, R, t1);
        for (size_t i = 0; i < (size_t)R * d; i++) x[i] += t1[i];
        }
        if (taps)
            for (int r = 0; r < R; r++)
                memcpy(taps + (((size_t)r * L + l) * 2 + 0) * d, x + (size_t)r * d, sizeof(double) * d);
        /* MLP sub-block: x += Wd (silu(Wg h) * (Wu h)),  silu(z) = z / (1 + exp(-z)) */
        if (!skip_mlp) {
        for (int r = 0; r < R; r++) rmsnorm(x + (size_t)r * d, m->mlp_norm[l], d, c->rms_eps, h + (size_t)r * d);
        matmul_wt(m->wg[l], wt, f, d, h, R, gt);
        matmul_wt(m->wu[l], wt, f, d, h, R, up);
        for (size_t i = 0; i < (size_t)R * f; i++) gt[i] = gt[i] / (1.0 + exp(-gt[i])) * up[i];
        matmul_wt(m->wd[l], wt, d, f, gt, R, t1);
        for (size_t i = 0; i < (size_t)R * d; i++) x[i] += t1[i];
        }
        if (taps)
            for (int r = 0; r < R; r++)
                memcpy(taps + (((size_t)r * L + l) * 2 + 1) * d, x + (size_t)r * d, sizeof(double) * d);
    }
    if (hidden) memcpy(hidden, x, sizeof(double) * R * d);
    if (logits) {
        for (int r = 0; r < R; r++) rmsnorm(x + (size_t)r * d, m->final_norm, d, c->rms_eps, h + (size_t)r * d);
        matmul_wt(m->lm_head, wt, V, d, h, R, logits);
    }
    free(x); free(h); free(q); free(kk); free(vv); free(att); free(t1); free(gt); free(up);
    return 0;
}

/* The draft model of Section 3: layers with skip[l] != 0 (the skip set S) are left out entirely. */
int orc_forward(orc_model *m, const int32_t *tokens, int R, int pos0, const uint8_t *skip,
                double *taps, double *logits, double *hidden)
{
    if (!skip) return orc_forward_sub(m, tokens, R, pos0, NULL, taps, logits, hidden);
    int L = m->c.n_layers;
    uint8_t *sub = (uint8_t *)malloc((size_t)2 * L);
    for (int l = 0; l < L; l++) sub[2 * l] = sub[2 * l + 1] = skip[l] ? 1 : 0;
    int rc = orc_forward_sub(m, tokens, R, pos0, sub, taps, logits, hidden);
    free(sub);
    return rc;
}

/* Index of the largest logit; the lowest index wins a tie. */
int32_t orc_argmax(const double *z, int V)
{
    int32_t best = 0;
    for (int i = 1; i < V; i++) if (z[i] > z[best]) best = i;
    return best;
}

/*
 * Confidence of one logit vector (Eq. 1-4): round to fp32 ("cast to FP32"), clamp to
 * [-clamp, clamp], softmax, H = -sum p_i log(p_i + eps), confidence = 1 - H / log K.
 * Also reports max_i p_i and the arg-max (lowest index on ties) of the clamped logits.
 */
void orc_confidence_from_logits(const double *z, int V, double clamp, double eps,
                                double *conf, double *maxprob, int32_t *argmax)
{
    double *c = (double *)malloc(sizeof(double) * V);
    for (int i = 0; i < V; i++) {
        double v = (double)(float)z[i];
        if (v > clamp) v = clamp;
        if (v < -clamp) v = -clamp;
        c[i] = v;
    }
    int32_t am = orc_argmax(c, V);
    double mx = c[am], Z = 0.0;
    for (int i = 0; i < V; i++) Z += exp(c[i] - mx);
    double Hs = 0.0;
    for (int i = 0; i < V; i++) {
        double p = exp(c[i] - mx) / Z;
        Hs -= p * log(p + eps);
    }
    if (conf) *conf = 1.0 - Hs / log((double)V);
    if (maxprob) *maxprob = 1.0 / Z;
    if (argmax) *argmax = am;
    free(c);
}

/*
 * Confidence of n hidden-state rows [n][d]: final RMSNorm, shared LM head, then Eq. 1-4.
 * logits_out (optional) [n][V] receives the un-clamped logits.
 */
void orc_confidence(orc_model *m, const double *hidden, int n, double clamp, double eps,
                    double *conf, double *maxprob, int32_t *argmax, double *logits_out)
{
    int d = m->c.d_model, V = m->c.vocab;
    double *h = (double *)malloc(sizeof(double) * n * d);
    double *z = logits_out ? logits_out : (double *)malloc(sizeof(double) * n * V);
    for (int r = 0; r < n; r++) rmsnorm(hidden + (size_t)r * d, m->final_norm, d, m->c.rms_eps, h + (size_t)r * d);
    matmul_wt(m->lm_head, m->c.weight_dtype, V, d, h, n, z);
    for (int r = 0; r < n; r++)
        orc_confidence_from_logits(z + (size_t)r * V, V, clamp, eps, conf ? conf + r : NULL,
                                   maxprob ? maxprob + r : NULL, argmax ? argmax + r : NULL);
    free(h);
    if (!logits_out) free(z);
}
