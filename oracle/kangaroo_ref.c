/*
 * TEST INFRASTRUCTURE, NOT THE PRODUCT.  Plain CPU reference ("oracle") for the model arithmetic of
 * Kangaroo self-speculative decoding (arXiv 2404.18911).  Only tests, the smoke check and the
 * cpu_baseline leg of the benchmark may use it.  It shares no code with the HIP library.
 *
 * What it computes (all arithmetic in fp64; weights are read as stored, fp32 or bfloat16 bits,
 * and widened exactly):
 *   - the target model M^b of the Notation paragraph of Section 3: a LLaMA-style decoder
 *     (the paper names Vicuna, Section 4.1): token embedding, L pre-norm blocks of
 *     {RMSNorm, multi-head causal self-attention with rotary position embedding, residual,
 *      RMSNorm, SwiGLU feed-forward, residual}, final RMSNorm, LM head;
 *   - the shallow sub-network M^b[:l] and the remaining layers M^b[l:] of Section 3.1, as the
 *     same blocks run over a layer range, with a key/value cache per layer;
 *   - the adapter A of Section 3.1 / Figure 2 / Table 2 row "Kangaroo": input RMSNorm, one
 *     multi-head attention (its own key/value cache), residual, last RMSNorm, shared LM head;
 *   - the other adapter architectures of Table 2's ablation (adapter_kind): 1 "Kangaroo + Head" =
 *     the same with an LM head of its own; 2 "1-Layer Transformer" = one whole decoder block
 *     (attention, post norm, feed-forward, both residuals), last norm, shared head; 3 "MLP Only" =
 *     input norm, two d x d linear maps, last norm, own head.
 *
 * The key/value cache is exact by default (kv_round = 0): that is the plain definition every GPU
 * result is compared with.  A device keeps the cache in 2 bytes per element (16 KB per token and
 * layer at d = 4096); to study what such a storage format costs, kv_round = 1 holds the rotated keys
 * and the values rounded to bfloat16 and kv_round = 2 rounded to IEEE half precision, and attention
 * reads the rounded numbers.
 *
 * Readings where the paper is silent: rotate-half RoPE pairing (i, i+hd/2), base theta, no
 * biases, residual connection around the adapter's attention, early feature = residual stream
 * after block l-1; for the "MLP Only" adapter, h = f + W2 silu(W1 RMSNorm(f)) (the table lists two
 * linear maps and no activation or residual; SiLU is the model's own activation, the residual is
 * what the other rows have).  The decode loops (plain, draft-and-verify, acceptance) live in
 * kangaroo_oracle.py, which calls the routines below.
 *
 * Loops are written as the definitions read: no blocking, no fusion.  OpenMP only spreads
 * independent output elements over threads.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
    int exit_layer;
    int wdtype;            /* 0 = float32, 1 = bfloat16 bit patterns */
    int max_seq;
    int kv_round;          /* cache storage: 0 exact, 1 rounded to bfloat16, 2 rounded to IEEE half */
    int adapter_kind;      /* Table 2: 0 attention, 1 attention + own head, 2 decoder block, 3 two linear maps + own head */
    double rms_eps, rope_theta;
} ko_config;

typedef struct {
    const void *embed, *lm_head, *final_norm;
    const void *const *wq, *const *wk, *const *wv, *const *wo, *const *wg, *const *wu, *const *wd;
    const void *const *norm1, *const *norm2;
    const void *a_wq, *a_wk, *a_wv, *a_wo, *a_norm_in, *a_norm_last;
    const void *a_head, *a_norm_post, *a_wg, *a_wu, *a_wd, *a_w1, *a_w2;   /* NULL unless the kind has them */
} ko_weights;

typedef struct {
    ko_config c;
    ko_weights w;
    /* key/value caches, [n_layers + 1][max_seq][d_model]; index n_layers is the adapter's */
    double *kc, *vc;
} ko_model;

/* weight element i of a stored tensor, widened exactly to double */
static inline double wget(const void *p, int wdtype, size_t i)
{
    if (wdtype == 0) return (double)((const float *)p)[i];
    uint32_t u = (uint32_t)((const uint16_t *)p)[i] << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* value as a bfloat16 cache would hold it: to float (nearest), then to 8 significant bits (nearest even) */
static inline double round_bf16(double x)
{
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    u &= 0xFFFF0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* value as an IEEE half-precision cache would hold it: to float (nearest), then to the nearest
 * number with 11 significant bits in the half range (ties to even; subnormal spacing 2^-24 below
 * 2^-14; beyond the largest half, 65504, rounds to infinity from 65520 on) */
static inline double round_f16(double x)
{
    double f = (double)(float)x;
    if (f == 0.0 || isnan(f) || isinf(f)) return f;
    int e;
    (void)frexp(f, &e);                      /* |f| = m 2^e, 0.5 <= m < 1 */
    int ulp_exp = (e - 1 < -14 ? -14 : e - 1) - 10;
    double r = ldexp(nearbyint(ldexp(f, -ulp_exp)), ulp_exp);   /* nearbyint: ties to even */
    if (fabs(r) > 65504.0) return r > 0 ? INFINITY : -INFINITY;
    return r;
}

static inline double round_kv(const ko_config *c, double x)
{
    return c->kv_round == 1 ? round_bf16(x) : c->kv_round == 2 ? round_f16(x) : x;
}

ko_model *ko_create(const ko_config *c, const ko_weights *w)
{
    ko_model *m = (ko_model *)calloc(1, sizeof(ko_model));
    if (!m) return NULL;
    m->c = *c;
    m->w = *w;
    size_t n = (size_t)(c->n_layers + 1) * c->max_seq * c->d_model;
    m->kc = (double *)calloc(n, sizeof(double));
    m->vc = (double *)calloc(n, sizeof(double));
    if (!m->kc || !m->vc) { free(m->kc); free(m->vc); free(m); return NULL; }
    return m;
}

void ko_destroy(ko_model *m)
{
    if (!m) return;
    free(m->kc); free(m->vc); free(m);
}

/* y[m][n] = sum_k W[n][k] x[m][k],  W is [N][K] row-major */
static void matvec(const void *W, int wdtype, int N, int K, const double *x, int M, double *y)
{
#pragma omp parallel for schedule(static) if ((size_t)N * K * M > 262144)
    for (int n = 0; n < N; n++) {
        for (int m = 0; m < M; m++) {
            const double *xm = x + (size_t)m * K;
            double acc = 0.0;
            if (wdtype == 0) {
                const float *wr = (const float *)W + (size_t)n * K;
#pragma omp simd reduction(+ : acc)
                for (int k = 0; k < K; k++) acc += (double)wr[k] * xm[k];
            } else {
                const uint16_t *wr = (const uint16_t *)W + (size_t)n * K;
#pragma omp simd reduction(+ : acc)
                for (int k = 0; k < K; k++) {
                    union { uint32_t u; float f; } cv;
                    cv.u = (uint32_t)wr[k] << 16;
                    acc += (double)cv.f * xm[k];
                }
            }
            y[(size_t)m * N + n] = acc;
        }
    }
}

/* RMSNorm: y = x * rsqrt(mean(x^2) + eps) * g */
void ko_rmsnorm(const double *x, const void *g, int wdtype, int d, double eps, double *y)
{
    double ss = 0.0;
    for (int i = 0; i < d; i++) ss += x[i] * x[i];
    double s = 1.0 / sqrt(ss / d + eps);
    for (int i = 0; i < d; i++) y[i] = x[i] * s * wget(g, wdtype, i);
}

/* rotary embedding of one head vector at absolute position pos; pairs (i, i + hd/2) */
void ko_rope(double *v, int hd, int pos, double theta)
{
    int half = hd / 2;
    for (int i = 0; i < half; i++) {
        double ang = (double)pos * pow(theta, -2.0 * i / hd);
        double c = cos(ang), s = sin(ang);
        double a = v[i], b = v[i + half];
        v[i] = a * c - b * s;
        v[i + half] = b * c + a * s;
    }
}

/* in-place softmax of n numbers */
void ko_softmax(double *z, int n)
{
    double mx = z[0];
    for (int i = 1; i < n; i++) if (z[i] > mx) mx = z[i];
    double sum = 0.0;
    for (int i = 0; i < n; i++) { z[i] = exp(z[i] - mx); sum += z[i]; }
    for (int i = 0; i < n; i++) z[i] /= sum;
}

/* one head: o = softmax(q.K^T / sqrt(hd)) V over n_keys keys; K,V rows are `stride` apart */
void ko_attend(const double *q, const double *K, const double *V, int n_keys, int hd, int stride,
               double *o)
{
    double *p = (double *)malloc(sizeof(double) * (size_t)n_keys);
    double inv = 1.0 / sqrt((double)hd);
    for (int j = 0; j < n_keys; j++) {
        double s = 0.0;
        for (int i = 0; i < hd; i++) s += q[i] * K[(size_t)j * stride + i];
        p[j] = s * inv;
    }
    ko_softmax(p, n_keys);
    for (int i = 0; i < hd; i++) o[i] = 0.0;
    for (int j = 0; j < n_keys; j++)
        for (int i = 0; i < hd; i++) o[i] += p[j] * V[(size_t)j * stride + i];
    free(p);
}

/*
 * Attention sub-layer with residual on M rows at absolute positions pos0 .. pos0+M-1:
 *   x <- x + Wo . MHA(RMSNorm(x; g)),   keys/values appended to cache slot `slot` at those positions.
 * Row m attends to cache positions 0 .. pos0+m (causal).  Whatever the cache holds beyond
 * pos0+M-1 is neither read nor kept valid: truncating a cache is just using a smaller pos0 next time.
 */
static void attn_sublayer(ko_model *mo, int slot, const void *g, const void *wq, const void *wk,
                          const void *wv, const void *wo, double *x, int pos0, int M)
{
    const ko_config *c = &mo->c;
    int d = c->d_model, H = c->n_heads, hd = c->head_dim, wt = c->wdtype;
    double *a = (double *)malloc(sizeof(double) * (size_t)M * d);
    double *q = (double *)malloc(sizeof(double) * (size_t)M * d);
    double *k = (double *)malloc(sizeof(double) * (size_t)M * d);
    double *v = (double *)malloc(sizeof(double) * (size_t)M * d);
    double *o = (double *)malloc(sizeof(double) * (size_t)M * d);
    double *y = (double *)malloc(sizeof(double) * (size_t)M * d);
    for (int m = 0; m < M; m++) ko_rmsnorm(x + (size_t)m * d, g, wt, d, c->rms_eps, a + (size_t)m * d);
    matvec(wq, wt, d, d, a, M, q);
    matvec(wk, wt, d, d, a, M, k);
    matvec(wv, wt, d, d, a, M, v);
    double *Kc = mo->kc + (size_t)slot * c->max_seq * d;
    double *Vc = mo->vc + (size_t)slot * c->max_seq * d;
    for (int m = 0; m < M; m++) {
        int pos = pos0 + m;
        for (int h = 0; h < H; h++) {
            ko_rope(q + (size_t)m * d + h * hd, hd, pos, c->rope_theta);
            ko_rope(k + (size_t)m * d + h * hd, hd, pos, c->rope_theta);
        }
        if (c->kv_round)
            for (int i = 0; i < d; i++) {
                k[(size_t)m * d + i] = round_kv(c, k[(size_t)m * d + i]);
                v[(size_t)m * d + i] = round_kv(c, v[(size_t)m * d + i]);
            }
        memcpy(Kc + (size_t)pos * d, k + (size_t)m * d, sizeof(double) * d);
        memcpy(Vc + (size_t)pos * d, v + (size_t)m * d, sizeof(double) * d);
    }
#pragma omp parallel for collapse(2) schedule(static) if ((size_t)M * d * (pos0 + M) > 262144)
    for (int m = 0; m < M; m++)
        for (int h = 0; h < H; h++)
            ko_attend(q + (size_t)m * d + h * hd, Kc + h * hd, Vc + h * hd, pos0 + m + 1, hd, d,
                      o + (size_t)m * d + h * hd);
    matvec(wo, wt, d, d, o, M, y);
    for (size_t i = 0; i < (size_t)M * d; i++) x[i] += y[i];
    free(a); free(q); free(k); free(v); free(o); free(y);
}

/* feed-forward sub-layer with residual: x <- x + Wd( silu(Wg b) * (Wu b) ), b = RMSNorm(x; g) */
static void ffn_sublayer(ko_model *mo, const void *g, const void *wg, const void *wu, const void *wd,
                         double *x, int M)
{
    const ko_config *c = &mo->c;
    int d = c->d_model, f = c->d_ffn, wt = c->wdtype;
    double *b = (double *)malloc(sizeof(double) * (size_t)M * d);
    double *gt = (double *)malloc(sizeof(double) * (size_t)M * f);
    double *up = (double *)malloc(sizeof(double) * (size_t)M * f);
    double *y = (double *)malloc(sizeof(double) * (size_t)M * d);
    for (int m = 0; m < M; m++)
        ko_rmsnorm(x + (size_t)m * d, g, wt, d, c->rms_eps, b + (size_t)m * d);
    matvec(wg, wt, f, d, b, M, gt);
    matvec(wu, wt, f, d, b, M, up);
    for (size_t i = 0; i < (size_t)M * f; i++) {
        double z = gt[i];
        gt[i] = z / (1.0 + exp(-z)) * up[i];
    }
    matvec(wd, wt, d, f, gt, M, y);
    for (size_t i = 0; i < (size_t)M * d; i++) x[i] += y[i];
    free(b); free(gt); free(up); free(y);
}

/* x[m] = E[tok[m]] */
void ko_embed(const ko_model *mo, const int32_t *tok, int M, double *x)
{
    int d = mo->c.d_model;
    for (int m = 0; m < M; m++)
        for (int i = 0; i < d; i++)
            x[(size_t)m * d + i] = wget(mo->w.embed, mo->c.wdtype, (size_t)tok[m] * d + i);
}

/* decoder blocks lo .. hi-1 on M rows at positions pos0..; x is [M][d], updated in place.
 * With lo = 0, hi = l this is the shallow sub-network M^b[:l] (its output is the early feature);
 * with lo = l, hi = L it is M^b[l:] (Section 3.1). */
void ko_layers(ko_model *mo, int lo, int hi, double *x, int pos0, int M)
{
    for (int i = lo; i < hi; i++) {
        attn_sublayer(mo, i, mo->w.norm1[i], mo->w.wq[i], mo->w.wk[i], mo->w.wv[i], mo->w.wo[i], x,
                      pos0, M);
        ffn_sublayer(mo, mo->w.norm2[i], mo->w.wg[i], mo->w.wu[i], mo->w.wd[i], x, M);
    }
}

/* adapter A without its last norm, f is [M][d], h likewise (Table 2):
 *   kinds 0, 1: h = f + Wo^A . MHA(RMSNorm(f; g_in))
 *   kind 2:     the same, then h <- h + Wd^A( silu(Wg^A b) * (Wu^A b) ), b = RMSNorm(h; g_post)
 *   kind 3:     h = f + W2 . silu(W1 . RMSNorm(f; g_in)), row by row (no cache, pos0 unused) */
void ko_adapter(ko_model *mo, const double *f, int pos0, int M, double *h)
{
    const ko_config *c = &mo->c;
    int d = c->d_model, wt = c->wdtype;
    memcpy(h, f, sizeof(double) * (size_t)M * d);
    if (c->adapter_kind == 3) {
        double *a = (double *)malloc(sizeof(double) * (size_t)M * d);
        double *u = (double *)malloc(sizeof(double) * (size_t)M * d);
        double *y = (double *)malloc(sizeof(double) * (size_t)M * d);
        for (int m = 0; m < M; m++)
            ko_rmsnorm(f + (size_t)m * d, mo->w.a_norm_in, wt, d, c->rms_eps, a + (size_t)m * d);
        matvec(mo->w.a_w1, wt, d, d, a, M, u);
        for (size_t i = 0; i < (size_t)M * d; i++) u[i] = u[i] / (1.0 + exp(-u[i]));
        matvec(mo->w.a_w2, wt, d, d, u, M, y);
        for (size_t i = 0; i < (size_t)M * d; i++) h[i] += y[i];
        free(a); free(u); free(y);
        return;
    }
    attn_sublayer(mo, mo->c.n_layers, mo->w.a_norm_in, mo->w.a_wq, mo->w.a_wk, mo->w.a_wv,
                  mo->w.a_wo, h, pos0, M);
    if (c->adapter_kind == 2)
        ffn_sublayer(mo, mo->w.a_norm_post, mo->w.a_wg, mo->w.a_wu, mo->w.a_wd, h, M);
}

/* logits[m] = W_head . RMSNorm(x[m]; g), g = final norm (which = 0) or the adapter's last norm (1);
 * the draft head (which = 1) is the adapter's own for kinds 1 and 3, else the shared LM head */
void ko_head(const ko_model *mo, const double *x, int M, int which, double *logits)
{
    const ko_config *c = &mo->c;
    int d = c->d_model;
    double *a = (double *)malloc(sizeof(double) * (size_t)M * d);
    const void *g = which ? mo->w.a_norm_last : mo->w.final_norm;
    for (int m = 0; m < M; m++) ko_rmsnorm(x + (size_t)m * d, g, c->wdtype, d, c->rms_eps, a + (size_t)m * d);
    const void *W = (which && (c->adapter_kind == 1 || c->adapter_kind == 3)) ? mo->w.a_head : mo->w.lm_head;
    matvec(W, c->wdtype, c->vocab, d, a, M, logits);
    free(a);
}

/* copy out the cached key and value rows of one cache slot at one position (for rollback checks) */
void ko_kv_read(const ko_model *mo, int slot, int pos, double *k, double *v)
{
    int d = mo->c.d_model;
    memcpy(k, mo->kc + ((size_t)slot * mo->c.max_seq + pos) * d, sizeof(double) * d);
    memcpy(v, mo->vc + ((size_t)slot * mo->c.max_seq + pos) * d, sizeof(double) * d);
}

/* overwrite every cache entry at positions >= from with NaN, so that a stale read shows up */
void ko_kv_poison(ko_model *mo, int from)
{
    int d = mo->c.d_model;
    for (int s = 0; s <= mo->c.n_layers; s++)
        for (int p = from; p < mo->c.max_seq; p++)
            for (int i = 0; i < d; i++) {
                mo->kc[((size_t)s * mo->c.max_seq + p) * d + i] = NAN;
                mo->vc[((size_t)s * mo->c.max_seq + p) * d + i] = NAN;
            }
}

/* the cache roundings (exposed so that tests can pin ties and the double -> float step) */
double ko_round_bf16(double x)
{
    return round_bf16(x);
}
double ko_round_f16(double x)
{
    return round_f16(x);
}

/* y = W x for a bare stored matrix (exposed so that tests can pin the widening and the loop) */
void ko_matvec(const void *W, int wdtype, int N, int K, const double *x, int M, double *y)
{
    matvec(W, wdtype, N, K, x, M, y);
}
