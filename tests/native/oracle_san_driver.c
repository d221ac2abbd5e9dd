/*
 * TEST INFRASTRUCTURE.  Driver that runs the CPU oracle's C routines (oracle/kangaroo_ref.c,
 * oracle/philox_ref.c) natively, so that they can be built with -fsanitize=address,undefined and
 * exercised without a Python interpreter in the process.  tests/test_oracle_sanitized.py writes the
 * input file (shape, weights, tokens), runs this program and compares its output file, number for
 * number, with what the regular build of the oracle returns for the same calls.
 *
 * Input file:  int32 header[16] = {n_layers, d_model, n_heads, head_dim, d_ffn, vocab, exit_layer,
 *              wdtype, max_seq, kv_round, adapter_kind, n_tokens, 0...}, double rms_eps, rope_theta,
 *              int32 tokens[n_tokens], then the tensors as raw bytes in the order the test and this
 *              file agree on: embed, lm_head, final_norm, per layer (wq wk wv wo wg wu wd norm1 norm2),
 *              a_wq a_wk a_wv a_wo a_norm_in a_norm_last.
 * Output file: doubles: early features, adapter outputs, final hidden states, target logits, draft
 *              logits of all tokens (the prompt is fed in pieces of 4, 1, 1, 3, ... rows), the cached
 *              key/value rows of every cache at two positions, the two cache roundings of a few
 *              numbers, 64 Philox words (as doubles) and a row of uniforms.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
    int exit_layer;
    int wdtype;
    int max_seq;
    int kv_round;
    int adapter_kind;
    double rms_eps, rope_theta;
} ko_config;

typedef struct {
    const void *embed, *lm_head, *final_norm;
    const void *const *wq, *const *wk, *const *wv, *const *wo, *const *wg, *const *wu, *const *wd;
    const void *const *norm1, *const *norm2;
    const void *a_wq, *a_wk, *a_wv, *a_wo, *a_norm_in, *a_norm_last;
    const void *a_head, *a_norm_post, *a_wg, *a_wu, *a_wd, *a_w1, *a_w2;
} ko_weights;

typedef struct ko_model ko_model;
ko_model *ko_create(const ko_config *c, const ko_weights *w);
void ko_destroy(ko_model *m);
void ko_embed(const ko_model *mo, const int32_t *tok, int M, double *x);
void ko_layers(ko_model *mo, int lo, int hi, double *x, int pos0, int M);
void ko_adapter(ko_model *mo, const double *f, int pos0, int M, double *h);
void ko_head(const ko_model *mo, const double *x, int M, int which, double *logits);
void ko_kv_read(const ko_model *mo, int slot, int pos, double *k, double *v);
void ko_kv_poison(ko_model *mo, int from);
double ko_round_bf16(double x);
double ko_round_f16(double x);
void ko_philox_words(uint64_t seed, uint32_t pos0, uint32_t purpose, int n, uint32_t *out);
void ko_philox_uniforms(uint64_t seed, int n_positions, float *u);

/* every buffer of the driver is remembered and freed at the end, so that the leak check speaks
 * about the oracle only */
static void *held[4096];
static int n_held;
static void *hold(size_t bytes)
{
    void *p = malloc(bytes ? bytes : 1);
    if (!p || n_held == 4096) { fprintf(stderr, "out of memory\n"); exit(2); }
    held[n_held++] = p;
    return p;
}
static void *take(FILE *f, size_t bytes)
{
    void *p = hold(bytes);
    if (fread(p, 1, bytes, f) != bytes) { fprintf(stderr, "short input\n"); exit(2); }
    return p;
}

int main(int argc, char **argv)
{
    if (argc != 3) return 2;
    FILE *in = fopen(argv[1], "rb"), *out = fopen(argv[2], "wb");
    if (!in || !out) return 2;
    int32_t h[16];
    double dd[2];
    if (fread(h, 4, 16, in) != 16 || fread(dd, 8, 2, in) != 2) return 2;
    ko_config c = {h[0], h[1], h[2], h[3], h[4], h[5], h[6], h[7], h[8], h[9], h[10], dd[0], dd[1]};
    const int T = h[11], L = c.n_layers, d = c.d_model, f = c.d_ffn, V = c.vocab;
    const size_t es = c.wdtype ? 2 : 4;
    int32_t *tok = (int32_t *)take(in, (size_t)T * 4);
    ko_weights w;
    memset(&w, 0, sizeof(w));
    w.embed = take(in, (size_t)V * d * es);
    w.lm_head = take(in, (size_t)V * d * es);
    w.final_norm = take(in, (size_t)d * es);
    const void **per[9];
    for (int k = 0; k < 9; k++) per[k] = (const void **)hold(sizeof(void *) * L);
    const size_t sz[9] = {(size_t)d * d, (size_t)d * d, (size_t)d * d, (size_t)d * d, (size_t)f * d, (size_t)f * d,
                          (size_t)d * f, (size_t)d, (size_t)d};
    for (int i = 0; i < L; i++)
        for (int k = 0; k < 9; k++) per[k][i] = take(in, sz[k] * es);
    w.wq = per[0]; w.wk = per[1]; w.wv = per[2]; w.wo = per[3]; w.wg = per[4]; w.wu = per[5]; w.wd = per[6];
    w.norm1 = per[7]; w.norm2 = per[8];
    w.a_wq = take(in, (size_t)d * d * es); w.a_wk = take(in, (size_t)d * d * es);
    w.a_wv = take(in, (size_t)d * d * es); w.a_wo = take(in, (size_t)d * d * es);
    w.a_norm_in = take(in, (size_t)d * es); w.a_norm_last = take(in, (size_t)d * es);

    ko_model *m = ko_create(&c, &w);
    if (!m) return 3;
    double *F = (double *)hold(sizeof(double) * T * d), *Hh = (double *)hold(sizeof(double) * T * d);
    double *X = (double *)hold(sizeof(double) * T * d);
    double *Zt = (double *)hold(sizeof(double) * T * V), *Zd = (double *)hold(sizeof(double) * T * V);
    const int pieces[5] = {4, 1, 1, 3, 2};
    int pos = 0, pi = 0;
    while (pos < T) {
        int M = pieces[pi++ % 5];
        if (M > T - pos) M = T - pos;
        double *x = F + (size_t)pos * d;
        ko_embed(m, tok + pos, M, x);
        ko_layers(m, 0, c.exit_layer, x, pos, M);
        ko_adapter(m, x, pos, M, Hh + (size_t)pos * d);
        memcpy(X + (size_t)pos * d, x, sizeof(double) * M * d);
        ko_layers(m, c.exit_layer, L, X + (size_t)pos * d, pos, M);
        ko_head(m, X + (size_t)pos * d, M, 0, Zt + (size_t)pos * V);
        ko_head(m, Hh + (size_t)pos * d, M, 1, Zd + (size_t)pos * V);
        pos += M;
    }
    fwrite(F, 8, (size_t)T * d, out); fwrite(Hh, 8, (size_t)T * d, out); fwrite(X, 8, (size_t)T * d, out);
    fwrite(Zt, 8, (size_t)T * V, out); fwrite(Zd, 8, (size_t)T * V, out);
    double *kv = (double *)hold(sizeof(double) * 2 * d);
    ko_kv_poison(m, T);                                  /* the tail up to max_seq: must not touch what is read below */
    for (int s = 0; s <= L; s++)
        for (int p = 0; p < T; p += T - 1 > 0 ? T - 1 : 1) {
            ko_kv_read(m, s, p, kv, kv + d);
            fwrite(kv, 8, (size_t)2 * d, out);
        }
    const double probe[6] = {1.0 + 1.0 / 256, -3.14159, 65519.9, 1e-7, 0.0, 1.0 + 3.0 / 2048};
    for (int i = 0; i < 6; i++) {
        double r[2] = {ko_round_bf16(probe[i]), ko_round_f16(probe[i])};
        fwrite(r, 8, 2, out);
    }
    uint32_t words[64];
    ko_philox_words(0x0123456789ABCDEFull, 4294967290u, 2, 64, words);
    for (int i = 0; i < 64; i++) { double v = (double)words[i]; fwrite(&v, 8, 1, out); }
    float u[3 * 16];
    ko_philox_uniforms(77, 16, u);
    for (int i = 0; i < 48; i++) { double v = (double)u[i]; fwrite(&v, 8, 1, out); }
    ko_destroy(m);
    while (n_held) free(held[--n_held]);
    fclose(in);
    if (fclose(out)) return 4;
    return 0;
}
