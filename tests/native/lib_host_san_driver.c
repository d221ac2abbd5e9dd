/* Host-only paths of libkangaroo's sources under AddressSanitizer and UndefinedBehaviorSanitizer:
 * this driver is compiled together with csrc/kangaroo.hip (host code instrumented, device code as
 * usual) and calls what the library does without touching a device: configuration checks, size
 * arithmetic, call-order errors, the metrics of Eq. 1 / Eq. 2, the tile order, argument checks of
 * the stand-alone ops.  Prints one line per check; exit status 0 when every check held. */
#include <stdint.h>
#include <stdio.h>
#include <string.h>
#include "kangaroo.h"

static int failures;
#define CHECK(cond) do { if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); failures++; } } while (0)

static kg_config toy(void)
{
    kg_config c;
    memset(&c, 0, sizeof(c));
    c.n_layers = 4; c.d_model = 256; c.n_heads = 4; c.head_dim = 64; c.d_ffn = 688; c.vocab = 1024;
    c.exit_layer = 1; c.dtype = 0; c.kv_dtype = 0; c.rms_eps = 1e-6f; c.rope_theta = 10000.f;
    c.max_seq = 128; c.gamma_max = 6; c.kv_page_tokens = 16; c.adapter_kind = 0;
    return c;
}

int main(void)
{
    kg_ctx *h = NULL;
    kg_config c = toy();
    CHECK(kg_create(&c, &h) == KG_OK && h);
    size_t wb = 0, kb = 0, sb = 0;
    CHECK(kg_workspace_bytes(h, &wb, &kb, &sb) == KG_OK && wb > 0 && sb > 0);
    CHECK(kb == (size_t)8 * 16 * 5 * 2 * 256 * 4);            /* pages x tokens x caches x (K, V) x d x fp32 */
    kg_params p;
    memset(&p, 0, sizeof(p));
    p.temperature = 1.f; p.eta = 0.6f; p.gamma = 6;
    int32_t tok = 0, buf[8] = {0}, prompt[4] = {1, 2, 3, 4};
    float conf = 0.f;
    int stop = 0, n = 0;
    CHECK(kg_prefill(h, &p, prompt, 4, &tok) == KG_ESTATE);
    CHECK(strstr(kg_last_error(h), "kg_bind") != NULL);
    CHECK(kg_draft_step(h, &p, &tok, &conf, &stop) == KG_ESTATE);
    CHECK(kg_verify(h, &p, buf, &n) == KG_ESTATE);
    CHECK(kg_accept(h, &p, buf, &n) == KG_ESTATE);
    CHECK(kg_load_tensor(h, 0, -1, NULL, 0) == KG_ESTATE);
    CHECK(kg_bind(h, NULL, 0, NULL, 0, NULL, 0, NULL) == KG_EINVAL);
    CHECK(kg_bind(h, (void *)256, 1, (void *)256, 1, (void *)512, 1, NULL) == KG_ENOSPC);
    int32_t bad_perm[8] = {0, 1, 2, 2, 4, 5, 6, 7}, perm[8] = {7, 1, 2, 0, 4, 5, 6, 3};       /* 128 / 16 pages */
    CHECK(kg_set_page_order(h, bad_perm, 8) == KG_EINVAL);
    CHECK(kg_set_page_order(h, perm, 4) == KG_EINVAL);
    CHECK(kg_set_page_order(h, perm, 8) == KG_OK);
    size_t tb = 0;
    CHECK(kg_train_workspace_bytes(h, 64, &tb) == KG_OK && tb > 0);
    CHECK(kg_train_workspace_bytes(h, 0, &tb) == KG_EINVAL);
    kg_destroy(h);

    /* every field the configuration check looks at, out of range */
    struct { int field, value; } bad[] = {{0, 0}, {0, 5}, {1, 48}, {2, 3}, {3, 8}, {4, 24}, {4, 256}, {5, 2}, {6, 3}, {7, 1000},
                                          {8, 1}, {9, 4}, {9, -1}};
    for (unsigned i = 0; i < sizeof(bad) / sizeof(bad[0]); i++) {
        kg_config b = toy();
        switch (bad[i].field) {
        case 0: b.exit_layer = bad[i].value; break;
        case 1: b.head_dim = bad[i].value; break;
        case 2: b.n_heads = bad[i].value; break;
        case 3: b.gamma_max = bad[i].value; break;
        case 4: b.kv_page_tokens = bad[i].value; break;
        case 5: b.dtype = bad[i].value; break;
        case 6: b.kv_dtype = bad[i].value; break;
        case 7: b.vocab = bad[i].value; break;
        case 8: b.max_seq = bad[i].value; break;
        default: b.adapter_kind = bad[i].value; break;
        }
        kg_ctx *hb = (kg_ctx *)1;
        CHECK(kg_create(&b, &hb) == KG_EINVAL && hb == NULL);
    }
    CHECK(kg_create(NULL, NULL) == KG_EINVAL);

    /* Eq. 1 and Eq. 2 on S = (1, 3, 2, 7, 1): CR = 14 / 5, CTAR(1) = 3 / 5, CTAR(2) = 2 / 5, CTAR(6) = 1 / 5 */
    kg_stats st;
    memset(&st, 0, sizeof(st));
    st.rounds = 5; st.s_hist[1] = 2; st.s_hist[2] = 1; st.s_hist[3] = 1; st.s_hist[7] = 1; st.emitted = 15;
    double v = 0.0;
    CHECK(kg_stats_cr(&st, &v) == KG_OK && v > 2.799 && v < 2.801);
    CHECK(kg_stats_ctar(&st, 1, &v) == KG_OK && v > 0.599 && v < 0.601);
    CHECK(kg_stats_ctar(&st, 2, &v) == KG_OK && v > 0.399 && v < 0.401);
    CHECK(kg_stats_ctar(&st, 6, &v) == KG_OK && v > 0.199 && v < 0.201);
    memset(&st, 0, sizeof(st));
    CHECK(kg_stats_cr(&st, &v) == KG_EINVAL);

    /* sizes, the tile order (a permutation for every K), argument checks of the stand-alone ops */
    CHECK(kg_op_packed_bytes(1, 4096, 4096) == (size_t)4096 * 4096 * 2);
    CHECK(kg_op_packed_bytes(1, 1024, 688) == (size_t)1024 * 704 * 2);
    CHECK(kg_op_work_bytes(4096) == (size_t)4096 * 32);
    for (int KS = 1; KS <= 600; KS++) {
        unsigned char seen[600];
        memset(seen, 0, sizeof(seen));
        int ok = 1;
        for (int ks = 0; ks < KS; ks++) {
            const int pos = kg_op_tile_pos(ks, KS);
            if (pos < 0 || pos >= KS || seen[pos]) ok = 0; else seen[pos] = 1;
        }
        if (!ok) { printf("FAILED tile order at KS = %d\n", KS); failures++; }
    }
    CHECK(kg_op_tile_pos(-1, 8) == -1 && kg_op_tile_pos(8, 8) == -1);
    CHECK(kg_op_pack(1, (void *)256, 17, 64, (void *)256, NULL) == KG_EINVAL);
    CHECK(kg_op_linear(1, (void *)256, 64, 64, (float *)256, 9, (float *)256, (void *)256, NULL) == KG_EINVAL);
    CHECK(kg_op_stream_read(NULL, 1 << 20, (void *)256, NULL) == KG_EINVAL);
    CHECK(kg_op_linear_static(1, (void *)256, 64, KG_OP_STATIC_MAX_K + 32, (float *)256, 1, (float *)256, NULL) == KG_ENOSPC);
    printf("%s (%d failed)\n", failures ? "FAILED" : "OK", failures);
    return failures ? 1 : 0;
}
