/* Host-sanitizer driver: runs the CPU oracle and the input generator on a tiny model inside one
 * executable built with -fsanitize=address,undefined (tests/test_sanitizers.py builds and runs it).
 * It checks memory safety and undefined behaviour of the two C sources, not numerics. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

/* oracle/ref_decoder.c (double build) */
typedef struct { int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn_dim, vocab; double rms_eps, rope_base; } ref_config;
typedef struct ref_model ref_model;
typedef struct ref_cache ref_cache;
ref_model *ref_model_new(const ref_config *c);
void ref_model_free(ref_model *m);
int ref_model_set_tensor(ref_model *m, int kind, int layer, const void *data, int dtype);
ref_cache *ref_cache_new(const ref_model *m, int max_tokens, int kv_store);
void ref_cache_free(ref_cache *c);
int ref_cache_len(const ref_cache *c);
int ref_truncate(ref_cache *c, int new_len);
void ref_cache_export(const ref_cache *c, double *out);
int ref_decode_one(ref_cache *c, int token, double *logits);
int ref_forward_block(ref_cache *c, const int32_t *tokens, int n, double *logits, int only_last);
int ref_verify(ref_cache *c, int prefix_len, const int32_t *draft, int gamma, int32_t *pending, int32_t *accepted_len,
               int32_t *next_token, int32_t *pred_out, double *logits);
int ref_embed_block(const ref_model *m, const int32_t *tokens, int n, double *X);
int ref_layer_block(ref_cache *c, int l, int T, double *X, int n);
int ref_head_block(const ref_model *m, const double *X, int n, double *logits);
int ref_cache_set_len(ref_cache *c, int len);
double ref_store_round(double v, int mode);

/* pv_inputs/synth.c */
int pvs_fill_table(uint64_t seed, uint64_t stream, uint64_t start, uint64_t count, const void *table, int elt, void *out);
int pvs_quantize_q4(const void *w_bits, int64_t rows, int64_t cols, void *codes, void *scales);

#define CHECK(x) do { if (!(x)) { fprintf(stderr, "san_driver: check failed: %s (line %d)\n", #x, __LINE__); return 1; } } while (0)

int main(void)
{
    const ref_config cfg = { 2, 64, 4, 2, 16, 96, 128, 1e-5, 10000.0 };
    const int d = cfg.d_model, qd = cfg.n_q_heads * cfg.head_dim, kvd = cfg.n_kv_heads * cfg.head_dim, F = cfg.ffn_dim, V = cfg.vocab;
    /* a 65536-entry bf16 table of small values and tensors drawn from it by the generator */
    uint16_t *table = (uint16_t *)malloc(65536 * sizeof(uint16_t));
    for (int i = 0; i < 65536; ++i) { float f = ((float)i - 32768.0f) * (0.06f / 65536.0f); uint32_t u; memcpy(&u, &f, 4); table[i] = (uint16_t)(u >> 16); }
    const size_t sizes[12] = { (size_t)V * d, d, (size_t)qd * d, (size_t)kvd * d, (size_t)kvd * d, (size_t)d * qd, d, (size_t)F * d, (size_t)F * d, (size_t)d * F, d, (size_t)V * d };
    ref_model *m = ref_model_new(&cfg);
    CHECK(m);
    uint16_t *bufs[3][12] = {{0}};
    for (int l = -1; l < cfg.n_layers; ++l)
        for (int k = 0; k < 12; ++k) {
            const int global = (k == 0 || k == 10 || k == 11);
            if ((l < 0) != global) continue;
            uint16_t *w = (uint16_t *)malloc(sizes[k] * sizeof(uint16_t));
            CHECK(pvs_fill_table(1234, (uint64_t)((l + 1) * 16 + k), 0, sizes[k], table, 2, w) == 0);
            if (k == 1 || k == 6 || k == 10) for (size_t i = 0; i < sizes[k]; ++i) w[i] = 0x3F80;    /* gains of 1.0 */
            bufs[l + 1][k] = w;
            CHECK(ref_model_set_tensor(m, k, l, w, 1) == 0);
        }
    /* the 4-bit quantiser on one matrix */
    {
        uint8_t *codes = (uint8_t *)malloc((size_t)F * d / 2);
        uint16_t *scales = (uint16_t *)malloc((size_t)F * d / 32 * sizeof(uint16_t));
        CHECK(pvs_quantize_q4(bufs[1][7], F, d, codes, scales) == 0);
        free(codes); free(scales);
    }
    for (int kv = 0; kv < 3; ++kv) {
        ref_cache *c = ref_cache_new(m, 40, kv);
        CHECK(c);
        int32_t prompt[21];
        for (int i = 0; i < 21; ++i) prompt[i] = (i * 37 + 5) % V;
        double *lg = (double *)malloc(sizeof(double) * 8 * V);
        CHECK(ref_forward_block(c, prompt, 13, NULL, 0) == 0);
        CHECK(ref_forward_block(c, prompt + 13, 8, lg, 1) == 0);
        CHECK(ref_cache_len(c) == 21);
        CHECK(ref_decode_one(c, 3, lg) == 0 && ref_truncate(c, 21) == 0);
        int32_t draft[8] = { 1, 2, 3, 4, 5, 6, 7, 8 }, pred[8], pending = -1, acc = -1, nxt = -1;
        CHECK(ref_verify(c, 21, draft, 8, &pending, &acc, &nxt, pred, lg) == 0);
        CHECK(acc >= 1 && acc <= 8 && nxt >= 0 && nxt < V && ref_cache_len(c) == 21 + acc);
        CHECK(ref_verify(c, 20, draft, 8, &pending, &acc, &nxt, pred, NULL) != 0);            /* wrong prefix length is refused */
        CHECK(ref_forward_block(c, prompt, 21, NULL, 0) != 0);                                /* would not fit */
        double *ex = (double *)malloc(sizeof(double) * cfg.n_layers * 2 * ref_cache_len(c) * kvd);
        ref_cache_export(c, ex);
        /* the layer-by-layer routines over the same cache */
        double *X = (double *)malloc(sizeof(double) * 8 * d);
        const int T = ref_cache_len(c);
        CHECK(ref_embed_block(m, draft, 8, X) == 0);
        for (int l = 0; l < cfg.n_layers; ++l) CHECK(ref_layer_block(c, l, T, X, 8) == 0);
        CHECK(ref_head_block(m, X, 8, lg) == 0 && ref_cache_set_len(c, T + 8) == 0 && ref_cache_set_len(c, 41) != 0);
        CHECK(ref_truncate(c, 0) == 0 && ref_truncate(c, 1) != 0);
        free(X); free(ex); free(lg);
        ref_cache_free(c);
    }
    CHECK(ref_store_round(1.00390625, 1) == 1.0);
    for (int l = 0; l < 3; ++l) for (int k = 0; k < 12; ++k) free(bufs[l][k]);
    ref_model_free(m);
    free(table);
    puts("san_driver ok");
    return 0;
}
