/* The plain-C oracle under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only): layer steps with shared
 * prefix pages, chunked prefill, decode rows, a model step and the greedy choice on small random inputs, with
 * exactly sized buffers so that any read or write outside them is reported. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "relserve_oracle.h"

static unsigned long long g_rng = 0x2545f4914f6cdd1dull;
static unsigned rnd(void) { g_rng = g_rng * 6364136223846793005ull + 1442695040888963407ull; return (unsigned)(g_rng >> 33); }
static float rnd_unit(void) { return (float)(rnd() % 20001) / 10000.0f - 1.0f; }
static uint16_t* rnd_bf16(size_t n, float scale, float mean) {
    uint16_t* p = (uint16_t*)malloc(sizeof(uint16_t) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = oracle_f32_to_bf16(mean + scale * rnd_unit());
    return p;
}
#define EXPECT(cond) do { if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

int main(void) {
    const int shapes[3][5] = {{64, 4, 4, 16, 96}, {64, 8, 2, 16, 80}, {128, 2, 1, 64, 160}};   /* H, n_q, n_kv, d, I */
    for (int s = 0; s < 3; ++s) {
        oracle_config c = {shapes[s][0], shapes[s][1], shapes[s][2], shapes[s][3], shapes[s][4], 8, 1e-5f, 10000.0f};
        const int H = c.hidden, qd = c.n_q_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim, I = c.mlp_dim, P = c.page_size;
        /* 5 requests: three share a 2-page prefix; chunk continuation, decode rows, a fresh prompt */
        const int32_t q_len[5] = {9, 1, 4, 1, 13}, past[5] = {2 * P + 3, 2 * P + 11, 2 * P, 21, 0};
        int32_t q_start[6] = {0}, ctx[5], blocks[5], max_blocks = 0;
        for (int r = 0; r < 5; ++r) {
            q_start[r + 1] = q_start[r] + q_len[r];
            ctx[r] = past[r] + q_len[r];
            blocks[r] = (ctx[r] + P - 1) / P;
            if (blocks[r] > max_blocks) max_blocks = blocks[r];
        }
        int32_t* bt = (int32_t*)calloc((size_t)5 * max_blocks, sizeof(int32_t));
        int next = 2;                                   /* pages 0, 1 = the shared prefix */
        for (int r = 0; r < 5; ++r)
            for (int i = 0; i < blocks[r]; ++i) bt[r * max_blocks + i] = (r < 3 && i < 2) ? i : next++;
        const int num_pages = next;                     /* exactly as many pages as the block tables name */
        oracle_batch b = {5, max_blocks, q_start, ctx, bt};
        const int T = q_start[5];
        oracle_weights w = {rnd_bf16(H, 0.02f, 1.0f), rnd_bf16((size_t)(qd + 2 * kvd) * H, 0.05f, 0), rnd_bf16((size_t)H * qd, 0.05f, 0),
                            rnd_bf16(H, 0.02f, 1.0f), rnd_bf16((size_t)2 * I * H, 0.05f, 0), rnd_bf16((size_t)H * I, 0.05f, 0)};
        uint16_t* x = rnd_bf16((size_t)T * H, 1.0f, 0);
        uint16_t* kp = rnd_bf16((size_t)num_pages * P * kvd, 1.0f, 0);
        uint16_t* vp = rnd_bf16((size_t)num_pages * P * kvd, 1.0f, 0);
        float* y = (float*)malloc(sizeof(float) * (size_t)T * H);
        uint16_t* yb = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)T * H);
        float* attn = (float*)malloc(sizeof(float) * (size_t)T * qd);
        float* x1 = (float*)malloc(sizeof(float) * (size_t)T * H);
        EXPECT(oracle_layer_step(&c, &b, &w, x, kp, vp, num_pages, NULL, 0, y, yb, attn, x1) == 0);
        for (int i = 0; i < T * H; ++i) EXPECT(isfinite(y[i]));
        /* a selection of rows, exactly sized outputs */
        const int32_t rows[3] = {0, q_start[2], T - 1};
        float* ys = (float*)malloc(sizeof(float) * 3 * (size_t)H);
        EXPECT(oracle_layer_step(&c, &b, &w, x, kp, vp, num_pages, rows, 3, ys, NULL, NULL, NULL) == 0);
        for (int i = 0; i < H; ++i) EXPECT(ys[2 * H + i] == y[(size_t)(T - 1) * H + i]);   /* the step is idempotent on the cache */
        /* stand-alone append with a slot list, and a page count one too small */
        uint16_t* k = rnd_bf16((size_t)T * kvd, 1.0f, 0);
        int32_t* slots = (int32_t*)malloc(sizeof(int32_t) * (size_t)T);
        EXPECT(oracle_kv_append(&c, &b, k, k, kp, vp, num_pages, slots) == 0);
        EXPECT(oracle_kv_append(&c, &b, k, k, kp, vp, num_pages - 1, slots) != 0);
        /* model step: 2 layers, vocabulary 50 */
        const int V = 50;
        oracle_weights lw[2] = {w, w};
        uint16_t* emb = rnd_bf16((size_t)V * H, 1.0f, 0);
        uint16_t* head = rnd_bf16((size_t)V * H, 0.05f, 0);
        oracle_model m = {2, V, emb, lw, w.w_in_norm, head};
        int32_t* ids = (int32_t*)malloc(sizeof(int32_t) * (size_t)T);
        for (int t = 0; t < T; ++t) ids[t] = (int32_t)(rnd() % V);
        uint16_t* kp2 = rnd_bf16((size_t)num_pages * P * kvd, 1.0f, 0);
        uint16_t* vp2 = rnd_bf16((size_t)num_pages * P * kvd, 1.0f, 0);
        uint16_t* kps[2] = {kp, kp2};
        uint16_t* vps[2] = {vp, vp2};
        float* logits = (float*)malloc(sizeof(float) * 5 * (size_t)V);
        uint16_t* hidden = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)T * H);
        EXPECT(oracle_model_step(&c, &m, &b, ids, kps, vps, num_pages, logits, hidden) == 0);
        ids[0] = V;
        EXPECT(oracle_model_step(&c, &m, &b, ids, kps, vps, num_pages, logits, hidden) == -6);
        int32_t next_tok[5];
        oracle_greedy_sample(logits, 5, V, next_tok);
        for (int r = 0; r < 5; ++r) EXPECT(next_tok[r] >= 0 && next_tok[r] < V);
        /* the quantised variants on exactly sized buffers: 8-bit pools, then 8-bit projections over 16-bit and 8-bit pools */
        {
            const size_t pool = (size_t)num_pages * P * kvd;
            uint8_t* k8 = (uint8_t*)malloc(pool);
            uint8_t* v8 = (uint8_t*)malloc(pool);
            for (size_t i = 0; i < pool; ++i) k8[i] = (uint8_t)(rnd() % 0x60), v8[i] = (uint8_t)(0x80 | (rnd() % 0x60));
            EXPECT(oracle_layer_step_fp8kv(&c, &b, &w, x, k8, v8, num_pages, 0.05f, 0.04f, rows, 3, ys, NULL, NULL, NULL) == 0);
            EXPECT(oracle_layer_step_fp8kv(&c, &b, &w, x, k8, v8, num_pages, 0.0f, 0.04f, rows, 3, ys, NULL, NULL, NULL) == -7);
            const size_t n_w[4] = {(size_t)(qd + 2 * kvd) * H, (size_t)H * qd, (size_t)2 * I * H, (size_t)H * I};
            const int n_rows_w[4] = {qd + 2 * kvd, H, 2 * I, H};
            uint8_t* wc[4];
            float* sw[4];
            for (int m = 0; m < 4; ++m) {
                wc[m] = (uint8_t*)malloc(n_w[m]);
                sw[m] = (float*)malloc(sizeof(float) * (size_t)n_rows_w[m]);
                for (size_t i = 0; i < n_w[m]; ++i) wc[m][i] = (uint8_t)((rnd() % 0x70) | ((rnd() & 1) << 7));
                for (int i = 0; i < n_rows_w[m]; ++i) sw[m][i] = 1e-3f * (1.0f + 0.5f * rnd_unit());
            }
            oracle_weights_w8a8 q8 = {w.w_in_norm, wc[0], sw[0], wc[1], sw[1], w.w_post_norm, wc[2], sw[2], wc[3], sw[3],
                                      0.02f, 0.01f, 0.02f, 0.05f};
            EXPECT(oracle_layer_step_w8a8(&c, &b, &q8, x, kp, vp, num_pages, 0, 1.0f, 1.0f, NULL, 0, y, yb, attn, x1) == 0);
            for (int i = 0; i < T * H; ++i) EXPECT(isfinite(y[i]));
            EXPECT(oracle_layer_step_w8a8(&c, &b, &q8, x, k8, v8, num_pages, 1, 0.05f, 0.04f, rows, 3, ys, NULL, NULL, NULL) == 0);
            q8.a_o = 0.0f;
            EXPECT(oracle_layer_step_w8a8(&c, &b, &q8, x, kp, vp, num_pages, 0, 1.0f, 1.0f, rows, 3, ys, NULL, NULL, NULL) == -7);
            for (int m = 0; m < 4; ++m) { free(wc[m]); free(sw[m]); }
            free(k8); free(v8);
        }
        free(bt); free((void*)w.w_in_norm); free((void*)w.w_qkv); free((void*)w.w_o); free((void*)w.w_post_norm);
        free((void*)w.w_gate_up); free((void*)w.w_down); free(x); free(kp); free(vp); free(y); free(yb); free(attn); free(x1);
        free(ys); free(k); free(slots); free(emb); free(head); free(ids); free(kp2); free(vp2); free(logits); free(hidden);
    }
    printf("oracle under ASan + UBSan: ok\n");
    return 0;
}
