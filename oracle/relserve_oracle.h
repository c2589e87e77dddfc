/*
 * RelServe layer-step ORACLE -- test infrastructure, not product code.
 *
 * A plain, slow CPU statement of what one forward step of a decoder layer
 * computes over a mixed prefill+decode batch whose requests keep their keys
 * and values in a paged cache.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it; the GPU library never links or loads it and
 * shares no source with it.
 *
 * What the paper fixes: the q/k/v projections (Sec. 2.3 "Self-Attention
 * Module", Eq. 3), causal softmax attention with scale 1/sqrt(d) (Eq. 4), the
 * weighted value sum followed by W_o (Eq. 5), the KV cache as a pure memo of
 * earlier tokens' keys and values (Sec. 2.3 "KV Cache"), the prefill / decode
 * split (Sec. 2.3 "Prefill and Decode Phases") and prefix reuse (Sec. 2.3
 * "Prefix Cache").  Everything else (pre-norm layer wiring, RMSNorm, rotary
 * embedding, SwiGLU, grouped-query head mapping, page layout) is the reading
 * listed below; the paper is silent on it.
 *
 * Readings (each is also listed in the design notes of the repository):
 *   R1  layer = x1 = x + W_o attn(rope(W_qkv rmsnorm(x)));  y = x1 + W_d(silu(W_g h2) * W_u h2),
 *       h2 = rmsnorm(x1); no biases.
 *   R2  rmsnorm(x)_i = x_i * w_i / sqrt(mean_j x_j^2 + eps)   (eps inside the root).
 *   R3  rotary embedding pairs (i, i + d/2), angle = pos * base^(-2i/d), applied
 *       to q and k only; pos = index of the token in its own request's sequence
 *       (a shared prefix occupies positions 0..prefix_len-1 of every member).
 *   R4  d in Eq. 4 is the head dimension.
 *   R5  the sum in Eq. 4/5 includes j = i; the step's own keys/values are first
 *       rounded to bf16 and written to the cache, then read back from it, so a
 *       key seen "this step" and "a later step" has the same bits.
 *   R6  ctx_len[r] counts keys visible to the request's LAST query token of this
 *       step, i.e. the sequence length after the append.
 *   R7  query head a reads kv head a / (n_q_heads / n_kv_heads).
 *   R8  weights are row-major [out_features, in_features]; w_qkv rows are
 *       [q heads | k heads | v heads]; w_gate_up rows are [gate | up].
 *   R9  cache: k_pages and v_pages are [num_pages, P, n_kv_heads, d] bf16;
 *       token at position pos of request r lives in
 *       slot = block_table[r][pos / P] * P + pos % P.
 *   R10 a shared prefix is nothing but equal leading block-table entries; the
 *       oracle has no notion of prefix ids.
 *   R14 greedy next token: the largest logit, the lowest token id among equal ones.
 *   R15 quantised cache (a variant; the paper runs 16-bit caches): the pools hold 8-bit floating point
 *       codes (1 sign, 4 exponent, 3 mantissa bits, bias 7, largest magnitude 448, no infinity) of
 *       x / scale with one scale per pool, given by the caller (as an engine calibrates it offline).
 *       The step's rotated keys and its values are quantised ONCE from their fp32 values:
 *       code = round-to-nearest-even(x * (1 / scale)), magnitudes above 448 become 448, with the
 *       reciprocal formed in double and rounded to fp32; a cached element reads back as
 *       value(code) * scale in fp32.  A code is an integer decided by floating point, so the decision is
 *       taken in the precision the kernel takes it in: in this variant the normed activations are
 *       rounded to bf16 before the q/k/v projection (bf16 inputs, fp32 sums); otherwise two correct
 *       implementations would disagree on the ~5 % of codes whose value lies next to a rounding boundary.
 *       Everything else is unchanged.
 *   R16 quantised projections (a variant; the paper runs 16-bit models): each of the four projection matrices
 *       holds 8-bit codes (the format of R15) of W[n, :] / s_w[n] with one fp32 scale per output row, and the
 *       input of each projection is quantised to codes of a / s_a with one scale per projection, given by the
 *       caller (static, as an engine calibrates it offline): code = round-to-nearest-even(a * (1 / s_a)),
 *       magnitudes above 448 become 448, the reciprocal formed in double and rounded to fp32.
 *       out[t, n] = (sum_k value(a_code[t, k]) * value(w_code[n, k])) * (s_a * s_w[n]); the products are exact in
 *       fp32, the sum is an fp32 sum, the two scales are multiplied first.  What is quantised: the normed
 *       activations from their fp32 values (both norms); the attention output after its rounding to bf16 (it
 *       exists as bf16 between the attention and W_o); silu(g) * u from its fp32 value.  With R16 the bf16
 *       rounding of R15 before the q/k/v projection does not apply (its input is the codes).  Residuals, norms,
 *       rotary embedding, attention and the cache are unchanged.
 *
 * Precision: inputs, weights and the cache hold bf16 bit patterns (uint16_t);
 * all arithmetic is fp32 with acc_t accumulators (float, or double when built
 * with -DORACLE_ACC_F64, which is how the oracle's own rounding error is
 * measured); rotary angles and the softmax scale are formed in double and
 * rounded once.  y is returned in fp32 before the final rounding and, when
 * asked, as round-to-nearest-even bf16.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py (brute
 * force attention, library routines, closed forms and the memoisation /
 * paging / prefix / chunking invariants); nothing is "parity unpinned".
 */
#ifndef RELSERVE_ORACLE_H
#define RELSERVE_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t hidden;      /* H */
    int32_t n_q_heads;   /* n_h */
    int32_t n_kv_heads;  /* n_kv, divides n_h */
    int32_t head_dim;    /* d, even */
    int32_t mlp_dim;     /* I */
    int32_t page_size;   /* P */
    float   rms_eps;
    float   rope_base;
} oracle_config;

typedef struct {
    int32_t num_reqs;
    int32_t max_blocks;           /* row stride of block_table */
    const int32_t* q_start;       /* [num_reqs + 1] packed query-token ranges */
    const int32_t* ctx_len;       /* [num_reqs] sequence length after this step (R6) */
    const int32_t* block_table;   /* [num_reqs, max_blocks] page ids */
} oracle_batch;

typedef struct {
    const uint16_t* w_in_norm;    /* [H] */
    const uint16_t* w_qkv;        /* [(n_h + 2 n_kv) d, H] */
    const uint16_t* w_o;          /* [H, n_h d] */
    const uint16_t* w_post_norm;  /* [H] */
    const uint16_t* w_gate_up;    /* [2 I, H] */
    const uint16_t* w_down;       /* [H, I] */
} oracle_weights;

/* bf16 <-> fp32 (bit patterns); round-to-nearest-even on the way down. */
float    oracle_bf16_to_f32(uint16_t b);
uint16_t oracle_f32_to_bf16(float f);

/* R2. x, out: [n_rows, H] fp32; w: [H] bf16 bits. */
void oracle_rmsnorm(const float* x, const uint16_t* w, float eps,
                    int32_t n_rows, int32_t H, float* out);

/* Eq. 3 and every other dense map: out[t, n] = sum_k W[n, k] * in[t, k]. */
void oracle_linear(const uint16_t* W, int32_t N, int32_t K,
                   const float* in, int32_t n_rows, float* out);

/* R3, in place on one head vector of length d. */
void oracle_rope(float* vec, int32_t d, int32_t pos, float base);

/* Cache write (R9) of already-rotated bf16 keys and values, k/v: [T, n_kv, d].
 * Returns 0, or -1 if a slot falls outside num_pages. slots_out (optional,
 * [T]) receives the slot of every token. */
int32_t oracle_kv_append(const oracle_config* c, const oracle_batch* b,
                         const uint16_t* k, const uint16_t* v,
                         uint16_t* k_pages, uint16_t* v_pages, int32_t num_pages,
                         int32_t* slots_out);

/* Eq. 4 and the sum of Eq. 5 (before W_o) for one query token of request r at
 * position pos: q [n_h, d] fp32 -> out [n_h, d] fp32, keys 0..pos read from the
 * paged cache through r's block-table row. */
void oracle_attention_token(const oracle_config* c, const oracle_batch* b,
                            int32_t r, int32_t pos, const float* q,
                            const uint16_t* k_pages, const uint16_t* v_pages,
                            float* out);

/* R15: the 8-bit format of the quantised cache. */
float   oracle_e4m3_to_f32(uint8_t code);
uint8_t oracle_f32_to_e4m3(float x);

/* oracle_attention_token over a quantised cache (R15). */
void oracle_attention_token_fp8kv(const oracle_config* c, const oracle_batch* b,
                                  int32_t r, int32_t pos, const float* q,
                                  const uint8_t* k_pages, const uint8_t* v_pages, float k_scale, float v_scale,
                                  float* out);

/* R16: quantised projections. */
typedef struct {
    const uint16_t* w_in_norm;    /* [H] bf16 */
    const uint8_t*  w_qkv;        /* [(n_h + 2 n_kv) d, H] codes */
    const float*    s_qkv;        /* [(n_h + 2 n_kv) d] scale of each output row */
    const uint8_t*  w_o;          /* [H, n_h d] */
    const float*    s_o;          /* [H] */
    const uint16_t* w_post_norm;  /* [H] bf16 */
    const uint8_t*  w_gate_up;    /* [2 I, H] */
    const float*    s_gate_up;    /* [2 I] */
    const uint8_t*  w_down;       /* [H, I] */
    const float*    s_down;       /* [H] */
    float a_qkv, a_o, a_gate_up, a_down;   /* scale of each projection's input */
} oracle_weights_w8a8;

void oracle_quantise(const float* in, int64_t n, float scale, uint8_t* codes);
void oracle_linear_w8a8(const uint8_t* Wc, const float* s_w, int32_t N, int32_t K,
                        const uint8_t* in_c, float a_scale, int32_t n_rows, float* out);

/* The whole step.  x: [T, H] bf16.  The cache is updated in place for every
 * token of the batch.  rows/n_rows select which token rows get the rest of the
 * layer (NULL/0 = all T, in order); y_f32 [n_out, H] and optional y_bf16 are
 * indexed by position in that selection.  Optional taps (any may be NULL), each
 * indexed like y: attn_out [n_out, n_h d] (input of W_o), x1 [n_out, H].
 * Returns 0 or a negative code for an inconsistent batch. */
int32_t oracle_layer_step(const oracle_config* c, const oracle_batch* b,
                          const oracle_weights* w, const uint16_t* x,
                          uint16_t* k_pages, uint16_t* v_pages, int32_t num_pages,
                          const int32_t* rows, int32_t n_rows,
                          float* y_f32, uint16_t* y_bf16,
                          float* tap_attn_out, float* tap_x1);

/* oracle_layer_step with the quantised cache of R15: pools [num_pages, P, n_kv, d] of 8-bit codes.
 * Returns -7 for a scale that is not positive. */
int32_t oracle_layer_step_fp8kv(const oracle_config* c, const oracle_batch* b,
                                const oracle_weights* w, const uint16_t* x,
                                uint8_t* k_pages, uint8_t* v_pages, int32_t num_pages, float k_scale, float v_scale,
                                const int32_t* rows, int32_t n_rows,
                                float* y_f32, uint16_t* y_bf16,
                                float* tap_attn_out, float* tap_x1);

/* oracle_layer_step with the quantised projections of R16, over a 16-bit cache (kv_fp8 = 0: pools of bf16, the
 * scales are ignored) or the quantised cache of R15 (kv_fp8 = 1: pools of codes).  Returns -7 for a scale that
 * is not positive. */
int32_t oracle_layer_step_w8a8(const oracle_config* c, const oracle_batch* b,
                               const oracle_weights_w8a8* q8, const uint16_t* x,
                               void* k_pages, void* v_pages, int32_t num_pages, int32_t kv_fp8, float k_scale, float v_scale,
                               const int32_t* rows, int32_t n_rows,
                               float* y_f32, uint16_t* y_bf16,
                               float* tap_attn_out, float* tap_x1);

/* A stack of identical-shape layers between an embedding table and an output
 * layer (Sec. 2.3 "LLM Inference": embedding layer, Transformer layers, output
 * layer that turns the final hidden representation of the LAST token into
 * logits for the next token).  Readings: R11 the residual stream is rounded to
 * bf16 between layers (it is the layer step's bf16 output); R12 a final RMSNorm
 * (R2) precedes the output layer; R13 logits are produced for the last query
 * token of every request of the batch, in fp32. */
typedef struct {
    int32_t n_layers;
    int32_t vocab;
    const uint16_t* embedding;        /* [vocab, H] */
    const oracle_weights* layers;     /* [n_layers] */
    const uint16_t* w_final_norm;     /* [H] */
    const uint16_t* w_lm_head;        /* [vocab, H] */
} oracle_model;

/* token_ids [T]; k_pages / v_pages: one pool per layer; logits [num_reqs, vocab];
 * hidden_out (optional) [T, H] bf16 = the last layer's output.  Returns 0 or a
 * negative code (-6: token id outside the vocabulary). */
int32_t oracle_model_step(const oracle_config* c, const oracle_model* m, const oracle_batch* b,
                          const int32_t* token_ids, uint16_t* const* k_pages, uint16_t* const* v_pages,
                          int32_t num_pages, float* logits, uint16_t* hidden_out);

/* Sec. 2.3 "LLM Inference": the output layer's logits of a request's last token give its next token.
 * Greedy choice (reading R14): the largest logit, the lowest token id among equals, NaN never chosen.
 * logits [n_rows, vocab] fp32 -> next_token [n_rows].  Pinned by numpy's argmax, planted ties and
 * hand-written rows (tests/test_oracle_pins.py). */
void oracle_greedy_sample(const float* logits, int32_t n_rows, int32_t vocab, int32_t* next_token);

/* 1 when built with double accumulators. */
int32_t oracle_acc_is_f64(void);
/* Threads the parallel loops (oracle_linear, the per-token attention loop) use. */
int32_t oracle_num_threads(void);

/* oracle_model_step with the quantised projections of R16 in every layer (layers [m->n_layers]; m->layers is not
 * read); embedding, final norm and output layer are the 16-bit ones of m; 16-bit cache pools. */
int32_t oracle_model_step_w8a8(const oracle_config* c, const oracle_model* m, const oracle_weights_w8a8* layers,
                               const oracle_batch* b, const int32_t* token_ids,
                               uint16_t* const* k_pages, uint16_t* const* v_pages,
                               int32_t num_pages, float* logits, uint16_t* hidden_out);

#ifdef __cplusplus
}
#endif
#endif
