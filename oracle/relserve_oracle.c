/*
 * RelServe layer-step ORACLE -- test infrastructure, not product code.
 * See relserve_oracle.h for what is computed, the readings taken where the
 * paper is silent, and the precision.  Everything below is the definition
 * written out: no tiling, no online softmax, no fusion.
 */
#include "relserve_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#ifdef ORACLE_ACC_F64
typedef double acc_t;
#else
typedef float acc_t;
#endif

int32_t oracle_acc_is_f64(void) { return (int32_t)(sizeof(acc_t) == sizeof(double)); }

#ifdef _OPENMP
#include <omp.h>
int32_t oracle_num_threads(void) { return (int32_t)omp_get_max_threads(); }
#else
int32_t oracle_num_threads(void) { return 1; }
#endif

float oracle_bf16_to_f32(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

uint16_t oracle_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u)        /* NaN stays NaN, quiet */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;              /* ties go to the even mantissa */
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

/* R15: 8-bit floating point of the quantised cache: 1 sign, 4 exponent (bias 7), 3 mantissa bits; the largest
 * finite magnitude is 448 (0x7e); 0x7f / 0xff are NaN; there is no infinity.  Subnormals are multiples of 2^-9. */
float oracle_e4m3_to_f32(uint8_t code)
{
    int e = (code >> 3) & 0xf, m = code & 7;
    float mag;
    if (e == 0xf && m == 7) return NAN;
    if (e == 0) mag = ldexpf((float)m, -9);
    else        mag = ldexpf((float)(8 + m), e - 7 - 3);
    return (code & 0x80) ? -mag : mag;
}

/* round to nearest, ties to the even mantissa; magnitudes above 448 (and infinities) become 448; NaN stays NaN */
uint8_t oracle_f32_to_e4m3(float x)
{
    if (x != x) return 0x7f;
    uint8_t sign = signbit(x) ? 0x80 : 0x00;
    float a = fabsf(x);
    if (a >= 448.0f) return (uint8_t)(sign | 0x7e);
    int e;
    (void)frexpf(a, &e);                 /* a = f * 2^e, f in [0.5, 1): the binade of a is [2^(e-1), 2^e) */
    int q = e - 1 - 3;                   /* spacing 2^q keeps 4 significant bits ...                      */
    if (q < -9) q = -9;                  /* ... but never finer than the subnormal spacing                */
    float n = nearbyintf(ldexpf(a, -q)); /* exact scaling, then ties-to-even (default rounding mode)      */
    if (n == 0.0f) return sign;
    float r = ldexpf(n, q);              /* the rounded magnitude; may have moved up into the next binade */
    (void)frexpf(r, &e);
    int E = e - 1 + 7;                   /* biased exponent of r                                          */
    if (E <= 0) return (uint8_t)(sign | (uint8_t)ldexpf(r, 9));          /* subnormal: r / 2^-9 in 1..7    */
    int m = (int)ldexpf(r, 3 - (e - 1)) - 8;
    return (uint8_t)(sign | (E << 3) | m);
}

/* R2: x_i * w_i / sqrt(mean(x^2) + eps) */
void oracle_rmsnorm(const float* x, const uint16_t* w, float eps,
                    int32_t n_rows, int32_t H, float* out)
{
    for (int32_t t = 0; t < n_rows; ++t) {
        const float* xr = x + (size_t)t * H;
        acc_t ss = 0;
        for (int32_t i = 0; i < H; ++i) ss += (acc_t)xr[i] * (acc_t)xr[i];
        float inv = (float)(1.0 / sqrt((double)ss / (double)H + (double)eps));
        for (int32_t i = 0; i < H; ++i)
            out[(size_t)t * H + i] = xr[i] * inv * oracle_bf16_to_f32(w[i]);
    }
}

/* out[t, n] = <W[n, :], in[t, :]>  (Eq. 3; R8 for the orientation) */
void oracle_linear(const uint16_t* W, int32_t N, int32_t K,
                   const float* in, int32_t n_rows, float* out)
{
#pragma omp parallel for schedule(static)
    for (int32_t n = 0; n < N; ++n) {
        const uint16_t* wr = W + (size_t)n * K;
        for (int32_t t = 0; t < n_rows; ++t) {
            const float* xr = in + (size_t)t * K;
            acc_t acc = 0;
#pragma omp simd reduction(+ : acc)
            for (int32_t k = 0; k < K; ++k)
                acc += (acc_t)oracle_bf16_to_f32(wr[k]) * (acc_t)xr[k];
            out[(size_t)t * N + n] = (float)acc;
        }
    }
}

/* R16: codes of in[i] / scale: round to nearest even in the 8-bit format, magnitudes above 448 become 448;
 * the reciprocal of the scale is formed in double and rounded to fp32, the product is an fp32 product. */
void oracle_quantise(const float* in, int64_t n, float scale, uint8_t* codes)
{
    float inv = (float)(1.0 / (double)scale);
    for (int64_t i = 0; i < n; ++i) codes[i] = oracle_f32_to_e4m3(in[i] * inv);
}

/* R16: out[t, n] = (sum_k value(Wc[n, k]) * value(in_c[t, k])) * (a_scale * s_w[n]); the products of two 8-bit
 * values are exact in fp32, the sum runs in acc_t, the two scales are multiplied in fp32 first. */
void oracle_linear_w8a8(const uint8_t* Wc, const float* s_w, int32_t N, int32_t K,
                        const uint8_t* in_c, float a_scale, int32_t n_rows, float* out)
{
    float lut[256];
    for (int i = 0; i < 256; ++i) lut[i] = oracle_e4m3_to_f32((uint8_t)i);
    /* the values of the input codes, once (a table look-up, no arithmetic) */
    float* xv = (float*)malloc(sizeof(float) * ((size_t)n_rows * K + 1));
    for (size_t i = 0; i < (size_t)n_rows * K; ++i) xv[i] = lut[in_c[i]];
#pragma omp parallel
    {
        float* wv = (float*)malloc(sizeof(float) * ((size_t)K + 1));
#pragma omp for schedule(static)
        for (int32_t n = 0; n < N; ++n) {
            for (int32_t k = 0; k < K; ++k) wv[k] = lut[Wc[(size_t)n * K + k]];
            const float scale = a_scale * s_w[n];
            for (int32_t t = 0; t < n_rows; ++t) {
                const float* xr = xv + (size_t)t * K;
                acc_t acc = 0;
#pragma omp simd reduction(+ : acc)
                for (int32_t k = 0; k < K; ++k)
                    acc += (acc_t)wv[k] * (acc_t)xr[k];
                out[(size_t)t * N + n] = (float)acc * scale;
            }
        }
        free(wv);
    }
    free(xv);
}

/* One projection of the layer: 16-bit weights on fp32 inputs, or (R16) 8-bit codes on quantised inputs. */
static void project(const uint16_t* W, const uint8_t* Wc, const float* s_w, float a_scale,
                    int32_t N, int32_t K, const float* in, int32_t n_rows, float* out)
{
    if (!Wc) {
        oracle_linear(W, N, K, in, n_rows, out);
        return;
    }
    uint8_t* codes = (uint8_t*)malloc((size_t)n_rows * K + 1);
    oracle_quantise(in, (int64_t)n_rows * K, a_scale, codes);
    oracle_linear_w8a8(Wc, s_w, N, K, codes, a_scale, n_rows, out);
    free(codes);
}

/* R3: (v_i, v_{i+d/2}) rotated by angle pos * base^(-2i/d) */
void oracle_rope(float* vec, int32_t d, int32_t pos, float base)
{
    int32_t half = d / 2;
    for (int32_t i = 0; i < half; ++i) {
        double theta = pow((double)base, -2.0 * (double)i / (double)d);
        double ang = (double)pos * theta;
        float c = (float)cos(ang), s = (float)sin(ang);
        float a = vec[i], b = vec[i + half];
        vec[i]        = a * c - b * s;
        vec[i + half] = a * s + b * c;
    }
}

/* R9: where the token at position pos of request r lives */
static int64_t slot_of(const oracle_config* c, const oracle_batch* b, int32_t r, int32_t pos)
{
    int32_t page = b->block_table[(size_t)r * b->max_blocks + pos / c->page_size];
    return (int64_t)page * c->page_size + pos % c->page_size;
}

int32_t oracle_kv_append(const oracle_config* c, const oracle_batch* b,
                         const uint16_t* k, const uint16_t* v,
                         uint16_t* k_pages, uint16_t* v_pages, int32_t num_pages,
                         int32_t* slots_out)
{
    size_t row = (size_t)c->n_kv_heads * c->head_dim;
    for (int32_t r = 0; r < b->num_reqs; ++r) {
        int32_t q_len = b->q_start[r + 1] - b->q_start[r];
        int32_t past = b->ctx_len[r] - q_len;
        for (int32_t j = 0; j < q_len; ++j) {
            int32_t t = b->q_start[r] + j;
            int64_t slot = slot_of(c, b, r, past + j);
            if (slot < 0 || slot >= (int64_t)num_pages * c->page_size) return -1;
            memcpy(k_pages + (size_t)slot * row, k + (size_t)t * row, row * sizeof(uint16_t));
            memcpy(v_pages + (size_t)slot * row, v + (size_t)t * row, row * sizeof(uint16_t));
            if (slots_out) slots_out[t] = (int32_t)slot;
        }
    }
    return 0;
}

/* One cached element: a bf16 value, or (R15) an 8-bit code times the pool's scale */
static float cache_value(const void* pages, size_t idx, int fp8, float scale)
{
    if (fp8) return oracle_e4m3_to_f32(((const uint8_t*)pages)[idx]) * scale;
    return oracle_bf16_to_f32(((const uint16_t*)pages)[idx]);
}

/* Eq. 4, then the weighted value sum of Eq. 5, for every query head of one token */
static void attention_token(const oracle_config* c, const oracle_batch* b,
                            int32_t r, int32_t pos, const float* q,
                            const void* k_pages, const void* v_pages, int fp8, float k_scale, float v_scale,
                            float* out)
{
    int32_t d = c->head_dim, n_kv = c->n_kv_heads;
    int32_t group = c->n_q_heads / n_kv;                       /* R7 */
    float scale = (float)(1.0 / sqrt((double)d));              /* R4 */
    int32_t n_keys = pos + 1;                                  /* R5: j <= i */
    float* s = (float*)malloc((size_t)n_keys * sizeof(float));

    for (int32_t a = 0; a < c->n_q_heads; ++a) {
        int32_t kvh = a / group;
        const float* qa = q + (size_t)a * d;
        float m = -INFINITY;
        for (int32_t j = 0; j < n_keys; ++j) {
            size_t kj = ((size_t)slot_of(c, b, r, j) * n_kv + kvh) * d;
            acc_t dot = 0;
            for (int32_t i = 0; i < d; ++i) dot += (acc_t)qa[i] * (acc_t)cache_value(k_pages, kj + i, fp8, k_scale);
            s[j] = (float)dot * scale;
            if (s[j] > m) m = s[j];
        }
        acc_t denom = 0;
        for (int32_t j = 0; j < n_keys; ++j) {
            s[j] = expf(s[j] - m);          /* same ratio as Eq. 4; the shift only avoids overflow */
            denom += (acc_t)s[j];
        }
        acc_t o[d];
        for (int32_t i = 0; i < d; ++i) o[i] = 0;
        for (int32_t j = 0; j < n_keys; ++j) {
            size_t vj = ((size_t)slot_of(c, b, r, j) * n_kv + kvh) * d;
            for (int32_t i = 0; i < d; ++i) o[i] += (acc_t)s[j] * (acc_t)cache_value(v_pages, vj + i, fp8, v_scale);
        }
        for (int32_t i = 0; i < d; ++i) out[(size_t)a * d + i] = (float)(o[i] / denom);
    }
    free(s);
}

void oracle_attention_token(const oracle_config* c, const oracle_batch* b,
                            int32_t r, int32_t pos, const float* q,
                            const uint16_t* k_pages, const uint16_t* v_pages,
                            float* out)
{
    attention_token(c, b, r, pos, q, k_pages, v_pages, 0, 1.0f, 1.0f, out);
}

void oracle_attention_token_fp8kv(const oracle_config* c, const oracle_batch* b,
                                  int32_t r, int32_t pos, const float* q,
                                  const uint8_t* k_pages, const uint8_t* v_pages, float k_scale, float v_scale,
                                  float* out)
{
    attention_token(c, b, r, pos, q, k_pages, v_pages, 1, k_scale, v_scale, out);
}

/* R15: the step's keys and values as 8-bit codes of x / scale, written to their slots */
static int32_t kv_append_fp8(const oracle_config* c, const oracle_batch* b, const float* qkv, int32_t qkv_dim, int32_t q_dim,
                             uint8_t* k_pages, uint8_t* v_pages, int32_t num_pages, float k_scale, float v_scale)
{
    size_t row = (size_t)c->n_kv_heads * c->head_dim;
    float k_inv = (float)(1.0 / (double)k_scale), v_inv = (float)(1.0 / (double)v_scale);
    for (int32_t r = 0; r < b->num_reqs; ++r) {
        int32_t q_len = b->q_start[r + 1] - b->q_start[r];
        int32_t past = b->ctx_len[r] - q_len;
        for (int32_t j = 0; j < q_len; ++j) {
            const float* src = qkv + (size_t)(b->q_start[r] + j) * qkv_dim + q_dim;
            int64_t slot = slot_of(c, b, r, past + j);
            if (slot < 0 || slot >= (int64_t)num_pages * c->page_size) return -1;
            for (size_t i = 0; i < row; ++i) {
                k_pages[(size_t)slot * row + i] = oracle_f32_to_e4m3(src[i] * k_inv);
                v_pages[(size_t)slot * row + i] = oracle_f32_to_e4m3(src[row + i] * v_inv);
            }
        }
    }
    return 0;
}

static int32_t layer_step(const oracle_config* c, const oracle_batch* b,
                          const oracle_weights* w, const uint16_t* x,
                          void* k_pages, void* v_pages, int32_t num_pages, int fp8, float k_scale, float v_scale,
                          const oracle_weights_w8a8* q8,
                          const int32_t* rows, int32_t n_rows,
                          float* y_f32, uint16_t* y_bf16,
                          float* tap_attn_out, float* tap_x1)
{
    const int32_t H = c->hidden, d = c->head_dim, n_h = c->n_q_heads, n_kv = c->n_kv_heads;
    const int32_t I = c->mlp_dim, P = c->page_size;
    const int32_t q_dim = n_h * d, kv_dim = n_kv * d, qkv_dim = q_dim + 2 * kv_dim;
    if (H <= 0 || d <= 0 || (d & 1) || n_kv <= 0 || n_h % n_kv || I <= 0 || P <= 0) return -2;
    if (b->num_reqs < 0 || b->q_start[0] != 0) return -3;
    const int32_t T = b->q_start[b->num_reqs];

    /* token -> (request, position in its own sequence) */
    int32_t* tok_req = (int32_t*)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
    int32_t* tok_pos = (int32_t*)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
    for (int32_t r = 0; r < b->num_reqs; ++r) {
        int32_t q_len = b->q_start[r + 1] - b->q_start[r];
        int32_t past = b->ctx_len[r] - q_len;
        if (q_len < 0 || past < 0 || (b->ctx_len[r] + P - 1) / P > b->max_blocks) {
            free(tok_req); free(tok_pos);
            return -3;
        }
        for (int32_t j = 0; j < q_len; ++j) {
            tok_req[b->q_start[r] + j] = r;
            tok_pos[b->q_start[r] + j] = past + j;
        }
    }
    if (T == 0) { free(tok_req); free(tok_pos); return 0; }

    /* widen x */
    float* xf = (float*)calloc((size_t)T * H, sizeof(float));
    for (size_t i = 0; i < (size_t)T * H; ++i) xf[i] = oracle_bf16_to_f32(x[i]);

    /* 1. input norm (R2), 2. q/k/v (Eq. 3) for every token of the batch */
    float* h = (float*)malloc(sizeof(float) * (size_t)T * H);
    oracle_rmsnorm(xf, w->w_in_norm, c->rms_eps, T, H, h);
    if (fp8 && !q8)    /* R15: the quantisation decision is taken in the kernel's precision: bf16 inputs, fp32 sums */
        for (size_t i = 0; i < (size_t)T * H; ++i) h[i] = oracle_bf16_to_f32(oracle_f32_to_bf16(h[i]));
    float* qkv = (float*)malloc(sizeof(float) * (size_t)T * qkv_dim);
    project(w->w_qkv, q8 ? q8->w_qkv : NULL, q8 ? q8->s_qkv : NULL, q8 ? q8->a_qkv : 0.0f, qkv_dim, H, h, T, qkv);
    free(h);

    /* 3. rotary embedding on q and k (R3), 4. round k, v to bf16 and append (R5, R9) */
    uint16_t* kb = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)T * kv_dim);
    uint16_t* vb = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)T * kv_dim);
    for (int32_t t = 0; t < T; ++t) {
        float* row = qkv + (size_t)t * qkv_dim;
        for (int32_t a = 0; a < n_h; ++a) oracle_rope(row + (size_t)a * d, d, tok_pos[t], c->rope_base);
        for (int32_t g = 0; g < n_kv; ++g) oracle_rope(row + q_dim + (size_t)g * d, d, tok_pos[t], c->rope_base);
        for (int32_t i = 0; i < kv_dim; ++i) {
            kb[(size_t)t * kv_dim + i] = oracle_f32_to_bf16(row[q_dim + i]);
            vb[(size_t)t * kv_dim + i] = oracle_f32_to_bf16(row[q_dim + kv_dim + i]);
        }
    }
    int32_t rc = fp8 ? kv_append_fp8(c, b, qkv, qkv_dim, q_dim, (uint8_t*)k_pages, (uint8_t*)v_pages, num_pages, k_scale, v_scale)
                     : oracle_kv_append(c, b, kb, vb, (uint16_t*)k_pages, (uint16_t*)v_pages, num_pages, NULL);
    free(kb); free(vb);
    if (rc) { free(tok_req); free(tok_pos); free(xf); free(qkv); return -4; }

    /* the rows that get the rest of the layer */
    int32_t n_out = (rows && n_rows > 0) ? n_rows : T;
    int32_t* sel = (int32_t*)malloc(sizeof(int32_t) * (size_t)n_out);
    for (int32_t i = 0; i < n_out; ++i) {
        sel[i] = (rows && n_rows > 0) ? rows[i] : i;
        if (sel[i] < 0 || sel[i] >= T) {
            free(tok_req); free(tok_pos); free(xf); free(qkv); free(sel);
            return -5;
        }
    }

    /* 5. attention over the cache (Eq. 4, Eq. 5 without W_o) */
    float* attn = (float*)malloc(sizeof(float) * (size_t)n_out * q_dim);
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t i = 0; i < n_out; ++i) {
        int32_t t = sel[i];
        attention_token(c, b, tok_req[t], tok_pos[t], qkv + (size_t)t * qkv_dim,
                        k_pages, v_pages, fp8, k_scale, v_scale, attn + (size_t)i * q_dim);
    }
    free(qkv);
    if (tap_attn_out) memcpy(tap_attn_out, attn, sizeof(float) * (size_t)n_out * q_dim);

    /* 6. W_o (Eq. 5) and the residual (R1) */
    float* x1 = (float*)malloc(sizeof(float) * (size_t)n_out * H);
    if (q8)     /* R16: the attention output exists as bf16 before it is quantised */
        for (size_t i = 0; i < (size_t)n_out * q_dim; ++i) attn[i] = oracle_bf16_to_f32(oracle_f32_to_bf16(attn[i]));
    project(w->w_o, q8 ? q8->w_o : NULL, q8 ? q8->s_o : NULL, q8 ? q8->a_o : 0.0f, H, q_dim, attn, n_out, x1);
    free(attn);
    for (int32_t i = 0; i < n_out; ++i)
        for (int32_t j = 0; j < H; ++j)
            x1[(size_t)i * H + j] += xf[(size_t)sel[i] * H + j];
    free(xf);
    if (tap_x1) memcpy(tap_x1, x1, sizeof(float) * (size_t)n_out * H);

    /* 7. post norm, gate/up, silu(g) * u, down, residual (R1) */
    float* h2 = (float*)malloc(sizeof(float) * (size_t)n_out * H);
    oracle_rmsnorm(x1, w->w_post_norm, c->rms_eps, n_out, H, h2);
    float* gu = (float*)malloc(sizeof(float) * (size_t)n_out * 2 * I);
    project(w->w_gate_up, q8 ? q8->w_gate_up : NULL, q8 ? q8->s_gate_up : NULL, q8 ? q8->a_gate_up : 0.0f, 2 * I, H, h2, n_out, gu);
    free(h2);
    float* act = (float*)malloc(sizeof(float) * (size_t)n_out * I);
    for (int32_t i = 0; i < n_out; ++i)
        for (int32_t j = 0; j < I; ++j) {
            float g = gu[(size_t)i * 2 * I + j], u = gu[(size_t)i * 2 * I + I + j];
            act[(size_t)i * I + j] = g / (1.0f + expf(-g)) * u;
        }
    free(gu);
    float* mlp = (float*)malloc(sizeof(float) * (size_t)n_out * H);
    project(w->w_down, q8 ? q8->w_down : NULL, q8 ? q8->s_down : NULL, q8 ? q8->a_down : 0.0f, H, I, act, n_out, mlp);
    free(act);

    /* 8. y = x1 + mlp, fp32 and (optionally) rounded to bf16 */
    for (size_t i = 0; i < (size_t)n_out * H; ++i) {
        float y = x1[i] + mlp[i];
        y_f32[i] = y;
        if (y_bf16) y_bf16[i] = oracle_f32_to_bf16(y);
    }
    free(mlp); free(x1); free(sel); free(tok_req); free(tok_pos);
    return 0;
}

int32_t oracle_layer_step(const oracle_config* c, const oracle_batch* b,
                          const oracle_weights* w, const uint16_t* x,
                          uint16_t* k_pages, uint16_t* v_pages, int32_t num_pages,
                          const int32_t* rows, int32_t n_rows,
                          float* y_f32, uint16_t* y_bf16,
                          float* tap_attn_out, float* tap_x1)
{
    return layer_step(c, b, w, x, k_pages, v_pages, num_pages, 0, 1.0f, 1.0f, NULL, rows, n_rows, y_f32, y_bf16, tap_attn_out, tap_x1);
}

int32_t oracle_layer_step_fp8kv(const oracle_config* c, const oracle_batch* b,
                                const oracle_weights* w, const uint16_t* x,
                                uint8_t* k_pages, uint8_t* v_pages, int32_t num_pages, float k_scale, float v_scale,
                                const int32_t* rows, int32_t n_rows,
                                float* y_f32, uint16_t* y_bf16,
                                float* tap_attn_out, float* tap_x1)
{
    if (!(k_scale > 0.0f) || !(v_scale > 0.0f)) return -7;
    return layer_step(c, b, w, x, k_pages, v_pages, num_pages, 1, k_scale, v_scale, NULL, rows, n_rows, y_f32, y_bf16, tap_attn_out, tap_x1);
}

int32_t oracle_layer_step_w8a8(const oracle_config* c, const oracle_batch* b,
                               const oracle_weights_w8a8* q8, const uint16_t* x,
                               void* k_pages, void* v_pages, int32_t num_pages, int32_t kv_fp8, float k_scale, float v_scale,
                               const int32_t* rows, int32_t n_rows,
                               float* y_f32, uint16_t* y_bf16,
                               float* tap_attn_out, float* tap_x1)
{
    if (!(q8->a_qkv > 0.0f) || !(q8->a_o > 0.0f) || !(q8->a_gate_up > 0.0f) || !(q8->a_down > 0.0f)) return -7;
    if (kv_fp8 && (!(k_scale > 0.0f) || !(v_scale > 0.0f))) return -7;
    oracle_weights w = {q8->w_in_norm, NULL, NULL, q8->w_post_norm, NULL, NULL};
    return layer_step(c, b, &w, x, k_pages, v_pages, num_pages, kv_fp8 ? 1 : 0, kv_fp8 ? k_scale : 1.0f, kv_fp8 ? v_scale : 1.0f,
                      q8, rows, n_rows, y_f32, y_bf16, tap_attn_out, tap_x1);
}

/* Embedding -> n_layers x layer step -> final norm -> output layer on each request's last token */
static int32_t model_step(const oracle_config* c, const oracle_model* m, const oracle_weights_w8a8* q8, const oracle_batch* b,
                          const int32_t* token_ids, uint16_t* const* k_pages, uint16_t* const* v_pages,
                          int32_t num_pages, float* logits, uint16_t* hidden_out)
{
    const int32_t H = c->hidden, T = b->q_start[b->num_reqs];
    if (T == 0) return 0;
    uint16_t* x = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)T * H);
    float* y = (float*)malloc(sizeof(float) * (size_t)T * H);
    for (int32_t t = 0; t < T; ++t) {
        if (token_ids[t] < 0 || token_ids[t] >= m->vocab) { free(x); free(y); return -6; }
        memcpy(x + (size_t)t * H, m->embedding + (size_t)token_ids[t] * H, sizeof(uint16_t) * (size_t)H);
    }
    for (int32_t l = 0; l < m->n_layers; ++l) {      /* R11: x <- bf16(layer(x)) */
        int32_t rc = q8 ? oracle_layer_step_w8a8(c, b, &q8[l], x, (void*)k_pages[l], (void*)v_pages[l], num_pages, 0, 1.0f, 1.0f,
                                                 NULL, 0, y, /* rounded stream */ x, NULL, NULL)
                        : oracle_layer_step(c, b, &m->layers[l], x, k_pages[l], v_pages[l], num_pages,
                                       NULL, 0, y, x, NULL, NULL);
        if (rc) { free(x); free(y); return rc; }
    }
    if (hidden_out) memcpy(hidden_out, x, sizeof(uint16_t) * (size_t)T * H);
    /* R13: the last query token of every request; R12: final norm, then the output layer */
    float* last = (float*)malloc(sizeof(float) * (size_t)b->num_reqs * H);
    float* normed = (float*)malloc(sizeof(float) * (size_t)b->num_reqs * H);
    for (int32_t r = 0; r < b->num_reqs; ++r)
        for (int32_t i = 0; i < H; ++i)
            last[(size_t)r * H + i] = oracle_bf16_to_f32(x[(size_t)(b->q_start[r + 1] - 1) * H + i]);
    oracle_rmsnorm(last, m->w_final_norm, c->rms_eps, b->num_reqs, H, normed);
    oracle_linear(m->w_lm_head, m->vocab, H, normed, b->num_reqs, logits);
    free(last); free(normed); free(x); free(y);
    return 0;
}

int32_t oracle_model_step(const oracle_config* c, const oracle_model* m, const oracle_batch* b,
                          const int32_t* token_ids, uint16_t* const* k_pages, uint16_t* const* v_pages,
                          int32_t num_pages, float* logits, uint16_t* hidden_out)
{
    return model_step(c, m, NULL, b, token_ids, k_pages, v_pages, num_pages, logits, hidden_out);
}

/* The stack with quantised projections (R16) in every layer; embedding, final norm and output layer stay 16-bit. */
int32_t oracle_model_step_w8a8(const oracle_config* c, const oracle_model* m, const oracle_weights_w8a8* layers,
                               const oracle_batch* b, const int32_t* token_ids,
                               uint16_t* const* k_pages, uint16_t* const* v_pages,
                               int32_t num_pages, float* logits, uint16_t* hidden_out)
{
    if (!layers) return -2;
    return model_step(c, m, layers, b, token_ids, k_pages, v_pages, num_pages, logits, hidden_out);
}

/* Greedy decoding: the next token of a request is the vocabulary entry with the largest logit.
 * Reading R14: among equal largest logits the lowest token id wins; NaN logits never win
 * (a row of only NaN gives token 0). */
void oracle_greedy_sample(const float* logits, int32_t n_rows, int32_t vocab, int32_t* next_token)
{
    for (int32_t r = 0; r < n_rows; ++r) {
        const float* row = logits + (size_t)r * vocab;
        int32_t best = 0;
        int have = 0;
        for (int32_t v = 0; v < vocab; ++v) {
            if (row[v] != row[v]) continue;
            if (!have || row[v] > row[best]) { best = v; have = 1; }
        }
        next_token[r] = best;
    }
}

