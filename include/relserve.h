/*
 * relserve.h -- C ABI of the MI355X (gfx950) layer-step library.
 *
 * What it runs: the GPU worker's share of one serving iteration (Sec. 4.1,
 * step 4 "Batch Processing": the scheduler hands over a batch together with
 * its KV-cache allocation; the worker runs the forward computation and keeps
 * the per-layer KV cache) for ONE decoder layer: input RMSNorm, q/k/v
 * projections (Sec. 2.3, Eq. 3), rotary embedding, KV append into a paged
 * cache (Sec. 2.3 "KV Cache"), causal softmax attention over the cached keys
 * and values (Eq. 4-5) for prefill rows (several query tokens) and decode rows
 * (one query token) of the same batch, with a template prefix shared by the
 * requests of one relQuery (Sec. 2.2 Def. 2.1, Sec. 2.3 "Prefix Cache") stored
 * once and read once per group, W_o + residual, post RMSNorm and SwiGLU MLP +
 * residual.
 *
 * Conventions
 *   - every function returns 0 (RELSERVE_OK) or a negative relserve_status;
 *     nothing throws or aborts; a failed call launches nothing.
 *   - "host" pointers are read during the call and not kept; "device" pointers
 *     are HIP device memory owned by the caller and must stay valid until the
 *     stream work that uses them has finished.
 *   - the library owns only the opaque handles it returns (and the device
 *     copy of the batch descriptor inside a relserve_batch).
 *   - stream arguments are hipStream_t passed as void*; all GPU work is
 *     enqueued there asynchronously, no call synchronises except
 *     relserve_batch_prepare (one blocking descriptor upload) and the
 *     relserve_profile_* readers.
 *   - a call that enqueues GPU work first discards the error, if any, that an
 *     earlier HIP call of the calling thread left pending in the runtime, so that
 *     RELSERVE_ERR_HIP always refers to this call's own launches.
 *   - all 16-bit floating point data are bfloat16, all matrices row-major.
 *   - layouts: activations [T, features]; weights [out_features, in_features];
 *     w_qkv rows = [q heads | k heads | v heads]; w_gate_up rows = [gate | up];
 *     cache pools k_pages / v_pages = [num_pages, page_size, n_kv_heads,
 *     head_dim]; the token at position pos of request r lives in
 *     slot = block_table[r][pos / page_size] * page_size + pos % page_size.
 */
#ifndef RELSERVE_H
#define RELSERVE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RELSERVE_OK = 0,
    RELSERVE_ERR_NULL_POINTER = -1,
    RELSERVE_ERR_BAD_CONFIG = -2,         /* shape the kernels do not cover */
    RELSERVE_ERR_BAD_Q_START = -3,        /* q_start[0] != 0, not increasing, or an empty request */
    RELSERVE_ERR_BAD_CTX_LEN = -4,        /* ctx_len[r] < number of query tokens of r */
    RELSERVE_ERR_BLOCK_TABLE_SHORT = -5,  /* ceil(ctx_len[r] / page_size) > max_blocks */
    RELSERVE_ERR_PAGE_RANGE = -6,         /* a used block-table entry is outside [0, num_pages) */
    RELSERVE_ERR_BAD_PREFIX = -7,         /* prefix id/length inconsistent with the block tables */
    RELSERVE_ERR_SLOT_ALIAS = -8,         /* two query tokens of the batch would write the same slot */
    RELSERVE_ERR_WORKSPACE = -9,          /* workspace missing, misaligned or too small */
    RELSERVE_ERR_HIP = -10,               /* a HIP runtime call failed */
    RELSERVE_ERR_NO_DEVICE = -11,         /* no gfx950 device is current */
    RELSERVE_ERR_TOO_LARGE = -12,         /* a size overflows the 32-bit indices used on the device, or the fixed scratch */
    RELSERVE_ERR_MISMATCH = -13,          /* batch prepared for another layer shape, or cache smaller than the batch's */
    RELSERVE_ERR_BAD_ARGUMENT = -14
} relserve_status;

typedef struct relserve_layer relserve_layer;   /* opaque: one layer shape */
typedef struct relserve_batch relserve_batch;   /* opaque: one prepared batch */

/* Layer shape.  Supported: head_dim in {64, 128}; n_q_heads a multiple of
 * n_kv_heads with ratio <= 16; hidden, mlp_dim multiples of 8; page_size a
 * power of two in [8, 256]. */
typedef struct {
    int32_t hidden;       /* H */
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t head_dim;     /* d of Eq. 4 */
    int32_t mlp_dim;      /* I */
    int32_t page_size;    /* P, tokens per cache page */
    float   rms_eps;
    float   rope_base;
} relserve_layer_config;

/* Batch descriptor; every pointer is HOST memory.
 * Request r owns packed rows q_start[r] .. q_start[r+1]-1 of the activation
 * matrices; its query token j sits at sequence position ctx_len[r] - q_len + j,
 * and ctx_len[r] is the request's length AFTER this step's append.
 * prefix_id[r] (or -1; the array may be NULL) names a template prefix of
 * prefix_len[prefix_id[r]] tokens (a multiple of page_size, not longer than the
 * request's past) whose pages are the leading block-table entries of every
 * member.  It is a hint that lets members' prefix attention be computed
 * together; results are defined by the block tables alone. */
typedef struct {
    int32_t        num_reqs;
    int32_t        max_blocks;     /* row stride of block_table */
    const int32_t* q_start;        /* [num_reqs + 1] */
    const int32_t* ctx_len;        /* [num_reqs] */
    const int32_t* block_table;    /* [num_reqs, max_blocks] */
    const int32_t* prefix_id;      /* [num_reqs] or NULL */
    int32_t        num_prefixes;
    const int32_t* prefix_len;     /* [num_prefixes] */
    int32_t        num_pages;      /* pages in the cache pools the batch addresses */
} relserve_batch_desc;

/* Cache pools.  dtype RELSERVE_KV_BF16: 16-bit pools as described at the top.  dtype RELSERVE_KV_FP8: a
 * variant with half the bytes per cached token (the paper runs 16-bit caches; decode attention is bound by
 * exactly these bytes, Sec. 2.3 "Prefill and Decode Phases"): the pools hold one byte per element, an 8-bit
 * floating point code (1 sign, 4 exponent, 3 mantissa bits, bias 7, largest magnitude 448, no infinity) of
 * x / scale, with one positive scale per pool given by the caller.  The step's rotated keys and its values are
 * quantised once from their fp32 values: round to nearest even of x * (1 / scale), magnitudes above 448 become
 * 448 (the code of a NaN input is unspecified); attention reads value(code) * scale.  Served by
 * relserve_layer_step(_static), relserve_model_step, relserve_qkv_rope_append and relserve_attention; the
 * stand-alone relserve_kv_append / relserve_rope_append take 16-bit pools only. */
enum { RELSERVE_KV_BF16 = 0, RELSERVE_KV_FP8 = 1 };
typedef struct {
    void*   k_pages;     /* device, [num_pages, P, n_kv, d] bf16 (or 8-bit codes) */
    void*   v_pages;     /* device, same shape */
    int32_t num_pages;
    int32_t dtype;       /* RELSERVE_KV_BF16 or RELSERVE_KV_FP8 */
    float   k_scale;     /* RELSERVE_KV_FP8 only: > 0 */
    float   v_scale;
} relserve_kv_cache;

typedef struct {          /* all device, bf16 */
    const void* w_in_norm;     /* [H] */
    const void* w_qkv;         /* [(n_q + 2 n_kv) d, H] */
    const void* w_o;           /* [H, n_q d] */
    const void* w_post_norm;   /* [H] */
    const void* w_gate_up;     /* [2 I, H] */
    const void* w_down;        /* [H, I] */
    int32_t packed;            /* 0: the four matrices are row-major [out, in]; 1: each was converted with
                                * relserve_pack_weight (needs hidden, n_q d and I to be multiples of 64) */
} relserve_layer_weights;

typedef struct {
    int32_t num_tokens;        /* T */
    int32_t num_reqs;
    int32_t num_decode_rows;   /* requests with one query token */
    int32_t num_prefill_rows;
    int32_t num_prefix_groups; /* groups whose prefix attention is computed jointly */
    int32_t num_attn_items;    /* workgroup-level work items of the attention kernels */
} relserve_batch_info;

int32_t     relserve_version(void);
const char* relserve_strerror(int32_t status);

/* Checks a layer shape.  Host only. */
int32_t relserve_config_validate(const relserve_layer_config* cfg);

/* Creates / destroys a layer-shape handle.  Host only, touches no device. */
int32_t relserve_layer_create(const relserve_layer_config* cfg, relserve_layer** out);
int32_t relserve_layer_destroy(relserve_layer* layer);

/* Checks a descriptor against a layer shape: every rule named beside the
 * relserve_status codes.  Host only, no device needed. */
int32_t relserve_batch_validate(const relserve_layer_config* cfg, const relserve_batch_desc* desc);

/* Host-only: the cache slot every query token of the batch is appended to
 * (slots_out: host, [T]).  The placement contract, checkable without a GPU. */
int32_t relserve_batch_slots(const relserve_layer_config* cfg, const relserve_batch_desc* desc,
                             int32_t* slots_out);

/* Validates, expands the descriptor into per-token tables (request, position,
 * slot, rotary cos/sin), builds the attention work lists and uploads them.
 * One prepared batch serves every layer of the model step.  Blocks until the
 * upload has finished. */
int32_t relserve_batch_prepare(const relserve_layer* layer, const relserve_batch_desc* desc,
                               void* stream, relserve_batch** out);
int32_t relserve_batch_destroy(relserve_batch* batch);
int32_t relserve_batch_get_info(const relserve_batch* batch, relserve_batch_info* out);

/* Bytes of device workspace relserve_layer_step needs for up to max_tokens
 * packed query tokens. */
int32_t relserve_workspace_bytes(const relserve_layer* layer, int32_t max_tokens, size_t* out);

/* KV append alone (Sec. 2.3 "KV Cache"): k, v are device [T, n_kv, d] bf16,
 * rotary embedding already applied by the caller; rows are copied bit for bit
 * into their slots; no other byte of the pools is written. */
int32_t relserve_kv_append(const relserve_layer* layer, const relserve_batch* batch,
                           const void* k, const void* v, relserve_kv_cache cache, void* stream);

/* The whole layer step (Eq. 3-5 and the wiring listed at the top).  x, y:
 * device [T, H] bf16; y may alias x.  workspace: device, 256-byte aligned,
 * at least relserve_workspace_bytes(layer, T); pure scratch: its contents on
 * entry do not matter and nothing is kept in it between calls, so calls that
 * may overlap (other streams) need workspaces of their own.  The cache pools
 * are updated in place at the batch's slots and nowhere else. */
int32_t relserve_layer_step(const relserve_layer* layer, const relserve_batch* batch,
                            const relserve_layer_weights* weights,
                            const void* x, void* y, relserve_kv_cache cache,
                            void* workspace, size_t workspace_bytes, void* stream);

/* relserve_layer_step for callers that cannot allocate or carry a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same results bit for bit;
 * the workspace is a fixed array of RELSERVE_STATIC_SCRATCH_BYTES in device memory that belongs to the
 * library (one copy per GPU it runs on, held until the process ends).  The call allocates nothing and frees
 * nothing.  A batch whose relserve_workspace_bytes exceeds the array (the 13B shape up to 256 query
 * tokens, the 70B shape up to 128) is refused with RELSERVE_ERR_TOO_LARGE and nothing is launched.  Every
 * call on a GPU uses that GPU's one array: calls that may overlap on one GPU (two streams, two threads)
 * race; the array is pure scratch (written before it is read), so nothing has to be cleared between
 * calls.  relserve_static_scratch_bytes reports the size. */
#define RELSERVE_STATIC_SCRATCH_BYTES (80u << 20)
int32_t relserve_static_scratch_bytes(size_t* out);
int32_t relserve_layer_step_static(const relserve_layer* layer, const relserve_batch* batch,
                                   const relserve_layer_weights* weights,
                                   const void* x, void* y, relserve_kv_cache cache, void* stream);

/* The layer step with quantised projections (a variant beside the paper's 16-bit models, Sec. 5.1
 * "Models"; the four dense maps are Eq. 3, W_o of Eq. 5 and the two of the feed-forward block).
 * Each projection matrix holds 8-bit floating point codes (1 sign, 4 exponent, 3 mantissa bits, bias 7,
 * largest magnitude 448) of W[n, :] / s[n] with one fp32 scale per output row; the input of each projection is
 * quantised with one scale per projection, given by the caller (static, as an engine calibrates it offline):
 * code = round-to-nearest-even(a * (1 / a_scale)), magnitudes above 448 become 448.  A projection is
 * out[t, n] = (sum_k value(a_code[t, k]) * value(w_code[n, k])) * (a_scale * s[n]), products exact, fp32 sums.
 * What is quantised: the normed activations (from fp32), the attention output (after its rounding to bf16),
 * silu(g) * u (from fp32).  Norms, rotary embedding, attention, residuals and the cache are those of
 * relserve_layer_step; the cache may be 16-bit or quantised.
 * Pointers are device memory.  w_*: uint8 [out, in] row-major, or (packed != 0) relserve_pack_weight applied to
 * the matrix seen as [out, in / 2] two-byte units.  s_*: fp32 [out].  hidden, n_q_heads * head_dim and mlp_dim
 * must be multiples of 128 (RELSERVE_ERR_BAD_ARGUMENT otherwise); scales must be positive and finite. */
typedef struct {
    const void* w_in_norm;     /* [H] bf16 */
    const void* w_qkv;         /* [(n_q + 2 n_kv) d, H] codes */
    const float* s_qkv;        /* [(n_q + 2 n_kv) d] */
    const void* w_o;           /* [H, n_q d] */
    const float* s_o;          /* [H] */
    const void* w_post_norm;   /* [H] bf16 */
    const void* w_gate_up;     /* [2 I, H], gate rows then up rows */
    const float* s_gate_up;    /* [2 I] */
    const void* w_down;        /* [H, I] */
    const float* s_down;       /* [H] */
    float a_qkv, a_o, a_gate_up, a_down;   /* scale of each projection's input */
    int32_t packed;
} relserve_layer_weights_w8a8;

/* Arguments, workspace (relserve_workspace_bytes), ownership and errors as relserve_layer_step. */
int32_t relserve_layer_step_w8a8(const relserve_layer* layer, const relserve_batch* batch,
                                 const relserve_layer_weights_w8a8* weights,
                                 const void* x, void* y, relserve_kv_cache cache,
                                 void* workspace, size_t workspace_bytes, void* stream);

/* A stack of n_layers identical-shape layers between an embedding table and an
 * output layer (Sec. 2.3 "LLM Inference": the output layer turns the final
 * hidden representation of a request's LAST token into next-token logits).
 * `layers` and `caches` are HOST arrays of n_layers entries holding device
 * pointers; the other pointers are device bf16.  vocab must be a multiple of 4. */
typedef struct {
    int32_t n_layers;
    int32_t vocab;
    const void* embedding;                  /* [vocab, H] */
    const relserve_layer_weights* layers;   /* host array [n_layers] */
    const relserve_kv_cache* caches;        /* host array [n_layers], one pool pair per layer */
    const void* w_final_norm;               /* [H] */
    const void* w_lm_head;                  /* [vocab, H] */
} relserve_model;

/* Workspace of relserve_model_step: one layer's workspace plus the residual
 * stream [T, H] and the gathered last rows [num_reqs, H]. */
int32_t relserve_model_workspace_bytes(const relserve_layer* layer, int32_t max_tokens, int32_t max_reqs,
                                       size_t* out);

/* One model step over a prepared batch: x = embedding[token_ids] (ids outside
 * [0, vocab) are clamped, never dereferenced out of range), n_layers layer
 * steps with the stream rounded to bf16 between layers, final RMSNorm and the
 * output layer on the last query token of every request.  token_ids: device
 * int32 [T]; logits: device fp32 [num_reqs, vocab]. */
int32_t relserve_model_step(const relserve_layer* layer, const relserve_batch* batch,
                            const relserve_model* model, const int32_t* token_ids, void* logits,
                            void* workspace, size_t workspace_bytes, void* stream);

/* relserve_model_step with the quantised projections of relserve_layer_step_w8a8 in every layer: `layers` is a HOST
 * array of model->n_layers entries (model->layers is not read); the embedding table, the final norm and the output
 * layer are the 16-bit ones of `model`; caches as in relserve_model_step.  Workspace: relserve_model_workspace_bytes. */
int32_t relserve_model_step_w8a8(const relserve_layer* layer, const relserve_batch* batch,
                                 const relserve_model* model, const relserve_layer_weights_w8a8* layers,
                                 const int32_t* token_ids, void* logits,
                                 void* workspace, size_t workspace_bytes, void* stream);

/* Greedy decoding after the output layer (Sec. 2.3 "LLM Inference": the output layer's result for a
 * request's last token determines its next token): next_token[r] = the vocabulary entry with the largest
 * logit of row r, the lowest id among equal largest ones; NaN entries never win, a row without any number
 * gives 0.  logits: device fp32 [n_rows, vocab] (what relserve_model_step writes); next_token: device
 * int32 [n_rows].  Integer result, defined exactly. */
int32_t relserve_greedy_sample(const void* logits, int32_t n_rows, int32_t vocab, int32_t* next_token, void* stream);

/* ---- single stages, exported so that each kernel can be checked alone ---- */

/* out[t, :] = x[t, :] * w / sqrt(mean(x[t, :]^2) + eps); x is bf16 when
 * x_is_f32 == 0, else fp32; out bf16. */
int32_t relserve_rmsnorm(const void* x, int32_t x_is_f32, const void* w, float eps,
                         int32_t n_rows, int32_t hidden, void* out, void* stream);

/* Stages of the quantised-projection variant.  relserve_rmsnorm_codes: relserve_rmsnorm whose output is uint8
 * codes of the normed value / scale (taken from the fp32 value).  relserve_quantise_bf16: codes [n] of a bf16
 * array / scale (n a multiple of 8).  relserve_linear_w8a8: relserve_linear on codes a [T, K], w [N, K] (row-major,
 * or packed as described at relserve_layer_weights_w8a8) with row scales w_scale [N] and input scale a_scale;
 * K a multiple of 128; epilogues as relserve_linear (the residuals and 16-bit outputs unchanged); out_scale > 0
 * with epilogue 3 stores uint8 codes of silu(g) * u / out_scale instead of bf16. */
int32_t relserve_rmsnorm_codes(const void* x, int32_t x_is_f32, const void* w, float eps,
                               int32_t n_rows, int32_t hidden, float scale, void* out, void* stream);
int32_t relserve_quantise_bf16(const void* in, int64_t n, float scale, void* codes, void* stream);
int32_t relserve_linear_w8a8(const void* a, const void* w, const float* w_scale, float a_scale,
                             int32_t T, int32_t N, int32_t K, int32_t epilogue, const void* residual, void* out,
                             float out_scale, int32_t packed, void* stream);

/* out[T, N] = a[T, K] * w[N, K]^T (Eq. 3 and every other dense map), bf16 in,
 * fp32 accumulate.  epilogue: 0 = store bf16; 1 = add residual (bf16 [T, N],
 * or none when NULL) and store fp32; 2 = add residual (fp32 [T, N]) and store bf16; 3 = SwiGLU:
 * w holds [gate | up] rows (N = 2 * n_half), out[T, n_half] = silu(g) * u bf16.
 * K must be a multiple of 8, N of 4 (of 16 for SwiGLU). */
int32_t relserve_linear(const void* a, const void* w, int32_t T, int32_t N, int32_t K,
                        int32_t epilogue, const void* residual, void* out, void* stream);

/* Tiled weight layout for streaming.  A row-major matrix w [N, K] (K a multiple of 64) becomes
 * out[N / 256][K / 64][N % 256][K % 64] with N padded to a multiple of 256 (zero rows): one 64-wide k
 * slice of 256 output features is 32 KB of consecutive memory, which is what one pipeline stage of the
 * GEMM kernels reads; with row-major weights the same stage is 256 pieces of 128 bytes 2 K bytes apart,
 * and the weight-bound (small T) projections reach only about half of the streaming rate.
 * relserve_packed_weight_elems: bf16 elements of the packed matrix.  relserve_pack_weight: device to
 * device, out must not overlap w.  relserve_linear_packed: relserve_linear on a packed w. */
int32_t relserve_packed_weight_elems(int32_t N, int32_t K, int64_t* out);
int32_t relserve_pack_weight(const void* w, int32_t N, int32_t K, void* out, void* stream);
int32_t relserve_linear_packed(const void* a, const void* w_packed, int32_t T, int32_t N, int32_t K,
                               int32_t epilogue, const void* residual, void* out, void* stream);

/* Rotary embedding of q and k inside qkv [T, (n_q + 2 n_kv) d] (in place on the
 * q part) and append of the rotated k and of v into the cache. */
int32_t relserve_rope_append(const relserve_layer* layer, const relserve_batch* batch,
                             void* qkv, relserve_kv_cache cache, void* stream);

/* q/k/v projection (Eq. 3) of normed activations h [T, H] with the rotary embedding
 * and the KV append fused into the GEMM epilogue: rotated q -> q_out [T, n_q d]
 * bf16, rotated k and v -> their cache slots; each value is rounded to bf16 once. */
int32_t relserve_qkv_rope_append(const relserve_layer* layer, const relserve_batch* batch,
                                 const void* h, const void* w_qkv, void* q_out,
                                 relserve_kv_cache cache, void* stream);

/* Attention of every query token over its request's cached keys/values
 * (Eq. 4, Eq. 5 before W_o).  q: device rows of pitch q_pitch elements holding
 * [n_q, d] rotated queries; out [T, n_q d] bf16.  workspace as for the step. */
int32_t relserve_attention(const relserve_layer* layer, const relserve_batch* batch,
                           const void* q, int32_t q_pitch, relserve_kv_cache cache,
                           void* out, void* workspace, size_t workspace_bytes, void* stream);

/* ---- batch-duration model (Sec. 4.2, Eq. 9) ----
 * The scheduler predicts the duration of a prefill batch p as alpha_p * utok(p) + beta_p (utok = query
 * tokens the batch really computes, i.e. not served by the prefix cache) and of a decode batch d as
 * alpha_d * req(d) + beta_d (req = its requests); the coefficients come from fitting durations measured
 * offline.  relserve_duration_fit is that fit (ordinary least squares): units[i] = size measure of run
 * i, seconds[i] = its measured duration, both HOST arrays of n >= 2 finite values that are read only;
 * *out receives slope, intercept, the coefficient of determination r2 = 1 - SS_res / SS_tot (1 when all
 * durations are equal and fitted exactly) and n.  RELSERVE_ERR_BAD_ARGUMENT: n < 2, a non-finite value,
 * or all units equal.  relserve_duration_predict evaluates Eq. 9 for one batch.  Host only; no device
 * work, no allocation. */
typedef struct relserve_duration_model {
    double  alpha;   /* seconds per unit */
    double  beta;    /* seconds */
    double  r2;
    int32_t n;
} relserve_duration_model;
int32_t relserve_duration_fit(const double* units, const double* seconds, int32_t n, relserve_duration_model* out);
int32_t relserve_duration_predict(const relserve_duration_model* model, double units, double* seconds);

/* ---- Priority Estimation Model (Sec. 4.2: Algorithm 1 "Batch Decomposition", Eq. 10) ----
 * The scheduler's priority of a relQuery is its predicted remaining duration: its requests, in order, are
 * decomposed into the prefill batches and decode batches the engine would run, and Eq. 9 is summed over them.
 * utok[i] >= 0: uncached tokens request i still has to prefill (0 = already prefilled; it joins no prefill
 * batch); decodes (may be NULL = all 1): whether request i still decodes; out_len = OL(R), the decode
 * iterations of each group; limits: tokens the KV cache manager admits at once (cap), max_num_seqs and
 * max_num_batched_tokens.  Walking the requests: request i first closes the open prefill batch and decodes the
 * open group to completion if it would exceed cap or max_num_seqs (the token count restarts with them), then
 * closes the open prefill batch if it would exceed max_num_batched_tokens, then joins both; the leftovers are
 * closed at the end.  Empty batches are never emitted; a request above max_num_batched_tokens is a batch of
 * its own.
 * relserve_batch_decompose: outputs (any may be NULL except the counts): prefill_batch_of[i] / decode_group_of[i]
 * = index of the batch / group request i joined (-1 = none); prefill_utok[b] = tokens of prefill batch b and
 * group_req[g] = requests of decode group g (arrays of n entries are always large enough); *n_prefill, *n_groups.
 * Every decode group stands for out_len identical decode batches.
 * relserve_pem_estimate: *seconds = sum over prefill batches of (alpha_p utok + beta_p) + out_len x sum over
 * decode groups of (alpha_d req + beta_d).  All pointers are HOST memory, read (or written) during the call.
 * RELSERVE_ERR_BAD_ARGUMENT: negative n / out_len / utok / cap, or a limit below 1. */
typedef struct relserve_pem_limits {
    int32_t cap;
    int32_t max_num_seqs;
    int32_t max_num_batched_tokens;
} relserve_pem_limits;
int32_t relserve_batch_decompose(const int32_t* utok, const uint8_t* decodes, int32_t n, int32_t out_len,
                                 const relserve_pem_limits* limits, int32_t* prefill_batch_of, int32_t* decode_group_of,
                                 int32_t* prefill_utok, int32_t* n_prefill, int32_t* group_req, int32_t* n_groups);
int32_t relserve_pem_estimate(const int32_t* utok, const uint8_t* decodes, int32_t n, int32_t out_len,
                              const relserve_pem_limits* limits, const relserve_duration_model* prefill,
                              const relserve_duration_model* decode, double* seconds);

/* ---- Adaptive Batch Arranger decision (Sec. 4.3, Eq. 14-17) and starvation rule (Sec. 4.2, Eq. 13) ----
 * Each iteration runs either the candidate decode batch (all running requests) or the candidate prefill batch
 * (requests of the first waiting relQuery).  relserve_aba_decide: both candidates empty -> IDLE; one empty ->
 * the other; otherwise with m_running / m_waiting the smallest priority values in the two candidates (Eq. 14):
 * m_running >= m_waiting -> PREFILL (a shorter relQuery preempts, or the running relQuery is still being
 * prefilled); m_running < m_waiting -> *delta = delta_plus - delta_minus, where delta_plus (Eq. 15) =
 * L_prefill(candidate) x running relQueries + sum over running relQueries R of alpha_d x req(candidate) x
 * min(OL(R), OL(candidate)) and delta_minus (Eq. 16) = waiting relQueries x beta_d x min(OL(candidate), max OL(R));
 * PREFILL iff *delta < 0 (Eq. 16 is a reduction: it is subtracted).  running_out_len: HOST array of
 * n_running_relqueries entries, read only in the last case.  delta may be NULL; it is 0 in the other cases.
 * relserve_starved_priority: *out = 0 if waiting_seconds / n_requests_submitted > threshold, else priority.
 * Host only. */
enum { RELSERVE_ABA_IDLE = 0, RELSERVE_ABA_PREFILL = 1, RELSERVE_ABA_DECODE = 2 };
typedef struct relserve_aba_input {
    double         m_running;               /* smallest priority value among the running requests */
    double         m_waiting;               /* smallest priority value in the candidate prefill batch */
    int32_t        n_running_reqs;          /* requests of the candidate decode batch (0 = empty) */
    int32_t        cand_prefill_reqs;       /* requests of the candidate prefill batch (0 = empty) */
    int32_t        cand_prefill_utok;       /* its uncached tokens */
    int32_t        cand_prefill_out_len;    /* OL of its relQuery */
    int32_t        n_running_relqueries;
    int32_t        n_waiting_relqueries;
    const int32_t* running_out_len;         /* OL of every running relQuery */
} relserve_aba_input;
int32_t relserve_aba_decide(const relserve_aba_input* in, const relserve_duration_model* prefill,
                            const relserve_duration_model* decode, int32_t* decision, double* delta);
int32_t relserve_starved_priority(double priority, double waiting_seconds, int32_t n_requests_submitted, double threshold,
                                  double* out);

/* ---- the remaining per-iteration arithmetic of the scheduler; all host only, no device work, no allocation ----
 * relserve_static_priority (Sec. 3, Eq. 6-7, the static-priority baseline): *priority = sum over the n requests
 * of L1(tok[i]) + L2(out_len) with linear L1(x) = l1->alpha x + l1->beta and L2(x) = l2->alpha x + l2->beta
 * (identity and constant mappings are special cases); computed once when a relQuery arrives and never updated.
 * relserve_utok_estimate (Sec. 4.2 "Fast Priority Estimation", Eq. 11): cache miss ratio of a sample of the
 * relQuery's requests = sum sample_utok / sum sample_tok; utok_out[i] = tok[i] x ratio rounded to the nearest
 * integer (ties to even).  Which requests are sampled is the caller's random draw.
 * relserve_priority_reuse (Eq. 12): *reuse = 1 iff every request of the relQuery was waiting at the previous
 * iteration and still is (n_waiting_before == n_waiting_now == n_submitted).
 * relserve_prefill_candidate (Sec. 4.3, the candidate prefill batch): requests are added from the front of utok
 * (the waiting requests of ONE relQuery, in order) while the three limits hold: a sequence slot is free
 * (seqs_free), the KV cache manager has room for the request's uncached tokens (tokens_free), and the batch stays
 * within max_num_batched_tokens (tokens_in_batch = tokens other relQueries already put into it; a request that
 * alone exceeds the limit is still taken into an empty batch).  Outputs: requests taken and their tokens.
 * RELSERVE_ERR_BAD_ARGUMENT on negative counts or sample_utok > sample_tok. */
int32_t relserve_static_priority(const int32_t* tok, int32_t n, int32_t out_len, const relserve_duration_model* l1,
                                 const relserve_duration_model* l2, double* priority);
int32_t relserve_utok_estimate(const int32_t* tok, int32_t n, const int32_t* sample_tok, const int32_t* sample_utok,
                               int32_t n_sample, int32_t* utok_out);
int32_t relserve_priority_reuse(int32_t n_submitted, int32_t n_waiting_before, int32_t n_waiting_now, int32_t* reuse);
int32_t relserve_prefill_candidate(const int32_t* utok, int32_t n, int64_t tokens_free, int32_t seqs_free,
                                   int32_t tokens_in_batch, int32_t max_num_batched_tokens, int32_t* n_taken,
                                   int64_t* tokens_taken);

/* ---- peak probes: what this GPU sustains, reported by bench.py beside the published peaks ----
 * relserve_peak_probe_mfma enqueues 256 workgroups of 4 waves that each issue iters x 16 independent
 * 32x32x16 bf16 MFMAs on random operands (no memory traffic) and writes the flop count of the launch to
 * *flops (host).  relserve_peak_probe_stream enqueues one read of `bytes` bytes of device memory at src
 * (16-byte aligned).  sink: device memory, at least 16 bytes, never written in practice.  The caller
 * times the launches on `stream`. */
int32_t relserve_peak_probe_mfma(void* sink, int32_t iters, double* flops, void* stream);
int32_t relserve_peak_probe_stream(const void* src, size_t bytes, void* sink, void* stream);
/* The read patterns relserve_peak_probe_stream's was chosen from, for the record of that choice: pattern 0 = grid-stride
 * walk with plain 16-byte loads; 1 = 32 KB pieces per workgroup, plain loads; 2 = the same with the non-temporal hint
 * (= relserve_peak_probe_stream); 3 / 4 = the pieces loaded directly into LDS without / with the hint (the form the GEMM and
 * attention kernels use).  bytes >= 32768. */
int32_t relserve_peak_probe_stream_pattern(const void* src, size_t bytes, int32_t pattern, void* sink, void* stream);

/* ---- test hook (the only one; not part of the serving interface) ----
 * Forces the tile shape and the tail split of every later GEMM launch of this process, so that tests can
 * drive each tile shape and the split-tail path on shapes the automatic choice would serve otherwise:
 * tile = 0..4 (256x256, 192x256, 128x256, 128x128, 64x128 tokens x features), -1 = automatic choice.
 * tail_splits = 2..8 makes the tiles of the incomplete last round split their k range that many ways
 * (0 or 1 = whole tiles only).  Shapes a tile cannot serve (the fused q/k/v epilogue needs 256 features per
 * tile) fall back to the nearest one that can.  Process-wide; the setting is one atomic word, so a launch
 * on another host thread sees either the old or the new pair. */
int32_t relserve_debug_force_gemm_plan(int32_t tile, int32_t tail_splits);

/* ---- per-kernel timing with HIP events on the caller's stream ---- */

#define RELSERVE_PROFILE_SLOTS 12
/* names, in launch order, of the kernels one layer step runs */
const char* relserve_profile_slot_name(int32_t slot);
/* slot_mask: bit i set = relserve_layer_step records an event pair around the
 * kernel of slot i (-1 = every kernel, 0 = off); the durations are accumulated
 * at the next relserve_profile_read, which synchronises the stream.  Each pair
 * costs a few microseconds of stream time.  ms_sum / launches: host arrays of
 * RELSERVE_PROFILE_SLOTS entries. */
int32_t relserve_profile_enable(relserve_layer* layer, int32_t slot_mask);
int32_t relserve_profile_read(relserve_layer* layer, double* ms_sum, int64_t* launches, int32_t reset);

#ifdef __cplusplus
}
#endif
#endif
