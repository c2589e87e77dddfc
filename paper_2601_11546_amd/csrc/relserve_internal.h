// Internal declarations shared by the host boundary and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "relserve.h"

namespace relserve {

// ---- attention work items (one workgroup each) -------------------------------------------
// An item is a set of query tokens that read the same run of cached keys through one
// block-table row: either the members of a shared-prefix group against the prefix pages,
// or consecutive query tokens of one request against that request's own keys.
enum : int32_t {
    ITEM_CAUSAL = 1,        // a row at position p sees keys <= p
    ITEM_INIT_PARTIAL = 2,  // running softmax state starts from the stored prefix partial
    ITEM_WRITE_PARTIAL = 4  // store the running state instead of the normalised output
};

struct AttnItem {
    int32_t tok_off;    // first entry of this item in the attn_tok list
    int32_t n_tok;      // query tokens of the item (rows = n_tok * heads per kv head)
    int32_t bt_req;     // request whose block-table row addresses the keys
    int32_t key_begin;  // first key position (page aligned)
    int32_t key_end;    // one past the last key position any row may see
    int32_t flags;
    int32_t pad0;       // decode items: the query token
    int32_t pad1;       // decode items that write partial state: the slot
};

// A decode row whose own keys were cut into several wave items (chunks): each chunk stores its running softmax state
// in a slot, and one merge combines the slots [first_slot, first_slot + n_chunks) into the row's output.
struct MergeItem {
    int32_t tok;
    int32_t first_slot;
    int32_t n_chunks;
    int32_t pad;
};

// Slots of partial state the chunked decode rows of a batch of T tokens may use (rows T .. T + cap of the partial-state
// buffers, behind the T rows that hold the shared-prefix pass's state).
inline int64_t split_slot_cap(int64_t T) { return 2 * (T < 2048 ? T : 2048); }

// Device-side view of a prepared batch (all pointers into one device allocation).
struct BatchDev {
    int32_t T, num_reqs, max_blocks, num_pages;
    const int32_t* tok_req;      // [T]
    const int32_t* tok_pos;      // [T] position of the token in its own sequence
    const int32_t* tok_slot;     // [T] cache slot the token is appended to
    const int32_t* last_tok;     // [num_reqs] packed row of each request's last query token
    const int32_t* block_table;  // [num_reqs, max_blocks]
    const float2* rope_cs;       // [T, head_dim / 2] (cos, sin) of pos * base^(-2i/d)
    const int32_t* attn_tok;     // token lists of the attention items
    const AttnItem* items_prefix;  // joint prefix passes (write partial state)
    const AttnItem* items_tile;    // row-tiled passes (prefill rows)
    const AttnItem* items_split;   // wave items (decode rows, or chunks of their keys)
    const MergeItem* merge_items;  // decode rows cut into chunks
    int32_t n_items_prefix, n_items_tile, n_items_split, n_merge;
};

}  // namespace relserve

struct relserve_layer {
    relserve_layer_config cfg;
    int32_t group;  // q heads per kv head
    int32_t q_dim, kv_dim, qkv_dim;
    std::vector<float> inv_freq;  // [head_dim / 2] base^(-2i/d), rounded from double
    // profiling
    uint32_t profile = 0;   // bit i set: time the kernel of slot i
    struct Pending { int slot; hipEvent_t a, b; };
    std::vector<Pending> pending;
    std::vector<hipEvent_t> event_pool;   // events of earlier reads, reused
    hipStream_t pending_stream = nullptr;
    double ms_sum[RELSERVE_PROFILE_SLOTS] = {0};
    int64_t launches[RELSERVE_PROFILE_SLOTS] = {0};
};

struct relserve_batch {
    relserve_layer_config cfg;  // shape it was prepared for
    relserve::BatchDev dev;
    void* blob = nullptr;  // the one device allocation
    relserve_batch_info info;
};

namespace relserve {

// Host-side expansion of a descriptor (no device calls); shared by validate / slots / prepare.
struct HostBatch {
    int32_t T = 0;
    std::vector<int32_t> tok_req, tok_pos, tok_slot;
    std::vector<int32_t> attn_tok;
    std::vector<AttnItem> items_prefix, items_tile, items_split;
    std::vector<MergeItem> merge_items;
    int32_t n_decode = 0, n_prefill = 0, n_groups = 0;
};
int32_t expand_batch(const relserve_layer_config& cfg, const relserve_batch_desc& d, bool build_items,
                     HostBatch* out);

// Rows of queries one attention workgroup covers (4 waves x 32 MFMA columns).
constexpr int ATTN_BLOCK_M = 128;
constexpr int SKINNY_MAX_T = 256;      // batches up to this many tokens take the split-K GEMM path
constexpr int64_t GEMM_TAIL_FLOATS = 256 * 65536;      // GEMM scratch at T > 256: partial tiles of one round of split 256 x 256 tiles
constexpr int ATTN_SPLIT_ROWS = 16;   // query heads per kv head the decode kernel's 16-column MFMA holds

// ---- kernel launchers (each enqueues on `s` and returns the launch status) ----------------
hipError_t launch_rope_table(const int32_t* tok_pos, const float* inv_freq_dev, int32_t T, int32_t half,
                             float2* out, hipStream_t s);
// code_scale > 0: out holds 8-bit codes of the normed value / code_scale instead of bf16
hipError_t launch_rmsnorm(const void* x, bool x_is_f32, const void* w, float eps, int32_t rows, int32_t H,
                          void* out, hipStream_t s, const int32_t* row_index = nullptr, float code_scale = 0.0f);
hipError_t launch_embedding(const int32_t* ids, const void* table, int32_t vocab, int32_t H, int32_t T, void* out,
                            hipStream_t s);
hipError_t launch_greedy_sample(const float* logits, int32_t n_rows, int32_t vocab, int32_t* next_token, hipStream_t s);
hipError_t launch_kv_append(const BatchDev& b, const void* k, const void* v, void* k_pages, void* v_pages,
                            int32_t row_elems, hipStream_t s);
hipError_t launch_rope_append(const BatchDev& b, const relserve_layer& L, void* qkv, void* k_pages,
                              void* v_pages, hipStream_t s);
// accum: optional fp32 scratch (gemm_scratch_floats(T, widest N) floats, contents irrelevant on entry);
// lets skinny problems (T <= 256), narrow outputs at mid-size T and the incomplete last round of larger
// ones split K over workgroups (partial tiles written there, summed by a second kernel).
int64_t gemm_scratch_floats(int64_t T, int64_t n_max);
void gemm_force_plan(int cand, int splits);   // test hook, see relserve_debug_force_gemm_plan
// Quantised projection: a [T, K] and w [N, K] hold 8-bit codes (K % 128 == 0); the sums take the factor
// a_scale * w_scale[n]; out_scale > 0 makes a SwiGLU epilogue store codes of value / out_scale.
struct CodeScales {
    const float* w_scale = nullptr;   // [N] device
    float a_scale = 1.0f;
    float out_scale = 0.0f;
};
hipError_t launch_linear(const void* a, const void* w, int32_t T, int32_t N, int32_t K, int32_t epilogue,
                         const void* residual, void* out, hipStream_t s, float* accum = nullptr, bool w_packed = false,
                         const CodeScales* codes = nullptr);
// w [N, K] row-major -> the tiled streaming layout (ceil(N / 256) * 256 * K elements), K % 64 == 0
hipError_t launch_pack_weight(const void* w, int32_t N, int32_t K, void* out, hipStream_t s);
// q/k/v projection with rotary embedding and KV append fused into the epilogue: q_out [T, n_q d] bf16.
// How the cache pools store an element: 16-bit, or an 8-bit code of x / scale (relserve_kv_cache).
struct KvFormat {
    bool fp8 = false;
    float k_scale = 1.0f, v_scale = 1.0f;
};
hipError_t launch_qkv_rope_append(const BatchDev& b, const relserve_layer& L, const void* h, const void* w_qkv,
                                  void* q_out, void* k_pages, void* v_pages, hipStream_t s, float* accum = nullptr,
                                  bool w_packed = false, KvFormat kv = KvFormat{}, const CodeScales* codes = nullptr);
// bf16 [n] -> 8-bit codes of value / scale (n % 8 == 0)
hipError_t launch_quantise_bf16(const void* in, int64_t n, float scale, void* codes, hipStream_t s);
// Attention passes; part_o [T + split_slot_cap(T), n_q, d] fp32 and part_ml [.., n_q, 2] fp32 hold the prefix partials
// (rows of the tokens) and the chunk partials of split decode rows (rows T + slot).
hipError_t launch_attention(const BatchDev& b, const relserve_layer& L, const void* q, int32_t q_pitch,
                            const void* k_pages, const void* v_pages, void* out, float* part_o,
                            float* part_ml, hipStream_t s, relserve_layer* prof, KvFormat kv = KvFormat{});

void profile_mark(relserve_layer* L, int slot, hipStream_t s, bool begin);

// Peak probes (kernels_peaks.hip): 256 workgroups x 4 waves x iters x 16 MFMAs of 32768 flop; a read of `bytes`.
hipError_t launch_peak_mfma(float* sink, int32_t iters, hipStream_t s);
hipError_t launch_peak_stream(const void* src, int64_t bytes, uint32_t* sink, hipStream_t s);
hipError_t launch_peak_stream_pattern(const void* src, int64_t bytes, int32_t pattern, uint32_t* sink, hipStream_t s);

}  // namespace relserve
