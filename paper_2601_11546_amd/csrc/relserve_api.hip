// Host boundary of the layer-step library: validation, descriptor expansion, upload,
// workspace carving and kernel sequencing.  No arithmetic of the method lives here.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>

#include "relserve_internal.h"

using namespace relserve;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

const char* const kSlotNames[RELSERVE_PROFILE_SLOTS] = {
    "rmsnorm_in", "gemm_qkv_rope_append", "attn_own_keys", "attn_prefix", "attn_tile", "attn_split",
    "gemm_o",     "rmsnorm_post", "gemm_gate_up", "gemm_down",  "attn_merge", "quantise_attn"};
enum { S_NORM1 = 0, S_QKV, S_ATTN_OWN, S_ATTN_PREFIX, S_ATTN_TILE, S_ATTN_SPLIT, S_O, S_NORM2, S_GU, S_DOWN, S_ATTN_MERGE, S_QUANT };

struct Workspace {
    char* h;         // [T, H] bf16 (normed activations; reused for the post norm)
    char* q;         // [T, q_dim] bf16 rotated queries
    char* attn;      // [T, q_dim] bf16
    char* x1;        // [T, H] fp32 residual stream after attention
    char* act;       // [T, I] bf16
    float* part_o;   // [T + split slots, n_q, d] fp32
    float* part_ml;  // [T + split slots, n_q, 2] fp32
    float* accum;    // fp32 split-K scratch of the GEMMs
    size_t accum_floats;
    size_t total;
};

Workspace carve(const relserve_layer& L, int64_t T, void* base) {
    Workspace w;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char* p = base ? static_cast<char*>(base) + off : nullptr;
        off += align_up(bytes);
        return p;
    };
    const relserve_layer_config& c = L.cfg;
    w.h = take((size_t)T * c.hidden * 2);
    w.q = take((size_t)T * L.q_dim * 2);
    w.attn = take((size_t)T * L.q_dim * 2);
    w.x1 = take((size_t)T * c.hidden * 4);
    w.act = take((size_t)T * c.mlp_dim * 2);
    const size_t part_rows = (size_t)(T + split_slot_cap(T));
    w.part_o = reinterpret_cast<float*>(take(part_rows * L.q_dim * 4));
    w.part_ml = reinterpret_cast<float*>(take(part_rows * c.n_q_heads * 2 * 4));
    w.accum_floats = (size_t)gemm_scratch_floats(T, std::max({L.qkv_dim, 2 * c.mlp_dim, c.hidden}));
    w.accum = reinterpret_cast<float*>(take(w.accum_floats * 4));
    w.total = off;
    return w;
}

bool is_pow2(int32_t v) { return v > 0 && (v & (v - 1)) == 0; }

// Workspace of relserve_layer_step_static: a fixed array in device memory, one copy per GPU the library runs on,
// held until the process ends.  `scratch` is only a host-side stand-in for the symbol: the device address comes
// from hipGetSymbolAddress, once per device, and only that address is handed to kernels.
constexpr size_t kStaticScratchBytes = (size_t)RELSERVE_STATIC_SCRATCH_BYTES;
__device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int32_t static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return RELSERVE_ERR_NO_DEVICE;
    if (dev < 0 || dev >= kMaxDevices) return RELSERVE_ERR_BAD_ARGUMENT;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return RELSERVE_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return RELSERVE_OK;
}

KvFormat kv_format(const relserve_kv_cache& cache) {
    KvFormat f;
    f.fp8 = cache.dtype == RELSERVE_KV_FP8;
    if (f.fp8) f.k_scale = cache.k_scale, f.v_scale = cache.v_scale;
    return f;
}

int32_t check_cache(const relserve_batch* b, const relserve_kv_cache& cache, bool fp8_ok = true) {
    if (!cache.k_pages || !cache.v_pages) return RELSERVE_ERR_NULL_POINTER;
    if (cache.dtype != RELSERVE_KV_BF16 && cache.dtype != RELSERVE_KV_FP8) return RELSERVE_ERR_BAD_ARGUMENT;
    if (cache.dtype == RELSERVE_KV_FP8) {
        if (!fp8_ok) return RELSERVE_ERR_BAD_ARGUMENT;
        if (!(cache.k_scale > 0.0f) || !(cache.v_scale > 0.0f) || !std::isfinite(cache.k_scale) || !std::isfinite(cache.v_scale))
            return RELSERVE_ERR_BAD_ARGUMENT;
    }
    if (cache.num_pages < b->dev.num_pages) return RELSERVE_ERR_MISMATCH;
    return RELSERVE_OK;
}

int32_t check_pair(const relserve_layer* L, const relserve_batch* b) {
    if (!L || !b) return RELSERVE_ERR_NULL_POINTER;
    if (std::memcmp(&L->cfg, &b->cfg, sizeof(relserve_layer_config)) != 0) return RELSERVE_ERR_MISMATCH;
    return RELSERVE_OK;
}

}  // namespace

// ------------------------------------------------------------------------------------------
// descriptor expansion (host only)
// ------------------------------------------------------------------------------------------
int32_t relserve::expand_batch(const relserve_layer_config& cfg, const relserve_batch_desc& d,
                               bool build_items, HostBatch* out) {
    if (d.num_reqs < 0 || d.max_blocks < 0 || d.num_pages < 0 || d.num_prefixes < 0)
        return RELSERVE_ERR_BAD_ARGUMENT;
    if (!d.q_start) return RELSERVE_ERR_NULL_POINTER;
    if (d.num_reqs > 0 && (!d.ctx_len || !d.block_table)) return RELSERVE_ERR_NULL_POINTER;
    if (d.num_prefixes > 0 && !d.prefix_len) return RELSERVE_ERR_NULL_POINTER;
    const int32_t P = cfg.page_size, B = d.num_reqs;
    if ((int64_t)d.num_pages * P >= (int64_t)1 << 31) return RELSERVE_ERR_TOO_LARGE;
    if (d.q_start[0] != 0) return RELSERVE_ERR_BAD_Q_START;
    for (int32_t r = 0; r < B; ++r)
        if (d.q_start[r + 1] <= d.q_start[r]) return RELSERVE_ERR_BAD_Q_START;
    const int32_t T = d.q_start[B];
    if (T > (1 << 22)) return RELSERVE_ERR_TOO_LARGE;

    for (int32_t p = 0; p < d.num_prefixes; ++p)
        if (d.prefix_len[p] < 0 || d.prefix_len[p] % P != 0) return RELSERVE_ERR_BAD_PREFIX;

    HostBatch hb;
    hb.T = T;
    hb.tok_req.resize(T);
    hb.tok_pos.resize(T);
    hb.tok_slot.resize(T);
    std::vector<int32_t> first_member(d.num_prefixes, -1), members(d.num_prefixes, 0);
    for (int32_t r = 0; r < B; ++r) {
        const int32_t q_len = d.q_start[r + 1] - d.q_start[r];
        const int32_t L = d.ctx_len[r];
        if (L < q_len) return RELSERVE_ERR_BAD_CTX_LEN;
        const int32_t blocks = (L + P - 1) / P;
        if (blocks > d.max_blocks) return RELSERVE_ERR_BLOCK_TABLE_SHORT;
        const int32_t* bt = d.block_table + (size_t)r * d.max_blocks;
        for (int32_t i = 0; i < blocks; ++i)
            if (bt[i] < 0 || bt[i] >= d.num_pages) return RELSERVE_ERR_PAGE_RANGE;
        const int32_t past = L - q_len;
        const int32_t pid = d.prefix_id ? d.prefix_id[r] : -1;
        if (pid < -1 || pid >= d.num_prefixes) return RELSERVE_ERR_BAD_PREFIX;
        if (pid >= 0) {
            const int32_t pl = d.prefix_len[pid];
            if (pl > past) return RELSERVE_ERR_BAD_PREFIX;  // a member never writes a shared page
            if (first_member[pid] < 0) {
                first_member[pid] = r;
            } else {
                const int32_t* bt0 = d.block_table + (size_t)first_member[pid] * d.max_blocks;
                for (int32_t i = 0; i < pl / P; ++i)
                    if (bt[i] != bt0[i]) return RELSERVE_ERR_BAD_PREFIX;
            }
            ++members[pid];
        }
        for (int32_t j = 0; j < q_len; ++j) {
            const int32_t t = d.q_start[r] + j, pos = past + j;
            hb.tok_req[t] = r;
            hb.tok_pos[t] = pos;
            hb.tok_slot[t] = bt[pos / P] * P + pos % P;
        }
    }
    {   // no two appended tokens may land in the same slot
        std::vector<int32_t> s(hb.tok_slot);
        std::sort(s.begin(), s.end());
        for (size_t i = 1; i < s.size(); ++i)
            if (s[i] == s[i - 1]) return RELSERVE_ERR_SLOT_ALIAS;
    }
    {   // and none may land in a page that serves as a shared prefix page
        std::vector<uint8_t> shared(d.num_pages > 0 ? d.num_pages : 1, 0);
        bool any = false;
        for (int32_t p = 0; p < d.num_prefixes; ++p) {
            if (first_member[p] < 0) continue;
            const int32_t* bt0 = d.block_table + (size_t)first_member[p] * d.max_blocks;
            for (int32_t i = 0; i < d.prefix_len[p] / P; ++i) shared[bt0[i]] = 1, any = true;
        }
        if (any)
            for (int32_t t = 0; t < T; ++t)
                if (shared[hb.tok_slot[t] / P]) return RELSERVE_ERR_BAD_PREFIX;
    }

    for (int32_t r = 0; r < B; ++r) (d.q_start[r + 1] - d.q_start[r] == 1 ? hb.n_decode : hb.n_prefill)++;

    if (build_items) {
        const int32_t group = cfg.n_q_heads / cfg.n_kv_heads;
        const int32_t tile_tok = ATTN_BLOCK_M / group;    // tokens per row-tiled item (rows past tile_tok * group stay idle)
        // a prefix is handled jointly when at least two requests of the batch carry it
        std::vector<uint8_t> joint(d.num_prefixes, 0);
        for (int32_t p = 0; p < d.num_prefixes; ++p)
            joint[p] = (members[p] >= 2 && d.prefix_len[p] > 0);
        for (int32_t p = 0; p < d.num_prefixes; ++p) {
            if (!joint[p]) continue;
            ++hb.n_groups;
            const int32_t start = (int32_t)hb.attn_tok.size();
            for (int32_t r = 0; r < B; ++r)
                if (d.prefix_id[r] == p)
                    for (int32_t t = d.q_start[r]; t < d.q_start[r + 1]; ++t) hb.attn_tok.push_back(t);
            const int32_t n = (int32_t)hb.attn_tok.size() - start;
            for (int32_t o = 0; o < n; o += tile_tok) {
                AttnItem it{};
                it.tok_off = start + o;
                it.n_tok = std::min(tile_tok, n - o);
                it.bt_req = first_member[p];
                it.key_begin = 0;
                it.key_end = d.prefix_len[p];
                it.flags = ITEM_WRITE_PARTIAL;
                hb.items_prefix.push_back(it);
            }
        }
        // Decode rows with many own keys are cut into chunks (one wave item each, merged afterwards), so that one long
        // context does not set the kernel's duration and the waves come in several even rounds.  The chunk length is
        // the smallest of 128 .. 1024 keys whose chunks fit the partial-state slots of the workspace.
        auto own_keys = [&](int32_t r) {
            const int32_t pid = d.prefix_id ? d.prefix_id[r] : -1;
            return d.ctx_len[r] - ((pid >= 0 && joint[pid]) ? d.prefix_len[pid] : 0);
        };
        auto chunks_of = [](int32_t own, int32_t len) { return len > 0 ? std::max(1, (own + len / 2) / len) : 1; };
        int32_t chunk_len = 0;   // 0 = no row is cut
        // (with two rounds of waves or more -- 256 CUs x 8 resident waves each -- the rows balance by themselves: cutting
        // the 128 rows x 40 heads of 1024 keys of a 13B decode batch in two left its kernel at 6.5 TB/s and added the merge)
        if ((int64_t)hb.n_decode * cfg.n_kv_heads < 2 * 2048) {
            const int64_t cap = split_slot_cap(T);
            for (int32_t len = 128; len <= 1024 && chunk_len == 0; len *= 2) {
                int64_t slots = 0;
                bool any = false;
                for (int32_t r = 0; r < B; ++r)
                    if (d.q_start[r + 1] - d.q_start[r] == 1) {
                        const int32_t n = chunks_of(own_keys(r), len);
                        if (n > 1) slots += n, any = true;
                    }
                if (!any) break;               // no row is longer than a chunk and a half: nothing to cut at any larger length
                if (slots <= cap) chunk_len = len;
            }
        }
        int32_t next_slot = 0;
        for (int32_t r = 0; r < B; ++r) {
            const int32_t q_len = d.q_start[r + 1] - d.q_start[r];
            const int32_t pid = d.prefix_id ? d.prefix_id[r] : -1;
            const bool grouped = pid >= 0 && joint[pid];
            const int32_t kb = grouped ? d.prefix_len[pid] : 0;
            const int32_t flags = ITEM_CAUSAL | (grouped ? ITEM_INIT_PARTIAL : 0);
            const int32_t past = d.ctx_len[r] - q_len;
            if (q_len == 1) {
                const int32_t own = d.ctx_len[r] - kb;
                const int32_t n_chunks = chunks_of(own, chunk_len);
                // chunk boundaries on multiples of 32 keys (the wave kernel's block) counted from the first own key
                const int32_t per = n_chunks > 1 ? ((own + n_chunks - 1) / n_chunks + 31) / 32 * 32 : own;
                if (n_chunks > 1) hb.merge_items.push_back(MergeItem{d.q_start[r], next_slot, 0, 0});
                for (int32_t c = 0; c < n_chunks; ++c) {
                    const int32_t b0 = kb + c * per, b1 = std::min(kb + (c + 1) * per, d.ctx_len[r]);
                    if (b0 >= b1) break;
                    AttnItem it{};
                    it.tok_off = (int32_t)hb.attn_tok.size();
                    hb.attn_tok.push_back(d.q_start[r]);
                    it.n_tok = 1;
                    it.pad0 = d.q_start[r];  // the decode kernel takes its single token from here
                    it.bt_req = r;
                    it.key_begin = b0;
                    it.key_end = b1;
                    it.flags = c == 0 ? flags : ITEM_CAUSAL;      // only the first chunk continues from the prefix pass's state
                    if (n_chunks > 1) {
                        it.flags |= ITEM_WRITE_PARTIAL;
                        it.pad1 = next_slot++;
                        ++hb.merge_items.back().n_chunks;
                    }
                    hb.items_split.push_back(it);
                }
            } else {
                for (int32_t o = 0; o < q_len; o += tile_tok) {
                    AttnItem it{};
                    it.tok_off = (int32_t)hb.attn_tok.size();
                    it.n_tok = std::min(tile_tok, q_len - o);
                    for (int32_t j = 0; j < it.n_tok; ++j) hb.attn_tok.push_back(d.q_start[r] + o + j);
                    it.bt_req = r;
                    it.key_begin = kb;
                    it.key_end = past + o + it.n_tok;  // the item's last row sees keys up to itself
                    it.flags = flags;
                    hb.items_tile.push_back(it);
                }
            }
        }
        // longest first: the tail of the launch then consists of short items
        auto longer = [](const AttnItem& a, const AttnItem& b) {
            return (a.key_end - a.key_begin) > (b.key_end - b.key_begin);
        };
        std::stable_sort(hb.items_tile.begin(), hb.items_tile.end(), longer);
        std::stable_sort(hb.items_split.begin(), hb.items_split.end(), longer);
    }
    *out = std::move(hb);
    return RELSERVE_OK;
}

// ------------------------------------------------------------------------------------------
// plain entry points
// ------------------------------------------------------------------------------------------
// The launchers report hipGetLastError() after a launch; an error an earlier, unrelated HIP call of this thread left
// behind (the runtime keeps the last one until it is read) must not be taken for theirs.
static inline void drop_stale_hip_error() { (void)hipGetLastError(); }

extern "C" {

int32_t relserve_version(void) { return 100; }

const char* relserve_strerror(int32_t s) {
    switch (s) {
        case RELSERVE_OK: return "ok";
        case RELSERVE_ERR_NULL_POINTER: return "null pointer";
        case RELSERVE_ERR_BAD_CONFIG: return "unsupported layer shape";
        case RELSERVE_ERR_BAD_Q_START: return "q_start must start at 0 and increase strictly";
        case RELSERVE_ERR_BAD_CTX_LEN: return "ctx_len shorter than the request's query tokens";
        case RELSERVE_ERR_BLOCK_TABLE_SHORT: return "block table row too short for ctx_len";
        case RELSERVE_ERR_PAGE_RANGE: return "block table entry outside the page pool";
        case RELSERVE_ERR_BAD_PREFIX: return "shared prefix inconsistent with the block tables";
        case RELSERVE_ERR_SLOT_ALIAS: return "two query tokens map to the same cache slot";
        case RELSERVE_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case RELSERVE_ERR_HIP: return "HIP runtime error";
        case RELSERVE_ERR_NO_DEVICE: return "no gfx950 device";
        case RELSERVE_ERR_TOO_LARGE: return "size exceeds 32-bit device indices or the fixed scratch";
        case RELSERVE_ERR_MISMATCH: return "batch / layer / cache do not belong together";
        case RELSERVE_ERR_BAD_ARGUMENT: return "bad argument";
        default: return "unknown status";
    }
}

int32_t relserve_config_validate(const relserve_layer_config* c) {
    if (!c) return RELSERVE_ERR_NULL_POINTER;
    if (c->hidden <= 0 || c->hidden % 8) return RELSERVE_ERR_BAD_CONFIG;
    if (c->mlp_dim <= 0 || c->mlp_dim % 8) return RELSERVE_ERR_BAD_CONFIG;
    if (c->head_dim != 64 && c->head_dim != 128) return RELSERVE_ERR_BAD_CONFIG;
    if (c->n_kv_heads <= 0 || c->n_q_heads <= 0 || c->n_q_heads % c->n_kv_heads) return RELSERVE_ERR_BAD_CONFIG;
    if (c->n_q_heads / c->n_kv_heads > ATTN_SPLIT_ROWS) return RELSERVE_ERR_BAD_CONFIG;  // one wave's query rows
    if (!is_pow2(c->page_size) || c->page_size < 8 || c->page_size > 256) return RELSERVE_ERR_BAD_CONFIG;
    if (!(c->rms_eps >= 0.0f) || !(c->rope_base > 0.0f)) return RELSERVE_ERR_BAD_CONFIG;
    return RELSERVE_OK;
}

int32_t relserve_layer_create(const relserve_layer_config* cfg, relserve_layer** out) {
    if (!cfg || !out) return RELSERVE_ERR_NULL_POINTER;
    *out = nullptr;
    if (int32_t rc = relserve_config_validate(cfg)) return rc;
    relserve_layer* L = new (std::nothrow) relserve_layer();
    if (!L) return RELSERVE_ERR_BAD_ARGUMENT;
    L->cfg = *cfg;
    L->group = cfg->n_q_heads / cfg->n_kv_heads;
    L->q_dim = cfg->n_q_heads * cfg->head_dim;
    L->kv_dim = cfg->n_kv_heads * cfg->head_dim;
    L->qkv_dim = L->q_dim + 2 * L->kv_dim;
    const int half = cfg->head_dim / 2;
    L->inv_freq.resize(half);
    for (int i = 0; i < half; ++i)
        L->inv_freq[i] = (float)std::pow((double)cfg->rope_base, -2.0 * i / (double)cfg->head_dim);
    *out = L;
    return RELSERVE_OK;
}

int32_t relserve_layer_destroy(relserve_layer* L) {
    if (!L) return RELSERVE_OK;
    for (auto& p : L->pending) {
        (void)hipEventDestroy(p.a);
        (void)hipEventDestroy(p.b);
    }
    for (hipEvent_t e : L->event_pool) (void)hipEventDestroy(e);
    delete L;
    return RELSERVE_OK;
}

int32_t relserve_batch_validate(const relserve_layer_config* cfg, const relserve_batch_desc* desc) {
    if (!cfg || !desc) return RELSERVE_ERR_NULL_POINTER;
    if (int32_t rc = relserve_config_validate(cfg)) return rc;
    HostBatch hb;
    return expand_batch(*cfg, *desc, false, &hb);
}

int32_t relserve_batch_slots(const relserve_layer_config* cfg, const relserve_batch_desc* desc,
                             int32_t* slots_out) {
    if (!cfg || !desc || !slots_out) return RELSERVE_ERR_NULL_POINTER;
    if (int32_t rc = relserve_config_validate(cfg)) return rc;
    HostBatch hb;
    if (int32_t rc = expand_batch(*cfg, *desc, false, &hb)) return rc;
    std::memcpy(slots_out, hb.tok_slot.data(), sizeof(int32_t) * hb.tok_slot.size());
    return RELSERVE_OK;
}

int32_t relserve_batch_prepare(const relserve_layer* L, const relserve_batch_desc* desc, void* stream,
                               relserve_batch** out) {
    drop_stale_hip_error();
    if (!L || !desc || !out) return RELSERVE_ERR_NULL_POINTER;
    *out = nullptr;
    HostBatch hb;
    if (int32_t rc = expand_batch(L->cfg, *desc, true, &hb)) return rc;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev == 0) return RELSERVE_ERR_NO_DEVICE;
    {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess)
            return RELSERVE_ERR_HIP;
        if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return RELSERVE_ERR_NO_DEVICE;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int32_t T = hb.T, B = desc->num_reqs, half = L->cfg.head_dim / 2;

    // one host blob, one device allocation
    size_t off = 0;
    auto reserve = [&](size_t bytes) { size_t o = off; off += align_up(bytes ? bytes : 1); return o; };
    const size_t o_req = reserve(sizeof(int32_t) * T), o_pos = reserve(sizeof(int32_t) * T);
    const size_t o_slot = reserve(sizeof(int32_t) * T);
    const size_t o_last = reserve(sizeof(int32_t) * B);
    const size_t o_bt = reserve(sizeof(int32_t) * (size_t)B * desc->max_blocks);
    const size_t o_tok = reserve(sizeof(int32_t) * hb.attn_tok.size());
    const size_t o_ip = reserve(sizeof(AttnItem) * hb.items_prefix.size());
    const size_t o_it = reserve(sizeof(AttnItem) * hb.items_tile.size());
    const size_t o_is = reserve(sizeof(AttnItem) * hb.items_split.size());
    const size_t o_mi = reserve(sizeof(MergeItem) * hb.merge_items.size());
    const size_t o_freq = reserve(sizeof(float) * half);
    const size_t host_bytes = off;
    const size_t o_cs = reserve(sizeof(float2) * (size_t)T * half);
    const size_t total = off;

    std::vector<char> host(host_bytes, 0);
    auto put = [&](size_t o, const void* src, size_t bytes) { if (bytes) std::memcpy(host.data() + o, src, bytes); };
    put(o_req, hb.tok_req.data(), sizeof(int32_t) * T);
    put(o_pos, hb.tok_pos.data(), sizeof(int32_t) * T);
    put(o_slot, hb.tok_slot.data(), sizeof(int32_t) * T);
    {
        std::vector<int32_t> last(B);
        for (int32_t r = 0; r < B; ++r) last[r] = desc->q_start[r + 1] - 1;
        put(o_last, last.data(), sizeof(int32_t) * B);
    }
    put(o_bt, desc->block_table, sizeof(int32_t) * (size_t)B * desc->max_blocks);
    put(o_tok, hb.attn_tok.data(), sizeof(int32_t) * hb.attn_tok.size());
    put(o_ip, hb.items_prefix.data(), sizeof(AttnItem) * hb.items_prefix.size());
    put(o_it, hb.items_tile.data(), sizeof(AttnItem) * hb.items_tile.size());
    put(o_is, hb.items_split.data(), sizeof(AttnItem) * hb.items_split.size());
    put(o_mi, hb.merge_items.data(), sizeof(MergeItem) * hb.merge_items.size());
    put(o_freq, L->inv_freq.data(), sizeof(float) * half);

    relserve_batch* b = new (std::nothrow) relserve_batch();
    if (!b) return RELSERVE_ERR_BAD_ARGUMENT;
    b->cfg = L->cfg;
    if (hipMalloc(&b->blob, total) != hipSuccess) {
        delete b;
        return RELSERVE_ERR_HIP;
    }
    char* base = static_cast<char*>(b->blob);
    BatchDev& dv = b->dev;
    dv.T = T;
    dv.num_reqs = B;
    dv.max_blocks = desc->max_blocks;
    dv.num_pages = desc->num_pages;
    dv.tok_req = reinterpret_cast<int32_t*>(base + o_req);
    dv.tok_pos = reinterpret_cast<int32_t*>(base + o_pos);
    dv.tok_slot = reinterpret_cast<int32_t*>(base + o_slot);
    dv.last_tok = reinterpret_cast<int32_t*>(base + o_last);
    dv.block_table = reinterpret_cast<int32_t*>(base + o_bt);
    dv.attn_tok = reinterpret_cast<int32_t*>(base + o_tok);
    dv.items_prefix = reinterpret_cast<AttnItem*>(base + o_ip);
    dv.items_tile = reinterpret_cast<AttnItem*>(base + o_it);
    dv.items_split = reinterpret_cast<AttnItem*>(base + o_is);
    dv.merge_items = reinterpret_cast<MergeItem*>(base + o_mi);
    dv.n_merge = (int32_t)hb.merge_items.size();
    dv.rope_cs = reinterpret_cast<float2*>(base + o_cs);
    dv.n_items_prefix = (int32_t)hb.items_prefix.size();
    dv.n_items_tile = (int32_t)hb.items_tile.size();
    dv.n_items_split = (int32_t)hb.items_split.size();
    b->info = relserve_batch_info{T, B, hb.n_decode, hb.n_prefill, hb.n_groups,
                                  dv.n_items_prefix + dv.n_items_tile + dv.n_items_split};

    hipError_t e = hipMemcpyAsync(b->blob, host.data(), host_bytes, hipMemcpyHostToDevice, s);
    if (e == hipSuccess && T > 0)
        e = launch_rope_table(dv.tok_pos, reinterpret_cast<float*>(base + o_freq), T, half,
                              reinterpret_cast<float2*>(base + o_cs), s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) {
        (void)hipFree(b->blob);
        delete b;
        return RELSERVE_ERR_HIP;
    }
    *out = b;
    return RELSERVE_OK;
}

int32_t relserve_batch_destroy(relserve_batch* b) {
    if (!b) return RELSERVE_OK;
    hipError_t e = b->blob ? hipFree(b->blob) : hipSuccess;
    delete b;
    return e == hipSuccess ? RELSERVE_OK : RELSERVE_ERR_HIP;
}

int32_t relserve_batch_get_info(const relserve_batch* b, relserve_batch_info* out) {
    if (!b || !out) return RELSERVE_ERR_NULL_POINTER;
    *out = b->info;
    return RELSERVE_OK;
}

int32_t relserve_workspace_bytes(const relserve_layer* L, int32_t max_tokens, size_t* out) {
    if (!L || !out) return RELSERVE_ERR_NULL_POINTER;
    if (max_tokens < 0) return RELSERVE_ERR_BAD_ARGUMENT;
    *out = carve(*L, max_tokens, nullptr).total + kAlign;
    return RELSERVE_OK;
}

int32_t relserve_kv_append(const relserve_layer* L, const relserve_batch* b, const void* k, const void* v,
                           relserve_kv_cache cache, void* stream) {
    drop_stale_hip_error();
    if (int32_t rc = check_pair(L, b)) return rc;
    if (int32_t rc = check_cache(b, cache, false)) return rc;
    if (b->dev.T == 0) return RELSERVE_OK;
    if (!k || !v) return RELSERVE_ERR_NULL_POINTER;
    hipError_t e = launch_kv_append(b->dev, k, v, cache.k_pages, cache.v_pages, L->kv_dim,
                                    static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RELSERVE_OK : RELSERVE_ERR_HIP;
}

int32_t relserve_rmsnorm(const void* x, int32_t x_is_f32, const void* w, float eps, int32_t n_rows,
                         int32_t hidden, void* out, void* stream) {
    drop_stale_hip_error();
    if (n_rows < 0 || hidden <= 0 || hidden % 8) return RELSERVE_ERR_BAD_ARGUMENT;
    if (n_rows == 0) return RELSERVE_OK;
    if (!x || !w || !out) return RELSERVE_ERR_NULL_POINTER;
    hipError_t e = launch_rmsnorm(x, x_is_f32 != 0, w, eps, n_rows, hidden, out, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RELSERVE_OK : RELSERVE_ERR_HIP;
}

namespace {
int32_t linear_entry(const void* a, const void* w, int32_t T, int32_t N, int32_t K, int32_t epilogue,
                     const void* residual, void* out, void* stream, bool packed) {
    if (T < 0 || N <= 0 || K <= 0 || K % 8 || epilogue < 0 || epilogue > 3) return RELSERVE_ERR_BAD_ARGUMENT;
    if (epilogue == 3 ? (N % 16) : (N % 4)) return RELSERVE_ERR_BAD_ARGUMENT;
    if (packed && K % 64) return RELSERVE_ERR_BAD_ARGUMENT;
    const int64_t n_rows = packed ? ((int64_t)N + 255) / 256 * 256 : N;
    if ((int64_t)T * K >= ((int64_t)1 << 31) || n_rows * K >= ((int64_t)1 << 31)) return RELSERVE_ERR_TOO_LARGE;
    if (T == 0) return RELSERVE_OK;
    if (!a || !w || !out) return RELSERVE_ERR_NULL_POINTER;
    if (epilogue == 2 && !residual) return RELSERVE_ERR_NULL_POINTER;
    hipError_t e = launch_linear(a, w, T, N, K, epilogue, residual, out, static_cast<hipStream_t>(stream), nullptr, packed);
    return e == hipSuccess ? RELSERVE_OK : RELSERVE_ERR_HIP;
}
}  // namespace

int32_t relserve_linear(const void* a, const void* w, int32_t T, int32_t N, int32_t K, int32_t epilogue,
                        const void* residual, void* out, void* stream) {
    drop_stale_hip_error();
    return linear_entry(a, w, T, N, K, epilogue, residual, out, stream, false);
}

int32_t relserve_linear_packed(const void* a, const void* w_packed, int32_t T, int32_t N, int32_t K, int32_t epilogue,
                               const void* residual, void* out, void* stream) {
    drop_stale_hip_error();
    return linear_entry(a, w_packed, T, N, K, epilogue, residual, out, stream, true);
}

int32_t relserve_packed_weight_elems(int32_t N, int32_t K, int64_t* out) {
    if (!out) return RELSERVE_ERR_NULL_POINTER;
    if (N <= 0 || K <= 0 || K % 64) return RELSERVE_ERR_BAD_ARGUMENT;
    *out = ((int64_t)N + 255) / 256 * 256 * K;
    return *out >= ((int64_t)1 << 31) ? RELSERVE_ERR_TOO_LARGE : RELSERVE_OK;
}

int32_t relserve_pack_weight(const void* w, int32_t N, int32_t K, void* out, void* stream) {
    drop_stale_hip_error();
    int64_t elems = 0;
    if (int32_t rc = relserve_packed_weight_elems(N, K, &elems)) return rc;
    if (!w || !out) return RELSERVE_ERR_NULL_POINTER;
    return launch_pack_weight(w, N, K, out, static_cast<hipStream_t>(stream)) == hipSuccess ? RELSERVE_OK
                                                                                              : RELSERVE_ERR_HIP;
}

int32_t relserve_rope_append(const relserve_layer* L, const relserve_batch* b, void* qkv,
                             relserve_kv_cache cache, void* stream) {
    drop_stale_hip_error();
    if (int32_t rc = check_pair(L, b)) return rc;
    if (int32_t rc = check_cache(b, cache, false)) return rc;
    if (b->dev.T == 0) return RELSERVE_OK;
    if (!qkv) return RELSERVE_ERR_NULL_POINTER;
    hipError_t e = launch_rope_append(b->dev, *L, qkv, cache.k_pages, cache.v_pages, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RELSERVE_OK : RELSERVE_ERR_HIP;
}

int32_t relserve_qkv_rope_append(const relserve_layer* L, const relserve_batch* b, const void* h, const void* w_qkv,
                                 void* q_out, relserve_kv_cache cache, void* stream) {
    drop_stale_hip_error();
    if (int32_t rc = check_pair(L, b)) return rc;
    if (int32_t rc = check_cache(b, cache)) return rc;
    if (b->dev.T == 0) return RELSERVE_OK;
    if (!h || !w_qkv || !q_out) return RELSERVE_ERR_NULL_POINTER;
    hipError_t e = launch_qkv_rope_append(b->dev, *L, h, w_qkv, q_out, cache.k_pages, cache.v_pages,
                                          static_cast<hipStream_t>(stream), nullptr, false, kv_format(cache));
    return e == hipSuccess ? RELSERVE_OK : RELSERVE_ERR_HIP;
}

int32_t relserve_attention(const relserve_layer* L, const relserve_batch* b, const void* q, int32_t q_pitch,
                           relserve_kv_cache cache, void* out, void* workspace, size_t workspace_bytes,
                           void* stream) {
    drop_stale_hip_error();
    if (int32_t rc = check_pair(L, b)) return rc;
    if (int32_t rc = check_cache(b, cache)) return rc;
    if (b->dev.T == 0) return RELSERVE_OK;
    if (!q || !out) return RELSERVE_ERR_NULL_POINTER;
    if (q_pitch < L->q_dim || q_pitch % 8) return RELSERVE_ERR_BAD_ARGUMENT;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kAlign)) return RELSERVE_ERR_WORKSPACE;
    Workspace w = carve(*L, b->dev.T, workspace);
    if (w.total > workspace_bytes) return RELSERVE_ERR_WORKSPACE;
    hipError_t e = launch_attention(b->dev, *L, q, q_pitch, cache.k_pages, cache.v_pages, out, w.part_o,
                                    w.part_ml, static_cast<hipStream_t>(stream), nullptr, kv_format(cache));
    return e == hipSuccess ? RELSERVE_OK : RELSERVE_ERR_HIP;
}

int32_t relserve_layer_step(const relserve_layer* L, const relserve_batch* b, const relserve_layer_weights* wt,
                            const void* x, void* y, relserve_kv_cache cache, void* workspace,
                            size_t workspace_bytes, void* stream) {
    drop_stale_hip_error();
    if (int32_t rc = check_pair(L, b)) return rc;
    if (!wt) return RELSERVE_ERR_NULL_POINTER;
    if (int32_t rc = check_cache(b, cache)) return rc;
    const int32_t T = b->dev.T;
    if (T == 0) return RELSERVE_OK;
    if (!x || !y || !wt->w_in_norm || !wt->w_qkv || !wt->w_o || !wt->w_post_norm || !wt->w_gate_up || !wt->w_down)
        return RELSERVE_ERR_NULL_POINTER;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kAlign)) return RELSERVE_ERR_WORKSPACE;
    Workspace w = carve(*L, T, workspace);
    if (w.total > workspace_bytes) return RELSERVE_ERR_WORKSPACE;
    const bool packed = wt->packed != 0;
    if (packed && (L->cfg.hidden % 64 || L->q_dim % 64 || L->cfg.mlp_dim % 64)) return RELSERVE_ERR_BAD_ARGUMENT;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const relserve_layer_config& c = L->cfg;
    relserve_layer* prof = L->profile ? const_cast<relserve_layer*>(L) : nullptr;
    hipError_t e = hipSuccess;
    auto run = [&](int slot, auto&& launch) {
        if (e != hipSuccess) return;
        profile_mark(prof, slot, s, true);
        e = launch();
        profile_mark(prof, slot, s, false);
    };
    // the GEMMs split K across workgroups (whole skinny problems, narrow outputs at mid-size T, or the
    // incomplete last round of tiles) through an fp32 scratch that they write before they read
    float* accum = w.accum;
    run(S_NORM1, [&] { return launch_rmsnorm(x, false, wt->w_in_norm, c.rms_eps, T, c.hidden, w.h, s); });
    run(S_QKV, [&] {
        return launch_qkv_rope_append(b->dev, *L, w.h, wt->w_qkv, w.q, cache.k_pages, cache.v_pages, s, accum, packed,
                                      kv_format(cache));
    });
    if (e == hipSuccess)
        e = launch_attention(b->dev, *L, w.q, L->q_dim, cache.k_pages, cache.v_pages, w.attn, w.part_o,
                             w.part_ml, s, prof, kv_format(cache));
    run(S_O, [&] { return launch_linear(w.attn, wt->w_o, T, c.hidden, L->q_dim, 1, x, w.x1, s, accum, packed); });
    run(S_NORM2, [&] { return launch_rmsnorm(w.x1, true, wt->w_post_norm, c.rms_eps, T, c.hidden, w.h, s); });
    run(S_GU, [&] {
        return launch_linear(w.h, wt->w_gate_up, T, 2 * c.mlp_dim, c.hidden, 3, nullptr, w.act, s, accum, packed);
    });
    run(S_DOWN, [&] { return launch_linear(w.act, wt->w_down, T, c.hidden, c.mlp_dim, 2, w.x1, y, s, accum, packed); });
    return e == hipSuccess ? RELSERVE_OK : RELSERVE_ERR_HIP;
}

int32_t relserve_layer_step_w8a8(const relserve_layer* L, const relserve_batch* b, const relserve_layer_weights_w8a8* wt,
                                 const void* x, void* y, relserve_kv_cache cache, void* workspace,
                                 size_t workspace_bytes, void* stream) {
    drop_stale_hip_error();
    if (int32_t rc = check_pair(L, b)) return rc;
    if (!wt) return RELSERVE_ERR_NULL_POINTER;
    if (int32_t rc = check_cache(b, cache)) return rc;
    const relserve_layer_config& c = L->cfg;
    if (c.hidden % 128 || L->q_dim % 128 || c.mlp_dim % 128) return RELSERVE_ERR_BAD_ARGUMENT;
    for (float a : {wt->a_qkv, wt->a_o, wt->a_gate_up, wt->a_down})
        if (!(a > 0.0f) || !std::isfinite(a)) return RELSERVE_ERR_BAD_ARGUMENT;
    const int32_t T = b->dev.T;
    if (T == 0) return RELSERVE_OK;
    if (!x || !y || !wt->w_in_norm || !wt->w_qkv || !wt->w_o || !wt->w_post_norm || !wt->w_gate_up || !wt->w_down ||
        !wt->s_qkv || !wt->s_o || !wt->s_gate_up || !wt->s_down)
        return RELSERVE_ERR_NULL_POINTER;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kAlign)) return RELSERVE_ERR_WORKSPACE;
    Workspace w = carve(*L, T, workspace);   // the 16-bit step's buffers hold the codes too (half of each is used)
    if (w.total > workspace_bytes) return RELSERVE_ERR_WORKSPACE;
    const bool packed = wt->packed != 0;

    hipStream_t s = static_cast<hipStream_t>(stream);
    relserve_layer* prof = L->profile ? const_cast<relserve_layer*>(L) : nullptr;
    hipError_t e = hipSuccess;
    auto run = [&](int slot, auto&& launch) {
        if (e != hipSuccess) return;
        profile_mark(prof, slot, s, true);
        e = launch();
        profile_mark(prof, slot, s, false);
    };
    float* accum = w.accum;
    const CodeScales qkv{wt->s_qkv, wt->a_qkv, 0.0f}, o{wt->s_o, wt->a_o, 0.0f}, gu{wt->s_gate_up, wt->a_gate_up, wt->a_down},
        down{wt->s_down, wt->a_down, 0.0f};
    run(S_NORM1, [&] { return launch_rmsnorm(x, false, wt->w_in_norm, c.rms_eps, T, c.hidden, w.h, s, nullptr, wt->a_qkv); });
    run(S_QKV, [&] {
        return launch_qkv_rope_append(b->dev, *L, w.h, wt->w_qkv, w.q, cache.k_pages, cache.v_pages, s, accum, packed,
                                      kv_format(cache), &qkv);
    });
    if (e == hipSuccess)
        e = launch_attention(b->dev, *L, w.q, L->q_dim, cache.k_pages, cache.v_pages, w.attn, w.part_o,
                             w.part_ml, s, prof, kv_format(cache));
    // the attention output exists as bf16; its codes go where the rotated queries were (read by now)
    run(S_QUANT, [&] { return launch_quantise_bf16(w.attn, (int64_t)T * L->q_dim, wt->a_o, w.q, s); });
    run(S_O, [&] { return launch_linear(w.q, wt->w_o, T, c.hidden, L->q_dim, 1, x, w.x1, s, accum, packed, &o); });
    run(S_NORM2, [&] { return launch_rmsnorm(w.x1, true, wt->w_post_norm, c.rms_eps, T, c.hidden, w.h, s, nullptr, wt->a_gate_up); });
    run(S_GU, [&] {
        return launch_linear(w.h, wt->w_gate_up, T, 2 * c.mlp_dim, c.hidden, 3, nullptr, w.act, s, accum, packed, &gu);
    });
    run(S_DOWN, [&] { return launch_linear(w.act, wt->w_down, T, c.hidden, c.mlp_dim, 2, w.x1, y, s, accum, packed, &down); });
    return e == hipSuccess ? RELSERVE_OK : RELSERVE_ERR_HIP;
}

int32_t relserve_rmsnorm_codes(const void* x, int32_t x_is_f32, const void* w, float eps, int32_t n_rows,
                               int32_t hidden, float scale, void* out, void* stream) {
    drop_stale_hip_error();
    if (n_rows < 0 || hidden <= 0 || hidden % 8 || !(scale > 0.0f) || !std::isfinite(scale)) return RELSERVE_ERR_BAD_ARGUMENT;
    if (n_rows == 0) return RELSERVE_OK;
    if (!x || !w || !out) return RELSERVE_ERR_NULL_POINTER;
    hipError_t e = launch_rmsnorm(x, x_is_f32 != 0, w, eps, n_rows, hidden, out, static_cast<hipStream_t>(stream), nullptr, scale);
    return e == hipSuccess ? RELSERVE_OK : RELSERVE_ERR_HIP;
}

int32_t relserve_quantise_bf16(const void* in, int64_t n, float scale, void* codes, void* stream) {
    drop_stale_hip_error();
    if (n < 0 || n % 8 || !(scale > 0.0f) || !std::isfinite(scale)) return RELSERVE_ERR_BAD_ARGUMENT;
    if (n == 0) return RELSERVE_OK;
    if (!in || !codes) return RELSERVE_ERR_NULL_POINTER;
    return launch_quantise_bf16(in, n, scale, codes, static_cast<hipStream_t>(stream)) == hipSuccess ? RELSERVE_OK : RELSERVE_ERR_HIP;
}

int32_t relserve_linear_w8a8(const void* a, const void* w, const float* w_scale, float a_scale, int32_t T, int32_t N,
                             int32_t K, int32_t epilogue, const void* residual, void* out, float out_scale,
                             int32_t packed, void* stream) {
    drop_stale_hip_error();
    if (T < 0 || N <= 0 || K <= 0 || K % 128 || epilogue < 0 || epilogue > 3) return RELSERVE_ERR_BAD_ARGUMENT;
    if (epilogue != 3 && N % 4) return RELSERVE_ERR_BAD_ARGUMENT;
    if (epilogue == 3 && N % 16) return RELSERVE_ERR_BAD_ARGUMENT;
    if (!(a_scale > 0.0f) || !std::isfinite(a_scale) || out_scale < 0.0f || !std::isfinite(out_scale)) return RELSERVE_ERR_BAD_ARGUMENT;
    if (out_scale > 0.0f && epilogue != 3) return RELSERVE_ERR_BAD_ARGUMENT;
    if (T == 0) return RELSERVE_OK;
    if (!a || !w || !w_scale || !out) return RELSERVE_ERR_NULL_POINTER;
    if (epilogue == 2 && !residual) return RELSERVE_ERR_NULL_POINTER;
    const CodeScales codes{w_scale, a_scale, out_scale};
    hipError_t e = launch_linear(a, w, T, N, K, epilogue, residual, out, static_cast<hipStream_t>(stream), nullptr, packed != 0, &codes);
    return e == hipSuccess ? RELSERVE_OK : RELSERVE_ERR_HIP;
}

int32_t relserve_static_scratch_bytes(size_t* out) {
    if (!out) return RELSERVE_ERR_NULL_POINTER;
    *out = kStaticScratchBytes;
    return RELSERVE_OK;
}

int32_t relserve_layer_step_static(const relserve_layer* L, const relserve_batch* b, const relserve_layer_weights* wt,
                                   const void* x, void* y, relserve_kv_cache cache, void* stream) {
    drop_stale_hip_error();
    if (int32_t rc = check_pair(L, b)) return rc;
    if (carve(*L, b->dev.T, nullptr).total > kStaticScratchBytes) return RELSERVE_ERR_TOO_LARGE;
    void* ws = nullptr;
    if (int32_t rc = static_scratch(&ws)) return rc;
    return relserve_layer_step(L, b, wt, x, y, cache, ws, kStaticScratchBytes, stream);
}

int32_t relserve_model_workspace_bytes(const relserve_layer* L, int32_t max_tokens, int32_t max_reqs, size_t* out) {
    if (!L || !out) return RELSERVE_ERR_NULL_POINTER;
    if (max_tokens < 0 || max_reqs < 0) return RELSERVE_ERR_BAD_ARGUMENT;
    *out = carve(*L, max_tokens, nullptr).total + align_up((size_t)max_tokens * L->cfg.hidden * 2) +
           align_up((size_t)max_reqs * L->cfg.hidden * 2) + kAlign;
    return RELSERVE_OK;
}

namespace {
// q8 != nullptr: every layer runs relserve_layer_step_w8a8 on q8[l] instead of relserve_layer_step on m->layers[l]
int32_t model_step(const relserve_layer* L, const relserve_batch* b, const relserve_model* m,
                   const relserve_layer_weights_w8a8* q8, const int32_t* token_ids, void* logits, void* workspace,
                   size_t workspace_bytes, void* stream) {
    if (int32_t rc = check_pair(L, b)) return rc;
    if (!m) return RELSERVE_ERR_NULL_POINTER;
    if (m->n_layers < 0 || m->vocab <= 0 || m->vocab % 4) return RELSERVE_ERR_BAD_ARGUMENT;
    const int32_t T = b->dev.T, B = b->dev.num_reqs, H = L->cfg.hidden;
    if (T == 0) return RELSERVE_OK;
    if (!token_ids || !logits || !m->embedding || !m->w_final_norm || !m->w_lm_head) return RELSERVE_ERR_NULL_POINTER;
    if (m->n_layers > 0 && ((!q8 && !m->layers) || !m->caches)) return RELSERVE_ERR_NULL_POINTER;
    for (int32_t l = 0; l < m->n_layers; ++l) {
        if (!q8) {
            const relserve_layer_weights& w = m->layers[l];
            if (!w.w_in_norm || !w.w_qkv || !w.w_o || !w.w_post_norm || !w.w_gate_up || !w.w_down)
                return RELSERVE_ERR_NULL_POINTER;
        }
        if (int32_t rc = check_cache(b, m->caches[l])) return rc;
    }
    if ((int64_t)m->vocab * H >= ((int64_t)1 << 31)) return RELSERVE_ERR_TOO_LARGE;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kAlign)) return RELSERVE_ERR_WORKSPACE;
    const size_t layer_ws = carve(*L, T, nullptr).total;
    const size_t x_bytes = align_up((size_t)T * H * 2), last_bytes = align_up((size_t)B * H * 2);
    if (layer_ws + x_bytes + last_bytes > workspace_bytes) return RELSERVE_ERR_WORKSPACE;
    char* x = static_cast<char*>(workspace) + layer_ws;
    char* h_last = x + x_bytes;

    hipStream_t s = static_cast<hipStream_t>(stream);
    if (launch_embedding(token_ids, m->embedding, m->vocab, H, T, x, s) != hipSuccess) return RELSERVE_ERR_HIP;
    for (int32_t l = 0; l < m->n_layers; ++l) {   // the residual stream stays in x, rounded to bf16 between layers
        const int32_t rc = q8 ? relserve_layer_step_w8a8(L, b, &q8[l], x, x, m->caches[l], workspace, layer_ws, stream)
                              : relserve_layer_step(L, b, &m->layers[l], x, x, m->caches[l], workspace, layer_ws, stream);
        if (rc) return rc;
    }
    if (launch_rmsnorm(x, false, m->w_final_norm, L->cfg.rms_eps, B, H, h_last, s, b->dev.last_tok) != hipSuccess)
        return RELSERVE_ERR_HIP;
    if (launch_linear(h_last, m->w_lm_head, B, m->vocab, H, 1, nullptr, logits, s) != hipSuccess)
        return RELSERVE_ERR_HIP;
    return RELSERVE_OK;
}
}  // namespace

int32_t relserve_model_step(const relserve_layer* L, const relserve_batch* b, const relserve_model* m,
                            const int32_t* token_ids, void* logits, void* workspace, size_t workspace_bytes,
                            void* stream) {
    drop_stale_hip_error();
    return model_step(L, b, m, nullptr, token_ids, logits, workspace, workspace_bytes, stream);
}

int32_t relserve_model_step_w8a8(const relserve_layer* L, const relserve_batch* b, const relserve_model* m,
                                 const relserve_layer_weights_w8a8* layers, const int32_t* token_ids, void* logits,
                                 void* workspace, size_t workspace_bytes, void* stream) {
    drop_stale_hip_error();
    if (!layers) return RELSERVE_ERR_NULL_POINTER;
    return model_step(L, b, m, layers, token_ids, logits, workspace, workspace_bytes, stream);
}

int32_t relserve_greedy_sample(const void* logits, int32_t n_rows, int32_t vocab, int32_t* next_token, void* stream) {
    drop_stale_hip_error();
    if (n_rows < 0 || vocab <= 0) return RELSERVE_ERR_BAD_ARGUMENT;
    if (n_rows == 0) return RELSERVE_OK;
    if (!logits || !next_token) return RELSERVE_ERR_NULL_POINTER;
    if (reinterpret_cast<uintptr_t>(logits) % 4) return RELSERVE_ERR_BAD_ARGUMENT;
    return launch_greedy_sample(static_cast<const float*>(logits), n_rows, vocab, next_token,
                                static_cast<hipStream_t>(stream)) == hipSuccess
               ? RELSERVE_OK
               : RELSERVE_ERR_HIP;
}

int32_t relserve_peak_probe_mfma(void* sink, int32_t iters, double* flops, void* stream) {
    drop_stale_hip_error();
    if (!sink || !flops) return RELSERVE_ERR_NULL_POINTER;
    if (iters <= 0) return RELSERVE_ERR_BAD_ARGUMENT;
    *flops = 256.0 * 4.0 * iters * 16.0 * 32768.0;
    return launch_peak_mfma(static_cast<float*>(sink), iters, static_cast<hipStream_t>(stream)) == hipSuccess
               ? RELSERVE_OK
               : RELSERVE_ERR_HIP;
}

int32_t relserve_peak_probe_stream(const void* src, size_t bytes, void* sink, void* stream) {
    drop_stale_hip_error();
    if (!src || !sink) return RELSERVE_ERR_NULL_POINTER;
    if (bytes < 16 || (reinterpret_cast<uintptr_t>(src) % 16)) return RELSERVE_ERR_BAD_ARGUMENT;
    return launch_peak_stream(src, (int64_t)bytes, static_cast<uint32_t*>(sink), static_cast<hipStream_t>(stream)) ==
                   hipSuccess
               ? RELSERVE_OK
               : RELSERVE_ERR_HIP;
}

int32_t relserve_peak_probe_stream_pattern(const void* src, size_t bytes, int32_t pattern, void* sink, void* stream) {
    drop_stale_hip_error();
    if (!src || !sink) return RELSERVE_ERR_NULL_POINTER;
    if (bytes < 32768 || (reinterpret_cast<uintptr_t>(src) % 16) || pattern < 0 || pattern > 4) return RELSERVE_ERR_BAD_ARGUMENT;
    return launch_peak_stream_pattern(src, (int64_t)bytes, pattern, static_cast<uint32_t*>(sink), static_cast<hipStream_t>(stream)) ==
                   hipSuccess
               ? RELSERVE_OK
               : RELSERVE_ERR_HIP;
}

int32_t relserve_debug_force_gemm_plan(int32_t tile, int32_t tail_splits) {
    if (tile < -1 || tile > 4 || tail_splits < 0 || tail_splits > 8) return RELSERVE_ERR_BAD_ARGUMENT;
    gemm_force_plan(tile, tail_splits);
    return RELSERVE_OK;
}

// ---- profiling ---------------------------------------------------------------------------
const char* relserve_profile_slot_name(int32_t slot) {
    return (slot >= 0 && slot < RELSERVE_PROFILE_SLOTS) ? kSlotNames[slot] : "";
}

int32_t relserve_profile_enable(relserve_layer* L, int32_t slot_mask) {
    if (!L) return RELSERVE_ERR_NULL_POINTER;
    L->profile = static_cast<uint32_t>(slot_mask);
    return RELSERVE_OK;
}

int32_t relserve_profile_read(relserve_layer* L, double* ms_sum, int64_t* launches, int32_t reset) {
    if (!L) return RELSERVE_ERR_NULL_POINTER;
    int32_t rc = RELSERVE_OK;
    if (!L->pending.empty()) {
        if (hipStreamSynchronize(L->pending_stream) != hipSuccess) rc = RELSERVE_ERR_HIP;
        for (auto& p : L->pending) {
            float ms = 0.f;
            if (rc == RELSERVE_OK && hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) {
                L->ms_sum[p.slot] += ms;
                L->launches[p.slot] += 1;
            }
            L->event_pool.push_back(p.a);
            L->event_pool.push_back(p.b);
        }
        L->pending.clear();
    }
    for (int i = 0; i < RELSERVE_PROFILE_SLOTS; ++i) {
        if (ms_sum) ms_sum[i] = L->ms_sum[i];
        if (launches) launches[i] = L->launches[i];
        if (reset) L->ms_sum[i] = 0, L->launches[i] = 0;
    }
    return rc;
}

}  // extern "C"

void relserve::profile_mark(relserve_layer* L, int slot, hipStream_t s, bool begin) {
    if (!L || !((L->profile >> slot) & 1u)) return;
    if (begin) {
        relserve_layer::Pending p{slot, nullptr, nullptr};
        auto get = [&](hipEvent_t* e) {
            if (!L->event_pool.empty()) {
                *e = L->event_pool.back();
                L->event_pool.pop_back();
                return true;
            }
            return hipEventCreate(e) == hipSuccess;
        };
        if (!get(&p.a) || !get(&p.b)) return;
        (void)hipEventRecord(p.a, s);
        L->pending.push_back(p);
        L->pending_stream = s;
    } else if (!L->pending.empty() && L->pending.back().slot == slot) {
        (void)hipEventRecord(L->pending.back().b, s);
    }
}
