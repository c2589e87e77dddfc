// Host boundary of the layer-step library under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).
// relserve_api.hip and duration_model.hip are compiled with the sanitizers on their host side and linked with
// this driver; the kernel launchers they call are stubbed out below, so no device is touched.  The driver
// feeds the host-only entry points valid, malformed and randomly mutated inputs; a wrong status ends it
// with a message, a memory or arithmetic fault ends it through the sanitizer.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "relserve_internal.h"

namespace relserve {
hipError_t launch_rope_table(const int32_t*, const float*, int32_t, int32_t, float2*, hipStream_t) { return hipSuccess; }
hipError_t launch_rmsnorm(const void*, bool, const void*, float, int32_t, int32_t, void*, hipStream_t, const int32_t*, float) { return hipSuccess; }
hipError_t launch_quantise_bf16(const void*, int64_t, float, void*, hipStream_t) { return hipSuccess; }
hipError_t launch_embedding(const int32_t*, const void*, int32_t, int32_t, int32_t, void*, hipStream_t) { return hipSuccess; }
hipError_t launch_greedy_sample(const float*, int32_t, int32_t, int32_t*, hipStream_t) { return hipSuccess; }
hipError_t launch_kv_append(const BatchDev&, const void*, const void*, void*, void*, int32_t, hipStream_t) { return hipSuccess; }
hipError_t launch_rope_append(const BatchDev&, const relserve_layer&, void*, void*, void*, hipStream_t) { return hipSuccess; }
int64_t gemm_scratch_floats(int64_t T, int64_t n_max) { return T <= SKINNY_MAX_T ? (T * n_max > 256 * 128 * 256 ? T * n_max : 256 * 128 * 256) : GEMM_TAIL_FLOATS; }
void gemm_force_plan(int, int) {}
hipError_t launch_linear(const void*, const void*, int32_t, int32_t, int32_t, int32_t, const void*, void*, hipStream_t, float*, bool, const CodeScales*) { return hipSuccess; }
hipError_t launch_pack_weight(const void*, int32_t, int32_t, void*, hipStream_t) { return hipSuccess; }
hipError_t launch_qkv_rope_append(const BatchDev&, const relserve_layer&, const void*, const void*, void*, void*, void*, hipStream_t, float*, bool, KvFormat, const CodeScales*) { return hipSuccess; }
hipError_t launch_attention(const BatchDev&, const relserve_layer&, const void*, int32_t, const void*, const void*, void*, float*, float*, hipStream_t, relserve_layer*, KvFormat) { return hipSuccess; }
hipError_t launch_peak_mfma(float*, int32_t, hipStream_t) { return hipSuccess; }
hipError_t launch_peak_stream(const void*, int64_t, uint32_t*, hipStream_t) { return hipSuccess; }
hipError_t launch_peak_stream_pattern(const void*, int64_t, int32_t, uint32_t*, hipStream_t) { return hipSuccess; }
}  // namespace relserve

static uint64_t g_rng = 0x9e3779b97f4a7c15ull;
static uint32_t rnd() { g_rng = g_rng * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(g_rng >> 33); }
static int rnd_in(int lo, int hi) { return lo + (int)(rnd() % (uint32_t)(hi - lo + 1)); }

#define EXPECT(cond) do { if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

struct Desc {
    std::vector<int32_t> q_start, ctx, bt, pid, plen;
    int32_t max_blocks = 0, num_pages = 0;
    relserve_batch_desc view() const {
        relserve_batch_desc d{};
        d.num_reqs = (int32_t)ctx.size();
        d.max_blocks = max_blocks;
        d.q_start = q_start.data();
        d.ctx_len = ctx.data();
        d.block_table = bt.data();
        d.prefix_id = pid.empty() ? nullptr : pid.data();
        d.num_prefixes = (int32_t)plen.size();
        d.prefix_len = plen.data();
        d.num_pages = num_pages;
        return d;
    }
};

// A valid batch: n requests, an optional shared prefix of `shared` pages for the first `members` of them.
static Desc make_valid(int P, int n, int shared, int members) {
    Desc d;
    d.q_start.push_back(0);
    std::vector<int> blocks(n);
    int max_blocks = 1;
    for (int r = 0; r < n; ++r) {
        const bool member = r < members && shared > 0;
        const int q = rnd_in(1, 40), past = (member ? shared * P : 0) + rnd_in(0, 60);
        d.q_start.push_back(d.q_start.back() + q);
        d.ctx.push_back(past + q);
        d.pid.push_back(member ? 0 : -1);
        blocks[r] = (past + q + P - 1) / P;
        if (blocks[r] > max_blocks) max_blocks = blocks[r];
    }
    if (shared > 0) d.plen.push_back(shared * P);
    d.max_blocks = max_blocks;
    int next = 0;
    std::vector<int> prefix_pages(shared);
    for (int i = 0; i < shared; ++i) prefix_pages[i] = next++;
    d.bt.assign((size_t)n * max_blocks, 0);
    for (int r = 0; r < n; ++r) {
        int i = 0;
        if (d.pid[r] == 0)
            for (; i < shared; ++i) d.bt[(size_t)r * max_blocks + i] = prefix_pages[i];
        for (; i < blocks[r]; ++i) d.bt[(size_t)r * max_blocks + i] = next++;
    }
    d.num_pages = next + 2;
    return d;
}

static bool known_status(int32_t rc) { return rc <= 0 && rc >= -14; }

int main() {
    relserve_layer_config cfg{256, 8, 2, 64, 688, 16, 1e-5f, 10000.0f};
    EXPECT(relserve_config_validate(&cfg) == RELSERVE_OK);
    EXPECT(relserve_config_validate(nullptr) == RELSERVE_ERR_NULL_POINTER);
    {
        relserve_layer_config bad = cfg;
        bad.head_dim = 96;
        EXPECT(relserve_config_validate(&bad) == RELSERVE_ERR_BAD_CONFIG);
        bad = cfg; bad.page_size = 12;
        EXPECT(relserve_config_validate(&bad) == RELSERVE_ERR_BAD_CONFIG);
        bad = cfg; bad.n_kv_heads = 0;
        EXPECT(relserve_config_validate(&bad) == RELSERVE_ERR_BAD_CONFIG);
    }
    relserve_layer* layer = nullptr;
    EXPECT(relserve_layer_create(&cfg, &layer) == RELSERVE_OK && layer);
    size_t ws = 0;
    EXPECT(relserve_workspace_bytes(layer, 300, &ws) == RELSERVE_OK && ws > 0);
    EXPECT(relserve_workspace_bytes(layer, -1, &ws) == RELSERVE_ERR_BAD_ARGUMENT);
    EXPECT(relserve_model_workspace_bytes(layer, 300, 20, &ws) == RELSERVE_OK);
    EXPECT(std::strcmp(relserve_strerror(RELSERVE_ERR_SLOT_ALIAS), "two query tokens map to the same cache slot") == 0);

    // ---- descriptors: valid ones place every token at block_table[r][pos / P] * P + pos % P; every rule has its status
    int n_valid = 0, n_rejected = 0;
    for (int iter = 0; iter < 400; ++iter) {
        const int P = cfg.page_size, n = rnd_in(1, 12), shared = rnd_in(0, 3), members = rnd_in(2, n > 2 ? n : 2);
        Desc d = make_valid(P, n, shared, members);
        relserve_batch_desc v = d.view();
        EXPECT(relserve_batch_validate(&cfg, &v) == RELSERVE_OK);
        std::vector<int32_t> slots(d.q_start.back());
        EXPECT(relserve_batch_slots(&cfg, &v, slots.data()) == RELSERVE_OK);
        for (int r = 0; r < n; ++r) {
            const int q = d.q_start[r + 1] - d.q_start[r], past = d.ctx[r] - q;
            for (int j = 0; j < q; ++j) {
                const int pos = past + j;
                EXPECT(slots[d.q_start[r] + j] == d.bt[(size_t)r * d.max_blocks + pos / P] * P + pos % P);
            }
        }
        ++n_valid;
        // the rule table on this batch
        { Desc m = d; m.q_start[0] = 1; v = m.view(); EXPECT(relserve_batch_validate(&cfg, &v) == RELSERVE_ERR_BAD_Q_START); }
        { Desc m = d; m.q_start[1] = m.q_start[0]; v = m.view(); EXPECT(relserve_batch_validate(&cfg, &v) == RELSERVE_ERR_BAD_Q_START); }
        { Desc m = d; m.ctx[0] = (m.q_start[1] - m.q_start[0]) - 1; v = m.view(); EXPECT(relserve_batch_validate(&cfg, &v) == RELSERVE_ERR_BAD_CTX_LEN); }
        { Desc m = d; m.ctx[n - 1] = m.max_blocks * P + 1; if (m.pid[n - 1] < 0 || true) { v = m.view(); const int32_t rc = relserve_batch_validate(&cfg, &v); EXPECT(rc == RELSERVE_ERR_BLOCK_TABLE_SHORT); } }
        { Desc m = d; m.bt[0] = m.num_pages; v = m.view(); EXPECT(relserve_batch_validate(&cfg, &v) == RELSERVE_ERR_PAGE_RANGE); }
        { Desc m = d; m.bt[0] = -1; v = m.view(); EXPECT(relserve_batch_validate(&cfg, &v) == RELSERVE_ERR_PAGE_RANGE); }
        { Desc m = d; m.pid[0] = 7; v = m.view(); EXPECT(relserve_batch_validate(&cfg, &v) == RELSERVE_ERR_BAD_PREFIX); }
        if (shared > 0) {
            { Desc m = d; m.plen[0] = shared * P - 8; v = m.view(); EXPECT(relserve_batch_validate(&cfg, &v) == RELSERVE_ERR_BAD_PREFIX); }
            { Desc m = d; m.plen[0] = 4096 * P; v = m.view(); EXPECT(relserve_batch_validate(&cfg, &v) == RELSERVE_ERR_BAD_PREFIX); }
            if (members >= 2 && n >= 2) { Desc m = d; m.bt[(size_t)1 * m.max_blocks] = m.num_pages - 1; v = m.view(); EXPECT(relserve_batch_validate(&cfg, &v) == RELSERVE_ERR_BAD_PREFIX); }
        }
        { Desc m = d; m.num_pages = 1 << 28; v = m.view(); EXPECT(relserve_batch_validate(&cfg, &v) == RELSERVE_ERR_TOO_LARGE); }
        // random mutations: whatever comes back is a known status, and nothing is read out of bounds
        for (int k = 0; k < 20; ++k) {
            Desc m = d;
            switch (rnd() % 6) {
                case 0: m.q_start[rnd() % m.q_start.size()] += rnd_in(-3, 3); break;
                case 1: m.ctx[rnd() % m.ctx.size()] = rnd_in(-5, 200); break;
                case 2: m.bt[rnd() % m.bt.size()] = rnd_in(-2, m.num_pages + 1); break;
                case 3: m.pid[rnd() % m.pid.size()] = rnd_in(-2, 2); break;
                case 4: if (!m.plen.empty()) m.plen[0] = rnd_in(-16, 400); break;
                default: m.num_pages = rnd_in(0, m.num_pages); break;
            }
            // keep q_start a sequence the library may index with: it checks monotonicity before using it
            v = m.view();
            const int32_t rc = relserve_batch_validate(&cfg, &v);
            EXPECT(known_status(rc));
            if (rc != RELSERVE_OK) ++n_rejected;
        }
        // without a device the prepare call validates, then reports that there is none (or rejects the descriptor)
        relserve_batch* pb = nullptr;
        v = d.view();
        const int32_t rc = relserve_batch_prepare(layer, &v, nullptr, &pb);
        EXPECT(rc == RELSERVE_ERR_NO_DEVICE || rc == RELSERVE_OK || rc == RELSERVE_ERR_HIP);
        if (pb) relserve_batch_destroy(pb);
    }
    EXPECT(n_valid == 400 && n_rejected > 1000);
    {   // the empty batch
        int32_t q0 = 0;
        relserve_batch_desc e{};
        e.q_start = &q0;
        e.num_pages = 4;
        e.max_blocks = 1;
        EXPECT(relserve_batch_validate(&cfg, &e) == RELSERVE_OK);
        e.q_start = nullptr;
        EXPECT(relserve_batch_validate(&cfg, &e) == RELSERVE_ERR_NULL_POINTER);
    }

    // ---- quantised-projection stages: every argument rule has its status before anything is launched
    {
        unsigned char buf[64] = {0};
        float sc[16] = {1.f};
        EXPECT(relserve_linear_w8a8(buf, buf, sc, 1.0f, 4, 8, 128, 1, nullptr, buf, 0.0f, 0, nullptr) == RELSERVE_OK);       // stub launcher
        EXPECT(relserve_linear_w8a8(buf, buf, sc, 1.0f, 4, 8, 192, 1, nullptr, buf, 0.0f, 0, nullptr) == RELSERVE_ERR_BAD_ARGUMENT);
        EXPECT(relserve_linear_w8a8(buf, buf, sc, 0.0f, 4, 8, 128, 1, nullptr, buf, 0.0f, 0, nullptr) == RELSERVE_ERR_BAD_ARGUMENT);
        EXPECT(relserve_linear_w8a8(buf, buf, sc, -1.0f, 4, 8, 128, 1, nullptr, buf, 0.0f, 0, nullptr) == RELSERVE_ERR_BAD_ARGUMENT);
        EXPECT(relserve_linear_w8a8(buf, buf, sc, 1.0f, 4, 8, 128, 1, nullptr, buf, 1.0f, 0, nullptr) == RELSERVE_ERR_BAD_ARGUMENT);   // codes out: SwiGLU only
        EXPECT(relserve_linear_w8a8(buf, buf, sc, 1.0f, 4, 6, 128, 0, nullptr, buf, 0.0f, 0, nullptr) == RELSERVE_ERR_BAD_ARGUMENT);
        EXPECT(relserve_linear_w8a8(buf, buf, sc, 1.0f, 4, 24, 128, 3, nullptr, buf, 0.0f, 0, nullptr) == RELSERVE_ERR_BAD_ARGUMENT);
        EXPECT(relserve_linear_w8a8(buf, buf, nullptr, 1.0f, 4, 8, 128, 1, nullptr, buf, 0.0f, 0, nullptr) == RELSERVE_ERR_NULL_POINTER);
        EXPECT(relserve_linear_w8a8(buf, buf, sc, 1.0f, 4, 8, 128, 2, nullptr, buf, 0.0f, 0, nullptr) == RELSERVE_ERR_NULL_POINTER);   // fp32 residual missing
        EXPECT(relserve_linear_w8a8(nullptr, nullptr, nullptr, 1.0f, 0, 8, 128, 1, nullptr, nullptr, 0.0f, 0, nullptr) == RELSERVE_OK);   // no tokens
        EXPECT(relserve_quantise_bf16(buf, 16, 1.0f, buf, nullptr) == RELSERVE_OK);
        EXPECT(relserve_quantise_bf16(buf, 12, 1.0f, buf, nullptr) == RELSERVE_ERR_BAD_ARGUMENT);
        EXPECT(relserve_quantise_bf16(buf, 16, 0.0f, buf, nullptr) == RELSERVE_ERR_BAD_ARGUMENT);
        EXPECT(relserve_quantise_bf16(nullptr, 16, 1.0f, buf, nullptr) == RELSERVE_ERR_NULL_POINTER);
        EXPECT(relserve_rmsnorm_codes(buf, 0, buf, 1e-5f, 2, 8, 1.0f, buf, nullptr) == RELSERVE_OK);
        EXPECT(relserve_rmsnorm_codes(buf, 0, buf, 1e-5f, 2, 12, 1.0f, buf, nullptr) == RELSERVE_ERR_BAD_ARGUMENT);
        EXPECT(relserve_rmsnorm_codes(buf, 0, buf, 1e-5f, 2, 8, -2.0f, buf, nullptr) == RELSERVE_ERR_BAD_ARGUMENT);
        EXPECT(relserve_layer_step_w8a8(layer, nullptr, nullptr, buf, buf, relserve_kv_cache{}, buf, 64, nullptr) == RELSERVE_ERR_NULL_POINTER);
    }

    // ---- scheduler arithmetic: random arguments, invalid ones included
    relserve_duration_model mp{2.2e-5, 8.6e-3, 0, 0}, md{4.0e-5, 6.6e-3, 0, 0};
    for (int iter = 0; iter < 3000; ++iter) {
        const int n = rnd_in(0, 60);
        std::vector<int32_t> utok(n), pb(n), dg(n), pu(n ? n : 1), gr(n ? n : 1);
        std::vector<uint8_t> dec(n);
        for (int i = 0; i < n; ++i) utok[i] = rnd_in(iter % 50 == 0 ? -1 : 0, 1500), dec[i] = rnd() & 1;
        relserve_pem_limits lim{rnd_in(iter % 40 == 0 ? -1 : 0, 9000), rnd_in(iter % 45 == 0 ? 0 : 1, 64), rnd_in(iter % 55 == 0 ? 0 : 1, 4096)};
        int32_t npre = 0, ngrp = 0;
        const int ol = rnd_in(0, 12);
        int32_t rc = relserve_batch_decompose(utok.data(), iter & 1 ? dec.data() : nullptr, n, ol, &lim, pb.data(), dg.data(), pu.data(), &npre,
                                              gr.data(), &ngrp);
        EXPECT(rc == RELSERVE_OK || rc == RELSERVE_ERR_BAD_ARGUMENT || rc == RELSERVE_ERR_NULL_POINTER);
        if (rc == RELSERVE_OK) {
            EXPECT(npre >= 0 && npre <= n && ngrp >= 0 && ngrp <= n);
            int64_t sum_p = 0, sum_u = 0;
            for (int i = 0; i < npre; ++i) sum_p += pu[i];
            for (int i = 0; i < n; ++i) sum_u += utok[i];
            EXPECT(sum_p == sum_u);                                   // every uncached token is in exactly one prefill batch
        }
        double secs = -1;
        rc = relserve_pem_estimate(utok.data(), nullptr, n, ol, &lim, &mp, &md, &secs);
        EXPECT(rc == RELSERVE_OK ? secs >= 0 : rc == RELSERVE_ERR_BAD_ARGUMENT || rc == RELSERVE_ERR_NULL_POINTER);
        int32_t taken = 0;
        int64_t toks = 0;
        rc = relserve_prefill_candidate(utok.data(), n, rnd_in(0, 5000), rnd_in(0, 20), rnd_in(0, 300), rnd_in(iter % 30 == 0 ? 0 : 1, 2000), &taken, &toks);
        EXPECT(rc == RELSERVE_OK ? (taken >= 0 && taken <= n) : rc == RELSERVE_ERR_BAD_ARGUMENT || rc == RELSERVE_ERR_NULL_POINTER);
        double prio = 0;
        rc = relserve_static_priority(utok.data(), n, ol, &mp, &md, &prio);
        EXPECT(known_status(rc));
        std::vector<int32_t> est(n ? n : 1);
        const int ns = rnd_in(1, 5);
        int32_t st[5], su[5];
        for (int i = 0; i < ns; ++i) st[i] = rnd_in(0, 900), su[i] = rnd_in(0, st[i] + (iter % 25 == 0 ? 3 : 0));
        rc = relserve_utok_estimate(utok.data(), n, st, su, ns, est.data());
        EXPECT(known_status(rc));
        int32_t running_ol[4] = {rnd_in(0, 50), rnd_in(0, 50), rnd_in(0, 50), rnd_in(0, 50)};
        relserve_aba_input in{(double)rnd_in(0, 100) * 1e-2, (double)rnd_in(0, 100) * 1e-2, rnd_in(0, 30), rnd_in(0, 30), rnd_in(0, 4000), rnd_in(0, 50),
                              rnd_in(0, 4), rnd_in(0, 9), running_ol};
        int32_t decision = -1;
        double delta = 0;
        rc = relserve_aba_decide(&in, &mp, &md, &decision, &delta);
        EXPECT(rc == RELSERVE_OK ? (decision >= 0 && decision <= 2) : rc == RELSERVE_ERR_BAD_ARGUMENT);
        int32_t reuse = -1;
        rc = relserve_priority_reuse(rnd_in(0, 9), rnd_in(0, 9), rnd_in(0, 9), &reuse);
        EXPECT(known_status(rc));
        double out = 0;
        rc = relserve_starved_priority(1.5, (double)rnd_in(0, 100), rnd_in(0, 5), 2.0, &out);
        EXPECT(known_status(rc));
    }
    {
        double u[5] = {1, 2, 3, 4, 5}, s[5] = {2.1, 3.9, 6.2, 7.8, 10.1};
        relserve_duration_model m{};
        EXPECT(relserve_duration_fit(u, s, 5, &m) == RELSERVE_OK && m.alpha > 1.9 && m.alpha < 2.1);
        EXPECT(relserve_duration_fit(u, s, 1, &m) == RELSERVE_ERR_BAD_ARGUMENT);
        EXPECT(relserve_duration_fit(nullptr, s, 5, &m) == RELSERVE_ERR_NULL_POINTER);
    }
    EXPECT(relserve_layer_destroy(layer) == RELSERVE_OK);
    std::printf("host boundary under ASan + UBSan: %d valid descriptors, %d rejected mutations, ok\n", n_valid, n_rejected);
    return 0;
}
