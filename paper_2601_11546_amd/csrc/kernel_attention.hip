// Causal softmax attention over the paged KV cache (Eq. 4, and Eq. 5 before W_o) with bf16
// MFMA and an online (running max / running sum) softmax.
//
// One workgroup = one attention item (a set of query rows that read the same run of keys
// through one block-table row) x one kv head.  A "row" is (query token, query head of the kv
// head's group), so grouped-query heads share every K/V tile that is staged.
//
// Scores are computed transposed, S^T = K Q^T (keys on the MFMA row index, query rows on the
// column index): a lane then owns ONE query row (lane % 32) and 16 of each 32 keys, so the
// row max / row sum are in-register reductions plus one exchange with lane ^ 32, and the
// probabilities are already laid out as the B operand of O^T = V^T P^T.  V is transposed on
// its way into LDS (two keys packed per 32-bit write, 16-byte column groups XOR-swizzled).
//
// Three passes use the same kernel:
//   prefix : rows = all query tokens of the requests sharing a template prefix, keys = the
//            prefix pages (read once per group), no mask; stores the running state
//            (unnormalised O, max, sum) per (token, head);
//   tile   : rows = consecutive query tokens of one request (prefill), keys = the request's
//            own keys after the shared prefix, causal; continues from the stored state;
//   split  : decode rows (one token); same as tile.
#include "device_utils.h"
#include "relserve_internal.h"

namespace relserve {

namespace {

constexpr int BLOCK_N = 64;  // keys per staged block

struct AttnArgs {
    const AttnItem* items;
    const int32_t* attn_tok;
    const int32_t* tok_pos;
    const int32_t* block_table;
    const uint16_t* q;
    const uint16_t* k_pages;
    const uint16_t* v_pages;
    uint16_t* out;
    float* part_o;
    float* part_ml;
    int32_t max_blocks, page_shift, page_mask;
    int32_t q_pitch, n_q, n_kv, group;
    float scale_log2;  // log2(e) / sqrt(d)
};

template <int D>
struct Smem {
    static constexpr int K_STRIDE = (D + 8) * 2;           // bytes per key row (16-byte pad)
    static constexpr int K_BYTES = BLOCK_N * K_STRIDE;
    static constexpr int V_STRIDE = (BLOCK_N + 8) * 2;     // bytes per d row of V^T (36 dwords)
    static constexpr int V_BYTES = D * V_STRIDE;
    static constexpr int STAGE = K_BYTES + V_BYTES;
};

template <int D>
__global__ void __launch_bounds__(256) attn_kernel(AttnArgs p) {
    using SM = Smem<D>;
    constexpr int CH = D / 8;            // 16-byte chunks per K/V row
    constexpr int K_IT = CH / 4;         // K chunks per thread per block
    constexpr int V_IT = CH / 8;         // V key pairs per thread per block
    constexpr int ROWS_PER_PASS = 256 / CH;
    constexpr int KS = D / 16;           // MFMA k steps over the head dimension
    constexpr int TD = D / 32;           // 32-row tiles of O^T
    extern __shared__ __align__(16) unsigned char smem[];

    const AttnItem it = p.items[blockIdx.x];
    const int kvh = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;

    // ---- this lane's query row
    const int R = wave * 32 + l32;
    const bool valid = R < it.n_tok * p.group;
    const int ti = R / p.group;
    const int hq = kvh * p.group + (R - ti * p.group);
    const int tok = valid ? p.attn_tok[it.tok_off + ti] : 0;
    int klim = it.key_end;  // first key this row does NOT see
    if (valid && (it.flags & ITEM_CAUSAL)) klim = min(klim, p.tok_pos[tok] + 1);
    int wave_klim_max = klim, wave_klim_min = klim;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        wave_klim_max = max(wave_klim_max, __shfl_xor(wave_klim_max, o, 64));
        wave_klim_min = min(wave_klim_min, __shfl_xor(wave_klim_min, o, 64));
    }
    const bool wave_active = wave * 32 < it.n_tok * p.group;

    bf16x8_t qf[KS];
    {
        const uint16_t* qrow = p.q + (int64_t)tok * p.q_pitch + hq * D + 8 * g;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            qf[ks] = as_bf16x8(valid ? *reinterpret_cast<const uint4*>(qrow + 16 * ks) : make_uint4(0, 0, 0, 0));
    }

    // ---- running state
    float m_run = -INFINITY, l_run = 0.f;
    f32x16_t o_acc[TD];
#pragma unroll
    for (int td = 0; td < TD; ++td)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[td][r] = 0.f;
    const int64_t row_id = (int64_t)tok * p.n_q + hq;
    if ((it.flags & ITEM_INIT_PARTIAL) && valid) {
        const float2 ml = *reinterpret_cast<const float2*>(p.part_ml + row_id * 2);
        m_run = ml.x;
        l_run = g == 0 ? ml.y : 0.f;
        const float* po = p.part_o + row_id * D + 4 * g;
#pragma unroll
        for (int td = 0; td < TD; ++td)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const float4 v = *reinterpret_cast<const float4*>(po + 32 * td + 8 * q4);
                o_acc[td][4 * q4 + 0] = v.x; o_acc[td][4 * q4 + 1] = v.y;
                o_acc[td][4 * q4 + 2] = v.z; o_acc[td][4 * q4 + 3] = v.w;
            }
    }

    // ---- staging: K rows as they are, V transposed
    const int32_t* bt = p.block_table + (int64_t)it.bt_req * p.max_blocks;
    const int kc = tid % CH, krow0 = tid / CH;
    uint4 k_reg[K_IT], v_reg[V_IT][2];
    auto slot_of = [&](int key) -> int64_t {
        return ((int64_t)bt[key >> p.page_shift] << p.page_shift) + (key & p.page_mask);
    };
    auto stage_load = [&](int kb0) {
#pragma unroll
        for (int i = 0; i < K_IT; ++i) {
            const int key = kb0 + krow0 + ROWS_PER_PASS * i;
            k_reg[i] = make_uint4(0, 0, 0, 0);
            if (key < it.key_end)
                k_reg[i] = *reinterpret_cast<const uint4*>(p.k_pages + (slot_of(key) * p.n_kv + kvh) * D + kc * 8);
        }
#pragma unroll
        for (int i = 0; i < V_IT; ++i) {
            const int key = kb0 + 2 * (krow0 + ROWS_PER_PASS * i);
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                v_reg[i][e] = make_uint4(0, 0, 0, 0);  // keys past the end contribute exact zeros
                if (key + e < it.key_end)
                    v_reg[i][e] = *reinterpret_cast<const uint4*>(p.v_pages + (slot_of(key + e) * p.n_kv + kvh) * D + kc * 8);
            }
        }
    };
    auto stage_store = [&](int buf) {
        unsigned char* sk = smem + buf * SM::STAGE;
        unsigned char* sv = sk + SM::K_BYTES;
#pragma unroll
        for (int i = 0; i < K_IT; ++i)
            *reinterpret_cast<uint4*>(sk + (krow0 + ROWS_PER_PASS * i) * SM::K_STRIDE + kc * 16) = k_reg[i];
#pragma unroll
        for (int i = 0; i < V_IT; ++i) {
            const int pi = krow0 + ROWS_PER_PASS * i;                             // key pair index 0..31
            const int kp = (pi & ~6) | ((pi & 2) << 1) | ((pi & 4) >> 1);         // swap key bits 2 and 3
            const uint32_t e[4] = {v_reg[i][0].x, v_reg[i][0].y, v_reg[i][0].z, v_reg[i][0].w};
            const uint32_t o[4] = {v_reg[i][1].x, v_reg[i][1].y, v_reg[i][1].z, v_reg[i][1].w};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int d = 8 * kc + j;
                const uint32_t ev = (j & 1) ? (e[j >> 1] >> 16) : (e[j >> 1] & 0xffffu);
                const uint32_t ov = (j & 1) ? (o[j >> 1] & 0xffff0000u) : (o[j >> 1] << 16);
                const int col = (((kp >> 2) ^ (kc & 7)) << 2) | (kp & 3);          // dword column, swizzled
                *reinterpret_cast<uint32_t*>(sv + d * SM::V_STRIDE + col * 4) = ev | ov;
            }
        }
    };

    const int n_blocks = (it.key_end - it.key_begin + BLOCK_N - 1) / BLOCK_N;
    if (n_blocks > 0) {
        stage_load(it.key_begin);
        stage_store(0);
    }
    __syncthreads();
    for (int b = 0; b < n_blocks; ++b) {
        const int kb0 = it.key_begin + b * BLOCK_N;
        const bool more = b + 1 < n_blocks;
        if (more) stage_load(kb0 + BLOCK_N);
        if (wave_active && kb0 < wave_klim_max) {
            const unsigned char* sk = smem + (b & 1) * SM::STAGE;
            const unsigned char* sv = sk + SM::K_BYTES;
            // S^T = K Q^T for two 32-key tiles
            f32x16_t s[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[t][r] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8_t kf = as_bf16x8(*reinterpret_cast<const uint4*>(
                        sk + (32 * t + l32) * SM::K_STRIDE + (2 * ks + g) * 16));
                    s[t] = mfma_32x32x16(kf, qf[ks], s[t]);
                }
            }
            // scale to log2 units, mask, running max
            const bool need_mask = kb0 + BLOCK_N > wave_klim_min;
            float mx = -INFINITY;
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float v = s[t][r] * p.scale_log2;
                    if (need_mask) {
                        const int key = kb0 + 32 * t + 8 * (r >> 2) + 4 * g + (r & 3);
                        if (key >= klim) v = -INFINITY;
                    }
                    s[t][r] = v;
                    mx = fmaxf(mx, v);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run, mx);
            const float m_use = m_new == -INFINITY ? 0.f : m_new;   // a row that has seen no key yet
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
            m_run = m_new;
            float psum = 0.f;
            bf16x8_t pf[2][2];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    uint32_t w[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float p0 = __builtin_amdgcn_exp2f(s[t][8 * h + 2 * j] - m_use);
                        const float p1 = __builtin_amdgcn_exp2f(s[t][8 * h + 2 * j + 1] - m_use);
                        psum += p0 + p1;
                        w[j] = pack_bf16x2(p0, p1);
                    }
                    pf[t][h] = as_bf16x8(make_uint4(w[0], w[1], w[2], w[3]));
                }
            l_run = l_run * alpha + psum;
            if (__any(alpha != 1.0f)) {
#pragma unroll
                for (int td = 0; td < TD; ++td)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o_acc[td][r] *= alpha;
            }
            // O^T += V^T P^T
#pragma unroll
            for (int td = 0; td < TD; ++td) {
                const int d = 32 * td + l32;
                const unsigned char* vrow = sv + d * SM::V_STRIDE;
                const int sw = (d >> 3) & 7;
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int cg = (4 * t + 2 * h + g) ^ sw;
                        const bf16x8_t vf = as_bf16x8(*reinterpret_cast<const uint4*>(vrow + cg * 16));
                        o_acc[td] = mfma_32x32x16(vf, pf[t][h], o_acc[td]);
                    }
            }
        }
        if (more) stage_store((b + 1) & 1);
        __syncthreads();
    }

    if (!valid) return;
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if (it.flags & ITEM_WRITE_PARTIAL) {
        if (g == 0) *reinterpret_cast<float2*>(p.part_ml + row_id * 2) = make_float2(m_run, l_tot);
        float* po = p.part_o + row_id * D + 4 * g;
#pragma unroll
        for (int td = 0; td < TD; ++td)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                *reinterpret_cast<float4*>(po + 32 * td + 8 * q4) =
                    make_float4(o_acc[td][4 * q4], o_acc[td][4 * q4 + 1], o_acc[td][4 * q4 + 2], o_acc[td][4 * q4 + 3]);
    } else {
        const float inv = 1.0f / l_tot;
        uint16_t* orow = p.out + row_id * D + 4 * g;
#pragma unroll
        for (int td = 0; td < TD; ++td)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                *reinterpret_cast<uint2*>(orow + 32 * td + 8 * q4) =
                    make_uint2(pack_bf16x2(o_acc[td][4 * q4] * inv, o_acc[td][4 * q4 + 1] * inv),
                               pack_bf16x2(o_acc[td][4 * q4 + 2] * inv, o_acc[td][4 * q4 + 3] * inv));
    }
}

hipError_t launch_items(const AttnArgs& base, const AttnItem* items, int32_t n_items, int32_t d, hipStream_t s) {
    if (n_items == 0) return hipSuccess;
    AttnArgs p = base;
    p.items = items;
    const dim3 grid(n_items, p.n_kv);
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_kernel<128>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 2 * Smem<128>::STAGE);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_kernel<64>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 2 * Smem<64>::STAGE);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    if (d == 128)
        attn_kernel<128><<<grid, dim3(256), 2 * Smem<128>::STAGE, s>>>(p);
    else
        attn_kernel<64><<<grid, dim3(256), 2 * Smem<64>::STAGE, s>>>(p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attention(const BatchDev& b, const relserve_layer& L, const void* q, int32_t q_pitch,
                            const void* k_pages, const void* v_pages, void* out, float* part_o, float* part_ml,
                            hipStream_t s, relserve_layer* prof) {
    AttnArgs p{};
    p.attn_tok = b.attn_tok;
    p.tok_pos = b.tok_pos;
    p.block_table = b.block_table;
    p.q = static_cast<const uint16_t*>(q);
    p.k_pages = static_cast<const uint16_t*>(k_pages);
    p.v_pages = static_cast<const uint16_t*>(v_pages);
    p.out = static_cast<uint16_t*>(out);
    p.part_o = part_o;
    p.part_ml = part_ml;
    p.max_blocks = b.max_blocks;
    p.page_shift = __builtin_ctz((unsigned)L.cfg.page_size);
    p.page_mask = L.cfg.page_size - 1;
    p.q_pitch = q_pitch;
    p.n_q = L.cfg.n_q_heads;
    p.n_kv = L.cfg.n_kv_heads;
    p.group = L.group;
    p.scale_log2 = (float)(1.4426950408889634 / sqrt((double)L.cfg.head_dim));
    const int d = L.cfg.head_dim;
    hipError_t e = hipSuccess;
    struct Pass { int slot; const AttnItem* items; int32_t n; };
    const Pass passes[3] = {{3, b.items_prefix, b.n_items_prefix},
                            {4, b.items_tile, b.n_items_tile},
                            {5, b.items_split, b.n_items_split}};
    for (const Pass& ps : passes) {
        if (e != hipSuccess || ps.n == 0) continue;
        profile_mark(prof, ps.slot, s, true);
        e = launch_items(p, ps.items, ps.n, d, s);
        profile_mark(prof, ps.slot, s, false);
    }
    return e;
}

}  // namespace relserve
