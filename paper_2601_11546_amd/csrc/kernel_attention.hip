// Causal softmax attention over the paged KV cache (Eq. 4, and Eq. 5 before W_o) with bf16
// MFMA and an online (running max / running sum) softmax.
//
// A "row" is (query token, query head of one kv head's group), so grouped-query heads share
// every K/V tile that is staged.  Scores are computed transposed, S^T = K Q^T (keys on the
// MFMA row index, query rows on the column index): a lane then owns ONE query row
// (lane % 32) and 16 of each 32 keys, so the row max / row sum are in-register reductions
// plus one exchange with lane ^ 32, and the probabilities are already laid out as the B
// operand of O^T = V^T P^T.  The tiled kernel keeps V row-major in LDS and transposes it in the
// LDS read (ds_read_b64_tr_b16); the decode kernel transposes V on its way into LDS.
//
// Two kernels:
//   attn_tile_kernel   one workgroup = up to 128 rows x one kv head; the four waves own 32
//                      rows each and share K/V blocks of 64 keys staged by all 256 threads.
//                      Used for the joint shared-prefix pass (rows = every query token of the
//                      requests carrying the prefix, keys = the prefix pages, read once per
//                      group; the running state is stored) and for prefill rows (keys = the
//                      request's own keys, causal, continuing from the stored state).
//   attn_decode_kernel one WAVE = one decode token x one kv head (rows = the heads of the
//                      group); each wave streams its own 32-key blocks through a private LDS
//                      region, so a workgroup needs no barrier and short contexts still fill
//                      the chip.  The four waves of a workgroup take four adjacent kv heads of
//                      one token, i.e. 1 KB of every cached row.  HBM-bound: the MFMA work is a
//                      few percent of the time.
#include <mutex>
#include <type_traits>

#include "device_utils.h"
#include "relserve_internal.h"

namespace relserve {

namespace {

struct AttnArgs {
    const AttnItem* items;
    const AttnItem* items_b;   // fused launch only: the decode items (items = the row-tiled items)
    int32_t n_items_b;
    const int32_t* attn_tok;
    const int32_t* tok_pos;
    const int32_t* block_table;
    const uint16_t* q;
    const uint16_t* k_pages;
    const uint16_t* v_pages;
    uint16_t* out;
    float* part_o;
    float* part_ml;
    int32_t n_items;
    int32_t T;                 // rows T + slot of part_o / part_ml hold the chunk partials of split decode rows
    const MergeItem* merge_items;
    int32_t max_blocks, page_shift, page_mask;
    int32_t q_pitch, n_q, n_kv, group;
    int32_t dec_by_head;   // decode workgroups take four adjacent kv heads of one token (n_kv % 4 == 0)
    float scale_log2;  // log2(e) / sqrt(d), times the key pool's scale when the cache is quantised
    float v_scale;     // the value pool's scale (1 for 16-bit pools): applied where a row is normalised
};

// Per-lane running softmax state of one query row (shared by lanes l and l ^ 32, which hold
// complementary halves of the keys and of the output columns).
template <int D>
struct RowState {
    float m, l;
    f32x16_t o[D / 32];
};

template <int D>
__device__ __forceinline__ void state_init(RowState<D>& st, const AttnArgs& p, const AttnItem& it, bool valid,
                                           int64_t row_id, int g) {
    st.m = -INFINITY;
    st.l = 0.f;
#pragma unroll
    for (int td = 0; td < D / 32; ++td)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.o[td][r] = 0.f;
    if ((it.flags & ITEM_INIT_PARTIAL) && valid) {
        const float2 ml = *reinterpret_cast<const float2*>(p.part_ml + row_id * 2);
        st.m = ml.x;
        st.l = g == 0 ? ml.y : 0.f;
        const float* po = p.part_o + row_id * D + 4 * g;
#pragma unroll
        for (int td = 0; td < D / 32; ++td)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const float4 v = *reinterpret_cast<const float4*>(po + 32 * td + 8 * q4);
                st.o[td][4 * q4 + 0] = v.x; st.o[td][4 * q4 + 1] = v.y;
                st.o[td][4 * q4 + 2] = v.z; st.o[td][4 * q4 + 3] = v.w;
            }
    }
}

template <int D>
__device__ __forceinline__ void state_store(const RowState<D>& st, const AttnArgs& p, const AttnItem& it,
                                            int64_t row_id, int g) {
    const float l_tot = st.l + __shfl_xor(st.l, 32, 64);
    if (it.flags & ITEM_WRITE_PARTIAL) {
        if (g == 0) *reinterpret_cast<float2*>(p.part_ml + row_id * 2) = make_float2(st.m, l_tot);
        float* po = p.part_o + row_id * D + 4 * g;
#pragma unroll
        for (int td = 0; td < D / 32; ++td)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                *reinterpret_cast<float4*>(po + 32 * td + 8 * q4) =
                    make_float4(st.o[td][4 * q4], st.o[td][4 * q4 + 1], st.o[td][4 * q4 + 2], st.o[td][4 * q4 + 3]);
    } else {
        const float inv = p.v_scale / l_tot;
        uint16_t* orow = p.out + row_id * D + 4 * g;
#pragma unroll
        for (int td = 0; td < D / 32; ++td)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                *reinterpret_cast<uint2*>(orow + 32 * td + 8 * q4) =
                    make_uint2(pack_bf16x2(st.o[td][4 * q4] * inv, st.o[td][4 * q4 + 1] * inv),
                               pack_bf16x2(st.o[td][4 * q4 + 2] * inv, st.o[td][4 * q4 + 3] * inv));
    }
}

// ------------------------------------------------------------------------------------------
// row-tiled kernel (prefix pass, prefill rows)
// ------------------------------------------------------------------------------------------
// K and V blocks of 64 keys go global -> LDS directly (global_load_lds_dwordx4, no register
// staging), both row-major [key][d] with XOR-swizzled 16-byte chunks:
//   K chunk c of row r sits at c ^ kswz(r): the 16 rows that 16 lanes read together (same chunk)
//     then cover all 64 banks;
//   V chunk c of row r sits at c ^ vswz(r): the four key rows x 64 bytes that one transposing read
//     of 32 lanes touches then cover all 64 banks.
// The V^T operand of O^T = V^T P^T is produced by ds_read_b64_tr_b16: within 16 lanes, lane s points
// at V[key0 + s / 4][d0 + 4 (s % 4) .. + 3] and lane i receives V[key0 + 0..3][d0 + i], i.e. four
// keys of one d, which is the MFMA operand layout (checked on the device: lane i, element e comes
// from source lane 4 e + i / 4, element i % 4).
template <int D>
struct TileSmem {
    static constexpr int BLOCK_N = 64;
    static constexpr int ROWB = D * 2;                  // bytes per key row, no padding
    static constexpr int K_BYTES = BLOCK_N * ROWB;
    static constexpr int V_BYTES = BLOCK_N * ROWB;
    static constexpr int STAGE = K_BYTES + V_BYTES;
};

template <int D>
__device__ __forceinline__ int kswz(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
template <int D>
__device__ __forceinline__ int vswz(int row) { return D == 128 ? 4 * (row & 3) : 4 * ((row >> 1) & 1); }

// 64 lanes x 16 bytes from per-lane global addresses to 1 KB of LDS starting at lds_addr.
__device__ __forceinline__ void dma16_ptr(const void* gptr, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_addr) : "memory");
}
// The same with the non-temporal hint, for keys and values that one wave reads once (decode rows): a streaming
// read of 256-byte head rows reaches 7.2 TB/s with it against 6.4 TB/s without.
__device__ __forceinline__ void dma16_ptr_nt(const void* gptr, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off nt" ::"v"(gptr), "s"(lds_addr) : "memory");
}

typedef short short4_t __attribute__((ext_vector_type(4)));

// FP8: the pools hold one byte per element (8-bit codes).  A block then goes global -> registers -> LDS: each lane loads
// the 8 bytes of the chunk it would have received directly, widens them to bf16 (exact) and stores the 16 bytes where the
// direct load would have put them, so that everything behind the staging is the 16-bit kernel.
template <int D, bool FP8>
__device__ __forceinline__ void attn_tile_body(const AttnArgs& p, int item_idx, int kvh) {
    using SM = TileSmem<D>;
    constexpr int BLOCK_N = SM::BLOCK_N;
    constexpr int CH = D / 8;                 // 16-byte chunks per K/V row
    constexpr int RPI = 64 / CH;              // rows one 1 KB wave load covers
    constexpr int IT = BLOCK_N / (4 * RPI);   // wave loads per wave, per tensor and block
    extern __shared__ __align__(16) unsigned char smem[];

    const AttnItem it = p.items[item_idx];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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

    bf16x8_t qf[D / 16];
    {
        const uint16_t* qrow = p.q + (int64_t)tok * p.q_pitch + hq * D + 8 * g;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks)
            qf[ks] = as_bf16x8(valid ? *reinterpret_cast<const uint4*>(qrow + 16 * ks) : make_uint4(0, 0, 0, 0));
    }
    const int64_t row_id = (int64_t)tok * p.n_q + hq;
    RowState<D> st;
    state_init<D>(st, p, it, valid, row_id, g);

    // ---- staging.  Wave load j of this wave fills LDS rows (4 j + wave) * RPI ..; lane l owns row
    // l / CH of those and the 16-byte slot l % CH.  Keys past the end re-read the last key: their
    // scores are masked and their probabilities are exact zeros.
    const int32_t* bt = p.block_table + (int64_t)it.bt_req * p.max_blocks;
    const int last_key = it.key_end - 1;
    const int lrow = lane / CH, lslot = lane % CH;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
    // A lookup keeps the page numbers as they were loaded; the slot arithmetic waits until the block is issued, one
    // iteration later.  (The compiler places the wait for a load in front of its first use, and it does not count the
    // direct-to-LDS loads, which sit in inline assembly: arithmetic on a page number straight after the lookup would
    // wait for every load issued before it -- the next block's keys and values -- and undo the double buffer.)
    struct Pages { int32_t page[IT]; int kb0; };
    Pages pg_cur, pg_nxt;
    auto lookup = [&](int kb0, Pages& pg) {   // block-table entries of this lane's rows
        pg.kb0 = kb0;
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            const int key = min(kb0 + (4 * j + wave) * RPI + lrow, last_key);
            pg.page[j] = bt[key >> p.page_shift];
        }
    };
    auto slot_of = [&](const Pages& pg, int j) -> int64_t {
        const int key = min(pg.kb0 + (4 * j + wave) * RPI + lrow, last_key);
        return ((int64_t)pg.page[j] << p.page_shift) + (key & p.page_mask);
    };
    auto issue = [&](int buf, const Pages& pg) {
        const uint32_t base = lds0 + buf * SM::STAGE + wave * 1024;
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            const int row = (4 * j + wave) * RPI + lrow;
            const int64_t off = (slot_of(pg, j) * p.n_kv + kvh) * D;
            dma16_ptr(p.k_pages + off + ((lslot ^ kswz<D>(row)) << 3), base + j * 4096);
            dma16_ptr(p.v_pages + off + ((lslot ^ vswz<D>(row)) << 3), base + SM::K_BYTES + j * 4096);
        }
    };
    uint2 k_raw[IT], v_raw[IT];   // FP8 only: the block on its way through registers
    auto load_raw = [&](const Pages& pg) {
        const uint8_t* k8 = reinterpret_cast<const uint8_t*>(p.k_pages);
        const uint8_t* v8 = reinterpret_cast<const uint8_t*>(p.v_pages);
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            const int row = (4 * j + wave) * RPI + lrow;
            const int64_t off = (slot_of(pg, j) * p.n_kv + kvh) * D;
            k_raw[j] = *reinterpret_cast<const uint2*>(k8 + off + ((lslot ^ kswz<D>(row)) << 3));
            v_raw[j] = *reinterpret_cast<const uint2*>(v8 + off + ((lslot ^ vswz<D>(row)) << 3));
        }
    };
    auto store_raw = [&](int buf) {
        unsigned char* base = smem + buf * SM::STAGE + wave * 1024 + lane * 16;
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            *reinterpret_cast<uint4*>(base + j * 4096) = fp8x8_to_bf16x8(k_raw[j]);
            *reinterpret_cast<uint4*>(base + SM::K_BYTES + j * 4096) = fp8x8_to_bf16x8(v_raw[j]);
        }
    };

    const int n_blocks = (it.key_end - it.key_begin + BLOCK_N - 1) / BLOCK_N;
    if (n_blocks > 0) {
        lookup(it.key_begin, pg_cur);
#pragma unroll
        for (int j = 0; j < IT; ++j) asm volatile("" ::"v"(pg_cur.page[j]));   // all of them before the first direct load (see the loop)
        if (FP8) {
            load_raw(pg_cur);
            store_raw(0);
        } else {
            issue(0, pg_cur);
        }
        lookup(min(it.key_begin + BLOCK_N, last_key), pg_nxt);
    }
    // Operand addresses inside a stage that do not change from block to block.  K: key row
    // 32 t + l32, chunk (2 ks + g) ^ kswz (the swizzle only depends on l32).  V: the transposing read
    // of (t, h, half) points lane (G, s16) at key 32 t + 16 h + 8 half + 4 (G >> 1) + s16 / 4 and at
    // d = 32 td + 16 (G & 1) + 4 (s16 % 4); its swizzle only depends on s16.
    const int G = lane >> 4, s16 = lane & 15;
    uint32_t k_off[D / 16], v_off[D / 32];
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) k_off[ks] = l32 * SM::ROWB + (((2 * ks + g) ^ kswz<D>(l32)) << 4);
    {
        const int key = 4 * (G >> 1) + (s16 >> 2);
#pragma unroll
        for (int td = 0; td < D / 32; ++td) {
            const int chunk = 4 * td + 2 * (G & 1) + ((s16 & 3) >> 1);
            v_off[td] = SM::K_BYTES + key * SM::ROWB + ((chunk ^ vswz<D>(key)) << 4) + (s16 & 1) * 8;
        }
    }
    const float scale = p.scale_log2;
    // A 32-key tile: S^T = K Q^T, online softmax in the log2 domain (the scale is folded into the
    // exponent's multiply-add; the running maximum is kept scaled), O^T += V^T P^T.
    // The three phases of a 32-key tile.  The block loop issues the score MFMAs of BOTH tiles first, so
    // that the second tile's MFMAs (and later the first tile's P V MFMAs) run while the VALU does the
    // other tile's softmax.
    // Operand reads are issued in batches ahead of the MFMAs that use them, with explicit waits: left to itself the
    // compiler keeps one fragment in flight (read, wait, MFMA, read, ...) to save registers, and every MFMA then
    // waits out an LDS round trip.
    auto read_k = [&](int t, const unsigned char* stage, bf16x8_t (&kf)[D / 16]) {
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks)
            kf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(stage + k_off[ks] + t * 32 * SM::ROWB));
    };
    auto scores = [&](const bf16x8_t (&kf)[D / 16]) {
        f32x16_t sc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) sc = mfma_32x32x16(kf[ks], qf[ks], sc);
        return sc;
    };
    auto softmax = [&](f32x16_t& sc, bool masked, int key0, bf16x8_t (&pf)[2]) {
        if (masked) {   // wave-uniform: only the blocks that straddle some row's limit pay for the mask
            const int lim = klim - key0 - 4 * g;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (8 * (r >> 2) + (r & 3) >= lim) sc[r] = -INFINITY;
        }
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sc[r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        // The reference value of the exponents only follows the running maximum when that grew by more
        // than 8 (a factor 256): probabilities then stay below 2^8, harmless in bf16 / fp32, and the
        // rescaling of the 64 output accumulators becomes rare instead of happening for some row of
        // the wave in almost every tile.
        const float m_cand = mx * scale;
        const float m_new = m_cand > st.m + 8.0f ? m_cand : st.m;
        const float m_use = m_new == -INFINITY ? 0.f : m_new;  // a row that has seen no key yet
        const float alpha = __builtin_amdgcn_exp2f(st.m - m_use);
        st.m = m_new;
        float psum = 0.f;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            uint32_t w[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[8 * h + 2 * j], scale, -m_use));
                const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[8 * h + 2 * j + 1], scale, -m_use));
                psum += p0 + p1;
                w[j] = pack_bf16x2(p0, p1);
            }
            pf[h] = as_bf16x8(make_uint4(w[0], w[1], w[2], w[3]));
        }
        st.l = st.l * alpha + psum;
        if (__any(alpha != 1.0f)) {
#pragma unroll
            for (int td = 0; td < D / 32; ++td)
#pragma unroll
                for (int r = 0; r < 16; ++r) st.o[td][r] *= alpha;
        }
    };
    // Element e of lane group g's probabilities is key 32 t + 16 h + 8 (e / 4) + 4 g + e % 4; the two
    // transposing reads fetch those keys.
    auto read_v = [&](int t, const unsigned char* stage, bf16x8_t (&vf)[D / 32][2]) {
        typedef short short8_t __attribute__((ext_vector_type(8)));
        typedef short4_t __attribute__((address_space(3))) * lds_v4;
#pragma unroll
        for (int td = 0; td < D / 32; ++td)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                unsigned char* a0 = const_cast<unsigned char*>(stage) + v_off[td] + (32 * t + 16 * h) * SM::ROWB;
                const short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(a0));
                const short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(a0 + 8 * SM::ROWB));
                const short8_t v8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                vf[td][h] = __builtin_bit_cast(bf16x8_t, v8);
            }
    };
    auto weighted_values = [&](const bf16x8_t (&vf)[D / 32][2], const bf16x8_t (&pf)[2]) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int td = 0; td < D / 32; ++td) st.o[td] = mfma_32x32x16(vf[td][h], pf[h], st.o[td]);
    };
    for (int b = 0; b < n_blocks; ++b) {
        const int kb0 = it.key_begin + b * BLOCK_N;
        // this block has landed for every wave, and every wave is done with the other buffer
        if (!FP8) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        // the page numbers looked up during the previous iteration count as used from here on: the compiler's own
        // waits for them (it does not see the direct-to-LDS loads) all fall here, where nothing is in flight, and
        // not between the loads issued below
#pragma unroll
        for (int j = 0; j < IT; ++j) asm volatile("" ::"v"(pg_nxt.page[j]));
        __syncthreads();
        if (b + 1 < n_blocks) {
            if (FP8)
                load_raw(pg_nxt);                               // into registers; stored behind this block's arithmetic
            else
                issue((b + 1) & 1, pg_nxt);
            lookup(min(kb0 + 2 * BLOCK_N, last_key), pg_nxt);   // consumed one iteration later
        }
        if (wave_active && kb0 < wave_klim_max) {
            const unsigned char* stage = smem + (b & 1) * SM::STAGE;
            const bool masked = __builtin_amdgcn_readfirstlane(kb0 + BLOCK_N > wave_klim_min);
            bf16x8_t kf0[D / 16], kf1[D / 16], vf[D / 32][2], pf[2];
            read_k(0, stage, kf0);
            read_k(1, stage, kf1);
            __builtin_amdgcn_sched_barrier(0);     // (MFMAs are no memory operations: only this keeps them behind the batch)
            asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(D / 16) : "memory");    // the first tile's keys (LDS reads return in order)
            f32x16_t sc0 = scores(kf0);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            read_v(0, stage, vf);                  // land while the second tile's scores and the first tile's softmax run
            __builtin_amdgcn_sched_barrier(0);
            f32x16_t sc1 = scores(kf1);
            __builtin_amdgcn_sched_barrier(0);
            softmax(sc0, masked, kb0, pf);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            weighted_values(vf, pf);
            __builtin_amdgcn_sched_barrier(0);
            read_v(1, stage, vf);                  // behind the MFMAs that read the first tile's values
            __builtin_amdgcn_sched_barrier(0);
            softmax(sc1, masked, kb0 + 32, pf);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            weighted_values(vf, pf);
        }
        // the other buffer is free since the barrier above: every wave had finished the previous block before it
        if (FP8 && b + 1 < n_blocks) store_raw((b + 1) & 1);
    }
    if (valid) state_store<D>(st, p, it, row_id, g);
}

// ------------------------------------------------------------------------------------------
// wave-per-item kernel (decode rows)
// ------------------------------------------------------------------------------------------
// Uses the 16x16x32 MFMA (A[i = l % 16][k = 8 (l / 16) ..+7], B[k][j = l % 16], accumulator
// register r = D[4 (l / 16) + r][l % 16]): 16 query rows are enough for the heads of one kv
// group, and accumulators, query fragments and scores take half the registers of the 32-wide
// form.  Each wave owns 32 key rows of K and of V in LDS (row-major, XOR-swizzled 16-byte chunks)
// and fills them with direct global -> LDS loads; V^T operands come from transposing LDS reads.
// One buffer per wave: eight waves per CU (D = 128) overlap each other's load and compute phases,
// and no wave ever waits for another (no barrier).
template <int D>
struct DecodeSmem {
    static constexpr int BLOCK_N = 32;
    static constexpr int ROWB = D * 2;
    static constexpr int K_BYTES = BLOCK_N * ROWB;
    static constexpr int V_BYTES = BLOCK_N * ROWB;
    static constexpr int WAVE_BYTES = K_BYTES + V_BYTES;
};
// V chunk c of key row r sits at c ^ dvswz(r): a transposing read of 64 lanes touches 16 key rows x 32 bytes,
// which this spreads over all banks twice (the minimum for 512 bytes).
template <int D>
__device__ __forceinline__ int dvswz(int row) { return D == 128 ? 2 * (row & 7) : 2 * ((row >> 1) & 3); }

template <int D, bool FP8>
__device__ __forceinline__ void attn_decode_body(const AttnArgs& p, const AttnItem* items, int n_items, int w) {
    using SM = DecodeSmem<D>;
    constexpr int CH = D / 8;                 // 16-byte chunks per K/V row
    constexpr int RPI = 64 / CH;              // rows one 1 KB wave load covers
    constexpr int IT = SM::BLOCK_N / RPI;     // wave loads per tensor and block
    constexpr int KS = D / 32, TD = D / 16;
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, gq = lane >> 4;
    // Decode workgroup w: with a multiple of four kv heads, its four waves take four ADJACENT heads of ONE token, so
    // the workgroup reads 1 KB of every key / value row where four tokens' single heads would read 256 bytes each
    // (a row is all heads of a token, back to back), and consecutive workgroups finish the row; otherwise the waves
    // take four tokens of one head.
    int item_idx, kvh;
    if (p.dec_by_head) {
        const int hg = p.n_kv >> 2;
        item_idx = w / hg;
        kvh = (w % hg) * 4 + wave;
    } else {
        const int n_wg = (n_items + 3) / 4;
        item_idx = (w % n_wg) * 4 + wave;
        kvh = w / n_wg;
    }
    if (item_idx >= n_items) return;             // whole wave leaves; this path has no workgroup barrier
    const AttnItem it = items[item_idx];
    unsigned char* sk = smem + wave * SM::WAVE_BYTES;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)sk;

    // a decode item is one token (pad0) whose last visible key is its own: klim = key_end
    const int tok = it.pad0;
    const bool valid = l16 < p.group;
    const int hq = kvh * p.group + (valid ? l16 : 0);
    const int klim = it.key_end;

    bf16x8_t qf[KS];
    {
        const uint16_t* qrow = p.q + (int64_t)tok * p.q_pitch + hq * D + 8 * gq;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            qf[ks] = as_bf16x8(valid ? *reinterpret_cast<const uint4*>(qrow + 32 * ks) : make_uint4(0, 0, 0, 0));
    }
    const int64_t row_id = (int64_t)tok * p.n_q + hq;
    float m_run = -INFINITY, l_run = 0.f;
    f32x4_t o_acc[TD];
#pragma unroll
    for (int td = 0; td < TD; ++td) o_acc[td] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    if ((it.flags & ITEM_INIT_PARTIAL) && valid) {
        const float2 ml = *reinterpret_cast<const float2*>(p.part_ml + row_id * 2);
        m_run = ml.x;
        l_run = gq == 0 ? ml.y : 0.f;
        const float* po = p.part_o + row_id * D + 4 * gq;
#pragma unroll
        for (int td = 0; td < TD; ++td) {
            const float4 v = *reinterpret_cast<const float4*>(po + 16 * td);
            o_acc[td] = f32x4_t{v.x, v.y, v.z, v.w};
        }
    }

    // ---- staging: wave load j fills rows j * RPI ..; lane l owns row l / CH of those and the 16-byte
    // slot l % CH.  Keys past the end re-read the last key: their scores are masked, their
    // probabilities exact zeros.  Block-table entries are looked up one block ahead of the loads.
    const int32_t* bt = p.block_table + (int64_t)it.bt_req * p.max_blocks;
    const int last_key = it.key_end - 1;
    const int lrow = lane / CH, lslot = lane % CH;
    // page numbers as loaded; the slot arithmetic waits until the block is issued (see the tiled kernel's lookup)
    int32_t pg[IT];
    int pg_kb0 = 0;
    auto lookup = [&](int kb0) {
        pg_kb0 = kb0;
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            const int key = min(kb0 + j * RPI + lrow, last_key);
            pg[j] = bt[key >> p.page_shift];
        }
    };
    auto slot_of = [&](int j) -> int64_t {
        const int key = min(pg_kb0 + j * RPI + lrow, last_key);
        return ((int64_t)pg[j] << p.page_shift) + (key & p.page_mask);
    };
    auto issue_k = [&]() {
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            const int row = j * RPI + lrow;
            const int64_t off = (slot_of(j) * p.n_kv + kvh) * D;
            dma16_ptr_nt(p.k_pages + off + ((lslot ^ kswz<D>(row)) << 3), lds0 + j * 1024);
        }
    };
    auto issue_v = [&]() {
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            const int row = j * RPI + lrow;
            const int64_t off = (slot_of(j) * p.n_kv + kvh) * D;
            dma16_ptr_nt(p.v_pages + off + ((lslot ^ dvswz<D>(row)) << 3), lds0 + SM::K_BYTES + j * 1024);
        }
    };
    auto issue = [&]() {
        issue_k();
        issue_v();
    };
    uint2 k_raw[IT], v_raw[IT];   // FP8 only (see attn_tile_body): the block on its way through registers
    auto load_raw = [&]() {
        const uint8_t* k8 = reinterpret_cast<const uint8_t*>(p.k_pages);
        const uint8_t* v8 = reinterpret_cast<const uint8_t*>(p.v_pages);
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            const int row = j * RPI + lrow;
            const int64_t off = (slot_of(j) * p.n_kv + kvh) * D;
            // read once: non-temporal, as the direct loads of the 16-bit path
            const uint64_t kk = __builtin_nontemporal_load(reinterpret_cast<const uint64_t*>(k8 + off + ((lslot ^ kswz<D>(row)) << 3)));
            const uint64_t vv = __builtin_nontemporal_load(reinterpret_cast<const uint64_t*>(v8 + off + ((lslot ^ dvswz<D>(row)) << 3)));
            k_raw[j] = make_uint2((uint32_t)kk, (uint32_t)(kk >> 32));
            v_raw[j] = make_uint2((uint32_t)vv, (uint32_t)(vv >> 32));
        }
    };
    auto store_raw = [&]() {
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            *reinterpret_cast<uint4*>(sk + j * 1024 + lane * 16) = fp8x8_to_bf16x8(k_raw[j]);
            *reinterpret_cast<uint4*>(sk + SM::K_BYTES + j * 1024 + lane * 16) = fp8x8_to_bf16x8(v_raw[j]);
        }
    };
    // operand addresses: K fragment (t, ks) = key row 16 t + l16, chunk 4 ks + gq; the transposing V read
    // (td, half) points lane (gq, s = l16) at key 16 half + 4 gq + s / 4 and d = 16 td + 4 (s % 4)
    uint32_t k_off[KS], v_off[TD];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) k_off[ks] = l16 * SM::ROWB + (((4 * ks + gq) ^ kswz<D>(l16)) << 4);
    {
        const int key = 4 * gq + (l16 >> 2);
#pragma unroll
        for (int td = 0; td < TD; ++td)
            v_off[td] = SM::K_BYTES + key * SM::ROWB + (((2 * td + ((l16 & 3) >> 1)) ^ dvswz<D>(key)) << 4) + (l16 & 1) * 8;
    }
    typedef short short8_t __attribute__((ext_vector_type(8)));
    typedef short4_t __attribute__((address_space(3))) * lds_v4;

    const int n_blocks = (it.key_end - it.key_begin + SM::BLOCK_N - 1) / SM::BLOCK_N;
    if (n_blocks > 0) {
        lookup(it.key_begin);
#pragma unroll
        for (int j = 0; j < IT; ++j) asm volatile("" ::"v"(pg[j]));   // all of them before the first direct load (see the loop)
        if (FP8) load_raw(); else issue();
        if (n_blocks > 1) lookup(it.key_begin + SM::BLOCK_N);
    }
    for (int b = 0; b < n_blocks; ++b) {
        const int kb0 = it.key_begin + b * SM::BLOCK_N;
        if (FP8) {
            // the block's bytes are in registers: widen them into this wave's LDS rows (the reads below follow the
            // stores in the wave's own LDS queue), then start the next block's loads
            store_raw();
            if (b + 1 < n_blocks) {
                load_raw();
                if (b + 2 < n_blocks) lookup(kb0 + 2 * SM::BLOCK_N);
            }
        } else {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the block has landed
#pragma unroll
            for (int j = 0; j < IT; ++j) asm volatile("" ::"v"(pg[j]));   // the compiler's waits for the page numbers fall here
        }

        // S^T = K Q^T for two 16-key tiles; lane holds keys kb0 + 16 t + 4 gq + r of query row l16
        f32x4_t s[2];
        bf16x8_t kf[2][KS];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                kf[t][ks] = as_bf16x8(*reinterpret_cast<const uint4*>(sk + k_off[ks] + t * 16 * SM::ROWB));
        if (!FP8) {
            // the keys are in registers: the next block's keys may overwrite them while the values are still being read
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            if (b + 1 < n_blocks) issue_k();
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            s[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) s[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[t][ks], qf[ks], s[t], 0, 0, 0);
        }
        // the block's 32 key rows of V, as the operand of O^T += V^T P^T (rows d = 16 td + l16)
        bf16x8_t vf[TD];
#pragma unroll
        for (int td = 0; td < TD; ++td) {
            const short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(sk + v_off[td]));
            const short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(sk + v_off[td] + 16 * SM::ROWB));
            vf[td] = __builtin_bit_cast(bf16x8_t, (short8_t)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
        // everything of this block is in registers: the next block may overwrite the buffer
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (!FP8 && b + 1 < n_blocks) {
            issue_v();
            if (b + 2 < n_blocks) lookup(kb0 + 2 * SM::BLOCK_N);
        }
        const bool need_mask = kb0 + SM::BLOCK_N > klim;
        float mx = -INFINITY;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float v = s[t][r] * p.scale_log2;
                if (need_mask && kb0 + 16 * t + 4 * gq + r >= klim) v = -INFINITY;
                s[t][r] = v;
                mx = fmaxf(mx, v);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
        m_run = m_new;
        float pv[8];
        float psum = 0.f;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                pv[4 * t + r] = __builtin_amdgcn_exp2f(s[t][r] - m_use);
                psum += pv[4 * t + r];
            }
        // element e of the operand: key 4 gq + e (e < 4), 16 + 4 gq + e - 4 (e >= 4), the keys the two
        // transposing reads fetched
        const bf16x8_t pf = as_bf16x8(make_uint4(pack_bf16x2(pv[0], pv[1]), pack_bf16x2(pv[2], pv[3]),
                                                 pack_bf16x2(pv[4], pv[5]), pack_bf16x2(pv[6], pv[7])));
        l_run = l_run * alpha + psum;
        if (__any(alpha != 1.0f)) {
#pragma unroll
            for (int td = 0; td < TD; ++td) o_acc[td] *= alpha;
        }
#pragma unroll
        for (int td = 0; td < TD; ++td) o_acc[td] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[td], pf, o_acc[td], 0, 0, 0);
    }
    if (!valid) return;
    float l_tot = l_run + __shfl_xor(l_run, 16, 64);
    l_tot += __shfl_xor(l_tot, 32, 64);
    if (it.flags & ITEM_WRITE_PARTIAL) {
        // one chunk of a split row: its running state goes to the chunk's slot, the merge kernel finishes the row
        const int64_t prow = (int64_t)(p.T + it.pad1) * p.n_q + hq;
        if (gq == 0) *reinterpret_cast<float2*>(p.part_ml + prow * 2) = make_float2(m_run, l_tot);
        float* po = p.part_o + prow * D + 4 * gq;
#pragma unroll
        for (int td = 0; td < TD; ++td)
            *reinterpret_cast<float4*>(po + 16 * td) = make_float4(o_acc[td][0], o_acc[td][1], o_acc[td][2], o_acc[td][3]);
        return;
    }
    const float inv = p.v_scale / l_tot;
    uint16_t* orow = p.out + row_id * D + 4 * gq;
#pragma unroll
    for (int td = 0; td < TD; ++td)
        *reinterpret_cast<uint2*>(orow + 16 * td) =
            make_uint2(pack_bf16x2(o_acc[td][0] * inv, o_acc[td][1] * inv),
                       pack_bf16x2(o_acc[td][2] * inv, o_acc[td][3] * inv));
}

// Finishes the decode rows whose keys were cut into chunks: with chunk states (m_c, l_c, O_c) in the log2 domain,
// out = sum_c 2^(m_c - M) O_c / sum_c 2^(m_c - M) l_c with M the largest m_c, accumulated in chunk order with a running
// maximum.  A thread per four output values of one row; blockIdx.x = row, blockIdx.y = 256 of its units.
template <int D>
__global__ void __launch_bounds__(256) attn_merge_kernel(AttnArgs p) {
    const MergeItem mi = p.merge_items[blockIdx.x];
    const int u = blockIdx.y * 256 + threadIdx.x;
    if (u >= p.n_q * (D / 4)) return;
    const int hq = u / (D / 4), d0 = (u % (D / 4)) * 4;
    const int64_t row0 = (int64_t)(p.T + mi.first_slot) * p.n_q + hq;
    float M = -INFINITY, L = 0.f;
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
    for (int c = 0; c < mi.n_chunks; ++c) {
        const int64_t prow = row0 + (int64_t)c * p.n_q;
        const float2 ml = *reinterpret_cast<const float2*>(p.part_ml + prow * 2);
        const float4 v = *reinterpret_cast<const float4*>(p.part_o + prow * D + d0);
        const float m_new = fmaxf(M, ml.x);
        const float a = __builtin_amdgcn_exp2f(M - m_new), w = __builtin_amdgcn_exp2f(ml.x - m_new);   // a = 0 at the first chunk
        M = m_new;
        L = L * a + w * ml.y;
        o.x = o.x * a + w * v.x; o.y = o.y * a + w * v.y; o.z = o.z * a + w * v.z; o.w = o.w * a + w * v.w;
    }
    const float inv = p.v_scale / L;
    *reinterpret_cast<uint2*>(p.out + ((int64_t)mi.tok * p.n_q + hq) * D + d0) =
        make_uint2(pack_bf16x2(o.x * inv, o.y * inv), pack_bf16x2(o.z * inv, o.w * inv));
}

template <int D, bool FP8>
__global__ void __launch_bounds__(256, 2) attn_tile_kernel(AttnArgs p) {
    attn_tile_body<D, FP8>(p, blockIdx.x, blockIdx.y);
}

template <int D, bool FP8>
__global__ void __launch_bounds__(256, 2) attn_decode_kernel(AttnArgs p) {
    attn_decode_body<D, FP8>(p, p.items, p.n_items, blockIdx.x);
}

// Prefill rows (row-tiled items) and decode rows (wave items) over their own keys in ONE launch: the two
// item lists are independent, each alone leaves part of the chip idle at its end, and both need the same
// registers and LDS.  Workgroups [0, n_items n_kv) take the tiled items (the longer ones), the rest the
// decode items, four per workgroup.
template <int D, bool FP8>
__global__ void __launch_bounds__(256, 2) attn_own_keys_kernel(AttnArgs p) {
    const int n_tile_wg = p.n_items * p.n_kv;
    const int b = blockIdx.x;
    if (b < n_tile_wg) {
        attn_tile_body<D, FP8>(p, b % p.n_items, b / p.n_items);
    } else {
        attn_decode_body<D, FP8>(p, p.items_b, p.n_items_b, b - n_tile_wg);
    }
}

inline int decode_wgs(const AttnArgs& p, int n_items) {
    return p.dec_by_head ? n_items * (p.n_kv >> 2) : (n_items + 3) / 4 * p.n_kv;
}

template <int D, bool FP8>
hipError_t launch_d(const AttnArgs& base, const AttnItem* items, int32_t n_items, const AttnItem* items_b,
                    int32_t n_items_b, bool decode, hipStream_t s) {
    constexpr int tile_smem = 2 * TileSmem<D>::STAGE, dec_smem = 4 * DecodeSmem<D>::WAVE_BYTES;
    constexpr int both_smem = tile_smem > dec_smem ? tile_smem : dec_smem;
    // the dynamic-LDS limits are raised once per process, whichever host thread launches first
    static std::once_flag once;
    static hipError_t attr_status = hipSuccess;
    std::call_once(once, [] {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_tile_kernel<D, FP8>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, tile_smem);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_decode_kernel<D, FP8>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, dec_smem);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_own_keys_kernel<D, FP8>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, both_smem);
        attr_status = e;
    });
    if (attr_status != hipSuccess) return attr_status;
    AttnArgs p = base;
    p.items = items;
    p.n_items = n_items;
    p.items_b = items_b;
    p.n_items_b = n_items_b;
    if (items_b)
        attn_own_keys_kernel<D, FP8><<<dim3(n_items * p.n_kv + decode_wgs(p, n_items_b)), dim3(256), both_smem, s>>>(p);
    else if (decode)
        attn_decode_kernel<D, FP8><<<dim3(decode_wgs(p, n_items)), dim3(256), dec_smem, s>>>(p);
    else
        attn_tile_kernel<D, FP8><<<dim3(n_items, p.n_kv), dim3(256), tile_smem, s>>>(p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attention(const BatchDev& b, const relserve_layer& L, const void* q, int32_t q_pitch,
                            const void* k_pages, const void* v_pages, void* out, float* part_o, float* part_ml,
                            hipStream_t s, relserve_layer* prof, KvFormat kv) {
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
    p.dec_by_head = L.cfg.n_kv_heads % 4 == 0 ? 1 : 0;
    // a quantised key reads back as code x k_scale: the scale moves into the score's factor, the value pool's to the end
    p.scale_log2 = (float)(1.4426950408889634 / sqrt((double)L.cfg.head_dim) * (double)kv.k_scale);
    p.v_scale = kv.v_scale;
    const bool d128 = L.cfg.head_dim == 128;
    hipError_t e = hipSuccess;
    auto launch = [&](int slot, const AttnItem* items, int32_t n, const AttnItem* items_b, int32_t n_b, bool decode) {
        if (e != hipSuccess || n == 0) return;
        profile_mark(prof, slot, s, true);
        if (kv.fp8)
            e = d128 ? launch_d<128, true>(p, items, n, items_b, n_b, decode, s) : launch_d<64, true>(p, items, n, items_b, n_b, decode, s);
        else
            e = d128 ? launch_d<128, false>(p, items, n, items_b, n_b, decode, s) : launch_d<64, false>(p, items, n, items_b, n_b, decode, s);
        profile_mark(prof, slot, s, false);
    };
    p.T = b.T;
    p.merge_items = b.merge_items;
    launch(3, b.items_prefix, b.n_items_prefix, nullptr, 0, false);
    if (b.n_items_tile > 0 && b.n_items_split > 0) {   // both kinds of rows: one launch for their own keys
        launch(2, b.items_tile, b.n_items_tile, b.items_split, b.n_items_split, false);
    } else {
        launch(4, b.items_tile, b.n_items_tile, nullptr, 0, false);
        launch(5, b.items_split, b.n_items_split, nullptr, 0, true);
    }
    if (e == hipSuccess && b.n_merge > 0) {
        profile_mark(prof, 10, s, true);
        const unsigned y_blocks = (unsigned)((p.n_q * (L.cfg.head_dim / 4) + 255) / 256);
        if (d128)
            attn_merge_kernel<128><<<dim3(b.n_merge, y_blocks), dim3(256), 0, s>>>(p);
        else
            attn_merge_kernel<64><<<dim3(b.n_merge, y_blocks), dim3(256), 0, s>>>(p);
        e = hipGetLastError();
        profile_mark(prof, 10, s, false);
    }
    return e;
}

}  // namespace relserve
