// bf16 MFMA GEMM for the dense maps of the layer (Eq. 3, W_o of Eq. 5, gate/up, down):
//   out[T, N] = a[T, K] * w[N, K]^T, fp32 accumulate, fused epilogues.
//
// Both operands are K-contiguous, which is the natural MFMA operand layout: a lane's 8
// consecutive k values are one 16-byte load.  The weight rows take the MFMA row index and
// the tokens the column index, so that an accumulator quad holds 4 consecutive output
// features of one token (one 8/16-byte store).
//
// Workgroup = a grid of waves (2 x 2 in production) over a BM (tokens) x BN (features) tile, BK = 64.
// Main kernel (gemm_dma_kernel, K % 64 == 0): tiles go global -> LDS directly, XOR-swizzled 16-byte
// chunks, two stages, one barrier per k iteration, every k step issued in a fixed order that
// slots the refill loads and the next fragment reads between the MFMAs.  Fallback kernel
// (gemm_bf16_kernel): global -> registers -> LDS with zero-filled tails for any K % 8 == 0.
// Workgroup ids are remapped so that each of the 8 XCDs (own L2 each) walks a contiguous run of
// tiles, inside it token tiles fastest within panels of GROUP_M token tiles.
// Launch plans: tile shape by a cost model; the incomplete last round of tiles may split k over
// workgroups; batches of at most 256 tokens, and narrow outputs at a few hundred, split k everywhere.
// Every split writes partial tiles to fp32 slabs that a second kernel sums and finishes.
#include <algorithm>
#include <atomic>
#include <mutex>
#include <type_traits>

#include "device_utils.h"
#include "relserve_internal.h"

namespace relserve {

namespace {

constexpr int BK = 64;
constexpr int NUM_XCD = 8;
constexpr int64_t kTailFloats = GEMM_TAIL_FLOATS;          // fp32 partial tiles (slabs) of the split paths at T > 256

struct GemmArgs {
    const uint16_t* a;
    const uint16_t* w;
    int32_t w_packed;   // weights in the tiled layout of pack_weight_kernel instead of row-major [N, K]
    const void* residual;
    void* out;
    int32_t T, N, K;
    int32_t n_half;  // SwiGLU: gate rows [0, n_half), up rows [n_half, 2 n_half)
    int32_t tiles_m, tiles_n;
    // fused q/k/v epilogue: rotary embedding + KV append (out = q buffer [T, n_q d])
    const int32_t* tok_slot;
    const float2* rope_cs;
    uint16_t* k_pages;
    uint16_t* v_pages;
    int32_t n_q, n_kv;
    int32_t kv_fp8;          // the pools hold 8-bit codes of x * k_inv / x * v_inv (one byte per element)
    float k_inv, v_inv;
    // split-K (skinny and mid-size T): workgroup b handles tile b % tiles and k steps [split * k_per_split, ...)
    // of that tile and stores its partial sums to slab `split` of accum [n_splits][T, N] fp32; the finish
    // kernel adds the slabs in split order
    float* accum;
    int32_t k_per_split;   // in units of 64; 0 = no split
    int32_t n_splits;
    // tail split (main path): the last tail_tiles tiles (those of the incomplete last round) are each
    // computed by tail_splits workgroups over k_per_split k steps each.  The partial tiles are stored
    // to tail_buf (tail_splits x tail_tiles x BM x BN fp32); a second kernel adds them up and runs the
    // epilogue.
    int32_t tail_tiles, tail_splits;
    float* tail_buf;
    // quantised projections: a and w hold 8-bit codes (one byte per element; K then counts PAIRS of codes, so that a row
    // is K * 2 bytes as in the 16-bit case), the sums are scaled by a_scale * w_scale[n], and a SwiGLU output is
    // stored as codes of value * out_inv
    int32_t f8;
    const float* w_scale;
    float a_scale;
    int32_t out_f8;
    float out_inv;
};

// Test hook (relserve_debug_force_gemm_plan): tile candidate (index into kTiles) and tail splits every launch
// must use; -1 = cost model.  One word, so that a launch on another host thread sees a consistent pair.
std::atomic<int> g_forced_plan{-1};   // -1, or cand | splits << 8
inline int forced_cand() { const int v = g_forced_plan.load(std::memory_order_relaxed); return v < 0 ? -1 : (v & 0xff); }
inline int forced_splits() { const int v = g_forced_plan.load(std::memory_order_relaxed); return v < 0 ? 0 : (v >> 8); }

// The dynamic-LDS limit of a kernel is raised once per process, whichever host thread launches it first.
template <typename Kernel>
hipError_t allow_smem_once(std::once_flag& once, hipError_t& status, Kernel kernel, int bytes) {
    std::call_once(once, [&] {
        status = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    });
    return status;
}

enum { EPI_BF16 = 0, EPI_RES_BF16_OUT_F32 = 1, EPI_RES_F32_OUT_BF16 = 2, EPI_SWIGLU = 3, EPI_QKV_ROPE = 4, EPI_SLAB = 5 };

__device__ __forceinline__ int remap_xcd(int bid, int num) {
    const int per = num / NUM_XCD, rem = num % NUM_XCD;
    const int xcd = bid % NUM_XCD, idx = bid / NUM_XCD;
    return xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
}

// Tile order inside an XCD's run: token tiles fastest within panels of about GROUP_M token tiles, then
// feature tiles, then the next panel.  The ~32 tiles an XCD works on at a time then cover about
// GROUP_M token tiles x 32 / GROUP_M feature tiles, so that its L2 serves ~12 distinct operand
// slices per k step instead of 33 when the batch has many token tiles.  The token tiles are divided
// evenly over the panels (9 token tiles: panels of 5 and 4, not of 8 and 1 -- a panel of one token tile
// shares nothing but its activation slice).
constexpr int GROUP_M = 8;
__device__ __forceinline__ void tile_coords(int t, int tiles_m, int tiles_n, int& tile_m, int& tile_n) {
    const int n_panels = (tiles_m + GROUP_M - 1) / GROUP_M;
    const int base = tiles_m / n_panels, extra = tiles_m % n_panels;   // the first `extra` panels hold base + 1 token tiles
    const int big = (base + 1) * tiles_n;
    int first_m, gsz, in_group;
    if (t < extra * big) {
        gsz = base + 1;
        first_m = (t / big) * gsz;
        in_group = t % big;
    } else {
        const int u = t - extra * big, per = base * tiles_n;
        gsz = base;
        first_m = extra * (base + 1) + (u / per) * base;
        in_group = u % per;
    }
    tile_m = first_m + in_group % gsz;
    tile_n = in_group / gsz;
}

// Epilogue shared by both GEMM kernels: register r of accumulator tile (tn, tm) holds feature
// 32 tn + 8 (r / 4) + 4 g + r % 4 of the wave's feature range and token 32 tm + l32 of its token range.
// TMX of the wave's BM / (32 WGM) rows of accumulator tiles are held in acc, starting at row tm_base (the GEMM kernels
// hold all of them; the tail finish kernel one per workgroup, which lets several workgroups share a CU).
// SC: the sums are products of 8-bit codes and take the factor a_scale * w_scale[feature] as they are read.
template <int BM, int BN, int EPI, int D, int WGM = 2, int WGN = 2, int TMX = BM / (32 * WGM), bool SC = false>
__device__ __forceinline__ void gemm_epilogue(const f32x16_t (&acc)[BN / (32 * WGN)][TMX], const GemmArgs& p,
                                              int tile_m, int tile_n, int wm, int wn, int l32, int g, int tm_base = 0,
                                              int split = 0) {
    constexpr int TM = TMX, TN = BN / (32 * WGN);
    const int t0 = tile_m * BM + 32 * tm_base;
    // factors of the 4 consecutive features n .. n + 3 (n a multiple of 4 below the feature count)
    auto scale4 = [&](int n) -> float4 {
        if constexpr (SC) {
            const float4 w = *reinterpret_cast<const float4*>(p.w_scale + n);
            return make_float4(w.x * p.a_scale, w.y * p.a_scale, w.z * p.a_scale, w.w * p.a_scale);
        } else {
            return make_float4(1.f, 1.f, 1.f, 1.f);
        }
    };
    if (EPI == EPI_SLAB) {
        // Split-K partial sums -> this split's slab.  These tiles were accumulated with the operands
        // swapped: register r holds token 8 (r / 4) + 4 g + r % 4 and feature l32, so one store
        // instruction writes two runs of 32 consecutive floats.  Plain stores: nothing is read back in
        // this kernel, and fp32 atomics into a shared accumulator ran at a quarter of the rate.
        float* slab = p.accum + (int64_t)split * p.T * p.N;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const int n = tile_n * BN + wn * (BN / WGN) + 32 * tn + l32;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int t = t0 + wm * (BM / WGM) + 32 * tm + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (t < p.T && n < p.N) slab[(int64_t)t * p.N + n] = acc[tn][tm][r];
                }
            }
        return;
    }
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int t = t0 + wm * (BM / WGM) + 32 * tm + l32;
        if (t >= p.T) continue;
        if (EPI == EPI_SLAB) {
            // handled before this loop (transposed accumulator layout)
        } else if (EPI == EPI_QKV_ROPE) {
            // The wave owns features [nb, nb + 128): one head (d = 128) or two (d = 64).  The rotation
            // partner of feature i is i + d/2: same lane, same register, D/64 tiles further on.
            constexpr int TPH = (D > 0 ? D : 64) / 32;   // tiles per head
            constexpr int HPW = 4 / TPH;                 // heads per wave
            const int nb = tile_n * BN + wn * 128;
            const int64_t slot = p.tok_slot[t];
            const float2* cs = p.rope_cs + (int64_t)t * (D / 2);
            const int kv_dim = p.n_kv * D;
#pragma unroll
            for (int hh = 0; hh < HPW; ++hh) {
                const int head = nb / D + hh;
                if (head >= p.n_q + 2 * p.n_kv) continue;
                if (head < p.n_q + p.n_kv) {
                    uint16_t* dst = head < p.n_q
                                        ? static_cast<uint16_t*>(p.out) + (int64_t)t * (p.n_q * D) + head * D
                                        : p.k_pages + slot * kv_dim + (head - p.n_q) * D;
#pragma unroll
                    for (int tl = 0; tl < TPH / 2; ++tl) {
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const int i = 32 * tl + 8 * q + 4 * g;
                            const float4 c01 = *reinterpret_cast<const float4*>(cs + i);
                            const float4 c23 = *reinterpret_cast<const float4*>(cs + i + 2);
                            const float co[4] = {c01.x, c01.z, c23.x, c23.z}, si[4] = {c01.y, c01.w, c23.y, c23.w};
                            const float4 sa4 = scale4(head * D + i), sb4 = scale4(head * D + i + D / 2);
                            const float sa[4] = {sa4.x, sa4.y, sa4.z, sa4.w}, sb[4] = {sb4.x, sb4.y, sb4.z, sb4.w};
                            float lo[4], hi[4];
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                float a = acc[hh * TPH + tl][tm][4 * q + j];
                                float b = acc[hh * TPH + tl + TPH / 2][tm][4 * q + j];
                                if constexpr (SC) a *= sa[j], b *= sb[j];
                                lo[j] = a * co[j] - b * si[j];
                                hi[j] = a * si[j] + b * co[j];
                            }
                            if (p.kv_fp8 && head >= p.n_q) {   // quantised cache: one byte per element, quantised from fp32
                                uint8_t* dst8 = reinterpret_cast<uint8_t*>(p.k_pages) + slot * kv_dim + (head - p.n_q) * D + i;
                                const float s = p.k_inv;
                                *reinterpret_cast<uint32_t*>(dst8) = pack_fp8x4(lo[0] * s, lo[1] * s, lo[2] * s, lo[3] * s);
                                *reinterpret_cast<uint32_t*>(dst8 + D / 2) = pack_fp8x4(hi[0] * s, hi[1] * s, hi[2] * s, hi[3] * s);
                            } else {
                                *reinterpret_cast<uint2*>(dst + i) = make_uint2(pack_bf16x2(lo[0], lo[1]), pack_bf16x2(lo[2], lo[3]));
                                *reinterpret_cast<uint2*>(dst + i + D / 2) =
                                    make_uint2(pack_bf16x2(hi[0], hi[1]), pack_bf16x2(hi[2], hi[3]));
                            }
                            // every register is taken by the accumulators: keep the scheduler from starting the
                            // next quads' table loads early (they would spill)
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    }
                } else {
                    uint16_t* dst = p.v_pages + slot * kv_dim + (head - p.n_q - p.n_kv) * D;
#pragma unroll
                    for (int tl = 0; tl < TPH; ++tl) {
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const int i = 32 * tl + 8 * q + 4 * g;
                            f32x16_t a = acc[hh * TPH + tl][tm];
                            if constexpr (SC) {
                                const float4 sv = scale4(head * D + i);
                                a[4 * q] *= sv.x; a[4 * q + 1] *= sv.y; a[4 * q + 2] *= sv.z; a[4 * q + 3] *= sv.w;
                            }
                            if (p.kv_fp8) {
                                const float s = p.v_inv;
                                *reinterpret_cast<uint32_t*>(reinterpret_cast<uint8_t*>(p.v_pages) + slot * kv_dim +
                                                             (head - p.n_q - p.n_kv) * D + i) =
                                    pack_fp8x4(a[4 * q] * s, a[4 * q + 1] * s, a[4 * q + 2] * s, a[4 * q + 3] * s);
                            } else {
                                *reinterpret_cast<uint2*>(dst + i) = make_uint2(pack_bf16x2(a[4 * q], a[4 * q + 1]),
                                                                                pack_bf16x2(a[4 * q + 2], a[4 * q + 3]));
                            }
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    }
                }
            }
        } else if (EPI == EPI_SWIGLU) {
#pragma unroll
            for (int tn = 0; tn < TN / 2; ++tn) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int i = tile_n * (BN / 2) + wn * (BN / (2 * WGN)) + 32 * tn + 8 * q + 4 * g;
                    if (i >= p.n_half) continue;  // n_half is a multiple of 8, i of 4: whole quad in or out
                    float o[4];
                    const float4 sg4 = scale4(i), su4 = scale4(p.n_half + i);
                    const float sg[4] = {sg4.x, sg4.y, sg4.z, sg4.w}, su[4] = {su4.x, su4.y, su4.z, su4.w};
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        float gate = acc[tn][tm][4 * q + j], up = acc[tn + TN / 2][tm][4 * q + j];
                        if constexpr (SC) gate *= sg[j], up *= su[j];
                        o[j] = silu_mul(gate, up);
                    }
                    if (SC && p.out_f8) {   // the down projection reads codes
                        const float s = p.out_inv;
                        *reinterpret_cast<uint32_t*>(static_cast<uint8_t*>(p.out) + (int64_t)t * p.n_half + i) =
                            pack_fp8x4(o[0] * s, o[1] * s, o[2] * s, o[3] * s);
                        continue;
                    }
                    uint2 st = make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
                    *reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.out) + (int64_t)t * p.n_half + i) = st;
                }
            }
        } else {
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = tile_n * BN + wn * (BN / WGN) + 32 * tn + 8 * q + 4 * g;
                    if (n >= p.N) continue;  // N is a multiple of 4 on every path that reaches here
                    const int64_t o = (int64_t)t * p.N + n;
                    float v[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) v[j] = acc[tn][tm][4 * q + j];
                    if constexpr (SC) {
                        const float4 sc = scale4(n);
                        v[0] *= sc.x; v[1] *= sc.y; v[2] *= sc.z; v[3] *= sc.w;
                    }
                    if (EPI == EPI_RES_BF16_OUT_F32) {
                        uint2 r = make_uint2(0, 0);  // no residual given: plain fp32 output
                        if (p.residual) r = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(p.residual) + o);
                        float4 st = make_float4(v[0] + bf16_lo(r.x), v[1] + bf16_hi(r.x), v[2] + bf16_lo(r.y),
                                                v[3] + bf16_hi(r.y));
                        *reinterpret_cast<float4*>(static_cast<float*>(p.out) + o) = st;
                    } else {
                        if (EPI == EPI_RES_F32_OUT_BF16) {
                            const float4 r = *reinterpret_cast<const float4*>(static_cast<const float*>(p.residual) + o);
                            v[0] += r.x; v[1] += r.y; v[2] += r.z; v[3] += r.w;
                        }
                        uint2 st = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
                        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.out) + o) = st;
                    }
                    __builtin_amdgcn_sched_barrier(0);   // see the q/k/v epilogue
                }
            }
        }
    }
}

template <int BM, int BN, int EPI, int D = 0>
__global__ void __launch_bounds__(256) gemm_bf16_kernel(GemmArgs p) {
    constexpr int TM = BM / 64, TN = BN / 64;          // 32x32 MFMA tiles per wave
    constexpr int A_IT = BM / 32, W_IT = BN / 32;      // 16-byte chunks per thread and k step
    constexpr int A_BYTES = BM * BK * 2, W_BYTES = BN * BK * 2, STAGE = A_BYTES + W_BYTES;
    static_assert(EPI != EPI_SWIGLU || TN % 2 == 0, "SwiGLU needs gate and up tiles in one wave");
    static_assert(EPI != EPI_QKV_ROPE || (BN == 256 && (D == 64 || D == 128)), "a wave must own whole heads");
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, g = lane >> 5;

    const int tile = remap_xcd(blockIdx.x, p.tiles_m * p.tiles_n);
    int tile_m, tile_n;
    tile_coords(tile, p.tiles_m, p.tiles_n, tile_m, tile_n);
    const int t0 = tile_m * BM;
    const int K = p.K;

    // ---- global -> register staging: element offsets of this thread's chunks (-1 = zero fill)
    const int c8 = (tid & 7) * 8, lrow = tid >> 3;
    int a_off[A_IT], w_off[W_IT];
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
        const int t = t0 + lrow + 32 * i;
        a_off[i] = t < p.T ? t * K + c8 : -1;
    }
#pragma unroll
    for (int i = 0; i < W_IT; ++i) {
        const int lr = lrow + 32 * i;
        int n;
        bool ok;
        if (EPI == EPI_SWIGLU) {
            constexpr int HALF = BN / 2;
            const int gi = tile_n * HALF + (lr % HALF);
            ok = gi < p.n_half;
            n = lr < HALF ? gi : p.n_half + gi;
        } else {
            n = tile_n * BN + lr;
            ok = n < p.N;
        }
        w_off[i] = ok ? n * K + c8 : -1;
    }
    const int st_off = lrow * 128 + (((tid & 7) ^ (lrow & 7)) << 4);  // swizzled LDS store offset

    uint4 a_reg[A_IT], w_reg[W_IT];
    auto load_global = [&](int k0) {
        const bool k_ok = k0 + c8 < K;
#pragma unroll
        for (int i = 0; i < A_IT; ++i)
            a_reg[i] = (a_off[i] >= 0 && k_ok) ? *reinterpret_cast<const uint4*>(p.a + a_off[i] + k0)
                                               : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < W_IT; ++i)
            w_reg[i] = (w_off[i] >= 0 && k_ok) ? *reinterpret_cast<const uint4*>(p.w + w_off[i] + k0)
                                               : make_uint4(0, 0, 0, 0);
    };
    auto store_lds = [&](int buf) {
        unsigned char* sa = smem + buf * STAGE;
        unsigned char* sw = sa + A_BYTES;
#pragma unroll
        for (int i = 0; i < A_IT; ++i) *reinterpret_cast<uint4*>(sa + i * 32 * 128 + st_off) = a_reg[i];
#pragma unroll
        for (int i = 0; i < W_IT; ++i) *reinterpret_cast<uint4*>(sw + i * 32 * 128 + st_off) = w_reg[i];
    };

    // ---- LDS -> MFMA operand offsets
    int a_rd[TM], w_rd[TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) a_rd[tm] = (wm * (BM / 2) + 32 * tm + l32) * 128;
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        int row;
        if (EPI == EPI_SWIGLU)
            row = (tn < TN / 2 ? 0 : BN / 2) + wn * (BN / 4) + 32 * (tn % (TN / 2)) + l32;
        else
            row = wn * (BN / 2) + 32 * tn + l32;
        w_rd[tn] = row * 128;
    }
    const int sw7 = l32 & 7;

    f32x16_t acc[TN][TM];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tn][tm][r] = 0.f;

    const int nk = (K + BK - 1) / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const bool more = kt + 1 < nk;
        if (more) load_global((kt + 1) * BK);
        const unsigned char* sa = smem + (kt & 1) * STAGE;
        const unsigned char* sw = sa + A_BYTES;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int ch = ((2 * ks + g) ^ sw7) << 4;
            bf16x8_t wf[TN], af[TM];
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) wf[tn] = as_bf16x8(*reinterpret_cast<const uint4*>(sw + w_rd[tn] + ch));
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) af[tm] = as_bf16x8(*reinterpret_cast<const uint4*>(sa + a_rd[tm] + ch));
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) acc[tn][tm] = mfma_32x32x16(wf[tn], af[tm], acc[tn][tm]);
        }
        if (more) store_lds((kt + 1) & 1);
        __syncthreads();
    }
    gemm_epilogue<BM, BN, EPI, D>(acc, p, tile_m, tile_n, wm, wn, l32, g);
}

// ------------------------------------------------------------------------------------------
// Main kernel for K % 64 == 0: tiles go global -> LDS directly (global_load_lds_dwordx4, no
// register staging and no LDS store instructions), two LDS stages, operand fragments double
// buffered in registers.  The barrier that hands over a stage sits one k step BEFORE the stage
// boundary: the last 16 MFMAs of a stage run while the first fragments of the next stage are
// being read, and the loads of the stage after that are issued at once, so they have a whole
// k iteration to land.
// ------------------------------------------------------------------------------------------
// 64 lanes x 16 bytes from (base + per-lane byte offset) to 1 KB of LDS starting at lds_addr.
// A pointer every lane holds the same value of, moved to scalar registers (the compiler cannot always prove it).
__device__ __forceinline__ const char* uniform_ptr(const char* ptr) {
    const uint64_t v = reinterpret_cast<uint64_t>(ptr);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const char*>(((uint64_t)hi << 32) | lo);
}

// NT = non-temporal: for bytes that are read once (the weights of a batch of one token tile).  A streaming read of
// HBM reaches 7.1-7.4 TB/s with the hint against 6.3-6.4 TB/s without (measured with 32 KB per workgroup in flight);
// operands that other workgroups read again keep the default policy, which lets the L2 hold them.
template <bool NT = false>
__device__ __forceinline__ void dma16(const void* base, uint32_t voff, uint32_t lds_addr) {
    if (NT)
        asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1 nt" ::"v"(voff), "s"(base), "s"(lds_addr) : "memory");
    else
        asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(base), "s"(lds_addr) : "memory");
}

// BKD = k extent of one LDS stage (64 or 32), NS = stages in the ring (NS - 1 are in flight).
// WGM x WGN = grid of waves over the tile (4 or 8 waves; 8 waves = two per SIMD, each with a quarter
// of the registers, so that one wave's MFMAs cover the other's memory-instruction issue).
// WNT: the weights are loaded with the non-temporal hint (launches in which no other workgroup reads them again).
// F8: both operands hold 8-bit codes.  Nothing changes in how bytes travel (K counts pairs of codes, a stage row is
// still 128 bytes); a k step covers 32 bytes of every row instead of 16, as one 32x32x64 MFMA whose operand is the
// two adjacent 16-byte chunks (2 ks' + g) * 2, + 1 of the row for k half g (both operands alike, so which codes
// meet which is fixed), and the epilogue applies the scales.
template <int BM, int BN, int EPI, int D, int BKD, int NS, int WGM = 2, int WGN = 2, bool WNT = false, bool F8 = false>
__global__ void __launch_bounds__(64 * WGM * WGN) gemm_dma_kernel(GemmArgs p) {
    constexpr int NW = WGM * WGN;
    constexpr int TM = BM / (32 * WGM), TN = BN / (32 * WGN);
    constexpr int ROWB = BKD * 2;                        // bytes per LDS row
    constexpr int CPR = BKD / 8;                         // 16-byte chunks per row
    constexpr int RPI = 1024 / ROWB;                     // rows one 1 KB wave load covers
    constexpr int A_IT = BM / (NW * RPI), W_IT = BN / (NW * RPI);
    constexpr int A_BYTES = BM * ROWB, W_BYTES = BN * ROWB, STAGE = A_BYTES + W_BYTES;
    constexpr int KSTEPS = F8 ? BKD / 32 : BKD / 16;
    constexpr int LOADS = A_IT + W_IT;                   // wave loads per stage
    static_assert(BKD == 64 || BKD == 32, "stage depth");
    static_assert(!F8 || BKD == 64, "the fragment double buffer needs an even number of k steps per stage");
    static_assert((NS - 1) * LOADS < 64, "vmcnt field");
    static_assert(EPI != EPI_SWIGLU || TN % 2 == 0, "SwiGLU needs gate and up tiles in one wave");
    static_assert(EPI != EPI_QKV_ROPE || (BN / WGN == 128 && (D == 64 || D == 128)), "a wave must own whole heads");
    static_assert(BM % (NW * RPI) == 0 && BN % (NW * RPI) == 0, "whole wave loads");
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    const int l32 = lane & 31, g = lane >> 5;

    const int n_tiles = p.tiles_m * p.tiles_n;
    int tile, split;
    bool tail = false;
    int tail_idx = 0;
    if (EPI == EPI_SLAB) {
        tile = remap_xcd(blockIdx.x % n_tiles, n_tiles);
        split = blockIdx.x / n_tiles;
    } else {
        // the tail units come first in the grid: their short k ranges and slab stores are over before the
        // last whole tiles finish
        const int tail_units = p.tail_tiles * p.tail_splits, dp_tiles = n_tiles - p.tail_tiles;
        tail = (int)blockIdx.x < tail_units;
        if (tail) {
            const int u = remap_xcd(blockIdx.x, tail_units);   // runs of one split, consecutive tiles, per XCD
            split = u / p.tail_tiles;
            tail_idx = u % p.tail_tiles;
            tile = dp_tiles + tail_idx;
        } else {
            split = 0;
            tile = remap_xcd(blockIdx.x - tail_units, dp_tiles);
        }
    }
    int tile_m, tile_n;
    tile_coords(tile, p.tiles_m, p.tiles_n, tile_m, tile_n);
    const int t0 = tile_m * BM;
    const int K = p.K;

    // ---- per-lane source offsets: wave load j of this wave fills LDS rows (NW j + wave) * RPI .. ;
    // lane l owns row l / CPR of those and slot l % CPR, which holds the row's chunk slot ^ swz(row).
    // The LDS has 64 four-byte banks and serves a 16-byte-per-lane read 16 lanes at a time, so the
    // 16 consecutive rows those lanes read must cover all 64 banks once: swz = (row >> 1) & 7 for
    // 128-byte rows (row parity picks the bank half), (row >> 2) & 3 for 64-byte rows.
    // Rows past the end of a matrix re-read its last row: their products are never stored.
    const uint32_t lrow = lane / CPR;
    const uint32_t row_lo = (uint32_t)(wave * RPI) + lrow;   // LDS row modulo NW * RPI (>= 32): all the swizzle needs
    const uint32_t chunk = (lane % CPR) ^ (BKD == 64 ? ((row_lo >> 1) & 7) : ((row_lo >> 2) & 3));
    uint32_t a_voff[A_IT], w_voff[W_IT];
#pragma unroll
    for (int j = 0; j < A_IT; ++j) {
        const int t = min(t0 + (NW * j + wave) * RPI + (int)lrow, p.T - 1);
        a_voff[j] = ((uint32_t)t * (uint32_t)K + chunk * 8) * 2;
    }
#pragma unroll
    for (int j = 0; j < W_IT; ++j) {
        const int lr = (NW * j + wave) * RPI + (int)lrow;
        int n;
        if (EPI == EPI_SWIGLU) {
            constexpr int HALF = BN / 2;
            const int gi = min(tile_n * HALF + (lr % HALF), p.n_half - 1);
            n = lr < HALF ? gi : p.n_half + gi;
        } else {
            n = min(tile_n * BN + lr, p.N - 1);
        }
        // row-major: row n starts at n * K; packed: block n / 256 holds, k slice after k slice, 256 rows of 128 bytes
        // (a 32-wide stage is the first or the second half of every row of a slice)
        w_voff[j] = p.w_packed ? (uint32_t)(n >> 8) * (uint32_t)K * 512u + (uint32_t)(n & 255) * 128u + chunk * 16
                               : ((uint32_t)n * (uint32_t)K + chunk * 8) * 2;
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
    auto issue_stage = [&](int stage, int k0) {
        const char* abase = reinterpret_cast<const char*>(p.a) + (size_t)k0 * 2;
        const char* wbase = reinterpret_cast<const char*>(p.w) + (p.w_packed ? (size_t)(k0 >> 6) * 32768 + (size_t)(k0 & 63) * 2 : (size_t)k0 * 2);
        const uint32_t la = lds0 + stage * STAGE + wave * 1024;
#pragma unroll
        for (int j = 0; j < A_IT; ++j) dma16(abase, a_voff[j], la + j * (NW * 1024));
#pragma unroll
        for (int j = 0; j < W_IT; ++j) dma16<WNT>(wbase, w_voff[j], la + A_BYTES + j * (NW * 1024));
    };

    // ---- LDS -> MFMA operand offsets
    int a_rd[TM], w_rd[TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) a_rd[tm] = (wm * (BM / WGM) + 32 * tm + l32) * ROWB;
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        int row;
        if (EPI == EPI_SWIGLU)
            row = (tn < TN / 2 ? 0 : BN / 2) + wn * (BN / (2 * WGN)) + 32 * (tn % (TN / 2)) + l32;
        else
            row = wn * (BN / WGN) + 32 * tn + l32;
        w_rd[tn] = A_BYTES + row * ROWB;
    }
    const int swz = BKD == 64 ? ((l32 >> 1) & 7) : ((l32 >> 2) & 3);

    f32x16_t acc[TN][TM];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tn][tm][r] = 0.f;

    using frag_t = std::conditional_t<F8, i32x8_t, bf16x8_t>;
    frag_t wf[2][TN], af[2][TM];
    auto read_frag = [&](const unsigned char* row, int ks) __attribute__((always_inline)) -> frag_t {
        if constexpr (F8) {
            const uint4 lo = *reinterpret_cast<const uint4*>(row + (((4 * ks + 2 * g) ^ swz) << 4));
            const uint4 hi = *reinterpret_cast<const uint4*>(row + (((4 * ks + 2 * g + 1) ^ swz) << 4));
            return i32x8_t{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
        } else {
            return as_bf16x8(*reinterpret_cast<const uint4*>(row + (((2 * ks + g) ^ swz) << 4)));
        }
    };
    auto load_frags = [&](int buf, int stage, int ks) __attribute__((always_inline)) {
        const unsigned char* st = smem + stage * STAGE;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) wf[buf][tn] = read_frag(st + w_rd[tn], ks);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) af[buf][tm] = read_frag(st + a_rd[tm], ks);
    };

    // k range of this workgroup (the whole K unless the launch splits it)
    const bool part = EPI == EPI_SLAB || tail;
    const int kbeg = part ? split * p.k_per_split * (64 / BKD) : 0;
    const int nk = part ? min(p.k_per_split * (64 / BKD), K / BKD - kbeg) : K / BKD;
    // prologue: fill the whole ring, wait for stage 0 only
#pragma unroll
    for (int s = 0; s < NS; ++s)
        if (s < nk) issue_stage(s, (kbeg + s) * BKD);
    if (nk >= NS)
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 1) * LOADS) : "memory");
    else
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    load_frags(0, 0, 0);
    auto mfma_one = [&](int buf, int i) __attribute__((always_inline)) {   // i-th of the TN * TM products of a k step
        const int tn = i / TM, tm = i % TM;
        if constexpr (F8)
            acc[tn][tm] = EPI == EPI_SLAB ? mfma_32x32x64_f8(af[buf][tm], wf[buf][tn], acc[tn][tm])
                                            : mfma_32x32x64_f8(wf[buf][tn], af[buf][tm], acc[tn][tm]);
        else
            acc[tn][tm] = EPI == EPI_SLAB ? mfma_32x32x16(af[buf][tm], wf[buf][tn], acc[tn][tm])
                                            : mfma_32x32x16(wf[buf][tn], af[buf][tm], acc[tn][tm]);
    };
    auto load_frag_one = [&](int buf, int stage, int ks, int i) __attribute__((always_inline)) {   // i-th of the TN + TM fragment reads of a k step
        const unsigned char* st = smem + stage * STAGE;
        if (i < TN)
            wf[buf][i] = read_frag(st + w_rd[i], ks);
        else
            af[buf][i - TN] = read_frag(st + a_rd[i - TN], ks);
    };
    // Source of the refill in progress (set at a hand-over): the k slice's first byte in both operands and the
    // freed stage's LDS address, so that a load costs its own two instructions plus one scalar add.
    const char* rf_a = nullptr;
    const char* rf_w = nullptr;
    uint32_t rf_la = 0;
    auto issue_one = [&](int i) __attribute__((always_inline)) {   // i-th of the LOADS wave loads of a stage
        // weights first: they come from further away (HBM) than the activations (L2)
        if (i < W_IT)
            dma16<WNT>(rf_w, w_voff[i], rf_la + A_BYTES + i * (NW * 1024));
        else
            dma16(rf_a, a_voff[i - W_IT], rf_la + (i - W_IT) * (NW * 1024));
    };
    // A flag that is either a run-time bool or std::true_type: the steady-state iterations pass the latter, so their
    // loads sit in straight-line code (a branch and its scalar set-up around each load cost more issue slots than
    // the load itself, and a wave has seven slots between two MFMAs).
    auto on = [](auto flag) {
        if constexpr (std::is_same_v<decltype(flag), std::true_type>) return true;
        else return flag;
    };
    constexpr int NM = TN * TM, NF = TN + TM;
    // One k step, issued in a fixed order: MFMA i, then the share of the refill loads and of the next
    // step's fragment reads that falls between MFMA i and i + 1.  A CU's address unit takes one
    // 1 KB load per ~16 cycles and an MFMA lasts 32, so the refill loads of a stage (LOADS per wave,
    // four waves) are spread over SPREAD k steps; issued back to back they would hold up the MFMAs
    // behind them.  The MFMAs sit on ONE control path on purpose: at a join the compiler would make
    // them wait for the newest reads.
    constexpr int SPREAD = KSTEPS > 1 ? KSTEPS - 1 : 1;   // the last k step before the next hand-over stays free: landing time
    auto k_step = [&](int buf, int rd_stage, int rd_ks, int part, auto refill) __attribute__((always_inline)) {
        // share of the stage's loads issued in each part, cumulative, in sixteenths: the weights (first half
        // of the loads) go out at once, the activations (L2 hits, quick to land) trail over two more steps
        constexpr int cut[5] = {0, 8, 13, 16, 16};
        const int pc = part < SPREAD ? part : SPREAD;
        const int d_lo = SPREAD == 3 ? cut[pc] * LOADS / 16 : pc * LOADS / SPREAD;
        const int d_n = (SPREAD == 3 ? cut[pc + 1] * LOADS / 16 : (pc + 1) * LOADS / SPREAD) - d_lo;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < NM; ++i) {
            mfma_one(buf, i);
            __builtin_amdgcn_sched_barrier(0);
            if (part < SPREAD && on(refill)) {
#pragma unroll
                for (int d = d_lo + i * d_n / NM; d < d_lo + (i + 1) * d_n / NM; ++d) issue_one(d);
            }
            if (i < NM / 2) {   // all reads in the first half: the last one has half a step to come back
#pragma unroll
                for (int f = i * NF / (NM / 2); f < (i + 1) * NF / (NM / 2); ++f)
                    load_frag_one(buf ^ 1, rd_stage, rd_ks, f);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // Small tiles (two or three workgroups per CU, a handful of MFMAs per k step) do better when the
    // compiler orders the steps between hand-overs and the other resident workgroups fill the gaps;
    // only their hand-over step keeps the fixed order, with the whole refill in it.
    constexpr bool FIXED = NM >= 12;
    int cur = 0;  // stage being computed
    // One k iteration (one LDS stage).  refill_open: the refill begun at the previous hand-over is still being
    // issued; refill_next: this iteration's hand-over starts another one.
    auto iteration = [&](int kt, auto refill_open, auto refill_next) __attribute__((always_inline)) {
        const int nxt = cur + 1 == NS ? 0 : cur + 1;
#pragma unroll
        for (int ks = 0; ks + 1 < KSTEPS; ++ks) {
            if (FIXED) {
                k_step(ks & 1, cur, ks + 1, ks + 1, refill_open);
            } else {
                load_frags((ks + 1) & 1, cur, ks + 1);
#pragma unroll
                for (int i = 0; i < NM; ++i) mfma_one(ks & 1, i);
            }
        }
        // Last k step of the stage: all its fragments are in registers.  Wait for the next stage (the
        // NS - 2 younger ones may stay in flight), hand over, and start refilling the freed buffer.
        // After the last stage this reads fragments nobody uses.
        constexpr int LB = (KSTEPS - 1) & 1;
        constexpr bool steady = std::is_same_v<decltype(refill_next), std::true_type>;   // then kt + NS < nk
        if (NS == 2 || (!steady && kt + NS - 1 >= nk))
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        else
            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((NS - 2) * LOADS) : "memory");
        __syncthreads();
        if (on(refill_next)) {
            const int k0 = (kbeg + kt + NS) * BKD;
            rf_a = uniform_ptr(reinterpret_cast<const char*>(p.a) + (size_t)k0 * 2);
            rf_w = uniform_ptr(reinterpret_cast<const char*>(p.w) +
                               (p.w_packed ? (size_t)(k0 >> 6) * 32768 + (size_t)(k0 & 63) * 2 : (size_t)k0 * 2));
            rf_la = __builtin_amdgcn_readfirstlane(lds0 + cur * STAGE + wave * 1024);
        }
        if (FIXED) {
            k_step(LB, nxt, 0, 0, refill_next);
        } else {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                mfma_one(LB, i);
                __builtin_amdgcn_sched_barrier(0);
                if (on(refill_next)) {
#pragma unroll
                    for (int d = i * LOADS / NM; d < (i + 1) * LOADS / NM; ++d) issue_one(d);
                }
                if (i >= NM / 2) {
#pragma unroll
                    for (int f = (i - NM / 2) * NF / (NM - NM / 2); f < (i + 1 - NM / 2) * NF / (NM - NM / 2); ++f)
                        load_frag_one(LB ^ 1, nxt, 0, f);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        cur = nxt;
    };
    // first iteration (nothing to refill yet), steady state (every hand-over refills), drain
    int kt = 0;
    if (nk > 0) {
        iteration(0, false, NS < nk);
        kt = 1;
    }
    for (; kt < nk - NS; ++kt) iteration(kt, std::true_type{}, std::true_type{});
    for (; kt < nk; ++kt) iteration(kt, kt - 1 + NS < nk, kt + NS < nk);
    if (EPI != EPI_SLAB && tail) {
        // Partial tile -> this split's slab (registers 4 c .. 4 c + 3 of accumulator tile (tn, tm) of
        // thread tid are the 16 bytes at ((tn TM + tm) 4 + c) * threads + tid: coalesced).
        // gemm_tail_finish_kernel, launched behind this kernel, adds the slabs of a tile in split order and
        // runs the epilogue; the kernel boundary is what makes the slabs of workgroups on other XCDs
        // (other L2s) visible, so nothing here waits or fences.
        typedef float vec4_t __attribute__((ext_vector_type(4)));
        constexpr int AREA4 = BM * BN / 4, NT = 64 * NW;
        vec4_t* slab = reinterpret_cast<vec4_t*>(p.tail_buf) + ((size_t)split * p.tail_tiles + tail_idx) * AREA4 + tid;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    vec4_t v = {acc[tn][tm][4 * c], acc[tn][tm][4 * c + 1], acc[tn][tm][4 * c + 2], acc[tn][tm][4 * c + 3]};
                    slab[((tn * TM + tm) * 4 + c) * NT] = v;
                }
        return;
    }
    gemm_epilogue<BM, BN, EPI, D, WGM, WGN, BM / (32 * WGM), F8>(acc, p, tile_m, tile_n, wm, wn, l32, g, 0, split);
}

// Second half of a tail split: workgroup (tail tile, row tm of accumulator tiles) has the thread layout of
// the GEMM workgroup that wrote the slabs, adds its part of the tile's slabs in split order (so the sum
// does not depend on scheduling) and runs the GEMM's own epilogue on it.
template <int BM, int BN, int EPI, int D, int WGM, int WGN, bool SC = false>
__global__ void __launch_bounds__(64 * WGM * WGN) gemm_tail_finish_kernel(GemmArgs p) {
    constexpr int NW = WGM * WGN, NT = 64 * NW, TM = BM / (32 * WGM), TN = BN / (32 * WGN), AREA4 = BM * BN / 4;
    typedef float vec4_t __attribute__((ext_vector_type(4)));
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    const int l32 = lane & 31, g = lane >> 5;
    const int tail_idx = blockIdx.x / TM, tm_sel = blockIdx.x % TM;
    int tile_m, tile_n;
    tile_coords(p.tiles_m * p.tiles_n - p.tail_tiles + tail_idx, p.tiles_m, p.tiles_n, tile_m, tile_n);
    f32x16_t acc[TN][1];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[tn][0][r] = 0.f;
    for (int q = 0; q < p.tail_splits; ++q) {
        const vec4_t* src = reinterpret_cast<const vec4_t*>(p.tail_buf) + ((size_t)q * p.tail_tiles + tail_idx) * AREA4 + tid;
        vec4_t v[TN][4];
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int c = 0; c < 4; ++c) v[tn][c] = src[((tn * TM + tm_sel) * 4 + c) * NT];
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[tn][0][4 * c + e] += v[tn][c][e];
    }
    gemm_epilogue<BM, BN, EPI, D, WGM, WGN, 1, SC>(acc, p, tile_m, tile_n, wm, wn, l32, g, tm_sel);
}

// ------------------------------------------------------------------------------------------
// Split-K companion kernel: adds the splits' slabs in split order (the sum does not depend on scheduling)
// and applies the same epilogues as the fused path; each thread owns 4 consecutive features of one token.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ float4 slab_sum(const float* first, int64_t slab_stride, int n_splits) {
    float4 v = *reinterpret_cast<const float4*>(first);
    for (int q = 1; q < n_splits; ++q) {
        const float4 w = *reinterpret_cast<const float4*>(first + q * slab_stride);
        v.x += w.x; v.y += w.y; v.z += w.z; v.w += w.w;
    }
    return v;
}

// sums of products of 8-bit codes take the factor a_scale * w_scale[n .. n + 3] (w_scale is null for 16-bit operands)
__device__ __forceinline__ float4 code_scale(float4 v, const GemmArgs& p, int n) {
    if (p.w_scale) {
        const float4 w = *reinterpret_cast<const float4*>(p.w_scale + n);
        v.x *= w.x * p.a_scale; v.y *= w.y * p.a_scale; v.z *= w.z * p.a_scale; v.w *= w.w * p.a_scale;
    }
    return v;
}

template <int EPI, int D>
__global__ void __launch_bounds__(256) gemm_finish_kernel(GemmArgs p) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)p.T * p.N;
    if (EPI == EPI_SWIGLU) {
        const int q_per_row = p.n_half / 4;
        if (i >= (int64_t)p.T * q_per_row) return;
        const int t = (int)(i / q_per_row), c = (int)(i % q_per_row) * 4;
        const float4 gt = code_scale(slab_sum(p.accum + (int64_t)t * p.N + c, stride, p.n_splits), p, c);
        const float4 up = code_scale(slab_sum(p.accum + (int64_t)t * p.N + p.n_half + c, stride, p.n_splits), p, p.n_half + c);
        const float o0 = silu_mul(gt.x, up.x), o1 = silu_mul(gt.y, up.y), o2 = silu_mul(gt.z, up.z), o3 = silu_mul(gt.w, up.w);
        if (p.out_f8) {
            const float sc = p.out_inv;
            *reinterpret_cast<uint32_t*>(static_cast<uint8_t*>(p.out) + (int64_t)t * p.n_half + c) = pack_fp8x4(o0 * sc, o1 * sc, o2 * sc, o3 * sc);
            return;
        }
        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.out) + (int64_t)t * p.n_half + c) =
            make_uint2(pack_bf16x2(o0, o1), pack_bf16x2(o2, o3));
    } else if (EPI == EPI_QKV_ROPE) {
        // units per token: rotated heads need (lo, hi) quads: (n_q + n_kv) * D / 8; v heads: n_kv * D / 4
        constexpr int HALF = (D > 0 ? D : 64) / 2;
        const int rot_units = (p.n_q + p.n_kv) * (HALF / 4), v_units = p.n_kv * (2 * HALF / 4);
        const int units = rot_units + v_units;
        if (i >= (int64_t)p.T * units) return;
        const int t = (int)(i / units), u = (int)(i % units);
        const int64_t slot = p.tok_slot[t];
        const int kv_dim = p.n_kv * 2 * HALF;
        const float* row = p.accum + (int64_t)t * p.N;
        if (u < rot_units) {
            const int head = u / (HALF / 4), i0 = (u % (HALF / 4)) * 4;
            const float4 lo = code_scale(slab_sum(row + head * 2 * HALF + i0, stride, p.n_splits), p, head * 2 * HALF + i0);
            const float4 hi = code_scale(slab_sum(row + head * 2 * HALF + HALF + i0, stride, p.n_splits), p, head * 2 * HALF + HALF + i0);
            const float2* cs = p.rope_cs + (int64_t)t * HALF + i0;
            const float4 c01 = *reinterpret_cast<const float4*>(cs), c23 = *reinterpret_cast<const float4*>(cs + 2);
            const float a[4] = {lo.x, lo.y, lo.z, lo.w}, b[4] = {hi.x, hi.y, hi.z, hi.w};
            const float co[4] = {c01.x, c01.z, c23.x, c23.z}, si[4] = {c01.y, c01.w, c23.y, c23.w};
            float l2[4], h2[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                l2[j] = a[j] * co[j] - b[j] * si[j];
                h2[j] = a[j] * si[j] + b[j] * co[j];
            }
            if (p.kv_fp8 && head >= p.n_q) {
                uint8_t* dst8 = reinterpret_cast<uint8_t*>(p.k_pages) + slot * kv_dim + (head - p.n_q) * 2 * HALF + i0;
                const float s = p.k_inv;
                *reinterpret_cast<uint32_t*>(dst8) = pack_fp8x4(l2[0] * s, l2[1] * s, l2[2] * s, l2[3] * s);
                *reinterpret_cast<uint32_t*>(dst8 + HALF) = pack_fp8x4(h2[0] * s, h2[1] * s, h2[2] * s, h2[3] * s);
                return;
            }
            uint16_t* dst = head < p.n_q ? static_cast<uint16_t*>(p.out) + (int64_t)t * (p.n_q * 2 * HALF) + head * 2 * HALF
                                         : p.k_pages + slot * kv_dim + (head - p.n_q) * 2 * HALF;
            *reinterpret_cast<uint2*>(dst + i0) = make_uint2(pack_bf16x2(l2[0], l2[1]), pack_bf16x2(l2[2], l2[3]));
            *reinterpret_cast<uint2*>(dst + HALF + i0) = make_uint2(pack_bf16x2(h2[0], h2[1]), pack_bf16x2(h2[2], h2[3]));
        } else {
            const int c = (u - rot_units) * 4;
            const float4 v = code_scale(slab_sum(row + (p.n_q + p.n_kv) * 2 * HALF + c, stride, p.n_splits), p, (p.n_q + p.n_kv) * 2 * HALF + c);
            if (p.kv_fp8) {
                const float s = p.v_inv;
                *reinterpret_cast<uint32_t*>(reinterpret_cast<uint8_t*>(p.v_pages) + slot * kv_dim + c) =
                    pack_fp8x4(v.x * s, v.y * s, v.z * s, v.w * s);
            } else {
                *reinterpret_cast<uint2*>(p.v_pages + slot * kv_dim + c) = make_uint2(pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w));
            }
        }
    } else {
        const int q_per_row = p.N / 4;
        if (i >= (int64_t)p.T * q_per_row) return;
        const int64_t o = i * 4;
        float4 v = code_scale(slab_sum(p.accum + o, stride, p.n_splits), p, (int)(i % q_per_row) * 4);
        if (EPI == EPI_RES_BF16_OUT_F32) {
            if (p.residual) {
                const uint2 r = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(p.residual) + o);
                v.x += bf16_lo(r.x); v.y += bf16_hi(r.x); v.z += bf16_lo(r.y); v.w += bf16_hi(r.y);
            }
            *reinterpret_cast<float4*>(static_cast<float*>(p.out) + o) = v;
        } else {
            if (EPI == EPI_RES_F32_OUT_BF16) {
                const float4 r = *reinterpret_cast<const float4*>(static_cast<const float*>(p.residual) + o);
                v.x += r.x; v.y += r.y; v.z += r.z; v.w += r.w;
            }
            *reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.out) + o) = make_uint2(pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w));
        }
    }
}

// Skinny path: T <= 256.  The weights are streamed once; to fill 256 CUs the k range of every
// BM x BN tile (BM = 64 / 128 tokens, BN = 128 / 256 features) is split over several workgroups, each
// storing its partial tile to its split's slab.  The LDS ring is as deep as 160 KB allow (one workgroup
// per CU); all stages but the one being computed are in flight.
template <int BM, int EPI, int D, int BN = 256, bool WNT = false>
hipError_t launch_split(GemmArgs p, int splits, hipStream_t s) {
    constexpr int NS = BM + BN <= 192 ? 6 : BM + BN <= 256 ? 4 : BM + BN <= 320 ? 4 : BM + BN <= 384 ? 3 : 2;
    constexpr int smem = NS * (BM + BN) * 64 * 2;
    static_assert(smem <= 160 * 1024, "ring exceeds the LDS");
    p.tiles_m = (p.T + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    const int nk = p.K / 64;
    p.k_per_split = (nk + splits - 1) / splits;
    splits = (nk + p.k_per_split - 1) / p.k_per_split;   // no empty split: the finish kernel reads every slab
    p.n_splits = splits;
    // the slabs [split][T, N] have to fit what the workspace reserves (a lower bound of it: this projection's own N)
    if ((int64_t)splits * p.T * p.N > gemm_scratch_floats(p.T, p.N)) return hipErrorInvalidValue;
    auto go = [&](auto f8) -> hipError_t {
        constexpr bool F8 = decltype(f8)::value;
        static std::once_flag once;
        static hipError_t attr_status = hipSuccess;
        if (hipError_t e = allow_smem_once(once, attr_status, &gemm_dma_kernel<BM, BN, EPI_SLAB, 0, 64, NS, 2, 2, WNT, F8>, smem)) return e;
        gemm_dma_kernel<BM, BN, EPI_SLAB, 0, 64, NS, 2, 2, WNT, F8><<<dim3(p.tiles_m * p.tiles_n * splits), dim3(256), smem, s>>>(p);
        return hipGetLastError();
    };
    hipError_t e = p.f8 ? go(std::true_type{}) : go(std::false_type{});
    if (e != hipSuccess) return e;
    int64_t units;
    if (EPI == EPI_SWIGLU)
        units = (int64_t)p.T * (p.n_half / 4);
    else if (EPI == EPI_QKV_ROPE)
        units = (int64_t)p.T * ((p.n_q + p.n_kv) * (D / 8) + p.n_kv * (D / 4));
    else
        units = (int64_t)p.T * (p.N / 4);
    gemm_finish_kernel<EPI, D><<<dim3((unsigned)((units + 255) / 256)), dim3(256), 0, s>>>(p);
    return hipGetLastError();
}

// Number of k splits for a skinny GEMM: enough workgroups for every CU, at least 4 k steps each.
int choose_splits(int T, int N, int K, int BM, int BN = 256) {
    const int tiles = ((T + BM - 1) / BM) * ((N + BN - 1) / BN);
    const int nk = K / 64;
    int splits = 256 / tiles;   // one workgroup per CU: a single full round
    splits = std::min(splits, std::max(1, nk / 4));
    return std::max(1, splits);
}

// The fused kernel on 128-feature tiles with a deep ring, one workgroup per CU: for a skinny GEMM whose
// tiles fill the CUs without any k split (the gate/up projection), so no slabs and no finish kernel.
template <int BM, int EPI, int D = 0, int BN = 128, bool WNT = true>
hipError_t launch_skinny_whole(GemmArgs p, hipStream_t s) {
    // (256 x 256 tiles have room for two 64-k stages only; four 32-k stages measured no faster)
    constexpr int BKD = 64;
    constexpr int NS = BM + BN <= 192 ? 6 : BM + BN <= 256 ? 4 : BM + BN <= 384 ? 3 : 2;
    constexpr int smem = NS * (BM + BN) * BKD * 2;
    static_assert(smem <= 160 * 1024, "ring exceeds the LDS");
    p.tiles_m = (p.T + BM - 1) / BM;
    p.tiles_n = EPI == EPI_SWIGLU ? (p.n_half + BN / 2 - 1) / (BN / 2) : (p.N + BN - 1) / BN;
    p.tail_tiles = 0;
    p.tail_splits = 1;
    auto go = [&](auto f8) -> hipError_t {
        constexpr bool F8 = decltype(f8)::value;
        static std::once_flag once;
        static hipError_t attr_status = hipSuccess;
        constexpr int GM = (F8 && BM == 256 && BN == 256) ? 4 : 2;   // eight waves for the largest 8-bit tile, as in launch_cfg
        if (hipError_t e = allow_smem_once(once, attr_status, &gemm_dma_kernel<BM, BN, EPI, D, BKD, NS, GM, 2, WNT, F8>, smem)) return e;
        gemm_dma_kernel<BM, BN, EPI, D, BKD, NS, GM, 2, WNT, F8><<<dim3(p.tiles_m * p.tiles_n), dim3(64 * GM * 2), smem, s>>>(p);
        return hipGetLastError();
    };
    return p.f8 ? go(std::true_type{}) : go(std::false_type{});
}

template <int EPI, int D>
hipError_t launch_skinny(const GemmArgs& p, hipStream_t s) {
    if (p.T <= 128) {
        // One token tile: the MFMA work is small next to the weight stream, so 128-feature tiles cost nothing
        // and need half the k splits (half the slab traffic); the gate/up projection has enough of them to
        // fill the CUs unsplit and runs the fused kernel.
        if constexpr (EPI == EPI_SWIGLU) {
            const int tiles = (p.n_half + 63) / 64, rounds = (tiles + 255) / 256;
            if (tiles >= 0.8 * 256 * rounds)
                return p.T <= 64 ? launch_skinny_whole<64, EPI>(p, s) : launch_skinny_whole<128, EPI>(p, s);
        }
        if (p.T <= 64) return launch_split<64, EPI, D, 128, true>(p, choose_splits(p.T, p.N, p.K, 64, 128), s);
        return launch_split<128, EPI, D, 128, true>(p, choose_splits(p.T, p.N, p.K, 128, 128), s);
    }
    // two token tiles: 256-feature tiles; a projection wide enough to need no k split runs the fused kernel
    const int splits = choose_splits(p.T, p.N, p.K, 128);
    if (splits == 1) {
        // wide enough that one 256 x 256 tile per CU is (nearly) a full round: one token tile instead of two
        // halves the weight fragments read from LDS per flop
        const int tiles256 = EPI == EPI_SWIGLU ? (p.n_half + 127) / 128 : (p.N + 255) / 256;
        if (p.T > 192 && tiles256 >= 200 && tiles256 <= 256) return launch_skinny_whole<256, EPI, D, 256>(p, s);
        return launch_skinny_whole<128, EPI, D, 256>(p, s);
    }
    return launch_split<128, EPI, D, 256, true>(p, splits, s);
}

bool skinny_applies(int T, int N, int K, const float* accum) {
    return accum != nullptr && T <= SKINNY_MAX_T && K % 64 == 0 && N % 4 == 0;
}

// Mid-size batches on a narrow output (W_o and W_down at a few hundred tokens): whole tiles are too few
// for 256 CUs and splitting them through the fenced partial-tile protocol costs more than it gains, so
// these run like the skinny path (k ranges stored to slabs, then the finish kernel) on tiles
// of 128 rows while every tile gets at least two k ranges, or of 256 rows while it gets at least three
// and k is long.  Returns the tile rows, 0 = not this path.  The slabs (at most 256 units x 256 x 256
// floats) use the tail scratch.
int split_rows(int T, int N, int K, bool has_accum) {
    if (!has_accum || T <= SKINNY_MAX_T || K % 64 || N % 4 || forced_cand() >= 0) return 0;
    const int tn = (N + 255) / 256;
    if (((T + 127) / 128) * tn <= 128) return 128;
    if (((T + 255) / 256) * tn <= 85 && K >= 8192) return 256;
    return 0;
}

template <int EPI>
hipError_t launch_mid_split(GemmArgs p, int bm, hipStream_t s) {
    if (bm == 128) return launch_split<128, EPI, 0>(p, choose_splits(p.T, p.N, p.K, 128), s);
    return launch_split<256, EPI, 0>(p, choose_splits(p.T, p.N, p.K, 256), s);
}

// What a launch does beyond whole tiles: the last tail_tiles tiles split their k range over `splits` workgroups.
struct Plan { int cand, tail_tiles, splits; };

template <int BM, int BN, int EPI, int D = 0, int WGM = 2, int WGN = 2>
hipError_t launch_cfg(const GemmArgs& base, hipStream_t s, const Plan& plan = Plan{0, 0, 1}) {
    GemmArgs p = base;
    p.tiles_m = (p.T + BM - 1) / BM;
    p.tiles_n = EPI == EPI_SWIGLU ? (p.n_half + BN / 2 - 1) / (BN / 2) : (p.N + BN - 1) / BN;
    constexpr int smem = 2 * (BM + BN) * BK * 2;
    // 128 x 256 tiles are one workgroup per CU either way, so they take the third stage that fits (144 KB)
    constexpr int DMA_BK = 64, DMA_NS = (BM == 128 && BN == 256) ? 3 : 2;
    constexpr int dma_smem = DMA_NS * (BM + BN) * DMA_BK * 2;
    const int tiles = p.tiles_m * p.tiles_n;
    if (p.K % 64 != 0) {
        if (p.f8) return hipErrorInvalidValue;   // codes go through the direct-to-LDS kernel only
        static std::once_flag once_generic;
        static hipError_t st_generic = hipSuccess;
        if (hipError_t e = allow_smem_once(once_generic, st_generic, &gemm_bf16_kernel<BM, BN, EPI, D>, smem)) return e;
        gemm_bf16_kernel<BM, BN, EPI, D><<<dim3(tiles), dim3(256), smem, s>>>(p);
        return hipGetLastError();
    }
    int grid = tiles;
    if (plan.tail_tiles > 0 && plan.splits > 1 && p.accum && p.T > SKINNY_MAX_T) {
        const int nk = p.K / 64;
        p.k_per_split = (nk + plan.splits - 1) / plan.splits;
        p.tail_splits = (nk + p.k_per_split - 1) / p.k_per_split;   // no empty split
        p.tail_tiles = std::min(plan.tail_tiles, tiles);
        p.tail_buf = p.accum;
        if ((int64_t)p.tail_tiles * p.tail_splits * BM * BN > kTailFloats)
            return hipErrorInvalidValue;   // a plan that does not fit the scratch: choose_plan never makes one
        grid = tiles - p.tail_tiles + p.tail_tiles * p.tail_splits;
    }
    auto go = [&](auto f8) -> hipError_t {
        constexpr bool F8 = decltype(f8)::value;
        // 8-bit operands on the largest tile: eight waves (two per SIMD, each with half the registers), so that one
        // wave's MFMAs cover the other's waits for its loads.  That kernel is bound by load latency (matrix pipes 58 %
        // busy with four waves); the 16-bit one is bound by the power limit and loses with eight waves (measured both).
        constexpr int GM = (F8 && BM == 256 && BN == 256) ? 4 : WGM;
        constexpr int GN = WGN;
        static std::once_flag once_dma;
        static hipError_t st_dma = hipSuccess;
        if (hipError_t e = allow_smem_once(once_dma, st_dma, &gemm_dma_kernel<BM, BN, EPI, D, DMA_BK, DMA_NS, GM, GN, false, F8>, dma_smem))
            return e;
        gemm_dma_kernel<BM, BN, EPI, D, DMA_BK, DMA_NS, GM, GN, false, F8>
            <<<dim3(grid), dim3(64 * GM * GN), dma_smem, s>>>(p);
        if (p.tail_tiles > 0) {
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
            gemm_tail_finish_kernel<BM, BN, EPI, D, GM, GN, F8>
                <<<dim3(p.tail_tiles * (BM / (32 * GM))), dim3(64 * GM * GN), 0, s>>>(p);
        }
        return hipGetLastError();
    };
    return p.f8 ? go(std::true_type{}) : go(std::false_type{});
}

// Tile choice.  A launch runs ceil(tiles / resident workgroups) rounds; the cost of a round is the
// tile's MFMA work divided by the tile shape's measured in-tile efficiency (relative to 256 x 256).
// The candidate with the lowest estimated cost wins: this trades tile quantisation in T (padding
// to BM), the tail round, and the per-tile efficiency against each other.
struct TileCand { int bm, bn, wg_per_cu; float eff; bool qkv; };   // qkv: usable by the fused q/k/v epilogue (128 features per wave)
constexpr TileCand kTiles[] = {
    // efficiencies from per-round times of forced plans at T = 288 ... 1282 on the 13B layer's projections
    {256, 256, 1, 1.00f, true}, {192, 256, 1, 0.92f, true}, {128, 256, 1, 0.68f, true}, {128, 128, 2, 0.76f, false},
    {64, 128, 3, 0.60f, false}};

// A tail (the tiles of the incomplete last round) may split its k range over workgroups, so that the
// round takes 1 / splits of a tile time; the price is that every partial tile is written to memory
// and read back by the workgroup that finishes the tile.  Costs in seconds.
constexpr double kCuFlops = 5.2e12;          // sustained MFMA rate of one CU inside a 256 x 256 tile
constexpr double kSlabBytesPerSec = 3.0e12;  // partial tiles through memory (written by the GEMM, read by the finish kernel)
constexpr double kTailFinishSec = 6e-6;      // the finish kernel's launch and ramp

Plan choose_plan(int T, int64_t n_eff, int K, bool need_bn256, bool allow_tail) {
    const int n_cand = (int)(sizeof(kTiles) / sizeof(kTiles[0]));
    const int f_cand = forced_cand(), f_splits = forced_splits();
    const bool force = f_cand >= 0 && f_cand < n_cand;
    Plan best{0, 0, 1};
    double best_cost = 1e300;
    for (int i = 0; i < n_cand; ++i) {
        const TileCand& c = kTiles[i];
        int forced_splits = 0;
        if (need_bn256 && !c.qkv) continue;
        if (force) {
            if (f_cand != i && !(need_bn256 && !kTiles[f_cand].qkv)) continue;
            if (f_cand == i) forced_splits = f_splits;
        }
        const double eff = c.eff;
        const int64_t tiles = ((T + c.bm - 1) / c.bm) * ((n_eff + c.bn - 1) / c.bn);
        const int64_t slots = 256 * c.wg_per_cu;
        // resident workgroups of a CU share its MFMA pipes: a round of wg_per_cu tiles costs wg_per_cu tile times
        double t_round = c.wg_per_cu * 2.0 * c.bm * c.bn * (double)K / (eff * kCuFlops);
        // a launch that leaves CUs idle runs its big tiles faster (the chip is power-limited: up to 2.2 GHz
        // instead of ~1.9); the small tiles are bound by L2 traffic and gain nothing
        if (tiles < slots && c.bm >= 192) t_round /= 1.0 + 0.25 * (1.0 - (double)tiles / (double)slots);
        const int64_t full = tiles / slots, rem = tiles % slots;
        const double whole = (double)(full + (rem ? 1 : 0)) * t_round;
        if (whole < best_cost && forced_splits <= 1) best_cost = whole, best = Plan{i, 0, 1};
        const int nk = K / 64;
        // tiles that share a CU (two or three workgroups) gained nothing from split tails in any measured case
        const bool can_tail = allow_tail && rem > 0 && K % 64 == 0 && (c.wg_per_cu == 1 || forced_splits > 1);
        for (int sp = 2; can_tail && sp <= 8 && nk / sp >= 8; ++sp) {
            if (forced_splits > 1 && sp != forced_splits) continue;
            const int64_t units = rem * sp;
            if (units * c.bm * c.bn > kTailFloats) break;
            const double rounds = (double)((units + slots - 1) / slots);
            const double slabs = (double)units * c.bm * c.bn * 4.0 * 2.0 / kSlabBytesPerSec;
            const double cost = full * t_round + rounds * t_round / sp + slabs + kTailFinishSec;
            if (cost < best_cost || forced_splits > 1) best_cost = cost, best = Plan{i, (int)rem, sp};
        }
    }
    return best;
}

template <int EPI>
hipError_t launch_epi(const GemmArgs& p, hipStream_t s) {
    const int64_t n_eff = EPI == EPI_SWIGLU ? 2 * (int64_t)p.n_half : p.N;
    const Plan plan = choose_plan(p.T, n_eff, p.K, false, p.accum != nullptr);
    switch (plan.cand) {
        case 0: return launch_cfg<256, 256, EPI>(p, s, plan);
        case 1: return launch_cfg<192, 256, EPI>(p, s, plan);
        case 2: return launch_cfg<128, 256, EPI>(p, s, plan);
        case 3: return launch_cfg<128, 128, EPI>(p, s, plan);
        default: return launch_cfg<64, 128, EPI>(p, s, plan);
    }
}

}  // namespace

void gemm_force_plan(int cand, int splits) {
    g_forced_plan.store(cand < 0 ? -1 : (cand | (splits << 8)), std::memory_order_relaxed);
}

int64_t gemm_scratch_floats(int64_t T, int64_t n_max) {
    // skinny: one slab per split, at most 256 units of 128 x 256 floats, or a single slab of T x N
    return T <= SKINNY_MAX_T ? std::max<int64_t>(T * n_max, 256 * 128 * 256) : kTailFloats;
}


// Tiled weight layout for streaming: out[n / 256][k / 64][n % 256][k % 64], rows past N are zeros.  One k
// slice of 256 rows is 32 KB of consecutive memory, so a stage of the GEMM reads whole DRAM pages
// instead of 128-byte pieces 2 K bytes apart.
__global__ void pack_weight_kernel(const uint4* w, uint4* out, int32_t N, int32_t K, int64_t n_chunks) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // 16-byte chunk of the output
    if (i >= n_chunks) return;
    const int c = (int)(i & 7), r = (int)((i >> 3) & 255);
    const int64_t slice = i >> 11;                                       // (block, k slice)
    const int ks = (int)(slice % (K / 64));
    const int64_t n = (slice / (K / 64)) * 256 + r;
    out[i] = n < N ? w[(n * K + ks * 64) / 8 + c] : make_uint4(0, 0, 0, 0);
}

hipError_t launch_pack_weight(const void* w, int32_t N, int32_t K, void* out, hipStream_t s) {
    const int64_t n_chunks = (int64_t)((N + 255) / 256) * 256 * K / 8;
    if (n_chunks == 0) return hipSuccess;
    pack_weight_kernel<<<dim3((unsigned)((n_chunks + 255) / 256)), dim3(256), 0, s>>>(
        static_cast<const uint4*>(w), static_cast<uint4*>(out), N, K, n_chunks);
    return hipGetLastError();
}


// 8-bit operands: the kernels see rows of K / 2 two-byte units (same bytes, same layouts) and the scales
static hipError_t set_codes(GemmArgs& p, const CodeScales* codes) {
    if (!codes) return hipSuccess;
    if (p.K % 128 || !codes->w_scale || !(codes->a_scale > 0.0f)) return hipErrorInvalidValue;
    p.f8 = 1;
    p.K /= 2;
    p.w_scale = codes->w_scale;
    p.a_scale = codes->a_scale;
    p.out_f8 = codes->out_scale > 0.0f ? 1 : 0;
    p.out_inv = p.out_f8 ? (float)(1.0 / (double)codes->out_scale) : 0.0f;   // reciprocal in double, rounded once
    return hipSuccess;
}

hipError_t launch_linear(const void* a, const void* w, int32_t T, int32_t N, int32_t K, int32_t epilogue,
                         const void* residual, void* out, hipStream_t s, float* accum, bool w_packed, const CodeScales* codes) {
    if (T == 0) return hipSuccess;
    if ((int64_t)T * K >= ((int64_t)1 << 31) || (int64_t)N * K >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
    if (epilogue != EPI_SWIGLU && (N % 4)) return hipErrorInvalidValue;
    if (epilogue == EPI_SWIGLU && ((N / 2) % 8)) return hipErrorInvalidValue;
    if (w_packed && K % 64) return hipErrorInvalidValue;   // only the direct-to-LDS kernel reads it
    GemmArgs p{};
    p.w_packed = w_packed;
    p.a = static_cast<const uint16_t*>(a);
    p.w = static_cast<const uint16_t*>(w);
    p.residual = residual;
    p.out = out;
    p.T = T;
    p.N = N;
    p.K = K;
    p.n_half = N / 2;
    p.accum = accum;
    if (hipError_t e = set_codes(p, codes)) return e;
    K = p.K;
    if (skinny_applies(T, N, K, accum)) {
        switch (epilogue) {
            case EPI_BF16: return launch_skinny<EPI_BF16, 0>(p, s);
            case EPI_RES_BF16_OUT_F32: return launch_skinny<EPI_RES_BF16_OUT_F32, 0>(p, s);
            case EPI_RES_F32_OUT_BF16: return launch_skinny<EPI_RES_F32_OUT_BF16, 0>(p, s);
            case EPI_SWIGLU: return launch_skinny<EPI_SWIGLU, 0>(p, s);
            default: return hipErrorInvalidValue;
        }
    }
    if (const int bm = split_rows(T, N, K, accum != nullptr)) {
        switch (epilogue) {
            case EPI_BF16: return launch_mid_split<EPI_BF16>(p, bm, s);
            case EPI_RES_BF16_OUT_F32: return launch_mid_split<EPI_RES_BF16_OUT_F32>(p, bm, s);
            case EPI_RES_F32_OUT_BF16: return launch_mid_split<EPI_RES_F32_OUT_BF16>(p, bm, s);
            case EPI_SWIGLU: return launch_mid_split<EPI_SWIGLU>(p, bm, s);
            default: return hipErrorInvalidValue;
        }
    }
    switch (epilogue) {
        case EPI_BF16: return launch_epi<EPI_BF16>(p, s);
        case EPI_RES_BF16_OUT_F32: return launch_epi<EPI_RES_BF16_OUT_F32>(p, s);
        case EPI_RES_F32_OUT_BF16: return launch_epi<EPI_RES_F32_OUT_BF16>(p, s);
        case EPI_SWIGLU: return launch_epi<EPI_SWIGLU>(p, s);
        default: return hipErrorInvalidValue;
    }
}

namespace {
template <int D>
hipError_t launch_qkv_d(const GemmArgs& p, hipStream_t s) {
    if (p.T <= 64) return launch_cfg<64, 256, EPI_QKV_ROPE, D>(p, s);
    const Plan plan = choose_plan(p.T, p.N, p.K, true, p.accum != nullptr);   // the rotation needs 128 features per wave
    switch (plan.cand) {
        case 0: return launch_cfg<256, 256, EPI_QKV_ROPE, D>(p, s, plan);
        case 1: return launch_cfg<192, 256, EPI_QKV_ROPE, D>(p, s, plan);
        default: return launch_cfg<128, 256, EPI_QKV_ROPE, D>(p, s, plan);
    }
}
}  // namespace

hipError_t launch_qkv_rope_append(const BatchDev& b, const relserve_layer& L, const void* h, const void* w_qkv,
                                  void* q_out, void* k_pages, void* v_pages, hipStream_t s, float* accum,
                                  bool w_packed, KvFormat kv, const CodeScales* codes) {
    if (b.T == 0) return hipSuccess;
    const int32_t K = L.cfg.hidden;
    if ((int64_t)b.T * K >= ((int64_t)1 << 31) || (int64_t)L.qkv_dim * K >= ((int64_t)1 << 31))
        return hipErrorInvalidValue;
    GemmArgs p{};
    if (w_packed && K % 64) return hipErrorInvalidValue;
    p.w_packed = w_packed;
    p.a = static_cast<const uint16_t*>(h);
    p.w = static_cast<const uint16_t*>(w_qkv);
    p.out = q_out;
    p.T = b.T;
    p.N = L.qkv_dim;
    p.K = K;
    p.tok_slot = b.tok_slot;
    p.rope_cs = b.rope_cs;
    p.k_pages = static_cast<uint16_t*>(k_pages);
    p.v_pages = static_cast<uint16_t*>(v_pages);
    p.n_q = L.cfg.n_q_heads;
    p.n_kv = L.cfg.n_kv_heads;
    p.kv_fp8 = kv.fp8 ? 1 : 0;
    p.k_inv = (float)(1.0 / (double)kv.k_scale);      // reciprocal in double, rounded once
    p.v_inv = (float)(1.0 / (double)kv.v_scale);
    p.accum = accum;
    if (hipError_t e = set_codes(p, codes)) return e;
    if (skinny_applies(p.T, p.N, p.K, accum))
        return L.cfg.head_dim == 128 ? launch_skinny<EPI_QKV_ROPE, 128>(p, s) : launch_skinny<EPI_QKV_ROPE, 64>(p, s);
    return L.cfg.head_dim == 128 ? launch_qkv_d<128>(p, s) : launch_qkv_d<64>(p, s);
}

}  // namespace relserve
