// HBM-bound helper kernels of the layer step: rotary table, RMSNorm, rotary embedding +
// KV append, and the stand-alone KV append.  All are pure streaming kernels: 16-byte
// accesses per lane, one pass over the data (RMSNorm re-reads its row from cache).
#include "device_utils.h"
#include "relserve_internal.h"

namespace relserve {

// ---- rotary (cos, sin) table: one entry per (token, frequency) ----------------------------
__global__ void rope_table_kernel(const int32_t* __restrict__ tok_pos, const float* __restrict__ inv_freq,
                                  int32_t T, int32_t half, float2* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)T * half) return;
    const int32_t t = (int32_t)(i / half), f = (int32_t)(i % half);
    const float ang = (float)tok_pos[t] * inv_freq[f];
    float s, c;
    sincosf(ang, &s, &c);
    out[i] = make_float2(c, s);
}

hipError_t launch_rope_table(const int32_t* tok_pos, const float* inv_freq_dev, int32_t T, int32_t half,
                             float2* out, hipStream_t s) {
    const int64_t n = (int64_t)T * half;
    if (n == 0) return hipSuccess;
    rope_table_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(tok_pos, inv_freq_dev, T, half, out);
    return hipGetLastError();
}

// ---- RMSNorm: one workgroup per row --------------------------------------------------------
template <bool IN_F32>
__global__ void __launch_bounds__(256) rmsnorm_kernel(const void* __restrict__ xv, const uint16_t* __restrict__ w,
                                                      float eps, int32_t H, uint16_t* __restrict__ out,
                                                      const int32_t* __restrict__ row_index, float code_inv) {
    const int64_t orow = blockIdx.x;
    const int64_t row = row_index ? row_index[orow] : orow;  // optional gather of the input row
    const int tid = threadIdx.x;
    __shared__ float red[4];
    float ss = 0.f;
    const int chunks = H / 8;
    auto load8 = [&](int c, float* v) {
        if (IN_F32) {
            const float4* p = reinterpret_cast<const float4*>(static_cast<const float*>(xv) + row * H + (int64_t)c * 8);
            float4 a = p[0], b = p[1];
            v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
        } else {
            const uint4 u = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(xv) + row * H + (int64_t)c * 8);
            v[0] = bf16_lo(u.x); v[1] = bf16_hi(u.x); v[2] = bf16_lo(u.y); v[3] = bf16_hi(u.y);
            v[4] = bf16_lo(u.z); v[5] = bf16_hi(u.z); v[6] = bf16_lo(u.w); v[7] = bf16_hi(u.w);
        }
    };
    for (int c = tid; c < chunks; c += 256) {
        float v[8];
        load8(c, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) ss += v[i] * v[i];
    }
    ss = wave_sum(ss);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    const float tot = red[0] + red[1] + red[2] + red[3];
    const float inv = 1.0f / sqrtf(tot / (float)H + eps);
    for (int c = tid; c < chunks; c += 256) {
        float v[8];
        load8(c, v);
        const uint4 wu = *reinterpret_cast<const uint4*>(w + (int64_t)c * 8);
        if (code_inv > 0.0f) {   // quantised projections read 8-bit codes of the normed value / scale, taken from fp32
            const float s = code_inv;
            uint2 o8;
            o8.x = pack_fp8x4(v[0] * inv * bf16_lo(wu.x) * s, v[1] * inv * bf16_hi(wu.x) * s, v[2] * inv * bf16_lo(wu.y) * s,
                              v[3] * inv * bf16_hi(wu.y) * s);
            o8.y = pack_fp8x4(v[4] * inv * bf16_lo(wu.z) * s, v[5] * inv * bf16_hi(wu.z) * s, v[6] * inv * bf16_lo(wu.w) * s,
                              v[7] * inv * bf16_hi(wu.w) * s);
            *reinterpret_cast<uint2*>(reinterpret_cast<uint8_t*>(out) + orow * H + (int64_t)c * 8) = o8;
            continue;
        }
        uint4 o;
        o.x = pack_bf16x2(v[0] * inv * bf16_lo(wu.x), v[1] * inv * bf16_hi(wu.x));
        o.y = pack_bf16x2(v[2] * inv * bf16_lo(wu.y), v[3] * inv * bf16_hi(wu.y));
        o.z = pack_bf16x2(v[4] * inv * bf16_lo(wu.z), v[5] * inv * bf16_hi(wu.z));
        o.w = pack_bf16x2(v[6] * inv * bf16_lo(wu.w), v[7] * inv * bf16_hi(wu.w));
        *reinterpret_cast<uint4*>(out + orow * H + (int64_t)c * 8) = o;
    }
}

hipError_t launch_rmsnorm(const void* x, bool x_is_f32, const void* w, float eps, int32_t rows, int32_t H,
                          void* out, hipStream_t s, const int32_t* row_index, float code_scale) {
    if (rows == 0) return hipSuccess;
    const float code_inv = code_scale > 0.0f ? (float)(1.0 / (double)code_scale) : 0.0f;   // reciprocal in double, rounded once
    if (x_is_f32)
        rmsnorm_kernel<true><<<dim3(rows), dim3(256), 0, s>>>(x, static_cast<const uint16_t*>(w), eps, H,
                                                              static_cast<uint16_t*>(out), row_index, code_inv);
    else
        rmsnorm_kernel<false><<<dim3(rows), dim3(256), 0, s>>>(x, static_cast<const uint16_t*>(w), eps, H,
                                                               static_cast<uint16_t*>(out), row_index, code_inv);
    return hipGetLastError();
}

// ---- bf16 -> 8-bit codes of value / scale (the attention output on its way into a quantised W_o) ------------
__global__ void __launch_bounds__(256) quantise_bf16_kernel(const uint4* __restrict__ in, int64_t n8, float inv,
                                                            uint2* __restrict__ codes) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n8) return;
    const uint4 u = in[i];
    uint2 o;
    o.x = pack_fp8x4(bf16_lo(u.x) * inv, bf16_hi(u.x) * inv, bf16_lo(u.y) * inv, bf16_hi(u.y) * inv);
    o.y = pack_fp8x4(bf16_lo(u.z) * inv, bf16_hi(u.z) * inv, bf16_lo(u.w) * inv, bf16_hi(u.w) * inv);
    codes[i] = o;
}

hipError_t launch_quantise_bf16(const void* in, int64_t n, float scale, void* codes, hipStream_t s) {
    if (n == 0) return hipSuccess;
    if (n % 8 || !(scale > 0.0f)) return hipErrorInvalidValue;
    const int64_t n8 = n / 8;
    quantise_bf16_kernel<<<dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, s>>>(
        static_cast<const uint4*>(in), n8, (float)(1.0 / (double)scale), static_cast<uint2*>(codes));
    return hipGetLastError();
}

// ---- embedding gather: x[t, :] = table[clamp(id[t]), :] -----------------------------------
__global__ void embedding_kernel(const int32_t* __restrict__ ids, const uint4* __restrict__ table, int32_t vocab,
                                 int32_t row_chunks, int32_t T, uint4* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)T * row_chunks) return;
    const int32_t t = (int32_t)(i / row_chunks), c = (int32_t)(i % row_chunks);
    const int32_t id = min(max(ids[t], 0), vocab - 1);  // ids are the caller's contract; never read outside the table
    out[i] = table[(int64_t)id * row_chunks + c];
}

hipError_t launch_embedding(const int32_t* ids, const void* table, int32_t vocab, int32_t H, int32_t T, void* out,
                            hipStream_t s) {
    const int64_t n = (int64_t)T * (H / 8);
    if (n == 0) return hipSuccess;
    embedding_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(
        ids, static_cast<const uint4*>(table), vocab, H / 8, T, static_cast<uint4*>(out));
    return hipGetLastError();
}

// ---- stand-alone KV append: copy rows into their slots -----------------------------------
__global__ void kv_append_kernel(const int32_t* __restrict__ tok_slot, const uint4* __restrict__ k,
                                 const uint4* __restrict__ v, uint4* __restrict__ k_pages,
                                 uint4* __restrict__ v_pages, int32_t T, int32_t row_chunks) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)T * row_chunks) return;
    const int32_t t = (int32_t)(i / row_chunks), c = (int32_t)(i % row_chunks);
    const int64_t dst = (int64_t)tok_slot[t] * row_chunks + c;
    k_pages[dst] = k[i];
    v_pages[dst] = v[i];
}

hipError_t launch_kv_append(const BatchDev& b, const void* k, const void* v, void* k_pages, void* v_pages,
                            int32_t row_elems, hipStream_t s) {
    const int32_t row_chunks = row_elems / 8;
    const int64_t n = (int64_t)b.T * row_chunks;
    if (n == 0) return hipSuccess;
    kv_append_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(
        b.tok_slot, static_cast<const uint4*>(k), static_cast<const uint4*>(v), static_cast<uint4*>(k_pages),
        static_cast<uint4*>(v_pages), b.T, row_chunks);
    return hipGetLastError();
}

// ---- rotary embedding of q (in place) and k (into the cache), v copied into the cache -------
// One workgroup per token.  A unit of work is 8 rotation pairs of one head (two 16-byte
// pieces, columns i..i+7 and i+d/2..i+d/2+7) or one 16-byte piece of v.
__global__ void __launch_bounds__(256) rope_append_kernel(const int32_t* __restrict__ tok_slot,
                                                          const float2* __restrict__ rope_cs,
                                                          uint16_t* __restrict__ qkv, uint16_t* __restrict__ k_pages,
                                                          uint16_t* __restrict__ v_pages, int32_t n_q, int32_t n_kv,
                                                          int32_t d) {
    const int64_t t = blockIdx.x;
    const int32_t half = d / 2, upc = half / 8;  // units per rotated head
    const int32_t qkv_dim = (n_q + 2 * n_kv) * d, kv_dim = n_kv * d;
    uint16_t* row = qkv + t * qkv_dim;
    const int64_t slot = tok_slot[t];
    const float2* cs = rope_cs + t * half;
    const int32_t rot_units = (n_q + n_kv) * upc, v_units = kv_dim / 8;
    for (int32_t u = threadIdx.x; u < rot_units + v_units; u += 256) {
        if (u < rot_units) {
            const int32_t head = u / upc, i0 = (u % upc) * 8;
            uint16_t* src = row + (int64_t)head * d + i0;
            const uint4 lo = *reinterpret_cast<const uint4*>(src);
            const uint4 hi = *reinterpret_cast<const uint4*>(src + half);
            const uint32_t lw[4] = {lo.x, lo.y, lo.z, lo.w}, hw[4] = {hi.x, hi.y, hi.z, hi.w};
            uint32_t ol[4], oh[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float2 c0 = cs[i0 + 2 * j], c1 = cs[i0 + 2 * j + 1];
                const float a0 = bf16_lo(lw[j]), a1 = bf16_hi(lw[j]);
                const float b0 = bf16_lo(hw[j]), b1 = bf16_hi(hw[j]);
                ol[j] = pack_bf16x2(a0 * c0.x - b0 * c0.y, a1 * c1.x - b1 * c1.y);
                oh[j] = pack_bf16x2(a0 * c0.y + b0 * c0.x, a1 * c1.y + b1 * c1.x);
            }
            uint16_t* dst = src;  // q: in place
            if (head >= n_q) dst = k_pages + slot * kv_dim + (int64_t)(head - n_q) * d + i0;
            *reinterpret_cast<uint4*>(dst) = make_uint4(ol[0], ol[1], ol[2], ol[3]);
            *reinterpret_cast<uint4*>(dst + half) = make_uint4(oh[0], oh[1], oh[2], oh[3]);
        } else {
            const int32_t c = u - rot_units;
            const uint4 val = *reinterpret_cast<const uint4*>(row + (int64_t)(n_q + n_kv) * d + (int64_t)c * 8);
            *reinterpret_cast<uint4*>(v_pages + slot * kv_dim + (int64_t)c * 8) = val;
        }
    }
}

hipError_t launch_rope_append(const BatchDev& b, const relserve_layer& L, void* qkv, void* k_pages,
                              void* v_pages, hipStream_t s) {
    if (b.T == 0) return hipSuccess;
    rope_append_kernel<<<dim3(b.T), dim3(256), 0, s>>>(b.tok_slot, b.rope_cs, static_cast<uint16_t*>(qkv),
                                                       static_cast<uint16_t*>(k_pages),
                                                       static_cast<uint16_t*>(v_pages), L.cfg.n_q_heads,
                                                       L.cfg.n_kv_heads, L.cfg.head_dim);
    return hipGetLastError();
}

// ---- greedy next token: first largest logit of every row ------------------------------------
// One workgroup per row.  A candidate (value, id) beats another if its value is larger, or equal with a lower id;
// NaN never competes; a row without any number gives id 0.
__device__ __forceinline__ void greedy_take(float& bv, int32_t& bi, float v, int32_t i) {
    if (v > bv || (v == bv && i < bi)) bv = v, bi = i;
}

__global__ void __launch_bounds__(256) greedy_sample_kernel(const float* __restrict__ logits, int32_t vocab,
                                                            int32_t* __restrict__ next_token) {
    const float* row = logits + (int64_t)blockIdx.x * vocab;
    const int tid = threadIdx.x;
    float bv = -INFINITY;
    int32_t bi = INT32_MAX;
    const int32_t n4 = (reinterpret_cast<uintptr_t>(row) % 16 == 0) ? vocab / 4 : 0;   // 16-byte loads when the row allows
    for (int32_t c = tid; c < n4; c += 256) {
        const float4 v = reinterpret_cast<const float4*>(row)[c];
        greedy_take(bv, bi, v.x, 4 * c);
        greedy_take(bv, bi, v.y, 4 * c + 1);
        greedy_take(bv, bi, v.z, 4 * c + 2);
        greedy_take(bv, bi, v.w, 4 * c + 3);
    }
    for (int32_t i = 4 * n4 + tid; i < vocab; i += 256) greedy_take(bv, bi, row[i], i);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) greedy_take(bv, bi, __shfl_xor(bv, o, 64), __shfl_xor(bi, o, 64));
    __shared__ float sv[4];
    __shared__ int32_t si[4];
    if ((tid & 63) == 0) sv[tid >> 6] = bv, si[tid >> 6] = bi;
    __syncthreads();
    if (tid == 0) {
#pragma unroll
        for (int w = 1; w < 4; ++w) greedy_take(bv, bi, sv[w], si[w]);
        next_token[blockIdx.x] = bi == INT32_MAX ? 0 : bi;
    }
}

hipError_t launch_greedy_sample(const float* logits, int32_t n_rows, int32_t vocab, int32_t* next_token, hipStream_t s) {
    if (n_rows == 0) return hipSuccess;
    greedy_sample_kernel<<<dim3(n_rows), dim3(256), 0, s>>>(logits, vocab, next_token);
    return hipGetLastError();
}

}  // namespace relserve
