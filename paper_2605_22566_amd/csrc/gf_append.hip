// gf_kv_append: write the K/V of every request's new tokens into its private tail
// blocks (paper, Topology-Aware State Management: the states produced at run time
// extend the KV assembled from the operation nodes; Effective Path Pruning: a state
// that is not stored is computed on the fly and then put where attention reads it).
//
// One workgroup per (request, tail block).  K keeps its token-major order inside the
// block, so its rows are copied with 16-byte loads and stores.  V is stored
// head-dim-major: one kv head at a time, the 16 x D tile of the new tokens goes
// through LDS and comes out as D rows of 16 slots.  Slots beyond the block's token
// count are written as zero.  With an e4m3 pool the block's two scales come first
// (amax over the block's valid tokens / 448, workgroup reduction), then every value
// is divided by its scale in fp32, clamped to +-448 and rounded to e4m3.
#include "gf_internal.h"

namespace gf {

constexpr int kAppendThreads = 256;

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// 8 bf16 (one 16-byte chunk) -> 8 e4m3 codes (two dwords), x / scale clamped to the finite range
__device__ __forceinline__ u32x2 quantize8(u32x4 raw, float scale) {
    float x[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x[2 * i] = bf16_bits_to_float(raw[i] & 0xffffu);
        x[2 * i + 1] = bf16_bits_to_float(raw[i] >> 16);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = fminf(fmaxf(x[i] / scale, -448.0f), 448.0f);
    u32x2 out;
    int w = 0;
    w = __builtin_amdgcn_cvt_pk_fp8_f32(x[0], x[1], w, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(x[2], x[3], w, true);
    out[0] = (uint32_t)w;
    w = 0;
    w = __builtin_amdgcn_cvt_pk_fp8_f32(x[4], x[5], w, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(x[6], x[7], w, true);
    out[1] = (uint32_t)w;
    return out;
}

template <int D, bool FP8>
__global__ __launch_bounds__(kAppendThreads) void append_kernel(
    void *__restrict__ k_pool, void *__restrict__ v_pool, float *__restrict__ k_scale, float *__restrict__ v_scale,
    int pool_blocks, int hkv, const int32_t *__restrict__ block_table, const int32_t *__restrict__ num_blocks,
    const int32_t *__restrict__ ctx_lens, const int32_t *__restrict__ seq_lens, const int32_t *__restrict__ status,
    int max_blocks, const uint16_t *__restrict__ k_new, const uint16_t *__restrict__ v_new,
    const int32_t *__restrict__ q_ptr, int total_q) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[kBlock][D];      // one kv head of V, token-major
    __shared__ float red[2][kAppendThreads / 64];
    const int r = blockIdx.x, j = blockIdx.y;
    const int tid = threadIdx.x;
    if (status && status[r] != 0) return;
    const int n = seq_lens[r] - ctx_lens[r];
    if (n <= 0 || kBlock * j >= n) return;
    const int q0 = q_ptr[r];
    if (q_ptr[r + 1] - q0 != n || q0 < 0 || q0 + n > total_q) return;
    const int nb = min(num_blocks[r], max_blocks);
    const int ntail = (n + kBlock - 1) / kBlock;
    const int e = nb - ntail + j;
    if (e < 0) return;
    const int blk = block_table[(size_t)r * max_blocks + e];
    if (blk < 0 || blk >= pool_blocks) return;
    const int ntok = min(kBlock, n - kBlock * j);
    const size_t row_elems = (size_t)hkv * D;                               // elements of one token
    const uint16_t *ksrc = k_new + (size_t)(q0 + kBlock * j) * row_elems;
    const uint16_t *vsrc = v_new + (size_t)(q0 + kBlock * j) * row_elems;

    float sk = 1.f, sv = 1.f;
    if constexpr (FP8) {
        // block scales: amax over the valid tokens of the block (rows of a token are contiguous)
        float ak = 0.f, av = 0.f;
        const size_t chunks = (size_t)ntok * row_elems / 8;
        for (size_t c = tid; c < chunks; c += kAppendThreads) {
            const u32x4 a = *(const u32x4 *)(ksrc + 8 * c), b = *(const u32x4 *)(vsrc + 8 * c);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ak = fmaxf(ak, fmaxf(fabsf(bf16_bits_to_float(a[i] & 0xffffu)), fabsf(bf16_bits_to_float(a[i] >> 16))));
                av = fmaxf(av, fmaxf(fabsf(bf16_bits_to_float(b[i] & 0xffffu)), fabsf(bf16_bits_to_float(b[i] >> 16))));
            }
        }
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) {
            ak = fmaxf(ak, __shfl_xor(ak, o, 64));
            av = fmaxf(av, __shfl_xor(av, o, 64));
        }
        if ((tid & 63) == 0) {
            red[0][tid >> 6] = ak;
            red[1][tid >> 6] = av;
        }
        __syncthreads();
        ak = fmaxf(fmaxf(red[0][0], red[0][1]), fmaxf(red[0][2], red[0][3]));
        av = fmaxf(fmaxf(red[1][0], red[1][1]), fmaxf(red[1][2], red[1][3]));
        sk = ak > 0.f ? ak / 448.0f : 1.0f;
        sv = av > 0.f ? av / 448.0f : 1.0f;
        if (tid == 0) {
            k_scale[blk] = sk;
            v_scale[blk] = sv;
        }
    }

    // K: destination image [h][slot][d]; chunk c = ((h * 16 + slot) * D + d8) / 8
    {
        const int chunks = hkv * kBlock * D / 8;
        for (int c = tid; c < chunks; c += kAppendThreads) {
            const int d8 = (c % (D / 8)) * 8, slot = (c / (D / 8)) % kBlock, h = c / (D / 8 * kBlock);
            u32x4 raw = {0, 0, 0, 0};
            if (slot < ntok) raw = *(const u32x4 *)(ksrc + (size_t)slot * row_elems + h * D + d8);
            if constexpr (FP8) {
                u32x2 q = {0, 0};
                if (slot < ntok) q = quantize8(raw, sk);
                *(u32x2 *)((uint8_t *)k_pool + (size_t)blk * hkv * kBlock * D + (size_t)c * 8) = q;
            } else {
                *(u32x4 *)((uint16_t *)k_pool + (size_t)blk * hkv * kBlock * D + (size_t)c * 8) = raw;
            }
        }
    }
    // V: destination image [h][d][slot], one kv head at a time through LDS
    for (int h = 0; h < hkv; ++h) {
        __syncthreads();
        for (int c = tid; c < kBlock * D / 8; c += kAppendThreads) {
            const int d8 = (c % (D / 8)) * 8, slot = c / (D / 8);
            u32x4 raw = {0, 0, 0, 0};
            if (slot < ntok) raw = *(const u32x4 *)(vsrc + (size_t)slot * row_elems + h * D + d8);
            *(u32x4 *)(&tile[slot][d8]) = raw;
        }
        __syncthreads();
        // thread (d, half) gathers slots 8 half .. 8 half + 7 of head-dim row d
        for (int t = tid; t < 2 * D; t += kAppendThreads) {
            const int d = t % D, half = t / D;
            u32x4 raw;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                raw[i] = (uint32_t)tile[8 * half + 2 * i][d] | ((uint32_t)tile[8 * half + 2 * i + 1][d] << 16);
            const size_t row = ((size_t)blk * hkv + h) * D + d;             // head-dim row of the V pool
            if constexpr (FP8) {
                // pad slots hold zero bits: they quantise to code 0 under any scale
                *(u32x2 *)((uint8_t *)v_pool + row * kBlock + 8 * half) = quantize8(raw, sv);
            } else {
                *(u32x4 *)((uint16_t *)v_pool + row * kBlock + 8 * half) = raw;
            }
        }
    }
}

// ---- decode-step form: one token per request --------------------------------------------------
// gf_kv_append_token.  One workgroup per request: the newest token's K row and V column go into slot
// s = (n - 1) % 16 of the request's last table entry.  s == 0 opens a fresh block, written whole (zeros
// beside the token).  An e4m3 block grows in place: the token's amax / 448 is compared with the block's
// scale (per tensor); if it is larger the scale is raised to it and the codes already in slots [0, s) are
// decoded, multiplied by the old scale, divided by the new one (fp32) and rounded again; the token is then
// coded with the block's scale.  V is handled one head-dim row (16 slots) per thread, so that a row is only
// ever written by one thread.

// 8 e4m3 codes -> 8 floats (exact)
__device__ __forceinline__ void decode8(u32x2 w, float *x) {
    const bf16x8 b = fp8x8_to_bf16x8(w);
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = (float)b[i];
}
__device__ __forceinline__ u32x2 encode8(const float *x) {
    u32x2 out;
    int w = 0;
    w = __builtin_amdgcn_cvt_pk_fp8_f32(x[0], x[1], w, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(x[2], x[3], w, true);
    out[0] = (uint32_t)w;
    w = 0;
    w = __builtin_amdgcn_cvt_pk_fp8_f32(x[4], x[5], w, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(x[6], x[7], w, true);
    out[1] = (uint32_t)w;
    return out;
}
// codes under scale `old` -> codes under scale `now`
__device__ __forceinline__ u32x2 recode8(u32x2 w, float old, float now) {
    float x[8];
    decode8(w, x);
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = fminf(fmaxf((x[i] * old) / now, -448.0f), 448.0f);
    return encode8(x);
}
__device__ __forceinline__ uint32_t quantize1(uint16_t bits, float scale) {
    const float y = fminf(fmaxf(bf16_bits_to_float(bits) / scale, -448.0f), 448.0f);
    return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(y, 0.f, 0, false) & 0xffu;
}

template <int D, bool FP8>
__global__ __launch_bounds__(kAppendThreads) void append_token_kernel(
    void *__restrict__ k_pool, void *__restrict__ v_pool, float *__restrict__ k_scale, float *__restrict__ v_scale,
    int pool_blocks, int hkv, const int32_t *__restrict__ block_table, const int32_t *__restrict__ num_blocks,
    const int32_t *__restrict__ ctx_lens, const int32_t *__restrict__ seq_lens, const int32_t *__restrict__ status,
    int max_blocks, const uint16_t *__restrict__ k_tok, const uint16_t *__restrict__ v_tok) {
    __shared__ float red[2][kAppendThreads / 64];
    const int r = blockIdx.x;
    const int tid = threadIdx.x;
    if (status && status[r] != 0) return;
    const int n = seq_lens[r] - ctx_lens[r];
    const int nb = min(num_blocks[r], max_blocks);
    if (n <= 0 || nb <= 0) return;
    const int blk = block_table[(size_t)r * max_blocks + nb - 1];
    if (blk < 0 || blk >= pool_blocks) return;
    const int slot = (n - 1) % kBlock;
    const int row_elems = hkv * D;                                          // elements of one token
    const uint16_t *ksrc = k_tok + (size_t)r * row_elems;
    const uint16_t *vsrc = v_tok + (size_t)r * row_elems;
    constexpr int ES = FP8 ? 1 : 2;
    uint8_t *kimg = (uint8_t *)k_pool + (size_t)blk * hkv * kBlock * D * ES;  // [h][slot][d]
    uint8_t *vimg = (uint8_t *)v_pool + (size_t)blk * hkv * kBlock * D * ES;  // [h][d][slot]

    float sk = 1.f, sv = 1.f, old_k = 1.f, old_v = 1.f;
    bool grow_k = false, grow_v = false;
    if constexpr (FP8) {
        if (slot > 0) {
            old_k = k_scale[blk];
            old_v = v_scale[blk];
        }
        float ak = 0.f, av = 0.f;
        for (int c = tid; c < row_elems / 8; c += kAppendThreads) {
            const u32x4 a = *(const u32x4 *)(ksrc + 8 * c), b = *(const u32x4 *)(vsrc + 8 * c);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ak = fmaxf(ak, fmaxf(fabsf(bf16_bits_to_float(a[i] & 0xffffu)), fabsf(bf16_bits_to_float(a[i] >> 16))));
                av = fmaxf(av, fmaxf(fabsf(bf16_bits_to_float(b[i] & 0xffffu)), fabsf(bf16_bits_to_float(b[i] >> 16))));
            }
        }
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) {
            ak = fmaxf(ak, __shfl_xor(ak, o, 64));
            av = fmaxf(av, __shfl_xor(av, o, 64));
        }
        if ((tid & 63) == 0) {
            red[0][tid >> 6] = ak;
            red[1][tid >> 6] = av;
        }
        __syncthreads();                                                    // also: every thread has read the old scales
        ak = fmaxf(fmaxf(red[0][0], red[0][1]), fmaxf(red[0][2], red[0][3]));
        av = fmaxf(fmaxf(red[1][0], red[1][1]), fmaxf(red[1][2], red[1][3]));
        const float need_k = ak / 448.0f, need_v = av / 448.0f;
        if (slot == 0) {
            sk = ak > 0.f ? need_k : 1.0f;
            sv = av > 0.f ? need_v : 1.0f;
        } else {
            grow_k = need_k > old_k;
            grow_v = need_v > old_v;
            sk = grow_k ? need_k : old_k;
            sv = grow_v ? need_v : old_v;
        }
        if (tid == 0) {
            k_scale[blk] = sk;
            v_scale[blk] = sv;
        }
    }

    // ---- K image: 8-element chunks c = (h * 16 + s) * D/8 + d8 ----
    const int kchunks = hkv * kBlock * (D / 8);
    for (int c = tid; c < kchunks; c += kAppendThreads) {
        const int d8 = (c % (D / 8)) * 8, s = (c / (D / 8)) % kBlock, h = c / (D / 8 * kBlock);
        uint8_t *dst = kimg + (size_t)c * 8 * ES;
        if (s == slot) {
            const u32x4 raw = *(const u32x4 *)(ksrc + h * D + d8);
            if constexpr (FP8) *(u32x2 *)dst = quantize8(raw, sk);
            else *(u32x4 *)dst = raw;
        } else if (slot == 0) {
            if constexpr (FP8) *(u32x2 *)dst = u32x2{0, 0};
            else *(u32x4 *)dst = u32x4{0, 0, 0, 0};
        } else if (FP8 && grow_k && s < slot) {
            *(u32x2 *)dst = recode8(*(const u32x2 *)dst, old_k, sk);
        }
    }
    // ---- V image: one head-dim row of 16 slots per thread ----
    for (int row = tid; row < row_elems; row += kAppendThreads) {          // row = h * D + d
        const uint16_t tok = vsrc[row];
        if constexpr (FP8) {
            uint8_t *dst = vimg + (size_t)row * kBlock;
            u32x4 w = {0, 0, 0, 0};
            if (slot > 0) {
                w = *(const u32x4 *)dst;
                if (grow_v) {
                    // slots [0, slot) are re-coded; the slots at and beyond `slot` keep their bits
                    const u32x2 lo = recode8(u32x2{w[0], w[1]}, old_v, sv), hi = recode8(u32x2{w[2], w[3]}, old_v, sv);
                    const u32x4 rec = {lo[0], lo[1], hi[0], hi[1]};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int keep = slot - 4 * i;                       // bytes of dword i that are re-coded
                        const uint32_t m = keep >= 4 ? 0xffffffffu : keep <= 0 ? 0u : (1u << (8 * keep)) - 1u;
                        w[i] = (rec[i] & m) | (w[i] & ~m);
                    }
                }
            }
            const uint32_t code = quantize1(tok, sv);
            const int i = slot >> 2, sh = 8 * (slot & 3);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (j == i) w[j] = (w[j] & ~(0xffu << sh)) | (code << sh);
            *(u32x4 *)dst = w;
        } else {
            uint16_t *dst = (uint16_t *)vimg + (size_t)row * kBlock;
            if (slot == 0) {
                *(u32x4 *)dst = u32x4{tok, 0, 0, 0};
                *(u32x4 *)(dst + 8) = u32x4{0, 0, 0, 0};
            } else {
                dst[slot] = tok;
            }
        }
    }
}

hipError_t launch_append_token(void *k_pool, void *v_pool, float *k_scale, float *v_scale, int32_t pool_blocks,
                               int32_t hkv, int32_t head_dim, int kv_dtype, const gf_tables &t, const void *k_tok,
                               const void *v_tok, hipStream_t s) {
    if (t.num_req == 0) return hipSuccess;
#define GF_APPEND_TOKEN(DD, FF)                                                                                      \
    hipLaunchKernelGGL((append_token_kernel<DD, FF>), dim3((unsigned)t.num_req), dim3(kAppendThreads), 0, s, k_pool, \
                       v_pool, k_scale, v_scale, pool_blocks, hkv, t.block_table, t.num_blocks, t.ctx_lens,         \
                       t.seq_lens, t.status, t.max_blocks, (const uint16_t *)k_tok, (const uint16_t *)v_tok)
    const bool fp8 = kv_dtype == GF_FP8_E4M3;
    if (head_dim == 128 && fp8) GF_APPEND_TOKEN(128, true);
    else if (head_dim == 128) GF_APPEND_TOKEN(128, false);
    else if (head_dim == 64 && fp8) GF_APPEND_TOKEN(64, true);
    else if (head_dim == 64) GF_APPEND_TOKEN(64, false);
    else return hipErrorNotSupported;
#undef GF_APPEND_TOKEN
    return hipGetLastError();
}

hipError_t launch_append(void *k_pool, void *v_pool, float *k_scale, float *v_scale, int32_t pool_blocks, int32_t hkv,
                         int32_t head_dim, int kv_dtype, const gf_tables &t, const void *k_new, const void *v_new,
                         const int32_t *q_ptr, int32_t total_q, int32_t max_q, hipStream_t s) {
    if (t.num_req == 0 || total_q == 0 || max_q == 0) return hipSuccess;
    const unsigned by = (unsigned)((max_q + kBlock - 1) / kBlock);
    if (by > 65535u) return hipErrorInvalidValue;
    const dim3 grid((unsigned)t.num_req, by);
#define GF_APPEND(DD, FF)                                                                                           \
    hipLaunchKernelGGL((append_kernel<DD, FF>), grid, dim3(kAppendThreads), 0, s, k_pool, v_pool, k_scale, v_scale, \
                       pool_blocks, hkv, t.block_table, t.num_blocks, t.ctx_lens, t.seq_lens, t.status,            \
                       t.max_blocks, (const uint16_t *)k_new, (const uint16_t *)v_new, q_ptr, total_q)
    const bool fp8 = kv_dtype == GF_FP8_E4M3;
    if (head_dim == 128 && fp8) GF_APPEND(128, true);
    else if (head_dim == 128) GF_APPEND(128, false);
    else if (head_dim == 64 && fp8) GF_APPEND(64, true);
    else if (head_dim == 64) GF_APPEND(64, false);
    else return hipErrorNotSupported;
#undef GF_APPEND
    return hipGetLastError();
}

}  // namespace gf
