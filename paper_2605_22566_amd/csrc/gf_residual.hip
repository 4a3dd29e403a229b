// gf_kv_apply_residual: reconstruct prefix-conditioned KV blocks (paper,
// Differential-based KV Cache, Eq. 7: KV(P, v) = KV_base(v) + dKV(P, v); the
// base KV of an operation node is loaded and the sparse residual of the current
// prefix is applied to it).
//
// Bandwidth path.  One workgroup of four waves per 16-token pool block; a wave takes whole
// "images" -- the 16 x D elements of one tensor (K or V) and one kv head, contiguous in the
// pool in either layout -- one after the other, with no workgroup barrier in between:
//   1. the base image is loaded into the wave's own LDS region with 16-byte loads;
//   2. every residual entry of the image (its own CSR row, 16-bit index slot*D + d) adds its
//      value to its element in LDS: fp32 sum, rounded to bf16 nearest-even.  Entries name
//      distinct elements, so no two lanes touch the same one; for V the element sits at
//      d*16 + slot of the image;
//   3. the image is written to the destination block with 16-byte stores.
// Global memory sees only whole-line traffic; the 2-byte scatter stays in LDS.
#include "gf_internal.h"

namespace gf {

constexpr int kResidualThreads = 256;
constexpr int kResidualWaves = kResidualThreads / 64;

// Calls f(index, value bits) for every entry of the CSR row [e0, e1), 64 lanes sharing the row.  Where the row
// covers whole aligned groups of 8 entries a lane reads a group with one 16-byte load of indices and one of
// values (whole row by single entries if the arrays do not start on a 16-byte boundary); the loads of the two
// ends and of the first 512 grouped entries are all issued before the first call, so a row of the paper's density
// costs one memory round trip instead of one per 64 entries.
template <typename F>
__device__ __forceinline__ void for_row_entries(const uint16_t *__restrict__ idx, const uint16_t *__restrict__ val,
                                                int e0, int e1, int lane, F f) {
    if (e0 >= e1) return;
    const bool vec = (((uintptr_t)idx | (uintptr_t)val) & 15) == 0;
    const int a0 = vec ? min(e1, (e0 + 7) & ~7) : e1;        // [e0, a0) and [a1, e1): single entries
    const int a1 = vec ? a0 + ((e1 - a0) & ~7) : e1;         // [a0, a1): aligned groups of 8
    const int head = a0 - e0, singles = head + (e1 - a1);
    uint32_t si = 0, sv = 0;
    const bool has_single = lane < singles;
    if (has_single) {
        const int es = lane < head ? e0 + lane : a1 + (lane - head);
        si = idx[es];
        sv = val[es];
    }
    int g = a0 + 8 * lane;
    u32x4 gi = {0, 0, 0, 0}, gv = {0, 0, 0, 0};
    if (g < a1) {
        gi = *(const u32x4 *)(idx + g);
        gv = *(const u32x4 *)(val + g);
    }
    if (has_single) f(si, sv);
    for (int s = lane + 64; s < singles; s += 64) {          // only without the 16-byte alignment
        const int e = s < head ? e0 + s : a1 + (s - head);
        f((uint32_t)idx[e], (uint32_t)val[e]);
    }
    while (g < a1) {
#pragma unroll
        for (int j = 0; j < 8; ++j) f((gi[j / 2] >> (16 * (j % 2))) & 0xFFFFu, (gv[j / 2] >> (16 * (j % 2))) & 0xFFFFu);
        g += 512;
        if (g < a1) {
            gi = *(const u32x4 *)(idx + g);
            gv = *(const u32x4 *)(val + g);
        }
    }
}

template <int D>
__global__ __launch_bounds__(kResidualThreads) void residual_kernel(
    uint16_t *__restrict__ k_pool, uint16_t *__restrict__ v_pool, int num_pool_blocks, int hkv,
    const int32_t *__restrict__ src_blocks, const int32_t *__restrict__ dst_blocks,
    const int32_t *__restrict__ res_ptr, const uint16_t *__restrict__ res_idx,
    const uint16_t *__restrict__ res_val, int32_t *__restrict__ status) {
    constexpr int kImg = kBlock * D;                       // elements of one image
    __shared__ __attribute__((aligned(16))) uint16_t lds[kResidualWaves][kImg];
    __shared__ int bad_index;
    const int item = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int src = src_blocks[item], dst = dst_blocks[item];
    if (src < 0 || src >= num_pool_blocks || dst < 0 || dst >= num_pool_blocks) {
        if (status && tid == 0) status[item] = GF_RS_BAD_BLOCK;
        return;
    }
    if (tid == 0) bad_index = 0;
    __syncthreads();
    uint16_t *img = lds[wave];
    const int rows = 2 * hkv;                              // images of a block: K heads, then V heads
    bool bad = false;
    for (int row = wave; row < rows; row += kResidualWaves) {
        const bool is_v = row >= hkv;
        const int h = is_v ? row - hkv : row;
        uint16_t *pool = is_v ? v_pool : k_pool;
        const uint16_t *g_src = pool + ((size_t)src * hkv + h) * kImg;
        uint16_t *g_dst = pool + ((size_t)dst * hkv + h) * kImg;
        // 1. base image -> LDS
#pragma unroll
        for (int c = 8 * lane; c < kImg; c += 8 * 64) *(u32x4 *)(img + c) = *(const u32x4 *)(g_src + c);
        wave_lds_order();
        // 2. this image's residual entries (LDS operations of one wave complete in order)
        const size_t r = (size_t)item * rows + row;
        const int e0 = res_ptr[r], e1 = res_ptr[r + 1];
        for_row_entries(res_idx, res_val, e0, e1, lane, [&](uint32_t i, uint32_t bits) {
            if (i >= (uint32_t)kImg) {
                bad = true;
                return;
            }
            const uint32_t phys = is_v ? (i % D) * kBlock + i / D : i;   // V image: [d][slot]
            const float base = __uint_as_float((uint32_t)img[phys] << 16);
            const float delta = __uint_as_float(bits << 16);
            const __bf16 sum = (__bf16)(base + delta);                   // round to nearest even
            img[phys] = __builtin_bit_cast(uint16_t, sum);
        });
        wave_lds_order();
        // 3. LDS -> destination image
#pragma unroll
        for (int c = 8 * lane; c < kImg; c += 8 * 64) *(u32x4 *)(g_dst + c) = *(const u32x4 *)(img + c);
    }
    if (bad) bad_index = 1;                                              // benign race: every writer stores 1
    __syncthreads();
    if (status && tid == 0) status[item] = bad_index ? GF_RS_BAD_INDEX : GF_RS_OK;
}

// e4m3 pool: the same reconstruction with a quantised base and a quantised result.  A base image is widened
// (code -> value, times the source block's scale), the residual entries are added in fp32 (fp32 images in the
// wave's LDS region), and the destination block gets a scale of its own: amax / 448 per tensor over the whole
// block.  That maximum is only known once every image has been summed, so the block is walked twice: pass 1
// leaves the two maxima, pass 2 repeats the sums (the base is still in L2) and writes the codes.
template <int D>
__global__ __launch_bounds__(kResidualThreads) void residual_e4m3_kernel(
    uint8_t *__restrict__ k_pool, uint8_t *__restrict__ v_pool, float *__restrict__ k_scale,
    float *__restrict__ v_scale, int num_pool_blocks, int hkv, const int32_t *__restrict__ src_blocks,
    const int32_t *__restrict__ dst_blocks, const int32_t *__restrict__ res_ptr,
    const uint16_t *__restrict__ res_idx, const uint16_t *__restrict__ res_val, int32_t *__restrict__ status) {
    constexpr int kImg = kBlock * D;                       // elements (= bytes) of one image
    __shared__ __attribute__((aligned(16))) float lds[kResidualWaves][kImg];
    __shared__ float red[2][kResidualWaves];
    __shared__ int bad_index;
    const int item = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int src = src_blocks[item], dst = dst_blocks[item];
    if (src < 0 || src >= num_pool_blocks || dst < 0 || dst >= num_pool_blocks) {
        if (status && tid == 0) status[item] = GF_RS_BAD_BLOCK;
        return;
    }
    const float src_scale[2] = {k_scale[src], v_scale[src]};   // read before the destination's are written (src may be dst)
    if (tid == 0) bad_index = 0;
    __syncthreads();
    float *img = lds[wave];
    const int rows = 2 * hkv;
    bool bad = false;
    float dst_scale[2] = {1.f, 1.f};
    for (int pass = 0; pass < 2; ++pass) {
        float amax[2] = {0.f, 0.f};
        for (int row = wave; row < rows; row += kResidualWaves) {
            const bool is_v = row >= hkv;
            const int h = is_v ? row - hkv : row;
            uint8_t *pool = is_v ? v_pool : k_pool;
            const uint8_t *g_src = pool + ((size_t)src * hkv + h) * kImg;
            uint8_t *g_dst = pool + ((size_t)dst * hkv + h) * kImg;
            const float s_in = src_scale[is_v];
            // 1. base image -> fp32 in LDS
#pragma unroll
            for (int c = 16 * lane; c < kImg; c += 16 * 64) {
                const u32x4 w = *(const u32x4 *)(g_src + c);
                const bf16x8 lo = fp8x8_to_bf16x8(u32x2{w[0], w[1]}), hi = fp8x8_to_bf16x8(u32x2{w[2], w[3]});
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    img[c + i] = __fmul_rn((float)lo[i], s_in);
                    img[c + 8 + i] = __fmul_rn((float)hi[i], s_in);
                }
            }
            wave_lds_order();
            // 2. this image's residual entries
            const size_t r = (size_t)item * rows + row;
            const int e0 = res_ptr[r], e1 = res_ptr[r + 1];
            for_row_entries(res_idx, res_val, e0, e1, lane, [&](uint32_t i, uint32_t bits) {
                if (i >= (uint32_t)kImg) {
                    bad = true;
                    return;
                }
                const uint32_t phys = is_v ? (i % D) * kBlock + i / D : i;   // V image: [d][slot]
                img[phys] = __fadd_rn(img[phys], __uint_as_float(bits << 16));
            });
            wave_lds_order();
            if (pass == 0) {
                // 3a. this image's share of the tensor's maximum
                float m = 0.f;
#pragma unroll 8
                for (int c = lane; c < kImg; c += 64) m = fmaxf(m, fabsf(img[c]));
                amax[is_v] = fmaxf(amax[is_v], m);
            } else {
                // 3b. quantise under the destination scale and write the image
                const float s_out = dst_scale[is_v];
#pragma unroll
                for (int c = 8 * lane; c < kImg; c += 8 * 64) {
                    float x[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) x[i] = fminf(fmaxf(img[c + i] / s_out, -448.0f), 448.0f);
                    u32x2 out;
                    int w = 0;
                    w = __builtin_amdgcn_cvt_pk_fp8_f32(x[0], x[1], w, false);
                    w = __builtin_amdgcn_cvt_pk_fp8_f32(x[2], x[3], w, true);
                    out[0] = (uint32_t)w;
                    w = 0;
                    w = __builtin_amdgcn_cvt_pk_fp8_f32(x[4], x[5], w, false);
                    w = __builtin_amdgcn_cvt_pk_fp8_f32(x[6], x[7], w, true);
                    out[1] = (uint32_t)w;
                    *(u32x2 *)(g_dst + c) = out;
                }
            }
            wave_lds_order();                   // the image region is reused by the wave's next row
        }
        if (pass == 0) {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
#pragma unroll
                for (int o = 32; o >= 1; o >>= 1) amax[t] = fmaxf(amax[t], __shfl_xor(amax[t], o, 64));
                if (lane == 0) red[t][wave] = amax[t];
            }
            __syncthreads();
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const float m = fmaxf(fmaxf(red[t][0], red[t][1]), fmaxf(red[t][2], red[t][3]));
                dst_scale[t] = m > 0.f ? m / 448.0f : 1.0f;
            }
            if (tid == 0) {
                k_scale[dst] = dst_scale[0];
                v_scale[dst] = dst_scale[1];
            }
        }
    }
    if (bad) bad_index = 1;                                              // benign race: every writer stores 1
    __syncthreads();
    if (status && tid == 0) status[item] = bad_index ? GF_RS_BAD_INDEX : GF_RS_OK;
}

// The same in one pass, one wave per kv head.  A wave keeps its image in registers (16 consecutive elements per
// lane and 1 KB of codes) and only the residual goes through LDS: a 2-byte image per head, preset to a "no
// entry" mark, into which the row's bf16 values are stored (plain stores: the entries of a row name distinct
// elements), and from which every lane then reads the 16 values beside its 16 codes.  K first, then V: every wave
// sums its image, the workgroup reduces the tensor's maximum, every wave quantises and writes its image.
template <int D, int HKV>
__global__ __launch_bounds__(64 * HKV) void residual_e4m3_onepass_kernel(
    uint8_t *__restrict__ k_pool, uint8_t *__restrict__ v_pool, float *__restrict__ k_scale,
    float *__restrict__ v_scale, int num_pool_blocks, const int32_t *__restrict__ src_blocks,
    const int32_t *__restrict__ dst_blocks, const int32_t *__restrict__ res_ptr,
    const uint16_t *__restrict__ res_idx, const uint16_t *__restrict__ res_val, int32_t *__restrict__ status) {
    constexpr int kImg = kBlock * D;
    constexpr int NJ = kImg / 1024;                               // 16-element pieces per lane
    constexpr uint16_t kNone = 0xFFFFu;                           // a NaN pattern no stored entry keeps (see below)
    __shared__ __attribute__((aligned(16))) uint16_t lds[HKV][kImg];
    __shared__ float red[2][HKV];
    __shared__ int bad_index;
    const int item = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int h = __builtin_amdgcn_readfirstlane(tid >> 6);       // this wave's kv head
    const int src = src_blocks[item], dst = dst_blocks[item];
    if (src < 0 || src >= num_pool_blocks || dst < 0 || dst >= num_pool_blocks) {
        if (status && tid == 0) status[item] = GF_RS_BAD_BLOCK;
        return;
    }
    const float src_scale[2] = {k_scale[src], v_scale[src]};      // read before the destination's are written (src may be dst)
    if (tid == 0) bad_index = 0;
    __syncthreads();
    uint16_t *img = lds[h];
    bool bad = false;
    for (int t = 0; t < 2; ++t) {
        uint8_t *pool = t ? v_pool : k_pool;
        const uint8_t *g_src = pool + ((size_t)src * HKV + h) * kImg;
        uint8_t *g_dst = pool + ((size_t)dst * HKV + h) * kImg;
        const float s_in = src_scale[t];
        u32x4 codes[NJ];
#pragma unroll
        for (int j = 0; j < NJ; ++j) codes[j] = *(const u32x4 *)(g_src + 16 * lane + 1024 * j);
        const u32x4 none = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu};
#pragma unroll
        for (int c = 8 * lane; c < kImg; c += 8 * 64) *(u32x4 *)(img + c) = none;
        wave_lds_order();
        const size_t r = ((size_t)item * 2 + t) * HKV + h;
        const int e0 = res_ptr[r], e1 = res_ptr[r + 1];
        for_row_entries(res_idx, res_val, e0, e1, lane, [&](uint32_t i, uint32_t bits) {
            if (i >= (uint32_t)kImg) {
                bad = true;
                return;
            }
            const uint32_t phys = t ? (i % D) * kBlock + i / D : i;          // V image: [d][slot]
            img[phys] = bits == kNone ? (uint16_t)0xFFFEu : (uint16_t)bits;  // still a negative NaN: the sum is one too
        });
        wave_lds_order();
        float x[NJ][16];
        float m = 0.f;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const bf16x8 lo = fp8x8_to_bf16x8(u32x2{codes[j][0], codes[j][1]});
            const bf16x8 hi = fp8x8_to_bf16x8(u32x2{codes[j][2], codes[j][3]});
            const u32x4 d0 = *(const u32x4 *)(img + 16 * lane + 1024 * j);
            const u32x4 d1 = *(const u32x4 *)(img + 16 * lane + 1024 * j + 8);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float base = __fmul_rn(i < 8 ? (float)lo[i] : (float)hi[i - 8], s_in);
                // the product is an fp32 value of its own (the oracle rounds it): nothing may fuse it with the sum
                // below into one multiply-add -- the compiler does so even across the two rounding intrinsics
                asm volatile("" : "+v"(base));
                const uint32_t w = (i < 8 ? d0 : d1)[(i % 8) / 2];
                const uint32_t bits = (i % 2) ? (w >> 16) : (w & 0xFFFFu);
                // an element no entry names keeps its value bit for bit (a sum with zero would lose the sign of -0)
                x[j][i] = bits == kNone ? base : __fadd_rn(base, __uint_as_float(bits << 16));
                m = fmaxf(m, fabsf(x[j][i]));
            }
        }
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
        if (lane == 0) red[t][h] = m;
        __syncthreads();
        float amax = 0.f;
#pragma unroll
        for (int i = 0; i < HKV; ++i) amax = fmaxf(amax, red[t][i]);
        const float s_out = amax > 0.f ? amax / 448.0f : 1.0f;
        if (tid == 0) (t ? v_scale : k_scale)[dst] = s_out;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            u32x4 out;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float y[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) y[i] = fminf(fmaxf(x[j][4 * q + i] / s_out, -448.0f), 448.0f);
                int w = 0;
                w = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], w, false);
                w = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], w, true);
                out[q] = (uint32_t)w;
            }
            *(u32x4 *)(g_dst + 16 * lane + 1024 * j) = out;
        }
    }
    if (bad) bad_index = 1;                                                  // benign race: every writer stores 1
    __syncthreads();
    if (status && tid == 0) status[item] = bad_index ? GF_RS_BAD_INDEX : GF_RS_OK;
}

hipError_t launch_residual(void *k_pool, void *v_pool, float *k_scale, float *v_scale, int32_t num_pool_blocks,
                           int32_t hkv, int32_t head_dim, int kv_dtype, int32_t num_items, const int32_t *src_blocks,
                           const int32_t *dst_blocks, const int32_t *res_ptr, const uint16_t *res_idx,
                           const uint16_t *res_val, int32_t *status, hipStream_t s) {
    if (num_items == 0) return hipSuccess;
    const dim3 grid((unsigned)num_items), block(kResidualThreads);
    const bool fp8 = kv_dtype == GF_FP8_E4M3;
#define GF_RES_BF16(DD)                                                                                              \
    hipLaunchKernelGGL(residual_kernel<DD>, grid, block, 0, s, (uint16_t *)k_pool, (uint16_t *)v_pool, num_pool_blocks, \
                       hkv, src_blocks, dst_blocks, res_ptr, res_idx, res_val, status)
#define GF_RES_E4M3(DD)                                                                                            \
    hipLaunchKernelGGL(residual_e4m3_kernel<DD>, grid, block, 0, s, (uint8_t *)k_pool, (uint8_t *)v_pool, k_scale, \
                       v_scale, num_pool_blocks, hkv, src_blocks, dst_blocks, res_ptr, res_idx, res_val, status)
#define GF_RES_ONEPASS(DD, HH)                                                                                     \
    hipLaunchKernelGGL((residual_e4m3_onepass_kernel<DD, HH>), grid, dim3(64 * HH), 0, s, (uint8_t *)k_pool,      \
                       (uint8_t *)v_pool, k_scale, v_scale, num_pool_blocks, src_blocks, dst_blocks, res_ptr,     \
                       res_idx, res_val, status)
    // e4m3: one pass with a wave per kv head (1024 threads at most)
    if (head_dim == 128 && fp8 && hkv == 8) GF_RES_ONEPASS(128, 8);
    else if (head_dim == 128 && fp8 && hkv == 4) GF_RES_ONEPASS(128, 4);
    else if (head_dim == 128 && fp8 && hkv == 2) GF_RES_ONEPASS(128, 2);
    else if (head_dim == 128 && fp8 && hkv == 1) GF_RES_ONEPASS(128, 1);
    else if (head_dim == 64 && fp8 && hkv == 8) GF_RES_ONEPASS(64, 8);
    else if (head_dim == 64 && fp8 && hkv == 4) GF_RES_ONEPASS(64, 4);
    else if (head_dim == 64 && fp8 && hkv == 2) GF_RES_ONEPASS(64, 2);
    else if (head_dim == 64 && fp8 && hkv == 1) GF_RES_ONEPASS(64, 1);
    else if (head_dim == 128 && fp8) GF_RES_E4M3(128);
    else if (head_dim == 128) GF_RES_BF16(128);
    else if (head_dim == 64 && fp8) GF_RES_E4M3(64);
    else if (head_dim == 64) GF_RES_BF16(64);
    else return hipErrorNotSupported;
#undef GF_RES_BF16
#undef GF_RES_E4M3
#undef GF_RES_ONEPASS
    return hipGetLastError();
}

}  // namespace gf
