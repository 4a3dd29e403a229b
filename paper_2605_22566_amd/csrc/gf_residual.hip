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
        __builtin_amdgcn_wave_barrier();
        // 2. this image's residual entries (LDS operations of one wave complete in order)
        const size_t r = (size_t)item * rows + row;
        const int e0 = res_ptr[r], e1 = res_ptr[r + 1];
        for (int e = e0 + lane; e < e1; e += 64) {
            const uint32_t i = res_idx[e];
            if (i >= (uint32_t)kImg) {
                bad = true;
                continue;
            }
            const uint32_t phys = is_v ? (i % D) * kBlock + i / D : i;   // V image: [d][slot]
            const float base = __uint_as_float((uint32_t)img[phys] << 16);
            const float delta = __uint_as_float((uint32_t)res_val[e] << 16);
            const __bf16 sum = (__bf16)(base + delta);                   // round to nearest even
            img[phys] = __builtin_bit_cast(uint16_t, sum);
        }
        __builtin_amdgcn_wave_barrier();
        // 3. LDS -> destination image
#pragma unroll
        for (int c = 8 * lane; c < kImg; c += 8 * 64) *(u32x4 *)(g_dst + c) = *(const u32x4 *)(img + c);
    }
    if (bad) bad_index = 1;                                              // benign race: every writer stores 1
    __syncthreads();
    if (status && tid == 0) status[item] = bad_index ? GF_RS_BAD_INDEX : GF_RS_OK;
}

hipError_t launch_residual(void *k_pool, void *v_pool, int32_t num_pool_blocks, int32_t hkv, int32_t head_dim,
                           int32_t num_items, const int32_t *src_blocks, const int32_t *dst_blocks,
                           const int32_t *res_ptr, const uint16_t *res_idx, const uint16_t *res_val,
                           int32_t *status, hipStream_t s) {
    if (num_items == 0) return hipSuccess;
    if (head_dim == 128)
        hipLaunchKernelGGL(residual_kernel<128>, dim3((unsigned)num_items), dim3(kResidualThreads), 0, s,
                           (uint16_t *)k_pool, (uint16_t *)v_pool, num_pool_blocks, hkv, src_blocks, dst_blocks,
                           res_ptr, res_idx, res_val, status);
    else if (head_dim == 64)
        hipLaunchKernelGGL(residual_kernel<64>, dim3((unsigned)num_items), dim3(kResidualThreads), 0, s,
                           (uint16_t *)k_pool, (uint16_t *)v_pool, num_pool_blocks, hkv, src_blocks, dst_blocks,
                           res_ptr, res_idx, res_val, status);
    else
        return hipErrorNotSupported;
    return hipGetLastError();
}

}  // namespace gf
