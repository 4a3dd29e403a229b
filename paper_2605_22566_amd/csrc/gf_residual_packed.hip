// The packed form of a sparse residual (paper, "Differential-based KV Cache", Eq. 7, and its KV-sparsity appendix:
// more than 75 % of the key and 70 % of the value entries of a prefix-induced difference are negligible).  The
// coordinate list the attention kernels read costs 2 B of index + 2 B of value per kept element: 0.55 of a dense
// bf16 block at those densities.  At rest a residual is kept smaller: per (item, tensor, kv head) image one bit
// per element -- bit i % 32 of word i / 32 for logical element i = slot * D + d -- and the kept values alone, in
// rising element order: 0.34 of a dense block.  The row pointers are the same in both forms.
//   gf_kv_residual_pack          coordinate rows (any order inside a row) -> masks + ordered values
//   gf_kv_residual_unpack        masks -> element indices in rising order (the ordered values are the row's values)
//   gf_kv_apply_residual_packed  gf_kv_apply_residual straight from the packed form
// One workgroup of four waves per item; a wave takes whole rows, one after the other, with no workgroup barrier
// in between.  A mask has 16 * D / 32 <= 64 words: lane l holds word l, a wave-wide exclusive scan of the
// population counts gives every lane the position of its first value.
#include "gf_internal.h"

namespace gf {

constexpr int kPackedThreads = 256;
constexpr int kPackedWaves = kPackedThreads / 64;

// exclusive prefix sum over the 64 lanes; `total` receives the sum of all lanes
__device__ __forceinline__ int wave_exscan(int x, int lane, int &total) {
    int incl = x;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int y = __shfl_up(incl, o, 64);
        if (lane >= o) incl += y;
    }
    total = __shfl(incl, 63, 64);
    return incl - x;
}

template <int D>
__global__ __launch_bounds__(kPackedThreads) void residual_pack_kernel(
    int hkv, const int32_t *__restrict__ res_ptr, const uint16_t *__restrict__ res_idx,
    const uint16_t *__restrict__ res_val, uint32_t *__restrict__ res_mask, uint16_t *__restrict__ packed_val,
    int32_t *__restrict__ status) {
    constexpr int kImg = kBlock * D, kWords = kImg / 32;
    __shared__ uint32_t mask[kPackedWaves][64];
    __shared__ int32_t before[kPackedWaves][64];        // set bits in the words before word l
    __shared__ int bad_row;
    const int item = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (tid == 0) bad_row = 0;
    __syncthreads();
    const int rows = 2 * hkv;
    bool bad = false;
    for (int row = wave; row < rows; row += kPackedWaves) {
        const size_t r = (size_t)item * rows + row;
        const int e0 = res_ptr[r], e1 = res_ptr[r + 1];
        mask[wave][lane] = 0;
        wave_lds_order();
        for (int e = e0 + lane; e < e1; e += 64) {
            const uint32_t i = res_idx[e];
            if (i >= (uint32_t)kImg) {
                bad = true;
                continue;
            }
            const uint32_t bit = 1u << (i & 31);
            if (atomicOr(&mask[wave][i >> 5], bit) & bit) bad = true;     // the element is named twice
        }
        wave_lds_order();
        const uint32_t w = mask[wave][lane];
        int total;
        before[wave][lane] = wave_exscan(__popc(w), lane, total);
        wave_lds_order();
        if (total != e1 - e0) bad = true;
        for (int e = e0 + lane; e < e1; e += 64) {
            const uint32_t i = res_idx[e];
            if (i >= (uint32_t)kImg) continue;
            const int pos = before[wave][i >> 5] + __popc(mask[wave][i >> 5] & ((1u << (i & 31)) - 1u));
            if (pos < e1 - e0) packed_val[(size_t)e0 + pos] = res_val[e];
        }
        if (lane < kWords) res_mask[r * kWords + lane] = w;
        wave_lds_order();
    }
    if (bad) bad_row = 1;                                                  // benign race: every writer stores 1
    __syncthreads();
    if (status && tid == 0) status[item] = bad_row ? GF_RS_BAD_INDEX : GF_RS_OK;
}

template <int D>
__global__ __launch_bounds__(kPackedThreads) void residual_unpack_kernel(
    int hkv, const int32_t *__restrict__ res_ptr, const uint32_t *__restrict__ res_mask,
    uint16_t *__restrict__ res_idx, int32_t *__restrict__ status) {
    constexpr int kImg = kBlock * D, kWords = kImg / 32;
    __shared__ int bad_row;
    const int item = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (tid == 0) bad_row = 0;
    __syncthreads();
    const int rows = 2 * hkv;
    bool bad = false;
    for (int row = wave; row < rows; row += kPackedWaves) {
        const size_t r = (size_t)item * rows + row;
        const int e0 = res_ptr[r], e1 = res_ptr[r + 1];
        uint32_t w = lane < kWords ? res_mask[r * kWords + lane] : 0u;
        int total;
        int e = e0 + wave_exscan(__popc(w), lane, total);
        if (total != e1 - e0) bad = true;
        while (w) {
            const int b = __builtin_ctz(w);
            w &= w - 1;
            if (e < e1) res_idx[e] = (uint16_t)(32 * lane + b);
            ++e;
        }
    }
    if (bad) bad_row = 1;
    __syncthreads();
    if (status && tid == 0) status[item] = bad_row ? GF_RS_BAD_INDEX : GF_RS_OK;
}

// gf_kv_apply_residual's bf16 kernel with the entries read from the packed form: base image -> the wave's LDS
// region, every set bit of the image's mask adds the next value of the row to its element (fp32 sum rounded to
// bf16 nearest-even; the V image keeps [d][slot]), image -> destination block.
template <int D>
__global__ __launch_bounds__(kPackedThreads) void residual_packed_kernel(
    uint16_t *__restrict__ k_pool, uint16_t *__restrict__ v_pool, int num_pool_blocks, int hkv,
    const int32_t *__restrict__ src_blocks, const int32_t *__restrict__ dst_blocks,
    const int32_t *__restrict__ res_ptr, const uint32_t *__restrict__ res_mask,
    const uint16_t *__restrict__ packed_val, int32_t *__restrict__ status) {
    constexpr int kImg = kBlock * D, kWords = kImg / 32;
    __shared__ __attribute__((aligned(16))) uint16_t lds[kPackedWaves][kImg];
    __shared__ int bad_row;
    const int item = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int src = src_blocks[item], dst = dst_blocks[item];
    if (src < 0 || src >= num_pool_blocks || dst < 0 || dst >= num_pool_blocks) {
        if (status && tid == 0) status[item] = GF_RS_BAD_BLOCK;
        return;
    }
    if (tid == 0) bad_row = 0;
    __syncthreads();
    uint16_t *img = lds[wave];
    const int rows = 2 * hkv;
    bool bad = false;
    for (int row = wave; row < rows; row += kPackedWaves) {
        const bool is_v = row >= hkv;
        const int h = is_v ? row - hkv : row;
        uint16_t *pool = is_v ? v_pool : k_pool;
        const uint16_t *g_src = pool + ((size_t)src * hkv + h) * kImg;
        uint16_t *g_dst = pool + ((size_t)dst * hkv + h) * kImg;
        const size_t r = (size_t)item * rows + row;
        const int e0 = res_ptr[r], e1 = res_ptr[r + 1];
        uint32_t w = lane < kWords ? res_mask[r * kWords + lane] : 0u;
#pragma unroll
        for (int c = 8 * lane; c < kImg; c += 8 * 64) *(u32x4 *)(img + c) = *(const u32x4 *)(g_src + c);
        int total;
        int e = e0 + wave_exscan(__popc(w), lane, total);
        if (total != e1 - e0) bad = true;
        wave_lds_order();
        while (w) {
            const int b = __builtin_ctz(w);
            w &= w - 1;
            if (e < e1) {
                const uint32_t i = 32 * lane + b;
                const uint32_t at = is_v ? (i % D) * kBlock + i / D : i;
                const float base = __uint_as_float((uint32_t)img[at] << 16);
                const float delta = __uint_as_float((uint32_t)packed_val[e] << 16);
                img[at] = __builtin_bit_cast(uint16_t, (__bf16)(base + delta));      // round to nearest even
            }
            ++e;
        }
        wave_lds_order();
#pragma unroll
        for (int c = 8 * lane; c < kImg; c += 8 * 64) *(u32x4 *)(g_dst + c) = *(const u32x4 *)(img + c);
        wave_lds_order();
    }
    if (bad) bad_row = 1;
    __syncthreads();
    if (status && tid == 0) status[item] = bad_row ? GF_RS_BAD_INDEX : GF_RS_OK;
}

hipError_t launch_residual_pack(int32_t hkv, int32_t head_dim, int32_t num_items, const int32_t *res_ptr,
                                const uint16_t *res_idx, const uint16_t *res_val, uint32_t *res_mask,
                                uint16_t *packed_val, int32_t *status, hipStream_t s) {
    if (num_items == 0) return hipSuccess;
    const dim3 grid((unsigned)num_items), block(kPackedThreads);
    if (head_dim == 128)
        hipLaunchKernelGGL(residual_pack_kernel<128>, grid, block, 0, s, hkv, res_ptr, res_idx, res_val, res_mask,
                           packed_val, status);
    else if (head_dim == 64)
        hipLaunchKernelGGL(residual_pack_kernel<64>, grid, block, 0, s, hkv, res_ptr, res_idx, res_val, res_mask,
                           packed_val, status);
    else return hipErrorNotSupported;
    return hipGetLastError();
}

hipError_t launch_residual_unpack(int32_t hkv, int32_t head_dim, int32_t num_items, const int32_t *res_ptr,
                                  const uint32_t *res_mask, uint16_t *res_idx, int32_t *status, hipStream_t s) {
    if (num_items == 0) return hipSuccess;
    const dim3 grid((unsigned)num_items), block(kPackedThreads);
    if (head_dim == 128)
        hipLaunchKernelGGL(residual_unpack_kernel<128>, grid, block, 0, s, hkv, res_ptr, res_mask, res_idx, status);
    else if (head_dim == 64)
        hipLaunchKernelGGL(residual_unpack_kernel<64>, grid, block, 0, s, hkv, res_ptr, res_mask, res_idx, status);
    else return hipErrorNotSupported;
    return hipGetLastError();
}

hipError_t launch_residual_packed(void *k_pool, void *v_pool, int32_t num_pool_blocks, int32_t hkv, int32_t head_dim,
                                  int32_t num_items, const int32_t *src_blocks, const int32_t *dst_blocks,
                                  const int32_t *res_ptr, const uint32_t *res_mask, const uint16_t *packed_val,
                                  int32_t *status, hipStream_t s) {
    if (num_items == 0) return hipSuccess;
    const dim3 grid((unsigned)num_items), block(kPackedThreads);
    if (head_dim == 128)
        hipLaunchKernelGGL(residual_packed_kernel<128>, grid, block, 0, s, (uint16_t *)k_pool, (uint16_t *)v_pool,
                           num_pool_blocks, hkv, src_blocks, dst_blocks, res_ptr, res_mask, packed_val, status);
    else if (head_dim == 64)
        hipLaunchKernelGGL(residual_packed_kernel<64>, grid, block, 0, s, (uint16_t *)k_pool, (uint16_t *)v_pool,
                           num_pool_blocks, hkv, src_blocks, dst_blocks, res_ptr, res_mask, packed_val, status);
    else return hipErrorNotSupported;
    return hipGetLastError();
}

}  // namespace gf
