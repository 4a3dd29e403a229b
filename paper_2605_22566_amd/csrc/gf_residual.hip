// gf_kv_apply_residual: reconstruct prefix-conditioned KV blocks (paper,
// Differential-based KV Cache, Eq. 7: KV(P, v) = KV_base(v) + dKV(P, v); the
// base KV of an operation node is loaded and the sparse residual of the current
// prefix is applied to it).
//
// Bandwidth path.  One workgroup per 16-token pool block (all kv heads, K and V):
//   1. the base block is copied to the destination block with 16-byte loads and
//      stores (coalesced, both tensors are contiguous per block);
//   2. after a workgroup barrier, every residual entry reads its base element from
//      the SOURCE block, adds its value in fp32, rounds to bf16 (nearest even) and
//      overwrites the element of the destination block.  Reading the source keeps
//      the read away from lines this workgroup has just written; the barrier (with
//      its workgroup-scope fence) puts the entry's store behind the copy's.
// A residual entry names the logical element ((t*Hkv + h)*16 + slot)*D + d; for
// V the physical position inside the block is (h*D + d)*16 + slot.
#include "gf_internal.h"

namespace gf {

constexpr int kResidualThreads = 256;

__global__ __launch_bounds__(kResidualThreads) void residual_kernel(
    uint16_t *__restrict__ k_pool, uint16_t *__restrict__ v_pool, int num_pool_blocks, int hkv, int dim,
    const int32_t *__restrict__ src_blocks, const int32_t *__restrict__ dst_blocks,
    const int32_t *__restrict__ res_ptr, const uint32_t *__restrict__ res_idx,
    const uint16_t *__restrict__ res_val, int32_t *__restrict__ status) {
    __shared__ int bad_index;
    const int item = blockIdx.x;
    const int tid = threadIdx.x;
    const int src = src_blocks[item], dst = dst_blocks[item];
    if (src < 0 || src >= num_pool_blocks || dst < 0 || dst >= num_pool_blocks) {
        if (status && tid == 0) status[item] = GF_RS_BAD_BLOCK;
        return;
    }
    if (tid == 0) bad_index = 0;
    const uint32_t per_tensor = (uint32_t)hkv * kBlock * dim;          // elements of one tensor in a block
    const size_t src_off = (size_t)src * per_tensor, dst_off = (size_t)dst * per_tensor;

    // 1. copy (per_tensor is a multiple of 8 elements: head_dim is 64 or 128)
    const uint32_t chunks = per_tensor / 8;
    const u32x4 *ks = (const u32x4 *)(k_pool + src_off), *vs = (const u32x4 *)(v_pool + src_off);
    u32x4 *kd = (u32x4 *)(k_pool + dst_off), *vd = (u32x4 *)(v_pool + dst_off);
    for (uint32_t c = tid; c < chunks; c += kResidualThreads) {
        kd[c] = ks[c];
        vd[c] = vs[c];
    }
    __syncthreads();

    // 2. residual entries
    const int e0 = res_ptr[item], e1 = res_ptr[item + 1];
    bool bad = false;
    for (int e = e0 + tid; e < e1; e += kResidualThreads) {
        const uint32_t i = res_idx[e];
        if (i >= 2 * per_tensor) {
            bad = true;
            continue;
        }
        const uint32_t t = i >= per_tensor ? 1u : 0u;
        const uint32_t rem = i - t * per_tensor;
        uint32_t phys = rem;                                             // K: [h][slot][d]
        if (t) {                                                         // V: [h][d][slot]
            const uint32_t h = rem / (kBlock * dim), r2 = rem % (kBlock * dim);
            const uint32_t slot = r2 / dim, d = r2 % dim;
            phys = (h * dim + d) * kBlock + slot;
        }
        uint16_t *pool = t ? v_pool : k_pool;
        const float base = __uint_as_float((uint32_t)pool[src_off + phys] << 16);
        const float delta = __uint_as_float((uint32_t)res_val[e] << 16);
        const __bf16 sum = (__bf16)(base + delta);                       // round to nearest even
        pool[dst_off + phys] = __builtin_bit_cast(uint16_t, sum);
    }
    if (bad) bad_index = 1;                                              // benign race: every writer stores 1
    __syncthreads();
    if (status && tid == 0) status[item] = bad_index ? GF_RS_BAD_INDEX : GF_RS_OK;
}

hipError_t launch_residual(void *k_pool, void *v_pool, int32_t num_pool_blocks, int32_t hkv, int32_t head_dim,
                           int32_t num_items, const int32_t *src_blocks, const int32_t *dst_blocks,
                           const int32_t *res_ptr, const uint32_t *res_idx, const uint16_t *res_val,
                           int32_t *status, hipStream_t s) {
    if (num_items == 0) return hipSuccess;
    hipLaunchKernelGGL(residual_kernel, dim3((unsigned)num_items), dim3(kResidualThreads), 0, s, (uint16_t *)k_pool,
                       (uint16_t *)v_pool, num_pool_blocks, hkv, head_dim, src_blocks, dst_blocks, res_ptr, res_idx,
                       res_val, status);
    return hipGetLastError();
}

}  // namespace gf
