// gf_hbm_read_probe: a plain read-only streaming kernel, the ceiling the bandwidth-bound decode kernels are
// measured against on the same box.  Every lane reads 16 bytes per trip, a workgroup walks the buffer with a
// grid stride (four independent loads in flight per lane), and the words read are folded into one sum per
// workgroup so that the loads cannot be dropped.  Nothing of the method is computed here.
//
// gf_mfma_probe: the same kind of ceiling for the matrix pipes the prefill kernel is measured against -- nothing
// but v_mfma_f32_32x32x16_bf16 (the prefill's instruction) on operands the caller supplies, so that the rate the
// chip sustains can be read for zeroed operands and for operands distributed like K, V and Q.
#include "gf_internal.h"

namespace gf {

constexpr int kProbeThreads = 256;

__global__ __launch_bounds__(kProbeThreads) void hbm_read_probe_kernel(const u32x4 *__restrict__ src, size_t n16,
                                                                      uint32_t *__restrict__ wg_sums) {
    const size_t stride = (size_t)gridDim.x * kProbeThreads;
    size_t i = (size_t)blockIdx.x * kProbeThreads + threadIdx.x;
    uint32_t acc = 0;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + stride);
        const u32x4 c = __builtin_nontemporal_load(src + i + 2 * stride), d = __builtin_nontemporal_load(src + i + 3 * stride);
        acc += (a[0] + a[1]) + (a[2] + a[3]) + (b[0] + b[1]) + (b[2] + b[3]) + (c[0] + c[1]) + (c[2] + c[3]) +
               (d[0] + d[1]) + (d[2] + d[3]);
    }
    for (; i < n16; i += stride) {
        const u32x4 a = __builtin_nontemporal_load(src + i);
        acc += (a[0] + a[1]) + (a[2] + a[3]);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    __shared__ uint32_t part[kProbeThreads / 64];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t t = 0;
#pragma unroll
        for (int w = 0; w < kProbeThreads / 64; ++w) t += part[w];
        wg_sums[blockIdx.x] = t;
    }
}

// The same ceiling for the access pattern of a block table: the buffer is read as tiles of `tile_bytes`
// contiguous bytes (a multiple of 1 KB; 4 KB is one (block, kv head) image of K or V at head_dim 128) in the order
// an index array gives.  One wave takes a tile at a time, 16 bytes per lane and load, two tiles in flight; ids
// outside [0, num_src_tiles) are folded into the range, so every access stays inside the buffer.
__global__ __launch_bounds__(kProbeThreads) void hbm_tile_probe_kernel(const char *__restrict__ src, int tile_bytes,
                                                                      int num_src_tiles, const int32_t *__restrict__ ids,
                                                                      long num_tiles, uint32_t *__restrict__ wg_sums) {
    const int lane = threadIdx.x & 63;
    const long wave = (long)blockIdx.x * (kProbeThreads / 64) + (threadIdx.x >> 6);
    const long waves = (long)gridDim.x * (kProbeThreads / 64);
    const int loads = tile_bytes / 1024;
    uint32_t acc = 0;
    auto tile_of = [&](long i) -> const u32x4 * {
        const int t = (int)((uint32_t)ids[i] % (uint32_t)num_src_tiles);
        return (const u32x4 *)(src + (size_t)t * tile_bytes) + lane;
    };
    long i = wave;
    for (; i + waves < num_tiles; i += 2 * waves) {
        const u32x4 *pa = tile_of(i), *pb = tile_of(i + waves);
        for (int j = 0; j < loads; ++j) {
            const u32x4 a = __builtin_nontemporal_load(pa + 64 * j), b = __builtin_nontemporal_load(pb + 64 * j);
            acc += (a[0] + a[1]) + (a[2] + a[3]) + (b[0] + b[1]) + (b[2] + b[3]);
        }
    }
    for (; i < num_tiles; i += waves) {
        const u32x4 *pa = tile_of(i);
        for (int j = 0; j < loads; ++j) {
            const u32x4 a = __builtin_nontemporal_load(pa + 64 * j);
            acc += (a[0] + a[1]) + (a[2] + a[3]);
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    __shared__ uint32_t part[kProbeThreads / 64];
    if (lane == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t t = 0;
#pragma unroll
        for (int w = 0; w < kProbeThreads / 64; ++w) t += part[w];
        wg_sums[blockIdx.x] = t;
    }
}

// One wave per SIMD and workgroup (more waves per SIMD through more workgroups per CU).  A wave reads eight A
// and four B fragments (64 lanes x 8 bf16 each) from `operands` once, then issues `iters` rounds of eight MFMAs
// into four independent accumulators, every MFMA with another pair of fragments than the one before it, so the
// multiplier inputs change at the rate they do in an attention tile.  With MIX every MFMA is followed by the
// vector instructions a softmax spends per MFMA at head_dim 128 -- six, one of them an exponential -- on values
// that keep changing (x <- fract(x * k + y) walks over [0, 1) without settling).  The accumulators and the
// vector values are folded into one float per lane at the end so that nothing can be dropped.
constexpr int kProbeA = 8, kProbeB = 4;

template <bool MIX>
__global__ __launch_bounds__(kProbeThreads) void mfma_probe_kernel(const u32x4 *__restrict__ operands, uint32_t n_chunks,
                                                                  int iters, float *__restrict__ lane_sums) {
    const int lane = threadIdx.x & 63;
    const uint32_t wave = blockIdx.x * (kProbeThreads / 64) + (threadIdx.x >> 6);
    bf16x8 a[kProbeA], b[kProbeB];
#pragma unroll
    for (int f = 0; f < kProbeA + kProbeB; ++f) {
        const uint32_t chunk = (wave * (kProbeA + kProbeB) + f) % n_chunks;          // 1 KB chunks of the buffer
        const bf16x8 x = __builtin_bit_cast(bf16x8, operands[(size_t)chunk * 64 + lane]);
        if (f < kProbeA) a[f] = x;
        else b[f - kProbeA] = x;
    }
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    // vector state: four values in [0, 1) taken from the mantissas of the first fragment (zero operands: zeros)
    float x[4], esum = 0.f;
    {
        const u32x4 w = __builtin_bit_cast(u32x4, a[0]);
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] = __uint_as_float((w[i] & 0x007fffffu) | 0x3f800000u) - 1.0f;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < kProbeA; ++j) {
            acc[j % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[(j + j / 4) % kProbeB], acc[j % 4], 0, 0, 0);
            if constexpr (MIX) {
                float &p = x[j % 4], &q = x[(j + 1) % 4];
                p = __builtin_amdgcn_fractf(__builtin_fmaf(p, 1.6180340f, q));
                q = __builtin_amdgcn_fractf(__builtin_fmaf(q, 2.4142137f, p));
                esum = __builtin_fmaf(fast_exp2(p), 0.001f, esum);
                __builtin_amdgcn_sched_barrier(0);                  // the vector work stays behind its MFMA
            }
        }
    }
    float sum = MIX ? (x[0] + x[1]) + (x[2] + x[3]) + esum : 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) sum += acc[j][i];
    lane_sums[(size_t)blockIdx.x * kProbeThreads + threadIdx.x] = sum;
}

hipError_t launch_mfma_probe(const void *operands, int64_t operand_bytes, int32_t iters, int32_t softmax_mix,
                             float *lane_sums, int32_t num_wg, hipStream_t s) {
    const dim3 grid((unsigned)num_wg), block(kProbeThreads);
    if (softmax_mix)
        hipLaunchKernelGGL(mfma_probe_kernel<true>, grid, block, 0, s, (const u32x4 *)operands,
                           (uint32_t)(operand_bytes / 1024), iters, lane_sums);
    else
        hipLaunchKernelGGL(mfma_probe_kernel<false>, grid, block, 0, s, (const u32x4 *)operands,
                           (uint32_t)(operand_bytes / 1024), iters, lane_sums);
    return hipGetLastError();
}

hipError_t launch_hbm_tile_probe(const void *src, int32_t tile_bytes, int32_t num_src_tiles, const int32_t *ids,
                                 int64_t num_tiles, uint32_t *wg_sums, int32_t num_wg, hipStream_t s) {
    hipLaunchKernelGGL(hbm_tile_probe_kernel, dim3((unsigned)num_wg), dim3(kProbeThreads), 0, s, (const char *)src,
                       tile_bytes, num_src_tiles, ids, (long)num_tiles, wg_sums);
    return hipGetLastError();
}

hipError_t launch_hbm_read_probe(const void *src, size_t bytes, uint32_t *wg_sums, int32_t num_wg, hipStream_t s) {
    hipLaunchKernelGGL(hbm_read_probe_kernel, dim3((unsigned)num_wg), dim3(kProbeThreads), 0, s, (const u32x4 *)src,
                       bytes / 16, wg_sums);
    return hipGetLastError();
}

}  // namespace gf
