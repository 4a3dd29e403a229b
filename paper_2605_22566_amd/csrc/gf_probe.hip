// gf_hbm_read_probe: a plain read-only streaming kernel, the ceiling the bandwidth-bound decode kernels are
// measured against on the same box.  Every lane reads 16 bytes per trip, a workgroup walks the buffer with a
// grid stride (four independent loads in flight per lane), and the words read are folded into one sum per
// workgroup so that the loads cannot be dropped.  Nothing of the method is computed here.
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

hipError_t launch_hbm_read_probe(const void *src, size_t bytes, uint32_t *wg_sums, int32_t num_wg, hipStream_t s) {
    hipLaunchKernelGGL(hbm_read_probe_kernel, dim3((unsigned)num_wg), dim3(kProbeThreads), 0, s, (const u32x4 *)src,
                       bytes / 16, wg_sums);
    return hipGetLastError();
}

}  // namespace gf
