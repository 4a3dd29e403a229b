// gf_kv_make_residual: from dense prefix-conditioned KV to the stored sparse residual (paper, Differential-based
// KV Cache, Eq. 7, and the selection rule of its sparsity appendix: of the difference between the KV of an
// operation under a prefix and its base KV, keep the largest-magnitude entries that hold a given share -- 95 % --
// of the Frobenius energy).  Item b compares pool block full_blocks[b] with pool block base_blocks[b]; every
// (item, tensor, kv head) image of 16 x D elements becomes one row of the CSR that gf_kv_apply_residual and
// gf_attn_decode_residual read (16-bit logical index slot * D + d, bf16 value = the rounded difference).
//
// One workgroup per image, three launches: count (entries kept per row), scan (row pointers, one workgroup),
// fill (the selection is taken again, the entries are written in index order).  Inside an image: difference in
// fp32, a bitonic sort in LDS by (magnitude descending, index ascending), the squared magnitudes summed in
// fp64 along that order, and the shortest prefix whose sum reaches share x total.  An offline step (a residual
// is made once per (prefix, node) pair and read many times): written for clarity of the rule, not for speed.
#include "gf_internal.h"

namespace gf {

constexpr int kMakeThreads = 256;
constexpr int kMakeScanThreads = 1024;

// Exclusive scan over the workgroup of one value per thread: returns the sum of the values of the threads before
// this one (no subtraction: the offset of thread t is the scanned value of thread t - 1); `sh` has kMakeThreads
// entries.  `total` = offset of the last thread + its value, so that a running sum carried on from an offset
// ends exactly on it.
template <typename T>
__device__ __forceinline__ T block_offset(T mine, T *sh, T &total) {
    const int tid = threadIdx.x;
    sh[tid] = mine;
    __syncthreads();
    for (int off = 1; off < kMakeThreads; off <<= 1) {
        const T add = tid >= off ? sh[tid - off] : T(0);
        __syncthreads();
        sh[tid] += add;
        __syncthreads();
    }
    const T excl = tid > 0 ? sh[tid - 1] : T(0);
    __syncthreads();
    if (tid == kMakeThreads - 1) sh[0] = excl + mine;
    __syncthreads();
    total = sh[0];
    __syncthreads();
    return excl;
}

template <int D, bool FILL>
__global__ __launch_bounds__(kMakeThreads) void make_residual_kernel(
    const uint16_t *__restrict__ k_pool, const uint16_t *__restrict__ v_pool, int num_pool_blocks, int hkv,
    const int32_t *__restrict__ base_blocks, const int32_t *__restrict__ full_blocks, double share, int capacity,
    int32_t *__restrict__ res_ptr, uint16_t *__restrict__ res_idx, uint16_t *__restrict__ res_val,
    int32_t *__restrict__ status) {
    constexpr int N = kBlock * D;                          // elements of an image
    constexpr int PER = N / kMakeThreads;                  // per thread
    static_assert(N % kMakeThreads == 0 && (N & (N - 1)) == 0, "power-of-two image, whole elements per thread");
    __shared__ unsigned long long key[N];                  // magnitude bits << 17 | (0xFFFF - index) << 1 | sign
    __shared__ double dsum[kMakeThreads];
    __shared__ uint16_t kept[N];                           // FILL: 1 where the element is kept, by logical index
    __shared__ int isum[kMakeThreads];
    __shared__ int cut;                                    // entries kept
    const int tid = threadIdx.x;
    const int rows = 2 * hkv;
    const int row = blockIdx.x, item = row / rows, t = (row % rows) / hkv, h = row % hkv;
    const int base = base_blocks[item], full = full_blocks[item];
    const bool ok = base >= 0 && base < num_pool_blocks && full >= 0 && full < num_pool_blocks;
    if (!ok) {                                             // uniform: the whole workgroup leaves
        if (!FILL && tid == 0) res_ptr[row + 1] = 0;
        if (FILL && status && tid == 0 && row % rows == 0) status[item] = GF_RS_BAD_BLOCK;
        return;
    }
    const uint16_t *pool = t ? v_pool : k_pool;
    const uint16_t *pb = pool + ((size_t)base * hkv + h) * N, *pf = pool + ((size_t)full * hkv + h) * N;
    // 1. differences, keyed for the sort (logical index i; the V image is stored [d][slot])
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int i = u * kMakeThreads + tid;
        const int phys = t ? (i % D) * kBlock + i / D : i;
        const float d = __uint_as_float((uint32_t)pf[phys] << 16) - __uint_as_float((uint32_t)pb[phys] << 16);
        const uint32_t bits = __float_as_uint(d);
        key[i] = ((unsigned long long)(bits & 0x7fffffffu) << 17) | ((unsigned long long)(0xFFFFu - (uint32_t)i) << 1) |
                 (bits >> 31);
    }
    __syncthreads();
    // 2. bitonic sort, descending: largest magnitude first, equal magnitudes by rising index
    for (int k = 2; k <= N; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
#pragma unroll
            for (int u = 0; u < PER; ++u) {
                const int i = u * kMakeThreads + tid, l = i ^ j;
                if (l > i) {
                    const unsigned long long a = key[i], b = key[l];
                    const bool desc = (i & k) == 0;
                    if (desc ? a < b : a > b) {
                        key[i] = b;
                        key[l] = a;
                    }
                }
            }
            __syncthreads();
        }
    // 3. energy along the sorted order: thread tid owns sorted positions [tid * PER, (tid + 1) * PER)
    double e[PER], mine = 0.0;
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const double m = (double)__uint_as_float((uint32_t)(key[tid * PER + u] >> 17));
        e[u] = m * m;
        mine += e[u];                                      // the same additions, in the same order, as `run` below
    }
    double total;
    double run = block_offset(mine, dsum, total);
    const double thr = share * total;
    if (tid == 0) cut = N;
    __syncthreads();
    if (total > 0.0) {
        // first sorted position whose running sum reaches the threshold (the sums rise: one thread finds it)
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const double before = run;
            run += e[u];
            if (run >= thr && !(before >= thr && (tid * PER + u) > 0)) atomicMin(&cut, tid * PER + u + 1);
        }
    } else if (tid == 0) {
        cut = 0;
    }
    __syncthreads();
    const int n_keep = cut;
    if constexpr (!FILL) {
        if (tid == 0) res_ptr[row + 1] = n_keep;
        return;
    } else {
        // 4. the kept elements in index order
#pragma unroll
        for (int u = 0; u < PER; ++u) kept[u * kMakeThreads + tid] = 0;
        __syncthreads();
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int pos = u * kMakeThreads + tid;
            if (pos < n_keep) kept[0xFFFFu - (uint32_t)((key[pos] >> 1) & 0xFFFFu)] = 1;
        }
        __syncthreads();
        int cnt = 0;
#pragma unroll
        for (int u = 0; u < PER; ++u) cnt += kept[tid * PER + u];      // thread tid owns indices [tid * PER, +PER)
        int tot;
        int off = block_offset(cnt, isum, tot);
        const int out0 = res_ptr[row];
        bool cutoff = false;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int i = tid * PER + u;
            if (kept[i]) {
                const int phys = t ? (i % D) * kBlock + i / D : i;
                const float d = __uint_as_float((uint32_t)pf[phys] << 16) - __uint_as_float((uint32_t)pb[phys] << 16);
                const long o = (long)out0 + off;
                if (o < capacity) {
                    res_idx[o] = (uint16_t)i;
                    res_val[o] = __builtin_bit_cast(uint16_t, (__bf16)d);     // round to nearest even
                } else {
                    cutoff = true;
                }
                ++off;
            }
        }
        if (status && cutoff) status[item] = GF_RS_TRUNCATED;              // benign race: every writer stores the same
    }
}

// counts in res_ptr[1 .. rows] -> row pointers (exclusive prefix, res_ptr[0] = 0), in place, one workgroup
__global__ __launch_bounds__(kMakeScanThreads) void make_residual_scan_kernel(int32_t *__restrict__ res_ptr, long rows) {
    __shared__ int sh[kMakeScanThreads];
    const int tid = threadIdx.x;
    int carry = 0;
    if (tid == 0) res_ptr[0] = 0;
    for (long b = 0; b < rows; b += kMakeScanThreads) {
        const long i = b + tid;
        const int x = i < rows ? res_ptr[i + 1] : 0;
        sh[tid] = x;
        __syncthreads();
        for (int o = 1; o < kMakeScanThreads; o <<= 1) {
            const int y = tid >= o ? sh[tid - o] : 0;
            __syncthreads();
            sh[tid] += y;
            __syncthreads();
        }
        if (i < rows) res_ptr[i + 1] = carry + sh[tid];
        carry += sh[kMakeScanThreads - 1];
        __syncthreads();
    }
}

__global__ void make_residual_status_kernel(int32_t *status, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) status[i] = GF_RS_OK;
}

template <int D>
static hipError_t launch_make_t(const void *k_pool, const void *v_pool, int32_t num_pool_blocks, int32_t hkv,
                                int32_t num_items, const int32_t *base_blocks, const int32_t *full_blocks, double share,
                                int32_t capacity, int32_t *res_ptr, uint16_t *res_idx, uint16_t *res_val, int32_t *status,
                                hipStream_t s) {
    const long rows = (long)num_items * 2 * hkv;
    if (status)
        hipLaunchKernelGGL(make_residual_status_kernel, dim3((num_items + 255) / 256), dim3(256), 0, s, status, num_items);
    hipLaunchKernelGGL((make_residual_kernel<D, false>), dim3((unsigned)rows), dim3(kMakeThreads), 0, s,
                       (const uint16_t *)k_pool, (const uint16_t *)v_pool, num_pool_blocks, hkv, base_blocks, full_blocks,
                       share, capacity, res_ptr, res_idx, res_val, status);
    hipLaunchKernelGGL(make_residual_scan_kernel, dim3(1), dim3(kMakeScanThreads), 0, s, res_ptr, rows);
    hipLaunchKernelGGL((make_residual_kernel<D, true>), dim3((unsigned)rows), dim3(kMakeThreads), 0, s,
                       (const uint16_t *)k_pool, (const uint16_t *)v_pool, num_pool_blocks, hkv, base_blocks, full_blocks,
                       share, capacity, res_ptr, res_idx, res_val, status);
    return hipGetLastError();
}

hipError_t launch_make_residual(const void *k_pool, const void *v_pool, int32_t num_pool_blocks, int32_t hkv,
                                int32_t head_dim, int32_t num_items, const int32_t *base_blocks,
                                const int32_t *full_blocks, double share, int32_t capacity, int32_t *res_ptr,
                                uint16_t *res_idx, uint16_t *res_val, int32_t *status, hipStream_t s) {
    if (num_items == 0) return hipSuccess;
    if (head_dim == 64)
        return launch_make_t<64>(k_pool, v_pool, num_pool_blocks, hkv, num_items, base_blocks, full_blocks, share, capacity,
                                 res_ptr, res_idx, res_val, status, s);
    if (head_dim == 128)
        return launch_make_t<128>(k_pool, v_pool, num_pool_blocks, hkv, num_items, base_blocks, full_blocks, share, capacity,
                                  res_ptr, res_idx, res_val, status, s);
    return hipErrorNotSupported;
}

}  // namespace gf
