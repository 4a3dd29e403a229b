// gf_kv_make_residual: from dense prefix-conditioned KV to the stored sparse residual (paper, Differential-based
// KV Cache, Eq. 7, and the selection rule of its sparsity appendix: of the difference between the KV of an
// operation under a prefix and its base KV, keep the largest-magnitude entries that hold a given share -- 95 % --
// of the Frobenius energy).  Item b compares pool block full_blocks[b] with pool block base_blocks[b]; every
// (item, tensor, kv head) image of 16 x D elements becomes one row of the CSR that gf_kv_apply_residual and
// gf_attn_decode_residual read (16-bit logical index slot * D + d, bf16 value = the rounded difference).
//
// One workgroup per image, three launches: count (entries kept per row, and the sort key of the last kept one),
// scan (row pointers, one workgroup), fill (the elements whose key reaches the row's last kept key, written in
// index order).  Inside an image: difference in fp32, a bitonic sort by (magnitude descending, index ascending),
// the squared magnitudes summed in fp64 along that order, and the shortest prefix whose sum reaches share x total.  The sort keeps the keys in registers:
// thread t owns the eight sorted positions 8 t .. 8 t + 7, so a compare-exchange at distance below 8 stays inside
// a thread, one at distance below 512 is a lane exchange inside a wave, and only the three stages at distance
// 512 or 1024 (D = 128) go through LDS.  An offline step (a residual is made once per (prefix, node) pair and
// read many times).
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

// sort key of logical element i with difference d: magnitude bits << 17 | (0xFFFF - i) << 1 | sign -- larger
// magnitude first, equal magnitudes by rising index; unique within an image
__device__ __forceinline__ unsigned long long sort_key(float d, int i) {
    const uint32_t bits = __float_as_uint(d);
    return ((unsigned long long)(bits & 0x7fffffffu) << 17) | ((unsigned long long)(0xFFFFu - (uint32_t)i) << 1) |
           (bits >> 31);
}
constexpr unsigned long long kKeepNone = ~0ull;            // above every key: a row that keeps nothing

// full - base for the PER elements stored from position p0 of an image on (PER = 8 or 4: one 16- or 8-byte load each)
template <int PER>
__device__ __forceinline__ void load_differences(const uint16_t *pf, const uint16_t *pb, int p0, float (&d)[PER]) {
    static_assert(PER == 8 || PER == 4, "whole vector loads");
    uint32_t f[PER / 2], b[PER / 2];
    if constexpr (PER == 8) {
        const u32x4 vf = *(const u32x4 *)(pf + p0), vb = *(const u32x4 *)(pb + p0);
#pragma unroll
        for (int w = 0; w < 4; ++w) { f[w] = vf[w]; b[w] = vb[w]; }
    } else {
        const u32x2 vf = *(const u32x2 *)(pf + p0), vb = *(const u32x2 *)(pb + p0);
#pragma unroll
        for (int w = 0; w < 2; ++w) { f[w] = vf[w]; b[w] = vb[w]; }
    }
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const uint32_t xf = (u & 1) ? (f[u / 2] & 0xffff0000u) : (f[u / 2] << 16);
        const uint32_t xb = (u & 1) ? (b[u / 2] & 0xffff0000u) : (b[u / 2] << 16);
        d[u] = __uint_as_float(xf) - __uint_as_float(xb);
    }
}
// logical index slot * D + d of the element stored at position p of a K image ([slot][d]) or a V image ([d][slot])
template <int D>
__device__ __forceinline__ int logical_index(int tensor, int p) {
    return tensor ? (p % kBlock) * D + p / kBlock : p;
}

template <int D>
__global__ __launch_bounds__(kMakeThreads) void make_residual_count_kernel(
    const uint16_t *__restrict__ k_pool, const uint16_t *__restrict__ v_pool, int num_pool_blocks, int hkv,
    const int32_t *__restrict__ base_blocks, const int32_t *__restrict__ full_blocks, double share,
    int32_t *__restrict__ res_ptr, unsigned long long *__restrict__ cut_keys) {
    constexpr int N = kBlock * D;                          // elements of an image
    constexpr int PER = N / kMakeThreads;                  // per thread
    static_assert(N % kMakeThreads == 0 && (N & (N - 1)) == 0, "power-of-two image, whole elements per thread");
    static_assert(PER == 8 || PER == 4, "sorted positions per thread");
    __shared__ unsigned long long xch[N];                  // exchange buffer of the sort's cross-wave stages
    __shared__ double dsum[kMakeThreads];
    __shared__ int cut;                                    // entries kept
    const int tid = threadIdx.x;
    const int rows = 2 * hkv;
    const int row = blockIdx.x, item = row / rows, t = (row % rows) / hkv, h = row % hkv;
    const int base = base_blocks[item], full = full_blocks[item];
    const bool ok = base >= 0 && base < num_pool_blocks && full >= 0 && full < num_pool_blocks;
    if (!ok) {                                             // uniform: the whole workgroup leaves
        if (tid == 0) {
            res_ptr[row + 1] = 0;
            cut_keys[row] = kKeepNone;
        }
        return;
    }
    const uint16_t *pool = t ? v_pool : k_pool;
    const uint16_t *pb = pool + ((size_t)base * hkv + h) * N, *pf = pool + ((size_t)full * hkv + h) * N;
    // 1. differences, keyed for the sort by their logical index.  Which thread starts with which element does
    //    not matter to a sort: every thread takes PER consecutive stored elements.
    unsigned long long key[PER];
    {
        float d[PER];
        load_differences<PER>(pf, pb, tid * PER, d);
#pragma unroll
        for (int u = 0; u < PER; ++u) key[u] = sort_key(d[u], logical_index<D>(t, tid * PER + u));
    }
    // 2. bitonic sort, descending over positions PER * tid + u: largest magnitude first, equal magnitudes by rising
    //    index.  Stage (k, j) pairs position i with i ^ j; the pair is in falling order where (i & k) == 0.
#pragma unroll
    for (int k = 2; k <= N; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
            if (j < PER) {                                 // both positions in this thread
#pragma unroll
                for (int u = 0; u < PER; ++u) {
                    if ((u & j) == 0) {
                        const bool desc = ((tid * PER + u) & k) == 0;
                        const unsigned long long a = key[u], b = key[u | j];
                        const unsigned long long hi = a > b ? a : b, lo = a > b ? b : a;
                        key[u] = desc ? hi : lo;
                        key[u | j] = desc ? lo : hi;
                    }
                }
            } else {                                       // the same u in thread tid ^ (j / PER)
                const int dt = j / PER;
                const bool take_max = ((tid & dt) == 0) == (((tid * PER) & k) == 0);
                if (dt < 64) {
#pragma unroll
                    for (int u = 0; u < PER; ++u) {
                        const unsigned long long a = key[u], b = __shfl_xor(a, dt, 64);
                        key[u] = (a > b) == take_max ? a : b;
                    }
                } else {
#pragma unroll
                    for (int u = 0; u < PER; ++u) xch[u * kMakeThreads + tid] = key[u];
                    __syncthreads();
#pragma unroll
                    for (int u = 0; u < PER; ++u) {
                        const unsigned long long a = key[u], b = xch[u * kMakeThreads + (tid ^ dt)];
                        key[u] = (a > b) == take_max ? a : b;
                    }
                    __syncthreads();
                }
            }
        }
    }
    // 3. energy along the sorted order: thread tid owns sorted positions [tid * PER, (tid + 1) * PER)
    double e[PER], mine = 0.0;
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const double m = (double)__uint_as_float((uint32_t)(key[u] >> 17));
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
    if (tid == 0) {
        res_ptr[row + 1] = n_keep;
        if (n_keep == 0) cut_keys[row] = kKeepNone;
    }
#pragma unroll
    for (int u = 0; u < PER; ++u)
        if (tid * PER + u == n_keep - 1) cut_keys[row] = key[u];           // the last kept one: kept <=> key >= this
}

// The kept elements of an image, in index order: thread t owns logical indices 8 t .. 8 t + 7 (PER in general).
template <int D>
__global__ __launch_bounds__(kMakeThreads) void make_residual_fill_kernel(
    const uint16_t *__restrict__ k_pool, const uint16_t *__restrict__ v_pool, int num_pool_blocks, int hkv,
    const int32_t *__restrict__ base_blocks, const int32_t *__restrict__ full_blocks, int capacity,
    const int32_t *__restrict__ res_ptr, const unsigned long long *__restrict__ cut_keys,
    uint16_t *__restrict__ res_idx, uint16_t *__restrict__ res_val, int32_t *__restrict__ status) {
    constexpr int N = kBlock * D, PER = N / kMakeThreads;
    __shared__ int isum[kMakeThreads];
    __shared__ __attribute__((aligned(16))) float dif[N];  // V: the differences by logical index
    const int tid = threadIdx.x;
    const int rows = 2 * hkv;
    const int row = blockIdx.x, item = row / rows, t = (row % rows) / hkv, h = row % hkv;
    const int base = base_blocks[item], full = full_blocks[item];
    const bool ok = base >= 0 && base < num_pool_blocks && full >= 0 && full < num_pool_blocks;
    if (!ok) {                                             // uniform: the whole workgroup leaves
        if (status && tid == 0 && row % rows == 0) status[item] = GF_RS_BAD_BLOCK;
        return;
    }
    const uint16_t *pool = t ? v_pool : k_pool;
    const uint16_t *pb = pool + ((size_t)base * hkv + h) * N, *pf = pool + ((size_t)full * hkv + h) * N;
    const unsigned long long cut_key = cut_keys[row];
    float d[PER];
    load_differences<PER>(pf, pb, tid * PER, d);           // PER consecutive stored elements
    if (t) {                                               // V is stored [d][slot]: to logical order through LDS
#pragma unroll
        for (int u = 0; u < PER; ++u) dif[logical_index<D>(1, tid * PER + u)] = d[u];
        __syncthreads();
#pragma unroll
        for (int u = 0; u < PER; ++u) d[u] = dif[tid * PER + u];
    }
    int cnt = 0;
#pragma unroll
    for (int u = 0; u < PER; ++u) cnt += sort_key(d[u], tid * PER + u) >= cut_key;
    int tot;
    int off = block_offset(cnt, isum, tot);
    const int out0 = res_ptr[row];
    bool cutoff = false;
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int i = tid * PER + u;
        if (sort_key(d[u], i) >= cut_key) {
            const long o = (long)out0 + off;
            if (o < capacity) {
                res_idx[o] = (uint16_t)i;
                res_val[o] = __builtin_bit_cast(uint16_t, (__bf16)d[u]);   // round to nearest even
            } else {
                cutoff = true;
            }
            ++off;
        }
    }
    if (status && cutoff) status[item] = GF_RS_TRUNCATED;                  // benign race: every writer stores the same
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
                                void *cut_keys, hipStream_t s) {
    const long rows = (long)num_items * 2 * hkv;
    if (status)
        hipLaunchKernelGGL(make_residual_status_kernel, dim3((num_items + 255) / 256), dim3(256), 0, s, status, num_items);
    hipLaunchKernelGGL((make_residual_count_kernel<D>), dim3((unsigned)rows), dim3(kMakeThreads), 0, s,
                       (const uint16_t *)k_pool, (const uint16_t *)v_pool, num_pool_blocks, hkv, base_blocks, full_blocks,
                       share, res_ptr, (unsigned long long *)cut_keys);
    hipLaunchKernelGGL(make_residual_scan_kernel, dim3(1), dim3(kMakeScanThreads), 0, s, res_ptr, rows);
    hipLaunchKernelGGL((make_residual_fill_kernel<D>), dim3((unsigned)rows), dim3(kMakeThreads), 0, s,
                       (const uint16_t *)k_pool, (const uint16_t *)v_pool, num_pool_blocks, hkv, base_blocks, full_blocks,
                       capacity, res_ptr, (const unsigned long long *)cut_keys, res_idx, res_val, status);
    return hipGetLastError();
}

size_t make_residual_scratch_bytes(int32_t hkv, int32_t num_items) { return (size_t)num_items * 2 * hkv * 8; }

hipError_t launch_make_residual(const void *k_pool, const void *v_pool, int32_t num_pool_blocks, int32_t hkv,
                                int32_t head_dim, int32_t num_items, const int32_t *base_blocks,
                                const int32_t *full_blocks, double share, int32_t capacity, int32_t *res_ptr,
                                uint16_t *res_idx, uint16_t *res_val, int32_t *status, void *cut_keys, hipStream_t s) {
    if (num_items == 0) return hipSuccess;
    if (head_dim == 64)
        return launch_make_t<64>(k_pool, v_pool, num_pool_blocks, hkv, num_items, base_blocks, full_blocks, share, capacity,
                                 res_ptr, res_idx, res_val, status, cut_keys, s);
    if (head_dim == 128)
        return launch_make_t<128>(k_pool, v_pool, num_pool_blocks, hkv, num_items, base_blocks, full_blocks, share, capacity,
                                  res_ptr, res_idx, res_val, status, cut_keys, s);
    return hipErrorNotSupported;
}

}  // namespace gf
