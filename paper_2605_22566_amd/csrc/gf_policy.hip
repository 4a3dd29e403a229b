// State-management policy on the device (paper, Differential-based KV Cache and Effective Path Pruning):
// a directory of the stored residuals, keyed by (prefix path, node) pairs; path resolution that also says, per
// table entry, which residual item the entry reads (or none: base block as it is / pair pruned, to be computed
// on the fly); execution statistics (how often each transition of E_op and each stored pair was used); and the
// pruning pass that drops the residuals of rarely taken transitions.  Integer work only; results are exact.
//
// The directory is an open-addressing hash table (linear probing, capacity a power of two) in caller-owned
// device arrays.  A pair's key is a 64-bit rolling hash of its prefix path (prefix_mix below, the published
// splitmix64 finaliser chained over the node ids); a slot matches when key, node and previous node all agree.
#include "gf_internal.h"

namespace gf {

__host__ __device__ __forceinline__ uint64_t prefix_mix(uint64_t h, int32_t v) {
    uint64_t z = (h ^ (uint64_t)(uint32_t)v) + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
__host__ __device__ __forceinline__ uint64_t prefix_key_final(uint64_t h) { return h ? h : 1; }   // 0 marks an empty slot

uint64_t prefix_key_host(const int32_t *nodes, int32_t len) {
    uint64_t h = 0;
    for (int32_t i = 0; i < len; ++i) h = prefix_mix(h, nodes[i]);
    return prefix_key_final(h);
}

constexpr int kPolicyThreads = 256;

__global__ __launch_bounds__(kPolicyThreads) void dir_clear_kernel(gf_residual_dir d) {
    const int i = blockIdx.x * kPolicyThreads + threadIdx.x;
    if (i >= d.capacity) return;
    d.key[i] = 0;
    d.prev[i] = -1;
    d.node[i] = -1;
    d.first_item[i] = -1;
    d.uses[i] = 0;
}

__global__ __launch_bounds__(kPolicyThreads) void dir_insert_kernel(gf_residual_dir d, int num_pairs,
                                                                    const uint64_t *__restrict__ keys,
                                                                    const int32_t *__restrict__ prev,
                                                                    const int32_t *__restrict__ node,
                                                                    const int32_t *__restrict__ first_item,
                                                                    int32_t *__restrict__ status) {
    const int i = blockIdx.x * kPolicyThreads + threadIdx.x;
    if (i >= num_pairs) return;
    const uint64_t k = keys[i];
    int st = GF_DIR_FULL;
    if (k == 0 || first_item[i] < 0) {
        st = GF_DIR_BAD_PAIR;
    } else {
        uint32_t slot = (uint32_t)k & (uint32_t)(d.capacity - 1);
        for (int probe = 0; probe < d.capacity; ++probe) {
            const unsigned long long old = atomicCAS((unsigned long long *)&d.key[slot], 0ull, (unsigned long long)k);
            if (old == 0ull) {           // the slot is this pair's
                d.prev[slot] = prev[i];
                d.node[slot] = node[i];
                d.first_item[slot] = first_item[i];
                d.uses[slot] = 0;
                st = GF_DIR_OK;
                break;
            }
            slot = (slot + 1) & (uint32_t)(d.capacity - 1);
        }
    }
    if (status) status[i] = st;
}

// position of w in v's successor list, or -1
__device__ __forceinline__ int edge_index(const int32_t *__restrict__ edge_ptr, const int32_t *__restrict__ edge_dst, int v,
                                          int w) {
    for (int e = edge_ptr[v]; e < edge_ptr[v + 1]; ++e)
        if (edge_dst[e] == w) return e;
    return -1;
}

// One workgroup per request, after resolve_kernel has written status[]: the handle row of the request.
__global__ __launch_bounds__(kPolicyThreads) void resolve_residual_kernel(
    int32_t num_nodes, const int32_t *__restrict__ node_len, const int32_t *__restrict__ edge_ptr,
    const int32_t *__restrict__ edge_dst, const int32_t *__restrict__ path_ptr, const int32_t *__restrict__ path_nodes,
    const int32_t *__restrict__ status, int32_t max_blocks, gf_residual_dir d, int32_t *__restrict__ trans_count,
    int32_t *__restrict__ res_handle, int32_t *__restrict__ num_fallback) {
    __shared__ unsigned long long keys[kPolicyThreads];
    __shared__ int scan[kPolicyThreads];
    __shared__ int chunk_nb[kPolicyThreads];
    __shared__ int chunk_first[kPolicyThreads];
    __shared__ int missing;
    __shared__ unsigned long long carry;

    const int r = blockIdx.x, tid = threadIdx.x;
    int32_t *row = res_handle + (size_t)r * max_blocks;
    int written = 0;
    if (tid == 0) {
        missing = 0;
        carry = 0;
    }
    __syncthreads();
    if (status[r] == GF_ST_OK) {            // a resolved request: every node id is valid, the table fits
        const int p0 = path_ptr[r];
        const int plen = path_ptr[r + 1] - p0;
        int base = 0;
        for (int c0 = 0; c0 < plen; c0 += kPolicyThreads) {
            const int cn = min(kPolicyThreads, plen - c0);
            if (tid == 0) {                  // the rolling key is a chain: one thread walks the chunk
                unsigned long long h = carry;
                for (int k = 0; k < cn; ++k) {
                    h = prefix_mix(h, path_nodes[p0 + c0 + k]);
                    keys[k] = h;
                }
                carry = h;
            }
            const int i = c0 + tid;
            int nb = 0, v = 0;
            if (i < plen) {
                v = path_nodes[p0 + i];
                const int len = node_len[v];
                nb = len > 0 ? (len + kBlock - 1) / kBlock : 0;
            }
            scan[tid] = nb;
            __syncthreads();
            for (int off = 1; off < kPolicyThreads; off <<= 1) {
                const int add = tid >= off ? scan[tid - off] : 0;
                __syncthreads();
                scan[tid] += add;
                __syncthreads();
            }
            const int incl = scan[tid];
            const int chunk_total = scan[kPolicyThreads - 1];
            __syncthreads();
            scan[tid] = base + incl - nb;
            chunk_nb[tid] = nb;
            int first = -1;
            if (i >= 1 && i < plen) {        // a node with a non-empty prefix: look its pair up
                const int u = path_nodes[p0 + i - 1];
                const unsigned long long key = prefix_key_final(keys[tid]);
                if (d.capacity > 0) {
                    uint32_t slot = (uint32_t)key & (uint32_t)(d.capacity - 1);
                    for (int probe = 0; probe < d.capacity; ++probe) {
                        const unsigned long long k = d.key[slot];
                        if (k == 0ull) break;
                        if (k == key && d.node[slot] == v && d.prev[slot] == u) {
                            atomicAdd(&d.uses[slot], 1);
                            first = d.first_item[slot];
                            break;
                        }
                        slot = (slot + 1) & (uint32_t)(d.capacity - 1);
                    }
                }
                if (first < 0) {
                    first = -1;
                    atomicAdd(&missing, 1);
                }
                if (trans_count && edge_ptr) {
                    const int e = edge_index(edge_ptr, edge_dst, u, v);
                    if (e >= 0) atomicAdd(&trans_count[e], 1);
                }
            }
            chunk_first[tid] = first;
            __syncthreads();
            for (int k = 0; k < cn; ++k) {
                const int knb = chunk_nb[k], off = scan[k], f = chunk_first[k];
                for (int j = tid; j < knb; j += kPolicyThreads)
                    if (off + j < max_blocks) row[off + j] = f >= 0 ? f + j : -1;
            }
            base += chunk_total;
            __syncthreads();
        }
        written = min(base, max_blocks);
    }
    for (int j = written + tid; j < max_blocks; j += kPolicyThreads) row[j] = -1;     // tail entries and padding
    __syncthreads();
    if (tid == 0) num_fallback[r] = missing;
}

__global__ __launch_bounds__(kPolicyThreads) void dir_prune_kernel(gf_residual_dir d, int32_t num_nodes,
                                                                   const int32_t *__restrict__ node_len,
                                                                   const int32_t *__restrict__ edge_ptr,
                                                                   const int32_t *__restrict__ edge_dst,
                                                                   const int32_t *__restrict__ trans_count, int min_count,
                                                                   int32_t *__restrict__ pruned) {
    const int i = blockIdx.x * kPolicyThreads + threadIdx.x;
    if (i >= d.capacity) return;
    if (d.key[i] == 0 || d.first_item[i] < 0) return;
    const int u = d.prev[i], v = d.node[i];
    int taken = 0, nb = 0;
    if (u >= 0 && u < num_nodes && v >= 0 && v < num_nodes) {
        const int e = edge_index(edge_ptr, edge_dst, u, v);
        taken = e >= 0 ? trans_count[e] : 0;
        const int len = node_len[v];
        nb = len > 0 ? (len + kBlock - 1) / kBlock : 0;
    }
    if (taken < min_count) {
        d.first_item[i] = -2 - d.first_item[i];          // pruned; the freed items stay readable
        if (pruned) {
            atomicAdd(&pruned[0], 1);
            atomicAdd(&pruned[1], nb);
        }
    }
}

hipError_t launch_dir_clear(const gf_residual_dir &d, hipStream_t s) {
    if (d.capacity == 0) return hipSuccess;
    hipLaunchKernelGGL(dir_clear_kernel, dim3((d.capacity + kPolicyThreads - 1) / kPolicyThreads), dim3(kPolicyThreads), 0,
                       s, d);
    return hipGetLastError();
}

hipError_t launch_dir_insert(const gf_residual_dir &d, int32_t num_pairs, const uint64_t *keys, const int32_t *prev,
                             const int32_t *node, const int32_t *first_item, int32_t *status, hipStream_t s) {
    if (num_pairs == 0) return hipSuccess;
    hipLaunchKernelGGL(dir_insert_kernel, dim3((num_pairs + kPolicyThreads - 1) / kPolicyThreads), dim3(kPolicyThreads), 0,
                       s, d, num_pairs, keys, prev, node, first_item, status);
    return hipGetLastError();
}

hipError_t launch_resolve_residual(const gf_graph &g, int32_t num_req, const int32_t *path_ptr, const int32_t *path_nodes,
                                   const int32_t *status, int32_t max_blocks, const gf_residual_dir &d,
                                   int32_t *trans_count, int32_t *res_handle, int32_t *num_fallback, hipStream_t s) {
    if (num_req == 0) return hipSuccess;
    hipLaunchKernelGGL(resolve_residual_kernel, dim3(num_req), dim3(kPolicyThreads), 0, s, g.num_nodes, g.node_len,
                       g.edge_ptr, g.edge_dst, path_ptr, path_nodes, status, max_blocks, d, trans_count, res_handle,
                       num_fallback);
    return hipGetLastError();
}

hipError_t launch_dir_prune(const gf_graph &g, const gf_residual_dir &d, const int32_t *trans_count, int32_t min_count,
                            int32_t *pruned, hipStream_t s) {
    if (d.capacity == 0) return hipSuccess;
    hipLaunchKernelGGL(dir_prune_kernel, dim3((d.capacity + kPolicyThreads - 1) / kPolicyThreads), dim3(kPolicyThreads), 0,
                       s, d, g.num_nodes, g.node_len, g.edge_ptr, g.edge_dst, trans_count, min_count, pruned);
    return hipGetLastError();
}

}  // namespace gf
