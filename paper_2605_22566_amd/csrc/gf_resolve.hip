// gf_resolve_path: wGraph node path -> per-request block table.
// (Paper, Topology-Aware State Management: a workflow's KV is assembled from
//  the precomputed KV of its selected operation nodes; Eq. 7's prefix path P is
//  the input; Overview: edges of E_op are the valid transitions.)
//
// One workgroup per request.  Pass 1 validates the path (node ids, edges,
// block ownership, block-id range) and counts blocks and context tokens with
// workgroup reductions; pass 2 walks the path in chunks of 256 nodes, scans
// the per-node block counts, and all threads copy each node's block list into
// the table with coalesced stores.  Integer work only.
#include "gf_internal.h"

namespace gf {

constexpr int kResolveThreads = 256;

__device__ __forceinline__ int block_reduce_sum(int v, int *lds) {
    // wave reduce then across the 4 waves
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds[wave] = v;
    __syncthreads();
    return lds[0] + lds[1] + lds[2] + lds[3];
}

__global__ __launch_bounds__(kResolveThreads) void resolve_kernel(
    int32_t num_nodes, const int32_t *__restrict__ node_len, const int32_t *__restrict__ node_block_ptr,
    const int32_t *__restrict__ node_blocks, const int32_t *__restrict__ edge_ptr,
    const int32_t *__restrict__ edge_dst, const int32_t *__restrict__ path_ptr,
    const int32_t *__restrict__ path_nodes, const int32_t *__restrict__ new_lens,
    const int32_t *__restrict__ tail_ptr, const int32_t *__restrict__ tail_blocks, int32_t max_blocks,
    int32_t num_pool_blocks, int32_t *__restrict__ block_table, int32_t *__restrict__ block_ntok,
    int32_t *__restrict__ num_blocks, int32_t *__restrict__ ctx_lens, int32_t *__restrict__ seq_lens,
    int32_t *__restrict__ status) {
    __shared__ int red[4];
    __shared__ int flags;                       // bit0 bad node, bit1 bad edge, bit2 bad block
    __shared__ int scan[kResolveThreads];       // per-chunk exclusive scan of block counts
    __shared__ int chunk_node[kResolveThreads];
    __shared__ int chunk_nb[kResolveThreads];
    __shared__ int chunk_len[kResolveThreads];

    const int r = blockIdx.x;
    const int tid = threadIdx.x;
    const int p0 = path_ptr[r];
    const int plen = path_ptr[r + 1] - p0;
    const int n_new = new_lens ? new_lens[r] : 0;
    const int t0 = tail_ptr ? tail_ptr[r] : 0;
    const int tail_have = tail_ptr ? tail_ptr[r + 1] - t0 : 0;
    const int tail_need = n_new > 0 ? (n_new + kBlock - 1) / kBlock : 0;

    if (tid == 0) flags = 0;
    __syncthreads();

    // ---- pass 1a: node ids -------------------------------------------------
    int f = 0;
    for (int i = tid; i < plen; i += kResolveThreads) {
        const int v = path_nodes[p0 + i];
        if (v < 0 || v >= num_nodes) f |= 1;
    }
    if (f) atomicOr(&flags, f);
    __syncthreads();
    const bool bad_node = flags & 1;

    // ---- pass 1b: edges, block ownership, counts (only with valid ids) ------
    int my_blocks = 0, my_ctx = 0;
    f = 0;
    if (!bad_node) {
        for (int i = tid; i < plen; i += kResolveThreads) {
            const int v = path_nodes[p0 + i];
            if (edge_ptr && i + 1 < plen) {
                const int w = path_nodes[p0 + i + 1];
                bool found = false;
                for (int e = edge_ptr[v]; e < edge_ptr[v + 1]; ++e) found |= (edge_dst[e] == w);
                if (!found) f |= 2;
            }
            const int len = node_len[v];
            const int own = node_block_ptr[v + 1] - node_block_ptr[v];
            const int nb = len > 0 ? (len + kBlock - 1) / kBlock : 0;
            if (len < 0 || own < nb) f |= 4;
            my_blocks += nb;
            my_ctx += len > 0 ? len : 0;
        }
    }
    if (f) atomicOr(&flags, f);
    const int ctx_blocks = block_reduce_sum(my_blocks, red);
    const int ctx = block_reduce_sum(my_ctx, red);
    __syncthreads();
    const int flags1 = flags;
    __syncthreads();   // every thread has read flags before pass 1c updates it
    const bool bad_edge = flags1 & 2;
    const bool bad_tail = n_new < 0 || tail_have < tail_need;

    // ---- pass 1c: block-id range (only if everything before it is fine) -----
    f = 0;
    if (!bad_node && !bad_edge && !bad_tail && !(flags1 & 4)) {
        for (int i = 0; i < plen; ++i) {      // nodes serially, blocks in parallel
            const int v = path_nodes[p0 + i];
            const int len = node_len[v];
            const int nb = (len + kBlock - 1) / kBlock;
            const int b0 = node_block_ptr[v];
            for (int j = tid; j < nb; j += kResolveThreads) {
                const int b = node_blocks[b0 + j];
                if (b < 0 || b >= num_pool_blocks) f |= 4;
            }
        }
        for (int j = tid; j < tail_need; j += kResolveThreads) {
            const int b = tail_blocks[t0 + j];
            if (b < 0 || b >= num_pool_blocks) f |= 4;
        }
    }
    if (f) atomicOr(&flags, f);
    __syncthreads();
    const bool bad_block = flags & 4;

    const int total_blocks = ctx_blocks + tail_need;
    int st = GF_ST_OK;
    if (bad_node) st = GF_ST_BAD_NODE;
    else if (bad_edge) st = GF_ST_BAD_EDGE;
    else if (bad_tail) st = GF_ST_BAD_TAIL;
    else if (bad_block) st = GF_ST_BAD_BLOCK;
    else if (total_blocks > max_blocks) st = GF_ST_OVERFLOW;

    int32_t *tab = block_table + (size_t)r * max_blocks;
    int32_t *ntk = block_ntok + (size_t)r * max_blocks;

    int written = 0;
    if (st == GF_ST_OK) {
        // ---- pass 2: expand node block lists in path order -------------------
        int base = 0;
        for (int c0 = 0; c0 < plen; c0 += kResolveThreads) {
            const int i = c0 + tid;
            int nb = 0, len = 0, v = 0;
            if (i < plen) {
                v = path_nodes[p0 + i];
                len = node_len[v];
                nb = (len + kBlock - 1) / kBlock;
            }
            // inclusive Hillis-Steele scan over the chunk
            scan[tid] = nb;
            __syncthreads();
            for (int off = 1; off < kResolveThreads; off <<= 1) {
                const int add = tid >= off ? scan[tid - off] : 0;
                __syncthreads();
                scan[tid] += add;
                __syncthreads();
            }
            const int incl = scan[tid];
            const int chunk_total = scan[kResolveThreads - 1];
            __syncthreads();
            scan[tid] = base + incl - nb;   // exclusive offset in the table
            chunk_node[tid] = v;
            chunk_nb[tid] = nb;
            chunk_len[tid] = len;
            __syncthreads();
            const int cn = min(kResolveThreads, plen - c0);
            for (int k = 0; k < cn; ++k) {
                const int knb = chunk_nb[k];
                const int off = scan[k];
                const int src = node_block_ptr[chunk_node[k]];
                const int last_tok = chunk_len[k] - kBlock * (knb - 1);
                for (int j = tid; j < knb; j += kResolveThreads) {
                    tab[off + j] = node_blocks[src + j];
                    ntk[off + j] = (j == knb - 1) ? last_tok : kBlock;
                }
            }
            base += chunk_total;
            __syncthreads();
        }
        // tail blocks
        const int last_tok = n_new - kBlock * (tail_need - 1);
        for (int j = tid; j < tail_need; j += kResolveThreads) {
            tab[base + j] = tail_blocks[t0 + j];
            ntk[base + j] = (j == tail_need - 1) ? last_tok : kBlock;
        }
        written = total_blocks;
    }
    for (int j = written + tid; j < max_blocks; j += kResolveThreads) {
        tab[j] = -1;
        ntk[j] = 0;
    }
    if (tid == 0) {
        const bool ok = st == GF_ST_OK;
        num_blocks[r] = ok ? total_blocks : 0;
        ctx_lens[r] = ok ? ctx : 0;
        seq_lens[r] = ok ? ctx + n_new : 0;
        status[r] = st;
    }
}

hipError_t launch_resolve(const gf_graph &g, int32_t num_req, const int32_t *path_ptr,
                          const int32_t *path_nodes, const int32_t *new_lens, const int32_t *tail_ptr,
                          const int32_t *tail_blocks, int32_t max_blocks, int32_t num_pool_blocks,
                          int32_t *block_table, int32_t *block_ntok, int32_t *num_blocks,
                          int32_t *ctx_lens, int32_t *seq_lens, int32_t *status, hipStream_t s) {
    if (num_req == 0) return hipSuccess;
    hipLaunchKernelGGL(resolve_kernel, dim3(num_req), dim3(kResolveThreads), 0, s, g.num_nodes, g.node_len,
                       g.node_block_ptr, g.node_blocks, g.edge_ptr, g.edge_dst, path_ptr, path_nodes,
                       new_lens, tail_ptr, tail_blocks, max_blocks, num_pool_blocks, block_table, block_ntok,
                       num_blocks, ctx_lens, seq_lens, status);
    return hipGetLastError();
}

}  // namespace gf
