// gf_attn_decode_shared: the decode step of gf_attn_decode, reading every shared node once per
// group of requests instead of once per request (paper, Topology-Aware State Management and the
// operation-level overlap it rests on: the KV of an operation node is shared by all workflows
// that pass through it -- here the sharing is used for the reads as well as for the storage).
//
// Node-centric order.  The batch's path lists are inverted on the device into node -> requests
// lists.  One wavefront then reduces one (node, kv head, chunk of the node's blocks, group of 16
// score columns), where a column is a (request through that node, query head of the group) pair:
// the K/V blocks it loads feed 16/G requests at once (v_mfma_f32_16x16x32_bf16 with all 16
// columns in use, where the request-centric kernel pads G heads to 16).  It leaves one fp32
// partial (max, sum, weighted values) per (request, path node, chunk).  The private tail blocks
// of a request (its new tokens) are reduced request by request as before, and one merge kernel
// combines a request's partials -- path nodes in order, then tail -- with the log-sum-exp rule.
// The result is the request-centric one up to fp32 summation order.
//
// Integer preparation (all on the device, no host round trip):
//   count   per request: its path entries -> cnt[node] (atomics), request of every entry
//   scan    one workgroup: node_ptr = scan(cnt); items per node = chunks * column groups ->
//           item_ptr; partial slots per request = sum over its path of chunks(node) + tail
//           chunks -> slot_ptr, and the first slot of every path entry
//   fill    per request: row of each of its path entries in the node's list (atomic cursor)
// The order in which requests land in a node's list depends on the atomics, the values do not:
// a column's result does not depend on which column it is.
#include "gf_internal.h"
#include "gf_decode_frag.h"

namespace gf {

constexpr int kSharedThreads = 256;
constexpr int kSharedWaves = kSharedThreads / 64;
constexpr int kScanThreads = 1024;

struct SharedPlan {
    // graph and batch (device, caller's)
    const int32_t *node_len, *node_block_ptr, *node_blocks, *path_ptr, *path_nodes;
    int32_t num_nodes, num_entries;
    // scratch (device, context's)
    int32_t *cnt, *cursor, *node_ptr, *item_ptr, *entry_req, *entry_slot, *inv_entry, *slot_ptr, *totals;
    int32_t chunk_blocks, item_cap, slot_cap;
};

__device__ __forceinline__ bool request_ok(const AttnArgs &a, int r) { return !(a.status && a.status[r] != 0); }

// path entries of request r, kept inside the entry arrays whatever path_ptr holds
__device__ __forceinline__ int path_lo(const SharedPlan &p, int r) { return max(p.path_ptr[r], 0); }
__device__ __forceinline__ int path_hi(const SharedPlan &p, int r) { return min(p.path_ptr[r + 1], p.num_entries); }

// blocks of node v that hold tokens (0 for an id outside the graph), and the chunks they are cut into
__device__ __forceinline__ int node_blocks_of(const SharedPlan &p, int v) {
    if (v < 0 || v >= p.num_nodes) return 0;
    const int own = p.node_block_ptr[v + 1] - p.node_block_ptr[v];
    const int need = (max(p.node_len[v], 0) + kBlock - 1) / kBlock;
    return max(min(own, need), 0);
}
__device__ __forceinline__ int node_chunks_of(const SharedPlan &p, int v) {
    return (node_blocks_of(p, v) + p.chunk_blocks - 1) / p.chunk_blocks;
}
// table entries of request r that hold its new tokens (the last ones of its table)
__device__ __forceinline__ int tail_blocks_of(const AttnArgs &a, int r) {
    const int n = max(a.seq_lens[r] - a.ctx_lens[r], 0);
    return min((n + kBlock - 1) / kBlock, max(min(a.num_blocks[r], a.max_blocks), 0));
}

__global__ void shared_zero_kernel(SharedPlan p) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < p.num_nodes) {
        p.cnt[i] = 0;
        p.cursor[i] = 0;
    }
}

__global__ void shared_count_kernel(SharedPlan p, AttnArgs a) {
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= a.num_req) return;
    const bool ok = request_ok(a, r);
    for (int e = path_lo(p, r); e < path_hi(p, r); ++e) {
        p.entry_req[e] = r;
        const int v = p.path_nodes[e];
        if (ok && v >= 0 && v < p.num_nodes) atomicAdd(&p.cnt[v], 1);
    }
}

// exclusive scan of f(i), i in [0, n), by one workgroup; out[n] = total
template <class F>
__device__ void block_exscan(int n, F f, int32_t *out, int32_t *sh) {
    const int tid = threadIdx.x;
    int carry = 0;
    for (int base = 0; base < n; base += kScanThreads) {
        const int i = base + tid;
        const int x = i < n ? f(i) : 0;
        sh[tid] = x;
        __syncthreads();
        for (int o = 1; o < kScanThreads; o <<= 1) {
            const int y = tid >= o ? sh[tid - o] : 0;
            __syncthreads();
            sh[tid] += y;
            __syncthreads();
        }
        if (i < n) out[i] = carry + sh[tid] - x;
        carry += sh[kScanThreads - 1];
        __syncthreads();
    }
    if (tid == 0) out[n] = carry;
    __syncthreads();
}

__global__ __launch_bounds__(kScanThreads) void shared_scan_kernel(SharedPlan p, AttnArgs a, int group) {
    __shared__ int32_t sh[kScanThreads];
    auto chunks_of = [&](int v) -> int { return node_chunks_of(p, v); };
    block_exscan(p.num_nodes, [&](int v) { return p.cnt[v]; }, p.node_ptr, sh);
    block_exscan(p.num_nodes, [&](int v) { return chunks_of(v) * ((p.cnt[v] * group + 15) / 16); }, p.item_ptr, sh);
    // partial slots per request: its path nodes' chunks, then the chunks of its tail
    auto tail_chunks = [&](int r) -> int { return (tail_blocks_of(a, r) + p.chunk_blocks - 1) / p.chunk_blocks; };
    block_exscan(a.num_req, [&](int r) {
        if (!request_ok(a, r)) return 0;
        int s = tail_chunks(r);
        for (int e = path_lo(p, r); e < path_hi(p, r); ++e) s += chunks_of(p.path_nodes[e]);
        return s;
    }, p.slot_ptr, sh);
    for (int r = threadIdx.x; r < a.num_req; r += kScanThreads) {
        if (!request_ok(a, r)) continue;
        int s = p.slot_ptr[r];
        for (int e = path_lo(p, r); e < path_hi(p, r); ++e) {
            p.entry_slot[e] = s;
            s += chunks_of(p.path_nodes[e]);
        }
    }
    if (threadIdx.x == 0) p.totals[0] = min(p.item_ptr[p.num_nodes], p.item_cap);
}

__global__ void shared_fill_kernel(SharedPlan p, AttnArgs a) {
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= a.num_req || !request_ok(a, r)) return;
    for (int e = path_lo(p, r); e < path_hi(p, r); ++e) {
        const int v = p.path_nodes[e];
        if (v < 0 || v >= p.num_nodes) continue;
        const int pos = atomicAdd(&p.cursor[v], 1);
        if (p.node_ptr[v] + pos < p.num_entries) p.inv_entry[p.node_ptr[v] + pos] = e;   // always, unless paths overlap
    }
}

// One (segment, kv head, chunk, 16 columns) reduction.  Column n of the wave is the pair
// (request col_req, query head kvh*G + col_head) or nothing (col_req < 0); its partial goes to
// slot col_slot.  `tab` lists the segment's blocks; token counts come from ntk or from seg_len.
template <int D, int G, bool FP8>
__device__ __forceinline__ void reduce_chunk(const AttnArgs &a, const int32_t *tab, const int32_t *ntk, int seg_len,
                                             int e0, int e1, int kvh, int lane, int col_req, int col_head,
                                             int col_slot, float *__restrict__ part_o, float *__restrict__ part_ml) {
    const int q4 = lane >> 4;
    bf16x8 qf[D / 32];
#pragma unroll
    for (int t = 0; t < D / 32; ++t) {
        const int d0 = FP8 ? 64 * (t / 2) + 16 * q4 + 8 * (t % 2) : 32 * t + 8 * q4;
        u32x4 raw = {0, 0, 0, 0};
        if (col_req >= 0)
            raw = *(const u32x4 *)((const char *)a.q + (((size_t)col_req * a.hq + kvh * G + col_head) * D + d0) * 2);
        qf[t] = __builtin_bit_cast(bf16x8, raw);
    }
    const float c = a.scale_log2;
    float m_run = -1.0e30f, l_run = 0.f;
    f32x4 oacc[D / 16];
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) oacc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    PairRegs<D, FP8> cur, nxt;
    load_pair(cur, a, tab, ntk, e0, e1, kvh, lane, seg_len);
    for (int e = e0; e < e1; e += 2) {
        const bool more = e + 2 < e1;
        if (more) load_pair(nxt, a, tab, ntk, e + 2, e1, kvh, lane, seg_len);
        f32x4 sT[2];
#pragma unroll
        for (int T = 0; T < 2; ++T) {
            sT[T] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < D / 32; ++t)
                sT[T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k_operand<D, FP8>(cur, T, t), qf[t], sT[T], 0, 0, 0);
            if constexpr (FP8) sT[T] *= cur.ks;
        }
        if (cur.n0 < kBlock || cur.n1 < kBlock) {
            const int lim = ((q4 >= 2) ? cur.n1 : cur.n0) - 8 * (q4 & 1);
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (4 * T + i >= lim) sT[T][i] = -INFINITY;
        }
        float mx = fmaxf(fmaxf(fmaxf(sT[0][0], sT[0][1]), fmaxf(sT[0][2], sT[0][3])),
                         fmaxf(fmaxf(sT[1][0], sT[1][1]), fmaxf(sT[1][2], sT[1][3])));
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = fast_exp2((m_run - m_new) * c);
        const float mc = m_new * c;
        m_run = m_new;
        f32x8 p;
        float psum = 0.f;
#pragma unroll
        for (int T = 0; T < 2; ++T)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float e2 = fast_exp2(sT[T][i] * c - mc);
                p[4 * T + i] = e2;
                psum += e2;
            }
        l_run = l_run * alpha + psum;
        if constexpr (FP8) p *= cur.vs;
        const bf16x8 pb = __builtin_convertvector(p, bf16x8);
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) {
            oacc[dt] *= alpha;
            oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(v_operand<D, FP8>(cur, dt), pb, oacc[dt], 0, 0, 0);
        }
        if (more) cur = nxt;
    }
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);
    if (col_req >= 0) {
        const size_t pi = (size_t)col_slot * a.hq + kvh * G + col_head;
        if (q4 == 0) {
            part_ml[pi * 2 + 0] = m_run * c;   // max in log2 units
            part_ml[pi * 2 + 1] = l_run;
        }
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) *(f32x4 *)(part_o + pi * D + 16 * dt + 4 * q4) = oacc[dt];
    }
}

// node-centric items: work id w -> (item, kv head); item -> (node, chunk, column group)
template <int D, int G, bool FP8>
__global__ __launch_bounds__(kSharedThreads) void shared_node_kernel(AttnArgs a, SharedPlan p, float *__restrict__ part_o,
                                                                      float *__restrict__ part_ml) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long w = (long)blockIdx.x * kSharedWaves + wave;
    const int item = (int)(w / a.hkv), kvh = (int)(w % a.hkv);
    if (item >= p.totals[0]) return;
    // node of the item: last v with item_ptr[v] <= item
    int lo = 0, hi = p.num_nodes;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (p.item_ptr[mid] <= item) lo = mid;
        else hi = mid;
    }
    const int v = lo;
    const int cnt = p.cnt[v];
    const int groups = (cnt * G + 15) / 16;
    if (groups <= 0) return;
    const int local = item - p.item_ptr[v];
    const int chunk = local / groups, cg = local % groups;      // column groups of a chunk run back to back
    const int seg_len = p.node_len[v];
    const int nblk = node_blocks_of(p, v);
    const int e0 = chunk * p.chunk_blocks, e1 = min(nblk, e0 + p.chunk_blocks);
    if (e0 >= e1) return;
    const int col = cg * 16 + (lane & 15);
    const int row = col / G;
    int col_req = -1, col_slot = 0;
    if (row < cnt && p.node_ptr[v] + row < p.num_entries) {
        const int e = p.inv_entry[p.node_ptr[v] + row];
        col_req = p.entry_req[e];
        col_slot = p.entry_slot[e] + chunk;
        if (col_slot >= p.slot_cap) col_req = -1;   // only with tables that break the resolve contract
    }
    reduce_chunk<D, G, FP8>(a, p.node_blocks + p.node_block_ptr[v], nullptr, seg_len, e0, e1, kvh, lane, col_req,
                            col % G, col_slot, part_o, part_ml);
}

// tails: one wave per (request, kv head, chunk of the request's tail entries), G columns in use
template <int D, int G, bool FP8>
__global__ __launch_bounds__(kSharedThreads) void shared_tail_kernel(AttnArgs a, SharedPlan p, int tail_splits,
                                                                      float *__restrict__ part_o,
                                                                      float *__restrict__ part_ml) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long w = (long)blockIdx.x * kSharedWaves + wave;
    const long pairs = (long)a.num_req * a.hkv;
    if (w >= pairs * tail_splits) return;
    const int s = (int)(w / pairs);
    const int rem = (int)(w % pairs);
    const int r = rem / a.hkv, kvh = rem % a.hkv;
    if (!request_ok(a, r)) return;
    const int nb = max(min(a.num_blocks[r], a.max_blocks), 0);
    const int ntail = tail_blocks_of(a, r);
    const int e0 = nb - ntail + s * p.chunk_blocks;
    const int e1 = min(nb, e0 + p.chunk_blocks);
    if (e0 >= e1) return;
    const int tail_chunks = (ntail + p.chunk_blocks - 1) / p.chunk_blocks;
    const int n16 = lane & 15;
    const int slot = p.slot_ptr[r + 1] - tail_chunks + s;
    reduce_chunk<D, G, FP8>(a, a.block_table + (size_t)r * a.max_blocks, a.block_ntok + (size_t)r * a.max_blocks, 0, e0,
                            e1, kvh, lane, (n16 < G && slot < p.slot_cap) ? r : -1, n16 % G, slot, part_o, part_ml);
}

// One wave per (request, query head): combine the request's partial slots.
template <int D>
__global__ __launch_bounds__(256) void shared_merge_kernel(AttnArgs a, SharedPlan p, const float *__restrict__ part_o,
                                                           const float *__restrict__ part_ml) {
    const int lane = threadIdx.x & 63;
    const long idx = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (idx >= (long)a.num_req * a.hq) return;
    const int r = (int)(idx / a.hq), h = (int)(idx % a.hq);
    const bool ok = request_ok(a, r);
    const int s0 = ok ? p.slot_ptr[r] : 0, s1 = ok ? min(p.slot_ptr[r + 1], p.slot_cap) : 0;
    __bf16 *out = (__bf16 *)a.o + ((size_t)r * a.hq + h) * D;
    constexpr int PER = D / 64;
    float acc[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) acc[i] = 0.f;
    float M = -INFINITY, L = 0.f;
    for (int s = s0; s < s1; ++s) M = fmaxf(M, part_ml[((size_t)s * a.hq + h) * 2]);
    for (int s = s0; s < s1; ++s) {
        const size_t pi = (size_t)s * a.hq + h;
        const float wgt = fast_exp2(part_ml[pi * 2] - M);
        L += wgt * part_ml[pi * 2 + 1];
#pragma unroll
        for (int i = 0; i < PER; ++i) acc[i] += wgt * part_o[pi * D + lane + 64 * i];
    }
    const float inv = s1 > s0 ? 1.f / L : 0.f;
#pragma unroll
    for (int i = 0; i < PER; ++i) out[lane + 64 * i] = (__bf16)(acc[i] * inv);
    if (a.lse && lane == 0)
        a.lse[(size_t)r * a.hq + h] = s1 > s0 ? (M + __builtin_log2f(L)) * 0.6931471805599453f : -INFINITY;
}

// ---- host side ---------------------------------------------------------------------------------
size_t shared_slot_cap(int32_t num_req, int32_t num_entries, int32_t max_blocks, int32_t chunk_blocks) {
    // per request: sum over its path of ceil(node blocks / chunk) + tail chunks <= blocks/chunk + entries + 1
    return (size_t)num_req * ((size_t)(max_blocks + chunk_blocks - 1) / chunk_blocks + 1) + (size_t)num_entries;
}

size_t shared_int_words(int32_t num_nodes, int32_t num_req, int32_t num_entries) {
    return 4 * ((size_t)num_nodes + 1) + 3 * ((size_t)num_entries + 1) + ((size_t)num_req + 2) + 8;
}

size_t shared_workspace_bytes(int32_t num_nodes, int32_t num_req, int32_t num_entries, int32_t max_blocks,
                              int32_t chunk_blocks, int32_t hq, int32_t head_dim) {
    const size_t slots = shared_slot_cap(num_req, num_entries, max_blocks, chunk_blocks);
    return shared_int_words(num_nodes, num_req, num_entries) * sizeof(int32_t) + 256 +
           slots * hq * ((size_t)head_dim + 2) * sizeof(float);
}

template <int D, int G>
static hipError_t launch_shared_t(const AttnArgs &a, int kv_dtype, SharedPlan p, int tail_splits, float *part_o,
                                  float *part_ml, hipStream_t s) {
    const unsigned nz = (unsigned)((p.num_nodes + 255) / 256), nr = (unsigned)((a.num_req + 255) / 256);
    hipLaunchKernelGGL(shared_zero_kernel, dim3(nz ? nz : 1), dim3(256), 0, s, p);
    hipLaunchKernelGGL(shared_count_kernel, dim3(nr), dim3(256), 0, s, p, a);
    hipLaunchKernelGGL(shared_scan_kernel, dim3(1), dim3(kScanThreads), 0, s, p, a, G);
    hipLaunchKernelGGL(shared_fill_kernel, dim3(nr), dim3(256), 0, s, p, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t node_waves = (size_t)p.item_cap * a.hkv;
    const size_t tail_waves = (size_t)a.num_req * a.hkv * tail_splits;
    const unsigned g_node = (unsigned)((node_waves + kSharedWaves - 1) / kSharedWaves);
    const unsigned g_tail = (unsigned)((tail_waves + kSharedWaves - 1) / kSharedWaves);
    if (kv_dtype == GF_FP8_E4M3) {
        if (g_node) hipLaunchKernelGGL((shared_node_kernel<D, G, true>), dim3(g_node), dim3(kSharedThreads), 0, s, a, p, part_o, part_ml);
        if (g_tail) hipLaunchKernelGGL((shared_tail_kernel<D, G, true>), dim3(g_tail), dim3(kSharedThreads), 0, s, a, p, tail_splits, part_o, part_ml);
    } else {
        if (g_node) hipLaunchKernelGGL((shared_node_kernel<D, G, false>), dim3(g_node), dim3(kSharedThreads), 0, s, a, p, part_o, part_ml);
        if (g_tail) hipLaunchKernelGGL((shared_tail_kernel<D, G, false>), dim3(g_tail), dim3(kSharedThreads), 0, s, a, p, tail_splits, part_o, part_ml);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t rows = (size_t)a.num_req * a.hq;
    hipLaunchKernelGGL((shared_merge_kernel<D>), dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, a, p, part_o, part_ml);
    return hipGetLastError();
}

hipError_t launch_decode_shared(const AttnArgs &a, int head_dim, int group, int kv_dtype, const gf_graph &g,
                                const int32_t *path_ptr, const int32_t *path_nodes, int32_t num_entries,
                                int32_t chunk_blocks, void *workspace, hipStream_t s) {
    if (a.num_req == 0) return hipSuccess;
    SharedPlan p;
    p.node_len = g.node_len;
    p.node_block_ptr = g.node_block_ptr;
    p.node_blocks = g.node_blocks;
    p.path_ptr = path_ptr;
    p.path_nodes = path_nodes;
    p.num_nodes = g.num_nodes;
    p.num_entries = num_entries;
    p.chunk_blocks = chunk_blocks;
    int32_t *w = (int32_t *)workspace;
    const size_t n1 = (size_t)g.num_nodes + 1, e1 = (size_t)num_entries + 1;
    p.cnt = w;            w += n1;
    p.cursor = w;         w += n1;
    p.node_ptr = w;       w += n1;
    p.item_ptr = w;       w += n1;
    p.entry_req = w;      w += e1;
    p.entry_slot = w;     w += e1;
    p.inv_entry = w;      w += e1;
    p.slot_ptr = w;       w += (size_t)a.num_req + 2;
    p.totals = w;         w += 8;
    const size_t slots = shared_slot_cap(a.num_req, num_entries, a.max_blocks, chunk_blocks);
    // node items: sum over (request, path entry) of chunks * column groups <= the slot bound (a column group
    // holds at least one request)
    if (slots > 0x7fffffffu / (size_t)(a.hkv > 0 ? a.hkv : 1)) return hipErrorInvalidValue;
    p.item_cap = (int32_t)slots;
    p.slot_cap = (int32_t)slots;
    float *part_o = (float *)(((uintptr_t)w + 255) & ~(uintptr_t)255);
    float *part_ml = part_o + slots * a.hq * (size_t)head_dim;
    // the host does not know how long the tails are: bound their chunks by the table width
    const int tail_splits = (a.max_blocks + chunk_blocks - 1) / chunk_blocks;
#define GF_CASE(DD, GG) \
    if (head_dim == DD && group == GG) return launch_shared_t<DD, GG>(a, kv_dtype, p, tail_splits, part_o, part_ml, s);
    GF_CASE(64, 1) GF_CASE(64, 2) GF_CASE(64, 4) GF_CASE(64, 8)
    GF_CASE(128, 1) GF_CASE(128, 2) GF_CASE(128, 4) GF_CASE(128, 8)
#undef GF_CASE
    return hipErrorNotSupported;
}

}  // namespace gf
