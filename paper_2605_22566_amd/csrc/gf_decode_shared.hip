// gf_attn_decode_shared: the decode step of gf_attn_decode, reading every shared node once per
// group of requests instead of once per request (paper, Topology-Aware State Management and the
// operation-level overlap it rests on: the KV of an operation node is shared by all workflows
// that pass through it -- here the sharing is used for the reads as well as for the storage).
//
// Node-centric order.  The batch's path lists are inverted on the device into node -> requests
// lists.  A score column is a (request through the node, query head of a kv head's group) pair;
// one workgroup reduces one item = (node, chunk of the node's blocks, kv head, up to 64 or 128
// columns): the chunk's K/V blocks are staged through LDS once and feed every column of the item
// (v_mfma_f32_16x16x32_bf16 with all 16 columns of a tile in use, where the request-centric kernel
// pads G heads to 16).  An item leaves one fp32 partial (reference max, sum, weighted values) per
// (request, path node, chunk).  The private tail blocks of a request (its new tokens) are items of
// their own with G columns, and one merge kernel combines a request's partials -- path nodes in
// order, then tail -- with the log-sum-exp rule.  The result is the request-centric one up to
// fp32 summation order.
//
// Integer preparation (all on the device, no host round trip; "node" below reads "list key" when residual
// handles are given, see the next paragraph):
//   count   per path entry: cnt[node] (atomics) and the entry's number of chunks
//   scan    one workgroup: node_ptr = scan(cnt); item_ptr = scan(chunks * column quads per node);
//           entry_slot = scan(chunks per path entry): the partial slots of a request's nodes are
//           contiguous, in path order; tail_ptr = scan(tail chunks per request), the tail slots
//           follow all node slots
//   fill    per path entry: its row in the node's list (atomic cursor) = (request, first slot);
//           per node and per request: the item records
// The order in which requests land in a node's list depends on the atomics, the values do not:
// a column's result does not depend on which column it is.
//
// Differential KV (paper, "Differential-based KV Cache", Eq. 7: the KV of a node under a prefix is its base KV
// plus that prefix's sparse residual).  With residual handles the lists are kept per KEY instead of per node: a
// request that reads node v with the residual whose first item is b0 is listed under key num_nodes + b0, one
// that reads v as stored under key v.  Requests that reach v through the same prefix carry the same residual
// and still share one read of it; the workgroup that stages a block adds the residual rows into the LDS
// image -- fp32 sum rounded to bf16, as gf_kv_apply_residual does -- before the barrier that publishes it.
#include "gf_internal.h"
#include "gf_residual_row.h"

namespace gf {

constexpr int kSharedThreads = 256;
constexpr int kScanThreads = 1024;
constexpr int kXcds = 8;                 // workgroups are dealt to the XCDs round robin
constexpr int kMaxChunk = 64;            // table entries per item: one per lane of a wave

struct SharedPlan {
    // graph and batch (device, caller's)
    const int32_t *node_len, *node_block_ptr, *node_blocks, *path_ptr, *path_nodes;
    int32_t num_nodes, num_entries;
    // residual handles of the table entries ([num_req][max_blocks], or nullptr) and the number of residual items;
    // num_keys = num_nodes + num_items lists are kept (see the file header)
    const int32_t *res_handle;
    int32_t num_items, num_keys;
    // scratch (device, context's); cnt, cursor, node_ptr, item_ptr are per key
    int32_t *cnt, *cursor, *node_ptr, *item_ptr, *entry_slot, *row_req, *row_slot, *tail_ptr, *totals;
    int32_t *key_node;    // [num_items]: the node whose list key num_nodes + b is, -1 while unused
    int32_t *entry_key;   // [num_entries]: list key of a path entry, -1 if the entry does not take part
    int4 *item_rec;   // three per item, see ItemRec
    int32_t *perm;    // launch order of the items: node items by falling length, then the tail items
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

// node a list key stands for (-1 for a residual key nothing uses)
__device__ __forceinline__ int key_base(const SharedPlan &p, int key) {
    return key < p.num_nodes ? key : p.key_node[key - p.num_nodes];
}

__global__ void shared_zero_kernel(SharedPlan p) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < p.num_keys) {
        p.cnt[i] = 0;
        p.cursor[i] = 0;
    }
    if (i < p.num_items) p.key_node[i] = -1;
}

// request that owns path entry e: the last r with path_ptr[r] <= e (-1 if none does)
__device__ __forceinline__ int request_of_entry(const SharedPlan &p, const AttnArgs &a, int e) {
    int lo = 0, hi = a.num_req;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (p.path_ptr[mid] <= e) lo = mid;
        else hi = mid;
    }
    return (e >= p.path_ptr[lo] && e < p.path_ptr[lo + 1]) ? lo : -1;
}

// one thread per path entry: count it for its node, note its chunks (0 for an entry that does not take part)
__global__ void shared_count_kernel(SharedPlan p, AttnArgs a) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= p.num_entries) return;
    const int r = request_of_entry(p, a, e);
    const int v = p.path_nodes[e];
    int chunks = 0, key = -1;
    if (r >= 0 && request_ok(a, r) && v >= 0 && v < p.num_nodes) {
        key = v;
        const int nblk = node_blocks_of(p, v);
        if (p.res_handle && nblk > 0) {
            // the node's first table entry: the blocks of the path entries before it (the order gf_resolve_path
            // writes).  Its handle b0 names the residual of the whole node: block j of the node reads item b0 + j.
            int pos = 0;
            for (int x = path_lo(p, r); x < e; ++x) pos += node_blocks_of(p, p.path_nodes[x]);
            if (pos + nblk <= a.max_blocks) {
                const int b0 = p.res_handle[(size_t)r * a.max_blocks + pos];
                if (b0 >= 0 && b0 <= p.num_items - nblk) {
                    // a residual belongs to one node; a second node that claims the same items is read as stored
                    const int old = atomicCAS(&p.key_node[b0], -1, v);
                    if (old == -1 || old == v) key = p.num_nodes + b0;
                }
            }
        }
        atomicAdd(&p.cnt[key], 1);
        chunks = node_chunks_of(p, v);
    }
    p.entry_key[e] = key;
    p.row_slot[e] = chunks;            // scratch until the fill kernel writes the rows
}

// exclusive scan of f(i), i in [0, n), by one workgroup; out[n] = total.  Every wave takes a contiguous run of
// whole 64-element tiles, lane l reading element l of a tile (consecutive lanes read consecutive words: a large
// range -- the key space of a call with residuals -- would otherwise cost one cache line per element): a first
// walk sums the run, the run totals give every wave its offset, a second walk scans tile by tile with a carry.
// Four tiles are fetched before the first is used (out may alias what f reads, so the compiler cannot batch
// the loads by itself).
template <class F>
__device__ void block_exscan(int n, F f, int32_t *out, int32_t *sh) {
    constexpr int kWaves = kScanThreads / 64, kBatch = 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seg = ((n + kWaves - 1) / kWaves + 63) & ~63;
    const int w0 = min(wave * seg, n), w1 = min(w0 + seg, n);
    int sum = 0;
    for (int t0 = w0; t0 < w1; t0 += 64 * kBatch) {
        int v[kBatch];
#pragma unroll
        for (int j = 0; j < kBatch; ++j) v[j] = t0 + 64 * j + lane < w1 ? f(t0 + 64 * j + lane) : 0;
#pragma unroll
        for (int j = 0; j < kBatch; ++j) sum += v[j];
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) sum += __shfl_xor(sum, o, 64);
    if (lane == 0) sh[wave] = sum;
    __syncthreads();
    int carry = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const int x = sh[w];
        carry += w < wave ? x : 0;
        total += x;
    }
    for (int t0 = w0; t0 < w1; t0 += 64 * kBatch) {
        int v[kBatch];
#pragma unroll
        for (int j = 0; j < kBatch; ++j) v[j] = t0 + 64 * j + lane < w1 ? f(t0 + 64 * j + lane) : 0;
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            int incl = v[j];
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int y = __shfl_up(incl, o, 64);
                if (lane >= o) incl += y;
            }
            if (t0 + 64 * j + lane < w1) out[t0 + 64 * j + lane] = carry + incl - v[j];
            carry += __shfl(incl, 63, 64);
        }
    }
    __syncthreads();
    if (tid == 0) out[n] = total;
    __syncthreads();
}

__global__ __launch_bounds__(kScanThreads) void shared_scan_kernel(SharedPlan p, AttnArgs a, int group, int item_cols) {
    __shared__ int32_t sh[kScanThreads];
    block_exscan(p.num_keys, [&](int k) { return p.cnt[k]; }, p.node_ptr, sh);
    block_exscan(p.num_keys, [&](int k) {
        const int n = p.cnt[k];
        return n > 0 ? node_chunks_of(p, key_base(p, k)) * ((n * group + item_cols - 1) / item_cols) : 0;
    }, p.item_ptr, sh);
    block_exscan(p.num_entries, [&](int e) { return p.row_slot[e]; }, p.entry_slot, sh);
    block_exscan(a.num_req, [&](int r) {
        return request_ok(a, r) ? (tail_blocks_of(a, r) + p.chunk_blocks - 1) / p.chunk_blocks : 0;
    }, p.tail_ptr, sh);
    if (threadIdx.x == 0) {
        p.totals[0] = min(p.item_ptr[p.num_keys], p.item_cap);                   // node items
        p.totals[1] = min(p.tail_ptr[a.num_req], p.item_cap - p.totals[0]);       // tail items
        p.totals[2] = min(p.entry_slot[p.num_entries], p.slot_cap);              // node slots; tail slots follow
    }
}

// What the attention kernel needs to know of an item, written once by the fill kernel (8 ints):
struct ItemRec {
    int32_t seg;        // node id, or -(request + 1) for a tail item
    int32_t tab_off;    // first table entry of the chunk: index into node_blocks (node) or block_table (tail)
    int32_t entries;    // table entries of the chunk (1 .. 64)
    int32_t tokens;     // tokens in those entries (all blocks full but possibly the last)
    int32_t row0;       // node: first row of the node's request list
    int32_t cnt;        // node: requests in that list
    int32_t quad;       // node: which group of 64 * col_groups columns
    int32_t slot;       // node: chunk index, added to a row's first slot; tail: the partial slot itself
    int32_t res0;       // residual item of the chunk's first block (block j reads item res0 + j), or -1
    int32_t pad[3];
};
constexpr int kRecWords = 3;
static_assert(sizeof(ItemRec) == kRecWords * sizeof(int4), "item record = three 16-byte words");

__device__ __forceinline__ void store_rec(const SharedPlan &p, int item, const ItemRec &r) {
    p.item_rec[kRecWords * (size_t)item] = make_int4(r.seg, r.tab_off, r.entries, r.tokens);
    p.item_rec[kRecWords * (size_t)item + 1] = make_int4(r.row0, r.cnt, r.quad, r.slot);
    p.item_rec[kRecWords * (size_t)item + 2] = make_int4(r.res0, 0, 0, 0);
}

// Threads [0, E): the rows of the lists (request and first partial slot of every path entry).
// Threads [E, E + K): a key's item records.  Threads [E + K, E + K + R): a request's tail item records.
__global__ void shared_fill_kernel(SharedPlan p, AttnArgs a, int group, int item_cols) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < p.num_entries) {
        const int e = i;
        const int r = request_of_entry(p, a, e);
        const int key = p.entry_key[e];
        if (r < 0 || key < 0) return;
        const int row = p.node_ptr[key] + atomicAdd(&p.cursor[key], 1);
        if (row < p.num_entries) {                             // always, unless paths overlap
            p.row_req[row] = r;
            p.row_slot[row] = p.entry_slot[e];
        }
        return;
    }
    i -= p.num_entries;
    if (i < p.num_keys) {
        const int key = i, base = p.item_ptr[key], n = p.item_ptr[key + 1] - base;
        if (n <= 0) return;
        const int v = key_base(p, key);
        if (v < 0 || v >= p.num_nodes) return;
        const int cnt = p.cnt[key], nblk = node_blocks_of(p, v);
        const int quads = max((cnt * group + item_cols - 1) / item_cols, 1);
        for (int j = 0; j < n && base + j < p.totals[0]; ++j) {
            const int chunk = j / quads, e0 = chunk * p.chunk_blocks, e1 = min(nblk, e0 + p.chunk_blocks);
            ItemRec rec;
            rec.seg = v;
            rec.tab_off = p.node_block_ptr[v] + e0;
            rec.entries = max(e1 - e0, 0);
            rec.tokens = max(min(p.node_len[v] - kBlock * e0, kBlock * (e1 - e0)), 0);
            rec.row0 = p.node_ptr[key];
            rec.cnt = cnt;
            rec.quad = j % quads;
            rec.slot = chunk;
            rec.res0 = key >= p.num_nodes ? key - p.num_nodes + e0 : -1;
            store_rec(p, base + j, rec);
        }
        return;
    }
    i -= p.num_keys;
    if (i < a.num_req) {
        const int r = i, base = p.totals[0] + p.tail_ptr[r], n = p.tail_ptr[r + 1] - p.tail_ptr[r];
        if (n <= 0) return;
        const int nb = max(min(a.num_blocks[r], a.max_blocks), 0), ntail = tail_blocks_of(a, r);
        const int n_new = max(a.seq_lens[r] - a.ctx_lens[r], 0);
        for (int j = 0; j < n && base + j < p.totals[0] + p.totals[1]; ++j) {
            const int e0 = nb - ntail + j * p.chunk_blocks, e1 = min(nb, e0 + p.chunk_blocks);
            ItemRec rec;
            rec.seg = -(r + 1);
            rec.tab_off = r * a.max_blocks + e0;
            rec.entries = max(e1 - e0, 0);
            rec.tokens = max(min(n_new - kBlock * j * p.chunk_blocks, kBlock * (e1 - e0)), 0);
            rec.row0 = 0;
            rec.cnt = 0;
            rec.quad = 0;
            rec.slot = p.totals[2] + p.tail_ptr[r] + j;
            rec.res0 = -1;
            store_rec(p, base + j, rec);
        }
    }
}

// Launch order of the items (one workgroup).  Items differ in length by a factor of 32 and a resident workgroup
// only gets a handful of them, so the order decides how evenly the work spreads: node items are sorted by
// falling number of table entries (counting sort, 64 classes; the order inside a class depends on the atomics,
// the results do not), the tail items (one or two steps each) follow.  The attention kernel deals the list
// out round by round, every other round backwards, so that a workgroup that drew a long item in one round
// draws a short one in the next (measured with in-kernel timers on config 3: in node order the workgroups
// finished between 133 and 244 us).
__global__ __launch_bounds__(kScanThreads) void shared_order_kernel(SharedPlan p) {
    __shared__ int hist[kMaxChunk + 2], start[kMaxChunk + 2];
    const int tid = threadIdx.x;
    const int n_node = p.totals[0], n_tail = p.totals[1];
    for (int i = tid; i < kMaxChunk + 2; i += kScanThreads) hist[i] = 0;
    __syncthreads();
    auto klass = [&](int i) -> int { return min(max(p.item_rec[kRecWords * (size_t)i].z, 0), kMaxChunk); };
    for (int i = tid; i < n_node; i += kScanThreads) atomicAdd(&hist[klass(i)], 1);
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int c = kMaxChunk; c >= 0; --c) {
            start[c] = run;
            run += hist[c];
        }
    }
    __syncthreads();
    for (int i = tid; i < kMaxChunk + 2; i += kScanThreads) hist[i] = 0;
    __syncthreads();
    for (int i = tid; i < n_node; i += kScanThreads) {
        const int c = klass(i);
        p.perm[start[c] + atomicAdd(&hist[c], 1)] = i;
    }
    for (int i = tid; i < n_tail; i += kScanThreads) p.perm[n_node + i] = n_node + i;
}

// ---- the attention kernel -------------------------------------------------------------------------
// One workgroup (4 waves) reduces one item: a chunk of one segment's blocks for one kv head and up to
// 64 * col_groups(G) score columns.  The chunk's K/V blocks go HBM -> LDS once per workgroup through direct
// loads, two blocks (32 keys) per step, into a ring of step buffers that keeps the next steps in flight;
// every wave reads its MFMA operand fragments from LDS and applies them to its groups of 16 columns, so a
// block read from HBM once serves up to 128 (request, head) columns.  Items are node items (columns = the
// requests through the node; 16 columns = 16/G requests) followed by tail items (a request's own tail
// blocks, G columns).  The grid is as large as fits on the device at once, and workgroups loop over the item
// list (in the launch order shared_order_kernel left) with the grid as stride, every other round backwards.
// groups of 16 columns per wave: two when a request brings 8 heads per kv head (its node lists are twice as
// wide in columns, and a fragment read from LDS then feeds two MFMAs), else one (more workgroups per CU)
constexpr int col_groups(int G) { return G >= 8 ? 2 : 1; }
// workgroups per CU the kernel is built for: registers and the LDS ring are sized to it
constexpr int wgs_per_cu(int G) { return col_groups(G) == 1 ? 4 : 3; }
constexpr int kLdsPerCu = 160 * 1024;

template <int D, bool FP8, int WGS>
struct StageCfg {
    static constexpr int kLdsPerWg = kLdsPerCu / WGS;           // LDS bytes one workgroup may take
    static constexpr int ES = FP8 ? 1 : 2;                      // bytes per pool element
    static constexpr int kRowB = D * ES;                        // K row
    static constexpr int kCPR = kRowB / 16;                     // 16-byte chunks per K row: 16, 8 or 4
    static constexpr int kBlkB = kBlock * D * ES;               // one (block, kv head) image of K or of V
    static constexpr int kLoads = kBlkB / 1024;                 // wave-wide direct loads per image
    static constexpr int kPair = 2 * kBlkB;                     // the K (or V) images of one step: two blocks
    // a ring of step buffers (K pair + V pair each): kRing - 1 steps are in flight per workgroup
    static constexpr int kRing = (kLdsPerWg / (2 * kPair)) < 9 ? (kLdsPerWg / (2 * kPair)) : 9;
    static constexpr int kVBase = kRing * kPair;                // K pairs first, then V pairs
    static constexpr int kLds = 2 * kRing * kPair;
    static_assert(kRing >= 2 && (kRing - 1) * kLoads < 64, "ring depth: two buffers at least, and wait counts that vmcnt can hold");
};

// Where a residual entry (logical element slot * D + d of a block) sits in a staged image of a bf16 pool (see the
// staging constants in the kernel): K keeps [slot][d] with the 16-byte pieces of a row at position
// piece ^ k_swz(block of the step, slot), V keeps [d][slot] with the two 8-slot halves of a row swapped on
// every other group of 8 rows.
template <int D, int TENSOR>
struct SharedStagedMap {
    static constexpr bool kPredicated = true;
    int blk;                                         // which of the step's two blocks (sets the K swizzle)
    __device__ __forceinline__ uint32_t operator()(uint32_t i) const {
        const uint32_t slot = i / D, d = i % D;
        uint32_t at;
        if constexpr (TENSOR == 0) {
            const uint32_t bits = (slot & 3) | (((slot >> 3) & 1) << 2) | ((uint32_t)blk << 3);
            const uint32_t sw = D == 128 ? bits : D == 64 ? bits >> 1 : bits >> 2;
            at = slot * D + (((d >> 3) ^ sw) << 3) + (d & 7);
        } else {
            at = d * kBlock + ((((slot >> 3) ^ (d >> 3)) & 1) << 3) + (slot & 7);
        }
        return i < (uint32_t)(kBlock * D) ? at : kNoElem;
    }
};

template <int D, int G, bool FP8, bool RES>
__global__ __launch_bounds__(kSharedThreads, wgs_per_cu(G)) void shared_attn_kernel(AttnArgs a, SharedPlan p, float *__restrict__ part_o,
                                                                      float *__restrict__ part_ml, ResidualRefs rr) {
    static_assert(!(RES && FP8), "residuals are read in place on bf16 pools only");
    constexpr int kColGroups = col_groups(G);
    using C = StageCfg<D, FP8, wgs_per_cu(G)>;
    __shared__ __attribute__((aligned(1024))) char lds[C::kLds];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n16 = lane & 15, q4 = lane >> 4;
    const long total_w = ((long)p.totals[0] + p.totals[1]) * a.hkv;
    // neighbours in the item list (same K/V blocks, other columns) run on the same XCD at the same time
    const int grid = gridDim.x;
    const int first = (grid % kXcds == 0) ? (int)(blockIdx.x % kXcds) * (grid / kXcds) + (int)(blockIdx.x / kXcds)
                                          : (int)blockIdx.x;
    const float c = a.scale_log2;
    const float slack = 8.f / c;                               // 2^8 in the exponent, in score units (inf for a zero scale)

    // ---- per-kernel constants of the staging and of the operand fetches ----
    // Wave w brings in one of the four images of a step: K of block w & 1 (w < 2) or V of block w & 1.
    // Lane l of load i fills LDS chunk q = 64 i + l of the image and picks its source so that the image is
    // XOR-swizzled: K row (q / CPR) holds chunk c at position c ^ k_swz(block, row); the two halves of a
    // bf16 V row swap on every other group of 8 rows.  Every 16-lane group of an operand fetch then hits
    // 16 different 16-byte bank groups.
    auto k_swz = [](int blk, int slot) -> int {
        const int bits = (slot & 3) | (((slot >> 3) & 1) << 2) | (blk << 3);     // the 16 rows a tile reads
        return C::kCPR == 16 ? bits : C::kCPR == 8 ? bits >> 1 : bits >> 2;
    };
    uint32_t src_off[C::kLoads];
#pragma unroll
    for (int i = 0; i < C::kLoads; ++i) {
        const int q = 64 * i + lane;
        if (wave < 2) {
            const int row = q / C::kCPR, pos = q % C::kCPR;
            src_off[i] = row * C::kRowB + ((pos ^ k_swz(wave & 1, row)) * 16);
        } else if constexpr (FP8) {
            src_off[i] = q * 16;
        } else {
            const int d = q >> 1;
            src_off[i] = d * 32 + (((q & 1) ^ ((d >> 3) & 1)) * 16);
        }
    }
    // operand fragments out of LDS (same geometry as the per-request kernel reads from HBM)
    const int k_slot = 8 * ((n16 >> 2) & 1) + (n16 & 3);
    const int k_row = (n16 >= 8 ? C::kBlkB : 0) + k_slot * C::kRowB;
    const int k_x = (q4 ^ k_swz(n16 >= 8 ? 1 : 0, k_slot)) * 16;                // chunk (4 t + q4) sits at k_x ^ 64 t
    const int v_frag = (q4 >= 2 ? C::kBlkB : 0) +
                       (FP8 ? n16 * 16 + (q4 & 1) * 8 : n16 * 32 + (((q4 & 1) ^ ((n16 >> 3) & 1)) * 16));

    // ---- items, two in flight: while item i is reduced, the per-lane data of item i + 1 is on its way ----
    // Per-lane data of an item.  The chunk's table entries (at most kMaxChunk = 64) live in lane registers,
    // lane j = entry j of the chunk: block id (clamped into the pool), token count and, for an e4m3 pool, the
    // block's two scales; the step loop reads them with v_readlane and touches memory only through the K/V
    // requests and LDS.  The columns of this wave: (request, query head, partial slot) per lane.
    struct LaneData {
        int blk, ntok;
        float ks, vs;
        int col_req[kColGroups], col_head[kColGroups], col_slot[kColGroups];
        int my_groups;                                         // groups of this wave that hold columns
    };
    // Work id w -> item record + kv head: position w / hkv of the launch order, kv head w % hkv.  The column
    // quads of a (node, chunk) have equal length, so they stay neighbours in the launch order and run on the
    // same XCD in the same round: the blocks they share come from HBM once.  In odd rounds the list is dealt
    // backwards (whole rounds only: the last, partial round keeps its direction).
    struct Item : ItemRec {
        int kvh;
    };
    auto load_rec = [&](long w) -> Item {
        Item r;
        r.seg = 0; r.tab_off = 0; r.entries = 0; r.tokens = 0; r.row0 = 0; r.cnt = 0; r.quad = 0; r.slot = 0; r.kvh = 0;
        r.res0 = -1;
        if (w < total_w) {
            const long round = w / grid, pos = w % grid;
            if ((round & 1) && (round + 1) * grid <= total_w) w = round * grid + (grid - 1 - pos);
            const long idx = min(max(p.perm[w / a.hkv], 0), p.totals[0] + p.totals[1] - 1);
            const int4 x = p.item_rec[kRecWords * idx], y = p.item_rec[kRecWords * idx + 1];
            r.seg = x.x; r.tab_off = x.y; r.entries = min(x.z, kMaxChunk); r.tokens = x.w;
            r.row0 = y.x; r.cnt = y.y; r.quad = y.z; r.slot = y.w;
            if constexpr (RES) {
                const int b0 = p.item_rec[kRecWords * idx + 2].x;
                r.res0 = (b0 >= 0 && b0 <= rr.num_items - r.entries) ? b0 : -1;
            }
            r.kvh = (int)(w % a.hkv);
        }
        return r;
    };
    auto load_lane = [&](const ItemRec &rec) -> LaneData {
        LaneData d;
        d.blk = 0;
        d.ks = d.vs = 1.f;
        d.ntok = min(max(rec.tokens - kBlock * lane, 0), kBlock);
        if (lane < rec.entries) {
            const int32_t *tab = rec.seg >= 0 ? p.node_blocks : a.block_table;
            d.blk = min(max(tab[(size_t)rec.tab_off + lane], 0), a.pool_blocks - 1);
            if constexpr (FP8) {
                d.ks = a.k_scale[d.blk];
                d.vs = a.v_scale[d.blk];
            }
        }
        const int groups = (rec.cnt * G + 15) / 16;
        d.my_groups = 0;
#pragma unroll
        for (int g = 0; g < kColGroups; ++g) {
            d.col_req[g] = -1;
            d.col_head[g] = n16 % G;
            d.col_slot[g] = 0;
            if (rec.seg >= 0) {
                const int cg = rec.quad * 4 * kColGroups + g * 4 + wave;   // groups dealt to the waves round robin
                if (cg < groups) d.my_groups = g + 1;
                const int col = cg * 16 + n16;
                const int row = col / G;
                d.col_head[g] = col % G;
                if (row < rec.cnt && rec.row0 + row < p.num_entries) {
                    d.col_req[g] = p.row_req[rec.row0 + row];
                    d.col_slot[g] = p.row_slot[rec.row0 + row] + rec.slot;
                }
            } else if (g == 0 && wave == 0) {
                d.my_groups = 1;
                if (n16 < G) {
                    d.col_req[g] = -rec.seg - 1;
                    d.col_slot[g] = rec.slot;
                }
            }
            if (d.col_slot[g] < 0 || d.col_slot[g] >= p.slot_cap) d.col_req[g] = -1;   // only with tables that break the resolve contract
        }
        return d;
    };

    Item rec = load_rec(first);
    LaneData cur = load_lane(rec);
    Item rec_next = load_rec((long)first + grid);
    for (long w = first; w < total_w; w += grid) {
        const int kvh = rec.kvh;
        const int entries = rec.entries;
        const int res0 = __builtin_amdgcn_readfirstlane(rec.res0);
        const int nsteps = (entries + 1) / 2;
        const int lane_blk = cur.blk, lane_ntok = cur.ntok;
        const float lane_ks = cur.ks, lane_vs = cur.vs;
        int col_req[kColGroups], col_head[kColGroups], col_slot[kColGroups];
#pragma unroll
        for (int g = 0; g < kColGroups; ++g) {
            col_req[g] = cur.col_req[g];
            col_head[g] = cur.col_head[g];
            col_slot[g] = cur.col_slot[g];
        }
        const int my_groups = __builtin_amdgcn_readfirstlane(cur.my_groups);

        // ---- staging: HBM -> LDS direct loads ----
        // wave w < 2 requests the K image of block w & 1 of a step, wave w >= 2 the V image; `slot` is the
        // buffer of the wave's own ring
        auto issue = [&](int step, int slot) {
            const int j = 2 * step + (wave & 1);
            const int b = __builtin_amdgcn_readlane(lane_blk, j < entries ? j : 2 * step);   // odd tail: block 0 again
            const uintptr_t addr = (uintptr_t)(wave < 2 ? a.k : a.v) + ((size_t)b * a.hkv + kvh) * C::kBlkB;
            // wave-uniform by construction; said explicitly so that the address lives in scalar registers
            const char *src = (const char *)(((uintptr_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(addr >> 32)) << 32) |
                                             (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)addr));
            char *dst = lds + (wave < 2 ? 0 : C::kVBase) + slot * C::kPair + (wave & 1) * C::kBlkB;
#pragma unroll
            for (int i = 0; i < C::kLoads; ++i) dma_load(src, src_off[i], dst + 1024 * i);
        };
        constexpr int my_ring = C::kRing;
#pragma unroll
        for (int j = 0; j < C::kRing - 1; ++j)
            if (j < nsteps && j < my_ring - 1) issue(j, j);
        // ---- Q^T operands of this wave's columns ----
        bf16x8 qf[kColGroups][D / 32];
#pragma unroll
        for (int g = 0; g < kColGroups; ++g)
#pragma unroll
            for (int t = 0; t < D / 32; ++t) {
                const int d0 = FP8 ? 64 * (t / 2) + 16 * q4 + 8 * (t % 2) : 32 * t + 8 * q4;
                u32x4 raw = {0, 0, 0, 0};
                if (col_req[g] >= 0)
                    raw = *(const u32x4 *)((const char *)a.q +
                                           (((size_t)col_req[g] * a.hq + kvh * G + col_head[g]) * D + d0) * 2);
                qf[g][t] = __builtin_bit_cast(bf16x8, raw);
            }
        float m_run[kColGroups], l_run[kColGroups];
        f32x4 oacc[kColGroups][D / 16];
#pragma unroll
        for (int g = 0; g < kColGroups; ++g) {
            m_run[g] = -1.0e30f;
            l_run[g] = 0.f;
#pragma unroll
            for (int dt = 0; dt < D / 16; ++dt) oacc[g][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }

        // Everything this item loaded through the compiler (table entries, Q) is waited for here, once: a wait
        // the compiler placed at the first use inside the loop would be a vmcnt(0) in every step and drain the ring.
        __builtin_amdgcn_s_waitcnt(0x0070);                    // vmcnt(0) lgkmcnt(0)
        int slot = 0;
        for (int step = 0; step < nsteps; ++step) {
            // this wave's image of `step` has landed when at most its younger requests are outstanding
            if (step + C::kRing - 2 < nsteps) dma_wait<(C::kRing - 2) * C::kLoads>();
            else dma_wait<0>();
            if constexpr (RES) {
                // the image this wave staged for `step` is still its own: add the block's residual row for this
                // kv head (K for waves 0 and 1, V for waves 2 and 3)
                const int j = 2 * step + (wave & 1);
                if (res0 >= 0 && j < entries) {
                    constexpr int kK = 0, kV = 1;
                    const int tensor = wave < 2 ? kK : kV;
                    const int32_t *rp = rr.ptr + ((size_t)(res0 + j) * 2 + tensor) * a.hkv + kvh;
                    const int e_first = __builtin_amdgcn_readfirstlane(rp[0]), e_end = __builtin_amdgcn_readfirstlane(rp[1]);
                    if (e_first < e_end) {
                        uint16_t *img = (uint16_t *)(lds + (wave < 2 ? 0 : C::kVBase) + slot * C::kPair + (wave & 1) * C::kBlkB);
                        RowLoad<D, 1> row;
                        row.issue(rr, e_first, e_end, lane);
                        if (wave < 2) row.apply(img, rr, lane, SharedStagedMap<D, kK>{wave & 1});
                        else row.apply(img, rr, lane, SharedStagedMap<D, kV>{wave & 1});
                    }
                }
            }
            __syncthreads();           // all four images of `step` are in LDS; everybody is done with step - 1
            if (step + my_ring - 1 < nsteps) {
                issue(step + my_ring - 1, slot == 0 ? my_ring - 1 : slot - 1);
            }
            const bool two = 2 * step + 1 < entries;
            const int n0 = __builtin_amdgcn_readlane(lane_ntok, 2 * step);
            const int n1 = two ? __builtin_amdgcn_readlane(lane_ntok, 2 * step + 1) : 0;
            float ks = 1.f, vs = 1.f;
            if constexpr (FP8) {
                const int jj = 2 * step + (q4 >= 2 && two ? 1 : 0);        // this lane's keys: block q4 / 2 of the step
                ks = __shfl(lane_ks, jj, 64);
                vs = __shfl(lane_vs, jj, 64);
            }
            const char *base = lds + slot * C::kPair;
            const char *vbase = lds + C::kVBase + slot * C::kPair;
            bf16x8 pb[kColGroups];
            if (my_groups > 0) {
                f32x4 sT[kColGroups][2];
#pragma unroll
                for (int T = 0; T < 2; ++T) {
#pragma unroll
                    for (int g = 0; g < kColGroups; ++g) sT[g][T] = f32x4{0.f, 0.f, 0.f, 0.f};
                    if constexpr (FP8) {
#pragma unroll
                        for (int tp = 0; tp < D / 64; ++tp) {
                            const u32x4 raw = *(const u32x4 *)(base + k_row + 4 * T * C::kRowB + (k_x ^ (64 * tp)));
                            const bf16x8 k0 = fp8x8_to_bf16x8(u32x2{raw[0], raw[1]});
                            const bf16x8 k1 = fp8x8_to_bf16x8(u32x2{raw[2], raw[3]});
#pragma unroll
                            for (int g = 0; g < kColGroups; ++g)
                                if (g < my_groups) {
                                    sT[g][T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0, qf[g][2 * tp], sT[g][T], 0, 0, 0);
                                    sT[g][T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1, qf[g][2 * tp + 1], sT[g][T], 0, 0, 0);
                                }
                        }
                    } else {
#pragma unroll
                        for (int t = 0; t < D / 32; ++t) {
                            const bf16x8 kf = __builtin_bit_cast(
                                bf16x8, *(const u32x4 *)(base + k_row + 4 * T * C::kRowB + (k_x ^ (64 * t))));
#pragma unroll
                            for (int g = 0; g < kColGroups; ++g)
                                if (g < my_groups)
                                    sT[g][T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[g][t], sT[g][T], 0, 0, 0);
                        }
                    }
                }
#pragma unroll
                for (int g = 0; g < kColGroups; ++g) {
                    pb[g] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
                    if (g < my_groups) {
                        if constexpr (FP8) { sT[g][0] *= ks; sT[g][1] *= ks; }
                        if (n0 < kBlock || n1 < kBlock) {
                            const int lim = ((q4 >= 2) ? n1 : n0) - 8 * (q4 & 1);
#pragma unroll
                            for (int T = 0; T < 2; ++T)
#pragma unroll
                                for (int i = 0; i < 4; ++i)
                                    if (4 * T + i >= lim) sT[g][T][i] = -INFINITY;
                        }
                        float mx = fmaxf(fmaxf(fmaxf(sT[g][0][0], sT[g][0][1]), fmaxf(sT[g][0][2], sT[g][0][3])),
                                         fmaxf(fmaxf(sT[g][1][0], sT[g][1][1]), fmaxf(sT[g][1][2], sT[g][1][3])));
                        // m_run is the reference the exponentials are taken against, the same in the four lanes
                        // of a column, not the exact running maximum: it is only moved (and sums and values
                        // rescaled) when some score outgrows it by more than 2^8 in the exponent, which keeps
                        // everything well inside fp32 and bf16 range.  Most steps therefore need neither the
                        // cross-lane maximum nor the rescaling multiplies.
                        if (__builtin_amdgcn_ballot_w64(mx > m_run[g] + slack) != 0) {
                            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
                            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
                            const float m_new = fmaxf(m_run[g], mx);
                            const float al = fast_exp2((m_run[g] - m_new) * c);
                            m_run[g] = m_new;
                            l_run[g] *= al;
#pragma unroll
                            for (int dt = 0; dt < D / 16; ++dt) oacc[g][dt] *= al;
                        }
                        const float mc = m_run[g] * c;
                        f32x8 pr;
                        float psum = 0.f;
#pragma unroll
                        for (int T = 0; T < 2; ++T)
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const float e2 = fast_exp2(sT[g][T][i] * c - mc);
                                pr[4 * T + i] = e2;
                                psum += e2;
                            }
                        l_run[g] += psum;
                        if constexpr (FP8) pr *= vs;
                        pb[g] = __builtin_convertvector(pr, bf16x8);
                    }
                }
#pragma unroll
                for (int dt = 0; dt < D / 16; ++dt) {
                    bf16x8 vf;
                    if constexpr (FP8) vf = fp8x8_to_bf16x8(*(const u32x2 *)(vbase + v_frag + dt * 256));
                    else vf = __builtin_bit_cast(bf16x8, *(const u32x4 *)(vbase + v_frag + dt * 512));
#pragma unroll
                    for (int g = 0; g < kColGroups; ++g)
                        if (g < my_groups) {
                            oacc[g][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pb[g], oacc[g][dt], 0, 0, 0);
                        }
                }
            }
            slot = slot + 1 == C::kRing ? 0 : slot + 1;
        }
        __syncthreads();               // the ring is free again before the next item writes into it

        // the next item's per-lane data is requested now, ahead of this item's stores (which use the copies
        // taken above), straight into the registers the next round reads; its successor's record follows
        cur = load_lane(rec_next);
        const Item rec_after = load_rec(w + 2 * (long)grid);

        // ---- partials of this wave's columns ----
#pragma unroll
        for (int g = 0; g < kColGroups; ++g) {
            float l = l_run[g];
            l += __shfl_xor(l, 16, 64);
            l += __shfl_xor(l, 32, 64);
            if (g < my_groups && col_req[g] >= 0 && nsteps > 0) {
                const size_t pi = (size_t)col_slot[g] * a.hq + kvh * G + col_head[g];
                if (q4 == 0) {
                    part_ml[pi * 2 + 0] = m_run[g] * c;   // max in log2 units
                    part_ml[pi * 2 + 1] = l;
                }
#pragma unroll
                for (int dt = 0; dt < D / 16; ++dt) *(f32x4 *)(part_o + pi * D + 16 * dt + 4 * q4) = oacc[g][dt];
            }
        }
        rec = rec_next;
        rec_next = rec_after;
    }
}

// One wave per (request, query head): combine the request's partial slots -- those of its path entries, which
// are contiguous and in path order, then those of its tail.  The maxima are in log2 units: w_s = 2^(m_s - M),
// L = sum w_s l_s, O = sum w_s O_s / L, lse = (M + log2 L) ln 2.  Lanes first work slot-parallel (maximum,
// weights), then each lane owns D/64 output elements and the weights go round by v_readlane.
template <int D>
__global__ __launch_bounds__(256) void shared_merge_kernel(AttnArgs a, SharedPlan p, const float *__restrict__ part_o,
                                                           const float *__restrict__ part_ml) {
    const int lane = threadIdx.x & 63;
    const long idx = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (idx >= (long)a.num_req * a.hq) return;
    const int r = (int)(idx / a.hq), h = (int)(idx % a.hq);
    int s0[2] = {0, 0}, n[2] = {0, 0};                           // the two slot ranges
    if (request_ok(a, r)) {
        const int lo = path_lo(p, r), hi = max(path_hi(p, r), lo);
        s0[0] = min(p.entry_slot[lo], p.slot_cap);
        n[0] = max(min(p.entry_slot[hi], p.slot_cap) - s0[0], 0);
        s0[1] = min(p.totals[2] + p.tail_ptr[r], p.slot_cap);
        n[1] = max(min(p.totals[2] + p.tail_ptr[r + 1], p.slot_cap) - s0[1], 0);
    }
    const int ns = n[0] + n[1];
    auto slot_of = [&](int i) -> int { return i < n[0] ? s0[0] + i : s0[1] + (i - n[0]); };
    __bf16 *out = (__bf16 *)a.o + ((size_t)r * a.hq + h) * D;
    constexpr int PER = D / 64;
    float acc[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) acc[i] = 0.f;
    float M = -INFINITY, L = 0.f;
    for (int base = 0; base < ns; base += 64)
        if (base + lane < ns) M = fmaxf(M, part_ml[((size_t)slot_of(base + lane) * a.hq + h) * 2]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off, 64));
    for (int base = 0; base < ns; base += 64) {
        float wgt = 0.f;
        int slot = 0;
        if (base + lane < ns) {
            slot = slot_of(base + lane);
            const size_t pi = (size_t)slot * a.hq + h;
            wgt = fast_exp2(part_ml[pi * 2] - M);
            L += wgt * part_ml[pi * 2 + 1];
        }
        const int m = min(64, ns - base);
        for (int j0 = 0; j0 < m; j0 += 4) {                     // four slots' loads in flight together
            float x[4][PER];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = min(j0 + u, m - 1);
                const size_t pj = (size_t)__builtin_amdgcn_readlane(slot, j) * a.hq + h;
#pragma unroll
                for (int i = 0; i < PER; ++i) x[u][i] = part_o[pj * D + lane + 64 * i];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float wj = j0 + u < m ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(wgt), min(j0 + u, m - 1))) : 0.f;
#pragma unroll
                for (int i = 0; i < PER; ++i) acc[i] += wj * x[u][i];
            }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) L += __shfl_xor(L, off, 64);
    // no visible token at all (no chunk, or only entries without tokens): zero row, lse -inf
    const float inv = L > 0.f ? 1.f / L : 0.f;
#pragma unroll
    for (int i = 0; i < PER; ++i) out[lane + 64 * i] = (__bf16)(acc[i] * inv);
    if (a.lse && lane == 0)
        a.lse[(size_t)r * a.hq + h] = L > 0.f ? (M + __builtin_log2f(L)) * 0.6931471805599453f : -INFINITY;
}

// ---- host side ---------------------------------------------------------------------------------
size_t shared_slot_cap(int32_t num_req, int32_t num_entries, int32_t max_blocks, int32_t chunk_blocks) {
    // per request: sum over its path of ceil(node blocks / chunk) + tail chunks <= blocks/chunk + entries + 1
    return (size_t)num_req * ((size_t)(max_blocks + chunk_blocks - 1) / chunk_blocks + 1) + (size_t)num_entries;
}

size_t shared_int_words(int32_t num_keys, int32_t num_items, int32_t num_req, int32_t num_entries) {
    return 4 * ((size_t)num_keys + 1) + 4 * ((size_t)num_entries + 1) + (size_t)num_items + ((size_t)num_req + 2) + 8;
}
// + one item record per partial slot (items <= slots: a node item serves at least one request)

size_t shared_workspace_bytes(int32_t num_nodes, int32_t num_items, int32_t num_req, int32_t num_entries,
                              int32_t max_blocks, int32_t chunk_blocks, int32_t hq, int32_t head_dim) {
    const size_t slots = shared_slot_cap(num_req, num_entries, max_blocks, chunk_blocks);
    return shared_int_words(num_nodes + num_items, num_items, num_req, num_entries) * sizeof(int32_t) + 16 +
           slots * sizeof(ItemRec) + slots * sizeof(int32_t) + 256 + slots * hq * ((size_t)head_dim + 2) * sizeof(float);
}

// resident workgroups of the attention kernel on the whole device (the item loop strides by the grid, so
// every workgroup of the grid has to be resident from the start), a multiple of the XCD count
template <class K>
static int resident_grid(K kernel) {
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kSharedThreads, 0) != hipSuccess) return 0;
    const int g = cus * per_cu;
    return g >= kXcds ? g / kXcds * kXcds : g;
}

template <int D, int G, bool FP8, bool RES>
static hipError_t launch_attn(const AttnArgs &a, SharedPlan p, float *part_o, float *part_ml, const ResidualRefs &rr,
                              hipStream_t s) {
    static int grid = resident_grid(shared_attn_kernel<D, G, FP8, RES>);  // one device per process
    if (grid <= 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL((shared_attn_kernel<D, G, FP8, RES>), dim3(grid), dim3(kSharedThreads), 0, s, a, p, part_o,
                       part_ml, rr);
    return hipGetLastError();
}

template <int D, int G>
static hipError_t launch_shared_t(const AttnArgs &a, int kv_dtype, SharedPlan p, float *part_o, float *part_ml,
                                  int phases, const ResidualRefs *rr, hipStream_t s) {
    if (rr && kv_dtype == GF_FP8_E4M3) return hipErrorNotSupported;
    if (phases & kSharedBuildLists) {
        const unsigned nz = (unsigned)((p.num_keys + 255) / 256), ne = (unsigned)((p.num_entries + 255) / 256);
        hipLaunchKernelGGL(shared_zero_kernel, dim3(nz ? nz : 1), dim3(256), 0, s, p);
        if (ne) hipLaunchKernelGGL(shared_count_kernel, dim3(ne), dim3(256), 0, s, p, a);
        hipLaunchKernelGGL(shared_scan_kernel, dim3(1), dim3(kScanThreads), 0, s, p, a, G, 64 * col_groups(G));
        const unsigned nf = (unsigned)(((size_t)p.num_entries + p.num_keys + a.num_req + 255) / 256);
        hipLaunchKernelGGL(shared_fill_kernel, dim3(nf), dim3(256), 0, s, p, a, G, 64 * col_groups(G));
        hipLaunchKernelGGL(shared_order_kernel, dim3(1), dim3(kScanThreads), 0, s, p);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (phases & kSharedAttend) {
        const ResidualRefs none = {nullptr, nullptr, nullptr, nullptr, 0};
        const hipError_t e = kv_dtype == GF_FP8_E4M3 ? launch_attn<D, G, true, false>(a, p, part_o, part_ml, none, s)
                             : rr                    ? launch_attn<D, G, false, true>(a, p, part_o, part_ml, *rr, s)
                                                     : launch_attn<D, G, false, false>(a, p, part_o, part_ml, none, s);
        if (e != hipSuccess) return e;
        const size_t rows = (size_t)a.num_req * a.hq;
        hipLaunchKernelGGL((shared_merge_kernel<D>), dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, a, p, part_o,
                           part_ml);
    }
    return hipGetLastError();
}

hipError_t launch_decode_shared(const AttnArgs &a, int head_dim, int group, int kv_dtype, const gf_graph &g,
                                const int32_t *path_ptr, const int32_t *path_nodes, int32_t num_entries,
                                int32_t chunk_blocks, void *workspace, int phases, const ResidualRefs *rr,
                                hipStream_t s) {
    if (a.num_req == 0) return hipSuccess;
    SharedPlan p;
    p.res_handle = rr ? rr->handle : nullptr;
    p.num_items = rr ? rr->num_items : 0;
    if ((size_t)g.num_nodes + (size_t)p.num_items > 0x7ffffff0u) return hipErrorInvalidValue;
    p.num_keys = g.num_nodes + p.num_items;
    p.node_len = g.node_len;
    p.node_block_ptr = g.node_block_ptr;
    p.node_blocks = g.node_blocks;
    p.path_ptr = path_ptr;
    p.path_nodes = path_nodes;
    p.num_nodes = g.num_nodes;
    p.num_entries = num_entries;
    p.chunk_blocks = chunk_blocks < kMaxChunk ? chunk_blocks : kMaxChunk;
    int32_t *w = (int32_t *)workspace;
    const size_t n1 = (size_t)p.num_keys + 1, e1 = (size_t)num_entries + 1;
    p.cnt = w;            w += n1;
    p.cursor = w;         w += n1;
    p.node_ptr = w;       w += n1;
    p.item_ptr = w;       w += n1;
    p.entry_slot = w;     w += e1;
    p.row_req = w;        w += e1;
    p.row_slot = w;       w += e1;
    p.entry_key = w;      w += e1;
    p.key_node = w;       w += (size_t)p.num_items;
    p.tail_ptr = w;       w += (size_t)a.num_req + 2;
    p.totals = w;         w += 8;
    const size_t slots = shared_slot_cap(a.num_req, num_entries, a.max_blocks, chunk_blocks);
    // node items: sum over (request, path entry) of chunks * column groups <= the slot bound (a column group
    // holds at least one request)
    if (slots > 0x7fffffffu / (size_t)(a.hkv > 0 ? a.hkv : 1)) return hipErrorInvalidValue;
    if ((size_t)a.num_req * (size_t)a.max_blocks > 0x7fffffffu) return hipErrorInvalidValue;   // table offsets are int32
    p.item_cap = (int32_t)slots;
    p.slot_cap = (int32_t)slots;
    p.item_rec = (int4 *)(((uintptr_t)w + 15) & ~(uintptr_t)15);
    p.perm = (int32_t *)(p.item_rec + kRecWords * slots);
    float *part_o = (float *)(((uintptr_t)(p.perm + slots) + 255) & ~(uintptr_t)255);
    float *part_ml = part_o + slots * a.hq * (size_t)head_dim;
#define GF_CASE(DD, GG) \
    if (head_dim == DD && group == GG) return launch_shared_t<DD, GG>(a, kv_dtype, p, part_o, part_ml, phases, rr, s);
    GF_CASE(64, 1) GF_CASE(64, 2) GF_CASE(64, 4) GF_CASE(64, 8)
    GF_CASE(128, 1) GF_CASE(128, 2) GF_CASE(128, 4) GF_CASE(128, 8)
#undef GF_CASE
    return hipErrorNotSupported;
}

}  // namespace gf
