/*
 * graphflow.h -- C ABI of the MI355X (gfx950) graph-KV attention library.
 *
 * The operation (paper: "Topology-Aware State Management"): every operation
 * node of the wGraph (paper: "Overview", G_op = (V_op, E_op)) owns one
 * precomputed KV segment, stored ONCE in a paged block pool and shared by all
 * requests whose workflow passes through the node.  A request's context is the
 * prefix path P of nodes (paper: Eq. 7, taken with a zero residual), its KV is
 * assembled from those nodes' blocks through a per-request block table, and
 * new prefill tokens / decode steps attend to it without recomputing or
 * copying the shared part.
 *
 * Conventions
 *   - Every call returns int32: GF_OK (0) or a negative GF_ERR_* code.  No
 *     exception crosses the boundary.  gf_strerror() names a code.
 *   - All data pointers are DEVICE pointers owned by the caller, unless a
 *     parameter says "host".  The gf_graph / gf_attn_params / gf_kv_pool /
 *     gf_tables structs themselves are small HOST structs read during the call.
 *   - Calls are asynchronous on the caller's HIP stream (`stream`, a
 *     hipStream_t passed as void*; NULL = the default stream).  The only
 *     synchronisation inside is the one named below: a call whose context
 *     buffer must grow waits for the stream before it frees the old buffer.
 *     Data-dependent failures are reported per request
 *     in the device array status[] (GF_ST_*), not through the return value.
 *   - The library owns only a gf_ctx: device scratch memory (the split-KV
 *     partials of gf_attn_decode, the work list of gf_attn_prefill, the lists and
 *     partials of gf_attn_decode_shared / gf_decode_shared_plan; their
 *     residual-reading forms use the same buffers; gf_kv_make_residual keeps
 *     8 bytes per CSR row in the decode buffer between its passes), grown on
 *     demand -- these calls may therefore call hipMalloc, and hipFree after a
 *     stream synchronisation when it outgrows what it has (a buffer that grows
 *     again takes half as much more than it had, so a loop whose sizes creep up
 *     drains its stream a few times, not at every step) -- and released by
 *     gf_destroy.  A gf_ctx must not be used from two streams at once.  Once a
 *     call has run with given sizes, repeating it allocates nothing, so a sequence
 *     of calls can be recorded into a HIP graph after one warm-up pass.
 *   - Index arrays are int32.  Block size is 16 tokens.
 *
 * Pool layout (one layer), block size B = 16, element = bf16 or e4m3 byte:
 *     K[num_blocks][num_kv_heads][B][head_dim]      token-major inside a block
 *     V[num_blocks][num_kv_heads][head_dim][B]      head-dim-major inside a block
 *   Token t of a node lives in that node's block t/16, slot t%16.  Slots at or
 *   beyond a block's token count hold finite, unspecified values; NaN/Inf there
 *   is a contract violation.  With GF_FP8_E4M3 (OCP E4M3, finite-only, max 448)
 *   every block has one fp32 scale per tensor: value = decode(code) * scale[blk].
 *
 * Supported shapes: head_dim in {64,128}; block_size 16; num_q_heads a
 * multiple of num_kv_heads with group size in {1,2,4,8}.  Anything else
 * returns GF_ERR_UNSUPPORTED; there is no fallback path.
 */
#ifndef GRAPHFLOW_H
#define GRAPHFLOW_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* return codes */
#define GF_OK               0
#define GF_ERR_NULL        -1   /* a required pointer is NULL                   */
#define GF_ERR_BAD_SHAPE   -2   /* negative / inconsistent sizes                */
#define GF_ERR_UNSUPPORTED -3   /* shape or dtype outside the supported set     */
#define GF_ERR_WORKSPACE   -4   /* device workspace could not be (re)allocated  */
#define GF_ERR_HIP         -5   /* a HIP runtime call or kernel launch failed   */

/* per-request status words written by gf_resolve_path */
#define GF_ST_OK         0
#define GF_ST_BAD_NODE   1   /* a path entry is not a node id                        */
#define GF_ST_BAD_EDGE   2   /* consecutive path nodes are not joined by an edge     */
#define GF_ST_BAD_TAIL   3   /* fewer tail blocks than ceil(new_len/16), or new_len<0 */
#define GF_ST_BAD_BLOCK  4   /* a node owns too few blocks, or a block id is outside the pool */
#define GF_ST_OVERFLOW   5   /* the request needs more than max_blocks table entries */

/* kv_dtype */
#define GF_BF16     0
#define GF_FP8_E4M3 1

typedef struct gf_ctx gf_ctx;

/* wGraph as CSR arrays (device).  Node v owns the token segment of length
 * node_len[v] stored in blocks node_blocks[node_block_ptr[v] .. node_block_ptr[v+1]).
 * edge_dst[edge_ptr[v] .. edge_ptr[v+1]) are v's valid successors; edge_ptr and
 * edge_dst may both be NULL, which skips edge validation (one of them alone is
 * GF_ERR_NULL: a graph that validates edges and has none still hands over an
 * edge_dst address, which is never read). */
typedef struct {
    int32_t        num_nodes;
    const int32_t *node_len;        /* [num_nodes]     */
    const int32_t *node_block_ptr;  /* [num_nodes + 1] */
    const int32_t *node_blocks;     /* [node_block_ptr[num_nodes]] */
    const int32_t *edge_ptr;        /* [num_nodes + 1] or NULL */
    const int32_t *edge_dst;        /* [edge_ptr[num_nodes]] or NULL */
} gf_graph;

typedef struct {
    int32_t num_q_heads;
    int32_t num_kv_heads;
    int32_t head_dim;
    int32_t block_size;   /* must be 16 */
    int32_t kv_dtype;     /* GF_BF16 | GF_FP8_E4M3 */
    float   sm_scale;     /* softmax scale; 0 selects 1/sqrt(head_dim); must not be negative */
} gf_attn_params;

typedef struct {
    const void  *k;        /* K pool, layout above (device) */
    const void  *v;        /* V pool, layout above (device) */
    const float *k_scale;  /* [num_blocks] fp32, GF_FP8_E4M3 only, else NULL */
    const float *v_scale;  /* [num_blocks] fp32, GF_FP8_E4M3 only, else NULL */
    int32_t      num_blocks;
} gf_kv_pool;

/* The outputs of gf_resolve_path, handed to the attention calls (device). */
typedef struct {
    const int32_t *block_table;  /* [num_req][max_blocks], pad -1 */
    const int32_t *block_ntok;   /* [num_req][max_blocks], pad 0  */
    const int32_t *num_blocks;   /* [num_req] */
    const int32_t *ctx_lens;     /* [num_req] */
    const int32_t *seq_lens;     /* [num_req] */
    const int32_t *status;       /* [num_req] or NULL (all requests taken as valid) */
    int32_t        num_req;
    int32_t        max_blocks;
} gf_tables;

/* Create / destroy a context on HIP device `device`.  gf_create makes that
 * device current for the calling thread. */
int32_t gf_create(gf_ctx **out, int32_t device);
int32_t gf_destroy(gf_ctx *ctx);

/* Text for a GF_ERR_* code (static string, host). */
const char *gf_strerror(int32_t code);

/* Text of the last HIP error seen by this context (host string owned by ctx). */
const char *gf_last_hip_error(const gf_ctx *ctx);

/*
 * gf_resolve_path -- wGraph node path -> block table + lengths.
 * (Paper: the KV of a workflow is assembled from its selected operation nodes;
 *  P in Eq. 7 is the prefix path; E_op holds the valid transitions.)
 *
 * Request r has the node path path_nodes[path_ptr[r] .. path_ptr[r+1]) (may be
 * empty), new_lens[r] new tokens (new_lens NULL = 0 for all) whose K/V live in
 * the private tail blocks tail_blocks[tail_ptr[r] .. tail_ptr[r+1]) (tail_ptr
 * and tail_blocks NULL = no tail blocks; then new_lens must be 0).
 * For a valid request it writes
 *   block_table[r][:]  the nodes' block lists in path order, then the first
 *                      ceil(new_len/16) tail blocks, then -1 up to max_blocks
 *   block_ntok[r][:]   valid tokens per entry: 16, except the last block of
 *                      each segment (remainder); 0 in the padding
 *   num_blocks[r], ctx_lens[r] = sum node_len, seq_lens[r] = ctx + new_len,
 *   status[r] = GF_ST_OK.
 * For an invalid request it writes status[r] = the first failing class in the
 * order BAD_NODE, BAD_EDGE, BAD_TAIL, BAD_BLOCK, OVERFLOW, and pad outputs
 * (table -1, ntok 0, num_blocks 0, both lengths 0).
 * Integer work only; results are exact.  Every output array is fully written.
 */
int32_t gf_resolve_path(gf_ctx *ctx, const gf_graph *graph, int32_t num_req,
                        const int32_t *path_ptr,    /* [num_req+1] device */
                        const int32_t *path_nodes,  /* device */
                        const int32_t *new_lens,    /* [num_req] device or NULL */
                        const int32_t *tail_ptr,    /* [num_req+1] device or NULL */
                        const int32_t *tail_blocks, /* device or NULL */
                        int32_t max_blocks, int32_t num_pool_blocks,
                        int32_t *block_table,       /* [num_req][max_blocks] device, out */
                        int32_t *block_ntok,        /* [num_req][max_blocks] device, out */
                        int32_t *num_blocks,        /* [num_req] device, out */
                        int32_t *ctx_lens,          /* [num_req] device, out */
                        int32_t *seq_lens,          /* [num_req] device, out */
                        int32_t *status,            /* [num_req] device, out */
                        void *stream);

/*
 * gf_attn_prefill -- new tokens attend to the ancestor-node KV (and causally
 * to each other) through the block table, with no second prefill of the
 * shared prefix; it is also the on-the-fly fallback of the paper's "Effective
 * Path Pruning".
 *
 * Request r owns query rows q_ptr[r] .. q_ptr[r+1) (n_r = seq_lens[r] -
 * ctx_lens[r] of them; the K/V of those new tokens are already in the tail
 * blocks).  For row i and query head h (kv head h / G):
 *   o[i,h,:] = sum_j softmax_j( sm_scale * <q[i,h,:], K_j> ) V_j
 * over j in {all ctx_lens[r] context tokens} U {new tokens 0..i}.
 *   q   [total_q][num_q_heads][head_dim] bf16 (device, in)
 *   o   same shape, bf16 round-to-nearest-even (device, out)
 *   lse [total_q][num_q_heads] fp32 natural-log log-sum-exp of the scaled
 *       scores, or NULL (device, out)
 *   max_q  an upper bound on n_r over the batch (host value; only checked to be
 *          non-negative: the work list is built on the device from the tables).
 * Rows of requests whose status is non-zero, or whose row count
 * q_ptr[r+1]-q_ptr[r] differs from seq_lens[r]-ctx_lens[r], are left untouched.
 * Accumulation and softmax are fp32.
 */
int32_t gf_attn_prefill(gf_ctx *ctx, const gf_attn_params *params, const gf_kv_pool *pool,
                        const gf_tables *tables,
                        const void *q, const int32_t *q_ptr /* [num_req+1] device */,
                        int32_t total_q, int32_t max_q,
                        void *o, float *lse, void *stream);

/*
 * gf_attn_prefill_noalloc -- gf_attn_prefill for callers that cannot allocate:
 * code under HIP graph capture, serving loops that must not reach hipMalloc,
 * harnesses that forbid it.  Same arguments, same kernels, same result (bit for
 * bit) as gf_attn_prefill; the one difference is where the work list of the
 * call lives: in a fixed device array of 1 MiB inside the library (one per GPU,
 * held until the process ends; its address is looked up by gf_create) instead
 * of a buffer of the context that grows on demand.  The call never allocates,
 * frees or synchronises.  It returns GF_ERR_WORKSPACE (and says so in
 * gf_last_hip_error) when the batch's work list does not fit:
 *     8 + 8 * (total_q / (128 / G) + num_req) bytes <= 1 MiB,   G = num_q_heads / num_kv_heads
 * (about 131 000 work items: e.g. 4 M new tokens at G = 4), and GF_ERR_BAD_SHAPE
 * when the context's device is not the calling thread's current device.
 * All calls on one GPU share the array, whatever their context: two such calls
 * that overlap in time on one GPU (different streams) race; calls on one stream
 * are ordered and need no clearing in between (the list is rebuilt by every call).
 */
int32_t gf_attn_prefill_noalloc(gf_ctx *ctx, const gf_attn_params *params, const gf_kv_pool *pool,
                                const gf_tables *tables,
                                const void *q, const int32_t *q_ptr /* [num_req+1] device */,
                                int32_t total_q, int32_t max_q,
                                void *o, float *lse, void *stream);

/*
 * gf_attn_decode -- one decode step per request: the query of request r is the
 * last of its seq_lens[r] tokens and attends to all of them (all context
 * tokens of the path plus every token in its tail blocks), by the same formula.
 *   q   [num_req][num_q_heads][head_dim] bf16 (device, in)
 *   o   same shape bf16 (device, out);  lse [num_req][num_q_heads] fp32 or NULL
 * The context is cut into chunks of blocks that are reduced independently
 * (fp32 partial max / sum / weighted values in the context's workspace) and
 * merged with the log-sum-exp rule.  Requests whose status is non-zero, or
 * whose seq_len is 0, get zero rows (lse -inf).
 */
int32_t gf_attn_decode(gf_ctx *ctx, const gf_attn_params *params, const gf_kv_pool *pool,
                       const gf_tables *tables,
                       const void *q, void *o, float *lse, void *stream);

/* per-block status words written by gf_kv_apply_residual */
#define GF_RS_OK         0
#define GF_RS_BAD_BLOCK  1   /* source or destination block id outside the pool: block skipped */
#define GF_RS_BAD_INDEX  2   /* a residual entry addresses an element outside its image: entry ignored */
#define GF_RS_TRUNCATED  3   /* gf_kv_make_residual: entries of the item fell beyond `capacity` and were not written */

/*
 * gf_kv_apply_residual -- reconstruct prefix-conditioned KV blocks from base
 * blocks and sparse residuals (paper, "Differential-based KV Cache", Eq. 7:
 * KV(P, v) = KV_base(v) + dKV(P, v): the base KV of an operation node is loaded
 * and the residual of the current prefix is applied to it).
 *
 * Item b (one 16-token pool block, all kv heads, K and V):
 *   block dst_blocks[b]  <-  block src_blocks[b]  +  its residual entries.
 * The residual is a CSR with one row per (item, tensor, kv head) "image" of
 * 16 x head_dim elements: row r = (b * 2 + t) * num_kv_heads + h, t = 0 for K and
 * 1 for V, holds the entries res_idx[res_ptr[r] .. res_ptr[r+1]), res_val[...].
 * An entry adds the bf16 value res_val[e] to the LOGICAL element
 *   res_idx[e] = slot * head_dim + d          (token slot 0..15 of the block)
 * of its image, whatever the physical layout of the tensor inside the block.
 * Each sum is taken in fp32 and rounded to bf16 (nearest even); the elements no
 * entry names are copied bit for bit.  The base blocks are not modified.  The
 * caller then lists the destination blocks as the block list of a
 * prefix-conditioned instance of the node in the wGraph handed to
 * gf_resolve_path; the attention calls read them like any other block.
 *
 * Contract: the destination blocks are distinct from each other and from every
 * source block of the call; the entries of one row name distinct elements
 * (a repeated element is a race); res_ptr is non-decreasing from 0.
 * GF_FP8_E4M3 pools: the base block is widened (code -> value, times the source
 * block's scale, fp32), the entries are added in fp32, and the destination block
 * is quantised under a scale of its own, per tensor: scale = amax / 448 over the
 * whole block (all kv heads, all 16 slots; 1.0 if 0), code = e4m3(clamp(x /
 * scale, +-448)), fp32 division, nearest even; k_scale[dst] / v_scale[dst] are
 * written.  There the destination may be the source block itself.
 *   k_pool, v_pool    the pool tensors (device, read and written)
 *   k_scale, v_scale  [num_pool_blocks] fp32 (device, read and written), GF_FP8_E4M3 only, else NULL
 *   status          [num_items] device, out, or NULL: GF_RS_* per item
 */
int32_t gf_kv_apply_residual(gf_ctx *ctx, const gf_attn_params *params,
                             void *k_pool, void *v_pool, float *k_scale, float *v_scale,
                             int32_t num_pool_blocks, int32_t num_items,
                             const int32_t *src_blocks,  /* [num_items] device */
                             const int32_t *dst_blocks,  /* [num_items] device */
                             const int32_t *res_ptr,     /* [num_items * 2 * num_kv_heads + 1] device */
                             const uint16_t *res_idx,    /* [res_ptr[last]] device */
                             const uint16_t *res_val,    /* [res_ptr[last]] device, bf16 bits */
                             int32_t *status, void *stream);

/*
 * gf_kv_make_residual -- from dense prefix-conditioned KV to the stored sparse residual (paper,
 * "Differential-based KV Cache", Eq. 7, and the selection rule of its KV-sparsity appendix: of the difference
 * between the KV of an operation under a prefix and its base KV, the largest-magnitude entries that hold a
 * given share -- 95 % -- of the Frobenius energy are kept).  The inverse of gf_kv_apply_residual: item b
 * compares pool block full_blocks[b] (the node's KV computed under the prefix, e.g. by the on-the-fly fallback)
 * with pool block base_blocks[b] and writes the CSR rows (b * 2 + t) * num_kv_heads + h of that call's format:
 * per (item, tensor, kv head) image, difference = full - base in fp32; the entries are ranked by magnitude
 * (largest first, equal magnitudes by rising index); the squared magnitudes are summed in fp64 along that
 * order and the shortest prefix whose sum reaches energy_share x total is kept (nothing for an all-zero
 * difference); the kept differences are rounded to bf16 (nearest even) and written in rising index order.
 *   energy_share  in (0, 1]; 1 keeps every non-zero difference
 *   capacity      entries res_idx / res_val can hold.  res_ptr [num_items * 2 * num_kv_heads + 1] (device, out)
 *                 always holds the full row pointers; entries at positions >= capacity are not written and
 *                 their items report GF_RS_TRUNCATED (compare res_ptr[last] with capacity and call again)
 *   status        [num_items] device, out, or NULL: GF_RS_OK, GF_RS_BAD_BLOCK (an id outside the pool: the
 *                 item's rows are empty) or GF_RS_TRUNCATED
 * GF_BF16 pools only.  num_items * 2 * num_kv_heads * 16 * head_dim must stay below 2^31.  The pool is only read.
 */
int32_t gf_kv_make_residual(gf_ctx *ctx, const gf_attn_params *params, const void *k_pool, const void *v_pool,
                            int32_t num_pool_blocks, int32_t num_items,
                            const int32_t *base_blocks,  /* [num_items] device */
                            const int32_t *full_blocks,  /* [num_items] device */
                            double energy_share, int32_t capacity,
                            int32_t *res_ptr, uint16_t *res_idx, uint16_t *res_val, int32_t *status, void *stream);

/*
 * The packed form of a residual -- what is kept at rest (paper, "Differential-based KV Cache", Eq. 7, and the
 * KV-sparsity appendix: more than 75 % of key and 70 % of value entries of a prefix-induced difference are
 * negligible).  The coordinate rows above cost 2 B of index + 2 B of value per kept element (0.55 of a dense
 * bf16 block at those densities); the packed form keeps, per (item, tensor, kv head) image, one bit per element
 *   res_mask[row][w]  bit (i % 32) of word w = i / 32 is set iff logical element i = slot * head_dim + d is kept
 *                     (16 * head_dim / 32 words per row, rows as in gf_kv_apply_residual)
 * and the kept values alone, in rising element order, row after row: packed_val[res_ptr[row] ..
 * res_ptr[row + 1]) -- 0.34 of a dense block.  res_ptr is the same array in both forms.  A coordinate list whose
 * rows are sorted by element (gf_kv_make_residual writes such rows) already has its values in packed order.
 *   gf_kv_residual_pack          rows in any order -> res_mask, packed_val (not in place: packed_val != res_val).
 *                                An item with an entry outside its image or an element named twice reports
 *                                GF_RS_BAD_INDEX and its output is unspecified (all writes stay inside the item's
 *                                rows).
 *   gf_kv_residual_unpack        res_mask -> res_idx in rising order (the row's values are packed_val as they are).
 *                                An item with a row whose bit count differs from its row length reports
 *                                GF_RS_BAD_INDEX (indices are written as far as the row reaches).
 *   gf_kv_apply_residual_packed  gf_kv_apply_residual from the packed form: same arithmetic, same contract, same
 *                                result bit for bit.  GF_BF16 pools only.  A row whose bit count differs from its
 *                                row length reports GF_RS_BAD_INDEX (it is applied as far as its values reach).
 * All arrays device memory; status [num_items] or NULL.
 */
int32_t gf_kv_residual_pack(gf_ctx *ctx, const gf_attn_params *params, int32_t num_items,
                            const int32_t *res_ptr, const uint16_t *res_idx, const uint16_t *res_val,
                            uint32_t *res_mask, uint16_t *packed_val, int32_t *status, void *stream);
int32_t gf_kv_residual_unpack(gf_ctx *ctx, const gf_attn_params *params, int32_t num_items,
                              const int32_t *res_ptr, const uint32_t *res_mask, uint16_t *res_idx,
                              int32_t *status, void *stream);
int32_t gf_kv_apply_residual_packed(gf_ctx *ctx, const gf_attn_params *params, void *k_pool, void *v_pool,
                                    int32_t num_pool_blocks, int32_t num_items,
                                    const int32_t *src_blocks, const int32_t *dst_blocks,
                                    const int32_t *res_ptr, const uint32_t *res_mask, const uint16_t *packed_val,
                                    int32_t *status, void *stream);

/*
 * gf_attn_decode_residual -- gf_attn_decode with the sparse residuals applied
 * while the blocks are read, instead of being reconstructed into pool blocks
 * first (paper, "Differential-based KV Cache", Eq. 7: only the base KV of a node
 * is stored in full; the KV under a given prefix is the base plus that prefix's
 * sparse residual).  The pool then holds base blocks only.
 *
 * res_handle[r * max_blocks + e] = b in [0, num_items) makes table entry e of
 * request r read as  block_table[r][e] + residual item b  (the CSR of
 * gf_kv_apply_residual: rows (b * 2 + t) * num_kv_heads + h, logical element
 * indices, bf16 values); any other value (e.g. -1) reads the base block as it
 * is.  The sum of an element is taken in fp32 and rounded to bf16 before it is
 * used, so the result equals, bit for bit, gf_attn_decode over a table whose
 * entries point at blocks reconstructed by gf_kv_apply_residual.  An entry that
 * names an element outside its image is ignored; entries that name slots at or
 * beyond the block's token count change nothing visible (those slots are
 * masked).  The entries of one row name distinct elements.
 *   res_handle  [num_req][max_blocks] int32 (device, in)
 *   res_ptr     [num_items * 2 * num_kv_heads + 1], res_idx / res_val
 *               [res_ptr[last]] (device, in); may be NULL when num_items is 0
 * GF_BF16 pools only (GF_ERR_UNSUPPORTED otherwise: an e4m3 block reconstructed
 * by gf_kv_apply_residual carries a scale of its own, which no read-time sum
 * reproduces).  Everything else as in gf_attn_decode.
 */
int32_t gf_attn_decode_residual(gf_ctx *ctx, const gf_attn_params *params, const gf_kv_pool *pool,
                                const gf_tables *tables,
                                const int32_t *res_handle, int32_t num_items,
                                const int32_t *res_ptr, const uint16_t *res_idx, const uint16_t *res_val,
                                const void *q, void *o, float *lse, void *stream);

/*
 * gf_attn_prefill_residual -- gf_attn_prefill with the sparse residuals applied while the blocks are read
 * (paper, "Differential-based KV Cache", Eq. 7; with "Effective Path Pruning" this is also the on-the-fly
 * fallback itself: the new node's tokens attend to ancestors whose KV under the current prefix is base +
 * residual).  res_handle, num_items and the CSR are those of gf_attn_decode_residual: table entry e of request r
 * with res_handle[r * max_blocks + e] = b in [0, num_items) is read as its base block plus residual item b,
 * any other value reads the block as it is; each sum is taken in fp32 and rounded to bf16 before use, so the
 * result equals, bit for bit, gf_attn_prefill over a table whose entries point at blocks reconstructed by
 * gf_kv_apply_residual.  Entries outside their image are ignored; the entries of one row name distinct
 * elements.  Tail entries (the new tokens' own blocks) normally carry no handle.
 * GF_BF16 pools only (GF_ERR_UNSUPPORTED otherwise).  Everything else as in gf_attn_prefill.
 */
int32_t gf_attn_prefill_residual(gf_ctx *ctx, const gf_attn_params *params, const gf_kv_pool *pool,
                                 const gf_tables *tables,
                                 const int32_t *res_handle, int32_t num_items,
                                 const int32_t *res_ptr, const uint16_t *res_idx, const uint16_t *res_val,
                                 const void *q, const int32_t *q_ptr, int32_t total_q, int32_t max_q,
                                 void *o, float *lse, void *stream);

/*
 * State-management policy (paper, "Differential-based KV Cache": the KV of operation v under prefix path P
 * is the node's base KV plus a sparse residual that belongs to the pair (P, v); "Effective Path Pruning":
 * execution statistics identify the frequently taken transitions, only their residuals stay stored, a pair
 * without a stored residual falls back to on-the-fly KV computation).
 *
 * gf_residual_dir is the directory of the stored residuals: an open-addressing hash table (linear probing)
 * over (prefix path, node) pairs in CALLER-OWNED device arrays of `capacity` slots (a power of two, at
 * least twice the number of pairs is a good size).  A pair is the path (v_0 .. v_i), i >= 1, ending in the
 * node v_i; its stored residual is one residual item (see gf_kv_apply_residual) per block of v_i, items
 * first_item .. first_item + ceil(node_len/16) - 1 in block order; its transition is (v_{i-1}, v_i).  The
 * first node of a path has an empty prefix: its base KV is exact and it never has a residual.
 *   key[slot]         0 = empty, else gf_prefix_key of the pair's path
 *   prev / node       v_{i-1} and v_i (a slot matches when key, node and prev all agree)
 *   first_item        >= 0: stored; < 0: pruned, and the items it named were -2 - first_item .. (the caller
 *                     owns the residual storage and may reuse those items)
 *   uses              how many resolved requests walked this pair (kept by gf_resolve_path_residual)
 */
typedef struct {
    uint64_t *key;
    int32_t  *prev;
    int32_t  *node;
    int32_t  *first_item;
    int32_t  *uses;
    int32_t   capacity;
} gf_residual_dir;

/* per-pair status words written by gf_residual_dir_insert */
#define GF_DIR_OK        0
#define GF_DIR_FULL      1   /* no free slot: pair not inserted                 */
#define GF_DIR_BAD_PAIR  2   /* key 0 or negative first_item: pair not inserted */

/* Key of a prefix path (HOST function, host array): h = 0; for every node id v of the path, in order,
 * h = mix(h ^ (uint64)(uint32)v) with mix = the splitmix64 finaliser (z += 0x9E3779B97F4A7C15;
 * z = (z ^ z >> 30) * 0xBF58476D1CE4E5B9; z = (z ^ z >> 27) * 0x94D049BB133111EB; z ^= z >> 31); 0 maps to 1.
 * Two different paths share a key with probability 2^-64; a slot also compares node and prev. */
uint64_t gf_prefix_key(const int32_t *nodes, int32_t len);

/* Empty every slot of the directory (device arrays; asynchronous). */
int32_t gf_residual_dir_clear(gf_ctx *ctx, const gf_residual_dir *dir, void *stream);

/* Insert num_pairs pairs (device arrays keys / prev / node / first_item of that length; the pairs of one call
 * are distinct and not yet in the directory).  status [num_pairs] (device, out) or NULL: GF_DIR_* per pair. */
int32_t gf_residual_dir_insert(gf_ctx *ctx, const gf_residual_dir *dir, int32_t num_pairs,
                               const uint64_t *keys, const int32_t *prev, const int32_t *node,
                               const int32_t *first_item, int32_t *status, void *stream);

/*
 * gf_resolve_path_residual -- gf_resolve_path (same arguments, same outputs) plus, for the residual-aware
 * attention calls, the residual handle of every table entry:
 *   res_handle[r][e]  the residual item table entry e of request r is read with (first_item of the pair
 *                     that owns the entry + the entry's block index inside its node), or -1: tail entries,
 *                     padding, the first node of the path, pairs that are not in the directory or pruned,
 *                     and every entry of a request whose status is not GF_ST_OK
 *   num_fallback[r]   how many nodes of the path (beyond the first) have no stored residual: their KV under
 *                     this prefix has to be computed on the fly (gf_attn_prefill + gf_kv_append into blocks
 *                     of an instance node) if the base KV is not good enough
 * and the execution statistics of the requests with status GF_ST_OK: trans_count[e] += 1 per hop along
 * edge e (position in graph->edge_dst; trans_count [number of edges] device, may be NULL, needs the graph's
 * edge arrays) and dir->uses[slot] += 1 per walked pair that has a slot.  dir may have capacity 0.
 */
int32_t gf_resolve_path_residual(gf_ctx *ctx, const gf_graph *graph, int32_t num_req,
                                 const int32_t *path_ptr, const int32_t *path_nodes, const int32_t *new_lens,
                                 const int32_t *tail_ptr, const int32_t *tail_blocks,
                                 int32_t max_blocks, int32_t num_pool_blocks,
                                 int32_t *block_table, int32_t *block_ntok, int32_t *num_blocks,
                                 int32_t *ctx_lens, int32_t *seq_lens, int32_t *status,
                                 const gf_residual_dir *dir, int32_t *trans_count,
                                 int32_t *res_handle /* [num_req][max_blocks] device, out */,
                                 int32_t *num_fallback /* [num_req] device, out */, void *stream);

/*
 * gf_residual_dir_prune -- Effective Path Pruning: every stored pair whose transition (prev -> node) was
 * taken fewer than min_count times according to trans_count (an edge the graph does not have counts as
 * never taken) loses its residual: first_item becomes -2 - first_item.  pruned [2] (device, or NULL) is
 * ADDED to: [0] += pairs pruned, [1] += residual items freed.  The graph's edge arrays are required.
 */
int32_t gf_residual_dir_prune(gf_ctx *ctx, const gf_graph *graph, const gf_residual_dir *dir,
                              const int32_t *trans_count, int32_t min_count, int32_t *pruned, void *stream);

/*
 * gf_block_pool -- HOST-side owner of the physical block ids of a K/V pool (paper, "Topology-Aware State
 * Management": a node's KV is stored once and shared by every workflow through it; "Effective Path Pruning":
 * storage follows the working set).  A free list with reference counts; it never touches the pool tensors.
 *   alloc    hands out n free blocks with one reference each (ids[n], host, out); all or nothing:
 *            GF_ERR_WORKSPACE when fewer than n blocks are free
 *   retain   one more reference on each listed block (a second workflow through the node, a request in flight)
 *   release  one reference less on each listed block (a block listed k times loses k); a block whose count
 *            reaches zero goes back to the free list; *num_freed (host, may be NULL) = blocks freed
 *   retain / release fail with GF_ERR_BAD_SHAPE, changing nothing, when an id is outside the pool or a block
 *   does not hold the references asked for
 *   stats    free blocks, blocks in use, references in total, most blocks ever in use (any pointer may be NULL)
 *   refcount references on one block (>= 0), or a negative GF_ERR_* code
 * Calls on one pool are serialised internally.
 */
typedef struct gf_block_pool gf_block_pool;
int32_t gf_block_pool_create(gf_block_pool **out, int32_t num_blocks);
int32_t gf_block_pool_destroy(gf_block_pool *pool);
int32_t gf_block_pool_alloc(gf_block_pool *pool, int32_t n, int32_t *ids);
int32_t gf_block_pool_retain(gf_block_pool *pool, int32_t n, const int32_t *ids);
int32_t gf_block_pool_release(gf_block_pool *pool, int32_t n, const int32_t *ids, int32_t *num_freed);
int32_t gf_block_pool_stats(gf_block_pool *pool, int32_t *num_free, int32_t *num_in_use, int64_t *total_refs,
                            int32_t *peak_in_use);
int32_t gf_block_pool_refcount(gf_block_pool *pool, int32_t block);

/*
 * gf_kv_append -- write the K/V of every request's new tokens into its private
 * tail blocks (paper, "Topology-Aware State Management": states produced at run
 * time extend the KV assembled from the operation nodes; "Effective Path
 * Pruning": a state that is not stored is computed on the fly and must then be
 * put where attention reads it).  It closes the loop resolve -> append ->
 * prefill / decode.
 *
 * Request r has n_r = seq_lens[r] - ctx_lens[r] new tokens, rows q_ptr[r] ..
 * q_ptr[r+1) of k_new / v_new; its tail blocks are the last ceil(n_r/16) entries of
 * its block table.  Token i goes to tail block i/16, slot i%16:
 *   K[block][h][slot][d] = k_new[i][h][d]      V[block][h][d][slot] = v_new[i][h][d]
 * and the slots beyond the block's token count are written as zero.  A call
 * writes the whole tail of every request (growing a block in place: gf_kv_append_token).
 * GF_BF16: the bf16 bits are copied.  GF_FP8_E4M3: per block and tensor,
 *   scale = amax / 448 (amax over the block's valid tokens, all kv heads; 1.0 if 0),
 *   code  = e4m3(clamp(x / scale, -448, 448)), fp32 division, round to nearest even,
 * and k_scale[block] / v_scale[block] are written.
 * Requests with a non-zero status, or whose row count differs from n_r, are
 * skipped; so is a tail entry whose block id is outside the pool.
 *   k_new, v_new  [total_q][num_kv_heads][head_dim] bf16 (device, in)
 *   max_q         an upper bound on n_r over the batch (host value; sizes the grid;
 *                 tokens of a request beyond it are not written)
 * Of `tables`, block_table, num_blocks, ctx_lens, seq_lens and status are read.
 */
int32_t gf_kv_append(gf_ctx *ctx, const gf_attn_params *params,
                     void *k_pool, void *v_pool, float *k_scale, float *v_scale,
                     int32_t num_pool_blocks, const gf_tables *tables,
                     const void *k_new, const void *v_new,
                     const int32_t *q_ptr /* [num_req+1] device */,
                     int32_t total_q, int32_t max_q, void *stream);

/*
 * gf_kv_append_token -- the decode-step form of gf_kv_append: only the newest token of every
 * request is written (paper: as gf_kv_append; a decode loop produces one token per step and must
 * not rewrite the whole tail).  k_tok / v_tok [num_req][num_kv_heads][head_dim] bf16 hold that
 * token's K and V; it is token n_r - 1 of the request's new tokens (seq_lens already counts it) and
 * goes to slot s = (n_r - 1) % 16 of the block behind the request's LAST table entry.
 *   s == 0: the block is fresh and is written whole: zeros beside the token; GF_FP8_E4M3: its scale
 *           becomes amax(token) / 448 per tensor (1.0 if 0).
 *   s  > 0: GF_BF16: the token's row / column is written, nothing else.  GF_FP8_E4M3: per tensor,
 *           need = amax(token) / 448; if need <= scale[block] the token is coded with the block's
 *           scale; otherwise scale[block] = need and the codes in slots [0, s) are decoded,
 *           multiplied by the old scale, divided by the new one (fp32) and rounded to e4m3 again
 *           before the token is coded.  Slots beyond s are left as they are.
 * Requests with a non-zero status, without new tokens or without table entries are skipped, and so
 * is a block id outside the pool.  Of `tables`, block_table, num_blocks, ctx_lens, seq_lens and
 * status are read.  Two requests must not share a tail block.
 */
int32_t gf_kv_append_token(gf_ctx *ctx, const gf_attn_params *params,
                           void *k_pool, void *v_pool, float *k_scale, float *v_scale,
                           int32_t num_pool_blocks, const gf_tables *tables,
                           const void *k_tok, const void *v_tok, void *stream);

/*
 * gf_attn_decode_shared -- the same decode step as gf_attn_decode (same inputs,
 * same outputs, same skipping of failed requests), computed node by node: the
 * KV of an operation node is read once for a group of requests that pass
 * through it instead of once per request (paper: "Topology-Aware State
 * Management" stores a node's KV once for all workflows through it; here the
 * reads are shared as well as the storage).
 *
 * `graph`, path_ptr and path_nodes are the ones `tables` was resolved from
 * (gf_resolve_path): request r's table must be the block lists of its path
 * nodes in path order (ceil(node_len/16) entries each) followed by its tail
 * entries, which is what gf_resolve_path writes for a request with status 0.
 *   num_path_entries  the length of path_nodes, i.e. path_ptr[num_req] (HOST value)
 * The batch's node -> requests lists are built on the device inside the call.
 * One partial (max, sum, weighted values; fp32) is kept per (request, path
 * node, chunk of the node's blocks) and per chunk of tail entries, and a
 * request's partials are merged in path order: the result equals
 * gf_attn_decode's up to fp32 summation order and does not depend on the order
 * in which the device builds the lists.  Workspace: a buffer of the context's own
 * (grown on demand like gf_attn_decode's).
 */
int32_t gf_attn_decode_shared(gf_ctx *ctx, const gf_attn_params *params, const gf_kv_pool *pool,
                              const gf_graph *graph,
                              const int32_t *path_ptr   /* [num_req+1] device */,
                              const int32_t *path_nodes /* [num_path_entries] device */,
                              int32_t num_path_entries,
                              const gf_tables *tables, const void *q, void *o, float *lse, void *stream);

/*
 * gf_attn_decode_shared_residual -- gf_attn_decode_shared with the sparse residuals applied while the blocks
 * are read (paper, "Differential-based KV Cache", Eq. 7).  The KV of node v under prefix P is base(v) + the
 * residual of the pair (P, v), so requests share a read of v exactly when they reach it through the same
 * prefix: the lists are kept per (node, residual) pair instead of per node, and requests without a residual on
 * v share the base read as before.  res_handle, num_items and the CSR are those of gf_attn_decode_residual,
 * with one more rule, which gf_resolve_path_residual's output obeys: the handle b0 at a node's FIRST table
 * entry names the residual of the whole node for that request -- block j of the node reads item b0 + j -- and
 * a b0 outside [0, num_items - node blocks] (e.g. -1) reads every block of the node as stored; a residual's
 * items belong to one node.  Each sum is taken in fp32 and rounded to bf16 before use, so the result is
 * gf_attn_decode_shared's over a graph whose nodes are blocks reconstructed by gf_kv_apply_residual (same
 * tolerance against gf_attn_decode_residual as gf_attn_decode_shared has against gf_attn_decode).
 * GF_BF16 pools only (GF_ERR_UNSUPPORTED otherwise).  The lists of this call are not kept for
 * gf_attn_decode_shared_planned.  Everything else as in gf_attn_decode_shared.
 */
int32_t gf_attn_decode_shared_residual(gf_ctx *ctx, const gf_attn_params *params, const gf_kv_pool *pool,
                                       const gf_graph *graph, const int32_t *path_ptr, const int32_t *path_nodes,
                                       int32_t num_path_entries, const gf_tables *tables,
                                       const int32_t *res_handle, int32_t num_items,
                                       const int32_t *res_ptr, const uint16_t *res_idx, const uint16_t *res_val,
                                       const void *q, void *o, float *lse, void *stream);

/*
 * gf_decode_shared_plan / gf_attn_decode_shared_planned -- gf_attn_decode_shared in two parts, for callers
 * that run the same batch through many layers: the node -> requests lists and item records depend on the
 * batch (graph, paths, tables) only, not on the pool or the queries, so they are built once
 * (gf_decode_shared_plan) and every layer then calls gf_attn_decode_shared_planned with its own pool, q and o.
 * Same arguments, same meaning and same result as gf_attn_decode_shared (which is the two in a row).
 * The lists live in the context and stay valid until the next gf_decode_shared_plan or
 * gf_attn_decode_shared on that context, as long as the graph, path and table arrays they were built from
 * are not modified (a decode loop that grows the tails re-plans once per step).
 * gf_attn_decode_shared_planned returns GF_ERR_BAD_SHAPE when the context holds no lists, or lists built for
 * other arrays, sizes or head shape than the ones passed.  params->kv_dtype is ignored by the plan call.
 */
int32_t gf_decode_shared_plan(gf_ctx *ctx, const gf_attn_params *params, const gf_graph *graph,
                              const int32_t *path_ptr, const int32_t *path_nodes, int32_t num_path_entries,
                              const gf_tables *tables, void *stream);
int32_t gf_attn_decode_shared_planned(gf_ctx *ctx, const gf_attn_params *params, const gf_kv_pool *pool,
                                      const gf_graph *graph, const int32_t *path_ptr, const int32_t *path_nodes,
                                      int32_t num_path_entries, const gf_tables *tables,
                                      const void *q, void *o, float *lse, void *stream);

/*
 * gf_hbm_read_probe -- measurement aid, no part of the method: a plain read-only
 * streaming kernel over `bytes` bytes at `src` (device; a multiple of 16), 16
 * bytes per lane and trip, num_wg workgroups of 256 threads walking the buffer
 * with a grid stride; wg_sums[num_wg] (device, out) receives one word per
 * workgroup folded from everything it read.  Timed by the benchmark as the
 * streaming ceiling of the box, next to the bandwidth-bound decode kernels.
 */
int32_t gf_hbm_read_probe(gf_ctx *ctx, const void *src, int64_t bytes, uint32_t *wg_sums, int32_t num_wg,
                          void *stream);

/*
 * gf_hbm_tile_probe -- measurement aid, no part of the method: the read-only ceiling for the access pattern of
 * a block table.  The buffer at `src` (device) holds num_src_tiles tiles of tile_bytes bytes (a multiple of
 * 1024, at most 1 MiB); tile_ids[num_tiles] (device) gives the order in which tiles are read (an id outside the
 * buffer is folded into it), one wave per tile, 16 bytes per lane and load; wg_sums[num_wg] as above.
 */
int32_t gf_hbm_tile_probe(gf_ctx *ctx, const void *src, int32_t tile_bytes, int32_t num_src_tiles,
                          const int32_t *tile_ids, int64_t num_tiles, uint32_t *wg_sums, int32_t num_wg,
                          void *stream);

/*
 * gf_mfma_probe -- measurement aid, no part of the method: the rate at which the box issues the prefill kernel's
 * matrix instruction (v_mfma_f32_32x32x16_bf16) on operands the caller chooses, alone (softmax_mix = 0) or with
 * the vector instructions a softmax spends per MFMA at head_dim 128 riding along (softmax_mix = 1: six per MFMA,
 * one of them an exponential, on values that keep changing; no LDS or memory traffic in either form).
 * `operands` (device) holds operand_bytes bytes of bf16 values (a multiple of 1024, at least 1024); every wave
 * takes twelve 1 KB fragments from it (eight A, four B; wave w starts at fragment 12 w, wrapping round) and
 * issues iters x 8 MFMAs (32 x 32 x 16 each: 32 768 flop) into four independent accumulators, a different
 * fragment pair for every MFMA.  num_wg workgroups of 256 threads (one wave per SIMD each);
 * lane_sums[num_wg * 256] (device, out) receives one float per lane folded from its accumulators (and, with
 * softmax_mix, its vector values).  Timed by the benchmark on zeroed and on normally distributed operands: the
 * difference is what the chip's power management takes from the clock.
 * GF_ERR_BAD_SHAPE for sizes or a softmax_mix outside the above, GF_ERR_NULL for missing buffers.
 */
int32_t gf_mfma_probe(gf_ctx *ctx, const void *operands, int64_t operand_bytes, int32_t iters, int32_t softmax_mix,
                      float *lane_sums, int32_t num_wg, void *stream);

/* Tuning knob (host): table entries (16-token blocks) per split-KV chunk in
 * gf_attn_decode and gf_attn_decode_residual (built-in choice 64) and gf_attn_decode_shared (built-in choice and upper limit 64);
 * 0 restores the built-in choice.  Must be even. */
int32_t gf_set_decode_chunk_blocks(gf_ctx *ctx, int32_t chunk_blocks);

#ifdef __cplusplus
}
#endif
#endif /* GRAPHFLOW_H */
