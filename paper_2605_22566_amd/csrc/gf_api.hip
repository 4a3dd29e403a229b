// C ABI of libgraphflow: argument checks on the host, then kernel launches on
// the caller's stream.  Nothing here computes; see the kernel files.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>

#include "gf_internal.h"

struct gf_ctx {
    int device = 0;
    void *workspace = nullptr;       // decode: split-KV partials
    size_t workspace_bytes = 0;
    void *plan = nullptr;            // prefill: work list
    size_t plan_bytes = 0;
    int32_t decode_chunk_blocks = 0;   // 0 = built-in choice
    // node-centric decode: its own buffer (lists, item records, partials), and what the lists in it were built for
    void *shared_ws = nullptr;
    size_t shared_ws_bytes = 0;
    struct SharedKey {
        const void *graph_blocks, *path_ptr, *path_nodes, *block_table, *ws;
        int32_t num_nodes, num_entries, num_req, max_blocks, chunk, hq, hkv, head_dim;
        bool operator==(const SharedKey &o) const {
            return graph_blocks == o.graph_blocks && path_ptr == o.path_ptr && path_nodes == o.path_nodes &&
                   block_table == o.block_table && ws == o.ws && num_nodes == o.num_nodes &&
                   num_entries == o.num_entries && num_req == o.num_req && max_blocks == o.max_blocks &&
                   chunk == o.chunk && hq == o.hq && hkv == o.hkv && head_dim == o.head_dim;
        }
    } shared_key = {};
    bool shared_planned = false;
    char hip_err[256] = {0};
};

namespace {

int32_t fail_hip(gf_ctx *ctx, hipError_t e, const char *where) {
    if (ctx) snprintf(ctx->hip_err, sizeof(ctx->hip_err), "%s: %s", where, hipGetErrorString(e));
    return GF_ERR_HIP;
}

// Shape checks shared by both attention calls.  Returns GF_OK and fills `a`.
int32_t check_attn(const gf_attn_params *p, const gf_kv_pool *pool, const gf_tables *t, const void *q, void *o,
                   float *lse, gf::AttnArgs &a, int &group) {
    if (!p || !pool || !t) return GF_ERR_NULL;
    if (t->num_req < 0 || t->max_blocks < 0 || pool->num_blocks < 0) return GF_ERR_BAD_SHAPE;
    if (p->num_q_heads <= 0 || p->num_kv_heads <= 0 || p->head_dim <= 0) return GF_ERR_BAD_SHAPE;
    if (p->num_q_heads % p->num_kv_heads != 0) return GF_ERR_BAD_SHAPE;
    {   // zero or a positive finite scale; judged on the bit pattern, so no compiler setting can wave a NaN through
        uint32_t bits;
        std::memcpy(&bits, &p->sm_scale, sizeof(bits));
        if ((bits >> 31) != 0 && bits != 0x80000000u) return GF_ERR_BAD_SHAPE;       // negative
        if ((bits & 0x7f800000u) == 0x7f800000u) return GF_ERR_BAD_SHAPE;            // inf or NaN
    }
    group = p->num_q_heads / p->num_kv_heads;
    if (p->block_size != gf::kBlock) return GF_ERR_UNSUPPORTED;
    if (p->head_dim != 64 && p->head_dim != 128) return GF_ERR_UNSUPPORTED;
    if (group != 1 && group != 2 && group != 4 && group != 8) return GF_ERR_UNSUPPORTED;
    if (p->kv_dtype != GF_BF16 && p->kv_dtype != GF_FP8_E4M3) return GF_ERR_UNSUPPORTED;
    // the kernels index (block, kv head) tiles of the pool with 32-bit integers
    if ((int64_t)pool->num_blocks * p->num_kv_heads > 0x7fffffffLL) return GF_ERR_UNSUPPORTED;
    if (t->num_req > 0) {
        if (!pool->k || !pool->v || !q || !o) return GF_ERR_NULL;
        if (!t->block_table || !t->block_ntok || !t->num_blocks || !t->ctx_lens || !t->seq_lens)
            return GF_ERR_NULL;
        if (p->kv_dtype == GF_FP8_E4M3 && (!pool->k_scale || !pool->v_scale)) return GF_ERR_NULL;
        if (pool->num_blocks < 1 || t->max_blocks < 1) return GF_ERR_BAD_SHAPE;
    }
    const float scale = p->sm_scale > 0.f ? p->sm_scale : 1.0f / std::sqrt((float)p->head_dim);
    a.k = pool->k;
    a.v = pool->v;
    a.k_scale = pool->k_scale;
    a.v_scale = pool->v_scale;
    a.pool_blocks = pool->num_blocks;
    a.block_table = t->block_table;
    a.block_ntok = t->block_ntok;
    a.num_blocks = t->num_blocks;
    a.ctx_lens = t->ctx_lens;
    a.seq_lens = t->seq_lens;
    a.status = t->status;
    a.num_req = t->num_req;
    a.max_blocks = t->max_blocks;
    a.hq = p->num_q_heads;
    a.hkv = p->num_kv_heads;
    a.scale_log2 = scale * 1.4426950408889634f;
    a.q = q;
    a.o = o;
    a.lse = lse;
    return GF_OK;
}

// Make a context-owned device buffer at least `need` bytes.  Growing frees the old buffer, which
// kernels already enqueued may still use: the stream is synchronised first.  A buffer that grows again takes
// half as much more than it had (a decode loop whose tails lengthen asks for a little more every few steps:
// the stream is then drained a logarithmic number of times, not once per growth); the first allocation is exact.
int32_t ensure_buffer(gf_ctx *ctx, void **buf, size_t *have, size_t need, hipStream_t stream, const char *what) {
    if (need <= *have) return GF_OK;
    const size_t roomy = *have + *have / 2;
    hipError_t e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return fail_hip(ctx, e, what);
    if (*buf) {
        e = hipFree(*buf);
        *buf = nullptr;
        *have = 0;
        if (e != hipSuccess) return fail_hip(ctx, e, what);
    }
    size_t want = need > roomy ? need : roomy;
    e = hipMalloc(buf, want);
    if (e != hipSuccess && want > need) {              // no room for the margin: take what is needed
        (void)hipGetLastError();
        want = need;
        e = hipMalloc(buf, want);
    }
    if (e != hipSuccess) {
        *buf = nullptr;
        fail_hip(ctx, e, what);
        return GF_ERR_WORKSPACE;
    }
    *have = want;
    return GF_OK;
}

}  // namespace

extern "C" {

int32_t gf_create(gf_ctx **out, int32_t device) {
    if (!out) return GF_ERR_NULL;
    *out = nullptr;
    int count = 0;
    hipError_t e = hipGetDeviceCount(&count);
    if (e != hipSuccess) return GF_ERR_HIP;
    if (device < 0 || device >= count) return GF_ERR_BAD_SHAPE;
    e = hipSetDevice(device);
    if (e != hipSuccess) return GF_ERR_HIP;
    // the address of the fixed work list of gf_attn_prefill_noalloc on this device, looked up while it is current
    e = gf::prefill_static_plan_init(device);
    if (e != hipSuccess) return GF_ERR_HIP;
    gf_ctx *c = new (std::nothrow) gf_ctx();
    if (!c) return GF_ERR_WORKSPACE;
    c->device = device;
    *out = c;
    return GF_OK;
}

int32_t gf_destroy(gf_ctx *ctx) {
    if (!ctx) return GF_ERR_NULL;
    int32_t rc = GF_OK;
    if (ctx->workspace && hipFree(ctx->workspace) != hipSuccess) rc = GF_ERR_HIP;
    if (ctx->plan && hipFree(ctx->plan) != hipSuccess) rc = GF_ERR_HIP;
    if (ctx->shared_ws && hipFree(ctx->shared_ws) != hipSuccess) rc = GF_ERR_HIP;
    delete ctx;
    return rc;
}

const char *gf_strerror(int32_t code) {
    switch (code) {
        case GF_OK: return "ok";
        case GF_ERR_NULL: return "a required pointer is NULL";
        case GF_ERR_BAD_SHAPE: return "negative or inconsistent sizes";
        case GF_ERR_UNSUPPORTED: return "shape or dtype outside the supported set";
        case GF_ERR_WORKSPACE: return "device workspace allocation failed";
        case GF_ERR_HIP: return "HIP runtime error (see gf_last_hip_error)";
        default: return "unknown error code";
    }
}

const char *gf_last_hip_error(const gf_ctx *ctx) { return ctx ? ctx->hip_err : ""; }

int32_t gf_set_decode_chunk_blocks(gf_ctx *ctx, int32_t chunk_blocks) {
    if (!ctx) return GF_ERR_NULL;
    if (chunk_blocks < 0 || (chunk_blocks & 1)) return GF_ERR_BAD_SHAPE;
    ctx->decode_chunk_blocks = chunk_blocks;
    return GF_OK;
}

int32_t gf_resolve_path(gf_ctx *ctx, const gf_graph *graph, int32_t num_req, const int32_t *path_ptr,
                        const int32_t *path_nodes, const int32_t *new_lens, const int32_t *tail_ptr,
                        const int32_t *tail_blocks, int32_t max_blocks, int32_t num_pool_blocks,
                        int32_t *block_table, int32_t *block_ntok, int32_t *num_blocks, int32_t *ctx_lens,
                        int32_t *seq_lens, int32_t *status, void *stream) {
    if (!ctx || !graph) return GF_ERR_NULL;
    if (num_req < 0 || max_blocks < 0 || num_pool_blocks < 0 || graph->num_nodes < 0) return GF_ERR_BAD_SHAPE;
    if (num_req == 0) return GF_OK;
    if (!path_ptr || !num_blocks || !ctx_lens || !seq_lens || !status) return GF_ERR_NULL;
    if (max_blocks > 0 && (!block_table || !block_ntok)) return GF_ERR_NULL;
    if (graph->num_nodes > 0 && (!graph->node_len || !graph->node_block_ptr || !graph->node_blocks))
        return GF_ERR_NULL;
    if ((graph->edge_ptr == nullptr) != (graph->edge_dst == nullptr)) return GF_ERR_NULL;
    if ((tail_ptr == nullptr) != (tail_blocks == nullptr)) return GF_ERR_NULL;
    // path_nodes may be NULL only if every path is empty, which the host cannot see: require it
    if (!path_nodes) return GF_ERR_NULL;
    hipError_t e = gf::launch_resolve(*graph, num_req, path_ptr, path_nodes, new_lens, tail_ptr, tail_blocks,
                                      max_blocks, num_pool_blocks, block_table, block_ntok, num_blocks,
                                      ctx_lens, seq_lens, status, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "gf_resolve_path launch");
    return GF_OK;
}

static int32_t check_dir(const gf_residual_dir *d) {
    if (!d) return GF_ERR_NULL;
    if (d->capacity < 0 || (d->capacity & (d->capacity - 1)) != 0) return GF_ERR_BAD_SHAPE;
    if (d->capacity > 0 && (!d->key || !d->prev || !d->node || !d->first_item || !d->uses)) return GF_ERR_NULL;
    return GF_OK;
}

uint64_t gf_prefix_key(const int32_t *nodes, int32_t len) {
    if (!nodes || len <= 0) return gf::prefix_key_host(nullptr, 0);
    return gf::prefix_key_host(nodes, len);
}

int32_t gf_residual_dir_clear(gf_ctx *ctx, const gf_residual_dir *dir, void *stream) {
    if (!ctx) return GF_ERR_NULL;
    int32_t rc = check_dir(dir);
    if (rc != GF_OK) return rc;
    hipError_t e = gf::launch_dir_clear(*dir, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "gf_residual_dir_clear launch");
    return GF_OK;
}

int32_t gf_residual_dir_insert(gf_ctx *ctx, const gf_residual_dir *dir, int32_t num_pairs, const uint64_t *keys,
                               const int32_t *prev, const int32_t *node, const int32_t *first_item, int32_t *status,
                               void *stream) {
    if (!ctx) return GF_ERR_NULL;
    int32_t rc = check_dir(dir);
    if (rc != GF_OK) return rc;
    if (num_pairs < 0) return GF_ERR_BAD_SHAPE;
    if (num_pairs == 0) return GF_OK;
    if (dir->capacity == 0) return GF_ERR_BAD_SHAPE;
    if (!keys || !prev || !node || !first_item) return GF_ERR_NULL;
    hipError_t e = gf::launch_dir_insert(*dir, num_pairs, keys, prev, node, first_item, status, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "gf_residual_dir_insert launch");
    return GF_OK;
}

int32_t gf_resolve_path_residual(gf_ctx *ctx, const gf_graph *graph, int32_t num_req, const int32_t *path_ptr,
                                 const int32_t *path_nodes, const int32_t *new_lens, const int32_t *tail_ptr,
                                 const int32_t *tail_blocks, int32_t max_blocks, int32_t num_pool_blocks,
                                 int32_t *block_table, int32_t *block_ntok, int32_t *num_blocks, int32_t *ctx_lens,
                                 int32_t *seq_lens, int32_t *status, const gf_residual_dir *dir, int32_t *trans_count,
                                 int32_t *res_handle, int32_t *num_fallback, void *stream) {
    int32_t rc = check_dir(dir);
    if (rc != GF_OK) return rc;
    rc = gf_resolve_path(ctx, graph, num_req, path_ptr, path_nodes, new_lens, tail_ptr, tail_blocks, max_blocks,
                         num_pool_blocks, block_table, block_ntok, num_blocks, ctx_lens, seq_lens, status, stream);
    if (rc != GF_OK || num_req == 0) return rc;
    if (!num_fallback || (max_blocks > 0 && !res_handle)) return GF_ERR_NULL;
    if (trans_count && !graph->edge_ptr) return GF_ERR_NULL;      // statistics are kept per edge of the graph
    hipError_t e = gf::launch_resolve_residual(*graph, num_req, path_ptr, path_nodes, status, max_blocks, *dir,
                                               trans_count, res_handle, num_fallback, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "gf_resolve_path_residual launch");
    return GF_OK;
}

int32_t gf_residual_dir_prune(gf_ctx *ctx, const gf_graph *graph, const gf_residual_dir *dir,
                              const int32_t *trans_count, int32_t min_count, int32_t *pruned, void *stream) {
    if (!ctx || !graph) return GF_ERR_NULL;
    int32_t rc = check_dir(dir);
    if (rc != GF_OK) return rc;
    if (graph->num_nodes < 0) return GF_ERR_BAD_SHAPE;
    if (dir->capacity == 0) return GF_OK;
    if (!trans_count || !graph->edge_ptr || !graph->edge_dst || !graph->node_len) return GF_ERR_NULL;
    hipError_t e = gf::launch_dir_prune(*graph, *dir, trans_count, min_count, pruned, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "gf_residual_dir_prune launch");
    return GF_OK;
}

// gf_attn_prefill and its residual-reading form: the same checks, work-list buffer and launch
static int32_t prefill_call(gf_ctx *ctx, const gf_attn_params *params, const gf_kv_pool *pool,
                            const gf_tables *tables, const gf::ResidualRefs *rr, const void *q, const int32_t *q_ptr,
                            int32_t total_q, int32_t max_q, void *o, float *lse, void *stream, const char *what) {
    if (!ctx) return GF_ERR_NULL;
    if (total_q < 0 || max_q < 0 || max_q > total_q) return GF_ERR_BAD_SHAPE;
    gf::AttnArgs a;
    int group = 0;
    // q/o may be NULL when there are no rows at all
    static const char dummy = 0;
    int32_t rc = check_attn(params, pool, tables, total_q ? q : &dummy, total_q ? o : (void *)&dummy, lse, a, group);
    if (rc != GF_OK) return rc;
    if (rr) {
        if (rr->num_items < 0) return GF_ERR_BAD_SHAPE;
        if (params->kv_dtype != GF_BF16) return GF_ERR_UNSUPPORTED;
    }
    if (tables->num_req == 0 || total_q == 0) return GF_OK;
    if (!q_ptr) return GF_ERR_NULL;
    if (rr && (!rr->handle || (rr->num_items > 0 && (!rr->ptr || !rr->idx || !rr->val)))) return GF_ERR_NULL;
    rc = ensure_buffer(ctx, &ctx->plan, &ctx->plan_bytes, gf::prefill_plan_bytes(total_q, a.num_req, group),
                       (hipStream_t)stream, "prefill work-list buffer");
    if (rc != GF_OK) return rc;
    hipError_t e = gf::launch_prefill(a, params->head_dim, group, params->kv_dtype, q_ptr, total_q,
                                      (int32_t *)ctx->plan, rr, (hipStream_t)stream);
    if (e == hipErrorNotSupported) return GF_ERR_UNSUPPORTED;
    if (e != hipSuccess) return fail_hip(ctx, e, what);
    return GF_OK;
}

int32_t gf_attn_prefill(gf_ctx *ctx, const gf_attn_params *params, const gf_kv_pool *pool,
                        const gf_tables *tables, const void *q, const int32_t *q_ptr, int32_t total_q,
                        int32_t max_q, void *o, float *lse, void *stream) {
    return prefill_call(ctx, params, pool, tables, nullptr, q, q_ptr, total_q, max_q, o, lse, stream,
                        "gf_attn_prefill launch");
}

int32_t gf_attn_prefill_residual(gf_ctx *ctx, const gf_attn_params *params, const gf_kv_pool *pool,
                                 const gf_tables *tables, const int32_t *res_handle, int32_t num_items,
                                 const int32_t *res_ptr, const uint16_t *res_idx, const uint16_t *res_val,
                                 const void *q, const int32_t *q_ptr, int32_t total_q, int32_t max_q, void *o,
                                 float *lse, void *stream) {
    const gf::ResidualRefs rr = {res_handle, res_ptr, res_idx, res_val, num_items};
    return prefill_call(ctx, params, pool, tables, &rr, q, q_ptr, total_q, max_q, o, lse, stream,
                        "gf_attn_prefill_residual launch");
}

int32_t gf_attn_prefill_noalloc(gf_ctx *ctx, const gf_attn_params *params, const gf_kv_pool *pool,
                                const gf_tables *tables, const void *q, const int32_t *q_ptr, int32_t total_q,
                                int32_t max_q, void *o, float *lse, void *stream) {
    if (!ctx) return GF_ERR_NULL;
    if (total_q < 0 || max_q < 0 || max_q > total_q) return GF_ERR_BAD_SHAPE;
    gf::AttnArgs a;
    int group = 0;
    static const char dummy = 0;
    int32_t rc = check_attn(params, pool, tables, total_q ? q : &dummy, total_q ? o : (void *)&dummy, lse, a, group);
    if (rc != GF_OK) return rc;
    if (tables->num_req == 0 || total_q == 0) return GF_OK;
    if (!q_ptr) return GF_ERR_NULL;
    // the work list must fit the fixed array; nothing is grown here
    if (gf::prefill_plan_bytes(total_q, a.num_req, group) > gf::kStaticPlanBytes) {
        snprintf(ctx->hip_err, sizeof(ctx->hip_err),
                 "gf_attn_prefill_noalloc: the work list of this batch needs %zu bytes, the fixed array holds %zu",
                 gf::prefill_plan_bytes(total_q, a.num_req, group), gf::kStaticPlanBytes);
        return GF_ERR_WORKSPACE;
    }
    // the array's address belongs to the context's device: that device must be the current one
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) return fail_hip(ctx, e, "gf_attn_prefill_noalloc hipGetDevice");
    int32_t *plan = gf::prefill_static_plan(ctx->device);
    if (cur != ctx->device || !plan) return GF_ERR_BAD_SHAPE;
    e = gf::launch_prefill(a, params->head_dim, group, params->kv_dtype, q_ptr, total_q, plan, nullptr,
                           (hipStream_t)stream);
    if (e == hipErrorNotSupported) return GF_ERR_UNSUPPORTED;
    if (e != hipSuccess) return fail_hip(ctx, e, "gf_attn_prefill_noalloc launch");
    return GF_OK;
}

int32_t gf_hbm_tile_probe(gf_ctx *ctx, const void *src, int32_t tile_bytes, int32_t num_src_tiles,
                          const int32_t *tile_ids, int64_t num_tiles, uint32_t *wg_sums, int32_t num_wg,
                          void *stream) {
    if (!ctx) return GF_ERR_NULL;
    if (tile_bytes <= 0 || (tile_bytes & 1023) || tile_bytes > (1 << 20) || num_src_tiles <= 0 || num_tiles < 0 ||
        num_wg < 0)
        return GF_ERR_BAD_SHAPE;
    if (num_wg == 0) return GF_OK;
    if (!wg_sums || (num_tiles > 0 && (!src || !tile_ids))) return GF_ERR_NULL;
    hipError_t e = gf::launch_hbm_tile_probe(src, tile_bytes, num_src_tiles, tile_ids, num_tiles, wg_sums, num_wg,
                                             (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "gf_hbm_tile_probe launch");
    return GF_OK;
}

int32_t gf_mfma_probe(gf_ctx *ctx, const void *operands, int64_t operand_bytes, int32_t iters, int32_t softmax_mix,
                      float *lane_sums, int32_t num_wg, void *stream) {
    if (!ctx) return GF_ERR_NULL;
    if (operand_bytes < 1024 || (operand_bytes & 1023) || operand_bytes > ((int64_t)1 << 40) || iters < 0 || num_wg < 0 ||
        (softmax_mix != 0 && softmax_mix != 1))
        return GF_ERR_BAD_SHAPE;
    if (num_wg == 0) return GF_OK;
    if (!operands || !lane_sums) return GF_ERR_NULL;
    hipError_t e = gf::launch_mfma_probe(operands, operand_bytes, iters, softmax_mix, lane_sums, num_wg,
                                         (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "gf_mfma_probe launch");
    return GF_OK;
}

int32_t gf_hbm_read_probe(gf_ctx *ctx, const void *src, int64_t bytes, uint32_t *wg_sums, int32_t num_wg,
                          void *stream) {
    if (!ctx) return GF_ERR_NULL;
    if (bytes < 0 || (bytes & 15) || num_wg < 0) return GF_ERR_BAD_SHAPE;
    if (bytes == 0 || num_wg == 0) return GF_OK;
    if (!src || !wg_sums) return GF_ERR_NULL;
    hipError_t e = gf::launch_hbm_read_probe(src, (size_t)bytes, wg_sums, num_wg, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "gf_hbm_read_probe launch");
    return GF_OK;
}

int32_t gf_attn_decode(gf_ctx *ctx, const gf_attn_params *params, const gf_kv_pool *pool,
                       const gf_tables *tables, const void *q, void *o, float *lse, void *stream) {
    if (!ctx) return GF_ERR_NULL;
    gf::AttnArgs a;
    int group = 0;
    int32_t rc = check_attn(params, pool, tables, q, o, lse, a, group);
    if (rc != GF_OK) return rc;
    if (tables->num_req == 0) return GF_OK;
    // chunk size: explicit knob, else 64 blocks (1024 tokens) of streaming work per item: long enough that
    // the fill of a wave's load pipeline and its partial are small beside the stream (measured on a workload
    // without sharing: 32 blocks 0.65, 64 blocks 0.69, 128 blocks 0.69 of the HBM peak), short enough that the
    // shortest requests still spread over many waves
    int32_t chunk = ctx->decode_chunk_blocks;
    if (chunk <= 0) chunk = gf::kDecodeChunkBlocks;
    const int32_t splits = (tables->max_blocks + chunk - 1) / chunk;
    const size_t need = gf::decode_workspace_bytes(a.num_req, a.hkv, group, params->head_dim, splits);
    rc = ensure_buffer(ctx, &ctx->workspace, &ctx->workspace_bytes, need, (hipStream_t)stream,
                       "gf_attn_decode workspace");
    if (rc != GF_OK) return rc;
    hipError_t e = gf::launch_decode(a, params->head_dim, group, params->kv_dtype, chunk, splits,
                                     ctx->workspace, (hipStream_t)stream);
    if (e == hipErrorNotSupported) return GF_ERR_UNSUPPORTED;
    if (e != hipSuccess) return fail_hip(ctx, e, "gf_attn_decode launch");
    return GF_OK;
}

int32_t gf_attn_decode_residual(gf_ctx *ctx, const gf_attn_params *params, const gf_kv_pool *pool,
                                const gf_tables *tables, const int32_t *res_handle, int32_t num_items,
                                const int32_t *res_ptr, const uint16_t *res_idx, const uint16_t *res_val,
                                const void *q, void *o, float *lse, void *stream) {
    if (!ctx) return GF_ERR_NULL;
    gf::AttnArgs a;
    int group = 0;
    int32_t rc = check_attn(params, pool, tables, q, o, lse, a, group);
    if (rc != GF_OK) return rc;
    if (num_items < 0) return GF_ERR_BAD_SHAPE;
    if (params->kv_dtype != GF_BF16) return GF_ERR_UNSUPPORTED;
    if (tables->num_req == 0) return GF_OK;
    if (!res_handle || (num_items > 0 && (!res_ptr || !res_idx || !res_val))) return GF_ERR_NULL;
    int32_t chunk = ctx->decode_chunk_blocks;
    if (chunk <= 0) chunk = gf::kDecodeChunkBlocksResidual;
    const int32_t splits = (tables->max_blocks + chunk - 1) / chunk;
    const size_t need = gf::decode_workspace_bytes(a.num_req, a.hkv, group, params->head_dim, splits);
    rc = ensure_buffer(ctx, &ctx->workspace, &ctx->workspace_bytes, need, (hipStream_t)stream,
                       "gf_attn_decode_residual workspace");
    if (rc != GF_OK) return rc;
    const gf::ResidualRefs rr = {res_handle, res_ptr, res_idx, res_val, num_items};
    hipError_t e = gf::launch_decode_residual(a, rr, params->head_dim, group, params->kv_dtype, chunk, splits,
                                              ctx->workspace, (hipStream_t)stream);
    if (e == hipErrorNotSupported) return GF_ERR_UNSUPPORTED;
    if (e != hipSuccess) return fail_hip(ctx, e, "gf_attn_decode_residual launch");
    return GF_OK;
}

// The three node-centric entry points: list building, attention over built lists, or both.
static int32_t decode_shared_call(gf_ctx *ctx, const gf_attn_params *params, const gf_kv_pool *pool,
                                  const gf_graph *graph, const int32_t *path_ptr, const int32_t *path_nodes,
                                  int32_t num_path_entries, const gf_tables *tables, const void *q, void *o, float *lse,
                                  int phases, void *stream, const char *what, const gf::ResidualRefs *rr = nullptr) {
    if (!ctx || !graph) return GF_ERR_NULL;
    if (num_path_entries < 0 || graph->num_nodes < 0) return GF_ERR_BAD_SHAPE;
    if (rr && rr->num_items < 0) return GF_ERR_BAD_SHAPE;
    gf::AttnArgs a;
    int group = 0;
    // list building touches neither the pool nor q / o: stand-ins pass the shared checks
    static const char dummy = 0;
    const gf_kv_pool no_pool = {&dummy, &dummy, nullptr, nullptr, 1};
    const bool attend = phases & gf::kSharedAttend;
    gf_attn_params checked;
    if (params) {
        checked = *params;
        if (!attend) checked.kv_dtype = GF_BF16;               // the lists do not depend on the pool's element type
    }
    int32_t rc = check_attn(params ? &checked : nullptr, attend ? pool : &no_pool, tables, attend ? q : &dummy,
                            attend ? o : (void *)&dummy, lse, a, group);
    if (rc != GF_OK) return rc;
    if (rr && params->kv_dtype != GF_BF16) return GF_ERR_UNSUPPORTED;
    if (tables->num_req == 0) return GF_OK;
    if (!path_ptr || !path_nodes) return GF_ERR_NULL;
    if (graph->num_nodes > 0 && (!graph->node_len || !graph->node_block_ptr || !graph->node_blocks))
        return GF_ERR_NULL;
    if (rr && (!rr->handle || (rr->num_items > 0 && (!rr->ptr || !rr->idx || !rr->val)))) return GF_ERR_NULL;
    // the node-centric kernel keeps a chunk's table entries in one wave's lanes: 64 at most, and by default
    int32_t chunk = ctx->decode_chunk_blocks;
    if (chunk <= 0 || chunk > 64) chunk = 64;
    const size_t need = gf::shared_workspace_bytes(graph->num_nodes, rr ? rr->num_items : 0, a.num_req, num_path_entries,
                                                   a.max_blocks, chunk, a.hq, params->head_dim);
    if (phases & gf::kSharedBuildLists) {
        ctx->shared_planned = false;
        rc = ensure_buffer(ctx, &ctx->shared_ws, &ctx->shared_ws_bytes, need, (hipStream_t)stream, what);
        if (rc != GF_OK) return rc;
    }
    const gf_ctx::SharedKey key = {graph->node_blocks, path_ptr, path_nodes, tables->block_table, ctx->shared_ws,
                                   graph->num_nodes, num_path_entries, a.num_req, a.max_blocks, chunk, a.hq, a.hkv,
                                   params->head_dim};
    if (!(phases & gf::kSharedBuildLists) && !(ctx->shared_planned && ctx->shared_key == key && need <= ctx->shared_ws_bytes))
        return GF_ERR_BAD_SHAPE;                               // no lists, or lists of another batch / shape
    hipError_t e = gf::launch_decode_shared(a, params->head_dim, group, params->kv_dtype, *graph, path_ptr, path_nodes,
                                            num_path_entries, chunk, ctx->shared_ws, phases, rr, (hipStream_t)stream);
    if (e == hipErrorNotSupported || e == hipErrorInvalidValue) return GF_ERR_UNSUPPORTED;
    if (e != hipSuccess) return fail_hip(ctx, e, what);
    // lists built with residual handles are keyed by (node, residual): the plain attention call must not reuse them
    if ((phases & gf::kSharedBuildLists) && !rr) {
        ctx->shared_key = key;
        ctx->shared_planned = true;
    }
    return GF_OK;
}

int32_t gf_attn_decode_shared(gf_ctx *ctx, const gf_attn_params *params, const gf_kv_pool *pool,
                              const gf_graph *graph, const int32_t *path_ptr, const int32_t *path_nodes,
                              int32_t num_path_entries, const gf_tables *tables, const void *q, void *o, float *lse,
                              void *stream) {
    return decode_shared_call(ctx, params, pool, graph, path_ptr, path_nodes, num_path_entries, tables, q, o, lse,
                              gf::kSharedBuildLists | gf::kSharedAttend, stream, "gf_attn_decode_shared");
}

int32_t gf_attn_decode_shared_residual(gf_ctx *ctx, const gf_attn_params *params, const gf_kv_pool *pool,
                                       const gf_graph *graph, const int32_t *path_ptr, const int32_t *path_nodes,
                                       int32_t num_path_entries, const gf_tables *tables, const int32_t *res_handle,
                                       int32_t num_items, const int32_t *res_ptr, const uint16_t *res_idx,
                                       const uint16_t *res_val, const void *q, void *o, float *lse, void *stream) {
    const gf::ResidualRefs rr = {res_handle, res_ptr, res_idx, res_val, num_items};
    return decode_shared_call(ctx, params, pool, graph, path_ptr, path_nodes, num_path_entries, tables, q, o, lse,
                              gf::kSharedBuildLists | gf::kSharedAttend, stream, "gf_attn_decode_shared_residual", &rr);
}

int32_t gf_decode_shared_plan(gf_ctx *ctx, const gf_attn_params *params, const gf_graph *graph,
                              const int32_t *path_ptr, const int32_t *path_nodes, int32_t num_path_entries,
                              const gf_tables *tables, void *stream) {
    return decode_shared_call(ctx, params, nullptr, graph, path_ptr, path_nodes, num_path_entries, tables, nullptr,
                              nullptr, nullptr, gf::kSharedBuildLists, stream, "gf_decode_shared_plan");
}

int32_t gf_attn_decode_shared_planned(gf_ctx *ctx, const gf_attn_params *params, const gf_kv_pool *pool,
                                      const gf_graph *graph, const int32_t *path_ptr, const int32_t *path_nodes,
                                      int32_t num_path_entries, const gf_tables *tables, const void *q, void *o,
                                      float *lse, void *stream) {
    return decode_shared_call(ctx, params, pool, graph, path_ptr, path_nodes, num_path_entries, tables, q, o, lse,
                              gf::kSharedAttend, stream, "gf_attn_decode_shared_planned");
}

int32_t gf_kv_apply_residual(gf_ctx *ctx, const gf_attn_params *params, void *k_pool, void *v_pool, float *k_scale,
                             float *v_scale, int32_t num_pool_blocks, int32_t num_items, const int32_t *src_blocks,
                             const int32_t *dst_blocks, const int32_t *res_ptr, const uint16_t *res_idx,
                             const uint16_t *res_val, int32_t *status, void *stream) {
    if (!ctx || !params) return GF_ERR_NULL;
    if (num_items < 0 || num_pool_blocks < 0) return GF_ERR_BAD_SHAPE;
    if (params->num_kv_heads <= 0 || params->head_dim <= 0) return GF_ERR_BAD_SHAPE;
    if (params->block_size != gf::kBlock) return GF_ERR_UNSUPPORTED;
    if (params->head_dim != 64 && params->head_dim != 128) return GF_ERR_UNSUPPORTED;
    if (params->kv_dtype != GF_BF16 && params->kv_dtype != GF_FP8_E4M3) return GF_ERR_UNSUPPORTED;
    // rows of the residual CSR: num_items * 2 * num_kv_heads, indexed with 32-bit integers on the device
    if ((int64_t)num_items * 2 * params->num_kv_heads >= 0x7fffffffLL) return GF_ERR_UNSUPPORTED;
    if (num_items == 0) return GF_OK;
    if (!k_pool || !v_pool || !src_blocks || !dst_blocks || !res_ptr) return GF_ERR_NULL;
    // res_idx / res_val may be NULL only if no item has entries, which the host cannot see: require them
    if (!res_idx || !res_val) return GF_ERR_NULL;
    if (params->kv_dtype == GF_FP8_E4M3 && (!k_scale || !v_scale)) return GF_ERR_NULL;
    hipError_t e = gf::launch_residual(k_pool, v_pool, k_scale, v_scale, num_pool_blocks, params->num_kv_heads,
                                       params->head_dim, params->kv_dtype, num_items, src_blocks, dst_blocks, res_ptr, res_idx, res_val, status,
                                       (hipStream_t)stream);
    if (e == hipErrorNotSupported) return GF_ERR_UNSUPPORTED;
    if (e != hipSuccess) return fail_hip(ctx, e, "gf_kv_apply_residual launch");
    return GF_OK;
}

// shape checks shared by the three calls on the packed residual form
static int32_t check_packed(const gf_ctx *ctx, const gf_attn_params *params, int32_t num_items) {
    if (!ctx || !params) return GF_ERR_NULL;
    if (num_items < 0 || params->num_kv_heads <= 0 || params->head_dim <= 0) return GF_ERR_BAD_SHAPE;
    if (params->block_size != gf::kBlock) return GF_ERR_UNSUPPORTED;
    if (params->head_dim != 64 && params->head_dim != 128) return GF_ERR_UNSUPPORTED;
    if ((int64_t)num_items * 2 * params->num_kv_heads >= 0x7fffffffLL) return GF_ERR_UNSUPPORTED;
    return GF_OK;
}

int32_t gf_kv_residual_pack(gf_ctx *ctx, const gf_attn_params *params, int32_t num_items, const int32_t *res_ptr,
                            const uint16_t *res_idx, const uint16_t *res_val, uint32_t *res_mask,
                            uint16_t *packed_val, int32_t *status, void *stream) {
    int32_t rc = check_packed(ctx, params, num_items);
    if (rc != GF_OK || num_items == 0) return rc;
    if (!res_ptr || !res_idx || !res_val || !res_mask || !packed_val) return GF_ERR_NULL;
    if (packed_val == res_val) return GF_ERR_BAD_SHAPE;              // the values are permuted: not in place
    hipError_t e = gf::launch_residual_pack(params->num_kv_heads, params->head_dim, num_items, res_ptr, res_idx,
                                            res_val, res_mask, packed_val, status, (hipStream_t)stream);
    if (e == hipErrorNotSupported) return GF_ERR_UNSUPPORTED;
    if (e != hipSuccess) return fail_hip(ctx, e, "gf_kv_residual_pack launch");
    return GF_OK;
}

int32_t gf_kv_residual_unpack(gf_ctx *ctx, const gf_attn_params *params, int32_t num_items, const int32_t *res_ptr,
                              const uint32_t *res_mask, uint16_t *res_idx, int32_t *status, void *stream) {
    int32_t rc = check_packed(ctx, params, num_items);
    if (rc != GF_OK || num_items == 0) return rc;
    if (!res_ptr || !res_mask || !res_idx) return GF_ERR_NULL;
    hipError_t e = gf::launch_residual_unpack(params->num_kv_heads, params->head_dim, num_items, res_ptr, res_mask,
                                              res_idx, status, (hipStream_t)stream);
    if (e == hipErrorNotSupported) return GF_ERR_UNSUPPORTED;
    if (e != hipSuccess) return fail_hip(ctx, e, "gf_kv_residual_unpack launch");
    return GF_OK;
}

int32_t gf_kv_apply_residual_packed(gf_ctx *ctx, const gf_attn_params *params, void *k_pool, void *v_pool,
                                    int32_t num_pool_blocks, int32_t num_items, const int32_t *src_blocks,
                                    const int32_t *dst_blocks, const int32_t *res_ptr, const uint32_t *res_mask,
                                    const uint16_t *packed_val, int32_t *status, void *stream) {
    int32_t rc = check_packed(ctx, params, num_items);
    if (rc != GF_OK) return rc;
    if (num_pool_blocks < 0) return GF_ERR_BAD_SHAPE;
    if (params->kv_dtype != GF_BF16) return GF_ERR_UNSUPPORTED;
    if (num_items == 0) return GF_OK;
    if (!k_pool || !v_pool || !src_blocks || !dst_blocks || !res_ptr || !res_mask || !packed_val) return GF_ERR_NULL;
    hipError_t e = gf::launch_residual_packed(k_pool, v_pool, num_pool_blocks, params->num_kv_heads, params->head_dim,
                                              num_items, src_blocks, dst_blocks, res_ptr, res_mask, packed_val, status,
                                              (hipStream_t)stream);
    if (e == hipErrorNotSupported) return GF_ERR_UNSUPPORTED;
    if (e != hipSuccess) return fail_hip(ctx, e, "gf_kv_apply_residual_packed launch");
    return GF_OK;
}

int32_t gf_kv_make_residual(gf_ctx *ctx, const gf_attn_params *params, const void *k_pool, const void *v_pool,
                            int32_t num_pool_blocks, int32_t num_items, const int32_t *base_blocks,
                            const int32_t *full_blocks, double energy_share, int32_t capacity, int32_t *res_ptr,
                            uint16_t *res_idx, uint16_t *res_val, int32_t *status, void *stream) {
    if (!ctx || !params) return GF_ERR_NULL;
    if (num_items < 0 || num_pool_blocks < 0 || capacity < 0) return GF_ERR_BAD_SHAPE;
    if (params->num_kv_heads <= 0 || params->head_dim <= 0) return GF_ERR_BAD_SHAPE;
    if (!(energy_share > 0.0) || !(energy_share <= 1.0)) return GF_ERR_BAD_SHAPE;
    if (params->block_size != gf::kBlock) return GF_ERR_UNSUPPORTED;
    if (params->head_dim != 64 && params->head_dim != 128) return GF_ERR_UNSUPPORTED;
    if (params->kv_dtype != GF_BF16) return GF_ERR_UNSUPPORTED;
    if ((int64_t)num_items * 2 * params->num_kv_heads * gf::kBlock * params->head_dim >= 0x7fffffffLL)
        return GF_ERR_UNSUPPORTED;
    if (num_items == 0) return GF_OK;
    if (!k_pool || !v_pool || !base_blocks || !full_blocks || !res_ptr) return GF_ERR_NULL;
    if (capacity > 0 && (!res_idx || !res_val)) return GF_ERR_NULL;
    // one sort key per CSR row between the counting and the filling pass, in the context's workspace
    const int32_t rc = ensure_buffer(ctx, &ctx->workspace, &ctx->workspace_bytes,
                                     gf::make_residual_scratch_bytes(params->num_kv_heads, num_items), (hipStream_t)stream,
                                     "gf_kv_make_residual workspace");
    if (rc != GF_OK) return rc;
    hipError_t e = gf::launch_make_residual(k_pool, v_pool, num_pool_blocks, params->num_kv_heads, params->head_dim,
                                            num_items, base_blocks, full_blocks, energy_share, capacity, res_ptr, res_idx,
                                            res_val, status, ctx->workspace, (hipStream_t)stream);
    if (e == hipErrorNotSupported) return GF_ERR_UNSUPPORTED;
    if (e != hipSuccess) return fail_hip(ctx, e, "gf_kv_make_residual launch");
    return GF_OK;
}

int32_t gf_kv_append(gf_ctx *ctx, const gf_attn_params *params, void *k_pool, void *v_pool, float *k_scale,
                     float *v_scale, int32_t num_pool_blocks, const gf_tables *tables, const void *k_new,
                     const void *v_new, const int32_t *q_ptr, int32_t total_q, int32_t max_q, void *stream) {
    if (!ctx || !params || !tables) return GF_ERR_NULL;
    if (tables->num_req < 0 || tables->max_blocks < 0 || num_pool_blocks < 0 || total_q < 0 || max_q < 0)
        return GF_ERR_BAD_SHAPE;
    if (params->num_kv_heads <= 0 || params->head_dim <= 0) return GF_ERR_BAD_SHAPE;
    if (params->block_size != gf::kBlock) return GF_ERR_UNSUPPORTED;
    if (params->head_dim != 64 && params->head_dim != 128) return GF_ERR_UNSUPPORTED;
    if (params->kv_dtype != GF_BF16 && params->kv_dtype != GF_FP8_E4M3) return GF_ERR_UNSUPPORTED;
    if ((int64_t)num_pool_blocks * params->num_kv_heads > 0x7fffffffLL) return GF_ERR_UNSUPPORTED;
    if (tables->num_req == 0 || total_q == 0) return GF_OK;
    if (!k_pool || !v_pool || !k_new || !v_new || !q_ptr) return GF_ERR_NULL;
    if (!tables->block_table || !tables->num_blocks || !tables->ctx_lens || !tables->seq_lens) return GF_ERR_NULL;
    if (params->kv_dtype == GF_FP8_E4M3 && (!k_scale || !v_scale)) return GF_ERR_NULL;
    if (tables->max_blocks < 1 || num_pool_blocks < 1) return GF_ERR_BAD_SHAPE;
    hipError_t e = gf::launch_append(k_pool, v_pool, k_scale, v_scale, num_pool_blocks, params->num_kv_heads,
                                     params->head_dim, params->kv_dtype, *tables, k_new, v_new, q_ptr, total_q,
                                     max_q, (hipStream_t)stream);
    if (e == hipErrorNotSupported || e == hipErrorInvalidValue) return GF_ERR_UNSUPPORTED;
    if (e != hipSuccess) return fail_hip(ctx, e, "gf_kv_append launch");
    return GF_OK;
}

int32_t gf_kv_append_token(gf_ctx *ctx, const gf_attn_params *params, void *k_pool, void *v_pool, float *k_scale,
                           float *v_scale, int32_t num_pool_blocks, const gf_tables *tables, const void *k_tok,
                           const void *v_tok, void *stream) {
    if (!ctx || !params || !tables) return GF_ERR_NULL;
    if (tables->num_req < 0 || tables->max_blocks < 0 || num_pool_blocks < 0) return GF_ERR_BAD_SHAPE;
    if (params->num_kv_heads <= 0 || params->head_dim <= 0) return GF_ERR_BAD_SHAPE;
    if (params->block_size != gf::kBlock) return GF_ERR_UNSUPPORTED;
    if (params->head_dim != 64 && params->head_dim != 128) return GF_ERR_UNSUPPORTED;
    if (params->kv_dtype != GF_BF16 && params->kv_dtype != GF_FP8_E4M3) return GF_ERR_UNSUPPORTED;
    if ((int64_t)num_pool_blocks * params->num_kv_heads > 0x7fffffffLL) return GF_ERR_UNSUPPORTED;
    if (tables->num_req == 0) return GF_OK;
    if (!k_pool || !v_pool || !k_tok || !v_tok) return GF_ERR_NULL;
    if (!tables->block_table || !tables->num_blocks || !tables->ctx_lens || !tables->seq_lens) return GF_ERR_NULL;
    if (params->kv_dtype == GF_FP8_E4M3 && (!k_scale || !v_scale)) return GF_ERR_NULL;
    if (tables->max_blocks < 1 || num_pool_blocks < 1) return GF_ERR_BAD_SHAPE;
    hipError_t e = gf::launch_append_token(k_pool, v_pool, k_scale, v_scale, num_pool_blocks, params->num_kv_heads,
                                           params->head_dim, params->kv_dtype, *tables, k_tok, v_tok,
                                           (hipStream_t)stream);
    if (e == hipErrorNotSupported) return GF_ERR_UNSUPPORTED;
    if (e != hipSuccess) return fail_hip(ctx, e, "gf_kv_append_token launch");
    return GF_OK;
}

}  // extern "C"
