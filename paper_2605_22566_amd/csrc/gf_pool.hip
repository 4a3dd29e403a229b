// gf_block_pool: host-side owner of the physical block ids of a K/V pool (paper, Topology-Aware State
// Management: a node's KV is stored once and shared by every workflow through it; Effective Path Pruning: storage
// follows the working set).  Free list + reference counts: a block is handed out with one reference; sharing it
// (a second workflow through the node, a request in flight that must not lose its blocks) adds references;
// dropping the last one returns the block to the free list.  Host code only: the pool tensors stay the caller's.
#include <mutex>
#include <new>
#include <vector>

#include "gf_internal.h"

struct gf_block_pool {
    std::mutex mu;
    std::vector<int32_t> refs;        // per block
    std::vector<int32_t> free_list;   // stack of free ids (lowest ids on top at creation)
    int64_t total_refs = 0;
    int32_t peak_in_use = 0;
};

extern "C" {

int32_t gf_block_pool_create(gf_block_pool **out, int32_t num_blocks) {
    if (!out) return GF_ERR_NULL;
    *out = nullptr;
    if (num_blocks < 0) return GF_ERR_BAD_SHAPE;
    gf_block_pool *p = new (std::nothrow) gf_block_pool();
    if (!p) return GF_ERR_WORKSPACE;
    try {
        p->refs.assign((size_t)num_blocks, 0);
        p->free_list.resize((size_t)num_blocks);
    } catch (const std::bad_alloc &) {
        delete p;
        return GF_ERR_WORKSPACE;
    }
    for (int32_t i = 0; i < num_blocks; ++i) p->free_list[(size_t)i] = num_blocks - 1 - i;
    *out = p;
    return GF_OK;
}

int32_t gf_block_pool_destroy(gf_block_pool *pool) {
    if (!pool) return GF_ERR_NULL;
    delete pool;
    return GF_OK;
}

int32_t gf_block_pool_alloc(gf_block_pool *pool, int32_t n, int32_t *ids) {
    if (!pool) return GF_ERR_NULL;
    if (n < 0) return GF_ERR_BAD_SHAPE;
    if (n == 0) return GF_OK;
    if (!ids) return GF_ERR_NULL;
    std::lock_guard<std::mutex> lock(pool->mu);
    if ((size_t)n > pool->free_list.size()) return GF_ERR_WORKSPACE;      // all or nothing
    for (int32_t i = 0; i < n; ++i) {
        const int32_t b = pool->free_list.back();
        pool->free_list.pop_back();
        pool->refs[(size_t)b] = 1;
        ids[i] = b;
    }
    pool->total_refs += n;
    const int32_t in_use = (int32_t)(pool->refs.size() - pool->free_list.size());
    if (in_use > pool->peak_in_use) pool->peak_in_use = in_use;
    return GF_OK;
}

// ids outside the pool, or blocks that are not allocated, make the whole call fail before anything changes
static int32_t check_live(const gf_block_pool *pool, int32_t n, const int32_t *ids) {
    for (int32_t i = 0; i < n; ++i) {
        const int32_t b = ids[i];
        if (b < 0 || (size_t)b >= pool->refs.size() || pool->refs[(size_t)b] <= 0) return GF_ERR_BAD_SHAPE;
    }
    return GF_OK;
}

int32_t gf_block_pool_retain(gf_block_pool *pool, int32_t n, const int32_t *ids) {
    if (!pool) return GF_ERR_NULL;
    if (n < 0) return GF_ERR_BAD_SHAPE;
    if (n == 0) return GF_OK;
    if (!ids) return GF_ERR_NULL;
    std::lock_guard<std::mutex> lock(pool->mu);
    const int32_t rc = check_live(pool, n, ids);
    if (rc != GF_OK) return rc;
    for (int32_t i = 0; i < n; ++i) ++pool->refs[(size_t)ids[i]];
    pool->total_refs += n;
    return GF_OK;
}

int32_t gf_block_pool_release(gf_block_pool *pool, int32_t n, const int32_t *ids, int32_t *num_freed) {
    if (!pool) return GF_ERR_NULL;
    if (n < 0) return GF_ERR_BAD_SHAPE;
    if (num_freed) *num_freed = 0;
    if (n == 0) return GF_OK;
    if (!ids) return GF_ERR_NULL;
    std::lock_guard<std::mutex> lock(pool->mu);
    // a block may be named several times in one call: it needs that many references
    {
        std::vector<int32_t> need;
        try {
            need.assign(pool->refs.size(), 0);
        } catch (const std::bad_alloc &) {
            return GF_ERR_WORKSPACE;
        }
        for (int32_t i = 0; i < n; ++i) {
            const int32_t b = ids[i];
            if (b < 0 || (size_t)b >= pool->refs.size()) return GF_ERR_BAD_SHAPE;
            if (++need[(size_t)b] > pool->refs[(size_t)b]) return GF_ERR_BAD_SHAPE;
        }
    }
    int32_t freed = 0;
    for (int32_t i = 0; i < n; ++i) {
        const int32_t b = ids[i];
        if (--pool->refs[(size_t)b] == 0) {
            pool->free_list.push_back(b);
            ++freed;
        }
    }
    pool->total_refs -= n;
    if (num_freed) *num_freed = freed;
    return GF_OK;
}

int32_t gf_block_pool_stats(gf_block_pool *pool, int32_t *num_free, int32_t *num_in_use, int64_t *total_refs,
                            int32_t *peak_in_use) {
    if (!pool) return GF_ERR_NULL;
    std::lock_guard<std::mutex> lock(pool->mu);
    if (num_free) *num_free = (int32_t)pool->free_list.size();
    if (num_in_use) *num_in_use = (int32_t)(pool->refs.size() - pool->free_list.size());
    if (total_refs) *total_refs = pool->total_refs;
    if (peak_in_use) *peak_in_use = pool->peak_in_use;
    return GF_OK;
}

int32_t gf_block_pool_refcount(gf_block_pool *pool, int32_t block) {
    if (!pool) return GF_ERR_NULL;
    std::lock_guard<std::mutex> lock(pool->mu);
    if (block < 0 || (size_t)block >= pool->refs.size()) return GF_ERR_BAD_SHAPE;
    return pool->refs[(size_t)block];
}

}  // extern "C"
