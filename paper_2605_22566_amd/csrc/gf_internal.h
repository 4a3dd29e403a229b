// Internal declarations shared by the translation units of libgraphflow.
// Device helpers for gfx950 (wave64, MFMA) and the host-side launcher
// prototypes the C ABI entry points call.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "graphflow.h"

namespace gf {

constexpr int kBlock = 16;  // tokens per pool block

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct AttnArgs {
    const void *k, *v;
    const float *k_scale, *v_scale;
    int32_t pool_blocks;
    const int32_t *block_table, *block_ntok, *num_blocks, *ctx_lens, *seq_lens, *status;
    int32_t num_req, max_blocks;
    int32_t hq, hkv;
    float scale_log2;  // sm_scale * log2(e)
    const void *q;
    void *o;
    float *lse;
};

// Sparse residuals applied while a decode step streams the pool (same CSR as gf_kv_apply_residual): table entry
// (request, e) with handle[request * max_blocks + e] = b in [0, num_items) is read as base block + residual item b.
struct ResidualRefs {
    const int32_t *handle;
    const int32_t *ptr;
    const uint16_t *idx, *val;
    int32_t num_items;
};

// launchers (return hipError_t of the launch)
hipError_t launch_resolve(const gf_graph &g, int32_t num_req, const int32_t *path_ptr,
                          const int32_t *path_nodes, const int32_t *new_lens, const int32_t *tail_ptr,
                          const int32_t *tail_blocks, int32_t max_blocks, int32_t num_pool_blocks,
                          int32_t *block_table, int32_t *block_ntok, int32_t *num_blocks,
                          int32_t *ctx_lens, int32_t *seq_lens, int32_t *status, hipStream_t s);

// bytes of the work-list buffer a prefill call needs, and the launcher (plan kernel + attention kernel)
size_t prefill_plan_bytes(int32_t total_q, int32_t num_req, int group);
// `rr`: residual items read in place (bf16 pools), or nullptr for the plain call
hipError_t launch_prefill(const AttnArgs &a, int head_dim, int group, int kv_dtype, const int32_t *q_ptr,
                          int32_t total_q, int32_t *plan, const ResidualRefs *rr, hipStream_t s);

// The work list of gf_attn_prefill_noalloc: a file-scope device array of kStaticPlanBytes instead of a buffer
// of the context.  prefill_static_plan_init looks the array's address up once per device (that device must be
// current) and keeps it; prefill_static_plan returns the address kept for a device, or nullptr.
constexpr size_t kStaticPlanBytes = size_t(1) << 20;
hipError_t prefill_static_plan_init(int device);
int32_t *prefill_static_plan(int device);

// read-only streaming probe (bandwidth ceiling): bytes a multiple of 16, one sum per workgroup
hipError_t launch_hbm_read_probe(const void *src, size_t bytes, uint32_t *wg_sums, int32_t num_wg, hipStream_t s);
hipError_t launch_hbm_tile_probe(const void *src, int32_t tile_bytes, int32_t num_src_tiles, const int32_t *ids,
                                 int64_t num_tiles, uint32_t *wg_sums, int32_t num_wg, hipStream_t s);
// MFMA issue probe: operand_bytes a multiple of 1024, one float per lane of num_wg workgroups of 256 threads
hipError_t launch_mfma_probe(const void *operands, int64_t operand_bytes, int32_t iters, int32_t softmax_mix,
                             float *lane_sums, int32_t num_wg, hipStream_t s);

// built-in split-KV chunk sizes (table entries per work item) of gf_attn_decode and gf_attn_decode_residual
constexpr int32_t kDecodeChunkBlocks = 64, kDecodeChunkBlocksResidual = 64;   // equal: the two calls are interchangeable bit for bit

// workspace floats needed by decode for (num_req, hkv, group, head_dim, splits)
size_t decode_workspace_bytes(int32_t num_req, int32_t hkv, int32_t group, int32_t head_dim, int32_t splits);
hipError_t launch_decode(const AttnArgs &a, int head_dim, int group, int kv_dtype, int32_t chunk_blocks,
                         int32_t splits, void *workspace, hipStream_t s);
// the same step with residuals applied on the fly (bf16 pools; hipErrorNotSupported otherwise)
hipError_t launch_decode_residual(const AttnArgs &a, const ResidualRefs &rr, int head_dim, int group, int kv_dtype,
                                  int32_t chunk_blocks, int32_t splits, void *workspace, hipStream_t s);

// node-centric decode: workspace bytes and the launcher (list building + node, tail and merge kernels)
// (`num_items`: residual items the call may be given, 0 for the plain call)
size_t shared_workspace_bytes(int32_t num_nodes, int32_t num_items, int32_t num_req, int32_t num_entries,
                              int32_t max_blocks, int32_t chunk_blocks, int32_t hq, int32_t head_dim);
// `phases`: build the lists and item records, run attention + merge over them, or both; the two phases of one
// batch must be given the same workspace and the same sizes
constexpr int kSharedBuildLists = 1, kSharedAttend = 2;
hipError_t launch_decode_shared(const AttnArgs &a, int head_dim, int group, int kv_dtype, const gf_graph &g,
                                const int32_t *path_ptr, const int32_t *path_nodes, int32_t num_entries,
                                int32_t chunk_blocks, void *workspace, int phases, const ResidualRefs *rr,
                                hipStream_t s);

// state-management policy: residual directory, resolution with residual handles, statistics, pruning
uint64_t prefix_key_host(const int32_t *nodes, int32_t len);
hipError_t launch_dir_clear(const gf_residual_dir &d, hipStream_t s);
hipError_t launch_dir_insert(const gf_residual_dir &d, int32_t num_pairs, const uint64_t *keys, const int32_t *prev,
                             const int32_t *node, const int32_t *first_item, int32_t *status, hipStream_t s);
hipError_t launch_resolve_residual(const gf_graph &g, int32_t num_req, const int32_t *path_ptr, const int32_t *path_nodes,
                                   const int32_t *status, int32_t max_blocks, const gf_residual_dir &d,
                                   int32_t *trans_count, int32_t *res_handle, int32_t *num_fallback, hipStream_t s);
hipError_t launch_dir_prune(const gf_graph &g, const gf_residual_dir &d, const int32_t *trans_count, int32_t min_count,
                            int32_t *pruned, hipStream_t s);

// residual application: one workgroup per pool block
hipError_t launch_residual(void *k_pool, void *v_pool, float *k_scale, float *v_scale, int32_t num_pool_blocks,
                           int32_t hkv, int32_t head_dim, int kv_dtype, int32_t num_items, const int32_t *src_blocks,
                           const int32_t *dst_blocks, const int32_t *res_ptr, const uint16_t *res_idx,
                           const uint16_t *res_val, int32_t *status, hipStream_t s);
// the packed form of a residual (bit mask per image + values in element order): converters and reconstruction
hipError_t launch_residual_pack(int32_t hkv, int32_t head_dim, int32_t num_items, const int32_t *res_ptr,
                                const uint16_t *res_idx, const uint16_t *res_val, uint32_t *res_mask,
                                uint16_t *packed_val, int32_t *status, hipStream_t s);
hipError_t launch_residual_unpack(int32_t hkv, int32_t head_dim, int32_t num_items, const int32_t *res_ptr,
                                  const uint32_t *res_mask, uint16_t *res_idx, int32_t *status, hipStream_t s);
hipError_t launch_residual_packed(void *k_pool, void *v_pool, int32_t num_pool_blocks, int32_t hkv, int32_t head_dim,
                                  int32_t num_items, const int32_t *src_blocks, const int32_t *dst_blocks,
                                  const int32_t *res_ptr, const uint32_t *res_mask, const uint16_t *packed_val,
                                  int32_t *status, hipStream_t s);

// residual producer: dense prefix-conditioned blocks -> CSR by the energy rule (count, scan, fill); cut_keys is
// device scratch of make_residual_scratch_bytes() bytes (one 8-byte sort key per CSR row)
size_t make_residual_scratch_bytes(int32_t hkv, int32_t num_items);
hipError_t launch_make_residual(const void *k_pool, const void *v_pool, int32_t num_pool_blocks, int32_t hkv,
                                int32_t head_dim, int32_t num_items, const int32_t *base_blocks,
                                const int32_t *full_blocks, double share, int32_t capacity, int32_t *res_ptr,
                                uint16_t *res_idx, uint16_t *res_val, int32_t *status, void *cut_keys, hipStream_t s);

// KV write path: one workgroup per (request, tail block); max_q bounds the new tokens of a request
hipError_t launch_append(void *k_pool, void *v_pool, float *k_scale, float *v_scale, int32_t pool_blocks, int32_t hkv,
                         int32_t head_dim, int kv_dtype, const gf_tables &t, const void *k_new, const void *v_new,
                         const int32_t *q_ptr, int32_t total_q, int32_t max_q, hipStream_t s);

// decode-step KV write: one workgroup per request, its newest token into the last table entry's block
hipError_t launch_append_token(void *k_pool, void *v_pool, float *k_scale, float *v_scale, int32_t pool_blocks,
                               int32_t hkv, int32_t head_dim, int kv_dtype, const gf_tables &t, const void *k_tok,
                               const void *v_tok, hipStream_t s);

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// 8 OCP e4m3 bytes (two dwords, element j in byte j) -> 8 bf16, exact (every e4m3 value is a bf16 value)
__device__ __forceinline__ bf16x8 fp8x8_to_bf16x8(u32x2 w) {
    const bf16x2 a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[0], 1.0f, false);
    const bf16x2 b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[0], 1.0f, true);
    const bf16x2 c = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[1], 1.0f, false);
    const bf16x2 d = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[1], 1.0f, true);
    return bf16x8{a[0], a[1], b[0], b[1], c[0], c[1], d[0], d[1]};
}

// Orders the LDS accesses of a wave's lanes before and after this point: a wave-private LDS image is written
// with 16-byte stores, patched element by element by other lanes, and read back with 16-byte loads.  For the
// compiler a fence at wavefront scope (accesses of different types to the image must not pass each other); the
// hardware runs one wave's LDS operations in order.
__device__ __forceinline__ void wave_lds_order() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// 16-byte-per-lane global -> LDS direct load: lane l fetches the 16 bytes at base + off + IMM (uniform base in
// scalar registers, 32-bit lane offset) and writes LDS bytes [lds_dst + IMM + 16 l, +16): the instruction's
// immediate offset is added to both addresses, so one base and one M0 value serve all loads of an image.  Issued
// through inline assembly and waited for by hand (dma_wait<N>: at most N of this wave's vector memory operations
// still in flight; they complete in order), so that a kernel can keep several tiles in flight and wait for its
// own loads right before the barrier that publishes a tile; the compiler's own waits do not know these loads and
// can only over-wait.
typedef __attribute__((address_space(3))) void *lds_ptr_t;
template <int IMM = 0>
__device__ __forceinline__ void dma_load(const void *base, uint32_t off, void *lds_dst) {
    static_assert(IMM >= 0 && IMM < 4096, "immediate offset range of the instruction");
    const uint32_t dst = (uint32_t)(uintptr_t)(lds_ptr_t)lds_dst;
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %2, %1 offset:%3"
                 ::"s"(dst), "s"(base), "v"(off), "n"(IMM) : "memory", "m0");
}
template <int N = 0>
__device__ __forceinline__ void dma_wait() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// value held by the lane 32 away (the other half of the wave)
__device__ __forceinline__ float other_half(float x) { return __shfl_xor(x, 32, 64); }

}  // namespace gf
