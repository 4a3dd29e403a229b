// gf_attn_prefill: the new tokens of each request attend to the KV of the
// ancestor nodes on its path (shared, read through the block table) and,
// causally, to each other (paper, Topology-Aware State Management: assembling
// a workflow's KV from its nodes "without repeated prefill"; also the
// on-the-fly fallback of Effective Path Pruning).
//
// MFMA path.  One workgroup owns (request, kv head, tile of BM new tokens) and
// all G query heads of the group: BM*G score rows share every K/V tile that is
// staged through LDS, so each byte fetched feeds G times the flops.  Each wave
// owns MT 32-row tiles (one query head, 32 tokens).  Scores are computed
// transposed so the softmax statistics of a row live in one lane pair:
//   S^T[key][row]  = K[key][d]   * Q^T[d][row]      (A = K from LDS, B = Q regs)
//   O^T[d][row]   += V^T[d][key] * P^T[key][row]    (A = V^T from LDS, B = P regs)
// with v_mfma_f32_32x32x16_bf16: operand lane l holds row/col l%32 and the 8
// contraction elements of half l/32; accumulator lane l holds column l%32 and
// rows 8*(i/4) + 4*(l/32) + i%4.  K rows are fetched in the order "row m reads
// key m with bits 2 and 3 swapped", which makes accumulator registers 8c..8c+7
// of a lane the 8 consecutive slots 8*(l/32)..+7 of 16-key chunk c -- exactly
// the contraction group the V^T operand reads as one 16-byte LDS load from the
// pool's [d][slot] V layout.  P never leaves registers.
//
// KV tiles are 64 keys (4 table entries); per-entry token counts mask partial
// blocks anywhere in the sequence, and tail entries are masked causally.
#include "gf_internal.h"

namespace gf {

template <int D, int G, int NW, int MT>
struct PrefillCfg {
    static constexpr int kThreads = NW * 64;
    static constexpr int kRows = 32 * NW * MT;       // score rows per workgroup
    static constexpr int kBM = kRows / G;            // new tokens per workgroup
    static constexpr int kBN = 64;                   // keys per KV tile
    static constexpr int kEntries = kBN / kBlock;    // table entries per tile (4)
    static constexpr int kKStride = D * 2 + 16;      // padded K row in LDS (bytes)
    static constexpr int kKTile = kBN * kKStride;
    static constexpr int kVBlk = D * kBlock * 2;     // one V block in LDS (bytes)
    static constexpr int kVTile = kEntries * kVBlk;
    static constexpr int kStage = kKTile + kVTile;
    static constexpr int kLds = 2 * kStage;
    static constexpr int kChunks = kEntries * 2 * D; // 16-byte chunks per tensor per tile
    static constexpr int kLoads = kChunks / kThreads;  // per thread per tensor
    static_assert(kRows % G == 0 && (NW * MT) % G == 0, "row tiles must split evenly over heads");
    static_assert(kChunks % kThreads == 0, "staging must divide evenly");
    static_assert((2 * D) % 64 == 0, "a wave must stay inside one block while staging");
};

template <int D, int G, int NW, int MT, bool FP8>
__global__ __launch_bounds__(NW * 64) void prefill_kernel(AttnArgs a, const int32_t *__restrict__ q_ptr,
                                                          int q_tiles, int total_q) {
    using C = PrefillCfg<D, G, NW, MT>;
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 31, hh = lane >> 5;

    // work item: q tile fastest, then kv head, then request
    const int qt = blockIdx.x % q_tiles;
    const int rk = blockIdx.x / q_tiles;
    const int kvh = rk % a.hkv;
    const int r = rk / a.hkv;
    if (a.status && a.status[r] != 0) return;
    const int ctx = a.ctx_lens[r];
    const int n_new = a.seq_lens[r] - ctx;
    const int i0 = qt * C::kBM;
    if (i0 >= n_new) return;
    const int q0 = q_ptr[r];
    // a request whose query rows do not match its table is skipped, never read out of bounds
    if (q_ptr[r + 1] - q0 != n_new || q0 < 0 || q0 + n_new > total_q) return;
    const int nb = min(a.num_blocks[r], a.max_blocks);
    const int ncb = max(nb - (n_new + kBlock - 1) / kBlock, 0);  // context entries
    const int rows_end = min(n_new, i0 + C::kBM);
    const int e_end = min(nb, ncb + (rows_end + kBlock - 1) / kBlock);
    const int ntiles = (e_end + C::kEntries - 1) / C::kEntries;
    const int32_t *tab = a.block_table + (size_t)r * a.max_blocks;
    const int32_t *ntk = a.block_ntok + (size_t)r * a.max_blocks;

    // ---- Q^T operand fragments (registers, whole kernel) ----------------------
    bf16x8 qf[MT][D / 16];
    int row_tok[MT];
    int row_head[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int tile = wave * MT + mt;
        const int g = tile % G, tt = tile / G;
        const int tok = i0 + 32 * tt + m;
        row_tok[mt] = tok;
        row_head[mt] = kvh * G + g;
        const int tokc = min(tok, n_new - 1);
        const char *qp = (const char *)a.q + (((size_t)(q0 + tokc)) * a.hq + row_head[mt]) * (D * 2);
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks)
            qf[mt][ks] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(qp + (16 * ks + 8 * hh) * 2));
    }

    // ---- staging helpers ----------------------------------------------------------
    u32x4 kst[C::kLoads], vst[C::kLoads];
    const size_t blk_bytes = (size_t)kBlock * D * 2;
    auto issue_loads = [&](int tile) {
        const int e = tile * C::kEntries;
#pragma unroll
        for (int i = 0; i < C::kLoads; ++i) {
            const int u = tid + i * C::kThreads;
            const int cb = __builtin_amdgcn_readfirstlane(u / (2 * D));   // entry within the tile
            const int within = u % (2 * D);
            int bid = (e + cb < e_end) ? tab[e + cb] : 0;
            bid = min(max(bid, 0), a.pool_blocks - 1);
            const size_t off = ((size_t)bid * a.hkv + kvh) * blk_bytes + (size_t)within * 16;
            kst[i] = *(const u32x4 *)((const char *)a.k + off);
            vst[i] = *(const u32x4 *)((const char *)a.v + off);
        }
    };
    auto store_stage = [&](int buf) {
        char *base = lds + buf * C::kStage;
#pragma unroll
        for (int i = 0; i < C::kLoads; ++i) {
            const int u = tid + i * C::kThreads;
            const int cb = u / (2 * D);
            const int within = u % (2 * D);
            const int slot = within / (D / 8), dch = within % (D / 8);
            *(u32x4 *)(base + (kBlock * cb + slot) * C::kKStride + dch * 16) = kst[i];
            const int d = within >> 1, hv = within & 1;
            *(u32x4 *)(base + C::kKTile + cb * C::kVBlk + hv * (D * 16) + d * 16) = vst[i];
        }
    };

    // ---- running state --------------------------------------------------------------
    const float c = a.scale_log2;
    float m_run[MT], l_run[MT];
    f32x16 o[MT][D / 32];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        m_run[mt] = -1.0e30f;
        l_run[mt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[mt][dt][i] = 0.f;
    }

    // K operand row m reads key (m with bits 2,3 swapped)
    const int krow = (m & 0x13) | ((m & 4) << 1) | ((m & 8) >> 1);
    const int k_lane_off = krow * C::kKStride + 8 * hh * 2;
    const int v_lane_off = C::kKTile + hh * (D * 16) + m * 16;

    issue_loads(0);
    store_stage(0);
    __syncthreads();

    for (int t = 0; t < ntiles; ++t) {
        const int buf = t & 1;
        const bool more = t + 1 < ntiles;
        if (more) issue_loads(t + 1);
        const char *sb = lds + buf * C::kStage;
        const int e = t * C::kEntries;

        // ---- S^T = K Q^T ----------------------------------------------------------
        f32x16 s[MT][2];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int i = 0; i < 16; ++i) s[mt][kt][i] = 0.f;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) {
                const bf16x8 kf = __builtin_bit_cast(
                    bf16x8, *(const u32x4 *)(sb + k_lane_off + 32 * kt * C::kKStride + 16 * ks * 2));
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    s[mt][kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[mt][ks], s[mt][kt], 0, 0, 0);
            }

        // ---- masks: partial blocks and the causal tail -------------------------------
#pragma unroll
        for (int cb = 0; cb < C::kEntries; ++cb) {
            const int ent = e + cb;
            const int nt = ent < e_end ? ntk[ent] : 0;
            const bool tail = ent >= ncb;
            if (nt < kBlock || tail) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    int lim = nt;
                    if (tail) lim = min(lim, row_tok[mt] - (ent - ncb) * kBlock + 1);
                    lim -= 8 * hh;
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (j >= lim) s[mt][cb >> 1][8 * (cb & 1) + j] = -INFINITY;
                }
            }
        }

        // ---- online softmax (fp32), P -> bf16 operand fragments ----------------------
        bf16x8 pf[MT][C::kEntries];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            float mx = s[mt][0][0];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[mt][kt][i]);
            mx = fmaxf(mx, other_half(mx));
            const float m_new = fmaxf(m_run[mt], mx);
            const float alpha = fast_exp2((m_run[mt] - m_new) * c);
            const float mc = m_new * c;
            m_run[mt] = m_new;
            float psum = 0.f;
#pragma unroll
            for (int cb = 0; cb < C::kEntries; ++cb) {
                f32x8 p;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    p[j] = fast_exp2(s[mt][cb >> 1][8 * (cb & 1) + j] * c - mc);
                    psum += p[j];
                }
                pf[mt][cb] = __builtin_convertvector(p, bf16x8);
            }
            l_run[mt] = l_run[mt] * alpha + psum;
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt) o[mt][dt] *= alpha;
        }

        // ---- O^T += V^T P^T ------------------------------------------------------------
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
            for (int cb = 0; cb < C::kEntries; ++cb) {
                const bf16x8 vf = __builtin_bit_cast(
                    bf16x8, *(const u32x4 *)(sb + v_lane_off + cb * C::kVBlk + 32 * dt * 16));
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    o[mt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[mt][cb], o[mt][dt], 0, 0, 0);
            }

        if (more) store_stage(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: normalise, round to bf16, store ------------------------------------
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const float l_tot = l_run[mt] + other_half(l_run[mt]);
        const int tok = row_tok[mt];
        if (tok < n_new) {
            const float inv = 1.f / l_tot;
            char *op = (char *)a.o + (((size_t)(q0 + tok)) * a.hq + row_head[mt]) * (D * 2);
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    f32x4 v4 = {o[mt][dt][4 * q] * inv, o[mt][dt][4 * q + 1] * inv, o[mt][dt][4 * q + 2] * inv,
                                o[mt][dt][4 * q + 3] * inv};
                    const bf16x4 b4 = __builtin_convertvector(v4, bf16x4);
                    *(bf16x4 *)(op + (32 * dt + 8 * q + 4 * hh) * 2) = b4;
                }
            if (a.lse && hh == 0)
                a.lse[(size_t)(q0 + tok) * a.hq + row_head[mt]] =
                    (m_run[mt] * c + __builtin_log2f(l_tot)) * 0.6931471805599453f;
        }
    }
}

template <int D, int G, int NW, int MT>
static hipError_t launch_prefill_t(const AttnArgs &a, int kv_dtype, const int32_t *q_ptr, int32_t total_q,
                                   int32_t max_q, hipStream_t s) {
    using C = PrefillCfg<D, G, NW, MT>;
    if (kv_dtype != GF_BF16) return hipErrorNotSupported;
    auto kern = prefill_kernel<D, G, NW, MT, false>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, C::kLds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int q_tiles = (max_q + C::kBM - 1) / C::kBM;
    const size_t grid = (size_t)a.num_req * a.hkv * q_tiles;
    if (grid == 0) return hipSuccess;
    if (grid > 0x7fffffffu) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(C::kThreads), C::kLds, s, a, q_ptr, q_tiles, total_q);
    return hipGetLastError();
}

hipError_t launch_prefill(const AttnArgs &a, int head_dim, int group, int kv_dtype, const int32_t *q_ptr,
                          int32_t total_q, int32_t max_q, hipStream_t s) {
    if (a.num_req == 0 || total_q == 0 || max_q == 0) return hipSuccess;
#define GF_CASE(DD, GG) \
    if (head_dim == DD && group == GG) return launch_prefill_t<DD, GG, 8, 1>(a, kv_dtype, q_ptr, total_q, max_q, s);
    GF_CASE(64, 1) GF_CASE(64, 2) GF_CASE(64, 4) GF_CASE(64, 8)
    GF_CASE(128, 1) GF_CASE(128, 2) GF_CASE(128, 4) GF_CASE(128, 8)
#undef GF_CASE
    return hipErrorNotSupported;
}

}  // namespace gf
