// gf_attn_decode: one query token per request attends to the whole KV of its
// node path through the block table (paper, Topology-Aware State Management:
// decode steps reuse the per-node KV instead of recomputing past context).
//
// Bandwidth path.  The table of a request is cut into chunks of `chunk_blocks`
// entries; one wavefront reduces one (request, kv head, chunk) item for all G
// query heads of the group at once, streaming K and V blocks straight from HBM
// into MFMA operand registers (16 B per lane, two blocks = 32 keys per step,
// the next step's loads in flight while the current one is reduced), and
// leaves an fp32 partial (max, sum, weighted values).  A second kernel merges
// the partials of a request with the log-sum-exp rule and rounds to bf16.
//
// MFMA use (v_mfma_f32_16x16x32_bf16, D = A(16x32) * B(32x16)):
//   S^T[key][head]  = K[key][d]   * Q^T[d][head]       (A = K rows, B = Q)
//   O^T[d][head]   += V^T[d][key] * P^T[key][head]     (A = V^T rows, B = P)
// Lane l holds operand row/col l%16 and the 8 contraction elements of group
// l/16; an accumulator lane holds column l%16, rows 4*(l/16)+i.  The K rows of
// the two score tiles are chosen so that after both tiles lane group q4 holds
// the 8 consecutive slots 8*(q4%2)..+7 of block q4/2: exactly the contraction
// group the V^T operand reads as one 16-byte load from the [d][slot] V layout.
#include "gf_internal.h"
#include "gf_decode_frag.h"

namespace gf {

constexpr int kDecodeThreads = 256;          // 4 independent waves
constexpr int kWavesPerWg = kDecodeThreads / 64;

// RES: table entries may carry a residual handle (ResidualRefs); a pair with one is patched in the wave's LDS
// image before it is reduced (patch_pair), every other pair takes the plain path.
template <int D, int G, bool FP8, bool RES = false>
__global__ __launch_bounds__(kDecodeThreads, RES ? 2 : 1) void decode_split_kernel(AttnArgs a, int chunk_blocks, int splits,
                                                                     float *__restrict__ part_o,
                                                                     float *__restrict__ part_ml,
                                                                     ResidualRefs rr = ResidualRefs{}) {
    static_assert(!(RES && FP8), "residuals are applied on the fly to bf16 pools only");
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int pairs = a.num_req * a.hkv;
    const long item = (long)blockIdx.x * kWavesPerWg + wave;
    if (item >= (long)pairs * splits) return;
    const int s = (int)(item / pairs);
    const int rem = (int)(item % pairs);
    const int r = rem / a.hkv, kvh = rem % a.hkv;
    if (a.status && a.status[r] != 0) return;
    const int nb = min(a.num_blocks[r], a.max_blocks);
    const int e0 = s * chunk_blocks;
    const int e1 = min(nb, e0 + chunk_blocks);
    if (e0 >= e1) return;
    const int32_t *tab = a.block_table + (size_t)r * a.max_blocks;
    const int32_t *ntk = a.block_ntok + (size_t)r * a.max_blocks;

    const int n = lane & 15, q4 = lane >> 4;
    // Q^T operand: column n = query head of the group (zero beyond G)
    bf16x8 qf[D / 32];
#pragma unroll
    for (int t = 0; t < D / 32; ++t) {
        u32x4 raw = {0, 0, 0, 0};
        // contraction elements of lane group q4 in step t (the e4m3 path pairs steps, see PairRegs)
        const int d0 = FP8 ? 64 * (t / 2) + 16 * q4 + 8 * (t % 2) : 32 * t + 8 * q4;
        if (n < G)
            raw = *(const u32x4 *)((const char *)a.q + (((size_t)r * a.hq + kvh * G + n) * D + d0) * 2);
        qf[t] = __builtin_bit_cast(bf16x8, raw);
    }

    const float c = a.scale_log2;
    const float slack = 8.f / c;     // 2^8 in the exponent, in score units (inf for a zero scale)
    float m_run = -1.0e30f;   // reference max of raw scores (finite sentinel)
    float l_run = 0.f;        // lane-local partial sum of exp
    f32x4 oacc[D / 16];
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) oacc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // residual handles of the pair in `cur` / `nxt` (-1: none, also for ids outside the CSR)
    const int32_t *rh = RES ? rr.handle + (size_t)r * a.max_blocks : nullptr;
    auto handle_of = [&](int e) -> int {
        if (e >= e1) return -1;
        const int h = rh[e];
        return h >= 0 && h < rr.num_items ? h : -1;
    };
    // ... and the entry ranges of the four CSR rows of a pair (empty without a residual), fetched two pairs ahead,
    // so that the K rows of the next pair can be requested while the current pair is reduced
    auto load_rows = [&](int e, int *out) {
        row_ranges(rr, handle_of(e), kvh, a.hkv, out);
        row_ranges(rr, handle_of(e + 1), kvh, a.hkv, out + 4);
    };
    auto rows_any = [](const int *x) {
        return (x[1] - x[0]) + (x[3] - x[2]) + (x[5] - x[4]) + (x[7] - x[6]) > 0;
    };
    int rows[8] = {0, 0, 0, 0, 0, 0, 0, 0}, rows_n[8] = {0, 0, 0, 0, 0, 0, 0, 0}, rows_nn[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    RowLoad<D, 1> krow0, krow1;
    if constexpr (RES) {
        load_rows(e0, rows);
        load_rows(e0 + 2, rows_n);
        krow0.issue(rr, rows[0], rows[1], lane);
        krow1.issue(rr, rows[4], rows[5], lane);
    }

    PairRegs<D, FP8> cur, nxt;
    load_pair(cur, a, tab, ntk, e0, e1, kvh, lane);
    for (int e = e0; e < e1; e += 2) {
        const bool more = e + 2 < e1;
        if (more) load_pair(nxt, a, tab, ntk, e + 2, e1, kvh, lane);
        if constexpr (RES) {
            load_rows(e + 4, rows_nn);
            if (rows_any(rows)) {
                __shared__ __attribute__((aligned(16))) uint16_t patch_img[kWavesPerWg][2 * kBlock * D + kPatchSpare];
                patch_pair<D>(cur, patch_img[wave], rr, rows, krow0, krow1, lane);
            }
            krow0.issue(rr, rows_n[0], rows_n[1], lane);      // empty rows (no residual, or no next pair): no loads
            krow1.issue(rr, rows_n[4], rows_n[5], lane);
        }

        f32x4 sT[2];
#pragma unroll
        for (int T = 0; T < 2; ++T) {
            sT[T] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < D / 32; ++t)
                sT[T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k_operand<D, FP8>(cur, T, t), qf[t], sT[T], 0, 0, 0);
            if constexpr (FP8) sT[T] *= cur.ks;      // scores of this lane's keys, in the block's K scale
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
        // m_run is the reference the exponentials are taken against, the same in the four lanes of a column, not
        // the exact running maximum: it moves (and sum and values are rescaled) only when some score outgrows it
        // by more than 2^8 in the exponent, so most steps need neither the cross-lane maximum nor the rescaling
        if (__builtin_amdgcn_ballot_w64(mx > m_run + slack) != 0) {
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run, mx);
            const float alpha = fast_exp2((m_run - m_new) * c);
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int dt = 0; dt < D / 16; ++dt) oacc[dt] *= alpha;
        }
        const float mc = m_run * c;
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
        l_run += psum;
        if constexpr (FP8) p *= cur.vs;              // V scale of this lane's keys rides on P; the row sum does not
        const bf16x8 pb = __builtin_convertvector(p, bf16x8);
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) {
            oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(v_operand<D, FP8>(cur, dt), pb, oacc[dt], 0, 0, 0);
        }
        if (more) cur = nxt;
        if constexpr (RES) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                rows[i] = rows_n[i];
                rows_n[i] = rows_nn[i];
            }
        }
    }

    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);
    if (n < G) {
        const size_t pi = ((size_t)rem * splits + s) * G + n;
        if (q4 == 0) {
            part_ml[pi * 2 + 0] = m_run * c;   // max in log2 units
            part_ml[pi * 2 + 1] = l_run;
        }
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) *(f32x4 *)(part_o + pi * D + 16 * dt + 4 * q4) = oacc[dt];
    }
}

// One wave per (request, query head): combine the partials of the request's
// chunks.  m_s are in log2 units: w_s = 2^(m_s - M), L = sum w_s l_s,
// O = sum w_s O_s / L, lse = (M + log2 L) * ln 2.  Lanes first work chunk-parallel
// (maximum, weights), then each lane owns D/64 output elements, the weights go
// round by v_readlane and four chunks' loads are in flight together.
template <int D, int G>
__global__ __launch_bounds__(256) void decode_merge_kernel(AttnArgs a, int chunk_blocks, int splits,
                                                           const float *__restrict__ part_o,
                                                           const float *__restrict__ part_ml) {
    const int lane = threadIdx.x & 63;
    const long idx = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (idx >= (long)a.num_req * a.hq) return;
    const int r = (int)(idx / a.hq), h = (int)(idx % a.hq);
    const int kvh = h / G, g = h % G;
    const bool ok = !(a.status && a.status[r] != 0);
    const int nb = ok ? min(a.num_blocks[r], a.max_blocks) : 0;
    const int ns = (nb + chunk_blocks - 1) / chunk_blocks;
    __bf16 *out = (__bf16 *)a.o + ((size_t)r * a.hq + h) * D;
    constexpr int PER = D / 64;
    float acc[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) acc[i] = 0.f;
    float M = -INFINITY, L = 0.f;
    const size_t base = ((size_t)(r * a.hkv + kvh) * splits) * G + g;     // chunk s sits at base + s * G
    for (int s0 = 0; s0 < ns; s0 += 64)
        if (s0 + lane < ns) M = fmaxf(M, part_ml[(base + (size_t)(s0 + lane) * G) * 2]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off, 64));
    for (int s0 = 0; s0 < ns; s0 += 64) {
        float wgt = 0.f;
        if (s0 + lane < ns) {
            const size_t pi = base + (size_t)(s0 + lane) * G;
            wgt = fast_exp2(part_ml[pi * 2] - M);
            L += wgt * part_ml[pi * 2 + 1];
        }
        const int m = min(64, ns - s0);
        for (int j0 = 0; j0 < m; j0 += 4) {
            float x[4][PER];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const size_t pj = base + (size_t)(s0 + min(j0 + u, m - 1)) * G;
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

size_t decode_workspace_bytes(int32_t num_req, int32_t hkv, int32_t group, int32_t head_dim, int32_t splits) {
    return (size_t)num_req * hkv * splits * group * (head_dim + 2) * sizeof(float);
}

template <int D, int G>
static hipError_t launch_decode_t(const AttnArgs &a, int kv_dtype, int32_t chunk_blocks, int32_t splits,
                                  void *workspace, hipStream_t s) {
    const size_t n_items = (size_t)a.num_req * a.hkv * splits;
    float *part_o = (float *)workspace;
    float *part_ml = part_o + n_items * G * D;
    const unsigned grid = (unsigned)((n_items + kWavesPerWg - 1) / kWavesPerWg);
    if (kv_dtype == GF_FP8_E4M3)
        hipLaunchKernelGGL((decode_split_kernel<D, G, true>), dim3(grid), dim3(kDecodeThreads), 0, s, a,
                           chunk_blocks, splits, part_o, part_ml);
    else
        hipLaunchKernelGGL((decode_split_kernel<D, G, false>), dim3(grid), dim3(kDecodeThreads), 0, s, a,
                           chunk_blocks, splits, part_o, part_ml);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t rows = (size_t)a.num_req * a.hq;
    hipLaunchKernelGGL((decode_merge_kernel<D, G>), dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, a,
                       chunk_blocks, splits, part_o, part_ml);
    return hipGetLastError();
}

template <int D, int G>
static hipError_t launch_decode_residual_t(const AttnArgs &a, const ResidualRefs &rr, int32_t chunk_blocks,
                                           int32_t splits, void *workspace, hipStream_t s) {
    const size_t n_items = (size_t)a.num_req * a.hkv * splits;
    float *part_o = (float *)workspace;
    float *part_ml = part_o + n_items * G * D;
    const unsigned grid = (unsigned)((n_items + kWavesPerWg - 1) / kWavesPerWg);
    hipLaunchKernelGGL((decode_split_kernel<D, G, false, true>), dim3(grid), dim3(kDecodeThreads), 0, s, a,
                       chunk_blocks, splits, part_o, part_ml, rr);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t rows = (size_t)a.num_req * a.hq;
    hipLaunchKernelGGL((decode_merge_kernel<D, G>), dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, a,
                       chunk_blocks, splits, part_o, part_ml);
    return hipGetLastError();
}

hipError_t launch_decode_residual(const AttnArgs &a, const ResidualRefs &rr, int head_dim, int group, int kv_dtype,
                                  int32_t chunk_blocks, int32_t splits, void *workspace, hipStream_t s) {
    if (kv_dtype != GF_BF16) return hipErrorNotSupported;
    if (a.num_req == 0) return hipSuccess;
#define GF_CASE(DD, GG) \
    if (head_dim == DD && group == GG) return launch_decode_residual_t<DD, GG>(a, rr, chunk_blocks, splits, workspace, s);
    GF_CASE(64, 1) GF_CASE(64, 2) GF_CASE(64, 4) GF_CASE(64, 8)
    GF_CASE(128, 1) GF_CASE(128, 2) GF_CASE(128, 4) GF_CASE(128, 8)
#undef GF_CASE
    return hipErrorNotSupported;
}

hipError_t launch_decode(const AttnArgs &a, int head_dim, int group, int kv_dtype, int32_t chunk_blocks,
                         int32_t splits, void *workspace, hipStream_t s) {
    if (a.num_req == 0) return hipSuccess;
#define GF_CASE(DD, GG) \
    if (head_dim == DD && group == GG) return launch_decode_t<DD, GG>(a, kv_dtype, chunk_blocks, splits, workspace, s);
    GF_CASE(64, 1) GF_CASE(64, 2) GF_CASE(64, 4) GF_CASE(64, 8)
    GF_CASE(128, 1) GF_CASE(128, 2) GF_CASE(128, 4) GF_CASE(128, 8)
#undef GF_CASE
    return hipErrorNotSupported;
}

}  // namespace gf
