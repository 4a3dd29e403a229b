// Operand fragments of the per-request decode kernel: two pool blocks (32 keys) of one kv head, loaded from
// HBM straight into the registers the 16x16x32 MFMAs read (see gf_decode.hip for the geometry), and the
// on-the-fly application of sparse residuals to such a pair.
#pragma once
#include "gf_internal.h"
#include "gf_residual_row.h"

namespace gf {

template <int D, bool FP8>
struct PairRegs {
    // K: 2 tiles x D/32 steps, V: D/16 tiles; each a 16-byte (bf16) fragment
    u32x4 k[2][D / 32];
    u32x4 v[D / 16];
    int n0, n1;   // valid tokens in the two blocks
};
template <int D>
struct PairRegs<D, true> {
    // e4m3 pool: this lane's K / V block scales ride along.  K is fetched 16 bytes at a time: the
    // contraction elements of lane group q4 in MFMA step t are d = 64 (t/2) + 16 q4 + 8 (t%2) .. +7
    // (Q uses the same assignment), so one load carries the operands of two steps and a wave-wide
    // load reads 64 contiguous bytes of every K row.  V fragments are 8 bytes (8 slots of one d row).
    u32x4 k[2][D / 64];
    u32x2 v[D / 16];
    float ks, vs;
    int n0, n1;
};

template <int D>
__device__ __forceinline__ void load_pair(PairRegs<D, false> &p, const AttnArgs &a, const int32_t *tab,
                                          const int32_t *ntk, int e, int e_end, int kvh, int lane) {
    int b0 = tab[e];
    p.n0 = ntk[e];
    int b1 = b0;
    p.n1 = 0;
    if (e + 1 < e_end) {
        b1 = tab[e + 1];
        p.n1 = ntk[e + 1];
    }
    b0 = min(max(b0, 0), a.pool_blocks - 1);
    b1 = min(max(b1, 0), a.pool_blocks - 1);
    const size_t blk_bytes = (size_t)kBlock * D * 2;
    const char *k0 = (const char *)a.k + ((size_t)b0 * a.hkv + kvh) * blk_bytes;
    const char *k1 = (const char *)a.k + ((size_t)b1 * a.hkv + kvh) * blk_bytes;
    const char *v0 = (const char *)a.v + ((size_t)b0 * a.hkv + kvh) * blk_bytes;
    const char *v1 = (const char *)a.v + ((size_t)b1 * a.hkv + kvh) * blk_bytes;
    const int m = lane & 15, q4 = lane >> 4;
    // K operand row m of tile T: block (m>=8), slot 8*((m/4)&1) + 4T + m%4
    const char *kb = (m >= 8) ? k1 : k0;
    const int slot0 = 8 * ((m >> 2) & 1) + (m & 3);
#pragma unroll
    for (int T = 0; T < 2; ++T)
#pragma unroll
        for (int t = 0; t < D / 32; ++t)
            p.k[T][t] = *(const u32x4 *)(kb + (size_t)(slot0 + 4 * T) * D * 2 + (32 * t + 8 * q4) * 2);
    // V^T operand row m (d = 16dt + m): block (q4>=2), slots 8*(q4&1)..+7
    const char *vb = (q4 >= 2) ? v1 : v0;
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt)
        p.v[dt] = *(const u32x4 *)(vb + (size_t)(16 * dt + m) * (kBlock * 2) + (q4 & 1) * 16);
}

// e4m3 pool: same operand geometry with one byte per element; the scales of the lane's block
// (K operand rows and score rows of lane group q4 belong to block q4/2) ride along.
template <int D>
__device__ __forceinline__ void load_pair(PairRegs<D, true> &p, const AttnArgs &a, const int32_t *tab,
                                          const int32_t *ntk, int e, int e_end, int kvh, int lane) {
    int b0 = tab[e];
    p.n0 = ntk[e];
    int b1 = b0;
    p.n1 = 0;
    if (e + 1 < e_end) {
        b1 = tab[e + 1];
        p.n1 = ntk[e + 1];
    }
    b0 = min(max(b0, 0), a.pool_blocks - 1);
    b1 = min(max(b1, 0), a.pool_blocks - 1);
    const size_t blk_bytes = (size_t)kBlock * D;
    const char *k0 = (const char *)a.k + ((size_t)b0 * a.hkv + kvh) * blk_bytes;
    const char *k1 = (const char *)a.k + ((size_t)b1 * a.hkv + kvh) * blk_bytes;
    const char *v0 = (const char *)a.v + ((size_t)b0 * a.hkv + kvh) * blk_bytes;
    const char *v1 = (const char *)a.v + ((size_t)b1 * a.hkv + kvh) * blk_bytes;
    const int m = lane & 15, q4 = lane >> 4;
    const char *kb = (m >= 8) ? k1 : k0;
    const int slot0 = 8 * ((m >> 2) & 1) + (m & 3);
#pragma unroll
    for (int T = 0; T < 2; ++T)
#pragma unroll
        for (int tp = 0; tp < D / 64; ++tp)
            p.k[T][tp] = *(const u32x4 *)(kb + (size_t)(slot0 + 4 * T) * D + (64 * tp + 16 * q4));
    const char *vb = (q4 >= 2) ? v1 : v0;
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt)
        p.v[dt] = *(const u32x2 *)(vb + (size_t)(16 * dt + m) * kBlock + (q4 & 1) * 8);
    p.ks = a.k_scale[(q4 >= 2) ? b1 : b0];
    p.vs = a.v_scale[(q4 >= 2) ? b1 : b0];
}

// Differential KV (paper, "Differential-based KV Cache", Eq. 7) applied to a loaded pair of a bf16 pool: the
// fragments go to the wave's LDS image `img` (2 * 16 * D elements: the two blocks back to back, and kPatchSpare
// spare elements behind them), the residual entries of the blocks that have one are added there -- fp32 sum
// rounded to bf16, the arithmetic of gf_kv_apply_residual, so the operands equal a reconstructed block bit for
// bit -- and the fragments are read back; first K, then V through the same image.  K rows keep the pool's
// [slot][d] order with the 16-byte pieces of a row XOR-ed by the slot (fragment stores and loads then spread
// over the banks); V keeps [d][slot].  Entries outside the image change nothing.
constexpr int kPatchSpare = 8;

// LDS element of logical element i = slot * D + d of an image: K keeps [slot][d] with the 16-byte pieces of a row
// XOR-ed by the slot, V is [d][slot].  An entry outside the image lands on `spare`, an element beside the images
// that nothing reads: no lane has to be switched off for it.
template <int D, int TENSOR>
__device__ __forceinline__ uint32_t patch_elem(uint32_t i, uint32_t spare) {
    const uint32_t slot = i / D, d = i % D;
    const uint32_t phys = TENSOR ? d * kBlock + slot : i ^ ((slot & (D / 8 - 1)) << 3);
    return i >= (uint32_t)(kBlock * D) ? spare : phys;
}
// Where a residual entry lands: a map takes the logical element of an entry to an element of the LDS image.
// This one is the wave-private image of the decode kernels, with its spare element.
template <int D, int TENSOR>
struct SpareMap {
    static constexpr bool kPredicated = false;     // every entry is written somewhere
    uint32_t spare;
    __device__ __forceinline__ uint32_t operator()(uint32_t i) const { return patch_elem<D, TENSOR>(i, spare); }
};
// `rows`: row_ranges of the pair's two blocks (8 values: K0, V0, K1, V1); k0, k1: the pair's two K rows, issued
// by the caller a pair ahead (a K row of the paper's density fits 512 entries, a V row 1024)
template <int D>
__device__ __forceinline__ void patch_pair(PairRegs<D, false> &p, uint16_t *img, const ResidualRefs &rr,
                                           const int *rows, RowLoad<D, 1> &k0, RowLoad<D, 1> &k1, int lane) {
    constexpr int kImg = kBlock * D;
    RowLoad<D, 2> v0, v1;
    const int m = lane & 15, q4 = lane >> 4;
    uint16_t *kimg = img + (m >= 8 ? kImg : 0);
    const int slot0 = 8 * ((m >> 2) & 1) + (m & 3);
#pragma unroll
    for (int T = 0; T < 2; ++T)
#pragma unroll
        for (int t = 0; t < D / 32; ++t) {
            const int slot = slot0 + 4 * T;
            *(u32x4 *)(kimg + slot * D + ((((4 * t + q4) ^ slot) & (D / 8 - 1)) << 3)) = p.k[T][t];
        }
    wave_lds_order();
    k0.apply(img, rr, lane, SpareMap<D, 0>{2 * kImg});
    k1.apply(img + kImg, rr, lane, SpareMap<D, 0>{kImg});
    v0.issue(rr, rows[2], rows[3], lane);             // in flight while the K fragments go back and V comes in
    v1.issue(rr, rows[6], rows[7], lane);
    wave_lds_order();
#pragma unroll
    for (int T = 0; T < 2; ++T)
#pragma unroll
        for (int t = 0; t < D / 32; ++t) {
            const int slot = slot0 + 4 * T;
            p.k[T][t] = *(const u32x4 *)(kimg + slot * D + ((((4 * t + q4) ^ slot) & (D / 8 - 1)) << 3));
        }
    wave_lds_order();
    uint16_t *vimg = img + (q4 >= 2 ? kImg : 0);
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) *(u32x4 *)(vimg + (16 * dt + m) * kBlock + (q4 & 1) * 8) = p.v[dt];
    wave_lds_order();
    v0.apply(img, rr, lane, SpareMap<D, 1>{2 * kImg});
    v1.apply(img + kImg, rr, lane, SpareMap<D, 1>{kImg});
    wave_lds_order();
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) p.v[dt] = *(const u32x4 *)(vimg + (16 * dt + m) * kBlock + (q4 & 1) * 8);
    wave_lds_order();
}

template <int D, bool FP8>
__device__ __forceinline__ bf16x8 k_operand(const PairRegs<D, FP8> &p, int T, int t) {
    if constexpr (FP8) return fp8x8_to_bf16x8(u32x2{p.k[T][t / 2][2 * (t % 2)], p.k[T][t / 2][2 * (t % 2) + 1]});
    else return __builtin_bit_cast(bf16x8, p.k[T][t]);
}
template <int D, bool FP8>
__device__ __forceinline__ bf16x8 v_operand(const PairRegs<D, FP8> &p, int dt) {
    if constexpr (FP8) return fp8x8_to_bf16x8(p.v[dt]);
    else return __builtin_bit_cast(bf16x8, p.v[dt]);
}

}  // namespace gf
