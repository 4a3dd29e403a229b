// Operand fragments of the per-request decode kernel: two pool blocks (32 keys) of one kv head, loaded from
// HBM straight into the registers the 16x16x32 MFMAs read (see gf_decode.hip for the geometry), and the
// on-the-fly application of sparse residuals to such a pair.
#pragma once
#include "gf_internal.h"

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
// fragments go to the wave's LDS image `img` (2 * 16 * D elements: the two blocks back to back), the residual
// entries of the blocks that have one (items h0 / h1 of the CSR, -1 = none) are added there -- fp32 sum rounded to
// bf16, the arithmetic of gf_kv_apply_residual, so the operands equal a reconstructed block bit for bit -- and the
// fragments are read back; first K, then V through the same image.  K rows keep the pool's [slot][d] order with the
// 16-byte pieces of a row XOR-ed by the slot (fragment stores and loads then spread over the banks); V keeps
// [d][slot].  Entries outside the image are ignored.  The LDS operations of one wave complete in order.
// orders the LDS accesses of a wave's lanes before and after this point (for the compiler: a fence at
// wavefront scope; the hardware runs one wave's LDS operations in order)
__device__ __forceinline__ void wave_lds_order() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// one residual entry: logical element i of the image (slot * D + d), bf16 bits in the low half of `bits`
template <int D>
__device__ __forceinline__ void add_entry(uint16_t *img, int tensor, uint32_t i, uint32_t bits) {
    if (i >= (uint32_t)(kBlock * D)) return;
    const uint32_t slot = i / D, d = i % D;
    const uint32_t phys = tensor ? d * kBlock + slot : slot * D + ((((d >> 3) ^ slot) & (D / 8 - 1)) << 3) + (d & 7);
    const float base = __uint_as_float((uint32_t)img[phys] << 16);
    const float delta = __uint_as_float(bits << 16);
    const __bf16 sum = (__bf16)(base + delta);                           // round to nearest even
    img[phys] = __builtin_bit_cast(uint16_t, sum);
}

// A CSR row is read 8 entries (16 bytes of indices, 16 of values) per lane where the row covers whole aligned
// groups of 8, and entry by entry at its two ends; all those loads are issued before the first sum, so a row of
// the paper's density (about 512 of 2048 elements) costs one memory round trip, not one per 64 entries.
template <int D>
__device__ __forceinline__ void add_entries(uint16_t *img, const ResidualRefs &rr, int item, int tensor, int kvh,
                                            int hkv, int lane) {
    const size_t row = ((size_t)item * 2 + tensor) * hkv + kvh;
    const int e0 = rr.ptr[row], e1 = rr.ptr[row + 1];
    const bool vec = (((uintptr_t)rr.idx | (uintptr_t)rr.val) & 15) == 0;
    const int a0 = vec ? min(e1, (e0 + 7) & ~7) : e1;        // [e0, a0) and [a1, e1): single entries
    const int a1 = vec ? a0 + ((e1 - a0) & ~7) : e1;         // [a0, a1): aligned groups of 8
    const int head = a0 - e0, singles = head + (e1 - a1);
    const int es = lane < head ? e0 + lane : a1 + (lane - head);
    uint32_t si = 0xFFFFFFFFu, sv = 0;
    if (lane < singles) {
        si = rr.idx[es];
        sv = rr.val[es];
    }
    int g = a0 + 8 * lane;
    u32x4 gi = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu}, gv = {0, 0, 0, 0};
    if (g < a1) {
        gi = *(const u32x4 *)(rr.idx + g);
        gv = *(const u32x4 *)(rr.val + g);
    }
    add_entry<D>(img, tensor, si, sv);
    for (int s = lane + 64; s < singles; s += 64) {          // only without the 16-byte alignment
        const int e = s < head ? e0 + s : a1 + (s - head);
        add_entry<D>(img, tensor, rr.idx[e], rr.val[e]);
    }
    while (true) {
        // the 8 elements are distinct (contract of the CSR), so all are read before any is written
        uint32_t phys[8];
        uint16_t sum[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t i = (gi[j / 2] >> (16 * (j % 2))) & 0xFFFFu;   // 0xFFFF (no load) is outside every image
            const uint32_t slot = i / D, d = i % D;
            phys[j] = i >= (uint32_t)(kBlock * D) ? 0xFFFFFFFFu
                      : tensor ? d * kBlock + slot
                               : slot * D + ((((d >> 3) ^ slot) & (D / 8 - 1)) << 3) + (d & 7);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float base = phys[j] != 0xFFFFFFFFu ? __uint_as_float((uint32_t)img[phys[j]] << 16) : 0.f;
            const float delta = __uint_as_float((gv[j / 2] >> (16 * (j % 2))) << 16);
            sum[j] = __builtin_bit_cast(uint16_t, (__bf16)(base + delta));
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (phys[j] != 0xFFFFFFFFu) img[phys[j]] = sum[j];
        g += 512;
        if (__builtin_amdgcn_ballot_w64(g < a1) == 0) break;
        gi = u32x4{0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu};
        if (g < a1) {
            gi = *(const u32x4 *)(rr.idx + g);
            gv = *(const u32x4 *)(rr.val + g);
        }
    }
}

template <int D>
__device__ __forceinline__ void patch_pair(PairRegs<D, false> &p, uint16_t *img, const ResidualRefs &rr, int h0, int h1,
                                           int kvh, int hkv, int lane) {
    constexpr int kImg = kBlock * D;
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
    if (h0 >= 0) add_entries<D>(img, rr, h0, 0, kvh, hkv, lane);
    if (h1 >= 0) add_entries<D>(img + kImg, rr, h1, 0, kvh, hkv, lane);
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
    if (h0 >= 0) add_entries<D>(img, rr, h0, 1, kvh, hkv, lane);
    if (h1 >= 0) add_entries<D>(img + kImg, rr, h1, 1, kvh, hkv, lane);
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
