// Reading a sparse residual (paper, "Differential-based KV Cache", Eq. 7) while a kernel holds a pool block in
// LDS: one CSR row -- the entries of one (item, tensor, kv head) image -- is loaded by a wave and added into the
// image, fp32 sum rounded to bf16 (the arithmetic of gf_kv_apply_residual, so the patched image equals a
// reconstructed block bit for bit).  Where an entry lands is the kernel's business: a map takes the logical
// element slot * D + d of an entry to an element of the kernel's LDS image.
#pragma once
#include "gf_internal.h"

namespace gf {

// A map is a callable uint32_t(uint32_t logical element) with a constant kPredicated: false if every entry is
// written somewhere (the map sends entries outside the image to a spare element), true if the map answers
// kNoElem for them and they are skipped.
constexpr uint32_t kNoElem = 0xFFFFFFFFu;          // a predicated map's answer for an entry outside the image

// one residual entry: logical element i of the image, bf16 bits in the low half of `bits`
template <class MAP>
__device__ __forceinline__ void add_entry(uint16_t *img, uint32_t i, uint32_t bits, const MAP &map) {
    const uint32_t at = map(i);
    if constexpr (MAP::kPredicated) {
        if (at == kNoElem) return;
    }
    const float base = __uint_as_float((uint32_t)img[at] << 16);
    const float delta = __uint_as_float(bits << 16);
    const __bf16 sum = (__bf16)(base + delta);                           // round to nearest even
    img[at] = __builtin_bit_cast(uint16_t, sum);
}

// The four CSR rows of a pair (K and V of the two blocks) as entry ranges: [2i], [2i+1] = first and end entry of
// row i in the order K0, V0, K1, V1; an absent residual (item < 0) gives empty rows.  Wave-uniform values.
__device__ __forceinline__ void row_ranges(const ResidualRefs &rr, int item, int kvh, int hkv, int *out) {
    out[0] = out[1] = out[2] = out[3] = 0;
    if (item < 0) return;
    const int32_t *pk = rr.ptr + ((size_t)item * 2 + 0) * hkv + kvh;
    const int32_t *pv = rr.ptr + ((size_t)item * 2 + 1) * hkv + kvh;
    out[0] = pk[0];
    out[1] = pk[1];
    out[2] = pv[0];
    out[3] = pv[1];
}

// A CSR row in flight.  It is read 8 entries (16 bytes of indices, 16 of values) per lane where it covers whole
// aligned groups of 8, and entry by entry at its two ends (or everywhere, if the arrays do not start on a
// 16-byte boundary); issue() starts the loads of the ends and of the first 512 * NG grouped entries, apply() adds
// them into the image and walks the rest of a longer row.  The two K rows of a pair are issued together, then the two
// V rows, so a pair of the paper's density (about a quarter of the 2048 elements of an image) costs two memory
// round trips (the row ranges come a pair ahead).
template <int D, int NG>
struct RowLoad {
    u32x4 gi[NG], gv[NG];        // NG groups of 8 entries per lane: 512 * NG entries per round trip
    uint32_t si, sv;
    int e0, a0, a1, e1;

    __device__ __forceinline__ void load_groups(const ResidualRefs &rr, int g) {
#pragma unroll
        for (int n = 0; n < NG; ++n) {
            gi[n] = u32x4{0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu};   // outside every image: nothing to add
            gv[n] = u32x4{0, 0, 0, 0};
            if (g + 512 * n < a1) {
                gi[n] = *(const u32x4 *)(rr.idx + g + 512 * n);
                gv[n] = *(const u32x4 *)(rr.val + g + 512 * n);
            }
        }
    }

    __device__ __forceinline__ void issue(const ResidualRefs &rr, int first, int end, int lane) {
        e0 = first;
        e1 = end;
        const bool vec = (((uintptr_t)rr.idx | (uintptr_t)rr.val) & 15) == 0;
        a0 = vec ? min(e1, (e0 + 7) & ~7) : e1;        // [e0, a0) and [a1, e1): single entries
        a1 = vec ? a0 + ((e1 - a0) & ~7) : e1;         // [a0, a1): aligned groups of 8
        const int head = a0 - e0, singles = head + (e1 - a1);
        const int es = lane < head ? e0 + lane : a1 + (lane - head);
        si = 0xFFFFFFFFu;
        sv = 0;
        if (lane < singles) {
            si = rr.idx[es];
            sv = rr.val[es];
        }
        load_groups(rr, a0 + 8 * lane);
    }

    template <class MAP>
    __device__ __forceinline__ void apply(uint16_t *img, const ResidualRefs &rr, int lane, const MAP &map) {
        if (e0 >= e1) return;
        add_entry(img, si, sv, map);
        const int head = a0 - e0, singles = head + (e1 - a1);
        for (int s = lane + 64; s < singles; s += 64) {          // only without the 16-byte alignment
            const int e = s < head ? e0 + s : a1 + (s - head);
            add_entry(img, rr.idx[e], rr.val[e], map);
        }
        for (int g = a0 + 8 * lane;; g += 512 * NG) {
#pragma unroll
            for (int n = 0; n < NG; ++n) {
                // the 8 elements are distinct (contract of the CSR), so all are read before any is written
                uint32_t at[8];
                uint16_t sum[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) at[j] = map((gi[n][j / 2] >> (16 * (j % 2))) & 0xFFFFu);
                if constexpr (!MAP::kPredicated) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const float base = __uint_as_float((uint32_t)img[at[j]] << 16);
                        const float delta = __uint_as_float((gv[n][j / 2] >> (16 * (j % 2))) << 16);
                        sum[j] = __builtin_bit_cast(uint16_t, (__bf16)(base + delta));
                    }
#pragma unroll
                    for (int j = 0; j < 8; ++j) img[at[j]] = sum[j];
                } else {
                    // a lane either holds 8 entries of the row or none; entries outside the image are rare, so
                    // the group is written under one lane mask unless some lane of the wave holds a stray
                    const bool mine = g + 512 * n < a1;
                    bool stray = false;
#pragma unroll
                    for (int j = 0; j < 8; ++j) stray |= at[j] == kNoElem;
                    if (__builtin_amdgcn_ballot_w64(mine && stray) == 0) {
                        if (mine) {
#pragma unroll
                            for (int j = 0; j < 8; ++j) {
                                const float base = __uint_as_float((uint32_t)img[at[j]] << 16);
                                const float delta = __uint_as_float((gv[n][j / 2] >> (16 * (j % 2))) << 16);
                                sum[j] = __builtin_bit_cast(uint16_t, (__bf16)(base + delta));
                            }
#pragma unroll
                            for (int j = 0; j < 8; ++j) img[at[j]] = sum[j];
                        }
                    } else {
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            const float base = __uint_as_float((uint32_t)img[at[j] == kNoElem ? 0u : at[j]] << 16);
                            const float delta = __uint_as_float((gv[n][j / 2] >> (16 * (j % 2))) << 16);
                            sum[j] = __builtin_bit_cast(uint16_t, (__bf16)(base + delta));
                        }
#pragma unroll
                        for (int j = 0; j < 8; ++j)
                            if (at[j] != kNoElem) img[at[j]] = sum[j];
                    }
                }
            }
            if (__builtin_amdgcn_ballot_w64(g + 512 * NG < a1) == 0) break;
            load_groups(rr, g + 512 * NG);
        }
    }
};

}  // namespace gf
