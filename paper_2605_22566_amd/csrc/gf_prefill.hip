// gf_attn_prefill: the new tokens of each request attend to the KV of the
// ancestor nodes on its path (shared, read through the block table) and,
// causally, to each other (paper, Topology-Aware State Management: assembling
// a workflow's KV from its nodes "without repeated prefill"; also the
// on-the-fly fallback of Effective Path Pruning).
//
// MFMA path.  One workgroup owns (request, kv head, tile of BM new tokens) and
// all G query heads of the group: BM*G = 256 score rows share every K/V tile
// that is staged through LDS, so each byte fetched feeds G times the flops.
// Each of the 8 waves owns one 32-row tile (one query head, 32 tokens).
// Scores are computed transposed so the softmax statistics of a row live in
// one lane pair:
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
// Staging.  KV tiles are 64 keys (4 table entries), double buffered in LDS with
// K one tile ahead of V, and filled by 16-byte global->LDS direct loads (no
// staging registers): lane l of a wave-wide load writes LDS bytes 16*l.. of a
// 1 KB span, and picks its global source so that the LDS image is XOR-swizzled
// (K: chunk position = chunk ^ row bits; V: the two 16-byte halves of a head-dim
// row swap on every other group of 8 rows), which makes every 16-lane group of
// an operand fetch hit 16 distinct 16-byte bank groups.
//
// Pipeline.  Inside a wave the scores run one tile
// ahead of the softmax: iteration t issues, as one straight-line stream of 32
// slots, the 16 score MFMAs of tile t+1 and the 16 P*V MFMAs of tile t, and in
// the shadow of every MFMA a fixed share of the vector work (exponentials, row
// sums and bf16 packing of tile t; row maximum of tile t+1) and one LDS operand
// fetch, four slots ahead of its use.  Scheduling barriers pin that order.
// The reference row maximum is refreshed (and O rescaled) only when some row's
// new maximum exceeds it by more than 2^8; the final normalisation uses the
// same reference, so the result is unchanged.  Per-entry token counts mask
// partial blocks anywhere in the sequence and tail entries causally, in a side
// path taken only by tiles that need it.

#include "gf_internal.h"
#include <type_traits>
#include <utility>

namespace gf {

typedef float f32x2 __attribute__((ext_vector_type(2)));

template <int D, int G, int NW, int ES>   // ES = bytes per pool element (2 bf16, 1 e4m3)
struct PrefillCfg {
    static constexpr int kWaves = NW;
    static constexpr int kThreads = kWaves * 64;
    static constexpr int kRows = 32 * kWaves;        // score rows per workgroup
    static constexpr int kBM = kRows / G;            // new tokens per workgroup
    static constexpr int kBN = 64;                   // keys per KV tile
    static constexpr int kEntries = kBN / kBlock;    // table entries per tile (4)
    static constexpr int kRowBytes = D * ES;         // one K row
    static constexpr int kCPR = kRowBytes / 16;      // 16-byte chunks per K row
    static constexpr int kKTile = kBN * kRowBytes;   // swizzled, unpadded
    static constexpr int kVBlk = D * kBlock * ES;    // one V block in LDS (bytes)
    static constexpr int kVRow = kBlock * ES;        // one head-dim row of a V block (bytes)
    static constexpr int kVTile = kEntries * kVBlk;
    static constexpr int kLds = 2 * kKTile + 2 * kVTile;
    static constexpr int kDmaPerTile = kKTile / 1024;      // 1 KB wave-wide direct loads per tensor per tile
    static constexpr int kDmaPerWave = kDmaPerTile / NW;
    static constexpr int kDmaPerEntry = kDmaPerTile / kEntries;
    static constexpr int kKS = D / 16;               // contraction steps of the score MFMAs
    static constexpr int kDT = D / 32;               // 32-wide output tiles of P*V
    static constexpr int kQK = 2 * kKS;              // score MFMAs per tile
    static constexpr int kPV = kDT * kEntries;       // P*V MFMAs per tile
    static_assert(kRows % G == 0, "rows must split evenly over heads");
    static_assert(kDmaPerTile % NW == 0 && kDmaPerWave >= 1, "staging must divide evenly over waves");
    static_assert(kDmaPerEntry % kDmaPerWave == 0 || kDmaPerWave % kDmaPerEntry == 0, "a direct load stays in one block");
};

constexpr float kRescaleSlack = 8.0f;   // log2 units a row max may exceed its reference
constexpr int kGroup = 4;               // LDS operand fragments fetched (and waited for) together
constexpr int kWaitLds = 0xC07F;        // s_waitcnt lgkmcnt(0), other counters untouched
#ifndef GF_ABL
#define GF_ABL 0
#endif

typedef __attribute__((address_space(3))) void *lptr_t;

// compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), in order.
// The slot schedule of the main loop is written with it, so that "which slot carries which piece
// of vector work" is decided by if constexpr and never exists as a runtime branch.
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// 16-byte-per-lane global -> LDS direct load: lane l writes LDS bytes [dst + 16 l, +16).
// Issued through inline assembly so that it is ordered by hand: the kernel waits for its
// own direct loads (dma_wait) right before the workgroup barrier that publishes a tile,
// instead of before every LDS read that follows their issue.
__device__ __forceinline__ void dma16(const void *src, void *lds_dst) {
    const uint32_t dst = (uint32_t)(uintptr_t)(lptr_t)lds_dst;
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(dst), "v"(src) : "memory", "m0");
}
__device__ __forceinline__ void dma_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

template <int D, int G, int NW, bool FP8>
__global__ __launch_bounds__(NW * 64, 2) void prefill_kernel(AttnArgs a, const int32_t *__restrict__ tab_base,
                                                          const int32_t *__restrict__ ntk_base,
                                                          const int32_t *__restrict__ q_ptr,
                                                          const float *__restrict__ k_scale,
                                                          const float *__restrict__ v_scale,
                                                          const int32_t *__restrict__ plan, int total_q) {
    constexpr int ES = FP8 ? 1 : 2;
    using C = PrefillCfg<D, G, NW, ES>;
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    char *const kbuf = lds;                       // [2][kKTile]
    char *const vbuf = lds + 2 * C::kKTile;       // [2][kVTile]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 31, hh = lane >> 5;

    // Work item.  The plan kernel lists the (request, q tile) items of the batch, heaviest
    // request first and the q tiles of a request back to back; workgroup id u takes item
    // u / Hkv for kv head u % Hkv.  Workgroups are dealt to the 8 XCDs round-robin by id and
    // each XCD has its own L2: with 8 kv heads XCD x carries head x of every request, so the
    // q tiles of a (request, head) pair stream the same K/V through one L2, one after the
    // other, and the work is balanced across XCDs by symmetry.
    const int item = blockIdx.x / a.hkv;
    const int kvh = blockIdx.x % a.hkv;
    if (item >= plan[0]) return;
    const int r = plan[2 + 2 * item];
    const int qt = plan[3 + 2 * item];
    if (r < 0 || r >= a.num_req) return;
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
    const int32_t *__restrict__ tab = tab_base + (size_t)r * a.max_blocks;
    const int32_t *__restrict__ ntk = ntk_base + (size_t)r * a.max_blocks;

    // ---- Q^T operand fragments (registers, whole kernel) ----------------------
    // score row R = 32*wave + m of the workgroup is (token i0 + R/G, head R%G of the group)
    bf16x8 qf[C::kKS];
    const int row_tok = i0 + (32 * wave + m) / G;
    const int row_head = kvh * G + (32 * wave + m) % G;
    {
        const int tokc = min(row_tok, n_new - 1);
        const char *qp = (const char *)a.q + (((size_t)(q0 + tokc)) * a.hq + row_head) * (D * 2);
#pragma unroll
        for (int ks = 0; ks < C::kKS; ++ks)
            qf[ks] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(qp + (16 * ks + 8 * hh) * 2));
    }

    // ---- table window: lane l of every wave caches entry 64*w + l of window w and of window w+1:
    // the pool index of the (block, kv head) tile and the entry's token count; the loop reads them
    // with v_readlane (uniform index), so no memory load sits between a tile and its addresses.
    // Entries beyond e_end read as block 0 with 0 tokens.  One bit per entry says whether the entry
    // needs masking (partial block, causal cut, or beyond the end); a tile tests its 4 bits at once.
    // With an e4m3 pool the window also carries the entry's K scale, log2 of its V scale and the
    // reciprocal of its V scale.
    int win = 0;
    struct Win {
        int idx, nt;
        float ks, lvs, ivs;
    };
    Win w_cur, w_nxt, w_new = {0, 0, 1.f, 0.f, 1.f};
    uint64_t mbits_cur, mbits_nxt;
    auto load_window = [&](int w, Win &x) {
        const int e = 64 * w + lane;
        const bool ok = e < e_end;
        int id = ok ? tab[ok ? e : 0] : 0;
        x.nt = ok ? ntk[ok ? e : 0] : 0;
        if constexpr (FP8) {
            id = min(max(id, 0), a.pool_blocks - 1);
            x.ks = k_scale[id];
            const float vs = v_scale[id];
            x.lvs = __builtin_log2f(vs);
            x.ivs = 1.0f / vs;
        }
        x.idx = id;                          // block id until the window is adopted
    };
    // block id (clamped into the pool) -> index of the (block, kv head) tile; mask bits of the window
    auto adopt_window = [&](int w, Win &x) -> uint64_t {
        const int e = 64 * w + lane;
        x.idx = min(max(x.idx, 0), a.pool_blocks - 1) * a.hkv + kvh;
        const bool need = x.nt < kBlock || (e >= ncb && (e - ncb) * kBlock + kBlock - 1 > i0);
        return __builtin_amdgcn_ballot_w64(need);
    };
    load_window(0, w_cur);
    load_window(1, w_nxt);
    mbits_cur = adopt_window(0, w_cur);
    mbits_nxt = adopt_window(1, w_nxt);
    auto entry_i = [&](int Win::*f, int e) -> int {       // e uniform, within the two cached windows
        const int a0 = __builtin_amdgcn_readlane(w_cur.*f, e & 63), a1 = __builtin_amdgcn_readlane(w_nxt.*f, e & 63);
        return (e >> 6) == win ? a0 : a1;
    };
    auto entry_f = [&](float Win::*f, int e) -> float {
        const int a0 = __builtin_amdgcn_readlane(__float_as_int(w_cur.*f), e & 63);
        const int a1 = __builtin_amdgcn_readlane(__float_as_int(w_nxt.*f), e & 63);
        return __int_as_float((e >> 6) == win ? a0 : a1);
    };

    // ---- staging: global -> LDS direct loads -----------------------------------------
    // Wave w stages table entry w of every tile (K rows / V block image of one pool block).
    static_assert(C::kDmaPerWave == C::kDmaPerEntry && NW == C::kEntries, "one table entry per wave");
    constexpr size_t blk_bytes = (size_t)kBlock * D * ES;
    // K: lane l of direct load i lands at tile row 4i + l/CPR (D=128), chunk position l%CPR, and
    // fetches the chunk (position ^ swizzle(row)) of that row
    constexpr int kRPI = 1024 / C::kRowBytes;            // K rows per direct load
    auto k_swizzle = [](int rho) -> int {
        return C::kCPR == 16 ? (rho & 15) : C::kCPR == 8 ? ((rho >> 1) & 7) : ((rho >> 2) & 3);
    };
    const char *k_src[C::kDmaPerWave], *v_src[C::kDmaPerWave];   // kv head 0 of block 0, this lane's chunk
#pragma unroll
    for (int j = 0; j < C::kDmaPerWave; ++j) {
        const int i = wave * C::kDmaPerWave + j;         // direct load index within the tile
        const int rho = i * kRPI + lane / C::kCPR;       // tile row
        const int pos = lane % C::kCPR;
        k_src[j] = (const char *)a.k + (rho % kBlock) * C::kRowBytes + ((pos ^ k_swizzle(rho)) * 16);
        const int q = j * 64 + lane;                     // 16-byte chunk within the V block image
        if constexpr (FP8) {
            v_src[j] = (const char *)a.v + q * 16;       // one chunk per head-dim row: image = pool block
        } else {
            const int d = q >> 1, vpos = q & 1;
            v_src[j] = (const char *)a.v + d * 32 + ((vpos ^ ((d >> 3) & 1)) * 16);
        }
    }
    auto issue_k = [&](int tile, int buf) {
        const size_t off = (size_t)(uint32_t)entry_i(&Win::idx, tile * C::kEntries + wave) * blk_bytes;
#pragma unroll
        for (int j = 0; j < C::kDmaPerWave; ++j)
            dma16(k_src[j] + off, kbuf + buf * C::kKTile + (wave * C::kDmaPerWave + j) * 1024);
    };
    auto issue_v = [&](int tile, int buf) {
        const size_t off = (size_t)(uint32_t)entry_i(&Win::idx, tile * C::kEntries + wave) * blk_bytes;
#pragma unroll
        for (int j = 0; j < C::kDmaPerWave; ++j)
            dma16(v_src[j] + off, vbuf + buf * C::kVTile + (wave * C::kDmaPerWave + j) * 1024);
    };

    // K operand row m reads key row (m with bits 2,3 swapped); chunk c of row rho sits at
    // position c ^ swizzle(rho)
    const int krow = (m & 0x13) | ((m & 4) << 1) | ((m & 8) >> 1);
    // bf16: contraction step ks of half hh is chunk 2ks+hh, at position (2ks) ^ (hh ^ swizzle);
    // e4m3: it is the half hh of chunk ks, at position ks ^ swizzle
    const int k_sw = k_swizzle(krow);
    const int k_row_off = krow * C::kRowBytes + (FP8 ? 8 * hh : 0);
    const int k_x = FP8 ? k_sw * 16 : (hh ^ k_sw) * 16;
    const int v_lane_off = FP8 ? m * 16 + 8 * hh : m * 32 + ((hh ^ ((m >> 3) & 1)) * 16);
    using frag_t = std::conditional_t<FP8, u32x2, u32x4>;
    auto to_operand = [](frag_t f) -> bf16x8 {
        if constexpr (FP8) return fp8x8_to_bf16x8(f);
        else return __builtin_bit_cast(bf16x8, f);
    };

    // ---- running state --------------------------------------------------------------
    // m_ref is the same in the two lanes of a row; mx, l_run, the per-tile sums and maxima are
    // per-lane partials over the keys of the lane's half and are combined only when needed.
    const float c = a.scale_log2;
    float m_ref = -1.0e30f, l_run = 0.f;
    float mx = -INFINITY;             // partial row maximum (log2 units) of the tile whose scores are pending
    f32x16 o[C::kDT];
#pragma unroll
    for (int dt = 0; dt < C::kDT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[dt][i] = 0.f;
    f32x16 s_a[2], s_b[2];            // score tiles, ping-pong (2 x 32 keys each)

    // Per-chunk exponent constants of tile t.  A raw score of chunk cb becomes
    //   2^(s * mult[cb] + addc[cb]),  mult = sm_scale*log2(e) [* K scale],  addc = -m_ref [+ log2(V scale)]
    // (the V scale rides on P so that P*V needs no further scaling; the row sum divides it out again).
    // A bf16 pool has one set of constants, so one running sum and one running maximum serve the tile.
    constexpr int kAcc = FP8 ? C::kEntries : 1;
    auto acc_of = [](int cb) constexpr -> int { return FP8 ? cb : 0; };
    struct TileScale {
        float mult[kAcc], lvs[kAcc], ivs[kAcc];
    };
    auto tile_scale = [&](int t) -> TileScale {
        TileScale ts;
#pragma unroll
        for (int cb = 0; cb < kAcc; ++cb) {
            if constexpr (FP8) {
                const int ent = t * C::kEntries + cb;
                ts.mult[cb] = c * entry_f(&Win::ks, ent);
                ts.lvs[cb] = entry_f(&Win::lvs, ent);
                ts.ivs[cb] = entry_f(&Win::ivs, ent);
            } else {
                ts.mult[cb] = c;
                ts.lvs[cb] = 0.f;
                ts.ivs[cb] = 1.f;
            }
        }
        return ts;
    };
    // partial row maximum of a score tile in log2 units (this lane's half of the keys)
    auto row_max = [&](const f32x16 (&s)[2], const TileScale &ts) -> float {
        float best = -INFINITY;
#pragma unroll
        for (int cb = 0; cb < C::kEntries; ++cb) {
            float v = s[cb >> 1][8 * (cb & 1)];
#pragma unroll
            for (int j = 1; j < 8; ++j) v = fmaxf(v, s[cb >> 1][8 * (cb & 1) + j]);
            best = fmaxf(best, v * ts.mult[acc_of(cb)]);
        }
        return best;
    };
    auto apply_mask = [&](int t, f32x16 (&s)[2]) {
#pragma unroll
        for (int cb = 0; cb < C::kEntries; ++cb) {
            const int ent = t * C::kEntries + cb;
            const int nt = entry_i(&Win::nt, ent);
            const int tail_base = ent >= ncb ? (ent - ncb) * kBlock : -(1 << 28);
            const int lim = min(nt, row_tok - tail_base + 1) - 8 * hh;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float x = s[cb >> 1][8 * (cb & 1) + j];
                s[cb >> 1][8 * (cb & 1) + j] = (j < lim) ? x : -INFINITY;
            }
        }
    };
    auto k_frag = [&](const char *kb, int n) -> frag_t {     // n = kt * kKS + ks
        const int kt = n / C::kKS, ks = n % C::kKS;
        return *(const frag_t *)(kb + 32 * kt * C::kRowBytes + k_row_off + (((FP8 ? 16 : 32) * ks) ^ k_x));
    };

    // ---- prologue: K(0), V(0), K(1) into LDS; scores of tile 0 ---------------------------
    issue_k(0, 0);
    issue_v(0, 0);
    if (ntiles > 1) issue_k(1, 1);
    dma_wait();
    __syncthreads();
    {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
            for (int x = 0; x < 16; ++x) s_a[kt][x] = 0.f;
#pragma unroll
            for (int ks = 0; ks < C::kKS; ++ks)
                s_a[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(to_operand(k_frag(kbuf, kt * C::kKS + ks)), qf[ks],
                                                                   s_a[kt], 0, 0, 0);
        }
        mx = row_max(s_a, tile_scale(0));
    }

    // ---- one iteration: softmax + P*V of tile t (scores in sc), scores of tile t+1 -> sn ----
    auto body = [&](int t, f32x16 (&sc)[2], f32x16 (&sn)[2]) {
        const bool has_next = t + 1 < ntiles;
        const bool k2 = t + 2 < ntiles;
        // operand stream of this iteration: the K fragments of tile t+1, then the V fragments of tile t,
        // fetched from LDS in groups of kGroup, one group ahead (one wait per group, not per MFMA)
        constexpr int NSLOT = C::kQK + C::kPV;
        static_assert(NSLOT % kGroup == 0, "whole groups");
        const char *kb = kbuf + ((t + 1) & 1) * C::kKTile;
        const char *vb = vbuf + (t & 1) * C::kVTile + v_lane_off;
        auto frag = [&](int n) -> frag_t {
            if (n < C::kQK) return k_frag(kb, n);
            const int j = n - C::kQK;
            return *(const frag_t *)(vb + (j / C::kDT) * C::kVBlk + 32 * (j % C::kDT) * C::kVRow);
        };
        frag_t f[2][kGroup];
        if constexpr (!(GF_ABL & 1)) {
#pragma unroll
            for (int i = 0; i < kGroup; ++i) f[0][i] = frag(i);
        }
        // the table window slides at the end of this iteration if the next tile opens a new one:
        // fetch the window after next now, adopt it after the wait that precedes the barrier
        const bool slide = (t + 1) * C::kEntries == 64 * (win + 1);
        if (slide) load_window(win + 2, w_new);
        const TileScale ts = tile_scale(t);          // constants of this tile ...
        const TileScale tn = tile_scale(t + 1);      // ... and of the next (for its row maximum)
        if (!(GF_ABL & 8) && k2) issue_k(t + 2, t & 1);             // K(t+2) replaces K(t), read last iteration
        if (!(GF_ABL & 8) && has_next) issue_v(t + 1, (t + 1) & 1); // V(t+1) replaces V(t-1)
        // side path: partial blocks / causal tail / end of the sequence in tile t
        if (!(GF_ABL & 32) && ((mbits_cur >> ((t * C::kEntries) & 63)) & ((1u << C::kEntries) - 1)) != 0) {
            apply_mask(t, sc);
            mx = row_max(sc, ts);
        }
        // refresh the reference maximum only when some row outgrew it
        if (__builtin_amdgcn_ballot_w64(mx > m_ref + kRescaleSlack) != 0) {
            const float m_new = fmaxf(m_ref, fmaxf(mx, other_half(mx)));
            const float alpha = fast_exp2(m_ref - m_new);
            m_ref = m_new;
            l_run *= alpha;
#pragma unroll
            for (int dt = 0; dt < C::kDT; ++dt) o[dt] *= alpha;
        }

        // main stream: NSLOT slots of {MFMA, its share of the vector work}
        constexpr int kExpEnd = NSLOT - 5;           // last slot that may carry an exponential
        constexpr auto exp_slot = [](int e) constexpr -> int { return (e * kExpEnd) / 32; };
        static_assert((7 * kExpEnd) / 32 + 1 < C::kQK && (15 * kExpEnd) / 32 + 1 < C::kQK + C::kDT &&
                          (23 * kExpEnd) / 32 + 1 < C::kQK + 2 * C::kDT && (31 * kExpEnd) / 32 + 1 < C::kQK + 3 * C::kDT,
                      "every chunk is packed before its P*V MFMA");
        uint32_t pw[C::kEntries][4];                 // P^T operand, 2 bf16 per word
        float pe[32];                                // exponentials awaiting their bf16 pack
        float addc[kAcc], psum[kAcc], vmax[kAcc];
#pragma unroll
        for (int cb = 0; cb < kAcc; ++cb) {
            addc[cb] = ts.lvs[cb] - m_ref;
            psum[cb] = 0.f;
            vmax[cb] = -INFINITY;
        }
        __builtin_amdgcn_s_waitcnt(kWaitLds);        // group 0 has arrived
        __builtin_amdgcn_sched_barrier(0);
        static_for<NSLOT>([&](auto slot_c) {
            constexpr int i = decltype(slot_c)::value;
            constexpr int g = i / kGroup;
            if constexpr (i < C::kQK) {
                constexpr int kt = i / C::kKS, ks = i % C::kKS;
                if constexpr (ks == 0) {
#pragma unroll
                    for (int x = 0; x < 16; ++x) sn[kt][x] = 0.f;
                }
                sn[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(to_operand(f[g & 1][i % kGroup]), qf[ks], sn[kt], 0, 0, 0);
            } else {
                constexpr int j = i - C::kQK;
                constexpr int cb = j / C::kDT, dt = j % C::kDT;
                u32x4 pq = {pw[cb][0], pw[cb][1], pw[cb][2], pw[cb][3]};
                o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(to_operand(f[g & 1][i % kGroup]),
                                                                __builtin_bit_cast(bf16x8, pq), o[dt], 0, 0, 0);
                // vector share: running maximum of the next tile's scores, two elements per v_max3
                constexpr int kMaxPerSlot = 32 / C::kPV;
                static_assert(kMaxPerSlot % 2 == 0, "maximum taken in pairs");
                static_for<kMaxPerSlot / 2>([&](auto e_c) {
                    constexpr int idx = j * kMaxPerSlot + 2 * decltype(e_c)::value;
                    float &vm = vmax[acc_of(idx / 8)];
                    vm = fmaxf(fmaxf(vm, sn[idx / 16][idx % 16]), sn[idx / 16][idx % 16 + 1]);
                    asm volatile("" : "+v"(vm));      // keep the running maximum in this slot
                });
            }
            // the first MFMA of a group is followed by the fetch of the next group
            if constexpr (!(GF_ABL & 1) && i % kGroup == 0 && i + kGroup < NSLOT) {
#pragma unroll
                for (int x = 0; x < kGroup; ++x) f[(g + 1) & 1][x] = frag(i + kGroup + x);
            }
            // vector share of every slot: the 32 exponentials of tile t are spread evenly over the
            // slots up to kExpEnd.  An exponential joins the row sum one step later (its consumer
            // is never the next instruction), each pair is packed to bf16 one slot after its second
            // exponential, and chunk c is complete before its first P*V MFMA.
            static_for<32>([&](auto e_c) {
                constexpr int e2 = decltype(e_c)::value;
                if constexpr (exp_slot(e2) == i) {
                    constexpr int cb = acc_of(e2 / 8);
                    const float x = sc[e2 / 16][e2 % 16];
                    pe[e2] = (GF_ABL & 2) ? x * ts.mult[cb] + addc[cb] : fast_exp2(x * ts.mult[cb] + addc[cb]);
                    if constexpr (e2 > 0) psum[acc_of((e2 - 1) / 8)] += pe[e2 - 1];
                    asm volatile("" : "+v"(psum[acc_of(e2 > 0 ? (e2 - 1) / 8 : 0)]), "+v"(pe[e2]));   // stay in this slot
                }
                if constexpr ((e2 & 1) && exp_slot(e2) + 1 == i) {
                    const f32x2 p = {pe[e2 - 1], pe[e2]};
                    pw[e2 / 8][(e2 % 8) / 2] = __builtin_bit_cast(uint32_t, __builtin_convertvector(p, bf16x2));
                    if constexpr (e2 == 31) psum[acc_of(3)] += pe[31];
                }
            });
            // one wait per group, at the end of the slot before it: the whole group has arrived
            if constexpr ((i + 1) % kGroup == 0 && i + 1 < NSLOT) __builtin_amdgcn_s_waitcnt(kWaitLds);
            __builtin_amdgcn_sched_barrier(0);
        });
        {
            float best = -INFINITY;
#pragma unroll
            for (int cb = 0; cb < kAcc; ++cb) {
                l_run += psum[cb] * ts.ivs[cb];
                best = fmaxf(best, vmax[cb] * tn.mult[cb]);
            }
            mx = best;
        }
        if (!(GF_ABL & 16)) dma_wait();                              // this wave's direct loads have landed ...
        // (the window fetch is waited for here, nowhere earlier)
        asm volatile("" : "+v"(w_new.idx), "+v"(w_new.nt), "+v"(w_new.ks), "+v"(w_new.lvs), "+v"(w_new.ivs));
        if (slide) {
            w_cur = w_nxt;
            mbits_cur = mbits_nxt;
            w_nxt = w_new;
            mbits_nxt = adopt_window(win + 2, w_nxt);
            ++win;
        }
        if (!(GF_ABL & 4)) __syncthreads();                             // ... and every wave's are visible
    };

    int t = 0;
    for (; t + 2 <= ntiles; t += 2) {
        body(t, s_a, s_b);
        body(t + 1, s_b, s_a);
    }
    if (t < ntiles) body(t, s_a, s_b);
    // ---- epilogue: normalise, round to bf16, store ------------------------------------
    {
        const float l_tot = l_run + other_half(l_run);
        if (row_tok < n_new) {
            const float inv = 1.f / l_tot;
            char *op = (char *)a.o + (((size_t)(q0 + row_tok)) * a.hq + row_head) * (D * 2);
#pragma unroll
            for (int dt = 0; dt < C::kDT; ++dt)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    f32x4 v4 = {o[dt][4 * q] * inv, o[dt][4 * q + 1] * inv, o[dt][4 * q + 2] * inv,
                                o[dt][4 * q + 3] * inv};
                    const bf16x4 b4 = __builtin_convertvector(v4, bf16x4);
                    *(bf16x4 *)(op + (32 * dt + 8 * q + 4 * hh) * 2) = b4;
                }
            if (a.lse && hh == 0)
                a.lse[(size_t)(q0 + row_tok) * a.hq + row_head] =
                    (m_ref + __builtin_log2f(l_tot)) * 0.6931471805599453f;
        }
    }
}

// Work list of a prefill call.  plan[0] = number of items, plan[2 + 2w], plan[3 + 2w] = (request,
// q tile) of item w.  Valid requests only (status 0, query rows matching the table); requests
// are ranked by tokens to attend (context + new, descending; up to kPlanSortMax requests, beyond
// that in batch order) so that the long ones start first; a request's tiles are listed last tile
// (most causal tail) first.  One workgroup; integer work only.
size_t prefill_plan_items(int32_t total_q, int32_t num_req, int bm);
constexpr int kPlanThreads = 256;
constexpr int kPlanSortMax = 2048;

__global__ __launch_bounds__(kPlanThreads) void prefill_plan_kernel(
    int num_req, int bm, int total_q, int cap, const int32_t *__restrict__ q_ptr,
    const int32_t *__restrict__ ctx_lens, const int32_t *__restrict__ seq_lens,
    const int32_t *__restrict__ status, int32_t *__restrict__ plan) {
    __shared__ int cost[kPlanSortMax];
    __shared__ int order[kPlanSortMax];
    __shared__ int part[kPlanThreads];
    const int tid = threadIdx.x;
    const bool sorted = num_req <= kPlanSortMax;
    auto tiles_of = [&](int r) -> int {
        if (status && status[r] != 0) return 0;
        const int n = seq_lens[r] - ctx_lens[r];
        const int q0 = q_ptr[r];
        if (n <= 0 || q_ptr[r + 1] - q0 != n || q0 < 0 || q0 + n > total_q) return 0;
        return (n + bm - 1) / bm;
    };
    if (sorted) {
        for (int r = tid; r < num_req; r += kPlanThreads) cost[r] = tiles_of(r) ? seq_lens[r] : -1;
        __syncthreads();
        for (int r = tid; r < num_req; r += kPlanThreads) {
            const int c = cost[r];
            int rank = 0;
            for (int x = 0; x < num_req; ++x) rank += (cost[x] > c) || (cost[x] == c && x < r);
            order[rank] = r;
        }
        __syncthreads();
    }
    // two-level exclusive scan of the tile counts in list order
    const int per = (num_req + kPlanThreads - 1) / kPlanThreads;
    const int k0 = min(tid * per, num_req), k1 = min(k0 + per, num_req);
    int sum = 0;
    for (int k = k0; k < k1; ++k) sum += tiles_of(sorted ? order[k] : k);
    part[tid] = sum;
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int i = 0; i < kPlanThreads; ++i) {
            const int v = part[i];
            part[i] = run;
            run += v;
        }
        plan[0] = min(run, cap);
        plan[1] = 0;
    }
    __syncthreads();
    int off = part[tid];
    for (int k = k0; k < k1; ++k) {
        const int r = sorted ? order[k] : k;
        const int nt = tiles_of(r);
        for (int j = 0; j < nt; ++j)
            if (off + j < cap) {
                plan[2 + 2 * (off + j)] = r;
                plan[3 + 2 * (off + j)] = nt - 1 - j;
            }
        off += nt;
    }
}

template <int D, int G, int NW, bool FP8>
static hipError_t launch_prefill_k(const AttnArgs &a, const int32_t *q_ptr, int32_t total_q, int32_t *plan,
                                   hipStream_t s);

template <int D, int G, int NW>
static hipError_t launch_prefill_t(const AttnArgs &a, int kv_dtype, const int32_t *q_ptr, int32_t total_q,
                                   int32_t *plan, hipStream_t s) {
    if (kv_dtype == GF_FP8_E4M3) return launch_prefill_k<D, G, NW, true>(a, q_ptr, total_q, plan, s);
    return launch_prefill_k<D, G, NW, false>(a, q_ptr, total_q, plan, s);
}

template <int D, int G, int NW, bool FP8>
static hipError_t launch_prefill_k(const AttnArgs &a, const int32_t *q_ptr, int32_t total_q, int32_t *plan,
                                   hipStream_t s) {
    using C = PrefillCfg<D, G, NW, FP8 ? 1 : 2>;
    auto kern = prefill_kernel<D, G, NW, FP8>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, C::kLds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    // sum_r ceil(n_r / BM) <= total_q / BM + num_req: the item capacity the host can know
    const size_t cap = prefill_plan_items(total_q, a.num_req, C::kBM);
    const size_t grid = cap * a.hkv;
    if (grid == 0) return hipSuccess;
    if (grid > 0x7fffffffu) return hipErrorInvalidValue;
    hipLaunchKernelGGL(prefill_plan_kernel, dim3(1), dim3(kPlanThreads), 0, s, a.num_req, C::kBM, total_q, (int)cap,
                       q_ptr, a.ctx_lens, a.seq_lens, a.status, plan);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(C::kThreads), C::kLds, s, a, a.block_table, a.block_ntok,
                       q_ptr, a.k_scale, a.v_scale, plan, total_q);
    return hipGetLastError();
}

size_t prefill_plan_items(int32_t total_q, int32_t num_req, int bm) { return (size_t)total_q / bm + num_req; }

size_t prefill_plan_bytes(int32_t total_q, int32_t num_req, int group) {
    // 4-wave workgroups: 128 score rows = 128 / group new tokens per item
    return (2 + 2 * prefill_plan_items(total_q, num_req, 128 / group)) * sizeof(int32_t);
}

hipError_t launch_prefill(const AttnArgs &a, int head_dim, int group, int kv_dtype, const int32_t *q_ptr,
                          int32_t total_q, int32_t *plan, hipStream_t s) {
    if (a.num_req == 0 || total_q == 0) return hipSuccess;
    // 4-wave workgroups, two resident per CU: their barriers stay local to one wave per SIMD and
    // the two workgroups drift apart, so one's vector phases fall under the other's MFMAs
#define GF_CASE(DD, GG) \
    if (head_dim == DD && group == GG) return launch_prefill_t<DD, GG, 4>(a, kv_dtype, q_ptr, total_q, plan, s);
    GF_CASE(64, 1) GF_CASE(64, 2) GF_CASE(64, 4) GF_CASE(64, 8)
    GF_CASE(128, 1) GF_CASE(128, 2) GF_CASE(128, 4) GF_CASE(128, 8)
#undef GF_CASE
    return hipErrorNotSupported;
}

}  // namespace gf
