// gf_attn_prefill: the new tokens of each request attend to the KV of the
// ancestor nodes on its path (shared, read through the block table) and,
// causally, to each other (paper, Topology-Aware State Management: a workflow's
// KV is assembled from its nodes' stored KV, so the shared prefix is never
// prefilled again; also the on-the-fly fallback of Effective Path Pruning).
//
// MFMA path.  One workgroup (4 waves) owns (request, kv head, tile of BM new tokens) and all G
// query heads of the group: every K/V tile staged through LDS is shared by BM*G score rows, so each
// byte fetched feeds G times the flops.  A wave owns RS "row sets" of 32 score rows (one query
// head x 32 tokens each).  Scores are computed transposed so the softmax statistics of a row live
// in one lane pair:
//   S^T[key][row]  = K[key][d]   * Q^T[d][row]      (A = K from LDS, B = Q registers)
//   O^T[d][row]   += V^T[d][key] * P^T[key][row]    (A = V^T from LDS, B = P registers)
// with v_mfma_f32_32x32x16_bf16: operand lane l holds row/col l%32 and the 8 contraction elements
// of half l/32; accumulator lane l holds column l%32 and rows 8*(i/4) + 4*(l/32) + i%4.  K rows
// are fetched in the order "row m reads key m with bits 2 and 3 swapped", which makes accumulator
// registers 8c..8c+7 of a lane the 8 consecutive slots 8*(l/32)..+7 of 16-key chunk c -- exactly
// the contraction group the V^T operand reads as one 16-byte LDS load from the pool's [d][slot]
// V layout.  P never leaves registers.  Every fragment read from LDS feeds RS MFMAs.
//
// Staging.  KV tiles are 64 keys (4 table entries; wave w stages entry w).  They are filled by
// 16-byte global->LDS direct loads (no staging registers): lane l of a wave-wide load writes LDS
// bytes 16*l.. of a 1 KB span, and picks its global source so that the LDS image is XOR-swizzled
// (K: chunk position = chunk ^ row bits; V: the two 16-byte halves of a head-dim row swap on every
// other group of 8 rows), which makes every 16-lane group of an operand fetch hit 16 distinct
// 16-byte bank groups.  LDS holds two K tiles and three V tiles.
//
// Pipeline.  Inside a wave the scores run one tile ahead of the softmax: iteration t issues, as
// one straight-line stream of slots, the score MFMAs of tile t+1 and the P*V MFMAs of tile t, and
// in the shadow of every MFMA a fixed share of the vector work (exponentials, row sums and bf16
// packing of tile t; running maximum of tile t+1) and the LDS operand fetches (grouped, one wait per
// group).  Three quarters into the stream comes the wait for this wave's direct loads -- K(t+2) and
// V(t+1), issued a whole iteration earlier -- and the one workgroup barrier of the iteration; right
// behind it the direct loads of K(t+3) and V(t+2) are issued, into the buffers every wave has left by
// then, and the first fragments of the next iteration are fetched.  The slot schedule is fixed at
// compile time (static_for / if constexpr) and pinned with scheduling barriers.
// The reference row maximum is refreshed (and O rescaled) only when some row's new maximum
// exceeds it by more than 2^8; the final normalisation uses the same reference, so the result is
// unchanged.  Per-entry token counts mask partial blocks anywhere in the sequence and tail entries
// causally, in a side path taken only by tiles whose mask bits say so.
//
// Differential KV read in place (RES; paper, "Differential-based KV Cache", Eq. 7: the KV of a node under a
// prefix is its stored base KV plus that prefix's sparse residual).  A table entry may carry a residual item;
// the wave that staged the entry's block adds the item's K row and V row for this kv head into the LDS image --
// fp32 sum rounded to bf16, as gf_kv_apply_residual does -- between the wait for its own direct loads and the
// barrier that publishes the tile, when no other wave reads or writes that part of LDS.  The operands then
// equal a reconstructed block bit for bit.  bf16 pools.

#include "gf_internal.h"
#include "gf_residual_row.h"
#include <mutex>
#include <type_traits>
#include <utility>

namespace gf {

typedef float f32x2 __attribute__((ext_vector_type(2)));

// RS = 32-row score tiles ("row sets") per wave.  Every K / V fragment a wave fetches from LDS
// feeds RS MFMAs, so RS = 2 halves the LDS and staging traffic per flop; it needs the register
// budget of one wave per SIMD.
template <int D, int G, int NW, int RS, int ES>   // ES = bytes per pool element (2 bf16, 1 e4m3)
struct PrefillCfg {
    static constexpr int kWaves = NW;
    static constexpr int kThreads = kWaves * 64;
    static constexpr int kRows = 32 * kWaves * RS;   // score rows per workgroup
    static constexpr int kBM = kRows / G;            // new tokens per workgroup
    static constexpr int kBN = 64;                   // keys per KV tile
    static constexpr int kEntries = kBN / kBlock;    // table entries per tile (4)
    static constexpr int kRowBytes = D * ES;         // one K row
    static constexpr int kCPR = kRowBytes / 16;      // 16-byte chunks per K row
    static constexpr int kKTile = kBN * kRowBytes;   // swizzled, unpadded
    static constexpr int kVBlk = D * kBlock * ES;    // one V block in LDS (bytes)
    static constexpr int kVRow = kBlock * ES;        // one head-dim row of a V block (bytes)
    static constexpr int kVTile = kEntries * kVBlk;
    static constexpr int kVBufs = 3;                 // V tiles in LDS (see the pipeline notes in the kernel)
    static constexpr int kLds = 2 * kKTile + kVBufs * kVTile;
    static constexpr int kDmaPerTile = kKTile / 1024;      // 1 KB wave-wide direct loads per tensor per tile
    static constexpr int kDmaPerWave = kDmaPerTile / NW;
    static constexpr int kDmaPerEntry = kDmaPerTile / kEntries;
    static constexpr int kKS = D / 16;               // contraction steps of the score MFMAs
    static constexpr int kDT = D / 32;               // 32-wide output tiles of P*V
    static constexpr int kQK = 2 * kKS;              // K fragments (score MFMAs per row set) per tile
    static constexpr int kPV = kDT * kEntries;       // V fragments (P*V MFMAs per row set) per tile
    static constexpr int kFrags = kQK + kPV;
    static constexpr int kSlots = kFrags * RS;       // MFMAs per tile and wave
    static_assert(kRows % G == 0, "rows must split evenly over heads");
    static_assert(kDmaPerTile % NW == 0 && kDmaPerWave >= 1, "staging must divide evenly over waves");
    static_assert(kDmaPerWave == kDmaPerEntry && NW == kEntries, "one table entry per wave");
};

constexpr int kPrefillWaves = 4;
// Row sets per wave.  A bf16 pool runs one (two workgroups per CU cover each other's stalls; measured
// faster there); an e4m3 pool runs two, where every fragment converted to bf16 serves two MFMAs.
constexpr int prefill_row_sets(bool fp8) { return fp8 ? 2 : 1; }
constexpr int kPrefillRowsMin = 32 * kPrefillWaves;   // fewest score rows a workgroup covers (sizes the work list)

constexpr float kRescaleSlack = 8.0f;   // log2 units a row max may exceed its reference
// LDS operand fragments live in a ring of kRing register sets.  The fetches of fragments
// n + kAhead .. n + kAhead + kFetch - 1 are issued right behind the first MFMA of fragment n
// (n a multiple of kFetch), and the wave waits once per kFetch fragments, for exactly those.
constexpr int kRing = 8, kAhead = 4, kFetch = 4;
static_assert(kAhead % kFetch == 0 && kAhead + kFetch <= kRing, "a fetch never lands in a register set still to be used");
// s_waitcnt lgkmcnt(n), other counters untouched
constexpr int wait_lds(int n) { return 0xC07F | (n << 8); }

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

// MFMA issue of the main loop.  With one row set per wave the compiler's builtin is used.  With
// two, the wave owns the whole register file of its SIMD lane (256 VGPRs + 256 accumulation
// registers) and the operands are placed by hand: O accumulators and the Q fragments live in
// accumulation registers (only MFMAs touch them in the loop), scores and P in VGPRs (the vector
// unit reads and writes them).  The instruction is then issued through inline assembly, which the
// compiler's hazard recogniser does not see through: the one software-managed hazard that applies,
// "MFMA writes VGPRs -> vector instruction reads them" (passes + 3 wait states), is kept by the
// slot schedule itself, which never reads a score tile within kScoreReadGap slots of the MFMA
// that completes it.
constexpr int kScoreReadGap = 4;
template <bool HAND, bool ZERO>
__device__ __forceinline__ void mma_scores(f32x16 &d, bf16x8 kf, bf16x8 qf) {
    if constexpr (!HAND) {
        if constexpr (ZERO) {
#pragma unroll
            for (int x = 0; x < 16; ++x) d[x] = 0.f;
        }
        d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf, d, 0, 0, 0);
    } else if constexpr (ZERO) {
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(kf), "a"(qf));
    } else {
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(kf), "a"(qf));
    }
}
// Element access to an O accumulator outside the MFMA stream (rescale, epilogue).  With hand-placed
// operands the accumulator is never used as a whole by the vector unit: its elements are moved one
// by one, so the tuple itself stays an accumulation-register value everywhere.
template <bool HAND>
__device__ __forceinline__ float acc_get(const f32x16 &v, int i) {
    if constexpr (!HAND) return v[i];
    const float e = v[i];
    float t;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(t) : "a"(e));
    return t;
}
template <bool HAND>
__device__ __forceinline__ void acc_set(f32x16 &v, int i, float t) {
    if constexpr (!HAND) {
        v[i] = t;
    } else {
        float e;
        asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(e) : "v"(t));
        v[i] = e;
    }
}
template <bool HAND>
__device__ __forceinline__ void mma_out(f32x16 &d, bf16x8 vf, bf16x8 pf) {
    if constexpr (!HAND) d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, d, 0, 0, 0);
    else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(d) : "v"(vf), "v"(pf));
}

// Where a residual entry (logical element slot * D + d of a block) sits in the staged images of a bf16 pool:
// K keeps [slot][d] with the 16-byte pieces of a row at position piece ^ swizzle(tile row), V keeps [d][slot]
// with the two 8-slot halves of a row swapped on every other group of 8 rows (see "Staging" above).
template <int D, int TENSOR>
struct StagedMap {
    static constexpr bool kPredicated = true;        // LDS is full: there is no spare element to absorb strays
    int entry;                                       // the block's place in the tile (sets the K swizzle for D < 128)
    __device__ __forceinline__ uint32_t operator()(uint32_t i) const {
        const uint32_t slot = i / D, d = i % D;
        uint32_t at;
        if constexpr (TENSOR == 0) {
            const uint32_t rho = entry * kBlock + slot;
            const uint32_t sw = D == 128 ? (rho & 15) : D == 64 ? ((rho >> 1) & 7) : ((rho >> 2) & 3);
            at = slot * D + (((d >> 3) ^ sw) << 3) + (d & 7);
        } else {
            at = d * kBlock + ((((slot >> 3) ^ (d >> 3)) & 1) << 3) + (slot & 7);
        }
        return i < (uint32_t)(kBlock * D) ? at : kNoElem;
    }
};

template <int D, int G, int NW, int RS, bool FP8, bool RES>
__global__ __launch_bounds__(NW * 64, RS == 1 ? 2 : 1) void prefill_kernel(
    AttnArgs a, const int32_t *__restrict__ tab_base, const int32_t *__restrict__ ntk_base,
    const int32_t *__restrict__ q_ptr, const float *__restrict__ k_scale, const float *__restrict__ v_scale,
    const int32_t *__restrict__ plan, int total_q, ResidualRefs rr) {
    static_assert(!(RES && FP8), "residuals are read in place on bf16 pools only");
    constexpr int ES = FP8 ? 1 : 2;
    using C = PrefillCfg<D, G, NW, RS, ES>;
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    char *const kbuf = lds;                       // [2][kKTile]
    char *const vbuf = lds + 2 * C::kKTile;       // [kVBufs][kVTile]

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
    // score row R = 32*(RS*wave + rs) + m of the workgroup is (token i0 + R/G, head R%G of the group)
    bf16x8 qf[RS][C::kKS];
    int row_tok[RS], row_head[RS];
#pragma unroll
    for (int rs = 0; rs < RS; ++rs) {
        const int R = 32 * (RS * wave + rs) + m;
        row_tok[rs] = i0 + R / G;
        row_head[rs] = kvh * G + R % G;
        const int tokc = min(row_tok[rs], n_new - 1);
        const char *qp = (const char *)a.q + (((size_t)(q0 + tokc)) * a.hq + row_head[rs]) * (D * 2);
#pragma unroll
        for (int ks = 0; ks < C::kKS; ++ks)
            qf[rs][ks] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(qp + (16 * ks + 8 * hh) * 2));
        if constexpr (RS > 1) {                          // from here on they live in accumulation registers
#pragma unroll
            for (int ks = 0; ks < C::kKS; ++ks) asm volatile("" : "+a"(qf[rs][ks]));
        }
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
        int item;                            // RES: residual item of the entry, or -1
    };
    Win w_cur, w_nxt, w_new = {0, 0, 1.f, 0.f, 1.f, -1};
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
        if constexpr (RES) {
            const int it = ok ? rr.handle[(size_t)r * a.max_blocks + (ok ? e : 0)] : -1;
            x.item = (it >= 0 && it < rr.num_items) ? it : -1;
        }
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
    constexpr size_t blk_bytes = (size_t)kBlock * D * ES;
    // K: lane l of direct load i lands at tile row 4i + l/CPR (D=128), chunk position l%CPR, and
    // fetches the chunk (position ^ swizzle(row)) of that row
    constexpr int kRPI = 1024 / C::kRowBytes;            // K rows per direct load
    auto k_swizzle = [](int rho) -> int {
        return C::kCPR == 16 ? (rho & 15) : C::kCPR == 8 ? ((rho >> 1) & 7) : ((rho >> 2) & 3);
    };
    // lane offsets inside a pool block, less the 1024 j that load j's immediate offset adds
    uint32_t k_off[C::kDmaPerWave], v_off[C::kDmaPerWave];
#pragma unroll
    for (int j = 0; j < C::kDmaPerWave; ++j) {
        const int i = wave * C::kDmaPerWave + j;         // direct load index within the tile
        const int rho = i * kRPI + lane / C::kCPR;       // tile row
        const int pos = lane % C::kCPR;
        k_off[j] = (rho % kBlock) * C::kRowBytes + ((pos ^ k_swizzle(rho)) * 16) - 1024 * j;
        const int q = j * 64 + lane;                     // 16-byte chunk within the V block image
        if constexpr (FP8) {
            v_off[j] = q * 16 - 1024 * j;                // one chunk per head-dim row: image = pool block
        } else {
            const int d = q >> 1, vpos = q & 1;
            v_off[j] = d * 32 + ((vpos ^ ((d >> 3) & 1)) * 16) - 1024 * j;
        }
    }
    // address of the pool block behind table entry (tile, this wave), for K or V
    auto block_of = [&](const void *pool, int tile) -> const char * {
        return (const char *)pool + (size_t)(uint32_t)entry_i(&Win::idx, tile * C::kEntries + wave) * blk_bytes;
    };
    auto issue_k = [&](int tile, int buf) {
        const char *src = block_of(a.k, tile);
        static_for<C::kDmaPerWave>([&](auto j_c) {
            constexpr int j = decltype(j_c)::value;
            dma_load<1024 * j>(src, k_off[j], kbuf + buf * C::kKTile + wave * C::kDmaPerWave * 1024);
        });
    };
    auto issue_v = [&](int tile, int buf) {
        const char *src = block_of(a.v, tile);
        static_for<C::kDmaPerWave>([&](auto j_c) {
            constexpr int j = decltype(j_c)::value;
            dma_load<1024 * j>(src, v_off[j], vbuf + buf * C::kVTile + wave * C::kDmaPerWave * 1024);
        });
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
        if constexpr (FP8) {
            bf16x8 x = fp8x8_to_bf16x8(f);
            // the result of a scaled conversion must not be consumed by the next instruction; the
            // compiler keeps that distance for instructions it issues itself, not for hand-issued MFMAs
            if constexpr (RS > 1) asm volatile("s_nop 1" : "+v"(x));
            return x;
        } else {
            return __builtin_bit_cast(bf16x8, f);
        }
    };

    // ---- running state (per row set) ---------------------------------------------------
    // m_ref is the same in the two lanes of a row; mx, l_run, the per-tile sums and maxima are
    // per-lane partials over the keys of the lane's half and are combined only when needed.
    const float c = a.scale_log2;
    float m_ref[RS], l_run[RS];
    float mx[RS];                     // partial row maximum (log2 units) of the tile whose scores are pending
    f32x16 o[RS][C::kDT];
#pragma unroll
    for (int rs = 0; rs < RS; ++rs) {
        m_ref[rs] = -1.0e30f;
        l_run[rs] = 0.f;
        mx[rs] = -INFINITY;
#pragma unroll
        for (int dt = 0; dt < C::kDT; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[rs][dt][i] = 0.f;
        if constexpr (RS > 1) {
#pragma unroll
            for (int dt = 0; dt < C::kDT; ++dt) asm volatile("" : "+a"(o[rs][dt]));   // home: accumulation registers
        }
    }
    f32x16 s_a[RS][2], s_b[RS][2];    // score tiles, ping-pong (2 x 32 keys each)

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
    auto apply_mask = [&](int t, f32x16 (&s)[2], int tok) {
#pragma unroll
        for (int cb = 0; cb < C::kEntries; ++cb) {
            const int ent = t * C::kEntries + cb;
            const int nt = entry_i(&Win::nt, ent);
            const int tail_base = ent >= ncb ? (ent - ncb) * kBlock : -(1 << 28);
            const int lim = min(nt, tok - tail_base + 1) - 8 * hh;
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
    // RES: this wave adds the residual rows of the entries it staged (entry `wave` of a tile) into the images it
    // filled.  The rows of one call are requested together, so a K tile and a V tile cost one memory round trip.
    auto row_issue = [&](auto &row, int tensor, int tile) {
        const int item = tile >= 0 ? entry_i(&Win::item, tile * C::kEntries + wave) : -1;
        int first = 0, end = 0;
        if (item >= 0) {
            const int32_t *rp = rr.ptr + ((size_t)item * 2 + tensor) * a.hkv + kvh;
            first = __builtin_amdgcn_readfirstlane(rp[0]);
            end = __builtin_amdgcn_readfirstlane(rp[1]);
        }
        row.issue(rr, first, end, lane);             // an empty range loads nothing
    };
    // K of `ktile` in K buffer `kb_i`, V of `vtile` in V buffer `vb_i`; a tile of -1 is skipped
    auto patch_tiles = [&](int ktile, int kb_i, int vtile, int vb_i) {
        RowLoad<D, 1> krow, vrow;                    // (two groups per lane for V would not fit the register budget)
        row_issue(krow, 0, ktile);
        row_issue(vrow, 1, vtile);
        krow.apply((uint16_t *)(kbuf + kb_i * C::kKTile + wave * C::kDmaPerWave * 1024), rr, lane, StagedMap<D, 0>{wave});
        vrow.apply((uint16_t *)(vbuf + vb_i * C::kVTile + wave * C::kDmaPerWave * 1024), rr, lane, StagedMap<D, 1>{wave});
    };
    if constexpr (RES) {
        patch_tiles(0, 0, 0, 0);
        if (ntiles > 1) patch_tiles(1, 1, -1, 0);
    }
    __syncthreads();
    {
        const TileScale t0 = tile_scale(0);
        constexpr bool kHand = RS > 1;
        static_for<2 * C::kKS>([&](auto n_c) {
            constexpr int n = decltype(n_c)::value;
            constexpr int kt = n / C::kKS, ks = n % C::kKS;
            const bf16x8 kf = to_operand(k_frag(kbuf, n));
            static_for<RS>([&](auto r_c) {
                constexpr int rs = decltype(r_c)::value;
                mma_scores<kHand, ks == 0>(s_a[rs][kt], kf, qf[rs][ks]);
            });
        });
        if constexpr (kHand) {
            // scores written by hand-issued MFMAs: the wait states the vector unit needs before it may
            // read them; the tiles pass through the statement so that every read is ordered behind it
            static_for<RS>([&](auto r_c) {
                constexpr int rs = decltype(r_c)::value;
                f32x16 &t0 = s_a[rs][0], &t1 = s_a[rs][1];
                asm volatile("s_nop 7\n\ts_nop 7" : "+v"(t0), "+v"(t1));
            });
        }
#pragma unroll
        for (int rs = 0; rs < RS; ++rs) mx[rs] = row_max(s_a[rs], t0);
    }
    // Every wave is done with K(0) before its buffer is staged again; from here on the loads of an iteration
    // are issued right behind the barrier of the iteration before (K(2) and V(1) are the ones "iteration -1" owes).
    __syncthreads();
    if (ntiles > 2) issue_k(2, 0);
    if (ntiles > 1) issue_v(1, 1 % C::kVBufs);

    // The reference maxima are refreshed (and O, l rescaled) only when some row's pending maximum
    // outgrew its reference by more than the slack: a cold path.
    // Side path, before tile t is taken up: partial blocks / causal tail / end of the sequence in it
    // (pad slots may hold any finite value, so the pending maxima are taken again after masking).
    auto premask = [&](int t, f32x16 (&sc)[RS][2]) {
        if (((mbits_cur >> ((t * C::kEntries) & 63)) & ((1u << C::kEntries) - 1)) != 0) {
            const TileScale ts = tile_scale(t);
#pragma unroll
            for (int rs = 0; rs < RS; ++rs) {
                apply_mask(t, sc[rs], row_tok[rs]);
                mx[rs] = row_max(sc[rs], ts);
            }
        }
    };
    auto need_rescale = [&]() -> bool {
        bool grow = false;
#pragma unroll
        for (int rs = 0; rs < RS; ++rs) grow |= mx[rs] > m_ref[rs] + kRescaleSlack;
        return __builtin_amdgcn_ballot_w64(grow) != 0;
    };
    auto rescale = [&]() {
        if constexpr (RS > 1) asm volatile("s_nop 7\n\ts_nop 7" ::: "memory");   // O written by hand-issued MFMAs
#pragma unroll
        for (int rs = 0; rs < RS; ++rs) {
            const float m_new = fmaxf(m_ref[rs], fmaxf(mx[rs], other_half(mx[rs])));
            const float alpha = fast_exp2(m_ref[rs] - m_new);
            m_ref[rs] = m_new;
            l_run[rs] *= alpha;
#pragma unroll
            for (int dt = 0; dt < C::kDT; ++dt)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc_set<(RS > 1)>(o[rs][dt], i, acc_get<(RS > 1)>(o[rs][dt], i) * alpha);
        }
    };

    // ---- one iteration: softmax + P*V of tile t (scores in sc), scores of tile t+1 -> sn ----
    frag_t f[kRing];                  // operand fragments; the first kAhead of an iteration are fetched by the one before
#pragma unroll
    for (int x = 0; x < kAhead; ++x) f[x] = k_frag(kbuf + C::kKTile, x);   // K(1), staged by the prologue
    auto body = [&](int t, f32x16 (&sc)[RS][2], f32x16 (&sn)[RS][2]) {
        const bool has_next = t + 1 < ntiles;
        const bool k2 = t + 2 < ntiles;
        const bool k3 = t + 3 < ntiles;
        // operand stream of this iteration: the K fragments of tile t+1, then the V fragments of tile t,
        // fetched from LDS kAhead fragments ahead of their use;
        // every fragment feeds one MFMA per row set
        constexpr int NSLOT = C::kSlots;
        constexpr bool kHand = RS > 1;
        constexpr int kLdsPerFrag = 1;               // LDS operations per fragment
        // Pipeline of one iteration (slots of the MFMA stream):
        //   kSyncSlot      wait for this wave's loads -- K(t+2) and V(t+1), issued behind the barrier of the
        //                  iteration before, a whole iteration ago -- and workgroup barrier: they are published;
        //                  it comes after the last read of K(t+1) and before the first read of K(t+2)
        //   kStageKSlot..  behind that barrier: direct loads of K(t+3), one per slot, into the buffer K(t+1)
        //                  left (every wave has passed its last read of it)
        //   kStageVSlot..  direct loads of V(t+2) into the buffer V(t-1) left (read in the iteration before, which
        //                  every wave has left); V(t) may still be read by a wave that is behind this barrier and
        //                  V(t+1) has just landed, hence three V buffers
        //   from fragment kFirstNext on, the fetches are those of the next iteration's first fragments
        constexpr int kFirstNext = C::kFrags - kAhead;
        constexpr int kSyncSlot = RS * (C::kQK + C::kPV / 2 < kFirstNext ? C::kQK + C::kPV / 2 : kFirstNext);
        constexpr int kStageKSlot = kSyncSlot, kStageVSlot = kSyncSlot + RS * C::kDmaPerWave;
        static_assert(C::kFrags % kRing == 0 && kAhead <= C::kQK, "the ring position of a fragment is the same in every iteration");
        static_assert(kSyncSlot >= RS * C::kQK && kSyncSlot <= RS * kFirstNext, "barrier between the K reads");
        static_assert(kStageVSlot + RS * C::kDmaPerWave <= NSLOT, "loads issued inside the iteration");
        static_assert(C::kFrags % kFetch == 0, "whole wait groups");
        const char *kb = kbuf + ((t + 1) & 1) * C::kKTile;
        const char *vb = vbuf + (t % C::kVBufs) * C::kVTile + v_lane_off;
        const char *kb_next = kbuf + (t & 1) * C::kKTile;          // K(t+2), once this iteration's barrier is passed
        auto frag = [&](int n) -> frag_t {
            if (n < C::kQK) return k_frag(kb, n);
            const int j = n - C::kQK;
            return *(const frag_t *)(vb + (j / C::kDT) * C::kVBlk + 32 * (j % C::kDT) * C::kVRow);
        };
        // the table window slides in this iteration if the next tile opens a new one: fetch the
        // window after next now, adopt it after the wait that precedes the barrier
        const bool slide = (t + 1) * C::kEntries == 64 * (win + 1);
        if (slide) load_window(win + 2, w_new);
        const TileScale ts = tile_scale(t);          // constants of this tile ...
        const TileScale tn = tile_scale(t + 1);      // ... and of the next (for its row maximum)
        premask(t, sc);
        if (need_rescale()) rescale();

        // main stream: NSLOT slots of {MFMA, its share of the vector work}; slot i uses fragment
        // i / RS for row set i % RS
        constexpr int kExps = 32 * RS;               // exponentials per tile, in the order (key, row set)
        constexpr int kExpEnd = NSLOT - 4 * RS - 1;  // last slot that may carry an exponential
        constexpr auto exp_slot = [](int x) constexpr -> int { return (x * kExpEnd) / kExps; };
        constexpr auto packed_in_time = [exp_slot]() constexpr -> bool {
            for (int cb = 0; cb < C::kEntries; ++cb)
                for (int rs = 0; rs < RS; ++rs)
                    if (exp_slot((8 * cb + 7) * RS + rs) + 1 >= RS * (C::kQK + cb * C::kDT) + rs) return false;
            return true;
        };
        static_assert(packed_in_time(), "every chunk is packed before its first P*V MFMA");
        bf16x8 opnd;                                 // the fragment in use, as an MFMA operand
        const char *stage_src = nullptr;              // pool block being staged (uniform)
        uint32_t pw[RS][C::kEntries][4];             // P^T operands, 2 bf16 per word
        float pe[RS][32];                            // exponentials awaiting their bf16 pack
        float addc[RS][kAcc], psum[RS][kAcc], vmax[RS][kAcc];
#pragma unroll
        for (int rs = 0; rs < RS; ++rs)
#pragma unroll
            for (int cb = 0; cb < kAcc; ++cb) {
                addc[rs][cb] = ts.lvs[cb] - m_ref[rs];
                psum[rs][cb] = 0.f;
                vmax[rs][cb] = -INFINITY;
            }
        __builtin_amdgcn_s_waitcnt(wait_lds((kAhead - kFetch) * kLdsPerFrag));        // the first fragments have arrived
        __builtin_amdgcn_sched_barrier(0);
        static_for<NSLOT>([&](auto slot_c) {
            constexpr int i = decltype(slot_c)::value;
            constexpr int n = i / RS, rs = i % RS;   // fragment, row set
            if constexpr (i == kSyncSlot) {
                dma_wait();                      // this wave's direct loads have landed ...
                // (the window fetch is waited for here, nowhere earlier)
                asm volatile("" : "+v"(w_new.idx), "+v"(w_new.nt), "+v"(w_new.ks), "+v"(w_new.lvs), "+v"(w_new.ivs));
                if constexpr (RES) {
                    // the tiles staged in this iteration are still this wave's alone (their windows are the
                    // ones cached before the slide below)
                    patch_tiles(k2 ? t + 2 : -1, t & 1, has_next ? t + 1 : -1, (t + 1) % C::kVBufs);
                }
                if (slide) {
                    w_cur = w_nxt;
                    mbits_cur = mbits_nxt;
                    w_nxt = w_new;
                    mbits_nxt = adopt_window(win + 2, w_nxt);
                    ++win;
                }
                __syncthreads();                  // ... and every wave's are visible
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (n < C::kQK) {
                constexpr int kt = n / C::kKS, ks = n % C::kKS;
                if constexpr (rs == 0) opnd = to_operand(f[n % kRing]);
                mma_scores<kHand, ks == 0>(sn[rs][kt], opnd, qf[rs][ks]);
            } else {
                if constexpr (kHand && i == C::kQK * RS) {
                    // no read of the new score tiles is placed ahead of the P*V phase (the schedule keeps
                    // kScoreReadGap slots between a hand-issued MFMA and the first read of its result)
                    static_for<RS>([&](auto r_c) {
                        constexpr int r2 = decltype(r_c)::value;
                        f32x16 &t0 = sn[r2][0], &t1 = sn[r2][1];
                        asm volatile("" : "+v"(t0), "+v"(t1));
                    });
                }
                constexpr int j = n - C::kQK;
                constexpr int cb = j / C::kDT, dt = j % C::kDT;
                u32x4 pq = {pw[rs][cb][0], pw[rs][cb][1], pw[rs][cb][2], pw[rs][cb][3]};
                if constexpr (rs == 0) opnd = to_operand(f[n % kRing]);
                mma_out<kHand>(o[rs][dt], opnd, __builtin_bit_cast(bf16x8, pq));
                // vector share: running maxima of the next tile's scores, two elements per v_max3
                constexpr int kMaxPerSlot = 32 / C::kPV;
                static_assert(kMaxPerSlot % 2 == 0, "maximum taken in pairs");
                static_for<kMaxPerSlot / 2>([&](auto e_c) {
                    constexpr int y = (i - C::kQK * RS) * kMaxPerSlot + 2 * decltype(e_c)::value;   // in [0, 32 RS)
                    constexpr int r2 = y / 32, idx = y % 32;
                    // the score tile read here was completed by slot RS * kKS * (idx / 16 + 1) - RS + r2
                    static_assert(i - (RS * C::kKS * (idx / 16 + 1) - RS + r2) >= kScoreReadGap, "MFMA result read too early");
                    float &vm = vmax[r2][acc_of(idx / 8)];
                    vm = fmaxf(fmaxf(vm, sn[r2][idx / 16][idx % 16]), sn[r2][idx / 16][idx % 16 + 1]);
                    asm volatile("" : "+v"(vm));      // keep the running maximum in this slot
                });
            }
            // the first MFMA of a fetch group is followed by the fetch of the group kAhead fragments on;
            // near the end of the iteration those are K fragments of tile t+2, for the next iteration
            if constexpr (rs == 0 && n % kFetch == 0) {
                static_for<kFetch>([&](auto x_c) {
                    constexpr int nn = n + kAhead + decltype(x_c)::value;
                    if constexpr (nn < C::kFrags) f[nn % kRing] = frag(nn);
                    else f[nn % kRing] = k_frag(kb_next, nn - C::kFrags);
                });
            }
            // staging for the coming iterations rides in early slots, one direct load per slot
            if constexpr (i >= kStageKSlot && i < kStageKSlot + RS * C::kDmaPerWave && (i - kStageKSlot) % RS == 0) {
                constexpr int j = (i - kStageKSlot) / RS;
                if constexpr (j == 0) stage_src = block_of(a.k, t + 3);
                if (k3)                                               // K(t+3) replaces K(t+1)
                    dma_load<1024 * j>(stage_src, k_off[j], kbuf + ((t + 1) & 1) * C::kKTile + wave * C::kDmaPerWave * 1024);
            }
            if constexpr (i >= kStageVSlot && i < kStageVSlot + RS * C::kDmaPerWave && (i - kStageVSlot) % RS == 0) {
                constexpr int j = (i - kStageVSlot) / RS;
                if constexpr (j == 0) stage_src = block_of(a.v, t + 2);
                if (k2)                                               // V(t+2) replaces V(t-1)
                    dma_load<1024 * j>(stage_src, v_off[j], vbuf + ((t + 2) % C::kVBufs) * C::kVTile + wave * C::kDmaPerWave * 1024);
            }
            // vector share of every slot: the exponentials of tile t are spread evenly over the
            // slots up to kExpEnd.  An exponential joins the row sum one step later (its consumer
            // is never the next instruction), each pair is packed to bf16 one slot after its second
            // exponential, and chunk c of a row set is complete before its first P*V MFMA.
            static_for<kExps>([&](auto e_c) {
                constexpr int x = decltype(e_c)::value;
                constexpr int e2 = x / RS, r2 = x % RS;
                if constexpr (exp_slot(x) == i) {
                    constexpr int cb = acc_of(e2 / 8);
                    const float sv = sc[r2][e2 / 16][e2 % 16];
                    const float arg = sv * ts.mult[cb] + addc[r2][cb];
                    pe[r2][e2] = fast_exp2(arg);
                    constexpr int xp = x > 0 ? x - 1 : 0;                  // the exponential before this one
                    if constexpr (x > 0) psum[xp % RS][acc_of(xp / RS / 8)] += pe[xp % RS][xp / RS];
                    asm volatile("" : "+v"(psum[xp % RS][acc_of(xp / RS / 8)]), "+v"(pe[r2][e2]));   // stay in this slot
                }
                if constexpr ((e2 & 1) && exp_slot(x) + 1 == i) {
                    const f32x2 p = {pe[r2][e2 - 1], pe[r2][e2]};
                    pw[r2][e2 / 8][(e2 % 8) / 2] = __builtin_bit_cast(uint32_t, __builtin_convertvector(p, bf16x2));
                    if constexpr (x == kExps - 1) psum[r2][acc_of(3)] += pe[r2][31];
                }
            });
            // one wait per kFetch fragments, at the end of the slot before them: they have arrived
            // (the fetches issued behind them stay in flight)
            if constexpr (rs == RS - 1 && (n + 1) % kFetch == 0 && n + 1 < C::kFrags)
                __builtin_amdgcn_s_waitcnt(wait_lds((kAhead - kFetch) * kLdsPerFrag));
            __builtin_amdgcn_sched_barrier(0);
        });
#pragma unroll
        for (int rs = 0; rs < RS; ++rs) {
            float best = -INFINITY;
#pragma unroll
            for (int cb = 0; cb < kAcc; ++cb) {
                l_run[rs] += psum[rs][cb] * ts.ivs[cb];
                best = fmaxf(best, vmax[rs][cb] * tn.mult[cb]);
            }
            mx[rs] = best;
        }
    };

    int t = 0;
    for (; t + 2 <= ntiles; t += 2) {
        body(t, s_a, s_b);
        body(t + 1, s_b, s_a);
    }
    if (t < ntiles) body(t, s_a, s_b);
    // ---- epilogue: normalise, round to bf16, store ------------------------------------
    if constexpr (RS > 1) asm volatile("s_nop 7\n\ts_nop 7" ::: "memory");   // O written by hand-issued MFMAs
#pragma unroll
    for (int rs = 0; rs < RS; ++rs) {
        const float l_tot = l_run[rs] + other_half(l_run[rs]);
        if (row_tok[rs] < n_new) {
            const float inv = 1.f / l_tot;
            char *op = (char *)a.o + (((size_t)(q0 + row_tok[rs])) * a.hq + row_head[rs]) * (D * 2);
#pragma unroll
            for (int dt = 0; dt < C::kDT; ++dt)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    f32x4 v4;
#pragma unroll
                    for (int x = 0; x < 4; ++x) v4[x] = acc_get<(RS > 1)>(o[rs][dt], 4 * q + x) * inv;
                    const bf16x4 b4 = __builtin_convertvector(v4, bf16x4);
                    *(bf16x4 *)(op + (32 * dt + 8 * q + 4 * hh) * 2) = b4;
                }
            if (a.lse && hh == 0)
                a.lse[(size_t)(q0 + row_tok[rs]) * a.hq + row_head[rs]] =
                    (m_ref[rs] + __builtin_log2f(l_tot)) * 0.6931471805599453f;
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

template <int D, int G, int NW, bool FP8, bool RES>
static hipError_t launch_prefill_k(const AttnArgs &a, const int32_t *q_ptr, int32_t total_q, int32_t *plan,
                                   const ResidualRefs &rr, hipStream_t s);

template <int D, int G, int NW>
static hipError_t launch_prefill_t(const AttnArgs &a, int kv_dtype, const int32_t *q_ptr, int32_t total_q,
                                   int32_t *plan, const ResidualRefs *rr, hipStream_t s) {
    const ResidualRefs none = {nullptr, nullptr, nullptr, nullptr, 0};
    if (kv_dtype == GF_FP8_E4M3)
        return rr ? hipErrorNotSupported : launch_prefill_k<D, G, NW, true, false>(a, q_ptr, total_q, plan, none, s);
    if (rr) return launch_prefill_k<D, G, NW, false, true>(a, q_ptr, total_q, plan, *rr, s);
    return launch_prefill_k<D, G, NW, false, false>(a, q_ptr, total_q, plan, none, s);
}

template <int D, int G, int NW, bool FP8, bool RES>
static hipError_t launch_prefill_k(const AttnArgs &a, const int32_t *q_ptr, int32_t total_q, int32_t *plan,
                                   const ResidualRefs &rr, hipStream_t s) {
    constexpr int RS = prefill_row_sets(FP8);
    using C = PrefillCfg<D, G, NW, RS, FP8 ? 1 : 2>;
    static_assert(C::kRows >= kPrefillRowsMin, "the work list is sized for the smallest tile height");
    auto kern = prefill_kernel<D, G, NW, RS, FP8, RES>;
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
                       q_ptr, a.k_scale, a.v_scale, plan, total_q, rr);
    return hipGetLastError();
}

size_t prefill_plan_items(int32_t total_q, int32_t num_req, int bm) { return (size_t)total_q / bm + num_req; }

// Work list for callers that cannot allocate (gf_attn_prefill_noalloc).  Every GPU the library runs on holds
// its own copy of this array, at its own address, until the process ends.  In host code the array's name is
// only a stand-in for the symbol: the device address is looked up once per device and kept, and that pointer
// -- never the name -- is what the launches are given.  All calls on one GPU share the array; the plan kernel
// writes the item count and every item the attention kernel reads, so nothing has to be cleared between calls.
static __device__ __align__(256) int32_t scratch[kStaticPlanBytes / sizeof(int32_t)];

constexpr int kMaxDevices = 64;
static int32_t *g_static_plan[kMaxDevices];
static std::mutex g_static_plan_mutex;

hipError_t prefill_static_plan_init(int device) {
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_static_plan_mutex);
    if (g_static_plan[device]) return hipSuccess;
    int32_t *ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_static_plan[device] = ptr;
    return hipSuccess;
}

int32_t *prefill_static_plan(int device) {
    if (device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_static_plan_mutex);
    return g_static_plan[device];
}

size_t prefill_plan_bytes(int32_t total_q, int32_t num_req, int group) {
    // one item covers at least kPrefillRowsMin score rows = kPrefillRowsMin / group new tokens
    return (2 + 2 * prefill_plan_items(total_q, num_req, kPrefillRowsMin / group)) * sizeof(int32_t);
}

hipError_t launch_prefill(const AttnArgs &a, int head_dim, int group, int kv_dtype, const int32_t *q_ptr,
                          int32_t total_q, int32_t *plan, const ResidualRefs *rr, hipStream_t s) {
    if (a.num_req == 0 || total_q == 0) return hipSuccess;
    // 4-wave workgroups, two resident per CU: their barriers stay local to one wave per SIMD and
    // the two workgroups drift apart, so one's vector phases fall under the other's MFMAs
#define GF_CASE(DD, GG) \
    if (head_dim == DD && group == GG) return launch_prefill_t<DD, GG, kPrefillWaves>(a, kv_dtype, q_ptr, total_q, plan, rr, s);
    GF_CASE(64, 1) GF_CASE(64, 2) GF_CASE(64, 4) GF_CASE(64, 8)
    GF_CASE(128, 1) GF_CASE(128, 2) GF_CASE(128, 4) GF_CASE(128, 8)
#undef GF_CASE
    return hipErrorNotSupported;
}

}  // namespace gf
