"""Oracle for the differential KV cache (paper, "Differential-based KV Cache", Eq. 7):

    KV(P, v) = KV_base(v) + dKV(P, v)

the KV state of operation node v under prefix path P is its base KV plus a sparse,
prefix-specific residual.  TEST INFRASTRUCTURE ONLY (see the package header).

What is computed here, block by block of the paged pool:
  * reconstruct(): copy the base blocks of a node to destination blocks and add the
    residual entries.  The residual is a CSR with one row per (item, tensor, kv
    head) image of 16 x D elements, row = (item * 2 + t) * Hkv + h with t = 0 for K
    and 1 for V; an entry addresses the LOGICAL element slot * D + d of its image,
    whatever the physical layout of the tensor inside the block (K is stored
    [h][slot][d], V is stored [h][d][slot]).  The sum is taken in fp32 and rounded
    to bf16 round-to-nearest-even -- the stored code is a quantisation decision, so
    the oracle takes it in the kernel's precision (fp32), not in fp64.
  * select_by_energy(): the offline selection rule of the paper's appendix (keep the
    largest-magnitude entries that hold a given share, 95 %, of the Frobenius energy
    of the dense difference), and make_residual(), which applies it image by image to
    the difference between a prefix-conditioned block and its base block and emits the CSR.

Readings: the paper does not fix the storage format of a residual (coordinate list
here, one CSR row per block, tensor and kv head, 16-bit element index), its value
precision (bf16 here, like the pool), or what happens to malformed input (a block
id outside the pool skips the item, an element index outside the image is ignored;
both are reported per item).

e4m3 pools, reconstruct_e4m3(): the base block is widened (code -> value, times the source
block's scale, one fp32 product), the residual entries are added in fp32 in row order, and the
result is quantised again under a scale of its own: per tensor, scale = amax / 448 over the
whole destination block (all kv heads, all 16 slots -- a block carries no token count, so pad
slots take part; the write path leaves them zero), 1.0 for an all-zero block, code =
e4m3(clamp(x / scale)), fp32 division, round to nearest even.  Reading: the paper keeps KV in
16 bits; a quantised pool with a residual on top is this build's combination of the two.

Packed form (pack_rows, unpack_rows, reconstruct_packed): the same residual stored as one bit mask per image (bit
i of the image = logical element i = slot * D + d, kept in 32-bit words, bit i % 32 of word i // 32) plus the kept
values alone, in rising element order; the row pointers are those of the CSR.  At the densities the paper reports
this is 0.34 of a dense bf16 block where the CSR (2 B index + 2 B value) is 0.55.  Reading: the paper does not fix
a storage format; the arithmetic of a reconstruction from either form is the same.

Pins (tests/test_oracle_residual.py): the bf16 rounding against torch's cast on
random values, ties and extremes; an empty residual is the identity; the residual
-base gives all zeros; a full-density residual equals torch's element-wise bf16 add;
single entries land on the hand-indexed physical element of K and of V; a node
reconstructed block by block equals base + delta formed on the [token][head][dim]
segment without any block arithmetic; select_by_energy against brute force over all
subsets on tiny inputs, plus its defining invariants.  make_residual: with share 1 and differences that bf16 holds
exactly, reconstruct(base, make_residual(base, full)) gives back `full` bit for bit; a hand-built image whose
energy sits in three entries keeps exactly those; K and V entries land on the hand-indexed logical positions.  reconstruct_e4m3: an empty residual
re-codes a block onto itself (same codes, same scale) when its largest code is the largest
finite one; codes and scales against torch's float8 casts of the same fp32 sums; the
dequantised result within half a code step of base + delta; bad blocks and indices reported.
Packed form: a hand-written image (bits and value order typed in by hand); unpack(pack(x)) gives x with rows sorted
by element; the mask's population count is the row length; reconstruct_packed equals reconstruct() on the CSR it
was packed from (which is pinned above) and lands hand-indexed single entries on the same physical K / V elements.
"""
import numpy as np

from .append import f32_to_e4m3_codes
from .formats import E4M3_TABLE

BLOCK = 16
ST_OK, ST_BAD_BLOCK, ST_BAD_INDEX = 0, 1, 2


def f32_to_bf16_bits_rne(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bits, round to nearest, ties to even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    return ((u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits).astype(np.uint32) << np.uint32(16)).view(np.float32)


def csr_row(item: int, t: int, h: int, hkv: int) -> int:
    return (item * 2 + t) * hkv + h


def reconstruct(k_pool: np.ndarray, v_pool: np.ndarray, src_blocks, dst_blocks, res_ptr, res_idx, res_val):
    """k_pool uint16 [nb, Hkv, 16, D], v_pool uint16 [nb, Hkv, D, 16] (bf16 bits).
    Returns (k_pool', v_pool', status[num_items]); the inputs are not modified."""
    k_out, v_out = k_pool.copy(), v_pool.copy()
    nb, hkv, _, dim = k_pool.shape
    n_items = len(src_blocks)
    status = np.zeros(n_items, dtype=np.int32)
    for b in range(n_items):
        s, t = int(src_blocks[b]), int(dst_blocks[b])
        if not (0 <= s < nb and 0 <= t < nb):
            status[b] = ST_BAD_BLOCK
            continue
        kb = bf16_bits_to_f32(k_pool[s]).copy()          # [Hkv, 16, D]
        vb = bf16_bits_to_f32(v_pool[s]).copy()          # [Hkv, D, 16]
        for tensor in (0, 1):
            for h in range(hkv):
                r = (b * 2 + tensor) * hkv + h
                for e in range(int(res_ptr[r]), int(res_ptr[r + 1])):
                    i = int(res_idx[e])
                    if not (0 <= i < BLOCK * dim):
                        status[b] = ST_BAD_INDEX
                        continue
                    val = bf16_bits_to_f32(np.array([res_val[e]], dtype=np.uint16))[0]
                    slot, d = divmod(i, dim)
                    if tensor == 0:
                        kb[h, slot, d] = np.float32(kb[h, slot, d]) + np.float32(val)
                    else:
                        vb[h, d, slot] = np.float32(vb[h, d, slot]) + np.float32(val)
        k_out[t] = f32_to_bf16_bits_rne(kb)
        v_out[t] = f32_to_bf16_bits_rne(vb)
    return k_out, v_out, status


def reconstruct_e4m3(k_pool, v_pool, k_scale, v_scale, src_blocks, dst_blocks, res_ptr, res_idx, res_val):
    """k_pool uint8 [nb, Hkv, 16, D], v_pool uint8 [nb, Hkv, D, 16] (e4m3 codes), k_scale / v_scale fp32 [nb].
    Returns (k_pool', v_pool', k_scale', v_scale', status[num_items]); the inputs are not modified."""
    k_out, v_out = k_pool.copy(), v_pool.copy()
    ks_out, vs_out = k_scale.copy(), v_scale.copy()
    nb, hkv, _, dim = k_pool.shape
    n_items = len(src_blocks)
    status = np.zeros(n_items, dtype=np.int32)
    for b in range(n_items):
        s, t = int(src_blocks[b]), int(dst_blocks[b])
        if not (0 <= s < nb and 0 <= t < nb):
            status[b] = ST_BAD_BLOCK
            continue
        kb = (E4M3_TABLE[k_pool[s]].astype(np.float32) * np.float32(k_scale[s])).astype(np.float32)   # [Hkv, 16, D]
        vb = (E4M3_TABLE[v_pool[s]].astype(np.float32) * np.float32(v_scale[s])).astype(np.float32)   # [Hkv, D, 16]
        for tensor in (0, 1):
            for h in range(hkv):
                r = (b * 2 + tensor) * hkv + h
                for e in range(int(res_ptr[r]), int(res_ptr[r + 1])):
                    i = int(res_idx[e])
                    if not (0 <= i < BLOCK * dim):
                        status[b] = ST_BAD_INDEX
                        continue
                    val = bf16_bits_to_f32(np.array([res_val[e]], dtype=np.uint16))[0]
                    slot, d = divmod(i, dim)
                    if tensor == 0:
                        kb[h, slot, d] = np.float32(kb[h, slot, d]) + np.float32(val)
                    else:
                        vb[h, d, slot] = np.float32(vb[h, d, slot]) + np.float32(val)
        for x, pool, scale in ((kb, k_out, ks_out), (vb, v_out, vs_out)):
            amax = np.float32(np.abs(x).max())
            sc = np.float32(amax / np.float32(448.0)) if amax > 0 else np.float32(1.0)
            y = np.clip((x / sc).astype(np.float32), np.float32(-448.0), np.float32(448.0))
            pool[t] = f32_to_e4m3_codes(y)
            scale[t] = sc
    return k_out, v_out, ks_out, vs_out, status


def mask_words(dim: int) -> int:
    """32-bit words of one image's bit mask."""
    return BLOCK * dim // 32


def pack_rows(res_ptr, res_idx, res_val, dim: int):
    """CSR rows -> packed form: (mask uint32 [rows, 16 * dim / 32], values uint16 [nnz]) with the values of a
    row in rising element order (the rows of the CSR may be in any order; they name distinct elements inside
    the image)."""
    rows = len(res_ptr) - 1
    mask = np.zeros((rows, mask_words(dim)), dtype=np.uint32)
    val = np.zeros(len(res_val), dtype=np.uint16)
    for r in range(rows):
        e0, e1 = int(res_ptr[r]), int(res_ptr[r + 1])
        order = np.argsort(np.asarray(res_idx[e0:e1], dtype=np.int64), kind="stable")
        for k, o in enumerate(order):
            i = int(res_idx[e0 + o])
            assert 0 <= i < BLOCK * dim and not (int(mask[r, i // 32]) >> (i % 32)) & 1
            mask[r, i // 32] |= np.uint32(1 << (i % 32))
            val[e0 + k] = res_val[e0 + o]
    return mask, val


def unpack_rows(res_ptr, mask, dim: int) -> np.ndarray:
    """Element indices (uint16, rising inside a row) of a packed residual; row r must hold res_ptr[r+1] -
    res_ptr[r] set bits."""
    idx = np.zeros(int(res_ptr[-1]), dtype=np.uint16)
    for r in range(len(res_ptr) - 1):
        e = int(res_ptr[r])
        for i in range(BLOCK * dim):
            if (int(mask[r, i // 32]) >> (i % 32)) & 1:
                idx[e] = i
                e += 1
        assert e == int(res_ptr[r + 1])
    return idx


def reconstruct_packed(k_pool: np.ndarray, v_pool: np.ndarray, src_blocks, dst_blocks, res_ptr, mask, val):
    """reconstruct() from the packed form, read as the format is defined: the elements of an image are walked in
    rising order and every set bit consumes the next value of its row.  Returns (k_pool', v_pool', status);
    status is ST_BAD_INDEX for an item with a row whose bit count is not its row length (the row is applied as
    far as its values reach)."""
    k_out, v_out = k_pool.copy(), v_pool.copy()
    nb, hkv, _, dim = k_pool.shape
    status = np.zeros(len(src_blocks), dtype=np.int32)
    for b in range(len(src_blocks)):
        s, t = int(src_blocks[b]), int(dst_blocks[b])
        if not (0 <= s < nb and 0 <= t < nb):
            status[b] = ST_BAD_BLOCK
            continue
        kb = bf16_bits_to_f32(k_pool[s]).copy()          # [Hkv, 16, D]
        vb = bf16_bits_to_f32(v_pool[s]).copy()          # [Hkv, D, 16]
        for tensor in (0, 1):
            for h in range(hkv):
                r = (b * 2 + tensor) * hkv + h
                e, e1 = int(res_ptr[r]), int(res_ptr[r + 1])
                for i in range(BLOCK * dim):
                    if not (int(mask[r, i // 32]) >> (i % 32)) & 1:
                        continue
                    if e >= e1:
                        status[b] = ST_BAD_INDEX
                        break
                    delta = bf16_bits_to_f32(np.array([val[e]], dtype=np.uint16))[0]
                    e += 1
                    slot, d = divmod(i, dim)
                    if tensor == 0:
                        kb[h, slot, d] = np.float32(kb[h, slot, d]) + np.float32(delta)
                    else:
                        vb[h, d, slot] = np.float32(vb[h, d, slot]) + np.float32(delta)
                if e != e1:
                    status[b] = ST_BAD_INDEX
        k_out[t] = f32_to_bf16_bits_rne(kb)
        v_out[t] = f32_to_bf16_bits_rne(vb)
    return k_out, v_out, status


def make_residual(k_pool: np.ndarray, v_pool: np.ndarray, base_blocks, full_blocks, share: float = 0.95):
    """From dense prefix-conditioned KV to the stored residual (the paper's sparsity appendix: of the difference
    between the KV of an operation under a prefix and its base KV, keep the largest-magnitude entries that hold
    `share` of its Frobenius energy).  Item b compares block full_blocks[b] (the KV under the prefix) with block
    base_blocks[b]; per (item, tensor, kv head) image the difference is formed in fp32 (full - base, both
    widened exactly), select_by_energy picks the entries, and the kept differences are rounded to bf16.
    Returns the CSR of reconstruct(): (res_ptr, res_idx, res_val) with logical indices slot * D + d, every
    row sorted by index.  Readings: energy is taken per image (the paper measures per layer and head), and the
    stored value is the rounded difference itself, not a value re-fitted so that base + value rounds to full."""
    nb, hkv, _, dim = k_pool.shape
    ptr, idx, val = [0], [], []
    for b in range(len(base_blocks)):
        s, f = int(base_blocks[b]), int(full_blocks[b])
        for tensor in (0, 1):
            for h in range(hkv):
                if tensor == 0:
                    d = bf16_bits_to_f32(k_pool[f, h]) - bf16_bits_to_f32(k_pool[s, h])          # [16, D]
                else:
                    d = (bf16_bits_to_f32(v_pool[f, h]) - bf16_bits_to_f32(v_pool[s, h])).T      # [D, 16] -> [16, D]
                d = np.ascontiguousarray(d, dtype=np.float32)
                keep = select_by_energy(d, share)
                idx.append(keep.astype(np.uint16))
                val.append(f32_to_bf16_bits_rne(d.ravel()[keep]))
                ptr.append(ptr[-1] + keep.size)
    cat = lambda parts, dt: np.concatenate(parts).astype(dt) if parts else np.zeros(0, dt)
    return np.asarray(ptr, dtype=np.int32), cat(idx, np.uint16), cat(val, np.uint16)


def select_by_energy(delta: np.ndarray, share: float = 0.95) -> np.ndarray:
    """Indices (into delta.ravel()) of the fewest largest-magnitude entries whose
    squared sum is at least `share` of the total; ties broken by lower index.
    An all-zero difference keeps nothing.  The total is the end of the same running
    sum the prefixes are taken from (one summation, along the ranking), so that
    share = 1 keeps exactly the non-zero entries whatever the rounding."""
    flat = np.ascontiguousarray(delta, dtype=np.float64).ravel()
    energy = flat * flat
    order = np.lexsort((np.arange(flat.size), -energy))    # by energy descending, then index
    cum = np.cumsum(energy[order])
    total = cum[-1] if cum.size else 0.0
    if total == 0.0:
        return np.zeros(0, dtype=np.int64)
    keep = int(np.searchsorted(cum, share * total, side="left")) + 1
    return np.sort(order[:min(keep, flat.size)])
