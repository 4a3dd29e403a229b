"""Oracle for the KV write path: the K/V of a request's new tokens are written into
its private tail blocks (paper, Topology-Aware State Management: the states of the
tokens a workflow produces at run time extend the KV assembled from its operation
nodes; Effective Path Pruning: a state that is not stored is computed on the fly and
then has to be put where attention reads it).  TEST INFRASTRUCTURE ONLY.

What is computed, per request r with n new tokens and table entries from
oracle.resolve (its last ceil(n/16) entries are the tail blocks):
  token i goes to tail block i // 16, slot i % 16:
      K[block][h][slot][d] = k_new[i][h][d]        V[block][h][d][slot] = v_new[i][h][d]
  slots at or beyond the block's token count are written as zero (a block that was
  never written before must not be left with arbitrary bits, the pool contract
  wants finite values there).
bf16 pool: the bits are copied.  e4m3 pool (per block and tensor one fp32 scale):
      amax  = max |x| over the block's valid tokens, all kv heads, all d
      scale = amax / 448 in fp32 (1.0 for an all-zero block)
      code  = e4m3( clamp(x / scale, -448, 448) ), fp32 division, round to nearest even
-- the stored code is a quantisation decision, so it is taken in the kernel's
precision (fp32), not in fp64.  Requests with a non-zero status, or whose row count
does not match the table, are skipped; a tail block id outside the pool is skipped.

Readings: the paper does not describe the write path at all; the layout is the pool's
(see oracle.attention), the scale rule is the one the synthetic e4m3 pools are built
with, and append() always writes a request's whole tail (growing a block in place is
append_token(), below).

Decode-step form, append_token(): only a request's newest token (index n-1 of its new
tokens, the one seq_lens already counts) is written, into the last table entry's block at
slot s = (n-1) % 16.  With s == 0 the block is fresh: it is zeroed and, for e4m3, gets the
scale amax/448 of the token (1.0 if zero).  With s > 0 (e4m3) the block grows in place:
      need = amax(token) / 448                    old = scale[block]
      need <= old : the token is quantised with the old scale, nothing else changes
      need >  old : scale[block] = need, and every code c in slots [0, s) is re-quantised,
                    c' = e4m3( clamp( (decode(c) * old) / need ) ), fp32 product, fp32
                    division, round to nearest even; the token is quantised with `need`
(per tensor, K and V on their own).  Reading: the paper says nothing about growing a
quantised block; this rule keeps one scale per block and tensor and pays one extra
rounding of the older codes each time the scale has to grow.

Pins (tests/test_oracle_append.py): e4m3 rounding against torch's float8_e4m3fn cast
on random values and on every midpoint between neighbouring codes; append followed
by the attention oracle's table walk returns the new tokens' K/V exactly (bf16) or
within half a code step (e4m3), token by token; block scale and codes against torch's
cast of the same block; pad slots zero; untouched blocks untouched; skipped requests.
append_token: bf16 token by token equals the whole-tail append bit for bit; the table walk
reads the token back; e4m3 without growth leaves scale and older codes alone and codes the
token like torch's cast; e4m3 growth sets amax/448 and re-codes like torch's casts of the
same products, within half a code step of the new grid; a fresh block is zero elsewhere.
"""
import numpy as np

from .formats import E4M3_TABLE

BLOCK = 16
_POS = E4M3_TABLE[:0x7F].astype(np.float32)          # codes 0x00..0x7E: 0 .. 448, ascending


def f32_to_e4m3_codes(y: np.ndarray) -> np.ndarray:
    """fp32 (|y| <= 448) -> e4m3 code, round to nearest, ties to the even code."""
    y = np.ascontiguousarray(y, dtype=np.float32)
    a = np.abs(y).astype(np.float64)
    hi = np.searchsorted(_POS.astype(np.float64), a, side="left")       # first code with value >= a
    hi = np.clip(hi, 0, 0x7E)
    lo = np.clip(hi - 1, 0, 0x7E)
    dlo = a - _POS[lo].astype(np.float64)
    dhi = _POS[hi].astype(np.float64) - a
    pick_hi = (dhi < dlo) | ((dhi == dlo) & (hi % 2 == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    sign = (y.view(np.uint32) >> np.uint32(31)).astype(np.uint8) << np.uint8(7)
    return (code | sign).astype(np.uint8)


def _bf16_to_f32(bits):
    return (np.ascontiguousarray(bits).astype(np.uint32) << np.uint32(16)).view(np.float32)


def append(k_pool, v_pool, k_scale, v_scale, tables, k_new_bits, v_new_bits, q_ptr):
    """k_pool [nb, Hkv, 16, D], v_pool [nb, Hkv, D, 16]: uint16 (bf16 bits) or uint8 (e4m3 codes, then
    k_scale / v_scale fp32 [nb]); k_new_bits / v_new_bits uint16 [total_q, Hkv, D].
    Returns new (k_pool, v_pool, k_scale, v_scale); the inputs are not modified."""
    fp8 = k_pool.dtype == np.uint8
    k_out, v_out = k_pool.copy(), v_pool.copy()
    ks = None if k_scale is None else k_scale.copy()
    vs = None if v_scale is None else v_scale.copy()
    nb = k_pool.shape[0]
    for r in range(len(tables["status"])):
        if tables["status"][r] != 0:
            continue
        n = tables["seq_lens"][r] - tables["ctx_lens"][r]
        q0 = int(q_ptr[r])
        if n <= 0 or int(q_ptr[r + 1]) - q0 != n:
            continue
        nblk = tables["num_blocks"][r]
        ntail = (n + BLOCK - 1) // BLOCK
        for j in range(ntail):
            blk = tables["block_table"][r][nblk - ntail + j]
            if not (0 <= blk < nb):
                continue
            ntok = min(BLOCK, n - j * BLOCK)
            kb = k_new_bits[q0 + j * BLOCK: q0 + j * BLOCK + ntok]       # [ntok, Hkv, D]
            vb = v_new_bits[q0 + j * BLOCK: q0 + j * BLOCK + ntok]
            for pool, scale, src, is_v in ((k_out, ks, kb, False), (v_out, vs, vb, True)):
                if fp8:
                    x = _bf16_to_f32(src)
                    amax = np.float32(np.abs(x).max())
                    s = np.float32(amax / np.float32(448.0)) if amax > 0 else np.float32(1.0)
                    y = np.clip((x / s).astype(np.float32), np.float32(-448.0), np.float32(448.0))
                    vals = f32_to_e4m3_codes(y)
                    scale[blk] = s
                else:
                    vals = src
                pool[blk] = 0
                if is_v:
                    pool[blk][:, :, :ntok] = np.transpose(vals, (1, 2, 0))
                else:
                    pool[blk][:, :ntok, :] = np.transpose(vals, (1, 0, 2))
    return k_out, v_out, ks, vs


def append_token(k_pool, v_pool, k_scale, v_scale, tables, k_tok_bits, v_tok_bits):
    """Decode-step append: k_tok_bits / v_tok_bits uint16 [num_req, Hkv, D] hold the K/V of every
    request's newest token.  Pools and scales as in append().  Returns new (k_pool, v_pool,
    k_scale, v_scale); the inputs are not modified."""
    fp8 = k_pool.dtype == np.uint8
    k_out, v_out = k_pool.copy(), v_pool.copy()
    ks = None if k_scale is None else k_scale.copy()
    vs = None if v_scale is None else v_scale.copy()
    nb = k_pool.shape[0]
    for r in range(len(tables["status"])):
        if tables["status"][r] != 0:
            continue
        n = tables["seq_lens"][r] - tables["ctx_lens"][r]
        nblk = tables["num_blocks"][r]
        if n <= 0 or nblk <= 0:
            continue
        blk = tables["block_table"][r][nblk - 1]
        if not (0 <= blk < nb):
            continue
        slot = (n - 1) % BLOCK
        for pool, scale, src, is_v in ((k_out, ks, k_tok_bits[r], False), (v_out, vs, v_tok_bits[r], True)):
            if slot == 0:
                pool[blk] = 0
            if fp8:
                x = _bf16_to_f32(src)                                      # [Hkv, D]
                amax = np.float32(np.abs(x).max())
                need = np.float32(amax / np.float32(448.0))
                if slot == 0:
                    sc = need if amax > 0 else np.float32(1.0)
                else:
                    old = np.float32(scale[blk])
                    if need > old:
                        sc = need
                        codes = pool[blk][:, :, :slot] if is_v else pool[blk][:, :slot, :]
                        y = (E4M3_TABLE[codes].astype(np.float32) * old).astype(np.float32)
                        y = np.clip((y / sc).astype(np.float32), np.float32(-448.0), np.float32(448.0))
                        if is_v:
                            pool[blk][:, :, :slot] = f32_to_e4m3_codes(y)
                        else:
                            pool[blk][:, :slot, :] = f32_to_e4m3_codes(y)
                    else:
                        sc = old
                scale[blk] = sc
                vals = f32_to_e4m3_codes(np.clip((x / sc).astype(np.float32), np.float32(-448.0), np.float32(448.0)))
            else:
                vals = src
            if is_v:
                pool[blk][:, :, slot] = vals
            else:
                pool[blk][:, slot, :] = vals
    return k_out, v_out, ks, vs
