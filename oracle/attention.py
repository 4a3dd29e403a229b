"""Attention oracle over the shared paged pool (numpy, fp64).

What it computes, in the paper's terms: the "stateful" view of a request (the
full KV of its prefix path, Topology-Aware State Management section) is
materialised by walking the request's block table over the store-once pool
(Eq. 7 with the residual identically zero), and the new tokens then attend to
it with ordinary scaled-dot-product softmax attention.  New token i sees every
context token and new tokens 0..i (bottom-right causal alignment); query head h
reads kv head h // G.

Steps, in this order and nothing else: materialise -> scores -> max -> exp ->
normalise -> weighted sum.  No blocking, no online softmax, no reordering.

Pool layout understood here (block size 16):
  K[blk, kv_head, slot, d]      V[blk, kv_head, d, slot]
bf16 pools arrive as uint16 bit patterns, e4m3 pools as uint8 codes with one
fp32 scale per block and tensor.

Pins: tests/test_oracle_attention.py (pool-free brute force on tiny graphs,
uniform-key closed form, block-permutation invariance, torch SDPA special case,
private-copy equivalence, split/merge invariance, convex hull, pad independence).
"""
import numpy as np

from .formats import bf16_bits_to_f64, e4m3_codes_to_f64

BLOCK = 16


def _widen(x, scale_per_block=None):
    """Stored pool/Q values -> fp64.  uint16 = bf16 bits, uint8 = e4m3 codes."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return bf16_bits_to_f64(x)
    if x.dtype == np.uint8:
        v = e4m3_codes_to_f64(x)
        if scale_per_block is not None:
            s = np.asarray(scale_per_block, dtype=np.float32).astype(np.float64)
            v = v * s.reshape((-1,) + (1,) * (v.ndim - 1))
        return v
    return x.astype(np.float64)


def materialize_kv(k_pool, v_pool, table_row, ntok_row, num_blocks, k_scale=None, v_scale=None):
    """Concatenate the first ntok slots of every block of one request.
    Returns K, V as fp64 [T, Hkv, D]."""
    ks, vs = [], []
    for e in range(int(num_blocks)):
        blk = int(table_row[e])
        n = int(ntok_row[e])
        kb = _widen(k_pool[blk:blk + 1], None if k_scale is None else k_scale[blk:blk + 1])[0]
        vb = _widen(v_pool[blk:blk + 1], None if v_scale is None else v_scale[blk:blk + 1])[0]
        ks.append(np.transpose(kb[:, :n, :], (1, 0, 2)))     # [n, Hkv, D]
        vs.append(np.transpose(vb[:, :, :n], (2, 0, 1)))     # [n, Hkv, D]
    hkv, d = k_pool.shape[1], k_pool.shape[3]
    if not ks:
        return np.zeros((0, hkv, d)), np.zeros((0, hkv, d))
    return np.concatenate(ks, axis=0), np.concatenate(vs, axis=0)


def attend(q, K, V, ctx_len, sm_scale=None):
    """q: fp64 [n, Hq, D] new-token queries; K, V: fp64 [ctx_len + n, Hkv, D].
    Returns (O [n, Hq, D], lse [n, Hq]) in fp64; lse is the natural-log
    log-sum-exp of the scaled scores over the visible set."""
    n, hq, d = q.shape
    hkv = K.shape[1]
    g = hq // hkv
    scale = (1.0 / np.sqrt(d)) if not sm_scale else float(sm_scale)
    T = K.shape[0]
    assert T == ctx_len + n
    O = np.zeros((n, hq, d))
    lse = np.zeros((n, hq))
    if n == 0:
        return O, lse
    # visible[i, j] : j < ctx_len  or  j - ctx_len <= i
    j = np.arange(T)[None, :]
    i = np.arange(n)[:, None]
    visible = (j < ctx_len) | (j - ctx_len <= i)
    for h in range(hq):
        kv = h // g
        s = scale * (q[:, h, :] @ K[:, kv, :].T)            # [n, T]
        s = np.where(visible, s, -np.inf)
        m = s.max(axis=1, keepdims=True)
        p = np.exp(s - m)
        l = p.sum(axis=1, keepdims=True)
        O[:, h, :] = (p @ V[:, kv, :]) / l
        lse[:, h] = (m + np.log(l))[:, 0]
    return O, lse


def prefill(q_bits, q_ptr, k_pool, v_pool, tables, k_scale=None, v_scale=None, sm_scale=None,
            req_ids=None):
    """Prefill attention for the requests of a resolved batch.
    q_bits: uint16 [total_q, Hq, D]; q_ptr: [R+1]; tables: dict from
    oracle.resolve.resolve_paths.  Requests with a non-zero status produce
    nothing.  Returns (O fp64 [total_q, Hq, D], lse fp64 [total_q, Hq])."""
    qf = _widen(q_bits)
    O = np.zeros(qf.shape)
    lse = np.zeros(qf.shape[:2])
    R = len(q_ptr) - 1
    for r in (range(R) if req_ids is None else req_ids):
        if tables["status"][r] != 0:
            continue
        lo, hi = int(q_ptr[r]), int(q_ptr[r + 1])
        K, V = materialize_kv(k_pool, v_pool, tables["block_table"][r], tables["block_ntok"][r],
                              tables["num_blocks"][r], k_scale, v_scale)
        ctx = int(tables["ctx_lens"][r])
        assert K.shape[0] == int(tables["seq_lens"][r]) and hi - lo == K.shape[0] - ctx
        O[lo:hi], lse[lo:hi] = attend(qf[lo:hi], K, V, ctx, sm_scale)
    return O, lse


def decode(q_bits, k_pool, v_pool, tables, k_scale=None, v_scale=None, sm_scale=None, req_ids=None):
    """Decode attention: request r has one query (q_bits[r]) which is the last
    of its seq_len tokens and therefore sees all of them.
    Returns (O fp64 [R, Hq, D], lse fp64 [R, Hq])."""
    qf = _widen(q_bits)
    O = np.zeros(qf.shape)
    lse = np.zeros(qf.shape[:2])
    for r in (range(qf.shape[0]) if req_ids is None else req_ids):
        if tables["status"][r] != 0:
            continue
        K, V = materialize_kv(k_pool, v_pool, tables["block_table"][r], tables["block_ntok"][r],
                              tables["num_blocks"][r], k_scale, v_scale)
        T = K.shape[0]
        assert T == int(tables["seq_lens"][r]) and T >= 1
        o, l = attend(qf[r:r + 1], K, V, T - 1, sm_scale)
        O[r], lse[r] = o[0], l[0]
    return O, lse


def merge_partials(m_parts, l_parts, o_parts):
    """Combine softmax partials of disjoint key sets (the split-KV merge).
    m_parts[s]: max scaled score of part s; l_parts[s]: sum exp(score - m_s);
    o_parts[s]: sum exp(score - m_s) * v (unnormalised), shape [..., D].
    Returns (O, lse)."""
    m = np.max(np.stack(m_parts), axis=0)
    l = sum(lp * np.exp(mp - m) for mp, lp in zip(m_parts, l_parts))
    o = sum(op * np.exp(mp - m)[..., None] for mp, op in zip(m_parts, o_parts))
    return o / l[..., None], m + np.log(l)
