"""Pins for the attention oracle (CPU only).  Each test pins the pool-aware fp64
oracle to something other than itself: a pool-free brute force, a closed form,
an invariance the mathematics fixes, or a library routine."""
import numpy as np
import pytest
import torch

from oracle import attention as A
from oracle import bruteforce as BF
from oracle.formats import bf16_bits_to_f64
from paper_2605_22566_amd import workload as W
from tests.helpers import oracle_resolve


def _small(seed, shape=None, **kw):
    shape = shape or W.Shape(4, 2, 16)
    return W.small_layered(seed, shape, **kw)


def _oracle_prefill(wl, t, tables=None, **kw):
    tables = tables or oracle_resolve(wl)
    return A.prefill(t.q, t.q_ptr, t.k_pool, t.v_pool, tables, t.k_scale, t.v_scale, **kw)


@pytest.mark.parametrize("seed,shape", [(1, W.Shape(4, 2, 16)), (2, W.Shape(2, 2, 8)), (3, W.Shape(8, 1, 8))])
def test_matches_pool_free_bruteforce(seed, shape):
    """Full recompute from the per-node source segments (never touches blocks or
    tables) equals the pool-aware oracle, ragged segment lengths included."""
    wl = _small(seed, shape, num_nodes=12, num_layers=4, len_lo=3, len_hi=37, num_req=4, hops=(1, 4),
                new_hi=21)
    t = W.make_tensors(wl)
    O, lse = _oracle_prefill(wl, t)
    qf = bf16_bits_to_f64(t.q)
    b = wl.batch
    for r in range(b.num_req):
        lo, hi = int(t.q_ptr[r]), int(t.q_ptr[r + 1])
        path = b.path_nodes[b.path_ptr[r]:b.path_ptr[r + 1]].tolist()
        o_bf, lse_bf = BF.attend_bruteforce(qf[lo:hi], t.node_k, t.node_v, path, t.new_k[r], t.new_v[r],
                                            shape.group)
        np.testing.assert_allclose(O[lo:hi], np.array(o_bf), rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(lse[lo:hi], np.array(lse_bf), rtol=1e-11, atol=1e-12)


def test_tiny_config_matches_bruteforce_on_one_request():
    wl = W.config_tiny()
    t = W.make_tensors(wl)
    O, lse = _oracle_prefill(wl, t)
    qf = bf16_bits_to_f64(t.q)
    r = 1
    lo, hi = int(t.q_ptr[r]), int(t.q_ptr[r + 1])
    path = wl.batch.path_nodes[wl.batch.path_ptr[r]:wl.batch.path_ptr[r + 1]].tolist()
    o_bf, _ = BF.attend_bruteforce(qf[lo:lo + 3], t.node_k, t.node_v, path, t.new_k[r][:3], t.new_v[r][:3], 1)
    np.testing.assert_allclose(O[lo:lo + 3], np.array(o_bf), rtol=1e-11, atol=1e-12)


def test_uniform_keys_closed_form():
    """All keys equal => softmax is uniform over the visible set => O[i] is the
    plain mean of the visible V rows and lse = s + ln|J_i| (s = common score)."""
    sh = W.Shape(4, 2, 16)
    wl = _small(11, sh)
    t = W.make_tensors(wl, value_mode="uniform_keys")
    tables = oracle_resolve(wl)
    O, lse = _oracle_prefill(wl, t, tables)
    qf = bf16_bits_to_f64(t.q)
    for r in range(wl.batch.num_req):
        K, V = A.materialize_kv(t.k_pool, t.v_pool, tables["block_table"][r], tables["block_ntok"][r],
                                tables["num_blocks"][r])
        ctx = tables["ctx_lens"][r]
        lo = int(t.q_ptr[r])
        for i in range(int(wl.batch.new_lens[r])):
            for h in range(sh.num_q_heads):
                g = h // sh.group
                vis = ctx + i + 1
                np.testing.assert_allclose(O[lo + i, h], V[:vis, g].mean(axis=0), rtol=1e-12, atol=1e-13)
                s = float(qf[lo + i, h] @ K[0, g]) / np.sqrt(sh.head_dim)
                assert abs(lse[lo + i, h] - (s + np.log(vis))) < 1e-10


def test_zero_query_gives_mean_of_values():
    sh = W.Shape(4, 4, 8)
    wl = _small(12, sh)
    t = W.make_tensors(wl)
    t.q[:] = 0
    tables = oracle_resolve(wl)
    O, lse = _oracle_prefill(wl, t, tables)
    r = 0
    _, V = A.materialize_kv(t.k_pool, t.v_pool, tables["block_table"][r], tables["block_ntok"][r],
                            tables["num_blocks"][r])
    ctx = tables["ctx_lens"][r]
    np.testing.assert_allclose(O[0, 2], V[:ctx + 1, 2].mean(axis=0), rtol=1e-12, atol=1e-13)
    assert abs(lse[0, 2] - np.log(ctx + 1)) < 1e-12


def _permute_pool(wl, t, seed):
    """Relabel physical blocks: new id = perm[old id]; move pool rows accordingly."""
    import copy
    rng = np.random.default_rng(seed)
    nb = wl.num_pool_blocks
    perm = rng.permutation(nb)
    wl2 = copy.deepcopy(wl)
    wl2.graph.node_blocks = perm[wl.graph.node_blocks].astype(np.int32)
    wl2.batch.tail_blocks = perm[wl.batch.tail_blocks].astype(np.int32)
    t2 = copy.deepcopy(t)
    t2.k_pool[perm] = t.k_pool
    t2.v_pool[perm] = t.v_pool
    if t.k_scale is not None:
        t2.k_scale[perm] = t.k_scale
        t2.v_scale[perm] = t.v_scale
    return wl2, t2


@pytest.mark.parametrize("dtype", [W.KV_BF16, W.KV_FP8_E4M3])
def test_block_permutation_invariance_bit_identical(dtype):
    wl = _small(21, W.Shape(4, 2, 16, dtype))
    t = W.make_tensors(wl)
    O, lse = _oracle_prefill(wl, t)
    wl2, t2 = _permute_pool(wl, t, 99)
    O2, lse2 = _oracle_prefill(wl2, t2)
    assert np.array_equal(O, O2) and np.array_equal(lse, lse2)


def test_pad_slots_do_not_matter_bit_identical():
    wl = _small(22)
    t1 = W.make_tensors(wl, pad_std=10.0)
    t2 = W.make_tensors(wl, pad_std=1000.0)
    assert not np.array_equal(t1.k_pool, t2.k_pool)      # garbage differs...
    O1, l1 = _oracle_prefill(wl, t1)
    O2, l2 = _oracle_prefill(wl, t2)
    assert np.array_equal(O1, O2) and np.array_equal(l1, l2)   # ...outputs do not


def test_single_aligned_node_equals_torch_sdpa():
    """One block-aligned node + new tokens is plain causal attention with a
    bottom-right mask: compare with torch's scaled_dot_product_attention (fp64,
    CPU, kv heads repeated for GQA)."""
    sh = W.Shape(8, 2, 32)
    rng = np.random.default_rng(31)
    node_len = np.array([48])
    new_lens = np.array([19])
    wl = W._finish("sdpa", sh, node_len, [], [[0]], new_lens, rng, True, 31, np.arange(1), np.zeros(0), 0.0)
    t = W.make_tensors(wl)
    tables = oracle_resolve(wl)
    O, _ = _oracle_prefill(wl, t, tables)
    K = np.concatenate([t.node_k[0], t.new_k[0]]).astype(np.float64)   # [T, Hkv, D]
    V = np.concatenate([t.node_v[0], t.new_v[0]]).astype(np.float64)
    q = torch.from_numpy(bf16_bits_to_f64(t.q)).permute(1, 0, 2)[None]            # [1,Hq,n,D]
    k = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(sh.group, dim=0)[None]
    v = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(sh.group, dim=0)[None]
    n, T = 19, 67
    mask = torch.ones(n, T, dtype=torch.bool).tril(diagonal=T - n)
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=mask)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(O, ref, rtol=1e-10, atol=1e-12)


def test_store_once_equals_private_copies():
    """Eq. 7 with a zero residual: giving every request its own private copy of
    each node's blocks (the stateful layout) changes nothing but the footprint."""
    sh = W.Shape(4, 2, 16)
    wl = _small(41, sh, num_req=5)
    t = W.make_tensors(wl)
    tables = oracle_resolve(wl)
    O, lse = _oracle_prefill(wl, t, tables)
    # build a duplicated pool: every (request, table entry) gets a fresh block
    nb_priv = sum(tables["num_blocks"])
    k2 = np.zeros((nb_priv,) + t.k_pool.shape[1:], t.k_pool.dtype)
    v2 = np.zeros((nb_priv,) + t.v_pool.shape[1:], t.v_pool.dtype)
    priv = {k: [list(x) for x in v] if isinstance(v[0], list) else list(v) for k, v in tables.items()}
    nxt = 0
    for r in range(wl.batch.num_req):
        for e in range(tables["num_blocks"][r]):
            k2[nxt] = t.k_pool[tables["block_table"][r][e]]
            v2[nxt] = t.v_pool[tables["block_table"][r][e]]
            priv["block_table"][r][e] = nxt
            nxt += 1
    O2, lse2 = A.prefill(t.q, t.q_ptr, k2, v2, priv)
    assert np.array_equal(O, O2) and np.array_equal(lse, lse2)
    shared_blocks = len({b for r in range(wl.batch.num_req) for b in tables["block_table"][r][:tables["num_blocks"][r]]})
    assert nb_priv > shared_blocks


def test_split_at_node_boundary_and_merge():
    """Attending each part of the context separately and combining the partials
    with the log-sum-exp merge equals attending the whole."""
    sh = W.Shape(4, 2, 16)
    wl = _small(51, sh, hops=(3, 6))
    t = W.make_tensors(wl)
    tables = oracle_resolve(wl)
    O, lse = _oracle_prefill(wl, t, tables)
    qf = bf16_bits_to_f64(t.q)
    g, b = wl.graph, wl.batch
    for r in range(b.num_req):
        K, V = A.materialize_kv(t.k_pool, t.v_pool, tables["block_table"][r], tables["block_ntok"][r],
                                tables["num_blocks"][r])
        ctx = tables["ctx_lens"][r]
        path = b.path_nodes[b.path_ptr[r]:b.path_ptr[r + 1]]
        cut = int(g.node_len[path[:max(1, len(path) // 2)]].sum())
        if cut >= ctx:
            continue
        lo, hi = int(t.q_ptr[r]), int(t.q_ptr[r + 1])
        n = hi - lo
        # part 1: first `cut` context tokens only (no causal part): emulate with ctx_len=cut and
        # zero new tokens visible -> use full visibility by giving each query row its own pass
        scale = 1.0 / np.sqrt(sh.head_dim)
        for h in range(sh.num_q_heads):
            kv = h // sh.group
            for i in (0, n - 1):
                s = scale * (K[:ctx + i + 1, kv] @ qf[lo + i, h])
                parts = [(s[:cut], V[:cut, kv]), (s[cut:], V[cut:ctx + i + 1, kv])]
                ms = [p[0].max() for p in parts]
                ls = [np.exp(p[0] - m).sum() for p, m in zip(parts, ms)]
                os_ = [np.exp(p[0] - m) @ p[1] for p, m in zip(parts, ms)]
                om, lm = A.merge_partials([np.array(m) for m in ms], [np.array(l) for l in ls],
                                          [o for o in os_])
                np.testing.assert_allclose(om, O[lo + i, h], rtol=1e-11, atol=1e-12)
                assert abs(float(lm) - lse[lo + i, h]) < 1e-10


def test_outputs_in_convex_hull_of_visible_values():
    sh = W.Shape(4, 2, 16)
    wl = _small(61, sh)
    t = W.make_tensors(wl)
    tables = oracle_resolve(wl)
    O, _ = _oracle_prefill(wl, t, tables)
    for r in range(wl.batch.num_req):
        _, V = A.materialize_kv(t.k_pool, t.v_pool, tables["block_table"][r], tables["block_ntok"][r],
                                tables["num_blocks"][r])
        ctx = tables["ctx_lens"][r]
        lo = int(t.q_ptr[r])
        for i in range(int(wl.batch.new_lens[r])):
            for h in range(sh.num_q_heads):
                vis = V[:ctx + i + 1, h // sh.group]
                assert (O[lo + i, h] <= vis.max(axis=0) + 1e-12).all()
                assert (O[lo + i, h] >= vis.min(axis=0) - 1e-12).all()


def test_causality_future_new_tokens_do_not_matter():
    """Changing the K/V of new token j leaves rows i < j untouched and changes row j."""
    sh = W.Shape(2, 1, 16)
    wl = _small(71, sh, num_req=1, new_lo=9, new_hi=9)
    t = W.make_tensors(wl)
    tables = oracle_resolve(wl)
    O, _ = _oracle_prefill(wl, t, tables)
    n = int(wl.batch.new_lens[0])
    j = n - 3
    blk = wl.batch.tail_blocks[j // 16]
    t.k_pool[blk, :, j % 16, :] ^= np.uint16(0x8000)      # flip the sign of new token j's key
    O2, _ = _oracle_prefill(wl, t, tables)
    assert np.array_equal(O[:j], O2[:j])
    assert not np.array_equal(O[j], O2[j])


def test_decode_is_last_row_of_prefill():
    sh = W.Shape(4, 2, 16)
    wl = _small(81, sh, new_lo=1, new_hi=20)
    t = W.make_tensors(wl)
    tables = oracle_resolve(wl)
    O, lse = _oracle_prefill(wl, t, tables)
    last = (t.q_ptr[1:] - 1).astype(np.int64)
    Od, lsed = A.decode(t.q[last], t.k_pool, t.v_pool, tables)
    np.testing.assert_allclose(Od, O[last], rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(lsed, lse[last], rtol=1e-13, atol=1e-14)


def test_fp8_pool_matches_manual_dequant():
    """e4m3 pool: oracle output equals attention over K/V dequantised with
    torch's independent e4m3 cast and the per-block scales."""
    sh = W.Shape(4, 2, 16, W.KV_FP8_E4M3)
    wl = _small(91, sh)
    t = W.make_tensors(wl)
    tables = oracle_resolve(wl)
    O, _ = _oracle_prefill(wl, t, tables)
    kd = torch.from_numpy(t.k_pool).view(torch.float8_e4m3fn).to(torch.float64).numpy() * \
        t.k_scale.astype(np.float64)[:, None, None, None]
    vd = torch.from_numpy(t.v_pool).view(torch.float8_e4m3fn).to(torch.float64).numpy() * \
        t.v_scale.astype(np.float64)[:, None, None, None]
    O2, _ = A.prefill(t.q, t.q_ptr, kd, vd, tables)
    np.testing.assert_allclose(O, O2, rtol=1e-13, atol=1e-14)
    assert np.isfinite(O).all()


def test_sm_scale_override():
    sh = W.Shape(2, 2, 16)
    wl = _small(95, sh, num_req=2)
    t = W.make_tensors(wl)
    tables = oracle_resolve(wl)
    O_default, _ = _oracle_prefill(wl, t, tables)
    O_same, _ = _oracle_prefill(wl, t, tables, sm_scale=0.25)        # 1/sqrt(16)
    O_other, _ = _oracle_prefill(wl, t, tables, sm_scale=0.5)
    assert np.array_equal(O_default, O_same)
    assert not np.allclose(O_default, O_other)
