"""gf_attn_decode_shared (node-centric decode) through the C ABI vs the fp64 oracle of the decode
step -- the same plain definition gf_attn_decode is held to, at the same tolerance -- on batches
whose paths overlap a little, a lot, not at all, and on the degenerate cases of the list building."""
import numpy as np
import pytest

from paper_2605_22566_amd import workload as W
from tests.gpu_common import assert_close, oracle_decode, run_decode

pytestmark = pytest.mark.gpu

SHAPES = [W.Shape(4, 4, 64), W.Shape(8, 2, 64), W.Shape(32, 8, 128), W.Shape(16, 2, 128), W.Shape(4, 2, 128),
          W.Shape(32, 8, 128, W.KV_FP8_E4M3), W.Shape(8, 1, 128, W.KV_FP8_E4M3), W.Shape(8, 2, 64, W.KV_FP8_E4M3)]


def _sid(s):
    return f"hq{s.num_q_heads}kv{s.num_kv_heads}d{s.head_dim}" + ("fp8" if s.kv_dtype == W.KV_FP8_E4M3 else "")


def _check(wl, t, what, **kw):
    od, lsed, tables, _, last = run_decode(wl, t, shared=True, **kw)
    Od, LSEd = oracle_decode(wl, t, last)
    assert np.isfinite(od).all(), what
    assert_close(od, Od, wl.shape.kv_dtype, what)
    assert np.abs(lsed - LSEd).max() < 1e-2, what
    return od, lsed, tables


def test_tiny_config():
    wl = W.config_tiny()
    _check(wl, W.make_tensors(wl), "tiny")


@pytest.mark.parametrize("shape", SHAPES, ids=_sid)
@pytest.mark.parametrize("chunk", [0, 2, 6])
def test_ragged_small(shape, chunk):
    """Ragged node segments, nodes longer and shorter than a chunk, tails of 1..3 blocks."""
    wl = W.small_layered(300 + shape.num_q_heads + shape.head_dim + shape.kv_dtype, shape, num_nodes=30, num_layers=6,
                         len_lo=3, len_hi=150, num_req=7, hops=(1, 6), new_lo=1, new_hi=40)
    _check(wl, W.make_tensors(wl), "ragged", chunk_blocks=chunk)


@pytest.mark.parametrize("shape", [W.Shape(4, 4, 64), W.Shape(8, 2, 128), W.Shape(16, 2, 128),
                                   W.Shape(8, 2, 128, W.KV_FP8_E4M3)], ids=_sid)
def test_many_requests_through_few_nodes(shape):
    """More (request, head) columns per node than one wave takes: several column groups per node,
    the last one partly filled; few nodes, so every node list is long."""
    wl = W.small_layered(410 + shape.num_q_heads, shape, num_nodes=8, num_layers=4, len_lo=20, len_hi=90, num_req=45,
                         hops=(1, 4), new_lo=1, new_hi=20)
    cnt = np.bincount(wl.batch.path_nodes, minlength=wl.graph.num_nodes)
    assert (cnt * shape.group > 16).any()
    _check(wl, W.make_tensors(wl), "many through few", chunk_blocks=4)


def test_empty_paths_single_tokens_and_a_node_visited_twice():
    rng = np.random.default_rng(18)
    sh = W.Shape(8, 2, 128)
    node_len = np.array([20, 33, 0, 16])
    paths = [[], [0, 1, 0], [], [1, 0, 1, 0], [3], [0, 2, 3]]
    edges = [(0, 1), (1, 0), (0, 2), (2, 3)]
    wl = W._finish("edge", sh, node_len, edges, paths, np.array([37, 1, 1, 70, 16, 17]), rng, True, 18,
                   np.arange(len(paths)), np.zeros(0), 0.0)
    _, _, tables = _check(wl, W.make_tensors(wl), "degenerate paths", chunk_blocks=2)
    assert tables["status"].cpu().tolist() == [0] * len(paths)


def test_failed_requests_get_zero_rows_and_do_not_disturb_the_others():
    sh = W.Shape(8, 2, 128)
    wl = W.small_layered(66, sh, num_req=6, hops=(3, 5))
    t = W.make_tensors(wl)
    b = wl.batch
    for r in (1, 4):
        p0, p1 = int(b.path_ptr[r]), int(b.path_ptr[r + 1])
        assert p1 - p0 >= 2
        b.path_nodes[p0:p1] = b.path_nodes[p0:p1][::-1].copy()     # reversed path: edges point the wrong way
    od, lsed, tables, _, last = run_decode(wl, t, shared=True)
    st = tables["status"].cpu().tolist()
    assert st[1] != 0 and st[4] != 0 and sum(s != 0 for s in st) == 2
    for r in (1, 4):
        assert (od[r] == 0).all() and np.isneginf(lsed[r]).all()
    Od, _ = oracle_decode(wl, t, last)
    keep = np.array([s == 0 for s in st])
    assert_close(od[keep], Od[keep], sh.kv_dtype, "others")


def test_bit_identical_run_to_run_and_close_to_the_per_request_kernel():
    """The node lists are filled through atomics, so their order may differ between runs; the
    values may not.  The per-request kernel reduces the same chunks in another grouping."""
    sh = W.Shape(32, 8, 128)
    wl = W.small_layered(57, sh, num_nodes=12, num_layers=4, len_lo=10, len_hi=200, num_req=40, hops=(2, 4),
                         new_lo=1, new_hi=30)
    t = W.make_tensors(wl)
    runs = [run_decode(wl, t, shared=True)[0] for _ in range(3)]
    assert np.array_equal(runs[0], runs[1]) and np.array_equal(runs[0], runs[2])
    per_request = run_decode(wl, t)[0]
    assert np.abs(runs[0] - per_request).max() <= 2.0 ** -7 * max(1.0, np.abs(per_request).max())


def test_plan_once_then_several_layers():
    """gf_decode_shared_plan + gf_attn_decode_shared_planned: the lists are built once and serve several
    'layers' (other pools, other queries); each result is the one-shot call's, bit for bit.  Without lists,
    or with lists of another batch, the planned call is refused."""
    import torch
    from paper_2605_22566_amd import binding as B
    from paper_2605_22566_amd import runner as R
    from tests.gpu_common import run_resolve
    sh = W.Shape(32, 8, 128)
    wl = W.small_layered(58, sh, num_nodes=12, num_layers=4, len_lo=10, len_hi=200, num_req=20, hops=(2, 4),
                         new_lo=1, new_hi=30)
    sess, tables = run_resolve(wl)
    db = sess.upload_batch(wl.batch)
    dev = sess.device
    pool0 = R.DevicePool.from_host(W.make_tensors(wl), dev)
    q0 = torch.zeros((wl.batch.num_req, sh.num_q_heads, sh.head_dim), dtype=torch.bfloat16, device=dev)
    with pytest.raises(B.GraphFlowError) as e:
        sess.decode_shared_planned(pool0, db, tables, q0, torch.zeros_like(q0))      # nothing planned yet
    assert e.value.code == B.GF_ERR_BAD_SHAPE
    sess.decode_shared_plan(pool0, db, tables)
    gen = torch.Generator(device=dev)
    gen.manual_seed(5)
    oneshot = R.Session(wl)                                         # a context of its own: leaves the plan alone
    db1 = oneshot.upload_batch(wl.batch)
    for layer in range(3):
        pool = R.DevicePool.random(wl, dev, seed=100 + layer) if layer else pool0
        q = torch.randn((wl.batch.num_req, sh.num_q_heads, sh.head_dim), generator=gen, device=dev).to(torch.bfloat16)
        o1, o2 = torch.zeros_like(q), torch.zeros_like(q)
        sess.decode_shared_planned(pool, db, tables, q, o1)
        oneshot.decode_shared(pool, db1, tables, q, o2)
        torch.cuda.synchronize()
        assert torch.equal(o1, o2), layer
    other = sess.upload_batch(wl.batch)                             # same contents, other arrays: not the planned batch
    with pytest.raises(B.GraphFlowError) as e:
        sess.decode_shared_planned(pool0, other, tables, q0, torch.zeros_like(q0))
    assert e.value.code == B.GF_ERR_BAD_SHAPE


def test_long_nodes_and_an_oversized_chunk_setting():
    """Nodes longer than a chunk (several chunks per node, ragged last one) at the default setting, and a
    chunk setting above the kernel's limit of 64 entries, which the call clamps."""
    sh = W.Shape(8, 2, 128)
    wl = W.small_layered(91, sh, num_nodes=6, num_layers=3, len_lo=1030, len_hi=2300, num_req=6, hops=(1, 3),
                         new_lo=1, new_hi=20)
    t = W.make_tensors(wl)
    _check(wl, t, "long nodes, default chunk")
    _check(wl, t, "long nodes, chunk 128 asked", chunk_blocks=128)
