"""gf_attn_prefill / gf_attn_decode through the C ABI vs the fp64 oracle.
Tolerance (the benchmark spec): |gpu - oracle| <= 1e-2 + 1e-2*|oracle| for bf16 pools."""
import copy

import numpy as np
import pytest
import torch

from paper_2605_22566_amd import runner as R
from paper_2605_22566_amd import workload as W
from tests.gpu_common import (assert_close, bf16_out_to_f64, oracle_decode, oracle_prefill, run_decode, run_prefill,
                              run_resolve)

pytestmark = pytest.mark.gpu

SHAPES = [W.Shape(4, 4, 64), W.Shape(8, 2, 64), W.Shape(32, 8, 128), W.Shape(16, 2, 128), W.Shape(4, 2, 128),
          W.Shape(32, 8, 128, W.KV_FP8_E4M3), W.Shape(8, 1, 128, W.KV_FP8_E4M3), W.Shape(8, 2, 64, W.KV_FP8_E4M3)]


def _sid(s):
    return f"hq{s.num_q_heads}kv{s.num_kv_heads}d{s.head_dim}" + ("fp8" if s.kv_dtype == W.KV_FP8_E4M3 else "")


def test_tiny_config_prefill_and_decode():
    wl = W.config_tiny()
    t = W.make_tensors(wl)
    o, lse, _, _ = run_prefill(wl, t)
    O, LSE = oracle_prefill(wl, t)
    assert_close(o, O, W.KV_BF16, "tiny prefill")
    assert np.abs(lse - LSE).max() < 1e-2
    od, lsed, _, _, last = run_decode(wl, t)
    Od, LSEd = oracle_decode(wl, t, last)
    assert_close(od, Od, W.KV_BF16, "tiny decode")
    assert np.abs(lsed - LSEd).max() < 1e-2


@pytest.mark.parametrize("shape", SHAPES, ids=_sid)
def test_prefill_ragged_small(shape):
    """Ragged node segments (partial blocks mid-sequence), several KV tiles, q
    tiles with a ragged tail, shuffled pool, N(0,100) garbage in pad slots."""
    wl = W.small_layered(100 + shape.num_q_heads + shape.head_dim + shape.kv_dtype, shape, num_nodes=30, num_layers=6, len_lo=3,
                         len_hi=150, num_req=5, hops=(1, 6), new_lo=1, new_hi=150)
    t = W.make_tensors(wl)
    o, lse, _, _ = run_prefill(wl, t)
    O, LSE = oracle_prefill(wl, t)
    assert np.isfinite(o).all()
    assert_close(o, O, shape.kv_dtype, "prefill")
    assert np.abs(lse - LSE).max() < 1e-2


@pytest.mark.parametrize("shape", SHAPES, ids=_sid)
@pytest.mark.parametrize("chunk", [0, 2, 6])
def test_decode_ragged_small(shape, chunk):
    wl = W.small_layered(200 + shape.num_q_heads + shape.head_dim + shape.kv_dtype, shape, num_nodes=30, num_layers=6, len_lo=3,
                         len_hi=150, num_req=7, hops=(1, 6), new_lo=1, new_hi=40)
    t = W.make_tensors(wl)
    od, lsed, _, _, last = run_decode(wl, t, chunk_blocks=chunk)
    Od, LSEd = oracle_decode(wl, t, last)
    assert np.isfinite(od).all()
    assert_close(od, Od, shape.kv_dtype, "decode")
    assert np.abs(lsed - LSEd).max() < 1e-2


def test_empty_context_and_single_token():
    """Requests with an empty path (pure causal self-attention) and 1-token requests."""
    rng = np.random.default_rng(8)
    sh = W.Shape(8, 2, 128)
    node_len = np.array([20, 33])
    wl = W._finish("edge", sh, node_len, [(0, 1)], [[], [0, 1], [], [1]], np.array([37, 1, 1, 70]), rng, True, 8,
                   np.arange(4), np.zeros(0), 0.0)
    t = W.make_tensors(wl)
    o, lse, _, _ = run_prefill(wl, t)
    O, LSE = oracle_prefill(wl, t)
    assert_close(o, O, sh.kv_dtype, "prefill empty ctx")
    od, _, _, _, last = run_decode(wl, t)
    Od, _ = oracle_decode(wl, t, last)
    assert_close(od, Od, sh.kv_dtype, "decode empty ctx")


def test_sm_scale_override_and_no_lse():
    sh = W.Shape(8, 2, 128)
    wl = W.small_layered(77, sh, num_req=3)
    t = W.make_tensors(wl)
    o, lse, _, _ = run_prefill(wl, t, sm_scale=0.05, want_lse=False)
    O, _ = oracle_prefill(wl, t, sm_scale=0.05)
    assert lse is None
    assert_close(o, O, sh.kv_dtype, "prefill sm_scale")


def test_run_to_run_and_block_permutation_bit_identical():
    """The reduction order depends on the logical order only: two runs, and a run
    on a pool with permuted physical blocks, give identical bits."""
    sh = W.Shape(32, 8, 128)
    wl = W.small_layered(55, sh, num_nodes=20, num_layers=5, len_lo=10, len_hi=200, num_req=4, hops=(2, 5),
                         new_lo=5, new_hi=90)
    t = W.make_tensors(wl)
    o1, _, _, _ = run_prefill(wl, t)
    o2, _, _, _ = run_prefill(wl, t)
    assert np.array_equal(o1, o2)
    d1 = run_decode(wl, t)[0]
    rng = np.random.default_rng(1)
    perm = rng.permutation(wl.num_pool_blocks)
    wl2, t2 = copy.deepcopy(wl), copy.deepcopy(t)
    wl2.graph.node_blocks = perm[wl.graph.node_blocks].astype(np.int32)
    wl2.batch.tail_blocks = perm[wl.batch.tail_blocks].astype(np.int32)
    t2.k_pool[perm] = t.k_pool
    t2.v_pool[perm] = t.v_pool
    o3, _, _, _ = run_prefill(wl2, t2)
    assert np.array_equal(o1, o3)
    d3 = run_decode(wl2, t2)[0]
    assert np.array_equal(d1, d3)


def test_failed_requests_are_skipped():
    """A request with a bad edge gets status != 0; prefill leaves its rows alone,
    decode zero-fills them; the others are unaffected."""
    sh = W.Shape(8, 2, 128)
    wl = W.small_layered(66, sh, num_req=4, hops=(3, 5))
    b = wl.batch
    p0, p1 = int(b.path_ptr[1]), int(b.path_ptr[2])
    assert p1 - p0 >= 2
    b.path_nodes[p0:p1] = b.path_nodes[p0:p1][::-1].copy()     # reversed path: edges point the wrong way
    t = W.make_tensors(wl)
    o, _, tables, _ = run_prefill(wl, t)
    assert tables["status"].cpu().tolist()[1] != 0
    lo, hi = int(t.q_ptr[1]), int(t.q_ptr[2])
    assert np.isnan(o[lo:hi]).all()                            # untouched (prefilled with NaN by the harness)
    O, _ = oracle_prefill(wl, t)
    keep = np.ones(o.shape[0], bool)
    keep[lo:hi] = False
    assert_close(o[keep], O[keep], sh.kv_dtype, "prefill others")
    od, lsed, _, _, last = run_decode(wl, t)
    assert (od[1] == 0).all() and np.isneginf(lsed[1]).all()


def test_fp8_block_scales_differ_widely():
    """e4m3 pool whose blocks have very different magnitudes (scales spread over 2^6): the per-block
    K and V scales must be applied per 16-key chunk."""
    sh = W.Shape(8, 2, 128, W.KV_FP8_E4M3)
    wl = W.small_layered(901, sh, num_nodes=20, num_layers=5, len_lo=10, len_hi=120, num_req=4, hops=(2, 5),
                         new_lo=3, new_hi=70)
    t = W.make_tensors(wl)
    rng = np.random.default_rng(4)
    f = (2.0 ** rng.integers(-3, 4, size=t.k_scale.shape[0])).astype(np.float32)
    t.k_scale *= f
    t.v_scale *= f[::-1].copy()
    o, lse, _, _ = run_prefill(wl, t)
    O, LSE = oracle_prefill(wl, t)
    assert_close(o, O, sh.kv_dtype, "fp8 prefill, spread scales")
    od, _, _, _, last = run_decode(wl, t)
    Od, _ = oracle_decode(wl, t, last)
    assert_close(od, Od, sh.kv_dtype, "fp8 decode, spread scales")


@pytest.mark.parametrize("shape", [W.Shape(2, 1, 128, W.KV_FP8_E4M3), W.Shape(4, 1, 128, W.KV_FP8_E4M3),
                                   W.Shape(4, 1, 128), W.Shape(2, 2, 64, W.KV_FP8_E4M3)], ids=_sid)
def test_prefill_many_table_windows(shape):
    """Contexts of more than 260 table entries (the kernel keeps the table in windows of 64 entries per lane
    register set and slides them: at least four slides here, with the per-entry e4m3 scales riding in the
    windows), several q tiles per request, few heads so that the oracle stays fast."""
    wl = W.small_layered(300 + shape.num_q_heads + shape.head_dim + shape.kv_dtype, shape, num_nodes=48, num_layers=8,
                         len_lo=300, len_hi=900, num_req=3, hops=(7, 8), new_lo=70, new_hi=200)
    from tests.helpers import max_blocks_of
    assert max_blocks_of(wl) >= 260 + 5
    t = W.make_tensors(wl)
    o, lse, _, _ = run_prefill(wl, t)
    O, LSE = oracle_prefill(wl, t)
    assert np.isfinite(o).all()
    assert_close(o, O, shape.kv_dtype, "prefill, many windows")
    assert np.abs(lse - LSE).max() < 1e-2
    od, lsed, _, _, last = run_decode(wl, t)
    Od, LSEd = oracle_decode(wl, t, last)
    assert_close(od, Od, shape.kv_dtype, "decode, long context")


def test_decode_entries_without_tokens_give_zero_rows():
    """A valid request whose table entries all carry zero tokens has nothing to attend to: zero row and
    lse = -inf, never NaN (every partial of it has a zero sum).  The other requests are unaffected."""
    from tests.gpu_common import run_resolve
    sh = W.Shape(8, 2, 128)
    wl = W.small_layered(91, sh, num_nodes=20, num_layers=5, len_lo=10, len_hi=120, num_req=4, hops=(2, 5),
                         new_lo=3, new_hi=40)
    t = W.make_tensors(wl)
    sess, tables = run_resolve(wl)
    tables["block_ntok"][1].zero_()
    for chunk in (0, 2):
        od, lsed, _, _, last = run_decode(wl, t, chunk_blocks=chunk, tables=tables, sess=sess)
        assert np.isfinite(od).all()
        assert (od[1] == 0).all() and np.isneginf(lsed[1]).all()
        Od, _ = oracle_decode(wl, t, last)
        keep = np.array([0, 2, 3])
        assert_close(od[keep], Od[keep], sh.kv_dtype, "decode, others")


def test_one_context_through_growing_batches():
    """A context's workspace grows three times here (2, 5 and 12 requests through the same gf_ctx, then 3 again):
    every call gives the rows a call on a fresh context gives."""
    sh = W.Shape(8, 2, 128)
    wl = W.small_layered(77, sh, num_nodes=24, num_layers=6, len_lo=20, len_hi=300, num_req=12, hops=(2, 5),
                         new_lo=1, new_hi=4)
    t = W.make_tensors(wl)
    want = run_decode(wl, t)[0]
    sess, tables = run_resolve(wl)
    dev = sess.device
    pool = R.DevicePool.from_host(t, dev)
    last = (t.q_ptr[1:] - 1).astype(np.int64)
    qd = R.bits_to_device(np.ascontiguousarray(t.q[last]), dev)
    for n in (2, 5, 12, 3):
        sub = {k: tables[k][:n] for k in ("block_table", "block_ntok", "num_blocks", "ctx_lens", "seq_lens", "status")}
        sub["num_req"], sub["max_blocks"] = n, tables["max_blocks"]
        o = torch.full((n,) + tuple(qd.shape[1:]), float("nan"), dtype=torch.bfloat16, device=dev)
        sess.decode(pool, sub, qd[:n], o)
        torch.cuda.synchronize()
        assert np.array_equal(bf16_out_to_f64(o), want[:n]), n

