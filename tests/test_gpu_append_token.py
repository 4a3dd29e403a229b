"""gf_kv_append_token through the C ABI vs oracle/append.py's append_token: a token-by-token trace whose
pools and scales stay bit-identical to the oracle's at every step (fresh blocks, in-place growth of e4m3
blocks with and without a larger scale), and the decode loop resolve -> append_token -> decode."""
import copy

import numpy as np
import pytest
import torch

from oracle import append as OP
from oracle import attention as OA
from paper_2605_22566_amd import runner as R
from paper_2605_22566_amd import workload as W
from tests.gpu_common import assert_close, bf16_out_to_f64
from tests.helpers import max_blocks_of, oracle_resolve

pytestmark = pytest.mark.gpu

SHAPES = [W.Shape(8, 2, 64), W.Shape(32, 8, 128), W.Shape(4, 1, 128), W.Shape(32, 8, 128, W.KV_FP8_E4M3),
          W.Shape(8, 2, 64, W.KV_FP8_E4M3)]


def _sid(s):
    return f"kv{s.num_kv_heads}d{s.head_dim}" + ("fp8" if s.kv_dtype == W.KV_FP8_E4M3 else "")


def _pool_host(pool):
    if pool.k.dtype == torch.bfloat16:
        return R.bf16_to_bits(pool.k), R.bf16_to_bits(pool.v), None, None
    return pool.k.cpu().numpy(), pool.v.cpu().numpy(), pool.k_scale.cpu().numpy(), pool.v_scale.cpu().numpy()


def _trace(shape, seed, steps, spread):
    """A batch whose requests gain one token per step; yields per step the workload at that length, the
    token rows and the decode queries."""
    wl = W.small_layered(seed, shape, num_nodes=16, num_layers=4, len_lo=3, len_hi=80, num_req=5, hops=(1, 4),
                         new_lo=steps, new_hi=steps + 1)           # tail lists long enough for `steps` tokens
    t = W.make_tensors(wl)
    rng = np.random.default_rng(seed + 1)
    R_ = wl.batch.num_req
    # magnitudes wander over the trace so that e4m3 scales sometimes have to grow and sometimes not
    mag = (np.float32(4.0) ** rng.integers(-2, 3, (steps, R_, 1, 1))) if spread else np.ones((steps, R_, 1, 1), np.float32)
    ktok = W.f32_to_bf16_bits((rng.standard_normal((steps, R_, shape.num_kv_heads, shape.head_dim)) * mag).astype(np.float32))
    vtok = W.f32_to_bf16_bits((rng.standard_normal((steps, R_, shape.num_kv_heads, shape.head_dim)) * mag[::-1]).astype(np.float32))
    qtok = W.f32_to_bf16_bits(rng.standard_normal((steps, R_, shape.num_q_heads, shape.head_dim)).astype(np.float32))
    return wl, t, ktok, vtok, qtok


def _at(wl, n):
    w2 = copy.deepcopy(wl)
    w2.batch.new_lens = np.full(wl.batch.num_req, n, dtype=np.int32)
    return w2


@pytest.mark.parametrize("shape", SHAPES, ids=_sid)
def test_token_trace_is_bit_exact_at_every_step(shape):
    steps = 35                                                     # two block boundaries
    wl, t, ktok, vtok, _ = _trace(shape, 70 + shape.head_dim + shape.kv_dtype, steps, spread=True)
    sess = R.Session(wl)
    dev = sess.device
    pool = R.DevicePool.from_host(t, dev)
    mb = max_blocks_of(wl)
    hk, hv, hks, hvs = t.k_pool, t.v_pool, t.k_scale, t.v_scale
    grew = 0
    for i in range(steps):
        w_i = _at(wl, i + 1)
        tables = sess.resolve(sess.upload_batch(w_i.batch), sess.alloc_tables(wl.batch.num_req, mb))
        sess.append_token(pool, tables, R.bits_to_device(ktok[i], dev), R.bits_to_device(vtok[i], dev))
        torch.cuda.synchronize()
        want = OP.append_token(hk, hv, hks, hvs, oracle_resolve(w_i, max_blocks=mb), ktok[i], vtok[i])
        if hks is not None and i % 16 != 0:
            grew += int((want[2] > hks).sum())
        hk, hv, hks, hvs = want
        got = _pool_host(pool)
        assert np.array_equal(got[0], hk), f"K pool differs at step {i}"
        assert np.array_equal(got[1], hv), f"V pool differs at step {i}"
        if hks is not None:
            assert np.array_equal(got[2], hks) and np.array_equal(got[3], hvs), f"scales differ at step {i}"
    if hks is not None:
        assert grew > 5                                            # the growth path was exercised


@pytest.mark.parametrize("shape", [W.Shape(32, 8, 128), W.Shape(8, 2, 64, W.KV_FP8_E4M3)], ids=_sid)
def test_decode_loop_resolve_append_token_decode(shape):
    """Every step: one more token per request, written by gf_kv_append_token, then a decode step whose output
    matches the attention oracle run on the oracle's own pools of that step."""
    steps = 20
    wl, t, ktok, vtok, qtok = _trace(shape, 90 + shape.kv_dtype, steps, spread=False)
    sess = R.Session(wl)
    dev = sess.device
    pool = R.DevicePool.from_host(t, dev)
    mb = max_blocks_of(wl)
    hk, hv, hks, hvs = t.k_pool, t.v_pool, t.k_scale, t.v_scale
    for i in range(steps):
        w_i = _at(wl, i + 1)
        db = sess.upload_batch(w_i.batch)
        tables = sess.resolve(db, sess.alloc_tables(wl.batch.num_req, mb))
        sess.append_token(pool, tables, R.bits_to_device(ktok[i], dev), R.bits_to_device(vtok[i], dev))
        q = R.bits_to_device(qtok[i], dev)
        o, o2 = torch.zeros_like(q), torch.zeros_like(q)
        sess.decode(pool, tables, q, o)
        sess.decode_shared(pool, db, tables, q, o2)
        torch.cuda.synchronize()
        want_t = oracle_resolve(w_i, max_blocks=mb)
        hk, hv, hks, hvs = OP.append_token(hk, hv, hks, hvs, want_t, ktok[i], vtok[i])
        if i in (0, 7, 15, 16, 19):
            O, _ = OA.decode(qtok[i], hk, hv, want_t, hks, hvs)
            assert_close(bf16_out_to_f64(o), O, shape.kv_dtype, f"decode at step {i}")
            assert_close(bf16_out_to_f64(o2), O, shape.kv_dtype, f"node-centric decode at step {i}")


def test_failed_and_empty_requests_are_left_alone():
    shape = W.Shape(8, 2, 64, W.KV_FP8_E4M3)
    wl, t, ktok, vtok, _ = _trace(shape, 77, 3, spread=True)
    w_i = _at(wl, 2)
    w_i.batch.new_lens[3] = 0                                     # no new token: nothing to write
    b = w_i.batch
    p0, p1 = int(b.path_ptr[1]), int(b.path_ptr[2])
    if p1 - p0 >= 2:
        b.path_nodes[p0:p1] = b.path_nodes[p0:p1][::-1].copy()     # a failed request
    sess = R.Session(wl)
    pool = R.DevicePool.from_host(t, sess.device)
    mb = max_blocks_of(wl)
    tables = sess.resolve(sess.upload_batch(b), sess.alloc_tables(b.num_req, mb))
    sess.append_token(pool, tables, R.bits_to_device(ktok[1], sess.device), R.bits_to_device(vtok[1], sess.device))
    torch.cuda.synchronize()
    want = OP.append_token(t.k_pool, t.v_pool, t.k_scale, t.v_scale, oracle_resolve(w_i, max_blocks=mb), ktok[1], vtok[1])
    got = _pool_host(pool)
    for g, w in zip(got, want):
        assert np.array_equal(g, w)
