"""gf_kv_append through the C ABI vs oracle/append.py (bit-exact pools and scales), and the closed
loop resolve -> append -> prefill / decode vs the attention oracle."""
import numpy as np
import pytest
import torch

from oracle import append as OP
from oracle import attention as OA
from paper_2605_22566_amd import runner as R
from paper_2605_22566_amd import workload as W
from tests.gpu_common import assert_close, bf16_out_to_f64, run_resolve
from tests.helpers import oracle_resolve

pytestmark = pytest.mark.gpu

SHAPES = [W.Shape(8, 2, 64), W.Shape(32, 8, 128), W.Shape(4, 1, 128), W.Shape(32, 8, 128, W.KV_FP8_E4M3),
          W.Shape(8, 2, 64, W.KV_FP8_E4M3)]


def _sid(s):
    return f"kv{s.num_kv_heads}d{s.head_dim}" + ("fp8" if s.kv_dtype == W.KV_FP8_E4M3 else "")


def _case(shape, seed, new_hi=70, spread=True):
    wl = W.small_layered(seed, shape, num_nodes=20, num_layers=5, len_lo=3, len_hi=90, num_req=6, hops=(1, 5),
                         new_lo=1, new_hi=new_hi)
    t = W.make_tensors(wl)
    rng = np.random.default_rng(seed + 1)
    total_q = int(t.q_ptr[-1])
    # blocks of very different amax for the bit-exact checks; N(0,1) like the workloads for attention parity
    mag = np.float32(10.0) ** rng.integers(-2, 2, (total_q, 1, 1)) if spread else np.float32(1.0)
    kn = W.f32_to_bf16_bits((rng.standard_normal((total_q, shape.num_kv_heads, shape.head_dim)) * mag).astype(np.float32))
    vn = W.f32_to_bf16_bits((rng.standard_normal((total_q, shape.num_kv_heads, shape.head_dim)) * mag).astype(np.float32))
    return wl, t, kn, vn


def _pool_host(pool):
    if pool.k.dtype == torch.bfloat16:
        return R.bf16_to_bits(pool.k), R.bf16_to_bits(pool.v), None, None
    return pool.k.cpu().numpy(), pool.v.cpu().numpy(), pool.k_scale.cpu().numpy(), pool.v_scale.cpu().numpy()


def _append_gpu(wl, t, kn, vn, max_q=None, q_ptr=None):
    sess, tables = run_resolve(wl)
    pool = R.DevicePool.from_host(t, sess.device)
    dk, dv = R.bits_to_device(kn, sess.device), R.bits_to_device(vn, sess.device)
    qp = torch.from_numpy(t.q_ptr if q_ptr is None else q_ptr).to(sess.device)
    mq = int(wl.batch.new_lens.max()) if max_q is None else max_q
    sess.append(pool, tables, dk, dv, qp, int(kn.shape[0]), mq)
    torch.cuda.synchronize()
    return sess, tables, pool


@pytest.mark.parametrize("shape", SHAPES, ids=_sid)
def test_append_is_bit_exact(shape):
    wl, t, kn, vn = _case(shape, 500 + shape.head_dim + shape.num_kv_heads + shape.kv_dtype)
    want = OP.append(t.k_pool, t.v_pool, t.k_scale, t.v_scale, oracle_resolve(wl), kn, vn, t.q_ptr)
    _, _, pool = _append_gpu(wl, t, kn, vn)
    got = _pool_host(pool)
    assert np.array_equal(got[0], want[0]), "K pool"
    assert np.array_equal(got[1], want[1]), "V pool"
    if shape.kv_dtype == W.KV_FP8_E4M3:
        assert np.array_equal(got[2], want[2]) and np.array_equal(got[3], want[3]), "scales"


@pytest.mark.parametrize("shape", [W.Shape(32, 8, 128), W.Shape(32, 8, 128, W.KV_FP8_E4M3)], ids=_sid)
def test_loop_resolve_append_prefill_decode(shape):
    wl, t, kn, vn = _case(shape, 61 + shape.kv_dtype, spread=False)
    want = OP.append(t.k_pool, t.v_pool, t.k_scale, t.v_scale, oracle_resolve(wl), kn, vn, t.q_ptr)
    sess, tables, pool = _append_gpu(wl, t, kn, vn)
    dev = sess.device
    q = R.bits_to_device(t.q, dev)
    o = torch.full(q.shape, float("nan"), dtype=torch.bfloat16, device=dev)
    sess.prefill(pool, tables, q, torch.from_numpy(t.q_ptr).to(dev), int(t.q.shape[0]), int(wl.batch.new_lens.max()), o)
    last = (t.q_ptr[1:] - 1).astype(np.int64)
    qd = R.bits_to_device(np.ascontiguousarray(t.q[last]), dev)
    od = torch.full(qd.shape, float("nan"), dtype=torch.bfloat16, device=dev)
    sess.decode(pool, tables, qd, od)
    torch.cuda.synchronize()
    ot = oracle_resolve(wl)
    O, _ = OA.prefill(t.q, t.q_ptr, want[0], want[1], ot, want[2], want[3])
    Od, _ = OA.decode(np.ascontiguousarray(t.q[last]), want[0], want[1], ot, want[2], want[3])
    assert_close(bf16_out_to_f64(o), O, shape.kv_dtype, "prefill after append")
    assert_close(bf16_out_to_f64(od), Od, shape.kv_dtype, "decode after append")


def test_skipped_requests_row_mismatch_and_grid_bound():
    shape = W.Shape(8, 2, 64)
    wl, t, kn, vn = _case(shape, 71)
    b = wl.batch
    p0, p1 = int(b.path_ptr[1]), int(b.path_ptr[2])
    if p1 - p0 >= 2:
        b.path_nodes[p0:p1] = b.path_nodes[p0:p1][::-1].copy()           # request 1 fails to resolve
    ot = oracle_resolve(wl)
    # request 3 claims one row fewer than its table says: skipped on both sides
    qp = t.q_ptr.copy()
    want = OP.append(t.k_pool, t.v_pool, None, None, ot, kn, vn, qp)
    _, tables, pool = _append_gpu(wl, t, kn, vn)
    assert tables["status"].cpu().numpy().tolist() == ot["status"]
    got = _pool_host(pool)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
    # a grid bound below the longest request: only whole-or-partial leading tail blocks up to the bound change,
    # and every block that is written matches the oracle's
    small = 16
    _, _, pool2 = _append_gpu(wl, t, kn, vn, max_q=small)
    g2 = _pool_host(pool2)
    changed = np.nonzero((g2[0] != t.k_pool).reshape(t.k_pool.shape[0], -1).any(axis=1))[0]
    assert len(changed) > 0
    assert np.array_equal(g2[0][changed], want[0][changed]) and np.array_equal(g2[1][changed], want[1][changed])
    first_tail = {int(b.tail_blocks[b.tail_ptr[r]]) for r in range(b.num_req) if ot["status"][r] == 0}
    assert set(changed.tolist()) <= first_tail
