"""gf_attn_decode_shared_residual on the GPU: the node-centric decode step with each prefix's sparse residual applied
while the base blocks are read (paper, Differential-based KV Cache, Eq. 7).  Requests that reach a node through the
same prefix carry the same residual and share one read of it; the others are listed apart.  Checked against (1) the
fp64 oracle attending over the oracle's reconstructed blocks, (2) gf_attn_decode_residual, the per-request
read-time form (same tolerance as the node-centric step has against the per-request one), and (3) its own two-step
form -- gf_kv_apply_residual, then gf_attn_decode_shared over the instance nodes -- which groups the requests the
same way and must therefore agree bit for bit."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import attention as OA
from oracle import residual as OR
from paper_2605_22566_amd import binding as B
from paper_2605_22566_amd import runner as R
from paper_2605_22566_amd import workload as W
from tests.gpu_common import assert_close, bf16_out_to_f64, run_resolve
from tests.helpers import oracle_resolve

pytestmark = pytest.mark.gpu


def _case(shape, seed, last_nodes=3, num_req=12, by_prefix=True, num_nodes=10, len_hi=90, hops=(2, 4), **kw):
    wl = W.small_layered(seed, shape, num_nodes=num_nodes, num_layers=4, len_lo=3, len_hi=len_hi, num_req=num_req,
                         hops=hops, new_lo=1, new_hi=40)
    t = W.make_tensors(wl)
    wl2, res = W.add_residual_instances(wl, last_nodes=last_nodes, by_prefix=by_prefix, **kw)
    extra = wl2.num_pool_blocks - wl.num_pool_blocks
    k2 = np.concatenate([t.k_pool, np.full((extra,) + t.k_pool.shape[1:], 0x7FC0, np.uint16)])
    v2 = np.concatenate([t.v_pool, np.full((extra,) + t.v_pool.shape[1:], 0x7FC0, np.uint16)])
    base_tab, inst_tab = oracle_resolve(wl), oracle_resolve(wl2)
    bt, it = np.asarray(base_tab["block_table"], np.int32), np.asarray(inst_tab["block_table"], np.int32)
    handles = W.residual_handles(bt, it, res)
    return wl, wl2, t, res, k2, v2, inst_tab, handles


def _queries(sess, t):
    last = (t.q_ptr[1:] - 1).astype(np.int64)
    qd = R.bits_to_device(np.ascontiguousarray(t.q[last]), sess.device)
    o = torch.full(qd.shape, float("nan"), dtype=torch.bfloat16, device=sess.device)
    lse = torch.full(qd.shape[:2], float("nan"), dtype=torch.float32, device=sess.device)
    return last, qd, o, lse


def _shared_fused(wl, t, res, handles, chunk=0):
    sess, tables = run_resolve(wl)
    B.gf_set_decode_chunk_blocks(sess.ctx, chunk)
    pool = R.DevicePool.from_host(t, sess.device)
    dres = sess.upload_residuals(res)
    dh = torch.from_numpy(np.ascontiguousarray(handles)).to(sess.device)
    last, qd, o, lse = _queries(sess, t)
    sess.decode_shared_residual(pool, sess.upload_batch(wl.batch), tables, dh, dres, qd, o, lse)
    torch.cuda.synchronize()
    return o, lse, last


def _per_request_fused(wl, t, res, handles, chunk=0):
    sess, tables = run_resolve(wl)
    B.gf_set_decode_chunk_blocks(sess.ctx, chunk)
    pool = R.DevicePool.from_host(t, sess.device)
    dh = torch.from_numpy(np.ascontiguousarray(handles)).to(sess.device)
    last, qd, o, lse = _queries(sess, t)
    sess.decode_residual(pool, tables, dh, sess.upload_residuals(res), qd, o, lse)
    torch.cuda.synchronize()
    return o, lse


def _shared_two_step(wl2, t, k2, v2, res, chunk=0):
    t2 = dataclasses.replace(t, k_pool=k2, v_pool=v2)
    sess, tables = run_resolve(wl2)
    B.gf_set_decode_chunk_blocks(sess.ctx, chunk)
    pool = R.DevicePool.from_host(t2, sess.device)
    sess.apply_residual(pool, sess.upload_residuals(res))
    last, qd, o, lse = _queries(sess, t)
    sess.decode_shared(pool, sess.upload_batch(wl2.batch), tables, qd, o, lse)
    torch.cuda.synchronize()
    return o, lse


@pytest.mark.parametrize("shape,chunk", [(W.Shape(8, 2, 64), 0), (W.Shape(32, 8, 128), 0), (W.Shape(4, 1, 128), 4),
                                         (W.Shape(8, 8, 64), 2), (W.Shape(16, 2, 128), 6), (W.Shape(8, 1, 64), 0)],
                         ids=lambda x: str(x))
def test_pairs_shared_by_prefix_match_oracle_per_request_and_two_step_forms(shape, chunk):
    wl, wl2, t, res, k2, v2, inst_tab, handles = _case(shape, 81)
    # the case is only worth its name if some (prefix, node) pair serves several requests and some node is
    # read both with and without a residual
    firsts = [tuple(r[r >= 0][:1]) for r in handles]
    assert len(set(map(tuple, handles.tolist()))) < handles.shape[0] or len(firsts) > len(set(firsts))
    assert (handles >= 0).sum() > 8 and (handles < 0).sum() > 8
    o, lse, last = _shared_fused(wl, t, res, handles, chunk)
    want_k, want_v, _ = OR.reconstruct(k2, v2, res.src_blocks, res.dst_blocks, res.res_ptr, res.res_idx, res.res_val)
    O, LSE = OA.decode(np.ascontiguousarray(t.q[last]), want_k, want_v, inst_tab)
    assert_close(bf16_out_to_f64(o), O, W.KV_BF16, "node-centric read-time residual decode")
    np.testing.assert_allclose(lse.double().cpu().numpy(), LSE, atol=1e-2, rtol=1e-2)
    o1, lse1 = _per_request_fused(wl, t, res, handles, chunk)
    assert_close(bf16_out_to_f64(o), bf16_out_to_f64(o1), W.KV_BF16, "against the per-request read-time form")
    o2, lse2 = _shared_two_step(wl2, t, k2, v2, res, chunk)
    assert torch.equal(o.view(torch.int16), o2.view(torch.int16))
    assert torch.equal(lse.view(torch.int32), lse2.view(torch.int32))


def test_private_residuals_on_every_request_and_long_nodes():
    """Every request its own residuals (nothing shared under a residual), nodes of several chunks."""
    shape = W.Shape(8, 2, 128)
    wl, wl2, t, res, k2, v2, inst_tab, handles = _case(shape, 82, by_prefix=False, num_req=6, len_hi=400, last_nodes=2)
    o, lse, last = _shared_fused(wl, t, res, handles, chunk=4)
    want_k, want_v, _ = OR.reconstruct(k2, v2, res.src_blocks, res.dst_blocks, res.res_ptr, res.res_idx, res.res_val)
    O, LSE = OA.decode(np.ascontiguousarray(t.q[last]), want_k, want_v, inst_tab)
    assert_close(bf16_out_to_f64(o), O, W.KV_BF16, "private residuals")
    o2, lse2 = _shared_two_step(wl2, t, k2, v2, res, chunk=4)
    assert torch.equal(o.view(torch.int16), o2.view(torch.int16))


def test_no_handles_is_the_plain_node_centric_step_and_wild_handles_read_the_base():
    shape = W.Shape(32, 8, 128)
    wl, wl2, t, res, k2, v2, inst_tab, handles = _case(shape, 83, std=1.0)
    o, lse, last = _shared_fused(wl, t, res, handles)
    o0, lse0, _ = _shared_fused(wl, t, res, np.full_like(handles, -1))
    assert not torch.equal(o.view(torch.int16), o0.view(torch.int16))
    wild = np.where(handles >= 0, res.num_items + 5, -7).astype(np.int32)
    o1, lse1, _ = _shared_fused(wl, t, res, wild)
    empty = W.Residuals(np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros(1, np.int32), np.zeros(0, np.uint16),
                        np.zeros(0, np.uint16))
    o3, lse3, _ = _shared_fused(wl, t, empty, handles)
    sess, tables = run_resolve(wl)
    pool = R.DevicePool.from_host(t, sess.device)
    _, qd, op, lsep = _queries(sess, t)
    sess.decode_shared(pool, sess.upload_batch(wl.batch), tables, qd, op, lsep)
    torch.cuda.synchronize()
    for a, b in ((o0, lse0), (o1, lse1), (o3, lse3)):
        assert torch.equal(a.view(torch.int16), op.view(torch.int16))
        assert torch.equal(b.view(torch.int32), lsep.view(torch.int32))
    # the plain call after a residual call builds its own lists again
    dh = torch.from_numpy(np.ascontiguousarray(handles)).to(sess.device)
    _, _, o4, lse4 = _queries(sess, t)
    sess.decode_shared_residual(pool, sess.upload_batch(wl.batch), tables, dh, sess.upload_residuals(res), qd, o4, lse4)
    with pytest.raises(B.GraphFlowError):
        sess.decode_shared_planned(pool, sess.upload_batch(wl.batch), tables, qd, op, lsep)
    sess.decode_shared(pool, sess.upload_batch(wl.batch), tables, qd, op, lsep)
    torch.cuda.synchronize()
    assert torch.equal(o4.view(torch.int16), o.view(torch.int16))
    assert torch.equal(op.view(torch.int16), o0.view(torch.int16))


def test_e4m3_pool_is_refused():
    shape = W.Shape(8, 2, 64, W.KV_FP8_E4M3)
    wl = W.small_layered(84, shape, num_nodes=12, num_layers=3, len_lo=3, len_hi=40, num_req=3, hops=(1, 3),
                         new_lo=1, new_hi=8)
    t = W.make_tensors(wl)
    sess, tables = run_resolve(wl)
    pool = R.DevicePool.from_host(t, sess.device)
    _, qd, o, lse = _queries(sess, t)
    dh = torch.full((3, int(tables["max_blocks"])), -1, dtype=torch.int32, device=sess.device)
    empty = W.Residuals(np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros(1, np.int32), np.zeros(0, np.uint16),
                        np.zeros(0, np.uint16))
    with pytest.raises(B.GraphFlowError) as ei:
        sess.decode_shared_residual(pool, sess.upload_batch(wl.batch), tables, dh, sess.upload_residuals(empty), qd, o,
                                    lse)
    assert ei.value.code == B.GF_ERR_UNSUPPORTED


def test_arbitrary_handles_stay_in_bounds_and_give_finite_rows():
    """Handles that follow no rule at all (any value from below -1 to beyond the CSR, per table entry; nodes that
    claim each other's items): every read stays inside the CSR and the pool, every output row is finite and inside
    the hull of what base + residual values can reach -- for the node-centric call and for the two per-request
    ones."""
    shape = W.Shape(8, 2, 128)
    wl, wl2, t, res, k2, v2, inst_tab, handles = _case(shape, 85, num_req=16)
    rng = np.random.default_rng(85)
    wild = rng.integers(-3, res.num_items + 3, handles.shape).astype(np.int32)
    sess, tables = run_resolve(wl)
    pool = R.DevicePool.from_host(t, sess.device)
    dres = sess.upload_residuals(res)
    dh = torch.from_numpy(wild).to(sess.device)
    last, qd, o, lse = _queries(sess, t)
    sess.decode_shared_residual(pool, sess.upload_batch(wl.batch), tables, dh, dres, qd, o, lse)
    o2 = torch.full_like(o, float("nan"))
    sess.decode_residual(pool, tables, dh, dres, qd, o2)
    q = R.bits_to_device(t.q, sess.device)
    op = torch.full(q.shape, float("nan"), dtype=torch.bfloat16, device=sess.device)
    sess.prefill_residual(pool, tables, dh, dres, q, torch.from_numpy(t.q_ptr).to(sess.device), int(q.shape[0]),
                          int(wl.batch.new_lens.max()), op)
    torch.cuda.synchronize()
    from oracle import residual as OR
    vmax = float(np.abs(OR.bf16_bits_to_f32(t.v_pool)).max())
    dmax = float(np.abs(OR.bf16_bits_to_f32(res.res_val)).max()) if res.res_val.size else 0.0
    for out in (o, o2, op):
        x = out.float()
        assert bool(torch.isfinite(x).all())
        assert float(x.abs().max()) <= (vmax + dmax) * 1.01 + 1e-2
