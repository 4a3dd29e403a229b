"""gf_attn_prefill_residual on the GPU: a prefill that applies each prefix's sparse residual while it reads the base
blocks (paper, Differential-based KV Cache, Eq. 7; the on-the-fly fallback of Effective Path Pruning attends to
ancestors whose KV under the current prefix is base + residual) against (1) the fp64 oracle attending over the
oracle's reconstructed blocks and (2) the library's own two-step form (gf_kv_apply_residual, then gf_attn_prefill
over the instance blocks), whose output it must reproduce bit for bit: both round base + residual to bf16 first."""
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


def _case(shape, seed, last_nodes=2, num_req=5, len_lo=3, len_hi=90, hops=(1, 5), new_hi=70, num_nodes=24, **kw):
    wl = W.small_layered(seed, shape, num_nodes=num_nodes, num_layers=max(hops[1], 5), len_lo=len_lo, len_hi=len_hi,
                         num_req=num_req, hops=hops, new_lo=1, new_hi=new_hi)
    t = W.make_tensors(wl)
    wl2, res = W.add_residual_instances(wl, last_nodes=last_nodes, **kw)
    extra = wl2.num_pool_blocks - wl.num_pool_blocks
    # instance blocks: NaN in the pool the read-time form sees (it must never read them)
    k2 = np.concatenate([t.k_pool, np.full((extra,) + t.k_pool.shape[1:], 0x7FC0, np.uint16)])
    v2 = np.concatenate([t.v_pool, np.full((extra,) + t.v_pool.shape[1:], 0x7FC0, np.uint16)])
    base_tab, inst_tab = oracle_resolve(wl), oracle_resolve(wl2)
    bt, it = np.asarray(base_tab["block_table"], np.int32), np.asarray(inst_tab["block_table"], np.int32)
    assert bt.shape == it.shape and bt.ndim == 2
    handles = W.residual_handles(bt, it, res)
    return wl, wl2, t, res, k2, v2, inst_tab, handles


def _io(sess, t, wl):
    dev = sess.device
    q = R.bits_to_device(t.q, dev)
    q_ptr = torch.from_numpy(t.q_ptr).to(dev)
    o = torch.full(q.shape, float("nan"), dtype=torch.bfloat16, device=dev)
    lse = torch.full(q.shape[:2], float("nan"), dtype=torch.float32, device=dev)
    return q, q_ptr, int(t.q.shape[0]), int(wl.batch.new_lens.max()), o, lse


def _prefill_fused(wl, t, res, handles, sm_scale=0.0, misalign=False):
    sess, tables = run_resolve(wl)
    dev = sess.device
    pool = R.DevicePool.from_host(t, dev)
    dres = sess.upload_residuals(res)
    if misalign:      # entry arrays that do not start on a 16-byte boundary take the entry-by-entry path
        for key in ("idx", "val"):
            dres[key] = torch.cat([torch.zeros(3, dtype=dres[key].dtype, device=dev), dres[key]])[3:]
            assert dres[key].data_ptr() % 16 != 0
    dh = torch.from_numpy(np.ascontiguousarray(handles)).to(dev)
    q, q_ptr, total_q, max_q, o, lse = _io(sess, t, wl)
    sess.prefill_residual(pool, tables, dh, dres, q, q_ptr, total_q, max_q, o, lse, sm_scale)
    torch.cuda.synchronize()
    return o, lse


def _prefill_two_step(wl2, t, k2, v2, res, sm_scale=0.0):
    t2 = dataclasses.replace(t, k_pool=k2, v_pool=v2)
    sess, tables = run_resolve(wl2)
    pool = R.DevicePool.from_host(t2, sess.device)
    sess.apply_residual(pool, sess.upload_residuals(res))
    q, q_ptr, total_q, max_q, o, lse = _io(sess, t, wl2)
    sess.prefill(pool, tables, q, q_ptr, total_q, max_q, o, lse, sm_scale)
    torch.cuda.synchronize()
    return o, lse


def _oracle(t, k2, v2, res, inst_tab):
    want_k, want_v, _ = OR.reconstruct(k2, v2, res.src_blocks, res.dst_blocks, res.res_ptr, res.res_idx, res.res_val)
    return OA.prefill(t.q, t.q_ptr, want_k, want_v, inst_tab)


def _same_bits(a, b):
    return torch.equal(a.view(torch.int16), b.view(torch.int16))


@pytest.mark.parametrize("shape", [W.Shape(8, 2, 64), W.Shape(32, 8, 128), W.Shape(4, 1, 128), W.Shape(8, 8, 64),
                                   W.Shape(16, 2, 128), W.Shape(4, 2, 64)], ids=lambda x: str(x))
def test_read_time_residual_matches_oracle_and_the_two_step_form(shape):
    wl, wl2, t, res, k2, v2, inst_tab, handles = _case(shape, 71)
    assert (handles >= 0).sum() > 4 and (handles < 0).sum() > 4
    o, lse = _prefill_fused(wl, t, res, handles)
    O, LSE = _oracle(t, k2, v2, res, inst_tab)
    assert_close(bf16_out_to_f64(o), O, W.KV_BF16, "read-time residual prefill")
    np.testing.assert_allclose(lse.double().cpu().numpy(), LSE, atol=1e-2, rtol=1e-2)
    o2, lse2 = _prefill_two_step(wl2, t, k2, v2, res)
    assert _same_bits(o, o2)
    assert torch.equal(lse.view(torch.int32), lse2.view(torch.int32))
    o3, lse3 = _prefill_fused(wl, t, res, handles, misalign=True)
    assert _same_bits(o3, o2)
    assert torch.equal(lse3.view(torch.int32), lse2.view(torch.int32))


def test_every_node_under_a_prefix_carries_a_residual_over_several_table_windows():
    """The paper's own regime: every node of the path beyond the first has a residual; contexts of more than 130
    table entries, so the kernel's cached table window slides twice with handles in it."""
    shape = W.Shape(4, 1, 128)
    wl, wl2, t, res, k2, v2, inst_tab, handles = _case(shape, 72, last_nodes=7, num_req=3, len_lo=200, len_hi=420,
                                                       hops=(7, 8), new_hi=150, num_nodes=40)
    nb = np.asarray(inst_tab["num_blocks"])
    assert nb.max() > 135 and (handles >= 0).sum() > 250
    o, lse = _prefill_fused(wl, t, res, handles)
    O, LSE = _oracle(t, k2, v2, res, inst_tab)
    assert_close(bf16_out_to_f64(o), O, W.KV_BF16, "residual on every node")
    o2, lse2 = _prefill_two_step(wl2, t, k2, v2, res)
    assert _same_bits(o, o2)
    assert torch.equal(lse.view(torch.int32), lse2.view(torch.int32))


def test_residual_changes_the_result_and_no_handles_is_plain_prefill():
    shape = W.Shape(32, 8, 128)
    wl, wl2, t, res, k2, v2, inst_tab, handles = _case(shape, 73, std=1.0)
    o, lse = _prefill_fused(wl, t, res, handles)
    o0, lse0 = _prefill_fused(wl, t, res, np.full_like(handles, -1))
    assert not _same_bits(o, o0)
    # handles outside the CSR read the base block as it is
    wild = np.where(handles >= 0, res.num_items + 5, -7).astype(np.int32)
    o1, lse1 = _prefill_fused(wl, t, res, wild)
    # an empty CSR: nothing to apply whatever the handles say
    empty = W.Residuals(np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros(1, np.int32), np.zeros(0, np.uint16),
                        np.zeros(0, np.uint16))
    o3, lse3 = _prefill_fused(wl, t, empty, handles)
    sess, tables = run_resolve(wl)
    pool = R.DevicePool.from_host(t, sess.device)
    q, q_ptr, total_q, max_q, op, lsep = _io(sess, t, wl)
    sess.prefill(pool, tables, q, q_ptr, total_q, max_q, op, lsep)
    torch.cuda.synchronize()
    for a, b in ((o0, lse0), (o1, lse1), (o3, lse3)):
        assert _same_bits(a, op)
        assert torch.equal(b.view(torch.int32), lsep.view(torch.int32))


def test_out_of_image_entries_are_ignored_and_dense_rows_work():
    shape = W.Shape(8, 2, 64)
    wl, wl2, t, res, k2, v2, inst_tab, handles = _case(shape, 74, density_k=1.0, density_v=1.0)
    # one entry beyond the image appended to every row: the two-step form flags and ignores it, so does this one
    ptr = res.res_ptr.astype(np.int64)
    rows = ptr.size - 1
    idx, val = [], []
    for r in range(rows):
        idx += [res.res_idx[ptr[r]:ptr[r + 1]], np.array([16 * shape.head_dim + r % 7], np.uint16)]
        val += [res.res_val[ptr[r]:ptr[r + 1]], np.array([0x4000], np.uint16)]
    res_bad = W.Residuals(res.src_blocks, res.dst_blocks, (ptr + np.arange(rows + 1)).astype(np.int32),
                          np.concatenate(idx), np.concatenate(val))
    o, lse = _prefill_fused(wl, t, res_bad, handles)
    o_ok, lse_ok = _prefill_fused(wl, t, res, handles)
    assert _same_bits(o, o_ok)
    O, _ = _oracle(t, k2, v2, res, inst_tab)
    assert_close(bf16_out_to_f64(o), O, W.KV_BF16, "dense residual rows")
    # dense rows at head_dim 128: 2048 entries per row, four rounds of the row loader
    shape = W.Shape(4, 1, 128)
    wl, wl2, t, res, k2, v2, inst_tab, handles = _case(shape, 75, density_k=1.0, density_v=1.0, num_req=3)
    o, lse = _prefill_fused(wl, t, res, handles)
    o2, lse2 = _prefill_two_step(wl2, t, k2, v2, res)
    assert _same_bits(o, o2)


def test_e4m3_pool_is_refused():
    shape = W.Shape(8, 2, 64, W.KV_FP8_E4M3)
    wl = W.small_layered(76, shape, num_nodes=12, num_layers=3, len_lo=3, len_hi=40, num_req=3, hops=(1, 3),
                         new_lo=1, new_hi=8)
    t = W.make_tensors(wl)
    sess, tables = run_resolve(wl)
    pool = R.DevicePool.from_host(t, sess.device)
    q, q_ptr, total_q, max_q, o, lse = _io(sess, t, wl)
    dh = torch.full((3, int(tables["max_blocks"])), -1, dtype=torch.int32, device=sess.device)
    empty = W.Residuals(np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros(1, np.int32), np.zeros(0, np.uint16),
                        np.zeros(0, np.uint16))
    with pytest.raises(B.GraphFlowError) as ei:
        sess.prefill_residual(pool, tables, dh, sess.upload_residuals(empty), q, q_ptr, total_q, max_q, o, lse)
    assert ei.value.code == B.GF_ERR_UNSUPPORTED
