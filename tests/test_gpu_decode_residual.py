"""gf_attn_decode_residual on the GPU: a decode step that applies each prefix's sparse residual while it reads the
base blocks (paper, Differential-based KV Cache, Eq. 7) against (1) the fp64 oracle attending over the oracle's
reconstructed blocks and (2) the library's own two-step form (gf_kv_apply_residual, then gf_attn_decode over the
instance blocks), whose output it must reproduce bit for bit: both round base + residual to bf16 first."""
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


def _case(shape, seed, last_nodes=2, num_req=5, len_hi=90, **kw):
    wl = W.small_layered(seed, shape, num_nodes=24, num_layers=5, len_lo=3, len_hi=len_hi, num_req=num_req,
                         hops=(1, 5), new_lo=1, new_hi=40)
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


def _decode_fused(wl, t, res, handles, chunk_blocks=0, sm_scale=0.0, misalign=False):
    sess, tables = run_resolve(wl)
    dev = sess.device
    B.gf_set_decode_chunk_blocks(sess.ctx, chunk_blocks)
    pool = R.DevicePool.from_host(t, dev)
    dres = sess.upload_residuals(res)
    if misalign:      # entry arrays that do not start on a 16-byte boundary take the entry-by-entry path
        for key in ("idx", "val"):
            dres[key] = torch.cat([torch.zeros(3, dtype=dres[key].dtype, device=dev), dres[key]])[3:]
            assert dres[key].data_ptr() % 16 != 0
    dh = torch.from_numpy(np.ascontiguousarray(handles)).to(dev)
    last = (t.q_ptr[1:] - 1).astype(np.int64)
    qd = R.bits_to_device(np.ascontiguousarray(t.q[last]), dev)
    o = torch.full(qd.shape, float("nan"), dtype=torch.bfloat16, device=dev)
    lse = torch.full(qd.shape[:2], float("nan"), dtype=torch.float32, device=dev)
    sess.decode_residual(pool, tables, dh, dres, qd, o, lse, sm_scale)
    torch.cuda.synchronize()
    return o, lse, last


def _decode_two_step(wl2, t, k2, v2, res, chunk_blocks=0, sm_scale=0.0):
    t2 = dataclasses.replace(t, k_pool=k2, v_pool=v2)
    sess, tables = run_resolve(wl2)
    dev = sess.device
    B.gf_set_decode_chunk_blocks(sess.ctx, chunk_blocks)
    pool = R.DevicePool.from_host(t2, dev)
    sess.apply_residual(pool, sess.upload_residuals(res))
    last = (t.q_ptr[1:] - 1).astype(np.int64)
    qd = R.bits_to_device(np.ascontiguousarray(t.q[last]), dev)
    o = torch.full(qd.shape, float("nan"), dtype=torch.bfloat16, device=dev)
    lse = torch.full(qd.shape[:2], float("nan"), dtype=torch.float32, device=dev)
    sess.decode(pool, tables, qd, o, lse, sm_scale)
    torch.cuda.synchronize()
    return o, lse


@pytest.mark.parametrize("shape,chunk", [(W.Shape(8, 2, 64), 0), (W.Shape(32, 8, 128), 0), (W.Shape(4, 1, 128), 4),
                                         (W.Shape(8, 8, 64), 2), (W.Shape(16, 2, 128), 6), (W.Shape(4, 2, 64), 2)],
                         ids=lambda x: str(x))
def test_read_time_residual_matches_oracle_and_the_two_step_form(shape, chunk):
    wl, wl2, t, res, k2, v2, inst_tab, handles = _case(shape, 61)
    assert (handles >= 0).sum() > 4 and (handles < 0).sum() > 4
    o, lse, last = _decode_fused(wl, t, res, handles, chunk)
    want_k, want_v, _ = OR.reconstruct(k2, v2, res.src_blocks, res.dst_blocks, res.res_ptr, res.res_idx, res.res_val)
    O, LSE = OA.decode(np.ascontiguousarray(t.q[last]), want_k, want_v, inst_tab)
    assert_close(bf16_out_to_f64(o), O, W.KV_BF16, "read-time residual decode")
    np.testing.assert_allclose(lse.double().cpu().numpy(), LSE, atol=1e-2, rtol=1e-2)
    o2, lse2 = _decode_two_step(wl2, t, k2, v2, res, chunk)
    assert torch.equal(o.view(torch.int16), o2.view(torch.int16))
    assert torch.equal(lse.view(torch.int32), lse2.view(torch.int32))
    o3, lse3, _ = _decode_fused(wl, t, res, handles, chunk, misalign=True)
    assert torch.equal(o3.view(torch.int16), o2.view(torch.int16))
    assert torch.equal(lse3.view(torch.int32), lse2.view(torch.int32))


def test_residual_changes_the_result_and_no_handles_is_plain_decode():
    shape = W.Shape(32, 8, 128)
    wl, wl2, t, res, k2, v2, inst_tab, handles = _case(shape, 62, std=1.0)
    o, lse, last = _decode_fused(wl, t, res, handles)
    none = np.full_like(handles, -1)
    o0, lse0, _ = _decode_fused(wl, t, res, none)
    assert not torch.equal(o.view(torch.int16), o0.view(torch.int16))
    # handles outside the CSR read the base block as it is
    wild = np.where(handles >= 0, res.num_items + 5, -7).astype(np.int32)
    o1, lse1, _ = _decode_fused(wl, t, res, wild)
    # an empty CSR: nothing to apply whatever the handles say
    empty = W.Residuals(np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros(1, np.int32), np.zeros(0, np.uint16),
                        np.zeros(0, np.uint16))
    o3, lse3, _ = _decode_fused(wl, t, empty, handles)
    sess, tables = run_resolve(wl)
    pool = R.DevicePool.from_host(t, sess.device)
    qd = R.bits_to_device(np.ascontiguousarray(t.q[last]), sess.device)
    op = torch.full(qd.shape, float("nan"), dtype=torch.bfloat16, device=sess.device)
    lsep = torch.full(qd.shape[:2], float("nan"), dtype=torch.float32, device=sess.device)
    sess.decode(pool, tables, qd, op, lsep)
    torch.cuda.synchronize()
    for a, b in ((o0, lse0), (o1, lse1), (o3, lse3)):
        assert torch.equal(a.view(torch.int16), op.view(torch.int16))
        assert torch.equal(b.view(torch.int32), lsep.view(torch.int32))


def test_out_of_image_entries_are_ignored_and_dense_rows_work():
    shape = W.Shape(8, 2, 64)
    wl, wl2, t, res, k2, v2, inst_tab, handles = _case(shape, 63, density_k=1.0, density_v=1.0)
    # append one entry beyond the image to every row: the two-step form flags it and ignores it, so does this one
    ptr = res.res_ptr.astype(np.int64)
    rows = ptr.size - 1
    idx, val = [], []
    for r in range(rows):
        idx += [res.res_idx[ptr[r]:ptr[r + 1]], np.array([16 * shape.head_dim + r % 7], np.uint16)]
        val += [res.res_val[ptr[r]:ptr[r + 1]], np.array([0x4000], np.uint16)]
    res_bad = W.Residuals(res.src_blocks, res.dst_blocks, (ptr + np.arange(rows + 1)).astype(np.int32),
                          np.concatenate(idx), np.concatenate(val))
    o, lse, last = _decode_fused(wl, t, res_bad, handles)
    o_ok, lse_ok, _ = _decode_fused(wl, t, res, handles)
    assert torch.equal(o.view(torch.int16), o_ok.view(torch.int16))
    want_k, want_v, _ = OR.reconstruct(k2, v2, res.src_blocks, res.dst_blocks, res.res_ptr, res.res_idx, res.res_val)
    O, _ = OA.decode(np.ascontiguousarray(t.q[last]), want_k, want_v, inst_tab)
    assert_close(bf16_out_to_f64(o), O, W.KV_BF16, "dense residual rows")


def test_e4m3_pool_is_refused():
    shape = W.Shape(8, 2, 64, W.KV_FP8_E4M3)
    wl = W.small_layered(64, shape, num_nodes=12, num_layers=3, len_lo=3, len_hi=40, num_req=3, hops=(1, 3),
                         new_lo=1, new_hi=8)
    t = W.make_tensors(wl)
    sess, tables = run_resolve(wl)
    pool = R.DevicePool.from_host(t, sess.device)
    qd = torch.zeros((3, 8, 64), dtype=torch.bfloat16, device=sess.device)
    o = torch.zeros_like(qd)
    dh = torch.full((3, int(tables["max_blocks"])), -1, dtype=torch.int32, device=sess.device)
    empty = W.Residuals(np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros(1, np.int32), np.zeros(0, np.uint16),
                        np.zeros(0, np.uint16))
    with pytest.raises(B.GraphFlowError) as ei:
        sess.decode_residual(pool, tables, dh, sess.upload_residuals(empty), qd, o)
    assert ei.value.code == B.GF_ERR_UNSUPPORTED
