"""Helpers for the GPU parity tests: run the HIP path through the C ABI on a
workload and hand back host arrays; compare with the oracle."""
import numpy as np
import torch

from oracle import attention as OA
from paper_2605_22566_amd import runner as R
from paper_2605_22566_amd import workload as W
from tests.helpers import max_blocks_of, oracle_resolve

TOL = {W.KV_BF16: (1e-2, 1e-2), W.KV_FP8_E4M3: (5e-2, 5e-2)}   # (atol, rtol), the benchmark spec's tolerances


def bf16_out_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def run_resolve(wl, batch=None, max_blocks=None, with_edges=True, num_pool_blocks=None):
    sess = R.Session(wl)
    b = wl.batch if batch is None else batch
    db = sess.upload_batch(b)
    mb = max_blocks_of(wl) if max_blocks is None else max_blocks
    tables = sess.alloc_tables(b.num_req, mb)
    for k in ("block_table", "block_ntok", "num_blocks", "ctx_lens", "seq_lens", "status"):
        tables[k].fill_(-77)                     # every output must be overwritten
    sess.resolve(db, tables, with_edges=with_edges, num_pool_blocks=num_pool_blocks)
    torch.cuda.synchronize()
    return sess, tables


def assert_tables_equal(dev_tables, want: dict):
    got = R.tables_to_host(dev_tables)
    for k in ("status", "num_blocks", "ctx_lens", "seq_lens", "block_table", "block_ntok"):
        assert got[k] == want[k], k


def assert_close(got, want, kv_dtype, what=""):
    atol, rtol = TOL[kv_dtype]
    err = np.abs(got - want)
    bound = atol + rtol * np.abs(want)
    bad = err > bound
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside tolerance; max err {err.max():.4g}"
    return float(err.max())


def run_prefill(wl, t, sm_scale=0.0, want_lse=True, tables=None, sess=None):
    if sess is None:
        sess, tables = run_resolve(wl)
    dev = sess.device
    pool = R.DevicePool.from_host(t, dev)
    q = R.bits_to_device(t.q, dev)
    q_ptr = torch.from_numpy(t.q_ptr).to(dev)
    total_q = int(t.q.shape[0])
    max_q = int(wl.batch.new_lens.max()) if wl.batch.num_req else 0
    o = torch.full(q.shape, float("nan"), dtype=torch.bfloat16, device=dev)
    lse = torch.full(q.shape[:2], float("nan"), dtype=torch.float32, device=dev) if want_lse else None
    sess.prefill(pool, tables, q, q_ptr, total_q, max_q, o, lse, sm_scale)
    torch.cuda.synchronize()
    return bf16_out_to_f64(o), (None if lse is None else lse.double().cpu().numpy()), tables, sess


def run_decode(wl, t, sm_scale=0.0, chunk_blocks=0, tables=None, sess=None, shared=False, with_edges=True):
    """Decode with each request's LAST new token as the query (shared: the node-centric entry point)."""
    if sess is None:
        sess, tables = run_resolve(wl, with_edges=with_edges)
    dev = sess.device
    from paper_2605_22566_amd import binding as B
    B.gf_set_decode_chunk_blocks(sess.ctx, chunk_blocks)
    pool = R.DevicePool.from_host(t, dev)
    last = (t.q_ptr[1:] - 1).astype(np.int64)
    qd = R.bits_to_device(np.ascontiguousarray(t.q[last]), dev)
    o = torch.full(qd.shape, float("nan"), dtype=torch.bfloat16, device=dev)
    lse = torch.full(qd.shape[:2], float("nan"), dtype=torch.float32, device=dev)
    if shared:
        sess.decode_shared(pool, sess.upload_batch(wl.batch), tables, qd, o, lse, sm_scale)
    else:
        sess.decode(pool, tables, qd, o, lse, sm_scale)
    torch.cuda.synchronize()
    return bf16_out_to_f64(o), lse.double().cpu().numpy(), tables, sess, last


def oracle_prefill(wl, t, sm_scale=None):
    tables = oracle_resolve(wl)
    return OA.prefill(t.q, t.q_ptr, t.k_pool, t.v_pool, tables, t.k_scale, t.v_scale, sm_scale)


def oracle_decode(wl, t, last, sm_scale=None):
    tables = oracle_resolve(wl)
    return OA.decode(np.ascontiguousarray(t.q[last]), t.k_pool, t.v_pool, tables, t.k_scale, t.v_scale, sm_scale)
