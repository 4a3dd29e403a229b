"""Full-size benchmark configurations in the launch configuration bench.py times (device-filled pools),
checked on sampled requests the oracle can compute one by one, plus properties that hold at any size."""
import numpy as np
import pytest
import torch

from oracle import attention as OA
from paper_2605_22566_amd import runner as R
from paper_2605_22566_amd import workload as W
from tests.gpu_common import TOL
from tests.helpers import max_blocks_of, oracle_resolve

pytestmark = pytest.mark.gpu


def _setup(name):
    wl = W.CONFIGS[name]()
    sess = R.Session(wl)
    dev = sess.device
    b = wl.batch
    tables = sess.resolve(sess.upload_batch(b), sess.alloc_tables(b.num_req, max_blocks_of(wl)))
    pool = R.DevicePool.random(wl, dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(wl.seed + 1)
    sh = wl.shape
    q = torch.randn((int(b.new_lens.sum()), sh.num_q_heads, sh.head_dim), generator=gen, device=dev,
                    dtype=torch.float32).to(torch.bfloat16)
    q_ptr = np.concatenate([[0], np.cumsum(b.new_lens)]).astype(np.int32)
    return wl, sess, tables, pool, q, q_ptr


def _check_rows(wl, pool, want_tables, q_bits_rows, got_rows, r, decode):
    nb = want_tables["num_blocks"][r]
    ids = np.array(want_tables["block_table"][r][:nb], dtype=np.int64)
    kk, vv, ks, vs = pool.gather_host(ids)
    local = {k: [v[r]] for k, v in want_tables.items()}
    local["block_table"] = [list(range(nb))]
    if decode:
        O, _ = OA.decode(q_bits_rows, kk, vv, local, ks, vs)
    else:
        O, _ = OA.prefill(q_bits_rows, np.array([0, q_bits_rows.shape[0]]), kk, vv, local, ks, vs)
    atol, rtol = TOL[wl.shape.kv_dtype]
    err = np.abs(got_rows - O)
    assert (err <= atol + rtol * np.abs(O)).all(), f"request {r}: max err {err.max()}"


def test_prefill_8b_full_size_sampled():
    wl, sess, tables, pool, q, q_ptr = _setup("prefill_8b")
    want = oracle_resolve(wl)
    assert R.tables_to_host(tables)["block_table"] == want["block_table"]
    o = torch.full_like(q, float("nan"))
    sess.prefill(pool, tables, q, torch.from_numpy(q_ptr).to(sess.device), int(q.shape[0]),
                 int(wl.batch.new_lens.max()), o)
    torch.cuda.synchronize()
    og = o.double().cpu().numpy()
    assert np.isfinite(og).all()                       # every row of every request was written
    qb = R.bf16_to_bits(q)
    n = wl.batch.new_lens
    for r in (int(np.argmin(n)), int(np.argmax(n)), 17):          # shortest, longest, one more
        lo, hi = int(q_ptr[r]), int(q_ptr[r + 1])
        _check_rows(wl, pool, want, qb[lo:hi], og[lo:hi], r, decode=False)


@pytest.mark.parametrize("name", ["decode_8b", "mixed_fp8"])
def test_decode_full_size_sampled(name):
    wl, sess, tables, pool, q, q_ptr = _setup(name)
    want = oracle_resolve(wl)
    last = torch.from_numpy((q_ptr[1:] - 1).astype(np.int64)).to(sess.device)
    qd = q[last].contiguous()
    od = torch.full_like(qd, float("nan"))
    lse = torch.empty(qd.shape[:2], dtype=torch.float32, device=sess.device)
    sess.decode(pool, tables, qd, od, lse)
    torch.cuda.synchronize()
    og = od.double().cpu().numpy()
    assert np.isfinite(og).all()
    # convex-hull property at full size: |o| cannot exceed the largest |v| in the pool
    vmax = float(pool.v.float().abs().max()) if pool.v.dtype == torch.bfloat16 else \
        float((pool.v.view(torch.float8_e4m3fn).float().abs().amax(dim=(1, 2, 3)) * pool.v_scale).max())
    assert np.abs(og).max() <= vmax * 1.01 + 1e-2
    qb = R.bf16_to_bits(qd)
    L = W.context_lens(wl)
    for r in (int(np.argmin(L)), int(np.argmax(L)), wl.batch.num_req - 1):
        _check_rows(wl, pool, want, qb[r:r + 1], og[r:r + 1], r, decode=True)
