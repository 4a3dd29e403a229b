"""The calls can be recorded into a HIP graph once a warm-up call has sized the context's buffers (no call
allocates or synchronises after that): a captured resolve -> prefill -> decode (per request, per node, and the three residual-reading calls) sequence, replayed
several times with inputs changed in place and eager work in between, gives the eager result bit for bit."""
import numpy as np
import pytest
import torch

from paper_2605_22566_amd import runner as R
from paper_2605_22566_amd import workload as W
from tests.helpers import max_blocks_of

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape", [W.Shape(32, 8, 128), W.Shape(8, 2, 64, W.KV_FP8_E4M3)],
                         ids=["bf16", "fp8"])
def test_captured_sequence_replays_like_eager(shape):
    wl = W.small_layered(444 + shape.kv_dtype, shape, num_nodes=16, num_layers=4, len_lo=10, len_hi=150, num_req=12,
                         hops=(2, 4), new_lo=1, new_hi=60)
    t = W.make_tensors(wl)
    sess = R.Session(wl)
    dev = sess.device
    pool = R.DevicePool.from_host(t, dev)
    db = sess.upload_batch(wl.batch)
    tables = sess.alloc_tables(wl.batch.num_req, max_blocks_of(wl))
    q = R.bits_to_device(t.q, dev)
    q_ptr = torch.from_numpy(t.q_ptr).to(dev)
    last = torch.from_numpy((t.q_ptr[1:] - 1).astype(np.int64)).to(dev)
    total_q, max_q = int(q.shape[0]), int(wl.batch.new_lens.max())
    o = torch.zeros_like(q)
    qd = q[last].contiguous()
    od, ods, odr, odsr = (torch.zeros_like(qd) for _ in range(4))
    opr = torch.zeros_like(q)
    # bf16 pools: the read-time residual step too (the first two table entries of every request carry an item)
    bf16 = shape.kv_dtype == W.KV_BF16
    handles = torch.full((wl.batch.num_req, max_blocks_of(wl)), -1, dtype=torch.int32, device=dev)
    handles[:, :2] = torch.arange(2 * wl.batch.num_req, dtype=torch.int32, device=dev).view(-1, 2)
    dres = R.random_residuals(shape, 2 * wl.batch.num_req, dev)[0] if bf16 else None

    def sequence():
        sess.resolve(db, tables)
        sess.prefill(pool, tables, q, q_ptr, total_q, max_q, o)
        sess.decode(pool, tables, qd, od)
        sess.decode_shared(pool, db, tables, qd, ods)
        if bf16:
            sess.decode_residual(pool, tables, handles, dres, qd, odr)
            sess.prefill_residual(pool, tables, handles, dres, q, q_ptr, total_q, max_q, opr)
            sess.decode_shared_residual(pool, db, tables, handles, dres, qd, odsr)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                       # warm-up: buffers sized, occupancy queried
        sequence()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sequence()
    torch.cuda.synchronize()
    for rep in range(3):
        q.mul_(-0.5 if rep == 1 else 1.5)               # new inputs in the same buffers
        qd.copy_(q[last])
        bufs = (o, od, ods, odr, opr, odsr)
        for buf in bufs:
            buf.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = [x.clone() for x in bufs]
        for buf in bufs:
            buf.fill_(float("nan"))
        sequence()                                      # the program's own eager work between replays
        torch.cuda.synchronize()
        names = ("prefill", "decode", "decode_shared", "decode_residual", "prefill_residual", "decode_shared_residual")
        for name, g, e in zip(names, got, bufs):
            if name.endswith("residual") and not bf16:
                continue
            assert torch.equal(g, e), f"{name}, replay {rep}"
            assert torch.isfinite(e.float()).all()
        if bf16:
            assert not torch.equal(odr, od) and not torch.equal(opr, o)      # the residuals are seen
