"""gf_attn_prefill_noalloc (the work list in the library's fixed device array, nothing allocated) against
gf_attn_prefill on the same inputs: bit-identical outputs, on two calls in a row, the second with a smaller
batch (the array keeps the first call's list); a batch whose list does not fit is refused with a clear error."""
import numpy as np
import pytest
import torch

from paper_2605_22566_amd import binding as B
from paper_2605_22566_amd import runner as R
from paper_2605_22566_amd import workload as W
from tests.gpu_common import assert_close, oracle_prefill, run_resolve

pytestmark = pytest.mark.gpu


def _both(wl):
    t = W.make_tensors(wl)
    sess, tables = run_resolve(wl)
    dev = sess.device
    pool = R.DevicePool.from_host(t, dev)
    q = R.bits_to_device(t.q, dev)
    q_ptr = torch.from_numpy(t.q_ptr).to(dev)
    total_q, max_q = int(t.q.shape[0]), int(wl.batch.new_lens.max())
    outs = []
    for fn in (sess.prefill, sess.prefill_noalloc):
        o = torch.full(q.shape, float("nan"), dtype=torch.bfloat16, device=dev)
        lse = torch.full(q.shape[:2], float("nan"), dtype=torch.float32, device=dev)
        fn(pool, tables, q, q_ptr, total_q, max_q, o, lse)
        torch.cuda.synchronize()
        outs.append((o, lse))
    return t, outs


@pytest.mark.parametrize("shape", [W.Shape(32, 8, 128), W.Shape(8, 2, 64, W.KV_FP8_E4M3)],
                         ids=["bf16_hq32kv8d128", "fp8_hq8kv2d64"])
def test_noalloc_prefill_matches_prefill_on_two_calls_in_a_row(shape):
    big = W.small_layered(41, shape, num_nodes=30, num_layers=6, len_lo=3, len_hi=150, num_req=6, hops=(1, 6),
                          new_lo=20, new_hi=150)
    small = W.small_layered(42, shape, num_nodes=12, num_layers=4, len_lo=3, len_hi=60, num_req=2, hops=(1, 3),
                            new_lo=1, new_hi=30)
    for wl in (big, small):                               # the second call has fewer, shorter requests
        t, ((o_ref, lse_ref), (o, lse)) = _both(wl)
        assert not bool(torch.isnan(o.float()).any().item())
        assert torch.equal(o_ref, o) and torch.equal(lse_ref, lse)
        O, _ = oracle_prefill(wl, t)
        assert_close(o.double().cpu().numpy(), O, shape.kv_dtype, "noalloc prefill vs oracle")


def test_noalloc_prefill_refuses_a_batch_whose_work_list_does_not_fit():
    sh = W.Shape(8, 1, 128)                               # G = 8: 16 new tokens per work item
    wl = W.small_layered(43, sh, num_req=2)
    sess, tables = run_resolve(wl)
    params, dpool, dt = sess._common(R.DevicePool.from_host(W.make_tensors(wl), sess.device), tables, 0.0)
    total_q = 16 * (1 << 17)                              # 131072 items + requests: just over the 1 MiB array
    z = torch.zeros(1, dtype=torch.bfloat16, device=sess.device)
    q_ptr = torch.zeros(3, dtype=torch.int32, device=sess.device)
    with pytest.raises(B.GraphFlowError) as e:
        B.gf_attn_prefill_noalloc(sess.ctx, params, dpool, dt, z, q_ptr, total_q, 1, z)
    assert e.value.code == B.GF_ERR_WORKSPACE and "fixed array" in str(e.value)
