"""gf_kv_apply_residual through the C ABI vs oracle/residual.py (bit-exact), and
attention over the reconstructed blocks vs the attention oracle."""
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


def _setup(shape, seed, last_nodes=2, **kw):
    wl = W.small_layered(seed, shape, num_nodes=24, num_layers=5, len_lo=3, len_hi=90, num_req=5, hops=(1, 5),
                         new_lo=1, new_hi=40)
    t = W.make_tensors(wl)
    wl2, res = W.add_residual_instances(wl, last_nodes=last_nodes, **kw)
    extra = wl2.num_pool_blocks - wl.num_pool_blocks
    nan_k = np.full((extra,) + t.k_pool.shape[1:], 0x7FC0, np.uint16)      # must be overwritten completely
    nan_v = np.full((extra,) + t.v_pool.shape[1:], 0x7FC0, np.uint16)
    t.k_pool = np.concatenate([t.k_pool, nan_k])
    t.v_pool = np.concatenate([t.v_pool, nan_v])
    return wl2, t, res


def _apply_on_gpu(wl2, t, res):
    sess, tables = run_resolve(wl2)
    pool = R.DevicePool.from_host(t, sess.device)
    dres = sess.upload_residuals(res)
    sess.apply_residual(pool, dres)
    torch.cuda.synchronize()
    return sess, tables, pool, dres


@pytest.mark.parametrize("shape", [W.Shape(8, 2, 64), W.Shape(32, 8, 128), W.Shape(4, 1, 128)],
                         ids=lambda s: f"kv{s.num_kv_heads}d{s.head_dim}")
def test_reconstruction_is_bit_exact(shape):
    wl2, t, res = _setup(shape, 300 + shape.head_dim + shape.num_kv_heads)
    want_k, want_v, want_st = OR.reconstruct(t.k_pool, t.v_pool, res.src_blocks, res.dst_blocks, res.res_ptr,
                                             res.res_idx, res.res_val)
    sess, _, pool, dres = _apply_on_gpu(wl2, t, res)
    assert dres["status"].cpu().numpy().tolist() == want_st.tolist() == [0] * res.num_items
    assert np.array_equal(R.bf16_to_bits(pool.k), want_k)
    assert np.array_equal(R.bf16_to_bits(pool.v), want_v)
    assert not np.isnan(OR.bf16_bits_to_f32(want_k[res.dst_blocks])).any()
    # entry arrays off the 16-byte grid are read entry by entry: same blocks
    pool2 = R.DevicePool.from_host(t, sess.device)
    for key in ("idx", "val"):
        dres[key] = torch.cat([torch.zeros(3, dtype=dres[key].dtype, device=sess.device), dres[key]])[3:]
        assert dres[key].data_ptr() % 16 != 0
    dres["status"].fill_(-77)
    sess.apply_residual(pool2, dres)
    torch.cuda.synchronize()
    assert dres["status"].cpu().numpy().tolist() == [0] * res.num_items
    assert torch.equal(pool2.k.view(torch.int16), pool.k.view(torch.int16))
    assert torch.equal(pool2.v.view(torch.int16), pool.v.view(torch.int16))


def test_densities_zero_and_one_and_no_items():
    shape = W.Shape(8, 2, 64)
    for dk, dv in ((0.0, 0.0), (1.0, 1.0)):
        wl2, t, res = _setup(shape, 41, last_nodes=1, density_k=dk, density_v=dv)
        want_k, want_v, _ = OR.reconstruct(t.k_pool, t.v_pool, res.src_blocks, res.dst_blocks, res.res_ptr,
                                           res.res_idx, res.res_val)
        _, _, pool, _ = _apply_on_gpu(wl2, t, res)
        assert np.array_equal(R.bf16_to_bits(pool.k), want_k) and np.array_equal(R.bf16_to_bits(pool.v), want_v)
    wl2, t, res = _setup(shape, 42, last_nodes=1)
    empty = W.Residuals(res.src_blocks[:0], res.dst_blocks[:0], res.res_ptr[:1], res.res_idx[:0], res.res_val[:0])
    _, _, pool, _ = _apply_on_gpu(wl2, t, empty)
    assert np.array_equal(R.bf16_to_bits(pool.k), t.k_pool)


def test_bad_block_and_bad_index_are_reported_and_contained():
    shape = W.Shape(8, 2, 64)
    wl2, t, res = _setup(shape, 43, last_nodes=1)
    res.src_blocks[1] = wl2.num_pool_blocks + 5             # outside the pool
    res.dst_blocks[2] = -1
    e = int(res.res_ptr[0])
    res.res_idx[e] = 16 * shape.head_dim                     # first entry of item 0: outside its image
    want_k, want_v, want_st = OR.reconstruct(t.k_pool, t.v_pool, res.src_blocks, res.dst_blocks, res.res_ptr,
                                             res.res_idx, res.res_val)
    assert want_st[:3].tolist() == [OR.ST_BAD_INDEX, OR.ST_BAD_BLOCK, OR.ST_BAD_BLOCK]
    _, _, pool, dres = _apply_on_gpu(wl2, t, res)
    assert dres["status"].cpu().numpy().tolist() == want_st.tolist()
    got_k, got_v = R.bf16_to_bits(pool.k), R.bf16_to_bits(pool.v)
    assert np.array_equal(got_k, want_k) and np.array_equal(got_v, want_v)


def test_e4m3_pool_without_scales_is_refused():
    shape = W.Shape(8, 2, 64, W.KV_FP8_E4M3)
    wl = W.small_layered(44, shape, num_req=2)
    sess = R.Session(wl)
    params = B.make_params(8, 2, 64, W.KV_FP8_E4M3)
    z = torch.zeros(4, dtype=torch.int32, device=sess.device)
    with pytest.raises(B.GraphFlowError) as ei:
        B.gf_kv_apply_residual(sess.ctx, params, z, z, 1, 1, z, z, z, z, z, None)
    assert ei.value.code == B.GF_ERR_NULL


def test_attention_over_reconstructed_instances_matches_the_oracle():
    """base + residual -> instance blocks -> resolve (instances on the paths) -> prefill and decode."""
    shape = W.Shape(32, 8, 128)
    wl2, t, res = _setup(shape, 45, last_nodes=2)
    want_k, want_v, _ = OR.reconstruct(t.k_pool, t.v_pool, res.src_blocks, res.dst_blocks, res.res_ptr,
                                       res.res_idx, res.res_val)
    sess, tables, pool, _ = _apply_on_gpu(wl2, t, res)
    assert tables["status"].cpu().numpy().tolist() == [0] * wl2.batch.num_req
    dev = sess.device
    q = R.bits_to_device(t.q, dev)
    q_ptr = torch.from_numpy(t.q_ptr).to(dev)
    o = torch.full(q.shape, float("nan"), dtype=torch.bfloat16, device=dev)
    sess.prefill(pool, tables, q, q_ptr, int(t.q.shape[0]), int(wl2.batch.new_lens.max()), o)
    last = (t.q_ptr[1:] - 1).astype(np.int64)
    qd = R.bits_to_device(np.ascontiguousarray(t.q[last]), dev)
    od = torch.full(qd.shape, float("nan"), dtype=torch.bfloat16, device=dev)
    sess.decode(pool, tables, qd, od)
    torch.cuda.synchronize()
    ot = oracle_resolve(wl2)
    O, _ = OA.prefill(t.q, t.q_ptr, want_k, want_v, ot)
    Od, _ = OA.decode(np.ascontiguousarray(t.q[last]), want_k, want_v, ot)
    assert_close(bf16_out_to_f64(o), O, W.KV_BF16, "prefill over instances")
    assert_close(bf16_out_to_f64(od), Od, W.KV_BF16, "decode over instances")


# ---- e4m3 pools ---------------------------------------------------------------------------------
def _setup_e4m3(shape, seed, last_nodes=2, **kw):
    wl = W.small_layered(seed, shape, num_nodes=24, num_layers=5, len_lo=3, len_hi=90, num_req=5, hops=(1, 5),
                         new_lo=1, new_hi=40)
    t = W.make_tensors(wl)
    wl2, res = W.add_residual_instances(wl, last_nodes=last_nodes, **kw)
    extra = wl2.num_pool_blocks - wl.num_pool_blocks
    t.k_pool = np.concatenate([t.k_pool, np.full((extra,) + t.k_pool.shape[1:], 0x55, np.uint8)])   # to be overwritten
    t.v_pool = np.concatenate([t.v_pool, np.full((extra,) + t.v_pool.shape[1:], 0x55, np.uint8)])
    t.k_scale = np.concatenate([t.k_scale, np.full(extra, -7.0, np.float32)])
    t.v_scale = np.concatenate([t.v_scale, np.full(extra, -7.0, np.float32)])
    return wl2, t, res


# 2 and 8 kv heads take the one-pass kernel (a wave per head), 3 the two-pass one
@pytest.mark.parametrize("shape", [W.Shape(8, 2, 64, W.KV_FP8_E4M3), W.Shape(32, 8, 128, W.KV_FP8_E4M3),
                                   W.Shape(6, 3, 64, W.KV_FP8_E4M3), W.Shape(12, 3, 128, W.KV_FP8_E4M3)],
                         ids=lambda s: f"kv{s.num_kv_heads}d{s.head_dim}fp8")
def test_e4m3_reconstruction_is_bit_exact_and_attention_reads_it(shape):
    wl2, t, res = _setup_e4m3(shape, 500 + shape.head_dim)
    want = OR.reconstruct_e4m3(t.k_pool, t.v_pool, t.k_scale, t.v_scale, res.src_blocks, res.dst_blocks, res.res_ptr,
                               res.res_idx, res.res_val)
    sess, tables, pool, dres = _apply_on_gpu(wl2, t, res)
    assert dres["status"].cpu().numpy().tolist() == want[4].tolist() == [0] * res.num_items
    assert np.array_equal(pool.k.cpu().numpy(), want[0]) and np.array_equal(pool.v.cpu().numpy(), want[1])
    assert np.array_equal(pool.k_scale.cpu().numpy(), want[2]) and np.array_equal(pool.v_scale.cpu().numpy(), want[3])
    assert (want[2][res.dst_blocks] > 0).all()
    # decode over the instance nodes reads the reconstructed blocks
    last = (t.q_ptr[1:] - 1).astype(np.int64)
    q = R.bits_to_device(np.ascontiguousarray(t.q[last]), sess.device)
    o = torch.zeros_like(q)
    sess.decode(pool, tables, q, o)
    torch.cuda.synchronize()
    O, _ = OA.decode(np.ascontiguousarray(t.q[last]), want[0], want[1], oracle_resolve(wl2), want[2], want[3])
    assert_close(bf16_out_to_f64(o), O, shape.kv_dtype, "decode over reconstructed e4m3 blocks")


def test_e4m3_in_place_and_bad_items():
    """Source = destination is allowed on an e4m3 pool (an image is read before it is written, the source scale
    before the destination's); bad block ids and indices are reported as on bf16 pools."""
    for shape in (W.Shape(8, 2, 64, W.KV_FP8_E4M3), W.Shape(6, 3, 64, W.KV_FP8_E4M3)):      # one-pass and two-pass kernel
        _in_place_case(shape)


def _in_place_case(shape):
    wl = W.small_layered(61, shape, num_req=3)
    t = W.make_tensors(wl)
    rng = np.random.default_rng(62)
    img = 16 * shape.head_dim
    src = np.array([3, 5, wl.num_pool_blocks + 3, 7], np.int32)          # the third item has a bad source
    dst = np.array([3, 5, 0, 7], np.int32)                               # the others are rebuilt in place
    ptr, idx, val = [0], [], []
    for item in range(len(src)):
        for row in range(2 * shape.num_kv_heads):
            ii = np.sort(rng.choice(img, size=int(rng.integers(0, 200)), replace=False))
            idx.extend(ii.tolist())
            val.extend(W.f32_to_bf16_bits((rng.standard_normal(ii.size) * 0.5).astype(np.float32)).tolist())
            ptr.append(len(idx))
    idx = np.array(idx, np.uint16)
    idx[0] = img                                                         # one entry outside its image
    res = W.Residuals(src, dst, np.array(ptr, np.int32), idx, np.array(val, np.uint16))
    want = OR.reconstruct_e4m3(t.k_pool, t.v_pool, t.k_scale, t.v_scale, src, dst, res.res_ptr, res.res_idx, res.res_val)
    assert want[4].tolist() == [OR.ST_BAD_INDEX, 0, OR.ST_BAD_BLOCK, 0]
    _, _, pool, dres = _apply_on_gpu(wl, t, res)
    assert dres["status"].cpu().numpy().tolist() == want[4].tolist()
    assert np.array_equal(pool.k.cpu().numpy(), want[0]) and np.array_equal(pool.v.cpu().numpy(), want[1])
    assert np.array_equal(pool.k_scale.cpu().numpy(), want[2]) and np.array_equal(pool.v_scale.cpu().numpy(), want[3])
