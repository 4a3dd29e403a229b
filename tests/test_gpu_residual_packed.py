"""The packed residual form on the GPU (bit mask per image + values in element order; paper, Differential-based KV
Cache, Eq. 7): gf_kv_residual_pack / gf_kv_residual_unpack against oracle.residual.pack_rows / unpack_rows bit for
bit, gf_kv_apply_residual_packed against oracle.residual.reconstruct_packed bit for bit (and against the library's
own coordinate-list reconstruction), and the chain produce -> pack -> reconstruct."""
import numpy as np
import pytest
import torch

from oracle import residual as OR
from paper_2605_22566_amd import binding as B
from paper_2605_22566_amd import runner as R
from paper_2605_22566_amd import workload as W
from tests.gpu_common import run_resolve
from tests.test_gpu_residual import _setup

pytestmark = pytest.mark.gpu


def _shuffled_rows(res, seed):
    """The same residual with the entries of every row in random order (pack must not depend on it)."""
    rng = np.random.default_rng(seed)
    idx, val = res.res_idx.copy(), res.res_val.copy()
    p = res.res_ptr.astype(np.int64)
    for r in range(p.size - 1):
        o = rng.permutation(int(p[r + 1] - p[r])) + int(p[r])
        idx[p[r]:p[r + 1]], val[p[r]:p[r + 1]] = res.res_idx[o], res.res_val[o]
    return W.Residuals(res.src_blocks, res.dst_blocks, res.res_ptr, idx, val)


def _u16(t):
    return t.cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("shape", [W.Shape(8, 2, 64), W.Shape(32, 8, 128), W.Shape(4, 1, 128), W.Shape(12, 3, 64)],
                         ids=lambda s: f"kv{s.num_kv_heads}d{s.head_dim}")
def test_pack_unpack_and_reconstruction_are_bit_exact(shape):
    wl2, t, res0 = _setup(shape, 500 + shape.head_dim + shape.num_kv_heads)
    res = _shuffled_rows(res0, 5)
    want_mask, want_val = OR.pack_rows(res.res_ptr, res.res_idx, res.res_val, shape.head_dim)
    sess, tables = run_resolve(wl2)
    dres = sess.upload_residuals(res)
    packed = sess.pack_residuals(dres)
    torch.cuda.synchronize()
    assert packed["pack_status"].cpu().numpy().tolist() == [0] * res.num_items
    assert np.array_equal(packed["mask"].cpu().numpy().view(np.uint32), want_mask)
    assert np.array_equal(_u16(packed["pval"]), want_val)
    idx, st = sess.unpack_residuals(packed)
    torch.cuda.synchronize()
    assert st.cpu().numpy().tolist() == [0] * res.num_items
    assert np.array_equal(_u16(idx), OR.unpack_rows(res.res_ptr, want_mask, shape.head_dim))
    assert np.array_equal(_u16(idx), res0.res_idx)                  # the generator's rows are sorted by element
    assert np.array_equal(want_val, res0.res_val)
    # reconstruction from the packed form: the oracle's, and the coordinate-list kernel's
    want_k, want_v, want_st = OR.reconstruct_packed(t.k_pool, t.v_pool, res.src_blocks, res.dst_blocks, res.res_ptr,
                                                    want_mask, want_val)
    pool = R.DevicePool.from_host(t, sess.device)
    sess.apply_residual_packed(pool, packed)
    torch.cuda.synchronize()
    assert packed["status"].cpu().numpy().tolist() == want_st.tolist() == [0] * res.num_items
    assert np.array_equal(R.bf16_to_bits(pool.k), want_k) and np.array_equal(R.bf16_to_bits(pool.v), want_v)
    pool2 = R.DevicePool.from_host(t, sess.device)
    sess.apply_residual(pool2, dres)
    torch.cuda.synchronize()
    assert torch.equal(pool2.k.view(torch.int16), pool.k.view(torch.int16))
    assert torch.equal(pool2.v.view(torch.int16), pool.v.view(torch.int16))


def test_densities_zero_and_one_and_no_items():
    shape = W.Shape(8, 2, 128)
    for dk, dv in ((0.0, 0.0), (1.0, 1.0)):
        wl2, t, res = _setup(shape, 51, last_nodes=1, density_k=dk, density_v=dv)
        sess, _ = run_resolve(wl2)
        packed = sess.pack_residuals(sess.upload_residuals(res))
        want_mask, want_val = OR.pack_rows(res.res_ptr, res.res_idx, res.res_val, shape.head_dim)
        assert np.array_equal(packed["mask"].cpu().numpy().view(np.uint32), want_mask)
        want_k, want_v, _ = OR.reconstruct_packed(t.k_pool, t.v_pool, res.src_blocks, res.dst_blocks, res.res_ptr,
                                                  want_mask, want_val)
        pool = R.DevicePool.from_host(t, sess.device)
        sess.apply_residual_packed(pool, packed)
        torch.cuda.synchronize()
        assert np.array_equal(R.bf16_to_bits(pool.k), want_k) and np.array_equal(R.bf16_to_bits(pool.v), want_v)
    sh = shape
    params = B.make_params(sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.kv_dtype)
    B.gf_kv_residual_pack(sess.ctx, params, 0, None, None, None, None, None)          # nothing to do, nothing read
    B.gf_kv_residual_unpack(sess.ctx, params, 0, None, None, None)
    B.gf_kv_apply_residual_packed(sess.ctx, params, None, None, 4, 0, None, None, None, None, None)


def test_bad_rows_are_reported_and_contained():
    shape = W.Shape(8, 2, 64)
    wl2, t, res = _setup(shape, 52, last_nodes=1)
    assert res.num_items >= 3
    rows_per_item = 2 * shape.num_kv_heads
    p = res.res_ptr.astype(np.int64)
    # item 0: an entry outside the image; item 1: an element named twice (first row with two entries or more)
    idx = res.res_idx.copy()
    r0 = next(r for r in range(rows_per_item) if p[r + 1] - p[r] >= 1)
    idx[p[r0]] = 16 * shape.head_dim + 3
    r1 = next(r for r in range(rows_per_item, 2 * rows_per_item) if p[r + 1] - p[r] >= 2)
    idx[p[r1] + 1] = idx[p[r1]]
    bad = W.Residuals(res.src_blocks, res.dst_blocks, res.res_ptr, idx, res.res_val)
    sess, _ = run_resolve(wl2)
    dres = sess.upload_residuals(bad)
    packed = sess.pack_residuals(dres)
    torch.cuda.synchronize()
    st = packed["pack_status"].cpu().numpy()
    assert st[0] == B.GF_RS_BAD_INDEX and st[1] == B.GF_RS_BAD_INDEX and (st[2:] == 0).all()
    # the other items are packed as if nothing had happened
    want_mask, want_val = OR.pack_rows(res.res_ptr, res.res_idx, res.res_val, shape.head_dim)
    lo = int(p[2 * rows_per_item])
    assert np.array_equal(packed["mask"].cpu().numpy().view(np.uint32)[2 * rows_per_item:], want_mask[2 * rows_per_item:])
    assert np.array_equal(_u16(packed["pval"])[lo:], want_val[lo:])
    # a mask with one bit too many / too few: reported by unpack and by the reconstruction, all writes in bounds
    good = sess.pack_residuals(sess.upload_residuals(res))
    m = good["mask"].clone()
    row = next(r for r in range(rows_per_item) if p[r + 1] - p[r] >= 1)
    free = next(b for b in range(31) if not (int(want_mask[row, 0]) >> b) & 1)
    m[row, 0] |= 1 << free
    broken = dict(good, mask=m)
    idx_out, st = sess.unpack_residuals(broken)
    torch.cuda.synchronize()
    st = st.cpu().numpy()
    assert st[0] == B.GF_RS_BAD_INDEX and (st[1:] == 0).all()
    pool = R.DevicePool.from_host(t, sess.device)
    broken["status"].fill_(-77)
    sess.apply_residual_packed(pool, broken)
    torch.cuda.synchronize()
    st = broken["status"].cpu().numpy()
    assert st[0] == B.GF_RS_BAD_INDEX and (st[1:] == 0).all()
    want_k, want_v, want_st = OR.reconstruct_packed(t.k_pool, t.v_pool, res.src_blocks, res.dst_blocks, res.res_ptr,
                                                    m.cpu().numpy().view(np.uint32), want_val)
    assert want_st.tolist() == st.tolist()
    d = res.dst_blocks[1:]
    assert np.array_equal(R.bf16_to_bits(pool.k)[d], want_k[d]) and np.array_equal(R.bf16_to_bits(pool.v)[d], want_v[d])
    # blocks outside the pool
    wild = dict(good, src=good["src"].clone())
    wild["src"][0] = 10 ** 6
    wild["status"].fill_(-77)
    sess.apply_residual_packed(R.DevicePool.from_host(t, sess.device), wild)
    torch.cuda.synchronize()
    assert wild["status"].cpu().numpy()[0] == B.GF_RS_BAD_BLOCK


def test_made_residual_packs_without_moving_its_values_and_reconstructs_the_instance_blocks():
    """gf_kv_make_residual at share 1 -> pack -> reconstruct from the packed form gives back the prefix-conditioned
    blocks bit for bit wherever bf16 holds the differences exactly (small-integer test values do)."""
    shape = W.Shape(8, 2, 128)
    wl = W.small_layered(1, shape, num_req=1)
    rng = np.random.default_rng(53)
    n = 6
    nb = 3 * n
    k = OR.f32_to_bf16_bits_rne(rng.integers(-8, 9, (nb, 2, 16, 128)).astype(np.float32))
    v = OR.f32_to_bf16_bits_rne(rng.integers(-8, 9, (nb, 2, 128, 16)).astype(np.float32))
    base = np.arange(n, dtype=np.int32)
    full = np.arange(n, 2 * n, dtype=np.int32)
    # the "full" blocks differ from their base in about a third of the elements
    for b in range(n):
        mk, mv = rng.random(k[0].shape) < 0.3, rng.random(v[0].shape) < 0.3
        k[full[b]] = np.where(mk, OR.f32_to_bf16_bits_rne(rng.integers(-8, 9, k[0].shape).astype(np.float32)), k[base[b]])
        v[full[b]] = np.where(mv, OR.f32_to_bf16_bits_rne(rng.integers(-8, 9, v[0].shape).astype(np.float32)), v[base[b]])
    sess = R.Session(wl)
    dev = sess.device
    pool = R.DevicePool(R.bits_to_device(k, dev), R.bits_to_device(v, dev), nb)
    made = sess.make_residual(pool, torch.from_numpy(base).to(dev), torch.from_numpy(full).to(dev), share=1.0)
    torch.cuda.synchronize()
    nnz = int(made["ptr"][-1].item())
    made["idx"], made["val"] = made["idx"][:max(nnz, 1)], made["val"][:max(nnz, 1)]
    packed = sess.pack_residuals(made)
    torch.cuda.synchronize()
    assert torch.equal(packed["pval"][:nnz], made["val"][:nnz])       # sorted rows: the values do not move
    out = torch.arange(2 * n, 3 * n, dtype=torch.int32, device=dev)
    packed["dst"], packed["src"] = out, torch.from_numpy(base).to(dev)
    packed["status"] = torch.full((n,), -77, dtype=torch.int32, device=dev)
    sess.apply_residual_packed(pool, packed)
    torch.cuda.synchronize()
    assert packed["status"].cpu().numpy().tolist() == [0] * n
    got_k, got_v = R.bf16_to_bits(pool.k), R.bf16_to_bits(pool.v)
    assert np.array_equal(got_k[2 * n:3 * n], k[full]) and np.array_equal(got_v[2 * n:3 * n], v[full])
