"""Pins of oracle/append.py: torch's float8_e4m3fn cast, the attention oracle's table
walk (what was appended is what attention reads back), hand-built expectations."""
import numpy as np
import torch

from oracle import append as OP
from oracle import attention as OA
from oracle.formats import E4M3_TABLE
from paper_2605_22566_amd import workload as W
from tests.helpers import oracle_resolve


def _torch_e4m3(y):
    return torch.from_numpy(np.ascontiguousarray(y, dtype=np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def test_e4m3_rounding_matches_torch_on_random_values_and_all_midpoints():
    rng = np.random.default_rng(1)
    y = (rng.standard_normal(300000) * np.float32(10.0) ** rng.integers(-4, 3, 300000)).astype(np.float32)
    y = np.clip(y, -448, 448)
    assert np.array_equal(OP.f32_to_e4m3_codes(y), _torch_e4m3(y))
    pos = E4M3_TABLE[:0x7F]
    mids = ((pos[:-1] + pos[1:]) / 2).astype(np.float32)              # exact in fp32
    for sgn in (1.0, -1.0):
        m = (sgn * mids).astype(np.float32)
        assert np.array_equal(OP.f32_to_e4m3_codes(m), _torch_e4m3(m))
        near = np.nextafter(m, np.float32(0)), np.nextafter(m, np.float32(sgn * 1000))
        for z in near:
            assert np.array_equal(OP.f32_to_e4m3_codes(z), _torch_e4m3(z))
    edge = np.array([0.0, -0.0, 448.0, -448.0, 2.0 ** -9, 2.0 ** -10, 2.0 ** -11, 1e-30], dtype=np.float32)
    assert np.array_equal(OP.f32_to_e4m3_codes(edge), _torch_e4m3(edge))


def _case(shape, seed):
    wl = W.small_layered(seed, shape, num_nodes=16, num_layers=4, len_lo=3, len_hi=60, num_req=5, hops=(1, 4),
                         new_lo=1, new_hi=50)
    t = W.make_tensors(wl)
    rng = np.random.default_rng(seed + 1)
    total_q = int(t.q_ptr[-1])
    kn = W.f32_to_bf16_bits(rng.standard_normal((total_q, shape.num_kv_heads, shape.head_dim)).astype(np.float32))
    vn = W.f32_to_bf16_bits(rng.standard_normal((total_q, shape.num_kv_heads, shape.head_dim)).astype(np.float32))
    return wl, t, kn, vn


def test_bf16_append_is_read_back_exactly_by_the_table_walk():
    shape = W.Shape(8, 2, 64)
    wl, t, kn, vn = _case(shape, 21)
    tables = oracle_resolve(wl)
    k2, v2, _, _ = OP.append(t.k_pool, t.v_pool, None, None, tables, kn, vn, t.q_ptr)
    touched = set()
    for r in range(wl.batch.num_req):
        nb = tables["num_blocks"][r]
        K, V = OA.materialize_kv(k2, v2, tables["block_table"][r], tables["block_ntok"][r], nb)
        n = int(wl.batch.new_lens[r])
        q0 = int(t.q_ptr[r])
        assert np.array_equal(K[-n:], W.bf16_bits_to_f32(kn[q0:q0 + n]).astype(np.float64))
        assert np.array_equal(V[-n:], W.bf16_bits_to_f32(vn[q0:q0 + n]).astype(np.float64))
        ntail = (n + 15) // 16
        tail = tables["block_table"][r][nb - ntail:nb]
        touched.update(tail)
        last = tail[-1]
        pad = n - 16 * (ntail - 1)
        assert not k2[last][:, pad:, :].any() and not v2[last][:, :, pad:].any()      # pad slots written as zero
    others = [b for b in range(wl.num_pool_blocks) if b not in touched]
    assert np.array_equal(k2[others], t.k_pool[others]) and np.array_equal(v2[others], t.v_pool[others])


def test_e4m3_append_scales_codes_and_read_back():
    shape = W.Shape(8, 2, 64, W.KV_FP8_E4M3)
    wl, t, kn, vn = _case(shape, 22)
    tables = oracle_resolve(wl)
    k2, v2, ks, vs = OP.append(t.k_pool, t.v_pool, t.k_scale, t.v_scale, tables, kn, vn, t.q_ptr)
    for r in range(wl.batch.num_req):
        nb = tables["num_blocks"][r]
        n = int(wl.batch.new_lens[r])
        q0 = int(t.q_ptr[r])
        ntail = (n + 15) // 16
        for j in range(ntail):
            blk = tables["block_table"][r][nb - ntail + j]
            ntok = min(16, n - 16 * j)
            x = torch.from_numpy(W.bf16_bits_to_f32(kn[q0 + 16 * j:q0 + 16 * j + ntok]))       # [ntok, Hkv, D]
            s = x.abs().max() / 448.0
            assert np.float32(ks[blk]) == np.float32(s.item())
            want = (x / s).clamp(-448, 448).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
            assert np.array_equal(k2[blk][:, :ntok, :], np.transpose(want, (1, 0, 2)))
            xv = torch.from_numpy(W.bf16_bits_to_f32(vn[q0 + 16 * j:q0 + 16 * j + ntok]))
            sv = xv.abs().max() / 448.0
            wantv = (xv / sv).clamp(-448, 448).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
            assert np.float32(vs[blk]) == np.float32(sv.item())
            assert np.array_equal(v2[blk][:, :, :ntok], np.transpose(wantv, (1, 2, 0)))
        K, V = OA.materialize_kv(k2, v2, tables["block_table"][r], tables["block_ntok"][r], nb, ks, vs)
        ref = W.bf16_bits_to_f32(kn[q0:q0 + n]).astype(np.float64)
        # within half a code step of the largest binade: 448 * scale / 16 / 2 per block, loosely 4 % of amax
        assert np.abs(K[-n:] - ref).max() <= 0.04 * np.abs(ref).max()


def test_skipped_requests_and_all_zero_block():
    shape = W.Shape(8, 2, 64, W.KV_FP8_E4M3)
    wl, t, kn, vn = _case(shape, 23)
    tables = oracle_resolve(wl)
    tables["status"][1] = 2                                   # a failed request is left alone
    q0, q1 = int(t.q_ptr[2]), int(t.q_ptr[3])
    kn[q0:q1] = 0                                             # an all-zero tail: scale 1, codes 0
    k2, v2, ks, vs = OP.append(t.k_pool, t.v_pool, t.k_scale, t.v_scale, tables, kn, vn, t.q_ptr)
    # (a failed request has num_blocks 0 in resolved tables; its would-be tail blocks keep their bits)
    tail1 = wl.batch.tail_blocks[wl.batch.tail_ptr[1]:wl.batch.tail_ptr[2]]
    assert np.array_equal(k2[tail1], t.k_pool[tail1]) and np.array_equal(ks[tail1], t.k_scale[tail1])
    nb2 = tables["num_blocks"][2]
    n2 = q1 - q0
    for blk in tables["block_table"][2][nb2 - (n2 + 15) // 16:nb2]:
        assert ks[blk] == 1.0 and not k2[blk].any()


# ---- append_token: the decode-step form ---------------------------------------------------------
def _tables_at(wl, lens):
    """Resolved tables of the same batch when request r has lens[r] new tokens so far."""
    import copy
    w2 = copy.deepcopy(wl)
    w2.batch.new_lens = np.asarray(lens, dtype=np.int32)
    return oracle_resolve(w2)


def _token_rows(t, kn, vn, lens):
    idx = np.array([int(t.q_ptr[r]) + int(lens[r]) - 1 for r in range(len(lens))])
    return kn[idx], vn[idx]


def test_token_by_token_bf16_equals_the_whole_tail_append_and_reads_back():
    shape = W.Shape(8, 2, 64)
    wl, t, kn, vn = _case(shape, 31)
    n = wl.batch.new_lens.astype(np.int64)
    whole = OP.append(t.k_pool, t.v_pool, None, None, oracle_resolve(wl), kn, vn, t.q_ptr)
    k, v = t.k_pool, t.v_pool
    for i in range(int(n.max())):
        lens = np.minimum(i + 1, n)
        tables = _tables_at(wl, lens)
        kt, vt = _token_rows(t, kn, vn, lens)
        k, v, _, _ = OP.append_token(k, v, None, None, tables, kt, vt)
        if i in (0, 16, 17):
            for r in range(wl.batch.num_req):                 # the table walk finds the token where attention reads it
                K, V = OA.materialize_kv(k, v, tables["block_table"][r], tables["block_ntok"][r], tables["num_blocks"][r])
                assert np.array_equal(K[-1], W.bf16_bits_to_f32(kt[r]).astype(np.float64))
                assert np.array_equal(V[-1], W.bf16_bits_to_f32(vt[r]).astype(np.float64))
    assert np.array_equal(k, whole[0]) and np.array_equal(v, whole[1])


def _deq(codes, scale):
    return E4M3_TABLE[codes].astype(np.float64) * np.float64(scale)


def test_token_e4m3_without_growth_with_growth_and_fresh_block():
    shape = W.Shape(8, 2, 64, W.KV_FP8_E4M3)
    wl, t, kn, vn = _case(shape, 32)
    n = wl.batch.new_lens.astype(np.int64)
    r = int(np.argmax(n))                                      # a request with at least 18 new tokens
    assert n[r] >= 18
    lens = np.minimum(5, n)                                    # 5 tokens in: slots 0..4 of the first tail block
    tables = _tables_at(wl, lens)
    q_ptr5 = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    rows = np.concatenate([np.arange(int(t.q_ptr[q]), int(t.q_ptr[q]) + int(lens[q])) for q in range(len(lens))])
    k, v, ks, vs = OP.append(t.k_pool, t.v_pool, t.k_scale, t.v_scale, tables, kn[rows], vn[rows], q_ptr5)
    blk = tables["block_table"][r][tables["num_blocks"][r] - 1]
    lens6 = lens.copy()
    lens6[r] = 6
    tables6 = _tables_at(wl, lens6)
    kt, vt = _token_rows(t, kn, vn, lens6)
    # (a) a small token: no growth.  Scale and older codes keep their bits, the token is coded like torch's cast
    kt_small = kt.copy()
    kt_small[r] = W.f32_to_bf16_bits(W.bf16_bits_to_f32(kt[r]) * np.float32(0.25))
    k2, v2, ks2, vs2 = OP.append_token(k, v, ks, vs, tables6, kt_small, vt)
    assert ks2[blk] == ks[blk]
    assert np.array_equal(k2[blk][:, :5, :], k[blk][:, :5, :]) and np.array_equal(k2[blk][:, 6:, :], k[blk][:, 6:, :])
    x = torch.from_numpy(W.bf16_bits_to_f32(kt_small[r]))
    want = (x / float(ks[blk])).clamp(-448, 448).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(k2[blk][:, 5, :], want)
    # (b) a large token: the scale grows to amax / 448 and the older codes are re-coded
    kt_big = kt.copy()
    kt_big[r] = W.f32_to_bf16_bits(W.bf16_bits_to_f32(kt[r]) * np.float32(8.0))
    vt_small = vt.copy()
    vt_small[r] = W.f32_to_bf16_bits(W.bf16_bits_to_f32(vt[r]) * np.float32(0.25))
    k3, v3, ks3, vs3 = OP.append_token(k, v, ks, vs, tables6, kt_big, vt_small)
    xb = torch.from_numpy(W.bf16_bits_to_f32(kt_big[r]))
    s_new = (xb.abs().max() / 448.0).item()
    assert np.float32(ks3[blk]) == np.float32(s_new) and ks3[blk] > ks[blk]
    old = torch.from_numpy(k[blk][:, :5, :].copy()).view(torch.float8_e4m3fn).float()        # torch's own decode
    want_old = ((old * float(ks[blk])) / s_new).clamp(-448, 448).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(k3[blk][:, :5, :], want_old)
    want_tok = (xb / s_new).clamp(-448, 448).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(k3[blk][:, 5, :], want_tok)
    before, after = _deq(k[blk][:, :5, :], ks[blk]), _deq(k3[blk][:, :5, :], ks3[blk])
    half_step = np.maximum(np.abs(before) * 2.0 ** -4, 2.0 ** -10 * float(ks3[blk]))          # of the new grid
    assert (np.abs(after - before) <= half_step * 1.0001).all()
    assert np.array_equal(v3[blk][:, :, :5], v[blk][:, :, :5]) and vs3[blk] == vs[blk]       # V did not grow
    others = [b for b in range(wl.num_pool_blocks) if b not in {tables6["block_table"][q][tables6["num_blocks"][q] - 1]
                                                                for q in range(len(lens6))}]
    assert np.array_equal(k3[others], k[others]) and np.array_equal(ks3[others], ks[others])
    # (c) token 17 opens a fresh block: zero everywhere but slot 0, scale from the token alone
    lens17 = lens.copy()
    lens17[r] = 17
    tables17 = _tables_at(wl, lens17)
    kt17, vt17 = _token_rows(t, kn, vn, lens17)
    k4, v4, ks4, vs4 = OP.append_token(k, v, ks, vs, tables17, kt17, vt17)
    blk17 = tables17["block_table"][r][tables17["num_blocks"][r] - 1]
    assert blk17 != blk
    x17 = torch.from_numpy(W.bf16_bits_to_f32(kt17[r]))
    assert np.float32(ks4[blk17]) == np.float32((x17.abs().max() / 448.0).item())
    assert not k4[blk17][:, 1:, :].any() and not v4[blk17][:, :, 1:].any()
    assert np.array_equal(k4[blk17][:, 0, :], (x17 / float(ks4[blk17])).clamp(-448, 448).to(torch.float8_e4m3fn).view(torch.uint8).numpy())


def test_token_skips_failed_and_empty_requests():
    shape = W.Shape(8, 2, 64)
    wl, t, kn, vn = _case(shape, 33)
    lens = np.minimum(3, wl.batch.new_lens)
    tables = _tables_at(wl, lens)
    tables["status"][0] = 2
    kt, vt = _token_rows(t, kn, vn, lens)
    k2, v2, _, _ = OP.append_token(t.k_pool, t.v_pool, None, None, tables, kt, vt)
    tail0 = wl.batch.tail_blocks[wl.batch.tail_ptr[0]:wl.batch.tail_ptr[1]]
    assert np.array_equal(k2[tail0], t.k_pool[tail0])
    blk1 = tables["block_table"][1][tables["num_blocks"][1] - 1]
    assert np.array_equal(k2[blk1][:, 2, :], kt[1]) and np.array_equal(v2[blk1][:, :, 2], vt[1])
