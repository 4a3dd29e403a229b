"""Pins of oracle/residual.py against things other than itself: torch's bf16 cast
and element-wise add, hand-indexed physical elements, a block-free construction
of base + delta on the token-major segment, and brute force over subsets."""
import itertools

import numpy as np
import torch

from oracle import attention as OA
from oracle import residual as OR


def _torch_bf16_bits(x):
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def test_bf16_rounding_matches_torch_on_random_ties_and_extremes():
    rng = np.random.default_rng(3)
    x = rng.standard_normal(200000).astype(np.float32) * np.float32(10.0) ** rng.integers(-20, 20, 200000)
    assert np.array_equal(OR.f32_to_bf16_bits_rne(x), _torch_bf16_bits(x))
    # exact ties: low 16 bits = 0x8000, both parities of the kept lsb
    hi = rng.integers(0x0080, 0x7F00, 5000).astype(np.uint32)
    ties = ((hi << 16) | 0x8000).view(np.float32)
    assert np.array_equal(OR.f32_to_bf16_bits_rne(ties), _torch_bf16_bits(ties))
    assert np.array_equal(OR.f32_to_bf16_bits_rne(-ties), _torch_bf16_bits(-ties))
    ext = np.array([0.0, -0.0, 1.0, 3.3895314e38, 1e-40, -1e-40, 1.17549435e-38], dtype=np.float32)
    assert np.array_equal(OR.f32_to_bf16_bits_rne(ext), _torch_bf16_bits(ext))


def _pool(rng, nb, hkv, dim):
    k = _torch_bf16_bits(rng.standard_normal((nb, hkv, 16, dim)).astype(np.float32)).copy()
    v = _torch_bf16_bits(rng.standard_normal((nb, hkv, dim, 16)).astype(np.float32)).copy()
    return k, v


def test_empty_residual_is_identity_and_minus_base_gives_zero():
    rng = np.random.default_rng(4)
    hkv, dim = 2, 64
    k, v = _pool(rng, 4, hkv, dim)
    k2, v2, st = OR.reconstruct(k, v, [0, 1], [2, 3], [0] * (2 * 2 * hkv + 1), np.zeros(0, np.uint16), np.zeros(0, np.uint16))
    assert st.tolist() == [0, 0]
    assert np.array_equal(k2[2], k[0]) and np.array_equal(v2[3], v[1])
    assert np.array_equal(k2[:2], k[:2]) and np.array_equal(v2[:2], v[:2])       # sources untouched
    # residual = -base on every element of block 0 (rows: K heads then V heads; inside a row [slot][d])
    img = 16 * dim
    vals = np.concatenate([k[0].ravel() ^ 0x8000, np.transpose(v[0], (0, 2, 1)).ravel() ^ 0x8000]).astype(np.uint16)
    full_ptr = np.arange(2 * hkv + 1) * img
    full_idx = np.tile(np.arange(img, dtype=np.uint16), 2 * hkv)
    k3, v3, st = OR.reconstruct(k, v, [0], [2], full_ptr, full_idx, vals)
    assert st.tolist() == [0]
    assert not (k3[2] & 0x7FFF).any() and not (v3[2] & 0x7FFF).any()


def test_full_density_equals_torch_elementwise_add():
    rng = np.random.default_rng(5)
    hkv, dim = 2, 128
    k, v = _pool(rng, 3, hkv, dim)
    img = 16 * dim
    dk = _torch_bf16_bits((rng.standard_normal((hkv, 16, dim)) * 0.3).astype(np.float32))
    dv = _torch_bf16_bits((rng.standard_normal((hkv, 16, dim)) * 0.3).astype(np.float32))   # logical [h][slot][d]
    vals = np.concatenate([dk.ravel(), dv.ravel()])
    k2, v2, _ = OR.reconstruct(k, v, [1], [2], np.arange(2 * hkv + 1) * img, np.tile(np.arange(img, dtype=np.uint16), 2 * hkv), vals)

    def tb(bits):
        return torch.from_numpy(bits.astype(np.int16)).view(torch.bfloat16)
    want_k = (tb(k[1]).float() + tb(dk).float()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    want_v = (tb(v[1]).float() + tb(np.transpose(dv, (0, 2, 1)).copy()).float()).to(torch.bfloat16)
    want_v = want_v.view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(k2[2], want_k)
    assert np.array_equal(v2[2], want_v)


def test_single_entries_land_on_the_hand_indexed_physical_element():
    rng = np.random.default_rng(6)
    hkv, dim = 4, 64
    k, v = _pool(rng, 2, hkv, dim)
    two = np.array([0x4000], np.uint16)                       # bf16 2.0
    for (t, h, slot, d) in [(0, 0, 0, 0), (0, 3, 15, 63), (0, 1, 7, 20), (1, 0, 0, 0), (1, 2, 9, 33), (1, 3, 15, 63)]:
        row = t * hkv + h                                     # written out, not via the oracle's helper
        ptr = [0] * (row + 1) + [1] * (2 * hkv - row)
        k2, v2, st = OR.reconstruct(k, v, [0], [1], ptr, np.array([slot * dim + d], np.uint16), two)
        assert st.tolist() == [0]
        dk = k2[1] != k[0]
        dv = v2[1] != v[0]
        if t == 0:
            assert dk.sum() == 1 and dk[h, slot, d] and not dv.any()
            got = OR.bf16_bits_to_f32(k2[1][h, slot, d:d + 1])[0]
            assert got == OR.bf16_bits_to_f32(OR.f32_to_bf16_bits_rne(OR.bf16_bits_to_f32(k[0][h, slot, d:d + 1]) + 2))[0]
        else:
            assert dv.sum() == 1 and dv[h, d, slot] and not dk.any()


def test_bad_block_and_bad_index_are_reported():
    rng = np.random.default_rng(7)
    hkv, dim = 1, 64
    k, v = _pool(rng, 3, hkv, dim)
    idx = np.array([5, 16 * dim, 7], np.uint16)              # the middle one is outside the image
    val = np.array([0x3F80, 0x3F80, 0x3F80], np.uint16)
    # rows per item: K h0, V h0; all three entries sit in the K row of item 0
    k2, v2, st = OR.reconstruct(k, v, [0, 9, 1], [1, 2, -1], [0, 3, 3, 3, 3, 3, 3], idx, val)
    assert st.tolist() == [OR.ST_BAD_INDEX, OR.ST_BAD_BLOCK, OR.ST_BAD_BLOCK]
    assert (k2[1] != k[0]).sum() == 2                          # the two valid entries were applied
    assert np.array_equal(k2[2], k[2]) and np.array_equal(v2[2], v[2])


def test_node_reconstruction_equals_segment_level_base_plus_delta():
    """Blocks of a ragged node, reconstructed one by one, then read back through the
    attention oracle's table walk, equal base + delta formed on the [token][head][dim]
    arrays directly (token = 16 * block + slot is the only bridge)."""
    rng = np.random.default_rng(8)
    hkv, dim, length = 2, 64, 41                               # 3 blocks, the last with 9 tokens
    nblk = 3
    k, v = _pool(rng, 8, hkv, dim)
    src, dst = [5, 0, 3], [1, 6, 2]
    base_k = np.concatenate([np.transpose(OR.bf16_bits_to_f32(k[b]), (1, 0, 2)) for b in src])[:length]   # [tok][h][d]
    base_v = np.concatenate([np.transpose(OR.bf16_bits_to_f32(v[b]), (2, 0, 1)) for b in src])[:length]
    mask = rng.random((2, length, hkv, dim)) < 0.2
    delta = OR.bf16_bits_to_f32(_torch_bf16_bits((rng.standard_normal((2, length, hkv, dim)) * 0.5).astype(np.float32)))
    delta = np.where(mask, delta, np.float32(0))
    ptr, idx, val = [0], [], []
    for bi in range(nblk):
        for t in (0, 1):
            for h in range(hkv):
                for tok, d in zip(*np.nonzero(mask[t, :, h, :])):
                    if tok // 16 == bi:
                        idx.append((tok % 16) * dim + d)
                        val.append(delta[t, tok, h, d])
                ptr.append(len(idx))
    val_bits = _torch_bf16_bits(np.array(val, np.float32))
    k2, v2, st = OR.reconstruct(k, v, src, dst, ptr, np.array(idx, np.uint16), val_bits)
    assert st.tolist() == [0, 0, 0]
    K, V = OA.materialize_kv(k2, v2, dst, [16, 16, 9], 3)
    want_k = OR.bf16_bits_to_f32(_torch_bf16_bits(base_k + delta[0])).astype(np.float64)
    want_v = OR.bf16_bits_to_f32(_torch_bf16_bits(base_v + delta[1])).astype(np.float64)
    assert K.shape == (length, hkv, dim)
    assert np.array_equal(K, want_k) and np.array_equal(V, want_v)


def test_select_by_energy_matches_brute_force_and_its_invariants():
    rng = np.random.default_rng(9)
    for trial in range(30):
        n = int(rng.integers(1, 11))
        x = rng.standard_normal(n) * rng.choice([0.01, 1.0, 5.0], n)
        total = float((x * x).sum())
        keep = OR.select_by_energy(x, 0.95)
        # brute force: the smallest subset size that reaches the share, and the best energy at that size
        best_size = None
        for size in range(1, n + 1):
            best = max(float((x[list(c)] ** 2).sum()) for c in itertools.combinations(range(n), size))
            if best >= 0.95 * total:
                best_size, best_energy = size, best
                break
        assert len(keep) == best_size
        assert np.isclose(float((x[keep] ** 2).sum()), best_energy)
    y = rng.standard_normal((4, 50)) * (rng.random((4, 50)) < 0.25)
    keep = OR.select_by_energy(y)
    e = (y.ravel() ** 2)
    assert e[keep].sum() >= 0.95 * e.sum()
    assert e[keep].sum() - e[keep].min() < 0.95 * e.sum()      # dropping the smallest kept entry falls short
    assert e[keep].min() >= np.delete(e, keep).max()           # nothing larger was left out
    assert OR.select_by_energy(np.zeros(7)).size == 0
    # the whole energy = every non-zero entry and nothing else, whatever the rounding of the sums (a total taken by
    # another summation than the running sum can stay above every prefix and would keep the zeros too)
    for seed in range(20):
        r2 = np.random.default_rng(seed)
        d = (r2.standard_normal((16, 128)) * (r2.random((16, 128)) < 0.6)).astype(np.float32)
        assert np.array_equal(OR.select_by_energy(d, 1.0), np.flatnonzero(d.ravel()))


# ---- e4m3 pools ---------------------------------------------------------------------------------
def _pool_e4m3(rng, nb, hkv, dim):
    import torch
    x = torch.from_numpy(rng.standard_normal((2, nb, hkv, 16, dim)).astype(np.float32))
    scale = x.abs().amax(dim=(2, 3, 4)) / 448.0                       # [2, nb]
    codes = (x / scale[:, :, None, None, None]).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    k = codes[0].copy()
    v = np.ascontiguousarray(np.transpose(codes[1], (0, 1, 3, 2)))     # [nb, Hkv, D, 16]
    return k, v, scale[0].numpy().copy(), scale[1].numpy().copy()


def test_e4m3_empty_residual_recodes_a_block_onto_itself():
    rng = np.random.default_rng(14)
    hkv, dim = 2, 64
    k, v, ks, vs = _pool_e4m3(rng, 4, hkv, dim)
    k2, v2, ks2, vs2, st = OR.reconstruct_e4m3(k, v, ks, vs, [0, 1], [2, 3], [0] * (2 * 2 * hkv + 1),
                                               np.zeros(0, np.uint16), np.zeros(0, np.uint16))
    assert st.tolist() == [0, 0]
    # the largest code of a block built with scale = amax / 448 is +-448: amax(deq) / 448 gives the scale back
    assert (k[0] & 0x7F).max() == 0x7E and ks2[2] == ks[0] and vs2[3] == vs[1]
    assert np.array_equal(k2[2], k[0]) and np.array_equal(v2[3], v[1])
    assert np.array_equal(k2[:2], k[:2]) and np.array_equal(ks2[:2], ks[:2])


def test_e4m3_codes_and_scales_match_torch_casts_of_the_same_sums():
    import torch
    rng = np.random.default_rng(15)
    hkv, dim = 2, 128
    k, v, ks, vs = _pool_e4m3(rng, 3, hkv, dim)
    img = 16 * dim
    mask = rng.random((2, hkv, img)) < 0.3
    vals = _torch_bf16_bits((rng.standard_normal((2, hkv, img)) * 0.5).astype(np.float32))
    ptr, idx, val = [0], [], []
    for t in (0, 1):
        for h in range(hkv):
            ii = np.nonzero(mask[t, h])[0]
            idx.extend(ii.tolist())
            val.extend(vals[t, h][ii].tolist())
            ptr.append(len(idx))
    k2, v2, ks2, vs2, st = OR.reconstruct_e4m3(k, v, ks, vs, [1], [2], ptr, np.array(idx, np.uint16), np.array(val, np.uint16))
    assert st.tolist() == [0]
    delta = np.where(mask, OR.bf16_bits_to_f32(vals), np.float32(0)).reshape(2, hkv, 16, dim)        # logical [slot][d]
    base_k = torch.from_numpy(k[1].copy()).view(torch.float8_e4m3fn).float() * float(ks[1])             # torch's own decode
    base_v = torch.from_numpy(v[1].copy()).view(torch.float8_e4m3fn).float() * float(vs[1])
    sum_k = base_k + torch.from_numpy(delta[0])
    sum_v = base_v + torch.from_numpy(np.ascontiguousarray(np.transpose(delta[1], (0, 2, 1))))
    for x, codes, scale in ((sum_k, k2[2], ks2[2]), (sum_v, v2[2], vs2[2])):
        s = x.abs().max() / 448.0
        assert np.float32(scale) == np.float32(s.item())
        want = (x / s).clamp(-448, 448).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        assert np.array_equal(codes, want)
        deq = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).float().numpy().astype(np.float64) * float(scale)
        half = np.maximum(np.abs(x.numpy()) * 2.0 ** -4, 2.0 ** -10 * float(scale))
        assert (np.abs(deq - x.numpy().astype(np.float64)) <= half * 1.0001).all()


def test_e4m3_bad_block_and_bad_index_are_reported():
    rng = np.random.default_rng(16)
    hkv, dim = 1, 64
    k, v, ks, vs = _pool_e4m3(rng, 3, hkv, dim)
    idx = np.array([5, 16 * dim, 7], np.uint16)
    val = np.array([0x3F80, 0x3F80, 0x3F80], np.uint16)
    k2, v2, ks2, vs2, st = OR.reconstruct_e4m3(k, v, ks, vs, [0, 9, 1], [1, 2, -1], [0, 3, 3, 3, 3, 3, 3], idx, val)
    assert st.tolist() == [OR.ST_BAD_INDEX, OR.ST_BAD_BLOCK, OR.ST_BAD_BLOCK]
    assert np.array_equal(k2[2], k[2]) and ks2[2] == ks[2]
    assert not np.array_equal(k2[1], k[1])


def test_residual_handles_name_the_item_of_every_instance_block_and_nothing_else():
    """Host logic of the read-time form: per table entry, the residual item whose source is the entry's base block
    and whose destination is the instance block that the two-step form would read there."""
    from paper_2605_22566_amd import workload as W
    from tests.helpers import oracle_resolve
    wl = W.small_layered(71, W.Shape(8, 2, 64), num_nodes=24, num_layers=5, len_lo=3, len_hi=90, num_req=6, hops=(1, 5),
                         new_lo=1, new_hi=40)
    wl2, res = W.add_residual_instances(wl, last_nodes=2)
    bt = np.asarray(oracle_resolve(wl)["block_table"], np.int32)
    it = np.asarray(oracle_resolve(wl2)["block_table"], np.int32)
    h = W.residual_handles(bt, it, res)
    assert h.shape == bt.shape and h.dtype == np.int32
    named = h >= 0
    assert named.sum() == res.num_items and sorted(h[named].tolist()) == list(range(res.num_items))
    assert (res.src_blocks[h[named]] == bt[named]).all() and (res.dst_blocks[h[named]] == it[named]).all()
    assert (bt[~named] == it[~named]).all() and (h[~named] == -1).all()
    # every request's handles sit on the entries of its last two nodes: a suffix of its context entries
    for r in range(wl.batch.num_req):
        cols = np.nonzero(named[r])[0]
        assert cols.size > 0 and (np.diff(cols) == 1).all()


def test_make_residual_round_trip_hand_image_and_layouts():
    """make_residual: (1) share 1 with exactly representable differences reproduces the prefix-conditioned blocks
    bit for bit through reconstruct(); (2) an image whose energy sits in three hand-placed entries keeps exactly
    those at 95 %; (3) a K difference at (slot, d) and a V difference at (d, slot) get the logical index slot*D+d."""
    from oracle import residual as OR
    rng = np.random.default_rng(17)
    hkv, dim = 2, 64
    f32 = lambda bits: OR.bf16_bits_to_f32(bits)
    base_k = OR.f32_to_bf16_bits_rne(rng.integers(-8, 9, size=(4, hkv, 16, dim)).astype(np.float32))
    base_v = OR.f32_to_bf16_bits_rne(rng.integers(-8, 9, size=(4, hkv, dim, 16)).astype(np.float32))
    k, v = base_k.copy(), base_v.copy()
    # blocks 2, 3 = blocks 0, 1 plus small-integer differences on a third of the elements (all sums exact in bf16)
    for pool in (k, v):
        d = rng.integers(-3, 4, size=pool[:2].shape).astype(np.float32) * (rng.random(pool[:2].shape) < 0.33)
        pool[2:4] = OR.f32_to_bf16_bits_rne(f32(pool[:2]) + d)
    ptr, idx, val = OR.make_residual(k, v, [0, 1], [2, 3], share=1.0)
    assert ptr[0] == 0 and ptr[-1] == idx.size == val.size and np.all(np.diff(ptr) >= 0)
    scratch_k, scratch_v = k.copy(), v.copy()
    scratch_k[2:4] = 0
    scratch_v[2:4] = 0
    k2, v2, st = OR.reconstruct(scratch_k, scratch_v, [0, 1], [2, 3], ptr, idx, val)
    assert (st == 0).all() and np.array_equal(k2[2:4], k[2:4]) and np.array_equal(v2[2:4], v[2:4])
    # nothing kept where nothing differs; every kept entry is a non-zero difference
    assert np.all(f32(val) != 0)
    # (2) + (3): one block pair, differences by hand
    k3, v3 = base_k[:2].copy(), base_v[:2].copy()
    k3[1], v3[1] = k3[0], v3[0]
    kf, vf = f32(k3), f32(v3)
    kf[1, 1, 5, 9] += 16.0          # K head 1, slot 5, d 9
    kf[1, 1, 0, 63] -= 16.0
    kf[1, 1, 15, 0] += 8.0
    kf[1, 1, 7, 7] += 0.5           # 0.25 of 576.25: below the 5 % that may be dropped
    vf[1, 0, 20, 3] += 4.0          # V head 0, d 20, slot 3 -> logical 3 * 64 + 20
    k3, v3 = OR.f32_to_bf16_bits_rne(kf), OR.f32_to_bf16_bits_rne(vf)
    ptr, idx, val = OR.make_residual(k3, v3, [0], [1], share=0.95)
    rows = {r: (idx[ptr[r]:ptr[r + 1]].tolist(), f32(val[ptr[r]:ptr[r + 1]]).tolist()) for r in range(2 * hkv)}
    assert rows[0] == ([], []) and rows[3] == ([], [])
    assert rows[1] == ([63, 5 * 64 + 9, 15 * 64], [-16.0, 16.0, 8.0])         # K head 1, by index; 0.5 dropped
    assert rows[2] == ([3 * 64 + 20], [4.0])                                  # V head 0


def test_packed_form_hand_image_round_trip_and_equivalence_to_the_csr():
    dim = 64
    # one image written out by hand: elements 0, 33, 64 (slot 1, d 0) and 1023 (slot 15, d 63), listed unsorted
    ptr = np.array([0, 4], np.int32)
    idx = np.array([1023, 0, 64, 33], np.uint16)
    val = np.array([0x4080, 0x3F80, 0x4040, 0x4000], np.uint16)         # 4.0, 1.0, 3.0, 2.0
    mask, pv = OR.pack_rows(ptr, idx, val, dim)
    assert mask.shape == (1, 16 * dim // 32) and mask.dtype == np.uint32
    want = np.zeros(32, np.uint32)
    want[0] = 1            # element 0: word 0, bit 0
    want[1] = 1 << 1       # element 33: word 1, bit 1
    want[2] = 1            # element 64: word 2, bit 0
    want[31] = 1 << 31     # element 1023: word 31, bit 31
    assert (mask[0] == want).all()
    assert pv.tolist() == [0x3F80, 0x4000, 0x4040, 0x4080]              # values follow the elements: 1, 2, 3, 4
    assert OR.unpack_rows(ptr, mask, dim).tolist() == [0, 33, 64, 1023]
    # random rows at both head dims: round trip, bit counts, and the reconstruction equals the CSR's
    rng = np.random.default_rng(14)
    for hkv, dim in ((2, 64), (1, 128)):
        k, v = _pool(rng, 6, hkv, dim)
        rows = 3 * 2 * hkv
        parts, p = [], [0]
        for r in range(rows):
            n = int(rng.integers(0, 16 * dim // 3)) if r % 5 else 0     # some rows empty
            parts.append(rng.permutation(16 * dim)[:n].astype(np.uint16))
            p.append(p[-1] + n)
        idx = np.concatenate(parts)
        val = OR.f32_to_bf16_bits_rne(rng.standard_normal(idx.size).astype(np.float32))
        p = np.asarray(p, np.int32)
        mask, pv = OR.pack_rows(p, idx, val, dim)
        bits = np.array([sum(bin(int(w)).count("1") for w in mask[r]) for r in range(rows)])
        assert (bits == np.diff(p)).all()
        got_idx = OR.unpack_rows(p, mask, dim)
        for r in range(rows):
            seg = slice(int(p[r]), int(p[r + 1]))
            order = np.argsort(idx[seg].astype(np.int64))
            assert (got_idx[seg] == idx[seg][order]).all() and (pv[seg] == val[seg][order]).all()
        src, dst = [0, 2, 1], [3, 4, 5]
        k1, v1, s1 = OR.reconstruct(k, v, src, dst, p, idx, val)
        k2, v2, s2 = OR.reconstruct_packed(k, v, src, dst, p, mask, pv)
        assert (k1 == k2).all() and (v1 == v2).all() and s1.tolist() == s2.tolist() == [0, 0, 0]


def test_packed_single_entries_land_on_the_hand_indexed_physical_element_and_bad_rows_are_reported():
    rng = np.random.default_rng(15)
    hkv, dim = 4, 64
    k, v = _pool(rng, 2, hkv, dim)
    two = np.array([0x4000], np.uint16)
    for (t, h, slot, d) in [(0, 0, 0, 0), (0, 3, 15, 63), (1, 0, 0, 0), (1, 2, 9, 33), (1, 3, 15, 63)]:
        row = t * hkv + h
        ptr = [0] * (row + 1) + [1] * (2 * hkv - row)
        mask = np.zeros((2 * hkv, 16 * dim // 32), np.uint32)
        i = slot * dim + d
        mask[row, i // 32] = 1 << (i % 32)
        k2, v2, st = OR.reconstruct_packed(k, v, [0], [1], ptr, mask, two)
        assert st.tolist() == [0]
        dk, dv = k2[1] != k[0], v2[1] != v[0]
        if t == 0:
            assert dk.sum() == 1 and dk[h, slot, d] and not dv.any()
        else:
            assert dv.sum() == 1 and dv[h, d, slot] and not dk.any()
    # a row with more bits than values, a row with fewer, a block outside the pool
    ptr = np.zeros(2 * hkv + 1, np.int32)
    ptr[1:] = 1
    mask = np.zeros((2 * hkv, 16 * dim // 32), np.uint32)
    mask[0, 0] = 0b11
    _, _, st = OR.reconstruct_packed(k, v, [0], [1], ptr, mask, two)
    assert st.tolist() == [OR.ST_BAD_INDEX]
    mask[0, 0] = 0
    _, _, st = OR.reconstruct_packed(k, v, [0], [1], ptr, mask, two)
    assert st.tolist() == [OR.ST_BAD_INDEX]
    _, _, st = OR.reconstruct_packed(k, v, [0], [7], ptr, mask, two)
    assert st.tolist() == [OR.ST_BAD_BLOCK]
