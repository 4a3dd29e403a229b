"""State-management policy on the device (gf_residual_dir_*, gf_resolve_path_residual) against
oracle/policy.py: residual handles per table entry, fallback counts, transition statistics, pair uses and
pruning are exact integers and must be equal; and the end-to-end property of the paper's pruning: a pruned
pair whose KV is computed on the fly gives the same attention result as the stored residual did."""
import json
import os

import numpy as np
import pytest
import torch

from oracle import attention as OA
from oracle import policy as OP
from oracle import residual as OR
from paper_2605_22566_amd import binding as B
from paper_2605_22566_amd import runner as R
from paper_2605_22566_amd import workload as W
from tests.gpu_common import assert_close, assert_tables_equal
from tests.helpers import GOLDEN, load_example_dag, max_blocks_of, oracle_resolve

pytestmark = pytest.mark.gpu


def _session(wl, capacity):
    sess = R.Session(wl)
    return sess, R.ResidualDirectory(sess, capacity), sess.upload_batch(wl.batch)


def _dir_host(d):
    return {k: getattr(d, k).cpu().numpy() for k in ("key", "prev", "node", "first_item", "uses")}


def _example_workload():
    fx, a = load_example_dag()
    g = W.WGraph(a["num_nodes"], a["node_len"], a["node_block_ptr"], a["node_blocks"], a["edge_ptr"], a["edge_dst"])
    b = W.Batch(a["path_ptr"], a["path_nodes"], a["new_lens"], a["tail_ptr"], a["tail_blocks"])
    wl = W.Workload("example", W.Shape(4, 4, 64), g, b, a["num_pool_blocks"], 0, np.arange(b.num_req), np.zeros(0))
    return fx, a, wl


def test_example_dag_matches_the_hand_computed_values():
    fx, a, wl = _example_workload()
    with open(os.path.join(GOLDEN, "example_residual_policy.json")) as f:
        pol = json.load(f)
    ids = {n: i for i, n in enumerate(fx["nodes"])}
    prefixes = [[ids[v] for v in d["prefix"]] for d in pol["directory"]]
    sess, d, db = _session(wl, 16)
    st = d.insert(prefixes, [p["first_item"] for p in pol["directory"]])
    assert st.cpu().tolist() == [B.GF_DIR_OK] * len(prefixes)
    tables = sess.alloc_tables(wl.batch.num_req, a["max_blocks"])
    handle, fallback = d.resolve(db, tables)
    torch.cuda.synchronize()
    want_tables = oracle_resolve(wl, max_blocks=a["max_blocks"])
    assert_tables_equal(tables, want_tables)                       # the table outputs are gf_resolve_path's
    for r in range(wl.batch.num_req):
        assert handle[r].cpu().tolist() == pol["handles"].get(str(r), [-1] * a["max_blocks"]), r
    assert fallback.cpu().tolist() == pol["num_fallback"]
    assert d.trans_count.cpu().tolist() == pol["transition_counts"]
    d.prune(pol["min_count"])
    handle2, fallback2 = d.resolve(db, tables, count=False)
    torch.cuda.synchronize()
    assert d.pruned.cpu().tolist() == [len(pol["pruned"]), pol["items_freed"]]
    for r in range(wl.batch.num_req):
        assert handle2[r].cpu().tolist() == pol["handles_after_prune"].get(str(r), [-1] * a["max_blocks"]), r
    assert fallback2.cpu().tolist() == pol["num_fallback_after_prune"]
    # a pruned slot keeps the items it named: -2 - first_item
    h = _dir_host(d)
    freed = sorted(-2 - int(x) for x, k in zip(h["first_item"], h["key"]) if k != 0 and x < -1)
    assert freed == [0, 5, 6]


def _all_pairs(wl, rng, drop=0.0):
    b, g = wl.batch, wl.graph
    directory, nxt = {}, 0
    for r in range(b.num_req):
        p = [int(v) for v in b.path_nodes[b.path_ptr[r]:b.path_ptr[r + 1]]]
        for i in range(1, len(p)):
            key = tuple(p[:i + 1])
            if key not in directory:
                directory[key] = nxt
                nxt += -(-int(g.node_len[p[i]]) // 16)
    if drop > 0:
        directory = {k: v for k, v in directory.items() if rng.random() >= drop}
    return directory


def _check_against_oracle(wl, drop, min_counts, mutate=None):
    rng = np.random.default_rng(wl.seed + 5)
    if mutate:
        mutate(wl)
    b, g = wl.batch, wl.graph
    directory = _all_pairs(wl, rng, drop)
    cap = 1
    while cap < 2 * max(len(directory), 1):
        cap *= 2
    sess, d, db = _session(wl, cap)
    keys = list(directory)
    if keys:
        st = d.insert([list(k) for k in keys], [directory[k] for k in keys])
        assert bool((st == B.GF_DIR_OK).all().item())
    mb = max_blocks_of(wl)
    tables = sess.alloc_tables(b.num_req, mb)
    handle, fallback = d.resolve(db, tables)
    torch.cuda.synchronize()
    want_tables = oracle_resolve(wl)
    assert_tables_equal(tables, want_tables)
    wh, wf = OP.residual_handles(want_tables["status"], g.node_len, b.path_ptr, b.path_nodes, directory, mb)
    assert np.array_equal(handle.cpu().numpy(), np.array(wh, dtype=np.int32))
    assert fallback.cpu().tolist() == wf
    counts = OP.transition_counts(want_tables["status"], g.edge_ptr, g.edge_dst, b.path_ptr, b.path_nodes)
    assert d.trans_count.cpu().tolist()[:len(counts)] == counts
    uses = OP.pair_uses(want_tables["status"], b.path_ptr, b.path_nodes, keys)
    h = _dir_host(d)
    slot_of = {int(k): i for i, k in enumerate(h["key"]) if k != 0}
    for k in keys:
        s = slot_of[np.uint64(B.gf_prefix_key(list(k))).astype(np.int64).item()]
        assert (h["prev"][s], h["node"][s], h["first_item"][s], h["uses"][s]) == (k[-2], k[-1], directory[k], uses[k]), k
    kept = dict(directory)
    total_pruned, total_freed = 0, 0
    for m in min_counts:
        kept, pruned, freed = OP.prune(kept, g.node_len, g.edge_ptr, g.edge_dst, counts, m)
        total_pruned, total_freed = total_pruned + len(pruned), total_freed + freed
        d.prune(m)
        handle, fallback = d.resolve(db, tables, count=False)
        torch.cuda.synchronize()
        assert d.pruned.cpu().tolist() == [total_pruned, total_freed]
        wh, wf = OP.residual_handles(want_tables["status"], g.node_len, b.path_ptr, b.path_nodes, kept, mb)
        assert np.array_equal(handle.cpu().numpy(), np.array(wh, dtype=np.int32)), m
        assert fallback.cpu().tolist() == wf, m
    return sess


@pytest.mark.parametrize("seed", [3, 4])
def test_small_layered_graphs_with_missing_pairs_and_failed_requests(seed):
    def mutate(wl):                       # one request walks its path backwards: BAD_EDGE, counts nothing
        b = wl.batch
        p0, p1 = int(b.path_ptr[2]), int(b.path_ptr[3])
        if p1 - p0 >= 2:
            b.path_nodes[p0:p1] = b.path_nodes[p0:p1][::-1].copy()
    wl = W.small_layered(seed, W.Shape(8, 2, 64), num_nodes=30, num_layers=6, len_lo=3, len_hi=90, num_req=40,
                         hops=(1, 6), new_lo=1, new_hi=40)
    _check_against_oracle(wl, drop=0.3, min_counts=(2, 3, 6), mutate=mutate)


@pytest.mark.parametrize("name", ["tiny", "prefill_8b", "decode_8b", "decode_70b", "mixed_fp8"])
def test_all_benchmark_configs(name):
    _check_against_oracle(W.CONFIGS[name](), drop=0.1, min_counts=(2, 4))


def test_long_path_spans_several_chunks_of_the_walk():
    """A 700-node chain (the key chain is carried across chunks of 256 path positions)."""
    n = 700
    rng = np.random.default_rng(5)
    node_len = rng.integers(1, 40, size=n)
    edges = [(i, i + 1) for i in range(n - 1)]
    wl = W._finish("chain", W.Shape(4, 4, 64), node_len, edges, [list(range(n)), list(range(300))], np.array([3, 1]),
                   rng, True, 5, np.arange(2), np.zeros(0), 0.0)
    _check_against_oracle(wl, drop=0.2, min_counts=(2,))


def test_insert_reports_full_table_and_bad_pairs_and_empty_directory_is_fine():
    fx, a, wl = _example_workload()
    sess, d, db = _session(wl, 2)
    st = d.insert([[0, 1], [0, 2], [0, 1, 3]], [0, 5, 8])
    torch.cuda.synchronize()
    assert sorted(st.cpu().tolist()) == [B.GF_DIR_OK, B.GF_DIR_OK, B.GF_DIR_FULL]
    dev = sess.device
    z = torch.zeros(1, dtype=torch.int64, device=dev)
    i32 = lambda v: torch.tensor([v], dtype=torch.int32, device=dev)
    st = torch.full((1,), -77, dtype=torch.int32, device=dev)
    B.gf_residual_dir_insert(sess.ctx, d.struct(), 1, z, i32(0), i32(1), i32(3), st)        # key 0
    assert st.cpu().tolist() == [B.GF_DIR_BAD_PAIR]
    with pytest.raises(B.GraphFlowError) as e:
        B.gf_residual_dir_clear(sess.ctx, B.make_residual_dir(d.key, d.prev, d.node, d.first_item, d.uses, 3))
    assert e.value.code == B.GF_ERR_BAD_SHAPE                                                  # not a power of two
    empty = R.ResidualDirectory(sess, 0)
    tables = sess.alloc_tables(wl.batch.num_req, a["max_blocks"])
    handle, fallback = empty.resolve(db, tables)
    torch.cuda.synchronize()
    assert bool((handle == -1).all().item())
    assert fallback.cpu().tolist() == [3, 3, 0, 0, 0, 0, 0, 0]       # every node beyond the first lacks a residual


def test_host_key_is_a_function_of_the_whole_path():
    ks = {B.gf_prefix_key(p) for p in ([0, 1], [1, 0], [0, 1, 2], [0, 2, 1], [0], [1], [0, 0], [5, 6, 7, 8])}
    assert len(ks) == 8 and 0 not in ks
    assert B.gf_prefix_key([3, 4]) == B.gf_prefix_key([3, 4])


def test_pruned_pair_computed_on_the_fly_equals_the_stored_residual():
    """Effective Path Pruning end to end.  Every request's last node carries a prefix-specific residual.
    (1) All residuals stored: resolve with handles, decode with the residuals applied at read time.
    (2) The statistics of that batch prune the pairs whose transition was taken once; their KV under the
        prefix is then produced on the fly (here: the exact prefix-conditioned values, which the test takes
        from the reconstruction oracle, written by gf_kv_append into blocks of an instance node) while the
        surviving pairs keep reading base + residual.  Both runs must give the same output, bit for bit."""
    sh = W.Shape(8, 2, 128)
    wl = W.small_layered(21, sh, num_nodes=24, num_layers=5, len_lo=10, len_hi=70, num_req=12, hops=(2, 5),
                         new_lo=1, new_hi=20)
    wl2, res = W.add_residual_instances(wl, last_nodes=1)
    b, g = wl.batch, wl.graph
    t = W.make_tensors(wl)
    nb_extra = wl2.num_pool_blocks - wl.num_pool_blocks
    pad = lambda x: np.concatenate([x, np.zeros((nb_extra,) + x.shape[1:], x.dtype)])
    k_pool, v_pool = pad(t.k_pool), pad(t.v_pool)
    # one residual per distinct pair: the items of the first request that walks it
    nbl = (g.node_len.astype(np.int64) + 15) // 16
    directory, first_of_req, item = {}, [], 0
    for r in range(b.num_req):
        p = tuple(int(v) for v in b.path_nodes[b.path_ptr[r]:b.path_ptr[r + 1]])
        first_of_req.append(item)
        if len(p) >= 2:
            directory.setdefault(p, item)
        item += int(nbl[p[-1]])
    assert item == res.num_items
    sess = R.Session(wl2)                                  # graph with the instance nodes; base nodes unchanged
    dev = sess.device
    d = R.ResidualDirectory(sess, 64)
    keys = list(directory)
    assert bool((d.insert([list(k) for k in keys], [directory[k] for k in keys]) == 0).all().item())
    pool = R.DevicePool(R.bits_to_device(k_pool, dev), R.bits_to_device(v_pool, dev), wl2.num_pool_blocks)
    dres = sess.upload_residuals(res)
    mb = max_blocks_of(wl)
    last = (t.q_ptr[1:] - 1).astype(np.int64)
    qd = R.bits_to_device(np.ascontiguousarray(t.q[last]), dev)

    def run(batch):
        db = sess.upload_batch(batch)
        tables = sess.alloc_tables(batch.num_req, mb)
        handle, fallback = d.resolve(db, tables)
        o = torch.full(qd.shape, float("nan"), dtype=torch.bfloat16, device=dev)
        sess.decode_residual(pool, tables, handle, dres, qd, o)
        torch.cuda.synchronize()
        assert tables["status"].cpu().tolist() == [0] * batch.num_req
        return o, handle.cpu().numpy(), fallback.cpu().numpy()

    o_stored, h1, f1 = run(b)
    # the pairs stored are whole request paths: a node further up a path has a residual only where another
    # request's path ends there
    wh, wf = OP.residual_handles([0] * b.num_req, g.node_len, b.path_ptr, b.path_nodes, directory, mb)
    assert np.array_equal(h1, np.array(wh, dtype=np.int32)) and f1.tolist() == wf and (h1 >= 0).any()
    # oracle: every request attends over base + its pair's residual
    want = oracle_resolve(wl)
    for r in range(b.num_req):
        n = want["num_blocks"][r]
        ids = np.array(want["block_table"][r][:n], dtype=np.int64)
        kk, vv = k_pool[ids].copy(), v_pool[ids].copy()
        ents = np.nonzero(h1[r, :n] >= 0)[0]
        if ents.size:
            rows = 2 * sh.num_kv_heads
            lptr, lidx, lval = [0], [], []
            for e in ents:
                it = int(h1[r, e])
                lo, hi = int(res.res_ptr[it * rows]), int(res.res_ptr[(it + 1) * rows])
                lptr += list(res.res_ptr[it * rows + 1:(it + 1) * rows + 1] - lo + lptr[-1])
                lidx.append(res.res_idx[lo:hi])
                lval.append(res.res_val[lo:hi])
            kk, vv, st = OR.reconstruct(kk, vv, ents, ents, np.array(lptr), np.concatenate(lidx), np.concatenate(lval))
            assert (st == 0).all()
        local = {k: [v[r]] for k, v in want.items()}
        local["block_table"] = [list(range(n))]
        O, _ = OA.decode(np.ascontiguousarray(t.q[last[r]:last[r] + 1]), kk, vv, local)
        assert_close(o_stored[r:r + 1].double().cpu().numpy(), O, sh.kv_dtype, f"stored residuals, request {r}")

    d.prune(2)
    torch.cuda.synchronize()
    hd = _dir_host(d)
    pruned_keys = {int(k) for k, f in zip(hd["key"], hd["first_item"]) if k != 0 and f < -1}
    assert 0 < len(pruned_keys) < len(keys)
    # on-the-fly fallback for the pruned pairs: exact KV of the node under the prefix -> blocks of its instance node
    b2 = wl2.batch
    path_nodes = b.path_nodes.copy()
    tok_k, tok_v, fake_paths, fake_tails, fake_new = [], [], [], [], []
    for r in range(b.num_req):
        p = tuple(int(v) for v in b.path_nodes[b.path_ptr[r]:b.path_ptr[r + 1]])
        if len(p) < 2 or np.uint64(B.gf_prefix_key(list(p))).astype(np.int64).item() not in pruned_keys:
            continue
        pos = int(b.path_ptr[r + 1]) - 1
        inst = int(b2.path_nodes[pos])
        path_nodes[pos] = inst
        it0 = directory[p]                                         # the pair's own residual (first walker's items)
        nb = int(nbl[p[-1]])
        src = res.src_blocks[it0:it0 + nb]
        dst = wl2.graph.node_blocks[wl2.graph.node_block_ptr[inst]:wl2.graph.node_block_ptr[inst + 1]]
        rows = 2 * sh.num_kv_heads
        lo, hi = int(res.res_ptr[it0 * rows]), int(res.res_ptr[(it0 + nb) * rows])
        k2, v2, st = OR.reconstruct(k_pool, v_pool, src, dst, res.res_ptr[it0 * rows:(it0 + nb) * rows + 1] - lo,
                                    res.res_idx[lo:hi], res.res_val[lo:hi])
        assert (st == 0).all()
        n_tok = int(g.node_len[p[-1]])
        tok_k.append(np.transpose(k2[dst], (0, 2, 1, 3)).reshape(nb * 16, sh.num_kv_heads, sh.head_dim)[:n_tok])
        tok_v.append(np.transpose(v2[dst], (0, 3, 1, 2)).reshape(nb * 16, sh.num_kv_heads, sh.head_dim)[:n_tok])
        fake_paths.append([])
        fake_tails.append(list(dst))
        fake_new.append(n_tok)
    assert fake_new
    # the write path: one "request" per recomputed node, empty path, its tokens go to the instance's blocks
    i32 = lambda x: np.asarray(x, dtype=np.int32)
    wb = W.Batch(i32(np.zeros(len(fake_new) + 1)), i32([]), i32(fake_new),
                 i32(np.concatenate([[0], np.cumsum([len(x) for x in fake_tails])])), i32(np.concatenate(fake_tails)))
    wdb = sess.upload_batch(wb)
    wmb = max(len(x) for x in fake_tails)
    wt = sess.resolve(wdb, sess.alloc_tables(wb.num_req, wmb))
    kn = R.bits_to_device(np.ascontiguousarray(np.concatenate(tok_k)), dev)
    vn = R.bits_to_device(np.ascontiguousarray(np.concatenate(tok_v)), dev)
    qp = torch.from_numpy(np.concatenate([[0], np.cumsum(fake_new)]).astype(np.int32)).to(dev)
    sess.append(pool, wt, kn, vn, qp, int(sum(fake_new)), int(max(fake_new)))
    torch.cuda.synchronize()
    assert wt["status"].cpu().tolist() == [0] * wb.num_req
    mixed = W.Batch(b.path_ptr.copy(), path_nodes, b.new_lens.copy(), b.tail_ptr.copy(), b.tail_blocks.copy())
    o_mixed, h2, f2 = run(mixed)
    assert f2.sum() == f1.sum() + len(fake_new) and (h2 >= 0).any() and (h2 >= 0).sum() < (h1 >= 0).sum()
    assert torch.equal(o_stored, o_mixed)
