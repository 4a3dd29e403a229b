"""Pins of oracle/policy.py: hand-computed values on the paper's example workflow DAG, counting invariants,
and an entry-by-entry reformulation of the handle table."""
import json
import os

import numpy as np

from oracle import policy as OP
from oracle import resolve as ORS
from paper_2605_22566_amd import workload as W
from tests.helpers import GOLDEN, load_example_dag, max_blocks_of, oracle_resolve


def _example():
    fx, a = load_example_dag()
    with open(os.path.join(GOLDEN, "example_residual_policy.json")) as f:
        pol = json.load(f)
    ids = {n: i for i, n in enumerate(fx["nodes"])}
    directory = {tuple(ids[v] for v in d["prefix"]): d["first_item"] for d in pol["directory"]}
    tables = ORS.resolve_paths(a["num_nodes"], a["node_len"], a["node_block_ptr"], a["node_blocks"], a["edge_ptr"],
                               a["edge_dst"], a["path_ptr"], a["path_nodes"], a["new_lens"], a["tail_ptr"],
                               a["tail_blocks"], a["max_blocks"], a["num_pool_blocks"])
    return fx, a, pol, ids, directory, tables


def test_example_dag_handles_statistics_and_pruning_match_the_hand_computed_values():
    fx, a, pol, ids, directory, tables = _example()
    handles, fallback = OP.residual_handles(tables["status"], a["node_len"], a["path_ptr"], a["path_nodes"], directory,
                                            a["max_blocks"])
    for r in range(len(fx["requests"])):
        want = pol["handles"].get(str(r), [-1] * a["max_blocks"])
        assert handles[r] == want, r
    assert fallback == pol["num_fallback"]
    counts = OP.transition_counts(tables["status"], a["edge_ptr"], a["edge_dst"], a["path_ptr"], a["path_nodes"])
    assert counts == pol["transition_counts"]
    # every stored pair lies on exactly one of the two resolved walks; (OP_01, OP_03, OP_04) is walked but not stored
    uses = OP.pair_uses(tables["status"], a["path_ptr"], a["path_nodes"], list(directory) + [(0, 2, 3), (0, 1, 2)])
    assert [uses[k] for k in directory] == [1, 1, 1, 1, 1] and uses[(0, 2, 3)] == 1 and uses[(0, 1, 2)] == 0
    kept, pruned, freed = OP.prune(directory, a["node_len"], a["edge_ptr"], a["edge_dst"], counts, pol["min_count"])
    assert pruned == sorted(tuple(ids[v] for v in p) for p in pol["pruned"])
    assert freed == pol["items_freed"]
    handles2, fallback2 = OP.residual_handles(tables["status"], a["node_len"], a["path_ptr"], a["path_nodes"], kept,
                                              a["max_blocks"])
    for r in range(len(fx["requests"])):
        assert handles2[r] == pol["handles_after_prune"].get(str(r), [-1] * a["max_blocks"]), r
    assert fallback2 == pol["num_fallback_after_prune"]
    # a second batch of the same requests doubles the statistics, after which nothing is pruned at 2
    counts2 = OP.transition_counts(tables["status"], a["edge_ptr"], a["edge_dst"], a["path_ptr"], a["path_nodes"], counts)
    assert counts2 == [2 * c for c in counts]
    assert OP.prune(directory, a["node_len"], a["edge_ptr"], a["edge_dst"], counts2, 2)[1] == []


def _all_pairs(wl, first=0):
    """Every distinct (prefix, node) pair of the batch, numbered in order of first appearance."""
    b, g = wl.batch, wl.graph
    directory, nxt = {}, first
    for r in range(b.num_req):
        p = [int(v) for v in b.path_nodes[b.path_ptr[r]:b.path_ptr[r + 1]]]
        for i in range(1, len(p)):
            key = tuple(p[:i + 1])
            if key not in directory:
                directory[key] = nxt
                nxt += -(-int(g.node_len[p[i]]) // 16)
    return directory, nxt


def test_counting_invariants_and_entrywise_reformulation_on_a_layered_graph():
    wl = W.small_layered(12, W.Shape(8, 2, 64), num_nodes=30, num_layers=6, len_lo=3, len_hi=90, num_req=24,
                         hops=(1, 6), new_lo=1, new_hi=40)
    b, g = wl.batch, wl.graph
    mb = max_blocks_of(wl)
    tables = oracle_resolve(wl)
    assert all(s == 0 for s in tables["status"])
    directory, n_items = _all_pairs(wl)
    handles, fallback = OP.residual_handles(tables["status"], g.node_len, b.path_ptr, b.path_nodes, directory, mb)
    assert fallback == [0] * b.num_req
    # entry by entry: the node that owns table entry e of request r is found from the cumulative block counts;
    # its handle is the pair's first item plus the entry's offset inside the node
    nbl = (g.node_len.astype(np.int64) + 15) // 16
    for r in range(b.num_req):
        p = b.path_nodes[b.path_ptr[r]:b.path_ptr[r + 1]]
        ends = np.cumsum(nbl[p])
        for e in range(mb):
            i = int(np.searchsorted(ends, e, side="right"))
            if i == 0 or i >= len(p):
                want = -1                                   # first node, tail entries and padding
            else:
                want = directory[tuple(int(v) for v in p[:i + 1])] + e - int(ends[i - 1])
            assert handles[r][e] == want, (r, e)
        # every item of every stored pair on the path appears exactly once
        got = sorted(h for h in handles[r] if h >= 0)
        assert len(got) == len(set(got)) == int(nbl[p[1:]].sum())
    counts = OP.transition_counts(tables["status"], g.edge_ptr, g.edge_dst, b.path_ptr, b.path_nodes)
    assert sum(counts) == sum(max(int(b.path_ptr[r + 1] - b.path_ptr[r]) - 1, 0) for r in range(b.num_req))
    # pruning is monotone in the threshold, frees exactly the items of the pairs it drops, and a dropped pair
    # turns into one fallback per request through it
    prev_kept = dict(directory)
    for m in (1, 2, 3, 5, 100):
        kept, pruned, freed = OP.prune(directory, g.node_len, g.edge_ptr, g.edge_dst, counts, m)
        assert set(kept) <= set(prev_kept) and len(kept) + len(pruned) == len(directory)
        assert freed == sum(int(nbl[k[-1]]) for k in pruned)
        _, fb = OP.residual_handles(tables["status"], g.node_len, b.path_ptr, b.path_nodes, kept, mb)
        through = sum(1 for r in range(b.num_req) for i in range(1, int(b.path_ptr[r + 1] - b.path_ptr[r]))
                      if tuple(int(v) for v in b.path_nodes[b.path_ptr[r]:b.path_ptr[r] + i + 1]) not in kept)
        assert sum(fb) == through
        prev_kept = kept
    assert OP.prune(directory, g.node_len, g.edge_ptr, g.edge_dst, counts, 1)[1] == []   # every pair was taken once
    assert OP.prune(directory, g.node_len, g.edge_ptr, g.edge_dst, counts, 10 ** 6)[0] == {}


def test_failed_requests_neither_count_nor_get_handles():
    fx, a, pol, ids, directory, tables = _example()
    handles, fallback = OP.residual_handles(tables["status"], a["node_len"], a["path_ptr"], a["path_nodes"], directory,
                                            a["max_blocks"])
    for r, rq in enumerate(fx["requests"]):
        if rq["status"] != 0:
            assert handles[r] == [-1] * a["max_blocks"] and fallback[r] == 0
    # request 4 (overflow) walks OP_01 -> OP_02 -> OP_04 -> OP_05 but is not counted: OP_01->OP_02 stays at 1
    assert OP.transition_counts(tables["status"], a["edge_ptr"], a["edge_dst"], a["path_ptr"], a["path_nodes"])[0] == 1
