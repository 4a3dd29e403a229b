"""Host-side footprint accounting (paper_2605_22566_amd/footprint.py) against explicit enumeration on a
hand-built graph, and the orderings that hold on any batch."""
import numpy as np

from paper_2605_22566_amd import footprint as F
from paper_2605_22566_amd import workload as W


def _hand():
    sh = W.Shape(4, 2, 64)
    node_len = np.array([16, 40, 5, 33])                       # 1, 3, 1, 3 blocks
    paths = [[0, 1], [0, 1], [0, 2], [0, 1, 3], [2]]
    edges = [(0, 1), (0, 2), (1, 3)]
    rng = np.random.default_rng(0)
    return W._finish("hand", sh, node_len, edges, paths, np.array([1, 17, 16, 3, 40]), rng, False, 0,
                     np.arange(len(paths)), np.zeros(0), 0.0)


def test_hand_built_graph_against_explicit_enumeration():
    wl = _hand()
    f = F.footprint(wl, density_k=0.25, density_v=0.5, min_count=2)
    blk = 2 * 2 * 16 * 64 * 2                                  # K + V, 2 kv heads, bf16
    tails = (1 + 2 + 1 + 1 + 3) * blk
    # distinct (prefix, node) pairs: (0) (0,1) (0,2) (0,1,3) (2) -> blocks 1 + 3 + 1 + 3 + 1
    assert f["prefix_node_pairs"] == 5 and f["nodes"] == 4
    assert f["stateful_bytes"] == 9 * blk + tails
    assert f["stateless_bytes"] == (1 + 3 + 1 + 3) * blk + tails
    # packed form per block: 2 B per kept value, one bit per element of the 4 images, 4 row pointers, 2 block ids
    res_blk = 2 * 16 * 64 * (0.25 + 0.5) * 2 + 4 * 16 * 64 / 8 + 2 * 2 * 4 + 8
    # residuals for (0,1) (0,2) (0,1,3): 3 + 1 + 3 blocks
    assert np.isclose(f["differential_bytes"], 8 * blk + 7 * res_blk + tails)
    # the form the attention kernels read: 2 B index + 2 B value per kept element
    fc = F.footprint(wl, density_k=0.25, density_v=0.5, min_count=2, residual_form="coordinate")
    res_coo = 2 * 16 * 64 * (0.25 + 0.5) * 4 + 2 * 2 * 4 + 8
    assert np.isclose(fc["differential_bytes"], 8 * blk + 7 * res_coo + tails)
    assert fc["stateful_bytes"] == f["stateful_bytes"] and fc["stateless_bytes"] == f["stateless_bytes"]
    # transitions: 0->1 three times, 0->2 once, 1->3 once: only (0,1) survives min_count = 2
    assert F.transition_counts(wl.batch) == {(0, 1): 3, (0, 2): 1, (1, 3): 1}
    assert f["pairs_kept_by_pruning"] == 1 and f["fallback_pairs"] == 2
    assert np.isclose(f["pruned_bytes"], 8 * blk + 3 * res_blk + tails)
    sub = F.footprint(wl, [2, 4])                              # requests (0,2) and (2): node 2 once, node 0 once
    assert sub["nodes"] == 2 and sub["prefix_node_pairs"] == 3
    assert sub["stateless_bytes"] == 2 * blk + (1 + 3) * blk


def test_orderings_and_growth_on_a_benchmark_workload():
    wl = W.config_prefill_8b()
    rows = F.footprint_by_batch_size(wl)
    assert [r["requests"] for r in rows] == [10, 20, 30, 40, 50]
    for r in rows:
        assert r["stateless_bytes"] <= r["pruned_bytes"] <= r["differential_bytes"]
    # a packed residual at 25-30 % density costs 0.34 of a dense bf16 copy: the differential design holds less
    # than private copies at every batch size (the shape of the paper's memory-against-concurrency figure); in the
    # coordinate form (0.55) it only does once prefixes are shared enough
    assert all(r["differential_bytes"] < r["stateful_bytes"] for r in rows)
    assert all(r["pruned_bytes"] < r["stateful_bytes"] for r in rows)
    coo = F.footprint_by_batch_size(wl, residual_form="coordinate")
    assert all(c["differential_bytes"] > r["differential_bytes"] for c, r in zip(coo, rows))
    assert all(c["differential_bytes"] < c["stateful_bytes"] for c in coo[2:])
    for key in ("stateful_bytes", "stateless_bytes", "differential_bytes", "pruned_bytes"):
        vals = [r[key] for r in rows]
        assert all(a <= b for a, b in zip(vals, vals[1:]))     # more requests never hold less
    # the shared designs grow more slowly with concurrency than the private copies
    grow = lambda key: rows[-1][key] - rows[0][key]
    assert grow("stateless_bytes") < grow("differential_bytes") < grow("stateful_bytes")
    # pruning with an unreachable threshold keeps nothing; with threshold 1 it keeps everything
    none = F.footprint(wl, min_count=10 ** 9)
    allp = F.footprint(wl, min_count=1)
    assert none["pruned_bytes"] == none["stateless_bytes"] and allp["pruned_bytes"] == allp["differential_bytes"]
