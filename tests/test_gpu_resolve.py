"""gf_resolve_path through the C ABI vs the oracle: bit-exact, pads included."""
import numpy as np
import pytest
import torch

from oracle import resolve as oresolve
from paper_2605_22566_amd import runner as R
from paper_2605_22566_amd import workload as W
from tests.gpu_common import assert_tables_equal, run_resolve
from tests.helpers import load_example_dag, max_blocks_of, oracle_resolve

pytestmark = pytest.mark.gpu


def _example_workload():
    fx, a = load_example_dag()
    g = W.WGraph(a["num_nodes"], a["node_len"], a["node_block_ptr"], a["node_blocks"], a["edge_ptr"], a["edge_dst"])
    b = W.Batch(a["path_ptr"], a["path_nodes"], a["new_lens"], a["tail_ptr"], a["tail_blocks"])
    wl = W.Workload("example", W.Shape(4, 4, 64), g, b, a["num_pool_blocks"], 0, np.zeros(0, np.int32),
                    np.zeros(0, np.int32))
    return fx, a, wl


def test_example_workflow_dag_bit_exact():
    fx, a, wl = _example_workload()
    want = oresolve.resolve_paths(**a)
    _, tables = run_resolve(wl, max_blocks=a["max_blocks"])
    assert_tables_equal(tables, want)
    got = R.tables_to_host(tables)
    for r, rq in enumerate(fx["requests"]):          # and against the hand-written golden values
        assert got["status"][r] == rq["status"]
        if rq["status"] == 0:
            assert got["block_table"][r] == rq["block_table"] and got["block_ntok"][r] == rq["block_ntok"]


def test_example_dag_without_edges():
    fx, a, wl = _example_workload()
    a2 = dict(a, edge_ptr=None, edge_dst=None, max_blocks=32)
    want = oresolve.resolve_paths(**a2)
    _, tables = run_resolve(wl, max_blocks=32, with_edges=False)
    assert_tables_equal(tables, want)


@pytest.mark.parametrize("cfg", list(W.CONFIGS))
def test_all_benchmark_configs_bit_exact(cfg):
    wl = W.CONFIGS[cfg]()
    want = oracle_resolve(wl)
    _, tables = run_resolve(wl)
    assert_tables_equal(tables, want)
    assert all(s == 0 for s in want["status"])


def test_single_layer_graph_has_no_edges_and_still_validates():
    """One layer: every path is one node, the graph has no edge at all, and edge validation is on."""
    wl = W.small_layered(61, W.Shape(4, 4, 64), num_nodes=9, num_layers=1, len_lo=3, len_hi=80, num_req=7, hops=(1, 4),
                         new_lo=1, new_hi=30)
    assert wl.graph.edge_dst.size == 0 and (np.diff(wl.batch.path_ptr) == 1).all()
    sess, tables = run_resolve(wl)
    assert_tables_equal(tables, oracle_resolve(wl))


def test_long_path_spans_several_scan_chunks():
    """A 700-node chain (more than two 256-node chunks of the kernel's scan) with
    ragged lengths, zero-length nodes included."""
    rng = np.random.default_rng(3)
    n = 700
    node_len = rng.integers(0, 40, size=n)
    edges = [(i, i + 1) for i in range(n - 1)]
    paths = [list(range(n)), list(range(100, 650)), [5], []]
    wl = W._finish("chain", W.Shape(4, 4, 64), node_len, edges, paths, np.array([3, 0, 17, 1]), rng, True, 3,
                   np.arange(4), np.zeros(0), 0.0)
    want = oracle_resolve(wl)
    assert want["status"] == [0, 0, 0, 0]
    _, tables = run_resolve(wl)
    assert_tables_equal(tables, want)


def test_error_precedence_and_pool_range():
    wl = W.small_layered(5, W.Shape(4, 2, 64), num_req=6)
    want = oracle_resolve(wl, max_blocks=max_blocks_of(wl))
    # shrink the pool so that some block ids fall outside it
    small_pool = wl.num_pool_blocks // 2
    want2 = oresolve.resolve_paths(wl.graph.num_nodes, wl.graph.node_len, wl.graph.node_block_ptr,
                                   wl.graph.node_blocks, wl.graph.edge_ptr, wl.graph.edge_dst, wl.batch.path_ptr,
                                   wl.batch.path_nodes, wl.batch.new_lens, wl.batch.tail_ptr, wl.batch.tail_blocks,
                                   max_blocks_of(wl), small_pool)
    assert any(s == oresolve.ST_BAD_BLOCK for s in want2["status"])
    _, tables = run_resolve(wl, num_pool_blocks=small_pool)
    assert_tables_equal(tables, want2)
    # a table that is too narrow for some requests
    mb = max(1, max_blocks_of(wl) // 2)
    want3 = oracle_resolve(wl, max_blocks=mb)
    assert any(s == oresolve.ST_OVERFLOW for s in want3["status"])
    _, tables = run_resolve(wl, max_blocks=mb)
    assert_tables_equal(tables, want3)
