"""Pins for the path-resolution oracle (CPU only)."""
import numpy as np
import pytest

from oracle import resolve as oresolve
from paper_2605_22566_amd import workload as W
from tests.helpers import load_example_dag, max_blocks_of, oracle_resolve


def test_example_workflow_dag_golden():
    """Hand-computed tables on the paper's example workflow DAG (appendix
    'Example of a Workflow'): both root-to-sink paths, an invalid hop
    OP_02 -> OP_03, an unknown node, overflow, short tail, bad block, empty path."""
    fx, a = load_example_dag()
    out = oresolve.resolve_paths(**a)
    for r, rq in enumerate(fx["requests"]):
        assert out["status"][r] == rq["status"], r
        assert out["ctx_lens"][r] == rq["ctx_len"], r
        assert out["seq_lens"][r] == rq["seq_len"], r
        assert out["num_blocks"][r] == rq["num_blocks"], r
        if rq["status"] == 0:
            assert out["block_table"][r] == rq["block_table"], r
            assert out["block_ntok"][r] == rq["block_ntok"], r
        else:
            assert out["block_table"][r] == [-1] * fx["max_blocks"]
            assert out["block_ntok"][r] == [0] * fx["max_blocks"]


def test_shared_nodes_give_identical_blocks_at_different_offsets():
    fx, a = load_example_dag()
    out = oresolve.resolve_paths(**a)
    t0, t1 = out["block_table"][0], out["block_table"][1]
    assert t0[:9] == t1[:9]                 # OP_01 shared, same offset
    assert t0[14:16] == t1[12:14] == [17, 18]  # OP_04, OP_05 shared, shifted by the middle node


def test_edges_none_skips_validation():
    fx, a = load_example_dag()
    a = dict(a, edge_ptr=None, edge_dst=None, max_blocks=32)   # 19 blocks would overflow 18
    out = oresolve.resolve_paths(**a)
    assert out["status"][2] == 0           # OP_02 -> OP_03 accepted without edges
    assert out["ctx_lens"][2] == 135 + 65 + 40 + 16


@pytest.mark.parametrize("cfg", ["tiny", "prefill_8b", "decode_8b", "mixed_fp8"])
def test_counting_invariants(cfg):
    wl = W.CONFIGS[cfg]()
    out = oracle_resolve(wl)
    g, b = wl.graph, wl.batch
    L = W.context_lens(wl)
    for r in range(b.num_req):
        nodes = b.path_nodes[b.path_ptr[r]:b.path_ptr[r + 1]]
        assert out["status"][r] == 0
        assert out["ctx_lens"][r] == int(L[r])
        assert out["seq_lens"][r] == int(L[r]) + int(b.new_lens[r])
        nb = out["num_blocks"][r]
        assert nb == int(((g.node_len[nodes] + 15) // 16).sum()) + (int(b.new_lens[r]) + 15) // 16
        nt = out["block_ntok"][r]
        assert sum(nt) == out["seq_lens"][r]
        assert all(1 <= x <= 16 for x in nt[:nb]) and all(x == 0 for x in nt[nb:])
        assert all(x == -1 for x in out["block_table"][r][nb:])
        assert len(set(nodes.tolist())) == len(nodes)          # a DAG path never repeats a node
        # every block of a node except its last is full
        e = 0
        for v in nodes:
            k = (int(g.node_len[v]) + 15) // 16
            assert all(x == 16 for x in nt[e:e + k - 1])
            assert nt[e + k - 1] == int(g.node_len[v]) - 16 * (k - 1)
            e += k


def test_tiny_hand_table():
    """Tiny config: 32-token nodes own blocks (2v, 2v+1) (sequential ids), so the
    table of a root-to-leaf path is written down directly from the path."""
    wl = W.config_tiny()
    out = oracle_resolve(wl)
    b = wl.batch
    assert max_blocks_of(wl) == 9
    for r in range(4):
        path = b.path_nodes[b.path_ptr[r]:b.path_ptr[r + 1]].tolist()
        assert len(path) == 4 and path[0] == 0
        expect = [x for v in path for x in (2 * v, 2 * v + 1)] + [16 + r]
        assert out["block_table"][r] == expect
        assert out["block_ntok"][r] == [16] * 9
        assert out["ctx_lens"][r] == 128 and out["seq_lens"][r] == 144


def test_pool_bytes_independent_of_batch_size():
    """Store-once footprint: the node part of the pool does not grow with the
    number of requests while the per-request (stateful) total does (the shape of
    the paper's memory-vs-batch-size figure)."""
    sh = W.Shape(32, 8, 128)
    sizes = []
    for nreq in (10, 50):
        wl = W._layered_config("fp", 1234, sh, 256, 12, 64, 512, 1.1, num_req=nreq, hops=(4, 12),
                               new_lo=1, new_hi=1, num_prefill=0)
        node_blocks = int(wl.graph.node_block_ptr[-1])
        stateful = int(W.context_lens(wl).sum())
        sizes.append((node_blocks, stateful))
    assert sizes[0][0] == sizes[1][0]
    assert sizes[1][1] > 3 * sizes[0][1]
