"""Shared test helpers: load the golden example-workflow fixture, run the oracle
resolver on a workload."""
import json
import os

import numpy as np

from oracle import resolve as oresolve

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def load_example_dag():
    with open(os.path.join(GOLDEN, "example_workflow_dag.json")) as f:
        fx = json.load(f)
    name_to_id = {n: i for i, n in enumerate(fx["nodes"])}
    n = len(fx["nodes"])
    adj = [[] for _ in range(n)]
    for a, b in fx["edges"]:
        adj[name_to_id[a]].append(name_to_id[b])
    edge_ptr, edge_dst = [0], []
    for a in range(n):
        edge_dst += sorted(adj[a])
        edge_ptr.append(len(edge_dst))
    path_ptr, path_nodes, new_lens, tail_ptr, tail_blocks = [0], [], [], [0], []
    for rq in fx["requests"]:
        path_nodes += [name_to_id.get(v, v) for v in rq["path"]]
        path_ptr.append(len(path_nodes))
        new_lens.append(rq["new_len"])
        tail_blocks += rq["tail_blocks"]
        tail_ptr.append(len(tail_blocks))
    i32 = lambda x: np.asarray(x, dtype=np.int32)
    arrays = dict(num_nodes=n, node_len=i32(fx["node_len"]), node_block_ptr=i32(fx["node_block_ptr"]),
                  node_blocks=i32(fx["node_blocks"]), edge_ptr=i32(edge_ptr), edge_dst=i32(edge_dst),
                  path_ptr=i32(path_ptr), path_nodes=i32(path_nodes), new_lens=i32(new_lens),
                  tail_ptr=i32(tail_ptr), tail_blocks=i32(tail_blocks),
                  max_blocks=fx["max_blocks"], num_pool_blocks=fx["num_pool_blocks"])
    return fx, arrays


def max_blocks_of(wl):
    g, b = wl.graph, wl.batch
    best = 1
    for r in range(b.num_req):
        nodes = b.path_nodes[b.path_ptr[r]:b.path_ptr[r + 1]]
        nb = int(((g.node_len[nodes].astype(np.int64) + 15) // 16).sum()) + (int(b.new_lens[r]) + 15) // 16
        best = max(best, nb)
    return best


def oracle_resolve(wl, batch=None, max_blocks=None, with_edges=True):
    g = wl.graph
    b = wl.batch if batch is None else batch
    mb = max_blocks_of(wl) if max_blocks is None else max_blocks
    return oresolve.resolve_paths(
        g.num_nodes, g.node_len, g.node_block_ptr, g.node_blocks,
        g.edge_ptr if with_edges else None, g.edge_dst if with_edges else None,
        b.path_ptr, b.path_nodes, b.new_lens, b.tail_ptr, b.tail_blocks, mb, wl.num_pool_blocks)
