"""KV memory footprint of a batch under the three state-management designs the paper compares
(Effectiveness of topology-aware state management; Memory footprint under different request batch
sizes) and under transition pruning (Effective Path Pruning).  Host-side accounting only: no tensor
is touched, the byte counts follow from the graph, the batch and the pool / residual formats of this
library (one layer; K and V; blocks of 16 tokens are allocated whole).

  stateful      one private KV copy per distinct (prefix path, node) pair the batch contains: exact states,
                shared only between requests whose whole prefix up to the node is identical
  stateless     every node once (what the block pool holds when every residual is zero)
  differential  every node once + a sparse residual per distinct (prefix, node) pair with a non-empty
                prefix, `density_k` / `density_v` of the elements kept, in the form it is stored in at rest
                (`residual_form="packed"`: one bit per element of every (block, tensor, kv head) image + 2 B per
                kept value) or in the form the attention kernels read (`"coordinate"`: 2 B index + 2 B value
                per kept element)
  pruned        differential, but residuals only for pairs reached through a transition (previous node ->
                node) seen at least `min_count` times in the execution statistics; the others fall back
                to on-the-fly computation and store nothing
Every design also holds the requests' private tails (their new tokens).
"""
from typing import Dict, Iterable, Optional

import numpy as np

from . import workload as W


def _blocks(n_tokens) -> np.ndarray:
    return (np.asarray(n_tokens, dtype=np.int64) + W.BLOCK - 1) // W.BLOCK


def transition_counts(batch: W.Batch) -> Dict[tuple, int]:
    """How often each (previous node, node) transition occurs in the batch's paths."""
    cnt: Dict[tuple, int] = {}
    for r in range(batch.num_req):
        p = batch.path_nodes[batch.path_ptr[r]:batch.path_ptr[r + 1]]
        for a, b in zip(p[:-1], p[1:]):
            cnt[(int(a), int(b))] = cnt.get((int(a), int(b)), 0) + 1
    return cnt


def residual_block_bytes(shape: W.Shape, density_k: float, density_v: float, form: str = "packed") -> float:
    """Bytes a residual holds per pool block of its node (all kv heads, K and V)."""
    img_elems = W.BLOCK * shape.head_dim                               # one (tensor, kv head) image of a block
    kept = shape.num_kv_heads * img_elems * (density_k + density_v)
    rows = 2 * shape.num_kv_heads
    if form == "packed":
        return kept * 2.0 + rows * img_elems / 8.0 + rows * 4 + 8      # values, masks, row pointers, block ids
    if form == "coordinate":
        return kept * 4.0 + rows * 4 + 8                               # 2 B index + 2 B value
    raise ValueError(form)


def footprint(wl: W.Workload, requests: Optional[Iterable[int]] = None, density_k: float = 0.25,
              density_v: float = 0.30, min_count: int = 2, stats: Optional[Dict[tuple, int]] = None,
              residual_form: str = "packed") -> dict:
    """Bytes held for the given requests (default: the whole batch) under each design.  `stats` are the
    transition counts pruning looks at (default: those of the whole batch)."""
    sh, g, b = wl.shape, wl.graph, wl.batch
    req = list(range(b.num_req)) if requests is None else [int(r) for r in requests]
    esz = 2 if sh.kv_dtype == W.KV_BF16 else 1
    blk_bytes = 2 * sh.num_kv_heads * W.BLOCK * sh.head_dim * esz + (8 if esz == 1 else 0)   # K + V (+ two scales)
    res_blk_bytes = residual_block_bytes(sh, density_k, density_v, residual_form)
    stats = transition_counts(b) if stats is None else stats
    nblk = _blocks(g.node_len)
    nodes, pairs, pruned_pairs = set(), {}, {}
    tail_blocks = 0
    for r in req:
        p = [int(v) for v in b.path_nodes[b.path_ptr[r]:b.path_ptr[r + 1]]]
        tail_blocks += int(_blocks(b.new_lens[r]))
        for i, v in enumerate(p):
            nodes.add(v)
            key = tuple(p[:i + 1])                                     # the prefix path ending in v
            pairs[key] = int(nblk[v])
            if i > 0 and stats.get((p[i - 1], v), 0) >= min_count:
                pruned_pairs[key] = int(nblk[v])
    base = sum(int(nblk[v]) for v in nodes)
    with_prefix = sum(n for k, n in pairs.items() if len(k) > 1)
    kept = sum(pruned_pairs.values())
    tails = tail_blocks * blk_bytes
    return {
        "requests": len(req), "residual_form": residual_form, "nodes": len(nodes), "prefix_node_pairs": len(pairs),
        "pairs_with_residual": sum(1 for k in pairs if len(k) > 1), "pairs_kept_by_pruning": len(pruned_pairs),
        "stateful_bytes": float(sum(pairs.values())) * blk_bytes + tails,
        "stateless_bytes": float(base) * blk_bytes + tails,
        "differential_bytes": float(base) * blk_bytes + with_prefix * res_blk_bytes + tails,
        "pruned_bytes": float(base) * blk_bytes + kept * res_blk_bytes + tails,
        "fallback_pairs": sum(1 for k in pairs if len(k) > 1) - len(pruned_pairs),
    }


def footprint_by_batch_size(wl: W.Workload, sizes=(10, 20, 30, 40, 50), **kw) -> list:
    """The accounting for the first n requests of the batch, n in `sizes` (clipped to the batch): the shape of
    the paper's memory-against-concurrency figure on a synthetic graph."""
    out = []
    for n in sizes:
        n = min(int(n), wl.batch.num_req)
        out.append(footprint(wl, range(n), **kw))
    return out
