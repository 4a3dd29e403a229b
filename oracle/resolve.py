"""Path resolution oracle: wGraph node path -> block table (pure Python lists).

Follows the paper's description of assembling a workflow's KV from the selected
operation nodes (Topology-Aware State Management, first paragraphs) with the
prefix path P of Eq. 7 as the input, and the Overview's definition of edges as
the valid transitions between operations.

Per request r with path (v_0 .. v_{d-1}), new_len n and a private tail block list:
  * every v_i must be a node id; with edges given, every (v_i, v_{i+1}) must be
    an edge; the tail list must hold at least ceil(n/16) blocks; every node
    must own at least ceil(len/16) blocks and every block id used must lie in
    [0, num_pool_blocks) (else BAD_BLOCK); the table must fit max_blocks.
  * ctx_len = sum of node_len over the path; seq_len = ctx_len + n.
  * table = the nodes' block lists concatenated in path order, then the first
    ceil(n/16) tail blocks; each segment's blocks hold 16 tokens except its last
    one, which holds the remainder.
  * a failed request reports its status and pad outputs (table -1, ntok 0,
    num_blocks 0, lengths 0).  Status precedence when several checks fail:
    BAD_NODE, BAD_EDGE, BAD_TAIL, BAD_BLOCK, OVERFLOW.

Pins: tests/test_oracle_resolve.py (the paper's example workflow DAG with a
hand-written expected table in tests/golden/, counting invariants, and a
hand-computed table for a tree).
"""

BLOCK = 16
ST_OK, ST_BAD_NODE, ST_BAD_EDGE, ST_BAD_TAIL, ST_BAD_BLOCK, ST_OVERFLOW = 0, 1, 2, 3, 4, 5


def _segment(blocks, length):
    """Blocks and per-block token counts of one token segment of ``length``."""
    nb = -(-length // BLOCK)
    ids = [int(b) for b in blocks[:nb]]
    ntok = [BLOCK] * nb
    if nb:
        ntok[-1] = length - BLOCK * (nb - 1)
    return ids, ntok


def resolve_paths(num_nodes, node_len, node_block_ptr, node_blocks, edge_ptr, edge_dst,
                  path_ptr, path_nodes, new_lens, tail_ptr, tail_blocks,
                  max_blocks, num_pool_blocks):
    """Returns dict of Python lists: block_table[R][max_blocks], block_ntok[R][max_blocks],
    num_blocks[R], ctx_lens[R], seq_lens[R], status[R].  ``edge_ptr`` None skips
    edge validation; ``tail_ptr`` None means no request has tail blocks."""
    R = len(path_ptr) - 1
    out = {k: [] for k in ("block_table", "block_ntok", "num_blocks", "ctx_lens", "seq_lens", "status")}
    for r in range(R):
        path = [int(v) for v in path_nodes[path_ptr[r]:path_ptr[r + 1]]]
        n_new = int(new_lens[r]) if new_lens is not None else 0
        tails = [] if tail_ptr is None else [int(b) for b in tail_blocks[tail_ptr[r]:tail_ptr[r + 1]]]
        status = ST_OK
        bad_node = any(v < 0 or v >= num_nodes for v in path)
        if bad_node:
            status = ST_BAD_NODE
        if status == ST_OK and edge_ptr is not None:
            for a, b in zip(path[:-1], path[1:]):
                succ = [int(x) for x in edge_dst[edge_ptr[a]:edge_ptr[a + 1]]]
                if b not in succ:
                    status = ST_BAD_EDGE
                    break
        ids, ntok, ctx = [], [], 0
        if status == ST_OK:
            if n_new < 0 or len(tails) < -(-n_new // BLOCK):
                status = ST_BAD_TAIL
        if status == ST_OK:
            short = False
            for v in path:
                length = int(node_len[v])
                own = node_blocks[node_block_ptr[v]:node_block_ptr[v + 1]]
                short = short or length < 0 or len(own) < -(-length // BLOCK)
                seg_ids, seg_ntok = _segment(own, max(length, 0))
                ids += seg_ids
                ntok += seg_ntok
                ctx += length
            seg_ids, seg_ntok = _segment(tails, n_new)
            ids += seg_ids
            ntok += seg_ntok
            if short or any(b < 0 or b >= num_pool_blocks for b in ids):
                status = ST_BAD_BLOCK
            elif len(ids) > max_blocks:
                status = ST_OVERFLOW
        if status != ST_OK:
            ids, ntok, ctx, n_new = [], [], 0, 0
        pad = max_blocks - len(ids)
        out["block_table"].append(ids + [-1] * pad)
        out["block_ntok"].append(ntok + [0] * pad)
        out["num_blocks"].append(len(ids))
        out["ctx_lens"].append(ctx)
        out["seq_lens"].append(ctx + n_new)
        out["status"].append(status)
    return out
