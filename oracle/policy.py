"""State-management policy oracle (pure Python): which table entries read a stored residual, the
execution statistics, and path pruning.  TEST INFRASTRUCTURE ONLY: nothing in the product imports it.

Follows the paper's Differential-based KV Cache (Eq. 7: the KV of operation v under prefix path P is
the node's base KV plus a sparse residual that belongs to the pair (P, v)) and Effective Path Pruning
(execution statistics identify the frequently exercised transitions; only their residuals are kept;
a pair without a stored residual falls back to computing its KV on the fly).

Conventions taken here (the paper names none):
  * a pair is identified by the whole prefix path ending in v, as a tuple (v_0, ..., v_i), i >= 1;
    the first node of a path has an empty prefix, so its base KV is exact and it never has a residual;
  * a stored residual of a pair covers all ceil(node_len / 16) blocks of v: residual items
    first_item .. first_item + nb - 1, one per block, in block order;
  * the transition of a pair is its last hop (v_{i-1}, v_i); the statistics count, per edge of the
    graph's edge list (position e in edge_dst), how often requests with status 0 took it;
  * pruning with threshold min_count drops the stored residual of every pair whose transition was
    taken fewer than min_count times.
The directory is a dict {prefix tuple: first_item}; a pruned or missing pair has no entry.

Pins: tests/test_oracle_policy.py (hand-computed values on the paper's example workflow DAG in
tests/golden/example_residual_policy.json, counting invariants, an entry-by-entry reformulation).
"""

BLOCK = 16


def _nb(length):
    return -(-max(int(length), 0) // BLOCK)


def residual_handles(status, node_len, path_ptr, path_nodes, directory, max_blocks):
    """Per request: handle per table entry (residual item id, or -1: read the base block as it is) and the
    number of path nodes with a non-empty prefix whose residual is not stored (to be computed on the fly).
    Requests with a non-zero status get no handles and count nothing."""
    handles, fallback = [], []
    for r in range(len(path_ptr) - 1):
        row = [-1] * max_blocks
        missing = 0
        if status[r] == 0:
            path = [int(v) for v in path_nodes[path_ptr[r]:path_ptr[r + 1]]]
            off = 0
            for i, v in enumerate(path):
                nb = _nb(node_len[v])
                if i >= 1:
                    first = directory.get(tuple(path[:i + 1]))
                    if first is None:
                        missing += 1
                    else:
                        for j in range(nb):
                            row[off + j] = first + j
                off += nb
        handles.append(row)
        fallback.append(missing)
    return handles, fallback


def transition_counts(status, edge_ptr, edge_dst, path_ptr, path_nodes, counts=None):
    """Execution statistics: counts[e] += 1 for every hop (u, v) of every request with status 0, e being the
    position of v in u's successor list.  `counts` continues earlier statistics (default: zeros)."""
    counts = [0] * len(edge_dst) if counts is None else list(counts)
    for r in range(len(path_ptr) - 1):
        if status[r] != 0:
            continue
        path = [int(v) for v in path_nodes[path_ptr[r]:path_ptr[r + 1]]]
        for u, v in zip(path[:-1], path[1:]):
            for e in range(int(edge_ptr[u]), int(edge_ptr[u + 1])):
                if int(edge_dst[e]) == v:
                    counts[e] += 1
                    break
    return counts


def pair_uses(status, path_ptr, path_nodes, pairs):
    """How many times requests with status 0 walk each of the given pairs (prefix tuples)."""
    uses = {tuple(k): 0 for k in pairs}
    for r in range(len(path_ptr) - 1):
        if status[r] != 0:
            continue
        path = [int(v) for v in path_nodes[path_ptr[r]:path_ptr[r + 1]]]
        for i in range(1, len(path)):
            key = tuple(path[:i + 1])
            if key in uses:
                uses[key] += 1
    return uses


def prune(directory, node_len, edge_ptr, edge_dst, counts, min_count):
    """Drop the stored residual of every pair whose last hop was taken fewer than min_count times.
    Returns (kept directory, sorted list of pruned prefix tuples, number of residual items freed)."""
    kept, pruned, freed = {}, [], 0
    for key, first in directory.items():
        u, v = key[-2], key[-1]
        taken = 0
        for e in range(int(edge_ptr[u]), int(edge_ptr[u + 1])):
            if int(edge_dst[e]) == v:
                taken = counts[e]
                break
        if taken >= min_count:
            kept[key] = first
        else:
            pruned.append(key)
            freed += _nb(node_len[v])
    return kept, sorted(pruned), freed
