"""Pool-free brute force ("full recompute"), explicit loops, tiny inputs only.

It never sees blocks, tables or the pool: a request's keys and values are the
per-node *source* segments concatenated in path order followed by the new
tokens' own K/V, exactly the fully stateful per-workflow cache the paper
contrasts against (Topology-Aware State Management section), and attention is
the textbook definition written element by element.
"""
import math


def attend_bruteforce(q, node_k, node_v, path, new_k, new_v, group, sm_scale=None):
    """q: [n][Hq][D] nested sequences (or arrays) of floats; node_k/node_v: dict
    node -> [len][Hkv][D]; new_k/new_v: [n][Hkv][D].  Returns O as nested lists
    [n][Hq][D] and lse [n][Hq]."""
    keys, vals = [], []
    for v in path:
        for t in range(len(node_k[v])):
            keys.append(node_k[v][t])
            vals.append(node_v[v][t])
    ctx = len(keys)
    for t in range(len(new_k)):
        keys.append(new_k[t])
        vals.append(new_v[t])
    n = len(q)
    hq = len(q[0]) if n else 0
    d = len(q[0][0]) if n else 0
    scale = 1.0 / math.sqrt(d) if not sm_scale else sm_scale
    O = [[[0.0] * d for _ in range(hq)] for _ in range(n)]
    lse = [[0.0] * hq for _ in range(n)]
    for i in range(n):
        last = ctx + i                      # new token i sees keys 0..ctx+i
        for h in range(hq):
            kvh = h // group
            scores = []
            for j in range(last + 1):
                acc = 0.0
                for x in range(d):
                    acc += float(q[i][h][x]) * float(keys[j][kvh][x])
                scores.append(acc * scale)
            mx = max(scores)
            w = [math.exp(s - mx) for s in scores]
            tot = sum(w)
            for x in range(d):
                acc = 0.0
                for j in range(last + 1):
                    acc += w[j] * float(vals[j][kvh][x])
                O[i][h][x] = acc / tot
            lse[i][h] = mx + math.log(tot)
    return O, lse
