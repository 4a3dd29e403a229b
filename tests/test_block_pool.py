"""gf_block_pool (host-side free list with reference counts) through the C ABI; no GPU needed.  The expected
states are counted by hand: a node's blocks are allocated once and retained by every further workflow through
the node; they return to the free list only when the last holder lets go."""
import os

import numpy as np
import pytest

from paper_2605_22566_amd import binding as B

pytestmark = pytest.mark.skipif(not os.path.exists(B.LIB_PATH), reason="libgraphflow.so not built")


def test_alloc_retain_release_follow_the_reference_counts():
    p = B.BlockPool(10)
    assert p.stats() == {"free": 10, "in_use": 0, "total_refs": 0, "peak_in_use": 0}
    node_a = p.alloc(3)                        # a node's base KV: stored once
    node_b = p.alloc(2)
    assert node_a == [0, 1, 2] and node_b == [3, 4]          # lowest free ids first
    p.retain(node_a)                           # a second workflow passes through node a
    p.retain(node_a)                           # and a third
    assert [p.refcount(b) for b in range(6)] == [3, 3, 3, 1, 1, 0]
    assert p.stats() == {"free": 5, "in_use": 5, "total_refs": 11, "peak_in_use": 5}
    assert p.release(node_a) == 0              # two holders left
    assert p.release(node_b) == 2              # node b is gone: its blocks are free again
    assert p.release(node_a + node_a) == 3     # both remaining holders at once
    assert p.stats() == {"free": 10, "in_use": 0, "total_refs": 0, "peak_in_use": 5}
    again = p.alloc(4)
    assert sorted(again) == sorted(set(again)) and set(again) <= set(range(10))
    p.close()


def test_errors_change_nothing():
    p = B.BlockPool(4)
    ids = p.alloc(3)
    with pytest.raises(B.GraphFlowError) as e:
        p.alloc(2)                              # only one block left: all or nothing
    assert e.value.code == B.GF_ERR_WORKSPACE and p.stats()["free"] == 1
    for bad in ([7], [-1], [3], ids + [ids[0], ids[0]]):       # outside, outside, not allocated, too many releases
        with pytest.raises(B.GraphFlowError) as e:
            p.release(bad)
        assert e.value.code == B.GF_ERR_BAD_SHAPE
        assert p.stats() == {"free": 1, "in_use": 3, "total_refs": 3, "peak_in_use": 3}
    with pytest.raises(B.GraphFlowError):
        p.retain([3])                           # not allocated
    assert p.release(ids) == 3
    lib = B.load_library()
    assert lib.gf_block_pool_alloc(None, 1, None) == B.GF_ERR_NULL
    assert lib.gf_block_pool_destroy(None) == B.GF_ERR_NULL
    p.close()


def test_serving_a_batch_keeps_shared_nodes_once():
    """Blocks in use while a batch of requests over a shared graph is alive = every touched node once + the
    requests' tails (the store-once footprint), against one copy per request for private caches."""
    from paper_2605_22566_amd import workload as W
    wl = W.small_layered(9, W.Shape(8, 2, 64), num_nodes=20, num_layers=5, len_lo=20, len_hi=90, num_req=16,
                         hops=(2, 5), new_lo=1, new_hi=30)
    g, b = wl.graph, wl.batch
    nbl = (g.node_len.astype(np.int64) + 15) // 16
    p = B.BlockPool(4096)
    node_blocks, held = {}, []
    for r in range(b.num_req):
        mine = []
        for v in b.path_nodes[b.path_ptr[r]:b.path_ptr[r + 1]]:
            v = int(v)
            if v in node_blocks:
                p.retain(node_blocks[v])
            else:
                node_blocks[v] = p.alloc(int(nbl[v]))
            mine += node_blocks[v]
        mine += p.alloc((int(b.new_lens[r]) + 15) // 16)
        held.append(mine)
    used = np.unique(b.path_nodes)
    tails = int(((b.new_lens.astype(np.int64) + 15) // 16).sum())
    assert p.stats()["in_use"] == int(nbl[used].sum()) + tails
    private = sum(len(h) for h in held)
    assert p.stats()["total_refs"] == private and private > p.stats()["in_use"]
    for h in held[:-1]:
        p.release(h)
    last_nodes = {int(v) for v in b.path_nodes[b.path_ptr[-2]:b.path_ptr[-1]]}
    assert p.stats()["in_use"] == int(nbl[sorted(last_nodes)].sum()) + (int(b.new_lens[-1]) + 15) // 16
    assert p.release(held[-1]) == len(held[-1])            # the last holder frees everything it held
    assert p.stats()["in_use"] == 0
    p.close()
