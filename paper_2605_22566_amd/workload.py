"""Seeded synthetic wGraph workloads (inputs only).

This module builds the *inputs* of the graph-KV attention path: a wGraph (the
global operation DAG of the paper's Overview section), per-node token-segment
lengths, the physical block lists of the paged K/V pool, request node paths,
and the random tensors that fill Q and the pool.  It serves both the CPU
oracle's tests and the GPU path, so it holds none of the method's arithmetic:
no path resolution, no attention, no format decoding.  Number formats are
produced only through library conversions (torch's bf16 / float8_e4m3fn casts).

Layouts produced here (block size B = 16 tokens):
  K pool  : [num_blocks, Hkv, B, D]   (token-major inside a block)
  V pool  : [num_blocks, Hkv, D, B]   (head-dim-major inside a block)
  bf16 is carried as raw uint16 bit patterns, e4m3 as raw uint8 codes.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional

import numpy as np

BLOCK = 16
SEED_BASE = 20260522  # per-config seed = SEED_BASE + config index

KV_BF16 = 0
KV_FP8_E4M3 = 1


# --------------------------------------------------------------------------- #
# data model
# --------------------------------------------------------------------------- #
@dataclasses.dataclass
class WGraph:
    """wGraph as CSR arrays (all int32)."""
    num_nodes: int
    node_len: np.ndarray        # [N] tokens in the node's KV segment
    node_block_ptr: np.ndarray  # [N+1]
    node_blocks: np.ndarray     # [sum ceil(len/16)] physical block ids
    edge_ptr: np.ndarray        # [N+1]
    edge_dst: np.ndarray        # [E] valid transitions v -> edge_dst[...]


@dataclasses.dataclass
class Batch:
    """A batch of requests: node paths (CSR) + new-token counts + tail blocks."""
    path_ptr: np.ndarray     # [R+1]
    path_nodes: np.ndarray   # [sum path lengths]
    new_lens: np.ndarray     # [R]
    tail_ptr: np.ndarray     # [R+1]
    tail_blocks: np.ndarray  # [sum ceil(new_len/16)]

    @property
    def num_req(self) -> int:
        return int(self.new_lens.shape[0])


@dataclasses.dataclass
class Shape:
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    kv_dtype: int = KV_BF16
    block_size: int = BLOCK

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads


@dataclasses.dataclass
class Workload:
    name: str
    shape: Shape
    graph: WGraph
    batch: Batch
    num_pool_blocks: int
    seed: int
    # request classes for mixed batches: indices into the batch
    prefill_req: np.ndarray
    decode_req: np.ndarray
    zipf_s: float = 1.1


def _i32(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x, dtype=np.int32))


def _nblk(n: int) -> int:
    return (int(n) + BLOCK - 1) // BLOCK


# --------------------------------------------------------------------------- #
# graph builders
# --------------------------------------------------------------------------- #
def edges_to_csr(num_nodes: int, edges: List[tuple]) -> tuple:
    adj: List[List[int]] = [[] for _ in range(num_nodes)]
    for a, b in edges:
        adj[a].append(b)
    ptr = [0]
    dst: List[int] = []
    for a in range(num_nodes):
        dst.extend(sorted(adj[a]))
        ptr.append(len(dst))
    return _i32(ptr), _i32(dst)


def assign_blocks(node_len: np.ndarray, new_lens: np.ndarray, rng: Optional[np.random.Generator],
                  shuffle: bool) -> tuple:
    """Give every node ceil(len/16) blocks and every request ceil(new/16) private
    tail blocks.  Ids are sequential (nodes first, then tails) or, with
    ``shuffle``, a random permutation of the whole pool."""
    nb_node = [(int(l) + BLOCK - 1) // BLOCK for l in node_len]
    nb_tail = [(int(l) + BLOCK - 1) // BLOCK for l in new_lens]
    total = sum(nb_node) + sum(nb_tail)
    ids = np.arange(total, dtype=np.int64)
    if shuffle:
        assert rng is not None
        ids = rng.permutation(total)
    node_block_ptr = np.concatenate([[0], np.cumsum(nb_node)])
    tail_ptr = np.concatenate([[0], np.cumsum(nb_tail)])
    n_node_blocks = int(node_block_ptr[-1])
    return (_i32(node_block_ptr), _i32(ids[:n_node_blocks]), _i32(tail_ptr),
            _i32(ids[n_node_blocks:]), total)


def random_tree(rng: np.random.Generator, num_nodes: int, min_depth: int):
    """Random recursive tree: parent of node k uniform in [0,k); resampled until
    its depth reaches ``min_depth``.  Returns (parent[], depth[])."""
    while True:
        parent = np.full(num_nodes, -1, dtype=np.int64)
        depth = np.zeros(num_nodes, dtype=np.int64)
        for k in range(1, num_nodes):
            parent[k] = rng.integers(0, k)
            depth[k] = depth[parent[k]] + 1
        if depth.max() >= min_depth:
            return parent, depth


def layered_dag(rng: np.random.Generator, num_nodes: int, num_layers: int, fanout: int, zipf_s: float):
    """Layered DAG: nodes are split into ``num_layers`` layers of ceil(N/layers)
    nodes (last layer takes the remainder); every node gets ``fanout`` distinct
    successors in the next layer, drawn with probability proportional to the
    successor's popularity weight rank^-s (rank = a fixed random permutation of
    the layer).  Returns (layer lists, weight[N], succ lists)."""
    per = math.ceil(num_nodes / num_layers)
    layers: List[np.ndarray] = []
    start = 0
    while start < num_nodes:
        layers.append(np.arange(start, min(start + per, num_nodes)))
        start += per
    weight = np.zeros(num_nodes, dtype=np.float64)
    for lay in layers:
        ranks = rng.permutation(len(lay)) + 1
        weight[lay] = ranks.astype(np.float64) ** (-zipf_s)
    succ: List[np.ndarray] = [np.zeros(0, dtype=np.int64) for _ in range(num_nodes)]
    for li in range(len(layers) - 1):
        nxt = layers[li + 1]
        p = weight[nxt] / weight[nxt].sum()
        k = min(fanout, len(nxt))
        for v in layers[li]:
            succ[v] = np.sort(rng.choice(nxt, size=k, replace=False, p=p))
    return layers, weight, succ


def _walk_fixed_hops(rng, layers, weight, succ, hops: int) -> List[int]:
    lay0 = layers[0]
    p0 = weight[lay0] / weight[lay0].sum()
    v = int(rng.choice(lay0, p=p0))
    path = [v]
    while len(path) < hops and len(succ[v]) > 0:
        s = succ[v]
        p = weight[s] / weight[s].sum()
        v = int(rng.choice(s, p=p))
        path.append(v)
    return path


def _walk_token_target(rng, layers, weight, succ, node_len, lo: int, hi: int) -> List[int]:
    """Walk until the next node would push the context over a target drawn
    uniformly in [lo, hi]; resample the whole request if the total stays
    below ``lo``."""
    lay0 = layers[0]
    p0 = weight[lay0] / weight[lay0].sum()
    while True:
        tau = int(rng.integers(lo, hi + 1))
        v = int(rng.choice(lay0, p=p0))
        if node_len[v] > tau:
            continue
        path = [v]
        total = int(node_len[v])
        while len(succ[v]) > 0:
            s = succ[v]
            p = weight[s] / weight[s].sum()
            nv = int(rng.choice(s, p=p))
            if total + int(node_len[nv]) > tau:
                break
            v = nv
            path.append(v)
            total += int(node_len[v])
        if total >= lo:
            return path


def _finish(name, shape, node_len, edges, paths, new_lens, rng, shuffle, seed,
            prefill_req, decode_req, zipf_s) -> Workload:
    n = len(node_len)
    edge_ptr, edge_dst = edges_to_csr(n, edges)
    nbp, nblocks, tail_ptr, tail_blocks, total = assign_blocks(node_len, new_lens, rng, shuffle)
    graph = WGraph(n, _i32(node_len), nbp, nblocks, edge_ptr, edge_dst)
    path_ptr = np.concatenate([[0], np.cumsum([len(p) for p in paths])])
    flat = [v for p in paths for v in p]
    batch = Batch(_i32(path_ptr), _i32(flat), _i32(new_lens), tail_ptr, tail_blocks)
    return Workload(name, shape, graph, batch, total, seed, _i32(prefill_req), _i32(decode_req), zipf_s)


# --------------------------------------------------------------------------- #
# the five benchmark configurations
# --------------------------------------------------------------------------- #
def config_tiny(seed: int = SEED_BASE + 0) -> Workload:
    """Random 8-node tree, 32-token segments, 4 root-to-depth-3 requests with 16
    new tokens each; 4 q heads = 4 kv heads, head_dim 64."""
    rng = np.random.default_rng(seed)
    parent, depth = random_tree(rng, 8, 3)
    node_len = np.full(8, 32, dtype=np.int64)
    edges = [(int(parent[k]), k) for k in range(1, 8)]
    leaves = np.nonzero(depth == 3)[0]
    paths = []
    for _ in range(4):
        t = int(rng.choice(leaves))
        p = [t]
        while parent[p[-1]] >= 0:
            p.append(int(parent[p[-1]]))
        paths.append(p[::-1])
    new_lens = np.full(4, 16, dtype=np.int64)
    shape = Shape(4, 4, 64)
    return _finish("tiny", shape, node_len, edges, paths, new_lens, rng, False, seed,
                   np.arange(4), np.zeros(0), 0.0)


def _layered_config(name, seed, shape, num_nodes, num_layers, len_lo, len_hi, zipf_s,
                    num_req, hops=None, tokens=None, new_lo=1, new_hi=1, shuffle=False,
                    num_prefill=None) -> Workload:
    rng = np.random.default_rng(seed)
    layers, weight, succ = layered_dag(rng, num_nodes, num_layers, 8, zipf_s)
    node_len = rng.integers(len_lo, len_hi + 1, size=num_nodes)
    paths = []
    for _ in range(num_req):
        if hops is not None:
            d = int(rng.integers(hops[0], hops[1] + 1))
            paths.append(_walk_fixed_hops(rng, layers, weight, succ, d))
        else:
            paths.append(_walk_token_target(rng, layers, weight, succ, node_len, tokens[0], tokens[1]))
    if num_prefill is None:
        num_prefill = num_req if new_hi > 1 else 0
    new_lens = np.ones(num_req, dtype=np.int64)
    if num_prefill > 0:
        new_lens[:num_prefill] = rng.integers(new_lo, new_hi + 1, size=num_prefill)
    prefill_req = np.arange(num_prefill)
    decode_req = np.arange(num_prefill, num_req)
    edges = [(a, int(b)) for a in range(num_nodes) for b in succ[a]]
    return _finish(name, shape, node_len, edges, paths, new_lens, rng, shuffle, seed,
                   prefill_req, decode_req, zipf_s)


def config_prefill_8b(seed: int = SEED_BASE + 1) -> Workload:
    return _layered_config("prefill_8b", seed, Shape(32, 8, 128), 256, 12, 64, 512, 1.1,
                           num_req=64, hops=(4, 12), new_lo=128, new_hi=1024)


def config_decode_8b(seed: int = SEED_BASE + 2) -> Workload:
    return _layered_config("decode_8b", seed, Shape(32, 8, 128), 1024, 32, 128, 2048, 1.1,
                           num_req=256, tokens=(2048, 16384), shuffle=True)


def config_decode_70b(seed: int = SEED_BASE + 3) -> Workload:
    return _layered_config("decode_70b", seed, Shape(64, 8, 128), 4096, 64, 128, 2048, 1.2,
                           num_req=512, tokens=(8192, 32768), shuffle=True)


def config_mixed_fp8(seed: int = SEED_BASE + 4) -> Workload:
    return _layered_config("mixed_fp8", seed, Shape(32, 8, 128, KV_FP8_E4M3), 2048, 32, 128, 2048, 1.1,
                           num_req=512, tokens=(4096, 16384), new_lo=256, new_hi=2048,
                           shuffle=True, num_prefill=128)


CONFIGS = {
    "tiny": config_tiny,
    "prefill_8b": config_prefill_8b,
    "decode_8b": config_decode_8b,
    "decode_70b": config_decode_70b,
    "mixed_fp8": config_mixed_fp8,
}
# measurement workloads beside the five configurations (filled below)
MEASUREMENT_CONFIGS = {}


def small_layered(seed: int, shape: Shape, num_nodes=24, num_layers=6, len_lo=5, len_hi=70,
                  num_req=6, hops=(1, 6), new_lo=1, new_hi=40, shuffle=True, zipf_s=1.1) -> Workload:
    """A reduced layered-DAG workload with ragged segment lengths, for parity
    tests that the oracle finishes in seconds."""
    return _layered_config(f"small_{seed}", seed, shape, num_nodes, num_layers, len_lo, len_hi, zipf_s,
                           num_req=num_req, hops=hops, new_lo=new_lo, new_hi=max(new_hi, 2),
                           shuffle=shuffle)


def private_copies(wl: Workload, shuffle: bool = True) -> Workload:
    """The same requests with nothing shared: every (request, path position) becomes a node of its own with
    its own pool blocks (the "stateful" per-workflow cache the paper compares against).  Request-centric bytes,
    unique bytes and HBM bytes of a decode step then coincide, which makes the step's time a direct reading
    of the kernel's HBM rate.  Edges follow the private chains."""
    g, b = wl.graph, wl.batch
    rng = np.random.default_rng([wl.seed, 23])
    node_len, paths, edges = [], [], []
    for r in range(b.num_req):
        p = []
        for v in b.path_nodes[b.path_ptr[r]:b.path_ptr[r + 1]]:
            p.append(len(node_len))
            node_len.append(int(g.node_len[v]))
        edges += list(zip(p[:-1], p[1:]))
        paths.append(p)
    return _finish(wl.name + "_private", wl.shape, np.asarray(node_len, dtype=np.int64), edges, paths,
                   b.new_lens.astype(np.int64), rng, shuffle, wl.seed, wl.prefill_req, wl.decode_req, wl.zipf_s)


def config_decode_8b_private(seed: int = SEED_BASE + 2) -> Workload:
    """Config 3's requests with private copies of every node (no sharing): a measurement workload, not one of
    the five configurations."""
    return private_copies(config_decode_8b(seed))


MEASUREMENT_CONFIGS["decode_8b_private"] = config_decode_8b_private
# the same with every request's blocks laid out one after the other in the pool (no shuffle): what random block
# placement costs at the DRAM shows as the difference between the two
MEASUREMENT_CONFIGS["decode_8b_private_seq"] = lambda: private_copies(config_decode_8b(), shuffle=False)


def subset(wl: Workload, req_ids) -> Batch:
    """The batch restricted to ``req_ids`` (block ids unchanged)."""
    b = wl.batch
    paths, tails, news = [], [], []
    for r in req_ids:
        paths.append(b.path_nodes[b.path_ptr[r]:b.path_ptr[r + 1]])
        tails.append(b.tail_blocks[b.tail_ptr[r]:b.tail_ptr[r + 1]])
        news.append(int(b.new_lens[r]))
    return Batch(_i32(np.concatenate([[0], np.cumsum([len(p) for p in paths])])),
                 _i32(np.concatenate(paths) if paths else []),
                 _i32(news),
                 _i32(np.concatenate([[0], np.cumsum([len(t) for t in tails])])),
                 _i32(np.concatenate(tails) if tails else []))


# --------------------------------------------------------------------------- #
# tensors
# --------------------------------------------------------------------------- #
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even, torch's cast) -> uint16 bits."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    import torch
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16)
    return t.to(torch.float32).numpy()


def quantize_e4m3_per_block(x: np.ndarray) -> tuple:
    """x: [num_blocks, ...] fp32.  One fp32 scale per block: scale = amax/448
    (1.0 for an all-zero block), codes = e4m3fn(x/scale) via torch's cast."""
    import torch
    nb = x.shape[0]
    flat = np.ascontiguousarray(x, dtype=np.float32).reshape(nb, -1)
    amax = np.abs(flat).max(axis=1)
    scale = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
    y = np.clip(flat / scale[:, None], -448.0, 448.0).astype(np.float32)
    codes = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy().reshape(x.shape).copy()
    return codes, scale


@dataclasses.dataclass
class Tensors:
    """Host copies of everything the attention calls read.

    q        uint16 [total_q, Hq, D]  bf16 bits, requests concatenated in order
    q_ptr    int32  [R+1]
    k_pool   uint16 [nb, Hkv, B, D] (bf16) or uint8 (e4m3)
    v_pool   uint16 [nb, Hkv, D, B] (bf16) or uint8 (e4m3)
    k_scale, v_scale  float32 [nb] (fp8 only, else None)
    node_k/node_v, new_k/new_v: the *source* segments ([len, Hkv, D] fp32 values
    exactly representable in the pool format) kept for pool-free brute force.
    """
    q: np.ndarray
    q_ptr: np.ndarray
    k_pool: np.ndarray
    v_pool: np.ndarray
    k_scale: Optional[np.ndarray]
    v_scale: Optional[np.ndarray]
    node_k: Dict[int, np.ndarray]
    node_v: Dict[int, np.ndarray]
    new_k: List[np.ndarray]
    new_v: List[np.ndarray]


def _scatter_segment(k_pool, v_pool, blocks, seg_k, seg_v):
    """Copy a [len, Hkv, D] segment into its blocks (K token-major, V dim-major)."""
    n = seg_k.shape[0]
    for bi, blk in enumerate(blocks):
        lo = bi * BLOCK
        hi = min(lo + BLOCK, n)
        if hi <= lo:
            break
        k_pool[blk, :, : hi - lo, :] = np.transpose(seg_k[lo:hi], (1, 0, 2))
        v_pool[blk, :, :, : hi - lo] = np.transpose(seg_v[lo:hi], (1, 2, 0))


def make_tensors(wl: Workload, pad_std: float = 10.0, value_mode: str = "normal") -> Tensors:
    """Fill Q and the pool on the host with N(0,1) values (bf16-rounded), pad
    slots with N(0, pad_std^2) garbage.  ``value_mode='uniform_keys'`` makes all
    keys identical (closed-form tests)."""
    sh, g, b = wl.shape, wl.graph, wl.batch
    rng = np.random.default_rng([wl.seed, 7])
    hkv, d = sh.num_kv_heads, sh.head_dim
    nb = wl.num_pool_blocks
    kf = (rng.standard_normal((nb, hkv, BLOCK, d)) * pad_std).astype(np.float32)
    vf = (rng.standard_normal((nb, hkv, d, BLOCK)) * pad_std).astype(np.float32)
    const_key = rng.standard_normal((hkv, d)).astype(np.float32)

    def seg(n):
        k = rng.standard_normal((n, hkv, d)).astype(np.float32)
        v = rng.standard_normal((n, hkv, d)).astype(np.float32)
        if value_mode == "uniform_keys":
            k = np.broadcast_to(const_key, (n, hkv, d)).copy()
        return bf16_bits_to_f32(f32_to_bf16_bits(k)), bf16_bits_to_f32(f32_to_bf16_bits(v))

    node_k, node_v = {}, {}
    used = sorted(set(int(v) for v in b.path_nodes))
    for v in used:
        node_k[v], node_v[v] = seg(int(g.node_len[v]))
        _scatter_segment(kf, vf, g.node_blocks[g.node_block_ptr[v]:g.node_block_ptr[v + 1]],
                         node_k[v], node_v[v])
    new_k, new_v = [], []
    for r in range(b.num_req):
        k, v = seg(int(b.new_lens[r]))
        new_k.append(k)
        new_v.append(v)
        _scatter_segment(kf, vf, b.tail_blocks[b.tail_ptr[r]:b.tail_ptr[r + 1]], k, v)

    total_q = int(b.new_lens.sum())
    q = f32_to_bf16_bits(rng.standard_normal((total_q, sh.num_q_heads, d)).astype(np.float32))
    q_ptr = _i32(np.concatenate([[0], np.cumsum(b.new_lens)]))

    if sh.kv_dtype == KV_BF16:
        return Tensors(q, q_ptr, f32_to_bf16_bits(kf), f32_to_bf16_bits(vf), None, None,
                       node_k, node_v, new_k, new_v)
    kc, ks = quantize_e4m3_per_block(kf)
    vc, vs = quantize_e4m3_per_block(vf)
    # the pool-free brute force must see what the pool really stores: keep the
    # sources as None for fp8 (tests use the pool-aware oracle there)
    return Tensors(q, q_ptr, kc, vc, ks, vs, {}, {}, [], [])


# --------------------------------------------------------------------------- #
# prefix-conditioned node instances with sparse residuals (differential KV cache)
# --------------------------------------------------------------------------- #
@dataclasses.dataclass
class Residuals:
    """One item per pool block of every instance: copy block src to block dst and
    add the residual entries.  CSR with one row per (item, tensor, kv head):
    row (b*2 + t)*Hkv + h (t = 0 K, 1 V) holds res_idx/res_val[res_ptr[row]:
    res_ptr[row+1]], res_idx = slot*D + d inside that 16 x D image, bf16 bits."""
    src_blocks: np.ndarray   # int32 [items]
    dst_blocks: np.ndarray   # int32 [items]
    res_ptr: np.ndarray      # int32 [items * 2 * Hkv + 1]
    res_idx: np.ndarray      # uint16
    res_val: np.ndarray      # uint16

    @property
    def num_items(self) -> int:
        return int(self.src_blocks.shape[0])

    def bytes_moved(self, shape: Shape) -> float:
        """Algorithmic bytes of one application: base block read, reconstructed
        block written (K and V, all kv heads), entries (2 B index + 2 B value),
        8 B of block ids per item and 4 B of row pointer per image."""
        blk = 2 * shape.num_kv_heads * BLOCK * shape.head_dim * 2
        return (float(self.num_items) * (2 * blk + 8 + 4 * 2 * shape.num_kv_heads)
                + 4.0 * float(self.res_idx.shape[0]))


def add_residual_instances(wl: Workload, last_nodes: int = 1, density_k: float = 0.25, density_v: float = 0.30,
                           std: float = 0.3, seed: int = 11, by_prefix: bool = False) -> tuple:
    """Give every request private, prefix-conditioned instances of the last
    ``last_nodes`` nodes of its path: new node ids with their own (new) pool
    blocks, an edge from the predecessor, and a sparse residual against the
    original node's blocks (entries on valid token slots only; a share
    density_k / density_v of the K / V elements, values N(0, std^2) in bf16 --
    the paper reports that more than 75 % of key and 70 % of value entries of a
    prefix-induced difference are negligible).  Returns (workload', Residuals);
    the pool of the new workload is larger by the instance blocks, which hold
    nothing until the residuals are applied.  With by_prefix the instances belong to (prefix path, node) pairs
    instead of requests: requests that reach a node through the same prefix share one instance and its residual
    (the paper's KV(P, v)); the first node of a path, whose prefix is empty, then keeps its base KV."""
    rng = np.random.default_rng([wl.seed, seed])
    g, b, sh = wl.graph, wl.batch, wl.shape
    hkv, dim = sh.num_kv_heads, sh.head_dim
    node_len = list(g.node_len)
    node_blocks = [list(g.node_blocks[g.node_block_ptr[v]:g.node_block_ptr[v + 1]]) for v in range(g.num_nodes)]
    edges = [(v, int(d)) for v in range(g.num_nodes) for d in g.edge_dst[g.edge_ptr[v]:g.edge_ptr[v + 1]]]
    path_nodes = b.path_nodes.copy()
    next_block = wl.num_pool_blocks
    src, dst, ptr, idx, val = [], [], [0], [], []
    inst_of = {}
    for r in range(b.num_req):
        p0, p1 = int(b.path_ptr[r]), int(b.path_ptr[r + 1])
        for pos in range(max(p0 + (1 if by_prefix else 0), p1 - last_nodes), p1):
            v = int(path_nodes[pos])
            pair = tuple(int(x) for x in b.path_nodes[p0:pos + 1])
            if by_prefix and pair in inst_of:
                inst = inst_of[pair]
                if pos > p0:
                    edges.append((int(path_nodes[pos - 1]), inst))
                path_nodes[pos] = inst
                continue
            inst = len(node_len)
            inst_of[pair] = inst
            node_len.append(node_len[v])
            nb = _nblk(node_len[v])
            blocks = list(range(next_block, next_block + nb))
            next_block += nb
            node_blocks.append(blocks)
            if pos > p0:
                edges.append((int(path_nodes[pos - 1]), inst))
            if pos + 1 < p1:
                edges.append((inst, int(path_nodes[pos + 1])))
            path_nodes[pos] = inst
            for bi in range(nb):
                ntok = min(BLOCK, int(node_len[v]) - bi * BLOCK)
                src.append(node_blocks[v][bi])
                dst.append(blocks[bi])
                for t, dens in ((0, density_k), (1, density_v)):
                    for h in range(hkv):
                        m = rng.random((ntok, dim)) < dens
                        slot, d = np.nonzero(m)
                        e = (slot * dim + d).astype(np.uint16)
                        idx.append(e)
                        val.append(f32_to_bf16_bits((rng.standard_normal(e.size) * std).astype(np.float32)))
                        ptr.append(ptr[-1] + e.size)
    n = len(node_len)
    edge_ptr, edge_dst = edges_to_csr(n, sorted(set(edges)))
    nbp = np.concatenate([[0], np.cumsum([len(x) for x in node_blocks])])
    graph = WGraph(n, _i32(node_len), _i32(nbp), _i32([x for bl in node_blocks for x in bl]), edge_ptr, edge_dst)
    batch = Batch(b.path_ptr.copy(), _i32(path_nodes), b.new_lens.copy(), b.tail_ptr.copy(), b.tail_blocks.copy())
    wl2 = Workload(wl.name + "+residual", sh, graph, batch, next_block, wl.seed, wl.prefill_req.copy(),
                   wl.decode_req.copy(), wl.zipf_s)
    res = Residuals(_i32(src), _i32(dst), _i32(ptr),
                    np.concatenate(idx).astype(np.uint16) if idx else np.zeros(0, np.uint16),
                    np.concatenate(val).astype(np.uint16) if val else np.zeros(0, np.uint16))
    return wl2, res


def residual_handles(base_table: np.ndarray, inst_table: np.ndarray, res: Residuals) -> np.ndarray:
    """Per-table-entry residual handles for the read-time form: `base_table` is the block table resolved on the
    workload WITHOUT instances, `inst_table` the one resolved on add_residual_instances' workload (same shape: an
    instance has its base node's length).  Where the two differ the entry is an instance block, and its handle is
    the residual item that writes that block; -1 everywhere else."""
    item_of = {int(d): i for i, d in enumerate(res.dst_blocks)}
    h = np.full(base_table.shape, -1, np.int32)
    rr, ee = np.nonzero(base_table != inst_table)
    for r, e in zip(rr, ee):
        item = item_of[int(inst_table[r, e])]
        assert int(res.src_blocks[item]) == int(base_table[r, e])
        h[r, e] = item
    return h


def prefix_pair_handles(wl: Workload, req_lo: int, req_hi: int, max_blocks: int, depth: int = 1 << 30,
                        min_uses: int = 1) -> tuple:
    """Residual handles for requests [req_lo, req_hi) with one stored residual per (prefix path, node) pair -- the
    paper's KV(P, v): every node of a path beyond the first (at most the last ``depth`` of them) reads the
    residual of its pair; pairs are numbered as they are met and a pair's items (one per block of its node) are
    consecutive.  With ``min_uses`` > 1 only the pairs that at least so many of these requests walk keep a
    residual (what Effective Path Pruning leaves stored); the others read their node as it is.  Returns (handles
    int32 [req_hi - req_lo, max_blocks], number of items, number of pairs, number of (request, node) uses of a
    pair)."""
    g, b = wl.graph, wl.batch
    nbl = (g.node_len.astype(np.int64) + BLOCK - 1) // BLOCK
    handles = np.full((req_hi - req_lo, max_blocks), -1, np.int32)
    first_item, items, uses = {}, 0, 0
    walked = {}
    if min_uses > 1:
        for r in range(req_lo, req_hi):
            path = [int(v) for v in b.path_nodes[b.path_ptr[r]:b.path_ptr[r + 1]]]
            for i in range(1, len(path)):
                key = tuple(path[:i + 1])
                walked[key] = walked.get(key, 0) + 1
    for r in range(req_lo, req_hi):
        path = [int(v) for v in b.path_nodes[b.path_ptr[r]:b.path_ptr[r + 1]]]
        pos = 0
        for i, v in enumerate(path):
            n = int(nbl[v])
            key = tuple(path[:i + 1])
            if i >= 1 and i >= len(path) - depth and walked.get(key, min_uses) >= min_uses:
                if key not in first_item:
                    first_item[key] = items
                    items += n
                handles[r - req_lo, pos:pos + n] = first_item[key] + np.arange(n, dtype=np.int32)
                uses += 1
            pos += n
    return handles, items, len(first_item), uses


# --------------------------------------------------------------------------- #
# accounting (pure counting; used by bench and docs)
# --------------------------------------------------------------------------- #
def context_lens(wl: Workload) -> np.ndarray:
    b, g = wl.batch, wl.graph
    return np.array([int(g.node_len[b.path_nodes[b.path_ptr[r]:b.path_ptr[r + 1]]].sum())
                     for r in range(b.num_req)], dtype=np.int64)


def prefill_flops(wl: Workload, req_ids=None) -> float:
    """4*D*Hq * sum_r [ n_r*L_r + n_r(n_r+1)/2 ] over visible (row, key) pairs."""
    L = context_lens(wl)
    n = wl.batch.new_lens.astype(np.int64)
    ids = np.arange(wl.batch.num_req) if req_ids is None else np.asarray(req_ids)
    pairs = (n[ids] * L[ids] + n[ids] * (n[ids] + 1) // 2).sum()
    return 4.0 * wl.shape.head_dim * wl.shape.num_q_heads * float(pairs)


def decode_bytes(wl: Workload, req_ids=None) -> float:
    """Request-centric logical bytes of one decode call: K and V of every visible
    token, Q in, O out, 8 B of table per block (+8 B of scales per block, fp8)."""
    L = context_lens(wl)
    n = wl.batch.new_lens.astype(np.int64)
    ids = np.arange(wl.batch.num_req) if req_ids is None else np.asarray(req_ids)
    sh = wl.shape
    esz = 2 if sh.kv_dtype == KV_BF16 else 1
    g = wl.graph
    b = wl.batch
    nblk = 0
    for r in ids:
        nodes = b.path_nodes[b.path_ptr[r]:b.path_ptr[r + 1]]
        nblk += int(((g.node_len[nodes].astype(np.int64) + BLOCK - 1) // BLOCK).sum()) + _nblk(n[r])
    tok = float((L[ids] + n[ids]).sum())
    per_blk = 8 + (8 if sh.kv_dtype != KV_BF16 else 0)
    return (tok * 2 * sh.num_kv_heads * sh.head_dim * esz
            + 2.0 * len(ids) * sh.num_q_heads * sh.head_dim * 2 + nblk * per_blk)


def sharing_stats(wl: Workload) -> dict:
    """Sharing factor = sum_r L_r / unique context tokens touched."""
    L = context_lens(wl)
    used = np.unique(wl.batch.path_nodes)
    uniq = int(wl.graph.node_len[used].astype(np.int64).sum())
    sh = wl.shape
    esz = 2 if sh.kv_dtype == KV_BF16 else 1
    per_tok = 2 * sh.num_kv_heads * sh.head_dim * esz            # K and V bytes of one token, one layer
    tail = int(wl.batch.new_lens.astype(np.int64).sum())
    return {"sum_ctx_tokens": int(L.sum()), "unique_ctx_tokens": uniq,
            "sharing_factor": float(L.sum()) / max(uniq, 1),
            # what per-request (stateful) KV copies would hold vs what the shared pool holds for this batch
            "stateful_kv_bytes": float(L.sum() + tail) * per_tok,
            "shared_kv_bytes": float(uniq + tail) * per_tok}
