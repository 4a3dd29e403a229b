"""Device-side plumbing around the binding: upload a workload's index arrays,
allocate outputs, call the three entry points.  No arithmetic of the method
happens here; pools and queries are inputs (uploaded from the host generator or
filled by torch's device RNG for the large configurations)."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from . import workload as W


def bits_to_device(bits: np.ndarray, device) -> torch.Tensor:
    """uint16 bf16 bit patterns -> bf16 tensor; uint8 e4m3 codes -> uint8 tensor."""
    if bits.dtype == np.uint16:
        return torch.from_numpy(bits.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(bits).to(device)


def bf16_to_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


class DevicePool:
    """K/V pool resident on the GPU (+ per-block scales for e4m3)."""

    def __init__(self, k, v, num_blocks, k_scale=None, v_scale=None):
        self.k, self.v, self.k_scale, self.v_scale, self.num_blocks = k, v, k_scale, v_scale, num_blocks

    @classmethod
    def from_host(cls, t: W.Tensors, device):
        ks = None if t.k_scale is None else torch.from_numpy(t.k_scale).to(device)
        vs = None if t.v_scale is None else torch.from_numpy(t.v_scale).to(device)
        return cls(bits_to_device(t.k_pool, device), bits_to_device(t.v_pool, device), t.k_pool.shape[0], ks, vs)

    @classmethod
    def random(cls, wl: W.Workload, device, seed=None, chunk_blocks=1 << 14):
        """Fill the whole pool with N(0,1) on the device (pad slots included:
        finite garbage).  e4m3 pools are quantised per block: scale = amax/448."""
        sh = wl.shape
        nb, hkv, d = wl.num_pool_blocks, sh.num_kv_heads, sh.head_dim
        gen = torch.Generator(device=device)
        gen.manual_seed(wl.seed if seed is None else seed)
        fp8 = sh.kv_dtype == W.KV_FP8_E4M3
        dt = torch.uint8 if fp8 else torch.bfloat16
        k = torch.empty((nb, hkv, W.BLOCK, d), dtype=dt, device=device)
        v = torch.empty((nb, hkv, d, W.BLOCK), dtype=dt, device=device)
        ks = torch.empty(nb, dtype=torch.float32, device=device) if fp8 else None
        vs = torch.empty(nb, dtype=torch.float32, device=device) if fp8 else None
        for dst, sc in ((k, ks), (v, vs)):
            for lo in range(0, nb, chunk_blocks):
                hi = min(nb, lo + chunk_blocks)
                x = torch.randn((hi - lo,) + tuple(dst.shape[1:]), generator=gen, device=device,
                                dtype=torch.float32)
                if fp8:
                    amax = x.abs().amax(dim=(1, 2, 3))
                    s = torch.where(amax > 0, amax / 448.0, torch.ones_like(amax))
                    y = (x / s[:, None, None, None]).clamp_(-448.0, 448.0)
                    dst[lo:hi] = y.to(torch.float8_e4m3fn).view(torch.uint8)
                    sc[lo:hi] = s
                else:
                    dst[lo:hi] = x.to(torch.bfloat16)
                del x
        return cls(k, v, nb, ks, vs)

    def gather_host(self, block_ids: np.ndarray):
        """Copy the given blocks back to the host in the oracle's input format."""
        idx = torch.from_numpy(np.asarray(block_ids, dtype=np.int64)).to(self.k.device)
        kk, vv = self.k[idx], self.v[idx]
        if kk.dtype == torch.bfloat16:
            return bf16_to_bits(kk), bf16_to_bits(vv), None, None
        return (kk.cpu().numpy(), vv.cpu().numpy(), self.k_scale[idx].cpu().numpy(),
                self.v_scale[idx].cpu().numpy())


def random_residuals(shape: W.Shape, num_items: int, device, density_k=0.25, density_v=0.30, std=0.3, seed=1):
    """Synthetic residuals for `num_items` blocks, generated on the device: item b
    copies block b (source half of a pool of 2*num_items blocks) to block
    num_items + b and carries a random share of the K / V elements of every
    (tensor, kv head) image (N(0, std^2) values in bf16).  Returns the dict that
    Session.apply_residual takes, plus the number of entries."""
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    rows, img = 2 * shape.num_kv_heads, W.BLOCK * shape.head_dim      # images per block, elements per image
    thr = torch.cat([torch.full((shape.num_kv_heads, 1), density_k, device=device),
                     torch.full((shape.num_kv_heads, 1), density_v, device=device)])
    counts, idx_parts = [], []
    step = 512
    for lo in range(0, num_items, step):
        n = min(step, num_items - lo)
        m = torch.rand((n, rows, img), generator=gen, device=device) < thr
        counts.append(m.sum(dim=2, dtype=torch.int32).reshape(-1))
        idx_parts.append(m.nonzero()[:, 2].to(torch.int16))
        del m
    counts = torch.cat(counts)
    idx = torch.cat(idx_parts)
    ptr = torch.zeros(num_items * rows + 1, dtype=torch.int32, device=device)
    ptr[1:] = torch.cumsum(counts, 0)
    val = (torch.randn(idx.numel(), generator=gen, device=device) * std).to(torch.bfloat16).view(torch.int16)
    src = torch.randperm(num_items, generator=gen, device=device).to(torch.int32)
    dst = torch.arange(num_items, 2 * num_items, dtype=torch.int32, device=device)
    return dict(src=src, dst=dst, ptr=ptr, idx=idx, val=val, num_items=num_items,
                status=torch.full((num_items,), -77, dtype=torch.int32, device=device)), int(idx.numel())


class Session:
    """One gf_ctx + the device copies of a workload's graph."""

    def __init__(self, wl: W.Workload, device="cuda:0"):
        self.wl = wl
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.ctx = B.gf_create(self.device.index or 0)
        g = wl.graph
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(self.device)
        self.node_len, self.node_block_ptr, self.node_blocks = up(g.node_len), up(g.node_block_ptr), up(g.node_blocks)
        # a graph without edges still hands over an edge array (an empty tensor has no address)
        self.edge_ptr, self.edge_dst = up(g.edge_ptr), up(g.edge_dst if len(g.edge_dst) else [0])
        self._up = up

    def close(self):
        if self.ctx:
            B.gf_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def upload_batch(self, batch: W.Batch):
        up = self._up
        return dict(path_ptr=up(batch.path_ptr), path_nodes=up(batch.path_nodes if len(batch.path_nodes) else [0]),
                    new_lens=up(batch.new_lens), tail_ptr=up(batch.tail_ptr),
                    tail_blocks=up(batch.tail_blocks if len(batch.tail_blocks) else [0]), num_req=batch.num_req,
                    num_path_entries=int(len(batch.path_nodes)))

    def alloc_tables(self, num_req, max_blocks):
        z = lambda *s: torch.empty(s, dtype=torch.int32, device=self.device)
        return dict(block_table=z(num_req, max_blocks), block_ntok=z(num_req, max_blocks), num_blocks=z(num_req),
                    ctx_lens=z(num_req), seq_lens=z(num_req), status=z(num_req), num_req=num_req,
                    max_blocks=max_blocks)

    def resolve(self, dbatch, tables, with_edges=True, num_pool_blocks=None):
        graph = B.make_graph(self.wl.graph.num_nodes, self.node_len, self.node_block_ptr, self.node_blocks,
                             self.edge_ptr if with_edges else None, self.edge_dst if with_edges else None)
        B.gf_resolve_path(self.ctx, graph, dbatch["num_req"], dbatch["path_ptr"], dbatch["path_nodes"],
                          dbatch["new_lens"], dbatch["tail_ptr"], dbatch["tail_blocks"], tables["max_blocks"],
                          self.wl.num_pool_blocks if num_pool_blocks is None else num_pool_blocks,
                          tables["block_table"], tables["block_ntok"], tables["num_blocks"], tables["ctx_lens"],
                          tables["seq_lens"], tables["status"])
        return tables

    def _common(self, pool: DevicePool, tables, sm_scale):
        sh = self.wl.shape
        params = B.make_params(sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.kv_dtype, sm_scale)
        dpool = B.make_pool(pool.k, pool.v, pool.num_blocks, pool.k_scale, pool.v_scale)
        dt = B.make_tables(tables["block_table"], tables["block_ntok"], tables["num_blocks"], tables["ctx_lens"],
                           tables["seq_lens"], tables["status"], tables["num_req"], tables["max_blocks"])
        return params, dpool, dt

    def prefill(self, pool, tables, q, q_ptr, total_q, max_q, o, lse=None, sm_scale=0.0):
        params, dpool, dt = self._common(pool, tables, sm_scale)
        B.gf_attn_prefill(self.ctx, params, dpool, dt, q, q_ptr, total_q, max_q, o, lse)

    def prefill_noalloc(self, pool, tables, q, q_ptr, total_q, max_q, o, lse=None, sm_scale=0.0):
        """gf_attn_prefill with the work list in the library's fixed device array (nothing is allocated)."""
        params, dpool, dt = self._common(pool, tables, sm_scale)
        B.gf_attn_prefill_noalloc(self.ctx, params, dpool, dt, q, q_ptr, total_q, max_q, o, lse)

    def prefill_residual(self, pool, tables, res_handle, dres, q, q_ptr, total_q, max_q, o, lse=None, sm_scale=0.0):
        """Prefill with residuals applied as the blocks are read (`res_handle`, `dres` as in decode_residual)."""
        params, dpool, dt = self._common(pool, tables, sm_scale)
        B.gf_attn_prefill_residual(self.ctx, params, dpool, dt, res_handle, dres["num_items"], dres["ptr"],
                                   dres["idx"], dres["val"], q, q_ptr, total_q, max_q, o, lse)

    def upload_residuals(self, res: W.Residuals):
        dev = self.device
        i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
        idx = res.res_idx if res.res_idx.size else np.zeros(1, np.uint16)
        val = res.res_val if res.res_val.size else np.zeros(1, np.uint16)
        return dict(src=i32(res.src_blocks if res.num_items else [0]), dst=i32(res.dst_blocks if res.num_items else [0]),
                    ptr=i32(res.res_ptr), idx=torch.from_numpy(idx.view(np.int16)).to(dev),
                    val=torch.from_numpy(val.view(np.int16)).to(dev), num_items=res.num_items,
                    status=torch.full((max(res.num_items, 1),), -77, dtype=torch.int32, device=dev))

    def apply_residual(self, pool, dres):
        sh = self.wl.shape
        params = B.make_params(sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.kv_dtype)
        B.gf_kv_apply_residual(self.ctx, params, pool.k, pool.v, pool.num_blocks, dres["num_items"], dres["src"],
                               dres["dst"], dres["ptr"], dres["idx"], dres["val"], dres["status"], pool.k_scale,
                               pool.v_scale)

    def pack_residuals(self, dres):
        """gf_kv_residual_pack: the packed form (bit masks + values in element order) of an uploaded residual;
        returns the dict with `mask` and `pval` added (and a status of its own under `pack_status`)."""
        sh = self.wl.shape
        n = dres["num_items"]
        rows = n * 2 * sh.num_kv_heads
        words = W.BLOCK * sh.head_dim // 32
        out = dict(dres)
        out["mask"] = torch.full((max(rows, 1), words), -1, dtype=torch.int32, device=self.device)
        out["pval"] = torch.zeros_like(dres["val"])
        out["pack_status"] = torch.full((max(n, 1),), -77, dtype=torch.int32, device=self.device)
        params = B.make_params(sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.kv_dtype)
        B.gf_kv_residual_pack(self.ctx, params, n, dres["ptr"], dres["idx"], dres["val"], out["mask"], out["pval"],
                              out["pack_status"])
        return out

    def unpack_residuals(self, packed):
        """gf_kv_residual_unpack: element indices (rising inside a row) of a packed residual."""
        sh = self.wl.shape
        idx = torch.full_like(packed["idx"], -1)
        status = torch.full((max(packed["num_items"], 1),), -77, dtype=torch.int32, device=self.device)
        params = B.make_params(sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.kv_dtype)
        B.gf_kv_residual_unpack(self.ctx, params, packed["num_items"], packed["ptr"], packed["mask"], idx, status)
        return idx, status

    def apply_residual_packed(self, pool, packed):
        sh = self.wl.shape
        params = B.make_params(sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.kv_dtype)
        B.gf_kv_apply_residual_packed(self.ctx, params, pool.k, pool.v, pool.num_blocks, packed["num_items"],
                                      packed["src"], packed["dst"], packed["ptr"], packed["mask"], packed["pval"],
                                      packed["status"])

    def make_residual(self, pool, base_blocks, full_blocks, share=0.95, capacity=None):
        """gf_kv_make_residual: the residual of blocks `full_blocks` against `base_blocks` (device int32 tensors) as
        the dict apply_residual / decode_residual take (src = base, dst = full), plus the number of entries."""
        sh = self.wl.shape
        n = int(base_blocks.numel())
        rows = n * 2 * sh.num_kv_heads
        if capacity is None:
            capacity = rows * W.BLOCK * sh.head_dim
        dev = self.device
        ptr = torch.full((rows + 1,), -77, dtype=torch.int32, device=dev)
        idx = torch.zeros(max(capacity, 1), dtype=torch.int16, device=dev)
        val = torch.zeros(max(capacity, 1), dtype=torch.int16, device=dev)
        status = torch.full((max(n, 1),), -77, dtype=torch.int32, device=dev)
        params = B.make_params(sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.kv_dtype)
        B.gf_kv_make_residual(self.ctx, params, pool.k, pool.v, pool.num_blocks, n, base_blocks, full_blocks, share,
                              capacity, ptr, idx, val, status)
        return dict(src=base_blocks, dst=full_blocks, ptr=ptr, idx=idx, val=val, num_items=n, status=status)

    def append(self, pool, tables, k_new, v_new, q_ptr, total_q, max_q):
        params, _, dt = self._common(pool, tables, 0.0)
        B.gf_kv_append(self.ctx, params, pool.k, pool.v, pool.k_scale, pool.v_scale, pool.num_blocks, dt, k_new,
                       v_new, q_ptr, total_q, max_q)

    def append_token(self, pool, tables, k_tok, v_tok):
        params, _, dt = self._common(pool, tables, 0.0)
        B.gf_kv_append_token(self.ctx, params, pool.k, pool.v, pool.k_scale, pool.v_scale, pool.num_blocks, dt, k_tok,
                             v_tok)

    def decode(self, pool, tables, q, o, lse=None, sm_scale=0.0):
        params, dpool, dt = self._common(pool, tables, sm_scale)
        B.gf_attn_decode(self.ctx, params, dpool, dt, q, o, lse)

    def decode_residual(self, pool, tables, res_handle, dres, q, o, lse=None, sm_scale=0.0):
        """Decode with residuals applied as the blocks are read: `res_handle` [R, max_blocks] int32 names, per table
        entry, an item of the uploaded residual `dres` (upload_residual) or -1."""
        params, dpool, dt = self._common(pool, tables, sm_scale)
        B.gf_attn_decode_residual(self.ctx, params, dpool, dt, res_handle, dres["num_items"], dres["ptr"], dres["idx"],
                                  dres["val"], q, o, lse)

    def decode_shared(self, pool, dbatch, tables, q, o, lse=None, sm_scale=0.0):
        """Node-centric decode; `dbatch` is the uploaded batch `tables` was resolved from."""
        params, dpool, dt = self._common(pool, tables, sm_scale)
        graph = B.make_graph(self.wl.graph.num_nodes, self.node_len, self.node_block_ptr, self.node_blocks)
        B.gf_attn_decode_shared(self.ctx, params, dpool, graph, dbatch["path_ptr"], dbatch["path_nodes"],
                                dbatch["num_path_entries"], dt, q, o, lse)

    def decode_shared_residual(self, pool, dbatch, tables, res_handle, dres, q, o, lse=None, sm_scale=0.0):
        """Node-centric decode with residuals applied as the blocks are read (`res_handle`, `dres` as in
        decode_residual; a node's first handle names the residual of the whole node)."""
        params, dpool, dt = self._common(pool, tables, sm_scale)
        graph = B.make_graph(self.wl.graph.num_nodes, self.node_len, self.node_block_ptr, self.node_blocks)
        B.gf_attn_decode_shared_residual(self.ctx, params, dpool, graph, dbatch["path_ptr"], dbatch["path_nodes"],
                                         dbatch["num_path_entries"], dt, res_handle, dres["num_items"], dres["ptr"],
                                         dres["idx"], dres["val"], q, o, lse)

    def decode_shared_plan(self, pool, dbatch, tables):
        """Build the node lists of a batch once; decode_shared_planned() then runs any number of layers on them."""
        params, _, dt = self._common(pool, tables, 0.0)
        graph = B.make_graph(self.wl.graph.num_nodes, self.node_len, self.node_block_ptr, self.node_blocks)
        B.gf_decode_shared_plan(self.ctx, params, graph, dbatch["path_ptr"], dbatch["path_nodes"],
                                dbatch["num_path_entries"], dt)

    def decode_shared_planned(self, pool, dbatch, tables, q, o, lse=None, sm_scale=0.0):
        params, dpool, dt = self._common(pool, tables, sm_scale)
        graph = B.make_graph(self.wl.graph.num_nodes, self.node_len, self.node_block_ptr, self.node_blocks)
        B.gf_attn_decode_shared_planned(self.ctx, params, dpool, graph, dbatch["path_ptr"], dbatch["path_nodes"],
                                        dbatch["num_path_entries"], dt, q, o, lse)


class ResidualDirectory:
    """Device arrays of a gf_residual_dir plus the execution statistics (one counter per edge of the graph)."""

    def __init__(self, sess: "Session", capacity: int):
        assert capacity & (capacity - 1) == 0
        dev = sess.device
        self.sess, self.capacity = sess, capacity
        n = max(capacity, 1)
        self.key = torch.empty(n, dtype=torch.int64, device=dev)
        self.prev, self.node, self.first_item, self.uses = (torch.empty(n, dtype=torch.int32, device=dev) for _ in range(4))
        self.trans_count = torch.zeros(max(int(sess.edge_dst.numel()), 1), dtype=torch.int32, device=dev)
        self.pruned = torch.zeros(2, dtype=torch.int32, device=dev)
        B.gf_residual_dir_clear(sess.ctx, self.struct())

    def struct(self):
        return B.make_residual_dir(self.key, self.prev, self.node, self.first_item, self.uses, self.capacity)

    def insert(self, prefixes, first_items):
        """prefixes: host lists of node ids (each of length >= 2); first_items: the pairs' first residual items."""
        dev = self.sess.device
        keys = np.array([B.gf_prefix_key(p) for p in prefixes], dtype=np.uint64)
        i32 = lambda a: torch.from_numpy(np.asarray(a, dtype=np.int32)).to(dev)
        status = torch.full((len(prefixes),), -77, dtype=torch.int32, device=dev)
        B.gf_residual_dir_insert(self.sess.ctx, self.struct(), len(prefixes),
                                 torch.from_numpy(keys.view(np.int64)).to(dev), i32([p[-2] for p in prefixes]),
                                 i32([p[-1] for p in prefixes]), i32(first_items), status)
        return status

    def resolve(self, dbatch, tables, count=True):
        """gf_resolve_path_residual: fills `tables` and returns (res_handle [R, max_blocks], num_fallback [R])."""
        sess = self.sess
        graph = B.make_graph(sess.wl.graph.num_nodes, sess.node_len, sess.node_block_ptr, sess.node_blocks,
                             sess.edge_ptr, sess.edge_dst)
        R_, mb = dbatch["num_req"], tables["max_blocks"]
        handle = torch.full((R_, mb), -77, dtype=torch.int32, device=sess.device)
        fallback = torch.full((R_,), -77, dtype=torch.int32, device=sess.device)
        B.gf_resolve_path_residual(sess.ctx, graph, R_, dbatch["path_ptr"], dbatch["path_nodes"], dbatch["new_lens"],
                                   dbatch["tail_ptr"], dbatch["tail_blocks"], mb, sess.wl.num_pool_blocks,
                                   tables["block_table"], tables["block_ntok"], tables["num_blocks"],
                                   tables["ctx_lens"], tables["seq_lens"], tables["status"], self.struct(),
                                   self.trans_count if count else None, handle, fallback)
        return handle, fallback

    def prune(self, min_count):
        sess = self.sess
        graph = B.make_graph(sess.wl.graph.num_nodes, sess.node_len, sess.node_block_ptr, sess.node_blocks,
                             sess.edge_ptr, sess.edge_dst)
        B.gf_residual_dir_prune(sess.ctx, graph, self.struct(), self.trans_count, min_count, self.pruned)


def tables_to_host(tables) -> dict:
    """Device tables -> dict of Python lists (the oracle resolver's format)."""
    out = {}
    for k in ("block_table", "block_ntok", "num_blocks", "ctx_lens", "seq_lens", "status"):
        out[k] = tables[k].cpu().numpy().tolist()
    return out
