#!/usr/bin/env python3
"""Benchmark of the graph-KV attention hot path on one MI355X.

One "step" is one pass of the whole path over one batch of a synthetic wGraph
workload: gf_resolve_path -> gf_attn_prefill (requests with new tokens) ->
gf_attn_decode (one decode step for the decode requests; for a prefill-only
workload, the step after prefill: every request decodes with its last token),
split-KV merge included.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line.  `value` is the headline metric of the chosen workload
over the whole step; `roofline` describes the dominant kernel, timed live with
HIP events on the launch stream; `cpu_baseline` is the fp64 oracle timed on the
host cores on a bounded sample of the same workload (and used to check the GPU
outputs of that sample); `extra` carries the other workloads' figures.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E


def _event_ms(fn, torch, iters):
    """Average duration of fn() in ms with HIP events on the current stream."""
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s.record()
    for _ in range(iters):
        fn()
    e.record()
    e.synchronize()
    return s.elapsed_time(e) / iters


def _event_median_ms(fn, torch, iters, before=None):
    """Median over `iters` launches of fn(), each between its own pair of HIP events; `before()` runs ahead of
    every launch outside the timed pair (a cache flush, for a cold figure)."""
    times = []
    for _ in range(iters):
        if before is not None:
            before()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        fn()
        e.record()
        e.synchronize()
        times.append(s.elapsed_time(e))
    return float(np.median(times))


def _read_traffic(name):
    """HBM bytes per launch of a kernel (read + written) from the rocprofv3 --pmc summary kept under
    profiles/ (TCC request counters at the memory side of L2, summed over channels: 32-byte DRAM read and
    write requests x 32; no calibration factor), or None.  The file names the command that produced it."""
    p = os.path.join(ROOT, "profiles", f"{name}_traffic.txt")
    if not os.path.exists(p):
        return None
    vals = {}
    for line in open(p):
        if "=" in line and not line.lstrip().startswith("#"):
            k, v = line.split("=", 1)
            try:
                vals[k.strip()] = float(v.split()[0])
            except ValueError:
                pass
    if "DRAM_READ_BYTES_PER_LAUNCH" in vals and "DRAM_WRITE_BYTES_PER_LAUNCH" in vals:
        return vals["DRAM_READ_BYTES_PER_LAUNCH"] + vals["DRAM_WRITE_BYTES_PER_LAUNCH"]
    return None


def hbm_roofline(kernel, alg_bytes, ms, traffic, logical_bytes=None, unique_bytes=None):
    """Roofline object of a bandwidth-bound kernel.  `achieved` counts only bytes that must cross the HBM pins:
    the algorithmic bytes where nothing is shared between the kernel's work items (then they equal the unique
    bytes), else the unique bytes the launch touches -- a lower bound, since a block shared by several requests
    may be served from L2 or the Infinity Cache after its first read.  Request-centric logical bytes are a
    rate, never a fraction; `traffic` is what the counters saw leaving L2 (requests to the memory fabric, which
    the Infinity Cache may still serve), also a rate."""
    sec = ms * 1e-3
    shared = logical_bytes is not None
    nbytes = unique_bytes if shared else alg_bytes
    out = {"bound": "hbm", "kernel": kernel, "achieved": nbytes / sec / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
           "frac": nbytes / sec / 1e9 / PEAK_HBM_GBS, "traffic": traffic, "kernel_ms": ms,
           "bytes_basis": "unique bytes touched (lower bound of the HBM traffic; shared blocks are re-read from cache)"
           if shared else "algorithmic bytes (nothing shared: equal to the unique bytes)",
           "algorithmic_bytes_per_launch": alg_bytes}
    if traffic is not None:
        out["l2_fabric_gbs"] = traffic / sec / 1e9              # L2 misses; the Infinity Cache serves part of them
    if shared:
        out["logical_gbs"] = logical_bytes / sec / 1e9          # request-centric rate, cache hits included
        out["unique_bytes"] = unique_bytes
    return out


class Job:
    """A workload set up on the device: tables, pool, queries, outputs."""

    def __init__(self, name, torch, R, W, decode_after_prefill=True):
        self.torch, self.R, self.W = torch, R, W
        self.wl = wl = (W.CONFIGS.get(name) or W.MEASUREMENT_CONFIGS[name])()
        self.name = name
        dev = torch.device("cuda:0")
        self.sess = R.Session(wl, dev)
        b = wl.batch
        self.dbatch = self.sess.upload_batch(b)
        g = wl.graph
        nbl = ((g.node_len.astype(np.int64) + 15) // 16)
        self.max_blocks = int(max(int(nbl[b.path_nodes[b.path_ptr[r]:b.path_ptr[r + 1]]].sum())
                                  + (int(b.new_lens[r]) + 15) // 16 for r in range(b.num_req)))
        self.tables = self.sess.alloc_tables(b.num_req, self.max_blocks)
        self.pool = R.DevicePool.random(wl, dev)
        sh = wl.shape
        gen = torch.Generator(device=dev)
        gen.manual_seed(wl.seed + 1)
        self.total_q = int(b.new_lens.sum())
        self.max_q = int(b.new_lens.max())
        self.q = torch.randn((self.total_q, sh.num_q_heads, sh.head_dim), generator=gen, device=dev,
                             dtype=torch.float32).to(torch.bfloat16)
        self.q_ptr = torch.from_numpy(np.concatenate([[0], np.cumsum(b.new_lens)]).astype(np.int32)).to(dev)
        self.o = torch.zeros_like(self.q)
        self.has_prefill = len(wl.prefill_req) > 0
        self.has_decode = len(wl.decode_req) > 0 or decode_after_prefill
        # decode queries: the last new token of every request
        last = torch.from_numpy((np.cumsum(b.new_lens) - 1).astype(np.int64)).to(dev)
        self.qd = self.q[last].contiguous()
        self.od = torch.zeros_like(self.qd)
        self.od_shared = torch.zeros_like(self.qd)
        self.last = last
        # request classes: the generator puts the prefill requests first.  A prefill-only workload
        # decodes all its requests after prefill; a mixed batch prefills [0, P) and decodes [P, R).
        P = len(wl.prefill_req)
        Rn = b.num_req
        self.pf_rng = (0, P)
        self.dec_rng = (P, Rn) if len(wl.decode_req) > 0 else (0, Rn)
        self.pf_rows = int(b.new_lens[:P].sum())
        self.pf_max_q = int(b.new_lens[:P].max()) if P else 0
        # K/V of the new tokens, as the write path receives them
        self.k_new = torch.randn((self.total_q, sh.num_kv_heads, sh.head_dim), generator=gen, device=dev,
                                 dtype=torch.float32).to(torch.bfloat16)
        self.v_new = torch.randn((self.total_q, sh.num_kv_heads, sh.head_dim), generator=gen, device=dev,
                                 dtype=torch.float32).to(torch.bfloat16)
        self.resolve()
        self.append()          # the tail blocks hold the new tokens' K/V from here on (every later call rewrites the same)
        torch.cuda.synchronize()

    def _slice(self, lo, hi):
        t = self.tables
        out = {k: t[k][lo:hi] for k in ("block_table", "block_ntok", "num_blocks", "ctx_lens", "seq_lens", "status")}
        out["num_req"], out["max_blocks"] = hi - lo, t["max_blocks"]
        return out

    def resolve(self):
        self.sess.resolve(self.dbatch, self.tables)

    def prefill(self):
        lo, hi = self.pf_rng
        self.sess.prefill(self.pool, self._slice(lo, hi), self.q, self.q_ptr[lo:hi + 1], self.pf_rows,
                          self.pf_max_q, self.o)

    def append(self):
        self.sess.append(self.pool, self.tables, self.k_new, self.v_new, self.q_ptr, self.total_q, self.max_q)

    def append_token(self):
        """The decode-step write: every request's newest token once more (same bits, same slot)."""
        if not hasattr(self, "k_tok"):
            self.k_tok = self.k_new[self.last].contiguous()
            self.v_tok = self.v_new[self.last].contiguous()
        self.sess.append_token(self.pool, self.tables, self.k_tok, self.v_tok)

    def append_bytes(self):
        sh = self.wl.shape
        esz = 2 if sh.kv_dtype == self.W.KV_BF16 else 1
        per_tok = 2 * sh.num_kv_heads * sh.head_dim
        nblk = int(((self.wl.batch.new_lens.astype(np.int64) + 15) // 16).sum())
        # new K/V read once (bf16), tail blocks written whole (pad slots included), 4 B of table per block
        return float(self.total_q) * per_tok * 2 + float(nblk) * 16 * per_tok * esz + 4.0 * nblk

    def decode(self):
        lo, hi = self.dec_rng
        self.sess.decode(self.pool, self._slice(lo, hi), self.qd[lo:hi], self.od[lo:hi])

    def decode_shared(self):
        """The same decode step through the node-centric entry point."""
        lo, hi = self.dec_rng
        db = dict(self.dbatch)
        db["path_ptr"] = self.dbatch["path_ptr"][lo:hi + 1]
        self.sess.decode_shared(self.pool, db, self._slice(lo, hi), self.qd[lo:hi], self.od_shared[lo:hi])

    def _shared_args(self):
        lo, hi = self.dec_rng
        if not hasattr(self, "_shared_db"):
            self._shared_db = dict(self.dbatch)
            self._shared_db["path_ptr"] = self.dbatch["path_ptr"][lo:hi + 1]
            self._shared_tables = self._slice(lo, hi)
        return lo, hi

    def decode_shared_plan(self):
        """List building alone (once per batch and model step; every layer shares it)."""
        self._shared_args()
        self.sess.decode_shared_plan(self.pool, self._shared_db, self._shared_tables)

    def decode_shared_planned(self):
        """Attention + merge over lists built before (what one layer costs)."""
        lo, hi = self._shared_args()
        self.sess.decode_shared_planned(self.pool, self._shared_db, self._shared_tables, self.qd[lo:hi],
                                        self.od_shared[lo:hi])

    def decode_shared_bytes(self, chunk_blocks=64):
        """What the node-centric decode has to move: every node the decode requests touch once, their
        tails, one fp32 partial (max, sum, values) per (request, path node, chunk) written and read
        back, the block lists, q and o."""
        wl, sh = self.wl, self.wl.shape
        b, g = wl.batch, wl.graph
        lo, hi = self.dec_rng
        esz = 2 if sh.kv_dtype == self.W.KV_BF16 else 1
        per_blk = 2 * sh.num_kv_heads * 16 * sh.head_dim * esz + (8 if esz == 1 else 0)
        nbl = (g.node_len.astype(np.int64) + 15) // 16
        nodes = b.path_nodes[b.path_ptr[lo]:b.path_ptr[hi]]
        tail_blk = (b.new_lens[lo:hi].astype(np.int64) + 15) // 16
        uniq_blocks = int(nbl[np.unique(nodes)].sum()) + int(tail_blk.sum())
        slots = int(((nbl[nodes] + chunk_blocks - 1) // chunk_blocks).sum()) \
            + int(((tail_blk + chunk_blocks - 1) // chunk_blocks).sum())
        partial = slots * sh.num_q_heads * (sh.head_dim + 2) * 4
        qo = 2 * (hi - lo) * sh.num_q_heads * sh.head_dim * 2
        return {"unique_blocks": uniq_blocks, "partial_slots": slots,
                "bytes": float(uniq_blocks) * (per_blk + 4) + 2.0 * partial + qo}

    def step(self):
        self.resolve()
        if self.has_prefill:
            self.prefill()
        if self.has_decode:
            self.decode()

    # ---- algorithmic work -------------------------------------------------------
    def prefill_flops(self):
        return self.W.prefill_flops(self.wl, np.arange(*self.pf_rng)) if self.has_prefill else 0.0

    def decode_bytes(self):
        return self.W.decode_bytes(self.wl, np.arange(*self.dec_rng))


def measure(job, steps, warmup):
    torch = job.torch
    for _ in range(warmup):
        job.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        job.step()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / steps
    out = {"ms_per_step": ms_step}
    it = max(steps, 5)
    out["resolve_ms"] = _event_ms(job.resolve, torch, it)
    if job.has_prefill:
        out["prefill_ms"] = _event_ms(job.prefill, torch, it)
        out["prefill_tflops_kernel"] = job.prefill_flops() / (out["prefill_ms"] * 1e-3) / 1e12
        out["prefill_median_ms"] = _event_median_ms(job.prefill, torch, max(it, 20))
        # cold: L2 and the 256 MB Infinity Cache are overwritten by a 1 GiB fill before every launch
        flush = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0")
        out["prefill_cold_median_ms"] = _event_median_ms(job.prefill, torch, 7, before=lambda: flush.fill_(1.0))
        del flush
    if job.has_decode:
        out["decode_ms"] = _event_ms(job.decode, torch, it)
        out["decode_gbs_kernel"] = job.decode_bytes() / (out["decode_ms"] * 1e-3) / 1e9
        out["decode_median_ms"] = _event_median_ms(job.decode, torch, max(it, 20))
        # the same step computed node by node (shared KV read once per group of requests)
        job.decode()
        job.decode_shared()
        torch.cuda.synchronize()
        out["decode_shared_max_abs_diff"] = float((job.od.float() - job.od_shared.float()).abs().max().item())
        out["decode_shared_ms"] = _event_ms(job.decode_shared, torch, it)
        out["decode_shared_plan_ms"] = _event_ms(job.decode_shared_plan, torch, it)
        out["decode_shared_planned_ms"] = _event_ms(job.decode_shared_planned, torch, it)   # after a plan call
    # the write path (not part of the step): it rewrites the tail blocks with the same new-token K/V every time
    out["append_ms"] = _event_ms(job.append, torch, it)
    out["append_gbs_kernel"] = job.append_bytes() / (out["append_ms"] * 1e-3) / 1e9
    out["append_token_ms"] = _event_ms(job.append_token, torch, it)
    return out


def decode_shared_entry(job, m):
    """Figures of gf_attn_decode_shared beside gf_attn_decode on the same decode step."""
    alg = job.decode_shared_bytes()
    sec = m["decode_shared_ms"] * 1e-3
    return {"kernel": "shared_attn_kernel(+list building, merge)", "kernel_ms": m["decode_shared_ms"],
            "speedup_over_decode": m["decode_ms"] / m["decode_shared_ms"],
            # the two halves on their own: the lists depend on the batch only, a model builds them once per step
            "plan_ms": m["decode_shared_plan_ms"], "planned_ms": m["decode_shared_planned_ms"],
            "speedup_over_decode_planned": m["decode_ms"] / m["decode_shared_planned_ms"],
            "max_abs_diff_to_decode": m["decode_shared_max_abs_diff"],
            # the per-request kernel's bytes over this call's time: what the sharing is worth, not an HBM rate
            "per_request_bytes_rate_gbs": job.decode_bytes() / sec / 1e9,
            "algorithmic_bytes_per_launch": alg["bytes"], "unique_blocks": alg["unique_blocks"],
            "partial_slots": alg["partial_slots"], "gbs_kernel": alg["bytes"] / sec / 1e9,
            # every block is read once by design, so these algorithmic bytes are HBM bytes: a true fraction
            "frac_of_hbm_peak": alg["bytes"] / sec / 1e9 / PEAK_HBM_GBS,
            "frac_of_hbm_peak_planned": alg["bytes"] / (m["decode_shared_planned_ms"] * 1e-3) / 1e9 / PEAK_HBM_GBS,
            "hbm_bytes_per_launch_rocprof": _read_traffic(f"decode_shared_{job.name}")}


def measure_decode_residual(job, decode_ms, share=0.25, density=(0.25, 0.30), iters=20):
    """gf_attn_decode_residual beside gf_attn_decode on the same decode step: the last `share` of every request's
    table entries are read as base block + a residual item of their own (25 % of the K and 30 % of the V elements,
    the density the paper reports), the pool holding base blocks only.  bf16 pools."""
    torch, R, W = job.torch, job.R, job.W
    sh = job.wl.shape
    if sh.kv_dtype != W.KV_BF16:
        return None
    lo, hi = job.dec_rng
    t = job._slice(lo, hi)
    dev = job.qd.device
    nb = t["num_blocks"].to(torch.int64)
    first = nb - (nb.to(torch.float64) * share).to(torch.int64)
    ar = torch.arange(job.max_blocks, device=dev)[None, :]
    mask = (ar >= first[:, None]) & (ar < nb[:, None])
    num_items = int(mask.sum().item())
    handles = torch.full(mask.shape, -1, dtype=torch.int32, device=dev)
    handles[mask] = torch.arange(num_items, dtype=torch.int32, device=dev)
    dres, nnz = R.random_residuals(sh, num_items, dev, density_k=density[0], density_v=density[1])
    o = torch.zeros_like(job.od[lo:hi])
    fn = lambda: job.sess.decode_residual(job.pool, t, handles, dres, job.qd[lo:hi], o)
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    ms = _event_ms(fn, torch, iters)
    changed = float((o.float() - job.od[lo:hi].float()).abs().max().item())
    blk = 2 * sh.num_kv_heads * W.BLOCK * sh.head_dim * 2
    nbytes = job.decode_bytes() + 4.0 * nnz + 4.0 * handles.numel() + 4.0 * 2 * sh.num_kv_heads * num_items
    return {"kernel": "decode_split_kernel<RES>(+merge)", "kernel_ms": ms, "decode_ms": decode_ms,
            "slowdown_over_decode": ms / decode_ms, "entries_with_residual": num_items,
            "share_of_table_entries": num_items / max(1.0, float(nb.sum().item())), "residual_entries": nnz,
            "density_k_v": list(density),
            # request-centric bytes (shared blocks counted once per request) + the residual's own: a rate, cache
            # hits included, not an HBM fraction
            "logical_bytes_per_launch": nbytes, "logical_gbs": nbytes / (ms * 1e-3) / 1e9,
            # what the pool does not hold: the reconstructed copies of these blocks, against the sparse form kept
            "dense_instance_bytes": float(num_items) * blk, "sparse_residual_bytes": 4.0 * nnz,
            "max_abs_diff_to_base_decode": changed}


def measure_prefill_residual(job, prefill_ms, shares=(0.25, 1.0), density=(0.25, 0.30), iters=10):
    """gf_attn_prefill_residual beside gf_attn_prefill on the same prefill: the last `share` of every request's
    CONTEXT entries (ancestor blocks; the new tokens' own blocks carry none) are read as base block + a residual
    item of their own at the density the paper reports.  share 1 is the paper's regime: every ancestor block under
    a prefix has a residual.  bf16 pools."""
    torch, R, W = job.torch, job.R, job.W
    sh = job.wl.shape
    if sh.kv_dtype != W.KV_BF16 or not job.has_prefill:
        return None
    lo, hi = job.pf_rng
    t = job._slice(lo, hi)
    dev = job.q.device
    nb = t["num_blocks"].to(torch.int64)
    new = (t["seq_lens"] - t["ctx_lens"]).to(torch.int64)
    ncb = nb - (new + 15) // 16                       # context entries
    ar = torch.arange(job.max_blocks, device=dev)[None, :]
    o = torch.zeros_like(job.o)
    out = {"kernel": "prefill_kernel<RES>", "prefill_ms": prefill_ms, "density_k_v": list(density), "runs": []}
    for share in shares:
        first = ncb - (ncb.to(torch.float64) * share).to(torch.int64)
        mask = (ar >= first[:, None]) & (ar < ncb[:, None])
        num_items = int(mask.sum().item())
        handles = torch.full(mask.shape, -1, dtype=torch.int32, device=dev)
        handles[mask] = torch.arange(num_items, dtype=torch.int32, device=dev)
        dres, nnz = R.random_residuals(sh, num_items, dev, density_k=density[0], density_v=density[1])
        fn = lambda: job.sess.prefill_residual(job.pool, t, handles, dres, job.q, job.q_ptr[lo:hi + 1], job.pf_rows,
                                               job.pf_max_q, o)
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        ms = _event_ms(fn, torch, iters)
        out["runs"].append({"share_of_context_entries": share, "entries_with_residual": num_items,
                            "residual_entries": nnz, "kernel_ms": ms, "slowdown_over_prefill": ms / prefill_ms,
                            "tflops": job.prefill_flops() / (ms * 1e-3) / 1e12,
                            "max_abs_diff_to_base_prefill": float((o.float() - job.o.float()).abs().max().item())})
        del dres, handles
    return out


def measure_shared_residual(job, m, density=(0.25, 0.30), iters=10):
    """gf_attn_decode_shared_residual on the decode step with one stored residual per (prefix path, node) pair of
    the batch, beside the per-request read-time form on the same handles and the plain node-centric step.  Two
    regimes: every pair keeps its residual (every node beyond the first of a path is read as base + residual;
    requests that reach a node through the same prefix share one read of it), and only the pairs that at least two
    requests of the batch walk keep one (what Effective Path Pruning leaves stored; the others read the node as it
    is, standing in for the dense blocks an on-the-fly fallback leaves).  bf16 pools."""
    torch, R, W = job.torch, job.R, job.W
    sh = job.wl.shape
    if sh.kv_dtype != W.KV_BF16 or not job.has_decode:
        return None
    lo, hi = job._shared_args()
    t = job._shared_tables
    dev = job.qd.device
    out = {"kernel": "shared_attn_kernel<RES>(+list building, merge)", "plain_node_centric_ms": m["decode_shared_ms"],
           "density_k_v": list(density), "runs": []}
    for regime, min_uses in (("every pair", 1), ("pairs walked by two requests or more", 2)):
        handles_h, num_items, pairs, uses = W.prefix_pair_handles(job.wl, lo, hi, job.max_blocks, min_uses=min_uses)
        handles = torch.from_numpy(handles_h).to(dev)
        dres, nnz = R.random_residuals(sh, num_items, dev, density_k=density[0], density_v=density[1])
        o = torch.zeros_like(job.od[lo:hi])
        o_req = torch.zeros_like(o)
        fn = lambda: job.sess.decode_shared_residual(job.pool, job._shared_db, t, handles, dres, job.qd[lo:hi], o)
        fn_req = lambda: job.sess.decode_residual(job.pool, t, handles, dres, job.qd[lo:hi], o_req)
        for f in (fn, fn_req):
            f()
        torch.cuda.synchronize()
        ms, ms_req = _event_ms(fn, torch, iters), _event_ms(fn_req, torch, iters)
        out["runs"].append({"pairs_with_residual": regime, "kernel_ms": ms, "per_request_read_time_ms": ms_req,
                            "speedup_over_per_request_read_time": ms_req / ms, "prefix_node_pairs": pairs,
                            "request_node_uses": uses, "residual_items": num_items, "residual_entries": nnz,
                            "sparse_residual_bytes": 4.0 * nnz,
                            "max_abs_diff_to_per_request_read_time":
                                float((o.float() - o_req.float()).abs().max().item())})
        del dres, handles
        torch.cuda.empty_cache()
    return out


def measure_zero_data(torch, R, W, name="prefill_8b", iters=20):
    """The prefill kernel on the same workload with the operands' values changed and nothing else: same launch,
    same instruction stream, same tables and traffic.  What changes is what the MFMA and vector units draw, and
    with it the clock the chip holds: the time on zeroed K/V is what this instruction stream costs when the chip
    is not limited by power."""
    job = Job(name, torch, R, W, decode_after_prefill=False)
    if not job.has_prefill:
        return None

    def timed():
        for _ in range(5):
            job.prefill()
        torch.cuda.synchronize()
        return _event_ms(job.prefill, torch, iters)

    out = {"kernel": "prefill_kernel", "workload": name, "kernel_ms_random": timed()}
    k, v = job.pool.k.clone(), job.pool.v.clone()
    job.pool.k.zero_()
    job.pool.v.zero_()
    out["kernel_ms_zero_kv"] = timed()
    q = job.q.clone()
    job.q.zero_()
    out["kernel_ms_zero_kv_and_q"] = timed()
    job.pool.k.copy_(k)
    job.pool.v.copy_(v)
    job.q.copy_(q)
    out["kernel_ms_random_again"] = timed()
    flops = job.prefill_flops()
    out["tflops_random"] = flops / (out["kernel_ms_random"] * 1e-3) / 1e12
    out["tflops_zero_kv"] = flops / (out["kernel_ms_zero_kv"] * 1e-3) / 1e12
    out["frac_of_mfma_peak_zero_kv"] = out["tflops_zero_kv"] / PEAK_MFMA_BF16_TFLOPS
    out["random_over_zero_kv"] = out["kernel_ms_random"] / out["kernel_ms_zero_kv"]
    del job
    return out


def measure_stream_copy(torch, iters=10):
    """What a plain device-to-device copy of 1 GiB reaches on this machine (bytes read + bytes written
    per second): the practical streaming ceiling next to the 8 TB/s on paper."""
    src = torch.ones(1 << 29, dtype=torch.bfloat16, device="cuda:0")
    dst = torch.empty_like(src)
    fn = lambda: dst.copy_(src)
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    ms = _event_ms(fn, torch, iters)
    del src, dst
    torch.cuda.empty_cache()
    return {"kernel": "torch copy_ (1 GiB)", "kernel_ms": ms, "gbs_read_plus_write": 2.0 * (1 << 30) / (ms * 1e-3) / 1e9}


def measure_stream_read(torch, R, W, iters=10, gib=2):
    """The read-only ceiling of the box: gf_hbm_read_probe (hand-written, 16 B per lane, grid stride, one sum
    per workgroup) over a buffer several times the 256 MB Infinity Cache, for a few grid sizes."""
    from paper_2605_22566_amd import binding as B
    dev = torch.device("cuda:0")
    sess = R.Session(W.small_layered(1, W.Shape(8, 2, 128), num_req=1), dev)
    nbytes = gib << 30
    src = torch.ones(nbytes // 2, dtype=torch.bfloat16, device=dev)
    best = None
    for num_wg in (2048, 4096, 8192, 16384):
        sums = torch.zeros(num_wg, dtype=torch.int32, device=dev)
        fn = lambda: B.gf_hbm_read_probe(sess.ctx, src, nbytes, sums, num_wg)
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        ms = _event_ms(fn, torch, iters)
        # every 32-bit word of the buffer is 0x3f803f80 (two bf16 ones): the sums must add up to that, mod 2^32
        got = int(sums.to(torch.int64).sum().item()) & 0xffffffff
        ent = {"workgroups": num_wg, "kernel_ms": ms, "gbs_read": nbytes / (ms * 1e-3) / 1e9,
               "every_word_summed": got == ((nbytes // 4) * 0x3f803f80) & 0xffffffff}
        if best is None or ent["gbs_read"] > best["gbs_read"]:
            best = ent
    del src
    torch.cuda.empty_cache()
    best.update({"kernel": "hbm_read_probe_kernel", "bytes": nbytes, "frac_of_hbm_peak": best["gbs_read"] / PEAK_HBM_GBS})
    return best


def measure_stream_tiles(torch, R, W, iters=10, gib=4):
    """The read-only ceiling for the access pattern of a block table (gf_hbm_tile_probe): a 4 GiB buffer read once
    as tiles in a random order -- 4 KB tiles (one (block, kv head) image of K or V at head_dim 128, what a wave of
    the decode kernels requests at a time), 32 KB tiles (all kv heads of a block) and, for comparison, the same
    tiles in rising order."""
    from paper_2605_22566_amd import binding as B
    dev = torch.device("cuda:0")
    sess = R.Session(W.small_layered(1, W.Shape(8, 2, 128), num_req=1), dev)
    nbytes = gib << 30
    src = torch.ones(nbytes // 2, dtype=torch.bfloat16, device=dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    out = {"kernel": "hbm_tile_probe_kernel", "bytes": nbytes, "runs": []}
    for tile, order in ((4096, "random"), (32768, "random"), (4096, "rising")):
        n = nbytes // tile
        ids = (torch.randperm(n, generator=gen, device=dev) if order == "random"
               else torch.arange(n, device=dev)).to(torch.int32)
        best = None
        for num_wg in (4096, 8192, 16384):
            sums = torch.zeros(num_wg, dtype=torch.int32, device=dev)
            fn = lambda: B.gf_hbm_tile_probe(sess.ctx, src, tile, n, ids, n, sums, num_wg)
            for _ in range(2):
                fn()
            torch.cuda.synchronize()
            ms = _event_ms(fn, torch, iters)
            got = int(sums.to(torch.int64).sum().item()) & 0xffffffff
            ent = {"tile_bytes": tile, "order": order, "workgroups": num_wg, "kernel_ms": ms,
                   "gbs_read": nbytes / (ms * 1e-3) / 1e9, "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                   "every_word_summed": got == ((nbytes // 4) * 0x3f803f80) & 0xffffffff}
            if best is None or ent["gbs_read"] > best["gbs_read"]:
                best = ent
        out["runs"].append(best)
        del ids
    del src
    torch.cuda.empty_cache()
    return out


def measure_mfma_probe(torch, R, W, iters=10, mfma_rounds=(4000, 32000)):
    """The matrix-pipe ceiling of the box for the prefill's instruction (gf_mfma_probe: v_mfma_f32_32x32x16_bf16 alone,
    and with the six vector instructions -- one exponential -- that a softmax spends per MFMA at head_dim 128), on
    zeroed operands and on N(0, 1) bf16 operands (what K, V and Q hold), at one and at two waves per SIMD, in
    launches of about 0.5-1.5 ms and of about 4-12 ms: the instruction stream is the same, what differs is what the
    datapaths toggle -- and with it the clock the chip's power management allows."""
    from paper_2605_22566_amd import binding as B
    dev = torch.device("cuda:0")
    sess = R.Session(W.small_layered(1, W.Shape(8, 2, 128), num_req=1), dev)
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    gen = torch.Generator(device=dev)
    gen.manual_seed(11)
    nbytes = 64 << 20
    operands = {"zeros": torch.zeros(nbytes // 2, dtype=torch.bfloat16, device=dev),
                "normal": torch.randn(nbytes // 2, generator=gen, device=dev).to(torch.bfloat16)}
    out = {"kernel": "mfma_probe_kernel", "instruction": "v_mfma_f32_32x32x16_bf16", "runs": []}
    for mix in (0, 1):
        for rounds in mfma_rounds:
            for what, buf in operands.items():
                for waves_per_simd in (1, 2):
                    num_wg = cus * waves_per_simd
                    sums = torch.zeros(num_wg * 256, dtype=torch.float32, device=dev)
                    fn = lambda: B.gf_mfma_probe(sess.ctx, buf, nbytes, rounds, sums, num_wg, softmax_mix=mix)
                    for _ in range(3):
                        fn()
                    torch.cuda.synchronize()
                    ms = _event_ms(fn, torch, iters)
                    flops = num_wg * 4 * rounds * 8 * 32768.0
                    tf = flops / (ms * 1e-3) / 1e12
                    out["runs"].append({"operands": what, "softmax_mix": mix, "waves_per_simd": waves_per_simd,
                                        "mfma_per_wave": 8 * rounds, "kernel_ms": ms, "tflops": tf,
                                        "frac_of_mfma_peak": tf / PEAK_MFMA_BF16_TFLOPS,
                                        "sums_finite": bool(torch.isfinite(sums).all().item())})
    del operands
    torch.cuda.empty_cache()

    def best(what, mix):                                   # the long launches
        return max(r["tflops"] for r in out["runs"] if r["operands"] == what and r["softmax_mix"] == mix
                   and r["mfma_per_wave"] == 8 * mfma_rounds[-1])
    out["tflops_zeros"], out["tflops_normal"] = best("zeros", 0), best("normal", 0)
    out["tflops_zeros_softmax_mix"], out["tflops_normal_softmax_mix"] = best("zeros", 1), best("normal", 1)
    out["normal_over_zeros"] = out["tflops_normal"] / out["tflops_zeros"]
    out["frac_of_mfma_peak_normal"] = out["tflops_normal"] / PEAK_MFMA_BF16_TFLOPS
    out["frac_of_mfma_peak_normal_softmax_mix"] = out["tflops_normal_softmax_mix"] / PEAK_MFMA_BF16_TFLOPS
    return out


def measure_residual(torch, R, W, num_items=8192, iters=20):
    """gf_kv_apply_residual on the 8B head shape: num_items pool blocks reconstructed from base
    blocks and residuals of the density the paper reports (25 % of K, 30 % of V elements)."""
    sh = W.Shape(32, 8, 128)
    dev = torch.device("cuda:0")
    wl = W.small_layered(1, sh, num_req=1)                    # only carries the shape for the session
    sess = R.Session(wl, dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(5)
    nb = 2 * num_items
    k = torch.randn((nb, sh.num_kv_heads, W.BLOCK, sh.head_dim), generator=gen, device=dev).to(torch.bfloat16)
    v = torch.randn((nb, sh.num_kv_heads, sh.head_dim, W.BLOCK), generator=gen, device=dev).to(torch.bfloat16)
    pool = R.DevicePool(k, v, nb)
    dres, nnz = R.random_residuals(sh, num_items, dev)
    fn = lambda: sess.apply_residual(pool, dres)
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    ms = _event_ms(fn, torch, iters)
    blk = 2 * sh.num_kv_heads * W.BLOCK * sh.head_dim * 2
    nbytes = num_items * (2 * blk + 8 + 4 * 2 * sh.num_kv_heads) + 4.0 * nnz
    ok = bool((dres["status"] == 0).all().item())
    out = {"kernel": "residual_kernel", "kernel_ms": ms, "blocks": num_items, "entries": nnz,
           "algorithmic_bytes_per_launch": nbytes, "gbs_kernel": nbytes / (ms * 1e-3) / 1e9,
           "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "all_items_ok": ok,
           "hbm_bytes_per_launch_rocprof": _read_traffic("residual_kv_residual")}
    # the packed form (bit mask per image + values in element order): what a residual costs at rest, the
    # conversion, and the reconstruction straight from it
    packed = sess.pack_residuals(dres)
    torch.cuda.synchronize()
    ms_pack = _event_ms(lambda: sess.pack_residuals(dres), torch, 5)
    ms_unpack = _event_ms(lambda: sess.unpack_residuals(packed), torch, 5)
    before = pool.k[num_items:].clone()
    fnp = lambda: sess.apply_residual_packed(pool, packed)
    fnp()
    torch.cuda.synchronize()
    same = bool(torch.equal(before.view(torch.int16), pool.k[num_items:].view(torch.int16)))
    del before
    ms_p = _event_ms(fnp, torch, iters)
    rows = num_items * 2 * sh.num_kv_heads
    mask_bytes = rows * (W.BLOCK * sh.head_dim // 8)
    nbytes_p = num_items * (2 * blk + 8 + 4 * 2 * sh.num_kv_heads) + 2.0 * nnz + mask_bytes
    out["packed"] = {"kernel": "residual_packed_kernel", "kernel_ms": ms_p, "algorithmic_bytes_per_launch": nbytes_p,
                     "gbs_kernel": nbytes_p / (ms_p * 1e-3) / 1e9,
                     "frac_of_hbm_peak": nbytes_p / (ms_p * 1e-3) / 1e9 / PEAK_HBM_GBS,
                     "same_blocks_as_coordinate_form": same, "pack_ms": ms_pack, "unpack_ms": ms_unpack,
                     "coordinate_bytes": 4.0 * nnz + 4.0 * (rows + 1),
                     "packed_bytes": 2.0 * nnz + mask_bytes + 4.0 * (rows + 1),
                     "dense_bytes": float(num_items) * blk,
                     "packed_over_dense": (2.0 * nnz + mask_bytes + 4.0 * (rows + 1)) / (float(num_items) * blk),
                     "coordinate_over_dense": (4.0 * nnz + 4.0 * (rows + 1)) / (float(num_items) * blk)}
    del packed
    # the way back: gf_kv_make_residual recovers a residual from the reconstructed blocks against their base blocks
    # (95 % energy rule; per image a sort in LDS, two passes over the blocks): an offline step, timed for the record
    fnm = lambda: sess.make_residual(pool, dres["src"], dres["dst"], 0.95)
    made = fnm()
    torch.cuda.synchronize()
    msm = _event_ms(fnm, torch, 3)
    nnz_made = int(made["ptr"][-1].item())
    out["make_residual"] = {"kernel": "make_residual_count_kernel + make_residual_scan_kernel + make_residual_fill_kernel", "kernel_ms": msm, "blocks": num_items,
                            "entries_kept_at_95pct_energy": nnz_made, "entries_of_the_source_residual": nnz,
                            "algorithmic_bytes_per_launch": 2.0 * num_items * 2 * blk + 4.0 * nnz_made,
                            "gbs_kernel": (2.0 * num_items * 2 * blk + 4.0 * nnz_made) / (msm * 1e-3) / 1e9,
                            "all_items_ok": bool((made["status"] == 0).all().item())}
    del made
    # the same items on an e4m3 pool (codes of N(0,1) blocks, scale amax / 448): half the block bytes, two passes
    del pool, k, v
    sh8 = W.Shape(32, 8, 128, W.KV_FP8_E4M3)
    sess8 = R.Session(W.small_layered(1, sh8, num_req=1), dev)
    x = torch.randn((2, nb, sh.num_kv_heads * W.BLOCK * sh.head_dim), generator=gen, device=dev)
    sc = x.abs().amax(dim=2) / 448.0
    codes = (x / sc[:, :, None]).to(torch.float8_e4m3fn).view(torch.uint8)
    pool8 = R.DevicePool(codes[0].view(nb, sh.num_kv_heads, W.BLOCK, sh.head_dim).contiguous(),
                         codes[1].view(nb, sh.num_kv_heads, sh.head_dim, W.BLOCK).contiguous(), nb,
                         sc[0].contiguous(), sc[1].contiguous())
    del x, codes
    dres["status"].fill_(-77)
    fn8 = lambda: sess8.apply_residual(pool8, dres)
    for _ in range(3):
        fn8()
    torch.cuda.synchronize()
    ms8 = _event_ms(fn8, torch, iters)
    nbytes8 = num_items * (blk + 16 + 8 + 4 * 2 * sh.num_kv_heads) + 4.0 * nnz      # blk / 2 read + blk / 2 written, scales
    out["e4m3"] = {"kernel": "residual_e4m3_onepass_kernel", "kernel_ms": ms8, "algorithmic_bytes_per_launch": nbytes8,
                   "gbs_kernel": nbytes8 / (ms8 * 1e-3) / 1e9, "frac_of_hbm_peak": nbytes8 / (ms8 * 1e-3) / 1e9 / PEAK_HBM_GBS,
                   "all_items_ok": bool((dres["status"] == 0).all().item())}
    return out


def cpu_baseline(job, budget_s=20.0, mode=None, windows=False):
    """Time the fp64 oracle on a bounded sample of the workload's requests and check the GPU outputs of the
    sample against it.  mode: "prefill" or "decode" (default: what the workload's headline is).  With
    `windows`, a prefill request is checked on its first and last 48 rows instead of whole (rows i0..i1 of a
    request are plain attention of those queries over its first ctx + i1 tokens, ctx + i0 of them context), so
    that long requests fit a small budget."""
    from oracle import attention as OA
    from oracle import resolve as ORS
    torch, R, W = job.torch, job.R, job.W
    wl = job.wl
    b, g = wl.batch, wl.graph
    sh = wl.shape
    tables = ORS.resolve_paths(g.num_nodes, g.node_len, g.node_block_ptr, g.node_blocks, g.edge_ptr, g.edge_dst,
                               b.path_ptr, b.path_nodes, b.new_lens, b.tail_ptr, b.tail_blocks, job.max_blocks,
                               wl.num_pool_blocks)
    # GPU tables must be bit-exact
    dev_tables = R.tables_to_host(job.tables)
    tables_exact = all(dev_tables[k] == tables[k] for k in tables)
    prefill_mode = job.has_prefill if mode is None else mode == "prefill"
    lo_r, hi_r = job.pf_rng if prefill_mode else job.dec_rng
    order = lo_r + np.random.default_rng(wl.seed + 9).permutation(hi_r - lo_r)
    q_host = R.bf16_to_bits(job.q)
    o_gpu = job.o.double().cpu().numpy() if prefill_mode else job.od.double().cpu().numpy()
    atol, rtol = (1e-2, 1e-2) if sh.kv_dtype == W.KV_BF16 else (5e-2, 5e-2)
    spent, work, used, max_err, ok = 0.0, 0.0, 0, 0.0, True
    pair_flops = 4.0 * sh.head_dim * sh.num_q_heads
    for r in order:
        r = int(r)
        nb = tables["num_blocks"][r]
        ids = np.array(tables["block_table"][r][:nb], dtype=np.int64)
        kk, vv, ks, vs = job.pool.gather_host(ids)
        local = {k_: [v_[r]] for k_, v_ in tables.items()}
        local["block_table"] = [list(range(nb))]
        lo, hi = int(job.q_ptr[r]), int(job.q_ptr[r + 1])
        t0 = time.perf_counter()
        checks = []
        if prefill_mode and windows and hi - lo > 96:
            K, V = OA.materialize_kv(kk, vv, local["block_table"][0], tables["block_ntok"][r], nb, ks, vs)
            ctx, n_r = int(tables["ctx_lens"][r]), hi - lo
            for i0, i1 in ((0, 48), (n_r - 48, n_r)):
                O, _ = OA.attend(OA._widen(q_host[lo + i0:lo + i1]), K[:ctx + i1], V[:ctx + i1], ctx + i0)
                checks.append((o_gpu[lo + i0:lo + i1], O))
                work += pair_flops * sum(ctx + i + 1 for i in range(i0, i1))
        elif prefill_mode:
            O, _ = OA.prefill(q_host[lo:hi], np.array([0, hi - lo]), kk, vv, local, ks, vs)
            checks.append((o_gpu[lo:hi], O))
            work += W.prefill_flops(wl, [r])
        else:
            O, _ = OA.decode(q_host[hi - 1:hi], kk, vv, local, ks, vs)
            checks.append((o_gpu[r:r + 1], O))
            work += W.decode_bytes(wl, [r])
        spent += time.perf_counter() - t0
        for got, O in checks:
            err = np.abs(got - O)
            max_err = max(max_err, float(err.max()))
            ok = ok and bool((err <= atol + rtol * np.abs(O)).all())
        used += 1
        if spent > budget_s:
            break
    try:
        import threadpoolctl
        threads = max(i["num_threads"] for i in threadpoolctl.threadpool_info())
    except Exception:
        threads = os.cpu_count()
    unit = "TFLOP/s" if prefill_mode else "GB/s"
    value = work / spent / (1e12 if prefill_mode else 1e9)
    what = "requests" if not (prefill_mode and windows) else "requests (first and last 48 rows of each)"
    return {"value": value, "unit": unit, "cores": int(threads), "host_cpu_count": os.cpu_count(), "kind": "oracle",
            "sample": f"{used} of {hi_r - lo_r} {'prefill' if prefill_mode else 'decode'} {what} of {wl.name} "
                      f"(seeded order), {spent:.1f} s of numpy fp64",
            "gpu_matches_oracle_on_sample": ok, "max_abs_err": max_err, "tables_bit_exact": tables_exact}


def prefill_roofline(job, m, workload):
    return {"bound": "mfma", "kernel": "prefill_kernel", "achieved": m["prefill_tflops_kernel"],
            "peak": PEAK_MFMA_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": m["prefill_tflops_kernel"] / PEAK_MFMA_BF16_TFLOPS,
            "traffic": _read_traffic(f"prefill_{workload}"),
            "kernel_ms": m["prefill_ms"], "kernel_ms_median": m["prefill_median_ms"],
            "kernel_ms_cold_cache_median": m["prefill_cold_median_ms"],
            "algorithmic_flops_per_launch": job.prefill_flops()}


def decode_roofline(job, m, workload):
    """The per-request decode kernel (+ merge).  On a workload with shared nodes its request-centric bytes are
    mostly cache hits: they are reported as a rate, the fraction rests on HBM bytes."""
    stats = job.W.sharing_stats(job.wl)
    shared = stats["sharing_factor"] > 1.0 + 1e-9
    lo, hi = job.dec_rng
    sh = job.wl.shape
    unique = stats["shared_kv_bytes"] + 2.0 * (hi - lo) * sh.num_q_heads * sh.head_dim * 2
    out = hbm_roofline("decode_split_kernel(+merge)", job.decode_bytes(), m["decode_ms"],
                       _read_traffic(f"decode_{workload}"), job.decode_bytes() if shared else None,
                       unique if shared else None)
    out["kernel_ms_median"] = m["decode_median_ms"]
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="prefill_8b",
                    choices=["tiny", "prefill_8b", "decode_8b", "decode_70b", "mixed_fp8", "decode_8b_private",
                             "decode_8b_private_seq"])
    ap.add_argument("--decode-chunk", type=int, default=0,
                    help="table entries per split-KV chunk of the decode kernels (0 = the library's choice)")
    ap.add_argument("--extra", default="decode_8b,decode_70b,mixed_fp8,decode_8b_private,decode_8b_private_seq,kv_residual,stream,zero_data",
                    help="comma list of further workloads reported under 'extra' (the five configs, decode_8b_private = "
                         "config 3 with nothing shared, decode_8b_private_seq = the same with an unshuffled pool, "
                         "kv_residual, stream = the box's read-only and copy rates)")
    ap.add_argument("--extra-cpu-budget", type=float, default=5.0,
                    help="seconds of oracle time per extra workload and phase for the sampled output check")
    ap.add_argument("--residual-share", type=float, default=0.25,
                    help="decode_residual: share of every request's table entries (its last ones) that carry a residual")
    ap.add_argument("--residual-density", default="0.25,0.30",
                    help="decode_residual: share of the K,V elements of such an entry that the residual names (> 0)")
    ap.add_argument("--kv-data", choices=("random", "zeros"), default="random",
                    help="zeros: the K/V pool is cleared before the timed region -- a measurement aid (same kernel, "
                         "same instruction stream and traffic, operands that draw less power), never the metric")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-budget", type=float, default=20.0)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run three plain 1 GiB device copies (known traffic, for scaling rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_22566_amd import binding as B
    from paper_2605_22566_amd import runner as R
    from paper_2605_22566_amd import workload as W
    B.load_library()           # fails loudly if the HIP library is not built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)

    if args.copy_calibration:
        src = torch.ones(1 << 29, dtype=torch.bfloat16, device="cuda:0")   # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    job = Job(args.workload, torch, R, W)
    if args.kv_data == "zeros":
        job.pool.k.zero_()
        job.pool.v.zero_()
        args.no_cpu_baseline = True          # the oracle sample would be checked against other data
    if args.decode_chunk:
        B.gf_set_decode_chunk_blocks(job.sess.ctx, args.decode_chunk)
    m = measure(job, args.steps, args.warmup)
    wl = job.wl
    if job.has_prefill:
        metric, unit = "prefill_tflops", "TFLOP/s"
        value = job.prefill_flops() / (m["ms_per_step"] * 1e-3) / 1e12
        roof = prefill_roofline(job, m, args.workload)
    else:
        # whole-step rate of the request-centric bytes (what attention through per-request tables moves,
        # cache hits on shared nodes included); the roofline fraction rests on HBM bytes
        metric, unit = "decode_logical_gbs", "GB/s"
        value = job.decode_bytes() / (m["ms_per_step"] * 1e-3) / 1e9
        roof = decode_roofline(job, m, args.workload)
    res = {
        "metric": metric, "value": value, "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": m["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.shape.kv_dtype == W.KV_BF16 else "fp8_e4m3 KV / bf16 Q, fp32 accumulate",
        "data": "synthetic" if args.kv_data == "random" else "synthetic, K/V pool zeroed (measurement aid, not the metric)",
        "config": {"workload": args.workload, "requests": wl.batch.num_req, "q_heads": wl.shape.num_q_heads,
                   "kv_heads": wl.shape.num_kv_heads, "head_dim": wl.shape.head_dim, "block": 16,
                   "nodes": wl.graph.num_nodes, "pool_blocks": wl.num_pool_blocks,
                   "new_tokens": int(wl.batch.new_lens.sum()), "ctx_tokens": int(W.context_lens(wl).sum()),
                   "sharing_factor": W.sharing_stats(wl)["sharing_factor"],
                   "stateful_over_shared_kv_bytes": W.sharing_stats(wl)["stateful_kv_bytes"]
                   / W.sharing_stats(wl)["shared_kv_bytes"], "seed": wl.seed,
                   "step": "resolve+prefill+decode(+merge)"},
        "roofline": roof,
        "breakdown_ms": {k: v for k, v in m.items() if k.endswith("_ms")},
    }
    if job.has_prefill and job.has_decode:
        res["decode_roofline"] = decode_roofline(job, m, args.workload)
    if job.has_decode:
        res["decode_shared"] = decode_shared_entry(job, m)
    pr = measure_prefill_residual(job, m["prefill_ms"]) if job.has_prefill else None
    if pr is not None:
        res["prefill_residual"] = pr
    res["kv_append"] = {"kernel": "append_kernel", "kernel_ms": m["append_ms"], "gbs_kernel": m["append_gbs_kernel"],
                        "frac_of_hbm_peak": m["append_gbs_kernel"] / PEAK_HBM_GBS,
                        "algorithmic_bytes_per_launch": job.append_bytes(),
                        "hbm_bytes_per_launch_rocprof": _read_traffic(f"append_{args.workload}")}
    res["kv_append_token"] = {"kernel": "append_token_kernel", "kernel_ms": m["append_token_ms"],
                              "requests": wl.batch.num_req, "bound": "latency (one small workgroup per request)"}
    # host-side accounting (no GPU work): KV bytes held for the first 10..50 requests under the designs the
    # paper compares, and with transition pruning
    from paper_2605_22566_amd import footprint as FP
    res["footprint"] = [{k: v for k, v in row.items()} for row in FP.footprint_by_batch_size(wl)]
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(job, args.cpu_budget)
    extra = {}
    del job
    torch.cuda.empty_cache()
    names = [x for x in args.extra.split(",") if x and x != args.workload]
    if "zero_data" in names:
        names.remove("zero_data")
        zd = measure_zero_data(torch, R, W)
        if zd is not None:
            extra["prefill_zero_data"] = zd
        torch.cuda.empty_cache()
    if "stream" in names:
        names.remove("stream")
        extra["stream_read"] = measure_stream_read(torch, R, W)
        extra["stream_tiles"] = measure_stream_tiles(torch, R, W)
        extra["stream_copy"] = measure_stream_copy(torch)
        extra["mfma_probe"] = measure_mfma_probe(torch, R, W)
    if "kv_residual" in names:
        names.remove("kv_residual")
        extra["kv_residual"] = measure_residual(torch, R, W)
        torch.cuda.empty_cache()
    for name in names:
        j = Job(name, torch, R, W, decode_after_prefill=False)
        mm = measure(j, max(5, args.steps // 2), max(3, args.warmup // 2))
        ent = {"ms_per_step": mm["ms_per_step"], "breakdown_ms": {k: v for k, v in mm.items() if k.endswith("_ms")},
               "sharing_factor": W.sharing_stats(j.wl)["sharing_factor"]}
        if j.has_prefill:
            ent["prefill_tflops_kernel"] = mm["prefill_tflops_kernel"]
            ent["roofline"] = prefill_roofline(j, mm, name)
        if j.has_decode:
            ent["decode_roofline" if j.has_prefill else "roofline"] = decode_roofline(j, mm, name)
            ent["decode_shared"] = decode_shared_entry(j, mm)
            if name in ("decode_8b",):
                dr = measure_decode_residual(j, mm["decode_ms"], args.residual_share,
                                             tuple(float(x) for x in args.residual_density.split(",")))
                if dr is not None:
                    ent["decode_residual"] = dr
                sr = measure_shared_residual(j, mm)
                if sr is not None:
                    ent["decode_shared_residual"] = sr
        if not args.no_cpu_baseline:
            # bounded oracle check of this workload's GPU outputs (a few seconds per call)
            if j.has_prefill:
                ent["oracle_check_prefill"] = cpu_baseline(j, args.extra_cpu_budget, "prefill", windows=True)
            if j.has_decode:
                ent["oracle_check_decode"] = cpu_baseline(j, args.extra_cpu_budget, "decode")
            ent["gpu_matches_oracle_on_sample"] = all(
                ent[k]["gpu_matches_oracle_on_sample"] for k in ("oracle_check_prefill", "oracle_check_decode") if k in ent)
        extra[name] = ent
        del j
        torch.cuda.empty_cache()
    if extra:
        res["extra"] = extra
    # the headline beside the ceilings measured in this run: an MFMA-bound line against the probe on N(0, 1)
    # operands with a softmax's vector work riding along (issued flops against issued flops would be fairer still:
    # the kernel's masked pairs are not in `achieved`), an HBM-bound line against the tile-order read probe
    rf = res.get("roofline") or {}
    if rf.get("bound") == "mfma" and "mfma_probe" in extra:
        rf["probe_tflops_normal_operands"] = extra["mfma_probe"]["tflops_normal"]
        rf["probe_tflops_normal_operands_softmax_mix"] = extra["mfma_probe"]["tflops_normal_softmax_mix"]
        rf["frac_of_probe_softmax_mix"] = rf["achieved"] / extra["mfma_probe"]["tflops_normal_softmax_mix"]
    if rf.get("bound") == "hbm" and "stream_tiles" in extra:
        best = max(r["gbs_read"] for r in extra["stream_tiles"]["runs"])
        rf["probe_gbs_tile_reads"] = best
        rf["frac_of_probe_tile_reads"] = rf["achieved"] / best
    print(json.dumps(res))


if __name__ == "__main__":
    main()
