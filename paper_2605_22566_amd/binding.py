"""ctypes binding of libgraphflow.so: argument marshalling only.

Every function here has the name and the arguments of the C entry point it
calls (include/graphflow.h); tensors are torch tensors that already live on the
GPU and are passed as raw device pointers, and the HIP stream is torch's
current stream.  Nothing is computed in Python and there is no fallback: if the
library is not built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libgraphflow.so")

GF_OK = 0
GF_ERR_NULL, GF_ERR_BAD_SHAPE, GF_ERR_UNSUPPORTED, GF_ERR_WORKSPACE, GF_ERR_HIP = -1, -2, -3, -4, -5
GF_ST_OK, GF_ST_BAD_NODE, GF_ST_BAD_EDGE, GF_ST_BAD_TAIL, GF_ST_BAD_BLOCK, GF_ST_OVERFLOW = 0, 1, 2, 3, 4, 5
GF_BF16, GF_FP8_E4M3 = 0, 1
GF_RS_OK, GF_RS_BAD_BLOCK, GF_RS_BAD_INDEX, GF_RS_TRUNCATED = 0, 1, 2, 3

EXPORTS = ["gf_create", "gf_destroy", "gf_strerror", "gf_last_hip_error", "gf_resolve_path",
           "gf_attn_prefill", "gf_attn_prefill_residual", "gf_attn_decode", "gf_attn_decode_residual", "gf_attn_decode_shared", "gf_attn_decode_shared_residual", "gf_decode_shared_plan", "gf_attn_decode_shared_planned",
           "gf_set_decode_chunk_blocks", "gf_kv_apply_residual", "gf_kv_residual_pack", "gf_kv_residual_unpack",
           "gf_kv_apply_residual_packed",
           "gf_kv_append", "gf_kv_append_token", "gf_attn_prefill_noalloc", "gf_hbm_read_probe", "gf_hbm_tile_probe", "gf_mfma_probe",
           "gf_prefix_key", "gf_residual_dir_clear", "gf_residual_dir_insert", "gf_resolve_path_residual",
           "gf_residual_dir_prune", "gf_kv_make_residual", "gf_block_pool_create", "gf_block_pool_destroy", "gf_block_pool_alloc",
           "gf_block_pool_retain", "gf_block_pool_release", "gf_block_pool_stats", "gf_block_pool_refcount"]
GF_DIR_OK, GF_DIR_FULL, GF_DIR_BAD_PAIR = 0, 1, 2

_i32p = C.c_void_p  # device pointers travel as plain addresses


class gf_graph(C.Structure):
    _fields_ = [("num_nodes", C.c_int32), ("node_len", _i32p), ("node_block_ptr", _i32p),
                ("node_blocks", _i32p), ("edge_ptr", _i32p), ("edge_dst", _i32p)]


class gf_attn_params(C.Structure):
    _fields_ = [("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("block_size", C.c_int32), ("kv_dtype", C.c_int32), ("sm_scale", C.c_float)]


class gf_kv_pool(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("k_scale", C.c_void_p), ("v_scale", C.c_void_p),
                ("num_blocks", C.c_int32)]


class gf_tables(C.Structure):
    _fields_ = [("block_table", _i32p), ("block_ntok", _i32p), ("num_blocks", _i32p), ("ctx_lens", _i32p),
                ("seq_lens", _i32p), ("status", _i32p), ("num_req", C.c_int32), ("max_blocks", C.c_int32)]


class gf_residual_dir(C.Structure):
    _fields_ = [("key", C.c_void_p), ("prev", _i32p), ("node", _i32p), ("first_item", _i32p), ("uses", _i32p),
                ("capacity", C.c_int32)]


class GraphFlowError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libgraphflow error {code}: {msg}")
        self.code = code


_lib = None


def load_library(path: Optional[str] = None):
    """Load libgraphflow.so (built in-tree by paper_2605_22566_amd/build.py)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or os.environ.get("GRAPHFLOW_LIB") or LIB_PATH
    if not os.path.exists(p):
        raise FileNotFoundError(
            f"{p} is missing: build it with `python paper_2605_22566_amd/build.py` "
            "(or __graft_entry__.build()); there is no fallback path")
    lib = C.CDLL(p)
    lib.gf_create.argtypes = [C.POINTER(C.c_void_p), C.c_int32]
    lib.gf_create.restype = C.c_int32
    lib.gf_destroy.argtypes = [C.c_void_p]
    lib.gf_destroy.restype = C.c_int32
    lib.gf_strerror.argtypes = [C.c_int32]
    lib.gf_strerror.restype = C.c_char_p
    lib.gf_last_hip_error.argtypes = [C.c_void_p]
    lib.gf_last_hip_error.restype = C.c_char_p
    lib.gf_set_decode_chunk_blocks.argtypes = [C.c_void_p, C.c_int32]
    lib.gf_set_decode_chunk_blocks.restype = C.c_int32
    lib.gf_resolve_path.argtypes = [C.c_void_p, C.POINTER(gf_graph), C.c_int32] + [C.c_void_p] * 5 + \
        [C.c_int32, C.c_int32] + [C.c_void_p] * 6 + [C.c_void_p]
    lib.gf_resolve_path.restype = C.c_int32
    lib.gf_attn_prefill.argtypes = [C.c_void_p, C.POINTER(gf_attn_params), C.POINTER(gf_kv_pool),
                                    C.POINTER(gf_tables), C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                    C.c_void_p, C.c_void_p, C.c_void_p]
    lib.gf_attn_prefill.restype = C.c_int32
    lib.gf_attn_prefill_noalloc.argtypes = lib.gf_attn_prefill.argtypes
    lib.gf_kv_residual_pack.argtypes = [C.c_void_p, C.POINTER(gf_attn_params), C.c_int32] + [C.c_void_p] * 7
    lib.gf_kv_residual_pack.restype = C.c_int32
    lib.gf_kv_residual_unpack.argtypes = [C.c_void_p, C.POINTER(gf_attn_params), C.c_int32] + [C.c_void_p] * 5
    lib.gf_kv_residual_unpack.restype = C.c_int32
    lib.gf_kv_apply_residual_packed.argtypes = [C.c_void_p, C.POINTER(gf_attn_params), C.c_void_p, C.c_void_p,
                                                C.c_int32, C.c_int32] + [C.c_void_p] * 7
    lib.gf_kv_apply_residual_packed.restype = C.c_int32
    lib.gf_attn_prefill_residual.argtypes = [C.c_void_p, C.POINTER(gf_attn_params), C.POINTER(gf_kv_pool),
                                             C.POINTER(gf_tables), C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                             C.c_void_p, C.c_void_p]
    lib.gf_attn_prefill_residual.restype = C.c_int32
    lib.gf_attn_prefill_noalloc.restype = C.c_int32
    lib.gf_hbm_read_probe.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.c_void_p]
    lib.gf_hbm_read_probe.restype = C.c_int32
    lib.gf_hbm_tile_probe.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p,
                                      C.c_int32, C.c_void_p]
    lib.gf_hbm_tile_probe.restype = C.c_int32
    lib.gf_mfma_probe.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_int32,
                                  C.c_void_p]
    lib.gf_mfma_probe.restype = C.c_int32
    lib.gf_attn_decode.argtypes = [C.c_void_p, C.POINTER(gf_attn_params), C.POINTER(gf_kv_pool),
                                   C.POINTER(gf_tables), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.gf_attn_decode.restype = C.c_int32
    lib.gf_attn_decode_residual.argtypes = [C.c_void_p, C.POINTER(gf_attn_params), C.POINTER(gf_kv_pool),
                                            C.POINTER(gf_tables), C.c_void_p, C.c_int32] + [C.c_void_p] * 7
    lib.gf_attn_decode_residual.restype = C.c_int32
    lib.gf_attn_decode_shared_residual.argtypes = [C.c_void_p, C.POINTER(gf_attn_params), C.POINTER(gf_kv_pool),
                                                   C.POINTER(gf_graph), C.c_void_p, C.c_void_p, C.c_int32,
                                                   C.POINTER(gf_tables), C.c_void_p, C.c_int32] + [C.c_void_p] * 7
    lib.gf_attn_decode_shared_residual.restype = C.c_int32
    lib.gf_attn_decode_shared.argtypes = [C.c_void_p, C.POINTER(gf_attn_params), C.POINTER(gf_kv_pool),
                                          C.POINTER(gf_graph), C.c_void_p, C.c_void_p, C.c_int32,
                                          C.POINTER(gf_tables), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.gf_attn_decode_shared.restype = C.c_int32
    lib.gf_attn_decode_shared_planned.argtypes = lib.gf_attn_decode_shared.argtypes
    lib.gf_attn_decode_shared_planned.restype = C.c_int32
    lib.gf_decode_shared_plan.argtypes = [C.c_void_p, C.POINTER(gf_attn_params), C.POINTER(gf_graph), C.c_void_p,
                                          C.c_void_p, C.c_int32, C.POINTER(gf_tables), C.c_void_p]
    lib.gf_decode_shared_plan.restype = C.c_int32
    lib.gf_kv_apply_residual.argtypes = [C.c_void_p, C.POINTER(gf_attn_params)] + [C.c_void_p] * 4 + [C.c_int32,
                                         C.c_int32] + [C.c_void_p] * 6 + [C.c_void_p]
    lib.gf_kv_apply_residual.restype = C.c_int32
    lib.gf_kv_append.argtypes = [C.c_void_p, C.POINTER(gf_attn_params)] + [C.c_void_p] * 4 + [C.c_int32,
                                 C.POINTER(gf_tables)] + [C.c_void_p] * 3 + [C.c_int32, C.c_int32, C.c_void_p]
    lib.gf_kv_append.restype = C.c_int32
    lib.gf_kv_append_token.argtypes = [C.c_void_p, C.POINTER(gf_attn_params)] + [C.c_void_p] * 4 + [C.c_int32,
                                       C.POINTER(gf_tables)] + [C.c_void_p] * 3
    lib.gf_kv_append_token.restype = C.c_int32
    lib.gf_prefix_key.argtypes = [C.POINTER(C.c_int32), C.c_int32]
    lib.gf_prefix_key.restype = C.c_uint64
    lib.gf_residual_dir_clear.argtypes = [C.c_void_p, C.POINTER(gf_residual_dir), C.c_void_p]
    lib.gf_residual_dir_clear.restype = C.c_int32
    lib.gf_residual_dir_insert.argtypes = [C.c_void_p, C.POINTER(gf_residual_dir), C.c_int32] + [C.c_void_p] * 6
    lib.gf_residual_dir_insert.restype = C.c_int32
    lib.gf_resolve_path_residual.argtypes = [C.c_void_p, C.POINTER(gf_graph), C.c_int32] + [C.c_void_p] * 5 + \
        [C.c_int32, C.c_int32] + [C.c_void_p] * 6 + [C.POINTER(gf_residual_dir)] + [C.c_void_p] * 4
    lib.gf_resolve_path_residual.restype = C.c_int32
    lib.gf_residual_dir_prune.argtypes = [C.c_void_p, C.POINTER(gf_graph), C.POINTER(gf_residual_dir), C.c_void_p,
                                          C.c_int32, C.c_void_p, C.c_void_p]
    lib.gf_residual_dir_prune.restype = C.c_int32
    lib.gf_kv_make_residual.argtypes = [C.c_void_p, C.POINTER(gf_attn_params), C.c_void_p, C.c_void_p, C.c_int32,
                                        C.c_int32, C.c_void_p, C.c_void_p, C.c_double, C.c_int32] + [C.c_void_p] * 5
    lib.gf_kv_make_residual.restype = C.c_int32
    lib.gf_block_pool_create.argtypes = [C.POINTER(C.c_void_p), C.c_int32]
    lib.gf_block_pool_destroy.argtypes = [C.c_void_p]
    lib.gf_block_pool_alloc.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32)]
    lib.gf_block_pool_retain.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32)]
    lib.gf_block_pool_release.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.gf_block_pool_stats.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int64),
                                        C.POINTER(C.c_int32)]
    lib.gf_block_pool_refcount.argtypes = [C.c_void_p, C.c_int32]
    for name in ("create", "destroy", "alloc", "retain", "release", "stats", "refcount"):
        getattr(lib, "gf_block_pool_" + name).restype = C.c_int32
    if path is None:
        _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    """Device address of a torch tensor (None -> NULL)."""
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _check(ctx, rc: int):
    if rc != GF_OK:
        lib = load_library()
        msg = lib.gf_strerror(rc).decode()
        if rc in (GF_ERR_HIP, GF_ERR_WORKSPACE) and ctx:
            msg += " / " + lib.gf_last_hip_error(ctx).decode()
        raise GraphFlowError(rc, msg)


def gf_create(device: int = 0) -> int:
    lib = load_library()
    h = C.c_void_p()
    _check(None, lib.gf_create(C.byref(h), device))
    return h.value


def gf_destroy(ctx: int) -> None:
    _check(None, load_library().gf_destroy(ctx))


def gf_set_decode_chunk_blocks(ctx: int, chunk_blocks: int) -> None:
    _check(ctx, load_library().gf_set_decode_chunk_blocks(ctx, chunk_blocks))


def make_graph(num_nodes, node_len, node_block_ptr, node_blocks, edge_ptr=None, edge_dst=None) -> gf_graph:
    return gf_graph(num_nodes, _ptr(node_len), _ptr(node_block_ptr), _ptr(node_blocks), _ptr(edge_ptr),
                    _ptr(edge_dst))


def gf_resolve_path(ctx, graph: gf_graph, num_req, path_ptr, path_nodes, new_lens, tail_ptr, tail_blocks,
                    max_blocks, num_pool_blocks, block_table, block_ntok, num_blocks, ctx_lens, seq_lens,
                    status) -> None:
    rc = load_library().gf_resolve_path(
        ctx, C.byref(graph), num_req, _ptr(path_ptr), _ptr(path_nodes), _ptr(new_lens), _ptr(tail_ptr),
        _ptr(tail_blocks), max_blocks, num_pool_blocks, _ptr(block_table), _ptr(block_ntok),
        _ptr(num_blocks), _ptr(ctx_lens), _ptr(seq_lens), _ptr(status), _stream())
    _check(ctx, rc)


def make_params(num_q_heads, num_kv_heads, head_dim, kv_dtype=GF_BF16, sm_scale=0.0, block_size=16):
    return gf_attn_params(num_q_heads, num_kv_heads, head_dim, block_size, kv_dtype, sm_scale)


def make_pool(k, v, num_blocks, k_scale=None, v_scale=None) -> gf_kv_pool:
    return gf_kv_pool(_ptr(k), _ptr(v), _ptr(k_scale), _ptr(v_scale), num_blocks)


def make_tables(block_table, block_ntok, num_blocks, ctx_lens, seq_lens, status, num_req, max_blocks):
    return gf_tables(_ptr(block_table), _ptr(block_ntok), _ptr(num_blocks), _ptr(ctx_lens), _ptr(seq_lens),
                     _ptr(status), num_req, max_blocks)


def gf_attn_prefill(ctx, params, pool, tables, q, q_ptr, total_q, max_q, o, lse=None) -> None:
    rc = load_library().gf_attn_prefill(ctx, C.byref(params), C.byref(pool), C.byref(tables), _ptr(q),
                                        _ptr(q_ptr), total_q, max_q, _ptr(o), _ptr(lse), _stream())
    _check(ctx, rc)


def gf_attn_prefill_noalloc(ctx, params, pool, tables, q, q_ptr, total_q, max_q, o, lse=None) -> None:
    rc = load_library().gf_attn_prefill_noalloc(ctx, C.byref(params), C.byref(pool), C.byref(tables), _ptr(q),
                                                _ptr(q_ptr), total_q, max_q, _ptr(o), _ptr(lse), _stream())
    _check(ctx, rc)


def gf_kv_residual_pack(ctx, params, num_items, res_ptr, res_idx, res_val, res_mask, packed_val, status=None) -> None:
    rc = load_library().gf_kv_residual_pack(ctx, C.byref(params), num_items, _ptr(res_ptr), _ptr(res_idx),
                                            _ptr(res_val), _ptr(res_mask), _ptr(packed_val), _ptr(status), _stream())
    _check(ctx, rc)


def gf_kv_residual_unpack(ctx, params, num_items, res_ptr, res_mask, res_idx, status=None) -> None:
    rc = load_library().gf_kv_residual_unpack(ctx, C.byref(params), num_items, _ptr(res_ptr), _ptr(res_mask),
                                              _ptr(res_idx), _ptr(status), _stream())
    _check(ctx, rc)


def gf_kv_apply_residual_packed(ctx, params, k_pool, v_pool, num_pool_blocks, num_items, src_blocks, dst_blocks,
                                res_ptr, res_mask, packed_val, status=None) -> None:
    rc = load_library().gf_kv_apply_residual_packed(ctx, C.byref(params), _ptr(k_pool), _ptr(v_pool), num_pool_blocks,
                                                    num_items, _ptr(src_blocks), _ptr(dst_blocks), _ptr(res_ptr),
                                                    _ptr(res_mask), _ptr(packed_val), _ptr(status), _stream())
    _check(ctx, rc)


def gf_attn_prefill_residual(ctx, params, pool, tables, res_handle, num_items, res_ptr, res_idx, res_val, q, q_ptr,
                             total_q, max_q, o, lse=None) -> None:
    rc = load_library().gf_attn_prefill_residual(ctx, C.byref(params), C.byref(pool), C.byref(tables),
                                                 _ptr(res_handle), num_items, _ptr(res_ptr), _ptr(res_idx),
                                                 _ptr(res_val), _ptr(q), _ptr(q_ptr), total_q, max_q, _ptr(o),
                                                 _ptr(lse), _stream())
    _check(ctx, rc)


def gf_hbm_read_probe(ctx, src, nbytes, wg_sums, num_wg) -> None:
    rc = load_library().gf_hbm_read_probe(ctx, _ptr(src), nbytes, _ptr(wg_sums), num_wg, _stream())
    _check(ctx, rc)


def gf_hbm_tile_probe(ctx, src, tile_bytes, num_src_tiles, tile_ids, num_tiles, wg_sums, num_wg) -> None:
    rc = load_library().gf_hbm_tile_probe(ctx, _ptr(src), tile_bytes, num_src_tiles, _ptr(tile_ids), num_tiles,
                                          _ptr(wg_sums), num_wg, _stream())
    _check(ctx, rc)


def gf_mfma_probe(ctx, operands, operand_bytes, iters, lane_sums, num_wg, softmax_mix=0) -> None:
    rc = load_library().gf_mfma_probe(ctx, _ptr(operands), operand_bytes, iters, softmax_mix, _ptr(lane_sums), num_wg,
                                      _stream())
    _check(ctx, rc)


def gf_attn_decode(ctx, params, pool, tables, q, o, lse=None) -> None:
    rc = load_library().gf_attn_decode(ctx, C.byref(params), C.byref(pool), C.byref(tables), _ptr(q),
                                       _ptr(o), _ptr(lse), _stream())
    _check(ctx, rc)


def gf_attn_decode_residual(ctx, params, pool, tables, res_handle, num_items, res_ptr, res_idx, res_val, q, o,
                            lse=None) -> None:
    rc = load_library().gf_attn_decode_residual(ctx, C.byref(params), C.byref(pool), C.byref(tables), _ptr(res_handle),
                                                num_items, _ptr(res_ptr), _ptr(res_idx), _ptr(res_val), _ptr(q),
                                                _ptr(o), _ptr(lse), _stream())
    _check(ctx, rc)


def gf_attn_decode_shared_residual(ctx, params, pool, graph: gf_graph, path_ptr, path_nodes, num_path_entries, tables,
                                   res_handle, num_items, res_ptr, res_idx, res_val, q, o, lse=None) -> None:
    rc = load_library().gf_attn_decode_shared_residual(ctx, C.byref(params), C.byref(pool), C.byref(graph),
                                                       _ptr(path_ptr), _ptr(path_nodes), num_path_entries,
                                                       C.byref(tables), _ptr(res_handle), num_items, _ptr(res_ptr),
                                                       _ptr(res_idx), _ptr(res_val), _ptr(q), _ptr(o), _ptr(lse),
                                                       _stream())
    _check(ctx, rc)


def gf_attn_decode_shared(ctx, params, pool, graph: gf_graph, path_ptr, path_nodes, num_path_entries, tables, q, o,
                          lse=None) -> None:
    rc = load_library().gf_attn_decode_shared(ctx, C.byref(params), C.byref(pool), C.byref(graph), _ptr(path_ptr),
                                              _ptr(path_nodes), num_path_entries, C.byref(tables), _ptr(q), _ptr(o),
                                              _ptr(lse), _stream())
    _check(ctx, rc)


def gf_kv_apply_residual(ctx, params, k_pool, v_pool, num_pool_blocks, num_items, src_blocks, dst_blocks, res_ptr,
                         res_idx, res_val, status=None, k_scale=None, v_scale=None) -> None:
    rc = load_library().gf_kv_apply_residual(ctx, C.byref(params), _ptr(k_pool), _ptr(v_pool), _ptr(k_scale),
                                             _ptr(v_scale), num_pool_blocks, num_items, _ptr(src_blocks), _ptr(dst_blocks), _ptr(res_ptr),
                                             _ptr(res_idx), _ptr(res_val), _ptr(status), _stream())
    _check(ctx, rc)


def gf_kv_append(ctx, params, k_pool, v_pool, k_scale, v_scale, num_pool_blocks, tables, k_new, v_new, q_ptr,
                 total_q, max_q) -> None:
    rc = load_library().gf_kv_append(ctx, C.byref(params), _ptr(k_pool), _ptr(v_pool), _ptr(k_scale), _ptr(v_scale),
                                     num_pool_blocks, C.byref(tables), _ptr(k_new), _ptr(v_new), _ptr(q_ptr),
                                     total_q, max_q, _stream())
    _check(ctx, rc)


def gf_kv_append_token(ctx, params, k_pool, v_pool, k_scale, v_scale, num_pool_blocks, tables, k_tok, v_tok) -> None:
    rc = load_library().gf_kv_append_token(ctx, C.byref(params), _ptr(k_pool), _ptr(v_pool), _ptr(k_scale),
                                           _ptr(v_scale), num_pool_blocks, C.byref(tables), _ptr(k_tok), _ptr(v_tok),
                                           _stream())
    _check(ctx, rc)


def gf_decode_shared_plan(ctx, params, graph: gf_graph, path_ptr, path_nodes, num_path_entries, tables) -> None:
    rc = load_library().gf_decode_shared_plan(ctx, C.byref(params), C.byref(graph), _ptr(path_ptr), _ptr(path_nodes),
                                              num_path_entries, C.byref(tables), _stream())
    _check(ctx, rc)


def gf_attn_decode_shared_planned(ctx, params, pool, graph: gf_graph, path_ptr, path_nodes, num_path_entries, tables, q,
                                  o, lse=None) -> None:
    rc = load_library().gf_attn_decode_shared_planned(ctx, C.byref(params), C.byref(pool), C.byref(graph),
                                                      _ptr(path_ptr), _ptr(path_nodes), num_path_entries,
                                                      C.byref(tables), _ptr(q), _ptr(o), _ptr(lse), _stream())
    _check(ctx, rc)


def gf_prefix_key(nodes) -> int:
    """Key of a prefix path (host list of node ids)."""
    arr = (C.c_int32 * len(nodes))(*[int(v) for v in nodes])
    return int(load_library().gf_prefix_key(arr, len(nodes)))


def make_residual_dir(key, prev, node, first_item, uses, capacity) -> gf_residual_dir:
    return gf_residual_dir(_ptr(key), _ptr(prev), _ptr(node), _ptr(first_item), _ptr(uses), capacity)


def gf_residual_dir_clear(ctx, d: gf_residual_dir) -> None:
    _check(ctx, load_library().gf_residual_dir_clear(ctx, C.byref(d), _stream()))


def gf_residual_dir_insert(ctx, d: gf_residual_dir, num_pairs, keys, prev, node, first_item, status=None) -> None:
    rc = load_library().gf_residual_dir_insert(ctx, C.byref(d), num_pairs, _ptr(keys), _ptr(prev), _ptr(node),
                                               _ptr(first_item), _ptr(status), _stream())
    _check(ctx, rc)


def gf_resolve_path_residual(ctx, graph: gf_graph, num_req, path_ptr, path_nodes, new_lens, tail_ptr, tail_blocks,
                             max_blocks, num_pool_blocks, block_table, block_ntok, num_blocks, ctx_lens, seq_lens,
                             status, d: gf_residual_dir, trans_count, res_handle, num_fallback) -> None:
    rc = load_library().gf_resolve_path_residual(
        ctx, C.byref(graph), num_req, _ptr(path_ptr), _ptr(path_nodes), _ptr(new_lens), _ptr(tail_ptr),
        _ptr(tail_blocks), max_blocks, num_pool_blocks, _ptr(block_table), _ptr(block_ntok), _ptr(num_blocks),
        _ptr(ctx_lens), _ptr(seq_lens), _ptr(status), C.byref(d), _ptr(trans_count), _ptr(res_handle),
        _ptr(num_fallback), _stream())
    _check(ctx, rc)


def gf_residual_dir_prune(ctx, graph: gf_graph, d: gf_residual_dir, trans_count, min_count, pruned=None) -> None:
    rc = load_library().gf_residual_dir_prune(ctx, C.byref(graph), C.byref(d), _ptr(trans_count), min_count,
                                              _ptr(pruned), _stream())
    _check(ctx, rc)


class BlockPool:
    """gf_block_pool: host-side free list with reference counts over the pool's block ids."""

    def __init__(self, num_blocks: int):
        h = C.c_void_p()
        _check(None, load_library().gf_block_pool_create(C.byref(h), num_blocks))
        self._h = h.value

    def close(self):
        if self._h:
            load_library().gf_block_pool_destroy(self._h)
            self._h = None

    __del__ = close

    @staticmethod
    def _arr(ids):
        return (C.c_int32 * len(ids))(*[int(b) for b in ids])

    def alloc(self, n: int):
        out = (C.c_int32 * max(n, 1))()
        _check(None, load_library().gf_block_pool_alloc(self._h, n, out))
        return list(out[:n])

    def retain(self, ids):
        _check(None, load_library().gf_block_pool_retain(self._h, len(ids), self._arr(ids)))

    def release(self, ids) -> int:
        freed = C.c_int32()
        _check(None, load_library().gf_block_pool_release(self._h, len(ids), self._arr(ids), C.byref(freed)))
        return freed.value

    def stats(self) -> dict:
        f, u, p, t = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int64()
        _check(None, load_library().gf_block_pool_stats(self._h, C.byref(f), C.byref(u), C.byref(t), C.byref(p)))
        return {"free": f.value, "in_use": u.value, "total_refs": t.value, "peak_in_use": p.value}

    def refcount(self, block: int) -> int:
        rc = load_library().gf_block_pool_refcount(self._h, block)
        if rc < 0:
            _check(None, rc)
        return rc


def gf_kv_make_residual(ctx, params, k_pool, v_pool, num_pool_blocks, num_items, base_blocks, full_blocks, energy_share,
                        capacity, res_ptr, res_idx, res_val, status=None) -> None:
    rc = load_library().gf_kv_make_residual(ctx, C.byref(params), _ptr(k_pool), _ptr(v_pool), num_pool_blocks, num_items,
                                            _ptr(base_blocks), _ptr(full_blocks), energy_share, capacity, _ptr(res_ptr),
                                            _ptr(res_idx), _ptr(res_val), _ptr(status), _stream())
    _check(ctx, rc)
