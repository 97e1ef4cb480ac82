"""Thin ctypes binding over the streaming-edge-partitioner calls of include/tig.h (tig_sep_*).
Argument marshalling only; PyTorch supplies device memory and the stream handle."""
from __future__ import annotations

import ctypes
from ctypes import POINTER, Structure, c_double, c_int32, c_int64, c_size_t, c_uint32, c_void_p

import numpy as np

from . import tig

EXPORTS = ("tig_sep_centrality", "tig_sep_topk_scratch_bytes", "tig_sep_top_k", "tig_sep_assign",
           "tig_sep_scratch_bytes", "tig_sep_partition")


class tig_sep_config(Structure):
    _fields_ = [("struct_size", c_uint32), ("num_parts", c_int32), ("beta", c_double), ("top_k", c_double),
                ("lambda_", c_double), ("epsilon", c_double)]


def make_config(num_parts, beta, top_k, lam=1.0, eps=1e-3) -> tig_sep_config:
    return tig_sep_config(ctypes.sizeof(tig_sep_config), num_parts, beta, top_k, lam, eps)


_ready = False


def _lib():
    global _ready
    lib = tig.load_library()
    if not _ready:
        lib.tig_sep_centrality.argtypes = [c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_double, c_void_p, c_void_p]
        lib.tig_sep_topk_scratch_bytes.argtypes = [c_int64]
        lib.tig_sep_topk_scratch_bytes.restype = c_size_t
        lib.tig_sep_top_k.argtypes = [c_void_p, c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
        lib.tig_sep_assign.argtypes = [POINTER(tig_sep_config), c_void_p, c_void_p, c_int64, c_int64, c_void_p,
                                       c_void_p, c_void_p, c_void_p, c_void_p]
        lib.tig_sep_scratch_bytes.argtypes = [c_int64]
        lib.tig_sep_scratch_bytes.restype = c_size_t
        lib.tig_sep_partition.argtypes = [POINTER(tig_sep_config), c_void_p, c_void_p, c_void_p, c_int64, c_int64,
                                          c_void_p, c_size_t, c_void_p] + [c_void_p] * 5
        for n in ("tig_sep_centrality", "tig_sep_top_k", "tig_sep_assign", "tig_sep_partition"):
            getattr(lib, n).restype = ctypes.c_int
        _ready = True
    return lib


def _check(rc):
    if rc != tig.TIG_OK:
        lib = tig.load_library()
        raise tig.TigError(rc, lib.tig_strerror(rc).decode() + " / " + lib.tig_last_error(None).decode())


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(c_void_p)


def assign(cfg, src, dst, num_nodes, cent, is_hub):
    """tig_sep_assign on host arrays.  Returns (edge_part [E] int32, node_parts [N] uint64, part_edges [|P|])."""
    lib = _lib()
    src = np.ascontiguousarray(src, dtype=np.int32)
    dst = np.ascontiguousarray(dst, dtype=np.int32)
    cent = np.ascontiguousarray(cent, dtype=np.float64)
    is_hub = np.ascontiguousarray(is_hub, dtype=np.uint8)
    edge_part = np.empty(len(src), dtype=np.int32)
    node_parts = np.empty(num_nodes, dtype=np.uint64)
    part_edges = np.empty(cfg.num_parts, dtype=np.int64)
    _check(lib.tig_sep_assign(ctypes.byref(cfg), _ptr(src), _ptr(dst), len(src), num_nodes, _ptr(cent), _ptr(is_hub),
                              _ptr(edge_part), _ptr(node_parts), _ptr(part_edges)))
    return edge_part, node_parts, part_edges


def node_lists(node_parts, num_parts):
    """The node loop of Alg. 1 from the masks: (node list per partition, shared-node list)."""
    bits = np.array([bin(int(m)).count("1") for m in node_parts]) if len(node_parts) < 1 << 16 else \
        np.unpackbits(node_parts.view(np.uint8).reshape(-1, 8), axis=1).sum(axis=1)
    shared = np.flatnonzero(bits > 1)
    parts = []
    for p in range(num_parts):
        own = ((node_parts >> np.uint64(p)) & np.uint64(1)).astype(bool) & (bits == 1)
        parts.append(np.flatnonzero(own | (bits > 1)))
    return parts, shared


def centrality(src_dev, dst_dev, ts_dev, num_nodes, beta):
    """tig_sep_centrality on device tensors; returns a device tensor [N] fp64."""
    import torch
    lib = _lib()
    cent = torch.empty(num_nodes, dtype=torch.float64, device=src_dev.device)
    stream = torch.cuda.current_stream(src_dev.device).cuda_stream
    _check(lib.tig_sep_centrality(src_dev.data_ptr(), dst_dev.data_ptr(), ts_dev.data_ptr(), src_dev.numel(),
                                  num_nodes, beta, cent.data_ptr(), stream))
    return cent


def top_k(cent_dev, n_hubs):
    """tig_sep_top_k on a device tensor; returns (hubs [n_hubs] int32, is_hub [N] uint8) device tensors."""
    import torch
    lib = _lib()
    n = cent_dev.numel()
    scratch = torch.empty(lib.tig_sep_topk_scratch_bytes(n) + 256, dtype=torch.uint8, device=cent_dev.device)
    base = (scratch.data_ptr() + 255) // 256 * 256
    hubs = torch.empty(max(n_hubs, 1), dtype=torch.int32, device=cent_dev.device)
    is_hub = torch.empty(n, dtype=torch.uint8, device=cent_dev.device)
    stream = torch.cuda.current_stream(cent_dev.device).cuda_stream
    _check(lib.tig_sep_top_k(cent_dev.data_ptr(), n, n_hubs, hubs.data_ptr(), is_hub.data_ptr(), base,
                             lib.tig_sep_topk_scratch_bytes(n), stream))
    torch.cuda.synchronize()
    return hubs[:n_hubs], is_hub


def partition(cfg, src_dev, dst_dev, ts_dev, num_nodes):
    """tig_sep_partition: device event arrays in, host results out (dict)."""
    import torch
    lib = _lib()
    E = src_dev.numel()
    need = lib.tig_sep_scratch_bytes(num_nodes)
    scratch = torch.empty(need + 256, dtype=torch.uint8, device=src_dev.device)
    base = (scratch.data_ptr() + 255) // 256 * 256
    cent = np.empty(num_nodes, dtype=np.float64)
    is_hub = np.empty(num_nodes, dtype=np.uint8)
    edge_part = np.empty(E, dtype=np.int32)
    node_parts = np.empty(num_nodes, dtype=np.uint64)
    part_edges = np.empty(cfg.num_parts, dtype=np.int64)
    stream = torch.cuda.current_stream(src_dev.device).cuda_stream
    _check(lib.tig_sep_partition(ctypes.byref(cfg), src_dev.data_ptr(), dst_dev.data_ptr(), ts_dev.data_ptr(), E,
                                 num_nodes, base, need, stream, _ptr(cent), _ptr(is_hub), _ptr(edge_part),
                                 _ptr(node_parts), _ptr(part_edges)))
    return {"cent": cent, "is_hub": is_hub, "edge_part": edge_part, "node_parts": node_parts,
            "part_edges": part_edges}
