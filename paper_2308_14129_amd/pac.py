"""Thin ctypes binding over the epoch-machinery calls of include/tig.h (tig_pac_*).
Argument marshalling only; PyTorch supplies device memory and the stream handle."""
from __future__ import annotations

import ctypes
from ctypes import POINTER, Structure, c_int32, c_int64, c_size_t, c_uint32, c_uint64, c_void_p

import numpy as np

from . import tig

EXPORTS = ("tig_pac_combine", "tig_pac_scratch_bytes", "tig_pac_subgraph", "tig_pac_gather", "tig_pac_epoch",
           "tig_pac_sync_shared")


class tig_pac_part(Structure):
    _fields_ = [("struct_size", c_uint32), ("batch", c_int32), ("ctx", c_void_p), ("num_events", c_int64),
                ("neg_dst", c_void_p), ("backup_mem", c_void_p), ("backup_lu", c_void_p), ("out", c_void_p)]


_ready = False


def _lib():
    global _ready
    lib = tig.load_library()
    if not _ready:
        lib.tig_pac_combine.argtypes = [c_void_p, c_int32, c_int32, c_void_p]
        lib.tig_pac_scratch_bytes.argtypes = [c_int64, c_int64]
        lib.tig_pac_scratch_bytes.restype = c_size_t
        lib.tig_pac_subgraph.argtypes = [c_void_p, c_void_p, c_int64, c_void_p, c_int64, c_uint64, c_void_p, c_void_p,
                                         c_void_p, c_void_p, c_size_t, c_void_p]
        lib.tig_pac_gather.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int32, c_void_p, c_int64, c_void_p,
                                       c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
        lib.tig_pac_epoch.argtypes = [POINTER(tig_pac_part), c_int32, POINTER(c_int64)]
        lib.tig_pac_sync_shared.argtypes = [POINTER(c_void_p), c_int32, POINTER(c_void_p), c_int64, c_int32]
        for n in ("tig_pac_combine", "tig_pac_subgraph", "tig_pac_gather", "tig_pac_epoch", "tig_pac_sync_shared"):
            getattr(lib, n).restype = ctypes.c_int
        _ready = True
    return lib


def _check(rc):
    if rc != tig.TIG_OK:
        lib = tig.load_library()
        raise tig.TigError(rc, lib.tig_strerror(rc).decode() + " / " + lib.tig_last_error(None).decode())


def combine(order, num_groups):
    lib = _lib()
    order = np.ascontiguousarray(order, dtype=np.int32)
    out = np.zeros(num_groups, dtype=np.uint64)
    _check(lib.tig_pac_combine(order.ctypes.data, len(order), num_groups, out.ctypes.data))
    return [int(m) for m in out]


def subgraph(src_dev, dst_dev, node_parts_dev, group_mask):
    """Returns (eid [|E_k|] int32 device tensor, local [N] int32 device tensor, |V_k|)."""
    import torch
    lib = _lib()
    E, N = src_dev.numel(), node_parts_dev.numel()
    need = lib.tig_pac_scratch_bytes(E, N)
    scratch = torch.empty(need + 256, dtype=torch.uint8, device=src_dev.device)
    base = (scratch.data_ptr() + 255) // 256 * 256
    eid = torch.empty(max(E, 1), dtype=torch.int32, device=src_dev.device)
    local = torch.empty(N, dtype=torch.int32, device=src_dev.device)
    counts = np.zeros(2, dtype=np.int64)
    stream = torch.cuda.current_stream(src_dev.device).cuda_stream
    _check(lib.tig_pac_subgraph(src_dev.data_ptr(), dst_dev.data_ptr(), E, node_parts_dev.data_ptr(), N,
                                int(group_mask), eid.data_ptr(), local.data_ptr(), counts.ctypes.data, base, need,
                                stream))
    return eid[:int(counts[0])], local, int(counts[1])


def gather(src_dev, dst_dev, ts_dev, feat_dev, eid_dev, local_dev):
    """The sub-graph's event arrays (device tensors): src, dst (local ids), ts, edge features."""
    import torch
    lib = _lib()
    n, F = eid_dev.numel(), feat_dev.shape[1]
    dev = src_dev.device
    s = torch.empty(n, dtype=torch.int32, device=dev)
    d = torch.empty(n, dtype=torch.int32, device=dev)
    t = torch.empty(n, dtype=torch.float64, device=dev)
    f = torch.empty((n, F), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    _check(lib.tig_pac_gather(src_dev.data_ptr(), dst_dev.data_ptr(), ts_dev.data_ptr(), feat_dev.data_ptr(), F,
                              eid_dev.data_ptr(), n, local_dev.data_ptr(), s.data_ptr(), d.data_ptr(), t.data_ptr(),
                              f.data_ptr(), stream))
    return s, d, t, f


def epoch(parts):
    """parts: dicts with ctx (TigContext), batch, num_events, neg (device tensor or None), backup_mem,
    backup_lu (device tensors), out (StepOutputs).  Returns the number of lock-step steps."""
    lib = _lib()
    arr = (tig_pac_part * len(parts))()
    keep = []
    for k, p in enumerate(parts):
        o = p["out"]
        out = tig.tig_out(ctypes.sizeof(tig.tig_out), 0, tig._addr(o.emb), tig._addr(o.score_pos),
                          tig._addr(o.score_neg), tig._addr(o.nbr_node), tig._addr(o.nbr_eid), tig._addr(o.nbr_ts),
                          tig._addr(o.nbr_cnt), tig._addr(o.is_winner))
        keep.append(out)
        arr[k] = tig_pac_part(ctypes.sizeof(tig_pac_part), p["batch"], p["ctx"].handle, p["num_events"],
                              tig._addr(p.get("neg")), p["backup_mem"].data_ptr(), p["backup_lu"].data_ptr(),
                              ctypes.addressof(out))
    steps = c_int64(0)
    _check(lib.tig_pac_epoch(arr, len(parts), ctypes.byref(steps)))
    return steps.value


def sync_shared(ctxs, local_ids_dev, mode="latest"):
    """local_ids_dev[k]: device int32 tensor [n_shared] with the row of every shared node in partition k."""
    lib = _lib()
    n = len(ctxs)
    handles = (c_void_p * n)(*[c.handle for c in ctxs])
    ids = (c_void_p * n)(*[t.data_ptr() for t in local_ids_dev])
    _check(lib.tig_pac_sync_shared(handles, n, ids, local_ids_dev[0].numel(), {"latest": 0, "mean": 1}[mode]))
