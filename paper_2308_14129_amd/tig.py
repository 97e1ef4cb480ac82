"""Thin ctypes binding over the C ABI in include/tig.h.

Argument marshalling only: every step of the batch step runs in the HIP kernels of libtig.so.
PyTorch is used for device allocations and the stream handle, nothing else.  There is no CPU
fallback: if libtig.so is missing or cannot be loaded, importing names from here works but
every call raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, c_double, c_float, c_int32, c_int64, c_size_t, c_uint8, c_uint32, c_void_p

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("TIG_LIB_PATH") or os.path.join(_HERE, "libtig.so")

TIG_OK = 0
TIG_EINVAL, TIG_ERANGE, TIG_EUNSORTED, TIG_ESELFLOOP, TIG_ENOSPACE, TIG_EHIP, TIG_ENOMEM, TIG_EORDER = (
    -1, -2, -3, -4, -5, -6, -7, -8)
TIG_FP32, TIG_BF16_MFMA = 0, 1
PRECISIONS = {"fp32": TIG_FP32, "bf16": TIG_BF16_MFMA}
TIG_UPDATE_FIRST, TIG_DEFERRED = 0, 1
MESSAGE_ORDERS = {"update_first": TIG_UPDATE_FIRST, "deferred": TIG_DEFERRED}

AGGREGATORS = {"last": 0, "mean": 1}
UPDATERS = {"gru": 0, "rnn": 1}
EMBEDDINGS = {"attention": 0, "identity": 1, "time_projection": 2}

WEIGHT_NAMES = ("time_w", "time_b", "W_i", "b_i", "W_h", "b_h", "W_Q", "b_Q", "W_K", "b_K", "W_V",
                "b_V", "W_O", "b_O", "W_m1", "b_m1", "W_m2", "b_m2", "W_d1", "b_d1", "w_d2", "b_d2")


class tig_config(Structure):
    _fields_ = [("struct_size", c_uint32), ("mem_dim", c_int32), ("time_dim", c_int32),
                ("feat_dim", c_int32), ("emb_dim", c_int32), ("num_neighbors", c_int32),
                ("num_heads", c_int32), ("max_batch", c_int32), ("precision", c_int32),
                ("message_order", c_int32)]


class tig_graph(Structure):
    _fields_ = [("struct_size", c_uint32), ("reserved", c_uint32), ("num_nodes", c_int64),
                ("num_events", c_int64), ("src", c_void_p), ("dst", c_void_p), ("ts", c_void_p),
                ("edge_feat", c_void_p)]


class tig_weights(Structure):
    _fields_ = [("struct_size", c_uint32), ("reserved", c_uint32)] + [(n, c_void_p) for n in WEIGHT_NAMES]


LAYER_WEIGHT_NAMES = ("W_Q", "b_Q", "W_K", "b_K", "W_V", "b_V", "W_O", "b_O", "W_m1", "b_m1", "W_m2", "b_m2")


class tig_layer_weights(Structure):
    _fields_ = [("struct_size", c_uint32), ("reserved", c_uint32)] + [(n, c_void_p) for n in LAYER_WEIGHT_NAMES]


class tig_modules(Structure):
    _fields_ = [("struct_size", c_uint32), ("aggregator", c_int32), ("updater", c_int32), ("embedding", c_int32),
                ("node_feat", c_void_p), ("time_proj_w", c_void_p), ("num_layers", c_int32), ("reserved", c_int32),
                ("layer2", POINTER(tig_layer_weights))]


class tig_batch(Structure):
    _fields_ = [("struct_size", c_uint32), ("count", c_int32), ("first_eid", c_int64),
                ("neg_dst", c_void_p)]


class tig_out(Structure):
    _fields_ = [("struct_size", c_uint32), ("reserved", c_uint32), ("emb", c_void_p),
                ("score_pos", c_void_p), ("score_neg", c_void_p), ("nbr_node", c_void_p),
                ("nbr_eid", c_void_p), ("nbr_ts", c_void_p), ("nbr_cnt", c_void_p),
                ("is_winner", c_void_p)]


EXPORTS = ("tig_workspace_bytes", "tig_init", "tig_step", "tig_step_static", "tig_step_profiled", "tig_reset", "tig_state_export",
           "tig_state_import", "tig_destroy", "tig_strerror", "tig_last_error", "tig_launch_info",
           "tig_train_workspace_bytes", "tig_train_attach", "tig_train_step", "tig_train_get",
           "tig_modules_workspace_bytes", "tig_modules_attach")

_lib = None


class TigError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"libtig status {status}: {text}")
        self.status = status


def load_library() -> ctypes.CDLL:
    """Loads libtig.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2308_14129_amd.build`")
    # PyTorch supplies the device memory, so its HIP runtime must be the one this process uses: it
    # is loaded first, and the library's own dependency on the runtime then resolves to it.
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    lib.tig_workspace_bytes.argtypes = [POINTER(tig_config), POINTER(tig_graph), POINTER(c_size_t),
                                        POINTER(c_size_t)]
    lib.tig_init.argtypes = [POINTER(tig_config), POINTER(tig_graph), POINTER(tig_weights), c_void_p,
                             c_size_t, c_void_p, c_size_t, c_void_p, POINTER(c_void_p)]
    lib.tig_step.argtypes = [c_void_p, POINTER(tig_batch), POINTER(tig_out)]
    lib.tig_step_static.argtypes = [c_void_p, POINTER(tig_batch), POINTER(tig_out)]
    lib.tig_step_profiled.argtypes = [c_void_p, POINTER(tig_batch), POINTER(tig_out), POINTER(c_float)]
    lib.tig_reset.argtypes = [c_void_p]
    lib.tig_state_export.argtypes = [c_void_p, c_void_p, c_void_p]
    lib.tig_state_import.argtypes = [c_void_p, c_void_p, c_void_p]
    lib.tig_destroy.argtypes = [c_void_p]
    lib.tig_destroy.restype = None
    lib.tig_strerror.argtypes = [ctypes.c_int]
    lib.tig_strerror.restype = ctypes.c_char_p
    lib.tig_last_error.argtypes = [c_void_p]
    lib.tig_last_error.restype = ctypes.c_char_p
    lib.tig_launch_info.argtypes = [c_void_p, POINTER(c_int32), POINTER(c_int32), POINTER(c_int32)]
    lib.tig_train_workspace_bytes.argtypes = [POINTER(tig_config), POINTER(c_size_t)]
    lib.tig_train_attach.argtypes = [c_void_p, POINTER(tig_weights), c_void_p, c_size_t]
    lib.tig_train_step.argtypes = [c_void_p, POINTER(tig_batch), POINTER(tig_out), c_float, c_void_p]
    lib.tig_train_get.argtypes = [c_void_p, c_int32, POINTER(tig_weights)]
    lib.tig_modules_workspace_bytes.argtypes = [POINTER(tig_config), POINTER(tig_modules), c_int64, POINTER(c_size_t)]
    lib.tig_modules_attach.argtypes = [c_void_p, POINTER(tig_modules), POINTER(tig_weights), c_void_p, c_size_t]
    lib.tig_modules_workspace_bytes.restype = ctypes.c_int
    lib.tig_modules_attach.restype = ctypes.c_int
    for n in ("tig_workspace_bytes", "tig_init", "tig_step", "tig_step_static", "tig_step_profiled", "tig_reset", "tig_state_export",
              "tig_state_import", "tig_launch_info", "tig_train_workspace_bytes", "tig_train_attach", "tig_train_step",
              "tig_train_get"):
        getattr(lib, n).restype = ctypes.c_int
    _lib = lib
    return lib


def make_config(mem_dim, time_dim, feat_dim, emb_dim, num_neighbors, num_heads, max_batch,
                precision="fp32", message_order="update_first") -> tig_config:
    prec = PRECISIONS[precision] if isinstance(precision, str) else int(precision)
    order = MESSAGE_ORDERS[message_order] if isinstance(message_order, str) else int(message_order)
    return tig_config(ctypes.sizeof(tig_config), mem_dim, time_dim, feat_dim, emb_dim, num_neighbors,
                      num_heads, max_batch, prec, order)


def workspace_bytes(cfg: tig_config, num_nodes: int, num_events: int):
    lib = load_library()
    g = tig_graph(ctypes.sizeof(tig_graph), 0, num_nodes, num_events, None, None, None, None)
    p, s = c_size_t(0), c_size_t(0)
    rc = lib.tig_workspace_bytes(ctypes.byref(cfg), ctypes.byref(g), ctypes.byref(p), ctypes.byref(s))
    if rc != TIG_OK:
        raise TigError(rc, lib.tig_strerror(rc).decode())
    return p.value, s.value


def _addr(x) -> int:
    """Address of a numpy array (host) or torch tensor (host or device)."""
    if x is None:
        return 0
    if isinstance(x, np.ndarray):
        if not x.flags["C_CONTIGUOUS"]:
            raise ValueError("array must be C-contiguous")
        return x.ctypes.data
    if not x.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return x.data_ptr()


class StepOutputs:
    """Caller-owned device buffers of one step (torch tensors)."""

    def __init__(self, emb, score_pos, score_neg, nbr_node, nbr_eid, nbr_ts, nbr_cnt, is_winner):
        self.emb, self.score_pos, self.score_neg = emb, score_pos, score_neg
        self.nbr_node, self.nbr_eid, self.nbr_ts, self.nbr_cnt = nbr_node, nbr_eid, nbr_ts, nbr_cnt
        self.is_winner = is_winner


class TigContext:
    """Owns the two device workspaces (torch tensors) and the tig_ctx handle."""

    def __init__(self, cfg: tig_config, num_nodes: int, src, dst, ts, edge_feat, weights: dict,
                 device="cuda:0", stream=None):
        import torch
        self._torch = torch
        self.lib = load_library()
        self.cfg = cfg
        self.device = torch.device(device)
        self.num_nodes = int(num_nodes)
        self.num_events = int(src.shape[0])
        self.M, self.E, self.K = cfg.mem_dim, cfg.emb_dim, cfg.num_neighbors
        pbytes, sbytes = workspace_bytes(cfg, self.num_nodes, self.num_events)
        self.persistent = torch.empty(pbytes, dtype=torch.uint8, device=self.device)
        self.scratch = torch.empty(sbytes, dtype=torch.uint8, device=self.device)
        self.persistent_bytes, self.scratch_bytes = pbytes, sbytes
        with torch.cuda.device(self.device):
            self.stream = stream if stream is not None else torch.cuda.current_stream()
        g = tig_graph(ctypes.sizeof(tig_graph), 0, self.num_nodes, self.num_events, _addr(src),
                      _addr(dst), _addr(ts), _addr(edge_feat))
        w = (tig_weights(ctypes.sizeof(tig_weights), 0, *[_addr(weights[n]) for n in WEIGHT_NAMES])
             if weights is not None else None)
        h = c_void_p(None)
        with torch.cuda.device(self.device):
            rc = self.lib.tig_init(ctypes.byref(cfg), ctypes.byref(g), ctypes.byref(w) if w is not None else None,
                                   self.persistent.data_ptr(), pbytes, self.scratch.data_ptr(), sbytes,
                                   c_void_p(self.stream.cuda_stream), ctypes.byref(h))
        if rc != TIG_OK:
            detail = self.lib.tig_last_error(None).decode()
            raise TigError(rc, self.lib.tig_strerror(rc).decode() + (f" ({detail})" if detail else ""))
        self.handle = h

    # -- helpers ---------------------------------------------------------------------------
    def _check(self, rc: int):
        if rc != TIG_OK:
            raise TigError(rc, self.lib.tig_strerror(rc).decode() + " / " +
                           self.lib.tig_last_error(self.handle).decode())

    def alloc_outputs(self, count: int, with_neg: bool = True, inspect: bool = False) -> StepOutputs:
        torch = self._torch
        Q = (3 if with_neg else 2) * count
        dev = self.device
        emb = torch.empty((Q, self.E), dtype=torch.float32, device=dev)
        sp = torch.empty(count, dtype=torch.float32, device=dev)
        sn = torch.empty(count, dtype=torch.float32, device=dev) if with_neg else None
        if inspect:
            nn_ = torch.empty((Q, self.K), dtype=torch.int32, device=dev)
            ne = torch.empty((Q, self.K), dtype=torch.int32, device=dev)
            nt = torch.empty((Q, self.K), dtype=torch.float64, device=dev)
            nc = torch.empty(Q, dtype=torch.int32, device=dev)
            iw = torch.empty(2 * count, dtype=torch.uint8, device=dev)
        else:
            nn_ = ne = nt = nc = iw = None
        return StepOutputs(emb, sp, sn, nn_, ne, nt, nc, iw)

    # -- the C calls -------------------------------------------------------------------------
    def step(self, first_eid: int, count: int, neg_dst, out: StepOutputs, static: bool = False):
        """Enqueues one batch step on the context's stream (does not synchronise).
        static=True calls tig_step_static (intermediates in the library's static device array)."""
        b = tig_batch(ctypes.sizeof(tig_batch), count, first_eid, _addr(neg_dst))
        o = tig_out(ctypes.sizeof(tig_out), 0, _addr(out.emb), _addr(out.score_pos), _addr(out.score_neg),
                    _addr(out.nbr_node), _addr(out.nbr_eid), _addr(out.nbr_ts), _addr(out.nbr_cnt),
                    _addr(out.is_winner))
        fn = self.lib.tig_step_static if static else self.lib.tig_step
        self._check(fn(self.handle, ctypes.byref(b), ctypes.byref(o)))

    KERNEL_NAMES = ("k_scatter", "k_select", "k_prepare", "k_gru", "k_embed", "k_closing")

    def step_profiled(self, first_eid: int, count: int, neg_dst, out: StepOutputs):
        """One step with HIP events around every kernel; returns the durations in ms, one per
        entry of KERNEL_NAMES (0 for a kernel the step did not need)."""
        b = tig_batch(ctypes.sizeof(tig_batch), count, first_eid, _addr(neg_dst))
        o = tig_out(ctypes.sizeof(tig_out), 0, _addr(out.emb), _addr(out.score_pos), _addr(out.score_neg),
                    _addr(out.nbr_node), _addr(out.nbr_eid), _addr(out.nbr_ts), _addr(out.nbr_cnt),
                    _addr(out.is_winner))
        ms = (c_float * len(self.KERNEL_NAMES))()
        self._check(self.lib.tig_step_profiled(self.handle, ctypes.byref(b), ctypes.byref(o), ms))
        return [float(x) for x in ms]

    # -- other instances of the general architecture -------------------------------------------
    def modules_attach(self, weights: dict, aggregator="last", updater="gru", embedding="attention", node_feat=None,
                       layers=1, layer2=None):
        """Allocates the workspace of a module selection and attaches it with `weights` (a dict that may
        lack the attention / merge weights unless the embedding is attention; "time_proj_w" for the
        time projection; `layer2`: the dict of a second attention layer's weights for layers = 2)."""
        torch = self._torch
        l2 = None
        if layer2 is not None:
            l2 = tig_layer_weights(ctypes.sizeof(tig_layer_weights), 0, *[_addr(layer2[k]) for k in LAYER_WEIGHT_NAMES])
        m = tig_modules(ctypes.sizeof(tig_modules), AGGREGATORS[aggregator], UPDATERS[updater], EMBEDDINGS[embedding],
                        _addr(node_feat), _addr(weights.get("time_proj_w")), layers, 0,
                        ctypes.pointer(l2) if l2 is not None else None)
        n = c_size_t(0)
        self._check(self.lib.tig_modules_workspace_bytes(ctypes.byref(self.cfg), ctypes.byref(m), self.num_nodes,
                                                         ctypes.byref(n)))
        self.mods_ws = torch.empty(n.value, dtype=torch.uint8, device=self.device)
        w = tig_weights(ctypes.sizeof(tig_weights), 0, *[_addr(weights.get(k)) for k in WEIGHT_NAMES])
        self._check(self.lib.tig_modules_attach(self.handle, ctypes.byref(m), ctypes.byref(w), self.mods_ws.data_ptr(),
                                                n.value))

    # -- training ----------------------------------------------------------------------------
    def train_attach(self, weights: dict):
        """Allocates the training workspace and makes `weights` the master weights."""
        torch = self._torch
        n = c_size_t(0)
        self._check(self.lib.tig_train_workspace_bytes(ctypes.byref(self.cfg), ctypes.byref(n)))
        self.train_ws = torch.empty(n.value, dtype=torch.uint8, device=self.device)
        w = tig_weights(ctypes.sizeof(tig_weights), 0, *[_addr(weights[k]) for k in WEIGHT_NAMES])
        self._check(self.lib.tig_train_attach(self.handle, ctypes.byref(w), self.train_ws.data_ptr(), n.value))
        self._shapes = {k: np.asarray(weights[k]).shape for k in WEIGHT_NAMES}
        self._loss = torch.zeros(1, dtype=torch.float32, device=self.device)

    def train_step(self, first_eid: int, count: int, neg_dst, out: StepOutputs, lr: float):
        """Enqueues one training step; returns the device tensor [1] that receives the loss."""
        b = tig_batch(ctypes.sizeof(tig_batch), count, first_eid, _addr(neg_dst))
        o = tig_out(ctypes.sizeof(tig_out), 0, _addr(out.emb), _addr(out.score_pos), _addr(out.score_neg),
                    _addr(out.nbr_node), _addr(out.nbr_eid), _addr(out.nbr_ts), _addr(out.nbr_cnt),
                    _addr(out.is_winner))
        self._check(self.lib.tig_train_step(self.handle, ctypes.byref(b), ctypes.byref(o), c_float(lr),
                                            self._loss.data_ptr()))
        return self._loss

    def train_get(self, what: str) -> dict:
        """The master weights ("weights") or the last step's gradients ("grads") as host arrays."""
        arrs = {k: np.empty(self._shapes[k], dtype=np.float32) for k in WEIGHT_NAMES}
        w = tig_weights(ctypes.sizeof(tig_weights), 0, *[arrs[k].ctypes.data for k in WEIGHT_NAMES])
        self._check(self.lib.tig_train_get(self.handle, {"weights": 0, "grads": 1}[what], ctypes.byref(w)))
        return arrs

    def step_raw(self, batch: tig_batch, out: tig_out) -> int:
        return self.lib.tig_step(self.handle, ctypes.byref(batch), ctypes.byref(out))

    def reset(self):
        self._check(self.lib.tig_reset(self.handle))

    def state_export(self):
        mem = np.empty((self.num_nodes, self.M), dtype=np.float32)
        lu = np.empty(self.num_nodes, dtype=np.float64)
        self._check(self.lib.tig_state_export(self.handle, mem.ctypes.data, lu.ctypes.data))
        return mem, lu

    def state_import(self, mem, last_update):
        self._check(self.lib.tig_state_import(self.handle, _addr(mem), _addr(last_update)))

    def launch_info(self):
        k, g, e = c_int32(0), c_int32(0), c_int32(0)
        self._check(self.lib.tig_launch_info(self.handle, ctypes.byref(k), ctypes.byref(g), ctypes.byref(e)))
        return {"kernels_per_step": k.value, "gru_lds_bytes": g.value, "embed_lds_bytes": e.value}

    def close(self):
        if getattr(self, "handle", None):
            self.lib.tig_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
