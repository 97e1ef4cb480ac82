"""Seeded synthetic temporal-interaction-graph workloads (inputs only).

Shared by the CPU oracle's tests and by the GPU library's tests and benchmark.
Holds no model arithmetic: it draws event endpoints, timestamps, edge features,
negatives, weights and warm-start state from a counter-based generator
implemented in ``gen.c`` (compiled with gcc into ``libtig_gen.so``).

The five named workloads take their node / event counts, feature widths and
batch sizes from the paper's dataset table and experimental setup (Sec. III-A);
they are synthetic stand-ins, not copies of any dataset.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtig_gen.so")
_SRC_PATH = os.path.join(_HERE, "gen.c")
_lib = None

SECONDS_30_DAYS = 30 * 24 * 3600.0


def build(force: bool = True) -> str:
    """Compile gen.c -> libtig_gen.so with gcc (OpenMP)."""
    if force or not os.path.exists(_LIB_PATH):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-fvisibility=hidden", "-std=c11",
               "-o", _LIB_PATH, _SRC_PATH, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        build(force=True)
    lib = ctypes.CDLL(_LIB_PATH)
    i64, u64, dbl, ci = ctypes.c_int64, ctypes.c_uint64, ctypes.c_double, ctypes.c_int
    vp = ctypes.c_void_p
    lib.tig_gen_zipf_cdf.argtypes = [i64, dbl, vp]
    lib.tig_gen_endpoints.argtypes = [u64, i64, i64, i64, vp, vp, vp, vp]
    lib.tig_gen_timestamps.argtypes = [u64, i64, dbl, ci, vp]
    lib.tig_gen_normal_f32.argtypes = [u64, u64, i64, vp]
    lib.tig_gen_edge_feat.argtypes = [u64, i64, i64, vp]
    lib.tig_gen_uniform_f32.argtypes = [u64, u64, i64, dbl, dbl, vp]
    lib.tig_gen_negatives.argtypes = [u64, i64, i64, i64, i64, vp, vp]
    lib.tig_gen_warm_state.argtypes = [u64, i64, i64, i64, vp, vp, vp, vp, vp]
    for name in ("tig_gen_zipf_cdf", "tig_gen_endpoints", "tig_gen_timestamps", "tig_gen_normal_f32",
                 "tig_gen_edge_feat", "tig_gen_uniform_f32", "tig_gen_negatives",
                 "tig_gen_warm_state"):
        getattr(lib, name).restype = ci
    _lib = lib
    return lib


def _ptr(a: np.ndarray) -> int:
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError(f"{what} failed with code {rc}")


# --------------------------------------------------------------------------- configs


@dataclass(frozen=True)
class Workload:
    """Shape of one synthetic workload (one entry of the benchmark's config list)."""
    name: str
    index: int                 # 1..5, selects the seed
    n_src: int                 # ids on the source side (all ids when not bipartite)
    n_dst: int                 # ids on the destination side; 0 = not bipartite
    num_events: int
    alpha_src: float
    alpha_dst: float
    span: float                # timestamps lie in [0, span)
    integer_seconds: bool
    feat_dim: int              # F
    mem_dim: int               # M
    time_dim: int              # T
    emb_dim: int               # E
    num_neighbors: int         # K
    num_heads: int             # H
    batch_size: int            # B
    precision: str = "fp32"    # precision variant the config names

    @property
    def num_nodes(self) -> int:
        return self.n_src + self.n_dst

    @property
    def bipartite(self) -> bool:
        return self.n_dst > 0

    @property
    def seed(self) -> int:
        return 0x5EED0000 + self.index

    @property
    def msg_dim(self) -> int:   # D_msg = 2M + T + F
        return 2 * self.mem_dim + self.time_dim + self.feat_dim

    @property
    def attn_dim(self) -> int:  # d_a = M + T
        return self.mem_dim + self.time_dim

    @property
    def kv_dim(self) -> int:    # d_kv = M + F + T
        return self.mem_dim + self.feat_dim + self.time_dim

    def scaled(self, num_events: int | None = None, n_src: int | None = None,
               n_dst: int | None = None, **kw) -> "Workload":
        """A smaller workload of the same shape (for quick tests)."""
        d = dict(self.__dict__)
        if num_events is not None:
            d["num_events"] = num_events
        if n_src is not None:
            d["n_src"] = n_src
        if n_dst is not None:
            d["n_dst"] = n_dst
        d.update(kw)
        return Workload(**d)


WORKLOADS = {
    "c1_tiny": Workload("c1_tiny", 1, 1000, 0, 10_000, 1.2, 1.2, 1e5, False,
                        16, 32, 16, 32, 10, 2, 200, "fp32"),
    "c2_bipartite_medium": Workload("c2_bipartite_medium", 2, 8227, 1000, 157_474, 1.1, 1.3,
                                    SECONDS_30_DAYS, True, 172, 172, 100, 100, 10, 2, 200, "fp32"),
    "c3_bipartite_dense": Workload("c3_bipartite_dense", 3, 10_000, 984, 672_447, 1.2, 1.2,
                                   SECONDS_30_DAYS, True, 172, 172, 100, 100, 20, 2, 2000, "fp32"),
    "c4_million_node": Workload("c4_million_node", 4, 1_000_000, 0, 20_000_000, 1.5, 1.5,
                                SECONDS_30_DAYS, True, 16, 100, 100, 100, 10, 2, 1000, "bf16"),
    "c5_gpu_partition": Workload("c5_gpu_partition", 5, 2_600_000, 0, 250_000_000, 1.6, 1.6,
                                 SECONDS_30_DAYS, True, 8, 100, 100, 100, 10, 2, 4000, "bf16"),
}


# --------------------------------------------------------------------------- graph


@dataclass
class Graph:
    num_nodes: int
    src: np.ndarray        # int32 [E]
    dst: np.ndarray        # int32 [E]
    ts: np.ndarray         # float64 [E], non-decreasing
    edge_feat: np.ndarray  # float32 [E, F]

    @property
    def num_events(self) -> int:
        return int(self.src.shape[0])


def zipf_cdf(n: int, alpha: float) -> np.ndarray:
    cdf = np.empty(n, dtype=np.float64)
    _check(_load().tig_gen_zipf_cdf(n, alpha, _ptr(cdf)), "tig_gen_zipf_cdf")
    return cdf


def make_graph(w: Workload, with_features: bool = True) -> Graph:
    lib = _load()
    E = w.num_events
    src = np.empty(E, dtype=np.int32)
    dst = np.empty(E, dtype=np.int32)
    ts = np.empty(E, dtype=np.float64)
    cdf_s = zipf_cdf(w.n_src, w.alpha_src)
    cdf_d = zipf_cdf(w.n_dst, w.alpha_dst) if w.bipartite else None
    _check(lib.tig_gen_endpoints(w.seed, E, w.n_src, w.n_dst, _ptr(cdf_s),
                                 _ptr(cdf_d) if cdf_d is not None else None, _ptr(src), _ptr(dst)),
           "tig_gen_endpoints")
    _check(lib.tig_gen_timestamps(w.seed, E, w.span, 1 if w.integer_seconds else 0, _ptr(ts)),
           "tig_gen_timestamps")
    if with_features:
        feat = np.empty((E, w.feat_dim), dtype=np.float32)
        _check(lib.tig_gen_edge_feat(w.seed, E, w.feat_dim, _ptr(feat)), "tig_gen_edge_feat")
    else:
        feat = np.zeros((0, w.feat_dim), dtype=np.float32)
    return Graph(w.num_nodes, src, dst, ts, feat)


def make_edge_feat(w: Workload, num_events: int) -> np.ndarray:
    """i.i.d. N(0, 1) fp32 edge features [num_events, F] from the workload's seed (for an event list that
    was not drawn by make_graph, e.g. a partition's sub-graph)."""
    feat = np.empty((num_events, w.feat_dim), dtype=np.float32)
    _check(_load().tig_gen_edge_feat(w.seed, num_events, w.feat_dim, _ptr(feat)), "tig_gen_edge_feat")
    return feat


def make_negatives(w: Workload, g: Graph, first_eid: int, count: int) -> np.ndarray:
    """One negative destination per event of the batch (never equal to the source)."""
    neg = np.empty(count, dtype=np.int32)
    id_lo, id_count = (w.n_src, w.n_dst) if w.bipartite else (0, w.n_src)
    _check(_load().tig_gen_negatives(w.seed, first_eid, count, id_lo, id_count, _ptr(g.src),
                                     _ptr(neg)), "tig_gen_negatives")
    return neg


def make_warm_state(w: Workload, g: Graph, window_first_eid: int):
    """(mem float32 [N, M], last_update float64 [N]) for a window starting mid-stream."""
    mem = np.empty((g.num_nodes, w.mem_dim), dtype=np.float32)
    lu = np.empty(g.num_nodes, dtype=np.float64)
    _check(_load().tig_gen_warm_state(w.seed, g.num_nodes, w.mem_dim, window_first_eid,
                                      _ptr(g.src), _ptr(g.dst), _ptr(g.ts), _ptr(mem), _ptr(lu)),
           "tig_gen_warm_state")
    return mem, lu


# --------------------------------------------------------------------------- weights

# name -> (shape builder, kind); kind: "xavier" matrices, "bias", "time_w", "time_b"
def weight_shapes(M: int, T: int, F: int, E: int) -> dict:
    D = 2 * M + T + F
    da = M + T
    dkv = M + F + T
    return {
        "time_w": (T,), "time_b": (T,),
        "W_i": (3 * M, D), "b_i": (3 * M,), "W_h": (3 * M, M), "b_h": (3 * M,),
        "W_Q": (da, da), "b_Q": (da,), "W_K": (da, dkv), "b_K": (da,),
        "W_V": (da, dkv), "b_V": (da,), "W_O": (da, da), "b_O": (da,),
        "W_m1": (E, da + M), "b_m1": (E,), "W_m2": (E, E), "b_m2": (E,),
        "W_d1": (E, 2 * E), "b_d1": (E,), "w_d2": (E,), "b_d2": (1,),
    }


def make_weights(w: Workload) -> dict:
    """fp32 weights: matrices Xavier-uniform U(-a, a), a = sqrt(6 / (fan_in + fan_out)); biases
    U(-0.1, 0.1); time-encoding frequencies a geometric ladder 1 .. 1e-9; phases U(-pi, pi)."""
    lib = _load()
    out = {}
    for k, (name, shape) in enumerate(weight_shapes(w.mem_dim, w.time_dim, w.feat_dim,
                                                    w.emb_dim).items()):
        n = int(np.prod(shape))
        a = np.empty(shape, dtype=np.float32)
        stream = 100 + k
        if name == "time_w":
            T = shape[0]
            expo = np.arange(T, dtype=np.float64) * (-9.0 / max(T - 1, 1))
            a[:] = (10.0 ** expo).astype(np.float32)
        elif name == "time_b":
            _check(lib.tig_gen_uniform_f32(w.seed, stream, n, -math.pi, math.pi, _ptr(a)), name)
        elif name.startswith("W_") :
            fan_out, fan_in = shape
            lim = math.sqrt(6.0 / (fan_in + fan_out))
            _check(lib.tig_gen_uniform_f32(w.seed, stream, n, -lim, lim, _ptr(a)), name)
        elif name == "w_d2":
            lim = math.sqrt(6.0 / (shape[0] + 1))
            _check(lib.tig_gen_uniform_f32(w.seed, stream, n, -lim, lim, _ptr(a)), name)
        else:
            _check(lib.tig_gen_uniform_f32(w.seed, stream, n, -0.1, 0.1, _ptr(a)), name)
        out[name] = a
    return out


def make_module_weights(w: Workload, updater: str = "gru", embedding: str = "attention") -> dict:
    """Weights of another instance of the general architecture: as make_weights, with the plain
    recurrent cell's shapes (W_i [M, D_msg], b_i [M], W_h [M, M], b_h [M]; Xavier / U(-0.1, 0.1) from
    streams of their own) for updater "rnn", without the attention and merge weights and with a
    decoder over M-wide embeddings for the embeddings that are not "attention", and with the
    time-projection vector time_proj_w [M] ~ U(-1e-6, 1e-6) (time differences reach 2.6e6)."""
    lib = _load()
    M, T, F = w.mem_dim, w.time_dim, w.feat_dim
    D = 2 * M + T + F
    out = dict(make_weights(w))

    def draw(name, shape, stream, lim):
        a = np.empty(shape, dtype=np.float32)
        _check(lib.tig_gen_uniform_f32(w.seed, stream, int(np.prod(shape)), -lim, lim, _ptr(a)), name)
        out[name] = a

    if updater == "rnn":
        draw("W_i", (M, D), 200, math.sqrt(6.0 / (M + D)))
        draw("b_i", (M,), 201, 0.1)
        draw("W_h", (M, M), 202, math.sqrt(6.0 / (2 * M)))
        draw("b_h", (M,), 203, 0.1)
    if embedding != "attention":
        for k in ("W_Q", "b_Q", "W_K", "b_K", "W_V", "b_V", "W_O", "b_O", "W_m1", "b_m1", "W_m2", "b_m2"):
            out.pop(k)
        draw("W_d1", (M, 2 * M), 204, math.sqrt(6.0 / (3 * M)))
        draw("b_d1", (M,), 205, 0.1)
        draw("w_d2", (M,), 206, math.sqrt(6.0 / (M + 1)))
        draw("b_d2", (1,), 207, 0.1)
    if embedding == "time_projection":
        draw("time_proj_w", (M,), 208, 1e-6)
    return out


def make_layer2_weights(w: Workload) -> dict:
    """Weights of a second attention layer (inputs of the first layer's width E where the first layer
    has the state width M): W_Q, W_O [E+T, E+T], W_K, W_V [E+T, E+F+T], W_m1 [E, 2E+T], W_m2 [E, E],
    biases; Xavier-uniform / U(-0.1, 0.1) from streams of their own."""
    lib = _load()
    E, T, F = w.emb_dim, w.time_dim, w.feat_dim
    da, dkv = E + T, E + F + T
    shapes = {"W_Q": (da, da), "b_Q": (da,), "W_K": (da, dkv), "b_K": (da,), "W_V": (da, dkv), "b_V": (da,),
              "W_O": (da, da), "b_O": (da,), "W_m1": (E, da + E), "b_m1": (E,), "W_m2": (E, E), "b_m2": (E,)}
    out = {}
    for k, (name, shape) in enumerate(shapes.items()):
        a = np.empty(shape, dtype=np.float32)
        lim = math.sqrt(6.0 / (shape[0] + shape[1])) if name.startswith("W_") else 0.1
        _check(lib.tig_gen_uniform_f32(w.seed, 220 + k, int(np.prod(shape)), -lim, lim, _ptr(a)), name)
        out[name] = a
    return out


def make_node_feat(w: Workload, num_nodes: int) -> np.ndarray:
    """Static node features [N, M] ~ U(-0.5, 0.5) (the paper's datasets mostly have none: zero vectors)."""
    a = np.empty((num_nodes, w.mem_dim), dtype=np.float32)
    _check(_load().tig_gen_uniform_f32(w.seed, 209, int(a.size), -0.5, 0.5, _ptr(a)), "node_feat")
    return a


def num_params(weights: dict) -> int:
    return int(sum(int(v.size) for v in weights.values()))


def batches(num_events: int, batch_size: int, first: int = 0, stop: int | None = None):
    """Contiguous chronological (first_eid, count) batches; the last may be short."""
    stop = num_events if stop is None else min(stop, num_events)
    e = first
    while e < stop:
        c = min(batch_size, stop - e)
        yield e, c
        e += c
