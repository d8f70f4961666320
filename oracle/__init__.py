"""ctypes front end of the CPU oracle (``acrobat_oracle.c``).  TEST INFRASTRUCTURE ONLY.

May be imported by ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline``
leg of ``bench.py`` and by nothing else.  It shares no code with the GPU path, and
never imports it.  All results are float64; inputs are the float32 arrays the
GPU path receives, converted exactly.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "acrobat_oracle.c")
_LIB = os.path.join(_HERE, "libacrobat_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no fast-math: summation order is as written)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC,
             "-lm", "-lpthread"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
    return _lib


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def default_threads() -> int:
    try:
        return max(1, len(os.sched_getaffinity(0)))
    except AttributeError:  # pragma: no cover
        return os.cpu_count() or 1


def treelstm(w: dict, nthreads: int = 1, topo: bool = False):
    """Evaluate a TreeLSTM batch (fields as made by workloads.treelstm_workload). Returns h, c [N,H] f64."""
    lib = _load()
    H, D = int(w["H"]), int(w["D"])
    off, left, right, tok = _i32(w["tree_off"]), _i32(w["left"]), _i32(w["right"]), _i32(w["token"])
    N = int(off[-1])
    emb, Wl, bl, U, b = (_f32(w[k]) for k in ("emb", "W_leaf", "b_leaf", "U", "b"))
    h = np.full((N, H), np.nan, dtype=np.float64)
    c = np.full((N, H), np.nan, dtype=np.float64)
    args = [C.c_int(int(w["n_trees"])), _p(off), _p(left), _p(right), _p(tok), C.c_int(H), C.c_int(D),
            _p(emb), _p(Wl), _p(bl), _p(U), _p(b), _p(h), _p(c)]
    if topo:
        lib.oracle_treelstm_topo(*args)
    else:
        lib.oracle_treelstm(*args, C.c_int(int(nthreads)))
    return h, c


def tree_depths(trees: dict):
    lib = _load()
    off, left, right = _i32(trees["tree_off"]), _i32(trees["left"]), _i32(trees["right"])
    N = int(off[-1])
    depth = np.empty(N, dtype=np.int32)
    n_levels = lib.oracle_tree_depths(C.c_int(int(trees["n_trees"])), _p(off), _p(left), _p(right),
                                      _p(depth))
    return int(n_levels), depth


def tree_schedule(trees: dict):
    """Returns (level_off[n_levels+1], level_nodes[N], lrow[N], rrow[N])."""
    lib = _load()
    off, left, right = _i32(trees["tree_off"]), _i32(trees["left"]), _i32(trees["right"])
    N = int(off[-1])
    level_off = np.zeros(N + 1, dtype=np.int32)
    level_nodes = np.empty(N, dtype=np.int32)
    lrow = np.empty(N, dtype=np.int32)
    rrow = np.empty(N, dtype=np.int32)
    n_levels = lib.oracle_tree_schedule(C.c_int(int(trees["n_trees"])), _p(off), _p(left), _p(right),
                                        _p(level_off), _p(level_nodes), _p(lrow), _p(rrow))
    return level_off[: n_levels + 1].copy(), level_nodes, lrow, rrow


def mvrnn(w: dict, nthreads: int = 1):
    """Evaluate an MV-RNN batch. Returns vec [N,d], mat [N,d,d] f64 (leaf rows = table rows)."""
    lib = _load()
    d = int(w["d"])
    off, left, right, tok = _i32(w["tree_off"]), _i32(w["left"]), _i32(w["right"]), _i32(w["token"])
    N = int(off[-1])
    vt, mt, W, WM = (_f32(w[k]) for k in ("vec_tab", "mat_tab", "W", "WM"))
    vec = np.full((N, d), np.nan, dtype=np.float64)
    mat = np.full((N, d, d), np.nan, dtype=np.float64)
    lib.oracle_mvrnn(C.c_int(int(w["n_trees"])), _p(off), _p(left), _p(right), _p(tok), C.c_int(d),
                     _p(vt), _p(mt), _p(W), _p(WM), _p(vec), _p(mat), C.c_int(int(nthreads)))
    return vec, mat


def varlen_lstm(w: dict, nthreads: int = 1):
    """Evaluate a variable-length LSTM batch. Returns h, c [sum len, H] f64."""
    lib = _load()
    H, D = int(w["H"]), int(w["D"])
    lens = _i32(w["len"])
    total = int(lens.sum())
    x, Wx, Wh, b = (_f32(w[k]) for k in ("x", "Wx", "Wh", "b"))
    h = np.full((total, H), np.nan, dtype=np.float64)
    c = np.full((total, H), np.nan, dtype=np.float64)
    lib.oracle_varlen_lstm(C.c_int(int(w["n_seq"])), _p(lens), C.c_int(H), C.c_int(D), _p(x), _p(Wx),
                           _p(Wh), _p(b), _p(h), _p(c), C.c_int(int(nthreads)))
    return h, c


def seq_schedule(lens):
    lib = _load()
    lens = _i32(lens)
    total = int(lens.sum())
    tmax = int(lens.max()) if lens.size else 0
    level_off = np.zeros(tmax + 1, dtype=np.int32)
    level_rows = np.empty(total, dtype=np.int32)
    n = lib.oracle_seq_schedule(C.c_int(lens.size), _p(lens), _p(level_off), _p(level_rows))
    assert n == tmax
    return level_off, level_rows


def birnn(w: dict, nthreads: int = 1):
    """Evaluate a bidirectional-RNN batch. Returns hf, hb [sum len, H] and y [sum len, n_out] (f64)."""
    lib = _load()
    H, D, n_out = int(w["H"]), int(w["D"]), int(w["n_out"])
    lens = _i32(w["len"])
    total = int(lens.sum())
    names = ("x", "fWx", "fWh", "fb", "finit", "bWx", "bWh", "bb", "binit", "C", "cb")
    arrs = [_f32(w[k]) for k in names]
    hf = np.full((total, H), np.nan, dtype=np.float64)
    hb = np.full((total, H), np.nan, dtype=np.float64)
    y = np.full((total, n_out), np.nan, dtype=np.float64)
    lib.oracle_birnn(C.c_int(int(w["n_seq"])), _p(lens), C.c_int(H), C.c_int(D), C.c_int(n_out),
                     *[_p(a) for a in arrs], _p(hf), _p(hb), _p(y), C.c_int(int(nthreads)))
    return hf, hb, y


def phase_schedule(prod_lists, phase):
    """Generic (phase, depth, id) schedule of an explicit dataflow graph.
    prod_lists[n] = producers of node n.  Returns (depth[n], order[n], batch_off)."""
    lib = _load()
    n = len(prod_lists)
    prod_off = np.zeros(n + 1, np.int32)
    prod_off[1:] = np.cumsum([len(p) for p in prod_lists])
    prod = _i32(np.concatenate([np.asarray(p, np.int32) for p in prod_lists]) if prod_off[-1] else np.zeros(0, np.int32))
    phase = _i32(phase)
    depth = np.empty(n, np.int32)
    order = np.empty(n, np.int32)
    batch_off = np.zeros(n + 1, np.int32)
    nb = lib.oracle_phase_schedule(C.c_int(n), _p(prod_off), _p(prod), _p(phase), _p(depth), _p(order), _p(batch_off))
    return depth, order, batch_off[: nb + 1].copy()


def mix64(z: int) -> int:
    lib = _load()
    lib.oracle_mix64.restype = C.c_uint64
    return int(lib.oracle_mix64(C.c_uint64(z & (2**64 - 1))))


def drnn_decide(key: int, depth: int, k: int, is_root: bool, w: dict):
    """(has_child, has_sibling, label) of the node at position key `key`."""
    lib = _load()
    out = np.zeros(3, np.int32)
    lib.oracle_drnn_decide(C.c_uint64(key), C.c_int(depth), C.c_int(k), C.c_int(int(is_root)), C.c_int(int(w["max_depth"])),
                           C.c_int(int(w["max_children"])), C.c_double(float(w["p_child"])), C.c_double(float(w["p_sibling"])),
                           C.c_int(int(w["n_labels"])), _p(out))
    return int(out[0]), int(out[1]), int(out[2])


def drnn_keys(seed: int, inst: int, path=()):
    """Position key of the node reached from the root of instance `inst` by the child indices in `path`."""
    lib = _load()
    lib.oracle_drnn_root_key.restype = C.c_uint64
    lib.oracle_drnn_child_key.restype = C.c_uint64
    key = lib.oracle_drnn_root_key(C.c_uint64(seed), C.c_int(inst))
    for k in path:
        key = lib.oracle_drnn_child_key(C.c_uint64(key), C.c_int(int(k)))
    return int(key)


def drnn(w: dict, cap: int | None = None):
    """Generate the trees of a doubly-recurrent-network batch (fields as made by
    workloads.drnn_workload).  Returns a dict: structure arrays inst, parent, prev, sib_index,
    depth, label (int32, pre-order per instance) and states a, f, g [N,H], y [N,n_out] (f64)."""
    lib = _load()
    H, n_out, n_inst = int(w["H"]), int(w["n_out"]), int(w["n_inst"])
    cap = int(cap if cap is not None else w["cap"])
    names = ("x0", "emb", "Wa", "ba", "Wf", "bf", "Wp", "bp", "Wo", "bo")
    arrs = [_f32(w[k]) for k in names]
    ints = {k: np.full(cap, -7, np.int32) for k in ("inst", "parent", "prev", "sib_index", "depth", "label")}
    st = {k: np.full((cap, H), np.nan) for k in ("a", "f", "g")}
    y = np.full((cap, n_out), np.nan)
    n = lib.oracle_drnn(C.c_int(n_inst), C.c_int(H), C.c_int(int(w["n_labels"])), C.c_int(n_out),
                        *[_p(a) for a in arrs], C.c_uint64(int(w["seed_decisions"])), C.c_int(int(w["max_depth"])),
                        C.c_int(int(w["max_children"])), C.c_double(float(w["p_child"])), C.c_double(float(w["p_sibling"])),
                        C.c_int(int(bool(w.get("from_scores", False)))), C.c_int(cap), *[_p(ints[k]) for k in ("inst", "parent", "prev", "sib_index", "depth", "label")],
                        _p(st["a"]), _p(st["f"]), _p(st["g"]), _p(y))
    if n < 0:
        raise ValueError("drnn: more than cap nodes")
    out = {k: v[:n].copy() for k, v in ints.items()}
    out.update({k: v[:n].copy() for k, v in st.items()})
    out["y"] = y[:n].copy()
    return out
