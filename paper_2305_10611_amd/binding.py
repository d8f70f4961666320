"""Thin ctypes binding of libacrobat.so: same names as include/acrobat.h, argument
marshalling only.  Every step of the hot path runs inside the library; there is no Python
or CPU fallback - if the library is missing, importing this module raises."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch  # noqa: F401  (first: the library must bind to the HIP runtime PyTorch ships, one runtime per process)

from . import build as _build

OK, EINVAL, ESTRUCT, ENOMEM, EHIP, ETIMEOUT = 0, -1, -2, -3, -4, -5
K_TREE_LEAF, K_TREE_INTERNAL, K_MVRNN_LEVEL, K_MVRNN_LEAFCOPY, K_LSTM_INPUT, K_LSTM_STEP = 1, 2, 3, 4, 5, 6
K_RNN_INPUT, K_RNN_STEP, K_RNN_OUTPUT, K_SPLITK_REDUCE = 7, 8, 9, 10
K_GATHER, K_DFG_BUCKET, K_LSTM_PERSISTENT, K_MVRNN_PERSISTENT, K_RNN_PERSISTENT = 11, 12, 13, 14, 15


class AcrobatError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"acrobat error {code}: {msg}")
        self.code = code


class acrobat_trees(C.Structure):
    _fields_ = [("n_trees", C.c_int32), ("tree_off", C.c_void_p), ("left", C.c_void_p),
                ("right", C.c_void_p), ("token", C.c_void_p)]


class acrobat_launch_record(C.Structure):
    _fields_ = [("kind", C.c_int32), ("level", C.c_int32), ("n", C.c_int32), ("tile", C.c_int32), ("ksplit", C.c_int32), ("ms", C.c_float)]


class acrobat_rnn_dir(C.Structure):
    _fields_ = [("Wx", C.c_void_p), ("Wh", C.c_void_p), ("b", C.c_void_p), ("h_init", C.c_void_p)]


class acrobat_op_desc(C.Structure):
    _fields_ = [("epilogue", C.c_int32), ("H", C.c_int32), ("nseg", C.c_int32), ("kseg", C.c_int32),
                ("src0", C.c_void_p), ("ld0", C.c_int32), ("src1", C.c_void_p), ("ld1", C.c_int32),
                ("W", C.c_void_p), ("ldw", C.c_int32), ("bias", C.c_void_p), ("h", C.c_void_p), ("c", C.c_void_p),
                ("cprev_src", C.c_void_p), ("zadd", C.c_void_p), ("zout", C.c_void_p),
                ("n_cols", C.c_int32), ("y", C.c_void_p), ("ldo", C.c_int32),
                ("src0_rows", C.c_int32), ("src1_rows", C.c_int32), ("out_rows", C.c_int32), ("W2", C.c_void_p)]


EPI_TREE_LEAF, EPI_TREE_INTERNAL, EPI_LSTM_STEP, EPI_STORE_Z, EPI_RNN_STEP, EPI_RELU_OUT, EPI_STORE_Z1, EPI_MVRNN = range(8)
TDC_SEQUENTIAL, TDC_INSTANCE_FIBERS, TDC_FORK_JOIN = 0, 1, 2


class acrobat_drnn_decisions(C.Structure):
    _fields_ = [("seed", C.c_uint64), ("max_depth", C.c_int32), ("max_children", C.c_int32),
                ("p_child", C.c_float), ("p_sibling", C.c_float), ("from_scores", C.c_int32)]


class acrobat_drnn_params(C.Structure):
    _fields_ = [("H", C.c_int32), ("n_labels", C.c_int32), ("n_out", C.c_int32), ("emb", C.c_void_p),
                ("Wa", C.c_void_p), ("ba", C.c_void_p), ("Wf", C.c_void_p), ("bf", C.c_void_p),
                ("Wp", C.c_void_p), ("bp", C.c_void_p), ("Wo", C.c_void_p), ("bo", C.c_void_p)]


DRNN_TREE_FIELDS = ("inst", "parent", "prev", "sib_index", "depth", "label", "round")


class acrobat_drnn_trees(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in DRNN_TREE_FIELDS]


class acrobat_drnn_stats(C.Structure):
    _fields_ = [("n_nodes", C.c_int32), ("n_rounds", C.c_int32), ("n_buckets", C.c_int32), ("n_fibers", C.c_int32),
                ("n_ghosts", C.c_int32)]

EXPORTS = (
    "acrobat_create", "acrobat_destroy", "acrobat_last_error", "acrobat_strerror",
    "acrobat_schedule_trees", "acrobat_schedule_seqs", "acrobat_treelstm_forward",
    "acrobat_mvrnn_forward", "acrobat_varlen_lstm_forward", "acrobat_last_schedule",
    "acrobat_set_profiling", "acrobat_last_profile", "acrobat_schedule_birnn", "acrobat_birnn_forward",
    "acrobat_set_gather_fusion", "acrobat_set_tuning", "acrobat_treelstm_forward_noalloc",
    "acrobat_set_persistent", "acrobat_device_status", "acrobat_sync_probe",
    "acrobat_dfg_create", "acrobat_dfg_destroy", "acrobat_dfg_last_error", "acrobat_dfg_register_op", "acrobat_dfg_clear", "acrobat_dfg_invoke",
    "acrobat_dfg_build_treelstm", "acrobat_dfg_run", "acrobat_dfg_schedule", "acrobat_dfg_ghost",
    "acrobat_drnn_forward", "acrobat_drnn_schedule",
)


def _load():
    if not os.path.exists(_build.LIB):
        _build.build()
    lib = C.CDLL(_build.LIB)
    vp, i32 = C.c_void_p, C.c_int32
    lib.acrobat_create.argtypes = [C.POINTER(vp), C.c_int]
    lib.acrobat_destroy.argtypes = [vp]
    lib.acrobat_destroy.restype = None
    lib.acrobat_last_error.argtypes = [vp]
    lib.acrobat_last_error.restype = C.c_char_p
    lib.acrobat_strerror.argtypes = [C.c_int]
    lib.acrobat_strerror.restype = C.c_char_p
    lib.acrobat_schedule_trees.argtypes = [C.POINTER(acrobat_trees), i32, C.POINTER(i32), vp, vp, vp, vp]
    lib.acrobat_schedule_seqs.argtypes = [i32, vp, C.POINTER(i32), vp, vp]
    lib.acrobat_treelstm_forward.argtypes = [vp, C.POINTER(acrobat_trees), i32, i32, i32] + [vp] * 8
    lib.acrobat_treelstm_forward_noalloc.argtypes = lib.acrobat_treelstm_forward.argtypes
    lib.acrobat_mvrnn_forward.argtypes = [vp, C.POINTER(acrobat_trees), i32, i32] + [vp] * 6 + [i32, vp]
    lib.acrobat_varlen_lstm_forward.argtypes = [vp, i32, vp, i32, i32] + [vp] * 7
    lib.acrobat_schedule_birnn.argtypes = [i32, vp, C.POINTER(i32), vp, vp]
    lib.acrobat_birnn_forward.argtypes = ([vp, i32, vp, i32, i32, i32, vp, C.POINTER(acrobat_rnn_dir),
                                           C.POINTER(acrobat_rnn_dir)] + [vp] * 6)
    lib.acrobat_dfg_create.argtypes = [vp, C.POINTER(vp)]
    lib.acrobat_dfg_destroy.argtypes = [vp]
    lib.acrobat_dfg_destroy.restype = None
    lib.acrobat_dfg_last_error.argtypes = [vp]
    lib.acrobat_dfg_last_error.restype = C.c_char_p
    lib.acrobat_dfg_register_op.argtypes = [vp, C.POINTER(acrobat_op_desc), C.POINTER(i32)]
    lib.acrobat_dfg_clear.argtypes = [vp]
    lib.acrobat_dfg_invoke.argtypes = [vp] + [i32] * 8 + [C.POINTER(i32)]
    lib.acrobat_dfg_build_treelstm.argtypes = [vp, C.POINTER(acrobat_trees), i32, i32, i32]
    lib.acrobat_dfg_ghost.argtypes = [vp, i32, i32, i32, C.POINTER(i32)]
    lib.acrobat_drnn_forward.argtypes = ([vp, i32, vp, C.POINTER(acrobat_drnn_params), C.POINTER(acrobat_drnn_decisions),
                                          i32, i32, i32, C.POINTER(acrobat_drnn_trees)] + [vp] * 4 +
                                         [C.POINTER(acrobat_drnn_stats), vp])
    lib.acrobat_drnn_schedule.argtypes = [i32, i32, C.POINTER(acrobat_drnn_decisions), i32, i32, i32,
                                          C.POINTER(acrobat_drnn_trees), C.POINTER(acrobat_drnn_stats)]
    lib.acrobat_dfg_run.argtypes = [vp, vp]
    lib.acrobat_dfg_schedule.argtypes = [vp, C.POINTER(i32), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp)]
    lib.acrobat_last_schedule.argtypes = [vp, C.POINTER(i32), C.POINTER(vp), C.POINTER(vp)]
    lib.acrobat_set_profiling.argtypes = [vp, i32]
    lib.acrobat_set_gather_fusion.argtypes = [vp, i32]
    lib.acrobat_set_tuning.argtypes = [vp, i32, i32, i32]
    lib.acrobat_set_persistent.argtypes = [vp, i32, i32]
    lib.acrobat_device_status.argtypes = [vp]
    lib.acrobat_sync_probe.argtypes = [vp] + [i32] * 8 + [C.POINTER(C.c_double), C.POINTER(C.c_double), vp]
    lib.acrobat_last_profile.argtypes = [vp, C.POINTER(i32), C.POINTER(C.POINTER(acrobat_launch_record))]
    return lib


lib = _load()


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _hp(a):  # host pointer of a numpy array (None -> NULL)
    return None if a is None else a.ctypes.data


def _dp(t):  # device pointer of a torch tensor (None -> NULL)
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous() and t.dtype.is_floating_point and t.element_size() == 4
    return t.data_ptr()


def _trees_struct(trees: dict):
    keep = [_i32(trees["tree_off"]), _i32(trees["left"]), _i32(trees["right"]),
            None if trees.get("token") is None else _i32(trees["token"])]
    st = acrobat_trees(int(trees["n_trees"]), *(_hp(a) for a in keep))
    return st, keep


def acrobat_strerror(code: int) -> str:
    return lib.acrobat_strerror(code).decode()


def acrobat_schedule_trees(trees: dict, vocab: int = -1):
    """-> (rc, level_off[n_levels+1], level_nodes[N], lrow[N], rrow[N])"""
    st, keep = _trees_struct(trees)
    N = int(keep[0][-1]) if keep[0].size else 0
    level_off = np.zeros(max(N, 0) + 1, np.int32)
    level_nodes, lrow, rrow = (np.empty(max(N, 0), np.int32) for _ in range(3))
    n_levels = C.c_int32(0)
    rc = lib.acrobat_schedule_trees(C.byref(st), vocab, C.byref(n_levels), _hp(level_off), _hp(level_nodes),
                                    _hp(lrow), _hp(rrow))
    if rc != OK:
        return rc, None, None, None, None
    return rc, level_off[: n_levels.value + 1].copy(), level_nodes, lrow, rrow


def prepared_schedule_trees(trees: dict, vocab: int = -1):
    """-> a callable that runs acrobat_schedule_trees on `trees` with its arguments marshalled and its output
    arrays allocated once, for timing the library call itself; it returns the C return code."""
    st, keep = _trees_struct(trees)
    N = int(keep[0][-1]) if keep[0].size else 0
    out = [np.zeros(max(N, 0) + 1, np.int32)] + [np.empty(max(N, 0), np.int32) for _ in range(3)]
    n_levels = C.c_int32(0)
    args = (C.byref(st), vocab, C.byref(n_levels), *(_hp(a) for a in out))

    def call(_keep=(st, keep, out, n_levels)):
        return lib.acrobat_schedule_trees(*args)
    return call


def acrobat_schedule_seqs(lens):
    """-> (rc, level_off[n_levels+1], level_rows[sum len])"""
    lens = _i32(lens)
    tmax = int(lens.max()) if lens.size and lens.max() > 0 else 0
    total = int(np.maximum(lens, 0).sum())
    level_off = np.zeros(tmax + 1, np.int32)
    level_rows = np.empty(total, np.int32)
    n_levels = C.c_int32(0)
    rc = lib.acrobat_schedule_seqs(int(lens.size), _hp(lens), C.byref(n_levels), _hp(level_off), _hp(level_rows))
    if rc != OK:
        return rc, None, None
    return rc, level_off, level_rows


def acrobat_schedule_birnn(lens):
    """-> (rc, level_off[n_levels+1], level_codes[3 sum len])"""
    lens = _i32(lens)
    tmax = int(lens.max()) if lens.size and lens.max() > 0 else 0
    total = int(np.maximum(lens, 0).sum())
    level_off = np.zeros(tmax + 2, np.int32)
    level_codes = np.empty(3 * total, np.int32)
    n_levels = C.c_int32(0)
    rc = lib.acrobat_schedule_birnn(int(lens.size), _hp(lens), C.byref(n_levels), _hp(level_off), _hp(level_codes))
    if rc != OK:
        return rc, None, None
    return rc, level_off[: n_levels.value + 1].copy(), level_codes


def _drnn_decisions(w: dict):
    return acrobat_drnn_decisions(int(w["seed_decisions"]), int(w["max_depth"]), int(w["max_children"]),
                                  float(w["p_child"]), float(w["p_sibling"]), int(bool(w.get("from_scores", False))))


def _drnn_outputs(max_nodes: int):
    arrs = {k: np.empty(max(max_nodes, 1), np.int32) for k in DRNN_TREE_FIELDS}
    return arrs, acrobat_drnn_trees(*(_hp(arrs[k]) for k in DRNN_TREE_FIELDS))


def _drnn_result(arrs, stats):
    n = stats.n_nodes
    trees = {k: v[:n].copy() for k, v in arrs.items()}
    return trees, {k: getattr(stats, k) for k, _ in acrobat_drnn_stats._fields_}


def acrobat_drnn_schedule(w: dict, mode=TDC_FORK_JOIN, use_ghosts=True, max_nodes=None):
    """Host only. -> (rc, trees dict of int32 arrays, stats dict)"""
    max_nodes = int(w["cap"] if max_nodes is None else max_nodes)
    arrs, out = _drnn_outputs(max_nodes)
    dec, stats = _drnn_decisions(w), acrobat_drnn_stats()
    rc = lib.acrobat_drnn_schedule(int(w["n_inst"]), int(w["n_labels"]), C.byref(dec), mode, int(bool(use_ghosts)),
                                   max_nodes, C.byref(out), C.byref(stats))
    return (rc,) + _drnn_result(arrs, stats)


class Dfg:
    """Owns one acrobat_dfg of a Context.  Methods mirror the C entry points and return the C return code."""

    def __init__(self, ctx: "Context | None"):
        """ctx None: a graph that can be built and scheduled but not run (needs no GPU)."""
        self.ctx = ctx
        self._g = C.c_void_p()
        rc = lib.acrobat_dfg_create(ctx._h if ctx else None, C.byref(self._g))
        if rc != OK:
            raise AcrobatError(rc, acrobat_strerror(rc))
        self._keep = []

    def acrobat_dfg_last_error(self) -> str:
        return lib.acrobat_dfg_last_error(self._g).decode()

    def acrobat_dfg_register_op_desc(self, desc: "acrobat_op_desc"):
        """-> (rc, op_id) for a prepared descriptor (raw pointers)."""
        op = C.c_int32(-1)
        rc = lib.acrobat_dfg_register_op(self._g, C.byref(desc), C.byref(op))
        return rc, op.value

    def close(self):
        if self._g:
            lib.acrobat_dfg_destroy(self._g)
            self._g = C.c_void_p()

    def acrobat_dfg_register_op(self, epilogue, H, nseg=0, kseg=0, src0=None, ld0=0, src1=None, ld1=0, W=None, ldw=0,
                                bias=None, h=None, c=None, cprev_src=None, zadd=None, zout=None, n_cols=0, y=None, ldo=0,
                                src0_rows=0, src1_rows=0, out_rows=0, W2=None):
        """-> (rc, op_id); tensors are device tensors (kept alive by this object)."""
        t = (src0, src1, W, bias, h, c, cprev_src, zadd, zout, y, W2)
        self._keep.append(t)
        d = acrobat_op_desc(epilogue, H, nseg, kseg, _dp(src0), ld0, _dp(src1), ld1, _dp(W), ldw, _dp(bias), _dp(h),
                            _dp(c), _dp(cprev_src), _dp(zadd), _dp(zout), n_cols, _dp(y), ldo, src0_rows, src1_rows,
                            out_rows, _dp(W2))
        op = C.c_int32(-1)
        rc = lib.acrobat_dfg_register_op(self._g, C.byref(d), C.byref(op))
        return rc, op.value

    def acrobat_dfg_clear(self) -> int:
        return lib.acrobat_dfg_clear(self._g)

    def acrobat_dfg_invoke(self, op, phase, depth, out_row, arg0=0, arg1=0, prod0=-1, prod1=-1):
        """-> (rc, node id)"""
        node = C.c_int32(-1)
        rc = lib.acrobat_dfg_invoke(self._g, op, phase, depth, out_row, arg0, arg1, prod0, prod1, C.byref(node))
        return rc, node.value

    def acrobat_dfg_ghost(self, phase, depth, prod=-1):
        """-> (rc, node id)"""
        node = C.c_int32(-1)
        rc = lib.acrobat_dfg_ghost(self._g, phase, depth, prod, C.byref(node))
        return rc, node.value

    def acrobat_dfg_build_treelstm(self, trees: dict, vocab, op_leaf, op_internal) -> int:
        st, keep = _trees_struct(trees)
        return lib.acrobat_dfg_build_treelstm(self._g, C.byref(st), vocab, op_leaf, op_internal)

    def acrobat_dfg_run(self, stream=0) -> int:
        return lib.acrobat_dfg_run(self._g, stream)

    def acrobat_dfg_schedule(self):
        """-> (bucket_off, order, bucket_op)"""
        nb, po, pn, pp = C.c_int32(0), C.c_void_p(), C.c_void_p(), C.c_void_p()
        rc = lib.acrobat_dfg_schedule(self._g, C.byref(nb), C.byref(po), C.byref(pn), C.byref(pp))
        if rc != OK:
            raise AcrobatError(rc, self.acrobat_dfg_last_error())
        B = nb.value
        as_arr = lambda p, n: (np.ctypeslib.as_array(C.cast(p, C.POINTER(C.c_int32)), shape=(n,)).copy()
                               if n else np.zeros(0, np.int32))
        off = as_arr(po, B + 1) if B else np.zeros(1, np.int32)
        return off, as_arr(pn, int(off[-1])), as_arr(pp, B)


class Context:
    """Owns one acrobat_ctx.  Methods mirror the C entry points and return the C return code."""

    def __init__(self, device: int = 0):
        self._h = C.c_void_p()
        rc = lib.acrobat_create(C.byref(self._h), device)
        if rc != OK:
            raise AcrobatError(rc, acrobat_strerror(rc) + " (acrobat_create: is a GPU present?)")

    def close(self):
        if self._h:
            lib.acrobat_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def acrobat_last_error(self) -> str:
        return lib.acrobat_last_error(self._h).decode()

    def check(self, rc):
        if rc != OK:
            raise AcrobatError(rc, self.acrobat_last_error() or acrobat_strerror(rc))

    def acrobat_treelstm_forward(self, trees: dict, H, D, V, emb, W_leaf, b_leaf, U, b, h, c, stream=0) -> int:
        st, keep = _trees_struct(trees)
        return lib.acrobat_treelstm_forward(self._h, C.byref(st), H, D, V, _dp(emb), _dp(W_leaf), _dp(b_leaf),
                                            _dp(U), _dp(b), _dp(h), _dp(c), stream)

    def acrobat_treelstm_forward_noalloc(self, trees: dict, H, D, V, emb, W_leaf, b_leaf, U, b, h, c, stream=0) -> int:
        st, keep = _trees_struct(trees)
        return lib.acrobat_treelstm_forward_noalloc(self._h, C.byref(st), H, D, V, _dp(emb), _dp(W_leaf), _dp(b_leaf),
                                                    _dp(U), _dp(b), _dp(h), _dp(c), stream)

    def acrobat_mvrnn_forward(self, trees: dict, d, V, vec_tab, mat_tab, W, WM, vec, mat, copy_leaves=0,
                              stream=0) -> int:
        st, keep = _trees_struct(trees)
        return lib.acrobat_mvrnn_forward(self._h, C.byref(st), d, V, _dp(vec_tab), _dp(mat_tab), _dp(W), _dp(WM),
                                         _dp(vec), _dp(mat), int(copy_leaves), stream)

    def acrobat_varlen_lstm_forward(self, lens, H, D, x, Wx, Wh, b, h, c, stream=0) -> int:
        lens = _i32(lens)
        return lib.acrobat_varlen_lstm_forward(self._h, int(lens.size), _hp(lens), H, D, _dp(x), _dp(Wx), _dp(Wh),
                                               _dp(b), _dp(h), _dp(c), stream)

    def acrobat_birnn_forward(self, lens, H, D, n_out, x, fwd, bwd, Cw, cb, hf, hb, y, stream=0) -> int:
        """fwd / bwd: (Wx, Wh, b, h_init) device tensors of one direction."""
        lens = _i32(lens)
        f = acrobat_rnn_dir(*(_dp(t) for t in fwd))
        b = acrobat_rnn_dir(*(_dp(t) for t in bwd))
        return lib.acrobat_birnn_forward(self._h, int(lens.size), _hp(lens), H, D, n_out, _dp(x), C.byref(f),
                                         C.byref(b), _dp(Cw), _dp(cb), _dp(hf), _dp(hb), _dp(y), stream)

    def acrobat_drnn_forward(self, w: dict, x0, params: dict, a, f, g, y, mode=TDC_FORK_JOIN, use_ghosts=True,
                             max_nodes=None, stream=0):
        """params: device tensors emb, Wa, ba, Wf, bf, Wp, bp, Wo, bo (biases may be None); a, f, g
        [max_nodes, H] and y [max_nodes, n_out] are written.  -> (rc, trees dict, stats dict)"""
        max_nodes = int(w["cap"] if max_nodes is None else max_nodes)
        arrs, out = _drnn_outputs(max_nodes)
        dec, stats = _drnn_decisions(w), acrobat_drnn_stats()
        p = acrobat_drnn_params(int(w["H"]), int(w["n_labels"]), int(w["n_out"]),
                                *(_dp(params.get(k)) for k in ("emb", "Wa", "ba", "Wf", "bf", "Wp", "bp", "Wo", "bo")))
        rc = lib.acrobat_drnn_forward(self._h, int(w["n_inst"]), _dp(x0), C.byref(p), C.byref(dec), mode,
                                      int(bool(use_ghosts)), max_nodes, C.byref(out), _dp(a), _dp(f), _dp(g), _dp(y),
                                      C.byref(stats), stream)
        return (rc,) + _drnn_result(arrs, stats)

    def acrobat_last_schedule(self):
        n_levels, po, pn = C.c_int32(0), C.c_void_p(), C.c_void_p()
        self.check(lib.acrobat_last_schedule(self._h, C.byref(n_levels), C.byref(po), C.byref(pn)))
        L = n_levels.value
        level_off = np.ctypeslib.as_array(C.cast(po, C.POINTER(C.c_int32)), shape=(L + 1,)).copy()
        n = int(level_off[-1])
        level_nodes = (np.ctypeslib.as_array(C.cast(pn, C.POINTER(C.c_int32)), shape=(n,)).copy()
                       if n else np.zeros(0, np.int32))
        return level_off, level_nodes

    def acrobat_set_profiling(self, enabled: bool) -> int:
        return lib.acrobat_set_profiling(self._h, int(bool(enabled)))

    def acrobat_set_gather_fusion(self, enabled: bool) -> int:
        return lib.acrobat_set_gather_fusion(self._h, int(bool(enabled)))

    def acrobat_set_tuning(self, force_tile=0, force_ksplit=0, mvrnn_variant=0) -> int:
        return lib.acrobat_set_tuning(self._h, force_tile, force_ksplit, mvrnn_variant)

    def acrobat_set_persistent(self, enabled=True, max_polls=-1) -> int:
        return lib.acrobat_set_persistent(self._h, int(bool(enabled)), max_polls)

    def acrobat_device_status(self) -> int:
        return lib.acrobat_device_status(self._h)

    def acrobat_sync_probe(self, groups, group_size, rounds, same_xcd, style, write_through, store_floats, load_floats,
                           stream=0):
        """-> (rc, microseconds per round, [5 phase times in microseconds, number of stale payload elements read])"""
        us, phases = C.c_double(0.0), (C.c_double * 6)()
        rc = lib.acrobat_sync_probe(self._h, groups, group_size, rounds, int(bool(same_xcd)), style, int(bool(write_through)),
                                    store_floats, load_floats, C.byref(us), phases, stream)
        return rc, us.value, list(phases)

    def acrobat_last_profile(self):
        n, p = C.c_int32(0), C.POINTER(acrobat_launch_record)()
        self.check(lib.acrobat_last_profile(self._h, C.byref(n), C.byref(p)))
        return [(p[i].kind, p[i].level, p[i].n, p[i].ms, p[i].tile, p[i].ksplit) for i in range(n.value)]
