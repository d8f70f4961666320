"""Helpers of the GPU parity tests: run a workload through the C-ABI binding, compare with
the oracle under the stated tolerances."""
import numpy as np
import torch

ABS_TOL = 1e-4  # max abs error on every element of every node's state
REL_TOL = 1e-3  # per node: max-norm of the error over max-norm of the oracle's row


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def stream_handle():
    return torch.cuda.current_stream().cuda_stream


def nan_filled(*shape):
    return torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")


def run_treelstm(ctx, w, use_bias=True, stream=None):
    N, H = int(w["tree_off"][-1]), int(w["H"])
    t = {k: dev(w[k]) for k in ("emb", "W_leaf", "b_leaf", "U", "b")}
    h, c = nan_filled(max(N, 1), H), nan_filled(max(N, 1), H)
    rc = ctx.acrobat_treelstm_forward(w, H, int(w["D"]), int(w["V"]), t["emb"], t["W_leaf"],
                                      t["b_leaf"] if use_bias else None, t["U"], t["b"] if use_bias else None,
                                      h, c, stream_handle() if stream is None else stream)
    ctx.check(rc)
    torch.cuda.synchronize()
    return h[:N].cpu().numpy(), c[:N].cpu().numpy()


def run_mvrnn(ctx, w, copy_leaves=1):
    N, d = int(w["tree_off"][-1]), int(w["d"])
    t = {k: dev(w[k]) for k in ("vec_tab", "mat_tab", "W", "WM")}
    vec, mat = nan_filled(max(N, 1), d), nan_filled(max(N, 1), d, d)
    rc = ctx.acrobat_mvrnn_forward(w, d, int(w["V"]), t["vec_tab"], t["mat_tab"], t["W"], t["WM"], vec, mat,
                                   copy_leaves, stream_handle())
    ctx.check(rc)
    torch.cuda.synchronize()
    return vec[:N].cpu().numpy(), mat[:N].cpu().numpy()


def run_lstm(ctx, w, use_bias=True):
    R, H = int(np.sum(w["len"])), int(w["H"])
    t = {k: dev(w[k]) for k in ("x", "Wx", "Wh", "b")}
    h, c = nan_filled(max(R, 1), H), nan_filled(max(R, 1), H)
    rc = ctx.acrobat_varlen_lstm_forward(w["len"], H, int(w["D"]), t["x"], t["Wx"], t["Wh"],
                                         t["b"] if use_bias else None, h, c, stream_handle())
    ctx.check(rc)
    torch.cuda.synchronize()
    return h[:R].cpu().numpy(), c[:R].cpu().numpy()


def run_birnn(ctx, w, use_bias=True):
    R, H, n_out = int(np.sum(w["len"])), int(w["H"]), int(w["n_out"])
    names = ("x", "fWx", "fWh", "fb", "finit", "bWx", "bWh", "bb", "binit", "C", "cb")
    t = {k: dev(np.asarray(w[k], np.float32)) for k in names}
    hf, hb, y = nan_filled(max(R, 1), H), nan_filled(max(R, 1), H), nan_filled(max(R, 1), n_out)
    fwd = (t["fWx"], t["fWh"], t["fb"] if use_bias else None, t["finit"])
    bwd = (t["bWx"], t["bWh"], t["bb"] if use_bias else None, t["binit"])
    rc = ctx.acrobat_birnn_forward(w["len"], H, int(w["D"]), n_out, t["x"], fwd, bwd, t["C"],
                                   t["cb"] if use_bias else None, hf, hb, y, stream_handle())
    ctx.check(rc)
    torch.cuda.synchronize()
    return hf[:R].cpu().numpy(), hb[:R].cpu().numpy(), y[:R].cpu().numpy()


def run_drnn(ctx, w, mode=2, use_ghosts=True, use_bias=True, max_nodes=None, check=True):
    """-> (rc, trees, stats, (a, f, g, y) as numpy arrays of the generated nodes)"""
    H, n_out = int(w["H"]), int(w["n_out"])
    cap = int(w["cap"] if max_nodes is None else max_nodes)
    t = {k: dev(np.asarray(w[k], np.float32)) for k in ("x0", "emb", "Wa", "ba", "Wf", "bf", "Wp", "bp", "Wo", "bo")}
    params = {k: (t[k] if use_bias or not k.startswith("b") else None) for k in t if k != "x0"}
    a, f, g = (nan_filled(max(cap, 1), H) for _ in range(3))
    y = nan_filled(max(cap, 1), n_out)
    rc, trees, stats = ctx.acrobat_drnn_forward(w, t["x0"], params, a, f, g, y, mode, use_ghosts, cap, stream_handle())
    if check:
        ctx.check(rc)
    torch.cuda.synchronize()
    n = stats["n_nodes"]
    return rc, trees, stats, tuple(v[:n].cpu().numpy() for v in (a, f, g, y))


from workloads.generators import match_trees, tree_paths  # noqa: E402,F401  (structure helpers, shared with bench.py)


def errors(got, want, ref_floor=1e-30):
    """(max abs error, max over rows of max-norm relative error).  ref_floor bounds a row's
    reference norm from below: rows a ReLU clamps to exactly zero have no relative error."""
    got = np.asarray(got, np.float64).reshape(want.shape[0], -1)
    want = np.asarray(want, np.float64).reshape(want.shape[0], -1)
    if want.size == 0:
        return 0.0, 0.0
    diff = np.abs(got - want)
    row_err = diff.max(axis=1)
    row_ref = np.maximum(np.abs(want).max(axis=1), ref_floor)
    return float(diff.max()), float((row_err / row_ref).max())


def assert_close(got, want, what="", ref_floor=1e-30):
    assert got.shape[0] == want.shape[0]
    assert not np.isnan(got).any(), f"{what}: NaN in the GPU result (a row was read before it was written, or never written)"
    abs_err, rel_err = errors(got, want, ref_floor)
    assert abs_err <= ABS_TOL, f"{what}: max abs error {abs_err:.3e} > {ABS_TOL}"
    assert rel_err <= REL_TOL, f"{what}: max per-node relative error {rel_err:.3e} > {REL_TOL}"
    return abs_err, rel_err
