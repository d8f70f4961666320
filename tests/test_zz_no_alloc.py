"""The entry point that allocates nothing (acrobat_treelstm_forward_noalloc, for callers that cannot call
hipMalloc) against the ordinary entry point, through the C ABI: two calls in a row on one stream, the second
with a smaller mini-batch, so the library's static device array still holds the first call's index lists and
partial tiles when the second call starts."""
import numpy as np
import pytest

import oracle
from workloads import generators as gen

pytestmark = pytest.mark.gpu

NT = oracle.default_threads()


def enqueue(fn, ctx, P, w, t):
    N, H = int(w["tree_off"][-1]), int(w["H"])
    h, c = P.nan_filled(N, H), P.nan_filled(N, H)
    ctx.check(fn(w, H, int(w["D"]), int(w["V"]), t["emb"], t["W_leaf"], t["b_leaf"], t["U"], t["b"], h, c, P.stream_handle()))
    return h, c


def test_noalloc_entry_point_matches_the_ordinary_one_on_two_calls_in_a_row():
    import torch
    import paper_2305_10611_amd as A
    from tests import parity as P
    ctx = A.Context(0)
    try:
        # first: several node tiles per level, and levels that the launcher cuts into equal shares per compute
        # unit (their partial tiles are parked in the static array); second: a much smaller batch right behind it
        big = gen.treelstm_workload(150, 4, 48, 512, 500, "zipf1.1", seed=311, bias_scale=0.2)
        small = gen.treelstm_workload(9, 1, 14, 512, 500, "zipf1.1", seed=312, bias_scale=0.2)
        tb = {k: P.dev(big[k]) for k in ("emb", "W_leaf", "b_leaf", "U", "b")}
        ts = {k: P.dev(small[k]) for k in ("emb", "W_leaf", "b_leaf", "U", "b")}
        # the ordinary entry point: expected values, and its launch records say which variants the batch takes
        ctx.acrobat_set_profiling(True)
        want_big = enqueue(ctx.acrobat_treelstm_forward, ctx, P, big, tb)
        assert any(r[5] != 1 for r in ctx.acrobat_last_profile()), "no level of this batch parks partial tiles in the workspace"
        ctx.acrobat_set_profiling(False)
        want_small = enqueue(ctx.acrobat_treelstm_forward, ctx, P, small, ts)
        torch.cuda.synchronize()
        # the entry point that allocates nothing: both calls enqueued back to back on one stream
        got_big = enqueue(ctx.acrobat_treelstm_forward_noalloc, ctx, P, big, tb)
        got_small = enqueue(ctx.acrobat_treelstm_forward_noalloc, ctx, P, small, ts)
        level_off, level_nodes = ctx.acrobat_last_schedule()
        o_off, o_nodes, _, _ = oracle.tree_schedule(small)
        assert np.array_equal(level_off, o_off) and np.array_equal(level_nodes, o_nodes)
        torch.cuda.synchronize()
        for w, want, got in ((big, want_big, got_big), (small, want_small, got_small)):
            ref = oracle.treelstm(w, nthreads=NT)
            for name, g, e, o in zip("hc", got, want, ref):
                g, e = g.cpu().numpy(), e.cpu().numpy()
                P.assert_close(g, e.astype(np.float64), f"noalloc {name} vs the ordinary entry point")
                assert np.array_equal(g, e)  # same kernels, same variants: same bits
                P.assert_close(g, o, f"noalloc {name} vs oracle")
    finally:
        ctx.close()


def test_noalloc_entry_point_rejects_sizes_beyond_its_limit():
    import paper_2305_10611_amd as A
    from tests import parity as P
    ctx = A.Context(0)
    try:
        n = 65536 + 1  # ACROBAT_NOALLOC_MAX_NODES + 1 single-leaf trees
        w = dict(n_trees=n, tree_off=np.arange(n + 1, dtype=np.int32), left=np.full(n, -1, np.int32),
                 right=np.full(n, -1, np.int32), token=np.zeros(n, np.int32))
        H = 32
        z = lambda *s: P.dev(np.zeros(s, np.float32))
        h, c = P.nan_filled(n, H), P.nan_filled(n, H)
        rc = ctx.acrobat_treelstm_forward_noalloc(w, H, H, 4, z(4, H), z(5 * H, H), None, z(5 * H, 2 * H), None, h, c,
                                                  P.stream_handle())
        assert rc == A.EINVAL and "ACROBAT_NOALLOC_MAX_NODES" in ctx.acrobat_last_error()
        import torch
        torch.cuda.synchronize()
        assert torch.isnan(h).all() and torch.isnan(c).all()  # nothing was launched
        # exactly at the limit it runs
        w = dict(w, n_trees=n - 1, tree_off=w["tree_off"][:n], left=w["left"][: n - 1], right=w["right"][: n - 1],
                 token=w["token"][: n - 1])
        rc = ctx.acrobat_treelstm_forward_noalloc(w, H, H, 4, z(4, H), z(5 * H, H), None, z(5 * H, 2 * H), None, h, c,
                                                  P.stream_handle())
        assert rc == A.OK, ctx.acrobat_last_error()
        torch.cuda.synchronize()
        assert (h[: n - 1] == 0).all() and (c[: n - 1] == 0).all()  # zero weights: sigmoid(0) tanh(0) = 0
    finally:
        ctx.close()
