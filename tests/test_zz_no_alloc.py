"""The entry point that allocates nothing: gr_materialize_into_static against gr_materialize_into
(same kernels, so the same bits), twice in a row with the second input smaller, through the C ABI."""
import ctypes

import numpy as np
import pytest

from cases import _rand
from paper_1901_03771_amd import workloads as wl

pytestmark = pytest.mark.gpu
f32 = np.float32


def _programs():
    # (name, program, input maker by size step): each needs device memory beyond inputs and output
    def logreg_inputs(step):
        return wl.make_inputs("logreg", rows=(3001, 700)[step], cols=(200, 136)[step])       # stored residual r + partial vectors

    def vec_inputs(step):
        return dict(a=np.abs(_rand(((1 << 22) + 77, 300_001)[step], 401)) + f32(0.25))

    def mat_inputs(step):
        return dict(a=_rand(((1003, 300), (257, 300))[step], 402))

    return [
        ("logistic regression step (one-pass contraction pair)", wl.logreg, logreg_inputs),
        ("two-stage sum", lambda xp, a: xp.sum(xp.sqrt(a)), vec_inputs),
        ("chunked prefix sum", lambda xp, a: xp.cumsum(a, 0), vec_inputs),
        ("column prefix sums feeding a map", lambda xp, a: xp.cumsum(a, 0) * 2.0 - a, mat_inputs),
        ("column sums", lambda xp, a: xp.sum(a, axis=0), mat_inputs),
        ("softmax of a product", lambda xp, a: wl.softmax(xp, a @ xp.transpose(a[:64], (1, 0))), mat_inputs),
    ]


def test_static_entry_matches_materialize_into_twice_in_a_row():
    import torch
    from paper_1901_03771_amd import lazy as gr
    ctx = gr.Context()
    ctx.set_option("interp", 0)
    L = gr.lib()
    cap = ctypes.c_size_t()
    assert L.gr_static_scratch_bytes(ctypes.byref(cap)) == 0 and cap.value == 16 << 20
    for name, prog, make in _programs():
        for step in (0, 1):                                  # second call: smaller input, same static array
            arrays = make(step)
            keep = {k: torch.from_numpy(v).cuda() for k, v in arrays.items()}
            want_a = prog(gr, **{k: ctx.array(t) for k, t in keep.items()})
            want = torch.empty(want_a.shape, dtype=torch.float32, device="cuda")
            want_a.materialize_into(want)                    # the existing entry point (also loads the kernels)
            lazy = prog(gr, **{k: ctx.array(t) for k, t in keep.items()})
            got = torch.full(lazy.shape, float("nan"), dtype=torch.float32, device="cuda")
            before = ctx.stats()
            mem = torch.cuda.memory_allocated()
            st = L.gr_materialize_into_static(ctx._p, lazy.h, got.data_ptr(), got.numel() * 4)
            assert st == 0, (name, step, ctx.last_error())
            after = ctx.stats()
            assert after["bytes_allocated"] == before["bytes_allocated"] and after["pool_bytes"] == before["pool_bytes"], name
            assert torch.cuda.memory_allocated() == mem
            assert after["kernel_launches"] > before["kernel_launches"]
            assert torch.equal(got, want), f"{name}, call {step}: {int((got != want).sum())} elements differ"
            assert lazy.is_materialized
    ctx.close()


def test_static_entry_refuses_what_it_cannot_serve():
    import torch
    from paper_1901_03771_amd import lazy as gr
    ctx = gr.Context()
    ctx.set_option("interp", 0)
    L = gr.lib()
    # a kernel that is not loaded yet: refused, nothing launched; after gr_plan_compile it runs
    t = torch.from_numpy(_rand((70000,), 403)).cuda()
    a = ctx.array(t)
    lazy = gr.cumsum(gr.tanh(a) * 3.0 + gr.erf(a), 0)
    out = torch.empty(70000, device="cuda")
    n0 = ctx.stats()["kernel_launches"]
    assert gr.STATUS[L.gr_materialize_into_static(ctx._p, lazy.h, out.data_ptr(), out.numel() * 4)] == "GR_ERR_UNSUPPORTED"
    assert "not loaded" in ctx.last_error() and ctx.stats()["kernel_launches"] == n0 and not lazy.is_materialized
    lazy.compile()
    assert L.gr_materialize_into_static(ctx._p, lazy.h, out.data_ptr(), out.numel() * 4) == 0
    want = gr.cumsum(gr.tanh(a) * 3.0 + gr.erf(a), 0).torch()
    assert torch.equal(out, want)
    # a matrix product whose K the planner divides over three workgroups per tile (28 MiB of partial tiles): planned for
    # this entry point it keeps one workgroup per tile and needs nothing beyond inputs and output; gr_plan_compile
    # prepares that kernel too (small integers: the order of the additions does not show)
    g = np.random.default_rng(404)
    A = torch.from_numpy(g.integers(-3, 4, (1536, 1536)).astype(f32)).cuda()
    B = torch.from_numpy(g.integers(-3, 4, (1536, 1536)).astype(f32)).cuda()
    lazy = ctx.array(A) @ ctx.array(B)
    assert "direct split=3" in lazy.plan()
    want = torch.empty(1536, 1536, device="cuda")
    lazy.materialize_into(want)
    lazy = ctx.array(A) @ ctx.array(B)
    got = torch.full((1536, 1536), float("nan"), device="cuda")
    assert gr.STATUS[L.gr_materialize_into_static(ctx._p, lazy.h, got.data_ptr(), got.numel() * 4)] == "GR_ERR_UNSUPPORTED"
    lazy.compile()
    before = ctx.stats()
    assert L.gr_materialize_into_static(ctx._p, lazy.h, got.data_ptr(), got.numel() * 4) == 0, ctx.last_error()
    assert ctx.stats()["bytes_allocated"] == before["bytes_allocated"] and ctx.stats()["kernel_launches"] == before["kernel_launches"] + 1
    assert torch.equal(got, want)
    # an intermediate result beyond the 16 MiB of the static array: refused with both sizes named
    big = ctx.array(torch.ones((5 << 20,), device="cuda"))
    lazy = gr.sum(gr.cumsum(big, 0))                         # the prefix sums (20 MiB) are stored for the sum
    lazy.compile()
    one = torch.empty((), device="cuda")
    n0 = ctx.stats()["kernel_launches"]
    assert gr.STATUS[L.gr_materialize_into_static(ctx._p, lazy.h, one.data_ptr(), 4)] == "GR_ERR_OOM"
    assert str(16 << 20) in ctx.last_error() and ctx.stats()["kernel_launches"] == n0
    lazy.materialize_into(one)                               # the allocating entry point still serves it
    n = 5 << 20
    assert float(one) == float(np.float32(n * (n + 1) / 2))
    # an intermediate that the request stored in the static array is unevaluated again afterwards
    arrays = wl.make_inputs("logreg", rows=300, cols=40)
    keep = {k: torch.from_numpy(v).cuda() for k, v in arrays.items()}
    X, w, y = (ctx.array(keep[k]) for k in ("X", "w", "y"))
    r = 1.0 / (1.0 + gr.exp(-(X @ w))) - y
    res = w - 0.1 * ((X.T @ r) / 300 + 1e-4 * w)
    res.compile()
    outw = torch.empty(40, device="cuda")
    assert L.gr_materialize_into_static(ctx._p, res.h, outw.data_ptr(), 160) == 0
    assert res.is_materialized and not r.is_materialized
    r_later = r.torch()                                      # evaluated on request, into storage of its own
    ref_r = 1.0 / (1.0 + torch.exp(-(keep["X"] @ keep["w"]))) - keep["y"]
    assert torch.allclose(r_later, ref_r, rtol=1e-4, atol=1e-5)
    ctx.close()
