"""Host logic of the library on a device-less context (no GPU needed): the C
ABI loads and exports every declared symbol, shapes and element types are
inferred with NumPy semantics, errors are reported at record time, the
partitioner produces the sub-graph lists the paper describes, and every
program used by the GPU parity tests generates HIP source that hipRTC
compiles for gfx950."""
import ctypes
import os
import re

import numpy as np
import pytest

from cases import DOT_CASES, ELEMENTWISE_CASES, NARROW_CASES, REDUCTION_CASES, ROWRED_PROGRAMS, SCAN_CASES
from paper_1901_03771_amd import lazy as gr, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture()
def ctx():
    c = gr.Context(device=-1)
    yield c
    c.close()


def groups(arr):
    """[(kind, [op names]), ...] of the planned sub-graph list."""
    out = []
    for line in arr.plan().strip().splitlines():
        kind = line.split()[1]
        members = re.search(r"members=\[(.*?)\]", line).group(1)
        out.append((kind, [m.split(":")[1] for m in members.split(",") if m]))
    return out


# ------------------------------------------------------------------ the boundary --
def test_library_exports_every_declared_symbol():
    header = "".join(open(os.path.join(ROOT, "include", h)).read() for h in sorted(os.listdir(os.path.join(ROOT, "include"))) if h.endswith(".h"))
    declared = set(re.findall(r"^(?:gr_status|const char\*)\s+(gr_[a-z_0-9]+)\s*\(", header, flags=re.M))
    assert len(declared) > 25
    L = ctypes.CDLL(gr.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(L, name), f"{name} declared in the header but not exported"
    assert declared == set(gr.SYMBOLS), declared ^ set(gr.SYMBOLS)


def test_deviceless_context_refuses_to_execute(ctx):
    a = ctx.spec((4,))
    with pytest.raises(gr.GrError) as ei:
        (a + 1.0).materialize()
    assert ei.value.code == "GR_ERR_NODEVICE"
    with pytest.raises(gr.GrError):
        gr.Context(device=9999)


# ------------------------------------------------------- shape / dtype inference --
@pytest.mark.parametrize("sa,sb,expect", [
    ((10, 20), (20,), (10, 20)), ((8192, 8192), (1, 8192), (8192, 8192)), ((8192, 8192), (8192,), (8192, 8192)),
    ((16384, 4096), (16384, 1), (16384, 4096)), ((3, 1), (1, 4), (3, 4)), ((), (5,), (5,)), ((0, 3), (1, 3), (0, 3)),
    ((2, 1, 4), (3, 1), (2, 3, 4)), ((2, 3), (2,), None), ((4,), (5,), None)])
def test_broadcast_inference(ctx, sa, sb, expect):
    a, b = ctx.spec(sa), ctx.spec(sb)
    if expect is None:
        with pytest.raises(gr.GrError) as ei:
            a + b
        assert ei.value.code == "GR_ERR_SHAPE"
    else:
        assert (a + b).shape == expect == np.broadcast_shapes(sa, sb)


def test_slice_shapes_match_python(ctx):
    a = ctx.spec((6, 7))
    vals = [None, -8, -7, -6, -3, -1, 0, 1, 3, 6, 7, 9]
    for st in vals:
        for sp in vals:
            for step in (None, 1, 2, 3):
                assert a[st:sp:step, ::2].shape == (len(range(6)[st:sp:step]), 4)
    assert a[1:3].shape == (2, 7)
    with pytest.raises(gr.GrError) as ei:
        a[::-1]
    assert ei.value.code == "GR_ERR_UNSUPPORTED"
    with pytest.raises(gr.GrError):
        a[:, :, :]


def test_transpose_reduce_dot_shapes_and_errors(ctx):
    a = ctx.spec((2, 3, 4))
    assert a.T.shape == (4, 3, 2)
    assert gr.transpose(a, (1, 2, 0)).shape == (3, 4, 2)
    with pytest.raises(gr.GrError) as ei:
        gr.transpose(a, (0, 0, 1))
    assert ei.value.code == "GR_ERR_AXIS"
    assert a.sum(axis=1).shape == (2, 4)
    assert a.sum(axis=(0, 2), keepdims=True).shape == (1, 3, 1)
    assert a.max().shape == ()
    assert a.sum(axis=-1).shape == (2, 3)
    for bad in (3, -4, (1, 1)):
        with pytest.raises(gr.GrError) as ei:
            a.sum(axis=bad)
        assert ei.value.code == "GR_ERR_AXIS"
    m, v = ctx.spec((5, 7)), ctx.spec((7,))
    assert (m @ v).shape == (5,) and (v @ v).shape == () and (m.T @ ctx.spec((5,))).shape == (7,)
    with pytest.raises(gr.GrError) as ei:
        m @ ctx.spec((5,))
    assert ei.value.code == "GR_ERR_SHAPE"
    assert (m @ ctx.spec((7, 2))).shape == (5, 2)
    with pytest.raises(gr.GrError) as ei:
        v @ ctx.spec((7, 2))
    assert ei.value.code == "GR_ERR_UNSUPPORTED"
    with pytest.raises(gr.GrError) as ei:
        m @ ctx.spec((6, 2))
    assert ei.value.code == "GR_ERR_SHAPE"


def test_dtype_rules(ctx):
    f, i = ctx.spec((4,), gr.GR_F32), ctx.spec((4,), gr.GR_I32)
    assert (i * 2 + i).dtype_code == gr.GR_I32
    assert (f * 2 + 1).dtype_code == gr.GR_F32
    assert i.sum().dtype_code == gr.GR_I64 and i.max().dtype_code == gr.GR_I32 and f.sum().dtype_code == gr.GR_F32
    for bad, code in [(lambda: i * 0.5, "GR_ERR_DTYPE"), (lambda: i + f, "GR_ERR_DTYPE"), (lambda: gr.exp(i), "GR_ERR_DTYPE"),
                      (lambda: i / i, "GR_ERR_UNSUPPORTED"), (lambda: i.sum() + 1, "GR_ERR_UNSUPPORTED"),
                      (lambda: i * (2 ** 40), "GR_ERR_DTYPE"), (lambda: f ** 3, "GR_ERR_UNSUPPORTED")]:
        with pytest.raises(gr.GrError) as ei:
            bad()
        assert ei.value.code == code


def test_failed_record_leaves_the_dag_unchanged(ctx):
    a, b = ctx.spec((2, 3)), ctx.spec((2,))
    before = ctx.stats()["nodes_alive"]
    with pytest.raises(gr.GrError):
        a + b
    assert ctx.stats()["nodes_alive"] == before
    with pytest.raises(gr.GrError) as ei:
        gr.Array(ctx, 424242).shape
    assert ei.value.code == "GR_ERR_HANDLE"


def test_nodes_are_freed_with_their_last_reference(ctx):
    a = ctx.spec((8,))
    base = ctx.stats()["nodes_alive"]
    z = gr.exp(a * 2.0 + a) - a
    assert ctx.stats()["nodes_alive"] > base
    del z
    assert ctx.stats()["nodes_alive"] == base
    # a diamond: the shared node must be freed exactly once
    t = a + 1.0
    u = t * t + t
    del t
    del u
    assert ctx.stats()["nodes_alive"] == base


# ------------------------------------------------------------------ partitioning --
def test_five_configurations_partition_as_designed(ctx):
    c1 = wl.chain(gr, ctx.spec((1 << 20,)), ctx.spec((1 << 20,)))
    assert groups(c1) == [("MAP", ["add", "sub", "mul", "mul", "add", "abs", "add", "div", "neg", "mul", "exp", "sub"])]
    c2 = wl.normalize(gr, ctx.spec((8192, 8192)), ctx.spec((1, 8192)), ctx.spec((1, 8192)), ctx.spec((8192,)), ctx.spec((8192,)))
    assert groups(c2) == [("MAP", ["sub", "div", "mul", "add", "maximum"])]
    c3 = wl.softmax(gr, ctx.spec((16384, 4096)))
    assert groups(c3) == [("ROWRED", ["max", "sub", "exp", "sum", "div"])]
    c4 = wl.stencil(gr, ctx.spec((8192, 8192)))
    g4 = groups(c4)
    assert len(g4) == 1 and g4[0][0] == "MAP" and "loads=13" in c4.plan()  # the radius-2 diamond of 13 input points
    ctx.set_option("gemv_pair", 0)
    c5 = wl.logreg(gr, ctx.spec((262144, 512)), ctx.spec((512,)), ctx.spec((262144,)))
    g5 = groups(c5)
    assert [k for k, _ in g5] == ["GEMV", "GEMV"]
    assert g5[0][1] == ["dot", "neg", "exp", "add", "div", "sub"]       # X@w with the sigmoid/residual epilogue
    assert g5[1][1] == ["dot", "div", "mul", "add", "mul", "sub"]       # X.T@r with the update epilogue
    plan = c5.plan().splitlines()
    assert "row-dot" in plan[0] and "column-accumulate" in plan[1]
    # by default the two contractions share one pass over X: one kernel group, both sub-graphs listed
    ctx.set_option("gemv_pair", 1)
    plan = c5.plan().splitlines()
    assert len(plan) == 1 and "row-dot+column-accumulate" in plan[0]
    fused = re.search(r"fused-with=\[root=\d+ members=\[(.*?)\]\]", plan[0]).group(1)
    assert [m.split(":")[1] for m in fused.split(",")] == ["dot", "div", "mul", "add", "mul", "sub"]
    # rows too long to stay in registers: two passes
    far = wl.logreg(gr, ctx.spec((4096, 3000)), ctx.spec((3000,)), ctx.spec((4096,)))
    assert len(far.plan().splitlines()) == 2


def test_blackscholes_is_one_fused_kernel(ctx):
    # Section 4.2: "a lot of point-wise operations which could be completely fused"
    n = 1 << 20
    out = wl.blackscholes(gr, ctx.spec((n,)), ctx.spec((n,)), ctx.spec((n,)))
    g = groups(out)
    assert len(g) == 1 and g[0][0] == "MAP" and len(g[0][1]) >= 20 and g[0][1].count("erf") == 2
    assert "loads=3" in out.plan()
    out.compile()


def test_jacobi_slices_fuse_into_one_kernel(ctx):
    # Section 4.2: the stencil is fused into a single kernel even when slicing
    out = wl.jacobi_sweep(gr, ctx.spec((512, 512)))
    g = groups(out)
    assert len(g) == 1 and g[0] == ("MAP", ["add", "add", "add", "add", "mul"])
    assert "leaves=[1]" in out.plan() and "loads=5" in out.plan()


def test_mnist_walkthrough(ctx):
    # Section 2 on Listing 2: max is computed first, the transposed W is folded into the
    # contraction, and the pointwise tail reads the contraction's result
    W, a, b = ctx.spec((200, 10)), ctx.spec((200,)), ctx.spec((10,))
    out = wl.mnist(gr, W, a, b)
    g = groups(out)
    assert g[0] == ("MAP", ["maximum"])
    assert g[1][0] == "GEMV" and g[1][1] == ["dot", "add", "neg", "exp", "add", "div"]
    assert "column-accumulate" in out.plan().splitlines()[1]
    assert len(g) == 2


def test_unfused_mode_cuts_at_every_op(ctx):
    ctx.set_option("fusion", 0)
    out = wl.softmax(gr, ctx.spec((64, 256)))
    assert [ops for _, ops in groups(out)] == [["max"], ["sub"], ["exp"], ["sum"], ["div"]]
    ctx.set_option("fusion", 1)


def test_multiple_use_across_subgraphs_materialises_once(ctx):
    a = ctx.spec((100, 64))
    t = gr.exp(a)                    # used by a non-resident reduction and by the final map
    s = t.sum(axis=0, keepdims=True)
    out = t / s
    g = groups(out)
    owners = [ops for _, ops in g]
    assert sum(ops.count("exp") for ops in owners) == 1, "exp must belong to exactly one sub-graph"
    assert owners == [["exp"], ["sum"], ["div"]]
    lines = out.plan().splitlines()
    exp_root = re.search(r"root=(\d+)", lines[0]).group(1)
    for line in lines[1:]:
        assert exp_root in re.search(r"leaves=\[(.*?)\]", line).group(1).split(",")


def test_equal_pending_reductions_scans_and_dots_are_merged_at_record_time(ctx):
    # common subexpressions (Section 5): an expensive operation recorded twice on equal pending
    # expressions is one node; cheap pointwise duplicates stay separate nodes (value numbering inside
    # the kernel merges them without forcing a store)
    X = ctx.spec((64, 5000))
    m1, m2 = gr.max(X, axis=1, keepdims=True), gr.max(X, axis=1, keepdims=True)
    assert m1.h == m2.h
    assert gr.max(X, axis=1).h != m1.h and gr.max(X, axis=0, keepdims=True).h != m1.h and gr.min(X, axis=1, keepdims=True).h != m1.h
    d1, d2 = X - m1, X - m2
    assert d1.h != d2.h
    s1, s2 = gr.sum(gr.exp(d1), axis=1, keepdims=True), gr.sum(gr.exp(d2), axis=1, keepdims=True)
    assert s1.h == s2.h                                   # equal below different pointwise nodes
    assert gr.sum(gr.exp(d1 * 2.0), axis=1, keepdims=True).h != s1.h
    assert gr.sum(gr.exp(d1 * 1.0), axis=1, keepdims=True).h != s1.h
    out = gr.exp(d1) / s1 + gr.exp(d2) / s2
    kinds = groups(out)
    assert [k for k, _ in kinds] == ["ROWRED"] and kinds[0][1].count("max") == 1 and kinds[0][1].count("sum") == 1
    v = ctx.spec((1 << 22,))
    two = gr.sum(v * v) + gr.sum(v * v)
    assert [k for k, _ in groups(two)] == ["REDUCE", "MAP"]
    A, w = ctx.spec((300, 200)), ctx.spec((200,))
    assert gr.dot(A, w).h == gr.dot(A, w).h and gr.dot(A, w).h != gr.dot(A, w * 2.0).h
    assert gr.dot(A.T[:, 1:], A[1:, :]).h == gr.dot(A.T[:, 1:], A[1:, :]).h
    assert gr.dot(A.T[:, 1:], A[1:, :]).h != gr.dot(A.T[:, :-1], A[1:, :]).h
    assert gr.cumsum(v * 2.0, 0).h == gr.cumsum(v * 2.0, 0).h and gr.cumsum(v, 0).h != gr.cummax(v, 0).h
    merged = ctx.stats()["nodes_merged"]
    assert merged >= 6
    # every handle given out is its own reference: dropping one of two leaves the node alive
    del m2
    assert m1.shape == (64, 1) and (X - m1).shape == (64, 5000)
    ctx.set_option("merge", 0)
    assert gr.max(X, axis=1, keepdims=True).h != m1.h
    assert ctx.stats()["nodes_merged"] == merged


def test_merged_nodes_do_not_leak(ctx):
    X = ctx.spec((100, 100))
    base = ctx.stats()["nodes_alive"]
    a = gr.sum(X * X)
    b = gr.sum(X * X)
    c = gr.sum(X * X) + 1.0
    assert a.h == b.h
    del a
    assert b.shape == ()
    del b, c
    assert ctx.stats()["nodes_alive"] == base


def test_random_programs_partition_into_valid_subgraph_lists(ctx):
    # 400 seeded random programs (tests/fuzz.py): each partitions, every recorded node that the result
    # needs is computed by exactly one sub-graph, and sub-graphs only read leaves or earlier roots
    import fuzz
    kinds = set()
    for seed in range(400):
        dtype, shapes, steps, res = fuzz.make_recipe(seed)
        leaves = [ctx.spec(s_, gr.GR_I32 if dtype == "i32" else gr.GR_F32) for s_ in shapes]
        pool = fuzz.apply(gr, [st for st in steps if st[0] != "materialize"], leaves)
        lines = pool[res].plan().strip().splitlines()
        assert lines, seed
        seen_members, roots = set(), set()
        leaf_ids = {x.h for x in leaves}
        for line in lines:
            kinds.add(line.split()[1])
            members = [int(m.split(":")[0]) for m in re.search(r"members=\[(.*?)\]", line).group(1).split(",") if m]
            reads = [int(m) for m in re.search(r"leaves=\[(.*?)\]", line).group(1).split(",") if m]
            root = int(re.search(r"root=(\d+)", line).group(1))
            assert not (set(members) & seen_members), (seed, "a node is computed twice")
            assert all(x in leaf_ids or x in roots for x in reads), (seed, "reads something that is neither a leaf nor an earlier root")
            seen_members |= set(members)
            roots.add(root)
        assert pool[res].h in roots or pool[res].h in leaf_ids or not seen_members
        for a in pool:
            del a
    assert {"MAP", "REDUCE", "ROWRED", "SCAN"} <= kinds


def test_dry_run_exercises_materialise_and_assign_without_a_device(ctx):
    # option dry_run: everything but the launches.  Random programs with slice assignments and
    # intermediate materialisations run through partitioning, buffer and node bookkeeping on the CPU.
    import fuzz
    x = ctx.spec((100, 50))
    with pytest.raises(gr.GrError) as ei:
        (x + 1.0).materialize()
    assert ei.value.code == "GR_ERR_NODEVICE"
    ctx.set_option("dry_run", 2)      # 2: no compilation either
    del x, ei
    import gc
    gc.collect()
    base = ctx.stats()["nodes_alive"]
    launches = 0
    for seed in range(5000, 5250):
        dtype, shapes, steps, res = fuzz.make_recipe(seed, assign=True)
        leaves = [ctx.spec(s_, gr.GR_I32 if dtype == "i32" else gr.GR_F32) for s_ in shapes]
        pool = fuzz.apply(gr, steps, leaves)
        for a in pool:
            a.materialize()
            assert a.is_materialized and a.shape is not None
        del pool, leaves, a
        assert ctx.stats()["nodes_alive"] == base, seed      # nothing leaks
    # assignments into evaluated results as well (values living in another array's storage among them)
    for seed in range(800000, 800150):
        dtype, shapes, steps, res = fuzz.make_recipe(seed, max_steps=14, assign=True, assign_values=True, reshape=(seed % 3 == 0))
        leaves = [ctx.spec(s_, gr.GR_I32 if dtype == "i32" else gr.GR_F32) for s_ in shapes]
        pool = fuzz.apply(gr, steps, leaves)
        for a in pool:
            a.materialize()
        del pool, leaves, a
        assert ctx.stats()["nodes_alive"] == base, seed
    st = ctx.stats()
    assert st["kernel_launches"] > 500 and st["compile_ms"] == 0.0
    # one kernel per op: intermediate results without a handle are freed while the plan finishes
    ctx.set_option("fusion", 0)
    for seed in range(6000, 6100):
        dtype, shapes, steps, res = fuzz.make_recipe(seed, assign=True)
        leaves = [ctx.spec(s_, gr.GR_I32 if dtype == "i32" else gr.GR_F32) for s_ in shapes]
        for a in fuzz.apply(gr, steps, leaves):
            a.materialize()
        del leaves, a
        assert ctx.stats()["nodes_alive"] == base, seed
    ctx.set_option("fusion", 1)
    # an evaluated scan / reduction / contraction assigned somewhere else is a plain copy
    t = ctx.spec((6, 40))
    for v in (gr.cummax(t, 1), gr.max(t, axis=1, keepdims=True) + t * 0.0, gr.dot(t, gr.transpose(t))[:, :]):
        v.materialize()
    c1, m1, d1 = gr.cummax(t, 1).materialize(), gr.max(t, axis=0).materialize(), gr.dot(t, gr.transpose(t)).materialize()
    dst = ctx.spec((6, 40))
    dst[:] = c1
    dst[:, 0:6] = d1
    row = ctx.spec((40,))
    row[:] = m1
    del row
    del t, v, c1, m1, d1, dst
    # with dry_run = 1 the kernels are generated and compiled as well
    ctx.set_option("dry_run", 1)
    y = ctx.spec((64, 4096))
    s = gr.exp(y - gr.max(y, axis=1, keepdims=True))
    (s / gr.sum(s, axis=1, keepdims=True)).materialize()
    st = ctx.stats()
    assert st["cache_misses"] == 1 and (st["compile_ms"] > 0 or st["disk_hits"] == 1)


def test_reshape_records_shapes_and_is_a_fused_copy(ctx):
    x, y = ctx.spec((4, 6, 5)), ctx.spec((5,))
    assert x.reshape(6, 20).shape == (6, 20) and x.reshape(-1).shape == (120,) and x.reshape((2, -1, 5)).shape == (2, 12, 5)
    assert gr.reshape(x, (1, 120, 1)).shape == (1, 120, 1) and x.T.reshape(10, 12).shape == (10, 12)
    for bad in [(7, 17), (-1, -1), (-2, 60)]:
        with pytest.raises(gr.GrError) as ei:
            x.reshape(*bad)
        assert ei.value.code == "GR_ERR_SHAPE"
    r = (x * 2.0 + y).reshape(6, 20)
    kinds = groups(r)
    assert kinds == [("MAP", ["mul", "add", "reshape"])]             # producers fuse into the copy
    z = gr.sum(r, axis=1) + 1.0
    assert [k for k, _ in groups(z)] == ["MAP", "ROWRED"]             # consumers read the stored result
    z.compile()
    x.T.reshape(-1).compile()
    assert ctx.spec((0, 4)).reshape(4, 0).shape == (4, 0)
    # reductions and contractions below a reshape are evaluated first (also the row-resident ones that
    # would otherwise stay fused with their consumers), the pointwise rest fuses into the copy
    m = ctx.spec((64, 100))
    assert groups((m - gr.max(m, axis=1, keepdims=True)).reshape(100, 64)) == [("ROWRED", ["max"]), ("MAP", ["sub", "reshape"])]
    assert [k for k, _ in groups(gr.min(ctx.spec((1,))).reshape(1))] == ["ROWRED", "MAP"]
    assert [k for k, _ in groups((m @ ctx.spec((100,))).reshape(8, 8))] == ["GEMV", "MAP"]
    assert [k for k, _ in groups((m @ ctx.spec((100, 32)) + 1.0).reshape(-1))] == ["GEMM", "MAP"]
    (m - gr.max(m, axis=1, keepdims=True)).reshape(100, 64).compile()


def test_random_programs_with_reshapes_dry_run(ctx):
    import fuzz
    ctx.set_option("dry_run", 2)
    for seed in range(400000, 400150):
        dtype, shapes, steps, res = fuzz.make_recipe(seed, reshape=True, assign=(seed % 2 == 0))
        leaves = [ctx.spec(s_, gr.GR_I32 if dtype == "i32" else gr.GR_F32) for s_ in shapes]
        for a in fuzz.apply(gr, steps, leaves):
            a.materialize()


def test_leaves_and_only_leaves_are_materialised(ctx):
    a = ctx.spec((33, 65))
    out = (a.T @ (a @ ctx.spec((65,)))) * 2.0
    all_members = []
    for line in out.plan().splitlines():
        members = re.search(r"members=\[(.*?)\]", line).group(1)
        ids = [int(m.split(":")[0]) for m in members.split(",") if m]
        leaves = [int(x) for x in re.search(r"leaves=\[(.*?)\]", line).group(1).split(",") if x]
        assert not set(ids) & set(leaves)
        all_members += ids
    assert len(all_members) == len(set(all_members)), "a node is computed by exactly one sub-graph"


def test_row_resident_limit_turns_reduction_into_a_cut(ctx):
    x = ctx.spec((8, 20000))
    out = wl.softmax(gr, x)
    # max is cut; exp(X-m) feeds both the (cut) sum and the final division, so the
    # multiple-use rule materialises it once: the paper's own partition of a softmax
    assert groups(out) == [("REDUCE", ["max"]), ("MAP", ["sub", "exp"]), ("REDUCE", ["sum"]), ("MAP", ["div"])]
    ctx.set_option("rowred_max_cols", 512)
    assert [k for k, _ in groups(wl.softmax(gr, ctx.spec((8, 1000))))] == ["REDUCE", "MAP", "REDUCE", "MAP"]
    assert [k for k, _ in groups(wl.softmax(gr, ctx.spec((8, 512))))] == ["ROWRED"]


# ------------------------------------------------- code generation on the host ----
def _specs(ctx, arrays):
    code = {np.dtype(np.float32): gr.GR_F32, np.dtype(np.int32): gr.GR_I32}
    return {k: ctx.spec(v.shape, code[v.dtype]) for k, v in arrays.items()}


@pytest.mark.parametrize("name", ["chain", "normalize", "softmax", "stencil", "logreg"])
@pytest.mark.parametrize("size", ["small", "full"])
def test_configurations_compile_for_gfx950(ctx, name, size):
    p = wl.SMALL[name] if size == "small" else wl.FULL[name]
    shapes = {k: v.shape for k, v in wl.make_inputs(name, **wl.SMALL[name]).items()} if size == "small" else None
    if size == "full":
        r, c = p.get("rows"), p.get("cols")
        shapes = {"chain": dict(a=(p.get("n"),), b=(p.get("n"),)),
                  "normalize": dict(X=(r, c), mu=(1, c), sigma=(1, c), gamma=(c,), beta=(c,)),
                  "softmax": dict(X=(r, c)), "stencil": dict(I=(r, c)), "logreg": dict(X=(r, c), w=(c,), y=(r,))}[name]
    out = wl.PROGRAMS[name](gr, **{k: ctx.spec(s) for k, s in shapes.items()})
    out.compile()
    src = out.source(0)
    assert "extern \"C\" __global__" in src and "f4u" in src


@pytest.mark.parametrize("name", sorted(ELEMENTWISE_CASES))
def test_elementwise_cases_compile(ctx, name):
    prog, mk = ELEMENTWISE_CASES[name]
    prog(gr, **_specs(ctx, mk())).compile()


@pytest.mark.parametrize("shape,axis,keep", REDUCTION_CASES)
def test_reduction_cases_compile(ctx, shape, axis, keep):
    for op in ("sum", "max", "min"):
        getattr(gr, op)(ctx.spec(shape) * 1.5, axis=axis, keepdims=keep).compile()
    gr.sum(ctx.spec(shape, gr.GR_I32), axis=axis, keepdims=keep).compile()


def test_long_reductions_are_split_into_two_stages(ctx):
    full = gr.sum(gr.sqrt(ctx.spec((1 << 22,))))
    assert [k for k, _ in groups(full)] == ["REDUCE"]
    src = full.source(0)
    assert "gr_reduce_combine" in src and "NSPLIT" in src
    full.compile()
    gr.sum(ctx.spec((50000, 48)), axis=0).compile()
    gr.max(ctx.spec((300, 40, 50), gr.GR_I32), axis=(0, 2)).compile()


@pytest.mark.parametrize("shape,axis", SCAN_CASES)
def test_scan_cases_plan_and_compile(ctx, shape, axis):
    out = gr.cumsum(ctx.spec(shape) * 0.5 + 1.0, axis)
    assert out.shape == tuple(shape)
    assert groups(out) == [("SCAN", ["mul", "add", "cumsum"])]      # map-scan: the operand expression is fused
    out.compile()
    (gr.cummax(ctx.spec(shape), axis) - gr.cummin(ctx.spec(shape), axis)).compile()
    i = gr.cumsum(ctx.spec(shape, gr.GR_I32), axis)
    assert i.dtype_code == gr.GR_I64
    i.compile()


def test_scan_is_a_cut_and_checks_its_axis(ctx):
    a = ctx.spec((8, 9))
    out = gr.exp(gr.cumsum(a, 1)) + a
    assert [k for k, _ in groups(out)] == ["SCAN", "MAP"]
    for bad in (2, -3):
        with pytest.raises(gr.GrError) as ei:
            gr.cumsum(a, bad)
        assert ei.value.code == "GR_ERR_AXIS"
    # a long contiguous line: one pass with chained tiles of 8192 elements (a kernel that clears the
    # published totals, then the scan); with the option off, or for 8-byte running values, three kernels
    long_line = gr.cumsum(ctx.spec((1 << 22,)), 0)
    assert "mode=one-pass-tiles" in long_line.plan() and "chunks=512" in long_line.plan()
    assert "gr_scan_clear" in long_line.source(0) and "gr_scan_sums" not in long_line.source(0)
    as_i64 = gr.cumsum(ctx.spec((1 << 22,), gr.GR_I32), 0)
    assert "mode=lanes-along-axis" in as_i64.plan() and "gr_scan_sums" in as_i64.source(0) and "gr_scan_offsets" in as_i64.source(0)
    ctx.set_option("scan_one_pass", 0)
    long_line = gr.cumsum(ctx.spec((1 << 22,)), 0)
    assert "chunks=512" in long_line.plan() and "gr_scan_sums" in long_line.source(0) and "gr_scan_offsets" in long_line.source(0)
    ctx.set_option("scan_one_pass", 1)


def test_matrix_product_plans_and_compiles(ctx):
    A, B, bias = ctx.spec((300, 200)), ctx.spec((200, 150)), ctx.spec((150,))
    out = gr.tanh(A @ B + bias) * 2.0
    assert groups(out) == [("GEMM", ["dot", "add", "tanh", "mul"])]      # pointwise consumers run as the epilogue
    src = out.source(0)
    assert "__builtin_amdgcn_mfma_f32_32x32x2f32" in src and "__shared__" in src
    out.compile()
    (ctx.spec((200, 300)).T @ B).compile()                # left operand contiguous along m
    (A @ ctx.spec((150, 200)).T).compile()                # right operand contiguous along k
    (A[::2, ::2] @ B[::2, ::3]).compile()                 # neither: scalar loads
    chain = (A @ B) @ ctx.spec((150, 64))                 # a product feeding a product: two sub-graphs
    assert [k for k, _ in groups(chain)] == ["GEMM", "GEMM"]
    lazy_operand = gr.exp(A) @ B                          # operands are materialised first (Section 2)
    assert [k for k, _ in groups(lazy_operand)] == ["MAP", "GEMM"]


def test_rowred_and_dot_cases_compile(ctx):
    for i, p in enumerate(ROWRED_PROGRAMS):
        p(gr, ctx.spec((50, 50) if i >= 5 else (50, 333))).compile()
    for prog, what in DOT_CASES:
        prog(gr, ctx.spec((70, 130)), ctx.spec((130,)), ctx.spec((70,))).compile()
    wl.mnist(gr, ctx.spec((200, 10)), ctx.spec((200,)), ctx.spec((10,))).compile()
    wl.listing1(gr, ctx.spec((10, 20), gr.GR_I32), ctx.spec((20,), gr.GR_I32)).compile()


def test_streaming_store_hint_rule(ctx):
    hint = "__builtin_nontemporal_store"
    big, small = ctx.spec((8192, 8192)), ctx.spec((1024, 1024))
    assert hint in (big * 2.0).source(0) and hint not in (small * 2.0).source(0)
    assert hint in wl.softmax(gr, ctx.spec((16384, 4096))).source(0)
    # an intermediate result of the same request keeps plain stores; the requested value is streamed
    out = gr.cumsum(big, 1) * 2.0
    assert hint not in out.source(0) and hint in out.source(1)
    # a transposed operand read through LDS tiles: only where output rows start on 64-byte boundaries
    assert hint in (big.T * 1.0).source(0) and hint not in (ctx.spec((8191, 8191)).T * 1.0).source(0)
    ctx.set_option("nontemporal", 0)
    assert hint not in (big * 3.0).source(0) and "__builtin_nontemporal_load" not in (big * 3.0).source(0)
    ctx.set_option("nontemporal", 9)
    assert hint in (small * 3.0).source(0)
    ctx.set_option("nontemporal", 1)


def test_same_structure_hits_the_kernel_cache(ctx):
    (ctx.spec((64, 300)) * 2.0 + 1.0).compile()
    s0 = ctx.stats()
    (ctx.spec((80, 500)) * 3.0 + 7.0).compile()
    s1 = ctx.stats()
    assert s1["cache_misses"] == s0["cache_misses"] and s1["cache_hits"] == s0["cache_hits"] + 1


def test_disk_cache_round_trip_and_corruption(tmp_path, monkeypatch):
    monkeypatch.setenv("GR_CACHE_DIR", str(tmp_path / "kernels"))
    monkeypatch.setenv("GR_KERNEL_PACK", "")   # no ahead-of-time pack in this test

    def program(c):
        x = c.spec((64, 300))
        return gr.tanh(x * 3.0 + 0.125) - gr.sum(gr.sqrt(abs(x)), axis=0, keepdims=True)

    c1 = gr.Context(device=-1)
    program(c1).compile()
    s1 = c1.stats()
    assert s1["cache_misses"] == 2 and s1["disk_hits"] == 0 and s1["compile_ms"] > 0
    files = sorted((tmp_path / "kernels").iterdir())
    assert len(files) == 2 and all(f.suffix == ".co" for f in files)
    c2 = gr.Context(device=-1)          # a new context (a new process would do the same): served from disk
    program(c2).compile()
    s2 = c2.stats()
    assert s2["disk_hits"] == 2 and s2["compile_ms"] == 0
    files[0].write_bytes(b"garbage")     # a damaged file is ignored and rewritten
    c3 = gr.Context(device=-1)
    program(c3).compile()
    s3 = c3.stats()
    assert s3["disk_hits"] == 1 and s3["compile_ms"] > 0
    assert files[0].stat().st_size > 100
    c4 = gr.Context(device=-1)
    c4.set_option("disk_cache", 0)
    program(c4).compile()
    assert c4.stats()["disk_hits"] == 0
    for c in (c1, c2, c3, c4):
        c.close()


def test_kernel_pack_is_read_after_the_user_cache_and_never_written(tmp_path, monkeypatch):
    # a directory of code objects written by one context serves as the read-only pack of another
    pack, user = tmp_path / "pack", tmp_path / "user"

    def program(c):
        x = c.spec((300, 70))
        return gr.tanh(x) * 3.0 + gr.sum(x, axis=1, keepdims=True)

    monkeypatch.setenv("GR_KERNEL_PACK", "")
    monkeypatch.setenv("GR_CACHE_DIR", str(pack))
    c1 = gr.Context(device=-1)
    program(c1).compile()
    s1 = c1.stats()
    assert s1["disk_hits"] == 0 and s1["cache_misses"] >= 1 and s1["compile_ms"] > 0
    packed = sorted(f.name for f in pack.iterdir())
    assert len(packed) == s1["cache_misses"]
    monkeypatch.setenv("GR_KERNEL_PACK", str(pack))
    monkeypatch.setenv("GR_CACHE_DIR", str(user))
    c2 = gr.Context(device=-1)
    program(c2).compile()
    s2 = c2.stats()
    assert s2["disk_hits"] == s1["cache_misses"] and s2["compile_ms"] == 0
    assert not list(user.iterdir()) and sorted(f.name for f in pack.iterdir()) == packed
    (c2.spec((300, 70)) * 2.0 - 1.0).compile()            # not in the pack: compiled, stored in the user's cache only
    assert c2.stats()["compile_ms"] > 0 and len(list(user.iterdir())) == 1 and sorted(f.name for f in pack.iterdir()) == packed
    c3 = gr.Context(device=-1)
    c3.set_option("disk_cache", 0)                          # switches the pack off as well
    program(c3).compile()
    assert c3.stats()["disk_hits"] == 0
    for c in (c1, c2, c3):
        c.close()


def test_built_kernel_pack_covers_the_benchmark_programs(monkeypatch, tmp_path):
    from paper_1901_03771_amd import kernel_pack
    if not os.path.isdir(kernel_pack.PACK_DIR) or not any(f.endswith(".co") for f in os.listdir(kernel_pack.PACK_DIR)):
        pytest.skip("the kernel pack has not been built")
    monkeypatch.delenv("GR_KERNEL_PACK", raising=False)
    monkeypatch.setenv("GR_CACHE_DIR", str(tmp_path / "user"))
    c = gr.Context(device=-1)
    X = c.spec((8192, 8192))
    wl.normalize(gr, X, c.spec((1, 8192)), c.spec((1, 8192)), c.spec((8192,)), c.spec((8192,))).compile()
    wl.softmax(gr, c.spec((16384, 4096))).compile()
    gr.sum(c.spec((1 << 24,))).compile()
    st = c.stats()
    assert st["compile_ms"] == 0 and st["disk_hits"] == st["cache_misses"] >= 3
    c.close()


def test_async_and_serial_compilation_agree(ctx):
    ctx.set_option("disk_cache", 0)
    x = ctx.spec((32, 200))
    out = gr.exp(gr.cumsum(x, 1)) + gr.sum(x * x, axis=0) * 2.0 + gr.max(x, axis=1, keepdims=True)
    n = len(out.plan().splitlines())
    assert n >= 3
    ctx.set_option("async_compile", 0)
    out.compile()
    serial = ctx.stats()["cache_misses"]
    c2 = gr.Context(device=-1)
    c2.set_option("disk_cache", 0)
    x2 = c2.spec((32, 200))
    out2 = gr.exp(gr.cumsum(x2, 1)) + gr.sum(x2 * x2, axis=0) * 2.0 + gr.max(x2, axis=1, keepdims=True)
    out2.compile()                        # all kernels of the request compiled concurrently
    assert c2.stats()["cache_misses"] == serial == n
    assert [out.source(i) for i in range(n)] == [out2.source(i) for i in range(n)]
    c2.close()


def test_kernel_signature_determines_the_source(ctx):
    # Kernels are cached by a signature of the sub-graph, not by their text.  In the self-checking mode a cache hit
    # regenerates the source and compares it with the one the cached kernel was compiled from: variants of a matrix
    # product that differ only in how the planner runs them (K divided over workgroups or not, tiles loaded straight
    # into LDS or staged through registers, narrow tiles) must not share a signature unless they share their text.
    # (A product without a split once found the kernel of a split one under its signature and wrote its partial tile
    # through a workspace pointer that nobody had set.)
    ctx.set_option("plan_cache", 2)
    ctx.set_option("disk_cache", 0)
    seen = set()
    for big, split, bn in [(1, 1, 0), (1, 2, 0), (1, 1, 0), (1, 3, 0), (0, 2, 0), (0, 1, 0), (1, 2, 0), (0, 1, 32), (1, 1, 0)]:
        for k, v in (("gemm_big", big), ("gemm_split", split), ("gemm_bn", bn)):
            ctx.set_option(k, v)
        out = ctx.spec((512, 384)) @ ctx.spec((384, 512)) + ctx.spec((512,))
        out.compile()                      # fails with "source differs" if a signature stands for two texts
        seen.add(out.source(0))
    assert len(seen) == 4 and ctx.stats()["cache_misses"] == 4
    for k in ("gemm_split", "gemm_bn"):
        ctx.set_option(k, 0)
    ctx.set_option("gemm_big", 1)


def test_signatures_determine_sources_over_random_products_and_options():
    # The same invariant without compiling anything: a dry run in the self-checking mode generates the source of
    # every sub-graph it would launch and compares it with the source of any earlier sub-graph of the same signature.
    # Four hundred matrix products: random extents (K a multiple of 16 or not), layouts, epilogues and planner options.
    c = gr.Context(device=-1)
    c.set_option("dry_run", 2)
    c.set_option("plan_cache", 2)
    g = np.random.default_rng(77)
    for case in range(400):
        c.set_option("gemm_split", int(g.choice([0, 0, 0, 1, 2, 3, 7])))
        c.set_option("gemm_big", int(g.choice([1, 1, 0])))
        c.set_option("gemm_bn", int(g.choice([0, 0, 0, 32, 128])))
        M, N = (int(v) for v in g.choice([64, 128, 200, 256, 516, 1024, 2048, 4096], 2))
        K = int(g.choice([32, 48, 100, 256, 1040, 4096]))
        A = c.spec((K, M)).T if g.integers(2) else c.spec((M, K))
        B = c.spec((N, K)).T if g.integers(2) else c.spec((K, N))
        out = A @ B
        if g.integers(2): out = gr.tanh(out + c.spec((N,)))
        if g.integers(3) == 0: out = out * c.spec((M, N))
        out.materialize()
    del A, B, out
    assert c.stats()["nodes_alive"] == 0
    c.close()


def test_generated_code_has_no_contraction_or_packed_math(ctx):
    src = wl.chain(gr, ctx.spec((4096,)), ctx.spec((4096,))).source(0)
    # the only fused multiply-adds are inside the math helpers: two in the square root (its Newton step needs the
    # exact residual; its results are the IEEE square root's, checked for every float32 on the device), the
    # polynomial steps of erf, the extended-precision products of exp and log (two each, log in both of its branches;
    # within 2 ulp of the oracle for every float32 pattern tested on the device), and the refinement steps of a
    # quotient by a constant (the steps of the compiler's own IEEE division; checked bit for bit on the device).
    # The recorded operations themselves are never contracted.
    helper = src[src.index("gr_sqrtf(float x) {"):]
    helper = helper[:helper.index("\n}\n") + 3]
    assert helper.count("fmaf") == 2
    rest = src.replace(helper, "")
    shared = [line for line in rest.splitlines() if "gr_erff(float x)" in line]
    assert len(shared) == 1 and "gr_divc(float x, float c)" in shared[0] and shared[0].count("__builtin_fmaf") == 11 + 2 + 4 + 6
    shared = shared[0]
    rest = rest.replace(shared, "")
    assert "fmaf" not in rest and "__fdividef" not in src and "__expf" not in src


def test_asm_statements_of_the_direct_loads_leave_the_condition_code_alone(ctx):
    # The compiler splits its own 64-bit scalar additions (s_add_u32 .. s_addc_u32) around an asm statement, which
    # therefore must not write the scalar condition code: the only instructions allowed in one are a move into M0,
    # wait states and the load itself, and M0 is declared clobbered.
    import re
    for out in (ctx.spec((4096, 1024)) @ ctx.spec((1024, 4096)), ctx.spec((1024, 2048)).T @ ctx.spec((2048, 1024)).T + ctx.spec((2048,))):
        assert "direct" in out.plan()
        src = out.source(0)
        stmts = re.findall(r'asm volatile\("([^"]*)"([^;]*);', src)
        assert len(stmts) >= 12
        for text, rest in stmts:
            assert text == r"s_mov_b32 m0, %2\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %0, %1", text
            assert '"memory", "m0"' in rest


def test_generated_kernels_keep_their_values_in_registers(ctx, tmp_path):
    # Large point functions (tanh, erf, exp, log in an epilogue) must not push accumulators or patch values
    # into scratch memory: the kernels are compiled to gfx950 assembly offline and searched for scratch
    # accesses and a private segment.  (A matrix-product epilogue with tanh once did exactly that.)
    import re
    import shutil
    import subprocess
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")

    def heavy(x):
        return gr.erf(gr.tanh(x) * 0.5) + gr.exp(-abs(x)) * gr.log(abs(x) + 1.0)

    X, V, M2 = ctx.spec((4096, 1024)), ctx.spec((1024,)), ctx.spec((1024, 512))
    progs = {
        "gemm": heavy(X @ M2) + ctx.spec((512,)),
        "gemm narrow": heavy(X @ ctx.spec((1024, 32))),
        "gemm, 256 x 256 tiles": heavy(X @ ctx.spec((1024, 4096))) + ctx.spec((4096,)),
        "gemm, 256 x 256 tiles, transposed views": heavy(ctx.spec((1024, 4096)).T @ ctx.spec((4096, 1024)).T),
        # (the loops over the accumulators are unrolled in the generated text: the compiler gives up on "#pragma unroll"
        # beyond a size that this epilogue passes several times over, and the accumulators would move to scratch memory)
        "gemm, 256 x 256 tiles, an epilogue four times as long": heavy(heavy(heavy(heavy(X @ ctx.spec((1024, 4096)))))) + ctx.spec((4096,)),
        "gemm, an epilogue four times as long": heavy(heavy(heavy(heavy(X @ M2)))),
        "gemv": heavy(X @ V),
        "rowred": heavy(X - gr.max(X, axis=1, keepdims=True)) / gr.sum(heavy(X), axis=1, keepdims=True),
        "map": heavy(wl.stencil(gr, X)),
        "scan": gr.cumsum(heavy(X), 0),
    }
    assert all("tile=256x256" in out.plan() for name, out in progs.items() if "256 x 256" in name)
    for name, out in progs.items():
        src = tmp_path / "k.hip"
        src.write_text("#include <hip/hip_runtime.h>\n" + out.source(0))
        asm = tmp_path / "k.s"
        subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                        "-S", "--cuda-device-only", "-o", str(asm), str(src)], check=True, capture_output=True, timeout=600)
        text = asm.read_text()
        assert "scratch_" not in text, name
        assert all(int(v) == 0 for v in re.findall(r"\.private_segment_fixed_size:\s+(\d+)", text)), name


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_api_arguments_are_answered_with_statuses(seed):
    """Arbitrary arguments (stale handles, absurd ranks, extents of 2^40, empty axes, misaligned pointers) end in
    a status code, never in a crash, a hang or an arithmetic overflow: planning runs on a device-less context
    that skips launches, so everything short of the kernels themselves is exercised."""
    import ctypes
    import random

    L = gr.lib()
    ctx = gr.Context(device=-1)
    ctx.set_option("dry_run", 2)
    P = ctx._p
    r = random.Random(seed)
    handles = [0, 1, 2, 999999, 2**63]
    I64 = ctypes.c_int64
    out = ctypes.c_uint64()

    def h():
        return ctypes.c_uint64(r.choice(handles))

    def extents(n):
        n = max(n, 1)
        return (I64 * n)(*[r.choice([-5, -1, 0, 1, 2, 3, 7, 64, 2**40]) for _ in range(n)])

    made = 0
    for _ in range(6000):
        k = r.randrange(15)
        st = None
        if k == 0:
            nd = r.choice([-1, 0, 1, 2, 3, 8, 9, 100])
            m = min(max(nd, 0), 12)
            st = L.gr_array_from_device(P, ctypes.c_void_p(r.choice([0, 0x1000, 0x1003])), r.choice([0, 1, 2, 3, -1]), nd,
                                        extents(m) if r.random() < 0.9 else None, extents(m) if r.random() < 0.3 else None,
                                        ctypes.byref(out))
        elif k == 1:
            st = L.gr_unary(P, r.choice([0, 1, 2, 3, 4, 5, 6, 7, 8, 16, -1, 99]), h(), ctypes.byref(out))
        elif k == 2:
            st = L.gr_binary(P, r.choice([16, 17, 18, 19, 20, 21, 0, 22, -3]), h(), h(), ctypes.byref(out))
        elif k == 3:
            st = L.gr_binary_scalar(P, r.choice([16, 17, 18, 19, 20, 21, 5]), h(), r.choice([0.0, 1.5, -2.0, float("nan"), 1e40, 3.0]),
                                    r.choice([0, 1]), r.choice([0, 1]), ctypes.byref(out))
        elif k == 4:
            n = r.choice([0, 1, 2, 3, 9, -1])
            m = max(n, 1)
            U8 = ctypes.c_uint8 * m
            st = L.gr_slice(P, h(), n, extents(m), extents(m), (I64 * m)(*[r.choice([1, 2, 3, 0, -1]) for _ in range(m)]),
                            U8(*[r.choice([0, 1]) for _ in range(m)]), U8(*[r.choice([0, 1]) for _ in range(m)]), ctypes.byref(out))
        elif k == 5:
            perm = (ctypes.c_int * 8)(*[r.choice([0, 1, 2, 3, -1, 7, 9]) for _ in range(8)])
            st = L.gr_transpose(P, h(), perm if r.random() < 0.8 else None, ctypes.byref(out))
        elif k == 6:
            axes = (ctypes.c_int * 8)(*[r.choice([0, 1, 2, -1, -2, 5, 9]) for _ in range(8)])
            st = L.gr_reduce(P, r.choice([32, 33, 34, 0, 35]), h(), axes, r.choice([0, 1, 2, 3, 9, -1]), r.choice([0, 1]), ctypes.byref(out))
        elif k == 7:
            st = L.gr_scan(P, r.choice([32, 33, 34, 1]), h(), r.choice([0, 1, -1, 5, -9]), ctypes.byref(out))
        elif k == 8:
            st = L.gr_dot(P, h(), h(), ctypes.byref(out))
        elif k == 9:
            nd = r.choice([0, 1, 2, 3, 9, -1])
            st = L.gr_reshape(P, h(), nd, extents(nd), ctypes.byref(out))
        elif k == 10:
            st = L.gr_materialize(P, h())
        elif k == 11:
            st = L.gr_assign(P, h(), h())
        elif k == 12 and r.random() < 0.2:
            st = L.gr_release(P, h())
        elif k == 13:
            need = ctypes.c_size_t()
            st = L.gr_plan_describe(P, h(), None, 0, ctypes.byref(need))
        elif k == 14:
            st = L.gr_materialize_into(P, h(), ctypes.c_void_p(r.choice([0, 0x2000, 0x2002])), r.choice([0, 4, 16, 4096]))
        assert st is None or 0 <= st <= 11
        if st == 0 and k <= 9:
            made += 1
            handles.append(out.value)
            if len(handles) > 60:
                handles.pop(r.randrange(5, len(handles)))
    assert made > 200
    ctx.close()


def test_repeated_requests_reuse_the_remembered_plan(ctx):
    # An iterative program records the same expression again over new nodes: from the second sweep on the
    # partition comes from the plan cache.  With "plan_cache" = 2 every hit is also planned afresh and the
    # request fails if the two plans differ, so this doubles as the check of the cache's fingerprint.
    import fuzz
    ctx.set_option("dry_run", 2)
    ctx.set_option("plan_cache", 2)
    from paper_1901_03771_amd import workloads as W
    grid = ctx.spec((130, 258))
    for _ in range(4):
        grid[1:-1, 1:-1] = W.jacobi_sweep(gr, grid)
    X, w, y = ctx.spec((3001, 200)), ctx.spec((200,)), ctx.spec((3001,))
    for _ in range(3):
        w = W.logreg(gr, X, w, y).materialize()
    h0 = ctx.stats()["plan_hits"]
    assert h0 >= 4
    # the same structure over different constants, shapes, strides, sharing or recording order is a different request
    a, b = ctx.spec((64, 32)), ctx.spec((64, 32))
    def hits_after(f):
        before = ctx.stats()["plan_hits"]
        f().materialize()
        return ctx.stats()["plan_hits"] - before
    assert hits_after(lambda: a * 2.0 + b) == 0
    assert hits_after(lambda: a * 2.0 + b) == 1
    assert hits_after(lambda: a * 3.0 + b) == 0                       # another constant
    assert hits_after(lambda: a * 2.0 + a) == 0                       # operands shared
    assert hits_after(lambda: ctx.spec((64, 33)) * 2.0 + ctx.spec((64, 33))) == 0
    assert hits_after(lambda: ctx.spec((64, 32), strides=(1, 64)) * 2.0 + b) == 0
    assert hits_after(lambda: a[:, 1:] * 2.0 + b[:, :-1]) == 0
    assert hits_after(lambda: a[:, 1:] * 2.0 + b[:, :-1]) == 1
    assert hits_after(lambda: a[:, 2:] * 2.0 + b[:, :-2]) == 0
    def other_order():
        t = b + 0.0
        return a * 2.0 + t
    def this_order():
        t = a * 2.0
        return t + (b + 0.0)
    assert hits_after(this_order) == 0 and hits_after(this_order) == 1 and hits_after(other_order) == 0
    ctx.set_option("fusion", 0)                                       # options are part of the fingerprint
    assert hits_after(lambda: a * 2.0 + b) == 0
    ctx.set_option("fusion", 1)
    # random programs, each run three times in a row on the same context
    before = ctx.stats()["plan_hits"]
    for seed in list(range(7000, 7150)) + list(range(400000, 400060)):
        dtype, shapes, steps, res = fuzz.make_recipe(seed, assign=(seed % 2 == 0), reshape=seed >= 400000)
        for rep in range(3):
            leaves = [ctx.spec(s_, gr.GR_I32 if dtype == "i32" else gr.GR_F32) for s_ in shapes]
            for x in fuzz.apply(gr, steps, leaves):
                x.materialize()
    assert ctx.stats()["plan_hits"] - before > 300
    ctx.set_option("plan_cache", 0)
    assert hits_after(lambda: a * 2.0 + b) == 0


_BINDING_PROBE = r"""
import sys, json
import numpy as np
from paper_1901_03771_amd import lazy as gr, workloads as W
ctx = gr.Context(device=-1)
out = {"fast": gr._fastbind is not None}
a, b = ctx.spec((6, 40)), ctx.spec((6, 40))
i = ctx.spec((6, 40), gr.GR_I32)
progs = {
    "ops": lambda: gr.maximum(abs(-a) * 2 + 1.5 - b / 3.0, 0.25) ** 2 @ b.T,
    "rops": lambda: 2 * a + (1.0 - b) + 3 / (a * a) - np.float32(0.5) * b,
    "int": lambda: (i * 3 - i) + 7,
    "slices": lambda: a[1:-1, ::2] + b[:-2, 1::2] + a[..., 0:20][1:5] if False else a[1:-1, ::2] + b[:-2, 1::2],
    "reduce": lambda: gr.sum(gr.exp(a - gr.max(a, axis=1, keepdims=True)), axis=(0, 1)) + a.sum(axis=-1).max(),
    "softmax": lambda: W.softmax(gr, a),
    "stencil": lambda: W.stencil(gr, ctx.spec((40, 50))),
}
for k, f in progs.items():
    r = f()
    out[k] = [list(r.shape), r.ndim, r.plan().count("\n")]
def code_of(f):
    try:
        f()
    except gr.GrError as e:
        return e.code
    except Exception as e:
        return type(e).__name__
    return "no error"
out["errors"] = [code_of(lambda: a + True), code_of(lambda: a + "x"), code_of(lambda: a[0]), code_of(lambda: a ** 3),
                 code_of(lambda: a + ctx.spec((7, 40))), code_of(lambda: i * 0.5), code_of(lambda: i + 2**40),
                 code_of(lambda: a.__setitem__((slice(None), slice(None)), 1.0)), code_of(lambda: gr.sum(a, axis=())),
                 code_of(lambda: gr.sum(a, axis=5)), code_of(lambda: a @ 3), code_of(lambda: a + gr.Context(device=-1).spec((6, 40)))]
ctx.set_option("dry_run", 2)
del r
import gc
gc.collect()
g = ctx.spec((34, 66))
base = ctx.stats()["nodes_alive"]
for _ in range(3):
    g[1:-1, 1:-1] = W.jacobi_sweep(gr, g)
tmp = a * 2.0 + g[0:6, 0:40]
del tmp
out["alive_after_jacobi"] = ctx.stats()["nodes_alive"] - base
ctx2 = gr.Context(device=-1)
z = ctx2.spec((3,)) + 1.0
ctx2.close()
out["closed"] = code_of(lambda: z + 1.0)
del z
print(json.dumps(out))
"""


def test_c_fast_paths_and_ctypes_route_of_the_binding_agree():
    # The Array type's operators run in C (_fastbind); GRUMPY_NO_FASTBIND=1 selects the ctypes-only
    # implementation of the same calls.  Both record the same DAGs, raise the same errors and release
    # every handle.
    import json
    import subprocess
    import sys
    outs = []
    for no_fast in ("0", "1"):
        env = dict(os.environ, GRUMPY_NO_FASTBIND=no_fast)
        r = subprocess.run([sys.executable, "-c", _BINDING_PROBE], env=env, capture_output=True, text=True, timeout=300,
                           cwd=os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
        assert r.returncode == 0, r.stderr[-2000:]
        outs.append(json.loads(r.stdout.strip().splitlines()[-1]))
    assert outs[0].pop("fast") is True and outs[1].pop("fast") is False
    assert outs[0].pop("closed") in ("RuntimeError", "GR_ERR_ARG") and outs[1].pop("closed") in ("RuntimeError", "GR_ERR_ARG")
    assert outs[0] == outs[1]
    assert outs[0]["alive_after_jacobi"] == 0
    assert outs[0]["errors"] == ["GR_ERR_UNSUPPORTED", "TypeError", "GR_ERR_UNSUPPORTED", "GR_ERR_UNSUPPORTED", "GR_ERR_SHAPE", "GR_ERR_DTYPE",
                                 "GR_ERR_DTYPE", "GR_ERR_UNSUPPORTED", "GR_ERR_AXIS", "GR_ERR_AXIS", "TypeError", "ValueError"]



@pytest.mark.parametrize("case", NARROW_CASES, ids=[c[0] for c in NARROW_CASES])
def test_narrow_arrays_and_small_contractions_plan_and_compile(ctx, case):
    name, shapes, prog = case
    out = prog(gr, **{k: ctx.spec(s_) for k, s_ in shapes.items()})
    kinds = [k for k, _ in groups(out)]
    # a contraction over at most eight terms is part of the point function: no contraction kernel
    assert ("GEMV" in kinds or "GEMM" in kinds) == (name == "small product feeding a large one"), kinds
    out.compile()


def test_small_contractions_fuse_with_their_neighbours(ctx):
    x, m, v = ctx.spec((1000, 3)), ctx.spec((3, 3)), ctx.spec((3,))
    assert groups(gr.tanh((x * 2.0) @ m + v)) == [("MAP", ["mul", "dot", "add", "tanh"])]
    assert [k for k, _ in groups(x @ v)] == ["MAP"]
    assert [k for k, _ in groups(ctx.spec((100, 9)) @ ctx.spec((9,)))] == ["GEMV"]        # nine terms: a contraction kernel
    src = (x - v).source(0)
    assert "c0 + 3 == C" in src                                                           # narrow arrays: straight-line code for the last columns
    assert "c0 + 3 == C" not in (ctx.spec((1000, 67)) - ctx.spec((67,))).source(0)        # wide ones keep the generic edge path



def test_mean_records_a_sum_and_a_division(ctx):
    x = ctx.spec((64, 1000))
    assert gr.mean(x, axis=1).shape == (64,) and gr.mean(x).shape == () and x.mean(axis=0, keepdims=True).shape == (1, 1000)
    d = x - gr.mean(x, axis=1, keepdims=True)
    ln = d / gr.sqrt(gr.mean(d * d, axis=1, keepdims=True) + 1e-5)
    assert groups(ln) == [("ROWRED", ["sum", "div", "sub", "mul", "sum", "div", "add", "sqrt", "div"])]   # layer norm: one kernel
    ln.compile()


def test_var_std_clip_are_recorded_from_existing_ops(ctx):
    x = ctx.spec((64, 1000))
    assert gr.var(x, axis=1).shape == (64,) and x.std(axis=0, keepdims=True).shape == (1, 1000) and gr.clip(x, -1.0, 1.0).shape == (64, 1000)
    z = (x - gr.mean(x, axis=1, keepdims=True)) / (gr.std(x, axis=1, keepdims=True) + 1e-6)
    assert [k for k, _ in groups(z)] == ["ROWRED"]            # standardising rows: one row-resident kernel
    assert groups(gr.clip(x * 2.0, 0.0, 6.0)) == [("MAP", ["mul", "maximum", "minimum"])]
    z.compile()


# ------------------------------------------------- lifetime of wrapped leaf memory --
@pytest.mark.parametrize("fast", [True, False])
def test_results_keep_the_memory_of_their_leaves_alive(fast, monkeypatch):
    # The recorded DAG outlives the handles of its leaves: a result must hold whatever keeps the leaves'
    # device memory alive until it has storage of its own.  Both binding routes (the C type and ctypes).
    import gc
    import subprocess
    import sys
    code = r'''
import gc, weakref, sys
from paper_1901_03771_amd import lazy as gr
class Mem:            # stands for a tensor
    pass
ctx = gr.Context(device=-1)
ctx.set_option("dry_run", 2)
def leaf(shape):
    m = Mem()
    return ctx.from_device(0x10000, gr.GR_F32, shape, owner=m), weakref.ref(m)
a, wa = leaf((8, 8)); b, wb = leaf((8,)); c, wc = leaf((8, 8))
z = gr.exp(a * 2.0 + b)[1:3].T @ gr.sum(c, axis=1)[1:3]
del a, b, c
gc.collect()
assert wa() is not None and wb() is not None and wc() is not None, "a leaf's memory was released while a recorded array still reads it"
z.materialize()
gc.collect()
assert wa() is None and wb() is None and wc() is None, "an evaluated array still holds its leaves' memory"
# a view keeps its base's memory, evaluated or not; a copy lets go of it
a, wa = leaf((8, 8))
v = a[2:4]
del a
v.materialize(); gc.collect()
assert wa() is not None
w = v.copy()
del v; gc.collect()
assert wa() is None
# materialize_into: bound to the caller's buffer (an array without storage) or copied (a leaf, a view)
a, wa = leaf((8,))
t = Mem(); t.data_ptr = lambda: 0x20000; t.numel = lambda: 8; t.element_size = lambda: 4
wt = weakref.ref(t)
y = a + 1.0
y.materialize_into(t)
del a; gc.collect()
assert wa() is None and y._owner is t
a, wa = leaf((8,))
a.materialize_into(t)
assert a._owner is not t and wa() is not None
# an iteration x = f(x) that evaluates every step does not accumulate owners
x, wx = leaf((8,))
for _ in range(50):
    x = (x * 0.5 + 1.0).materialize()
gc.collect()
assert wx() is None and x._owner is None
print("ok")
'''
    env = dict(os.environ, PYTHONPATH=ROOT)
    if not fast:
        env["GRUMPY_NO_FASTBIND"] = "1"
    r = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout + r.stderr
