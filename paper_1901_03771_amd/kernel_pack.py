"""Ahead-of-time kernel pack: compiles the kernels of common sub-graphs at build time.

The paper names JIT compilation time as the main bottleneck of deferred evaluation (Section 6).
Besides overlapping compilation with execution and caching code objects per user, the library
reads a read-only directory of code objects beside the shared library: this module fills it, on a
machine without a GPU (hipRTC cross-compiles for gfx950), by planning the programs below on a
device-less context and compiling their sub-graphs.  Entries are matched by the full text of the
generated source, so a program that is planned differently at run time simply misses."""
from __future__ import annotations

import os
import time

HERE = os.path.dirname(os.path.abspath(__file__))
PACK_DIR = os.path.join(HERE, "kernel_pack")


def _programs(gr, wl, ctx):
    """Yields (name, thunk): each thunk records one program on `ctx` and returns its root."""
    shapes = {
        "chain": lambda p: dict(a=(p["n"],), b=(p["n"],)),
        "normalize": lambda p: dict(X=(p["rows"], p["cols"]), mu=(1, p["cols"]), sigma=(1, p["cols"]), gamma=(p["cols"],), beta=(p["cols"],)),
        "softmax": lambda p: dict(X=(p["rows"], p["cols"])),
        "stencil": lambda p: dict(I=(p["rows"], p["cols"])),
        "logreg": lambda p: dict(X=(p["rows"], p["cols"]), w=(p["cols"],), y=(p["rows"],)),
        "blackscholes": lambda p: dict(S=(p["n"],), K=(p["n"],), T=(p["n"],)),
        "cumsum": lambda p: dict(x=(p["n"],)),
        "cumsum_axis0": lambda p: dict(X=(p["rows"], p["cols"])),
        "gemm": lambda p: dict(A=(p["m"], p["k"]), B=(p["k"], p["n"])),
    }
    for name, prog in wl.PROGRAMS.items():
        for tag, sizes in (("full", wl.FULL[name]), ("small", wl.SMALL[name])):
            def thunk(prog=prog, sh=shapes[name](sizes)):
                return prog(gr, **{k: ctx.spec(s) for k, s in sh.items()})
            yield f"{name}/{tag}", thunk
    # the streamed sizes of the two pointwise chains, the paper's small listings
    yield "chain 2^27", (lambda: wl.chain(gr, ctx.spec((1 << 27,)), ctx.spec((1 << 27,))))
    yield "blackscholes 2^26", (lambda: wl.blackscholes(gr, ctx.spec((1 << 26,)), ctx.spec((1 << 26,)), ctx.spec((1 << 26,))))
    for n in (1 << 26, 1 << 16):
        yield f"listing 1 {n}", (lambda n=n: wl.listing1(gr, ctx.spec((n,), gr.GR_I32), ctx.spec((n,), gr.GR_I32)))
    yield "listing 2", (lambda: wl.mnist(gr, ctx.spec((200, 10)), ctx.spec((200,)), ctx.spec((10,))))
    for n in (8192, 1024):
        yield f"jacobi sweep {n}", (lambda n=n: wl.jacobi_sweep(gr, ctx.spec((n, n))))
    # 32-bit integers: pointwise, reductions (sums widen to 64 bits), scans
    for shp in ((1 << 26,), (1 << 16,), (4096, 4096)):
        yield f"i32 a*3+b {shp}", (lambda shp=shp: ctx.spec(shp, gr.GR_I32) * 3 + ctx.spec(shp, gr.GR_I32))
        for op in ("sum", "max", "min"):
            yield f"i32 {op} {shp}", (lambda op=op, shp=shp: gr.reduce(op, ctx.spec(shp, gr.GR_I32), None, False))
        yield f"i32 cumsum {shp}", (lambda shp=shp: gr.cumsum(ctx.spec(shp, gr.GR_I32), len(shp) - 1))
    # plain pointwise operations, large (streamed stores) and small, one and two dimensions
    unary = dict(neg=lambda x: -x, abs=abs, exp=gr.exp, log=gr.log, sqrt=gr.sqrt, tanh=gr.tanh, square=lambda x: x * x)
    binary = dict(add=lambda x, y: x + y, sub=lambda x, y: x - y, mul=lambda x, y: x * y, div=lambda x, y: x / y,
                  maximum=gr.maximum, minimum=gr.minimum)
    for shp in ((1 << 24,), (1 << 16,), (4096, 4096), (512, 512)):
        for n, f in unary.items():
            yield f"{n}{shp}", (lambda f=f, shp=shp: f(ctx.spec(shp)))
        for n, f in binary.items():
            yield f"{n}{shp}", (lambda f=f, shp=shp: f(ctx.spec(shp), ctx.spec(shp)))
            yield f"{n}{shp} scalar", (lambda f=f, shp=shp: f(ctx.spec(shp), 1.5))
        if len(shp) == 2:
            for n, f in binary.items():
                yield f"{n}{shp} row", (lambda f=f, shp=shp: f(ctx.spec(shp), ctx.spec(shp[1:])))
            yield f"transpose{shp}", (lambda shp=shp: ctx.spec(shp).T * 1.0)
    # reductions and scans
    for shp in ((1 << 24,), (1 << 16,), (4096, 4096), (512, 512)):
        for op in ("sum", "max", "min"):
            yield f"{op}{shp}", (lambda op=op, shp=shp: gr.reduce(op, ctx.spec(shp), None, False))
            if len(shp) == 2:
                for ax in (0, 1):
                    yield f"{op}{shp} axis {ax}", (lambda op=op, shp=shp, ax=ax: gr.reduce(op, ctx.spec(shp), ax, False))
        yield f"mean{shp}", (lambda shp=shp: gr.mean(ctx.spec(shp)))
        for ax in range(len(shp)):
            yield f"cumsum{shp} axis {ax}", (lambda shp=shp, ax=ax: gr.cumsum(ctx.spec(shp), ax))
    # contractions
    for m, k, n in ((4096, 4096, 4096), (1024, 1024, 1024), (512, 256, 64)):
        yield f"matmul {m}x{k}x{n}", (lambda m=m, k=k, n=n: ctx.spec((m, k)) @ ctx.spec((k, n)))
        yield f"matvec {m}x{k}", (lambda m=m, k=k: ctx.spec((m, k)) @ ctx.spec((k,)))
        yield f"vecmat {m}x{k}", (lambda m=m, k=k: ctx.spec((m, k)).T @ ctx.spec((m,)))
    yield "inner product", (lambda: wl.inner_product(gr, ctx.spec((1 << 20,)), ctx.spec((1 << 20,))))
    # row-resident reductions at common row lengths (lanes per row and positions per lane depend on it)
    for cols in (64, 256, 1000, 1024, 2048, 4096, 8192):
        rows = max(64, (1 << 24) // cols)
        yield f"softmax rows of {cols}", (lambda rows=rows, cols=cols: wl.softmax(gr, ctx.spec((rows, cols))))

        def layernorm(rows=rows, cols=cols):
            x = ctx.spec((rows, cols))
            return (x - gr.mean(x, axis=1, keepdims=True)) / gr.sqrt(gr.var(x, axis=1, keepdims=True) + 1e-5)
        yield f"layernorm rows of {cols}", layernorm

        def l2norm(rows=rows, cols=cols):
            x = ctx.spec((rows, cols))
            return x / gr.sqrt(gr.sum(x * x, axis=1, keepdims=True))
        yield f"l2-normalised rows of {cols}", l2norm
    # a dense layer: matrix product with bias and activation in the epilogue
    for m, k, n in ((8192, 512, 512), (65536, 64, 64)):
        for act in (None, gr.tanh, lambda y: gr.maximum(y, 0)):
            def dense(m=m, k=k, n=n, act=act):
                y = ctx.spec((m, k)) @ ctx.spec((k, n)) + ctx.spec((n,))
                return act(y) if act else y
            yield f"dense {m}x{k}x{n}", dense


def build_pack(verbose: bool = False) -> int:
    """(Re)builds the pack; returns the number of code objects in it."""
    from . import lazy as gr, workloads as wl
    os.makedirs(PACK_DIR, exist_ok=True)
    for f in os.listdir(PACK_DIR):
        if f.endswith(".co") or ".co.tmp" in f:
            os.remove(os.path.join(PACK_DIR, f))
    saved = {k: os.environ.get(k) for k in ("GR_CACHE_DIR", "GR_KERNEL_PACK")}
    os.environ["GR_CACHE_DIR"] = PACK_DIR
    os.environ["GR_KERNEL_PACK"] = ""   # (empty: no pack is consulted while this one is written)
    t0 = time.time()
    try:
        ctx = gr.Context(device=-1)
        ctx.set_option("disk_cache", 1)
        pending = []
        for name, thunk in _programs(gr, wl, ctx):
            try:
                pending.append(thunk().compile())
            except gr.GrError as e:  # a program this build cannot plan is left out of the pack
                if verbose:
                    print(f"kernel pack: skipped {name}: {e}")
            if len(pending) >= 16:
                pending.clear()
        ctx.compile_wait()
        pending.clear()
        ctx.close()
    finally:
        for k, v in saved.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v
    n = sum(1 for f in os.listdir(PACK_DIR) if f.endswith(".co"))
    if verbose:
        print(f"kernel pack: {n} code objects in {time.time() - t0:.1f} s -> {PACK_DIR}")
    return n


if __name__ == "__main__":
    build_pack(verbose=True)
