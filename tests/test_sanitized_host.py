"""The host side of the library (recorder, planner, plan cache, code generator, runtime bookkeeping) under
AddressSanitizer and UndefinedBehaviorSanitizer, without a GPU: the library is built with its host code
instrumented (paper_1901_03771_amd.build.build_sanitized) and driven, in a process that preloads the sanitizer
runtime, through a device-less context in dry-run mode -- materialise and assign calls then run completely except
for the launches.  Driven by the seeded random programs of fuzz.py (every array of a program evaluated, slice
assignments and reshapes included, each request planned twice in the self-checking plan-cache mode), by the
programs of the five configurations through every entry point that evaluates (plain, into a buffer, without
allocating, recorded and replayed), and by random, mostly invalid calls into the C ABI (fuzz_api.py)."""
import os
import subprocess
import sys

import pytest

from paper_1901_03771_amd import build as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = r'''
import sys
sys.path.insert(0, ROOT); sys.path.insert(0, ROOT + "/tests")
import fuzz, fuzz_api
from paper_1901_03771_amd import lazy as gr, workloads as wl
assert gr.LIB_PATH.endswith("_san.so")

# ---- random programs, every array evaluated; compiled (dry_run 1) for a few, planned only (2) for the rest
for mode, seeds, kw in (("plain", range(0, 120), {}), ("assign", range(500000, 500080), dict(assign=True)),
                        ("assign values + reshape", range(800000, 800060), dict(assign=True, assign_values=True, reshape=True)),
                        ("big", range(900000, 900020), dict(big=True))):
    ctx = gr.Context(device=-1)
    ctx.set_option("dry_run", 2)
    ctx.set_option("plan_cache", 2)        # reuse remembered plans, and plan afresh to compare
    for seed in seeds:
        dtype, shapes, steps, res = fuzz.make_recipe(seed, max_steps=14, **kw)
        dt = gr.GR_I32 if dtype == "i32" else gr.GR_F32
        for rep in range(2):               # the second time round every request hits the plan cache
            pool = fuzz.apply(gr, steps, [ctx.spec(s, dt) for s in shapes])
            for i in (range(len(pool)) if "assign" in kw else [res]):
                pool[i].materialize()
            del pool
    assert ctx.stats()["nodes_alive"] == 0, mode
    ctx.close()
    print("random programs:", mode, "ok", flush=True)

# ---- the configurations through every evaluating entry point, kernels compiled for real
ctx = gr.Context(device=-1)
ctx.set_option("dry_run", 1)
ctx.set_option("disk_cache", 0)
class Buf:                                  # stands for a tensor: an address and a size
    def __init__(self, ptr, n): self.ptr, self.n = ptr, n
    def data_ptr(self): return self.ptr
    def numel(self): return self.n
    def element_size(self): return 4
for name, shapes in (("chain", dict(a=(5000,), b=(5000,))), ("softmax", dict(X=(33, 700))), ("stencil", dict(I=(40, 300))),
                     ("logreg", dict(X=(3001, 200), w=(200,), y=(3001,))), ("normalize", dict(X=(20, 300), mu=(1, 300), sigma=(1, 300), gamma=(300,), beta=(300,)))):
    leaves = {k: ctx.spec(s) for k, s in shapes.items()}
    def value(): return wl.PROGRAMS[name](gr, **leaves)
    n = 1
    for d in value().shape: n *= d
    value().materialize()                   # (map and row-resident sub-graphs: answered by the interpreter while hipRTC compiles)
    value().materialize_into(Buf(0x40000000, n))
    ctx.compile_wait()                      # the non-allocating entry point wants its kernels loaded
    value().materialize_into_static(Buf(0x40000000, n))
    prog = ctx.program(value(), list(leaves.values()))
    for _ in range(3):
        prog.run([Buf(0x50000000 + 0x1000000 * i, 1) for i in range(len(leaves))], Buf(0x40000000, n))
    prog.close()
grid = ctx.from_device(0x60000000, gr.GR_F32, (64, 300))
ctx.check(gr.lib().gr_array_lend_buffer(ctx._p, grid.h, 0x61000000, 64 * 300 * 4))
wl.jacobi(gr, grid, 3)
x = ctx.spec((1 << 22,))
gr.cumsum(x * 2.0, 0).materialize()
gr.sum(gr.sqrt(abs(x))).materialize()
del leaves, grid, x, prog, value
assert ctx.stats()["nodes_alive"] == 0
ctx.close()
print("entry points: ok", flush=True)

# ---- random calls into the C ABI
for seed in range(6):
    print("api fuzz", seed, fuzz_api.run(gr, seed, 6000), flush=True)
print("all ok")
'''


def test_host_logic_under_address_and_undefined_behaviour_sanitizers():
    rt = b.sanitizer_runtime()
    if not rt:
        pytest.skip("the compiler's AddressSanitizer runtime was not found")
    lib = b.build_sanitized()
    env = dict(os.environ, LD_PRELOAD=rt, GRUMPY_HIP_LIB=lib, PYTHONPATH=ROOT, GR_KERNEL_PACK="",
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([sys.executable, "-X", "faulthandler", "-c", "ROOT = %r\n" % ROOT + DRIVER], env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout[-3000:] + "\n" + r.stderr[-6000:])
    assert r.returncode == 0 and r.stdout.strip().endswith("all ok"), tail
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, tail
