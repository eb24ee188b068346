"""GPU parity on arrays of more than 2^32 elements (16 GiB of float32 each): the five
configurations, the reductions, the scans and the contractions at sizes where every
element offset, tile number and row number that is computed in 32 bits would be wrong.

Inputs are a fixed integer function of the element's flat index, written on the device by
torch in chunks and re-evaluated by numpy for the sampled positions, so the oracle never
sees a value that came from the device.  What the oracle can evaluate in seconds (windows
around the 2^31 and 2^32 element boundaries, the first and last elements, random rows) is
compared element by element; results that need every input are compared on sampled outputs
the oracle can evaluate one by one (columns for column sums and for the products with the
transposed matrix) or, for inputs with a closed form that the oracle confirms on a prefix
(periodic values for the sum of everything, scans whose partial sums are exact), everywhere.

All big arrays live in one allocation with 8 GiB of unused memory in front of the first and
16 GiB behind the last: an offset whose upper bits were lost, or that was sign-extended from
32 bits, would still point into that allocation and give a wrong value instead of a fault.
"""
import os

import numpy as np
import pytest

import oracle as ora
from helpers import elementwise_close, reduction_check
from paper_1901_03771_amd import workloads as wl

pytestmark = pytest.mark.gpu

GIB = 1 << 30
GUARD_FRONT, GUARD_BACK, SLOT = 8 * GIB, 16 * GIB, 17 * GIB
N = (1 << 32) + 4099                 # one line
ROWS, COLS = (1 << 21) + 3, 2048     # a matrix of 2^32 + 6144 elements; row 2^20 starts at element 2^31
TALL = (1 << 23) + 1                 # rows of the 512-column matrix of the logistic regression
DEEP = (1 << 20) + 1                 # rows of the 4096-column left operand of the matrix product


def lattice(i):
    """A fixed, well-mixed function of the flat index with values in [0, 2^24); `i` is an int64
    numpy array or torch tensor (only %, *, + on int64, no intermediate reaches 2^48)."""
    return ((i % 2147483629) * 48271 + 11) % 16777213


def as_unit(v):       # [-1, 1), exact in float32
    return (v - 8388608) * (1.0 / 8388608.0)


def as_positive(v):   # [2^-24, 1], exact in float32
    return (v + 1) * (1.0 / 16777216.0)


class Slab:
    def __init__(self, torch):
        self.torch = torch
        torch.cuda.empty_cache()
        need = GUARD_FRONT + 3 * SLOT + GUARD_BACK
        free, _ = torch.cuda.mem_get_info()
        if free < need + 4 * GIB:
            pytest.skip(f"needs {need >> 30} GiB of free device memory, {free >> 30} GiB are free")
        self.mem = torch.empty(need, dtype=torch.uint8, device="cuda")

    def array(self, slot, shape, dtype, slots=1):
        nbytes = int(np.prod(shape)) * self.torch.empty(0, dtype=dtype).element_size()
        assert nbytes <= slots * SLOT and slot + slots <= 3
        off = GUARD_FRONT + slot * SLOT
        return self.mem[off:off + nbytes].view(dtype).view(*shape)

    def fill(self, t, fn):
        """t.flat[i] = fn(i) for every i, 2^27 elements at a time."""
        flat = t.view(-1)
        for lo in range(0, flat.numel(), 1 << 27):
            hi = min(lo + (1 << 27), flat.numel())
            i = self.torch.arange(lo, hi, device="cuda", dtype=self.torch.int64)
            flat[lo:hi] = fn(i).to(t.dtype)


@pytest.fixture(scope="module")
def big():
    import torch
    from paper_1901_03771_amd import lazy as gr
    ctx = gr.Context()
    ctx.set_option("interp", 0)
    ora.set_threads(min(16, os.cpu_count() or 1))
    slab = Slab(torch)
    yield gr, ctx, torch, slab
    ctx.sync()
    ctx.close()
    del slab.mem
    torch.cuda.empty_cache()


def windows(n, rng, random_count, width=2048):
    """Sorted unique positions in [0, n): both ends, around 2^31 and 2^32, and random ones."""
    parts = [np.arange(0, min(n, 2 * width)), np.arange(max(0, n - 2 * width - 4099), n)]
    for edge in (1 << 31, 1 << 32):
        if edge < n:
            parts.append(np.arange(edge - width, min(n, edge + width)))
    parts.append(rng.integers(0, n, random_count))
    return np.unique(np.concatenate(parts).astype(np.int64))


def row_sample(rows, rng, count):
    """Row numbers: both ends, around the row whose first element is element 2^31, random ones."""
    mid = (1 << 31) // COLS
    parts = [np.arange(0, 8), np.arange(rows - 8, rows), np.arange(mid - 4, mid + 4), rng.integers(0, rows, count)]
    return np.unique(np.concatenate(parts).astype(np.int64))


def rows_of(fn, rows, cols, dtype=np.float32):
    """The rows `rows` of the (.., cols) matrix whose flat element i holds fn(lattice(i))."""
    i = rows[:, None] * cols + np.arange(cols, dtype=np.int64)[None, :]
    return np.ascontiguousarray(fn(lattice(i)).astype(dtype))


def check_elementwise(got, ref, what, floor=None):
    ok = elementwise_close(got, ref, ulps=2.0, rel=1e-6, floor=floor)
    bad = np.argwhere(~ok)
    assert ok.all(), f"{what}: {len(bad)} of {ok.size} outside tolerance, first at {bad[:3].tolist()}"


def check_reduction(got, ref, what, scale=None):
    ok, _ = reduction_check(np.asarray(got), np.asarray(ref), rel=1e-5, scale=scale)
    bad = np.argwhere(~ok)
    assert ok.all(), f"{what}: {len(bad)} of {ok.size} outside 1e-5, first at {bad[:3].tolist()}"


# ------------------------------------------------------------------ pointwise --
def test_chain_of_more_than_2_to_32_elements(big):
    gr, ctx, torch, slab = big
    a_t, b_t, out_t = (slab.array(k, (N,), torch.float32) for k in range(3))
    slab.fill(a_t, lambda i: as_unit(lattice(i)))
    slab.fill(b_t, lambda i: as_unit(lattice(i + 977)))
    out_t.fill_(float("nan"))
    wl.chain(gr, a=ctx.array(a_t), b=ctx.array(b_t)).materialize_into(out_t)
    ctx.sync()
    idx = windows(N, np.random.default_rng(1), 1 << 16)
    a = as_unit(lattice(idx)).astype(np.float32)
    b = as_unit(lattice(idx + 977)).astype(np.float32)
    it = torch.from_numpy(idx).cuda()
    assert np.array_equal(a_t[it].cpu().numpy(), a) and np.array_equal(b_t[it].cpu().numpy(), b), "device inputs are the lattice"
    ref = wl.chain(ora, a=ora.array(a), b=ora.array(b)).numpy()
    u = (((ora.array(a) + ora.array(b)) * (ora.array(a) - ora.array(b)) + 2.5 * ora.array(a)) / (abs(ora.array(b)) + 1.0)).numpy()
    v = ora.exp(-ora.array(a) * ora.array(a)).numpy()
    floor = 2.0 * np.maximum(np.spacing(np.abs(u)), np.spacing(np.abs(v))).astype(np.float64)
    check_elementwise(out_t[it].cpu().numpy(), ref, "chain", floor=floor)
    assert not bool(torch.isnan(out_t).any()), "every element was written"

    # views far into the line: a tail, a long stride, and an assignment to a tail
    tail = (ctx.array(a_t)[N - 5000:] * 2.0).numpy()
    assert np.array_equal(tail, (ora.array(as_unit(lattice(np.arange(N - 5000, N))).astype(np.float32)) * 2.0).numpy())
    far = np.arange(5, N, 1 << 20)
    strided = (ctx.array(a_t)[5::1 << 20] + 1.0).numpy()
    assert np.array_equal(strided, (ora.array(as_unit(lattice(far)).astype(np.float32)) + 1.0).numpy())
    dst = ctx.array(b_t)
    dst[N - 4099:] = ctx.array(a_t)[:4099] * 3.0
    ctx.sync()
    expect = (ora.array(as_unit(lattice(np.arange(4099))).astype(np.float32)) * 3.0).numpy()
    assert np.array_equal(b_t[N - 4099:].cpu().numpy(), expect)
    assert float(b_t[N - 4100]) == np.float32(as_unit(lattice(np.int64(N - 4100 + 977)))), "the element before the box is untouched"


def test_normalize_softmax_and_stencil_of_more_than_2_to_32_elements(big):
    gr, ctx, torch, slab = big
    X_t = slab.array(0, (ROWS, COLS), torch.float32)
    out_t = slab.array(1, (ROWS, COLS), torch.float32)
    slab.fill(X_t, lambda i: as_unit(lattice(i)))
    rng = np.random.default_rng(2)
    rows = row_sample(ROWS, rng, 48)
    rt = torch.from_numpy(rows).cuda()
    Xs = rows_of(as_unit, rows, COLS)
    assert np.array_equal(X_t[rt].cpu().numpy(), Xs)

    vec = wl.make_inputs("normalize", rows=4, cols=COLS)
    vec.pop("X")
    keep = {k: torch.from_numpy(v).cuda() for k, v in vec.items()}
    out_t.fill_(float("nan"))
    wl.normalize(gr, X=ctx.array(X_t), **{k: ctx.array(t) for k, t in keep.items()}).materialize_into(out_t)
    ctx.sync()
    ref = wl.normalize(ora, X=ora.array(Xs), **{k: ora.array(v) for k, v in vec.items()}).numpy()
    assert np.array_equal(out_t[rt].cpu().numpy(), ref), "normalize: correctly rounded operations only, identical bits expected"
    assert not bool(torch.isnan(out_t).any())

    out_t.fill_(float("nan"))
    wl.softmax(gr, X=ctx.array(X_t)).materialize_into(out_t)
    ctx.sync()
    check_reduction(out_t[rt].cpu().numpy(), wl.softmax(ora, X=ora.array(Xs)).numpy(), "softmax")
    sums = out_t.sum(dim=1, dtype=torch.float64)
    assert bool(((sums - 1).abs() < 1e-5).all()), "every row of the softmax sums to one"

    # the transposed matrix as an operand (its tiles go through LDS)
    outT_t = slab.array(1, (COLS, ROWS), torch.float32)
    outT_t.fill_(float("nan"))
    (ctx.array(X_t).T + 1.0).materialize_into(outT_t)
    ctx.sync()
    assert np.array_equal(outT_t[:, rt].cpu().numpy(), (ora.array(Xs).T + 1.0).numpy())
    assert not bool(torch.isnan(outT_t).any())

    # stencil: bands of 8 output rows (each needs 12 input rows)
    slab.fill(X_t, lambda i: as_positive(lattice(i)))
    st_t = slab.array(1, (ROWS - 4, COLS - 4), torch.float32)
    st_t.fill_(float("nan"))
    wl.stencil(gr, I=ctx.array(X_t)).materialize_into(st_t)
    ctx.sync()
    mid = (1 << 31) // COLS
    for r0 in [0, mid - 6, mid - 2, ROWS - 4 - 8] + [int(r) for r in rng.integers(0, ROWS - 12, 12)]:
        band = rows_of(as_positive, np.arange(r0, r0 + 12, dtype=np.int64), COLS)
        ref = wl.stencil(ora, I=ora.array(band)).numpy()
        check_elementwise(st_t[r0:r0 + 8].cpu().numpy(), ref, f"stencil rows {r0}..{r0 + 8}")
    assert not bool(torch.isnan(st_t).any())


# ------------------------------------------------------- reductions and scans --
def column_sample(count, rows, cols, rng):
    """(column numbers, the (rows, count) matrix of those columns of the lattice matrix)."""
    js = np.unique(np.concatenate([[0, 1, cols - 1], rng.integers(0, cols, count)]).astype(np.int64))
    i = np.arange(rows, dtype=np.int64)[:, None] * cols + js[None, :]
    return js, np.ascontiguousarray(as_unit(lattice(i)).astype(np.float32))


def test_reductions_over_more_than_2_to_32_elements(big):
    gr, ctx, torch, slab = big
    rng = np.random.default_rng(3)
    X_t = slab.array(0, (ROWS, COLS), torch.float32)
    slab.fill(X_t, lambda i: as_unit(lattice(i)))
    X = ctx.array(X_t)
    rows = row_sample(ROWS, rng, 256)
    Xs = rows_of(as_unit, rows, COLS)
    assert np.array_equal(X_t[torch.from_numpy(rows).cuda()].cpu().numpy(), Xs)
    absum = ora.sum(abs(ora.array(Xs)), axis=1).numpy()
    check_reduction(X.sum(axis=1).numpy()[rows], ora.sum(ora.array(Xs), axis=1).numpy(), "row sums", scale=absum)
    assert np.array_equal(X.max(axis=1).numpy()[rows], ora.max(ora.array(Xs), axis=1).numpy())

    # column sums (each over 2^21 + 3 rows): the oracle evaluates sampled columns
    js, cols = column_sample(29, ROWS, COLS, rng)
    got = X.sum(axis=0).numpy()
    check_reduction(got[js], ora.sum(ora.array(cols), axis=0).numpy(), "column sums", scale=ora.sum(abs(ora.array(cols)), axis=0).numpy())
    assert np.array_equal(X.min(axis=0).numpy()[js], ora.min(ora.array(cols), axis=0).numpy())

    # extrema of everything: planted beyond the range of the lattice, far into the array
    X_t[ROWS - 2, 1000] = 5.0
    X_t[(1 << 20) + 1, 7] = -7.0
    assert float(X.max().numpy()) == 5.0 and float(X.min().numpy()) == -7.0
    assert float(ctx.array(X_t.view(-1)[:1 << 32]).max().numpy()) < 1.0, "the planted maximum lies beyond element 2^32"

    # the sum of everything: x[i] = (i % 1024 + 1) / 1024, whose sum has a closed form (512.5 per period)
    x_t = slab.array(1, (N,), torch.float32)
    slab.fill(x_t, lambda i: (i % 1024 + 1) * (1.0 / 1024.0))

    def total(n):
        k = n % 1024
        return 512.5 * (n // 1024) + k * (k + 1) / 2048.0

    head = ((np.arange(1 << 20, dtype=np.int64) % 1024 + 1) * (1.0 / 1024.0)).astype(np.float32)
    assert float(ora.sum(ora.array(head)).numpy()) == np.float32(total(1 << 20)), "the closed form is the oracle's sum"
    check_reduction(ctx.array(x_t).sum().numpy(), np.float32(total(N)), "sum of everything")

    # int32 elements, summed in int64 (exact): x[i] = i % 1000 - 300, 199500 per period
    i_t = slab.array(1, (N,), torch.int32)
    slab.fill(i_t, lambda i: i % 1000 - 300)
    k = N % 1000
    want = 199500 * (N // 1000) + k * (k - 1) // 2 - 300 * k
    head = (np.arange(123457, dtype=np.int64) % 1000 - 300).astype(np.int32)
    assert int(ora.sum(ora.array(head)).numpy()) == 199500 * 123 + 457 * 456 // 2 - 300 * 457
    assert int(ctx.array(i_t).sum().numpy()) == want and want > 1 << 32


def test_scans_over_more_than_2_to_32_elements(big):
    gr, ctx, torch, slab = big
    # int32 along a line, accumulated in int64 (chunk sums, their scan, the chunks with their offsets):
    # x[i] = i % 7 + 1, so cumsum[i] = 28 * ((i + 1) // 7) + r (r + 1) / 2 with r = (i + 1) % 7
    x_t = slab.array(0, (N,), torch.int32)
    out_t = slab.array(1, (N,), torch.int64, slots=2)
    slab.fill(x_t, lambda i: i % 7 + 1)
    out_t.fill_(-1)
    ctx.array(x_t).cumsum(0).materialize_into(out_t)
    ctx.sync()

    def closed(i):
        r = (i + 1) % 7
        return 28 * ((i + 1) // 7) + r * (r + 1) // 2

    head = np.arange(1 << 20, dtype=np.int64)
    assert np.array_equal(closed(head), ora.cumsum(ora.array((head % 7 + 1).astype(np.int32)), 0).numpy()), "the closed form is the oracle's scan"
    idx = windows(N, np.random.default_rng(4), 1 << 16)
    assert np.array_equal(out_t[torch.from_numpy(idx).cuda()].cpu().numpy(), closed(idx))
    for lo in range(0, N, 1 << 27):      # and everywhere
        i = torch.arange(lo, min(lo + (1 << 27), N), device="cuda", dtype=torch.int64)
        assert torch.equal(out_t[lo:lo + (1 << 27)], closed(i)), f"cumsum, elements from {lo}"

    # float32 along a line in one pass (chained tiles that publish their totals): ones at every 512th
    # element, so that every partial sum is an integer below 2^24 and exact in any order of addition
    f_t = slab.array(0, (N,), torch.float32)
    o_t = slab.array(1, (N,), torch.float32)
    slab.fill(f_t, lambda i: (i % 512 == 0))
    o_t.fill_(-1.0)
    ctx.array(f_t).cumsum(0).materialize_into(o_t)
    ctx.sync()
    head = np.arange(1 << 20, dtype=np.int64)
    assert np.array_equal((head // 512 + 1).astype(np.float32), ora.cumsum(ora.array((head % 512 == 0).astype(np.float32)), 0).numpy())
    for lo in range(0, N, 1 << 27):
        i = torch.arange(lo, min(lo + (1 << 27), N), device="cuda", dtype=torch.int64)
        assert torch.equal(o_t[lo:lo + (1 << 27)], (i // 512 + 1).to(torch.float32)), f"one-pass cumsum, elements from {lo}"

    # down the columns of a matrix in one pass (register tiles of neighbouring lines):
    # x[r, c] = c % 3 in every fourth row, so cumsum[r, c] = (c % 3) (r // 4 + 1)
    X_t = slab.array(0, (ROWS, COLS), torch.float32)
    O_t = slab.array(1, (ROWS, COLS), torch.float32)
    slab.fill(X_t, lambda i: ((i // COLS) % 4 == 0) * ((i % COLS) % 3))
    O_t.fill_(-1.0)
    ctx.array(X_t).cumsum(0).materialize_into(O_t)
    ctx.sync()
    first = np.arange(1500 * COLS, dtype=np.int64)
    top = (((first // COLS) % 4 == 0) * ((first % COLS) % 3)).astype(np.float32).reshape(1500, COLS)
    assert np.array_equal(O_t[:1500].cpu().numpy(), ora.cumsum(ora.array(top), 0).numpy())
    c = torch.arange(COLS, device="cuda", dtype=torch.int64)[None, :]
    for lo in range(0, ROWS, 1 << 16):
        r = torch.arange(lo, min(lo + (1 << 16), ROWS), device="cuda", dtype=torch.int64)[:, None]
        assert torch.equal(O_t[lo:lo + (1 << 16)], ((c % 3) * (r // 4 + 1)).to(torch.float32)), f"column cumsum, rows from {lo}"

    # along the rows of a matrix (many short lines): x[r, c] = (r + c) % 5, sampled rows through the oracle
    slab.fill(X_t, lambda i: ((i // COLS) + (i % COLS)) % 5)
    O_t.fill_(-1.0)
    ctx.array(X_t).cumsum(1).materialize_into(O_t)
    ctx.sync()
    rows = row_sample(ROWS, np.random.default_rng(5), 64)
    i = rows[:, None] * COLS + np.arange(COLS, dtype=np.int64)[None, :]
    sample = (((i // COLS) + (i % COLS)) % 5).astype(np.float32)
    assert np.array_equal(O_t[torch.from_numpy(rows).cuda()].cpu().numpy(), ora.cumsum(ora.array(sample), 1).numpy())
    assert float(O_t.min()) >= 0.0, "every element was written"


# ------------------------------------------------------------------ contractions --
def test_contractions_over_more_than_2_to_32_elements(big):
    gr, ctx, torch, slab = big
    rng = np.random.default_rng(6)
    # a (2^23 + 1) x 512 matrix times a vector: sampled rows
    X_t = slab.array(0, (TALL, 512), torch.float32)
    slab.fill(X_t, lambda i: as_unit(lattice(i)))
    w = wl.make_inputs("logreg", rows=8, cols=512)["w"]
    w_t = torch.from_numpy(w).cuda()
    rows = np.unique(np.concatenate([np.arange(8), np.arange(TALL - 8, TALL), np.arange((1 << 22) - 4, (1 << 22) + 4), rng.integers(0, TALL, 2048)]))
    Xs = rows_of(as_unit, rows, 512)
    assert np.array_equal(X_t[torch.from_numpy(rows).cuda()].cpu().numpy(), Xs)
    z = (ctx.array(X_t) @ ctx.array(w_t)).numpy()
    check_reduction(z[rows], (ora.array(Xs) @ ora.array(w)).numpy(), "X.w", scale=(ora.array(np.abs(Xs)) @ ora.array(np.abs(w))).numpy())

    # its transpose times a vector: sampled outputs (columns of X)
    r = as_unit(lattice(np.arange(TALL, dtype=np.int64) + 555)).astype(np.float32)
    r_t = torch.from_numpy(r).cuda()
    js, cols = column_sample(21, TALL, 512, rng)
    g = (ctx.array(X_t).T @ ctx.array(r_t)).numpy()
    check_reduction(g[js], (ora.array(cols).T @ ora.array(r)).numpy(), "X^T.r", scale=(ora.array(np.abs(cols)).T @ ora.array(np.abs(r))).numpy())

    # the logistic-regression step (one pass: X.w, the residual, X^T.residual, the update) with a weight vector
    # that is zero outside four columns, so that the oracle needs only those columns for the residual of every
    # row and one more column per sampled output (adding exact zeros changes no sum)
    ks = np.array([0, 77, 300, 511])
    w4 = np.zeros(512, np.float32)
    w4[ks] = w[ks]
    y = (lattice(np.arange(TALL, dtype=np.int64) + 31) & 1).astype(np.float32)
    w4_t, y_t = torch.from_numpy(w4).cuda(), torch.from_numpy(y).cuda()
    got = wl.logreg(gr, X=ctx.array(X_t), w=ctx.array(w4_t), y=ctx.array(y_t)).numpy()
    i = np.arange(TALL, dtype=np.int64)[:, None] * 512 + ks[None, :]
    X4 = ora.array(np.ascontiguousarray(as_unit(lattice(i)).astype(np.float32)))
    res = 1.0 / (1.0 + ora.exp(-(X4 @ ora.array(w4[ks])))) - ora.array(y)
    grad = (ora.array(cols).T @ res) / TALL + 1e-4 * ora.array(w4[js])
    ref = (ora.array(w4[js]) - 0.1 * grad).numpy()
    scale = np.abs(w4[js]) + 0.1 * ((ora.array(np.abs(cols)).T @ abs(res)) / TALL).numpy()
    check_reduction(got[js], ref, "logistic-regression step", scale=scale)

    # matrix product on the matrix cores: (2^20 + 1) x 4096 times 4096 x 64, with an epilogue; sampled rows
    A_t = slab.array(0, (DEEP, 4096), torch.float32)
    slab.fill(A_t, lambda i: as_unit(lattice(i)))
    B = ((rng.random((4096, 64), dtype=np.float32) - np.float32(0.5)) * np.float32(0.05)).astype(np.float32)
    B_t = torch.from_numpy(B).cuda()
    C = gr.tanh(ctx.array(A_t) @ ctx.array(B_t)).numpy()
    rows = np.unique(np.concatenate([np.arange(8), np.arange(DEEP - 8, DEEP), np.arange((1 << 19) - 4, (1 << 19) + 4), rng.integers(0, DEEP, 512)]))
    As = rows_of(as_unit, rows, 4096)
    ref = ora.tanh(ora.array(As) @ ora.array(B)).numpy()
    check_reduction(C[rows], ref, "tanh(A.B)", scale=(ora.array(np.abs(As)) @ ora.array(np.abs(B))).numpy())
    assert np.isfinite(C).all()
