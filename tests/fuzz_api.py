"""Random calls into the C ABI with arguments that are often invalid: stale and foreign handles, ranks of 100,
extents of 2^40, empty axes, misaligned pointers, enumeration values that do not exist.  Every call has to come
back with a status; on a device-less context in dry-run mode nothing touches a GPU, so the host logic can run
under AddressSanitizer / UndefinedBehaviorSanitizer (tests/test_sanitized_host.py)."""
import ctypes
import random


def run(gr, seed: int, calls: int) -> dict:
    L = gr.lib()
    ctx = gr.Context(device=-1)
    ctx.set_option("dry_run", 2)
    P = ctx._p
    r = random.Random(seed)
    handles = [0, 1, 2, 999999, 2 ** 63]
    programs = []
    I64, VP = ctypes.c_int64, ctypes.c_void_p
    out = ctypes.c_uint64()

    def h():
        return ctypes.c_uint64(r.choice(handles))

    def shape_arr(n):
        return (I64 * max(n, 1))(*[r.choice([-5, -1, 0, 1, 2, 3, 7, 64, 2 ** 40]) for _ in range(max(n, 1))])

    ok = 0
    for _ in range(calls):
        k = r.randrange(21)
        st = None
        if k == 0:
            nd = r.choice([-1, 0, 1, 2, 3, 8, 9, 100])
            m = min(max(nd, 0), 12)
            st = L.gr_array_from_device(P, VP(r.choice([0, 0x1000, 0x1003])), r.choice([0, 1, 2, 3, -1]), nd,
                                        shape_arr(m) if r.random() < 0.9 else None, shape_arr(m) if r.random() < 0.3 else None, ctypes.byref(out))
        elif k == 1:
            st = L.gr_unary(P, r.choice([0, 1, 2, 3, 4, 5, 6, 7, 8, 16, -1, 99]), h(), ctypes.byref(out))
        elif k == 2:
            st = L.gr_binary(P, r.choice([16, 17, 18, 19, 20, 21, 0, 22, 23, -3]), h(), h(), ctypes.byref(out))
        elif k == 3:
            st = L.gr_binary_scalar(P, r.choice([16, 17, 18, 19, 20, 21, 22, 5, 1000]), h(), r.choice([0.0, 1.5, -2.0, 2.0, float("nan"), 1e40, 3.0]),
                                    r.choice([0, 1]), r.choice([0, 1]), ctypes.byref(out))
        elif k == 4:
            n = r.choice([0, 1, 2, 3, 9, -1])
            m = max(n, 1)
            U8 = ctypes.c_uint8 * m
            st = L.gr_slice(P, h(), n, shape_arr(m), shape_arr(m), (I64 * m)(*[r.choice([1, 2, 3, 0, -1]) for _ in range(m)]),
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
            st = L.gr_reshape(P, h(), nd, shape_arr(max(nd, 1)), ctypes.byref(out))
        elif k == 10:
            st = L.gr_materialize(P, h())
        elif k == 11:
            st = L.gr_assign(P, h(), h())
        elif k == 12:
            st = L.gr_release(P, h()) if r.random() < 0.2 else 0
        elif k == 13:
            st = L.gr_retain(P, h()) if r.random() < 0.05 else 0
        elif k == 14:
            need = ctypes.c_size_t()
            st = L.gr_plan_describe(P, h(), None, 0, ctypes.byref(need))
        elif k == 15:
            st = L.gr_materialize_into(P, h(), VP(r.choice([0, 0x2000, 0x2002])), r.choice([0, 4, 16, 4096]))
        elif k == 16:
            st = L.gr_materialize_into_static(P, h(), VP(r.choice([0, 0x2000, 0x2002])), r.choice([0, 4, 16, 4096]))
        elif k == 17:
            st = L.gr_array_lend_buffer(P, h(), VP(r.choice([0, 0x1000, 0x3000, 0x3002])), r.choice([0, 4, 16, 28, 4096]))
        elif k == 18:
            n = r.choice([0, 1, 2, 3, -1])
            arr = (ctypes.c_uint64 * max(n, 1))(*[r.choice(handles) for _ in range(max(n, 1))])
            pp = VP()
            st = L.gr_program_create(P, h(), arr if r.random() < 0.9 else None, n, ctypes.byref(pp))
            if st == 0:
                programs.append((pp.value, max(n, 0)))
        elif k == 19 and programs:
            pv, n = r.choice(programs)
            ptrs = (VP * max(n, 1))(*[r.choice([0, 0x1000, 0x5000]) for _ in range(max(n, 1))])
            st = L.gr_program_run(VP(pv), ptrs if r.random() < 0.9 else None, VP(r.choice([0, 0x1000, 0x9000])))
        elif k == 20 and programs and r.random() < 0.3:
            pv, n = programs.pop(r.randrange(len(programs)))
            st = L.gr_program_destroy(VP(pv))
        if st == 0 and k in (0, 1, 2, 3, 4, 5, 6, 7, 8, 9):
            ok += 1
            handles.append(out.value)
            if len(handles) > 60:
                handles.pop(r.randrange(5, len(handles)))
    stats = dict(recorded=ok, nodes_alive=ctx.stats()["nodes_alive"], programs_left=len(programs))
    ctx.close()
    return stats
