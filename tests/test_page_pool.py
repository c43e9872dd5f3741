"""KV page pool: the reference model (oracle/page_pool_ref.py) against hand-worked cases and
invariants, then the library's host code against the reference on random traces (exact)."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle.page_pool_ref import PagePoolRef, OK, INVALID, NO_PAGES
from paper_2602_09578_amd import binding as B

MAXP = 6   # pages per row in the traces (96 tokens)


# ---- the reference, pinned ------------------------------------------------------------------
def test_reference_by_hand():
    pool = PagePoolRef(5)
    rc, a = pool.alloc(2)
    assert (rc, a) == (OK, [0, 1])                       # pops 0, 1, 2, ...
    row_a = list(a)                                      # sample A holds 20 tokens: page 0 full, page 1 has 4
    rc, row_b = pool.fork(row_a, 20)                     # B shares both pages
    assert rc == OK and row_b == [0, 1] and pool.count[:2] == [2, 2]
    # A appends token 20 (slot 4 of a shared page): copy-on-write to the next free page, B keeps page 1
    assert pool.prepare_append(row_a, MAXP, 20) == (OK, 1, 2)
    assert row_a == [0, 2] and row_b == [0, 1] and pool.count[:3] == [2, 1, 1]
    # B appends token 20 too: it is now the sole holder of page 1, no copy
    assert pool.prepare_append(row_b, MAXP, 20) == (OK, -1, -1) and row_b == [0, 1]
    # A reaches a page boundary at 32: fresh page, no copy
    assert pool.prepare_append(row_a, MAXP, 32) == (OK, -1, -1) and row_a == [0, 2, 3]
    # B finishes: page 1 is free again (on top of the stack), page 0 stays with A
    assert pool.drop(row_b, 21) == OK and pool.count[:2] == [1, 0]
    assert pool.alloc(1) == (OK, [1]) and pool.alloc(1) == (OK, [4])
    assert pool.alloc(1) == (NO_PAGES, None)             # all five in use
    assert pool.prepare_append(row_a, MAXP, 48) == (NO_PAGES, -1, -1) and row_a == [0, 2, 3]
    assert pool.release([0, 0]) == INVALID and pool.count[0] == 1    # more releases than references
    assert pool.retain([7]) == INVALID and pool.release([-1]) == INVALID
    assert pool.prepare_append(row_a, MAXP, MAXP * 16) == (INVALID, -1, -1)


def run_trace(pool, ops, is_ref):
    """Applies a trace to a pool; rows are lists (reference) or numpy arrays (library).  Returns the log."""
    rows, lens, log = [], [], []
    for op, x, y in ops:
        if op == "new":                                   # a new sample with a prompt of y tokens in its own pages
            n = -(-y // 16)
            rc, pages = pool.alloc(n)
            log.append(("new", rc, None if pages is None else [int(p) for p in pages]))
            if rc == 0:
                row = [int(p) for p in pages] if is_ref else np.full(MAXP, -1, dtype=np.int32)
                if not is_ref:
                    row[:n] = pages
                rows.append(row)
                lens.append(y)
        elif not rows:
            continue
        elif op == "fork":
            k = x % len(rows)
            if is_ref:
                rc, child = pool.fork(rows[k], lens[k])
            else:
                child = np.full(MAXP, -1, dtype=np.int32)
                rc = pool.fork(rows[k], lens[k], child)
            log.append(("fork", rc))
            if rc == 0:
                rows.append(child)
                lens.append(lens[k])
        elif op == "append":
            k = x % len(rows)
            if lens[k] >= MAXP * 16:
                continue
            if is_ref:
                rc, s, d = pool.prepare_append(rows[k], MAXP, lens[k])
            else:
                rc, s, d = pool.prepare_append(rows[k], lens[k])
            log.append(("append", rc, s, d))
            if rc == 0:
                lens[k] += 1
        elif op == "drop":
            k = x % len(rows)
            log.append(("drop", pool.drop(rows[k], lens[k])))
            rows.pop(k)
            lens.pop(k)
        used = [[int(p) for p in r[: -(-l // 16)]] for r, l in zip(rows, lens)]
        log.append(("rows", used))
    return log, rows, lens


op_strategy = st.lists(st.tuples(st.sampled_from(["new", "fork", "fork", "append", "append", "append", "drop"]),
                                 st.integers(0, 1000), st.integers(1, 40)), min_size=1, max_size=120)


@given(op_strategy, st.integers(3, 24))
@settings(max_examples=150, deadline=None)
def test_reference_invariants(ops, num_pages):
    pool = PagePoolRef(num_pages)
    log, rows, lens = run_trace(pool, ops, True)
    refs = [0] * num_pages
    for r, l in zip(rows, lens):
        for p in r[: -(-l // 16)]:
            refs[p] += 1
    assert refs == pool.count                                     # counts = references held by the rows
    assert sorted(pool.free) == [p for p in range(num_pages) if refs[p] == 0]   # free = unreferenced, no duplicates
    for entry in log:                                             # a copy never targets a page somebody else holds
        if entry[0] == "append" and entry[1] == OK and entry[3] >= 0:
            assert entry[2] != entry[3]


# ---- the library against the reference ------------------------------------------------------
@given(op_strategy, st.integers(3, 24))
@settings(max_examples=150, deadline=None)
def test_library_matches_the_reference_on_random_traces(ops, num_pages):
    want, _, _ = run_trace(PagePoolRef(num_pages), ops, True)
    pool = B.PagePool(num_pages)
    got, rows, lens = run_trace(pool, ops, False)
    assert got == want
    ref_pool = PagePoolRef(num_pages)
    run_trace(ref_pool, ops, True)
    assert [pool.refcount(p) for p in range(num_pages)] == ref_pool.count
    assert pool.free_pages() == len(ref_pool.free)


def test_library_by_hand_and_argument_errors():
    pool = B.PagePool(5)
    rc, a = pool.alloc(2)
    assert rc == 0 and list(a) == [0, 1]
    row_a = np.array([0, 1, -1, -1, -1, -1], dtype=np.int32)
    row_b = np.full(MAXP, -1, dtype=np.int32)
    assert pool.fork(row_a, 20, row_b) == 0 and list(row_b[:2]) == [0, 1]
    assert pool.prepare_append(row_a, 20) == (0, 1, 2) and list(row_a[:2]) == [0, 2]
    assert pool.prepare_append(row_b, 20) == (0, -1, -1)
    assert pool.release(np.array([0, 0, 0])) == -1 and pool.refcount(0) == 2     # nothing changed
    assert pool.retain([9]) == -1 and pool.release([-1]) == -1 and pool.release([4]) == -1   # page 4 is free
    assert pool.prepare_append(row_a, MAXP * 16)[0] == -1
    assert pool.alloc(3)[0] == -3 and pool.free_pages() == 2                      # only two left: nothing taken
    lib = B.load_library()
    assert lib.marl_page_pool_create(0, None) == -1
    assert lib.marl_page_pool_alloc(None, 1, None) == -1
    assert lib.marl_page_pool_query(None, 0, None, None) == -1


def test_page_pool_host_code_runs_clean_under_asan_ubsan(tmp_path):
    """The pool is host C++: built alone with g++ and the sanitizers, a seeded trace (valid and
    invalid calls) runs clean and ends with the reference's counts."""
    import os, subprocess, sys, textwrap
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    lib = tmp_path / "libpool_san.so"
    subprocess.check_call(["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=undefined", "-fPIC", "-shared", "-x", "c++",
                           "-I" + os.path.join(root, "include"), "-o", str(lib),
                           os.path.join(root, "paper_2602_09578_amd", "csrc", "page_pool.hip")])
    script = textwrap.dedent(f"""
        import ctypes, sys
        import numpy as np
        sys.path.insert(0, {root!r})
        from oracle.page_pool_ref import PagePoolRef
        lib = ctypes.CDLL({str(lib)!r})
        I32, VP = ctypes.c_int32, ctypes.c_void_p
        P = ctypes.POINTER(I32)
        lib.marl_page_pool_create.argtypes = [I32, ctypes.POINTER(VP)]
        lib.marl_page_pool_destroy.argtypes = [VP]; lib.marl_page_pool_destroy.restype = None
        lib.marl_page_pool_alloc.argtypes = [VP, I32, P]
        lib.marl_page_pool_release.argtypes = [VP, P, I32]
        lib.marl_page_pool_retain.argtypes = [VP, P, I32]
        lib.marl_page_pool_fork.argtypes = [VP, P, I32, P]
        lib.marl_page_pool_prepare_append.argtypes = [VP, P, I32, I32, P, P]
        lib.marl_page_pool_drop.argtypes = [VP, P, I32]
        lib.marl_page_pool_query.argtypes = [VP, I32, P, P]
        N, MAXP = 37, 5
        h = VP(); assert lib.marl_page_pool_create(N, ctypes.byref(h)) == 0
        ref = PagePoolRef(N)
        rng = np.random.default_rng(5)
        rows, lens, rrows = [], [], []
        ptr = lambda a: a.ctypes.data_as(P)
        for it in range(3000):
            op = rng.integers(0, 6)
            if op == 0 or not rows:
                n = int(rng.integers(1, 4)); out = np.empty(4, dtype=np.int32)
                rc = lib.marl_page_pool_alloc(h, n, ptr(out)); rrc, pages = ref.alloc(n)
                assert rc == rrc
                if rc == 0:
                    assert list(out[:n]) == pages
                    row = np.full(MAXP, -1, dtype=np.int32); row[:n] = out[:n]
                    rows.append(row); rrows.append(list(pages)); lens.append(16 * (n - 1) + int(rng.integers(1, 17)))
            elif op == 1:
                k = int(rng.integers(len(rows))); child = np.full(MAXP, -1, dtype=np.int32)
                rc = lib.marl_page_pool_fork(h, ptr(rows[k]), lens[k], ptr(child)); rrc, rchild = ref.fork(rrows[k], lens[k])
                assert rc == rrc == 0 and [int(x) for x in child[:len(rchild)]] == rchild
                rows.append(child); rrows.append(rchild); lens.append(lens[k])
            elif op in (2, 3):
                k = int(rng.integers(len(rows)))
                if lens[k] < MAXP * 16:
                    s, d = I32(-1), I32(-1)
                    rc = lib.marl_page_pool_prepare_append(h, ptr(rows[k]), MAXP, lens[k], ctypes.byref(s), ctypes.byref(d))
                    assert (rc, s.value, d.value) == ref.prepare_append(rrows[k], MAXP, lens[k])
                    if rc == 0:
                        lens[k] += 1
            elif op == 4:
                k = int(rng.integers(len(rows)))
                assert lib.marl_page_pool_drop(h, ptr(rows[k]), lens[k]) == ref.drop(rrows[k], lens[k]) == 0
                rows.pop(k); rrows.pop(k); lens.pop(k)
            else:                                   # invalid calls must change nothing
                bad = np.array([int(rng.integers(0, N)), int(rng.choice([-1, N, N + 2])), int(rng.integers(0, N))], dtype=np.int32)
                assert lib.marl_page_pool_release(h, ptr(bad), 3) == ref.release([int(x) for x in bad]) == -1
                assert lib.marl_page_pool_retain(h, ptr(bad), 3) == ref.retain([int(x) for x in bad]) == -1
        for p in range(N):
            c = I32(0); assert lib.marl_page_pool_query(h, p, ctypes.byref(c), None) == 0
            assert c.value == ref.count[p], (p, c.value, ref.count[p])
        lib.marl_page_pool_destroy(h)
        print("clean")
    """)
    asan = subprocess.check_output(["g++", "-print-file-name=libasan.so"], text=True).strip()
    env = dict(os.environ, LD_PRELOAD=(os.environ.get("LD_PRELOAD", "") + " " + asan).strip(), ASAN_OPTIONS="detect_leaks=0")   # the interpreter itself leaks at exit
    r = subprocess.run([sys.executable, "-c", script], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0 and "clean" in r.stdout, r.stdout[-3000:]
