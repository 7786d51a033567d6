"""Host-side checks of libccdc.so that need no GPU: the library loads, exports
every declared entry point, its plan tables equal the oracle's (the two share
no code, only the numbering conventions), and its error paths answer with
status codes.  No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle as O
from paper_1805_01993_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_1805_01993_amd.build import build_library
        build_library()
    return B.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ccdc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ccdc_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert len(names) >= 12
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(B.EXPORTS) == names        # the binding covers the whole header


def test_header_is_plain_c_and_the_binding_uses_its_numbers(tmp_path):
    """include/ccdc.h compiles as C11 on its own, and every enumerator the binding
    hard-codes has the value the header gives it."""
    import subprocess
    text = open(os.path.join(ROOT, "include", "ccdc.h")).read()
    names = sorted(set(re.findall(r"\b(CCDC_[A-Z0-9_]+)\b", re.sub(r"/\*.*?\*/", "", text, flags=re.S))) - {"CCDC_H"})
    prog = '#include "ccdc.h"\n#include <stdio.h>\nint main(void) {\n' + "".join(
        f'    printf("{n} %d\\n", (int){n});\n' for n in names) + "    return 0;\n}\n"
    src, exe = tmp_path / "enums.c", tmp_path / "enums"
    src.write_text(prog)
    subprocess.run(["gcc", "-std=c11", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)],
                   check=True)
    got = dict(line.split() for line in subprocess.run([str(exe)], capture_output=True, text=True, check=True)
               .stdout.splitlines())
    got = {k: int(v) for k, v in got.items()}
    for name, value in got.items():
        short = name[len("CCDC_"):]
        assert hasattr(B, short), f"the binding has no constant for {name}"
        assert getattr(B, short) == value, name
    assert len(got) >= 45


def test_library_does_not_link_the_oracle():
    import subprocess
    needed = subprocess.run(["readelf", "-d", B.LIB_PATH], capture_output=True, text=True).stdout
    assert "oracle" not in needed
    syms = subprocess.run(["nm", "-D", B.LIB_PATH], capture_output=True, text=True).stdout
    assert "orc_" not in syms


SWEEP = [(K, r, c, m) for K in range(2, 8) for r in range(1, K) for c in (1, 2) for m in (1, 2)]


@pytest.mark.parametrize("jobs", [False, True])
def test_plan_tables_equal_the_oracles(lib, jobs):
    from math import comb
    n = 0
    for (K, r, c, m) in SWEEP:
        nb = (r + 1) if jobs else comb(K, r)
        while m * nb < K:
            m += 1
        Q, N = c * K, m * nb
        p = B.Plan(K, r, Q, N, jobs=jobs)
        o = O.build_plan(K, r, Q, N, "paper" if jobs else "single")
        assert (p.J, p.c, p.m, p.n_batch, p.n_round) == (o.J, o.c, o.m, o.n_batch, o.n_round)
        for name, tab in p.tables().items():
            assert np.array_equal(tab, getattr(o, name)), (K, r, c, m, name)
        for T in (1, 3, 4, 8, 10, 12, 40):
            p.bind(T, "u32")
            W = c * T
            assert p.W == W and p.T == T
            assert p.seg_len == O.segment_len(W, r)
            assert p.scheduled_elems == O.scheduled_elems(o, T)
            assert p.closed_form_elems == O.closed_form_elems(o, T)
            assert p.packet_len().tolist() == [O.packet_len(W, r, a) for a in range(r + 1)]
            sh, osh = p.shapes(), o.shapes(T)
            assert all(tuple(sh[k]) == tuple(osh[k]) for k in osh)
        p.close()
        n += 1
    assert n == len(SWEEP)


@pytest.mark.parametrize("jobs", [False, True])
def test_node_rows_list_what_each_node_sends(lib, jobs):
    """Every member of every round sends one packet (coded-packet equation of Sec. IV-B):
    node k's list is exactly the packets (round u, position a) with s_a = k, ascending."""
    from math import comb
    for (K, r, c, m) in SWEEP[::3]:
        nb = (r + 1) if jobs else comb(K, r)
        while m * nb < K:
            m += 1
        p = B.Plan(K, r, c * K, m * nb, jobs=jobs)
        o = O.build_plan(K, r, c * K, m * nb, "paper" if jobs else "single")
        rows = p.node_rows()
        member = o.round_member.reshape(-1)
        assert rows.shape == (K, member.size // K)
        for k in range(K):
            assert rows[k].tolist() == np.flatnonzero(member == k).tolist()
        p.close()
    cp = B.ccdc_plan_compression(4, 2, 4, 8)
    assert cp.query(B.Q_ROWS_PER_NODE) == 0
    cp.close()


@pytest.mark.parametrize("jobs", [False, True])
def test_file_placement_queries(lib, jobs):
    """FILE_NODES and NODE_FILES answer Sec. IV-A's placement directly: file -> the r nodes of
    its batch label, node k -> the set M_k.  Checked against the oracle's batch tables (built
    by different code) and against the properties the paper states: every file on exactly r
    nodes, |M_k| = mu*J*N for every k."""
    from math import comb
    for (K, r, c, m) in SWEEP[::2]:
        nb = (r + 1) if jobs else comb(K, r)
        while m * nb < K:
            m += 1
        N = m * nb
        p = B.Plan(K, r, c * K, N, jobs=jobs)
        o = O.build_plan(K, r, c * K, N, "paper" if jobs else "single")
        want = np.full((o.J * N, r), -1, dtype=np.int32)
        for bt in range(o.n_batch):
            first = o.batch_job[bt] * N + o.batch_file0[bt]
            want[first:first + o.m] = o.batch_label[bt]
        fn = p.file_nodes()
        assert np.array_equal(fn, want), (K, r, c, m)
        assert (np.diff(fn, axis=1) > 0).all() if r > 1 else True           # r distinct nodes, ascending
        nf = p.node_files()
        assert nf.shape == (K, r * o.J * N // K)                            # |M_k| = mu*J*N
        for k in range(K):
            assert nf[k].tolist() == np.flatnonzero((want == k).any(axis=1)).tolist()
        p.close()
    # the paper's K = 3 example: with the 1-based numbers of Sec. II every node stores 4 of the 6 files
    p = B.ccdc_plan(3, 2, 3, 6)
    assert p.node_files().shape == (3, 4)
    assert sorted(np.bincount(p.file_nodes().reshape(-1), minlength=3).tolist()) == [4, 4, 4]
    p.close()
    cp = B.ccdc_plan_compression(4, 2, 4, 8)
    out = np.zeros(64, dtype=np.int32)
    for what in (B.Q_FILE_NODES, B.Q_FILES_PER_NODE, B.Q_NODE_FILES):
        assert lib.ccdc_plan_query(cp._h, what, out.ctypes.data_as(C.c_void_p), out.nbytes) == B.ESTATE
    cp.close()


def test_repeated_jobs_plan_equals_the_oracles(lib):
    for (K, r, gamma) in [(4, 2, 2), (5, 2, 3), (4, 3, 4), (6, 1, 2)]:
        N = (r + 1) * max(1, -(-K // (r + 1)))
        p = B.ccdc_plan_jobs_repeated(K, r, 2 * K, N, gamma)
        o = O.build_plan(K, r, 2 * K, N, "paper", gamma=gamma)
        assert (p.J, p.n_batch, p.n_round) == (o.J, o.n_batch, o.n_round)
        for name, tab in p.tables().items():
            assert np.array_equal(tab, getattr(o, name)), (K, r, gamma, name)
        p.bind(12, "u32")
        assert p.scheduled_elems == O.scheduled_elems(o, 12)
        assert tuple(p.shapes()["V"]) == (o.J, N, 2 * K, 12)
        p.close()
    h = C.c_void_p()
    assert lib.ccdc_plan_jobs_repeated(4, 2, 4, 6, 0, C.byref(h)) == B.EINVAL and not h.value
    assert lib.ccdc_plan_jobs_repeated(4, 2, 4, 6, 2, None) == B.EINVAL
    assert lib.ccdc_plan_jobs_repeated(20, 9, 20, 20, 1 << 20, C.byref(h)) in (B.ESIZE, B.EINVAL)


@pytest.mark.parametrize("K,r,jobs", [(40, 3, False), (30, 2, True), (64, 2, False)])
def test_large_plans(lib, K, r, jobs):
    """Tables of plans with 10^4 to 10^5 rounds: equal to the oracle's, every (node, batch it
    does not store) served exactly once, every node in the same number of rounds."""
    from math import comb
    N = (r + 1) * 10 if jobs else comb(K, r)
    p = B.Plan(K, r, K, N, jobs=jobs)
    o = O.build_plan(K, r, K, N, "paper" if jobs else "single")
    t = p.tables()
    for name, tab in t.items():
        assert np.array_equal(tab, getattr(o, name)), name
    member, batch = t["round_member"].reshape(-1).astype(np.int64), t["round_batch"].reshape(-1).astype(np.int64)
    pairs = member * p.n_batch + batch
    assert np.unique(pairs).size == pairs.size                       # no batch twice to the same node
    stores = np.zeros((K, p.n_batch), dtype=bool)
    stores[t["batch_label"].reshape(-1), np.repeat(np.arange(p.n_batch), r)] = True
    assert not stores[member, batch].any()                           # never a batch the node already stores
    assert pairs.size == (~stores).sum()                             # and every missing one is served
    assert (np.bincount(member, minlength=K) == pairs.size // K).all()
    rows = p.node_rows()
    assert np.array_equal(np.sort(rows.reshape(-1)), np.arange(pairs.size))
    assert (member[rows] == np.arange(K)[:, None]).all()
    p.close()


def test_random_plans_equal_the_oracles(lib):
    """Seeded random parameters over K <= 12, every schedule: tables, segment split and
    scheduled traffic of the library equal the oracle's."""
    from math import comb
    rng = np.random.default_rng(7)
    for _ in range(80):
        K = int(rng.integers(2, 13))
        r = int(rng.integers(1, K))
        jobs = bool(rng.integers(0, 2)) and comb(K, r + 1) * (K - r) <= 4000
        gamma = int(rng.integers(1, 4)) if jobs else 1
        c = int(rng.integers(1, 4))
        nb = (r + 1) if jobs else comb(K, r)
        m = int(rng.integers(1, 4))
        while m * nb < K:
            m += 1
        T = int(rng.integers(1, 300))
        p = B.Plan(K, r, c * K, m * nb, jobs=jobs, gamma=gamma)
        o = O.build_plan(K, r, c * K, m * nb, "paper" if jobs else "single", gamma=gamma)
        for name, tab in p.tables().items():
            assert np.array_equal(tab, getattr(o, name)), (K, r, jobs, gamma, name)
        p.bind(T, "f32")
        assert p.seg_len == O.segment_len(c * T, r) and p.scheduled_elems == O.scheduled_elems(o, T)
        assert all(tuple(p.shapes()[k]) == tuple(v) for k, v in o.shapes(T).items())
        p.close()


def test_workload_plans(lib):
    from workloads import CONFIGS
    for w in CONFIGS.values():
        if w.compression:
            continue                      # covered by test_compression_plan_tables_equal_the_oracles
        p = B.Plan(w.K, w.r, w.Q, w.N, jobs=w.jobs).bind(w.T, w.modes[0])
        o = O.build_plan(w.K, w.r, w.Q, w.N, "paper" if w.jobs else "single")
        assert p.n_round == w.G and p.m == w.m and p.J == w.J
        assert np.array_equal(p.tables()["round_batch"], o.round_batch)
        assert p.scheduled_elems == O.scheduled_elems(o, w.T)
        assert p.query(B.Q_V_ELEMS) == w.v_elems


@pytest.mark.parametrize("args", [
    (1, 1, 1, 4), (4, 0, 4, 12), (4, 4, 4, 12), (4, 2, 6, 12), (4, 2, 4, 3), (4, 2, 4, 13), (4, 2, 0, 12),
])
def test_invalid_parameters(lib, args):
    h = C.c_void_p()
    assert lib.ccdc_plan(*args, C.byref(h)) == B.EINVAL
    assert not h.value
    assert lib.ccdc_plan(4, 2, 4, 12, None) == B.EINVAL


def test_too_many_subsets_is_a_size_error(lib):
    h = C.c_void_p()
    assert lib.ccdc_plan(64, 31, 64, 64, C.byref(h)) in (B.ESIZE, B.EINVAL)
    assert lib.ccdc_plan(40, 19, 40, 40, C.byref(h)) in (B.ESIZE, B.EINVAL)
    assert not h.value


def test_state_and_argument_errors(lib):
    p = B.ccdc_plan(4, 2, 4, 12)
    v = C.c_int64()
    assert lib.ccdc_plan_query(p._h, B.Q_K, C.byref(v), 8) == B.OK and v.value == 4
    assert lib.ccdc_plan_query(p._h, B.Q_W, C.byref(v), 8) == B.ESTATE          # not bound yet
    assert lib.ccdc_plan_query(p._h, 9999, C.byref(v), 8) == B.EINVAL
    assert lib.ccdc_plan_query(p._h, B.Q_K, C.byref(v), 4) == B.EINVAL          # buffer too small
    assert lib.ccdc_plan_query(p._h, B.Q_K, None, 8) == B.EINVAL
    assert lib.ccdc_plan_query(None, B.Q_K, C.byref(v), 8) == B.EINVAL
    small = (C.c_int32 * 2)()
    assert lib.ccdc_plan_query(p._h, B.Q_ROUND_MEMBER, small, 8) == B.EINVAL
    assert lib.ccdc_plan_upload(p._h) == B.ESTATE                                # not bound yet
    assert lib.ccdc_plan_bind(p._h, 0, B.F32_SUM) == B.EINVAL
    assert lib.ccdc_plan_bind(p._h, 16, 7) == B.EINVAL
    assert lib.ccdc_plan_bind(None, 16, 0) == B.EINVAL
    assert lib.ccdc_plan_bind(p._h, 1 << 41, B.F32_SUM) == B.ESIZE               # buffers past 2^40 elements
    assert lib.ccdc_plan_bind(p._h, 1 << 33, B.F32_SUM) == B.ESIZE               # launch past 2^31-1 items
    assert lib.ccdc_plan_bind(p._h, 16, B.F32_SUM) == B.OK
    # stage calls on a plan that was never uploaded: refused, nothing launched
    for fn, nptr in ((lib.ccdc_combine, 2), (lib.ccdc_encode, 2), (lib.ccdc_decode, 3), (lib.ccdc_reduce, 3),
                     (lib.ccdc_shuffle_fused, 3)):
        assert fn(p._h, *([C.c_void_p(256)] * nptr), None) == B.ESTATE
        assert fn(None, *([C.c_void_p(256)] * nptr), None) == B.EINVAL
    lib.ccdc_plan_destroy(None)                                                  # allowed
    assert B.strerror(B.ESIZE) and B.strerror(-99) == "unknown status"


def test_payload_modes(lib):
    p = B.ccdc_plan(4, 2, 4, 12)
    for name, code in B.MODES.items():
        p.bind(24, name)
        assert p.query(B.Q_MODE) == code and p.W == 24 and p.seg_len == 12
        assert p._elem_bytes == (2 if name in ("bf16", "f16") else 4)
    assert lib.ccdc_plan_bind(p._h, 24, 5) == B.EINVAL and lib.ccdc_plan_bind(p._h, 24, -1) == B.EINVAL
    p.close()
    cp = B.ccdc_plan_compression(4, 2, 4, 8)
    for name, code in B.MODES.items():            # the uncoded scheme has no hybrid of sums and XOR-coded packets
        want = B.OK if name in ("f32", "u32") else B.EINVAL
        assert lib.ccdc_plan_bind(cp._h, 24, code) == want
    cp.close()


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "libccdc.so"))
    with pytest.raises(FileNotFoundError):
        B.ccdc_plan(4, 2, 4, 12)


def test_product_path_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_1805_01993_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower().replace("no cpu fallback", ""), f


def test_compression_plan_tables_equal_the_oracles(lib):
    n = 0
    for K in range(2, 10):
        for r in range(1, K):
            for c in (1, 2):
                N = 2 * K * r
                p = B.ccdc_plan_compression(K, r, c * K, N)
                o = O.CompressionPlan(K, r, c * K, N)
                assert p.query(B.Q_SCHEME) == 2 and p.n_batch == o.nb and p.query(B.Q_NROWS) == o.n_packet
                for name, tab in p.compression_tables().items():
                    assert np.array_equal(tab, getattr(o, name)), (K, r, name)
                for T in (1, 6, 8):
                    p.bind(T, "u32")
                    assert p.W == c * T and p.seg_len == c * T
                    assert p.scheduled_elems == o.scheduled_elems(T) == p.closed_form_elems
                    assert p.packet_len().tolist() == [c * T]
                    assert p.shapes()["Vbar"] == (o.n_packet, c * T) and p.query(B.Q_X_ELEMS) == 0
                p.close()
                n += 1
    assert n == 72
    h = C.c_void_p()
    assert lib.ccdc_plan_compression(5, 2, 5, 6, C.byref(h)) == B.EINVAL      # mu*N not whole
    assert lib.ccdc_plan_compression(4, 3, 4, 5, C.byref(h)) == B.EINVAL      # mu > 1/2 needs even N
    assert lib.ccdc_plan_compression(4, 2, 4, 8, None) == B.EINVAL


def test_load_comparison_reproduces_the_papers_remark(lib, golden):
    """Remark after the K = 4 example: 3/4 (compressed CDC), 1 (combining only), 3/2 (CDC only)."""
    from fractions import Fraction

    from paper_1805_01993_amd.loads import comparison
    g = golden("example_k4.txt")
    rows = comparison(int(g["K"]), int(g["r"]), int(g["Q"]), int(g["N"]))
    assert rows["compressed CDC (Theorem 1, J jobs)"] == Fraction(g["load_total"])
    assert rows["compression only (appendix)"] == Fraction(g["load_compression_only"])
    assert rows["CDC only (formula of Sec. III)"] == Fraction(g["load_cdc_only"])
    # a shape whose N fits only some schemes still answers for the others
    rows = comparison(8, 2, 8, 28)
    assert rows["compressed CDC (Theorem 1, J jobs)"] is None
    assert rows["compressed CDC, single-job schedule"] == Fraction(21, 2)
    assert rows["compression only (appendix)"] == 3
