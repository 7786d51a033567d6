"""Parity of the HIP path with the CPU oracle, element by element, through the
C entry points.  Same seeded inputs on both sides; uint32/XOR must be bit-exact,
fp32 must be within 1e-5 (max abs error over max abs reference, per artefact)
of the fp64 oracle.  Needs a GPU."""
import numpy as np
import pytest

import oracle as O
from workloads import CONFIGS, generate_numpy, generate_torch

pytestmark = pytest.mark.gpu

F32_TOL = 1e-5


@pytest.fixture(scope="module")
def torch():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the parity tests cannot run")
    torch.cuda.set_device(0)
    return torch


@pytest.fixture(scope="module")
def L(torch):
    import paper_1805_01993_amd as lib
    lib.load_library()          # fails loudly when the extension is not built
    return lib


def to_dev(torch, a):
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_host(t, mode):
    a = t.cpu().numpy()
    return a.view(np.uint32) if mode == "u32" else a


def dev_empty(torch, shape, mode, fill=None):
    dt = torch.int32 if mode == "u32" else torch.float32
    t = torch.empty(shape, dtype=dt, device="cuda")
    if fill is not None:
        t.fill_(fill)
    return t


def oracle_run(op, T, Vh, mode):
    return O.run_all_h32(op, T, Vh) if mode == "h32" else O.run_all(op, T, Vh)


def assert_close(got, want, mode, name):
    """u32: every word equal.  h32: packets (Vbar, X, D) equal bit for bit, the
    reduced outputs within tolerance.  f32: everything within tolerance."""
    assert got.shape == want.shape, name
    if mode == "u32" or (mode == "h32" and "Phi" not in name):
        g = np.ascontiguousarray(got).view(np.uint32).ravel()
        w = np.ascontiguousarray(want).view(np.uint32).ravel()
        bad = np.flatnonzero(g != w)
        assert bad.size == 0, f"{name}: {bad.size} words differ, first at {bad[:4]}"
    else:
        scale = float(np.abs(want).max())
        err = float(np.abs(got.astype(np.float64) - want).max())
        assert err <= F32_TOL * max(scale, 1e-300), f"{name}: err {err:.3e} scale {scale:.3e}"


def run_case(torch, L, K, r, Q, N, T, mode, jobs=False, seed=1, sigma=1.0, gamma=1):
    op = O.build_plan(K, r, Q, N, "paper" if jobs else "single", gamma=gamma)
    Vh = generate_numpy(op.J, N, Q, T, seed, "u32" if mode == "u32" else "f32", sigma)
    ref = oracle_run(op, T, Vh, mode)
    ref_phi = O.direct(op, T, Vh)

    plan = L.Plan(K, r, Q, N, jobs=jobs, gamma=gamma).bind(T, mode).upload()
    sh = plan.shapes()
    V = to_dev(torch, Vh)
    poison = -1 if mode == "u32" else float("nan")
    Vbar = dev_empty(torch, sh["Vbar"], mode, poison)
    X = dev_empty(torch, sh["X"], mode, poison)
    D = dev_empty(torch, sh["D"], mode, poison)
    Phi = dev_empty(torch, sh["Phi"], mode, poison)
    plan.combine(V, Vbar)
    plan.encode(Vbar, X)
    plan.decode(X, Vbar, D)
    plan.reduce(V, D, Phi)
    torch.cuda.synchronize()
    got = {"Vbar": to_host(Vbar, mode), "X": to_host(X, mode), "D": to_host(D, mode), "Phi": to_host(Phi, mode)}
    for name in ("Vbar", "X", "D", "Phi"):
        assert_close(got[name], ref[name], mode, name)
    assert_close(got["Phi"], ref_phi, mode, "Phi vs eq.(1)")

    # fused combine+encode+decode: same artefacts, never materialising Vbar
    X2 = dev_empty(torch, sh["X"], mode, poison)
    D2 = dev_empty(torch, sh["D"], mode, poison)
    plan.shuffle_fused(V, X2, D2)
    torch.cuda.synchronize()
    assert_close(to_host(X2, mode), ref["X"], mode, "fused X")
    assert_close(to_host(D2, mode), ref["D"], mode, "fused D")
    # same operation order as the separate stages: identical bits in every mode, except
    # that ccdc_combine adds short packets of long batches in a cross-lane tree (fp32 only)
    W = (Q // K) * T
    tree_combine = mode == "f32" and op.m >= 8 and W // (4 if T % 4 == 0 else 1) <= 16
    if not tree_combine:
        assert torch.equal(X2.view(torch.int32), X.view(torch.int32))
        assert torch.equal(D2.view(torch.int32), D.view(torch.int32))
    Phi2 = dev_empty(torch, sh["Phi"], mode, poison)
    plan.reduce(V, D2, Phi2)
    torch.cuda.synchronize()
    if not tree_combine:
        assert torch.equal(Phi2.view(torch.int32), Phi.view(torch.int32))
    assert_close(to_host(Phi2, mode), ref_phi, mode, "Phi from fused D vs eq.(1)")

    # the whole path in one pass (single-job plans, r <= 5, K*r <= 256)
    X3 = dev_empty(torch, sh["X"], mode, poison)
    Phi3 = dev_empty(torch, sh["Phi"], mode, poison)
    if not jobs and r <= 5 and K * r <= 256:
        plan.pipeline_fused(V, X3, Phi3)
        torch.cuda.synchronize()
        assert torch.equal(X3.view(torch.int32), X2.view(torch.int32))
        assert_close(to_host(X3, mode), ref["X"], mode, "pipeline X")
        assert_close(to_host(Phi3, mode), ref["Phi"], mode, "pipeline Phi")
        assert_close(to_host(Phi3, mode), ref_phi, mode, "pipeline Phi vs eq.(1)")
    else:
        with pytest.raises(L.CcdcError) as err:
            plan.pipeline_fused(V, X3, Phi3)
        assert err.value.status == L.binding.ESIZE
    plan.close()
    return got


# ---------------------------------------------------------------- workloads

@pytest.mark.parametrize("name,mode", [("cfg1_tiny", "f32"), ("cfg1_tiny", "u32"), ("cfg1_tiny", "h32"),
                                       ("cfg2_k10", "f32"), ("cfg2_k10", "u32"), ("cfg2_k10", "h32"),
                                       ("cfg4_k16", "f32")])
@pytest.mark.parametrize("seed", [1, 2])
def test_small_workloads_full_compare(torch, L, name, mode, seed):
    w = CONFIGS[name]
    run_case(torch, L, w.K, w.r, w.Q, w.N, w.T, mode, seed=seed, sigma=w.sigma)


# ------------------------------------------------------ shapes and edge cases

EDGE = [
    # K, r, Q, N, T, jobs      what it exercises
    (3, 2, 3, 6, 1024, False),    # K = r+1: one round, the paper's own motivating example shape
    (6, 1, 6, 12, 520, False),    # r = 1: uncoded unicast packets
    (5, 4, 5, 10, 64, False),     # r = K-1 with 4r | W
    (5, 3, 10, 20, 1000, False),  # c = 2, m = 2, r does not divide W (aligned split, short tail)
    (4, 2, 4, 12, 7, False),      # T not a multiple of 4: scalar path, ragged tail
    (4, 3, 4, 4, 10, False),      # tiny W: ell = 4, segments 4,4,2
    (4, 3, 4, 4, 1, False),       # W = 1: all but the first segment empty
    (6, 3, 12, 40, 333, False),   # scalar path over several tiles, c = 2, m = 2
    (7, 5, 7, 21, 2052, False),   # r = 5
    (10, 8, 10, 45, 36, False),   # r = 8: largest unrolled fused kernel
    (11, 9, 11, 55, 40, False),   # r = 9: any-r fused fallback
    (4, 2, 4, 6, 512, True),      # paper's 4-job running example shape
    (5, 2, 10, 6, 258, True),     # J = 10 jobs, c = 2, scalar path
    (6, 3, 6, 8, 1200, True),     # J = 15 jobs, m = 2
    (4, 2, 4, 240, 12, False),    # short packets, m = 40: wavefront-wide combiner, 3 packs in segments of 4
    (4, 2, 8, 96, 5, False),      # same with c = 2, scalar packs: 10 packs in segments of 16, m = 16
    (4, 2, 4, 48, 8, True),       # same under the J-job schedule: 2 packs, m = 16
    (5, 1, 5, 45, 64, False),     # m = 9 with exactly 16 packs
]


@pytest.mark.parametrize("K,r,Q,N,T,jobs", EDGE)
@pytest.mark.parametrize("mode", ["u32", "f32", "h32"])
def test_edge_shapes(torch, L, K, r, Q, N, T, jobs, mode):
    run_case(torch, L, K, r, Q, N, T, mode, jobs=jobs, seed=K * 10 + r)


@pytest.mark.parametrize("K,r,N,T", [(40, 3, 9880, 64),      # 91 390 rounds, K*r = 120: one-element packs in the one-pass kernel
                                     (64, 2, 2016, 128),     # 64 nodes, K*r = 128
                                     (24, 5, 42504, 24)])    # r = 5 at 24 nodes: 134 596 rounds of 6 members
@pytest.mark.parametrize("mode", ["u32", "f32"])
def test_many_nodes(torch, L, K, r, N, T, mode):
    run_case(torch, L, K, r, K, N, T, mode, seed=K)


def random_shape(rng):
    """A valid (K, r, Q, N, T, jobs) drawn over the whole parameter space at small sizes."""
    from math import comb
    K = int(rng.integers(2, 10))
    r = int(rng.integers(1, K))
    jobs = bool(K <= 6 and rng.integers(0, 3) == 0)
    c = int(rng.integers(1, 4))
    nb = (r + 1) if jobs else comb(K, r)
    m = int(rng.integers(1, 4))
    while m * nb < K:
        m += 1
    T = int(rng.choice([1, 2, 3, 4, 5, 8, 12, 16, 24, 31, 64, 100, 128, 250, 256, 511, 520]))
    return K, r, c * K, m * nb, T, jobs


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes(torch, L, seed):
    rng = np.random.default_rng(1000 + seed)
    K, r, Q, N, T, jobs = random_shape(rng)
    mode = ["u32", "f32", "h32"][seed % 3]
    run_case(torch, L, K, r, Q, N, T, mode, jobs=jobs, seed=seed)


@pytest.mark.parametrize("K,r,Q,N,T,gamma", [(4, 2, 4, 6, 512, 2), (5, 2, 10, 6, 258, 3), (4, 3, 4, 8, 40, 5)])
@pytest.mark.parametrize("mode", ["u32", "f32", "h32"])
def test_repeated_jobs_schedule(torch, L, K, r, Q, N, T, gamma, mode):
    """J = gamma*C(K, r+1) jobs: the J-job scheme repeated on consecutive blocks of jobs (Sec. IV)."""
    run_case(torch, L, K, r, Q, N, T, mode, jobs=True, seed=gamma, gamma=gamma)


@pytest.mark.parametrize("K,r,Q,N,T,jobs", [(5, 3, 10, 20, 1000, False),     # c = 2, m = 2, short last segment
                                            (8, 2, 8, 28, 4096, False),      # the gradient shape's plan
                                            (4, 2, 4, 12, 7, False),         # one-element packs
                                            (4, 2, 4, 6, 512, True)])        # the paper's four-job schedule
@pytest.mark.parametrize("mode", ["f32", "u32"])
def test_decode_never_reads_the_packet_it_recovers(torch, L, K, r, Q, N, T, jobs, mode):
    """Decoding paragraph of Sec. IV-B: receiver b gets its packet as the coded packets minus
    side information it computes itself; the packet Vbar[u][b] is exactly what it does NOT
    have.  So with row b of Vbar overwritten by junk (NaN in fp32, all-ones words in XOR mode),
    in every round, ccdc_decode must still give the same D[:, b, :], bit for bit - a decode
    that copied the packet, or touched it at all, would not."""
    plan = L.Plan(K, r, Q, N, jobs=jobs).bind(T, mode).upload()
    sh = plan.shapes()
    Vh = generate_numpy(plan.J, N, Q, T, 5, mode)
    V = to_dev(torch, Vh)
    poison = -1 if mode == "u32" else float("nan")
    Vbar, X, D0 = (dev_empty(torch, sh[k], mode, poison) for k in ("Vbar", "X", "D"))
    plan.combine(V, Vbar)
    plan.encode(Vbar, X)
    plan.decode(X, Vbar, D0)
    torch.cuda.synchronize()
    assert not torch.isnan(D0).any() if mode == "f32" else True
    for b in range(r + 1):
        junk = Vbar.clone()
        junk[:, b, :] = poison
        Db = dev_empty(torch, sh["D"], mode, poison)
        plan.decode(X, junk, Db)
        torch.cuda.synchronize()
        assert torch.equal(Db[:, b, :].view(torch.int32), D0[:, b, :].view(torch.int32)), f"receiver position {b}"
        if r >= 2:                  # the junk is side information of the OTHER receivers: they must see it
            others = [b2 for b2 in range(r + 1) if b2 != b]
            assert not torch.equal(Db[:, others, :].view(torch.int32), D0[:, others, :].view(torch.int32))
    plan.close()


def test_unaligned_pointers_take_the_scalar_path(torch, L):
    """Buffers that are only 4-byte aligned still work; others are refused."""
    K, r, Q, N, T, mode = 5, 2, 5, 10, 64, "u32"
    op = O.build_plan(K, r, Q, N)
    Vh = generate_numpy(1, N, Q, T, 3, mode)
    ref = O.run_all(op, T, Vh)
    plan = L.ccdc_plan(K, r, Q, N).bind(T, mode).upload()
    sh = plan.shapes()

    def shifted(shape):
        n = int(np.prod(shape))
        return torch.zeros(n + 1, dtype=torch.int32, device="cuda")[1:]

    V = shifted(sh["V"])
    V.copy_(to_dev(torch, Vh).reshape(-1))
    X, D, Phi = shifted(sh["X"]), shifted(sh["D"]), shifted(sh["Phi"])
    assert V.data_ptr() % 16 == 4
    plan.shuffle_fused(V, X, D)
    plan.reduce(V, D, Phi)
    torch.cuda.synchronize()
    assert_close(to_host(X, mode).reshape(sh["X"]), ref["X"], mode, "X")
    assert_close(to_host(D, mode).reshape(sh["D"]), ref["D"], mode, "D")
    assert_close(to_host(Phi, mode).reshape(sh["Phi"]), ref["Phi"], mode, "Phi")
    import ctypes as C
    lib = L.load_library()
    assert lib.ccdc_encode(plan._h, C.c_void_p(D.data_ptr() + 1), C.c_void_p(X.data_ptr()), None) == L.binding.EINVAL
    assert lib.ccdc_encode(plan._h, None, C.c_void_p(X.data_ptr()), None) == L.binding.EINVAL
    plan.close()


def test_results_are_deterministic_and_on_the_given_stream(torch, L):
    w = CONFIGS["cfg2_k10"]
    plan = L.ccdc_plan(w.K, w.r, w.Q, w.N).bind(w.T, "f32").upload()
    sh = plan.shapes()
    V = generate_torch(1, w.N, w.Q, w.T, 5, "f32", device="cuda")
    outs = []
    side = torch.cuda.Stream()
    for stream in (None, side, None):
        X = dev_empty(torch, sh["X"], "f32", float("nan"))
        D = dev_empty(torch, sh["D"], "f32", float("nan"))
        Phi = dev_empty(torch, sh["Phi"], "f32", float("nan"))
        if stream is not None:
            stream.wait_stream(torch.cuda.current_stream())
        plan.shuffle_fused(V, X, D, stream=stream)
        plan.reduce(V, D, Phi, stream=stream)
        if stream is not None:
            stream.synchronize()
        torch.cuda.synchronize()
        outs.append((X, D, Phi))
    for X, D, Phi in outs[1:]:
        assert torch.equal(X, outs[0][0]) and torch.equal(D, outs[0][1]) and torch.equal(Phi, outs[0][2])
    plan.close()


def test_one_plan_on_two_streams_is_put_in_order(torch, L):
    """Two calls that both keep partial sums in the plan's workspace, issued back to back
    on different streams with different inputs: the library orders them, so each gives
    exactly what it gives alone."""
    K, r, Q, N, T = 10, 3, 10, 120, 32768
    plan = L.ccdc_plan(K, r, Q, N).bind(T, "f32").upload()
    assert plan.workspace_bytes > 0
    sh = plan.shapes()
    Va = generate_torch(1, N, Q, T, 11, "f32", device="cuda")
    Vb = generate_torch(1, N, Q, T, 12, "f32", device="cuda")
    alone = []
    for V in (Va, Vb):
        X, Phi = dev_empty(torch, sh["X"], "f32", float("nan")), dev_empty(torch, sh["Phi"], "f32", float("nan"))
        plan.pipeline_fused(V, X, Phi)
        torch.cuda.synchronize()
        alone.append((X, Phi))
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    for rep in range(3):
        outs = [(dev_empty(torch, sh["X"], "f32", float("nan")), dev_empty(torch, sh["Phi"], "f32", float("nan")))
                for _ in range(4)]
        torch.cuda.synchronize()
        for i, (X, Phi) in enumerate(outs):          # a, b, a, b with no host wait in between
            plan.pipeline_fused((Va, Vb)[i % 2], X, Phi, stream=(sa, sb)[i % 2])
        torch.cuda.synchronize()
        for i, (X, Phi) in enumerate(outs):
            assert torch.equal(X, alone[i % 2][0]), (rep, i)
            assert torch.equal(Phi, alone[i % 2][1]), (rep, i)
    # the separate reduction and the node-local reduction use the same workspace
    D = dev_empty(torch, sh["D"], "f32", float("nan"))
    X = dev_empty(torch, sh["X"], "f32", float("nan"))
    plan.shuffle_fused(Va, X, D)
    P0, P1, P2 = (dev_empty(torch, sh["Phi"], "f32", float("nan")) for _ in range(3))
    plan.reduce(Va, D, P0)
    torch.cuda.synchronize()
    plan.reduce(Va, D, P1, stream=sa)
    plan.node_decode_reduce(-1, Va, X, P2, stream=sb)
    plan.reduce(Va, D, P1, stream=sa)
    torch.cuda.synchronize()
    assert torch.equal(P0, P1)
    assert_close(to_host(P2, "f32"), to_host(P0, "f32").astype(np.float64), "f32", "node-local Phi")
    plan.close()


def test_rebinding_a_plan(torch, L):
    plan = L.ccdc_plan(4, 2, 4, 12)
    for T, mode in ((256, "f32"), (100, "u32"), (256, "u32")):
        plan.bind(T, mode)
        with pytest.raises(L.CcdcError):          # binding drops the device tables
            plan.combine(torch.zeros(12 * 4 * T, dtype=torch.int32, device="cuda"),
                         torch.zeros(plan.query(L.binding.Q_VBAR_ELEMS), dtype=torch.int32, device="cuda"))
        plan.upload()
        op = O.build_plan(4, 2, 4, 12)
        Vh = generate_numpy(1, 12, 4, T, 9, mode)
        V = to_dev(torch, Vh)
        sh = plan.shapes()
        X, D, Phi = (dev_empty(torch, sh[k], mode) for k in ("X", "D", "Phi"))
        plan.shuffle_fused(V, X, D)
        plan.reduce(V, D, Phi)
        torch.cuda.synchronize()
        assert_close(to_host(Phi, mode), O.direct(op, T, Vh), mode, "Phi")
    plan.close()


# --------------------------------- full-size workloads, every round compared

def full_size_case(torch, L, name, mode, slice_bytes=1 << 29, seed=1):
    """Inputs are generated on the device and copied back, so both sides see the same
    bits.  EVERY round is compared: the oracle walks the schedule in slices of rounds (so
    that its fp64 artefacts stay bounded in host memory) and each slice's Vbar, X and D are
    compared element by element with the staged calls' and the fused pass's, and its X also
    with the one-pass pipeline's.  The outputs are compared in full with eq. (1)."""
    w = CONFIGS[name]
    plan = L.Plan(w.K, w.r, w.Q, w.N, jobs=w.jobs).bind(w.T, mode).upload()
    sh = plan.shapes()
    V = generate_torch(w.J, w.N, w.Q, w.T, seed, "u32" if mode == "u32" else "f32", sigma=w.sigma, device="cuda")
    poison = -1 if mode == "u32" else float("nan")
    X = dev_empty(torch, sh["X"], mode, poison)
    D = dev_empty(torch, sh["D"], mode, poison)
    Phi = dev_empty(torch, sh["Phi"], mode, poison)
    plan.shuffle_fused(V, X, D)
    plan.reduce(V, D, Phi)
    torch.cuda.synchronize()
    Vh = to_host(V, mode)
    if mode == "u32":
        want_phi = np.bitwise_xor.reduce(Vh, axis=1)
    else:
        want_phi = Vh.sum(axis=1, dtype=np.float64)
    assert_close(to_host(Phi, mode), want_phi, mode, "Phi vs eq.(1)")

    # the separate stages on the same inputs give the same bits as the fused pass
    Vbar = dev_empty(torch, sh["Vbar"], mode, poison)
    X1 = dev_empty(torch, sh["X"], mode, poison)
    plan.combine(V, Vbar)
    plan.encode(Vbar, X1)
    torch.cuda.synchronize()
    assert torch.equal(X1.view(torch.int32), X.view(torch.int32))
    del X1
    D1 = dev_empty(torch, sh["D"], mode, poison)
    plan.decode(X, Vbar, D1)
    torch.cuda.synchronize()
    assert torch.equal(D1.view(torch.int32), D.view(torch.int32))
    del D1
    X3 = None
    if not w.jobs:                     # the one-pass kernel covers single-job plans only
        # in the launch configuration the benchmark times
        X3 = dev_empty(torch, sh["X"], mode, poison)
        Phi3 = dev_empty(torch, sh["Phi"], mode, poison)
        plan.pipeline_fused(V, X3, Phi3)
        torch.cuda.synchronize()
        assert_close(to_host(Phi3, mode), want_phi, mode, "pipeline Phi vs eq.(1)")

    op = O.build_plan(w.K, w.r, w.Q, w.N, "paper" if w.jobs else "single")
    per_round = (w.r + 1) * w.W * 8 * 3                    # fp64 Vbar, D and (about) X of one round
    step = max(1, min(op.n_round, slice_bytes // per_round))
    compared = 0
    for u0 in range(0, op.n_round, step):
        rounds = list(range(u0, min(op.n_round, u0 + step)))
        sub = O.select_rounds(op, rounds)
        if mode == "h32":
            vb = O.combine_h32(sub, w.T, Vh)
            xr = O.encode_h32(sub, w.T, vb)
            dr = O.decode_h32(sub, w.T, xr, vb)
        else:
            vb = O.combine(sub, w.T, Vh)
            xr = O.encode(sub, w.T, vb)
            dr = O.decode(sub, w.T, xr, vb)
        lo, hi = rounds[0], rounds[-1] + 1
        assert_close(to_host(Vbar[lo:hi], mode), vb, mode, f"Vbar rounds {lo}..{hi}")
        assert_close(to_host(X[lo:hi], mode), xr, mode, f"X rounds {lo}..{hi}")
        assert_close(to_host(D[lo:hi], mode), dr, mode, f"D rounds {lo}..{hi}")
        if X3 is not None:
            assert_close(to_host(X3[lo:hi], mode), xr, mode, f"pipeline X rounds {lo}..{hi}")
        compared += len(rounds)
    assert compared == op.n_round == plan.n_round
    plan.close()


@pytest.mark.parametrize("mode", ["f32", "u32", "h32"])
def test_full_size_many_node_workload(torch, L, mode):
    full_size_case(torch, L, "cfg5_k24", mode)


def test_full_size_gradient_workload(torch, L):
    full_size_case(torch, L, "cfg3_gradient", "f32")


@pytest.mark.parametrize("mode", ["f32", "u32"])
def test_full_size_paper_schedule(torch, L, mode):
    """J = 56 jobs on K = 8 nodes, stage 1 and the five stage-2 rounds of every subset."""
    full_size_case(torch, L, "jobs_k8", mode)


# ------------------------------------- compression-only comparison scheme

@pytest.mark.parametrize("K,r,c,N,T", [(4, 2, 1, 6, 1024), (8, 2, 1, 28, 4096), (7, 2, 2, 14, 333), (6, 1, 1, 12, 520),
                                       (5, 3, 1, 10, 7), (9, 2, 1, 36, 64)])
@pytest.mark.parametrize("mode", ["u32", "f32"])
def test_compression_scheme(torch, L, K, r, c, N, T, mode):
    """Uncoded pre-combined packets (appendix): ccdc_combine makes them, ccdc_reduce
    adds them to the receiver's own batch; the coding entry points refuse the plan."""
    Q = c * K
    cp = O.CompressionPlan(K, r, Q, N)
    Vh = generate_numpy(1, N, Q, T, K + r, mode)
    want_p = cp.combine(T, Vh[0])
    want_phi = cp.reduce(T, Vh[0], want_p)
    plan = L.ccdc_plan_compression(K, r, Q, N).bind(T, mode).upload()
    sh = plan.shapes()
    V = to_dev(torch, Vh)
    poison = -1 if mode == "u32" else float("nan")
    P = dev_empty(torch, sh["Vbar"], mode, poison)
    Phi = dev_empty(torch, sh["Phi"], mode, poison)
    plan.combine(V, P)
    plan.reduce(V, P, Phi)
    torch.cuda.synchronize()
    assert_close(to_host(P, mode), want_p, mode, "packets")
    assert_close(to_host(Phi, mode)[0], want_phi, mode, "Phi")
    direct = np.bitwise_xor.reduce(Vh[0], axis=0) if mode == "u32" else Vh[0].sum(axis=0, dtype=np.float64)
    assert_close(to_host(Phi, mode)[0], direct, mode, "Phi vs eq.(1)")
    import ctypes as C
    lib, ptr = L.load_library(), C.c_void_p(P.data_ptr())
    assert lib.ccdc_encode(plan._h, ptr, ptr, None) == L.binding.ESTATE
    assert lib.ccdc_decode(plan._h, ptr, ptr, ptr, None) == L.binding.ESTATE
    assert lib.ccdc_shuffle_fused(plan._h, ptr, ptr, ptr, None) == L.binding.ESTATE
    assert lib.ccdc_pipeline_fused(plan._h, ptr, ptr, ptr, None) == L.binding.ESTATE
    plan.close()
