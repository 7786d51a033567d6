"""Parity of the HIP path with the CPU oracle for the 16-bit hybrid modes
(bfloat16 / binary16 payloads, fp32 sums rounded once, XOR-coded patterns),
through the C entry points.  Packets (Vbar, X, D) must be equal bit for bit; an
output must be the oracle's unrounded fp64 sum rounded once to the format, up
to the fp32 summation error.  Needs a GPU."""
import numpy as np
import pytest

import oracle as O
from workloads import CONFIGS, generate_numpy, generate_torch, half_bits_to_float

pytestmark = pytest.mark.gpu

FORMATS = ["bf16", "f16"]
HALF_ULP = {"bf16": 2.0 ** -8, "f16": 2.0 ** -11}      # 7 / 10 fraction bits
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
    lib.load_library()
    return lib


def to_dev(torch, bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()


def to_host(t):
    return t.cpu().numpy().view(np.uint16)


def dev_poison(torch, shape):
    return torch.full(tuple(shape), 0x7FFF, dtype=torch.int16, device="cuda")      # a NaN pattern in both formats


def assert_bits(got, want, name):
    assert got.shape == want.shape, name
    bad = np.flatnonzero(got.ravel() != want.ravel())
    assert bad.size == 0, f"{name}: {bad.size} patterns differ, first at {bad[:4]}"


def assert_rounded(got_bits, want64, fmt, name):
    """got = the fp32 sum rounded once to the format: within half a unit in the last
    place of the exact value, plus what fp32 summation in another order can move it."""
    assert got_bits.shape == want64.shape, name
    got = half_bits_to_float(got_bits, fmt).astype(np.float64)
    scale = max(float(np.abs(want64).max()), 1e-300)
    slack = HALF_ULP[fmt] * 1.001 * np.abs(want64) + F32_TOL * scale + (2.0 ** -25 if fmt == "f16" else 0.0)
    over = np.abs(got - want64) - slack
    assert np.isfinite(got).all() and over.max() <= 0, f"{name}: exceeds the rounding bound by {over.max():.3e}"


def run_case(torch, L, K, r, Q, N, T, fmt, jobs=False, seed=1, sigma=1.0):
    op = O.build_plan(K, r, Q, N, "paper" if jobs else "single")
    Vh = generate_numpy(op.J, N, Q, T, seed, fmt, sigma)
    ref = O.run_all_h16(op, T, Vh, fmt)
    ref_phi = O.direct_h16(op, T, Vh, fmt)

    plan = L.Plan(K, r, Q, N, jobs=jobs).bind(T, fmt).upload()
    sh = plan.shapes()
    V = to_dev(torch, Vh)
    Vbar, X, D, Phi = (dev_poison(torch, sh[k]) for k in ("Vbar", "X", "D", "Phi"))
    plan.combine(V, Vbar)
    plan.encode(Vbar, X)
    plan.decode(X, Vbar, D)
    plan.reduce(V, D, Phi)
    torch.cuda.synchronize()
    for name, t in (("Vbar", Vbar), ("X", X), ("D", D)):
        assert_bits(to_host(t), ref[name], name)
    assert_rounded(to_host(Phi), ref["Phi"], fmt, "Phi")
    if op.m == 1:                      # one-file batches are sent unrounded: the scheme's sum is eq. (1)
        assert_rounded(to_host(Phi), ref_phi, fmt, "Phi vs eq.(1)")

    X2, D2, Phi2 = (dev_poison(torch, sh[k]) for k in ("X", "D", "Phi"))
    plan.shuffle_fused(V, X2, D2)
    plan.reduce(V, D2, Phi2)
    torch.cuda.synchronize()
    assert torch.equal(X2, X) and torch.equal(D2, D) and torch.equal(Phi2, Phi)

    X3, Phi3 = dev_poison(torch, sh["X"]), dev_poison(torch, sh["Phi"])
    if not jobs and r <= 5 and K * r <= 256:
        plan.pipeline_fused(V, X3, Phi3)
        torch.cuda.synchronize()
        assert torch.equal(X3, X)
        assert_rounded(to_host(Phi3), ref["Phi"], fmt, "pipeline Phi")
    else:
        with pytest.raises(L.CcdcError) as err:
            plan.pipeline_fused(V, X3, Phi3)
        assert err.value.status == L.binding.ESIZE
    plan.close()


SHAPES = [
    # K, r, Q, N, T, jobs        what it exercises
    (4, 2, 4, 12, 256, False),    # the tiny workload: m = 2, 16-byte packs
    (3, 2, 3, 6, 1024, False),    # K = r+1
    (6, 1, 6, 12, 520, False),    # r = 1
    (5, 4, 5, 10, 64, False),     # r = K-1
    (5, 3, 10, 20, 1000, False),  # c = 2, m = 2, ragged split; ell not a multiple of 8: 8-byte packs
    (4, 2, 4, 12, 7, False),      # odd T: one element per pack
    (4, 2, 4, 12, 12, False),     # T a multiple of 4 only: 8-byte packs
    (4, 3, 4, 4, 10, False),      # tiny W, segments 4, 4, 2
    (4, 3, 4, 4, 1, False),       # W = 1
    (6, 3, 12, 40, 333, False),   # scalar path over several tiles, c = 2, m = 2
    (7, 5, 7, 21, 2056, False),   # r = 5
    (10, 8, 10, 45, 40, False),   # r = 8: no one-pass kernel
    (11, 9, 11, 55, 40, False),   # any-r fused fallback
    (4, 2, 4, 6, 512, True),      # J-job schedule
    (6, 3, 6, 8, 1200, True),     # J = 15 jobs, m = 2
    (4, 2, 4, 240, 16, False),    # m = 40: long fp32 sums before the one rounding
    (10, 3, 10, 120, 4096, False),  # the 10-node workload
]


@pytest.mark.parametrize("K,r,Q,N,T,jobs", SHAPES)
@pytest.mark.parametrize("fmt", FORMATS)
def test_shapes(torch, L, K, r, Q, N, T, jobs, fmt):
    run_case(torch, L, K, r, Q, N, T, fmt, jobs=jobs, seed=K * 10 + r)


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes(torch, L, seed):
    from math import comb
    rng = np.random.default_rng(2000 + seed)
    K = int(rng.integers(2, 10))
    r = int(rng.integers(1, K))
    jobs = bool(K <= 6 and rng.integers(0, 3) == 0)
    c = int(rng.integers(1, 4))
    nb = (r + 1) if jobs else comb(K, r)
    m = int(rng.integers(1, 4))
    while m * nb < K:
        m += 1
    T = int(rng.choice([1, 2, 3, 4, 5, 8, 12, 16, 24, 31, 64, 100, 128, 250, 256, 511, 520]))
    run_case(torch, L, K, r, c * K, m * nb, T, FORMATS[seed % 2], jobs=jobs, seed=seed)


CANON_NAN = {"bf16": 0x7FC0, "f16": 0x7E00}
INF = {"bf16": 0x7F80, "f16": 0x7C00}
LARGEST = {"bf16": 3.3895314e38, "f16": 65504.0}


@pytest.mark.parametrize("K,r,Q,N,T", [(5, 2, 5, 10, 1024),      # one-file batches: packets are the files' patterns
                                       (5, 2, 5, 20, 1024),      # m = 2: every packet is a rounded sum
                                       (4, 3, 8, 12, 100),       # m = 3, c = 2, short last segment, 8-byte packs
                                       (6, 2, 6, 30, 7)])        # m = 2, one-element packs
@pytest.mark.parametrize("fmt", FORMATS)
def test_special_patterns_in_the_payload(torch, L, K, r, Q, N, T, fmt):
    """Infinities, quiet and signalling NaNs with payloads and signs, subnormals, the largest
    finite values, sums that leave the format: packets (Vbar, X, D) of every path must equal
    the oracle's bit for bit (a sum that is not a number is stored as the one canonical NaN
    pattern on both sides, a one-file batch passes through untouched); an output is NaN
    exactly where the exact sum is, the same infinity where that is infinite, and within the
    rounding bound elsewhere."""
    from workloads import special_payload
    op = O.build_plan(K, r, Q, N)
    Vh = special_payload(op.shapes(T)["V"], fmt, seed=K * 100 + r * 10 + T % 7, density=0.03)
    ref = O.run_all_h16(op, T, Vh, fmt)
    plan = L.Plan(K, r, Q, N).bind(T, fmt).upload()
    sh = plan.shapes()
    V = to_dev(torch, Vh)
    Vbar, X, D, Phi = (dev_poison(torch, sh[k]) for k in ("Vbar", "X", "D", "Phi"))
    plan.combine(V, Vbar)
    plan.encode(Vbar, X)
    plan.decode(X, Vbar, D)
    plan.reduce(V, D, Phi)
    X2, D2, X3, Phi3, X4, Phi4 = (dev_poison(torch, sh[k]) for k in ("X", "D", "X", "Phi", "X", "Phi"))
    plan.shuffle_fused(V, X2, D2)
    plan.pipeline_fused(V, X3, Phi3)
    plan.node_encode(-1, V, X4)
    plan.node_decode_reduce(-1, V, X4, Phi4)
    torch.cuda.synchronize()
    for name, t in (("Vbar", Vbar), ("X", X), ("D", D), ("fused X", X2), ("fused D", D2), ("pipeline X", X3),
                    ("node-local X", X4)):
        assert_bits(to_host(t), ref[name.split()[-1]], name)
    want = ref["Phi"]
    # outputs whose finite terms cannot overflow an fp32 partial sum in any order: elsewhere
    # (bfloat16 only) the kernels' fp32 running sum may pass through infinity where the exact
    # sum does not, and nothing is claimed
    vals = half_bits_to_float(Vh, fmt).astype(np.float64)
    safe = np.where(np.isfinite(vals), np.abs(vals), 0.0).sum(axis=1) <= 1e38
    nan, inf = np.isnan(want), np.isinf(want) & safe
    assert nan.any() and (op.m > 1 or inf.any())
    plain = np.isfinite(want) & safe & (np.abs(want) <= LARGEST[fmt] * (1 - 2.0 ** -8))
    for name, t in (("Phi", Phi), ("pipeline Phi", Phi3), ("node-local Phi", Phi4)):
        got = to_host(t)
        assert (got[nan] == CANON_NAN[fmt]).all(), name
        assert np.array_equal(got[inf], np.where(want[inf] > 0, INF[fmt], 0x8000 | INF[fmt]).astype(np.uint16)), name
        val = half_bits_to_float(got[plain], fmt).astype(np.float64)
        scale = float(np.abs(want[plain]).max())
        over = np.abs(val - want[plain]) - (HALF_ULP[fmt] * 1.001 * np.abs(want[plain]) + F32_TOL * scale
                                            + (2.0 ** -25 if fmt == "f16" else 0.0))
        assert over.max() <= 0, f"{name}: exceeds the rounding bound by {over.max():.3e}"
    plan.close()


@pytest.mark.parametrize("fmt", FORMATS)
def test_two_byte_aligned_pointers(torch, L, fmt):
    """Buffers that are only 2-byte aligned take the one-element path; odd addresses are refused."""
    K, r, Q, N, T = 5, 2, 5, 10, 64
    op = O.build_plan(K, r, Q, N)
    Vh = generate_numpy(1, N, Q, T, 3, fmt)
    ref = O.run_all_h16(op, T, Vh, fmt)
    plan = L.ccdc_plan(K, r, Q, N).bind(T, fmt).upload()
    sh = plan.shapes()

    def shifted(shape):
        return torch.zeros(int(np.prod(shape)) + 1, dtype=torch.int16, device="cuda")[1:]

    V = shifted(sh["V"])
    V.copy_(to_dev(torch, Vh).reshape(-1))
    X, D, Phi, X3, Phi3 = (shifted(sh[k]) for k in ("X", "D", "Phi", "X", "Phi"))
    assert V.data_ptr() % 16 == 2
    plan.shuffle_fused(V, X, D)
    plan.reduce(V, D, Phi)
    plan.pipeline_fused(V, X3, Phi3)
    torch.cuda.synchronize()
    assert_bits(to_host(X).reshape(sh["X"]), ref["X"], "X")
    assert_bits(to_host(D).reshape(sh["D"]), ref["D"], "D")
    assert_bits(to_host(X3).reshape(sh["X"]), ref["X"], "pipeline X")
    assert_rounded(to_host(Phi).reshape(sh["Phi"]), ref["Phi"], fmt, "Phi")
    assert_rounded(to_host(Phi3).reshape(sh["Phi"]), ref["Phi"], fmt, "pipeline Phi")
    import ctypes as C
    lib = L.load_library()
    assert lib.ccdc_encode(plan._h, C.c_void_p(D.data_ptr() + 1), C.c_void_p(X.data_ptr()), None) == L.binding.EINVAL
    plan.close()


def test_element_size_is_checked(torch, L):
    plan = L.ccdc_plan(4, 2, 4, 12).bind(16, "bf16").upload()
    sh = plan.shapes()
    V = torch.zeros(sh["V"], dtype=torch.float32, device="cuda")
    with pytest.raises(ValueError):
        plan.combine(V, torch.zeros(sh["Vbar"], dtype=torch.int16, device="cuda"))
    plan.close()
    import ctypes as C
    h = L.ccdc_plan_compression(4, 2, 4, 8)
    assert L.load_library().ccdc_plan_bind(h._h, 16, L.binding.BF16_SUM_XOR) == L.binding.EINVAL
    h.close()


@pytest.mark.parametrize("name,fmt", [("cfg3_gradient", "bf16"), ("cfg5_k24", "bf16"), ("cfg5_k24", "f16")])
def test_full_size_workloads(torch, L, name, fmt, slice_bytes=1 << 28):
    """Full-size shapes in the launch configuration the benchmark times.  EVERY round is
    compared: the oracle walks the schedule in slices of rounds and each slice's coded and
    decoded packets must equal the one-pass pipeline's X and the fused pass's X and D bit for
    bit; every output is compared with eq. (1) (one-file batches: nothing but the output is
    rounded)."""
    w = CONFIGS[name]
    plan = L.Plan(w.K, w.r, w.Q, w.N).bind(w.T, fmt).upload()
    sh = plan.shapes()
    V = generate_torch(1, w.N, w.Q, w.T, 1, fmt, sigma=w.sigma, device="cuda").view(torch.int16)
    X, Phi = dev_poison(torch, sh["X"]), dev_poison(torch, sh["Phi"])
    plan.pipeline_fused(V, X, Phi)
    torch.cuda.synchronize()
    Vh = to_host(V)
    assert w.m == 1
    want_phi = half_bits_to_float(Vh, fmt).sum(axis=1, dtype=np.float64)
    assert_rounded(to_host(Phi), want_phi, fmt, "pipeline Phi vs eq.(1)")
    X2, D2, Phi2 = dev_poison(torch, sh["X"]), dev_poison(torch, sh["D"]), dev_poison(torch, sh["Phi"])
    plan.shuffle_fused(V, X2, D2)
    plan.reduce(V, D2, Phi2)
    torch.cuda.synchronize()
    assert torch.equal(X2, X)
    assert_rounded(to_host(Phi2), want_phi, fmt, "Phi vs eq.(1)")

    op = O.build_plan(w.K, w.r, w.Q, w.N)
    step = max(1, min(op.n_round, slice_bytes // ((w.r + 1) * w.W * 2 * 3)))
    compared = 0
    for u0 in range(0, op.n_round, step):
        rounds = list(range(u0, min(op.n_round, u0 + step)))
        part = O.shuffle_h16(O.select_rounds(op, rounds), w.T, Vh, fmt)
        lo, hi = rounds[0], rounds[-1] + 1
        assert_bits(to_host(X[lo:hi]), part["X"], f"pipeline X rounds {lo}..{hi}")
        assert_bits(to_host(D2[lo:hi]), part["D"], f"D rounds {lo}..{hi}")
        compared += len(rounds)
    assert compared == op.n_round
    plan.close()
