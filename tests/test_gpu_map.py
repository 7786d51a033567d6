"""The Map stand-in on the GPU (ccdc_map: V = theta - files, Sec. III Map phase) against the
oracle's, bit for bit in every payload mode, also in place; and the whole path run from
files: the reduced outputs must be the full gradient N*theta - sum_n w_n.  Needs a GPU."""
import numpy as np
import pytest

import oracle as O
from workloads import CONFIGS, generate_numpy, generate_torch, half_bits_to_float

pytestmark = pytest.mark.gpu

DT = {"f32": np.float32, "u32": np.uint32, "bf16": np.uint16, "f16": np.uint16}


@pytest.fixture(scope="module")
def torch():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    torch.cuda.set_device(0)
    return torch


@pytest.fixture(scope="module")
def L(torch):
    import paper_1805_01993_amd as lib
    lib.load_library()
    return lib


def to_dev(torch, a):
    view = {np.dtype(np.uint32): np.int32, np.dtype(np.uint16): np.int16}.get(a.dtype)
    return torch.from_numpy(np.ascontiguousarray(a.view(view) if view else a)).cuda()


def bits(t):
    a = t.cpu().numpy()
    return a.view({2: np.uint16, 4: np.uint32}[a.dtype.itemsize])


@pytest.mark.parametrize("K,r,Q,N,T,jobs", [(5, 2, 5, 20, 1000, False),     # m = 2
                                            (4, 2, 4, 12, 7, False),        # one-element packs
                                            (6, 3, 12, 40, 328, False),     # c = 2, eight-element packs for 16 bits
                                            (4, 2, 4, 6, 512, True)])       # four jobs, one model each
@pytest.mark.parametrize("mode", ["f32", "u32", "bf16", "f16"])
def test_map_equals_the_oracles_and_feeds_the_path(torch, L, K, r, Q, N, T, jobs, mode):
    op = O.build_plan(K, r, Q, N, "paper" if jobs else "single")
    files = generate_numpy(op.J, N, Q, T, 21, mode)
    theta = np.ascontiguousarray(generate_numpy(op.J, 1, Q, T, 22, mode)[:, 0])
    fmt = mode if mode in ("bf16", "f16") else None
    want = O.map_files(files, theta, fmt)
    plan = L.Plan(K, r, Q, N, jobs=jobs).bind(T, mode).upload()
    sh = plan.shapes()
    Fd, Td = to_dev(torch, files), to_dev(torch, theta)
    V = torch.full(sh["V"], -1, dtype=Fd.dtype, device="cuda")
    plan.map(Fd, Td, V)
    torch.cuda.synchronize()
    assert np.array_equal(bits(V), want.view(bits(V).dtype)), "V differs from the oracle's map"
    assert torch.equal(Fd, to_dev(torch, files))                      # inputs untouched
    inplace = Fd.clone()
    plan.map(inplace, Td, inplace)                                    # the values replace the files
    torch.cuda.synchronize()
    assert torch.equal(inplace, V)

    # the shuffle path on the mapped values: outputs = N*theta - sum of the files
    X, D, Phi = (torch.empty(sh[k], dtype=Fd.dtype, device="cuda") for k in ("X", "D", "Phi"))
    plan.shuffle_fused(V, X, D)
    plan.reduce(V, D, Phi)
    torch.cuda.synchronize()
    if mode == "u32":
        full = np.bitwise_xor.reduce(files, axis=1) ^ (theta if N % 2 else np.zeros_like(theta))
        assert np.array_equal(bits(Phi), full)
    elif mode == "f32":
        full = N * theta.astype(np.float64) - files.astype(np.float64).sum(axis=1)
        got = Phi.cpu().numpy().astype(np.float64)
        # every mapped value carries one fp32 rounding of a difference of N(0,1) numbers
        assert np.abs(got - full).max() <= 1e-5 * np.abs(full).max()
    else:
        ref = O.run_all_h16(op, T, want, mode)["Phi"]                 # exact sum of the 16-bit mapped values
        got = half_bits_to_float(bits(Phi), mode).astype(np.float64)
        half_ulp = 2.0 ** -8 if mode == "bf16" else 2.0 ** -11
        slack = half_ulp * 1.001 * np.abs(ref) + 1e-5 * np.abs(ref).max() + 2.0 ** -25
        assert (np.abs(got - ref) <= slack).all()
    plan.close()


def test_gradient_workload_from_files(torch, L):
    """The gradient shape end to end from files: ccdc_map, then the one-pass pipeline in the
    launch configuration the benchmark times."""
    w = CONFIGS["cfg3_gradient"]
    plan = L.ccdc_plan(w.K, w.r, w.Q, w.N).bind(w.T, "f32").upload()
    sh = plan.shapes()
    files = generate_torch(1, w.N, w.Q, w.T, 31, "f32", sigma=w.sigma, device="cuda")
    theta = generate_torch(1, 1, w.Q, w.T, 32, "f32", sigma=w.sigma, device="cuda")[:, 0].contiguous()
    fh, th = files.cpu().numpy(), theta.cpu().numpy()
    full = w.N * th.astype(np.float64) - fh.sum(axis=1, dtype=np.float64)
    plan.map(files, theta, files)                                     # in place
    X = torch.empty(sh["X"], dtype=torch.float32, device="cuda")
    Phi = torch.empty(sh["Phi"], dtype=torch.float32, device="cuda")
    plan.pipeline_fused(files, X, Phi)
    torch.cuda.synchronize()
    # sampled rows of the mapped values against the oracle's map (bit for bit)
    for n in (0, 13, w.N - 1):
        want = O.map_files(np.ascontiguousarray(fh[:, n:n + 1]), th)
        assert np.array_equal(files[:, n:n + 1].cpu().numpy().view(np.uint32), want.view(np.uint32)), n
    got = Phi.cpu().numpy().astype(np.float64)
    assert np.abs(got - full).max() <= 1e-5 * np.abs(full).max()
    plan.close()
