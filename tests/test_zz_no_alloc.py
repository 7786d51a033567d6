"""ccdc_pipeline_fused_noalloc, the entry point that allocates nothing: through the C
symbols, its X and Phi must equal ccdc_pipeline_fused's on the same inputs, on two calls
in a row of which the second has the smaller input (the scratch array still holds the
first call's partial sums).  Needs a GPU."""
import ctypes as C

import numpy as np
import pytest

import oracle as O
from workloads import generate_numpy

pytestmark = pytest.mark.gpu


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


def run_both(torch, L, K, r, Q, N, T, mode, seed):
    lib = L.load_library()
    plan = L.ccdc_plan(K, r, Q, N).bind(T, mode).upload()
    sh = plan.shapes()
    Vh = generate_numpy(1, N, Q, T, seed, mode)
    V = torch.from_numpy(Vh.view(np.int32) if mode == "u32" else Vh).cuda()
    dt = torch.int32 if mode == "u32" else torch.float32
    poison = -1 if mode == "u32" else float("nan")
    new = lambda key: torch.full(sh[key], poison, dtype=dt, device="cuda")
    X0, P0, X1, P1 = new("X"), new("Phi"), new("X"), new("Phi")
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    ptr = lambda t: C.c_void_p(t.data_ptr())
    assert lib.ccdc_pipeline_fused(plan._h, ptr(V), ptr(X0), ptr(P0), st) == 0
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    assert lib.ccdc_pipeline_fused_noalloc(plan._h, ptr(V), ptr(X1), ptr(P1), st) == 0
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(X1.view(torch.int32), X0.view(torch.int32)), "X differs"
    assert torch.equal(P1.view(torch.int32), P0.view(torch.int32)), "Phi differs"
    # and against the oracle's plain sum (bit-exact for XOR, 1e-5 of the largest output for fp32)
    want = O.direct(O.build_plan(K, r, Q, N), T, Vh)
    got = P1.cpu().numpy()
    if mode == "u32":
        assert np.array_equal(got.view(np.uint32), want)
    else:
        assert np.abs(got.astype(np.float64) - want).max() <= 1e-5 * np.abs(want).max()
    chunked = plan.workspace_bytes > 0
    plan.close()
    return chunked


@pytest.mark.parametrize("mode", ["f32", "u32"])
def test_two_calls_in_a_row_second_smaller(torch, L, mode):
    # both shapes cut their rounds into chunks, so both calls really use the scratch array
    assert run_both(torch, L, 10, 3, 10, 120, 4096, mode, seed=1)
    assert run_both(torch, L, 6, 2, 6, 30, 1000, mode, seed=2)
    # a launch with a single chunk needs no scratch and is accepted at any size
    run_both(torch, L, 8, 2, 8, 28, 200_000, mode, seed=3)
