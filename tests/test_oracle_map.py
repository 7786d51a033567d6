"""Pins of the oracle's Map stand-in (Sec. III, Map phase, with g_q = chunk q of the
gradient of 1/2 |theta - w_n|^2): against numpy / torch doing the subtraction in their own
arithmetic, and against the closed form the shuffle path must then reach,
Phi = N*theta - sum_n w_n.  CPU only."""
import numpy as np
import pytest
import torch

import oracle as O
from workloads import generate_numpy


def test_map_is_the_elementwise_difference():
    J, N, Q, T = 2, 5, 4, 33
    files = generate_numpy(J, N, Q, T, 3, "f32")
    theta = generate_numpy(J, 1, Q, T, 4, "f32")[:, 0]
    V = O.map_files(files, theta)
    assert np.array_equal(V, theta[:, None] - files)                       # numpy's fp32 subtraction
    assert V.dtype == np.float32 and V.shape == files.shape
    fu = generate_numpy(J, N, Q, T, 5, "u32")
    tu = generate_numpy(J, 1, Q, T, 6, "u32")[:, 0]
    assert np.array_equal(O.map_files(fu, tu), tu[:, None] ^ fu)
    # a transposed or shifted operand changes the result
    assert not np.array_equal(V, files - theta[:, None])
    assert not np.array_equal(V, np.roll(theta, 1, axis=1)[:, None] - files)


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_map_on_16_bit_payloads_rounds_the_fp32_difference_once(fmt):
    J, N, Q, T = 1, 6, 3, 50
    files = generate_numpy(J, N, Q, T, 7, fmt)
    theta = generate_numpy(J, 1, Q, T, 8, fmt)[:, 0]
    got = O.map_files(files, theta, fmt)
    if fmt == "f16":
        want = (theta.view(np.float16).astype(np.float32)[:, None] - files.view(np.float16).astype(np.float32)) \
            .astype(np.float16).view(np.uint16)
    else:
        tf = torch.from_numpy(theta.view(np.int16).copy()).view(torch.bfloat16).float()
        ff = torch.from_numpy(files.view(np.int16).copy()).view(torch.bfloat16).float()
        want = (tf[:, None] - ff).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("schedule,K,r,N", [("single", 5, 2, 20), ("paper", 4, 2, 6)])
def test_the_path_after_the_map_gives_the_full_gradient(schedule, K, r, N):
    """With integer-valued data every operation is exact: the reduced outputs of the scheme
    run on the mapped values equal N*theta - sum_n w_n, the gradient of the whole job."""
    plan = O.build_plan(K, r, K, N, schedule)
    T = 12
    rng = np.random.default_rng(9)
    files = rng.integers(-40, 40, size=(plan.J, N, K, T)).astype(np.float32)
    theta = rng.integers(-40, 40, size=(plan.J, K, T)).astype(np.float32)
    out = O.run_all(plan, T, O.map_files(files, theta))
    want = N * theta.astype(np.float64) - files.astype(np.float64).sum(axis=1)
    assert np.array_equal(out["Phi"], want)
    fu = rng.integers(0, 2 ** 32, size=(plan.J, N, K, T), dtype=np.uint64).astype(np.uint32)
    tu = rng.integers(0, 2 ** 32, size=(plan.J, K, T), dtype=np.uint64).astype(np.uint32)
    got = O.run_all(plan, T, O.map_files(fu, tu))["Phi"]
    want = np.bitwise_xor.reduce(fu, axis=1) ^ (tu if N % 2 else np.zeros_like(tu))   # N copies of theta cancel in pairs
    assert np.array_equal(got, want)
