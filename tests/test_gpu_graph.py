"""The stage calls only enqueue kernels and allocate nothing, so a caller may
record them into a HIP graph.  The graph is replayed several times, with new
inputs and eager work between the replays, and every replay must equal the
eager result bit for bit.  Needs a GPU."""
import pytest

from workloads import generate_torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the graph test cannot run")
    torch.cuda.set_device(0)
    return torch


@pytest.fixture(scope="module")
def L(torch):
    import paper_1805_01993_amd as lib
    lib.load_library()
    return lib


@pytest.mark.parametrize("K,r,Q,N,T,mode", [(10, 3, 10, 120, 4096, "f32"),      # rounds cut into chunks: two kernels
                                            (8, 2, 8, 28, 65536, "u32"),        # one kernel, no workspace
                                            (10, 3, 10, 120, 4096, "bf16")])
def test_replays_equal_eager(torch, L, K, r, Q, N, T, mode):
    plan = L.ccdc_plan(K, r, Q, N).bind(T, mode).upload()
    sh = plan.shapes()
    kind = {"f32": "f32", "u32": "u32", "bf16": "bf16"}[mode]
    inputs = [generate_torch(1, N, Q, T, seed, kind, device="cuda") for seed in (1, 2, 3)]
    V = inputs[0].clone()
    new = lambda key: torch.zeros(sh[key], dtype=V.dtype, device="cuda")
    X, D, Phi, Xp, Php, Xn, Phn = new("X"), new("D"), new("Phi"), new("X"), new("Phi"), new("X"), new("Phi")
    Xs, Phs, Vm, Phm = new("X"), new("Phi"), new("V"), new("Phi")
    theta = generate_torch(1, 1, Q, T, 9, kind, device="cuda")[:, 0].contiguous()

    def enqueue(stream):
        plan.shuffle_fused(V, X, D, stream=stream)
        plan.reduce(V, D, Phi, stream=stream)
        plan.pipeline_fused(V, Xp, Php, stream=stream)
        plan.node_encode(-1, V, Xn, stream=stream)
        plan.node_decode_reduce(-1, V, Xn, Phn, stream=stream)
        plan.pipeline_fused_noalloc(V, Xs, Phs, stream=stream)      # the entry point meant for captured code
        plan.map(V, theta, Vm, stream=stream)                       # a step that starts from files
        plan.pipeline_fused_noalloc(Vm, Xs, Phm, stream=stream)

    outs = (X, D, Phi, Xp, Php, Xn, Phn, Phs, Vm, Phm)
    bits = lambda t: t.view(torch.int16 if t.element_size() == 2 else torch.int32)
    eager = []
    for inp in inputs:
        V.copy_(inp)
        enqueue(torch.cuda.current_stream())
        torch.cuda.synchronize()
        eager.append([bits(t).clone() for t in outs])

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        V.copy_(inputs[0])
        enqueue(side)                                   # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            enqueue(side)
    torch.cuda.synchronize()

    for rep in range(2):
        for i, inp in enumerate(inputs):
            V.copy_(inp)
            for t in outs:
                t.zero_()                               # eager work between replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for t, want in zip(outs, eager[i]):
                assert torch.equal(bits(t), want), (rep, i)
    plan.close()
