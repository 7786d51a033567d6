"""Pins of the oracle's compression-only comparison scheme (appendix of the
paper) and of the load comparison the paper draws between the three schemes.
CPU only."""
from fractions import Fraction
from math import ceil

import numpy as np
import pytest

import oracle as O
from workloads import generate_numpy


def load(cp, T):
    return Fraction(cp.scheduled_elems(T), cp.Q * T)


CASES = [(K, r) for K in range(2, 10) for r in range(1, K)]


@pytest.mark.parametrize("K,r", CASES)
def test_load_and_placement(K, r):
    """L = ceil(1/mu) - 1 for 1/K <= mu < 1/2 and 1 for 1/2 <= mu < 1 (Sec. III,
    compression load), reached with the cyclic batch placement of the appendix."""
    c = 2
    N = 2 * K * r            # mu*N = 2*r*r whole, N even, K <= N
    cp = O.CompressionPlan(K, r, c * K, N)
    mu = Fraction(r, K)
    want = Fraction(ceil(1 / mu) - 1) if mu < Fraction(1, 2) else Fraction(1)
    assert load(cp, 12) == want
    mu_used = min(mu, Fraction(1, 2))
    assert cp.nb == ceil(1 / mu_used)
    # batches: consecutive, cover all files, the first nb-1 hold mu*N files, the last the rest
    sizes = np.diff(cp.batch_first)
    assert cp.batch_first[0] == 0 and cp.batch_first[-1] == N and (sizes > 0).all()
    assert (sizes[:-1] == mu_used * N).all() and sizes[-1] == N - (cp.nb - 1) * mu_used * N
    # node k stores batch k mod nb: within its storage, and every batch is stored somewhere
    assert cp.node_batch.tolist() == [k % cp.nb for k in range(K)]
    assert all(sizes[cp.node_batch[k]] <= mu * N for k in range(K))
    assert set(cp.node_batch.tolist()) == set(range(cp.nb))
    # every node receives one packet per batch it does not store, from a node that stores it
    assert cp.n_packet == K * (cp.nb - 1)
    seen = set()
    for i in range(cp.n_packet):
        k, t, s = int(cp.pkt_recv[i]), int(cp.pkt_batch[i]), int(cp.pkt_send[i])
        assert t != cp.node_batch[k] and cp.node_batch[s] == t and s != k
        seen.add((k, t))
    assert len(seen) == cp.n_packet


@pytest.mark.parametrize("K,r,c,N,T", [(3, 2, 1, 6, 8), (4, 2, 1, 6, 5), (6, 1, 2, 12, 7), (7, 2, 1, 14, 4),
                                       (5, 2, 1, 10, 3), (8, 3, 1, 16, 6)])
@pytest.mark.parametrize("mode", ["u32", "f32"])
def test_every_output_is_the_plain_sum(K, r, c, N, T, mode):
    cp = O.CompressionPlan(K, r, c * K, N)
    V = generate_numpy(1, N, c * K, T, 5, "u32")[0]
    if mode == "f32":
        V = ((V % 201).astype(np.int64) - 100).astype(np.float32)      # exact arithmetic
    P = cp.combine(T, V)
    Phi = cp.reduce(T, V, P)
    want = np.bitwise_xor.reduce(V, axis=0) if mode == "u32" else V.astype(np.float64).sum(axis=0)
    assert np.array_equal(Phi, want)
    # a packet is the sum over exactly the files of its batch for the receiver's functions
    for i in range(cp.n_packet):
        k, t = int(cp.pkt_recv[i]), int(cp.pkt_batch[i])
        files = V[cp.batch_first[t]:cp.batch_first[t + 1], k * c:(k + 1) * c].reshape(-1, c * T)
        part = np.bitwise_xor.reduce(files, axis=0) if mode == "u32" else files.astype(np.float64).sum(axis=0)
        assert np.array_equal(P[i], part)


def test_k4_example_comparison(golden):
    """Remark after the K = 4 example: combining only sends 4 pre-combined packets
    (load 1), CDC only gives 3/2, compressed CDC 3/4."""
    g = golden("example_k4.txt")
    K, r, N, Q = (int(g[k]) for k in ("K", "r", "N", "Q"))
    cp = O.CompressionPlan(K, r, Q, N)
    assert cp.n_packet == 4
    assert load(cp, 16) == Fraction(g["load_compression_only"])
    pj = O.build_plan(K, r, Q, N, "paper")
    ccdc = Fraction(O.scheduled_elems(pj, 16), pj.J * Q * 16)
    mu = Fraction(r, K)
    cdc = (1 - mu) * N / (mu * K)                                   # L_CDC of Sec. III
    assert (load(cp, 16), cdc, ccdc) == (1, Fraction(g["load_cdc_only"]), Fraction(g["load_total"]))
    assert ccdc < load(cp, 16) < cdc


def test_k3_example_compression_load(golden):
    """Sec. II: the compression scheme of the motivating example moves 3 values of
    size T (one pre-combined packet per node)."""
    g = golden("example_k3.txt")
    cp = O.CompressionPlan(int(g["K"]), int(g["r"]), int(g["Q"]), int(g["N"]))
    assert Fraction(cp.scheduled_elems(32), 32) == Fraction(g["load_compression"])


@pytest.mark.parametrize("K,r", [(K, r) for K in range(3, 12) for r in range(1, K)])
def test_compressed_cdc_beats_both(K, r):
    """Remarks after Theorem 1: compressed CDC is below compression only (by about
    mu for small mu, 1-mu for large) and, unlike CDC only, independent of N."""
    mu = Fraction(r, K)
    thm1 = (1 - mu) * (mu * K + 1) / (mu * K)
    comp = Fraction(ceil(1 / mu) - 1) if mu < Fraction(1, 2) else Fraction(1)
    assert thm1 <= comp
    if r == 1:
        assert thm1 == Fraction(2 * (K - 1), K) and comp == K - 1
    for N in (K, 4 * K):                     # Sec. III: K <= N
        cdc = (1 - mu) * N / (mu * K)
        assert thm1 <= cdc
    # growing N leaves Theorem 1 alone and inflates CDC only
    assert (1 - mu) * (8 * K) / (mu * K) == 2 * (1 - mu) * (4 * K) / (mu * K)


@pytest.mark.parametrize("args", [(1, 1, 1, 4), (4, 0, 4, 12), (4, 4, 4, 12), (4, 2, 6, 12), (4, 2, 4, 3),
                                  (5, 2, 5, 6), (4, 3, 4, 5)])
def test_invalid_parameters(args):
    with pytest.raises(ValueError):
        O.CompressionPlan(*args)
