"""Pins of the oracle's scheduled-traffic count against the paper's load
analysis: Theorem 1, the per-stage loads of Sec. IV-B, the printed example
values (tests/golden) and the special cases.  CPU only."""
from fractions import Fraction
from math import comb

import pytest

import oracle as O


def load(plan, T):
    """Definition 1: bits in all broadcast messages over J*Q*T."""
    return Fraction(O.scheduled_elems(plan, T), plan.J * plan.Q * T)


def test_k3_example_loads(golden):
    g = golden("example_k3.txt")
    K, r, Q, N = (int(g[k]) for k in ("K", "r", "Q", "N"))
    T = 64
    p = O.build_plan(K, r, Q, N)
    # Sec. II normalises by the size of one intermediate value (T), not by Q*T
    assert Fraction(O.scheduled_elems(p, T), T) == Fraction(g["load_compressed_cdc"])
    # each of the 3 coded packets is half an intermediate value
    W = p.c * T
    for a in range(r + 1):
        assert Fraction(O.packet_len(W, r, a), T) == Fraction(g["coded_packet_fraction"])
    # the same example through Theorem 1 (normalised by J*Q*T): (1-mu)(mu K+1)/(mu K) = 1/2
    assert load(p, T) == Fraction((K - r) * (r + 1), r * K) == Fraction(1, 2)
    # uncoded, uncombined unicast would move N*Q*(1-mu) values = 6 T per ... check the
    # "reduces by half" statements: compression and CDC both give 3, twice compressed CDC
    assert Fraction(g["load_compression"]) == Fraction(g["load_cdc"]) == 2 * Fraction(g["load_compressed_cdc"])


def test_k4_example_loads(golden):
    g = golden("example_k4.txt")
    K, r, J, N, Q = (int(g[k]) for k in ("K", "r", "J", "N", "Q"))
    T = 32
    p = O.build_plan(K, r, Q, N, "paper")
    W = p.c * T
    per_round = sum(O.packet_len(W, r, a) for a in range(r + 1))
    assert Fraction(per_round, J * Q * T) == Fraction(g["load_stage1"]) == Fraction(g["load_stage2"])
    assert load(p, T) == Fraction(g["load_total"])
    # remark after the example: the two baselines it is compared with
    mu = Fraction(r, K)
    assert (1 - mu) * N / (mu * K) == Fraction(g["load_cdc_only"])            # L_CDC, Sec. III
    assert Fraction(g["load_compression_only"]) == 1                           # mu = 1/2 branch
    assert load(p, T) < Fraction(g["load_compression_only"]) < Fraction(g["load_cdc_only"])


@pytest.mark.parametrize("K,r", [(K, r) for K in range(2, 9) for r in range(1, K)])
def test_theorem1_load_for_paper_schedule(K, r):
    """L = (1-mu)(mu K+1)/(mu K) with J = C(K, mu K+1) jobs (Theorem 1)."""
    c = 2
    T = 4 * r * 3                      # 4r | c*T: the split is exact
    p = O.build_plan(K, r, c * K, max(r + 1, (r + 1) * -(-K // (r + 1))), "paper")
    mu = Fraction(r, K)
    assert load(p, T) == (1 - mu) * (mu * K + 1) / (mu * K)
    assert O.scheduled_elems(p, T) == O.closed_form_elems(p, T)
    # per stage and subset (Sec. IV-B): stage 1 is 1 round, stage 2 is K-r-1 rounds
    J = comb(K, r + 1)
    per_round = Fraction((r + 1) * c * T, r)
    assert per_round / (J * c * K * T) == Fraction(r + 1, r) / (J * K)


@pytest.mark.parametrize("K,r", [(K, r) for K in range(2, 9) for r in range(1, K)])
def test_single_job_schedule_load(K, r):
    """One stage-1 round per (r+1)-subset: G*(r+1)*c*T/r elements, i.e. C(K-1,r)/r
    when normalised by Q*T; equals Theorem 1 times C(K,r+1)/(K-r)."""
    c, T = 1, 4 * r * 5
    nb = comb(K, r)
    p = O.build_plan(K, r, c * K, nb * max(1, -(-K // nb)))
    G = comb(K, r + 1)
    assert O.scheduled_elems(p, T) == G * (r + 1) * c * T // r
    assert load(p, T) == Fraction(comb(K - 1, r), r)
    thm1 = Fraction((K - r) * (r + 1), r * K)
    assert load(p, T) == thm1 * G / (K - r)
    if r == K - 1:
        assert load(p, T) == thm1            # one subset: the schedule IS the paper's
    if r == 1:
        # packets are uncoded unicasts of pre-combined values: the compression-only
        # load of the appendix at mu = 1/K, ceil(1/mu) - 1 = K - 1
        assert load(p, T) == K - 1


def test_tiny_workload_scheduled_elements():
    p = O.build_plan(4, 2, 4, 12)
    assert O.scheduled_elems(p, 256) == 4 * 3 * 128 == 1536


@pytest.mark.parametrize("W,r", [(W, r) for r in range(1, 7) for W in list(range(1, 70)) + [4096, 4095, 2048, 3200000]])
def test_segment_split_properties(W, r):
    """Reading of 'evenly split into mu*K segments' when r does not divide W:
    segments tile [0,W) in order, all but the tail have length ell, ell is a
    multiple of 4 unless the split is exact, and the overhead is bounded."""
    ell = O.segment_len(W, r)
    counts = [O.segment_count(W, r, rho) for rho in range(r)]
    assert sum(counts) == W
    assert all(cnt in (0, ell) or cnt == W - i * ell for i, cnt in enumerate(counts))
    assert counts == sorted(counts, reverse=True)
    if W % (4 * r) == 0:
        assert ell * r == W and counts == [ell] * r
    else:
        assert ell % 4 == 0 and ell >= -(-W // r) and ell - (-(-W // r)) < 4
    # label_rank(a,b): position of s_a inside S minus s_b
    for a in range(r + 1):
        for b in range(r + 1):
            if a != b:
                assert O.label_rank(a, b) == sorted(set(range(r + 1)) - {b}).index(a)
    # a sender's packet is as long as the longest segment it carries; summed over the
    # r+1 senders this is W plus one full first segment
    assert sum(O.packet_len(W, r, a) for a in range(r + 1)) == W + min(ell, W)
    closed = Fraction((r + 1) * W, r)
    sched = W + min(ell, W)
    if W % (4 * r) == 0:
        assert sched == closed
    elif W >= ell:
        assert 0 <= sched - closed < 4


def test_workload_scheduled_bytes():
    """Byte counts of the five workloads (4-byte elements)."""
    from workloads import CONFIGS
    want = {"cfg1_tiny": 6144, "cfg2_k10": 4589760, "cfg3_gradient": 1075200000,
            "cfg4_k16": 39777920, "cfg5_k24": 435240960}
    for name, w in CONFIGS.items():
        if w.jobs or w.compression:
            continue
        p = O.build_plan(w.K, w.r, w.Q, w.N)
        got = 4 * O.scheduled_elems(p, w.T)
        closed = 4 * O.closed_form_elems(p, w.T)
        assert got == want[name]
        if w.W % (4 * w.r) == 0:
            assert got == closed
        else:
            assert 0 < got - closed < 16 * w.G
