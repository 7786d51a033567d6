"""Pins of the oracle's placement and round schedule against what the paper fixes:
the printed examples (tests/golden) and the counting invariants of Sec. IV-A/IV-B.
CPU only."""
from itertools import combinations
from math import comb

import numpy as np
import pytest

import oracle as O

# lexicographic label rank -> block of files, chosen so that the plan reproduces
# the labelling the paper prints (its batch labelling is not lexicographic)
K3_ORDER = [1, 0, 2]
K4_ORDERS = [[1, 0, 2],   # job 1 on {1,2,3}: B12={3,4} B13={1,2} B23={5,6}   (printed)
             [2, 0, 1],   # job 2 on {1,2,4}: B12={5,6} printed, the other two free
             [0, 1, 2],   # job 3 on {1,3,4}: B13={1,2} printed, the other two free
             [1, 0, 2]]   # job 4 on {2,3,4}: B23={3,4} B24={1,2} B34={5,6}   (printed)


def ints(s):
    return sorted(int(x) for x in s.split())


def stored_files(plan, node, job=None):
    """Files (job, n) node stores: union of the batches whose label holds it."""
    out = set()
    for bt in range(plan.n_batch):
        if node in plan.batch_label[bt]:
            j = int(plan.batch_job[bt])
            if job is None or job == j:
                f0 = int(plan.batch_file0[bt])
                out |= {(j, n) for n in range(f0, f0 + plan.m)}
    return out


def batch_files(plan, bt):
    f0 = int(plan.batch_file0[bt])
    return list(range(f0, f0 + plan.m))


def test_k3_example_placement(golden):
    g = golden("example_k3.txt")
    K, r, Q, N = (int(g[k]) for k in ("K", "r", "Q", "N"))
    for schedule in ("single", "paper"):       # K = r+1: both schedules are the paper's
        p = O.build_plan(K, r, Q, N, schedule, K3_ORDER)
        assert (p.J, p.n_round, p.n_batch, p.m) == (1, 1, 3, 2)
        for node in (1, 2, 3):
            got = sorted(n + 1 for (_, n) in stored_files(p, node - 1))
            assert got == ints(g[f"node{node}_files"])
        # each node pre-combines two packets of two values each (Sec. II)
        per_node = [sum(1 for b in range(3) if node in p.batch_label[p.round_batch[0, b]])
                    for node in range(3)]
        assert per_node == [int(g["precombined_packets_per_node"])] * 3
        assert p.m == int(g["values_per_precombined_packet"])


def test_k3_single_and_paper_schedules_coincide():
    a = O.build_plan(3, 2, 3, 6, "single")
    b = O.build_plan(3, 2, 3, 6, "paper")
    for name in ("batch_job", "batch_file0", "batch_label", "round_member", "round_batch"):
        assert np.array_equal(getattr(a, name), getattr(b, name)), name


def test_k4_example(golden):
    g = golden("example_k4.txt")
    K, r, J, N, Q = (int(g[k]) for k in ("K", "r", "J", "N", "Q"))
    p = O.build_plan(K, r, Q, N, "paper", K4_ORDERS)
    assert p.J == J and p.n_round == J * (K - r) and p.m == 2

    def batch_of(job, label):            # 1-based job / nodes -> 1-based files
        for bt in range(p.n_batch):
            if p.batch_job[bt] == job - 1 and sorted(p.batch_label[bt] + 1) == sorted(label):
                return [n + 1 for n in batch_files(p, bt)]
        raise AssertionError("no such batch")

    # placement of job 1 (Sec. IV-A example)
    job1 = ints(g["job1_nodes"])
    assert sorted({k + 1 for bt in range(p.n_batch) if p.batch_job[bt] == 0
                   for k in p.batch_label[bt]}) == job1
    assert batch_of(1, [1, 2]) == ints(g["job1_batch_12"])
    assert batch_of(1, [1, 3]) == ints(g["job1_batch_13"])
    assert batch_of(1, [2, 3]) == ints(g["job1_batch_23"])

    # rounds of subset {1,2,3}: first is stage 1 (job 1), second is stage 2 (outside node 4)
    rounds = [u for u in range(p.n_round) if list(p.round_member[u] + 1) == [1, 2, 3]]
    assert len(rounds) == 2
    s1, s2 = rounds
    assert {int(p.batch_job[bt]) for bt in p.round_batch[s1]} == {0}
    # in stage 2 Node 1 maps the batches served to the OTHER two members
    mapped = {}
    for b in range(r + 1):
        bt = p.round_batch[s2, b]
        if 0 in p.batch_label[bt]:
            mapped[int(p.batch_job[bt]) + 1] = [n + 1 for n in batch_files(p, bt)]
    assert mapped == {2: ints(g["stage2_node1_job2_files"]), 3: ints(g["stage2_node1_job3_files"])}
    assert sum(len(v) for v in mapped.values()) == int(g["stage2_files_mapped_per_node"])

    # final reduction example: what Node 1 receives for job 4 in each subset it is in
    got = {}
    for u in range(p.n_round):
        for b in range(r + 1):
            bt = p.round_batch[u, b]
            if p.round_member[u, b] == 0 and p.batch_job[bt] == 3:
                got[tuple(int(x) + 1 for x in p.round_member[u])] = [n + 1 for n in batch_files(p, bt)]
    assert got == {(1, 2, 3): ints(g["node1_subset_123_job4_files"]),
                   (1, 2, 4): ints(g["node1_subset_124_job4_files"]),
                   (1, 3, 4): ints(g["node1_subset_134_job4_files"])}


SWEEP = [(K, r) for K in range(2, 8) for r in range(1, K)]


@pytest.mark.parametrize("K,r", SWEEP)
@pytest.mark.parametrize("schedule", ["single", "paper"])
def test_placement_and_delivery_invariants(K, r, schedule):
    c = 2
    nb = comb(K, r) if schedule == "single" else r + 1
    m = max(2, -(-K // nb))                          # keeps K <= N
    Q, N = c * K, m * nb
    p = O.build_plan(K, r, Q, N, schedule)
    G = comb(K, r + 1)
    J = 1 if schedule == "single" else G
    assert (p.J, p.c, p.m) == (J, c, m)
    assert p.n_round == (G if schedule == "single" else G * (K - r))

    # Sec. IV-A: the batches partition each job's files; every file sits on exactly r nodes
    copies = np.zeros((J, N), dtype=int)
    for bt in range(p.n_batch):
        lab = list(p.batch_label[bt])
        assert lab == sorted(set(lab)) and len(lab) == r and 0 <= lab[0] and lab[-1] < K
        for n in batch_files(p, bt):
            copies[p.batch_job[bt], n] += 1
    assert (copies == 1).all()                       # one batch per file ...
    per_node = [len(stored_files(p, k)) for k in range(K)]
    assert per_node == [r * J * N // K] * K          # ... stored r times: |M_k| = mu*J*N
    if schedule == "paper":
        # each job lives on exactly r+1 nodes and a member stores r*N/(r+1) of its files
        for j in range(J):
            holders = [k for k in range(K) if stored_files(p, k, j)]
            assert len(holders) == r + 1
            assert all(len(stored_files(p, k, j)) == r * N // (r + 1) for k in holders)

    # Sec. IV-B: rounds run in (r+1)-subsets; member b is served the batch stored on the others
    per_node_rounds = np.zeros(K, dtype=int)
    delivered = {}
    for u in range(p.n_round):
        S = list(p.round_member[u])
        assert S == sorted(set(S)) and len(S) == r + 1
        for b, k in enumerate(S):
            per_node_rounds[k] += 1
            bt = int(p.round_batch[u, b])
            assert sorted(p.batch_label[bt]) == [s for s in S if s != k]
            key = (k, bt)
            assert key not in delivered              # never the same batch twice to a node
            delivered[key] = u
    rounds_per_subset = 1 if schedule == "single" else K - r
    assert (per_node_rounds == comb(K - 1, r) * rounds_per_subset).all()
    # completeness: a node is served every batch it does not store, exactly once
    for k in range(K):
        need = {bt for bt in range(p.n_batch) if k not in p.batch_label[bt]}
        assert {bt for (kk, bt) in delivered if kk == k} == need
    # every (r+1)-subset is used
    assert {tuple(s) for s in p.round_member.tolist()} == set(combinations(range(K), r + 1))


def test_batch_order_is_respected():
    p = O.build_plan(4, 2, 4, 12, "single", [5, 4, 3, 2, 1, 0])
    assert p.batch_file0.tolist() == [10, 8, 6, 4, 2, 0]


@pytest.mark.parametrize("args", [
    (1, 1, 1, 4), (4, 0, 4, 12), (4, 4, 4, 12),      # K>=2, 1<=r<=K-1 (Theorem 1)
    (4, 2, 6, 12),                                   # K | Q (Sec. III network model)
    (4, 2, 4, 3),                                    # K <= N (Sec. III network model)
    (4, 2, 4, 13),                                   # batches must be even (Sec. IV-A)
])
def test_invalid_parameters_are_rejected(args):
    with pytest.raises(ValueError):
        O.build_plan(*args)


def test_bad_batch_order_rejected():
    with pytest.raises(ValueError):
        O.build_plan(3, 2, 3, 6, "single", [0, 0, 1])
    with pytest.raises(ValueError):
        O.build_plan(4, 2, 4, 6, "paper", [[0, 1, 2], [0, 1, 2]])   # neither 1 nor J sets


def test_binom_against_math_comb():
    lib = O.ccdc_oracle._load()
    for n in range(0, 40):
        for k in range(0, n + 1):
            assert lib.orc_binom(n, k) == comb(n, k)
    assert lib.orc_binom(5, 6) == -1 and lib.orc_binom(200, 100) == -1


def test_full_size_shapes():
    """Counts of the five workloads (one batch per r-subset, Q = K)."""
    from workloads import CONFIGS
    for w in CONFIGS.values():
        if w.compression:
            cp = O.CompressionPlan(w.K, w.r, w.Q, w.N)
            assert cp.nb == 4 and cp.n_packet == 24
            continue
        if w.jobs:
            p = O.build_plan(w.K, w.r, w.Q, w.N, "paper")
            assert p.J == comb(w.K, w.r + 1) == w.J and p.n_round == w.G and p.m == w.m
            continue
        p = O.build_plan(w.K, w.r, w.Q, w.N)
        assert p.n_round == comb(w.K, w.r + 1) and p.n_batch == comb(w.K, w.r) and p.m == w.m


@pytest.mark.parametrize("K,r,gamma", [(4, 2, 2), (5, 2, 3), (4, 3, 4), (6, 1, 2)])
def test_repeated_scheme(K, r, gamma):
    """J = gamma*C(K, r+1) jobs (Sec. IV): the scheme works on C(K, r+1) jobs at a time and
    repeats the same operations gamma times; the load per job is Theorem 1's."""
    from fractions import Fraction
    N = (r + 1) * max(1, -(-K // (r + 1)))
    one = O.build_plan(K, r, 2 * K, N, "paper")
    rep = O.build_plan(K, r, 2 * K, N, "paper", gamma=gamma)
    G = comb(K, r + 1)
    assert one.J == G and rep.J == gamma * G and rep.n_round == gamma * one.n_round and rep.n_batch == gamma * one.n_batch
    for g in range(gamma):
        b = slice(g * one.n_batch, (g + 1) * one.n_batch)
        u = slice(g * one.n_round, (g + 1) * one.n_round)
        assert np.array_equal(rep.batch_job[b], one.batch_job + g * G)          # the next block of jobs ...
        assert np.array_equal(rep.batch_file0[b], one.batch_file0)              # ... placed the same way
        assert np.array_equal(rep.batch_label[b], one.batch_label)
        assert np.array_equal(rep.round_member[u], one.round_member)            # ... in the same rounds
        assert np.array_equal(rep.round_batch[u], one.round_batch + g * one.n_batch)
    # every job's files are each stored r times, |M_k| = mu*J*N
    assert [len(stored_files(rep, k)) for k in range(K)] == [r * rep.J * N // K] * K
    T = 4 * r
    mu = Fraction(r, K)
    assert Fraction(O.scheduled_elems(rep, T), rep.J * rep.Q * T) == (1 - mu) * (mu * K + 1) / (mu * K)
    with pytest.raises(ValueError):
        O.build_plan(K, r, 2 * K, N, "paper", gamma=0)
