"""Pins of the oracle's four stages: the definition of the result (eq. (1)),
set-labelled brute force straight from the equations of Sec. IV-B, exact
recovery, and locality/faithfulness properties.  CPU only, tiny sizes."""
from itertools import combinations
from math import comb

import numpy as np
import pytest

import oracle as O
from workloads import generate_numpy


def make_inputs(plan, T, mode, seed=1):
    """uint32 words, or small-integer-valued fp32 (every fp64 operation exact)."""
    if mode == "u32":
        return generate_numpy(plan.J, plan.N, plan.Q, T, seed, "u32")
    w = generate_numpy(plan.J, plan.N, plan.Q, T, seed, "u32")
    return ((w % 201).astype(np.int64) - 100).astype(np.float32)


def plan_for(K, r, c, m, schedule):
    nb = comb(K, r) if schedule == "single" else r + 1
    while m * nb < K:
        m += 1
    return O.build_plan(K, r, c * K, m * nb, schedule)


# ---------------------------------------------------------------- eq. (1)

@pytest.mark.parametrize("mode", ["u32", "f32"])
def test_direct_is_the_plain_sum(mode):
    p = O.build_plan(4, 2, 8, 12)
    V = make_inputs(p, 7, mode)
    got = O.direct(p, 7, V)
    if mode == "u32":
        want = np.bitwise_xor.reduce(V, axis=1)
    else:
        want = V.astype(np.float64).sum(axis=1)
    assert got.shape == (1, 8, 7) and np.array_equal(got, want)


SWEEP = [(K, r, c, m, T)
         for K in range(2, 7) for r in range(1, K)
         for c in (1, 2) for m in (1, 2, 3) for T in (1, 2, 3, 5, 8)]


@pytest.mark.parametrize("schedule", ["single", "paper"])
@pytest.mark.parametrize("mode", ["u32", "f32"])
def test_scheme_recovers_every_output_exactly(schedule, mode):
    """Every reducer ends with exactly sum_n v_{q,n} (eq. (1)), and every receiver
    decodes exactly the pre-combined packet meant for it (Sec. IV-B, decoding)."""
    checked = 0
    for (K, r, c, m, T) in SWEEP:
        if schedule == "paper" and (K > 5 or m == 3):
            continue
        p = plan_for(K, r, c, m, schedule)
        V = make_inputs(p, T, mode, seed=K * 100 + r)
        art = O.run_all(p, T, V)
        assert np.array_equal(art["Phi"], O.direct(p, T, V)), (K, r, c, m, T)
        assert np.array_equal(art["D"], art["Vbar"]), (K, r, c, m, T)
        checked += 1
    assert checked > 100


def test_real_valued_inputs_match_direct_sum_to_rounding():
    p = O.build_plan(5, 2, 10, 20)
    T = 37                                             # r does not divide W
    V = generate_numpy(1, p.N, p.Q, T, 3, "f32")
    art = O.run_all(p, T, V)
    ref = O.direct(p, T, V)
    assert np.abs(art["Phi"] - ref).max() <= 1e-12 * np.abs(ref).max()
    assert np.abs(art["D"] - art["Vbar"]).max() <= 1e-12 * np.abs(art["Vbar"]).max()


# ------------------------------------------------ stage by stage, from the sets

def stored_at(plan):
    """node -> set of (job, file) it stores, from the batch labels (Sec. IV-A)."""
    out = {k: set() for k in range(plan.K)}
    for bt in range(plan.n_batch):
        for n in range(plan.batch_file0[bt], plan.batch_file0[bt] + plan.m):
            for k in plan.batch_label[bt]:
                out[int(k)].add((int(plan.batch_job[bt]), n))
    return out


@pytest.mark.parametrize("schedule,K,r,c,m", [("single", 5, 2, 2, 2), ("single", 4, 3, 1, 3),
                                              ("single", 6, 1, 1, 1), ("paper", 4, 2, 2, 2),
                                              ("paper", 5, 3, 1, 1)])
@pytest.mark.parametrize("mode", ["u32", "f32"])
def test_combine_is_the_sum_over_the_shared_batch(schedule, K, r, c, m, mode):
    """vbar_{q,P} = sum of v_{q,n} over the files that all nodes of P store and the
    target does not (Sec. IV-B, pre-combining), for the c functions of the target."""
    p = plan_for(K, r, c, m, schedule)
    T = 6
    V = make_inputs(p, T, mode)
    Vbar = O.combine(p, T, V)
    store = stored_at(p)
    for u in range(p.n_round):
        S = [int(s) for s in p.round_member[u]]
        for b, t in enumerate(S):
            others = [s for s in S if s != t]
            job = int(p.batch_job[p.round_batch[u, b]])
            shared = set.intersection(*[store[s] for s in others]) - store[t]
            shared = sorted(n for (j, n) in shared if j == job)
            assert len(shared) == p.m
            vals = V[job, shared][:, t * c:(t + 1) * c, :].reshape(p.m, c * T)
            want = np.bitwise_xor.reduce(vals, axis=0) if mode == "u32" else vals.astype(np.float64).sum(axis=0)
            assert np.array_equal(Vbar[u, b], want)


@pytest.mark.parametrize("K,r,c,T", [(3, 2, 1, 8), (4, 2, 2, 12), (5, 3, 1, 12), (5, 4, 1, 16), (4, 1, 1, 4)])
@pytest.mark.parametrize("mode", ["u32", "f32"])
def test_encode_matches_label_brute_force(K, r, c, T, mode):
    """X_k = sum over the r-subsets P of the group that contain k of V_{P,k}, where
    V_P = (V_{P,i_1}, ..., V_{P,i_r}) is cut evenly and labelled by P's members in
    ascending order (Sec. IV-B, split and coded-packet equations).  Sizes with r | W."""
    p = plan_for(K, r, c, 1, "single")
    W = c * T
    assert W % (4 * r) == 0 or W % r == 0
    if W % (4 * r) != 0:
        pytest.skip("exact split needs 4r | W in this reading")
    V = make_inputs(p, T, mode)
    Vbar = O.combine(p, T, V)
    X = O.encode(p, T, Vbar)
    seg = W // r
    assert X.shape[-1] == seg
    for u in range(p.n_round):
        S = [int(s) for s in p.round_member[u]]
        labelled = {}                                   # (P, node label) -> segment
        for b, t in enumerate(S):
            P = tuple(s for s in S if s != t)
            for i, node in enumerate(P):
                labelled[(P, node)] = Vbar[u, b, i * seg:(i + 1) * seg]
        for a, k in enumerate(S):
            parts = [labelled[(P, k)] for P in combinations(S, r) if k in P]
            assert len(parts) == r
            want = np.bitwise_xor.reduce(parts, axis=0) if mode == "u32" else np.sum(parts, axis=0)
            assert np.array_equal(X[u, a], want)


@pytest.mark.parametrize("K,r,T", [(4, 2, 10), (5, 3, 7), (4, 3, 9), (6, 2, 5)])
def test_single_bit_of_a_packet_reaches_exactly_one_coded_word(K, r, T):
    """Flipping one bit of Vbar[u][b][e] flips that bit in exactly one word of X:
    position e mod ell of the packet sent by the node labelling the segment."""
    p = plan_for(K, r, 1, 1, "single")
    V = make_inputs(p, T, "u32")
    Vbar = O.combine(p, T, V)
    X0 = O.encode(p, T, Vbar)
    ell = O.segment_len(T, r)
    rng = np.random.default_rng(5)
    for _ in range(40):
        u, b, e = int(rng.integers(p.n_round)), int(rng.integers(r + 1)), int(rng.integers(T))
        Vb = Vbar.copy()
        Vb[u, b, e] ^= np.uint32(1 << 7)
        diff = O.encode(p, T, Vb) ^ X0
        S = [int(s) for s in p.round_member[u]]
        P = [s for s in S if s != S[b]]
        sender = S.index(P[e // ell])                   # node whose label the segment carries
        assert np.count_nonzero(diff) == 1
        assert diff[u, sender, e % ell] == 1 << 7


@pytest.mark.parametrize("mode", ["u32", "f32"])
def test_decode_uses_only_what_the_receiver_stores(mode):
    """Receiver b must get its packet from the coded packets and from packets of
    batches it stores (Sec. IV-B, decoding); overwriting the packets meant for b
    with garbage must not change what b decodes."""
    p = O.build_plan(5, 3, 5, 20)
    T = 10
    V = make_inputs(p, T, mode)
    Vbar = O.combine(p, T, V)
    X = O.encode(p, T, Vbar)
    D = O.decode(p, T, X, Vbar)
    assert np.array_equal(D, Vbar)
    for b in range(p.r + 1):
        poisoned = Vbar.copy()
        poisoned[:, b, :] = 12345
        assert np.array_equal(O.decode(p, T, X, poisoned)[:, b, :], Vbar[:, b, :])
    # and it does need the coded packets: a changed X changes the result
    X2 = X.copy()
    X2[0, 1, 0] = X2[0, 1, 0] + 1 if mode == "f32" else X2[0, 1, 0] ^ np.uint32(1)
    assert not np.array_equal(O.decode(p, T, X2, Vbar), D)


def test_reduce_adds_local_values_and_decoded_packets():
    """With D forced to zero, reduce must give exactly the sum over the files the
    reducer itself stores (Sec. IV-B: 'together with the local Map results')."""
    p = O.build_plan(5, 2, 10, 20)
    T = 4
    V = make_inputs(p, T, "f32")
    D0 = np.zeros(p.shapes(T)["D"])
    Phi = O.reduce(p, T, V, D0)
    store = stored_at(p)
    for k in range(p.K):
        mine = sorted(n for (_, n) in store[k])
        want = V[0, mine][:, k * p.c:(k + 1) * p.c, :].astype(np.float64).sum(axis=0)
        assert np.array_equal(Phi[0, k * p.c:(k + 1) * p.c], want)
    # a unit packet decoded by (round u, member b) lands on that member's functions only
    D1 = D0.copy()
    D1[3, 1, :] = 1.0
    delta = O.reduce(p, T, V, D1) - Phi
    k = int(p.round_member[3, 1])
    want = np.zeros_like(delta)
    want[0, k * p.c:(k + 1) * p.c] = 1.0
    assert np.array_equal(delta, want)


def test_stages_are_linear_in_xor_mode():
    p = O.build_plan(4, 2, 4, 12)
    T = 9
    A = generate_numpy(1, p.N, p.Q, T, 11, "u32")
    B = generate_numpy(1, p.N, p.Q, T, 12, "u32")
    ra, rb, rab = O.run_all(p, T, A), O.run_all(p, T, B), O.run_all(p, T, A ^ B)
    for name in ("Vbar", "X", "D", "Phi"):
        assert np.array_equal(ra[name] ^ rb[name], rab[name]), name


def test_ragged_tail_is_zero_padded():
    """When r does not divide W the coded packets keep stride ell and the words a
    sender has nothing to put in are the zero of the algebra."""
    p = O.build_plan(4, 3, 4, 4)
    T = 10                                              # ell = 4, segments 4,4,2
    V = make_inputs(p, T, "u32")
    art = O.run_all(p, T, V)
    assert art["X"].shape == (1, 4, 4)
    assert [O.packet_len(T, 3, a) for a in range(4)] == [4, 4, 4, 2]
    assert (art["X"][0, 3, 2:] == 0).all()
    assert np.array_equal(art["Phi"], O.direct(p, T, V))


# ------------------------------------------- "h32": real sums, XOR-coded packets

def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


@pytest.mark.parametrize("schedule,K,r,c,m,T", [("single", 3, 2, 1, 2, 8), ("single", 5, 2, 2, 3, 6), ("single", 4, 3, 1, 2, 10),
                                                ("single", 6, 1, 1, 1, 5), ("paper", 4, 2, 1, 2, 12), ("paper", 5, 3, 2, 1, 7)])
def test_h32_recovers_the_combined_packets_bit_for_bit(schedule, K, r, c, m, T):
    """Sec. II: packets are pre-combined by summing, coded by bit-wise XOR, and every
    node decodes 'the intended pre-combined packet' - for real-valued data the
    decoded bits must be exactly the combined packet's, not just close."""
    p = plan_for(K, r, c, m, schedule)
    V = generate_numpy(p.J, p.N, p.Q, T, 21, "f32")
    art = O.run_all_h32(p, T, V)
    assert art["Vbar"].dtype == np.float32 and art["X"].dtype == np.uint32 and art["D"].dtype == np.float32
    assert np.array_equal(bits(art["D"]), bits(art["Vbar"]))
    ref = O.direct(p, T, V)
    assert np.abs(art["Phi"] - ref).max() <= 1e-6 * np.abs(ref).max()
    if p.m == 1:                                   # nothing is rounded: only the order of fp64 adds differs
        assert np.abs(art["Phi"] - ref).max() <= 1e-12 * np.abs(ref).max()


def test_h32_combine_is_the_fp32_sum_in_file_order():
    p = O.build_plan(4, 2, 8, 18)                  # m = 3, c = 2
    T = 5
    V = generate_numpy(1, p.N, p.Q, T, 4, "f32")
    Vbar = O.run_all_h32(p, T, V)["Vbar"]
    for u in range(p.n_round):
        for b in range(p.r + 1):
            t = int(p.round_member[u, b])
            f0 = int(p.batch_file0[p.round_batch[u, b]])
            acc = V[0, f0, t * p.c:(t + 1) * p.c].reshape(-1).copy()
            for n in range(f0 + 1, f0 + p.m):
                acc = (acc + V[0, n, t * p.c:(t + 1) * p.c].reshape(-1)).astype(np.float32)
            assert np.array_equal(bits(Vbar[u, b]), bits(acc))


def test_h32_coded_packet_is_the_xor_of_labelled_segment_bits():
    p = O.build_plan(4, 2, 4, 12)
    T = 8
    V = generate_numpy(1, p.N, p.Q, T, 6, "f32")
    art = O.run_all_h32(p, T, V)
    seg = T // p.r
    for u in range(p.n_round):
        S = [int(s) for s in p.round_member[u]]
        labelled = {}
        for b, t in enumerate(S):
            P = tuple(s for s in S if s != t)
            for i, node in enumerate(P):
                labelled[(P, node)] = bits(art["Vbar"][u, b, i * seg:(i + 1) * seg])
        for a, k in enumerate(S):
            parts = [labelled[(P, k)] for P in combinations(S, p.r) if k in P]
            assert np.array_equal(art["X"][u, a], np.bitwise_xor.reduce(parts, axis=0))


def test_h32_agrees_with_the_real_algebra_on_exact_inputs():
    """Integer-valued inputs: every sum is exact in fp32 and fp64, so the two
    algebras must give the same packets and the same outputs."""
    p = O.build_plan(5, 2, 5, 20)
    T = 9
    V = make_inputs(p, T, "f32")
    h, f = O.run_all_h32(p, T, V), O.run_all(p, T, V)
    assert np.array_equal(h["Vbar"].astype(np.float64), f["Vbar"])
    assert np.array_equal(h["D"].astype(np.float64), f["D"])
    assert np.array_equal(h["Phi"], f["Phi"])
    # but the coded packets differ in kind: XOR of patterns is not the pattern of the sum
    assert not np.array_equal(h["X"], bits(f["X"].astype(np.float32)))


@pytest.mark.parametrize("mode", ["u32", "f32"])
def test_repeated_scheme_recovers_every_output(mode):
    """gamma repetitions on consecutive blocks of jobs (Sec. IV): every job's outputs are eq. (1)."""
    p = O.build_plan(4, 2, 8, 6, "paper", gamma=3)
    assert p.J == 12
    V = make_inputs(p, 5, mode, seed=77)
    art = O.run_all(p, 5, V)
    assert np.array_equal(art["Phi"], O.direct(p, 5, V)) and np.array_equal(art["D"], art["Vbar"])


# ---------------------------------------------------------------- sampling a schedule

@pytest.mark.parametrize("K,r,c,m,T,schedule", [(5, 2, 1, 1, 12, "single"), (6, 3, 2, 2, 10, "single"),
                                                 (4, 2, 1, 2, 7, "paper"), (5, 2, 2, 1, 9, "paper")])
def test_a_plan_of_selected_rounds_gives_the_parents_rows(K, r, c, m, T, schedule):
    """orc_plan_select_rounds keeps the batches and takes the listed rounds, in the order
    listed: its tables are the parent's rows, and every artefact of the stages run on it
    (Vbar, X, D) equals the parent's artefact at those rounds, in both algebras.  Repeats
    and arbitrary order are allowed; a bad index is refused."""
    from math import comb
    nb = (r + 1) if schedule == "paper" else comb(K, r)
    while m * nb < K:
        m += 1
    plan = O.build_plan(K, r, c * K, m * nb, schedule)
    rng = np.random.default_rng(K * 100 + r)
    rounds = rng.permutation(plan.n_round)[: max(1, plan.n_round // 2)].tolist()
    rounds += [rounds[0], plan.n_round - 1, 0]                       # repeats, last and first
    sub = O.select_rounds(plan, rounds)
    assert (sub.K, sub.r, sub.Q, sub.N, sub.J, sub.c, sub.m, sub.n_batch) == \
           (plan.K, plan.r, plan.Q, plan.N, plan.J, plan.c, plan.m, plan.n_batch)
    assert sub.n_round == len(rounds)
    for name in ("batch_job", "batch_file0", "batch_label"):
        assert np.array_equal(getattr(sub, name), getattr(plan, name)), name
    assert np.array_equal(sub.round_member, plan.round_member[rounds])
    assert np.array_equal(sub.round_batch, plan.round_batch[rounds])
    for dtype in (np.uint32, np.float32):
        if dtype == np.uint32:
            V = rng.integers(0, 2 ** 32, size=plan.shapes(T)["V"], dtype=np.uint64).astype(np.uint32)
        else:
            V = rng.integers(-50, 50, size=plan.shapes(T)["V"]).astype(np.float32)
        full = O.run_all(plan, T, V)
        vb = O.combine(sub, T, V)
        xs = O.encode(sub, T, vb)
        ds = O.decode(sub, T, xs, vb)
        assert np.array_equal(vb, full["Vbar"][rounds])
        assert np.array_equal(xs, full["X"][rounds])
        assert np.array_equal(ds, full["D"][rounds])
    if plan.J == 1:
        h = O.run_all_h32(plan, T, V)
        hs = O.run_all_h32(sub, T, V)
        for name in ("Vbar", "X", "D"):
            assert np.array_equal(hs[name].view(np.uint32), h[name].view(np.uint32)[rounds]), name
    assert O.select_rounds(plan, []).n_round == 0
    for bad in ([-1], [plan.n_round], [0, plan.n_round + 5]):
        with pytest.raises(ValueError):
            O.select_rounds(plan, bad)
