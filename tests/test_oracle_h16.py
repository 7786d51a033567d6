"""Pins of the oracle's hybrid algebra for 16-bit floating-point payloads
("h16": numbers are summed, packets are XOR-coded bit patterns, Sec. II):
the two format conversions against numpy's float16 and torch's bfloat16, the
stages against library sums and a set-labelled brute force, bit-exact
recovery, and agreement with the real algebra where every sum is exact.
CPU only, tiny sizes."""
from itertools import combinations
from math import comb

import numpy as np
import pytest
import torch

import oracle as O
from workloads import generate_numpy, half_bits_to_float, to_half_bits

FORMATS = ["bf16", "f16"]


def lib_widen(bits, fmt):
    """Independent conversion: numpy's float16, torch's bfloat16."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if fmt == "f16":
        return bits.view(np.float16).astype(np.float32)
    return torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).float().numpy()


def lib_narrow(values, fmt):
    values = np.ascontiguousarray(values, dtype=np.float32)
    if fmt == "f16":
        with np.errstate(over="ignore"):
            return values.astype(np.float16).view(np.uint16)
    return torch.from_numpy(values.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def plan_for(K, r, c, m, schedule):
    nb = comb(K, r) if schedule == "single" else r + 1
    while m * nb < K:
        m += 1
    return O.build_plan(K, r, c * K, m * nb, schedule)


# ------------------------------------------------------------- conversions

@pytest.mark.parametrize("fmt", FORMATS)
def test_widen_every_pattern(fmt):
    bits = np.arange(65536, dtype=np.uint16)
    got, want = O.h16_widen(bits, fmt), lib_widen(bits, fmt)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))      # signed zeros included


@pytest.mark.parametrize("fmt", FORMATS)
def test_narrow_inverts_widen(fmt):
    bits = np.arange(65536, dtype=np.uint16)
    vals = O.h16_widen(bits, fmt)
    ok = ~np.isnan(vals)
    assert np.array_equal(O.h16_narrow(vals[ok], fmt), bits[ok])


@pytest.mark.parametrize("fmt", FORMATS)
def test_narrow_rounds_to_nearest_even(fmt):
    rng = np.random.default_rng(5)
    scales = [1e-9, 6e-8, 1e-6, 6.1e-5, 1e-3, 1.0, 37.0, 3e4, 65504.0, 7e4, 1e30]
    vals = np.concatenate([(s * rng.standard_normal(4000)).astype(np.float32) for s in scales])
    # every value half way between two neighbours of the format, and its fp32 neighbours
    bits = np.arange(0, 0x7C00 if fmt == "f16" else 0x7F80, dtype=np.uint16)
    lo, hi = O.h16_widen(bits[:-1], fmt).astype(np.float64), O.h16_widen(bits[1:], fmt).astype(np.float64)
    mid = ((lo + hi) / 2).astype(np.float32)
    assert np.array_equal(mid.astype(np.float64), (lo + hi) / 2)                 # the ties are exact in fp32
    ties = np.concatenate([mid, np.nextafter(mid, np.float32(np.inf)), np.nextafter(mid, np.float32(0))])
    edge = np.array([0.0, -0.0, 65504.0, 65519.99, 65520.0, 65536.0, np.inf, -np.inf, 3.3895314e38, 3.4e38,
                     5.9604645e-08, 2.9802322e-08, 2.98e-08, 6.1035156e-05, 6.0975552e-05, 1e-45], dtype=np.float32)
    allv = np.concatenate([vals, ties, -ties, edge, -edge])
    got, want = O.h16_narrow(allv, fmt), lib_narrow(allv, fmt)
    assert np.array_equal(got, want)
    # a tie goes to the neighbour whose last fraction bit is 0
    tied = O.h16_narrow(mid, fmt)
    assert ((tied & 1) == 0).all() and ((tied == bits[:-1]) | (tied == bits[1:])).all()
    nan = O.h16_narrow(np.array([np.nan], dtype=np.float32), fmt)
    assert np.isnan(lib_widen(nan, fmt)).all()


@pytest.mark.parametrize("fmt", FORMATS)
def test_generator_patterns_are_the_rounded_fp32_payload(fmt):
    f = generate_numpy(1, 3, 4, 50, 9, "f32")
    h = generate_numpy(1, 3, 4, 50, 9, fmt)
    assert h.dtype == np.uint16 and np.array_equal(h, O.h16_narrow(f, fmt)) and np.array_equal(h, to_half_bits(f, fmt))
    assert np.array_equal(half_bits_to_float(h, fmt).view(np.uint32), O.h16_widen(h, fmt).view(np.uint32))
    t = torch.from_numpy(f).to(torch.bfloat16 if fmt == "bf16" else torch.float16)
    assert np.array_equal(t.view(torch.int16).numpy().view(np.uint16), h)


# ------------------------------------------------------------------ stages

CASES = [("single", 3, 2, 1, 2, 8), ("single", 5, 2, 2, 3, 6), ("single", 4, 3, 1, 2, 10), ("single", 6, 1, 1, 1, 5),
         ("paper", 4, 2, 1, 2, 12), ("paper", 5, 3, 2, 1, 7)]


@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("schedule,K,r,c,m,T", CASES)
def test_h16_recovers_the_combined_packets_bit_for_bit(fmt, schedule, K, r, c, m, T):
    """Every receiver decodes exactly the bits of the packet pre-combined for it
    (Sec. II), and every output is the plain sum (eq. (1)) up to the one rounding of
    each received packet."""
    p = plan_for(K, r, c, m, schedule)
    V = generate_numpy(p.J, p.N, p.Q, T, 21, fmt)
    art = O.run_all_h16(p, T, V, fmt)
    assert all(art[k].dtype == np.uint16 for k in ("Vbar", "X", "D")) and art["Phi"].dtype == np.float64
    assert np.array_equal(art["D"], art["Vbar"])
    ref = O.direct_h16(p, T, V, fmt)
    assert np.array_equal(ref, half_bits_to_float(V, fmt).astype(np.float64).sum(axis=1))
    half_ulp = 2.0 ** -8 if fmt == "bf16" else 2.0 ** -11     # 7 / 10 fraction bits
    received = comb(K - 1, r) * (1 if schedule == "single" else K - r)      # packets a node decodes per job
    bound = received * half_ulp * np.abs(O.h16_widen(art["Vbar"], fmt)).max() * 1.0001
    assert np.abs(art["Phi"] - ref).max() <= bound
    if p.m == 1:                                   # a one-file batch is sent as it is: nothing is rounded
        assert np.abs(art["Phi"] - ref).max() <= 1e-12 * np.abs(ref).max()


@pytest.mark.parametrize("fmt", FORMATS)
def test_h16_combine_is_the_fp32_sum_in_file_order_rounded_once(fmt):
    p = O.build_plan(4, 2, 8, 30)                  # m = 5, c = 2
    T = 5
    V = generate_numpy(1, p.N, p.Q, T, 4, fmt)
    Vf = lib_widen(V, fmt)
    Vbar = O.run_all_h16(p, T, V, fmt)["Vbar"]
    twice = 0
    for u in range(p.n_round):
        for b in range(p.r + 1):
            t = int(p.round_member[u, b])
            f0 = int(p.batch_file0[p.round_batch[u, b]])
            acc = Vf[0, f0, t * p.c:(t + 1) * p.c].reshape(-1).copy()
            each = lib_narrow(acc, fmt)
            for n in range(f0 + 1, f0 + p.m):
                nxt = Vf[0, n, t * p.c:(t + 1) * p.c].reshape(-1)
                acc = (acc + nxt).astype(np.float32)
                each = lib_narrow(lib_widen(each, fmt) + nxt, fmt)
            assert np.array_equal(Vbar[u, b], lib_narrow(acc, fmt))
            twice += int((each != Vbar[u, b]).sum())
    assert twice > 0            # rounding after every addition would give other bits: the pin can tell


@pytest.mark.parametrize("fmt", FORMATS)
def test_h16_coded_packet_is_the_xor_of_labelled_segment_bits(fmt):
    p = O.build_plan(4, 2, 4, 12)
    T = 8
    V = generate_numpy(1, p.N, p.Q, T, 6, fmt)
    art = O.run_all_h16(p, T, V, fmt)
    seg = T // p.r
    for u in range(p.n_round):
        S = [int(s) for s in p.round_member[u]]
        labelled = {}
        for b, t in enumerate(S):
            P = tuple(s for s in S if s != t)
            for i, node in enumerate(P):
                labelled[(P, node)] = art["Vbar"][u, b, i * seg:(i + 1) * seg]
        for a, k in enumerate(S):
            parts = [labelled[(P, k)] for P in combinations(S, p.r) if k in P]
            assert np.array_equal(art["X"][u, a], np.bitwise_xor.reduce(parts, axis=0))


@pytest.mark.parametrize("fmt", FORMATS)
def test_h16_agrees_with_the_real_algebra_on_exact_inputs(fmt):
    """Small integers: every sum is exact in the 16-bit format, in fp32 and in fp64,
    so the packets and outputs equal those of the real algebra."""
    p = O.build_plan(5, 2, 5, 20)                  # m = 2
    T = 9
    w = generate_numpy(1, p.N, p.Q, T, 2, "u32")
    Vf = ((w % 17).astype(np.int64) - 8).astype(np.float32)          # |sum of 20| <= 160 < 256
    V = to_half_bits(Vf, fmt)
    h, f = O.run_all_h16(p, T, V, fmt), O.run_all(p, T, Vf)
    assert np.array_equal(lib_widen(h["Vbar"], fmt).astype(np.float64), f["Vbar"])
    assert np.array_equal(lib_widen(h["D"], fmt).astype(np.float64), f["D"])
    assert np.array_equal(h["Phi"], f["Phi"]) and np.array_equal(h["Phi"], O.direct(p, T, Vf))


@pytest.mark.parametrize("fmt", FORMATS)
def test_h16_ragged_split(fmt):
    p = O.build_plan(4, 3, 4, 4)                   # r = 3, W = 10: segments 4, 4, 2
    T = 10
    V = generate_numpy(1, p.N, p.Q, T, 8, fmt)
    art = O.run_all_h16(p, T, V, fmt)
    assert art["X"].shape == (1, 4, 4) and (art["X"][0, 3, 2:] == 0).all()
    assert np.array_equal(art["D"], art["Vbar"])


# ------------------------------------------------ special patterns in the payload

CANON_NAN = {"bf16": 0x7FC0, "f16": 0x7E00}
EXP_MASK = {"bf16": 0x7F80, "f16": 0x7C00}
FRAC_MASK = {"bf16": 0x007F, "f16": 0x03FF}


def is_nan_bits(bits, fmt):
    return ((bits & EXP_MASK[fmt]) == EXP_MASK[fmt]) & ((bits & FRAC_MASK[fmt]) != 0)


@pytest.mark.parametrize("fmt", FORMATS)
def test_a_sum_that_is_not_a_number_is_stored_as_the_canonical_nan(fmt):
    """Every NaN the conversion can be handed (any sign, any payload, quiet or signalling)
    comes out as the one quiet pattern with sign and payload clear; infinities keep their
    sign; values past the largest finite one round to infinity."""
    nans = np.array([0x7FC00000, 0xFFC00000, 0x7F800001, 0xFF800001, 0x7FFFFFFF, 0xFFFFFFFF, 0x7FA55555],
                    dtype=np.uint32).view(np.float32)
    assert (O.h16_narrow(nans, fmt) == CANON_NAN[fmt]).all()
    inf = np.array([np.inf, -np.inf], dtype=np.float32)
    assert O.h16_narrow(inf, fmt).tolist() == [EXP_MASK[fmt], 0x8000 | EXP_MASK[fmt]]
    big = np.array([3.4e38, -3.4e38] if fmt == "bf16" else [65520.0, -1e6], dtype=np.float32)
    assert O.h16_narrow(big, fmt).tolist() == [EXP_MASK[fmt], 0x8000 | EXP_MASK[fmt]]


@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("m", [1, 2, 3])
def test_special_patterns_through_the_stages(fmt, m):
    """Payloads holding infinities, NaNs of every kind, subnormals and the largest finite
    values.  One-file batches (m = 1) are not sums: the packet is the file's patterns
    untouched, NaN payloads included.  Longer batches: the fp32 sum of the exact values,
    files ascending, rounded once - checked against numpy / torch doing exactly that in
    their own arithmetic - with every NaN stored as the canonical pattern, sums of opposite
    infinities included, and sums past the format's range stored as infinity.  Coding is on
    patterns, so every receiver recovers every packet bit for bit whatever it holds."""
    from workloads import special_payload
    K, r, c, T = 5, 2, 1, 24
    plan = O.build_plan(K, r, c * K, m * comb(K, r))
    V = special_payload(plan.shapes(T)["V"], fmt, seed=7 * m, density=0.2)
    assert is_nan_bits(V, fmt).any() and (V == EXP_MASK[fmt]).any()
    out = O.run_all_h16(plan, T, V, fmt)
    Vbar, r1 = out["Vbar"], r + 1
    vals = lib_widen(V, fmt)
    saw_nan_sum = False
    for u in range(plan.n_round):
        for b in range(r1):
            target, bt = int(plan.round_member[u, b]), int(plan.round_batch[u, b])
            f0 = int(plan.batch_file0[bt])
            if m == 1:
                assert np.array_equal(Vbar[u, b], V[0, f0, target])              # untouched, pattern for pattern
                continue
            acc = vals[0, f0, target].copy()
            with np.errstate(invalid="ignore", over="ignore"):
                for n in range(f0 + 1, f0 + m):
                    acc = (acc + vals[0, n, target]).astype(np.float32)
            want = lib_narrow(acc, fmt)
            nan = np.isnan(acc)
            assert np.array_equal(Vbar[u, b][~nan], want[~nan])
            assert (Vbar[u, b][nan] == CANON_NAN[fmt]).all()
            saw_nan_sum |= bool(nan.any())
    assert m == 1 or saw_nan_sum
    assert np.array_equal(out["D"], Vbar)                                         # exact recovery of any pattern
    # the final reduction is exact fp64 arithmetic on the values: NaN where a NaN or opposite
    # infinities meet, else the plain sum
    with np.errstate(invalid="ignore"):
        direct = lib_widen(V, fmt).astype(np.float64).sum(axis=1)
    got = out["Phi"]
    if m == 1:
        assert np.array_equal(np.isnan(got), np.isnan(direct))
        ok = ~np.isnan(direct)
        assert np.array_equal(got[ok], direct[ok])


@pytest.mark.parametrize("fmt", FORMATS)
def test_sums_that_leave_the_format(fmt):
    """Two largest finite values add up, in fp32, to a number the format cannot hold:
    the pre-combined packet stores infinity (binary16: 65504 + 65504; bfloat16: the fp32
    sum itself overflows)."""
    top = {"bf16": 0x7F7F, "f16": 0x7BFF}[fmt]
    plan = O.build_plan(3, 2, 3, 6)                                               # m = 2
    T = 4
    V = np.full(plan.shapes(T)["V"], top, dtype=np.uint16)
    V[0, 1::2] = top | 0x8000                                                    # second file of each batch: the negative
    V[0, :, :, 0] = top                                                           # column 0: both positive
    out = O.run_all_h16(plan, T, V, fmt)
    assert (out["Vbar"][..., 0] == EXP_MASK[fmt]).all()                           # +inf
    assert (out["Vbar"][..., 1:] == 0).all()                                      # top + (-top) = +0
