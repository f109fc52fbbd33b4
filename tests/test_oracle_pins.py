"""Pins for the CPU oracle: closed forms, identities of Sections 2.3 and 3, exact rational arithmetic
on tiny inputs, special cases that reduce to an exact product, and the accuracy behaviour the paper
describes.  Everything here runs without a GPU and uses Python integers / Fractions as the independent
arithmetic."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2504_08009_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def paper_moduli_s16():
    with open(os.path.join(GOLDEN, "moduli_s16_paper.txt")) as f:
        for line in f:
            if not line.startswith("#"):
                return [int(x) for x in line.split()]


# ------------------------------------------------------------------ Section 2.1: symmetric modulo
def test_sym_mod_named_values():
    # nearest-to-zero representative; the even modulus sends +p/2 to -p/2
    assert orc.sym_mod(128, 256) == -128
    assert orc.sym_mod(-128, 256) == -128
    assert orc.sym_mod(127, 256) == 127
    assert orc.sym_mod(128, 255) == -127
    assert orc.sym_mod(127, 255) == 127
    assert orc.sym_mod(0, 199) == 0


def test_sym_mod_bruteforce_against_definition():
    # r = a - p*floor(a/p + 1/2) with exact rationals, and the characterisation "closest to zero"
    for p in orc.moduli(26) + [2, 3, 4]:
        for a in list(range(-700, 701)) + [2**40 + 12345, -(2**40) - 777, 2**62 - 1, -(2**62)]:
            want = a - p * math.floor(Fraction(a, p) + Fraction(1, 2))
            got = orc.sym_mod(a, p)
            assert got == want
            assert (got - a) % p == 0 and -p / 2 <= got < p / 2


# ------------------------------------------------------------------ Section 3.1: moduli
def test_moduli_pairwise_coprime_and_greedy():
    mods = orc.moduli(26)
    assert mods[0] == 256 and all(2 <= p <= 256 for p in mods)
    assert mods == sorted(mods, reverse=True)
    for i in range(len(mods)):
        for j in range(i):
            assert math.gcd(mods[i], mods[j]) == 1
    # "largest possible": every skipped value shares a factor with a larger kept one
    for c in range(mods[-1], 257):
        if c not in mods:
            assert any(math.gcd(c, p) != 1 for p in mods if p > c)
    # prefix property: N moduli are the first N of the one table
    assert orc.moduli(7) == mods[:7]


def test_paper_printed_list_properties():
    pm = paper_moduli_s16()
    assert len(pm) == 16 and pm[0] == 256 and pm[-1] == 191
    assert abs(pm[-1] / pm[0] - 0.74) < 0.01  # the ratio the paper quotes
    for i in range(16):
        for j in range(i):
            assert math.gcd(pm[i], pm[j]) == 1
    # the greedy table differs from the printed one only by containing 241
    g = orc.moduli(17)
    assert sorted(set(g) - set(pm)) == [241]


# ------------------------------------------------------------------ Section 2.3: CRT constants
@pytest.mark.parametrize("N", [2, 3, 8, 16, 20, 26])
def test_crt_weights_identities(N):
    mods = orc.moduli(N)
    M, W = orc.crt_constants(N)
    assert M == math.prod(mods)
    for t, p in enumerate(mods):
        assert 0 < W[t] < M
        assert W[t] % p == 1
        assert W[t] % (M // p) == 0
        for u, q in enumerate(mods):
            if u != t:
                assert W[t] % q == 0
    assert sum(W) % M == 1


def test_crt_closed_form_two_moduli():
    M, W = orc.crt_constants(2)
    assert M == 256 * 255 and W == [255 * 255, 256]


def test_crt_round_trip_paper_list():
    pm = paper_moduli_s16()
    M, W = orc.crt_constants(16, pm)
    rng = np.random.default_rng(5)
    for _ in range(200):
        x = int(rng.integers(-2**62, 2**62)) * int(rng.integers(1, 2**60)) % M - M // 2
        y = sum((x % p) * w for p, w in zip(pm, W)) % M
        if y >= M - M // 2:
            y -= M
        assert y == x


# ------------------------------------------------------------------ Section 3: bit budget kappa
def test_kappa_invariant_and_table():
    for N in range(2, 27):
        M, _ = orc.crt_constants(N)
        for k in [1, 2, 255, 256, 1024, 4096, 16384, 65536, 2**17]:
            kap = orc.kappa(N, k)
            if kap < 0:
                assert k > M // 2 - 1
                continue
            assert k * 4**kap <= M // 2 - 1 < k * 4 ** (kap + 1)
            # same number from the printed formula, evaluated with exact integer logarithms
            assert kap == (((M // 2 - 1) // k).bit_length() - 1) // 2
    assert [orc.kappa(N, 1024) for N in range(8, 21)] == [26, 30, 34, 38, 41, 45, 49, 53, 57, 60, 64, 68, 72]


def test_kappa_sixteen_moduli_reach_53_bits():
    # Section 3.1: with s = 16 the budget reaches 53 bits for p = q = r in {1024, 4096, 16384};
    # fifteen moduli do not at every size.  Holds for the greedy table and for the printed list.
    pm = paper_moduli_s16()
    sizes = [1024, 4096, 16384]
    assert min(orc.kappa(16, k) for k in sizes) >= 53
    assert min(orc.kappa(15, k) for k in sizes) < 53
    assert min(orc.kappa(16, k, pm) for k in sizes) >= 53
    assert min(orc.kappa(15, k, pm[:15]) for k in sizes) < 53


def test_int32_exactness_limit():
    # Section 3.1: no INT32 overflow for q < 2^17
    assert (2**17 - 1) * 128 * 128 < 2**31 <= 2**17 * 128 * 128


# ------------------------------------------------------------------ Algorithm 1 on tiny inputs, exact arithmetic
def _tiny(seed, m, n, k, phi):
    rng = np.random.default_rng(seed)
    A = (rng.random((m, k)) - 0.5) * np.exp(phi * rng.standard_normal((m, k)))
    B = (rng.random((k, n)) - 0.5) * np.exp(phi * rng.standard_normal((k, n)))
    return A, B


@pytest.mark.parametrize("N,phi,use_paper_list", [(3, 0.5, False), (8, 0.5, False), (14, 1.0, False),
                                                  (16, 0.5, True), (20, 4.0, False), (26, 4.0, False)])
def test_every_step_against_exact_rationals(N, phi, use_paper_list):
    m, n, k = 5, 4, 7
    A, B = _tiny(100 + N, m, n, k, phi)
    A[2, 3] = 0.0
    mods = paper_moduli_s16() if use_paper_list else orc.moduli(N)
    M = math.prod(mods)
    kap = orc.kappa(N, k, mods)
    r = orc.dgemm(A, B, N, mods=mods, want=("C", "shifts", "Ap", "Bp", "Ares", "Bres", "Cprod", "Cres", "X"))

    # line 1: the row/column maximum lands in [2^(kappa-1), 2^kappa)
    for i in range(m):
        mx = max(abs(Fraction(float(x))) for x in A[i, :]) * Fraction(2) ** int(r.sa[i])
        assert Fraction(2) ** (kap - 1) <= mx < Fraction(2) ** kap
    for j in range(n):
        mx = max(abs(Fraction(float(x))) for x in B[:, j]) * Fraction(2) ** int(r.sb[j])
        assert Fraction(2) ** (kap - 1) <= mx < Fraction(2) ** kap

    # lines 2-3: truncation toward zero of the exactly scaled value
    for i in range(m):
        for l in range(k):
            assert r.Ap[i][l] == math.trunc(Fraction(float(A[i, l])) * Fraction(2) ** int(r.sa[i]))
    for l in range(k):
        for j in range(n):
            assert r.Bp[l][j] == math.trunc(Fraction(float(B[l, j])) * Fraction(2) ** int(r.sb[j]))

    # uniqueness premise of Section 3: (|A'||B'|)_ij < M/2
    for i in range(m):
        for j in range(n):
            assert sum(abs(r.Ap[i][l]) * abs(r.Bp[l][j]) for l in range(k)) < M // 2

    for t, p in enumerate(mods):
        for i in range(m):
            for l in range(k):
                a = int(r.Ares[t, i, l])
                assert (a - r.Ap[i][l]) % p == 0 and -p / 2 <= a < p / 2 and -128 <= a <= 127
        for j in range(n):
            for l in range(k):
                b = int(r.Bres[t, j, l])
                assert (b - r.Bp[l][j]) % p == 0 and -p / 2 <= b < p / 2
        for i in range(m):
            for j in range(n):
                # line 6 and the congruence of Section 2.3
                cp = sum(int(r.Ares[t, i, l]) * int(r.Bres[t, j, l]) for l in range(k))
                assert int(r.Cprod[t, i, j]) == cp
                exact_ij = sum(r.Ap[i][l] * r.Bp[l][j] for l in range(k))
                assert int(r.Cres[t, i, j]) == exact_ij % p  # line 7, floor-mod in [0, p)

    # lines 8-10: the CRT recovers the integer product itself
    for i in range(m):
        for j in range(n):
            exact_ij = sum(r.Ap[i][l] * r.Bp[l][j] for l in range(k))
            assert r.X[i][j] == exact_ij
            # line 11: one correctly rounded conversion, then an exact scaling
            want = float(Fraction(exact_ij, 1) / Fraction(2) ** (int(r.sa[i]) + int(r.sb[j])))
            assert r.C[i, j] == want


def test_subnormal_inputs_are_decomposed_exactly():
    # Section 2.1 assumes no underflow; the oracle still has to read subnormal inputs for what they are: the
    # shift comes from floor(log2) of the row maximum and the truncation acts on the exact value (a subnormal has
    # no hidden bit and the fixed exponent -1074).  Rationals are the independent arithmetic.
    m, n, k, N = 4, 3, 6, 14
    A, B = _tiny(77, m, n, k, 0.5)
    A[0] *= 2.0**-1040            # a row of subnormals only
    A[1, ::2] *= 2.0**-1065       # subnormals mixed into a normal row (some vanish under truncation)
    A[2, 1] = 5e-324              # the smallest subnormal
    B[:, 1] *= 2.0**-1030         # a subnormal column
    B[0, 2] = -2.0**-1074
    assert np.any((A != 0) & (np.abs(A) < 2.0**-1022)) and np.any((B != 0) & (np.abs(B) < 2.0**-1022))
    kap = orc.kappa(N, k)
    r = orc.dgemm(A, B, N, want=("C", "shifts", "Ap", "Bp", "X"))
    for i in range(m):
        mx = max(abs(Fraction(float(x))) for x in A[i, :])
        e = mx.numerator.bit_length() - mx.denominator.bit_length()
        e = e if Fraction(2) ** e <= mx else e - 1            # floor(log2 mx) from the exact rational
        assert Fraction(2) ** e <= mx < Fraction(2) ** (e + 1)
        assert int(r.sa[i]) == kap - 1 - e
        for l in range(k):
            assert r.Ap[i][l] == math.trunc(Fraction(float(A[i, l])) * Fraction(2) ** int(r.sa[i]))
    for j in range(n):
        mx = max(abs(Fraction(float(x))) for x in B[:, j])
        e = mx.numerator.bit_length() - mx.denominator.bit_length()
        e = e if Fraction(2) ** e <= mx else e - 1
        assert int(r.sb[j]) == kap - 1 - e
        for l in range(k):
            assert r.Bp[l][j] == math.trunc(Fraction(float(B[l, j])) * Fraction(2) ** int(r.sb[j]))
    for i in range(m):
        for j in range(n):
            assert r.X[i][j] == sum(r.Ap[i][l] * r.Bp[l][j] for l in range(k))


def test_results_in_the_subnormal_range_are_rounded_to_53_bits_and_then_scaled():
    # Algorithm 1 line 11 read as FP64 arithmetic would carry it out: X is rounded to FP64 once (53 bits, nearest
    # even), then multiplied by the power of two 2^-(sa+sb).  Above the subnormal range the scaling is exact and the
    # result is the correctly rounded X 2^-(sa+sb); below it the scaling is a second rounding (the IEEE result of
    # that multiplication).  Python's int -> float conversion and math.ldexp are the independent implementations
    # of the two steps; X itself is pinned against the integer product above.
    m, n, k, N = 6, 6, 5, 12
    differs = 0
    landed = 0
    for seed in range(40):
        A, B = _tiny(500 + seed, m, n, k, 0.5)
        A *= 2.0**-510
        B *= 2.0**-(510 + seed % 24)   # results from just below 2^-1022 (one bit lost) down to 30 bits lost
        r = orc.dgemm(A, B, N, want=("C", "shifts", "X"))
        for i in range(m):
            for j in range(n):
                s = int(r.sa[i]) + int(r.sb[j])
                x = r.X[i][j]
                want = math.ldexp(float(x), -s)
                assert r.C[i, j] == want and math.copysign(1.0, r.C[i, j]) == math.copysign(1.0, want)
                landed += 0.0 < abs(want) < 2.0**-1022
                differs += want != float(Fraction(x, 2**s))   # one rounding of the exact quotient
    assert landed > 1000 and differs < landed
    # the two readings really differ on some elements, so this test tells them apart
    assert differs > 0


def test_small_integer_matrices_are_multiplied_exactly():
    # |a|,|b| < 2^10 and k*2^20 < 2^53: nothing is truncated once kappa >= 11, so C == A B exactly
    rng = np.random.default_rng(7)
    m, n, k = 9, 11, 33
    A = rng.integers(-1023, 1024, (m, k)).astype(np.float64)
    B = rng.integers(-1023, 1024, (k, n)).astype(np.float64)
    A[:, 0] = 1023.0  # make every row/column maximum sit in the same binade
    B[0, :] = 1023.0
    want = (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float64)
    for N in [5, 8, 16]:
        assert orc.kappa(N, k) >= 11
        assert np.array_equal(orc.dgemm(A, B, N).C, want)


def test_large_moduli_count_gives_correctly_rounded_product():
    # When kappa exceeds 53 plus the exponent spread of every row/column nothing is truncated and the
    # result is the exact product rounded once.
    m, n, k = 6, 5, 16
    A, B = _tiny(11, m, n, k, 0.5)
    N = 26
    r = orc.dgemm(A, B, N, want=("C", "shifts"))
    for i in range(m):
        for j in range(n):
            s = sum(Fraction(float(A[i, l])) * Fraction(float(B[l, j])) for l in range(k))
            assert r.C[i, j] == float(s)


def test_zero_rows_columns_and_k_zero():
    A, B = _tiny(3, 4, 3, 6, 0.5)
    A[1, :] = 0.0
    B[:, 2] = 0.0
    r = orc.dgemm(A, B, 10, want=("C", "shifts"))
    assert r.sa[1] == 0 and r.sb[2] == 0
    assert np.all(r.C[1, :] == 0.0) and np.all(r.C[:, 2] == 0.0)
    r0 = orc.dgemm(np.zeros((3, 0)), np.zeros((0, 2)), 10)
    assert r0.C.shape == (3, 2) and np.all(r0.C == 0.0)


def test_subset_equals_full():
    A, B = _tiny(21, 12, 10, 20, 1.0)
    full = orc.dgemm(A, B, 12).C
    rows, cols = [11, 0, 5], [9, 3]
    sub = orc.dgemm(A, B, 12, rows=rows, cols=cols).C
    assert np.array_equal(sub, full[np.ix_(rows, cols)])


def test_exact_reference_against_fractions():
    A, B = _tiny(31, 4, 3, 50, 2.0)
    C, S = orc.exact(A, B)
    for i in range(4):
        for j in range(3):
            s = sum(Fraction(float(A[i, l])) * Fraction(float(B[l, j])) for l in range(50))
            sa = sum(abs(Fraction(float(A[i, l])) * Fraction(float(B[l, j]))) for l in range(50))
            assert C[i, j] == float(s) and S[i, j] == float(sa)


# ------------------------------------------------------------------ accuracy behaviour (Sections 3 and 4.1)
def test_error_bound_and_decay_with_moduli():
    cfg = inputs.CONFIGS["c2"]
    k = cfg["k"]
    rows = np.arange(0, 1024, 16)
    cols = np.arange(3, 1024, 16)
    A = inputs.block(cfg["seed"], 0, cfg["m"], k, cfg["phi"], row_idx=rows)
    B = inputs.block(cfg["seed"], 1, k, cfg["n"], cfg["phi"], col_idx=cols)
    Cx, S = orc.exact(A, B)
    native = np.max(np.abs(A @ B - Cx) / S)
    errs = {}
    for N in range(8, 21):
        r = orc.dgemm(A, B, N, want=("C", "shifts"))
        err = np.abs(r.C - Cx)
        # truncation bound from the scaling equations: each a' differs from a*2^sa by less than one unit;
        # plus one final rounding of the result and one of the reference
        sumA = np.sum(np.abs(A), axis=1)[:, None]
        sumB = np.sum(np.abs(B), axis=0)[None, :]
        ea = np.ldexp(1.0, -r.sa.astype(np.int64))[:, None]
        eb = np.ldexp(1.0, -r.sb.astype(np.int64))[None, :]
        bound = ea * sumB + eb * sumA + k * ea * eb + 2.0**-53 * (np.abs(r.C) + np.abs(Cx))
        assert np.all(err <= bound * (1 + 1e-12))
        errs[N] = float(np.max(err / S))
    # error falls monotonically until it reaches the final-rounding floor
    for N in range(9, 21):
        assert errs[N] <= errs[N - 1] * 1.0001 or errs[N] < 2.0**-52
    assert errs[8] > 1e-9 and errs[20] < 2.0**-53 * 1.01
    # Section 4.1: at phi = 0.5 fourteen or fifteen moduli reach the accuracy of native FP64
    assert errs[13] > native
    assert errs[15] <= 2 * native
    assert errs[16] < native


def test_planted_mistakes_are_caught_by_the_pins():
    # a Python model of the CRT step with a wrong weight, a wrong sign convention or a missing modulus
    # fails the identity X == A'B'; this guards the pins themselves against being vacuous
    A, B = _tiny(41, 3, 3, 5, 0.5)
    N = 6
    mods = orc.moduli(N)
    M, W = orc.crt_constants(N)
    r = orc.dgemm(A, B, N, want=("Ap", "Bp", "Cres", "X"))

    def rebuild(weights, residues, symmetric=True):
        out = []
        for i in range(3):
            row = []
            for j in range(3):
                y = sum(int(residues[t, i, j]) * weights[t] for t in range(N)) % M
                if symmetric and y >= M - M // 2:
                    y -= M
                row.append(y)
            out.append(row)
        return out

    assert rebuild(W, r.Cres) == r.X
    bad_w = list(W)
    bad_w[2] += M // mods[2]
    assert rebuild(bad_w, r.Cres) != r.X
    assert rebuild(W, r.Cres, symmetric=False) != r.X
    shifted = r.Cres.copy()
    shifted[1] = (shifted[1].astype(np.int64) + 1) % mods[1]
    assert rebuild(W, shifted) != r.X


def test_hand_worked_example_three_moduli():
    # A 2 x 2 x 2 product small enough to follow with pencil and paper (Algorithm 1 with the moduli 256, 255,
    # 253: M = 16515840, kappa = 10 for k = 2).  Every number below follows from the definitions:
    # e.g. 512 = trunc(1.0 * 2^9), 153 = trunc(0.3 * 2^9), 153 mod 256 = -103 (symmetric), 5253 = (-103)(-51),
    # 5253 mod 256 = 133, and X = A'B' = [[512*358 + 153*(-563), 512*768], [-640*358, -640*768]].
    A = np.array([[1.0, 0.3], [-2.5, 1e-3]])
    B = np.array([[0.7, 3.0], [-1.1, 0.001]])
    assert orc.moduli(3) == [256, 255, 253] and orc.kappa(3, 2) == 10
    M, W = orc.crt_constants(3)
    assert M == 16515840 and [int(w) for w in W] == [64515 * 171, 64768 * 127, 65280 * 211]
    r = orc.dgemm(A, B, 3, want=("C", "shifts", "Ap", "Bp", "Ares", "Bres", "Cprod", "Cres", "X"))
    assert r.sa.tolist() == [9, 8] and r.sb.tolist() == [9, 8]
    assert r.Ap == [[512, 153], [-640, 0]] and r.Bp == [[358, 768], [-563, 0]]
    assert r.Ares[0].tolist() == [[0, -103], [-128, 0]]                 # rows of A' modulo 256
    assert r.Bres[0].tolist() == [[102, -51], [0, 0]]                   # columns of B' modulo 256
    assert r.Cprod.tolist() == [[[5253, 0], [-13056, 0]], [[5612, 6], [12875, 375]], [[6330, 54], [12495, 1071]]]
    assert r.Cres.tolist() == [[[133, 0], [0, 0]], [[2, 6], [125, 120]], [[5, 54], [98, 59]]]
    assert r.X == [[97157, 393216], [-229120, -491520]]
    assert r.X == [[512 * 358 + 153 * -563, 512 * 768], [-640 * 358, -640 * 768]]
    assert r.C.tolist() == [[97157 / 2.0**18, 3.0], [-229120 / 2.0**17, -7.5]]


# ------------------------------------------------------------------ Section 4.1: Cauchy-Schwarz shift selection
@pytest.mark.parametrize("N,phi", [(4, 0.5), (10, 1.0), (16, 0.5), (20, 4.0), (26, 4.0)])
def test_cauchy_schwarz_shifts_are_rigorous_and_maximal(N, phi):
    m, n, k = 6, 5, 9
    A, B = _tiny(500 + N, m, n, k, phi)
    A[1, :] = 0.0
    A[2, 1:] = 0.0            # a single nonzero: the norm equals the maximum
    mods = orc.moduli(N)
    M = math.prod(mods)
    beta = orc.beta(N)
    assert 4**beta <= M // 2 - 1 < 4 ** (beta + 1)
    r = orc.dgemm(A, B, N, mode=1, want=("C", "shifts", "Ap", "Bp", "X"))
    assert r.sa[1] == 0

    def check(vec, s):
        sq = sum(Fraction(float(x)) ** 2 for x in vec)
        if sq == 0:
            return
        # 2^s * ||vec||_2 <= 2^beta, compared on the squares with exact rationals
        assert sq * Fraction(4) ** int(s) <= Fraction(4) ** beta
        # maximal for the integer norm bound: with e, q, S, h as defined in the oracle's header
        e = max(math.frexp(abs(float(x)))[1] - 1 for x in vec if x != 0)
        S = sum(math.ceil(abs(Fraction(float(x))) * Fraction(2) ** (19 - e)) ** 2 for x in vec)
        h = 0
        while 4**h < S:
            h += 1
        assert s == beta - (e - 19 + h)
        assert 4 ** (h - 1) < S                       # h is the smallest such exponent
        assert sq <= Fraction(4) ** (e - 19) * S      # the integer norm bound is an upper bound

    for i in range(m):
        check(A[i, :], r.sa[i])
    for j in range(n):
        check(B[:, j], r.sb[j])
    # uniqueness premise and exact reconstruction still hold
    for i in range(m):
        for j in range(n):
            ex = sum(r.Ap[i][l] * r.Bp[l][j] for l in range(k))
            assert sum(abs(r.Ap[i][l]) * abs(r.Bp[l][j]) for l in range(k)) < M // 2
            assert r.X[i][j] == ex
            assert r.C[i, j] == float(Fraction(ex) / Fraction(2) ** (int(r.sa[i]) + int(r.sb[j])))
    # truncation toward zero with these shifts
    for i in range(m):
        for l in range(k):
            assert r.Ap[i][l] == math.trunc(Fraction(float(A[i, l])) * Fraction(2) ** int(r.sa[i]))


def test_cauchy_schwarz_reaches_native_accuracy_with_14_or_15_moduli():
    # Section 4.1: at phi = 0.5 the variants the paper measures need 14 or 15 moduli for the accuracy of
    # native FP64; the Cauchy-Schwarz shifts are never smaller than the simple ones by more than the
    # norm/max ratio allows and the error is smaller at every moduli count below the rounding floor
    cfg = inputs.CONFIGS["c2"]
    k = cfg["k"]
    rows = np.arange(0, 1024, 16)
    cols = np.arange(3, 1024, 16)
    A = inputs.block(cfg["seed"], 0, cfg["m"], k, cfg["phi"], row_idx=rows)
    B = inputs.block(cfg["seed"], 1, k, cfg["n"], cfg["phi"], col_idx=cols)
    Cx, S = orc.exact(A, B)
    native = np.max(np.abs(A @ B - Cx) / S)
    err = {}
    for N in (10, 12, 13, 14, 15):
        e0 = np.max(np.abs(orc.dgemm(A, B, N).C - Cx) / S)
        e1 = np.max(np.abs(orc.dgemm(A, B, N, mode=1).C - Cx) / S)
        assert e1 < e0
        err[N] = e1
    assert err[13] > native
    assert err[15] < native
    assert err[14] < 4 * native


# ------------------------------------------------------------------ Section 4.1: INT8-product shift selection
@pytest.mark.parametrize("N,phi", [(4, 0.5), (10, 1.0), (16, 0.5), (20, 4.0), (26, 4.0)])
def test_int8_product_shifts_are_rigorous_and_tight(N, phi):
    m, n, k = 7, 6, 11
    A, B = _tiny(700 + N, m, n, k, phi)
    A[1, :] = 0.0
    B[:, 2] = 0.0
    A[3, 0] = 5e-324 if phi > 1 else A[3, 0]      # a subnormal entry still needs a bound of at least one unit
    mods = orc.moduli(N)
    M = math.prod(mods)
    b = orc.log2_budget(N)
    assert 2**b <= M // 2 - 1 < 2 ** (b + 1)
    r = orc.dgemm(A, B, N, mode=2, want=("C", "shifts", "Ap", "Bp", "X"))
    assert r.sa[1] == 0 and r.sb[2] == 0

    def expo(vec):
        return max(math.frexp(abs(float(x)))[1] - 1 for x in vec if x != 0)

    # the 6-bit upper bounds and their product, from exact rationals
    ea = [expo(A[i, :]) if np.any(A[i, :]) else 0 for i in range(m)]
    fb = [expo(B[:, j]) if np.any(B[:, j]) else 0 for j in range(n)]
    A2 = [[math.ceil(abs(Fraction(float(A[i, l]))) * Fraction(2) ** (5 - ea[i])) for l in range(k)] for i in range(m)]
    B2 = [[math.ceil(abs(Fraction(float(B[l, j]))) * Fraction(2) ** (5 - fb[j])) for j in range(n)] for l in range(k)]
    assert max(max(row) for row in A2) <= 64 and max(max(row) for row in B2) <= 64
    P = [[sum(A2[i][l] * B2[l][j] for l in range(k)) for j in range(n)] for i in range(m)]
    for i in range(m):
        R = max(P[i])
        if R == 0:
            continue
        u = int(r.sa[i]) + ea[i] - 5
        # tight: the row's largest bound, scaled by 4^u, lands in the top two bits of the budget
        assert Fraction(2) ** (b - 2) < Fraction(4) ** u * R <= Fraction(2) ** b
    for j in range(n):
        Cm = max(P[i][j] for i in range(m))
        if Cm == 0:
            continue
        v = int(r.sb[j]) + fb[j] - 5
        assert Fraction(2) ** (b - 2) < Fraction(4) ** v * Cm <= Fraction(2) ** b
    # rigorous: the uniqueness premise of Section 3 on the truncated integers themselves, and the bound chain
    for i in range(m):
        for j in range(n):
            absprod = sum(abs(r.Ap[i][l]) * abs(r.Bp[l][j]) for l in range(k))
            bound = Fraction(2) ** (int(r.sa[i]) + ea[i] - 5 + int(r.sb[j]) + fb[j] - 5) * P[i][j]
            assert absprod <= bound <= M // 2 - 1
            ex = sum(r.Ap[i][l] * r.Bp[l][j] for l in range(k))
            assert r.X[i][j] == ex
            assert r.C[i, j] == float(Fraction(ex) / Fraction(2) ** (int(r.sa[i]) + int(r.sb[j])))
    for i in range(m):
        for l in range(k):
            assert r.Ap[i][l] == math.trunc(Fraction(float(A[i, l])) * Fraction(2) ** int(r.sa[i]))


def test_int8_product_shifts_subset_and_accuracy():
    # the maxima run over all rows and columns: a subset call must give the shifts of the full call; the
    # bound is never worse than a few bits below the Cauchy-Schwarz one and the error at 14 moduli is at the
    # level of native FP64 (Section 4.1: both variants need 14 or 15 moduli at phi = 0.5)
    cfg = inputs.CONFIGS["c1"]
    m, n, k = cfg["m"], cfg["n"], cfg["k"]
    A = inputs.block(cfg["seed"], 0, m, k, cfg["phi"])
    B = inputs.block(cfg["seed"], 1, k, n, cfg["phi"])
    full = orc.dgemm(A, B, 14, mode=2, want=("C", "shifts"))
    rows, cols = np.array([0, 5, 77, 255]), np.array([3, 128, 254])
    sub = orc.dgemm(A, B, 14, mode=2, rows=rows, cols=cols, want=("C", "shifts"))
    assert np.array_equal(sub.sa, full.sa[rows]) and np.array_equal(sub.sb, full.sb[cols])
    assert np.array_equal(sub.C, full.C[np.ix_(rows, cols)])
    Cx, S = orc.exact(A, B)
    native = np.max(np.abs(A @ B - Cx) / S)
    e2 = np.max(np.abs(full.C - Cx) / S)
    e1 = np.max(np.abs(orc.dgemm(A, B, 14, mode=1).C - Cx) / S)
    e0 = np.max(np.abs(orc.dgemm(A, B, 14).C - Cx) / S)
    assert e2 < e0 and e2 < 4 * e1 and e2 < 4 * native


def test_blas_update_against_rationals():
    # C := alpha * P + beta * C: one rounding of beta*C, then a fused multiply-add; beta == 0 ignores C
    A, B = _tiny(61, 4, 3, 6, 0.5)
    C0 = np.asfortranarray(np.random.default_rng(1).standard_normal((4, 3)))
    P = orc.dgemm(A, B, 12).C
    for alpha, beta in [(1.0, 0.0), (0.75, -1.25), (-3.0, 1.0), (1e-3, 7.0), (0.0, 0.5), (2.0, 0.0)]:
        got = orc.dgemm_ex("N", "N", alpha, A, B, beta, C0, 12)
        for i in range(4):
            for j in range(3):
                t = 0.0 if beta == 0.0 else float(Fraction(beta) * Fraction(float(C0[i, j])))
                want = float(Fraction(alpha) * Fraction(float(P[i, j])) + Fraction(t))
                assert got[i, j] == want
    Cn = np.full((4, 3), np.nan, order="F")
    assert np.array_equal(orc.dgemm_ex("N", "N", 1.0, A, B, 0.0, Cn, 12), P)
    # transposes only change how the operands are read
    assert np.array_equal(orc.dgemm_ex("T", "N", 1.0, np.asfortranarray(A.T), B, 0.0, Cn, 12), P)
    assert np.array_equal(orc.dgemm_ex("N", "T", 1.0, A, np.asfortranarray(B.T), 0.0, Cn, 12), P)


# ------------------------------------------------------------------ Section 3.1, closing remark: exceptional values
def test_native_fallback_follows_ieee_rules_and_the_textbook_sum():
    inf, nan = float("inf"), float("nan")
    A, B = _tiny(91, 5, 4, 7, 0.5)
    # finite inputs: within the classical bound k * 2^-53 * (|A||B|) of the exact product
    P = orc.native_gemm(A, B)
    for i in range(5):
        for j in range(4):
            ex = sum(Fraction(float(A[i, l])) * Fraction(float(B[l, j])) for l in range(7))
            ab = sum(abs(Fraction(float(A[i, l])) * Fraction(float(B[l, j]))) for l in range(7))
            assert abs(Fraction(float(P[i, j])) - ex) <= 7 * Fraction(2) ** -53 * ab
    assert not orc.has_nonfinite(A) and not orc.has_nonfinite(B)
    # special values, by the rules of IEEE 754 arithmetic
    A2 = A.copy()
    B2 = B.copy()
    A2[0, 2] = inf              # row 0: inf * b_2j decides the sign unless b_2j == 0 (inf * 0 = NaN)
    B2[2, 1] = 0.0
    A2[1, 3] = nan              # row 1: NaN everywhere
    A2[2, 0], A2[2, 1] = inf, inf   # row 2: inf * b_0j + inf * b_1j: NaN when the signs differ
    B2[0, :] = [1.0, 1.0, -2.0, 3.0]
    B2[1, :] = [1.0, -1.0, -5.0, 0.5]
    assert orc.has_nonfinite(A2) and not orc.has_nonfinite(B2)
    P2 = orc.native_gemm(A2, B2)
    for j in range(4):
        if B2[2, j] == 0.0:
            assert math.isnan(P2[0, j])
        else:
            assert P2[0, j] == math.copysign(inf, B2[2, j])
        assert math.isnan(P2[1, j])
    assert P2[2, 0] == inf and math.isnan(P2[2, 1]) and P2[2, 2] == -inf and P2[2, 3] == inf
    # rows without exceptional values are what the finite product gives
    P_fin = orc.native_gemm(A, B2)
    assert np.array_equal(P2[3:, :], P_fin[3:, :])
    # the BLAS-form oracle switches to this product exactly when an input is not finite
    C0 = np.zeros((5, 4), order="F")
    assert np.array_equal(orc.dgemm_ex("N", "N", 1.0, A2, B2, 0.0, C0, 12), P2, equal_nan=True)
    assert np.array_equal(orc.dgemm_ex("N", "N", 1.0, A, B, 0.0, C0, 12), orc.dgemm(A, B, 12).C)
    At = np.asfortranarray(A2.T)
    assert np.array_equal(orc.dgemm_ex("T", "N", 1.0, At, B2, 0.0, C0, 12), P2, equal_nan=True)


# ------------------------------------------------------------------ Section 2.3: structured products (SYRK shape)
def _with_signed_zeros(seed, m, n, k):
    rng = np.random.default_rng(seed)
    A = (rng.random((m, k)) - 0.5) * np.exp(rng.standard_normal((m, k)))
    B = (rng.random((k, n)) - 0.5) * np.exp(rng.standard_normal((k, n)))
    A[rng.random((m, k)) < 0.2] = -0.0
    A[rng.random((m, k)) < 0.1] = 0.0
    B[rng.random((k, n)) < 0.2] = -0.0
    A[1, :] = -0.0                 # a row of negative zeros: every product of that row is a zero
    A[2, :] = 0.0
    A[2, ::2] = -0.0               # zeros of both signs
    B[:, 1] = -0.0
    B[:, 3] = np.where(B[:, 3] < 0, -0.0, B[:, 3])
    A[4, :] = np.where(np.arange(k) % 2 == 0, -0.0, 1.0)   # the non-zero entries meet only zeros of column 5
    B[:, 5] = np.where(np.arange(k) % 2 == 0, -3.0, -0.0)
    return np.asfortranarray(A), np.asfortranarray(B)


def test_signed_zeros_in_the_inputs_change_nothing():
    # Section 3.1 (closing remark) names signed zeros among the values that need separate handling.  For a
    # product whose sums start from +0 they need none: in round-to-nearest (+0) + (-0) = +0 and x + (-x) = +0, so
    # a sum of products that are all zero is +0 whatever their signs, and a zero term never changes a non-zero
    # sum.  Pinned here on the FP64 routine the fallback stands for (its zeros are all +0, and replacing every
    # -0 of the inputs by +0 leaves every bit of its result as it is) and on the emulation (same statement):
    # there is nothing a detection of -0 could route differently.
    m, n, k, N = 9, 8, 12, 12
    A, B = _with_signed_zeros(9, m, n, k)
    assert np.signbit(A[A == 0]).any() and np.signbit(B[B == 0]).any()
    Ap, Bp = A + 0.0, B + 0.0      # x + (+0): -0 becomes +0, everything else is unchanged
    assert not np.signbit(Ap[Ap == 0]).any() and np.array_equal(A, Ap)
    P, Pp = orc.native_gemm(A, B), orc.native_gemm(Ap, Bp)
    assert np.array_equal(P.view(np.uint64), Pp.view(np.uint64))
    assert (P == 0).sum() >= m + n - 1 and not np.signbit(P[P == 0]).any()
    # exact rationals agree on where the zeros are
    for i in range(m):
        for j in range(n):
            s = sum(Fraction(float(A[i, l])) * Fraction(float(B[l, j])) for l in range(k))
            assert (s == 0) == (P[i, j] == 0) or abs(s) < Fraction(1, 2**60)
    C, Cp = orc.dgemm(A, B, N).C, orc.dgemm(Ap, Bp, N).C
    assert np.array_equal(C.view(np.uint64), Cp.view(np.uint64))
    assert not np.signbit(C[C == 0]).any() and np.array_equal(C == 0, P == 0)
    # the BLAS update: alpha * (+0) + (+0) is +0 for either sign of alpha; beta * C keeps the sign IEEE gives it
    C0 = np.asfortranarray(np.where(np.arange(m * n).reshape(m, n) % 3 == 0, -0.0, 1.5))
    for alpha, beta in [(-0.5, 0.0), (-0.5, 2.0), (1.0, -1.0)]:
        U = orc.dgemm_ex("N", "N", alpha, A, B, beta, C0, N)
        for i in range(m):
            for j in range(n):
                if C[i, j] == 0.0:          # the product is an exact zero: alpha * (+0) + t with IEEE signs
                    want = alpha * 0.0 + (0.0 if beta == 0.0 else beta * C0[i, j])
                    assert U[i, j] == want and np.signbit(U[i, j]) == np.signbit(want)


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_symmetric_product_is_exactly_symmetric_and_touches_one_triangle(mode):
    # A' A'^T is a symmetric integer matrix and the shifts of its columns are those of its rows, so the
    # emulated product of (A, A^T) is symmetric bit for bit; the update only writes the named triangle
    A, _ = _tiny(33, 9, 2, 13, 1.0)
    P = orc.dgemm(A, A.T, 12, mode=mode, want=("C", "shifts"))
    assert np.array_equal(P.C, P.C.T) and np.array_equal(P.sa, P.sb)
    C0 = np.asfortranarray(np.random.default_rng(3).standard_normal((9, 9)))
    for uplo in "LU":
        for trans, As in (("N", A), ("T", np.asfortranarray(A.T))):
            got = orc.dsyrk(uplo, trans, 0.5, As, -2.0, C0, 12, mode=mode)
            for i in range(9):
                for j in range(9):
                    inside = i >= j if uplo == "L" else i <= j
                    if inside:
                        t = float(Fraction(-2.0) * Fraction(float(C0[i, j])))
                        assert got[i, j] == float(Fraction(0.5) * Fraction(float(P.C[i, j])) + Fraction(t))
                    else:
                        assert got[i, j] == C0[i, j]


# ------------------------------------------------------------------ Section 2.3: structured products (TRMM shape)
def test_triangular_product_reads_one_triangle_and_is_exact_on_integers():
    rng = np.random.default_rng(17)
    m, n = 7, 5
    for side in "LR":
        ka = m if side == "L" else n
        for uplo in "LU":
            for transa in "NT":
                for diag in "NU":
                    A = rng.integers(-50, 50, (ka, ka)).astype(np.float64)
                    B = rng.integers(-50, 50, (m, n)).astype(np.float64)
                    # the triangle seen by the routine, as Python integers
                    T = [[0] * ka for _ in range(ka)]
                    for r in range(ka):
                        for c in range(ka):
                            if (r > c and uplo == "L") or (r < c and uplo == "U"):
                                T[r][c] = int(A[r, c])
                            elif r == c:
                                T[r][c] = 1 if diag == "U" else int(A[r, c])
                    if transa == "T":
                        T = [[T[c][r] for c in range(ka)] for r in range(ka)]
                    Bi = [[int(B[i, j]) for j in range(n)] for i in range(m)]
                    if side == "L":
                        want = [[-3 * sum(T[i][l] * Bi[l][j] for l in range(m)) for j in range(n)] for i in range(m)]
                    else:
                        want = [[-3 * sum(Bi[i][l] * T[l][j] for l in range(n)) for j in range(n)] for i in range(m)]
                    # what is not referenced may hold anything
                    G = A.copy()
                    for r in range(ka):
                        for c in range(ka):
                            if (r < c and uplo == "L") or (r > c and uplo == "U") or (r == c and diag == "U"):
                                G[r, c] = np.nan
                    got = orc.dtrmm(side, uplo, transa, diag, -3.0, G, B, 10)
                    assert got.tolist() == [[float(v) for v in row] for row in want]
    assert np.array_equal(orc.dtrmm("L", "U", "N", "N", 0.0, np.full((m, m), np.nan), B, 10), np.zeros((m, n)))


# ------------------------------------------------------------------ Section 3: unequal bit budgets k_A != k_B
@pytest.mark.parametrize("N,k,delta", [(8, 9, 3), (8, 9, -5), (13, 9, 7), (14, 1024, 10), (5, 3, 1)])
def test_unequal_bit_budgets_keep_the_premise_and_use_the_whole_sum(N, k, delta):
    m, n = 5, 4
    A, B = _tiny(900 + N, m, n, k, 1.0)
    mods = orc.moduli(N)
    M = math.prod(mods)
    S, kap = orc.kappa_sum(N, k), orc.kappa(N, k)
    assert k * 2**S <= M // 2 - 1 < k * 2 ** (S + 1) and S in (2 * kap, 2 * kap + 1)
    ka, kb = kap - delta, S - (kap - delta)
    r = orc.dgemm(A, B, N, delta=delta, want=("C", "shifts", "Ap", "Bp", "X"))
    for i in range(m):
        assert 2 ** (ka - 1) <= max(abs(v) for v in r.Ap[i]) < 2**ka
    for j in range(n):
        assert 2 ** (kb - 1) <= max(abs(r.Bp[l][j]) for l in range(k)) < 2**kb
    for i in range(m):
        for j in range(n):
            assert sum(abs(r.Ap[i][l]) * abs(r.Bp[l][j]) for l in range(k)) <= M // 2 - 1
            ex = sum(r.Ap[i][l] * r.Bp[l][j] for l in range(k))
            assert r.X[i][j] == ex
            assert r.C[i, j] == float(Fraction(ex) / Fraction(2) ** (int(r.sa[i]) + int(r.sb[j])))
    # the other two shift selections: the premise holds for the same delta
    for mode in (1, 2):
        q = orc.dgemm(A, B, N, mode=mode, delta=delta, want=("shifts", "Ap", "Bp", "X"))
        z = orc.dgemm(A, B, N, mode=mode, want=("shifts",))
        assert np.array_equal(q.sa, z.sa - delta) and np.all(q.sb >= z.sb + delta) and np.all(q.sb <= z.sb + delta + 1)
        for i in range(m):
            for j in range(n):
                assert sum(abs(q.Ap[i][l]) * abs(q.Bp[l][j]) for l in range(k)) <= M // 2 - 1
                assert q.X[i][j] == sum(q.Ap[i][l] * q.Bp[l][j] for l in range(k))


def test_unequal_bit_budgets_serve_operands_of_different_precision():
    # A holds single-precision values within one binade per row (24 significant bits, no spread), B full doubles:
    # A needs 25 bits of budget and no more, so moving the rest to B gives with 12 moduli the accuracy that the
    # equal split only reaches with more moduli.  (With a wide spread inside the rows of A the truncation of its
    # small entries costs 2^-k_A of the row maximum whatever their own precision, and the equal split is best.)
    m, n, k = 64, 48, 256
    rng = np.random.default_rng(5)
    A = (np.where(rng.random((m, k)) < 0.5, -1.0, 1.0) * (0.5 + 0.5 * rng.random((m, k)))).astype(np.float32).astype(np.float64)
    B = (rng.random((k, n)) - 0.5) * np.exp(0.5 * rng.standard_normal((k, n)))
    Cx, S = orc.exact(A, B)
    err = lambda C: np.max(np.abs(C - Cx) / S)
    kap = orc.kappa(12, k)
    assert kap - 8 >= 25
    e_equal = err(orc.dgemm(A, B, 12).C)
    e_split = err(orc.dgemm(A, B, 12, delta=8).C)
    e_more = err(orc.dgemm(A, B, 14).C)
    assert e_split < e_equal / 50 and e_split < 4 * e_more
    # A is not truncated at all with this budget
    r = orc.dgemm(A[:4], B[:, :3], 12, delta=8, want=("shifts", "Ap"))
    for i in range(4):
        for l in range(k):
            assert Fraction(r.Ap[i][l]) == Fraction(float(A[i, l])) * Fraction(2) ** int(r.sa[i])
