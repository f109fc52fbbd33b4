"""GPU parity on seeded random problems: shapes, moduli counts, shift modes, transposes, scalars, leading dimensions
and the form of the INT8 products are drawn at random; every result must be bit-identical with the oracle."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2504_08009_amd as oz
from oracle import oracle as orc


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x.T)).cuda().t()


def _draw(rng):
    big = rng.random() < 0.25
    hi = 1400 if big else 300
    m, n, k = (int(rng.integers(1, hi + 1)) for _ in range(3))
    N = int(rng.integers(2, 27))
    mode = int(rng.integers(0, 3))
    # a budget of at least one bit
    while orc.kappa(N, k) < 1:
        N += 1
    phi = float(rng.choice([0.5, 1.0, 4.0]))
    ta, tb = (str(rng.choice(["N", "T"])) for _ in range(2))
    alpha, beta = ((1.0, 0.0) if rng.random() < 0.5 else (float(rng.normal()), float(rng.normal())))
    algorithm = int(rng.choice([oz.OZ2_GEMM_CLASSICAL, oz.OZ2_GEMM_STRASSEN]))
    pad = tuple(int(v) for v in rng.integers(0, 4, size=3))
    return m, n, k, N, mode, phi, ta, tb, alpha, beta, algorithm, pad


@pytest.mark.parametrize("seed", range(160))
def test_random_problem_is_bit_identical_with_the_oracle(seed):
    rng = np.random.default_rng(7000 + seed)
    m, n, k, N, mode, phi, ta, tb, alpha, beta, algorithm, pad = _draw(rng)
    opA = (rng.random((m, k)) - 0.5) * np.exp(phi * rng.standard_normal((m, k)))
    opB = (rng.random((k, n)) - 0.5) * np.exp(phi * rng.standard_normal((k, n)))
    # a few structural extremes: zero rows / columns, tiny and huge rows
    if m > 3:
        opA[int(rng.integers(m))] = 0.0
        opA[int(rng.integers(m))] *= 2.0**-300
    if n > 3:
        opB[:, int(rng.integers(n))] = 0.0
        opB[:, int(rng.integers(n))] *= 2.0**200
    As = np.asfortranarray(opA.T if ta == "T" else opA)
    Bs = np.asfortranarray(opB.T if tb == "T" else opB)
    lda, ldb, ldc = As.shape[0] + pad[0], Bs.shape[0] + pad[1], m + pad[2]
    Abig = np.full((lda, As.shape[1]), np.nan, order="F")
    Abig[:As.shape[0]] = As
    Bbig = np.full((ldb, Bs.shape[1]), np.nan, order="F")
    Bbig[:Bs.shape[0]] = Bs
    C0 = np.asfortranarray(rng.standard_normal((m, n)))
    if beta == 0.0:
        C0[:] = np.nan
    Cbig = np.full((ldc, n), 3.0, order="F")
    Cbig[:m] = C0
    dA, dB, dC = _dev(Abig), _dev(Bbig), _dev(Cbig)
    print("seed %d: m=%d n=%d k=%d N=%d mode=%d phi=%g op=%s%s alpha=%g beta=%g algorithm=%d ld+%s"
          % (seed, m, n, k, N, mode, phi, ta, tb, alpha, beta, algorithm, pad), flush=True)
    oz.oz2_set_gemm_algorithm(algorithm)
    oz.oz2_set_shift_mode(mode)
    try:
        ws = oz.Workspace(m, n, k, N)
        oz.oz2_dgemm_ex(ta, tb, m, n, k, alpha, dA.data_ptr(), lda, dB.data_ptr(), ldb, beta, dC.data_ptr(), ldc, N)
        torch.cuda.synchronize()
    finally:
        oz.oz2_set_gemm_algorithm(oz.OZ2_GEMM_AUTO)
        oz.oz2_set_shift_mode(0)
    got = dC.cpu().numpy()
    ref = orc.dgemm_ex(ta, tb, alpha, As, Bs, beta, C0, N, mode=mode)
    assert np.array_equal(got[:m], ref)
    assert np.all(got[m:] == 3.0)
    del ws


@pytest.mark.parametrize("seed", range(60))
def test_random_structured_problem_is_bit_identical_with_the_oracle(seed):
    """Symmetric rank-k updates and in-place triangular products with random shapes and options."""
    rng = np.random.default_rng(9000 + seed)
    N = int(rng.integers(4, 27))
    mode = int(rng.integers(0, 3))
    phi = float(rng.choice([0.5, 1.0, 4.0]))
    hi = 700 if rng.random() < 0.3 else 260
    oz.oz2_set_shift_mode(mode)
    try:
        if seed % 2 == 0:
            n, k = int(rng.integers(1, hi + 1)), int(rng.integers(1, hi + 1))
            while orc.kappa(N, k) < 1:
                N += 1
            uplo, trans = str(rng.choice(["L", "U"])), str(rng.choice(["N", "T"]))
            alpha, beta = float(rng.normal()), float(rng.choice([0.0, 1.0, rng.normal()]))
            opA = (rng.random((n, k)) - 0.5) * np.exp(phi * rng.standard_normal((n, k)))
            As = np.asfortranarray(opA.T if trans == "T" else opA)
            lda, ldc = As.shape[0] + int(rng.integers(0, 3)), n + int(rng.integers(0, 3))
            Abig = np.full((lda, As.shape[1]), np.nan, order="F")
            Abig[:As.shape[0]] = As
            C0 = np.asfortranarray(rng.standard_normal((n, n)))
            ii, jj = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
            outside = (ii < jj) if uplo == "L" else (ii > jj)
            Cbig = np.full((ldc, n), -2.0, order="F")
            Cbig[:n] = np.where(outside, np.nan, C0)        # the other triangle is never read or written
            dA, dC = _dev(Abig), _dev(Cbig)
            print("seed %d: dsyrk %s%s n=%d k=%d N=%d mode=%d phi=%g alpha=%g beta=%g" % (seed, uplo, trans, n, k, N, mode, phi, alpha, beta),
                  flush=True)
            ws = oz.Workspace(n, n, k, N)
            oz.oz2_dsyrk(uplo, trans, n, k, alpha, dA.data_ptr(), lda, beta, dC.data_ptr(), ldc, N)
            torch.cuda.synchronize()
            got = dC.cpu().numpy()
            ref = orc.dsyrk(uplo, trans, alpha, As, beta, np.asfortranarray(np.where(outside, 0.0, C0)), N, mode=mode)
            assert np.all(np.isnan(got[:n][outside])) and np.all(got[n:] == -2.0)
            assert np.array_equal(got[:n][~outside], ref[~outside])
        else:
            m, n = int(rng.integers(1, hi + 1)), int(rng.integers(1, hi + 1))
            side, uplo = str(rng.choice(["L", "R"])), str(rng.choice(["L", "U"]))
            transa, diag = str(rng.choice(["N", "T"])), str(rng.choice(["N", "U"]))
            ka = m if side == "L" else n
            while orc.kappa(N, ka) < 1:
                N += 1
            alpha = float(rng.normal())
            A = (rng.random((ka, ka)) - 0.5) * np.exp(phi * rng.standard_normal((ka, ka)))
            B = np.asfortranarray((rng.random((m, n)) - 0.5) * np.exp(phi * rng.standard_normal((m, n))))
            G = A.copy()                                    # NaN wherever the routine must not look
            ii, jj = np.meshgrid(np.arange(ka), np.arange(ka), indexing="ij")
            G[(ii < jj) if uplo == "L" else (ii > jj)] = np.nan
            if diag == "U":
                G[np.arange(ka), np.arange(ka)] = np.nan
            G = np.asfortranarray(G)
            ldb = m + int(rng.integers(0, 3))
            hB = np.full((ldb, n), 7.0, order="F")
            hB[:m] = B
            dA, dB = _dev(G), _dev(hB)
            print("seed %d: dtrmm %s%s%s%s m=%d n=%d N=%d mode=%d phi=%g alpha=%g" % (seed, side, uplo, transa, diag, m, n, N, mode, phi, alpha),
                  flush=True)
            ws = oz.Workspace(m, n, ka, N)
            oz.oz2_dtrmm(side, uplo, transa, diag, m, n, alpha, dA.data_ptr(), ka, dB.data_ptr(), ldb, N)
            torch.cuda.synchronize()
            got = dB.cpu().numpy()
            ref = orc.dtrmm(side, uplo, transa, diag, alpha, G, B, N, mode=mode)
            assert np.array_equal(got[:m], ref) and np.all(got[m:] == 7.0)
        del ws
    finally:
        oz.oz2_set_shift_mode(0)


@pytest.mark.parametrize("algorithm", [0, 1])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_subnormal_inputs_match_the_oracle(algorithm, mode):
    """Rows and columns of subnormal numbers, subnormals mixed into normal rows, and a huge column: the shifts come
    from the bit patterns of the maxima, so nothing special happens; the results (some of them subnormal or zero
    after the final scaling) are the oracle's."""
    rng = np.random.default_rng(5)
    m, n, k, N = 70, 50, 90, 14
    A = np.asfortranarray((rng.random((m, k)) - 0.5) * np.exp(rng.standard_normal((m, k))))
    B = np.asfortranarray((rng.random((k, n)) - 0.5) * np.exp(rng.standard_normal((k, n))))
    A[3] *= 2.0**-1040
    A[5, ::2] *= 2.0**-1060
    B[:, 7] *= 2.0**-1030
    B[:, 9] *= 2.0**600
    assert np.any((A != 0) & (np.abs(A) < 2.0**-1022)) and np.any((B != 0) & (np.abs(B) < 2.0**-1022))
    oz.oz2_set_gemm_algorithm(algorithm)
    oz.oz2_set_shift_mode(mode)
    try:
        ws = oz.Workspace(m, n, k, N)
        C = oz.dgemm(_dev(A), _dev(B), N, workspace=ws)
        torch.cuda.synchronize()
    finally:
        oz.oz2_set_gemm_algorithm(oz.OZ2_GEMM_AUTO)
        oz.oz2_set_shift_mode(0)
    got, ref = C.cpu().numpy(), orc.dgemm(A, B, N, mode=mode).C
    # bit patterns: a result that underflows keeps its sign, zero included
    assert np.array_equal(got.view(np.uint64), ref.view(np.uint64))
    assert np.any((ref != 0) & (np.abs(ref) < 2.0**-1022))
    del ws
