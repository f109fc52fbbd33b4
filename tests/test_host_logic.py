"""CPU-only tests of the product library: it loads, exports every symbol that include/oz2.h declares,
validates arguments, computes the same host constants as the oracle, and its exact-arithmetic element
routines (the same source the kernels use, compiled for the host) agree with Python big integers on
random and adversarial inputs.  No GPU call is made here."""
import ctypes
import math
import os
import random
import re

import numpy as np
import pytest

import paper_2504_08009_amd as oz
from oracle import oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "oz2.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(oz2_[a-z0-9_]+)\s*\(", header))
    assert len(declared) >= 14
    lib = oz.lib()
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(oz.binding.SYMBOLS)


def test_moduli_and_kappa_match_the_oracle():
    assert oz.min_moduli() == 2 and oz.max_moduli() == 26
    for N in range(2, 27):
        for k in (1, 7, 256, 1024, 4096, 16384, 65536, 1 << 20):
            mods, kap = oz.get_moduli(N, k)
            assert mods == orc.moduli(N)
            assert kap == orc.kappa(N, k)


def test_moduli_for_bits_matches_the_papers_statement():
    # Section 3.1: sixteen moduli give 53 bits for all of the inner dimensions 1024, 4096 and 16384, fifteen
    # only for the first
    assert [oz.moduli_for_bits(k, 53) for k in (1024, 4096, 16384)] == [15, 16, 16]
    assert [orc.kappa(15, k) for k in (1024, 4096, 16384)] == [53, 52, 51]
    assert [orc.kappa(16, k) for k in (1024, 4096, 16384)] == [57, 56, 55]
    for k, bits in [(1, 1), (100, 24), (65536, 53), (10**6, 40)]:
        N = oz.moduli_for_bits(k, bits)
        assert orc.kappa(N, k) >= bits and (N == 2 or orc.kappa(N - 1, k) < bits)
    assert oz.moduli_for_bits(16384, 200) == 0
    assert oz.lib().oz2_moduli_for_bits(0, 53) == -1 and oz.lib().oz2_moduli_for_bits(5, 0) == -2


def test_argument_validation_without_gpu():
    L = oz.lib()
    assert L.oz2_get_moduli(1, None, None, 5) == -1
    assert L.oz2_get_moduli(27, None, None, 5) == -1
    assert L.oz2_get_moduli(5, None, None, 0) == -4
    assert oz.workspace_bytes(-1, 4, 4, 4) == 0
    assert oz.workspace_bytes(4, 4, 4, 1) == 0
    assert oz.workspace_bytes(4, 4, 4, 27) == 0
    assert L.oz2_set_workspace(None, 16) == -1
    assert L.oz2_set_workspace(ctypes.c_void_p(0x1001), 4096) == -1   # not 256-byte aligned
    assert L.oz2_set_workspace(None, 0) == 0
    assert L.oz2_set_kblock(0) == -1 and L.oz2_set_kblock(100) == -1 and L.oz2_set_kblock(1 << 17) == -1
    assert L.oz2_set_kblock(65536) == 0
    # calls that fail before anything is launched
    assert L.oz2_dgemm(-1, 1, 1, None, 1, None, 1, None, 1, 4, None) == -1
    assert L.oz2_dgemm(1, -1, 1, None, 1, None, 1, None, 1, 4, None) == -2
    assert L.oz2_dgemm(1, 1, -1, None, 1, None, 1, None, 1, 4, None) == -3
    assert L.oz2_dgemm(4, 4, 4, None, 3, None, 4, None, 4, 4, None) == -5
    assert L.oz2_dgemm(4, 4, 4, None, 4, None, 4, None, 4, 4, None) == -8     # C is NULL
    assert L.oz2_dgemm(0, 0, 0, None, 1, None, 1, None, 1, 4, None) == 0      # empty: nothing to do
    assert L.oz2_stage2_gemm(4, 4, 4, 4, None) == 1                          # no workspace registered
    assert L.oz2_set_shift_mode(3) == -1 and L.oz2_set_shift_mode(-1) == -1
    assert L.oz2_set_nonfinite_check(2) == -1 and L.oz2_set_nonfinite_check(1) == 0
    # the INT8 product of 6-bit bounds must fit INT32: the inner dimension stays below 2^19 in that mode
    assert L.oz2_set_shift_mode(2) == 0
    try:
        assert L.oz2_stage2_gemm(4, 4, (1 << 19) - 64, 26, None) == 1         # accepted; fails later: no workspace
        assert L.oz2_stage2_gemm(4, 4, (1 << 19) - 63, 26, None) == 2         # budget
    finally:
        assert L.oz2_set_shift_mode(0) == 0
    assert oz.lib().oz2_status_string(1).decode().startswith("workspace")
    assert oz.lib().oz2_status_string(-3).decode() == "invalid argument"


def test_dropped_workspace_is_unregistered():
    """The library keeps a bare pointer to the workspace; when the Python owner of the buffer goes away the
    registration must go with it, so that a later call reports a missing workspace instead of writing into memory
    the allocator has handed to someone else.  Host memory stands in for device memory: nothing is launched."""
    L = oz.lib()
    ws = oz.Workspace(64, 64, 64, 8, device="cpu")
    assert oz.binding._registered_ptr == ws.ptr
    other = oz.Workspace(32, 32, 32, 8, device="cpu")      # a second registration replaces the first
    del ws                                                 # ... so dropping the first one changes nothing
    assert oz.binding._registered_ptr == other.ptr
    del other
    assert oz.binding._registered_ptr is None
    assert L.oz2_stage2_gemm(32, 32, 32, 8, None) == 1     # OZ2_ERR_WORKSPACE, before any launch
    assert L.oz2_dgemm(32, 32, 32, ctypes.c_void_p(256), 32, ctypes.c_void_p(256), 32, ctypes.c_void_p(256), 32, 8, None) == 1


def test_contexts_keep_their_own_settings_and_workspace():
    """A context is a private copy of the settings and of the workspace registration; the process-wide ones stay
    as they are.  Host side only: calls stop at the missing workspace before anything is launched."""
    L = oz.lib()
    a, b = oz.Context(), oz.Context()
    assert a.get(oz.OZ2_OPT_SHIFT_MODE) == 0 and a.get(oz.OZ2_OPT_PRODUCT_FORMAT) == oz.OZ2_PRODUCT_RESIDUE_U8
    assert a.get(oz.OZ2_OPT_KBLOCK) == 65536 and a.get(oz.OZ2_OPT_GEMM_ALGORITHM) == oz.OZ2_GEMM_AUTO
    a.set(oz.OZ2_OPT_SHIFT_MODE, 2)
    a.set(oz.OZ2_OPT_KBLOCK, 4096)
    b.set(oz.OZ2_OPT_BIT_SPLIT, -3)
    assert (a.get(oz.OZ2_OPT_SHIFT_MODE), b.get(oz.OZ2_OPT_SHIFT_MODE)) == (2, 0)
    assert (a.get(oz.OZ2_OPT_KBLOCK), b.get(oz.OZ2_OPT_KBLOCK)) == (4096, 65536)
    assert (a.get(oz.OZ2_OPT_BIT_SPLIT), b.get(oz.OZ2_OPT_BIT_SPLIT)) == (0, -3)
    # the process-wide context saw none of it
    assert L.oz2_context_set(None, oz.OZ2_OPT_NONFINITE_CHECK, 1) == 0
    v = ctypes.c_int64(-1)
    assert L.oz2_context_get(None, oz.OZ2_OPT_SHIFT_MODE, ctypes.byref(v)) == 0 and v.value == 0
    assert L.oz2_context_set(a.handle, 99, 0) == -2 and L.oz2_context_set(a.handle, oz.OZ2_OPT_SHIFT_MODE, 7) == -3
    assert L.oz2_context_set(a.handle, oz.OZ2_OPT_KBLOCK, 1 << 40) == -3 and L.oz2_context_get(a.handle, 0, None) == -3
    # in mode 2 the inner dimension is limited: a's setting decides for a, not for b
    p = ctypes.c_void_p(256)
    args = (b"N", b"N", 4, 4, (1 << 19), 1.0, p, 4, p, 1 << 19, 0.0, p, 4, 26, None)
    assert L.oz2_context_dgemm(a.handle, *args) == 2          # OZ2_ERR_BUDGET under a's shift mode
    assert L.oz2_context_dgemm(b.handle, *args) == 1          # b: accepted, stops at the missing workspace
    # workspaces are per context
    buf = np.zeros(1 << 20, dtype=np.uint8)
    base = buf.ctypes.data + (-buf.ctypes.data) % 256
    assert L.oz2_context_set_workspace(b.handle, ctypes.c_void_p(base), 64) == 0
    small = (b"N", b"N", 4, 4, 4, 1.0, p, 4, p, 4, 0.0, p, 4, 4, None)
    assert L.oz2_context_dgemm(b.handle, *small) == 1         # registered but too small
    assert L.oz2_stage2_gemm(4, 4, 4, 4, None) == 1           # the process-wide context has none at all
    # argument codes count the context as the first argument
    assert L.oz2_context_dgemm(a.handle, b"X", b"N", 4, 4, 4, 1.0, p, 4, p, 4, 0.0, p, 4, 4, None) == -2
    assert L.oz2_context_dgemm(a.handle, b"N", b"N", -1, 4, 4, 1.0, p, 4, p, 4, 0.0, p, 4, 4, None) == -4
    assert L.oz2_context_dsyrk(a.handle, b"Q", b"N", 4, 4, 1.0, p, 4, 0.0, p, 4, 4, None) == -2
    assert L.oz2_context_dtrmm(a.handle, b"L", b"L", b"N", b"N", -1, 4, 1.0, p, 4, p, 4, 4, None) == -6
    assert L.oz2_context_create(None) == -1 and L.oz2_context_destroy(None) == -1
    a.close()
    b.close()


def test_round_sync_setting_is_validated():
    L = oz.lib()
    assert L.oz2_set_round_sync(-1) == -1 and L.oz2_set_round_sync((1 << 20) + 1) == -1
    assert L.oz2_set_round_sync(0) == 0 and L.oz2_set_round_sync(4096) == 0


def test_traffic_profile_belongs_to_the_gemm_source_in_the_tree():
    """bench.py reports roofline.traffic from profiles/gemm_hbm_traffic.txt only while that file names the GEMM source
    it was measured on; this fails when the kernel was edited and the counters were not taken again."""
    import bench
    tr = bench.measured_traffic("c4.strassen.u8")
    assert tr is not None, "profiles/gemm_hbm_traffic.txt was taken on another oz2_stage2.hip: profile again"
    assert tr["bytes"] > tr["algorithmic_GiB"] * 2**30 and bench.measured_traffic("no.such.entry") is None


def test_workspace_layout_is_consistent():
    for fmt, bpe in ((oz.OZ2_PRODUCT_RESIDUE_U8, 1), (oz.OZ2_PRODUCT_INT32, 4)):
        oz.oz2_set_product_format(fmt)
        try:
            for (m, n, k, N) in [(1, 1, 1, 2), (300, 200, 100, 3), (256, 256, 64, 14), (16384, 16384, 16384, 16)]:
                lay = oz.workspace_layout(m, n, k, N)
                mp, npad, kp = lay["m_pad"], lay["n_pad"], lay["k_pad"]
                assert mp % 256 == 0 and npad % 256 == 0 and kp % 64 == 0
                assert mp >= m and npad >= n and kp >= k and mp - m < 256 and kp - k < 64
                order = ["rowmax", "flags", "colmax", "sa", "sb", "a_planes", "b_planes", "c_planes", "rownorm", "colnorm"]
                # the product region: N planes of the format in force, and never less than 8 bytes per element
                sizes = [8 * mp, 256, 8 * npad, 4 * mp, 4 * npad, N * mp * kp, N * npad * kp, max(bpe * N, 8) * npad * mp,
                         8 * mp, 8 * npad]
                for a, b, sz in zip(order, order[1:], sizes):
                    assert lay[a] % 256 == 0 and lay[a] + sz <= lay[b]
                assert lay["flags"] == lay["rowmax"] + 8 * mp      # cleared by the same fill as the row maxima
                exact = oz.workspace_bytes(m, n, k, N, fmt)
                assert lay["colnorm"] + sizes[-1] <= exact <= oz.workspace_bytes(m, n, k, N)
        finally:
            oz.oz2_set_product_format(oz.OZ2_PRODUCT_RESIDUE_U8)
    assert oz.workspace_bytes(16384, 16384, 16384, 16) < 25 * 2**30
    assert oz.workspace_bytes(16384, 16384, 16384, 16, oz.OZ2_PRODUCT_RESIDUE_U8) < 13 * 2**30
    assert oz.workspace_bytes(4, 4, 4, 4, 7) == 0


# ----------------------------------------------------------------------------------------------
# Algorithm 1 lines 2-5 on one element: the FP64 split-and-reduce routine against exact integers
# ----------------------------------------------------------------------------------------------
def _exact_residues(a, shift, mods):
    from fractions import Fraction
    ap = math.trunc(Fraction(a) * Fraction(2) ** shift)
    return [orc.sym_mod(ap, p) if abs(ap) < 2**62 else _sym_big(ap, p) for p in mods]


def _sym_big(x, p):
    r = x % p
    if 2 * r >= p:
        r -= p
    return r


@pytest.mark.parametrize("N,kappa", [(8, 26), (14, 50), (16, 55), (20, 72), (20, 75), (22, 80), (26, 99)])
def test_host_residues_match_exact_integers(N, kappa):
    mods = orc.moduli(N)
    rng = random.Random(1000 * N + kappa)
    cases = []
    for _ in range(3000):
        e = rng.randint(-40, 40)
        a = math.ldexp(rng.random() + 1.0, e) * rng.choice((-1, 1))       # |a| in [2^e, 2^(e+1))
        emax = e + rng.randint(0, 60)                                      # row maximum exponent
        cases.append((a, kappa - 1 - emax))
    # adversarial: full 53-bit mantissas at the top of the range, values that land on multiples of p,
    # on p/2 boundaries and on +-128 modulo 256
    top = (2**53 - 1) / 2**52
    cases += [(top, kappa - 1), (-top, kappa - 1), (1.0, kappa - 1), (1.0, 0), (0.0, 5), (-0.0, 5)]
    for p in mods:
        for mult in (1, 2, 3, 1000003):
            for delta in (0, 1, -1, p // 2, -(p // 2), p // 2 + 1):
                v = p * mult + delta
                if abs(v) < 2**min(kappa, 52):
                    cases.append((float(v), 0))
    for v in (128.0, -128.0, 384.0, -384.0, 127.0, -129.0, 2.0**40 + 128, -(2.0**40) - 128):
        cases.append((v, 0))
    for a, shift in cases:
        got = oz.host_residues(N, kappa, a, shift)
        want = _exact_residues(a, shift, mods)
        want8 = [((w + 128) % 256) - 128 for w in want]   # INT8 wrap-around of +128 for p = 256
        assert got == want8, (a, shift, got, want8)
        for g, p in zip(got, mods):
            assert -128 <= g <= 127 and (p == 256 or abs(g) <= (p - 1) // 2)


# ----------------------------------------------------------------------------------------------
# Algorithm 1 lines 7-11 on one element: residues of INT32 products -> double nearest to X
# ----------------------------------------------------------------------------------------------
def _crt_cases(N, rng):
    mods = orc.moduli(N)
    M = math.prod(mods)
    half = M // 2
    xs = []
    for _ in range(4000):
        xs.append(rng.randrange(-half, half))
        b = rng.randrange(1, M.bit_length())
        xs.append(rng.randrange(-(2**b), 2**b) % M - (M if rng.random() < 0.5 else 0))
    # range boundaries (Section 3: X in [-M/2, M/2)), zero, small values, powers of two
    xs += [0, 1, -1, half - 1, -half, -half + 1, half - 2, 2, -2]
    for b in range(0, M.bit_length() - 1):
        for d in (-1, 0, 1):
            xs += [2**b + d, -(2**b) + d]
    # rounding ties and near-ties: 54-bit patterns times a power of two, plus or minus one
    for _ in range(3000):
        mant = (rng.getrandbits(52) | (1 << 52)) * 2 + 1          # odd 54-bit integer: an exact tie
        sh = rng.randrange(0, max(1, M.bit_length() - 56))
        for d in (0, 1, -1, 2**max(sh - 1, 0), -(2**max(sh - 1, 0))):
            xs.append(mant * 2**sh + d)
            xs.append(-(mant * 2**sh) + d)
    # digit boundaries of the 40-bit limb representation
    for l in range(1, (M.bit_length() + 39) // 40):
        for d in (-2, -1, 0, 1, 2):
            for mul in (1, 3, 2**39, 2**39 + 1, 2**39 - 1):
                xs.append(mul * 2**(40 * l) + d)
                xs.append(-mul * 2**(40 * l) + d)
    out = []
    for x in xs:
        x = (x + half) % M - half
        out.append(x)
    return mods, M, out


@pytest.mark.parametrize("N", [2, 3, 5, 8, 11, 14, 16, 18, 20, 21, 24, 26])
def test_host_crt_element_is_correctly_rounded(N):
    rng = random.Random(77 + N)
    mods, M, xs = _crt_cases(N, rng)
    for x in xs:
        # any INT32 representative of the residue must give the same result (line 7 takes floor-mod)
        c = []
        for p in mods:
            r = x % p
            span = (2**31 - 1 - r) // p
            c.append(r + p * rng.randrange(-span, span + 1) if rng.random() < 0.7 else r)
        assert all(-2**31 <= v < 2**31 for v in c)
        got = oz.host_crt_element(N, c)
        assert got == float(x), (N, x, got, float(x))


@pytest.mark.parametrize("N", list(range(2, 17)))
def test_host_crt_element_by_digits_is_correctly_rounded(N):
    """The route of the matrix-core CRT kernel (weights in the symmetric range as balanced base-256 digits, digit
    sums, the same exact tail) on the same random and adversarial values of X, and on all-equal residues at both
    ends of their range, where the digit sums are largest."""
    rng = random.Random(177 + N)
    mods, M, xs = _crt_cases(N, rng)
    for x in xs:
        got = oz.host_crt_element_digits(N, [x % p for p in mods])
        assert got == float(x), (N, x, got, float(x))
    _, W = orc.crt_constants(N)
    half = M // 2
    for res in ([p - 1 for p in mods], [0] * N, [p - 1 if t % 2 else 0 for t, p in enumerate(mods)],
                [0 if t % 2 else p - 1 for t, p in enumerate(mods)], [1] * N):
        y = sum(r * w for r, w in zip(res, W)) % M
        y = y - M if y >= M - half else y
        assert oz.host_crt_element_digits(N, res) == float(y)
    assert oz.lib().oz2_host_crt_element_digits(17, None, None) == -1


def test_host_crt_extreme_int32_products():
    # products at the INT32 limits and negative values: floor-mod must stay in [0, p)
    N = 16
    mods = orc.moduli(N)
    M, W = orc.crt_constants(N)
    for c0 in (-2**31, 2**31 - 1, -1, 0, -255, -256, -257, 2**30 + 1):
        c = [c0] * N
        y = sum((c0 % p) * w for p, w in zip(mods, W)) % M
        if y >= M - M // 2:
            y -= M
        assert oz.host_crt_element(N, c) == float(y)


def test_strassen_form_sizes_and_choice_without_gpu():
    L = oz.lib()
    up = lambda v, a: (v + a - 1) // a * a
    for (m, n, k, N) in [(16384, 16384, 16384, 16), (700, 900, 1100, 14), (1, 1, 1, 2), (8192, 8192, 65536, 18)]:
        mh, nh, kh = up((m + 1) // 2, 256), up((n + 1) // 2, 256), up((k + 1) // 2, 64)
        planes = 7 * N * (mh * kh + nh * kh) + max(7 * N, 16) * mh * nh
        total = oz.workspace_bytes_strassen(m, n, k, N)
        small = 2 * mh * (8 + 4 + 8) + 2 * nh * (8 + 4 + 8) + 256
        assert planes + small <= total <= planes + small + 16 * 256
    assert oz.workspace_bytes_strassen(-1, 4, 4, 4) == 0 and oz.workspace_bytes_strassen(4, 4, 4, 27) == 0
    assert L.oz2_set_gemm_algorithm(2) == -1 and L.oz2_set_gemm_algorithm(-2) == -1
    assert L.oz2_gemm_algorithm_for(-1, 4, 4, 4) == -1 and L.oz2_gemm_algorithm_for(4, 4, 4, 1) == -4
    big = 16384
    try:
        oz.set_workspace(None, 0)
        # automatic: the form is preferred at this size, but nothing is registered that could hold it
        assert oz.workspace_bytes_preferred(big, big, big, 16) == oz.workspace_bytes_strassen(big, big, big, 16)
        assert oz.workspace_bytes_preferred(4096, 4096, 4096, 16) == oz.workspace_bytes(4096, 4096, 4096, 16, oz.OZ2_PRODUCT_RESIDUE_U8)
        assert oz.workspace_bytes_preferred(big, big, 8192, 16) == oz.workspace_bytes(big, big, 8192, 16, oz.OZ2_PRODUCT_RESIDUE_U8)
        assert oz.oz2_gemm_algorithm_for(big, big, big, 16) == oz.OZ2_GEMM_CLASSICAL
        oz.oz2_set_gemm_algorithm(oz.OZ2_GEMM_STRASSEN)
        assert oz.oz2_gemm_algorithm_for(300, 200, 100, 16) == oz.OZ2_GEMM_STRASSEN
        assert oz.oz2_gemm_algorithm_for(300, 0, 100, 16) == oz.OZ2_GEMM_CLASSICAL
        oz.oz2_set_product_format(oz.OZ2_PRODUCT_INT32)   # the form needs residues in the product planes
        assert oz.oz2_gemm_algorithm_for(300, 200, 100, 16) == oz.OZ2_GEMM_CLASSICAL
        oz.oz2_set_product_format(oz.OZ2_PRODUCT_RESIDUE_U8)
        oz.oz2_set_gemm_algorithm(oz.OZ2_GEMM_CLASSICAL)
        assert oz.workspace_bytes_preferred(big, big, big, 16) == oz.workspace_bytes(big, big, big, 16, oz.OZ2_PRODUCT_RESIDUE_U8)
    finally:
        oz.oz2_set_product_format(oz.OZ2_PRODUCT_RESIDUE_U8)
        oz.oz2_set_gemm_algorithm(oz.OZ2_GEMM_AUTO)


def test_strassen_identities_reproduce_the_oracles_residues():
    """The recipe of the Strassen form, carried out with numpy on the oracle's own INT8 planes: seven products of
    block sums and differences, each operand brought back into [-128, 127] modulo p_t and each product formed in
    INT32, recombined modulo p_t, must give the oracle's residues c''_t of Algorithm 1 line 7."""
    rng = np.random.default_rng(31)
    m, n, k, N = 10, 14, 12, 9
    A = np.asfortranarray((rng.random((m, k)) - 0.5) * np.exp(rng.standard_normal((m, k))))
    B = np.asfortranarray((rng.random((k, n)) - 0.5) * np.exp(rng.standard_normal((k, n))))
    ref = orc.dgemm(A, B, N, want=("C", "Ares", "Bres", "Cres"))
    mods = orc.moduli(N)
    mh, nh, kh = m // 2, n // 2, k // 2

    def int8(x, p):   # any representative in [-128, 127]
        r = np.mod(x, p)
        return np.where(r >= 128, r - p, r).astype(np.int64)

    for t, p in enumerate(mods):
        Ar = ref.Ares[t].astype(np.int64)            # m x k
        Br = ref.Bres[t].astype(np.int64).T          # planes of B hold its columns as rows: back to k x n
        A11, A12, A21, A22 = Ar[:mh, :kh], Ar[:mh, kh:], Ar[mh:, :kh], Ar[mh:, kh:]
        B11, B12, B21, B22 = Br[:kh, :nh], Br[:kh, nh:], Br[kh:, :nh], Br[kh:, nh:]
        ops = [(A11 + A22, B11 + B22), (A21 + A22, B11), (A11, B12 - B22), (A22, B21 - B11), (A11 + A12, B22),
               (A21 - A11, B11 + B12), (A12 - A22, B21 + B22)]
        M = []
        for X, Y in ops:
            X8, Y8 = int8(X, p), int8(Y, p)
            assert np.abs(X8).max() <= 128 and np.abs(Y8).max() <= 128
            prod = X8 @ Y8
            assert np.abs(prod).max() < 2**31
            M.append(np.mod(prod, p))
        Cr = np.empty((m, n), dtype=np.int64)
        Cr[:mh, :nh] = np.mod(M[0] + M[3] - M[4] + M[6], p)
        Cr[:mh, nh:] = np.mod(M[2] + M[4], p)
        Cr[mh:, :nh] = np.mod(M[1] + M[3], p)
        Cr[mh:, nh:] = np.mod(M[0] - M[1] + M[2] + M[5], p)
        assert np.array_equal(Cr, ref.Cres[t].astype(np.int64)), "modulus %d" % p


def test_bench_refuses_more_than_one_gpu():
    """The path runs on one GPU: bench.py --gpus N with N above 1 exits with a message and touches no GPU."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""
