"""GPU parity: every stage of the HIP path against the CPU oracle, element by element, through the C ABI.

Bars: shifts, INT8 residue planes and INT32 products bit-exact; final C within 1e-15 * (|A||B|)_ij of the
oracle (the design aims at bit equality and the tests report it)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2504_08009_amd as oz
from oracle import oracle as orc
from paper_2504_08009_amd import inputs


def _dev(x):
    """numpy (rows x cols, any order) -> column-major device tensor of the same logical shape"""
    return torch.from_numpy(np.ascontiguousarray(x.T)).cuda().t()


def run_stages(A, B, N, kblock=None, mode=0, fmt=0, delta=0):
    m, k = A.shape
    _, n = B.shape
    ws = oz.Workspace(m, n, k, N)
    lay = oz.workspace_layout(m, n, k, N)
    dA, dB = _dev(A), _dev(B)
    dC = torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda").t()
    if kblock is not None:
        oz.oz2_set_kblock(kblock)
    oz.oz2_set_shift_mode(mode)
    oz.oz2_set_product_format(fmt)
    oz.oz2_set_bit_split(delta)
    try:
        print("stage1 m=%d n=%d k=%d N=%d mode=%d fmt=%d delta=%d" % (m, n, k, N, mode, fmt, delta), flush=True)
        oz.oz2_stage1_convert(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, N)
        torch.cuda.synchronize()
        print("stage2", flush=True)
        oz.oz2_stage2_gemm(m, n, k, N)
        torch.cuda.synchronize()
        print("stage3", flush=True)
        oz.oz2_stage3_crt(m, n, k, dC.data_ptr(), m, N)
        torch.cuda.synchronize()
    finally:
        oz.oz2_set_shift_mode(0)
        oz.oz2_set_product_format(1)
        oz.oz2_set_bit_split(0)
        if kblock is not None:
            oz.oz2_set_kblock(65536)
    mp, np_, kp = lay["m_pad"], lay["n_pad"], lay["k_pad"]

    def planes(off, rows_pad):
        # blocked layout of include/oz2.h: [t][row block][k tile][256 rows][64 bytes] -> [t][row][l]
        raw = ws.view(off, N * rows_pad * kp, torch.int8).view(N, rows_pad // 256, kp // 64, 256, 64)
        return raw.permute(0, 1, 3, 2, 4).reshape(N, rows_pad, kp).cpu().numpy()

    out = dict(
        sa=ws.view(lay["sa"], mp, torch.int32).cpu().numpy(),
        sb=ws.view(lay["sb"], np_, torch.int32).cpu().numpy(),
        Ap=planes(lay["a_planes"], mp),
        Bp=planes(lay["b_planes"], np_),
        Cp=(ws.view(lay["c_planes"], N * np_ * mp, torch.int32) if fmt == 0 else
            ws.view(lay["c_planes"], N * np_ * mp, torch.uint8)).view(N, np_, mp).cpu().numpy(),
        C=dC.cpu().numpy(),
    )
    return out


def check_against_oracle(A, B, N, kblock=None, products_exact=True, mode=0, fmt=0, delta=0):
    """fmt 0: INT32 product planes (compared with the exact products); fmt 1: UINT8 residue planes written by
    the GEMM epilogue (compared with the oracle's residues of line 7)."""
    m, k = A.shape
    _, n = B.shape
    got = run_stages(A, B, N, kblock, mode, fmt, delta)
    ref = orc.dgemm(A, B, N, want=("C", "shifts", "Ares", "Bres", "Cprod", "Cres"), mode=mode, delta=delta)
    assert np.array_equal(got["sa"][:m], ref.sa), "row shifts"
    assert np.array_equal(got["sb"][:n], ref.sb), "column shifts"
    assert np.array_equal(got["Ap"][:, :m, :k], ref.Ares), "A residue planes"
    assert np.array_equal(got["Bp"][:, :n, :k], ref.Bres), "B residue planes"
    # padding must be zero: the GEMM reads it
    assert not got["Ap"][:, m:, :].any() and not got["Ap"][:, :, k:].any()
    assert not got["Bp"][:, n:, :].any() and not got["Bp"][:, :, k:].any()
    prod = got["Cp"][:, :n, :m].transpose(0, 2, 1).astype(np.int64)
    if fmt == 1:
        assert np.array_equal(prod, ref.Cres.astype(np.int64)), "UINT8 residues of the products"
    elif products_exact:
        assert np.array_equal(prod, ref.Cprod), "INT32 products"
    else:
        mods = np.array(orc.moduli(N), dtype=np.int64)[:, None, None]
        assert np.array_equal(np.mod(prod, mods), ref.Cres.astype(np.int64)), "products modulo p_t"
    _, S = orc.exact(A, B)
    err = np.abs(got["C"] - ref.C)
    assert np.all(err <= 1e-15 * S), "final C tolerance"
    nbad = int(np.count_nonzero(got["C"] != ref.C))
    print("C elements differing from the oracle in the last bit or more: %d of %d" % (nbad, m * n), flush=True)
    assert nbad == 0, "final C not bit-identical"
    return got, ref


@pytest.mark.parametrize("fmt", [0, 1])
def test_c1_all_stages(fmt):
    cfg = inputs.CONFIGS["c1"]
    A, B = inputs.gemm_inputs(cfg["seed"], cfg["m"], cfg["n"], cfg["k"], cfg["phi"])
    check_against_oracle(A, B, 14, fmt=fmt)


@pytest.mark.parametrize("m,n,k,N,phi", [
    (300, 200, 333, 5, 0.5),      # ragged in every dimension, two row tiles
    (257, 513, 129, 14, 1.0),     # one past the tile in each dimension
    (64, 40, 1000, 20, 4.0),      # wide exponent range, 4 limbs at the limit
    (33, 17, 50, 23, 4.0),        # kappa > 75: two-level split, 5 limbs
    (5, 3, 1, 26, 0.5),           # k = 1, largest moduli count
    (1, 1, 7, 2, 0.5),            # smallest everything
    (5000, 1, 7, 12, 0.5),        # tall and thin: twenty row tiles, one column
    (1, 3000, 2000, 15, 1.0),     # one row, twelve column tiles
    (2100, 3, 5000, 16, 0.5),     # long inner dimension against a sliver of C
])
@pytest.mark.parametrize("fmt", [0, 1])
def test_ragged_shapes(m, n, k, N, phi, fmt):
    rng = np.random.default_rng(m * 1000 + n)
    A = (rng.random((m, k)) - 0.5) * np.exp(phi * rng.standard_normal((m, k)))
    B = (rng.random((k, n)) - 0.5) * np.exp(phi * rng.standard_normal((k, n)))
    check_against_oracle(A, B, N, fmt=fmt)


@pytest.mark.parametrize("fmt", [0, 1])
def test_tile_grid_of_8_by_12_all_stages(fmt):
    """A tile grid that is a multiple of 8 x 4 but not of 16 x 16, with enough planes that the GEMM takes the list
    order of its 8 x 4 sub-blocks (3 per plane, 66 in all: eight full rounds of the eight XCDs and a last one with
    two entries); every plane is compared."""
    rng = np.random.default_rng(88)
    m, n, k, N = 2048, 3072, 70, 22
    A = np.asfortranarray((rng.random((m, k)) - 0.5) * np.exp(rng.standard_normal((m, k))))
    B = np.asfortranarray((rng.random((k, n)) - 0.5) * np.exp(rng.standard_normal((k, n))))
    check_against_oracle(A, B, N, fmt=fmt)


def test_zero_rows_columns_and_extreme_exponents():
    rng = np.random.default_rng(77)
    m, n, k, N = 70, 90, 200, 16
    A = rng.standard_normal((m, k))
    B = rng.standard_normal((k, n))
    A[3, :] = 0.0
    B[:, 5] = 0.0
    A[10, :] *= 2.0**300      # rows and columns of very different scale
    A[11, :] *= 2.0**-300
    B[:, 7] *= 2.0**200
    B[:, 8] *= 2.0**-250
    A[12, 1:] = 0.0           # a single nonzero in the row
    A[20, :] = np.ldexp(np.round(rng.standard_normal(k) * 1000), 0)  # integers
    got, _ = check_against_oracle(A, B, N)
    assert np.all(got["C"][3, :] == 0.0) and np.all(got["C"][:, 5] == 0.0)


def test_dgemm_single_call_equals_stages_and_handles_ld():
    rng = np.random.default_rng(5)
    m, n, k, N = 120, 75, 260, 15
    lda, ldb, ldc = m + 8, k + 3, m + 5
    Af = np.zeros((lda, k), order="F")
    Bf = np.zeros((ldb, n), order="F")
    Af[:m, :] = rng.standard_normal((m, k))
    Bf[:k, :] = rng.standard_normal((k, n))
    Af[m:, :] = 1e300   # must never be read as data
    Bf[k:, :] = 1e300
    dA = torch.from_numpy(np.ascontiguousarray(Af.T)).cuda()   # (k, lda) contiguous == column-major lda x k
    dB = torch.from_numpy(np.ascontiguousarray(Bf.T)).cuda()
    dC = torch.full((n, ldc), -7.0, dtype=torch.float64, device="cuda")
    ws = oz.Workspace(m, n, k, N)
    oz.oz2_dgemm(m, n, k, dA.data_ptr(), lda, dB.data_ptr(), ldb, dC.data_ptr(), ldc, N)
    torch.cuda.synchronize()
    C = dC.cpu().numpy().T
    ref = orc.dgemm(Af[:m, :], Bf[:k, :], N).C
    assert np.array_equal(C[:m, :], ref)
    assert np.all(C[m:, :] == -7.0)   # rows beyond m of the ldc-padded output untouched
    del ws


def test_quick_returns_and_errors():
    ws = oz.Workspace(8, 8, 8, 4)
    dC = torch.full((4, 6), 3.0, dtype=torch.float64, device="cuda")
    L = oz.lib()
    st = torch.cuda.current_stream().cuda_stream
    # k == 0: C := 0
    assert L.oz2_dgemm(6, 4, 0, None, 6, None, 1, dC.data_ptr(), 6, 4, st) == 0
    torch.cuda.synchronize()
    assert torch.all(dC == 0.0)
    # m == 0 or n == 0: nothing happens
    assert L.oz2_dgemm(0, 4, 5, None, 1, None, 5, None, 1, 4, st) == 0
    assert L.oz2_dgemm(3, 0, 5, None, 3, None, 5, None, 3, 4, st) == 0
    # bad arguments
    assert L.oz2_dgemm(-1, 4, 4, None, 1, None, 4, None, 1, 4, st) == -1
    assert L.oz2_dgemm(4, 4, 4, dC.data_ptr(), 3, dC.data_ptr(), 4, dC.data_ptr(), 4, 4, st) == -5
    assert L.oz2_dgemm(4, 4, 4, dC.data_ptr(), 4, dC.data_ptr(), 3, dC.data_ptr(), 4, 4, st) == -7
    assert L.oz2_dgemm(4, 4, 4, dC.data_ptr(), 4, dC.data_ptr(), 4, dC.data_ptr(), 3, 4, st) == -9
    assert L.oz2_dgemm(4, 4, 4, dC.data_ptr(), 4, dC.data_ptr(), 4, dC.data_ptr(), 4, 1, st) == -10
    assert L.oz2_dgemm(4, 4, 4, dC.data_ptr(), 4, dC.data_ptr(), 4, dC.data_ptr(), 4, 27, st) == -10
    # workspace too small for a bigger problem
    assert L.oz2_dgemm(600, 600, 600, dC.data_ptr(), 600, dC.data_ptr(), 600, dC.data_ptr(), 600, 8, st) == 1
    # two moduli cannot carry k = 2^15 (kappa < 1)
    big = oz.Workspace(4, 4, 1 << 15, 2)
    assert L.oz2_dgemm(4, 4, 1 << 15, dC.data_ptr(), 4, dC.data_ptr(), 1 << 15, dC.data_ptr(), 4, 2, st) == 2
    del big, ws


def test_k_blocking_matches_unblocked():
    # the block length is a parameter; blocked accumulation must give the same residues and the same C
    rng = np.random.default_rng(9)
    m, n, k, N = 40, 50, 1500, 12
    A = rng.standard_normal((m, k))
    B = rng.standard_normal((k, n))
    base, ref = check_against_oracle(A, B, N)
    blocked, _ = check_against_oracle(A, B, N, kblock=256, products_exact=False)
    assert np.array_equal(blocked["C"], base["C"])
    assert not np.array_equal(blocked["Cp"], base["Cp"])  # the reduction between blocks really ran
    blocked8, _ = check_against_oracle(A, B, N, kblock=256, fmt=1)
    assert np.array_equal(blocked8["C"], base["C"])


def test_determinism_two_runs():
    cfg = inputs.CONFIGS["c1"]
    A, B = inputs.gemm_inputs(cfg["seed"] + 100, 384, 320, 512, 1.0)
    r1 = run_stages(A, B, 16)
    r2 = run_stages(A, B, 16)
    for key in ("sa", "sb", "Ap", "Bp", "Cp"):
        assert np.array_equal(r1[key], r2[key])
    r3 = run_stages(A, B, 16, fmt=1)
    assert np.array_equal(r1["C"].view(np.uint64), r3["C"].view(np.uint64))  # both product formats, same C
    assert np.array_equal(r1["C"].view(np.uint64), r2["C"].view(np.uint64))


def test_c2_sampled_rows_and_error_decay():
    # config 2 at full size on the GPU; the oracle checks a sampled block of outputs for several N
    cfg = inputs.CONFIGS["c2"]
    m, n, k = cfg["m"], cfg["n"], cfg["k"]
    A, B = inputs.gemm_inputs(cfg["seed"], m, n, k, cfg["phi"])
    rows = np.unique(np.concatenate([np.arange(0, m, 37), [m - 1]]))
    cols = np.unique(np.concatenate([np.arange(5, n, 41), [0, n - 1]]))
    Cx, S = orc.exact(A, B, rows=rows, cols=cols)
    dA, dB = _dev(A), _dev(B)
    errs = {}
    for N in range(8, 21):
        ws = oz.Workspace(m, n, k, N)
        dC = torch.empty((n, m), dtype=torch.float64, device="cuda").t()
        oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N)
        torch.cuda.synchronize()
        C = dC.cpu().numpy()[np.ix_(rows, cols)]
        ref = orc.dgemm(A, B, N, rows=rows, cols=cols).C
        assert np.all(np.abs(C - ref) <= 1e-15 * S)
        assert np.array_equal(C, ref), "N=%d not bit-identical with the oracle" % N
        errs[N] = float(np.max(np.abs(C - Cx) / S))
        del ws
    native = float(np.max(np.abs((dA @ dB).cpu().numpy()[np.ix_(rows, cols)] - Cx) / S))
    print("componentwise error vs exact:", errs, "native FP64:", native, flush=True)
    # every modulus more buys about four bits until the final rounding dominates
    for N in range(8, 16):
        assert errs[N + 1] < errs[N] / 4, N
    assert errs[16] < native and max(errs[N] for N in range(17, 21)) <= errs[16]


@pytest.mark.parametrize("name,kblock,algorithm,N", [
    ("c3", None, -1, 14), ("c3", None, -1, 18), ("c5a", None, -1, 18), ("c4", None, -1, 16), ("c4", None, 0, 16),
    ("c5b", 32768, 0, 18), ("c5b", 16384, -1, 18)])
def test_full_size_configs_on_sampled_outputs(name, kblock, algorithm, N):
    """The benchmark configurations at full size through oz2_dgemm (the call bench.py times); the oracle
    recomputes a sample of output rows and columns (first, last and random ones) with the full inner
    dimension.  algorithm -1 is the library's own choice of the form of the INT8 products (the Strassen form at
    c4 and c5b, which is what bench.py times), 0 the classical form.  c5b runs with k-blocks of half the inner
    dimension each product walks (32768 of 65536 classical, 16384 of 32768 per half in the Strassen form) so
    that the reduction between k-blocks is exercised; the result must still be bit-identical."""
    cfg = inputs.CONFIGS[name]
    m, n, k, phi = cfg["m"], cfg["n"], cfg["k"], cfg["phi"]
    assert N == 16 if name == "c4" else N in cfg["N"]
    print("generating %s: m=%d n=%d k=%d N=%d" % (name, m, n, k, N), flush=True)
    A = inputs.block(cfg["seed"], 0, m, k, phi)
    B = inputs.block(cfg["seed"], 1, k, n, phi)
    rng = np.random.default_rng(3)
    rows = np.unique(np.concatenate([[0, 255, 256, m - 1], rng.choice(m, 44, replace=False)]))
    cols = np.unique(np.concatenate([[0, 255, 256, n - 1], rng.choice(n, 44, replace=False)]))
    dA = torch.from_numpy(A.T).cuda().t()
    dB = torch.from_numpy(B.T).cuda().t()
    dC = torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda").t()
    oz.oz2_set_gemm_algorithm(algorithm)
    if kblock:
        oz.oz2_set_kblock(kblock)
    try:
        ws = oz.Workspace(m, n, k, N)
        strassen = oz.oz2_gemm_algorithm_for(m, n, k, N) == oz.OZ2_GEMM_STRASSEN
        assert strassen == (algorithm == -1 and name in ("c4", "c5b"))
        print("oz2_dgemm (%s form)" % ("Strassen" if strassen else "classical"), flush=True)
        oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N)
        torch.cuda.synchronize()
    finally:
        oz.oz2_set_kblock(65536)
        oz.oz2_set_gemm_algorithm(oz.OZ2_GEMM_AUTO)
    assert not bool(torch.isnan(dC).any())
    got = dC[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()].cpu().numpy()
    Asub = np.asfortranarray(A[rows, :])
    Bsub = np.asfortranarray(B[:, cols])
    print("oracle on %d x %d outputs" % (len(rows), len(cols)), flush=True)
    ref = orc.dgemm(Asub, Bsub, N).C
    _, S = orc.exact(Asub, Bsub)
    assert np.all(np.abs(got - ref) <= 1e-15 * S)
    assert np.array_equal(got, ref), "%s: not bit-identical with the oracle" % name
    del ws


@pytest.mark.parametrize("N,algorithm", [(8, 0), (17, 0), (8, 1)])
def test_more_than_2_to_the_32_elements_of_c(N, algorithm):
    """A product whose C (and, in the classical form, every residue plane) has more than 2^32 elements, so that an
    element index does not fit 32 bits: 66000 x 65600 with a short inner dimension, 8 moduli (matrix-core CRT
    kernel) and 17 (FP64 accumulation) in the classical form, 8 moduli with the Strassen form forced (56 planes of
    2^30 elements).  Every element is written (C starts as NaN), and a sample of rows and columns including the last
    ones is compared with the oracle."""
    m, n, k, phi = 66000, 65600, 64 if algorithm == 0 else 128, 0.5
    assert m * n > 1 << 32
    A = inputs.block(91, 0, m, k, phi)
    B = inputs.block(91, 1, k, n, phi)
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, 255, 256, 65535, 65536, m - 1], rng.choice(m, 42, replace=False)]))
    cols = np.unique(np.concatenate([[0, 255, 256, 65535, 65536, n - 1], rng.choice(n, 42, replace=False)]))
    dA = torch.from_numpy(A.T).cuda().t()
    dB = torch.from_numpy(B.T).cuda().t()
    dC = torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda").t()
    oz.oz2_set_gemm_algorithm(algorithm)
    try:
        ws = oz.Workspace(m, n, k, N, product_format=oz.OZ2_PRODUCT_RESIDUE_U8)   # 8, 17 or 14 bytes per element of C
        assert (oz.oz2_gemm_algorithm_for(m, n, k, N) == oz.OZ2_GEMM_STRASSEN) == (algorithm == 1)
        print("C of %d x %d = %.2f * 2^32 elements, N=%d, form %d" % (m, n, m * n / 2.0**32, N, algorithm), flush=True)
        oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N)
        torch.cuda.synchronize()
    finally:
        oz.oz2_set_gemm_algorithm(oz.OZ2_GEMM_AUTO)
    del ws
    # column by column blocks, to keep the temporaries of the check small
    for j0 in range(0, n, 8192):
        assert not bool(torch.isnan(dC[:, j0:j0 + 8192]).any()), j0
    got = dC[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()].cpu().numpy()
    del dC
    ref = orc.dgemm(np.asfortranarray(A[rows, :]), np.asfortranarray(B[:, cols]), N).C
    assert np.array_equal(got, ref)


def test_operand_planes_beyond_2_to_the_32_bytes():
    """An operand whose every residue plane is larger than 2^32 bytes (A: 66000 x 66000, 35 GB of FP64), so that a
    byte offset inside one plane does not fit 32 bits, against a narrow B.  A is drawn on the device with torch's
    seeded generator (on the host the 4.4e9 values would take minutes), the sampled rows are copied back for the
    oracle; all columns of those rows are compared."""
    m, k, n, N, phi = 66000, 66000, 192, 4, 0.5
    assert m * k > 1 << 32
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20250408)
    dAt = torch.empty((k, m), dtype=torch.float64, device="cuda")   # column-major m x k
    for c0 in range(0, k, 2048):
        c1 = min(k, c0 + 2048)
        u = torch.rand((c1 - c0, m), dtype=torch.float64, device="cuda", generator=gen)
        z = torch.randn((c1 - c0, m), dtype=torch.float64, device="cuda", generator=gen)
        dAt[c0:c1] = (u - 0.5) * torch.exp(phi * z)
        del u, z
    B = inputs.block(92, 1, k, n, phi)
    dB = torch.from_numpy(B.T).cuda().t()
    dC = torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda").t()
    rng = np.random.default_rng(6)
    rows = np.unique(np.concatenate([[0, 255, 256, 65535, 65536, 65792, m - 1], rng.choice(m, 25, replace=False)]))
    Asub = np.asfortranarray(dAt[:, torch.from_numpy(rows).cuda()].t().cpu().numpy())
    ws = oz.Workspace(m, n, k, N, product_format=oz.OZ2_PRODUCT_RESIDUE_U8)
    print("A planes of %.2f * 2^32 bytes each" % (m * k / 2.0**32), flush=True)
    oz.oz2_dgemm(m, n, k, dAt.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N)
    torch.cuda.synchronize()
    del ws, dAt
    assert not bool(torch.isnan(dC).any())
    got = dC[torch.from_numpy(rows).cuda()].cpu().numpy()
    ref = orc.dgemm(Asub, B, N).C
    assert np.array_equal(got, ref)


def test_two_contexts_with_different_settings_on_two_streams():
    """Two contexts, each with its own workspace and settings (Cauchy-Schwarz shifts with 12 moduli and INT32 product
    planes in one, the simple bound with 15 moduli and a short k-block in the other), called alternately on two
    streams so that their kernels may overlap: every result is the oracle's for that context's settings, and the
    process-wide settings are what they were."""
    rng = np.random.default_rng(71)
    m, n, k = 700, 520, 900
    A = np.asfortranarray((rng.random((m, k)) - 0.5) * np.exp(rng.standard_normal((m, k))))
    B = np.asfortranarray((rng.random((k, n)) - 0.5) * np.exp(rng.standard_normal((k, n))))
    dA, dB = _dev(A), _dev(B)
    ca, cb = oz.Context(), oz.Context()
    ca.set(oz.OZ2_OPT_SHIFT_MODE, oz.OZ2_SHIFT_CAUCHY_SCHWARZ)
    ca.set(oz.OZ2_OPT_PRODUCT_FORMAT, oz.OZ2_PRODUCT_INT32)
    cb.set(oz.OZ2_OPT_KBLOCK, 256)
    ca.allocate_workspace(m, n, k, 12)
    cb.allocate_workspace(m, n, k, 15)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    Ca = [torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda").t() for _ in range(3)]
    Cb = [torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda").t() for _ in range(3)]
    torch.cuda.synchronize()
    for r in range(3):
        print("contexts: round %d" % r, flush=True)
        ca.dgemm("N", "N", m, n, k, 1.0, dA.data_ptr(), m, dB.data_ptr(), k, 0.0, Ca[r].data_ptr(), m, 12, sa)
        cb.dgemm("N", "N", m, n, k, 1.0, dA.data_ptr(), m, dB.data_ptr(), k, 0.0, Cb[r].data_ptr(), m, 15, sb)
    torch.cuda.synchronize()
    ref_a = orc.dgemm(A, B, 12, mode=1).C
    ref_b = orc.dgemm(A, B, 15, mode=0).C
    for r in range(3):
        assert np.array_equal(Ca[r].cpu().numpy(), ref_a), "context a, call %d" % r
        assert np.array_equal(Cb[r].cpu().numpy(), ref_b), "context b, call %d" % r
    assert not np.array_equal(ref_a, ref_b)
    # the process-wide context still has the defaults and no part in this
    probe = oz.Context()
    for opt in (oz.OZ2_OPT_SHIFT_MODE, oz.OZ2_OPT_PRODUCT_FORMAT, oz.OZ2_OPT_KBLOCK):
        v = __import__("ctypes").c_int64(-1)
        assert oz.lib().oz2_context_get(None, opt, __import__("ctypes").byref(v)) == 0 and v.value == probe.get(opt)
    ca.close(), cb.close(), probe.close()


_sync_case = {}


@pytest.mark.parametrize("spins", [1, 0, 4096])
def test_round_synchronisation_bound_and_switch(spins):
    """The GEMM's per-die round synchronisation with its wait bound forced down to one poll (so that waits run to
    their bound, the die's counter is pushed past every target and the rest of the launch runs unsynchronised),
    switched off, and at its default: the residues and C are the oracle's every time.  2048 x 1024 x 6400 with 22
    moduli: 704 tiles for 256 workgroups (two or three tiles each, two synchronised rounds, early arrival), an inner
    dimension of 100 k-tiles, which puts the launch among those that synchronise; every element of every plane is
    compared."""
    m, n, k, N = 2048, 1024, 6400, 22
    if not _sync_case:
        rng = np.random.default_rng(61)
        _sync_case["A"] = np.asfortranarray((rng.random((m, k)) - 0.5) * np.exp(0.5 * rng.standard_normal((m, k))))
        _sync_case["B"] = np.asfortranarray((rng.random((k, n)) - 0.5) * np.exp(0.5 * rng.standard_normal((k, n))))
        print("oracle for the round-synchronisation case", flush=True)
        _sync_case["ref"] = orc.dgemm(_sync_case["A"], _sync_case["B"], N, want=("C", "Cres"))
    A, B, ref = _sync_case["A"], _sync_case["B"], _sync_case["ref"]
    oz.oz2_set_round_sync(spins)
    try:
        got = run_stages(A, B, N, fmt=1)
        ws = oz.Workspace(m, n, k, N)
        C = oz.dgemm(_dev(A), _dev(B), N, workspace=ws)
        torch.cuda.synchronize()
    finally:
        oz.oz2_set_round_sync(4096)
    assert np.array_equal(got["Cp"][:, :n, :m].transpose(0, 2, 1), ref.Cres)
    assert np.array_equal(got["C"], ref.C) and np.array_equal(C.cpu().numpy(), ref.C)
    del ws


@pytest.mark.parametrize("N,alpha,beta", [(16, 1.0, 0.0), (13, 1.0, 0.0), (9, 1.0, 0.0), (4, 1.0, 0.0), (16, -0.75, 2.0),
                                          (17, 1.0, 0.0)])
def test_matrix_core_crt_every_element_ragged(N, alpha, beta):
    """Alg. 1 line 9 on the matrix cores (the kernel taken from 2^24 elements of C on, classical form, up to 16
    moduli): a ragged shape above that size with a short inner dimension, EVERY element of C compared with the
    oracle, for moduli counts whose product needs one, two, three and four 40-bit limbs, as the update with alpha
    and beta, and with 17 moduli (the first count that stays with the FP64 accumulation at this size)."""
    m, n, k, phi = 5801, 5791, 40, 1.0
    assert m * n >= 1 << 25
    A = inputs.block(77, 0, m, k, phi)
    B = inputs.block(77, 1, k, n, phi)
    C0 = inputs.block(77, 2, m, n, 0.5)
    dA = torch.from_numpy(A.T).cuda().t()
    dB = torch.from_numpy(B.T).cuda().t()
    dC = torch.from_numpy(C0.T).cuda().t()
    oz.oz2_set_gemm_algorithm(oz.OZ2_GEMM_CLASSICAL)
    try:
        ws = oz.Workspace(m, n, k, N)
        print("matrix-core CRT, every element of %d x %d, N=%d alpha=%g beta=%g" % (m, n, N, alpha, beta), flush=True)
        oz.oz2_dgemm_ex("N", "N", m, n, k, alpha, dA.data_ptr(), m, dB.data_ptr(), k, beta, dC.data_ptr(), m, N)
        torch.cuda.synchronize()
    finally:
        oz.oz2_set_gemm_algorithm(oz.OZ2_GEMM_AUTO)
    got = dC.cpu().numpy()
    del ws, dA, dB, dC
    ref = orc.dgemm_ex("N", "N", alpha, A, B, beta, C0, N)
    bad = np.argwhere(got != ref)
    assert len(bad) == 0, "%d elements differ from the oracle, first at %s" % (len(bad), bad[:5].tolist())
    assert not np.isnan(got).any()


_c3_oracle = {}


@pytest.mark.parametrize("algorithm", [0, 1])
def test_c3_every_element_both_forms(algorithm):
    """Config c3 (4096^3, phi = 1, 16 moduli) through oz2_dgemm with EVERY element of C compared with the oracle,
    in the classical form (16 x 16 tile grid: the super-block order, 16 tiles per workgroup slot of the persistent
    loop) and with the Strassen form forced (seven 2048^3 products per modulus on an 8 x 8 tile grid: the list order
    of the 8 x 4 sub-blocks, 28 tiles per slot).  The oracle forms line 6 as printed either way, so one oracle run
    (about half a minute on the host cores) serves both."""
    cfg = inputs.CONFIGS["c3"]
    m, n, k, phi, N = cfg["m"], cfg["n"], cfg["k"], cfg["phi"], 16
    A = inputs.block(cfg["seed"], 0, m, k, phi)
    B = inputs.block(cfg["seed"], 1, k, n, phi)
    dA = torch.from_numpy(A.T).cuda().t()
    dB = torch.from_numpy(B.T).cuda().t()
    dC = torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda").t()
    oz.oz2_set_gemm_algorithm(algorithm)
    try:
        ws = oz.Workspace(m, n, k, N)
        assert (oz.oz2_gemm_algorithm_for(m, n, k, N) == oz.OZ2_GEMM_STRASSEN) == (algorithm == 1)
        print("c3 every element, %s form" % ("Strassen" if algorithm else "classical"), flush=True)
        oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N)
        torch.cuda.synchronize()
    finally:
        oz.oz2_set_gemm_algorithm(oz.OZ2_GEMM_AUTO)
    got = dC.cpu().numpy()
    del ws, dA, dB, dC
    if "C" not in _c3_oracle:
        print("oracle on all %d x %d outputs" % (m, n), flush=True)
        _c3_oracle["C"] = orc.dgemm(A, B, N).C
    ref = _c3_oracle["C"]
    bad = np.argwhere(got != ref)
    assert len(bad) == 0, "%d elements differ from the oracle, first at %s" % (len(bad), bad[:5].tolist())
    # same zeros with the same signs, and nothing that is not a number
    assert np.array_equal(np.signbit(got), np.signbit(ref)) and not np.isnan(got).any()


@pytest.mark.parametrize("m,n,k,N,phi", [
    (256, 256, 256, 14, 0.5),     # config 1
    (300, 200, 333, 5, 0.5),
    (64, 40, 1000, 20, 4.0),      # beta + 1 = 78 bits: two-level split
    (33, 17, 50, 26, 4.0),
    (70, 90, 4200, 16, 1.0),      # more than one chunk of the column-norm kernel
    (1, 1, 1, 2, 0.5),
])
def test_cauchy_schwarz_mode_all_stages(m, n, k, N, phi):
    rng = np.random.default_rng(m * 7 + n)
    A = (rng.random((m, k)) - 0.5) * np.exp(phi * rng.standard_normal((m, k)))
    B = (rng.random((k, n)) - 0.5) * np.exp(phi * rng.standard_normal((k, n)))
    if m > 4:
        A[3, :] = 0.0
        A[4, 1:] = 0.0
        A[2, :] *= 2.0**-200
    check_against_oracle(A, B, N, mode=1)


def test_cauchy_schwarz_mode_full_size_c4_sampled():
    cfg = inputs.CONFIGS["c4"]
    m, n, k, phi, N = cfg["m"], cfg["n"], cfg["k"], cfg["phi"], 14
    A = inputs.block(cfg["seed"], 0, m, k, phi)
    B = inputs.block(cfg["seed"], 1, k, n, phi)
    rng = np.random.default_rng(4)
    rows = np.unique(np.concatenate([[0, m - 1], rng.choice(m, 30, replace=False)]))
    cols = np.unique(np.concatenate([[0, n - 1], rng.choice(n, 30, replace=False)]))
    dA = torch.from_numpy(A.T).cuda().t()
    dB = torch.from_numpy(B.T).cuda().t()
    dC = torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda").t()
    ws = oz.Workspace(m, n, k, N)
    oz.oz2_set_shift_mode(1)
    try:
        oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N)
        torch.cuda.synchronize()
    finally:
        oz.oz2_set_shift_mode(0)
    got = dC[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()].cpu().numpy()
    Asub, Bsub = np.asfortranarray(A[rows, :]), np.asfortranarray(B[:, cols])
    ref = orc.dgemm(Asub, Bsub, N, mode=1).C
    Cx, S = orc.exact(Asub, Bsub)
    assert np.array_equal(got, ref)
    plain = orc.dgemm(Asub, Bsub, N, mode=0).C
    e_fast, e_plain = np.max(np.abs(got - Cx) / S), np.max(np.abs(plain - Cx) / S)
    print("N=14 at 16384^3: componentwise error Cauchy-Schwarz %.3g, simple bound %.3g" % (e_fast, e_plain), flush=True)
    assert e_fast < e_plain
    del ws


@pytest.mark.parametrize("m,n,k,N,phi", [
    (256, 256, 256, 14, 0.5),     # config 1
    (300, 200, 333, 5, 0.5),
    (64, 40, 1000, 20, 4.0),
    (33, 17, 50, 26, 4.0),        # 2^(b/2 + 7) > 2^75: two-level split
    (530, 70, 130, 16, 1.0),      # three row blocks and two column chunks of the product-maximum kernel
    (1, 1, 1, 2, 0.5),
])
def test_int8_product_mode_all_stages(m, n, k, N, phi):
    rng = np.random.default_rng(m * 11 + n)
    A = (rng.random((m, k)) - 0.5) * np.exp(phi * rng.standard_normal((m, k)))
    B = (rng.random((k, n)) - 0.5) * np.exp(phi * rng.standard_normal((k, n)))
    if m > 4:
        A[3, :] = 0.0
        A[4, 1:] = 0.0
        A[2, :] *= 2.0**-200
        A[5, 0] = 2.0**-1074      # far below the row's unit: its bound is one unit, not zero
        B[:, 1] = 0.0
    check_against_oracle(A, B, N, mode=2)


def test_int8_product_mode_full_size_c3_sampled_and_transposed():
    # the shifts depend on all rows and columns; both operands are handed over transposed, so each is read
    # by the stage-1 kernels of the other orientation
    cfg = inputs.CONFIGS["c3"]
    m, n, k, phi, N = cfg["m"], cfg["n"], cfg["k"], cfg["phi"], 15
    A = inputs.block(cfg["seed"], 0, m, k, phi)
    B = inputs.block(cfg["seed"], 1, k, n, phi)
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, m - 1], rng.choice(m, 20, replace=False)]))
    cols = np.unique(np.concatenate([[0, n - 1], rng.choice(n, 20, replace=False)]))
    ref = orc.dgemm(A, B, N, mode=2, rows=rows, cols=cols, want=("C", "shifts"))
    dAt, dBt = _dev(A.T), _dev(B.T)      # stored k x m and n x k, column-major
    dC = torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda").t()
    ws = oz.Workspace(m, n, k, N)
    oz.oz2_set_shift_mode(2)
    try:
        print("int8-product mode, transposed operands, m=%d n=%d k=%d N=%d" % (m, n, k, N), flush=True)
        oz.oz2_dgemm_ex("T", "T", m, n, k, 1.0, dAt.data_ptr(), k, dBt.data_ptr(), n, 0.0, dC.data_ptr(), m, N)
        torch.cuda.synchronize()
    finally:
        oz.oz2_set_shift_mode(0)
    lay = oz.workspace_layout(m, n, k, N)
    sa = ws.view(lay["sa"], lay["m_pad"], torch.int32).cpu().numpy()
    sb = ws.view(lay["sb"], lay["n_pad"], torch.int32).cpu().numpy()
    assert np.array_equal(sa[rows], ref.sa) and np.array_equal(sb[cols], ref.sb)
    got = dC[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()].cpu().numpy()
    assert np.array_equal(got, ref.C)
    Asub, Bsub = np.asfortranarray(A[rows, :]), np.asfortranarray(B[:, cols])
    Cx, S = orc.exact(Asub, Bsub)
    e_prod = np.max(np.abs(got - Cx) / S)
    e_plain = np.max(np.abs(orc.dgemm(Asub, Bsub, N, mode=0).C - Cx) / S)
    print("N=15 at 4096^3: componentwise error INT8-product bound %.3g, simple bound %.3g" % (e_prod, e_plain), flush=True)
    assert e_prod < e_plain
    del ws


@pytest.mark.parametrize("ta,tb", [("N", "N"), ("T", "N"), ("N", "T"), ("T", "T")])
@pytest.mark.parametrize("alpha,beta", [(1.0, 0.0), (-0.75, 1.5), (2.0, 1.0)])
def test_dgemm_ex_transposes_and_scalars(ta, tb, alpha, beta):
    rng = np.random.default_rng(11)
    m, n, k, N = 300, 270, 333, 15
    opA = (rng.random((m, k)) - 0.5) * np.exp(rng.standard_normal((m, k)))
    opB = (rng.random((k, n)) - 0.5) * np.exp(rng.standard_normal((k, n)))
    As = np.asfortranarray(opA.T if ta == "T" else opA)   # as stored
    Bs = np.asfortranarray(opB.T if tb == "T" else opB)
    C0 = np.asfortranarray(rng.standard_normal((m, n)))
    if beta == 0.0:
        C0[:] = np.nan      # must not be read
    dA, dB = _dev(As), _dev(Bs)
    dC = torch.from_numpy(np.ascontiguousarray(C0.T)).cuda().t()
    ws = oz.Workspace(m, n, k, N)
    oz.oz2_dgemm_ex(ta, tb, m, n, k, alpha, dA.data_ptr(), As.shape[0], dB.data_ptr(), Bs.shape[0], beta,
                    dC.data_ptr(), m, N)
    torch.cuda.synchronize()
    got = dC.cpu().numpy()
    ref = orc.dgemm_ex(ta, tb, alpha, As, Bs, beta, C0, N)
    assert np.array_equal(got, ref)
    del ws


def test_dgemm_ex_degenerate_cases():
    m, n, k, N = 40, 30, 50, 8
    rng = np.random.default_rng(2)
    C0 = np.asfortranarray(rng.standard_normal((m, n)))
    dC = torch.from_numpy(np.ascontiguousarray(C0.T)).cuda().t()
    dX = torch.full((64, 64), float("nan"), dtype=torch.float64, device="cuda")
    ws = oz.Workspace(m, n, k, N)
    # alpha == 0: C := beta * C, A and B untouched (NaN-filled here)
    oz.oz2_dgemm_ex("N", "N", m, n, k, 0.0, dX.data_ptr(), 64, dX.data_ptr(), 64, 0.5, dC.data_ptr(), m, N)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), 0.5 * C0)
    # k == 0 and beta == 0: zeros
    oz.oz2_dgemm_ex("T", "T", m, n, 0, 1.0, None, 1, None, n, 0.0, dC.data_ptr(), m, N)
    torch.cuda.synchronize()
    assert not dC.cpu().numpy().any()
    L = oz.lib()
    st = torch.cuda.current_stream().cuda_stream
    assert L.oz2_dgemm_ex(b"X", b"N", 4, 4, 4, 1.0, dX.data_ptr(), 4, dX.data_ptr(), 4, 0.0, dC.data_ptr(), 4, 8, st) == -1
    assert L.oz2_dgemm_ex(b"T", b"N", 4, 4, 9, 1.0, dX.data_ptr(), 8, dX.data_ptr(), 9, 0.0, dC.data_ptr(), 4, 8, st) == -8
    assert L.oz2_dgemm_ex(b"N", b"T", 4, 7, 9, 1.0, dX.data_ptr(), 4, dX.data_ptr(), 6, 0.0, dC.data_ptr(), 4, 8, st) == -10
    del ws


def test_inner_dimension_beyond_int32_exactness():
    # k > 2^17: one INT32 accumulation would overflow (Section 3.1); the default k-block of 65536 applies
    rng = np.random.default_rng(13)
    m, n, k, N = 48, 40, 140000, 16
    A = rng.standard_normal((m, k))
    B = rng.standard_normal((k, n))
    # a row and a column whose scaled integers are 2^(kappa-1) + 128: residue -128 modulo 256 in every
    # position, so the exact product for that modulus is k * 16384 > 2^31
    kap = orc.kappa(N, k)
    A[0, :] = 1.0 + 128.0 * 2.0 ** -(kap - 1)
    B[:, 0] = 1.0 + 128.0 * 2.0 ** -(kap - 1)
    B[:, 1] = 1.0 + 127.0 * 2.0 ** -(kap - 1)      # residue +127: the most negative products, -128 * 127 each
    got, ref = check_against_oracle(A, B, N, products_exact=False)
    check_against_oracle(A, B, N, fmt=1)
    # the exact products really exceed INT32 somewhere, on both sides, so blocking was needed
    assert np.max(ref.Cprod) > 2**31 and np.min(ref.Cprod) < -2**31


# ------------------------------------------------------------------ exceptional inputs: detection and FP64 fallback
def _flag(ws, m, n, k, N):
    lay = oz.workspace_layout(m, n, k, N)
    return int(ws.view(lay["flags"], 32, torch.int64).cpu().numpy()[0])


@pytest.mark.parametrize("ta,tb", [("N", "N"), ("T", "N"), ("N", "T"), ("T", "T")])
@pytest.mark.parametrize("where", ["A", "B"])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_nonfinite_inputs_fall_back_to_fp64(ta, tb, where, mode):
    # two sizes of C: up to 2^18 elements the blocks of the fallback ride in the launch of stage 3, above that
    # the fallback is a launch of its own
    for m, n in ((300, 200), (700, 600)):
        _nonfinite_case(ta, tb, where, mode, m, n)


def _nonfinite_case(ta, tb, where, mode, m, n):
    rng = np.random.default_rng(21)
    k, N = 150, 12
    opA = (rng.random((m, k)) - 0.5) * np.exp(rng.standard_normal((m, k)))
    opB = (rng.random((k, n)) - 0.5) * np.exp(rng.standard_normal((k, n)))
    X = opA if where == "A" else opB
    X[7, 3] = np.inf
    X[7, 9] = -np.inf
    X[140, 100] = np.nan
    X[m - 1 if where == "A" else k - 1, 0] = np.inf
    opB[3, 5] = 0.0 if where == "A" else opB[3, 5]          # inf * 0
    alpha, beta = -0.5, 2.0
    As = np.asfortranarray(opA.T if ta == "T" else opA)
    Bs = np.asfortranarray(opB.T if tb == "T" else opB)
    C0 = np.asfortranarray(rng.standard_normal((m, n)))
    dA, dB = _dev(As), _dev(Bs)
    dC = torch.from_numpy(np.ascontiguousarray(C0.T)).cuda().t()
    ws = oz.Workspace(m, n, k, N)
    oz.oz2_set_shift_mode(mode)
    try:
        print("non-finite %s, op %s%s, shift mode %d" % (where, ta, tb, mode), flush=True)
        oz.oz2_dgemm_ex(ta, tb, m, n, k, alpha, dA.data_ptr(), As.shape[0], dB.data_ptr(), Bs.shape[0], beta,
                        dC.data_ptr(), m, N)
        torch.cuda.synchronize()
    finally:
        oz.oz2_set_shift_mode(0)
    assert _flag(ws, m, n, k, N) == 1
    got = dC.cpu().numpy()
    ref = orc.dgemm_ex(ta, tb, alpha, As, Bs, beta, C0, N)
    # what is unique: where the NaNs and the infinities are, and the signs of the infinities
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    inf = np.isinf(ref)
    assert np.array_equal(np.isinf(got), inf) and np.array_equal(got[inf], ref[inf])
    # the rest: two FP64 evaluations of the same sums in different orders
    fin = np.isfinite(ref)
    S = abs(alpha) * (np.abs(np.nan_to_num(opA, nan=0.0, posinf=0.0, neginf=0.0)) @
                      np.abs(np.nan_to_num(opB, nan=0.0, posinf=0.0, neginf=0.0))) + abs(beta) * np.abs(C0)
    assert np.all(np.abs(got[fin] - ref[fin]) <= 2 * (k + 2) * 2.0**-53 * S[fin])
    assert fin.sum() > m * n // 2
    # the same buffers with finite inputs again: the flag clears and the emulation is back
    X[~np.isfinite(X)] = 1.0
    As = np.asfortranarray(opA.T if ta == "T" else opA)
    Bs = np.asfortranarray(opB.T if tb == "T" else opB)
    dA, dB = _dev(As), _dev(Bs)
    dC = torch.from_numpy(np.ascontiguousarray(C0.T)).cuda().t()
    oz.oz2_dgemm_ex(ta, tb, m, n, k, alpha, dA.data_ptr(), As.shape[0], dB.data_ptr(), Bs.shape[0], beta, dC.data_ptr(), m, N)
    torch.cuda.synchronize()
    assert _flag(ws, m, n, k, N) == 0
    assert np.array_equal(dC.cpu().numpy(), orc.dgemm_ex(ta, tb, alpha, As, Bs, beta, C0, N))
    del ws


@pytest.mark.parametrize("m,n,k", [(1, 5000, 7), (5000, 1, 7), (1, 1, 1), (129, 2031, 3), (262144, 1, 2)])
def test_nonfinite_fallback_on_skinny_shapes(m, n, k):
    """The fallback's tiles ride in the launch of stage 3 for small C: shapes where its tile grid and the CRT grid
    have nothing in common (one row, one column, one element), an infinity in A and a NaN in B."""
    rng = np.random.default_rng(m + 3 * n)
    A = np.asfortranarray(rng.standard_normal((m, k)))
    B = np.asfortranarray(rng.standard_normal((k, n)))
    A[m - 1, k - 1] = np.inf
    B[0, n // 2] = np.nan
    N = 10
    dA, dB = _dev(A), _dev(B)
    dC = torch.full((n, m), 7.0, dtype=torch.float64, device="cuda").t()
    ws = oz.Workspace(m, n, k, N)
    oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N)
    torch.cuda.synchronize()
    assert _flag(ws, m, n, k, N) == 1
    got = dC.cpu().numpy()
    with np.errstate(invalid="ignore"):
        ref = A @ B
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    inf = np.isinf(ref)
    assert np.array_equal(np.isinf(got), inf) and np.array_equal(got[inf], ref[inf])
    fin = np.isfinite(ref)
    assert np.allclose(got[fin], ref[fin], rtol=1e-13, atol=1e-13)
    # and finite again: the emulation, bit for bit
    A[m - 1, k - 1] = 1.0
    B[0, n // 2] = -1.0
    dA, dB = _dev(A), _dev(B)
    oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N)
    torch.cuda.synchronize()
    assert _flag(ws, m, n, k, N) == 0
    assert np.array_equal(dC.cpu().numpy(), orc.dgemm(A, B, N).C)
    del ws


@pytest.mark.parametrize("algorithm", [0, 1])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_signed_zeros_every_bit_of_c(algorithm, mode):
    """Negative zeros in A and B (scattered, whole rows and columns, products that meet only zeros): they count as
    zeros, an emulated zero is +0 as in an FP64 sum that starts from +0, and the update alpha P + beta C gives its
    zeros the IEEE signs.  Compared with the oracle on the bit patterns, so the sign of every zero is checked."""
    rng = np.random.default_rng(31)
    m, n, k, N = 300, 260, 150, 13
    A = (rng.random((m, k)) - 0.5) * np.exp(rng.standard_normal((m, k)))
    B = (rng.random((k, n)) - 0.5) * np.exp(rng.standard_normal((k, n)))
    A[rng.random((m, k)) < 0.2] = -0.0
    B[rng.random((k, n)) < 0.2] = -0.0
    A[1, :] = -0.0
    A[2, ::2] = -0.0
    A[2, 1::2] = 0.0
    B[:, 1] = -0.0
    A[4, :] = np.where(np.arange(k) % 2 == 0, -0.0, 1.0)
    B[:, 5] = np.where(np.arange(k) % 2 == 0, -3.0, -0.0)
    A, B = np.asfortranarray(A), np.asfortranarray(B)
    C0 = np.asfortranarray(np.where(rng.random((m, n)) < 0.3, -0.0, rng.standard_normal((m, n))))
    dA, dB = _dev(A), _dev(B)
    oz.oz2_set_gemm_algorithm(algorithm)
    oz.oz2_set_shift_mode(mode)
    try:
        ws = oz.Workspace(m, n, k, N)
        for alpha, beta in [(1.0, 0.0), (-0.5, 0.0), (-0.5, 2.0), (1.0, -1.0)]:
            print("signed zeros: form %d, shift mode %d, alpha %g beta %g" % (algorithm, mode, alpha, beta), flush=True)
            dC = torch.from_numpy(np.ascontiguousarray(C0.T)).cuda().t()
            oz.oz2_dgemm_ex("N", "N", m, n, k, alpha, dA.data_ptr(), m, dB.data_ptr(), k, beta, dC.data_ptr(), m, N)
            torch.cuda.synchronize()
            assert _flag(ws, m, n, k, N) == 0     # nothing to fall back for
            got = dC.cpu().numpy()
            ref = orc.dgemm_ex("N", "N", alpha, A, B, beta, C0, N, mode=mode)
            assert np.array_equal(got.view(np.uint64), ref.view(np.uint64))
            if beta == 0.0:
                assert (got == 0).sum() >= m + n - 1 and not np.signbit(got[got == 0]).any()
        del ws
    finally:
        oz.oz2_set_gemm_algorithm(oz.OZ2_GEMM_AUTO)
        oz.oz2_set_shift_mode(0)


def test_nonfinite_check_can_be_switched_off():
    rng = np.random.default_rng(22)
    m, n, k, N = 64, 64, 64, 10
    A = rng.standard_normal((m, k))
    B = rng.standard_normal((k, n))
    A[1, 1] = np.nan
    dA, dB = _dev(A), _dev(B)
    dC = torch.full((n, m), 7.0, dtype=torch.float64, device="cuda").t()
    ws = oz.Workspace(m, n, k, N)
    oz.oz2_set_nonfinite_check(0)
    try:
        oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N)
        torch.cuda.synchronize()
    finally:
        oz.oz2_set_nonfinite_check(1)
    assert _flag(ws, m, n, k, N) == 1          # stage 1 still records what it saw
    got = dC.cpu().numpy()
    # rows of A without the NaN are untouched by it: the emulated values, not the 7.0 fill
    ref = orc.dgemm(np.delete(A, 1, axis=0), B, N).C
    assert np.array_equal(np.delete(got, 1, axis=0), ref)
    del ws


# ------------------------------------------------------------------ symmetric rank-k update
@pytest.mark.parametrize("uplo", ["L", "U"])
@pytest.mark.parametrize("trans", ["N", "T"])
@pytest.mark.parametrize("mode,fmt", [(0, 1), (1, 1), (2, 1), (0, 0)])
def test_dsyrk_matches_the_oracle_and_leaves_the_other_triangle(uplo, trans, mode, fmt):
    rng = np.random.default_rng(31)
    n, k, N = 600, 200, 13          # 3 x 3 tiles: six of them in the triangle
    opA = (rng.random((n, k)) - 0.5) * np.exp(rng.standard_normal((n, k)))
    opA[5, :] = 0.0
    As = np.asfortranarray(opA.T if trans == "T" else opA)
    alpha, beta = 1.5, -0.25
    C0 = np.asfortranarray(rng.standard_normal((n, n)))
    ii, jj = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    outside = (ii < jj) if uplo == "L" else (ii > jj)
    C0[outside] = np.nan            # never read, never written
    dA = _dev(As)
    dC = torch.from_numpy(np.ascontiguousarray(C0.T)).cuda().t()
    ws = oz.Workspace(n, n, k, N)
    oz.oz2_set_shift_mode(mode)
    oz.oz2_set_product_format(fmt)
    try:
        print("dsyrk uplo=%s trans=%s mode=%d fmt=%d" % (uplo, trans, mode, fmt), flush=True)
        oz.oz2_dsyrk(uplo, trans, n, k, alpha, dA.data_ptr(), As.shape[0], beta, dC.data_ptr(), n, N)
        torch.cuda.synchronize()
    finally:
        oz.oz2_set_shift_mode(0)
        oz.oz2_set_product_format(1)
    got = dC.cpu().numpy()
    assert np.all(np.isnan(got[outside])) and not np.any(np.isnan(got[~outside]))
    C0z = np.where(outside, 0.0, C0)
    ref = orc.dsyrk(uplo, trans, alpha, As, beta, np.asfortranarray(C0z), N, mode=mode)
    assert np.array_equal(got[~outside], ref[~outside])
    del ws


@pytest.mark.parametrize("uplo", ["L", "U"])
def test_dsyrk_every_element_where_the_crt_runs_on_the_matrix_cores(uplo):
    """A symmetric update with more than 2^24 elements of C and 12 moduli: stages 3 and 4 run in the matrix-core
    kernel, which has to keep to the triangle (rows of a thread's four on both sides of the diagonal, ragged last
    rows); every element of the triangle against the oracle, the other triangle untouched."""
    rng = np.random.default_rng(33)
    n, k, N = 4100, 48, 12
    assert n * n >= 1 << 24
    A = np.asfortranarray((rng.random((n, k)) - 0.5) * np.exp(rng.standard_normal((n, k))))
    alpha, beta = -0.5, 1.25
    C0 = np.asfortranarray(rng.standard_normal((n, n)))
    ii, jj = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    outside = (ii < jj) if uplo == "L" else (ii > jj)
    C0[outside] = np.nan            # never read, never written
    dA = _dev(A)
    dC = torch.from_numpy(np.ascontiguousarray(C0.T)).cuda().t()
    ws = oz.Workspace(n, n, k, N)
    print("dsyrk %d x %d, uplo=%s" % (n, n, uplo), flush=True)
    oz.oz2_dsyrk(uplo, "N", n, k, alpha, dA.data_ptr(), n, beta, dC.data_ptr(), n, N)
    torch.cuda.synchronize()
    got = dC.cpu().numpy()
    del ws, dC
    assert np.all(np.isnan(got[outside])) and not np.any(np.isnan(got[~outside]))
    ref = orc.dsyrk(uplo, "N", alpha, A, beta, np.asfortranarray(np.where(outside, 0.0, C0)), N)
    assert np.array_equal(got[~outside], ref[~outside])


def test_dsyrk_degenerate_and_nonfinite():
    rng = np.random.default_rng(32)
    n, k, N = 70, 40, 9
    A = np.asfortranarray(rng.standard_normal((n, k)))
    C0 = np.asfortranarray(rng.standard_normal((n, n)))
    low = np.tril(np.ones((n, n), dtype=bool))
    ws = oz.Workspace(n, n, k, N)
    dA = _dev(A)
    # alpha == 0 and k == 0: only the triangle is scaled
    for kk, alpha in ((k, 0.0), (0, 1.0)):
        dC = torch.from_numpy(np.ascontiguousarray(C0.T)).cuda().t()
        oz.oz2_dsyrk("L", "N", n, kk, alpha, dA.data_ptr(), n, 3.0, dC.data_ptr(), n, N)
        torch.cuda.synchronize()
        got = dC.cpu().numpy()
        assert np.array_equal(got[low], 3.0 * C0[low]) and np.array_equal(got[~low], C0[~low])
    # an infinity in A: FP64 fallback on the triangle only
    A2 = A.copy()
    A2[3, 4] = np.inf
    dA2 = _dev(A2)
    dC = torch.from_numpy(np.ascontiguousarray(C0.T)).cuda().t()
    oz.oz2_dsyrk("L", "N", n, k, 1.0, dA2.data_ptr(), n, 0.0, dC.data_ptr(), n, N)
    torch.cuda.synchronize()
    got = dC.cpu().numpy()
    ref = orc.dsyrk("L", "N", 1.0, A2, 0.0, C0, N)
    assert np.array_equal(got[~low], C0[~low])
    assert np.array_equal(np.isnan(got), np.isnan(ref)) and np.array_equal(np.isinf(got), np.isinf(ref))
    fin = np.isfinite(ref) & low
    S = np.abs(np.nan_to_num(A2, posinf=0.0)) @ np.abs(np.nan_to_num(A2, posinf=0.0)).T
    assert np.all(np.abs(got[fin] - ref[fin]) <= 2 * (k + 2) * 2.0**-53 * S[fin])
    # argument checks
    L = oz.lib()
    assert L.oz2_dsyrk(b"X", b"N", n, k, 1.0, dA.data_ptr(), n, 0.0, dC.data_ptr(), n, N, None) == -1
    assert L.oz2_dsyrk(b"L", b"Q", n, k, 1.0, dA.data_ptr(), n, 0.0, dC.data_ptr(), n, N, None) == -2
    assert L.oz2_dsyrk(b"L", b"N", n, k, 1.0, dA.data_ptr(), n - 1, 0.0, dC.data_ptr(), n, N, None) == -7
    assert L.oz2_dsyrk(b"L", b"T", n, k, 1.0, dA.data_ptr(), k - 1, 0.0, dC.data_ptr(), n, N, None) == -7
    assert L.oz2_dsyrk(b"L", b"N", n, k, 1.0, dA.data_ptr(), n, 0.0, dC.data_ptr(), n - 1, N, None) == -10
    del ws


# ------------------------------------------------------------------ stream capture
def test_hip_graph_replays_match_eager_calls():
    # the whole call is kernel launches on the caller's stream (no allocation, no memset, no synchronisation),
    # so it can be captured once and replayed; every replay is checked, with eager work and synchronisation
    # in between, and with new input values in the captured buffers
    m, n, k, N = 300, 260, 400, 14
    rng = np.random.default_rng(41)
    ws = oz.Workspace(m, n, k, N)
    dA = torch.zeros((k, m), dtype=torch.float64, device="cuda").t()
    dB = torch.zeros((n, k), dtype=torch.float64, device="cuda").t()
    dC = torch.zeros((n, m), dtype=torch.float64, device="cuda").t()
    dE = torch.zeros((n, m), dtype=torch.float64, device="cuda").t()

    def load(seed):
        r = np.random.default_rng(seed)
        A = (r.random((m, k)) - 0.5) * np.exp(r.standard_normal((m, k)))
        B = (r.random((k, n)) - 0.5) * np.exp(r.standard_normal((k, n)))
        dA.copy_(_dev(A))
        dB.copy_(_dev(B))
        return A, B

    load(0)
    oz.oz2_init()            # kernel attributes cannot be set under capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    print("capturing oz2_dgemm", flush=True)
    with torch.cuda.graph(graph, stream=side):
        oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N, torch.cuda.current_stream())
    for rep in range(4):
        A, B = load(100 + rep)
        if rep == 2:
            A[5, 7] = np.nan            # the fallback decision is taken on the device: it replays too
            dA.copy_(_dev(A))
        oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dE.data_ptr(), m, N)    # eager
        torch.cuda.synchronize()
        dC.fill_(-1.0)
        print("replay %d" % rep, flush=True)
        graph.replay()
        torch.cuda.synchronize()
        got, eager = dC.cpu().numpy(), dE.cpu().numpy()
        assert np.array_equal(got, eager, equal_nan=True)
        if rep != 2:
            assert np.array_equal(got, orc.dgemm(A, B, N).C)
        else:
            assert np.isnan(got[5, :]).all() and np.isfinite(np.delete(got, 5, axis=0)).all()
    del graph, ws


# ------------------------------------------------------------------ triangular product, in place
def _garbage_outside(A, uplo, diag):
    """NaN wherever the routine must not look."""
    G = A.copy()
    ka = A.shape[0]
    ii, jj = np.meshgrid(np.arange(ka), np.arange(ka), indexing="ij")
    G[(ii < jj) if uplo == "L" else (ii > jj)] = np.nan
    if diag == "U":
        G[np.arange(ka), np.arange(ka)] = np.nan
    return np.asfortranarray(G)


@pytest.mark.parametrize("side", ["L", "R"])
@pytest.mark.parametrize("uplo", ["L", "U"])
@pytest.mark.parametrize("transa", ["N", "T"])
@pytest.mark.parametrize("diag,mode", [("N", 0), ("U", 0), ("N", 1), ("U", 2)])
def test_dtrmm_matches_the_oracle_in_place(side, uplo, transa, diag, mode):
    rng = np.random.default_rng(51)
    m, n, N = 300, 520, 13          # order of A: 300 (two diagonal blocks) or 520 (three)
    ka = m if side == "L" else n
    A = (rng.random((ka, ka)) - 0.5) * np.exp(rng.standard_normal((ka, ka)))
    B = np.asfortranarray((rng.random((m, n)) - 0.5) * np.exp(rng.standard_normal((m, n))))
    B[4, :] = 0.0
    G = _garbage_outside(A, uplo, diag)
    ldb = m + 3
    hB = np.full((ldb, n), 7.0, order="F")
    hB[:m, :] = B
    dA = _dev(G)
    dB = torch.from_numpy(np.ascontiguousarray(hB.T)).cuda().t()
    ws = oz.Workspace(m, n, ka, N)
    oz.oz2_set_shift_mode(mode)
    try:
        print("dtrmm side=%s uplo=%s trans=%s diag=%s mode=%d" % (side, uplo, transa, diag, mode), flush=True)
        oz.oz2_dtrmm(side, uplo, transa, diag, m, n, -1.25, dA.data_ptr(), ka, dB.data_ptr(), ldb, N)
        torch.cuda.synchronize()
    finally:
        oz.oz2_set_shift_mode(0)
    lay = oz.workspace_layout(m, n, ka, N)
    assert int(ws.view(lay["flags"], 32, torch.int64).cpu().numpy()[0]) == 0     # the NaNs outside were never looked at
    got = dB.cpu().numpy()
    ref = orc.dtrmm(side, uplo, transa, diag, -1.25, G, B, N, mode=mode)
    assert np.array_equal(got[:m, :], ref)
    assert np.all(got[m:, :] == 7.0)            # the padding rows of B's array are untouched
    del ws


def test_dtrmm_every_element_where_the_crt_runs_on_the_matrix_cores():
    """A triangular product with more than 2^24 elements of B and 12 moduli (stages 3 and 4 in the matrix-core
    kernel, written into the staging buffer of the in-place product): every element against the oracle."""
    rng = np.random.default_rng(52)
    m, n, N = 16390, 1030, 12       # B := alpha * B * op(A), A of order 1030
    assert m * n >= 1 << 24
    A = (rng.random((n, n)) - 0.5) * np.exp(rng.standard_normal((n, n)))
    B = np.asfortranarray((rng.random((m, n)) - 0.5) * np.exp(rng.standard_normal((m, n))))
    G = _garbage_outside(A, "L", "N")
    dA = _dev(G)
    dB = _dev(B)
    ws = oz.Workspace(m, n, n, N)
    print("dtrmm %d x %d, right lower" % (m, n), flush=True)
    oz.oz2_dtrmm("R", "L", "N", "N", m, n, 0.75, dA.data_ptr(), n, dB.data_ptr(), m, N)
    torch.cuda.synchronize()
    got = dB.cpu().numpy()
    del ws, dA, dB
    ref = orc.dtrmm("R", "L", "N", "N", 0.75, G, B, N)
    assert np.array_equal(got, ref)


def test_dtrmm_degenerate_nonfinite_and_arguments():
    rng = np.random.default_rng(52)
    m, n, N = 90, 60, 9
    A = np.asfortranarray(np.tril(rng.standard_normal((m, m))))
    B = np.asfortranarray(rng.standard_normal((m, n)))
    ws = oz.Workspace(m, n, m, N)
    dA = _dev(A)
    # alpha == 0: B := 0, A not read
    dB = _dev(B).clone()
    dN = torch.full((m, m), float("nan"), dtype=torch.float64, device="cuda")
    oz.oz2_dtrmm("L", "L", "N", "N", m, n, 0.0, dN.data_ptr(), m, dB.data_ptr(), m, N)
    torch.cuda.synchronize()
    assert np.array_equal(dB.cpu().numpy(), np.zeros((m, n)))
    # an infinity inside the triangle: FP64 fallback, in place through the workspace
    A2 = A.copy()
    A2[40, 3] = np.inf
    B2 = B.copy()
    B2[3, 5] = 0.0
    dA2, dB = _dev(A2), _dev(B2).clone()
    oz.oz2_dtrmm("L", "L", "N", "N", m, n, 2.0, dA2.data_ptr(), m, dB.data_ptr(), m, N)
    torch.cuda.synchronize()
    got = dB.cpu().numpy()
    ref = orc.dtrmm("L", "L", "N", "N", 2.0, A2, B2, N)
    assert np.array_equal(np.isnan(got), np.isnan(ref)) and np.isnan(ref[40, 5])
    inf = np.isinf(ref)
    assert np.array_equal(np.isinf(got), inf) and np.array_equal(got[inf], ref[inf]) and inf.sum() == n - 1
    fin = np.isfinite(ref)
    S = 2.0 * np.abs(np.nan_to_num(A2, posinf=0.0)) @ np.abs(B2)
    assert np.all(np.abs(got[fin] - ref[fin]) <= 2 * (m + 2) * 2.0**-53 * S[fin])
    # argument checks
    L = oz.lib()
    args = lambda **kw: [kw.get("side", b"L"), kw.get("uplo", b"L"), kw.get("trans", b"N"), kw.get("diag", b"N"),
                         kw.get("m", m), kw.get("n", n), 1.0, dA.data_ptr(), kw.get("lda", m), dB.data_ptr(), kw.get("ldb", m),
                         kw.get("N", N), None]
    assert L.oz2_dtrmm(*args(side=b"X")) == -1 and L.oz2_dtrmm(*args(uplo=b"X")) == -2
    assert L.oz2_dtrmm(*args(trans=b"X")) == -3 and L.oz2_dtrmm(*args(diag=b"X")) == -4
    assert L.oz2_dtrmm(*args(m=-1)) == -5 and L.oz2_dtrmm(*args(n=-1)) == -6
    assert L.oz2_dtrmm(*args(lda=m - 1)) == -9 and L.oz2_dtrmm(*args(ldb=m - 1)) == -11
    assert L.oz2_dtrmm(*args(side=b"R", lda=n - 1)) == -9 and L.oz2_dtrmm(*args(N=1)) == -12
    del ws


# ------------------------------------------------------------------ structured products on the super-block tile order
def test_dsyrk_and_dtrmm_at_4096_sampled():
    # 16 x 16 tiles: the tile order that shares a super-block between the XCDs, with its triangle of tiles
    # skipped (dsyrk) or its inner dimension cut at the diagonal block (dtrmm); outputs checked on sampled rows
    # and columns, the diagonal blocks included
    n = k = 4096
    N = 15
    A = inputs.block(250408003, 0, n, k, 1.0)
    B = inputs.block(250408003, 1, k, n, 1.0)
    rng = np.random.default_rng(8)
    rows = np.unique(np.concatenate([[0, 255, 256, n - 1], rng.choice(n, 12, replace=False)]))
    cols = np.unique(np.concatenate([[0, 255, 256, n - 1], rng.choice(n, 12, replace=False)]))
    drows, dcols = torch.from_numpy(rows).cuda(), torch.from_numpy(cols).cuda()
    dA = _dev(A)
    ws = oz.Workspace(n, n, k, N)
    # --- dsyrk, lower
    dC = torch.zeros((n, n), dtype=torch.float64, device="cuda").t()
    print("dsyrk n=k=4096", flush=True)
    oz.oz2_dsyrk("L", "N", n, k, 1.0, dA.data_ptr(), n, 0.0, dC.data_ptr(), n, N)
    torch.cuda.synchronize()
    got = dC[drows][:, dcols].cpu().numpy()
    ref = orc.dgemm(A, A.T, N, rows=rows, cols=cols).C
    low = rows[:, None] >= cols[None, :]
    assert np.array_equal(got[low], ref[low]) and np.all(got[~low] == 0.0)
    # --- dtrmm, left, upper, transposed: op(A) = A^T is lower triangular
    T = orc.triangular(A, "U", "N")
    dB = _dev(B).clone()
    print("dtrmm n=k=4096", flush=True)
    oz.oz2_dtrmm("L", "U", "T", "N", n, n, 1.0, dA.data_ptr(), n, dB.data_ptr(), n, N)
    torch.cuda.synchronize()
    got = dB[drows][:, dcols].cpu().numpy()
    ref = orc.dgemm(T.T, B, N, rows=rows, cols=cols).C
    assert np.array_equal(got, ref)
    # --- dtrmm, right, upper: the second operand is triangular
    dB = _dev(B).clone()
    oz.oz2_dtrmm("R", "U", "N", "N", n, n, 1.0, dA.data_ptr(), n, dB.data_ptr(), n, N)
    torch.cuda.synchronize()
    got = dB[drows][:, dcols].cpu().numpy()
    ref = orc.dgemm(B, T, N, rows=rows, cols=cols).C
    assert np.array_equal(got, ref)
    del ws


# ------------------------------------------------------------------ unequal bit budgets
@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("N,delta", [(12, 8), (12, -5), (15, 1), (26, 8)])
def test_unequal_bit_budgets_all_stages(mode, N, delta):
    rng = np.random.default_rng(61 + N)
    m, n, k = 300, 200, 333
    A = (rng.random((m, k)) - 0.5) * np.exp(rng.standard_normal((m, k)))
    B = (rng.random((k, n)) - 0.5) * np.exp(rng.standard_normal((k, n)))
    A[3, :] = 0.0
    check_against_oracle(A, B, N, mode=mode, delta=delta)


def test_bit_split_out_of_budget_is_refused():
    m = n = k = 64
    ws = oz.Workspace(m, n, k, 4)
    dX = torch.zeros((64, 64), dtype=torch.float64, device="cuda")
    kap = orc.kappa(4, k)
    oz.oz2_set_bit_split(kap)           # k_A = 0
    try:
        assert oz.lib().oz2_stage1_convert(m, n, k, dX.data_ptr(), m, dX.data_ptr(), k, 4, None) == 2
        oz.oz2_set_bit_split(kap - 1)   # k_A = 1
        assert oz.lib().oz2_stage1_convert(m, n, k, dX.data_ptr(), m, dX.data_ptr(), k, 4, None) == 0
        torch.cuda.synchronize()
    finally:
        oz.oz2_set_bit_split(0)
    assert oz.lib().oz2_set_bit_split(101) == -1
    del ws
