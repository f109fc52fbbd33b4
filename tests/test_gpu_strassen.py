"""GPU parity of the Strassen form of the INT8 products (oz2_set_gemm_algorithm): the seven half-size products per
modulus are integer arithmetic modulo p_t, so the final C must be bit-identical with the oracle, which forms
Algorithm 1 line 6 as printed.  Sizes span several tiles per half, ragged tails and halves that are all padding."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2504_08009_amd as oz
from oracle import oracle as orc
from paper_2504_08009_amd import inputs


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x.T)).cuda().t()


class _Settings:
    """library settings for one test, restored afterwards"""

    def __init__(self, algorithm, mode=0, delta=0, kblock=None):
        self.algorithm, self.mode, self.delta, self.kblock = algorithm, mode, delta, kblock

    def __enter__(self):
        oz.oz2_set_gemm_algorithm(self.algorithm)
        oz.oz2_set_shift_mode(self.mode)
        oz.oz2_set_bit_split(self.delta)
        if self.kblock:
            oz.oz2_set_kblock(self.kblock)

    def __exit__(self, *exc):
        oz.oz2_set_gemm_algorithm(oz.OZ2_GEMM_AUTO)
        oz.oz2_set_shift_mode(0)
        oz.oz2_set_bit_split(0)
        oz.oz2_set_kblock(65536)


@pytest.mark.parametrize("m,n,k,N,phi,mode", [
    (300, 200, 333, 5, 0.5, 0),       # one tile per half, ragged everywhere
    (700, 900, 1100, 14, 1.0, 0),     # two row tiles per half, nine k-tiles per half, ragged tails
    (1030, 520, 130, 16, 0.5, 0),     # second halves nearly empty
    (64, 40, 1000, 20, 4.0, 0),       # wide exponent range
    (33, 17, 50, 23, 4.0, 0),         # kappa > 75: two-level split of the elements, 5 limbs
    (5, 3, 1, 26, 0.5, 0),            # k = 1: the second inner half is all padding
    (1, 1, 7, 2, 0.5, 0),             # smallest everything
    (1, 3000, 2000, 15, 1.0, 0),      # one row
    (2100, 3, 5000, 16, 0.5, 0),      # long inner dimension against a sliver of C
    (700, 900, 1100, 14, 1.0, 1),     # Cauchy-Schwarz shifts
    (520, 300, 700, 12, 4.0, 2),      # shifts from the INT8 product of bounds (its planes share the regions)
    (40, 30, 300000, 12, 0.5, 0),     # halves of 150016 > 2^17: three k-blocks per product by INT32 exactness alone
])
def test_strassen_form_is_bit_identical_with_the_oracle(m, n, k, N, phi, mode):
    rng = np.random.default_rng(m * 1000 + n + mode)
    A = np.asfortranarray((rng.random((m, k)) - 0.5) * np.exp(phi * rng.standard_normal((m, k))))
    B = np.asfortranarray((rng.random((k, n)) - 0.5) * np.exp(phi * rng.standard_normal((k, n))))
    dA, dB = _dev(A), _dev(B)
    dC = torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda").t()
    with _Settings(oz.OZ2_GEMM_STRASSEN, mode):
        ws = oz.Workspace(m, n, k, N)
        assert ws.nbytes >= oz.workspace_bytes_strassen(m, n, k, N)
        assert oz.oz2_gemm_algorithm_for(m, n, k, N) == oz.OZ2_GEMM_STRASSEN
        print("strassen m=%d n=%d k=%d N=%d mode=%d" % (m, n, k, N, mode), flush=True)
        oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N)
        torch.cuda.synchronize()
    got = dC.cpu().numpy()
    ref = orc.dgemm(A, B, N, mode=mode).C
    _, S = orc.exact(A, B)
    assert np.all(np.abs(got - ref) <= 1e-15 * S)
    assert np.array_equal(got, ref)
    del ws


@pytest.mark.parametrize("ta,tb", [("N", "N"), ("T", "N"), ("N", "T"), ("T", "T")])
@pytest.mark.parametrize("alpha,beta", [(1.0, 0.0), (-0.75, 1.5)])
def test_strassen_form_transposes_scalars_and_leading_dimensions(ta, tb, alpha, beta):
    rng = np.random.default_rng(17)
    m, n, k, N = 600, 530, 777, 15
    opA = (rng.random((m, k)) - 0.5) * np.exp(rng.standard_normal((m, k)))
    opB = (rng.random((k, n)) - 0.5) * np.exp(rng.standard_normal((k, n)))
    As = np.asfortranarray(opA.T if ta == "T" else opA)
    Bs = np.asfortranarray(opB.T if tb == "T" else opB)
    # stored inside larger arrays: leading dimensions above the row counts
    lda, ldb, ldc = As.shape[0] + 3, Bs.shape[0] + 5, m + 7
    Abig = np.full((lda, As.shape[1]), np.nan, order="F")
    Abig[:As.shape[0]] = As
    Bbig = np.full((ldb, Bs.shape[1]), np.nan, order="F")
    Bbig[:Bs.shape[0]] = Bs
    C0 = np.asfortranarray(rng.standard_normal((m, n)))
    if beta == 0.0:
        C0[:] = np.nan
    Cbig = np.full((ldc, n), -7.0, order="F")
    Cbig[:m] = C0
    dA, dB, dC = _dev(Abig), _dev(Bbig), _dev(Cbig)
    with _Settings(oz.OZ2_GEMM_STRASSEN):
        ws = oz.Workspace(m, n, k, N)
        oz.oz2_dgemm_ex(ta, tb, m, n, k, alpha, dA.data_ptr(), lda, dB.data_ptr(), ldb, beta, dC.data_ptr(), ldc, N)
        torch.cuda.synchronize()
    got = dC.cpu().numpy()
    ref = orc.dgemm_ex(ta, tb, alpha, As, Bs, beta, C0, N)
    assert np.array_equal(got[:m], ref)
    assert np.all(got[m:] == -7.0), "rows beyond m of the array holding C were written"
    del ws


def test_strassen_form_with_k_blocking_bit_split_and_nonfinite_fallback():
    rng = np.random.default_rng(23)
    m, n, k, N = 300, 280, 1500, 14
    A = np.asfortranarray((rng.random((m, k)) - 0.5) * np.exp(rng.standard_normal((m, k))))
    B = np.asfortranarray((rng.random((k, n)) - 0.5) * np.exp(rng.standard_normal((k, n))))
    dA, dB = _dev(A), _dev(B)
    # modular reductions of the accumulators between k-blocks of 128 (six per half)
    for delta in (0, 6):
        dC = torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda").t()
        with _Settings(oz.OZ2_GEMM_STRASSEN, 0, delta, kblock=128):
            ws = oz.Workspace(m, n, k, N)
            oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N)
            torch.cuda.synchronize()
        assert np.array_equal(dC.cpu().numpy(), orc.dgemm(A, B, N, delta=delta).C), "delta=%d" % delta
        del ws
    # an infinity in B: stage 1 flags it, the Strassen products and CRT pass stand back, the FP64 kernel forms C
    B2 = B.copy()
    B2[k // 2 + 5, n // 2 + 3] = np.inf
    dB2 = _dev(B2)
    dC = torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda").t()
    with _Settings(oz.OZ2_GEMM_STRASSEN):
        ws = oz.Workspace(m, n, k, N)
        oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB2.data_ptr(), k, dC.data_ptr(), m, N)
        torch.cuda.synchronize()
    ref = orc.dgemm_ex("N", "N", 1.0, A, B2, 0.0, np.zeros((m, n), order="F"), N)
    got = dC.cpu().numpy()
    # what is unique: where the NaNs and the infinities are, and the signs of the infinities
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    inf = np.isinf(ref)
    assert np.array_equal(np.isinf(got), inf) and np.array_equal(got[inf], ref[inf])
    # the rest: two FP64 evaluations of the same sums in different orders
    fin = np.isfinite(ref)
    S = np.abs(A) @ np.abs(np.where(np.isfinite(B2), B2, 0.0))
    assert np.all(np.abs(got[fin] - ref[fin]) <= 2 * (k + 2) * 2.0**-53 * S[fin])
    assert fin.sum() > m * n // 2
    del ws


def test_strassen_choice_and_workspace_rules():
    m = n = k = 700
    N = 12
    rng = np.random.default_rng(5)
    A = np.asfortranarray(rng.standard_normal((m, k)))
    B = np.asfortranarray(rng.standard_normal((k, n)))
    dA, dB = _dev(A), _dev(B)
    dC = torch.empty((n, m), dtype=torch.float64, device="cuda").t()
    # automatic choice: classical at this size
    ws = oz.Workspace(m, n, k, N)
    assert oz.oz2_gemm_algorithm_for(m, n, k, N) == oz.OZ2_GEMM_CLASSICAL
    del ws
    with _Settings(oz.OZ2_GEMM_STRASSEN):
        # forced, but the registered workspace only holds the classical form: refused, nothing launched
        small = oz.workspace_bytes(m, n, k, N, oz.OZ2_PRODUCT_RESIDUE_U8)
        assert small < oz.workspace_bytes_strassen(m, n, k, N)
        buf = torch.empty(small + 256, dtype=torch.uint8, device="cuda")
        ptr = buf.data_ptr() + (-buf.data_ptr()) % 256
        oz.set_workspace(ptr, small)
        with pytest.raises(oz.Oz2Error, match="status 1"):
            oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N)
        # INT32 product planes: the form does not apply, the classical one runs
        oz.oz2_set_product_format(oz.OZ2_PRODUCT_INT32)
        try:
            ws = oz.Workspace(m, n, k, N)
            assert oz.oz2_gemm_algorithm_for(m, n, k, N) == oz.OZ2_GEMM_CLASSICAL
            oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N)
            torch.cuda.synchronize()
        finally:
            oz.oz2_set_product_format(oz.OZ2_PRODUCT_RESIDUE_U8)
        assert np.array_equal(dC.cpu().numpy(), orc.dgemm(A, B, N).C)
        del ws
    # at the headline size the automatic choice is the Strassen form once the workspace holds it
    big = 16384
    assert oz.workspace_bytes_preferred(big, big, big, 16) == oz.workspace_bytes_strassen(big, big, big, 16)
    oz.set_workspace(None, 0)


def test_strassen_form_at_4096_sampled_outputs():
    """Many tiles per half (8 x 8 x 32 k-tiles, the super-block order of the GEMM, the round synchronisation) on
    config c3's inputs; the oracle recomputes sampled rows and columns, among them both sides of every half
    boundary."""
    cfg = inputs.CONFIGS["c3"]
    m, n, k, phi = cfg["m"], cfg["n"], cfg["k"], cfg["phi"]
    N = 16
    A = inputs.block(cfg["seed"], 0, m, k, phi)
    B = inputs.block(cfg["seed"], 1, k, n, phi)
    rng = np.random.default_rng(9)
    rows = np.unique(np.concatenate([[0, m // 2 - 1, m // 2, m - 1], rng.choice(m, 28, replace=False)]))
    cols = np.unique(np.concatenate([[0, n // 2 - 1, n // 2, n - 1], rng.choice(n, 28, replace=False)]))
    dA = torch.from_numpy(A.T).cuda().t()
    dB = torch.from_numpy(B.T).cuda().t()
    dC = torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda").t()
    with _Settings(oz.OZ2_GEMM_STRASSEN):
        ws = oz.Workspace(m, n, k, N)
        print("strassen c3", flush=True)
        oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N)
        torch.cuda.synchronize()
        # the classical form on the same inputs gives the same matrix, every element
        dC2 = torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda").t()
        oz.oz2_set_gemm_algorithm(oz.OZ2_GEMM_CLASSICAL)
        oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC2.data_ptr(), m, N)
        torch.cuda.synchronize()
    assert not bool(torch.isnan(dC).any())
    assert bool(torch.equal(dC, dC2)), "Strassen and classical forms differ"
    got = dC[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()].cpu().numpy()
    ref = orc.dgemm(np.asfortranarray(A[rows, :]), np.asfortranarray(B[:, cols]), N).C
    assert np.array_equal(got, ref)
    del ws


def test_strassen_form_in_a_hip_graph():
    """The Strassen form is kernel launches on the caller's stream like the classical one: captured once, replayed
    with new inputs in the captured buffers, every replay checked against an eager call and the oracle."""
    m, n, k, N = 520, 300, 700, 13
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

    with _Settings(oz.OZ2_GEMM_STRASSEN):
        ws = oz.Workspace(m, n, k, N)
        load(0)
        oz.oz2_init()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        print("capturing oz2_dgemm (Strassen form)", flush=True)
        with torch.cuda.graph(graph, stream=side):
            oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N, torch.cuda.current_stream())
        for rep in range(3):
            A, B = load(200 + rep)
            oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dE.data_ptr(), m, N)
            torch.cuda.synchronize()
            dC.fill_(-1.0)
            print("replay %d" % rep, flush=True)
            graph.replay()
            torch.cuda.synchronize()
            got = dC.cpu().numpy()
            assert np.array_equal(got, dE.cpu().numpy())
            assert np.array_equal(got, orc.dgemm(A, B, N).C)
        del graph, ws


def test_strassen_form_chosen_by_itself_at_a_large_ragged_size():
    """Just above the sizes from which the library takes the Strassen form by itself, with nothing a multiple of a
    tile: halves of 17 x 17 tiles (outside the super-block order of the GEMM), a ragged last tile in every
    dimension, the second halves one element shorter than the first.  Sampled rows and columns, among them both
    sides of the half boundaries and the last ones, against the oracle."""
    m, n, k, N, phi = 8193, 8447, 12289, 15, 1.0
    A = inputs.block(77, 0, m, k, phi)
    B = inputs.block(77, 1, k, n, phi)
    rng = np.random.default_rng(13)
    mh, nh = 4352, 4352   # halves: ceil(m/2), ceil(n/2) rounded up to 256
    rows = np.unique(np.concatenate([[0, mh - 1, mh, m - 1, 4096, 4097], rng.choice(m, 20, replace=False)]))
    cols = np.unique(np.concatenate([[0, nh - 1, nh, n - 1, 4223, 4224], rng.choice(n, 20, replace=False)]))
    dA = torch.from_numpy(A.T).cuda().t()
    dB = torch.from_numpy(B.T).cuda().t()
    dC = torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda").t()
    ws = oz.Workspace(m, n, k, N)
    assert oz.oz2_gemm_algorithm_for(m, n, k, N) == oz.OZ2_GEMM_STRASSEN
    print("strassen (automatic) m=%d n=%d k=%d N=%d" % (m, n, k, N), flush=True)
    oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(dC).any())
    got = dC[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()].cpu().numpy()
    ref = orc.dgemm(np.asfortranarray(A[rows, :]), np.asfortranarray(B[:, cols]), N).C
    assert np.array_equal(got, ref)
    del ws
