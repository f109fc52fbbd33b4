"""oz2_dgemm_static -- the entry point for callers that cannot allocate -- against oz2_dgemm, through the C ABI.

The static workspace is shared by all calls on the GPU and keeps the last call's contents, so the check is made on
two calls in a row, the second with a smaller problem: every byte the second call reads must be its own."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2504_08009_amd as oz
from oracle import oracle as orc
from paper_2504_08009_amd import inputs


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x.T)).cuda().t()


def _both(L, A, B, N, stream):
    """C from oz2_dgemm (registered workspace) and from oz2_dgemm_static (no workspace registered), bit patterns"""
    m, k = A.shape
    _, n = B.shape
    dA, dB = _dev(A), _dev(B)
    out = []
    for static in (False, True):
        dC = torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda").t()
        args = (m, n, k, ctypes.c_void_p(dA.data_ptr()), m, ctypes.c_void_p(dB.data_ptr()), k,
                ctypes.c_void_p(dC.data_ptr()), m, N, ctypes.c_void_p(stream))
        if static:
            oz.set_workspace(None, 0)          # nothing registered: the call must not need it
            rc = L.oz2_dgemm_static(*args)
        else:
            ws = oz.Workspace(m, n, k, N)
            rc = L.oz2_dgemm(*args)
        assert rc == 0, rc
        torch.cuda.synchronize()
        out.append(dC.cpu().numpy().copy())
        if not static:
            del ws
    return out


def test_static_workspace_entry_point_matches_oz2_dgemm():
    L = oz.lib()
    assert L.oz2_init() == 0
    stream = torch.cuda.current_stream().cuda_stream
    # first call: 1000 x 900 x 1024 with 16 moduli (ragged tiles, close to the limit of the static buffer);
    # second call: a smaller, differently shaped problem on the same buffer
    for (m, n, k, N, seed) in [(1000, 900, 1024, 16, 11), (300, 257, 200, 14, 12)]:
        print("static entry point: m=%d n=%d k=%d N=%d" % (m, n, k, N), flush=True)
        assert oz.workspace_bytes(m, n, k, N, oz.OZ2_PRODUCT_RESIDUE_U8) <= oz.OZ2_STATIC_SCRATCH_BYTES
        A, B = inputs.gemm_inputs(seed, m, n, k, 0.5)
        ref, got = _both(L, A, B, N, stream)
        assert np.array_equal(got.view(np.uint64), ref.view(np.uint64))
        assert np.array_equal(got, orc.dgemm(A, B, N).C)


def test_static_workspace_entry_point_rejects_what_does_not_fit():
    L = oz.lib()
    m = n = k = 2048
    assert oz.workspace_bytes(m, n, k, 16, oz.OZ2_PRODUCT_RESIDUE_U8) > oz.OZ2_STATIC_SCRATCH_BYTES
    buf = torch.zeros(m * k, dtype=torch.float64, device="cuda")
    p = ctypes.c_void_p(buf.data_ptr())
    assert L.oz2_dgemm_static(m, n, k, p, m, p, k, p, m, 16, None) == 4        # OZ2_ERR_STATIC_LIMIT, nothing enqueued
    assert b"static" in L.oz2_status_string(4)
    assert L.oz2_dgemm_static(-1, n, k, p, m, p, k, p, m, 16, None) == -1      # argument codes as oz2_dgemm
    assert L.oz2_dgemm_static(0, n, k, p, 1, p, k, p, 1, 16, None) == 0        # empty: nothing to do
