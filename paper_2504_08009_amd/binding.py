"""ctypes binding of liboz2.so.  Function names follow include/oz2.h; arguments are marshalled only."""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboz2.so")
_lib = None

SYMBOLS = [
    "oz2_init", "oz2_min_moduli", "oz2_moduli_for_bits", "oz2_max_moduli", "oz2_get_moduli", "oz2_workspace_bytes", "oz2_workspace_bytes_for", "oz2_set_workspace",
    "oz2_workspace_layout", "oz2_dgemm", "oz2_dgemm_static", "oz2_dgemm_ex", "oz2_dsyrk", "oz2_dtrmm", "oz2_stage1_convert", "oz2_stage2_gemm", "oz2_stage3_crt",
    "oz2_set_gemm_algorithm", "oz2_gemm_algorithm_for", "oz2_workspace_bytes_strassen", "oz2_workspace_bytes_preferred",
    "oz2_context_create", "oz2_context_destroy", "oz2_context_set_workspace", "oz2_context_set", "oz2_context_get",
    "oz2_context_workspace_bytes", "oz2_context_dgemm", "oz2_context_dsyrk", "oz2_context_dtrmm",
    "oz2_set_kblock", "oz2_set_round_sync", "oz2_set_shift_mode", "oz2_set_product_format", "oz2_set_bit_split", "oz2_set_nonfinite_check", "oz2_set_stage_events", "oz2_calibrate_mfma", "oz2_host_crt_element", "oz2_host_crt_element_digits", "oz2_host_residues", "oz2_status_string",
]


class Oz2Error(RuntimeError):
    pass


def lib():
    """Load liboz2.so (built by paper_2504_08009_amd/build.py).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise Oz2Error("liboz2.so is missing: run `python -c 'import __graft_entry__ as g; g.build()'` first")
        L = ctypes.CDLL(_LIB_PATH)
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        L.oz2_get_moduli.argtypes = [ci, vp, vp, i64]
        L.oz2_moduli_for_bits.argtypes = [i64, ci]
        L.oz2_workspace_bytes.restype = ctypes.c_size_t
        L.oz2_workspace_bytes.argtypes = [i64, i64, i64, ci]
        L.oz2_workspace_bytes_for.restype = ctypes.c_size_t
        L.oz2_workspace_bytes_for.argtypes = [i64, i64, i64, ci, ci]
        L.oz2_workspace_bytes_strassen.restype = ctypes.c_size_t
        L.oz2_workspace_bytes_strassen.argtypes = [i64, i64, i64, ci]
        L.oz2_workspace_bytes_preferred.restype = ctypes.c_size_t
        L.oz2_workspace_bytes_preferred.argtypes = [i64, i64, i64, ci]
        L.oz2_set_gemm_algorithm.argtypes = [ci]
        L.oz2_gemm_algorithm_for.argtypes = [i64, i64, i64, ci]
        L.oz2_set_workspace.argtypes = [vp, ctypes.c_size_t]
        L.oz2_workspace_layout.argtypes = [i64, i64, i64, ci, vp, vp]
        L.oz2_dgemm.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, ci, vp]
        L.oz2_dgemm_static.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, ci, vp]
        L.oz2_dgemm_ex.argtypes = [ctypes.c_char, ctypes.c_char, i64, i64, i64, ctypes.c_double, vp, i64, vp, i64,
                                   ctypes.c_double, vp, i64, ci, vp]
        L.oz2_dsyrk.argtypes = [ctypes.c_char, ctypes.c_char, i64, i64, ctypes.c_double, vp, i64, ctypes.c_double, vp, i64,
                                ci, vp]
        L.oz2_dtrmm.argtypes = [ctypes.c_char] * 4 + [i64, i64, ctypes.c_double, vp, i64, vp, i64, ci, vp]
        L.oz2_stage1_convert.argtypes = [i64, i64, i64, vp, i64, vp, i64, ci, vp]
        L.oz2_stage2_gemm.argtypes = [i64, i64, i64, ci, vp]
        L.oz2_stage3_crt.argtypes = [i64, i64, i64, vp, i64, ci, vp]
        L.oz2_set_kblock.argtypes = [i64]
        L.oz2_context_create.argtypes = [vp]
        L.oz2_context_destroy.argtypes = [vp]
        L.oz2_context_set_workspace.argtypes = [vp, vp, ctypes.c_size_t]
        L.oz2_context_set.argtypes = [vp, ci, i64]
        L.oz2_context_get.argtypes = [vp, ci, vp]
        L.oz2_context_workspace_bytes.restype = ctypes.c_size_t
        L.oz2_context_workspace_bytes.argtypes = [vp, i64, i64, i64, ci]
        L.oz2_context_dgemm.argtypes = [vp, ctypes.c_char, ctypes.c_char, i64, i64, i64, ctypes.c_double, vp, i64, vp, i64,
                                        ctypes.c_double, vp, i64, ci, vp]
        L.oz2_context_dsyrk.argtypes = [vp, ctypes.c_char, ctypes.c_char, i64, i64, ctypes.c_double, vp, i64, ctypes.c_double,
                                        vp, i64, ci, vp]
        L.oz2_context_dtrmm.argtypes = [vp] + [ctypes.c_char] * 4 + [i64, i64, ctypes.c_double, vp, i64, vp, i64, ci, vp]
        L.oz2_set_round_sync.argtypes = [ci]
        L.oz2_set_shift_mode.argtypes = [ci]
        L.oz2_set_product_format.argtypes = [ci]
        L.oz2_set_nonfinite_check.argtypes = [ci]
        L.oz2_set_bit_split.argtypes = [ci]
        L.oz2_set_stage_events.argtypes = [vp]
        L.oz2_calibrate_mfma.argtypes = [ci, ci, ci, vp, vp, vp]
        L.oz2_host_crt_element.argtypes = [ci, vp, vp]
        L.oz2_host_crt_element_digits.argtypes = [ci, vp, vp]
        L.oz2_host_residues.argtypes = [ci, ci, ctypes.c_double, ci, vp]
        L.oz2_status_string.restype = ctypes.c_char_p
        L.oz2_status_string.argtypes = [ci]
        _lib = L
    return _lib


def _check(rc, what):
    if rc != 0:
        raise Oz2Error("%s failed: status %d (%s)" % (what, rc, lib().oz2_status_string(rc).decode()))


def min_moduli():
    return lib().oz2_min_moduli()


def max_moduli():
    return lib().oz2_max_moduli()


def get_moduli(num_moduli, k=1):
    """(moduli list, kappa) for this moduli count and inner dimension."""
    mods = (ctypes.c_int * num_moduli)()
    kap = ctypes.c_int(0)
    _check(lib().oz2_get_moduli(num_moduli, mods, ctypes.byref(kap), k), "oz2_get_moduli")
    return list(mods), kap.value


def workspace_bytes(m, n, k, num_moduli, product_format=None):
    """Bytes that serve either product format (None), or exactly one of them."""
    if product_format is None:
        return int(lib().oz2_workspace_bytes(m, n, k, num_moduli))
    return int(lib().oz2_workspace_bytes_for(m, n, k, num_moduli, int(product_format)))


def workspace_bytes_strassen(m, n, k, num_moduli):
    """Bytes the Strassen form of the products needs."""
    return int(lib().oz2_workspace_bytes_strassen(m, n, k, num_moduli))


def workspace_bytes_preferred(m, n, k, num_moduli):
    """Bytes with which a general product takes the form the settings in force prefer."""
    return int(lib().oz2_workspace_bytes_preferred(m, n, k, num_moduli))


OZ2_GEMM_AUTO, OZ2_GEMM_CLASSICAL, OZ2_GEMM_STRASSEN = -1, 0, 1


def oz2_set_gemm_algorithm(algorithm):
    """-1 (default): Strassen form for large general products; 0: never; 1: whenever it applies."""
    _check(lib().oz2_set_gemm_algorithm(int(algorithm)), "oz2_set_gemm_algorithm")


def oz2_gemm_algorithm_for(m, n, k, num_moduli):
    """Form (0 classical, 1 Strassen) a general product of this shape takes under the settings and workspace in force."""
    rc = lib().oz2_gemm_algorithm_for(m, n, k, num_moduli)
    if rc < 0:
        raise Oz2Error("oz2_gemm_algorithm_for: invalid argument %d" % -rc)
    return rc


def oz2_init():
    _check(lib().oz2_init(), "oz2_init")


def moduli_for_bits(k, bits=53):
    """Smallest number of moduli whose bit budget reaches `bits` for inner dimension k (0: none does)."""
    rc = lib().oz2_moduli_for_bits(int(k), int(bits))
    if rc < 0:
        raise Oz2Error("oz2_moduli_for_bits: invalid argument %d" % -rc)
    return rc


def workspace_layout(m, n, k, num_moduli):
    """dict of byte offsets and padded dims (see include/oz2.h)."""
    offs = (ctypes.c_size_t * 10)()
    dims = (ctypes.c_int64 * 3)()
    _check(lib().oz2_workspace_layout(m, n, k, num_moduli, offs, dims), "oz2_workspace_layout")
    names = ["rowmax", "colmax", "sa", "sb", "a_planes", "b_planes", "c_planes", "rownorm", "colnorm", "flags"]
    out = {nm: int(o) for nm, o in zip(names, offs)}
    out.update(m_pad=int(dims[0]), n_pad=int(dims[1]), k_pad=int(dims[2]))
    return out


_registered_ptr = None   # what this module last registered with the library (None: nothing)


def set_workspace(dev_ptr, nbytes):
    global _registered_ptr
    _check(lib().oz2_set_workspace(dev_ptr, nbytes), "oz2_set_workspace")
    _registered_ptr = dev_ptr if dev_ptr else None


def oz2_set_round_sync(spins):
    """Bound (in polls) of a wait of the GEMM's per-die round synchronisation; 0 switches it off (default 4096)."""
    _check(lib().oz2_set_round_sync(int(spins)), "oz2_set_round_sync")


def oz2_set_kblock(kblock):
    _check(lib().oz2_set_kblock(kblock), "oz2_set_kblock")


def oz2_set_shift_mode(mode):
    """0: shifts from maxima (Section 3); 1: Cauchy-Schwarz bound; 2: INT8-product bound (both Section 4.1)."""
    _check(lib().oz2_set_shift_mode(int(mode)), "oz2_set_shift_mode")


OZ2_SHIFT_MAX, OZ2_SHIFT_CAUCHY_SCHWARZ, OZ2_SHIFT_INT8_PRODUCT = 0, 1, 2
OZ2_PRODUCT_INT32, OZ2_PRODUCT_RESIDUE_U8 = 0, 1


def oz2_set_product_format(fmt):
    """0: INT32 products in the C planes; 1 (default): UINT8 residues written by the GEMM epilogue."""
    _check(lib().oz2_set_product_format(int(fmt)), "oz2_set_product_format")


def oz2_set_bit_split(delta):
    """Bits of budget moved from op(A) to op(B) (0: the equal split)."""
    _check(lib().oz2_set_bit_split(int(delta)), "oz2_set_bit_split")


def oz2_set_nonfinite_check(on):
    """1 (default): infinities / NaNs in A or B are detected and C is formed by the FP64 fallback kernel."""
    _check(lib().oz2_set_nonfinite_check(int(on)), "oz2_set_nonfinite_check")


def oz2_set_stage_events(events):
    """events: four hipEvent_t handles (ints) or None."""
    if events is None:
        _check(lib().oz2_set_stage_events(None), "oz2_set_stage_events")
    else:
        arr = (ctypes.c_void_p * 4)(*events)
        _check(lib().oz2_set_stage_events(arr), "oz2_set_stage_events")


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return getattr(stream, "cuda_stream", stream)


def oz2_dgemm(m, n, k, A_ptr, lda, B_ptr, ldb, C_ptr, ldc, num_moduli, stream=None):
    _check(lib().oz2_dgemm(m, n, k, A_ptr, lda, B_ptr, ldb, C_ptr, ldc, num_moduli, _stream_ptr(stream)), "oz2_dgemm")


OZ2_STATIC_SCRATCH_BYTES = 64 << 20


def oz2_dgemm_static(m, n, k, A_ptr, lda, B_ptr, ldb, C_ptr, ldc, num_moduli, stream=None):
    """oz2_dgemm on the library's static workspace: allocates nothing, needs no registered workspace."""
    _check(lib().oz2_dgemm_static(m, n, k, A_ptr, lda, B_ptr, ldb, C_ptr, ldc, num_moduli, _stream_ptr(stream)),
           "oz2_dgemm_static")


def oz2_dgemm_ex(transa, transb, m, n, k, alpha, A_ptr, lda, B_ptr, ldb, beta, C_ptr, ldc, num_moduli, stream=None):
    _check(lib().oz2_dgemm_ex(transa.encode(), transb.encode(), m, n, k, float(alpha), A_ptr, lda, B_ptr, ldb,
                              float(beta), C_ptr, ldc, num_moduli, _stream_ptr(stream)), "oz2_dgemm_ex")


def oz2_dsyrk(uplo, trans, n, k, alpha, A_ptr, lda, beta, C_ptr, ldc, num_moduli, stream=None):
    _check(lib().oz2_dsyrk(uplo.encode(), trans.encode(), n, k, float(alpha), A_ptr, lda, float(beta), C_ptr, ldc,
                           num_moduli, _stream_ptr(stream)), "oz2_dsyrk")


def oz2_dtrmm(side, uplo, transa, diag, m, n, alpha, A_ptr, lda, B_ptr, ldb, num_moduli, stream=None):
    _check(lib().oz2_dtrmm(side.encode(), uplo.encode(), transa.encode(), diag.encode(), m, n, float(alpha), A_ptr, lda,
                           B_ptr, ldb, num_moduli, _stream_ptr(stream)), "oz2_dtrmm")


def oz2_stage1_convert(m, n, k, A_ptr, lda, B_ptr, ldb, num_moduli, stream=None):
    _check(lib().oz2_stage1_convert(m, n, k, A_ptr, lda, B_ptr, ldb, num_moduli, _stream_ptr(stream)),
           "oz2_stage1_convert")


def oz2_stage2_gemm(m, n, k, num_moduli, stream=None):
    _check(lib().oz2_stage2_gemm(m, n, k, num_moduli, _stream_ptr(stream)), "oz2_stage2_gemm")


def oz2_stage3_crt(m, n, k, C_ptr, ldc, num_moduli, stream=None):
    _check(lib().oz2_stage3_crt(m, n, k, C_ptr, ldc, num_moduli, _stream_ptr(stream)), "oz2_stage3_crt")


def oz2_calibrate_mfma(workgroups, iters, random_operands, sink_ptr, clocks_ptr, stream=None):
    _check(lib().oz2_calibrate_mfma(workgroups, iters, int(random_operands), sink_ptr, clocks_ptr,
                                    _stream_ptr(stream)), "oz2_calibrate_mfma")


def host_crt_element(num_moduli, cprod):
    arr = (ctypes.c_int32 * num_moduli)(*[int(c) for c in cprod])
    out = ctypes.c_double(0.0)
    _check(lib().oz2_host_crt_element(num_moduli, arr, ctypes.byref(out)), "oz2_host_crt_element")
    return out.value


def host_crt_element_digits(num_moduli, residues):
    arr = (ctypes.c_uint8 * num_moduli)(*[int(c) for c in residues])
    out = ctypes.c_double(0.0)
    _check(lib().oz2_host_crt_element_digits(num_moduli, arr, ctypes.byref(out)), "oz2_host_crt_element_digits")
    return out.value


def host_residues(num_moduli, kappa, a, shift):
    out = (ctypes.c_int8 * num_moduli)()
    _check(lib().oz2_host_residues(num_moduli, kappa, float(a), int(shift), out), "oz2_host_residues")
    return list(out)


OZ2_OPT_SHIFT_MODE, OZ2_OPT_PRODUCT_FORMAT, OZ2_OPT_GEMM_ALGORITHM, OZ2_OPT_KBLOCK, OZ2_OPT_BIT_SPLIT, OZ2_OPT_NONFINITE_CHECK = range(6)


class Context:
    """oz2_context: settings, workspace registration and lock of its own (see include/oz2.h).  The device buffer
    is torch's; the object keeps it alive as long as the context points at it."""

    def __init__(self):
        self.handle = ctypes.c_void_p()
        _check(lib().oz2_context_create(ctypes.byref(self.handle)), "oz2_context_create")
        self.buf = None

    def set(self, option, value):
        _check(lib().oz2_context_set(self.handle, int(option), int(value)), "oz2_context_set")

    def get(self, option):
        v = ctypes.c_int64(0)
        _check(lib().oz2_context_get(self.handle, int(option), ctypes.byref(v)), "oz2_context_get")
        return v.value

    def workspace_bytes(self, m, n, k, num_moduli):
        return int(lib().oz2_context_workspace_bytes(self.handle, m, n, k, num_moduli))

    def allocate_workspace(self, m, n, k, num_moduli, device="cuda:0"):
        import torch
        nbytes = self.workspace_bytes(m, n, k, num_moduli)
        if nbytes == 0:
            raise Oz2Error("invalid problem for a workspace")
        self.buf = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
        off = (-self.buf.data_ptr()) % 256
        _check(lib().oz2_context_set_workspace(self.handle, self.buf.data_ptr() + off, nbytes), "oz2_context_set_workspace")
        return nbytes

    def dgemm(self, transa, transb, m, n, k, alpha, A_ptr, lda, B_ptr, ldb, beta, C_ptr, ldc, num_moduli, stream=None):
        _check(lib().oz2_context_dgemm(self.handle, transa.encode(), transb.encode(), m, n, k, float(alpha), A_ptr, lda,
                                       B_ptr, ldb, float(beta), C_ptr, ldc, num_moduli, _stream_ptr(stream)),
               "oz2_context_dgemm")

    def dsyrk(self, uplo, trans, n, k, alpha, A_ptr, lda, beta, C_ptr, ldc, num_moduli, stream=None):
        _check(lib().oz2_context_dsyrk(self.handle, uplo.encode(), trans.encode(), n, k, float(alpha), A_ptr, lda,
                                       float(beta), C_ptr, ldc, num_moduli, _stream_ptr(stream)), "oz2_context_dsyrk")

    def dtrmm(self, side, uplo, transa, diag, m, n, alpha, A_ptr, lda, B_ptr, ldb, num_moduli, stream=None):
        _check(lib().oz2_context_dtrmm(self.handle, side.encode(), uplo.encode(), transa.encode(), diag.encode(), m, n,
                                       float(alpha), A_ptr, lda, B_ptr, ldb, num_moduli, _stream_ptr(stream)),
               "oz2_context_dtrmm")

    def close(self):
        if self.handle:
            lib().oz2_context_destroy(self.handle)
            self.handle = ctypes.c_void_p()
        self.buf = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Workspace:
    """A torch-owned device buffer registered with the library (device memory only; no arithmetic)."""

    def __init__(self, m, n, k, num_moduli, device="cuda:0", product_format=None):
        import torch
        self.nbytes = workspace_bytes(m, n, k, num_moduli, product_format)
        if self.nbytes == 0:
            raise Oz2Error("invalid problem for a workspace")
        # enough for the form of the products that the settings in force prefer
        self.nbytes = max(self.nbytes, workspace_bytes_preferred(m, n, k, num_moduli))
        self.buf = torch.empty(self.nbytes + 256, dtype=torch.uint8, device=device)
        base = self.buf.data_ptr()
        self.offset = (-base) % 256
        self.ptr = base + self.offset
        set_workspace(self.ptr, self.nbytes)

    def close(self):
        """Unregister the buffer if the library still points at it.  The library keeps a bare pointer: once this
        object is gone the memory returns to the allocator, and a later call must find no workspace (status
        OZ2_ERR_WORKSPACE) instead of writing into memory that belongs to another tensor."""
        if getattr(self, "ptr", None) is not None and _registered_ptr == self.ptr and _lib is not None:
            set_workspace(None, 0)
        self.ptr = None

    def __del__(self):
        try:
            self.close()
        except Exception:   # interpreter shutdown: nothing left to protect
            pass

    def view(self, off, count, dtype):
        """1-D torch view of `count` elements of `dtype` starting `off` bytes into the workspace."""
        import torch
        esz = torch.empty((), dtype=dtype).element_size()
        return self.buf[self.offset + off: self.offset + off + count * esz].view(dtype)


def dgemm(A, B, num_moduli, C=None, workspace=None):
    """C = A @ B for column-major float64 torch tensors on the GPU (A: m x k, B: k x n given as the
    transposes of contiguous tensors, i.e. A.t().is_contiguous()).  Thin convenience wrapper."""
    import torch
    m, k = A.shape
    k2, n = B.shape
    assert k == k2 and A.dtype == torch.float64 and B.dtype == torch.float64
    assert A.t().is_contiguous() and B.t().is_contiguous(), "pass column-major matrices"
    if C is None:
        C = torch.empty((n, m), dtype=torch.float64, device=A.device).t()
    if workspace is None:
        workspace = Workspace(m, n, k, num_moduli, device=A.device)
    oz2_dgemm(m, n, k, A.data_ptr(), max(1, m), B.data_ptr(), max(1, k), C.data_ptr(), max(1, m), num_moduli)
    return C
