"""ctypes binding of include/pe.h.  Argument marshalling only."""
import ctypes as C
import os

PE_F32, PE_BF16 = 0, 1
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpe_mi355x.so")


class PEError(RuntimeError):
    pass


class PEDims(C.Structure):
    _fields_ = [("s", C.c_int), ("r", C.c_int), ("c_m", C.c_int), ("c_z", C.c_int),
                ("h_msa", C.c_int), ("d_msa", C.c_int), ("h_pair", C.c_int), ("d_pair", C.c_int),
                ("c_tri", C.c_int), ("c_opm", C.c_int), ("n_trans", C.c_int), ("col_global", C.c_int),
                ("dtype", C.c_int), ("ln_eps", C.c_float), ("opm_eps", C.c_float), ("variant", C.c_int)]

    @classmethod
    def from_dict(cls, d):
        return cls(**{k: d.get(k, 0) if k == "variant" else d[k] for k, _ in cls._fields_})


class _ParamEntry(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("offset", C.c_longlong), ("ndim", C.c_int),
                ("shape", C.c_int * 2), ("fan_in", C.c_int), ("kind", C.c_int)]


class _CtxEntry(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("offset_bytes", C.c_longlong), ("count", C.c_longlong),
                ("dtype", C.c_int)]


class _TimingEntry(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("kernel", C.c_char * 64), ("launches", C.c_int), ("total_ms", C.c_double),
                ("flops", C.c_double), ("bytes", C.c_double)]


_lib = None
_KINDS = {0: "weight", 1: "ln_gamma", 2: "ln_beta", 3: "bias"}


def lib():
    """Load the HIP library; fails loudly when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise PEError("HIP library %s is missing: run paper_2211_00235_amd.build.build() "
                      "(there is no CPU fallback)" % _LIB_PATH)
    L = C.CDLL(_LIB_PATH)
    vp, dp, fp = C.c_void_p, C.POINTER(PEDims), C.c_void_p
    L.pe_create.argtypes = [C.POINTER(vp)]
    L.pe_destroy.argtypes = [vp]
    L.pe_set_option.argtypes = [vp, C.c_int, C.c_int]
    L.pe_check_dims.argtypes = [dp]
    L.pe_dims_error.argtypes = [dp]
    L.pe_dims_error.restype = C.c_char_p
    L.pe_param_count.argtypes = [dp]
    L.pe_param_count.restype = C.c_longlong
    L.pe_param_table.argtypes = [dp, C.POINTER(_ParamEntry), C.c_int]
    L.pe_ctx_table.argtypes = [dp, C.POINTER(_CtxEntry), C.c_int]
    L.pe_ctx_bytes.argtypes = [dp]
    L.pe_ctx_bytes.restype = C.c_size_t
    L.pe_workspace_bytes.argtypes = [dp, C.c_int]
    L.pe_workspace_bytes.restype = C.c_size_t
    L.pe_stack_workspace_bytes.argtypes = [C.c_int, dp, C.c_int, dp]
    L.pe_stack_workspace_bytes.restype = C.c_size_t
    L.pe_stack_workspace_bytes_keep.argtypes = [C.c_int, dp, C.c_int, dp]
    L.pe_stack_workspace_bytes_keep.restype = C.c_size_t
    L.pe_block_fwd.argtypes = [vp, dp, vp, vp, fp, fp, fp, vp, vp, vp, vp, C.c_size_t, vp, vp]
    L.pe_static_scratch_bytes.argtypes = []
    L.pe_static_scratch_bytes.restype = C.c_size_t
    L.pe_block_fwd_static.argtypes = [vp, dp, vp, vp, fp, fp, fp, vp, vp, vp, vp]
    L.pe_block_bwd.argtypes = [vp, dp, vp, vp, fp, fp, fp, vp, vp, vp, vp, fp, vp, vp, C.c_size_t, vp, vp]
    L.pe_stack_fwd_bwd.argtypes = [vp, C.c_int, dp, C.c_int, dp, vp, vp, vp, fp, fp, fp, fp, vp, vp,
                                   vp, vp, vp, vp, vp, fp, vp, C.c_size_t, vp, vp]
    L.pe_timing_collect.argtypes = [vp, C.POINTER(_TimingEntry), C.c_int]
    L.pe_strerror.argtypes = [C.c_int]
    L.pe_strerror.restype = C.c_char_p
    L.pe_last_error.argtypes = [vp]
    L.pe_last_error.restype = C.c_char_p
    _lib = L
    return L


def strerror(code):
    return lib().pe_strerror(code).decode()


def _dims(d):
    return d if isinstance(d, PEDims) else PEDims.from_dict(d)


def check_dims(d):
    return lib().pe_check_dims(C.byref(_dims(d)))


def dims_error(d):
    """Text of the requirement that check_dims found violated ('' if the dims are supported)."""
    return lib().pe_dims_error(C.byref(_dims(d))).decode()


def param_count(d):
    return int(lib().pe_param_count(C.byref(_dims(d))))


def param_table(d):
    dd = _dims(d)
    n = lib().pe_param_table(C.byref(dd), None, 0)
    if n < 0:
        raise PEError(strerror(n))
    arr = (_ParamEntry * n)()
    lib().pe_param_table(C.byref(dd), arr, n)
    return [dict(name=e.name.decode(), offset=int(e.offset),
                 shape=tuple(e.shape[:e.ndim]), fan_in=int(e.fan_in), kind=_KINDS[e.kind]) for e in arr]


def ctx_table(d):
    dd = _dims(d)
    n = lib().pe_ctx_table(C.byref(dd), None, 0)
    if n < 0:
        raise PEError(strerror(n))
    arr = (_CtxEntry * n)()
    lib().pe_ctx_table(C.byref(dd), arr, n)
    return [dict(name=e.name.decode(), offset_bytes=int(e.offset_bytes), count=int(e.count), dtype=int(e.dtype))
            for e in arr]


def ctx_bytes(d):
    return int(lib().pe_ctx_bytes(C.byref(_dims(d))))


def workspace_bytes(d, with_ctx):
    return int(lib().pe_workspace_bytes(C.byref(_dims(d)), int(with_ctx)))


def stack_workspace_bytes(n_extra, extra, n_main, main, keep=False):
    e = C.byref(_dims(extra)) if extra is not None else None
    m = C.byref(_dims(main)) if main is not None else None
    f = lib().pe_stack_workspace_bytes_keep if keep else lib().pe_stack_workspace_bytes
    return int(f(n_extra, e, n_main, m))


class Handle:
    def __init__(self):
        self._h = C.c_void_p()
        rc = lib().pe_create(C.byref(self._h))
        if rc:
            raise PEError("pe_create: " + strerror(rc))

    def set_option(self, opt, value):
        rc = lib().pe_set_option(self._h, opt, value)
        if rc:
            raise PEError(strerror(rc))

    def timing_collect(self):
        """Per-label kernel timings since the last call (PE_OPT_KERNEL_TIMING = 3 must be on)."""
        n = lib().pe_timing_collect(self._h, None, 0)
        if n < 0:
            raise PEError(strerror(n))
        arr = (_TimingEntry * max(n, 1))()
        n = lib().pe_timing_collect(self._h, arr, n)
        if n < 0:
            raise PEError(strerror(n))
        return [dict(name=e.name.decode(), kernel=e.kernel.decode(), launches=int(e.launches), total_ms=float(e.total_ms),
                     flops=float(e.flops), bytes=float(e.bytes)) for e in arr[:n]]

    def last_error(self):
        return lib().pe_last_error(self._h).decode()

    def close(self):
        if self._h:
            lib().pe_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _p(t):
    """Device pointer of a torch tensor (or None / int passthrough)."""
    if t is None:
        return None
    if isinstance(t, int):
        return C.c_void_p(t)
    return C.c_void_p(t.data_ptr())


def _s(stream):
    if stream is None:
        return None
    return C.c_void_p(getattr(stream, "cuda_stream", stream))


def _raise(h, rc, what, dims=None):
    if rc:
        why = dims_error(dims) if (rc == -2 and dims is not None) else h.last_error()
        raise PEError("%s: %s %s" % (what, strerror(rc), why))


def block_fwd(h, dims, msa_in, pair_in, msa_mask, pair_mask, params, msa_out, pair_out, ctx, workspace,
              stream_msa=None, stream_pair=None):
    rc = lib().pe_block_fwd(h._h, C.byref(_dims(dims)), _p(msa_in), _p(pair_in), _p(msa_mask), _p(pair_mask),
                            _p(params), _p(msa_out), _p(pair_out), _p(ctx), _p(workspace),
                            workspace.numel() * workspace.element_size(), _s(stream_msa), _s(stream_pair))
    _raise(h, rc, "pe_block_fwd", dims)


def static_scratch_bytes():
    return int(lib().pe_static_scratch_bytes())


def block_fwd_static(h, dims, msa_in, pair_in, msa_mask, pair_mask, params, msa_out, pair_out,
                     stream_msa=None, stream_pair=None):
    rc = lib().pe_block_fwd_static(h._h, C.byref(_dims(dims)), _p(msa_in), _p(pair_in), _p(msa_mask), _p(pair_mask),
                                   _p(params), _p(msa_out), _p(pair_out), _s(stream_msa), _s(stream_pair))
    _raise(h, rc, "pe_block_fwd_static", dims)


def block_bwd(h, dims, msa_in, pair_in, msa_mask, pair_mask, params, d_msa_out, d_pair_out, d_msa_in, d_pair_in,
              d_params, ctx, workspace, stream_msa=None, stream_pair=None):
    rc = lib().pe_block_bwd(h._h, C.byref(_dims(dims)), _p(msa_in), _p(pair_in), _p(msa_mask), _p(pair_mask),
                            _p(params), _p(d_msa_out), _p(d_pair_out), _p(d_msa_in), _p(d_pair_in), _p(d_params),
                            _p(ctx), _p(workspace), workspace.numel() * workspace.element_size(),
                            _s(stream_msa), _s(stream_pair))
    _raise(h, rc, "pe_block_bwd", dims)


def stack_fwd_bwd(h, n_extra, extra, n_main, main, extra_msa_in, msa_in, pair_in, extra_mask, msa_mask, pair_mask,
                  params, d_msa_out, d_pair_out, msa_out, pair_out, d_extra_msa_in, d_msa_in, d_pair_in, d_params,
                  workspace, stream_msa=None, stream_pair=None):
    e = C.byref(_dims(extra)) if extra is not None else None
    m = C.byref(_dims(main)) if main is not None else None
    rc = lib().pe_stack_fwd_bwd(h._h, n_extra, e, n_main, m, _p(extra_msa_in), _p(msa_in), _p(pair_in),
                                _p(extra_mask), _p(msa_mask), _p(pair_mask), _p(params), _p(d_msa_out),
                                _p(d_pair_out), _p(msa_out), _p(pair_out), _p(d_extra_msa_in), _p(d_msa_in),
                                _p(d_pair_in), _p(d_params), _p(workspace),
                                workspace.numel() * workspace.element_size(), _s(stream_msa), _s(stream_pair))
    _raise(h, rc, "pe_stack_fwd_bwd")
