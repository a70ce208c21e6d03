"""ctypes binding for libabed.so: argument marshalling only.  Every function has
the name and meaning of the C entry point it calls (include/abed.h); tensors
are torch tensors on the GPU, used for their device pointers only."""
import ctypes
import enum
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class AbedError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("libabed: %s (status %d)" % (text, status))
        self.status = status


class Variant(enum.IntEnum):
    NONE = 0
    UNFUSED = 1
    FUSED_WRITE = 2
    FUSED_PARTIAL_REDUCTION = 3
    FUSED_OCG = 4
    FUSED_IOCG = 5
    DUPLICATE = 6


# OR one of these into a checked variant to run one scheme alone (include/abed.h)
ONLY_FC = 0x100
ONLY_IC = 0x200
L1_THRESHOLD = 0x1000   # fp16: threshold relative to the sum of magnitudes of the reduced elements
PACKED_FC = 0x400   # checksum filters in the free rows of the last block of 16 filters (wchk must follow w)
LOCAL = 0x800       # checksums local to a workgroup: FC per filter tile, IC per batch tile, formed inside the kernel


class ConvDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "H", "W", "C", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w")]


class _Epilogue(ctypes.Structure):
    _fields_ = [("scale", ctypes.c_void_p), ("bias", ctypes.c_void_p), ("relu", ctypes.c_int32)]


class _Inject(ctypes.Structure):
    _fields_ = [("site", ctypes.c_int32), ("index", ctypes.c_int64), ("bit", ctypes.c_int32)]


class Layout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("tile_pixels", "tile_batch", "tile_n", "grid_m", "grid_b", "grid_n", "d_f", "d_i")] + \
               [(n, ctypes.c_int64) for n in
                ("n_flag_words", "workspace_bytes", "wchk_bytes", "xchk_bytes", "xchk_next_bytes")] + \
               [("tile_box", ctypes.c_int32), ("local_checksums", ctypes.c_int32), ("local_preferred", ctypes.c_int32),
                ("reserved_", ctypes.c_int32)]


class FicLayout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in ("workspace_bytes", "wsum_bytes", "xrows_bytes")] + [("xrows_parts", ctypes.c_int32), ("xsum_bytes", ctypes.c_int64), ("xsum_next_bytes", ctypes.c_int64)]


class FicInloopLayout(ctypes.Structure):
    _fields_ = [("workspace_bytes", ctypes.c_int64), ("wdig_bytes", ctypes.c_int64)]


FIC_INLOOP = 0x1000   # abed_fic_verify's variant value for layers run by abed_fic_inloop_conv_int8


class Ic2Layout(ctypes.Structure):
    _fields_ = [("workspace_bytes", ctypes.c_int64), ("xrows_bytes", ctypes.c_int64), ("xrows_parts", ctypes.c_int32), ("n_values", ctypes.c_int32)]


EXPORTS = ["abed_fic_inloop_get_layout", "abed_fic_inloop_filter_prepare_int8", "abed_fic_inloop_conv_int8", "abed_fic_verify", "abed_ic2_get_layout", "abed_ic2_conv_int8", "abed_fic_get_layout", "abed_fic_filter_prepare_int8", "abed_fic_input_checksum_int8", "abed_fic_conv_int8",
           "abed_get_layout", "abed_filter_prepare_int8", "abed_filter_prepare_local_int8", "abed_filter_prepare_fp16",
           "abed_input_checksum_int8", "abed_input_checksum_fp16", "abed_workspace_init",
           "abed_conv_int8", "abed_conv_int8_static", "abed_conv_fp16", "abed_status_string", "abed_last_hip_error", "abed_probe", "abed_pad_channels", "abed_abft_gemm_get_layout", "abed_abft_gemm_int8"]


def lib_path():
    return os.path.join(_HERE, "libabed.so")


def lib():
    """Open libabed.so (built by `python -m paper_2006_04984_amd.build`); fails loudly if absent."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise FileNotFoundError("%s not built: run python -m paper_2006_04984_amd.build" % path)
        # torch first: it brings its own copy of the HIP runtime, and the library must resolve its HIP symbols
        # to that copy.  Loaded the other way round the process holds two runtimes, and the second one to
        # initialise finds no device.
        import torch  # noqa: F401
        L = ctypes.CDLL(path)
        for name in EXPORTS:
            getattr(L, name)
        L.abed_status_string.restype = ctypes.c_char_p
        L.abed_status_string.argtypes = [ctypes.c_int]
        L.abed_last_hip_error.restype = ctypes.c_char_p
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        L.abed_get_layout.argtypes = [ctypes.POINTER(ConvDesc), i32, i32, ctypes.POINTER(Layout)]
        L.abed_filter_prepare_int8.argtypes = [ctypes.POINTER(ConvDesc), vp, vp, vp]
        L.abed_input_checksum_int8.argtypes = [ctypes.POINTER(ConvDesc), vp, vp, vp]
        L.abed_filter_prepare_local_int8.argtypes = [ctypes.POINTER(ConvDesc), i32, vp, vp, vp]
        L.abed_workspace_init.argtypes = [vp, ctypes.c_size_t, vp]
        L.abed_conv_int8.argtypes = [ctypes.POINTER(ConvDesc), vp, vp, vp, vp, i32, vp, ctypes.POINTER(_Epilogue), i32,
                                     vp, vp, vp, ctypes.c_size_t, ctypes.POINTER(_Inject), vp, vp]
        L.abed_conv_int8_static.argtypes = [ctypes.POINTER(ConvDesc), vp, vp, vp, vp, i32, vp, ctypes.POINTER(_Epilogue), i32,
                                            vp, vp, ctypes.POINTER(_Inject), vp, vp]
        L.abed_probe.argtypes = [i32, vp, vp, ctypes.c_size_t, i32, vp]
        f32 = ctypes.c_float
        L.abed_filter_prepare_fp16.argtypes = [ctypes.POINTER(ConvDesc), vp, vp, vp]
        L.abed_input_checksum_fp16.argtypes = [ctypes.POINTER(ConvDesc), vp, vp, vp]
        L.abed_conv_fp16.argtypes = [ctypes.POINTER(ConvDesc), vp, vp, vp, vp, i32, vp, i32, i32, f32, f32,
                                     vp, vp, ctypes.c_size_t, ctypes.POINTER(_Inject), vp, vp]
        L.abed_fic_get_layout.argtypes = [ctypes.POINTER(ConvDesc), i32, ctypes.POINTER(FicLayout)]
        L.abed_fic_filter_prepare_int8.argtypes = [ctypes.POINTER(ConvDesc), vp, vp, vp]
        L.abed_fic_input_checksum_int8.argtypes = [ctypes.POINTER(ConvDesc), i32, vp, vp, vp]
        L.abed_fic_conv_int8.argtypes = [ctypes.POINTER(ConvDesc), vp, vp, vp, vp, i32, vp, ctypes.POINTER(_Epilogue), i32,
                                         vp, vp, vp, vp, vp, ctypes.c_size_t, ctypes.POINTER(_Inject), vp]
        L.abed_fic_inloop_get_layout.argtypes = [ctypes.POINTER(ConvDesc), ctypes.POINTER(FicInloopLayout)]
        L.abed_fic_inloop_filter_prepare_int8.argtypes = [ctypes.POINTER(ConvDesc), vp, vp, vp]
        L.abed_fic_inloop_conv_int8.argtypes = [ctypes.POINTER(ConvDesc), vp, vp, vp, vp, ctypes.POINTER(_Epilogue), vp, vp,
                                                vp, ctypes.c_size_t, ctypes.POINTER(_Inject), vp]
        L.abed_fic_verify.argtypes = [i32, ctypes.POINTER(ConvDesc), ctypes.POINTER(i32), ctypes.POINTER(vp), vp, vp, vp]
        L.abed_ic2_get_layout.argtypes = [ctypes.POINTER(ConvDesc), i32, ctypes.POINTER(Ic2Layout)]
        L.abed_ic2_conv_int8.argtypes = [ctypes.POINTER(ConvDesc), vp, vp, vp, i32, vp, ctypes.POINTER(_Epilogue), i32,
                                         vp, vp, vp, ctypes.c_size_t, ctypes.POINTER(_Inject), vp]
        _LIB = L
    return _LIB


def _check(status):
    if status != 0:
        L = lib()
        text = L.abed_status_string(status).decode()
        if status == 4:
            text += ": " + L.abed_last_hip_error().decode()
        raise AbedError(status, text)


def _p(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    return ctypes.c_void_p(stream if isinstance(stream, int) else stream.cuda_stream)


def desc_from_shape(s):
    return ConvDesc(s.N, s.H, s.W, s.C, s.K, s.R, s.S, s.stride_h, s.stride_w, s.pad_h, s.pad_w)


def get_layout(desc, dtype=0, variant=Variant.FUSED_OCG):
    out = Layout()
    _check(lib().abed_get_layout(ctypes.byref(desc), int(dtype), int(variant), ctypes.byref(out)))
    return out


def filter_prepare_int8(desc, w, wchk, stream=None):
    _check(lib().abed_filter_prepare_int8(ctypes.byref(desc), _p(w), _p(wchk), _stream(stream)))


def filter_prepare_local_int8(desc, variant, w, wchk, stream=None):
    _check(lib().abed_filter_prepare_local_int8(ctypes.byref(desc), int(variant), _p(w), _p(wchk), _stream(stream)))


def input_checksum_int8(desc, x, xchk, stream=None):
    _check(lib().abed_input_checksum_int8(ctypes.byref(desc), _p(x), _p(xchk), _stream(stream)))


def workspace_init(workspace, stream=None):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().abed_workspace_init(_p(workspace), nbytes, _stream(stream)))


class AbftLayout(ctypes.Structure):
    _fields_ = [("d_a", ctypes.c_int32), ("d_b", ctypes.c_int32), ("ld_c", ctypes.c_int32), ("reserved_", ctypes.c_int32),
                ("rows_padded", ctypes.c_int64), ("workspace_bytes", ctypes.c_uint64), ("c_offset", ctypes.c_uint64)]


ABFT_TASKS = {"copy_in": 1, "checksums": 2, "gemm": 4, "verify": 8, "copy_out": 16}


def abft_gemm_get_layout(M, Ng, Kg):
    out = AbftLayout()
    _check(lib().abed_abft_gemm_get_layout(ctypes.c_int64(M), int(Ng), int(Kg), ctypes.byref(out)))
    return out


def abft_gemm_int8(M, Ng, Kg, A, B, C, flags, workspace, tasks=0, inject=None, stream=None):
    """abed_abft_gemm_int8: the traditional ABFT-GEMM baseline.  inject = (2, index in the larger output, bit) or None."""
    inj = None
    if inject is not None:
        inj = ctypes.byref(_Inject(int(inject[0]), int(inject[1]), int(inject[2])))
    _check(lib().abed_abft_gemm_int8(ctypes.c_int64(M), int(Ng), int(Kg), _p(A), _p(B), _p(C), _p(flags), _p(workspace),
                                     ctypes.c_size_t(workspace.numel() * workspace.element_size()), int(tasks), inj, _stream(stream)))


def pad_channels(src, dst, c, c_pad, stream=None):
    """abed_pad_channels: dst[..., :c] = src, dst[..., c:] = 0 for tensors whose last axis is the channels."""
    rows = src.numel() // c
    _check(lib().abed_pad_channels(_p(src), _p(dst), ctypes.c_int64(rows), int(c), int(c_pad), int(src.element_size()),
                                   _stream(stream)))


def conv_int8(desc, x, w, wchk, xchk, compute_xchk, y, variant, flags=None, epilogue=None, xchk_next=None,
              workspace=None, inject=None, y2=None, stream=None):
    """abed_conv_int8.  epilogue = (scale, bias, relu) tensors/bool or None;
    inject = (site, index, bit) or None."""
    epi = None
    if epilogue is not None:
        epi = ctypes.byref(_Epilogue(epilogue[0].data_ptr(), epilogue[1].data_ptr(), int(bool(epilogue[2]))))
    inj = None
    if inject is not None:
        inj = ctypes.byref(_Inject(int(inject[0]), int(inject[1]), int(inject[2])))
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().abed_conv_int8(ctypes.byref(desc), _p(x), _p(w), _p(wchk), _p(xchk), int(bool(compute_xchk)),
                                _p(y), epi, int(variant), _p(flags), _p(xchk_next), _p(workspace), nbytes,
                                inj, _p(y2), _stream(stream)))


def conv_int8_static(desc, x, w, wchk, xchk, compute_xchk, y, variant, flags=None, epilogue=None, xchk_next=None,
                     inject=None, y2=None, stream=None):
    """abed_conv_int8_static: abed_conv_int8 on the library's own per-GPU scratch array (no workspace)."""
    epi = None
    if epilogue is not None:
        epi = ctypes.byref(_Epilogue(epilogue[0].data_ptr(), epilogue[1].data_ptr(), int(bool(epilogue[2]))))
    inj = None
    if inject is not None:
        inj = ctypes.byref(_Inject(int(inject[0]), int(inject[1]), int(inject[2])))
    _check(lib().abed_conv_int8_static(ctypes.byref(desc), _p(x), _p(w), _p(wchk), _p(xchk), int(bool(compute_xchk)),
                                       _p(y), epi, int(variant), _p(flags), _p(xchk_next), inj, _p(y2), _stream(stream)))


def probe(kind, a, b=None, iters=1, stream=None):
    """abed_probe: machine ceilings for roofline reports (0: int8 matrix instruction loop, 1: fill a, 2: copy a -> b)."""
    _check(lib().abed_probe(int(kind), _p(a), _p(b), a.numel() * a.element_size(), int(iters), _stream(stream)))


def filter_prepare_fp16(desc, w, wchk, stream=None):
    _check(lib().abed_filter_prepare_fp16(ctypes.byref(desc), _p(w), _p(wchk), _stream(stream)))


def input_checksum_fp16(desc, x, xchk, stream=None):
    _check(lib().abed_input_checksum_fp16(ctypes.byref(desc), _p(x), _p(xchk), _stream(stream)))


def conv_fp16(desc, x, w, wchk, xchk, compute_xchk, y, variant, rtol=1e-3, atol=0.0, flags=None, out_fp32=False,
              workspace=None, inject=None, y2=None, stream=None):
    """abed_conv_fp16.  inject = (site, index, bit) or None."""
    inj = None
    if inject is not None:
        inj = ctypes.byref(_Inject(int(inject[0]), int(inject[1]), int(inject[2])))
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().abed_conv_fp16(ctypes.byref(desc), _p(x), _p(w), _p(wchk), _p(xchk), int(bool(compute_xchk)),
                                _p(y), int(bool(out_fp32)), int(variant), float(rtol), float(atol), _p(flags),
                                _p(workspace), nbytes, inj, _p(y2), _stream(stream)))


def fic_get_layout(desc, variant):
    out = FicLayout()
    _check(lib().abed_fic_get_layout(ctypes.byref(desc), int(variant), ctypes.byref(out)))
    return out


def fic_filter_prepare_int8(desc, w, wsum, stream=None):
    _check(lib().abed_fic_filter_prepare_int8(ctypes.byref(desc), _p(w), _p(wsum), _stream(stream)))


def fic_input_checksum_int8(desc, variant, x, xrows, stream=None):
    _check(lib().abed_fic_input_checksum_int8(ctypes.byref(desc), int(variant), _p(x), _p(xrows), _stream(stream)))


def fic_conv_int8(desc, x, w, wsum, xrows, compute_xrows, y, variant, result, flag, epilogue=None,
                  workspace=None, inject=None, stream=None, xsum_in=None, xsum_next=None):
    """abed_fic_conv_int8.  result: int64[2] tensor, flag: int32[1] tensor (device)."""
    epi = None
    if epilogue is not None:
        epi = ctypes.byref(_Epilogue(epilogue[0].data_ptr(), epilogue[1].data_ptr(), int(bool(epilogue[2]))))
    inj = None
    if inject is not None:
        inj = ctypes.byref(_Inject(int(inject[0]), int(inject[1]), int(inject[2])))
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().abed_fic_conv_int8(ctypes.byref(desc), _p(x), _p(w), _p(wsum), _p(xrows), int(bool(compute_xrows)),
                                    _p(y), epi, int(variant), _p(result), _p(flag), _p(xsum_in), _p(xsum_next),
                                    _p(workspace), nbytes, inj, _stream(stream)))


def fic_inloop_get_layout(desc):
    out = FicInloopLayout()
    _check(lib().abed_fic_inloop_get_layout(ctypes.byref(desc), ctypes.byref(out)))
    return out


def fic_inloop_filter_prepare_int8(desc, w, wdig, stream=None):
    _check(lib().abed_fic_inloop_filter_prepare_int8(ctypes.byref(desc), _p(w), _p(wdig), _stream(stream)))


def fic_inloop_conv_int8(desc, x, w, wdig, y, result, flag, epilogue=None, workspace=None, inject=None, stream=None):
    """abed_fic_inloop_conv_int8.  result: int64[2] tensor, flag: int32[1] tensor (device), or both None."""
    epi = None
    if epilogue is not None:
        epi = ctypes.byref(_Epilogue(epilogue[0].data_ptr(), epilogue[1].data_ptr(), int(bool(epilogue[2]))))
    inj = None
    if inject is not None:
        inj = ctypes.byref(_Inject(int(inject[0]), int(inject[1]), int(inject[2])))
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().abed_fic_inloop_conv_int8(ctypes.byref(desc), _p(x), _p(w), _p(wdig), _p(y), epi, _p(result), _p(flag),
                                           _p(workspace), nbytes, inj, _stream(stream)))


def ic2_get_layout(desc, variant):
    out = Ic2Layout()
    _check(lib().abed_ic2_get_layout(ctypes.byref(desc), int(variant), ctypes.byref(out)))
    return out


def ic2_conv_int8(desc, x, w, xrows, compute_xrows, y, variant, result, flags, epilogue=None,
                  workspace=None, inject=None, stream=None):
    """abed_ic2_conv_int8.  epilogue = (scale, bias, relu) or None; inject = (site, index, bit) or None."""
    epi = None
    if epilogue is not None:
        epi = ctypes.byref(_Epilogue(epilogue[0].data_ptr(), epilogue[1].data_ptr(), int(bool(epilogue[2]))))
    inj = None
    if inject is not None:
        inj = ctypes.byref(_Inject(int(inject[0]), int(inject[1]), int(inject[2])))
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().abed_ic2_conv_int8(ctypes.byref(desc), _p(x), _p(w), _p(xrows), int(bool(compute_xrows)),
                                    _p(y), epi, int(variant), _p(result), _p(flags), _p(workspace), nbytes,
                                    inj, _stream(stream)))


def fic_verify(descs, variants, workspaces, results, flags, stream=None):
    """abed_fic_verify: the deferred comparisons of several layers run with result = flag = None."""
    n = len(descs)
    d = (ConvDesc * n)(*descs)
    v = (ctypes.c_int32 * n)(*[int(x) for x in variants])
    w = (ctypes.c_void_p * n)(*[t.data_ptr() for t in workspaces])
    _check(lib().abed_fic_verify(n, d, v, w, _p(results), _p(flags), _stream(stream)))
