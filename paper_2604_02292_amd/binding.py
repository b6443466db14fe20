"""Thin ctypes binding over libhccs.so.  Argument marshalling only: every step
of the method runs in the HIP kernels behind the C ABI (include/hccs.h).

PyTorch is used for device memory and streams.  There is no CPU fallback: if
the shared library is missing or a call fails, an exception is raised.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhccs.so")

BAND_U8, BAND_STRICT = 0, 1
RECIP_EXACT, RECIP_CLB = 0, 1

EXPORTS = ["hccs_validate_params", "hccs_calibrated_softmax_i8", "hccs_calibrated_softmax_i8_ex", "hccs_attention_i8", "hccs_attention_i8_ex",
           "hccs_calibrate_workspace_bytes", "hccs_calibrate_grid", "hccs_calibrate_grid_static",
           "hccs_exp_softmax_i8_f32", "hccs_reciprocal_u8", "hccs_normalise_table_u8", "hccs_largest_probability_u8",
           "hccs_copy_bytes", "hccs_status_string"]


class HccsError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"hccs status {status}: {message}")
        self.status = status


class HeadParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("S", ctypes.c_int32), ("Dmax", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


class Requant(ctypes.Structure):
    _fields_ = [("mult", ctypes.c_int32), ("shift", ctypes.c_int32)]


_lib = None


def lib():
    """Opens the library on first use; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise HccsError(-8, f"{LIB_PATH} not found: build it with `python -m paper_2604_02292_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        i32, i64, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
        L.hccs_validate_params.argtypes = [ctypes.POINTER(HeadParams), i32, i32, i32, ctypes.POINTER(i32)]
        L.hccs_calibrated_softmax_i8.argtypes = [vp, vp, i32, i32, i32, i32, ctypes.POINTER(HeadParams), i32, i32, vp]
        L.hccs_calibrated_softmax_i8_ex.argtypes = [vp, vp, i32, i32, i32, i32, ctypes.POINTER(HeadParams), i32, i32,
                                                    i32, vp]
        L.hccs_attention_i8.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, ctypes.POINTER(HeadParams),
                                        ctypes.POINTER(Requant), i32, i32, vp]
        L.hccs_attention_i8_ex.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, ctypes.POINTER(HeadParams),
                                           ctypes.POINTER(Requant), i32, i32, vp]
        L.hccs_calibrate_workspace_bytes.argtypes = [i32, i32, i32, i32]
        L.hccs_calibrate_workspace_bytes.restype = i64
        L.hccs_calibrate_grid.argtypes = [vp, i32, i32, i32, i32, ctypes.POINTER(ctypes.c_double), vp, i32, vp, vp, vp,
                                          i64, vp]
        L.hccs_calibrate_grid_static.argtypes = [vp, i32, i32, i32, i32, ctypes.POINTER(ctypes.c_double), vp, i32, vp,
                                                 vp, vp]
        L.hccs_exp_softmax_i8_f32.argtypes = [vp, vp, i32, i32, i32, i32, ctypes.POINTER(ctypes.c_float), vp]
        L.hccs_reciprocal_u8.argtypes = [vp, vp, i64, vp]
        L.hccs_copy_bytes.argtypes = [vp, vp, i64, vp]
        L.hccs_largest_probability_u8.argtypes = [vp, i32, i32, vp]
        L.hccs_normalise_table_u8.argtypes = [vp, vp, i64, vp]
        L.hccs_status_string.argtypes = [i32]
        L.hccs_status_string.restype = ctypes.c_char_p
        for name in EXPORTS[:-1]:
            if name != "hccs_calibrate_workspace_bytes":
                getattr(L, name).restype = i32
        _lib = L
    return _lib


def status_string(status):
    return lib().hccs_status_string(int(status)).decode()


def _check(status):
    if status != 0:
        raise HccsError(status, status_string(status))


def head_table(table):
    """[H,3] integers (B, S, Dmax) -> C array of hccs_head_params (values beyond 32 bits are
    clipped to the int32 range, which the library then rejects as out of range)."""
    t = np.clip(np.asarray(table, dtype=np.int64).reshape(-1, 3), -2**31, 2**31 - 1)
    packed = np.zeros((t.shape[0], 4), dtype=np.int32)
    packed[:, :3] = t
    return (HeadParams * t.shape[0]).from_buffer_copy(packed.tobytes()), t.shape[0]


def requant_table(requant):
    t = np.clip(np.asarray(requant, dtype=np.int64).reshape(-1, 2), -2**31, 2**31 - 1).astype(np.int32)
    return (Requant * t.shape[0]).from_buffer_copy(np.ascontiguousarray(t).tobytes()), t.shape[0]


def validate_params(table, n, band):
    """Returns (status, first_bad_head).  Host only; needs no GPU."""
    arr, H = head_table(table)
    bad = ctypes.c_int32(-1)
    rc = lib().hccs_validate_params(arr, H, int(n), int(band), ctypes.byref(bad))
    return rc, bad.value


def _stream_handle(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def calibrated_softmax_i8(logits, table, band, out=None, out_scale_T=255, stream=None):
    """logits: int8 CUDA tensor [B,H,Lq,Lk] (contiguous).  Returns the uint8 tensor of
    probabilities (allocated here unless `out` is given)."""
    import torch
    assert logits.is_cuda and logits.dtype == torch.int8 and logits.is_contiguous() and logits.dim() == 4
    if out is None:
        out = torch.empty(logits.shape, dtype=torch.uint8, device=logits.device)
    assert out.is_cuda and out.dtype == torch.uint8 and out.is_contiguous() and out.shape == logits.shape
    B, H, Lq, Lk = logits.shape
    arr, Ht = head_table(table)
    if Ht != H:
        raise HccsError(-2, "table must have one entry per head")
    _check(lib().hccs_calibrated_softmax_i8(ctypes.c_void_p(logits.data_ptr()), ctypes.c_void_p(out.data_ptr()),
                                            B, H, Lq, Lk, arr, int(out_scale_T), int(band),
                                            _stream_handle(stream)))
    return out


def calibrated_softmax_i8_ex(logits, table, band, out_scale_T=255, reciprocal=RECIP_EXACT, out=None, stream=None):
    """Any output mode: uint8 result for out_scale_T = 255, uint16 (held in an int16 tensor,
    values 0..32767) for out_scale_T = 32767; exact or leading-bit reciprocal."""
    import torch
    assert logits.is_cuda and logits.dtype == torch.int8 and logits.is_contiguous() and logits.dim() == 4
    dtype = torch.uint8 if out_scale_T == 255 else torch.int16
    if out is None:
        out = torch.empty(logits.shape, dtype=dtype, device=logits.device)
    assert out.is_cuda and out.dtype == dtype and out.is_contiguous() and out.shape == logits.shape
    assert out.device == logits.device
    B, H, Lq, Lk = logits.shape
    arr, Ht = head_table(table)
    if Ht != H:
        raise HccsError(-2, "table must have one entry per head")
    _check(lib().hccs_calibrated_softmax_i8_ex(ctypes.c_void_p(logits.data_ptr()), ctypes.c_void_p(out.data_ptr()),
                                               B, H, Lq, Lk, arr, int(out_scale_T), int(reciprocal), int(band),
                                               _stream_handle(stream)))
    return out


def prepare_softmax(logits, out, table, band, out_scale_T=255):
    """Marshals one hccs_calibrated_softmax_i8 call once and returns `launch(stream=None)`,
    for loops where the per-call Python cost matters.  The tensors must stay alive."""
    import torch
    assert logits.is_cuda and logits.dtype == torch.int8 and logits.is_contiguous() and logits.dim() == 4
    assert out.is_cuda and out.dtype == torch.uint8 and out.is_contiguous() and out.shape == logits.shape
    B, H, Lq, Lk = logits.shape
    arr, Ht = head_table(table)
    if Ht != H:
        raise HccsError(-2, "table must have one entry per head")
    fn = lib().hccs_calibrated_softmax_i8
    args = (ctypes.c_void_p(logits.data_ptr()), ctypes.c_void_p(out.data_ptr()), B, H, Lq, Lk, arr,
            int(out_scale_T), int(band))

    def launch(stream=None):
        rc = fn(*args, _stream_handle(stream))
        if rc != 0:
            _check(rc)

    return launch


def _check_attention_tensors(q, k, v, out):
    import torch
    for t in (q, k, v):
        assert t.is_cuda and t.dtype == torch.int8 and t.is_contiguous() and t.dim() == 4 and t.device == q.device
    assert k.shape == v.shape and q.shape[:2] == k.shape[:2] and q.shape[3] == k.shape[3]
    assert out.is_cuda and out.dtype == torch.int32 and out.is_contiguous() and out.shape == q.shape
    assert out.device == q.device


def prepare_attention(q, k, v, out, table, requant, band, out_scale_T=255):
    """Same as prepare_softmax for hccs_attention_i8 (square blocks: Lq = Lk)."""
    _check_attention_tensors(q, k, v, out)
    assert q.shape == k.shape, "prepare_attention takes square blocks; use attention_i8 for Lq != Lk"
    B, H, L, d = q.shape
    arr, Ht = head_table(table)
    rq, Hr = requant_table(requant)
    if Ht != H or Hr != H:
        raise HccsError(-2, "table and requant must have one entry per head")
    fn = lib().hccs_attention_i8
    args = (ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(k.data_ptr()), ctypes.c_void_p(v.data_ptr()),
            ctypes.c_void_p(out.data_ptr()), B, H, L, d, arr, rq, int(out_scale_T), int(band))

    def launch(stream=None):
        rc = fn(*args, _stream_handle(stream))
        if rc != 0:
            _check(rc)

    return launch


def attention_i8(q, k, v, table, requant, band, out=None, out_scale_T=255, stream=None):
    """q: int8 CUDA [B,H,Lq,d]; k, v: int8 CUDA [B,H,Lk,d].  Returns O int32 [B,H,Lq,d].
    Square inputs go through hccs_attention_i8, others through hccs_attention_i8_ex."""
    import torch
    if out is None:
        out = torch.empty(q.shape, dtype=torch.int32, device=q.device)
    _check_attention_tensors(q, k, v, out)
    B, H, Lq, d = q.shape
    Lk = k.shape[2]
    arr, Ht = head_table(table)
    rq, Hr = requant_table(requant)
    if Ht != H or Hr != H:
        raise HccsError(-2, "table and requant must have one entry per head")
    ptrs = (ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(k.data_ptr()), ctypes.c_void_p(v.data_ptr()),
            ctypes.c_void_p(out.data_ptr()))
    if Lq == Lk:
        _check(lib().hccs_attention_i8(*ptrs, B, H, Lk, d, arr, rq, int(out_scale_T), int(band),
                                       _stream_handle(stream)))
    else:
        _check(lib().hccs_attention_i8_ex(*ptrs, B, H, Lq, Lk, d, arr, rq, int(out_scale_T), int(band),
                                          _stream_handle(stream)))
    return out


def calibrate_grid(logits, alpha, candidates, stream=None):
    """Grid-search calibration.  logits int8 CUDA [B,H,Lq,Lk]; alpha: H floats; candidates: [nc,3] integers
    (B, S, Dmax).  Returns (objective float64 CUDA [H,nc], best int32 CUDA [H])."""
    import torch
    assert logits.is_cuda and logits.dtype == torch.int8 and logits.is_contiguous() and logits.dim() == 4
    B, H, Lq, Lk = logits.shape
    assert len(alpha) == H
    cand = np.zeros((len(candidates), 4), dtype=np.int32)
    cand[:, :3] = np.asarray(candidates, dtype=np.int64).reshape(-1, 3).clip(-2**31, 2**31 - 1)
    nc = cand.shape[0]
    need = lib().hccs_calibrate_workspace_bytes(B, H, Lq, Lk)
    if need < 0:
        _check(int(need))
    if stream is None:
        stream = torch.cuda.current_stream(logits.device)
    # the temporaries are allocated, filled and used on `stream`, and told to the allocator as in use
    # there, so that freeing them on return cannot hand their memory out while the kernels still run
    with torch.cuda.stream(stream):
        cand_dev = torch.from_numpy(cand).to(logits.device)
        work = torch.empty(need // 8 + 1, dtype=torch.float64, device=logits.device)
        obj = torch.empty((H, nc), dtype=torch.float64, device=logits.device)
        best = torch.empty(H, dtype=torch.int32, device=logits.device)
    al = (ctypes.c_double * H)(*[float(a) for a in alpha])
    _check(lib().hccs_calibrate_grid(ctypes.c_void_p(logits.data_ptr()), B, H, Lq, Lk, al,
                                     ctypes.c_void_p(cand_dev.data_ptr()), nc, ctypes.c_void_p(obj.data_ptr()),
                                     ctypes.c_void_p(best.data_ptr()), ctypes.c_void_p(work.data_ptr()),
                                     work.numel() * 8, _stream_handle(stream)))
    for t in (cand_dev, work):
        t.record_stream(stream)
    return obj, best


def calibrate_grid_static(logits, alpha, candidates_dev, objective, best, stream=None):
    """hccs_calibrate_grid_static: every buffer is the caller's (candidates_dev int32 CUDA [nc,4] rows of
    (B, S, Dmax, 0), objective float64 CUDA [H,nc], best int32 CUDA [H]); nothing is allocated."""
    import torch
    assert logits.is_cuda and logits.dtype == torch.int8 and logits.is_contiguous() and logits.dim() == 4
    B, H, Lq, Lk = logits.shape
    nc = candidates_dev.shape[0]
    assert candidates_dev.is_cuda and candidates_dev.dtype == torch.int32 and candidates_dev.is_contiguous()
    assert candidates_dev.dim() == 2 and candidates_dev.shape[1] == 4
    assert objective.is_cuda and objective.dtype == torch.float64 and objective.is_contiguous()
    assert tuple(objective.shape) == (H, nc)
    assert best.is_cuda and best.dtype == torch.int32 and best.is_contiguous() and tuple(best.shape) == (H,)
    assert len(alpha) == H
    al = (ctypes.c_double * H)(*[float(a) for a in alpha])
    _check(lib().hccs_calibrate_grid_static(ctypes.c_void_p(logits.data_ptr()), B, H, Lq, Lk, al,
                                            ctypes.c_void_p(candidates_dev.data_ptr()), nc,
                                            ctypes.c_void_p(objective.data_ptr()), ctypes.c_void_p(best.data_ptr()),
                                            _stream_handle(stream)))
    return objective, best


def exp_softmax_i8_f32(logits, scale, out=None, stream=None):
    """Benchmark comparison kernel: uint8 rint(255*softmax(scale_h*x))."""
    import torch
    assert logits.is_cuda and logits.dtype == torch.int8 and logits.is_contiguous() and logits.dim() == 4
    if out is None:
        out = torch.empty(logits.shape, dtype=torch.uint8, device=logits.device)
    assert out.is_cuda and out.dtype == torch.uint8 and out.is_contiguous() and out.shape == logits.shape
    B, H, Lq, Lk = logits.shape
    assert len(scale) == H
    sc = (ctypes.c_float * H)(*[float(s) for s in scale])
    _check(lib().hccs_exp_softmax_i8_f32(ctypes.c_void_p(logits.data_ptr()), ctypes.c_void_p(out.data_ptr()),
                                         B, H, Lq, Lk, sc, _stream_handle(stream)))
    return out


def reciprocal_u8(z, out=None, stream=None):
    """z: uint32 values held in an int32/uint32 CUDA tensor; returns floor(255*2^15 / z) per element."""
    import torch
    assert z.is_cuda and z.dtype == torch.int32 and z.is_contiguous()
    if out is None:
        out = torch.empty_like(z)
    assert out.is_cuda and out.dtype == torch.int32 and out.is_contiguous() and out.numel() == z.numel()
    _check(lib().hccs_reciprocal_u8(ctypes.c_void_p(z.data_ptr()), ctypes.c_void_p(out.data_ptr()),
                                    z.numel(), _stream_handle(stream)))
    return out


def normalise_table_u8(bsdz, stream=None):
    """bsdz: int32 CUDA tensor [count,4] of (B, S, Dmax, Z).  Returns uint8 [count,256]: p(delta)."""
    import torch
    assert bsdz.is_cuda and bsdz.dtype == torch.int32 and bsdz.is_contiguous() and bsdz.shape[1] == 4
    out = torch.empty((bsdz.shape[0], 256), dtype=torch.uint8, device=bsdz.device)
    _check(lib().hccs_normalise_table_u8(ctypes.c_void_p(bsdz.data_ptr()), ctypes.c_void_p(out.data_ptr()),
                                         bsdz.shape[0], _stream_handle(stream)))
    return out


def largest_probability_u8(params, n):
    """Per head, the largest 8-bit probability a row of n keys can get under (B, S, Dmax) (host only)."""
    table = np.ascontiguousarray(params, dtype=np.int32)
    assert table.ndim == 2 and table.shape[1] == 3
    out = np.zeros(table.shape[0], np.int32)
    _check(lib().hccs_largest_probability_u8(table.ctypes.data_as(ctypes.c_void_p), table.shape[0], int(n),
                                             out.ctypes.data_as(ctypes.c_void_p)))
    return out


def copy_bytes(src, dst, stream=None):
    assert src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()
    nbytes = src.numel() * src.element_size()
    assert nbytes == dst.numel() * dst.element_size()
    _check(lib().hccs_copy_bytes(ctypes.c_void_p(src.data_ptr()), ctypes.c_void_p(dst.data_ptr()),
                                 nbytes, _stream_handle(stream)))
    return dst
