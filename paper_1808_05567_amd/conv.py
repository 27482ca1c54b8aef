"""Thin ctypes binding over libconv_mi355x.so (the C ABI of include/conv_mi355x.h).

Argument marshalling only: every step of the convolution runs in the HIP
kernels of the library.  torch is used for device memory and streams.  If the
library is not built this module raises; there is no fallback.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
# (CONVMI_LIB: another build of the same library, for tuning experiments)
LIB_PATH = os.environ.get("CONVMI_LIB") or os.path.join(_HERE, "libconv_mi355x.so")

CONV_F32 = 0
CONV_BF16 = 1
PASS_FWD, PASS_BWD_DATA, PASS_UPD = 0, 1, 2

CONV_OK, CONV_EINVAL, CONV_EUNSUPPORTED, CONV_EWORKSPACE, CONV_ELAUNCH, CONV_ESCRATCH = range(6)

EXPORTS = (
    "conv_create", "conv_create_rect", "conv_create_chunked", "conv_destroy", "conv_query", "conv_status_str",
    "conv_fwd", "conv_fwd_fused", "conv_fwd_fused_norm", "conv_bwd_data", "conv_upd",
    "conv_fwd_ws", "conv_bwd_data_ws", "conv_upd_ws",
    "conv_bwd_data_noalloc", "conv_noalloc_scratch_bytes",
    "conv_pack_in", "conv_pack_out", "conv_pack_wt",
    "conv_unpack_in", "conv_unpack_out", "conv_unpack_wt", "conv_unpack_dwt",
    "conv_describe",
    "conv_ceiling_mfma", "conv_ceiling_copy", "conv_ceiling_read", "conv_ceiling_write",
    "conv_ceiling_l2_to_lds", "conv_ceiling_lds_read", "conv_ceiling_shader_clock",
)


class ConvDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "C", "K", "H", "W", "R", "S", "stride", "pad", "dtype")]


class ConvInfo(ctypes.Structure):
    _fields_ = [("P", ctypes.c_int32), ("Q", ctypes.c_int32), ("vlen", ctypes.c_int32),
                ("Cb", ctypes.c_int32), ("Kb", ctypes.c_int32),
                ("Cp", ctypes.c_int32), ("Kp", ctypes.c_int32),
                ("in_bytes", ctypes.c_size_t), ("out_bytes", ctypes.c_size_t),
                ("wt_bytes", ctypes.c_size_t), ("dwt_bytes", ctypes.c_size_t),
                ("workspace_bytes", ctypes.c_size_t),
                ("upd_splits", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class ConvError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s: %s" % (what, status_str(status)))


_lib = None


def load():
    """Load the HIP library (after torch, so both share one HIP runtime)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "libconv_mi355x.so is not built; run `python -m paper_1808_05567_amd.build` "
            "(there is no fallback implementation)")
    try:
        import torch  # noqa: F401  (loads libamdhip64 first)
    except ImportError:
        pass
    lib = ctypes.CDLL(LIB_PATH)
    vp = ctypes.c_void_p
    lib.conv_create.argtypes = [ctypes.POINTER(ConvDesc), ctypes.POINTER(vp)]
    lib.conv_create_rect.argtypes = [ctypes.POINTER(ConvDesc), ctypes.c_int32, ctypes.c_int32,
                                     ctypes.POINTER(vp)]
    lib.conv_create_chunked.argtypes = [ctypes.POINTER(ConvDesc), ctypes.c_int32, ctypes.c_int32,
                                        ctypes.c_int32, ctypes.POINTER(vp)]
    lib.conv_destroy.argtypes = [vp]
    lib.conv_query.argtypes = [vp, ctypes.POINTER(ConvInfo)]
    lib.conv_status_str.argtypes = [ctypes.c_int]
    lib.conv_status_str.restype = ctypes.c_char_p
    for name in ("conv_fwd", "conv_bwd_data", "conv_upd"):
        getattr(lib, name).argtypes = [vp, vp, vp, vp, vp, vp]
    for name in ("conv_fwd_ws", "conv_bwd_data_ws", "conv_upd_ws"):
        getattr(lib, name).argtypes = [vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.conv_fwd_fused.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.c_int32, vp, vp]
    lib.conv_fwd_fused_norm.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.c_int32, vp, vp]
    for name in ("conv_pack_in", "conv_pack_out", "conv_pack_wt", "conv_unpack_in",
                 "conv_unpack_out", "conv_unpack_wt", "conv_unpack_dwt"):
        getattr(lib, name).argtypes = [vp, vp, vp, vp]
    lib.conv_describe.argtypes = [vp, ctypes.c_int32, ctypes.c_char_p, ctypes.c_size_t]
    lib.conv_ceiling_mfma.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp]
    lib.conv_ceiling_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    lib.conv_ceiling_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
    lib.conv_ceiling_write.argtypes = [vp, ctypes.c_size_t, vp]
    lib.conv_ceiling_l2_to_lds.argtypes = [vp, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                           vp, vp]
    lib.conv_ceiling_lds_read.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp]
    lib.conv_ceiling_shader_clock.argtypes = [ctypes.c_int32, ctypes.c_int32, vp, vp]
    lib.conv_bwd_data_noalloc.argtypes = [vp, vp, vp, vp, vp]
    lib.conv_noalloc_scratch_bytes.argtypes = []
    lib.conv_noalloc_scratch_bytes.restype = ctypes.c_size_t
    for name in EXPORTS:
        if name not in ("conv_status_str", "conv_noalloc_scratch_bytes"):
            getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def status_str(status: int) -> str:
    return load().conv_status_str(int(status)).decode()


def _ptr(x):
    """Device pointer of a torch tensor, or an int/None passed through."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(status, what):
    if status != CONV_OK:
        raise ConvError(status, what)


def conv_create(N, C, K, H, W, R, S, stride, pad, dtype=CONV_F32):
    """``pad``: one value for both axes, or a pair (pad_h, pad_w) (conv_create_rect)."""
    if isinstance(pad, (tuple, list)):
        return conv_create_rect(N, C, K, H, W, R, S, stride, pad[0], pad[1], dtype)
    d = ConvDesc(N, C, K, H, W, R, S, stride, pad, dtype)
    h = ctypes.c_void_p()
    _check(load().conv_create(ctypes.byref(d), ctypes.byref(h)), "conv_create")
    return h


def conv_create_rect(N, C, K, H, W, R, S, stride, pad_h, pad_w, dtype=CONV_F32):
    d = ConvDesc(N, C, K, H, W, R, S, stride, 0, dtype)
    h = ctypes.c_void_p()
    _check(load().conv_create_rect(ctypes.byref(d), int(pad_h), int(pad_w), ctypes.byref(h)),
           "conv_create_rect")
    return h


def conv_create_chunked(N, C, K, H, W, R, S, stride, pad, max_images, dtype=CONV_F32):
    """The minibatch in chunks of at most ``max_images`` images per launch."""
    ph, pw = pad if isinstance(pad, (tuple, list)) else (pad, pad)
    d = ConvDesc(N, C, K, H, W, R, S, stride, 0, dtype)
    h = ctypes.c_void_p()
    _check(load().conv_create_chunked(ctypes.byref(d), int(ph), int(pw), int(max_images),
                                      ctypes.byref(h)), "conv_create_chunked")
    return h


def conv_destroy(h):
    _check(load().conv_destroy(h), "conv_destroy")


def conv_query(h) -> ConvInfo:
    info = ConvInfo()
    _check(load().conv_query(h, ctypes.byref(info)), "conv_query")
    return info


def conv_describe(h, which: int) -> str:
    buf = ctypes.create_string_buffer(512)
    _check(load().conv_describe(h, which, buf, 512), "conv_describe")
    return buf.value.decode()


def conv_fwd(h, inp, wt, out, ws=None, stream=None):
    _check(load().conv_fwd(h, _ptr(inp), _ptr(wt), _ptr(out), _ptr(ws), _stream(stream)), "conv_fwd")


def conv_fwd_fused(h, inp, wt, out, bias=None, residual=None, relu=False, ws=None, stream=None):
    _check(load().conv_fwd_fused(h, _ptr(inp), _ptr(wt), _ptr(out), _ptr(bias), _ptr(residual),
                                 1 if relu else 0, _ptr(ws), _stream(stream)), "conv_fwd_fused")


def conv_fwd_fused_norm(h, inp, wt, out, scale=None, bias=None, residual=None, relu=False, ws=None,
                        stream=None):
    _check(load().conv_fwd_fused_norm(h, _ptr(inp), _ptr(wt), _ptr(out), _ptr(scale), _ptr(bias),
                                      _ptr(residual), 1 if relu else 0, _ptr(ws), _stream(stream)),
           "conv_fwd_fused_norm")


def conv_bwd_data(h, dout, wt, din, ws, stream=None):
    _check(load().conv_bwd_data(h, _ptr(dout), _ptr(wt), _ptr(din), _ptr(ws), _stream(stream)),
           "conv_bwd_data")


def conv_upd(h, inp, dout, dwt, ws, stream=None):
    _check(load().conv_upd(h, _ptr(inp), _ptr(dout), _ptr(dwt), _ptr(ws), _stream(stream)),
           "conv_upd")


def conv_bwd_data_noalloc(h, dout, wt, din, stream=None):
    _check(load().conv_bwd_data_noalloc(h, _ptr(dout), _ptr(wt), _ptr(din), _stream(stream)),
           "conv_bwd_data_noalloc")


def _ws_bytes(ws):
    return 0 if ws is None else ws.numel() * ws.element_size()


def conv_fwd_ws(h, inp, wt, out, ws, stream=None):
    _check(load().conv_fwd_ws(h, _ptr(inp), _ptr(wt), _ptr(out), _ptr(ws), _ws_bytes(ws),
                              _stream(stream)), "conv_fwd_ws")


def conv_bwd_data_ws(h, dout, wt, din, ws, stream=None):
    _check(load().conv_bwd_data_ws(h, _ptr(dout), _ptr(wt), _ptr(din), _ptr(ws), _ws_bytes(ws),
                                   _stream(stream)), "conv_bwd_data_ws")


def conv_upd_ws(h, inp, dout, dwt, ws, stream=None):
    _check(load().conv_upd_ws(h, _ptr(inp), _ptr(dout), _ptr(dwt), _ptr(ws), _ws_bytes(ws),
                              _stream(stream)), "conv_upd_ws")


def conv_ceiling_mfma(dtype, blocks, iters, sink, stream=None):
    _check(load().conv_ceiling_mfma(dtype, blocks, iters, _ptr(sink), _stream(stream)),
           "conv_ceiling_mfma")


def conv_ceiling_copy(dst, src, nbytes, stream=None):
    _check(load().conv_ceiling_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)), "conv_ceiling_copy")


def conv_ceiling_read(src, nbytes, sink, stream=None):
    _check(load().conv_ceiling_read(_ptr(src), nbytes, _ptr(sink), _stream(stream)), "conv_ceiling_read")


def conv_ceiling_write(dst, nbytes, stream=None):
    _check(load().conv_ceiling_write(_ptr(dst), nbytes, _stream(stream)), "conv_ceiling_write")


def conv_ceiling_lds_read(blocks, iters, sink, row_len=0, row_pitch=0, stream=None):
    _check(load().conv_ceiling_lds_read(blocks, iters, row_len, row_pitch, _ptr(sink), _stream(stream)),
           "conv_ceiling_lds_read")


def conv_ceiling_shader_clock(blocks, duration_us, ticks, stream=None):
    """ticks: int64 device tensor of 2 * blocks elements (cycles, 100 MHz ticks per workgroup)."""
    _check(load().conv_ceiling_shader_clock(blocks, duration_us, _ptr(ticks), _stream(stream)),
           "conv_ceiling_shader_clock")


def conv_ceiling_l2_to_lds(src, src_bytes, blocks, iters, sink, through_registers=False, stream=None):
    _check(load().conv_ceiling_l2_to_lds(_ptr(src), src_bytes, blocks, iters,
                                         1 if through_registers else 0, _ptr(sink),
                                         _stream(stream)), "conv_ceiling_l2_to_lds")


def _perm(name):
    def f(h, src, dst, stream=None):
        _check(getattr(load(), name)(h, _ptr(src), _ptr(dst), _stream(stream)), name)
    f.__name__ = name
    return f


conv_pack_in = _perm("conv_pack_in")
conv_pack_out = _perm("conv_pack_out")
conv_pack_wt = _perm("conv_pack_wt")
conv_unpack_in = _perm("conv_unpack_in")
conv_unpack_out = _perm("conv_unpack_out")
conv_unpack_wt = _perm("conv_unpack_wt")
conv_unpack_dwt = _perm("conv_unpack_dwt")


class ConvLayer:
    """Convenience holder: a handle plus torch device buffers of the sizes
    conv_query reports.  Logical tensors go in and come out as torch tensors in
    NCHW / KCRS; all computation and all layout conversion is done by the
    library's kernels."""

    def __init__(self, N, C, K, H, W, R, S, stride, pad, dtype=CONV_F32, device="cuda:0",
                 max_images=None):
        import torch
        self.torch = torch
        self.shape = (N, C, K, H, W, R, S, stride, pad)
        self.dtype = dtype
        self.tdtype = torch.bfloat16 if dtype == CONV_BF16 else torch.float32
        self.device = torch.device(device)
        if max_images is None:
            self.h = conv_create(N, C, K, H, W, R, S, stride, pad, dtype)
        else:
            self.h = conv_create_chunked(N, C, K, H, W, R, S, stride, pad, max_images, dtype)
        self.info = conv_query(self.h)
        es = 2 if dtype == CONV_BF16 else 4
        i = self.info
        self.in_blk = torch.empty(i.in_bytes // es, dtype=self.tdtype, device=self.device)
        self.out_blk = torch.empty(i.out_bytes // es, dtype=self.tdtype, device=self.device)
        self.wt_blk = torch.empty(i.wt_bytes // es, dtype=self.tdtype, device=self.device)
        self.dwt_blk = torch.empty(i.dwt_bytes // 4, dtype=torch.float32, device=self.device)
        self.ws = torch.empty(max(16, i.workspace_bytes), dtype=torch.uint8, device=self.device)

    def close(self):
        if self.h is not None:
            conv_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _dev(self, a, dtype):
        t = a if isinstance(a, self.torch.Tensor) else self.torch.from_numpy(a)
        return t.to(device=self.device, dtype=dtype).contiguous()

    # -- logical -> blocked
    def set_input(self, I):
        N, C, K, H, W = self.shape[:5]
        t = self._dev(I, self.tdtype)
        assert tuple(t.shape) == (N, C, H, W)
        conv_pack_in(self.h, t, self.in_blk)

    def set_weights(self, Wt):
        N, C, K, H, W, R, S = self.shape[:7]
        t = self._dev(Wt, self.tdtype)
        assert tuple(t.shape) == (K, C, R, S)
        conv_pack_wt(self.h, t, self.wt_blk)

    def set_outgrad(self, dO):
        N, C, K = self.shape[:3]
        t = self._dev(dO, self.tdtype)
        assert tuple(t.shape) == (N, K, self.info.P, self.info.Q)
        conv_pack_out(self.h, t, self.out_blk)

    # -- passes on the blocked buffers
    def fwd(self):
        conv_fwd(self.h, self.in_blk, self.wt_blk, self.out_blk, self.ws)

    def fwd_fused(self, bias=None, residual=None, relu=False, scale=None):
        """scale, bias: fp32 device tensors of Kp entries; residual: blocked tensor like out_blk."""
        if scale is not None:
            conv_fwd_fused_norm(self.h, self.in_blk, self.wt_blk, self.out_blk, scale, bias, residual,
                                relu, self.ws)
            return
        conv_fwd_fused(self.h, self.in_blk, self.wt_blk, self.out_blk, bias, residual, relu, self.ws)

    def bwd_data(self):
        conv_bwd_data(self.h, self.out_blk, self.wt_blk, self.in_blk, self.ws)

    def upd(self):
        conv_upd(self.h, self.in_blk, self.out_blk, self.dwt_blk, self.ws)

    # -- blocked -> logical
    def get_output(self):
        N, C, K = self.shape[:3]
        t = self.torch.empty((N, K, self.info.P, self.info.Q), dtype=self.tdtype, device=self.device)
        conv_unpack_out(self.h, self.out_blk, t)
        return t

    def get_input(self):
        N, C, K, H, W = self.shape[:5]
        t = self.torch.empty((N, C, H, W), dtype=self.tdtype, device=self.device)
        conv_unpack_in(self.h, self.in_blk, t)
        return t

    def get_weights(self):
        N, C, K, H, W, R, S = self.shape[:7]
        t = self.torch.empty((K, C, R, S), dtype=self.tdtype, device=self.device)
        conv_unpack_wt(self.h, self.wt_blk, t)
        return t

    def get_dweights(self):
        N, C, K, H, W, R, S = self.shape[:7]
        t = self.torch.empty((K, C, R, S), dtype=self.torch.float32, device=self.device)
        conv_unpack_dwt(self.h, self.dwt_blk, t)
        return t
