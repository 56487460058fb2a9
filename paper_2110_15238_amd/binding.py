"""Thin ctypes binding of libbolt.so (include/bolt.h).  Argument marshalling only.

Every function takes torch CUDA (ROCm) float16 tensors, passes their device pointers and the
current HIP stream to the C ABI, and raises BoltError on a non-zero status.  There is no fallback:
if the library is missing the import of this module fails.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbolt.so")

OP_GEMM, OP_CONV2D, OP_B2B_GEMM, OP_B2B_CONV, OP_GEMM_CHAIN3, OP_CONV_CHAIN3 = 0, 1, 2, 3, 4, 5
OP_B2B_GEMM_RES, OP_B2B_CONV_RES = 6, 7
ACT = {"none": 0, "relu": 1, "gelu": 2, "hardswish": 3, "softplus": 4}
LAYOUT_KN, LAYOUT_NK = 0, 1
STATUS_NAMES = ["BOLT_OK", "BOLT_ERR_INVALID_ARG", "BOLT_ERR_UNSUPPORTED", "BOLT_ERR_ALIGNMENT",
                "BOLT_ERR_WORKSPACE", "BOLT_ERR_LAUNCH", "BOLT_ERR_ILLEGAL_FUSION"]


class BoltConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("kernel_id", "tile_m", "tile_n", "tile_k", "waves_m", "waves_n",
                                         "mfma_shape", "stages", "swizzle", "split_k", "b2b_mode")]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}

    @classmethod
    def from_dict(cls, d):
        c = cls()
        for n, _ in cls._fields_:
            setattr(c, n, int(d.get(n, 0)))
        return c


class GemmDesc(C.Structure):
    _fields_ = [("M", C.c_int32), ("N", C.c_int32), ("K", C.c_int32), ("lda", C.c_int32), ("ldb", C.c_int32),
                ("ldd", C.c_int32), ("alpha", C.c_float), ("beta", C.c_float), ("act", C.c_int32),
                ("b_layout", C.c_int32)]


class ConvDesc(C.Structure):
    _fields_ = [("N", C.c_int32), ("H", C.c_int32), ("W", C.c_int32), ("C", C.c_int32), ("K", C.c_int32),
                ("R", C.c_int32), ("S", C.c_int32), ("stride_h", C.c_int32), ("stride_w", C.c_int32),
                ("pad_h", C.c_int32), ("pad_w", C.c_int32), ("alpha", C.c_float), ("beta", C.c_float),
                ("act", C.c_int32), ("x_layout", C.c_int32), ("y_layout", C.c_int32)]


TENSOR_NHWC, TENSOR_NCHW = 0, 1


class BoltError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        name = STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else str(status)
        super().__init__("%s: %s (%s)" % (where, name, status_string(status)))


if not os.path.exists(LIB_PATH):
    raise ImportError("libbolt.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                      "(or `make -C paper_2110_15238_amd/csrc`) first; there is no fallback path")

_lib = C.CDLL(LIB_PATH)
_vp, _i32, _sz = C.c_void_p, C.c_int32, C.c_size_t
_lib.bolt_status_string.restype = C.c_char_p
_lib.bolt_status_string.argtypes = [C.c_int]
_lib.bolt_num_instances.restype = _i32
_lib.bolt_num_instances.argtypes = [C.c_int]
_lib.bolt_instance_config.restype = C.c_int
_lib.bolt_instance_config.argtypes = [C.c_int, _i32, C.POINTER(BoltConfig)]
_lib.bolt_instance_supports.restype = _i32
_lib.bolt_instance_supports.argtypes = [C.c_int, _i32, _vp, _vp]
_lib.bolt_check.restype = C.c_int
_lib.bolt_check.argtypes = [C.c_int, _vp, _vp, C.POINTER(BoltConfig)]
_lib.bolt_workspace_bytes.restype = _sz
_lib.bolt_workspace_bytes.argtypes = [C.c_int, _vp, _vp, C.POINTER(BoltConfig)]
_lib.bolt_gemm_epilogue.restype = C.c_int
_lib.bolt_gemm_epilogue.argtypes = [C.POINTER(GemmDesc), _vp, _vp, _vp, _vp, C.POINTER(BoltConfig), _vp, _sz, _vp]
_lib.bolt_gemm_epilogue_noalloc.restype = C.c_int
_lib.bolt_gemm_epilogue_noalloc.argtypes = [C.POINTER(GemmDesc), _vp, _vp, _vp, _vp, C.POINTER(BoltConfig), _vp]
_lib.bolt_conv2d_fprop_nhwc.restype = C.c_int
_lib.bolt_conv2d_fprop_nhwc.argtypes = [C.POINTER(ConvDesc), _vp, _vp, _vp, _vp, C.POINTER(BoltConfig), _vp, _sz, _vp]
_lib.bolt_b2b_gemm.restype = C.c_int
_lib.bolt_b2b_gemm.argtypes = [C.POINTER(GemmDesc), C.POINTER(GemmDesc), _vp, _vp, _vp, _vp, _vp, _vp,
                               C.POINTER(BoltConfig), _vp, _sz, _vp]
_lib.bolt_b2b_conv.restype = C.c_int
_lib.bolt_b2b_conv.argtypes = [C.POINTER(ConvDesc), C.POINTER(ConvDesc), _vp, _vp, _vp, _vp, _vp, _vp,
                               C.POINTER(BoltConfig), _vp, _sz, _vp]
_lib.bolt_tune.restype = C.c_int
_lib.bolt_tune.argtypes = [C.c_int, _vp, _vp, C.POINTER(_vp), _vp, _sz, _vp, C.POINTER(BoltConfig),
                           C.POINTER(C.c_float), C.POINTER(_i32)]
_lib.bolt_gemm_epilogue_residual.restype = C.c_int
_lib.bolt_gemm_epilogue_residual.argtypes = [C.POINTER(GemmDesc), _vp, _vp, _vp, _vp, _i32, C.c_float, _vp,
                                             C.POINTER(BoltConfig), _vp, _sz, _vp]
_lib.bolt_conv2d_fprop_nhwc_residual.restype = C.c_int
_lib.bolt_conv2d_fprop_nhwc_residual.argtypes = [C.POINTER(ConvDesc), _vp, _vp, _vp, _vp, C.c_float, _vp,
                                                 C.POINTER(BoltConfig), _vp, _sz, _vp]
_lib.bolt_b2b_gemm_residual.restype = C.c_int
_lib.bolt_b2b_gemm_residual.argtypes = [C.POINTER(GemmDesc), C.POINTER(GemmDesc), _vp, _vp, _vp, _vp, _vp, _vp, _i32,
                                        C.c_float, _vp, C.POINTER(BoltConfig), _vp, _sz, _vp]
_lib.bolt_b2b_conv_residual.restype = C.c_int
_lib.bolt_b2b_conv_residual.argtypes = [C.POINTER(ConvDesc), C.POINTER(ConvDesc), _vp, _vp, _vp, _vp, _vp, _vp,
                                        C.c_float, _vp, C.POINTER(BoltConfig), _vp, _sz, _vp]
_pp = C.POINTER(_vp)
_lib.bolt_b2b_gemm_chain.restype = C.c_int
_lib.bolt_b2b_gemm_chain.argtypes = [_i32, _pp, _vp, _pp, _pp, _vp, C.POINTER(BoltConfig), _vp]
_lib.bolt_b2b_conv_chain.restype = C.c_int
_lib.bolt_b2b_conv_chain.argtypes = [_i32, _pp, _vp, _pp, _pp, _vp, C.POINTER(BoltConfig), _vp]
_lib.bolt_b2b_gemm_chain_residual.restype = C.c_int
_lib.bolt_b2b_gemm_chain_residual.argtypes = [_i32, _pp, _vp, _pp, _pp, _vp, _i32, C.c_float, _vp, C.POINTER(BoltConfig), _vp]
_lib.bolt_b2b_conv_chain_residual.restype = C.c_int
_lib.bolt_b2b_conv_chain_residual.argtypes = [_i32, _pp, _vp, _pp, _pp, _vp, C.c_float, _vp, C.POINTER(BoltConfig), _vp]
_lib.bolt_tune_chain.restype = C.c_int
_lib.bolt_tune_chain.argtypes = [C.c_int, _i32, _pp, _pp, _vp, C.POINTER(BoltConfig), C.POINTER(C.c_float), C.POINTER(_i32)]
_lib.bolt_check_chain.restype = C.c_int
_lib.bolt_check_chain.argtypes = [C.c_int, _i32, _pp, C.POINTER(BoltConfig)]
_lib.bolt_chain_instance_supports.restype = _i32
_lib.bolt_chain_instance_supports.argtypes = [C.c_int, _i32, _i32, _pp]
_lib.bolt_pad_channels_nhwc.restype = C.c_int
_lib.bolt_pad_channels_nhwc.argtypes = [_vp, _vp, C.c_int64, _i32, _i32, _vp]
_lib.bolt_bias_act.restype = C.c_int
_lib.bolt_bias_act.argtypes = [_vp, _vp, C.c_int64, _i32, _i32, C.c_float, C.c_float, C.c_int, _vp]
_lib.bolt_nchw_to_nhwc.restype = C.c_int
_lib.bolt_nchw_to_nhwc.argtypes = [_vp, _vp, _i32, _i32, _i32, _i32, _i32, _vp]
_lib.bolt_nhwc_to_nchw.restype = C.c_int
_lib.bolt_nhwc_to_nchw.argtypes = [_vp, _vp, _i32, _i32, _i32, _i32, _i32, _vp]
_lib.bolt_probe_mfma_peak.restype = C.c_int
_lib.bolt_probe_mfma_peak.argtypes = [_i32, _vp, C.POINTER(C.c_float)]
_lib.bolt_probe_copy_bandwidth.restype = C.c_int
_lib.bolt_probe_copy_bandwidth.argtypes = [_vp, _sz, _i32, _vp, C.POINTER(C.c_float)]

EXPORTED = ["bolt_gemm_epilogue", "bolt_gemm_epilogue_noalloc", "bolt_conv2d_fprop_nhwc", "bolt_b2b_gemm", "bolt_b2b_conv", "bolt_tune",
            "bolt_gemm_epilogue_residual", "bolt_conv2d_fprop_nhwc_residual", "bolt_b2b_gemm_residual",
            "bolt_b2b_conv_residual", "bolt_b2b_gemm_chain", "bolt_b2b_conv_chain",
            "bolt_b2b_gemm_chain_residual", "bolt_b2b_conv_chain_residual", "bolt_tune_chain", "bolt_check_chain",
            "bolt_chain_instance_supports",
            "bolt_pad_channels_nhwc", "bolt_nchw_to_nhwc", "bolt_nhwc_to_nchw", "bolt_bias_act", "bolt_workspace_bytes", "bolt_check", "bolt_status_string",
            "bolt_num_instances", "bolt_instance_config", "bolt_instance_supports", "bolt_probe_mfma_peak",
            "bolt_probe_copy_bandwidth"]


def status_string(status: int) -> str:
    return _lib.bolt_status_string(int(status)).decode()


def raw():
    """The ctypes library handle (tests call the C ABI directly through it)."""
    return _lib


_torch = None
_raw_stream = None


def _load_torch():
    global _torch, _raw_stream
    import torch
    _torch = torch
    # the raw-handle query skips building a Stream object (about a microsecond per call)
    _raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)
    return torch


def _stream() -> int:
    torch = _torch or _load_torch()
    if _raw_stream is not None:
        return _raw_stream(torch.cuda.current_device())
    return int(torch.cuda.current_stream().cuda_stream)


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    torch = _torch or _load_torch()
    assert t.is_cuda and t.dtype is torch.float16 and t.is_contiguous(), "expects contiguous CUDA float16 tensors"
    return t.data_ptr()


def _cfg(config) -> Optional[BoltConfig]:
    if config is None:
        return None
    if isinstance(config, BoltConfig):
        return config
    return BoltConfig.from_dict(config)


def _ws(workspace) -> Tuple[Optional[int], int]:
    if workspace is None:
        return None, 0
    assert workspace.is_cuda and workspace.is_contiguous()
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def gemm_desc(M, N, K, lda=None, ldb=None, ldd=None, alpha=1.0, beta=1.0, act="relu", b_layout=LAYOUT_KN) -> GemmDesc:
    if ldb is None:
        ldb = N if b_layout == LAYOUT_KN else K
    return GemmDesc(M, N, K, K if lda is None else lda, ldb, N if ldd is None else ldd, alpha, beta, ACT[act], b_layout)


def conv_desc(N, H, W, Cin, K, R, S, stride=1, pad=0, alpha=1.0, beta=1.0, act="relu", x_layout="nhwc",
              y_layout="nhwc") -> ConvDesc:
    """x_layout: "nhwc" or "nchw" (the latter for first layers with at most 4 channels); y_layout: "nhwc" or "nchw"
    (the latter for last layers: the output tensor is then [N][K][P][Q])."""
    sh, sw = (stride, stride) if isinstance(stride, int) else stride
    ph, pw = (pad, pad) if isinstance(pad, int) else pad
    return ConvDesc(N, H, W, Cin, K, R, S, sh, sw, ph, pw, alpha, beta, ACT[act],
                    {"nhwc": TENSOR_NHWC, "nchw": TENSOR_NCHW}[x_layout], {"nhwc": TENSOR_NHWC, "nchw": TENSOR_NCHW}[y_layout])


def conv_out_hw(d: ConvDesc) -> Tuple[int, int]:
    return ((d.H + 2 * d.pad_h - d.R) // d.stride_h + 1, (d.W + 2 * d.pad_w - d.S) // d.stride_w + 1)


def _check(status: int, where: str):
    if status != 0:
        raise BoltError(status, where)


def num_instances(op: int) -> int:
    return int(_lib.bolt_num_instances(op))


def instance_config(op: int, kernel_id: int) -> BoltConfig:
    c = BoltConfig()
    _check(_lib.bolt_instance_config(op, kernel_id, C.byref(c)), "bolt_instance_config")
    return c


def instance_supports(op: int, kernel_id: int, desc0, desc1=None) -> bool:
    return bool(_lib.bolt_instance_supports(op, kernel_id, C.addressof(desc0),
                                            None if desc1 is None else C.addressof(desc1)))


def check(op: int, desc0, desc1=None, config=None) -> int:
    """Validation only (works without a GPU): returns the bolt_status code."""
    c = _cfg(config)
    return int(_lib.bolt_check(op, None if desc0 is None else C.addressof(desc0),
                               None if desc1 is None else C.addressof(desc1), None if c is None else C.byref(c)))


def workspace_bytes(op: int, desc0, desc1=None, config=None) -> int:
    c = _cfg(config)
    return int(_lib.bolt_workspace_bytes(op, C.addressof(desc0), None if desc1 is None else C.addressof(desc1),
                                         None if c is None else C.byref(c)))


def gemm_epilogue(desc: GemmDesc, A, B, bias, D, config=None, workspace=None):
    c = _cfg(config)
    wp, wb = _ws(workspace)
    _check(_lib.bolt_gemm_epilogue(C.byref(desc), _ptr(A), _ptr(B), _ptr(bias), _ptr(D),
                                   None if c is None else C.byref(c), wp, wb, _stream()), "bolt_gemm_epilogue")
    return D


def gemm_epilogue_noalloc(desc: GemmDesc, A, B, bias, D, config=None):
    """bolt_gemm_epilogue with the split-K partial sums in the library's own fixed device array."""
    c = _cfg(config)
    _check(_lib.bolt_gemm_epilogue_noalloc(C.byref(desc), _ptr(A), _ptr(B), _ptr(bias), _ptr(D),
                                           None if c is None else C.byref(c), _stream()), "bolt_gemm_epilogue_noalloc")
    return D


def conv2d_fprop_nhwc(desc: ConvDesc, x, w, bias, y, config=None, workspace=None):
    c = _cfg(config)
    wp, wb = _ws(workspace)
    _check(_lib.bolt_conv2d_fprop_nhwc(C.byref(desc), _ptr(x), _ptr(w), _ptr(bias), _ptr(y),
                                       None if c is None else C.byref(c), wp, wb, _stream()),
           "bolt_conv2d_fprop_nhwc")
    return y


def gemm_epilogue_residual(desc: GemmDesc, A, B, bias, Cres, D, gamma: float = 1.0, config=None, workspace=None):
    """D = act(alpha A.B + beta bias + gamma Cres); Cres is a contiguous M x N tensor."""
    c = _cfg(config)
    wp, wb = _ws(workspace)
    _check(_lib.bolt_gemm_epilogue_residual(C.byref(desc), _ptr(A), _ptr(B), _ptr(bias), _ptr(Cres), Cres.shape[-1], gamma,
                                            _ptr(D), None if c is None else C.byref(c), wp, wb, _stream()),
           "bolt_gemm_epilogue_residual")
    return D


def conv2d_fprop_nhwc_residual(desc: ConvDesc, x, w, bias, residual, y, gamma: float = 1.0, config=None, workspace=None):
    c = _cfg(config)
    wp, wb = _ws(workspace)
    _check(_lib.bolt_conv2d_fprop_nhwc_residual(C.byref(desc), _ptr(x), _ptr(w), _ptr(bias), _ptr(residual), gamma, _ptr(y),
                                                None if c is None else C.byref(c), wp, wb, _stream()),
           "bolt_conv2d_fprop_nhwc_residual")
    return y


def b2b_gemm(g0: GemmDesc, g1: GemmDesc, A0, W0, b0, W1, b1, D1, config=None):
    c = _cfg(config)
    _check(_lib.bolt_b2b_gemm(C.byref(g0), C.byref(g1), _ptr(A0), _ptr(W0), _ptr(b0), _ptr(W1), _ptr(b1), _ptr(D1),
                              None if c is None else C.byref(c), None, 0, _stream()), "bolt_b2b_gemm")
    return D1


def b2b_conv(c0: ConvDesc, c1: ConvDesc, x, w0, b0, w1, b1, y, config=None):
    c = _cfg(config)
    _check(_lib.bolt_b2b_conv(C.byref(c0), C.byref(c1), _ptr(x), _ptr(w0), _ptr(b0), _ptr(w1), _ptr(b1), _ptr(y),
                              None if c is None else C.byref(c), None, 0, _stream()), "bolt_b2b_conv")
    return y


def b2b_gemm_residual(g0: GemmDesc, g1: GemmDesc, A0, W0, b0, W1, b1, Cres, D1, gamma: float = 1.0, config=None):
    """D1 = act1(alpha1 D0.W1 + beta1 b1 + gamma Cres), D0 the first op's output; Cres is a contiguous M x N1 tensor."""
    c = _cfg(config)
    _check(_lib.bolt_b2b_gemm_residual(C.byref(g0), C.byref(g1), _ptr(A0), _ptr(W0), _ptr(b0), _ptr(W1), _ptr(b1),
                                       _ptr(Cres), Cres.shape[-1], gamma, _ptr(D1), None if c is None else C.byref(c),
                                       None, 0, _stream()), "bolt_b2b_gemm_residual")
    return D1


def b2b_conv_residual(c0: ConvDesc, c1: ConvDesc, x, w0, b0, w1, b1, residual, y, gamma: float = 1.0, config=None):
    c = _cfg(config)
    _check(_lib.bolt_b2b_conv_residual(C.byref(c0), C.byref(c1), _ptr(x), _ptr(w0), _ptr(b0), _ptr(w1), _ptr(b1),
                                       _ptr(residual), gamma, _ptr(y), None if c is None else C.byref(c), None, 0,
                                       _stream()), "bolt_b2b_conv_residual")
    return y


@dataclass
class TuneResult:
    config: BoltConfig
    ms: float
    tried: int


def tune(op: int, desc0, desc1, tensors: Sequence, workspace=None) -> TuneResult:
    """tensors: the op call's device tensors in call order (None allowed for a bias)."""
    ptrs = (_vp * len(tensors))(*[_ptr(t) for t in tensors])
    best, ms, tried = BoltConfig(), C.c_float(0), _i32(0)
    wp, wb = _ws(workspace)
    _check(_lib.bolt_tune(op, C.addressof(desc0), None if desc1 is None else C.addressof(desc1), ptrs, wp, wb,
                          _stream(), C.byref(best), C.byref(ms), C.byref(tried)), "bolt_tune")
    return TuneResult(best, float(ms.value), int(tried.value))


def _desc_array(descs):
    return (_vp * len(descs))(*[C.addressof(d) for d in descs])


def _ptr_array(tensors):
    return (_vp * len(tensors))(*[_ptr(t) for t in tensors])


def b2b_gemm_chain(descs, A0, weights, biases, D, config=None):
    """descs: GemmDesc list; weights / biases: lists of device tensors (a bias may be None)."""
    c = _cfg(config)
    _check(_lib.bolt_b2b_gemm_chain(len(descs), _desc_array(descs), _ptr(A0), _ptr_array(weights), _ptr_array(biases),
                                    _ptr(D), None if c is None else C.byref(c), _stream()), "bolt_b2b_gemm_chain")
    return D


def b2b_conv_chain(descs, x, weights, biases, y, config=None):
    c = _cfg(config)
    _check(_lib.bolt_b2b_conv_chain(len(descs), _desc_array(descs), _ptr(x), _ptr_array(weights), _ptr_array(biases),
                                    _ptr(y), None if c is None else C.byref(c), _stream()), "bolt_b2b_conv_chain")
    return y


def b2b_gemm_chain_residual(descs, A0, weights, biases, Cmat, D, gamma=1.0, ldc=None, config=None):
    """The chain with gamma * Cmat (M x N_2, row stride ldc) added in the last op's epilogue."""
    c = _cfg(config)
    _check(_lib.bolt_b2b_gemm_chain_residual(len(descs), _desc_array(descs), _ptr(A0), _ptr_array(weights),
                                             _ptr_array(biases), _ptr(Cmat), int(ldc if ldc is not None else descs[-1].N),
                                             C.c_float(gamma), _ptr(D), None if c is None else C.byref(c), _stream()),
           "bolt_b2b_gemm_chain_residual")
    return D


def b2b_conv_chain_residual(descs, x, weights, biases, residual, y, gamma=1.0, config=None):
    c = _cfg(config)
    _check(_lib.bolt_b2b_conv_chain_residual(len(descs), _desc_array(descs), _ptr(x), _ptr_array(weights),
                                             _ptr_array(biases), _ptr(residual), C.c_float(gamma), _ptr(y),
                                             None if c is None else C.byref(c), _stream()),
           "bolt_b2b_conv_chain_residual")
    return y


def tune_chain(op: int, descs, tensors) -> TuneResult:
    """tensors: [x, w0, b0, w1, b1, w2, b2, y] (biases may be None)."""
    best, ms, tried = BoltConfig(), C.c_float(0), _i32(0)
    _check(_lib.bolt_tune_chain(op, len(descs), _desc_array(descs), _ptr_array(tensors), _stream(), C.byref(best),
                                C.byref(ms), C.byref(tried)), "bolt_tune_chain")
    return TuneResult(best, float(ms.value), int(tried.value))


def check_chain(op: int, descs, config=None) -> int:
    c = _cfg(config)
    return int(_lib.bolt_check_chain(op, len(descs), _desc_array(descs) if descs else None,
                                     None if c is None else C.byref(c)))


def chain_instance_supports(op: int, kernel_id: int, descs) -> bool:
    return bool(_lib.bolt_chain_instance_supports(op, kernel_id, len(descs), _desc_array(descs)))


def pad_channels_nhwc(src, dst, C_padded: int):
    Cin = src.shape[-1]
    pixels = src.numel() // Cin
    _check(_lib.bolt_pad_channels_nhwc(_ptr(src), _ptr(dst), pixels, Cin, C_padded, _stream()),
           "bolt_pad_channels_nhwc")
    return dst


def nchw_to_nhwc(src, dst):
    """src [N][C][H][W] -> dst [N][H][W][C_padded] (dst's last extent; extra channels are zeroed)."""
    N, Cc, H, W = src.shape
    assert dst.shape[:3] == (N, H, W)
    _check(_lib.bolt_nchw_to_nhwc(_ptr(src), _ptr(dst), N, Cc, H, W, dst.shape[3], _stream()), "bolt_nchw_to_nhwc")
    return dst


def nhwc_to_nchw(src, dst):
    """src [N][H][W][C_src] -> dst [N][C][H][W] (the first C channels of src)."""
    N, Cc, H, W = dst.shape
    assert src.shape[:3] == (N, H, W)
    _check(_lib.bolt_nhwc_to_nchw(_ptr(src), _ptr(dst), N, Cc, H, W, src.shape[3], _stream()), "bolt_nhwc_to_nchw")
    return dst


def bias_act(D, bias=None, alpha: float = 1.0, beta: float = 1.0, act="relu"):
    """In place on a 2-D FP16 tensor (row stride = its stride(0)): D = act(alpha * D + beta * bias)."""
    M, N = D.shape
    a = ACT[act] if isinstance(act, str) else int(act)
    _check(_lib.bolt_bias_act(_ptr(D), _ptr(bias), M, N, D.stride(0) if M > 1 else N, alpha, beta, a, _stream()),
           "bolt_bias_act")
    return D


def probe_mfma_peak(iterations: int = 20000) -> float:
    out = C.c_float(0)
    _check(_lib.bolt_probe_mfma_peak(iterations, _stream(), C.byref(out)), "bolt_probe_mfma_peak")
    return float(out.value)


def probe_copy_bandwidth(buffer, repeats: int = 10) -> float:
    out = C.c_float(0)
    _check(_lib.bolt_probe_copy_bandwidth(buffer.data_ptr(), buffer.numel() * buffer.element_size(), repeats,
                                          _stream(), C.byref(out)), "bolt_probe_copy_bandwidth")
    return float(out.value)
