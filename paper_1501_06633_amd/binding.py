"""Thin ctypes binding of ``libmdnn.so``: same names as ``include/mdnn.h``,
argument marshalling only.  PyTorch appears here for device pointers and the
current stream, nothing else; every step of the convolution runs in the HIP
kernels.  A missing library raises -- there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmdnn.so")

MDNN_OK, MDNN_EINVAL, MDNN_ENULL, MDNN_EALIGN, MDNN_ETOOBIG, MDNN_ELAUNCH = range(6)

_lib = None


class MdnnError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: mdnn status {status} ({status_string(status)})")
        self.status = status


def lib() -> ctypes.CDLL:
    """Open libmdnn.so (built by ``__graft_entry__.build()`` / ``build.build_lib()``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_1501_06633_amd.build` "
            "(there is no CPU fallback)")
    L = ctypes.CDLL(LIB_PATH)
    i, f, p, s = ctypes.c_int, ctypes.c_float, ctypes.c_void_p, ctypes.c_char_p
    L.mdnn_conv_fprop.argtypes = [p, p, p, i, i, i, i, i, i, i, i, f, p]
    L.mdnn_conv_fprop.restype = i
    L.mdnn_conv_fprop_variant.argtypes = [p, p, p, i, i, i, i, i, i, i, i, f, p, s]
    L.mdnn_conv_fprop_variant.restype = i
    L.mdnn_out_dims.argtypes = [i, i, i, i, i, ctypes.POINTER(i), ctypes.POINTER(i)]
    L.mdnn_out_dims.restype = i
    L.mdnn_conv_flops.argtypes = [i] * 6
    L.mdnn_conv_flops.restype = ctypes.c_uint64
    L.mdnn_status_string.argtypes = [i]
    L.mdnn_status_string.restype = s
    L.mdnn_variant_count.argtypes = []
    L.mdnn_variant_count.restype = i
    L.mdnn_variant_name.argtypes = [i]
    L.mdnn_variant_name.restype = s
    L.mdnn_choose_variant.argtypes = [i] * 8
    L.mdnn_choose_variant.restype = s
    L.mdnn_describe_launch.argtypes = [i] * 8 + [s, ctypes.c_char_p, ctypes.c_size_t]
    L.mdnn_describe_launch.restype = i
    L.mdnn_conv_bprop_data_workspace.argtypes = [i] * 8 + [ctypes.POINTER(ctypes.c_size_t)]
    L.mdnn_conv_bprop_data_workspace.restype = i
    L.mdnn_conv_bprop_data.argtypes = [p, p, p, p, ctypes.c_size_t, i, i, i, i, i, i, i, i, f, p]
    L.mdnn_conv_bprop_data.restype = i
    L.mdnn_conv_bprop_data_static.argtypes = [p, p, p, i, i, i, i, i, i, i, i, f, p]
    L.mdnn_conv_bprop_data_static.restype = i
    L.mdnn_conv_bprop_filter_workspace.argtypes = [i] * 8 + [ctypes.POINTER(ctypes.c_size_t)]
    L.mdnn_conv_bprop_filter_workspace.restype = i
    L.mdnn_conv_bprop_filter.argtypes = [p, p, p, p, ctypes.c_size_t, i, i, i, i, i, i, i, i, f, p]
    L.mdnn_conv_bprop_filter.restype = i
    L.mdnn_sgemm_tn.argtypes = [p, p, p, i, i, i, f, p]
    L.mdnn_sgemm_tn.restype = i
    L.mdnn_mfma_peak_probe.argtypes = [p, i, i, i, ctypes.POINTER(ctypes.c_uint64), p]
    L.mdnn_mfma_peak_probe.restype = i
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().mdnn_status_string(int(status)).decode()


def mdnn_out_dims(Wi, Hi, Sk, stride, pad):
    """-> (status, Wo, Ho)"""
    wo, ho = ctypes.c_int(0), ctypes.c_int(0)
    st = lib().mdnn_out_dims(Wi, Hi, Sk, stride, pad, ctypes.byref(wo), ctypes.byref(ho))
    return st, wo.value, ho.value


def mdnn_conv_flops(Nb, Wo, Ho, Nc, No, Sk) -> int:
    return int(lib().mdnn_conv_flops(Nb, Wo, Ho, Nc, No, Sk))


def mdnn_variant_names():
    L = lib()
    return [L.mdnn_variant_name(k).decode() for k in range(L.mdnn_variant_count())]


def mdnn_choose_variant(Nb, Wi, Hi, Nc, No, Sk, stride, pad):
    r = lib().mdnn_choose_variant(Nb, Wi, Hi, Nc, No, Sk, stride, pad)
    return r.decode() if r else None


def mdnn_describe_launch(Nb, Wi, Hi, Nc, No, Sk, stride, pad, variant=None) -> dict:
    """Launch plan as a dict (variant, tiles, whole, split, pieces, grid, lds_bytes, ...)."""
    buf = ctypes.create_string_buffer(512)
    st = lib().mdnn_describe_launch(Nb, Wi, Hi, Nc, No, Sk, stride, pad,
                                    variant.encode() if variant else None, buf, len(buf))
    if st != MDNN_OK:
        raise MdnnError(st, "mdnn_describe_launch")
    out = {}
    for item in buf.value.decode().split():
        k, v = item.split("=", 1)
        out[k] = int(v) if v.lstrip("-").isdigit() else v
    return out


def mdnn_conv_fprop_raw(in_ptr, filt_ptr, out_ptr, Nb, Wi, Hi, Nc, No, Sk, stride, pad, alpha,
                        stream_ptr=None, variant=None) -> int:
    """Raw pointer form (ints or None); returns the status code, raises nothing."""
    L = lib()
    if variant is None:
        return L.mdnn_conv_fprop(in_ptr, filt_ptr, out_ptr, Nb, Wi, Hi, Nc, No, Sk, stride, pad,
                                 float(alpha), stream_ptr)
    return L.mdnn_conv_fprop_variant(in_ptr, filt_ptr, out_ptr, Nb, Wi, Hi, Nc, No, Sk, stride, pad,
                                     float(alpha), stream_ptr, variant.encode())


def mdnn_conv_fprop(inp, filt, stride, pad, alpha=1.0, out=None, variant=None, stream=None):
    """inp (Nc,Hi,Wi,Nb), filt (Nc,Sk,Sk,No): contiguous fp32 CUDA(HIP) tensors.
    Returns out (No,Ho,Wo,Nb), enqueued on ``stream`` (default: torch's current
    stream); the caller synchronises."""
    import torch

    if not (inp.is_cuda and filt.is_cuda):
        raise ValueError("mdnn_conv_fprop needs device tensors (no CPU path exists)")
    if inp.dtype != torch.float32 or filt.dtype != torch.float32:
        raise ValueError("fp32 only")
    if not (inp.is_contiguous() and filt.is_contiguous()):
        raise ValueError("tensors must be contiguous")
    Nc, Hi, Wi, Nb = inp.shape
    Nc2, Sk, Sk2, No = filt.shape
    if Nc2 != Nc or Sk2 != Sk:
        raise ValueError("filter shape does not match input")
    st, Wo, Ho = mdnn_out_dims(Wi, Hi, Sk, stride, pad)
    if st != MDNN_OK:
        raise MdnnError(st, "mdnn_out_dims")
    if out is None:
        out = torch.empty((No, Ho, Wo, Nb), dtype=torch.float32, device=inp.device)
    elif tuple(out.shape) != (No, Ho, Wo, Nb) or out.dtype != torch.float32 or not out.is_contiguous():
        raise ValueError("out has the wrong shape / dtype / layout")
    if stream is None:
        stream = torch.cuda.current_stream(inp.device)
    st = mdnn_conv_fprop_raw(inp.data_ptr(), filt.data_ptr(), out.data_ptr(),
                             Nb, Wi, Hi, Nc, No, Sk, stride, pad, alpha,
                             stream.cuda_stream or None, variant)
    if st != MDNN_OK:
        raise MdnnError(st, "mdnn_conv_fprop")
    return out


def mdnn_sgemm_tn(a, b, alpha=1.0, c=None, stream=None):
    """a (K,N), b (K,M): contiguous fp32 device tensors.  Returns c (N,M) = alpha * a^T b,
    enqueued on ``stream`` (default: torch's current stream); the caller synchronises."""
    import torch

    if not (a.is_cuda and b.is_cuda):
        raise ValueError("mdnn_sgemm_tn needs device tensors (no CPU path exists)")
    if a.dtype != torch.float32 or b.dtype != torch.float32:
        raise ValueError("fp32 only")
    if not (a.is_contiguous() and b.is_contiguous()) or a.dim() != 2 or b.dim() != 2:
        raise ValueError("operands must be contiguous matrices")
    K, N = a.shape
    K2, M = b.shape
    if K2 != K:
        raise ValueError("a and b must have the same number of rows")
    if c is None:
        c = torch.empty((N, M), dtype=torch.float32, device=a.device)
    elif tuple(c.shape) != (N, M) or c.dtype != torch.float32 or not c.is_contiguous():
        raise ValueError("c has the wrong shape / dtype / layout")
    if stream is None:
        stream = torch.cuda.current_stream(a.device)
    st = lib().mdnn_sgemm_tn(a.data_ptr(), b.data_ptr(), c.data_ptr(), N, M, K, alpha,
                             stream.cuda_stream or None)
    if st != MDNN_OK:
        raise MdnnError(st, "mdnn_sgemm_tn")
    return c


def mdnn_conv_bprop_data_workspace(Nb, Wi, Hi, Nc, No, Sk, stride, pad):
    """-> (status, bytes)"""
    n = ctypes.c_size_t(0)
    st = lib().mdnn_conv_bprop_data_workspace(Nb, Wi, Hi, Nc, No, Sk, stride, pad, ctypes.byref(n))
    return st, int(n.value)


def mdnn_conv_bprop_data(dout, filt, in_hw, stride, pad, alpha=1.0, din=None, workspace=None, stream=None):
    """dout (No,Ho,Wo,Nb), filt (Nc,Sk,Sk,No): contiguous fp32 device tensors; in_hw = (Hi, Wi)
    of the forward input.  Returns din (Nc,Hi,Wi,Nb) enqueued on ``stream``.  ``workspace`` is a
    uint8/float device tensor of at least mdnn_conv_bprop_data_workspace() bytes; one is allocated
    with torch if none is given (allocation is the binding's, the library itself never allocates)."""
    import torch

    if not (dout.is_cuda and filt.is_cuda):
        raise ValueError("mdnn_conv_bprop_data needs device tensors (no CPU path exists)")
    if dout.dtype != torch.float32 or filt.dtype != torch.float32:
        raise ValueError("fp32 only")
    if not (dout.is_contiguous() and filt.is_contiguous()):
        raise ValueError("tensors must be contiguous")
    No, Ho, Wo, Nb = dout.shape
    Nc, Sk, Sk2, No2 = filt.shape
    Hi, Wi = in_hw
    if No2 != No or Sk2 != Sk:
        raise ValueError("filter shape does not match dout")
    st, wo, ho = mdnn_out_dims(Wi, Hi, Sk, stride, pad)
    if st != MDNN_OK:
        raise MdnnError(st, "mdnn_out_dims")
    if (wo, ho) != (Wo, Ho):
        raise ValueError("dout spatial size does not match the forward geometry")
    st, need = mdnn_conv_bprop_data_workspace(Nb, Wi, Hi, Nc, No, Sk, stride, pad)
    if st != MDNN_OK:
        raise MdnnError(st, "mdnn_conv_bprop_data_workspace")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dout.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    if din is None:
        din = torch.empty((Nc, Hi, Wi, Nb), dtype=torch.float32, device=dout.device)
    elif tuple(din.shape) != (Nc, Hi, Wi, Nb) or din.dtype != torch.float32 or not din.is_contiguous():
        raise ValueError("din has the wrong shape / dtype / layout")
    if stream is None:
        stream = torch.cuda.current_stream(dout.device)
    st = lib().mdnn_conv_bprop_data(dout.data_ptr(), filt.data_ptr(), din.data_ptr(),
                                    workspace.data_ptr(), ws_bytes, Nb, Wi, Hi, Nc, No, Sk, stride, pad,
                                    float(alpha), stream.cuda_stream or None)
    if st != MDNN_OK:
        raise MdnnError(st, "mdnn_conv_bprop_data")
    return din


MDNN_STATIC_SCRATCH_BYTES = 40 << 20


def mdnn_conv_bprop_data_static(dout, filt, in_hw, stride, pad, alpha, din, stream=None):
    """mdnn_conv_bprop_data over the library's static device array instead of a workspace: the
    caller passes the result tensor ``din`` (Nc,Hi,Wi,Nb) too, so nothing is allocated anywhere."""
    import torch

    if not (dout.is_cuda and filt.is_cuda and din.is_cuda):
        raise ValueError("mdnn_conv_bprop_data_static needs device tensors (no CPU path exists)")
    if dout.dtype != torch.float32 or filt.dtype != torch.float32 or din.dtype != torch.float32:
        raise ValueError("fp32 only")
    if not (dout.is_contiguous() and filt.is_contiguous() and din.is_contiguous()):
        raise ValueError("tensors must be contiguous")
    No, Ho, Wo, Nb = dout.shape
    Nc, Sk, Sk2, No2 = filt.shape
    Hi, Wi = in_hw
    if No2 != No or Sk2 != Sk or tuple(din.shape) != (Nc, Hi, Wi, Nb):
        raise ValueError("tensor shapes do not match")
    st, wo, ho = mdnn_out_dims(Wi, Hi, Sk, stride, pad)
    if st != MDNN_OK:
        raise MdnnError(st, "mdnn_out_dims")
    if (wo, ho) != (Wo, Ho):
        raise ValueError("dout spatial size does not match the forward geometry")
    if stream is None:
        stream = torch.cuda.current_stream(dout.device)
    st = lib().mdnn_conv_bprop_data_static(dout.data_ptr(), filt.data_ptr(), din.data_ptr(),
                                           Nb, Wi, Hi, Nc, No, Sk, stride, pad, float(alpha),
                                           stream.cuda_stream or None)
    if st != MDNN_OK:
        raise MdnnError(st, "mdnn_conv_bprop_data_static")
    return din


def mdnn_conv_bprop_filter_workspace(Nb, Wi, Hi, Nc, No, Sk, stride, pad):
    """-> (status, bytes)"""
    n = ctypes.c_size_t(0)
    st = lib().mdnn_conv_bprop_filter_workspace(Nb, Wi, Hi, Nc, No, Sk, stride, pad, ctypes.byref(n))
    return st, int(n.value)


def mdnn_conv_bprop_filter(inp, dout, Sk, stride, pad, alpha=1.0, dfilt=None, workspace=None, stream=None):
    """inp (Nc,Hi,Wi,Nb), dout (No,Ho,Wo,Nb): contiguous fp32 device tensors.  Returns dfilt
    (Nc,Sk,Sk,No) enqueued on ``stream``.  ``workspace`` is a device tensor of at least
    mdnn_conv_bprop_filter_workspace() bytes; one is allocated with torch if none is given
    (allocation is the binding's, the library itself never allocates)."""
    import torch

    if not (inp.is_cuda and dout.is_cuda):
        raise ValueError("mdnn_conv_bprop_filter needs device tensors (no CPU path exists)")
    if inp.dtype != torch.float32 or dout.dtype != torch.float32:
        raise ValueError("fp32 only")
    if not (inp.is_contiguous() and dout.is_contiguous()):
        raise ValueError("tensors must be contiguous")
    Nc, Hi, Wi, Nb = inp.shape
    No, Ho, Wo, Nb2 = dout.shape
    if Nb2 != Nb:
        raise ValueError("batch sizes differ")
    st, wo, ho = mdnn_out_dims(Wi, Hi, Sk, stride, pad)
    if st != MDNN_OK:
        raise MdnnError(st, "mdnn_out_dims")
    if (wo, ho) != (Wo, Ho):
        raise ValueError("dout spatial size does not match the forward geometry")
    st, need = mdnn_conv_bprop_filter_workspace(Nb, Wi, Hi, Nc, No, Sk, stride, pad)
    if st != MDNN_OK:
        raise MdnnError(st, "mdnn_conv_bprop_filter_workspace")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=inp.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    if dfilt is None:
        dfilt = torch.empty((Nc, Sk, Sk, No), dtype=torch.float32, device=inp.device)
    elif tuple(dfilt.shape) != (Nc, Sk, Sk, No) or dfilt.dtype != torch.float32 or not dfilt.is_contiguous():
        raise ValueError("dfilt has the wrong shape / dtype / layout")
    if stream is None:
        stream = torch.cuda.current_stream(inp.device)
    st = lib().mdnn_conv_bprop_filter(inp.data_ptr(), dout.data_ptr(), dfilt.data_ptr(),
                                      workspace.data_ptr(), ws_bytes, Nb, Wi, Hi, Nc, No, Sk, stride, pad,
                                      float(alpha), stream.cuda_stream or None)
    if st != MDNN_OK:
        raise MdnnError(st, "mdnn_conv_bprop_filter")
    return dfilt


def mdnn_mfma_peak_probe(sink, blocks, waves_per_block, iters, stream=None) -> int:
    """Enqueue the register-only MFMA loop; returns the FLOPs one launch performs."""
    import torch

    need = blocks * waves_per_block * 64
    if sink.numel() < need or sink.dtype != torch.float32 or not sink.is_cuda:
        raise ValueError(f"sink must be a CUDA fp32 tensor with at least {need} elements")
    if stream is None:
        stream = torch.cuda.current_stream(sink.device)
    fl = ctypes.c_uint64(0)
    st = lib().mdnn_mfma_peak_probe(sink.data_ptr(), blocks, waves_per_block, iters,
                                    ctypes.byref(fl), stream.cuda_stream or None)
    if st != MDNN_OK:
        raise MdnnError(st, "mdnn_mfma_peak_probe")
    return int(fl.value)
