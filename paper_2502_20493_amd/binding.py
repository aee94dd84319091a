"""Thin ctypes binding of libukst: same names as include/ukst.h, argument marshalling only.

Every step of the computation runs in the HIP kernels behind the C ABI.  There is no CPU
fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libukst.so")
BENCH_LIB_PATH = os.path.join(_HERE, "libukst_bench.so")

UKST_F32, UKST_BF16_F32, UKST_BF16_BF16 = 0, 1, 2
(UKST_OK, UKST_ERR_NULL, UKST_ERR_SHAPE, UKST_ERR_DTYPE, UKST_ERR_UNSUPPORTED, UKST_ERR_LAUNCH,
 UKST_ERR_WORKSPACE) = range(7)
UKST_OP_FORWARD, UKST_OP_GRAD_INPUT, UKST_OP_GRAD_WEIGHT = 0, 1, 2
UKST_PATH_AUTO, UKST_PATH_DIRECT, UKST_PATH_MFMA = 0, 1, 2
UKST_MAX_N = 7
UKST_ACT_NONE, UKST_ACT_RELU, UKST_ACT_TANH = 0, 1, 2

# every symbol include/ukst.h declares
EXPORTS = ["ukst_version", "ukst_status_string", "ukst_output_shape", "ukst_mac_count",
           "ukst_select_path", "ukst_conv_transpose2d", "ukst_conv_transpose2d_path",
           "ukst_kernel_name", "ukst_conv_transpose2d_bias_act", "ukst_workspace_bytes",
           "ukst_conv_transpose2d_ws", "ukst_conv_transpose2d_grad_input",
           "ukst_conv_transpose2d_grad_weight", "ukst_grad_kernel_name",
           "ukst_conv_transpose2d_grad_weight_static", "ukst_static_workspace_bytes",
           "ukst_output_shape_strided", "ukst_output_shape_dilated",
           "ukst_conv_transpose2d_strided", "ukst_dilated_conv2d", "ukst_mac_count_strided",
           "ukst_mac_count_dilated"]
# every symbol include/ukst_bench.h declares (libukst_bench.so: measurement helpers)
BENCH_EXPORTS = ["ukst_bench_mfma_ceiling", "ukst_bench_stream_ceiling"]

_lib = None
_bench_lib = None


class UkstError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"ukst status {status}: {message}")
        self.status = status


def lib():
    """Load libukst.so (once).  Raises if it is missing: build it with
    ``python -m paper_2502_20493_amd.build`` (or ``__graft_entry__.build()``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: the HIP library has not been built "
                "(python -m paper_2502_20493_amd.build). There is no fallback path.")
        # PyTorch bundles its own HIP runtime.  It has to be in the process before this library
        # is loaded, otherwise the two ends see different runtimes and the first HIP call made
        # from here reports that there is no device.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        i, vp = ctypes.c_int, ctypes.c_void_p
        ip = ctypes.POINTER(ctypes.c_int)
        L.ukst_version.argtypes, L.ukst_version.restype = [], i
        L.ukst_status_string.argtypes, L.ukst_status_string.restype = [i], ctypes.c_char_p
        L.ukst_output_shape.argtypes, L.ukst_output_shape.restype = [i, i, i, i, ip, ip], i
        L.ukst_mac_count.argtypes = [i] * 8
        L.ukst_mac_count.restype = ctypes.c_ulonglong
        L.ukst_select_path.argtypes, L.ukst_select_path.restype = [i] * 8, i
        L.ukst_conv_transpose2d.argtypes = [vp, vp, vp] + [i] * 8 + [vp]
        L.ukst_conv_transpose2d.restype = i
        L.ukst_conv_transpose2d_path.argtypes = [vp, vp, vp] + [i] * 9 + [vp]
        L.ukst_conv_transpose2d_path.restype = i
        L.ukst_kernel_name.argtypes, L.ukst_kernel_name.restype = [i] * 9, ctypes.c_char_p
        L.ukst_conv_transpose2d_bias_act.argtypes = [vp, vp, vp, vp] + [i] * 10 + [vp]
        L.ukst_conv_transpose2d_bias_act.restype = i
        L.ukst_workspace_bytes.argtypes, L.ukst_workspace_bytes.restype = [i] * 9, ctypes.c_size_t
        L.ukst_conv_transpose2d_ws.argtypes = [vp, vp, vp, vp] + [i] * 10 + [vp, ctypes.c_size_t, vp]
        L.ukst_conv_transpose2d_ws.restype = i
        L.ukst_grad_kernel_name.argtypes, L.ukst_grad_kernel_name.restype = [i] * 9, ctypes.c_char_p
        for f in (L.ukst_conv_transpose2d_grad_input, L.ukst_conv_transpose2d_grad_weight):
            f.argtypes = [vp, vp, vp] + [i] * 8 + [vp, ctypes.c_size_t, vp]
            f.restype = i
        L.ukst_conv_transpose2d_grad_weight_static.argtypes = [vp, vp, vp] + [i] * 8 + [vp]
        L.ukst_conv_transpose2d_grad_weight_static.restype = i
        for f in (L.ukst_output_shape_strided, L.ukst_output_shape_dilated):
            f.argtypes, f.restype = [i] * 5 + [ip, ip], i
        for f in (L.ukst_conv_transpose2d_strided, L.ukst_dilated_conv2d):
            f.argtypes, f.restype = [vp, vp, vp] + [i] * 9 + [vp], i
        for f in (L.ukst_mac_count_strided, L.ukst_mac_count_dilated):
            f.argtypes, f.restype = [i] * 9, ctypes.c_ulonglong
        L.ukst_static_workspace_bytes.argtypes = []
        L.ukst_static_workspace_bytes.restype = ctypes.c_size_t
        _lib = L
    return _lib


def bench_lib():
    """Load libukst_bench.so (once): the measured ceilings of include/ukst_bench.h."""
    global _bench_lib
    if _bench_lib is None:
        if not os.path.exists(BENCH_LIB_PATH):
            raise RuntimeError(f"{BENCH_LIB_PATH} is missing: python -m paper_2502_20493_amd.build")
        import torch  # noqa: F401  (same load-order requirement as lib())
        L = ctypes.CDLL(BENCH_LIB_PATH)
        i, vp = ctypes.c_int, ctypes.c_void_p
        L.ukst_bench_mfma_ceiling.argtypes = [i, i, vp, vp]
        L.ukst_bench_mfma_ceiling.restype = ctypes.c_double
        L.ukst_bench_stream_ceiling.argtypes = [vp, ctypes.c_size_t, vp, ctypes.c_size_t, vp]
        L.ukst_bench_stream_ceiling.restype = i
        _bench_lib = L
    return _bench_lib


def _check(status: int):
    if status != UKST_OK:
        raise UkstError(status, ukst_status_string(status))


def ukst_version() -> int:
    return int(lib().ukst_version())


def ukst_status_string(status: int) -> str:
    return lib().ukst_status_string(int(status)).decode()


def ukst_output_shape(H: int, W: int, n: int, P: int):
    oh, ow = ctypes.c_int(0), ctypes.c_int(0)
    _check(lib().ukst_output_shape(H, W, n, P, ctypes.byref(oh), ctypes.byref(ow)))
    return oh.value, ow.value


def ukst_mac_count(B, Cin, Cout, H, W, n, P, kind: int) -> int:
    return int(lib().ukst_mac_count(B, Cin, Cout, H, W, n, P, kind))


def ukst_select_path(B, Cin, Cout, H, W, n, P, dtype) -> int:
    r = int(lib().ukst_select_path(B, Cin, Cout, H, W, n, P, dtype))
    if r < 0:
        _check(-r)
    return r


def ukst_kernel_name(B, Cin, Cout, H, W, n, P, dtype, path=UKST_PATH_AUTO) -> str:
    return lib().ukst_kernel_name(B, Cin, Cout, H, W, n, P, dtype, path).decode()


def ukst_bench_mfma_ceiling(dtype: int, iters: int, sink, stream=None) -> float:
    """Enqueue the register-resident MFMA loop; returns the FLOPs of that launch (0.0 on failure).
    sink: float32 device tensor with at least 64 elements."""
    import torch

    if not (sink.is_cuda and sink.dtype == torch.float32 and sink.numel() >= 64):
        raise ValueError("sink must be a float32 device tensor with at least 64 elements")
    if stream is None:
        stream = torch.cuda.current_stream(sink.device)
    return float(bench_lib().ukst_bench_mfma_ceiling(int(dtype), int(iters), sink.data_ptr(),
                                                     stream.cuda_stream))


def ukst_bench_stream_ceiling(src, dst, stream=None) -> None:
    """Enqueue the streaming kernel: reads all of src, writes all of dst (device tensors whose
    byte sizes are multiples of 16)."""
    import torch

    if stream is None:
        stream = torch.cuda.current_stream(src.device)
    rc = bench_lib().ukst_bench_stream_ceiling(src.data_ptr(), src.numel() * src.element_size(),
                                               dst.data_ptr(), dst.numel() * dst.element_size(),
                                               stream.cuda_stream)
    if rc != 0:
        raise RuntimeError("ukst_bench_stream_ceiling failed")


def ukst_workspace_bytes(op: int, B, Cin, Cout, H, W, n, P, dtype) -> int:
    return int(lib().ukst_workspace_bytes(int(op), B, Cin, Cout, H, W, n, P, dtype))


def _workspace(workspace, need: int, device, stream):
    """The (pointer, size) pair of a call.  workspace: None = allocate `need` bytes with torch for
    this call (torch supplies device memory; the library itself never allocates), False = pass
    none, or a caller-provided uint8 device tensor."""
    import torch

    if workspace is False or (workspace is None and need == 0):
        return None, 0, None
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=device)
        if hasattr(stream, "cuda_stream"):
            workspace.record_stream(stream)  # the block must outlive the work enqueued on `stream`
    if not (workspace.is_cuda and workspace.dtype == torch.uint8 and workspace.is_contiguous()):
        raise ValueError("workspace must be a contiguous uint8 device tensor")
    return workspace.data_ptr(), workspace.numel(), workspace


def ukst_conv_transpose2d_raw(x_ptr, w_ptr, y_ptr, B, Cin, Cout, H, W, n, P, dtype,
                              path=UKST_PATH_AUTO, stream_ptr=None) -> int:
    """Direct call with raw device addresses (ints or None).  Returns the status code."""
    return int(lib().ukst_conv_transpose2d_path(x_ptr, w_ptr, y_ptr, B, Cin, Cout, H, W, n, P,
                                                dtype, path, stream_ptr))


def ukst_conv_transpose2d_bias_act(x, w, P: int, bias=None, act: int = UKST_ACT_NONE, y=None,
                                   path: int = UKST_PATH_AUTO, stream=None, out_bf16: bool = False,
                                   workspace=False):
    """Marshal torch device tensors into ukst_conv_transpose2d_bias_act:
    y = act(conv_transpose(x, w) + bias[co]); bias: float32 device tensor [Cout] or None."""
    import torch

    if bias is not None:
        if not (bias.is_cuda and bias.dtype == torch.float32 and bias.is_contiguous()
                and tuple(bias.shape) == (w.shape[0],)):
            raise ValueError("bias must be a contiguous float32 device tensor [Cout]")
    return ukst_conv_transpose2d(x, w, P, y=y, path=path, stream=stream, out_bf16=out_bf16,
                                 workspace=workspace, _bias=bias, _act=act)


def ukst_conv_transpose2d_ws(x, w, P: int, bias=None, act: int = UKST_ACT_NONE, y=None,
                             path: int = UKST_PATH_AUTO, stream=None, out_bf16: bool = False,
                             workspace=None):
    """Marshal torch device tensors into ukst_conv_transpose2d_ws.  workspace: a uint8 device
    tensor of at least ukst_workspace_bytes(UKST_OP_FORWARD, ...) bytes, or None to have one
    allocated with torch for this call."""
    return ukst_conv_transpose2d_bias_act(x, w, P, bias=bias, act=act, y=y, path=path, stream=stream,
                                          out_bf16=out_bf16, workspace=workspace)


def ukst_conv_transpose2d(x, w, P: int, y=None, path: int = UKST_PATH_AUTO, stream=None,
                          out_bf16: bool = False, workspace=False, _bias=None, _act=None):
    """Marshal torch device tensors into ukst_conv_transpose2d (workspace=False, the default: the
    entry points that take no workspace) or ukst_conv_transpose2d_ws (workspace=None: allocated
    with torch for this call; or a uint8 device tensor).

    x: [B,Cin,H,W] float32 or bfloat16, w: [Cout,Cin,n,n] same dtype, both contiguous on the GPU.
    y: optional preallocated float32 [B,Cout,OH,OW]; allocated with torch when omitted.
    out_bf16 (bf16 inputs only), or a bfloat16 y: the output is bfloat16 (UKST_BF16_BF16).
    The call is asynchronous on ``stream`` (default: torch's current stream).
    """
    import torch

    if not (x.is_cuda and w.is_cuda):
        raise ValueError("x and w must be device tensors")
    if not (x.is_contiguous() and w.is_contiguous()):
        raise ValueError("x and w must be contiguous")
    if x.dtype != w.dtype or x.dtype not in (torch.float32, torch.bfloat16):
        raise ValueError("x and w must both be float32 or both bfloat16")
    if x.dim() != 4 or w.dim() != 4 or w.shape[2] != w.shape[3] or w.shape[1] != x.shape[1]:
        raise ValueError("expected x[B,Cin,H,W] and w[Cout,Cin,n,n]")
    B, Cin, H, W = x.shape
    Cout, _, n, _ = w.shape
    if y is not None and y.dtype == torch.bfloat16:
        out_bf16 = True
    if out_bf16 and x.dtype != torch.bfloat16:
        raise ValueError("a bfloat16 output needs bfloat16 inputs")
    dtype = UKST_F32 if x.dtype == torch.float32 else (UKST_BF16_BF16 if out_bf16 else UKST_BF16_F32)
    ydt = torch.bfloat16 if out_bf16 else torch.float32
    OH, OW = ukst_output_shape(H, W, n, P)
    if y is None:
        y = torch.empty((B, Cout, OH, OW), dtype=ydt, device=x.device)
    elif (tuple(y.shape) != (B, Cout, OH, OW) or y.dtype != ydt
          or not y.is_contiguous() or not y.is_cuda):
        raise ValueError("y must be a contiguous device tensor [B,Cout,OH,OW], float32 or, for a "
                         "bfloat16 output, bfloat16")
    if stream is None:
        stream = torch.cuda.current_stream(x.device)
    sp = stream.cuda_stream if hasattr(stream, "cuda_stream") else stream
    with torch.cuda.device(x.device):
        if workspace is not False:
            need = ukst_workspace_bytes(UKST_OP_FORWARD, B, Cin, Cout, H, W, n, P, dtype)
            wp, wb, _keep = _workspace(workspace, need, x.device, stream)
            _check(int(lib().ukst_conv_transpose2d_ws(
                x.data_ptr(), w.data_ptr(), None if _bias is None else _bias.data_ptr(),
                y.data_ptr(), B, Cin, Cout, H, W, n, P, dtype,
                UKST_ACT_NONE if _act is None else int(_act), path, wp, wb, sp)))
        elif _act is None:
            _check(ukst_conv_transpose2d_raw(x.data_ptr(), w.data_ptr(), y.data_ptr(), B, Cin, Cout,
                                             H, W, n, P, dtype, path, sp))
        else:
            _check(int(lib().ukst_conv_transpose2d_bias_act(
                x.data_ptr(), w.data_ptr(), None if _bias is None else _bias.data_ptr(),
                y.data_ptr(), B, Cin, Cout, H, W, n, P, dtype, int(_act), path, sp)))
    return y


def ukst_grad_kernel_name(which: int, B, Cin, Cout, H, W, n, P, dtype) -> str:
    return lib().ukst_grad_kernel_name(int(which), B, Cin, Cout, H, W, n, P, dtype).decode()


def _backward_operands(p0, p1):
    import torch

    if not (p0.is_cuda and p1.is_cuda and p0.is_contiguous() and p1.is_contiguous()):
        raise ValueError("operands must be contiguous device tensors")
    if p0.dtype != p1.dtype or p0.dtype not in (torch.float32, torch.bfloat16):
        raise ValueError("operands must both be float32 or both bfloat16")
    if p0.dim() != 4 or p1.dim() != 4:
        raise ValueError("operands must be 4-D")
    return UKST_F32 if p0.dtype == torch.float32 else UKST_BF16_F32


def _out(t, shape, device):
    import torch

    if t is None:
        return torch.empty(shape, dtype=torch.float32, device=device)
    if tuple(t.shape) != tuple(shape) or t.dtype != torch.float32 or not t.is_contiguous() or not t.is_cuda:
        raise ValueError(f"output must be a contiguous float32 device tensor {tuple(shape)}")
    return t


def ukst_conv_transpose2d_grad_input(dy, w, H: int, W: int, P: int, dx=None, stream=None,
                                     workspace=None):
    """Marshal torch device tensors into ukst_conv_transpose2d_grad_input.
    dy: [B,Cout,OH,OW], w: [Cout,Cin,n,n] (float32 or bfloat16) -> dx float32 [B,Cin,H,W].
    workspace: uint8 device tensor (>= ukst_workspace_bytes(UKST_OP_GRAD_INPUT, ...)), or None to
    have it allocated with torch for this call."""
    import torch

    dtype = _backward_operands(dy, w)
    B, Cout = dy.shape[:2]
    Cout2, Cin, n, n2 = w.shape
    if Cout2 != Cout or n != n2 or tuple(dy.shape[2:]) != ukst_output_shape(H, W, n, P):
        raise ValueError("expected dy[B,Cout,2H+2P-n,2W+2P-n] and w[Cout,Cin,n,n]")
    dx = _out(dx, (B, Cin, H, W), dy.device)
    if stream is None:
        stream = torch.cuda.current_stream(dy.device)
    sp = stream.cuda_stream if hasattr(stream, "cuda_stream") else stream
    with torch.cuda.device(dy.device):
        need = ukst_workspace_bytes(UKST_OP_GRAD_INPUT, B, Cin, Cout, H, W, n, P, dtype)
        wp, wb, _keep = _workspace(workspace, need, dy.device, stream)
        _check(int(lib().ukst_conv_transpose2d_grad_input(dy.data_ptr(), w.data_ptr(), dx.data_ptr(),
                                                          B, Cin, Cout, H, W, n, P, dtype, wp, wb, sp)))
    return dx


def ukst_static_workspace_bytes() -> int:
    return int(lib().ukst_static_workspace_bytes())


def ukst_conv_transpose2d_grad_weight_static(x, dy, n: int, P: int, dw, stream=None):
    """Marshal torch device tensors into ukst_conv_transpose2d_grad_weight_static (the partial sums
    live in the library's static device array; dw must be preallocated: nothing is allocated)."""
    import torch

    dtype = _backward_operands(x, dy)
    B, Cin, H, W = x.shape
    B2, Cout = dy.shape[:2]
    if B2 != B or tuple(dy.shape[2:]) != ukst_output_shape(H, W, n, P):
        raise ValueError("expected x[B,Cin,H,W] and dy[B,Cout,2H+2P-n,2W+2P-n]")
    dw = _out(dw, (Cout, Cin, n, n), x.device)
    if stream is None:
        stream = torch.cuda.current_stream(x.device)
    sp = stream.cuda_stream if hasattr(stream, "cuda_stream") else stream
    with torch.cuda.device(x.device):
        _check(int(lib().ukst_conv_transpose2d_grad_weight_static(
            x.data_ptr(), dy.data_ptr(), dw.data_ptr(), B, Cin, Cout, H, W, n, P, dtype, sp)))
    return dw


def ukst_conv_transpose2d_grad_weight(x, dy, n: int, P: int, dw=None, stream=None, workspace=None):
    """Marshal torch device tensors into ukst_conv_transpose2d_grad_weight.
    x: [B,Cin,H,W], dy: [B,Cout,OH,OW] (float32 or bfloat16) -> dw float32 [Cout,Cin,n,n].
    workspace: uint8 device tensor (>= ukst_workspace_bytes(UKST_OP_GRAD_WEIGHT, ...)), or None to
    have it allocated with torch for this call."""
    import torch

    dtype = _backward_operands(x, dy)
    B, Cin, H, W = x.shape
    B2, Cout = dy.shape[:2]
    if B2 != B or tuple(dy.shape[2:]) != ukst_output_shape(H, W, n, P):
        raise ValueError("expected x[B,Cin,H,W] and dy[B,Cout,2H+2P-n,2W+2P-n]")
    dw = _out(dw, (Cout, Cin, n, n), x.device)
    if stream is None:
        stream = torch.cuda.current_stream(x.device)
    sp = stream.cuda_stream if hasattr(stream, "cuda_stream") else stream
    with torch.cuda.device(x.device):
        need = ukst_workspace_bytes(UKST_OP_GRAD_WEIGHT, B, Cin, Cout, H, W, n, P, dtype)
        wp, wb, _keep = _workspace(workspace, need, x.device, stream)
        _check(int(lib().ukst_conv_transpose2d_grad_weight(x.data_ptr(), dy.data_ptr(), dw.data_ptr(),
                                                           B, Cin, Cout, H, W, n, P, dtype, wp, wb, sp)))
    return dw


def ukst_output_shape_strided(H: int, W: int, n: int, P: int, s: int):
    oh, ow = ctypes.c_int(0), ctypes.c_int(0)
    _check(lib().ukst_output_shape_strided(H, W, n, P, s, ctypes.byref(oh), ctypes.byref(ow)))
    return oh.value, ow.value


def ukst_output_shape_dilated(H: int, W: int, n: int, P: int, d: int):
    oh, ow = ctypes.c_int(0), ctypes.c_int(0)
    _check(lib().ukst_output_shape_dilated(H, W, n, P, d, ctypes.byref(oh), ctypes.byref(ow)))
    return oh.value, ow.value


def ukst_mac_count_strided(B, Cin, Cout, H, W, n, P, s, kind: int) -> int:
    return int(lib().ukst_mac_count_strided(B, Cin, Cout, H, W, n, P, s, kind))


def ukst_mac_count_dilated(B, Cin, Cout, H, W, n, P, d, kind: int) -> int:
    return int(lib().ukst_mac_count_dilated(B, Cin, Cout, H, W, n, P, d, kind))


def _general(fn, shape_fn, x, w, P, k, y, stream):
    import torch

    if not (x.is_cuda and w.is_cuda and x.is_contiguous() and w.is_contiguous()):
        raise ValueError("x and w must be contiguous device tensors")
    if x.dtype != w.dtype or x.dtype not in (torch.float32, torch.bfloat16):
        raise ValueError("x and w must both be float32 or both bfloat16")
    if x.dim() != 4 or w.dim() != 4 or w.shape[2] != w.shape[3] or w.shape[1] != x.shape[1]:
        raise ValueError("expected x[B,Cin,H,W] and w[Cout,Cin,n,n]")
    B, Cin, H, W = x.shape
    Cout, _, n, _ = w.shape
    OH, OW = shape_fn(H, W, n, P, k)
    y = _out(y, (B, Cout, OH, OW), x.device)
    if stream is None:
        stream = torch.cuda.current_stream(x.device)
    sp = stream.cuda_stream if hasattr(stream, "cuda_stream") else stream
    dtype = UKST_F32 if x.dtype == torch.float32 else UKST_BF16_F32
    with torch.cuda.device(x.device):
        _check(int(fn(x.data_ptr(), w.data_ptr(), y.data_ptr(), B, Cin, Cout, H, W, n, P, k, dtype, sp)))
    return y


def ukst_conv_transpose2d_strided(x, w, P: int, s: int, y=None, stream=None):
    """Marshal torch device tensors into ukst_conv_transpose2d_strided (stride-s transpose
    convolution; float32 output [B,Cout,s(H-1)+2P-n+2,s(W-1)+2P-n+2])."""
    return _general(lib().ukst_conv_transpose2d_strided, ukst_output_shape_strided, x, w, P, s, y, stream)


def ukst_dilated_conv2d(x, w, P: int, d: int, y=None, stream=None):
    """Marshal torch device tensors into ukst_dilated_conv2d (dilation-d convolution; float32
    output [B,Cout,H+2P-d(n-1),W+2P-d(n-1)])."""
    return _general(lib().ukst_dilated_conv2d, ukst_output_shape_dilated, x, w, P, d, y, stream)
