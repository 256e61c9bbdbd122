"""Thin ctypes binding of libsquant_hip.so: argument marshalling only.

Every step of the solver runs in the HIP kernels; torch is used for device
memory and streams.  There is no CPU fallback: a missing library is an error.
"""
from __future__ import annotations

import ctypes
import os
from typing import Iterable, List, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsquant_hip.so")

MODE_E, MODE_EK, MODE_EKC, MODE_EC = 0, 1, 2, 3
MODES = {"E": MODE_E, "EK": MODE_EK, "EKC": MODE_EKC, "EC": MODE_EC}
OUT_INT8, OUT_INT4, OUT_F32, OUT_BF16 = 0, 1, 2, 3
OUTPUTS = {"int8": OUT_INT8, "int4": OUT_INT4, "f32": OUT_F32, "bf16": OUT_BF16}
W_F32, W_F16, W_BF16 = 0, 1, 2
_WTYPES = {torch.float32: W_F32, torch.float16: W_F16, torch.bfloat16: W_BF16}


class squant_tensor_t(ctypes.Structure):
    _fields_ = [("w", ctypes.c_void_p), ("codes", ctypes.c_void_p), ("scales", ctypes.c_void_p),
                ("cout", ctypes.c_int32), ("cin", ctypes.c_int32), ("kh", ctypes.c_int32),
                ("kw", ctypes.c_int32)]


class squant_bn_t(ctypes.Structure):
    _fields_ = [("gamma", ctypes.c_void_p), ("beta", ctypes.c_void_p), ("channels", ctypes.c_int32),
                ("relu", ctypes.c_int32)]


class squant_act_range_t(ctypes.Structure):
    _fields_ = [("lo", ctypes.c_float), ("hi", ctypes.c_float), ("scale", ctypes.c_float),
                ("zero_point", ctypes.c_int32)]


class squant_layer_t(ctypes.Structure):
    _fields_ = [("weight", squant_tensor_t), ("bn", squant_bn_t)]


class SQuantError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"squant status {status}: {text}")
        self.status = status


_lib = None


def lib():
    """Loads the in-tree HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; "
                "g.build()'); there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        i32, vp, sz = ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t
        L.squant_quantize.argtypes = [vp, i32, i32, i32, i32, i32, ctypes.c_int, vp, vp, vp]
        L.squant_quantize.restype = ctypes.c_int
        L.squant_batched_workspace_bytes.argtypes = [i32]
        L.squant_batched_workspace_bytes.restype = sz
        L.squant_quantize_batched.argtypes = [ctypes.POINTER(squant_tensor_t), i32, i32,
                                              ctypes.c_int, vp, sz, vp]
        L.squant_quantize_batched.restype = ctypes.c_int
        L.squant_output_bytes.argtypes = [i32, i32, i32, i32, ctypes.c_int]
        L.squant_output_bytes.restype = sz
        L.squant_quantize_ex.argtypes = [vp, ctypes.c_int, i32, i32, i32, i32, i32, ctypes.c_int,
                                         ctypes.c_int, vp, vp, vp]
        L.squant_quantize_ex.restype = ctypes.c_int
        L.squant_quantize_batched_ex.argtypes = [ctypes.POINTER(squant_tensor_t), i32, ctypes.c_int,
                                                 i32, ctypes.c_int, ctypes.c_int, vp, sz, vp]
        L.squant_quantize_batched_ex.restype = ctypes.c_int
        L.squant_activation_workspace_bytes.argtypes = [i32]
        L.squant_activation_workspace_bytes.restype = sz
        L.squant_activation_ranges.argtypes = [ctypes.POINTER(squant_bn_t), i32, ctypes.c_float, i32,
                                               vp, vp, sz, vp]
        L.squant_activation_ranges.restype = ctypes.c_int
        L.squant_network_workspace_bytes.argtypes = [i32]
        L.squant_network_workspace_bytes.restype = sz
        L.squant_quantize_network.argtypes = [ctypes.POINTER(squant_layer_t), i32, i32, ctypes.c_int,
                                              i32, ctypes.c_float, vp, vp, sz, vp]
        L.squant_quantize_network.restype = ctypes.c_int
        L.squant_max_channel_elems.argtypes = [i32, i32]
        L.squant_max_channel_elems.restype = ctypes.c_int64
        L.squant_status_string.argtypes = [ctypes.c_int]
        L.squant_status_string.restype = ctypes.c_char_p
        L.squant_version.restype = ctypes.c_int
        _lib = L
    return _lib


def squant_status_string(status: int) -> str:
    return lib().squant_status_string(status).decode()


def squant_version() -> int:
    return int(lib().squant_version())


def squant_max_channel_elems(kh: int, kw: int) -> int:
    return int(lib().squant_max_channel_elems(kh, kw))


def squant_output_bytes(cout: int, cin: int, kh: int, kw: int, output: int) -> int:
    return int(lib().squant_output_bytes(cout, cin, kh, kw, output))


def squant_batched_workspace_bytes(n_tensors: int) -> int:
    return int(lib().squant_batched_workspace_bytes(n_tensors))


def _check(rc: int):
    if rc != 0:
        raise SQuantError(rc, squant_status_string(rc))


def _shape4(w: torch.Tensor) -> Tuple[int, int, int, int]:
    if w.dim() == 2:
        return (w.shape[0], w.shape[1], 1, 1)
    if w.dim() == 4:
        return tuple(w.shape)  # type: ignore[return-value]
    raise ValueError("weight must be [cout, cin] or [cout, cin, kh, kw]")


def _stream_ptr(stream) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _ws_ptr(ws):
    return ws.data_ptr() if ws is not None else None


def _check_weight(w: torch.Tensor):
    if not (w.is_cuda and w.dtype == torch.float32 and w.is_contiguous()):
        raise ValueError("weight must be a contiguous float32 tensor in device memory")


def _wtype(w: torch.Tensor) -> int:
    if not (w.is_cuda and w.dtype in _WTYPES and w.is_contiguous()):
        raise ValueError("weight must be a contiguous float32, float16 or bfloat16 tensor in device memory")
    return _WTYPES[w.dtype]


def _new_output(shape, output: int, device) -> torch.Tensor:
    """An output buffer of the format's shape: int8 / float32 / bfloat16 like the weights, or uint8
    [cout, (cin*kh*kw + 1) // 2] for packed 4-bit codes."""
    if output == OUT_INT8:
        return torch.empty(shape, dtype=torch.int8, device=device)
    if output == OUT_F32:
        return torch.empty(shape, dtype=torch.float32, device=device)
    if output == OUT_BF16:
        return torch.empty(shape, dtype=torch.bfloat16, device=device)
    if output == OUT_INT4:
        n = 1
        for d in shape[1:]:
            n *= d
        return torch.empty((shape[0], (n + 1) // 2), dtype=torch.uint8, device=device)
    raise ValueError(f"unknown output format {output}")


def squant_quantize(w: torch.Tensor, bits: int, mode: int = MODE_EKC, codes: torch.Tensor = None,
                    scales: torch.Tensor = None, stream=None):
    """Quantize one weight tensor; returns (codes int8 like w, scales float32 [cout]).

    Asynchronous on `stream` (default: torch's current stream)."""
    _check_weight(w)
    cout, cin, kh, kw = _shape4(w)
    if codes is None:
        codes = torch.empty(w.shape, dtype=torch.int8, device=w.device)
    if scales is None:
        scales = torch.empty(cout, dtype=torch.float32, device=w.device)
    _check(lib().squant_quantize(w.data_ptr(), cout, cin, kh, kw, bits, mode, codes.data_ptr(),
                                 scales.data_ptr(), _stream_ptr(stream)))
    return codes, scales


def squant_quantize_ex(w: torch.Tensor, bits: int, mode: int = MODE_EKC, output: int = OUT_INT8,
                       out: torch.Tensor = None, scales: torch.Tensor = None, stream=None):
    """squant_quantize for float32 / float16 / bfloat16 weights with the output format chosen:
    returns (out, scales), out being int8 codes, packed 4-bit codes or dequantised float32."""
    wtype = _wtype(w)
    cout, cin, kh, kw = _shape4(w)
    if out is None:
        out = _new_output(w.shape, output, w.device)
    if scales is None:
        scales = torch.empty(cout, dtype=torch.float32, device=w.device)
    _check(lib().squant_quantize_ex(w.data_ptr(), wtype, cout, cin, kh, kw, bits, mode, output,
                                    out.data_ptr(), scales.data_ptr(), _stream_ptr(stream)))
    return out, scales


class BatchPlan:
    """Descriptor array + workspace + outputs of a batched call, built once and reusable."""

    def __init__(self, weights: Sequence[torch.Tensor], output: int = OUT_INT8):
        self.weights = list(weights)
        self.output = output
        self.wtype = _wtype(self.weights[0]) if self.weights else W_F32
        n = len(self.weights)
        dev = self.weights[0].device if n else torch.device("cuda")
        self.codes: List[torch.Tensor] = []
        self.scales: List[torch.Tensor] = []
        self.desc = (squant_tensor_t * max(n, 1))()
        for i, w in enumerate(self.weights):
            if _wtype(w) != self.wtype:
                raise ValueError("all weights of a batch must share one dtype")
            cout, cin, kh, kw = _shape4(w)
            c = _new_output(w.shape, output, dev)
            s = torch.empty(cout, dtype=torch.float32, device=dev)
            self.codes.append(c)
            self.scales.append(s)
            self.desc[i] = squant_tensor_t(w.data_ptr(), c.data_ptr(), s.data_ptr(), cout, cin, kh, kw)
        self.n = n
        self.ws_bytes = squant_batched_workspace_bytes(n)      # 0: the library needs none
        self.workspace = (torch.empty(self.ws_bytes, dtype=torch.uint8, device=dev)
                          if self.ws_bytes else None)

    def run(self, bits: int, mode: int = MODE_EKC, stream=None):
        _check(lib().squant_quantize_batched_ex(self.desc, self.n, self.wtype, bits, mode,
                                                self.output, _ws_ptr(self.workspace),
                                                self.ws_bytes, _stream_ptr(stream)))
        return self.codes, self.scales


def squant_quantize_batched(weights: Iterable[torch.Tensor], bits: int, mode: int = MODE_EKC,
                            stream=None):
    """Quantize a set of float32 weight tensors in one call; returns (list of codes, list of scales)."""
    ws = list(weights)
    for w in ws:
        _check_weight(w)
    plan = BatchPlan(ws)
    _check(lib().squant_quantize_batched(plan.desc, plan.n, bits, mode, _ws_ptr(plan.workspace),
                                         plan.ws_bytes, _stream_ptr(stream)))
    return plan.codes, plan.scales


def squant_quantize_batched_ex(weights: Iterable[torch.Tensor], bits: int, mode: int = MODE_EKC,
                               output: int = OUT_INT8, stream=None):
    """The batched call for float32 / float16 / bfloat16 weights and any output format."""
    plan = BatchPlan(list(weights), output)
    return plan.run(bits, mode, stream)


def _ranges_from(buf: torch.Tensor, n: int):
    """The device result array (n x {lo, hi, scale, zero_point}) as host tuples."""
    raw = buf.cpu().numpy().reshape(n, 4)
    import numpy as np
    return [(np.float32(r[0]), np.float32(r[1]), np.float32(r[2]), int(r[3:4].view(np.int32)[0]))
            for r in raw]


def squant_activation_ranges(bn_layers, n_sigma: float, bits: int, stream=None):
    """bn_layers: sequence of (gamma, beta, relu) with float32 device tensors; returns one
    (lo, hi, scale, zero_point) per layer (synchronises to read the result back)."""
    layers = list(bn_layers)
    n = len(layers)
    desc = (squant_bn_t * max(n, 1))()
    for i, (g, b, relu) in enumerate(layers):
        for t in (g, b):
            _check_weight(t)
        if g.numel() != b.numel():
            raise ValueError("gamma and beta differ in length")
        desc[i] = squant_bn_t(g.data_ptr(), b.data_ptr(), g.numel(), int(bool(relu)))
    dev = layers[0][0].device if n else torch.device("cuda")
    out = torch.zeros(max(n, 1) * 4, dtype=torch.float32, device=dev)
    ws_bytes = int(lib().squant_activation_workspace_bytes(n))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev) if ws_bytes else None
    _check(lib().squant_activation_ranges(desc, n, n_sigma, bits, out.data_ptr(), _ws_ptr(ws),
                                          ws_bytes, _stream_ptr(stream)))
    torch.cuda.synchronize()
    return _ranges_from(out, n)


def squant_quantize_network(layers, weight_bits: int, mode: int = MODE_EKC, act_bits: int = 8,
                            n_sigma: float = 6.0, stream=None):
    """layers: sequence of (weight, bn) with bn = None or (gamma, beta, relu).  Returns
    (codes list, scales list, ranges list with None where a layer has no batch norm)."""
    layers = list(layers)
    n = len(layers)
    dev = layers[0][0].device if n else torch.device("cuda")
    desc = (squant_layer_t * max(n, 1))()
    codes, scales = [], []
    for i, (w, bn) in enumerate(layers):
        _check_weight(w)
        cout, cin, kh, kw = _shape4(w)
        c = torch.empty(w.shape, dtype=torch.int8, device=dev)
        s = torch.empty(cout, dtype=torch.float32, device=dev)
        codes.append(c)
        scales.append(s)
        wt = squant_tensor_t(w.data_ptr(), c.data_ptr(), s.data_ptr(), cout, cin, kh, kw)
        if bn is None:
            desc[i] = squant_layer_t(wt, squant_bn_t(None, None, 0, 0))
        else:
            g, b, relu = bn
            _check_weight(g)
            _check_weight(b)
            desc[i] = squant_layer_t(wt, squant_bn_t(g.data_ptr(), b.data_ptr(), g.numel(), int(bool(relu))))
    out = torch.zeros(max(n, 1) * 4, dtype=torch.float32, device=dev)
    ws_bytes = int(lib().squant_network_workspace_bytes(n))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev) if ws_bytes else None
    _check(lib().squant_quantize_network(desc, n, weight_bits, mode, act_bits, n_sigma, out.data_ptr(),
                                         _ws_ptr(ws), ws_bytes, _stream_ptr(stream)))
    torch.cuda.synchronize()
    ranges = _ranges_from(out, n)
    return codes, scales, [r if layers[i][1] is not None else None for i, r in enumerate(ranges)]
