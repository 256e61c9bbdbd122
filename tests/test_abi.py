"""Host-side checks that need no GPU: the library loads, exports what the header declares,
and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2202_07471_amd", "libsquant_hip.so")
HEADER = os.path.join(ROOT, "include", "squant.h")


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(LIB):
        import __graft_entry__
        __graft_entry__.build()
    from paper_2202_07471_amd import binding
    return binding.lib()


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(squant_[a-z_0-9]+)\s*\(", src)))


def test_header_symbols_are_exported(L):
    names = declared_functions()
    assert {"squant_quantize", "squant_quantize_batched", "squant_batched_workspace_bytes",
            "squant_status_string", "squant_version"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_status_strings(L):
    seen = set()
    for s in range(0, 9):
        txt = L.squant_status_string(s).decode()
        assert txt and txt not in seen
        seen.add(txt)
    assert L.squant_status_string(99).decode() == "unknown status"
    assert L.squant_version() >= 100


def test_bad_arguments_are_rejected_on_the_host(L):
    p = ctypes.c_void_p(0x1000)   # never dereferenced: validation precedes any launch
    q = lambda *a: L.squant_quantize(*a)
    assert q(None, 4, 4, 3, 3, 4, 2, p, p, None) == 1
    assert q(p, 4, 4, 3, 3, 4, 2, None, p, None) == 1
    assert q(p, 4, 4, 3, 3, 4, 2, p, None, None) == 1
    assert q(p, 0, 4, 3, 3, 4, 2, p, p, None) == 2
    assert q(p, 4, -1, 3, 3, 4, 2, p, p, None) == 2
    assert q(p, 4, 4, 0, 3, 4, 2, p, p, None) == 2
    assert q(p, 4, 1 << 20, 1 << 10, 1 << 10, 4, 2, p, p, None) == 2
    assert q(p, 4, 4, 3, 3, 1, 2, p, p, None) == 3
    assert q(p, 4, 4, 3, 3, 9, 2, p, p, None) == 3
    assert q(p, 4, 4, 3, 3, 4, 4, p, p, None) == 4
    assert q(p, 4, 4, 3, 3, 4, -1, p, p, None) == 4


def test_batched_argument_checks(L):
    from paper_2202_07471_amd.binding import squant_tensor_t
    assert L.squant_batched_workspace_bytes(0) == 0
    assert L.squant_batched_workspace_bytes(3) == 0      # descriptors travel in the kernel arguments
    arr = (squant_tensor_t * 2)()
    arr[0] = squant_tensor_t(0x1000, 0x2000, 0x3000, 4, 4, 3, 3)
    arr[1] = squant_tensor_t(0x1000, 0x2000, 0x3000, 4, 4, 1, 1)
    ws = ctypes.c_void_p(0x4000)
    assert L.squant_quantize_batched(arr, 0, 4, 2, None, 0, None) == 0      # empty batch
    assert L.squant_quantize_batched(None, 2, 4, 2, ws, 1024, None) == 1
    assert L.squant_quantize_batched(arr, -1, 4, 2, ws, 1024, None) == 2
    assert L.squant_quantize_batched(arr, 2, 10, 2, ws, 1024, None) == 3
    assert L.squant_quantize_batched(arr, 2, 4, 9, ws, 1024, None) == 4
    assert L.squant_quantize_batched(arr, 2, 4, 2, None, 1024, None) == 5   # a size without a buffer
    arr[1].codes = None
    assert L.squant_quantize_batched(arr, 2, 4, 2, ws, 1024, None) == 1
    arr[1].codes = 0x2000
    arr[1].cin = 0
    assert L.squant_quantize_batched(arr, 2, 4, 2, ws, 1024, None) == 2


def test_binding_refuses_host_tensors():
    import torch
    import paper_2202_07471_amd as sq
    with pytest.raises(ValueError):
        sq.squant_quantize(torch.zeros(4, 4, 3, 3), 4)


def test_output_bytes_and_format_checks(L):
    assert L.squant_output_bytes(4, 3, 3, 3, 0) == 4 * 27
    assert L.squant_output_bytes(4, 3, 3, 3, 1) == 4 * 14      # odd rows round up
    assert L.squant_output_bytes(4, 4, 3, 3, 1) == 4 * 18
    assert L.squant_output_bytes(4, 3, 3, 3, 2) == 4 * 27 * 4
    assert L.squant_output_bytes(4, 3, 3, 3, 3) == 4 * 27 * 2
    assert L.squant_output_bytes(4, 3, 3, 3, 7) == 0
    assert L.squant_output_bytes(0, 3, 3, 3, 0) == 0
    p = ctypes.c_void_p(0x1000)
    q = lambda *a: L.squant_quantize_ex(*a)
    assert q(None, 0, 4, 4, 3, 3, 4, 2, 0, p, p, None) == 1
    assert q(p, 0, 4, 4, 3, 3, 4, 2, 1, None, p, None) == 1
    assert q(p, 0, 4, 0, 3, 3, 4, 2, 1, p, p, None) == 2
    assert q(p, 0, 4, 4, 3, 3, 9, 2, 0, p, p, None) == 3
    assert q(p, 0, 4, 4, 3, 3, 5, 2, 1, p, p, None) == 3       # packed 4-bit output needs bits <= 4
    assert q(p, 0, 4, 4, 3, 3, 8, 2, 1, p, p, None) == 3
    assert q(p, 0, 4, 4, 3, 3, 4, 5, 0, p, p, None) == 4
    assert q(p, 3, 4, 4, 3, 3, 4, 2, 0, p, p, None) == 8       # unknown weight type
    assert q(p, -1, 4, 4, 3, 3, 4, 2, 0, p, p, None) == 8
    assert q(p, 0, 4, 4, 3, 3, 4, 2, 4, p, p, None) == 8       # unknown output format
    assert q(p, 0, 4, 4, 3, 3, 4, 2, 3, ctypes.c_void_p(0x1001), p, None) == 8  # bfloat16 output off 2 bytes
    assert q(ctypes.c_void_p(0x1002), 0, 4, 4, 3, 3, 4, 2, 0, p, p, None) == 8   # float weights off 4 bytes
    assert q(p, 0, 4, 4, 3, 3, 4, 2, 2, ctypes.c_void_p(0x1002), p, None) == 8  # float output off 4 bytes
    from paper_2202_07471_amd.binding import squant_tensor_t
    arr = (squant_tensor_t * 1)()
    arr[0] = squant_tensor_t(0x1000, 0x2000, 0x3000, 4, 4, 3, 3)
    ws = ctypes.c_void_p(0x4000)
    assert L.squant_quantize_batched_ex(arr, 1, 0, 8, 2, 1, ws, 1024, None) == 3
    assert L.squant_quantize_batched_ex(arr, 1, 5, 4, 2, 0, ws, 1024, None) == 8
    assert L.squant_quantize_batched_ex(arr, 1, 0, 4, 2, 9, ws, 1024, None) == 8
    assert L.squant_quantize_batched_ex(arr, 0, 0, 4, 2, 1, None, 0, None) == 0


def test_activation_and_network_argument_checks(L):
    from paper_2202_07471_amd.binding import squant_bn_t, squant_layer_t, squant_tensor_t
    assert L.squant_activation_workspace_bytes(0) == 0
    assert L.squant_activation_workspace_bytes(5) == 0
    assert L.squant_network_workspace_bytes(5) == 0
    bn = (squant_bn_t * 2)()
    bn[0] = squant_bn_t(0x1000, 0x2000, 8, 1)
    bn[1] = squant_bn_t(0x1000, 0x2000, 8, 0)
    out, ws = ctypes.c_void_p(0x3000), ctypes.c_void_p(0x4000)
    f = L.squant_activation_ranges
    assert f(bn, 0, 6.0, 8, None, None, 0, None) == 0
    assert f(None, 2, 6.0, 8, out, ws, 1024, None) == 1
    assert f(bn, 2, 6.0, 8, None, ws, 1024, None) == 1
    assert f(bn, -1, 6.0, 8, out, ws, 1024, None) == 2
    assert f(bn, 2, 6.0, 1, out, ws, 1024, None) == 3
    assert f(bn, 2, 6.0, 17, out, ws, 1024, None) == 3
    assert f(bn, 2, -1.0, 8, out, ws, 1024, None) == 2
    assert f(bn, 2, float("nan"), 8, out, ws, 1024, None) == 2
    assert f(bn, 2, float("inf"), 8, out, ws, 1024, None) == 2
    assert f(bn, 2, 6.0, 8, out, None, 1024, None) == 5
    bn[1].channels = 0
    assert f(bn, 2, 6.0, 8, out, ws, 1024, None) == 2
    bn[1].channels = 8
    bn[1].beta = None
    assert f(bn, 2, 6.0, 8, out, ws, 1024, None) == 1
    layers = (squant_layer_t * 1)()
    layers[0] = squant_layer_t(squant_tensor_t(0x1000, 0x2000, 0x3000, 4, 4, 3, 3), squant_bn_t(0x1000, 0x2000, 4, 1))
    g = L.squant_quantize_network
    assert g(layers, 0, 4, 2, 8, 6.0, None, None, 0, None) == 0
    assert g(None, 1, 4, 2, 8, 6.0, out, ws, 4096, None) == 1
    assert g(layers, 1, 4, 2, 8, 6.0, None, ws, 4096, None) == 1      # batch norm given, no result array
    assert g(layers, 1, 4, 2, 1, 6.0, out, ws, 4096, None) == 3
    assert g(layers, 1, 9, 2, 8, 6.0, out, ws, 4096, None) == 3
    assert g(layers, 1, 4, 7, 8, 6.0, out, ws, 4096, None) == 4
    assert g(layers, 1, 4, 2, 8, 6.0, out, None, 8, None) == 5


def test_header_is_plain_c(tmp_path):
    """The boundary is a C header: it must compile as C99 on its own."""
    import subprocess
    src = tmp_path / "use_header.c"
    src.write_text('#include "squant.h"\n'
                   'int probe(void) { squant_tensor_t t; squant_layer_t l; squant_act_range_t r;\n'
                   '  (void)t; (void)l; (void)r; return (int)SQUANT_OUT_BF16 + (int)SQUANT_W_BF16 + (int)SQUANT_MODE_EC; }\n')
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only",
                           "-I", os.path.join(ROOT, "include"), str(src)])
