"""The streaming fallback kernel: output channels that fit none of the on-chip kernels (3x3 beyond
cin 4096, other kernel sizes beyond what LDS holds, unaligned or very long 1x1 / FC rows), every
mode, several bit widths, weight types and output formats, against the CPU reference bit for bit."""
import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def sq():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2202_07471_amd as sq
    sq.binding.lib()
    return sq


def weights(shape, seed, kind):
    rng = np.random.default_rng(seed)
    if kind == "normal":
        return (rng.standard_normal(shape) * 0.05).astype(np.float32)
    if kind == "heavy":
        return (rng.standard_t(3, shape) * 0.05).astype(np.float32)
    if kind == "grid":      # coarse grid: ties by the thousand, exact halves, exact zero sums
        w = rng.integers(-28, 29, shape).astype(np.float32) / 4.0
        w.reshape(shape[0], -1)[:, 0] = 7.0
        return w
    if kind == "constant":  # every candidate equal: the selection is decided by the kernel index alone
        w = np.full(shape, 0.3, np.float32)
        w.reshape(shape[0], -1)[:, 0] = 7.0
        return w
    raise ValueError(kind)


def check(sq, w, bits, mode, what):
    codes, scales = sq.squant_quantize(torch.from_numpy(w).cuda(), bits, mode)
    torch.cuda.synchronize()
    want_c, want_s = oracle.quantize(w, bits, mode, threads=8)
    assert np.array_equal(scales.cpu().numpy().view(np.uint32), want_s.view(np.uint32)), f"scales differ: {what}"
    got = codes.cpu().numpy()
    if not np.array_equal(got, want_c):
        bad = np.argwhere(got != want_c)
        raise AssertionError(f"codes differ: {what}: {len(bad)} elements, first at {bad[0].tolist()}")


SHAPES = [(2, 8192, 3, 3), (1, 1200, 7, 7), (2, 2100, 5, 5), (3, 4100, 3, 3), (1, 300000, 1, 1),
          (2, 9000, 2, 2), (1, 48, 64, 64), (2, 30001, 1, 3)]


@pytest.mark.parametrize("kind", ["normal", "heavy", "grid", "constant"])
@pytest.mark.parametrize("shape", SHAPES)
def test_oversize_channels(sq, shape, kind):
    w = weights(shape, 31 + shape[1], kind)
    for bits, mode in ((4, 2), (8, 2), (3, 1), (4, 0), (5, 3)):
        print(f"stream {shape} {kind} bits={bits} mode={mode}", flush=True)
        check(sq, w, bits, mode, f"{shape} {kind} bits={bits} mode={mode}")


def test_unaligned_long_rows(sq):
    """A 1x1 / FC tensor whose rows start 4 bytes off a 16-byte boundary and are too long for the
    kernel that holds such a channel in LDS."""
    for n in (20000, 45001):
        buf = torch.from_numpy(weights((2 * n + 1,), 5 + n, "normal")).cuda()
        view = buf[1:].view(2, n, 1, 1)
        assert view.data_ptr() % 16 == 4
        w = view.cpu().numpy()
        for bits, mode in ((4, 2), (8, 3), (2, 0)):
            codes, scales = sq.squant_quantize(view, bits, mode)
            torch.cuda.synchronize()
            want_c, want_s = oracle.quantize(w, bits, mode, threads=8)
            assert np.array_equal(scales.cpu().numpy(), want_s)
            assert np.array_equal(codes.cpu().numpy(), want_c), f"unaligned n={n} bits={bits} mode={mode}"


@pytest.mark.parametrize("shape", [(3, 1201, 7, 7), (2, 4111, 3, 3), (2, 12001, 1, 5)])
def test_oversize_channels_other_types_and_formats(sq, shape):
    """binary16 / bfloat16 weights and the other output forms through the streaming kernel; odd
    kernel sizes and odd kernel counts put the packed 4-bit byte boundaries inside kernels."""
    w = weights(shape, 77, "normal")
    for wtype, tdtype in (("f16", torch.float16), ("bf16", torch.bfloat16)):
        t16 = torch.from_numpy(w).to(tdtype)
        w16 = oracle.widen(t16.view(torch.int16).numpy().view(np.uint16), wtype)
        for bits, mode, fmt in ((4, 2, "int4"), (3, 3, "int4"), (8, 2, "f32"), (6, 1, "bf16"), (4, 2, "int8")):
            print(f"stream {shape} {wtype} -> {fmt} bits={bits} mode={mode}", flush=True)
            want_c, want_s = oracle.quantize(w16, bits, mode, threads=8)
            out, scales = sq.squant_quantize_ex(t16.cuda(), bits, mode, sq.OUTPUTS[fmt])
            torch.cuda.synchronize()
            assert np.array_equal(scales.cpu().numpy().view(np.uint32), want_s.view(np.uint32))
            if fmt == "int4":
                ok = np.array_equal(out.cpu().numpy(), oracle.pack_int4(want_c))
            elif fmt == "int8":
                ok = np.array_equal(out.cpu().numpy(), want_c)
            elif fmt == "f32":
                ok = np.array_equal(out.cpu().numpy().view(np.uint32), oracle.dequantize(want_c, want_s).view(np.uint32))
            else:
                ok = np.array_equal(out.view(torch.int16).cpu().numpy().view(np.uint16),
                                    oracle.dequantize_bf16(want_c, want_s))
            assert ok, f"{shape} {wtype} -> {fmt} bits={bits} mode={mode}"


def test_oversize_members_of_a_batch(sq):
    """Oversize tensors beside ordinary ones in one batched call."""
    shapes = [(4, 64, 3, 3), (2, 5000, 3, 3), (3, 512, 1, 1), (1, 1500, 7, 7), (2, 256, 3, 3)]
    ws = [weights(s, 9 + i, "normal") for i, s in enumerate(shapes)]
    codes, scales = sq.squant_quantize_batched([torch.from_numpy(w).cuda() for w in ws], 4, 2)
    torch.cuda.synchronize()
    for s, w, c, sc in zip(shapes, ws, codes, scales):
        want_c, want_s = oracle.quantize(w, 4, 2, threads=8)
        assert np.array_equal(sc.cpu().numpy(), want_s), s
        assert np.array_equal(c.cpu().numpy(), want_c), s
