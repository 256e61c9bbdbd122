"""Seeded random parity cases: shapes of every kernel family, value patterns chosen to hit the
rare branches of the selections (ties by the thousand, exact zeros, exact halves, one-sided
channels), every bit width and mode.  Each case is compared bit for bit with the CPU
reference; the case is printed before it runs so that a failure names it."""
import sys

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


def random_shape(rng):
    family = rng.integers(0, 4)
    m = int(rng.integers(1, 7))
    if family == 0:                                   # 3x3, cin % 4 == 0 (now and then a wide one)
        hi = 1025 if rng.random() < 0.1 else 160
        return (m, 4 * int(rng.integers(1, hi)), 3, 3)
    if family == 1:                                   # 1x1 / FC, cin % 4 == 0 (now and then very long)
        hi = 12000 if rng.random() < 0.15 else 2400
        return (min(m, 3), 4 * int(rng.integers(1, hi)), 1, 1)
    if family == 2:                                   # generic kernels
        kh, kw = [(2, 2), (1, 3), (3, 3), (5, 5), (7, 7), (4, 4), (1, 7), (3, 1)][rng.integers(0, 8)]
        n = int(rng.integers(1, 120))
        if (kh, kw) == (3, 3) and n % 4 == 0:
            n += 1
        return (m, n, kh, kw)
    return (m, int(rng.integers(1, 3000)) | 1, 1, 1)  # odd cin: generic 1x1


def random_values(rng, shape):
    kind = rng.integers(0, 7)
    if kind == 0:
        w = rng.standard_normal(shape) * 0.05
    elif kind == 1:
        w = rng.standard_t(3, shape) * 0.05
    elif kind == 2:                                   # few levels: ties, exact halves, zero sums
        levels = int(rng.integers(2, 40))
        w = rng.integers(-levels, levels + 1, shape) / float(rng.choice([2, 4, 8, 3, 5]))
    elif kind == 3:                                   # one-sided perturbations
        w = np.full(shape, 0.3) + rng.random(shape) * 0.1
    elif kind == 4:                                   # mostly zeros
        w = rng.standard_normal(shape) * (rng.random(shape) < 0.1)
    elif kind == 5:                                   # a constant with a few outliers
        w = np.full(shape, float(rng.choice([0.37, -1.25, 2.5])))
        idx = rng.random(shape) < 0.02
        w[idx] = rng.standard_normal(int(idx.sum())) * 3
    else:                                             # huge dynamic range
        w = rng.standard_normal(shape) * np.exp(rng.uniform(-20, 20, (shape[0], 1, 1, 1)))
    w = w.astype(np.float32)
    if shape[0] > 2 and rng.random() < 0.3:
        w[int(rng.integers(0, shape[0]))] = 0.0
    return w


@pytest.mark.parametrize("block", range(16))
def test_random_cases(sq, block):
    rng = np.random.default_rng(5000 + block)
    for case in range(60):
        shape = random_shape(rng)
        w = random_values(rng, shape)
        bits = int(rng.integers(2, 9))
        mode = int(rng.integers(0, 4))
        print(f"case block={block} #{case} shape={shape} bits={bits} mode={mode}", flush=True)
        sys.stdout.flush()
        codes, scales = sq.squant_quantize(torch.from_numpy(w).cuda(), bits, mode)
        torch.cuda.synchronize()
        want_c, want_s = oracle.quantize(w, bits, mode, threads=4)
        assert np.array_equal(scales.cpu().numpy().view(np.uint32), want_s.view(np.uint32)), \
            f"scales differ: block={block} case={case} shape={shape} bits={bits} mode={mode}"
        got = codes.cpu().numpy()
        if not np.array_equal(got, want_c):
            bad = np.argwhere(got != want_c)
            raise AssertionError(f"codes differ: block={block} case={case} shape={shape} bits={bits} "
                                 f"mode={mode}: {len(bad)} elements, first at {bad[0].tolist()}")
        if case % 3 == 0:                             # the same case through another type / format
            wtype = ["f16", "bf16"][int(rng.integers(0, 2))]
            t16 = torch.from_numpy(w).to(torch.float16 if wtype == "f16" else torch.bfloat16)
            w16 = oracle.widen(t16.view(torch.int16).numpy().view(np.uint16), wtype)
            if not np.isfinite(w16).all():
                continue                              # the huge-range pattern leaves binary16
            want_c, want_s = oracle.quantize(w16, bits, mode, threads=4)
            fmt = "int4" if bits <= 4 else ["f32", "bf16"][int(rng.integers(0, 2))]
            print(f"     again as {wtype} -> {fmt}", flush=True)
            out, scales = sq.squant_quantize_ex(t16.cuda(), bits, mode, sq.OUTPUTS[fmt])
            torch.cuda.synchronize()
            assert np.array_equal(scales.cpu().numpy().view(np.uint32), want_s.view(np.uint32)), \
                f"scales differ ({wtype}): block={block} case={case} shape={shape}"
            if fmt == "int4":
                ok = np.array_equal(out.cpu().numpy(), oracle.pack_int4(want_c))
            elif fmt == "f32":
                ok = np.array_equal(out.cpu().numpy().view(np.uint32),
                                    oracle.dequantize(want_c, want_s).view(np.uint32))
            else:
                ok = np.array_equal(out.view(torch.int16).cpu().numpy().view(np.uint16),
                                    oracle.dequantize_bf16(want_c, want_s))
            assert ok, f"{wtype} -> {fmt} differs: block={block} case={case} shape={shape} bits={bits} mode={mode}"


def test_random_batches(sq):
    """Random tensors in one batched call: mixed launches with arbitrary membership."""
    rng = np.random.default_rng(77)
    for rep in range(6):
        shapes = [random_shape(rng) for _ in range(int(rng.integers(2, 30)))]
        ws = [random_values(rng, s) for s in shapes]
        bits, mode = int(rng.integers(2, 9)), int(rng.integers(0, 4))
        print(f"batch #{rep}: {len(ws)} tensors bits={bits} mode={mode}", flush=True)
        codes, scales = sq.squant_quantize_batched([torch.from_numpy(w).cuda() for w in ws], bits, mode)
        torch.cuda.synchronize()
        for s, w, c, sc in zip(shapes, ws, codes, scales):
            want_c, want_s = oracle.quantize(w, bits, mode, threads=4)
            assert np.array_equal(sc.cpu().numpy().view(np.uint32), want_s.view(np.uint32)), (rep, s)
            assert np.array_equal(c.cpu().numpy(), want_c), f"batch {rep} shape {s} bits={bits} mode={mode}"
