"""GPU parity for the kernels held in registers other than 3x3 (1x3, 3x1, 2x2, 1x5, 1x7, 7x1 ...):
every kernel size the variant is built for, channel widths that select each number of kernels
per thread and both workgroup bounds, every mode, the other output formats and weight types,
degenerate inputs, and the shapes next to it that fall back to the generic kernel."""
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
    if kind == "grid":      # many equal perturbations, exact halves, zero kernel sums
        w = rng.integers(-28, 29, shape).astype(np.float32) / 4.0
        w.reshape(shape[0], -1)[:, 0] = 7.0
        return w
    if kind == "heavy":
        return (rng.standard_t(3, shape) * 0.05).astype(np.float32)
    if kind == "onesided":  # every perturbation of a channel has the same sign: many channel flips
        w = rng.integers(-7, 8, shape).astype(np.float32)
        w += np.float32(0.3) * np.where(np.arange(shape[0]) % 2 == 0, 1, -1).reshape(-1, 1, 1, 1).astype(np.float32)
        w.reshape(shape[0], -1)[:, 0] = 7.0
        return w
    w = (rng.standard_normal(shape) * 0.05).astype(np.float32)
    if shape[0] > 2:
        w[1] = 0.0
        w[2] = 0.25
    return w


def check(got, got_s, want, want_s, what):
    if got.dtype == torch.bfloat16:
        got = got.view(torch.int16)
    got, got_s = got.cpu().numpy(), got_s.cpu().numpy()
    if got.dtype == np.int16:
        got = got.view(np.uint16)
    got = got.reshape(want.shape)
    assert np.array_equal(got_s.view(np.uint32), want_s.view(np.uint32)), f"scales differ {what}"
    a = got.view(np.uint32) if got.dtype == np.float32 else got
    b = want.view(np.uint32) if want.dtype == np.float32 else want
    if not np.array_equal(a, b):
        bad = np.argwhere(a != b)
        raise AssertionError(f"{what}: {len(bad)} outputs differ, first at {bad[0].tolist()} "
                             f"gpu={got[tuple(bad[0])]} ref={want[tuple(bad[0])]}")


# (kh, kw) with kh*kw in {2, 3, 4, 5, 7, 25}; cin chosen to reach 1, 2, 4 and 8 kernels per thread,
# partly filled waves, more than 256 threads (the 1024-thread instantiation) and its maximum
KERNELS = [(1, 2), (1, 3), (3, 1), (2, 2), (1, 5), (1, 7), (7, 1), (4, 1), (5, 5)]
CINS = [4, 8, 20, 64, 96, 128, 192, 384, 448, 1024, 2056, 4096]


@pytest.mark.parametrize("kind", ["normal", "grid", "heavy", "onesided"])
@pytest.mark.parametrize("khw", KERNELS)
def test_small_kernels_every_width(sq, khw, kind):
    kh, kw = khw
    for cin in CINS:
        if kh * kw == 25 and cin > 1024:      # 5x5: one kernel per thread, so cin <= 1024; beyond it the
            cin = 1028 if cin == 2056 else 48  # generic kernel (1028 fits its LDS), and the common cin = 48
        cout = 5 if cin < 1024 else 3
        shape = (cout, cin, kh, kw)
        w = weights(shape, 97 + cin + 10 * kh + kw, kind)
        dw = torch.from_numpy(w).cuda()
        for bits, mode in ((4, 2), (8, 1), (3, 3), (2, 0), (6, 2)):
            want, want_s = oracle.quantize(w, bits, mode, threads=8)
            got, got_s = sq.squant_quantize(dw, bits, mode)
            torch.cuda.synchronize()
            check(got, got_s, want, want_s, f"{shape} {kind} bits={bits} mode={mode}")


@pytest.mark.parametrize("khw", [(1, 3), (1, 7), (2, 2), (1, 5), (1, 2), (5, 5)])
def test_small_kernels_largest_channels(sq, khw):
    kh, kw = khw
    K = kh * kw
    top = 8 if K <= 4 else 4 if K <= 7 else 1   # most kernels one thread holds
    cin = 1024 * top                            # the widest channel the variant takes
    for c in (cin, cin - max(4, top), cin + 8):   # ... and its neighbours
        shape = (2, c, kh, kw)
        w = weights(shape, 5 + c + K, "normal")
        if c > cin and c * K > sq.squant_max_channel_elems(kh, kw):
            # beyond the variant the generic kernel would have to hold the channel in LDS
            with pytest.raises(sq.SQuantError):
                sq.squant_quantize(torch.from_numpy(w).cuda(), 4, 2)
            continue
        want, want_s = oracle.quantize(w, 4, 2, threads=8)
        got, got_s = sq.squant_quantize(torch.from_numpy(w).cuda(), 4, 2)
        torch.cuda.synchronize()
        check(got, got_s, want, want_s, f"{shape}")


@pytest.mark.parametrize("shape", [(4, 6, 1, 3), (4, 10, 1, 2), (3, 5, 1, 7), (3, 7, 5, 1), (6, 1, 1, 7), (5, 1, 2, 2),
                                   (3, 33, 1, 3), (2, 4100, 1, 5)])
def test_neighbouring_shapes_use_the_generic_kernel(sq, shape):
    # cin * kh * kw not a multiple of 4, one kernel per channel, or a channel too wide
    w = weights(shape, 3 + sum(shape), "grid")
    for bits, mode in ((4, 2), (3, 3)):
        want, want_s = oracle.quantize(w, bits, mode, threads=8)
        got, got_s = sq.squant_quantize(torch.from_numpy(w).cuda(), bits, mode)
        torch.cuda.synchronize()
        check(got, got_s, want, want_s, f"{shape} bits={bits} mode={mode}")


@pytest.mark.parametrize("output", ["int4", "f32", "bf16"])
@pytest.mark.parametrize("shape", [(5, 192, 1, 7), (5, 384, 3, 1), (4, 48, 1, 5), (6, 8, 2, 2), (3, 2052, 1, 3),
                                   (5, 12, 1, 3), (4, 22, 1, 2), (5, 48, 5, 5)])
def test_small_kernels_other_outputs(sq, shape, output):
    out = {"int4": sq.OUT_INT4, "f32": sq.OUT_F32, "bf16": sq.OUT_BF16}[output]
    for kind in ("normal", "grid"):
        w = weights(shape, 41 + sum(shape), kind)
        for bits, mode in ((4, 2), (3, 1)):
            codes, scales = oracle.quantize(w, bits, mode, threads=8)
            want = {"int4": oracle.pack_int4, "f32": lambda c: oracle.dequantize(c, scales),
                    "bf16": lambda c: oracle.dequantize_bf16(c, scales)}[output](codes)
            got, got_s = sq.squant_quantize_ex(torch.from_numpy(w).cuda(), bits, mode, out)
            torch.cuda.synchronize()
            check(got, got_s, want, scales, f"{output} {shape} {kind} bits={bits} mode={mode}")


@pytest.mark.parametrize("wtype", ["f16", "bf16"])
@pytest.mark.parametrize("shape", [(5, 192, 1, 7), (5, 384, 3, 1), (4, 48, 1, 5), (6, 8, 2, 2), (3, 2052, 1, 3),
                                   (4, 22, 1, 2), (5, 48, 5, 5)])
def test_small_kernels_sixteen_bit_weights(sq, shape, wtype):
    for kind in ("normal", "grid"):
        t16 = torch.from_numpy(weights(shape, 53 + sum(shape), kind)).to(
            torch.float16 if wtype == "f16" else torch.bfloat16)
        w32 = oracle.widen(t16.view(torch.int16).numpy().view(np.uint16), wtype)
        for bits, mode in ((4, 2), (5, 3)):
            want, want_s = oracle.quantize(w32, bits, mode, threads=8)
            got, got_s = sq.squant_quantize_ex(t16.cuda(), bits, mode)
            torch.cuda.synchronize()
            check(got, got_s, want, want_s, f"{wtype} {shape} {kind} bits={bits} mode={mode}")


def test_small_kernels_degenerate_channels(sq):
    # all-zero tensor, one non-zero weight, equal weights (every perturbation ties), exact halves
    for kh, kw, cin in ((1, 3, 64), (1, 7, 32), (2, 2, 16), (1, 5, 12), (1, 2, 256), (5, 5, 8)):
        shape = (6, cin, kh, kw)
        w = np.zeros(shape, np.float32)
        w[1, 3, 0, 0] = -2.5
        w[2] = 0.3
        w[3] = np.float32(7.0)
        w[3].reshape(-1)[1:] = 3.5          # x = 3.5 at 4 bits with absmax 7: exact halves
        w[4] = -1.0
        w[4].reshape(-1)[::2] = 0.45
        w[5].reshape(-1)[0] = 1e-30
        for bits, mode in ((4, 2), (4, 3), (2, 2), (8, 1)):
            want, want_s = oracle.quantize(w, bits, mode, threads=8)
            got, got_s = sq.squant_quantize(torch.from_numpy(w).cuda(), bits, mode)
            torch.cuda.synchronize()
            check(got, got_s, want, want_s, f"{shape} bits={bits} mode={mode}")


def test_small_kernels_in_a_layer_set(sq):
    # factorised-convolution layers beside 3x3 and 1x1 ones in one batched call
    shapes = [(24, 128, 1, 7), (24, 128, 7, 1), (32, 384, 1, 3), (32, 384, 3, 1), (16, 48, 5, 5), (32, 64, 3, 3),
              (48, 192, 1, 1), (16, 3, 3, 3), (12, 160, 1, 7), (10, 1000, 1, 1), (20, 96, 2, 2)]
    ws = [weights(s, 700 + i, "normal" if i % 2 else "grid") for i, s in enumerate(shapes)]
    plan = sq.BatchPlan([torch.from_numpy(w).cuda() for w in ws])
    for bits, mode in ((4, 2), (4, 3), (8, 1)):
        codes, scales = plan.run(bits, mode)
        torch.cuda.synchronize()
        for w, c, sc in zip(ws, codes, scales):
            want, want_s = oracle.quantize(w, bits, mode, threads=8)
            check(c, sc, want, want_s, f"{w.shape} bits={bits} mode={mode}")


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


@pytest.mark.parametrize("block", range(8))
def test_random_small_kernel_cases(sq, block):
    """Seeded random cases on the shapes of this variant (cin * kh * kw a multiple of 4), value
    patterns that reach the rare branches, every bit width and mode; each case is printed
    before it runs."""
    rng = np.random.default_rng(9000 + block)
    kernels = [(1, 2), (2, 1), (1, 3), (3, 1), (2, 2), (1, 4), (1, 5), (5, 1), (1, 7), (7, 1), (5, 5)]
    for case in range(40):
        kh, kw = kernels[int(rng.integers(0, len(kernels)))]
        K = kh * kw
        step = 4 if K % 2 else (2 if K % 4 else 1)    # keeps cin * K a multiple of 4
        hi = (8200 if K <= 4 else 4200 if K <= 7 else 1030) if rng.random() < 0.15 else 520
        cin = step * int(rng.integers(1, hi // step + 1))
        if K == 25 and cin > 1024:
            cin = 1024                                 # beyond it the generic kernel's LDS limit decides
        shape = (int(rng.integers(1, 5)), cin, kh, kw)
        if cin * K > sq.squant_max_channel_elems(kh, kw) and cin % (8 if K <= 4 else 4):
            continue                                   # too wide for the generic kernel, not a multiple for this one
        w = random_values(rng, shape)
        bits, mode = int(rng.integers(2, 9)), int(rng.integers(0, 4))
        print(f"case block={block} #{case} shape={shape} bits={bits} mode={mode}", flush=True)
        want, want_s = oracle.quantize(w, bits, mode, threads=4)
        got, got_s = sq.squant_quantize(torch.from_numpy(w).cuda(), bits, mode)
        torch.cuda.synchronize()
        check(got, got_s, want, want_s, f"block={block} case={case} {shape} bits={bits} mode={mode}")
        if case % 3 == 0:                              # again from 16-bit weights into another format
            wtype = ["f16", "bf16"][int(rng.integers(0, 2))]
            t16 = torch.from_numpy(w).to(torch.float16 if wtype == "f16" else torch.bfloat16)
            w16 = oracle.widen(t16.view(torch.int16).numpy().view(np.uint16), wtype)
            if not np.isfinite(w16).all():
                continue
            codes, scales = oracle.quantize(w16, bits, mode, threads=4)
            fmt = "int4" if bits <= 4 else ["f32", "bf16"][int(rng.integers(0, 2))]
            want = {"int4": oracle.pack_int4, "f32": lambda c: oracle.dequantize(c, scales),
                    "bf16": lambda c: oracle.dequantize_bf16(c, scales)}[fmt](codes)
            print(f"     again as {wtype} -> {fmt}", flush=True)
            got, got_s = sq.squant_quantize_ex(t16.cuda(), bits, mode, sq.OUTPUTS[fmt])
            torch.cuda.synchronize()
            check(got, got_s, want, scales, f"{wtype}->{fmt} block={block} case={case} {shape} bits={bits} mode={mode}")
