"""GPU parity for binary16 / bfloat16 weights: the HIP path reads the 16-bit tensor, the
CPU reference gets the same bit patterns widened by its own routine."""
import numpy as np
import pytest

import oracle
from paper_2202_07471_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def sq():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2202_07471_amd as sq
    sq.binding.lib()
    return sq


def to16(w, wtype):
    """float32 array -> (torch 16-bit CPU tensor, uint16 bit patterns)."""
    t = torch.from_numpy(w).to(torch.float16 if wtype == "f16" else torch.bfloat16)
    bits = t.view(torch.int16).numpy().view(np.uint16)
    return t, bits


def weights(shape, seed, kind):
    rng = np.random.default_rng(seed)
    if kind == "grid":
        w = rng.integers(-28, 29, shape).astype(np.float32) / 4.0
        w.reshape(shape[0], -1)[:, 0] = 7.0
        return w
    if kind == "tiny":       # binary16 subnormals (below 6.1e-5) and near-subnormals
        return (rng.standard_normal(shape) * 2e-5).astype(np.float32)
    if kind == "large":
        return (rng.standard_normal(shape) * 9000.0).astype(np.float32).clip(-65000, 65000)
    w = (rng.standard_normal(shape) * 0.05).astype(np.float32)
    if shape[0] > 2:
        w[1] = 0.0
    return w


def check_codes(got, got_s, want, want_s, what):
    got, got_s = got.cpu().numpy().reshape(want.shape), got_s.cpu().numpy()
    assert np.array_equal(got_s.view(np.uint32), want_s.view(np.uint32)), f"scales differ {what}"
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        raise AssertionError(f"{what}: {len(bad)} differ, first at {bad[0].tolist()} "
                             f"gpu={got[tuple(bad[0])]} ref={want[tuple(bad[0])]}")


SHAPES = [
    (6, 64, 3, 3), (6, 128, 3, 3), (4, 512, 3, 3), (5, 4, 3, 3), (5, 12, 3, 3), (3, 36, 3, 3),
    (6, 96, 3, 3), (2, 4096, 3, 3), (4, 1100, 3, 3),
    (9, 512, 1, 1), (7, 1028, 1, 1), (40, 16, 1, 1), (3, 8192, 1, 1), (2, 32764, 1, 1),
    (33, 17, 3, 3), (96, 1, 3, 3), (8, 5, 3, 3), (5, 3, 7, 7), (4, 3, 11, 11), (17, 63, 1, 1),
    (1, 1, 1, 1), (130, 1, 3, 3),
]


@pytest.mark.parametrize("wtype", ["f16", "bf16"])
@pytest.mark.parametrize("kind", ["normal", "grid", "tiny", "large"])
@pytest.mark.parametrize("shape", SHAPES)
def test_sixteen_bit_weights(sq, shape, kind, wtype):
    t16, bits = to16(weights(shape, 31 + sum(shape), kind), wtype)
    w32 = oracle.widen(bits, wtype)
    assert np.array_equal(w32, t16.float().numpy())       # the two widenings agree
    d16 = t16.cuda()
    for bits_q, mode in ((4, 2), (8, 1), (3, 3)):
        want, want_s = oracle.quantize(w32, bits_q, mode, threads=8)
        got, got_s = sq.squant_quantize_ex(d16, bits_q, mode)
        torch.cuda.synchronize()
        check_codes(got, got_s, want, want_s, f"{wtype} {shape} {kind} bits={bits_q} mode={mode}")


@pytest.mark.parametrize("wtype", ["f16", "bf16"])
def test_sixteen_bit_weights_off_alignment(sq, wtype):
    """A tensor that starts 2 bytes off a dword boundary goes through the generic kernel."""
    for shape in [(6, 64, 3, 3), (9, 512, 1, 1)]:
        t16, bits = to16(weights(shape, 3, "normal"), wtype)
        big = torch.zeros(t16.numel() + 8, dtype=t16.dtype, device="cuda")
        view = big[1:1 + t16.numel()].view(shape)
        view.copy_(t16)
        assert view.data_ptr() % 4 == 2
        want, want_s = oracle.quantize(oracle.widen(bits, wtype), 4, 2, threads=8)
        got, got_s = sq.squant_quantize_ex(view, 4, 2)
        torch.cuda.synchronize()
        check_codes(got, got_s, want, want_s, f"offset {wtype} {shape}")


@pytest.mark.parametrize("wtype,output", [("f16", "int8"), ("bf16", "int4"), ("f16", "f32")])
def test_layer_set_batched_sixteen_bit(sq, wtype, output):
    specs = synth.config_specs(2)
    pairs = [to16(synth.generate(s), wtype) for s in specs]
    fmt = sq.OUTPUTS[output]
    outs, scales = sq.squant_quantize_batched_ex([t.cuda() for t, _ in pairs], 4, 2, fmt)
    torch.cuda.synchronize()
    for s, (t, bits), o, sc in zip(specs, pairs, outs, scales):
        codes, want_s = oracle.quantize(oracle.widen(bits, wtype), 4, 2, threads=8)
        want = {"int8": codes, "int4": oracle.pack_int4(codes) if output == "int4" else None,
                "f32": oracle.dequantize(codes, want_s)}[output]
        got = o.cpu().numpy()
        assert np.array_equal(sc.cpu().numpy().view(np.uint32), want_s.view(np.uint32)), s.shape
        if output == "f32":
            got, want = got.view(np.uint32), want.view(np.uint32)
        assert np.array_equal(got.reshape(want.shape), want), f"batched {wtype} {output} {s.shape}"


@pytest.mark.parametrize("wtype,output", [("f16", "int4"), ("bf16", "bf16")])
def test_streaming_kernel_sixteen_bit_and_formats(sq, wtype, output):
    shape = (2, 50000, 1, 1)
    t16, bits = to16(weights(shape, 77, "normal"), wtype)
    codes, want_s = oracle.quantize(oracle.widen(bits, wtype), 4, 2, threads=8)
    got, got_s = sq.squant_quantize_ex(t16.cuda(), 4, 2, sq.OUTPUTS[output])
    torch.cuda.synchronize()
    assert np.array_equal(got_s.cpu().numpy().view(np.uint32), want_s.view(np.uint32))
    if output == "int4":
        assert np.array_equal(got.cpu().numpy(), oracle.pack_int4(codes))
    else:
        want = oracle.dequantize_bf16(codes, want_s)
        assert np.array_equal(got.view(torch.int16).cpu().numpy().view(np.uint16).reshape(want.shape), want)


def test_mixed_dtypes_in_one_batch_are_refused(sq):
    a = torch.zeros((4, 4, 3, 3), device="cuda")
    with pytest.raises(ValueError):
        sq.BatchPlan([a, a.half()])


def test_config5_full_size_bf16_to_packed_int4_sampled(sq):
    """The benchmark's 256 x [512,512,3,3] workload with bfloat16 weights and packed 4-bit
    output in one batched call; the reference checks sampled whole tensors and channels."""
    specs = synth.config_specs(5)
    shape = specs[0].shape
    rng = np.random.default_rng(2)
    sample_tensors = {3, 200}
    sample_channels = {int(t): sorted(set(int(c) for c in rng.integers(0, shape[0], 2)))
                       for t in rng.choice(256, 24, replace=False)}
    keep, dws = {}, []
    buf = np.empty(shape, np.float32)
    for s in specs:
        w = synth.generate(s, out=buf)
        d16 = torch.from_numpy(w).cuda().to(torch.bfloat16)
        if s.index in sample_tensors or s.index in sample_channels:
            keep[s.index] = d16.cpu().view(torch.int16).numpy().view(np.uint16)
        dws.append(d16)
    outs, scales = sq.squant_quantize_batched_ex(dws, 4, 2, sq.OUT_INT4)
    torch.cuda.synchronize()
    row = shape[1] * shape[2] * shape[3] // 2
    for t in sample_tensors:
        codes, want_s = oracle.quantize(oracle.widen(keep[t], "bf16"), 4, 2, threads=8)
        assert np.array_equal(outs[t].cpu().numpy(), oracle.pack_int4(codes)), f"tensor {t}"
        assert np.array_equal(scales[t].cpu().numpy().view(np.uint32), want_s.view(np.uint32))
    for t, chans in sample_channels.items():
        for c in chans:
            codes, want_s = oracle.quantize(oracle.widen(keep[t][c][None], "bf16"), 4, 2)
            got = outs[t][c].cpu().numpy()
            assert got.shape == (row,) and np.array_equal(got, oracle.pack_int4(codes)[0]), (t, c)
            assert scales[t][c].cpu().numpy().view(np.uint32) == want_s.view(np.uint32)[0]
