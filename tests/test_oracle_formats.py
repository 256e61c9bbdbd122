"""Pins for the reference's output forms and input widening: packed 4-bit codes, the
dequantised weight of Section 2.2, binary16 / bfloat16 to binary32."""
import numpy as np
import pytest

import oracle
from oracle import MODE_EKC
from paper_2202_07471_amd import synth


def unpack_int4_numpy(packed, n):
    """Independent inverse: split bytes into nibbles, sign-extend."""
    p = packed.astype(np.int16)
    lo, hi = p & 15, p >> 4
    both = np.stack([lo, hi], axis=-1).reshape(packed.shape[0], -1)[:, :n]
    return np.where(both >= 8, both - 16, both).astype(np.int8)


def test_pack_int4_hand_written_bytes():
    # -7 -> 0x9, 7 -> 0x7, -1 -> 0xF, 0 -> 0x0, 3 -> 0x3; odd length leaves a zero high nibble
    got = oracle.pack_int4(np.array([[-7, 7, -1, 0, 3], [1, 2, 3, 4, -8]], np.int8))
    assert got.tolist() == [[0x79, 0x0F, 0x03], [0x21, 0x43, 0x08]]


@pytest.mark.parametrize("shape", [(3, 9), (4, 2, 3, 3), (5, 1, 1, 1), (2, 7, 5, 5), (6, 64)])
def test_pack_int4_round_trip(shape):
    rng = np.random.default_rng(sum(shape))
    codes = rng.integers(-7, 8, shape).astype(np.int8)
    packed = oracle.pack_int4(codes)
    n = codes.size // shape[0]
    assert packed.shape == (shape[0], (n + 1) // 2)
    assert np.array_equal(unpack_int4_numpy(packed, n), codes.reshape(shape[0], -1))
    if n % 2:
        assert (packed[:, -1] >> 4 == 0).all()


def test_pack_int4_rejects_wide_codes():
    with pytest.raises(ValueError):
        oracle.pack_int4(np.array([[0, 8]], np.int8))
    with pytest.raises(ValueError):
        oracle.pack_int4(np.array([[-9, 0]], np.int8))


def test_dequantize_is_code_times_scale():
    w = synth.generate(synth.TensorSpec(5, 1, (16, 24, 3, 3), "normal", 0.05))
    codes, scales = oracle.quantize(w, 4, MODE_EKC)
    dq = oracle.dequantize(codes, scales)
    want = codes.astype(np.float32) * scales[:, None, None, None]
    assert dq.dtype == np.float32 and np.array_equal(dq.view(np.uint32), want.view(np.uint32))
    # every code is within one step of nearest rounding: |w - dq| < s (plus division rounding)
    err = np.abs(dq.astype(np.float64) - w.astype(np.float64))
    assert (err <= scales.astype(np.float64)[:, None, None, None] * (1 + 1e-6)).all()
    # and nearest rounding alone stays within s/2
    ce, _ = oracle.quantize(w, 4, oracle.MODE_E)
    err_e = np.abs(oracle.dequantize(ce, scales).astype(np.float64) - w.astype(np.float64))
    assert (err_e <= 0.5 * scales.astype(np.float64)[:, None, None, None] * (1 + 1e-6)).all()


def test_widen_f16_all_patterns_against_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.widen(bits, "f16")
    want = bits.view(np.float16).astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got.view(np.uint32)[~nan], want.view(np.uint32)[~nan])


def test_widen_bf16_all_patterns_against_bit_shift():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.widen(bits, "bf16")
    want = (bits.astype(np.uint32) << 16).view(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got.view(np.uint32)[~nan], want.view(np.uint32)[~nan])


def test_dequantize_bf16_against_torch_and_tie_cases():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(3)
    codes = rng.integers(-127, 128, (16, 999)).astype(np.int8)
    scales = (rng.random(16) * 0.02 + 1e-5).astype(np.float32)
    got = oracle.dequantize_bf16(codes, scales)
    f32 = oracle.dequantize(codes, scales)
    want = torch.from_numpy(f32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)
    # exact ties: code * scale with scale a power of two is exact, and codes whose low bits
    # end in ...1000 0000 after the 8 kept significand bits sit exactly between two bfloat16
    codes = np.array([[-127, -125, 125, 127, 3, 1, 0, 126, 124]], np.int8)   # 127 = 1111111b: 8 bits fit
    scales = np.array([2.0 ** -9 * (1 + 2.0 ** -8)], np.float32)            # forces 9+ significand bits
    got = oracle.dequantize_bf16(codes, scales)
    want = torch.from_numpy(oracle.dequantize(codes, scales)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)
    # a hand-made tie: 1 + 2^-8 lies exactly between bfloat16 1.0 (even) and 1 + 2^-7
    assert oracle.dequantize_bf16(np.array([[1]], np.int8), np.array([1 + 2.0 ** -8], np.float32))[0, 0] == 0x3F80
    # 1 + 3 * 2^-8 lies between 1 + 2^-7 (odd) and 1 + 2^-6 (even): goes up
    assert oracle.dequantize_bf16(np.array([[1]], np.int8), np.array([1 + 3 * 2.0 ** -8], np.float32))[0, 0] == 0x3F82
    assert oracle.dequantize_bf16(np.array([[-1]], np.int8), np.array([1 + 3 * 2.0 ** -8], np.float32))[0, 0] == 0xBF82
