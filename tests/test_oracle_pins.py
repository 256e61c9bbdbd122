"""Pins of the CPU reference solver against what the paper prints and what numpy fixes.

Hand-built channels use the trick that a channel holding one element equal to
+-qmax has scale exactly 1.0, so the scaled weight x equals the stored weight.
"""
import numpy as np
import pytest

import oracle
from oracle import HALF, ONE, MODE_E, MODE_EK, MODE_EKC, MODE_EC

Q = float(ONE)


def channel_with_unit_scale(kernels, bits=4):
    """One output channel [1, N+1, K]: the given kernels plus one that carries qmax."""
    qmax = (1 << (bits - 1)) - 1
    K = len(kernels[0])
    anchor = [float(qmax)] + [0.0] * (K - 1)
    w = np.array([list(k) for k in kernels] + [anchor], dtype=np.float32)[None, :, :]
    return w  # [1, N+1, K]


def test_scale_is_one_for_anchor_channel():
    w = channel_with_unit_scale([[0.7, 0.4, 0.0]])
    _, s = oracle.quantize(w, 4, MODE_E)
    assert s[0] == np.float32(1.0)


# ---- App. B.1 figure: sign convention of the perturbation and one flip each way ----
def test_flip_figure_values():
    # kernel A = three 0.7 (sum of perturbations +0.9 -> one flip down),
    # kernel B = two 0.4 (sum -0.8 -> one flip up)
    w = channel_with_unit_scale([[0.7, 0.7, 0.7], [0.4, 0.4, 0.0]])
    ce, _, te = oracle.quantize_trace(w, 4, MODE_E)
    assert ce[0, 0].ravel().tolist() == [1, 1, 1]           # 0.7 rounds up to 1
    assert ce[0, 1].ravel().tolist() == [0, 0, 0]           # 0.4 rounds down to 0
    np.testing.assert_allclose(te["perturbation"][0, 0] / Q, [0.3, 0.3, 0.3], atol=1e-6)
    np.testing.assert_allclose(te["perturbation"][0, 1] / Q, [-0.4, -0.4, 0.0], atol=1e-6)
    ck, _, tk = oracle.quantize_trace(w, 4, MODE_EK)
    assert ck[0, 0].ravel().tolist() == [0, 1, 1]           # -1 mutation, lowest index on a tie
    assert ck[0, 1].ravel().tolist() == [1, 0, 0]           # +1 mutation
    np.testing.assert_allclose(tk["perturbation"][0, 0] / Q, [-0.7, 0.3, 0.3], atol=1e-6)
    np.testing.assert_allclose(tk["perturbation"][0, 1] / Q, [0.6, -0.4, 0.0], atol=1e-6)
    # a flipped perturbation lies in [0.5, 1.0)
    assert 0.5 <= abs(tk["perturbation"][0, 0, 0]) / Q < 1.0
    assert 0.5 <= abs(tk["perturbation"][0, 1, 0]) / Q < 1.0


# ---- App. B.1 proof: a sum of 3.2 flips exactly three positive perturbations ----
def test_sum_3p2_flips_three():
    w = channel_with_unit_scale([[0.6] * 8])
    ce, _, te = oracle.quantize_trace(w, 4, MODE_E)
    assert abs(te["perturbation"][0, 0].sum() / Q - 3.2) < 1e-5
    ck, _, tk = oracle.quantize_trace(w, 4, MODE_EK)
    assert tk["kernel_k"][0, 0] == 3
    diff = ck[0, 0].ravel().astype(int) - ce[0, 0].ravel().astype(int)
    assert diff.tolist() == [-1, -1, -1, 0, 0, 0, 0, 0]     # -3.0 mutation in total
    assert abs(tk["kernel_sum"][0, 0] / Q - 0.2) < 1e-5


# ---- App. B.3 "Over SQuant": e = +1.6, {2.6, 2.7} -> {2, 2}, candidate 2.7 ----
def test_over_squant_worked_example():
    k_over = [2.6, 2.7, 0.75, 0.75, 0.8, 0.8]      # perturbations .4 .3 .25 .25 .2 .2 = +1.6
    k_neg = [0.4, 0.0, 0.0, 0.0, 0.0, 0.0]         # perturbation -0.4
    w = channel_with_unit_scale([k_over, k_neg])
    ce, _, te = oracle.quantize_trace(w, 4, MODE_E)
    assert abs(te["perturbation"][0, 0].sum() / Q - 1.6) < 1e-5
    ck, _, tk = oracle.quantize_trace(w, 4, MODE_EK)
    assert tk["kernel_k"][0, 0] == 2
    assert ck[0, 0].ravel().tolist() == [2, 2, 1, 1, 1, 1]
    assert abs(tk["kernel_sum"][0, 0] / Q - (-0.4)) < 1e-5          # inside (-0.5, 0.5]
    assert tk["cand_index"][0, 0] == 1                              # the element 2.7
    assert abs(tk["cand_value"][0, 0] / Q - (-0.7)) < 1e-5          # post-flip, 0.5 <= |v| < 1
    # the channel sum is -0.4 - 0.4 = -0.8 -> one channel-wise flip; the over-SQuanted
    # kernel's candidate (|v| = 0.7) outranks the other kernel's (|v| = 0.4)
    cc, _, tc = oracle.quantize_trace(w, 4, MODE_EKC)
    assert tc["channel_k"][0] == 1
    assert cc[0, 0].ravel().tolist() == [2, 3, 1, 1, 1, 1]          # 2.7 is back at 3
    assert cc[0, 1].ravel().tolist() == ck[0, 1].ravel().tolist()
    # kernel sum after the flip back: +0.6
    x = w[0, 0].ravel().astype(np.float64)
    assert abs((cc[0, 0].ravel() - x).sum() - 0.6) < 1e-5


# ---- App. B.3 "Under SQuant": candidate = first un-flipped same-sign element ----
def test_under_squant_candidate():
    k_under = [0.55, 0.6, 0.65, 0.85, 0.1, 0.0]    # perturbations .45 .4 .35 .15 -.1 0 = +1.25
    w = channel_with_unit_scale([k_under])
    ck, _, tk = oracle.quantize_trace(w, 4, MODE_EK)
    assert tk["kernel_k"][0, 0] == 1
    assert ck[0, 0].ravel().tolist() == [0, 1, 1, 1, 0, 0]          # largest (+.45) flipped
    assert abs(tk["kernel_sum"][0, 0] / Q - 0.25) < 1e-5
    assert tk["cand_index"][0, 0] == 1                              # next largest (+.4)
    assert abs(tk["cand_value"][0, 0] / Q - 0.4) < 1e-5             # |v| <= 0.5
    # flipping the candidate would leave |kernel sum| in (0.5, 1.0)
    after = abs(tk["kernel_sum"][0, 0] - np.sign(tk["cand_value"][0, 0]) * ONE) / Q
    assert 0.5 < after < 1.0


def test_under_squant_picked_by_channel_stage():
    # three kernels with sums +0.25, +0.3, +0.3 -> channel sum +0.85 -> one flip, taken from
    # the kernel whose candidate has the largest |v| (kernel 2: .3 beats .25 and .2/.1 splits)
    ka = [0.75, 0.0, 0.0]            # +.25 ; candidate value .25
    kb = [0.8, 0.9, 0.0]             # +.2 +.1 = +.3 ; candidate value .2
    kc = [0.7, 0.0, 0.0]             # +.3 ; candidate value .3
    w = channel_with_unit_scale([ka, kb, kc])
    ck, _, tk = oracle.quantize_trace(w, 4, MODE_EK)
    assert tk["kernel_k"][0, :3].tolist() == [0, 0, 0]
    np.testing.assert_allclose(tk["cand_value"][0, :3] / Q, [0.25, 0.2, 0.3], atol=1e-6)
    cc, _, tc = oracle.quantize_trace(w, 4, MODE_EKC)
    assert tc["channel_k"][0] == 1
    assert cc[0, 2].ravel().tolist() == [0, 0, 0] and ck[0, 2].ravel().tolist() == [1, 0, 0]
    assert (cc[0, :2] == ck[0, :2]).all()


# ---- the tie rule of k: an exact half takes the fewer flips ((-0.5, 0.5] for e > 0) ----
def test_half_sum_is_not_flipped():
    w = channel_with_unit_scale([[0.75, 0.75, 0.0], [1.75, 2.75, 3.75]])   # sums +0.5, +0.75
    _, _, tk = oracle.quantize_trace(w, 4, MODE_EK)
    assert tk["kernel_sum"][0, 0] == HALF and tk["kernel_k"][0, 0] == 0
    assert tk["kernel_k"][0, 1] == 1
    w = channel_with_unit_scale([[0.25, 0.25, 0.0]])                       # sum -0.5
    _, _, tk = oracle.quantize_trace(w, 4, MODE_EK)
    assert tk["kernel_sum"][0, 0] == -HALF and tk["kernel_k"][0, 0] == 0
    w = channel_with_unit_scale([[0.75] * 6])                              # sum +1.5 -> 1 flip
    _, _, tk = oracle.quantize_trace(w, 4, MODE_EK)
    assert tk["kernel_k"][0, 0] == 1 and tk["kernel_sum"][0, 0] == HALF


def test_exact_zero_kernel_takes_largest_of_either_sign():
    w = channel_with_unit_scale([[0.25, 0.75, 0.0], [0.0, 0.0, 0.0]])      # -.25 +.25 -> 0
    _, _, tk = oracle.quantize_trace(w, 4, MODE_EK)
    assert tk["kernel_sum"][0, 0] == 0 and tk["kernel_k"][0, 0] == 0
    assert tk["cand_index"][0, 0] == 0 and tk["cand_value"][0, 0] == -(ONE // 4)
    assert tk["cand_index"][0, 1] == -1 and tk["cand_value"][0, 1] == 0    # no candidate


# ---- closed forms: numpy fixes the scale and plain rounding (mode E) ----
@pytest.mark.parametrize("bits", [2, 3, 4, 5, 6, 8])
@pytest.mark.parametrize("shape", [(16, 8, 3, 3), (7, 33, 1, 1), (5, 3, 7, 7), (9, 1, 3, 3)])
def test_scale_and_rounding_match_numpy(bits, shape):
    rng = np.random.default_rng(bits * 1000 + shape[0])
    w = (rng.standard_normal(shape) * 0.05).astype(np.float32)
    w[0] = 0.0                                             # an all-zero channel
    qmax = np.float32((1 << (bits - 1)) - 1)
    codes, scales = oracle.quantize(w, bits, MODE_E)
    amax = np.abs(w).reshape(shape[0], -1).max(axis=1)
    want_s = np.where(amax > 0, amax / qmax, np.float32(1.0)).astype(np.float32)
    assert scales.dtype == np.float32 and (scales == want_s).all()
    x = w / want_s[:, None, None, None]
    want_c = np.rint(np.clip(x, -qmax, qmax)).astype(np.int8)
    assert (codes == want_c).all()
    assert (codes[0] == 0).all() and scales[0] == 1.0
    assert np.abs(codes.astype(int)).max() <= int(qmax)
    # every mode returns the same scales
    for mode in (MODE_EK, MODE_EKC, MODE_EC):
        _, s2 = oracle.quantize(w, bits, mode)
        assert (s2 == want_s).all()


def test_perturbation_is_fixed_point_of_code_minus_x():
    rng = np.random.default_rng(5)
    w = (rng.standard_normal((8, 16, 3, 3)) * 0.05).astype(np.float32)
    codes, scales, tr = oracle.quantize_trace(w, 4, MODE_E)
    x = np.clip(w / scales[:, None, None, None], -7, 7).astype(np.float32)
    p = (codes.astype(np.float32) - x).astype(np.float32)
    # exact in binary32: recomputing in float64 gives the same value
    assert (p.astype(np.float64) == codes.astype(np.float64) - x.astype(np.float64)).all()
    want = np.rint(p.astype(np.float64) * ONE).astype(np.int64).reshape(8, 16, 9)
    assert (tr["perturbation"] == want).all()
    assert np.abs(tr["perturbation"]).max() <= HALF


# ---- FC / 1x1: SQuant-K has nothing to do ----
@pytest.mark.parametrize("bits", [3, 4, 8])
def test_k1_layers_skip_kernel_stage(bits):
    rng = np.random.default_rng(11 + bits)
    w = (rng.standard_normal((32, 96, 1, 1)) * 0.1).astype(np.float32)
    ce, _ = oracle.quantize(w, bits, MODE_E)
    ck, _, tk = oracle.quantize_trace(w, bits, MODE_EK)
    assert (ce == ck).all() and (tk["kernel_k"] == 0).all()
    # and E&C equals E&K&C there
    c1, _ = oracle.quantize(w, bits, MODE_EKC)
    c2, _ = oracle.quantize(w, bits, MODE_EC)
    assert (c1 == c2).all()


def test_depthwise_channel_stage_is_noop():
    rng = np.random.default_rng(3)
    w = rng.standard_normal((64, 1, 3, 3)).astype(np.float32)
    ck, _ = oracle.quantize(w, 4, MODE_EK)
    cc, _, tc = oracle.quantize_trace(w, 4, MODE_EKC)
    assert (ck == cc).all() and (tc["channel_k"] == 0).all()


def test_argument_errors():
    w = np.zeros((2, 2, 1, 1), np.float32)
    for bits in (1, 9, 0, -3):
        with pytest.raises(ValueError):
            oracle.quantize(w, bits)
    with pytest.raises(ValueError):
        oracle.quantize(w, 4, 7)
    L = oracle.lib()
    c = np.zeros(4, np.int8); s = np.zeros(2, np.float32)
    assert L.squant_oracle_quantize(None, 2, 2, 1, 1, 4, 2, c.ctypes.data, s.ctypes.data) == 1
    assert L.squant_oracle_quantize(w.ctypes.data, 0, 2, 1, 1, 4, 2, c.ctypes.data, s.ctypes.data) == 2


def test_threaded_entry_is_identical():
    rng = np.random.default_rng(8)
    w = (rng.standard_normal((37, 20, 3, 3)) * 0.05).astype(np.float32)
    a = oracle.quantize(w, 4, MODE_EKC)
    b = oracle.quantize(w, 4, MODE_EKC, threads=5)
    assert (a[0] == b[0]).all() and (a[1] == b[1]).all()
