"""Exhaustive flip search on tiny problems: the reference solver must attain the optimum.

SQuant composes its sub-problems lexicographically (Section 3.3 "Relaxation" and "CASE
Flipping"): first the absolute sum of error of the group is made minimal, then, among the
flip sets that achieve it, the element perturbations are kept smallest.  The search below
does not assume the sign restriction or the top-k rule: it tries every subset of one-step
flips of either direction, so both are derived here, not presupposed (App. B.1, B.2).
"""
import zlib

import numpy as np
import pytest

import oracle
from oracle import HALF, ONE, MODE_E, MODE_EK, MODE_EKC


def seed_of(*parts):
    return zlib.crc32(repr(parts).encode())


def all_subset_masks(K):
    m = np.arange(1 << K, dtype=np.int64)
    return ((m[:, None] >> np.arange(K)[None, :]) & 1).astype(np.int64)   # [2^K, K]


def kernel_bruteforce(P):
    """P: [B, K] Q23 perturbations after rounding.  Lexicographic optimum (|sum|, sum sq)."""
    B, K = P.shape
    masks = all_subset_masks(K)                                  # [S, K]
    step = np.sign(P).astype(np.int64) * ONE                      # flipping i moves P_i by -step_i
    flippable = (P != 0).astype(np.int64)
    best_abs = np.full(B, np.iinfo(np.int64).max)
    best_sq = np.full(B, np.inf)
    for b0 in range(0, B, 256):
        p = P[b0:b0 + 256].astype(np.int64)[:, None, :]           # [b,1,K]
        valid = ((masks[None] & (1 - flippable[b0:b0 + 256][:, None, :])).sum(-1) == 0)
        newp = p - masks[None] * step[b0:b0 + 256][:, None, :]
        a = np.abs(newp.sum(-1))
        sq = (newp.astype(np.float64) ** 2).sum(-1)
        a = np.where(valid, a, np.iinfo(np.int64).max)
        amin = a.min(axis=1)
        sq = np.where(a == amin[:, None], sq, np.inf)
        best_abs[b0:b0 + 256] = amin
        best_sq[b0:b0 + 256] = sq.min(axis=1)
    return best_abs, best_sq


def make_weights(rng, shape, kind):
    if kind == "normal":
        return (rng.standard_normal(shape) * 0.05).astype(np.float32)
    if kind == "heavy":
        return (rng.standard_t(3, shape) * 0.05).astype(np.float32)
    if kind == "grid":     # coarse grid: many equal |p|, exact halves and exact zero sums
        w = rng.integers(-28, 29, shape).astype(np.float32) / 4.0
        w[:, 0, 0, 0] = 7.0                                        # scale exactly 1 at 4 bits
        return w
    raise ValueError(kind)


@pytest.mark.parametrize("kind", ["normal", "heavy", "grid"])
@pytest.mark.parametrize("khw", [(3, 3), (2, 2), (1, 5), (3, 4), (1, 1), (1, 2)])
def test_kernel_stage_attains_exhaustive_optimum(kind, khw):
    rng = np.random.default_rng(seed_of(kind, khw))
    kh, kw = khw
    K = kh * kw
    w = make_weights(rng, (24, 20, kh, kw), kind)
    _, _, te = oracle.quantize_trace(w, 4, MODE_E)
    _, _, tk = oracle.quantize_trace(w, 4, MODE_EK)
    P0 = te["perturbation"].reshape(-1, K)
    P1 = tk["perturbation"].reshape(-1, K).astype(np.int64)
    want_abs, want_sq = kernel_bruteforce(P0)
    got_abs = np.abs(P1.sum(-1))
    got_sq = (P1.astype(np.float64) ** 2).sum(-1)
    assert (got_abs == want_abs).all()
    np.testing.assert_allclose(got_sq, want_sq, rtol=0, atol=0)
    # the solver's own bookkeeping agrees with the recomputed sums
    assert (tk["kernel_sum"].reshape(-1) == P1.sum(-1)).all()
    # Eq. (6): every SQuanted kernel has |sum| <= 0.5
    assert got_abs.max() <= HALF
    # uniqueness of k (App. B.1, second proof): k-1 or k+1 flips miss the bound
    k = tk["kernel_k"].reshape(-1).astype(np.int64)
    a0 = np.abs(P0.astype(np.int64).sum(-1))
    assert (np.abs(a0 - (k - 1) * ONE)[k > 0] > HALF).all()
    assert (np.abs(a0 - (k + 1) * ONE) >= HALF).all()      # equality only on an exact half
    # k <= round(0.5 a) <= K/2 where a = number of same-sign elements (App. B.1, B.4)
    sgn = np.sign(P0.astype(np.int64).sum(-1))
    a_same = (np.sign(P0) == sgn[:, None]).sum(-1)
    assert (k <= a_same // 2).all() and (k <= K // 2).all()
    if K == 9:
        assert k.max() <= 4


def channel_bruteforce(V, EC):
    """Restricted search of the channel stage: one candidate element per kernel, only
    kernels whose candidate has the sign of the channel sum (Section 3.3: 'we can only
    flip one element for a kernel'; App. B.1: same-sign, single-step flips only).
    Optimum in the order: smallest |EC - sgn*|S|*ONE| (Eq. 7); fewest flips when an exact
    half leaves two counts equally good (the (-0.5, 0.5] convention of App. B.3); then the
    largest sum of |V| over the flipped kernels (Eq. (topk1), extended to SQuant-C as
    App. B.2 says).  An unrestricted search over sum of squares is NOT asserted: flipping an
    over-SQuanted candidate back lowers its element perturbation, so on an exact half one more
    flip could lower the sum of squares while breaking the kernel's own bound."""
    sgn = int(np.sign(EC))
    elig = [n for n in range(len(V)) if sgn != 0 and np.sign(V[n]) == sgn]
    best = (abs(int(EC)), 0, 0)
    for m in range(1 << len(elig)):
        S = [elig[j] for j in range(len(elig)) if (m >> j) & 1]
        a = abs(int(EC) - sgn * len(S) * ONE)
        cand = (a, len(S), -int(sum(abs(int(V[n])) for n in S)))
        if cand < best:
            best = cand
    return best


@pytest.mark.parametrize("kind", ["normal", "heavy", "grid"])
@pytest.mark.parametrize("shape", [(40, 12, 3, 3), (40, 10, 1, 1), (30, 7, 2, 2), (30, 12, 1, 3)])
def test_channel_stage_attains_restricted_optimum(kind, shape):
    rng = np.random.default_rng(seed_of(kind, shape))
    w = make_weights(rng, shape, kind)
    M, N, kh, kw = shape
    K = kh * kw
    ck, _, tk = oracle.quantize_trace(w, 4, MODE_EK)
    cc, _, tc = oracle.quantize_trace(w, 4, MODE_EKC)
    ck = ck.reshape(M, N, K).astype(int)
    cc = cc.reshape(M, N, K).astype(int)
    n_flipped_channels = 0
    for m in range(M):
        EC = int(tk["perturbation"][m].astype(np.int64).sum())
        assert EC == int(tc["channel_sum"][m])
        V = tk["cand_value"][m]
        idx = tk["cand_index"][m]
        changed = np.argwhere(ck[m] != cc[m])
        S = []
        for n, i in changed:
            assert i == idx[n]                          # only the kernel's candidate moves
            assert cc[m, n, i] - ck[m, n, i] == -np.sign(V[n])
            S.append(n)
        assert len(set(S)) == len(S)                    # at most one element per kernel
        sgn = int(np.sign(EC))
        got = (abs(EC - sgn * len(S) * ONE), len(S), -int(sum(abs(int(V[n])) for n in S)))
        assert got == channel_bruteforce(V, EC)
        # ties: among equal |V| the lowest kernel index is taken first
        if S:
            thr = min(abs(int(V[n])) for n in S)
            for n in range(N):
                if np.sign(V[n]) == sgn and n not in S:
                    assert abs(int(V[n])) <= thr
                    if abs(int(V[n])) == thr:
                        assert n > max(q for q in S if abs(int(V[q])) == thr)
            n_flipped_channels += 1
    assert n_flipped_channels > 0


@pytest.mark.parametrize("kind", ["normal", "heavy", "grid"])
def test_candidate_is_defined_by_rank_properties(kind):
    """Algorithm 3 restated without sorting: over SQuant -> among the flipped elements the
    one with the smallest pre-flip |p| (highest index on ties = last in rank order); under
    SQuant -> among the un-flipped elements with the sign of the kernel sum the largest |p|
    (lowest index on ties)."""
    rng = np.random.default_rng(77)
    w = make_weights(rng, (16, 24, 3, 3), kind)
    ce, _, te = oracle.quantize_trace(w, 4, MODE_E)
    ck, _, tk = oracle.quantize_trace(w, 4, MODE_EK)
    P0 = te["perturbation"].astype(np.int64)
    P1 = tk["perturbation"].astype(np.int64)
    ce = ce.reshape(P0.shape).astype(int)
    ck = ck.reshape(P0.shape).astype(int)
    seen = {"over": 0, "under": 0, "zero": 0, "none": 0}
    for m in range(P0.shape[0]):
        for n in range(P0.shape[1]):
            e0 = int(P0[m, n].sum())
            sgn = int(np.sign(e0))
            k = int(tk["kernel_k"][m, n])
            flipped = np.flatnonzero(ce[m, n] != ck[m, n])
            assert len(flipped) == k
            ci, cv = int(tk["cand_index"][m, n]), int(tk["cand_value"][m, n])
            if sgn == 0:
                mags = np.abs(P1[m, n])
                want = int(np.argmax(mags)) if mags.max() > 0 else -1
                seen["zero"] += 1
            elif k * ONE > abs(e0):
                mags = np.abs(P0[m, n][flipped])
                ties = flipped[mags == mags.min()]
                want = int(ties.max())
                assert HALF <= abs(int(P1[m, n, want])) < ONE + 1
                seen["over"] += 1
            else:
                rest = [i for i in range(9) if i not in flipped and np.sign(P0[m, n, i]) == sgn]
                if rest:
                    mags = np.array([abs(int(P0[m, n, i])) for i in rest])
                    want = rest[int(np.argmax(mags))]
                    assert abs(int(P1[m, n, want])) <= HALF
                    seen["under"] += 1
                else:
                    want = -1
                    seen["none"] += 1
            assert ci == want
            assert cv == (int(P1[m, n, want]) if want >= 0 else 0)
            if want >= 0 and cv != 0:
                # flipping the candidate moves the kernel sum into [0.5, 1.0]
                after = abs(int(P1[m, n].sum()) - int(np.sign(cv)) * ONE)
                assert HALF <= after <= ONE
    assert seen["over"] > 0 and seen["under"] > 0


@pytest.mark.parametrize("shape", [(12, 300, 1, 1), (12, 40, 7, 7), (6, 150, 3, 3)])
def test_tie_order_in_large_groups(shape):
    """Lowest index first among equal perturbations, on groups too large for the exhaustive
    search (many equal |p| on a coarse grid)."""
    rng = np.random.default_rng(seed_of("ties", shape))
    w = make_weights(rng, shape, "grid")
    M, N, kh, kw = shape
    K = kh * kw
    ce, _, te = oracle.quantize_trace(w, 4, MODE_E)
    ck, _, tk = oracle.quantize_trace(w, 4, MODE_EK)
    cc, _, _ = oracle.quantize_trace(w, 4, MODE_EKC)
    P0 = te["perturbation"].astype(np.int64)
    ce, ck, cc = (a.reshape(M, N, K).astype(int) for a in (ce, ck, cc))
    tie_seen = 0
    for m in range(M):
        for n in range(N):
            fl = np.flatnonzero(ce[m, n] != ck[m, n])
            if len(fl) == 0:
                continue
            sgn = np.sign(P0[m, n].sum())
            thr = np.abs(P0[m, n][fl]).min()
            last_tied = max(i for i in fl if abs(P0[m, n, i]) == thr)
            for i in range(K):
                if i not in fl and np.sign(P0[m, n, i]) == sgn:
                    assert abs(P0[m, n, i]) <= thr
                    if abs(P0[m, n, i]) == thr:
                        assert i > last_tied
                        tie_seen += 1
        V = tk["cand_value"][m].astype(np.int64)
        S = np.flatnonzero((ck[m] != cc[m]).any(-1))
        if len(S):
            sgn = np.sign(tk["channel_sum"][m])
            thr = np.abs(V[S]).min()
            last_tied = max(n for n in S if abs(V[n]) == thr)
            for n in range(N):
                if n not in S and np.sign(V[n]) == sgn:
                    assert abs(V[n]) <= thr
                    if abs(V[n]) == thr:
                        assert n > last_tied
                        tie_seen += 1
    assert tie_seen > 0


# ---- mode E&C (Section 4.3 ablation: SQuant-C straight after rounding) ----
#
# Reading pinned here: the kernel stage flips nothing, the perturbation update of Algorithm 3
# is taken with k = 0, i.e. every kernel offers its largest-|p| element among those with the
# sign of the kernel's own sum (either sign when that sum is exactly 0), and SQuant-C then
# ranks the kernels whose candidate has the sign of the channel sum.  A channel can run out of
# such kernels; Eq. (7) is then missed by whole steps and the test says by how many.

def ec_candidate_without_sorting(P):
    """P: [K] Q23 perturbations of one rounded kernel -> (index, value) or (-1, 0)."""
    e = int(P.astype(np.int64).sum())
    mags = np.abs(P.astype(np.int64))
    if e != 0:
        mags = np.where(np.sign(P) == np.sign(e), mags, 0)
    if mags.max() == 0:
        return -1, 0
    i = int(np.flatnonzero(mags == mags.max())[0])      # lowest index among the largest
    return i, int(P[i])


def test_mode_ec_hand_example():
    """Two 1x3 kernels, scale exactly 1 (one element equals qmax = 7 at 4 bits).
    kernel 0: x = (7, .4, .3)    -> codes (7,0,0), p = (0, -.4, -.3),   sum -.7
    kernel 1: x = (.45, .2, -.1) -> codes (0,0,0), p = (-.45, -.2, +.1), sum -.55
    channel sum -1.25 -> one flip towards +; candidates are -.4 (kernel 0, index 1) and -.45
    (kernel 1, index 0); the larger one flips: kernel 1 element 0 goes from 0 to 1."""
    w = np.array([[[7.0, 0.4, 0.3], [0.45, 0.2, -0.1]]], np.float32).reshape(1, 2, 1, 3)
    codes, scales, tr = oracle.quantize_trace(w, 4, oracle.MODE_EC)
    assert scales[0] == np.float32(1.0)
    assert tr["kernel_k"].tolist() == [[0, 0]]
    assert tr["cand_index"].tolist() == [[1, 0]]
    assert tr["cand_value"][0, 0] == -int(round(float(np.float32(0.4)) * ONE))
    assert tr["cand_value"][0, 1] == -int(round(float(np.float32(0.45)) * ONE))
    assert int(tr["channel_k"][0]) == 1
    assert codes.reshape(2, 3).tolist() == [[7, 0, 0], [1, 0, 0]]
    # with the kernel stage in between the answer is another one: kernel 0 (-.7) and kernel 1
    # (-.55) each flip their largest element, the channel sum becomes +.75 and SQuant-C takes
    # back the flip whose post-flip perturbation is larger (+.6 in kernel 0 against +.55)
    codes_ekc, _ = oracle.quantize(w, 4, MODE_EKC)
    assert codes_ekc.reshape(2, 3).tolist() == [[7, 0, 0], [1, 0, 0]]
    codes_ek, _ = oracle.quantize(w, 4, MODE_EK)
    assert codes_ek.reshape(2, 3).tolist() == [[7, 1, 0], [1, 0, 0]]


@pytest.mark.parametrize("kind", ["normal", "heavy", "grid"])
@pytest.mark.parametrize("shape", [(40, 12, 3, 3), (30, 7, 2, 2), (30, 12, 1, 3), (20, 9, 1, 5)])
def test_mode_ec_candidates_and_restricted_optimum(kind, shape):
    rng = np.random.default_rng(seed_of("ec", kind, shape))
    w = make_weights(rng, shape, kind)
    M, N, kh, kw = shape
    K = kh * kw
    ce, _, te = oracle.quantize_trace(w, 4, MODE_E)
    cc, _, tc = oracle.quantize_trace(w, 4, oracle.MODE_EC)
    ce = ce.reshape(M, N, K).astype(int)
    cc = cc.reshape(M, N, K).astype(int)
    P0 = te["perturbation"]
    # no kernel-stage flip: the perturbations SQuant-C sees are those of plain rounding
    assert (tc["kernel_k"] == 0).all()
    assert (tc["perturbation"] == P0).all()
    assert (tc["kernel_sum"].astype(np.int64) == P0.astype(np.int64).sum(-1)).all()
    seen = {"same": 0, "zero": 0, "none": 0, "short": 0, "flipped": 0}
    for m in range(M):
        for n in range(N):
            want_i, want_v = ec_candidate_without_sorting(P0[m, n])
            assert int(tc["cand_index"][m, n]) == want_i
            assert int(tc["cand_value"][m, n]) == want_v
            e = int(P0[m, n].astype(np.int64).sum())
            seen["none" if want_i < 0 else ("zero" if e == 0 else "same")] += 1
        EC = int(P0[m].astype(np.int64).sum())
        assert EC == int(tc["channel_sum"][m])
        V, idx = tc["cand_value"][m], tc["cand_index"][m]
        changed = np.argwhere(ce[m] != cc[m])
        S = []
        for n, i in changed:
            assert i == idx[n]
            assert cc[m, n, i] - ce[m, n, i] == -np.sign(V[n]) == -np.sign(EC)
            S.append(int(n))
        assert len(set(S)) == len(S)
        sgn = int(np.sign(EC))
        got = (abs(EC - sgn * len(S) * ONE), len(S), -int(sum(abs(int(V[n])) for n in S)))
        assert got == channel_bruteforce(V, EC)
        want_k = int(tc["channel_k"][m])
        elig = int((np.sign(V) == sgn).sum()) if sgn else 0
        assert len(S) == min(want_k, elig)
        if elig < want_k:
            seen["short"] += 1                         # Eq. (7) missed by want_k - elig steps
        else:
            assert got[0] <= HALF
        if S:
            seen["flipped"] += 1
            thr = min(abs(int(V[n])) for n in S)
            for n in range(N):
                if np.sign(V[n]) == sgn and n not in S:
                    assert abs(int(V[n])) <= thr
                    if abs(int(V[n])) == thr:
                        assert n > max(q for q in S if abs(int(V[q])) == thr)
    assert seen["same"] > 0 and seen["flipped"] > 0
    if kind == "grid":
        assert seen["zero"] > 0


def test_mode_ec_tie_and_running_out_of_candidates():
    """Hand cases at scale exactly 1 (one element equals qmax = 7 at 4 bits)."""
    #            x             p               kernel sum   candidate
    # kernel 0: (7, .3)      -> (0, -.3)       -.3          -.3  (index 1)
    # kernel 1: (-.45, .35)  -> (+.45, -.35)   +.1          +.45 (index 0)
    # kernel 2: (-.4, -.45)  -> (+.4, +.45)    +.85         +.45 (index 1)
    # kernel 3: (-.2, .3)    -> (+.2, -.3)     -.1          -.3  (index 1)
    # channel sum +.55 -> one flip towards -; kernels 1 and 2 tie at .45: the lower kernel goes
    w = np.array([[[7.0, 0.3], [-0.45, 0.35], [-0.4, -0.45], [-0.2, 0.3]]], np.float32)
    codes, _, tr = oracle.quantize_trace(w.reshape(1, 4, 1, 2), 4, oracle.MODE_EC)
    assert tr["cand_index"].tolist() == [[1, 0, 1, 1]]
    assert np.sign(tr["cand_value"]).tolist() == [[-1, 1, 1, -1]]
    assert int(tr["cand_value"][0, 1]) == int(tr["cand_value"][0, 2])
    assert int(tr["channel_k"][0]) == 1
    assert codes.reshape(4, 2).tolist() == [[7, 0], [-1, 0], [0, 0], [0, 0]]
    # running out: one kernel carries the whole sum +1.8, two flips are wanted, the kernel offers
    # one candidate, so one element flips and the channel is left at +.8 (Eq. 7 missed)
    w4 = np.array([[[7.0, 0.0, 0.0, 0.0], [-0.45, -0.45, -0.45, -0.45]]], np.float32)
    codes4, _, tr4 = oracle.quantize_trace(w4.reshape(1, 2, 1, 4), 4, oracle.MODE_EC)
    assert int(tr4["channel_k"][0]) == 2
    assert codes4.reshape(2, 4).tolist() == [[7, 0, 0, 0], [-1, 0, 0, 0]]
    assert abs(int(tr4["channel_sum"][0]) - ONE) > HALF
    # the full method on the same channel flips two elements inside the kernel and ends at -.2
    codes5, _ = oracle.quantize(w4.reshape(1, 2, 1, 4), 4, MODE_EKC)
    assert codes5.reshape(2, 4).tolist() == [[7, 0, 0, 0], [-1, -1, 0, 0]]
