"""GPU parity of the batch-norm based activation ranges and of the whole-network call."""
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


def bn_params(rng, channels, kind):
    if kind == "typical":
        g = rng.standard_normal(channels) * 0.5 + 1.0
        b = rng.standard_normal(channels) * 0.3
    elif kind == "negative":            # every channel below zero: empty range under a ReLU
        g = np.abs(rng.standard_normal(channels)) * 0.01
        b = -1.0 - np.abs(rng.standard_normal(channels))
    elif kind == "constant":
        g = np.zeros(channels)
        b = np.full(channels, 0.25)
    else:                               # zeros of either sign
        g = np.zeros(channels)
        b = np.where(rng.random(channels) < 0.5, 0.0, -0.0)
    return g.astype(np.float32), b.astype(np.float32)


def same_range(got, want):
    return (np.float32(got[0]).tobytes() == np.float32(want[0]).tobytes() and
            np.float32(got[1]).tobytes() == np.float32(want[1]).tobytes() and
            np.float32(got[2]).tobytes() == np.float32(want[2]).tobytes() and got[3] == want[3])


@pytest.mark.parametrize("bits", [2, 4, 8, 16])
@pytest.mark.parametrize("n_sigma", [0.0, 3.0, 6.0])
def test_activation_ranges_match_reference(sq, bits, n_sigma):
    rng = np.random.default_rng(bits * 10 + int(n_sigma))
    layers, host = [], []
    for channels in (1, 3, 64, 255, 256, 257, 1000, 5000):
        for kind in ("typical", "negative", "constant", "zeros"):
            for relu in (False, True):
                g, b = bn_params(rng, channels, kind)
                host.append((g, b, relu))
                layers.append((torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda(), relu))
    got = sq.squant_activation_ranges(layers, n_sigma, bits)
    assert len(got) == len(host)
    for i, ((g, b, relu), r) in enumerate(zip(host, got)):
        want = oracle.activation_range(g, b, n_sigma, relu, bits)
        assert same_range(r, want), (i, g.size, relu, r, want)


def test_many_layers_in_one_call(sq):
    rng = np.random.default_rng(4)
    host = [bn_params(rng, int(rng.integers(1, 300)), "typical") + (bool(i % 2),) for i in range(600)]
    layers = [(torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda(), r) for g, b, r in host]
    got = sq.squant_activation_ranges(layers, 6.0, 8)
    for (g, b, relu), r in zip(host, got):
        assert same_range(r, oracle.activation_range(g, b, 6.0, relu, 8))


@pytest.mark.parametrize("config", [2, 6])
def test_whole_network_call(sq, config):
    """ResNet-18 / InceptionV3-style weights, a batch norm after every layer but the last: the one
    call gives what the weight solver and the range kernel give separately, i.e. the reference."""
    specs = synth.config_specs(config)
    rng = np.random.default_rng(11)
    layers, host = [], []
    for i, s in enumerate(specs):
        w = synth.generate(s)
        if i == len(specs) - 1:
            bn, hbn = None, None
        else:
            g, b = bn_params(rng, s.shape[0], "typical")
            hbn = (g, b, True)
            bn = (torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda(), True)
        layers.append((torch.from_numpy(w).cuda(), bn))
        host.append((w, hbn))
    codes, scales, ranges = sq.squant_quantize_network(layers, 4, sq.MODE_EKC, 8, 6.0)
    for (w, hbn), c, sc, r in zip(host, codes, scales, ranges):
        want_c, want_s = oracle.quantize(w, 4, 2, threads=8)
        assert np.array_equal(c.cpu().numpy(), want_c)
        assert np.array_equal(sc.cpu().numpy().view(np.uint32), want_s.view(np.uint32))
        if hbn is None:
            assert r is None
        else:
            assert same_range(r, oracle.activation_range(hbn[0], hbn[1], 6.0, hbn[2], 8))
