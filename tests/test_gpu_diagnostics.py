"""GPU parity for the two analysis passes: distance to the consensus (Eq. 2 /
Eq. 5 quantity) and weighted average.  The weighted average sums in the order
of the definition and must equal the oracle bit for bit.  The distance is a sum
of P non-negative fp64 terms reduced in a tree, the oracle sums them one after
another: both carry a relative rounding error of at most about sqrt(P) * 2^-53
(random-walk growth; below 1e-11 even for 1e9 terms), so the test allows 1e-10."""
import numpy as np
import pytest

import oracle
from workloads import device_population, get_config

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def wash():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2405_17517_amd as w
    return w


@pytest.mark.parametrize("N,P", [(1, 7), (2, 1023), (3, 4096), (5, 100003), (10, 300001), (20, 70002), (32, 4099)])
def test_sqdist_and_weighted_average_small(wash, N, P):
    print(f"case N={N} P={P}", flush=True)
    rng = np.random.default_rng(N * 7 + P % 97)
    pop = (rng.standard_normal((N, P)) * 0.02).astype(np.float32)
    d = torch.from_numpy(pop).cuda()
    for a, b in [(0, P), (0, 0), (P // 3, P // 3 + 1), (min(1, P), P - 1), (max(0, P // 2 - 5), P)]:
        got = wash.wash_consensus_sqdist(d, a, b).cpu().numpy()
        ref = oracle.consensus_sqdist(pop, a, b)
        assert np.allclose(got, ref, rtol=1e-10, atol=0), (a, b)
        again = wash.wash_consensus_sqdist(d, a, b).cpu().numpy()
        assert np.array_equal(got, again)                       # fixed reduction shape: reproducible bits
    w = rng.random(N)
    w /= w.sum()
    got = wash.wash_weighted_average(d, list(w)).cpu().numpy()
    assert np.array_equal(got, oracle.weighted_average(pop, w))
    onehot = [0.0] * N
    onehot[N // 2] = 1.0
    assert np.array_equal(wash.wash_weighted_average(d, onehot).cpu().numpy(), pop[N // 2])


def test_eq2_and_eq5_on_device(wash):
    # the EMA contracts every model's squared distance by alpha^2 (Eq. 2); the shuffle keeps the total (Eq. 5)
    N, P = 8, 1_000_003
    rng = np.random.default_rng(3)
    pop = rng.standard_normal((N, P)).astype(np.float32)
    d = torch.from_numpy(pop).cuda()
    d0 = wash.wash_consensus_sqdist(d).cpu().numpy()
    wash.wash_shuffle(d, None, [(0, P, 0.2)], 5, 0)
    d1 = wash.wash_consensus_sqdist(d).cpu().numpy()
    assert abs(d1.sum() - d0.sum()) <= 1e-10 * d0.sum()
    wash.papa_ema(d, 0.9)
    d2 = wash.wash_consensus_sqdist(d).cpu().numpy()
    al = float(np.float32(0.9))
    assert np.allclose(d2, al * al * d1, rtol=1e-5)


@pytest.mark.parametrize("index", [2, 3, 4])
def test_full_size_configs(wash, index):
    cfg = get_config(index)
    pop, _ = device_population(cfg.tensors(), cfg.N, cfg.init, cfg.data_seed, False)
    host = pop.cpu().numpy()
    P = cfg.P
    for a, b in [(0, P), (P // 4, P // 2)]:                     # whole vector and the second quarter
        got = wash.wash_consensus_sqdist(pop, a, b).cpu().numpy()
        ref = oracle.consensus_sqdist(host, a, b)
        assert np.allclose(got, ref, rtol=1e-10, atol=0)
    w = np.linspace(1.0, 2.0, cfg.N)
    w /= w.sum()
    got = wash.wash_weighted_average(pop, list(w)).cpu().numpy()
    assert np.array_equal(got, oracle.weighted_average(host, w))


def test_errors(wash):
    d = torch.zeros((2, 100), dtype=torch.float32, device="cuda")
    with pytest.raises(wash.WashError):
        wash.wash_consensus_sqdist(d, 50, 20)
    with pytest.raises(wash.WashError):
        wash.wash_consensus_sqdist(d, 0, 101)
    with pytest.raises(wash.WashError):
        wash.wash_weighted_average(d, [0.5, float("inf")])
    with pytest.raises(TypeError):
        wash.wash_weighted_average(d, [1.0])
