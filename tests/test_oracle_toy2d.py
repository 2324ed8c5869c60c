"""The 2-D illustration of the paper with the oracle as the population update: separately trained
models and PAPA stay in the local minima near (3,8) / (8,3), WASH brings the population to the
global minimum (10,10) (appendix and the toy figure; qualitative, the noise level is ours)."""
import numpy as np

import oracle
import toy2d


def _wash(seed):
    def update(pop, t):
        oracle.shuffle(pop, None, [(0, 2, 0.01)], seed, t)
    return update


def _papa(pop, t):
    oracle.ema(pop, 0.99)


def test_wash_reaches_the_global_minimum_where_baseline_and_papa_do_not():
    seeds = range(8)
    base = [toy2d.distance_of_average_to_global_minimum(toy2d.run(lambda pop, t: None, s)) for s in seeds]
    papa = [toy2d.distance_of_average_to_global_minimum(toy2d.run(_papa, s)) for s in seeds]
    wash = [toy2d.distance_of_average_to_global_minimum(toy2d.run(_wash(s), s)) for s in seeds]
    assert min(base) > 5.0 and min(papa) > 5.0                 # both stay around the local minima
    assert sum(d < 1.0 for d in wash) >= 6                     # WASH: average at (10,10) in most runs
    assert np.mean(wash) < 0.5 * np.mean(base)


def test_without_noise_every_run_ends_at_the_global_minimum():
    end = toy2d.run(_wash(3), 3, sigma=0.0)
    assert np.all(np.abs(end - 10.0) < 0.1)
    sep = toy2d.run(lambda pop, t: None, 3, sigma=0.0)
    assert np.allclose(sep, [[3.05, 8.0], [8.0, 3.05]], atol=0.05)
