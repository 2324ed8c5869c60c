"""The paper's 2-D illustration (appendix, "2D optimization example"), restated: two models
start at (0,5) and (5,0) on f(x,y) = -10 g(10,10,0.1) - 5 g(8,3,0.3) - 5 g(3,8,0.3) with
g(x,y;xm,ym,lam) = exp(-lam sqrt(0.5((x-xm)^2 + (y-ym)^2))), noisy gradient descent with learning
rate 0.1 for 1000 steps; PAPA uses alpha = 0.99, WASH p = 0.01 on both coordinates.  The paper does
not give the noise level: SIGMA below is this repository's reading.  Helper for two tests, no
arithmetic of the method lives here (the population update is passed in as `update`)."""
import numpy as np

SIGMA = 0.25
MINIMA = ((10.0, 10.0, 10.0, 0.1), (5.0, 8.0, 3.0, 0.3), (5.0, 3.0, 8.0, 0.3))   # weight, xm, ym, lambda


def grad(x, y):
    gx = gy = 0.0
    for c, xm, ym, lam in MINIMA:
        r = np.sqrt(0.5 * ((x - xm) ** 2 + (y - ym) ** 2))
        if r > 1e-12:
            e = c * lam * np.exp(-lam * r) * 0.5 / r
            gx += e * (x - xm)
            gy += e * (y - ym)
    return np.array([gx, gy])


def run(update, seed, steps=1000, lr=0.1, sigma=SIGMA):
    """update(pop, step) applies the population update in place on a float32 [2, 2] array (or returns
    a new one); returns the final population."""
    rng = np.random.default_rng(seed)
    pop = np.array([[0.0, 5.0], [5.0, 0.0]], dtype=np.float32)
    for t in range(steps):
        for n in range(2):
            g = grad(float(pop[n, 0]), float(pop[n, 1])) + sigma * rng.standard_normal(2)
            pop[n] = (pop[n].astype(np.float64) - lr * g).astype(np.float32)
        new = update(pop, t)
        if new is not None:
            pop = new
    return pop


def distance_of_average_to_global_minimum(pop):
    return float(np.hypot(*(pop.mean(axis=0) - 10.0)))
