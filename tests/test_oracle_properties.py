"""Randomised property checks of the CPU oracle (hypothesis): the algebraic identities of the
round hold for any number of workers, dimension and hyper-parameters, not just the hand-picked
cases of test_oracle_pins.py."""
import numpy as np
from hypothesis import given, settings, strategies as st

from parity import O


def _workers(M, d, seed, spread):
    rng = np.random.default_rng(seed)
    return rng.standard_normal(d)[None, :] + spread * rng.standard_normal((M, d))


@settings(max_examples=60, deadline=None, derandomize=True)
@given(M=st.integers(2, 9), d=st.integers(1, 40), seed=st.integers(0, 10_000),
       alpha=st.floats(0.0, 1.0), lam=st.floats(0.0, 3.0), spread=st.floats(1e-3, 10.0))
def test_round_identities(M, d, seed, alpha, lam, spread):
    x = _workers(M, d, seed, spread)
    x_new, r, c, x_avg = O.pull_push_round(x, alpha, lam)
    assert np.allclose(x_avg, x.mean(axis=0), rtol=1e-12, atol=1e-12)
    assert np.allclose(r, np.linalg.norm(x - x_avg, axis=1), rtol=1e-12)
    assert np.all(r > 0)
    # every worker moves along its own gap by |alpha r - lambda| (Sec. 5, Eq. 5)
    step = x_new - x
    assert np.allclose(np.linalg.norm(step, axis=1), np.abs(alpha * r - lam), rtol=1e-9, atol=1e-12)
    gap = x_avg[None] - x
    cross = step * np.linalg.norm(gap, axis=1)[:, None] - gap * (c * r)[:, None]
    assert np.allclose(cross, 0.0, atol=1e-9 * (1 + np.abs(x).max()))
    # appendix, gap dynamics: the average moves by -(lambda/M) sum of unit gap vectors
    u = gap / r[:, None]
    assert np.allclose(x_new.mean(axis=0), x_avg - lam * u.mean(axis=0), rtol=1e-9, atol=1e-10)
    # Alg. 1 in its literal order gives the same point whenever alpha < 1
    if alpha < 0.999:
        seq, r_post = O.pull_then_push(x, x_avg, alpha, lam, "average")
        assert np.allclose(seq, x_new, rtol=1e-7, atol=1e-7 * (1 + np.abs(x).max()))
        assert np.allclose(r_post, (1 - alpha) * r, rtol=1e-9)


@settings(max_examples=40, deadline=None, derandomize=True)
@given(M=st.integers(2, 8), d=st.integers(1, 30), seed=st.integers(0, 10_000),
       alpha=st.floats(0.0, 1.0), lam_r=st.floats(0.0, 5.0))
def test_exact_gradient_preserves_the_average(M, d, seed, alpha, lam_r):
    x = _workers(M, d, seed, 1.0)
    x_new, r, x_avg = O.pull_push_round_exact(x, alpha, lam_r)
    assert np.allclose(x_new.mean(axis=0), x_avg, rtol=1e-10, atol=1e-11)
    # its first term alone is Eq. 5 with lambda = lambda_r / M
    one_term, _, _, _ = O.pull_push_round(x, alpha, lam_r / M)
    u = (x - x_avg) / r[:, None]
    assert np.allclose(x_new - one_term, -(lam_r / M ** 2) * u.sum(axis=0)[None], rtol=1e-8, atol=1e-10)


@settings(max_examples=40, deadline=None, derandomize=True)
@given(M=st.integers(1, 5), d=st.integers(1, 20), seed=st.integers(0, 10_000), steps=st.integers(1, 6),
       lr=st.floats(1e-3, 0.5), mu=st.floats(0.0, 0.99), wd=st.floats(0.0, 0.1))
def test_local_steps_compose_and_fuse(M, d, seed, steps, lr, mu, wd):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, d)); v = np.zeros((M, d))
    gs = rng.standard_normal((steps, M, d))
    for k in range(steps - 1):
        x, v = O.local_sgd_step(x, v, gs[k], lr, mu, wd)
    xa, va = O.local_sgd_step(x, v, gs[-1], lr, mu, wd)
    if M > 1:
        xr, rr, cr, _ = O.pull_push_round(xa, 0.3, 0.2)
        xf, vf, rf, cf, _ = O.dppf_round(x, v, gs[-1], lr, mu, wd, 0.3, 0.2)
        assert np.array_equal(xf, xr) and np.array_equal(vf, va) and np.array_equal(rf, rr)
    # with weight decay the step is plain SGD on the loss plus (wd/2)|x|^2
    x2, v2 = O.local_sgd_step(x, v, gs[-1] + wd * x, lr, mu, 0.0)
    assert np.allclose(x2, xa, rtol=1e-12, atol=1e-12) and np.allclose(v2, va, rtol=1e-12, atol=1e-12)
