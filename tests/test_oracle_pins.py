"""Pins for the CPU oracle: hand-worked fixtures, closed forms, invariants, exact rational
arithmetic and library routines.  Nothing here touches the GPU path.

The last test plants plausible mistakes into a copy of the oracle's source and checks that
the pins above catch every one of them."""
import os
import types
from fractions import Fraction

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE_PATH = os.path.join(os.path.dirname(HERE), "oracle", "dppf_oracle.py")


def _load_oracle(transform=None, name="dppf_oracle_under_test"):
    with open(ORACLE_PATH) as f:
        src = f.read()
    if transform is not None:
        new = transform(src)
        assert new != src, "mutation did not apply"
        src = new
    mod = types.ModuleType(name)
    mod.__file__ = ORACLE_PATH
    exec(compile(src, ORACLE_PATH, "exec"), mod.__dict__)
    return mod


ORACLE = _load_oracle()


def read_golden(name):
    out = {}
    with open(os.path.join(HERE, "golden", name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            key, *vals = line.split()
            out.setdefault(key, []).append([float(v) for v in vals])
    return {k: np.array(v if len(v) > 1 else v[0], dtype=np.float64) for k, v in out.items()}


def close(a, b, tol=1e-12):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape, (a.shape, b.shape)
    assert np.all(np.abs(a - b) <= tol * (1.0 + np.abs(b))), (a, b)


# ----------------------------------------------------------------------------- pins
def pin_golden_eq5(O):
    for name in ("eq5_m2_d4.txt", "eq5_fixed_point.txt", "eq5_m3_d2.txt"):
        g = read_golden(name)
        x = np.atleast_2d(g["x"])
        pull, push = float(g["pull"][0]), float(g["push"][0])
        x_new, r, c, x_avg = O.pull_push_round(x, pull, push)
        close(x_avg, g["x_avg"])
        close(r, g["r"])
        close(c, g["c"])
        close(x_new, np.atleast_2d(g["x_new"]))
        close(O.replica_mean(x), g["x_avg"])
        close(O.dist_norms(x), g["r"])
        close(O.dist_norms(x, g["x_avg"]), g["r"])
        close(O.pull_push_coefficients(g["r"], pull, push), g["c"])
        if "r_after" in g:
            close(O.dist_norms(x_new), g["r_after"])
        if "x_avg_after" in g:
            close(O.replica_mean(x_new), g["x_avg_after"])
        if "step_len" in g:
            close(np.linalg.norm(x_new - x, axis=1), g["step_len"])


def pin_golden_sequential(O):
    # Alg. 1 order (pull, then push along the pulled gap) == Eq. 5 when x_C = x_A, alpha < 1
    for name in ("eq5_m2_d4.txt", "eq5_m3_d2.txt"):
        g = read_golden(name)
        x = np.atleast_2d(g["x"])
        pull, push = float(g["pull"][0]), float(g["push"][0])
        for ref in ("average", "consensus"):
            x_new, r_post = O.pull_then_push(x, g["x_avg"], pull, push, push_from=ref)
            close(x_new, np.atleast_2d(g["x_new"]))
            close(r_post, (1.0 - pull) * g["r"])


def pin_golden_exact(O):
    g = read_golden("eq5_m3_d2.txt")
    x = np.atleast_2d(g["x"])
    x_new, r, x_avg = O.pull_push_round_exact(x, float(g["pull"][0]), float(g["push_r"][0]))
    close(x_new, np.atleast_2d(g["x_new_exact"]))
    close(r, g["r"])
    close(x_avg, g["x_avg"])


def pin_golden_local_step(O):
    g = read_golden("local_sgd_step.txt")
    lr, mu = float(g["lr"][0]), float(g["momentum"][0])
    x, v, gr = g["x"][None], g["v"][None], g["g"][None]
    x_new, v_new = O.local_sgd_step(x, v, gr, lr, mu)
    close(v_new[0], g["v_new"])
    close(x_new[0], g["x_new"])
    x_new, v_new = O.local_sgd_step(x, v, gr, lr, mu, float(g["weight_decay"][0]))
    close(v_new[0], g["v_new_wd"])
    close(x_new[0], g["x_new_wd"])


def _rand(M, d, seed, spread=1.0):
    rng = np.random.default_rng(seed)
    return rng.standard_normal(d)[None, :] + spread * rng.standard_normal((M, d))


def pin_identical_replicas(O):
    # rows are float32 values (the oracle's input domain): their float64 sum and average are exact
    for M in (2, 3, 4, 7, 8):
        row = np.random.default_rng(M).standard_normal(17).astype(np.float32)
        x = np.tile(row, (M, 1))
        x_new, r, c, x_avg = O.pull_push_round(x, 0.3, 0.7)
        assert np.array_equal(x_new, x)
        assert np.all(r == 0.0) and np.all(c == 0.3)
        assert np.all(np.isfinite(x_new))
    # one worker sitting exactly on the average while the others do not
    x = np.array([[1.0, 2.0], [3.0, 6.0], [2.0, 4.0]])
    x_new, r, c, _ = O.pull_push_round(x, 0.5, 0.25)
    assert r[2] == 0.0 and c[2] == 0.5 and np.array_equal(x_new[2], x[2])
    assert np.all(np.isfinite(x_new))


def pin_full_pull_collapses(O):
    # alpha = 1, lambda = 0: every worker lands on the average (LocalSGD / DDP special case)
    x = _rand(5, 33, 1)
    x_new, _, c, x_avg = O.pull_push_round(x, 1.0, 0.0)
    close(c, np.ones(5))
    for m in range(5):
        close(x_new[m], x_avg)


def pin_pure_pull(O):
    # lambda = 0: the average is preserved and every gap shrinks by (1 - alpha)
    x = _rand(4, 50, 2)
    for alpha in (0.1, 0.5, 0.9):
        x_new, r, _, x_avg = O.pull_push_round(x, alpha, 0.0)
        close(x_new.mean(axis=0), x_avg)
        close(np.linalg.norm(x_new - x_new.mean(axis=0), axis=1), (1 - alpha) * r)


def pin_pure_push(O):
    # alpha = 0: every worker moves exactly lambda, straight away from the average
    x = _rand(4, 40, 3)
    lam = 0.37
    x_new, r, c, x_avg = O.pull_push_round(x, 0.0, lam)
    close(np.linalg.norm(x_new - x, axis=1), np.full(4, lam))
    for m in range(4):
        away = (x[m] - x_avg) / r[m]
        close(x_new[m] - x[m], lam * away)
    close(c, -lam / r)


def pin_gap_dynamics(O):
    # appendix, proof of Theorem 1: with Delta_m = x_A - x_m, u_m = Delta_m / r_m,
    #   x_A+ = x_A - (lambda/M) sum_i u_i ;  Delta_m+ = (1-alpha) Delta_m + lambda u_m - (lambda/M) sum_i u_i
    for M, d, seed in ((3, 7, 4), (4, 64, 5), (8, 9, 6)):
        x = _rand(M, d, seed)
        alpha, lam = 0.3, 0.45
        x_new, r, c, x_avg = O.pull_push_round(x, alpha, lam)
        delta = x_avg[None] - x
        u = delta / np.linalg.norm(delta, axis=1)[:, None]
        ubar = u.mean(axis=0)
        close(x_new.mean(axis=0), x_avg - lam * ubar)
        delta_new = x_new.mean(axis=0)[None] - x_new
        close(delta_new, (1 - alpha) * delta + lam * u - lam * ubar[None])
        close(np.linalg.norm(x_new - x, axis=1), np.abs(alpha * r - lam))
        close(c, alpha - lam / np.linalg.norm(delta, axis=1))


def pin_m2_recurrence(O):
    # M = 2: unit vectors cancel, mean preserved, r+ = (1-alpha) r + lambda -> lambda/alpha
    x = _rand(2, 12, 7, spread=3.0)
    alpha, lam = 0.25, 0.5
    mean0 = x.mean(axis=0)
    r_prev = O.dist_norms(x)
    for _ in range(80):
        x, r, _, _ = O.pull_push_round(x, alpha, lam)
        close(r, r_prev)
        r_prev = (1 - alpha) * r + lam
        close(x.mean(axis=0), mean0, 1e-10)
    close(O.dist_norms(x), np.full(2, lam / alpha), 1e-8)


def pin_regular_polygon(O):
    # symmetric arrangement (unit vectors sum to zero): same recurrence for any M
    M, rad = 6, 4.0
    ang = 2 * np.pi * np.arange(M) / M
    x = np.stack([rad * np.cos(ang), rad * np.sin(ang), np.zeros(M)], axis=1) + np.array([1.0, -2.0, 0.5])
    alpha, lam = 0.5, 1.5
    x_new, r, c, x_avg = O.pull_push_round(x, alpha, lam)
    close(x_avg, [1.0, -2.0, 0.5])
    close(r, np.full(M, rad))
    close(x_new.mean(axis=0), x_avg)
    close(O.dist_norms(x_new), np.full(M, (1 - alpha) * rad + lam))


def pin_equivariances(O):
    x = _rand(4, 21, 8)
    alpha, lam = 0.2, 0.3
    x_new, r, c, x_avg = O.pull_push_round(x, alpha, lam)
    perm_m = np.array([2, 0, 3, 1])
    xn2, r2, c2, xa2 = O.pull_push_round(x[perm_m], alpha, lam)
    close(xn2, x_new[perm_m]); close(r2, r[perm_m]); close(c2, c[perm_m]); close(xa2, x_avg)
    perm_d = np.random.default_rng(0).permutation(21)
    xn3, r3, _, _ = O.pull_push_round(x[:, perm_d], alpha, lam)
    close(xn3, x_new[:, perm_d]); close(r3, r)
    s = 3.5
    xn4, r4, c4, _ = O.pull_push_round(s * x, alpha, s * lam)
    close(xn4, s * x_new); close(r4, s * r); close(c4, c)
    shift = np.linspace(-1, 1, 21)
    xn5, r5, c5, _ = O.pull_push_round(x + shift, alpha, lam)
    close(xn5, x_new + shift, 1e-10); close(r5, r, 1e-10); close(c5, c, 1e-10)


def pin_library_forms(O):
    # the same quantities through numpy's own reductions
    x = _rand(8, 1000, 9, spread=0.01)
    alpha, lam = 0.1, 0.01
    xb = x.mean(axis=0)
    r = np.linalg.norm(x - xb, axis=1)
    c = alpha - lam / r
    ref = x + (xb - x) * c[:, None]
    x_new, r_o, c_o, xb_o = O.pull_push_round(x, alpha, lam)
    close(xb_o, xb); close(r_o, r); close(c_o, c); close(x_new, ref)
    # float32 inputs are widened, never computed in float32
    x32 = x.astype(np.float32)
    x_new32, r32, _, _ = O.pull_push_round(x32, alpha, lam)
    assert x_new32.dtype == np.float64
    x64 = x32.astype(np.float64)
    close(r32, np.linalg.norm(x64 - x64.mean(axis=0), axis=1))


def pin_rational_bruteforce(O):
    # exact rational arithmetic on tiny inputs; r^2 is kept exact and squared results compared
    rng = np.random.default_rng(10)
    for M, d in ((2, 1), (2, 3), (3, 2), (4, 4), (5, 3)):
        xi = rng.integers(-9, 10, size=(M, d))
        if any(all(xi[m, i] * M == xi[:, i].sum() for i in range(d)) for m in range(M)):
            xi[0, 0] += 1
        alpha, lam = Fraction(3, 10), Fraction(7, 5)
        xq = [[Fraction(int(v)) for v in row] for row in xi]
        avg = [sum(xq[m][i] for m in range(M)) / M for i in range(d)]
        r2 = [sum((xq[m][i] - avg[i]) ** 2 for i in range(d)) for m in range(M)]
        x_new, r, c, x_avg = O.pull_push_round(xi.astype(np.float64), float(alpha), float(lam))
        close(x_avg, [float(a) for a in avg])
        close(r * r, [float(v) for v in r2])
        for m in range(M):
            rm = float(r2[m]) ** 0.5
            for i in range(d):
                # x + (avg - x)*(alpha - lam/r): rational except for the single sqrt
                want = float(xq[m][i]) + float(avg[i] - xq[m][i]) * (float(alpha) - float(lam) / rm)
                assert abs(x_new[m, i] - want) <= 1e-12 * (1 + abs(want))
            # the displacement length squared is (alpha*r - lam)^2 = alpha^2 r^2 - 2 alpha lam r + lam^2
            disp2 = float(np.sum((x_new[m] - xi[m]) ** 2))
            want2 = float(alpha * alpha * r2[m] + lam * lam) - 2 * float(alpha * lam) * rm
            assert abs(disp2 - want2) <= 1e-10 * (1 + abs(want2))


def pin_local_step_recurrence(O):
    # textbook heavy-ball: x_t = x_0 - eta * sum_{k<=t} v_k, v_k = sum_{j<=k} mu^(k-j) g_j  (v_0 = 0)
    rng = np.random.default_rng(11)
    M, d, steps = 3, 5, 6
    x0 = rng.standard_normal((M, d))
    gs = rng.standard_normal((steps, M, d))
    eta, mu = 0.05, 0.9
    x, v = x0.copy(), np.zeros((M, d))
    for k in range(steps):
        x, v = O.local_sgd_step(x, v, gs[k], eta, mu)
    v_closed = sum(mu ** (steps - 1 - j) * gs[j] for j in range(steps))
    x_closed = x0 - eta * sum(sum(mu ** (k - j) * gs[j] for j in range(k + 1)) for k in range(steps))
    close(v, v_closed); close(x, x_closed)
    # first step from v = 0 is plain SGD (Alg. 1's line)
    x1, v1 = O.local_sgd_step(x0, np.zeros((M, d)), gs[0], eta, mu)
    close(x1, x0 - eta * gs[0]); close(v1, gs[0])
    # equivalent "velocity includes the learning rate" form, constant eta
    xa, va = x0.copy(), np.zeros((M, d))
    for k in range(steps):
        va = mu * va - eta * gs[k]
        xa = xa + va
    close(x, xa)


def pin_local_step_torch(O):
    # the library optimizer the experiments name (SGD with momentum, coupled weight decay)
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(12)
    d, steps = 9, 5
    x0 = rng.standard_normal(d)
    gs = rng.standard_normal((steps, d))
    for wd in (0.0, 1e-3):
        p = torch.nn.Parameter(torch.tensor(x0, dtype=torch.float64))
        opt = torch.optim.SGD([p], lr=0.1, momentum=0.9, weight_decay=wd)
        x, v = x0[None].copy(), np.zeros((1, d))
        for k in range(steps):
            p.grad = torch.tensor(gs[k], dtype=torch.float64)
            opt.step()
            x, v = O.local_sgd_step(x, v, gs[k][None], 0.1, 0.9, wd)
        close(x[0], p.detach().numpy())


def pin_fused_round_is_composition(O):
    rng = np.random.default_rng(13)
    M, d = 4, 30
    x = _rand(M, d, 14, 0.05); v = rng.standard_normal((M, d)); g = rng.standard_normal((M, d))
    x1, v1 = O.local_sgd_step(x, v, g, 0.1, 0.9, 1e-3)
    xb = x1.mean(axis=0); r = np.linalg.norm(x1 - xb, axis=1)
    ref = x1 + (xb - x1) * (0.2 - 0.05 / r)[:, None]
    x2, v2, r2, c2, xb2 = O.dppf_round(x, v, g, 0.1, 0.9, 1e-3, 0.2, 0.05)
    close(x2, ref); close(v2, v1); close(r2, r); close(xb2, xb); close(c2, 0.2 - 0.05 / r)


def pin_sequential_general_consensus(O):
    # pulling toward an arbitrary x_C then pushing away from the average, by direct formulas
    x = _rand(3, 8, 15)
    xc = np.random.default_rng(16).standard_normal(8)
    alpha, lam = 0.4, 0.6
    xa = x.mean(axis=0)
    pulled = (1 - alpha) * x + alpha * xc
    gap = pulled - xa
    want = pulled + lam * gap / np.linalg.norm(gap, axis=1)[:, None]
    got, r_post = O.pull_then_push(x, xc, alpha, lam, "average")
    close(got, want); close(r_post, np.linalg.norm(gap, axis=1))
    gap_c = pulled - xc
    want_c = pulled + lam * gap_c / np.linalg.norm(gap_c, axis=1)[:, None]
    got_c, r_c = O.pull_then_push(x, xc, alpha, lam, "consensus")
    close(got_c, want_c); close(r_c, (1 - alpha) * np.linalg.norm(x - xc, axis=1))
    # alpha = 1 toward x_C = x_A puts every worker on the average: no direction, no push
    got1, r1 = O.pull_then_push(x, xa, 1.0, lam, "average")
    close(got1, np.tile(xa, (3, 1))); close(r1, np.zeros(3), 1e-15)


def pin_golden_general_consensus(O):
    # Alg. 1 with a consensus variable that is not the average: hand-worked fixtures for both
    # reference points of the push
    for name in ("alg1_general_xc_m2.txt", "alg1_general_xc_m3_average.txt", "alg1_general_xc_m3_consensus.txt"):
        g = read_golden(name)
        x, xc = np.atleast_2d(g["x"]), g["x_c"]
        pull, push = float(g["pull"][0]), float(g["push"][0])
        if "x_avg" in g:
            close(O.replica_mean(x), g["x_avg"])
        for ref in ("average", "consensus"):
            if "x_new_" + ref not in g:
                continue
            x_new, r_post = O.pull_then_push(x, xc, pull, push, push_from=ref)
            close(x_new, np.atleast_2d(g["x_new_" + ref]))
            close(r_post, g["r_post_" + ref])
            # without the push only the pull is left
            only_pulled, _ = O.pull_then_push(x, xc, pull, 0.0, push_from=ref)
            close(only_pulled, np.atleast_2d(g["pulled"]))
        if "dist_to_xc_after" in g:
            x_new, _ = O.pull_then_push(x, xc, pull, push, push_from="consensus")
            close(np.linalg.norm(x_new - xc, axis=1), g["dist_to_xc_after"])


def pin_general_consensus_invariants(O):
    # properties of Alg. 1's consensus branch that hold for any x_C, stated without the update
    # formula: the pull is an interpolation, the push has length lambda and points straight away
    # from its reference point, which for Alg. 1 is the workers' average BEFORE the round
    for M, d, seed in ((2, 5, 21), (3, 8, 22), (5, 4, 23), (8, 16, 24)):
        x = _rand(M, d, seed)
        xc = np.random.default_rng(seed + 100).standard_normal(d) * 2.0 + 0.5
        xa = x.mean(axis=0)
        for alpha, lam in ((0.4, 0.6), (0.05, 2.0), (0.9, 0.01)):
            pulled, _ = O.pull_then_push(x, xc, alpha, 0.0, "average")
            # position of the pulled worker relative to the pre-round average
            close(pulled - xa, (1 - alpha) * (x - xa) + alpha * (xc - xa)[None], 1e-11)
            # the pulled worker lies on the segment from x_m to x_C, a fraction alpha of the way
            close(np.linalg.norm(pulled - x, axis=1), alpha * np.linalg.norm(x - xc, axis=1), 1e-11)
            close(np.linalg.norm(pulled - xc, axis=1), (1 - alpha) * np.linalg.norm(x - xc, axis=1), 1e-11)
            for ref_name, ref in (("average", xa), ("consensus", xc)):
                x_new, r_post = O.pull_then_push(x, xc, alpha, lam, ref_name)
                move = x_new - pulled
                close(np.linalg.norm(move, axis=1), np.full(M, lam), 1e-11)
                # straight away from the reference: the distance to it grows by exactly lambda
                close(np.linalg.norm(pulled - ref, axis=1), r_post, 1e-11)
                close(np.linalg.norm(x_new - ref, axis=1), r_post + lam, 1e-11)
            # pushing away from x_C: every worker ends at (1-alpha)||x_m - x_C|| + lambda from x_C
            x_new, _ = O.pull_then_push(x, xc, alpha, lam, "consensus")
            close(np.linalg.norm(x_new - xc, axis=1), (1 - alpha) * np.linalg.norm(x - xc, axis=1) + lam, 1e-11)
    # a leader as consensus variable (x_C = x_1): the pull leaves the leader where it is, so with
    # the push redirected away from x_C the leader has no direction and does not move at all
    x = np.round(8.0 * _rand(4, 6, 25))     # small integers and alpha = 1/4: the pull is exact
    x_new, r_post = O.pull_then_push(x, x[0], 0.25, 0.7, "consensus")
    assert r_post[0] == 0.0 and np.array_equal(x_new[0], x[0])
    # ... while Alg. 1's own push moves it away from the average by lambda
    x_new, r_post = O.pull_then_push(x, x[0], 0.25, 0.7, "average")
    close(np.linalg.norm(x_new[0] - x[0]), 0.7)
    close(np.linalg.norm(x_new[0] - x.mean(axis=0)), np.linalg.norm(x[0] - x.mean(axis=0)) + 0.7)


def pin_exact_update(O):
    # the exact two-term update is a gradient step on R = -(1/M) sum ||x_i - x_A||:
    # compare with a central finite difference of R, and check that it preserves the mean
    M, d = 4, 6
    x = _rand(M, d, 17)
    lam_r = 0.8

    def R(xx):
        return -np.mean(np.linalg.norm(xx - xx.mean(axis=0), axis=1))

    x_new, r, x_avg = O.pull_push_round_exact(x, 0.0, lam_r)
    step = x_new - x
    h = 1e-6
    grad = np.zeros_like(x)
    for m in range(M):
        for i in range(d):
            xp = x.copy(); xp[m, i] += h
            xm = x.copy(); xm[m, i] -= h
            grad[m, i] = (R(xp) - R(xm)) / (2 * h)
    close(step, -lam_r * grad, 1e-7)
    close(x_new.mean(axis=0), x_avg)
    xp, _, _ = O.pull_push_round_exact(x, 0.35, lam_r)
    close(xp.mean(axis=0), x_avg)
    # on a symmetric arrangement the second term vanishes: equals Eq. 5 with lambda = lambda_r / M
    ang = 2 * np.pi * np.arange(5) / 5
    xs = np.stack([np.cos(ang), np.sin(ang)], axis=1) * 2.0
    a, _, _ = O.pull_push_round_exact(xs, 0.3, 5 * 0.4)
    b, _, _, _ = O.pull_push_round(xs, 0.3, 0.4)
    close(a, b)


def pin_statistics_and_schedules(O):
    st = O.round_statistics(np.array([5.0, 5.0, 8.0]), 0.5, 2.0)
    assert st["relaxed_mv"] == 6.0
    close(st["pull_strength"], [2.5, 2.5, 4.0]); close(st["push_strength"], [2.0, 2.0, 2.0])
    assert "average_norm" not in st
    # norm of the average and valley width over that norm: x_A = (3, -4, 12) has norm 13
    st = O.round_statistics(np.array([5.0, 5.0, 8.0]), 0.5, 2.0, x_avg=np.array([3.0, -4.0, 12.0]))
    assert st["average_norm"] == 13.0 and st["relaxed_mv"] == 6.0
    close(st["width_over_norm"], 6.0 / 13.0)
    # ... and on the hand-worked M = 3 round, whose average is (1, 1)
    g = read_golden("eq5_m3_d2.txt")
    _, r, _, x_avg = O.pull_push_round(np.atleast_2d(g["x"]), 0.5, 2.0)
    st = O.round_statistics(r, 0.5, 2.0, x_avg)
    close(st["average_norm"], np.sqrt(2.0)); close(st["width_over_norm"], 6.0 / np.sqrt(2.0))
    T = 100
    assert O.push_schedule("fixed", 0.5, 37, T) == 0.5
    close(O.push_schedule("decreasing", 0.5, 0, T), 0.5)
    close(O.push_schedule("decreasing", 0.5, T, T), 0.0)
    close(O.push_schedule("decreasing", 0.5, T // 2, T), 0.25)
    close(O.push_schedule("increasing", 0.5, 0, T), 0.0)
    close(O.push_schedule("increasing", 0.5, T, T), 0.5)
    close(O.push_schedule("increasing", 0.5, 25, T), 0.25 * (1 - np.sqrt(0.5)))
    for t in (0, 13, 50, 99):   # the two cosine schedules mirror each other
        close(O.push_schedule("increasing", 0.5, t, T) + O.push_schedule("decreasing", 0.5, t, T), 0.5)


def pin_adamw(O):
    # step 1 with eps = 0 moves every coordinate by exactly lr against the gradient's sign
    x, m1, m2 = O.local_adamw_step(np.array([[1.0, -2.0]]), np.zeros((1, 2)), np.zeros((1, 2)),
                                   np.array([[0.5, -3.0]]), 0.1, 0.9, 0.999, 0.0, 0.1, 1)
    close(x, [[0.99 - 0.1, -1.98 + 0.1]]); close(m1, [[0.05, -0.3]]); close(m2, [[0.00025, 0.009]])
    # second step by rational arithmetic (one sqrt)
    g2 = Fraction(-1)
    mm = Fraction(9, 10) * Fraction(1, 20) + Fraction(1, 10) * g2
    ss = Fraction(999, 1000) * Fraction(1, 4000) + Fraction(1, 1000) * g2 * g2
    mhat = mm / (1 - Fraction(9, 10) ** 2)
    shat = ss / (1 - Fraction(999, 1000) ** 2)
    xq = Fraction(89, 100) * (1 - Fraction(1, 100))
    want = float(xq) - 0.1 * float(mhat) / (float(shat) ** 0.5)
    x2, _, _ = O.local_adamw_step(x[:, :1], m1[:, :1], m2[:, :1], np.array([[-1.0]]),
                                  0.1, 0.9, 0.999, 0.0, 0.1, 2)
    close(x2, [[want]])
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(18)
    d, steps = 7, 6
    x0 = rng.standard_normal(d); gs = rng.standard_normal((steps, d))
    p = torch.nn.Parameter(torch.tensor(x0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=5e-4, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.01)
    xx, a, b = x0[None].copy(), np.zeros((1, d)), np.zeros((1, d))
    for k in range(steps):
        p.grad = torch.tensor(gs[k], dtype=torch.float64)
        opt.step()
        xx, a, b = O.local_adamw_step(xx, a, b, gs[k][None], 5e-4, 0.9, 0.999, 1e-8, 0.01, k + 1)
    close(xx[0], p.detach().numpy())


PINS = [v for k, v in sorted(globals().items()) if k.startswith("pin_")]
# Pins that write the oracle's own expression out a second time.  They guard against accidental
# edits, but a restated formula cannot show that the formula is right: they do not count when the
# planted mistakes below are hunted.
RESTATING = {"pin_sequential_general_consensus"}


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_pin(pin):
    pin(ORACLE)


# ------------------------------------------------------------------ planted mistakes
def _sub(old, new, count=1):
    def tr(src):
        assert src.count(old) >= 1, old
        return src.replace(old, new) if count == 0 else src.replace(old, new, count)
    return tr


MUTANTS = {
    "push_sign": _sub("c[m] = pull - push / r[m]", "c[m] = pull + push / r[m]"),
    "push_dropped": _sub("c[m] = pull - push / r[m]", "c[m] = pull"),
    "push_over_r_squared": _sub("c[m] = pull - push / r[m]", "c[m] = pull - push / (r[m] * r[m])"),
    "update_direction": _sub("x_new[m] = x[m] + (x_avg - x[m]) * c[m]", "x_new[m] = x[m] - (x_avg - x[m]) * c[m]"),
    "update_other_worker": _sub("x_new[m] = x[m] + (x_avg - x[m]) * c[m]", "x_new[m] = x[m] + (x_avg - x[m]) * c[0]"),
    "mean_not_divided": _sub("return total / M", "return total"),
    "mean_skips_worker": _sub("for m in range(M):\n        total = total + x[m]", "for m in range(1, M):\n        total = total + x[m]"),
    "norm_not_rooted": _sub("r[m] = np.sqrt(np.sum(diff * diff))", "r[m] = np.sum(diff * diff)"),
    "norm_l1": _sub("r[m] = np.sqrt(np.sum(diff * diff))", "r[m] = np.sum(np.abs(diff))"),
    "norm_rms": _sub("r[m] = np.sqrt(np.sum(diff * diff))", "r[m] = np.sqrt(np.mean(diff * diff))"),
    "zero_gap_nan": _sub("if r[m] > 0.0:\n            c[m] = pull - push / r[m]", "if True:\n            c[m] = pull - push / r[m]"),
    "sequential_update": _sub("x_new = np.empty_like(x)\n    for m in range(M):\n        if r[m] > 0.0:\n            x_new[m] = x[m] + (x_avg - x[m]) * c[m]",
                              "x_new = np.empty_like(x)\n    for m in range(M):\n        x_avg = replica_mean(x if m == 0 else np.vstack([x_new[:m], x[m:]]))\n        if r[m] > 0.0:\n            x_new[m] = x[m] + (x_avg - x[m]) * c[m]"),
    "momentum_on_grad": _sub("v_new = momentum * v + g_eff", "v_new = momentum * (v + g_eff)"),
    "momentum_dampened": _sub("v_new = momentum * v + g_eff", "v_new = momentum * v + (1.0 - momentum) * g_eff"),
    "step_uses_old_v": _sub("x_new = x - lr * v_new\n    return x_new, v_new", "x_new = x - lr * v\n    return x_new, v_new"),
    "step_sign": _sub("x_new = x - lr * v_new\n    return x_new, v_new", "x_new = x + lr * v_new\n    return x_new, v_new"),
    "wd_sign": _sub("g_eff = g + weight_decay * x", "g_eff = g - weight_decay * x"),
    "wd_decoupled": _sub("g_eff = g + weight_decay * x\n    v_new = momentum * v + g_eff\n    x_new = x - lr * v_new",
                         "g_eff = g\n    v_new = momentum * v + g_eff\n    x_new = x - lr * v_new - lr * weight_decay * x"),
    "fused_round_before_step": _sub("x1, v1 = local_sgd_step(x, v, g, lr, momentum, weight_decay)\n    x2, r, c, x_avg = pull_push_round(x1, pull, push)",
                                    "x1, r, c, x_avg = pull_push_round(x, pull, push)\n    x2, v1 = local_sgd_step(x1, v, g, lr, momentum, weight_decay)"),
    "seq_push_prepull_gap": _sub("gap = pulled - ref", "gap = x[m] - ref"),
    "seq_pull_weights_swapped": _sub("pulled = (1.0 - pull) * x[m] + pull * x_c", "pulled = pull * x[m] + (1.0 - pull) * x_c"),
    "seq_push_toward": _sub("x_new[m] = pulled + push * gap / r_post[m]", "x_new[m] = pulled - push * gap / r_post[m]"),
    "seq_average_after_pull": _sub("gap = pulled - ref\n", "gap = pulled - (((1.0 - pull) * x + pull * x_c).mean(axis=0) if push_from == \"average\" else ref)\n"),
    "seq_ref_always_consensus": _sub("ref = x_avg if push_from == \"average\" else x_c", "ref = x_c"),
    "seq_ref_always_average": _sub("ref = x_avg if push_from == \"average\" else x_c", "ref = x_avg"),
    "exact_second_term_sign": _sub("(M * units[m] - unit_sum)", "(M * units[m] + unit_sum)"),
    "exact_scale": _sub("(push_r / (M * M)) * (M * units[m]", "(push_r / M) * (M * units[m]"),
    "exact_pull_sign": _sub("x_new[m] = x[m] - pull * d_m + ", "x_new[m] = x[m] + pull * d_m + "),
    "schedule_swapped": _sub("return 0.5 * push * (1.0 + np.cos(np.pi * t / t_total))", "return 0.5 * push * (1.0 - np.cos(np.pi * t / t_total))"),
    "schedule_period": _sub("return 0.5 * push * (1.0 - np.cos(np.pi * t / t_total))", "return 0.5 * push * (1.0 - np.cos(2.0 * np.pi * t / t_total))"),
    "relaxed_mv_sum": _sub('"relaxed_mv": float(np.sum(r) / r.shape[0])', '"relaxed_mv": float(np.sum(r))'),
    "average_norm_not_rooted": _sub('float(np.sqrt(np.sum(x_avg * x_avg)))', 'float(np.sum(x_avg * x_avg))'),
    "average_norm_l1": _sub('float(np.sqrt(np.sum(x_avg * x_avg)))', 'float(np.sum(np.abs(x_avg)))'),
    "width_ratio_inverted": _sub('out["relaxed_mv"] / out["average_norm"]', 'out["average_norm"] / out["relaxed_mv"]'),
    "adamw_no_bias_correction": _sub("m_hat = m1_new / (1.0 - beta1 ** step)", "m_hat = m1_new"),
    "adamw_coupled_decay": _sub("x = x - lr * weight_decay * x\n    m1_new = beta1 * m1 + (1.0 - beta1) * g", "g = g + weight_decay * x\n    m1_new = beta1 * m1 + (1.0 - beta1) * g"),
    "adamw_eps_inside": _sub("(np.sqrt(s_hat) + eps)", "np.sqrt(s_hat + eps)"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name):
    mutant = _load_oracle(MUTANTS[name], name="mutant_" + name)
    caught = []
    for pin in PINS:
        if pin.__name__ in RESTATING:
            continue
        try:
            with np.errstate(all="ignore"):
                pin(mutant)
        except Exception:
            caught.append(pin.__name__)
    assert caught, f"no pin notices the planted mistake '{name}'"
