"""GPU parity of the round's variants (exact two-term push, literal Alg. 1 with a supplied
consensus variable), the AdamW local step, the logged by-products, and a multi-round driver."""
import numpy as np
import pytest

from parity import (EPS32, O, assert_average_norm, assert_params_close, assert_rel, assert_update_close, download,
                    download_rows, f32, upload_tensors)

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2507_20424_amd import dppf, workloads as W  # noqa: E402


def _rows(inp, arrays, misalign=0):
    return [upload_tensors(a, inp.offsets, misalign) for a in arrays]


@pytest.mark.parametrize("M", [2, 3, 4, 5, 8, 9, 12, 17, 34, 39, 40, 47])
def test_exact_two_term_round(M):
    spec = W.small_spec(M=M, seed=300 + M)
    inp = W.make_inputs(spec)
    x_host = np.stack(inp.x)
    pull, push_r = f32(0.3), f32(0.08 * M)
    ref_x, ref_r, ref_avg = O.pull_push_round_exact(x_host, pull, push_r)
    x = _rows(inp, inp.x, 1)
    r = torch.zeros(M, device="cuda")
    c = torch.zeros(M, device="cuda")
    plan = dppf.Plan(M, spec.numel)
    plan.pull_push_round_exact(x, pull, push_r, r_out=r, c_out=c)
    got = download_rows(x)
    assert_rel(r.cpu().numpy(), ref_r, 1e-4, "r")
    assert_rel(c.cpu().numpy(), pull - (push_r / M) / ref_r, 1e-4, "c")
    assert_params_close(got, ref_x, inp.offsets, 0, "exact round x")
    assert_update_close(got, ref_x, x_host.astype(np.float64), "exact round")
    assert_average_norm(plan, ref_avg, "exact round")
    # the exact gradient preserves the average of the workers
    mean_err = np.max(np.abs(got.astype(np.float64).mean(axis=0) - ref_avg))
    assert mean_err <= 4 * EPS32 * np.max(np.abs(ref_avg))
    # and it differs from the one-term update by the dropped second term
    one_term, _, _, _ = O.pull_push_round(x_host, pull, push_r / M)
    if M > 2:
        assert np.max(np.abs(one_term - ref_x)) > 100 * EPS32 * np.max(np.abs(ref_x))
    plan.close()


def test_exact_round_zero_distance_worker():
    # a worker on the average has no unit vector of its own but still receives the others' sum
    base = ((np.arange(6000) - 3000) / 1024.0).astype(np.float32)
    bump = np.zeros(6000, np.float32); bump[:3000] = 0.5
    rows = [base - 0.25, base + 0.25 + bump, base - bump, base.copy()]
    rows = [r.astype(np.float32) for r in rows]
    x_host = np.stack(rows)
    offsets = np.array([0, 6000])
    ref_x, ref_r, _ = O.pull_push_round_exact(x_host, f32(0.25), f32(1.0))
    assert ref_r[3] == 0.0
    x = [upload_tensors(a, offsets) for a in rows]
    r = torch.zeros(4, device="cuda")
    plan = dppf.Plan(4, [6000])
    plan.pull_push_round_exact(x, f32(0.25), f32(1.0), r_out=r)
    assert r.cpu().numpy()[3] == 0.0
    assert_params_close(download_rows(x), ref_x, offsets, 0, "x")
    plan.close()


@pytest.mark.parametrize("M", [2, 4, 7, 8, 9, 11, 16, 17, 36, 43])
@pytest.mark.parametrize("push_from", ["average", "consensus"])
def test_pull_then_push_with_supplied_consensus(M, push_from):
    spec = W.small_spec(M=M, seed=400 + M)
    inp = W.make_inputs(spec)
    x_host = np.stack(inp.x)
    rng = np.random.default_rng(5)
    xc_host = (inp.x[0] + 2e-3 * rng.standard_normal(spec.d)).astype(np.float32)   # e.g. a "leader"
    pull, push = f32(0.4), f32(0.02)
    ref_x, ref_r = O.pull_then_push(x_host, xc_host, pull, push, push_from)
    x = _rows(inp, inp.x)
    xc = upload_tensors(xc_host, inp.offsets, 2)
    r = torch.zeros(M, device="cuda")
    plan = dppf.Plan(M, spec.numel)
    plan.pull_then_push(x, xc, pull, push, push_from, r_post_out=r)
    got = download_rows(x)
    assert_rel(r.cpu().numpy(), ref_r, 1e-4, "r_post")
    assert_params_close(got, ref_x, inp.offsets, 0, "x")
    assert_update_close(got, ref_x, x_host.astype(np.float64), "pull_then_push")
    assert np.array_equal(download(xc), xc_host), "the consensus variable was modified"
    plan.close()


def test_pull_then_push_toward_the_average_equals_eq5():
    # Sec. 5: with x_C = x_A the two steps of Alg. 1 collapse into Eq. 5
    spec = W.small_spec(M=4, seed=77)
    inp = W.make_inputs(spec)
    pull, push = f32(0.2), f32(0.03)
    plan = dppf.Plan(4, spec.numel)
    xa = upload_tensors(np.zeros(spec.d, np.float32), inp.offsets)
    x1 = _rows(inp, inp.x)
    plan.replica_mean(x1, xa)
    plan.pull_then_push(x1, xa, pull, push, "average")
    x2 = _rows(inp, inp.x)
    plan.pull_push_round(x2, pull, push)
    a, b = download_rows(x1).astype(np.float64), download_rows(x2).astype(np.float64)
    assert np.max(np.abs(a - b)) <= 8 * EPS32 * np.max(np.abs(b))
    # a worker that the pull puts exactly on the reference point gets no push (alpha = 1)
    x3 = _rows(inp, inp.x)
    r = torch.ones(4, device="cuda")
    plan.pull_then_push(x3, xa, 1.0, push, "consensus", r_post_out=r)
    assert np.all(r.cpu().numpy() == 0.0)
    avg = download(xa)
    for row in download_rows(x3):
        assert np.array_equal(row, avg)
    plan.close()


@pytest.mark.parametrize("M", [1, 4])
def test_adamw_local_step(M):
    spec = W.small_spec(M=M, seed=500 + M)
    inp = W.make_inputs(spec)
    lr, b1, b2, eps, wd = f32(5e-4), f32(0.9), f32(0.999), f32(1e-8), f32(0.01)
    x = _rows(inp, inp.x, 1)
    m1 = _rows(inp, inp.v, 2)
    m2 = _rows(inp, inp.v, 3)
    xo = np.stack(inp.x).astype(np.float64)
    ao, so = np.zeros_like(xo), np.zeros_like(xo)
    plan = dppf.Plan(M, spec.numel)
    for k in range(4):
        gk = inp.grads(k)
        g = _rows(inp, gk)
        plan.local_adamw_step(x, m1, m2, g, lr, b1, b2, eps, wd, k + 1)
        xo, ao, so = O.local_adamw_step(xo, ao, so, np.stack(gk), lr, b1, b2, eps, wd, k + 1)
        assert_params_close(download_rows(x), xo, inp.offsets, 2 * (k + 1), f"adamw x step {k}")
        assert_params_close(download_rows(m1), ao, inp.offsets, 2 * (k + 1), f"adamw m1 step {k}")
        assert_params_close(download_rows(m2), so, inp.offsets, 2 * (k + 1), f"adamw m2 step {k}")
        # the step itself (about lr per coordinate) must be right, not just x
        assert_update_close(download_rows(x), xo, np.stack(inp.x).astype(np.float64), f"adamw step {k}")
    plan.close()


@pytest.mark.parametrize("M", [2, 4, 8, 9, 16, 18, 39, 42])
def test_fused_adamw_round(M):
    # the ViT runs of the paper: AdamW local steps, then the pull-push round
    spec = W.small_spec(M=M, seed=520 + M)
    inp = W.make_inputs(spec)
    lr, b1, b2, eps, wd = f32(5e-4), f32(0.9), f32(0.999), f32(1e-8), f32(0.01)
    pull, push = f32(0.9), f32(0.05)
    x, m1, m2 = _rows(inp, inp.x), _rows(inp, inp.v), _rows(inp, inp.v)
    xo = np.stack(inp.x).astype(np.float64)
    ao, so = np.zeros_like(xo), np.zeros_like(xo)
    plan = dppf.Plan(M, spec.numel)
    r = torch.zeros(M, device="cuda")
    c = torch.zeros(M, device="cuda")
    for k in range(2):                                   # two plain steps, then the fused one
        gk = inp.grads(k)
        plan.local_adamw_step(x, m1, m2, _rows(inp, gk), lr, b1, b2, eps, wd, k + 1)
        xo, ao, so = O.local_adamw_step(xo, ao, so, np.stack(gk), lr, b1, b2, eps, wd, k + 1)
    gk = inp.grads(2)
    g = _rows(inp, gk)
    # unfused twin on copies, for the bit-for-bit claim
    x2 = [[t.clone() for t in row] for row in x]
    a2 = [[t.clone() for t in row] for row in m1]
    s2 = [[t.clone() for t in row] for row in m2]
    plan.round_adamw(x, m1, m2, g, lr, b1, b2, eps, wd, 3, pull, push, r_out=r, c_out=c)
    x_pre, ao, so = O.local_adamw_step(xo, ao, so, np.stack(gk), lr, b1, b2, eps, wd, 3)
    ref_x, ref_r, ref_c, ref_avg = O.pull_push_round(x_pre, pull, push)
    got = download_rows(x)
    assert_rel(r.cpu().numpy(), ref_r, 1e-4, "r")
    assert_rel(c.cpu().numpy(), ref_c, 1e-4, "c")
    assert_average_norm(plan, ref_avg, "fused adamw round")
    assert_params_close(got, ref_x, inp.offsets, 6, "x", c=ref_c)
    assert_params_close(download_rows(m1), ao, inp.offsets, 6, "m1")
    assert_params_close(download_rows(m2), so, inp.offsets, 6, "m2")
    assert_update_close(got, ref_x, x_pre, "fused adamw round")
    twin = dppf.Plan(M, spec.numel)
    twin.local_adamw_step(x2, a2, s2, g, lr, b1, b2, eps, wd, 3)
    twin.pull_push_round(x2, pull, push)
    assert np.array_equal(download_rows(x2), got)
    assert np.array_equal(download_rows(a2), download_rows(m1))
    plan.close()
    twin.close()


@pytest.mark.parametrize("M", [1, 3])
@pytest.mark.parametrize("shapes", [((4096,),), ((3 * 4096 + 5,), (17,)), ((4096,), (2 * 4096,), (100,), (2 * 4096 + 1,))])
def test_local_steps_take_full_tiles_in_pairs(M, shapes):
    # the local-step kernels handle one worker at a time, two full tiles per work item: lists with
    # one, three and five full tiles leave a single tile over, for one worker as for several
    spec = W.small_spec(M=M, seed=640 + M + len(shapes), shapes=shapes)
    inp = W.make_inputs(spec)
    gk = inp.grads(0)
    x_host, v_host, g_host = np.stack(inp.x), np.stack(inp.v), np.stack(gk)
    plan = dppf.Plan(M, spec.numel)
    x, v, g = _rows(inp, inp.x), _rows(inp, inp.v), _rows(inp, gk)
    plan.local_sgd_step(x, v, g, f32(0.1), f32(0.9), f32(1e-3))
    ref_x, ref_v = O.local_sgd_step(x_host, v_host, g_host, f32(0.1), f32(0.9), f32(1e-3))
    assert_params_close(download_rows(x), ref_x, inp.offsets, 1, "x")
    assert_params_close(download_rows(v), ref_v, inp.offsets, 1, "v")
    lr, b1, b2, eps, wd = f32(5e-4), f32(0.9), f32(0.999), f32(1e-8), f32(0.01)
    x, m1, m2 = _rows(inp, inp.x), _rows(inp, inp.v), _rows(inp, inp.v)
    plan.local_adamw_step(x, m1, m2, g, lr, b1, b2, eps, wd, 1)
    zero = np.zeros_like(x_host, dtype=np.float64)
    xo, ao, so = O.local_adamw_step(x_host.astype(np.float64), zero, zero, g_host, lr, b1, b2, eps, wd, 1)
    assert_params_close(download_rows(x), xo, inp.offsets, 2, "adamw x")
    assert_params_close(download_rows(m1), ao, inp.offsets, 2, "adamw m1")
    assert_params_close(download_rows(m2), so, inp.offsets, 2, "adamw m2")
    plan.close()


LONG_SHAPES = ((2_500_000,), (1_234_567,), (1_000_003,), (777,))


@pytest.mark.parametrize("M", [2, 12, 17, 40])
def test_every_entry_point_on_a_list_with_an_on_demand_tail(M):
    # With four or more tiles per thread block the read-write sweeps hand the tail of their tiles
    # out on demand; every entry point must give the oracle's result through that path too
    # (M = 12: two vectors per lane and worker, registers beyond the first 256; M = 17: the kernels
    # that stage the workers in LDS; M = 40: the kernels that store the average).
    spec = W.small_spec(M=M, seed=950 + M, shapes=LONG_SHAPES)
    _, nfull, _ = dppf.layout_tiles(spec.numel)      # the largest tiles any kernel uses
    assert nfull >= 4 * torch.cuda.get_device_properties(0).multi_processor_count
    inp = W.make_inputs(spec)
    gk = inp.grads(0)
    x_host, v_host, g_host = np.stack(inp.x), np.stack(inp.v), np.stack(gk)
    lr, mu, wd, pull, push = f32(0.1), f32(0.9), f32(1e-4), f32(0.3), f32(0.05)
    plan = dppf.Plan(M, spec.numel)
    r = torch.zeros(M, device="cuda")

    # local step
    x, v, g = _rows(inp, inp.x), _rows(inp, inp.v), _rows(inp, gk)
    plan.local_sgd_step(x, v, g, lr, mu, wd)
    ref_x1, ref_v1 = O.local_sgd_step(x_host, v_host, g_host, lr, mu, wd)
    assert_params_close(download_rows(x), ref_x1, inp.offsets, 1, "local step x")
    assert_params_close(download_rows(v), ref_v1, inp.offsets, 1, "local step v")

    # round, then fused step + round
    x = _rows(inp, inp.x)
    plan.pull_push_round(x, pull, push, r_out=r)
    ref_x, ref_r, ref_c, _ = O.pull_push_round(x_host, pull, push)
    assert_rel(r.cpu().numpy(), ref_r, 1e-4, "r")
    assert_params_close(download_rows(x), ref_x, inp.offsets, 0, "round x", c=ref_c)
    x, v = _rows(inp, inp.x), _rows(inp, inp.v)
    xbar = upload_tensors(np.zeros(spec.d, np.float32), inp.offsets)
    plan.round(x, v, g, lr, mu, wd, pull, push, r_out=r, xbar_out=xbar)
    ref_x, ref_v, ref_r, ref_c, ref_avg = O.dppf_round(x_host, v_host, g_host, lr, mu, wd, pull, push)
    assert_rel(r.cpu().numpy(), ref_r, 1e-4, "fused r")
    assert_params_close(download(xbar)[None, :], ref_avg[None, :], inp.offsets, 1, "fused round average")
    got = download_rows(x)
    assert_params_close(got, ref_x, inp.offsets, 1, "fused round x", c=ref_c)
    assert_params_close(download_rows(v), ref_v, inp.offsets, 1, "fused round v")
    assert_update_close(got, ref_x, ref_x1, "fused round")

    # the stand-alone average and distances
    x = _rows(inp, inp.x)
    plan.replica_mean(x, xbar)
    assert_params_close(download(xbar)[None, :], O.replica_mean(x_host)[None, :], inp.offsets, 0, "average")
    for given in (None, xbar):
        r.zero_()
        plan.dist_norms(x, r, xbar=given)
        assert_rel(r.cpu().numpy(), O.dist_norms(x_host, O.replica_mean(x_host)), 1e-4, "distances")

    # exact two-term round
    x = _rows(inp, inp.x)
    plan.pull_push_round_exact(x, pull, f32(push * M), r_out=r)
    ref_x, ref_r, _ = O.pull_push_round_exact(x_host, pull, f32(push * M))
    assert_rel(r.cpu().numpy(), ref_r, 1e-4, "exact r")
    got = download_rows(x)
    assert_params_close(got, ref_x, inp.offsets, 0, "exact round x")
    assert_update_close(got, ref_x, x_host.astype(np.float64), "exact round")

    # Alg. 1 literally, with a supplied consensus variable
    rng = np.random.default_rng(3)
    xc_host = (inp.x[0] + 2e-3 * rng.standard_normal(spec.d)).astype(np.float32)
    xc = upload_tensors(xc_host, inp.offsets)
    for push_from in ("average", "consensus"):
        x = _rows(inp, inp.x)
        plan.pull_then_push(x, xc, pull, push, push_from, r_post_out=r)
        ref_x, ref_r = O.pull_then_push(x_host, xc_host, pull, push, push_from)
        assert_rel(r.cpu().numpy(), ref_r, 1e-4, f"r_post ({push_from})")
        got = download_rows(x)
        assert_params_close(got, ref_x, inp.offsets, 0, f"pull_then_push x ({push_from})")
        assert_update_close(got, ref_x, x_host.astype(np.float64), f"pull_then_push ({push_from})")

    # AdamW step, then fused AdamW round
    a_lr, b1, b2, eps, a_wd = f32(5e-4), f32(0.9), f32(0.999), f32(1e-8), f32(0.01)
    x, m1, m2 = _rows(inp, inp.x), _rows(inp, inp.v), _rows(inp, inp.v)
    plan.local_adamw_step(x, m1, m2, g, a_lr, b1, b2, eps, a_wd, 1)
    zero = np.zeros_like(x_host, dtype=np.float64)
    xo, ao, so = O.local_adamw_step(x_host.astype(np.float64), zero, zero, g_host, a_lr, b1, b2, eps, a_wd, 1)
    assert_params_close(download_rows(x), xo, inp.offsets, 2, "adamw x")
    assert_params_close(download_rows(m1), ao, inp.offsets, 2, "adamw m1")
    assert_params_close(download_rows(m2), so, inp.offsets, 2, "adamw m2")
    g2_host = np.stack(inp.grads(1))
    g2 = _rows(inp, inp.grads(1))
    plan.round_adamw(x, m1, m2, g2, a_lr, b1, b2, eps, a_wd, 2, f32(0.9), push, r_out=r)
    x_pre, ao, so = O.local_adamw_step(xo, ao, so, g2_host, a_lr, b1, b2, eps, a_wd, 2)
    ref_x, ref_r, ref_c, _ = O.pull_push_round(x_pre, f32(0.9), push)
    assert_rel(r.cpu().numpy(), ref_r, 1e-4, "adamw round r")
    got = download_rows(x)
    assert_params_close(got, ref_x, inp.offsets, 4, "adamw round x", c=ref_c)
    assert_params_close(download_rows(m2), so, inp.offsets, 4, "adamw round m2")
    assert_update_close(got, ref_x, x_pre, "adamw round")
    plan.close()


def test_round_statistics_and_schedule():
    M = 5
    r_host = np.array([5.0, 5.0, 8.0, 0.0, 1.5], np.float32)
    r = torch.from_numpy(r_host).cuda()
    out = torch.full((2 * M + 3,), -7.0, device="cuda")
    dppf.round_statistics(r, M, f32(0.5), f32(2.0), out)
    st = O.round_statistics(r_host, f32(0.5), f32(2.0))
    got = out.cpu().numpy()
    assert_rel(got[0], st["relaxed_mv"], 1e-6, "relaxed MV")
    assert_rel(got[1:M + 1], st["pull_strength"], 1e-6, "pull strength")
    assert_rel(got[M + 1:2 * M + 1], st["push_strength"], 1e-6, "push strength")
    assert np.all(got[2 * M + 1:] == -7.0), "without the norm of the average the last two slots stay untouched"
    # with the norm of the average (here a made-up value on the device)
    x_avg = np.array([3.0, -4.0, 12.0])
    na = torch.tensor([13.0], device="cuda")
    dppf.round_statistics(r, M, f32(0.5), f32(2.0), out, avg_norm=na)
    st = O.round_statistics(r_host, f32(0.5), f32(2.0), x_avg=x_avg)
    got = out.cpu().numpy()
    assert_rel(got[2 * M + 1], st["average_norm"], 1e-6, "norm of the average")
    assert_rel(got[2 * M + 2], st["width_over_norm"], 1e-6, "valley width over norm")
    for kind in ("fixed", "decreasing", "increasing"):
        for t in (0, 1, 250, 777, 1000):
            assert abs(dppf.push_schedule(kind, f32(0.5), t, 1000) - O.push_schedule(kind, f32(0.5), t, 1000)) < 1e-7


def test_many_rounds_driver_tracks_the_oracle_and_the_valley_width():
    # tau local steps on pure-noise gradients, then a round, many times: the GPU trajectory must
    # follow the oracle's, and the distances must settle near lambda/alpha (Theorem 1) -- the
    # noise term of the bound, eta*sigma0 accumulated over tau steps and d coordinates, is kept small
    M, d, tau, rounds = 8, 20_000, 4, 40
    spec = W.small_spec(M=M, seed=900, shapes=((d - 7,), (7,)), tau=tau, sigma_grad=2e-4)
    inp = W.make_inputs(spec)
    lr, mu, wd, pull, push = f32(0.1), f32(0.9), 0.0, f32(0.25), f32(0.5)
    plan = dppf.Plan(M, spec.numel)
    x, v = _rows(inp, inp.x), _rows(inp, inp.v)
    xo, vo = np.stack(inp.x).astype(np.float64), np.stack(inp.v).astype(np.float64)
    r = torch.zeros(M, device="cuda")
    step = 0
    for k in range(rounds):
        for _ in range(tau - 1):
            gk = inp.grads(step); step += 1
            plan.local_sgd_step(x, v, _rows(inp, gk), lr, mu, wd)
            xo, vo = O.local_sgd_step(xo, vo, np.stack(gk), lr, mu, wd)
        gk = inp.grads(step); step += 1
        lam_k = dppf.push_schedule("fixed", push, k, rounds)
        plan.round(x, v, _rows(inp, gk), lr, mu, wd, pull, lam_k, r_out=r)
        xo, vo, ro, _, _ = O.dppf_round(xo, vo, np.stack(gk), lr, mu, wd, pull, lam_k)
        assert_rel(r.cpu().numpy(), ro, 1e-4, f"r in round {k}")
    assert_params_close(download_rows(x), xo, inp.offsets, tau * rounds, "x after all rounds")
    final = torch.zeros(M, device="cuda")
    plan.dist_norms(x, final)
    width = final.cpu().numpy()
    assert np.all(np.abs(width - push / pull) < 0.15 * push / pull), width
    plan.close()


def test_decaying_learning_rate_settles_the_valley_width_at_push_over_pull():
    # Theorem 1: the distance of a worker to the average tends to lambda/alpha + O(eta sigma0 + M^-1/2).
    # With a cosine-decayed learning rate and gradient noise large enough to matter (sigma0 = 0.7,
    # lambda/alpha = 2) the width first overshoots -- the eta*sigma0 term -- and then closes in on
    # lambda/alpha as eta goes to zero.  The GPU trajectory is checked against the oracle's all the way.
    M, d, tau, rounds = 8, 20_000, 4, 60
    spec = W.small_spec(M=M, seed=901, shapes=((d - 7,), (7,)), tau=tau, sigma_grad=5e-3)
    inp = W.make_inputs(spec)
    lr0, mu, wd, pull, push = 0.1, f32(0.9), 0.0, f32(0.25), f32(0.5)
    sigma0 = spec.sigma_grad * np.sqrt(d)
    plan = dppf.Plan(M, spec.numel)
    x, v = _rows(inp, inp.x), _rows(inp, inp.v)
    xo, vo = np.stack(inp.x).astype(np.float64), np.stack(inp.v).astype(np.float64)
    r = torch.zeros(M, device="cuda")
    total, t = tau * rounds, 0
    widths, etas = [], []
    for k in range(rounds):
        for s in range(tau):
            eta = f32(0.5 * lr0 * (1.0 + np.cos(np.pi * t / total)))
            gk = inp.grads(t); t += 1
            if s < tau - 1:
                plan.local_sgd_step(x, v, _rows(inp, gk), eta, mu, wd)
                xo, vo = O.local_sgd_step(xo, vo, np.stack(gk), eta, mu, wd)
            else:
                plan.round(x, v, _rows(inp, gk), eta, mu, wd, pull, push, r_out=r)
                xo, vo, ro, _, _ = O.dppf_round(xo, vo, np.stack(gk), eta, mu, wd, pull, push)
                assert_rel(r.cpu().numpy(), ro, 1e-4, f"r in round {k}")
        final = torch.zeros(M, device="cuda")
        plan.dist_norms(x, final)
        widths.append(final.cpu().numpy().astype(np.float64))
        etas.append(eta)
    assert_params_close(download_rows(x), xo, inp.offsets, tau * rounds, "x after all rounds")
    target = push / pull
    mean_width = np.array([w.mean() for w in widths])
    # while eta is large the noise term is visible ...
    assert mean_width[rounds // 5] > 1.2 * target, mean_width[rounds // 5]
    # ... and the excess over lambda/alpha shrinks with eta: within a fixed multiple of eta*sigma0 (plus 1 %)
    late = range(rounds // 2, rounds)
    for k in late:
        assert abs(mean_width[k] - target) <= 12.0 * etas[k] * sigma0 + 0.01 * target, (k, mean_width[k], etas[k])
    assert abs(mean_width[-1] - target) < 0.01 * target, mean_width[-1]
    assert np.all(np.abs(widths[-1] - target) < 0.05 * target), widths[-1]
    plan.close()


@pytest.mark.parametrize("schedule", ["fixed", "increasing"])
def test_alg1_loop_matches_the_oracle(schedule):
    # Alg. 1 end to end through the loop helper: tau-step periods, scheduled push, final average
    from paper_2507_20424_amd.training import DppfLoop
    M, tau, iters = 4, 3, 12
    spec = W.small_spec(M=M, seed=950, tau=tau, weight_decay=1e-3)
    inp = W.make_inputs(spec)
    lr, mu, wd, pull, push = f32(0.1), f32(0.9), f32(1e-3), f32(0.1), f32(0.02)
    x, v = _rows(inp, inp.x), _rows(inp, inp.v)
    g = _rows(inp, inp.v)
    loop = DppfLoop(x, v, g, tau=tau, pull=pull, push=push, lr=lr, momentum=mu, weight_decay=wd,
                    schedule=schedule, total_iterations=iters)
    xo, vo = np.stack(inp.x).astype(np.float64), np.stack(inp.v).astype(np.float64)
    host_g = {}

    def grad_fn(t):
        host_g[t] = inp.grads(t)
        for m in range(M):
            for j, dst in enumerate(g[m]):
                lo, hi = int(inp.offsets[j]), int(inp.offsets[j + 1])
                dst.copy_(torch.from_numpy(host_g[t][m][lo:hi]))

    rounds = 0
    for t in range(iters):
        did_round = loop.step(grad_fn)
        gk = np.stack(host_g[t])
        if (t + 1) % tau == 0:
            assert did_round
            rounds += 1
            lam = f32(O.push_schedule(schedule, push, t + 1, iters))
            xo, vo, ro, co, xa = O.dppf_round(xo, vo, gk, lr, mu, wd, pull, lam)
            mv, pull_strength, push_strength, avg_norm = loop.round_statistics()
            st = O.round_statistics(ro, pull, lam, x_avg=xa)
            assert_rel(mv, st["relaxed_mv"], 1e-4, "relaxed MV")
            assert_rel(pull_strength, st["pull_strength"], 1e-4, "pull strength")
            assert abs(push_strength - lam) <= 1e-7
            assert_rel(avg_norm, st["average_norm"], 1e-4, "norm of the average")
        else:
            assert not did_round
            xo, vo = O.local_sgd_step(xo, vo, gk, lr, mu, wd)
    assert rounds == iters // tau
    assert_params_close(download_rows(x), xo, inp.offsets, iters, "x after the loop")
    avg = upload_tensors(np.zeros(spec.d, np.float32), inp.offsets)
    loop.average(avg)
    assert_params_close(download(avg)[None], O.replica_mean(xo)[None], inp.offsets, iters, "returned average")
    loop.close()


def test_alg1_loop_on_torch_modules_with_autograd_gradients():
    # M replicas of a small network, real backward passes on synthetic regression data; the
    # parameters move through the library, the oracle follows with the downloaded gradients
    from paper_2507_20424_amd.training import DppfLoop
    torch.manual_seed(0)
    M, tau, iters = 4, 2, 6
    lr, mu, wd, pull, push = f32(0.05), f32(0.9), f32(1e-4), f32(0.5), f32(0.05)

    def make():
        return torch.nn.Sequential(torch.nn.Linear(13, 37), torch.nn.Tanh(), torch.nn.Linear(37, 5)).cuda()

    models = [make() for _ in range(M)]
    with torch.no_grad():                                   # Alg. 1: one random init, distributed to all
        for mod in models[1:]:
            for p, q in zip(mod.parameters(), models[0].parameters()):
                p.copy_(q)
    data = [(torch.randn(64, 13, device="cuda"), torch.randn(64, 5, device="cuda")) for _ in range(M)]
    loop = DppfLoop.from_modules(models, tau=tau, pull=pull, push=push, lr=lr, momentum=mu, weight_decay=wd)

    def flat(rows):
        return np.stack([torch.cat([t.reshape(-1) for t in row]).cpu().numpy() for row in rows])

    xo = flat(loop.x).astype(np.float64)
    vo = np.zeros_like(xo)
    numel = [int(t.numel()) for t in loop.x[0]]
    offsets = np.concatenate([[0], np.cumsum(numel)])

    def backward(_t):
        for mod, (inp_, tgt) in zip(models, data):
            mod.zero_grad(set_to_none=True)                 # fresh gradient tensors every iteration
            torch.nn.functional.mse_loss(mod(inp_), tgt).backward()

    for t in range(iters):
        did_round = loop.step(backward)
        go = flat(loop.g)
        if did_round:
            xo, vo, ro, _, _ = O.dppf_round(xo, vo, go, lr, mu, wd, pull, push)
            assert_rel(loop.r.cpu().numpy(), ro, 1e-4, "r")
        else:
            xo, vo = O.local_sgd_step(xo, vo, go, lr, mu, wd)
        # the modules' own parameters are the library's x: compare after every iteration, so the
        # oracle is always fed gradients taken at (numerically) the same point
        got = flat([[p.data for p in mod.parameters()] for mod in models])
        assert_params_close(got, xo, offsets, t + 1, f"parameters after iteration {t}")
        xo = got.astype(np.float64)                          # re-anchor: gradients depend on x itself
    loop.close()
