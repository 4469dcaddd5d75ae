"""The entry point for callers that cannot allocate (dppf_pull_push_round_flat_static) against
the plan-based dppf_pull_push_round_flat: same kernels, so the parameters must agree bit for
bit and the distances and coefficients to rounding.  Two calls in a row on the same GPU, the
second on a smaller problem, because all calls share one static scratch array that keeps the
previous call's contents."""
import numpy as np
import pytest

from parity import O, assert_params_close, assert_rel, f32

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2507_20424_amd import dppf  # noqa: E402


def _workers(M, d, ld, seed, spread=1e-3):
    rng = np.random.default_rng(seed)
    x0 = (0.02 * rng.standard_normal(d)).astype(np.float32)
    host = np.zeros((M, ld), dtype=np.float32)
    for m in range(M):
        host[m, :d] = x0 + (spread * (1 + m) * rng.standard_normal(d)).astype(np.float32)
    host[:, d:] = 7.0           # padding between the workers: must come back untouched
    return host


def _one_case(M, d, ld, seed, pull, push):
    print(f"\n[static round] M={M} d={d} ld={ld} seed={seed}", flush=True)
    host = _workers(M, d, ld, seed)
    pull, push = f32(pull), f32(push)
    # reference: the plan-based flat entry point
    x_plan = torch.from_numpy(host).cuda()
    r_plan = torch.zeros(M, device="cuda"); c_plan = torch.zeros(M, device="cuda")
    plan = dppf.Plan(M, [d])
    plan.pull_push_round_flat(x_plan, ld, pull, push, r_out=r_plan, c_out=c_plan)
    torch.cuda.synchronize()
    plan.close()
    # under test: no plan, no allocation inside the call (the outputs are allocated here, before it)
    x_stat = torch.from_numpy(host).cuda()
    r_stat = torch.full((M,), -1.0, device="cuda"); c_stat = torch.full((M,), -1.0, device="cuda")
    torch.cuda.synchronize()
    dppf.pull_push_round_flat_static(x_stat, M, d, ld, pull, push, r_out=r_stat, c_out=c_stat)
    torch.cuda.synchronize()
    got, want = x_stat.cpu().numpy(), x_plan.cpu().numpy()
    assert np.array_equal(got[:, d:], host[:, d:]), "padding between the workers was written"
    assert np.array_equal(got, want), f"parameters differ from the plan-based call: {np.abs(got - want).max()}"
    assert_rel(r_stat.cpu().numpy(), r_plan.cpu().numpy(), 1e-6, "r against the plan-based call")
    assert_rel(c_stat.cpu().numpy(), c_plan.cpu().numpy(), 1e-6, "c against the plan-based call")
    # and against the oracle, to the bar of every other parity test
    if d > 0:
        ref_x, ref_r, ref_c, _ = O.pull_push_round(host[:, :d], pull, push)
        assert_rel(r_stat.cpu().numpy(), ref_r, 1e-4, "r")
        assert_rel(c_stat.cpu().numpy(), ref_c, 1e-4, "c")
        assert_params_close(got[:, :d], ref_x, np.array([0, d]), 0, "x", c=ref_c)
    else:
        assert np.all(r_stat.cpu().numpy() == 0.0) and np.all(c_stat.cpu().numpy() == pull)


def test_static_round_matches_the_plan_based_round_twice_in_a_row():
    # large enough that sweep 2 takes part of its tiles on demand (the counter lives in the static
    # scratch), ragged tail, workers not 16-byte aligned relative to one another (odd ld) ...
    _one_case(M=4, d=4096 * 1500 + 77, ld=4096 * 1500 + 77 + 3, seed=31, pull=0.1, push=0.01)
    # ... then a much smaller problem with other M: stale tiles, pointers and sums must not leak in
    _one_case(M=3, d=5001, ld=5001, seed=32, pull=0.3, push=0.5)
    # the register-resident limit, a single partial tile, and an empty model
    _one_case(M=16, d=4096 * 40 + 1, ld=4096 * 41, seed=33, pull=0.1, push=0.01)
    _one_case(M=2, d=3, ld=8, seed=34, pull=0.2, push=0.05)
    _one_case(M=2, d=0, ld=4, seed=35, pull=0.2, push=0.05)


def test_static_round_rejects_what_does_not_fit():
    lib = dppf.load()
    x = torch.zeros(64, device="cuda")
    assert lib.dppf_pull_push_round_flat_static(x.data_ptr(), 17, 2, 2, 0.1, 0.1, None, None, None) == -4
    assert lib.dppf_pull_push_round_flat_static(x.data_ptr(), 2, (1 << 27) + 1, (1 << 27) + 1, 0.1, 0.1, None, None,
                                                None) == -4
    assert lib.dppf_pull_push_round_flat_static(x.data_ptr(), 0, 2, 2, 0.1, 0.1, None, None, None) == -1
    assert lib.dppf_pull_push_round_flat_static(x.data_ptr(), 2, 8, 4, 0.1, 0.1, None, None, None) == -1
    assert lib.dppf_pull_push_round_flat_static(None, 2, 8, 8, 0.1, 0.1, None, None, None) == -1
    assert lib.dppf_pull_push_round_flat_static(x.data_ptr() + 2, 2, 8, 8, 0.1, 0.1, None, None, None) == -1
    torch.cuda.synchronize()
    assert torch.all(x == 0)
