"""GPU parity at the full sizes of the five benchmark configurations, in the same launch
configuration the benchmark times (separately allocated per-layer tensors, prebuilt pointer
tables, default stream): tau local momentum-SGD steps on seeded synthetic gradients followed by
one pull-push round, every output compared with the CPU oracle element by element, plus the
push-only property ||x_m+ - x_m|| = lambda that holds at any size."""
import numpy as np
import pytest

from parity import (O, assert_average_norm, assert_params_close, assert_rel, assert_update_close, download_rows, f32,
                    oracle_local_steps, upload_tensors)

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2507_20424_amd import dppf, workloads as W  # noqa: E402


def _fill(rows, arrays, offsets):
    for row, a in zip(rows, arrays):
        for t, dst in enumerate(row):
            lo, hi = int(offsets[t]), int(offsets[t + 1])
            if hi > lo:
                dst.copy_(torch.from_numpy(a[lo:hi]))


def _clone(rows):
    return [[t.clone() for t in row] for row in rows]


def _restore(rows, saved):
    for row, srow in zip(rows, saved):
        for t, s in zip(row, srow):
            t.copy_(s)


@pytest.mark.parametrize("name,fused", [("flat1m_M2", False), ("flat1m_M2", True), ("resnet50_M4", False),
                                        ("resnet101_M4", False), ("vitb16_M4", True), ("pyramidnet_M8", False),
                                        ("pyramidnet_M8", True)])
def test_config(name, fused):
    spec = W.SPECS[name]
    print(f"\n[{name} fused={fused}] M={spec.M} T={spec.T} d={spec.d} tau={spec.tau}", flush=True)
    lr, mu, wd = f32(spec.lr), f32(spec.momentum), f32(spec.weight_decay)
    inp = W.make_inputs(spec)
    M, off = spec.M, inp.offsets
    x = [upload_tensors(a, off) for a in inp.x]
    v = [upload_tensors(a, off) for a in inp.v]
    g = [upload_tensors(np.zeros(spec.d, np.float32), off) for _ in range(M)]
    xt, vt, gt = dppf.PointerTable(x), dppf.PointerTable(v), dppf.PointerTable(g)
    r = torch.zeros(M, device="cuda")
    c = torch.zeros(M, device="cuda")
    plan = dppf.Plan(M, spec.numel)

    # ---- all local steps but the last, GPU and oracle side by side
    xo, vo = np.stack(inp.x).astype(np.float64), np.stack(inp.v).astype(np.float64)
    for k in range(spec.tau - 1):
        gk = inp.grads(k)
        _fill(g, gk, off)
        plan.local_sgd_step(xt, vt, gt, lr, mu, wd)
        xo, vo = oracle_local_steps(xo, vo, lambda _k, gk=gk: gk, 1, lr, mu, wd)
        del gk
    if spec.tau > 1:
        assert_params_close(download_rows(x), xo, off, spec.tau - 1, "x after the local steps")
        assert_params_close(download_rows(v), vo, off, spec.tau - 1, "v after the local steps")
        print("  local steps agree", flush=True)

    # ---- last step + round(s)
    g_last = inp.grads(spec.tau - 1)
    _fill(g, g_last, off)
    x_pre, v_ref = oracle_local_steps(xo, vo, lambda _k: g_last, 1, lr, mu, wd)
    del xo, vo
    pairs = [(spec.pull, spec.push)] + list(spec.sweep)
    if fused:
        x_saved, v_saved = _clone(x), _clone(v)
    else:
        plan.local_sgd_step(xt, vt, gt, lr, mu, wd)
        x_saved = _clone(x)
    for pull, push in pairs:
        pull, push = f32(pull), f32(push)
        _restore(x, x_saved)
        if fused:
            _restore(v, v_saved)
            plan.round(xt, vt, gt, lr, mu, wd, pull, push, r_out=r, c_out=c)
        else:
            plan.pull_push_round(xt, pull, push, r_out=r, c_out=c)
        ref_x, ref_r, ref_c, ref_avg = O.pull_push_round(x_pre, pull, push)
        got = download_rows(x)
        print(f"  pull={pull:.3g} push={push:.3g}: r gpu {r.cpu().numpy()} oracle {ref_r}", flush=True)
        assert_rel(r.cpu().numpy(), ref_r, 1e-4, "r")
        assert_rel(c.cpu().numpy(), ref_c, 1e-4, "c")
        assert_average_norm(plan, ref_avg, "round")
        del ref_avg
        assert_params_close(got, ref_x, off, spec.tau, "x after the round")
        assert_update_close(got, ref_x, x_pre, "round")
        del ref_x, got
    assert_params_close(download_rows(v), v_ref, off, spec.tau, "v after the last step")

    # ---- push only (alpha = 0): every worker moves exactly lambda, away from the average
    _restore(x, x_saved)
    lam = f32(spec.push)
    if fused:
        _restore(v, v_saved)
        plan.round(xt, vt, gt, lr, mu, wd, 0.0, lam)
        before = x_pre                                   # the stepped x exists only inside the kernels
    else:
        before = download_rows(x).astype(np.float64)
        plan.pull_push_round(xt, 0.0, lam)
    step = download_rows(x).astype(np.float64) - before
    assert_rel(np.linalg.norm(step, axis=1), np.full(M, lam), 1e-4, "push-only step length")
    avg = before.mean(axis=0)
    assert np.all(np.sum(step * (before - avg), axis=1) > 0), "push-only step does not point away from the average"
    plan.close()


def test_single_tensor_beyond_two_gib():
    # one tensor of 2^29 + 5 floats per worker: byte offsets inside a tensor pass 2^31, the tile
    # list has 131,073 entries and a ragged tail
    d = (1 << 29) + 5
    spec = W.WorkloadSpec("flat_2gib_M2", 2, ((d,),), seed=11, tau=1)
    print(f"\n[{spec.name}] d={d}", flush=True)
    lr, mu, wd, pull, push = f32(spec.lr), f32(spec.momentum), 0.0, f32(spec.pull), f32(spec.push)
    inp = W.make_inputs(spec)
    g_host = inp.grads(0)
    x = [upload_tensors(a, inp.offsets) for a in inp.x]
    v = [upload_tensors(a, inp.offsets) for a in inp.v]
    g = [upload_tensors(a, inp.offsets) for a in g_host]
    r = torch.zeros(2, device="cuda")
    c = torch.zeros(2, device="cuda")
    plan = dppf.Plan(2, spec.numel)
    plan.round(x, v, g, lr, mu, wd, pull, push, r_out=r, c_out=c)
    torch.cuda.synchronize()
    x_pre, v_ref = oracle_local_steps(np.stack(inp.x), np.stack(inp.v), lambda _k: g_host, 1, lr, mu, wd)
    del g_host
    ref_x, ref_r, ref_c, _ = O.pull_push_round(x_pre, pull, push)
    print(f"  r gpu {r.cpu().numpy()} oracle {ref_r}", flush=True)
    assert_rel(r.cpu().numpy(), ref_r, 1e-4, "r")
    assert_rel(c.cpu().numpy(), ref_c, 1e-4, "c")
    got = download_rows(x)
    assert_params_close(got, ref_x, inp.offsets, 1, "x")
    assert_update_close(got, ref_x, x_pre, "round")
    del got, ref_x, x_pre
    assert_params_close(download_rows(v), v_ref, inp.offsets, 1, "v")
    plan.close()
