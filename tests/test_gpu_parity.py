"""GPU parity: every entry point of the C ABI against the CPU oracle on the same seeded
inputs, element by element, on lists that span several tiles and have ragged tails, plus the
degenerate cases of the method."""
import numpy as np
import pytest

from parity import (O, assert_average_norm, assert_gap_close, assert_params_close, assert_rel, assert_update_close,
                    download, download_rows, f32, upload_tensors)

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2507_20424_amd import dppf, workloads as W  # noqa: E402


def _dev_rows(inp, arrays, misalign=0):
    return [upload_tensors(a, inp.offsets, misalign) for a in arrays]


def _hyper(spec):
    return dict(lr=f32(spec.lr), mu=f32(spec.momentum), wd=f32(spec.weight_decay), pull=f32(spec.pull),
                push=f32(spec.push))


WORKER_COUNTS = [1, 2, 3, 4, 5, 6, 7, 8, 9, 11, 16, 17, 24, 33, 39, 40, 45]


@pytest.mark.parametrize("M", WORKER_COUNTS)
@pytest.mark.parametrize("misalign", [0, 1])
def test_round_small_lists(M, misalign):
    spec = W.small_spec(M=M, seed=100 + M)
    h = _hyper(spec)
    inp = W.make_inputs(spec)
    x_host = np.stack(inp.x)
    x = _dev_rows(inp, inp.x, misalign)
    xbar = upload_tensors(np.zeros(spec.d, np.float32), inp.offsets, misalign)
    r = torch.zeros(M, device="cuda")
    c = torch.zeros(M, device="cuda")
    plan = dppf.Plan(M, spec.numel)

    ref_new, ref_r, ref_c, ref_avg = O.pull_push_round(x_host, h["pull"], h["push"])

    # the pieces on their own
    plan.replica_mean(x, xbar)
    assert_params_close(download(xbar)[None], ref_avg[None], inp.offsets, 0, "replica_mean")
    plan.dist_norms(x, r)
    if M > 1:
        assert_rel(r.cpu().numpy(), ref_r, 1e-4, "dist_norms")
    r.zero_()
    plan.dist_norms(x, r, xbar=xbar)
    if M > 1:
        assert_rel(r.cpu().numpy(), O.dist_norms(x_host, download(xbar)), 1e-4, "dist_norms(given average)")
    assert np.array_equal(download_rows(x), x_host), "read-only entry points changed x"

    # the round
    xbar2 = upload_tensors(np.zeros(spec.d, np.float32), inp.offsets, misalign)
    plan.pull_push_round(x, h["pull"], h["push"], r_out=r, c_out=c, xbar_out=xbar2)
    got = download_rows(x)
    if M > 1:
        assert_rel(r.cpu().numpy(), ref_r, 1e-4, "r")
        assert_rel(c.cpu().numpy(), ref_c, 1e-4, "c")
    assert_params_close(got, ref_new, inp.offsets, 0, "pull_push_round x")
    assert_update_close(got, ref_new, x_host.astype(np.float64), "pull_push_round")
    assert_params_close(download(xbar2)[None], ref_avg[None], inp.offsets, 0, "xbar_out")
    assert_average_norm(plan, ref_avg, "pull_push_round")
    plan.close()


@pytest.mark.parametrize("M", [2, 4, 8, 9, 16, 19, 39, 41])
@pytest.mark.parametrize("wd", [0.0, 1e-3])
def test_local_step_and_fused_round(M, wd):
    spec = W.small_spec(M=M, seed=200 + M, tau=3, weight_decay=wd)
    h = _hyper(spec)
    inp = W.make_inputs(spec)
    plan = dppf.Plan(M, spec.numel)
    x = _dev_rows(inp, inp.x, 2)
    v = _dev_rows(inp, inp.v, 3)
    xo, vo = np.stack(inp.x).astype(np.float64), np.stack(inp.v).astype(np.float64)
    # tau - 1 stand-alone steps, then the fused last step + round
    for k in range(spec.tau - 1):
        gk = inp.grads(k)
        g = _dev_rows(inp, gk, 1)
        plan.local_sgd_step(x, v, g, h["lr"], h["mu"], h["wd"])
        xo, vo = O.local_sgd_step(xo, vo, np.stack(gk), h["lr"], h["mu"], h["wd"])
        assert_params_close(download_rows(x), xo, inp.offsets, k + 1, f"local step {k} x")
        assert_params_close(download_rows(v), vo, inp.offsets, k + 1, f"local step {k} v")
    gk = inp.grads(spec.tau - 1)
    g = _dev_rows(inp, gk, 0)
    g_before = download_rows(g)
    r = torch.zeros(M, device="cuda")
    c = torch.zeros(M, device="cuda")
    xbar = upload_tensors(np.zeros(spec.d, np.float32), inp.offsets)
    x_pre, _ = O.local_sgd_step(xo, vo, np.stack(gk), h["lr"], h["mu"], h["wd"])
    ref_x, ref_v, ref_r, ref_c, ref_avg = O.dppf_round(xo, vo, np.stack(gk), h["lr"], h["mu"], h["wd"],
                                                       h["pull"], h["push"])
    plan.round(x, v, g, h["lr"], h["mu"], h["wd"], h["pull"], h["push"], r_out=r, c_out=c, xbar_out=xbar)
    got_x, got_v = download_rows(x), download_rows(v)
    assert_rel(r.cpu().numpy(), ref_r, 1e-4, "fused r")
    assert_rel(c.cpu().numpy(), ref_c, 1e-4, "fused c")
    assert_params_close(got_x, ref_x, inp.offsets, spec.tau, "fused x")
    assert_params_close(got_v, ref_v, inp.offsets, spec.tau, "fused v")
    assert_params_close(download(xbar)[None], ref_avg[None], inp.offsets, spec.tau, "fused xbar")
    assert_update_close(got_x, ref_x, x_pre, "fused round")
    assert_average_norm(plan, ref_avg, "fused round")
    assert np.array_equal(download_rows(g), g_before), "gradients were modified"
    plan.close()


def test_fused_equals_step_then_round_bitwise():
    # dppf_round is defined as dppf_local_sgd_step followed by dppf_pull_push_round
    spec = W.small_spec(M=4, seed=31)
    h = _hyper(spec)
    inp = W.make_inputs(spec)
    gk = inp.grads(0)
    plan = dppf.Plan(4, spec.numel)
    res = []
    for fused in (True, False):
        x, v, g = _dev_rows(inp, inp.x), _dev_rows(inp, inp.v), _dev_rows(inp, gk)
        r = torch.zeros(4, device="cuda")
        if fused:
            plan.round(x, v, g, h["lr"], h["mu"], h["wd"], h["pull"], h["push"], r_out=r)
        else:
            plan.local_sgd_step(x, v, g, h["lr"], h["mu"], h["wd"])
            plan.pull_push_round(x, h["pull"], h["push"], r_out=r)
        res.append((download_rows(x), download_rows(v), r.cpu().numpy()))
    assert np.array_equal(res[0][0], res[1][0]) and np.array_equal(res[0][1], res[1][1])
    assert np.array_equal(res[0][2], res[1][2])
    plan.close()


@pytest.mark.parametrize("M", [2, 3, 4, 7, 8, 12, 21])
def test_identical_replicas_do_not_move(M):
    # zero distance: no direction, no displacement, r = 0, c = alpha, no NaN/Inf -- bit for bit,
    # negative zeros included
    spec = W.small_spec(M=M, seed=5)
    inp = W.make_inputs(spec)
    row = inp.x[0].copy()
    row[::7] = -0.0
    rows = [row.copy() for _ in range(M)]
    x = _dev_rows(inp, rows, 1)
    r = torch.full((M,), -1.0, device="cuda")
    c = torch.full((M,), -1.0, device="cuda")
    plan = dppf.Plan(M, spec.numel)
    plan.pull_push_round(x, f32(0.3), f32(0.7), r_out=r, c_out=c)
    got = download_rows(x)
    assert np.array_equal(got.view(np.uint32), np.stack(rows).view(np.uint32))
    assert np.all(r.cpu().numpy() == 0.0)
    assert np.all(c.cpu().numpy() == np.float32(0.3))
    plan.close()


def test_one_worker_on_the_average():
    # worker 2 sits exactly on the average of the other two: it must stay, the others move
    base = ((np.arange(5000) - 2500) / 1024.0).astype(np.float32)      # exact in binary
    delta = np.full(5000, 0.25, np.float32)
    rows = [base - delta, base + delta, base.copy()]
    x_host = np.stack(rows)
    offsets = np.array([0, 5000])
    x = [upload_tensors(a, offsets) for a in rows]
    r = torch.zeros(3, device="cuda")
    plan = dppf.Plan(3, [5000])
    plan.pull_push_round(x, f32(0.5), f32(0.25), r_out=r)
    ref_new, ref_r, _, _ = O.pull_push_round(x_host, f32(0.5), f32(0.25))
    got = download_rows(x)
    assert ref_r[2] == 0.0 and r.cpu().numpy()[2] == 0.0
    assert np.array_equal(got[2], rows[2])
    assert_params_close(got, ref_new, offsets, 0, "x")
    plan.close()


def test_special_cases_of_the_update():
    spec = W.small_spec(M=4, seed=9)
    inp = W.make_inputs(spec)
    x_host = np.stack(inp.x).astype(np.float64)
    avg = x_host.mean(axis=0)
    plan = dppf.Plan(4, spec.numel)
    # alpha = 1, lambda = 0: everybody lands on the average (LocalSGD / gradient averaging)
    x = _dev_rows(inp, inp.x)
    plan.pull_push_round(x, 1.0, 0.0)
    got = download_rows(x)
    for m in range(4):
        assert np.max(np.abs(got[m] - avg)) <= 2 * 2.0 ** -24 * np.max(np.abs(avg))
    # lambda = 0: the average is preserved, gaps shrink by (1 - alpha)
    x = _dev_rows(inp, inp.x)
    r0 = torch.zeros(4, device="cuda")
    r1 = torch.zeros(4, device="cuda")
    plan.pull_push_round(x, f32(0.25), 0.0, r_out=r0)
    got = download_rows(x).astype(np.float64)
    assert np.max(np.abs(got.mean(axis=0) - avg)) <= 4 * 2.0 ** -24 * np.max(np.abs(avg))
    plan.dist_norms(x, r1)
    assert_rel(r1.cpu().numpy(), 0.75 * r0.cpu().numpy().astype(np.float64), 1e-4, "gap shrink")
    # alpha = 0: every worker moves exactly lambda, away from the average
    x = _dev_rows(inp, inp.x)
    lam = f32(0.05)
    plan.pull_push_round(x, 0.0, lam)
    got = download_rows(x).astype(np.float64)
    step = got - x_host
    assert_rel(np.linalg.norm(step, axis=1), np.full(4, lam), 1e-4, "push-only step length")
    assert np.all(np.sum(step * (x_host - avg), axis=1) > 0)
    plan.close()


def test_empty_and_tiny_lists():
    # no tensors at all; tensors of size zero inside a list; d smaller than one vector
    r = torch.full((3,), -1.0, device="cuda")
    c = torch.full((3,), -1.0, device="cuda")
    plan = dppf.Plan(3, [])
    plan.pull_push_round([[], [], []], f32(0.1), f32(0.2), r_out=r, c_out=c)
    assert np.all(r.cpu().numpy() == 0) and np.all(c.cpu().numpy() == np.float32(0.1))
    plan.close()

    spec = W.small_spec(M=2, seed=3, shapes=((0,), (1,), (0,), (2,), (0,)))
    inp = W.make_inputs(spec)
    x = _dev_rows(inp, inp.x)
    plan = dppf.Plan(2, spec.numel)
    r = torch.zeros(2, device="cuda")
    plan.pull_push_round(x, f32(0.1), f32(0.01), r_out=r)
    ref_new, ref_r, _, _ = O.pull_push_round(np.stack(inp.x), f32(0.1), f32(0.01))
    assert_rel(r.cpu().numpy(), ref_r, 1e-4, "r")
    assert_params_close(download_rows(x), ref_new, inp.offsets, 0, "x")
    plan.close()


def test_flat_forms_with_padding():
    M, d, ld = 4, 10_001, 10_240
    spec = W.small_spec(M=M, seed=17, shapes=((d,),))
    h = _hyper(spec)
    inp = W.make_inputs(spec)
    gk = inp.grads(0)

    def padded(rows, fill):
        buf = torch.full((M, ld), fill, dtype=torch.float32, device="cuda")
        buf[:, :d] = torch.from_numpy(np.stack(rows)).cuda()
        return buf

    x, v, g = padded(inp.x, 7.0), padded(inp.v, 8.0), padded(gk, 9.0)
    r = torch.zeros(M, device="cuda")
    c = torch.zeros(M, device="cuda")
    xbar = torch.zeros(d, device="cuda")
    plan = dppf.Plan(M, [d])
    xo, vo = O.local_sgd_step(np.stack(inp.x), np.stack(inp.v), np.stack(gk), h["lr"], h["mu"], h["wd"])
    plan.local_sgd_step_flat(x, v, g, ld, h["lr"], h["mu"], h["wd"])
    assert_params_close(x[:, :d].cpu().numpy(), xo, inp.offsets, 1, "flat step x")
    ref_x, ref_v, ref_r, ref_c, ref_avg = O.dppf_round(xo, vo, np.stack(gk), h["lr"], h["mu"], h["wd"],
                                                       h["pull"], h["push"])
    plan.round_flat(x, v, g, ld, h["lr"], h["mu"], h["wd"], h["pull"], h["push"], r_out=r, c_out=c, xbar_out=xbar)
    assert_params_close(x[:, :d].cpu().numpy(), ref_x, inp.offsets, 2, "flat fused x")
    assert_params_close(v[:, :d].cpu().numpy(), ref_v, inp.offsets, 2, "flat fused v")
    assert_rel(r.cpu().numpy(), ref_r, 1e-4, "flat r")
    assert_params_close(xbar.cpu().numpy()[None], ref_avg[None], inp.offsets, 2, "flat xbar")
    x2, r2, c2, _ = O.pull_push_round(ref_x, h["pull"], h["push"])
    plan.pull_push_round_flat(x, ld, h["pull"], h["push"], r_out=r, c_out=c)
    assert_rel(r.cpu().numpy(), r2, 1e-4, "flat round r")
    assert_params_close(x[:, :d].cpu().numpy(), x2, inp.offsets, 3, "flat round x")
    # the padding between workers is never touched
    assert torch.all(x[:, d:] == 7.0) and torch.all(v[:, d:] == 8.0) and torch.all(g[:, d:] == 9.0)
    plan.close()


def test_argument_errors_on_device():
    plan = dppf.Plan(2, [8, 8])
    a = torch.zeros(16, device="cuda")
    good = [[a[:8], a[8:]], [a[:8], a[8:]]]
    with pytest.raises(dppf.DppfError):
        plan.pull_push_round([[a[:8]], [a[:8]]], 0.1, 0.1)            # wrong table length
    lib = dppf.load()
    import ctypes
    tab = dppf.PointerTable(good)
    tab.array[1] = tab.array[1] + 2                                    # not 4-byte aligned
    assert lib.dppf_pull_push_round(plan._h, tab.ptr, 0.1, 0.1, None, None, None, None) == -1
    tab.array[1] = None                                                # null tensor of nonzero size
    assert lib.dppf_pull_push_round(plan._h, tab.ptr, 0.1, 0.1, None, None, None, None) == -1
    assert lib.dppf_dist_norms(plan._h, dppf.PointerTable(good).ptr, None, None, None) == -1
    flat_plan = dppf.Plan(2, [8])
    assert lib.dppf_pull_push_round_flat(flat_plan._h, ctypes.c_void_p(a.data_ptr()), 4, 0.1, 0.1, None, None,
                                         None, None) == -1             # ld < d
    assert lib.dppf_pull_push_round_flat(plan._h, ctypes.c_void_p(a.data_ptr()), 8, 0.1, 0.1, None, None,
                                         None, None) == -1             # plan has T != 1
    torch.cuda.synchronize()
    assert torch.all(a == 0)
    plan.close()
    flat_plan.close()


def test_results_are_reproducible_bitwise():
    spec = W.small_spec(M=4, seed=77, shapes=((300_000,), (17,), (123_457,)))
    inp = W.make_inputs(spec)
    plan = dppf.Plan(4, spec.numel)
    outs = []
    for _ in range(3):
        x = _dev_rows(inp, inp.x)
        r = torch.zeros(4, device="cuda")
        plan.pull_push_round(x, f32(0.1), f32(0.01), r_out=r)
        outs.append((download_rows(x), r.cpu().numpy()))
    for o in outs[1:]:
        assert np.array_equal(o[0], outs[0][0]) and np.array_equal(o[1], outs[0][1])
    plan.close()


@pytest.mark.parametrize("M", [2, 17, 40])
def test_pointer_tables_can_change_between_calls(M):
    # every kernel family reads the tables its own way (M = 17 and 40 entry by entry inside the loop
    # over the workers): a table that changed since the last launch must be seen by the next one
    spec = W.small_spec(M=M, seed=41)
    inp = W.make_inputs(spec)
    plan = dppf.Plan(M, spec.numel)
    ref_new, ref_r, _, _ = O.pull_push_round(np.stack(inp.x), f32(0.1), f32(0.01))
    r = torch.zeros(M, device="cuda")
    keep = []
    for _ in range(3):                       # fresh allocations every time -> new tables
        x = _dev_rows(inp, inp.x)
        keep.append(x)                       # so that no allocation is handed out twice
        plan.pull_push_round(x, f32(0.1), f32(0.01), r_out=r)
        assert_params_close(download_rows(x), ref_new, inp.offsets, 0, "x")
        assert_rel(r.cpu().numpy(), ref_r, 1e-4, "r")
    for x in keep[:-1]:                      # the earlier sets were updated once, not again
        assert_params_close(download_rows(x), ref_new, inp.offsets, 0, "x of an earlier call")
    plan.close()


def test_non_default_stream_and_timing_records():
    spec = W.small_spec(M=4, seed=43)
    h = _hyper(spec)
    inp = W.make_inputs(spec)
    gk = inp.grads(0)
    plan = dppf.Plan(4, spec.numel)
    s = torch.cuda.Stream()
    x, v, g = _dev_rows(inp, inp.x), _dev_rows(inp, inp.v), _dev_rows(inp, gk)
    r = torch.zeros(4, device="cuda")
    torch.cuda.synchronize()
    plan.timing_enable(True)
    with torch.cuda.stream(s):
        plan.round(x, v, g, h["lr"], h["mu"], h["wd"], h["pull"], h["push"], r_out=r)
    recs = plan.timing_read()
    plan.timing_enable(False)
    assert [name for name, _ in recs] == ["step_reduce", "step_update"]
    assert all(ms > 0 for _, ms in recs)
    s.synchronize()
    ref_x, _, ref_r, _, _ = O.dppf_round(np.stack(inp.x), np.stack(inp.v), np.stack(gk), h["lr"], h["mu"],
                                         h["wd"], h["pull"], h["push"])
    assert_params_close(download_rows(x), ref_x, inp.offsets, 1, "x on a side stream")
    assert_rel(r.cpu().numpy(), ref_r, 1e-4, "r")
    assert plan.timing_read() == []
    plan.close()


def test_round_captured_in_a_hip_graph_replays_like_eager_calls():
    # the entry points only enqueue, so a fused round can be captured once and replayed; every
    # replay (with eager work and synchronisation in between) must equal the eager call bit for bit
    spec = W.small_spec(M=4, seed=59, shapes=((50_000,), (333,), (70_001,)))
    h = _hyper(spec)
    inp = W.make_inputs(spec)
    gk = inp.grads(0)
    plan_a, plan_b = dppf.Plan(4, spec.numel), dppf.Plan(4, spec.numel)
    xa, va, ga = _dev_rows(inp, inp.x), _dev_rows(inp, inp.v), _dev_rows(inp, gk)
    xb, vb, gb = _dev_rows(inp, inp.x), _dev_rows(inp, inp.v), _dev_rows(inp, gk)
    ra = torch.zeros(4, device="cuda")
    rb = torch.zeros(4, device="cuda")
    ta = [dppf.PointerTable(t) for t in (xa, va, ga)]
    tb = [dppf.PointerTable(t) for t in (xb, vb, gb)]
    args = (h["lr"], h["mu"], h["wd"], h["pull"], h["push"])
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):                 # first call uploads the pointer tables
        plan_a.round(*ta, *args, r_out=ra)
    side.synchronize()
    plan_b.round(*tb, *args, r_out=rb)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        plan_a.round(*ta, *args, r_out=ra)
    for k in range(4):
        graph.replay()
        plan_b.round(*tb, *args, r_out=rb)        # eager twin
        torch.cuda.synchronize()
        scratch = torch.randn(1 << 16, device="cuda").sum().item()   # unrelated eager work between replays
        assert np.isfinite(scratch)
        assert np.array_equal(download_rows(xa), download_rows(xb)), f"replay {k}: x differs"
        assert np.array_equal(download_rows(va), download_rows(vb)), f"replay {k}: v differs"
        assert np.array_equal(ra.cpu().numpy(), rb.cpu().numpy()), f"replay {k}: r differs"
    plan_a.close()
    plan_b.close()


def test_on_demand_tail_is_reproducible_and_leaves_its_counter_clean():
    # Lists with several tiles per block hand the tail of every read-write sweep out on demand
    # (which block takes which tile then differs from run to run).  The results must not: the same
    # bits every time, in eager calls and in replays of a captured graph whose kernels find the
    # counter as the previous launch left it.
    shapes = ((3_000_000,), (1_234_567,), (2_000_003,), (777,))
    spec = W.small_spec(M=2, seed=91, shapes=shapes)
    _, nfull, _ = dppf.layout_tiles(spec.numel, dppf.sweep_tile_elems(2))
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert nfull >= 4 * cus, "the list must be long enough for the on-demand part of the walk"
    h = _hyper(spec)
    inp = W.make_inputs(spec)
    gk = inp.grads(0)
    args = (h["lr"], h["mu"], h["wd"], h["pull"], h["push"])
    ref_x, ref_v, ref_r, _, _ = O.dppf_round(np.stack(inp.x), np.stack(inp.v), np.stack(gk), *args)
    plan = dppf.Plan(2, spec.numel)
    outs = []
    for _ in range(3):
        x, v, g = _dev_rows(inp, inp.x), _dev_rows(inp, inp.v), _dev_rows(inp, gk)
        r = torch.zeros(2, device="cuda")
        plan.round(x, v, g, *args, r_out=r)
        outs.append((download_rows(x), download_rows(v), r.cpu().numpy()))
    assert_params_close(outs[0][0], ref_x, inp.offsets, 1, "x")
    assert_rel(outs[0][2], ref_r, 1e-4, "r")
    for o in outs[1:]:
        assert all(np.array_equal(a, b) for a, b in zip(o, outs[0]))

    # graph: a local step and a fused round (three kernels, so an odd number of launches per replay)
    plan_b = dppf.Plan(2, spec.numel)
    xa, va, ga = _dev_rows(inp, inp.x), _dev_rows(inp, inp.v), _dev_rows(inp, gk)
    xb, vb, gb = _dev_rows(inp, inp.x), _dev_rows(inp, inp.v), _dev_rows(inp, gk)
    ra, rb = torch.zeros(2, device="cuda"), torch.zeros(2, device="cuda")
    ta = [dppf.PointerTable(t) for t in (xa, va, ga)]
    tb = [dppf.PointerTable(t) for t in (xb, vb, gb)]

    def both(p, t, r):
        p.local_sgd_step(*t, h["lr"], h["mu"], h["wd"])
        p.round(*t, *args, r_out=r)

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):                 # first call uploads the pointer tables
        both(plan, ta, ra)
    side.synchronize()
    both(plan_b, tb, rb)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        both(plan, ta, ra)
    for k in range(3):
        graph.replay()
        both(plan_b, tb, rb)
        torch.cuda.synchronize()
        assert np.array_equal(download_rows(xa), download_rows(xb)), f"replay {k}: x differs"
        assert np.array_equal(download_rows(va), download_rows(vb)), f"replay {k}: v differs"
        assert np.array_equal(ra.cpu().numpy(), rb.cpu().numpy()), f"replay {k}: r differs"
    plan.close()
    plan_b.close()


@pytest.mark.parametrize("pull,push,wd", [(0.1, 0.5, 1e-3), (0.1, 0.75, 1e-3), (0.1, 1.0, 1e-4), (0.5, 5.0, 1e-4),
                                          (0.9, 9.0, 1e-4), (0.9, 90.0, 0.0), (1.0, 0.0, 1e-3), (0.05, 0.05, 0.0)])
def test_fused_round_with_the_hyperparameters_the_paper_uses(pull, push, wd):
    # (alpha, lambda) pairs and weight decays from the paper's experiment sections: alpha = 0.1 with
    # lambda 0.5..1.0 (CIFAR), lambda/alpha = 10 (ImageNet CNNs), alpha = 0.9 with lambda = 90 (ViT),
    # full consensus alpha = 1, lambda = 0 (LocalSGD)
    spec = W.small_spec(M=4, seed=600, tau=1, pull=pull, push=push, weight_decay=wd)
    h = _hyper(spec)
    inp = W.make_inputs(spec)
    gk = inp.grads(0)
    x, v, g = _dev_rows(inp, inp.x), _dev_rows(inp, inp.v), _dev_rows(inp, gk)
    r = torch.zeros(4, device="cuda")
    c = torch.zeros(4, device="cuda")
    plan = dppf.Plan(4, spec.numel)
    plan.round(x, v, g, h["lr"], h["mu"], h["wd"], h["pull"], h["push"], r_out=r, c_out=c)
    x_pre, _ = O.local_sgd_step(np.stack(inp.x), np.stack(inp.v), np.stack(gk), h["lr"], h["mu"], h["wd"])
    ref_x, ref_v, ref_r, ref_c, _ = O.dppf_round(np.stack(inp.x), np.stack(inp.v), np.stack(gk), h["lr"], h["mu"],
                                                 h["wd"], h["pull"], h["push"])
    got = download_rows(x)
    assert_rel(r.cpu().numpy(), ref_r, 1e-4, "r")
    assert_rel(c.cpu().numpy(), ref_c, 1e-4, "c")
    assert_params_close(got, ref_x, inp.offsets, 1, "x", c=ref_c)
    assert_params_close(download_rows(v), ref_v, inp.offsets, 1, "v")
    assert_update_close(got, ref_x, x_pre, "round")
    # The same hyper-parameters on the plain round, started from identical float32 numbers on both
    # sides: here nothing excuses an amplified tolerance, however strong the push -- every worker's
    # new gap to the average must agree to 1e-5.
    x_in = np.stack(inp.x)
    x2 = _dev_rows(inp, inp.x)
    plan.pull_push_round(x2, h["pull"], h["push"], r_out=r, c_out=c)
    ref2, ref_r2, ref_c2, ref_avg2 = O.pull_push_round(x_in, h["pull"], h["push"])
    assert_rel(r.cpu().numpy(), ref_r2, 1e-4, "r (plain round)")
    assert_rel(c.cpu().numpy(), ref_c2, 1e-4, "c (plain round)")
    assert_gap_close(download_rows(x2), ref2, ref_avg2, x_in, inp.offsets, f"plain round, pull {pull} push {push}")
    plan.close()


def test_non_finite_inputs_propagate_without_hanging():
    # an Inf in one worker makes its distance infinite; nothing hangs, nothing outside the
    # affected coordinates' arithmetic turns into garbage silently
    spec = W.small_spec(M=4, seed=61)
    inp = W.make_inputs(spec)
    rows = [a.copy() for a in inp.x]
    rows[1][12345] = np.inf
    x = _dev_rows(inp, rows)
    r = torch.zeros(4, device="cuda")
    c = torch.zeros(4, device="cuda")
    plan = dppf.Plan(4, spec.numel)
    plan.pull_push_round(x, f32(0.1), f32(0.01), r_out=r, c_out=c)
    torch.cuda.synchronize()
    rr = r.cpu().numpy()
    assert not np.all(np.isfinite(rr))
    got = download_rows(x)
    mask = np.ones(spec.d, bool)
    mask[12345] = False
    assert np.isfinite(got[:, 12345]).sum() < 4
    # workers with a finite distance keep finite values away from the poisoned coordinate
    for m in range(4):
        if np.isfinite(rr[m]):
            assert np.all(np.isfinite(got[m][mask]))
    plan.close()


def test_measurement_utilities():
    n = 1_000_003
    src = torch.randn(n, device="cuda")
    dst = torch.zeros(n + 8, device="cuda")
    dppf.util_copy(dst, src, n)
    assert torch.equal(dst[:n], src) and torch.all(dst[n:] == 0)
    dppf.util_copy(dst[1:], src[3:], n - 3)                      # 4-byte aligned only
    assert torch.equal(dst[1:n - 2], src[3:])
    lib = dppf.load()
    import ctypes
    assert lib.dppf_util_copy(ctypes.c_void_p(dst.data_ptr() + 2), ctypes.c_void_p(src.data_ptr()), 8, None) == -1
    # streaming probe: every written stream holds (w + 1) * (sum of the read streams)
    streams, length = 6, 16384 * 3
    stride = length + 64
    buf = torch.zeros(streams * stride, device="cuda")
    for k in range(4):
        buf[k * stride:k * stride + length] = float(k + 1)
    dppf.util_stream_probe(buf, stride, length, 4, 0, False, 1)   # read only: nothing changes
    assert torch.all(buf[4 * stride:] == 0)
    assert lib.dppf_util_stream_probe(ctypes.c_void_p(buf.data_ptr()), stride, length, 3, 3, 0, 1, 0, None) == -1
    dppf.util_stream_probe(buf, stride, length, 1, 1, False, 2)   # copy stream 0 -> stream 1
    assert torch.all(buf[stride:stride + length] == 1.0) and torch.all(buf[stride + length:2 * stride] == 0)
    # the same with part of the work handed out on demand, on an array long enough for that
    length = 16384 * 4096       # 1024 items of 16 tiles: four per block on 256 CUs
    big = torch.zeros(3 * length, device="cuda")
    big[:length] = torch.arange(length, device="cuda", dtype=torch.float32) % 1000.0
    for _ in range(2):                                              # twice: the counter must come back clean
        big[length:].zero_()
        dppf.util_stream_probe(big, length, length, 1, 1, False, 1, on_demand=True)
        assert torch.equal(big[length:2 * length], big[:length]) and torch.all(big[2 * length:] == 0)


def test_grouped_stream_probe_sums_each_group_into_its_first_array():
    lib = dppf.load()
    import ctypes
    groups, per_group, vectors, ahead = 8, 3, 2, 7
    tile = 256 * vectors * 4
    length = tile * 1500 + 100                       # the tail past the last whole tile stays untouched
    stride = length + 64
    for on_demand in (False, True):
        buf = torch.zeros(groups * per_group * stride, device="cuda")
        for k in range(groups * per_group):
            buf[k * stride:k * stride + length] = float(k + 1)
        before = buf.clone()
        dppf.util_stream_probe_grouped(buf, stride, length, groups, per_group, vectors, ahead, 1, on_demand)
        whole = tile * 1500
        for j in range(groups):
            first = j * per_group
            want = float(sum(first + r + 1 for r in range(per_group)))
            got = buf[first * stride:first * stride + stride]
            assert torch.all(got[:whole] == want)
            assert torch.equal(got[whole:], before[first * stride + whole:(first + 1) * stride])
            for r in range(1, per_group):
                k = first + r
                assert torch.equal(buf[k * stride:(k + 1) * stride], before[k * stride:(k + 1) * stride])
    buf = torch.zeros(12 * stride, device="cuda")
    assert lib.dppf_util_stream_probe_grouped(ctypes.c_void_p(buf.data_ptr()), stride, length, 5, 3, 4, 0, 1, 0,
                                              None) == -1


@pytest.mark.parametrize("M", [12, 17, 35])
def test_many_workers_on_a_list_that_fills_the_chip(M):
    # M = 12: register-resident sweeps on 2048-element tiles; M = 17, 35: every worker's vector staged
    # in LDS (1024-element tiles); here with more tiles than compute units, so part of the tiles is
    # handed out on demand and the partial sums have one row per such tile
    spec = W.small_spec(M=M, seed=900 + M, shapes=((1_300_000,), (777,), (1_200_003,), (5,)))
    h = _hyper(spec)
    inp = W.make_inputs(spec)
    gk = inp.grads(0)
    x, v, g = _dev_rows(inp, inp.x), _dev_rows(inp, inp.v), _dev_rows(inp, gk)
    r = torch.zeros(M, device="cuda")
    c = torch.zeros(M, device="cuda")
    xbar = upload_tensors(np.zeros(spec.d, np.float32), inp.offsets)
    plan = dppf.Plan(M, spec.numel)
    plan.round(x, v, g, h["lr"], h["mu"], h["wd"], h["pull"], h["push"], r_out=r, c_out=c, xbar_out=xbar)
    x_pre, _ = O.local_sgd_step(np.stack(inp.x), np.stack(inp.v), np.stack(gk), h["lr"], h["mu"], h["wd"])
    ref_x, ref_v, ref_r, ref_c, ref_avg = O.dppf_round(np.stack(inp.x), np.stack(inp.v), np.stack(gk), h["lr"],
                                                       h["mu"], h["wd"], h["pull"], h["push"])
    got = download_rows(x)
    assert_rel(r.cpu().numpy(), ref_r, 1e-4, "r")
    assert_rel(c.cpu().numpy(), ref_c, 1e-4, "c")
    assert_params_close(got, ref_x, inp.offsets, 1, "x")
    assert_params_close(download_rows(v), ref_v, inp.offsets, 1, "v")
    assert_params_close(download(xbar)[None], ref_avg[None], inp.offsets, 1, "xbar")
    assert_update_close(got, ref_x, x_pre, "round")
    # the same without asking for the average (the plan's own scratch vector is used)
    x2 = _dev_rows(inp, inp.x)
    r2 = torch.zeros(M, device="cuda")
    plan.local_sgd_step(x2, _dev_rows(inp, inp.v), g, h["lr"], h["mu"], h["wd"])
    plan.pull_push_round(x2, h["pull"], h["push"], r_out=r2)
    assert np.array_equal(download_rows(x2), got) and np.array_equal(r2.cpu().numpy(), r.cpu().numpy())
    plan.close()


@pytest.mark.parametrize("case", range(12))
def test_random_lists_with_mixed_alignment(case):
    # random tensor counts and sizes; every (worker, role, tensor) gets its own misalignment of
    # 0..3 elements, so the replicas of one tensor sit at different offsets modulo 16 bytes
    rng = np.random.default_rng(4000 + case)
    M = int(rng.integers(1, 10))
    T = int(rng.integers(1, 9))
    sizes = [int(rng.choice([0, 1, 2, 3, 5, 63, 64, 1000, 4095, 4096, 4097, 8191, 20_000, 70_001])) for _ in range(T)]
    spec = W.small_spec(M=M, seed=5000 + case, shapes=tuple((n,) for n in sizes), weight_decay=1e-3)
    h = _hyper(spec)
    inp = W.make_inputs(spec)
    gk = inp.grads(0)

    def scattered(arrays):
        rows = []
        for a in arrays:
            row = []
            for t in range(T):
                lo, hi = int(inp.offsets[t]), int(inp.offsets[t + 1])
                shift = int(rng.integers(0, 4))
                buf = torch.empty(hi - lo + shift, dtype=torch.float32, device="cuda")
                view = buf[shift:]
                if hi > lo:
                    view.copy_(torch.from_numpy(a[lo:hi]))
                row.append(view)
            rows.append(row)
        return rows

    x, v, g = scattered(inp.x), scattered(inp.v), scattered(gk)
    r = torch.zeros(M, device="cuda")
    c = torch.zeros(M, device="cuda")
    plan = dppf.Plan(M, spec.numel)
    plan.round(x, v, g, h["lr"], h["mu"], h["wd"], h["pull"], h["push"], r_out=r, c_out=c)
    ref_x, ref_v, ref_r, ref_c, _ = O.dppf_round(np.stack(inp.x), np.stack(inp.v), np.stack(gk), h["lr"], h["mu"],
                                                 h["wd"], h["pull"], h["push"])
    if M > 1 and spec.d > 0:
        assert_rel(r.cpu().numpy(), ref_r, 1e-4, "r")
        assert_rel(c.cpu().numpy(), ref_c, 1e-4, "c")
    assert_params_close(download_rows(x), ref_x, inp.offsets, 1, "x", c=ref_c)
    assert_params_close(download_rows(v), ref_v, inp.offsets, 1, "v")
    plan.close()


def test_thousands_of_tiny_tensors():
    # no full tile at all: 3000 tensors of 1..300 elements, every block walks partial tiles only
    rng = np.random.default_rng(77)
    sizes = [int(n) for n in rng.integers(1, 301, size=3000)]
    spec = W.small_spec(M=4, seed=78, shapes=tuple((n,) for n in sizes))
    h = _hyper(spec)
    inp = W.make_inputs(spec)
    gk = inp.grads(0)

    def rows(arrays):          # carve the tensors out of one buffer per worker (allocation count stays small)
        out = []
        for a in arrays:
            buf = torch.from_numpy(a).cuda()
            out.append([buf[int(inp.offsets[t]):int(inp.offsets[t + 1])] for t in range(spec.T)])
        return out

    x, v, g = rows(inp.x), rows(inp.v), rows(gk)
    r = torch.zeros(4, device="cuda")
    c = torch.zeros(4, device="cuda")
    plan = dppf.Plan(4, spec.numel)
    plan.round(x, v, g, h["lr"], h["mu"], h["wd"], h["pull"], h["push"], r_out=r, c_out=c)
    ref_x, ref_v, ref_r, ref_c, _ = O.dppf_round(np.stack(inp.x), np.stack(inp.v), np.stack(gk), h["lr"], h["mu"],
                                                 h["wd"], h["pull"], h["push"])
    assert_rel(r.cpu().numpy(), ref_r, 1e-4, "r")
    assert_rel(c.cpu().numpy(), ref_c, 1e-4, "c")
    assert_params_close(download_rows(x), ref_x, inp.offsets, 1, "x")
    assert_params_close(download_rows(v), ref_v, inp.offsets, 1, "v")
    plan.close()
