"""The synthetic parameter lists have the stated tensor counts and sizes, and the seeded
generator is reproducible and draws in the documented order."""
import numpy as np

from paper_2507_20424_amd import workloads as W


def test_list_sizes():
    for name, (T, d) in W.EXPECTED_SIZES.items():
        spec = W.SPECS[name]
        assert (spec.T, spec.d) == (T, d), name
    pyr = W.SPECS["pyramidnet_M8"]
    assert sum(1 for n in pyr.numel if n % 4) == 216
    assert sum(1 for n in pyr.numel if n < 10_000) == 229
    assert max(pyr.numel) == 665_856
    assert max(W.SPECS["resnet50_M4"].numel) == 2_359_296
    assert [W.SPECS[n].M for n in W.EXPECTED_SIZES] == [2, 4, 4, 4, 8]
    assert [W.SPECS[n].tau for n in W.EXPECTED_SIZES] == [1, 8, 16, 1, 4]


def test_generator_reproducible_and_scaled():
    spec = W.small_spec(M=3, seed=11)
    a = W.make_inputs(spec)
    b = W.make_inputs(spec)
    for m in range(spec.M):
        assert np.array_equal(a.x[m], b.x[m])
        assert a.x[m].dtype == np.float32 and a.x[m].shape == (spec.d,)
        assert not a.v[m].any()
    ga, gb = a.grads(0), b.grads(0)
    assert all(np.array_equal(p, q) for p, q in zip(ga, gb))
    assert not np.array_equal(ga[0], a.grads(1)[0])
    assert not np.array_equal(ga[0], ga[1])
    assert a.offsets[-1] == spec.d and len(a.tensor_views(a.x[0])) == spec.T


def test_value_scales():
    spec = W.SPECS["flat1m_M2"]
    inp = W.make_inputs(spec)
    x = np.stack(inp.x).astype(np.float64)
    assert abs(x.std() / 0.02 - 1) < 0.01
    assert abs((x[0] - x[1]).std() / (np.sqrt(2) * 1e-3) - 1) < 0.01
    g = inp.grads(0)
    assert abs(g[0].std() / 1e-2 - 1) < 0.01
    het = W.make_inputs(W.small_spec(M=8, seed=4, hetero_spread=True))
    assert np.all(het.sigma_m >= 1e-4) and np.all(het.sigma_m <= 1e-2)
    assert len(set(het.sigma_m.tolist())) == 8
