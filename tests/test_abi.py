"""Host-side checks that need no GPU: the library loads, exports every symbol the header
declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2507_20424_amd import dppf
    if not os.path.exists(dppf.lib_path()):
        from paper_2507_20424_amd.build import build_library
        build_library(verbose=False)
    return dppf.load()


def header_symbols():
    names = set()
    for header in ("dppf.h", "dppf_util.h"):
        with open(os.path.join(ROOT, "include", header)) as f:
            text = f.read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(dppf_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(lib):
    names = header_symbols()
    assert len(names) >= 14 and "dppf_round" in names and "dppf_plan_create" in names
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in include/dppf.h but not exported"


def test_binding_covers_the_header(lib):
    from paper_2507_20424_amd import dppf
    for name in header_symbols():
        assert getattr(lib, name).argtypes is not None, f"binding has no signature for {name}"
    for method in ("replica_mean", "dist_norms", "pull_push_round", "local_sgd_step", "round"):
        assert hasattr(dppf.Plan, method)


def test_error_strings(lib):
    assert lib.dppf_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -99):
        assert lib.dppf_strerror(code)
    assert lib.dppf_last_hip_error() == 0


def test_plan_create_rejects_bad_arguments(lib):
    h = ctypes.c_void_p()
    one = (ctypes.c_int64 * 1)(8)
    neg = (ctypes.c_int64 * 1)(-1)
    assert lib.dppf_plan_create(None, 2, 1, one) == -1
    assert lib.dppf_plan_create(ctypes.byref(h), 0, 1, one) == -1
    assert lib.dppf_plan_create(ctypes.byref(h), 2, -1, one) == -1
    assert lib.dppf_plan_create(ctypes.byref(h), 2, 1, None) == -1
    assert lib.dppf_plan_create(ctypes.byref(h), 2, 1, neg) == -1
    assert lib.dppf_plan_create(ctypes.byref(h), 1025, 1, one) == -4
    assert not h.value
    assert lib.dppf_plan_destroy(None) == 0


def test_null_plan_is_rejected(lib):
    assert lib.dppf_pull_push_round(None, None, 0.1, 0.01, None, None, None, None) == -1
    assert lib.dppf_round(None, None, None, None, 0.1, 0.9, 0.0, 0.1, 0.01, None, None, None, None) == -1
    assert lib.dppf_local_sgd_step(None, None, None, None, 0.1, 0.9, 0.0, None) == -1
    assert lib.dppf_replica_mean(None, None, None, None) == -1
    assert lib.dppf_dist_norms(None, None, None, None, None) == -1


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    from paper_2507_20424_amd import dppf
    monkeypatch.setattr(dppf, "_lib", None)
    monkeypatch.setattr(dppf, "_LIB_PATH", str(tmp_path / "libdppf.so"))
    with pytest.raises(dppf.DppfError):
        dppf.load()


def test_push_schedule_is_a_host_function(lib):
    import math
    assert lib.dppf_push_schedule(0, 0.5, 3, 10) == 0.5
    assert abs(lib.dppf_push_schedule(1, 0.5, 5, 10) - 0.25) < 1e-7
    assert abs(lib.dppf_push_schedule(2, 0.5, 10, 10) - 0.5) < 1e-7
    assert abs(lib.dppf_push_schedule(2, 0.5, 25, 100) - 0.25 * (1 - math.sqrt(0.5))) < 1e-7
    assert lib.dppf_round_statistics(None, 4, 0.1, 0.1, None, None, None) == -1
    assert lib.dppf_plan_average_norm(None, None, None) == -1
    assert lib.dppf_pull_then_push(None, None, None, 0.1, 0.1, 0, None, None) == -1
    assert lib.dppf_pull_push_round_exact(None, None, 0.1, 0.1, None, None, None) == -1
    assert lib.dppf_local_adamw_step(None, None, None, None, None, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1, None) == -1
    assert lib.dppf_round_adamw(None, None, None, None, None, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1, 0.1, 0.1, None, None,
                                None) == -1


def test_plain_c_client_builds_against_the_header():
    from paper_2507_20424_amd import build as B
    path = B.build_cli(verbose=False)
    assert os.access(path, os.X_OK)


def test_tile_layout_covers_every_element_exactly_once(lib):
    from paper_2507_20424_amd import dppf, workloads as W
    lists = [[], [0], [1], [4095], [4096], [4097], [3, 0, 8192, 1, 12289, 0, 5], list(W.SPECS["pyramidnet_M8"].numel),
             list(W.SPECS["vitb16_M4"].numel)]
    assert [dppf.sweep_tile_elems(M) for M in (1, 4, 5, 8, 16, 17, 39, 40, 1024)] == \
        [4096, 4096, 2048, 2048, 2048, 1024, 1024, 4096, 4096]
    assert lib.dppf_sweep_tile_elems(0) == -1 and lib.dppf_sweep_tile_elems(1025) == -1
    for tile in (4096, 2048, 1024):
        for numel in lists:
            d, nfull, tiles = dppf.layout_tiles(numel, tile)
            assert d == sum(numel)
            assert nfull == sum(n // tile for n in numel)
            assert len(tiles) == sum(-(-n // tile) for n in numel)
            assert all(c == tile for _, _, c in tiles[:nfull])
            assert all(0 < c < tile for _, _, c in tiles[nfull:])
            covered = {}
            for t, off, c in tiles:
                assert 0 <= t < len(numel) and off % tile == 0 and off + c <= numel[t]
                covered.setdefault(t, []).append((off, c))
            for t, n in enumerate(numel):
                pieces = sorted(covered.get(t, []))
                assert sum(c for _, c in pieces) == n
                assert [o for o, _ in pieces] == list(range(0, n, tile))
            # full tiles keep list order, partial tiles too
            assert [t for t, _, _ in tiles[:nfull]] == sorted(t for t, _, _ in tiles[:nfull])
            assert [t for t, _, _ in tiles[nfull:]] == sorted(t for t, _, _ in tiles[nfull:])
    import ctypes
    bad = (ctypes.c_int64 * 2)(5, -1)
    out = ctypes.c_int64()
    assert lib.dppf_layout_tiles(4096, 2, bad, ctypes.byref(out), ctypes.byref(out), ctypes.byref(out), 0, None, None,
                                 None) == -1
    assert lib.dppf_layout_tiles(4096, 1, None, ctypes.byref(out), ctypes.byref(out), ctypes.byref(out), 0, None, None,
                                 None) == -1
    assert lib.dppf_layout_tiles(0, 2, bad, ctypes.byref(out), ctypes.byref(out), ctypes.byref(out), 0, None, None,
                                 None) == -1
