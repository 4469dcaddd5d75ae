"""The C ABI used from plain C (no Python, no PyTorch in the process): `csrc/dppf_cli` reads the
workers' tensors from a file, runs one fused round through include/dppf.h with device memory
from the HIP runtime API alone, and writes the results, which are compared with the oracle."""
import os
import struct
import subprocess

import numpy as np
import pytest

from parity import O, assert_params_close, assert_rel, assert_update_close, f32

pytestmark = pytest.mark.gpu

from paper_2507_20424_amd import build as B, workloads as W  # noqa: E402


@pytest.mark.parametrize("M", [2, 4, 9, 18])
def test_fused_round_from_plain_c(M, tmp_path):
    if not os.path.exists(B.CLI):
        B.build_all(verbose=False)
    spec = W.small_spec(M=M, seed=800 + M, shapes=((3,), (0,), (5000,), (4096,), (12_345,), (1,)))
    inp = W.make_inputs(spec)
    g = inp.grads(0)
    hyper = [f32(spec.lr), f32(spec.momentum), f32(1e-3), f32(spec.pull), f32(spec.push)]
    src, dst = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(src, "wb") as f:
        f.write(struct.pack("<ii", M, spec.T))
        f.write(np.asarray(spec.numel, dtype="<i8").tobytes())
        f.write(np.asarray(hyper, dtype="<f4").tobytes())
        for arrays in (inp.x, inp.v, g):
            f.write(np.stack(arrays).astype("<f4").tobytes())
    res = subprocess.run([B.CLI, str(src), str(dst)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                         timeout=120)
    assert res.returncode == 0, res.stdout
    out = np.fromfile(dst, dtype="<f4")
    n = M * spec.d
    assert out.size == 2 * n + 2 * M
    got_x, got_v = out[:n].reshape(M, spec.d), out[n:2 * n].reshape(M, spec.d)
    got_r, got_c = out[2 * n:2 * n + M], out[2 * n + M:]
    x_pre, _ = O.local_sgd_step(np.stack(inp.x), np.stack(inp.v), np.stack(g), *hyper[:3])
    ref_x, ref_v, ref_r, ref_c, _ = O.dppf_round(np.stack(inp.x), np.stack(inp.v), np.stack(g), *hyper)
    assert_rel(got_r, ref_r, 1e-4, "r")
    assert_rel(got_c, ref_c, 1e-4, "c")
    assert_params_close(got_x, ref_x, inp.offsets, 1, "x", c=ref_c)
    assert_params_close(got_v, ref_v, inp.offsets, 1, "v")
    assert_update_close(got_x, ref_x, x_pre, "round")


def test_cli_rejects_bad_input(tmp_path):
    if not os.path.exists(B.CLI):
        B.build_all(verbose=False)
    bad = tmp_path / "bad.bin"
    bad.write_bytes(struct.pack("<ii", 0, 1))
    res = subprocess.run([B.CLI, str(bad), str(tmp_path / "o.bin")], stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    assert res.returncode == 2
