"""The C part of the oracle under AddressSanitizer + UndefinedBehaviorSanitizer (host code only): the row pins'
inputs - ragged lengths, a padded row pitch, masked entries, both storage types - go through a sanitized build,
which must report nothing and give bit for bit what the ordinary build gives, and what numpy/scipy give."""
import os
import shutil
import subprocess

import numpy as np
import pytest
from scipy.special import logsumexp

from gen import f32_to_bf16_bits
from oracle import csd_oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "csd_oracle_rows.c")


@pytest.fixture(scope="module")
def sanitized_driver(tmp_path_factory):
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    exe = str(tmp_path_factory.mktemp("san") / "oracle_rows_san")
    cmd = ["gcc", "-O1", "-g", "-std=c99", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-o", exe, os.path.join(HERE, "oracle_rows_driver.c"), SRC, "-lm"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0 and "asan" in (res.stderr + res.stdout).lower():
        pytest.skip("the sanitizer runtime is not installed: " + res.stderr.strip().splitlines()[-1])
    assert res.returncode == 0, res.stderr
    return exe


def _run(exe, tmp_path, z, V, stride):
    dtype = 0 if z.dtype == np.float32 else 1
    rows = z.size // stride
    fin, fout = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(fin, "wb") as f:
        np.array([dtype, rows, V, stride], np.int64).tofile(f)
        z.tofile(f)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)                    # the sanitizer runtime must come first in the driver's own process
    res = subprocess.run([exe, fin, fout], capture_output=True, text=True, env=env)
    if "does not come first in initial library list" in res.stderr:
        pytest.skip("another preloaded library keeps the sanitizer runtime from starting in this environment")
    assert res.returncode == 0 and "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr
    raw = np.fromfile(fout, np.uint8)
    m = raw[:rows * 8].view(np.float64)
    t = raw[rows * 8:rows * 16].view(np.int64)
    S = raw[rows * 16:].view(np.float64)
    return m, t, S


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V,stride", [(1, 1), (2, 2), (7, 7), (8, 8), (1000, 1000), (1000, 1016), (4097, 4104)])
def test_sanitized_build_agrees_and_reports_nothing(sanitized_driver, tmp_path, dtype, V, stride):
    rng = np.random.default_rng(V * 3 + stride)
    rows = 9
    z = (rng.standard_normal((rows, stride)) * 4).astype(np.float32)
    z[:, V:] = 1e30                                             # the padding of a row pitch must never be read as logits
    if V > 4:
        z[1, : V // 2] = -np.inf                                # a masked half
        z[2, :V] = -np.inf
        z[2, V - 1] = 0.5                                       # one finite entry, the last
        z[3, 1] = z[3, 3] = 50.0                                # a tie: the lower id
    if dtype == "bf16":
        fin = np.isfinite(z)
        bits = f32_to_bf16_bits(np.where(fin, z, 0).astype(np.float32)).reshape(z.shape)
        bits[~fin] = 0xFF80
        z = bits
    m, t, S = _run(sanitized_driver, tmp_path, z, V, stride)
    view = np.ascontiguousarray(z[:, :V])
    m0, t0, S0 = O.row_stats(view)
    assert np.array_equal(m, m0) and np.array_equal(t, t0) and np.array_equal(S, S0)
    z64 = view.astype(np.float64) if dtype == "f32" else (view.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    np.testing.assert_array_equal(m, z64.max(-1))
    np.testing.assert_array_equal(t, z64.argmax(-1))
    np.testing.assert_allclose(np.log(S) + m, logsumexp(z64, axis=-1), rtol=1e-13)
