"""Host-side checks of the C ABI that need no GPU: the library loads, exports every entry point the
header declares, and rejects bad arguments before enqueuing anything."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2604_13634_amd", "libcsd.so")

pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="libcsd.so not built (run __graft_entry__.build())")


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "csd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(csd_[a-z_]+)\s*\(", text)))


def test_every_declared_entry_point_is_exported():
    lib = ctypes.CDLL(LIB)
    names = _declared_functions()
    assert {"csd_verify", "csd_ocm_update", "csd_ocm_reset", "csd_verify_workspace_bytes"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_binding_exposes_the_same_names():
    from paper_2604_13634_amd import binding
    for n in _declared_functions():
        assert callable(getattr(binding, n)), n


def test_header_constants_match_binding():
    from paper_2604_13634_amd import binding
    text = open(os.path.join(ROOT, "include", "csd.h")).read()
    for name, val in re.findall(r"#define\s+(CSD_[A-Z_0-9]+)\s+\(?(-?\d+)u?\)?\s*(?:/\*.*)?\n", text):
        if hasattr(binding, name):
            assert getattr(binding, name) == int(val), name
    assert binding.CSD_OCM_EMPTY == 0xFFFFFFFFFF and binding.CSD_OCM_COUNT_MAX == 0xFFFFFF


def test_workspace_query_is_pure_host_arithmetic():
    from paper_2604_13634_amd import binding as b
    assert b.csd_verify_workspace_bytes(1, 4, 32000, b.CSD_DTYPE_F32) > 0
    big = b.csd_verify_workspace_bytes(256, 4, 256000, b.CSD_DTYPE_BF16)
    assert 0 < big < (1 << 22)
    assert b.csd_verify_workspace_bytes(0, 4, 100, 0) > 0
    for bad in [(-1, 4, 100, 0), (1, -1, 100, 0), (1, 64, 100, 0), (1, 4, 0, 0), (1, 4, (1 << 20) + 1, 0), (1, 4, 100, 2)]:
        assert b.csd_verify_workspace_bytes(*bad) == 0


def test_launch_plan_of_the_streaming_pass():
    """How many workgroups share a row (host arithmetic, visible through csd_row_partials_per_row = 4 waves per
    workgroup): two 32 KiB tiles per workgroup in general; every tile, and the row's remainder, a workgroup of its
    own when the whole launch is at most 1024 workgroups; three tiles where two would leave it just above that."""
    from paper_2604_13634_amd import binding as csd
    per_row = lambda rows, V, dt: csd.csd_row_partials_per_row(rows, V, dt) // 4
    F32, BF16 = csd.CSD_DTYPE_F32, csd.CSD_DTYPE_BF16
    assert per_row(256 * 5, 256000, BF16) == 8       # 15 tiles and a remainder: 7 x 2 tiles, 1 tile + remainder
    assert per_row(64 * 9, 152064, F32) == 9         # 18 tiles and a remainder
    assert per_row(32 * 8, 151936, BF16) == 3        # 9 tiles: 256 x 5 workgroups would be 1280 > 1024, 256 x 3 fit
    assert per_row(8 * 6, 128256, BF16) == 8         # small launch: 7 tiles + the remainder, one round of loads each
    assert per_row(1 * 5, 32000, F32) == 4           # 3 tiles + the remainder
    assert per_row(5, 8 * 2048 * 3, BF16) == 3       # exactly three tiles, no remainder
    assert per_row(7, 100, F32) == 1                 # less than a tile
    for B, k, V, dt in [(256, 4, 256000, BF16), (64, 8, 152064, F32), (1, 4, 32000, F32), (3, 0, 7, BF16)]:
        rows = B * (k + 1)            # control head, one 32-byte record per streaming workgroup, the log, a 16-byte word per sequence
        need = 256 + rows * per_row(rows, V, dt) * 32 + B * k * 8 + B * 16
        assert need <= csd.csd_verify_workspace_bytes(B, k, V, dt) <= need + 4 * 256


def test_grid_order_of_the_step_by_shape():
    """Launches of more than 1024 streaming workgroups (more than are resident at once) stream the bonus rows last;
    smaller ones, and steps without a draft position, keep the plain order (a library hook outside csd.h tells)."""
    from paper_2604_13634_amd import binding as csd
    lib = csd.load_library()
    lib.csd_test_step_order_of.restype = ctypes.c_int
    lib.csd_test_step_order_of.argtypes = [ctypes.c_int] * 4
    F32, BF16 = csd.CSD_DTYPE_F32, csd.CSD_DTYPE_BF16
    assert lib.csd_test_step_order_of(256, 4, 256000, BF16) == 1      # 10240 streaming workgroups
    assert lib.csd_test_step_order_of(64, 8, 152064, F32) == 1        # 5184
    assert lib.csd_test_step_order_of(32, 7, 151936, BF16) == 0       # 768
    assert lib.csd_test_step_order_of(8, 5, 128256, BF16) == 0
    assert lib.csd_test_step_order_of(1, 4, 32000, F32) == 0
    assert lib.csd_test_step_order_of(4096, 0, 256000, BF16) == 0     # no draft position: nothing to run early
    assert lib.csd_test_step_order_of(1, 64, 100, F32) == -1


def test_argument_errors_are_synchronous_and_enqueue_nothing():
    """Every call below fails validation on the host, so no pointer is ever dereferenced."""
    from paper_2604_13634_amd import binding as b
    lib = b.load_library()
    P = ctypes.c_void_p
    good = 0x10000                       # a fake, aligned, never-used address
    ws = b.csd_verify_workspace_bytes(2, 3, 1000, 0)

    def verify(logits=good, dtype=0, stride=1000, draft=good, B=2, k=3, V=1000, tau=0.3, lam=2, ocm=None, cap=0,
               flags=0, acc=good, nxt=good, am=good, work=good, wsz=ws):
        return lib.csd_verify(P(logits), dtype, stride, P(draft), B, k, V, tau, lam, P(ocm), cap, flags, P(acc), P(nxt),
                              P(am), None, None, None, None, None, None, None, P(work), wsz, None)

    assert verify(B=-1) == b.CSD_EINVAL
    assert verify(k=64) == b.CSD_EINVAL
    assert verify(V=0) == b.CSD_EINVAL
    assert verify(V=(1 << 20) + 1, stride=1 << 21) == b.CSD_EINVAL
    assert verify(dtype=3) == b.CSD_EINVAL
    assert verify(tau=float("nan")) == b.CSD_EINVAL
    assert verify(flags=2) == b.CSD_EINVAL
    assert verify(logits=None) == b.CSD_EINVAL
    assert verify(draft=None) == b.CSD_EINVAL
    assert verify(acc=None) == b.CSD_EINVAL
    assert verify(work=None) == b.CSD_EINVAL
    assert verify(stride=999) == b.CSD_EINVAL
    assert verify(ocm=good, cap=1000) == b.CSD_EINVAL          # capacity must be a power of two
    assert verify(ocm=good, cap=0) == b.CSD_EINVAL
    assert verify(logits=good + 4) == b.CSD_EALIGN
    assert verify(stride=1001) == b.CSD_EALIGN                 # 4004-byte pitch
    assert verify(dtype=1, stride=1004) == b.CSD_EALIGN        # bf16: 2008-byte pitch
    assert verify(am=good + 2) == b.CSD_EALIGN
    assert verify(ocm=good + 4, cap=1024) == b.CSD_EALIGN
    assert verify(wsz=ws - 1) == b.CSD_ENOSPACE
    assert verify(B=0, logits=None, draft=None, acc=None, nxt=None, am=None, work=None, wsz=0) == b.CSD_OK

    assert lib.csd_ocm_reset(None, 1024, None) == b.CSD_EINVAL
    assert lib.csd_ocm_reset(P(good), 1000, None) == b.CSD_EINVAL
    assert lib.csd_ocm_update(P(good), 1024, None, None, 5, None, None, None) == b.CSD_EINVAL
    assert lib.csd_ocm_update(P(good), 1024, None, None, 0, None, None, None) == b.CSD_OK
    assert lib.csd_ocm_update(P(good), 1024, P(good + 1), None, 5, None, None, None) == b.CSD_EALIGN
    assert lib.csd_ocm_update(P(good), 1024, P(good), None, 5, P(good + 4), None, None) == b.CSD_EALIGN
    assert lib.csd_ocm_lookup(P(good), 1024, P(good), None, 5, None) == b.CSD_EINVAL
    assert lib.csd_ocm_lookup(P(good), 3, P(good), P(good), 5, None) == b.CSD_EINVAL
    assert lib.csd_ocm_merge(P(good), 1024, P(good + 0x10000), 1000, None, None) == b.CSD_EINVAL
    assert lib.csd_ocm_merge(P(good), 1024, P(good + 64), 1024, None, None) == b.CSD_EINVAL     # overlapping tables
    assert lib.csd_ocm_merge(P(good), 1024, None, 1024, None, None) == b.CSD_EINVAL
    assert lib.csd_ocm_export(P(good), 1024, None, None, 5, P(good), None) == b.CSD_EINVAL
    assert lib.csd_ocm_export(P(good), 1024, P(good), P(good), 5, None, None) == b.CSD_EINVAL
    assert lib.csd_ocm_export(P(good), 1024, P(good), P(good + 2), 5, P(good), None) == b.CSD_EALIGN
    assert lib.csd_verify_shards(0, None, None, None, None, None, 2, 3, 1000, 0.3, 2, None, 0, 0, None, None, None, None, None,
                                 None, None, None, None, None, None, 0, None) == b.CSD_EINVAL
    assert lib.csd_verify_shards(9, P(good), P(good), P(good), P(good), P(good), 2, 3, 1000, 0.3, 2, None, 0, 0, P(good),
                                 P(good), P(good), None, None, None, None, None, None, None, P(good), 4096, None) == b.CSD_EINVAL
    assert b.csd_verify_shards_workspace_bytes(256, 4) >= 256 + 256 * 4 * 8 and b.csd_verify_shards_workspace_bytes(-1, 4) == 0
    assert lib.csd_shard_draft_logits(None, 0, 100, 2, 3, 100, 0, P(good), P(good), None) == b.CSD_EINVAL
    assert lib.csd_shard_draft_logits(P(good), 0, 99, 2, 3, 100, 0, P(good), P(good), None) == b.CSD_EINVAL
    assert lib.csd_verify_sampled_workspace_bytes(2, 3, 1000, 0) > 0
    assert lib.csd_verify_sampled(P(good), P(good), 0, 1000, 1000, P(good), 2, 3, 1000, 0.0, P(good), P(good), 0.3, 2, None, 0,
                                  0, P(good), P(good), None, None, None, None, None, None, None, None, None, P(good), 1 << 20,
                                  None) == b.CSD_EINVAL                                   # temperature must be positive
    assert lib.csd_verify_sampled(P(good), P(good), 0, 1000, 999, P(good), 2, 3, 1000, 1.0, P(good), P(good), 0.3, 2, None, 0,
                                  0, P(good), P(good), None, None, None, None, None, None, None, None, None, P(good), 1 << 20,
                                  None) == b.CSD_EINVAL                                   # draft stride below V
    assert lib.csd_verify_sampled(P(good), P(good), 0, 1000, 1000, P(good), 2, 3, 1000, 1.0, P(good), P(good), 0.3, 2, None, 0,
                                  0, P(good), P(good), None, None, None, None, None, None, None, None, None, P(good), 16,
                                  None) == b.CSD_ENOSPACE
    assert b.csd_strerror(b.CSD_ENOSPACE) == "workspace too small"
