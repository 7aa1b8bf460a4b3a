"""csd_verify_static (the entry point that allocates nothing and takes no workspace) against csd_verify,
through the C ABI, on two calls in a row, the second on a smaller input (needs an MI355X).

Collected last on purpose: a failure here must not hide the parity tests."""
import ctypes

import numpy as np
import pytest
import torch

from gen import CONFIGS, Workload
from gen.device import to_device_logits
from paper_2604_13634_amd import binding as csd
from parity_util import decode_ocm

pytestmark = pytest.mark.gpu

RTOL = 1e-5


def _call(lib, static, z, draft, tau, lam, ocm, bf):
    """One raw C-ABI call; every argument is a plain pointer or a scalar."""
    P = ctypes.c_void_p
    B, K1, V = z.shape
    k = K1 - 1
    dt = csd.CSD_DTYPE_F32 if z.dtype == torch.float32 else csd.CSD_DTYPE_BF16
    head = (P(z.data_ptr()), dt, z.stride(1), P(draft.data_ptr()), B, k, V, ctypes.c_float(tau), lam, P(ocm.data_ptr()),
            ocm.numel(), csd.CSD_APPLY_UPDATES, P(bf.accept_len.data_ptr()), P(bf.next_token.data_ptr()),
            P(bf.argmax.data_ptr()), P(bf.row_max.data_ptr()), P(bf.row_sumexp.data_ptr()), P(bf.ratio.data_ptr()),
            P(bf.p_draft.data_ptr()), P(bf.pos_flags.data_ptr()), P(bf.rej_log.data_ptr()), P(bf.status.data_ptr()))
    st = P(torch.cuda.current_stream().cuda_stream or None)
    if static:
        return lib.csd_verify_static(*head, st)
    return lib.csd_verify(*head, P(bf.workspace.data_ptr()), bf.workspace.numel(), st)


def _same(a: csd.VerifyBuffers, b: csd.VerifyBuffers, where: str):
    g = lambda t: t.cpu().numpy()
    for name in ("accept_len", "next_token", "argmax", "pos_flags", "rej_log", "status"):
        np.testing.assert_array_equal(g(getattr(a, name)), g(getattr(b, name)), err_msg="%s %s" % (where, name))
    assert np.array_equal(g(a.row_max), g(b.row_max)), where + " row_max"
    for name in ("row_sumexp", "ratio", "p_draft"):
        x, y = g(getattr(a, name)).astype(np.float64), g(getattr(b, name)).astype(np.float64)
        assert np.all(np.isfinite(x)) and np.all(np.abs(x - y) <= RTOL * np.abs(y) + 1.1754944e-38), "%s %s" % (where, name)


def test_static_scratch_entry_point_matches_csd_verify():
    lib = csd.load_library()
    torch.cuda.set_device(0)
    # the first call is the larger one (bf16, 12 sequences, ragged vocabulary), the second a smaller fp32 batch;
    # then a few more of each so that the memory evolves and rescues happen
    big = Workload(CONFIGS[1], B=12, V=50021, n_pairs=16)
    small = Workload(CONFIGS[0], B=3, V=7001, n_pairs=8)
    ocm_s, ocm_w = csd.new_ocm(1 << 12), csd.new_ocm(1 << 12)
    bufs = {}
    rescued = 0
    for step, w in enumerate([big, small, big, small, big, big, small, small]):
        cfg = w.cfg
        z_np, d_np = w.step(step)
        z, d = to_device_logits(z_np), torch.from_numpy(d_np).cuda()
        dt = csd.CSD_DTYPE_F32 if cfg.dtype == "f32" else csd.CSD_DTYPE_BF16
        if cfg.name not in bufs:
            bufs[cfg.name] = (csd.VerifyBuffers.allocate(cfg.B, cfg.k, cfg.V, dt), csd.VerifyBuffers.allocate(cfg.B, cfg.k, cfg.V, dt))
        bs, bw = bufs[cfg.name]
        print("csd_verify_static step %d: %s B=%d k=%d V=%d" % (step, cfg.dtype, cfg.B, cfg.k, cfg.V), flush=True)
        assert _call(lib, True, z, d, cfg.tau, 1, ocm_s, bs) == csd.CSD_OK
        assert _call(lib, False, z, d, cfg.tau, 1, ocm_w, bw) == csd.CSD_OK
        torch.cuda.synchronize()
        _same(bs, bw, "step %d" % step)
        assert decode_ocm(ocm_s) == decode_ocm(ocm_w), "memory differs after step %d" % step
        rescued = int(bs.status[csd.CSD_STATUS_RESCUED])
    assert rescued > 0 and len(decode_ocm(ocm_s)) > 0


def test_static_scratch_rejects_shapes_beyond_its_size():
    lib = csd.load_library()
    P = ctypes.c_void_p
    B, k, V = 4096, 7, 1 << 20                     # needs far more scratch than the array holds
    assert csd.csd_verify_workspace_bytes(B, k, V, csd.CSD_DTYPE_F32) > csd.CSD_STATIC_SCRATCH_BYTES
    good = 0x10000                                 # never dereferenced: the size check comes first
    rc = lib.csd_verify_static(P(good), 0, V, P(good), B, k, V, ctypes.c_float(0.3), 2, None, 0, 0, P(good), P(good), P(good),
                               None, None, None, None, None, None, None, None)
    assert rc == csd.CSD_ENOSPACE
    assert "workspace too small" in csd.csd_strerror(rc)
