"""ctypes binding of libcsd.so: argument marshalling only.

Every function here has the name of the C entry point it calls (see include/csd.h) and does no
arithmetic of the method: tensors are torch device memory, the stream is torch's current stream,
and all work runs in the HIP kernels.  If the library has not been built the import of this
module's functions fails loudly - there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libcsd.so")

CSD_OK, CSD_EINVAL, CSD_EALIGN, CSD_ENOSPACE, CSD_EHIP = 0, -1, -2, -3, -4
CSD_DTYPE_F32, CSD_DTYPE_BF16 = 0, 1
CSD_APPLY_UPDATES = 1
CSD_MAX_K = 63
CSD_MAX_V = 1 << 20
CSD_MAX_SHARDS = 8
CSD_STATIC_SCRATCH_BYTES = 4 << 20
CSD_OCM_KEY_BITS = 40
CSD_OCM_KEY_MASK = (1 << 40) - 1
CSD_OCM_EMPTY = (1 << 40) - 1
CSD_OCM_COUNT_MAX = (1 << 24) - 1
CSD_STATUS_DROPPED, CSD_STATUS_BAD_DRAFT, CSD_STATUS_RESCUED, CSD_STATUS_COUNTED, CSD_STATUS_ACCEPTED = 0, 1, 2, 3, 4
CSD_STATUS_STALLED = 5
CSD_STATUS_WORDS = 8
CSD_POS_MATCH, CSD_POS_FREQ, CSD_POS_SAFE, CSD_POS_ACCEPTED, CSD_POS_COUNTED = 1, 2, 4, 8, 16


class CsdError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (where, csd_strerror(code), code))


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libcsd.so (built by paper_2604_13634_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libcsd.so is not built: run `python -m paper_2604_13634_amd.build` "
                           "(there is no CPU or PyTorch fallback for the verification path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, u32, u64, f32, sz = (ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_uint32,
                                       ctypes.c_uint64, ctypes.c_float, ctypes.c_size_t)
    lib.csd_verify_workspace_bytes.restype = sz
    lib.csd_verify_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.csd_verify.restype = i32
    lib.csd_verify.argtypes = [vp, i32, i64, vp, i32, i32, i32, f32, u32, vp, u64, u32,
                               vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.csd_verify_static.restype = i32
    lib.csd_verify_static.argtypes = [vp, i32, i64, vp, i32, i32, i32, f32, u32, vp, u64, u32,
                                      vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.csd_verify_sampled_workspace_bytes.restype = sz
    lib.csd_verify_sampled_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.csd_verify_sampled.restype = i32
    lib.csd_verify_sampled.argtypes = [vp, vp, i32, i64, i64, vp, i32, i32, i32, f32, vp, vp, f32, u32, vp, u64, u32,
                                       vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.csd_verify_shards_workspace_bytes.restype = sz
    lib.csd_verify_shards_workspace_bytes.argtypes = [i32, i32]
    lib.csd_verify_shards.restype = i32
    lib.csd_verify_shards.argtypes = [i32, vp, vp, vp, vp, vp, i32, i32, i32, f32, u32, vp, u64, u32,
                                      vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.csd_shard_draft_logits.restype = i32
    lib.csd_shard_draft_logits.argtypes = [vp, i32, i64, i32, i32, i32, i32, vp, vp, vp]
    lib.csd_ocm_update.restype = i32
    lib.csd_ocm_update.argtypes = [vp, u64, vp, vp, u64, vp, vp, vp]
    lib.csd_ocm_reset.restype = i32
    lib.csd_ocm_reset.argtypes = [vp, u64, vp]
    lib.csd_ocm_lookup.restype = i32
    lib.csd_ocm_lookup.argtypes = [vp, u64, vp, vp, u64, vp]
    lib.csd_ocm_merge.restype = i32
    lib.csd_ocm_merge.argtypes = [vp, u64, vp, u64, vp, vp]
    lib.csd_ocm_export.restype = i32
    lib.csd_ocm_export.argtypes = [vp, u64, vp, vp, u64, vp, vp]
    lib.csd_row_partials_per_row.restype = i32
    lib.csd_row_partials_per_row.argtypes = [i32, i32, i32]
    lib.csd_row_partials.restype = i32
    lib.csd_row_partials.argtypes = [vp, i32, i64, i32, i32, vp, sz, vp]
    lib.csd_strerror.restype = ctypes.c_char_p
    lib.csd_strerror.argtypes = [i32]
    _lib = lib
    return lib


def csd_strerror(code: int) -> str:
    return load_library().csd_strerror(int(code)).decode()


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return CSD_DTYPE_F32
    if t.dtype == torch.bfloat16:
        return CSD_DTYPE_BF16
    raise TypeError("logits must be float32 or bfloat16")


def csd_verify_workspace_bytes(B: int, k: int, V: int, dtype: int) -> int:
    return int(load_library().csd_verify_workspace_bytes(B, k, V, dtype))


@dataclass
class VerifyBuffers:
    """Outputs and scratch of csd_verify for one shape, allocated once and reused across calls."""
    B: int
    k: int
    V: int
    dtype: int
    accept_len: torch.Tensor
    next_token: torch.Tensor
    argmax: torch.Tensor
    row_max: torch.Tensor
    row_sumexp: torch.Tensor
    ratio: torch.Tensor
    p_draft: torch.Tensor
    pos_flags: torch.Tensor
    rej_log: torch.Tensor
    status: torch.Tensor
    workspace: torch.Tensor

    @staticmethod
    def allocate(B: int, k: int, V: int, dtype: int, device="cuda") -> "VerifyBuffers":
        nbytes = csd_verify_workspace_bytes(B, k, V, dtype)
        if nbytes == 0:
            raise CsdError(CSD_EINVAL, "csd_verify_workspace_bytes")
        e = lambda shape, dt: torch.empty(shape, dtype=dt, device=device)
        return VerifyBuffers(
            B, k, V, dtype,
            accept_len=e((B,), torch.int32), next_token=e((B,), torch.int32), argmax=e((B, k + 1), torch.int32),
            row_max=e((B, k + 1), torch.float32), row_sumexp=e((B, k + 1), torch.float32),
            ratio=e((B, k), torch.float32), p_draft=e((B, k), torch.float32), pos_flags=e((B, k), torch.uint8),
            rej_log=e((B, k), torch.int64), status=torch.zeros((CSD_STATUS_WORDS,), dtype=torch.int32, device=device),
            workspace=e((nbytes,), torch.uint8))


def new_ocm(capacity: int, device="cuda") -> torch.Tensor:
    """An empty Online Correction Memory: int64 tensor of `capacity` slots, reset on the current stream."""
    ocm = torch.empty((capacity,), dtype=torch.int64, device=device)
    csd_ocm_reset(ocm)
    return ocm


def _current_stream_handle() -> int:
    return torch.cuda.current_stream().cuda_stream


def _marshal_verify(logits, draft, tau, lam, ocm, flags, buffers, stream, diagnostics, static_scratch):
    """Checks and argument list of one csd_verify / csd_verify_static call: (C function, its arguments, buffers, name)."""
    if logits.dim() != 3:
        raise ValueError("logits must be [B][k+1][V]")
    B, K1, V = logits.shape
    k = K1 - 1
    s0, s1, s2 = logits.stride()
    if s2 != 1 or (B > 1 and s0 != K1 * s1):
        raise ValueError("logits rows must be equally spaced with unit element stride")
    row_stride = s1 if K1 > 1 or B > 1 else max(V, s1)
    if draft is not None:
        if draft.dtype != torch.int32 or tuple(draft.shape) != (B, k) or not draft.is_contiguous():
            raise ValueError("draft must be a contiguous int32 [B][k] tensor")
    dt = _dtype_code(logits)
    if buffers is None:
        buffers = VerifyBuffers.allocate(B, k, V, dt, logits.device)
    elif (buffers.B, buffers.k, buffers.V, buffers.dtype) != (B, k, V, dt):
        raise ValueError("buffers were allocated for another shape")
    if ocm is not None and (ocm.dtype != torch.int64 or not ocm.is_contiguous()):
        raise ValueError("ocm must be a contiguous int64 tensor")
    bf = buffers
    # addresses of the outputs are fixed for the life of the buffers: marshal them once
    cache = bf.__dict__.get("_verify_args")
    if cache is None:
        full = (bf.accept_len.data_ptr(), bf.next_token.data_ptr(), bf.argmax.data_ptr(), bf.row_max.data_ptr(),
                bf.row_sumexp.data_ptr(), bf.ratio.data_ptr(), bf.p_draft.data_ptr(), bf.pos_flags.data_ptr(),
                bf.rej_log.data_ptr(), bf.status.data_ptr(), bf.workspace.data_ptr(), bf.workspace.numel())
        lean = full[:3] + (None,) * 6 + full[9:]
        cache = bf.__dict__["_verify_args"] = (full, lean)
    outs = cache[0] if diagnostics else cache[1]
    if stream is None:
        st = _current_stream_handle()
    else:
        st = stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)
    head = (logits.data_ptr(), dt, row_stride, None if draft is None else draft.data_ptr(), B, k, V, tau, lam & 0xFFFFFFFF,
            None if ocm is None else ocm.data_ptr(), 0 if ocm is None else ocm.numel(), flags)
    if static_scratch:
        return load_library().csd_verify_static, head + outs[:10] + (st or None,), bf, "csd_verify_static"
    return load_library().csd_verify, head + outs + (st or None,), bf, "csd_verify"


def csd_verify(logits: torch.Tensor, draft: Optional[torch.Tensor], tau: float, lam: int,
               ocm: Optional[torch.Tensor] = None, flags: int = CSD_APPLY_UPDATES,
               buffers: Optional[VerifyBuffers] = None, stream=None, diagnostics: bool = True,
               static_scratch: bool = False) -> VerifyBuffers:
    """Enqueue one verification step.  logits: [B][k+1][V] (float32 or bfloat16), draft: [B][k] int32.

    Returns the VerifyBuffers holding the outputs (valid once the stream has run the call).
    With diagnostics=False the optional outputs (row_max ... rej_log) are not written."""
    fn, args, bf, name = _marshal_verify(logits, draft, tau, lam, ocm, flags, buffers, stream, diagnostics, static_scratch)
    rc = fn(*args)
    if rc != CSD_OK:
        raise CsdError(rc, name)
    return bf


class PreparedVerify:
    """One csd_verify call with its arguments checked and marshalled once, for loops that verify into the same
    tensors step after step (a serving loop refills `logits` and `draft` in place): `launch()` is the C call and
    nothing else.  The tensors, the buffers and the stream handed to `prepare_verify` must stay alive and in
    place; `stream=None` fixes the stream that was current when the call was prepared."""
    __slots__ = ("_fn", "_args", "_name", "buffers", "_keep")

    def __init__(self, fn, args, name, buffers, keep):
        self._fn, self._args, self._name, self.buffers, self._keep = fn, args, name, buffers, keep

    def launch(self) -> VerifyBuffers:
        rc = self._fn(*self._args)
        if rc != CSD_OK:
            raise CsdError(rc, self._name)
        return self.buffers


def prepare_verify(logits: torch.Tensor, draft: Optional[torch.Tensor], tau: float, lam: int,
                   ocm: Optional[torch.Tensor] = None, flags: int = CSD_APPLY_UPDATES,
                   buffers: Optional[VerifyBuffers] = None, stream=None, diagnostics: bool = True,
                   static_scratch: bool = False) -> PreparedVerify:
    """The arguments of csd_verify, checked and marshalled once; see PreparedVerify."""
    fn, args, bf, name = _marshal_verify(logits, draft, tau, lam, ocm, flags, buffers, stream, diagnostics, static_scratch)
    return PreparedVerify(fn, args, name, bf, (logits, draft, ocm, stream))


def csd_verify_static(logits: torch.Tensor, draft: Optional[torch.Tensor], tau: float, lam: int,
                      ocm: Optional[torch.Tensor] = None, flags: int = CSD_APPLY_UPDATES,
                      buffers: Optional[VerifyBuffers] = None, stream=None, diagnostics: bool = True) -> VerifyBuffers:
    """csd_verify on the library's own per-GPU scratch array (the workspace of `buffers` is not used)."""
    return csd_verify(logits, draft, tau, lam, ocm, flags, buffers, stream, diagnostics, static_scratch=True)


def _rows_stride(t: torch.Tensor, what: str) -> int:
    if t.dim() != 3 or t.stride(2) != 1 or (t.shape[0] > 1 and t.shape[1] > 0 and t.stride(0) != t.shape[1] * t.stride(1)):
        raise ValueError(what + " must be [B][rows][V] with equally spaced rows and unit element stride")
    return t.stride(1) if (t.shape[0] * t.shape[1]) > 1 else max(t.shape[2], t.stride(1))


def csd_verify_shards_workspace_bytes(B: int, k: int) -> int:
    return int(load_library().csd_verify_shards_workspace_bytes(B, k))


def csd_shard_draft_logits(logits_shard: torch.Tensor, base: int, draft: torch.Tensor, draft_logit: torch.Tensor,
                           stream=None) -> None:
    """draft_logit[b][i] = logits_shard[b][i][draft[b][i] - base] for the draft tokens this shard owns."""
    B, K1, Vs = logits_shard.shape
    rc = load_library().csd_shard_draft_logits(_ptr(logits_shard), _dtype_code(logits_shard),
                                               _rows_stride(logits_shard, "logits_shard"), B, K1 - 1, Vs, int(base),
                                               _ptr(draft), _ptr(draft_logit), _stream(stream))
    if rc != CSD_OK:
        raise CsdError(rc, "csd_shard_draft_logits")


def csd_verify_shards(shard_partials, shard_base, draft_logit: torch.Tensor, draft: torch.Tensor, V: int, tau: float,
                      lam: int, ocm: Optional[torch.Tensor] = None, flags: int = CSD_APPLY_UPDATES,
                      buffers: Optional[VerifyBuffers] = None, stream=None) -> VerifyBuffers:
    """Enqueue one verification step from the row partials of vocabulary shards (tensors as returned by
    csd_row_partials, [rows][per_row][4] int32), their first token ids, and the [B][k] draft logits."""
    B, k = draft.shape
    n = len(shard_partials)
    if buffers is None:
        buffers = VerifyBuffers.allocate(B, k, V, CSD_DTYPE_F32, draft.device)
    bf = buffers
    need = csd_verify_shards_workspace_bytes(B, k)
    if bf.workspace.numel() < need:
        bf.workspace = torch.empty((need,), dtype=torch.uint8, device=draft.device)
    ptrs = (ctypes.c_void_p * n)(*[t.data_ptr() for t in shard_partials])
    per_row = (ctypes.c_int * n)(*[int(t.shape[1]) for t in shard_partials])
    bases = (ctypes.c_int * n)(*[int(x) for x in shard_base])
    rc = load_library().csd_verify_shards(
        n, ptrs, per_row, bases, _ptr(draft_logit), _ptr(draft), B, k, V, float(tau), int(lam) & 0xFFFFFFFF, _ptr(ocm),
        0 if ocm is None else ocm.numel(), int(flags), _ptr(bf.accept_len), _ptr(bf.next_token), _ptr(bf.argmax),
        _ptr(bf.row_max), _ptr(bf.row_sumexp), _ptr(bf.ratio), _ptr(bf.p_draft), _ptr(bf.pos_flags), _ptr(bf.rej_log),
        _ptr(bf.status), _ptr(bf.workspace), bf.workspace.numel(), _stream(stream))
    if rc != CSD_OK:
        raise CsdError(rc, "csd_verify_shards")
    return bf


def csd_verify_sampled_workspace_bytes(B: int, k: int, V: int, dtype: int) -> int:
    return int(load_library().csd_verify_sampled_workspace_bytes(B, k, V, dtype))


@dataclass
class SampledBuffers:
    """Outputs and scratch of csd_verify_sampled for one shape, allocated once and reused across calls."""
    B: int
    k: int
    V: int
    dtype: int
    accept_len: torch.Tensor
    next_token: torch.Tensor
    tstar: torch.Tensor
    bonus_token: torch.Tensor
    alpha: torch.Tensor
    p_draft: torch.Tensor
    q_draft: torch.Tensor
    ratio: torch.Tensor
    pos_flags: torch.Tensor
    rej_log: torch.Tensor
    status: torch.Tensor
    workspace: torch.Tensor

    @staticmethod
    def allocate(B: int, k: int, V: int, dtype: int, device="cuda") -> "SampledBuffers":
        nbytes = csd_verify_sampled_workspace_bytes(B, k, V, dtype)
        if nbytes == 0:
            raise CsdError(CSD_EINVAL, "csd_verify_sampled_workspace_bytes")
        e = lambda shape, dt: torch.empty(shape, dtype=dt, device=device)
        return SampledBuffers(
            B, k, V, dtype,
            accept_len=e((B,), torch.int32), next_token=e((B,), torch.int32), tstar=e((B, k), torch.int32),
            bonus_token=e((B,), torch.int32), alpha=e((B, k), torch.float32), p_draft=e((B, k), torch.float32),
            q_draft=e((B, k), torch.float32), ratio=e((B, k), torch.float32), pos_flags=e((B, k), torch.uint8),
            rej_log=e((B, k), torch.int64), status=torch.zeros((CSD_STATUS_WORDS,), dtype=torch.int32, device=device),
            workspace=e((nbytes,), torch.uint8))


def csd_verify_sampled(target_logits: torch.Tensor, draft_logits: torch.Tensor, draft: torch.Tensor, temperature: float,
                       u_accept: torch.Tensor, u_draw: torch.Tensor, tau: float, lam: int,
                       ocm: Optional[torch.Tensor] = None, flags: int = CSD_APPLY_UPDATES,
                       buffers: Optional[SampledBuffers] = None, stream=None, diagnostics: bool = True) -> SampledBuffers:
    """Enqueue one verification step at a sampling temperature.  target_logits [B][k+1][V], draft_logits [B][k][V]
    (same dtype), draft [B][k] int32, u_accept [B][k] and u_draw [B][k+1] float32."""
    B, K1, V = target_logits.shape
    k = K1 - 1
    if tuple(draft_logits.shape) != (B, k, V) or draft_logits.dtype != target_logits.dtype:
        raise ValueError("draft_logits must be [B][k][V] of the target's dtype")
    if draft.dtype != torch.int32 or tuple(draft.shape) != (B, k) or not draft.is_contiguous():
        raise ValueError("draft must be a contiguous int32 [B][k] tensor")
    for t, shape, name in ((u_accept, (B, k), "u_accept"), (u_draw, (B, K1), "u_draw")):
        if t.dtype != torch.float32 or tuple(t.shape) != shape or not t.is_contiguous():
            raise ValueError(name + " must be a contiguous float32 tensor of shape %r" % (shape,))
    dt = _dtype_code(target_logits)
    if buffers is None:
        buffers = SampledBuffers.allocate(B, k, V, dt, target_logits.device)
    elif (buffers.B, buffers.k, buffers.V, buffers.dtype) != (B, k, V, dt):
        raise ValueError("buffers were allocated for another shape")
    if ocm is not None and (ocm.dtype != torch.int64 or not ocm.is_contiguous()):
        raise ValueError("ocm must be a contiguous int64 tensor")
    bf = buffers
    opt = (lambda t: _ptr(t)) if diagnostics else (lambda t: None)
    rc = load_library().csd_verify_sampled(
        _ptr(target_logits), _ptr(draft_logits) if k else None, dt, _rows_stride(target_logits, "target_logits"),
        _rows_stride(draft_logits, "draft_logits") if k else V, _ptr(draft), B, k, V, float(temperature),
        _ptr(u_accept), _ptr(u_draw), float(tau), int(lam) & 0xFFFFFFFF, _ptr(ocm), 0 if ocm is None else ocm.numel(),
        int(flags), _ptr(bf.accept_len), _ptr(bf.next_token), opt(bf.tstar), opt(bf.bonus_token), opt(bf.alpha),
        opt(bf.p_draft), opt(bf.q_draft), opt(bf.ratio), opt(bf.pos_flags), opt(bf.rej_log), _ptr(bf.status),
        _ptr(bf.workspace), bf.workspace.numel(), _stream(stream))
    if rc != CSD_OK:
        raise CsdError(rc, "csd_verify_sampled")
    return bf


def csd_ocm_update(ocm: torch.Tensor, keys: torch.Tensor, weights: Optional[torch.Tensor] = None,
                   status: Optional[torch.Tensor] = None, stream=None, n_dev: Optional[torch.Tensor] = None) -> None:
    """T[key] += weight for every entry (keys: int64 CSD_OCM_KEY values; weights: int32 or None = 1).
    n_dev: optional int64 device tensor [1]; only the first min(len(keys), n_dev) entries are applied."""
    if n_dev is not None and (n_dev.dtype != torch.int64 or n_dev.numel() != 1):
        raise ValueError("n_dev must be an int64 tensor with one element")
    if keys.dtype != torch.int64 or not keys.is_contiguous():
        raise ValueError("keys must be contiguous int64")
    if weights is not None and (weights.dtype != torch.int32 or weights.numel() != keys.numel()
                                or not weights.is_contiguous()):
        raise ValueError("weights must be contiguous int32, one per key")
    rc = load_library().csd_ocm_update(_ptr(ocm), ocm.numel(), _ptr(keys), _ptr(weights), keys.numel(), _ptr(n_dev),
                                       _ptr(status), _stream(stream))
    if rc != CSD_OK:
        raise CsdError(rc, "csd_ocm_update")


def csd_ocm_reset(ocm: torch.Tensor, stream=None) -> None:
    rc = load_library().csd_ocm_reset(_ptr(ocm), ocm.numel(), _stream(stream))
    if rc != CSD_OK:
        raise CsdError(rc, "csd_ocm_reset")


def csd_ocm_lookup(ocm: torch.Tensor, keys: torch.Tensor, stream=None) -> torch.Tensor:
    counts = torch.empty((keys.numel(),), dtype=torch.int32, device=keys.device)
    rc = load_library().csd_ocm_lookup(_ptr(ocm), ocm.numel(), _ptr(keys), _ptr(counts), keys.numel(), _stream(stream))
    if rc != CSD_OK:
        raise CsdError(rc, "csd_ocm_lookup")
    return counts


def csd_ocm_merge(dst: torch.Tensor, src: torch.Tensor, status: Optional[torch.Tensor] = None, stream=None) -> None:
    """T_dst[pair] += T_src[pair] for every pair of src (both int64 tables of power-of-two size)."""
    rc = load_library().csd_ocm_merge(_ptr(dst), dst.numel(), _ptr(src), src.numel(), _ptr(status), _stream(stream))
    if rc != CSD_OK:
        raise CsdError(rc, "csd_ocm_merge")


def csd_ocm_export(ocm: torch.Tensor, max_entries: Optional[int] = None, stream=None, out=None):
    """Enqueue the export; returns (keys int64 [max_entries], counts int32 [max_entries], n int64 [1]) on the device.
    Entries beyond n are unwritten.  out: the three tensors to write into (nothing is allocated then)."""
    if out is not None:
        keys, counts, n = out
        max_entries = keys.numel()
    else:
        if max_entries is None:
            max_entries = ocm.numel()
        keys = torch.empty((max_entries,), dtype=torch.int64, device=ocm.device)
        counts = torch.empty((max_entries,), dtype=torch.int32, device=ocm.device)
        n = torch.empty((1,), dtype=torch.int64, device=ocm.device)
    rc = load_library().csd_ocm_export(_ptr(ocm), ocm.numel(), _ptr(keys) if max_entries else None,
                                       _ptr(counts) if max_entries else None, max_entries, _ptr(n), _stream(stream))
    if rc != CSD_OK:
        raise CsdError(rc, "csd_ocm_export")
    return keys, counts, n


def csd_row_partials_per_row(rows: int, V: int, dtype: int) -> int:
    return int(load_library().csd_row_partials_per_row(rows, V, dtype))


def csd_row_partials(logits: torch.Tensor, partials: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Enqueue the streaming pass alone.  logits: [rows][V] or [B][k+1][V]; returns an int32 tensor
    [rows][per_row][4] whose records are csd_row_partial {m, cref, s (float bits), idx}."""
    V = logits.shape[-1]
    rows = logits.numel() // V if V else 0
    if logits.stride(-1) != 1:
        raise ValueError("logits must have unit element stride")
    row_stride = logits.stride(-2) if logits.dim() > 1 and rows > 1 else max(V, logits.stride(-2) if logits.dim() > 1 else V)
    dt = _dtype_code(logits)
    per_row = csd_row_partials_per_row(rows, V, dt)
    if per_row == 0:
        raise CsdError(CSD_EINVAL, "csd_row_partials_per_row")
    if partials is None:
        partials = torch.empty((rows, per_row, 4), dtype=torch.int32, device=logits.device)
    rc = load_library().csd_row_partials(_ptr(logits), dt, row_stride, rows, V, _ptr(partials),
                                         partials.numel() * 4, _stream(stream))
    if rc != CSD_OK:
        raise CsdError(rc, "csd_row_partials")
    return partials
