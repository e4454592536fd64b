"""ctypes binding over libsd.so: argument marshalling only.

Every function mirrors the C entry point of the same name in include/sd.h.
Tensors are torch CUDA (ROCm) tensors; the binding checks dtype, device,
contiguity and sizes on the host, passes raw device pointers and the current
HIP stream, and never computes anything itself.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsd.so")

SD_SCOPE_GLOBAL = 0
SD_SCOPE_REQUESTS = 1

_STATUS = {0: "SD_OK", 1: "SD_ERR_INVALID_ARG", 2: "SD_ERR_OOM", 3: "SD_ERR_HIP",
           4: "SD_ERR_CAPACITY", 5: "SD_ERR_STATE"}


class SdError(RuntimeError):
    def __init__(self, code: int, msg: str = ""):
        super().__init__("%s%s" % (_STATUS.get(code, str(code)), (": " + msg) if msg else ""))
        self.code = code


class _Config(C.Structure):
    _fields_ = [("vocab", C.c_int32), ("D", C.c_int32), ("P", C.c_int32), ("alpha", C.c_double),
                ("min_score", C.c_double), ("max_batch_slots", C.c_int32),
                ("max_ctx_tokens", C.c_int32), ("max_global_tokens", C.c_int64),
                ("device", C.c_int32), ("den_mode", C.c_int32), ("linear", C.c_int32),
                ("tau", C.c_double)]


class _Trees(C.Structure):
    _fields_ = [("d_n_nodes", C.c_void_p), ("d_tokens", C.c_void_p), ("d_parents", C.c_void_p),
                ("d_match_len", C.c_void_p), ("d_source", C.c_void_p), ("d_scores", C.c_void_p),
                ("d_tree_score", C.c_void_p), ("max_nodes", C.c_int32),
                ("d_use_draft", C.c_void_p)]


class _Stats(C.Structure):
    _fields_ = [("global_tokens", C.c_int64), ("global_docs", C.c_int64),
                ("err_bad_token", C.c_int32), ("err_bad_slot", C.c_int32),
                ("err_ctx_overflow", C.c_int32), ("reserved", C.c_int32),
                ("index_bytes", C.c_int64), ("scratch_bytes", C.c_int64)] + [
        (k, C.c_int64) for k in (
            "spec_requests", "spec_trees", "spec_nodes", "spec_match_len", "spec_from_request",
            "spec_global_list", "spec_global_search", "spec_request_wide", "spec_occ_in_memory",
            "spec_list_rounds", "accept_requests", "accept_len")]

SD_STATIC_SCRATCH_BYTES = 16 << 20
SD_TICK_SLOTS = 1024   # requests the timing variant of sd_speculate keeps marks for


KERNEL_NAMES = ["speculate", "accept", "append", "req_build", "sort_hist", "sort_scan",
                "sort_scatter", "build_other", "insert", "accept_speculate"]


class _Profile(C.Structure):
    _fields_ = [("launches", C.c_int64 * len(KERNEL_NAMES)), ("ms", C.c_double * len(KERNEL_NAMES)),
                ("algo_bytes", C.c_int64 * len(KERNEL_NAMES))]


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libsd.so is not built (%s); run __graft_entry__.build() or "
                          "python -m paper_2411_04975_amd.build" % _LIB_PATH)
    L = C.CDLL(_LIB_PATH)
    vp = C.c_void_p
    L.sd_create.restype = C.c_int
    L.sd_create.argtypes = [C.POINTER(_Config), C.POINTER(vp)]
    L.sd_destroy.restype = None
    L.sd_destroy.argtypes = [vp]
    L.sd_last_error.restype = C.c_char_p
    L.sd_last_error.argtypes = [vp]
    L.sd_max_nodes.restype = C.c_int32
    L.sd_max_nodes.argtypes = [vp]
    L.sd_speculate_static.restype = C.c_int
    L.sd_speculate_static.argtypes = [vp, vp, C.c_int32, _Trees, vp]
    L.sd_index_build.restype = C.c_int
    L.sd_index_build.argtypes = [vp, C.c_int, vp, vp, vp, C.c_int32, C.c_int64, vp]
    L.sd_index_entropy.restype = C.c_int
    L.sd_index_entropy.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_double), vp]
    L.sd_index_insert.restype = C.c_int
    L.sd_index_insert.argtypes = [vp, vp, vp, C.c_int32, C.c_int64, vp]
    L.sd_index_append.restype = C.c_int
    L.sd_index_append.argtypes = [vp, vp, vp, vp, C.c_int32, vp]
    L.sd_speculate.restype = C.c_int
    L.sd_speculate.argtypes = [vp, vp, C.c_int32, _Trees, vp]
    L.sd_accept.restype = C.c_int
    L.sd_accept.argtypes = [vp, _Trees, C.c_int32, vp, vp, vp, vp, vp]
    L.sd_accept_append.restype = C.c_int
    L.sd_accept_append.argtypes = [vp, _Trees, vp, C.c_int32, vp, vp, vp, vp, vp]
    L.sd_accept_append_speculate.restype = C.c_int
    L.sd_accept_append_speculate.argtypes = [vp, _Trees, vp, C.c_int32, vp, vp, vp, vp, vp]
    L.sd_get_stats.restype = C.c_int
    L.sd_get_stats.argtypes = [vp, C.POINTER(_Stats)]
    L.sd_debug_profile.restype = C.c_int
    L.sd_debug_profile.argtypes = [vp, C.c_int32]
    L.sd_debug_profile_read.restype = C.c_int
    L.sd_debug_profile_read.argtypes = [vp, C.POINTER(_Profile)]
    L.sd_debug_read_request_ticks.restype = C.c_int
    L.sd_debug_read_request_ticks.argtypes = [vp, vp, C.c_int32, C.POINTER(C.c_int32)]
    L.sd_debug_read_unit_ticks.restype = C.c_int
    L.sd_debug_read_unit_ticks.argtypes = [vp, vp, C.c_int64, C.POINTER(C.c_int32)]
    L.sd_debug_read_global.restype = C.c_int
    L.sd_debug_read_global.argtypes = [vp, vp, vp, C.c_int64, C.POINTER(C.c_int64)]
    _lib = L
    return L


class _Ctx:
    """Opaque handle returned by sd_create."""

    def __init__(self, handle, cfg: _Config):
        self.handle = handle
        self.cfg = cfg
        self.max_nodes = int(_load().sd_max_nodes(handle))
        self.device = torch.device("cuda", cfg.device)


def _check(ctx: Optional[_Ctx], code: int):
    if code != 0:
        msg = ""
        if ctx is not None and ctx.handle:
            msg = (_load().sd_last_error(ctx.handle) or b"").decode()
        raise SdError(code, msg)


def _ptr(t: Optional[torch.Tensor], dtype, ctx: _Ctx, min_numel: int, name: str):
    if t is None:
        if min_numel > 0:
            raise ValueError("%s is required" % name)
        return None
    if not isinstance(t, torch.Tensor) or t.dtype != dtype:
        raise TypeError("%s must be a torch tensor of dtype %s" % (name, dtype))
    if t.device != ctx.device:
        raise ValueError("%s must live on %s" % (name, ctx.device))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if t.numel() < min_numel:
        raise ValueError("%s holds %d elements, %d needed" % (name, t.numel(), min_numel))
    return C.c_void_p(t.data_ptr())


def _stream(stream, ctx: _Ctx):
    if stream is None:
        stream = torch.cuda.current_stream(ctx.device)
    return C.c_void_p(stream.cuda_stream)


def sd_create(vocab: int, D: int, P: int, alpha: float, min_score: float, max_batch_slots: int,
              max_ctx_tokens: int, max_global_tokens: int, device: int = 0, den_mode: int = 0,
              linear: int = 0, tau: float = 0.0) -> _Ctx:
    L = _load()
    cfg = _Config(vocab, D, P, alpha, min_score, max_batch_slots, max_ctx_tokens, max_global_tokens,
                  device, den_mode, linear, tau)
    h = C.c_void_p()
    code = L.sd_create(C.byref(cfg), C.byref(h))
    if code != 0:
        raise SdError(code, "sd_create")
    return _Ctx(h, cfg)


def sd_destroy(ctx: _Ctx) -> None:
    if ctx is not None and ctx.handle:
        _load().sd_destroy(ctx.handle)
        ctx.handle = None


class Trees:
    """Caller-owned output buffers of sd_speculate (the sd_trees struct)."""

    def __init__(self, batch: int, max_nodes: int, device):
        i32, f64 = torch.int32, torch.float64
        self.batch, self.max_nodes = batch, max_nodes
        self.n_nodes = torch.zeros(batch, dtype=i32, device=device)
        self.tokens = torch.full((batch, max_nodes), -1, dtype=i32, device=device)
        self.parents = torch.full((batch, max_nodes), -1, dtype=i32, device=device)
        self.match_len = torch.zeros(batch, dtype=i32, device=device)
        self.source = torch.full((batch,), -1, dtype=i32, device=device)
        self.scores = torch.zeros((batch, max_nodes), dtype=f64, device=device)
        self.tree_score = torch.zeros(batch, dtype=f64, device=device)
        self.use_draft = torch.zeros(batch, dtype=i32, device=device)

    def _struct(self, ctx: _Ctx, batch: int) -> _Trees:
        i32, f64 = torch.int32, torch.float64
        mn = self.max_nodes
        return _Trees(_ptr(self.n_nodes, i32, ctx, batch, "n_nodes"),
                      _ptr(self.tokens, i32, ctx, batch * mn, "tokens"),
                      _ptr(self.parents, i32, ctx, batch * mn, "parents"),
                      _ptr(self.match_len, i32, ctx, batch, "match_len"),
                      _ptr(self.source, i32, ctx, batch, "source"),
                      _ptr(self.scores, f64, ctx, batch * mn, "scores"),
                      _ptr(self.tree_score, f64, ctx, batch, "tree_score"), mn,
                      _ptr(self.use_draft, i32, ctx, batch, "use_draft"))


def sd_index_build(ctx: _Ctx, scope: int, slot_ids: Optional[torch.Tensor], tokens: torch.Tensor,
                   seq_offsets: torch.Tensor, n_tokens: int, stream=None) -> None:
    """`n_tokens` = seq_offsets[-1], known to the caller (no device read happens here)."""
    n_seq = int(seq_offsets.numel()) - 1
    if n_seq < 0:
        raise ValueError("seq_offsets needs at least one entry")
    code = _load().sd_index_build(
        ctx.handle, scope,
        _ptr(slot_ids, torch.int32, ctx,
             n_seq if scope == SD_SCOPE_REQUESTS and slot_ids is not None else 0, "slot_ids"),
        _ptr(tokens, torch.int32, ctx, n_tokens, "tokens"),
        _ptr(seq_offsets, torch.int64, ctx, n_seq + 1, "seq_offsets"), n_seq, n_tokens,
        _stream(stream, ctx))
    _check(ctx, code)


def sd_index_insert(ctx: _Ctx, tokens: torch.Tensor, seq_offsets: torch.Tensor, n_tokens: int,
                    stream=None) -> None:
    """Adds documents to the global index; `n_tokens` = seq_offsets[-1], known to the caller."""
    n_seq = int(seq_offsets.numel()) - 1
    if n_seq < 0:
        raise ValueError("seq_offsets needs at least one entry")
    code = _load().sd_index_insert(
        ctx.handle, _ptr(tokens, torch.int32, ctx, n_tokens, "tokens"),
        _ptr(seq_offsets, torch.int64, ctx, n_seq + 1, "seq_offsets"), n_seq, n_tokens,
        _stream(stream, ctx))
    _check(ctx, code)


def sd_index_entropy(ctx: _Ctx, stream=None):
    """(weighted mean entropy of the global index in bits, total weight).  Synchronises."""
    h, w = C.c_double(), C.c_double()
    _check(ctx, _load().sd_index_entropy(ctx.handle, C.byref(h), C.byref(w), _stream(stream, ctx)))
    return float(h.value), float(w.value)


def sd_index_append(ctx: _Ctx, slot_ids: torch.Tensor, new_tokens: torch.Tensor,
                    new_offsets: torch.Tensor, stream=None) -> None:
    n = int(new_offsets.numel()) - 1 if slot_ids is None else int(slot_ids.numel())
    code = _load().sd_index_append(
        ctx.handle, _ptr(slot_ids, torch.int32, ctx, 0 if slot_ids is None else n, "slot_ids"),
        _ptr(new_tokens, torch.int32, ctx, 0 if n == 0 else 1, "new_tokens"),
        _ptr(new_offsets, torch.int32, ctx, n + 1, "new_offsets"), n, _stream(stream, ctx))
    _check(ctx, code)


def _batch_of(slot_ids, trees: "Trees") -> int:
    """slot_ids None: the identity over the trees' whole batch."""
    batch = trees.batch if slot_ids is None else int(slot_ids.numel())
    if batch > trees.batch:
        raise ValueError("trees hold %d requests, batch is %d" % (trees.batch, batch))
    return batch


def sd_speculate(ctx: _Ctx, slot_ids: Optional[torch.Tensor], trees: Trees, stream=None) -> None:
    batch = _batch_of(slot_ids, trees)
    code = _load().sd_speculate(ctx.handle, _ptr(slot_ids, torch.int32, ctx, 0 if slot_ids is None else batch, "slot_ids"),
                                batch, trees._struct(ctx, batch), _stream(stream, ctx))
    _check(ctx, code)


def sd_speculate_static(ctx: _Ctx, slot_ids: torch.Tensor, trees: Trees, stream=None) -> None:
    """sd_speculate with the library's static device array as working memory."""
    batch = _batch_of(slot_ids, trees)
    code = _load().sd_speculate_static(ctx.handle, _ptr(slot_ids, torch.int32, ctx, 0 if slot_ids is None else batch, "slot_ids"),
                                       batch, trees._struct(ctx, batch), _stream(stream, ctx))
    _check(ctx, code)


def sd_accept(ctx: _Ctx, trees: Trees, batch: int, target_tokens: torch.Tensor,
              accept_len: torch.Tensor, accept_path: torch.Tensor, bonus: torch.Tensor,
              stream=None) -> None:
    i32 = torch.int32
    mn = trees.max_nodes
    code = _load().sd_accept(ctx.handle, trees._struct(ctx, batch), batch,
                             _ptr(target_tokens, i32, ctx, batch * (mn + 1), "target_tokens"),
                             _ptr(accept_len, i32, ctx, batch, "accept_len"),
                             _ptr(accept_path, i32, ctx, batch * mn, "accept_path"),
                             _ptr(bonus, i32, ctx, batch, "bonus"), _stream(stream, ctx))
    _check(ctx, code)


def sd_accept_append(ctx: _Ctx, trees: Trees, slot_ids: torch.Tensor, target_tokens: torch.Tensor,
                     accept_len: torch.Tensor, accept_path: torch.Tensor, bonus: torch.Tensor,
                     stream=None) -> None:
    """sd_accept plus sd_index_append of the accepted tokens and the bonus token, one launch."""
    i32 = torch.int32
    mn = trees.max_nodes
    batch = _batch_of(slot_ids, trees)
    code = _load().sd_accept_append(ctx.handle, trees._struct(ctx, batch),
                                    _ptr(slot_ids, i32, ctx, 0 if slot_ids is None else batch, "slot_ids"), batch,
                                    _ptr(target_tokens, i32, ctx, batch * (mn + 1), "target_tokens"),
                                    _ptr(accept_len, i32, ctx, batch, "accept_len"),
                                    _ptr(accept_path, i32, ctx, batch * mn, "accept_path"),
                                    _ptr(bonus, i32, ctx, batch, "bonus"), _stream(stream, ctx))
    _check(ctx, code)


def sd_accept_append_speculate(ctx: _Ctx, trees: Trees, slot_ids: torch.Tensor,
                               target_tokens: torch.Tensor, accept_len: torch.Tensor,
                               accept_path: torch.Tensor, bonus: torch.Tensor, stream=None) -> None:
    """sd_accept_append of the verified drafts in `trees`, then sd_speculate of the next drafts into
    `trees`, one launch."""
    i32 = torch.int32
    mn = trees.max_nodes
    batch = _batch_of(slot_ids, trees)
    code = _load().sd_accept_append_speculate(
        ctx.handle, trees._struct(ctx, batch),
        _ptr(slot_ids, i32, ctx, 0 if slot_ids is None else batch, "slot_ids"), batch,
        _ptr(target_tokens, i32, ctx, batch * (mn + 1), "target_tokens"),
        _ptr(accept_len, i32, ctx, batch, "accept_len"),
        _ptr(accept_path, i32, ctx, batch * mn, "accept_path"),
        _ptr(bonus, i32, ctx, batch, "bonus"), _stream(stream, ctx))
    _check(ctx, code)


def sd_get_stats(ctx: _Ctx) -> dict:
    s = _Stats()
    _check(ctx, _load().sd_get_stats(ctx.handle, C.byref(s)))
    return {k: getattr(s, k) for k, _ in _Stats._fields_ if k != "reserved"}


def sd_debug_read_request_ticks(ctx: _Ctx, batch: int):
    """Per-request phase marks of the last sd_speculate made in profiling mode 3: array
    [batch, 16 waves, 8] of uint32 (see include/sd.h) and the tick rate in kHz."""
    import numpy as np
    t = np.zeros(batch * 16 * 8, np.uint32)
    khz = C.c_int32()
    _check(ctx, _load().sd_debug_read_request_ticks(ctx.handle, t.ctypes.data_as(C.c_void_p), batch,
                                                    C.byref(khz)))
    return t.reshape(batch, 16, 8), int(khz.value)


def sd_debug_read_global(ctx: _Ctx):
    """Test hook: (text, suffix array) of the global index as numpy int32 arrays."""
    import numpy as np
    L = _load()
    n = C.c_int64()
    L.sd_debug_read_global(ctx.handle, None, None, 0, C.byref(n))
    text = np.zeros(max(n.value, 1), np.int32)
    sa = np.zeros(max(n.value, 1), np.int32)
    _check(ctx, L.sd_debug_read_global(ctx.handle, text.ctypes.data_as(C.c_void_p),
                                       sa.ctypes.data_as(C.c_void_p), n.value, C.byref(n)))
    return text[:n.value], sa[:n.value]


def sd_debug_profile(ctx: _Ctx, mode: int) -> None:
    """0 = off, 1 = HIP-event timing of every kernel, 2 = timing + byte-counting variants."""
    _check(ctx, _load().sd_debug_profile(ctx.handle, mode))


def sd_debug_profile_read(ctx: _Ctx) -> dict:
    """Per kernel: launches, total ms and counted algorithmic bytes since the last read."""
    pr = _Profile()
    _check(ctx, _load().sd_debug_profile_read(ctx.handle, C.byref(pr)))
    return {n: dict(launches=int(pr.launches[i]), ms=float(pr.ms[i]),
                    algo_bytes=int(pr.algo_bytes[i])) for i, n in enumerate(KERNEL_NAMES)}


def sd_debug_read_unit_ticks(ctx: _Ctx, batch: int):
    """Microseconds since unit start at four marks (set-up, match, root children, end) for each
    unit expanded by the last sd_speculate made in profiling mode 3: array [batch, 2, P, 4]."""
    import numpy as np
    n = batch * 2 * ctx.cfg.P * 4
    t = np.zeros(n, np.uint32)
    khz = C.c_int32()
    _check(ctx, _load().sd_debug_read_unit_ticks(ctx.handle, t.ctypes.data_as(C.c_void_p), n,
                                                 C.byref(khz)))
    return t.reshape(batch, 2, ctx.cfg.P, 4).astype(np.float64) * (1e3 / max(khz.value, 1))
