"""Simulated greedy verifier and accepted-token collection on the device (workload glue).

The kernels live in csrc/verifier.hip and are built into workloads/libwlverifier.so.  They
stand in for the target LLM in decode-loop benchmarks: the target token at a draft node of
depth k is the k-th ground-truth future token of the request."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csrc", "verifier.hip")
LIB_PATH = os.path.join(_HERE, "libwlverifier.so")
_lib = None


def build() -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB_PATH + ".tmp.%d" % os.getpid()
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
                           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                           "-o", tmp, _SRC])
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libwlverifier.so is not built; run __graft_entry__.build()")
        L = C.CDLL(LIB_PATH)
        vp = C.c_void_p
        L.wl_targets.restype = C.c_int
        L.wl_targets.argtypes = [vp, vp, C.c_int, vp, C.c_int64, vp, vp, C.c_int, vp, vp]
        L.wl_collect.restype = C.c_int
        L.wl_collect.argtypes = [vp, C.c_int, vp, vp, vp, C.c_int, vp, vp, vp, vp]
        L.wl_stream_copy.restype = C.c_int
        L.wl_stream_copy.argtypes = [vp, vp, C.c_int64, vp]
        _lib = L
    return _lib


def _p(t: torch.Tensor):
    assert t.is_cuda and t.is_contiguous() and t.dtype == torch.int32
    return C.c_void_p(t.data_ptr())


def targets(n_nodes, parents, future, pos, target, advance=None) -> None:
    """target[b, 0] = future[b, pos[b]], target[b, 1+j] = future[b, pos[b] + depth(node j)].
    With `advance` (the previous step's accept lengths, -1 before the first step) pos moves on by
    advance + 1 first."""
    B, mn = parents.shape
    assert target.shape == (B, mn + 1) and future.shape[0] == B
    st = torch.cuda.current_stream(parents.device).cuda_stream
    rc = _load().wl_targets(_p(n_nodes), _p(parents), mn, _p(future), future.shape[1], _p(pos),
                            _p(advance) if advance is not None else C.c_void_p(0), B,
                            _p(target), C.c_void_p(st))
    assert rc == 0


def collect(tokens, accept_len, accept_path, bonus, new_tokens, new_offsets, pos) -> None:
    """new tokens of request b = its accepted draft tokens + the bonus token; pos += L + 1."""
    B, mn = tokens.shape
    assert new_tokens.numel() >= B * (mn + 1) and new_offsets.numel() >= B + 1
    st = torch.cuda.current_stream(tokens.device).cuda_stream
    rc = _load().wl_collect(_p(tokens), mn, _p(accept_len), _p(accept_path), _p(bonus), B,
                            _p(new_tokens), _p(new_offsets), _p(pos), C.c_void_p(st))
    assert rc == 0


def stream_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    """dst[:] = src[:] with the hand-written streaming copy kernel (sizes a multiple of 16 B)."""
    assert src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()
    nbytes = src.numel() * src.element_size()
    assert nbytes == dst.numel() * dst.element_size()
    st = torch.cuda.current_stream(src.device).cuda_stream
    rc = _load().wl_stream_copy(C.c_void_p(src.data_ptr()), C.c_void_p(dst.data_ptr()), nbytes,
                                C.c_void_p(st))
    assert rc == 0, rc
