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
        L.wl_chase.restype = C.c_int
        L.wl_chase.argtypes = [vp, C.c_uint32, C.c_int, vp, vp]
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


def dependent_load_ns(n_lines: int, hops: int, device) -> float:
    """Nanoseconds per load when every load's address comes from the load before it, over a
    working set of n_lines memory lines (128 bytes apart) visited in a seeded random cyclic
    order by one lane.  Every timed walk starts where no walk has been before (or, in a
    working set smaller than the walk, goes round the cycle), so the level of the memory
    system that answers is the one that holds the whole set.  Measurement glue: nothing of the
    method is in it."""
    g = torch.Generator(device="cpu")
    g.manual_seed(1234)
    perm = torch.randperm(n_lines, generator=g, dtype=torch.int64)
    nxt = torch.empty(n_lines, dtype=torch.int64)
    nxt[perm] = torch.roll(perm, -1)
    table = torch.zeros(n_lines * 32, dtype=torch.int32, device=device)
    table[::32] = nxt.to(torch.int32).to(device)
    out = torch.zeros(1, dtype=torch.int32, device=device)
    st = torch.cuda.current_stream(device).cuda_stream
    L = _load()
    times = []
    for rep in range(4):                       # the first walk also loads the kernel
        start = int(perm[(rep * hops) % n_lines])
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        rc = L.wl_chase(C.c_void_p(table.data_ptr()), start, hops, C.c_void_p(out.data_ptr()),
                        C.c_void_p(st))
        e1.record()
        torch.cuda.synchronize()
        assert rc == 0
        times.append(e0.elapsed_time(e1))
    return min(times[1:]) * 1e6 / hops
