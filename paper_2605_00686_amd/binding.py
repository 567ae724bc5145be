"""Thin ctypes binding of the C ABI in include/moe.h: same names, argument
marshalling only.  Torch supplies device memory and streams; every step of the
path runs in the HIP library.  There is no fallback: if libmoe_hip.so is
missing the import of this module fails."""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_hip.so")

MOE_OK = 0
MOE_ERR_INVALID_ARG, MOE_ERR_UNSUPPORTED, MOE_ERR_WORKSPACE = -1, -2, -3
MOE_ERR_NOT_READY, MOE_ERR_HIP, MOE_ERR_TIMEOUT, MOE_ERR_BAD_ROUTING, MOE_ERR_CAPACITY = -4, -5, -6, -7, -8
MOE_DT_F32, MOE_DT_BF16 = 0, 1
MOE_SIGNAL_PER_TILE, MOE_SIGNAL_PER_DEST = 0, 1
MOE_SCOPE_AGENT, MOE_SCOPE_SYSTEM = 0, 1
MOE_SCHED_STATIC, MOE_SCHED_READY_QUEUE = 0, 1
MOE_NUM_STATS = 20

EXPORTS = ("moe_workspace_bytes", "moe_num_flags", "moe_status_string", "moe_workspace_init", "moe_route",
           "moe_dispatch", "moe_dispatch_noalloc", "moe_megakernel_forward", "moe_combine", "moe_probe_mfma",
           "moe_probe_stream")


class MoeProblem(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("T", "d", "E", "k", "f", "R", "dtype", "tile_m", "tile_n",
                                              "signal_mode", "fence_scope")] + [("epoch", ctypes.c_uint32),
                                                                                 ("group_size", ctypes.c_int32),
                                                                                 ("scheduler", ctypes.c_int32),
                                                                                 ("capacity", ctypes.c_int32),
                                                                                 ("wait_ticks", ctypes.c_uint32),
                                                                                 ("fuse_ffn", ctypes.c_int32)]


class MoeError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
_lib = ctypes.CDLL(LIB_PATH)
_vp, _pp = ctypes.c_void_p, ctypes.POINTER(MoeProblem)
_lib.moe_workspace_bytes.restype = ctypes.c_size_t
_lib.moe_workspace_bytes.argtypes = [_pp]
_lib.moe_num_flags.restype = ctypes.c_size_t
_lib.moe_num_flags.argtypes = [_pp]
_lib.moe_status_string.restype = ctypes.c_char_p
_lib.moe_status_string.argtypes = [ctypes.c_int]
_lib.moe_workspace_init.argtypes = [_pp, _vp, _vp]
_lib.moe_route.argtypes = [_pp] + [_vp] * 6
_lib.moe_dispatch.argtypes = [_pp] + [_vp] * 10
_lib.moe_dispatch_noalloc.argtypes = [_pp] + [_vp] * 9
_lib.moe_megakernel_forward.argtypes = [_pp] + [_vp] * 19
_lib.moe_combine.argtypes = [_pp] + [_vp] * 7
_lib.moe_probe_mfma.argtypes = [_vp, ctypes.c_int32, ctypes.c_int32, _vp, _vp]
_lib.moe_probe_stream.argtypes = [_vp, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int32,
                                  ctypes.c_int32, _vp, _vp]
for _n in ("moe_workspace_init", "moe_route", "moe_dispatch", "moe_dispatch_noalloc", "moe_megakernel_forward",
           "moe_combine", "moe_probe_mfma", "moe_probe_stream"):
    getattr(_lib, _n).restype = ctypes.c_int


def problem(T, d, E, k, f, R, dtype, tile_m=0, tile_n=0, signal_mode=MOE_SIGNAL_PER_DEST,
            fence_scope=MOE_SCOPE_AGENT, epoch=1, group_size=0, scheduler=0, capacity=0, wait_ticks=0,
            fuse_ffn=0) -> MoeProblem:
    if isinstance(dtype, torch.dtype):
        dtype = MOE_DT_F32 if dtype == torch.float32 else MOE_DT_BF16
    elif isinstance(dtype, str):
        dtype = MOE_DT_F32 if dtype == "f32" else MOE_DT_BF16
    return MoeProblem(T, d, E, k, f, R, dtype, tile_m, tile_n, signal_mode, fence_scope, epoch, group_size, scheduler,
                      capacity, wait_ticks, fuse_ffn)


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors, contiguous"
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _check(rc, where):
    if rc != MOE_OK:
        raise MoeError(rc, where)


def status_string(status: int) -> str:
    return _lib.moe_status_string(int(status)).decode()


def moe_workspace_bytes(p: MoeProblem) -> int:
    return int(_lib.moe_workspace_bytes(ctypes.byref(p)))


def moe_num_flags(p: MoeProblem) -> int:
    return int(_lib.moe_num_flags(ctypes.byref(p)))


def moe_workspace_init(p, workspace, stream=None):
    _check(_lib.moe_workspace_init(ctypes.byref(p), _ptr(workspace), _stream(stream)), "moe_workspace_init")


def moe_route(p, x, Wg, gate_bias, topk_idx, topk_w, stream=None):
    _check(_lib.moe_route(ctypes.byref(p), _ptr(x), _ptr(Wg), _ptr(gate_bias), _ptr(topk_idx), _ptr(topk_w),
                          _stream(stream)), "moe_route")


def moe_dispatch(p, x, topk_idx, counts, offsets, perm, inv_perm, x_perm, status_dev, workspace, stream=None):
    _check(_lib.moe_dispatch(ctypes.byref(p), _ptr(x), _ptr(topk_idx), _ptr(counts), _ptr(offsets), _ptr(perm),
                             _ptr(inv_perm), _ptr(x_perm), _ptr(status_dev), _ptr(workspace), _stream(stream)),
           "moe_dispatch")


def moe_dispatch_noalloc(p, x, topk_idx, counts, offsets, perm, inv_perm, x_perm, status_dev, stream=None):
    _check(_lib.moe_dispatch_noalloc(ctypes.byref(p), _ptr(x), _ptr(topk_idx), _ptr(counts), _ptr(offsets), _ptr(perm),
                                     _ptr(inv_perm), _ptr(x_perm), _ptr(status_dev), _stream(stream)),
           "moe_dispatch_noalloc")


def moe_megakernel_forward(p, x, Wg, gate_bias, W1, W3, W2, topk_idx, topk_w, counts, offsets, perm, inv_perm,
                           slot_flag, staging, flags, out, stats, workspace, stream=None):
    _check(_lib.moe_megakernel_forward(ctypes.byref(p), _ptr(x), _ptr(Wg), _ptr(gate_bias), _ptr(W1), _ptr(W3),
                                       _ptr(W2), _ptr(topk_idx), _ptr(topk_w), _ptr(counts), _ptr(offsets),
                                       _ptr(perm), _ptr(inv_perm), _ptr(slot_flag), _ptr(staging), _ptr(flags),
                                       _ptr(out), _ptr(stats), _ptr(workspace), _stream(stream)),
           "moe_megakernel_forward")


def moe_combine(p, staging, flags, slot_flag, topk_w, out, status_dev, stream=None):
    _check(_lib.moe_combine(ctypes.byref(p), _ptr(staging), _ptr(flags), _ptr(slot_flag), _ptr(topk_w), _ptr(out),
                            _ptr(status_dev), _stream(stream)), "moe_combine")


def moe_probe_mfma(frag, iters, workgroups, sink, stream=None):
    _check(_lib.moe_probe_mfma(_ptr(frag), int(iters), int(workgroups), _ptr(sink), _stream(stream)), "moe_probe_mfma")


def moe_probe_stream(buf, span_bytes, stride_bytes, bytes_per_workgroup, workgroups, wavefronts, to_lds, sink, stream=None):
    _check(_lib.moe_probe_stream(_ptr(buf), int(span_bytes), int(stride_bytes), int(bytes_per_workgroup), int(workgroups),
                                 int(wavefronts), int(to_lds), _ptr(sink), _stream(stream)), "moe_probe_stream")


class Buffers:
    """Device buffers for one problem shape (allocation only; no arithmetic)."""

    def __init__(self, p: MoeProblem, device="cuda"):
        dt = torch.float32 if p.dtype == MOE_DT_F32 else torch.bfloat16
        N = p.T * p.k
        i32 = dict(dtype=torch.int32, device=device)
        self.p = p
        self.topk_idx = torch.empty((p.T, p.k), **i32)
        self.topk_w = torch.empty((p.T, p.k), dtype=torch.float32, device=device)
        self.counts = torch.empty(p.E, **i32)
        self.offsets = torch.empty(p.E + 1, **i32)
        self.perm = torch.empty(p.E * p.capacity if p.capacity > 0 else N, **i32)  # sorted rows, padded or ragged
        self.inv_perm = torch.empty(N, **i32)
        self.slot_flag = torch.empty(N, **i32)
        self.staging = torch.empty((N, p.d), dtype=dt, device=device)
        self.out = torch.empty((p.T, p.d), dtype=dt, device=device)
        self.flags = torch.zeros(max(1, moe_num_flags(p)), **i32)
        self.stats = torch.zeros(MOE_NUM_STATS, dtype=torch.int64, device=device)
        nbytes = moe_workspace_bytes(p)
        if nbytes == 0:
            raise MoeError(MOE_ERR_UNSUPPORTED, "moe_workspace_bytes")
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
        off = (-self.workspace.data_ptr()) % 256
        self.workspace = self.workspace[off:off + nbytes]
        moe_workspace_init(p, self.workspace)


def forward(p: MoeProblem, buf: Buffers, x, Wg, gate_bias, W1, W3, W2, stream=None):
    """One pass of the whole hot path.  With Wg None, buf.topk_idx / buf.topk_w are inputs."""
    moe_megakernel_forward(p, x, Wg, gate_bias, W1, W3, W2, buf.topk_idx, buf.topk_w, buf.counts, buf.offsets,
                           buf.perm, buf.inv_perm, buf.slot_flag, buf.staging, buf.flags, buf.out, buf.stats,
                           buf.workspace, stream)
    return buf.out
