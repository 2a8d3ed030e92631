"""ctypes binding of libmlpo.so: the same entry points as include/mlpo.h, argument marshalling only.

Every step of the update runs in the library's HIP kernels; nothing here computes.  Tensors may be anything with a
``data_ptr()`` (torch tensors on the device or in pinned host memory) or plain integer addresses; streams anything
with a ``cuda_stream`` attribute (torch.cuda.Stream) or an integer hipStream_t handle.  There is no fallback: if the
library has not been built, the first call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Iterable, Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmlpo.so")

MLPO_OK, MLPO_EINVAL, MLPO_EHIP, MLPO_ENOMEM, MLPO_EIO = 0, -1, -2, -3, -4
TIER_HBM, TIER_HOST, TIER_HOST_GRADS, TIER_FILE = 0, 1, 2, 3
HALF_BF16, HALF_FP16 = 0, 1
MAX_SLOTS = 64

TILE_DEFAULT = 8192

EXPORTS = ("mlpo_last_error", "mlpo_version", "mlpo_line_lead", "mlpo_state_floats", "mlpo_state_pack",
           "mlpo_state_unpack",
           "mlpo_norm_workspace_bytes", "mlpo_grad_unscale_norm", "mlpo_grad_unscale_norm_keep", "mlpo_grad_unscale_norm_static", "mlpo_grad_accumulate", "mlpo_grad_accumulate_norm",
           "mlpo_grad_norm_finish", "mlpo_adamw_step", "mlpo_stream_staging_bytes", "mlpo_stream_bounce_bytes",
           "mlpo_stream_update", "mlpo_stream_flush", "mlpo_assign_tiers", "mlpo_update_bandwidth",
           "mlpo_kernel_timing", "mlpo_kernel_times", "mlpo_shutdown")


class MlpoError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"mlpo error {code}: {text}")
        self.code = code


class HParamsC(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("bias_correction", C.c_int32), ("l2_mode", C.c_int32)]


class SubgroupC(C.Structure):
    _fields_ = [("p", C.c_void_p), ("m", C.c_void_p), ("v", C.c_void_p), ("g", C.c_void_p), ("p16", C.c_void_p),
                ("n", C.c_uint64), ("tier", C.c_int32), ("tile_elems", C.c_int32), ("half_format", C.c_int32),
                ("lead", C.c_int32)]


class StepScalarsC(C.Structure):
    _fields_ = [("norm", C.c_float), ("clip_coef", C.c_float), ("gmul", C.c_float), ("found_inf", C.c_uint32)]


class SlotCacheC(C.Structure):
    _fields_ = [("magic", C.c_uint32), ("n_slots", C.c_int32), ("clock", C.c_uint64),
                ("owner", C.c_int32 * MAX_SLOTS), ("dirty", C.c_uint8 * MAX_SLOTS), ("stamp", C.c_uint64 * MAX_SLOTS),
                ("owner_p", C.c_void_p * MAX_SLOTS), ("fetches", C.c_uint64), ("flushes", C.c_uint64),
                ("hits", C.c_uint64)]


class FileExtentC(C.Structure):
    _fields_ = [("fd", C.c_int32), ("reserved", C.c_int32), ("offset", C.c_uint64)]


class FileStatsC(C.Structure):
    _fields_ = [("bytes_read", C.c_uint64), ("bytes_written", C.c_uint64), ("read_seconds", C.c_double),
                ("write_seconds", C.c_double), ("wall_seconds", C.c_double)]


class PathStatsC(C.Structure):
    _fields_ = [("path_id", C.c_uint64), ("used", C.c_int32), ("reserved", C.c_int32), ("stats", FileStatsC)]


class FlushTargetC(C.Structure):
    _fields_ = [("tier", C.c_int32), ("reserved", C.c_int32), ("state", C.c_void_p), ("file", FileExtentC)]


FLUSH_IN_PLACE = -1


class StreamCfgC(C.Structure):
    _fields_ = [("n_slots", C.c_int32), ("mode", C.c_int32), ("chunk_elems", C.c_uint64),
                ("staging", C.c_void_p), ("staging_bytes", C.c_size_t), ("h2d", C.c_void_p), ("compute", C.c_void_p),
                ("d2h", C.c_void_p), ("direct_blocks", C.c_int32), ("reserved", C.c_int32),
                ("cache", C.POINTER(SlotCacheC)), ("files", C.POINTER(FileExtentC)), ("bounce", C.c_void_p),
                ("bounce_bytes", C.c_size_t), ("file_slots", C.c_int32), ("file_threads", C.c_int32),
                ("file_stats", C.POINTER(FileStatsC)), ("flush_to", C.POINTER(FlushTargetC)),
                ("path_stats", C.POINTER(PathStatsC)), ("path_stats_cap", C.c_int32), ("reserved2", C.c_int32)]


@dataclass
class HParams:
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.01
    bias_correction: bool = True
    l2_mode: bool = False

    def c(self) -> HParamsC:
        return HParamsC(self.lr, self.beta1, self.beta2, self.eps, self.weight_decay, int(self.bias_correction),
                        int(self.l2_mode))


_lib = None


def lib():
    """The loaded library.  Raises if it is missing: there is no other implementation to fall back to."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; "
                               "g.build()' at the repository root)")
        # Stream handles and device pointers are only meaningful inside one HIP runtime.  PyTorch wheels carry their
        # own copy of it, so when torch is installed it is imported first: the library then binds to the runtime
        # torch uses instead of bringing a second one into the process.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(LIB_PATH)
        L.mlpo_last_error.restype = C.c_char_p
        L.mlpo_last_error.argtypes = []
        L.mlpo_version.restype = C.c_int32
        L.mlpo_version.argtypes = []
        L.mlpo_line_lead.restype = C.c_int32
        L.mlpo_line_lead.argtypes = [C.c_void_p]
        L.mlpo_state_floats.restype = C.c_uint64
        L.mlpo_state_floats.argtypes = [C.c_uint64, C.c_int32]
        L.mlpo_state_pack.restype = C.c_int
        L.mlpo_state_pack.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_int32, C.c_int32, C.c_void_p,
                                      C.c_void_p]
        L.mlpo_state_unpack.restype = C.c_int
        L.mlpo_state_unpack.argtypes = [C.c_void_p, C.c_uint64, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_void_p]
        L.mlpo_norm_workspace_bytes.restype = C.c_size_t
        L.mlpo_norm_workspace_bytes.argtypes = []
        L.mlpo_grad_unscale_norm.restype = C.c_int
        L.mlpo_grad_unscale_norm.argtypes = [C.c_void_p, C.c_int32, C.c_float, C.c_float, C.c_void_p, C.c_size_t,
                                             C.c_void_p, C.c_void_p]
        L.mlpo_grad_unscale_norm_keep.restype = C.c_int
        L.mlpo_grad_unscale_norm_keep.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_float, C.c_float, C.c_void_p,
                                                  C.c_size_t, C.c_void_p, C.c_void_p]
        L.mlpo_grad_unscale_norm_static.restype = C.c_int
        L.mlpo_grad_unscale_norm_static.argtypes = [C.c_void_p, C.c_int32, C.c_float, C.c_float, C.c_void_p, C.c_void_p]
        L.mlpo_grad_accumulate.restype = C.c_int
        L.mlpo_grad_accumulate.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_int32, C.c_int32, C.c_int32,
                                           C.c_void_p]
        L.mlpo_grad_accumulate_norm.restype = C.c_int
        L.mlpo_grad_accumulate_norm.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_int32, C.c_int32, C.c_int32,
                                                C.c_float, C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p]
        L.mlpo_grad_norm_finish.restype = C.c_int
        L.mlpo_grad_norm_finish.argtypes = [C.c_void_p, C.c_size_t, C.c_float, C.c_float, C.c_void_p, C.c_void_p]
        L.mlpo_adamw_step.restype = C.c_int
        L.mlpo_adamw_step.argtypes = [C.c_void_p, C.c_int32, C.POINTER(HParamsC), C.c_int64, C.c_void_p, C.c_void_p]
        L.mlpo_stream_staging_bytes.restype = C.c_size_t
        L.mlpo_stream_staging_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_uint64]
        L.mlpo_stream_bounce_bytes.restype = C.c_size_t
        L.mlpo_stream_bounce_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_uint64, C.c_void_p]
        L.mlpo_stream_update.restype = C.c_int
        L.mlpo_stream_update.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.POINTER(HParamsC), C.c_int64,
                                         C.c_void_p, C.POINTER(StreamCfgC), C.POINTER(C.c_int32)]
        L.mlpo_stream_flush.restype = C.c_int
        L.mlpo_stream_flush.argtypes = [C.c_void_p, C.c_int32, C.POINTER(StreamCfgC)]
        L.mlpo_assign_tiers.restype = C.c_int
        L.mlpo_assign_tiers.argtypes = [C.c_int32, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_int32),
                                        C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.mlpo_update_bandwidth.restype = C.c_int
        L.mlpo_update_bandwidth.argtypes = [C.c_int32] + [C.POINTER(C.c_double)] * 3
        L.mlpo_kernel_timing.restype = C.c_int
        L.mlpo_kernel_timing.argtypes = [C.c_int32]
        L.mlpo_kernel_times.restype = C.c_int
        L.mlpo_kernel_times.argtypes = [C.c_int32, C.POINTER(C.c_float), C.c_int32, C.POINTER(C.c_int32)]
        L.mlpo_shutdown.restype = C.c_int
        L.mlpo_shutdown.argtypes = []
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != MLPO_OK:
        raise MlpoError(rc, lib().mlpo_last_error().decode("utf-8", "replace"))


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr())
    return int(x)


def _stream(s) -> Optional[int]:
    if s is None:
        return None
    h = getattr(s, "cuda_stream", s)
    return int(h) or None


def subgroup(p, m, v, g, p16, n: Optional[int] = None, tier: int = TIER_HBM, tile_elems: int = 0,
             half: int = HALF_BF16) -> SubgroupC:
    """One descriptor from five buffers (tensors or addresses).  ``n`` defaults to the gradient tensor's length."""
    if n is None:
        n = g.numel()
    return SubgroupC(_ptr(p), _ptr(m), _ptr(v), _ptr(g), _ptr(p16), int(n), int(tier), int(tile_elems), int(half), 0)


def tiled_subgroup(state, g, p16, n: Optional[int] = None, tier: int = TIER_HBM,
                   tile_elems: int = TILE_DEFAULT, half: int = HALF_BF16, lead: int = 0) -> SubgroupC:
    """Descriptor of a subgroup whose fp32 state is one tiled buffer (see mlpo.h): m and v follow from ``state``."""
    if n is None:
        n = g.numel()
    base = _ptr(state)
    return SubgroupC(base, base + 4 * tile_elems, base + 8 * tile_elems, _ptr(g), _ptr(p16), int(n), int(tier),
                     int(tile_elems), int(half), int(lead))


def mlpo_line_lead(p16) -> int:
    """The ``lead`` that makes the 128-byte lines of p16 begin at the same elements as those of the state buffer."""
    return int(lib().mlpo_line_lead(_ptr(p16)))


line_lead = mlpo_line_lead


def mlpo_state_floats(n: int, tile_elems: int) -> int:
    return int(lib().mlpo_state_floats(n, tile_elems))


def mlpo_state_pack(p, m, v, n: int, tile_elems: int, state, stream=None, lead: int = 0) -> None:
    _check(lib().mlpo_state_pack(_ptr(p), _ptr(m), _ptr(v), n, tile_elems, lead, _ptr(state), _stream(stream)))


def mlpo_state_unpack(state, n: int, tile_elems: int, p, m, v, stream=None, lead: int = 0) -> None:
    _check(lib().mlpo_state_unpack(_ptr(state), n, tile_elems, lead, _ptr(p), _ptr(m), _ptr(v), _stream(stream)))


class SubgroupTable:
    """A contiguous host array of descriptors, built once and passed to many calls."""

    def __init__(self, subgroups: Iterable[SubgroupC]):
        sgs = list(subgroups)
        self.n = len(sgs)
        self.array = (SubgroupC * max(self.n, 1))(*sgs)

    def __len__(self) -> int:
        return self.n


def _table(sgs) -> SubgroupTable:
    return sgs if isinstance(sgs, SubgroupTable) else SubgroupTable(sgs)


def mlpo_version() -> int:
    return int(lib().mlpo_version())


def mlpo_norm_workspace_bytes() -> int:
    return int(lib().mlpo_norm_workspace_bytes())


def mlpo_grad_unscale_norm(sgs, inv_scale: float, max_norm: float, workspace, workspace_bytes: int, out,
                           stream=None) -> None:
    t = _table(sgs)
    _check(lib().mlpo_grad_unscale_norm(t.array, t.n, inv_scale, max_norm, _ptr(workspace), workspace_bytes,
                                        _ptr(out), _stream(stream)))


def mlpo_grad_unscale_norm_keep(sgs, keep, inv_scale: float, max_norm: float, workspace, workspace_bytes: int, out,
                                stream=None) -> None:
    """The gradient pass that also leaves device copies of the gradients it reads: ``keep`` has one device tensor /
    address (or None) per subgroup; see mlpo.h."""
    t = _table(sgs)
    if len(keep) != t.n:
        raise ValueError("keep must have one entry per subgroup")
    arr = (C.c_void_p * max(t.n, 1))(*[_ptr(k) for k in keep])
    _check(lib().mlpo_grad_unscale_norm_keep(t.array, t.n, arr, inv_scale, max_norm, _ptr(workspace),
                                             workspace_bytes, _ptr(out), _stream(stream)))


def mlpo_grad_unscale_norm_static(sgs, inv_scale: float, max_norm: float, out, stream=None) -> None:
    """The gradient pass without a workspace argument (the library's own static device array); see mlpo.h."""
    t = _table(sgs)
    _check(lib().mlpo_grad_unscale_norm_static(t.array, t.n, inv_scale, max_norm, _ptr(out), _stream(stream)))


def mlpo_adamw_step(sgs, hp: HParams, step: int, scalars=None, stream=None) -> None:
    t = _table(sgs)
    h = hp.c() if isinstance(hp, HParams) else hp
    _check(lib().mlpo_adamw_step(t.array, t.n, C.byref(h), step, _ptr(scalars), _stream(stream)))


def mlpo_stream_staging_bytes(sgs, n_slots: int, chunk_elems: int = 0) -> int:
    t = _table(sgs)
    return int(lib().mlpo_stream_staging_bytes(t.array, t.n, n_slots, chunk_elems))


STREAM_STAGED, STREAM_DIRECT = 0, 1
CHUNK_WHOLE = (1 << 64) - 1      # chunk_elems: a whole subgroup per transfer (0 lets the library choose)


def stream_cfg(n_slots: int, staging, staging_bytes: int, h2d, compute, d2h, chunk_elems: int = 0,
               cache: Optional[SlotCacheC] = None, direct_blocks: int = 0) -> StreamCfgC:
    """Staged mode: host-tier subgroups travel through ``n_slots`` device staging slots.  ``cache`` (a zero-initialised
    SlotCacheC kept by the caller) lets slots keep their subgroups between steps; ``direct_blocks`` is then the number
    of workgroups of the kernel that exchanges a slot's occupants over the link (0 = the library's default)."""
    cfg = StreamCfgC(n_slots, STREAM_STAGED, chunk_elems, _ptr(staging), staging_bytes, _stream(h2d),
                     _stream(compute), _stream(d2h), direct_blocks, 0, None, None, None, 0, 0, 0, None, None, None, 0,
                     0)
    if cache is not None:
        cfg.cache = C.pointer(cache)
        cfg._keep = cache
    return cfg


def flush_targets(targets) -> "C.Array":
    """Array of mlpo_flush_target from a list with one entry per subgroup: None (stays where it is), a pinned-host
    tensor / address (goes to pinned memory), a device tensor (goes to HBM), an (fd, offset) pair (goes to a file) or a
    ready-made FlushTargetC."""
    arr = (FlushTargetC * max(len(targets), 1))()
    for i, t in enumerate(targets):
        if t is None:
            arr[i] = FlushTargetC(FLUSH_IN_PLACE, 0, None, FileExtentC(-1, 0, 0))
        elif isinstance(t, FlushTargetC):
            arr[i] = t
        elif isinstance(t, tuple):
            arr[i] = FlushTargetC(TIER_FILE, 0, None, FileExtentC(int(t[0]), 0, int(t[1])))
        else:
            tier = TIER_HBM if getattr(t, "is_cuda", False) else TIER_HOST
            arr[i] = FlushTargetC(tier, 0, _ptr(t), FileExtentC(-1, 0, 0))
    return arr


def direct_cfg(host_stream, compute, direct_blocks: int = 0, chunk_elems: int = 0, files=None, bounce=None,
               bounce_bytes: int = 0, file_slots: int = 0, want_file_stats: bool = False,
               file_threads: int = 0, flush_to=None) -> StreamCfgC:
    """Direct mode: the kernel updates the pinned host state in place with ``direct_blocks`` persistent workgroups.
    ``files`` (one (fd, offset) pair or None per subgroup), ``bounce`` (pinned host tensor) and ``file_slots``
    configure the file path; ``cfg.stats`` then holds what it moved after each call if ``want_file_stats``."""
    cfg = StreamCfgC(0, STREAM_DIRECT, chunk_elems, None, 0, _stream(host_stream), _stream(compute), _stream(compute),
                     direct_blocks, 0, None, None, _ptr(bounce), bounce_bytes, file_slots, file_threads, None, None,
                     None, 0, 0)
    if flush_to is not None:
        cfg._flush = flush_targets(flush_to)
        cfg.flush_to = cfg._flush
    if files is not None:
        arr = (FileExtentC * max(len(files), 1))()
        for i, f in enumerate(files):
            if f is not None:
                arr[i] = FileExtentC(int(f[0]), 0, int(f[1]))
            else:
                arr[i] = FileExtentC(-1, 0, 0)
        cfg.files = arr
        cfg._files = arr
    if want_file_stats:
        cfg.stats = FileStatsC()
        cfg.file_stats = C.pointer(cfg.stats)
        cfg.paths = (PathStatsC * 8)()          # per path, in the order the paths come up in the processing order
        cfg.path_stats = cfg.paths
        cfg.path_stats_cap = 8
    return cfg


def mlpo_stream_bounce_bytes(sgs, file_slots: int, chunk_elems: int = 0, flush_to=None) -> int:
    t = _table(sgs)
    arr = flush_targets(flush_to) if flush_to is not None else None
    return int(lib().mlpo_stream_bounce_bytes(t.array, t.n, file_slots, chunk_elems, arr))


def mlpo_stream_update(sgs, order: Optional[Sequence[int]], hp: HParams, step: int, scalars, cfg: StreamCfgC,
                       want_applied: bool = True) -> Optional[bool]:
    """Returns True if the step was enqueued, False if it was skipped because of a non-finite gradient; with
    ``want_applied=False`` the library is not asked (``applied`` = NULL, see mlpo.h) and None is returned."""
    t = _table(sgs)
    h = hp.c() if isinstance(hp, HParams) else hp
    ordp = None
    if order is not None:
        ordp = (C.c_int32 * max(len(order), 1))(*order)
        if len(order) != t.n:
            raise ValueError("order must have one entry per subgroup")
    applied = C.c_int32(-1)
    _check(lib().mlpo_stream_update(t.array, t.n, ordp, C.byref(h), step, _ptr(scalars), C.byref(cfg),
                                    C.byref(applied) if want_applied else None))
    return bool(applied.value) if want_applied else None


def mlpo_stream_flush(sgs, cfg: StreamCfgC) -> None:
    t = _table(sgs)
    _check(lib().mlpo_stream_flush(t.array, t.n, C.byref(cfg)))


def mlpo_assign_tiers(n_subgroups: int, bandwidth: Sequence[float], capacity: Optional[Sequence[int]] = None):
    """(counts per tier, tier of each subgroup id) by Eq. 1; see mlpo.h."""
    n = len(bandwidth)
    bw = (C.c_double * n)(*bandwidth)
    cap = (C.c_int32 * n)(*capacity) if capacity is not None else None
    cnt = (C.c_int32 * n)()
    tiers = (C.c_int32 * max(n_subgroups, 1))()
    _check(lib().mlpo_assign_tiers(n_subgroups, n, bw, cap, cnt, tiers))
    return list(cnt), list(tiers)[:n_subgroups]


def mlpo_update_bandwidth(bandwidth: Sequence[float], bytes_moved: Sequence[float], seconds: Sequence[float]):
    n = len(bandwidth)
    bw = (C.c_double * n)(*bandwidth)
    _check(lib().mlpo_update_bandwidth(n, bw, (C.c_double * n)(*bytes_moved), (C.c_double * n)(*seconds)))
    return list(bw)


def mlpo_grad_accumulate(acc, g, n: Optional[int] = None, first: bool = False, blocks: int = 0, stream=None,
                         half: int = HALF_BF16) -> None:
    """One micro-batch's half-precision gradients into the accumulation buffer; see mlpo.h."""
    if n is None:
        n = g.numel()
    _check(lib().mlpo_grad_accumulate(_ptr(acc), _ptr(g), int(n), 1 if first else 0, int(blocks), int(half),
                                      _stream(stream)))


def mlpo_grad_accumulate_norm(acc, g, n: Optional[int], first: bool, blocks: int, inv_scale: float, workspace,
                              workspace_bytes: int, begin: bool, stream=None, half: int = HALF_BF16) -> None:
    """The last micro-batch of a step: accumulate and gather the gradient statistics; see mlpo.h."""
    if n is None:
        n = g.numel()
    _check(lib().mlpo_grad_accumulate_norm(_ptr(acc), _ptr(g), int(n), 1 if first else 0, int(blocks), int(half),
                                           inv_scale, _ptr(workspace), int(workspace_bytes), 1 if begin else 0,
                                           _stream(stream)))


def mlpo_grad_norm_finish(workspace, workspace_bytes: int, inv_scale: float, max_norm: float, out, stream=None) -> None:
    _check(lib().mlpo_grad_norm_finish(_ptr(workspace), int(workspace_bytes), inv_scale, max_norm, _ptr(out),
                                       _stream(stream)))


def mlpo_kernel_timing(on: bool) -> None:
    _check(lib().mlpo_kernel_timing(1 if on else 0))


def mlpo_kernel_times(which: int, cap: int = 16384) -> list:
    """Durations (ms) of the launches recorded since the last call; see mlpo.h."""
    buf = (C.c_float * max(cap, 1))()
    n = C.c_int32(0)
    _check(lib().mlpo_kernel_times(which, buf, cap, C.byref(n)))
    return [buf[i] for i in range(n.value)]


def mlpo_shutdown() -> None:
    _check(lib().mlpo_shutdown())
