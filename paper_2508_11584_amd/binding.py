"""ctypes binding of the C ABI declared in include/vpe.h (same names, argument marshalling only).

There is no fallback: if libvpe.so is missing it is built with hipcc, and if that fails the
import of the library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

VPE_OK, VPE_SKIPPED, VPE_BUSY, VPE_EINVAL, VPE_ENOMEM, VPE_ESTALE, VPE_EHIP = 0, 1, 2, -1, -2, -3, -4
VPE_F32, VPE_BF16 = 0, 1
VPE_MLP_GELU, VPE_MLP_SWIGLU = 0, 1
VPE_HEAD_SEG, VPE_HEAD_DEPTH, VPE_HEAD_DET, VPE_HEAD_DPT = 0, 1, 2, 3
VPE_FLAG_GRAPHS, VPE_FLAG_HOST_ONLY, VPE_FLAG_WALL_CLOCK, VPE_FLAG_TIMING = 1, 2, 4, 8

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libvpe.so")
_lib = None


class vpe_feat(C.Structure):
    _fields_ = [("slot", C.c_int32), ("reserved", C.c_int32), ("frame", C.c_int64)]


class vpe_backbone_cfg(C.Structure):
    _fields_ = [("dim", C.c_int32), ("depth", C.c_int32), ("heads", C.c_int32), ("mlp_hidden", C.c_int32),
                ("mlp_kind", C.c_int32), ("registers", C.c_int32), ("img_h", C.c_int32), ("img_w", C.c_int32),
                ("batch", C.c_int32), ("dtype", C.c_int32), ("taps", C.c_int32 * 4), ("ring_slots", C.c_int32),
                ("flags", C.c_int32), ("ln_eps", C.c_float), ("encoder_lanes", C.c_int32), ("head_streams", C.c_int32),
                ("reserved", C.c_int32), ("weights", C.c_void_p),
                ("weights_bytes", C.c_uint64)]


class vpe_head_cfg(C.Structure):
    _fields_ = [("kind", C.c_int32), ("classes", C.c_int32), ("channels", C.c_int32), ("every_n", C.c_int32),
                ("weights", C.c_void_p), ("weights_bytes", C.c_uint64)]


class VpeError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"vpe error {code}: {msg}")
        self.code = code


def load_library(path: Optional[str] = None):
    """Load libvpe.so (building it first if it has never been built)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or _LIB_PATH
    if not os.path.exists(p):
        from .build import build
        build()
    L = C.CDLL(p)
    vp, i32, i64p = C.c_void_p, C.c_int, C.POINTER(C.c_int64)
    L.vpe_workspace_bytes.argtypes = [C.POINTER(vpe_backbone_cfg), C.POINTER(vpe_head_cfg), i32, C.POINTER(C.c_uint64)]
    L.vpe_create.argtypes = [C.POINTER(vpe_backbone_cfg), C.POINTER(vpe_head_cfg), i32, vp, C.c_uint64, C.POINTER(vp)]
    L.vpe_encode.argtypes = [vp, vp, vp, C.POINTER(vpe_feat)]
    L.vpe_run_head.argtypes = [vp, i32, vpe_feat, vp]
    L.vpe_run_head_static.argtypes = [vp, i32, vpe_feat, vp]
    L.vpe_run_head_latest.argtypes = [vp, i32, vp, C.POINTER(vpe_feat)]
    L.vpe_head_counters.argtypes = [vp, i32, i64p]
    L.vpe_frame_ready.argtypes = [vp, vpe_feat]
    L.vpe_set_head_rate.argtypes = [vp, i32, i32]
    L.vpe_next_encode_stream.argtypes = [vp, C.POINTER(C.c_void_p)]
    L.vpe_preprocess_u8.argtypes = [vp, i32, i32, i32, vp, i32, i32, C.POINTER(C.c_float), C.POINTER(C.c_float), vp]
    L.vpe_encode_at.argtypes = [vp, vp, vp, C.c_double, C.POINTER(vpe_feat)]
    L.vpe_set_head_rate_hz.argtypes = [vp, i32, C.c_double]
    L.vpe_feat_view.argtypes = [vp, vpe_feat, i32, C.POINTER(vp), i64p]
    L.vpe_head_output.argtypes = [vp, i32, i32, C.POINTER(vp), i64p]
    L.vpe_sync.argtypes = [vp]
    L.vpe_head_done.argtypes = [vp, i32]
    L.vpe_wait_head.argtypes = [vp, i32]
    L.vpe_stage_times.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(C.c_float), i32]
    L.vpe_stats.argtypes = [vp, i64p, i64p, i64p, i32]
    L.vpe_time_kernel.argtypes = [vp, i32, i32, C.POINTER(C.c_float), C.POINTER(C.c_double), C.POINTER(C.c_double)]
    L.vpe_last_error.argtypes = [vp]
    L.vpe_last_error.restype = C.c_char_p
    L.vpe_destroy.argtypes = [vp]
    L.vpe_destroy.restype = None
    for n in ("vpe_workspace_bytes", "vpe_create", "vpe_encode", "vpe_encode_at", "vpe_run_head", "vpe_set_head_rate",
              "vpe_set_head_rate_hz", "vpe_preprocess_u8", "vpe_next_encode_stream", "vpe_feat_view",
              "vpe_head_output", "vpe_sync", "vpe_run_head_static", "vpe_head_done", "vpe_wait_head", "vpe_stage_times", "vpe_stats", "vpe_time_kernel", "vpe_run_head_latest", "vpe_head_counters", "vpe_frame_ready"):
        getattr(L, n).restype = C.c_int
    if path is None:
        _lib = L
    return L


def lib():
    return load_library()


# ------------------------------------------------------------------ the C calls, same names
def vpe_last_error(engine=None) -> str:
    return (lib().vpe_last_error(engine) or b"").decode()


def vpe_workspace_bytes(cfg: vpe_backbone_cfg, heads, n_heads: int) -> int:
    out = C.c_uint64(0)
    rc = lib().vpe_workspace_bytes(C.byref(cfg), heads, n_heads, C.byref(out))
    if rc:
        raise VpeError(rc, vpe_last_error())
    return int(out.value)


def vpe_create(cfg: vpe_backbone_cfg, heads, n_heads: int, workspace_ptr: Optional[int], workspace_bytes: int):
    out = C.c_void_p()
    rc = lib().vpe_create(C.byref(cfg), heads, n_heads, workspace_ptr, workspace_bytes, C.byref(out))
    if rc:
        raise VpeError(rc, vpe_last_error())
    return out


def vpe_encode(engine, images_ptr: int, stream_ptr: Optional[int] = None) -> vpe_feat:
    fh = vpe_feat()
    rc = lib().vpe_encode(engine, images_ptr, stream_ptr, C.byref(fh))
    if rc:
        raise VpeError(rc, vpe_last_error(engine))
    return fh


def vpe_preprocess_u8(frames_ptr: int, batch: int, src_h: int, src_w: int, images_ptr: int, dst_h: int, dst_w: int,
                      mean, std, stream_ptr: Optional[int] = None) -> None:
    m = (C.c_float * 3)(*[float(v) for v in mean])
    s = (C.c_float * 3)(*[float(v) for v in std])
    rc = lib().vpe_preprocess_u8(frames_ptr, batch, src_h, src_w, images_ptr, dst_h, dst_w, m, s, stream_ptr)
    if rc:
        raise VpeError(rc, vpe_last_error(None))


def preprocess_u8(frames, out, mean, std, stream=None) -> None:
    """frames: torch uint8 CUDA tensor [B, Hs, Ws, 3]; out: torch float32 CUDA tensor [B, 3, H, W] (written).
    stream: a torch stream, a raw hipStream_t as int (e.g. Engine.next_encode_stream()), or None."""
    assert frames.is_cuda and frames.is_contiguous() and frames.element_size() == 1 and frames.dim() == 4 and frames.shape[3] == 3
    assert out.is_cuda and out.is_contiguous() and out.dtype.is_floating_point and out.element_size() == 4
    assert out.dim() == 4 and out.shape[0] == frames.shape[0] and out.shape[1] == 3
    vpe_preprocess_u8(frames.data_ptr(), frames.shape[0], frames.shape[1], frames.shape[2], out.data_ptr(),
                      out.shape[2], out.shape[3], mean, std,
                      None if stream is None else stream if isinstance(stream, int) else stream.cuda_stream)


def vpe_next_encode_stream(engine) -> Optional[int]:
    out = C.c_void_p()
    rc = lib().vpe_next_encode_stream(engine, C.byref(out))
    if rc:
        raise VpeError(rc, vpe_last_error(engine))
    return out.value


def vpe_encode_at(engine, images_ptr: int, stream_ptr: Optional[int], t_seconds: float) -> vpe_feat:
    fh = vpe_feat()
    rc = lib().vpe_encode_at(engine, images_ptr, stream_ptr, t_seconds, C.byref(fh))
    if rc:
        raise VpeError(rc, vpe_last_error(engine))
    return fh


def vpe_run_head(engine, head: int, fh: vpe_feat, stream_ptr: Optional[int] = None) -> int:
    rc = lib().vpe_run_head(engine, head, fh, stream_ptr)
    if rc < 0:
        raise VpeError(rc, vpe_last_error(engine))
    return rc


def vpe_run_head_static(engine, head: int, fh: vpe_feat, stream_ptr: Optional[int] = None) -> int:
    rc = lib().vpe_run_head_static(engine, head, fh, stream_ptr)
    if rc < 0:
        raise VpeError(rc, vpe_last_error(engine))
    return rc


def vpe_run_head_latest(engine, head: int, stream_ptr: Optional[int] = None):
    """Returns (status, handle): handle is the frame the head was started on, None unless status == VPE_OK."""
    fh = vpe_feat()
    rc = lib().vpe_run_head_latest(engine, head, stream_ptr, C.byref(fh))
    if rc < 0:
        raise VpeError(rc, vpe_last_error(engine))
    return rc, (fh if rc == VPE_OK else None)


def vpe_frame_ready(engine, fh: vpe_feat) -> int:
    """VPE_OK, VPE_BUSY or VPE_ESTALE."""
    rc = lib().vpe_frame_ready(engine, fh)
    if rc < 0 and rc != VPE_ESTALE:
        raise VpeError(rc, vpe_last_error(engine))
    return rc


HEAD_COUNTERS = ("runs", "skips", "missed", "overflow", "busy", "last_run_frame", "seen")


def vpe_head_counters(engine, head: int) -> dict:
    out = (C.c_int64 * 8)()
    rc = lib().vpe_head_counters(engine, head, out)
    if rc:
        raise VpeError(rc, vpe_last_error(engine))
    return {k: int(out[i]) for i, k in enumerate(HEAD_COUNTERS)}


def vpe_set_head_rate(engine, head: int, every_n_frames: int) -> None:
    rc = lib().vpe_set_head_rate(engine, head, every_n_frames)
    if rc:
        raise VpeError(rc, vpe_last_error(engine))


def vpe_set_head_rate_hz(engine, head: int, max_hz: float) -> None:
    rc = lib().vpe_set_head_rate_hz(engine, head, max_hz)
    if rc:
        raise VpeError(rc, vpe_last_error(engine))


def vpe_feat_view(engine, fh: vpe_feat, tap: int):
    ptr = C.c_void_p()
    shape = (C.c_int64 * 3)()
    rc = lib().vpe_feat_view(engine, fh, tap, C.byref(ptr), shape)
    if rc:
        raise VpeError(rc, vpe_last_error(engine))
    return ptr.value, tuple(shape)


def vpe_head_output(engine, head: int, which: int):
    ptr = C.c_void_p()
    shape = (C.c_int64 * 4)()
    rc = lib().vpe_head_output(engine, head, which, C.byref(ptr), shape)
    if rc:
        raise VpeError(rc, vpe_last_error(engine))
    return ptr.value, tuple(shape)


def vpe_sync(engine) -> None:
    rc = lib().vpe_sync(engine)
    if rc:
        raise VpeError(rc, vpe_last_error(engine))


def vpe_head_done(engine, head: int) -> int:
    """VPE_OK or VPE_BUSY."""
    rc = lib().vpe_head_done(engine, head)
    if rc < 0:
        raise VpeError(rc, vpe_last_error(engine))
    return rc


def vpe_wait_head(engine, head: int) -> None:
    rc = lib().vpe_wait_head(engine, head)
    if rc:
        raise VpeError(rc, vpe_last_error(engine))


def vpe_stage_times(engine, n_heads: int):
    """(encode_ms, [head_ms...]); -1 where there is no figure yet."""
    enc = C.c_float(-1.0)
    heads = (C.c_float * max(n_heads, 1))()
    rc = lib().vpe_stage_times(engine, C.byref(enc), heads, n_heads)
    if rc:
        raise VpeError(rc, vpe_last_error(engine))
    return float(enc.value), [float(v) for v in heads][:n_heads]


def vpe_stats(engine, n_heads: int):
    frames = C.c_int64(0)
    runs = (C.c_int64 * max(n_heads, 1))()
    skips = (C.c_int64 * max(n_heads, 1))()
    lib().vpe_stats(engine, C.byref(frames), runs, skips, n_heads)
    return int(frames.value), [int(v) for v in runs][:n_heads], [int(v) for v in skips][:n_heads]


def vpe_time_kernel(engine, which: int, reps: int):
    ms, fl, by = C.c_float(0), C.c_double(0), C.c_double(0)
    rc = lib().vpe_time_kernel(engine, which, reps, C.byref(ms), C.byref(fl), C.byref(by))
    if rc:
        raise VpeError(rc, vpe_last_error(engine))
    return float(ms.value), float(fl.value), float(by.value)


def vpe_destroy(engine) -> None:
    lib().vpe_destroy(engine)


# ------------------------------------------------------------------ convenience wrapper
@dataclass
class HeadCfg:
    kind: int
    weights: np.ndarray        # flat fp32 blob in the documented order
    classes: int = 0
    channels: int = 0
    every_n: int = 1


class Engine:
    """Owns one vpe_engine.  Device memory comes from torch (one uint8 tensor), streams are
    the library's own unless torch streams are passed in."""

    def __init__(self, *, dim, depth, heads, mlp_hidden, img_h, img_w, weights: np.ndarray, taps,
                 mlp_kind=VPE_MLP_GELU, registers=0, batch=1, dtype=VPE_BF16, ring_slots=2, flags=0, ln_eps=1e-6,
                 encoder_lanes=1, head_streams=0,
                 head_cfgs: Sequence[HeadCfg] = (), torch_workspace: bool = True):
        self._keep = [np.ascontiguousarray(weights, dtype=np.float32)]
        cfg = vpe_backbone_cfg()
        cfg.dim, cfg.depth, cfg.heads, cfg.mlp_hidden, cfg.mlp_kind = dim, depth, heads, mlp_hidden, mlp_kind
        cfg.registers, cfg.img_h, cfg.img_w, cfg.batch, cfg.dtype = registers, img_h, img_w, batch, dtype
        cfg.taps = (C.c_int32 * 4)(*taps)
        cfg.ring_slots, cfg.flags, cfg.ln_eps, cfg.encoder_lanes = ring_slots, flags, ln_eps, encoder_lanes
        cfg.head_streams = head_streams
        cfg.weights = self._keep[0].ctypes.data
        cfg.weights_bytes = self._keep[0].nbytes
        self.n_heads = len(head_cfgs)
        harr = (vpe_head_cfg * max(self.n_heads, 1))()
        for i, h in enumerate(head_cfgs):
            blob = np.ascontiguousarray(h.weights, dtype=np.float32)
            self._keep.append(blob)
            harr[i].kind, harr[i].classes, harr[i].channels, harr[i].every_n = h.kind, h.classes, h.channels, h.every_n
            harr[i].weights = blob.ctypes.data
            harr[i].weights_bytes = blob.nbytes
        self.cfg, self.head_arr = cfg, harr
        self.host_only = bool(flags & VPE_FLAG_HOST_ONLY)
        self.dtype = dtype
        self.workspace_bytes = vpe_workspace_bytes(cfg, harr, self.n_heads)
        self._ws = None
        ws_ptr, ws_bytes = None, 0
        if torch_workspace and not self.host_only:
            import torch
            self._ws = torch.empty(self.workspace_bytes + 256, dtype=torch.uint8, device="cuda")
            ws_ptr = (self._ws.data_ptr() + 255) // 256 * 256
            ws_bytes = self.workspace_bytes
        self.handle = vpe_create(cfg, harr, self.n_heads, ws_ptr, ws_bytes)

    # -- calls
    def encode(self, images, stream=None, t: Optional[float] = None) -> vpe_feat:
        """images: torch float32 CUDA tensor [B,3,H,W] (contiguous) -- or None in host-only mode.
        t: capture time of the frame in seconds (for per-head limits in Hz), or None."""
        ptr = sp = None
        if not self.host_only:
            assert images.is_cuda and images.is_contiguous() and images.dtype.is_floating_point and images.element_size() == 4
            assert tuple(images.shape) == (self.cfg.batch, 3, self.cfg.img_h, self.cfg.img_w), images.shape
            ptr, sp = images.data_ptr(), None if stream is None else stream.cuda_stream
        return vpe_encode(self.handle, ptr, sp) if t is None else vpe_encode_at(self.handle, ptr, sp, t)

    def run_head(self, head: int, fh: vpe_feat, stream=None) -> int:
        return vpe_run_head(self.handle, head, fh, None if stream is None else stream.cuda_stream)

    def run_head_static(self, head: int, fh: vpe_feat, stream=None) -> int:
        return vpe_run_head_static(self.handle, head, fh, None if stream is None else stream.cuda_stream)

    def run_head_latest(self, head: int, stream=None):
        return vpe_run_head_latest(self.handle, head, None if stream is None else stream.cuda_stream)

    def frame_ready(self, fh: vpe_feat) -> int:
        return vpe_frame_ready(self.handle, fh)

    def head_counters(self, head: int) -> dict:
        return vpe_head_counters(self.handle, head)

    def next_encode_stream(self) -> Optional[int]:
        """Raw handle of the engine stream the next encode() without a stream argument will run on."""
        return vpe_next_encode_stream(self.handle)

    def set_head_rate(self, head: int, every_n: int) -> None:
        vpe_set_head_rate(self.handle, head, every_n)

    def set_head_rate_hz(self, head: int, max_hz: float) -> None:
        vpe_set_head_rate_hz(self.handle, head, max_hz)

    def sync(self) -> None:
        vpe_sync(self.handle)

    def stats(self):
        return vpe_stats(self.handle, self.n_heads)

    def head_done(self, head: int) -> bool:
        return vpe_head_done(self.handle, head) == VPE_OK

    def wait_head(self, head: int) -> None:
        vpe_wait_head(self.handle, head)

    def stage_times(self):
        return vpe_stage_times(self.handle, self.n_heads)

    def time_kernel(self, which: int, reps: int):
        return vpe_time_kernel(self.handle, which, reps)

    # -- borrowed views as torch tensors (no copy)
    def _as_tensor(self, ptr: int, shape, torch_dtype):
        """Wrap library-owned device memory as a torch tensor (no copy, no ownership)."""
        import torch
        holder = _DevArray(ptr, tuple(int(s) for s in shape), torch_dtype)
        t = torch.as_tensor(holder, device="cuda")
        return t.view(torch.bfloat16) if torch_dtype == torch.bfloat16 else t

    def feat_view(self, fh: vpe_feat, tap: int):
        import torch
        ptr, shape = vpe_feat_view(self.handle, fh, tap)
        return self._as_tensor(ptr, shape, torch.bfloat16 if self.dtype == VPE_BF16 else torch.float32)

    def feat_ptr(self, fh: vpe_feat, tap: int) -> int:
        return vpe_feat_view(self.handle, fh, tap)[0]

    def head_output(self, head: int, which: int):
        import torch
        ptr, shape = vpe_head_output(self.handle, head, which)
        kind = self.head_arr[head].kind
        is_map = which == 1 and kind in (VPE_HEAD_SEG, VPE_HEAD_DET)
        shape = [s for s in shape]
        while len(shape) > 1 and shape[-1] == 1 and len(shape) > (3 if (is_map or kind in (VPE_HEAD_DEPTH, VPE_HEAD_DPT)) else 4):
            shape.pop()
        return self._as_tensor(ptr, shape, torch.uint8 if is_map else torch.float32)

    def close(self) -> None:
        if getattr(self, "handle", None):
            vpe_destroy(self.handle)
            self.handle = None
        self._ws = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class _DevArray:
    """Minimal __cuda_array_interface__ carrier so torch can wrap library-owned device memory."""
    _TYPESTR = {"torch.float32": "<f4", "torch.uint8": "|u1", "torch.bfloat16": "<i2"}

    def __init__(self, ptr: int, shape, torch_dtype):
        self.__cuda_array_interface__ = {"shape": shape, "typestr": self._TYPESTR[str(torch_dtype)],
                                         "data": (ptr, False), "version": 2, "strides": None}
