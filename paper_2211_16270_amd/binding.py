"""ctypes binding of include/rnnt_joint_loss.h: argument marshalling only.

Functions carry the names of the C entry points.  Device arrays are torch tensors (torch is
used for device memory and streams, nothing else); host arrays are numpy int32.  There is no
fallback: if the shared library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "lib", "librnnt_joint_loss.so")

RNNT_F32, RNNT_BF16 = 0, 1
STATUS_NAMES = ["RNNT_OK", "RNNT_ERR_NULL", "RNNT_ERR_SHAPE", "RNNT_ERR_LENGTH", "RNNT_ERR_LABEL",
                "RNNT_ERR_WORKSPACE", "RNNT_ERR_UNSUPPORTED", "RNNT_ERR_HIP", "RNNT_ERR_WEIGHT"]
EXPORTS = ["rnnt_status_string", "rnnt_last_hip_error", "rnnt_joint_loss_workspace_bytes", "rnnt_joint_loss_plan",
           "rnnt_parallel_iterations", "rnnt_validate_labels_host", "rnnt_joint_loss_fwd_bwd",
           "rnnt_joint_loss_fwd", "rnnt_debug_read_lattice", "rnnt_profile_enable",
           "rnnt_debug_copy_f32", "rnnt_debug_stream_read", "rnnt_debug_mfma_loop", "rnnt_debug_mfma_loop_fp8", "rnnt_profile_kernel_count", "rnnt_profile_kernel_name", "rnnt_profile_read",
           "rnnt_joint_proj_workspace_bytes", "rnnt_joint_proj_loss_fwd_bwd", "rnnt_joint_loss_fwd_bwd_weighted",
           "rnnt_joint_loss_fwd_bwd_static", "rnnt_plan_create", "rnnt_plan_workspace_bytes", "rnnt_plan_describe",
           "rnnt_plan_destroy", "rnnt_joint_loss_fwd_bwd_planned", "rnnt_debug_read_active_tiles"]
RNNT_STATIC_SCRATCH_BYTES = 128 << 20


class RnntDesc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("T_max", ctypes.c_int32), ("U_max", ctypes.c_int32),
                ("H", ctypes.c_int32), ("V", ctypes.c_int32), ("blank", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("accumulate_params", ctypes.c_int32),
                ("keep_scores", ctypes.c_int32), ("input_grads_bf16", ctypes.c_int32),
                ("skip_below_log2", ctypes.c_int32)]


class RnntPlanInfo(ctypes.Structure):
    _fields_ = [("rows_total", ctypes.c_int64), ("rows_padded", ctypes.c_int64),
                ("tiles_total", ctypes.c_int64), ("n_groups", ctypes.c_int32),
                ("n_chunks", ctypes.c_int32), ("group_rows_cap", ctypes.c_int64),
                ("chunk_rows", ctypes.c_int64), ("workspace_bytes", ctypes.c_size_t),
                ("lattice_bytes", ctypes.c_size_t), ("chunk_bytes", ctypes.c_size_t)]


class RnntError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        name = STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else str(status)
        text = lib().rnnt_status_string(status).decode()
        if name == "RNNT_ERR_HIP":
            text += ": " + lib().rnnt_last_hip_error().decode()
        super().__init__(f"{where}: {name} ({text})")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library.  Raises if it was not built (there is no other code path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                           "(hipcc, gfx950) first; this package has no fallback path")
    # PyTorch ships a HIP runtime of its own.  A process must use one runtime only: if this library were
    # loaded first it would bring in the system's, and the GPU calls made after torch has initialised its own
    # would find no device.  Importing torch first makes its runtime the one both sides resolve to.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    L = ctypes.CDLL(LIB_PATH)
    vp, i32p, f32p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32), ctypes.c_void_p
    dp = ctypes.POINTER(RnntDesc)
    L.rnnt_status_string.restype = ctypes.c_char_p
    L.rnnt_status_string.argtypes = [ctypes.c_int]
    L.rnnt_last_hip_error.restype = ctypes.c_char_p
    L.rnnt_last_hip_error.argtypes = []
    L.rnnt_joint_loss_workspace_bytes.restype = ctypes.c_size_t
    L.rnnt_joint_loss_workspace_bytes.argtypes = [dp, i32p, i32p, ctypes.c_size_t]
    L.rnnt_joint_loss_plan.restype = ctypes.c_int
    L.rnnt_joint_loss_plan.argtypes = [dp, i32p, i32p, ctypes.c_size_t, ctypes.POINTER(RnntPlanInfo), i32p]
    L.rnnt_parallel_iterations.restype = ctypes.c_int32
    L.rnnt_parallel_iterations.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64]
    L.rnnt_validate_labels_host.restype = ctypes.c_int
    L.rnnt_validate_labels_host.argtypes = [dp, i32p, i32p]
    L.rnnt_joint_loss_fwd_bwd.restype = ctypes.c_int
    L.rnnt_joint_loss_fwd_bwd.argtypes = [dp, vp, vp, vp, f32p, vp, i32p, i32p, f32p, f32p, f32p, f32p, f32p,
                                          vp, ctypes.c_size_t, vp]
    L.rnnt_joint_loss_fwd_bwd_static.restype = ctypes.c_int
    L.rnnt_joint_loss_fwd_bwd_static.argtypes = [dp, vp, vp, vp, f32p, vp, i32p, i32p, f32p, f32p, f32p, f32p, f32p, vp]
    L.rnnt_plan_create.restype = ctypes.c_int
    L.rnnt_plan_create.argtypes = [dp, i32p, i32p, ctypes.c_size_t, ctypes.c_int32, ctypes.POINTER(ctypes.c_void_p)]
    L.rnnt_plan_workspace_bytes.restype = ctypes.c_size_t
    L.rnnt_plan_workspace_bytes.argtypes = [vp]
    L.rnnt_plan_describe.restype = ctypes.c_int
    L.rnnt_plan_describe.argtypes = [vp, ctypes.POINTER(RnntPlanInfo)]
    L.rnnt_plan_destroy.restype = None
    L.rnnt_plan_destroy.argtypes = [vp]
    L.rnnt_joint_loss_fwd_bwd_planned.restype = ctypes.c_int
    L.rnnt_joint_loss_fwd_bwd_planned.argtypes = [vp, vp, vp, vp, f32p, vp, f32p, f32p, f32p, f32p, f32p, f32p, vp,
                                                   ctypes.c_size_t, vp, vp]
    L.rnnt_joint_loss_fwd_bwd_weighted.restype = ctypes.c_int
    L.rnnt_joint_loss_fwd_bwd_weighted.argtypes = [dp, vp, vp, vp, f32p, vp, i32p, i32p, f32p, f32p, f32p, f32p, f32p,
                                                    f32p, vp, ctypes.c_size_t, vp]
    L.rnnt_joint_proj_workspace_bytes.restype = ctypes.c_size_t
    L.rnnt_joint_proj_workspace_bytes.argtypes = [dp, ctypes.c_int32, ctypes.c_int32, i32p, i32p, ctypes.c_size_t]
    L.rnnt_joint_proj_loss_fwd_bwd.restype = ctypes.c_int
    L.rnnt_joint_proj_loss_fwd_bwd.argtypes = [dp, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, f32p, vp, vp, f32p, vp,
                                               i32p, i32p] + [f32p] * 8 + [vp, ctypes.c_size_t, vp]
    L.rnnt_joint_loss_fwd.restype = ctypes.c_int
    L.rnnt_joint_loss_fwd.argtypes = [dp, vp, vp, vp, f32p, vp, i32p, i32p, f32p, vp, ctypes.c_size_t, vp]
    L.rnnt_debug_read_lattice.restype = ctypes.c_int
    L.rnnt_debug_read_lattice.argtypes = [dp, i32p, i32p, vp, ctypes.c_size_t, ctypes.c_int32, vp, vp]
    L.rnnt_debug_read_active_tiles.restype = ctypes.c_int
    L.rnnt_debug_read_active_tiles.argtypes = [dp, i32p, i32p, vp, ctypes.c_size_t, ctypes.POINTER(ctypes.c_int64),
                                               ctypes.POINTER(ctypes.c_int64)]
    L.rnnt_debug_copy_f32.restype = ctypes.c_int
    L.rnnt_debug_copy_f32.argtypes = [vp, vp, ctypes.c_size_t, vp]
    L.rnnt_debug_stream_read.restype = ctypes.c_int
    L.rnnt_debug_stream_read.argtypes = [vp, ctypes.c_size_t, vp, ctypes.c_int32, ctypes.c_int32, vp]
    L.rnnt_debug_mfma_loop.restype = ctypes.c_int
    L.rnnt_debug_mfma_loop.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int32, vp]
    L.rnnt_debug_mfma_loop_fp8.restype = ctypes.c_int
    L.rnnt_debug_mfma_loop_fp8.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int32, vp]
    L.rnnt_profile_enable.restype = ctypes.c_int
    L.rnnt_profile_enable.argtypes = [ctypes.c_int32]
    L.rnnt_profile_kernel_count.restype = ctypes.c_int32
    L.rnnt_profile_kernel_count.argtypes = []
    L.rnnt_profile_kernel_name.restype = ctypes.c_char_p
    L.rnnt_profile_kernel_name.argtypes = [ctypes.c_int32]
    L.rnnt_profile_read.restype = ctypes.c_int
    L.rnnt_profile_read.argtypes = [ctypes.c_int32, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_double)]
    _lib = L
    return L


def make_desc(B, T_max, U_max, H, V, blank=0, dtype=RNNT_BF16, accumulate_params=0, keep_scores=0,
              input_grads_bf16=0, skip_below_log2=0) -> RnntDesc:
    return RnntDesc(int(B), int(T_max), int(U_max), int(H), int(V), int(blank), int(dtype),
                    int(accumulate_params), int(keep_scores), int(input_grads_bf16), int(skip_below_log2))


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ip(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def rnnt_joint_loss_workspace_bytes(desc: RnntDesc, T_len, U_len, budget_bytes: int = 0) -> int:
    T, U = _i32(T_len), _i32(U_len)
    return int(lib().rnnt_joint_loss_workspace_bytes(ctypes.byref(desc), _ip(T), _ip(U), int(budget_bytes)))


def rnnt_joint_loss_plan(desc: RnntDesc, T_len, U_len, workspace_bytes: int = 0):
    """Returns (status, info dict, sample_group int32[B])."""
    T, U = _i32(T_len), _i32(U_len)
    info = RnntPlanInfo()
    groups = np.full(desc.B, -1, dtype=np.int32)
    st = lib().rnnt_joint_loss_plan(ctypes.byref(desc), _ip(T), _ip(U), int(workspace_bytes),
                                    ctypes.byref(info), _ip(groups))
    d = {name: getattr(info, name) for name, _ in RnntPlanInfo._fields_}
    return int(st), d, groups


def rnnt_parallel_iterations(T: int, U: int, V: int) -> int:
    return int(lib().rnnt_parallel_iterations(int(T), int(U), int(V)))


def rnnt_validate_labels_host(desc: RnntDesc, labels, U_len) -> int:
    lab, U = _i32(labels), _i32(U_len)
    return int(lib().rnnt_validate_labels_host(ctypes.byref(desc), _ip(lab), _ip(U)))


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream_handle(stream) -> Optional[int]:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    h = int(s.cuda_stream)
    return h if h != 0 else None


def rnnt_joint_loss_fwd_bwd(desc: RnntDesc, enc, pred, W_out, b_out, labels, T_len, U_len,
                            loss, d_enc, d_pred, dW_out, db_out, workspace, stream=None) -> int:
    """Raw call: every array argument is a torch CUDA tensor (or numpy for T_len/U_len) of the
    layout the header states.  Returns the status code; enqueues on `stream` (default: torch's
    current stream) without synchronising."""
    T, U = _i32(T_len), _i32(U_len)
    return int(lib().rnnt_joint_loss_fwd_bwd(
        ctypes.byref(desc), _ptr(enc), _ptr(pred), _ptr(W_out), _ptr(b_out), _ptr(labels), _ip(T), _ip(U),
        _ptr(loss), _ptr(d_enc), _ptr(d_pred), _ptr(dW_out), _ptr(db_out), _ptr(workspace),
        int(workspace.numel() * workspace.element_size()) if workspace is not None else 0,
        _stream_handle(stream)))


def rnnt_joint_loss_fwd_bwd_static(desc: RnntDesc, enc, pred, W_out, b_out, labels, T_len, U_len,
                                   loss, d_enc, d_pred, dW_out, db_out, stream=None) -> int:
    """Raw call of the entry point whose workspace is the library's own static device array."""
    T, U = _i32(T_len), _i32(U_len)
    return int(lib().rnnt_joint_loss_fwd_bwd_static(
        ctypes.byref(desc), _ptr(enc), _ptr(pred), _ptr(W_out), _ptr(b_out), _ptr(labels), _ip(T), _ip(U),
        _ptr(loss), _ptr(d_enc), _ptr(d_pred), _ptr(dW_out), _ptr(db_out), _stream_handle(stream)))


class PlanHandle:
    """rnnt_plan_create / rnnt_plan_destroy as an object: the schedule and the pinned length tables of one batch
    geometry, kept between calls."""

    def __init__(self, desc: RnntDesc, T_len, U_len, budget_bytes: int = 0, overlap_lattice: bool = False):
        T, U = _i32(T_len), _i32(U_len)
        h = ctypes.c_void_p()
        st = lib().rnnt_plan_create(ctypes.byref(desc), _ip(T), _ip(U), int(budget_bytes), int(bool(overlap_lattice)),
                                    ctypes.byref(h))
        if st != 0:
            raise RnntError(int(st), "rnnt_plan_create")
        self.handle, self.desc = h, desc

    @property
    def workspace_bytes(self) -> int:
        return int(lib().rnnt_plan_workspace_bytes(self.handle))

    def describe(self) -> dict:
        info = RnntPlanInfo()
        st = lib().rnnt_plan_describe(self.handle, ctypes.byref(info))
        if st != 0:
            raise RnntError(int(st), "rnnt_plan_describe")
        return {name: getattr(info, name) for name, _ in RnntPlanInfo._fields_}

    def close(self):
        if self.handle:
            lib().rnnt_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def rnnt_joint_loss_fwd_bwd_planned(plan: PlanHandle, enc, pred, W_out, b_out, labels, sample_weight,
                                    loss, d_enc, d_pred, dW_out, db_out, workspace, stream=None,
                                    lattice_stream=None) -> int:
    """Raw call with a plan handle; lattice_stream: a torch stream for the lattice sweeps, or None."""
    w = None if sample_weight is None else np.ascontiguousarray(sample_weight, dtype=np.float32)
    wp = None if w is None else w.ctypes.data
    ls = None if lattice_stream is None else int(lattice_stream.cuda_stream)
    return int(lib().rnnt_joint_loss_fwd_bwd_planned(
        plan.handle, _ptr(enc), _ptr(pred), _ptr(W_out), _ptr(b_out), _ptr(labels), wp,
        _ptr(loss), _ptr(d_enc), _ptr(d_pred), _ptr(dW_out), _ptr(db_out), _ptr(workspace),
        int(workspace.numel() * workspace.element_size()) if workspace is not None else 0,
        _stream_handle(stream), ls))


def rnnt_joint_loss_fwd_bwd_weighted(desc: RnntDesc, enc, pred, W_out, b_out, labels, T_len, U_len, sample_weight,
                                     loss, d_enc, d_pred, dW_out, db_out, workspace, stream=None) -> int:
    """Raw call with one weight per sample (host array of B float32, or None for all ones)."""
    T, U = _i32(T_len), _i32(U_len)
    w = None if sample_weight is None else np.ascontiguousarray(sample_weight, dtype=np.float32)
    wp = None if w is None else w.ctypes.data_as(ctypes.POINTER(ctypes.c_float))
    return int(lib().rnnt_joint_loss_fwd_bwd_weighted(
        ctypes.byref(desc), _ptr(enc), _ptr(pred), _ptr(W_out), _ptr(b_out), _ptr(labels), _ip(T), _ip(U), wp,
        _ptr(loss), _ptr(d_enc), _ptr(d_pred), _ptr(dW_out), _ptr(db_out), _ptr(workspace),
        int(workspace.numel() * workspace.element_size()) if workspace is not None else 0,
        _stream_handle(stream)))


def rnnt_joint_loss_fwd(desc: RnntDesc, enc, pred, W_out, b_out, labels, T_len, U_len, loss, workspace,
                        stream=None) -> int:
    T, U = _i32(T_len), _i32(U_len)
    return int(lib().rnnt_joint_loss_fwd(
        ctypes.byref(desc), _ptr(enc), _ptr(pred), _ptr(W_out), _ptr(b_out), _ptr(labels), _ip(T), _ip(U),
        _ptr(loss), _ptr(workspace),
        int(workspace.numel() * workspace.element_size()) if workspace is not None else 0,
        _stream_handle(stream)))


def rnnt_joint_proj_workspace_bytes(desc: RnntDesc, H_A: int, H_L: int, T_len, U_len, budget_bytes: int = 0) -> int:
    T, U = _i32(T_len), _i32(U_len)
    return int(lib().rnnt_joint_proj_workspace_bytes(ctypes.byref(desc), int(H_A), int(H_L), _ip(T), _ip(U),
                                                     int(budget_bytes)))


def rnnt_joint_proj_loss_fwd_bwd(desc: RnntDesc, H_A: int, H_L: int, hA, hL, W_A, b_Z, W_L, W_out, b_out, labels,
                                 T_len, U_len, loss, d_hA, d_hL, dW_A, db_Z, dW_L, dW_out, db_out, workspace,
                                 stream=None) -> int:
    """Raw call of the path with the input projections of Eq. (4) inside (see the header)."""
    T, U = _i32(T_len), _i32(U_len)
    return int(lib().rnnt_joint_proj_loss_fwd_bwd(
        ctypes.byref(desc), int(H_A), int(H_L), _ptr(hA), _ptr(hL), _ptr(W_A), _ptr(b_Z), _ptr(W_L), _ptr(W_out),
        _ptr(b_out), _ptr(labels), _ip(T), _ip(U), _ptr(loss), _ptr(d_hA), _ptr(d_hL), _ptr(dW_A), _ptr(db_Z),
        _ptr(dW_L), _ptr(dW_out), _ptr(db_out), _ptr(workspace),
        int(workspace.numel() * workspace.element_size()) if workspace is not None else 0,
        _stream_handle(stream)))


def rnnt_debug_read_lattice(desc: RnntDesc, T_len, U_len, workspace, b: int):
    """(status, alpha [T_b, U_b+1], beta [T_b, U_b+1]) of sample b after a single-group call."""
    T, U = _i32(T_len), _i32(U_len)
    n = int(T[b]) * (int(U[b]) + 1)
    al = np.zeros(n, dtype=np.float32)
    be = np.zeros(n, dtype=np.float32)
    st = lib().rnnt_debug_read_lattice(ctypes.byref(desc), _ip(T), _ip(U), _ptr(workspace),
                                       int(workspace.numel() * workspace.element_size()), int(b),
                                       al.ctypes.data, be.ctypes.data)
    shape = (int(T[b]), int(U[b]) + 1)
    return int(st), al.reshape(shape), be.reshape(shape)


def rnnt_debug_read_active_tiles(desc: RnntDesc, T_len, U_len, workspace):
    """(status, tiles that went through the backward pass, all tiles) after a call on this workspace."""
    T, U = _i32(T_len), _i32(U_len)
    a, n = ctypes.c_int64(0), ctypes.c_int64(0)
    st = lib().rnnt_debug_read_active_tiles(ctypes.byref(desc), _ip(T), _ip(U), _ptr(workspace),
                                            int(workspace.numel() * workspace.element_size()),
                                            ctypes.byref(a), ctypes.byref(n))
    return int(st), int(a.value), int(n.value)


def rnnt_debug_copy_f32(src, dst, stream=None) -> int:
    """Copies the float32 tensor src into dst (same size, multiple of 4 elements) with the library's
    plain copy kernel."""
    return int(lib().rnnt_debug_copy_f32(_ptr(src), _ptr(dst), int(src.numel()), _stream_handle(stream)))


def rnnt_debug_stream_read(src, out, workgroups: int, iters: int, stream=None) -> int:
    """Every workgroup reads all of `src` (a torch tensor) `iters` times; out: a tensor of workgroups * 4096 bytes."""
    return int(lib().rnnt_debug_stream_read(_ptr(src), int(src.numel() * src.element_size()), _ptr(out),
                                            int(workgroups), int(iters), _stream_handle(stream)))


def rnnt_debug_mfma_loop_fp8(frags, out, workgroups: int, iters: int, stream=None) -> int:
    return int(lib().rnnt_debug_mfma_loop_fp8(_ptr(frags), _ptr(out), int(workgroups), int(iters), _stream_handle(stream)))


def rnnt_debug_mfma_loop(frags, out, workgroups: int, iters: int, stream=None) -> int:
    """Runs the library's MFMA-only loop on the 32 KiB of bf16 operand fragments in `frags`."""
    return int(lib().rnnt_debug_mfma_loop(_ptr(frags), _ptr(out), int(workgroups), int(iters), _stream_handle(stream)))


def rnnt_profile_enable(enable: bool) -> int:
    return int(lib().rnnt_profile_enable(1 if enable else 0))


def rnnt_profile_kernel_count() -> int:
    return int(lib().rnnt_profile_kernel_count())


def rnnt_profile_kernel_name(cls: int) -> str:
    return lib().rnnt_profile_kernel_name(int(cls)).decode()


def rnnt_profile_read():
    """{kernel name: (launches, total_ms)} of everything recorded since rnnt_profile_enable(True)."""
    n = rnnt_profile_kernel_count()
    cnt = (ctypes.c_int64 * n)()
    ms = (ctypes.c_double * n)()
    st = lib().rnnt_profile_read(n, cnt, ms)
    if st != 0:
        raise RnntError(st, "rnnt_profile_read")
    return {rnnt_profile_kernel_name(i): (int(cnt[i]), float(ms[i])) for i in range(n)}


# --------------------------------------------------------------------------------------------
# Convenience on top of the raw calls (allocation of outputs and workspace with torch).
# --------------------------------------------------------------------------------------------
class Workspace:
    """A reusable device workspace (torch uint8 tensor, 256-byte aligned by the allocator)."""

    def __init__(self, nbytes: int, device="cuda:0"):
        import torch
        self.buf = torch.empty(int(nbytes), dtype=torch.uint8, device=device)
        assert self.buf.data_ptr() % 256 == 0


def to_device(batch, device="cuda:0"):
    """synth.Batch -> dict of torch tensors in the storage types the library expects."""
    import torch
    bf16 = batch.wl.dtype == "bf16"
    dt = torch.bfloat16 if bf16 else torch.float32

    def cvt(x):
        t = torch.from_numpy(np.ascontiguousarray(x))
        return t.to(device=device, dtype=dt)

    return dict(enc=cvt(batch.enc), pred=cvt(batch.pred), W_out=cvt(batch.W_out),
                b_out=torch.from_numpy(batch.b_out).to(device),
                labels=torch.from_numpy(np.ascontiguousarray(batch.labels)).to(device),
                T_len=_i32(batch.T_len), U_len=_i32(batch.U_len))


def run_fwd_bwd(dev: dict, B, T_max, U_max, H, V, blank, dtype, workspace: Optional[Workspace] = None,
                budget_bytes: int = 0, accumulate_into=None, stream=None, sample_weight=None, keep_scores=0,
                input_grads_bf16=0, skip_below_log2=0):
    """Allocates outputs (and a workspace unless given), calls rnnt_joint_loss_fwd_bwd (its weighted form if
    sample_weight is given), raises on a non-zero status.  keep_scores, input_grads_bf16: the descriptor's fields of
    those names (with the latter d_enc and d_pred are bfloat16 tensors).  Returns dict(loss, d_enc, d_pred, dW_out, db_out,
    workspace)."""
    import torch
    device = dev["enc"].device
    desc = make_desc(B, T_max, U_max, H, V, blank, dtype, 0 if accumulate_into is None else 1, keep_scores,
                     input_grads_bf16, skip_below_log2)
    if workspace is None:
        n = rnnt_joint_loss_workspace_bytes(desc, dev["T_len"], dev["U_len"], budget_bytes)
        if n == 0:
            raise RnntError(lib().rnnt_joint_loss_plan(ctypes.byref(desc), _ip(dev["T_len"]), _ip(dev["U_len"]),
                                                       0, ctypes.byref(RnntPlanInfo()), None), "plan")
        workspace = Workspace(n, device)
    loss = torch.empty(B, dtype=torch.float32, device=device)
    gdt = torch.bfloat16 if input_grads_bf16 else torch.float32
    d_enc = torch.empty(B, T_max, H, dtype=gdt, device=device)
    d_pred = torch.empty(B, U_max + 1, H, dtype=gdt, device=device)
    if accumulate_into is None:
        dW = torch.empty(H, V, dtype=torch.float32, device=device)
        db = torch.empty(V, dtype=torch.float32, device=device)
    else:
        dW, db = accumulate_into
    if sample_weight is None:
        st = rnnt_joint_loss_fwd_bwd(desc, dev["enc"], dev["pred"], dev["W_out"], dev["b_out"], dev["labels"],
                                     dev["T_len"], dev["U_len"], loss, d_enc, d_pred, dW, db, workspace.buf, stream)
    else:
        st = rnnt_joint_loss_fwd_bwd_weighted(desc, dev["enc"], dev["pred"], dev["W_out"], dev["b_out"], dev["labels"],
                                              dev["T_len"], dev["U_len"], sample_weight, loss, d_enc, d_pred, dW, db,
                                              workspace.buf, stream)
    if st != 0:
        raise RnntError(st, "rnnt_joint_loss_fwd_bwd")
    return dict(loss=loss, d_enc=d_enc, d_pred=d_pred, dW_out=dW, db_out=db, workspace=workspace, desc=desc)


def proj_to_device(proj, dtype: str, device="cuda:0"):
    """synth.ProjInputs -> dict of torch tensors in the storage types the library expects."""
    import torch
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32

    def cvt(x):
        return torch.from_numpy(np.ascontiguousarray(x)).to(device=device, dtype=dt)

    return dict(hA=cvt(proj.hA), hL=cvt(proj.hL), W_A=cvt(proj.W_A), W_L=cvt(proj.W_L),
                b_Z=torch.from_numpy(np.ascontiguousarray(proj.b_Z)).to(device))


def run_proj_fwd_bwd(dev: dict, devp: dict, B, T_max, U_max, H, V, blank, dtype, workspace: Optional[Workspace] = None,
                     budget_bytes: int = 0, accumulate_into=None, stream=None, keep_scores=0):
    """Allocates outputs (and a workspace unless given), calls rnnt_joint_proj_loss_fwd_bwd, raises on a
    non-zero status.  `dev` as from to_device (enc/pred unused), `devp` as from proj_to_device."""
    import torch
    device = devp["hA"].device
    H_A, H_L = int(devp["hA"].shape[-1]), int(devp["hL"].shape[-1])
    desc = make_desc(B, T_max, U_max, H, V, blank, dtype, 0 if accumulate_into is None else 1, keep_scores)
    if workspace is None:
        n = rnnt_joint_proj_workspace_bytes(desc, H_A, H_L, dev["T_len"], dev["U_len"], budget_bytes)
        if n == 0:
            raise RnntError(2, "rnnt_joint_proj_workspace_bytes")
        workspace = Workspace(n, device)
    f32 = dict(dtype=torch.float32, device=device)
    out = dict(loss=torch.empty(B, **f32), d_hA=torch.empty(B, T_max, H_A, **f32),
               d_hL=torch.empty(B, U_max + 1, H_L, **f32))
    if accumulate_into is None:
        out.update(dW_A=torch.empty(H_A, H, **f32), db_Z=torch.empty(H, **f32), dW_L=torch.empty(H_L, H, **f32),
                   dW_out=torch.empty(H, V, **f32), db_out=torch.empty(V, **f32))
    else:
        out.update(accumulate_into)
    st = rnnt_joint_proj_loss_fwd_bwd(desc, H_A, H_L, devp["hA"], devp["hL"], devp["W_A"], devp["b_Z"], devp["W_L"],
                                      dev["W_out"], dev["b_out"], dev["labels"], dev["T_len"], dev["U_len"],
                                      out["loss"], out["d_hA"], out["d_hL"], out["dW_A"], out["db_Z"], out["dW_L"],
                                      out["dW_out"], out["db_out"], workspace.buf, stream)
    if st != 0:
        raise RnntError(st, "rnnt_joint_proj_loss_fwd_bwd")
    out.update(workspace=workspace, desc=desc)
    return out
