"""ctypes binding of libtokenring.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI declared in
include/tokenring.h; torch tensors are used here for device memory and streams alone.
There is no fallback: if the library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libtokenring.so")

TR_BF16, TR_F32 = 0, 1
TR_MASK_NONE, TR_MASK_CAUSAL_DIAG = 0, 1
TR_SCHED_TOKENRING, TR_SCHED_RING_ATTENTION, TR_SCHED_ZIGZAG, TR_SCHED_HYBRID = 0, 1, 2, 3

STATUS_NAMES = {
    0: "TR_OK", 1: "TR_ERR_NULL", 2: "TR_ERR_DTYPE", 3: "TR_ERR_SHAPE", 4: "TR_ERR_STRIDE",
    5: "TR_ERR_ALIAS", 6: "TR_ERR_UNSUPPORTED", 7: "TR_ERR_WORKSPACE", 8: "TR_ERR_HIP",
}


class TrTensor(ctypes.Structure):
    """Mirror of `tr_tensor` in include/tokenring.h."""
    _fields_ = [
        ("ptr", ctypes.c_void_p), ("dtype", ctypes.c_int32),
        ("B", ctypes.c_int64), ("H", ctypes.c_int64), ("S", ctypes.c_int64), ("D", ctypes.c_int64),
        ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_s", ctypes.c_int64),
    ]


class TokenRingError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is not built. Build it with `python -m paper_2412_20501_amd.build` "
            "(or __graft_entry__.build()); there is no CPU or PyTorch fallback.")
    lib = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER(TrTensor)
    lib.tr_block_attn.argtypes = [P, P, P, ctypes.c_int, ctypes.c_float, P, P, ctypes.c_void_p]
    lib.tr_block_attn.restype = ctypes.c_int
    lib.tr_block_attn_causal_at.argtypes = [P, P, P, ctypes.c_int64, ctypes.c_int64, ctypes.c_float, P, P, ctypes.c_void_p]
    lib.tr_block_attn_causal_at.restype = ctypes.c_int
    lib.tr_block_attn_merge.argtypes = [P, P, P, ctypes.c_int, ctypes.c_float, P, P, ctypes.c_void_p]
    lib.tr_block_attn_merge.restype = ctypes.c_int
    lib.tr_merge.argtypes = [P, P, P, P, ctypes.c_void_p]
    lib.tr_merge.restype = ctypes.c_int
    lib.tr_ring_attn.argtypes = [P, P, P, ctypes.c_int, ctypes.c_int, P, P, ctypes.c_float,
                                 ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.tr_ring_attn.restype = ctypes.c_int
    lib.tr_ring_attn_noalloc.argtypes = [P, P, P, ctypes.c_int, ctypes.c_int, P, P, ctypes.c_float, ctypes.c_void_p]
    lib.tr_ring_attn_noalloc.restype = ctypes.c_int
    lib.tr_time_next_kernel.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    lib.tr_time_next_kernel.restype = ctypes.c_int
    lib.tr_merge_n.argtypes = [P, P, ctypes.POINTER(P), ctypes.POINTER(P), ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    lib.tr_merge_n.restype = ctypes.c_int
    lib.tr_ring_attn_sched.argtypes = [P, P, P, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, P, P, ctypes.c_float,
                                       ctypes.c_void_p]
    lib.tr_ring_attn_sched.restype = ctypes.c_int
    lib.tr_ring_attn_blocks.argtypes = [P, P, P, ctypes.c_int, ctypes.c_int, P, P, ctypes.c_float, ctypes.c_int,
                                        ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.tr_ring_attn_blocks.restype = ctypes.c_int
    lib.tr_ring_attn_blocks_workspace_bytes.argtypes = [P, ctypes.c_int, ctypes.c_int]
    lib.tr_ring_attn_blocks_workspace_bytes.restype = ctypes.c_size_t
    lib.tr_schedule_steps.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int32), ctypes.c_int64]
    lib.tr_schedule_steps.restype = ctypes.c_int64
    lib.tr_ring_attn_workspace_bytes.argtypes = [P, ctypes.c_int]
    lib.tr_ring_attn_workspace_bytes.restype = ctypes.c_size_t
    lib.tr_last_error.argtypes = []
    lib.tr_last_error.restype = ctypes.c_char_p
    lib.tr_version.argtypes = []
    lib.tr_version.restype = ctypes.c_char_p
    return lib


_lib = _load()


def raw_lib():
    """The loaded ctypes library (for tests that call the C ABI with hand-made descriptors)."""
    return _lib


def _check(status: int):
    if status != 0:
        raise TokenRingError(status, _lib.tr_last_error().decode())


def desc(t: torch.Tensor) -> TrTensor:
    """Descriptor of a [B,H,S,D] (or [B,H,S] for lse) torch tensor; no copy is made."""
    if t.dtype == torch.bfloat16:
        dt = TR_BF16
    elif t.dtype == torch.float32:
        dt = TR_F32
    else:
        raise TypeError(f"unsupported dtype {t.dtype}")
    if t.dim() == 3:
        B, H, S = t.shape
        D = 1
        sb, sh, ss = t.stride()
    elif t.dim() == 4:
        B, H, S, D = t.shape
        sb, sh, ss, sd = t.stride()
        if D > 1 and sd != 1:
            raise ValueError("innermost (D) stride must be 1")
    else:
        raise ValueError("expected a [B,H,S,D] or [B,H,S] tensor")
    return TrTensor(t.data_ptr() if t.numel() else None, dt, B, H, S, D, sb, sh, ss)


def _stream(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def tr_version() -> str:
    return _lib.tr_version().decode()


def tr_block_attn(q, k, v, mask_kind, scale, out, lse, stream=None):
    """block_out, block_lse <- Attention(Q, K, V) into `out`, `lse` (see tokenring.h)."""
    _check(_lib.tr_block_attn(desc(q), desc(k), desc(v), int(mask_kind), float(scale), desc(out), desc(lse), _stream(stream)))


def tr_block_attn_causal_at(q, k, v, q_pos0, k_pos0, scale, out, lse, stream=None):
    """Block step with the causal rule at chunk positions q_pos0 / k_pos0 (see tokenring.h)."""
    _check(_lib.tr_block_attn_causal_at(desc(q), desc(k), desc(v), int(q_pos0), int(k_pos0), float(scale),
                                        desc(out), desc(lse), _stream(stream)))


def tr_block_attn_merge(q, k, v, mask_kind, scale, out_acc, lse_acc, stream=None):
    """Block step whose epilogue applies the Update to the fp32 accumulators (see tokenring.h)."""
    _check(_lib.tr_block_attn_merge(desc(q), desc(k), desc(v), int(mask_kind), float(scale), desc(out_acc), desc(lse_acc),
                                    _stream(stream)))


def tr_merge(out_acc, lse_acc, block_out, block_lse, stream=None):
    """Out, Lse <- Update(block_out, block_lse), in place on out_acc / lse_acc."""
    _check(_lib.tr_merge(desc(out_acc), desc(lse_acc), desc(block_out), desc(block_lse), _stream(stream)))


def tr_merge_n(out, lse, block_outs, block_lses, accumulate=False, stream=None):
    """out, lse <- n-ary merge of the partial results (plus the old out/lse if accumulate)."""
    n = len(block_outs)
    if len(block_lses) != n:
        raise ValueError("block_outs and block_lses differ in length")
    P = ctypes.POINTER(TrTensor)
    bo = [desc(t) for t in block_outs]
    bl = [desc(t) for t in block_lses]
    bo_arr = (P * max(n, 1))(*[ctypes.pointer(d) for d in bo])
    bl_arr = (P * max(n, 1))(*[ctypes.pointer(d) for d in bl])
    _check(_lib.tr_merge_n(desc(out), desc(lse), bo_arr, bl_arr, n, int(bool(accumulate)), _stream(stream)))


def tr_time_next_kernel(start_event, stop_event):
    """Arms two timing events for this thread's next kernel launch (see tokenring.h).

    Accepts raw hipEvent_t handles (int) or torch.cuda.Event objects created with
    enable_timing=True; a torch event is recorded once first if it has no handle yet, so
    that torch creates it and later allows elapsed_time() on it.
    """
    def handle(ev):
        if ev is None or isinstance(ev, int):
            return ev
        if not ev.cuda_event:
            ev.record()
        return ev.cuda_event
    _check(_lib.tr_time_next_kernel(handle(start_event), handle(stop_event)))


def tr_ring_attn_sched(q, k, v, n_devices, causal, schedule, out, lse, scale=0.0, n_inner=1, stream=None):
    """tr_ring_attn with a selectable step order (TR_SCHED_*); Update fused into the attention epilogue."""
    _check(_lib.tr_ring_attn_sched(desc(q), desc(k), desc(v), int(n_devices), int(bool(causal)), int(schedule), int(n_inner),
                                   desc(out), desc(lse), float(scale), _stream(stream)))


def tr_ring_attn_blocks_workspace_bytes(q, n_chunks, block_dtype) -> int:
    return int(_lib.tr_ring_attn_blocks_workspace_bytes(desc(q), int(n_chunks), int(block_dtype)))


def tr_ring_attn_blocks(q, k, v, n_chunks, causal, out, lse, block_dtype, workspace, scale=0.0, stream=None):
    """Algorithm 1 as tr_block_attn + tr_merge per step, the block result stored as block_dtype (TR_F32 / TR_BF16)."""
    _check(_lib.tr_ring_attn_blocks(desc(q), desc(k), desc(v), int(n_chunks), int(bool(causal)), desc(out), desc(lse),
                                    float(scale), int(block_dtype), workspace.data_ptr(),
                                    workspace.numel() * workspace.element_size(), _stream(stream)))


def tr_schedule_steps(schedule, n_devices, causal, n_inner=1):
    """The block steps of a schedule in execution order: a list of (q_segment, kv_segment, launch_index)."""
    n = int(_lib.tr_schedule_steps(int(schedule), int(n_devices), int(n_inner), int(bool(causal)), None, 0))
    if n < 0:
        raise TokenRingError(-1, _lib.tr_last_error().decode())
    buf = (ctypes.c_int32 * (3 * max(n, 1)))()
    _lib.tr_schedule_steps(int(schedule), int(n_devices), int(n_inner), int(bool(causal)), buf, n)
    return [(buf[3 * i], buf[3 * i + 1], buf[3 * i + 2]) for i in range(n)]


def tr_ring_attn_workspace_bytes(q, n_chunks) -> int:
    return int(_lib.tr_ring_attn_workspace_bytes(desc(q), int(n_chunks)))


def tr_ring_attn(q, k, v, n_chunks, causal, out, lse, scale=0.0, workspace=None, stream=None):
    """Algorithm 1's schedule on one GPU into fp32 `out`, `lse`.

    `workspace` = None: the Update runs fused in the attention epilogue.  Otherwise a
    caller-owned uint8 device tensor of at least tr_ring_attn_workspace_bytes(q, n_chunks)
    bytes selects the two-kernel form (tr_block_attn into the workspace, then tr_merge).
    """
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    _check(_lib.tr_ring_attn(desc(q), desc(k), desc(v), int(n_chunks), int(bool(causal)), desc(out), desc(lse),
                             float(scale), ws_ptr, ws_bytes, _stream(stream)))


def tr_ring_attn_noalloc(q, k, v, n_chunks, causal, out, lse, scale=0.0, stream=None):
    """tr_ring_attn (two-kernel form) with the block workspace inside the library: nothing is allocated (see tokenring.h)."""
    _check(_lib.tr_ring_attn_noalloc(desc(q), desc(k), desc(v), int(n_chunks), int(bool(causal)), desc(out), desc(lse),
                                     float(scale), _stream(stream)))
