"""Thin ctypes binding over libslimspec.so: argument marshalling only.

Every step of the head (down-projection, vocabulary projection, online
log-sum-exp, top-k, merge) runs in the library's HIP kernels; torch is used here
for device memory and the current stream, nothing else.  There is no CPU or
PyTorch fallback: if the library is missing, loading fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch  # must be imported before the library so that both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libslimspec.so")

SLIMSPEC_BF16 = 0
SLIMSPEC_F32 = 1
SLIMSPEC_KMAX = 64

STATUS_OK = 0
STATUS_INVALID_ARGUMENT = -1
STATUS_UNSUPPORTED = -2
STATUS_WORKSPACE_TOO_SMALL = -3
STATUS_HIP_ERROR = -4
STATUS_SCRATCH_LIMIT = -5
STATIC_SCRATCH_BYTES = 64 << 20

EXPORTED_SYMBOLS = (
    "slimspec_version", "slimspec_workspace_bytes", "slimspec_head_topk", "slimspec_transpose_weights", "slimspec_head_topk_prepared", "slimspec_head_topk_static", "full_head_topk", "truncated_head_topk", "slimspec_head_topk_positions", "slimspec_head_topk_positions_prepared", "slimspec_head_sample", "slimspec_head_sample_prepared", "full_head_sample", "routed_workspace_bytes", "routed_head_topk", "routed_head_topk_prepared",
    "slimspec_status_string", "slimspec_last_hip_error", "slimspec_set_timing_events",
)


class SlimspecShape(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int32), ("d", ctypes.c_int32), ("r", ctypes.c_int32), ("V", ctypes.c_int32)]


class SlimspecError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"slimspec status {status}: {text}")
        self.status = status


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libslimspec.so (built in-tree by build.py); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it with `python -m paper_2605_10453_amd.build` "
            "(there is no fallback implementation)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    shp = ctypes.POINTER(SlimspecShape)
    lib.slimspec_version.restype = ctypes.c_int
    lib.slimspec_version.argtypes = []
    lib.slimspec_workspace_bytes.restype = sz
    lib.slimspec_workspace_bytes.argtypes = [shp, i32]
    lib.slimspec_head_topk.restype = ctypes.c_int
    lib.slimspec_head_topk.argtypes = [vp, vp, vp, shp, i32, vp, vp, vp, sz, vp]
    lib.slimspec_transpose_weights.restype = ctypes.c_int
    lib.slimspec_transpose_weights.argtypes = [vp, i32, i32, vp, vp]
    lib.slimspec_head_topk_prepared.restype = ctypes.c_int
    lib.slimspec_head_topk_prepared.argtypes = [vp, vp, vp, vp, shp, i32, vp, vp, vp, sz, vp]
    lib.slimspec_head_topk_static.restype = ctypes.c_int
    lib.slimspec_head_topk_static.argtypes = [vp, vp, vp, shp, i32, vp, vp, vp]
    lib.full_head_topk.restype = ctypes.c_int
    lib.full_head_topk.argtypes = [vp, vp, ctypes.c_int, shp, i32, vp, vp, vp, sz, vp]
    lib.slimspec_head_topk_positions.restype = ctypes.c_int
    lib.slimspec_head_topk_positions.argtypes = [vp, vp, i32, ctypes.POINTER(ctypes.c_int32), vp, shp, i32, vp, vp, vp, sz, vp]
    lib.slimspec_head_sample.restype = ctypes.c_int
    lib.slimspec_head_sample.argtypes = [vp, vp, vp, shp, i32, ctypes.c_uint64, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.slimspec_head_sample_prepared.restype = ctypes.c_int
    lib.slimspec_head_sample_prepared.argtypes = [vp, vp, vp, vp, shp, i32, ctypes.c_uint64, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.slimspec_head_topk_positions_prepared.restype = ctypes.c_int
    lib.slimspec_head_topk_positions_prepared.argtypes = [vp, vp, i32, ctypes.POINTER(ctypes.c_int32), vp, vp, shp, i32, vp, vp, vp, sz, vp]
    lib.full_head_sample.restype = ctypes.c_int
    lib.full_head_sample.argtypes = [vp, vp, ctypes.c_int, shp, i32, ctypes.c_uint64, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.routed_workspace_bytes.restype = sz
    lib.routed_workspace_bytes.argtypes = [shp, i32]
    lib.routed_head_topk.restype = ctypes.c_int
    lib.routed_head_topk.argtypes = [vp, vp, vp, vp, ctypes.c_int, shp, i32, i32, vp, vp, vp, sz, vp]
    lib.routed_head_topk_prepared.restype = ctypes.c_int
    lib.routed_head_topk_prepared.argtypes = [vp, vp, vp, vp, vp, ctypes.c_int, shp, i32, i32, vp, vp, vp, sz, vp]
    lib.truncated_head_topk.restype = ctypes.c_int
    lib.truncated_head_topk.argtypes = [vp, vp, ctypes.c_int, vp, shp, i32, vp, vp, vp, sz, vp]
    lib.slimspec_status_string.restype = ctypes.c_char_p
    lib.slimspec_status_string.argtypes = [ctypes.c_int]
    lib.slimspec_last_hip_error.restype = ctypes.c_char_p
    lib.slimspec_last_hip_error.argtypes = []
    lib.slimspec_set_timing_events.restype = ctypes.c_int
    lib.slimspec_set_timing_events.argtypes = [vp, vp]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().slimspec_status_string(status).decode()


def _raise(status: int):
    lib = load_library()
    text = lib.slimspec_status_string(status).decode()
    if status == STATUS_HIP_ERROR:
        text += ": " + lib.slimspec_last_hip_error().decode()
    raise SlimspecError(status, text)


def slimspec_version() -> int:
    return int(load_library().slimspec_version())


def slimspec_workspace_bytes(rows: int, d: int, r: int, V: int, k: int) -> int:
    shape = SlimspecShape(rows, d, r, V)
    return int(load_library().slimspec_workspace_bytes(ctypes.byref(shape), k))


def slimspec_set_timing_events(start_event: Optional[torch.cuda.Event],
                               stop_event: Optional[torch.cuda.Event]) -> None:
    """Have later calls record the two events around their vocabulary-projection kernel (None, None: off).

    The events must have been recorded once already so that their HIP handles exist.
    """
    a = None if start_event is None else int(start_event.cuda_event)
    b = None if stop_event is None else int(stop_event.cuda_event)
    st = load_library().slimspec_set_timing_events(a, b)
    if st != STATUS_OK:
        _raise(st)


def _stream_handle(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _dev_ptr(t: torch.Tensor, name: str) -> int:
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _outputs(rows, k, device, out_ids, out_logprobs):
    if out_ids is None:
        out_ids = torch.empty((rows, k), dtype=torch.int32, device=device)
    if out_logprobs is None:
        out_logprobs = torch.empty((rows, k), dtype=torch.float32, device=device)
    if out_ids.dtype != torch.int32 or out_logprobs.dtype != torch.float32:
        raise ValueError("out_ids must be int32 and out_logprobs float32")
    if tuple(out_ids.shape) != (rows, k) or tuple(out_logprobs.shape) != (rows, k):
        raise ValueError("outputs must be [rows, k]")
    return out_ids, out_logprobs


def _workspace(nbytes: int, device, workspace):
    if workspace is None:
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
    return workspace


def slimspec_head_topk(h: torch.Tensor, A: torch.Tensor, B: torch.Tensor, k: int,
                       out_ids: Optional[torch.Tensor] = None, out_logprobs: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None,
                       stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Low-rank head z = (h A) B -> per-row top-k ids and log-probabilities (device tensors).

    h [rows, d], A [d, r], B [r, V]: bf16 device tensors (torch.bfloat16, or int16/uint16 bit patterns).
    Work is enqueued on `stream` (default: torch's current stream); nothing is synchronised.
    """
    rows, d = h.shape
    d2, r = A.shape
    r2, V = B.shape
    if d != d2 or r != r2:
        raise ValueError("shape mismatch between h, A and B")
    for t, n in ((h, "h"), (A, "A"), (B, "B")):
        if t.element_size() != 2:
            raise ValueError(f"{n} must hold bf16 (2-byte) elements")
    out_ids, out_logprobs = _outputs(rows, k, h.device, out_ids, out_logprobs)
    lib = load_library()
    shape = SlimspecShape(rows, d, r, V)
    need = int(lib.slimspec_workspace_bytes(ctypes.byref(shape), k))
    workspace = _workspace(need, h.device, workspace)
    st = lib.slimspec_head_topk(_dev_ptr(h, "h"), _dev_ptr(A, "A"), _dev_ptr(B, "B"), ctypes.byref(shape), k,
                                _dev_ptr(out_ids, "out_ids"), _dev_ptr(out_logprobs, "out_logprobs"),
                                _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                                _stream_handle(stream))
    if st != STATUS_OK:
        _raise(st)
    return out_ids, out_logprobs


def slimspec_transpose_weights(M: torch.Tensor, out: Optional[torch.Tensor] = None,
                               stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """Column-major copy Mt [V, K] of a bf16 weight matrix M [K, V] (made once per matrix)."""
    K, V = M.shape
    if M.element_size() != 2:
        raise ValueError("M must hold bf16 (2-byte) elements")
    if out is None:
        out = torch.empty((V, K), dtype=M.dtype, device=M.device)
    if tuple(out.shape) != (V, K) or out.element_size() != 2:
        raise ValueError("out must be a [V, K] tensor of 2-byte elements")
    lib = load_library()
    st = lib.slimspec_transpose_weights(_dev_ptr(M, "M"), K, V, _dev_ptr(out, "out"), _stream_handle(stream))
    if st != STATUS_OK:
        _raise(st)
    return out


def slimspec_head_topk_prepared(h: torch.Tensor, A: torch.Tensor, B: torch.Tensor, Bt: torch.Tensor, k: int,
                                out_ids: Optional[torch.Tensor] = None, out_logprobs: Optional[torch.Tensor] = None,
                                workspace: Optional[torch.Tensor] = None,
                                stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """slimspec_head_topk with the column-major copy Bt [V, r] of B (see slimspec_transpose_weights) as well."""
    rows, d = h.shape
    d2, r = A.shape
    r2, V = B.shape
    if d != d2 or r != r2 or tuple(Bt.shape) != (V, r):
        raise ValueError("shape mismatch between h, A, B and Bt")
    for t, n in ((h, "h"), (A, "A"), (B, "B"), (Bt, "Bt")):
        if t.element_size() != 2:
            raise ValueError(f"{n} must hold bf16 (2-byte) elements")
    out_ids, out_logprobs = _outputs(rows, k, h.device, out_ids, out_logprobs)
    lib = load_library()
    shape = SlimspecShape(rows, d, r, V)
    need = int(lib.slimspec_workspace_bytes(ctypes.byref(shape), k))
    workspace = _workspace(need, h.device, workspace)
    st = lib.slimspec_head_topk_prepared(_dev_ptr(h, "h"), _dev_ptr(A, "A"), _dev_ptr(B, "B"), _dev_ptr(Bt, "Bt"),
                                         ctypes.byref(shape), k,
                                         _dev_ptr(out_ids, "out_ids"), _dev_ptr(out_logprobs, "out_logprobs"),
                                         _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                                         _stream_handle(stream))
    if st != STATUS_OK:
        _raise(st)
    return out_ids, out_logprobs


def slimspec_head_topk_static(h: torch.Tensor, A: torch.Tensor, B: torch.Tensor, k: int,
                              out_ids: Optional[torch.Tensor] = None, out_logprobs: Optional[torch.Tensor] = None,
                              stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """slimspec_head_topk on the library's built-in scratch: the C call allocates nothing and takes no workspace.

    Pass out_ids / out_logprobs to keep this wrapper from allocating them.
    """
    rows, d = h.shape
    d2, r = A.shape
    r2, V = B.shape
    if d != d2 or r != r2:
        raise ValueError("shape mismatch between h, A and B")
    for t, n in ((h, "h"), (A, "A"), (B, "B")):
        if t.element_size() != 2:
            raise ValueError(f"{n} must hold bf16 (2-byte) elements")
    out_ids, out_logprobs = _outputs(rows, k, h.device, out_ids, out_logprobs)
    shape = SlimspecShape(rows, d, r, V)
    st = load_library().slimspec_head_topk_static(
        _dev_ptr(h, "h"), _dev_ptr(A, "A"), _dev_ptr(B, "B"), ctypes.byref(shape), k,
        _dev_ptr(out_ids, "out_ids"), _dev_ptr(out_logprobs, "out_logprobs"), _stream_handle(stream))
    if st != STATUS_OK:
        _raise(st)
    return out_ids, out_logprobs


def full_head_topk(h: torch.Tensor, W: torch.Tensor, k: int,
                   out_ids: Optional[torch.Tensor] = None, out_logprobs: Optional[torch.Tensor] = None,
                   workspace: Optional[torch.Tensor] = None,
                   stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Full head z = h W -> per-row top-k ids and log-probabilities.  W [d, V] is bf16 or float32."""
    rows, d = h.shape
    d2, V = W.shape
    if d != d2:
        raise ValueError("shape mismatch between h and W")
    if h.element_size() != 2:
        raise ValueError("h must hold bf16 (2-byte) elements")
    if W.dtype == torch.float32:
        w_dtype = SLIMSPEC_F32
    elif W.element_size() == 2:
        w_dtype = SLIMSPEC_BF16
    else:
        raise ValueError("W must be bf16 or float32")
    out_ids, out_logprobs = _outputs(rows, k, h.device, out_ids, out_logprobs)
    lib = load_library()
    shape = SlimspecShape(rows, d, 0, V)
    need = int(lib.slimspec_workspace_bytes(ctypes.byref(shape), k))
    workspace = _workspace(need, h.device, workspace)
    st = lib.full_head_topk(_dev_ptr(h, "h"), _dev_ptr(W, "W"), w_dtype, ctypes.byref(shape), k,
                            _dev_ptr(out_ids, "out_ids"), _dev_ptr(out_logprobs, "out_logprobs"),
                            _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                            _stream_handle(stream))
    if st != STATUS_OK:
        _raise(st)
    return out_ids, out_logprobs


def truncated_head_topk(h: torch.Tensor, W_tr: torch.Tensor, id_map: torch.Tensor, k: int,
                        out_ids: Optional[torch.Tensor] = None, out_logprobs: Optional[torch.Tensor] = None,
                        workspace: Optional[torch.Tensor] = None,
                        stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Full head over the kept columns W_tr [d, V_tr]; ids come back as id_map[column] (id_map: int32 device [V_tr])."""
    rows, d = h.shape
    d2, V = W_tr.shape
    if d != d2:
        raise ValueError("shape mismatch between h and W_tr")
    if h.element_size() != 2:
        raise ValueError("h must hold bf16 (2-byte) elements")
    if id_map.dtype != torch.int32 or tuple(id_map.shape) != (V,):
        raise ValueError("id_map must be int32 [V_tr]")
    if W_tr.dtype == torch.float32:
        w_dtype = SLIMSPEC_F32
    elif W_tr.element_size() == 2:
        w_dtype = SLIMSPEC_BF16
    else:
        raise ValueError("W_tr must be bf16 or float32")
    out_ids, out_logprobs = _outputs(rows, k, h.device, out_ids, out_logprobs)
    lib = load_library()
    shape = SlimspecShape(rows, d, 0, V)
    need = int(lib.slimspec_workspace_bytes(ctypes.byref(shape), k))
    workspace = _workspace(need, h.device, workspace)
    st = lib.truncated_head_topk(_dev_ptr(h, "h"), _dev_ptr(W_tr, "W_tr"), w_dtype, _dev_ptr(id_map, "id_map"),
                                 ctypes.byref(shape), k, _dev_ptr(out_ids, "out_ids"), _dev_ptr(out_logprobs, "out_logprobs"),
                                 _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                                 _stream_handle(stream))
    if st != STATUS_OK:
        _raise(st)
    return out_ids, out_logprobs


def slimspec_head_topk_positions(h: torch.Tensor, A_stack: torch.Tensor, pos_offsets, B: torch.Tensor, k: int,
                                 out_ids: Optional[torch.Tensor] = None, out_logprobs: Optional[torch.Tensor] = None,
                                 workspace: Optional[torch.Tensor] = None,
                                 stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Low-rank head with one down-projection per drafted position: A_stack [n_pos, d, r]; rows
    [pos_offsets[p], pos_offsets[p + 1]) use matrix p (pos_offsets: a host sequence of n_pos + 1 ints)."""
    return _positions(h, A_stack, pos_offsets, B, None, k, out_ids, out_logprobs, workspace, stream)


def slimspec_head_topk_positions_prepared(h: torch.Tensor, A_stack: torch.Tensor, pos_offsets, B: torch.Tensor, Bt: torch.Tensor,
                                          k: int, out_ids: Optional[torch.Tensor] = None,
                                          out_logprobs: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                                          stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """slimspec_head_topk_positions with the column-major copy Bt [V, r] of B as well."""
    return _positions(h, A_stack, pos_offsets, B, Bt, k, out_ids, out_logprobs, workspace, stream)


def _positions(h, A_stack, pos_offsets, B, Bt, k, out_ids, out_logprobs, workspace, stream):
    rows, d = h.shape
    n_pos, d2, r = A_stack.shape
    r2, V = B.shape
    if d != d2 or r != r2:
        raise ValueError("shape mismatch between h, A_stack and B")
    off = [int(v) for v in pos_offsets]
    if len(off) != n_pos + 1:
        raise ValueError("pos_offsets must have n_pos + 1 entries")
    if Bt is not None and tuple(Bt.shape) != (V, r):
        raise ValueError("Bt must be [V, r]")
    for t, n in ((h, "h"), (A_stack, "A_stack"), (B, "B")) + (((Bt, "Bt"),) if Bt is not None else ()):
        if t.element_size() != 2:
            raise ValueError(f"{n} must hold bf16 (2-byte) elements")
    out_ids, out_logprobs = _outputs(rows, k, h.device, out_ids, out_logprobs)
    lib = load_library()
    shape = SlimspecShape(rows, d, r, V)
    need = int(lib.slimspec_workspace_bytes(ctypes.byref(shape), k))
    workspace = _workspace(need, h.device, workspace)
    off_arr = (ctypes.c_int32 * (n_pos + 1))(*off)
    tail = (ctypes.byref(shape), k, _dev_ptr(out_ids, "out_ids"), _dev_ptr(out_logprobs, "out_logprobs"),
            _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if Bt is None:
        st = lib.slimspec_head_topk_positions(_dev_ptr(h, "h"), _dev_ptr(A_stack, "A_stack"), n_pos, off_arr, _dev_ptr(B, "B"), *tail)
    else:
        st = lib.slimspec_head_topk_positions_prepared(_dev_ptr(h, "h"), _dev_ptr(A_stack, "A_stack"), n_pos, off_arr,
                                                       _dev_ptr(B, "B"), _dev_ptr(Bt, "Bt"), *tail)
    if st != STATUS_OK:
        _raise(st)
    return out_ids, out_logprobs


def _sample_outputs(rows, device):
    return (torch.empty((rows,), dtype=torch.float32, device=device), torch.empty((rows,), dtype=torch.int32, device=device),
            torch.empty((rows,), dtype=torch.float32, device=device))


def slimspec_head_sample(h: torch.Tensor, A: torch.Tensor, B: torch.Tensor, k: int, seed: int,
                         workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None):
    """Low-rank head with the outputs of stochastic decoding: (ids, logprobs, lse, sample_ids, sample_logprobs)."""
    return _sample(h, A, B, None, k, seed, workspace, stream)


def slimspec_head_sample_prepared(h: torch.Tensor, A: torch.Tensor, B: torch.Tensor, Bt: torch.Tensor, k: int, seed: int,
                                  workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None):
    """slimspec_head_sample with the column-major copy Bt [V, r] of B as well."""
    return _sample(h, A, B, Bt, k, seed, workspace, stream)


def _sample(h, A, B, Bt, k, seed, workspace, stream):
    rows, d = h.shape
    d2, r = A.shape
    r2, V = B.shape
    if d != d2 or r != r2:
        raise ValueError("shape mismatch between h, A and B")
    out_ids, out_logprobs = _outputs(rows, k, h.device, None, None)
    lse, sid, slp = _sample_outputs(rows, h.device)
    lib = load_library()
    shape = SlimspecShape(rows, d, r, V)
    workspace = _workspace(int(lib.slimspec_workspace_bytes(ctypes.byref(shape), k)), h.device, workspace)
    tail = (ctypes.byref(shape), k, seed, _dev_ptr(out_ids, "out_ids"), _dev_ptr(out_logprobs, "out_logprobs"),
            _dev_ptr(lse, "lse"), _dev_ptr(sid, "sample_ids"), _dev_ptr(slp, "sample_logprobs"),
            _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if Bt is None:
        st = lib.slimspec_head_sample(_dev_ptr(h, "h"), _dev_ptr(A, "A"), _dev_ptr(B, "B"), *tail)
    else:
        if tuple(Bt.shape) != (V, r) or Bt.element_size() != 2:
            raise ValueError("Bt must be a [V, r] tensor of bf16 (2-byte) elements")
        st = lib.slimspec_head_sample_prepared(_dev_ptr(h, "h"), _dev_ptr(A, "A"), _dev_ptr(B, "B"), _dev_ptr(Bt, "Bt"), *tail)
    if st != STATUS_OK:
        _raise(st)
    return out_ids, out_logprobs, lse, sid, slp


def full_head_sample(h: torch.Tensor, W: torch.Tensor, k: int, seed: int,
                     workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None):
    """Full head with the outputs of stochastic decoding: (ids, logprobs, lse, sample_ids, sample_logprobs)."""
    rows, d = h.shape
    d2, V = W.shape
    if d != d2:
        raise ValueError("shape mismatch between h and W")
    w_dtype = SLIMSPEC_F32 if W.dtype == torch.float32 else SLIMSPEC_BF16
    out_ids, out_logprobs = _outputs(rows, k, h.device, None, None)
    lse, sid, slp = _sample_outputs(rows, h.device)
    lib = load_library()
    shape = SlimspecShape(rows, d, 0, V)
    workspace = _workspace(int(lib.slimspec_workspace_bytes(ctypes.byref(shape), k)), h.device, workspace)
    st = lib.full_head_sample(_dev_ptr(h, "h"), _dev_ptr(W, "W"), w_dtype, ctypes.byref(shape), k, seed,
                              _dev_ptr(out_ids, "out_ids"), _dev_ptr(out_logprobs, "out_logprobs"),
                              _dev_ptr(lse, "lse"), _dev_ptr(sid, "sample_ids"), _dev_ptr(slp, "sample_logprobs"),
                              _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                              _stream_handle(stream))
    if st != STATUS_OK:
        _raise(st)
    return out_ids, out_logprobs, lse, sid, slp


def routed_head_topk(h: torch.Tensor, A: torch.Tensor, B: torch.Tensor, W: torch.Tensor, k_route: int, k: int,
                     out_ids: Optional[torch.Tensor] = None, out_logprobs: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None,
                     stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Router-then-exact head: the low-rank head picks k_route ids per row, the full head is evaluated on those only."""
    rows, d = h.shape
    d2, r = A.shape
    r2, V = B.shape
    if d != d2 or r != r2 or tuple(W.shape) != (d, V):
        raise ValueError("shape mismatch between h, A, B and W")
    w_dtype = SLIMSPEC_F32 if W.dtype == torch.float32 else SLIMSPEC_BF16
    out_ids, out_logprobs = _outputs(rows, k, h.device, out_ids, out_logprobs)
    lib = load_library()
    shape = SlimspecShape(rows, d, r, V)
    workspace = _workspace(int(lib.routed_workspace_bytes(ctypes.byref(shape), k_route)), h.device, workspace)
    st = lib.routed_head_topk(_dev_ptr(h, "h"), _dev_ptr(A, "A"), _dev_ptr(B, "B"), _dev_ptr(W, "W"), w_dtype,
                              ctypes.byref(shape), k_route, k, _dev_ptr(out_ids, "out_ids"), _dev_ptr(out_logprobs, "out_logprobs"),
                              _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                              _stream_handle(stream))
    if st != STATUS_OK:
        _raise(st)
    return out_ids, out_logprobs


def routed_head_topk_prepared(h: torch.Tensor, A: torch.Tensor, B: torch.Tensor, Wt: torch.Tensor, k_route: int, k: int,
                              Bt: Optional[torch.Tensor] = None,
                              out_ids: Optional[torch.Tensor] = None, out_logprobs: Optional[torch.Tensor] = None,
                              workspace: Optional[torch.Tensor] = None,
                              stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """routed_head_topk with the token-major full head Wt [V, d] (and, optionally, the column-major copy Bt [V, r] of B)."""
    rows, d = h.shape
    d2, r = A.shape
    r2, V = B.shape
    if d != d2 or r != r2 or tuple(Wt.shape) != (V, d) or (Bt is not None and tuple(Bt.shape) != (V, r)):
        raise ValueError("shape mismatch between h, A, B, Wt and Bt")
    w_dtype = SLIMSPEC_F32 if Wt.dtype == torch.float32 else SLIMSPEC_BF16
    out_ids, out_logprobs = _outputs(rows, k, h.device, out_ids, out_logprobs)
    lib = load_library()
    shape = SlimspecShape(rows, d, r, V)
    workspace = _workspace(int(lib.routed_workspace_bytes(ctypes.byref(shape), k_route)), h.device, workspace)
    st = lib.routed_head_topk_prepared(_dev_ptr(h, "h"), _dev_ptr(A, "A"), _dev_ptr(B, "B"),
                                       _dev_ptr(Bt, "Bt") if Bt is not None else None, _dev_ptr(Wt, "Wt"), w_dtype,
                                       ctypes.byref(shape), k_route, k, _dev_ptr(out_ids, "out_ids"), _dev_ptr(out_logprobs, "out_logprobs"),
                                       _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                                       _stream_handle(stream))
    if st != STATUS_OK:
        _raise(st)
    return out_ids, out_logprobs
