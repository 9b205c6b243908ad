"""Thin Python binding of libcoral_lmhead.so (argument marshalling only).

Every step of the grouped / dense LM head (paper section 3.3 and the appendix on
the LM head router) runs in the HIP kernels behind the C ABI declared in
include/coral_lmhead.h.  PyTorch is used for device memory and the current
stream, nothing else.  There is no CPU fallback: if the built library is missing
the import of this package fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcoral_lmhead.so")

CORAL_OK = 0
CORAL_F32 = 0
CORAL_BF16 = 1
CORAL_F16 = 2


class CoralError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"coral_lmhead status {status}: {message}")
        self.status = status


class _GroupIndexStruct(ctypes.Structure):
    _fields_ = [("G", ctypes.c_int32),
                ("group_offsets_host", ctypes.c_void_p),
                ("group_offsets", ctypes.c_void_p),
                ("group_rows", ctypes.c_void_p)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
            "(there is no fallback path)")
    L = ctypes.CDLL(LIB_PATH)
    c = ctypes
    L.coral_status_string.restype = c.c_char_p
    L.coral_status_string.argtypes = [c.c_int]
    L.coral_group_index_validate.restype = c.c_int
    L.coral_group_index_validate.argtypes = [c.c_void_p, c.c_void_p, c.c_int, c.c_int]
    L.coral_lmhead_workspace_bytes.restype = c.c_size_t
    L.coral_lmhead_workspace_bytes.argtypes = [c.c_int] * 7
    L.coral_lmhead_path.restype = c.c_int
    L.coral_lmhead_path.argtypes = [c.c_int] * 8
    L.coral_lmhead_logprob_path.restype = c.c_int
    L.coral_lmhead_logprob_path.argtypes = [c.c_int] * 7
    L.coral_lmhead_workspace_init.restype = c.c_int
    L.coral_lmhead_workspace_init.argtypes = [c.c_void_p, c.c_size_t, c.c_void_p]
    L.coral_lmhead_grouped.restype = c.c_int
    L.coral_lmhead_grouped.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
                                       c.POINTER(_GroupIndexStruct)] + [c.c_int] * 6 + \
                                      [c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_size_t,
                                       c.c_void_p]
    L.coral_lmhead_grouped_noalloc.restype = c.c_int
    L.coral_lmhead_grouped_noalloc.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
                                               c.POINTER(_GroupIndexStruct)] + [c.c_int] * 6 + \
                                              [c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p]
    L.coral_lmhead_dense.restype = c.c_int
    L.coral_lmhead_dense.argtypes = [c.c_void_p, c.c_void_p] + [c.c_int] * 5 + \
                                    [c.c_void_p, c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
    L.coral_lmhead_grouped_profiled.restype = c.c_int
    L.coral_lmhead_grouped_profiled.argtypes = L.coral_lmhead_grouped.argtypes + [c.c_void_p] * 2
    L.coral_lmhead_grouped_logprob.restype = c.c_int
    L.coral_lmhead_grouped_logprob.argtypes = L.coral_lmhead_grouped.argtypes
    L.coral_lmhead_grouped_logprob_profiled.restype = c.c_int
    L.coral_lmhead_grouped_logprob_profiled.argtypes = L.coral_lmhead_grouped_profiled.argtypes
    L.coral_lmhead_dense_profiled.restype = c.c_int
    L.coral_lmhead_dense_profiled.argtypes = L.coral_lmhead_dense.argtypes + [c.c_void_p] * 2
    L.coral_probe_read.restype = c.c_int
    L.coral_probe_read.argtypes = [c.c_void_p, c.c_size_t, c.c_int, c.c_void_p, c.c_void_p, c.c_void_p]
    L.coral_router_premix.restype = c.c_int
    L.coral_router_premix.argtypes = [c.c_void_p, c.c_void_p, c.c_int, c.c_int, c.c_int, c.c_int,
                                      c.c_void_p, c.c_void_p]
    L.coral_tree_expand.restype = c.c_int
    L.coral_tree_expand.argtypes = [c.c_void_p] * 3 + [c.c_int] * 3 + [c.c_void_p] * 4
    L.coral_lmhead_draft_level.restype = c.c_int
    L.coral_lmhead_draft_level.argtypes = [c.c_void_p] * 5 + [c.POINTER(_GroupIndexStruct)] + \
                                          [c.c_int] * 6 + [c.c_void_p, c.c_int] + [c.c_void_p] * 7 + \
                                          [c.c_size_t, c.c_void_p]
    L.coral_lmhead_grouped_routed.restype = c.c_int
    L.coral_lmhead_grouped_routed.argtypes = [c.c_void_p] * 5 + [c.POINTER(_GroupIndexStruct)] + \
                                             [c.c_int] * 7 + [c.c_void_p] * 4 + \
                                             [c.c_size_t, c.c_void_p]
    return L


_L = _load()


def coral_status_string(status: int) -> str:
    return _L.coral_status_string(int(status)).decode()


def _raise(status: int):
    if status != CORAL_OK:
        raise CoralError(status, coral_status_string(status))


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return CORAL_BF16
    if t.dtype == torch.float16:
        return CORAL_F16
    if t.dtype == torch.float32:
        return CORAL_F32
    raise TypeError(f"hidden/gate_W/lm_W must be bfloat16, float16 or float32, got {t.dtype}")


def _dev_ptr(t: Optional[torch.Tensor], name: str, dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous (row-major, no padding)")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream_ptr(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def device_tensor(a: np.ndarray, storage: str, device="cuda") -> torch.Tensor:
    """Upload a host array; storage 'bf16' and 'f16' take uint16 bit patterns, 'f32' float32."""
    if storage in ("bf16", "f16"):
        if a.dtype != np.uint16:
            raise TypeError(f"{storage} storage expects uint16 bit patterns")
        return torch.from_numpy(a.view(np.int16)).to(device).view(
            torch.bfloat16 if storage == "bf16" else torch.float16)
    if storage == "f32":
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
    raise ValueError(f"unknown storage {storage!r}")


class GroupIndex:
    """CSR partition of the vocabulary into groups: host offsets + device copies."""

    def __init__(self, group_offsets: np.ndarray, group_rows, device="cuda", validate=True):
        self.offsets_host = np.ascontiguousarray(group_offsets, dtype=np.int32)
        self.G = int(self.offsets_host.size - 1)
        if isinstance(group_rows, torch.Tensor):
            if validate:
                raise ValueError("validation needs the rows on the host; pass a numpy array")
            self.rows = group_rows
        else:
            rows_host = np.ascontiguousarray(group_rows, dtype=np.int32)
            if validate:
                group_index_validate(self.offsets_host, rows_host)
            self.rows = torch.from_numpy(rows_host).to(device)
        self.V = int(self.rows.numel())
        self.offsets = torch.from_numpy(self.offsets_host).to(device)
        self._struct = _GroupIndexStruct(self.G, self.offsets_host.ctypes.data,
                                         _dev_ptr(self.offsets, "group_offsets", torch.int32),
                                         _dev_ptr(self.rows, "group_rows", torch.int32))

    def struct(self):
        return ctypes.byref(self._struct)


def group_index_validate(group_offsets: np.ndarray, group_rows: np.ndarray) -> None:
    off = np.ascontiguousarray(group_offsets, dtype=np.int32)
    rows = np.ascontiguousarray(group_rows, dtype=np.int32)
    _raise(_L.coral_group_index_validate(off.ctypes.data, rows.ctypes.data, off.size - 1, rows.size))


def coral_lmhead_workspace_bytes(M: int, H: int, V: int, G: int, g: int, k: int, dt: int) -> int:
    return int(_L.coral_lmhead_workspace_bytes(M, H, V, G, g, k, dt))


PATH_NAMES = {0: "staged", 1: "single-launch", 2: "tiles", -1: "unsupported"}


def coral_lmhead_path(dense: bool, M: int, H: int, V: int, G: int, g: int, k: int, dt: int) -> int:
    return int(_L.coral_lmhead_path(1 if dense else 0, M, H, V, G, g, k, dt))


def coral_lmhead_logprob_path(M: int, H: int, V: int, G: int, g: int, k: int, dt: int) -> int:
    return int(_L.coral_lmhead_logprob_path(M, H, V, G, g, k, dt))


def coral_lmhead_workspace_init(workspace: torch.Tensor, stream=None) -> None:
    _raise(_L.coral_lmhead_workspace_init(_dev_ptr(workspace, "workspace"),
                                          workspace.numel() * workspace.element_size(),
                                          _stream_ptr(stream)))


def alloc_workspace(M, H, V, G, g, k, dt, device="cuda", stream=None) -> torch.Tensor:
    """A prepared workspace (allocated through PyTorch, control words zeroed on `stream`, the
    stream the head will be enqueued on; None = the current stream)."""
    n = coral_lmhead_workspace_bytes(M, H, V, G, g, k, dt)
    if n == 0:
        raise ValueError("invalid sizes for the workspace")
    ws = torch.empty(n, dtype=torch.uint8, device=device)
    coral_lmhead_workspace_init(ws, stream)
    if stream is not None:
        ws.record_stream(stream)       # the caching allocator must not reuse it under that stream
    return ws


def _marshal_grouped(hidden, gate_W, gate_bias, lm_W, gi, g, k, topk_ids, topk_logits, sel_groups,
                     workspace, stream, events, logprob, gate_hidden, level):
    """Checks and marshals the arguments of the grouped entry points once: returns the entry
    point, its arguments up to (not including) the stream, those behind the stream, and the
    output tensors."""
    dt = _dtype_code(hidden)
    if gate_W.dtype != hidden.dtype or lm_W.dtype != hidden.dtype:
        raise TypeError("hidden, gate_W and lm_W must share one dtype")
    if hidden.dim() != 2 or gate_W.dim() != 2 or lm_W.dim() != 2:
        raise ValueError("hidden, gate_W and lm_W must be 2-D")
    M, H = hidden.shape
    V = lm_W.shape[0]
    if lm_W.shape[1] != H or gate_W.shape != (gi.G, H) or gi.V != V:
        raise ValueError("inconsistent shapes")
    if gate_bias is not None and gate_bias.shape != (gi.G,):
        raise ValueError("gate_bias must be [G]")
    dev = hidden.device
    if topk_ids is None:
        topk_ids = torch.empty((M, k), dtype=torch.int32, device=dev)
    if topk_logits is None:
        topk_logits = torch.empty((M, k), dtype=torch.float32, device=dev)
    if sel_groups is None:
        sel_groups = torch.empty((M, g), dtype=torch.int32, device=dev)
    if topk_ids.shape != (M, k) or topk_logits.shape != (M, k) or sel_groups.shape != (M, g):
        raise ValueError("output shapes must be [M,k], [M,k], [M,g]")
    if workspace is None:
        workspace = alloc_workspace(M, H, V, gi.G, g, k, dt, dev, stream)
    args = (_dev_ptr(hidden, "hidden"), _dev_ptr(gate_W, "gate_W"),
            _dev_ptr(gate_bias, "gate_bias", torch.float32), _dev_ptr(lm_W, "lm_W"), gi.struct(),
            M, H, V, g, k, dt, _dev_ptr(topk_ids, "topk_ids", torch.int32),
            _dev_ptr(topk_logits, "topk_logits", torch.float32),
            _dev_ptr(sel_groups, "sel_groups", torch.int32), _dev_ptr(workspace, "workspace"),
            workspace.numel() * workspace.element_size())
    if gate_hidden is not None and (gate_hidden.dtype != hidden.dtype or gate_hidden.shape != hidden.shape):
        raise ValueError("gate_hidden must match hidden in dtype and shape")
    behind = ()
    if level is not None:
        if events is not None:
            raise ValueError("the draft-level entry point has no measurement variant")
        parent_score, n_next, next_parent, next_token, next_score = level
        fn = _L.coral_lmhead_draft_level
        args = (args[0], _dev_ptr(gate_hidden, "gate_hidden"), *args[1:11],
                _dev_ptr(parent_score, "parent_score", torch.float32), int(n_next), *args[11:14],
                _dev_ptr(next_parent, "next_parent", torch.int32),
                _dev_ptr(next_token, "next_token", torch.int32),
                _dev_ptr(next_score, "next_score", torch.float32), *args[14:])
    elif gate_hidden is not None:
        if events is not None:
            raise ValueError("the routed entry point has no measurement variant")
        fn = _L.coral_lmhead_grouped_routed
        args = (args[0], _dev_ptr(gate_hidden, "gate_hidden"), *args[1:11], 1 if logprob else 0, *args[11:])
    elif events is None:
        fn = _L.coral_lmhead_grouped_logprob if logprob else _L.coral_lmhead_grouped
    else:
        fn = _L.coral_lmhead_grouped_logprob_profiled if logprob else _L.coral_lmhead_grouped_profiled
        behind = (events[0], events[1])
    keep = (hidden, gate_W, gate_bias, lm_W, gi, workspace, gate_hidden, level)
    return fn, args, behind, (topk_ids, topk_logits, sel_groups), keep


def coral_lmhead_grouped(hidden: torch.Tensor, gate_W: torch.Tensor,
                         gate_bias: Optional[torch.Tensor], lm_W: torch.Tensor, gi: GroupIndex,
                         g: int, k: int, topk_ids: Optional[torch.Tensor] = None,
                         topk_logits: Optional[torch.Tensor] = None,
                         sel_groups: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None, stream=None, events=None,
                         logprob: bool = False, gate_hidden: Optional[torch.Tensor] = None,
                         level=None) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """events: optional (hipEvent_t, hipEvent_t) raw handles; selects the _profiled entry.
    logprob: call coral_lmhead_grouped_logprob (the second result then holds log p(x)).
    gate_hidden: call coral_lmhead_grouped_routed (the router sees this [M,H] tensor).
    level: (parent_score or None, n_next, next_parent, next_token, next_score): call
    coral_lmhead_draft_level (see coral_lmhead_draft_level below)."""
    fn, args, behind, out, _ = _marshal_grouped(hidden, gate_W, gate_bias, lm_W, gi, g, k, topk_ids,
                                                topk_logits, sel_groups, workspace, stream, events,
                                                logprob, gate_hidden, level)
    _raise(fn(*args, _stream_ptr(stream), *behind))
    return out


class PreparedGrouped:
    """A grouped-head call whose arguments are checked and marshalled once, for loops that
    issue the same call many times (a draft loop, a benchmark): calling the object only looks
    the stream up and enters the library.  Takes coral_lmhead_grouped's arguments (a workspace
    is required: the call must not allocate); .out holds the output tensors.  The tensors are
    kept alive by the object and must not be resized or freed while it is in use."""

    def __init__(self, hidden, gate_W, gate_bias, lm_W, gi, g, k, workspace, topk_ids=None,
                 topk_logits=None, sel_groups=None, logprob=False, gate_hidden=None, level=None):
        if workspace is None:
            raise ValueError("a prepared call needs its workspace")
        self._fn, self._args, _, self.out, self._keep = _marshal_grouped(
            hidden, gate_W, gate_bias, lm_W, gi, g, k, topk_ids, topk_logits, sel_groups, workspace,
            None, None, logprob, gate_hidden, level)

    def __call__(self, stream=None):
        st = self._fn(*self._args, _stream_ptr(stream))
        if st:
            _raise(st)
        return self.out


NOALLOC_SCRATCH_BYTES = 8 << 20      # CORAL_NOALLOC_SCRATCH_BYTES of the header


def coral_lmhead_grouped_noalloc(hidden: torch.Tensor, gate_W: torch.Tensor,
                                 gate_bias: Optional[torch.Tensor], lm_W: torch.Tensor, gi: GroupIndex,
                                 g: int, k: int, topk_ids: torch.Tensor, topk_logits: torch.Tensor,
                                 sel_groups: Optional[torch.Tensor] = None, stream=None) -> None:
    """coral_lmhead_grouped_noalloc of the C ABI: the grouped head on the library's static
    scratch.  Nothing is allocated here either: the caller passes every output tensor."""
    dt = _dtype_code(hidden)
    if gate_W.dtype != hidden.dtype or lm_W.dtype != hidden.dtype:
        raise TypeError("hidden, gate_W and lm_W must share one dtype")
    if hidden.dim() != 2 or gate_W.dim() != 2 or lm_W.dim() != 2:
        raise ValueError("hidden, gate_W and lm_W must be 2-D")
    M, H = hidden.shape
    V = lm_W.shape[0]
    if lm_W.shape[1] != H or gate_W.shape != (gi.G, H) or gi.V != V:
        raise ValueError("inconsistent shapes")
    if gate_bias is not None and gate_bias.shape != (gi.G,):
        raise ValueError("gate_bias must be [G]")
    if topk_ids.shape != (M, k) or topk_logits.shape != (M, k) or \
            (sel_groups is not None and sel_groups.shape != (M, g)):
        raise ValueError("output shapes must be [M,k], [M,k], [M,g]")
    _raise(_L.coral_lmhead_grouped_noalloc(
        _dev_ptr(hidden, "hidden"), _dev_ptr(gate_W, "gate_W"),
        _dev_ptr(gate_bias, "gate_bias", torch.float32), _dev_ptr(lm_W, "lm_W"), gi.struct(),
        M, H, V, g, k, dt, _dev_ptr(topk_ids, "topk_ids", torch.int32),
        _dev_ptr(topk_logits, "topk_logits", torch.float32),
        _dev_ptr(sel_groups, "sel_groups", torch.int32), _stream_ptr(stream)))


def coral_probe_read(src: torch.Tensor, nbytes: int, waves: int, events, stream=None) -> None:
    """coral_probe_read of the C ABI: a kernel that only reads the first nbytes of src."""
    if not src.is_cuda or not src.is_contiguous() or src.numel() * src.element_size() < nbytes:
        raise ValueError("src must be a contiguous device tensor of at least nbytes bytes")
    _raise(_L.coral_probe_read(src.data_ptr(), int(nbytes), int(waves), _stream_ptr(stream),
                               events[0], events[1]))


ACTIVATIONS = {"silu": 0, "relu": 1, "identity": 2}


def coral_router_premix(hidden: torch.Tensor, W1: torch.Tensor, act: str = "silu",
                        out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """coral_router_premix of the C ABI: u = act(W1 hidden) + hidden, [M,H] in hidden's dtype."""
    dt = _dtype_code(hidden)
    if W1.dtype != hidden.dtype:
        raise TypeError("hidden and W1 must share one dtype")
    if hidden.dim() != 2 or W1.shape != (hidden.shape[1], hidden.shape[1]):
        raise ValueError("W1 must be [H,H]")
    if act not in ACTIVATIONS:
        raise ValueError(f"unknown activation {act!r}")
    M, H = hidden.shape
    if out is None:
        out = torch.empty_like(hidden)
    if out.shape != hidden.shape or out.dtype != hidden.dtype:
        raise ValueError("out must match hidden")
    _raise(_L.coral_router_premix(_dev_ptr(hidden, "hidden"), _dev_ptr(W1, "W1"), M, H, dt,
                                  ACTIVATIONS[act], _dev_ptr(out, "out"), _stream_ptr(stream)))
    return out


def coral_tree_expand(parent_score: Optional[torch.Tensor], cand_ids: torch.Tensor,
                      cand_logp: torch.Tensor, n_next: int, stream=None
                      ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """coral_tree_expand of the C ABI: (parent index, token id, cumulative score), each [n_next]."""
    if cand_ids.dim() != 2 or cand_logp.shape != cand_ids.shape:
        raise ValueError("cand_ids and cand_logp must both be [M,k]")
    M, k = cand_ids.shape
    if parent_score is not None and parent_score.shape != (M,):
        raise ValueError("parent_score must be [M]")
    dev = cand_ids.device
    parent = torch.empty(n_next, dtype=torch.int32, device=dev)
    token = torch.empty(n_next, dtype=torch.int32, device=dev)
    score = torch.empty(n_next, dtype=torch.float32, device=dev)
    _raise(_L.coral_tree_expand(_dev_ptr(parent_score, "parent_score", torch.float32),
                                _dev_ptr(cand_ids, "cand_ids", torch.int32),
                                _dev_ptr(cand_logp, "cand_logp", torch.float32), M, k, int(n_next),
                                _dev_ptr(parent, "next_parent"), _dev_ptr(token, "next_token"),
                                _dev_ptr(score, "next_score"), _stream_ptr(stream)))
    return parent, token, score


def coral_lmhead_draft_level(hidden, gate_W, gate_bias, lm_W, gi, g, k, n_next: int,
                             parent_score: Optional[torch.Tensor] = None,
                             next_parent: Optional[torch.Tensor] = None,
                             next_token: Optional[torch.Tensor] = None,
                             next_score: Optional[torch.Tensor] = None, **kw):
    """coral_lmhead_draft_level of the C ABI: the log-probability head for the M nodes of a tree
    level and the level's expansion.  Returns (ids, log-probabilities, selected groups,
    parent index, token id, cumulative score), the last three [n_next]."""
    M = hidden.shape[0]
    dev = hidden.device
    if parent_score is not None and parent_score.shape != (M,):
        raise ValueError("parent_score must be [M]")
    if next_parent is None:
        next_parent = torch.empty(n_next, dtype=torch.int32, device=dev)
    if next_token is None:
        next_token = torch.empty(n_next, dtype=torch.int32, device=dev)
    if next_score is None:
        next_score = torch.empty(n_next, dtype=torch.float32, device=dev)
    if next_parent.shape != (n_next,) or next_token.shape != (n_next,) or next_score.shape != (n_next,):
        raise ValueError("next_parent, next_token and next_score must be [n_next]")
    ids, logp, sel = coral_lmhead_grouped(hidden, gate_W, gate_bias, lm_W, gi, g, k, logprob=True,
                                          level=(parent_score, n_next, next_parent, next_token, next_score),
                                          **kw)
    return ids, logp, sel, next_parent, next_token, next_score


def coral_lmhead_grouped_logprob(hidden, gate_W, gate_bias, lm_W, gi, g, k, **kw):
    """coral_lmhead_grouped_logprob of the C ABI: (ids, log-probabilities, selected groups)."""
    return coral_lmhead_grouped(hidden, gate_W, gate_bias, lm_W, gi, g, k, logprob=True, **kw)


def coral_lmhead_dense(hidden: torch.Tensor, lm_W: torch.Tensor, k: int,
                       topk_ids: Optional[torch.Tensor] = None,
                       topk_logits: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None, stream=None, events=None
                       ) -> Tuple[torch.Tensor, torch.Tensor]:
    dt = _dtype_code(hidden)
    if lm_W.dtype != hidden.dtype:
        raise TypeError("hidden and lm_W must share one dtype")
    if hidden.dim() != 2 or lm_W.dim() != 2 or lm_W.shape[1] != hidden.shape[1]:
        raise ValueError("inconsistent shapes")
    M, H = hidden.shape
    V = lm_W.shape[0]
    dev = hidden.device
    if topk_ids is None:
        topk_ids = torch.empty((M, k), dtype=torch.int32, device=dev)
    if topk_logits is None:
        topk_logits = torch.empty((M, k), dtype=torch.float32, device=dev)
    if topk_ids.shape != (M, k) or topk_logits.shape != (M, k):
        raise ValueError("output shapes must be [M,k]")
    if workspace is None:
        workspace = alloc_workspace(M, H, V, 0, 0, k, dt, dev, stream)
    args = (_dev_ptr(hidden, "hidden"), _dev_ptr(lm_W, "lm_W"), M, H, V, k, dt,
            _dev_ptr(topk_ids, "topk_ids", torch.int32),
            _dev_ptr(topk_logits, "topk_logits", torch.float32), _dev_ptr(workspace, "workspace"),
            workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    if events is None:
        st = _L.coral_lmhead_dense(*args)
    else:
        st = _L.coral_lmhead_dense_profiled(*args, events[0], events[1])
    _raise(st)
    return topk_ids, topk_logits
