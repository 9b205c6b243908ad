"""TEST INFRASTRUCTURE -- ctypes front end of the fp64 CPU oracle.

Only tests, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg may
import this package.  It never imports the HIP package and shares no code with
it.  The arithmetic lives in ``coral_oracle.c`` (paper section 3.3 and the
appendix on the LM head router); this file marshals numpy arrays only.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "coral_oracle.c")
_LIB = os.path.join(_HERE, "libcoral_oracle.so")

_DT = {"f32": 0, "bf16": 1, "f16": 2}


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over vocabulary rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
               "-fno-fast-math", "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        c = ctypes
        vp, ip, dp, fp = c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p
        L.coral_oracle_max_threads.restype = c.c_int
        L.coral_oracle_set_threads.argtypes = [c.c_int]
        L.coral_oracle_check_partition.argtypes = [ip, ip, c.c_int, c.c_int]
        L.coral_oracle_gate.argtypes = [vp, vp, fp, c.c_int, c.c_int, c.c_int, c.c_int, dp]
        L.coral_oracle_rank_groups.argtypes = [dp, c.c_int, c.c_int, ip]
        L.coral_oracle_logits_rows.argtypes = [vp, vp, c.c_int, c.c_int, ip, c.c_int64,
                                               c.c_int, dp]
        L.coral_oracle_top_k.argtypes = [dp, ip, c.c_int64, c.c_int, ip, dp, dp]
        L.coral_oracle_grouped.argtypes = [vp, vp, fp, vp, ip, ip] + [c.c_int] * 7 + \
                                          [ip, dp, ip, ip, dp, dp, dp, dp]
        L.coral_oracle_dense.argtypes = [vp, vp] + [c.c_int] * 5 + [ip, dp, dp]
        _lib = L
    return _lib


class OracleError(RuntimeError):
    pass


def _check(rc: int, what: str):
    if rc != 0:
        raise OracleError(f"{what}: oracle status {rc}")


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def _storage(a: np.ndarray, dtype: str) -> np.ndarray:
    want = np.float32 if dtype == "f32" else np.uint16
    if a.dtype != want:
        raise TypeError(f"expected {want} storage for dtype {dtype}, got {a.dtype}")
    return np.ascontiguousarray(a)


def max_threads() -> int:
    return int(lib().coral_oracle_max_threads())


def set_threads(n: int) -> None:
    lib().coral_oracle_set_threads(int(n))


def check_partition(offsets: np.ndarray, rows: np.ndarray, V: int) -> int:
    offsets = np.ascontiguousarray(offsets, dtype=np.int32)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    if rows.size != V:
        return -2
    return int(lib().coral_oracle_check_partition(offsets.ctypes.data, rows.ctypes.data,
                                                  offsets.size - 1, V))


def gate(hidden, gate_W, gate_bias, dtype: str) -> np.ndarray:
    hidden = _storage(hidden, dtype)
    gate_W = _storage(gate_W, dtype)
    M, H = hidden.shape
    G = gate_W.shape[0]
    assert gate_W.shape[1] == H
    if gate_bias is not None:
        gate_bias = np.ascontiguousarray(gate_bias, dtype=np.float32)
        assert gate_bias.shape == (G,)
    s = np.empty((M, G), dtype=np.float64)
    _check(lib().coral_oracle_gate(hidden.ctypes.data, gate_W.ctypes.data, _p(gate_bias),
                                   M, H, G, _DT[dtype], s.ctypes.data), "gate")
    return s


def rank_groups(s: np.ndarray) -> np.ndarray:
    s = np.ascontiguousarray(s, dtype=np.float64)
    M, G = s.shape
    order = np.empty((M, G), dtype=np.int32)
    _check(lib().coral_oracle_rank_groups(s.ctypes.data, M, G, order.ctypes.data), "rank_groups")
    return order


def logits_rows(hidden_row, lm_W, rows, dtype: str) -> np.ndarray:
    """fp64 logits of one token for the listed vocabulary rows."""
    hidden_row = _storage(hidden_row, dtype).reshape(-1)
    lm_W = _storage(lm_W, dtype)
    V, H = lm_W.shape
    assert hidden_row.size == H
    rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1)
    z = np.empty(rows.size, dtype=np.float64)
    _check(lib().coral_oracle_logits_rows(hidden_row.ctypes.data, lm_W.ctypes.data, H, V,
                                          rows.ctypes.data, rows.size, _DT[dtype],
                                          z.ctypes.data), "logits_rows")
    return z


def top_k(z, ids, k: int):
    z = np.ascontiguousarray(z, dtype=np.float64).reshape(-1)
    ids = np.ascontiguousarray(ids, dtype=np.int32).reshape(-1)
    assert z.size == ids.size
    out_ids = np.empty(k, dtype=np.int32)
    out_z = np.empty(k, dtype=np.float64)
    nxt = np.empty(1, dtype=np.float64)
    _check(lib().coral_oracle_top_k(z.ctypes.data, ids.ctypes.data, z.size, k,
                                    out_ids.ctypes.data, out_z.ctypes.data,
                                    nxt.ctypes.data), "top_k")
    return out_ids, out_z, float(nxt[0])


@dataclass
class GroupedResult:
    s: np.ndarray            # [M,G] gate scores
    sel: np.ndarray          # [M,g] selected groups, rank order
    topk_ids: np.ndarray     # [M,k]
    topk_z: np.ndarray       # [M,k] fp64 logits
    next_z: np.ndarray       # [M] logit ranked k+1 (-inf if none)
    lse: np.ndarray          # [M,g]
    logp_router: np.ndarray  # [M,G]


ACTIVATIONS = ("silu", "relu", "identity")


def widen(a: np.ndarray, dtype: str) -> np.ndarray:
    """Stored values as float64 (bf16 = the upper 16 bits of a float32)."""
    a = _storage(a, dtype)
    if dtype == "f32":
        return a.astype(np.float64)
    if dtype == "f16":
        return a.view(np.float16).astype(np.float64)
    return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """float64 -> float32 (nearest even) and, for bf16, on to the nearest bf16 (ties to
    even) of that float32, which is the order in which a kernel that accumulates in
    float32 rounds its result."""
    f = np.ascontiguousarray(x, dtype=np.float64).astype(np.float32)
    if dtype == "f32":
        return f
    if dtype == "f16":
        return f.astype(np.float16).view(np.uint16)
    b = f.view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    r = np.where(np.isnan(f), np.uint32(0x7FC0), r)
    return r.astype(np.uint16)


def premix(hidden, W1, dtype: str, act: str = "silu"):
    """The router's inner term of Eq. 7: u = act(W1 h) + h per token, W1 [d,d] with one
    row per output feature.  The paper does not name act; "silu" is this build's reading.
    Returns (u as float64, u rounded to the storage type)."""
    if act not in ACTIVATIONS:
        raise ValueError(f"unknown activation {act!r}")
    h = widen(hidden, dtype)
    w = widen(W1, dtype)
    M, H = h.shape
    assert w.shape == (H, H)
    y = h @ w.T                                   # y[m,i] = sum_j W1[i,j] h[m,j]
    if act == "silu":
        a = y / (1.0 + np.exp(-y))
    elif act == "relu":
        a = np.maximum(y, 0.0)
    else:
        a = y
    u = a + h
    return u, round_to_storage(u, dtype)


def grouped(hidden, gate_W, gate_bias, lm_W, offsets, rows, g: int, k: int, dtype: str,
            forced_sel=None, gate_hidden=None) -> GroupedResult:
    """gate_hidden: the vector the router's W2 projection sees (Eq. 7: u = act(W1 h) + h)
    when it differs from the vector the LM head sees; scores, selection and log p_router
    then come from gate_hidden, logits from hidden."""
    if gate_hidden is not None:
        s = gate(gate_hidden, gate_W, gate_bias, dtype)
        sel = rank_groups(s)[:, :g] if forced_sel is None else forced_sel
        r = grouped(hidden, gate_W, gate_bias, lm_W, offsets, rows, g, k, dtype, forced_sel=sel)
        mx = s.max(axis=1, keepdims=True)
        lse_s = mx + np.log(np.exp(s - mx).sum(axis=1, keepdims=True))
        return GroupedResult(s, r.sel, r.topk_ids, r.topk_z, r.next_z, r.lse, s - lse_s)
    hidden = _storage(hidden, dtype)
    gate_W = _storage(gate_W, dtype)
    lm_W = _storage(lm_W, dtype)
    M, H = hidden.shape
    V = lm_W.shape[0]
    G = gate_W.shape[0]
    assert lm_W.shape[1] == H and gate_W.shape[1] == H
    offsets = np.ascontiguousarray(offsets, dtype=np.int32)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    assert offsets.size == G + 1 and rows.size == V
    if gate_bias is not None:
        gate_bias = np.ascontiguousarray(gate_bias, dtype=np.float32)
    if forced_sel is not None:
        forced_sel = np.ascontiguousarray(forced_sel, dtype=np.int32)
        assert forced_sel.shape == (M, g)
    r = GroupedResult(np.empty((M, G)), np.empty((M, g), np.int32), np.empty((M, k), np.int32),
                      np.empty((M, k)), np.empty(M), np.empty((M, g)), np.empty((M, G)))
    _check(lib().coral_oracle_grouped(
        hidden.ctypes.data, gate_W.ctypes.data, _p(gate_bias), lm_W.ctypes.data,
        offsets.ctypes.data, rows.ctypes.data, M, H, V, G, g, k, _DT[dtype], _p(forced_sel),
        r.s.ctypes.data, r.sel.ctypes.data, r.topk_ids.ctypes.data, r.topk_z.ctypes.data,
        r.next_z.ctypes.data, r.lse.ctypes.data, r.logp_router.ctypes.data), "grouped")
    return r


@dataclass
class DenseResult:
    topk_ids: np.ndarray
    topk_z: np.ndarray
    next_z: np.ndarray


def dense(hidden, lm_W, k: int, dtype: str) -> DenseResult:
    hidden = _storage(hidden, dtype)
    lm_W = _storage(lm_W, dtype)
    M, H = hidden.shape
    V = lm_W.shape[0]
    assert lm_W.shape[1] == H
    r = DenseResult(np.empty((M, k), np.int32), np.empty((M, k)), np.empty(M))
    _check(lib().coral_oracle_dense(hidden.ctypes.data, lm_W.ctypes.data, M, H, V, k,
                                    _DT[dtype], r.topk_ids.ctypes.data, r.topk_z.ctypes.data,
                                    r.next_z.ctypes.data), "dense")
    return r


@dataclass
class LogprobResult:
    sel: np.ndarray          # [M,g] selected groups, rank order
    topk_ids: np.ndarray     # [M,k]
    topk_logp: np.ndarray    # [M,k] fp64 log p(x), descending
    next_logp: np.ndarray    # [M] log p ranked k+1 (-inf if none)
    s: np.ndarray            # [M,G] gate scores
    lse: np.ndarray          # [M,g] log-sum-exp of the logits inside each selected group
    logp_router: np.ndarray  # [M,G]


def grouped_logprob(hidden, gate_W, gate_bias, lm_W, offsets, rows, g: int, k: int, dtype: str,
                    forced_sel=None, gate_hidden=None) -> LogprobResult:
    """Eq. 8 as written: for every row x of a selected group n of token m,
    log p(x) = log p_router(n) + z[x] - lse_n, p_router the softmax of the gate scores over
    all G groups (Eq. 7), lse_n the log-sum-exp of the logits of group n's rows; the k largest
    log p(x) per token, best first, equal values by ascending id.  Gate, selection, logits,
    lse_n and log p_router come from the C oracle; the composition is the line below."""
    base = grouped(hidden, gate_W, gate_bias, lm_W, offsets, rows, g, k, dtype, forced_sel,
                   gate_hidden)
    offsets = np.asarray(offsets)
    rows = np.asarray(rows)
    M = np.asarray(hidden).shape[0]
    ids_out = np.empty((M, k), np.int32)
    lp_out = np.empty((M, k))
    nxt = np.empty(M)
    for m in range(M):
        all_ids, all_lp = [], []
        for j in range(g):
            n = int(base.sel[m, j])
            r = rows[offsets[n]:offsets[n + 1]]
            z = logits_rows(np.asarray(hidden)[m], lm_W, r, dtype)
            all_ids.append(r)
            all_lp.append(base.logp_router[m, n] + z - base.lse[m, j])
        ids_out[m], lp_out[m], nxt[m] = top_k(np.concatenate(all_lp), np.concatenate(all_ids), k)
    return LogprobResult(base.sel, ids_out, lp_out, nxt, base.s, base.lse, base.logp_router)



def tree_expand(parent_score, cand_ids, cand_logp, n_next: int):
    """One level of draft-tree expansion (the dynamic tree the paper drafts with, section 2.1
    and section 4.1 "Implementation": several candidates per node, a fixed number of nodes
    kept per level).  Node m of the current level carries the cumulative log-probability
    parent_score[m]; its k candidates have log-probabilities cand_logp[m,:] and token ids
    cand_ids[m,:] (id < 0: empty slot).  The score of candidate (m,i) is the float32 sum
    parent_score[m] + cand_logp[m,i] (both sides of a parity check add in float32, so the
    ranking is exact integer work); the n_next best scores become the next level, best
    first, equal scores by lower m, then lower i.  Returns (parent [n_next] int32,
    token [n_next] int32, score [n_next] float32); slots beyond the number of candidates
    hold (-1, -1, -inf)."""
    cand_ids = np.ascontiguousarray(cand_ids, dtype=np.int32)
    cand_logp = np.ascontiguousarray(cand_logp, dtype=np.float32)
    M, k = cand_ids.shape
    assert cand_logp.shape == (M, k)
    base = np.zeros(M, np.float32) if parent_score is None else np.ascontiguousarray(parent_score, dtype=np.float32)
    assert base.shape == (M,)
    score = (base[:, None] + cand_logp).astype(np.float32)
    items = [(-float(score[m, i]), m, i) for m in range(M) for i in range(k) if cand_ids[m, i] >= 0]
    items.sort()
    parent = np.full(n_next, -1, np.int32)
    token = np.full(n_next, -1, np.int32)
    out = np.full(n_next, -np.inf, np.float32)
    for r, (_, m, i) in enumerate(items[:n_next]):
        parent[r], token[r], out[r] = m, cand_ids[m, i], score[m, i]
    return parent, token, out
