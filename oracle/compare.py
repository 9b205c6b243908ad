"""TEST INFRASTRUCTURE -- tolerance-aware agreement check against the oracle.

The grouped head is an exactly defined computation, so a device result must
reproduce the oracle's groups and candidate ids bit for bit wherever the
oracle's neighbouring values are further apart than the float tolerance, and
may differ only inside such near-ties.  Rules checked per token (tol is the
logit tolerance, gate_tol the gate-score tolerance):

  groups   position i of the device's selection holds a group whose oracle
           score is within gate_tol of the oracle's i-th best score; the groups
           are distinct.  If the device's groups differ from the oracle's, the
           oracle is re-run with the device's groups forced, and the candidate
           rules below are checked against that run.
  (i)      every returned id has oracle logit >= z_k - tol (z_k: oracle's k-th)
  (ii)     every id with oracle logit > z_k + tol is returned
  (iii)    |device logit - oracle logit of the same id| <= tol
  (iv)     device logits are non-increasing; bitwise-equal device logits are in
           ascending id order; any inversion against the oracle's order is
           between ids whose oracle logits differ by < tol
  (v)      ids are distinct and belong to the token's selected groups
  exact    if every adjacent gap among the oracle's top k+1 logits exceeds
           2*tol, the id list must equal the oracle's exactly
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

from . import dense as oracle_dense
from . import grouped as oracle_grouped
from . import grouped_logprob as oracle_grouped_logprob
from . import logits_rows, rank_groups
from . import premix as oracle_premix
from . import widen

# f16 (the paper's storage type): products of two 11-bit significands are exact in float32
# as bf16's are, and the sums are the same float32 sums, so it takes bf16's tolerances.
TOL = {"bf16": 2e-3, "f16": 2e-3, "f32": 1e-5}
GATE_TOL = {"bf16": 1e-4, "f16": 1e-4, "f32": 1e-6}
# log p(x) = log p_router + z - lse: the logit's tolerance, the same again for lse (a
# log-sum-exp moves by at most the largest error of its terms) and twice the gate's for the
# router's log-softmax (score and its log-sum-exp).
LOGP_TOL = {d: 2 * TOL[d] + 2 * GATE_TOL[d] for d in TOL}


# The pre-mix u = act(W1 h) + h is stored in the head's storage type.  A kernel that
# accumulates in float32 lands within PREMIX_ABS of the exact value before it rounds, and
# rounding to storage moves it by at most half a unit in the last place of the result.
PREMIX_ABS = {"bf16": 2e-5, "f16": 2e-5, "f32": 1e-5}


@dataclass
class Report:
    tokens: int = 0
    exact_tokens: int = 0          # tokens held to bit-exact ids
    forced_tokens: int = 0         # tokens whose groups differed inside a near-tie
    max_abs_err: float = 0.0
    notes: list = field(default_factory=list)


def _check_topk_token(m, dev_ids, dev_z, ref_ids, ref_z, next_z, oz_dev, tol, rep,
                      member=None):
    k = len(ref_ids)
    zk = ref_z[k - 1]
    assert len(dev_ids) == k
    assert len(set(dev_ids.tolist())) == k, f"token {m}: duplicate ids {dev_ids}"
    if member is not None:
        assert member(dev_ids).all(), f"token {m}: id outside the selected groups {dev_ids}"
    assert np.all(np.isfinite(dev_z)), f"token {m}: non-finite logit {dev_z}"
    # (i)
    assert np.all(oz_dev >= zk - tol), \
        f"token {m}: returned id below the k-th logit by more than tol: {oz_dev} vs {zk}"
    # (ii)
    must = ref_ids[ref_z > zk + tol]
    missing = np.setdiff1d(must, dev_ids)
    assert missing.size == 0, f"token {m}: ids clearly inside the top-k missing: {missing}"
    # (iii)
    err = np.abs(dev_z.astype(np.float64) - oz_dev)
    rep.max_abs_err = max(rep.max_abs_err, float(err.max()))
    assert np.all(err <= tol), f"token {m}: logit error {err.max()} > {tol}"
    # (iv)
    d = np.diff(dev_z.astype(np.float64))
    assert np.all(d <= 0), f"token {m}: logits not descending {dev_z}"
    eq = np.nonzero(d == 0)[0]
    for i in eq:
        assert dev_ids[i] < dev_ids[i + 1], f"token {m}: equal logits not in id order"
    for i in range(k):
        for j in range(i + 1, k):
            assert oz_dev[i] > oz_dev[j] - tol or (oz_dev[i] == oz_dev[j]), \
                f"token {m}: order inversion beyond tol at ranks {i},{j}"
    # exact
    chain = np.concatenate([ref_z, [next_z]])
    if np.all(-np.diff(chain) > 2 * tol):
        assert np.array_equal(dev_ids, ref_ids), \
            f"token {m}: ids differ with no near-tie: {dev_ids} vs {ref_ids}"
        rep.exact_tokens += 1
    rep.tokens += 1


def check_grouped(hidden, gate_W, gate_bias, lm_W, offsets, rows, g, k, dtype,
                  dev_ids, dev_logits, dev_sel, tol=None, gate_tol=None, gate_hidden=None) -> Report:
    """gate_hidden: the router's input where it differs from the LM head's (Eq. 7)."""
    tol = TOL[dtype] if tol is None else tol
    gate_tol = GATE_TOL[dtype] if gate_tol is None else gate_tol
    rep = Report()
    dev_ids = np.asarray(dev_ids)
    dev_logits = np.asarray(dev_logits)
    dev_sel = np.asarray(dev_sel)
    M = hidden.shape[0]
    G = gate_W.shape[0]
    V = lm_W.shape[0]
    assert dev_ids.shape == (M, k) and dev_logits.shape == (M, k) and dev_sel.shape == (M, g)
    assert dev_ids.dtype == np.int32 and dev_sel.dtype == np.int32
    assert dev_logits.dtype == np.float32

    ref = oracle_grouped(hidden, gate_W, gate_bias, lm_W, offsets, rows, g, k, dtype,
                         gate_hidden=gate_hidden)
    order = rank_groups(ref.s)
    need_forced = False
    for m in range(M):
        sel = dev_sel[m]
        assert np.all((sel >= 0) & (sel < G)), f"token {m}: group id out of range {sel}"
        assert len(set(sel.tolist())) == g, f"token {m}: duplicate groups {sel}"
        if np.array_equal(sel, ref.sel[m]):
            continue
        best = ref.s[m, order[m, :g]]
        got = ref.s[m, sel]
        assert np.all(np.abs(got - best) < gate_tol), \
            f"token {m}: groups {sel} differ from {ref.sel[m]} beyond the gate tolerance"
        rep.forced_tokens += 1
        need_forced = True
    if need_forced:
        rep.notes.append("oracle re-run with the device's groups forced")
        ref = oracle_grouped(hidden, gate_W, gate_bias, lm_W, offsets, rows, g, k, dtype,
                             forced_sel=dev_sel, gate_hidden=gate_hidden)

    group_of = np.empty(V, dtype=np.int32)
    for n in range(G):
        group_of[rows[offsets[n]:offsets[n + 1]]] = n
    for m in range(M):
        ids = dev_ids[m]
        assert np.all((ids >= 0) & (ids < V)), f"token {m}: id out of range {ids}"
        oz = logits_rows(hidden[m], lm_W, ids, dtype)
        sel_m = dev_sel[m]
        _check_topk_token(m, ids, dev_logits[m], ref.topk_ids[m], ref.topk_z[m],
                          ref.next_z[m], oz, tol, rep,
                          member=lambda i, s=sel_m: np.isin(group_of[i], s))
    return rep


def check_dense(hidden, lm_W, k, dtype, dev_ids, dev_logits, tol=None, tokens=None) -> Report:
    """tokens: optional subset of token indices to check (each costs V dot products)."""
    tol = TOL[dtype] if tol is None else tol
    rep = Report()
    dev_ids = np.asarray(dev_ids)
    dev_logits = np.asarray(dev_logits)
    M = hidden.shape[0]
    V = lm_W.shape[0]
    assert dev_ids.shape == (M, k) and dev_logits.shape == (M, k)
    assert dev_ids.dtype == np.int32 and dev_logits.dtype == np.float32
    toks = list(range(M)) if tokens is None else list(tokens)
    sub = np.ascontiguousarray(hidden[toks])
    ref = oracle_dense(sub, lm_W, k, dtype)
    for i, m in enumerate(toks):
        ids = dev_ids[m]
        assert np.all((ids >= 0) & (ids < V)), f"token {m}: id out of range {ids}"
        oz = logits_rows(hidden[m], lm_W, ids, dtype)
        _check_topk_token(m, ids, dev_logits[m], ref.topk_ids[i], ref.topk_z[i],
                          ref.next_z[i], oz, tol, rep)
    return rep


def check_grouped_logprob(hidden, gate_W, gate_bias, lm_W, offsets, rows, g, k, dtype,
                          dev_ids, dev_logp, dev_sel, tol=None, gate_tol=None,
                          gate_hidden=None) -> Report:
    """Rules (i)-(v) and the exactness rule on log p(x) of Eq. 8 instead of the raw logit."""
    tol = LOGP_TOL[dtype] if tol is None else tol
    gate_tol = GATE_TOL[dtype] if gate_tol is None else gate_tol
    rep = Report()
    dev_ids = np.asarray(dev_ids)
    dev_logp = np.asarray(dev_logp)
    dev_sel = np.asarray(dev_sel)
    M = hidden.shape[0]
    G = gate_W.shape[0]
    V = lm_W.shape[0]
    assert dev_ids.shape == (M, k) and dev_logp.shape == (M, k) and dev_sel.shape == (M, g)
    assert dev_ids.dtype == np.int32 and dev_sel.dtype == np.int32 and dev_logp.dtype == np.float32

    ref = oracle_grouped_logprob(hidden, gate_W, gate_bias, lm_W, offsets, rows, g, k, dtype,
                                 gate_hidden=gate_hidden)
    order = rank_groups(ref.s)
    need_forced = False
    for m in range(M):
        sel = dev_sel[m]
        assert np.all((sel >= 0) & (sel < G)), f"token {m}: group id out of range {sel}"
        assert len(set(sel.tolist())) == g, f"token {m}: duplicate groups {sel}"
        if np.array_equal(sel, ref.sel[m]):
            continue
        best = ref.s[m, order[m, :g]]
        got = ref.s[m, sel]
        assert np.all(np.abs(got - best) < gate_tol), \
            f"token {m}: groups {sel} differ from {ref.sel[m]} beyond the gate tolerance"
        rep.forced_tokens += 1
        need_forced = True
    if need_forced:
        rep.notes.append("oracle re-run with the device's groups forced")
        ref = oracle_grouped_logprob(hidden, gate_W, gate_bias, lm_W, offsets, rows, g, k, dtype,
                                     forced_sel=dev_sel, gate_hidden=gate_hidden)

    group_of = np.empty(V, dtype=np.int32)
    for n in range(G):
        group_of[rows[offsets[n]:offsets[n + 1]]] = n
    for m in range(M):
        ids = dev_ids[m]
        assert np.all((ids >= 0) & (ids < V)), f"token {m}: id out of range {ids}"
        sel_m = dev_sel[m]
        assert np.isin(group_of[ids], sel_m).all(), f"token {m}: id outside the selected groups"
        slot = {int(n): j for j, n in enumerate(ref.sel[m])}
        z = logits_rows(hidden[m], lm_W, ids, dtype)
        olp = np.array([ref.logp_router[m, group_of[x]] + z[i] - ref.lse[m, slot[int(group_of[x])]]
                        for i, x in enumerate(ids)])
        _check_topk_token(m, ids, dev_logp[m], ref.topk_ids[m], ref.topk_logp[m],
                          ref.next_logp[m], olp, tol, rep)
    return rep



def check_premix(hidden, W1, dtype, act, dev_u) -> Report:
    """|device u - oracle u| <= PREMIX_ABS + half a unit in the last place of the storage
    type at that magnitude (bf16: 8 significand bits; f32: the absolute term only)."""
    rep = Report()
    u, _ = oracle_premix(hidden, W1, dtype, act)
    dev = widen(np.asarray(dev_u), dtype)
    assert dev.shape == u.shape
    assert np.all(np.isfinite(dev)), "non-finite pre-mix output"
    tol = np.full(u.shape, PREMIX_ABS[dtype])
    if dtype in ("bf16", "f16"):                   # 8 and 11 significand bits
        mag = np.maximum(np.abs(u), np.abs(dev))
        exp = np.floor(np.log2(np.maximum(mag, 2.0 ** -126)))
        if dtype == "f16":
            exp = np.maximum(exp, -14)             # below 2^-14 the spacing stays 2^-24
        tol = tol + 0.5 * 2.0 ** (exp - (7 if dtype == "bf16" else 10))
    err = np.abs(dev - u)
    bad = np.argwhere(err > tol)
    assert bad.size == 0, f"pre-mix: {len(bad)} elements off, first {bad[0]}: {dev[tuple(bad[0])]} vs {u[tuple(bad[0])]}"
    rep.tokens = u.shape[0]
    rep.max_abs_err = float(err.max())
    return rep
