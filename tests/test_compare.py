"""The agreement check itself: accepts the oracle's own answer and near-tie swaps,
rejects planted mistakes (all on the CPU, mistakes planted in oracle results)."""
import numpy as np
import pytest

import oracle
from oracle import compare
from coral_inputs import HeadConfig, make_head, make_hidden

CFG = HeadConfig("c16", "bf16", 64, 960, 8, 3, (5,), 6, 31, True)


def answer(head, hidden, g, k):
    c = head.cfg
    r = oracle.grouped(hidden, head.gate_W, head.gate_bias, head.lm_W, head.group_offsets,
                       head.group_rows, g, k, c.dtype)
    return r, r.topk_ids.copy(), r.topk_z.astype(np.float32), r.sel.copy()


def check(head, hidden, g, k, ids, z, sel):
    c = head.cfg
    return compare.check_grouped(hidden, head.gate_W, head.gate_bias, head.lm_W,
                                 head.group_offsets, head.group_rows, g, k, c.dtype, ids, z, sel)


def test_accepts_the_oracles_answer():
    head, hidden = make_head(CFG), make_hidden(CFG, 5)
    _, ids, z, sel = answer(head, hidden, CFG.g, CFG.k)
    rep = check(head, hidden, CFG.g, CFG.k, ids, z, sel)
    assert rep.tokens == 5 and rep.forced_tokens == 0 and rep.max_abs_err < 1e-6
    d = oracle.dense(hidden, head.lm_W, CFG.k, "bf16")
    rep = compare.check_dense(hidden, head.lm_W, CFG.k, "bf16", d.topk_ids,
                              d.topk_z.astype(np.float32))
    assert rep.tokens == 5


@pytest.mark.parametrize("mistake", ["wrong_id", "wrong_logit", "wrong_order", "wrong_group",
                                     "duplicate_id", "outside_group", "dropped_best"])
def test_rejects_planted_mistakes(mistake):
    head, hidden = make_head(CFG), make_hidden(CFG, 5)
    r, ids, z, sel = answer(head, hidden, CFG.g, CFG.k)
    if mistake == "wrong_id":
        # replace the last candidate by the worst row of the same group
        seg = head.group_rows[head.group_offsets[sel[2, 0]]:head.group_offsets[sel[2, 0] + 1]]
        zz = oracle.logits_rows(hidden[2], head.lm_W, seg, "bf16")
        ids[2, -1] = seg[np.argmin(zz)]
        z[2, -1] = zz.min()
    elif mistake == "wrong_logit":
        z[1, 3] += np.float32(4e-3)
        z[1, :3] += np.float32(4e-3)      # keep it descending: only the value is wrong
    elif mistake == "wrong_order":
        ids[0, [0, 1]] = ids[0, [1, 0]]
        assert r.topk_z[0, 0] - r.topk_z[0, 1] > 2e-3
    elif mistake == "wrong_group":
        order = oracle.rank_groups(r.s)
        sel[3, -1] = order[3, -1]          # worst group instead of the g-th best
    elif mistake == "duplicate_id":
        ids[4, 1] = ids[4, 0]
        z[4, 1] = z[4, 0]
    elif mistake == "outside_group":
        order = oracle.rank_groups(r.s)
        n = order[0, -1]
        ids[0, -1] = head.group_rows[head.group_offsets[n]]
    elif mistake == "dropped_best":
        ids[2] = np.roll(ids[2], -1)
        z[2] = np.roll(z[2], -1)
        z[2, -1] = z[2, -2] - 1.0
    with pytest.raises(AssertionError):
        check(head, hidden, CFG.g, CFG.k, ids, z, sel)


def test_accepts_swaps_inside_a_near_tie_only():
    """Two rows whose logits differ by far less than tol may come back in either order;
    rows further apart may not."""
    cfg = HeadConfig("tie", "f32", 32, 256, 4, 4, (1,), 4, 5, False)
    head, hidden = make_head(cfg), make_hidden(cfg, 1)
    d = oracle.dense(hidden, head.lm_W, 1, "f32")
    best = int(d.topk_ids[0, 0])
    twin = (best + 100) % cfg.V
    head.lm_W[twin] = head.lm_W[best]
    j = int(np.argmax(np.abs(hidden[0])))
    head.lm_W[twin, j] = np.nextafter(head.lm_W[twin, j], np.float32(np.inf))   # ~1e-9 apart
    r, ids, z, sel = answer(head, hidden, 4, 4)
    assert set(ids[0, :2]) == {best, twin} and abs(r.topk_z[0, 0] - r.topk_z[0, 1]) < 1e-6
    lo, hi = min(best, twin), max(best, twin)
    top = max(z[0, 0], z[0, 1])
    # a device that sees the two logits as equal in fp32 must list the lower id first
    ids[0, :2] = [lo, hi]
    z[0, :2] = top
    check(head, hidden, 4, 4, ids, z, sel)
    ids[0, :2] = [hi, lo]
    with pytest.raises(AssertionError):
        check(head, hidden, 4, 4, ids, z, sel)
    # a device whose rounding separates them may list either first
    z[0, 0] = np.nextafter(top, np.float32(np.inf))
    check(head, hidden, 4, 4, ids, z, sel)
    ids[0, :2] = [lo, hi]
    check(head, hidden, 4, 4, ids, z, sel)
    # ... but not a pair that is clearly apart
    ids[0, [1, 3]] = ids[0, [3, 1]]
    z[0, [1, 3]] = z[0, [3, 1]]
    assert r.topk_z[0, 1] - r.topk_z[0, 3] > 1e-5
    with pytest.raises(AssertionError):
        check(head, hidden, 4, 4, ids, z, sel)


def test_group_near_tie_uses_forced_selection():
    cfg = HeadConfig("gt", "f32", 32, 256, 4, 2, (2,), 4, 6, False)
    head, hidden = make_head(cfg), make_hidden(cfg, 2)
    r0 = oracle.grouped(hidden, head.gate_W, None, head.lm_W, head.group_offsets,
                        head.group_rows, 2, 4, "f32")
    order = oracle.rank_groups(r0.s)
    a, b = order[0, 1], order[0, 2]              # g-th and (g+1)-th group of token 0
    head.gate_W[b] = head.gate_W[a]              # identical scores: a wins by lower id or b does
    r, ids, z, sel = answer(head, hidden, 2, 4)
    other = b if sel[0, 1] == a else a
    sel2 = sel.copy()
    sel2[0, 1] = other
    rf = oracle.grouped(hidden, head.gate_W, None, head.lm_W, head.group_offsets,
                        head.group_rows, 2, 4, "f32", forced_sel=sel2)
    rep = check(head, hidden, 2, 4, rf.topk_ids, rf.topk_z.astype(np.float32), sel2)
    assert rep.forced_tokens == 1
    assert not np.array_equal(rf.topk_ids, ids)   # the swapped group changes the candidates
    with pytest.raises(AssertionError):           # so the oracle's own candidates do not fit sel2
        check(head, hidden, 2, 4, ids, z, sel2)


# ------------------------------------------------------------------ log-probability mode
def test_logprob_check_accepts_the_oracles_answer_and_rejects_the_logit_ranking():
    head, hidden = make_head(CFG), make_hidden(CFG, 5)
    c = head.cfg
    r = oracle.grouped_logprob(hidden, head.gate_W, head.gate_bias, head.lm_W, head.group_offsets,
                               head.group_rows, CFG.g, CFG.k, c.dtype)
    args = (hidden, head.gate_W, head.gate_bias, head.lm_W, head.group_offsets, head.group_rows,
            CFG.g, CFG.k, c.dtype)
    rep = compare.check_grouped_logprob(*args, r.topk_ids, r.topk_logp.astype(np.float32), r.sel)
    assert rep.tokens == 5 and rep.max_abs_err < 1e-6
    # a device that ranked raw logits (or returned them) must not pass
    b = oracle.grouped(*args)
    assert not np.array_equal(b.topk_ids, r.topk_ids)          # the two rankings differ here
    with pytest.raises(AssertionError):
        compare.check_grouped_logprob(*args, b.topk_ids, b.topk_z.astype(np.float32), b.sel)
    # right ids, log-probabilities off by the router term
    wrong = (r.topk_logp + 0.05).astype(np.float32)
    with pytest.raises(AssertionError):
        compare.check_grouped_logprob(*args, r.topk_ids, wrong, r.sel)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_premix_check_accepts_the_oracles_rounding_and_rejects_planted_mistakes(dtype):
    from coral_inputs import make_router_W1
    cfg = HeadConfig("premix_cmp", dtype, 64, 256, 4, 2, (3,), 4, 21, True)
    h = make_hidden(cfg, 3, 0)
    W1 = make_router_W1(cfg)
    u, stored = oracle.premix(h, W1, dtype, "silu")
    compare.check_premix(h, W1, dtype, "silu", stored)
    # a different activation, a dropped residual, a transposed projection
    for wrong in (oracle.premix(h, W1, dtype, "relu")[1],
                  oracle.round_to_storage(u - oracle.widen(h, dtype), dtype),
                  oracle.premix(h, np.ascontiguousarray(W1.T), dtype, "silu")[1]):
        with pytest.raises(AssertionError):
            compare.check_premix(h, W1, dtype, "silu", wrong)
    if dtype == "bf16":                            # one unit in the last place is too much
        off = stored.copy()
        off[1, 5] += 1
        with pytest.raises(AssertionError):
            compare.check_premix(h, W1, dtype, "silu", off)


def test_routed_check_follows_gate_hidden():
    cfg = HeadConfig("routed_cmp", "f32", 64, 512, 8, 2, (3,), 4, 22, False)
    head = make_head(cfg)
    h = make_hidden(cfg, 3, 0)
    gh = make_hidden(cfg, 3, 1)
    args = (head.gate_W, None, head.lm_W, head.group_offsets, head.group_rows, cfg.g, cfg.k, cfg.dtype)
    r = oracle.grouped(h, *args, gate_hidden=gh)
    ok = (r.topk_ids, r.topk_z.astype(np.float32), r.sel)
    compare.check_grouped(h, *args, *ok, gate_hidden=gh)
    plain = oracle.grouped(h, *args)
    assert not np.array_equal(plain.sel, r.sel)
    with pytest.raises(AssertionError):            # the unrouted answer is not the routed one
        compare.check_grouped(h, *args, plain.topk_ids, plain.topk_z.astype(np.float32), plain.sel,
                              gate_hidden=gh)
