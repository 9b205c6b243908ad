"""Pins for the fp64 CPU oracle (no GPU).

The paper prints no worked numbers for the grouped head, so the oracle is
pinned to what the mathematics fixes: a second implementation in numpy
(float64 matmul + lexsort, the library routines the dense head reduces to),
closed forms for one-hot inputs, and invariants that follow from section 3.3
(the groups partition the vocabulary; with every group active the grouped head
is the dense head; Eq. 8's distribution sums to one).
"""
import numpy as np
import pytest

import oracle
from coral_inputs import CONFIGS, HeadConfig, make_head, make_hidden, make_partition

TINY = HeadConfig("t", "f32", 4, 12, 3, 2, (3,), 3, 7, False)
SMALL_F32 = HeadConfig("s32", "f32", 24, 240, 6, 2, (5,), 7, 11, False)
SMALL_BF16 = HeadConfig("s16", "bf16", 40, 360, 8, 3, (6,), 9, 12, True, bias_std=2.0)
CASES = [TINY, SMALL_F32, SMALL_BF16]


def widen(a):
    """Independent widening of the storage types to float64."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def np_rank(vals, ids, k):
    o = np.lexsort((ids, -vals))          # primary: value descending; then id ascending
    return ids[o[:k]], vals[o[:k]]


def np_grouped(head, hidden, g, k, forced=None):
    """Brute force: every score, every row, full sorts."""
    h = widen(hidden)
    s = h @ widen(head.gate_W).T
    if head.gate_bias is not None:
        s = s + head.gate_bias.astype(np.float64)[None, :]
    Z = h @ widen(head.lm_W).T
    G = head.gate_W.shape[0]
    out_sel, out_ids, out_z = [], [], []
    for m in range(h.shape[0]):
        sel, _ = np_rank(s[m], np.arange(G, dtype=np.int32), g)
        if forced is not None:
            sel = forced[m]
        cand = np.concatenate([head.group_rows[head.group_offsets[n]:head.group_offsets[n + 1]]
                               for n in sel])
        ids, z = np_rank(Z[m, cand], cand, k)
        out_sel.append(sel), out_ids.append(ids), out_z.append(z)
    return s, np.array(out_sel), np.array(out_ids), np.array(out_z), Z


def run_oracle(head, hidden, g, k, forced=None):
    c = head.cfg
    return oracle.grouped(hidden, head.gate_W, head.gate_bias, head.lm_W, head.group_offsets,
                          head.group_rows, g, k, c.dtype, forced_sel=forced)


@pytest.mark.parametrize("cfg", CASES, ids=lambda c: c.name)
def test_brute_force_numpy(cfg):
    head = make_head(cfg)
    hidden = make_hidden(cfg, cfg.Ms[0])
    r = run_oracle(head, hidden, cfg.g, cfg.k)
    s, sel, ids, z, Z = np_grouped(head, hidden, cfg.g, cfg.k)
    np.testing.assert_allclose(r.s, s, rtol=0, atol=1e-12)
    assert np.array_equal(r.sel, sel)
    assert np.array_equal(r.topk_ids, ids)
    np.testing.assert_allclose(r.topk_z, z, rtol=0, atol=1e-12)
    d = oracle.dense(hidden, head.lm_W, cfg.k, cfg.dtype)
    for m in range(hidden.shape[0]):
        di, dz = np_rank(Z[m], np.arange(cfg.V, dtype=np.int32), cfg.k + 1)
        assert np.array_equal(d.topk_ids[m], di[:cfg.k])
        np.testing.assert_allclose(d.topk_z[m], dz[:cfg.k], rtol=0, atol=1e-12)
        assert abs(d.next_z[m] - dz[cfg.k]) < 1e-12


def test_tiny_config_of_the_workload_table():
    """configs[0] (H=256, V=8192, 16 groups of 512, top-2, k=8) against numpy."""
    cfg = CONFIGS["tiny_f32"]
    head = make_head(cfg)
    hidden = make_hidden(cfg, 4)
    r = run_oracle(head, hidden, cfg.g, cfg.k)
    s, sel, ids, z, _ = np_grouped(head, hidden, cfg.g, cfg.k)
    assert np.array_equal(r.sel, sel) and np.array_equal(r.topk_ids, ids)
    np.testing.assert_allclose(r.topk_z, z, rtol=0, atol=1e-12)


def test_non_square_operands_are_not_transposed():
    """gate_W is [G,H] and lm_W is [V,H] with G != H != V: a transposed read fails."""
    rng = np.random.default_rng(0)
    H, V, G = 5, 14, 7
    hidden = rng.standard_normal((2, H)).astype(np.float32)
    gate_W = rng.standard_normal((G, H)).astype(np.float32)
    lm_W = rng.standard_normal((V, H)).astype(np.float32)
    s = oracle.gate(hidden, gate_W, None, "f32")
    np.testing.assert_allclose(s, hidden.astype(np.float64) @ gate_W.astype(np.float64).T,
                               atol=1e-13)
    z = oracle.logits_rows(hidden[1], lm_W, np.arange(V), "f32")
    np.testing.assert_allclose(z, lm_W.astype(np.float64) @ hidden[1].astype(np.float64),
                               atol=1e-13)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_one_hot_hidden_reads_a_weight_column(dtype):
    """hidden = c*e_j  =>  z[r] = c*lm_W[r,j] and s[n] = c*gate_W[n,j] + bias[n], exactly."""
    cfg = SMALL_BF16.scaled(dtype=dtype)
    head = make_head(cfg)
    j, c = 17, -2.0
    hf = np.zeros((1, cfg.H), dtype=np.float32)
    hf[0, j] = c
    hidden = hf if dtype == "f32" else (hf.view(np.uint32) >> 16).astype(np.uint16)
    s = oracle.gate(hidden, head.gate_W, head.gate_bias, dtype)
    want = c * widen(head.gate_W)[:, j] + head.gate_bias.astype(np.float64)
    assert np.array_equal(s[0], want)
    z = oracle.logits_rows(hidden[0], head.lm_W, np.arange(cfg.V), dtype)
    assert np.array_equal(z, c * widen(head.lm_W)[:, j])
    # negative scale: the best candidates are the most negative column entries
    d = oracle.dense(hidden, head.lm_W, 4, dtype)
    col = widen(head.lm_W)[:, j]
    assert np.array_equal(d.topk_ids[0], np_rank(c * col, np.arange(cfg.V, dtype=np.int32), 4)[0])


def test_one_hot_gate_rows_make_the_selection_readable():
    """gate_W[n] = e_n: the selected groups are the largest hidden coordinates."""
    H, G, V = 8, 4, 16
    gate_W = np.zeros((G, H), dtype=np.float32)
    gate_W[np.arange(G), np.arange(G)] = 1.0
    hidden = np.array([[0.1, 0.9, -0.3, 0.5, 9, 9, 9, 9],
                       [-1.0, -2.0, -0.5, -3.0, 0, 0, 0, 0]], dtype=np.float32)
    s = oracle.gate(hidden, gate_W, None, "f32")
    order = oracle.rank_groups(s)
    assert order.tolist() == [[1, 3, 0, 2], [2, 0, 1, 3]]
    # a bias can overturn it
    bias = np.array([0, 0, 5, 0], dtype=np.float32)
    order = oracle.rank_groups(oracle.gate(hidden, gate_W, bias, "f32"))
    assert order[0, 0] == 2 and order[1, 0] == 2
    # identity LM head: the candidates are the largest hidden coordinates inside the groups
    lm_W = np.zeros((V, H), dtype=np.float32)
    lm_W[np.arange(H), np.arange(H)] = 2.0
    offsets = np.arange(G + 1, dtype=np.int32) * 4
    rows = np.array([0, 4, 8, 12, 1, 5, 9, 13, 2, 6, 10, 14, 3, 7, 11, 15], dtype=np.int32)
    r = oracle.grouped(hidden, gate_W, None, lm_W, offsets, rows, 2, 3, "f32")
    assert r.sel.tolist() == [[1, 3], [2, 0]]
    # token 0: groups 1,3 own rows {1,5,9,13,3,7,11,15}; z = 2*hidden[r] for r<8 else 0
    assert r.topk_ids[0].tolist() == [5, 7, 1]
    assert r.topk_z[0].tolist() == [18.0, 18.0, 2 * np.float64(np.float32(0.9))]
    # token 1: groups 2,0 own rows {2,6,10,14,0,4,8,12}; zeros tie -> lower id first
    assert r.topk_ids[1].tolist() == [4, 6, 8]
    assert r.topk_z[1].tolist() == [0.0, 0.0, 0.0]


@pytest.mark.parametrize("cfg", CASES, ids=lambda c: c.name)
def test_all_groups_active_equals_dense_bit_for_bit(cfg):
    head = make_head(cfg)
    hidden = make_hidden(cfg, cfg.Ms[0])
    r = run_oracle(head, hidden, cfg.G, cfg.k)
    d = oracle.dense(hidden, head.lm_W, cfg.k, cfg.dtype)
    assert np.array_equal(r.topk_ids, d.topk_ids)
    assert np.array_equal(r.topk_z, d.topk_z)
    assert np.array_equal(r.next_z, d.next_z)


@pytest.mark.parametrize("name", list(CONFIGS))
def test_groups_partition_the_vocabulary(name):
    cfg = CONFIGS[name]
    offsets, rows = make_partition(cfg)
    assert offsets[0] == 0 and offsets[-1] == cfg.V and np.all(np.diff(offsets) == cfg.v)
    assert np.array_equal(np.sort(rows), np.arange(cfg.V))
    for n in range(cfg.G):                       # ascending inside each group
        assert np.all(np.diff(rows[offsets[n]:offsets[n + 1]]) > 0)
    assert oracle.check_partition(offsets, rows, cfg.V) == 0
    bad = rows.copy()
    bad[5] = bad[6]
    assert oracle.check_partition(offsets, bad, cfg.V) != 0
    bad_off = offsets.copy()
    bad_off[-1] -= 1
    assert oracle.check_partition(bad_off, rows, cfg.V) != 0


def test_grouped_rejects_a_broken_partition():
    head = make_head(TINY)
    hidden = make_hidden(TINY, 2)
    rows = head.group_rows.copy()
    rows[0] = rows[1]
    with pytest.raises(oracle.OracleError):
        oracle.grouped(hidden, head.gate_W, None, head.lm_W, head.group_offsets, rows, 2, 3, "f32")


def test_top_k_is_the_prefix_of_a_full_sort_with_ties():
    rng = np.random.default_rng(3)
    z = rng.integers(-3, 4, size=200).astype(np.float64)      # many exact ties
    ids = rng.permutation(1000)[:200].astype(np.int32)
    for k in (1, 7, 199, 200):
        oi, oz, nxt = oracle.top_k(z, ids, k)
        wi, wz = np_rank(z, ids, 200)
        assert np.array_equal(oi, wi[:k]) and np.array_equal(oz, wz[:k])
        assert nxt == (wz[k] if k < 200 else -np.inf)
    # brute force by repeated max on a handful of values
    z = np.array([1.0, 3.0, 3.0, -1.0, 2.0])
    ids = np.array([9, 5, 2, 1, 7], dtype=np.int32)
    oi, oz, nxt = oracle.top_k(z, ids, 3)
    assert oi.tolist() == [2, 5, 7] and oz.tolist() == [3.0, 3.0, 2.0] and nxt == 1.0
    with pytest.raises(oracle.OracleError):
        oracle.top_k(z, ids, 6)


def test_duplicate_weight_rows_tie_break_to_the_lower_id():
    cfg = SMALL_F32
    head = make_head(cfg)
    hidden = make_hidden(cfg, 3)
    d0 = oracle.dense(hidden[:1], head.lm_W, 1, "f32")
    best = int(d0.topk_ids[0, 0])
    other = (best + 37) % cfg.V
    head.lm_W[other] = head.lm_W[best]
    d = oracle.dense(hidden[:1], head.lm_W, 2, "f32")
    assert d.topk_ids[0].tolist() == sorted([best, other])
    assert d.topk_z[0, 0] == d.topk_z[0, 1]


def test_candidate_sets_nest_and_bound_by_dense():
    cfg = SMALL_BF16
    head = make_head(cfg)
    hidden = make_hidden(cfg, 6)
    dense = oracle.dense(hidden, head.lm_W, cfg.k, cfg.dtype)
    group_of = np.empty(cfg.V, dtype=np.int32)
    for n in range(cfg.G):
        group_of[head.group_rows[head.group_offsets[n]:head.group_offsets[n + 1]]] = n
    prev = None
    for g in range(1, cfg.G + 1):
        r = run_oracle(head, hidden, g, cfg.k)
        assert np.all(r.topk_z[:, 0] <= dense.topk_z[:, 0])
        if prev is not None:
            assert np.array_equal(r.sel[:, :g - 1], prev.sel)          # selections nest
            assert np.all(r.topk_z >= prev.topk_z)                      # rank-wise dominance
        for m in range(6):
            assert np.isin(group_of[r.topk_ids[m]], r.sel[m]).all()
            if np.isin(group_of[dense.topk_ids[m]], r.sel[m]).all():
                assert np.array_equal(r.topk_ids[m], dense.topk_ids[m])
                assert np.array_equal(r.topk_z[m], dense.topk_z[m])
        prev = r


def test_relabelling_groups_and_shuffling_rows_changes_nothing():
    cfg = SMALL_BF16
    head = make_head(cfg)
    hidden = make_hidden(cfg, 4)
    base = run_oracle(head, hidden, cfg.g, cfg.k)
    rng = np.random.default_rng(5)
    relabel = rng.permutation(cfg.G)              # new group i is old group relabel[i]
    offs, rows = [0], []
    for i in range(cfg.G):
        n = relabel[i]
        seg = head.group_rows[head.group_offsets[n]:head.group_offsets[n + 1]]
        rows.append(rng.permutation(seg))         # shuffle inside the group too
        offs.append(offs[-1] + seg.size)
    r = oracle.grouped(hidden, head.gate_W[relabel], head.gate_bias[relabel], head.lm_W,
                       np.array(offs, np.int32), np.concatenate(rows).astype(np.int32),
                       cfg.g, cfg.k, cfg.dtype)
    assert np.array_equal(relabel[r.sel], base.sel)
    assert np.array_equal(r.topk_ids, base.topk_ids) and np.array_equal(r.topk_z, base.topk_z)


def test_duplicated_token_duplicates_its_outputs_and_forced_selection():
    cfg = SMALL_BF16
    head = make_head(cfg)
    hidden = make_hidden(cfg, 3)
    hidden2 = np.concatenate([hidden, hidden[1:2]], axis=0)
    r = run_oracle(head, hidden2, cfg.g, cfg.k)
    assert np.array_equal(r.topk_ids[3], r.topk_ids[1]) and np.array_equal(r.topk_z[3], r.topk_z[1])
    forced = np.tile(np.array([[5, 0, 2]], dtype=np.int32), (4, 1))
    rf = run_oracle(head, hidden2, cfg.g, cfg.k, forced=forced)
    _, _, ids, z, _ = np_grouped(head, hidden2, cfg.g, cfg.k, forced=forced)
    assert np.array_equal(rf.sel, forced) and np.array_equal(rf.topk_ids, ids)
    np.testing.assert_allclose(rf.topk_z, z, atol=1e-12)
    with pytest.raises(oracle.OracleError):       # a group listed twice
        run_oracle(head, hidden2, cfg.g, cfg.k, forced=np.tile(np.array([[1, 1, 2]], np.int32), (4, 1)))


def test_union_of_activated_groups_is_bounded(golden_dir):
    """Appendix, tree decoding: top-2 groups x 10 candidates activate at most 20 groups,
    so a 32-group head is never fully active."""
    vals = {}
    for line in open(f"{golden_dir}/table1_shapes.txt"):
        p = line.split()
        if len(p) == 2 and not line.startswith("#"):
            vals[p[0]] = float(p[1])
    g, M = int(vals["tree_top_groups"]), int(vals["tree_candidates"])
    assert g * M == vals["tree_worst_case_groups"] < vals["tree_safe_group_count"]
    for G in (16, 32):
        cfg = HeadConfig("u", "f32", 16, G * 4, G, g, (M,), 3, 21, False)
        head = make_head(cfg)
        for b in range(20):
            r = run_oracle(head, make_hidden(cfg, M, batch=b), g, 3)
            assert len(np.unique(r.sel)) <= min(G, g * M)
            assert all(len(set(row)) == g for row in r.sel.tolist())


@pytest.mark.parametrize("cfg", [SMALL_F32, SMALL_BF16], ids=lambda c: c.name)
def test_router_times_group_softmax_is_normalised(cfg):
    """Eq. 8: p(x) = p_router(n) * p_group(x^n) sums to one over the vocabulary (g = G)."""
    head = make_head(cfg)
    hidden = make_hidden(cfg, 3)
    r = run_oracle(head, hidden, cfg.G, cfg.k)
    np.testing.assert_allclose(np.exp(r.logp_router).sum(axis=1), 1.0, atol=1e-12)
    Z = widen(hidden) @ widen(head.lm_W).T
    for m in range(3):
        total = 0.0
        for i, n in enumerate(r.sel[m]):
            seg = head.group_rows[head.group_offsets[n]:head.group_offsets[n + 1]]
            pg = np.exp(Z[m, seg] - r.lse[m, i])
            assert abs(pg.sum() - 1.0) < 1e-12
            total += np.exp(r.logp_router[m, n]) * pg.sum()
        assert abs(total - 1.0) < 1e-12
    # log-softmax against its definition
    s = r.s
    want = s - np.log(np.exp(s - s.max(1, keepdims=True)).sum(1, keepdims=True)) - s.max(1, keepdims=True)
    np.testing.assert_allclose(r.logp_router, want, atol=1e-12)


def test_bf16_widening_on_known_bit_patterns():
    bits = np.array([[0x3F80, 0xC000, 0x0000, 0x3E00]], dtype=np.uint16)   # 1, -2, 0, 0.125
    W = np.array([[0x4000, 0x3F80, 0x7F7F, 0x4080],                          # 2, 1, big, 4
                  [0xBF80, 0xBF80, 0x0000, 0x0000]], dtype=np.uint16)        # -1, -1, 0, 0
    z = oracle.logits_rows(bits[0], W, [0, 1], "bf16")
    assert z.tolist() == [2.0 - 2.0 + 0.0 + 0.5, -1.0 + 2.0]


def test_generator_rounds_to_bf16_like_an_independent_library():
    import torch
    from coral_inputs import to_bf16_bits
    x = np.random.default_rng(0).standard_normal(100000).astype(np.float32) * 0.02
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 3.0e-39]    # exact ties and a subnormal
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(to_bf16_bits(x), want)


def test_thread_count_does_not_change_results():
    cfg = SMALL_BF16
    head = make_head(cfg)
    hidden = make_hidden(cfg, 4)
    n = oracle.max_threads()
    oracle.set_threads(1)
    a = run_oracle(head, hidden, cfg.g, cfg.k)
    oracle.set_threads(n)
    b = run_oracle(head, hidden, cfg.g, cfg.k)
    assert np.array_equal(a.topk_ids, b.topk_ids) and np.array_equal(a.topk_z, b.topk_z)


def test_inputs_follow_the_stated_recipe():
    cfg = CONFIGS["llama2_7b"].scaled(V=3200, G=16)
    a, b = make_head(cfg), make_head(cfg)
    assert np.array_equal(a.lm_W, b.lm_W) and np.array_equal(a.group_rows, b.group_rows)
    h = widen(make_hidden(cfg, 8))
    np.testing.assert_allclose(np.sqrt((h ** 2).mean(axis=1)), 1.0, atol=3e-3)   # unit RMS
    w = widen(a.lm_W)
    assert abs(w.std() - 0.02) < 2e-4 and abs(w.mean()) < 1e-4
    assert not np.array_equal(make_hidden(cfg, 8, batch=1), make_hidden(cfg, 8, batch=0))


# ------------------------------------------------------------------ Eq. 8 composition
def _np_logprob_reference(hidden, gate_W, bias, lm_W, offsets, rows, g, k):
    """Independent float64 numpy/scipy version of the log-probability head."""
    from scipy.special import log_softmax, logsumexp
    s = hidden @ gate_W.T + (0.0 if bias is None else bias)
    out_ids, out_lp = [], []
    for m in range(hidden.shape[0]):
        sel = np.lexsort((np.arange(s.shape[1]), -s[m]))[:g]
        lpr = log_softmax(s[m])
        ids, lp = [], []
        for n in sel:
            r = rows[offsets[n]:offsets[n + 1]]
            z = lm_W[r] @ hidden[m]
            ids.append(r)
            lp.append(lpr[n] + z - logsumexp(z))
        ids, lp = np.concatenate(ids), np.concatenate(lp)
        o = np.lexsort((ids, -lp))[:k]
        out_ids.append(ids[o])
        out_lp.append(lp[o])
    return np.array(out_ids), np.array(out_lp)


@pytest.mark.parametrize("seed,H,V,G,g,M,k", [(0, 16, 96, 6, 2, 3, 7), (1, 24, 120, 4, 4, 2, 12),
                                               (2, 8, 64, 8, 3, 5, 5)])
def test_logprob_matches_numpy_scipy(seed, H, V, G, g, M, k):
    rng = np.random.default_rng(seed)
    hidden = rng.standard_normal((M, H)).astype(np.float32)
    gate_W = rng.standard_normal((G, H)).astype(np.float32)
    lm_W = rng.standard_normal((V, H)).astype(np.float32)
    bias = rng.standard_normal(G).astype(np.float32)
    perm = rng.permutation(V).astype(np.int32)
    v = V // G
    offsets = (np.arange(G + 1) * v).astype(np.int32)
    rows = np.concatenate([np.sort(perm[n * v:(n + 1) * v]) for n in range(G)]).astype(np.int32)
    r = oracle.grouped_logprob(hidden, gate_W, bias, lm_W, offsets, rows, g, k, "f32")
    ids, lp = _np_logprob_reference(hidden.astype(np.float64), gate_W.astype(np.float64),
                                    bias.astype(np.float64), lm_W.astype(np.float64), offsets, rows, g, k)
    assert np.array_equal(r.topk_ids, ids)
    assert np.max(np.abs(r.topk_logp - lp)) < 1e-11


def test_logprob_sums_to_one_over_the_vocabulary_when_all_groups_are_active():
    rng = np.random.default_rng(5)
    H, V, G = 12, 60, 5
    hidden = rng.standard_normal((2, H)).astype(np.float32)
    gate_W = rng.standard_normal((G, H)).astype(np.float32)
    lm_W = rng.standard_normal((V, H)).astype(np.float32)
    offsets = (np.arange(G + 1) * (V // G)).astype(np.int32)
    rows = np.arange(V, dtype=np.int32)
    r = oracle.grouped_logprob(hidden, gate_W, None, lm_W, offsets, rows, G, V, "f32")
    assert np.allclose(np.exp(r.topk_logp).sum(axis=1), 1.0, atol=1e-12)
    assert np.all(np.diff(r.topk_logp, axis=1) <= 0)


def test_logprob_single_group_is_a_log_softmax():
    from scipy.special import log_softmax
    rng = np.random.default_rng(6)
    H, V = 10, 40
    hidden = rng.standard_normal((3, H)).astype(np.float32)
    lm_W = rng.standard_normal((V, H)).astype(np.float32)
    gate_W = rng.standard_normal((1, H)).astype(np.float32)
    r = oracle.grouped_logprob(hidden, gate_W, None, lm_W, np.array([0, V], np.int32),
                               np.arange(V, dtype=np.int32), 1, V, "f32")
    full = log_softmax(hidden.astype(np.float64) @ lm_W.astype(np.float64).T, axis=1)
    for m in range(3):
        assert np.allclose(r.topk_logp[m], np.sort(full[m])[::-1], atol=1e-12)


def test_logprob_ranking_differs_from_logit_ranking_in_a_hand_worked_case():
    """Groups A = {0, 1} with logits (2, 2) and B = {2, 3} with (1.5, -10), equal router
    scores: p(2) = 1/2 * ~1, p(0) = p(1) = 1/2 * 1/2, so row 2 comes first although its logit
    is the lower one.  Values by hand: log p(0) = -2 ln 2, log p(2) = -ln 2 - ln(1 + e^-11.5)."""
    hidden = np.array([[1.0, 0.0]], np.float32)
    lm_W = np.array([[2.0, 0.0], [2.0, 0.0], [1.5, 0.0], [-10.0, 0.0]], np.float32)
    gate_W = np.zeros((2, 2), np.float32)
    offsets = np.array([0, 2, 4], np.int32)
    rows = np.arange(4, dtype=np.int32)
    r = oracle.grouped_logprob(hidden, gate_W, None, lm_W, offsets, rows, 2, 3, "f32")
    assert r.topk_ids[0].tolist() == [2, 0, 1]
    want = [-np.log(2) - np.log1p(np.exp(-11.5)), -2 * np.log(2), -2 * np.log(2)]
    assert np.allclose(r.topk_logp[0], want, atol=1e-14)
    b = oracle.grouped(hidden, gate_W, None, lm_W, offsets, rows, 2, 3, "f32")
    assert b.topk_ids[0].tolist() == [0, 1, 2]


# ---------------------------------------------------------------- router pre-mix (Eq. 7)
def _f32(x):
    return np.ascontiguousarray(x, dtype=np.float32)


@pytest.mark.parametrize("act", oracle.ACTIVATIONS)
def test_premix_with_zero_projection_is_the_residual(act):
    rng = np.random.default_rng(5)
    h = _f32(rng.standard_normal((3, 16)))
    u, stored = oracle.premix(h, _f32(np.zeros((16, 16))), "f32", act)
    assert np.array_equal(u, h.astype(np.float64))          # act(0) = 0 for all three
    assert np.array_equal(stored, h)


def test_premix_single_weight_pins_orientation_and_residual():
    # W1[i0, j0] = c only: output feature i0 reads input feature j0 (y = W1 h, not W1^T h)
    H, i0, j0, c = 8, 2, 5, 0.5
    W1 = np.zeros((H, H), np.float32)
    W1[i0, j0] = c
    h = _f32(np.arange(1, 2 * H + 1).reshape(2, H))
    u, _ = oracle.premix(h, W1, "f32", "identity")
    want = h.astype(np.float64).copy()
    want[:, i0] += c * h[:, j0]
    assert np.array_equal(u, want)


def test_premix_activations_closed_forms():
    # H = 1: u = act(w h) + h
    one = _f32([[1.0]])
    for w, h, act, want in [
        (1.0, 1.0, "silu", 1.0 / (1.0 + np.exp(-1.0)) + 1.0),        # silu(1) = 0.73105857863...
        (-1.0, 1.0, "silu", -1.0 / (1.0 + np.exp(1.0)) + 1.0),       # silu(-1) = -0.26894142137...
        (2.0, -1.5, "relu", -1.5),                                   # relu(-3) = 0
        (2.0, 1.5, "relu", 4.5),
        (-3.0, 2.0, "identity", -4.0),
    ]:
        u, _ = oracle.premix(_f32([[h]]), _f32([[w]]), "f32", act)
        assert abs(u[0, 0] - want) < 1e-15, (w, h, act)
    assert abs(oracle.premix(one, one, "f32", "silu")[0][0, 0] - 1.7310585786300049) < 1e-15


def test_premix_matches_an_independent_formulation():
    from scipy.special import expit
    rng = np.random.default_rng(11)
    H, M = 48, 5
    h = to_bits(rng.standard_normal((M, H)))
    W1 = to_bits(rng.standard_normal((H, H)) * 0.2)
    hf = oracle.widen(h, "bf16")
    wf = oracle.widen(W1, "bf16")
    u, stored = oracle.premix(h, W1, "bf16", "silu")
    want = np.empty((M, H))
    for m in range(M):
        for i in range(H):
            y = float(np.dot(wf[i], hf[m]))
            want[m, i] = y * expit(y) + hf[m, i]
    assert np.allclose(u, want, rtol=0, atol=1e-13)
    # storage rounding: nearest bf16 of the float32 value, checked against torch
    import torch
    t = torch.from_numpy(u.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(stored, t)


def to_bits(x):
    from coral_inputs import to_bf16_bits
    return to_bf16_bits(np.asarray(x, dtype=np.float32))


def test_routed_head_selects_by_gate_hidden_and_scores_by_hidden():
    # two groups of two rows; W2 reads feature 0 for group 0 and feature 1 for group 1
    lm_W = _f32([[1, 0, 0], [0, 1, 0], [0, 0, 1], [1, 1, 1]])
    offsets = np.array([0, 2, 4], np.int32)
    rows = np.array([0, 1, 2, 3], np.int32)
    gate_W = _f32([[1, 0, 0], [0, 1, 0]])
    hidden = _f32([[3, 1, 2]])          # by itself: group 0 (3 > 1)
    gate_hidden = _f32([[0, 5, 0]])     # the router sees this: group 1
    plain = oracle.grouped(hidden, gate_W, None, lm_W, offsets, rows, 1, 2, "f32")
    assert plain.sel.tolist() == [[0]] and plain.topk_ids.tolist() == [[0, 1]]
    routed = oracle.grouped(hidden, gate_W, None, lm_W, offsets, rows, 1, 2, "f32",
                            gate_hidden=gate_hidden)
    assert routed.sel.tolist() == [[1]]
    assert routed.topk_ids.tolist() == [[3, 2]]                  # rows of group 1 only
    assert routed.topk_z.tolist() == [[6.0, 2.0]]                # logits from hidden
    assert routed.s.tolist() == [[0.0, 5.0]]                     # scores from gate_hidden
    lp = oracle.grouped_logprob(hidden, gate_W, None, lm_W, offsets, rows, 1, 2, "f32",
                                gate_hidden=gate_hidden)
    log_router = 5.0 - np.log(np.exp(0.0) + np.exp(5.0))
    lse = np.log(np.exp(6.0) + np.exp(2.0))
    assert np.allclose(lp.topk_logp, [[log_router + 6.0 - lse, log_router + 2.0 - lse]], atol=1e-14)


def test_routed_head_with_the_same_vector_is_the_plain_head():
    cfg = CONFIGS["tiny_f32"]
    head = make_head(cfg)
    h = make_hidden(cfg, 3, 1)
    a = oracle.grouped(h, head.gate_W, None, head.lm_W, head.group_offsets, head.group_rows,
                       cfg.g, cfg.k, cfg.dtype)
    b = oracle.grouped(h, head.gate_W, None, head.lm_W, head.group_offsets, head.group_rows,
                       cfg.g, cfg.k, cfg.dtype, gate_hidden=h)
    assert np.array_equal(a.sel, b.sel) and np.array_equal(a.topk_ids, b.topk_ids)
    assert np.array_equal(a.topk_z, b.topk_z) and np.array_equal(a.s, b.s)
    assert np.allclose(a.logp_router, b.logp_router, atol=1e-14)


# ---------------------------------------------------------------- draft-tree expansion
def test_tree_expand_hand_worked_level():
    # two nodes with cumulative scores -1 and -3; candidates' log-probabilities below
    parent = np.array([-1.0, -3.0], np.float32)
    ids = np.array([[11, 12, 13], [21, 22, 23]], np.int32)
    logp = np.array([[-0.5, -2.0, -4.0], [-0.25, -0.5, -9.0]], np.float32)
    # scores: node 0: -1.5, -3.0, -5.0; node 1: -3.25, -3.5, -12.0
    p, t, s = oracle.tree_expand(parent, ids, logp, 4)
    assert p.tolist() == [0, 0, 1, 1] and t.tolist() == [11, 12, 21, 22]
    assert s.tolist() == [-1.5, -3.0, -3.25, -3.5]


def test_tree_expand_ties_empty_slots_and_padding():
    ids = np.array([[5, 6], [7, -1]], np.int32)
    logp = np.array([[-1.0, -2.0], [-1.0, -0.5]], np.float32)      # (1,1) is an empty slot
    p, t, s = oracle.tree_expand(None, ids, logp, 5)
    assert p.tolist() == [0, 1, 0, -1, -1]                          # equal scores: lower node first
    assert t.tolist() == [5, 7, 6, -1, -1]
    assert s[:3].tolist() == [-1.0, -1.0, -2.0] and np.all(np.isneginf(s[3:]))


def test_tree_expand_is_a_prefix_of_the_full_sort_and_adds_in_float32():
    rng = np.random.default_rng(3)
    M, k = 7, 9
    parent = rng.standard_normal(M).astype(np.float32) * 3
    logp = -np.sort(rng.random((M, k)).astype(np.float32) * 8, axis=1)
    ids = rng.integers(0, 1000, (M, k)).astype(np.int32)
    full = oracle.tree_expand(parent, ids, logp, M * k)
    assert np.all(np.diff(full[2]) <= 0)
    assert sorted(zip(full[0].tolist(), full[1].tolist())) == sorted(
        (m, int(ids[m, i])) for m in range(M) for i in range(k))
    flat = (parent[:, None] + logp).astype(np.float32).reshape(-1)
    order = np.argsort(-flat.astype(np.float64), kind="stable")
    assert np.array_equal(full[2], flat[order])
    assert np.array_equal(full[0], (order // k).astype(np.int32))
    for n in (1, 10, 20):
        part = oracle.tree_expand(parent, ids, logp, n)
        for a, b in zip(part, full):
            assert np.array_equal(a, b[:n])
    # one node, no parent score: the node's own candidates in order
    one = oracle.tree_expand(None, ids[:1], logp[:1], k)
    assert np.array_equal(one[1], ids[0]) and np.array_equal(one[2], logp[0])


# ---------------------------------------------------------------- fp16 storage
def test_f16_widening_on_known_bit_patterns_and_against_numpy():
    # 1.0, -2.0, smallest subnormal 2^-24, largest subnormal, smallest normal 2^-14, 65504, 0.1 rounded
    bits = np.array([[0x3C00, 0xC000, 0x0001, 0x03FF, 0x0400, 0x7BFF, 0x2E66]], np.uint16)
    one = np.array([[0x3C00] * 7], np.uint16)
    # gate(hidden=bits, gate_W=one-hot rows) reads the widened values back one by one
    eye = np.zeros((7, 7), np.uint16)
    np.fill_diagonal(eye, 0x3C00)
    s = oracle.gate(bits, eye, None, "f16")
    want = [1.0, -2.0, 2.0 ** -24, 1023 * 2.0 ** -24, 2.0 ** -14, 65504.0, 0.0999755859375]
    assert s[0].tolist() == want
    rng = np.random.default_rng(0)
    anyb = rng.integers(0, 0x7C00, (1, 512)).astype(np.uint16)      # all finite non-negative patterns
    anyb[0, ::2] |= 0x8000
    ref = anyb.view(np.float16).astype(np.float64)
    assert np.array_equal(oracle.widen(anyb, "f16"), ref)
    ones = np.full((1, 512), 0x3C00, np.uint16)
    assert oracle.gate(anyb, ones, None, "f16")[0, 0] == pytest.approx(float(ref.sum()), rel=1e-15)
    # rounding to storage: nearest even, checked against torch
    import torch
    x = rng.standard_normal(4096) * 3
    got = oracle.round_to_storage(x, "f16")
    t = torch.from_numpy(x.astype(np.float32)).to(torch.float16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, t)


def test_f16_head_matches_numpy_brute_force():
    cfg = HeadConfig("small_f16", "f16", 64, 480, 6, 2, (3,), 5, 41, True)
    head = make_head(cfg)
    h = make_hidden(cfg, 3, 0)
    r = oracle.grouped(h, head.gate_W, None, head.lm_W, head.group_offsets, head.group_rows,
                       cfg.g, cfg.k, "f16")
    hf = h.view(np.float16).astype(np.float64)
    gw = head.gate_W.view(np.float16).astype(np.float64)
    lw = head.lm_W.view(np.float16).astype(np.float64)
    s = hf @ gw.T
    assert np.allclose(r.s, s, rtol=0, atol=1e-12)
    for m in range(3):
        sel = np.lexsort((np.arange(cfg.G), -s[m]))[:cfg.g]
        assert r.sel[m].tolist() == sel.tolist()
        rows = np.concatenate([head.group_rows[head.group_offsets[n]:head.group_offsets[n + 1]] for n in sel])
        z = lw[rows] @ hf[m]
        order = np.lexsort((rows, -z))[:cfg.k]
        assert r.topk_ids[m].tolist() == rows[order].tolist()
        assert np.allclose(r.topk_z[m], z[order], rtol=0, atol=1e-12)
