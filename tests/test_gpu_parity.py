"""Parity of the HIP path (through the C ABI) with the fp64 CPU oracle, on a real MI355X.

Bar: groups and ids bit-exact wherever the oracle's neighbouring values are more than
the float tolerance apart; logits within 2e-3 (bf16 storage, fp32 accumulation) or 1e-5
(fp32 storage).  The rules are in oracle/compare.py.
"""
import time

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from coral_inputs import CONFIGS, Head, HeadConfig, make_head, make_hidden, to_storage  # noqa: E402
import oracle  # noqa: E402
from oracle import compare  # noqa: E402


@pytest.fixture(scope="module")
def coral():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2502_16880_amd as c
    return c


class DeviceHead:
    def __init__(self, coral, head: Head):
        c = head.cfg
        self.head = head
        self.gate_W = coral.device_tensor(head.gate_W, c.dtype)
        self.lm_W = coral.device_tensor(head.lm_W, c.dtype)
        self.bias = None if head.gate_bias is None else torch.from_numpy(head.gate_bias).cuda()
        self.gi = coral.GroupIndex(head.group_offsets, head.group_rows)


def run_grouped(coral, dh: DeviceHead, hidden, g, k):
    c = dh.head.cfg
    d_hidden = coral.device_tensor(hidden, c.dtype)
    ids, logits, sel = coral.coral_lmhead_grouped(d_hidden, dh.gate_W, dh.bias, dh.lm_W, dh.gi, g, k)
    torch.cuda.synchronize()
    return ids.cpu().numpy(), logits.cpu().numpy(), sel.cpu().numpy()


def run_dense(coral, dh: DeviceHead, hidden, k):
    c = dh.head.cfg
    d_hidden = coral.device_tensor(hidden, c.dtype)
    ids, logits = coral.coral_lmhead_dense(d_hidden, dh.lm_W, k)
    torch.cuda.synchronize()
    return ids.cpu().numpy(), logits.cpu().numpy()


# Second tier, beside the comparator's pass/fail tolerances: what the kernels' arithmetic
# should achieve (products of 16-bit values are exact in fp32, sums are fp32 over lane-split
# partial sums: errors of about 1e-6 on logits of size <= 6).  A dropped term of size 1e-4 or
# a log-sum-exp off by 1e-3 passes the comparator's tolerance but not these.
TIGHT_LOGIT_ERR = {"bf16": 2e-5, "f16": 2e-5, "f32": 1e-5}
TIGHT_LOGP_ERR = {"bf16": 5e-5, "f16": 5e-5, "f32": 2.2e-5}


def check_grouped(dh, hidden, g, k, out):
    h = dh.head
    rep = compare.check_grouped(hidden, h.gate_W, h.gate_bias, h.lm_W, h.group_offsets,
                                h.group_rows, g, k, h.cfg.dtype, *out)
    assert rep.max_abs_err <= TIGHT_LOGIT_ERR[h.cfg.dtype], rep.max_abs_err
    return rep


def run_logprob(coral, dh: DeviceHead, hidden, g, k):
    c = dh.head.cfg
    d_hidden = coral.device_tensor(hidden, c.dtype)
    ids, logp, sel = coral.coral_lmhead_grouped_logprob(d_hidden, dh.gate_W, dh.bias, dh.lm_W, dh.gi, g, k)
    torch.cuda.synchronize()
    return ids.cpu().numpy(), logp.cpu().numpy(), sel.cpu().numpy()


def check_logprob(dh, hidden, g, k, out):
    h = dh.head
    rep = compare.check_grouped_logprob(hidden, h.gate_W, h.gate_bias, h.lm_W, h.group_offsets,
                                        h.group_rows, g, k, h.cfg.dtype, *out)
    assert rep.max_abs_err <= TIGHT_LOGP_ERR[h.cfg.dtype], rep.max_abs_err
    return rep


def check_dense(dh, hidden, k, out, tokens=None):
    h = dh.head
    rep = compare.check_dense(hidden, h.lm_W, k, h.cfg.dtype, *out, tokens=tokens)
    assert rep.max_abs_err <= TIGHT_LOGIT_ERR[h.cfg.dtype], rep.max_abs_err
    return rep


# ------------------------------------------------------------------ small and medium cases
SCALED = [
    # (config, M values): same recipe as the workload table at sizes the oracle does in
    # seconds; group sizes leave a ragged last chunk of rows and span many workgroups
    (CONFIGS["tiny_f32"], (4,)),
    (CONFIGS["llama2_7b"].scaled(V=16 * 250), (1, 4, 8)),
    (CONFIGS["llama3_8b"].scaled(V=32 * 203), (1, 4, 8, 16)),
    (CONFIGS["qwen25_7b"].scaled(V=32 * 297), (1, 8, 16)),
    (CONFIGS["wide_tree"].scaled(V=64 * 126), (64,)),
    (CONFIGS["paper_point"].scaled(V=16 * 375), (1, 10)),          # contiguous groups
    # fp16 storage on each of the three paths (single launch with all three gates, tiles,
    # multi-kernel: H = 4160 does not fit eight wave loads)
    (CONFIGS["llama3_8b"].scaled(name="llama3_f16", dtype="f16", V=32 * 203), (1, 4, 8, 16)),
    (CONFIGS["wide_tree"].scaled(name="wide_tree_f16", dtype="f16", V=64 * 126), (64,)),
    (CONFIGS["llama3_8b"].scaled(name="llama3_f16_h4160", dtype="f16", V=32 * 203, H=4160), (8,)),
]


@pytest.mark.parametrize("cfg,Ms", SCALED, ids=lambda x: x.name if isinstance(x, HeadConfig) else None)
def test_scaled_configs_grouped_and_dense(coral, cfg, Ms):
    dh = DeviceHead(coral, make_head(cfg))
    for M in Ms:
        for batch in (0, 1):
            hidden = make_hidden(cfg, M, batch)
            print(f"case {cfg.name} M={M} batch={batch}", flush=True)
            rep = check_grouped(dh, hidden, cfg.g, cfg.k, run_grouped(coral, dh, hidden, cfg.g, cfg.k))
            assert rep.tokens == M
            rep = check_dense(dh, hidden, cfg.k, run_dense(coral, dh, hidden, cfg.k))
            assert rep.tokens == M


@pytest.mark.parametrize("cfg,Ms", SCALED, ids=lambda x: x.name if isinstance(x, HeadConfig) else None)
def test_scaled_configs_logprob(coral, cfg, Ms):
    """Eq. 8's probability composition against the oracle, same shapes as above."""
    dh = DeviceHead(coral, make_head(cfg))
    for M in Ms:
        hidden = make_hidden(cfg, M, 2)
        print(f"case {cfg.name} M={M} log-prob", flush=True)
        rep = check_logprob(dh, hidden, cfg.g, cfg.k, run_logprob(coral, dh, hidden, cfg.g, cfg.k))
        assert rep.tokens == M


def test_logprob_edge_shapes(coral):
    """One group (a plain log-softmax), all groups active (probabilities of the whole
    vocabulary), ragged and single-row groups, two runs bit-identical."""
    cfg = HeadConfig("lp1", "f32", 64, 300, 1, 1, (3,), 9, 95, False)
    dh = DeviceHead(coral, make_head(cfg))
    hidden = make_hidden(cfg, 3)
    check_logprob(dh, hidden, 1, 9, run_logprob(coral, dh, hidden, 1, 9))
    cfg = HeadConfig("lpG", "bf16", 256, 6 * 111, 6, 6, (5,), 12, 96, True, bias_std=1.0)
    dh = DeviceHead(coral, make_head(cfg))
    hidden = make_hidden(cfg, 5)
    a = run_logprob(coral, dh, hidden, 6, 12)
    check_logprob(dh, hidden, 6, 12, a)
    b = run_logprob(coral, dh, hidden, 6, 12)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    sizes = [1, 31, 5, 32, 33, 500, 64, 7]
    V = sum(sizes)
    cfg = HeadConfig("lprag", "f32", 128, V, len(sizes), 3, (6,), 4, 97, False)
    rng = np.random.default_rng(97)
    perm = rng.permutation(V).astype(np.int32)
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    rows = np.concatenate([np.sort(perm[offsets[n]:offsets[n + 1]]) for n in range(len(sizes))])
    lm_W = rng.standard_normal((V, cfg.H)).astype(np.float32) * np.float32(0.05)
    gate_W = rng.standard_normal((len(sizes), cfg.H)).astype(np.float32) * np.float32(0.05)
    dh = DeviceHead(coral, Head(cfg, lm_W, gate_W, None, offsets, rows.astype(np.int32)))
    hidden = make_hidden(cfg, 6)
    check_logprob(dh, hidden, 3, 4, run_logprob(coral, dh, hidden, 3, 4))


LOGPROB_PATH_CASES = [
    # single-launch kernel: up to 64 activated groups with workgroups of their own
    (HeadConfig("lp64", "bf16", 256, 64 * 37, 64, 2, (32,), 4, 98, True, bias_std=0.5), 1),
    # ... every group active for every token (the probabilities of the whole vocabulary)
    (HeadConfig("lpall", "bf16", 512, 16 * 300, 16, 16, (4,), 10, 99, True), 1),
    # ... fp16 storage, contiguous groups, more candidates than a group's workgroups
    (HeadConfig("lpf16", "f16", 1024, 8 * 4000, 8, 2, (7,), 33, 102, True, grouping="contiguous"), 1),
    # tile path: 64 tokens do not fit the single-launch kernel; ragged last blocks, a second
    # token tile only partly used, fp16
    (CONFIGS["wide_tree"].scaled(V=64 * 300), 2),
    (HeadConfig("lptile40", "bf16", 2048, 16 * 777, 16, 5, (40,), 12, 104, True, bias_std=1.0), 2),
    (HeadConfig("lptilef16", "f16", 2048, 10 * 333, 10, 4, (33,), 16, 105, True), 2),
    # multi-kernel path: more than 64 groups can be active; more than 16 groups per token
    (HeadConfig("lpmany", "f32", 128, 128 * 20, 128, 4, (20,), 8, 100, False), 0),
    (HeadConfig("lpg17", "f32", 128, 64 * 20, 64, 17, (2,), 8, 101, False), 0),
]


@pytest.mark.parametrize("cfg,path", LOGPROB_PATH_CASES, ids=lambda x: x.name if isinstance(x, HeadConfig) else None)
def test_logprob_on_both_paths(coral, cfg, path):
    M = cfg.Ms[0]
    dt = {"f32": coral.CORAL_F32, "bf16": coral.CORAL_BF16, "f16": coral.CORAL_F16}[cfg.dtype]
    assert coral.coral_lmhead_logprob_path(M, cfg.H, cfg.V, cfg.G, cfg.g, cfg.k, dt) == path
    dh = DeviceHead(coral, make_head(cfg))
    for batch in (0, 1):
        hidden = make_hidden(cfg, M, batch)
        print(f"case {cfg.name} M={M} batch={batch} log-prob path {path}", flush=True)
        rep = check_logprob(dh, hidden, cfg.g, cfg.k, run_logprob(coral, dh, hidden, cfg.g, cfg.k))
        assert rep.tokens == M


def test_logprob_with_empty_and_tiny_groups(coral):
    """Groups without rows can be selected (their log-sum-exp is -inf and they offer no
    candidate); a group smaller than its share of workgroups leaves workgroups idle."""
    sizes = [0, 40, 0, 50, 3, 64, 5, 900]
    V = sum(sizes)
    cfg = HeadConfig("lpempty", "f32", 128, V, len(sizes), 3, (6,), 3, 103, False)
    rng = np.random.default_rng(103)
    perm = rng.permutation(V).astype(np.int32)
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    rows = np.concatenate([np.sort(perm[offsets[n]:offsets[n + 1]]) for n in range(len(sizes))])
    lm_W = rng.standard_normal((V, cfg.H)).astype(np.float32) * np.float32(0.05)
    gate_W = rng.standard_normal((len(sizes), cfg.H)).astype(np.float32) * np.float32(0.05)
    bias = np.array([2.0, 0, 1.5, 0, 0.5, 0, 0.5, 0], np.float32)    # the empty groups do get chosen
    dh = DeviceHead(coral, Head(cfg, lm_W, gate_W, bias, offsets, rows.astype(np.int32)))
    assert coral.coral_lmhead_logprob_path(6, cfg.H, V, len(sizes), 3, 3, coral.CORAL_F32) == 1
    hidden = make_hidden(cfg, 6)
    out = run_logprob(coral, dh, hidden, 3, 3)
    assert np.isin(out[2], [0, 2]).any()
    check_logprob(dh, hidden, 3, 3, out)


@pytest.mark.parametrize("dtype,H", [("bf16", 8), ("bf16", 264), ("bf16", 1032), ("f32", 4),
                                     ("f32", 260), ("f32", 1028)])
def test_hidden_sizes_that_do_not_fill_a_wave(coral, dtype, H):
    cfg = HeadConfig(f"h{H}", dtype, H, 12 * 70, 12, 3, (5,), 6, 40 + H, dtype == "bf16")
    dh = DeviceHead(coral, make_head(cfg))
    hidden = make_hidden(cfg, 5)
    check_grouped(dh, hidden, cfg.g, cfg.k, run_grouped(coral, dh, hidden, cfg.g, cfg.k))
    check_dense(dh, hidden, cfg.k, run_dense(coral, dh, hidden, cfg.k))


@pytest.mark.parametrize("M,g,k", [(1, 1, 1), (1, 8, 64), (64, 1, 64), (3, 8, 5), (64, 8, 1),
                                   (7, 2, 33)])
def test_extreme_m_g_k(coral, M, g, k):
    cfg = HeadConfig("ext", "bf16", 512, 8 * 130, 8, g, (M,), k, 77, True, bias_std=1.0)
    dh = DeviceHead(coral, make_head(cfg))
    hidden = make_hidden(cfg, M)
    check_grouped(dh, hidden, g, k, run_grouped(coral, dh, hidden, g, k))
    check_dense(dh, hidden, k, run_dense(coral, dh, hidden, k))


@pytest.mark.parametrize("M", [4, 9])
def test_all_groups_active_equals_dense_on_device(coral, M):
    cfg = HeadConfig("gG", "bf16", 1024, 6 * 111, 6, 6, (M,), 12, 78, True)
    dh = DeviceHead(coral, make_head(cfg))
    hidden = make_hidden(cfg, M)
    gi, gz, _ = run_grouped(coral, dh, hidden, 6, 12)
    di, dz = run_dense(coral, dh, hidden, 12)
    same_kernels = (coral.coral_lmhead_path(False, M, cfg.H, cfg.V, 6, 6, 12, coral.CORAL_BF16)
                    == coral.coral_lmhead_path(True, M, cfg.H, cfg.V, 0, 0, 12, coral.CORAL_BF16))
    assert np.array_equal(gi, di)
    if same_kernels:                      # same kernels, same summation order: same bits
        assert np.array_equal(gz, dz)
    else:                                 # vector units vs matrix cores: fp32 rounding differs
        assert M == 9 and np.max(np.abs(gz - dz)) < 1e-5


@pytest.mark.parametrize("dtype,M", [("f32", 3), ("bf16", 1), ("bf16", 9)])
def test_collected_candidates_beyond_one_wave(coral, dtype, M):
    """Groups so long that a workgroup meets three of its 16-pair windows per token: about
    96 rows per (workgroup, token), more than one candidate per lane in the final ranking,
    still within the 128 the host's bound allows (four groups, every one selected)."""
    cfg = HeadConfig("collect96", dtype, 64, 4 * 5000, 4, 4, (M,), 12, 120 + M, dtype != "f32")
    dh = DeviceHead(coral, make_head(cfg))
    for batch in (0, 1):
        hidden = make_hidden(cfg, M, batch)
        print(f"case {cfg.name} {dtype} M={M} batch={batch}", flush=True)
        check_grouped(dh, hidden, cfg.g, cfg.k, run_grouped(coral, dh, hidden, cfg.g, cfg.k))
    # one group more per token and the bound is exceeded: per-wave lists take over, same results
    cfg5 = HeadConfig("lists160", dtype, 64, 5 * 4000, 5, 5, (M,), 12, 130 + M, dtype != "f32")
    dh = DeviceHead(coral, make_head(cfg5))
    hidden = make_hidden(cfg5, M, 0)
    check_grouped(dh, hidden, cfg5.g, cfg5.k, run_grouped(coral, dh, hidden, cfg5.g, cfg5.k))


def test_every_path_is_exercised(coral):
    """The scaled and full-size cases above cover all three kernel paths."""
    P = coral.coral_lmhead_path
    B = coral.CORAL_BF16
    assert P(False, 16, 4096, 32 * 203, 32, 4, 10, B) == 1          # scaled Llama3: single launch
    assert P(False, 64, 4096, 64 * 126, 64, 8, 16, B) == 2          # scaled wide tree: tiles
    assert P(True, 16, 4096, 32 * 203, 0, 0, 10, B) == 1            # dense, small vocabulary
    assert P(True, 16, 4096, 128256, 0, 0, 10, B) == 2              # dense, full size: tiles
    assert P(False, 64, 2048, 16 * 300, 16, 6, 20, B) == 2          # test_tile_path_shapes
    assert P(False, 64, 512, 16 * 300, 16, 6, 16, B) == 2
    assert P(False, 64, 512, 8 * 130, 8, 1, 64, B) == 2             # extreme k: tiles as well
    assert P(False, 8, 4160, 32 * 203, 32, 4, 10, coral.CORAL_F16) == 0   # H = 4160: multi-kernel path


@pytest.mark.parametrize("H,k", [(2048, 20), (512, 16), (1024, 21)])
def test_tile_path_shapes(coral, H, k):
    """Matrix-core path away from the benchmark shapes: one, two and four 512-column chunks,
    groups of 300 rows (two whole 128-row blocks and a ragged one), popular groups with
    one to four token tiles (gate bias)."""
    cfg = HeadConfig("tiles", "bf16", H, 16 * 300, 16, 6, (64,), k, 90 + k, True, bias_std=1.5)
    assert coral.coral_lmhead_path(False, 64, H, cfg.V, 16, 6, k, coral.CORAL_BF16) == 2
    dh = DeviceHead(coral, make_head(cfg))
    for batch in range(2):
        hidden = make_hidden(cfg, 64, batch)
        check_grouped(dh, hidden, 6, k, run_grouped(coral, dh, hidden, 6, k))
    for M in (17, 40, 64):                                # two, three and four token tiles
        hidden = make_hidden(cfg, M, 7)
        if coral.coral_lmhead_path(False, M, H, cfg.V, 16, 16, k, coral.CORAL_BF16) == 2:
            check_grouped(dh, hidden, 16, k, run_grouped(coral, dh, hidden, 16, k))


def test_ragged_and_empty_groups(coral):
    """Any partition is accepted: groups of 1, 31, 32, 33 and 500 rows and an empty one."""
    sizes = [1, 31, 0, 32, 33, 500, 64, 7]
    V = sum(sizes)
    cfg = HeadConfig("rag", "f32", 128, V, len(sizes), 3, (6,), 4, 79, False)
    rng = np.random.default_rng(79)
    perm = rng.permutation(V).astype(np.int32)
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    rows = np.concatenate([np.sort(perm[offsets[n]:offsets[n + 1]]) for n in range(len(sizes))])
    lm_W = rng.standard_normal((V, cfg.H)).astype(np.float32) * np.float32(0.02)
    gate_W = rng.standard_normal((len(sizes), cfg.H)).astype(np.float32) * np.float32(0.02)
    head = Head(cfg, lm_W, gate_W, None, offsets, rows.astype(np.int32))
    dh = DeviceHead(coral, head)
    for batch in range(4):
        hidden = make_hidden(cfg, 6, batch)
        # the host check is on the g smallest groups: 0 + 1 + 7 = 8 rows >= k = 4
        check_grouped(dh, hidden, 3, 4, run_grouped(coral, dh, hidden, 3, 4))
    with pytest.raises(coral.CoralError):                 # 0 + 1 rows < k
        run_grouped(coral, dh, make_hidden(cfg, 6), 2, 4)


@pytest.mark.parametrize("seed", list(range(200, 264)) + list(range(300, 348)) + list(range(400, 420)))
def test_random_small_heads(coral, seed):
    """Seeded random shapes with ragged groups (some empty, some of one row): token counts,
    group counts, g and k drawn freely within the limits, fp32 heads so that the oracle is
    fast.  Logit ranking, log-probabilities (twice: they must repeat) and the dense head."""
    rng = np.random.default_rng(seed)
    G = int(rng.integers(1, 65))
    g = int(rng.integers(1, min(G, 16) + 1))
    M = int(rng.integers(1, 25))
    dtype = "f32" if seed < 300 else ("bf16", "f16")[seed % 2]  # 16-bit: matrix-core gate from 4 tokens on
    H = int(rng.choice([32, 64, 100, 256, 516] if dtype == "f32" else [64, 104, 256, 512]))
    if seed >= 400:                                             # many tokens x long rows: the tile path
        M, H = int(rng.integers(41, 65)), 2048
    sizes = rng.integers(0, 120, G)
    sizes[rng.integers(0, G)] += int(rng.integers(100, 2000))     # one large group
    if G > 3:
        sizes[rng.integers(0, G, 2)] = (0, 1)
    min_cand = int(np.sort(sizes)[:g].sum())
    while min_cand < 1:                                           # the g smallest must hold a row
        sizes[np.argsort(sizes)[0]] += 1
        min_cand = int(np.sort(sizes)[:g].sum())
    k = int(rng.integers(1, min(min_cand, 20) + 1))
    V = int(sizes.sum())
    cfg = HeadConfig(f"rand{seed}", dtype, H, V, G, g, (M,), k, seed, bool(rng.integers(0, 2)))
    perm = rng.permutation(V).astype(np.int32)
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    rows = np.concatenate([np.sort(perm[offsets[n]:offsets[n + 1]]) for n in range(G)]).astype(np.int32)
    lm_W = to_storage(rng.standard_normal((V, H)).astype(np.float32) * np.float32(0.05), dtype)
    gate_W = to_storage(rng.standard_normal((G, H)).astype(np.float32) * np.float32(0.05), dtype)
    bias = (rng.standard_normal(G) * 0.3).astype(np.float32) if rng.integers(0, 2) else None
    dh = DeviceHead(coral, Head(cfg, lm_W, gate_W, bias, offsets, rows))
    hidden = make_hidden(cfg, M, 1)
    dt = {"f32": coral.CORAL_F32, "bf16": coral.CORAL_BF16, "f16": coral.CORAL_F16}[dtype]
    print(f"case seed={seed} {dtype} M={M} H={H} V={V} G={G} g={g} k={k} "
          f"logprob path {coral.coral_lmhead_logprob_path(M, H, V, G, g, k, dt)}", flush=True)
    check_grouped(dh, hidden, g, k, run_grouped(coral, dh, hidden, g, k))
    out = run_logprob(coral, dh, hidden, g, k)
    check_logprob(dh, hidden, g, k, out)
    again = run_logprob(coral, dh, hidden, g, k)
    assert all(np.array_equal(x, y) for x, y in zip(out, again))
    check_dense(dh, hidden, k, run_dense(coral, dh, hidden, k))


@pytest.mark.parametrize("seed", list(range(500, 540)))
def test_random_tile_path_heads(coral, seed):
    """Seeded random shapes, most of them on the matrix-core path: 17 to 64 tokens, up to 160 ragged groups
    (more than 64: the gate kernel's general selection), a group of several thousand rows
    (its candidates take several chunks of the ranking kernel), k up to 64, with and without
    bias; both output modes where the log-probability mode takes this path."""
    rng = np.random.default_rng(seed)
    G = int(rng.integers(1, 161)) if seed % 3 == 0 else int(rng.integers(1, 65))
    g = int(rng.integers(1, min(G, 24) + 1))
    M = int(rng.integers(17, 65))
    H = int(rng.choice([512, 1024, 2048]))
    dtype = ("bf16", "f16")[seed % 2]
    sizes = rng.integers(0, 200, G)
    sizes[rng.integers(0, G)] += int(rng.integers(1000, 6000))    # one large group
    if G > 3:
        sizes[rng.integers(0, G, 2)] = (0, 1)
    min_cand = int(np.sort(sizes)[:g].sum())
    while min_cand < 1:                                           # the g smallest must hold a row
        sizes[np.argsort(sizes)[0]] += 1
        min_cand = int(np.sort(sizes)[:g].sum())
    k = int(rng.integers(1, min(min_cand, 64) + 1))
    V = int(sizes.sum())
    cfg = HeadConfig(f"tile{seed}", dtype, H, V, G, g, (M,), k, seed, True, bias_std=float(rng.choice([0.3, 2.0])))
    perm = rng.permutation(V).astype(np.int32)
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    rows = np.concatenate([np.sort(perm[offsets[n]:offsets[n + 1]]) for n in range(G)]).astype(np.int32)
    lm_W = to_storage(rng.standard_normal((V, H)).astype(np.float32) * np.float32(0.05), dtype)
    gate_W = to_storage(rng.standard_normal((G, H)).astype(np.float32) * np.float32(0.05), dtype)
    bias = (rng.standard_normal(G) * cfg.bias_std).astype(np.float32) if rng.integers(0, 2) else None
    dt = {"bf16": coral.CORAL_BF16, "f16": coral.CORAL_F16}[dtype]
    path = coral.coral_lmhead_path(False, M, H, V, G, g, k, dt)      # 2 for two in three of the seeds
    dh = DeviceHead(coral, Head(cfg, lm_W, gate_W, bias, offsets, rows))
    hidden = make_hidden(cfg, M, 1)
    lp_path = coral.coral_lmhead_logprob_path(M, H, V, G, g, k, dt)
    print(f"case seed={seed} {dtype} M={M} H={H} V={V} G={G} g={g} k={k} path {path} logprob path {lp_path}", flush=True)
    check_grouped(dh, hidden, g, k, run_grouped(coral, dh, hidden, g, k))
    if lp_path == 2:
        out = run_logprob(coral, dh, hidden, g, k)
        check_logprob(dh, hidden, g, k, out)
        again = run_logprob(coral, dh, hidden, g, k)
        assert all(np.array_equal(x, y) for x, y in zip(out, again))


def test_duplicate_rows_tie_break_to_the_lower_id(coral):
    cfg = HeadConfig("dup", "bf16", 256, 4 * 96, 4, 4, (2,), 6, 80, True)
    head = make_head(cfg)
    hidden = make_hidden(cfg, 2)
    dh0 = DeviceHead(coral, head)
    ids0, _ = run_dense(coral, dh0, hidden, 1)
    best = int(ids0[0, 0])
    twins = [(best + 97) % cfg.V, (best + 211) % cfg.V]
    for t in twins:
        head.lm_W[t] = head.lm_W[best]
    dh = DeviceHead(coral, head)
    ids, z = run_dense(coral, dh, hidden, 6)
    assert ids[0, :3].tolist() == sorted([best] + twins) and z[0, 0] == z[0, 1] == z[0, 2]
    check_dense(dh, hidden, 6, (ids, z))
    out = run_grouped(coral, dh, hidden, 4, 6)
    assert out[0][0, :3].tolist() == sorted([best] + twins)
    check_grouped(dh, hidden, 4, 6, out)


def test_equal_gate_scores_select_the_lower_group(coral):
    cfg = HeadConfig("gt", "f32", 64, 8 * 40, 8, 3, (4,), 5, 81, False)
    head = make_head(cfg)
    head.gate_W[5] = head.gate_W[2]
    head.gate_W[7] = head.gate_W[2]
    dh = DeviceHead(coral, head)
    hidden = make_hidden(cfg, 4)
    out = run_grouped(coral, dh, hidden, 3, 5)
    rep = check_grouped(dh, hidden, 3, 5, out)
    assert rep.forced_tokens == 0                          # identical rows: identical fp32 scores
    for row in out[2].tolist():                            # 2 before 5 before 7 whenever present
        pos = [row.index(n) for n in (2, 5, 7) if n in row]
        assert pos == sorted(pos)


@pytest.mark.parametrize("g", [3, 20])
def test_equal_gate_scores_on_the_tile_path(coral, g):
    """The tile path's selection (rounds of a wave maximum up to 16 groups per token, rank
    counting beyond): equal scores go to the lower group, for all 64 tokens."""
    cfg = HeadConfig("gt_tiles", "bf16", 512, 32 * 140, 32, g, (64,), 16, 83, True, bias_std=1.0)
    assert coral.coral_lmhead_path(False, 64, cfg.H, cfg.V, cfg.G, g, cfg.k, coral.CORAL_BF16) == 2
    head = make_head(cfg)
    head.gate_bias[4] += 2.0                               # (popular: many tokens select the three)
    for twin in (9, 30):
        head.gate_W[twin] = head.gate_W[4]
        head.gate_bias[twin] = head.gate_bias[4]
    dh = DeviceHead(coral, head)
    hidden = make_hidden(cfg, 64)
    out = run_grouped(coral, dh, hidden, g, cfg.k)
    rep = check_grouped(dh, hidden, g, cfg.k, out)
    assert rep.forced_tokens == 0                          # identical rows: identical fp32 scores
    seen = 0
    for row in out[2].tolist():                            # 4 before 9 before 30 whenever present
        pos = [row.index(n) for n in (4, 9, 30) if n in row]
        assert pos == sorted(pos)
        seen += len(pos) > 1
    assert seen > 0


@pytest.mark.parametrize("M,V", [(9, 65536 + 77), (33, 65536 + 128 + 1)])
def test_dense_head_on_the_tile_path_with_a_ragged_last_block(coral, M, V):
    """The dense head takes the tile path from 8 tokens and 65536 rows on; the configured
    vocabularies are multiples of the 128-row block, these are not (77 rows, one row)."""
    cfg = HeadConfig("dense_ragged", "bf16", 512, V, 1, 1, (M,), 12, 140 + M, False)
    assert coral.coral_lmhead_path(True, M, cfg.H, V, 0, 0, cfg.k, coral.CORAL_BF16) == 2
    dh = DeviceHead(coral, make_head(cfg))
    hidden = make_hidden(cfg, M)
    hidden[0] = hidden[1]                                  # two tokens with the same lists
    # the last rows must be reachable: make one of them every token's best
    w = oracle.widen(dh.head.lm_W, "bf16")
    mean = oracle.widen(hidden, "bf16").mean(axis=0)
    w[V - 1] = (3.0 / (mean @ mean)) * mean              # logits of about 2 to 6 there, 2 elsewhere at most
    dh.head.lm_W[:] = oracle.round_to_storage(w, "bf16")
    dh = DeviceHead(coral, dh.head)
    ids, z = run_dense(coral, dh, hidden, cfg.k)
    assert (ids[:, 0] == V - 1).sum() >= M // 2
    check_dense(dh, hidden, cfg.k, (ids, z))


def test_equal_logits_on_the_tile_path(coral):
    """All-zero hidden vectors: every logit is 0.0, so every block's largest logit reaches the
    bound, all 2048 candidates of the first chunk pass it (more than one per thread: the
    second bound from the waves' best keys takes over) and every later candidate loses to the
    list by its id.  Dense (k = 64, a thousand blocks per token) and grouped (the gate sees
    only its bias: all 64 tokens select the same groups, four token tiles each)."""
    cfg = HeadConfig("dense_zero", "bf16", 512, 65536, 1, 1, (8,), 64, 131, False)
    assert coral.coral_lmhead_path(True, 8, cfg.H, cfg.V, 0, 0, cfg.k, coral.CORAL_BF16) == 2
    dh = DeviceHead(coral, make_head(cfg))
    hidden = np.zeros_like(make_hidden(cfg, 8))
    ids, z = run_dense(coral, dh, hidden, cfg.k)
    assert (ids == np.arange(cfg.k)[None, :]).all() and (z == 0.0).all()
    check_dense(dh, hidden, cfg.k, (ids, z))
    wide = CONFIGS["wide_tree"].scaled(V=64 * 126)
    assert coral.coral_lmhead_path(False, 64, wide.H, wide.V, wide.G, wide.g, wide.k, coral.CORAL_BF16) == 2
    dh = DeviceHead(coral, make_head(wide))
    hidden = np.zeros_like(make_hidden(wide, 64))
    out = run_grouped(coral, dh, hidden, wide.g, wide.k)
    assert (out[1] == 0.0).all() and (out[2] == out[2][0]).all()
    check_grouped(dh, hidden, wide.g, wide.k, out)


def test_two_runs_are_bit_identical(coral):
    cfg = CONFIGS["llama3_8b"].scaled(V=32 * 203)
    dh = DeviceHead(coral, make_head(cfg))
    hidden = make_hidden(cfg, 16)
    a = run_grouped(coral, dh, hidden, cfg.g, cfg.k)
    b = run_grouped(coral, dh, hidden, cfg.g, cfg.k)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    a = run_dense(coral, dh, hidden, cfg.k)
    b = run_dense(coral, dh, hidden, cfg.k)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))


@pytest.mark.parametrize("M", [1, 8, 16])
def test_logprob_runs_are_bit_identical(coral, M):
    """The log-sum-exp of a group is a sum over thousands of rows taken by waves that draw
    their work dynamically, and the router's scores are computed by every workgroup for
    itself: neither may show in the result."""
    cfg = CONFIGS["llama3_8b"].scaled(V=32 * 203)
    dh = DeviceHead(coral, make_head(cfg))
    hidden = make_hidden(cfg, M, 4)
    first = run_logprob(coral, dh, hidden, cfg.g, cfg.k)
    for rep in range(8):
        again = run_logprob(coral, dh, hidden, cfg.g, cfg.k)
        assert all(np.array_equal(x, y) for x, y in zip(first, again)), rep


def test_caller_buffers_and_streams(coral):
    """Outputs land in the caller's tensors, on the caller's stream; the workspace is reusable."""
    cfg = CONFIGS["tiny_f32"]
    dh = DeviceHead(coral, make_head(cfg))
    hidden = make_hidden(cfg, 4)
    d_hidden = coral.device_tensor(hidden, "f32")
    ws = coral.alloc_workspace(4, cfg.H, cfg.V, cfg.G, cfg.g, cfg.k, coral.CORAL_F32)
    ws.fill_(0xAB)                                         # stale contents ...
    coral.coral_lmhead_workspace_init(ws)                  # ... are fine once it is prepared
    ids = torch.full((4, cfg.k), -7, dtype=torch.int32, device="cuda")
    z = torch.zeros((4, cfg.k), device="cuda")
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        for _ in range(3):
            r = coral.coral_lmhead_grouped(d_hidden, dh.gate_W, None, dh.lm_W, dh.gi, cfg.g, cfg.k,
                                           topk_ids=ids, topk_logits=z, workspace=ws)
    st.synchronize()
    assert r[0] is ids and r[1] is z
    check_grouped(dh, hidden, cfg.g, cfg.k, (ids.cpu().numpy(), z.cpu().numpy(), r[2].cpu().numpy()))
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(coral.CoralError) as e:
        coral.coral_lmhead_dense(d_hidden, dh.lm_W, cfg.k, workspace=small)
    assert e.value.status == 5


@pytest.mark.parametrize("name,M", [("llama2_7b_scaled", 8), ("tiny_f32", 4), ("wide_tree_scaled", 64),
                                    ("staged_f16", 8)])
def test_measurement_entry_points_time_the_kernel_and_change_nothing(coral, name, M):
    """The *_profiled variants return what the plain calls return, bit for bit, and the two
    events they bind to the weight-streaming kernel read a plausible duration: positive, and
    no longer than the whole call takes between two synchronisations."""
    cfg = {"llama2_7b_scaled": CONFIGS["llama2_7b"].scaled(name="llama2_s", V=16 * 250),
           "tiny_f32": CONFIGS["tiny_f32"],
           "wide_tree_scaled": CONFIGS["wide_tree"].scaled(name="wide_s", V=64 * 130),
           "staged_f16": CONFIGS["llama3_8b"].scaled(name="l3_h4160", dtype="f16", V=32 * 203, H=4160)}[name]
    dh = DeviceHead(coral, make_head(cfg))
    d_hidden = coral.device_tensor(make_hidden(cfg, M), cfg.dtype)
    plain = coral.coral_lmhead_grouped(d_hidden, dh.gate_W, dh.bias, dh.lm_W, dh.gi, cfg.g, cfg.k)
    dense_plain = coral.coral_lmhead_dense(d_hidden, dh.lm_W, cfg.k)
    torch.cuda.synchronize()
    for which in ("grouped", "dense"):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(), b.record()                             # creates the handles
        torch.cuda.synchronize()
        for rep in range(2):                               # the second call is warm
            t0 = time.perf_counter()
            if which == "grouped":
                out = coral.coral_lmhead_grouped(d_hidden, dh.gate_W, dh.bias, dh.lm_W, dh.gi, cfg.g, cfg.k,
                                                 events=(a.cuda_event, b.cuda_event))
            else:
                out = coral.coral_lmhead_dense(d_hidden, dh.lm_W, cfg.k, events=(a.cuda_event, b.cuda_event))
            torch.cuda.synchronize()
            wall_ms = (time.perf_counter() - t0) * 1e3
        kernel_ms = a.elapsed_time(b)
        assert 0.0 < kernel_ms <= wall_ms, (which, kernel_ms, wall_ms)
        for x, y in zip(out, plain if which == "grouped" else dense_plain):
            assert torch.equal(x, y), which


def test_probe_read_runs_and_times_itself(coral):
    """The read-only yardstick kernel: launches, leaves its source alone, and its events read
    a duration that grows with the bytes."""
    src = torch.arange(1 << 30, dtype=torch.uint8, device="cuda")     # (far beyond the last-level cache)
    keep = src.clone()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(), b.record()
    torch.cuda.synchronize()
    times = []
    for nbytes in (1 << 20, 1 << 30):
        for _ in range(3):
            coral.coral_probe_read(src, nbytes, 16, (a.cuda_event, b.cuda_event))
            torch.cuda.synchronize()
        times.append(a.elapsed_time(b))
    assert 0.0 < times[0] < times[1]
    assert torch.equal(src, keep)
    with pytest.raises(coral.CoralError):
        coral.coral_probe_read(src, 1000, 16, (a.cuda_event, b.cuda_event))


def test_prepared_call_is_the_plain_call(coral):
    """PreparedGrouped marshals once and enters the same entry point: same results, bit for
    bit, also on another stream and in the log-probability mode."""
    cfg = CONFIGS["llama2_7b"].scaled(name="llama2_s", V=16 * 250)
    dh = DeviceHead(coral, make_head(cfg))
    d_hidden = coral.device_tensor(make_hidden(cfg, 8), cfg.dtype)
    ws = coral.alloc_workspace(8, cfg.H, cfg.V, cfg.G, cfg.g, cfg.k, coral.CORAL_BF16)
    for logprob in (False, True):
        plain = coral.coral_lmhead_grouped(d_hidden, dh.gate_W, dh.bias, dh.lm_W, dh.gi, cfg.g, cfg.k,
                                           workspace=ws, logprob=logprob)
        torch.cuda.synchronize()
        plain = [t.clone() for t in plain]
        prep = coral.PreparedGrouped(d_hidden, dh.gate_W, dh.bias, dh.lm_W, dh.gi, cfg.g, cfg.k, ws,
                                     logprob=logprob)
        prep()
        st = torch.cuda.Stream()
        st.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(st):
            out = prep()
        st.synchronize()
        for x, y in zip(out, plain):
            assert torch.equal(x, y)
    with pytest.raises(ValueError):
        coral.PreparedGrouped(d_hidden, dh.gate_W, dh.bias, dh.lm_W, dh.gi, cfg.g, cfg.k, None)


def test_many_calls_on_one_workspace_stay_consistent(coral):
    """The single-launch path hands partial lists between workgroups through memory and
    re-arms its counters itself: 300 back-to-back calls on one workspace, alternating two
    inputs, must reproduce the first results bit for bit."""
    cfg = CONFIGS["llama3_8b"].scaled(V=32 * 1003)
    dh = DeviceHead(coral, make_head(cfg))
    for M in (1, 8):
        hs = [coral.device_tensor(make_hidden(cfg, M, b), cfg.dtype) for b in (0, 1)]
        ws = coral.alloc_workspace(M, cfg.H, cfg.V, cfg.G, cfg.g, cfg.k, coral.CORAL_BF16)
        first = []
        for h in hs:
            r = coral.coral_lmhead_grouped(h, dh.gate_W, None, dh.lm_W, dh.gi, cfg.g, cfg.k, workspace=ws)
            torch.cuda.synchronize()
            first.append([x.clone() for x in r])
        outs = []
        for i in range(300):
            ids = torch.empty((M, cfg.k), dtype=torch.int32, device="cuda")
            z = torch.empty((M, cfg.k), device="cuda")
            sel = torch.empty((M, cfg.g), dtype=torch.int32, device="cuda")
            coral.coral_lmhead_grouped(hs[i % 2], dh.gate_W, None, dh.lm_W, dh.gi, cfg.g, cfg.k,
                                       topk_ids=ids, topk_logits=z, sel_groups=sel, workspace=ws)
            outs.append((ids, z, sel))
        torch.cuda.synchronize()
        for i, o in enumerate(outs):
            for got, want in zip(o, first[i % 2]):
                assert torch.equal(got, want), f"call {i} (M={M}) differs from the first result"


def test_hip_graph_replays_match_eager(coral):
    """Captured once, replayed several times with eager work in between: every replay must
    give the eager result (the library records kernels only, no memset nodes)."""
    cfg = CONFIGS["llama3_8b"].scaled(V=32 * 501)
    dh = DeviceHead(coral, make_head(cfg))
    M = 4
    hidden = make_hidden(cfg, M)
    d_hidden = coral.device_tensor(hidden, cfg.dtype)
    ws = coral.alloc_workspace(M, cfg.H, cfg.V, cfg.G, cfg.g, cfg.k, coral.CORAL_BF16)
    ids = torch.empty((M, cfg.k), dtype=torch.int32, device="cuda")
    z = torch.empty((M, cfg.k), device="cuda")
    sel = torch.empty((M, cfg.g), dtype=torch.int32, device="cuda")

    def call():
        coral.coral_lmhead_grouped(d_hidden, dh.gate_W, None, dh.lm_W, dh.gi, cfg.g, cfg.k,
                                   topk_ids=ids, topk_logits=z, sel_groups=sel, workspace=ws)
        coral.coral_lmhead_dense(d_hidden, dh.lm_W, cfg.k, workspace=ws)

    call()
    torch.cuda.synchronize()
    want = (ids.clone(), z.clone(), sel.clone())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for rep in range(4):
        ids.fill_(-1), z.zero_(), sel.fill_(-1)             # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(ids, want[0]) and torch.equal(z, want[1]) and torch.equal(sel, want[2]), rep
    check_grouped(dh, hidden, cfg.g, cfg.k, (ids.cpu().numpy(), z.cpu().numpy(), sel.cpu().numpy()))


@pytest.mark.parametrize("M", [1, 4, 64])
def test_hip_graph_replays_of_the_logprob_head(coral, M):
    """The log-probability mode keeps several counters in the workspace (one per activated
    group with 4 tokens, one in all with 1 token; the tile path's block queue with 64): every
    replay, and an eager call after the replays, must find them as the first call did."""
    cfg = CONFIGS["llama3_8b"].scaled(V=32 * 501) if M < 64 else CONFIGS["wide_tree"].scaled(V=64 * 300)
    dh = DeviceHead(coral, make_head(cfg))
    hidden = make_hidden(cfg, M, 3)
    d_hidden = coral.device_tensor(hidden, cfg.dtype)
    assert coral.coral_lmhead_logprob_path(M, cfg.H, cfg.V, cfg.G, cfg.g, cfg.k,
                                           coral.CORAL_BF16) == (1 if M < 64 else 2)
    ws = coral.alloc_workspace(M, cfg.H, cfg.V, cfg.G, cfg.g, cfg.k, coral.CORAL_BF16)
    ids = torch.empty((M, cfg.k), dtype=torch.int32, device="cuda")
    lp = torch.empty((M, cfg.k), device="cuda")
    sel = torch.empty((M, cfg.g), dtype=torch.int32, device="cuda")

    def call():
        coral.coral_lmhead_grouped_logprob(d_hidden, dh.gate_W, dh.bias, dh.lm_W, dh.gi, cfg.g, cfg.k,
                                           topk_ids=ids, topk_logits=lp, sel_groups=sel, workspace=ws)

    call()
    torch.cuda.synchronize()
    want = (ids.clone(), lp.clone(), sel.clone())
    check_logprob(dh, hidden, cfg.g, cfg.k, tuple(x.cpu().numpy() for x in want))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
        call()
    for rep in range(3):
        ids.fill_(-1), lp.zero_(), sel.fill_(-1)            # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(ids, want[0]) and torch.equal(lp, want[1]) and torch.equal(sel, want[2]), rep
    ids.fill_(-1)
    call()
    torch.cuda.synchronize()
    assert torch.equal(ids, want[0]) and torch.equal(lp, want[1])


def test_nan_inputs_do_not_fault(coral):
    """Results are unspecified for NaN inputs, but every path must finish and stay in range."""
    for cfg, M in ((CONFIGS["tiny_f32"], 4), (CONFIGS["llama2_7b"].scaled(V=16 * 250), 12),
                   (CONFIGS["wide_tree"].scaled(V=64 * 126), 64)):
        head = make_head(cfg)
        hidden = make_hidden(cfg, M)
        if cfg.dtype == "f32":
            hidden[0, 3] = np.nan
            head.gate_W[1, 5] = np.nan
        else:
            hidden[0, 3] = 0x7FC0
            head.gate_W[1, 5] = 0x7FC0
        dh = DeviceHead(coral, head)
        ids, z, sel = run_grouped(coral, dh, hidden, cfg.g, cfg.k)
        assert np.all((sel >= 0) & (sel < cfg.G))
        assert np.all(ids[1:] >= 0) and np.all(ids[1:] < cfg.V)   # tokens without NaN are intact
        run_dense(coral, dh, hidden, cfg.k)
        ids, _, sel = run_logprob(coral, dh, hidden, cfg.g, cfg.k)
        assert np.all((sel >= 0) & (sel < cfg.G))


# ------------------------------------------------------------------ full-size workloads
FULL = [("llama2_7b", (1, 4, 8)), ("llama3_8b", (1, 4, 8, 16)), ("qwen25_7b", (1, 8, 16)),
        ("wide_tree", (64,)), ("paper_point", (1, 10)), ("paper_point_permuted", (1, 10)),
        ("paper_point_f16", (10,))]


@pytest.mark.parametrize("name,Ms", FULL)
def test_full_size_workloads(coral, name, Ms):
    """The benchmark's shapes and launch configuration.  The grouped head is compared in
    full (the oracle needs g*v rows per token); the dense head on sampled tokens."""
    cfg = CONFIGS[name]
    print(f"generating {name}", flush=True)
    dh = DeviceHead(coral, make_head(cfg))
    for M in Ms:
        hidden = make_hidden(cfg, M)
        print(f"case {name} M={M} grouped", flush=True)
        rep = check_grouped(dh, hidden, cfg.g, cfg.k, run_grouped(coral, dh, hidden, cfg.g, cfg.k))
        print(f"  exact {rep.exact_tokens}/{rep.tokens} forced {rep.forced_tokens} "
              f"max|err| {rep.max_abs_err:.2e}", flush=True)
        assert rep.tokens == M
        print(f"case {name} M={M} dense", flush=True)
        toks = sorted({0, M - 1})
        rep = check_dense(dh, hidden, cfg.k, run_dense(coral, dh, hidden, cfg.k), tokens=toks)
        print(f"  dense exact {rep.exact_tokens}/{rep.tokens} max|err| {rep.max_abs_err:.2e}",
              flush=True)
        print(f"case {name} M={M} log-prob", flush=True)
        out = run_logprob(coral, dh, hidden, cfg.g, cfg.k)
        rep = check_logprob(dh, hidden, cfg.g, cfg.k, out)
        print(f"  log-prob exact {rep.exact_tokens}/{rep.tokens} max|err| {rep.max_abs_err:.2e}",
              flush=True)
        again = run_logprob(coral, dh, hidden, cfg.g, cfg.k)    # (pieces through memory at M=16; tile path at M=64)
        assert all(np.array_equal(x, y) for x, y in zip(out, again))
    del dh
    torch.cuda.empty_cache()


# ------------------------------------------------------------------ router pre-mix (Eq. 7) and routed head
PREMIX_SHAPES = [
    # (dtype, H, M): one pair of rows per wave, several token batches, a ragged last pair,
    # a row longer than one pass of 8 segments, and the workload's own width
    ("f32", 256, 4), ("bf16", 512, 1), ("bf16", 1000, 9), ("bf16", 4104, 3), ("f32", 2052, 17),
    ("bf16", 4096, 16),
    # matrix-core kernel: fewer tokens than a tile, several ragged token batches, LDS that
    # only fits part of a tile's tokens, fewer lines than waves, more than one batch of lines
    ("bf16", 4096, 5), ("bf16", 4096, 40), ("bf16", 8192, 16), ("bf16", 192, 20), ("bf16", 4480, 4),
    ("f16", 4096, 16), ("f16", 1000, 3), ("f16", 4096, 1),
    # more than 16 tokens, H a multiple of 512 up to 4096: token vectors staged in chunks for
    # two, three and four token tiles (40 tokens at H = 4096 is in the list above); one chunk;
    # fp16
    ("bf16", 4096, 64), ("bf16", 4096, 17), ("bf16", 1024, 33), ("bf16", 512, 64), ("f16", 2048, 48),
]


@pytest.mark.parametrize("dtype,H,M", PREMIX_SHAPES)
def test_router_premix(coral, dtype, H, M):
    from coral_inputs import make_router_W1
    cfg = HeadConfig(f"premix_{dtype}_{H}", dtype, H, 64, 2, 1, (M,), 4, 31, True)
    W1 = make_router_W1(cfg)
    hidden = make_hidden(cfg, M, 0)
    d_W1 = coral.device_tensor(W1, dtype)
    d_h = coral.device_tensor(hidden, dtype)
    for act in ("silu", "relu", "identity"):
        print(f"case premix {dtype} H={H} M={M} act={act}", flush=True)
        u = coral.coral_router_premix(d_h, d_W1, act)
        torch.cuda.synchronize()
        raw = u.cpu().numpy() if dtype == "f32" else u.view(torch.int16).cpu().numpy().view(np.uint16)
        rep = compare.check_premix(hidden, W1, dtype, act, raw)
        assert rep.tokens == M


def test_router_premix_rejects_bad_arguments(coral):
    cfg = HeadConfig("premix_bad", "bf16", 256, 64, 2, 1, (2,), 4, 32, True)
    from coral_inputs import make_router_W1
    d_W1 = coral.device_tensor(make_router_W1(cfg), "bf16")
    d_h = coral.device_tensor(make_hidden(cfg, 2, 0), "bf16")
    with pytest.raises(coral.CoralError):                      # in place: u_out overlaps hidden
        coral.coral_router_premix(d_h, d_W1, "silu", out=d_h)
    with pytest.raises(ValueError):
        coral.coral_router_premix(d_h, d_W1, "tanh")


ROUTED = [
    (CONFIGS["tiny_f32"], (4,)),
    (CONFIGS["llama3_8b"].scaled(name="llama3_f16", dtype="f16", V=32 * 203), (8,)),
    (CONFIGS["llama3_8b"].scaled(V=32 * 203), (1, 4, 8, 16)),     # single-launch path, all three gates
    (CONFIGS["wide_tree"].scaled(V=64 * 126), (64,)),             # tile path
    (CONFIGS["llama3_8b"].scaled(V=32 * 203, H=4160), (8,)),      # multi-kernel path
]


@pytest.mark.parametrize("cfg,Ms", ROUTED, ids=lambda x: x.name if isinstance(x, HeadConfig) else None)
def test_routed_head_gate_sees_another_vector(coral, cfg, Ms):
    dh = DeviceHead(coral, make_head(cfg))
    h = dh.head
    for M in Ms:
        hidden = make_hidden(cfg, M, 0)
        gate_hidden = make_hidden(cfg, M, 7)                   # independent of hidden
        d_h = coral.device_tensor(hidden, cfg.dtype)
        d_gh = coral.device_tensor(gate_hidden, cfg.dtype)
        for logprob in (False, True):
            print(f"case routed {cfg.name} M={M} logprob={logprob}", flush=True)
            ids, out, sel = coral.coral_lmhead_grouped(d_h, dh.gate_W, dh.bias, dh.lm_W, dh.gi, cfg.g,
                                                       cfg.k, logprob=logprob, gate_hidden=d_gh)
            torch.cuda.synchronize()
            res = (ids.cpu().numpy(), out.cpu().numpy(), sel.cpu().numpy())
            check = compare.check_grouped_logprob if logprob else compare.check_grouped
            rep = check(hidden, h.gate_W, h.gate_bias, h.lm_W, h.group_offsets, h.group_rows, cfg.g,
                        cfg.k, cfg.dtype, *res, gate_hidden=gate_hidden)
            assert rep.tokens == M
        # NULL gate_hidden is the plain head
        a = coral.coral_lmhead_grouped(d_h, dh.gate_W, dh.bias, dh.lm_W, dh.gi, cfg.g, cfg.k)
        b = coral.coral_lmhead_grouped(d_h, dh.gate_W, dh.bias, dh.lm_W, dh.gi, cfg.g, cfg.k, gate_hidden=d_h)
        torch.cuda.synchronize()
        for x, y in zip(a, b):
            assert torch.equal(x, y)


def test_premix_then_routed_head_end_to_end(coral):
    """The paper's router as a chain of two calls: u = act(W1 h) + h, then W2 on u (Eq. 7).
    Checked link by link with the plain tolerances: the device's u against the oracle's u,
    then the head against the oracle whose router reads that same, verified, device u."""
    from coral_inputs import make_router_W1
    cfg = CONFIGS["llama3_8b"].scaled(V=32 * 203)
    dh = DeviceHead(coral, make_head(cfg))
    h = dh.head
    W1 = make_router_W1(cfg)
    d_W1 = coral.device_tensor(W1, cfg.dtype)
    M = 8
    hidden = make_hidden(cfg, M, 3)
    d_h = coral.device_tensor(hidden, cfg.dtype)
    d_u = coral.coral_router_premix(d_h, d_W1, "silu")
    ids, z, sel = coral.coral_lmhead_grouped(d_h, dh.gate_W, dh.bias, dh.lm_W, dh.gi, cfg.g, cfg.k,
                                             gate_hidden=d_u)
    torch.cuda.synchronize()
    u_dev = np.ascontiguousarray(d_u.view(torch.int16).cpu().numpy().view(np.uint16))
    compare.check_premix(hidden, W1, cfg.dtype, "silu", u_dev)
    rep = compare.check_grouped(hidden, h.gate_W, h.gate_bias, h.lm_W, h.group_offsets, h.group_rows,
                                cfg.g, cfg.k, cfg.dtype, ids.cpu().numpy(), z.cpu().numpy(),
                                sel.cpu().numpy(), gate_hidden=u_dev)
    assert rep.tokens == M and rep.max_abs_err <= TIGHT_LOGIT_ERR[cfg.dtype]


# ------------------------------------------------------------------ draft-tree expansion
TREE_SHAPES = [
    # (M, k, n_next): the root level, the paper's operating point (10 candidates per node, 60
    # nodes in the tree), a full sort, the largest level, lists longer than n_next
    (1, 10, 10), (10, 10, 10), (10, 10, 60), (8, 10, 80), (64, 64, 64), (64, 64, 4096), (60, 16, 7),
]


@pytest.mark.parametrize("M,k,n_next", TREE_SHAPES)
def test_tree_expand_is_bit_exact(coral, M, k, n_next):
    rng = np.random.default_rng(1000 * M + k)
    for case in range(3):
        print(f"case tree M={M} k={k} n_next={n_next} #{case}", flush=True)
        parent = (rng.standard_normal(M) * 2 - 3).astype(np.float32)
        logp = -np.sort(rng.random((M, k)).astype(np.float32) * 6, axis=1)
        ids = rng.integers(0, 128256, (M, k)).astype(np.int32)
        if case == 1:                       # ties across nodes and empty slots at list ends
            logp = np.round(logp * 2) / 2
            parent = np.round(parent)
            ids[rng.random((M, k)) < 0.1] = -1
            ids = np.where(np.cumsum(ids < 0, axis=1) > 0, -1, ids).astype(np.int32)
        use_parent = case != 2 or M == 1
        out = coral.coral_tree_expand(torch.from_numpy(parent).cuda() if use_parent else None,
                                      torch.from_numpy(ids).cuda(), torch.from_numpy(logp).cuda(), n_next)
        torch.cuda.synchronize()
        ref = oracle.tree_expand(parent if use_parent else None, ids, logp, n_next)
        for name, a, b in zip(("parent", "token", "score"), out, ref):
            assert np.array_equal(a.cpu().numpy(), b), f"{name}: {a.cpu().numpy()} vs {b}"


def test_tree_expand_after_the_logprob_head(coral):
    """Two calls chained on the device.  The expansion's inputs here are the device head's
    outputs, which are not oracle inputs, so this checks properties that hold for any input:
    scores non-increasing, every kept node is a candidate of its parent with the parent's
    score added, nothing better was left out.  (Exactness of the expansion itself is the test
    above; of the head, the log-probability parity tests.)"""
    cfg = CONFIGS["llama3_8b"].scaled(V=32 * 203)
    dh = DeviceHead(coral, make_head(cfg))
    M, n_next = 8, 10
    hidden = make_hidden(cfg, M, 5)
    ids, logp, _ = coral.coral_lmhead_grouped_logprob(coral.device_tensor(hidden, cfg.dtype), dh.gate_W,
                                                      dh.bias, dh.lm_W, dh.gi, cfg.g, cfg.k)
    parent = torch.linspace(-2.0, -0.25, M, device="cuda")
    p, t, s = (x.cpu().numpy() for x in coral.coral_tree_expand(parent, ids, logp, n_next))
    torch.cuda.synchronize()
    ids_h, logp_h, parent_h = ids.cpu().numpy(), logp.cpu().numpy(), parent.cpu().numpy()
    assert np.all(np.diff(s) <= 0)
    all_scores = (parent_h[:, None] + logp_h).astype(np.float32)
    for r in range(n_next):
        pos = np.where(ids_h[p[r]] == t[r])[0]
        assert len(pos) == 1 and all_scores[p[r], pos[0]] == s[r]
    assert np.sum(all_scores > s[-1]) <= n_next - 1
    with pytest.raises(coral.CoralError):
        coral.coral_tree_expand(parent, ids, logp, M * cfg.k + 1)


DRAFT_LEVEL_CASES = [
    # (config, M, n_next, parent scores?, expected log-probability path)
    (CONFIGS["llama3_8b"].scaled(V=32 * 203), 8, 10, True, 1),        # a group's last workgroup finishes it
    (CONFIGS["llama3_8b"].scaled(V=32 * 203), 1, 10, False, 1),       # root level: the last workgroup alone
    (CONFIGS["llama3_8b"].scaled(V=32 * 203), 16, 7, True, 1),        # fewer nodes kept than candidates per node
    (CONFIGS["paper_point"].scaled(V=16 * 501), 10, 10, True, 1),
    (CONFIGS["tiny_f32"], 4, 32, True, 1),                            # every candidate kept (n_next = M k)
    (CONFIGS["llama2_7b"].scaled(H=1024, V=16 * 250, k=40), 20, 64, True, 1),  # lists of 40, 20 nodes
    (CONFIGS["wide_tree"].scaled(V=64 * 126), 64, 64, True, 2),       # tile path: one more launch
    (CONFIGS["wide_tree"].scaled(H=4160, V=64 * 126), 64, 20, True, 0),   # staged path: one more launch
]


@pytest.mark.parametrize("cfg,M,n_next,with_parent,path", DRAFT_LEVEL_CASES,
                         ids=lambda x: x.name if isinstance(x, HeadConfig) else None)
def test_draft_level_is_the_head_followed_by_the_expansion(coral, cfg, M, n_next, with_parent, path):
    """coral_lmhead_draft_level against the two calls it stands for, bit for bit (the head
    against the oracle as well; the expansion kernel has its own exact test above)."""
    dt = {"f32": coral.CORAL_F32, "bf16": coral.CORAL_BF16, "f16": coral.CORAL_F16}[cfg.dtype]
    assert coral.coral_lmhead_logprob_path(M, cfg.H, cfg.V, cfg.G, cfg.g, cfg.k, dt) == path
    dh = DeviceHead(coral, make_head(cfg))
    hidden = make_hidden(cfg, M, 4)
    d_hidden = coral.device_tensor(hidden, cfg.dtype)
    parent = torch.linspace(-3.0, -0.5, M, device="cuda") if with_parent else None
    ws = coral.alloc_workspace(M, cfg.H, cfg.V, cfg.G, cfg.g, cfg.k, dt)
    for rep in range(2):                                   # the second call finds the counters reset
        print(f"case {cfg.name} M={M} n_next={n_next} call {rep}", flush=True)
        ids, logp, sel, p, t, s = coral.coral_lmhead_draft_level(
            d_hidden, dh.gate_W, dh.bias, dh.lm_W, dh.gi, cfg.g, cfg.k, n_next, parent_score=parent,
            workspace=ws)
        ids2, logp2, sel2 = coral.coral_lmhead_grouped_logprob(d_hidden, dh.gate_W, dh.bias, dh.lm_W,
                                                               dh.gi, cfg.g, cfg.k, workspace=ws)
        p2, t2, s2 = coral.coral_tree_expand(parent, ids2, logp2, n_next)
        torch.cuda.synchronize()
        for a, b in ((ids, ids2), (logp, logp2), (sel, sel2), (p, p2), (t, t2), (s, s2)):
            assert torch.equal(a, b)
    check_logprob(dh, hidden, cfg.g, cfg.k, (ids.cpu().numpy(), logp.cpu().numpy(), sel.cpu().numpy()))


def test_draft_level_rejects_bad_arguments(coral):
    cfg = CONFIGS["tiny_f32"]
    dh = DeviceHead(coral, make_head(cfg))
    d_hidden = coral.device_tensor(make_hidden(cfg, 4), cfg.dtype)
    for n_next in (0, 4 * cfg.k + 1):
        with pytest.raises(coral.CoralError):
            coral.coral_lmhead_draft_level(d_hidden, dh.gate_W, dh.bias, dh.lm_W, dh.gi, cfg.g, cfg.k,
                                           n_next)
    with pytest.raises(ValueError):
        coral.coral_lmhead_draft_level(d_hidden, dh.gate_W, dh.bias, dh.lm_W, dh.gi, cfg.g, cfg.k, 8,
                                       parent_score=torch.zeros(3, device="cuda"))

