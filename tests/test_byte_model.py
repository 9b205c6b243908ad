"""The byte model behind every roofline fraction that bench.py reports, pinned to the
numbers the paper prints (CPU only).

Table 1 gives, per model family, the hidden size d, the MLP's intermediate size, the
vocabulary V and the GEMM parameter counts of draft and target model in units of 1024^2;
the appendix paragraph "Backends" gives the bytes one token's FP16 Llama3-8B draft head
moves (1002 such units) and the time that takes at 768 GB/s (1.3 ms).  The workload
table's (H, V) and bench.py's dense_bytes / algorithmic_bytes must reproduce them.
"""
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import bench  # noqa: E402  (imports nothing that needs the GPU at module level)
from coral_inputs import CONFIGS  # noqa: E402

MI = 1024 * 1024

# Key/value projection width of the three target families (grouped-query attention:
# kv heads x head size; public model configurations, not in the paper's table).
KV_WIDTH = {"llama2_7b": 4096, "llama3_8b": 1024, "qwen25_7b": 512}
LAYERS = {"llama2_7b": 32, "llama3_8b": 32, "qwen25_7b": 28}


def read_golden(golden_dir):
    table, vals = {}, {}
    for line in open(os.path.join(golden_dir, "table1_shapes.txt")):
        p = line.split()
        if not p or line.startswith("#"):
            continue
        if len(p) == 6:
            table[p[0]] = tuple(int(x) for x in p[1:])
        elif len(p) == 2:
            vals[p[0]] = float(p[1])
    return table, vals


def test_workload_shapes_reproduce_table_1(golden_dir):
    """One decoder layer (q, o: d x d; k, v: d x kv; MLP: 3 d x intermediate) plus the
    draft model's 2d -> d input projection plus the LM head V x d is W_d; the target's
    layers plus its LM head is W_t.  Both match the table only if V x d is the head."""
    table, _ = read_golden(golden_dir)
    assert set(table) == set(KV_WIDTH)
    for name, (d, inter, V, W_d, W_t) in table.items():
        cfg = CONFIGS[name]
        assert (cfg.H, cfg.V) == (d, V)
        layer = 2 * d * d + 2 * d * KV_WIDTH[name] + 3 * d * inter
        head = cfg.V * cfg.H
        assert abs((layer + 2 * d * d + head) / MI - W_d) <= 0.5          # printed rounded
        assert abs((LAYERS[name] * layer + head) / MI - W_t) <= 0.5
    # the head's share of the draft model's parameters: what section 3.3 sets out to cut
    d, inter, V, W_d, _ = table["llama3_8b"]
    assert 0.67 < CONFIGS["llama3_8b"].V * CONFIGS["llama3_8b"].H / MI / W_d < 0.68
    d, inter, V, W_d, _ = table["llama2_7b"]
    assert 0.35 < CONFIGS["llama2_7b"].V * CONFIGS["llama2_7b"].H / MI / W_d < 0.36


def test_dense_bytes_is_the_appendix_figure(golden_dir):
    """Appendix "Backends": 1002 x 1024^2 bytes per token for the 16-bit Llama3-8B head,
    1.3 ms at 768 GB/s (binary units throughout)."""
    _, vals = read_golden(golden_dir)
    for name in ("llama3_8b", "paper_point_f16", "paper_point", "wide_tree"):
        cfg = CONFIGS[name]
        weights = bench.dense_bytes(cfg, 0)                 # no tokens: the weight term alone
        assert weights == vals["backends_llama3_head_fp16_mbytes"] * MI
        ms = weights / (vals["backends_bandwidth_gbps"] * 1024 ** 3) * 1e3
        assert round(ms, 1) == vals["backends_theoretical_ms"]
        # per token: its hidden vector in, k (id, logit) pairs out
        assert bench.dense_bytes(cfg, 3) - weights == 3 * (cfg.H * 2 + cfg.k * 8)
    assert bench.dense_bytes(CONFIGS["tiny_f32"], 0) == 8192 * 256 * 4


@pytest.mark.parametrize("name", sorted(CONFIGS))
def test_grouped_bytes_against_dense_bytes(name):
    """Every group activated: the dense head's weight bytes, plus what only the grouped head
    reads (gate matrix, row ids).  g of G groups activated by one token: that fraction of the
    weight term (section 3.3: the head is divided equally into the groups)."""
    cfg = CONFIGS[name]
    w = 4 if cfg.dtype == "f32" else 2
    all_active = bench.algorithmic_bytes(cfg, 0, cfg.G)
    assert all_active == bench.dense_bytes(cfg, 0) + cfg.G * cfg.H * w + cfg.V * 4
    one_token = bench.algorithmic_bytes(cfg, 1, cfg.g)
    fixed = cfg.G * cfg.H * w + cfg.H * w + cfg.k * 8
    assert (one_token - fixed) * cfg.G == cfg.g * (bench.dense_bytes(cfg, 0) + cfg.V * 4)
    # Table 4's best setting (16 groups, top 2) and the headline's (32 groups, top 4) both
    # read one eighth of the head for a single token
    if name in ("paper_point", "llama3_8b"):
        assert cfg.G == 8 * cfg.g
        assert abs((one_token - fixed) / bench.dense_bytes(cfg, 0) - 0.125) < 1e-3
