"""Host-side checks of the C ABI (no GPU): the library loads, exports every symbol
the header declares, and rejects bad arguments before anything is enqueued."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2502_16880_amd as coral

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "coral_lmhead.h")

OK, NULL, SHAPE, GROUP_INDEX, UNSUPPORTED, WORKSPACE, HIP = range(7)
F32, BF16 = 0, 1
FAKE = 0x7000_0000_1000          # never dereferenced: every check below fails before a launch


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(coral_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"coral_lmhead_grouped", "coral_lmhead_dense", "coral_lmhead_workspace_bytes",
            "coral_lmhead_workspace_init", "coral_lmhead_grouped_profiled",
            "coral_lmhead_dense_profiled",
            "coral_group_index_validate", "coral_status_string"} <= set(names)
    lib = ctypes.CDLL(coral.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in the header but not exported"


def test_probe_read_checks_its_arguments_on_the_host():
    L = coral._L
    assert L.coral_probe_read(None, 16384, 16, None, 1, 1) == 1               # CORAL_ERR_NULL
    assert L.coral_probe_read(4096, 16384, 16, None, None, 1) == 1
    assert L.coral_probe_read(4096, 1000, 16, None, 1, 1) == 2                # CORAL_ERR_SHAPE
    assert L.coral_probe_read(4096, 16384, 17, None, 1, 1) == 2
    assert L.coral_probe_read(4100, 16384, 16, None, 1, 1) == 4               # CORAL_ERR_UNSUPPORTED


def test_status_strings():
    seen = {coral.coral_status_string(i) for i in range(7)}
    assert len(seen) == 7 and coral.coral_status_string(0) == "ok"
    assert "unknown" in coral.coral_status_string(99)


def test_group_index_validate():
    L = coral._L
    off = np.array([0, 3, 6], dtype=np.int32)
    rows = np.array([5, 0, 2, 1, 4, 3], dtype=np.int32)
    v = lambda o, r, G, V: L.coral_group_index_validate(o.ctypes.data, r.ctypes.data, G, V)
    assert v(off, rows, 2, 6) == OK
    assert L.coral_group_index_validate(None, rows.ctypes.data, 2, 6) == NULL
    assert v(off, rows, 0, 6) == SHAPE
    bad = rows.copy(); bad[0] = 0
    assert v(off, bad, 2, 6) == GROUP_INDEX            # id 0 twice, id 5 missing
    bad = rows.copy(); bad[1] = 6
    assert v(off, bad, 2, 6) == GROUP_INDEX            # id out of range
    assert v(np.array([0, 4, 3], np.int32), rows, 2, 6) == GROUP_INDEX   # not ascending / end != V
    assert v(np.array([1, 3, 6], np.int32), rows, 2, 6) == GROUP_INDEX
    ragged = np.array([0, 1, 6], dtype=np.int32)       # ragged groups are a valid partition
    assert v(ragged, rows, 2, 6) == OK


def test_path_selection_covers_the_three_paths():
    path = coral.coral_lmhead_path
    assert path(False, 1, 4096, 128256, 32, 4, 10, BF16) == 1      # Llama3 shape, one token
    assert path(False, 16, 4096, 128256, 32, 4, 10, BF16) == 1
    assert path(False, 64, 4096, 128256, 64, 8, 16, BF16) == 2     # wide tree: hidden exceeds LDS
    assert path(True, 16, 4096, 128256, 0, 0, 10, BF16) == 2       # dense, many tokens
    assert path(True, 8, 4096, 32000, 0, 0, 10, BF16) == 1         # ... but a small vocabulary
    assert path(False, 64, 4160, 128256, 64, 8, 16, BF16) == 0     # H not a multiple of 512
    assert path(True, 1, 4096, 128256, 0, 0, 10, BF16) == 1
    assert path(False, 64, 512, 1040, 8, 1, 64, BF16) == 2         # k = 64 on the tile path too
    assert path(False, 4, 256, 8192, 16, 2, 8, F32) == 1
    assert path(True, 64, 4096, 8192, 0, 0, 8, F32) == 0           # fp32 rows longer than 8 KB
    assert path(True, 64, 8192, 8192, 0, 0, 8, F32) == -1          # ... than the staged path's LDS
    assert path(False, 65, 256, 8192, 16, 2, 8, F32) == -1


def test_logprob_path_selection():
    lp = coral.coral_lmhead_logprob_path
    assert lp(1, 4096, 128256, 32, 4, 10, BF16) == 1               # Llama3 shape
    assert lp(16, 4096, 128256, 32, 4, 10, BF16) == 1
    assert lp(16, 3584, 152064, 32, 4, 10, BF16) == 1              # Qwen shape
    assert lp(64, 4096, 128256, 64, 8, 16, BF16) == 2              # wide tree: hidden exceeds LDS
    assert lp(64, 4160, 128256, 64, 8, 16, BF16) == 0              # ... and H not a multiple of 512
    assert lp(64, 4096, 128256, 128, 8, 16, BF16) == 0             # tile path ranks 64 groups at most
    assert lp(20, 256, 8192, 128, 4, 8, F32) == 0                  # 80 groups may be active
    assert lp(2, 256, 8192, 64, 17, 8, F32) == 0                   # 17 lists per token
    assert lp(65, 256, 8192, 16, 2, 8, F32) == -1


def test_workspace_init_rejects_bad_arguments():
    L = coral._L
    assert L.coral_lmhead_workspace_init(None, 4096, None) == WORKSPACE
    assert L.coral_lmhead_workspace_init(FAKE + 8, 4096, None) == WORKSPACE
    assert L.coral_lmhead_workspace_init(FAKE, 16, None) == WORKSPACE


def test_workspace_bytes():
    wb = coral.coral_lmhead_workspace_bytes
    a = wb(1, 4096, 128256, 32, 4, 10, BF16)
    b = wb(16, 4096, 128256, 32, 4, 10, BF16)
    assert 0 < a < b
    assert wb(4, 256, 8192, 0, 0, 8, F32) > 0          # dense
    assert wb(0, 256, 8192, 16, 2, 8, F32) == 0
    assert wb(4, 256, 8192, 16, 0, 8, F32) == 0        # G without g
    assert wb(4, 256, 8192, 4, 5, 8, F32) == 0         # g > G
    assert b % 256 == 0
    # shapes that can take the matrix-core path carry its logits buffer, 512 B per (128-row
    # block, token) with V / 128 + G + 1 blocks; shapes that cannot (one token; fp32) do not
    z_wide = (128256 // 128 + 64 + 1) * 64 * 512
    assert wb(64, 4096, 128256, 64, 8, 16, BF16) - wb(64, 4096, 128256, 64, 8, 16, F32) >= z_wide
    # (the dense head takes that path from 8 tokens on: a workspace for 8 tokens serves it too)
    assert wb(8, 4096, 128256, 32, 4, 10, BF16) - wb(7, 4096, 128256, 32, 4, 10, BF16) >= (128256 // 128 + 32 + 1) * 8 * 512


class Call:
    """A grouped call with plausible arguments; tests override one at a time."""

    def __init__(self):
        self.G, self.v = 16, 512
        self.off = (np.arange(self.G + 1) * self.v).astype(np.int32)
        self.a = dict(hidden=FAKE, gate_W=FAKE + 0x100000, gate_bias=None, lm_W=FAKE + 0x200000,
                      M=4, H=256, V=8192, g=2, k=8, dt=F32, ids=FAKE + 0x300000,
                      logits=FAKE + 0x400000, sel=None, ws=FAKE + 0x500000, ws_bytes=1 << 30)
        self.gi = coral._GroupIndexStruct(self.G, self.off.ctypes.data, FAKE + 0x600000,
                                          FAKE + 0x700000)

    def grouped(self, gi="default", **kw):
        a = dict(self.a, **kw)
        gip = ctypes.byref(self.gi) if gi == "default" else gi
        return coral._L.coral_lmhead_grouped(a["hidden"], a["gate_W"], a["gate_bias"], a["lm_W"],
                                             gip, a["M"], a["H"], a["V"], a["g"], a["k"], a["dt"],
                                             a["ids"], a["logits"], a["sel"], a["ws"],
                                             a["ws_bytes"], None)

    def dense(self, **kw):
        a = dict(self.a, **kw)
        return coral._L.coral_lmhead_dense(a["hidden"], a["lm_W"], a["M"], a["H"], a["V"], a["k"],
                                           a["dt"], a["ids"], a["logits"], a["ws"], a["ws_bytes"],
                                           None)


@pytest.mark.parametrize("kw,want", [
    (dict(hidden=None), NULL), (dict(gate_W=None), NULL), (dict(lm_W=None), NULL),
    (dict(ids=None), NULL), (dict(logits=None), NULL),
    (dict(M=0), SHAPE), (dict(k=0), SHAPE), (dict(g=0), SHAPE), (dict(g=17), SHAPE),
    (dict(dt=7), SHAPE), (dict(V=8191), GROUP_INDEX),
    (dict(M=65), UNSUPPORTED), (dict(k=65), UNSUPPORTED),
    (dict(H=254), UNSUPPORTED), (dict(H=260, dt=BF16), UNSUPPORTED),
    (dict(hidden=FAKE + 8), UNSUPPORTED), (dict(lm_W=FAKE + 4), UNSUPPORTED),
    (dict(gate_W=FAKE + 2), UNSUPPORTED),
    (dict(ws=None), WORKSPACE), (dict(ws=FAKE + 64), WORKSPACE), (dict(ws_bytes=1024), WORKSPACE),
])
def test_grouped_rejects_bad_arguments_before_any_launch(kw, want):
    assert Call().grouped(**kw) == want


def test_grouped_group_index_errors():
    c = Call()
    assert c.grouped(gi=None) == NULL
    c.gi.group_rows = None
    assert c.grouped() == NULL
    c = Call()
    c.off[3] = c.off[2] - 1                            # descending offsets
    assert c.grouped() == GROUP_INDEX
    c = Call()
    c.gi.G = 2000
    assert c.grouped(g=2) in (UNSUPPORTED, SHAPE)
    c = Call()
    c.off[0] = 1
    assert c.grouped() == GROUP_INDEX


def test_k_larger_than_the_candidate_count():
    c = Call()
    c.off[:] = [0, 3, 6] + list(range(7, 7 + 13)) + [8192]    # two groups of 3 rows, many of 1
    assert c.grouped(g=2, k=3) == SHAPE                # the two smallest groups hold 2 rows
    assert c.grouped(g=2, k=2, ws=None) == WORKSPACE   # k = 2 passes that check


@pytest.mark.parametrize("kw,want", [
    (dict(hidden=None), NULL), (dict(lm_W=None), NULL), (dict(ids=None), NULL),
    (dict(M=0), SHAPE), (dict(k=0), SHAPE), (dict(V=4, k=8), SHAPE),
    (dict(M=65), UNSUPPORTED), (dict(k=65), UNSUPPORTED), (dict(H=258), UNSUPPORTED),
    (dict(ws=None), WORKSPACE), (dict(ws_bytes=16), WORKSPACE),
])
def test_dense_rejects_bad_arguments_before_any_launch(kw, want):
    assert Call().dense(**kw) == want


def test_binding_rejects_host_tensors_and_mixed_dtypes():
    import torch
    h = torch.zeros(2, 64)
    with pytest.raises(ValueError):
        coral.coral_lmhead_dense(h, torch.zeros(128, 64), 4,
                                 topk_ids=torch.zeros(2, 4, dtype=torch.int32),
                                 topk_logits=torch.zeros(2, 4),
                                 workspace=torch.zeros(1 << 20, dtype=torch.uint8))
    with pytest.raises(TypeError):
        coral.coral_lmhead_dense(h, torch.zeros(128, 64, dtype=torch.bfloat16), 4)
    with pytest.raises(TypeError):
        coral.coral_lmhead_dense(h.double(), torch.zeros(128, 64).double(), 4)


def test_rows_too_long_for_every_path_are_refused_before_any_launch():
    """A shape that only the staged path could take (H no multiple of 512) and whose batch of
    eight token vectors does not fit LDS: the path query says -1 and the call returns
    UNSUPPORTED with nothing enqueued (the fake pointers would fault otherwise)."""
    path, lp = coral.coral_lmhead_path, coral.coral_lmhead_logprob_path
    assert path(False, 8, 10248, 8192, 16, 2, 8, BF16) == -1
    assert path(True, 8, 10248, 8192, 0, 0, 8, BF16) == -1
    assert lp(8, 10248, 8192, 16, 2, 8, BF16) == -1
    assert path(False, 4, 10248, 8192, 16, 2, 8, BF16) == 0        # four token vectors do fit
    assert path(False, 8, 10240, 8192, 16, 2, 8, BF16) == 2        # whole 512-column chunks: tiles
    c = Call()
    assert c.grouped(M=8, H=10248, dt=BF16) == UNSUPPORTED
    assert c.dense(M=8, H=10248, dt=BF16) == UNSUPPORTED


def test_control_words_do_not_overlap(tmp_path):
    """The kernels' arrival counters and queues share the first words of the workspace; the
    map (csrc/control_words.h) is compiled here with the host compiler and checked: entries
    disjoint, inside the area that coral_lmhead_workspace_init zeroes, and the workspace of
    every shape at least that large."""
    import subprocess
    src = tmp_path / "ctrl.cpp"
    src.write_text('#include <cstdio>\n#include "control_words.h"\n'
                   'int main() { std::printf("words %d\\n", coral_ctrl::kWords);\n'
                   '  for (int i = 0; i < coral_ctrl::kMapEntries; ++i)\n'
                   '    std::printf("%s %d %d\\n", coral_ctrl::kMap[i].name, coral_ctrl::kMap[i].first_word,\n'
                   '                coral_ctrl::kMap[i].n_words);\n  return 0; }\n')
    exe = tmp_path / "ctrl"
    subprocess.run(["g++", "-std=c++17", "-I", os.path.join(ROOT, "paper_2502_16880_amd", "csrc"),
                    str(src), "-o", str(exe)], check=True)
    lines = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    words = int(lines[0].split()[1])
    entries = [(p[0], int(p[1]), int(p[2])) for p in (l.split() for l in lines[1:] if l.strip())]
    assert len(entries) >= 4 and len({e[0] for e in entries}) == len(entries)
    owner = {}
    for name, first, n in entries:
        assert n >= 1 and 0 <= first and first + n <= words, name
        for w in range(first, first + n):
            assert w not in owner, f"word {w}: {name} overlaps {owner.get(w)}"
            owner[w] = name
    names = {e[0]: e for e in entries}
    assert names["logprob_group_arrival"][2] >= 64          # one counter per activated group
    assert coral.coral_lmhead_workspace_bytes(1, 8, 1, 0, 0, 1, BF16) >= 4 * words
    # the preparation call insists on the whole area
    assert coral._L.coral_lmhead_workspace_init(FAKE, 4 * words - 4, None) == WORKSPACE


def test_noalloc_entry_point_checks_arguments_and_size_before_touching_the_device():
    """coral_lmhead_grouped_noalloc: the same argument errors as coral_lmhead_grouped, and a
    shape whose scratch need exceeds the library's static array is refused (WORKSPACE) with
    nothing looked up or enqueued."""
    c = Call()

    def noalloc(**kw):
        a = dict(c.a, **kw)
        return coral._L.coral_lmhead_grouped_noalloc(
            a["hidden"], a["gate_W"], a["gate_bias"], a["lm_W"], ctypes.byref(c.gi), a["M"], a["H"],
            a["V"], a["g"], a["k"], a["dt"], a["ids"], a["logits"], a["sel"], None)

    assert noalloc(hidden=None) == NULL
    assert noalloc(ids=None) == NULL
    assert noalloc(M=0) == SHAPE
    assert noalloc(M=65) == UNSUPPORTED
    assert noalloc(H=254) == UNSUPPORTED
    assert noalloc(g=17) == SHAPE
    # 64 tokens x 64 candidates: the published lists alone are 8 MiB
    assert coral.coral_lmhead_workspace_bytes(64, 256, 8192, 16, 2, 64, F32) > coral.NOALLOC_SCRATCH_BYTES
    assert noalloc(M=64, k=64) == WORKSPACE
    header = open(HEADER).read()
    m = re.search(r"#define\s+CORAL_NOALLOC_SCRATCH_BYTES\s+\((\d+)u\s*<<\s*(\d+)\)", header)
    assert m and int(m.group(1)) << int(m.group(2)) == coral.NOALLOC_SCRATCH_BYTES
