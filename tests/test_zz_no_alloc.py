"""The entry point that allocates nothing (coral_lmhead_grouped_noalloc) against
coral_lmhead_grouped, through the C ABI on a real MI355X: same kernels on the library's
static scratch array instead of a caller's workspace, so ids, logits and groups must agree
bit for bit.  Every case makes two calls in a row, the second with a smaller input: the
array keeps what the first call left there."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from coral_inputs import CONFIGS, HeadConfig, make_head, make_hidden  # noqa: E402


@pytest.fixture(scope="module")
def coral():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2502_16880_amd as c
    return c


def upload(coral, head):
    c = head.cfg
    return (coral.device_tensor(head.gate_W, c.dtype), coral.device_tensor(head.lm_W, c.dtype),
            None if head.gate_bias is None else torch.from_numpy(head.gate_bias).cuda(),
            coral.GroupIndex(head.group_offsets, head.group_rows))


def both(coral, cfg, dev, M, g, k, batch):
    """(reference entry point's outputs, new entry point's outputs) for one seeded batch."""
    gate_W, lm_W, bias, gi = dev
    d_hidden = coral.device_tensor(make_hidden(cfg, M, batch), cfg.dtype)
    want = coral.coral_lmhead_grouped(d_hidden, gate_W, bias, lm_W, gi, g, k)
    ids = torch.full((M, k), -5, dtype=torch.int32, device="cuda")
    z = torch.full((M, k), float("nan"), device="cuda")
    sel = torch.full((M, g), -5, dtype=torch.int32, device="cuda")
    coral.coral_lmhead_grouped_noalloc(d_hidden, gate_W, bias, lm_W, gi, g, k, ids, z, sel)
    torch.cuda.synchronize()
    return want, (ids, z, sel)


CASES = [
    # (config, expected path, (M, g, k) of the first call, of the second, smaller one)
    (CONFIGS["llama3_8b"].scaled(V=32 * 203), 1, (8, 4, 10), (3, 2, 7)),
    (CONFIGS["tiny_f32"], 1, (4, 2, 8), (1, 1, 3)),
    (CONFIGS["wide_tree"].scaled(V=64 * 126), 2, (64, 8, 16), (40, 8, 16)),
    (CONFIGS["llama3_8b"].scaled(name="llama3_f16_h4160", dtype="f16", V=32 * 203, H=4160), 0,
     (8, 4, 10), (2, 4, 10)),
]


@pytest.mark.parametrize("cfg,path,first,second", CASES,
                         ids=lambda x: x.name if isinstance(x, HeadConfig) else None)
def test_noalloc_matches_grouped_on_two_calls_in_a_row(coral, cfg, path, first, second):
    dt = {"f32": coral.CORAL_F32, "bf16": coral.CORAL_BF16, "f16": coral.CORAL_F16}[cfg.dtype]
    dev = upload(coral, make_head(cfg))
    for call, (M, g, k) in enumerate((first, second)):
        if call == 0:
            assert coral.coral_lmhead_path(False, M, cfg.H, cfg.V, cfg.G, g, k, dt) == path
        print(f"case {cfg.name} call {call}: M={M} g={g} k={k}", flush=True)
        want, got = both(coral, cfg, dev, M, g, k, batch=call)
        for name, a, b in zip(("ids", "logits", "groups"), want, got):
            assert torch.equal(a, b), f"{name} differ on call {call}"


def test_noalloc_at_full_size_then_a_smaller_vocabulary(coral):
    """The headline shape with 16 tokens (7 MB of scratch), then one token, then another,
    smaller head: a different layout over the same array."""
    cfg = CONFIGS["llama3_8b"]
    dev = upload(coral, make_head(cfg))
    for call, M in enumerate((16, 1)):
        print(f"case {cfg.name} M={M}", flush=True)
        want, got = both(coral, cfg, dev, M, cfg.g, cfg.k, batch=call)
        for a, b in zip(want, got):
            assert torch.equal(a, b)
    del dev
    torch.cuda.empty_cache()
    small = CONFIGS["llama2_7b"].scaled(V=16 * 250)
    want, got = both(coral, small, upload(coral, make_head(small)), 4, small.g, small.k, batch=0)
    for a, b in zip(want, got):
        assert torch.equal(a, b)


def test_noalloc_refuses_shapes_beyond_its_scratch(coral):
    """64 tokens x 16 candidates at the full vocabulary need 37 MB: refused before any launch
    (the weights here are a small dummy; the size check sees the declared shape only)."""
    cfg = CONFIGS["wide_tree"]
    need = coral.coral_lmhead_workspace_bytes(64, cfg.H, cfg.V, cfg.G, cfg.g, cfg.k, coral.CORAL_BF16)
    assert need > coral.NOALLOC_SCRATCH_BYTES
    head = make_head(cfg.scaled(V=64 * 126))
    gate_W, _, bias, _ = upload(coral, head)
    rows = np.arange(cfg.V, dtype=np.int32)
    offsets = (np.arange(cfg.G + 1) * cfg.v).astype(np.int32)
    gi = coral.GroupIndex(offsets, rows, validate=False)
    # a [V,H] weight tensor of 1 GB just to be refused would be wasteful: the C ABI is called
    # directly with a small buffer's address, which the refused call never reads
    lm_W = torch.zeros(4096, dtype=torch.bfloat16, device="cuda")
    d_hidden = coral.device_tensor(make_hidden(cfg, 64, 0), cfg.dtype)
    ids = torch.empty((64, cfg.k), dtype=torch.int32, device="cuda")
    z = torch.empty((64, cfg.k), device="cuda")
    st = coral._L.coral_lmhead_grouped_noalloc(
        d_hidden.data_ptr(), gate_W.data_ptr(), bias.data_ptr(), lm_W.data_ptr(), gi.struct(),
        64, cfg.H, cfg.V, cfg.g, cfg.k, coral.CORAL_BF16, ids.data_ptr(), z.data_ptr(), None, None)
    assert st == 5                                       # CORAL_ERR_WORKSPACE
    torch.cuda.synchronize()


def test_noalloc_under_graph_capture(coral):
    """The callers it is for: captured after one eager call (which looks the array up),
    replayed with eager work in between, every replay equal to the eager result."""
    cfg = CONFIGS["llama3_8b"].scaled(V=32 * 501)
    gate_W, lm_W, bias, gi = upload(coral, make_head(cfg))
    M = 4
    d_hidden = coral.device_tensor(make_hidden(cfg, M, 1), cfg.dtype)
    want = coral.coral_lmhead_grouped(d_hidden, gate_W, bias, lm_W, gi, cfg.g, cfg.k)
    ids = torch.empty((M, cfg.k), dtype=torch.int32, device="cuda")
    z = torch.empty((M, cfg.k), device="cuda")
    sel = torch.empty((M, cfg.g), dtype=torch.int32, device="cuda")

    def call():
        coral.coral_lmhead_grouped_noalloc(d_hidden, gate_W, bias, lm_W, gi, cfg.g, cfg.k, ids, z, sel)

    call()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
        call()
    for rep in range(3):
        ids.fill_(-1), z.zero_(), sel.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(want, (ids, z, sel)):
            assert torch.equal(a, b), rep
