"""GPU test of zf_compute_mask_noalloc, the entry point for callers that cannot allocate device
memory: its masks must equal zf_compute_mask's bit for bit (and, where checked, the oracle's),
on calls that follow each other on one GPU and share the static scratch array."""
import numpy as np
import pytest

from workloads import configs
from workloads import vocab as wvocab
from tests.helpers import load_trajectory

pytestmark = pytest.mark.gpu


def _states_after(eng, traj, rows, step):
    ss = [eng.new_state() for _ in range(rows)]
    for ids in traj[:step]:
        for b in range(rows):
            ss[b].reset() if ids[b] < 0 else ss[b].advance(ids[b])
    return ss


@pytest.mark.parametrize("mode", [0, 1, 2], ids=["automaton", "trie-walk", "store"])
def test_noalloc_equals_compute_mask_two_calls_in_a_row(mode, oracle_lib):
    import torch
    import paper_2506_01151_amd as zf
    assert torch.cuda.is_available()
    cfg = configs.CONFIGS[3]
    toks = cfg.vocab()
    g = cfg.grammar()
    eng = zf.Engine(g, toks, device=0, walk_mode=mode)
    traj = load_trajectory(3, cfg.batch, 200)
    big = _states_after(eng, traj, cfg.batch, 137)           # 16 rows in the middle of their objects
    small = _states_after(eng, traj, 5, 61)                   # then a smaller batch in other states
    off, data = wvocab.vocab_csr(toks)
    orc = oracle_lib.Oracle(g)
    for ss, steps in ((big, 137), (small, 61), (big, 137)):
        n = len(ss)
        want = torch.full((n, eng.W), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
        got = torch.full((n, eng.W), 0x33333333, dtype=torch.int32, device="cuda")
        zf.compute_mask_noalloc(eng, ss, got)
        zf.compute_mask(eng, ss, want)
        a, b = got.cpu().numpy().view(np.uint32), want.cpu().numpy().view(np.uint32)
        assert (a == b).all(), f"rows {np.unique(np.argwhere(a != b)[:, 0])} differ"
        so = orc.new_state()                                  # row 0 against the oracle as well
        for ids in traj[:steps]:
            so = orc.new_state() if ids[0] < 0 else so
            if ids[0] >= 0:
                assert so.feed_bytes(toks[ids[0]])
        assert (a[0] == so.mask(off, data, 8)).all()


def test_noalloc_fallback_pass_in_the_scratch_array():
    """A tiny item budget sends most strings through the fallback pass, whose list and arenas are
    slices of the static array here."""
    import torch
    import paper_2506_01151_amd as zf
    cfg = configs.CONFIGS[1]
    eng = zf.Engine(cfg.grammar(), cfg.vocab(), device=0, lane_item_cap=1, state_cache_entries=-1)
    for prefixes in ([b'{"a": [1, 2', b"[[", b'{"k": "v'], [b"[1.5e"]):
        ss = []
        for p in prefixes:
            s = eng.new_state()
            s.advance_bytes(p)
            ss.append(s)
        want = torch.zeros((len(ss), eng.W), dtype=torch.int32, device="cuda")
        got = torch.full((len(ss), eng.W), -1, dtype=torch.int32, device="cuda")
        zf.compute_mask_noalloc(eng, ss, got)
        assert eng.mask_report().overflow_chunks > 0
        zf.compute_mask(eng, ss, want)
        assert torch.equal(got, want)


def test_noalloc_refuses_what_does_not_fit():
    import torch
    import paper_2506_01151_amd as zf
    cfg = configs.CONFIGS[2]
    eng = zf.Engine(cfg.grammar(), cfg.vocab(), device=0, walk_mode=1)
    rows = 4096                                               # the trie walk's queue of 4096 rows x 32,000 tokens alone exceeds the array
    ss = [eng.new_state()] * rows
    d_mask = torch.zeros((rows, eng.W), dtype=torch.int32, device="cuda")
    with pytest.raises(zf.ZfError) as ei:
        zf.compute_mask_noalloc(eng, ss, d_mask)
    assert ei.value.code == zf.ZF_ERR_INVALID_ARG and "zf_compute_mask_noalloc" in str(ei.value)
    zf.compute_mask_noalloc(eng, ss[:3], d_mask[:3])          # and the engine still works afterwards
    want = torch.zeros((3, eng.W), dtype=torch.int32, device="cuda")
    zf.compute_mask(eng, ss[:3], want)
    assert torch.equal(d_mask[:3], want)
    # asynchronous calls in flight: refused until zf_mask_wait
    zf.compute_mask_async(eng, ss[:3], want)
    with pytest.raises(zf.ZfError) as ei:
        zf.compute_mask_noalloc(eng, ss[:3], d_mask[:3])
    assert ei.value.code == zf.ZF_ERR_INVALID_ARG
    zf.mask_wait(eng)
