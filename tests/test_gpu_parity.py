"""GPU parity: the HIP path against the CPU oracle, bit for bit, through the C boundary."""
import numpy as np
import pytest

from workloads import grammars, configs
from workloads.rng import stream
from tests.helpers import OracleRun, popcount

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def _run_parity(torch, zf, Oracle, grammar, tokens, batch, steps, seed, check_every=1, **engine_kw):
    eng = zf.Engine(grammar, tokens, device=0, **engine_kw)
    orc = Oracle(grammar)
    run = OracleRun(orc, tokens, [stream(seed, f"sample[{b}]") for b in range(batch)])
    states = [eng.new_state() for _ in range(batch)]
    d_mask = torch.empty((batch, eng.W), dtype=torch.int32, device="cuda")
    overflow = 0
    for step in range(steps):
        want = run.masks()
        if step % check_every == 0:
            d_mask.fill_(0x5A5A5A5A)
            zf.compute_mask(eng, states, d_mask)
            got = d_mask.cpu().numpy().view(np.uint32)
            overflow += eng.mask_report().overflow_chunks
            assert got.shape == want.shape
            if not (got == want).all():
                bad = np.argwhere(got != want)[0]
                w = int(bad[1])
                diff = int(got[bad[0], w]) ^ int(want[bad[0], w])
                v = w * 32 + (diff & -diff).bit_length() - 1
                raise AssertionError(f"step {step} row {bad[0]} token {v} {tokens[v]!r}: gpu={got[bad[0], w]:#x} oracle={want[bad[0], w]:#x}")
        toks = run.step(want)
        for b, t in enumerate(toks):
            if t < 0:
                states[b].reset()
            else:
                states[b].advance(t)
            assert states[b].accepting() == run.states[b].accepting()
    return overflow


def test_config1_json_v2k_all_steps(torch_cuda, oracle_lib):
    import paper_2506_01151_amd as zf
    cfg = configs.CONFIGS[1]
    _run_parity(torch_cuda, zf, oracle_lib.Oracle, cfg.grammar(), cfg.vocab(), cfg.batch, cfg.steps, cfg.seed)


def test_config2_json_v32k(torch_cuda, oracle_lib):
    import paper_2506_01151_amd as zf
    cfg = configs.CONFIGS[2]
    _run_parity(torch_cuda, zf, oracle_lib.Oracle, cfg.grammar(), cfg.vocab(), cfg.batch, cfg.steps, cfg.seed)


@pytest.mark.parametrize("cap", [1, 2, 4])
def test_forced_overflow_gives_same_bits(cap, torch_cuda, oracle_lib):
    import paper_2506_01151_amd as zf
    cfg = configs.CONFIGS[1]
    ov = _run_parity(torch_cuda, zf, oracle_lib.Oracle, cfg.grammar(), cfg.vocab(), 2, 24, cfg.seed + 77, lane_item_cap=cap)
    assert ov > 0, "the cap was meant to force the fallback pass"


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_apply_mask_bit_exact(dtype, torch_cuda, oracle_lib):
    import paper_2506_01151_amd as zf
    from oracle.frontend import apply_mask as oracle_apply
    torch = torch_cuda
    cfg = configs.CONFIGS[1]
    toks = cfg.vocab(2048 - 13)           # ragged V: not a multiple of 32 nor of the vector width
    eng = zf.Engine(cfg.grammar(), toks, device=0)
    B, V, W = 5, eng.V, eng.W
    rng = np.random.default_rng(11)
    mask = rng.integers(0, 2**32, size=(B, W), dtype=np.uint32)
    if dtype == "f32":
        bits = rng.integers(0, 2**32, size=(B, V), dtype=np.uint32)
        t = torch.from_numpy(bits.view(np.int32)).cuda().view(torch.float32)
    else:
        bits = rng.integers(0, 2**16, size=(B, V), dtype=np.uint16)
        t = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    d_mask = torch.from_numpy(mask.view(np.int32)).cuda()
    want = oracle_apply(bits, mask)
    out = torch.empty_like(t)
    zf.apply_mask(eng, t, d_mask, out=out)
    ivt = torch.int32 if dtype == "f32" else torch.int16
    got = out.view(ivt).cpu().numpy().view(bits.dtype)
    assert got.tobytes() == want.tobytes()
    zf.apply_mask(eng, t, d_mask)         # in place
    assert t.view(ivt).cpu().numpy().view(bits.dtype).tobytes() == want.tobytes()
