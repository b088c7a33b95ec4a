"""GPU parity: the HIP path against the CPU oracle, bit for bit, through the C boundary."""
import numpy as np
import pytest

from workloads import grammars, configs
from workloads.rng import stream
from tests.helpers import OracleRun, popcount, load_trajectory
from workloads import vocab as wvocab

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def _run_parity(torch, zf, Oracle, grammar, tokens, batch, steps, seed, check_every=1, **engine_kw):
    engine_kw.setdefault("state_cache_entries", -1)      # every step through the kernels unless a test asks for the state cache
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


MODES = {"automaton": 0, "trie-walk": 1, "store": 2}     # zf_options.walk_mode: all three mask kernels must give the oracle's bits


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("cache", [True, False], ids=["token-mask-cache", "parser-only"])
def test_config1_json_v2k_all_steps(cache, mode, torch_cuda, oracle_lib):
    import paper_2506_01151_amd as zf
    cfg = configs.CONFIGS[1]
    _run_parity(torch_cuda, zf, oracle_lib.Oracle, cfg.grammar(), cfg.vocab(), cfg.batch, cfg.steps, cfg.seed, token_mask_cache=cache, walk_mode=MODES[mode])


@pytest.mark.parametrize("mode", list(MODES))
def test_config2_json_v32k(mode, torch_cuda, oracle_lib):
    import paper_2506_01151_amd as zf
    cfg = configs.CONFIGS[2]
    _run_parity(torch_cuda, zf, oracle_lib.Oracle, cfg.grammar(), cfg.vocab(), cfg.batch, cfg.steps, cfg.seed, walk_mode=MODES[mode])


# the item budget bounds one set under construction (automaton) or the sets of one trie path (trie walk)
@pytest.mark.parametrize("mode,cap", [("automaton", 1), ("automaton", 2), ("automaton", 3), ("trie-walk", 1), ("trie-walk", 2), ("trie-walk", 4), ("trie-walk", 7)])
def test_forced_overflow_gives_same_bits(mode, cap, torch_cuda, oracle_lib):
    """A tiny LDS item budget pushes work to the global-memory fallback; the bits must not change."""
    import paper_2506_01151_amd as zf
    cfg = configs.CONFIGS[1]
    ov = _run_parity(torch_cuda, zf, oracle_lib.Oracle, cfg.grammar(), cfg.vocab(), 2, 24, cfg.seed + 77, lane_item_cap=cap, walk_mode=MODES[mode])
    assert ov > 0, "the cap was meant to force the fallback pass"


@pytest.mark.parametrize("seed", range(16))
def test_random_grammars(seed, torch_cuda, oracle_lib):
    """Seeded random grammars (empty rules, unit cycles, all kinds of recursion, ambiguity): both mask
    kernels against the oracle at every step, once with the default item budget and once with a
    budget of two or three items that sends much of the work through the fallback pass."""
    import paper_2506_01151_amd as zf
    from workloads import random_grammars
    g = random_grammars.random_grammar(seed)
    toks = random_grammars.random_vocab(seed, 400)
    for mode in MODES.values():
        _run_parity(torch_cuda, zf, oracle_lib.Oracle, g, toks, 3, 20, 1000 + seed, walk_mode=mode)
        if mode != 2:     # a budget of two or three items: the per-block kernels hand such sets to the fallback pass
            _run_parity(torch_cuda, zf, oracle_lib.Oracle, g, toks, 2, 12, 2000 + seed, lane_item_cap=3 - mode, token_mask_cache=seed % 2 == 0, walk_mode=mode)
        else:
            _run_parity(torch_cuda, zf, oracle_lib.Oracle, g, toks, 2, 12, 2000 + seed, token_mask_cache=seed % 2 == 0, walk_mode=mode)


def test_overflow_beyond_the_fallback_is_an_error(torch_cuda):
    """When even the fallback arena is too small the call must fail loudly (no silent wrong mask)."""
    import paper_2506_01151_amd as zf
    cfg = configs.CONFIGS[1]
    eng = zf.Engine(cfg.grammar(), cfg.vocab(), device=0, lane_item_cap=1, fallback_item_cap=1)
    s = eng.new_state()
    s.advance_bytes(b'{"a": [1')
    d_mask = torch_cuda.empty((1, eng.W), dtype=torch_cuda.int32, device="cuda")
    with pytest.raises(zf.ZfError) as ei:
        zf.compute_mask(eng, [s], d_mask)
    assert ei.value.code == zf.ZF_ERR_OVERFLOW


@pytest.mark.parametrize("chunk", [8, 16, 32])
def test_chunk_sizes(chunk, torch_cuda, oracle_lib):
    import paper_2506_01151_amd as zf
    cfg = configs.CONFIGS[1]
    _run_parity(torch_cuda, zf, oracle_lib.Oracle, cfg.grammar(), cfg.vocab(2048 - 37), 3, 32, cfg.seed + 5, chunk_strings=chunk)


def _replay_all_rows(torch, zf, oracle_lib, idx, variants, stride_of=None):
    """Replay configuration idx's oracle-sampled trajectory at its full batch and vocabulary on the oracle and on one
    engine per variant; at every step every row of every variant's mask is compared with the oracle's (variants named
    in stride_of only at every stride-th step and at the last one)."""
    cfg = configs.CONFIGS[idx]
    toks = cfg.vocab()
    off, data = wvocab.vocab_csr(toks)
    rows, steps = cfg.batch, cfg.steps
    traj = load_trajectory(idx, rows, steps)
    g = cfg.grammar()
    orc = oracle_lib.Oracle(g)
    so = [orc.new_state() for _ in range(rows)]
    engines = {name: zf.Engine(g, toks, device=0, state_cache_entries=-1, **kw) for name, kw in variants.items()}
    batches = {name: zf.StateBatch([e.new_state() for _ in range(rows)]) for name, e in engines.items()}
    d_mask = torch.empty((rows, engines[next(iter(engines))].W), dtype=torch.int32, device="cuda")
    n_checked = {name: 0 for name in engines}
    for step, ids in enumerate(traj):
        for b, t in enumerate(ids):
            if t < 0:
                so[b] = orc.new_state()
            else:
                assert so[b].feed_bytes(toks[t])
        want = np.stack([s.mask(off, data, 16) for s in so])
        for name, eng in engines.items():
            batches[name].advance(ids)
            if stride_of and name in stride_of and step % stride_of[name] and step != steps - 1:
                continue
            d_mask.fill_(-1)
            zf.compute_mask(eng, batches[name], d_mask)
            got = d_mask.cpu().numpy().view(np.uint32)
            if not np.array_equal(got, want):
                b = int(np.argwhere((got != want).any(axis=1))[0][0])
                raise AssertionError(f"cfg{idx} {name} step {step} row {b}")
            n_checked[name] += rows
    return n_checked, rows * steps


def test_config3_every_step_every_row(torch_cuda, oracle_lib):
    """Configuration 3 at its stated shape (16 rows x 512 steps, V = 128,256): all three mask kernels against the oracle at
    every step on every row; with the token-mask cache off (every token through the parser) at every 4th step."""
    import paper_2506_01151_amd as zf
    variants = {"store": dict(walk_mode=2), "automaton": dict(walk_mode=0), "trie-walk": dict(walk_mode=1), "store-parser-only": dict(walk_mode=2, token_mask_cache=False),
                "automaton-parser-only": dict(walk_mode=0, token_mask_cache=False), "trie-walk-parser-only": dict(walk_mode=1, token_mask_cache=False)}
    n, full = _replay_all_rows(torch_cuda, zf, oracle_lib, 3, variants, {"automaton-parser-only": 4, "trie-walk-parser-only": 4, "store-parser-only": 4})
    assert n["store"] == full == 16 * 512 and n["automaton"] == full and n["trie-walk"] == full


def test_config4_every_step_every_row(torch_cuda, oracle_lib):
    """Configuration 4 at its stated shape (64 rows x 256 steps, V = 128,256): all three mask kernels, every step, every row."""
    import paper_2506_01151_amd as zf
    n, full = _replay_all_rows(torch_cuda, zf, oracle_lib, 4, {"store": dict(walk_mode=2), "automaton": dict(walk_mode=0), "trie-walk": dict(walk_mode=1)})
    assert n["store"] == full == 64 * 256 and n["automaton"] == full and n["trie-walk"] == full


CFG5_CHECK_STEPS = 12      # steps of the trajectory at which masks are compared (spread evenly, the last one included) ...
CFG5_CHECK_ROWS = 6        # ... on this many seeded rows each: the oracle keeps every Earley set, a mask at step 600 costs it about a second


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("pruning", [True, False], ids=["pruned", "unpruned"])
def test_config5_full_batch_pruning_on_and_off(pruning, mode, torch_cuda, oracle_lib):
    """Configuration 5 at its stated batch and vocabulary (64 rows, V = 152,064) along the oracle-sampled trajectory, as far
    as the file goes: one compute_mask call covers all 64 rows (the launch shape the benchmark times); a seeded, reported
    subsample of (step, row) pairs is compared bit for bit with the oracle, with ZapFormat pruning on and off, every mask kernel (with pruning off the persistent automaton is not used: the per-block automaton runs in its place)."""
    import paper_2506_01151_amd as zf
    torch = torch_cuda
    cfg = configs.CONFIGS[5]
    toks = cfg.vocab()
    off, data = wvocab.vocab_csr(toks)
    rows = cfg.batch
    traj = load_trajectory(5, rows, None)
    steps = len(traj)
    assert steps >= 256
    g = cfg.grammar()
    eng = zf.Engine(g, toks, device=0, pruning=pruning, state_cache_entries=-1, walk_mode=MODES[mode])
    orc = oracle_lib.Oracle(g)
    so = [orc.new_state() for _ in range(rows)]
    ss = zf.StateBatch([eng.new_state() for _ in range(rows)])
    d_mask = torch.empty((rows, eng.W), dtype=torch.int32, device="cuda")
    check_at = sorted({(k + 1) * steps // CFG5_CHECK_STEPS - 1 for k in range(CFG5_CHECK_STEPS)} | {0, 7})
    pick = stream(cfg.seed, "parity-rows")
    pairs = []
    for step, ids in enumerate(traj):
        for b, t in enumerate(ids):
            if t < 0:
                so[b] = orc.new_state()
            else:
                assert so[b].feed_bytes(toks[t])
        ss.advance(ids)
        if step in check_at:
            d_mask.fill_(-1)
            zf.compute_mask(eng, ss, d_mask)
            got = d_mask.cpu().numpy().view(np.uint32)
            for b in sorted({pick.below(rows) for _ in range(CFG5_CHECK_ROWS)}):
                assert (got[b] == so[b].mask(off, data, 16)).all(), f"cfg5 step {step} row {b}"
                assert ss[b].accepting() == so[b].accepting()
                pairs.append((step, b))
    print(f"config 5 {'pruned' if pruning else 'unpruned'} {mode}: {steps} steps x {rows} rows replayed, compared (step, row): {pairs}")
    assert len(pairs) >= 40


LONG5 = [  # pruning, mask kernel, sentences with one long sum at the top level, compare every
    (True, "store", True, 8),
    (True, "store", False, 8),
    (True, "automaton", False, 16),
    (True, "trie-walk", False, 32),
    (False, "automaton", False, 32),
]


@pytest.mark.parametrize("pruning,mode,flat,every", LONG5, ids=[f"{'pruned' if p else 'unpruned'}-{m}-{'long-sums' if f else 'nested-groups'}" for p, m, f, _ in LONG5])
def test_config5_all_1024_steps_against_the_language_description(pruning, mode, flat, every, torch_cuda, oracle_lib):
    """Configuration 5 at its stated shape to its last decode step: 64 rows x 1,024 steps, V = 152,064.  The oracle-sampled
    trajectory ends at step 296 (the oracle keeps every Earley set of an ambiguous grammar: a mask at step 1,000 costs it
    minutes), so the rows here follow seeded sentences of the expression language cut into vocabulary tokens (valid by
    construction, workloads/sentences.py), and the masks of ALL 64 rows are compared, at every `every`-th step and at the last
    one, with the description of the language's viable prefixes in tests/expr_language.py, which the Earley oracle pins on short
    prefixes (tests/test_oracle_pins.py) and, here, on two rows at the full vocabulary during the first steps.  Two shapes of
    sentence: one long sum at the top level (every operator is another way to split it: even the pruned chart reaches 20,000
    items, which only the persistent automaton's kernel is asked to take), and nested groups of two to four operands (pruned
    charts of tens of items against 9,000 unpruned: every mask kernel, pruning on and off)."""
    import paper_2506_01151_amd as zf
    from tests.expr_language import ExprLanguage, ExprRow
    from workloads.sentences import expr_sentence, cut_into_tokens
    torch = torch_cuda
    cfg = configs.CONFIGS[5]
    toks = cfg.vocab()
    off, data = wvocab.vocab_csr(toks)
    rows, steps = cfg.batch, cfg.steps
    seqs = [cut_into_tokens(toks, expr_sentence(cfg.seed, f"sentence[{b}]", 4 * steps + 64, flat=flat), steps) for b in range(rows)]
    assert all(len(q) == steps for q in seqs)
    lang = ExprLanguage(toks)
    want_rows = [ExprRow() for _ in range(rows)]
    eng = zf.Engine(cfg.grammar(), toks, device=0, pruning=pruning, state_cache_entries=-1, walk_mode=MODES[mode])
    ss = zf.StateBatch([eng.new_state() for _ in range(rows)])
    orc = oracle_lib.Oracle(cfg.grammar())
    so = {b: orc.new_state() for b in (3, 40)}
    d_mask = torch.empty((rows, eng.W), dtype=torch.int32, device="cuda")
    n_checked = 0
    for step in range(steps):
        ids = [seqs[b][step] for b in range(rows)]
        for b in range(rows):
            assert want_rows[b].feed(toks[ids[b]]), (step, b)
        ss.advance(ids)
        if step < 24:
            for b, s in so.items():
                assert s.feed_bytes(toks[ids[b]])
        if step % every == every - 1 or step == steps - 1 or step in (0, 5, 23):
            d_mask.fill_(-1)
            zf.compute_mask(eng, ss, d_mask)
            got = d_mask.cpu().numpy().view(np.uint32)
            for b in range(rows):
                assert (got[b] == lang.mask(want_rows[b].mode, want_rows[b].depth)).all(), f"cfg5 step {step} row {b}"
                assert ss[b].accepting() == want_rows[b].accepting(), f"cfg5 step {step} row {b} accepting"
            if step in (0, 5, 23):
                for b, s in so.items():
                    assert (got[b] == s.mask(off, data, 16)).all(), f"cfg5 oracle step {step} row {b}"
            n_checked += rows
    print(f"config 5 {'pruned' if pruning else 'unpruned'} {mode}: {steps} steps x {rows} rows, {n_checked} masks compared")
    assert n_checked >= rows * (steps // every)


STATE_CACHE = [  # config, rows, steps, compare every, cache rows (0 = default), expect the cache to be used
    (3, 16, 512, 29, 0, True),
    (3, 16, 512, 41, 32, True),     # the smallest cache a batch of 16 may use: constant eviction
    (3, 16, 128, 17, 16, False),    # too small for the batch: bypassed
    (4, 64, 256, 37, 256, True),
]


@pytest.mark.parametrize("idx,rows,steps,every,entries,used", STATE_CACHE, ids=[f"cfg{r[0]}-{r[4] or 'default'}" for r in STATE_CACHE])
def test_state_cache_replay(idx, rows, steps, every, entries, used, torch_cuda, oracle_lib):
    """State cache (Section 5.2) on: compute_mask at every step of the trajectory, so that rows are
    served from cached masks as in real decoding; at sampled steps every row equals the oracle."""
    import paper_2506_01151_amd as zf
    torch = torch_cuda
    cfg = configs.CONFIGS[idx]
    toks = cfg.vocab()
    off, data = wvocab.vocab_csr(toks)
    traj = load_trajectory(idx, rows, steps)
    g = cfg.grammar()
    eng = zf.Engine(g, toks, device=0, state_cache_entries=entries)
    orc = oracle_lib.Oracle(g)
    so = [orc.new_state() for _ in range(rows)]
    ss = [eng.new_state() for _ in range(rows)]
    d_mask = torch.empty((rows, eng.W), dtype=torch.int32, device="cuda")
    hits = misses = 0
    for step, ids in enumerate(traj):
        for b, t in enumerate(ids):
            if t < 0:
                so[b] = orc.new_state()
                ss[b].reset()
            else:
                assert so[b].feed_bytes(toks[t])
                ss[b].advance(t)
        d_mask.fill_(0x33333333)
        zf.compute_mask(eng, ss, d_mask)
        r = eng.mask_report()
        assert r.cache_hits + r.cache_misses == (rows if used else 0)
        hits += r.cache_hits
        misses += r.cache_misses
        if step % every == 0 or step == steps - 1:
            got = d_mask.cpu().numpy().view(np.uint32)
            for b in range(rows):
                want = so[b].mask(off, data, 16)
                assert (got[b] == want).all(), f"cfg{idx} step {step} row {b} (hits so far {hits}, misses {misses})"
    if used:
        assert hits > misses > 0


def test_state_cache_rows_in_one_call_and_clearing(torch_cuda, oracle_lib):
    """Equal rows of one call are computed once; clearing the cache makes the next call start cold;
    a failed call leaves nothing behind that a later call could be served from."""
    import paper_2506_01151_amd as zf
    torch = torch_cuda
    cfg = configs.CONFIGS[2]
    toks = cfg.vocab()
    off, data = wvocab.vocab_csr(toks)
    g = cfg.grammar()
    eng = zf.Engine(g, toks, device=0)
    orc = oracle_lib.Oracle(g)
    o = orc.new_state()
    assert o.feed_bytes(b'{"key": [1, {"x": "a')
    want = o.mask(off, data, 4)
    ss = [eng.new_state() for _ in range(8)]
    for s in ss:
        s.advance_bytes(b'{"key": [1, {"x": "a')
    d_mask = torch.empty((8, eng.W), dtype=torch.int32, device="cuda")
    for expect in [(7, 1), (8, 0), None, (7, 1)]:
        if expect is None:
            eng.clear_state_cache()
            continue
        d_mask.fill_(0)
        zf.compute_mask(eng, ss, d_mask)
        r = eng.mask_report()
        assert (r.cache_hits, r.cache_misses) == expect
        assert (d_mask.cpu().numpy().view(np.uint32) == want[None, :]).all()
    # same prefix through an engine whose budgets are too small: the error must not poison its cache
    tiny = zf.Engine(g, toks, device=0, lane_item_cap=1, fallback_item_cap=1)
    t = tiny.new_state()
    t.advance_bytes(b'{"a": [1')
    for _ in range(2):
        with pytest.raises(zf.ZfError) as ei:
            zf.compute_mask(tiny, [t], d_mask[:1])
        assert ei.value.code == zf.ZF_ERR_OVERFLOW
        assert tiny.mask_report().cache_misses == 1


def test_async_calls_match_the_waiting_call(torch_cuda, oracle_lib):
    """compute_mask_async + mask_wait: several calls in flight on one stream, apply_mask queued right
    behind each; results equal the waiting call's and the oracle's; a fifth call in flight is refused;
    an overflow beyond the fallback arena surfaces in mask_wait."""
    import paper_2506_01151_amd as zf
    from oracle.frontend import apply_mask as oracle_apply
    torch = torch_cuda
    cfg = configs.CONFIGS[2]
    toks = cfg.vocab()
    off, data = wvocab.vocab_csr(toks)
    g = cfg.grammar()
    eng = zf.Engine(g, toks, device=0)
    orc = oracle_lib.Oracle(g)
    prefixes = [b'{"a', b'[1, 2', b' {"k": "\\', b"tr"]
    so, ss = [], []
    for p in prefixes:
        a, b = orc.new_state(), eng.new_state()
        assert a.feed_bytes(p)
        b.advance_bytes(p)
        so.append(a)
        ss.append(b)
    masks = [torch.full((1, eng.W), -1, dtype=torch.int32, device="cuda") for _ in prefixes]
    logits = configs.make_logits(cfg, 3, device="cuda", batch=1)
    outs = [torch.empty_like(logits) for _ in prefixes]
    for i in range(4):
        zf.compute_mask_async(eng, [ss[i]], masks[i])
        zf.apply_mask(eng, logits, masks[i], out=outs[i])
    with pytest.raises(zf.ZfError) as ei:
        zf.compute_mask_async(eng, [ss[0]], masks[0])
    assert ei.value.code == zf.ZF_ERR_INVALID_ARG
    zf.mask_wait(eng)
    lbits = logits.view(torch.int32).cpu().numpy().view(np.uint32)
    for i in range(4):
        want = so[i].mask(off, data, 4)
        assert (masks[i].cpu().numpy().view(np.uint32)[0] == want).all(), prefixes[i]
        assert outs[i].view(torch.int32).cpu().numpy().view(np.uint32).tobytes() == oracle_apply(lbits, want[None, :]).tobytes()
    tiny = zf.Engine(g, toks, device=0, lane_item_cap=1, fallback_item_cap=1)
    s = tiny.new_state()
    s.advance_bytes(b'{"a": [1')
    zf.compute_mask_async(tiny, [s], masks[0])
    with pytest.raises(zf.ZfError) as ei:
        zf.mask_wait(tiny)
    assert ei.value.code == zf.ZF_ERR_OVERFLOW


def test_persistent_automaton_bookkeeping(torch_cuda, oracle_lib):
    """The persistent automaton (walk_mode 2) keeps, per state, where the row stands in the device's store and which
    bytes were fed since.  Calls in flight while rows move on, a cleared store (rows come back in through their charts),
    a row fed more bytes than a call carries, clones, resets and a state destroyed while a call is in flight: the masks
    equal the oracle's every time, and a repeated call takes no Earley step at all."""
    import gc
    import paper_2506_01151_amd as zf
    torch = torch_cuda
    cfg = configs.CONFIGS[2]
    toks = cfg.vocab()
    off, data = wvocab.vocab_csr(toks)
    g = cfg.grammar()
    eng = zf.Engine(g, toks, device=0, state_cache_entries=-1, walk_mode=2)
    orc = oracle_lib.Oracle(g)
    rows = 6
    run = OracleRun(orc, toks, [stream(99, f"book[{b}]") for b in range(rows)])
    ss = zf.StateBatch([eng.new_state() for _ in range(rows)])

    def check(states, oracle_states, what):
        d = torch.full((len(states), eng.W), -1, dtype=torch.int32, device="cuda")
        zf.compute_mask(eng, states, d)
        got = d.cpu().numpy().view(np.uint32)
        for b, o in enumerate(oracle_states):
            assert (got[b] == o.mask(off, data, 8)).all(), (what, b)

    for _ in range(10):                                    # get going
        ss.advance(run.step(run.masks()))
    check(ss, run.states, "start")
    # four calls in flight, the rows advancing in between: each call walks what was fed since the last state the host knew of
    masks = [torch.full((rows, eng.W), -1, dtype=torch.int32, device="cuda") for _ in range(4)]
    want = []
    for k in range(4):
        ss.advance(run.step(run.masks()))
        want.append(run.masks())
        zf.compute_mask_async(eng, ss, masks[k])
    zf.mask_wait(eng)
    torch.cuda.synchronize()
    for k in range(4):
        assert (masks[k].cpu().numpy().view(np.uint32) == want[k]).all(), f"call {k} in flight"
    # the same states again: everything is in the table
    check(ss, run.states, "repeat")
    assert eng.mask_report().parser_steps == 0
    # the store cleared: the rows come back in from their host charts
    eng.clear_state_cache()
    check(ss, run.states, "after clearing the store")
    for _ in range(3):
        ss.advance(run.step(run.masks()))
    check(ss, run.states, "three steps after clearing")
    # a row fed far more bytes than a call carries
    long_o, long_s = orc.new_state(), eng.new_state()
    text = b'{"k": "' + b"abc def " * 700
    assert long_o.feed_bytes(text)
    long_s.advance_bytes(text)
    check([long_s], [long_o], "5,600 bytes at once")
    long_s.advance_bytes(b'", "n": [1, 2')
    assert long_o.feed_bytes(b'", "n": [1, 2')
    check([long_s], [long_o], "and a few more")
    # clones go their own ways; a reset row starts over
    c_s, c_o = ss[0].clone(), run.states[0].clone()
    m = c_o.mask(off, data, 8)
    t = next(v for v in range(300, len(toks)) if (m[v >> 5] >> (v & 31)) & 1)
    c_s.advance(t)
    assert c_o.feed_bytes(toks[t])
    check([c_s, ss[0]], [c_o, run.states[0]], "clone")
    ss[1].reset()
    run.states[1] = orc.new_state()
    check(ss, run.states, "reset")
    # a state destroyed while a call that names it is in flight
    doomed = eng.new_state()
    doomed.advance_bytes(b"[1, ")
    d2 = torch.full((2, eng.W), -1, dtype=torch.int32, device="cuda")
    zf.compute_mask_async(eng, [doomed, ss[0]], d2)
    del doomed
    gc.collect()
    zf.mask_wait(eng)
    torch.cuda.synchronize()
    assert (d2.cpu().numpy().view(np.uint32)[1] == run.states[0].mask(off, data, 8)).all()
    check(ss, run.states, "afterwards")


@pytest.mark.parametrize("cap", [2, 40], ids=["budget-2", "budget-40"])
def test_persistent_automaton_out_of_room(cap, torch_cuda, oracle_lib):
    """A set that outgrows a wavefront's scratch fails the call on the persistent automaton; the waiting call then answers
    through the per-block automaton and its fallback pass, the following calls go that way too for a while, and the masks
    are the oracle's throughout.  The call that does not wait reports the overflow from mask_wait."""
    import paper_2506_01151_amd as zf
    torch = torch_cuda
    cfg = configs.CONFIGS[5]
    g, toks = cfg.grammar(), cfg.vocab(6000)
    off, data = wvocab.vocab_csr(toks)
    orc = oracle_lib.Oracle(g)
    eng = zf.Engine(g, toks, device=0, state_cache_entries=-1, walk_mode=2, lane_item_cap=cap)
    prefixes = [b"a" + b"+b" * 30, b"(x*y" + b"+(z)" * 12, b"q"]
    so, ss = [], []
    for p in prefixes:
        a, b = orc.new_state(), eng.new_state()
        assert a.feed_bytes(p)
        b.advance_bytes(p)
        so.append(a)
        ss.append(b)
    d_mask = torch.full((len(ss), eng.W), -1, dtype=torch.int32, device="cuda")
    for rep in range(12):                                  # beyond the first back-off of 8 calls: the store is tried again, fails again
        d_mask.fill_(-1)
        zf.compute_mask(eng, ss, d_mask)
        got = d_mask.cpu().numpy().view(np.uint32)
        for i, a in enumerate(so):
            assert (got[i] == a.mask(off, data, 4)).all(), (rep, prefixes[i][:8])
    fresh = zf.Engine(g, toks, device=0, state_cache_entries=-1, walk_mode=2, lane_item_cap=cap)
    s = fresh.new_state()
    s.advance_bytes(prefixes[0])
    zf.compute_mask_async(fresh, [s], d_mask[:1])
    with pytest.raises(zf.ZfError) as ei:
        zf.mask_wait(fresh)
    assert ei.value.code == zf.ZF_ERR_OVERFLOW
    zf.compute_mask(fresh, [s], d_mask[:1])                # and the engine goes on working
    assert (d_mask[:1].cpu().numpy().view(np.uint32)[0] == so[0].mask(off, data, 4)).all()


def test_edge_cases(torch_cuda, oracle_lib):
    """Empty tokens, duplicates, a vocabulary smaller than one word, rows in different states,
    a finished sentence (empty mask), V not a multiple of 32."""
    import paper_2506_01151_amd as zf
    torch = torch_cuda
    g = grammars.json_grammar()
    orc = oracle_lib.Oracle(g)
    for toks in ([b"", b"1", b"1", b"", b"[", b"]", b"[]", b" ", b"x"],
                 [b'"', b""] * 20 + [bytes([c]) for c in range(256)] + [b"tru", b"true", b"e", b'{"a":1}', b"}"]):
        off, data = wvocab.vocab_csr(toks)
        eng = zf.Engine(g, toks, device=0)
        prefixes = [b"", b"[", b"[1", b"[]", b'{"a":1}', b"tr", b'{"k":"\\u12']
        so, ss = [], []
        for p in prefixes:
            a, b = orc.new_state(), eng.new_state()
            assert a.feed_bytes(p)
            b.advance_bytes(p)
            so.append(a)
            ss.append(b)
        d_mask = torch.full((len(prefixes), eng.W), -1, dtype=torch.int32, device="cuda")
        zf.compute_mask(eng, ss, d_mask)
        got = d_mask.cpu().numpy().view(np.uint32)
        for i, a in enumerate(so):
            assert (got[i] == a.mask(off, data, 1)).all(), (toks[:4], prefixes[i])
    # a grammar whose sentence cannot be extended: after the last byte the mask is all zero
    g2 = grammars.w2_grammar()
    toks = [b"a", b"b", b"ab"]
    eng = zf.Engine(g2, toks, device=0)
    s = eng.new_state()
    s.advance(2)
    d_mask = torch.full((1, eng.W), -1, dtype=torch.int32, device="cuda")
    zf.compute_mask(eng, [s], d_mask)
    assert d_mask.cpu().numpy().view(np.uint32).tolist() == [[0]] and s.accepting()


@pytest.mark.parametrize("mode", list(MODES))
def test_long_tokens_deep_nesting_many_classes(mode, torch_cuda, oracle_lib):
    """Tokens longer than the 16 bytes a lane fetches at once, nesting deeper than the automaton's state budget
    (those strings must come back through the fallback pass), and a grammar with more than 64 byte classes."""
    import paper_2506_01151_amd as zf
    from tests.helpers import edge_vocab_json
    torch = torch_cuda
    g = grammars.json_grammar()
    toks = edge_vocab_json()
    off, data = wvocab.vocab_csr(toks)
    orc = oracle_lib.Oracle(g)
    eng = zf.Engine(g, toks, device=0, state_cache_entries=-1, walk_mode=MODES[mode])
    prefixes = [b"", b"[", b'{"k":"', b"[1,", b'[[{"a":[', b'{"k":"v', b"[1", b'["\\']
    so, ss = [], []
    for p in prefixes:
        a, b = orc.new_state(), eng.new_state()
        assert a.feed_bytes(p)
        b.advance_bytes(p)
        so.append(a)
        ss.append(b)
    d_mask = torch.full((len(prefixes), eng.W), -1, dtype=torch.int32, device="cuda")
    zf.compute_mask(eng, ss, d_mask)
    got = d_mask.cpu().numpy().view(np.uint32)
    for i, a in enumerate(so):
        assert (got[i] == a.mask(off, data, 4)).all(), prefixes[i]
    if mode == "automaton":
        assert eng.mask_report().overflow_chunks > 0, "runs of 120 brackets were meant to outgrow the state budget"
    if mode == "store":
        assert eng.mask_report().overflow_chunks == 0      # the persistent automaton has room for every nesting depth
    g2 = grammars.many_classes_grammar(100)
    toks2 = [bytes([c]) for c in range(256)] + [bytes([32 + c, 32 + (c * 7 + 3) % 100]) for c in range(100)] + [bytes([32 + c, 32 + (c * 7 + 3) % 100, 32 + (c * 5) % 100]) for c in range(100)]
    assert zf.Engine(g2, toks2, device=-1).info.n_byte_classes > 64
    _run_parity(torch, zf, oracle_lib.Oracle, g2, toks2, 3, 12, 4242, walk_mode=MODES[mode])


def test_exploration_at_compile_time_changes_no_mask(torch_cuda, oracle_lib):
    """zf_options.precompute_states: the automaton explored from the empty prefix when the engine is compiled and
    whenever it is emptied.  A grammar without recursion (the W2 sequence, a JSON schema with fixed keys cut short
    by its budget) and a recursive one; masks against the oracle with the exploration on, off, and after the engine
    has been emptied in mid-sentence; and the first steps of a decode loop find more of their transitions
    computed with it than without."""
    import paper_2506_01151_amd as zf
    torch = torch_cuda
    cfg = configs.CONFIGS[2]
    g, toks = cfg.grammar(), cfg.vocab()
    for pre in (-1, 64, 0):
        _run_parity(torch, zf, oracle_lib.Oracle, g, toks, 4, 24, 991, walk_mode=2, precompute_states=pre)
    _run_parity(torch, zf, oracle_lib.Oracle, grammars.w2_grammar(), [b"a", b"b", b"ab", b"ba", b""], 2, 6, 5, walk_mode=2)
    cfg3 = configs.CONFIGS[3]
    g3, toks3 = cfg3.grammar(), cfg3.vocab(8000)
    steps_taken = {}
    for pre in (-1, 0):
        eng = zf.Engine(g3, toks3, device=0, state_cache_entries=-1, walk_mode=2, precompute_states=pre)
        orc = oracle_lib.Oracle(g3)
        run = OracleRun(orc, toks3, [stream(77, f"sample[{b}]") for b in range(4)])
        states = [eng.new_state() for _ in range(4)]
        d_mask = torch.empty((4, eng.W), dtype=torch.int32, device="cuda")
        total = 0
        for step in range(12):
            want = run.masks()
            zf.compute_mask(eng, states, d_mask)
            total += eng.mask_report().parser_steps
            assert (d_mask.cpu().numpy().view(np.uint32) == want).all(), (pre, step)
            if step == 6:
                eng.clear_state_cache()                     # emptied (and explored again) under the rows' feet
            for b, t in enumerate(run.step(want)):
                states[b].reset() if t < 0 else states[b].advance(t)
        steps_taken[pre] = total
    assert steps_taken[0] < steps_taken[-1], steps_taken


@pytest.mark.parametrize("cap", [None, 72, 200], ids=["default-budget", "budget-72", "budget-200"])
def test_wide_sets_of_an_ambiguous_grammar(cap, torch_cuda, oracle_lib):
    """Sets far beyond 64 items (the ambiguous expression grammar after sums of 20 to 150 operands: every
    operand is another origin) through the mask automaton: the set under construction then lives in LDS
    behind a hash table and Complete deals the origin sets' items to the lanes.  With a budget of 72 or
    200 items the wider sets run out of room and their strings must come back through the fallback pass."""
    import paper_2506_01151_amd as zf
    torch = torch_cuda
    cfg = configs.CONFIGS[5]
    g, toks = cfg.grammar(), cfg.vocab(6000)
    off, data = wvocab.vocab_csr(toks)
    orc = oracle_lib.Oracle(g)
    kw = {} if cap is None else {"lane_item_cap": cap}
    eng = zf.Engine(g, toks, device=0, state_cache_entries=-1, **kw)
    prefixes = [b"a" + b"+b" * 20, b"a" + b"*77" * 45 + b"+", b"(a" + b"+b" * 70 + b")*c" + b"+d" * 12, b"x" + b"+(y)" * 150, b"q" + b"*r" * 160 + b"*(",
                b"a+b", b"a" + b"+b" * 300]
    so, ss = [], []
    for p in prefixes:
        a, b = orc.new_state(), eng.new_state()
        assert a.feed_bytes(p)
        b.advance_bytes(p)
        so.append(a)
        ss.append(b)
    def last_set_size(st):
        items, n_sets = st.chart()
        return sum(1 for it in items if it[0] == n_sets - 1)
    assert max(last_set_size(s) for s in ss) > 250
    d_mask = torch.full((len(prefixes), eng.W), -1, dtype=torch.int32, device="cuda")
    zf.compute_mask(eng, ss, d_mask)
    got = d_mask.cpu().numpy().view(np.uint32)
    for i, a in enumerate(so):
        assert (got[i] == a.mask(off, data, 4)).all(), prefixes[i][:12]
    if cap is not None:
        assert eng.mask_report().overflow_chunks > 0, "the budget was meant to be too small for the widest sets"


@pytest.mark.parametrize("mode", list(MODES))
def test_many_rows_and_longest_token(mode, torch_cuda, oracle_lib):
    """A batch larger than the number of compute units (one block per row and less) and tokens of the
    maximum length the library takes (255 bytes), valid and invalid ones."""
    import paper_2506_01151_amd as zf
    torch = torch_cuda
    cfg = configs.CONFIGS[1]
    g = cfg.grammar()
    toks = cfg.vocab(600) + [b'"' + b"x" * 253 + b'"', b"[" * 255, b"1" * 255, b'"' + b"y" * 254, b" " * 254 + b"}", b"a" * 255]
    off, data = wvocab.vocab_csr(toks)
    orc = oracle_lib.Oracle(g)
    eng = zf.Engine(g, toks, device=0, state_cache_entries=-1, walk_mode=MODES[mode])
    rows = 300
    rs = stream(cfg.seed, "many-rows")
    pieces = [b"", b"[", b'{"a":', b'{"a": "', b"[1, 2", b'[{"k": [', b"tr", b'"abc', b"[[[", b'{"k":"v"', b"-1.5e", b'["\\u00']
    so, ss = [], []
    for r in range(rows):
        p = pieces[rs.below(len(pieces))]
        a, b = orc.new_state(), eng.new_state()
        assert a.feed_bytes(p)
        b.advance_bytes(p)
        so.append(a)
        ss.append(b)
    d_mask = torch.full((rows, eng.W), -1, dtype=torch.int32, device="cuda")
    zf.compute_mask(eng, ss, d_mask)
    got = d_mask.cpu().numpy().view(np.uint32)
    for r in range(rows):
        assert (got[r] == so[r].mask(off, data, 4)).all(), r


@pytest.mark.parametrize("mode", ["automaton", "store"])
def test_largest_batch_closing_kernel_loops_over_row_groups(mode, torch_cuda, oracle_lib):
    """4,096 rows (the largest batch a call takes) over a vocabulary of 1,000 tokens: the closing kernel's grid is capped at
    what the chip holds at once, so its blocks loop over the 1,024 row groups; with a budget of one item the per-block
    automaton sends strings through the fallback pass, whose wavefronts the other blocks of that grid wait for."""
    import paper_2506_01151_amd as zf
    torch = torch_cuda
    cfg = configs.CONFIGS[1]
    g = cfg.grammar()
    toks = cfg.vocab(1000)
    off, data = wvocab.vocab_csr(toks)
    orc = oracle_lib.Oracle(g)
    kw = {"lane_item_cap": 1} if mode == "automaton" else {}
    eng = zf.Engine(g, toks, device=0, state_cache_entries=-1, walk_mode=MODES[mode], **kw)
    pieces = [b"", b"[", b'{"a":', b'{"a": "', b"[1, 2", b'[{"k": [', b"tr", b'"abc', b"[[[", b'{"k":"v"', b"-1.5e", b'["\\u00', b"[1.0"]
    want, proto = [], []
    for p in pieces:
        a, b = orc.new_state(), eng.new_state()
        assert a.feed_bytes(p)
        b.advance_bytes(p)
        want.append(a.mask(off, data, 4))
        proto.append(b)
    rows = 4096
    rs = stream(cfg.seed, "largest-batch")
    pick = [rs.below(len(pieces)) for _ in range(rows)]
    ss = [proto[k] for k in pick]                          # a state may be named many times in one call
    d_mask = torch.full((rows, eng.W), -1, dtype=torch.int32, device="cuda")
    zf.compute_mask(eng, ss, d_mask)
    got = d_mask.cpu().numpy().view(np.uint32)
    assert (got == np.stack([want[k] for k in pick])).all()
    if mode == "automaton":
        assert eng.mask_report().overflow_chunks > 0


@pytest.mark.parametrize("cap", [None, 1], ids=["default-budget", "budget-1"])
def test_ragged_vocabulary_many_rows_closing_kernel(cap, torch_cuda, oracle_lib):
    """130 rows (a last group of two) over a vocabulary of 40,037 tokens (not a multiple of 32 or 64): the
    closing kernel then serves long runs of tokens per block from LDS copies of the rows, and the last
    block's run ends inside a mask word.  With an item budget of 1 most strings come back through the
    fallback pass, the closing kernel's first phase, whose wavefronts the other blocks wait for."""
    import paper_2506_01151_amd as zf
    torch = torch_cuda
    cfg = configs.CONFIGS[2]
    g = cfg.grammar()
    toks = cfg.vocab(40037)
    off, data = wvocab.vocab_csr(toks)
    orc = oracle_lib.Oracle(g)
    kw = {} if cap is None else {"lane_item_cap": cap}
    eng = zf.Engine(g, toks, device=0, state_cache_entries=-1, **kw)
    rows = 130
    rs = stream(cfg.seed, "ragged-rows")
    pieces = [b"", b"[", b'{"a":', b'{"a": "', b"[1, 2", b'[{"k": [', b"tr", b'"abc', b"[[[", b'{"k":"v"', b"-1.5e", b'["\\u00', b"[1.0", b'{"k": nul']
    so, ss = [], []
    for r in range(rows):
        p = pieces[rs.below(len(pieces))]
        a, b = orc.new_state(), eng.new_state()
        assert a.feed_bytes(p)
        b.advance_bytes(p)
        so.append(a)
        ss.append(b)
    d_mask = torch.full((rows, eng.W), -1, dtype=torch.int32, device="cuda")
    zf.compute_mask(eng, ss, d_mask)
    got = d_mask.cpu().numpy().view(np.uint32)
    for r in range(rows):
        assert (got[r] == so[r].mask(off, data, 8)).all(), r
    assert got[:, -1].max() < (1 << (40037 % 32)), "padding bits of the last word must be zero"
    if cap is not None:
        assert eng.mask_report().overflow_chunks > 0


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("n_words,word_len,lds_mode", [(1500, 5, 1), (1500, 8, 2)])
def test_grammar_tables_beyond_the_lds_budget(n_words, word_len, lds_mode, mode, torch_cuda, oracle_lib):
    """Grammars whose tables do not fit the kernels' LDS budget: only the small tables staged (mode 1) or
    none (mode 2); the kernels then read the rest from global memory."""
    import paper_2506_01151_amd as zf
    g = grammars.big_tables_grammar(n_words, word_len)
    words = [bytes(t.data) for t in g.terminals if len(t.data) == word_len]
    rs = stream(77, "big-tables-vocab")
    toks = [bytes([c]) for c in range(256)]
    for _ in range(400):
        w = words[rs.below(len(words))]
        k = rs.below(4)
        toks.append(w if k == 0 else (w[:1 + rs.below(word_len - 1)] if k == 1 else (w + b" " if k == 2 else w[2:] + b" " + words[rs.below(len(words))][:3])))
    eng = zf.Engine(g, toks, device=0, state_cache_entries=-1, walk_mode=MODES[mode])
    assert eng.info.table_lds_mode == lds_mode
    del eng
    _run_parity(torch_cuda, zf, oracle_lib.Oracle, g, toks, 3, 6, 31337, walk_mode=MODES[mode])


def test_apply_mask_full_size_bf16(torch_cuda, oracle_lib):
    """Configuration 3's logits shape [16, 128256] bf16, mask from a real state."""
    import paper_2506_01151_amd as zf
    from oracle.frontend import apply_mask as oracle_apply
    torch = torch_cuda
    cfg = configs.CONFIGS[3]
    eng = zf.Engine(cfg.grammar(), cfg.vocab(), device=0)
    rng = np.random.default_rng(5)
    mask = rng.integers(0, 2**32, size=(cfg.batch, eng.W), dtype=np.uint32)
    mask[3] = 0
    mask[4] = 0xFFFFFFFF
    logits = configs.make_logits(cfg, 1, device="cuda")
    d_mask = torch.from_numpy(mask.view(np.int32)).cuda()
    out = torch.empty_like(logits)
    zf.apply_mask(eng, logits, d_mask, out=out)
    bits = logits.view(torch.int16).cpu().numpy().view(np.uint16)
    want = oracle_apply(bits, mask)
    assert out.view(torch.int16).cpu().numpy().view(np.uint16).tobytes() == want.tobytes()


FUSED = [("store", "bf16", 0, True), ("store", "f32", 0, False), ("store", "bf16", 13, False), ("store-state-cache", "f32", 0, True),
         ("automaton", "bf16", 0, False), ("trie-walk", "f32", 0, True)]


@pytest.mark.parametrize("variant,dtype,ragged,in_place", FUSED, ids=[f"{v}-{d}-{'ragged' if r else 'even'}-{'in-place' if i else 'out'}" for v, d, r, i in FUSED])
def test_compute_mask_apply_in_one_call(variant, dtype, ragged, in_place, torch_cuda, oracle_lib):
    """zf_compute_mask_apply_async: the mask and the masked logits of every step against the oracle, bit for bit -- through the
    persistent automaton (one kernel does both), with a vocabulary size that is no multiple of a 16-byte piece, with the state
    cache on and through the other mask kernels (two kernels behind the one call)."""
    import paper_2506_01151_amd as zf
    from oracle.frontend import apply_mask as oracle_apply
    torch = torch_cuda
    cfg = configs.CONFIGS[1]
    toks = cfg.vocab(2048 - ragged)
    kw = {"store": dict(walk_mode=2, state_cache_entries=-1), "store-state-cache": dict(walk_mode=2, state_cache_entries=64),
          "automaton": dict(walk_mode=0, state_cache_entries=-1), "trie-walk": dict(walk_mode=1, state_cache_entries=-1)}[variant]
    eng = zf.Engine(cfg.grammar(), toks, device=0, **kw)
    B, V = 5, eng.V
    orc = oracle_lib.Oracle(cfg.grammar())
    run = OracleRun(orc, toks, [stream(cfg.seed + 77, f"sample[{b}]") for b in range(B)])
    states = [eng.new_state() for _ in range(B)]
    d_mask = torch.empty((B, eng.W), dtype=torch.int32, device="cuda")
    rng = np.random.default_rng(5)
    ivt = torch.int32 if dtype == "f32" else torch.int16
    for step in range(40):
        want_mask = run.masks()
        if dtype == "f32":
            bits = rng.integers(0, 2**32, size=(B, V), dtype=np.uint32)
            t = torch.from_numpy(bits.view(np.int32)).cuda().view(torch.float32)
        else:
            bits = rng.integers(0, 2**16, size=(B, V), dtype=np.uint16)
            t = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
        out = t if in_place else torch.full_like(t, 1.0)
        d_mask.fill_(0x5A5A5A5A)
        zf.compute_mask_apply_async(eng, states, d_mask, t, out=out)
        zf.mask_wait(eng)
        torch.cuda.synchronize()
        got_mask = d_mask.cpu().numpy().view(np.uint32)
        assert np.array_equal(got_mask, want_mask), f"{variant} step {step}: mask"
        want = oracle_apply(bits, want_mask)
        got = out.view(ivt).cpu().numpy().view(bits.dtype)
        assert got.tobytes() == want.tobytes(), f"{variant} step {step}: masked logits"
        for b, tk in enumerate(run.step(want_mask)):
            states[b].reset() if tk < 0 else states[b].advance(tk)


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
