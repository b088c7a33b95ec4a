"""Shared helpers for the parity tests (harness only: sampling, bookkeeping)."""
import numpy as np
from workloads import vocab as wvocab
from workloads.configs import pick_set_bit


def load_trajectory(idx, rows, steps):
    """Token ids per step and row from tests/golden/trajectory_cfgN.txt (-1 = reset)."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", f"trajectory_cfg{idx}.txt")
    traj = [[int(x) for x in line.split()] for line in open(path) if line.strip() and not line.startswith("#")]
    if steps is None:            # as far as the file goes
        steps = len(traj)
    assert len(traj) >= steps and len(traj[0]) >= rows, "trajectory file too small for this test"
    return [t[:rows] for t in traj[:steps]]


def popcount(words) -> int:
    return int(np.unpackbits(np.ascontiguousarray(words).view(np.uint8)).sum())


class OracleRun:
    """Drives oracle states along a seeded trajectory: at every step the next token is drawn
    uniformly from the oracle-valid mask; a row whose mask is empty (its sentence is complete
    and cannot be extended) is reset, which stands for 'query finished, next query'."""

    def __init__(self, oracle, tokens, samplers, n_threads=8):
        self.o, self.tokens = oracle, tokens
        self.off, self.data = wvocab.vocab_csr(tokens)
        self.samplers = samplers
        self.states = [oracle.new_state() for _ in samplers]
        self.n_threads = n_threads
        self.resets = 0

    def masks(self):
        return np.stack([s.mask(self.off, self.data, self.n_threads) for s in self.states])

    def step(self, masks):
        """Sample one token per row from `masks` and feed it.  Returns token ids (-1 = reset)."""
        out = []
        for b, s in enumerate(self.states):
            n = popcount(masks[b])
            if n == 0:
                self.states[b] = self.o.new_state()
                self.resets += 1
                out.append(-1)
                continue
            t = pick_set_bit(masks[b], self.samplers[b].below(n))
            assert s.feed_bytes(self.tokens[t])
            out.append(t)
        return out


def edge_vocab_json(seed: int = 7):
    """A JSON vocabulary that exercises the long and deep ends: every byte, tokens of 17-60 bytes (beyond the
    16 bytes a lane of the mask-automaton kernel fetches at once), and runs of up to 120 opening brackets
    (every nesting depth is another Earley set: more automaton states than a block keeps in LDS)."""
    from workloads.rng import stream
    rs = stream(seed, "edge-vocab")
    toks = [bytes([c]) for c in range(256)]
    alphabet = b'abcxyz019 ,:"[]{}-.e\\tn'
    for _ in range(300):
        n = 17 + rs.below(44)
        toks.append(bytes(alphabet[rs.below(len(alphabet))] for _ in range(n)))
    for k in range(1, 121):
        toks.append(b"[" * k)
        if k % 3 == 0:
            toks.append(b"[" * k + b"1,")
            toks.append(b"[" * (k // 2) + b'{"a":' + b"[" * (k // 2))
    toks += [b'"' + b"a" * 30 + b'"', b'"' + b"a" * 30 + b'":', b"1" * 40, b"1" * 20 + b"." + b"5" * 20 + b"e-" + b"3" * 10, b" " * 50, b'{"k":"' + b"v" * 25 + b'"}']
    return toks
