"""Writes tests/golden/trajectory_cfgN.txt: the seeded decode trajectories of the benchmark
configurations, produced by the CPU oracle alone.

At every step each row draws its next token uniformly from the oracle-valid mask
(r = next_u64(sample[row]) mod popcount, the r-th set bit in id order); a row whose mask is
empty is reset (token id -1).  Only `oracle/` and `workloads/` are used here, so the files
never depend on the HIP library.

usage: python tests/golden/make_trajectories.py CFG [ROWS [STEPS]]
"""
import os
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from oracle import Oracle                      # noqa: E402
from workloads import configs                  # noqa: E402
from tests.helpers import OracleRun            # noqa: E402


def main():
    idx = int(sys.argv[1])
    cfg = configs.CONFIGS[idx]
    rows = int(sys.argv[2]) if len(sys.argv) > 2 else cfg.batch
    steps = int(sys.argv[3]) if len(sys.argv) > 3 else cfg.steps
    toks = cfg.vocab()
    run = OracleRun(Oracle(cfg.grammar()), toks, [cfg.sampler(b) for b in range(rows)], n_threads=8)
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), f"trajectory_cfg{idx}.txt")
    t0 = time.time()
    lines = []
    for step in range(steps):
        ids = run.step(run.masks())
        lines.append(" ".join(map(str, ids)))
        if step % 16 == 0:
            print(f"cfg{idx} step {step}/{steps} {time.time() - t0:.0f}s", flush=True)
    with open(out, "w") as f:
        f.write(f"# config {idx} ({cfg.name}): V={cfg.V} rows={rows} steps={steps} seed={cfg.seed}\n")
        f.write("# one line per decode step: the token id fed to each row (-1 = the row was reset)\n")
        f.write("# written by tests/golden/make_trajectories.py from the CPU oracle only\n")
        f.write("\n".join(lines) + "\n")
    print("wrote", out, f"{time.time() - t0:.0f}s resets={run.resets}")


if __name__ == "__main__":
    main()
