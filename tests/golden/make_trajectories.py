"""Writes tests/golden/trajectory_cfgN.txt: the seeded decode trajectories of the benchmark
configurations, produced by the CPU oracle alone.

At every step each row draws its next token uniformly from the oracle-valid mask
(r = next_u64(sample[row]) mod popcount, the r-th set bit in id order); a row whose mask is
empty is reset (token id -1).  Only `oracle/` and `workloads/` are used here, so the files
never depend on the HIP library.

The oracle keeps every Earley set, so on the ambiguous expression grammar a mask costs more
with every step; `--budget-s` ends the run after that much wall time and the header states
how many steps were reached and how long they took.

With `--resume` a file cut short is continued: its steps are fed to fresh oracle states again
(one sampler draw per fed token, as in the original run) and sampling goes on from there.

usage: python tests/golden/make_trajectories.py CFG [ROWS [STEPS]] [--budget-s SECONDS] [--threads N] [--resume]
"""
import argparse
import os
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from oracle import Oracle                      # noqa: E402
from workloads import configs                  # noqa: E402
from tests.helpers import OracleRun            # noqa: E402


def write(path, cfg, rows, lines, seconds, threads, finished):
    tmp = path + ".tmp"
    with open(tmp, "w") as f:
        f.write(f"# config {cfg.index} ({cfg.name}): V={cfg.V} rows={rows} steps={len(lines)} seed={cfg.seed}\n")
        f.write("# one line per decode step: the token id fed to each row (-1 = the row was reset)\n")
        f.write("# written by tests/golden/make_trajectories.py from the CPU oracle only\n")
        f.write(f"# oracle wall time {seconds:.0f} s on {threads} threads" + ("" if finished else " (run still going or cut short)") + "\n")
        f.write("\n".join(lines) + "\n")
    os.replace(tmp, path)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("cfg", type=int)
    ap.add_argument("rows", type=int, nargs="?")
    ap.add_argument("steps", type=int, nargs="?")
    ap.add_argument("--budget-s", type=float, default=0.0, help="stop after this much wall time (0 = run all steps)")
    ap.add_argument("--threads", type=int, default=8)
    ap.add_argument("--out", default=None)
    ap.add_argument("--resume", action="store_true", help="continue the steps the output file already holds")
    a = ap.parse_args()
    cfg = configs.CONFIGS[a.cfg]
    rows = a.rows or cfg.batch
    steps = a.steps or cfg.steps
    toks = cfg.vocab()
    run = OracleRun(Oracle(cfg.grammar()), toks, [cfg.sampler(b) for b in range(rows)], n_threads=a.threads)
    out = a.out or os.path.join(os.path.dirname(os.path.abspath(__file__)), f"trajectory_cfg{a.cfg}.txt")
    t0 = time.time()
    lines = []
    if a.resume and os.path.exists(out):
        import re
        text = open(out).read()
        spent = re.search(r"oracle wall time (\d+) s", text)
        t0 -= float(spent.group(1)) if spent else 0.0
        for line in text.splitlines():
            if not line.strip() or line.startswith("#"):
                continue
            ids = [int(x) for x in line.split()]
            assert len(ids) == rows, "the file to resume has another number of rows"
            for b, t in enumerate(ids):
                if t < 0:
                    run.states[b] = run.o.new_state()
                    run.resets += 1
                else:
                    run.samplers[b].next_u64()             # the draw that picked t
                    assert run.states[b].feed_bytes(toks[t])
            lines.append(line.strip())
        print(f"resumed {len(lines)} steps", flush=True)
    for step in range(len(lines), steps):
        ids = run.step(run.masks())
        lines.append(" ".join(map(str, ids)))
        if step % 8 == 7 or step == steps - 1:     # the file on disk is always a usable prefix
            write(out, cfg, rows, lines, time.time() - t0, a.threads, step == steps - 1)
            print(f"cfg{a.cfg} step {step + 1}/{steps} {time.time() - t0:.0f}s", flush=True)
        if a.budget_s and time.time() - t0 > a.budget_s:
            break
    write(out, cfg, rows, lines, time.time() - t0, a.threads, True)
    print("wrote", out, f"{len(lines)} steps {time.time() - t0:.0f}s resets={run.resets}")


if __name__ == "__main__":
    main()
