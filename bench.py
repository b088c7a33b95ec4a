#!/usr/bin/env python3
"""Benchmark of the per-decode-step vocabulary mask on one MI355X.

A "step" is one pass of the whole hot path over one batch: advance every row by its next
token (host Earley + ZapFormat compaction), compute_mask (chart pack into a pinned slot the kernels read in place, mask-automaton
kernel, closing kernel = fallback pass + bit permutation; enqueued with compute_mask_async), apply_mask on that
step's logits, and mask_wait (waits until the mask kernels have reported their status: deferred error check).  The token
trajectory is fixed beforehand (tests/golden/trajectory_cfgN.txt, sampled by the CPU oracle;
if the file does not cover the request the library extends it untimed), so nothing is copied
back to the host inside the timed region.  Inputs are seeded and synthetic.

Prints ONE JSON line.  `value` = batch * V * steps / wall time of the timed region.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# instruction issue peak of the chip: 256 compute units x 4 SIMDs x one wavefront instruction per cycle x 2.4 GHz
ISSUE_PEAK_GINST = 256 * 4 * 2.4

# HBM traffic of one mask_automaton_kernel launch on the default workload, from rocprofv3 FETCH_SIZE / WRITE_SIZE runs
# scaled by a plain copy of known size (profiles/mask_automaton_kernel_cfg3_hbm_traffic.txt).  It describes the kernel
# sources with the digest below; once they change the figure is reported as null until it is measured again.
# instructions_per_launch: SQ_INSTS of the same kernel and workload (profiles/mask_automaton_kernel_cfg3_sq_counters.txt).
MEASURED_TRAFFIC = {"config": 3, "bytes_per_launch": 3752300, "apply_bytes_per_launch": 8508600, "instructions_per_launch": 8817397,
                    "kernel_sources_sha256": "fb07c53142256e51fdcb2b868376daab5f75595b7543af9a95834953dfdf91f2"}


def kernel_sources_digest():
    import hashlib
    h = hashlib.sha256()
    for name in ("zf_kernels.hip", "zf_mask_automaton.hip", "zf_mask_walk.hip", "zf_kernel_common.h", "zf_launch.h", "zf_device.h"):
        with open(os.path.join(ROOT, "paper_2506_01151_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def load_trajectory(idx, rows, steps):
    path = os.path.join(ROOT, "tests", "golden", f"trajectory_cfg{idx}.txt")
    if not os.path.exists(path):
        return []
    traj = [[int(x) for x in line.split()] for line in open(path) if line.strip() and not line.startswith("#")]
    if not traj or len(traj[0]) < rows:
        return []
    return [t[:rows] for t in traj[:steps]]


def extend_trajectory(zf, eng, cfg, traj, rows, steps):
    """Continue the trajectory with the library itself (untimed set-up work)."""
    import numpy as np
    import torch
    from workloads.configs import pick_set_bit
    from workloads.rng import stream
    states = [eng.new_state() for _ in range(rows)]
    for ids in traj:
        for b, t in enumerate(ids):
            states[b].reset() if t < 0 else states[b].advance(t)
    rs = [stream(cfg.seed, f"bench-extend[{b}]") for b in range(rows)]
    d_mask = torch.empty((rows, eng.W), dtype=torch.int32, device="cuda")
    while len(traj) < steps:
        zf.compute_mask(eng, states, d_mask)
        m = d_mask.cpu().numpy().view(np.uint32)
        ids = []
        for b in range(rows):
            n = int(np.unpackbits(m[b].view(np.uint8)).sum())
            if n == 0:
                states[b].reset()
                ids.append(-1)
            else:
                t = pick_set_bit(m[b], rs[b].below(n))
                states[b].advance(t)
                ids.append(t)
        traj.append(ids)
    return traj


def cpu_baseline(cfg, toks, traj, budget_s=15.0):
    """The CPU oracle's mask loop, timed on this host on a bounded sample of (step, row)."""
    from oracle import Oracle
    from workloads import vocab as wvocab
    orc = Oracle(cfg.grammar())
    off, data = wvocab.vocab_csr(toks)
    rows = len(traj[0])
    states = [orc.new_state() for _ in range(rows)]
    n_masks, spent, threads = 0, 0.0, 1
    sample_steps = []
    stride = 1
    for step, ids in enumerate(traj):
        if step % stride == 0 and spent < budget_s:
            t0 = time.perf_counter()
            for s in states:
                s.mask(off, data, 0)
                n_masks += 1
            spent += time.perf_counter() - t0
            threads = orc.last_threads
            sample_steps.append(step)
        for b, t in enumerate(ids):
            if t < 0:
                states[b] = orc.new_state()
            else:
                states[b].feed_bytes(toks[t])
    return {"value": n_masks * len(toks) / spent, "unit": "vocab tokens checked/s", "cores": threads, "kind": "oracle",
            "sample": f"{n_masks} masks: all {rows} rows at {len(sample_steps)} steps (every {stride}th) of the same trajectory, {spent:.1f} s"}


def apply_mask_sweep(zf, eng, torch, dtype, batches=(16, 64, 256, 1024), launches=24):
    """apply_mask alone at growing batch: each launch works on rows it has not touched for more than
    1.5 GB of traffic (input and output rotate through 3072-row tensors), so nothing is served from
    the last-level cache.  HIP events on the launch stream around `launches` back-to-back calls."""
    V, W = eng.V, eng.W
    R = 3072
    x = torch.randn((R, V), dtype=torch.float32, device="cuda").to(dtype) if dtype != torch.float32 else torch.randn((R, V), device="cuda")
    y = torch.empty_like(x)
    m = torch.randint(-2**31, 2**31 - 1, (R, W), dtype=torch.int32, device="cuda")
    esz = x.element_size()
    rows = []
    for B in batches:
        at = 0
        for timed in (False, True):
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(launches):
                zf.apply_mask(eng, x[at:at + B], m[at:at + B], out=y[at:at + B])
                at = (at + B) % R
            e1.record()
            torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / launches
        nbytes = 2 * B * V * esz + B * W * 4
        rows.append({"batch": B, "us_per_launch": us, "GB/s": nbytes / us / 1e3, "frac": nbytes / us / 1e3 / HBM_PEAK_GBS})
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=512)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pruning", type=int, default=1)
    ap.add_argument("--walk-mode", type=int, default=0, help="mask kernel of the headline pass: 0 = mask automaton (default), 1 = trie walk")
    ap.add_argument("--headline-only", action="store_true",
                    help="run the warm-up and timed steps of the headline pass and nothing else (for hardware-counter runs, "
                         "where every dispatch of a kernel should belong to the same workload); prints a short JSON line")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="only run apply_mask with an all-ones mask on a [1024, V] tensor three times: a plain copy of known "
                         "size, used to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("this benchmark runs on one GPU only: rows and vocabulary ranges would shard without any exchange, "
              "but no multi-GPU path is part of it; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2506_01151_amd as zf
    from workloads import configs

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    cfg = configs.CONFIGS[args.config]
    B, K, Wm = cfg.batch, args.steps, args.warmup
    toks = cfg.vocab()
    # headline engine: state cache off, so every row of every step goes through the mask kernels
    eng = zf.Engine(cfg.grammar(), toks, device=0, pruning=bool(args.pruning), state_cache_entries=-1, walk_mode=args.walk_mode)
    V, W = eng.V, eng.W
    need = max(K, Wm)
    traj = load_trajectory(args.config, B, need)
    traj_src = "oracle-sampled file"
    if len(traj) < need:
        traj_src = f"oracle-sampled file ({len(traj)} steps) extended by the library"
        traj = extend_trajectory(zf, eng, cfg, traj, B, need)

    if args.traffic_calibration:
        x = torch.zeros((1024, V), dtype=torch.bfloat16, device="cuda")
        y = torch.empty_like(x)
        ones = torch.full((1024, W), -1, dtype=torch.int32, device="cuda")
        for _ in range(3):
            zf.apply_mask(eng, x, ones, out=y)
        torch.cuda.synchronize()
        print(json.dumps({"calibration_copy_bytes_read": x.numel() * 2 + ones.numel() * 4, "calibration_copy_bytes_written": y.numel() * 2}))
        return

    n_logit_bufs = 4
    logits = [configs.make_logits(cfg, i, device="cuda") for i in range(n_logit_bufs)]
    out = torch.empty_like(logits[0])
    d_mask = torch.empty((B, W), dtype=torch.int32, device="cuda")
    esz = logits[0].element_size()

    def run(eng, n_warm, n_timed, profile, count_hits=False, sync_steps=True):
        eng.set_profiling(profile)
        states = zf.StateBatch([eng.new_state() for _ in range(B)])
        lat, adv, kern, ovf, hits, queued = [], [], {"main": [], "finish": [], "apply": []}, 0, 0, 0
        psteps = crows = 0
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_timed)] if profile else None
        t_begin = None
        stream = torch.cuda.current_stream()
        for i in range(n_warm + n_timed):
            if i == n_warm:     # the timed steps replay the trajectory from its first step
                for s in states:
                    s.reset()
                eng.clear_state_cache()                     # what warm-up cached must not serve the timed steps
                torch.cuda.synchronize()
                t_begin = time.perf_counter()
            ids = traj[i if i < n_warm else i - n_warm]
            t0 = time.perf_counter()
            states.advance(ids)                             # every row by its token (a negative id starts the row over)
            t1 = time.perf_counter()
            zf.compute_mask_async(eng, states, d_mask)      # enqueue only: apply_mask queues right behind the mask kernels
            if profile and i >= n_warm:
                evs[i - n_warm][0].record()
            zf.apply_mask(eng, logits[i % n_logit_bufs], d_mask, out=out)
            if profile and i >= n_warm:
                evs[i - n_warm][1].record()
            zf.mask_wait(eng)                               # returns once the mask kernels have reported (overflow, if any); apply_mask may still run
            if sync_steps:                                  # latency passes: until the masked logits are there
                stream.synchronize()
            t2 = time.perf_counter()
            if i >= n_warm:
                adv.append(t1 - t0)
                lat.append(t2 - t1)
                if count_hits:                              # bookkeeping of the state-cache pass only: it is not part of the step
                    hits += eng.mask_report().cache_hits
                if profile:
                    r = eng.mask_report()
                    kern["main"].append(r.main_ms)
                    kern["finish"].append(r.permute_ms)   # the closing kernel: fallback pass (if any) + permutation
                    ovf += r.overflow_chunks
                    queued += r.walk_chunks
                    psteps += r.parser_steps
                    crows += r.cache_rows
        torch.cuda.synchronize()
        total = time.perf_counter() - t_begin
        if profile:
            kern["apply"] = [a.elapsed_time(b) for a, b in evs]
        return total, lat, adv, kern, ovf, eng.mask_report().chart_bytes, hits, (queued, psteps, crows)

    # headline pass: K steps back to back (the host moves on to the next step's advance as soon as the mask kernels have reported; the
    # stream orders apply_mask before the next step's kernels), bracketed by full synchronisation
    total, _, adv, _, _, _, _, _ = run(eng, Wm, K, False, sync_steps=False)
    if args.headline_only:
        print(json.dumps({"headline_only": True, "steps": K, "warmup": Wm, "ms_per_step": total / K * 1e3, "value": B * V * K / total}))
        return
    sync_total, lat, _, _, _, _, _, _ = run(eng, Wm, K, False)                              # latency pass: every step waits for its masked logits
    _, _, _, kern, ovf, chart_bytes, _, (queued, psteps, crows) = run(eng, Wm, K, True)     # same steps again with HIP events around each kernel
    # the same steps with the state cache (Section 5.2) on, starting cold: reported beside the headline
    eng_sc = zf.Engine(cfg.grammar(), toks, device=0, pruning=bool(args.pruning), walk_mode=args.walk_mode)
    sc_total, sc_lat, _, _, _, _, sc_hits, _ = run(eng_sc, Wm, K, False, count_hits=True)
    del eng_sc
    # and with the other mask kernel (trie walk when the headline runs the mask automaton), state cache off
    eng_alt = zf.Engine(cfg.grammar(), toks, device=0, pruning=bool(args.pruning), state_cache_entries=-1, walk_mode=1 - args.walk_mode)
    alt_total, alt_lat, _, _, _, _, _, _ = run(eng_alt, Wm, K, False)
    del eng_alt
    # what one row's automaton looks like, from the host twin of the kernel on every 16th step (the kernel
    # builds a row's automaton once per block, so its own step count is a multiple of this)
    live = {"states": 0, "steps": 0, "lookups": 0, "undecided": 0, "masks": 0}
    tw = [eng.new_state() for _ in range(B)]
    for i, ids in enumerate(traj[:K]):
        for b in range(B):
            tw[b].reset() if ids[b] < 0 else tw[b].advance(ids[b])
        if i % 16 == 0:
            for b in range(B):
                _, st = tw[b].debug_host_mask_automaton()
                for k in ("states", "steps", "lookups", "undecided"):
                    live[k] += st[k]
                live["masks"] += 1

    ms_per_step = total / K * 1e3
    value = B * V * K / total
    pct = lambda xs, p: sorted(xs)[min(len(xs) - 1, int(p * len(xs)))]
    info = eng.info
    main_ms = statistics.fmean(kern["main"])
    apply_ms = statistics.fmean(kern["apply"])
    # algorithmic bytes of one mask-kernel launch (mask automaton): the token-mask-cache rows merged (two bitsets of
    # Wr words per selected row), the rank-ordered verdict words written, 24 bytes per undecided string (its first 16
    # byte classes and two offsets) and the uploaded charts.  (Trie walk: the trie nodes and chunk tables instead.)
    Wr = (info.n_strings + 31) // 32
    if args.walk_mode == 0:
        mask_bytes = int(crows / K * Wr * 8 + B * Wr * 4 + queued / K * 24 + chart_bytes)
    else:
        n_chunks = (info.n_strings + 31) // 32
        mask_bytes = info.n_trie_nodes * 16 + n_chunks * (8 + 64) + chart_bytes + B * n_chunks * 4
    apply_bytes = 2 * B * V * esz + B * W * 4
    traffic_ok = (args.config == MEASURED_TRAFFIC["config"] and args.pruning == 1 and args.walk_mode == 0
                  and kernel_sources_digest() == MEASURED_TRAFFIC["kernel_sources_sha256"])
    kname = "mask_automaton_kernel" if args.walk_mode == 0 else "mask_walk_kernel"
    result = {
        "metric": "vocab tokens checked/sec + p50 mask+apply latency per step (V=128k, B=16)",
        "value": value, "unit": "vocab tokens checked/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32", "data": "synthetic",
        "config": {"workload": f"configs[{args.config - 1}] {cfg.name}: grammar={cfg.grammar().name} V={V} batch={B} "
                               f"logits={cfg.dtype} pruning={'on' if args.pruning else 'off'}", "trajectory": traj_src,
                   "mask_kernel": kname},
        "decode_tokens_per_s": B * K / total,      # one constraint-satisfying token per row and step (the unit of the paper's Table 1)
        "paper_context": "Table 1 of the paper: 8,207.85 tokens/s for its CPU engine on Llama3 / json_schema (parsing + mask generation, "
                         "RTX 3090 + EPYC 7452 host, real tokenizer and data): other hardware, other inputs; context, not a baseline",
        "synchronised_steps": {"ms_per_step": sync_total / K * 1e3, "value": B * V * K / sync_total,
                               "note": "the same steps with the stream synchronised at the end of every step (a decode loop that samples on the "
                                       "host before it advances); the latency percentiles come from this pass"},
        "p50_mask_apply_latency_us": pct(lat, 0.5) * 1e6, "p90_mask_apply_latency_us": pct(lat, 0.9) * 1e6,
        "p99_mask_apply_latency_us": pct(lat, 0.99) * 1e6,
        "mean_advance_us_per_step": statistics.fmean(adv) * 1e6,
        "kernel_ms": {k: statistics.fmean(v) for k, v in kern.items()},
        "kernel_ms_p50": {k: pct(v, 0.5) for k, v in kern.items()},
        "overflow_chunks_per_step": ovf / K,
        "undecided_strings_per_step" if args.walk_mode == 0 else "walk_chunks_per_step": queued / K,
        "earley_steps_per_launch": psteps / K,
        "token_mask_cache_rows_per_step": crows / K,
        "automaton_per_mask_host_twin": {"states": live["states"] / live["masks"], "earley_steps": live["steps"] / live["masks"],
                                         "transition_lookups": live["lookups"] / live["masks"], "undecided_strings": live["undecided"] / live["masks"]},
        "with_state_cache": {"value": B * V * K / sc_total, "ms_per_step": sc_total / K * 1e3,
                             "p50_mask_apply_latency_us": pct(sc_lat, 0.5) * 1e6, "p99_mask_apply_latency_us": pct(sc_lat, 0.99) * 1e6,
                             "row_hit_rate": sc_hits / (B * K),
                             "note": "cache cleared when the timed steps start; the headline value runs with it off"},
        "other_mask_kernel": {"kernel": "mask_walk_kernel" if args.walk_mode == 0 else "mask_automaton_kernel", "value": B * V * K / alt_total,
                              "ms_per_step": alt_total / K * 1e3, "p50_mask_apply_latency_us": pct(alt_lat, 0.5) * 1e6},
        "roofline": {"bound": "hbm", "kernel": kname, "achieved": mask_bytes / (main_ms * 1e-3) / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": mask_bytes / (main_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "traffic": MEASURED_TRAFFIC["bytes_per_launch"] if traffic_ok else None, "algorithmic_bytes": mask_bytes,
                     "note": "integer work: lazily built automaton of Earley sets + table look-ups per string; bound by the latency of the "
                             "dependent chain of Earley byte steps a block has to take (a few microseconds each), far below the HBM roof; "
                             "the event pair also spans the dispatch gap before the kernel"},
        # second view of the mask kernel: wavefront instructions issued per second against what the SIMDs could issue.  The
        # kernel is neither: it waits (LDS round trips, transitions other wavefronts are computing); the fraction says how much.
        "roofline_issue": {"bound": "alu", "kernel": kname, "unit": "G wavefront instructions/s", "peak": ISSUE_PEAK_GINST,
                           "instructions": MEASURED_TRAFFIC["instructions_per_launch"] if traffic_ok else None,
                           "achieved": MEASURED_TRAFFIC["instructions_per_launch"] / (main_ms * 1e-3) / 1e9 if traffic_ok else None,
                           "frac": MEASURED_TRAFFIC["instructions_per_launch"] / (main_ms * 1e-3) / 1e9 / ISSUE_PEAK_GINST if traffic_ok else None,
                           "note": "instruction count from the SQ_INSTS counter of the profiled run (null once the kernel sources change)"},
        "roofline_apply_mask": {"bound": "hbm", "kernel": "apply_mask_vec_kernel", "achieved": apply_bytes / (apply_ms * 1e-3) / 1e9,
                                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": apply_bytes / (apply_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                "traffic": MEASURED_TRAFFIC["apply_bytes_per_launch"] if traffic_ok else None, "algorithmic_bytes": apply_bytes,
                                "note": "launch bound at this shape (8.5 MB per launch); see apply_mask_sweep for the bandwidth-bound shapes"},
    }
    result["apply_mask_sweep"] = {"dtype": str(logits[0].dtype).replace("torch.", ""), "V": V, "bound": "hbm", "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                  "rows": apply_mask_sweep(zf, eng, torch, logits[0].dtype)}
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, toks, traj[:K])
    print(json.dumps(result))


if __name__ == "__main__":
    main()
