#!/usr/bin/env python3
"""Benchmark of the constrained-decoding hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic input:
compile every constraint of the workload into its token-level table (plus the
stacking of tables for the multi-constraint workload), then run the workload's
decode steps (mask, argmax, advance) with states chained on the device.

    python bench.py --gpus 1 --steps K --warmup W [--workload c3]

prints ONE JSON line.  `value` is sequence-steps per second of the whole step
(compile time included); the compile-only and decode-only rates are extra keys.
`roofline` is for the decode-step kernel, `roofline_compile` for the table
kernel; both come from HIP events recorded inside the timed region.
`cpu_baseline` is the CPU oracle on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
METRIC = "token-DFA transitions/s (compile) + decode mask steps*seq/s, % HBM roofline"
WORKLOAD_NAMES = {
    "c1": "tiny: 15-state API-call regex, 512 tokens, batch 4 fp32, 16 steps",
    "c2": "JSON-schema-like object regex, 32,000 tokens, batch 64 bf16, 256 steps",
    "c3": "API-call union of 50 signatures, 128,256 tokens, batch 256 bf16, 512 steps",
    "c4": "stress compile: random 20,000-state DFA, 256,000 tokens (no decode stage)",
    "c5": "64 JSON-like constraints stacked, 128,256 tokens, batch 1,024 bf16, 512 steps",
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c3", choices=sorted(WORKLOAD_NAMES))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="launch decode steps one by one instead of a HIP graph")
    ap.add_argument("--cpu-seconds", type=float, default=20.0, help="target CPU time for the oracle sample")
    ap.add_argument("--roofline-launches", type=int, default=256,
                    help="launches of the decode step's byte-bound leg (every sequence in the widest state)")
    ap.add_argument("--roofline-repeats", type=int, default=8, help="times that leg is run, back to back")
    ap.add_argument("--logits-dtype", choices=["f32", "bf16"], default=None,
                    help="element type of the logits, instead of the workload's own")
    ap.add_argument("--write-masked", action="store_true",
                    help="decode steps also write the masked logits back in place (doubles the algorithmic bytes)")
    ap.add_argument("--no-union", action="store_true",
                    help="several constraints: one batched launch over the separate automata instead of their union")
    ap.add_argument("--no-create-in-step", action="store_true",
                    help="create the automata once, outside the timed steps (the kernels alone are timed)")
    ap.add_argument("--no-extras", action="store_true", help="skip the measurements that are not part of a step")
    ap.add_argument("--no-per-config", action="store_true",
                    help="default workload only: skip the extra c4 and c5 measurements")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="also run one plain 1 GiB device copy before the timed region (reference for HBM byte counters)")
    return ap.parse_args()


def cpu_baseline(w, units_per_step: float, unit: str, target_s: float):
    """The oracle as it stands, timed on this host on a bounded sample and scaled linearly."""
    import oracle
    from workloads import logits as LG
    threads = min(oracle.max_threads(), len(os.sched_getaffinity(0)))
    V = w.vocab.n_tokens
    total_rows = sum(d.n_states for d in w.dfas)
    # compile sample: composition oracle on the first rows of the first constraint(s)
    d0 = w.dfas[0]
    probe = min(d0.n_states, 2 * threads)
    t0 = time.perf_counter()
    oracle.compile_compose(d0.trans, w.vocab.data, w.vocab.offsets, q_lo=0, q_hi=probe, block=2, n_threads=threads)
    t_probe = time.perf_counter() - t0
    rows = int(min(d0.n_states, max(probe, probe * (0.5 * target_s) / max(t_probe, 1e-6))))
    t0 = time.perf_counter()
    oracle.compile_compose(d0.trans, w.vocab.data, w.vocab.offsets, q_lo=0, q_hi=rows, block=2, n_threads=threads)
    t_rows = time.perf_counter() - t0
    t_compile_full = t_rows * total_rows / rows
    sample = f"compile: {rows} of {total_rows} rows by explicit composition"
    t_mask_full = 0.0
    if w.mask is not None:
        m = w.mask
        # table rows the sampled steps can reach are those of the start state only: use a walk table of
        # the first constraint for the oracle's lookups
        tab = oracle.compile_walk(d0.trans, w.vocab.data, w.vocab.offsets, n_threads=threads)
        states = np.full(m.batch, d0.start, dtype=np.int32)
        dt = oracle.F32 if m.dtype == "f32" else oracle.BF16
        lg = [LG.gen_logits(1, s, min(m.batch, 64), V, m.sigma, m.dtype) for s in range(2)]
        lg = [np.tile(x, ((m.batch + x.shape[0] - 1) // x.shape[0], 1))[:m.batch] for x in lg]
        n_meas, t_meas = 0, 0.0
        while t_meas < 0.5 * target_s and n_meas < m.steps:
            t0 = time.perf_counter()
            tok, states_new = oracle.mask_step(tab, lg[n_meas % 2], dt, states, n_threads=threads)
            t_meas += time.perf_counter() - t0
            states = np.where(states_new >= 0, states_new, d0.start).astype(np.int32)
            n_meas += 1
        t_mask_full = t_meas * m.steps / n_meas
        sample += f"; decode: {n_meas} of {m.steps} steps at batch {m.batch}"
    sample += "; scaled linearly to one full step"
    return {"value": units_per_step / (t_compile_full + t_mask_full), "unit": unit, "cores": threads,
            "kind": "oracle", "sample": sample,
            "compile_s_full": t_compile_full, "decode_s_full": t_mask_full}


def recorded_traffic(workload, kernel):
    """HBM bytes per launch that the committed counter summary holds for `kernel` on `workload`, or None when
    there is no such summary or the kernel's source file has changed since the counters were taken."""
    import hashlib
    import re
    root = os.path.dirname(os.path.abspath(__file__))
    try:
        text = open(os.path.join(root, "profiles", f"hbm_traffic_{workload}.txt")).read()
    except OSError:
        return None
    for mt in re.finditer(r"^traffic kernel=(\S+) bytes_per_launch=(\d+) source=(\S+) sha256=([0-9a-f]+)$", text, re.M):
        if mt.group(1) != kernel:
            continue
        try:
            src = open(os.path.join(root, "paper_2407_08103_amd", "csrc", mt.group(3)), "rb").read()
        except OSError:
            return None
        return int(mt.group(2)) if hashlib.sha256(src).hexdigest() == mt.group(4) else None
    return None


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path; run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2407_08103_amd as T
    from workloads import configs, logits as LG

    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    out, w, units_per_step, unit = measure(args, args.workload, args.steps, args.warmup, not args.no_extras)
    # The other workloads, in the same run and on the same device: c1 and c2 (small: bound by their launches),
    # c4 (the largest table; no decode stage) and c5 (the largest decode).  Fewer repeats; HIP events.
    if args.workload == "c3" and not args.no_per_config:
        per = {}
        for name in ("c1", "c2", "c4", "c5"):
            torch.cuda.empty_cache()
            o, _, _, _ = measure(args, name, 3, 1, False)
            e = {"workload": o["config"]["workload"], "n_states": o["config"]["n_states"], "n_tokens": o["config"]["n_tokens"],
                 "compile_ms": o["compile"]["ms"], "dfa_create_ms": o["compile"]["dfa_create_ms"],
                 "compile_transitions_per_s": o["compile"]["transitions_per_s"]}
            rc = o["roofline_compile"] if "roofline_compile" in o else o["roofline"]
            e["compile_frac"] = rc["frac"]
            e["compile_traffic"] = rc["traffic"]
            if "decode" in o:
                e["decode_us_per_launch"] = o["decode"]["us_per_launch"]
                e["decode_steps_that_chose_a_token"] = o["decode"]["steps_that_chose_a_token"]
                e["decode_us_per_launch_over_those_steps"] = o["decode"]["us_per_launch_over_those_steps"]
                e["decode_seq_steps_per_s"] = o["decode"]["seq_steps_per_s"]
                e["decode_frac"] = o["roofline"]["frac"]              # of the byte-bound leg (widest state), not of the decode mix
                e["decode_frac_us_per_launch"] = o["roofline"]["us_per_launch"]
                e["decode_gb_per_s"] = o["roofline"]["achieved"]
                e["decode_traffic"] = o["roofline"]["traffic"]
            per[name] = e
        out["per_config"] = per
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, units_per_step, unit, args.cpu_seconds)
    print(json.dumps(out))


def measure(args, workload, steps, warmup, extras):
    """One workload: set-up, `warmup` untimed steps, `steps` timed steps; returns the result object.
    `extras` adds the measurements that are not part of a step (speculated runs, sampling, packed table)."""
    import torch
    import paper_2407_08103_amd as T
    from workloads import configs, logits as LG
    dev = torch.device("cuda:0")
    w = configs.get(workload)
    V = w.vocab.n_tokens
    n_constraints = len(w.dfas)
    total_rows = sum(d.n_states for d in w.dfas)
    entries = total_rows * V

    # ---- setup (untimed): vocabulary packing, automata upload, output buffers, logits
    vocab = T.Vocab(w.vocab.data, w.vocab.offsets)
    # Per constraint, and so inside every timed step: validation, the lane order and jump tables (host
    # threads), upload, and for several constraints their disjoint union (one automaton whose table is
    # the stacked table).  Returns the handles; the previous step's are released here, not timed.
    def create_all():
        if n_constraints > 1 and not args.no_union:
            # the union is made from the automata as they are on the host: one upload, one plan
            un, un_offs = T.dfa_union_host([(d.trans, d.accept, d.start) for d in w.dfas])
            return [un], un, un_offs
        return [T.CharDFA(d.trans, d.accept, d.start) for d in w.dfas], None, None

    torch.cuda.synchronize()
    t_create = time.perf_counter()
    dfas, union, union_offs = create_all()
    torch.cuda.synchronize()
    create_ms = [(time.perf_counter() - t_create) * 1e3]
    rw = T.allow_row_words(V)
    bufs = [(torch.empty((d.n_states, V), dtype=torch.int32, device=dev),
             torch.empty((d.n_states, rw), dtype=torch.int32, device=dev)) for d in w.dfas[:1]]
    m = w.mask
    if m is not None and args.logits_dtype:
        import dataclasses
        m = dataclasses.replace(m, dtype=args.logits_dtype)
        w = dataclasses.replace(w, mask=m)
    stream = torch.cuda.current_stream()

    big = None
    if n_constraints > 1:
        big = (torch.empty((total_rows, V), dtype=torch.int32, device=dev),
               torch.empty((total_rows, rw), dtype=torch.int32, device=dev))

    def compile_all():
        if n_constraints == 1:
            return T.compile_token_dfa(vocab, dfas[0], out=bufs[0]), np.array([0, w.dfas[0].n_states])
        if union is not None:
            return T.compile_token_dfa(vocab, union, out=big), union_offs
        return T.compile_stacked(vocab, dfas, out=big)      # each constraint straight into its slice

    table, offs = compile_all()
    torch.cuda.synchronize()

    graph = None
    if m is not None:
        B, S = m.batch, m.steps
        tdt = torch.float32 if m.dtype == "f32" else torch.bfloat16
        esz = 4 if m.dtype == "f32" else 2
        n_rot = max(2, min(S, int(np.ceil(640e6 / (B * V * esz)))))      # rotate > 2x the 256 MB last-level cache
        logits = [torch.empty((B, V), dtype=tdt, device=dev) for _ in range(n_rot)]
        seed = configs.logits_seed(w.config)
        for s in range(n_rot):
            LG.gen_logits_device(logits[s].data_ptr(), seed, s, B, V, V, m.sigma, m.dtype, stream.cuda_stream)
        binding = w.binding if w.binding is not None else np.zeros(B, dtype=np.int64)
        start = torch.from_numpy(np.array([offs[c] + w.dfas[c].start for c in binding], dtype=np.int32)).to(dev)
        states = torch.empty((S + 1, B), dtype=torch.int32, device=dev)
        tokens = torch.empty((S, B), dtype=torch.int32, device=dev)

        def decode_all(tab):
            states[0].copy_(start)
            for s in range(S):
                lg = logits[s % n_rot]
                T.mask_step(tab, lg, states[s], tokens[s], states[s + 1], lg if args.write_masked else None)

        decode_all(table)                      # also sizes the table's reduction scratch
        torch.cuda.synchronize()
        if not args.no_graph:
            # the table buffers are reused by every compile, so a graph captured once stays valid
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                decode_all(table)
            graph.replay()
            torch.cuda.synchronize()
        units_per_step = float(B * S)
        unit = "seq*steps/s"
    else:
        units_per_step = float(entries)
        unit = "state*token transitions/s"

    ev = lambda: torch.cuda.Event(enable_timing=True)

    def one_step(timed):
        nonlocal table, dfas, union, union_offs
        e0, e1, e2 = (ev(), ev(), ev()) if timed else (None, None, None)
        if not args.no_create_in_step:
            dfas = union = None                     # (their device memory goes back to the library's cache: no wait for the GPU)
            tc = time.perf_counter()
            dfas, union, union_offs = create_all()
            if timed:
                create_ms.append((time.perf_counter() - tc) * 1e3)
        if timed:
            e0.record()
        new_table, _ = compile_all()
        if graph is None:
            table = new_table          # same device buffers either way; the graph holds the first handle
        if timed:
            e1.record()
        if m is not None:
            if graph is not None:
                graph.replay()
            else:
                decode_all(table)
        if timed:
            e2.record()
        return e0, e1, e2

    if args.traffic_probe:
        src = torch.full((1 << 28,), 7, dtype=torch.int32, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(warmup):
        one_step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    events = [one_step(True) for _ in range(steps)]
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_compile = float(np.mean([e0.elapsed_time(e1) for e0, e1, _ in events]))
    dfa_create_ms = float(np.mean(create_ms[1:])) if len(create_ms) > 1 else create_ms[0]
    ms_decode = float(np.mean([e1.elapsed_time(e2) for _, e1, e2 in events])) if m is not None else 0.0
    ms_per_step = wall * 1e3 / steps
    value = units_per_step / (ms_per_step * 1e-3)

    pairs_path = (union if union is not None else dfas[0]).info()[2] == T.PATH_PAIRS if (n_constraints == 1 or union is not None) else False
    compile_kernel = ("sweep_expand_kernel (+ the sweep's list kernels)" if pairs_path
                      else "compile_tile_kernel (+ transpose_kernel, start_bytes_kernel)")
    compile_gbs = entries * 4 / (ms_compile * 1e-3) / 1e9
    roof_compile = {"bound": "hbm", "achieved": compile_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": compile_gbs / HBM_PEAK_GBS, "traffic": recorded_traffic(workload, "sweep" if pairs_path else "compile_tile"),
                    "kernel": compile_kernel, "ms_per_launch": ms_compile,
                    "bytes_per_launch": entries * 4, "includes_plan": False}
    out = {
        "metric": METRIC, "value": value, "unit": unit, "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int32" if m is None else ("int32+" + m.dtype), "data": "synthetic",
        "config": {"workload": f"{workload}: {WORKLOAD_NAMES[workload]}", "n_states": total_rows,
                   "n_tokens": V, "constraints": n_constraints, "table_entries": entries,
                   "decode_launch": "hip graph" if graph is not None else "stream"},
        "compile": {"ms": ms_compile, "transitions_per_s": entries / (ms_compile * 1e-3), "dfa_create_ms": dfa_create_ms,
                    "ms_with_dfa_create": ms_compile + dfa_create_ms,
                    "dfa_create_in_timed_step": not args.no_create_in_step,
                    "dfa_create_note": "tdfa_dfa_create for all constraints and their union (host-side check, lane order, jump "
                                       "tables, upload; blocking for the host): per constraint, so every timed step does it again, "
                                       "while the GPU still compiles and decodes the step before (the call waits for its own "
                                       "copies only, and a destroyed automaton's memory goes to a cache instead of hipFree); "
                                       "compile.ms and roofline_compile are the compile kernels alone"},
    }
    if m is not None:
        us_launch = ms_decode * 1e3 / m.steps
        logit_bytes = m.batch * V * esz * (2 if args.write_masked else 1)
        all_bytes = m.batch * (V * esz + V // 8 + 16)
        # What the decode's steps need of their logits: the 16-byte groups of eight tokens in which the
        # sequence's state allows a token (the step on 16-bit logits fetches only those where a state
        # allows few tokens), averaged over a sample of the steps.
        group_rows = table.allow.view(torch.uint8)
        probe = range(0, S, max(1, S // 16))
        needed = float(np.mean([(group_rows.index_select(0, states[s].clamp(min=0).long())[:, :V // 8] != 0).sum().item()
                                for s in probe])) * 8 * esz
        # The constraints of these workloads describe finite texts: a sequence that has completed its text sits in
        # a state that allows nothing (no token, state kept) for the rest of the steps.  How many steps still
        # chose a token, how many tokens were chosen, and the time per launch over just those first steps.
        chosen = tokens >= 0
        live_steps = int(chosen.any(dim=1).sum().item())
        n_chosen = int(chosen.sum().item())
        us_live = None
        if graph is not None and 0 < live_steps < S:
            prefix = torch.cuda.CUDAGraph()
            with torch.cuda.graph(prefix):
                states[0].copy_(start)
                for s in range(live_steps):
                    T.mask_step(table, logits[s % n_rot], states[s], tokens[s], states[s + 1],
                                logits[s % n_rot] if args.write_masked else None)
            prefix.replay()
            p0, p1 = ev(), ev()
            p0.record()
            for _ in range(3):
                prefix.replay()
            p1.record()
            torch.cuda.synchronize()
            us_live = p0.elapsed_time(p1) * 1e3 / (3 * live_steps)
        elif live_steps == S:
            us_live = us_launch
        out["decode"] = {"ms": ms_decode, "us_per_launch": us_launch, "seq_steps_per_s": units_per_step / (ms_decode * 1e-3),
                         "steps_that_chose_a_token": live_steps, "tokens_chosen": n_chosen,
                         "us_per_launch_over_those_steps": us_live,
                         "tokens_chosen_per_s": n_chosen / (ms_decode * 1e-3),
                         "batch": m.batch, "decode_steps": m.steps, "logits_buffers_rotated": n_rot,
                         "logit_bytes_per_launch": logit_bytes, "logit_bytes_in_groups_with_an_allowed_token": needed,
                         "traffic": recorded_traffic(workload, "mask_step_mix") if m.dtype == "bf16" and not args.write_masked else None,
                         "note": "steps in states that allow few tokens are bound by latency, not by bytes: see roofline for the "
                                 "byte-bound regime of the same kernel"}
        # The roofline of the step kernel is taken where the roofline binds: every sequence in the
        # workload's widest state, so that every group holds an allowed token and the whole row is
        # needed and read.  Timed here with events, after the timed steps; same launch shape.
        counts = torch.cat([(group_rows[r:r + 512, :V // 8] != 0).sum(1) for r in range(0, total_rows, 512)])
        widest = int(counts.argmax().item())
        wide_states = torch.full((B,), widest, dtype=torch.int32, device=dev)
        wide_new = torch.empty_like(wide_states)
        wide_tok = torch.empty_like(wide_states)
        n_wide = args.roofline_launches

        if args.write_masked:
            # the decode has masked the logits in place for its own states; this leg gets fresh ones
            for s in range(n_rot):
                LG.gen_logits_device(logits[s].data_ptr(), seed, s, B, V, V, m.sigma, m.dtype, stream.cuda_stream)
            wide_out = [torch.empty_like(x) for x in logits]

        def wide_all():
            for i in range(n_wide):
                lg = logits[i % n_rot]
                T.mask_step(table, lg, wide_states, wide_tok, wide_new, wide_out[i % n_rot] if args.write_masked else None)

        wide_all()
        torch.cuda.synchronize()
        wide_graph = None
        if not args.no_graph:                          # launched the way the decode is
            wide_graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(wide_graph):
                wide_all()
            wide_graph.replay()
            torch.cuda.synchronize()
        w0, w1 = ev(), ev()
        w0.record()
        for _ in range(args.roofline_repeats):
            wide_graph.replay() if wide_graph is not None else wide_all()
        w1.record()
        torch.cuda.synchronize()
        us_wide = w0.elapsed_time(w1) * 1e3 / (n_wide * args.roofline_repeats)
        gbs = logit_bytes / (us_wide * 1e-6) / 1e9
        out["roofline"] = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": gbs / HBM_PEAK_GBS,
                           "traffic": recorded_traffic(workload, "mask_step") if m.dtype == "bf16" and not args.write_masked else None,
                           "kernel": ("mask_step_bf16_kernel<true>" if args.write_masked else "mask_step_bf16_kernel<false>")
                           if m.dtype == "bf16" else ("mask_step_exact_kernel<0>" if args.write_masked else "mask_step_f32_kernel"),
                           "us_per_launch": us_wide, "bytes_per_launch": logit_bytes,
                           "achieved_with_mask_bytes": all_bytes / (us_wide * 1e-6) / 1e9,
                           "regime": f"{n_wide * args.roofline_repeats} launches with all {B} sequences in the state that allows the most tokens "
                                     f"({float(counts[widest].item()) * 8 / V:.0%} of the groups hold one): the whole row is needed and read",
                           "decode_mix_us_per_launch": us_launch}
        out["roofline_compile"] = roof_compile
        if extras:
            # not part of a step: runs of 8 speculated tokens (the greedy tokens of the first 8 decode
            # steps) checked under the constraint with their state history; latency-bound, 4 B per lookup
            k = min(8, m.steps)
            runs = tokens[:k].t().contiguous()
            hist = torch.empty((m.batch, k + 1), dtype=torch.int32, device=dev)
            n_valid = torch.empty((m.batch,), dtype=torch.int32, device=dev)
            for _ in range(3):
                T.advance_tokens(table, states[0], runs, hist, n_valid)
            a0, a1 = ev(), ev()
            a0.record()
            for _ in range(20):
                T.advance_tokens(table, states[0], runs, hist, n_valid)
            a1.record()
            torch.cuda.synchronize()
            out["speculated_runs"] = {"k": k, "batch": m.batch, "us_per_call": a0.elapsed_time(a1) * 1e3 / 20,
                                      "accepted": int(n_valid.sum().item()), "of": m.batch * k}
            # not part of a step: small automata (whose whole table fits the 160 KB of LDS of a compute unit)
            # compiled by the walk that reads the table from memory and by the one that stages it in LDS first
            from workloads.regex_dfa import compile_regex, random_dfa
            probe_rows = {}
            for pname, pd in (("key-value regex, 95 states", compile_regex(r'"[a-zA-Z_][a-zA-Z0-9_]{0,62}"\s*:\s*(-?\d{1,18}|true|false|null)')),
                              ("random automaton, 150 states", random_dfa(150, 0.6, 0.2, np.random.default_rng(2407)))):
                pt = (torch.empty((pd.n_states, V), dtype=torch.int32, device=dev), torch.empty((pd.n_states, rw), dtype=torch.int32, device=dev))
                res = {}
                for path_name, path in (("walk_ms", T.PATH_WALK), ("staged_ms", T.PATH_STAGED)):
                    ph = T.CharDFA(pd.trans, pd.accept, pd.start)
                    ph.compile_path(path)
                    for _ in range(3):
                        T.compile_token_dfa(vocab, ph, out=pt)
                    s0, s1 = ev(), ev()
                    s0.record()
                    for _ in range(20):
                        T.compile_token_dfa(vocab, ph, out=pt)
                    s1.record()
                    torch.cuda.synchronize()
                    res[path_name] = s0.elapsed_time(s1) / 20
                res["table_MB"] = pd.n_states * V * 4 / 1e6
                probe_rows[pname] = res
            out["lds_staged_walk"] = probe_rows
            # not part of a step either: the same decode with the token drawn at temperature 1 instead of
            # taken greedily.  Only allowed tokens cost arithmetic (a generator block and two logarithms
            # each), so the time follows the size of the allowed sets: reported for the decode as it runs
            # (small sets) and with every sequence put in the state that allows the most tokens.
            s_states = torch.empty_like(states)
            s_tokens = torch.empty_like(tokens)

            def sample_all():
                s_states[0].copy_(start)
                for s in range(S):
                    T.sample_step(table, logits[s % n_rot], s_states[s], 1.0, 2407, s, s_tokens[s], s_states[s + 1])

            sample_all()
            torch.cuda.synchronize()
            s_graph = None
            if not args.no_graph:
                s_graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(s_graph):
                    sample_all()
                s_graph.replay()
            b0, b1 = ev(), ev()
            b0.record()
            s_graph.replay() if s_graph is not None else sample_all()
            b1.record()
            torch.cuda.synchronize()
            probe = range(0, S, max(1, S // 8))
            allowed = float(np.mean([(table.delta.index_select(0, s_states[s].clamp(min=0).long()) >= 0).float().mean().item()
                                     for s in probe]))
            counts = torch.cat([(table.delta[r:r + 512] >= 0).sum(1) for r in range(0, total_rows, 512)])
            widest = int(counts.argmax().item())
            wide_states = torch.full((B,), widest, dtype=torch.int32, device=dev)
            wide_new = torch.empty_like(wide_states)
            for i in range(3):
                T.sample_step(table, logits[i % n_rot], wide_states, 1.0, 2407, i, s_tokens[0], wide_new)
            c0, c1 = ev(), ev()
            c0.record()
            for i in range(20):
                T.sample_step(table, logits[i % n_rot], wide_states, 1.0, 2407, i, s_tokens[0], wide_new)
            c1.record()
            torch.cuda.synchronize()
            c2 = ev()
            for i in range(20):                    # a sharper distribution: most logits cannot win whatever their noise
                T.sample_step(table, logits[i % n_rot], wide_states, 0.25, 2407, i, s_tokens[0], wide_new)
            c2.record()
            k0, k1, k2 = ev(), ev(), ev()
            for i in range(2):
                T.sample_step(table, logits[i % n_rot], s_states[S // 2], 1.0, 2407, i, s_tokens[0], wide_new, top_k=50)
            k0.record()
            for i in range(20):
                T.sample_step(table, logits[i % n_rot], s_states[S // 2], 1.0, 2407, i, s_tokens[0], wide_new, top_k=50)
            k1.record()
            for i in range(20):
                T.sample_step(table, logits[i % n_rot], wide_states, 1.0, 2407, i, s_tokens[0], wide_new, top_k=50)
            k2.record()
            torch.cuda.synchronize()
            out["sampled_decode"] = {"temperature": 1.0, "us_per_launch": b0.elapsed_time(b1) * 1e3 / S,
                                     "top_k_50": {"mid_decode_states_us_per_launch": k0.elapsed_time(k1) * 1e3 / 20,
                                                  "widest_state_us_per_launch": k1.elapsed_time(k2) * 1e3 / 20},
                                     "mean_allowed_fraction": allowed,
                                     "decode_launch": "hip graph" if s_graph is not None else "stream",
                                     "widest_state": {"allowed_fraction": float(counts[widest].item()) / V,
                                                      "us_per_launch": c0.elapsed_time(c1) * 1e3 / 20,
                                                      "us_per_launch_at_temperature_0.25": c1.elapsed_time(c2) * 1e3 / 20}}
            # not part of a step: the same table in edge-list form (targets of the edges only, the bit
            # rows kept), a set-up call, and the greedy decode on it
            torch.cuda.synchronize()
            tp0 = time.perf_counter()
            packed = T.table_pack(table)
            torch.cuda.synchronize()
            pack_ms = (time.perf_counter() - tp0) * 1e3
            p_targets, _, p_dir, _ = T.table_pack_arrays(packed)
            n_edges, dir_entries = int(p_targets.numel()), int(p_dir.numel())
            del p_targets, p_dir
            p_states = torch.empty_like(states)
            p_tokens = torch.empty_like(tokens)

            def decode_packed():
                p_states[0].copy_(start)
                for s in range(S):
                    T.mask_step(packed, logits[s % n_rot], p_states[s], p_tokens[s], p_states[s + 1])

            decode_packed()
            torch.cuda.synchronize()
            p_graph = None
            if not args.no_graph:
                p_graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(p_graph):
                    decode_packed()
                p_graph.replay()
            d0, d1 = ev(), ev()
            d0.record()
            p_graph.replay() if p_graph is not None else decode_packed()
            d1.record()
            torch.cuda.synchronize()
            out["packed_table"] = {"edges": n_edges, "bytes": 4 * n_edges + 4 * dir_entries + 8 * (total_rows + 1) + 4 * total_rows * rw,
                                   "dense_bytes": 4 * entries + 4 * total_rows * rw, "pack_ms": pack_ms,
                                   "decode_us_per_launch": d0.elapsed_time(d1) * 1e3 / S,
                                   "same_tokens_as_dense": bool(torch.equal(p_tokens, tokens) and torch.equal(p_states, states))}
            # not part of a step: a push-down constraint (Section 3) over the same vocabulary, a nested JSON grammar:
            # the composition with T_V (a set-up call) and the decode step that conditions the allowed set on the stack
            from workloads import pda as PD
            g = PD.json_like()
            torch.cuda.synchronize()
            tq0 = time.perf_counter()
            ptab = T.compile_token_pda(vocab, T.CharPDA(g.n_states, g.start, g.accept, g.src, g.input, g.dst, g.pop_begin, g.pop_syms,
                                                        g.push_begin, g.push_syms))
            torch.cuda.synchronize()
            pda_compile_ms = (time.perf_counter() - tq0) * 1e3
            cap = 32
            p_state = torch.full((B,), g.start, dtype=torch.int32, device=dev)
            p_stack = torch.zeros((B, cap), dtype=torch.int32, device=dev)
            p_depth = torch.ones((B,), dtype=torch.int32, device=dev)
            p_tok = torch.empty((B,), dtype=torch.int32, device=dev)
            n_pda_steps = min(S, 64)
            for s in range(3):
                T.pda_step(ptab, logits[s % n_rot], p_state, p_stack, p_depth, p_tok, p_state)

            def pda_all():
                p_state.fill_(g.start)
                p_depth.fill_(1)
                p_stack.zero_()
                for s in range(n_pda_steps):
                    T.pda_step(ptab, logits[s % n_rot], p_state, p_stack, p_depth, p_tok, p_state)

            torch.cuda.synchronize()
            pda_graph = None
            if not args.no_graph:                       # launched the way the decode is
                pda_graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(pda_graph):
                    pda_all()
                pda_graph.replay()
                torch.cuda.synchronize()
            q0, q1 = ev(), ev()
            q0.record()
            pda_graph.replay() if pda_graph is not None else pda_all()
            q1.record()
            torch.cuda.synchronize()
            out["pushdown"] = {"grammar": "nested JSON (23 states, 177 edges)", "token_edges": ptab.n_edges,
                               "compile_ms_blocking": pda_compile_ms, "steps": n_pda_steps,
                               "decode_launch": "hip graph" if pda_graph is not None else "stream",
                               "us_per_step": q0.elapsed_time(q1) * 1e3 / n_pda_steps,
                               "sequences_still_alive": int((p_state >= 0).sum().item()),
                               "max_stack_depth": int(p_depth.max().item())}
            # the same decode with the tokens drawn at temperature 1 (stream launches)
            p_state.fill_(g.start)
            p_depth.fill_(1)
            p_stack.zero_()
            T.pda_sample_step(ptab, logits[0], p_state, p_stack, p_depth, 1.0, 5, 0, p_tok, p_state)
            p_state.fill_(g.start)
            p_depth.fill_(1)
            p_stack.zero_()
            torch.cuda.synchronize()
            r0, r1 = ev(), ev()
            r0.record()
            for s in range(n_pda_steps):
                T.pda_sample_step(ptab, logits[s % n_rot], p_state, p_stack, p_depth, 1.0, 5, s, p_tok, p_state)
            r1.record()
            torch.cuda.synchronize()
            out["pushdown"]["sampled_us_per_step_stream_launch"] = r0.elapsed_time(r1) * 1e3 / n_pda_steps
            out["pushdown"]["sampled_sequences_still_alive"] = int((p_state >= 0).sum().item())
    else:
        out["roofline"] = roof_compile
    return out, w, units_per_step, unit


if __name__ == "__main__":
    main()
