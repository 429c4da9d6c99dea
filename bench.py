#!/usr/bin/env python3
"""Benchmark of the Data Coordinator reshard path on one MI355X.

A step is one pass of the whole path over one synthetic rollout batch already resident in
HBM, on one stream: dc_balance_plan_group_advantage (Algorithm 1, the advantage stage and the plan:
two launches), then dc_gather.  (--three-calls: dc_balance_group_advantage, dc_plan, dc_gather.)
Prints ONE JSON line.  Its headline is workload config 5 (the largest): repacked tokens/s for the
whole step, the gather kernel's achieved HBM bandwidth against the chip's peak (HIP events around
every gather launch of the timed region, on the stream it is launched on; mean, median and
minimum), and the CPU oracle timed on the host as a reported baseline.  "other_configs" carries
the same step figures for configs 3 and 4, measured the same way in the same process, so that one
run covers every configuration the bandwidth target names.
Outside the timed region it also times each call of the step on its own, the step with
dc_gather_advantage (no rollout-layout copy of the per-token advantages), the reverse path
(dc_scatter) and the PPO advantage stage (dc_gae) on the same batch, and a plain copy of the
gather's byte count as the box's ceiling ("stages", "no_rollout_adv", "reverse", "ppo_advantage",
"copy_ceiling").
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published

# HBM bytes per gather launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch), each
# scaled by what the same counter reads for the plain copy of --calibrate-copy (2^30 B in, 2^30 B
# out); valid only for the kernel sources with the digest below (profiles/ has the runs).
TRAFFIC_SOURCE = "profiles/hbm_traffic_config5_pmc.txt"
TRAFFIC = {
    # config: (fetch bytes + write bytes per gather launch, digest of csrc/gather.hip + csrc/dc_internal.h)
    5: (1044691600 + 985070200, "20a6592dc78a82a9"),
}
TRAFFIC_ADV = {                                          # the same for dc_gather_advantage's kernel
    5: (867921100 + 983753400, "20a6592dc78a82a9"),
}


def kernel_digest() -> str:
    h = hashlib.sha256()
    for f in ("gather.hip", "dc_internal.h"):
        with open(os.path.join(ROOT, "paper_2507_13833_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def host_description():
    """Cores this process may run on, and the CPU's model string."""
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return cores, model


def cpu_baseline(w, budget_s: float = 12.0, gather_budget_s: float = 6.0):
    """Time the oracle (as it stands) on the same workload.  value: whole oracle steps on ONE thread,
    repeated until about budget_s seconds of CPU work are done.  gather_all_cores: the oracle's gather
    alone (one copy per sequence: independent pieces of work), the slots cut into one contiguous
    range per host core, each range one call of the same oracle function from a thread of its own."""
    import concurrent.futures

    import numpy as np

    import oracle
    host_cores, cpu_model = host_description()
    mask = w.field_by_name("mask").shards
    reps, spent = 0, 0.0
    while reps == 0 or (spent < budget_s and reps < 1000):
        t0 = time.perf_counter()
        bal = oracle.balance(w.seq_len, w.n_shards)
        adv = oracle.group_advantage(w.reward, w.group_off, float(w.eps), w.ddof)
        adv_tok = oracle.adv_broadcast(adv, w.seq_len, w.src_tok_off, w.src_shard_seq_off, w.src_shard_tokens, mask)
        pl = oracle.plan(w.seq_len, bal.perm, bal.shard_seq_off, w.token_budget, w.align_tokens)
        arena = int(pl.shard_tok_off[-1])
        for f in w.fields:
            oracle.gather(w.seq_len, bal.perm, w.src_tok_off, w.src_shard_seq_off, f.shards, pl.dst_tok_off, arena)
        oracle.gather(w.seq_len, bal.perm, w.src_tok_off, w.src_shard_seq_off, adv_tok, pl.dst_tok_off, arena)
        spent += time.perf_counter() - t0
        reps += 1

    # the gather on every core: slot ranges of about equal token counts, destination arenas allocated
    # and touched beforehand (the single-thread figure above includes allocating them)
    n_thr = max(1, host_cores)
    cuts = np.searchsorted(pl.dst_tok_off, np.linspace(0, arena, n_thr + 1)).astype(int)
    cuts[0], cuts[-1] = 0, w.n_seq
    shards_of = [f.shards for f in w.fields] + [adv_tok]
    arenas = [np.zeros(arena, s[0].dtype) for s in shards_of]

    def part(t):
        for shards, dst in zip(shards_of, arenas):
            oracle.gather_slots(w.seq_len, bal.perm, w.src_tok_off, w.src_shard_seq_off, shards, pl.dst_tok_off,
                                dst, int(cuts[t]), int(cuts[t + 1]))

    g_reps, g_spent = 0, 0.0
    with concurrent.futures.ThreadPoolExecutor(n_thr) as pool:
        list(pool.map(part, range(n_thr)))                       # untimed: threads started, pages mapped
        while g_reps == 0 or (g_spent < gather_budget_s and g_reps < 1000):
            t0 = time.perf_counter()
            list(pool.map(part, range(n_thr)))                   # ctypes releases the interpreter lock during a call
            g_spent += time.perf_counter() - t0
            g_reps += 1
    payload = sum(a.dtype.itemsize for a in arenas)
    return {"value": w.total_tokens * reps / spent, "unit": "tokens/s", "cores": 1, "kind": "oracle",
            "sample": f"whole workload ({w.total_tokens} tokens per step), {reps} full oracle steps "
                      f"(balance, advantage, plan, gather of every field), {spent:.1f} s, one thread",
            "host_cores": host_cores, "cpu_model": cpu_model,
            "gather_all_cores": {"value": w.total_tokens * g_reps / g_spent, "unit": "tokens/s", "cores": n_thr,
                                 "GB_per_s": 2 * payload * w.total_tokens * g_reps / g_spent / 1e9,
                                 "sample": f"the oracle's gather alone, every field of the whole workload, {g_reps} "
                                           f"passes, {g_spent:.1f} s, {n_thr} threads over disjoint slot ranges, "
                                           f"arenas allocated beforehand"}}


def stats_ms(xs):
    return {"mean": statistics.fmean(xs), "median": statistics.median(xs), "min": min(xs)}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=5, help="headline workload 1..5 (default: 5, the largest)")
    ap.add_argument("--other-configs", type=str, default=None,
                    help="comma-separated workloads measured beside the headline one, step figures only "
                         "(default: 3,4 when the headline is config 5, else none; 'none' for none)")
    ap.add_argument("--sets", type=int, default=3, help="rotating buffer sets (defeats cache reuse)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sides", action="store_true", help="skip every side measurement (profiling runs)")
    ap.add_argument("--three-calls", action="store_true",
                    help="dc_balance_group_advantage, dc_plan, dc_gather (five launches) in place of "
                         "dc_balance_plan_group_advantage, dc_gather (three)")
    ap.add_argument("--single-stream", action="store_true", help="issue the four calls one after the other on one stream")
    ap.add_argument("--two-streams", action="store_true",
                    help="dc_group_advantage on a second stream beside dc_balance + dc_plan (two cross-stream waits per step)")
    ap.add_argument("--no-rollout-adv", action="store_true",
                    help="the step without the rollout-layout copy of the per-token advantages: the fused launch "
                         "computes adv_seq only, dc_gather_advantage makes the training-layout field from the mask")
    ap.add_argument("--no-double-buffer", action="store_true",
                    help="skip the double_buffer side measurement (its steps run beside another kernel, which "
                         "would enter a profiler's per-kernel averages)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch a plain elementwise copy of known size (1 GiB read + 1 GiB written per "
                         "launch): the yardstick that scales the HBM byte counters of a rocprofv3 --pmc run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on ONE GPU (all shards are logical shards on one device); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import torch
    from paper_2507_13833_amd import binding, runner, workloads
    binding.load()                                       # no fallback: raises if libdc.so is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2

    def one_step(b, ev=None):
        if args.single_stream:
            b.group_advantage(); b.balance(); b.plan()
            if ev is not None:
                ev[0].record()
            b.gather()
            if ev is not None:
                ev[1].record()
        elif args.two_streams:
            b.step_overlapped(ev)
        elif args.three_calls:
            if args.no_rollout_adv:
                b.step_no_rollout_adv(ev)
            else:
                b.step_fused(ev)
        elif ev is not None and timing["dispatch"]:
            b.step_two_calls(None, True, ev)             # the gather's dispatch carries the two events
        else:
            b.step_two_calls(ev, per_token=not args.no_rollout_adv)

    # How a gather launch is timed.  The step of the default mode hands the two events to dc_gather_timed, whose
    # kernel dispatch updates them with the kernel's own begin and end times (what a profiler's kernel trace
    # reports); the other modes record them before and after the call, which adds the gaps between the launches.
    timing = {"dispatch": not (args.single_stream or args.two_streams or args.three_calls or args.no_rollout_adv)}

    def fresh_events(n):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        if timing["dispatch"]:
            for a, b in ev:                              # torch creates the HIP event at its first record
                a.record()
                b.record()
        return ev

    def check_dispatch_timing(sets):
        """One step timed both ways; the dispatch's own figure must lie just below the bracketing one."""
        if not timing["dispatch"]:
            return
        inner, outer = fresh_events(1)[0], (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
        torch.cuda.synchronize()
        sets[0].step_two_calls(outer, True, inner)
        torch.cuda.synchronize()
        ti, to = inner[0].elapsed_time(inner[1]), outer[0].elapsed_time(outer[1])
        if not (0.5 * to <= ti <= 1.02 * to):
            print(f"bench.py: dispatch events give {ti:.4f} ms against {to:.4f} ms around the call; "
                  "timing the gather by events around the call", file=sys.stderr)
            timing["dispatch"] = False

    def timed_steps(w, sets, steps, warmup):
        """warmup untimed steps, then `steps` steps between two synchronisations.  Returns wall ms per
        step, the gather launches' durations (HIP events, see `timing`) and the steps' own durations
        (end of one step's gather to the end of the next one's: the steps are queued back to back)."""
        for i in range(warmup):
            one_step(sets[i % len(sets)])
        torch.cuda.synchronize()
        assert all(s.read_status() == 0 for s in sets)
        check_dispatch_timing(sets)
        ev = fresh_events(steps)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            one_step(sets[i % len(sets)], ev[i])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        assert all(s.read_status() == 0 for s in sets)
        gather_ms = [a.elapsed_time(b) for a, b in ev]
        step_ms = [ev[i - 1][1].elapsed_time(ev[i][1]) for i in range(1, steps)]
        return (t1 - t0) * 1e3 / steps, gather_ms, step_ms

    def step_record(w, sets, steps, warmup):
        T = w.total_tokens
        bpt = sets[0].payload_bytes_per_token          # payload incl. the per-token advantage
        nbytes = (2 * bpt - 4) * T if args.no_rollout_adv else 2 * bpt * T
        ms, g_ms, s_ms = timed_steps(w, sets, steps, warmup)
        g = stats_ms(g_ms)
        return {"workload": f"config {w.cfg} ({w.name}): {w.n_seq} sequences, {T} tokens, P={w.n_shards}, "
                            f"token budget {w.token_budget}, {bpt} payload B/token, {w.n_src_shards} rollout shard(s)",
                "tokens": T, "tokens_per_s": T / (ms * 1e-3), "ms_per_step": ms,
                "step_ms_device": stats_ms(s_ms) if s_ms else None,
                "gather": {"algorithmic_bytes_per_launch": nbytes, "launch_ms": g,
                           "achieved": nbytes / (g["mean"] * 1e-3) / 1e9, "unit": "GB/s",
                           "frac": nbytes / (g["mean"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                           "frac_median": nbytes / (g["median"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                           "frac_best": nbytes / (g["min"] * 1e-3) / 1e9 / HBM_PEAK_GBS}}

    # ---- the other configurations first (their buffers are released before the headline run) ----
    if args.other_configs is None:
        others = [3, 4] if args.config == 5 and not (args.single_stream or args.two_streams or args.three_calls) else []
    elif args.other_configs.strip().lower() in ("", "none"):
        others = []
    else:
        others = [int(x) for x in args.other_configs.split(",")]
    other_configs = {}
    for cfg in others:
        wo = workloads.make_workload(cfg)
        so = [runner.DeviceBatch(wo) for _ in range(max(1, args.sets))]
        other_configs[str(cfg)] = step_record(wo, so, args.steps, args.warmup)
        del so, wo
        torch.cuda.empty_cache()

    # ---- the headline configuration ----
    w = workloads.make_workload(args.config)
    T = w.total_tokens
    sets = [runner.DeviceBatch(w) for _ in range(max(1, args.sets))]
    bpt = sets[0].payload_bytes_per_token
    gather_bytes = 2 * bpt * T                         # algorithmic: read once + write once
    gather_adv_bytes = (2 * bpt - 4) * T               # dc_gather_advantage: the 4-byte advantage is written, not read
    head = step_record(w, sets, args.steps, args.warmup)
    ms_per_step = head["ms_per_step"]
    gather_ms = head["gather"]["launch_ms"]["mean"]
    timed_gather_bytes = head["gather"]["algorithmic_bytes_per_launch"]
    achieved = head["gather"]["achieved"]

    def device_ms(call, n=50, warm=3):
        """Device time of call(buffer set): n calls queued back to back with an event between each two (so the
        host's marshalling of one call overlaps the previous call's kernels), after warm untimed calls.
        Returns {"mean", "median", "min"} in ms."""
        for i in range(warm):
            call(sets[i % len(sets)])                   # a kernel's first launch in a process loads its code
        torch.cuda.synchronize()
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        marks[0].record()
        for i in range(n):
            call(sets[i % len(sets)])
            marks[i + 1].record()
        torch.cuda.synchronize()
        return stats_ms([marks[i].elapsed_time(marks[i + 1]) for i in range(n)])

    def bw(nbytes, st):
        return {"ms": round(st["median"], 4), "ms_mean": round(st["mean"], 4), "ms_min": round(st["min"], 4),
                "algorithmic_bytes": nbytes, "achieved": nbytes / (st["median"] * 1e-3) / 1e9, "unit": "GB/s",
                "frac": nbytes / (st["median"] * 1e-3) / 1e9 / HBM_PEAK_GBS}

    variant = stage = reverse = ppo = double_buffer = ceiling = None
    sides = not args.no_sides

    # the same step with dc_gather_advantage in place of the per-token advantage pass + dc_gather
    # (a shorter run of its own, outside the timed region)
    if sides and not (args.no_rollout_adv or args.single_stream or args.two_streams):
        n_var = max(2, min(args.steps, 60))
        var_step = (lambda b, ev=None: b.step_no_rollout_adv(ev)) if args.three_calls else \
                   (lambda b, ev=None: b.step_two_calls(ev, per_token=False))
        for i in range(3):
            var_step(sets[i % len(sets)])
        evv = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_var)]
        torch.cuda.synchronize()
        v0 = time.perf_counter()
        for i in range(n_var):
            var_step(sets[i % len(sets)], evv[i])
        torch.cuda.synchronize()
        v_ms = (time.perf_counter() - v0) * 1e3 / n_var
        vg = stats_ms([a.elapsed_time(b) for a, b in evv])
        assert all(s.read_status() == 0 for s in sets)
        variant = {"calls": ("dc_balance_group_advantage (adv_seq only), dc_plan, dc_gather_advantage" if args.three_calls
                             else "dc_balance_plan_group_advantage (adv_seq only), dc_gather_advantage"),
                   "steps": n_var, "ms_per_step": round(v_ms, 4), "tokens_per_s": T / (v_ms * 1e-3),
                   "gather_ms": round(vg["mean"], 4), "gather_ms_median": round(vg["median"], 4),
                   "gather_ms_min": round(vg["min"], 4), "algorithmic_bytes": gather_adv_bytes,
                   "achieved": gather_adv_bytes / (vg["mean"] * 1e-3) / 1e9, "unit": "GB/s",
                   "frac": gather_adv_bytes / (vg["mean"] * 1e-3) / 1e9 / HBM_PEAK_GBS}

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.int32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1, out=dst)                  # one elementwise kernel: 2^30 B in, 2^30 B out
        torch.cuda.synchronize()
        del src, dst

    if sides:
        # per-stage device times (median of 50 calls), outside the timed region
        stage = {}
        for name in ("group_advantage", "balance", "plan", "gather"):
            st = device_ms(lambda b, name=name: getattr(b, name)())
            stage[name + "_ms"] = round(st["median"], 4)
            stage[name + "_ms_min"] = round(st["min"], 4)
        st = device_ms(lambda b: b.balance_group_advantage())
        stage["balance_group_advantage_ms"] = round(st["median"], 4)
        stage["balance_group_advantage_ms_min"] = round(st["min"], 4)
        st = device_ms(lambda b: b.balance_plan_group_advantage())
        stage["balance_plan_group_advantage_ms"] = round(st["median"], 4)
        stage["balance_plan_group_advantage_ms_min"] = round(st["min"], 4)
        stage["group_advantage_algorithmic_bytes"] = 5 * T       # 1 B mask read + 4 B advantage written per token

        # the reverse path (training layout -> rollout layout), whole dc_scatter call
        for b in sets:
            b.prepare_scatter()
        reverse = {"call": "dc_scatter", **bw(gather_bytes, device_ms(lambda b: b.scatter()))}
        assert all(s.read_status() == 0 for s in sets)
        for b in sets:
            b.release_scatter()

        # PPO advantage stage (dc_gae) on the same batch, where the workload has a value field
        if "value" in sets[0].src_fields and sets[0].elem_bytes.get("value") == 4:
            res = {}
            for b in sets:
                b.prepare_gae()
            for tag, klc, bpt_gae in (("no_kl", 0.0, 13), ("kl", 0.05, 21)):
                res[tag] = bw(bpt_gae * T, device_ms(lambda b, klc=klc: b.gae(1.0, 0.95, klc)))
            assert all(s.read_status() == 0 for s in sets)
            ppo = {"call": "dc_gae", **res}

    # Algorithm 1 beyond what one workgroup's LDS holds (dc_balance_ws): 65 536 sequences of this workload's
    # length distribution over 64 shards
    beyond_lds = None
    if sides:
        import numpy as np
        from paper_2507_13833_amd import binding, workloads
        n_big, p_big = 65536, 64
        lens = workloads.sequence_lengths(args.config, n_big)
        prm = binding.make_params(n_big, p_big, 1 << 20, 1e-6, 1, 0, 1)
        dev = torch.device("cuda:0")
        d_len = torch.from_numpy(lens).to(dev)
        d_perm = torch.empty(n_big, dtype=torch.int32, device=dev)
        d_off = torch.empty(p_big + 1, dtype=torch.int32, device=dev)
        d_of = torch.empty(n_big, dtype=torch.int32, device=dev)
        d_load = torch.empty(p_big, dtype=torch.int64, device=dev)
        d_st = torch.zeros(1, dtype=torch.int32, device=dev)
        nb = binding.dc_balance_workspace_bytes(prm)
        d_ws = torch.empty(nb, dtype=torch.uint8, device=dev)
        st = device_ms(lambda b: binding.dc_balance_ws(prm, d_len, d_perm, d_off, d_of, d_load, d_ws, nb, d_st))
        assert int(d_st.item()) == 0 and int(d_load.sum().item()) == int(lens.astype(np.int64).sum())
        beyond_lds = {"call": "dc_balance_ws", "n_seq": n_big, "n_shards": p_big,
                      "lengths": f"the length recipe of config {args.config}", "workspace_bytes": nb,
                      "ms": round(st["median"], 4), "ms_min": round(st["min"], 4)}
        del d_len, d_perm, d_off, d_of, d_load, d_ws

    # Double buffer (Sec. 6.5): the step that fills one buffer set beside a consumer that still reads the set
    # filled before it (stand-in consumer: one reduction over each 4-byte arena of that set), on two streams of
    # the default priority, against the same two pieces of work issued one after the other; outside the timed region
    if sides and len(sets) >= 2 and not args.no_double_buffer:
        def consume(b):
            for n, v in b.dst_fields.items():
                if b.elem_bytes.get(n, 4) == 4:
                    v.view(torch.float32).sum()          # the bits read as floats: only the traffic matters
        main_s, side_s = torch.cuda.current_stream(), torch.cuda.Stream()
        ev_step, ev_cons = torch.cuda.Event(), torch.cuda.Event()

        def both(i, overlap):
            cur, prev = sets[i % len(sets)], sets[(i - 1) % len(sets)]
            if overlap:
                ev_step.record(main_s)                   # prev is complete, and so is the consumer's earlier pass
                side_s.wait_event(ev_step)
                with torch.cuda.stream(side_s):
                    consume(prev)
                    ev_cons.record(side_s)
                cur.step_two_calls()
                main_s.wait_event(ev_cons)
            else:
                consume(prev)
                cur.step_two_calls()

        res = {}
        for tag, overlap in (("serial_ms", False), ("overlapped_ms", True)):
            for i in range(3):
                both(i, overlap)
            torch.cuda.synchronize()
            d0, d1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            d0.record()
            for i in range(24):
                both(i, overlap)
            d1.record()
            torch.cuda.synchronize()
            res[tag] = round(d0.elapsed_time(d1) / 24, 4)
        assert all(s.read_status() == 0 for s in sets)
        double_buffer = {"what": "one step into buffer set i beside a reduction over the 4-byte arenas of set i-1 "
                                 "(two streams) vs one after the other", **res}

        # two independent batches in flight: the step of buffer set i on stream i mod 2 (default priority), so the
        # latency-bound balance + plan of one batch runs beside the other batch's gather; whole steps, none skipped
        lanes = [torch.cuda.Stream(), torch.cuda.Stream()]
        for q in lanes:
            q.wait_stream(main_s)

        def in_flight(n):
            for i in range(n):
                with torch.cuda.stream(lanes[i % 2]):
                    sets[i % 2].step_two_calls()
            for q in lanes:
                main_s.wait_stream(q)
        in_flight(4)
        torch.cuda.synchronize()
        d0, d1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n_fl = 40
        d0.record()
        for q in lanes:
            q.wait_stream(main_s)
        in_flight(n_fl)
        d1.record()
        torch.cuda.synchronize()
        assert all(s.read_status() == 0 for s in sets)
        fl_ms = d0.elapsed_time(d1) / n_fl
        double_buffer["two_batches_in_flight"] = {
            "what": "steps of two buffer sets alternating on two streams, each step complete; ms per step",
            "steps": n_fl, "ms_per_step": round(fl_ms, 4), "tokens_per_s": T / (fl_ms * 1e-3)}

    # the achievable ceiling on this machine: a plain elementwise copy (one torch kernel) of the gather's byte count,
    # 3 rotating buffer pairs, measured the same way
    if sides:
        n_words = gather_bytes // 2 // 4
        pairs = [(torch.ones(n_words, dtype=torch.int32, device="cuda:0"), torch.empty(n_words, dtype=torch.int32, device="cuda:0"))
                 for _ in range(3)]
        for i in range(3):
            torch.add(pairs[i][0], 1, out=pairs[i][1])
        torch.cuda.synchronize()
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(31)]
        marks[0].record()
        for i in range(30):
            torch.add(pairs[i % 3][0], 1, out=pairs[i % 3][1])
            marks[i + 1].record()
        torch.cuda.synchronize()
        cst = stats_ms([marks[i].elapsed_time(marks[i + 1]) for i in range(30)])
        ceiling = {"what": "plain elementwise copy (one torch kernel) of the gather's byte count, same box",
                   "ms": round(cst["median"], 4), "ms_min": round(cst["min"], 4),
                   "achieved": 2 * n_words * 4 / (cst["median"] * 1e-3) / 1e9, "unit": "GB/s"}
        del pairs

        # the same for the write-heavy stages: plain torch kernels with their mix of bytes read and written per
        # token, over T elements (three rotating buffer sets, median of 30 launches)
        def plain_ms(make, run):
            bufs = [make() for _ in range(3)]
            for i in range(3):
                run(bufs[i])
            torch.cuda.synchronize()
            mk = [torch.cuda.Event(enable_timing=True) for _ in range(31)]
            mk[0].record()
            for i in range(30):
                run(bufs[i % 3])
                mk[i + 1].record()
            torch.cuda.synchronize()
            return stats_ms([mk[i].elapsed_time(mk[i + 1]) for i in range(30)])

        def probe(what, nbytes, st):
            return {"what": what, "ms": round(st["median"], 4), "ms_min": round(st["min"], 4),
                    "achieved": nbytes / (st["median"] * 1e-3) / 1e9, "unit": "GB/s",
                    "frac": nbytes / (st["median"] * 1e-3) / 1e9 / HBM_PEAK_GBS}
        dev0 = torch.device("cuda:0")
        ceiling["write_only"] = probe(
            "fill of T float32 (0 B read, 4 B written per token: the advantage stage reads 1 B and writes 4 B)", 4 * T,
            plain_ms(lambda: torch.empty(T, dtype=torch.float32, device=dev0), lambda o: o.fill_(1.0)))
        ceiling["read4_write8"] = probe(
            "torch.frexp of T float32 (one kernel, 4 B read, 8 B written per token: dc_gae reads 5 B and writes 8 B)",
            12 * T,
            plain_ms(lambda: (torch.ones(T, dtype=torch.float32, device=dev0),
                              torch.empty(T, dtype=torch.float32, device=dev0),
                              torch.empty(T, dtype=torch.int32, device=dev0)),
                     lambda b: torch.frexp(b[0], out=(b[1], b[2]))))

    traffic = None
    table = TRAFFIC_ADV if args.no_rollout_adv else TRAFFIC
    if args.config in table and table[args.config][1] == kernel_digest():
        traffic = table[args.config][0]
    if variant is not None and args.config in TRAFFIC_ADV and TRAFFIC_ADV[args.config][1] == kernel_digest():
        variant["traffic"] = TRAFFIC_ADV[args.config][0]

    g = head["gather"]
    out = {
        "metric": "repacked tokens/sec and achieved HBM GB/s (fraction of peak), 1 MI355X",
        "value": T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_device": head["step_ms_device"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": head["workload"],
                   "buffer_sets": len(sets),
                   "streams": 2 if args.two_streams else 1,
                   "launches": "separate" if (args.single_stream or args.two_streams)
                               else (("dc_balance_group_advantage (adv_seq only), dc_plan, dc_gather_advantage"
                                      if args.no_rollout_adv else "dc_balance_group_advantage, dc_plan, dc_gather")
                                     if args.three_calls else
                                     ("dc_balance_plan_group_advantage (adv_seq only), dc_gather_advantage"
                                      if args.no_rollout_adv else "dc_balance_plan_group_advantage, dc_gather"))},
        "roofline": {"bound": "hbm", "kernel": "gather_adv_kernel" if args.no_rollout_adv else "gather_kernel",
                     "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "traffic_source": (TRAFFIC_SOURCE + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, taken earlier on "
                                        "these kernel sources; not measured in this run)") if traffic else None,
                     "algorithmic_bytes_per_launch": timed_gather_bytes, "avg_launch_ms": gather_ms,
                     "launch_timing": ("begin and end of the kernel's own dispatch (dc_gather_timed)" if timing["dispatch"]
                                       else "events recorded before and after the launch"),
                     "median_launch_ms": g["launch_ms"]["median"], "min_launch_ms": g["launch_ms"]["min"],
                     "frac_median": g["frac_median"], "frac_best": g["frac_best"]},
        "other_configs": other_configs,
        "copy_ceiling": ceiling,
        "stages": stage,
        "no_rollout_adv": variant,
        "reverse": reverse,
        "ppo_advantage": ppo,
        "double_buffer": double_buffer,
        "balance_beyond_lds": beyond_lds,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
