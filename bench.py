#!/usr/bin/env python3
"""Throughput of the structured-decoding hot path on one MI355X.

A step is one pass of the whole path over one decode batch: mask lookup / build /
gather (wg_fill_masks), logit masking (wg_apply_mask) and state advance
(wg_advance).  The workload is the mixed HTML / JSON configuration (B=256 requests,
V=151,936 tokens, bf16 logits, one template instance per request) on seeded
synthetic inputs.  "cold" clears the mask cache before every step, so every
distinct state key of the batch is rebuilt; "warm" replays the same trajectory with
every mask cached.  The headline value is the cold rate: the median over several passes
of the K timed steps, taken after the GPU has been kept busy long enough for its clocks to
settle, so that a short run reads the same as a long one.  The timed steps are always the
same window of the trajectory (it starts at step WINDOW_START), whatever K is.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

prints one JSON line.  Everything runs on one GPU; --gpus above 1 is refused.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth

# HBM bytes per launch in the cold steps of workloads 4 and 5, from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE (profiles/bench_config4_hbm_traffic.txt, profiles/bench_config5_hbm_traffic.txt; fetch
# scaled x2.000, write x1.000 by the counters of a 512 MiB device copy).  They describe the kernels
# whose source hashes to TRAFFIC_SOURCE_SHA256; with any other kernel source, or any other workload,
# the field is reported as null.
TRAFFIC_BYTES = {
    4: {"lookup": 0.17e6, "class_scan": 6.29e6, "key_build": 15.64e6, "gather": 0.04e6, "apply": 57.06e6, "advance": 0.21e6},
    5: {"lookup": 0.44e6, "class_scan": 26.85e6, "key_build": 34.19e6, "gather": 14.15e6, "apply": 314.61e6, "advance": 0.75e6},
}
TRAFFIC_SOURCE_SHA256 = "c1d8daad70d0835bc464156a5d396d9bf041c0cb349521bf7c01c30c35672916"
WINDOW_START = 64              # first timed step of the trajectory (the warm-up steps come right before it)
N_PASSES = 5                   # timed passes per figure; the median is reported
RAMP_SECONDS = 0.08            # GPU work done before timing, for the clocks to settle


def kernel_source_sha256():
    import hashlib
    path = os.path.join(ROOT, "paper_2507_16768_amd", "csrc", "wg_kernels.hip")
    with open(path, "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()


def _oracle_steps(w, lo, hi, n_steps):
    """Requests lo..hi-1 of the workload for n_steps steps through the CPU oracle: un-memoised
    mask rows, masking of a logits buffer, token choice and advance.  Returns the seconds spent."""
    import wg_synth as ws
    from oracle import oracle as O

    ov = O.OracleVocab(w.vocab.bytes, w.vocab.offsets, w.vocab.eos_id)
    o = O.Oracle(w.texts, w.args, ov, restart=True)
    n = hi - lo
    cur = np.array([[o.start_state(int(t)), 0] for t in w.request_template[lo:hi]], dtype=np.uint32)
    draws = w.token_draws(n_steps)[:, lo:hi]
    logits = ws.to_bf16_bits(ws.make_logits(w.seed, n, w.vocab.V, w.sigma))
    t0 = time.perf_counter()
    for k in range(n_steps):
        masks = o.fill_masks(cur)
        O.apply_mask(logits, masks)
        toks = np.empty(n, dtype=np.int32)
        for b in range(n):
            pop = int(np.unpackbits(masks[b].view(np.uint8)).sum())
            toks[b] = O.select_bit(masks[b], int(draws[k, b] % np.uint64(max(pop, 1))))
        cur = o.advance(cur, toks)
    return time.perf_counter() - t0


_fork_workload = None      # set before the worker pool forks, so that the jobs carry indexes only


def _oracle_worker(job):
    return _oracle_steps(_fork_workload, *job)


def cpu_baseline(w, n_steps):
    """The CPU oracle, as it stands, on the first n_steps steps of the same workload, on one
    thread; then independent copies of it on disjoint request ranges, one per host core (the
    work is independent per request), for an all-cores figure.  Call it before the process
    touches the GPU: the all-cores leg forks."""
    import multiprocessing as mp

    dt = _oracle_steps(w, 0, w.B, n_steps)
    out = {"value": w.B * n_steps / dt, "unit": "request-steps/s", "cores": 1, "kind": "oracle",
           "sample": "first %d steps of the same workload (%d request-steps, cold: every mask "
                     "rebuilt), %.1f s" % (n_steps, w.B * n_steps, dt)}
    cores = min(16, len(os.sched_getaffinity(0)), w.B)
    if cores > 1:
        steps_all = n_steps * 4
        cuts = [w.B * i // cores for i in range(cores + 1)]
        jobs = [(cuts[i], cuts[i + 1], steps_all) for i in range(cores)]
        global _fork_workload
        _fork_workload = w
        t0 = time.perf_counter()
        with mp.get_context("fork").Pool(cores) as pool:
            spent = pool.map(_oracle_worker, jobs)
        wall = time.perf_counter() - t0
        out["all_cores"] = {"value": w.B * steps_all / max(spent), "unit": "request-steps/s", "cores": cores,
                            "sample": "first %d steps, the %d requests split over %d processes; slowest "
                                      "process %.1f s (%.1f s with start-up)"
                                      % (steps_all, w.B, cores, max(spent), wall)}
    return out


def apply_patterns(B=256, V=151936, K=200):
    """wg_apply_mask on bf16 logits under synthetic mask patterns: what a store that covers only
    part of a 64-byte block costs.  Prints one line per pattern."""
    import torch
    import paper_2507_16768_amd as wg
    wg.load_library()
    W = (V + 31) // 32
    ring = [torch.randn((B, V), device="cuda").to(torch.bfloat16) for _ in range(4)]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(mask):
        for k in range(8):
            wg.apply_mask(ring[k & 3], mask)
        torch.cuda.synchronize()
        e0.record()
        for k in range(K):
            wg.apply_mask(ring[k & 3], mask)
        e1.record()
        torch.cuda.synchronize()
        return 1e3 * e0.elapsed_time(e1) / K

    def words(value):
        return torch.full((B, W), value, dtype=torch.int64, device="cuda").to(torch.int32)

    rows = torch.zeros((B, W), dtype=torch.int32, device="cuda")
    rows[::2, :] = -1
    halves = torch.zeros((B, W), dtype=torch.int32, device="cuda")
    halves[:, ::2] = -1
    cases = [("nothing disallowed (mask read only; the loop's launch rate)", words(-1)),
             ("everything disallowed: 16-byte stores, every block written whole", words(0)),
             ("every other row disallowed", rows),
             ("every other 64-byte block disallowed", halves),
             ("every other 16 bytes disallowed", words(0x00FF00FF)),
             ("1 token of 32 disallowed: one 2-byte store per 64-byte block", words(-2)),
             ("1 token of 8 disallowed", words(0xFEFEFEFE - (1 << 32))),
             ("4 tokens of 8 disallowed, alternating", words(0x55555555)),
             ("7 tokens of 8 disallowed", words(0x01010101))]
    print("wg_apply_mask, B=%d, V=%d, bf16 (%.1f MB of logits), mean of %d launches" % (B, V, B * V * 2 / 1e6, K))
    for name, mask in cases:
        print("%-68s %6.2f us" % (name, timed(mask)), flush=True)


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, help="workload index 1..5 (default: 4, mixed)")
    ap.add_argument("--cpu-steps", type=int, default=32, help="oracle steps timed for cpu_baseline (0 = skip)")
    ap.add_argument("--brief", action="store_true",
                    help="only the separate-call and wg_decode_step timings and the kernel table (for profiler runs)")
    ap.add_argument("--apply-patterns", action="store_true",
                    help="instead of the benchmark: time wg_apply_mask under synthetic mask patterns")
    args = ap.parse_args()
    if args.apply_patterns:
        apply_patterns()
        return
    if args.gpus != 1:
        print("bench.py measures one GPU; --gpus %d is not supported (the path shards by request or "
              "by vocabulary slice without collectives, so more GPUs add nothing to measure here)"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import wg_synth as ws

    w = ws.make_workload(args.config)
    # the CPU legs run first: they fork worker processes, which is done before the GPU is initialised
    cpu = cpu_baseline(w, args.cpu_steps) if args.cpu_steps > 0 else None

    import torch
    import paper_2507_16768_amd as wg

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    wg.load_library()
    torch.cuda.set_device(0)
    K, Wm = args.steps, args.warmup
    k0 = max(WINDOW_START, Wm)          # first timed step; steps k0 - Wm .. k0 - 1 are the warm-up
    total = k0 + K
    B, V = w.B, w.vocab.V
    tdt = torch.float32 if w.dtype == "f32" else torch.bfloat16
    esz = 4 if w.dtype == "f32" else 2

    t0 = time.perf_counter()
    vocab = wg.Vocab(w.vocab.bytes, w.vocab.offsets, w.vocab.eos_id)
    vocab_ms = (time.perf_counter() - t0) * 1e3
    t0 = time.perf_counter()
    h = wg.Handle(w.texts, w.args, vocab, flags=wg.EOS_RESTART)
    compile_ms = (time.perf_counter() - t0) * 1e3
    h.reserve_batch(B)
    # a request joining a running engine: one instance added to a live handle (host lowering of
    # its arguments into the cached static structure, upload of the new table slices)
    n_join = 0 if args.brief else min(64, len(w.texts) - 1)
    join_us, join_call_us = [], []
    if n_join > 0:
        hj = wg.Handle(w.texts[:1], w.args[:1] if w.args else None, vocab, flags=wg.EOS_RESTART)
        for i in range(1, n_join + 1):
            t0 = time.perf_counter()
            hj.add_instances(w.texts[i:i + 1], w.args[i:i + 1] if w.args else None)
            join_us.append((time.perf_counter() - t0) * 1e6)
        # the same for the next instances of the list, with the Python lists turned into C arrays
        # beforehand: the wg_add_instances call alone (lowering, upload of the new table slices)
        for i in range(n_join + 1, min(2 * n_join + 1, len(w.texts))):
            m = wg.marshal_templates(w.texts[i:i + 1], w.args[i:i + 1] if w.args else None)
            t0 = time.perf_counter()
            hj.add_instances(None, None, marshalled=m)
            join_call_us.append((time.perf_counter() - t0) * 1e6)
        del hj
    W = h.W
    start = torch.from_numpy(np.ascontiguousarray(h.start_states[w.request_template]).view(np.int32).copy()).cuda()

    # ---- untimed pre-pass: produce the token trajectory on the GPU (sampler stand-in), keep the
    # states at the first warm-up step and the masks of the timed steps ----
    draws = torch.from_numpy(w.token_draws(total).view(np.int64)).cuda()
    tokens = torch.empty((total, B), dtype=torch.int32, device="cuda")
    states = start.clone()
    mask = torch.empty((B, W), dtype=torch.int32, device="cuda")
    masks_timed = torch.empty((K, B, W), dtype=torch.int32, device="cuda")
    window_states = None
    for k in range(total):
        if k == k0 - Wm:
            window_states = states.clone()
        h.fill_masks(states, mask)
        if k >= k0:
            masks_timed[k - k0].copy_(mask)
        wg.select_tokens(mask, V, draws[k], tokens[k])
        h.advance(states, tokens[k])
    torch.cuda.synchronize()
    assert h.error_count() == 0, "trajectory generation fed an illegal token"
    pre = h.cache_stats()
    popcount8 = torch.tensor([bin(i).count("1") for i in range(256)], dtype=torch.int64, device="cuda")
    n_allowed = sum(int(popcount8[masks_timed[k].view(torch.uint8).long()].sum().item()) for k in range(K))
    disallowed_per_step = B * V - n_allowed / float(K)

    # a plain device copy of known size (512 MiB in, 512 MiB out, larger than every cache): the
    # reference against which the rocprofv3 FETCH_SIZE / WRITE_SIZE counters of the other kernels are
    # scaled, and the measured ceiling of a streaming kernel on this GPU
    calib_src = torch.randint(0, 255, (512 << 20,), dtype=torch.uint8, device="cuda")
    calib_dst = torch.empty_like(calib_src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    copy_ms = []
    for _ in range(6):
        torch.cuda.synchronize()
        e0.record()
        calib_dst.copy_(calib_src)
        e1.record()
        torch.cuda.synchronize()
        copy_ms.append(e0.elapsed_time(e1))
    copy_ceiling_gbs = 2.0 * (512 << 20) / (min(copy_ms[1:]) * 1e-3) / 1e9
    del calib_src, calib_dst

    # logits ring (values are irrelevant to the work done; N(0, sigma) as the workload says)
    ring = [(torch.randn((B, V), device="cuda", dtype=torch.float32) * w.sigma).to(tdt) for _ in range(4)]

    def step(cold, k):
        if cold:
            h.cache_clear()
        h.fill_masks(states, mask)
        wg.apply_mask(ring[k & 3], mask)
        h.advance(states, tokens[k])

    def rewind(cold):
        """Back to the first warm-up step, then the warm-up steps."""
        states.copy_(window_states)
        if cold:
            h.cache_clear()
        for k in range(k0 - Wm, k0):
            step(cold, k)

    def ramp(prepare, one_step):
        """Keeps the GPU busy with the loop that is about to be timed until its clocks have settled."""
        t_end = time.perf_counter() + RAMP_SECONDS
        while time.perf_counter() < t_end:
            prepare()
            for k in range(k0, total):
                one_step(k)
            torch.cuda.synchronize()

    def passes(prepare, one_step, n=N_PASSES):
        """n timed passes over the K steps of the window: seconds per step of each pass."""
        ramp(prepare, one_step)
        out = []
        for _ in range(n):
            prepare()
            torch.cuda.synchronize()
            t = time.perf_counter()
            for k in range(k0, total):
                one_step(k)
            torch.cuda.synchronize()
            out.append((time.perf_counter() - t) / K)
        return out

    def timed(cold):
        return passes(lambda: rewind(cold), lambda k: step(cold, k))

    # ---- per-kernel durations over the same timed steps, HIP events on the launch stream ----
    def kernel_times(cold):
        ramp(lambda: rewind(cold), lambda k: step(cold, k))
        rewind(cold)
        torch.cuda.synchronize()
        h.profile_enable(True)
        h.profile_read()
        for k in range(k0, total):
            if cold:
                h.cache_clear()
            h.fill_masks(states, mask)
            h.profile_apply_mask(ring[k & 3], mask)
            h.advance(states, tokens[k])
        torch.cuda.synchronize()
        p = h.profile_read()
        h.profile_enable(False)
        return {k[:-3] + "_us": 1e3 * p[k] / K
                for k in ("lookup_ms", "scan_ms", "build_ms", "gather_ms", "advance_ms", "apply_ms")}

    # ---- the whole step in one call: advance + fill + apply ----
    def single_step(cold, k):
        if cold:
            h.cache_clear()
        h.decode_step(states, tokens[k - 1], mask, ring[k & 3])

    def single_rewind(cold):
        # (the token before the first warm-up step is not part of the window: that step only fills)
        states.copy_(window_states)
        if cold:
            h.cache_clear()
        h.decode_step(states, None, mask, ring[0])
        for k in range(k0 - Wm + 1, k0):
            single_step(cold, k)

    def timed_single(cold):
        return passes(lambda: single_rewind(cold), lambda k: single_step(cold, k))

    def decode_kernel_times(cold):
        """Per-kernel durations of wg_decode_step: its first kernel counts as lookup, its last as gather."""
        ramp(lambda: single_rewind(cold), lambda k: single_step(cold, k))
        single_rewind(cold)
        torch.cuda.synchronize()
        h.profile_enable(True)
        h.profile_read()
        for k in range(k0, total):
            single_step(cold, k)
        torch.cuda.synchronize()
        p = h.profile_read()
        h.profile_enable(False)
        return {"advance_lookup_us": 1e3 * p["lookup_ms"] / K, "scan_us": 1e3 * p["scan_ms"] / K,
                "build_us": 1e3 * p["build_ms"] / K, "gather_apply_us": 1e3 * p["gather_ms"] / K}

    # ---- spread of the step time: one event per step boundary (their cost is inside the figures) ----
    def step_spread(cold):
        rewind(cold)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
        torch.cuda.synchronize()
        ev[0].record()
        for k in range(k0, total):
            step(cold, k)
            ev[k - k0 + 1].record()
        torch.cuda.synchronize()
        us = np.array([1e3 * ev[i].elapsed_time(ev[i + 1]) for i in range(K)])
        return {"median_us": float(np.median(us)), "p10_us": float(np.percentile(us, 10)),
                "p90_us": float(np.percentile(us, 90))}

    # ---- spread of the calls of a step: an event after each call (their cost is inside the figures) ----
    def parts_spread(cold):
        rewind(cold)
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(K)]
        torch.cuda.synchronize()
        for k in range(k0, total):
            e = ev[k - k0]
            if cold:
                h.cache_clear()
            e[0].record()
            h.fill_masks(states, mask)
            e[1].record()
            wg.apply_mask(ring[k & 3], mask)
            e[2].record()
            h.advance(states, tokens[k])
            e[3].record()
        torch.cuda.synchronize()

        def stats(a, b):
            us = np.array([1e3 * e[a].elapsed_time(e[b]) for e in ev])
            return {"median_us": float(np.median(us)), "p10_us": float(np.percentile(us, 10)),
                    "p90_us": float(np.percentile(us, 90))}
        return {"fill": stats(0, 1), "apply": stats(1, 2), "advance": stats(2, 3), "fill_apply": stats(0, 2)}

    # ---- the decode loop with advance and the next fill in one call ----
    def timed_fused(cold):
        def one(k):
            wg.apply_mask(ring[k & 3], mask)
            if cold:
                h.cache_clear()
            h.advance_fill_masks(states, tokens[k], mask)

        def prepare():
            states.copy_(window_states)
            if cold:
                h.cache_clear()
            h.fill_masks(states, mask)
            for k in range(k0 - Wm, k0):
                one(k)
        return passes(prepare, one)

    med = lambda xs: float(np.median(xs))

    # Warm first: every key of the window was cached by the pre-pass.
    s_w0 = h.cache_stats()
    warm_passes = timed(False)
    s_w1 = h.cache_stats()
    sec_warm = med(warm_passes)
    hit_rate = (s_w1["hits"] - s_w0["hits"]) / float(max(1, s_w1["lookups"] - s_w0["lookups"]))
    assert s_w1["builds"] == pre["builds"], "a warm pass built a mask"
    kt_warm = kernel_times(False)
    single_warm_passes = timed_single(False)
    sec_single_warm = med(single_warm_passes)
    dk_warm = decode_kernel_times(False)

    s0 = h.cache_stats()
    cold_passes = timed(True)
    s1 = h.cache_stats()
    sec_cold = med(cold_passes)
    # (per step of the timed loop: the ramp, the warm-up and the timed steps all clear before every fill)
    n_cold_steps = float(s1["lookups"] - s0["lookups"]) / B
    builds_per_step = (s1["builds"] - s0["builds"]) / n_cold_steps
    scans_per_step = (s1["class_scans"] - s0["class_scans"]) / n_cold_steps
    entries_per_step = (s1["entries_walked"] - s0["entries_walked"]) / n_cold_steps
    kt_cold = kernel_times(True)
    single_cold_passes = timed_single(True)
    sec_single_cold = med(single_cold_passes)
    dk_cold = decode_kernel_times(True)

    apply_us = kt_cold["apply_us"]
    # The masks of the timed steps, by groups of 32 tokens (one mask word; 64 bytes of bf16 logits):
    # a group that is disallowed as a whole is written as full blocks; a store into a mixed one
    # covers part of a block, which costs more than writing the block whole (--apply-patterns).
    n_words = float(K * B * W)
    words_full = (masks_timed == 0).sum().item() / n_words
    words_untouched = (masks_timed == -1).sum().item() / n_words
    words_mixed = 1.0 - words_full - words_untouched

    def recache():
        """After cold passes: one untimed pass without clears, so that the window's keys are all cached again."""
        rewind(False)
        for k in range(k0, total):
            step(False, k)
        torch.cuda.synchronize()

    extra = {}
    if not args.brief:
        spread_cold, parts_cold = step_spread(True), parts_spread(True)
        recache()
        spread_warm, parts_warm = step_spread(False), parts_spread(False)
        sec_fused_warm, sec_fused_cold = med(timed_fused(False)), med(timed_fused(True))

        # ---- the same K warm steps recorded once into a HIP graph and replayed (no host work per launch) ----
        def timed_graph_warm():
            side = torch.cuda.Stream()
            states.copy_(window_states)
            torch.cuda.synchronize()
            with torch.cuda.stream(side):
                h.decode_step(states, None, mask, ring[0], stream=side)
                for k in range(k0 - Wm + 1, k0):
                    h.decode_step(states, tokens[k - 1], mask, ring[k & 3], stream=side)
            side.synchronize()
            after_warmup = states.clone()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                for k in range(k0, total):
                    h.decode_step(states, tokens[k - 1], mask, ring[k & 3], stream=side)
            out = []
            for _ in range(N_PASSES):
                states.copy_(after_warmup)
                torch.cuda.synchronize()
                t = time.perf_counter()
                graph.replay()
                torch.cuda.synchronize()
                out.append((time.perf_counter() - t) / K)
            return med(out)

        recache()
        sec_graph_warm = timed_graph_warm()

        # ---- greedy variant of the step: fill, masked argmax (logits only read), advance ----
        greedy_tok = torch.empty(B, dtype=torch.int32, device="cuda")
        fresh = [(torch.randn((B, V), device="cuda", dtype=torch.float32) * w.sigma).to(tdt) for _ in range(4)]

        def greedy_step(cold, k):
            if cold:
                h.cache_clear()
            h.fill_masks(states, mask)
            wg.masked_argmax(fresh[k & 3], mask, greedy_tok)
            h.advance(states, greedy_tok)

        def timed_greedy(cold):
            def prepare():
                states.copy_(start)
                if cold:
                    h.cache_clear()
                for k in range(Wm):
                    greedy_step(cold, k)
            if not cold:                                  # a first pass over the same trajectory caches its keys
                h.cache_clear()
                prepare()
                for k in range(k0, total):
                    greedy_step(False, k)
            return med(passes(prepare, lambda k: greedy_step(cold, k), n=3))

        sec_greedy_cold = timed_greedy(True)
        sec_greedy_warm = timed_greedy(False)
        assert h.error_count() == 0, "greedy decoding chose an illegal token"
        torch.cuda.synchronize()
        e0.record()
        for k in range(K):
            wg.masked_argmax(fresh[k & 3], masks_timed[k], greedy_tok)
        e1.record()
        torch.cuda.synchronize()
        argmax_us = 1e3 * e0.elapsed_time(e1) / K
        # the candidates of top-k sampling under the same masks (logits only read)
        topk_k = 50
        topk_ids = torch.empty((B, topk_k), dtype=torch.int32, device="cuda")
        topk_vals = torch.empty((B, topk_k), dtype=tdt, device="cuda")
        topk_work = torch.empty(wg.masked_topk_workspace(B, V, topk_k), dtype=torch.uint8, device="cuda")
        for k in range(4):
            wg.masked_topk(fresh[k & 3], masks_timed[k % K], topk_ids, topk_vals, topk_work)
        torch.cuda.synchronize()
        e0.record()
        for k in range(K):
            wg.masked_topk(fresh[k & 3], masks_timed[k], topk_ids, topk_vals, topk_work)
        e1.record()
        torch.cuda.synchronize()
        topk_us = 1e3 * e0.elapsed_time(e1) / K
        row_b = V / 8.0
        extra = {
            "step_spread": {"note": "per-step times between events recorded at the step boundaries "
                                    "(fill + apply + advance, event cost included)",
                            "cold": spread_cold, "warm": spread_warm},
            "calls_spread": {"note": "the calls of a step between events recorded after each (event cost and the host's "
                                     "launch gaps included, so the parts add up to more than the step)",
                             "cold": parts_cold, "warm": parts_warm},
            "fused_advance_fill": {"note": "the same steps through wg_apply_mask + wg_advance_fill_masks",
                                   "cold_ms_per_step": sec_fused_cold * 1e3, "warm_ms_per_step": sec_fused_warm * 1e3,
                                   "cold_request_steps_per_s": B / sec_fused_cold,
                                   "warm_request_steps_per_s": B / sec_fused_warm},
            "greedy": {"note": "fill + wg_masked_argmax + advance; logits are read, never written",
                       "cold_ms_per_step": sec_greedy_cold * 1e3, "warm_ms_per_step": sec_greedy_warm * 1e3,
                       "cold_request_steps_per_s": B / sec_greedy_cold, "warm_request_steps_per_s": B / sec_greedy_warm,
                       "masked_argmax_us": argmax_us,
                       "masked_argmax_dense_read_GBs": B * (row_b + esz * V) / (argmax_us * 1e-6) / 1e9,
                       # the logits and the mask read once are this call's algorithmic bytes
                       "masked_argmax_frac_of_hbm_peak": B * (row_b + esz * V) / (argmax_us * 1e-6) / 1e9 / HBM_PEAK_GBS},
            "topk": {"note": "wg_masked_topk on the masks of the timed steps, k = %d; logits are read, never written" % topk_k,
                     "k": topk_k, "masked_topk_us": topk_us,
                     "masked_topk_dense_read_GBs": B * (row_b + esz * V) / (topk_us * 1e-6) / 1e9,
                     "masked_topk_frac_of_hbm_peak": B * (row_b + esz * V) / (topk_us * 1e-6) / 1e9 / HBM_PEAK_GBS},
            "host_setup": {"vocabulary_indexes_ms": vocab_ms, "compile_all_instances_ms": compile_ms,
                           "instances": len(w.texts),
                           "add_one_instance_us_median": float(np.median(join_us)) if join_us else None,
                           "add_one_instance_us_p90": float(np.percentile(join_us, 90)) if join_us else None,
                           "add_one_instance_call_only_us_median": float(np.median(join_call_us)) if join_call_us else None,
                           "add_one_instance_call_only_us_p90": float(np.percentile(join_call_us, 90)) if join_call_us else None},
            "hip_graph": {"note": "the K warm steps through wg_decode_step recorded once into a HIP graph and replayed",
                          "warm_ms_per_step": sec_graph_warm * 1e3},
        }

    # ---- algorithmic bytes per launch of each kernel: what the method has to move, not the
    # dense work it avoids ----
    sum_len = int(w.vocab.offsets[-1])
    row_bytes = V / 8.0
    n_class_rows = 3.0                                        # stay, end and their union
    scan_bytes_per_class = sum_len + V + n_class_rows * row_bytes      # token bytes + a length byte per token + the rows written
    key_bytes_per_key = 3 * row_bytes                           # one class row in, the row out twice (cache and bitmask)
    entry_bytes = 8.0
    gather_rows = B - builds_per_step                           # rows the gather copies (a claimer's row is written by key_build)
    gather_bytes_cold = gather_rows * 2 * row_bytes
    gather_bytes_warm = B * 2 * row_bytes
    apply_dense_bytes = B * (row_bytes + 2 * esz * V)
    apply_min_bytes = B * row_bytes + esz * disallowed_per_step      # mask in, -inf out, nothing else
    state_bytes = B * (8 + 4 + 8)                               # state in and out, token in
    alg = {
        "lookup": (B * 16.0, kt_cold["lookup_us"]),
        "class_scan": (scans_per_step * scan_bytes_per_class, kt_cold["scan_us"]),
        "key_build": (builds_per_step * key_bytes_per_key + entries_per_step * entry_bytes, kt_cold["build_us"]),
        "gather": (gather_bytes_cold, kt_cold["gather_us"]),
        "apply": (apply_min_bytes, kt_cold["apply_us"]),
        "advance": (state_bytes + B * (sum_len / float(V)), kt_cold["advance_us"]),
    }
    traffic_ok = kernel_source_sha256() == TRAFFIC_SOURCE_SHA256
    kernels = []
    for name, (nbytes, us) in alg.items():
        gbs = nbytes / (us * 1e-6) / 1e9 if us > 0 else 0.0
        kernels.append({"kernel": name, "algorithmic_bytes_per_launch": nbytes, "us_per_launch": us,
                        "achieved_GBs": gbs, "frac": gbs / HBM_PEAK_GBS,
                        "traffic": TRAFFIC_BYTES.get(w.index, {}).get(name) if traffic_ok else None,
                        "bound": "hbm" if name in ("class_scan", "key_build", "gather", "apply") else "latency"})
    dominant = max((k for k in kernels if k["bound"] == "hbm"), key=lambda k: k["us_per_launch"])
    method_bytes_cold = sum(v[0] for v in alg.values())
    method_bytes_warm = alg["lookup"][0] + gather_bytes_warm + apply_min_bytes + alg["advance"][0]
    # the same step in the accounting the throughput target is stated in: one streamed pass over the
    # vocabulary per built key, the gather, and a dense read-modify-write of the logits.  The kernels
    # move none of these bytes; the figure says what a scan-per-key design would have to sustain.
    scan_per_key_bytes = sum_len + V + row_bytes
    dense_cold = builds_per_step * scan_per_key_bytes + B * 2 * row_bytes + apply_dense_bytes
    dense_warm = B * 2 * row_bytes + apply_dense_bytes

    out = {
        "metric": "masked request-steps/sec at V=151,936 (cold cache)",
        "value": B / sec_cold,
        "unit": "request-steps/s",
        "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": sec_cold * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": "config %d (%s): B=%d, V=%d, %s logits, %d template instances, "
                               "seeded token stream" % (w.index, w.name, B, V, w.dtype, len(w.texts)),
                   "cache": "cold = cleared before every step; warm = all keys cached",
                   "window": "timed steps are steps %d .. %d of the trajectory" % (k0, total - 1),
                   "timing": "median of %d passes over the K steps, after %.0f ms of the same loop" % (N_PASSES, RAMP_SECONDS * 1e3),
                   "logits_dtype": w.dtype},
        "roofline": {"kernel": dominant["kernel"], "bound": "hbm", "achieved": dominant["achieved_GBs"],
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": dominant["frac"],
                     "traffic": dominant["traffic"],
                     "algorithmic_bytes_per_launch": dominant["algorithmic_bytes_per_launch"],
                     "us_per_launch": dominant["us_per_launch"],
                     "kernels": kernels,
                     "copy_ceiling_GBs": copy_ceiling_gbs},
        "cold": {"ms_per_step_passes": [s * 1e3 for s in cold_passes],
                 "keys_built_per_step": builds_per_step, "class_scans_per_step": scans_per_step,
                 "exit_entries_per_step": entries_per_step,
                 # token bytes taken through a checkpoint's byte table per second: by the class scan
                 # (every token once per scanned table, over the scan's own time), and what a walk of
                 # the whole vocabulary per built key would have to sustain at this step time
                 "byte_steps_per_s": {"class_scan": scans_per_step * sum_len / (kt_cold["scan_us"] * 1e-6) if kt_cold["scan_us"] > 0 else None,
                                      "scan_per_key_dense_equivalent": builds_per_step * sum_len / sec_cold},
                 "method_bytes_per_step": method_bytes_cold,
                 "step_frac_method_bytes": method_bytes_cold / sec_cold / 1e9 / HBM_PEAK_GBS,
                 "dense_equivalent_GBs": dense_cold / sec_cold / 1e9,
                 "frac_of_hbm_peak_dense_equivalent": dense_cold / sec_cold / 1e9 / HBM_PEAK_GBS},
        "warm": {"value": B / sec_warm, "unit": "request-steps/s", "ms_per_step": sec_warm * 1e3,
                 "ms_per_step_passes": [s * 1e3 for s in warm_passes],
                 "hit_rate": hit_rate,
                 "method_bytes_per_step": method_bytes_warm,
                 "step_frac_method_bytes": method_bytes_warm / sec_warm / 1e9 / HBM_PEAK_GBS,
                 "dense_equivalent_GBs": dense_warm / sec_warm / 1e9,
                 "frac_of_hbm_peak_dense_equivalent": dense_warm / sec_warm / 1e9 / HBM_PEAK_GBS},
        "kernels_us_per_step": {"cold": kt_cold, "warm": kt_warm},
        "single_call_step": {"note": "the same steps through wg_decode_step (advance + fill + apply, four launches)",
                             "cold_ms_per_step": sec_single_cold * 1e3, "warm_ms_per_step": sec_single_warm * 1e3,
                             "cold_request_steps_per_s": B / sec_single_cold,
                             "warm_request_steps_per_s": B / sec_single_warm,
                             "kernels_us_per_step": {"cold": dk_cold, "warm": dk_warm}},
        "apply": {"disallowed_fraction": disallowed_per_step / float(B * V),
                  "min_bytes_GBs": apply_min_bytes / (apply_us * 1e-6) / 1e9,
                  "dense_equivalent_GBs": apply_dense_bytes / (apply_us * 1e-6) / 1e9,
                  "groups_of_32_tokens": {"untouched": words_untouched, "fully_disallowed": words_full, "mixed": words_mixed}},
        "prepass": {"builds": pre["builds"], "lookups": pre["lookups"], "class_scans": pre["class_scans"]},
        "cpu_model": cpu_model(),
    }
    out.update(extra)
    if cpu is not None:
        cpu["cpu_model"] = cpu_model()
        out["cpu_baseline"] = cpu
    print(json.dumps(out))


if __name__ == "__main__":
    main()
