#!/usr/bin/env python3
"""Benchmark of the E3 hot path on one MI355X.

One step = one pass of the whole path over one decode batch of the paper's shape
(Section 5.1: 64 prompts x 8 rollouts; a 151,936-entry vocabulary, bf16 logits):

  1. + 2. e3_logprob_entropy_advantages  training side, one call: Eq. 2 over the 64 groups of
                         8 rewards (computed inside the vocabulary pass's launch), log-prob of
                         the previously sampled tokens, entropy, batch entropy sum/count on
                         the training-pass logits
  3. e3_sample_entropy   rollout side: token, log-prob, entropy per row      (dominant)
  4. e3_temperature_update (Eq. 4 / Eq. 5) on the host, from the 16 bytes that 2. stores into
     pinned host memory (the host waits for an event behind 2. only, so 4. overlaps 3.)

Inputs are resident in HBM before timing starts.  The batch is 156 MB, smaller than
the 256 MB memory-side cache, so the step rotates over enough distinct logit buffers
that more than 1 GB is touched between two uses of the same buffer.

Prints ONE JSON line.  `value` comes from K plain steps; `roofline` prices the sample kernel's
algorithmic bytes against the 8 TB/s HBM peak using HIP events attached to every dispatch in a
second run of the same K steps; `read_ceiling` is a read-only kernel over the same buffers timed
the same way; `other_configs` holds the kernel's figures on configs 3, 4 and 5;
`cpu_baseline` times the CPU oracle on the same workload (reported, not a target).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

V = 151_936
PROMPTS, ROLLOUTS = 64, 8
ROWS = PROMPTS * ROLLOUTS
HBM_PEAK_GBPS = 8000.0
# algorithmic bytes of one sampled row: V bf16 logits + tau (4) read, token/logp/entropy (12) written
BYTES_PER_ROW = V * 2 + 4 + 12
TRAFFIC_RECORD = os.path.join(ROOT, "profiles", "vocab_pass_decode_step_hbm_traffic.txt")
KERNEL_SOURCES = ("vocab_pass.hip", "vocab_common.h", "vocab_pass.h", "advantages.h")


def kernel_source_sha256() -> str:
    """Hash of the sources the vocabulary-pass kernels are compiled from."""
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2505_18573_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic_bytes():
    """HBM bytes per launch of the sample kernel from rocprofv3 FETCH_SIZE + WRITE_SIZE, each
    scaled by what the same counter reads for a device copy of known size.  The summary under
    profiles/ records the figure together with the hash of the kernel sources it was taken
    with; once the sources have changed the figure is stale and None is reported."""
    import re
    try:
        text = open(TRAFFIC_RECORD).read()
    except OSError:
        return None
    m = re.search(r"^traffic_bytes_per_launch sample: (\d+) kernel_sources_sha256: ([0-9a-f]{64})$", text, re.M)
    if m is None or m.group(2) != kernel_source_sha256():
        return None
    return int(m.group(1))


class DispatchEvents:
    """hipEvent_t pairs that the library attaches to a kernel dispatch (e3_time_next_launch):
    their difference is the kernel's own execution time, as a profiler reports it."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p,
                                                 ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def pair(self):
        a, b = ctypes.c_void_p(), ctypes.c_void_p()
        if self.hip.hipEventCreate(ctypes.byref(a)) != 0 or self.hip.hipEventCreate(ctypes.byref(b)) != 0:
            raise RuntimeError("hipEventCreate failed")
        return a, b

    def elapsed_ms(self, a, b) -> float:
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return ms.value

    def destroy(self, pairs):
        for a, b in pairs:
            self.hip.hipEventDestroy(a)
            self.hip.hipEventDestroy(b)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--buffers", type=int, default=8, help="distinct logit buffers rotated over")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the kernel timings on configs 3 (dynamic budgets), 4 (training pass) and "
                         "5 (large decode batch) that the default run reports in `other_configs`")
    ap.add_argument("--no-restricted", action="store_true",
                    help="skip the timings of e3_sample_restricted (top-k / top-p settings, bf16 and fp32 rows, on "
                         "the same rotating batches) that the default run reports in `restricted_sampling`; "
                         "they are not part of the step")
    ap.add_argument("--restricted", action="store_true", help="accepted for older command lines: the default now")
    ap.add_argument("--sizes", action="store_true",
                    help="also time the two vocabulary-pass kernels and the read probe on other batch "
                         "sizes and on fp32 logits (back-to-back launches, dispatch events)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain device copy of one logit buffer 10 times (a kernel of "
                         "known traffic: 155.6 MB read + 155.6 MB written) so that a rocprofv3 "
                         "--pmc run can scale FETCH_SIZE / WRITE_SIZE against it")
    ap.add_argument("--kernel-sources-sha256", action="store_true",
                    help="print the hash that a measured-traffic record under profiles/ is keyed to, and exit")
    args = ap.parse_args()
    if args.kernel_sources_sha256:
        print(kernel_source_sha256())
        return 0
    if args.gpus != 1:
        print("bench.py measures one GPU: the path has no cross-GPU step (rows are independent); "
              "run with --gpus 1", file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2

    import paper_2505_18573_amd as e3
    from paper_2505_18573_amd import workloads as wl

    e3.lib()                                   # fail loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    nb = max(2, args.buffers)
    batches = [wl.decode_step(dev, seed=1 + i, prompts=PROMPTS, rollouts=ROLLOUTS, V=V)
               for i in range(nb)]
    offsets = torch.arange(0, ROWS + 1, ROLLOUTS, dtype=torch.int32, device=dev)
    g = torch.Generator(device=dev).manual_seed(1234)
    rewards = (torch.rand(ROWS, generator=g, device=dev) < 0.4).float()

    tok = torch.empty(ROWS, dtype=torch.int32, device=dev)
    logp_s = torch.empty(ROWS, dtype=torch.float32, device=dev)
    ent_s = torch.empty(ROWS, dtype=torch.float32, device=dev)
    logp_t = torch.empty(ROWS, dtype=torch.float32, device=dev)
    ent_t = torch.empty(ROWS, dtype=torch.float32, device=dev)
    adv = torch.empty(ROWS, dtype=torch.float32, device=dev)
    # (sum of entropies fp64, count int64): 16 bytes of pinned host memory that the last
    # kernel of the training pass stores into directly, so no copy follows it
    stats_host = torch.zeros(2, dtype=torch.int64, pin_memory=True)
    hsum = stats_host[0:1].view(torch.float64)
    hcnt = stats_host[1:2]
    stats_np = stats_host.numpy()
    hsum_np = stats_np[0:1].view("float64")
    ws = e3.new_workspace(ROWS, V, dev)

    if args.copy_probe:
        dst = torch.empty_like(batches[0].logits)
        for i in range(10):
            dst.copy_(batches[i % nb].logits)
        torch.cuda.synchronize()
        del dst

    state = {"tau": 1.0, "H_init": None, "t": 0}
    stream = torch.cuda.current_stream(dev)

    stats_ready = torch.cuda.Event()

    def step(i: int, ev=None, ev_train=None):
        """One cycle of the method: advantages, training pass on the previous rollouts (its
        mean entropy H_t goes to the host), next rollouts, scheduler.  The host waits only for
        the event behind the training pass, whose 16 bytes land in pinned host memory, so Eq. 4 / Eq. 5 run on the host
        while the rollout kernel is still executing; the temperature they produce is the one
        the following step's rollouts would use.  `ev`: a HIP event pair that the library
        attaches to the sampling kernel's dispatch (begin and end of its execution); `ev_train`:
        the same for the training-side call (begin of its vocabulary pass, end of the reduction
        kernel that follows it)."""
        roll = batches[i % nb]
        train = batches[(i + nb // 2) % nb]
        if ev_train is not None:
            e3.e3_time_next_launch(ev_train[0].value, ev_train[1].value)
        e3.e3_logprob_entropy_advantages(train.logits, tok, None, train.tau_rows, 1.0, rewards, offsets,
                                         0, 0.0, logp_out=logp_t, entropy_out=ent_t,
                                         entropy_sum_out=hsum, entropy_count_out=hcnt, adv_out=adv,
                                         workspace=ws)
        stats_ready.record(stream)
        if ev is not None:
            e3.e3_time_next_launch(ev[0].value, ev[1].value)
        e3.e3_sample_entropy(roll.logits, roll.tau_rows, 1.0, seed=99, row_base=i * ROWS,
                             token_out=tok, logp_out=logp_s, entropy_out=ent_s, workspace=ws)
        stats_ready.synchronize()
        H_t = float(hsum_np[0]) / max(1, int(stats_np[1]))
        if state["H_init"] is None:
            state["H_init"] = H_t              # mean entropy of the first batch (Eq. 4)
        state["tau"], _ = e3.e3_temperature_update(state["tau"], H_t, state["H_init"], V,
                                                   t=state["t"], t_anneal=288, t_max=480, eta=0.9,
                                                   tau_min=0.05, tau_max=20.0)
        state["t"] += 1

    tok.zero_()                                # targets of the very first training pass
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    dev_events = DispatchEvents()
    # Timed region: K steps as a caller runs them, nothing attached.
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    # The same K steps once more with HIP events attached to every dispatch of the two calls,
    # for the kernels' own durations.  They are kept out of the timed region because they are
    # not free: an event-carrying dispatch costs the stream about 4 us (the step grows from
    # ~67 to ~82 us with three of them), and a dispatch that follows a plain one is charged
    # 1.5-2 us of its predecessor's retirement, so either every dispatch of the step carries
    # events (as under a profiler's kernel trace) or none does.
    events = [dev_events.pair() for _ in range(args.steps)]
    events_train = [dev_events.pair() for _ in range(args.steps)]
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + args.steps + i, events[i], events_train[i])
    torch.cuda.synchronize()
    t3 = time.perf_counter()

    # The same launches bracketed by marker events (torch.cuda.Event pairs recorded on the
    # stream), for reference: markers are packets of their own and read ~5 us more.
    markers = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(50)]
    for j, (a_ev, b_ev) in enumerate(markers):
        roll = batches[j % nb]
        e3.e3_grpo_advantages(rewards, offsets, 0, 0.0, adv_out=adv)
        a_ev.record(stream)
        e3.e3_sample_entropy(roll.logits, roll.tau_rows, 1.0, seed=99, row_base=j * ROWS,
                             token_out=tok, logp_out=logp_s, entropy_out=ent_s, workspace=ws)
        b_ev.record(stream)
    torch.cuda.synchronize()
    marker_ms = sorted(x.elapsed_time(y) for x, y in markers)

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    rows_per_s = ROWS * args.steps / (t1 - t0)
    kern_ms = sorted(dev_events.elapsed_ms(a, b) for a, b in events)
    dev_events.destroy(events)
    train_ms = sorted(dev_events.elapsed_ms(a, b) for a, b in events_train)
    dev_events.destroy(events_train)
    kern_avg_ms = sum(kern_ms) / len(kern_ms)
    achieved = ROWS * BYTES_PER_ROW / (kern_avg_ms * 1e-3) / 1e9

    out = {
        "metric": "fused temp-sample+entropy rows/s at V=151,936 (whole step: sample+entropy, "
                  "advantages, training-side logprob+entropy, scheduler)",
        "value": rows_per_s,
        "unit": "rows/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_with_dispatch_events": (t3 - t2) * 1e3 / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32 accumulation over bf16 logits",
        "data": "synthetic",
        "config": {
            "workload": "decode_step (config 2): 64 prompts x 8 rollouts = 512 rows, V=151936, "
                        "bf16 logits N(0,3^2) + 20 columns/row boosted by 8, per-row tau U[0.6,1.4]",
            "rows": ROWS, "V": V, "logits_dtype": "bf16", "rotating_buffers": nb,
            "bytes_per_step_sample": ROWS * BYTES_PER_ROW,
        },
        "sample_kernel": {
            "avg_ms": kern_avg_ms, "median_ms": kern_ms[len(kern_ms) // 2], "min_ms": kern_ms[0],
            "rows_per_s": ROWS / (kern_avg_ms * 1e-3),
            "timing": "HIP events attached to the kernel's dispatch (hipExtLaunchKernel start/stop events via "
                      "e3_time_next_launch) in a second run of the same K steps right after the timed region, "
                      "in which every dispatch of the step carries events; the timed region itself runs "
                      "without them (they cost the stream ~4 us per dispatch)",
            "marker_pair_avg_ms": sum(marker_ms) / len(marker_ms),
            "marker_pair_note": "the same launch bracketed by two recorded marker events instead",
        },
        "training_call": {
            "avg_ms": sum(train_ms) / len(train_ms), "median_ms": train_ms[len(train_ms) // 2],
            "what": "e3_logprob_entropy_advantages on the same shape: begin of the vocabulary pass (with the "
                    "64 groups' advantages aboard) to the end of the batch-sum kernel that follows it, "
                    "dispatch events, same instrumented run of the K steps as the sample kernel",
        },
        "roofline": {
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBPS, "traffic": measured_traffic_bytes(),
            "kernel": "vocab_pass_kernel<bf16, sample>",
        },
        "scheduler": {"tau_after": state["tau"], "H_init": state["H_init"]},
    }

    out["read_ceiling"] = read_ceiling_leg(e3, batches, dev_events)
    out["roofline"]["frac_of_read_ceiling"] = achieved / out["read_ceiling"]["GBps"]
    out["roofline"]["limiter"] = limiter(kern_avg_ms, out["read_ceiling"]["avg_ms"])
    out["roofline"]["limiter_rule"] = LIMITER_RULE
    if not args.no_restricted:                       # before the buffers are released: it rotates over them
        out["restricted_sampling"] = restricted_leg(e3, batches, stream)
    if not args.no_other_configs:
        keep = batches[0]
        del batches
        torch.cuda.empty_cache()
        batches = [keep]
        out["other_configs"] = other_configs_leg(e3, wl, dev, dev_events)
    if args.sizes:
        del batches[1:]
        torch.cuda.empty_cache()
        out["other_sizes"] = sizes_leg(e3, dev, dev_events)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(batches[0], rewards, offsets)
    print(json.dumps(out))
    return 0


LIMITER_RULE = ("hbm when the kernel takes at most 1.05x the read-only probe on the same buffers (the memory "
                "system sets its time), else valu (vector-ALU issue and the row epilogues hold it back; "
                "rocprofv3 SQ counters under profiles/)")


def limiter(kernel_ms: float, probe_ms: float) -> str:
    return "hbm" if kernel_ms <= 1.05 * probe_ms else "valu"


def timed_launches(e3, dev_events, fn, nbuf: int, reps: int):
    """Average execution time (ms) of the vocabulary-pass dispatch inside fn(i), launched back
    to back over rotating buffers, from events attached to the dispatch itself."""
    warm = nbuf + 2                                  # every buffer once before timing
    evs = [dev_events.pair() for _ in range(reps)]
    for i in range(warm + reps):
        if i >= warm:
            e3.e3_time_next_launch(evs[i - warm][0].value, evs[i - warm][1].value)
        fn(i)
    torch.cuda.synchronize()
    ms = sorted(dev_events.elapsed_ms(a, b) for a, b in evs)
    dev_events.destroy(evs)
    return sum(ms) / len(ms), ms[len(ms) // 2]


def read_ceiling_leg(e3, batches, dev_events, reps: int = 50):
    """What a pure read of the same logit buffers reaches on this machine, timed exactly like
    the sample kernel (events attached to the dispatch, back-to-back launches, rotating
    buffers)."""
    dev = batches[0].logits.device
    sums = torch.empty(e3.binding.E3_READ_PROBE_SUMS, dtype=torch.int32, device=dev)
    avg, med = timed_launches(e3, dev_events, lambda i: e3.e3_read_probe(batches[i % len(batches)].logits, sums),
                              len(batches), reps)
    nbytes = ROWS * V * 2
    return {"kernel": "read_probe_kernel (16-byte non-temporal loads, 8-wave workgroups over contiguous "
                      "16-KiB runs, xor checksum only)",
            "avg_ms": avg, "median_ms": med, "GBps": nbytes / (avg * 1e-3) / 1e9,
            "frac_of_hbm_peak": nbytes / (avg * 1e-3) / 1e9 / HBM_PEAK_GBPS}


def other_configs_leg(e3, wl, dev, dev_events):
    """The vocabulary-pass kernel of each of the other full-size configurations on its own
    generator's inputs: dynamic budgets (config 3: sample + entropy over 1024 rollouts, the
    128 variable-size groups' advantages in a launch of their own), training pass (config 4:
    log-prob of the target + entropy over 32,768 tokens, batch entropy sum), large decode
    batch (config 5: 4096 rows at tau 0.3 / 2.0 with near-tied rows).  Back-to-back launches
    over rotating buffers of more than 1 GB in total, dispatch events; the read-only probe on
    the same buffers beside each."""
    res = []
    sums = torch.empty(e3.binding.E3_READ_PROBE_SUMS, dtype=torch.int32, device=dev)

    def entry(name, kernel, rows, nbuf, reps, fn, probe_fn, extra=None):
        nbytes = rows * (V * 2 + 4 + 12)
        avg, med = timed_launches(e3, dev_events, fn, nbuf, reps)
        p_avg, _ = timed_launches(e3, dev_events, probe_fn, nbuf, reps)
        gbps = nbytes / (avg * 1e-3) / 1e9
        e = {"config": name, "kernel": kernel, "rows": rows, "V": V, "logits_dtype": "bf16",
             "kernel_avg_us": avg * 1e3, "kernel_median_us": med * 1e3, "rows_per_s": rows / (avg * 1e-3),
             "GBps": gbps, "frac": gbps / HBM_PEAK_GBPS,
             "read_probe_avg_us": p_avg * 1e3,
             "read_probe_frac": rows * V * 2 / (p_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS,
             "limiter": limiter(avg, p_avg)}
        if extra:
            e.update(extra)
        res.append(e)

    # config 3: 1024 rollouts in 128 groups of 2..32
    nbuf = 4
    ws3 = [wl.dynamic_budgets(dev, seed=2 + i) for i in range(nbuf)]
    rows = ws3[0].rows
    tok = torch.empty(rows, dtype=torch.int32, device=dev)
    lp = torch.empty(rows, dtype=torch.float32, device=dev)
    en = torch.empty(rows, dtype=torch.float32, device=dev)
    adv = torch.empty(rows, dtype=torch.float32, device=dev)
    ws = e3.new_workspace(rows, V, dev)
    a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(3):
        e3.e3_grpo_advantages(ws3[0].rewards, ws3[0].group_offsets, 0, 0.0, adv_out=adv)
    a0.record()
    for i in range(20):
        e3.e3_grpo_advantages(ws3[i % nbuf].rewards, ws3[i % nbuf].group_offsets, 0, 0.0, adv_out=adv)
    a1.record()
    torch.cuda.synchronize()
    entry("dynamic_budgets (config 3)", "vocab_pass_kernel<bf16, sample>", rows, nbuf, 40,
          lambda i: e3.e3_sample_entropy(ws3[i % nbuf].logits, ws3[i % nbuf].tau_rows, 1.0, seed=2, row_base=i * rows,
                                         token_out=tok, logp_out=lp, entropy_out=en, workspace=ws),
          lambda i: e3.e3_read_probe(ws3[i % nbuf].logits, sums),
          {"advantages_launch_us": a0.elapsed_time(a1) * 1e3 / 20, "groups": 128})
    del ws3
    torch.cuda.empty_cache()

    # config 5: 4096 rows, tau in {0.3, 2.0}, 10 % near-tied rows
    nbuf = 2
    ws5 = [wl.large_decode(dev, seed=4 + i) for i in range(nbuf)]
    rows = ws5[0].rows
    tok = torch.empty(rows, dtype=torch.int32, device=dev)
    lp = torch.empty(rows, dtype=torch.float32, device=dev)
    en = torch.empty(rows, dtype=torch.float32, device=dev)
    entry("large_decode (config 5)", "vocab_pass_kernel<bf16, sample>", rows, nbuf, 30,
          lambda i: e3.e3_sample_entropy(ws5[i % nbuf].logits, ws5[i % nbuf].tau_rows, 1.0, seed=4, row_base=i * rows,
                                         token_out=tok, logp_out=lp, entropy_out=en, workspace=False),
          lambda i: e3.e3_read_probe(ws5[i % nbuf].logits, sums))
    del ws5
    torch.cuda.empty_cache()

    # config 4: 32,768 response tokens (9.96 GB, far beyond every cache: one buffer)
    w4 = wl.training_pass(dev)
    rows = w4.rows
    lp = torch.empty(rows, dtype=torch.float32, device=dev)
    en = torch.empty(rows, dtype=torch.float32, device=dev)
    hs = torch.empty(1, dtype=torch.float64, device=dev)
    hc = torch.empty(1, dtype=torch.int64, device=dev)
    entry("training_pass (config 4)", "vocab_pass_kernel<bf16, logprob>", rows, 1, 10,
          lambda i: e3.e3_logprob_entropy(w4.logits, w4.target_ids, None, None, 1.0, logp_out=lp, entropy_out=en,
                                          entropy_sum_out=hs, entropy_count_out=hc, workspace=False),
          lambda i: e3.e3_read_probe(w4.logits, sums),
          {"batch_mean_entropy": None})
    torch.cuda.synchronize()
    res[-1]["batch_mean_entropy"] = hs.item() / max(1, hc.item())
    del w4
    torch.cuda.empty_cache()
    return res


def sizes_leg(e3, dev, dev_events, reps: int = 40):
    """Sample kernel, training-side kernel and read probe on other row counts of the same
    vocabulary, bf16 and fp32 logits N(0, 3^2), per-row tau U[0.6, 1.4]: back-to-back launches
    rotating over buffers that together exceed 1 GB, timed by dispatch events."""
    res = []
    for dtype, esz, row_list in ((torch.bfloat16, 2, (16, 64, 256, 1024, 2048, 4096, 16384)),
                                 (torch.float32, 4, (512, 2048, 8192))):
        for rows in row_list:
            nbytes = rows * V * esz
            nbuf = max(2, min(8, int(2.5e9 // nbytes)))
            bufs = [(torch.randn((rows, V), device=dev) * 3).to(dtype) for _ in range(nbuf)]
            tau = (0.6 + 0.8 * torch.rand(rows, device=dev)).float()
            tok = torch.empty(rows, dtype=torch.int32, device=dev)
            lp = torch.empty(rows, dtype=torch.float32, device=dev)
            en = torch.empty(rows, dtype=torch.float32, device=dev)
            tgt = torch.randint(0, V, (rows,), device=dev).to(torch.int32)
            ws = e3.new_workspace(rows, V, dev)
            sums = torch.empty(e3.binding.E3_READ_PROBE_SUMS, dtype=torch.int32, device=dev)
            calls = {
                "sample": lambda i: e3.e3_sample_entropy(bufs[i % nbuf], tau, 1.0, 1, 0, token_out=tok,
                                                         logp_out=lp, entropy_out=en, workspace=ws),
                "logprob": lambda i: e3.e3_logprob_entropy(bufs[i % nbuf], tgt, None, tau, 1.0, logp_out=lp,
                                                           entropy_out=en, want_sum=False, workspace=ws),
                "read": lambda i: e3.e3_read_probe(bufs[i % nbuf], sums),
            }
            entry = {"rows": rows, "logits_dtype": "bf16" if esz == 2 else "f32"}
            for name, fn in calls.items():
                warm = nbuf + 2                      # every buffer once before timing
                evs = [dev_events.pair() for _ in range(reps)]
                for i in range(warm + reps):
                    if i >= warm:
                        e3.e3_time_next_launch(evs[i - warm][0].value, evs[i - warm][1].value)
                    fn(i)
                torch.cuda.synchronize()
                ms = [dev_events.elapsed_ms(a, b) for a, b in evs]
                dev_events.destroy(evs)
                avg = sum(ms) / len(ms)
                entry[name] = {"avg_us": avg * 1e3, "frac_of_hbm_peak": nbytes / (avg * 1e-3) / 1e9 / HBM_PEAK_GBPS}
            res.append(entry)
            del bufs, calls
            torch.cuda.empty_cache()
    return res


def restricted_leg(e3, batches, stream, reps: int = 50):
    """Top-k / top-p sampling of the same decode batches (HIP events around each launch)."""
    dev = batches[0].logits.device
    tok = torch.empty(ROWS, dtype=torch.int32, device=dev)
    lp = torch.empty(ROWS, dtype=torch.float32, device=dev)
    kept = torch.empty(ROWS, dtype=torch.int32, device=dev)
    res = {}
    f32 = [b.logits.float() for b in batches[:4]]            # fp32 rows of the same batches (1.2 GB)
    settings = (("top_k50", 50, 1.0, 2), ("top_k50_top_p0.95", 50, 0.95, 2), ("top_k256_top_p0.9", 256, 0.9, 2),
                ("top_p0.9", 0, 0.9, 2), ("f32_top_k50", 50, 1.0, 4), ("f32_top_k50_top_p0.95", 50, 0.95, 4))
    for name, k, p, esz in settings:
        rot = len(batches) if esz == 2 else len(f32)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(reps)]
        for i in range(5 + reps):
            b = batches[i % rot]
            logits = b.logits if esz == 2 else f32[i % rot]
            if i >= 5:
                evs[i - 5][0].record(stream)
            e3.e3_sample_restricted(logits, b.tau_rows, 1.0, k, p, seed=7, row_base=i * ROWS,
                                    token_out=tok, logp_out=lp, kept_out=kept)
            if i >= 5:
                evs[i - 5][1].record(stream)
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in evs)
        avg = sum(ms) / len(ms)
        res[name] = {"avg_ms": avg, "median_ms": ms[len(ms) // 2], "rows_per_s": ROWS / (avg * 1e-3),
                     "logit_GBps": ROWS * V * esz / (avg * 1e-3) / 1e9,
                     "frac_of_hbm_peak": ROWS * V * esz / (avg * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "mean_kept": float(kept.float().mean().item())}
    return res


def cpu_baseline(batch, rewards, offsets):
    """The oracle as it stands, timed on this machine's host cores over the same step."""
    from oracle import e3_oracle as o
    from paper_2505_18573_amd import binding as e3b
    from paper_2505_18573_amd import workloads as wl

    threads = max(1, min(16, os.cpu_count() or 1, o.max_threads()))
    part = (e3b.E3_TILE_CHUNK, e3b.E3_TILE_LANES, e3b.E3_TILE_DEPTH)   # the sampler the library fixes
    bits = wl.host_bits(batch.logits)
    tau = batch.tau_rows.cpu().numpy()
    r = rewards.cpu().numpy()
    off = offsets.cpu().numpy()
    reps = 10
    o.sample_entropy(bits[:threads], tau[:threads], 1.0, 99, 0, partition=part, nthreads=threads)   # warm the pages
    t0 = time.perf_counter()
    for k in range(reps):
        s = o.sample_entropy(bits, tau, 1.0, 99, k * ROWS, partition=part, nthreads=threads)
        o.grpo_advantages(r, off)
        lp = o.logprob_entropy(bits, s.token, None, tau, 1.0, nthreads=threads)
        o.temperature_update(1.0, lp.entropy_mean, lp.entropy_mean, V)
    dt = time.perf_counter() - t0
    # the same step on one thread, over the first 64 rows (8 groups)
    n1 = 64
    t0 = time.perf_counter()
    s1 = o.sample_entropy(bits[:n1], tau[:n1], 1.0, 99, 0, partition=part, nthreads=1)
    o.grpo_advantages(r[:n1], off[:n1 // ROLLOUTS + 1])
    o.logprob_entropy(bits[:n1], s1.token, None, tau[:n1], 1.0, nthreads=1)
    dt1 = time.perf_counter() - t0
    return {
        "value": ROWS * reps / dt, "unit": "rows/s", "cores": threads, "host_cpus": os.cpu_count(),
        "cores_note": "threads the oracle ran on: at most 16, this box's CPU share, whatever os.cpu_count() shows",
        "kind": "oracle",
        "sample": f"{reps} full steps of the same 512-row batch ({ROWS * reps} rows), fp64, "
                  f"OpenMP over rows",
        "seconds": dt,
        "logit_GBps": ROWS * reps * 2 * V * 2 / dt / 1e9,
        "single_thread": {"value": n1 / dt1, "unit": "rows/s", "cores": 1,
                          "sample": f"one step over the first {n1} rows", "seconds": dt1},
    }


if __name__ == "__main__":
    sys.exit(main())
