#!/usr/bin/env python3
"""Benchmark: linear-attention forward + backward on one MI355X.

A step is one la_forward followed by one la_backward over one batch of
synthetic input that is already resident in device memory.  Prints one JSON
line with the tokens/s of the step, the roofline of the dominant kernel
(measured with HIP events recorded by the library between its kernels) and the
CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published


class HipEvents:
    """hipEvent_t handles created through the HIP runtime torch already loaded."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p,
                                                 ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.handles = (ctypes.c_void_p * n)()
        for i in range(n):
            h = ctypes.c_void_p()
            rc = self.hip.hipEventCreate(ctypes.byref(h))
            if rc != 0:
                raise RuntimeError("hipEventCreate failed: %d" % rc)
            self.handles[i] = h

    def elapsed_ms(self, i, j):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), self.handles[i], self.handles[j])
        if rc != 0:
            raise RuntimeError("hipEventElapsedTime failed: %d" % rc)
        return float(ms.value)

    def destroy(self):
        for h in self.handles:
            self.hip.hipEventDestroy(h)


def make_device_inputs(cfg, torch, n_sets):
    """Synthetic inputs with the workload's recipe, drawn on the device: Q, K
    Gaussian with unit-norm rows, V and dO standard Gaussian, cast to the I/O type."""
    td = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    gen = torch.Generator(device="cuda")
    gen.manual_seed(251021956)
    sets = []
    shape = (cfg.B, cfg.H, cfg.N, cfg.D)
    for _ in range(n_sets):
        t = {}
        for name in ("Q", "K", "V", "dO"):
            x = torch.randn(shape, device="cuda", dtype=torch.float32, generator=gen)
            if name in ("Q", "K"):
                x = x / x.norm(dim=-1, keepdim=True)
            t[name] = x.to(td).contiguous()
        t["O"] = torch.empty(shape, device="cuda", dtype=td)
        t["G"] = torch.empty(shape[:3], device="cuda", dtype=torch.float32)
        for name in ("dQ", "dK", "dV"):
            t[name] = torch.empty(shape, device="cuda", dtype=td)
        sets.append(t)
    return sets


def cpu_baseline(cfg, budget_slices):
    """Time the fp64 oracle (running-sum forward + backward) on a bounded sample
    of (batch, head) slices of the same workload, on the host cores."""
    import numpy as np

    import la_workloads as wl
    import oracle

    n = min(budget_slices, cfg.B * cfg.H)
    x = wl.workload_inputs(cfg, bh_subset=list(range(n)))
    Q, K, V, dO = (x[k][1] for k in ("Q", "K", "V", "dO"))
    oracle.forward_rec(Q[:1, :64], K[:1, :64], V[:1, :64], cfg.a, cfg.b, cfg.causal)  # load lib
    # repeat the sample until about a second of wall time (10-20 s of CPU work) has passed
    reps, dt = 0, 0.0
    t0 = time.perf_counter()
    while reps < 20 and dt < 1.0:
        O, G = oracle.forward_rec(Q, K, V, cfg.a, cfg.b, cfg.causal)
        oracle.backward_rec(Q, K, V, O, G, dO, cfg.a, cfg.b, cfg.causal)
        reps += 1
        dt = time.perf_counter() - t0
    tokens = reps * n * cfg.N / cfg.H  # a token is one (batch, position); it has H heads
    cores = min(oracle.num_threads(), n)
    return {
        "value": tokens / dt,
        "unit": "tokens/s",
        "cores": cores,
        "kind": "oracle",
        "sample": "%d of %d (batch,head) slices of %s, fp64 running-sum forward+backward, "
                  "%d passes, %.1f s wall on %d threads" % (n, cfg.B * cfg.H, cfg.name, reps, dt,
                                                            cores),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--clock-warmup-ms", type=float, default=150.0,
                    help="after the warm-up steps and a first timing of --steps steps, keep "
                         "running steps for this long, then time --steps steps again: that "
                         "second timing is the reported one (0 = report the first)")
    ap.add_argument("--config", type=int, default=1, help="index into la_workloads.CONFIGS")
    ap.add_argument("--workload", default=None,
                    help="a workload by name instead of --config: one of la_workloads.CONFIGS "
                         "or la_workloads.PAPER_SHAPES (the paper's own benchmark shapes)")
    ap.add_argument("--forward-only", action="store_true",
                    help="time la_forward alone (the quantity of the paper's Table 1)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--independent", action="store_true",
                    help="time la_forward + la_backward (no hand-over of running sums)")
    ap.add_argument("--no-all-configs", action="store_true",
                    help="skip the short runs of the other benchmark configurations")
    ap.add_argument("--extras", action="store_true",
                    help="also time the entry points beyond la_forward / la_backward (decode "
                         "step, normalisation inside the call, coefficient gradients, head size "
                         "256) and add them under the key 'extras'")
    ap.add_argument("--seg-len", type=int, default=0,
                    help="force the rows per segment (la_debug_override; 0: the library's plan)")
    ap.add_argument("--cpu-slices", type=int, default=64)
    ap.add_argument("--buffer-sets", type=int, default=0,
                    help="independent input/output sets rotated through (0: enough to exceed "
                         "the 256 MB last-level cache)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="instead of the benchmark, run a plain 1 GiB device copy a few times "
                         "(reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.copy_calibration:
        import torch
        n = 1 << 28  # 2^28 floats = 1 GiB
        src = torch.full((n,), 1.0, device="cuda")
        dst = torch.empty_like(src)
        flush = torch.empty(1 << 28, device="cuda")
        for _ in range(5):
            flush.fill_(0.0)      # push src/dst out of the caches
            dst.copy_(src)        # the copy kernel of known size: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": 4 * n}))
        return
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU only: this build has no multi-GPU path "
                 "(run with --gpus 1)")

    import torch

    import la_workloads as wl
    import paper_2510_21956_amd as la

    la.load_library()  # raises if the HIP library has not been built; no fallback
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    torch.cuda.set_device(0)
    la.la_debug_override(args.seg_len, 0)
    cfg = wl.find_workload(args.workload) if args.workload else wl.CONFIGS[args.config]
    out = measure(cfg, args, args.steps, args.warmup, torch, wl, la)
    if not args.no_all_configs and not args.workload and not args.forward_only:
        # the other benchmark configurations (the smallest is a parity case only), same
        # entry points, same step counts: timed rows next to the headline one
        rows = {}
        for i, c in enumerate(wl.CONFIGS):
            if i == 0 or c is cfg:
                continue
            r = measure(c, args, args.steps, args.warmup, torch, wl, la)
            rows[c.name] = {
                "ms_per_step": r["ms_per_step"], "tokens_per_s": r["value"],
                "first_steps_ms_per_step": r["first_steps"]["ms_per_step"],
                "whole_pass_frac_of_hbm_peak": r["whole_pass"]["frac_of_hbm_peak"],
                "dominant_kernel": r["roofline"]["kernel"] if r["roofline"] else None,
                "dominant_kernel_frac": r["roofline"]["frac"] if r["roofline"] else None,
                "kernels_ms": r["kernels_ms"], "steps": r["steps"], "dtype": r["dtype"]}
        out["all_configs"] = rows
    if args.extras:
        out["extras"] = extras(torch, wl, la)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, args.cpu_slices)
    print(json.dumps(out))


def extras(torch, wl, la):
    """Timings of the other entry points on synthetic inputs of the benchmark's recipe."""
    def timed(fn, reps, warm=5):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / reps

    res = {}
    # decode: one new token per slice, state carried in place
    B, H, D = 8, 16, 128
    x = {n: torch.randn((B, H, 1, D), device="cuda").to(torch.bfloat16) for n in "qkv"}
    o = torch.empty_like(x["q"])
    g = torch.empty((B, H, 1), device="cuda")
    st = torch.zeros(la.la_decode_state_bytes(B, H, D) // 4, device="cuda")
    ms = timed(lambda: la.la_decode_step(x["q"], x["k"], x["v"], o, g, st, 1.0, 0.5), 200)
    res["decode_step_bf16_B8_H16_D128_T1"] = {
        "us_per_step": ms * 1e3, "tokens_per_s": B / (ms * 1e-3),
        "state_GBs": 2 * st.numel() * 4 / (ms * 1e-3) / 1e9}
    # normalisation inside the call, coefficient gradients: the headline shape, raw Q and K
    cfg = wl.CONFIGS[1]
    t = make_device_inputs(cfg, torch, 1)[0]
    t["Q"] = (t["Q"] * 3.0).contiguous()
    t["K"] = (t["K"] * 0.25).contiguous()
    dt = la.LA_F32
    args6 = (cfg.B, cfg.H, cfg.N, cfg.D, dt, cfg.causal)
    wsf = torch.empty(la.la_workspace_bytes(*args6, 0), dtype=torch.uint8, device="cuda")
    wsb = torch.empty(la.la_workspace_bytes(*args6, 3), dtype=torch.uint8, device="cuda")

    def qknorm_step():
        la.la_forward_qknorm(t["Q"], t["K"], t["V"], t["O"], t["G"], cfg.a, cfg.b, cfg.causal, wsf)
        la.la_backward_qknorm(t["Q"], t["K"], t["V"], t["O"], t["G"], t["dO"], t["dQ"], t["dK"],
                              t["dV"], cfg.a, cfg.b, cfg.causal, wsb)
    res["qknorm_fwd_bwd_" + cfg.name] = {"ms_per_step": timed(qknorm_step, 30)}
    nsv = la.la_saved_state_bytes(*args6)
    sv = torch.empty(max(256, nsv), dtype=torch.uint8, device="cuda") if nsv else None

    def qknorm_saved_step():
        la.la_forward_qknorm_save(t["Q"], t["K"], t["V"], t["O"], t["G"], cfg.a, cfg.b, cfg.causal,
                                  wsf, sv)
        la.la_backward_qknorm_saved(t["Q"], t["K"], t["V"], t["O"], t["G"], t["dO"], t["dQ"],
                                    t["dK"], t["dV"], cfg.a, cfg.b, cfg.causal, wsb, sv)
    res["qknorm_save_fwd_bwd_" + cfg.name] = {"ms_per_step": timed(qknorm_saved_step, 30)}
    dab = torch.zeros(2, device="cuda")
    res["backward_ab_" + cfg.name] = {"ms": timed(
        lambda: la.la_backward_ab(t["Q"], t["K"], t["V"], t["O"], t["G"], t["dO"], dab, cfg.a,
                                  cfg.b, cfg.causal, wsb), 30)}
    del t, wsf, wsb
    torch.cuda.empty_cache()
    # the same with bf16 tensors (fp32 tiles on chip): the shape that stands in for an LLM layer
    cfg4 = wl.CONFIGS[3]
    t = make_device_inputs(cfg4, torch, 1)[0]
    t["Q"] = (t["Q"] * 3.0).contiguous()
    t["K"] = (t["K"] * 0.25).contiguous()
    b6 = (cfg4.B, cfg4.H, cfg4.N, cfg4.D, la.LA_BF16, cfg4.causal)
    wsf = torch.empty(la.la_workspace_bytes(*b6, 0), dtype=torch.uint8, device="cuda")
    wsb = torch.empty(la.la_workspace_bytes(*b6, 1), dtype=torch.uint8, device="cuda")

    def qknorm_step_bf16():
        la.la_forward_qknorm(t["Q"], t["K"], t["V"], t["O"], t["G"], cfg4.a, cfg4.b, cfg4.causal,
                             wsf)
        la.la_backward_qknorm(t["Q"], t["K"], t["V"], t["O"], t["G"], t["dO"], t["dQ"], t["dK"],
                              t["dV"], cfg4.a, cfg4.b, cfg4.causal, wsb)
    res["qknorm_fwd_bwd_" + cfg4.name] = {"ms_per_step": timed(qknorm_step_bf16, 30)}
    nsv = la.la_saved_state_bytes(*b6)
    sv = torch.empty(max(256, nsv), dtype=torch.uint8, device="cuda") if nsv else None

    def qknorm_saved_step_bf16():
        la.la_forward_qknorm_save(t["Q"], t["K"], t["V"], t["O"], t["G"], cfg4.a, cfg4.b,
                                  cfg4.causal, wsf, sv)
        la.la_backward_qknorm_saved(t["Q"], t["K"], t["V"], t["O"], t["G"], t["dO"], t["dQ"],
                                    t["dK"], t["dV"], cfg4.a, cfg4.b, cfg4.causal, wsb, sv)
    res["qknorm_save_fwd_bwd_" + cfg4.name] = {"ms_per_step": timed(qknorm_saved_step_bf16, 30)}
    del t, wsf, wsb
    torch.cuda.empty_cache()
    # head size 256: the top of the paper's head-size sweep, and the same shape in bf16
    c32 = wl.find_workload("paper_causal_f32_B4_H16_N4096_D256")
    c16 = wl.Config("causal_bf16_B4_H16_N4096_D256", c32.B, c32.H, c32.N, c32.D, True, "bf16")
    for c in (c32, c16):
        t = make_device_inputs(c, torch, 1)[0]
        a6 = (c.B, c.H, c.N, c.D, la.LA_F32 if c.dtype == "f32" else la.LA_BF16, c.causal)
        wsf = torch.empty(la.la_workspace_bytes(*a6, 0), dtype=torch.uint8, device="cuda")
        wsb = torch.empty(la.la_workspace_bytes(*a6, 1), dtype=torch.uint8, device="cuda")
        fwd = timed(lambda: la.la_forward(t["Q"], t["K"], t["V"], t["O"], t["G"], c.a, c.b,
                                          c.causal, wsf), 5, 2)
        bwd = timed(lambda: la.la_backward(t["Q"], t["K"], t["V"], t["O"], t["G"], t["dO"],
                                           t["dQ"], t["dK"], t["dV"], c.a, c.b, c.causal, wsb),
                    5, 2)
        res[c.name] = {"forward_ms": fwd, "backward_ms": bwd}
        del t, wsf, wsb
        torch.cuda.empty_cache()
    return res


def source_digest():
    """sha256 over the HIP sources: profiles/traffic.json records the digest of the sources
    its counters were collected with, so that stale counters are not quoted."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2510_21956_amd", "csrc", "*"))):
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()


def algorithmic_bytes(D, e, causal):
    """Algorithmic HBM bytes per token-head of each kernel: every operand the kernel needs
    read once, every result written once (G, delta' are one float per token-head).

      with the mask                                      without it (states are global sums)
      fwd_state: K, V in                      2De       the same
      fwd_apply: Q, K, V in; O, G out         4De + 4   Q in; O, G out                 2De + 4
      bwd_state: K, V in                      2De       the same
      bwd_dq   : Q, K, V, O, dO, G in;                  Q, O, dO, G in;
                 dQ, delta' out               6De + 8   dQ, delta' out                 4De + 8
      bwd_dkv  : Q, K, V, dO, G, delta' in;             K, V in; dK, dV out            4De
                 dK, dV out                   6De + 8
      plain-ALU path: generic_bwd_state reads Q, K, V, O, dO, G and writes delta (5De + 8);
      generic_bwd_apply reads Q, K, V, dO, G, delta and writes dQ, dK, dV (7De + 8)."""
    De = D * e
    m = bool(causal)
    return {"fwd_state": 2 * De, "fwd_apply": (4 * De + 4) if m else (2 * De + 4),
            "bwd_state": 2 * De, "bwd_dq": (6 * De + 8) if m else (4 * De + 8),
            "bwd_dkv": (6 * De + 8) if m else 4 * De,
            "generic_fwd_state": 2 * De, "generic_fwd_apply": (4 * De + 4) if m else (2 * De + 4),
            "generic_bwd_state": 5 * De + 8, "generic_bwd_apply": 7 * De + 8}


def measure(cfg, args, steps, warmup, torch, wl, la):
    """Time `steps` steps of one workload and the library's kernels inside a step."""
    B, H, N, D = cfg.B, cfg.H, cfg.N, cfg.D
    e = 4 if cfg.dtype == "f32" else 2
    dt = la.LA_F32 if cfg.dtype == "f32" else la.LA_BF16
    T = cfg.token_heads

    # Rotate through several buffer sets so that a step cannot find its inputs in
    # the 256 MB memory-side cache left there by the previous step.
    set_bytes = 8 * T * D * e + 4 * T
    n_sets = args.buffer_sets or max(2, min(8, int(1.5 * 1024 ** 3 // set_bytes) or 1))
    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()
    sets = make_device_inputs(cfg, torch, n_sets)
    wsf = torch.empty(max(256, la.la_workspace_bytes(B, H, N, D, dt, cfg.causal, 0)),
                      dtype=torch.uint8, device="cuda")
    wsb = torch.empty(max(256, la.la_workspace_bytes(B, H, N, D, dt, cfg.causal, 1)),
                      dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()

    # A step is the pair a training step runs: the forward pass, which also hands its
    # running sums at the segment boundaries to the backward pass (la_forward_save), and
    # the backward pass that starts from them (la_backward_saved).  --independent times
    # la_forward + la_backward instead, where the backward pass recomputes those sums.
    nsv = la.la_saved_state_bytes(B, H, N, D, dt, cfg.causal)
    saved = torch.empty(nsv, dtype=torch.uint8, device="cuda") if nsv else None

    def step(t, trf=None, trb=None):
        if args.forward_only:
            la.la_forward_traced(t["Q"], t["K"], t["V"], t["O"], t["G"], cfg.a, cfg.b,
                                 cfg.causal, wsf, None, trf)
        elif args.independent:
            la.la_forward_traced(t["Q"], t["K"], t["V"], t["O"], t["G"], cfg.a, cfg.b,
                                 cfg.causal, wsf, None, trf)
            la.la_backward_traced(t["Q"], t["K"], t["V"], t["O"], t["G"], t["dO"], t["dQ"],
                                  t["dK"], t["dV"], cfg.a, cfg.b, cfg.causal, wsb, None, trb)
        else:
            la.la_forward_save(t["Q"], t["K"], t["V"], t["O"], t["G"], cfg.a, cfg.b, cfg.causal,
                               wsf, saved, None, trf)
            la.la_backward_saved(t["Q"], t["K"], t["V"], t["O"], t["G"], t["dO"], t["dQ"],
                                 t["dK"], t["dV"], cfg.a, cfg.b, cfg.causal, wsb, saved, None,
                                 trb)

    # event handles for the per-kernel durations measured after the timed loops
    reps = max(5, min(steps, 50))
    traces = []
    for i in range(reps):
        evf, evb = HipEvents(la.LA_MAX_TRACE + 1), HipEvents(la.LA_MAX_TRACE + 1)
        trf, trb = la.la_trace(), la.la_trace()
        trf.events = ctypes.cast(evf.handles, ctypes.POINTER(ctypes.c_void_p))
        trb.events = ctypes.cast(evb.handles, ctypes.POINTER(ctypes.c_void_p))
        trf.capacity = trb.capacity = la.LA_MAX_TRACE + 1
        traces.append((trf, evf, trb, evb))

    def timed(n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            step(sets[i % n_sets])
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    for i in range(warmup):
        step(sets[i % n_sets])
    first_elapsed = timed(steps)  # the steps straight after the warm-up steps
    # On this chip the step time keeps falling for the first hundred or so steps of a run
    # (0.40 -> 0.33 ms on the headline configuration over 35 ms of continuous work; neither
    # copies nor library matrix products run beforehand change that, the path's own kernels
    # do), so a run of a few dozen steps measures the ramp and not the rate a job runs at.
    # The reported rate is therefore taken after the device has run the same steps for a
    # fixed time; the rate of the first steps is reported next to it.
    elapsed = first_elapsed
    if args.clock_warmup_ms > 0:
        t_end = time.perf_counter() + args.clock_warmup_ms * 1e-3
        while time.perf_counter() < t_end:
            for i in range(10):
                step(sets[i % n_sets])
            torch.cuda.synchronize()
        elapsed = timed(steps)
    ms_per_step = elapsed * 1e3 / steps
    peak_bytes = torch.cuda.max_memory_allocated()

    # Per-kernel durations: the same steps again, back to back and straight after the timed
    # loop (so at the same clocks), with the library recording HIP events between its kernels
    # on the stream it launches on.  Every repetition has event handles of its own (created
    # before the timed loops: the device must not sit idle in between); nothing waits until
    # all of them are enqueued.
    for i, (trf, evf, trb, evb) in enumerate(traces):
        step(sets[i % n_sets], trf, trb)
    torch.cuda.synchronize()
    ksum, kcount = {}, {}
    for trf, evf, trb, evb in traces:
        for tr, ev, tag in ((trf, evf, "fwd"), (trb, evb, "bwd")):
            for k in range(tr.recorded - 1):
                name = tag + ":" + tr.names[k].decode()
                ksum[name] = ksum.get(name, 0.0) + ev.elapsed_ms(k, k + 1)
                kcount[name] = kcount.get(name, 0) + 1
        evf.destroy()
        evb.destroy()
    kernels_ms = {k: ksum[k] / kcount[k] for k in ksum}

    # Roofline of the dominant kernel (the one with the longest average duration).
    alg_bytes = algorithmic_bytes(D, e, cfg.causal)
    dom = max(kernels_ms, key=kernels_ms.get)
    dom_key = dom.split(":")[1] if dom.split(":")[1] in alg_bytes else None
    dom_ms = kernels_ms[dom]
    # every input once, every output once: forward + backward, or the forward pass alone
    pass_bytes = ((4 * D * e + 4) if args.forward_only else (12 * D * e + 8)) * T
    pass_gbs = pass_bytes / (ms_per_step * 1e-3) / 1e9
    roofline = None
    if dom_key:
        achieved = alg_bytes[dom_key] * T / (dom_ms * 1e-3) / 1e9
        traffic, traffic_note = None, "no counter record for this workload"
        tpath = os.path.join(ROOT, "profiles", "traffic.json")
        if os.path.exists(tpath):
            # HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE,
            # scaled by a copy kernel of known size (see profiles/); quoted only while the
            # kernels are still the ones the counters were collected with
            tj = json.load(open(tpath))
            rec = tj.get(cfg.name, {}).get(dom.split(":")[1])
            if rec and tj.get("source_sha256") != source_digest():
                traffic_note = "profiles/traffic.json predates the current kernels: not quoted"
            elif rec:
                traffic = rec["fetch_bytes"] + rec["write_bytes"]
                traffic_note = "rocprofv3 FETCH_SIZE + WRITE_SIZE per launch (profiles/)"
                # a kernel cannot move less than its operands: if this fails, the table of
                # algorithmic bytes above credits the kernel with operands it does not touch
                assert alg_bytes[dom_key] * T <= 1.05 * traffic, (dom, alg_bytes[dom_key] * T,
                                                                    traffic)
        roofline = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                    "traffic_note": traffic_note,
                    "kernel_ms": dom_ms, "algorithmic_bytes_per_launch": alg_bytes[dom_key] * T,
                    "whole_pass_frac": pass_gbs / HBM_PEAK_GBS}
    # Algorithmic matrix flops of the recurrences per token-head (Sec. 3.1 / 3.2): forward
    # 4 D^2 (update S, read it out), backward 10 D^2 (rebuild S, S OmegaHat, update R, R v,
    # R^T k); without the mask the sums are formed once per slice and the rebuild is free.
    # The chunked kernels execute more (the chunk's own C x C blocks, the per-segment sums).
    pass_flops = (4 if args.forward_only else (14 if cfg.causal else 12)) * D * D * T
    pass_tflops = pass_flops / (ms_per_step * 1e-3) / 1e12
    mfma_peak = 157.3 if cfg.dtype == "f32" else 2516.0  # TFLOP/s, dense, datasheet

    out = {
        "metric": "fwd tokens/s" if args.forward_only else "fwd+bwd tokens/s",
        "value": cfg.tokens / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if cfg.dtype == "f32" else "bf16 I/O, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": cfg.name, "B": B, "H": H, "N": N, "D": D, "causal": cfg.causal,
                   "a": cfg.a, "b": cfg.b, "buffer_sets": n_sets, "seg_len_override": args.seg_len,
                   "clock_warmup_ms": args.clock_warmup_ms,
                   "entry_points": "la_forward + la_backward" if args.independent
                   else "la_forward_save + la_backward_saved"},
        "token_heads_per_s": T / (ms_per_step * 1e-3),
        # the same number of steps timed straight after the warm-up steps, before the device
        # had run for --clock-warmup-ms (see measure())
        "first_steps": {"ms_per_step": first_elapsed * 1e3 / steps,
                        "value": cfg.tokens / (first_elapsed / steps)},
        "whole_pass": {"compulsory_bytes": pass_bytes, "achieved_GBs": pass_gbs,
                       "frac_of_hbm_peak": pass_gbs / HBM_PEAK_GBS,
                       "algorithmic_flops": pass_flops, "achieved_TFLOPs": pass_tflops,
                       "mfma_peak_TFLOPs": mfma_peak, "frac_of_mfma_peak": pass_tflops / mfma_peak},
        "kernels_ms": kernels_ms,
        # the two passes separately: sums of the traced kernel intervals
        "forward_ms_traced": sum(v for k, v in kernels_ms.items() if k.startswith("fwd:")),
        "backward_ms_traced": sum(v for k, v in kernels_ms.items() if k.startswith("bwd:")),
        "peak_allocated_device_bytes": int(peak_bytes),
        "workspace_bytes": {"forward": wsf.numel(), "backward": wsb.numel(), "saved": nsv},
        "roofline": roofline,
    }
    del sets, wsf, wsb, saved
    torch.cuda.empty_cache()
    return out


if __name__ == "__main__":
    main()
