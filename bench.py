"""Benchmark of the LF-MMI hot path on one MI355X.

A step is one lfmmi_loss_grad call (device lengths only) on configuration 5 (the largest workload:
the 6000-state / ~60k-arc Zipf denominator graph shared by B=128 utterances,
128 packed numerator chains, D=3000, N_b = round(3.6 L_b) frames): numerator
and denominator alpha and beta recursions, log Z, state and pdf posteriors,
objective and gradient.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line: throughput in log-semiring arc-updates/s
(2 * sum_b N_b * E_b, real frames, denominator + numerator arcs), ms per batch,
the memory roofline of the dominant kernel (the denominator recursion launch,
timed live with HIP events on the launching stream) and the fp64 CPU oracle
timed on this machine's host cores on a bounded sample of the same workload.
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

HBM_PEAK_GBS = 8000.0        # MI355X published HBM3E bandwidth

# LDS gather rate: 256 CUs x 128 bytes per clock x 2.4 GHz
LDS_PEAK_GBS = 256 * 128 * 2.4
# HBM bytes per denominator-recursion launch on configuration 5 from rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, each
# scaled by what the same counter reads for a plain copy of known size): written by
# `python -m paper_2112_00709_amd.traffic_summary`, which names the kernel the figures belong to.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "lfmmi_config5_traffic.json")
DOMINANT_KERNEL = "fb_linear_kernel"


def measured_traffic(kernel: str):
    """Bytes per launch from the committed counter summary; None when it is missing or names another kernel."""
    try:
        with open(TRAFFIC_FILE) as f:
            t = json.load(f)
    except (OSError, ValueError):
        return None
    if kernel not in t.get("kernel", ""):
        return None
    return float(t["traffic_bytes_per_launch"])


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def context_workloads(fb, wl, torch, everything=True):
    """fb_alpha + fb_beta + fb_posteriors (three calls, vectors through HBM) on the other workloads."""
    out = {}
    side = torch.cuda.Stream()   # one for all workloads: the box has few hardware queues to map streams onto
    makers = (("config1", wl.config1), ("config2", wl.config2), ("config3", wl.config3),
              ("config4", wl.config4), ("paper_shape_den", wl.paper_shape_den))
    if not everything:
        makers = makers[3:]
    for name, make in makers:
        w = make()
        g = w.num if w.den is None else w.den
        t0 = time.time()
        G = fb.graph_from(g, w.D)
        create_s = time.time() - t0
        emis = torch.from_numpy(w.emis).cuda()
        lengths = torch.from_numpy(w.lengths).cuda()

        def run():   # the two recursions are independent: one on a second stream, as a caller would run them
            main = torch.cuda.current_stream()
            side.wait_stream(main)
            a, _, _ = fb.fb_alpha(G, emis, lengths)
            with torch.cuda.stream(side):
                b_, _, _ = fb.fb_beta(G, emis, lengths)
            main.wait_stream(side)
            b_.record_stream(main)
            fb.fb_posteriors(G, a, b_, lengths, w.B, w.N, want_state=False)

        for _ in range(2):
            run()
        torch.cuda.synchronize()
        n = 5
        t0 = time.perf_counter()
        for _ in range(n):
            run()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / n
        upd = w.arc_updates(g)
        frames = int(w.lengths.sum())
        if g.packed:
            k_frames = int(np.sum(w.lengths.astype(np.int64) * np.diff(g.state_off)))   # sum_b N_b K_b
            d_frames = k_frames                                                            # at most one pdf per state
        else:
            k_frames, d_frames = frames * g.K, frames * int(np.unique(g.pdf).size)
        # compulsory bytes: alpha and beta each read the used emissions and write the vector; the posteriors
        # read both vectors and write one pdf row per frame
        algo = 2 * (4 * d_frames + 4 * k_frames) + 8 * k_frames + 4 * frames * w.D
        out[name] = {"B": w.B, "N_max": w.N, "K": g.K, "E": g.E, "D": w.D, "ms": ms, "arc_updates": upd,
                     "arc_updates_per_s": upd / (ms * 1e-3), "algorithmic_bytes": algo,
                     "hbm_frac": algo / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "graph_create_s": create_s}
        if name == "paper_shape_den":   # Table 1: 1.04 s for the denominator forward-backward on an RTX 2080 Ti
            out[name]["paper_table1_s"] = 1.04
        log(f"[bench] {name}: {ms:.3f} ms, {upd / (ms * 1e-3):.3e} arc-updates/s, HBM fraction {out[name]['hbm_frac']:.3f}")
        if name in ("config4", "paper_shape_den"):
            # comparison mode beside the exact path (Table 1's leaky-HMM rows): log Z and pdf posteriors of the
            # leaky-HMM of the same graph in one call, a plain kernel (one workgroup per sequence, both sweeps)
            lws = torch.empty((fb.fb_leaky_workspace_bytes(G, w.B, w.N),), dtype=torch.uint8, device="cuda")
            fb.fb_leaky_posteriors(G, emis, lengths, 1e-5, ws=lws)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(3):
                fb.fb_leaky_posteriors(G, emis, lengths, 1e-5, ws=lws)
            torch.cuda.synchronize()
            out[name]["leaky_hmm_ms"] = (time.perf_counter() - t0) * 1e3 / 3
            out[name]["leaky_hmm_leak"] = 1e-5
            log(f"[bench] {name}: leaky-HMM comparison mode {out[name]['leaky_hmm_ms']:.3f} ms")
            del lws
        G.destroy()
        if everything and name in ("config4", "paper_shape_den"):   # best path (tropical semiring) on the same inputs
            Gv = fb.graph_from(g, w.D)
            for _ in range(2):
                fb.fb_viterbi(Gv, emis, lengths)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(n):
                fb.fb_viterbi(Gv, emis, lengths)
            torch.cuda.synchronize()
            vms = (time.perf_counter() - t0) * 1e3 / n
            valgo = 4 * d_frames + 2 * k_frames + 4 * frames     # used emissions read, back-pointers written, path written
            out[name + "_viterbi"] = {"ms": vms, "arc_updates": upd // 2, "arc_updates_per_s": upd / 2 / (vms * 1e-3),
                                      "algorithmic_bytes": valgo, "hbm_frac": valgo / (vms * 1e-3) / 1e9 / HBM_PEAK_GBS}
            log(f"[bench] {name} best path: {vms:.3f} ms, {upd / 2 / (vms * 1e-3):.3e} arc-updates/s")
            Gv.destroy()
        del emis
    return out


def paper_lfmmi_workload(fb, wl, torch):
    """LF-MMI loss + gradient with both graphs the size of the paper's (Table 3 gives 0.220 s for this stage on an
    RTX 2080 Ti), both entry points.  Runs in the main process: the call uses the library's own streams, which
    should not have to share the hardware queues with further streams of the caller's."""
    out = {}
    w = wl.paper_shape_lfmmi()
    den, num = fb.graph_from(w.den, w.D), fb.graph_from(w.num, w.D)
    emis, lengths = torch.from_numpy(w.emis).cuda(), torch.from_numpy(w.lengths).cuda()
    ws = torch.empty((fb.fb_lfmmi_workspace_bytes(den, num, w.B, w.N, w.D),), dtype=torch.uint8, device="cuda")
    grad = torch.empty((w.B, w.N, w.D), dtype=torch.float32, device="cuda")

    def timed(host_lengths):
        for _ in range(2):
            fb.lfmmi_loss_grad(den, num, emis, lengths, ws=ws, grad=grad, lengths_host=host_lengths)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            fb.lfmmi_loss_grad(den, num, emis, lengths, ws=ws, grad=grad, lengths_host=host_lengths)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / 5

    ms = timed(None)
    ms_ragged = timed(w.lengths)
    upd = w.arc_updates(w.den) + w.arc_updates(w.num)
    frames = int(w.lengths.sum())
    d_used = int(np.unique(w.den.pdf).size)
    fused = frames * (8 * w.den.K + 8 * d_used + 4 * w.D)   # the fully fused model of the main line (whole_step_hbm)
    out["paper_shape_lfmmi"] = {"B": w.B, "N_max": w.N, "D": w.D, "den_states": w.den.K, "den_arcs": w.den.E,
                                "num_states": w.num.K, "num_arcs": w.num.E, "ms": ms,
                                "lfmmi_loss_grad_ms": ms, "lfmmi_loss_grad_ragged_ms": ms_ragged, "arc_updates": upd,
                                "arc_updates_per_s": upd / (ms * 1e-3), "algorithmic_bytes": fused,
                                "hbm_frac": fused / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "paper_table3_s": 0.220}
    log(f"[bench] paper_shape_lfmmi: {ms:.3f} ms, {upd / (ms * 1e-3):.3e} arc-updates/s")
    den.destroy(); num.destroy()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, choices=[5], help="workload (configuration 5 is the benchmark)")
    ap.add_argument("--cpu-sample", type=int, default=0, help="sequences the CPU oracle is timed on (0 = 2 per thread)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--context", action="store_true",
                    help="time every other workload (configurations 1-4, the paper-shaped denominator and LF-MMI, the best "
                         "path) for other_workloads; without it: configuration 4 and the two paper-shaped ones")
    ap.add_argument("--no-context", action="store_true", help="leave other_workloads out")
    ap.add_argument("--context-only", choices=["all", "main"], default=None, help=argparse.SUPPRESS)   # the child process
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (sequences are independent, so the batch would be "
              "split across GPUs with one 8-byte all-reduce of the loss; no multi-GPU path is built).", file=sys.stderr)
        return 2

    import torch

    import paper_2112_00709_amd as fb
    import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    fb.lib()
    torch.cuda.set_device(0)
    if args.context_only:
        print(json.dumps(context_workloads(fb, wl, torch, everything=args.context_only == "all")), flush=True)
        return 0

    t_gen = time.time()
    w = wl.config5()
    log(f"[bench] config5 generated in {time.time() - t_gen:.1f}s: B={w.B} N={w.N} D={w.D} "
        f"den K={w.den.K} E={w.den.E}; num K={w.num.K} E={w.num.E}; frames={int(w.lengths.sum())}")
    t0 = time.time()
    den, num = fb.graph_from(w.den, w.D), fb.graph_from(w.num, w.D)
    graph_create_s = time.time() - t0
    log(f"[bench] graph layout + schedules + upload: {graph_create_s:.3f}s (not part of a step)")
    emis = torch.from_numpy(w.emis).cuda()
    lengths = torch.from_numpy(w.lengths).cuda()
    ws = torch.empty((fb.fb_lfmmi_workspace_bytes(den, num, w.B, w.N, w.D),), dtype=torch.uint8, device="cuda")
    grad = torch.empty((w.B, w.N, w.D), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()

    def step():   # the call the benchmark is about: lengths on the device only
        return fb.lfmmi_loss_grad(den, num, emis, lengths, ws=ws, grad=grad)

    def step_ragged():   # its sibling for callers who have the lengths on the host
        return fb.lfmmi_loss_grad(den, num, emis, lengths, ws=ws, grad=grad, lengths_host=w.lengths)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        out = step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    loss = float(out[0].item())
    # the same step timed one at a time (events on the launching stream): median and minimum
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for e0, e1 in evs:
        e0.record(); step(); e1.record()
    torch.cuda.synchronize()
    single = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    for _ in range(args.warmup):
        step_ragged()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step_ragged()
    torch.cuda.synchronize()
    ms_ragged = (time.perf_counter() - t0) * 1e3 / args.steps

    # stage times with HIP events recorded by the library on the launching stream
    fb.fb_profile_enable(True)
    stages = []
    for _ in range(max(3, min(args.steps, 10))):
        step()
        stages.append(fb.fb_profile_read())
    fb.fb_profile_enable(False)
    stage_ms = {k: float(np.mean([s[k] for s in stages])) for k in stages[0]}

    upd_den, upd_num = w.arc_updates(w.den), w.arc_updates(w.num)
    arc_updates = upd_den + upd_num
    frames = int(w.lengths.sum())
    d_used = int(np.unique(w.den.pdf).size)
    # algorithmic bytes of the denominator recursion launch: per real frame and direction,
    # the emission entries the graph uses are read once and the state vector is written once
    algo_bytes = frames * 2 * (4 * d_used + 4 * w.den.K)
    achieved = algo_bytes / (stage_ms["den_recursion"] * 1e-3) / 1e9
    traffic = measured_traffic(DOMINANT_KERNEL)
    plan_arcs = int(np.unique(w.den.src.astype(np.int64) * w.den.K + w.den.dst).size)
    upd_plan = 2 * frames * plan_arcs + upd_num   # arcs the plans walk: parallel arcs (same source and destination) are merged
    result = {
        "metric": "log-semiring arc-updates/sec (B*N*E*2) + LF-MMI loss+grad ms/batch",
        "value": arc_updates / (ms_per_step * 1e-3),
        "unit": "arc-updates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "config5: LF-MMI loss+grad, Zipf denominator K=6000 E~60k shared by B=128, "
                               "128 packed numerator chains, D=3000, N_b=round(3.6 L_b)",
                   "B": w.B, "N_max": w.N, "frames": frames, "D": w.D,
                   "den_states": w.den.K, "den_arcs": w.den.E, "num_states": w.num.K, "num_arcs": w.num.E,
                   "den_plan_arcs": plan_arcs, "entry_point": "lfmmi_loss_grad"},
        "lfmmi_ms_per_batch": ms_per_step,
        "lfmmi_loss_grad_ms": ms_per_step, "lfmmi_loss_grad_ragged_ms": ms_ragged,
        "value_on_plan_arcs": upd_plan / (ms_per_step * 1e-3),
        "ms_per_step_median": single[len(single) // 2], "ms_per_step_min": single[0],
        "graph_create_s": graph_create_s,
        "arc_updates_per_step": arc_updates,
        "arc_updates_padded": 2 * w.B * w.N * w.den.E,
        "stage_ms": stage_ms,
        "loss": loss,
        # the denominator recursion of a step is one launch of this kernel (alpha and beta of every sequence, 2 B
        # workgroups in order of length); den_recursion brackets it with events on the launching stream
        "roofline": {"kernel": DOMINANT_KERNEL + " (denominator alpha+beta, one launch)",
                     "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "algorithmic_bytes": algo_bytes, "launch_ms": stage_ms["den_recursion"]},
        # what holds that launch back: every arc-update is one 4-byte gather from the state vector in LDS (plus the
        # bank conflicts of 64 lanes reading 64 scattered words); the rate below counts the walked arcs only
        "roofline_lds": {"bound": "lds", "achieved": 4 * 2 * frames * plan_arcs / (stage_ms["den_recursion"] * 1e-3) / 1e9,
                         "peak": LDS_PEAK_GBS, "unit": "GB/s gathered (4 bytes per walked arc)",
                         "frac": 4 * 2 * frames * plan_arcs / (stage_ms["den_recursion"] * 1e-3) / 1e9 / LDS_PEAK_GBS},
    }

    # the rate a plain device copy reaches on this machine (1 GiB read + 1 GiB written per copy), beside the published peak
    src = torch.empty((1 << 28,), dtype=torch.float32, device="cuda").fill_(1.0)
    dst = torch.empty_like(src)
    dst.copy_(src)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(5):
        dst.copy_(src)
    c1.record()
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * src.numel() * 4 / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del src, dst
    result["roofline"]["copy_gbs"] = copy_gbs
    result["roofline"]["frac_of_copy"] = achieved / copy_gbs
    # the whole step against the bytes a fully fused loss+gradient would move per real frame (emission entries read
    # by both directions, alpha written and read once, gradient written): 8K + 8D' + 4D
    fused_bytes = frames * (8 * w.den.K + 8 * d_used + 4 * w.D)
    result["whole_step_hbm"] = {"model_bytes": fused_bytes, "achieved": fused_bytes / (ms_per_step * 1e-3) / 1e9,
                                "unit": "GB/s", "frac": fused_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS}

    if not args.no_context:
        # In a process of its own: these workloads run fb_alpha and fb_beta on two streams of the caller's, and a
        # process has only four hardware queues for all its streams (the LF-MMI calls use three of the library's).
        import subprocess
        child = subprocess.run([sys.executable, os.path.abspath(__file__), "--context-only", "all" if args.context else "main"],
                               stdout=subprocess.PIPE, check=True, text=True)
        result["other_workloads"] = json.loads(child.stdout.strip().splitlines()[-1])
        den.destroy(); num.destroy()
        del emis, ws, grad
        den = num = None
        result["other_workloads"].update(paper_lfmmi_workload(fb, wl, torch))

    if args.calibrate_copy:
        src = torch.empty((1 << 28,), dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)            # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    if not args.no_cpu_baseline:
        import oracle
        threads = oracle.num_threads()
        ns = args.cpu_sample or min(w.B, 4 * threads)
        order = np.argsort(w.lengths, kind="stable")
        sel = np.sort(order[np.linspace(0, w.B - 1, ns).round().astype(int)])
        sample_updates = int(2 * np.sum(w.lengths[sel].astype(np.int64) * (w.den.E + w.num.arcs_per_seq(w.B)[sel])))
        t0 = time.perf_counter()
        oracle.lfmmi(w.den, w.num, w.emis, w.lengths, sel=sel)
        dt = time.perf_counter() - t0
        # one utterance of median length on one thread (the single-thread reference figure)
        mid = np.array([int(order[w.B // 2])])
        mid_updates = int(2 * w.lengths[mid[0]] * (w.den.E + w.num.arcs_per_seq(w.B)[mid[0]]))
        oracle.set_num_threads(1)
        t1 = time.perf_counter()
        oracle.lfmmi(w.den, w.num, w.emis, w.lengths, sel=mid)
        dt1 = time.perf_counter() - t1
        oracle.set_num_threads(threads)
        result["cpu_baseline"] = {
            "value": sample_updates / dt, "unit": "arc-updates/s", "cores": int(min(threads, ns)), "kind": "oracle",
            "sample": f"{ns} of {w.B} utterances of config5 spread over the length range "
                      f"({sample_updates} arc-updates, {dt:.1f} s, fp64, OpenMP over utterances)",
            "single_thread_value": mid_updates / dt1,
            "single_thread_sample": f"the utterance of median length ({mid_updates} arc-updates, {dt1:.1f} s)"}
    print(json.dumps(result), flush=True)
    if den is not None:
        den.destroy(); num.destroy()
    return 0


if __name__ == "__main__":
    sys.exit(main())
