#!/usr/bin/env python3
"""Benchmark of the MOM prefill hot path on one MI355X.

One "step" is one pass of the whole mini-sequence MLP (every mini-sequence: gate/up GEMM with
the SiLU*up epilogue, then the down GEMM) over one synthetic Llama-3-8B-shaped layer input
(S=32768, H=4096, I=14336, mini_seq=4096, bf16) that is already resident in HBM.  Prints ONE
JSON line: whole-job TFLOP/s (6*S*H*I flop per step), the roofline of the dominant kernel
measured with HIP events on the launch stream, the CPU oracle timed on a bounded row sample, and
(outside the timed region) the side measurements of the path: what the matrix cores of this
machine sustain on the workload's own operands, socket power and clock under the kernels, the
mini_seq sweep, measured peak device memory with and without mini-sequences, the one-token
kernels against HBM bandwidth and the KV offload overlap.
"""
import argparse
import json
import os
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2500.0      # MI355X dense bf16 matrix peak (published figure)
HBM_PEAK_GBPS = 8000.0
# Bytes between the L2s and the memory fabric per launch of the gate/up kernel (rocprofv3 FETCH_SIZE + WRITE_SIZE,
# each scaled by what the same counter reads for a 1 GiB copy kernel: x 2.000 and x 1.000; the summary with the
# commands is profiles/gemm_kernels_llama3_8b_32k_counters.txt).  Not measured live: the figure is a property of
# the tiling (every operand panel once per block of 32 resident tiles per L2), not of the machine's clock.
GATEUP_TRAFFIC_BYTES = {("llama3_8b_32k", 4096): 1.527e9, ("llama3_8b_128k", 8192): 3.054e9,
                        ("qwen25_7b_256k", 8192): 3.599e9, ("mistral_7b_448k", 16384): 6.108e9}


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=20)
    p.add_argument("--warmup", type=int, default=3)
    p.add_argument("--workload", default="llama3_8b_32k")
    p.add_argument("--mini-seq", type=int, default=None, help="override the workload's mini_seq")
    p.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample; 0 skips")
    p.add_argument("--no-side", action="store_true", help="skip the side measurements (profiling runs)")
    p.add_argument("--calib", action="store_true",
                   help="also run a plain 1 GiB elementwise copy kernel (known HBM bytes) to scale profiler counters")
    p.add_argument("--extras", action="store_true",
                   help="also time the two-stream driver over the sweep and a six-layer offload schedule")
    return p.parse_args()


def device_info(torch, dev):
    """What the box reports, beside the published peak the roofline divides by: 256 CUs x 4 SIMDs x 1024 bf16
    flop per clock at the 2.4 GHz peak engine clock = 2.5 PFLOP/s."""
    p = torch.cuda.get_device_properties(dev)
    cus = int(p.multi_processor_count)
    return {"name": p.name, "arch": getattr(p, "gcnArchName", ""), "compute_units": cus,
            "bf16_mfma_peak_at_2400_mhz_tflops": round(cus * 4 * 1024 * 2.4e9 / 1e12, 1)}


def time_mlp(binding, torch, tensors, C, out, ws, steps, warmup):
    x, wg, wu, wd = tensors
    st = torch.cuda.current_stream()
    for _ in range(warmup):
        binding.mom_mlp_prefill(x, wg, wu, wd, C, out, ws, stream=st)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        binding.mom_mlp_prefill(x, wg, wu, wd, C, out, ws, stream=st)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def kernel_times(binding, torch, tensors, C, out, ws, S, reps):
    """Average duration (s) of the gate/up and the down kernel, from HIP events recorded on the
    launch stream around every kernel of `reps` whole passes."""
    x, wg, wu, wd = tensors
    st = torch.cuda.current_stream()
    n = -(-S // C)
    gu, dn = [], []
    for _ in range(reps):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(1 + 2 * n)]
        for e in evs:
            e.record(st)
        binding.mom_mlp_prefill_events(x, wg, wu, wd, C, out, ws, evs, stream=st)
        torch.cuda.synchronize()
        for c in range(n):
            gu.append(evs[2 * c].elapsed_time(evs[2 * c + 1]) * 1e-3)
            dn.append(evs[2 * c + 1].elapsed_time(evs[2 * c + 2]) * 1e-3)
    return sum(gu) / len(gu), sum(dn) / len(dn)


def event_time(torch, fn, reps, warmup=2):
    """Seconds per call of fn() (which enqueues on the current stream), from one pair of HIP events."""
    st = torch.cuda.current_stream()
    for _ in range(warmup):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(st)
    for _ in range(reps):
        fn()
    e1.record(st)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / reps


# ------------------------------------------------------------------ side measurements

def mfma_probe(binding, torch, tensors, dev):
    """What the matrix cores sustain on this machine: the library's register-only MFMA loop (one wavefront per
    SIMD on every CU, no LDS or memory traffic) on operand fragments taken from the workload's own W_gate and x,
    and on constant operands.  With real operands the chip runs into its power limit and lowers its clock; the
    rate left is the ceiling of any kernel made of this instruction on this data and this machine."""
    x, wg, _, _ = tensors
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    sink = torch.empty(cus * 256, dtype=torch.float32, device=dev)
    ones = torch.ones(4096, dtype=torch.bfloat16, device=dev)
    res = {}
    for name, a, b, order in (("workload_operands", wg, x, 0), ("workload_operands_k_half_by_k_half", wg, x, 1),
                              ("constant_operands", ones, ones, 0)):
        iters = 30000                                      # ~35 ms per launch at 1.9 GHz
        flop = None

        def launch():
            nonlocal flop
            flop = binding.mom_debug_mfma_probe(a, b, iters, cus, sink, order=order)
        t = event_time(torch, launch, reps=8, warmup=3)    # ~0.1 s of warm-up: the clock has settled
        res[name] = round(flop / t / 1e12, 1)
    return res


class PowerSampler:
    """Socket power and shader clock while the kernels run, polled from a host thread (amdsmi if it is
    importable, else the hwmon power sensor alone)."""

    def __init__(self):
        self.samples = []
        self.stop = False
        self.smi = None
        self.handle = None
        self.power_file = None
        self.cap_w = None
        try:
            import amdsmi
            amdsmi.amdsmi_init()
            self.smi = amdsmi
            self.handle = amdsmi.amdsmi_get_processor_handles()[0]
        except Exception:
            self.smi = None
        import glob
        for f in glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input"):
            self.power_file = f
            try:
                self.cap_w = int(open(f.replace("power1_input", "power1_cap")).read()) / 1e6
            except Exception:
                pass
            break

    def read(self):
        power = clock = None
        if self.smi is not None:
            try:
                m = self.smi.amdsmi_get_gpu_metrics_info(self.handle)
                p = m.get("current_socket_power")
                if isinstance(p, (int, float)) and 0 < p < 5000:
                    power = float(p)
                c = m.get("current_gfxclks") or m.get("current_gfxclk")
                if isinstance(c, (list, tuple)):
                    c = [v for v in c if isinstance(v, (int, float)) and 0 < v < 10000]
                    clock = sum(c) / len(c) if c else None
                elif isinstance(c, (int, float)) and 0 < c < 10000:
                    clock = float(c)
            except Exception:
                pass
        if power is None and self.power_file:
            try:
                power = int(open(self.power_file).read()) / 1e6
            except Exception:
                pass
        return power, clock

    def run(self, period=0.02):
        while not self.stop:
            self.samples.append(self.read())
            time.sleep(period)

    def available(self):
        return self.smi is not None or self.power_file is not None


def power_under_load(binding, torch, tensors, C, out, ws, S, H, I, seconds=1.5):
    """Mean socket power and shader clock over a loop of MLP steps (the first 0.4 s are dropped)."""
    ps = PowerSampler()
    if not ps.available():
        return None
    sec = time_mlp(binding, torch, tensors, C, out, ws, 3, 1)
    steps = max(10, int(seconds / sec))
    th = threading.Thread(target=ps.run, daemon=True)
    t0 = time.perf_counter()
    th.start()
    sec = time_mlp(binding, torch, tensors, C, out, ws, steps, 0)
    ps.stop = True
    th.join()
    dt = time.perf_counter() - t0
    keep = ps.samples[int(len(ps.samples) * min(0.5, 0.4 / dt)):]
    pw = [p for p, _ in keep if p is not None]
    ck = [c for _, c in keep if c is not None]
    return {"socket_power_w": round(sum(pw) / len(pw), 1) if pw else None,
            "power_cap_w": ps.cap_w,
            "shader_clock_mhz": round(sum(ck) / len(ck), 1) if ck else None,
            "peak_shader_clock_mhz": 2400, "samples": len(keep), "steps": steps,
            "tflops_meanwhile": round(6.0 * S * H * I / sec / 1e12, 1),
            "source": "amdsmi gpu_metrics" if ck else "hwmon power1_input"}


def mini_seq_sweep(binding, torch, tensors, out, dev, S, H, I, steps):
    """Whole-step rate over mini_seq; 128..512 is the regime of whole-forward chunked prefill (the comparison of
    the paper's Appendix B/C), where the weights are re-read once per 128..512 rows."""
    rows = []
    for C in (128, 256, 512, 1024, 2048, 4096, 8192, 0):
        if C > S:
            continue
        nb = binding.mom_mlp_workspace_bytes(S, H, I, C)
        ws = torch.empty(nb, dtype=torch.uint8, device=dev)
        sec = time_mlp(binding, torch, tensors, C, out, ws, steps, 1)
        rows.append({"mini_seq": C or S, "workspace_bytes": nb, "ms": round(sec * 1e3, 3),
                     "tflops": round(6.0 * S * H * I / sec / 1e12, 1)})
        del ws
    return rows


def peak_memory(binding, torch, tensors, out, dev, S, H, I, C):
    """Measured device memory of the intermediate, mini-sequences against the whole sequence at once: growth of
    torch's allocator peak and drop of the driver's free memory (hipMemGetInfo) from before the workspace is
    allocated until after the call has run."""
    res = {}
    for name, c in (("mini_seq", C), ("unchunked", 0)):
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        torch.cuda.reset_peak_memory_stats()
        base = torch.cuda.memory_allocated()
        free0, _ = torch.cuda.mem_get_info()
        ws = torch.empty(binding.mom_mlp_workspace_bytes(S, H, I, c), dtype=torch.uint8, device=dev)
        binding.mom_mlp_prefill(*tensors, c, out, ws)
        torch.cuda.synchronize()
        free1, _ = torch.cuda.mem_get_info()
        res[name] = {"analytic_workspace_bytes": binding.mom_mlp_workspace_bytes(S, H, I, c),
                     "allocator_peak_growth_bytes": torch.cuda.max_memory_allocated() - base,
                     "device_free_drop_bytes": free0 - free1}
        del ws
    torch.cuda.empty_cache()
    return res


def one_token_kernels(binding, synth, torch, tensors, dev, H, I, V):
    """Last-token branch: LM-head GEMV and the two GEMV passes of the last-token MLP against HBM bandwidth."""
    res = {}
    lm = synth.Workload("lm", S=1, H=H, I=I, mini_seq=0, V=V)
    xl, wlm = synth.lmhead_inputs(lm, device=dev)
    logits = torch.empty((V,), dtype=torch.float32, device=dev)
    t = event_time(torch, lambda: binding.mom_lmhead_last(xl, wlm, logits), reps=20, warmup=3)
    nbytes = V * H * 2 + H * 2 + V * 4
    res["lmhead"] = {"V": V, "H": H, "us": round(t * 1e6, 2), "bytes": nbytes, "GBps": round(nbytes / t / 1e9, 1),
                     "frac_hbm_peak": round(nbytes / t / 1e9 / HBM_PEAK_GBPS, 4)}
    del wlm
    x, wg, wu, wd = tensors
    o1 = torch.empty((H,), dtype=torch.bfloat16, device=dev)
    wsl = torch.empty(I * 2, dtype=torch.uint8, device=dev)
    t = event_time(torch, lambda: binding.mom_mlp_last(x[-1], wg, wu, wd, o1, wsl), reps=20, warmup=3)
    xl1 = x[-1:].contiguous()
    o2 = torch.empty((1, H), dtype=torch.bfloat16, device=dev)
    t2 = event_time(torch, lambda: binding.mom_mlp_prefill(xl1, wg, wu, wd, 0, o2, wsl), reps=10, warmup=2)
    mb = 6.0 * H * I + 4.0 * I + 4.0 * H
    res["last_token_mlp"] = {"H": H, "I": I, "us": round(t * 1e6, 2), "bytes": mb, "GBps": round(mb / t / 1e9, 1),
                             "frac_hbm_peak": round(mb / t / 1e9 / HBM_PEAK_GBPS, 4),
                             "us_through_gemm_kernels_S1": round(t2 * 1e6, 2)}
    both = res["lmhead"]["us"] + res["last_token_mlp"]["us"]
    res["last_token_branch"] = {"us": round(both, 2), "bytes": nbytes + mb,
                                "frac_hbm_peak": round((nbytes + mb) / (both * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)}
    # the whole branch (gate/up GEMV, down GEMV, LM head on the MLP's output) as ONE captured HIP graph
    try:
        wlm = synth.lmhead_inputs(lm, device=dev)[1]
        st = torch.cuda.current_stream()

        def branch():
            binding.mom_mlp_last(x[-1], wg, wu, wd, o1, wsl)
            binding.mom_lmhead_last(o1, wlm, logits)
        side = torch.cuda.Stream()
        side.wait_stream(st)
        with torch.cuda.stream(side):
            branch()
        st.wait_stream(side)
        torch.cuda.synchronize()
        eager = logits.clone()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            branch()
        torch.cuda.synchronize()
        logits.zero_()
        t = event_time(torch, graph.replay, reps=20, warmup=3)
        res["last_token_branch"]["hip_graph_us"] = round(t * 1e6, 2)
        res["last_token_branch"]["hip_graph_frac_hbm_peak"] = round((nbytes + mb) / t / 1e9 / HBM_PEAK_GBPS, 4)
        res["last_token_branch"]["hip_graph_matches_eager"] = bool(torch.equal(eager, logits))
    except Exception as e:                       # a side measurement must not take the benchmark down
        res["last_token_branch"]["hip_graph_error"] = repr(e)[:200]
    return res


def kv_offload_overlap(binding, synth, torch, tensors, out, dev, wl):
    """One layer's K and V of a 131072-token prefill ([131072,8,128] bf16 each, 512 MiB in all) copied to pinned
    host memory on a side stream while MLP steps of this workload run."""
    S, H, I = wl.S, wl.H, wl.I
    st = torch.cuda.current_stream()
    kvw = synth.Workload("kv", S=131072, H=H, I=I, mini_seq=wl.mini_seq, kv_heads=8)
    k, v = synth.kv_inputs(kvw, device=dev)
    host = torch.empty(2 * k.numel(), dtype=torch.bfloat16).pin_memory()
    side = torch.cuda.Stream()
    order, done = torch.cuda.Event(), torch.cuda.Event()
    order.record(st); done.record(st)
    ws = torch.empty(binding.mom_mlp_workspace_bytes(S, H, I, wl.mini_seq), dtype=torch.uint8, device=dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    # the first copy into a fresh pinned buffer pays for mapping its pages: warm it up once
    binding.mom_kv_offload(k, v, host, side, producer_stream=st, order_event=order, done_event=done)
    done.synchronize()
    t0 = time.perf_counter()
    binding.mom_kv_offload(k, v, host, side, producer_stream=st, order_event=order, done_event=done)
    done.synchronize()
    t_copy = time.perf_counter() - t0
    step = time_mlp(binding, torch, tensors, wl.mini_seq, out, ws, 4, 1)
    n_mlp = max(2, int(t_copy / step) + 1)               # enough MLP work to cover the copy
    t_mlp = n_mlp * time_mlp(binding, torch, tensors, wl.mini_seq, out, ws, n_mlp, 0)
    t_with, t_both = [], []
    for _ in range(3):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record(st)
        binding.mom_kv_offload(k, v, host, side, producer_stream=st, order_event=order, done_event=done)
        for _ in range(n_mlp):
            binding.mom_mlp_prefill(*tensors, wl.mini_seq, out, ws, stream=st)
        e1.record(st)
        torch.cuda.synchronize(); done.synchronize()
        t_both.append(time.perf_counter() - t0)
        t_with.append(e0.elapsed_time(e1) * 1e-3)
    kvb = 2 * k.numel() * 2
    res = {"bytes": kvb, "copy_alone_ms": round(t_copy * 1e3, 3), "d2h_GBps": round(kvb / t_copy / 1e9, 1),
           "mlp_steps": n_mlp, "mlp_alone_ms": round(t_mlp * 1e3, 3),
           "mlp_with_copy_in_flight_ms": round(min(t_with) * 1e3, 3), "both_done_ms": round(min(t_both) * 1e3, 3),
           "overlap_ratio": round(min(t_both) / max(t_mlp, t_copy), 4),
           "mlp_slowdown": round(min(t_with) / t_mlp - 1.0, 4),
           "kv_matches": bool(torch.equal(host[: k.numel()].view(torch.int16), k.cpu().view(torch.int16).ravel()))}
    return res


def cpu_baseline(wl, tensors, out, synth, torch, target_s):
    """The oracle as it stands, timed on the host cores over a bounded sample of rows (all threads, then one
    thread on a few rows); the rows it computes are also compared with what the GPU left in `out`."""
    import numpy as np
    import oracle
    x, wg, wu, wd = tensors
    threads = oracle.num_threads()
    wgb, wub, wdb = synth.bits(wg), synth.bits(wu), synth.bits(wd)
    flop_row = 6.0 * wl.H * wl.I
    # two probes separate the fixed cost (widening the weights) from the per-row cost
    def run(n):
        xb = synth.bits(x[:n])
        t0 = time.perf_counter()
        r = oracle.mlp_rows(xb, wgb, wub, wdb)
        return time.perf_counter() - t0, r
    (t_a, _), (t_b, _) = run(threads), run(3 * threads)
    per_batch = max((t_b - t_a) / 2.0, 1e-3)            # seconds per `threads` rows
    fixed = max(t_a - per_batch, 0.0)
    rows = int(max(1, min(512, (target_s - fixed) / per_batch))) * threads
    rows = min(rows, wl.S)
    dt, ref = run(rows)
    got = out[:rows].to(torch.float32).cpu().numpy()
    err = float(np.abs(got - ref).max() / np.abs(ref).max())
    # one thread: two row counts, so that the fixed cost drops out
    oracle.set_num_threads(1)
    (s_a, _), (s_b, _) = run(1), run(3)
    oracle.set_num_threads(threads)
    per_row_1 = max((s_b - s_a) / 2.0, 1e-6)
    return {"value": rows * flop_row / dt / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"first {rows} of {wl.S} rows of the same workload, all {wl.I} intermediate columns "
                      f"(includes widening the three weight matrices once), {dt:.1f} s",
            "extrapolated_full_job_s": wl.S * flop_row / (rows * flop_row / dt),
            "single_thread_gflops": flop_row / per_row_1 / 1e9,
            "single_thread_sample": "rows 0..2, marginal time per row",
            "parity_in_bench": {"rows": rows, "max_rel_err": err, "tolerance": 2e-2, "ok": bool(err <= 2e-2)}}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path has no cross-GPU step); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2504_12526_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    binding.lib()                      # fail loudly if the HIP library is missing
    binding.mom_init()
    dev = torch.device("cuda:0")
    wl = synth.WORKLOADS[args.workload]
    C = wl.mini_seq if args.mini_seq is None else args.mini_seq
    S, H, I = wl.S, wl.H, wl.I
    tensors = synth.mlp_inputs(wl, device=dev)
    out = torch.empty((S, H), dtype=torch.bfloat16, device=dev)
    ws_bytes = binding.mom_mlp_workspace_bytes(S, H, I, C)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()

    sec = time_mlp(binding, torch, tensors, C, out, ws, args.steps, args.warmup)
    flop = 6.0 * S * H * I
    tflops = flop / sec / 1e12

    t_gu, t_dn = kernel_times(binding, torch, tensors, C, out, ws, S, reps=max(2, min(5, args.steps)))
    n_full = S // C
    rows_per_launch = C if n_full else S
    gu_tflops = 4.0 * rows_per_launch * H * I / t_gu / 1e12
    dn_tflops = 2.0 * rows_per_launch * H * I / t_dn / 1e12

    result = {
        "metric": "mini-seq MLP prefill TFLOP/s (% bf16 MFMA peak) + peak workspace bytes",
        "value": round(tflops, 2), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: Llama-3-8B-shaped SwiGLU MLP layer S={S} H={H} I={I} mini_seq={C} bf16, "
                               f"unit-RMS rows, weights N(0,0.02), seed {wl.seed}"
                   if wl.name == "llama3_8b_32k" else f"{wl.name}: S={S} H={H} I={I} mini_seq={C} bf16",
                   "S": S, "H": H, "I": I, "mini_seq": C, "mini_sequences": -(-S // C)},
        "pct_bf16_mfma_peak": round(100.0 * tflops / BF16_MFMA_PEAK_TFLOPS, 2),
        "workspace_bytes": ws_bytes, "unchunked_workspace_bytes": S * I * 2,
        "device": device_info(torch, dev),
        "roofline": {"bound": "mfma", "kernel": "gemm4_kernel<EPI_GATEUP, ...> (gate/up GEMM + SiLU*up epilogue)",
                     "achieved": round(gu_tflops, 2), "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(gu_tflops / BF16_MFMA_PEAK_TFLOPS, 4),
                     "traffic": GATEUP_TRAFFIC_BYTES.get((wl.name, C)),
                     "avg_launch_ms": round(t_gu * 1e3, 4), "flop_per_launch": 4.0 * rows_per_launch * H * I,
                     "down_kernel": {"achieved": round(dn_tflops, 2), "avg_launch_ms": round(t_dn * 1e3, 4),
                                     "frac": round(dn_tflops / BF16_MFMA_PEAK_TFLOPS, 4)}},
    }

    if args.calib:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)       # 1 GiB read + 1 GiB written per launch
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        result["calib_copy_bytes_each_way"] = src.numel() * 4
        del src, dst

    if not args.no_side:
        # the CPU leg compares against `out`: run it on the timed configuration's output before anything reuses it
        probe = mfma_probe(binding, torch, tensors, dev)
        rf = result["roofline"]
        rf["sustained_peak"] = probe["workload_operands"]
        rf["sustained_peak_constant_operands"] = probe["constant_operands"]
        rf["sustained_peak_k_half_by_k_half"] = probe["workload_operands_k_half_by_k_half"]
        rf["frac_sustained"] = round(gu_tflops / probe["workload_operands"], 4)
        rf["sustained_peak_note"] = ("register-only v_mfma_f32_16x16x32_bf16 loop on all CUs (mom_debug_mfma_probe), operand "
                                     "fragments from this workload's W_gate and x, MFMAs in the kernels' order (both K-halves of a "
                                     "stage into an accumulator block back to back); k_half_by_k_half: the same MFMAs in the order "
                                     "the kernels used before; with constant operands the loop is not power-limited")
        result["whole_step_frac_sustained"] = round(tflops / probe["workload_operands"], 4)
        result["power"] = power_under_load(binding, torch, tensors, C, out, ws, S, H, I)
        side = {}
        side["mini_seq_sweep"] = mini_seq_sweep(binding, torch, tensors, out, dev, S, H, I, max(3, args.steps // 4))
        binding.mom_mlp_prefill(*tensors, C, out, ws)        # `out` of the timed configuration again (same bits anyway)
        torch.cuda.synchronize()
        side["peak_memory"] = peak_memory(binding, torch, tensors, out, dev, S, H, I, C)
        side.update(one_token_kernels(binding, synth, torch, tensors, dev, H, I, wl.V or (152064 if H == 3584 else 128256)))
        side["kv_offload"] = kv_offload_overlap(binding, synth, torch, tensors, out, dev, wl)
        result["side"] = side

    if args.extras:
        result["extras"] = extras(args, binding, synth, torch, wl, tensors, out, dev)

    if args.cpu_seconds > 0:
        result["cpu_baseline"] = cpu_baseline(wl, tensors, out, synth, torch, args.cpu_seconds)
        for k in ("value", "extrapolated_full_job_s", "single_thread_gflops"):
            result["cpu_baseline"][k] = float(f"{result['cpu_baseline'][k]:.4g}")
        result["cpu_baseline"]["parity_in_bench"]["max_rel_err"] = float(
            f"{result['cpu_baseline']['parity_in_bench']['max_rel_err']:.3g}")
    print(json.dumps(result))


def extras(args, binding, synth, torch, wl, tensors, out, dev):
    """Longer side measurements: the two-stream driver over the sweep and a six-layer offload schedule."""
    S, H, I = wl.S, wl.H, wl.I
    ex = {"pipelined_sweep": []}
    side2 = torch.cuda.Stream()
    pev = [torch.cuda.Event() for _ in range(5)]
    st = torch.cuda.current_stream()
    for e in pev:
        e.record(st)
    x, wg, wu, wd = tensors
    for C in (512, 1024, 2048, 4096):
        # the same step through mom_mlp_prefill_pipelined: down(c) on a second stream beside gate/up(c+1),
        # two workspace halves
        nb2 = binding.mom_mlp_pipelined_workspace_bytes(S, H, I, C)
        ws2 = torch.empty(nb2, dtype=torch.uint8, device=dev)
        reps = max(3, args.steps // 2)
        for i in range(2 + reps):
            if i == 2:
                torch.cuda.synchronize()
                t0 = time.perf_counter()
            binding.mom_mlp_prefill_pipelined(x, wg, wu, wd, C, out, ws2, st, side2, pev)
        torch.cuda.synchronize()
        sec2 = (time.perf_counter() - t0) / reps
        ex["pipelined_sweep"].append({"mini_seq": C, "workspace_bytes": nb2, "ms": round(sec2 * 1e3, 3),
                                      "tflops": round(6.0 * S * H * I / sec2 / 1e12, 1)})
        del ws2
    # a stack of layers (Algorithm 1 per layer): layer l's K/V (2 x 128 MiB) go to the host under layer l's MLP;
    # two device K/V buffers, buffer l%2 reused by layer l+2 only after the copy of layer l has finished
    side = torch.cuda.Stream()
    ws = torch.empty(binding.mom_mlp_workspace_bytes(S, H, I, wl.mini_seq), dtype=torch.uint8, device=dev)
    L = 6
    kvl = synth.Workload("kvl", S=65536, H=H, I=I, mini_seq=wl.mini_seq, kv_heads=8)
    bk, bv = synth.kv_inputs(kvl, device=dev)
    kb = [torch.empty_like(bk) for _ in range(2)]
    vb = [torch.empty_like(bv) for _ in range(2)]
    hosts = [torch.empty(2 * bk.numel(), dtype=torch.bfloat16).pin_memory() for _ in range(L)]
    orders = [torch.cuda.Event() for _ in range(L)]
    dones = [torch.cuda.Event() for _ in range(L)]
    for e in orders + dones:
        e.record(st)

    def stack(offload):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for l in range(L):
            b = l % 2
            if offload and l >= 2:
                st.wait_event(dones[l - 2])
            torch.mul(bk, float(l + 1), out=kb[b])
            torch.mul(bv, float(l + 1), out=vb[b])
            if offload:
                binding.mom_kv_offload(kb[b], vb[b], hosts[l], side, producer_stream=st, order_event=orders[l],
                                       done_event=dones[l])
            binding.mom_mlp_prefill(*tensors, wl.mini_seq, out, ws, stream=st)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    stack(True)                                   # maps the pinned pages
    t_plain = min(stack(False) for _ in range(2))
    t_off = min(stack(True) for _ in range(2))
    last_ok = bool(torch.equal(hosts[L - 1][: bk.numel()].view(torch.int16),
                               (bk * float(L)).cpu().view(torch.int16).ravel()))
    ex["layer_stack"] = {"layers": L, "kv_bytes_per_layer": 2 * bk.numel() * 2,
                         "mlp_only_ms": round(t_plain * 1e3, 3), "mlp_plus_offload_ms": round(t_off * 1e3, 3),
                         "offload_cost": round(t_off / t_plain - 1.0, 4), "last_layer_matches": last_ok}
    return ex


if __name__ == "__main__":
    main()
