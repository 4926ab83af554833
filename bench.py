#!/usr/bin/env python3
"""Benchmark of the inverse-convolution hot path on one MI355X.

One "step" = forward solve + log-determinant (invconv_fwd_logdet) and backward
pass (invconv_bwd) over one batch of the headline workload (B=16, C=3, 32x32,
k=3, fp32), inputs resident in HBM.  Prints ONE JSON line with images/s, the
roofline figures of the kernel that takes most of a step (the fused backward
kernel; the forward solve in a second block), both timed live with HIP events
on the launch stream, the cost of an empty dependent step as a floor, and the
CPU oracle timed on the host cores as a baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1] [--all]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
FP32_VECTOR_PEAK_TFLOPS = 157.3

PROFILES = os.path.join(ROOT, "profiles")
CALIBRATION_COPY_KIB = 65536.0   # the --calibration-copy run moves 64 MiB each way


def counter_traffic_bytes(summary: str, kernel: str, column: str = "median_KiB"):
    """HBM bytes per launch of `kernel` from a committed rocprofv3 --pmc summary under profiles/
    (sections '## FETCH_SIZE' and '## WRITE_SIZE', KiB per dispatch), each counter scaled by what it read for
    the 64 MiB device copy of the same run.  None if the file or the kernel is not there."""
    path = os.path.join(PROFILES, summary)
    if not os.path.exists(path):
        return None
    sect, rows = None, {"FETCH_SIZE": {}, "WRITE_SIZE": {}}
    col = 1 if column == "median_KiB" else 2
    with open(path) as f:
        for line in f:
            if line.startswith("## "):
                sect = line[3:].strip()
                continue
            parts = line.rsplit(None, 3)
            if sect in rows and len(parts) == 4 and not line.startswith(("#", "kernel")):
                try:
                    rows[sect][parts[0].strip()] = (float(parts[2]), float(parts[3]))
                except ValueError:
                    pass
    out = 0.0
    for sect in ("FETCH_SIZE", "WRITE_SIZE"):
        cal = [v[1] for k, v in rows[sect].items() if "copyBuffer" in k]
        hit = [v[col - 1] for k, v in rows[sect].items() if kernel in k]
        if not cal or not hit or cal[0] <= 0:
            return None
        out += hit[0] * CALIBRATION_COPY_KIB / cal[0] * 1024.0
    return int(out)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", type=int, default=1, help="workload id 0..4 (1 = headline)")
    ap.add_argument("--headline-only", action="store_true",
                    help="time only the selected workload (default: also workloads 0..4, reported under 'workloads')")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--variant", type=int, default=0)
    ap.add_argument("--variants", action="store_true",
                    help="also time the forward solve under every launch strategy (reported under 'variant_study')")
    ap.add_argument("--conv-only", action="store_true",
                    help="only time the sampling-direction convolution (invconv_conv_fwd) and print its table")
    ap.add_argument("--scale-study", action="store_true",
                    help="only the shapes of the paper's ablations (tall images, large batches, kernel sizes 2..11)")
    ap.add_argument("--flow-step", action="store_true",
                    help="only the flow step (inverse convolution + Actnorm + 1x1 convolution): fused kernels against "
                         "the same arithmetic as separate passes")
    ap.add_argument("--flow-shape", default=None, help="with --flow-step: only this named shape (for profiling)")
    ap.add_argument("--reps", type=int, default=None, help="with --flow-step: timed repetitions per form")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run three 64 MiB device copies (reference for the HBM byte counters)")
    return ap.parse_args()


class Layered:
    """Device buffers and raw-pointer launch closures for one workload (all layers)."""

    def __init__(self, cfg: int, variant: int = 0):
        import torch
        from paper_2410_14634_amd import binding as b
        from paper_2410_14634_amd import inputs
        self.b = b
        self.torch = torch
        wl = inputs.make_workload(cfg)
        self.wl = wl
        self.cfg = cfg
        self.variant = variant
        self.B, self.C, self.H, self.W, self.k, self.L = (wl[n] for n in ("B", "C", "H", "W", "k", "layers"))
        self.ws_d = [torch.from_numpy(w).cuda() for w in wl["w"]]
        self.acts = [torch.from_numpy(wl["y"]).cuda()] + [torch.empty(wl["y"].shape, device="cuda")
                                                          for _ in range(self.L)]
        self.g0 = torch.from_numpy(wl["g"]).cuda()
        # gradient ping-pong buffers (dL/dy of layer l is dL/dx of layer l-1)
        self.grads = [torch.empty_like(self.g0) for _ in range(2)]
        self.dws = [torch.empty_like(w) for w in self.ws_d]
        self.lds = torch.empty(self.L, device="cuda")
        need = b.bwd_workspace_bytes(self.B, self.C, self.H, self.W, self.k)
        self.wsp = b.new_workspace(need)            # header zeroed once, as the interface asks
        self.need = need
        self.lib = b.lib()
        self.n_elems = self.B * self.C * self.H * self.W
        if self.L > 1:
            # stacked layers go through the chain entry points (host arrays of device pointers)
            import ctypes
            arr = lambda ts: (ctypes.c_void_p * len(ts))(*[t.data_ptr() for t in ts])
            self.p_w, self.p_x, self.p_dw = arr(self.ws_d), arr(self.acts[1:]), arr(self.dws)
            self.cneed = b.chain_workspace_bytes(self.L, self.B, self.C, self.H, self.W, self.k)
            self.cws = b.new_workspace(self.cneed)

    # raw C-ABI calls: pointers and sizes only
    def fwd_layer(self, l, stream):
        st = self.lib.invconv_fwd_ex(self.acts[l].data_ptr(), self.ws_d[l].data_ptr(), self.acts[l + 1].data_ptr(),
                                     self.B, self.C, self.H, self.W, self.k, stream, self.variant)
        assert st == 0, self.b.status_string(st)

    def bwd_layer(self, l, gin, gout, stream):
        st = self.lib.invconv_bwd_ex(self.acts[l + 1].data_ptr(), self.ws_d[l].data_ptr(), gin.data_ptr(),
                                     gout.data_ptr(), self.dws[l].data_ptr(), self.B, self.C, self.H, self.W,
                                     self.k, self.wsp.data_ptr(), self.need, stream, self.variant)
        assert st == 0, self.b.status_string(st)

    def fwd_logdet_layer(self, l, stream):
        st = self.lib.invconv_fwd_logdet(self.acts[l].data_ptr(), self.ws_d[l].data_ptr(), self.acts[l + 1].data_ptr(),
                                         self.lds[l:l + 1].data_ptr(), self.B, self.C, self.H, self.W, self.k, stream)
        assert st == 0, self.b.status_string(st)

    def logdet_layer(self, l, stream):
        st = self.lib.invconv_logdet(self.ws_d[l].data_ptr(), self.C, self.H, self.W, self.k,
                                     self.lds[l:l + 1].data_ptr(), stream)
        assert st == 0, self.b.status_string(st)

    def fwd_all(self, stream):
        if self.L > 1 and self.variant == 0:
            st = self.lib.invconv_chain_fwd(self.acts[0].data_ptr(), self.p_w, self.p_x, self.L, self.B, self.C,
                                            self.H, self.W, self.k, self.cws.data_ptr(), self.cneed, stream)
            assert st == 0, self.b.status_string(st)
            return
        for l in range(self.L):
            self.fwd_layer(l, stream)

    def bwd_all(self, stream):
        # single layer: upstream gradient is the seeded dL/dx; chain: dL/dx_L = x_L (loss 0.5*sum x^2)
        if self.L > 1 and self.variant == 0:
            st = self.lib.invconv_chain_bwd(self.p_x, self.p_w, self.acts[self.L].data_ptr(), self.grads[0].data_ptr(),
                                            self.p_dw, self.L, self.B, self.C, self.H, self.W, self.k,
                                            self.cws.data_ptr(), self.cneed, stream)
            assert st == 0, self.b.status_string(st)
            return
        gin = self.g0 if self.L == 1 else self.acts[self.L]
        for i, l in enumerate(reversed(range(self.L))):
            gout = self.grads[i % 2]
            self.bwd_layer(l, gin, gout, stream)
            gin = gout

    def logdet_all(self, stream):
        if self.L > 1 and self.variant == 0:
            st = self.lib.invconv_chain_logdet(self.p_w, self.L, self.C, self.H, self.W, self.k,
                                               self.lds.data_ptr(), stream)
            assert st == 0, self.b.status_string(st)
            return
        for l in range(self.L):
            self.logdet_layer(l, stream)

    def step(self, stream):
        if self.L == 1 and self.variant == 0:
            # forward solve and log-determinant in one call, then the backward pass
            self.fwd_logdet_layer(0, stream)
            self.bwd_all(stream)
            return
        self.fwd_all(stream)
        self.bwd_all(stream)
        self.logdet_all(stream)


def time_region(torch, fn, reps, warmup):
    """Wall-clock of `reps` calls bracketed by device synchronisation; returns ms per call."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / reps


def event_time(torch, fn, reps, warmup):
    """Median / mean ms of single calls, each bracketed by HIP events on the launch stream."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for e0, e1 in evs:
        e0.record()
        fn()
        e1.record()
    torch.cuda.synchronize()
    ts = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    return ts[len(ts) // 2], sum(ts) / len(ts), ts[0]


def event_time_batch(torch, fn, reps, warmup):
    """Mean ms per call of `reps` back-to-back calls between one pair of HIP events."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def measure_workload(cfg, steps, warmup, variant=0):
    import torch
    L = Layered(cfg, variant)
    stream = torch.cuda.current_stream().cuda_stream
    ms_step = time_region(torch, lambda: L.step(stream), steps, warmup)
    ms_fwd = event_time_batch(torch, lambda: L.fwd_all(stream), max(steps // 4, 5), 3)
    ms_bwd = event_time_batch(torch, lambda: L.bwd_all(stream), max(steps // 4, 5), 3)
    bytes_step = 20.0 * L.n_elems * L.L
    macs_per_elt = L.C * (L.k * L.k - 1) + (L.C - 1) / 2.0          # one solve; the weight gradient costs as much again
    flops_step = 6.0 * macs_per_elt * L.n_elems * L.L               # fwd solve 2x, bwd solve 2x, dL/dw 2x (x2 flop/MAC)
    return L, dict(
        workload=cfg, B=L.B, C=L.C, H=L.H, W=L.W, k=L.k, layers=L.L,
        ms_per_step=ms_step, ms_fwd=ms_fwd, ms_bwd=ms_bwd,
        images_per_s=L.B / (ms_step * 1e-3),
        us_per_diagonal=(ms_fwd + ms_bwd) * 1e3 / (2 * L.L * (L.H + L.W - 1)),
        algorithmic_gbs=bytes_step / (ms_step * 1e-3) / 1e9,
        hbm_frac=bytes_step / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        fp32_tflops=flops_step / (ms_step * 1e-3) / 1e12,
        fp32_frac=flops_step / (ms_step * 1e-3) / 1e12 / FP32_VECTOR_PEAK_TFLOPS,
    )


def chain_roofline(torch, L, stream, reps):
    """Workload 4: the pipelined chain launch (all layers of one direction in one launch).  At 12 channels the
    arithmetic intensity (about 30 flop/byte) is past the ridge of the fp32 roofs, so the matrix/vector fp32
    peak is the bound that binds; the HBM fraction and the counter-measured traffic are reported beside it."""
    ms_f = event_time_batch(torch, lambda: L.fwd_all(stream), reps, 2)
    n = L.n_elems * L.L
    macs = L.C * (L.k * L.k - 1) + (L.C - 1) / 2.0
    flops = 2.0 * macs * n
    alg_bytes = 8.0 * n
    traffic = counter_traffic_bytes("hbm_counters_workload4_chain.txt", "k_chain_band<3, 3, 0", "max_KiB")
    tf = flops / (ms_f * 1e-3) / 1e12
    gbs = alg_bytes / (ms_f * 1e-3) / 1e9
    return dict(bound="mfma", achieved=tf, peak=FP32_VECTOR_PEAK_TFLOPS, unit="TFLOP/s", frac=tf / FP32_VECTOR_PEAK_TFLOPS,
                traffic=traffic, kernel="pipelined chain launch, forward direction (all layers, one launch)",
                kernel_ms_back_to_back=ms_f, algorithmic_bytes_per_launch=alg_bytes, flops_per_launch=flops,
                hbm=dict(achieved=gbs, peak=HBM_PEAK_GBS, unit="GB/s", frac=gbs / HBM_PEAK_GBS),
                traffic_over_algorithmic=(traffic / alg_bytes if traffic else None))


def device_info(torch):
    """What the runtime reports for the GPU, and a measured streaming copy (read + write) to hold beside the
    published HBM peak."""
    p = torch.cuda.get_device_properties(0)
    info = dict(name=p.name, compute_units=p.multi_processor_count,
                clock_mhz=(p.clock_rate / 1e3 if getattr(p, "clock_rate", 0) else None),   # None: not reported here
                published_clock_mhz=2400, memory_gib=p.total_memory / 2**30)
    n = 512 * 1024 * 1024 // 4
    src = torch.zeros(n, device="cuda")
    dst = torch.empty_like(src)
    ms = event_time_batch(torch, lambda: dst.copy_(src), 20, 3)
    info["measured_copy_gbs"] = 2.0 * n * 4 / (ms * 1e-3) / 1e9
    info["measured_copy_note"] = "512 MiB device-to-device copy, bytes read + bytes written over the mean of 20 copies"
    return info


def graph_replay_ms(torch, L, reps):
    """The same step captured once into a HIP graph and replayed: what is left when the host's launch work
    is taken out (reported beside ms_per_step, never instead of it)."""
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        L.step(side.cuda_stream)                  # warm up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            L.step(side.cuda_stream)
    torch.cuda.synchronize()
    return event_time_batch(torch, graph.replay, reps, 5)


def variant_study(cfg, reps=200):
    """Forward solve of one workload under every launch strategy (us per call, HIP events)."""
    import torch
    from paper_2410_14634_amd import binding as b
    names = {b.VARIANT_AUTO: "auto", b.VARIANT_BLOCK: "workgroup per image, LDS window, barrier per diagonal",
             b.VARIANT_DIAG_LAUNCH: "one launch per diagonal, eager", b.VARIANT_WAVE: "wave per image, registers + DPP",
             b.VARIANT_BAND: "wave per 16-row band, MFMA 16x16x4",
             b.VARIANT_PERSISTENT: "persistent cooperative grid, device barrier per diagonal"}
    out = {}
    stream = torch.cuda.current_stream().cuda_stream
    for var, name in names.items():
        L = Layered(cfg, var)
        try:
            L.fwd_layer(0, stream)
            torch.cuda.synchronize()
        except AssertionError:
            continue                     # variant does not cover this shape
        r = reps if var not in (b.VARIANT_DIAG_LAUNCH, b.VARIANT_PERSISTENT) else max(reps // 10, 5)
        out[name] = event_time_batch(torch, lambda: L.fwd_layer(0, stream), r, 3) * 1e3
    # launch-per-diagonal captured once into a HIP graph and replayed
    L = Layered(cfg, b.VARIANT_DIAG_LAUNCH)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        L.fwd_layer(0, side.cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        L.fwd_layer(0, torch.cuda.current_stream().cuda_stream)
    out["one launch per diagonal, HIP graph replay"] = event_time_batch(torch, graph.replay, max(reps // 4, 5), 3) * 1e3
    # cost of one dependent step under each ordering mechanism, no arithmetic (us per step)
    lib = b.lib()
    steps = 200
    probe = {}
    for mode, name in ((0, "kernel launch per step, eager"), (1, "device-wide barrier in a cooperative grid"),
                       (2, "workgroup barrier + LDS exchange")):
        for wgs in (16, 256):
            def run(mode=mode, wgs=wgs):
                assert lib.invconv_probe_step_sync(mode, steps, wgs, stream) == 0
            probe[f"{name}, {wgs} workgroups"] = event_time_batch(torch, run, 10, 2) * 1e3 / steps
    graph2 = torch.cuda.CUDAGraph()
    assert lib.invconv_probe_step_sync(0, steps, 16, stream) == 0
    torch.cuda.synchronize()
    with torch.cuda.graph(graph2):
        assert lib.invconv_probe_step_sync(0, steps, 16, torch.cuda.current_stream().cuda_stream) == 0
    probe["kernel launch per step, HIP graph replay, 16 workgroups"] = \
        event_time_batch(torch, graph2.replay, 10, 2) * 1e3 / steps
    out["empty step cost, us per step"] = probe
    return out


def cpu_baseline(cfg, seconds):
    """The CPU oracle, as it stands, on the same workload (bounded sample), all host cores."""
    import oracle
    from paper_2410_14634_amd import inputs
    wl = inputs.make_workload(cfg)
    layers = wl["layers"]
    B = wl["B"]
    sample = f"workload {cfg}, full batch of {B}, fwd+bwd+logdet"
    if cfg == 4:       # chain is ~15 GMAC per pass on the CPU: time a slice of the batch, one pass
        B = 4
        wl = inputs.make_workload(cfg, B=B)
        sample = f"workload {cfg}, {B} of 32 images, all {layers} layers, fwd+bwd+logdet, one pass"
    threads = oracle.max_threads()

    def one_pass():
        xs = [wl["y"]]
        for w in wl["w"]:
            xs.append(oracle.invconv_fwd(xs[-1], w, threads))
        g = wl["g"] if layers == 1 else xs[-1]
        for l in reversed(range(layers)):
            g, _ = oracle.invconv_bwd(xs[l + 1], wl["w"][l], g, threads)
            oracle.invconv_logdet(wl["w"][l], wl["H"], wl["W"])

    one_pass()
    n, t0 = 0, time.perf_counter()
    while True:
        one_pass()
        n += 1
        el = time.perf_counter() - t0
        if el >= seconds or (cfg == 4 and n >= 1):
            break
    out = dict(value=B * n / el, unit="images/s", cores=threads, kind="oracle",
               sample=f"{sample}; {n} passes in {el:.1f} s")
    # the same oracle on one thread (a short sample), and the host it ran on
    if cfg != 4:
        all_threads, threads = threads, 1
        one_pass()
        n1, t1 = 0, time.perf_counter()
        while time.perf_counter() - t1 < min(2.0, seconds):
            one_pass()
            n1 += 1
        out["value_single_thread"] = B * n1 / (time.perf_counter() - t1)
        threads = all_threads
    try:
        with open("/proc/cpuinfo") as f:
            models = [ln.split(":", 1)[1].strip() for ln in f if ln.startswith("model name")]
        out["cpu_model"] = models[0] if models else None
        out["host_logical_cpus"] = len(models) or os.cpu_count()
    except OSError:
        out["cpu_model"] = None
    return out


CONV_SHAPES = {  # the sampling-direction operator y = conv_w(x); streaming sizes besides the workload shapes
    "workload1": (16, 3, 32, 32, 3), "workload2": (64, 12, 16, 16, 3), "workload3": (32, 3, 64, 64, 5),
    "workload4_layer": (32, 12, 128, 128, 3),
    "stream_c3": (256, 3, 256, 256, 3), "stream_c12": (256, 12, 128, 128, 3),
}
FP32_MFMA_PEAK_TFLOPS = 157.3


def measure_conv(reps=100):
    """invconv_conv_fwd / invconv_conv_bwd on device-resident tensors: us per call, algorithmic GB/s
    (fwd: read x, write y; bwd: read x and dL/dy, write dL/dx), TFLOP/s."""
    import torch
    from paper_2410_14634_amd import binding as b
    lib = b.lib()
    stream = torch.cuda.current_stream().cuda_stream
    out = {}
    for name, (B, C, H, W, k) in CONV_SHAPES.items():
        g = torch.Generator(device="cpu").manual_seed(7)
        x = torch.randn(B, C, H, W, generator=g).cuda()
        w = (torch.randn(C, C, k, k, generator=g) * 0.05).cuda()
        y = torch.empty_like(x)

        def call():
            st = lib.invconv_conv_fwd(x.data_ptr(), w.data_ptr(), y.data_ptr(), B, C, H, W, k, stream)
            if st != 0:
                raise RuntimeError(f"invconv_conv_fwd failed with status {st}")
        g_ = torch.randn(B, C, H, W, generator=g).cuda()
        dx, dw = torch.empty_like(x), torch.empty_like(w)
        need = lib.invconv_bwd_workspace_bytes(B, C, H, W, k)
        ws = b.new_workspace(need)

        def call_bwd():
            st = lib.invconv_conv_bwd(x.data_ptr(), w.data_ptr(), g_.data_ptr(), dx.data_ptr(), dw.data_ptr(),
                                      B, C, H, W, k, ws.data_ptr(), need, stream)
            if st != 0:
                raise RuntimeError(f"invconv_conv_bwd failed with status {st}")
        ms = event_time_batch(torch, call, reps, 5)
        ms_bwd = event_time_batch(torch, call_bwd, max(reps // 2, 5), 3)
        byts = 8.0 * x.numel()
        flops = 2.0 * x.numel() * (C * k * k - (C - 1) / 2.0)
        out[name] = dict(B=B, C=C, H=H, W=W, k=k, us_per_call=ms * 1e3, algorithmic_gbs=byts / ms / 1e6,
                         hbm_frac=byts / ms / 1e6 / HBM_PEAK_GBS, fp32_tflops=flops / ms / 1e9,
                         mfma_fp32_frac=flops / ms / 1e9 / FP32_MFMA_PEAK_TFLOPS,
                         bwd_us_per_call=ms_bwd * 1e3, bwd_algorithmic_gbs=12.0 * x.numel() / ms_bwd / 1e6,
                         bwd_fp32_tflops=2.0 * flops / ms_bwd / 1e9)
    return out


SCALE_SHAPES = {  # (B, C, H, W, k): the paper's image-size / batch-size / kernel-size ablations, synthetic inputs
    "tall_b1": (1, 3, 256, 256, 3), "tall_b16": (16, 3, 256, 256, 3), "tall_b128": (128, 3, 256, 256, 3),
    "tall_512": (1, 3, 512, 512, 3),
    "batch_256": (256, 3, 32, 32, 3), "batch_1024": (1024, 3, 32, 32, 3), "batch_4096": (4096, 3, 32, 32, 3),
    "k2": (16, 3, 32, 32, 2), "k5": (16, 3, 32, 32, 5), "k7": (16, 3, 32, 32, 7), "k9": (16, 3, 32, 32, 9),
    "k11": (16, 3, 32, 32, 11), "mnist_like": (128, 1, 28, 28, 3),
    "c48_two_squeezes": (32, 48, 32, 32, 3), "c24": (32, 24, 64, 64, 3), "c32": (64, 32, 32, 32, 3),
    # a 3x32x32 input after one and two squeezes at the paper's batch size, and the kernel-size ablation on both
    "b100_c12": (100, 12, 16, 16, 3), "b100_c48": (100, 48, 8, 8, 3), "b100_c12_k2": (100, 12, 16, 16, 2),
    "b100_c12_k5": (100, 12, 16, 16, 5), "b100_c12_k7": (100, 12, 16, 16, 7),
    "b100_c12_k9": (100, 12, 16, 16, 9), "b100_c12_k11": (100, 12, 16, 16, 11),
    "b100_c48_k2": (100, 48, 8, 8, 2), "b100_c48_k5": (100, 48, 8, 8, 5), "b100_c48_k7": (100, 48, 8, 8, 7),
    "b100_c48_k9": (100, 48, 8, 8, 9), "b100_c48_k11": (100, 48, 8, 8, 11),
    "b1024_c12": (1024, 12, 16, 16, 3), "b1024_c48": (1024, 48, 8, 8, 3),
}


def scale_study(reps=30):
    """invconv_fwd / invconv_bwd at the shapes of the paper's ablations: us per call, images/s of forward + backward,
    algorithmic GB/s (20 bytes per element).  Not part of the default run."""
    import torch
    from paper_2410_14634_amd import binding as b
    from paper_2410_14634_amd import inputs
    out = {}
    for name, (B, C, H, W, k) in SCALE_SHAPES.items():
        cs = inputs.make_case(B, C, H, W, k, seed=5, tap_std=0.15 / k)
        y, w, g = (torch.from_numpy(cs[n]).cuda() for n in ("y", "g", "y"))
        w = torch.from_numpy(cs["w"][0]).cuda()
        g = torch.from_numpy(cs["g"]).cuda()
        x = torch.empty_like(y)
        v, dw = torch.empty_like(y), torch.empty_like(w)
        wsp = b.new_workspace(b.bwd_workspace_bytes(B, C, H, W, k))
        wsf = b.new_workspace(b.fwd_workspace_bytes(B, C, H, W, k))
        b.invconv_fwd(y, w, out=x, workspace=wsf)
        ms_f = event_time_batch(torch, lambda: b.invconv_fwd(y, w, out=x, workspace=wsf), reps, 3)
        ms_b = event_time_batch(torch, lambda: b.invconv_bwd(x, w, g, out=(v, dw), workspace=wsp), reps, 3)
        n = B * C * H * W
        extra = {}
        if name.startswith("batch_"):
            # the bf16-storage variant (half the HBM bytes, fp32 arithmetic) on the bandwidth-bound batches
            y16, g16 = y.to(torch.bfloat16), g.to(torch.bfloat16)
            x16, v16 = torch.empty_like(y16), torch.empty_like(y16)
            ws16 = b.new_workspace(b.bf16_workspace_bytes(B, C, H, W, k))
            b.invconv_fwd_bf16(y16, w, out=x16, workspace=ws16)
            ms_f16 = event_time_batch(torch, lambda: b.invconv_fwd_bf16(y16, w, out=x16, workspace=ws16), reps, 3)
            ms_b16 = event_time_batch(torch, lambda: b.invconv_bwd_bf16(x16, w, g16, out=(v16, dw), workspace=ws16),
                                      reps, 3)
            extra = dict(bf16_fwd_us=ms_f16 * 1e3, bf16_bwd_us=ms_b16 * 1e3,
                         bf16_images_per_s=B / ((ms_f16 + ms_b16) * 1e-3))
        out[name] = dict(B=B, C=C, H=H, W=W, k=k, fwd_us=ms_f * 1e3, bwd_us=ms_b * 1e3, **extra,
                         images_per_s=B / ((ms_f + ms_b) * 1e-3),
                         algorithmic_gbs=20.0 * n / ((ms_f + ms_b) * 1e-3) / 1e9,
                         us_per_diagonal=(ms_f + ms_b) * 1e3 / (2 * (H + W - 1)))
    return out


FLOW_SHAPES = {  # (B, C, H, W, k)
    "workload1": (16, 3, 32, 32, 3), "workload3": (32, 3, 64, 64, 5),
    "batch_1024": (1024, 3, 32, 32, 3), "batch_4096": (4096, 3, 32, 32, 3), "batch_1024_64x64": (1024, 3, 64, 64, 3),
    "workload4_layer": (32, 12, 128, 128, 3), "batch_256_c12": (256, 12, 64, 64, 3),
}


def flow_step_study(reps=50, only=None):
    """One flow step (Section 4.1: inverse convolution, Actnorm, 1 x 1 convolution) forward + backward: the fused
    kernels (read y, write z; read z and dL/dz, write dL/dy: 20 bytes per element, what the inverse convolution
    alone moves) against the same arithmetic as separate passes (60 bytes per element: each neighbour adds a read
    and a write in the forward pass and two reads and a write in the backward pass)."""
    import torch
    from paper_2410_14634_amd import binding as b
    from paper_2410_14634_amd import inputs
    out = {}
    for name, (B, C, H, W, k) in FLOW_SHAPES.items():
        if only and name != only:
            continue
        cs = inputs.make_case(B, C, H, W, k, seed=9, tap_std=0.05)
        p = inputs.make_flow_params(C, 9)
        y, w, g = (torch.from_numpy(cs[n] if n != "w" else cs["w"][0]).cuda() for n in ("y", "w", "g"))
        s, bb, Q = (torch.from_numpy(p[n]).cuda() for n in ("s", "b", "Q"))
        ws = b.new_workspace(b.flowstep_workspace_bytes(B, C, H, W, k))
        z = torch.empty_like(y)
        grads = dict(dy=torch.empty_like(y), dw=torch.empty_like(w), ds=torch.empty_like(s), db=torch.empty_like(bb),
                     dQ=torch.empty_like(Q))
        row = dict(B=B, C=C, H=H, W=W, k=k)
        n = B * C * H * W
        # 8-16 channels: forward fully fused (8), backward solve fused (8) + x recomputed once (8) + dL/dw (8) + sums (8);
        # separate passes: 24 forward, 40 backward (few channels: the fused dL/dw kernel saves 4 of them)
        fused_bytes = 20.0 if C <= 4 else 40.0
        sep_bytes = 60.0 if C <= 4 else 64.0
        # "auto" is what a caller gets: few images of few channels ride on the split solve kernels (map applied inside)
        for form, tag, bytes_per_elt in ((b.FLOW_FUSED, "fused", fused_bytes), (b.FLOW_SEPARATE, "separate", sep_bytes),
                                         (b.FLOW_AUTO, "auto", fused_bytes)):
            fwd = lambda: b.invconv_flowstep_fwd(y, w, s, bb, Q, out=z, workspace=ws, form=form)
            bwd = lambda: b.invconv_flowstep_bwd(z, w, s, bb, Q, g, logdet_weight=-float(B), workspace=ws, form=form,
                                                 out=grads)
            fwd()
            ms_f = event_time_batch(torch, fwd, reps, 3)
            ms_b = event_time_batch(torch, bwd, reps, 3)
            row[tag] = dict(fwd_us=ms_f * 1e3, bwd_us=ms_b * 1e3, images_per_s=B / ((ms_f + ms_b) * 1e-3),
                            hbm_bytes_per_element=bytes_per_elt,
                            gbs=bytes_per_elt * n / ((ms_f + ms_b) * 1e-3) / 1e9)
        row["speedup_fused_over_separate"] = (row["separate"]["fwd_us"] + row["separate"]["bwd_us"]) / \
            (row["fused"]["fwd_us"] + row["fused"]["bwd_us"])
        out[name] = row
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (every image is an independent solve, so more GPUs "
              "would each take a slice of the batch); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2410_14634_amd import binding as b
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    b.lib()   # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)
    if args.calibration_copy:
        # a plain device copy of known size: what the HBM byte counters read for it scales the
        # counter readings of the kernels (64 MiB read + 64 MiB written)
        src = torch.zeros(64 * 1024 * 1024 // 4, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    if args.conv_only:
        print(json.dumps(dict(sampling_conv=measure_conv())), flush=True)
        return
    if args.scale_study:
        print(json.dumps(dict(scale_study=scale_study())), flush=True)
        return
    if args.flow_step:
        print(json.dumps(dict(flow_step=flow_step_study(reps=args.reps or 50, only=args.flow_shape))), flush=True)
        return
    cfg = args.workload
    L, res = measure_workload(cfg, args.steps, args.warmup, args.variant)

    stream = torch.cuda.current_stream().cuda_stream
    reps = max(min(args.steps, 500), 20)
    nsteps = L.H + L.W - 1

    def kernel_block(name, fn, bytes_per_elt, traffic):
        """HIP-event timing of one call that is one kernel launch; algorithmic bytes over its mean duration."""
        k_med, k_mean, k_min = event_time(torch, fn, reps, 20)
        k_batch = event_time_batch(torch, fn, reps, 20)
        kernel_bytes = bytes_per_elt * L.n_elems
        achieved = kernel_bytes / (k_batch * 1e-3) / 1e9
        return dict(bound="hbm", achieved=achieved, peak=HBM_PEAK_GBS, unit="GB/s", frac=achieved / HBM_PEAK_GBS,
                    traffic=traffic, kernel=name, kernel_ms_back_to_back=k_batch, kernel_ms_event_pair_median=k_med,
                    kernel_ms_event_pair_min=k_min, algorithmic_bytes_per_launch=kernel_bytes,
                    traffic_over_algorithmic=(traffic / kernel_bytes if traffic else None),
                    dependent_steps=nsteps, us_per_dependent_step=k_batch * 1e3 / nsteps)

    if L.L == 1:
        gin, gout = L.g0, L.grads[0]
        summary = f"hbm_counters_workload{cfg}_headline.txt" if cfg == 1 else f"hbm_counters_workload{cfg}.txt"
        # the kernel with the most time per step: the fused backward (transposed solve + dL/dw), 12 B per element
        roofline = kernel_block("backward: transposed solve + weight gradient (the launch invconv_bwd makes"
                                + (")" if L.C <= 4 and L.H <= 64 and L.k <= 7 else "; first of several)"),
                                lambda: L.bwd_layer(0, gin, gout, stream), 12.0,
                                counter_traffic_bytes(summary, "k_bwd_wave"))
        roofline_fwd = kernel_block("forward wavefront solve + log-determinant (the launch invconv_fwd_logdet makes)",
                                    lambda: L.fwd_logdet_layer(0, stream), 8.0,
                                    counter_traffic_bytes(summary, "k_solve_wave"))
    else:
        roofline = chain_roofline(torch, L, stream, reps=max(args.steps // 20, 5))
        roofline_fwd = None
    # floor: an empty dependent step ordered by a workgroup barrier + LDS exchange (no arithmetic, no memory)
    lib = b.lib()
    probe_steps = 2000
    def probe():
        assert lib.invconv_probe_step_sync(2, probe_steps, max(min(L.B, 256), 1), stream) == 0
    floor_us = event_time_batch(torch, probe, 20, 3) * 1e3 / probe_steps
    for r in (roofline, roofline_fwd):
        if r and "us_per_dependent_step" in r:
            r["empty_step_floor_us"] = floor_us
            r["step_over_floor"] = r["us_per_dependent_step"] / floor_us

    out = dict(
        metric="inverse-conv fwd+bwd images/sec at m=32,C=3,k=3; achieved HBM GB/s fraction",
        value=res["images_per_s"], unit="images/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
        ms_per_step=res["ms_per_step"], higher_is_better=True, scaling="weak", vs_baseline=None,
        dtype="f32", data="synthetic",
        config=dict(workload=f"workload {cfg}: B={L.B} C={L.C} H=W={L.H} k={L.k} layers={L.L}, "
                             + ("step = invconv_fwd_logdet + invconv_bwd" if L.L == 1 else
                                "step = invconv_chain_fwd + invconv_chain_bwd + invconv_chain_logdet")
                             + ", eager launches on one stream",
                    variant=args.variant),
        ms_fwd=res["ms_fwd"], ms_bwd=res["ms_bwd"], algorithmic_gbs=res["algorithmic_gbs"],
        hbm_frac_whole_step=res["hbm_frac"],
        roofline=roofline, roofline_forward=roofline_fwd,
    )
    if not args.headline_only:
        dev = device_info(torch)
        out["device"] = dev
        if roofline.get("unit") == "GB/s":
            roofline["frac_of_measured_copy"] = roofline["achieved"] / dev["measured_copy_gbs"]
        if L.L == 1 and cfg in (0, 1):
            out["ms_per_step_graph_replay"] = graph_replay_ms(torch, L, max(min(args.steps, 500), 20))
        others = {}
        for c in range(5):
            if c == cfg:
                others[str(c)] = res
                continue
            st = {0: args.steps, 1: args.steps, 2: max(args.steps // 2, 10), 3: max(args.steps // 4, 10),
                  4: max(args.steps // 50, 10)}[c]
            # (the chain's heavy launches need a few more warm-up steps than the rest: the clocks ramp up)
            Lc, r = measure_workload(c, st, max(st // 10, 8 if c == 4 else 2), args.variant)
            if c in (0, 1):
                r["ms_per_step_graph_replay"] = graph_replay_ms(torch, Lc, max(min(st, 500), 20))
            if c == 4:
                r["roofline"] = chain_roofline(torch, Lc, torch.cuda.current_stream().cuda_stream, reps=5)
            others[str(c)] = r
            print(f"[bench] workload {c}: {json.dumps(r)}", file=sys.stderr, flush=True)
        for r in others.values():
            r["hbm_frac_of_measured_copy"] = r["algorithmic_gbs"] / dev["measured_copy_gbs"]
        out["workloads"] = others
        out["sampling_conv"] = measure_conv()
        print(f"[bench] sampling conv: {json.dumps(out['sampling_conv'])}", file=sys.stderr, flush=True)
    if args.variants:
        out["variant_study_us_per_fwd_call"] = variant_study(cfg)
        print(f"[bench] variants: {json.dumps(out['variant_study_us_per_fwd_call'])}", file=sys.stderr, flush=True)
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(cfg, args.cpu_seconds)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
