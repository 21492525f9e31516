#!/usr/bin/env python3
"""Benchmark of the decoder-layer linear-operator hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input:
thi_rmsnorm_qkv, thi_linear (O projection) and thi_swiglu_mlp enqueued
back-to-back on one stream.  Headline workload: the Llama-7B-shaped layer at
decode M=32 (the configuration the metric is quoted on); the same line carries
the prefill half of the metric (`prefill`: the 70B-shaped layer at M=2048 and
the 13B-shaped layer at M=512, each with its own `roofline`).  Weight copies are
rotated between steps so that the 256 MB last-level cache cannot serve them.

Every figure is the MEDIAN of >= 5 blocks of >= 50 launches, each block
bracketed by HIP events on the launch stream (`timing` in the output says how
many); --steps only raises the launches per block.

Prints ONE JSON line (see README for the fields).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
UP_OFFSET_BYTES = 65536      # w_up starts this far past the end of w_gate (see device_weights)
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


BLOCKS = 5                 # timed blocks per figure (the median is reported)
MIN_PER_BLOCK = 50         # launches per block at least


def committed_traffic():
    """Per-launch HBM KiB (fetch, write) of the gate/up kernel from the rocprofv3 --pmc runs summarised under
    profiles/, already scaled by the copy-kernel factor, keyed "config/M" -- with the commit they were
    measured at, which is reported next to the figure (a later kernel change makes them stale)."""
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as f:
            return json.load(f)
    except (OSError, ValueError):
        return {}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, help="layer config 1..5 (default 2 = Llama-7B shape)")
    ap.add_argument("--m", type=int, default=32, help="tokens per step (decode batch or prefill length)")
    ap.add_argument("--rotate-bytes", type=float, default=1.5e9, help="bytes of distinct weight copies to rotate through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--context", type=int, default=2048,
                    help="cached positions per request for the decode-attention timing (extra, decode only; 0 = skip)")
    ap.add_argument("--sweep", action="store_true", help="also time the other configs/M (extra, not the headline)")
    ap.add_argument("--no-prefill", action="store_true", help="skip the prefill legs (70B M=2048, 13B M=512)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="run one plain 1 GiB device copy before the timed region (scales rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--traffic-kib", type=float, nargs=2, default=None, metavar=("FETCH", "WRITE"),
                    help="per-launch HBM KiB of the dominant kernel from rocprofv3 --pmc runs, already scaled; reported as roofline.traffic")
    return ap.parse_args()


def device_weights(cfg, copies, host_layer):
    """copies of the layer's weights on the device: copy 0 is the seeded host layer,
    the others are seeded device draws with the same distribution."""
    import numpy as np
    import torch

    def to_dev(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.float16)

    names = ("w_qkv", "w_o", "w_gate", "w_up", "w_down")
    shapes = {"w_qkv": (cfg.n_qkv, cfg.hidden), "w_o": (cfg.hidden, cfg.hidden), "w_gate": (cfg.inter, cfg.hidden),
              "w_up": (cfg.inter, cfg.hidden), "w_down": (cfg.hidden, cfg.inter)}
    out = []
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20260525 + 100 * cfg.index)
    # Placement of w_up (include/thi.h, thi_swiglu_mlp): torch hands out large tensors on 2 MiB boundaries, which
    # puts w_up a whole multiple of 2 MiB behind w_gate; the gate/up kernel, which streams the same rows of both at
    # once, measured 1-2 % slower that way.  w_gate and w_up therefore share one allocation with w_up
    # UP_OFFSET_BYTES past the end of w_gate (THI_BENCH_UP_OFFSET overrides; 0 = back to back).
    up_off = int(os.environ.get("THI_BENCH_UP_OFFSET", UP_OFFSET_BYTES)) // 2
    gu = cfg.inter * cfg.hidden
    for c in range(copies):
        d = {}
        pair = torch.empty(2 * gu + up_off, dtype=torch.float16, device="cuda")
        d["w_gate"] = pair[:gu].view(cfg.inter, cfg.hidden)
        d["w_up"] = pair[gu + up_off:].view(cfg.inter, cfg.hidden)
        if c == 0 and host_layer is not None:
            for n in names:
                if n in d:
                    d[n].copy_(to_dev(host_layer[n]))
                else:
                    d[n] = to_dev(host_layer[n])
            out.append(d)
            continue
        for n in names:
            if n not in d:
                d[n] = torch.empty(shapes[n], dtype=torch.float16, device="cuda")
            d[n].normal_(0.0, cfg.sigma_w, generator=gen)
        out.append(d)
    return out


class LayerBench:
    def __init__(self, cfg, M, rotate_bytes, host_layer=None):
        import torch
        import paper_2605_25655_amd as thi
        self.thi, self.torch, self.cfg, self.M = thi, torch, cfg, M
        layer_bytes = 2 * cfg.weight_elems
        self.copies = max(1, min(8, int(-(-rotate_bytes // layer_bytes))))
        self.w = device_weights(cfg, self.copies, host_layer)
        gen = torch.Generator(device="cuda")
        gen.manual_seed(777 + cfg.index)
        H = cfg.hidden
        self.x_qkv = torch.randn((M, H), generator=gen, device="cuda", dtype=torch.float32).half()
        self.a_o = torch.randn((M, H), generator=gen, device="cuda", dtype=torch.float32).half()
        self.x_mlp = torch.randn((M, H), generator=gen, device="cuda", dtype=torch.float32).half()
        self.gamma = (1 + 0.1 * torch.randn((H,), generator=gen, device="cuda", dtype=torch.float32)).half()
        self.head_dim = 64 if cfg.index == 1 else 128
        self.n_rot = cfg.n_qkv - (cfg.n_qkv - H) // 2
        self.pos = (torch.arange(M, device="cuda", dtype=torch.int32) * 37) % 4096
        self.theta = (10000.0 ** (-torch.arange(0, self.head_dim, 2, device="cuda", dtype=torch.float64)
                                  / self.head_dim)).float()
        self.qkv = torch.empty((M, cfg.n_qkv), dtype=torch.float16, device="cuda")
        self.o = torch.empty((M, H), dtype=torch.float16, device="cuda")
        self.y = torch.empty((M, H), dtype=torch.float16, device="cuda")
        self.h = torch.empty((M, cfg.inter), dtype=torch.float16, device="cuda")
        need = max(thi.thi_workspace_bytes(0, M, cfg.n_qkv, H), thi.thi_workspace_bytes(1, M, H, H),
                   thi.thi_workspace_bytes(2, M, H, cfg.inter))
        self.ws = thi.Workspace(need)
        # The O projection alone is small (33.5 MB for the 7B shape): the rotated copies of w_o would fit the
        # 256 MB last-level cache together.  Its per-operator timing therefore also cycles through the
        # H-row blocks of the QKV matrices (same shape and layout as w_o, different values).
        self.o_mats = []
        for w in self.w:
            self.o_mats.append(w["w_o"])
            for b in range(cfg.n_qkv // H):
                self.o_mats.append(w["w_qkv"][b * H:(b + 1) * H])

    def step(self, i):
        w = self.w[i % self.copies]
        t = self.thi
        t.thi_rmsnorm_qkv(self.x_qkv, self.gamma, 1e-6, w["w_qkv"], self.qkv, self.ws)
        t.thi_linear(self.a_o, w["w_o"], self.o, self.ws)
        t.thi_swiglu_mlp(self.x_mlp, w["w_gate"], w["w_up"], w["w_down"], self.y, self.ws)

    def op(self, name, i):
        w = self.w[i % self.copies]
        t = self.thi
        if name == "rmsnorm_qkv":
            t.thi_rmsnorm_qkv(self.x_qkv, self.gamma, 1e-6, w["w_qkv"], self.qkv, self.ws)
        elif name == "rmsnorm_qkv_rope":
            t.thi_rmsnorm_qkv_rope(self.x_qkv, self.gamma, 1e-6, w["w_qkv"], self.pos, self.theta, self.n_rot,
                                   self.head_dim, self.qkv, self.ws)
        elif name == "o_proj":
            t.thi_linear(self.a_o, self.o_mats[i % len(self.o_mats)], self.o, self.ws)
        elif name == "gate_up":
            t.thi_swiglu_gate_up(self.x_mlp, w["w_gate"], w["w_up"], self.h, self.ws)
        elif name == "down":
            t.thi_linear(self.h, w["w_down"], self.y, self.ws)
        elif name == "swiglu_mlp":
            t.thi_swiglu_mlp(self.x_mlp, w["w_gate"], w["w_up"], w["w_down"], self.y, self.ws)
        elif name == "o_proj_residual":
            t.thi_linear_residual(self.a_o, self.o_mats[i % len(self.o_mats)], self.x_mlp, self.o, self.ws)
        elif name == "rmsnorm_swiglu_mlp_residual":
            t.thi_rmsnorm_swiglu_mlp(self.x_mlp, self.gamma, 1e-6, w["w_gate"], w["w_up"], w["w_down"], self.a_o,
                                     self.y, self.ws)
        else:
            raise KeyError(name)

    def time_loop(self, fn, per_block, warmup, blocks=BLOCKS):
        """ms per call of fn(i): the median over `blocks` blocks of `per_block` launches, each block between two
        HIP events on the stream the kernels are launched on (torch's current stream, which the binding
        passes to the library).  Also returns the host wall time per call and the per-block figures."""
        torch = self.torch
        for i in range(warmup):
            fn(i)
        torch.cuda.synchronize()
        per, n = [], warmup
        t0 = time.perf_counter()
        for _ in range(blocks):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(per_block):
                fn(n + i)
            e1.record()
            torch.cuda.synchronize()
            per.append(e0.elapsed_time(e1) / per_block)
            n += per_block
        wall = (time.perf_counter() - t0) * 1e3 / (blocks * per_block)
        per.sort()
        return per[len(per) // 2], wall, per


def op_bytes_flops(cfg, M, name):
    from paper_2605_25655_amd import roofline as rf
    H, I, Nq = cfg.hidden, cfg.inter, cfg.n_qkv
    if name in ("rmsnorm_qkv", "rmsnorm_qkv_rope"):
        return rf.linear_bytes(M, Nq, H, True), rf.linear_flops(M, Nq, H)
    if name in ("o_proj", "o_proj_residual"):
        return rf.linear_bytes(M, H, H), rf.linear_flops(M, H, H)
    if name == "gate_up":
        return 2.0 * (2 * I * H + M * H + M * I), 2 * rf.linear_flops(M, I, H)
    if name == "down":
        return rf.linear_bytes(M, H, I), rf.linear_flops(M, H, I)
    if name in ("swiglu_mlp", "rmsnorm_swiglu_mlp_residual"):
        return 2.0 * (3 * I * H + 2 * M * H), 3 * rf.linear_flops(M, I, H)
    raise KeyError(name)


def cpu_baseline(cfg, M, host_layer, target_seconds=12.0):
    """The fp64 oracle, as it stands, timed on this host's cores on a bounded sample of the workload:
    token rows of the same layer through all three calls.  A short calibration run sizes the sample to
    about target_seconds of CPU work (the oracle's cost is linear in rows)."""
    import numpy as np
    import oracle
    from paper_2605_25655_amd import synth
    oracle.build()
    rng = np.random.Generator(np.random.Philox(key=99))

    def run(rows):
        x = (rng.standard_normal((rows, cfg.hidden))).astype(np.float16)
        t0 = time.perf_counter()
        oracle.rmsnorm_qkv(x, host_layer["gamma"], synth.EPS, host_layer["w_qkv"])
        oracle.linear(x, host_layer["w_o"])
        oracle.swiglu_mlp(x, host_layer["w_gate"], host_layer["w_up"], host_layer["w_down"])
        return time.perf_counter() - t0

    t_small, t_big = run(4), run(20)                    # cost = fixed (weight widening) + per_row * rows
    per_row = max((t_big - t_small) / 16.0, 1e-6)
    fixed = max(t_small - 4 * per_row, 0.0)
    rows = int(max(8, min(8192, (target_seconds - fixed) / per_row)))
    dt = run(rows)
    return {"value": round(rows / dt, 2), "unit": "tokens/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"{rows} token rows of the same layer ({-(-rows // max(M, 1))} batch(es) of M={M}; all three "
                      f"calls, all output columns), {dt:.1f} s of CPU time"}


def measure_ceilings(same_bytes=None):
    """What this GPU sustains: streaming HBM read and register-only fp16 MFMA (random operands).
    same_bytes: also time the streaming read on that many bytes per launch, launched back to back the way
    the operators are timed (windows of a 2 GiB buffer in rotation): what a kernel that only reads the
    dominant kernel's bytes, and pays its own launch, gets."""
    import torch
    import paper_2605_25655_amd as thi
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    buf = torch.empty(1 << 31, dtype=torch.uint8, device="cuda").fill_(1)      # 2 GiB >> last-level cache
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    best = 0.0
    for _ in range(4):
        e0.record(); thi.thi_probe_stream_read(buf, sink); e1.record(); torch.cuda.synchronize()
        best = max(best, buf.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    out = {"hbm_stream_read_GBps": round(best, 1)}
    if same_bytes:
        nb = int(same_bytes) // 65536 * 65536
        windows = [buf[i * nb:(i + 1) * nb] for i in range(buf.numel() // nb)]
        for i in range(10):
            thi.thi_probe_stream_read(windows[i % len(windows)], sink)
        torch.cuda.synchronize()
        n = 100
        e0.record()
        for i in range(n):
            thi.thi_probe_stream_read(windows[i % len(windows)], sink)
        e1.record(); torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / n
        out["hbm_stream_read_same_bytes"] = {"bytes": nb, "us": round(us, 2), "GBps": round(nb / us / 1e3, 1)}
    del buf
    gen = torch.Generator(device="cuda"); gen.manual_seed(5)
    for name, ops in (("mfma_f16_random_operands_TFLOPs", torch.randn(32768, generator=gen, device="cuda").half()),
                      ("mfma_f16_constant_operands_TFLOPs", torch.full((32768,), 0.0625, device="cuda").half())):
        thi.thi_probe_mfma_f16(ops, 500, 256, sink); torch.cuda.synchronize()
        e0.record(); fl = thi.thi_probe_mfma_f16(ops, 20000, 256, sink); e1.record(); torch.cuda.synchronize()
        out[name] = round(fl / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    return out


def measure_layer(cfg, M, args, host_layer, per_block, warmup, op_names, traffic_kib=None):
    """Times the layer step and the named operators for one (config, M); returns the parts of the report:
    step figures, per-operator figures and the roofline object of the dominant kernel (gate/up projection with
    the fused SiLU*up epilogue, timed alone through thi_swiglu_gate_up with the same weight rotation)."""
    import torch
    from paper_2605_25655_amd import roofline as rf
    import paper_2605_25655_amd as thi

    decode = M <= 64
    lb = LayerBench(cfg, M, args.rotate_bytes, host_layer)
    ms_step, wall_ms, step_blocks = lb.time_loop(lb.step, per_block, warmup)
    layer_bytes = rf.layer_bytes(M, cfg.hidden, cfg.n_qkv, cfg.inter)
    layer_flops = rf.layer_flops(M, cfg.hidden, cfg.n_qkv, cfg.inter)
    ops = {}
    for name in op_names:
        ms, _, _ = lb.time_loop(lambda i, n=name: lb.op(n, i), per_block, max(5, warmup // 2))
        b, f = op_bytes_flops(cfg, M, name)
        ops[name] = {"us": round(ms * 1e3, 2), "GBps": round(b / (ms * 1e-3) / 1e9, 1),
                     "TFLOPs": round(f / (ms * 1e-3) / 1e12, 2)}
    gu_ms = ops["gate_up"]["us"] * 1e-3
    gu_bytes, gu_flops = op_bytes_flops(cfg, M, "gate_up")
    if decode:
        fam = thi.thi_query_kernel_family(M, cfg.inter, cfg.hidden, 2)
        roof = {"bound": "hbm",
                "kernel": f"gate_up ({ {3: 'skinny_rowslab', 4: 'skinny_rowblock'}.get(fam, 'skinny_streamk') }, SwiGLU epilogue)",
                "achieved": round(gu_bytes / (gu_ms * 1e-3) / 1e9, 1), "peak": rf.MI355X_HBM_GBS, "unit": "GB/s",
                "traffic": None}
    else:
        roof = {"bound": "mfma", "kernel": "gate_up (gemm_streamk, SwiGLU epilogue)",
                "achieved": round(gu_flops / (gu_ms * 1e-3) / 1e12, 2), "peak": rf.MI355X_FP16_TFLOPS,
                "unit": "TFLOP/s", "traffic": None}
    # HBM traffic of the dominant kernel per launch comes from separate rocprofv3 --pmc runs of this same
    # command (FETCH_SIZE, WRITE_SIZE, scaled by the --calib-copy kernel): --traffic-kib, else the committed
    # figure for this workload together with the commit it was measured at.
    src = "--traffic-kib"
    if traffic_kib is None:
        rec = committed_traffic().get(f"{cfg.index}/{M}")
        if rec:
            traffic_kib = (rec["fetch_kib"], rec["write_kib"])
            src = f"{rec['source']} (measured at commit {rec['commit']})"
    if traffic_kib is not None:
        roof["traffic"] = (traffic_kib[0] + traffic_kib[1]) * 1024
        roof["traffic_detail"] = {"fetch_bytes": traffic_kib[0] * 1024, "write_bytes": traffic_kib[1] * 1024,
                                  "algorithmic_bytes": gu_bytes, "source": src}
    roof["frac"] = round(roof["achieved"] / roof["peak"], 4)
    roof["launch_us"] = ops["gate_up"]["us"]
    part = {
        "ms_per_step": round(ms_step, 5),
        "ms_per_step_blocks": [round(v, 5) for v in step_blocks],
        "tokens_s": round(M / (ms_step * 1e-3), 1),
        "layer_GBps": round(layer_bytes / (ms_step * 1e-3) / 1e9, 1),
        "layer_hbm_frac": round(layer_bytes / (ms_step * 1e-3) / 1e9 / rf.MI355X_HBM_GBS, 4),
        "layer_TFLOPs": round(layer_flops / (ms_step * 1e-3) / 1e12, 2),
        "layer_mfma_frac": round(layer_flops / (ms_step * 1e-3) / 1e12 / rf.MI355X_FP16_TFLOPS, 4),
        "host_wall_ms_per_step": round(wall_ms, 5),
        "weight_copies_rotated": lb.copies,
        "ops": ops,
        "roofline": roof,
    }
    return lb, part, gu_bytes


def workload_name(cfg, M):
    return (f"{cfg.name} decoder-layer linear ops (rmsnorm_qkv + o_proj + swiglu_mlp), "
            f"{'decode' if M <= 64 else 'prefill'} M={M}")


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build targets ONE GPU (no collectives, no sharding); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2605_25655_amd import roofline as rf
    from paper_2605_25655_amd import synth
    import paper_2605_25655_amd as thi

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    thi.load_library()
    cfg = synth.CONFIGS[args.config]
    M = args.m
    decode = M <= 64
    host_layer = synth.make_layer(cfg, ms=())
    per_block = max(MIN_PER_BLOCK, args.steps)
    warmup = max(10, args.warmup)

    if args.calib_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)                       # 1 GiB read + 1 GiB written, a kernel of known size
        torch.cuda.synchronize()
        del src, dst
    all_ops = ("rmsnorm_qkv", "rmsnorm_qkv_rope", "o_proj", "gate_up", "down", "swiglu_mlp", "o_proj_residual",
               "rmsnorm_swiglu_mlp_residual")
    lb, head, gu_bytes = measure_layer(cfg, M, args, host_layer, per_block, warmup, all_ops, args.traffic_kib)
    roof = head["roofline"]

    out = {
        "metric": "decode layer tokens/s" if decode else "prefill layer tokens/s",
        "value": head["tokens_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 storage, f32 accumulate", "data": "synthetic (seeded random fp16 weights/activations, Llama shapes)",
        "config": {"workload": workload_name(cfg, M),
                   "hidden": cfg.hidden, "n_qkv": cfg.n_qkv, "intermediate": cfg.inter, "M": M,
                   "weight_copies_rotated": head["weight_copies_rotated"],
                   "w_up_offset_bytes": int(os.environ.get("THI_BENCH_UP_OFFSET", UP_OFFSET_BYTES))},
        "timing": {"blocks": BLOCKS, "launches_per_block": per_block, "warmup_launches": warmup,
                   "reported": "median of the blocks; HIP events on the launch stream",
                   "ms_per_step_blocks": head["ms_per_step_blocks"]},
        "layer_GBps": head["layer_GBps"],
        "layer_hbm_frac": head["layer_hbm_frac"],
        "layer_TFLOPs": head["layer_TFLOPs"],
        "layer_mfma_frac": head["layer_mfma_frac"],
        "host_wall_ms_per_step": head["host_wall_ms_per_step"],
        "ops": head["ops"],
        "roofline": roof,
    }

    # Extra: the same step replayed from a captured HIP graph (one graph launch per pass over all weight copies;
    # the paper's unified kernel scheduling, one launch per operator graph).  The eager figure above stays the
    # headline: on this GPU the gaps between dependent kernels are on the device side and a graph does not remove them.
    if decode:
        try:
            stream = torch.cuda.Stream()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(stream):
                lb.step(0)
                stream.synchronize()
                with torch.cuda.graph(graph, stream=stream):
                    for c in range(lb.copies):
                        lb.step(c)
                ms_g, _, _ = lb.time_loop(lambda i: graph.replay(), max(MIN_PER_BLOCK, per_block // lb.copies), 5)
            torch.cuda.synchronize()
            out["captured_graph"] = {"us_per_step": round(ms_g * 1e3 / lb.copies, 2), "steps_per_graph": lb.copies,
                                     "eager_us_per_step": round(head["ms_per_step"] * 1e3, 2)}
            del graph
        except Exception as e:      # reported, never fatal: the figure is an extra
            out["captured_graph"] = {"error": repr(e)[:200]}

    # Extra (not part of the step): decode attention for the same batch, every request with `--context`
    # cached positions, heads as in the Llama model of this shape.  Algorithmic bytes: K and V read once.
    if decode and args.context > 0:
        Hq, Hkv, D = {1: (8, 8, 64), 2: (32, 32, 128), 3: (40, 40, 128), 4: (52, 52, 128), 5: (64, 8, 128)}[args.config]
        S = args.context
        gen = torch.Generator(device="cuda")
        gen.manual_seed(4242)
        qa = torch.randn((M, Hq, D), generator=gen, device="cuda", dtype=torch.float32).half()
        ka = torch.randn((M, Hkv, S, D), generator=gen, device="cuda", dtype=torch.float32).half()
        va = torch.randn((M, Hkv, S, D), generator=gen, device="cuda", dtype=torch.float32).half()
        la = torch.full((M,), S, dtype=torch.int32, device="cuda")
        oa = torch.empty((M, Hq, D), dtype=torch.float16, device="cuda")
        wa = thi.Workspace(thi.thi_attention_workspace_bytes(M, Hq, Hkv, D, S), init=False)
        ms, _, _ = lb.time_loop(lambda i: thi.thi_decode_attention(qa, ka, va, la, D ** -0.5, oa, wa), MIN_PER_BLOCK, 5)
        kv_bytes = 2.0 * M * Hkv * S * D * 2
        out["decode_attention"] = {"context": S, "q_heads": Hq, "kv_heads": Hkv, "head_dim": D, "us": round(ms * 1e3, 2),
                                   "GBps": round(kv_bytes / (ms * 1e-3) / 1e9, 1),
                                   "hbm_frac": round(kv_bytes / (ms * 1e-3) / 1e9 / rf.MI355X_HBM_GBS, 4)}
        del qa, ka, va, oa, wa
    del lb
    torch.cuda.empty_cache()

    # The prefill half of the metric: TFLOP/s against the fp16 MFMA peak, per layer step and for the dominant
    # kernel, on the largest prefill workload (70B-shaped, M = 2048) and the hardest one (13B-shaped, M = 512).
    if decode and not args.no_prefill:
        legs = []
        for ci, m in ((5, 2048), (3, 512)):
            c2 = synth.CONFIGS[ci]
            lb2, part, _ = measure_layer(c2, m, args, None, MIN_PER_BLOCK, 10,
                                         ("rmsnorm_qkv", "o_proj", "gate_up", "down", "swiglu_mlp"))
            del lb2
            torch.cuda.empty_cache()
            legs.append({"workload": workload_name(c2, m), "metric": "prefill TFLOP/s vs fp16 MFMA peak",
                         "value": part["layer_TFLOPs"], "unit": "TFLOP/s", "frac_of_peak": part["layer_mfma_frac"],
                         "timing": {"blocks": BLOCKS, "launches_per_block": MIN_PER_BLOCK}, **part})
            print(f"# prefill {c2.name} M={m}: {part['ms_per_step']} ms/step, {part['layer_TFLOPs']} TFLOP/s", file=sys.stderr,
                  flush=True)
        out["prefill"] = legs

    if args.sweep:
        extra = {}
        for ci, m in ((2, 1), (2, 8), (3, 16), (3, 512), (5, 1), (5, 32), (4, 32), (4, 1024), (4, 2048), (5, 2048)):
            if (ci, m) == (args.config, M):
                continue
            c2 = synth.CONFIGS[ci]
            torch.cuda.empty_cache()
            lb = LayerBench(c2, m, args.rotate_bytes, None)
            ms, _, _ = lb.time_loop(lb.step, MIN_PER_BLOCK, 20)        # clocks ramp under load: warm up properly
            extra[f"{c2.name}/M={m}"] = {
                "ms_per_step": round(ms, 4), "tokens_s": round(m / (ms * 1e-3), 1),
                "GBps": round(rf.layer_bytes(m, c2.hidden, c2.n_qkv, c2.inter) / (ms * 1e-3) / 1e9, 1),
                "TFLOPs": round(rf.layer_flops(m, c2.hidden, c2.n_qkv, c2.inter) / (ms * 1e-3) / 1e12, 2)}
            print(f"# sweep {c2.name} M={m}: {extra[f'{c2.name}/M={m}']}", file=sys.stderr, flush=True)
            del lb
        out["sweep"] = extra

    out["ceilings"] = measure_ceilings(gu_bytes if decode else None)
    roof["attainable"] = (out["ceilings"]["hbm_stream_read_GBps"] if decode
                          else out["ceilings"]["mfma_f16_random_operands_TFLOPs"])
    roof["frac_of_attainable"] = round(roof["achieved"] / roof["attainable"], 4)
    if decode:      # against a kernel that only reads the same bytes, launch included
        roof["frac_of_read_only_kernel"] = round(out["ceilings"]["hbm_stream_read_same_bytes"]["us"] / roof["launch_us"], 4)
    for leg in out.get("prefill", []):      # the register-only MFMA probe beside each prefill roofline
        r2 = leg["roofline"]
        r2["attainable"] = out["ceilings"]["mfma_f16_random_operands_TFLOPs"]
        r2["frac_of_attainable"] = round(r2["achieved"] / r2["attainable"], 4)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, M, host_layer)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
