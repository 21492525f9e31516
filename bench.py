#!/usr/bin/env python3
"""Benchmark of the decoder-layer linear-operator hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input:
thi_rmsnorm_qkv, thi_linear (O projection) and thi_swiglu_mlp enqueued
back-to-back on one stream.  Default workload: the Llama-7B-shaped layer at
decode M=32 (the configuration the metric is quoted on).  Weight copies are
rotated between steps so that the 256 MB last-level cache cannot serve them.

Prints ONE JSON line (see README for the fields).
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


# per-launch HBM KiB (fetch, write) of the gate/up kernel, scaled, from the rocprofv3 --pmc runs in profiles/
MEASURED_TRAFFIC_KIB = {
    (2, 32): ((178861.0, 928.0), "profiles/skinny_rowblock_llama7b_decode_m32.txt"),
    (5, 2048): ((2770494.0, 115073.0), "profiles/gemm_streamk_llama70b_prefill_m2048.txt"),
}


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
    ap.add_argument("--calib-copy", action="store_true",
                    help="run one plain 1 GiB device copy before the timed region (scales rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--traffic-kib", type=float, nargs=2, default=None, metavar=("FETCH", "WRITE"),
                    help="per-launch HBM KiB of the dominant kernel from rocprofv3 --pmc runs, already scaled; reported as roofline.traffic")
    return ap.parse_args()


def device_weights(cfg, copies, host_layer):
    """copies of the layer's weights on the device: copy 0 is the seeded host layer,
    the others are seeded device draws with the same distribution."""
    import torch
    from tests.gpu_common import to_dev
    names = ("w_qkv", "w_o", "w_gate", "w_up", "w_down")
    shapes = {"w_qkv": (cfg.n_qkv, cfg.hidden), "w_o": (cfg.hidden, cfg.hidden), "w_gate": (cfg.inter, cfg.hidden),
              "w_up": (cfg.inter, cfg.hidden), "w_down": (cfg.hidden, cfg.inter)}
    out = []
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20260525 + 100 * cfg.index)
    for c in range(copies):
        if c == 0 and host_layer is not None:
            out.append({n: to_dev(host_layer[n]) for n in names})
            continue
        d = {}
        for n in names:
            t = torch.empty(shapes[n], dtype=torch.float16, device="cuda")
            t.normal_(0.0, cfg.sigma_w, generator=gen)
            d[n] = t
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

    def time_loop(self, fn, steps, warmup):
        """ms per call of fn(i): HIP events on the stream the kernels are launched on."""
        torch = self.torch
        for i in range(warmup):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for i in range(steps):
            fn(warmup + i)
        e1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / steps
        return e0.elapsed_time(e1) / steps, wall


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
    lb = LayerBench(cfg, M, args.rotate_bytes, host_layer)

    if args.calib_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)                       # 1 GiB read + 1 GiB written, a kernel of known size
        torch.cuda.synchronize()
        del src, dst
    ms_step, wall_ms = lb.time_loop(lb.step, args.steps, args.warmup)
    tokens_s = M / (ms_step * 1e-3)
    layer_bytes = rf.layer_bytes(M, cfg.hidden, cfg.n_qkv, cfg.inter)
    layer_flops = rf.layer_flops(M, cfg.hidden, cfg.n_qkv, cfg.inter)

    ops = {}
    for name in ("rmsnorm_qkv", "rmsnorm_qkv_rope", "o_proj", "gate_up", "down", "swiglu_mlp", "o_proj_residual",
                 "rmsnorm_swiglu_mlp_residual"):
        ms, _ = lb.time_loop(lambda i, n=name: lb.op(n, i), max(20, args.steps // 2), max(5, args.warmup // 2))
        b, f = op_bytes_flops(cfg, M, name)
        ops[name] = {"us": round(ms * 1e3, 2), "GBps": round(b / (ms * 1e-3) / 1e9, 1),
                     "TFLOPs": round(f / (ms * 1e-3) / 1e12, 2)}

    # roofline of the dominant kernel: the gate/up projection with the fused SiLU*up epilogue
    gu_ms = ops["gate_up"]["us"] * 1e-3
    gu_bytes, gu_flops = op_bytes_flops(cfg, M, "gate_up")
    if decode:
        fam = thi.thi_query_kernel_family(M, cfg.inter, cfg.hidden, 2)
        roof = {"bound": "hbm",
                "kernel": f"gate_up ({ {3: 'skinny_rowslab', 4: 'skinny_rowblock'}.get(fam, 'skinny_streamk') }, SwiGLU epilogue)",
                "achieved": round(gu_bytes / (gu_ms * 1e-3) / 1e9, 1), "peak": rf.MI355X_HBM_GBS, "unit": "GB/s",
                "traffic": None}
    else:
        roof = {"bound": "mfma", "kernel": "gate_up (gemm, SwiGLU epilogue)",
                "achieved": round(gu_flops / (gu_ms * 1e-3) / 1e12, 2), "peak": rf.MI355X_FP16_TFLOPS,
                "unit": "TFLOP/s", "traffic": None}
    # HBM traffic of the dominant kernel per launch comes from separate rocprofv3 --pmc runs of this same
    # command (FETCH_SIZE, WRITE_SIZE, scaled by the --calib-copy kernel).  For the two profiled workloads
    # the committed figures are used unless --traffic-kib gives fresher ones.
    traffic_kib, traffic_src = args.traffic_kib, "--traffic-kib"
    if traffic_kib is None and (args.config, M) in MEASURED_TRAFFIC_KIB:
        traffic_kib, traffic_src = MEASURED_TRAFFIC_KIB[(args.config, M)]
    if traffic_kib is not None:
        # HBM bytes per launch (reads + writes); the parts and where they come from next to it
        roof["traffic"] = (traffic_kib[0] + traffic_kib[1]) * 1024
        roof["traffic_detail"] = {"fetch_bytes": traffic_kib[0] * 1024, "write_bytes": traffic_kib[1] * 1024,
                                  "algorithmic_bytes": gu_bytes, "source": traffic_src}
    roof["frac"] = round(roof["achieved"] / roof["peak"], 4)
    roof["launch_us"] = ops["gate_up"]["us"]

    out = {
        "metric": "decode layer tokens/s" if decode else "prefill layer tokens/s",
        "value": round(tokens_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 storage, f32 accumulate", "data": "synthetic (seeded random fp16 weights/activations, Llama shapes)",
        "config": {"workload": f"{cfg.name} decoder-layer linear ops (rmsnorm_qkv + o_proj + swiglu_mlp), "
                               f"{'decode' if decode else 'prefill'} M={M}",
                   "hidden": cfg.hidden, "n_qkv": cfg.n_qkv, "intermediate": cfg.inter, "M": M,
                   "weight_copies_rotated": lb.copies},
        "layer_GBps": round(layer_bytes / (ms_step * 1e-3) / 1e9, 1),
        "layer_hbm_frac": round(layer_bytes / (ms_step * 1e-3) / 1e9 / rf.MI355X_HBM_GBS, 4),
        "layer_TFLOPs": round(layer_flops / (ms_step * 1e-3) / 1e12, 2),
        "layer_mfma_frac": round(layer_flops / (ms_step * 1e-3) / 1e12 / rf.MI355X_FP16_TFLOPS, 4),
        "host_wall_ms_per_step": round(wall_ms, 5),
        "ops": ops,
        "roofline": roof,
    }

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
        ms, _ = lb.time_loop(lambda i: thi.thi_decode_attention(qa, ka, va, la, D ** -0.5, oa, wa),
                             max(20, args.steps // 2), max(5, args.warmup // 2))
        kv_bytes = 2.0 * M * Hkv * S * D * 2
        out["decode_attention"] = {"context": S, "q_heads": Hq, "kv_heads": Hkv, "head_dim": D, "us": round(ms * 1e3, 2),
                                   "GBps": round(kv_bytes / (ms * 1e-3) / 1e9, 1),
                                   "hbm_frac": round(kv_bytes / (ms * 1e-3) / 1e9 / rf.MI355X_HBM_GBS, 4)}
        del qa, ka, va, oa, wa

    if args.sweep:
        extra = {}
        for ci, m in ((2, 1), (2, 8), (3, 16), (3, 512), (5, 1), (5, 32), (4, 1024), (5, 2048)):
            if (ci, m) == (args.config, M):
                continue
            c2 = synth.CONFIGS[ci]
            del lb
            torch.cuda.empty_cache()
            lb = LayerBench(c2, m, args.rotate_bytes, None)
            steps = max(50, min(args.steps, int(2e11 / (2.0 * m * c2.weight_elems + 2e8))))
            ms, _ = lb.time_loop(lb.step, steps, 20)        # clocks ramp under load: warm up properly
            extra[f"{c2.name}/M={m}"] = {
                "ms_per_step": round(ms, 4), "tokens_s": round(m / (ms * 1e-3), 1),
                "GBps": round(rf.layer_bytes(m, c2.hidden, c2.n_qkv, c2.inter) / (ms * 1e-3) / 1e9, 1),
                "TFLOPs": round(rf.layer_flops(m, c2.hidden, c2.n_qkv, c2.inter) / (ms * 1e-3) / 1e12, 2)}
            print(f"# sweep {c2.name} M={m}: {extra[f'{c2.name}/M={m}']}", file=sys.stderr, flush=True)
        out["sweep"] = extra

    out["ceilings"] = measure_ceilings(gu_bytes if decode else None)
    roof["attainable"] = (out["ceilings"]["hbm_stream_read_GBps"] if decode
                          else out["ceilings"]["mfma_f16_random_operands_TFLOPs"])
    roof["frac_of_attainable"] = round(roof["achieved"] / roof["attainable"], 4)
    if decode:      # against a kernel that only reads the same bytes, launch included
        roof["frac_of_read_only_kernel"] = round(out["ceilings"]["hbm_stream_read_same_bytes"]["us"] / roof["launch_us"], 4)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, M, host_layer)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
