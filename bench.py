#!/usr/bin/env python3
"""Benchmark of the streamed training step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config auto|tiny|1.3B|7B|14B|7B-128k]
                    [--second-config auto|none|NAME] [--overlap-check] [--copy-calibration]

A "step" is one pass of the whole hot path over one synthetic batch: mt_train_step
(weight streaming, forward, loss, per-block recompute + backward, gradient offload)
and the host Adam update of every parameter (which also refreshes the streamed bf16 copy).  By default
this is one call, mt_train_step_adam, which runs each unit's update on host threads as soon as its
gradients have landed; --separate-adam times mt_train_step followed by mt_adam_step instead.  Inputs are
resident in host memory, as the method prescribes, when the timed region starts; every step gets a fresh seeded
batch.  The default run (no --config) measures the 7B workload and then, under the key "second_workload", 1 + 3
steps of the 14B workload, the second configuration the metric is quoted on.

Prints ONE JSON line.  `value` is model TFLOP/s by the paper's accounting (6ND + 12LHT^2,
recompute not counted).  `roofline` is for the dominant kernel class (the MFMA GEMM unless
attention dominates), measured live with HIP events on the compute stream inside the timed
region.  `cpu_baseline` is the CPU oracle (fp32 build) timed on a bounded sample of the same
layer shapes on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from dataclasses import replace

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16, published
SAMPLE_TOKENS = {"tiny": 256, "1.3B": 2048, "7B": 1024, "14B": 768, "7B-128k": 1024, "7B-256k": 1024, "7B-512k": 1024}


def mem_available_gb() -> float:
    try:
        for line in open("/proc/meminfo"):
            if line.startswith("MemAvailable:"):
                return int(line.split()[1]) / 1e6
    except OSError:
        pass
    return 0.0


def host_bytes_needed(n_params: int) -> float:
    # caller fp32 master 4 + grads 4 + m 4 + v 4 + bf16 copy 2 bytes per parameter
    return 18.0 * n_params


def pick_config(name: str):
    import mt_inputs
    if name != "auto":
        return name
    # the metric is quoted at 7B and 14B; 7B is the default when the host can hold its state
    need = host_bytes_needed(mt_inputs.n_params(mt_inputs.CONFIGS["7B"][0])) / 1e9
    return "7B" if mem_available_gb() > need + 24 else "1.3B"


def cpu_baseline(name: str) -> dict:
    """The oracle as it stands (fp32 build) on a bounded sample: same layer shapes, one or two blocks,
    one short sequence; reported in the metric's unit (model TFLOP/s by the same formula)."""
    import mt_inputs
    import oracle
    import paper_2604_05091_amd as mt
    oracle.build()
    shape, _, T = {**mt_inputs.CONFIGS, **mt_inputs.LONG_CONTEXT}[name]
    Ls = 2 if name in ("tiny", "1.3B") else 1
    Ts = min(T, SAMPLE_TOKENS[name])
    Bs = 2 if name == "tiny" else 1
    s1 = replace(shape, n_layers=Ls)
    params = mt_inputs.make_params(s1, seed=0)
    tok, lab = mt_inputs.make_batch(s1.vocab, Bs, Ts, seed=1)
    orc = oracle.Oracle("f32")
    t0 = time.time()
    loss, grads = orc.train_step(s1, params, tok, lab, mode=1)
    for p, g in zip(params, grads):
        m, v = p * 0, p * 0
        orc.adam(p, g, m, v, 1e-4, 0.9, 0.999, 1e-8, 0.0, 1)
    dt = time.time() - t0
    flops = mt.model_flops(mt_inputs.n_params(s1), Ls, s1.hidden, Bs, Ts)
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count())),
            "kind": "oracle",
            "sample": f"{name} layer shapes, {Ls} block(s), batch {Bs} x seq {Ts}, fp32 oracle step + Adam, "
                      f"{dt:.2f} s, loss {loss:.4f}"}


def gemm_source_hash() -> str:
    import hashlib
    return hashlib.sha256(open(os.path.join(ROOT, "paper_2604_05091_amd", "csrc", "gemm.hip"), "rb").read()).hexdigest()[:16]


def measured_traffic(name: str, dom: int):
    """HBM-side bytes per launch of the dominant kernel from the rocprofv3 --pmc summary under profiles/ (FETCH_SIZE,
    WRITE_SIZE, scaled by a copy of known size).  The summary names the hash of the GEMM source it was measured on;
    when the source has changed since, the figure no longer belongs to the kernel that was timed and null is reported."""
    tpath = os.path.join(ROOT, "profiles", "gemm_kernels_7B_hbm_traffic.md")
    if dom != 0 or not os.path.exists(tpath):
        return None, "no counter summary for this kernel class and workload"
    import re
    text = open(tpath).read()
    m = re.search(r"traffic_bytes_per_launch\[%s\] = ([0-9.eE+]+)" % re.escape(name), text)
    if not m:
        return None, "no counter summary for this workload"
    hm = re.search(r"gemm_source_sha256_16 = ([0-9a-f]+)", text)
    if not hm or hm.group(1) != gemm_source_hash():
        return None, "profiles/gemm_kernels_7B_hbm_traffic.md was measured on an older csrc/gemm.hip"
    return float(m.group(1)), "profiles/gemm_kernels_7B_hbm_traffic.md (same csrc/gemm.hip)"


def run_workload(name: str, steps: int, warmup: int, args, flags: int = 0, adam: bool = True, quiet: bool = False) -> dict:
    """Create a handle for the workload, run warmup + steps on fresh seeded batches, return the measurements."""
    import gc
    import numpy as np
    import mt_inputs
    import paper_2604_05091_amd as mt
    shape, B, T = {**mt_inputs.CONFIGS, **mt_inputs.LONG_CONTEXT}[name]
    n_params = mt_inputs.n_params(shape)
    t_setup = time.time()
    params = mt_inputs.make_params(shape, seed=0)
    # a fresh batch for every step (stream_id = step number), generated before the timed region: the timed steps
    # never see a batch the model has already been updated on
    batches = [mt_inputs.make_batch(shape.vocab, B, T, seed=1, stream_id=i) for i in range(warmup + steps)]
    cfg = mt.ModelCfg.make(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.ffn,
                           shape.vocab, B, T, rope_base=shape.rope_base, rms_eps=shape.rms_eps,
                           flags=(0 if args.no_kernel_timing else mt.FLAG_KERNEL_TIMING) | args.flags | flags,
                           ckpt_interval=args.ckpt_interval, mlp_chunk=args.mlp_chunk)
    link = mt.link_probe(256 << 20, 4)     # copy-bandwidth probe of this session: the host-link roofline
    h = mt.TrainHandle(cfg, params)
    t_setup = time.time() - t_setup
    if not quiet:
        print(f"[bench] {name}: {n_params/1e9:.3f} B params, batch {B} x seq {T}, setup {t_setup:.1f} s, "
              f"link probe {link}", file=sys.stderr, flush=True)

    lr, step_no = 1e-4, 0
    losses = []

    def one_step(n):
        tok, lab = batches[n - 1]
        if not adam:
            loss = h.train_step(tok, lab)
            st = h.stats()
        elif args.separate_adam:
            loss = h.train_step(tok, lab)
            st = h.stats()
            h.adam_step(lr, step=n)
            st["adam_ms"] = h.stats()["adam_ms"]
        else:
            loss = h.train_step_adam(tok, lab, lr, step=n)
            st = h.stats()
        return loss, st

    for _ in range(warmup):
        step_no += 1
        losses.append(one_step(step_no)[0])
        if not quiet:
            print(f"[bench] warmup step {step_no} loss {losses[-1]:.4f}", file=sys.stderr, flush=True)
    mt.device_synchronize()
    per_step = []
    t0 = time.perf_counter()
    for _ in range(steps):
        step_no += 1
        loss, st = one_step(step_no)
        losses.append(loss)
        per_step.append(st)
        if not quiet:
            print(f"[bench] step {step_no} loss {losses[-1]:.4f} train {st['step_ms']:.0f} ms adam {st['adam_ms']:.0f} ms",
                  file=sys.stderr, flush=True)
    mt.device_synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / steps

    flops = mt.model_flops(n_params, shape.n_layers, shape.hidden, B, T)
    mean = lambda k: float(np.mean([s[k] for s in per_step]))
    cls_ms = np.sum([s["class_ms"] for s in per_step], axis=0)
    cls_fl = np.sum([s["class_flops"] for s in per_step], axis=0)
    cls_n = np.sum([s["class_launches"] for s in per_step], axis=0)
    cls_by = np.sum([s["class_bytes"] for s in per_step], axis=0)
    names = ["gemm_nt_w4e_kernel<*> + gemm_tn_w4e_kernel<*> (bf16 MFMA GEMM)", "flash_fwd_kernel", "flash_bwd_dkdv_kernel + flash_bwd_dq_kernel"]
    dom = int(np.argmax(cls_ms))
    achieved = cls_fl[dom] / (cls_ms[dom] * 1e-3) / 1e12 if cls_ms[dom] > 0 else 0.0
    traffic, traffic_note = measured_traffic(name, dom)
    roofline = {"bound": "mfma", "kernel": names[dom], "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": traffic, "traffic_source": traffic_note,
                "launches_per_step": int(cls_n[dom] / steps),
                "avg_launch_ms": float(cls_ms[dom] / max(cls_n[dom], 1)),
                "algorithmic_bytes_per_launch": float(cls_by[dom] / max(cls_n[dom], 1)),
                "algorithmic_flops_per_launch": float(cls_fl[dom] / max(cls_n[dom], 1)),
                "share_of_compute_busy": float(cls_ms[dom] / steps / max(mean("compute_busy_ms"), 1e-9)),
                "classes": {names[i]: {"ms_per_step": float(cls_ms[i] / steps),
                                       "tflops": float(cls_fl[i] / max(cls_ms[i] * 1e-3, 1e-12) / 1e12)}
                            for i in range(3)}}
    h2d_busy, d2h_busy = mean("h2d_busy_ms"), mean("d2h_busy_ms")
    link_stats = {
        "probe_h2d_gbs": link["h2d_gbs"], "probe_d2h_gbs": link["d2h_gbs"], "probe_bidir_gbs": link["bidir_gbs"],
        "h2d_gb_per_step": mean("h2d_bytes") / 1e9, "d2h_gb_per_step": mean("d2h_bytes") / 1e9,
        "h2d_achieved_gbs": mean("h2d_bytes") / 1e6 / max(h2d_busy, 1e-9),
        "d2h_achieved_gbs": mean("d2h_bytes") / 1e6 / max(d2h_busy, 1e-9),
        "h2d_hidden_frac": mean("h2d_hidden_ms") / max(h2d_busy, 1e-9),
        "d2h_hidden_frac": mean("d2h_hidden_ms") / max(d2h_busy, 1e-9),
        "link_hidden_frac": (mean("h2d_hidden_ms") + mean("d2h_hidden_ms")) / max(h2d_busy + d2h_busy, 1e-9),
    }
    out = {
        "value": flops / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s",
        "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "config": {"workload": f"{name}: {shape.n_layers} layers, hidden {shape.hidden}, {shape.n_q_heads}/"
                               f"{shape.n_kv_heads} heads x {shape.head_dim}, ffn {shape.ffn}, vocab {shape.vocab}, "
                               f"batch {B} x seq {T}", "n_params": n_params, "tokens_per_step": B * T,
                   "host_state": "fp32 master/grad/Adam on host, bf16 streamed weights",
                   "batches": "a fresh seeded batch every step",
                   "ckpt_interval": args.ckpt_interval, "mlp_chunk": args.mlp_chunk},
        "roofline": roofline,
        "train_step_ms": mean("step_ms"), "adam_step_ms": mean("adam_ms"),
        "train_only_tflops": (flops / (mean("step_ms") * 1e-3) / 1e12) if (args.separate_adam or not adam) else None,
        "compute_busy_ms": mean("compute_busy_ms"),
        "link": link_stats,
        "device_arena_gb": per_step[-1]["device_arena_bytes"] / 1e9,
        "host_pinned_gb": per_step[-1]["host_pinned_bytes"] / 1e9,
        "loss_first": losses[0], "loss_last": losses[-1],
    }
    h.close()
    del h, params, batches
    gc.collect()
    return out


def overlap_check(name: str, args) -> dict:
    """The train step alone (no optimizer) in four schedules: pipelined, every copy and unit followed by a device
    synchronisation, kernels only, copies only.  1 - (T_pipelined - T_compute_only) / T_copy_only is the share of the
    link time that the pipeline hides, measured without any event arithmetic."""
    import paper_2604_05091_amd as mt
    res = {}
    for key, fl in (("pipelined", 0), ("serial", mt.FLAG_SERIAL), ("compute_only", mt.FLAG_COMPUTE_ONLY),
                    ("copy_only", mt.FLAG_COPY_ONLY)):
        r = run_workload(name, 2, 1, args, flags=fl, adam=False, quiet=True)
        res[key + "_ms"] = r["train_step_ms"]
        if key == "pipelined":
            res["pipelined_event_hidden_frac"] = r["link"]["link_hidden_frac"]
            res["pipelined_compute_busy_ms"] = r["compute_busy_ms"]
        print(f"[bench] overlap check, {key}: train step {r['train_step_ms']:.0f} ms", file=sys.stderr, flush=True)
    res["hidden_frac_by_difference"] = 1.0 - max(0.0, res["pipelined_ms"] - res["compute_only_ms"]) / max(res["copy_only_ms"], 1e-9)
    res["serial_slowdown"] = res["serial_ms"] / res["pipelined_ms"]
    return res


def copy_calibration() -> int:
    """A plain device-to-device copy of known size (1 GiB read, 1 GiB written, three times) for scaling the
    FETCH_SIZE / WRITE_SIZE counters of `rocprofv3 --pmc`; torch only holds the two buffers."""
    import torch
    n = 1 << 30
    src = torch.full((n,), 1, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"copy_bytes_read": n, "copy_bytes_written": n, "dispatches": 3}))
    return 0


def gemm_occupancy_probe() -> int:
    """One round of 256 x 256 GEMM tiles on 32, 128 and 256 of the 256 CUs (and 16 rounds on all of them) for five
    reduction lengths: the slope over K is the time of one 64-deep k-step of the kernel, the intercept its fixed cost
    per tile.  The same kernel on an eighth of the chip is not held back by the chip's power limit; torch only holds
    the buffers.  MT_GEMM_VARIANT=6 sends every grid to the large-grid kernel."""
    os.environ["MT_GEMM_VARIANT"] = "6"
    import torch
    import paper_2604_05091_amd as mt
    L = mt.lib()
    out = []
    for (M, N) in ((2048, 1024), (4096, 2048), (8192, 2048), (65536, 4096)):
        tiles = (M // 256) * (N // 256)
        rounds = max(1.0, tiles / 256)
        pts = []
        for K in (512, 1024, 2048, 4096, 8192):
            g = torch.Generator(device="cuda").manual_seed(K + tiles)
            A = torch.randn((M, K), device="cuda", generator=g).to(torch.bfloat16)
            B = torch.randn((N, K), device="cuda", generator=g).to(torch.bfloat16)
            C = torch.empty((M, N), device="cuda", dtype=torch.bfloat16)
            run = lambda: L.mt_k_gemm_nt(A.data_ptr(), K, B.data_ptr(), K, C.data_ptr(), N, None, 0, M, N, K, 0, 0, None)
            if run() != 0:
                raise RuntimeError("mt_k_gemm_nt failed")
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                run()
            e1.record()
            torch.cuda.synchronize()
            pts.append((K, e0.elapsed_time(e1) / 20 / rounds * 1e3))
            del A, B, C
        (k1, t1), (k2, t2) = pts[1], pts[-1]
        step_us = (t2 - t1) / (k2 - k1) * 64
        out.append({"tiles": tiles, "cus_busy": min(tiles, 256), "us_per_round": {str(k): round(t, 2) for k, t in pts},
                    "us_per_k_step": round(step_us, 3), "fixed_us_per_tile": round(t1 - step_us * k1 / 64, 2),
                    "mfma_rate_of_peak_in_loop": round(64 * 32 / 2.4e3 / step_us, 3)})
    print(json.dumps({"gemm_occupancy_probe": out}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="auto")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--second-config", default="auto",
                    help="auto: after the default 7B run, also 1 + 3 steps of the 14B workload (the metric's second "
                         "configuration) when the host has room for its state; none; or a workload name")
    ap.add_argument("--flags", type=int, default=0, help="extra MT_FLAG_* bits (diagnostics)")
    ap.add_argument("--mlp-chunk", type=int, default=0, help="chunked MLP: tokens per chunk (0 = off)")
    ap.add_argument("--ckpt-interval", type=int, default=1,
                    help="checkpoint interval K of Algorithm 1 (the headline number is quoted at K = 1)")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="diagnostic: no HIP event pairs around the GEMM / attention launches (the roofline object is then empty)")
    ap.add_argument("--separate-adam", action="store_true",
                    help="call mt_train_step then mt_adam_step instead of the overlapped mt_train_step_adam")
    ap.add_argument("--overlap-check", action="store_true",
                    help="also time the train step pipelined / serial / kernels only / copies only (four more handles)")
    ap.add_argument("--gemm-occupancy-probe", action="store_true",
                    help="run only the GEMM kernel on 32 / 128 / 256 CUs over five K (k-step time and fixed cost per tile)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a 1 GiB device copy, three times (counter calibration under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        return 2
    if args.copy_calibration:
        return copy_calibration()
    if args.gemm_occupancy_probe:
        return gemm_occupancy_probe()

    import mt_inputs
    import paper_2604_05091_amd as mt
    # The library owns its device memory and streams; torch is deliberately not imported here, so the
    # HIP runtime in use is the system one that the library was linked against.
    mt.lib()  # fail loudly if the extension is not built
    if mt.device_count() < 1:
        print("bench.py: no GPU visible; the HIP library has no CPU fallback", file=sys.stderr)
        return 3

    name = pick_config(args.config)
    res = run_workload(name, args.steps, args.warmup, args)
    out = {
        "metric": "sustained model TFLOPS per step (6ND + 12LHT^2; train step + host Adam)",
        "adam": "separate call" if args.separate_adam else "overlapped per unit (mt_train_step_adam)",
        "value": res.pop("value"), "unit": res.pop("unit"),
        "n_gpus": 1, "steps": res.pop("steps"), "warmup": res.pop("warmup"), "ms_per_step": res.pop("ms_per_step"),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
    }
    out.update(res)
    if args.overlap_check:
        out["overlap_check"] = overlap_check(name, args)
    second = args.second_config
    if second == "auto":
        second = "none"
        if args.config == "auto" and name == "7B":
            need = host_bytes_needed(mt_inputs.n_params(mt_inputs.CONFIGS["14B"][0])) / 1e9
            if mem_available_gb() > need + 16:
                second = "14B"
            else:
                out["second_workload"] = {"skipped": f"14B needs {need:.0f} GB of host memory, {mem_available_gb():.0f} GB available"}
    if second != "none":
        r2 = run_workload(second, 3, 1, args)
        out["second_workload"] = {k: r2[k] for k in ("value", "unit", "steps", "warmup", "ms_per_step", "config", "roofline",
                                                      "adam_step_ms", "compute_busy_ms", "link", "device_arena_gb",
                                                      "host_pinned_gb", "loss_first", "loss_last")}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(name)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
