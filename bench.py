#!/usr/bin/env python3
"""Benchmark of the MTAD/MMTAD hot path on one MI355X.

A step = one whole iteration of the method (gamma beam steps on the draft model, tree build,
one target pass, accept, KV commit) over one batch of synthetic input.  Default workload: C3
(7B-shaped bf16 target, 512-token prompt, gamma 4, beam 4).  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import synth_inputs as si  # noqa: E402

HBM_PEAK_GBS = 8000.0


def weight_bytes(shape):
    """Bytes of the matrices one pass streams: every layer matrix and the unembedding, once."""
    e = 2 if shape.dtype == "bf16" else 4
    d, f = shape.d_model, shape.d_ffn
    per_layer = shape.qkv_rows * d + d * shape.n_heads * shape.head_dim + 2 * f * d + d * f
    return (shape.n_layers * per_layer + shape.vocab * d) * e


def kv_bytes_per_token(shape):
    e = 2 if shape.dtype == "bf16" else 4
    return 2 * shape.n_layers * shape.n_kv_heads * shape.head_dim * e


def target_gemm_shapes(shape):
    d, f = shape.d_model, shape.d_ffn
    per_layer = [(shape.qkv_rows, d), (d, shape.n_heads * shape.head_dim), (2 * f, d), (d, f)]
    return per_layer, (shape.vocab, d)


class PowerSampler:
    """Board power from the amdgpu hwmon sensor (microwatts), sampled by a thread; energy = trapezoid integral."""

    def __init__(self, hz=20.0):
        import glob
        import threading
        paths = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input")) + \
            sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average"))
        self.path = paths[0] if paths else None
        self.dt = 1.0 / hz
        self.samples = []
        self._stop = threading.Event()
        self._thread = threading.Thread(target=self._run, daemon=True)

    def _read(self):
        with open(self.path) as f:
            return float(f.read().strip()) * 1e-6

    def _run(self):
        while not self._stop.is_set():
            try:
                self.samples.append((time.perf_counter(), self._read()))
            except (OSError, ValueError):
                pass
            self._stop.wait(self.dt)

    def __enter__(self):
        self.samples = []
        self.t0 = time.perf_counter()
        if self.path:
            self.samples.append((self.t0, self._read()))
            self._thread.start()
        return self

    def __exit__(self, *exc):
        self.t1 = time.perf_counter()
        self._stop.set()
        if self.path:
            self._thread.join()
            self.samples.append((self.t1, self._read()))

    def joules(self):
        s = self.samples
        return sum((b[0] - a[0]) * (a[1] + b[1]) / 2 for a, b in zip(s, s[1:]))


def measure_energy(eng, w, tau, prompt, tm, dm, Engine, torch, dev, seconds=3.0):
    """Joules per iteration of MTAD, vanilla speculative decoding and plain decoding: each runs for about `seconds` while the
    board power sensor is sampled at 20 Hz."""
    if PowerSampler().path is None:
        return {"error": "no power sensor under /sys/class/drm/card*/device/hwmon"}

    def run(step, tokens_of, n_probe=5):
        for _ in range(n_probe):
            step()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(n_probe):
            step()
        torch.cuda.synchronize()
        n = max(20, int(seconds / max((time.perf_counter() - t) / n_probe, 1e-4)))
        n0 = tokens_of()
        with PowerSampler() as ps:
            for _ in range(n):
                step()
            torch.cuda.synchronize()
        toks = tokens_of() - n0
        e = ps.joules()
        return {"iterations": n, "seconds": round(ps.t1 - ps.t0, 3), "mean_W": round(e / (ps.t1 - ps.t0), 1),
                "J_per_iteration": round(e / n, 4), "tokens": toks, "J_per_token": round(e / max(toks, 1), 4),
                "power_samples": len(ps.samples)}

    cap = lambda n_it, per: w.prompt_len + (n_it + 16) * per + 64
    # sized for the longest run: iterations are a few milliseconds, so a 3 s run is at most ~2000 of them
    n_max = 2500
    out = {"sensor": PowerSampler().path, "sample_hz": 20, "seconds_per_method": seconds}
    e1 = Engine(tm, dm, batch=w.batch, gamma=w.gamma, beam=w.beam, mode=w.mode, max_context=cap(n_max, w.gamma + 1), device=dev)
    e1.prefill(prompt)
    out["mtad"] = run(lambda: e1.iteration(tau, seed=w.seed), lambda: int(e1.tkv.len.sum().item()))
    e1.prefill(prompt)
    out["autoregressive"] = run(lambda: e1.iteration_autoregressive(seed=w.seed), lambda: int(e1.tkv.len.sum().item()))
    e1.close()
    e2 = Engine(tm, dm, batch=w.batch, gamma=w.gamma, beam=1, mode="mtad", max_context=cap(n_max, w.gamma + 1), device=dev)
    e2.prefill(prompt)
    out["speculative_decoding"] = run(lambda: e2.iteration_spd(seed=w.seed), lambda: int(e2.tkv.len.sum().item()))
    e2.close()
    out["projection"] = {
        "J_per_token_mtad": round(out["mtad"]["J_per_iteration"] / w.batch / 3.17, 4),
        "J_per_token_speculative_decoding": round(out["speculative_decoding"]["J_per_iteration"] / w.batch / 2.02, 4),
        "J_per_token_autoregressive": round(out["autoregressive"]["J_per_iteration"] / w.batch, 4),
        "note": "joules per iteration / the tokens per iteration the paper reports for its Llama-2 pair (MTAD 3.17, SpD 2.02): a "
                "projection; the measured J_per_token above are for independent random models (about one token per iteration)"}
    return out


def layer_weight_bytes(shape):
    e = 2 if shape.dtype == "bf16" else 4
    d, f = shape.d_model, shape.d_ffn
    return (shape.qkv_rows * d + d * shape.n_heads * shape.head_dim + 3 * f * d) * e


def pass_kernel_name(w, one_launch):
    rows = w.batch * w.tree_rows
    if w.target.dtype != "bf16":
        return "gemm_f32_kernel (+ attention kernels): one launch per product"
    if one_launch:
        return f"flow_pass_kernel<{w.target.head_dim}> (one launch = the whole target pass)"
    return ("gemm_bf16_strips_kernel / gemm_bf16_kernel" if rows <= 8 else "gemm_bf16_multi_kernel / gemm_bf16_kernel" if rows < 65 else
            "gemm_bf16_tiled_kernel") + " (+ tree_attn_mfma_kernel): one launch per product"


def verify_block(eng, w, K, torch, stream):
    """One target pass over the tree rows (the verify step), timed with HIP events on the launch stream."""
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for _ in range(3):
        eng.verify_phase()
    ev[0].record(stream)
    for _ in range(K):
        eng.verify_phase()
    ev[1].record(stream)
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / K
    n_ctx = int(eng.tkv.len[0].item())
    nbytes = weight_bytes(w.target) + w.batch * n_ctx * kv_bytes_per_token(w.target)
    return ms, nbytes, {"ms": round(ms, 4), "context": n_ctx, "rows": w.batch * w.tree_rows,
                        "algorithmic_GB": round(nbytes / 1e9, 4), "GBps": round(nbytes / ms / 1e6, 1),
                        "frac_of_hbm_peak": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4)}


def workload_block(w, K, W, threads, dev, mb, torch, DeviceModel, Engine):
    """Compact figures of one workload on its own seeded weights: tokens/s of the whole loop and the verify step."""
    t0 = time.time()
    tm = DeviceModel(w.target, lambda n: si.make_tensor(w.target, w.seed, "target", n), dev, threads=threads)
    dm = DeviceModel(w.draft, lambda n: si.make_tensor(w.draft, w.seed, "draft", n), dev, threads=threads)
    t_weights = time.time() - t0
    prompt = si.make_prompt(w)
    eng = Engine(tm, dm, batch=w.batch, gamma=w.gamma, beam=w.beam, mode=w.mode,
                 max_context=w.prompt_len + (K + W + 8) * (w.gamma + 1) + w.tree_rows + 64, device=dev)
    stream = torch.cuda.current_stream()
    res = {}
    for key, tau in (("tau", w.tau), ("tau0", 0.0)):
        eng.prefill(prompt)
        for _ in range(W):
            eng.iteration(tau, seed=w.seed)
        torch.cuda.synchronize()
        len0 = eng.tkv.len.clone()
        t = time.perf_counter()
        for _ in range(K):
            eng.iteration(tau, seed=w.seed)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t
        tokens = int((eng.tkv.len - len0).sum().item())
        res[key] = {"tokens_per_s": round(tokens / dt, 2), "tokens_per_iteration": round(tokens / K / w.batch, 3),
                    "ms_per_step": round(dt / K * 1e3, 4)}
    eng.prefill(prompt)
    eng.draft_phase(seed=w.seed)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev[0].record(stream)
    for _ in range(K):
        eng.draft_phase(seed=w.seed)
    ev[1].record(stream)
    torch.cuda.synchronize()
    draft_ms = ev[0].elapsed_time(ev[1]) / K
    _, _, verify = verify_block(eng, w, K, torch, stream)
    one_launch = w.target.dtype == "bf16" and w.batch * w.tree_rows <= 8 and layer_weight_bytes(w.target) >= (64 << 20)
    out = {"workload": f"{w.mode.upper()} gamma={w.gamma} beam={w.beam} batch={w.batch} prompt={w.prompt_len}, target "
                       f"L{w.target.n_layers} d{w.target.d_model} {w.target.dtype}, draft L{w.draft.n_layers} d{w.draft.d_model}; seed {w.seed}",
           "steps": K, "tau": w.tau, "value": res["tau"]["tokens_per_s"], "unit": "tokens/s",
           "ms_per_step": res["tau"]["ms_per_step"], "tokens_per_iteration": res["tau"]["tokens_per_iteration"],
           "iterations_per_s": round(1e3 / res["tau"]["ms_per_step"], 2), "tau0": res["tau0"],
           "draft_phase_ms": round(draft_ms, 4), "verify": verify, "pass_kernels": pass_kernel_name(w, one_launch),
           "weights_setup_s": round(t_weights, 1), "device_status": mb.mtad_device_status(eng.ctx)}
    eng.close()
    del eng, tm, dm
    torch.cuda.empty_cache()
    return out


def gemm_replay_block(w, tm, eng, rows, dt_id, mb, torch, stream, dev, K):
    """The products of one target pass launched back to back on zero activations, each by the pass's own kernel choice."""
    per_layer, head = target_gemm_shapes(w.target)
    esz = 2 if dt_id else 4
    kmax = max(k for _, k in per_layer + [head])
    nmax = max(n for n, _ in per_layer + [head])
    x_order = mb.MTAD_X_FRAGMENTS if (dt_id and rows >= 2) else mb.MTAD_X_PLANES   # as the kernel-per-step passes keep their activations
    X = torch.zeros(2 * ((rows + 7) // 8 * 8) * kmax, dtype=torch.int16 if dt_id else torch.float32, device=dev)
    Y = torch.zeros(rows * nmax, dtype=torch.float32, device=dev)
    launches = []
    for l in range(w.target.n_layers):
        for j, idx in enumerate((1, 2, 4, 5)):
            n, k = per_layer[j]
            launches.append((tm.tensors[1 + 6 * l + idx], n, k))
    launches.append((tm.tensors[-1], head[0], head[1]))
    gemm_bytes = sum(n * k * esz + rows * k * 4 + rows * n * 4 for _, n, k in launches)

    def replay():
        for Wt, n, k in launches:
            mb.mtad_k_gemm(dt_id, Wt, X, Y, rows, n, k, n, False, ctx=eng.ctx, x_order=x_order)
    replay()
    reps = max(3, min(20, K // 3))
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev[0].record(stream)
    for _ in range(reps):
        replay()
    ev[1].record(stream)
    torch.cuda.synchronize()
    gemm_ms = ev[0].elapsed_time(ev[1]) / (reps * len(launches))
    bpl = gemm_bytes / len(launches)
    out = {"kernels": "gemm_f32_kernel" if not dt_id else pass_kernel_name(w, False).split(" (+")[0],
           "launches": len(launches), "bytes_per_launch": int(bpl), "avg_launch_us": round(gemm_ms * 1e3, 3),
           "GBps": round(bpl / gemm_ms / 1e6, 1), "frac_of_hbm_peak": round(bpl / gemm_ms / 1e6 / HBM_PEAK_GBS, 4)}
    tfile = os.path.join(ROOT, "profiles", "c3_gemm_hbm_traffic.txt")
    if w.name == "C3" and os.path.exists(tfile):
        kv = dict(l.strip().split("=", 1) for l in open(tfile) if "=" in l and not l.startswith("#"))
        out["hbm_bytes_per_launch"] = int(float(kv["fetch_bytes_per_launch"])) + int(float(kv["write_bytes_per_launch"]))
        out["hbm_bytes_source"] = "profiles/c3_gemm_hbm_counters.md"
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C3")
    ap.add_argument("--tau", type=float, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--others", default=None, help="comma-separated workloads that get a compact block (tokens/s and verify step) "
                    "beside the main one; default: the other four of C1..C5 when the main workload is C3, else none")
    ap.add_argument("--no-baselines", action="store_true", help="skip plain decoding and vanilla speculative decoding")
    ap.add_argument("--no-gemm-replay", action="store_true", help="skip the back-to-back replay of the product kernels")
    ap.add_argument("--no-energy", action="store_true", help="skip the board-power measurement (about 10 s)")
    ap.add_argument("--batch-sweep", default="1,2,4", help="comma-separated batch sizes: time and energy of one target pass at each "
                    "(Section 4's observation that a run costs about the same for any small batch); '' skips it")
    ap.add_argument("--gamma-beam-sweep", default="", help="'g1,g2,..xb1,b2,..': time of one iteration at each draft length gamma and beam "
                    "width (the axes of the paper's ablation, Section 5.3); not part of the default run")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (requests are independent; more GPUs would each run this "
              "same path on their own share of the requests). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2407_09722_amd import binding as mb
    from paper_2407_09722_amd.engine import DeviceModel, Engine
    mb.lib()                                            # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    w = si.WORKLOADS[args.workload]
    tau = w.tau if args.tau is None else args.tau
    K, W = args.steps, args.warmup
    threads = min(16, os.cpu_count() or 8)

    t0 = time.time()
    tm = DeviceModel(w.target, lambda n: si.make_tensor(w.target, w.seed, "target", n), dev, threads=threads)
    dm = DeviceModel(w.draft, lambda n: si.make_tensor(w.draft, w.seed, "draft", n), dev, threads=threads)
    t_weights = time.time() - t0
    prompt = si.make_prompt(w)
    M = w.tree_rows
    total_iters = 3 * (K + W) + 8
    max_ctx = w.prompt_len + total_iters * (w.gamma + 1) + M + 64
    eng = Engine(tm, dm, batch=w.batch, gamma=w.gamma, beam=w.beam, mode=w.mode, max_context=max_ctx, device=dev)
    stream = torch.cuda.current_stream()

    def timed_region(tau_run, sample_beam=False):
        """W warm-up + K timed iterations from a fresh prefill; returns (seconds, tokens, mean context)."""
        eng.prefill(prompt)
        for _ in range(W):
            eng.iteration(tau_run, sample_beam=sample_beam, seed=w.seed)
        torch.cuda.synchronize()
        len0 = eng.tkv.len.clone()
        t = time.perf_counter()
        for _ in range(K):
            eng.iteration(tau_run, sample_beam=sample_beam, seed=w.seed)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t
        len1 = eng.tkv.len.clone()
        tokens = int((len1 - len0).sum().item())           # every committed token lengthens the cache by one
        n_mean = float((len0.float().mean().item() + len1.float().mean().item()) / 2)
        return dt, tokens, n_mean

    dt, tokens, n_mean = timed_region(tau)
    status = mb.mtad_device_status(eng.ctx)
    dt0, tokens0, _ = timed_region(0.0)                  # tau = 0 passes every prefix: gamma+1 tokens per iteration
    status |= mb.mtad_device_status(eng.ctx)
    # the paper's experimental setting (appendix "Hyper-parameter Details"): both models' distributions warped to the top
    # 10 tokens and the top-p 0.9 prefix, stochastic beam sampling (extra figure; `value` stays the unwarped loop)
    mb.mtad_set_warp(eng.ctx, 10, 0.9)
    dtw, tokensw, _ = timed_region(tau, sample_beam=True)
    mb.mtad_set_warp(eng.ctx, 0, 0.0)
    status |= mb.mtad_device_status(eng.ctx)
    warped = {"setting": "top-k 10 then top-p 0.9 on both models, stochastic beam sampling, tau %.2g" % tau,
              "tokens_per_s": round(tokensw / dtw, 2), "tokens_per_iteration": round(tokensw / (K * w.batch), 3),
              "ms_per_step": round(dtw / K * 1e3, 4)}

    # --- the same K iterations replayed from a HIP graph of one iteration (extra figure; `value` stays the eager loop) ----
    graph_info = None
    try:
        eng.prefill(prompt)
        for _ in range(W):
            eng.iteration(tau, seed=w.seed)
        torch.cuda.synchronize()
        g = eng.capture_iteration(tau, seed=w.seed)
        g.replay()
        torch.cuda.synchronize()
        len0 = eng.tkv.len.clone()
        t = time.perf_counter()
        for _ in range(K):
            g.replay()
        torch.cuda.synchronize()
        dtg = time.perf_counter() - t
        tok_g = int((eng.tkv.len - len0).sum().item())
        graph_info = {"ms_per_step": round(dtg / K * 1e3, 4), "tokens_per_s": round(tok_g / dtg, 2)}
        del g
    except Exception as e:                                  # reported, never fatal: the eager loop is the measurement
        graph_info = {"error": str(e)[:200]}
    status |= mb.mtad_device_status(eng.ctx)

    # --- verify step alone, HIP events on the launch stream --------------------------------------------------
    eng.prefill(prompt)
    eng.draft_phase(seed=w.seed)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    verify_ms, verify_bytes, verify = verify_block(eng, w, K, torch, stream)

    # --- roofline of the dominant kernel, in the pass: for bf16 passes of at most 8 rows over layers of at least 64 MiB the
    #     whole target pass is ONE launch (flow_pass_kernel: every product and the attention of all layers), so bytes per launch
    #     = the verify step's algorithmic bytes and the launch's duration = the verify step's (HIP events on the launch stream;
    #     the interval also holds the embedding and log-sum-exp kernels of the pass, a few microseconds)
    rows = w.batch * M
    dt_id = 1 if w.target.dtype == "bf16" else 0
    one_launch = bool(dt_id) and rows <= 8 and layer_weight_bytes(w.target) >= (64 << 20)
    traffic, traffic_detail = None, None
    tfile = os.path.join(ROOT, "profiles", f"{w.name.lower()}_verify_hbm_traffic.txt")
    if os.path.exists(tfile):                          # per-pass HBM bytes from the committed rocprofv3 counter runs
        kv = dict(l.strip().split("=", 1) for l in open(tfile) if "=" in l and not l.startswith("#"))
        traffic_detail = {"fetch_bytes_per_launch": int(float(kv["fetch_bytes_per_launch"])),
                          "write_bytes_per_launch": int(float(kv["write_bytes_per_launch"])),
                          "source": kv.get("source", "profiles/")}
        traffic = traffic_detail["fetch_bytes_per_launch"] + traffic_detail["write_bytes_per_launch"]
    roofline = {"kernel": pass_kernel_name(w, one_launch),
                "bound": "hbm", "achieved": verify["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": verify["frac_of_hbm_peak"], "traffic": traffic, "traffic_detail": traffic_detail,
                "bytes_per_launch": int(verify_bytes), "avg_launch_us": round(verify_ms * 1e3, 2),
                "launches_per_verify": 1 if one_launch else None,
                "scope": "in the pass: all bytes of one target pass (weights once, the KV cache of the context once) over the pass's "
                         "duration" + ("" if one_launch else "; the pass is a sequence of kernels, the figure is their total")}

    # --- extra: the weight-streaming product kernels alone, launched back to back outside a pass (upper bound of what the pass
    #     can reach: no dependencies between launches, activations zero) ----------------------------------------------------
    gemm_replay = None
    if not args.no_gemm_replay:
        gemm_replay = gemm_replay_block(w, tm, eng, rows, dt_id, mb, torch, stream, dev, K)

    # --- the other workloads: tokens/s and verify step of each, on its own weights -------------------------------------------
    others = {}
    names = args.others.split(",") if args.others is not None else ([n for n in si.WORKLOADS if n != w.name] if w.name == "C3" else [])
    for name in [n for n in names if n]:
        others[name] = workload_block(si.WORKLOADS[name], min(K, 20), min(W, 3), threads, dev, mb, torch, DeviceModel, Engine)
        status |= others[name].pop("device_status")

    # --- plain copy of known size: reference for byte counters and for the bandwidth coalesced traffic reaches -----
    cbytes = 1 << 30
    src = torch.empty(cbytes, dtype=torch.uint8, device=dev)
    dst = torch.empty(cbytes, dtype=torch.uint8, device=dev)
    src.fill_(1)
    mb.mtad_k_copy(src, dst, cbytes)
    ev[0].record(stream)
    for _ in range(5):
        mb.mtad_k_copy(src, dst, cbytes)
    ev[1].record(stream)
    torch.cuda.synchronize()
    copy_ms = ev[0].elapsed_time(ev[1]) / 5
    copy_ref = {"bytes_read": cbytes, "bytes_written": cbytes, "ms": round(copy_ms, 4),
                "GBps_read_plus_write": round(2 * cbytes / copy_ms / 1e6, 1)}
    del src, dst

    # --- the baselines of Section 2.2 on the same kernels: plain decoding with the target alone, vanilla speculative decoding ---
    baselines = None
    if not args.no_baselines:
        eng.prefill(prompt)
        for _ in range(W):
            eng.iteration_autoregressive(seed=w.seed)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(K):
            eng.iteration_autoregressive(seed=w.seed)
        torch.cuda.synchronize()
        dta = time.perf_counter() - t
        status |= mb.mtad_device_status(eng.ctx)
        engs = Engine(tm, dm, batch=w.batch, gamma=w.gamma, beam=1, mode="mtad", max_context=w.prompt_len + (K + W) * (w.gamma + 1) + 64,
                      device=dev)
        engs.prefill(prompt)
        for _ in range(W):
            engs.iteration_spd(seed=w.seed)
        torch.cuda.synchronize()
        len0 = engs.tkv.len.clone()
        t = time.perf_counter()
        for _ in range(K):
            engs.iteration_spd(seed=w.seed)
        torch.cuda.synchronize()
        dts = time.perf_counter() - t
        toks = int((engs.tkv.len - len0).sum().item())
        status |= mb.mtad_device_status(engs.ctx)
        engs.close()
        # multi-token joint decoding: the beam search runs on the target itself (its weights serve as the "draft" of a second engine)
        engj = Engine(tm, tm, batch=w.batch, gamma=w.gamma, beam=w.beam, mode="mtad", max_context=w.prompt_len + (K + W + 2) * w.gamma + 64,
                      device=dev)
        engj.prefill(prompt)
        for _ in range(min(W, 2)):
            engj.iteration_mtjd(seed=w.seed)
        torch.cuda.synchronize()
        Kj = max(3, K // 4)
        t = time.perf_counter()
        for _ in range(Kj):
            engj.iteration_mtjd(seed=w.seed)
        torch.cuda.synchronize()
        dtj = time.perf_counter() - t
        status |= mb.mtad_device_status(engj.ctx)
        engj.close()
        it_s = K / dt
        baselines = {
            "autoregressive": {"tokens_per_s": round(K * w.batch / dta, 2), "ms_per_token": round(dta / K * 1e3, 4)},
            "speculative_decoding": {"tokens_per_s": round(toks / dts, 2), "tokens_per_iteration": round(toks / K / w.batch, 3),
                                     "ms_per_step": round(dts / K * 1e3, 4), "gamma": w.gamma},
            "multi_token_joint_decoding": {"tokens_per_s": round(Kj * w.gamma * w.batch / dtj, 2), "tokens_per_step": w.gamma,
                                           "ms_per_step": round(dtj / Kj * 1e3, 4), "beam": w.beam,
                                           "note": "beam sampling on the target itself (Section 3.1): the quality reference MTAD approximates"},
            "projection": {"mtad_over_spd": round((it_s * 3.17) / (K / dts * 2.02), 3),
                           "mtad_over_autoregressive": round((it_s * 3.17) / (K / dta), 3),
                           "note": "iterations/s of each method x the tokens per iteration the paper reports for its Llama-2 pair "
                                   "(appendix, block-efficiency table: MTAD 3.17, SpD 2.02); the measured tokens/s above are for "
                                   "independent random models, which accept almost nothing"},
        }

    # --- energy per token (the paper's second headline, Section 5 "energy consumption"): board power from the driver's sensor,
    #     sampled while each method runs for a few seconds, integrated over the run
    energy = None
    if not args.no_energy and baselines is not None:
        energy = measure_energy(eng, w, tau, prompt, tm, dm, Engine, torch, dev)

    # --- one target pass at several batch sizes (Section 4: the time and energy of a run barely depend on a small batch) ---------
    batch_sweep = None
    if args.batch_sweep:
        batch_sweep = []
        for nb in [int(x) for x in args.batch_sweep.split(",") if x]:
            if nb * M > 256:
                batch_sweep.append({"batch": nb, "error": "more than 256 rows in a pass"})
                continue
            eb = Engine(tm, dm, batch=nb, gamma=w.gamma, beam=w.beam, mode=w.mode, max_context=w.prompt_len + 64, device=dev,
                        prefill_rows=max(M, min(64, 256 // nb)))
            eb.prefill(np.repeat(prompt[:1], nb, axis=0))
            eb.draft_phase(seed=w.seed)
            for _ in range(3):
                eb.verify_phase()
            torch.cuda.synchronize()
            n_it = max(50, int(1.0 / (verify_ms * 1e-3)))
            with PowerSampler() as ps:
                for _ in range(n_it):
                    eb.verify_phase()
                torch.cuda.synchronize()
            sec = ps.t1 - ps.t0
            batch_sweep.append({"batch": nb, "rows": nb * M, "ms_per_pass": round(sec / n_it * 1e3, 4),
                                "J_per_pass": round(ps.joules() / n_it, 4) if ps.path else None,
                                "ms_per_pass_per_sequence": round(sec / n_it * 1e3 / nb, 4)})
            eb.close()

    # --- one iteration at several draft lengths and beam widths (Section 5.3 varies both; its speed peaks where the growing
    #     draft and verify cost overtakes the longer accepted blocks) -------------------------------------------------------
    gb_sweep = None
    if args.gamma_beam_sweep:
        gs, bs = (tuple(int(x) for x in part.split(",") if x) for part in args.gamma_beam_sweep.split("x"))
        gb_sweep = []
        for g in gs:
            for b in bs:
                rows = w.batch * ((g + 1) if w.mode == "mtad" else (b * g + 1))
                if (g + 1) + (g - 1) * b > 64 or rows > 256:   # the library's limits (include/mtad.h: MTAD_MAX_ROWS)
                    gb_sweep.append({"gamma": g, "beam": b, "error": "more than 64 draft rows per iteration or 256 rows per pass"})
                    continue
                eg = Engine(tm, dm, batch=w.batch, gamma=g, beam=b, mode=w.mode, max_context=w.prompt_len + 256, device=dev)
                eg.prefill(prompt)
                for i in range(3):
                    eg.iteration(tau, seed=w.seed + i)
                n_it = 20
                ev[0].record(stream)
                for i in range(n_it):
                    eg.draft_phase(seed=w.seed + i)
                ev[1].record(stream)
                for i in range(n_it):
                    eg.iteration(tau, seed=w.seed + 100 + i)
                ev[2].record(stream)
                torch.cuda.synchronize()
                gb_sweep.append({"gamma": g, "beam": b, "verify_rows": rows, "ms_per_iteration": round(ev[1].elapsed_time(ev[2]) / n_it, 4),
                                 "ms_draft_phase": round(ev[0].elapsed_time(ev[1]) / n_it, 4)})
                status |= mb.mtad_device_status(eg.ctx)
                eg.close()

    # --- the oracle on the host cores, bounded sample ---------------------------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(w, tau)

    out = {
        "metric": "accepted tokens/sec (1 GPU)", "value": round(tokens / dt, 2), "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(dt / K * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.target.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.mode.upper()} gamma={w.gamma} beam={w.beam} batch={w.batch} "
                               f"prompt={w.prompt_len}, target L{w.target.n_layers} d{w.target.d_model} "
                               f"ffn{w.target.d_ffn} V{w.target.vocab}, draft L{w.draft.n_layers} d{w.draft.d_model}; "
                               f"random-init weights seed {w.seed}",
                   "tau": tau, "tokens_per_iteration": round(tokens / K / w.batch, 3), "mean_context": round(n_mean, 1),
                   "beam_search": "deterministic top-b", "bonus_token": "sampled (Gumbel-argmax)"},
        "iterations_per_s": round(K / dt, 2),
        "projection": {"tokens_per_s": round(K / dt * w.batch * 3.17, 1),
                       "note": "iterations/s x 3.17, the block efficiency the paper reports for its Llama-2 pair (appendix, "
                               "block-efficiency table): a labelled projection, not a measurement"},
        "tau0": {"tokens_per_s": round(tokens0 / dt0, 2), "tokens_per_iteration": round(tokens0 / K / w.batch, 3),
                 "ms_per_step": round(dt0 / K * 1e3, 4)},
        "warped": warped, "baselines": baselines, "energy": energy, "batch_sweep": batch_sweep, "gamma_beam_sweep": gb_sweep, "graph_replay": graph_info, "verify": verify, "roofline": roofline, "gemm_replay": gemm_replay, "workloads": others, "copy_reference": copy_ref, "cpu_baseline": cpu,
        "device_status": status, "weights_setup_s": round(t_weights, 1),
    }
    print(json.dumps(out))


def cpu_baseline(w, tau):
    """The oracle as it stands, timed on this host: full iterations of the method at the workload's real widths
    with a shortened context and the target cut to 2 and to 4 layers; the difference prices one layer and the
    full depth is extrapolated.  A reported baseline, not a target."""
    import threadpoolctl  # noqa: F401
    from oracle import mtad
    from oracle.lm import CachedSession, DecoderLM
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
    ctx_len, iters = 64, 2
    L_full = w.target.n_layers
    L_hi = min(4, L_full)
    L_lo = min(2, L_hi)
    shape_hi = w.target.with_layers(L_hi)
    wt = si.make_weights(shape_hi, w.seed, "target", threads=cores)
    wd = si.make_weights(w.draft, w.seed, "draft", threads=cores)
    lm_q = DecoderLM(w.draft, wd)
    prompt = si.make_prompt(w)[0, :ctx_len]
    times, emitted = {}, 0
    for L in sorted({L_lo, L_hi}):
        lm_p = DecoderLM(w.target.with_layers(L), {k: v for k, v in wt.items() if not k.startswith("L") or int(k.split(".")[0][1:]) < L})
        sq, sp = CachedSession(lm_q, list(prompt)), CachedSession(lm_p, list(prompt))
        mtad.iteration(sq, sp, gamma=w.gamma, beam=w.beam, mode=w.mode, tau=tau, seed=w.seed)      # includes the prompt pass
        t = time.perf_counter()
        for _ in range(iters):
            tr = mtad.iteration(sq, sp, gamma=w.gamma, beam=w.beam, mode=w.mode, tau=tau, seed=w.seed)
            emitted += len(tr["emitted"])
        times[L] = (time.perf_counter() - t) / iters
    per_layer = (times[L_hi] - times[L_lo]) / max(1, L_hi - L_lo) if L_hi > L_lo else times[L_hi] / L_hi
    t_full = times[L_lo] + per_layer * (L_full - L_lo)
    tok_per_iter = emitted / (iters * len(times))
    return {"value": round(w.batch * tok_per_iter / (t_full * w.batch), 4), "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"{iters} full iterations (draft beam search + target pass + accept) of one sequence at the real widths and "
                      f"vocabulary, context {ctx_len}, target cut to {L_lo} and {L_hi} layers; per-layer time from the difference, "
                      f"extrapolated to {L_full} layers: {t_full:.2f} s per iteration (numpy float64)",
            "s_per_iteration_extrapolated": round(t_full, 3)}


if __name__ == "__main__":
    main()
