#!/usr/bin/env python3
"""Benchmark of the generation phase: `python bench.py --gpus 1 --steps K --warmup W`.

A step is one whole generation job (he_generate: prompt pass + G-1 KV-cached
decode steps + sampling) of the headline workload -- an OPT-13B-shaped actor,
batch 32, 256 prompt tokens, 256 generated tokens, bf16 weights with random
init, seeded Gumbel-max sampling.  All inputs are synthetic and resident in
HBM before the timed region.  Prints ONE JSON line: generated tokens/s, plus
`roofline` (the dominant decode kernel against the 8 TB/s HBM peak, its
duration taken live with HIP events) and `cpu_baseline` (the CPU oracle timed
on a bounded sample of the same workload).
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

HBM_PEAK = 8.0e12        # B/s, MI355X published
MFMA_BF16_PEAK = 2.5e15  # FLOP/s dense bf16, MI355X published


def algorithmic_bytes(d, fp8=False):
    """Bytes the method itself must move per decode step (weights once for the whole
    batch; K/V of every cached position read, the new position written).  With 8-bit layer
    matrices: one byte per weight plus a float scale per row."""
    H, F, L, V = d.hidden, d.ffn, d.n_layers, d.vocab
    wbytes = 2 * (L * (4 * H * H + 2 * H * F + 9 * H + F) + 2 * H + V * H)
    if fp8:
        wbytes = L * (4 * H * H + 2 * H * F) + L * 4 * (5 * H + F) + 2 * (L * (9 * H + F) + 2 * H + V * H)
    kvtok = L * 2 * H * 2
    return wbytes, kvtok


def measured_traffic(workload, kernel_class, fp8):
    """HBM bytes per launch of a decode kernel class from the tracked counter summary
    profiles/decode_kernels_traffic.txt (lines: workload class fetch_bytes write_bytes), or (None, None)."""
    if fp8:
        return None, None
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "decode_kernels_traffic.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) >= 4 and not line.startswith("#") and f[0] == workload and f[1] == kernel_class:
                return float(f[2]) + float(f[3]), "profiles/decode_kernels_traffic.txt"
    except OSError:
        pass
    return None, None


def prefill_flops(d):
    H, F, L, V, B, S = d.hidden, d.ffn, d.n_layers, d.vocab, d.batch, d.prompt_len
    return 2 * B * S * L * (4 * H * H + 2 * H * F) + L * B * 2 * S * S * H + 2 * B * V * H


def cpu_baseline(d, seconds_hint=20.0):
    """The oracle, as it stands, on a bounded sample of the workload: 2 of L layers,
    4 of B sequences, the full prompt, 3 decode steps; extrapolated linearly in
    layers, batch and steps to the whole job."""
    import numpy as np
    from oracle import opt_oracle as O
    from paper_2308_01320_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    Ls, Bs, steps = min(2, d.n_layers), min(4, d.batch), 3
    ds = d.sliced(n_layers=Ls, batch=Bs, max_positions=d.prompt_len + steps + 1)
    w = synth.make_weights(ds, seed=1)
    w = {k: (v.astype(np.float64) if k != "layers" else [{n: a.astype(np.float64) for n, a in lw.items()} for lw in v])
         for k, v in w.items()}
    w["lm_head"] = w["tok_emb"]
    prompts = synth.make_prompts(ds, seed=2)
    dec = O.CachedDecoder(w, ds.n_heads, ds.ln_eps, ds.pos_offset)
    t0 = time.perf_counter()
    z = dec.prefill(prompts)
    t_prefill = time.perf_counter() - t0
    t0 = time.perf_counter()
    for n in range(steps):
        tok = O.sample(z, d.sampling, 1.0, 42, n)[0]
        z = dec.step(tok)
    t_step = (time.perf_counter() - t0) / steps
    # the head (final LayerNorm + LM head + sampling) does not scale with layers
    x = np.zeros((Bs, 1, ds.hidden))
    t0 = time.perf_counter()
    zz = O.lm_logits(w, x, ds.ln_eps)
    O.sample(zz[:, 0, :], d.sampling, 1.0, 42, 0)
    t_head = time.perf_counter() - t0
    scale_l, scale_b = d.n_layers / Ls, d.batch / Bs
    full = scale_b * ((max(t_prefill - t_head, 0.0) * scale_l + t_head) +
                      (d.gen_len - 1) * (max(t_step - t_head, 0.0) * scale_l + t_head))
    return {"value": d.batch * d.gen_len / full, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{Ls} of {d.n_layers} layers, {Bs} of {d.batch} sequences, prompt {d.prompt_len}, "
                      f"{steps} decode steps; extrapolated linearly in layers, batch and steps",
            "measured_s": {"prefill": t_prefill, "decode_step": t_step, "head": t_head}}

class ClockSampler:
    """Samples the GPU's engine and memory clock levels while the timed region runs.

    Reads the amdgpu driver's text files under /sys (plain file reads from a thread of this process: no
    child process, no tool); where they are absent or unreadable the record says so.
    """

    def __init__(self, period_s=0.1):
        import glob
        import threading
        self.files = {}
        for card in sorted(glob.glob("/sys/class/drm/card[0-9]*/device")):
            if os.path.exists(os.path.join(card, "pp_dpm_sclk")):
                self.files = {"sclk": os.path.join(card, "pp_dpm_sclk"), "mclk": os.path.join(card, "pp_dpm_mclk"),
                              "level": os.path.join(card, "power_dpm_force_performance_level")}
                break
        self.period, self.samples, self.stop = period_s, {"sclk": [], "mclk": []}, threading.Event()
        self.thread = threading.Thread(target=self._run, daemon=True)

    @staticmethod
    def _current_mhz(path):
        try:
            for line in open(path).read().splitlines():
                if line.rstrip().endswith("*"):
                    return int("".join(ch for ch in line.split(":")[1] if ch.isdigit()))
        except (OSError, ValueError, IndexError):
            pass
        return None

    def _run(self):
        while not self.stop.is_set():
            for k in ("sclk", "mclk"):
                v = self._current_mhz(self.files[k])
                if v is not None:
                    self.samples[k].append(v)
            self.stop.wait(self.period)

    def start(self):
        if self.files:
            self.thread.start()
        return self

    def finish(self):
        self.stop.set()
        if self.files:
            self.thread.join()

    def record(self):
        if not self.files:
            return {"source": "amdgpu sysfs files not present", "sclk_mhz": None, "mclk_mhz": None}
        out = {"source": "amdgpu pp_dpm_sclk / pp_dpm_mclk, sampled during the timed region"}
        for k in ("sclk", "mclk"):
            v = sorted(self.samples[k])
            out[k + "_mhz"] = {"min": v[0], "median": v[len(v) // 2], "max": v[-1], "samples": len(v)} if v else None
        try:
            out["performance_level"] = open(self.files["level"]).read().strip()
        except OSError:
            out["performance_level"] = None
        return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="opt-13b", help="tiny | opt-1.3b | opt-6.7b | opt-13b | opt-66b")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (a reduced model: not the headline number)")
    ap.add_argument("--batch", type=int, default=0, help="override the batch (a batch sweep: not the headline number)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-score", action="store_true", help="skip the scoring pass measured after the timed region")
    ap.add_argument("--weights-tiled", action="store_true",
                    help="hand the engine pre-tiled matrices (no second copy); implied by opt-66b")
    ap.add_argument("--weights-fp8", action="store_true",
                    help="8-bit (E4M3) layer matrices: a second workload, not the headline number")
    ap.add_argument("--timing-steps", type=int, default=32,
                    help="decode steps run with per-kernel HIP events, spread evenly over the answer's contexts")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no cross-GPU sharding or collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2308_01320_amd import binding, synth

    d = synth.CONFIGS[args.workload]
    if args.layers:
        d = d.sliced(n_layers=args.layers)
    if args.batch:
        d = d.sliced(batch=args.batch)
    if d.dtype != "bf16":
        raise SystemExit("bench.py times the bf16 workloads; the tiny f32 configuration is a parity case")
    B, S, G = d.batch, d.prompt_len, d.gen_len
    H, F = d.hidden, d.ffn
    torch.cuda.set_device(0)
    stream = torch.cuda.Stream()  # default priority; the engine captures its decode step on it
    tiled = args.weights_tiled or d.name == "opt-66b"
    weights = synth.device_weights(d, torch, tile=binding.he_tile_matrix if tiled else None)
    torch.cuda.synchronize()
    cfg = binding.make_config(d, stream=stream.cuda_stream, weights_tiled=1 if tiled else 0,
                              weights_fp8=1 if args.weights_fp8 else 0)
    eng = binding.Engine(cfg, weights)
    prompts = torch.from_numpy(synth.make_prompts(d, seed=1234 + 3)).cuda()
    samp = binding.sampling(d.sampling, 1.0, 42)
    out_ids = torch.empty(B, G, dtype=torch.int32, device="cuda")
    out_lp = torch.empty(B, G, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()

    with torch.cuda.stream(stream):
        for _ in range(args.warmup):
            eng.he_generate(prompts, G, samp, out_ids, out_lp)
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        clocks = ClockSampler().start()
        t0 = time.perf_counter()
        ev0.record(stream)
        for _ in range(args.steps):
            eng.he_generate(prompts, G, samp, out_ids, out_lp)
        ev1.record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        clocks.finish()
        dev_ms = ev0.elapsed_time(ev1)
        # the timed work produced real tokens: ids in range, finite negative log-probs
        assert int(out_ids.min()) >= 0 and int(out_ids.max()) < d.vocab, "generated ids out of range"
        assert bool(torch.isfinite(out_lp).all()) and float(out_lp.max()) <= 0.0, "log-probs not finite"

        ms_per_step = wall * 1e3 / args.steps

        # split of one job: prompt pass (he_prefill) and the decode loop, HIP events on the same stream
        e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        eng.he_reset()
        e0.record(stream)
        ids, _, _ = eng.he_prefill(prompts, samp)
        e1.record(stream)
        torch.cuda.synchronize()
        prefill_ms = e0.elapsed_time(e1)
        decode_ms = dev_ms / args.steps - prefill_ms

        # Per-kernel durations of the decode step, live, with HIP events around every launch.  The job's decode steps
        # see contexts S+1 .. S+G-1, and attention's launch grows with the context, so the timed steps are spread
        # evenly over the whole answer (the other steps just run).
        nt = max(1, min(args.timing_steps, G - 1))
        timed_steps = sorted({1 + int((i + 0.5) * (G - 1) / nt) for i in range(nt)} & set(range(1, G)))
        timing = {k: [0.0, 0] for k in binding.KERNEL_CLASSES}
        timed_contexts = []
        for n in range(1, G):
            timed = n in timed_steps
            if timed:
                eng.he_timing_enable(True)
            ids, _, _ = eng.he_decode_step(ids, samp)
            if timed:
                for k, (ms, cnt) in eng.he_timing_read().items():
                    timing[k][0] += ms
                    timing[k][1] += cnt
                eng.he_timing_enable(False)
                timed_contexts.append(S + n)  # cached positions the step's attention reads
        torch.cuda.synchronize()
        # launch duration of each weight-streaming GEMM class without the per-launch cost of an event pair: one pair
        # around a sweep that launches the class once per layer (each launch streams a different layer's matrix, as
        # in a decode step); the median of five sweeps, one alone moves by a few per cent with the clocks
        sweep_reps = 4
        sweep_us = {}
        for cls in ("out_proj", "fc1", "fc2"):
            try:
                eng.he_kernel_sweep(cls, 1)  # warm
                runs = []
                for _ in range(5):
                    s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    s0.record(stream)
                    eng.he_kernel_sweep(cls, sweep_reps)
                    s1.record(stream)
                    torch.cuda.synchronize()
                    runs.append(s0.elapsed_time(s1) * 1e3 / (sweep_reps * d.n_layers))
                sweep_us[cls] = {"median": sorted(runs)[len(runs) // 2], "runs": runs}
            except binding.HeError as err:
                # no sweep for this combination (8-bit matrices at more than 32 sequences decode through
                # several kernels per GEMM): the per-launch event pairs of the decode steps above stand in
                if err.status != binding.HE_ERR_STATE:
                    raise
        # the scoring pass that follows generation: prompt + answer, all positions at once
        score = None
        if not args.no_score and S + G <= cfg.max_seq_len and S + G <= d.max_positions:
            seq = torch.cat([prompts, out_ids], dim=1).contiguous()
            sc_out = torch.empty(B, S + G - 1, dtype=torch.float32, device="cuda")
            eng.he_score(seq, sc_out)  # warm
            c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            c0.record(stream)
            eng.he_score(seq, sc_out)
            c1.record(stream)
            torch.cuda.synchronize()
            assert bool(torch.isfinite(sc_out).all()) and float(sc_out.max()) <= 0.0, "scores not finite"
            # the answer's scores are the log-probs generation reported (other kernels, same model)
            score_dev = float((sc_out[:, S - 1:] - out_lp).abs().max())
            T = S + G
            sf = 2 * B * T * d.n_layers * (4 * H * H + 2 * H * F) + d.n_layers * B * 2 * T * T * H + 2 * B * T * d.vocab * H
            sms = c0.elapsed_time(c1)
            score = {"ms": sms, "positions": B * T, "TFLOP/s": sf / (sms * 1e-3) / 1e12,
                     "mfma_frac": sf / (sms * 1e-3) / MFMA_BF16_PEAK, "max_abs_vs_generation_logprobs": score_dev}
        # a plain copy of known size (256 MiB read + 256 MiB written): the reference that
        # rocprofv3's FETCH_SIZE / WRITE_SIZE readings of this same command are scaled by
        cal_src = torch.empty(64 << 20, dtype=torch.float32, device="cuda").normal_()
        cal_dst = torch.empty_like(cal_src)
        binding.he_calibration_copy(cal_src, cal_dst, stream.cuda_stream)
        torch.cuda.synchronize()

    wbytes, kvtok = algorithmic_bytes(d, args.weights_fp8)
    # decode steps of a job see contexts S+1 .. S+G-1 (after appending the new position)
    step_bytes = [wbytes + B * T * kvtok + B * kvtok for T in range(S + 1, S + G)]
    decode_gbs = sum(step_bytes) / (decode_ms * 1e-3) / 1e9 if decode_ms > 0 else 0.0
    pf = prefill_flops(d)

    H, F = d.hidden, d.ffn
    kern_bytes = {  # algorithmic bytes per launch: the weights (and biases) the kernel must stream
        "qkv": 2 * (3 * H * H + 3 * H), "out_proj": 2 * (H * H + H), "fc1": 2 * (F * H + F), "fc2": 2 * (H * F + H),
        "lm_head": 2 * d.vocab * H,
        # attention over the timed decode steps: K and V of one layer at the contexts those steps saw
        "attention": sum(2 * B * T * H * 2 for T in timed_contexts) / max(1, len(timed_contexts)),
    }
    if args.weights_fp8:  # codes + row scales + bias
        kern_bytes.update({"qkv": 3 * H * H + 3 * H * 6, "out_proj": H * H + H * 6, "fc1": F * H + F * 6, "fc2": H * F + H * 6})
    # An event pair brackets more than the kernel (the two timestamp packets).  What that costs is calibrated live
    # on the classes that are also measured without events (the sweeps: launches back to back inside one pair,
    # which agree with a kernel trace's begin-to-end durations): bracket minus sweep, the median over those classes.
    # (The same pair around nothing reads 4-6 us, about 3 us more than it adds to a bracket with a kernel inside;
    # taking that off made every kernel look 3 us shorter than the trace shows it.)
    pair_ms = timing["empty"][0] / max(1, timing["empty"][1])
    over = sorted(timing[k][0] / timing[k][1] - sweep_us[k]["median"] * 1e-3
                  for k in sweep_us if k in timing and timing[k][1])
    over_ms = max(0.0, over[len(over) // 2]) if over else pair_ms
    kernels = {"event_pair_us": pair_ms * 1e3, "bracket_overhead_us": over_ms * 1e3, "timed_steps": len(timed_contexts),
               "timed_contexts": [timed_contexts[0], timed_contexts[-1]] if timed_contexts else None}
    for k, (ms, cnt) in timing.items():
        if cnt and k != "empty":
            avg = max(ms / cnt - over_ms, 1e-6)
            kernels[k] = {"avg_us": avg * 1e3, "launches": cnt}
            if k in kern_bytes:
                kernels[k]["GB/s"] = kern_bytes[k] / (avg * 1e-3) / 1e9
            if k in sweep_us:
                kernels[k]["sweep_us"] = sweep_us[k]["median"]
                kernels[k]["sweep_runs_us"] = sweep_us[k]["runs"]
    # The roofline object is about the DOMINANT kernel of the decode step: the class with the largest summed launch
    # time over the timed steps (per layer every class launches once, so that is the longest launch on average).
    # Its launch duration: the event-bracketed average; for a GEMM class the sweep's figure when there is one (it
    # carries no event-pair cost, and the two agree within a few per cent).
    per_layer = ("qkv", "attention", "out_proj", "fc1", "fc2")
    dom = max((k for k in per_layer if k in kernels), key=lambda k: kernels[k]["avg_us"] * kernels[k]["launches"])
    dom_avg_s = kernels[dom].get("sweep_us", kernels[dom]["avg_us"]) * 1e-6
    achieved = kern_bytes[dom] / dom_avg_s / 1e9 if dom_avg_s > 0 else 0.0
    names = {"qkv": "decode QKV GEMM, LayerNorm folded in, K/V appended to the cache (gemm_skinny_kernel / gemm_half_kernel, mode 2)",
             "attention": "decode attention over the KV cache (attn_kernel), mean context of the timed steps",
             "out_proj": "decode out-projection GEMM, k-split + residual + next LayerNorm's input (gemm_half_kernel, mode 4)",
             "fc1": "decode FC1 GEMM + bias + ReLU, LayerNorm folded in (gemm_half_kernel / gemm_skinny_kernel, mode 1)",
             "fc2": "decode FC2 GEMM, k-split + residual + next LayerNorm's input (gemm_half_kernel, mode 4)"}
    traffic, traffic_src = measured_traffic(d.name, dom, args.weights_fp8)
    roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                "frac": achieved / (HBM_PEAK / 1e9),
                # HBM bytes per launch from the tracked rocprofv3 --pmc summary (fetch measured and scaled by the plain
                # copy kernel's reading, write side stated as algorithmic); null where no such measurement is tracked
                "traffic": traffic, "traffic_source": traffic_src,
                "kernel": names[dom], "kernel_class": dom,
                "bytes_per_launch": kern_bytes[dom], "avg_launch_us": dom_avg_s * 1e6,
                # the whole decode step against the same peak (every kernel, launch gaps included)
                "decode_step_frac": decode_gbs / (HBM_PEAK / 1e9)}

    result = {
        "metric": "generated tokens/s (1 GPU) + decode HBM GB/s as % of 8 TB/s peak",
        "value": B * G * args.steps / wall, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        # the model is bf16 (weights, biases, LayerNorm parameters); the matrix cores take those weights converted
        # exactly to IEEE binary16 and activations / KV cache rounded once to binary16, and accumulate in f32
        "arithmetic": "bf16 model; fp16 MFMA operands (weights converted exactly), f32 accumulation",
        "config": {"workload": f"{d.name}-shaped actor, {d.n_layers} layers, hidden {H}, {d.n_heads} heads, ffn {F}, "
                               f"vocab {d.vocab}; batch {B}, prompt {S}, generate {G}, {d.sampling} sampling"
                               + ("; layer matrices stored as 8-bit E4M3 codes" if args.weights_fp8 else ""),
                   "global_batch": B, "prompt_len": S, "gen_len": G},
        "roofline": roofline,
        "decode": {"ms_per_token_step": decode_ms / (G - 1), "hbm_GB/s": decode_gbs,
                   "hbm_frac": decode_gbs / (HBM_PEAK / 1e9), "tokens/s": B * (G - 1) / (decode_ms * 1e-3)},
        "prefill": {"ms": prefill_ms, "TFLOP/s": pf / (prefill_ms * 1e-3) / 1e12,
                    "mfma_frac": pf / (prefill_ms * 1e-3) / MFMA_BF16_PEAK},
        "kernels": kernels,
        "clocks": clocks.record(),
    }
    if score is not None:
        result["score"] = score
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(d)
    eng.he_destroy()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
