#!/usr/bin/env python3
"""Decode-throughput benchmark of the single-launch megakernel on one MI355X.

A step = one decode step (the whole hot path: embedding -> L decoder layers -> final norm + LM
head, KV append included) as ONE kernel launch.  The default workload is the one the metric is
quoted on: the Qwen2.5-1.5B-shaped configuration at batch 1, KV context 2048 + step.  Inputs are
synthetic and resident in HBM before the timed region.  Prints one JSON line per workload.

    python bench.py                               # headline workload
    python bench.py --config c4_7b --batch 8      # another BASELINE workload
    python bench.py --w4                          # W4A16 decoder projections
    python bench.py --all                         # every BASELINE workload, one line each, also written
                                                  # to profiles/results.json

Protocol: W untimed warm-up steps, then K steps enqueued back to back on one stream between two
host synchronisations (`value`, `ms_per_step`); the same K steps again `--reps` times between a pair
of HIP events on the launch stream (`repetitions`: median and min); the kernel's own duration from
HIP events the library records around single launches (`roofline`); the device's streaming-read
ceiling measured in the same run (`roofline.ceiling_gbs`); the first step compared with the CPU
oracle's (`parity_rel_err`).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
SHAPE_NAMES = {"c0_tiny": "tiny Qwen2-style", "c1_0p5b": "Qwen2.5-0.5B-shaped", "c2_1p5b": "Qwen2.5-1.5B-shaped",
               "c3_4b": "Qwen3-4B-shaped", "c4_7b": "Qwen2.5-7B-shaped", "c5_1p7b": "Qwen3-1.7B-shaped"}
# --all: (config, batch, w4, context at the first step or 0 for the configuration's own, steps or 0).  First the
# BASELINE workloads, then the paper's fixed short workload (Sec. 5.2: 64-token prompts, 12 generated tokens, batch 1..16)
# on the two model shapes it measures.
ALL_WORKLOADS = [("c2_1p5b", 1, False, 0, 0), ("c1_0p5b", 1, False, 0, 0), ("c3_4b", 1, False, 0, 0), ("c4_7b", 1, False, 0, 0),
                 ("c4_7b", 4, False, 0, 0), ("c4_7b", 8, False, 0, 0), ("c2_1p5b", 1, True, 0, 0), ("c2_1p5b", 4, False, 0, 0),
                 ("c2_1p5b", 8, False, 0, 0), ("c2_1p5b", 4, True, 0, 0), ("c2_1p5b", 8, True, 0, 0)] + [
    (name, b, False, 64, 12) for name in ("c2_1p5b", "c5_1p7b") for b in (1, 2, 4, 8, 16)]


def algorithmic_bytes(cfg, batch: int, T: float, w4_group: int = 0) -> float:
    """Bytes one decode step must move: every weight once (bf16; with W4 the seven projections are
    half a byte per element plus one bf16 scale per group), K and V once per KV head for the T
    attended positions (bf16), logits written (fp32)."""
    L, H, d = cfg["n_layers"], cfg["hidden"], cfg["head_dim"]
    qd, kvd, I, V = cfg["n_q_heads"] * d, cfg["n_kv_heads"] * d, cfg["intermediate"], cfg["vocab"]
    mats = H * (qd + 2 * kvd) + qd * H + 3 * H * I
    vecs = 2 * H
    if cfg["qkv_bias"]:
        vecs += qd + 2 * kvd
    if cfg["qk_norm"]:
        vecs += 2 * d
    mat_bytes = mats * (0.5 + 2.0 / w4_group) if w4_group else 2.0 * mats
    weights = L * (mat_bytes + 2.0 * vecs) + 2.0 * (V * H + H)
    kv = batch * 4.0 * L * kvd * T
    return weights + kv + 4.0 * batch * V


def kernel_name(stats, w4: bool, multi: bool = False) -> str:
    fam = "_w4" if w4 else "_mfma" if stats["use_mfma"] else ""
    if stats["ring_pages"]:
        return "mk_megakernel_ring"
    return "mk_megakernel" + ("_steps" if multi else "") + fam


def recorded_traffic(kernel: str, config: str, batch: int):
    """HBM bytes per launch from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary of this kernel and
    workload (a recorded profile, not measured in this run), or None."""
    tag = f"{kernel}_{config}" + (f"_batch{batch}" if batch > 1 else "")
    path = os.path.join(ROOT, "profiles", f"{tag}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(line.split(":")[1]), os.path.relpath(path, ROOT)
    except OSError:
        pass
    return None, None


def note(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def set_oracle_threads(n: int) -> None:
    ctypes.CDLL("libgomp.so.1", mode=ctypes.RTLD_GLOBAL).omp_set_num_threads(int(n))


def run_workload(config: str, batch: int, w4: bool, steps: int, warmup: int, reps: int, context: int, opts: dict,
                 cpu_baseline: bool, per_op: bool, headline_metric: bool, weights_cache: dict) -> dict:
    import numpy as np
    import torch
    from paper_2605_11581_amd import binding as mk, synth
    from paper_2605_11581_amd.runtime import Decoder

    full = synth.CONFIGS[config]
    B = batch
    ctx0 = context if context > 0 else full["ctx0"]
    note(f"{config} batch {B}{' w4' if w4 else ''} context {ctx0}: generating inputs")
    cfg = synth.model_cfg(full, max_batch=max(B, 1), max_context=ctx0 + steps + warmup + 64)
    dev = "cuda:0"
    t0 = time.time()
    if config not in weights_cache:
        weights_cache.clear()
        weights_cache[config] = synth.make_weights(full)
    w = weights_cache[config]
    kv_h = synth.make_kv_fill(cfg, ctx0, seed=synth.seed_of(full), batch=B)
    t_gen = time.time() - t0
    w4_group = 128 if w4 else 0
    quant = None
    if w4:
        quant = synth.make_quant(full, group=w4_group)
        dec = Decoder(cfg, device=dev, weight_bits=4, group_size=w4_group, **opts)
        dec.load_weights(synth.library_weights(w, quant))
    else:
        dec = Decoder(cfg, device=dev, **opts)
        dec.load_weights(w)
    stream = torch.cuda.current_stream()
    kv_d = dec.new_kv(kv_h)
    n_all = steps + warmup
    rng = np.random.default_rng(synth.seed_of(full))
    toks = torch.from_numpy(rng.integers(0, cfg["vocab"], size=(n_all, B), dtype=np.int32)).to(dev)
    poss = torch.from_numpy((ctx0 + np.arange(n_all, dtype=np.int32))[:, None].repeat(B, 1)).to(dev)
    logits = torch.empty(B, cfg["vocab"], dtype=torch.float32, device=dev)

    def run(first: int, n: int, per_op_launches: bool = False):
        for i in range(first, first + n):
            dec.step(toks[i], poss[i], kv_d, logits, per_op=per_op_launches, stream=stream)

    # ---- step 0 of the run (kept for the parity check against the oracle below)
    note("weights loaded; stepping")
    run(0, 1)
    dec.check()
    logits0 = logits.cpu().numpy().copy()

    # ---- timed region: K steps back to back on one stream, one launch each
    run(1, warmup - 1) if warmup > 1 else None
    dec.check()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    run(warmup, steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t1
    dec.check()
    ms_per_step = elapsed * 1e3 / steps
    tok_s = steps * B / elapsed

    # ---- the same K steps again, `reps` times, between a pair of HIP events on the launch stream
    rep_ms = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        run(warmup, steps)
        e1.record(stream)
        e1.synchronize()
        rep_ms.append(e0.elapsed_time(e1) / steps)
    dec.check()

    # ---- kernel duration by HIP events the library records around each launch (same positions)
    mk.mk_set_flags(dec.h, mk.MK_F_TIMING)
    n_ev = min(steps, 64)
    durs = []
    for i in range(warmup, warmup + n_ev):
        dec.step(toks[i], poss[i], kv_d, logits, stream=stream)
        durs.append(mk.mk_last_step_ms(dec.h))
    mk.mk_set_flags(dec.h, 0)
    kern_ms = float(np.mean(durs))
    T_ev = ctx0 + warmup + (n_ev - 1) / 2.0 + 1
    bytes_launch = algorithmic_bytes(cfg, B, T_ev, w4_group)
    achieved = bytes_launch / (kern_ms * 1e-3) / 1e9
    T_run = ctx0 + warmup + (steps - 1) / 2.0 + 1
    bytes_step = algorithmic_bytes(cfg, B, T_run, w4_group)

    # ---- streaming-read ceiling of this device, same run: the library streams its own weight region
    ceil_ms, ceil_bytes = mk.mk_read_ceiling(dec.h, 5, stream=stream)
    ceiling = ceil_bytes / (float(np.median(ceil_ms)) * 1e-3) / 1e9

    st = dec.stats
    kname = kernel_name(st, w4)
    traffic, traffic_src = recorded_traffic(kname, config, B)
    shape = SHAPE_NAMES.get(config, config)
    precision = "W4A16 (group 128) decoder projections, bf16 embedding/LM head/KV" if w4 else "bf16 weights/KV"
    metric = ("decode tokens/s at batch 1 (1.5B shape); achieved HBM GB/s vs peak" if headline_metric
              else f"decode tokens/s at batch {B} ({shape}, {precision}); achieved HBM GB/s vs peak")
    out = {
        "metric": metric,
        "value": round(tok_s, 2), "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("w4 (group 128) projections, bf16 embedding/LM head/KV, f32 accumulate" if w4
                  else "bf16 weights/KV, f32 accumulate"), "data": "synthetic",
        "config": {"workload": f"{config}: {shape} decoder, {precision}, batch {B}, KV context {ctx0}+step, "
                               f"{steps} single-launch decode steps", "batch": B, "context0": ctx0,
                   "schedule": {k: st[k] for k in ("n_workgroups", "split_qkv", "split_o", "split_gateup", "split_down",
                                                   "attn_chunks", "rows_qkv", "rows_o", "rows_gateup", "rows_down",
                                                   "rows_head", "fuse_combine", "use_mfma", "ring_pages", "lds_bytes",
                                                   "from_table")}},
        "repetitions": {"n": reps, "timer": "HIP event pair on the launch stream around the K steps",
                        "ms_per_step_median": round(float(np.median(rep_ms)), 5), "ms_per_step_min": round(float(np.min(rep_ms)), 5),
                        "tokens_per_s_median": round(B * 1e3 / float(np.median(rep_ms)), 2)},
        "hbm_gbs_whole_run": round(bytes_step / (ms_per_step * 1e-3) / 1e9, 1),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": traffic_src,
                     "ceiling_gbs": round(ceiling, 1), "frac_of_ceiling": round(achieved / ceiling, 4),
                     "ceiling": f"persistent grid, 128-bit nontemporal loads over {ceil_bytes / 1e9:.2f} GB, median of 5 launches",
                     "kernel": kname, "kernel_ms": round(kern_ms, 5), "kernel_launches_timed": n_ev,
                     "algorithmic_bytes": int(bytes_launch)},
    }

    # ---- the same number of greedy steps as ONE launch (token feedback on the device)
    kv_ms = dec.new_kv(kv_h)
    first = toks[warmup].clone()
    p0 = poss[warmup].clone()
    dec.greedy(first, p0, kv_ms, logits, min(steps, 8))
    torch.cuda.synchronize()
    kv_ms.copy_(dec.new_kv(kv_h))
    t4 = time.perf_counter()
    dec.greedy(first, p0, kv_ms, logits, steps)
    torch.cuda.synchronize()
    ms_multi = (time.perf_counter() - t4) * 1e3 / steps
    dec.check()
    out["multi_step_launch"] = {"ms_per_step": round(ms_multi, 5), "tokens_per_s": round(B * 1e3 / ms_multi, 2),
                                "steps_in_one_launch": steps, "tokens": "greedy, fed back on the device",
                                "kernel": kernel_name(st, w4, multi=True)}
    del kv_ms

    if per_op:
        n_po = min(steps, 32)
        # (a level that sums the down projection's partial rows exists from 64 K floats of them on)
        residual_sum = int(st["split_down"] > 1 and st["split_down"] * cfg["max_batch"] * cfg["hidden"] >= 65536)
        run(warmup, 2, per_op_launches=True)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        run(warmup, n_po, per_op_launches=True)
        torch.cuda.synchronize()
        po = (time.perf_counter() - t2) / n_po
        out["per_op_baseline"] = {"ms_per_step": round(po * 1e3, 5), "tokens_per_s": round(B / po, 2),
                                  "launches_per_step": cfg["n_layers"] * (6 - st["fuse_combine"] + residual_sum) + 2, "steps": n_po,
                                  "speedup_of_one_launch": round(po * 1e3 / ms_per_step, 3)}
        # The same per-operator launches recorded ONCE into a HIP graph and replayed (Sec. 2: launch overhead that graphs
        # do not remove, since every operator is still a kernel boundary).  The recorded work is kernels only; positions
        # advance inside the graph.
        try:
            tg, pg = toks[warmup].clone(), poss[warmup].clone()
            side = torch.cuda.Stream()
            side.wait_stream(stream)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                dec.step(tg, pg, kv_d, logits, per_op=True, stream=side)      # (eager once on the capture stream)
                graph.capture_begin()
                dec.step(tg, pg, kv_d, logits, per_op=True, stream=side)
                pg.add_(1)
                graph.capture_end()
            stream.wait_stream(side)
            pg.copy_(poss[warmup])
            torch.cuda.synchronize()
            graph.replay(); graph.replay()
            pg.copy_(poss[warmup])
            torch.cuda.synchronize()
            t3 = time.perf_counter()
            for _ in range(n_po):
                graph.replay()
            torch.cuda.synchronize()
            pg_ms = (time.perf_counter() - t3) / n_po * 1e3
            dec.check()
            out["per_op_baseline"]["graph_replay_ms_per_step"] = round(pg_ms, 5)
            out["per_op_baseline"]["speedup_of_one_launch_over_graph"] = round(pg_ms / ms_per_step, 3)
            del graph
        except Exception as exc:                                            # the baseline is a side figure: never lose the line
            out["per_op_baseline"]["graph_replay_error"] = str(exc)[:200]

    if cpu_baseline:
        note("GPU legs done; CPU oracle")
        import oracle
        orc = oracle.Decoder(cfg, w, quant=quant)
        th = toks.cpu().numpy(); ph = poss.cpu().numpy()
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        set_oracle_threads(cores)
        t3 = time.perf_counter()
        want0 = orc.step(th[0], ph[0], kv_h)          # the step the GPU ran first: parity of this very run
        one = time.perf_counter() - t3
        err = float(max(np.abs(logits0[b] - want0[b]).max() / np.abs(want0[b]).max() for b in range(B)))
        same = all(int(logits0[b].argmax()) == int(oracle.argmax(want0[b])) for b in range(B))
        out["parity_rel_err"] = float(f"{err:.3e}")
        out["parity"] = {"step": 0, "max_abs_err_over_max_abs_logit": float(f"{err:.3e}"), "bound": 2e-2,
                         "greedy_token_equal": bool(same), "against": "CPU oracle, same inputs"}
        note(f"oracle step 0: {one:.1f} s on {cores} threads, parity {err:.2e}")
        # bounded sample: about 15 s of CPU work beyond the parity step (none when one step already takes that long)
        n_cpu = int(min(steps - 1, 15.0 / max(one, 1e-3)))
        if n_cpu >= 1:
            t3 = time.perf_counter()
            for i in range(1, 1 + n_cpu):
                orc.step(th[i], ph[i], kv_h)
            cpu = (time.perf_counter() - t3) / n_cpu
            sample = f"{n_cpu} decode steps of the same workload (of {steps}); OpenMP over output rows"
        else:
            cpu, sample = one, f"1 decode step of the same workload (of {steps}); OpenMP over output rows"
        out["cpu_baseline"] = {"value": round(B / cpu, 3), "unit": "tokens/s", "cores": cores, "kind": "oracle", "sample": sample}
        if one <= 1.5 and 1 + n_cpu < n_all:      # one thread: only where a step stays within about half a minute
            set_oracle_threads(1)
            note("oracle on one thread")
            t3 = time.perf_counter()
            orc.step(th[1 + n_cpu], ph[1 + n_cpu], kv_h)
            cpu1 = time.perf_counter() - t3
            set_oracle_threads(cores)
            out["cpu_baseline"]["one_thread"] = {"value": round(B / cpu1, 4), "unit": "tokens/s", "cores": 1, "sample": "1 decode step"}
        else:
            out["cpu_baseline"]["one_thread"] = None   # (a single-thread step of this workload would take minutes)
        if not (err <= 2e-2 and same):
            out["parity"]["FAILED"] = True
    out["setup_s"] = {"generate_inputs": round(t_gen, 1)}
    dec.close()
    del dec, kv_d
    torch.cuda.empty_cache()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--reps", type=int, default=5, help="repetitions of the K timed steps between HIP events (median, min)")
    ap.add_argument("--config", default="c2_1p5b")
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-op", action="store_true")
    ap.add_argument("--opt", action="append", default=[], help="schedule override key=value (e.g. split_down=4)")
    ap.add_argument("--w4", action="store_true", help="W4A16 decoder projections (group 128) instead of bf16")
    ap.add_argument("--context", type=int, default=0, help="KV context at the first step (default: the configuration's)")
    ap.add_argument("--calib-copy", action="store_true", help="also run a plain 1 GiB device-to-device copy (calibrates the FETCH_SIZE / WRITE_SIZE counters in profiler runs)")
    ap.add_argument("--all", action="store_true", help="every BASELINE workload, one line each; also written to profiles/results.json")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        return 2
    opts = {}
    for kv in args.opt:
        k, v = kv.split("=")
        opts[k] = int(v)
    cache: dict = {}
    if args.calib_copy:
        import torch
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").fill_(1.0)
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    if not args.all:
        headline = args.config == "c2_1p5b" and args.batch == 1 and not args.w4 and args.context == 0
        out = run_workload(args.config, args.batch, args.w4, args.steps, max(args.warmup, 1), args.reps, args.context, opts,
                           not args.no_cpu_baseline, not args.no_per_op, headline, cache)
        print(json.dumps(out))
        return 1 if out.get("parity", {}).get("FAILED") else 0
    from paper_2605_11581_amd import synth
    lines = []
    for config, batch, w4, context, n_steps in ALL_WORKLOADS:
        steps = n_steps or min(args.steps, synth.CONFIGS[config]["steps"])
        out = run_workload(config, batch, w4, steps, max(args.warmup, 1), args.reps, context, opts, not args.no_cpu_baseline,
                           not args.no_per_op, (config, batch, w4, context) == ("c2_1p5b", 1, False, 0), cache)
        print(json.dumps(out), flush=True)
        lines.append(out)
    with open(os.path.join(ROOT, "profiles", "results.json"), "w") as f:
        json.dump({"command": "python bench.py --all", "results": lines}, f, indent=1)
        f.write("\n")
    return 1 if any(o.get("parity", {}).get("FAILED") for o in lines) else 0


if __name__ == "__main__":
    sys.exit(main())
