#!/usr/bin/env python3
"""Decode-throughput benchmark of the single-launch megakernel on one MI355X.

A step = one decode step (the whole hot path: embedding -> 28 decoder layers ->
final norm + LM head) of the Qwen2.5-1.5B-shaped configuration at batch 1 and
KV context 2048+step, as ONE kernel launch.  Inputs are synthetic and resident
in HBM before the timed region.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


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


def measured_traffic(config: str):
    """HBM bytes per launch from the committed rocprofv3 counter summary of this workload (or None)."""
    path = os.path.join(ROOT, "profiles", f"mk_megakernel_{config}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(line.split(":")[1])
    except OSError:
        pass
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="c2_1p5b")
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-op", action="store_true")
    ap.add_argument("--calib-copy", action="store_true", help="also run a plain 1 GiB device copy (counter calibration)")
    ap.add_argument("--opt", action="append", default=[], help="schedule override key=value (e.g. split_down=4)")
    ap.add_argument("--w4", action="store_true", help="W4A16 decoder projections (group 128) instead of bf16")
    ap.add_argument("--context", type=int, default=0, help="KV context at the first timed step (default: the configuration's)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2605_11581_amd import binding as mk, synth
    from paper_2605_11581_amd.runtime import Decoder

    full = synth.CONFIGS[args.config]
    B = args.batch
    steps, warmup = args.steps, args.warmup
    ctx0 = args.context if args.context > 0 else full["ctx0"]
    cfg = synth.model_cfg(full, max_batch=max(B, 1), max_context=ctx0 + steps + warmup + 64)
    opts = {}
    for kv in args.opt:
        k, v = kv.split("=")
        opts[k] = int(v)
    dev = "cuda:0"
    t0 = time.time()
    w = synth.make_weights(full)
    kv_h = synth.make_kv_fill(cfg, ctx0, seed=synth.seed_of(full), batch=B)
    t_gen = time.time() - t0
    w4_group = 128 if args.w4 else 0
    quant = None
    if args.w4:
        quant = synth.make_quant(full, group=w4_group)
        dec = Decoder(cfg, device=dev, weight_bits=4, group_size=w4_group, **opts)
        dec.load_weights(synth.library_weights(w, quant))
    else:
        dec = Decoder(cfg, device=dev, **opts)
        dec.load_weights(w)
    kv_d = dec.new_kv(kv_h)
    n_all = steps + warmup
    rng = np.random.default_rng(synth.seed_of(full))
    toks = torch.from_numpy(rng.integers(0, cfg["vocab"], size=(n_all, B), dtype=np.int32)).to(dev)
    poss = torch.from_numpy((ctx0 + np.arange(n_all, dtype=np.int32))[:, None].repeat(B, 1)).to(dev)
    logits = torch.empty(B, cfg["vocab"], dtype=torch.float32, device=dev)

    def run(first: int, n: int, per_op: bool = False):
        for i in range(first, first + n):
            dec.step(toks[i], poss[i], kv_d, logits, per_op=per_op)

    if args.calib_copy:
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    # ---- timed region: K steps back to back on one stream, one launch each
    run(0, warmup)
    dec.check()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    run(warmup, steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t1
    dec.check()
    ms_per_step = elapsed * 1e3 / steps
    tok_s = steps * B / elapsed

    # ---- kernel duration by HIP events on the launch stream (separate pass, same positions)
    mk.mk_set_flags(dec.h, mk.MK_F_TIMING)
    n_ev = min(steps, 64)
    durs = []
    for i in range(warmup, warmup + n_ev):
        dec.step(toks[i], poss[i], kv_d, logits)
        durs.append(mk.mk_last_step_ms(dec.h))
    mk.mk_set_flags(dec.h, 0)
    kern_ms = float(np.mean(durs))
    T_ev = ctx0 + warmup + (n_ev - 1) / 2.0 + 1
    bytes_launch = algorithmic_bytes(cfg, B, T_ev, w4_group)
    achieved = bytes_launch / (kern_ms * 1e-3) / 1e9
    T_run = ctx0 + warmup + (steps - 1) / 2.0 + 1
    bytes_step = algorithmic_bytes(cfg, B, T_run, w4_group)

    out = {
        "metric": "decode tokens/s at batch 1 (1.5B shape); achieved HBM GB/s vs peak",
        "value": round(tok_s, 2), "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("w4 (group 128) projections, bf16 embedding/LM head/KV, f32 accumulate" if args.w4
                  else "bf16 weights/KV, f32 accumulate"), "data": "synthetic",
        "config": {"workload": f"{args.config}: Qwen2.5-1.5B-shaped decoder, batch {B}, KV context {ctx0}+step, "
                               f"{steps} single-launch decode steps", "batch": B, "context0": ctx0,
                   "schedule": {k: dec.stats[k] for k in ("n_workgroups", "split_qkv", "split_o", "split_gateup",
                                                          "split_down", "attn_chunks", "rows_qkv", "rows_o", "rows_gateup",
                                                          "rows_down", "rows_head", "use_mfma", "ring_pages", "lds_bytes")}},
        "hbm_gbs_whole_run": round(bytes_step / (ms_per_step * 1e-3) / 1e9, 1),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": measured_traffic(args.config) if B == 1 and not args.w4 else None,
                     "kernel": "mk_megakernel", "kernel_ms": round(kern_ms, 5), "algorithmic_bytes": int(bytes_launch)},
    }

    # ---- the same number of greedy steps as ONE launch (token feedback on the device)
    kv_ms = dec.new_kv(kv_h)
    first = toks[warmup].clone()
    p0 = poss[warmup].clone()
    dec.greedy(first, p0, kv_ms, logits, min(steps, 8))
    torch.cuda.synchronize()
    kv_ms.copy_(kv_d if False else dec.new_kv(kv_h))
    t4 = time.perf_counter()
    dec.greedy(first, p0, kv_ms, logits, steps)
    torch.cuda.synchronize()
    ms_multi = (time.perf_counter() - t4) * 1e3 / steps
    dec.check()
    out["multi_step_launch"] = {"ms_per_step": round(ms_multi, 5), "tokens_per_s": round(B * 1e3 / ms_multi, 2),
                                "steps_in_one_launch": steps, "tokens": "greedy, fed back on the device"}
    del kv_ms

    if not args.no_per_op:
        n_po = min(steps, 32)
        run(warmup, 2, per_op=True)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        run(warmup, n_po, per_op=True)
        torch.cuda.synchronize()
        po = (time.perf_counter() - t2) / n_po
        out["per_op_baseline"] = {"ms_per_step": round(po * 1e3, 5), "tokens_per_s": round(B / po, 2),
                                  "launches_per_step": cfg["n_layers"] * 6 + 1, "steps": n_po,
                                  "speedup_of_one_launch": round(po * 1e3 / ms_per_step, 3)}

    if not args.no_cpu_baseline:
        import oracle
        orc = oracle.Decoder(cfg, w, quant=quant)
        th = toks.cpu().numpy(); ph = poss.cpu().numpy()
        t3 = time.perf_counter()
        orc.step(th[0], ph[0], kv_h)
        one = time.perf_counter() - t3
        n_cpu = int(max(2, min(steps, 15.0 / max(one, 1e-3))))
        t3 = time.perf_counter()
        for i in range(1, 1 + n_cpu):
            orc.step(th[i], ph[i], kv_h)
        cpu = (time.perf_counter() - t3) / n_cpu
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        out["cpu_baseline"] = {"value": round(B / cpu, 3), "unit": "tokens/s", "cores": cores, "kind": "oracle",
                               "sample": f"{n_cpu} decode steps of the same workload (of {steps}); OpenMP over output rows"}
    out["setup_s"] = {"generate_inputs": round(t_gen, 1)}
    print(json.dumps(out))
    dec.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
