"""Per-level timeline of one decode step from the in-kernel task trace (MK_F_TRACE).

Every task records four device wall-clock stamps (begin, dependencies met, prologue done, end;
100 MHz).  This tool runs a few steps of a configuration with tracing on, reads the trace of the
last one back through the C ABI and prints, for one layer and for the whole step, how long each
dependency level (operator instance) takes and what the time is spent on: the gap between the
last producer's signal and the consumers' start, prologues, task bodies, and the spread between
the median and the slowest task.  It shows where the time of a step goes beyond its memory
traffic, and is the feedback signal for the profile-guided tiling search (paper Sec. 4.2.2 Step 4:
offline profiling of candidate traces).

    python -m paper_2605_11581_amd.trace_report --config c2_1p5b [--layer 13] [--w4] [--batch B] [--opt k=v ...]
"""
from __future__ import annotations

import argparse
import sys

import numpy as np

TICK_US = 0.01
STAGES = {0: "QKV", 1: "ATT", 2: "COMB", 3: "O", 4: "GU", 5: "DOWN", 6: "HEAD", 7: "ARGMAX"}


def collect(dec, tok, pos, kv, logits, steps: int = 5):
    """Run ``steps`` single-step launches and return (trace [n_wg][max_instr][8] int64, op, ref_seq) of the last."""
    from . import binding as mk
    for _ in range(steps):
        dec.step(tok, pos, kv, logits)
    dec.check()
    tr = mk.mk_read_trace(dec.h).astype(np.int64)
    n_wg, mi = dec.stats["n_workgroups"], dec.stats["max_instr_per_wg"] + 1
    tr = tr.reshape(n_wg, mi, 8)
    op = np.zeros((n_wg, mi), dtype=np.int64)
    seq = np.full((n_wg, mi), -1, dtype=np.int64)
    for w in range(n_wg):
        for i in range(mk.mk_instr_count(dec.h, w)):
            ins = mk.mk_instr_get(dec.h, w, i)
            op[w, i], seq[w, i] = ins[0], ins[2]
    return tr, op, seq


def report(tr, seq, layer: int, out=sys.stdout) -> None:
    valid = seq >= 0
    t_start = tr[..., 0][valid].min()
    us = lambda a: (a - t_start) * TICK_US
    print(f"step: {us(tr[..., 3][valid].max()):.1f} us from the first task's begin to the last task's end", file=out)
    print("level     tasks | begins (min p50 max) | deps met (p50 max) | ends (min p50 max)      | "
          "wait  prologue  body (mean us) | after the last producer's end: first / last start of a body", file=out)
    prev_end = None
    rows = {}
    for sq in np.unique(seq[valid]):
        m = valid & (seq == sq)
        t0, t1, t2, t3 = (us(tr[..., k][m]) for k in range(4))
        rows[int(sq)] = (t0, t1, t2, t3)
    per_stage = {}
    n_layers = int(seq[valid].max()) // 8       # the LM head and the arg-max tasks carry the index one past the last layer
    # stage 6 inside a layer is the residual-sum level that follows a K-sliced down projection
    name = lambda l, st: "RSUM" if (st == 6 and l < n_layers) else STAGES.get(st, st)
    for sq, (t0, t1, t2, t3) in rows.items():
        l, st = divmod(sq, 8)
        per_stage.setdefault((st, name(l, st)), []).append((t3.max() - t0.min(), (t1 - t0).mean(), (t2 - t1).mean(), (t3 - t2).mean()))
        if l != layer and l < n_layers:
            continue
        gap = ""
        if prev_end is not None:
            gap = f"{t2.min() - prev_end:6.1f} / {t2.max() - prev_end:6.1f}"
        print(f"L{l:02d} {name(l, st):6s} {len(t0):5d} | {t0.min():7.1f} {np.median(t0):7.1f} {t0.max():7.1f} | "
              f"{np.median(t1):7.1f} {t1.max():7.1f} | {t3.min():7.1f} {np.median(t3):7.1f} {t3.max():7.1f} | "
              f"{(t1 - t0).mean():5.2f} {(t2 - t1).mean():5.2f} {(t3 - t2).mean():6.2f} | {gap}", file=out)
        prev_end = t3.max()
    # inside the attention tasks (task-internal marks): q/k/v prologue, history loop, slot merge, store
    m = valid & (seq % 8 == 1) & (seq // 8 == layer)
    if m.any():
        t1, t3 = us(tr[..., 1][m]), us(tr[..., 3][m])
        k0, k1, k2, k3 = (us(tr[..., 4 + k][m]) for k in range(4))
        print(f"L{layer:02d} ATT inside a task (mean us): prologue {np.mean(k0 - t1):.2f}, history loop {np.mean(k1 - k0):.2f}, "
              f"slots to LDS {np.mean(k2 - k1):.2f}, merge + stores issued {np.mean(k3 - k2):.2f}, "
              f"store drain + signal {np.mean(t3 - k3):.2f}", file=out)
    # inside the GEMV bodies: weights consumed (partial sums in LDS), then cross-wave sum + epilogue + store drain + signal
    for st in (0, 3, 4, 5):
        m = valid & (seq % 8 == st) & (seq // 8 == layer)
        if m.any() and (tr[..., 7][m] > 0).all():
            t2, t3, k3 = us(tr[..., 2][m]), us(tr[..., 3][m]), us(tr[..., 7][m])
            print(f"L{layer:02d} {STAGES[st]:5s} inside a body (mean us): weight loop + flush {np.mean(k3 - t2):.2f}, "
                  f"reduce + epilogue + drain + signal {np.mean(t3 - k3):.2f}", file=out)
    print("mean over all layers: level span (first begin to last end), wait, prologue, body [us]", file=out)
    for st in sorted(per_stage):
        a = np.array(per_stage[st]).mean(0)
        print(f"  {st[1]:6s} {a[0]:7.2f} {a[1]:6.2f} {a[2]:6.2f} {a[3]:6.2f}", file=out)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="c2_1p5b")
    ap.add_argument("--layer", type=int, default=13)
    ap.add_argument("--w4", action="store_true")
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--opt", action="append", default=[])
    args = ap.parse_args()
    import torch
    from . import binding as mk, synth
    from .runtime import Decoder

    full = synth.CONFIGS[args.config]
    cfg = synth.model_cfg(full, max_batch=args.batch)
    opts = {k: int(v) for k, v in (kv.split("=") for kv in args.opt)}
    w = synth.make_weights(full)
    if args.w4:
        w = synth.library_weights(w, synth.make_quant(full))
        opts.update(weight_bits=4, group_size=128)
    dec = Decoder(cfg, flags=mk.MK_F_TRACE, **opts)
    print("schedule:", {k: v for k, v in dec.stats.items() if k.startswith(("split", "rows", "attn", "fuse", "ring", "lds"))})
    dec.load_weights(w)
    kv = dec.new_kv(synth.make_kv_fill(cfg, full["ctx0"], seed=synth.seed_of(full)))
    B = args.batch
    tok = torch.full((B,), 5, dtype=torch.int32, device="cuda")
    pos = torch.full((B,), full["ctx0"], dtype=torch.int32, device="cuda")
    logits = torch.empty(B, cfg["vocab"], dtype=torch.float32, device="cuda")
    tr, _, seq = collect(dec, tok, pos, kv, logits)
    report(tr, seq, args.layer)
    dec.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
