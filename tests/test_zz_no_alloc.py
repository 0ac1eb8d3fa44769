"""The allocation-free entry point (mk_decode_step_static) against mk_decode_step and the oracle.

Two calls in a row through the C ABI, the second on a smaller input (a batch-1 schedule after a batch-3 step of
a wider schedule), so that the second call finds the first one's contents in the GPU's static scratch array;
then the first handle again.  Same kernels and the same static schedule: the logits must be bit-identical to
mk_decode_step's, and within the stated tolerance of the oracle's."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_11581_amd import binding as mk, synth
from paper_2605_11581_amd.runtime import Decoder

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 2e-2


def _case(batch_max, batch, seed_off):
    full = dict(synth.CONFIGS["c0_tiny"])
    cfg = synth.model_cfg(full, max_batch=batch_max)
    w = synth.make_weights(full, gain_jitter=0.1)
    orc = oracle.Decoder(cfg, w)
    kv_h = synth.make_kv_fill(cfg, 40, seed=synth.seed_of(full) + seed_off, batch=batch)
    dec = Decoder(cfg, device=DEV)
    dec.load_weights(w)
    rng = np.random.default_rng(7 + seed_off)
    toks = rng.integers(0, cfg["vocab"], size=batch, dtype=np.int32)
    poss = np.array([40 - 3 * b for b in range(batch)], dtype=np.int32)
    return cfg, orc, dec, kv_h, toks, poss


def _step_both(cfg, orc, dec, kv_h, toks, poss):
    B = len(toks)
    t = torch.from_numpy(toks).to(DEV); p = torch.from_numpy(poss).to(DEV)
    want = orc.step(toks, poss, kv_h.copy())
    kv_a, kv_b = dec.new_kv(kv_h), dec.new_kv(kv_h)
    la = torch.full((B, cfg["vocab"]), float("nan"), device=DEV)
    lb = torch.full((B, cfg["vocab"]), float("nan"), device=DEV)
    mk.mk_decode_step(dec.h, t, p, kv_a, la, B)
    dec.check()
    mk.mk_decode_step_static(dec.h, t, p, kv_b, lb, B)
    dec.check()
    a, b = la.cpu().numpy(), lb.cpu().numpy()
    assert np.isfinite(b).all()
    assert np.array_equal(a, b), "static-scratch step differs from mk_decode_step"
    assert torch.equal(kv_a, kv_b), "appended K/V rows differ"
    for i in range(B):
        e = float(np.abs(b[i] - want[i]).max() / np.abs(want[i]).max())
        assert e <= TOL and int(b[i].argmax()) == oracle.argmax(want[i])


def test_static_scratch_entry_point_matches_the_workspace_one():
    big = _case(4, 3, 0)        # matrix-core schedule for up to 4 sequences, 3 present
    small = _case(1, 1, 1)      # batch-1 schedule: smaller activations, fewer counters
    _step_both(*big)
    _step_both(*small)          # finds the wider schedule's contents in the array
    _step_both(*small)          # same handle again: its counters carry on from the previous epoch
    _step_both(*big)
    # a schedule whose scratch cannot fit is refused before anything is launched
    cfg = synth.model_cfg(synth.CONFIGS["c5_1p7b"], max_batch=16)
    h = mk.mk_build_schedule(mk.make_config(cfg, attn_chunks=64))
    t = torch.zeros(16, dtype=torch.int32, device=DEV)
    with pytest.raises(mk.MkError) as e:
        mk.mk_decode_step_static(h, t, t, t, t, 16)
    assert e.value.code == mk.MK_ENOMEM and "static array" in str(e.value)
    mk.mk_destroy(h)
    for c in (big, small):
        c[2].close()


def test_static_scratch_step_recorded_into_a_graph_replays_correctly():
    """The step number of the static-array entry point lives on the device, so a recorded call can be replayed.  Every
    replay (with eager work and synchronisations of the program between the replays) must give what the eager
    workspace entry point gives for the same tokens and positions: bit-identical logits and cache rows."""
    cfg, orc, dec, kv_h, toks, poss = _case(2, 2, 5)
    B = 2
    t = torch.from_numpy(toks).to(DEV); p = torch.from_numpy(poss).to(DEV)
    kv_g, kv_e = dec.new_kv(kv_h), dec.new_kv(kv_h)
    lg = torch.full((B, cfg["vocab"]), float("nan"), device=DEV)
    le = torch.full((B, cfg["vocab"]), float("nan"), device=DEV)
    # one eager step first (the array then belongs to this schedule), then record one step
    mk.mk_decode_step_static(dec.h, t, p, kv_g, lg, B)
    dec.check()
    mk.mk_decode_step(dec.h, t, p, kv_e, le, B)
    dec.check()
    assert torch.equal(lg, le)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph.capture_begin()
        mk.mk_decode_step_static(dec.h, t, p, kv_g, lg, B, stream=side)
        graph.capture_end()
    torch.cuda.current_stream().wait_stream(side)
    for r in range(4):
        # eager work of the program between the replays: new tokens and positions, the reference step, a host sync
        t.copy_(torch.from_numpy(((toks.astype(np.int64) * (r + 3) + 11 * r) % cfg["vocab"]).astype(np.int32)))
        p.add_(1)
        lg.fill_(float("nan"))
        mk.mk_decode_step(dec.h, t, p, kv_e, le, B)
        dec.check()
        graph.replay()
        torch.cuda.synchronize()
        assert np.isfinite(lg.cpu().numpy()).all(), r
        assert torch.equal(lg, le), f"replay {r} differs from the eager step"
        assert torch.equal(kv_g, kv_e), f"replay {r}: cache rows differ"
    want = orc.step(t.cpu().numpy(), p.cpu().numpy(), kv_e.cpu().numpy().view(np.uint16).copy())
    got = lg.cpu().numpy()
    for i in range(B):
        assert float(np.abs(got[i] - want[i]).max() / np.abs(want[i]).max()) <= TOL
    dec.close()
