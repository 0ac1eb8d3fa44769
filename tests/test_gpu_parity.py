"""GPU parity: the HIP path (through the C ABI of libmk.so) against the CPU oracle, element by
element on the same seeded inputs.

Tolerance (from the benchmark spec): per-step logits max-abs error <= 2e-2 * max|logit| with bf16
weights and fp32 accumulation; identical greedy tokens over the 32-step decode of the tiny
configuration.  The tests below hold the GPU to a much tighter bound where the arithmetic allows
it (fp32 everywhere, different summation order only): 2e-4 * max|logit|.
"""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2605_11581_amd import binding as mk, synth
from paper_2605_11581_amd.runtime import Decoder

pytestmark = pytest.mark.gpu
TOL = 2e-2          # stated acceptance bound
TIGHT = 2e-4        # what fp32 accumulation in a different order actually needs
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)


def rel_err(got, want):
    return float(np.abs(got - want).max() / np.abs(want).max())


class Pair:
    """Oracle and GPU decoder over the same weights and the same KV cache content."""

    def __init__(self, cfg, weights, kv_host=None, **opts):
        self.cfg = cfg
        self.orc = oracle.Decoder(cfg, weights)
        self.kv_h = self.orc.new_kv() if kv_host is None else kv_host
        self.dec = Decoder(cfg, device=DEV, **opts)
        self.dec.load_weights(weights)
        self.kv_d = self.dec.new_kv(self.kv_h)
        B = cfg["max_batch"]
        self.logits = torch.zeros(B, cfg["vocab"], dtype=torch.float32, device=DEV)

    def prefill(self, prompt):
        self.orc.prefill(prompt, self.kv_h)
        self.kv_d.copy_(torch.from_numpy(self.kv_h.view(np.int16)).to(DEV))

    def gpu_step(self, toks, poss, per_op=False):
        t = torch.tensor(list(toks), dtype=torch.int32, device=DEV)
        p = torch.tensor(list(poss), dtype=torch.int32, device=DEV)
        self.logits.fill_(float("nan"))
        self.dec.step(t, p, self.kv_d, self.logits, per_op=per_op)
        self.dec.check()
        return self.logits[: len(toks)].cpu().numpy().copy()

    def close(self):
        self.dec.close()


def tiny(**over):
    full = dict(synth.CONFIGS["c0_tiny"])
    full.update(over)
    return full


def run_greedy(full, steps, prompt_len, tol=TIGHT, check_per_op=True, weights=None, **opts):
    cfg = synth.model_cfg(full)
    w = synth.make_weights(full) if weights is None else weights
    pr = Pair(cfg, w, **opts)
    prompt = synth.make_prompt(full, prompt_len)
    pr.prefill(prompt[:-1])
    cur_o = cur_g = int(prompt[-1])
    worst = 0.0
    for s in range(steps):
        p = prompt_len - 1 + s
        want = pr.orc.step([cur_o], [p], pr.kv_h)[0]
        got = pr.gpu_step([cur_g], [p])[0]
        assert np.isfinite(got).all()
        e = rel_err(got, want)
        worst = max(worst, e)
        assert e <= tol, f"step {s}: logits differ by {e}"
        assert int(got.argmax()) == oracle.argmax(want), f"step {s}: greedy token differs"
        if check_per_op and s in (0, steps - 1):
            # the per-operator launches run the same tile program in plain operator order:
            # bit-identical to the single-launch result (same KV slot rewritten with the same bits)
            again = pr.gpu_step([cur_g], [p], per_op=True)[0]
            assert np.array_equal(again, got), "per-operator order and emitted order disagree bitwise"
        cur_o, cur_g = oracle.argmax(want), int(got.argmax())
    pr.close()
    return worst


def test_c0_greedy_32_steps_match_oracle():
    say("c0: prefill 128 by the oracle, 32 greedy steps on both sides")
    full = tiny()
    worst = run_greedy(full, steps=full["steps"], prompt_len=full["ctx0"])
    say("worst rel err", worst)
    assert worst <= TOL


@pytest.mark.parametrize("opts", [
    dict(qkv_bias=1), dict(use_mfma=1), dict(chunk_rows=2), dict(chunk_rows=4), dict(chunk_rows=8),
    dict(chunk_rows=16, split_qkv=2, split_o=2, split_gateup=2, split_down=4, attn_chunks=4),
    dict(chunk_rows=8, split_gateup=2, split_down=2), dict(n_workgroups=40, attn_chunks=8), dict(attn_chunks=1),
    dict(use_mfma=1, split_qkv=2, split_o=4, split_gateup=2, split_down=2),
    # matrix-core kernels: attention on the matrix cores with one / many chunk tasks
    dict(use_mfma=1, attn_chunks=1), dict(use_mfma=1, attn_chunks=8, n_workgroups=40),
    # weight-page ring (LDS-DMA stream across task boundaries): shallow, deep, ragged stages, matrix-core path
    dict(ring_kb=16), dict(ring_kb=32, attn_chunks=2), dict(ring_kb=96, chunk_rows=2), dict(ring_kb=64, n_workgroups=24),
    dict(ring_kb=48, use_mfma=1, split_o=2, split_down=2),
    # O projection combining the attention partials itself (no combine tasks)
    dict(fuse_combine=1), dict(fuse_combine=1, split_o=2, attn_chunks=4), dict(fuse_combine=1, use_mfma=1, attn_chunks=2),
    dict(fuse_combine=1, split_o=4, rows_o=16, attn_chunks=8, n_workgroups=20), dict(fuse_combine=1, ring_kb=32, attn_chunks=4),
], ids=lambda o: ",".join(f"{k}={v}" for k, v in o.items()))
def test_c0_variants(opts):
    say("c0 variant", opts)
    full = tiny(qkv_bias=opts.pop("qkv_bias", 0))
    w = synth.make_weights(full, gain_jitter=0.1)
    worst = run_greedy(full, steps=6, prompt_len=40, weights=w, **opts)
    say("worst rel err", worst)


def test_qwen3_style_qk_norm_and_head_dim_128():
    full = tiny(qk_norm=1, head_dim=128, n_q_heads=6, n_kv_heads=2, hidden=384, intermediate=1000, index=7)
    w = synth.make_weights(full, gain_jitter=0.2)
    say("qk_norm, d=128, G=3, ragged intermediate")
    run_greedy(full, steps=5, prompt_len=70, weights=w)
    run_greedy(full, steps=3, prompt_len=33, weights=w, use_mfma=1, check_per_op=False)


def test_positions_zero_and_last_slot():
    full = tiny(max_context=64)
    cfg = synth.model_cfg(full)
    w = synth.make_weights(full)
    pr = Pair(cfg, w)
    say("position 0: empty history")
    want = pr.orc.step([11], [0], pr.kv_h)[0]
    got = pr.gpu_step([11], [0])[0]
    assert rel_err(got, want) <= TIGHT
    for p in range(1, 63):
        pr.orc.step([p % 50], [p], pr.kv_h, want_logits=False)
    pr.kv_d.copy_(torch.from_numpy(pr.kv_h.view(np.int16)).to(DEV))
    say("last slot of the cache")
    want = pr.orc.step([3], [63], pr.kv_h)[0]
    got = pr.gpu_step([3], [63])[0]
    assert rel_err(got, want) <= TIGHT
    # the appended K/V rows are bit-identical to the oracle's where both round the same fp32 value;
    # compare as values with one bf16 ulp of slack
    kv_g = pr.kv_d.cpu().numpy().view(np.uint16)
    a = synth.bf16_bits_to_f32(kv_g[:, :, 0, :, 63, :]); b = synth.bf16_bits_to_f32(pr.kv_h[:, :, 0, :, 63, :])
    assert np.abs(a - b).max() <= 2 ** -7 * max(1e-6, np.abs(b).max())
    pr.close()


def test_batched_sequences_with_ragged_positions():
    full = tiny(max_batch=4, index=9)
    cfg = synth.model_cfg(full)
    w = synth.make_weights(full, gain_jitter=0.1)
    pr = Pair(cfg, w)                      # max_batch > 1 selects the matrix-core path
    assert pr.dec.stats["use_mfma"] == 1
    lens = [5, 17, 1, 30]
    say("batch 4, prompts of", lens)
    prompts = [synth.make_prompt(full, n, name=f"p{i}") for i, n in enumerate(lens)]
    # prefill each sequence alone with a batch-1 oracle, then place its cache rows in its batch slot
    one = oracle.Decoder(synth.model_cfg(full, max_batch=1), w)
    for b, pmt in enumerate(prompts):
        kv1 = one.new_kv()
        one.prefill(pmt[:-1], kv1)
        pr.kv_h[:, :, b] = kv1[:, :, 0]
    pr.kv_d.copy_(torch.from_numpy(pr.kv_h.view(np.int16)).to(DEV))
    cur = [int(p[-1]) for p in prompts]
    for s in range(4):
        poss = [n - 1 + s for n in lens]
        want = pr.orc.step(cur, poss, pr.kv_h)
        got = pr.gpu_step(cur, poss)
        for b in range(4):
            assert rel_err(got[b], want[b]) <= TIGHT, (s, b)
            assert int(got[b].argmax()) == oracle.argmax(want[b])
        cur = [oracle.argmax(want[b]) for b in range(4)]
    say("batch 2 of max 4 (the other slots stay idle)")
    want = pr.orc.step(cur[:2], [n + 3 for n in lens[:2]], pr.kv_h)
    got = pr.gpu_step(cur[:2], [n + 3 for n in lens[:2]])
    assert rel_err(got[0], want[0]) <= TIGHT and rel_err(got[1], want[1]) <= TIGHT
    pr.close()


def test_partial_batches_of_a_wider_schedule():
    """A schedule built for eight sequences serves calls with fewer: the staging layout of the
    matrix-core path is a property of the schedule (max_batch), not of the batch of a call."""
    full = tiny(max_batch=8, index=11)
    cfg = synth.model_cfg(full)
    w = synth.make_weights(full, gain_jitter=0.1)
    pr = Pair(cfg, w)
    assert pr.dec.stats["use_mfma"] == 1
    # Tolerance: the matrix-core path carries activations as two bf16 terms (16 mantissa bits), and a
    # freshly appended K/V element that lands on the other side of a bf16 rounding boundary than the
    # oracle's moves a logit by up to ~2e-4 of the largest one on these tiny shapes (the batch-1 fp32
    # path shows up to 6e-5 on the same inputs).  The stated bar is 2e-2.
    tol = 1e-3
    for nb in (8, 5, 3, 1):
        say("batch", nb, "of max 8")
        toks = [3 + 5 * b for b in range(nb)]
        poss = [(7 * b) % 13 for b in range(nb)]
        want = pr.orc.step(toks, poss, pr.kv_h)
        got = pr.gpu_step(toks, poss)
        for b in range(nb):
            assert rel_err(got[b], want[b]) <= tol, (nb, b)
            assert int(got[b].argmax()) == oracle.argmax(want[b])
    pr.close()


def test_residual_sum_level_after_a_k_sliced_down_projection():
    """Eight sequences and a down projection in eight K slices (64 K floats of partial rows): its partial rows are summed into the residual by a level
    of their own (one slice of the rows per workgroup) instead of by every task of the next operator.  Same results as
    the oracle, and bit-identical to the per-operator launches of the same schedule."""
    full = tiny(max_batch=8, hidden=1024, index=13)
    cfg = synth.model_cfg(full)
    w = synth.make_weights(full, gain_jitter=0.1)
    pr = Pair(cfg, w, split_down=8, split_o=2)
    assert pr.dec.stats["split_down"] == 8 and pr.dec.stats["use_mfma"] == 1
    ops = {int(mk.mk_instr_get(pr.dec.h, wg, i)[0]) for wg in range(0, 256, 5) for i in range(mk.mk_instr_count(pr.dec.h, wg))}
    assert 5 in ops, "no residual-sum task in the schedule"
    toks = [3 + 5 * b for b in range(8)]
    for s_, poss in enumerate(([0] * 8, [1, 1, 1, 1, 1, 1, 1, 1], [2, 2, 2, 2, 2, 2, 2, 2])):
        say("residual-sum level, step", s_)
        want = pr.orc.step(toks, poss, pr.kv_h)
        got = pr.gpu_step(toks, poss)
        again = pr.gpu_step(toks, poss, per_op=True)
        for b in range(8):
            assert rel_err(got[b], want[b]) <= 1e-3, (s_, b)
            assert int(got[b].argmax()) == oracle.argmax(want[b])
        assert np.array_equal(got, again)
        toks = [oracle.argmax(want[b]) for b in range(8)]
    pr.close()


def test_ring_and_direct_kernels_agree_bit_for_bit():
    """The page ring changes where the weights wait (LDS instead of registers), not the arithmetic:
    on the same schedule the ring kernel, the direct-load kernel and the per-operator launches
    produce identical logits."""
    full = tiny(max_batch=2, index=3)
    cfg = synth.model_cfg(full)
    w = synth.make_weights(full, gain_jitter=0.1)
    pr = Pair(cfg, w, ring_kb=32)
    assert pr.dec.stats["ring_pages"] == 32
    pr.prefill(synth.make_prompt(full, 45)[:-1])
    ring = pr.gpu_step([7, 9], [44, 0])
    per_op = pr.gpu_step([7, 9], [44, 0], per_op=True)
    assert np.array_equal(ring, per_op)
    pr.close()
    pr = Pair(cfg, w, ring_kb=0)
    pr.prefill(synth.make_prompt(full, 45)[:-1])
    direct = pr.gpu_step([7, 9], [44, 0])
    # a different LDS budget may pick another tiling, hence another summation order
    assert rel_err(direct[0], ring[0]) <= TIGHT and rel_err(direct[1], ring[1]) <= TIGHT
    pr.close()


@pytest.mark.parametrize("batch_max,lens", [(1, [37]), (2, [21, 21]), (4, [9, 9, 9, 9])], ids=["b1", "b2", "b4"])
def test_cache_fill_from_a_prompt_matches_the_oracle_prefill(batch_max, lens):
    """mk_fill_cache: the prompt's K/V rows written by one launch of forced-token decode steps (no LM head) are the
    oracle prefill's rows (both round the same fp32 values to bf16: one ulp of slack), and the decode step that
    follows on the filled cache matches the oracle's.  Batch 1 runs the vector kernels, batch 2 / 4 the matrix cores."""
    full = tiny(max_batch=batch_max, index=19)
    cfg = synth.model_cfg(full)
    w = synth.make_weights(full, gain_jitter=0.1)
    pr = Pair(cfg, w)
    n = lens[0]
    prompts = np.stack([synth.make_prompt(full, n + 1, name=f"fill{b}") for b in range(batch_max)], axis=1)   # [n + 1][B]
    one = oracle.Decoder(synth.model_cfg(full, max_batch=1), w)
    for b in range(batch_max):
        kv1 = one.new_kv()
        one.prefill(prompts[:n, b], kv1)
        pr.kv_h[:, :, b] = kv1[:, :, 0]
    say("cache fill,", n, "tokens, batch", batch_max)
    toks = torch.from_numpy(prompts[:n].astype(np.int32)).to(DEV)
    pos0 = torch.zeros(batch_max, dtype=torch.int32, device=DEV)
    # in two launches (a first part, then the rest from where it ended), so that a start position > 0 is covered too
    k = n // 3
    pr.dec.fill_cache(toks[:k], pos0, pr.kv_d)
    pr.dec.fill_cache(toks[k:], pos0 + k, pr.kv_d)
    pr.dec.check()
    got = synth.bf16_bits_to_f32(pr.kv_d.cpu().numpy().view(np.uint16)[:, :, :, :, :n])
    want = synth.bf16_bits_to_f32(pr.kv_h[:, :, :, :, :n])
    assert np.abs(got - want).max() <= 2 ** -7 * np.abs(want).max()
    assert (pr.kv_d.cpu().numpy()[:, :, :, :, n:] == 0).all(), "rows beyond the prompt were touched"
    cur = [int(t) for t in prompts[n]]
    wl = pr.orc.step(cur, [n] * batch_max, pr.kv_h)
    gl = pr.gpu_step(cur, [n] * batch_max)
    for b in range(batch_max):
        assert rel_err(gl[b], wl[b]) <= 1e-3 and int(gl[b].argmax()) == oracle.argmax(wl[b])
    with pytest.raises(mk.MkError):
        mk.mk_fill_cache(pr.dec.h, toks, pos0, pr.kv_d, batch_max + 1, n)
    pr.close()


def test_per_operator_launches_replayed_from_a_graph_match_eager():
    """The per-operator baseline recorded once into a graph (kernels only) and replayed, with eager work and
    synchronisations between the replays: every replay equals the eager single-launch step bit for bit."""
    full = tiny(index=17)
    cfg = synth.model_cfg(full)
    w = synth.make_weights(full, gain_jitter=0.1)
    pr = Pair(cfg, w)
    pr.prefill(synth.make_prompt(full, 30)[:-1])
    kv_g = pr.kv_d.clone()
    t = torch.tensor([9], dtype=torch.int32, device=DEV)
    p = torch.tensor([29], dtype=torch.int32, device=DEV)
    lg = torch.zeros_like(pr.logits)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        pr.dec.step(t, p, kv_g, lg, per_op=True, stream=side)
        graph.capture_begin()
        pr.dec.step(t, p, kv_g, lg, per_op=True, stream=side)
        graph.capture_end()
    torch.cuda.current_stream().wait_stream(side)
    for r in range(4):
        say("graph replay", r)
        t.fill_(9 + 7 * r)
        p.fill_(29 + r)
        lg.fill_(float("nan"))
        eager = pr.gpu_step([9 + 7 * r], [29 + r])[0]
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(lg[0].cpu().numpy(), eager), f"replay {r} differs from the eager step"
        assert torch.equal(kv_g, pr.kv_d)
    pr.close()


def test_cache_rows_beyond_the_position_are_never_used():
    """KV slots at and after the current position hold whatever the caller left there (here NaN and
    Inf bit patterns); masked positions must contribute exactly nothing."""
    full = tiny(max_context=96)
    cfg = synth.model_cfg(full)
    w = synth.make_weights(full)
    for opts in (dict(), dict(attn_chunks=4), dict(ring_kb=32, attn_chunks=2), dict(use_mfma=1, attn_chunks=2)):
        pr = Pair(cfg, w, **opts)
        prompt = synth.make_prompt(full, 21)
        pr.orc.prefill(prompt[:-1], pr.kv_h)
        poisoned = pr.kv_h.copy()
        poisoned[:, :, :, :, 20:, :] = np.where(np.arange(poisoned.shape[-1]) % 2 == 0, 0x7FC0, 0x7F80).astype(poisoned.dtype)
        pr.kv_d.copy_(torch.from_numpy(poisoned.view(np.int16)).to(DEV))
        cur = int(prompt[-1])
        for s in range(3):
            want = pr.orc.step([cur], [20 + s], pr.kv_h)[0]
            got = pr.gpu_step([cur], [20 + s])[0]
            assert np.isfinite(got).all(), (opts, s)
            assert rel_err(got, want) <= TIGHT, (opts, s)
            cur = oracle.argmax(want)
        pr.close()


def _greedy_oracle(pr, first_tokens, first_positions, n_steps):
    toks, cur = [], list(first_tokens)
    last = None
    for s in range(n_steps):
        last = pr.orc.step(cur, [p + s for p in first_positions], pr.kv_h)
        cur = [oracle.argmax(last[b]) for b in range(len(cur))]
        toks.append(cur)
    return np.array(toks, dtype=np.int32), last


@pytest.mark.parametrize("opts", [dict(), dict(ring_kb=32), dict(n_workgroups=48, attn_chunks=4)],
                         ids=lambda o: ",".join(f"{k}={v}" for k, v in o.items()) or "default")
def test_c0_32_greedy_steps_in_one_launch(opts):
    """The acceptance run of the tiny configuration with the token feedback on the device: one
    launch walks the instruction lists 32 times; the greedy tokens equal the oracle's, the last
    step's logits and the appended cache rows agree, and single steps continue from there."""
    full = tiny()
    cfg = synth.model_cfg(full)
    w = synth.make_weights(full)
    pr = Pair(cfg, w, **opts)
    n0, n = full["ctx0"], full["steps"]
    prompt = synth.make_prompt(full, n0)
    pr.prefill(prompt[:-1])
    want_toks, want_last = _greedy_oracle(pr, [int(prompt[-1])], [n0 - 1], n)
    t = torch.tensor([int(prompt[-1])], dtype=torch.int32, device=DEV)
    p = torch.tensor([n0 - 1], dtype=torch.int32, device=DEV)
    pr.logits.fill_(float("nan"))
    got_toks = pr.dec.greedy(t, p, pr.kv_d, pr.logits, n)
    pr.dec.check()
    got_toks = got_toks.cpu().numpy()
    say("greedy tokens", got_toks[:, 0].tolist())
    assert np.array_equal(got_toks, want_toks)
    assert rel_err(pr.logits[:1].cpu().numpy()[0], want_last[0]) <= TIGHT
    kv_g = synth.bf16_bits_to_f32(pr.kv_d.cpu().numpy().view(np.uint16)[:, :, 0, :, n0 - 1:n0 - 1 + n, :])
    kv_o = synth.bf16_bits_to_f32(pr.kv_h[:, :, 0, :, n0 - 1:n0 - 1 + n, :])
    assert np.abs(kv_g - kv_o).max() <= 2 ** -7 * np.abs(kv_o).max()
    # a plain single step continues where the multi-step launch stopped
    nxt = int(want_toks[-1, 0])
    want = pr.orc.step([nxt], [n0 - 1 + n], pr.kv_h)[0]
    got = pr.gpu_step([nxt], [n0 - 1 + n])[0]
    assert rel_err(got, want) <= TIGHT and int(got.argmax()) == oracle.argmax(want)
    pr.close()


def test_batched_greedy_steps_in_one_launch_and_argument_checks():
    full = tiny(max_batch=3, index=5)
    cfg = synth.model_cfg(full)
    w = synth.make_weights(full, gain_jitter=0.1)
    pr = Pair(cfg, w)
    lens = [9, 1, 26]
    prompts = [synth.make_prompt(full, n, name=f"q{i}") for i, n in enumerate(lens)]
    one = oracle.Decoder(synth.model_cfg(full, max_batch=1), w)
    for b, pmt in enumerate(prompts):
        kv1 = one.new_kv()
        one.prefill(pmt[:-1], kv1)
        pr.kv_h[:, :, b] = kv1[:, :, 0]
    pr.kv_d.copy_(torch.from_numpy(pr.kv_h.view(np.int16)).to(DEV))
    first = [int(p[-1]) for p in prompts]
    pos0 = [n - 1 for n in lens]
    want_toks, want_last = _greedy_oracle(pr, first, pos0, 7)
    t = torch.tensor(first, dtype=torch.int32, device=DEV)
    p = torch.tensor(pos0, dtype=torch.int32, device=DEV)
    got = pr.dec.greedy(t, p, pr.kv_d, pr.logits, 7)
    pr.dec.check()
    assert np.array_equal(got.cpu().numpy(), want_toks)
    for b in range(3):
        assert rel_err(pr.logits[b].cpu().numpy(), want_last[b]) <= TIGHT
    for bad_n in (0, cfg["max_context"] + 1):
        with pytest.raises(mk.MkError) as e:
            pr.dec.greedy(t, p, pr.kv_d, pr.logits, bad_n)
        assert e.value.code == mk.MK_EINVAL
    say("running past the end of the cache raises the position error and still terminates")
    p_end = torch.tensor([cfg["max_context"] - 2] * 3, dtype=torch.int32, device=DEV)
    pr.dec.greedy(t, p_end, pr.kv_d, pr.logits, 4)
    with pytest.raises(mk.MkError) as e:
        pr.dec.check()
    assert e.value.code == mk.MK_EINVAL
    pr.close()


# ---- W4A16 form of the decoder projections (Sec. 4.3.2) ------------------------------------------

class PairW4(Pair):
    """Oracle and GPU decoder over the same W4 codes / scales (embedding and LM head stay bf16)."""

    def __init__(self, cfg, weights, quant, **opts):
        self.cfg = cfg
        self.orc = oracle.Decoder(cfg, weights, quant=quant)
        self.kv_h = self.orc.new_kv()
        self.dec = Decoder(cfg, device=DEV, weight_bits=4, group_size=quant["group"], **opts)
        self.dec.load_weights(synth.library_weights(weights, quant))
        self.kv_d = self.dec.new_kv(self.kv_h)
        self.logits = torch.zeros(cfg["max_batch"], cfg["vocab"], dtype=torch.float32, device=DEV)


@pytest.mark.parametrize("opts", [
    # VALU form (batch 1): a lane dequantises its 32 codes in registers
    dict(use_mfma=0), dict(use_mfma=0, group=64), dict(use_mfma=0, group=32, qkv_bias=1), dict(use_mfma=0, chunk_rows=16),
    dict(use_mfma=0, chunk_rows=16, split_o=2, split_down=2),
    dict(use_mfma=0, rows_gateup=16, split_gateup=2, split_qkv=2, attn_chunks=4), dict(use_mfma=0, n_workgroups=36, rows_down=4, rows_o=8),
    dict(use_mfma=0, fuse_combine=1, attn_chunks=4), dict(use_mfma=0, fuse_combine=1, rows_o=16, split_o=2),
    dict(),
    # matrix-core form (the default at batch > 1): codes expanded to bf16 numbers 128 + q, four instructions per chunk
    dict(use_mfma=1), dict(use_mfma=1, group=64), dict(use_mfma=1, group=32, qkv_bias=1), dict(use_mfma=1, split_o=2, split_down=2),
    dict(use_mfma=1, split_gateup=2, split_qkv=2, attn_chunks=4), dict(use_mfma=1, n_workgroups=36),
    dict(use_mfma=1, fuse_combine=1, attn_chunks=4),
], ids=lambda o: ",".join(f"{k}={v}" for k, v in o.items()) or "default")
def test_w4_c0_greedy_steps_match_oracle(opts):
    opts = dict(opts)
    group = opts.pop("group", 128)
    full = tiny(intermediate=640, qkv_bias=opts.pop("qkv_bias", 0), index=13)
    cfg = synth.model_cfg(full)
    w = synth.make_weights(full, gain_jitter=0.1)
    q = synth.make_quant(full, group=group)
    pr = PairW4(cfg, w, q, **opts)
    say("W4 schedule", {k: pr.dec.stats[k] for k in ("rows_qkv", "rows_o", "rows_gateup", "rows_down", "split_o", "split_down")})
    prompt = synth.make_prompt(full, 37)
    pr.prefill(prompt[:-1])
    cur_o = cur_g = int(prompt[-1])
    for s in range(6):
        p = 36 + s
        want = pr.orc.step([cur_o], [p], pr.kv_h)[0]
        got = pr.gpu_step([cur_g], [p])[0]
        err = rel_err(got, want)
        say("step", s, "rel err", err)
        assert err <= TIGHT
        if s == 0:
            assert np.array_equal(got, pr.gpu_step([cur_g], [p], per_op=True)[0])
        cur_o, cur_g = oracle.argmax(want), int(got.argmax())
        assert cur_o == cur_g
    # and the same as greedy steps of one launch
    want_toks, _ = _greedy_oracle(pr, [cur_o], [42], 5)
    t = torch.tensor([cur_g], dtype=torch.int32, device=DEV)
    p = torch.tensor([42], dtype=torch.int32, device=DEV)
    got_toks = pr.dec.greedy(t, p, pr.kv_d, pr.logits, 5)
    pr.dec.check()
    assert np.array_equal(got_toks.cpu().numpy(), want_toks)
    pr.close()


def test_w4_rejects_what_it_does_not_cover():
    full = tiny(intermediate=640)
    for bad in (dict(max_batch=9), dict(max_batch=2, use_mfma=0), dict(ring_kb=32), dict(group_size=48), dict(intermediate=688),
                dict(rows_qkv=8, use_mfma=1)):
        cfg = synth.model_cfg(dict(full, **{k: v for k, v in bad.items() if k in ("max_batch", "intermediate")}))
        opts = {k: v for k, v in bad.items() if k not in ("max_batch", "intermediate")}
        with pytest.raises(mk.MkError) as e:
            mk.mk_build_schedule(mk.make_config(cfg, n_workgroups=64, weight_bits=4, **opts))
        assert e.value.code == mk.MK_EINVAL, bad


@pytest.mark.parametrize("group,batch_max,present", [(128, 4, 3), (64, 8, 8), (32, 2, 2)])
def test_w4_batched_sequences_on_the_matrix_cores(group, batch_max, present):
    """W4A16 at batch > 1 (the paper measures batch 1..16 in this precision, Sec. 5.2): ragged positions,
    teacher-forced, every sequence against the oracle."""
    full = tiny(intermediate=640, qkv_bias=1, index=17)
    cfg = synth.model_cfg(full, max_batch=batch_max)
    w = synth.make_weights(full, gain_jitter=0.1)
    q = synth.make_quant(full, group=group)
    pr = PairW4(cfg, w, q)
    assert pr.dec.stats["use_mfma"] == 1
    pr.kv_h = synth.make_kv_fill(cfg, 50, seed=5, batch=present)
    pr.kv_d = pr.dec.new_kv(pr.kv_h)
    rng = np.random.default_rng(11)
    for s in range(3):
        toks = rng.integers(0, cfg["vocab"], size=present, dtype=np.int32)
        poss = [50 - 7 * b + s for b in range(present)]
        want = pr.orc.step(toks, poss, pr.kv_h)
        got = pr.gpu_step(toks, poss)
        for b in range(present):
            e = rel_err(got[b], want[b])
            say(f"W4 group {group} batch {present}/{batch_max} step {s} seq {b}: rel err {e:.2e}")
            assert e <= 1e-3 and int(got[b].argmax()) == oracle.argmax(want[b])
    pr.close()


def test_two_runs_are_bit_identical():
    full = tiny()
    cfg = synth.model_cfg(full)
    w = synth.make_weights(full)
    pr = Pair(cfg, w)
    pr.prefill(synth.make_prompt(full, 50)[:-1])
    a = pr.gpu_step([7], [49])
    b = pr.gpu_step([7], [49])
    assert np.array_equal(a, b)
    pr.close()


def test_error_paths_leave_the_kernel_running_to_completion():
    full = tiny()
    cfg = synth.model_cfg(full)
    w = synth.make_weights(full)
    dec = Decoder(cfg, device=DEV)
    tok = torch.tensor([1], dtype=torch.int32, device=DEV); pos = torch.tensor([0], dtype=torch.int32, device=DEV)
    logits = torch.zeros(1, cfg["vocab"], device=DEV)
    kv = dec.new_kv()
    with pytest.raises(mk.MkError) as e:
        dec.step(tok, pos, kv, logits)                 # before load_weights
    assert e.value.code == mk.MK_ESTATE
    dec.load_weights(w)
    with pytest.raises(mk.MkError) as e:
        mk.mk_decode_step(dec.h, tok, pos, kv, logits, 2)    # batch > max_batch
    assert e.value.code == mk.MK_EINVAL
    say("out-of-range token: clamped in the kernel, reported by mk_check")
    tok[0] = cfg["vocab"] + 5
    dec.step(tok, pos, kv, logits)
    with pytest.raises(mk.MkError) as e:
        dec.check()
    assert e.value.code == mk.MK_EINVAL
    tok[0] = 1
    dec.step(tok, pos, kv, logits); dec.check()       # healthy again
    dec.close()
    say("spin limit of one poll: waits give up, every wave still reaches the end of its list")
    dec = Decoder(cfg, device=DEV, spin_limit=1)
    dec.load_weights(w)
    kv = dec.new_kv()
    dec.step(tok, pos, kv, logits)
    with pytest.raises(mk.MkError) as e:              # one poll never sees 256 producers finished: the waits give up
        dec.check()
    assert e.value.code == mk.MK_ETIMEOUT
    dec.step(tok, pos, kv, logits)                    # counters were re-armed: the launch still terminates
    torch.cuda.synchronize()
    dec.close()


_WEIGHTS = {}


def _weights_of(name):
    """Host weights of one configuration, kept for the tests that follow (one configuration at a time:
    the 7B shape alone is 14 GB)."""
    if name not in _WEIGHTS:
        _WEIGHTS.clear()
        say(name, ": generating weights")
        _WEIGHTS[name] = synth.make_weights(synth.CONFIGS[name])
    return _WEIGHTS[name]


def _teacher_forced(name, steps_idx, tol=TIGHT, batch=1, w4=False, ctx0=None, **opts):
    full = synth.CONFIGS[name]
    ctx0 = full["ctx0"] if ctx0 is None else ctx0
    cfg = synth.model_cfg(full, max_batch=batch, max_context=max(full["max_context"], ctx0 + max(steps_idx) + 2))
    w = _weights_of(name)
    kv_h = synth.make_kv_fill(cfg, ctx0, seed=synth.seed_of(full), batch=batch)
    if w4:
        pr = PairW4(cfg, w, synth.make_quant(full), **opts)
        pr.kv_h = kv_h
        pr.kv_d = pr.dec.new_kv(kv_h)
    else:
        pr = Pair(cfg, w, kv_host=kv_h, **opts)
    say(name, ": schedule", {k: v for k, v in pr.dec.stats.items() if k.startswith(("split", "rows", "attn", "use"))})
    rng = np.random.default_rng(synth.seed_of(full))
    n = max(steps_idx) + 1
    toks = rng.integers(0, cfg["vocab"], size=(n, batch), dtype=np.int32)
    for s in range(n):
        poss = [ctx0 + s] * batch
        if s in steps_idx:
            want = pr.orc.step(toks[s], poss, pr.kv_h)
            got = pr.gpu_step(toks[s], poss)
            for b in range(batch):
                e = rel_err(got[b], want[b])
                say(f"{name} batch {batch} step {s} seq {b}: rel err {e:.2e}")
                assert e <= tol and int(got[b].argmax()) == oracle.argmax(want[b])
        else:   # advance both caches without comparing
            pr.orc.step(toks[s], poss, pr.kv_h, want_logits=False)
            pr.gpu_step(toks[s], poss)
    pr.close()
    del pr
    torch.cuda.empty_cache()


def test_c1_half_billion_shape_teacher_forced():
    _teacher_forced("c1_0p5b", (0, 1, 3))


def test_c2_headline_shape_in_bench_configuration():
    """Same configuration bench.py times (the library's own schedule choice, one launch per step)."""
    _teacher_forced("c2_1p5b", (0, 1, 3))


def test_c2_headline_shape_with_w4_weights():
    """The 1.5B shape in the precision the paper measures (Sec. 5.1: GPTQ-W4A16), as bench.py --w4 times it."""
    _teacher_forced("c2_1p5b", (0, 2), w4=True)


def test_c3_qwen3_4b_shape():
    """Per-head QK-norm at full size, 8 KV heads, context 4096."""
    _teacher_forced("c3_4b", (0, 1))


@pytest.mark.parametrize("batch", [1, 4, 8])
def test_c4_7b_shape(batch):
    """Batch 1 on the VALU path; batch 4 and 8 as thin GEMMs on the matrix cores (at batch 8 the staged
    activations no longer fit LDS whole: the K range of a task is staged in slices)."""
    _teacher_forced("c4_7b", (0,), batch=batch, tol=TIGHT if batch == 1 else 1e-3)
    if batch == 8:
        _WEIGHTS.clear()


@pytest.mark.parametrize("name,batch", [("c5_1p7b", 1), ("c5_1p7b", 16), ("c2_1p5b", 16), ("c2_1p5b", 2)])
def test_short_context_batch_sweep_workload(name, batch):
    """The paper's fixed workload (Sec. 5.2: 64-token prompts, 12 generated tokens, batch 1..16) on the two
    model shapes it measures (Sec. 5.1): first and last of the 12 steps, teacher-forced.  Batch 16 takes two
    matrix-core instructions per weight chunk (sequences 0..7 and 8..15)."""
    _teacher_forced(name, (0, 11), batch=batch, ctx0=64, tol=TIGHT if batch == 1 else 1e-3)
    _WEIGHTS.clear()


def test_profile_guided_search_walk_keeps_parity():
    """The on-device tiling search (Sec. 4.2.2 Step 4: candidates scored by profiling): a two-parameter walk
    on the tiny shape times every candidate through the C ABI, accepts only candidates whose logits agree
    with the starting schedule's, and its winner matches the oracle."""
    from paper_2605_11581_amd import autotune
    from paper_2605_11581_amd.runtime import stage_weights
    full = tiny()
    cfg = synth.model_cfg(full)
    w = synth.make_weights(full)
    space = [("attn_chunks", [1, 2, 4]), ("fuse_combine", [0, 1])]
    best, ms, hist = autotune.autotune(cfg, stage_weights(w, DEV), position=100, device=DEV, steps=6, warmup=2, rounds=1,
                                       space=space, log=say)
    assert ms is not None and ms > 0 and len(hist) >= 4
    assert set(best) == {"attn_chunks", "fuse_combine"}
    assert all(m is not None for _, m in hist), "a candidate of this space was infeasible or lost parity"
    worst = run_greedy(full, 4, 60, weights=w, **best)
    say("winner", best, f"{ms:.4f} ms/step, worst rel err {worst:.2e}")
