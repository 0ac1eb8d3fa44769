"""Pins of the CPU oracle against things other than itself: closed forms,
invariants, library routines, brute force on tiny inputs, and an independent
implementation of the same public model family (transformers, if importable).

The paper prints no logits, tokens or intermediate values, so there is no
worked numerical example of the decoder to pin to; the page-budget equations
(Sec. 4.1.1, Eq. 1-2) are pinned to the figures of Sec. 4.3.2 / Sec. 1 stored
in tests/golden/page_budget.txt.
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from w4_format import dequant
from paper_2605_11581_amd import synth

ONE = np.uint16(0x3F80)  # bf16(1.0)


def bits(a):
    return synth.to_bf16_bits(np.asarray(a, dtype=np.float32))


def vals(b):
    return synth.bf16_bits_to_f32(np.asarray(b, dtype=np.uint16))


# ---------------------------------------------------------------- bf16
def test_bf16_rne_ties_and_roundtrip():
    # ulp of bf16 at 1.0 is 2^-7: 1+2^-8 is a tie -> even (1.0); 1+3*2^-8 is a tie -> 1+2^-6
    assert oracle.f32_to_bf16([1.0 + 2.0 ** -8])[0] == 0x3F80
    assert oracle.f32_to_bf16([1.0 + 3 * 2.0 ** -8])[0] == 0x3F82
    assert oracle.f32_to_bf16([1.0 + 2.0 ** -8 + 2.0 ** -20])[0] == 0x3F81
    assert oracle.f32_to_bf16([-2.5])[0] == 0xC020
    allb = np.arange(0, 0x7F80, 37, dtype=np.uint16)  # finite positives
    assert np.array_equal(oracle.f32_to_bf16(oracle.bf16_to_f32(allb)), allb)
    assert np.array_equal(oracle.bf16_to_f32(allb), vals(allb))


def test_bf16_bulk_matches_torch_cast():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(4000).astype(np.float32) * s
                        for s in (1e-30, 1e-3, 1.0, 1e20)] + [np.float32([0.0, -0.0, np.inf, -np.inf, 1e-40])])
    assert np.array_equal(oracle.f32_to_bf16(x), bits(x))


# ---------------------------------------------------------------- RMSNorm
def test_rmsnorm_constant_vector_closed_form():
    n, c, eps = 48, 3.0, 1e-6
    g = bits(np.linspace(0.5, 2.0, n))
    y = oracle.rmsnorm(np.full(n, c, np.float32), g, eps)
    want = vals(g).astype(np.float64) * c / math.sqrt(c * c + eps)
    assert np.allclose(y, want, rtol=1e-6, atol=0)


def test_rmsnorm_unit_rms_and_scale_invariance():
    rng = np.random.default_rng(2)
    x = rng.standard_normal(100).astype(np.float32)
    g1 = np.full(100, ONE)
    y = oracle.rmsnorm(x, g1, 1e-6)
    assert abs(np.sqrt(np.mean(y.astype(np.float64) ** 2)) - 1.0) < 1e-5
    y2 = oracle.rmsnorm(1000.0 * x, g1, 1e-6)
    assert np.allclose(y, y2, rtol=1e-5, atol=1e-6)
    # eps sits inside the square root, added to the mean square (not to the rms)
    z = oracle.rmsnorm(np.zeros(4, np.float32) + 1e-3, np.full(4, ONE), 1.0)
    assert np.allclose(z, 1e-3 / math.sqrt(1e-6 + 1.0), rtol=1e-6)


# ---------------------------------------------------------------- RoPE
def test_rope_identity_at_position_zero():
    rng = np.random.default_rng(3)
    u = rng.standard_normal(64).astype(np.float32)
    assert np.array_equal(oracle.rope(u, 0, 1e4), u)


def test_rope_preserves_pair_norms():
    rng = np.random.default_rng(4)
    d = 64
    u = rng.standard_normal(d).astype(np.float32)
    y = oracle.rope(u, 1234, 1e6)
    pn_u = u[: d // 2].astype(np.float64) ** 2 + u[d // 2:].astype(np.float64) ** 2
    pn_y = y[: d // 2].astype(np.float64) ** 2 + y[d // 2:].astype(np.float64) ** 2
    assert np.allclose(pn_u, pn_y, rtol=1e-5)


def test_rope_relative_position_property():
    rng = np.random.default_rng(5)
    q = rng.standard_normal(32).astype(np.float32)
    k = rng.standard_normal(32).astype(np.float32)
    a = np.dot(oracle.rope(q, 17, 1e4).astype(np.float64), oracle.rope(k, 5, 1e4))
    b = np.dot(oracle.rope(q, 112, 1e4).astype(np.float64), oracle.rope(k, 100, 1e4))
    c = np.dot(oracle.rope(q, 12, 1e4).astype(np.float64), oracle.rope(k, 0, 1e4))
    assert abs(a - b) < 1e-4 and abs(a - c) < 1e-4


def test_rope_d2_is_plane_rotation_and_frequency_ladder():
    # d = 2: single pair (0,1), exponent 0 -> rotation by `pos` radians, counter-clockwise
    y = oracle.rope(np.float32([1.0, 0.0]), 1, 1e4)
    assert np.allclose(y, [math.cos(1.0), math.sin(1.0)], atol=1e-7)
    # d = 4, theta = 100: pair (1,3) rotates by pos * 100^(-2/4) = pos / 10
    y = oracle.rope(np.float32([0.0, 1.0, 0.0, 0.0]), 5, 100.0)
    assert np.allclose(y, [0.0, math.cos(0.5), 0.0, math.sin(0.5)], atol=1e-7)


# ---------------------------------------------------------------- softmax / attention
def test_softmax_sums_to_one_shift_invariant():
    rng = np.random.default_rng(6)
    s = (rng.standard_normal(300) * 5).astype(np.float32)
    w = oracle.softmax(s)
    assert (w >= 0).all() and abs(w.astype(np.float64).sum() - 1.0) < 1e-6
    assert np.allclose(oracle.softmax(s + 100.0), w, rtol=1e-4, atol=1e-9)
    assert np.allclose(w, torch.softmax(torch.from_numpy(s).double(), 0).numpy(), rtol=1e-6, atol=1e-12)


def test_attention_single_key_returns_v_exactly():
    rng = np.random.default_rng(7)
    d = 64
    q = rng.standard_normal(d).astype(np.float32)
    K = bits(rng.standard_normal((1, d))); V = bits(rng.standard_normal((1, d)))
    assert np.array_equal(oracle.attend(q, K, V), vals(V)[0])


def test_attention_equal_scores_gives_mean_and_dominant_key_selects_row():
    rng = np.random.default_rng(8)
    d, T = 32, 9
    V = bits(rng.standard_normal((T, d)))
    K = np.tile(bits(rng.standard_normal((1, d))), (T, 1))
    q = rng.standard_normal(d).astype(np.float32)
    assert np.allclose(oracle.attend(q, K, V), vals(V).astype(np.float64).mean(0), rtol=1e-6, atol=1e-7)
    Kf = np.zeros((T, d), np.float32); Kf[4, 0] = 64.0
    qd = np.zeros(d, np.float32); qd[0] = 64.0   # score of key 4 is 64*64/sqrt(32) ~ 724
    assert np.allclose(oracle.attend(qd, bits(Kf), V), vals(V)[4], rtol=1e-6, atol=1e-7)


def test_attention_matches_float64_bruteforce_with_scale():
    rng = np.random.default_rng(9)
    d, T = 16, 37
    q = rng.standard_normal(d).astype(np.float32)
    K = bits(rng.standard_normal((T, d))); V = bits(rng.standard_normal((T, d)))
    s = vals(K).astype(np.float64) @ q.astype(np.float64) / math.sqrt(d)
    w = torch.softmax(torch.from_numpy(s), 0).numpy()
    assert np.allclose(oracle.attend(q, K, V), w @ vals(V).astype(np.float64), rtol=1e-5, atol=1e-6)


# ---------------------------------------------------------------- GEMV / SiLU
def test_gemv_bruteforce_nonsquare_identity_onehot():
    rng = np.random.default_rng(10)
    W = bits(rng.standard_normal((5, 7))); x = rng.standard_normal(7).astype(np.float32)
    b = bits(rng.standard_normal(5))
    want = [sum(float(vals(W)[r, k]) * float(x[k]) for k in range(7)) + float(vals(b)[r]) for r in range(5)]
    assert np.allclose(oracle.gemv(W, x, b), want, rtol=1e-6)
    assert np.allclose(oracle.gemv(W, x), np.array(want) - vals(b), rtol=1e-5, atol=1e-6)
    assert np.array_equal(oracle.gemv(bits(np.eye(7)), x), x)
    E = np.zeros((3, 7), np.float32); E[0, 6] = 1; E[1, 0] = 1; E[2, 3] = 1
    assert np.array_equal(oracle.gemv(bits(E), x), x[[6, 0, 3]])


def test_silu_identities():
    assert oracle.silu(0.0) == 0.0
    assert abs(oracle.silu(30.0) - 30.0) < 1e-5
    for z in (0.3, 1.7, 4.0):
        assert abs(oracle.silu(-z) - (oracle.silu(z) - z)) < 1e-6
    assert abs(oracle.silu(1.0) - 1.0 / (1.0 + math.exp(-1.0))) < 1e-7


def test_argmax_lowest_index_on_ties():
    assert oracle.argmax(np.float32([1, 5, 5, 2])) == 1


# ---------------------------------------------------------------- whole step
TINY = dict(n_layers=2, hidden=32, n_q_heads=4, n_kv_heads=2, head_dim=8, intermediate=48, vocab=50,
            qkv_bias=1, qk_norm=0, tie_embeddings=0, rope_theta=1e4, rms_eps=1e-6, max_batch=2,
            max_context=16)


def _zero(ws, keys):
    for k in keys:
        ws[k] = [np.zeros_like(a) for a in ws[k]]


def test_step_all_layers_zero_closed_form():
    w = synth.make_weights(TINY, seed=11, std=0.5, gain_jitter=0.1)
    _zero(w, ["wq", "wk", "wv", "bq", "bk", "bv", "wo", "w_gate", "w_up", "w_down"])
    dec = oracle.Decoder(TINY, w)
    kv = dec.new_kv()
    tok = 13
    got = dec.step([tok], [3], kv)[0]
    x = vals(w["embed"])[tok].astype(np.float64)
    h = x / np.sqrt(np.mean(x * x) + 1e-6) * vals(w["final_norm"])
    want = vals(w["lm_head"]).astype(np.float64) @ h
    assert np.allclose(got, want, rtol=1e-5, atol=1e-6)


def test_step_zero_branch_isolation():
    base = synth.make_weights(TINY, seed=12, std=0.3)
    # wo = 0 removes the attention branch; w_down = 0 removes the MLP branch; both -> embedding only
    wa = dict(base); _zero(wa, ["wo"])
    wm = dict(base); _zero(wm, ["w_down"])
    wb = dict(base); _zero(wb, ["wo", "w_down"])
    w0 = dict(base); _zero(w0, ["wq", "wk", "wv", "bq", "bk", "bv", "wo", "w_gate", "w_up", "w_down"])
    outs = []
    for w in (wb, w0, wa, wm, base):
        dec = oracle.Decoder(TINY, w); kv = dec.new_kv()
        dec.step([7], [0], kv)
        outs.append(dec.step([9], [1], kv)[0])
    assert np.array_equal(outs[0], outs[1])
    assert not np.allclose(outs[2], outs[0]) and not np.allclose(outs[3], outs[0])
    # zero gate weights alone kill the MLP exactly (silu(0) * up = 0)
    wg = dict(base); _zero(wg, ["w_gate"])
    dec = oracle.Decoder(TINY, wg); kv = dec.new_kv(); dec.step([7], [0], kv)
    dec2 = oracle.Decoder(TINY, wm); kv2 = dec2.new_kv(); dec2.step([7], [0], kv2)
    assert np.array_equal(dec.step([9], [1], kv)[0], dec2.step([9], [1], kv2)[0])


def test_gqa_equals_mha_with_replicated_kv_heads():
    w = synth.make_weights(TINY, seed=13, std=0.3)
    mha = dict(TINY, n_kv_heads=4)
    d = TINY["head_dim"]
    rep = lambda a: np.concatenate([a[g * d:(g + 1) * d] for g in (0, 0, 1, 1)], axis=0)
    w2 = dict(w)
    for k in ("wk", "wv", "bk", "bv"):
        w2[k] = [rep(a) for a in w[k]]
    d1, d2 = oracle.Decoder(TINY, w), oracle.Decoder(mha, w2)
    kv1, kv2 = d1.new_kv(), d2.new_kv()
    for p, t in enumerate([3, 14, 15, 9, 2]):
        a = d1.step([t], [p], kv1)[0]; b = d2.step([t], [p], kv2)[0]
        assert np.array_equal(a, b)


def test_batch_rows_are_independent_sequences():
    w = synth.make_weights(TINY, seed=14, std=0.3)
    dec = oracle.Decoder(TINY, w)
    kvb = dec.new_kv(); kva = dec.new_kv()
    seq0, seq1 = [4, 8, 15], [16, 23, 42]
    for p in range(3):
        lb = dec.step([seq0[p], seq1[p]], [p, p], kvb)
        la = dec.step([seq1[p]], [p], kva)          # seq1 alone in slot 0
        assert np.array_equal(lb[1], la[0])


def _hf_compare(model_type):
    transformers = pytest.importorskip("transformers")
    torch.manual_seed(0)
    kw = dict(hidden_size=32, intermediate_size=48, num_hidden_layers=2, num_attention_heads=4,
              num_key_value_heads=2, vocab_size=50, max_position_embeddings=64, rms_norm_eps=1e-6,
              rope_theta=1e4, tie_word_embeddings=False, attention_dropout=0.0, head_dim=8)
    try:
        if model_type == "qwen2":
            cfg = transformers.Qwen2Config(**kw, use_sliding_window=False)
            model = transformers.Qwen2ForCausalLM(cfg)
        else:
            cfg = transformers.Qwen3Config(**kw, attention_bias=False, use_sliding_window=False)
            model = transformers.Qwen3ForCausalLM(cfg)
    except Exception as e:  # pragma: no cover - library drift
        pytest.skip(f"transformers cannot build the tiny model: {e}")
    model = model.float().eval()
    with torch.no_grad():
        for prm in model.parameters():
            prm.mul_(8.0 if prm.dim() > 1 else 1.0)           # larger weights -> conventions matter
            prm.copy_(prm.to(torch.bfloat16).float())
        for name, prm in model.named_parameters():
            if "norm" in name:
                prm.copy_((1.0 + 0.1 * torch.randn_like(prm)).to(torch.bfloat16).float())
            if name.endswith("bias"):
                prm.copy_((0.5 * torch.randn_like(prm)).to(torch.bfloat16).float())
    sd = {k: v.detach().numpy() for k, v in model.state_dict().items()}
    g = lambda k: bits(sd[k])
    L = 2
    ours = dict(TINY, qkv_bias=1 if model_type == "qwen2" else 0, qk_norm=0 if model_type == "qwen2" else 1,
                max_batch=1)
    w = {"embed": g("model.embed_tokens.weight"), "lm_head": g("lm_head.weight"),
         "final_norm": g("model.norm.weight")}
    lay = lambda fmt: [g(fmt.format(l)) for l in range(L)]
    w["attn_norm"] = lay("model.layers.{}.input_layernorm.weight")
    w["mlp_norm"] = lay("model.layers.{}.post_attention_layernorm.weight")
    for ours_k, hf_k in (("wq", "q_proj"), ("wk", "k_proj"), ("wv", "v_proj"), ("wo", "o_proj")):
        w[ours_k] = lay("model.layers.{}.self_attn." + hf_k + ".weight")
    for ours_k, hf_k in (("w_gate", "gate_proj"), ("w_up", "up_proj"), ("w_down", "down_proj")):
        w[ours_k] = lay("model.layers.{}.mlp." + hf_k + ".weight")
    if model_type == "qwen2":
        for ours_k, hf_k in (("bq", "q_proj"), ("bk", "k_proj"), ("bv", "v_proj")):
            w[ours_k] = lay("model.layers.{}.self_attn." + hf_k + ".bias")
        w["q_norm"] = w["k_norm"] = None
    else:
        w["bq"] = w["bk"] = w["bv"] = None
        w["q_norm"] = lay("model.layers.{}.self_attn.q_norm.weight")
        w["k_norm"] = lay("model.layers.{}.self_attn.k_norm.weight")
    toks = [5, 17, 33, 2, 41, 8, 29]
    with torch.no_grad():
        ref = model(torch.tensor([toks])).logits[0].numpy()
    dec = oracle.Decoder(ours, w); kv = dec.new_kv()
    worst = 0.0
    for p, t in enumerate(toks):
        got = dec.step([t], [p], kv)[0]
        worst = max(worst, np.abs(got - ref[p]).max() / np.abs(ref[p]).max())
    # the only modelled difference is the bf16 rounding of cached K/V (rel. 2^-9 per element)
    assert worst < 1e-2, worst
    return worst


def test_conventions_against_transformers_qwen2():
    _hf_compare("qwen2")


def test_conventions_against_transformers_qwen3():
    _hf_compare("qwen3")


# ---------------------------------------------------------------- page budget (Eq. 1 / Eq. 2)
def _golden():
    rows = []
    with open(os.path.join(os.path.dirname(__file__), "golden", "page_budget.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append([int(t) for t in line.split()])
    return rows


def test_page_model_matches_paper_figures():
    rows = _golden()
    page = 16 * 1024
    for nbytes, pages in rows[:2]:
        # pages occupied by one iteration's weights = what Eq. 1 yields for that many bytes, no overhead
        assert oracle.pages_available(nbytes, 0, 0, 0, 0, page) == pages
    small, large, st_small, st_large = rows[2]
    # Eq. 1 then Eq. 2 with 4 pages per stage (the un-split 64 KB iteration): 128 KB -> 2 stages;
    # the same demand on 227 KB gives strictly more, and never fewer, stages
    n_small = oracle.pages_available(small * 1024, 1, 0, 0, 0, page)
    n_large = oracle.pages_available(large * 1024, 1, 0, 0, 0, page)
    assert oracle.pipeline_stages(n_small, 0, 0, 0, 4) == st_small
    assert oracle.pipeline_stages(n_large, 0, 0, 0, 4) >= oracle.pipeline_stages(n_small, 0, 0, 0, 4)
    # K-split (2 pages per stage) restores the 4-stage optimum on 128 KB (Sec. 4.3.2 / Fig. 5)
    assert oracle.pipeline_stages(n_small, 0, 0, 0, 2) == st_large
    # floors and the stage overhead term
    assert oracle.pages_available(100, 1, 10, 10, 10, 30) == 2
    assert oracle.pages_available(100, 2, 10, 10, 10, 30) == 1
    assert oracle.pipeline_stages(10, 3, 1, 2, 3) == 1


# ---- W4A16 form of the projections (Sec. 4.3.2; format: see the oracle's header) -----------------

def test_w4_gemv_matches_unpacked_dequantised_matmul():
    rng = np.random.default_rng(5)
    for n_out, n_in, group in ((7, 64, 32), (16, 256, 128), (3, 128, 64)):
        codes = rng.integers(0, 256, size=(n_out, n_in // 2), dtype=np.uint8)
        scales = synth.to_bf16_bits(rng.normal(0.01, 0.003, size=(n_out, n_in // group)).astype(np.float32))
        x = rng.normal(size=n_in).astype(np.float32)
        bias = synth.to_bf16_bits(rng.normal(size=n_out).astype(np.float32))
        want = dequant(codes, scales, group) @ x.astype(np.float64) + synth.bf16_bits_to_f32(bias)
        got = oracle.gemv_w4(codes, scales, group, x, bias)
        assert np.abs(got - want).max() <= 1e-6 * np.abs(want).max()


def test_w4_nibble_order_zero_point_and_group_scale():
    n_out, n_in, group = 4, 64, 32
    codes = np.full((n_out, n_in // 2), 0x88, dtype=np.uint8)       # every code 8: all weights zero
    scales = synth.to_bf16_bits(np.array([[0.5, 2.0]] * n_out, dtype=np.float32))
    x = np.arange(1, n_in + 1, dtype=np.float32)
    assert np.array_equal(oracle.gemv_w4(codes, scales, group, x), np.zeros(n_out, dtype=np.float32))
    c = codes.copy()
    c[1, 3] = 0x8B                # low nibble of byte 3 -> k = 6, code 11 -> +3, first group (scale 0.5)
    assert oracle.gemv_w4(c, scales, group, x)[1] == 3 * 0.5 * x[6]
    c = codes.copy()
    c[2, 20] = 0x28               # high nibble of byte 20 -> k = 41, code 2 -> -6, second group (scale 2)
    y = oracle.gemv_w4(c, scales, group, x)
    assert y[2] == -6 * 2.0 * x[41] and y[0] == 0 and y[1] == 0 and y[3] == 0


def test_w4_step_equals_bf16_step_when_the_dequantised_weights_are_bf16_values():
    """With power-of-two scales every (q - 8) * s is a bf16 value: the W4 decoder must then
    reproduce the bf16 decoder run on those very weights, up to fp64 rounding order."""
    full = dict(synth.CONFIGS["c0_tiny"], intermediate=640, index=11)
    cfg = synth.model_cfg(full)
    w = synth.make_weights(full)
    q = synth.make_quant(full, group=64)
    rng = np.random.default_rng(1)
    for name in synth.W4_NAMES:
        for l in range(cfg["n_layers"]):
            exps = rng.integers(-9, -6, size=q["s_" + name][l].shape)
            q["s_" + name][l] = synth.to_bf16_bits(np.ldexp(1.0, exps).astype(np.float32))
            w[name][l] = synth.to_bf16_bits(dequant(q[name][l], q["s_" + name][l], 64).astype(np.float32))
    a = oracle.Decoder(cfg, w)
    b = oracle.Decoder(cfg, w, quant=q)
    kva, kvb = a.new_kv(), b.new_kv()
    for p, t in enumerate([5, 900, 17, 3000]):
        la = a.step([t], [p], kva)[0]
        lb = b.step([t], [p], kvb)[0]
        assert np.abs(la - lb).max() <= 1e-5 * np.abs(la).max()
    assert np.array_equal(kva, kvb)
