"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds none of the decoder's arithmetic: it only draws random
numbers and casts them to bf16 with torch's CPU cast (a library routine).  Both
the CPU oracle and the HIP path are fed from the buffers made here.

The paper measures trained GPTQ checkpoints of Qwen3-1.7B / Qwen2.5-1.5B on
fixed 64-token prompts and two public datasets (Sec. 5.2).  None of those is
available offline; the configurations below take the *shapes* of the Qwen2.5 /
Qwen3 decoder family and stand in for them with random-init weights.
"""
from __future__ import annotations

import os
import zlib
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List

import numpy as np
import torch

BASE_SEED = 20260511

# name -> decoder dimensions, flags, and the workload (start context, decode steps)
CONFIGS: Dict[str, Dict] = {
    "c0_tiny": dict(n_layers=2, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64,
                    intermediate=688, vocab=4096, qkv_bias=0, qk_norm=0, tie_embeddings=0,
                    rope_theta=1e4, rms_eps=1e-6, max_batch=1, max_context=192,
                    ctx0=128, steps=32, index=0),
    "c1_0p5b": dict(n_layers=24, hidden=896, n_q_heads=14, n_kv_heads=2, head_dim=64,
                    intermediate=4864, vocab=151936, qkv_bias=1, qk_norm=0, tie_embeddings=1,
                    rope_theta=1e6, rms_eps=1e-6, max_batch=1, max_context=1152,
                    ctx0=1024, steps=128, index=1),
    "c2_1p5b": dict(n_layers=28, hidden=1536, n_q_heads=12, n_kv_heads=2, head_dim=128,
                    intermediate=8960, vocab=151936, qkv_bias=1, qk_norm=0, tie_embeddings=1,
                    rope_theta=1e6, rms_eps=1e-6, max_batch=1, max_context=2304,
                    ctx0=2048, steps=256, index=2),
    "c3_4b": dict(n_layers=36, hidden=2560, n_q_heads=32, n_kv_heads=8, head_dim=128,
                  intermediate=9728, vocab=151936, qkv_bias=0, qk_norm=1, tie_embeddings=0,
                  rope_theta=1e6, rms_eps=1e-6, max_batch=1, max_context=4352,
                  ctx0=4096, steps=256, index=3),
    "c4_7b": dict(n_layers=28, hidden=3584, n_q_heads=28, n_kv_heads=4, head_dim=128,
                  intermediate=18944, vocab=152064, qkv_bias=1, qk_norm=0, tie_embeddings=0,
                  rope_theta=1e6, rms_eps=1e-6, max_batch=8, max_context=8320,
                  ctx0=8192, steps=128, index=4),
    # The paper's own fixed workload (Sec. 5.2: 64-token prompts, 12 generated tokens, batch 1..16) on the
    # second model it measures (Sec. 5.1: Qwen3-1.7B; public dimensions, random-init weights here).
    "c5_1p7b": dict(n_layers=28, hidden=2048, n_q_heads=16, n_kv_heads=8, head_dim=128,
                    intermediate=6144, vocab=151936, qkv_bias=0, qk_norm=1, tie_embeddings=1,
                    rope_theta=1e6, rms_eps=1e-6, max_batch=16, max_context=128,
                    ctx0=64, steps=12, index=5),
}

MODEL_KEYS = ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "intermediate", "vocab",
              "qkv_bias", "qk_norm", "tie_embeddings", "rope_theta", "rms_eps", "max_batch",
              "max_context")


def model_cfg(cfg: Dict, **overrides) -> Dict:
    out = {k: cfg[k] for k in MODEL_KEYS}
    out.update(overrides)
    return out


def seed_of(cfg: Dict) -> int:
    return BASE_SEED + int(cfg.get("index", 0))


def _rng(seed: int, name: str) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, zlib.crc32(name.encode())]))


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16) with torch's CPU cast."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16)
    return t.to(torch.float32).numpy()


def normal_bf16(seed: int, name: str, shape, std: float, mean: float = 0.0) -> np.ndarray:
    """One tensor ~ N(mean, std) as bf16 bits; its stream depends only on (seed, name)."""
    g = _rng(seed, name)
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        blk = g.standard_normal(hi - lo, dtype=np.float32)
        blk *= np.float32(std)
        if mean != 0.0:
            blk += np.float32(mean)
        out[lo:hi] = to_bf16_bits(blk)
    return out.reshape(shape)


def make_weights(cfg: Dict, seed: int | None = None, gain_jitter: float = 0.0,
                 std: float = 0.02) -> Dict:
    """All tensors of one decoder as bf16 bits.

    Matrices and biases ~ N(0, std); norm gains are exactly 1 unless
    ``gain_jitter`` > 0 (then 1 + jitter * N(0,1), used by unit tests so that
    the gain multiply is exercised)."""
    seed = seed_of(cfg) if seed is None else seed
    L, H, d = cfg["n_layers"], cfg["hidden"], cfg["head_dim"]
    qd, kvd, I, V = cfg["n_q_heads"] * d, cfg["n_kv_heads"] * d, cfg["intermediate"], cfg["vocab"]

    def gain(name, n):
        if gain_jitter == 0.0:
            return np.full(n, 0x3F80, dtype=np.uint16)  # bf16(1.0)
        return normal_bf16(seed, name, (n,), gain_jitter, 1.0)

    # every tensor has a random stream of its own, so the tensors can be drawn side by side (numpy's
    # generators release the interpreter lock); the values do not depend on the number of workers
    jobs: Dict[str, tuple] = {"embed": ((V, H), std)}
    if not cfg["tie_embeddings"]:
        jobs["lm_head"] = ((V, H), std)
    mats = {"wq": (qd, H), "wk": (kvd, H), "wv": (kvd, H), "wo": (H, qd), "w_gate": (I, H), "w_up": (I, H), "w_down": (H, I)}
    for l in range(L):
        for k, shp in mats.items():
            jobs[f"l{l}.{k}"] = (shp, std)
        if cfg["qkv_bias"]:
            for k, n in (("bq", qd), ("bk", kvd), ("bv", kvd)):
                jobs[f"l{l}.{k}"] = ((n,), std)
    workers = max(1, min(16, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))))
    with ThreadPoolExecutor(workers) as pool:
        futs = {name: pool.submit(normal_bf16, seed, name, shp, sd) for name, (shp, sd) in jobs.items()}
        drawn = {name: f.result() for name, f in futs.items()}

    w: Dict = {"embed": drawn["embed"], "final_norm": gain("final_norm", H)}
    w["lm_head"] = drawn.get("lm_head")
    per: Dict[str, List] = {k: [] for k in ("attn_norm", "wq", "wk", "wv", "bq", "bk", "bv",
                                            "q_norm", "k_norm", "wo", "mlp_norm", "w_gate", "w_up",
                                            "w_down")}
    for l in range(L):
        per["attn_norm"].append(gain(f"l{l}.attn_norm", H))
        per["mlp_norm"].append(gain(f"l{l}.mlp_norm", H))
        for k in mats:
            per[k].append(drawn[f"l{l}.{k}"])
        if cfg["qkv_bias"]:
            for k in ("bq", "bk", "bv"):
                per[k].append(drawn[f"l{l}.{k}"])
        if cfg["qk_norm"]:
            per["q_norm"].append(gain(f"l{l}.q_norm", d))
            per["k_norm"].append(gain(f"l{l}.k_norm", d))
    for k, v in per.items():
        w[k] = v if v else None
    return w


W4_NAMES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def make_quant(cfg: Dict, group: int = 128, seed: int | None = None, std: float = 0.02) -> Dict:
    """The seven decoder projections in W4A16 form (stand-in for a GPTQ checkpoint): unsigned 4-bit
    codes uniform in [0, 16), packed two per byte (k even in the low nibble), and one bf16 scale
    per (row, group of ``group`` consecutive k) ~ std / 4.6 * (1 + 0.1 N(0,1)), so that the
    dequantised weights (q - 8) * s have about the spread of the bf16 weights.  One Philox stream
    per tensor name.  Keys: ``group``, the projection names (uint8 [out][in/2]) and ``s_<name>``
    (uint16 bf16 bits [out][in/group]); per-layer entries are lists."""
    seed = seed_of(cfg) if seed is None else seed
    L, H, d = cfg["n_layers"], cfg["hidden"], cfg["head_dim"]
    qd, kvd, I = cfg["n_q_heads"] * d, cfg["n_kv_heads"] * d, cfg["intermediate"]
    shapes = {"wq": (qd, H), "wk": (kvd, H), "wv": (kvd, H), "wo": (H, qd), "w_gate": (I, H), "w_up": (I, H),
              "w_down": (H, I)}
    q: Dict = {"group": int(group)}
    for name in W4_NAMES:
        q[name], q["s_" + name] = [], []
    for l in range(L):
        for name in W4_NAMES:
            n_out, n_in = shapes[name]
            assert n_in % group == 0 and n_in % 2 == 0, f"{name}: K = {n_in} is not a multiple of the group size"
            g = _rng(seed, f"l{l}.{name}.q4")
            q[name].append(g.integers(0, 256, size=(n_out, n_in // 2), dtype=np.uint8))
            q["s_" + name].append(normal_bf16(seed, f"l{l}.{name}.s4", (n_out, n_in // group), 0.1 * std / 4.6, std / 4.6))
    return q


def library_weights(w: Dict, q: Dict) -> Dict:
    """The weight dict handed to the library for a W4 schedule: codes replace the seven bf16
    matrices, scales go under sq, sk, sv, so, s_gate, s_up, s_down."""
    out = dict(w)
    for name in W4_NAMES:
        out[name] = q[name]
        out["s" + name[1:]] = q["s_" + name]
    return out


def make_prompt(cfg: Dict, n: int, seed: int | None = None, name: str = "prompt") -> np.ndarray:
    seed = seed_of(cfg) if seed is None else seed
    return _rng(seed, name).integers(0, cfg["vocab"], size=n, dtype=np.int32)


def kv_shape(cfg: Dict):
    return (cfg["n_layers"], 2, cfg["max_batch"], cfg["n_kv_heads"], cfg["max_context"],
            cfg["head_dim"])


def make_kv_fill(cfg: Dict, ctx0: int, seed: int | None = None, batch: int | None = None) -> np.ndarray:
    """KV cache with positions [0, ctx0) of the first ``batch`` sequences ~ bf16(N(0,1)); rest 0."""
    seed = seed_of(cfg) if seed is None else seed
    batch = cfg["max_batch"] if batch is None else batch
    L, _, Bm, nkv, Tm, d = kv_shape(cfg)
    kv = np.zeros(kv_shape(cfg), dtype=np.uint16)
    for l in range(L):
        for which in range(2):
            kv[l, which, :batch, :, :ctx0, :] = normal_bf16(
                seed, f"kv.{l}.{which}", (batch, nkv, ctx0, d), 1.0)
    return kv
