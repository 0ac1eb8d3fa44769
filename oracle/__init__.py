"""ctypes front end of the CPU oracle (``decoder_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by
the benchmark's ``cpu_baseline`` leg.  It shares nothing with the HIP path and
the product package never imports it.

The oracle is the plain definition of one decoder step (the computation the
paper fuses into its megakernel, Sec. 3 Phase I / Sec. 4.2.3) in fp32 storage
with fp64 accumulation.  Weights are passed as ``numpy.uint16`` arrays holding
bf16 bit patterns; the KV cache is a ``numpy.uint16`` array laid out
``[layer][2][max_batch][n_kv_heads][max_context][head_dim]``.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "decoder_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over output rows only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "intermediate", "vocab",
        "qkv_bias", "qk_norm", "tie_embeddings")] + [
        ("rope_theta", C.c_float), ("rms_eps", C.c_float),
        ("max_batch", C.c_int32), ("max_context", C.c_int32)]


_PP = C.POINTER(C.c_void_p)


class _Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p)] + [
        (n, _PP) for n in ("attn_norm", "wq", "wk", "wv", "bq", "bk", "bv", "q_norm", "k_norm",
                           "wo", "mlp_norm", "w_gate", "w_up", "w_down")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.orc_bf16_to_f32.restype = C.c_float
        L.orc_bf16_to_f32.argtypes = [C.c_uint16]
        L.orc_f32_to_bf16.restype = C.c_uint16
        L.orc_f32_to_bf16.argtypes = [C.c_float]
        L.orc_silu.restype = C.c_float
        L.orc_silu.argtypes = [C.c_float]
        L.orc_rmsnorm.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_float, C.c_void_p]
        L.orc_gemv.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_rope.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_float]
        L.orc_softmax.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
        L.orc_attend.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        L.orc_argmax.restype = C.c_int32
        L.orc_argmax.argtypes = [C.c_void_p, C.c_int]
        L.orc_decode_step.restype = C.c_int
        L.orc_decode_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p]
        L.orc_decode_step_q.restype = C.c_int
        L.orc_decode_step_q.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_void_p]
        L.orc_gemv_w4.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_pages_available.restype = C.c_int64
        L.orc_pages_available.argtypes = [C.c_int64] * 6
        L.orc_pipeline_stages.restype = C.c_int64
        L.orc_pipeline_stages.argtypes = [C.c_int64] * 5
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, "bf16 data is passed as uint16 bit patterns"
    return a


# ---- scalar / vector operators ------------------------------------------------

def bf16_to_f32(bits) -> np.ndarray:
    bits = np.asarray(bits, dtype=np.uint16)
    return np.array([lib().orc_bf16_to_f32(int(b)) for b in bits.ravel()],
                    dtype=np.float32).reshape(bits.shape)


def f32_to_bf16(vals) -> np.ndarray:
    vals = np.asarray(vals, dtype=np.float32)
    return np.array([lib().orc_f32_to_bf16(float(v)) for v in vals.ravel()],
                    dtype=np.uint16).reshape(vals.shape)


def silu(z: float) -> float:
    return float(lib().orc_silu(float(z)))


def rmsnorm(x, g_bits, eps: float) -> np.ndarray:
    x = _f32(x); g = _u16(g_bits)
    y = np.empty_like(x)
    lib().orc_rmsnorm(_p(x), _p(g), x.size, eps, _p(y))
    return y


def gemv(w_bits, x, bias_bits=None) -> np.ndarray:
    w = _u16(w_bits); x = _f32(x)
    n_out, n_in = w.shape
    assert x.size == n_in
    b = None if bias_bits is None else _u16(bias_bits)
    y = np.empty(n_out, dtype=np.float32)
    lib().orc_gemv(_p(w), n_out, n_in, _p(x), _p(b), _p(y))
    return y


def rope(u, pos: int, theta: float) -> np.ndarray:
    u = _f32(u).copy()
    lib().orc_rope(_p(u), u.size, int(pos), float(theta))
    return u


def softmax(s) -> np.ndarray:
    s = _f32(s)
    w = np.empty_like(s)
    lib().orc_softmax(_p(s), s.size, _p(w))
    return w


def attend(q, k_bits, v_bits) -> np.ndarray:
    q = _f32(q); k = _u16(k_bits); v = _u16(v_bits)
    T, d = k.shape
    assert v.shape == (T, d) and q.size == d
    o = np.empty(d, dtype=np.float32)
    lib().orc_attend(_p(q), _p(k), _p(v), T, d, _p(o))
    return o


def argmax(v) -> int:
    v = _f32(v)
    return int(lib().orc_argmax(_p(v), v.size))


def pages_available(smem_max, n_stage, instr_buf, semaphores, scratch, page_size) -> int:
    return int(lib().orc_pages_available(smem_max, n_stage, instr_buf, semaphores, scratch, page_size))


def pipeline_stages(pages_total, pages_weight, pages_scale, pages_act, pages_per_stage) -> int:
    return int(lib().orc_pipeline_stages(pages_total, pages_weight, pages_scale, pages_act,
                                         pages_per_stage))


# ---- the decoder ---------------------------------------------------------------

_CFG_KEYS = ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "intermediate", "vocab",
             "qkv_bias", "qk_norm", "tie_embeddings", "rope_theta", "rms_eps", "max_batch",
             "max_context")
_LAYER_KEYS = ("attn_norm", "wq", "wk", "wv", "bq", "bk", "bv", "q_norm", "k_norm", "wo",
               "mlp_norm", "w_gate", "w_up", "w_down")


_W4_KEYS = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


class _W4(C.Structure):
    _fields_ = [("group", C.c_int32)] + [(k, _PP) for k in _W4_KEYS] + [
        ("s" + k[1:] if k[1] != "_" else "s" + k[1:], _PP) for k in _W4_KEYS]


def gemv_w4(codes, scales_bits, group: int, x, bias_bits=None) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    sc = _u16(scales_bits)
    x = _f32(x)
    n_out, half = codes.shape
    assert sc.shape == (n_out, 2 * half // group)
    b = _u16(bias_bits) if bias_bits is not None else None
    y = np.empty(n_out, dtype=np.float32)
    lib().orc_gemv_w4(_p(codes), _p(sc), n_out, 2 * half, int(group), _p(x), _p(b), _p(y))
    return y


@dataclass
class Decoder:
    """Holds a config + weights (dict of uint16 arrays; per-layer entries are lists).  With ``quant``
    (dict: ``group``, uint8 code arrays under the seven projection names, bf16 scale arrays under
    ``s_<name>``) those projections are taken in their W4A16 form."""
    cfg: Dict
    weights: Dict
    quant: Optional[Dict] = None

    def __post_init__(self):
        c = self.cfg
        self._c = _Config(**{k: c[k] for k in _CFG_KEYS})
        w = self.weights
        L = c["n_layers"]
        self._keep = []
        ws = _Weights()
        ws.embed = _p(_u16(w["embed"]))
        ws.lm_head = _p(_u16(w["lm_head"])) if w.get("lm_head") is not None else None
        ws.final_norm = _p(_u16(w["final_norm"]))
        for key in _LAYER_KEYS:
            arrs = w.get(key)
            if arrs is None:
                setattr(ws, key, None)
                continue
            assert len(arrs) == L
            tab = (C.c_void_p * L)(*[_u16(a).ctypes.data for a in arrs])
            self._keep.append(tab)
            setattr(ws, key, C.cast(tab, _PP))
        self._w = ws
        self._q = None
        if self.quant is not None:
            q4 = _W4()
            q4.group = int(self.quant["group"])
            for key in _W4_KEYS:
                skey = "s" + key[1:]
                codes = [np.ascontiguousarray(a, dtype=np.uint8) for a in self.quant[key]]
                scales = [_u16(a) for a in self.quant["s_" + key]]
                assert len(codes) == L and len(scales) == L
                tc = (C.c_void_p * L)(*[a.ctypes.data for a in codes])
                ts = (C.c_void_p * L)(*[a.ctypes.data for a in scales])
                self._keep += [codes, scales, tc, ts]
                setattr(q4, key, C.cast(tc, _PP))
                setattr(q4, skey, C.cast(ts, _PP))
            self._q = q4

    def kv_shape(self):
        c = self.cfg
        return (c["n_layers"], 2, c["max_batch"], c["n_kv_heads"], c["max_context"], c["head_dim"])

    def new_kv(self) -> np.ndarray:
        return np.zeros(self.kv_shape(), dtype=np.uint16)

    def step(self, tokens, positions, kv: np.ndarray, want_logits: bool = True):
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        positions = np.ascontiguousarray(positions, dtype=np.int32)
        B = tokens.size
        assert kv.dtype == np.uint16 and kv.shape == self.kv_shape() and kv.flags.c_contiguous
        logits = np.empty((B, self.cfg["vocab"]), dtype=np.float32) if want_logits else None
        rc = lib().orc_decode_step_q(C.byref(self._c), C.byref(self._w), C.byref(self._q) if self._q is not None else None,
                                     B, _p(tokens), _p(positions), _p(kv), _p(logits))
        if rc != 0:
            raise ValueError("orc_decode_step rejected its arguments")
        return logits

    def prefill(self, prompt, kv: np.ndarray, b: int = 0):
        """Token-by-token prefill of sequence 0 (batch 1 handles only b == 0)."""
        assert b == 0
        for p, t in enumerate(prompt):
            self.step([int(t)], [p], kv, want_logits=False)
