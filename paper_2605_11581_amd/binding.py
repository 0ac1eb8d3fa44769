"""ctypes binding of libmk.so: same names as include/mk.h, argument marshalling only.

Every step of the decode path runs inside the library's HIP kernels.  There is
no CPU or PyTorch fallback: if the shared library is missing or fails to load,
importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("MK_LIB_PATH") or os.path.join(_HERE, "libmk.so")   # override: A/B runs of two builds

MK_OK, MK_EINVAL, MK_ENOMEM, MK_EINFEASIBLE, MK_ESCHED, MK_EHIP, MK_ETIMEOUT, MK_ESTATE = 0, -1, -2, -3, -4, -5, -6, -7
MK_F_TRACE, MK_F_TIMING, MK_F_NO_TABLE = 1, 2, 4
INSTR_DWORDS = 32


class MkError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libmk error {code}: {text}")
        self.code = code


class mk_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim",
                                         "intermediate", "vocab", "qkv_bias", "qk_norm", "tie_embeddings")] + [
        ("rope_theta", C.c_float), ("rms_eps", C.c_float)] + [
        (n, C.c_int32) for n in ("max_batch", "max_context", "n_workgroups", "device_id", "use_mfma", "ring_kb",
                                 "split_qkv", "split_o", "split_gateup", "split_down", "attn_chunks", "chunk_rows",
                                 "rows_qkv", "rows_o", "rows_gateup", "rows_down", "rows_head", "fuse_combine", "weight_bits",
                                 "group_size")] + [
        ("spin_limit", C.c_uint32), ("flags", C.c_uint32)]


_PP = C.POINTER(C.c_void_p)


class mk_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p)] + [
        (n, _PP) for n in ("attn_norm", "wq", "wk", "wv", "bq", "bk", "bv", "q_norm", "k_norm", "wo", "mlp_norm",
                           "w_gate", "w_up", "w_down", "sq", "sk", "sv", "so", "s_gate", "s_up", "s_down")]


class mk_stats(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_workgroups", "threads_per_wg", "n_tasks", "n_counters", "max_instr_per_wg",
                                         "split_qkv", "split_o", "split_gateup", "split_down", "attn_chunks", "use_mfma",
                                         "lds_bytes", "ring_pages", "page_bytes", "n_stage")] + [
        ("_pad", C.c_int32), ("weight_bytes_per_step", C.c_int64), ("workspace_bytes", C.c_int64),
        ("sim_makespan_us", C.c_double), ("sim_duty_cycle", C.c_double),
        ("candidates_tried", C.c_int32), ("candidates_pruned", C.c_int32)] + [
        (n, C.c_int32) for n in ("rows_qkv", "rows_o", "rows_gateup", "rows_down", "rows_head", "fuse_combine", "from_table",
                                 "attention_mfma")]


EXPORTS = ("mk_build_schedule", "mk_schedule_verify", "mk_schedule_dump", "mk_schedule_load", "mk_get_stats",
           "mk_get_config", "mk_instr_count", "mk_instr_get", "mk_instr_set", "mk_pages_available",
           "mk_pipeline_stages", "mk_workspace_bytes", "mk_bind_workspace", "mk_load_weights", "mk_decode_step",
           "mk_decode_steps", "mk_decode_step_per_op", "mk_decode_step_static", "mk_fill_cache", "mk_check", "mk_last_step_ms", "mk_read_ceiling", "mk_set_flags", "mk_read_trace", "mk_destroy", "mk_last_error")

_lib = None


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """Load libmk.so (built in-tree by ``__graft_entry__.build()`` / ``build.py``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2605_11581_amd.build` "
                              "(there is no fallback path)")
        # torch brings its own HIP runtime: let it load first, so that this library binds to the same one
        # (two runtimes in one process do not see the device)
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(_LIB_PATH)
        H = C.c_void_p
        L.mk_last_error.restype = C.c_char_p
        L.mk_build_schedule.argtypes = [C.POINTER(mk_config), C.POINTER(H)]
        L.mk_schedule_verify.argtypes = [H]
        L.mk_schedule_dump.argtypes = [H, C.c_void_p, C.POINTER(C.c_size_t)]
        L.mk_schedule_load.argtypes = [C.c_void_p, C.c_size_t, C.POINTER(H)]
        L.mk_get_stats.argtypes = [H, C.POINTER(mk_stats)]
        L.mk_get_config.argtypes = [H, C.POINTER(mk_config)]
        L.mk_instr_count.argtypes = [H, C.c_int32]
        L.mk_instr_get.argtypes = [H, C.c_int32, C.c_int32, C.c_void_p]
        L.mk_instr_set.argtypes = [H, C.c_int32, C.c_int32, C.c_void_p]
        L.mk_pages_available.restype = C.c_int64
        L.mk_pages_available.argtypes = [C.c_int64] * 6
        L.mk_pipeline_stages.restype = C.c_int64
        L.mk_pipeline_stages.argtypes = [C.c_int64] * 5
        L.mk_workspace_bytes.restype = C.c_size_t
        L.mk_workspace_bytes.argtypes = [H]
        L.mk_bind_workspace.argtypes = [H, C.c_void_p, C.c_size_t, C.c_void_p]
        L.mk_load_weights.argtypes = [H, C.POINTER(mk_weights), C.c_void_p]
        for n in ("mk_decode_step", "mk_decode_step_per_op", "mk_decode_step_static"):
            getattr(L, n).argtypes = [H, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
        L.mk_decode_steps.argtypes = [H, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                      C.c_void_p]
        if hasattr(L, "mk_fill_cache"):      # (absent from older builds loaded through MK_LIB_PATH for A/B runs)
            L.mk_fill_cache.argtypes = [H, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        L.mk_check.argtypes = [H, C.c_void_p]
        L.mk_last_step_ms.argtypes = [H, C.POINTER(C.c_float)]
        L.mk_read_ceiling.argtypes = [H, C.c_int32, C.POINTER(C.c_float), C.POINTER(C.c_size_t), C.c_void_p]
        L.mk_set_flags.argtypes = [H, C.c_uint32]
        L.mk_read_trace.argtypes = [H, C.c_void_p, C.POINTER(C.c_size_t), C.c_void_p]
        L.mk_destroy.argtypes = [H]
        L.mk_destroy.restype = None
        _lib = L
    return _lib


def mk_last_error() -> str:
    return lib().mk_last_error().decode()


def _chk(rc: int) -> None:
    if rc != 0:
        raise MkError(rc, mk_last_error())


_CFG_DEFAULTS = dict(n_workgroups=0, device_id=0, use_mfma=-1, ring_kb=-1, split_qkv=0, split_o=0, split_gateup=0,
                     split_down=0, attn_chunks=0, chunk_rows=0, rows_qkv=0, rows_o=0, rows_gateup=0, rows_down=0,
                     rows_head=0, fuse_combine=-1, weight_bits=16, group_size=0, spin_limit=0, flags=0)


def make_config(model: Dict, **opts) -> mk_config:
    vals = dict(_CFG_DEFAULTS)
    vals.update({k: model[k] for k in model if k in {f[0] for f in mk_config._fields_}})
    vals.update(opts)
    return mk_config(**vals)


def mk_build_schedule(cfg: mk_config) -> C.c_void_p:
    h = C.c_void_p()
    _chk(lib().mk_build_schedule(C.byref(cfg), C.byref(h)))
    return h


def mk_schedule_verify(h) -> None:
    _chk(lib().mk_schedule_verify(h))


def mk_schedule_dump(h) -> bytes:
    n = C.c_size_t(0)
    _chk(lib().mk_schedule_dump(h, None, C.byref(n)))
    buf = C.create_string_buffer(n.value)
    _chk(lib().mk_schedule_dump(h, buf, C.byref(n)))
    return buf.raw[: n.value]


def mk_schedule_load(blob: bytes) -> C.c_void_p:
    h = C.c_void_p()
    _chk(lib().mk_schedule_load(blob, len(blob), C.byref(h)))
    return h


def mk_get_stats(h) -> Dict:
    st = mk_stats()
    _chk(lib().mk_get_stats(h, C.byref(st)))
    return {f[0]: getattr(st, f[0]) for f in mk_stats._fields_ if f[0] not in ("_pad", "reserved")}


def mk_get_config(h) -> mk_config:
    c = mk_config()
    _chk(lib().mk_get_config(h, C.byref(c)))
    return c


def mk_instr_count(h, wg: int) -> int:
    n = lib().mk_instr_count(h, wg)
    if n < 0:
        _chk(n)
    return n


def mk_instr_get(h, wg: int, idx: int) -> np.ndarray:
    out = np.zeros(INSTR_DWORDS, dtype=np.uint32)
    _chk(lib().mk_instr_get(h, wg, idx, out.ctypes.data_as(C.c_void_p)))
    return out


def mk_instr_set(h, wg: int, idx: int, words: np.ndarray) -> None:
    words = np.ascontiguousarray(words, dtype=np.uint32)
    assert words.size == INSTR_DWORDS
    _chk(lib().mk_instr_set(h, wg, idx, words.ctypes.data_as(C.c_void_p)))


def mk_pages_available(smem_max, n_stage, instr_buf, semaphores, scratch, page_size) -> int:
    return int(lib().mk_pages_available(smem_max, n_stage, instr_buf, semaphores, scratch, page_size))


def mk_pipeline_stages(pages_total, pages_weight, pages_scale, pages_act, pages_per_stage) -> int:
    return int(lib().mk_pipeline_stages(pages_total, pages_weight, pages_scale, pages_act, pages_per_stage))


def mk_workspace_bytes(h) -> int:
    return int(lib().mk_workspace_bytes(h))


def _ptr(t) -> Optional[int]:
    """Device pointer of a torch tensor (or None)."""
    return None if t is None else int(t.data_ptr())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)
    return int(getattr(stream, "cuda_stream", stream))


def mk_bind_workspace(h, workspace, stream=None) -> None:
    _chk(lib().mk_bind_workspace(h, _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def mk_load_weights(h, w: Dict, stream=None) -> None:
    """``w``: dict of torch device tensors (bf16 or int16/uint16 bit patterns); per-layer entries are lists."""
    ws = mk_weights()
    keep = []
    ws.embed = _ptr(w["embed"])
    ws.lm_head = _ptr(w.get("lm_head"))
    ws.final_norm = _ptr(w["final_norm"])
    for key in ("attn_norm", "wq", "wk", "wv", "bq", "bk", "bv", "q_norm", "k_norm", "wo", "mlp_norm", "w_gate",
                "w_up", "w_down", "sq", "sk", "sv", "so", "s_gate", "s_up", "s_down"):
        arrs: Optional[Sequence] = w.get(key)
        if arrs is None:
            setattr(ws, key, None)
            continue
        tab = (C.c_void_p * len(arrs))(*[_ptr(a) for a in arrs])
        keep.append(tab)
        setattr(ws, key, C.cast(tab, _PP))
    _chk(lib().mk_load_weights(h, C.byref(ws), _stream(stream)))


def mk_decode_step(h, token_ids, positions, kv_cache, logits_out, batch: int, stream=None) -> None:
    _chk(lib().mk_decode_step(h, _ptr(token_ids), _ptr(positions), _ptr(kv_cache), _ptr(logits_out), batch,
                              _stream(stream)))


def mk_decode_steps(h, token_ids, positions, kv_cache, logits_out, tokens_out, batch: int, n_steps: int, stream=None) -> None:
    _chk(lib().mk_decode_steps(h, _ptr(token_ids), _ptr(positions), _ptr(kv_cache), _ptr(logits_out), _ptr(tokens_out),
                               batch, n_steps, _stream(stream)))


def mk_fill_cache(h, token_ids, positions, kv_cache, batch: int, n_tokens: int, stream=None) -> None:
    _chk(lib().mk_fill_cache(h, _ptr(token_ids), _ptr(positions), _ptr(kv_cache), int(batch), int(n_tokens), _stream(stream)))


def mk_decode_step_static(h, token_ids, positions, kv_cache, logits_out, batch: int, stream=None) -> None:
    _chk(lib().mk_decode_step_static(h, _ptr(token_ids), _ptr(positions), _ptr(kv_cache), _ptr(logits_out), batch,
                                     _stream(stream)))


def mk_decode_step_per_op(h, token_ids, positions, kv_cache, logits_out, batch: int, stream=None) -> None:
    _chk(lib().mk_decode_step_per_op(h, _ptr(token_ids), _ptr(positions), _ptr(kv_cache), _ptr(logits_out), batch,
                                     _stream(stream)))


def mk_check(h, stream=None) -> None:
    _chk(lib().mk_check(h, _stream(stream)))


def mk_last_step_ms(h) -> float:
    ms = C.c_float(0)
    _chk(lib().mk_last_step_ms(h, C.byref(ms)))
    return float(ms.value)


def mk_read_ceiling(h, reps: int = 5, stream=None):
    """(durations in ms of ``reps`` launches of the streaming-read kernel, bytes each launch read)."""
    ms = (C.c_float * reps)()
    n = C.c_size_t(0)
    _chk(lib().mk_read_ceiling(h, reps, ms, C.byref(n), _stream(stream)))
    return [float(x) for x in ms], int(n.value)


def mk_set_flags(h, flags: int) -> None:
    _chk(lib().mk_set_flags(h, flags))


def mk_read_trace(h, stream=None) -> np.ndarray:
    st = mk_get_stats(h)
    cap = st["n_workgroups"] * (st["max_instr_per_wg"] + 1)
    out = np.zeros((cap, 8), dtype=np.uint64)
    n = C.c_size_t(cap)
    _chk(lib().mk_read_trace(h, out.ctypes.data_as(C.c_void_p), C.byref(n), _stream(stream)))
    return out[: n.value]


def mk_destroy(h) -> None:
    lib().mk_destroy(h)
