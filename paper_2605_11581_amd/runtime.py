"""Convenience wrapper: allocates the workspace with torch, uploads host weights, steps.

Only memory management and call sequencing live here; all arithmetic is in libmk.so."""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from . import binding as mk


def _dev_bits(a, device) -> torch.Tensor:
    if isinstance(a, torch.Tensor):
        return a
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint8:          # packed 4-bit codes
        return torch.from_numpy(a).to(device)
    return torch.from_numpy(a.view(np.int16)).to(device)


def stage_weights(w: Dict, device) -> Dict:
    """Upload host weights (numpy uint16 bf16 bit patterns; per-layer entries are lists) once, for
    callers that load the same tensors into several schedules."""
    dev: Dict = {}
    for k, v in w.items():
        if v is None:
            dev[k] = None
        elif isinstance(v, (list, tuple)):
            dev[k] = [_dev_bits(a, device) for a in v]
        else:
            dev[k] = _dev_bits(v, device)
    return dev


class Decoder:
    def __init__(self, model: Dict, device: str = "cuda:0", schedule_blob: Optional[bytes] = None, **opts):
        """``opts`` are fields of ``mk_config``; tiling parameters not given come from the library's own
        choice (the profiled tiling recorded for this deployment configuration, else its cost-model search)."""
        self.device = torch.device(device)
        self.model = dict(model)
        if schedule_blob is not None:
            self.h = mk.mk_schedule_load(schedule_blob)
        else:
            self.h = mk.mk_build_schedule(mk.make_config(model, device_id=self.device.index or 0, **opts))
        self.stats = mk.mk_get_stats(self.h)
        self.workspace = torch.empty(mk.mk_workspace_bytes(self.h), dtype=torch.uint8, device=self.device)
        mk.mk_bind_workspace(self.h, self.workspace)

    def load_weights(self, w: Dict) -> None:
        """``w``: numpy uint16 bf16 bit patterns or int16 device tensors (per-layer entries are lists)."""
        dev = stage_weights(w, self.device)
        mk.mk_load_weights(self.h, dev)
        torch.cuda.synchronize(self.device)   # the staged copies may be freed now

    def new_kv(self, host: Optional[np.ndarray] = None) -> torch.Tensor:
        m = self.model
        shape = (m["n_layers"], 2, m["max_batch"], m["n_kv_heads"], m["max_context"], m["head_dim"])
        if host is None:
            return torch.zeros(shape, dtype=torch.int16, device=self.device)
        assert host.shape == shape
        return _dev_bits(host, self.device)

    def step(self, tokens: torch.Tensor, positions: torch.Tensor, kv: torch.Tensor, logits: torch.Tensor,
             per_op: bool = False, stream=None) -> None:
        fn = mk.mk_decode_step_per_op if per_op else mk.mk_decode_step
        fn(self.h, tokens, positions, kv, logits, int(tokens.numel()), stream)

    def fill_cache(self, tokens: torch.Tensor, positions: torch.Tensor, kv: torch.Tensor) -> None:
        """Appends the K/V rows of ``tokens`` [n_tokens][batch] (int32, device), sequence b starting at ``positions[b]``:
        the decode path used as a prefill, one launch, no logits."""
        n_tokens, batch = int(tokens.shape[0]), int(tokens.shape[1])
        mk.mk_fill_cache(self.h, tokens.contiguous(), positions, kv, batch, n_tokens)

    def greedy(self, tokens: torch.Tensor, positions: torch.Tensor, kv: torch.Tensor, logits: torch.Tensor,
               n_steps: int) -> torch.Tensor:
        """``n_steps`` greedy decode steps in ONE launch; returns the chosen tokens [n_steps][batch] (int32, device)."""
        out = torch.empty(n_steps, int(tokens.numel()), dtype=torch.int32, device=self.device)
        mk.mk_decode_steps(self.h, tokens, positions, kv, logits, out, int(tokens.numel()), n_steps)
        return out

    def check(self) -> None:
        mk.mk_check(self.h)

    def close(self) -> None:
        if self.h is not None:
            mk.mk_destroy(self.h)
            self.h = None
