"""The W4A16 weight format written out a second time, for the pins of ``orc_gemv_w4`` (test infrastructure).

Reading of the paper's Sec. 4.3.2 / Sec. 5.1 (GPTQ-W4A16, layout not given): unsigned 4-bit codes q packed two
per byte along K (even k in the low nibble), one bf16 scale s per (row, group of consecutive k), w = (q - 8) s."""
import numpy as np

from paper_2605_11581_amd import synth


def dequant(codes: np.ndarray, scale_bits: np.ndarray, group: int) -> np.ndarray:
    """fp64 weights [out][in] of one W4 matrix given as uint8 codes [out][in/2] and bf16 scale bits [out][in/group]."""
    lo = (codes & 15).astype(np.int64)
    hi = (codes >> 4).astype(np.int64)
    qv = np.stack([lo, hi], axis=-1).reshape(codes.shape[0], -1) - 8
    s = synth.bf16_bits_to_f32(scale_bits).astype(np.float64)
    return qv * np.repeat(s, group, axis=1)
