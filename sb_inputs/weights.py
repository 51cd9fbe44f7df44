"""Seeded random-init weights of a LLaMA-style decoder with per-layer exit heads.

Every matrix is N(0, 0.02) from a counter-based generator keyed by
(seed, tensor id, chunk); output projections (attention W_o and FFN W_down) use
std 0.02/sqrt(2*n_layers).  Norm gains are 1 (optionally jittered for tests so
that a wrong gain vector cannot hide).  For bf16 configurations the float32
draws are rounded to bf16 (round-to-nearest-even) and stored as uint16.
"""
from concurrent.futures import ThreadPoolExecutor
import math
import os
from typing import Dict, List, Tuple

import numpy as np

from .configs import BF16, ModelShape

_CHUNK = 1 << 22  # elements per independently keyed chunk


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern (uint16), round to nearest even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def tensor_specs(shape: ModelShape) -> List[Tuple[str, Tuple[int, ...], float]]:
    """(name, shape, std) of every random matrix, in a fixed order (index = tensor id)."""
    d, f, V = shape.d_model, shape.d_ffn, shape.vocab
    out_std = 0.02 / math.sqrt(2.0 * shape.n_layers)
    specs = [("embed", (V, d), 0.02), ("lm_head", (V, d), 0.02)]
    for l in range(shape.n_layers):
        specs += [
            (f"w_qkv.{l}", (shape.qkv_rows, d), 0.02),
            (f"w_o.{l}", (d, shape.n_heads * shape.head_dim), out_std),
            (f"w_gate_up.{l}", (2 * f, d), 0.02),
            (f"w_down.{l}", (d, f), out_std),
        ]
    for l in range(shape.n_exit_heads):
        specs.append((f"exit_head.{l}", (V, d), 0.02))
    return specs


def _norm_names(shape: ModelShape) -> List[str]:
    names = ["final_norm"]
    for l in range(shape.n_layers):
        names += [f"attn_norm.{l}", f"ffn_norm.{l}"]
    for l in range(shape.n_exit_heads):
        names.append(f"exit_norm.{l}")
    return names


def make_weights(shape: ModelShape, seed: int, gain_jitter: float = 0.0,
                 n_threads: int = 0) -> Dict[str, np.ndarray]:
    """Return {name: array}.  Matrices are uint16 (bf16 bits) or float32, row-major
    [out, in]; w_gate_up stacks the gate rows above the up rows; w_qkv stacks
    q heads, then k heads, then v heads.  Norm gains are float32 vectors."""
    specs = tensor_specs(shape)
    bf16 = shape.weight_dtype == BF16
    out: Dict[str, np.ndarray] = {}
    jobs = []
    for tid, (name, shp, std) in enumerate(specs):
        n = int(np.prod(shp))
        arr = np.empty(n, dtype=np.uint16 if bf16 else np.float32)
        out[name] = arr.reshape(shp)
        for c, lo in enumerate(range(0, n, _CHUNK)):
            jobs.append((arr, lo, min(lo + _CHUNK, n), tid, c, std))

    def run(job):
        arr, lo, hi, tid, c, std = job
        g = np.random.Generator(np.random.Philox(key=[seed, (tid << 24) | c]))
        x = g.standard_normal(hi - lo, dtype=np.float32)
        x *= np.float32(std)
        arr[lo:hi] = round_to_bf16(x) if bf16 else x

    nt = n_threads or min(16, len(os.sched_getaffinity(0)) or 1)
    if nt > 1 and len(jobs) > 1:
        with ThreadPoolExecutor(nt) as ex:
            list(ex.map(run, jobs))
    else:
        for j in jobs:
            run(j)

    gj = np.random.Generator(np.random.Philox(key=[seed, (1 << 60)]))
    for name in _norm_names(shape):
        g = np.ones(shape.d_model, dtype=np.float32)
        if gain_jitter:
            g += gain_jitter * gj.standard_normal(shape.d_model, dtype=np.float32)
            g = bf16_to_f32(round_to_bf16(g)) if bf16 else g
        out[name] = g
    return out


def easy_token_weights(shape: ModelShape, weights: Dict[str, np.ndarray], decay: float = 0.5,
                       head_scale: float = 20.0, ramp: float = 0.0) -> Dict[str, np.ndarray]:
    """A structured variant of `weights` on which computed exits fire and drafts are often
    right (random heads never agree with the final head): the output projections of layer l
    (0-based) are scaled by decay**l, so deeper layers refine the hidden state less and less;
    every exit head is the final head (same matrix), with the final norm's gains times
    head_scale so that the soft-max is peaked enough for a confidence test to decide.
    ramp in [0, 1] makes shallow heads less peaked than deep ones (head l of n gets
    head_scale * (1 - ramp * (1 - l / n)), l = 1..n), which spreads the exits over the layers.
    A power-of-two decay keeps bf16 weights exact.  Returns a new dict (shares the untouched
    arrays)."""
    bf16 = shape.weight_dtype == BF16
    out = dict(weights)
    for l in range(shape.n_layers):
        s = np.float32(decay ** l)
        for name in (f"w_o.{l}", f"w_down.{l}"):
            a = bf16_to_f32(weights[name]) if bf16 else weights[name]
            a = a * s
            out[name] = round_to_bf16(a) if bf16 else a.astype(np.float32)
    for l in range(shape.n_exit_heads):
        out[f"exit_head.{l}"] = weights["lm_head"]
        hs = head_scale * (1.0 - ramp * (1.0 - (l + 1) / shape.n_exit_heads))
        out[f"exit_norm.{l}"] = (weights["final_norm"] * np.float32(hs)).astype(np.float32)
    return out
