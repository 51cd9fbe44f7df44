"""Shared test helpers (CPU side): tiny models and oracle parameter sets."""
from dataclasses import replace

import numpy as np

import sb_inputs as si
from oracle import Oracle, OrcParams


def tiny_model(n_layers=4, n_exit_heads=2, seed=1001, gain_jitter=0.1, max_seq=160, bits=64, **kw):
    shape = si.tiny_shape(n_layers=n_layers, n_exit_heads=n_exit_heads, **kw)
    w = si.make_weights(shape, seed, gain_jitter=gain_jitter)
    return shape, w, Oracle(shape, w, max_seq, bits=bits)


def linear_T(d_max, first=2.0, last=1.0):
    if d_max <= 1:
        return [first] * max(d_max, 0)
    return [first + (last - first) * i / (d_max - 1) for i in range(d_max)]


def params(d_max, w_max, threshold=0.5, forced_exit=None, forced_draft=None, T=None, eos_id=-1):
    return OrcParams(d_max, w_max, linear_T(d_max) if T is None else T, threshold,
                     forced_exit=forced_exit, forced_draft=forced_draft, eos_id=eos_id)


def all_accept_weights(shape, w, k):
    """Zero W_o and W_down of layers > k and alias every exit head to the final
    norm + LM head: every hidden state from layer k on equals the final one, so a
    draft that exits at a layer >= k is the full model's greedy token."""
    w = dict(w)
    for l in range(k, shape.n_layers):
        w[f"w_o.{l}"] = np.zeros_like(w[f"w_o.{l}"])
        w[f"w_down.{l}"] = np.zeros_like(w[f"w_down.{l}"])
    for l in range(shape.n_exit_heads):
        w[f"exit_head.{l}"] = w["lm_head"]
        w[f"exit_norm.{l}"] = w["final_norm"]
    return w


# ---------------------------------------------------------------- GPU side
def gpu_model(shape, w, max_seq, proj=0):
    import paper_2604_12247_amd as sb
    return sb.Model(shape, w, max_seq, proj_kernel=proj)


def gpu_params(d_max, w_max, threshold=0.5, forced_exit=None, forced_draft=None, T=None, eos_id=-1):
    import paper_2604_12247_amd as sb
    return sb.Params(d_max, w_max, linear_T(d_max) if T is None else T, threshold,
                     forced_exit=forced_exit, forced_draft=forced_draft, eos_id=eos_id)


def teacher_forced_check(oracle_model, prompt, gpu_tokens, gap_tol=1e-2):
    """Score the GPU's output with the oracle position by position.  A position
    passes if the GPU token is the oracle's arg max, or the oracle's logit gap
    between its arg max and the GPU token is below gap_tol (flagged near-tie).
    Returns (n_flagged, n_scored); raises on a real mismatch."""
    s = oracle_model.session()
    first = s.prefill(prompt)
    z = s.verify_logits(0)
    flagged = 0
    toks = list(gpu_tokens)
    for i, t in enumerate(toks):
        am = int(np.argmax(z))
        if t != am:
            gap = z[am] - z[t]
            assert gap < gap_tol, f"position {i}: gpu token {t}, oracle {am}, logit gap {gap}"
            flagged += 1
        if i + 1 < len(toks):
            _, z = s.step(t)
    return flagged, len(toks)
