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


def progress(msg):
    """A progress line on stdout and in test_progress.log under the folder SB_PROGRESS_DIR names
    (default: the run-output folder at the repository root), so that a long full-size test
    that prints nothing for minutes is not mistaken for a hung one."""
    import os, time
    print(msg, flush=True)
    d = os.environ.get("SB_PROGRESS_DIR") or os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                                                          "gpurun_out")
    try:
        os.makedirs(d, exist_ok=True)
        with open(os.path.join(d, "test_progress.log"), "a") as f:
            f.write(f"{time.strftime('%H:%M:%S')} {msg}\n")
    except OSError:
        pass


def teacher_forced_check(oracle_model, prompt, gpu_tokens, gap_tol=1e-2, report=None, every=0):
    """Score the GPU's output with the oracle position by position.  A position
    passes if the GPU token is the oracle's arg max, or the oracle's logit gap
    between its arg max and the GPU token is below gap_tol (flagged near-tie).
    Returns (n_flagged, n_scored); raises on a real mismatch.  report (a dict) receives
    the flagged gaps and the number of positions whose oracle top-2 gap is below gap_tol."""
    s = oracle_model.session()
    first = s.prefill(prompt)
    z = s.verify_logits(0)
    flagged = 0
    gaps, close = [], 0
    toks = list(gpu_tokens)
    for i, t in enumerate(toks):
        am = int(np.argmax(z))
        top2 = np.partition(z, -2)[-2:]
        close += int(top2[1] - top2[0] < gap_tol)
        if t != am:
            gap = float(z[am] - z[t])
            assert gap < gap_tol, f"position {i}: gpu token {t}, oracle {am}, logit gap {gap}"
            flagged += 1
            gaps.append(gap)
        if every and i % every == 0:
            progress(f"  oracle scored {i + 1}/{len(toks)} positions, {flagged} flagged")
        if i + 1 < len(toks):
            _, z = s.step(t)
    if report is not None:
        report.update(flagged=flagged, scored=len(toks), gaps=gaps, close_positions=close)
    return flagged, len(toks)


class NearTies:
    """Where a GPU-vs-oracle comparison of free-running rounds must end because the two sides
    chose different tokens, the choice has to be a near-tie FOR THE ORACLE: its logit gap
    between its own arg max and the GPU's token below `tol`.  Counts such endings."""

    def __init__(self, tol=1e-2):
        self.tol, self.flags = tol, []

    def flag(self, where, z_oracle, tok_gpu):
        gap = float(np.max(z_oracle) - z_oracle[tok_gpu])
        assert gap < self.tol, f"{where}: gpu token {tok_gpu}, oracle {int(np.argmax(z_oracle))}, oracle logit gap {gap}"
        self.flags.append((where, gap))
        print(f"near-tie ({where}): oracle gap {gap:.3g}", flush=True)

    def verify_rows(self, where, osn, vo, vg):
        """Emitted tokens of a verification differ: the first differing row must be a near-tie."""
        for i, (a, b) in enumerate(zip(vo["tokens"], vg["tokens"])):
            if a != b:
                self.flag(f"{where} row {i}", osn.verify_logits(i), b)
                return
        raise AssertionError(f"{where}: emitted counts differ with equal tokens: {vo} vs {vg}")


# ---------------------------------------------------------------- planted mistakes (CPU)
def oracle_with_mistake(monkeypatch, tmp_path, old, new):
    """Build the oracle from a copy of its source with `old` replaced by `new` and make the
    oracle package load that build for the rest of the test (monkeypatch undoes it)."""
    import subprocess
    import oracle.oracle as orc_mod
    import oracle.build as orc_build
    src = open(orc_build.SRC).read()
    assert src.count(old) == 1, "mutation site not unique in the oracle source"
    msrc = tmp_path / "mutant.c"
    msrc.write_text(src.replace(old, new))
    paths = {}
    for bits, defs in ((64, []), (32, ["-DORC_F32"])):
        paths[bits] = str(tmp_path / f"libmut{bits}.so")
        subprocess.check_call(["gcc", *orc_build.FLAGS, *defs, str(msrc), "-o", paths[bits], "-lm"])
    monkeypatch.setattr(orc_build, "lib_path", lambda bits: paths[bits])
    monkeypatch.setattr(orc_mod, "_libs", {})
