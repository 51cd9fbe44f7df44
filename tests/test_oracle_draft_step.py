"""Pins of the oracle's draft step (Sec. 3.2, Eq. 1-2; Sec. 3.3): which temperature, which
exit norm and which exit head belong to layer l, that the confidence is
max softmax(z^(l) / T_l), that the token exits at the FIRST layer with p >= tau and that the
comparison is inclusive.

Exactness of the output cannot see any of this (whatever the draft rule, verification
restores the greedy tokens), so the step is recomputed here from the hidden state the
oracle exposes, with numpy and with the separately pinned primitives.  The second half
plants the corresponding mistakes into a copy of the oracle's source, one at a time, and
requires that the pins above turn red for each of them.  CPU only."""
import numpy as np
import pytest

import sb_inputs as si
import oracle as orc
from helpers import tiny_model, params, oracle_with_mistake

D_MAX = 5
T_DISTINCT = [3.0, 0.7, 1.9, 1.3, 0.55]       # no symmetry: T[l-1] != T[d_max-l] for every l


def _model(bits=64):
    # one head more than d_max (so that "the next layer's head" exists), distinct norm gains
    return tiny_model(n_layers=7, n_exit_heads=D_MAX + 1, seed=77, gain_jitter=0.3, bits=bits)


def _numpy_confidence(w, shape, h, l, T):
    """Eq. 2 at layer l written out: z = W_l (h / sqrt(mean h^2 + eps) * g_l), p = max softmax(z / T)."""
    g = w[f"exit_norm.{l - 1}"].astype(np.float64)
    W = w[f"exit_head.{l - 1}"].astype(np.float64)
    xn = h / np.sqrt(np.mean(h * h) + float(np.float32(shape.rms_eps))) * g   # eps is a float in the config
    z = W @ xn
    e = np.exp((z - z.max()) / T)
    return z, int(np.argmax(z)), float(e.max() / e.sum())


def pin_layer_binding():
    """Forced exit at every layer l: confidence, logits and token must be those of head l,
    norm l and temperature T_l applied to the row's hidden state after layer l."""
    shape, w, m = _model()
    prompt = si.make_prompt(shape.vocab, 6, 701)
    for l in range(1, D_MAX + 1):
        s = m.session()
        s.prefill(prompt)
        r = s.draft_step(params(D_MAX, 4, 0.5, forced_exit=[l], T=T_DISTINCT))
        assert r["exit_layer"] == l and s.slot_reached(0) == l
        h = s.slot_hidden(0)
        z, am, p = _numpy_confidence(w, shape, h, l, T_DISTINCT[l - 1])
        np.testing.assert_allclose(s.head_logits(), z, rtol=0, atol=1e-12)
        assert r["token"] == am
        assert abs(r["confidence"] - p) <= 1e-7 * p, (l, r["confidence"], p)
        # the same through the oracle's own (separately pinned) primitives
        zz = orc.matvec(w[f"exit_head.{l - 1}"], orc.rmsnorm(h, w[f"exit_norm.{l - 1}"], shape.rms_eps))
        am2, p2 = orc.act(zz, T_DISTINCT[l - 1])
        assert am2 == am and np.float32(p2) == np.float32(r["confidence"])
        # and it is not what a neighbouring layer's parameters would give
        for other in range(1, D_MAX + 1):
            if other != l:
                assert abs(_numpy_confidence(w, shape, h, l, T_DISTINCT[other - 1])[2] - p) > 1e-5 * p


def _layer_confidences(m, prompt, bits):
    out = []
    for l in range(1, D_MAX + 1):
        s = m.session()
        s.prefill(prompt)
        out.append(s.draft_step(params(D_MAX, 4, 0.5, forced_exit=[l], T=T_DISTINCT))["confidence"])
    return out


def pin_first_layer_and_inclusive_threshold():
    """Computed exits in float arithmetic, where the confidence a step reports is the very
    number the test compares: with tau equal to layer l's confidence the token exits at the
    first layer whose confidence is >= tau (layer l itself if none before it), and with the
    next float above tau layer l no longer qualifies."""
    shape, w, m = _model(bits=32)
    prompt = si.make_prompt(shape.vocab, 6, 702)
    conf = [np.float32(c) for c in _layer_confidences(m, prompt, 32)]
    assert len(set(conf)) == D_MAX
    seen_later_first = False
    for l in range(1, D_MAX + 1):
        for tau, inclusive in ((conf[l - 1], True), (np.nextafter(conf[l - 1], np.float32(2)), False)):
            want = next((k for k in range(1, D_MAX + 1) if conf[k - 1] >= tau), 0)
            if inclusive:
                assert 1 <= want <= l
                seen_later_first |= want < l
            s = m.session()
            s.prefill(prompt)
            r = s.draft_step(params(D_MAX, 4, float(tau), T=T_DISTINCT))
            assert r["exit_layer"] == want, (l, float(tau), r, [float(c) for c in conf])
            assert r["status"] == (orc.EXITED if want else orc.DEPTH_BOUND)
            if want:
                assert np.float32(r["confidence"]) == conf[want - 1]
    assert seen_later_first   # some tau was reached by an earlier layer: "first" was exercised


def pin_exact_equality_in_double():
    """A zero exit head gives p = 1/V exactly (V a power of two): tau = 1/V must exit there."""
    shape, w, _ = _model()
    w = dict(w)
    w["exit_head.0"] = np.zeros_like(w["exit_head.0"])
    m = orc.Oracle(shape, w, 160)
    s = m.session()
    s.prefill(si.make_prompt(shape.vocab, 6, 703))
    r = s.draft_step(params(D_MAX, 4, 1.0 / shape.vocab, T=T_DISTINCT))
    assert r["exit_layer"] == 1 and r["confidence"] == 1.0 / shape.vocab and r["token"] == 0


PINS = (pin_layer_binding, pin_first_layer_and_inclusive_threshold, pin_exact_equality_in_double)


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_draft_step_pin(pin):
    pin()


# ---------------------------------------------------------------- planted mistakes
MUTANTS = {
    "temperature_of_layer_1_everywhere": ("(real)p->T[l - 1]", "(real)p->T[0]"),
    "temperature_schedule_reversed": ("(real)p->T[l - 1]", "(real)p->T[p->d_max - l]"),
    "head_of_the_next_layer": ("w.exit_head[l - 1], c->weight_dtype", "w.exit_head[l], c->weight_dtype"),
    "norm_of_layer_1_everywhere": ("w.exit_norm[l - 1], c->d_model", "w.exit_norm[0], c->d_model"),
    "strict_threshold": ("s->last_conf >= (real)p->threshold", "s->last_conf > (real)p->threshold"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_turns_a_pin_red(name, tmp_path, monkeypatch):
    oracle_with_mistake(monkeypatch, tmp_path, *MUTANTS[name])
    red = 0
    for pin in PINS:
        try:
            pin()
        except AssertionError:
            red += 1
    assert red >= 1, f"no pin notices the planted mistake '{name}'"
